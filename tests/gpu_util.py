"""Helpers shared by the GPU parity tests: upload seeded inputs, run the library through
its C ABI, run the fp64 oracle on the same arrays, compare."""
import numpy as np

from oracle import kd_oracle as O
from paper_2603_01875_amd import inputs as I

LOSS_RTOL = 1e-3          # loss relative error
GRAD_TOL = 2e-2           # gradient max-abs error, as a fraction of the oracle's max-abs value


def to_device(x, dtype):
    import torch
    if dtype == I.BF16:
        bits = I.bf16_bits(x)
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()


def to_host(t):
    import torch
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def run_gpu(cfg, data, **kw):
    import torch
    from paper_2603_01875_amd import kdloss as K
    d = {k: to_device(data[k], cfg.dtype) for k in ("h_t", "W_t", "h_s", "W_s")}
    mask = None if data["mask"] is None else torch.from_numpy(data["mask"]).cuda()
    out = K.kd_loss_fwd_bwd(d["h_t"], d["W_t"], d["h_s"], d["W_s"], mask, tau=cfg.tau, kind=cfg.kind,
                            beta=cfg.beta, w_layout=K.W_VH, **kw)
    torch.cuda.synchronize()
    return out


def run_oracle(cfg, data):
    return O.kd_loss_fwd_bwd(data["h_t"], data["W_t"], data["h_s"], data["W_s"], data["mask"], cfg.tau,
                             cfg.kind, cfg.beta, O.W_VH)


def check(out, ref, what=""):
    loss = float(out["loss"].item())
    rel = abs(loss - ref["loss"]) / max(abs(ref["loss"]), 1e-30)
    assert np.isfinite(loss), what
    assert rel <= LOSS_RTOL, f"{what}: loss {loss} vs {ref['loss']} (rel {rel:.2e})"
    ptl = to_host(out["per_token_loss"])
    scale = max(np.abs(ref["per_token_loss"]).max(), 1e-30)
    assert np.abs(ptl - ref["per_token_loss"]).max() <= 2e-3 * scale, f"{what}: per-token loss"
    for name in ("grad_h_s", "grad_W_s"):
        g = to_host(out[name])
        assert np.isfinite(g).all(), f"{what}: {name} not finite"
        mx = np.abs(ref[name]).max()
        err = np.abs(g - ref[name]).max()
        assert err <= GRAD_TOL * mx + 1e-30, f"{what}: {name} err {err:.3e} vs max {mx:.3e}"
    return rel
