"""GPU tests of the fp8 teacher head (KD_FLAG_TEACHER_FP8): the teacher hidden states and head are
e4m3 codes with one scale each, the teacher logit tiles run on the fp8 matrix pipe.  Parity is against
the fp64 oracle fed with the DE-QUANTISED teacher arrays, i.e. the exact values the codes stand for,
so the tolerances are the ones of the bf16 path.  The quantiser kernel is checked bit for bit."""
import numpy as np
import pytest

from oracle import e4m3 as E
from paper_2603_01875_amd import inputs as I
from tests import gpu_util as G

pytestmark = pytest.mark.gpu

# The fp8 MFMA sums its 64 products per instruction with about 14 bits below the largest one (measured
# 6e-5 relative on a single 32x32x64 block), so fp8 teacher logits deviate by up to 1e-4 relative from the
# exact sum of the same products: far below the quantisation step (2^-4) and the tolerances, but it widens
# the band in which TVD's sign(p_s - p_t) may come out either way.
FP8_TIE_GAP = 3e-4


def _run_fp8(cfg, data, f8, forward_only=False, **more):
    import torch
    from paper_2603_01875_amd import kdloss as K
    q_h = torch.from_numpy(f8["q_h_t"]).cuda()
    q_W = torch.from_numpy(f8["q_W_t"]).cuda()
    h_s = G.to_device(data["h_s"], cfg.dtype)
    W_s = G.to_device(data["W_s"], cfg.dtype)
    mask = None if data["mask"] is None else torch.from_numpy(data["mask"]).cuda()
    kw = dict(tau=cfg.tau, kind=cfg.kind, beta=cfg.beta, flags=K.FLAG_TEACHER_FP8, teacher_scale=f8["teacher_scale"],
              **more)
    out = (K.kd_loss_fwd if forward_only else K.kd_loss_fwd_bwd)(q_h, q_W, h_s, W_s, mask, **kw)
    torch.cuda.synchronize()
    return out


def _oracle_fp8(cfg, data, f8):
    d = dict(data)
    d["h_t"], d["W_t"] = f8["h_t"], f8["W_t"]
    return G.run_oracle(cfg, d)


@pytest.mark.parametrize("src", ["bf16", "f32"])
def test_quantiser_is_bit_exact(src):
    import torch
    from paper_2603_01875_amd import kdloss as K
    rng = np.random.default_rng(11)
    n = 100003                                            # ragged: not a multiple of 8
    x = (rng.standard_normal(n) * np.exp(rng.uniform(-9, 7, n))).astype(np.float32)
    x[:12] = [0.0, -0.0, 1.0625, 1.1875, 2.0 ** -10, 3 * 2.0 ** -10, 447.9, 448.0, 464.0, -1e9, np.inf, np.nan]
    if src == "bf16":
        x = I.round_to_bf16(x)
    xd = torch.from_numpy(x).cuda()
    if src == "bf16":
        xd = xd.to(torch.bfloat16)
    for scale in (1.0, 0.37, 3.0e-3):
        got = K.quantize_e4m3(xd, scale).cpu().numpy()
        want = E.quantize_e4m3(x, scale)
        np.testing.assert_array_equal(got, want)


KINDS = [("fkl_bf16", I.FKL, 0.5), ("rkl_bf16", I.RKL, 0.5), ("jsd_bf16", I.JSD, 0.5), ("long_peaked", I.JSD, 0.1)]


@pytest.mark.parametrize("name,kind,beta", KINDS)
def test_fp8_teacher_ragged_multi_tile(name, kind, beta):
    # 3 token tiles (last one ragged), 20 vocabulary tiles (last one 8 rows), 5 chunks, 3 fp8 k-steps
    cfg = I.scaled(I.workload(name), batch=3, seq=200, H_t=384, H_s=128, V=2440)
    data = I.generate(cfg)
    f8 = G.fp8_teacher(data)
    out = _run_fp8(cfg, data, f8, vocab_chunk=512)
    G.check(out, _oracle_fp8(cfg, data, f8), name + " fp8 teacher")
    keep = data["mask"].astype(bool)
    assert (G.to_host(out["grad_h_s"])[~keep] == 0).all()


@pytest.mark.parametrize("kind,beta", [(I.TVD, 0.5), (I.SKEW_FKL, 0.1), (I.SKEW_RKL, 0.1)])
def test_fp8_teacher_other_divergences(kind, beta):
    cfg = I.scaled(I.workload("fkl_bf16"), batch=2, seq=150, H_t=128, H_s=64, V=1000, kind=kind, beta=beta)
    data = I.generate(cfg)
    f8 = G.fp8_teacher(data)
    d = dict(data); d["h_t"], d["W_t"] = f8["h_t"], f8["W_t"]
    extra = G.tvd_tie_allowance(cfg, d, rel_gap=FP8_TIE_GAP) if kind == I.TVD else None
    G.check(_run_fp8(cfg, data, f8), _oracle_fp8(cfg, data, f8), f"kind {kind} fp8 teacher", extra)


@pytest.mark.parametrize("H_t", [128, 256, 1024])
def test_fp8_teacher_hidden_sizes_and_temperature(H_t):
    cfg = I.scaled(I.workload("fkl_bf16"), batch=1, seq=300, H_t=H_t, H_s=64, V=776, tau=2.5, mask="ones")
    data = I.generate(cfg)
    f8 = G.fp8_teacher(data)
    G.check(_run_fp8(cfg, data, f8), _oracle_fp8(cfg, data, f8), f"H_t={H_t} fp8 teacher")


def test_fp8_teacher_forward_only_matches_full_call():
    cfg = I.scaled(I.workload("jsd_bf16"), batch=2, seq=160, H_t=256, H_s=128, V=1288)
    data = I.generate(cfg)
    f8 = G.fp8_teacher(data)
    full = _run_fp8(cfg, data, f8)
    fwd = _run_fp8(cfg, data, f8, forward_only=True)
    assert float(full["loss"].item()) == float(fwd["loss"].item())
    assert (G.to_host(full["per_token_loss"]) == G.to_host(fwd["per_token_loss"])).all()


def test_codes_that_bf16_holds_exactly_give_the_bf16_result():
    """e4m3 values are exactly representable in bf16: feeding the de-quantised teacher to the bf16
    path must give the same loss to fp32 accumulation accuracy (same products, other summation order)."""
    import torch
    cfg = I.scaled(I.workload("fkl_bf16"), batch=2, seq=140, H_t=256, H_s=64, V=1000)
    data = I.generate(cfg)
    f8 = G.fp8_teacher(data)
    a = _run_fp8(cfg, data, f8)
    # power-of-two scales keep the de-quantised values bf16-exact: re-quantise with such scales
    d = dict(data)
    tab = E.e4m3_values()
    q = {}
    for k in ("h_t", "W_t"):
        s = float(2.0 ** np.ceil(np.log2(np.abs(data[k]).max() / 448.0)))
        q[k] = (E.quantize_e4m3(data[k], s), s)
        d[k] = (tab[q[k][0]] * s).astype(np.float32)
        assert (I.round_to_bf16(d[k]) == d[k]).all()
    f8p = dict(q_h_t=q["h_t"][0], q_W_t=q["W_t"][0], teacher_scale=q["h_t"][1] * q["W_t"][1])
    a = _run_fp8(cfg, data, f8p)
    b = G.run_gpu(cfg, d)
    la, lb = float(a["loss"].item()), float(b["loss"].item())
    assert abs(la - lb) <= 1e-5 * abs(lb)
    ga, gb = G.to_host(a["grad_W_s"]), G.to_host(b["grad_W_s"])
    assert np.abs(ga - gb).max() <= 2e-2 * np.abs(gb).max()


def test_two_fp8_teachers_with_their_own_scales():
    """Multi-teacher call with fp8 teachers: each teacher has its own joint scale; against the oracle on
    the de-quantised teachers."""
    import torch
    from oracle import kd_oracle as O
    from paper_2603_01875_amd import kdloss as K
    base = I.scaled(I.workload("fkl_bf16"), batch=2, seq=150, H_s=128, V=1544)
    ds = [I.generate(I.scaled(base, H_t=h, w_t_std=sd, seed=900 + i)) for i, (h, sd) in enumerate(((128, 0.02), (256, 0.05)))]
    f8 = [G.fp8_teacher(d) for d in ds]
    weights = (0.4, 0.6)
    h_s, W_s, mask = ds[0]["h_s"], ds[0]["W_s"], ds[0]["mask"]
    for kind, beta in ((I.FKL, 0.5), (I.JSD, 0.3)):
        ref = O.kd_loss_multi([f["h_t"] for f in f8], [f["W_t"] for f in f8], weights, h_s, W_s, mask, base.tau,
                              kind, beta, O.W_VH)
        ref["per_token_loss"] = ref["per_token_loss"] * (mask != 0)
        out = K.kd_loss_fwd_bwd_multi([torch.from_numpy(f["q_h_t"]).cuda() for f in f8],
                                      [torch.from_numpy(f["q_W_t"]).cuda() for f in f8], weights,
                                      G.to_device(h_s, I.BF16), G.to_device(W_s, I.BF16),
                                      torch.from_numpy(mask).cuda(), tau=base.tau, kind=kind, beta=beta,
                                      flags=K.FLAG_TEACHER_FP8, teacher_scales=[f["teacher_scale"] for f in f8],
                                      vocab_chunk=512)
        torch.cuda.synchronize()
        G.check(out, ref, f"two fp8 teachers kind={kind}")


def test_fp8_teacher_with_hidden_major_heads():
    """[H,V] heads with the fp8 teacher: the e4m3 head is transposed into a [V,H] copy inside the library;
    grad_W_s comes back as [H_s, V]."""
    import torch
    from oracle import kd_oracle as O
    from paper_2603_01875_amd import kdloss as K
    cfg = I.scaled(I.workload("rkl_bf16"), batch=2, seq=150, H_t=256, H_s=128, V=1608)
    data = I.generate(cfg)
    f8 = G.fp8_teacher(data)
    hv = lambda W: np.ascontiguousarray(W.T)
    ref = O.kd_loss_fwd_bwd(f8["h_t"], hv(f8["W_t"]), data["h_s"], hv(data["W_s"]), data["mask"], cfg.tau, cfg.kind,
                            cfg.beta, O.W_HV)
    ref["per_token_loss"] = ref["per_token_loss"] * (data["mask"] != 0)
    out = K.kd_loss_fwd_bwd(torch.from_numpy(f8["q_h_t"]).cuda(), torch.from_numpy(hv(f8["q_W_t"])).cuda(),
                            G.to_device(data["h_s"], I.BF16), G.to_device(hv(data["W_s"]), I.BF16),
                            torch.from_numpy(data["mask"]).cuda(), tau=cfg.tau, kind=cfg.kind, beta=cfg.beta,
                            w_layout=K.W_HV, flags=K.FLAG_TEACHER_FP8, teacher_scale=f8["teacher_scale"],
                            vocab_chunk=512)
    torch.cuda.synchronize()
    assert tuple(out["grad_W_s"].shape) == (cfg.H_s, cfg.V)
    G.check(out, ref, "fp8 teacher, [H,V] heads")
