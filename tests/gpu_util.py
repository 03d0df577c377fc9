"""Helpers shared by the GPU parity tests: upload seeded inputs, run the library through
its C ABI, run the fp64 oracle on the same arrays, compare."""
import numpy as np

from oracle import e4m3 as E
from oracle import kd_oracle as O
from paper_2603_01875_amd import inputs as I

LOSS_RTOL = 1e-3          # loss relative error
GRAD_TOL = 2e-2           # gradient max-abs error, as a fraction of the oracle's max-abs value


to_device = I.to_device


def fp8_teacher(data: dict) -> dict:
    """The teacher side of `data` quantised to e4m3 with one scale per array (max|x| / 448).
    Returns the codes (for the GPU), the scales, and the de-quantised arrays (for the oracle)."""
    tab = E.e4m3_values()
    out = {}
    for k in ("h_t", "W_t"):
        s = float(np.float32(np.abs(data[k]).max() / 448.0))
        q = E.quantize_e4m3(data[k], s)
        out["q_" + k], out["scale_" + k] = q, s
        out[k] = (tab[q] * np.float64(np.float32(s))).astype(np.float64)
    # the kernels apply the product of the two scales as one fp32 factor
    out["teacher_scale"] = float(np.float32(out["scale_h_t"]) * np.float32(out["scale_W_t"]))
    return out


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
    ref = O.kd_loss_fwd_bwd(data["h_t"], data["W_t"], data["h_s"], data["W_s"], data["mask"], cfg.tau,
                            cfg.kind, cfg.beta, O.W_VH)
    if data["mask"] is not None:        # the library reports 0 for masked tokens (it never computes them)
        ref["per_token_loss"] = ref["per_token_loss"] * (np.asarray(data["mask"]) != 0)
    return ref


def tvd_tie_allowance(cfg, data, rel_gap=2e-5):
    """TVD's gradient carries sign(p_s - p_t): where the two probabilities agree to within fp32
    rounding of the logits, either sign is a valid subgradient and the two sides may pick different
    ones.  Returns per-row allowances (grad_h_s rows, grad_W_s rows) equal to the size of the
    contribution such an element can flip, computed from the oracle's probabilities."""
    z_t = data["h_t"].astype(np.float64) @ data["W_t"].astype(np.float64).T
    z_s = data["h_s"].astype(np.float64) @ data["W_s"].astype(np.float64).T
    pt = np.exp(O.log_softmax(z_t, cfg.tau)); ps = np.exp(O.log_softmax(z_s, cfg.tau))
    m = (np.asarray(data["mask"]) != 0).astype(np.float64)
    s = m / (max(m.sum(), 1.0) * cfg.tau)
    t_idx, v_idx = np.nonzero(np.abs(ps - pt) <= rel_gap * ps)
    allow_h = np.zeros(cfg.T); allow_W = np.zeros(cfg.V)
    for t, v in zip(t_idx, v_idx):
        flip = s[t] * ps[t, v]                      # dz changes by at most this much
        allow_h[t] += flip * np.abs(data["W_s"][v]).max()
        allow_W[v] += flip * np.abs(data["h_s"][t]).max()
    return dict(grad_h_s=allow_h[:, None], grad_W_s=allow_W[:, None])


def akl_allowance(cfg, data, band2=8e-4, top2=2e-4):
    """AKL splits each token's vocabulary at a teacher probability that the library locates by a search over
    base-2 log-probabilities, to within 4.8e-4, in fp32.  Head entries less than `band2` above the first tail
    entry (and near-ties of the top entry, which is head whatever its mass) may therefore fall on either side
    of the split.  Each such entry can move its gap |p_t - p_s| between head and tail, which shifts the weight
    w_f by at most their summed gaps over the total gap; every output is linear in w_f, so the allowances
    follow.  Computed from the oracle's probabilities; zero for rows with no entry near the split."""
    ln2 = np.log(2.0)
    mu = cfg.beta
    z_t = data["h_t"].astype(np.float64) @ data["W_t"].astype(np.float64).T
    z_s = data["h_s"].astype(np.float64) @ data["W_s"].astype(np.float64).T
    lt = O.log_softmax(z_t, cfg.tau); ls = O.log_softmax(z_s, cfg.tau)
    pt = np.exp(lt); ps = np.exp(ls)
    head = O.akl_head(pt, mu)
    gap = np.abs(pt - ps)
    tot = np.maximum(gap.sum(axis=1), 1e-300)
    first_tail = np.where(head, -np.inf, lt).max(axis=1)                      # log-probability of the first tail entry
    # the search ends with a threshold in (first tail entry, first tail entry + resolution]: head entries that
    # close above the first tail entry may be cut off; the first tail entry itself never gets in this way
    near = (lt > first_tail[:, None]) & (lt <= first_tail[:, None] + band2 * ln2)
    top = lt.max(axis=1)
    near |= (lt >= top[:, None] - top2 * ln2) & (lt < top[:, None])
    # running mass within fp32 summation error of mu: that entry's membership is undecided, too
    order = np.argsort(-pt, axis=1, kind="stable")
    cum = np.cumsum(np.take_along_axis(pt, order, axis=1), axis=1)
    close = np.zeros_like(near)
    np.put_along_axis(close, order, np.abs(cum - mu) <= 2e-6, axis=1)
    near |= close
    dw = np.where(near, gap, 0.0).sum(axis=1) / tot                            # |shift of w_f| per token
    l_f, g_f = O.divergence_rows(z_t, z_s, cfg.tau, O.FKL)
    l_r, g_r = O.divergence_rows(z_t, z_s, cfg.tau, O.RKL)
    m = (np.asarray(data["mask"]) != 0).astype(np.float64) if data["mask"] is not None else np.ones(cfg.T)
    n = max(m.sum(), 1.0)
    ddz = (m * dw / (n * cfg.tau))[:, None] * np.abs(g_f - g_r)
    return dict(per_token_loss=m * dw * np.abs(l_f - l_r), loss=float((m * dw * np.abs(l_f - l_r)).sum() / n),
                grad_h_s=ddz @ np.abs(data["W_s"].astype(np.float64)),
                grad_W_s=ddz.T @ np.abs(data["h_s"].astype(np.float64)), max_dw=float(dw.max()),
                mean_dw=float(dw.mean()))


def check(out, ref, what="", extra_tol=None):
    """extra_tol: optional per-output absolute allowances (keys grad_h_s, grad_W_s, and optionally loss and
    per_token_loss) on top of the tolerances, for outputs that hinge on a discrete decision."""
    loss = float(out["loss"].item())
    extra_loss = 0.0 if extra_tol is None else extra_tol.get("loss", 0.0)
    rel = max(abs(loss - ref["loss"]) - extra_loss, 0.0) / max(abs(ref["loss"]), 1e-30)
    assert np.isfinite(loss), what
    assert rel <= LOSS_RTOL, f"{what}: loss {loss} vs {ref['loss']} (rel {rel:.2e})"
    ptl = to_host(out["per_token_loss"])
    scale = max(np.abs(ref["per_token_loss"]).max(), 1e-30)
    extra_ptl = 0.0 if extra_tol is None else extra_tol.get("per_token_loss", 0.0)
    # a row loss is summed in fp32 over V terms: below about 1e-4 its absolute resolution (a few 1e-7) shows
    assert (np.abs(ptl - ref["per_token_loss"]) - extra_ptl).max() <= 2e-3 * scale + 5e-7, f"{what}: per-token loss"
    for name in ("grad_h_s", "grad_W_s"):
        g = to_host(out[name])
        assert np.isfinite(g).all(), f"{what}: {name} not finite"
        mx = np.abs(ref[name]).max()
        excess = np.abs(g - ref[name]) - (0.0 if extra_tol is None else extra_tol[name])
        err = excess.max()
        assert err <= GRAD_TOL * mx + 1e-30, f"{what}: {name} err {err:.3e} vs max {mx:.3e}"
    return rel
