"""fp64 CPU oracle for the full-vocabulary knowledge-distillation loss.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain reference that the
GPU library is checked against.  Only the tests, the smoke check and the
`cpu_baseline` leg of the benchmark may import it; the product path never
does.  It shares no code with the HIP kernels and imports nothing from the
package.

What it computes (paper, abstract and Sec. 3.2 "Efficient Communication via
Hidden States"): on a student worker the teacher's final hidden states h_t are
turned back into full-vocabulary logits through a frozen copy of the teacher
output head, z_t = h_t . W_t, and compared with the student logits
z_s = h_s . W_s under one of the divergences the paper names in Sec. 3.4
(forward KL, reverse KL, Jensen-Shannon).  The paper's claim is that this is
mathematically the same as standard logit-based distillation, so the oracle is
the textbook definition with the logits fully materialised (row blocks only
bound the RAM; they do not change the arithmetic of any row).

The paper names the divergences without printing formulas.  Readings taken:
  * p = softmax(z / tau) for BOTH models, natural logarithm, no tau^2 factor;
  * FKL  = KL(p_t || p_s),  RKL = KL(p_s || p_t), per token;
  * JSD(beta) = beta KL(p_t || M) + (1-beta) KL(p_s || M),
    M = beta p_t + (1-beta) p_s   (generalised JSD of the GKD paper the
    authors cite; beta=0.5 is the classic symmetric JSD);
  * the loss is the masked mean over tokens: sum_t mask_t l_t / sum_t mask_t,
    and is 0 with zero gradients when every token is masked;
  * 0 log 0 := 0.
Further divergences of the paper's list (Sec. 3.4 names TVD; Table 1 lists skewed
forward / reverse KL), with `beta` doubling as the skew weight alpha:
  * TVD = 1/2 sum_v |p_t - p_s|;
  * skewed FKL = KL(p_t || alpha p_t + (1-alpha) p_s),
    skewed RKL = KL(p_s || (1-alpha) p_t + alpha p_s)   (the skew divergences of
    the DistiLLM paper the authors cite; alpha -> 0 recovers FKL / RKL).
  * AKL (Table 1 lists it; the adaptive KL of the paper by Wu et al. that the authors cite): per token,
    the vocabulary is split by the teacher: going through the teacher probabilities in descending order,
    the HEAD is the longest prefix whose cumulative teacher mass stays <= mu (the top entry always belongs
    to it), the TAIL is the rest; with the gaps g_head = sum_head |p_t - p_s|, g_tail = sum_tail |p_t - p_s|,
      AKL = g_head / (g_head + g_tail) * FKL + g_tail / (g_head + g_tail) * RKL
    (weights 1/2, 1/2 when both gaps vanish).  mu is passed in `beta` (the cited method fixes 1/2).
    The weights are constants for the gradient (the cited method forms them without gradient tracking):
    g = w_f g_FKL + w_r g_RKL.  The paper itself gives no formula: this is a reading.
For every divergence that is a function D(p_s) of the student probabilities, the
gradient through the softmax is g = p_s * (c - sum_v p_s c) with c = dD/dp_s:
  TVD: c = 1/2 sign(p_s - p_t);   skewed FKL: c = -(1-alpha) p_t / M;
  skewed RKL: c = (log p_s - log M) + 1 - alpha p_s / M.
Every function below is pinned by tests that do not call it to make their
expected values (closed forms, library routines for special cases, finite
differences, inequalities); see tests/test_oracle_pins.py.

Gradients are the exact derivatives of that loss:
  dL/dz_s[t,:] = mask_t / (n tau) * g_t,  with
    FKL: g = p_s - p_t
    RKL: g = p_s * ((log p_s - log p_t) - l_t)
    JSD: g = (1-beta) p_s * ((log p_s - log M) - K_t),  K_t = KL(p_s || M)
  grad_h_s = dz . W_s^T,   grad_W_s = h_s^T . dz        (Sec. 3.1, student backward)
"""
from __future__ import annotations

import numpy as np

FKL, RKL, JSD, TVD, SKEW_FKL, SKEW_RKL, AKL = 0, 1, 2, 3, 4, 5, 6
KIND_NAMES = {FKL: "fkl", RKL: "rkl", JSD: "jsd", TVD: "tvd", SKEW_FKL: "skew_fkl", SKEW_RKL: "skew_rkl",
              AKL: "akl"}

# storage order of an output head: W_HV is the mathematical [H, V] array,
# W_VH is its transpose [V, H] (the order lm_head.weight is kept in).
W_HV, W_VH = 0, 1


def _as_hv(W, w_layout):
    """Return the head as the mathematical [H, V] fp64 array."""
    W = np.asarray(W, dtype=np.float64)
    if w_layout == W_HV:
        return W
    if w_layout == W_VH:
        return W.T
    raise ValueError("unknown w_layout")


def logits(h, W, w_layout=W_HV):
    """z = h . W, [T,H] x [H,V] -> [T,V] (Sec. 3.2: logit recomputation)."""
    return np.asarray(h, dtype=np.float64) @ _as_hv(W, w_layout)


def log_softmax(z, tau=1.0):
    """Row-wise log softmax of z / tau, max-subtracted."""
    u = np.asarray(z, dtype=np.float64) / float(tau)
    u = u - u.max(axis=-1, keepdims=True)
    return u - np.log(np.exp(u).sum(axis=-1, keepdims=True))


def _xlogy_diff(p, la, lb):
    """sum_v p * (la - lb) with the convention 0 * anything := 0."""
    d = la - lb
    term = np.where(p > 0.0, p * np.where(p > 0.0, d, 0.0), 0.0)
    return term.sum(axis=-1)


def akl_head(pt, mu):
    """Boolean [T,V]: the head of each row of teacher probabilities (see the module header, AKL)."""
    order = np.argsort(-pt, axis=-1, kind="stable")               # descending teacher probability
    cum = np.cumsum(np.take_along_axis(pt, order, axis=-1), axis=-1)
    keep = cum <= mu                                              # prefix whose mass stays within mu
    keep[..., 0] = True                                           # the top entry is always head
    head = np.zeros(pt.shape, dtype=bool)
    np.put_along_axis(head, order, keep, axis=-1)
    return head


def akl_weights(pt, ps, mu):
    """(w_f, w_r) per row: the shares of the head and tail gaps (AKL)."""
    head = akl_head(pt, mu)
    gap = np.abs(pt - ps)
    g_head = np.where(head, gap, 0.0).sum(axis=-1)
    g_tail = np.where(head, 0.0, gap).sum(axis=-1)
    tot = g_head + g_tail
    safe = np.where(tot > 0.0, tot, 1.0)
    w_f = np.where(tot > 0.0, g_head / safe, 0.5)
    return w_f, 1.0 - w_f


def divergence_rows(z_t, z_s, tau, kind, beta=0.5):
    """Per-token divergence l[T] and g[T,V] = tau * d l_t / d z_s[t,:].

    z_t, z_s: [T,V] raw logits.  Sec. 3.4 names the divergences; formulas are
    the textbook ones stated in the module header.
    """
    lt = log_softmax(z_t, tau)
    ls = log_softmax(z_s, tau)
    pt = np.exp(lt)
    ps = np.exp(ls)
    if kind == FKL:
        l = _xlogy_diff(pt, lt, ls)
        g = ps - pt
    elif kind == RKL:
        l = _xlogy_diff(ps, ls, lt)
        g = ps * ((ls - lt) - l[:, None])
    elif kind == JSD:
        if not (0.0 < beta < 1.0):
            raise ValueError("JSD needs 0 < beta < 1")
        lm = np.logaddexp(np.log(beta) + lt, np.log1p(-beta) + ls)
        k_s = _xlogy_diff(ps, ls, lm)          # KL(p_s || M)
        k_t = _xlogy_diff(pt, lt, lm)          # KL(p_t || M)
        l = beta * k_t + (1.0 - beta) * k_s
        g = (1.0 - beta) * ps * ((ls - lm) - k_s[:, None])
    elif kind == TVD:
        d = ps - pt
        l = 0.5 * np.abs(d).sum(axis=-1)
        c = 0.5 * np.sign(d)
        g = ps * (c - (ps * c).sum(axis=-1, keepdims=True))
    elif kind in (SKEW_FKL, SKEW_RKL):
        alpha = beta
        if not (0.0 < alpha < 1.0):
            raise ValueError("skewed KL needs 0 < alpha < 1")
        if kind == SKEW_FKL:
            lm = np.logaddexp(np.log(alpha) + lt, np.log1p(-alpha) + ls)   # M = a pt + (1-a) ps
            l = _xlogy_diff(pt, lt, lm)
            c = -(1.0 - alpha) * np.exp(lt - lm)
        else:
            lm = np.logaddexp(np.log1p(-alpha) + lt, np.log(alpha) + ls)   # M = (1-a) pt + a ps
            l = _xlogy_diff(ps, ls, lm)
            c = (ls - lm) + 1.0 - alpha * np.exp(ls - lm)
        g = ps * (c - (ps * c).sum(axis=-1, keepdims=True))
    elif kind == AKL:
        if not (0.0 < beta < 1.0):
            raise ValueError("AKL needs 0 < mu < 1")
        w_f, w_r = akl_weights(pt, ps, beta)
        l_f = _xlogy_diff(pt, lt, ls)
        l_r = _xlogy_diff(ps, ls, lt)
        l = w_f * l_f + w_r * l_r
        g = w_f[:, None] * (ps - pt) + w_r[:, None] * (ps * ((ls - lt) - l_r[:, None]))
    else:
        raise ValueError("unknown kind")
    return l, g


def kd_loss_from_logits(z_t, z_s, mask=None, tau=1.0, kind=FKL, beta=0.5):
    """Standard logit-based KD: masked-mean loss, per-token loss and dL/dz_s.

    This is the computation the paper says hidden-state transfer must stay
    equivalent to (Sec. 3.2, last sentence).
    """
    z_t = np.asarray(z_t, dtype=np.float64)
    z_s = np.asarray(z_s, dtype=np.float64)
    T = z_t.shape[0]
    m = np.ones(T) if mask is None else (np.asarray(mask) != 0).astype(np.float64)
    n = m.sum()
    l, g = divergence_rows(z_t, z_s, tau, kind, beta)
    if n == 0:
        return 0.0, l, np.zeros_like(g)
    loss = float((m * l).sum() / n)
    dz = (m / (n * tau))[:, None] * g
    return loss, l, dz


def kd_loss_fwd_bwd(h_t, W_t, h_s, W_s, mask=None, tau=1.0, kind=FKL, beta=0.5,
                    w_layout=W_HV, row_block=512, tau2=False):
    """The whole hot path in fp64.

    Returns dict(loss, per_token_loss[T], n, grad_h_s[T,H_s], grad_W_s) with
    grad_W_s in the same storage order as W_s.  Rows are processed `row_block`
    at a time so that only a [row_block, V] slab of logits exists at once.
    """
    h_t = np.asarray(h_t, dtype=np.float64)
    h_s = np.asarray(h_s, dtype=np.float64)
    Wt = _as_hv(W_t, w_layout)
    Ws = _as_hv(W_s, w_layout)
    T = h_t.shape[0]
    if h_s.shape[0] != T or Wt.shape[1] != Ws.shape[1]:
        raise ValueError("shape mismatch")
    m = np.ones(T) if mask is None else (np.asarray(mask) != 0).astype(np.float64)
    n = m.sum()
    per_tok = np.empty(T)
    grad_h = np.zeros_like(h_s)
    grad_W = np.zeros_like(Ws)                       # [H_s, V]
    for r0 in range(0, T, row_block):
        r1 = min(T, r0 + row_block)
        z_t = h_t[r0:r1] @ Wt
        z_s = h_s[r0:r1] @ Ws
        l, g = divergence_rows(z_t, z_s, tau, kind, beta)
        per_tok[r0:r1] = l
        if n > 0:
            dz = (m[r0:r1] / (n * tau))[:, None] * g
            grad_h[r0:r1] = dz @ Ws.T
            grad_W += h_s[r0:r1].T @ dz
    loss = float((m * per_tok).sum() / n) if n > 0 else 0.0
    if w_layout == W_VH:
        grad_W = np.ascontiguousarray(grad_W.T)
    if tau2:                       # optional convention: everything times tau^2
        f = float(tau) ** 2
        loss, per_tok, grad_h, grad_W = loss * f, per_tok * f, grad_h * f, grad_W * f
    return dict(loss=loss, per_token_loss=per_tok, n=int(n),
                grad_h_s=grad_h, grad_W_s=grad_W)


def kd_loss_multi(h_ts, W_ts, weights, h_s, W_s, mask=None, tau=1.0, kind=FKL, beta=0.5,
                  w_layout=W_HV, row_block=512):
    """Multi-teacher distillation (Table 1): loss = sum_k weights[k] D(p_t^k, p_s); by linearity the
    outputs are the weighted sums of the single-teacher outputs."""
    tot = None
    for w, h_t, W_t in zip(weights, h_ts, W_ts):
        r = kd_loss_fwd_bwd(h_t, W_t, h_s, W_s, mask, tau, kind, beta, w_layout, row_block)
        if tot is None:
            tot = {k: (w * v if k != "n" else v) for k, v in r.items()}
        else:
            for k in ("loss", "per_token_loss", "grad_h_s", "grad_W_s"):
                tot[k] = tot[k] + w * r[k]
    return tot


def row_lse(h, W, tau=1.0, w_layout=W_HV, row_block=512):
    """lse_t = log sum_v exp(z[t,v]/tau) for every row (used to check sampled
    outputs of full-size problems one by one)."""
    h = np.asarray(h, dtype=np.float64)
    Whv = _as_hv(W, w_layout)
    out = np.empty(h.shape[0])
    for r0 in range(0, h.shape[0], row_block):
        u = (h[r0:r0 + row_block] @ Whv) / float(tau)
        mx = u.max(axis=-1)
        out[r0:r0 + row_block] = mx + np.log(np.exp(u - mx[:, None]).sum(axis=-1))
    return out
