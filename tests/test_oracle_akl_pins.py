"""Pins for the oracle's adaptive KL (AKL, Table 1 of the paper; defined in the cited paper by Wu et al.).
Expected values come from hand-worked examples, a brute-force head selection with Python's own sort,
library routines (scipy.stats.entropy, cityblock) and finite differences of a loss whose weights are held
fixed; nothing here calls the oracle to make its own expected value."""
import numpy as np
import pytest
import scipy.special as sps
import scipy.stats as sst
from scipy.spatial.distance import cityblock

from oracle import kd_oracle as O


def _logits(p):
    return np.log(np.asarray(p, dtype=np.float64))[None, :]


def test_hand_worked_examples():
    # teacher 0.4 0.3 0.2 0.1: running mass 0.4, 0.7 -> head = {0}.  gaps: head 0.3, tail 0.1 + 0.1 + 0.3
    pt = [0.4, 0.3, 0.2, 0.1]; ps = [0.1, 0.2, 0.3, 0.4]
    l, _ = O.divergence_rows(_logits(pt), _logits(ps), 1.0, O.AKL, 0.5)
    want = 0.375 * sst.entropy(pt, ps) + 0.625 * sst.entropy(ps, pt)
    assert l[0] == pytest.approx(want, rel=1e-13)
    # mu = 0.75: running mass 0.4, 0.7, 0.9 -> head = {0, 1}; gaps 0.4 and 0.4
    l, _ = O.divergence_rows(_logits(pt), _logits(ps), 1.0, O.AKL, 0.75)
    assert l[0] == pytest.approx(0.5 * sst.entropy(pt, ps) + 0.5 * sst.entropy(ps, pt), rel=1e-13)
    # top entry heavier than mu: it is the head on its own
    pt = [0.1, 0.7, 0.2]; ps = [0.3, 0.3, 0.4]
    l, _ = O.divergence_rows(_logits(pt), _logits(ps), 1.0, O.AKL, 0.5)
    want = (0.4 / 0.8) * sst.entropy(pt, ps) + (0.4 / 0.8) * sst.entropy(ps, pt)
    assert l[0] == pytest.approx(want, rel=1e-13)
    # running mass that lands exactly on mu stays in the head (0.25 + 0.25 = 0.5, in binary exactly)
    pt = [0.25, 0.125, 0.25, 0.375]; ps = [0.25, 0.25, 0.25, 0.25]
    head = O.akl_head(np.array([pt]), 0.5)[0]
    assert head.tolist() == [False, False, False, True]     # 0.375 first, then 0.375 + 0.25 > 0.5
    head = O.akl_head(np.array([[0.25, 0.25, 0.5 - 2 ** -20, 2 ** -20]]), 0.5)[0]
    assert head.sum() == 1 and head[2]


def _brute_force_weights(pt, ps, mu):
    idx = sorted(range(len(pt)), key=lambda i: -pt[i])
    head, run = set(), 0.0
    for rank, i in enumerate(idx):
        run += pt[i]
        if rank == 0 or run <= mu:
            head.add(i)
        else:
            break
    gh = sum(abs(pt[i] - ps[i]) for i in head)
    gt = sum(abs(pt[i] - ps[i]) for i in range(len(pt)) if i not in head)
    return gh / (gh + gt), gt / (gh + gt), head


@pytest.mark.parametrize("mu", [0.3, 0.5, 0.8])
def test_weights_against_brute_force_and_library_routines(mu):
    rng = np.random.default_rng(7)
    z_t = 1.5 * rng.standard_normal((6, 40)); z_s = rng.standard_normal((6, 40))
    tau = 1.3
    pt = sps.softmax(z_t / tau, axis=1); ps = sps.softmax(z_s / tau, axis=1)
    l, g = O.divergence_rows(z_t, z_s, tau, O.AKL, mu)
    w_f, w_r = O.akl_weights(pt, ps, mu)
    for r in range(6):
        bf, br, head = _brute_force_weights(list(pt[r]), list(ps[r]), mu)
        assert w_f[r] == pytest.approx(bf, rel=1e-12) and w_r[r] == pytest.approx(br, rel=1e-12)
        assert set(np.flatnonzero(O.akl_head(pt[r:r + 1], mu)[0])) == head
        mass = sum(pt[r][i] for i in head)
        assert mass <= mu or len(head) == 1
        # the next entry in line would push the mass past mu
        rest = [pt[r][i] for i in range(40) if i not in head]
        assert mass + max(rest) > mu
        assert l[r] == pytest.approx(bf * sst.entropy(pt[r], ps[r]) + br * sst.entropy(ps[r], pt[r]), rel=1e-12)
    assert np.allclose(w_f + w_r, 1.0) and (w_f >= 0).all() and (w_r >= 0).all()
    # head gap + tail gap = the whole L1 distance
    head = O.akl_head(pt, mu)
    gap = np.abs(pt - ps)
    for r in range(6):
        assert gap[r][head[r]].sum() + gap[r][~head[r]].sum() == pytest.approx(cityblock(pt[r], ps[r]), rel=1e-13)
    assert np.abs(g.sum(axis=1)).max() < 1e-14               # softmax tangent space


def test_reduces_to_fkl_or_rkl_when_one_gap_vanishes():
    rng = np.random.default_rng(8)
    V = 30
    z_t = 0.7 * rng.standard_normal((4, V))
    pt = sps.softmax(z_t, axis=1)
    head = O.akl_head(pt, 0.5)
    assert (head.sum(axis=1) >= 2).all() and ((~head).sum(axis=1) >= 2).all()
    for which, differs_on in (("fkl", head), ("rkl", ~head)):
        # the student equals the teacher except on one part, where the part's mass is redistributed:
        # the other part's gap vanishes and all the weight goes to one divergence
        ps = pt.copy()
        for r in range(4):
            part = np.flatnonzero(differs_on[r])
            w = rng.random(len(part)) + 0.1
            ps[r, part] = w / w.sum() * pt[r, part].sum()
        l, g = O.divergence_rows(z_t, np.log(ps), 1.0, O.AKL, 0.5)
        for r in range(4):
            want = sst.entropy(pt[r], ps[r]) if which == "fkl" else sst.entropy(ps[r], pt[r])
            assert l[r] == pytest.approx(want, rel=1e-12)
        if which == "fkl":                                   # textbook gradient of KL(p_t || softmax(z_s))
            assert np.abs(g - (ps - pt)).max() < 1e-15
    # identical distributions: both gaps vanish, loss 0, gradient 0
    l, g = O.divergence_rows(z_t, z_t, 1.0, O.AKL, 0.5)
    assert np.abs(l).max() < 1e-15 and np.abs(g).max() < 1e-15


def test_gradient_is_that_of_the_loss_with_the_weights_held_fixed():
    """The weights carry no gradient: the oracle's gradients must equal central differences of
    w_f KL(p_t || p_s) + w_r KL(p_s || p_t) with (w_f, w_r) frozen at their values at the point."""
    rng = np.random.default_rng(12)
    T, Ht, Hs, V = 3, 6, 5, 19
    h_t = rng.standard_normal((T, Ht)); W_t = 0.9 * rng.standard_normal((Ht, V))
    h_s = rng.standard_normal((T, Hs)); W_s = 0.6 * rng.standard_normal((Hs, V))
    mask = np.array([1, 0, 1], np.uint8); tau = 1.7; mu = 0.5
    pt = sps.softmax(h_t @ W_t / tau, axis=1)
    ps0 = sps.softmax(h_s @ W_s / tau, axis=1)
    w = [_brute_force_weights(list(pt[r]), list(ps0[r]), mu)[:2] for r in range(T)]

    def frozen_loss(hs, Ws):
        ps = sps.softmax(hs @ Ws / tau, axis=1)
        rows = [w[r][0] * sst.entropy(pt[r], ps[r]) + w[r][1] * sst.entropy(ps[r], pt[r]) for r in range(T)]
        return sum(m * x for m, x in zip(mask, rows)) / mask.sum()

    r = O.kd_loss_fwd_bwd(h_t, W_t, h_s, W_s, mask, tau, O.AKL, mu)
    assert r["loss"] == pytest.approx(frozen_loss(h_s, W_s), rel=1e-13)
    eps = 1e-6
    for name, x, grad in (("h_s", h_s, r["grad_h_s"]), ("W_s", W_s, r["grad_W_s"])):
        fd = np.zeros_like(x)
        for i in np.ndindex(*x.shape):
            up = x.copy(); up[i] += eps; dn = x.copy(); dn[i] -= eps
            fd[i] = ((frozen_loss(up, W_s) - frozen_loss(dn, W_s)) if name == "h_s" else
                     (frozen_loss(h_s, up) - frozen_loss(h_s, dn))) / (2 * eps)
        assert np.abs(fd - grad).max() < 2e-9, name
    assert (r["grad_h_s"][1] == 0).all()


def test_bounds_and_rejects_bad_mu():
    rng = np.random.default_rng(13)
    z_t = 3 * rng.standard_normal((5, 50)); z_s = rng.standard_normal((5, 50))
    l, _ = O.divergence_rows(z_t, z_s, 1.0, O.AKL, 0.5)
    f, _ = O.divergence_rows(z_t, z_s, 1.0, O.FKL); r, _ = O.divergence_rows(z_t, z_s, 1.0, O.RKL)
    assert (l >= np.minimum(f, r) - 1e-15).all() and (l <= np.maximum(f, r) + 1e-15).all()
    for mu in (0.0, 1.0):
        with pytest.raises(ValueError):
            O.divergence_rows(z_t, z_s, 1.0, O.AKL, mu)
