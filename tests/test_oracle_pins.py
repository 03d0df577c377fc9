"""Pins for the fp64 oracle: nothing here calls the oracle to make its own
expected value.  Expected values come from closed forms, library routines for
special cases, inequalities, and finite differences of the loss."""
import numpy as np
import pytest
import scipy.special as sps
import scipy.stats as sst
from scipy.spatial.distance import jensenshannon

from oracle import kd_oracle as O


def _rand_problem(rng, T=5, Ht=7, Hs=4, V=33, wt=0.7, ws=0.5):
    return dict(h_t=rng.standard_normal((T, Ht)), W_t=wt * rng.standard_normal((Ht, V)),
                h_s=rng.standard_normal((T, Hs)), W_s=ws * rng.standard_normal((Hs, V)))


KINDS = [(O.FKL, 0.5), (O.RKL, 0.5), (O.JSD, 0.5), (O.JSD, 0.1), (O.JSD, 0.8),
         (O.TVD, 0.5), (O.SKEW_FKL, 0.1), (O.SKEW_FKL, 0.6), (O.SKEW_RKL, 0.1), (O.SKEW_RKL, 0.6)]


# ---- 1. teacher == student -> 0 and zero gradient ---------------------------------------
@pytest.mark.parametrize("kind,beta", KINDS)
def test_identical_models_give_zero(kind, beta):
    rng = np.random.default_rng(1)
    h = rng.standard_normal((6, 5)); W = rng.standard_normal((5, 40))
    r = O.kd_loss_fwd_bwd(h, W, h, W, None, 1.7, kind, beta)
    assert abs(r["loss"]) < 1e-14
    assert np.abs(r["grad_h_s"]).max() < 1e-14 and np.abs(r["grad_W_s"]).max() < 1e-14


# ---- 2. inequalities -----------------------------------------------------------------------
@pytest.mark.parametrize("kind,beta", KINDS)
@pytest.mark.parametrize("tau", [0.5, 1.0, 3.0])
def test_bounds(kind, beta, tau):
    rng = np.random.default_rng(2)
    z_t = 4 * rng.standard_normal((50, 64)); z_s = 2 * rng.standard_normal((50, 64))
    l, g = O.divergence_rows(z_t, z_s, tau, kind, beta)
    assert (l >= -1e-15).all()
    if kind == O.JSD:
        bound = -beta * np.log(beta) - (1 - beta) * np.log1p(-beta)
        assert (l <= bound + 1e-12).all() and bound <= np.log(2) + 1e-15
    # softmax tangent space: every gradient row sums to zero
    assert np.abs(g.sum(axis=1)).max() < 1e-12


def test_tvd_and_skewed_kl_against_library_routines():
    from scipy.spatial.distance import cityblock
    rng = np.random.default_rng(21)
    z_t = 2 * rng.standard_normal((6, 40)); z_s = rng.standard_normal((6, 40)); tau = 1.5
    pt = sps.softmax(z_t / tau, axis=1); ps = sps.softmax(z_s / tau, axis=1)
    tv, _ = O.divergence_rows(z_t, z_s, tau, O.TVD)
    fkl, _ = O.divergence_rows(z_t, z_s, tau, O.FKL)
    for i in range(6):
        assert abs(tv[i] - 0.5 * cityblock(pt[i], ps[i])) < 1e-14
        assert 0 <= tv[i] <= 1 and tv[i] <= np.sqrt(fkl[i] / 2) + 1e-12        # Pinsker
    for a in (0.1, 0.6):
        sf, _ = O.divergence_rows(z_t, z_s, tau, O.SKEW_FKL, a)
        sr, _ = O.divergence_rows(z_t, z_s, tau, O.SKEW_RKL, a)
        for i in range(6):
            assert abs(sf[i] - sst.entropy(pt[i], a * pt[i] + (1 - a) * ps[i])) < 1e-13
            assert abs(sr[i] - sst.entropy(ps[i], (1 - a) * pt[i] + a * ps[i])) < 1e-13
    # alpha -> 0 recovers the plain divergences; the skew always shrinks them
    rkl, _ = O.divergence_rows(z_t, z_s, tau, O.RKL)
    sf, _ = O.divergence_rows(z_t, z_s, tau, O.SKEW_FKL, 1e-9)
    sr, _ = O.divergence_rows(z_t, z_s, tau, O.SKEW_RKL, 1e-9)
    assert np.allclose(sf, fkl, rtol=1e-6) and np.allclose(sr, rkl, rtol=1e-6)
    sf, _ = O.divergence_rows(z_t, z_s, tau, O.SKEW_FKL, 0.3)
    assert (sf < fkl).all()
    # disjoint supports: TVD = 1
    a = np.array([[300.0, 0.0, -300.0, -300.0]]); b = np.array([[-300.0, -300.0, 0.0, 300.0]])
    tv, _ = O.divergence_rows(a, b, 1.0, O.TVD)
    assert abs(tv[0] - 1.0) < 1e-12


def test_jsd_reaches_its_bound_for_disjoint_supports():
    z_t = np.array([[200.0, 0.0, -200.0, -200.0]]); z_s = np.array([[-200.0, -200.0, 0.0, 200.0]])
    for beta in (0.5, 0.1):
        l, _ = O.divergence_rows(z_t, z_s, 1.0, O.JSD, beta)
        bound = -beta * np.log(beta) - (1 - beta) * np.log1p(-beta)
        assert abs(l[0] - bound) < 1e-12


# ---- 3. library routines on special cases ---------------------------------------------------
def test_fkl_rkl_match_scipy_entropy():
    rng = np.random.default_rng(3)
    z_t = 2 * rng.standard_normal((9, 31)); z_s = rng.standard_normal((9, 31)); tau = 1.3
    pt = sps.softmax(z_t / tau, axis=1); ps = sps.softmax(z_s / tau, axis=1)
    lf, _ = O.divergence_rows(z_t, z_s, tau, O.FKL)
    lr, _ = O.divergence_rows(z_t, z_s, tau, O.RKL)
    for i in range(9):
        assert abs(lf[i] - sst.entropy(pt[i], ps[i])) < 1e-12     # KL(pt||ps)
        assert abs(lr[i] - sst.entropy(ps[i], pt[i])) < 1e-12


def test_jsd_half_matches_scipy_jensenshannon():
    rng = np.random.default_rng(4)
    z_t = 2 * rng.standard_normal((7, 20)); z_s = rng.standard_normal((7, 20))
    pt = sps.softmax(z_t, axis=1); ps = sps.softmax(z_s, axis=1)
    l, _ = O.divergence_rows(z_t, z_s, 1.0, O.JSD, 0.5)
    for i in range(7):
        assert abs(l[i] - jensenshannon(pt[i], ps[i]) ** 2) < 1e-12


def test_jsd_beta_weights_by_hand():
    # written out independently: beta on the teacher term, M = beta pt + (1-beta) ps
    rng = np.random.default_rng(5)
    z_t = rng.standard_normal((3, 11)); z_s = rng.standard_normal((3, 11)); beta = 0.3
    pt = sps.softmax(z_t, axis=1); ps = sps.softmax(z_s, axis=1)
    M = beta * pt + (1 - beta) * ps
    want = beta * sps.rel_entr(pt, M).sum(1) + (1 - beta) * sps.rel_entr(ps, M).sum(1)
    l, _ = O.divergence_rows(z_t, z_s, 1.0, O.JSD, beta)
    assert np.abs(l - want).max() < 1e-13


def test_v2_is_bernoulli_kl_of_sigmoids():
    a, b, tau = 0.9, -0.4, 0.7          # logit gaps
    z_t = np.array([[a, 0.0]]); z_s = np.array([[b, 0.0]])
    p = sps.expit(a / tau); q = sps.expit(b / tau)
    want = p * np.log(p / q) + (1 - p) * np.log((1 - p) / (1 - q))
    l, _ = O.divergence_rows(z_t, z_s, tau, O.FKL)
    assert abs(l[0] - want) < 1e-14
    l, _ = O.divergence_rows(z_t, z_s, tau, O.RKL)
    want_r = q * np.log(q / p) + (1 - q) * np.log((1 - q) / (1 - p))
    assert abs(l[0] - want_r) < 1e-14


def test_one_hot_teacher_limit_is_cross_entropy():
    rng = np.random.default_rng(6)
    z_s = rng.standard_normal((4, 30)); z_t = rng.standard_normal((4, 30))
    l, _ = O.divergence_rows(1e4 * z_t, z_s, 1.0, O.FKL)
    ce = -(sps.log_softmax(z_s, axis=1)[np.arange(4), z_t.argmax(1)])
    assert np.abs(l - ce).max() < 1e-9


def test_high_temperature_decay():
    rng = np.random.default_rng(7)
    z_t = rng.standard_normal((3, 40)); z_s = rng.standard_normal((3, 40))
    for kind, beta in KINDS:
        l1, _ = O.divergence_rows(z_t, z_s, 100.0, kind, beta)
        l2, _ = O.divergence_rows(z_t, z_s, 200.0, kind, beta)
        want = 2.0 if kind == O.TVD else 4.0             # KL-type: O(1/tau^2); TVD is a norm: O(1/tau)
        assert np.allclose(l1 / l2, want, rtol=2e-2)


def test_jsd_role_swap_and_small_beta_limit():
    rng = np.random.default_rng(8)
    z_t = 2 * rng.standard_normal((5, 25)); z_s = rng.standard_normal((5, 25))
    a, _ = O.divergence_rows(z_t, z_s, 1.0, O.JSD, 0.2)
    b, _ = O.divergence_rows(z_s, z_t, 1.0, O.JSD, 0.8)
    assert np.abs(a - b).max() < 1e-13
    # beta -> 0: JSD_beta / beta -> KL(pt || ps)  (beta weighs the TEACHER term)
    beta = 1e-6
    j, _ = O.divergence_rows(z_t, z_s, 1.0, O.JSD, beta)
    pt = sps.softmax(z_t, axis=1); ps = sps.softmax(z_s, axis=1)
    fkl = sps.rel_entr(pt, ps).sum(1); rkl = sps.rel_entr(ps, pt).sum(1)
    assert np.allclose(j / beta, fkl, rtol=1e-4)
    assert not np.allclose(j / beta, rkl, rtol=1e-2)


def test_gaussian_regime_value():
    # independent Gaussian logits with small std: FKL ~= RKL ~= (s_t^2 + s_s^2)/2
    rng = np.random.default_rng(9)
    V = 20000; st, ss = 0.32, 0.23
    z_t = st * rng.standard_normal((8, V)); z_s = ss * rng.standard_normal((8, V))
    for kind in (O.FKL, O.RKL):
        l, _ = O.divergence_rows(z_t, z_s, 1.0, kind)
        assert abs(l.mean() - (st ** 2 + ss ** 2) / 2) < 0.05 * (st ** 2 + ss ** 2) / 2


def test_underflowed_probabilities_contribute_zero():
    z_t = np.array([[0.0, -2000.0, 5.0]]); z_s = np.array([[1.0, 3.0, -3000.0]])
    for kind, beta in KINDS:
        l, g = O.divergence_rows(z_t, z_s, 1.0, kind, beta)
        assert np.isfinite(l).all() and np.isfinite(g).all()


# ---- 4. gradients: closed form and finite differences -------------------------------------
def test_fkl_gradient_closed_form():
    rng = np.random.default_rng(10)
    p = _rand_problem(rng); tau = 1.6
    mask = np.array([1, 0, 1, 1, 0], dtype=np.uint8)
    z_t = p["h_t"] @ p["W_t"]; z_s = p["h_s"] @ p["W_s"]
    _, _, dz = O.kd_loss_from_logits(z_t, z_s, mask, tau, O.FKL)
    want = (sps.softmax(z_s / tau, axis=1) - sps.softmax(z_t / tau, axis=1)) / tau
    want = want * (mask[:, None] / mask.sum())
    assert np.abs(dz - want).max() < 1e-15
    assert (dz[mask == 0] == 0).all()


def _loss_only(p, mask, tau, kind, beta, layout=O.W_HV):
    return O.kd_loss_fwd_bwd(p["h_t"], p["W_t"], p["h_s"], p["W_s"], mask, tau, kind, beta, layout)["loss"]


@pytest.mark.parametrize("kind,beta", KINDS)
@pytest.mark.parametrize("tau", [1.0, 2.5])
def test_gradients_match_central_differences(kind, beta, tau):
    rng = np.random.default_rng(11)
    p = _rand_problem(rng, T=3, Ht=6, Hs=5, V=17)
    mask = np.array([1, 1, 0], dtype=np.uint8)
    r = O.kd_loss_fwd_bwd(p["h_t"], p["W_t"], p["h_s"], p["W_s"], mask, tau, kind, beta)
    eps = 1e-6
    for name, grad in (("h_s", r["grad_h_s"]), ("W_s", r["grad_W_s"])):
        fd = np.zeros_like(p[name])
        it = np.nditer(p[name], flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            q = {k: v.copy() for k, v in p.items()}
            q[name][i] += eps; up = _loss_only(q, mask, tau, kind, beta)
            q[name][i] -= 2 * eps; dn = _loss_only(q, mask, tau, kind, beta)
            fd[i] = (up - dn) / (2 * eps)
        assert np.abs(fd - grad).max() < 2e-9, name
    assert (r["grad_h_s"][2] == 0).all()            # masked token: exactly zero row


@pytest.mark.parametrize("kind,beta", KINDS)
def test_directional_derivative_medium(kind, beta):
    rng = np.random.default_rng(12)
    p = _rand_problem(rng, T=40, Ht=24, Hs=16, V=300)
    mask = (rng.random(40) > 0.2).astype(np.uint8)
    r = O.kd_loss_fwd_bwd(p["h_t"], p["W_t"], p["h_s"], p["W_s"], mask, 1.2, kind, beta, row_block=16)
    dh = rng.standard_normal(p["h_s"].shape); dW = rng.standard_normal(p["W_s"].shape)
    eps = 1e-5
    up = dict(p, h_s=p["h_s"] + eps * dh, W_s=p["W_s"] + eps * dW)
    dn = dict(p, h_s=p["h_s"] - eps * dh, W_s=p["W_s"] - eps * dW)
    fd = (_loss_only(up, mask, 1.2, kind, beta) - _loss_only(dn, mask, 1.2, kind, beta)) / (2 * eps)
    an = (r["grad_h_s"] * dh).sum() + (r["grad_W_s"] * dW).sum()
    assert abs(fd - an) < 1e-8 * max(1.0, abs(an))


# ---- 5. structure: equivalence, layouts, blocking, masks ------------------------------------
@pytest.mark.parametrize("kind,beta", KINDS)
def test_hidden_state_path_equals_logit_path(kind, beta):
    # Sec. 3.2: recomputing logits from hidden states is the same as standard logit KD
    rng = np.random.default_rng(13)
    p = _rand_problem(rng, T=9, V=50)
    mask = (rng.random(9) > 0.3).astype(np.uint8)
    a = O.kd_loss_fwd_bwd(p["h_t"], p["W_t"], p["h_s"], p["W_s"], mask, 0.9, kind, beta, row_block=4)
    loss, l, dz = O.kd_loss_from_logits(p["h_t"] @ p["W_t"], p["h_s"] @ p["W_s"], mask, 0.9, kind, beta)
    assert a["loss"] == pytest.approx(loss, abs=1e-15)
    assert np.abs(a["grad_h_s"] - dz @ p["W_s"].T).max() < 1e-15
    assert np.abs(a["grad_W_s"] - p["h_s"].T @ dz).max() < 1e-15


def test_layout_flag_and_row_blocking_do_not_change_results():
    rng = np.random.default_rng(14)
    p = _rand_problem(rng, T=11, V=37)
    a = O.kd_loss_fwd_bwd(p["h_t"], p["W_t"], p["h_s"], p["W_s"], None, 1.0, O.JSD, 0.3, O.W_HV, row_block=512)
    b = O.kd_loss_fwd_bwd(p["h_t"], p["W_t"].T.copy(), p["h_s"], p["W_s"].T.copy(), None, 1.0, O.JSD, 0.3,
                          O.W_VH, row_block=3)
    assert a["loss"] == pytest.approx(b["loss"], abs=1e-15)
    assert np.abs(a["grad_W_s"] - b["grad_W_s"].T).max() < 1e-15
    assert np.abs(a["grad_h_s"] - b["grad_h_s"]).max() < 1e-15


def test_mask_semantics():
    rng = np.random.default_rng(15)
    p = _rand_problem(rng, T=6)
    mask = np.array([1, 0, 0, 1, 1, 0], dtype=np.uint8)
    full = O.kd_loss_fwd_bwd(p["h_t"], p["W_t"], p["h_s"], p["W_s"], mask, 1.0, O.FKL)
    keep = mask.astype(bool)
    sub = O.kd_loss_fwd_bwd(p["h_t"][keep], p["W_t"], p["h_s"][keep], p["W_s"], None, 1.0, O.FKL)
    assert full["loss"] == pytest.approx(sub["loss"], abs=1e-15)      # masked mean == mean over kept rows
    assert np.abs(full["grad_W_s"] - sub["grad_W_s"]).max() < 1e-15
    assert (full["grad_h_s"][~keep] == 0).all()
    none = O.kd_loss_fwd_bwd(p["h_t"], p["W_t"], p["h_s"], p["W_s"], np.zeros(6, np.uint8), 1.0, O.RKL)
    assert none["loss"] == 0.0 and not none["grad_h_s"].any() and not none["grad_W_s"].any()


def test_row_lse_matches_scipy():
    rng = np.random.default_rng(16)
    h = rng.standard_normal((7, 5)); W = rng.standard_normal((5, 60))
    assert np.abs(O.row_lse(h, W, 1.4, row_block=3) - sps.logsumexp(h @ W / 1.4, axis=1)).max() < 1e-13


def test_planted_mistakes_are_caught():
    """A wrong sign, a dropped 1/tau, or swapped JSD weights must move the result
    far outside every tolerance used above (guards against vacuous pins)."""
    rng = np.random.default_rng(17)
    z_t = 2 * rng.standard_normal((4, 20)); z_s = rng.standard_normal((4, 20)); tau = 2.0
    pt = sps.softmax(z_t / tau, axis=1); ps = sps.softmax(z_s / tau, axis=1)
    _, _, dz = O.kd_loss_from_logits(z_t, z_s, None, tau, O.FKL)
    good = (ps - pt) / tau / 4
    assert np.abs(dz - good).max() < 1e-15
    assert np.abs(dz - (pt - ps) / tau / 4).max() > 1e-3           # sign
    assert np.abs(dz - (ps - pt) / 4).max() > 1e-3                 # dropped 1/tau
    l, _ = O.divergence_rows(z_t, z_s, tau, O.JSD, 0.2)
    M = 0.8 * pt + 0.2 * ps                                        # weights on the wrong side
    wrong = 0.8 * sps.rel_entr(pt, M).sum(1) + 0.2 * sps.rel_entr(ps, M).sum(1)
    assert np.abs(l - wrong).max() > 1e-3


# ---- multi-teacher and tau^2 conventions (defined by linearity; checked by finite differences) ------
def _multi_loss(ps_, h_s, W_s, mask, tau, kind, beta, weights):
    return sum(w * O.kd_loss_fwd_bwd(p["h_t"], p["W_t"], h_s, W_s, mask, tau, kind, beta)["loss"]
               for w, p in zip(weights, ps_))


def test_multi_teacher_gradient_is_gradient_of_weighted_sum():
    rng = np.random.default_rng(31)
    teachers = [dict(h_t=rng.standard_normal((3, 5)), W_t=0.7 * rng.standard_normal((5, 13))),
                dict(h_t=rng.standard_normal((3, 8)), W_t=0.4 * rng.standard_normal((8, 13)))]
    h_s = rng.standard_normal((3, 4)); W_s = 0.5 * rng.standard_normal((4, 13))
    mask = np.array([1, 0, 1], np.uint8); w = (0.3, 1.7)
    r = O.kd_loss_multi([t["h_t"] for t in teachers], [t["W_t"] for t in teachers], w, h_s, W_s, mask, 1.4, O.JSD, 0.3)
    assert r["loss"] == pytest.approx(_multi_loss(teachers, h_s, W_s, mask, 1.4, O.JSD, 0.3, w), abs=1e-15)
    eps = 1e-6
    fd = np.zeros_like(W_s)
    for i in np.ndindex(*W_s.shape):
        up = W_s.copy(); up[i] += eps; dn = W_s.copy(); dn[i] -= eps
        fd[i] = (_multi_loss(teachers, h_s, up, mask, 1.4, O.JSD, 0.3, w) -
                 _multi_loss(teachers, h_s, dn, mask, 1.4, O.JSD, 0.3, w)) / (2 * eps)
    assert np.abs(fd - r["grad_W_s"]).max() < 2e-9
    # tau^2 convention: exactly tau^2 times everything
    a = O.kd_loss_fwd_bwd(teachers[0]["h_t"], teachers[0]["W_t"], h_s, W_s, mask, 1.4, O.FKL)
    b = O.kd_loss_fwd_bwd(teachers[0]["h_t"], teachers[0]["W_t"], h_s, W_s, mask, 1.4, O.FKL, tau2=True)
    assert b["loss"] == pytest.approx(1.96 * a["loss"], rel=1e-14)
    assert np.allclose(b["grad_h_s"], 1.96 * a["grad_h_s"], rtol=1e-13, atol=0)


def test_tau2_convention_by_finite_differences_and_high_temperature_limit():
    """tau2=True: the returned gradients are the derivatives of the returned (tau^2-scaled) loss, and the
    scaled loss has the textbook high-temperature limit: tau^2 KL(p_t || p_s) -> Var_v(z_t - z_s) / 2
    (variance over the vocabulary under the uniform distribution), independent of tau."""
    rng = np.random.default_rng(41)
    p = _rand_problem(rng, T=3, Ht=6, Hs=5, V=17)
    mask = np.array([1, 0, 1], dtype=np.uint8)
    tau = 2.5

    def f(q, kind):
        return O.kd_loss_fwd_bwd(q["h_t"], q["W_t"], q["h_s"], q["W_s"], mask, tau, kind, 0.3, tau2=True)
    eps = 1e-6
    for kind in (O.FKL, O.JSD):
        r = f(p, kind)
        for name, grad in (("h_s", r["grad_h_s"]), ("W_s", r["grad_W_s"])):
            fd = np.zeros_like(p[name])
            for i in np.ndindex(*p[name].shape):
                q = {k: v.copy() for k, v in p.items()}
                q[name][i] += eps; up = f(q, kind)["loss"]
                q[name][i] -= 2 * eps; dn = f(q, kind)["loss"]
                fd[i] = (up - dn) / (2 * eps)
            assert np.abs(fd - grad).max() < 1e-8, (kind, name)
    z_t = p["h_t"] @ p["W_t"]; z_s = p["h_s"] @ p["W_s"]
    want = 0.5 * np.var(z_t - z_s, axis=1)
    for big_tau in (1e3, 1e4):
        r = O.kd_loss_fwd_bwd(p["h_t"], p["W_t"], p["h_s"], p["W_s"], None, big_tau, O.FKL, tau2=True)
        assert np.allclose(r["per_token_loss"], want, rtol=5e-3 if big_tau == 1e3 else 5e-4)
    plain = O.kd_loss_fwd_bwd(p["h_t"], p["W_t"], p["h_s"], p["W_s"], None, 1e3, O.FKL)
    assert np.all(plain["per_token_loss"] < 1e-5 * want)          # without the factor the loss decays as 1 / tau^2
