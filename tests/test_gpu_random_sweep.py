"""Seeded sweep over shapes, divergences, temperatures, masks and dtypes: every case is compared
element by element with the fp64 oracle.  Sizes are small (the oracle takes milliseconds) but cross
tile, chunk and split borders in irregular ways."""
import numpy as np
import pytest

from paper_2603_01875_amd import inputs as I
from tests import gpu_util as G

pytestmark = pytest.mark.gpu


def _case(seed):
    rng = np.random.default_rng(1000 + seed)
    kind = int(rng.integers(0, 6))
    cfg = I.KDConfig(
        name=f"sweep{seed}", batch=int(rng.integers(1, 4)), seq=int(rng.integers(1, 260)),
        H_t=8 * int(rng.integers(1, 40)), H_s=8 * int(rng.integers(1, 24)), V=8 * int(rng.integers(1, 400)),
        dtype=I.F32 if seed % 5 == 4 else I.BF16,
        w_t_std=float(rng.choice([0.02, 0.05, 0.2])), w_s_std=float(rng.choice([0.02, 0.06])),
        rms_norm=bool(rng.integers(0, 2)), kind=kind, tau=float(np.exp(rng.uniform(np.log(0.3), np.log(5.0)))),
        beta=float(rng.uniform(0.05, 0.95)), mask=str(rng.choice(["ones", "tail25", "bernoulli10"])), seed=5000 + seed)
    return cfg, int(rng.choice([256, 512, 1024, 16384]))


@pytest.mark.parametrize("seed", range(30))
def test_random_case(seed, monkeypatch):
    cfg, chunk = _case(seed)
    monkeypatch.setenv("KD_VOCAB_CHUNK", str(chunk))
    data = I.generate(cfg)
    if seed % 7 == 3:                                  # sparse mask: most tokens dropped
        rng = np.random.default_rng(seed)
        data["mask"] = (rng.random(cfg.T) < 0.15).astype(np.uint8)
    extra = G.tvd_tie_allowance(cfg, data) if cfg.kind == I.TVD else None
    out = G.run_gpu(cfg, data)
    what = (f"seed={seed} T={cfg.T} H_t={cfg.H_t} H_s={cfg.H_s} V={cfg.V} kind={cfg.kind} tau={cfg.tau:.3f} "
            f"beta={cfg.beta:.2f} dtype={cfg.dtype} mask={cfg.mask} chunk={chunk}")
    G.check(out, G.run_oracle(cfg, data), what, extra)
