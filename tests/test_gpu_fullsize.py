"""Parity at the benchmark's full sizes, in the launch configuration bench.py times.

Every element of every output (loss, all per-token losses, all of grad_h_s, all of grad_W_s) is
compared with the complete fp64 oracle for fkl_bf16 (the headline), rkl_bf16, jsd_bf16 and
large_teacher at their full sizes.  long_peaked (T = 32768) would cost the oracle 173 TFLOP in
fp64 (a quarter of an hour on the host), so it is checked in two parts: its first 2048 tokens as a
problem of its own (full V and H, the vocabulary chunk of the full-size plan), every element; and
the full-T launch on sampled token rows that the oracle computes one by one.  Sampled rows of
grad_W_s at full T would need the log-sum-exps of all 32768 rows (92 TFLOP in fp64) and are not
checked there.
"""
import time

import numpy as np
import pytest

from oracle import kd_oracle as O
from paper_2603_01875_amd import inputs as I
from tests import gpu_util as G

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["fkl_bf16", "jsd_bf16"])
def test_medium_problem_full_oracle(name):
    cfg = I.scaled(I.workload(name), batch=4, seq=250, H_t=512, H_s=256, V=32776)
    data = I.generate(cfg)
    out = G.run_gpu(cfg, data)
    G.check(out, G.run_oracle(cfg, data), f"medium {name}")


def _every_element(name, cfg, data, **kw):
    t0 = time.perf_counter()
    out = G.run_gpu(cfg, data, **kw)
    ws_bytes = out["workspace"].numel()
    t1 = time.perf_counter()
    ref = G.run_oracle(cfg, data)
    t2 = time.perf_counter()
    rel = G.check(out, ref, name)
    print(f"[{name}] T={cfg.T} V={cfg.V}: GPU call {t1 - t0:.1f} s, oracle {t2 - t1:.1f} s, compare "
          f"{time.perf_counter() - t2:.1f} s, loss {ref['loss']:.6f} (rel err {rel:.1e}), n={ref['n']}", flush=True)
    assert ws_bytes < 0.35 * 2 * cfg.T * cfg.V            # never a [T, V] buffer
    return out, ref


@pytest.mark.parametrize("name", ["fkl_bf16", "rkl_bf16", "jsd_bf16", "large_teacher"])
def test_full_size_every_element(name):
    """The complete oracle on the complete workload; nothing rests on a sum or a norm."""
    cfg = I.workload(name)
    data = I.generate(cfg)
    out, ref = _every_element(name, cfg, data)
    if name == "fkl_bf16":
        assert abs(ref["loss"] - 1.02) < 0.03              # Gaussian-regime value (sigma_t^2 + sigma_s^2) / 2
    keep = data["mask"].astype(bool)
    assert (G.to_host(out["grad_h_s"])[~keep] == 0).all()  # masked tokens: exactly zero rows
    assert (G.to_host(out["per_token_loss"])[~keep] == 0).all()


@pytest.fixture(scope="module")
def long_peaked():
    cfg = I.workload("long_peaked")
    return cfg, I.generate(cfg)


def test_long_peaked_first_2048_tokens_every_element(long_peaked):
    """T = 2048 rows of the long-sequence workload as a self-contained problem (full V, H_t, H_s), with the
    vocabulary chunk the library uses at the full T = 32768, against the complete oracle."""
    from paper_2603_01875_amd import kdloss as K
    full_cfg, full = long_peaked
    vc_full, _ = K.kd_loss_plan_info(K.make_params(full_cfg.T, full_cfg.H_t, full_cfg.H_s, full_cfg.V,
                                                    full_cfg.kind, full_cfg.tau, full_cfg.beta))
    cfg = I.scaled(full_cfg, seq=2048)
    data = dict(h_t=full["h_t"][:2048], h_s=full["h_s"][:2048], W_t=full["W_t"], W_s=full["W_s"],
                mask=full["mask"][:2048])
    _, ref = _every_element("long_peaked[:2048]", cfg, data, vocab_chunk=vc_full)
    assert (ref["per_token_loss"] <= 0.3251 + 1e-9).all()  # JSD_0.1 <= H(0.1), near one-hot teacher


def _sampled_rows_check(cfg, data, out, rows):
    """Per-token loss and grad_h_s rows of the sampled tokens, computed by the oracle row by row
    (the vocabulary axis is walked in chunks only to bound the fp64 copies of the heads)."""
    n = float(data["mask"].sum())
    ht = data["h_t"][rows].astype(np.float64); hs = data["h_s"][rows].astype(np.float64)
    z_t = np.empty((len(rows), cfg.V)); z_s = np.empty((len(rows), cfg.V))
    for v0 in range(0, cfg.V, 16384):
        z_t[:, v0:v0 + 16384] = ht @ data["W_t"][v0:v0 + 16384].astype(np.float64).T
        z_s[:, v0:v0 + 16384] = hs @ data["W_s"][v0:v0 + 16384].astype(np.float64).T
    l, g = O.divergence_rows(z_t, z_s, cfg.tau, cfg.kind, cfg.beta)
    ptl = G.to_host(out["per_token_loss"])[rows]
    l = l * (data["mask"][rows] != 0)              # masked tokens are reported as 0
    assert np.abs(ptl - l).max() <= 1e-3 * np.abs(l).max()
    dz = (data["mask"][rows].astype(np.float64) / (n * cfg.tau))[:, None] * g
    gh_ref = np.zeros((len(rows), cfg.H_s))
    for v0 in range(0, cfg.V, 16384):
        gh_ref += dz[:, v0:v0 + 16384] @ data["W_s"][v0:v0 + 16384].astype(np.float64)
    gh = G.to_host(out["grad_h_s"][torch_index(rows)])
    assert np.abs(gh - gh_ref).max() <= G.GRAD_TOL * np.abs(gh_ref).max()
    return l


def torch_index(rows):
    import torch
    return torch.from_numpy(np.asarray(rows, dtype=np.int64)).cuda()


def test_long_peaked_full_T_sampled_token_rows(long_peaked):
    """The full T = 32768 launch: per-token loss and grad_h_s of sampled tokens (first, last, tile borders,
    random ones) against the oracle, every output finite, and the mean of the per-token losses."""
    import torch
    cfg, data = long_peaked
    out = G.run_gpu(cfg, data)
    rng = np.random.default_rng(5)
    rows = np.array([0, 255, 256, cfg.T // 2 + 1, cfg.T - 257, cfg.T - 1] + list(rng.integers(0, cfg.T, 10)))
    l = _sampled_rows_check(cfg, data, out, rows)
    assert (l <= 0.3251 + 1e-6).all()
    ptl = out["per_token_loss"].double()
    assert torch.isfinite(ptl).all() and float(ptl.max()) <= 0.3251 + 1e-5 and float(ptl.min()) >= 0.0
    loss = float(out["loss"].item())
    assert abs(loss - float(ptl.mean())) <= 1e-5 * abs(loss)
    assert torch.isfinite(out["grad_h_s"]).all() and torch.isfinite(out["grad_W_s"]).all()


def test_headline_workload_with_fp8_teacher():
    """The benchmark's optional fp8 mode at full size, against the complete oracle on the de-quantised
    teacher (the exact values the e4m3 codes stand for)."""
    import torch
    from paper_2603_01875_amd import kdloss as K
    cfg = I.workload("fkl_bf16")
    data = I.generate(cfg)
    f8 = G.fp8_teacher(data)
    out = K.kd_loss_fwd_bwd(torch.from_numpy(f8["q_h_t"]).cuda(), torch.from_numpy(f8["q_W_t"]).cuda(),
                            G.to_device(data["h_s"], cfg.dtype), G.to_device(data["W_s"], cfg.dtype),
                            torch.from_numpy(data["mask"]).cuda(), tau=cfg.tau, kind=cfg.kind, beta=cfg.beta,
                            flags=K.FLAG_TEACHER_FP8, teacher_scale=f8["teacher_scale"])
    torch.cuda.synchronize()
    d = dict(data); d["h_t"], d["W_t"] = f8["h_t"], f8["W_t"]
    G.check(out, G.run_oracle(cfg, d), "fkl_bf16 with fp8 teacher")
    assert abs(float(out["loss"].item()) - 1.02) < 0.03
