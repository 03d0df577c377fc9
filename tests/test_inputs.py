import numpy as np
import torch

from paper_2603_01875_amd import inputs as I


def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(100000) * np.exp(rng.uniform(-20, 20, 100000))).astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    got = I.round_to_bf16(x)
    assert (got.view(np.uint32) == want.view(np.uint32)).all()
    assert (I.bits_to_f32(I.bf16_bits(got)).view(np.uint32) == got.view(np.uint32)).all()


def test_recipe_small():
    cfg = I.scaled(I.workload("fkl_bf16"), batch=4, seq=64, H_t=96, H_s=40, V=512)
    d = I.generate(cfg); d2 = I.generate(cfg)
    for k in d:
        assert (d[k] == d2[k]).all()                       # seeded
    assert d["h_t"].shape == (256, 96) and d["W_s"].shape == (512, 40)
    assert np.allclose((d["h_t"].astype(np.float64) ** 2).mean(1), 1.0, atol=5e-3)   # unit RMS (bf16)
    assert abs(d["W_t"].std() - 0.02) < 2e-3
    m = d["mask"].reshape(4, 64)
    for row in m:                                          # a tail of zeros, at most a quarter
        k = int((row == 0).sum())
        assert k <= 16 and (row[:64 - k] == 1).all() and (row[64 - k:] == 0).all()


def test_workload_table():
    w = I.workload("long_peaked")
    assert (w.T, w.H_t, w.H_s, w.V, w.kind, w.beta) == (32768, 5120, 4096, 151936, I.JSD, 0.1)
    w = I.workload("tiny_fkl_f32")
    assert (w.T, w.dtype, w.rms_norm) == (128, I.F32, False)
    d = I.generate(I.scaled(I.workload("large_teacher"), batch=1, seq=4000, H_t=8, H_s=8, V=8))
    assert 0.07 < 1 - d["mask"].mean() < 0.13
