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


def test_e4m3_table_and_quantiser():
    """The e4m3 helpers used to build fp8 teacher inputs: table against the format's definition,
    quantiser against torch's float8_e4m3fn cast (a library routine) and hand-picked ties."""
    import torch
    tab = I.e4m3_values()
    assert tab[0x00] == 0.0 and tab[0x01] == 2.0 ** -9 and tab[0x07] == 7 * 2.0 ** -9
    assert tab[0x08] == 2.0 ** -6 and tab[0x38] == 1.0 and tab[0x7e] == 448.0
    assert np.isnan(tab[0x7f]) and np.isnan(tab[0xff]) and tab[0xb8] == -1.0
    assert (np.diff(tab[:127]) > 0).all()
    codes = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float32).numpy()
    np.testing.assert_array_equal(np.nan_to_num(codes, nan=-7.0), np.nan_to_num(tab, nan=-7.0).astype(np.float32))
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.standard_normal(200000) * 50, rng.standard_normal(50000) * 0.01,
                        np.array([0.0, -0.0, 1.0625, 1.1875, 2.0 ** -10, 3 * 2.0 ** -10, 447.9, 448.0])]).astype(np.float32)
    mine = I.quantize_e4m3(x, 1.0)
    ref = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    inside = np.abs(x) <= 448
    np.testing.assert_array_equal(mine[inside], ref[inside])
    # ties go to the even code; beyond the largest value the quantiser saturates; NaN keeps its sign
    np.testing.assert_array_equal(I.quantize_e4m3(np.array([1.0625, 1.1875, 2.0 ** -10, 500.0, -1e9], np.float32), 1.0),
                                  np.array([0x38, 0x3a, 0x00, 0x7e, 0xfe], np.uint8))
    assert I.quantize_e4m3(np.array([np.nan], np.float32), 1.0)[0] & 0x7f == 0x7f
    # scale: codes of x / s
    np.testing.assert_array_equal(I.quantize_e4m3(np.array([0.5, -3.0], np.float32), 0.25), np.array([0x40, 0xd4], np.uint8))


def test_fp8_teacher_inputs_roundtrip():
    cfg = I.scaled(I.workload("fkl_bf16"), batch=1, seq=64, H_t=128, H_s=64, V=512)
    data = I.generate(cfg)
    f8 = I.fp8_teacher(data)
    for k in ("h_t", "W_t"):
        assert f8["q_" + k].dtype == np.uint8 and f8["q_" + k].shape == data[k].shape
        # three mantissa bits: relative error at most 2^-4 for values in the normal range
        big = np.abs(data[k]) > f8["scale_" + k] * 2.0 ** -6
        assert (np.abs(f8[k] - data[k])[big] <= 2.0 ** -4 * np.abs(data[k])[big] * 1.0001).all()
        assert np.abs(f8[k]).max() <= np.abs(data[k]).max() * 1.0001
