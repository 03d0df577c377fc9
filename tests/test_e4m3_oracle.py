"""Pins of the NumPy e4m3 reference (oracle/e4m3.py): the table against the format's definition and
torch's decoding, the quantiser against torch's float8_e4m3fn cast (a library routine) and hand-picked
ties, and the fp8 teacher operands the GPU tests are built from."""
import numpy as np

from oracle import e4m3 as E
from paper_2603_01875_amd import inputs as I
from tests import gpu_util as G


def test_e4m3_table_and_quantiser():
    """The e4m3 helpers used to build fp8 teacher inputs: table against the format's definition,
    quantiser against torch's float8_e4m3fn cast (a library routine) and hand-picked ties."""
    import torch
    tab = E.e4m3_values()
    assert tab[0x00] == 0.0 and tab[0x01] == 2.0 ** -9 and tab[0x07] == 7 * 2.0 ** -9
    assert tab[0x08] == 2.0 ** -6 and tab[0x38] == 1.0 and tab[0x7e] == 448.0
    assert np.isnan(tab[0x7f]) and np.isnan(tab[0xff]) and tab[0xb8] == -1.0
    assert (np.diff(tab[:127]) > 0).all()
    codes = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float32).numpy()
    np.testing.assert_array_equal(np.nan_to_num(codes, nan=-7.0), np.nan_to_num(tab, nan=-7.0).astype(np.float32))
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.standard_normal(200000) * 50, rng.standard_normal(50000) * 0.01,
                        np.array([0.0, -0.0, 1.0625, 1.1875, 2.0 ** -10, 3 * 2.0 ** -10, 447.9, 448.0])]).astype(np.float32)
    mine = E.quantize_e4m3(x, 1.0)
    ref = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    inside = np.abs(x) <= 448
    np.testing.assert_array_equal(mine[inside], ref[inside])
    # ties go to the even code; beyond the largest value the quantiser saturates; NaN keeps its sign
    np.testing.assert_array_equal(E.quantize_e4m3(np.array([1.0625, 1.1875, 2.0 ** -10, 500.0, -1e9], np.float32), 1.0),
                                  np.array([0x38, 0x3a, 0x00, 0x7e, 0xfe], np.uint8))
    assert E.quantize_e4m3(np.array([np.nan], np.float32), 1.0)[0] & 0x7f == 0x7f
    # scale: codes of x / s
    np.testing.assert_array_equal(E.quantize_e4m3(np.array([0.5, -3.0], np.float32), 0.25), np.array([0x40, 0xd4], np.uint8))


def test_fp8_teacher_inputs_roundtrip():
    cfg = I.scaled(I.workload("fkl_bf16"), batch=1, seq=64, H_t=128, H_s=64, V=512)
    data = I.generate(cfg)
    f8 = G.fp8_teacher(data)
    for k in ("h_t", "W_t"):
        assert f8["q_" + k].dtype == np.uint8 and f8["q_" + k].shape == data[k].shape
        # three mantissa bits: relative error at most 2^-4 for values in the normal range
        big = np.abs(data[k]) > f8["scale_" + k] * 2.0 ** -6
        assert (np.abs(f8[k] - data[k])[big] <= 2.0 ** -4 * np.abs(data[k])[big] * 1.0001).all()
        assert np.abs(f8[k]).max() <= np.abs(data[k]).max() * 1.0001
