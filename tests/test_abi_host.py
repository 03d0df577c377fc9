"""Host-only checks of the C ABI: the library loads without a GPU, exports every
symbol the header declares, and rejects bad arguments before touching a device."""
import ctypes
import os
import re

import pytest

from paper_2603_01875_amd import kdloss as K

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    src = open(os.path.join(ROOT, "include", "kdloss.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(kd_[a-z_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    names = _declared_symbols()
    assert {"kd_loss_workspace_size", "kd_loss_fwd_bwd", "kd_loss_fwd", "kd_status_string",
            "kd_loss_plan_info"} <= set(names)
    L = K.lib()
    for n in names:
        assert hasattr(L, n), n


def test_header_is_plain_c():
    """The boundary is a C ABI: the header must compile as C99 on its own."""
    import subprocess
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only", "-x", "c",
                        os.path.join(ROOT, "include", "kdloss.h")], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr


def test_struct_layout_matches_header():
    assert ctypes.sizeof(K.KdLossParams) == 4 * 8 + 10 * 4          # 72 bytes, no padding


def test_status_strings():
    for s in range(8):
        assert len(K.lib().kd_status_string(s)) > 0


def _ws(**kw):
    base = dict(T=4096, H_t=4096, H_s=1024, V=151936)
    base.update(kw)
    return K.make_params(**base)


def test_workspace_is_far_below_T_times_V():
    p = _ws()
    n = K.kd_loss_workspace_size(p)
    vc, launches = K.kd_loss_plan_info(p)
    assert n < 0.35 * 2 * 4096 * 151936           # never a [T, V] buffer
    assert vc % 256 == 0 and vc <= 16384 and launches > 0
    # long-sequence workload: chunk shrinks so the staging buffers stay bounded
    p5 = K.make_params(32768, 5120, 4096, 151936, kind=K.JSD, beta=0.1)
    n5 = K.kd_loss_workspace_size(p5)
    assert n5 < 0.3 * 2 * 32768 * 151936           # dz chunk copies, fp32 grad_h_s sums, compact hidden copies
    # the full-logit volume the paper quotes (footnote of Sec. 1, kept in tests/golden) against what this
    # library needs for the same number of tokens processed one 4096-token batch at a time
    seqs, toks, vocab, width, approx_gb = [int(x) for x in
        [l for l in open(os.path.join(ROOT, "tests", "golden", "full_logit_volume.txt")) if l[0] != "#"][0].split()]
    full = seqs * toks * vocab * width
    assert abs(full / 1e9 - approx_gb) < 0.01 * approx_gb and vocab == 151936
    assert full / n > 300


@pytest.mark.parametrize("kw,status", [
    (dict(T=0), 2), (dict(V=-8), 2), (dict(H_t=100), 3), (dict(V=151937), 3),
    (dict(tau=0.0), 4), (dict(tau=float("nan")), 4), (dict(kind=7), 4),
    (dict(kind=K.JSD, beta=0.0), 4), (dict(kind=K.JSD, beta=1.0), 4), (dict(kind=K.SKEW_FKL, beta=0.0), 4),
    (dict(kind=K.SKEW_RKL, beta=1.5), 4), (dict(kind=-1), 4), (dict(in_dtype=5), 4),
    # [H][V] heads: everything but the fp8 teacher
    (dict(w_layout=K.W_HV, flags=K.FLAG_TEACHER_FP8, teacher_scale=1.0), 6),
    # fp8 teacher: needs a positive finite scale, a bf16 student side and H_t % 128 == 0
    (dict(flags=K.FLAG_TEACHER_FP8), 4), (dict(flags=K.FLAG_TEACHER_FP8, teacher_scale=float("inf")), 4),
    (dict(flags=K.FLAG_TEACHER_FP8, teacher_scale=1.0, in_dtype=K.F32), 6),
    (dict(flags=K.FLAG_TEACHER_FP8, teacher_scale=1.0, H_t=4160), 3),
    (dict(flags=8), 4),
])
def test_bad_params_are_rejected(kw, status):
    with pytest.raises(K.KdLossError) as e:
        K.kd_loss_workspace_size(_ws(**kw))
    assert e.value.status == status


def test_fp32_and_odd_hidden_sizes_need_more_workspace():
    base = K.kd_loss_workspace_size(K.make_params(512, 256, 128, 4096))
    odd = K.kd_loss_workspace_size(K.make_params(512, 200, 72, 4096))          # K padded to 256 / 128
    f32 = K.kd_loss_workspace_size(K.make_params(512, 256, 128, 4096, in_dtype=K.F32))
    assert odd > base and f32 > odd


def test_both_head_layouts_are_accepted():
    base = K.kd_loss_workspace_size(_ws(w_layout=K.W_VH))
    assert K.kd_loss_workspace_size(_ws(w_layout=K.W_HV)) == base           # read in place
    # [H][V] heads that cannot be read in place (fp32, sizes off the 64-element grid) are re-packed: both
    # heads then get a copy in the workspace
    for kw in (dict(in_dtype=K.F32), dict(H_s=1000), dict(V=151944)):
        assert K.kd_loss_workspace_size(_ws(w_layout=K.W_HV, **kw)) > base + 2 * 151936 * (4096 + 1000)


def test_beta_ignored_for_kl():
    K.kd_loss_workspace_size(_ws(kind=K.FKL, beta=5.0))
    K.kd_loss_workspace_size(_ws(kind=K.TVD, beta=-1.0))


def test_pointer_checks_run_before_any_gpu_work():
    # fake, never dereferenced addresses: every call must fail on the host
    p = _ws()
    L = K.lib()
    n = K.kd_loss_workspace_size(p)
    good = [ctypes.c_void_p(0x1000 * (i + 1)) for i in range(10)]

    def call(args, ws_bytes=n):
        return L.kd_loss_fwd_bwd(ctypes.byref(p), *args, ctypes.c_size_t(ws_bytes), None)

    for i in (0, 1, 2, 3, 5, 7, 8, 9):          # required pointers (mask=4, per_token=6 may be NULL)
        a = list(good); a[i] = None
        assert call(a) == 1, i
    a = list(good); a[0] = ctypes.c_void_p(0x1008)
    assert call(a) == 3
    a = list(good); a[9] = ctypes.c_void_p(0x1010)  # workspace needs 256-byte alignment
    assert call(a) == 3
    assert call(good, n - 1) == 5
    assert L.kd_loss_fwd_bwd(None, *good, ctypes.c_size_t(n), None) == 1


def test_fp8_teacher_params_and_workspace():
    bf = K.kd_loss_workspace_size(_ws())
    f8 = K.kd_loss_workspace_size(_ws(flags=K.FLAG_TEACHER_FP8, teacher_scale=1e-4))
    assert f8 < bf                                  # the compacted teacher hidden states are half the size
    # several fp8 teachers: the size query needs no scales, the call itself does
    p = _ws(flags=K.FLAG_TEACHER_FP8)
    H = (ctypes.c_int64 * 2)(4096, 2048)
    n = ctypes.c_size_t(0)
    assert K.lib().kd_loss_workspace_size_multi(ctypes.byref(p), 2, H, ctypes.byref(n)) == 0 and n.value > f8
    ptrs = (ctypes.c_void_p * 2)(0x1000, 0x2000)
    w = (ctypes.c_float * 2)(0.5, 0.5)
    g = [ctypes.c_void_p(0x1000 * (i + 3)) for i in range(8)]
    assert K.lib().kd_loss_fwd_bwd_multi(ctypes.byref(p), 2, ptrs, ptrs, H, w, None, *g, ctypes.c_size_t(n.value), None) == 1


def test_quantize_argument_checks():
    L = K.lib()
    a, b = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x2000)
    assert L.kd_quantize_e4m3(None, K.BF16, 16, 1.0, b, None) == 1
    assert L.kd_quantize_e4m3(a, K.BF16, 0, 1.0, b, None) == 2
    assert L.kd_quantize_e4m3(a, 7, 16, 1.0, b, None) == 4
    assert L.kd_quantize_e4m3(a, K.BF16, 16, 0.0, b, None) == 4
    assert L.kd_quantize_e4m3(a, K.BF16, 16, float("nan"), b, None) == 4
    assert L.kd_quantize_e4m3(ctypes.c_void_p(0x1004), K.BF16, 16, 1.0, b, None) == 3
