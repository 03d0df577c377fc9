"""Host-only checks of the C ABI: the library loads without a GPU, exports every
symbol the header declares, and rejects bad arguments before touching a device."""
import ctypes
import os
import re

import pytest

from paper_2603_01875_amd import kdloss as K

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    """Every function declared in any header under include/."""
    import glob
    names = set()
    for h in glob.glob(os.path.join(ROOT, "include", "*.h")):
        src = re.sub(r"/\*.*?\*/", "", open(h).read(), flags=re.S)
        names |= set(re.findall(r"\b(kd_[a-z0-9_]+)\s*\(", src))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    names = _declared_symbols()
    assert {"kd_loss_workspace_size", "kd_loss_fwd_bwd", "kd_loss_fwd", "kd_status_string",
            "kd_loss_plan_info", "kd_loss_fwd_bwd_multi", "kd_quantize_e4m3", "kd_loss_profile_hook",
            "kd_probe_mfma_rate"} <= set(names)
    L = K.lib()
    for n in names:
        assert hasattr(L, n), n


@pytest.mark.parametrize("header", ["kdloss.h", "kdloss_bench.h"])
def test_header_is_plain_c(header):
    """The boundary is a C ABI: each header must compile as C99 on its own."""
    import subprocess
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only", "-x", "c",
                        os.path.join(ROOT, "include", header)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr


def test_struct_layout_matches_header():
    assert ctypes.sizeof(K.KdLossParams) == 4 * 8 + 12 * 4          # 80 bytes, no padding


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
    (dict(kind=K.AKL, beta=0.0), 4), (dict(kind=K.AKL, beta=1.0), 4),
    (dict(kind=K.AKL, flags=K.FLAG_TEACHER_FP8, teacher_scale=1.0), 6),
    # fp8 teacher: needs a positive finite scale, a bf16 student side and H_t % 128 == 0
    (dict(flags=K.FLAG_TEACHER_FP8), 4), (dict(flags=K.FLAG_TEACHER_FP8, teacher_scale=float("inf")), 4),
    (dict(flags=K.FLAG_TEACHER_FP8, teacher_scale=1.0, in_dtype=K.F32), 6),
    (dict(flags=K.FLAG_TEACHER_FP8, teacher_scale=1.0, H_t=4160), 3),
    (dict(flags=8), 4),
    # vocabulary chunk: 0 or a multiple of 256 in [256, 2^20]; loss scale: finite, non-zero; reserved: 0
    (dict(vocab_chunk=100), 4), (dict(vocab_chunk=-256), 4), (dict(vocab_chunk=1000), 4),
    (dict(vocab_chunk=(1 << 20) + 256), 4), (dict(loss_scale=0.0), 4), (dict(loss_scale=float("inf")), 4),
    (dict(loss_scale=float("nan")), 4),
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


def test_reserved_word_must_be_zero():
    p = _ws()
    p.reserved = 1
    with pytest.raises(K.KdLossError) as e:
        K.kd_loss_workspace_size(p)
    assert e.value.status == 4


def test_vocab_chunk_enters_the_size_query_and_the_plan():
    """The chunk is a field of the parameter block (no environment variable): the size query, the plan
    report and the call all see the same value."""
    auto = _ws()
    vc_auto, n_auto = K.kd_loss_plan_info(auto)
    assert vc_auto == 16384
    small = _ws(vocab_chunk=2048)
    vc, n = K.kd_loss_plan_info(small)
    assert vc == 2048 and n > n_auto
    assert K.kd_loss_workspace_size(small) < K.kd_loss_workspace_size(auto)
    os.environ["KD_VOCAB_CHUNK"] = "512"          # the library reads no environment variable
    try:
        assert K.kd_loss_plan_info(auto)[0] == 16384
    finally:
        del os.environ["KD_VOCAB_CHUNK"]
    # a chunk wider than the vocabulary is clamped to it
    assert K.kd_loss_plan_info(K.make_params(512, 256, 128, 4096, vocab_chunk=1 << 20))[0] == 4096
    # a call with a workspace sized for another chunk is refused on the host
    n_small = K.kd_loss_workspace_size(small)
    good = [ctypes.c_void_p(0x1000 * (i + 1)) for i in range(10)]
    assert K.lib().kd_loss_fwd_bwd(ctypes.byref(auto), *good, ctypes.c_size_t(n_small), None) == 5


def test_multi_teacher_hidden_major_heads_share_one_student_plan():
    """[H,V] heads, one teacher on the 64-element grid and one off it: the student side must be planned
    once for the whole call (all heads re-packed), so the workspace holds one copy of the student head and
    one of each teacher head."""
    base = dict(T=512, H_s=128, V=4096, w_layout=K.W_HV)

    def size(hts):
        p = K.make_params(H_t=hts[0], **base)
        H = (ctypes.c_int64 * len(hts))(*hts)
        n = ctypes.c_size_t(0)
        assert K.lib().kd_loss_workspace_size_multi(ctypes.byref(p), len(hts), H, ctypes.byref(n)) == 0
        return n.value

    inplace = size([128, 256])
    mixed = size([128, 200])
    # every head copied: student 4096 x 128, teachers 4096 x 128 and 4096 x 256 (200 padded to 256), bf16
    assert mixed >= inplace + 2 * 4096 * (128 + 128 + 256)
    assert size([200, 128]) == mixed                       # whichever teacher needs it


def _cpu_ops(T=6, H_t=16, H_s=8, V=24, dtype=None):
    import torch
    dtype = dtype or torch.bfloat16
    return (torch.zeros(T, H_t, dtype=dtype), torch.zeros(V, H_t, dtype=dtype), torch.zeros(T, H_s, dtype=dtype),
            torch.zeros(V, H_s, dtype=dtype))


def test_wrapper_checks_operands_before_any_call():
    """The C ABI sees only addresses; dtype, shape, contiguity and device are checked by the binding."""
    import torch
    h_t, W_t, h_s, W_s = _cpu_ops()
    ok = K.check_operands(h_t, W_t, h_s, W_s, require_cuda=False)
    assert ok == (6, 16, 8, 24, K.BF16, K.BF16)
    with pytest.raises(ValueError, match="CUDA"):
        K.check_operands(h_t, W_t, h_s, W_s)                                  # CPU tensors
    with pytest.raises(ValueError, match="CUDA"):
        K.kd_loss_fwd_bwd(h_t, W_t, h_s, W_s)                                 # ... through the wrapper too
    bad = [
        dict(h_s=h_s.to(torch.float16), W_s=W_s.to(torch.float16)),           # fp16 is not a supported dtype
        dict(W_s=W_s.float()),                                                # student dtypes differ
        dict(h_t=h_t.float()),                                                # teacher dtype differs
        dict(h_s=h_s[:5]),                                                    # token counts differ
        dict(W_s=torch.zeros(25, 8, dtype=torch.bfloat16)),                   # vocabularies differ
        dict(W_t=torch.zeros(24, 17, dtype=torch.bfloat16)),                  # hidden size differs
        dict(W_t=W_t.t()),                                                    # wrong layout / not contiguous
        dict(h_t=torch.zeros(6, 32, dtype=torch.bfloat16)[:, ::2]),           # not contiguous
        dict(h_t=h_t.reshape(-1)),                                            # not 2-D
        dict(mask=torch.ones(6, dtype=torch.int64)),                          # 8-byte mask elements
        dict(mask=torch.ones(5, dtype=torch.uint8)),                          # wrong mask length
        dict(grad_W_s=torch.zeros(24, 8, dtype=torch.float32)),               # gradient buffer of the wrong dtype
        dict(grad_W_s=torch.zeros(8, 24, dtype=torch.bfloat16)),              # ... or shape
        dict(flags=K.FLAG_TEACHER_FP8),                                       # fp8 teacher needs uint8 codes
    ]
    for kw in bad:
        args = dict(h_t=h_t, W_t=W_t, h_s=h_s, W_s=W_s)
        args.update(kw)
        with pytest.raises(ValueError):
            K.check_operands(require_cuda=False, **args)
    # [H,V] layout and the fp8 teacher, accepted
    assert K.check_operands(h_t, W_t.t().contiguous(), h_s, W_s.t().contiguous(), w_layout=K.W_HV,
                            require_cuda=False)[3] == 24
    q = torch.zeros(6, 16, dtype=torch.uint8), torch.zeros(24, 16, dtype=torch.uint8)
    assert K.check_operands(q[0], q[1], h_s, W_s, flags=K.FLAG_TEACHER_FP8, mask=torch.ones(6, dtype=torch.bool),
                            require_cuda=False)[0] == 6


def test_thin_calls_check_sizes_against_the_parameter_block():
    import torch
    h_t, W_t, h_s, W_s = _cpu_ops()
    p = K.make_params(6, 16, 8, 24)
    loss = torch.zeros(1)
    with pytest.raises(ValueError):
        K.kd_loss_fwd_bwd_raw(p, h_t, W_t, h_s, W_s, None, loss, None, torch.zeros(6, 8), torch.zeros(24, 8),
                              torch.zeros(1024, dtype=torch.uint8))


def test_akl_needs_room_for_its_search_partials():
    base = K.kd_loss_workspace_size(_ws(kind=K.FKL))
    akl = K.kd_loss_workspace_size(_ws(kind=K.AKL))
    assert base < akl < base + 40 * (1 << 20)            # 16 partial sums per part instead of 5, six floats per token
    assert K.kd_loss_plan_info(_ws(kind=K.AKL))[1] == K.kd_loss_plan_info(_ws(kind=K.JSD))[1] + 8


def test_hidden_major_heads_with_fp8_teacher_are_repacked():
    vh = K.kd_loss_workspace_size(_ws(flags=K.FLAG_TEACHER_FP8, teacher_scale=1.0))
    hv = K.kd_loss_workspace_size(_ws(flags=K.FLAG_TEACHER_FP8, teacher_scale=1.0, w_layout=K.W_HV))
    assert hv >= vh + 151936 * (4096 + 2 * 1024)        # a byte copy of the teacher head, a bf16 one of the student's
