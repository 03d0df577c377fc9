"""ctypes binding of libkdloss (see include/kdloss.h for the contract).

Argument marshalling only: every step of the computation runs in the HIP
kernels of the shared library.  torch is used to own device memory and to name
the stream.  There is no fallback: if the library has not been built, loading
fails with an error that says how to build it.
"""
from __future__ import annotations

import ctypes
import os

FKL, RKL, JSD, TVD, SKEW_FKL, SKEW_RKL, AKL = 0, 1, 2, 3, 4, 5, 6
BF16, F32 = 0, 1
W_HV, W_VH = 0, 1

KD_OK = 0
STATUS_NAMES = {0: "KD_OK", 1: "KD_ERR_NULL", 2: "KD_ERR_SHAPE", 3: "KD_ERR_ALIGN", 4: "KD_ERR_PARAM",
                5: "KD_ERR_WORKSPACE", 6: "KD_ERR_UNSUPPORTED", 7: "KD_ERR_LAUNCH", 8: "KD_ERR_TOO_LARGE"}
STATIC_SCRATCH_BYTES = 128 << 20

# KDLOSS_LIBRARY names another build of the library (measurement builds for the profiles); default: the
# product build next to the sources
_LIB_PATH = os.environ.get("KDLOSS_LIBRARY") or os.path.join(os.path.dirname(os.path.abspath(__file__)), "csrc",
                                                             "libkdloss.so")
_lib = None


class KdLossParams(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int64), ("H_t", ctypes.c_int64), ("H_s", ctypes.c_int64), ("V", ctypes.c_int64),
                ("in_dtype", ctypes.c_int32), ("grad_dtype", ctypes.c_int32), ("w_layout", ctypes.c_int32),
                ("kind", ctypes.c_int32), ("tau", ctypes.c_float), ("beta", ctypes.c_float),
                ("accumulate_grad_W", ctypes.c_int32), ("flags", ctypes.c_int32),
                ("teacher_scale", ctypes.c_float), ("vocab_chunk", ctypes.c_int32),
                ("loss_scale", ctypes.c_float), ("reserved", ctypes.c_int32)]


class KdLossError(RuntimeError):
    def __init__(self, status):
        self.status = int(status)
        msg = lib().kd_status_string(self.status).decode()
        super().__init__(f"{STATUS_NAMES.get(self.status, self.status)}: {msg}")


def lib():
    """The loaded shared library (loads on first use; never falls back to anything else)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(f"{_LIB_PATH} is missing: build it with "
                               "`python -c 'import __graft_entry__ as g; g.build()'` "
                               "or paper_2603_01875_amd/csrc/build.sh")
        # The tensors handed to the library and the streams it launches on belong to torch's HIP runtime
        # (the wheel carries its own copy).  Import torch first, so that this library's HIP calls bind to
        # that same runtime; loaded before torch it would bring up a second one, which knows neither the
        # streams nor, on a box that admits one runtime per process, the device.
        import torch  # noqa: F401
        L = ctypes.CDLL(_LIB_PATH)
        P = ctypes.POINTER(KdLossParams)
        vp = ctypes.c_void_p
        L.kd_loss_workspace_size.argtypes = [P, ctypes.POINTER(ctypes.c_size_t)]
        L.kd_loss_workspace_size.restype = ctypes.c_int
        L.kd_loss_plan_info.argtypes = [P, ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int64)]
        L.kd_loss_plan_info.restype = ctypes.c_int
        L.kd_loss_fwd_bwd.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.kd_loss_fwd_bwd.restype = ctypes.c_int
        L.kd_loss_fwd_bwd_static.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.kd_loss_fwd_bwd_static.restype = ctypes.c_int
        L.kd_loss_fwd.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.kd_loss_fwd.restype = ctypes.c_int
        L.kd_loss_workspace_size_multi.argtypes = [P, ctypes.c_int, ctypes.POINTER(ctypes.c_int64),
                                                   ctypes.POINTER(ctypes.c_size_t)]
        L.kd_loss_workspace_size_multi.restype = ctypes.c_int
        L.kd_loss_fwd_bwd_multi.argtypes = [P, ctypes.c_int, ctypes.POINTER(vp), ctypes.POINTER(vp),
                                            ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_float),
                                            ctypes.POINTER(ctypes.c_float),
                                            vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.kd_loss_fwd_bwd_multi.restype = ctypes.c_int
        L.kd_quantize_e4m3.argtypes = [vp, ctypes.c_int32, ctypes.c_int64, ctypes.c_float, vp, vp]
        L.kd_quantize_e4m3.restype = ctypes.c_int
        L.kd_loss_profile_clock.argtypes = [vp]
        L.kd_loss_profile_clock.restype = ctypes.c_int
        L.kd_probe_mfma_rate.argtypes = [vp, ctypes.c_int, vp, vp]
        L.kd_probe_mfma_rate.restype = ctypes.c_int
        L.kd_loss_profile_hook.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_void_p), ctypes.c_int]
        L.kd_loss_profile_hook.restype = ctypes.c_int
        L.kd_loss_profile_count.argtypes = []
        L.kd_loss_profile_count.restype = ctypes.c_int
        L.kd_build_info.argtypes = []
        L.kd_build_info.restype = ctypes.c_char_p
        L.kd_build_ablation.argtypes = []
        L.kd_build_ablation.restype = ctypes.c_int
        L.kd_status_string.argtypes = [ctypes.c_int]
        L.kd_status_string.restype = ctypes.c_char_p
        _lib = L
    return _lib


FLAG_TAU2 = 1
FLAG_TEACHER_FP8 = 2

def make_params(T, H_t, H_s, V, kind=FKL, tau=1.0, beta=0.5, in_dtype=BF16, grad_dtype=None,
                w_layout=W_VH, accumulate_grad_W=False, flags=0, teacher_scale=0.0, vocab_chunk=0,
                loss_scale=1.0):
    if grad_dtype is None:
        grad_dtype = in_dtype
    return KdLossParams(int(T), int(H_t), int(H_s), int(V), int(in_dtype), int(grad_dtype), int(w_layout),
                        int(kind), float(tau), float(beta), int(bool(accumulate_grad_W)), int(flags),
                        float(teacher_scale), int(vocab_chunk), float(loss_scale), 0)


def quantize_e4m3(x, scale, out=None):
    """e4m3 codes (uint8 tensor of x's shape) of x / scale; x is a contiguous bf16 or fp32 CUDA tensor."""
    import torch
    if not (isinstance(x, torch.Tensor) and x.is_cuda and x.is_contiguous()
            and x.dtype in (torch.bfloat16, torch.float32)):
        raise ValueError("x must be a contiguous bfloat16 or float32 CUDA (HIP) tensor")
    if out is None:
        out = torch.empty(x.shape, dtype=torch.uint8, device=x.device)
    elif not (out.is_cuda and out.device == x.device and out.is_contiguous() and out.dtype == torch.uint8
              and out.numel() == x.numel()):
        raise ValueError("out must be a contiguous uint8 tensor of x's size on x's device")
    st = lib().kd_quantize_e4m3(_ptr(x), BF16 if x.dtype == torch.bfloat16 else F32, x.numel(), float(scale),
                                _ptr(out), ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    if st != KD_OK:
        raise KdLossError(st)
    return out


def kd_loss_workspace_size(params: KdLossParams) -> int:
    n = ctypes.c_size_t(0)
    st = lib().kd_loss_workspace_size(ctypes.byref(params), ctypes.byref(n))
    if st != KD_OK:
        raise KdLossError(st)
    return int(n.value)


def kd_loss_plan_info(params: KdLossParams):
    vc, nl = ctypes.c_int64(0), ctypes.c_int64(0)
    st = lib().kd_loss_plan_info(ctypes.byref(params), ctypes.byref(vc), ctypes.byref(nl))
    if st != KD_OK:
        raise KdLossError(st)
    return int(vc.value), int(nl.value)


PROF_STATS, PROF_ROWS, PROF_GRAD, PROF_GEMM_GRAD_W, PROF_GEMM_GRAD_H = range(5)


class KernelTimer:
    """Brackets every launch of one kernel family with HIP events (kd_loss_profile_hook).

    with KernelTimer(PROF_STATS, max_launches) as kt: ...calls...; then kt.durations_ms()
    after a device synchronisation.
    """

    def __init__(self, which, max_launches):
        import torch
        self.which = which
        self.events = [torch.cuda.Event(enable_timing=True) for _ in range(2 * max_launches)]
        for e in self.events:
            e.record()                      # materialise the underlying hipEvent_t
        self.arr = (ctypes.c_void_p * len(self.events))(*[e.cuda_event for e in self.events])
        self.count = 0

    def __enter__(self):
        st = lib().kd_loss_profile_hook(self.which, self.arr, len(self.events))
        if st != KD_OK:
            raise KdLossError(st)
        return self

    def __exit__(self, *exc):
        self.count = lib().kd_loss_profile_count()
        lib().kd_loss_profile_hook(-1, None, 0)

    def durations_ms(self):
        return [self.events[2 * i].elapsed_time(self.events[2 * i + 1]) for i in range(self.count)]


PROBE_FLOP_PER_ITER = 256.0 * 8 * 8 * 2 * 32 * 32 * 16


class ShaderClock:
    """with ShaderClock() as sc: <library calls>; sc.ghz() is the shader clock that workgroup 0 of the last
    statistics kernel (or MFMA probe) saw: cycles of its main loop over 100 MHz reference ticks."""

    def __enter__(self):
        import torch
        self.buf = torch.zeros(2, dtype=torch.int64, device="cuda")
        st = lib().kd_loss_profile_clock(_ptr(self.buf))
        if st != KD_OK:
            raise KdLossError(st)
        return self

    def __exit__(self, *exc):
        lib().kd_loss_profile_clock(None)

    def ghz(self):
        c, r = [int(x) for x in self.buf.cpu()]
        return c / r * 0.1 if r > 0 else float("nan")


def probe_mfma_rate(iters=20000, repeats=3):
    """TFLOP/s of an MFMA-only loop on random bf16 operands (best of `repeats`): the matrix-pipe
    ceiling of this GPU at the clock it holds under that load."""
    import torch
    ops = torch.randn(64 * 1024, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    sink = torch.empty(256 * 512, device="cuda", dtype=torch.float32)
    s = torch.cuda.current_stream().cuda_stream
    best = 0.0
    for _ in range(repeats + 1):                 # first launch warms up
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        st = lib().kd_probe_mfma_rate(_ptr(ops), int(iters), _ptr(sink), ctypes.c_void_p(s))
        if st != KD_OK:
            raise KdLossError(st)
        e1.record()
        torch.cuda.synchronize()
        best = max(best, PROBE_FLOP_PER_ITER * iters / (e0.elapsed_time(e1) * 1e-3) / 1e12)
    return best


def _ptr(t):
    return ctypes.c_void_p(0 if t is None else t.data_ptr())


def _nbytes(t):
    return t.numel() * t.element_size()


def check_operands(h_t, W_t, h_s, W_s, mask=None, w_layout=W_VH, flags=0, grad_dtype=None, grad_W_s=None,
                   workspace=None, require_cuda=True):
    """Host-side checks of the tensors handed to the convenience wrappers.  The C ABI sees only addresses, so
    a wrong dtype, shape, device or a non-contiguous tensor would become an out-of-bounds device access:
    everything the library cannot see is checked here, and a ValueError is raised before any call.
    Returns (T, H_t, H_s, V, in_dtype, grad_dtype)."""
    import torch
    names = ("h_t", "W_t", "h_s", "W_s")
    ts = (h_t, W_t, h_s, W_s)
    for n, t in zip(names, ts):
        if not isinstance(t, torch.Tensor):
            raise ValueError(f"{n} must be a torch tensor")
        if t.dim() != 2:
            raise ValueError(f"{n} must be 2-dimensional, got shape {tuple(t.shape)}")
        if not t.is_contiguous():
            raise ValueError(f"{n} must be contiguous")
        if require_cuda and not t.is_cuda:
            raise ValueError(f"{n} must be a CUDA (HIP) tensor")
        if t.device != h_s.device:
            raise ValueError(f"{n} is on {t.device}, h_s on {h_s.device}")
    if w_layout not in (W_HV, W_VH):
        raise ValueError("unknown w_layout")
    if h_s.dtype not in (torch.bfloat16, torch.float32):
        raise ValueError(f"h_s must be bfloat16 or float32, got {h_s.dtype}")
    if W_s.dtype != h_s.dtype:
        raise ValueError(f"W_s is {W_s.dtype}, h_s is {h_s.dtype}")
    want_t = torch.uint8 if (flags & FLAG_TEACHER_FP8) else h_s.dtype
    for n, t in (("h_t", h_t), ("W_t", W_t)):
        if t.dtype != want_t:
            raise ValueError(f"{n} must be {want_t} here, got {t.dtype}")
    in_dtype = BF16 if h_s.dtype == torch.bfloat16 else F32
    T, H_t = h_t.shape
    if h_s.shape[0] != T:
        raise ValueError(f"h_s has {h_s.shape[0]} rows, h_t has {T}")
    H_s = h_s.shape[1]
    V = W_t.shape[0] if w_layout == W_VH else W_t.shape[1]
    want_Wt = (V, H_t) if w_layout == W_VH else (H_t, V)
    want_Ws = (V, H_s) if w_layout == W_VH else (H_s, V)
    if tuple(W_t.shape) != want_Wt:
        raise ValueError(f"W_t has shape {tuple(W_t.shape)}, expected {want_Wt} for this layout")
    if tuple(W_s.shape) != want_Ws:
        raise ValueError(f"W_s has shape {tuple(W_s.shape)}, expected {want_Ws} for this layout")
    if mask is not None:
        if not isinstance(mask, torch.Tensor) or mask.numel() != T or mask.element_size() != 1:
            raise ValueError("mask must be a tensor of T one-byte elements (uint8 or bool)")
        if not mask.is_contiguous() or mask.device != h_s.device:
            raise ValueError("mask must be contiguous and on the operands' device")
    if grad_dtype is None:
        grad_dtype = in_dtype
    if grad_dtype not in (BF16, F32):
        raise ValueError("unknown grad_dtype")
    if grad_W_s is not None:
        tdt = torch.bfloat16 if grad_dtype == BF16 else torch.float32
        if (not isinstance(grad_W_s, torch.Tensor) or tuple(grad_W_s.shape) != want_Ws or grad_W_s.dtype != tdt
                or not grad_W_s.is_contiguous() or grad_W_s.device != h_s.device):
            raise ValueError(f"grad_W_s must be a contiguous {tdt} tensor of shape {want_Ws} on the operands' device")
    if workspace is not None:
        if not isinstance(workspace, torch.Tensor) or not workspace.is_contiguous() or workspace.device != h_s.device:
            raise ValueError("workspace must be a contiguous tensor on the operands' device")
    return int(T), int(H_t), int(H_s), int(V), in_dtype, grad_dtype


def _check_raw(params, h_t, W_t, h_s, W_s, mask, loss, per_token_loss, grad_h_s, grad_W_s, workspace):
    """The thin calls take a prepared parameter block: check that every tensor holds what that block says
    the library will read or write (byte counts, contiguity, one device)."""
    es_in = 2 if params.in_dtype == BF16 else 4
    es_t = 1 if (params.flags & FLAG_TEACHER_FP8) else es_in
    es_g = 2 if params.grad_dtype == BF16 else 4
    T, H_t, H_s, V = params.T, params.H_t, params.H_s, params.V
    need = [("h_t", h_t, T * H_t * es_t), ("W_t", W_t, V * H_t * es_t), ("h_s", h_s, T * H_s * es_in),
            ("W_s", W_s, V * H_s * es_in), ("loss", loss, 4)]
    if mask is not None:
        need.append(("mask", mask, T))
    if per_token_loss is not None:
        need.append(("per_token_loss", per_token_loss, 4 * T))
    if grad_h_s is not None:
        need.append(("grad_h_s", grad_h_s, T * H_s * es_g))
    if grad_W_s is not None:
        need.append(("grad_W_s", grad_W_s, V * H_s * es_g))
    dev = h_s.device
    for n, t, nb in need:
        if not t.is_cuda or t.device != dev:
            raise ValueError(f"{n} must be a CUDA (HIP) tensor on {dev}")
        if not t.is_contiguous():
            raise ValueError(f"{n} must be contiguous")
        if _nbytes(t) != nb:
            raise ValueError(f"{n} holds {_nbytes(t)} bytes, the parameter block implies {nb}")
    if mask is not None and mask.element_size() != 1:
        raise ValueError("mask must have one-byte elements")
    if workspace is not None and (not workspace.is_cuda or workspace.device != dev or not workspace.is_contiguous()):
        raise ValueError("workspace must be a contiguous CUDA (HIP) tensor on the operands' device")


def kd_loss_fwd_bwd_raw(params, h_t, W_t, h_s, W_s, mask, loss, per_token_loss, grad_h_s, grad_W_s,
                        workspace, stream=None):
    """Thin call: all tensors are caller-allocated torch CUDA tensors (or None where allowed)."""
    import torch
    _check_raw(params, h_t, W_t, h_s, W_s, mask, loss, per_token_loss, grad_h_s, grad_W_s, workspace)
    s = torch.cuda.current_stream().cuda_stream if stream is None else stream
    st = lib().kd_loss_fwd_bwd(ctypes.byref(params), _ptr(h_t), _ptr(W_t), _ptr(h_s), _ptr(W_s), _ptr(mask),
                               _ptr(loss), _ptr(per_token_loss), _ptr(grad_h_s), _ptr(grad_W_s),
                               _ptr(workspace), ctypes.c_size_t(_nbytes(workspace)), ctypes.c_void_p(s))
    if st != KD_OK:
        raise KdLossError(st)


def kd_loss_fwd_bwd_static_raw(params, h_t, W_t, h_s, W_s, mask, loss, per_token_loss, grad_h_s, grad_W_s,
                               stream=None):
    """Thin call of the entry point that needs no workspace (the library's static scratch array)."""
    import torch
    _check_raw(params, h_t, W_t, h_s, W_s, mask, loss, per_token_loss, grad_h_s, grad_W_s, None)
    s = torch.cuda.current_stream().cuda_stream if stream is None else stream
    st = lib().kd_loss_fwd_bwd_static(ctypes.byref(params), _ptr(h_t), _ptr(W_t), _ptr(h_s), _ptr(W_s), _ptr(mask),
                                      _ptr(loss), _ptr(per_token_loss), _ptr(grad_h_s), _ptr(grad_W_s),
                                      ctypes.c_void_p(s))
    if st != KD_OK:
        raise KdLossError(st)


def kd_loss_fwd_raw(params, h_t, W_t, h_s, W_s, mask, loss, per_token_loss, workspace, stream=None):
    import torch
    _check_raw(params, h_t, W_t, h_s, W_s, mask, loss, per_token_loss, None, None, workspace)
    s = torch.cuda.current_stream().cuda_stream if stream is None else stream
    st = lib().kd_loss_fwd(ctypes.byref(params), _ptr(h_t), _ptr(W_t), _ptr(h_s), _ptr(W_s), _ptr(mask),
                           _ptr(loss), _ptr(per_token_loss), _ptr(workspace),
                           ctypes.c_size_t(_nbytes(workspace)), ctypes.c_void_p(s))
    if st != KD_OK:
        raise KdLossError(st)


def alloc_workspace(params, device="cuda"):
    import torch
    n = kd_loss_workspace_size(params)
    return torch.empty((n + 255) // 256 * 256, dtype=torch.uint8, device=device)


def kd_loss_fwd_bwd(h_t, W_t, h_s, W_s, mask=None, tau=1.0, kind=FKL, beta=0.5, w_layout=W_VH,
                    grad_dtype=None, workspace=None, grad_W_s=None, accumulate_grad_W=False,
                    want_per_token=True, flags=0, teacher_scale=0.0, vocab_chunk=0, loss_scale=1.0):
    """Convenience wrapper: allocates outputs (and the workspace unless given) and calls the library.

    h_t [T,H_t], h_s [T,H_s]; W_t, W_s in `w_layout` ([V,H] for W_VH).  Returns a dict of CUDA tensors.
    With FLAG_TEACHER_FP8, h_t and W_t are uint8 tensors of e4m3 codes and teacher_scale their joint scale.
    """
    import torch
    T, H_t, H_s, V, in_dtype, grad_dtype = check_operands(h_t, W_t, h_s, W_s, mask, w_layout, flags, grad_dtype,
                                                          grad_W_s, workspace)
    p = make_params(T, H_t, H_s, V, kind, tau, beta, in_dtype, grad_dtype, w_layout, accumulate_grad_W, flags,
                    teacher_scale, vocab_chunk, loss_scale)
    tdt = torch.bfloat16 if grad_dtype == BF16 else torch.float32
    dev = h_t.device
    if workspace is None:
        workspace = alloc_workspace(p, dev)
    loss = torch.empty(1, dtype=torch.float32, device=dev)
    ptl = torch.empty(T, dtype=torch.float32, device=dev) if want_per_token else None
    grad_h = torch.empty((T, H_s), dtype=tdt, device=dev)
    if grad_W_s is None:
        grad_W_s = torch.empty_like(W_s, dtype=tdt)
    kd_loss_fwd_bwd_raw(p, h_t, W_t, h_s, W_s, mask, loss, ptl, grad_h, grad_W_s, workspace)
    return dict(loss=loss, per_token_loss=ptl, grad_h_s=grad_h, grad_W_s=grad_W_s, workspace=workspace)


def kd_loss_fwd_bwd_multi(h_ts, W_ts, weights, h_s, W_s, mask=None, tau=1.0, kind=FKL, beta=0.5, flags=0,
                          grad_dtype=None, teacher_scales=None, w_layout=W_VH, vocab_chunk=0, loss_scale=1.0):
    """Multi-teacher call: lists of teacher hidden states / heads (in `w_layout`) and weights; with
    FLAG_TEACHER_FP8 the teacher tensors are e4m3 codes and teacher_scales their joint scales."""
    import torch
    n = len(h_ts)
    if n < 1 or len(W_ts) != n or len(weights) != n or (teacher_scales is not None and len(teacher_scales) != n):
        raise ValueError("h_ts, W_ts, weights (and teacher_scales) must have one entry per teacher")
    if (flags & FLAG_TEACHER_FP8) and teacher_scales is None:
        raise ValueError("FLAG_TEACHER_FP8 needs teacher_scales")
    for h_t, W_t in zip(h_ts, W_ts):
        T, _, H_s, V, in_dtype, grad_dtype = check_operands(h_t, W_t, h_s, W_s, mask, w_layout, flags, grad_dtype)
    p = make_params(T, h_ts[0].shape[1], H_s, V, kind, tau, beta, in_dtype, grad_dtype, w_layout, False, flags,
                    0.0, vocab_chunk, loss_scale)
    H_t = (ctypes.c_int64 * n)(*[int(h.shape[1]) for h in h_ts])
    nbytes = ctypes.c_size_t(0)
    st = lib().kd_loss_workspace_size_multi(ctypes.byref(p), n, H_t, ctypes.byref(nbytes))
    if st != KD_OK:
        raise KdLossError(st)
    dev = h_s.device
    ws = torch.empty((nbytes.value + 255) // 256 * 256, dtype=torch.uint8, device=dev)
    tdt = torch.bfloat16 if grad_dtype == BF16 else torch.float32
    loss = torch.empty(1, dtype=torch.float32, device=dev)
    ptl = torch.empty(T, dtype=torch.float32, device=dev)
    grad_h = torch.empty((T, H_s), dtype=tdt, device=dev)
    grad_W = torch.empty_like(W_s, dtype=tdt)
    hp = (ctypes.c_void_p * n)(*[h.data_ptr() for h in h_ts])
    wp = (ctypes.c_void_p * n)(*[w.data_ptr() for w in W_ts])
    wt = (ctypes.c_float * n)(*[float(w) for w in weights])
    sc = None if teacher_scales is None else (ctypes.c_float * n)(*[float(x) for x in teacher_scales])
    st = lib().kd_loss_fwd_bwd_multi(ctypes.byref(p), n, hp, wp, H_t, wt, sc, _ptr(h_s), _ptr(W_s), _ptr(mask),
                                     _ptr(loss), _ptr(ptl), _ptr(grad_h), _ptr(grad_W), _ptr(ws),
                                     ctypes.c_size_t(ws.numel()),
                                     ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    if st != KD_OK:
        raise KdLossError(st)
    return dict(loss=loss, per_token_loss=ptl, grad_h_s=grad_h, grad_W_s=grad_W)


def kd_loss_fwd(h_t, W_t, h_s, W_s, mask=None, tau=1.0, kind=FKL, beta=0.5, w_layout=W_VH, workspace=None,
                flags=0, teacher_scale=0.0, loss_scale=1.0):
    import torch
    T, H_t, H_s, V, in_dtype, _ = check_operands(h_t, W_t, h_s, W_s, mask, w_layout, flags, None, None, workspace)
    p = make_params(T, H_t, H_s, V, kind, tau, beta, in_dtype, in_dtype, w_layout, False, flags, teacher_scale,
                    0, loss_scale)
    dev = h_t.device
    if workspace is None:
        workspace = alloc_workspace(p, dev)
    loss = torch.empty(1, dtype=torch.float32, device=dev)
    ptl = torch.empty(T, dtype=torch.float32, device=dev)
    kd_loss_fwd_raw(p, h_t, W_t, h_s, W_s, mask, loss, ptl, workspace)
    return dict(loss=loss, per_token_loss=ptl)
