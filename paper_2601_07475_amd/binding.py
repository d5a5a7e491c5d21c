"""Thin ctypes binding of libarcq.so: same names as include/arcq.h and include/arcq_bench.h, argument marshalling only.

PyTorch supplies device memory and the stream; every step of the path runs in the HIP
kernels.  There is no fallback: if the library is not built, or a call fails, an exception
is raised.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("ARCQ_LIBRARY") or os.path.join(_HERE, "libarcq.so")   # override: a differently built copy

OK, INVALID_ARG, BAD_SHAPE, BAD_ALIGN, HIP_ERROR, WORKSPACE_TOO_SMALL = range(6)
DTYPE_F16, DTYPE_F32 = 0, 1
LAYOUT_INTERLEAVED, SCALE_ROUND_UP, RMSNORM_EXACT_SUM = 1, 2, 4
MAX_K = 65536

# every symbol include/arcq.h and include/arcq_bench.h declare: name -> (restype, argtypes)
_i64, _f32, _vp, _sz, _u32 = ctypes.c_int64, ctypes.c_float, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_uint32
SIGNATURES = {
    "arcq_version": (ctypes.c_int, []),
    "arcq_last_error": (ctypes.c_char_p, []),
    "arcq_packed_sizes": (ctypes.c_int, [_i64, _i64, _i64, ctypes.POINTER(_sz), ctypes.POINTER(_sz)]),
    "arcq_quantize_act": (ctypes.c_int, [_vp, _i64, _i64, _i64, _vp, _i64, _f32, _vp, _vp, _vp]),
    "arcq_rmsnorm_quantize_act": (ctypes.c_int, [_vp, _i64, _i64, _i64, _vp, _f32, _vp, _i64, _f32, _vp, _vp, _vp]),
    "arcq_pack_weight": (ctypes.c_int, [_vp, _i64, _i64, _i64, _vp, _i64, _f32, _vp, _vp, _vp]),
    "arcq_quantize_act_ex": (ctypes.c_int, [_vp, _i64, _i64, _i64, _vp, _i64, _f32, _u32, _vp, _vp, _vp]),
    "arcq_rmsnorm_quantize_act_ex": (ctypes.c_int, [_vp, _i64, _i64, _i64, _vp, _f32, _vp, _i64, _f32, _u32, _vp, _vp, _vp]),
    "arcq_pack_weight_ex": (ctypes.c_int, [_vp, _i64, _i64, _i64, _vp, _i64, _f32, _u32, _vp, _vp, _vp]),
    "arcq_mx_quantize_act_ex": (ctypes.c_int, [_vp, _i64, _i64, _i64, _vp, _i64, _u32, _vp, _vp, _vp]),
    "arcq_mx_pack_weight_ex": (ctypes.c_int, [_vp, _i64, _i64, _i64, _vp, _i64, _u32, _vp, _vp, _vp]),
    "arcq_mx_packed_sizes": (ctypes.c_int, [_i64, _i64, _i64, ctypes.POINTER(_sz), ctypes.POINTER(_sz)]),
    "arcq_mx_quantize_act": (ctypes.c_int, [_vp, _i64, _i64, _i64, _vp, _i64, _vp, _vp, _vp]),
    "arcq_mx_pack_weight": (ctypes.c_int, [_vp, _i64, _i64, _i64, _vp, _i64, _vp, _vp, _vp]),
    "arcq_mx_gemm": (ctypes.c_int, [_vp, _vp, _vp, _vp, _i64, _i64, _i64, _vp, ctypes.c_int, _i64, _vp]),
    "arcq_mx_gemm_workspace_size": (ctypes.c_int, [_i64, _i64, _i64, ctypes.POINTER(_sz)]),
    "arcq_mx_gemm_ws": (ctypes.c_int, [_vp, _vp, _vp, _vp, _i64, _i64, _i64, _vp, ctypes.c_int, _i64, _vp, _sz, _vp]),
    "arcq_calib_absmax": (ctypes.c_int, [_vp, _i64, _i64, _i64, _vp, _vp]),
    "arcq_calib_select": (ctypes.c_int, [_vp, _i64, _vp, _vp, ctypes.POINTER(ctypes.c_int), _vp]),
    "arcq_gemm_workspace_size": (ctypes.c_int, [_i64, _i64, _i64, ctypes.POINTER(_sz)]),
    "arcq_gemm": (ctypes.c_int, [_vp, _vp, _f32, _vp, _vp, _f32, _i64, _i64, _i64, _vp, ctypes.c_int, _i64,
                                 _vp, _sz, _vp]),
    "arcq_gemm_noalloc": (ctypes.c_int, [_vp, _vp, _f32, _vp, _vp, _f32, _i64, _i64, _i64, _vp, ctypes.c_int, _i64, _vp]),
    "arcq_probe_mfma_f16": (ctypes.c_int, [ctypes.c_int, _vp, ctypes.POINTER(ctypes.c_double), _vp]),
    "arcq_probe_mfma_fp4": (ctypes.c_int, [ctypes.c_int, _vp, ctypes.POINTER(ctypes.c_double), _vp]),
    "arcq_ref_gemm_bf16": (ctypes.c_int, [_vp, _vp, _i64, _i64, _i64, _vp, _i64, _vp]),
    "arcq_check_perm": (ctypes.c_int, [_vp, _i64, _vp, ctypes.POINTER(ctypes.c_int), _vp]),
}


class ArcqError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"libarcq status {status}: {message}")
        self.status = status


_lib = None


def lib():
    """The loaded library; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2601_07475_amd.build`")
        handle = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype, fn.argtypes = res, args
        _lib = handle
    return _lib


def _check(status):
    if status != OK:
        raise ArcqError(status, lib().arcq_last_error().decode())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr() if t is not None and t.numel() else 0) if t is not None else None


def arcq_version():
    return lib().arcq_version()


def arcq_packed_sizes(rows, K, S):
    c, s = _sz(0), _sz(0)
    _check(lib().arcq_packed_sizes(rows, K, S, ctypes.byref(c), ctypes.byref(s)))
    return c.value, s.value


def _quantize(fn, x, perm, S, tensor_scale, codes=None, scales=None):
    assert x.is_cuda and x.dtype == torch.float16 and x.dim() == 2 and x.stride(1) == 1
    assert perm.is_cuda and perm.dtype == torch.int32 and perm.is_contiguous()
    rows, K = x.shape
    if perm.numel() != K:
        raise ArcqError(BAD_SHAPE, "perm must have K entries")
    ldx = x.stride(0) if rows > 1 else max(K, x.stride(0))
    cb, sb = arcq_packed_sizes(rows, K, S)
    Kp = K + S
    if codes is None:
        codes = torch.empty((rows, Kp // 2), dtype=torch.uint8, device=x.device)
    if scales is None:
        scales = torch.empty((rows, Kp // 16), dtype=torch.uint8, device=x.device)
    assert codes.numel() == cb and scales.numel() == sb and codes.is_contiguous() and scales.is_contiguous()
    _check(fn(_ptr(x), rows, K, ldx, _ptr(perm), S, float(tensor_scale), _ptr(codes), _ptr(scales), _stream()))
    return codes, scales


def arcq_quantize_act(x, perm, S, tensor_scale, codes=None, scales=None):
    """x fp16 [M, K] cuda, perm int32 [K] cuda -> (codes uint8 [M, K'/2], scales uint8 [M, K'/16])."""
    return _quantize(lib().arcq_quantize_act, x, perm, S, tensor_scale, codes, scales)


def arcq_rmsnorm_quantize_act(x, gamma, eps, perm, S, tensor_scale, codes=None, scales=None):
    """RMSNorm (weight gamma fp16 [K], eps) fused in front of arcq_quantize_act."""
    assert gamma.is_cuda and gamma.dtype == torch.float16 and gamma.is_contiguous() and gamma.numel() == x.shape[1]
    lib_fn = lib().arcq_rmsnorm_quantize_act

    def fn(xp, rows, K, ldx, permp, S_, sT, cp, sp, st):
        return lib_fn(xp, rows, K, ldx, _ptr(gamma), float(eps), permp, S_, sT, cp, sp, st)
    return _quantize(fn, x, perm, S, tensor_scale, codes, scales)


def arcq_pack_weight(w, perm, S, tensor_scale, codes=None, scales=None):
    """w fp16 [N, K] cuda -> packed [N, K'] with the outlier blocks duplicated."""
    return _quantize(lib().arcq_pack_weight, w, perm, S, tensor_scale, codes, scales)


def _with_flags(lib_fn, flags):
    """The *_ex entry points take `flags` right before the output pointers."""
    def fn(xp, rows, K, ldx, permp, S_, sT, cp, sp, st):
        return lib_fn(xp, rows, K, ldx, permp, S_, sT, int(flags), cp, sp, st)
    return fn


def arcq_quantize_act_ex(x, perm, S, tensor_scale, flags, codes=None, scales=None):
    """arcq_quantize_act with the layout / scale-rounding variants (LAYOUT_INTERLEAVED | SCALE_ROUND_UP)."""
    return _quantize(_with_flags(lib().arcq_quantize_act_ex, flags), x, perm, S, tensor_scale, codes, scales)


def arcq_rmsnorm_quantize_act_ex(x, gamma, eps, perm, S, tensor_scale, flags, codes=None, scales=None):
    assert gamma.is_cuda and gamma.dtype == torch.float16 and gamma.is_contiguous() and gamma.numel() == x.shape[1]
    lib_fn = lib().arcq_rmsnorm_quantize_act_ex

    def fn(xp, rows, K, ldx, permp, S_, sT, cp, sp, st):
        return lib_fn(xp, rows, K, ldx, _ptr(gamma), float(eps), permp, S_, sT, int(flags), cp, sp, st)
    return _quantize(fn, x, perm, S, tensor_scale, codes, scales)


def arcq_pack_weight_ex(w, perm, S, tensor_scale, flags, codes=None, scales=None):
    return _quantize(_with_flags(lib().arcq_pack_weight_ex, flags), w, perm, S, tensor_scale, codes, scales)


def arcq_gemm_workspace_size(M, N, Kp):
    b = _sz(0)
    _check(lib().arcq_gemm_workspace_size(M, N, Kp, ctypes.byref(b)))
    return b.value


def arcq_gemm(a_codes, a_scales, a_tensor_scale, w_codes, w_scales, w_tensor_scale,
              out_dtype=torch.float16, y=None, workspace=None):
    """y[M, N] = deq(A) deq(W)^T over K' (fp32 accumulate); returns y."""
    for t in (a_codes, a_scales, w_codes, w_scales):
        assert t.is_cuda and t.dtype == torch.uint8 and t.is_contiguous()
    M, N = a_codes.shape[0], w_codes.shape[0]
    Kp = a_codes.shape[1] * 2
    if w_codes.shape[1] * 2 != Kp or a_scales.shape != (M, Kp // 16) or w_scales.shape != (N, Kp // 16):
        raise ArcqError(BAD_SHAPE, "operand shapes disagree on K'")
    if y is None:
        y = torch.empty((M, N), dtype=out_dtype, device=a_codes.device)
    assert y.shape == (M, N) and y.stride(1) == 1 and y.dtype in (torch.float16, torch.float32)
    need = arcq_gemm_workspace_size(M, N, Kp)
    if need and (workspace is None or workspace.numel() * workspace.element_size() < need):
        workspace = torch.empty(need, dtype=torch.uint8, device=a_codes.device)
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    ldy = y.stride(0) if M > 1 else max(N, y.stride(0))
    _check(lib().arcq_gemm(_ptr(a_codes), _ptr(a_scales), float(a_tensor_scale),
                           _ptr(w_codes), _ptr(w_scales), float(w_tensor_scale), M, N, Kp,
                           _ptr(y), DTYPE_F16 if y.dtype == torch.float16 else DTYPE_F32, ldy,
                           _ptr(workspace) if workspace is not None else None, ws_bytes, _stream()))
    return y


NOALLOC_SCRATCH_BYTES = 8 << 20


def arcq_gemm_noalloc(a_codes, a_scales, a_tensor_scale, w_codes, w_scales, w_tensor_scale, y):
    """arcq_gemm without a workspace argument: split-K partial results go to the library's built-in scratch.
    The output tensor y [M, N] (fp16 or fp32) is the caller's; nothing is allocated here or in the library."""
    for t in (a_codes, a_scales, w_codes, w_scales):
        assert t.is_cuda and t.dtype == torch.uint8 and t.is_contiguous()
    M, N = a_codes.shape[0], w_codes.shape[0]
    Kp = a_codes.shape[1] * 2
    if w_codes.shape[1] * 2 != Kp or a_scales.shape != (M, Kp // 16) or w_scales.shape != (N, Kp // 16):
        raise ArcqError(BAD_SHAPE, "operand shapes disagree on K'")
    assert y.shape == (M, N) and y.stride(1) == 1 and y.dtype in (torch.float16, torch.float32)
    ldy = y.stride(0) if M > 1 else max(N, y.stride(0))
    _check(lib().arcq_gemm_noalloc(_ptr(a_codes), _ptr(a_scales), float(a_tensor_scale),
                                   _ptr(w_codes), _ptr(w_scales), float(w_tensor_scale), M, N, Kp,
                                   _ptr(y), DTYPE_F16 if y.dtype == torch.float16 else DTYPE_F32, ldy, _stream()))
    return y


def arcq_calib_absmax(x, colmax):
    """Folds x fp16 [M, K] into the running per-channel abs-max colmax fp32 [K] (zeros before the first batch)."""
    assert x.is_cuda and x.dtype == torch.float16 and x.dim() == 2 and x.stride(1) == 1
    assert colmax.is_cuda and colmax.dtype == torch.float32 and colmax.is_contiguous() and colmax.numel() == x.shape[1]
    M, K = x.shape
    _check(lib().arcq_calib_absmax(_ptr(x), M, K, x.stride(0) if M > 1 else max(K, x.stride(0)), _ptr(colmax), _stream()))
    return colmax


def arcq_calib_select(colmax, perm=None, info=None):
    """colmax fp32 [K] -> (perm int32 [K], S, info int32 [4] = {S, S_raw, bits(max), bits(tau)}); synchronises."""
    assert colmax.is_cuda and colmax.dtype == torch.float32 and colmax.is_contiguous()
    K = colmax.numel()
    if perm is None:
        perm = torch.empty(K, dtype=torch.int32, device=colmax.device)
    if info is None:
        info = torch.empty(4, dtype=torch.int32, device=colmax.device)
    S = ctypes.c_int(-1)
    _check(lib().arcq_calib_select(_ptr(colmax), K, _ptr(perm), _ptr(info), ctypes.byref(S), _stream()))
    return perm, S.value, info


def _mx_quantize(fn, x, perm, S, codes=None, scales=None):
    assert x.is_cuda and x.dtype == torch.float16 and x.dim() == 2 and x.stride(1) == 1
    assert perm.is_cuda and perm.dtype == torch.int32 and perm.is_contiguous()
    rows, K = x.shape
    if perm.numel() != K:
        raise ArcqError(BAD_SHAPE, "perm must have K entries")
    cb, sb = _sz(0), _sz(0)
    _check(lib().arcq_mx_packed_sizes(rows, K, S, ctypes.byref(cb), ctypes.byref(sb)))
    Kp = K + S
    if codes is None:
        codes = torch.empty((rows, Kp // 2), dtype=torch.uint8, device=x.device)
    if scales is None:
        scales = torch.empty((rows, Kp // 32), dtype=torch.uint8, device=x.device)
    assert codes.numel() == cb.value and scales.numel() == sb.value and codes.is_contiguous() and scales.is_contiguous()
    ldx = x.stride(0) if rows > 1 else max(K, x.stride(0))
    _check(fn(_ptr(x), rows, K, ldx, _ptr(perm), S, _ptr(codes), _ptr(scales), _stream()))
    return codes, scales


def arcq_mx_quantize_act(x, perm, S, codes=None, scales=None):
    """MXFP4: x fp16 [M, K] -> (codes uint8 [M, K'/2], scales uint8 [M, K'/32])."""
    return _mx_quantize(lib().arcq_mx_quantize_act, x, perm, S, codes, scales)


def arcq_mx_pack_weight(w, perm, S, codes=None, scales=None):
    return _mx_quantize(lib().arcq_mx_pack_weight, w, perm, S, codes, scales)


def _mx_with_flags(lib_fn, flags):
    def fn(xp, rows, K, ldx, permp, S_, cp, sp, st):
        return lib_fn(xp, rows, K, ldx, permp, S_, int(flags), cp, sp, st)
    return fn


def arcq_mx_quantize_act_ex(x, perm, S, flags, codes=None, scales=None):
    return _mx_quantize(_mx_with_flags(lib().arcq_mx_quantize_act_ex, flags), x, perm, S, codes, scales)


def arcq_mx_pack_weight_ex(w, perm, S, flags, codes=None, scales=None):
    return _mx_quantize(_mx_with_flags(lib().arcq_mx_pack_weight_ex, flags), w, perm, S, codes, scales)


def arcq_mx_gemm_workspace_size(M, N, Kp):
    b = _sz(0)
    _check(lib().arcq_mx_gemm_workspace_size(M, N, Kp, ctypes.byref(b)))
    return b.value


def arcq_mx_gemm(a_codes, a_scales, w_codes, w_scales, out_dtype=torch.float16, y=None, workspace=None):
    """MXFP4: y[M, N] = deq(A) deq(W)^T over K' on the scaled FP4 matrix instruction; returns y.
    workspace: a uint8 tensor of at least arcq_mx_gemm_workspace_size bytes lets few-tile problems split K'
    (arcq_mx_gemm_ws); without one the plain entry point runs."""
    for t in (a_codes, a_scales, w_codes, w_scales):
        assert t.is_cuda and t.dtype == torch.uint8 and t.is_contiguous()
    M, N = a_codes.shape[0], w_codes.shape[0]
    Kp = a_codes.shape[1] * 2
    if w_codes.shape[1] * 2 != Kp or a_scales.shape != (M, Kp // 32) or w_scales.shape != (N, Kp // 32):
        raise ArcqError(BAD_SHAPE, "operand shapes disagree on K'")
    if y is None:
        y = torch.empty((M, N), dtype=out_dtype, device=a_codes.device)
    assert y.shape == (M, N) and y.stride(1) == 1 and y.dtype in (torch.float16, torch.float32)
    ldy = y.stride(0) if M > 1 else max(N, y.stride(0))
    dt = DTYPE_F16 if y.dtype == torch.float16 else DTYPE_F32
    if workspace is not None:
        assert workspace.is_cuda and workspace.is_contiguous()
        _check(lib().arcq_mx_gemm_ws(_ptr(a_codes), _ptr(a_scales), _ptr(w_codes), _ptr(w_scales), M, N, Kp, _ptr(y), dt, ldy,
                                     _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))
    else:
        _check(lib().arcq_mx_gemm(_ptr(a_codes), _ptr(a_scales), _ptr(w_codes), _ptr(w_scales), M, N, Kp, _ptr(y), dt, ldy,
                                  _stream()))
    return y


def prepare_quantize_act(x, perm, S, tensor_scale, codes, scales):
    """Marshals the arguments of arcq_quantize_act once; returns a zero-argument callable that
    enqueues the call on the stream that was current at preparation time (for tight loops)."""
    rows, K = x.shape
    fn = lib().arcq_quantize_act
    args = (_ptr(x), rows, K, x.stride(0) if rows > 1 else K, _ptr(perm), S, float(tensor_scale),
            _ptr(codes), _ptr(scales), _stream())

    def call():
        _check(fn(*args))
    return call


def prepare_rmsnorm_quantize_act(x, gamma, eps, perm, S, tensor_scale, codes, scales):
    """Same for arcq_rmsnorm_quantize_act."""
    rows, K = x.shape
    fn = lib().arcq_rmsnorm_quantize_act
    args = (_ptr(x), rows, K, x.stride(0) if rows > 1 else K, _ptr(gamma), float(eps), _ptr(perm), S,
            float(tensor_scale), _ptr(codes), _ptr(scales), _stream())

    def call():
        _check(fn(*args))
    return call


def prepare_gemm(a_codes, a_scales, a_tensor_scale, w_codes, w_scales, w_tensor_scale, y, workspace=None):
    """Same for arcq_gemm."""
    M, N, Kp = a_codes.shape[0], w_codes.shape[0], a_codes.shape[1] * 2
    need = arcq_gemm_workspace_size(M, N, Kp)
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    if need > ws_bytes:
        raise ArcqError(WORKSPACE_TOO_SMALL, f"workspace of {need} bytes needed")
    fn = lib().arcq_gemm
    args = (_ptr(a_codes), _ptr(a_scales), float(a_tensor_scale), _ptr(w_codes), _ptr(w_scales),
            float(w_tensor_scale), M, N, Kp, _ptr(y), DTYPE_F16 if y.dtype == torch.float16 else DTYPE_F32,
            y.stride(0) if M > 1 else N, _ptr(workspace) if workspace is not None else None, ws_bytes, _stream())

    def call():
        _check(fn(*args))
    return call


def prepare_mx_quantize_act(x, perm, S, codes, scales):
    """Same for arcq_mx_quantize_act."""
    rows, K = x.shape
    fn = lib().arcq_mx_quantize_act
    args = (_ptr(x), rows, K, x.stride(0) if rows > 1 else K, _ptr(perm), S, _ptr(codes), _ptr(scales), _stream())

    def call():
        _check(fn(*args))
    return call


def prepare_mx_gemm(a_codes, a_scales, w_codes, w_scales, y, workspace=None):
    """Same for arcq_mx_gemm (arcq_mx_gemm_ws when a workspace tensor is given)."""
    M, N, Kp = a_codes.shape[0], w_codes.shape[0], a_codes.shape[1] * 2
    head = (_ptr(a_codes), _ptr(a_scales), _ptr(w_codes), _ptr(w_scales), M, N, Kp, _ptr(y),
            DTYPE_F16 if y.dtype == torch.float16 else DTYPE_F32, y.stride(0) if M > 1 else N)
    if workspace is not None:
        fn = lib().arcq_mx_gemm_ws
        args = head + (_ptr(workspace), workspace.numel() * workspace.element_size(), _stream())
    else:
        fn = lib().arcq_mx_gemm
        args = head + (_stream(),)

    def call():
        _check(fn(*args))
    return call


PROBE_SINK_FLOATS = 262144


def _probe(name, iters, sink):
    if sink is None:
        sink = torch.empty(PROBE_SINK_FLOATS, dtype=torch.float32, device="cuda")
    assert sink.is_cuda and sink.dtype == torch.float32 and sink.numel() >= PROBE_SINK_FLOATS and sink.is_contiguous()
    flop = ctypes.c_double(0.0)
    _check(getattr(lib(), name)(int(iters), _ptr(sink), ctypes.byref(flop), _stream()))
    return flop.value


def arcq_probe_mfma_f16(iters, sink=None):
    """Enqueues the fp16 matrix-rate probe; returns the floating-point operations of the launch."""
    return _probe("arcq_probe_mfma_f16", iters, sink)


def arcq_probe_mfma_fp4(iters, sink=None):
    """Enqueues the scaled-FP4 matrix-rate probe; returns the floating-point operations of the launch."""
    return _probe("arcq_probe_mfma_fp4", iters, sink)


def arcq_check_perm(perm):
    """True if the int32 cuda tensor perm is a permutation of 0..K-1 (synchronises)."""
    K = perm.numel()
    flags = torch.empty(K, dtype=torch.uint8, device=perm.device)
    res = ctypes.c_int(-1)
    _check(lib().arcq_check_perm(_ptr(perm), K, _ptr(flags), ctypes.byref(res), _stream()))
    return res.value == 1


def prepare_ref_gemm_bf16(x, w, y):
    """The hand-written bf16 comparison GEMM y = x w^T (x [M, K], w [N, K] bf16, y [M, N] fp16) as a prepared call."""
    for t in (x, w):
        assert t.is_cuda and t.dtype == torch.bfloat16 and t.is_contiguous()
    M, K = x.shape
    N = w.shape[0]
    assert w.shape[1] == K and y.shape == (M, N) and y.dtype == torch.float16 and y.stride(1) == 1
    fn = lib().arcq_ref_gemm_bf16
    args = (_ptr(x), _ptr(w), M, N, K, _ptr(y), y.stride(0) if M > 1 else N, _stream())

    def call():
        _check(fn(*args))
    return call


def arcq_ref_gemm_bf16(x, w, y=None):
    if y is None:
        y = torch.empty((x.shape[0], w.shape[0]), dtype=torch.float16, device=x.device)
    prepare_ref_gemm_bf16(x, w, y)()
    return y
