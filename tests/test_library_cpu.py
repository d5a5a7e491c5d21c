"""No-GPU checks of the C-ABI library: it loads, exports every declared symbol, and rejects
bad arguments before any HIP call (so these run on a machine without a GPU)."""
import ctypes
import os
import re

import pytest

from paper_2601_07475_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", h) for h in ("arcq.h", "arcq_bench.h")]

pytestmark = pytest.mark.skipif(not os.path.exists(B.LIB_PATH), reason="libarcq.so not built")


def declared_symbols():
    text = "".join(open(h).read() for h in HEADERS)
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(arcq_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound():
    names = declared_symbols()
    assert "arcq_quantize_act" in names and "arcq_pack_weight" in names and "arcq_gemm" in names
    handle = ctypes.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(handle, n), n
    assert sorted(B.SIGNATURES) == names
    assert B.arcq_version() >= 100


def test_packed_sizes():
    assert B.arcq_packed_sizes(16, 512, 32) == (16 * 544 // 2, 16 * 544 // 16)
    assert B.arcq_packed_sizes(0, 512, 0) == (0, 0)
    for K, S in ((0, 0), (24, 0), (512, 8), (512, 528), (512, -16), (B.MAX_K + 16, 0)):
        with pytest.raises(B.ArcqError) as e:
            B.arcq_packed_sizes(4, K, S)
        assert e.value.status == B.BAD_SHAPE


FAKE = ctypes.c_void_p(0x10000)       # never dereferenced: every call below must fail validation first
ODD = ctypes.c_void_p(0x10004)


def q(fn, x=FAKE, rows=4, K=512, ld=512, perm=FAKE, S=32, sT=1.0, codes=FAKE, scales=FAKE):
    return getattr(B.lib(), fn)(x, rows, K, ld, perm, S, sT, codes, scales, None)


@pytest.mark.parametrize("fn", ["arcq_quantize_act", "arcq_pack_weight"])
def test_quantizer_argument_errors(fn):
    assert q(fn, K=500) == B.BAD_SHAPE
    assert q(fn, S=24) == B.BAD_SHAPE
    assert q(fn, S=1024) == B.BAD_SHAPE
    assert q(fn, rows=-1) == B.BAD_SHAPE
    assert q(fn, ld=496) == B.BAD_SHAPE
    assert q(fn, K=B.MAX_K + 16, ld=B.MAX_K + 16) == B.BAD_SHAPE
    for bad in (0.0, -1.0, float("inf"), float("nan"), 2.0 ** -70, 2.0 ** 70):
        assert q(fn, sT=bad) == B.INVALID_ARG
    assert q(fn, x=None) == B.INVALID_ARG
    assert q(fn, perm=None) == B.INVALID_ARG
    assert q(fn, codes=None) == B.INVALID_ARG
    assert q(fn, scales=None) == B.INVALID_ARG
    assert q(fn, x=ODD) == B.BAD_ALIGN
    assert q(fn, ld=516) == B.BAD_ALIGN
    assert q(fn, codes=ODD) == B.BAD_ALIGN
    assert b"aligned" in B.lib().arcq_last_error()
    assert q(fn, perm=ODD) == B.BAD_ALIGN and q(fn, perm=ctypes.c_void_p(0x10008)) == B.BAD_ALIGN    # read as 16-byte vectors
    assert b"perm" in B.lib().arcq_last_error()
    assert q(fn, rows=0, x=None, perm=None, codes=None, scales=None) == B.OK      # empty input: nothing to do
    assert B.lib().arcq_last_error() == b""


def qn(x=FAKE, rows=4, K=512, ld=512, gamma=FAKE, eps=1e-5, perm=FAKE, S=32, sT=1.0, codes=FAKE, scales=FAKE):
    return B.lib().arcq_rmsnorm_quantize_act(x, rows, K, ld, gamma, eps, perm, S, sT, codes, scales, None)


def test_rmsnorm_quantizer_argument_errors():
    assert qn(K=500) == B.BAD_SHAPE
    assert qn(S=24) == B.BAD_SHAPE
    assert qn(ld=496) == B.BAD_SHAPE
    assert qn(sT=0.0) == B.INVALID_ARG
    for bad in (-1e-6, float("inf"), float("nan")):
        assert qn(eps=bad) == B.INVALID_ARG
    assert b"eps" in B.lib().arcq_last_error()
    assert qn(gamma=None) == B.INVALID_ARG
    assert qn(x=None) == B.INVALID_ARG
    assert qn(gamma=ctypes.c_void_p(0x10008)) == B.BAD_ALIGN
    assert qn(x=ODD) == B.BAD_ALIGN
    assert qn(codes=ODD) == B.BAD_ALIGN
    assert qn(rows=0, x=None, gamma=None, perm=None, codes=None, scales=None) == B.OK


def g(ac=FAKE, asc=FAKE, sa=1.0, wc=FAKE, wsc=FAKE, sw=1.0, M=4, N=8, Kp=64, y=FAKE, dt=0, ldy=8, ws=None, wsb=0):
    return B.lib().arcq_gemm(ac, asc, sa, wc, wsc, sw, M, N, Kp, y, dt, ldy, ws, wsb, None)


def test_gemm_argument_errors():
    assert g(Kp=0) == B.BAD_SHAPE
    assert g(Kp=40) == B.BAD_SHAPE
    assert g(M=-1) == B.BAD_SHAPE
    assert g(ldy=4) == B.BAD_SHAPE
    assert g(dt=7) == B.INVALID_ARG
    assert g(sa=0.0) == B.INVALID_ARG
    assert g(sw=float("nan")) == B.INVALID_ARG
    assert g(ac=None) == B.INVALID_ARG
    assert g(y=None) == B.INVALID_ARG
    assert g(wc=ODD) == B.BAD_ALIGN
    assert g(y=ctypes.c_void_p(0x10002)) == B.BAD_ALIGN
    assert g(M=0, ac=None, asc=None, y=None) == B.OK
    assert g(N=0, wc=None, wsc=None, y=None) == B.OK
    n = ctypes.c_size_t(123)
    assert B.lib().arcq_gemm_workspace_size(4, 8, 64, ctypes.byref(n)) == B.OK
    assert B.lib().arcq_gemm_workspace_size(4, 8, 40, ctypes.byref(n)) == B.BAD_SHAPE
    # few tiles and a long reduction: split into several runs (at most 8), fp32 partial results in the workspace
    assert B.lib().arcq_gemm_workspace_size(256, 512, 14592, ctypes.byref(n)) == B.OK
    assert n.value % (256 * 512 * 4) == 0 and 2 <= n.value // (256 * 512 * 4) <= 8
    assert g(M=256, N=512, Kp=14592, ldy=512) == B.WORKSPACE_TOO_SMALL
    assert g(M=256, N=512, Kp=14592, ldy=512, ws=FAKE, wsb=1024) == B.WORKSPACE_TOO_SMALL
    assert g(M=256, N=512, Kp=14592, ldy=512, ws=ctypes.c_void_p(0x10010), wsb=1 << 30) == B.BAD_ALIGN
    assert B.lib().arcq_gemm_workspace_size(2048, 4096, 4352, ctypes.byref(n)) == B.OK and n.value == 0


def test_gemm_noalloc_argument_errors_and_scratch_limit():
    """The entry point for callers that cannot allocate: the rules of arcq_gemm, and shapes whose partial results
    exceed the built-in scratch are turned away before anything touches the GPU."""
    ga = lambda ac=FAKE, M=4, N=8, Kp=64, y=FAKE, dt=0, ldy=8, sa=1.0: B.lib().arcq_gemm_noalloc(
        ac, FAKE, sa, FAKE, FAKE, 1.0, M, N, Kp, y, dt, ldy, None)
    assert ga(Kp=40) == B.BAD_SHAPE and ga(M=-1) == B.BAD_SHAPE and ga(ldy=4) == B.BAD_SHAPE
    assert ga(dt=7) == B.INVALID_ARG and ga(sa=0.0) == B.INVALID_ARG and ga(ac=None) == B.INVALID_ARG
    assert ga(ac=ODD) == B.BAD_ALIGN and ga(y=ctypes.c_void_p(0x10002)) == B.BAD_ALIGN
    assert ga(M=0, ac=None, y=None) == B.OK
    n = ctypes.c_size_t(0)
    # a few hundred rows against a few hundred weight rows over a very long reduction: K' split seven times
    assert B.lib().arcq_gemm_workspace_size(896, 640, 14592, ctypes.byref(n)) == B.OK
    assert n.value > B.NOALLOC_SCRATCH_BYTES == 8 << 20
    assert ga(M=896, N=640, Kp=14592, ldy=640) == B.WORKSPACE_TOO_SMALL
    assert b"built-in" in B.lib().arcq_last_error()


def test_check_perm_argument_errors():
    r = ctypes.c_int(0)
    assert B.lib().arcq_check_perm(None, 16, FAKE, ctypes.byref(r), None) == B.INVALID_ARG
    assert B.lib().arcq_check_perm(FAKE, 0, FAKE, ctypes.byref(r), None) == B.BAD_SHAPE


def test_calibration_argument_errors():
    L = B.lib()
    assert L.arcq_calib_absmax(FAKE, 4, 500, 512, FAKE, None) == B.BAD_SHAPE
    assert L.arcq_calib_absmax(FAKE, -1, 512, 512, FAKE, None) == B.BAD_SHAPE
    assert L.arcq_calib_absmax(FAKE, 4, 512, 496, FAKE, None) == B.BAD_SHAPE
    assert L.arcq_calib_absmax(None, 4, 512, 512, FAKE, None) == B.INVALID_ARG
    assert L.arcq_calib_absmax(FAKE, 4, 512, 512, None, None) == B.INVALID_ARG
    assert L.arcq_calib_absmax(ODD, 4, 512, 512, FAKE, None) == B.BAD_ALIGN
    assert L.arcq_calib_absmax(FAKE, 4, 512, 516, FAKE, None) == B.BAD_ALIGN
    assert L.arcq_calib_absmax(FAKE, 4, 512, 512, ctypes.c_void_p(0x10002), None) == B.BAD_ALIGN
    assert L.arcq_calib_absmax(None, 0, 512, 512, None, None) == B.OK                 # empty batch: nothing to do
    s = ctypes.c_int(0)
    assert L.arcq_calib_select(FAKE, 40, FAKE, FAKE, ctypes.byref(s), None) == B.BAD_SHAPE
    assert L.arcq_calib_select(FAKE, B.MAX_K + 16, FAKE, FAKE, ctypes.byref(s), None) == B.BAD_SHAPE
    assert L.arcq_calib_select(None, 64, FAKE, FAKE, ctypes.byref(s), None) == B.INVALID_ARG
    assert L.arcq_calib_select(FAKE, 64, None, FAKE, ctypes.byref(s), None) == B.INVALID_ARG
    assert L.arcq_calib_select(FAKE, 64, FAKE, None, ctypes.byref(s), None) == B.INVALID_ARG
    assert L.arcq_calib_select(FAKE, 64, ctypes.c_void_p(0x10002), FAKE, ctypes.byref(s), None) == B.BAD_ALIGN


def test_mx_argument_errors():
    L = B.lib()
    for fn in (L.arcq_mx_quantize_act, L.arcq_mx_pack_weight):
        assert fn(FAKE, 4, 528, 528, FAKE, 32, FAKE, FAKE, None) == B.BAD_SHAPE          # K % 32
        assert fn(FAKE, 4, 512, 512, FAKE, 16, FAKE, FAKE, None) == B.BAD_SHAPE          # S % 32
        assert fn(FAKE, 4, 512, 496, FAKE, 32, FAKE, FAKE, None) == B.BAD_SHAPE
        assert fn(None, 4, 512, 512, FAKE, 32, FAKE, FAKE, None) == B.INVALID_ARG
        assert fn(FAKE, 4, 512, 512, FAKE, 32, ctypes.c_void_p(0x10008), FAKE, None) == B.BAD_ALIGN
        assert fn(FAKE, 4, 512, 512, ctypes.c_void_p(0x10004), 32, FAKE, FAKE, None) == B.BAD_ALIGN
        assert fn(None, 0, 512, 512, None, 32, None, None, None) == B.OK
    cb, sb = ctypes.c_size_t(0), ctypes.c_size_t(0)
    assert L.arcq_mx_packed_sizes(10, 512, 64, ctypes.byref(cb), ctypes.byref(sb)) == B.OK
    assert (cb.value, sb.value) == (10 * 576 // 2, 10 * 576 // 32)
    mg = lambda M=4, N=8, Kp=64, ac=FAKE, y=FAKE, dt=0, ldy=8: L.arcq_mx_gemm(ac, FAKE, FAKE, FAKE, M, N, Kp, y, dt, ldy, None)
    assert mg(Kp=48) == B.BAD_SHAPE and mg(Kp=0) == B.BAD_SHAPE and mg(ldy=4) == B.BAD_SHAPE
    assert mg(dt=9) == B.INVALID_ARG and mg(ac=None) == B.INVALID_ARG
    assert mg(ac=ctypes.c_void_p(0x10002)) == B.BAD_ALIGN and mg(y=ctypes.c_void_p(0x10002)) == B.BAD_ALIGN
    assert mg(M=0, ac=None, y=None) == B.OK


def test_variant_entry_points_argument_errors():
    L = B.lib()
    for fn in (L.arcq_quantize_act_ex, L.arcq_pack_weight_ex):
        assert fn(FAKE, 4, 512, 512, FAKE, 32, 1.0, 4, FAKE, FAKE, None) == B.INVALID_ARG      # unknown flag bit
        assert b"flags" in L.arcq_last_error()
        assert fn(FAKE, 4, 512, 512, FAKE, 32, 1.0, 0x80000001, FAKE, FAKE, None) == B.INVALID_ARG
        assert fn(FAKE, 4, 520, 520, FAKE, 32, 1.0, 3, FAKE, FAKE, None) == B.BAD_SHAPE        # the plain rules still hold
        assert fn(None, 4, 512, 512, FAKE, 32, 1.0, 3, FAKE, FAKE, None) == B.INVALID_ARG
        for flags in (0, 1, 2, 3):
            assert fn(None, 0, 512, 512, None, 32, 1.0, flags, None, None, None) == B.OK      # nothing to do
    nq = L.arcq_rmsnorm_quantize_act_ex
    assert nq(FAKE, 4, 512, 512, FAKE, 1e-5, FAKE, 32, 1.0, 8, FAKE, FAKE, None) == B.INVALID_ARG
    # the exact-sum bit belongs to the RMSNorm call alone
    assert nq(None, 0, 512, 512, None, 1e-5, None, 32, 1.0, 4 | 3, None, None, None) == B.OK
    assert L.arcq_quantize_act_ex(None, 0, 512, 512, None, 32, 1.0, 4, None, None, None) == B.INVALID_ARG
    assert B.RMSNORM_EXACT_SUM == 4
    assert nq(FAKE, 4, 512, 512, None, 1e-5, FAKE, 32, 1.0, 1, FAKE, FAKE, None) == B.INVALID_ARG   # gamma
    assert nq(None, 0, 512, 512, None, 1e-5, None, 32, 1.0, 3, None, None, None) == B.OK
    for fn in (L.arcq_mx_quantize_act_ex, L.arcq_mx_pack_weight_ex):
        assert fn(FAKE, 4, 512, 512, FAKE, 32, 4, FAKE, FAKE, None) == B.INVALID_ARG
        assert fn(FAKE, 4, 512, 512, FAKE, 16, 1, FAKE, FAKE, None) == B.BAD_SHAPE
        assert fn(None, 0, 512, 512, None, 32, 3, None, None, None) == B.OK
    assert (B.LAYOUT_INTERLEAVED, B.SCALE_ROUND_UP) == (1, 2)


@pytest.mark.parametrize("name", ["arcq_probe_mfma_f16", "arcq_probe_mfma_fp4"])
def test_probe_argument_errors(name):
    probe = getattr(B.lib(), name)
    fl = ctypes.c_double(0)
    assert probe(0, FAKE, ctypes.byref(fl), None) == B.INVALID_ARG
    assert probe(1 << 21, FAKE, ctypes.byref(fl), None) == B.INVALID_ARG
    assert probe(10, None, ctypes.byref(fl), None) == B.INVALID_ARG
    assert probe(10, FAKE, None, None) == B.INVALID_ARG
    assert probe(10, ctypes.c_void_p(0x10002), ctypes.byref(fl), None) == B.BAD_ALIGN


def test_ref_gemm_bf16_argument_errors():
    L = B.lib()
    assert L.arcq_ref_gemm_bf16(FAKE, FAKE, 8, 8, 48, FAKE, 8, None) == B.BAD_SHAPE          # K % 32
    assert L.arcq_ref_gemm_bf16(FAKE, FAKE, 8, 8, 64, FAKE, 4, None) == B.BAD_SHAPE          # ldy < N
    assert L.arcq_ref_gemm_bf16(None, FAKE, 8, 8, 64, FAKE, 8, None) == B.INVALID_ARG
    assert L.arcq_ref_gemm_bf16(ctypes.c_void_p(0x10008), FAKE, 8, 8, 64, FAKE, 8, None) == B.BAD_ALIGN
    assert L.arcq_ref_gemm_bf16(FAKE, FAKE, 0, 8, 64, FAKE, 8, None) == B.OK                # empty


def test_mx_gemm_workspace_entry_points():
    L = B.lib()
    n = ctypes.c_size_t(7)
    assert L.arcq_mx_gemm_workspace_size(16, 4096, 4352, ctypes.byref(n)) == B.OK and n.value == 0       # weight-streaming kernel
    assert L.arcq_mx_gemm_workspace_size(2048, 4096, 4352, ctypes.byref(n)) == B.OK and n.value == 0     # enough tiles
    assert L.arcq_mx_gemm_workspace_size(256, 4096, 14592, ctypes.byref(n)) == B.OK
    assert n.value % (256 * 4096 * 4) == 0 and 2 <= n.value // (256 * 4096 * 4) <= 8
    need = n.value
    assert L.arcq_mx_gemm_workspace_size(256, 4096, 48, ctypes.byref(n)) == B.BAD_SHAPE
    assert L.arcq_mx_gemm_workspace_size(256, 4096, 14592, None) == B.INVALID_ARG
    args = (FAKE, FAKE, FAKE, FAKE, 256, 4096, 14592, FAKE, B.DTYPE_F16, 4096)
    assert L.arcq_mx_gemm_ws(*args, None, 0, None) == B.WORKSPACE_TOO_SMALL
    assert L.arcq_mx_gemm_ws(*args, FAKE, need - 1, None) == B.WORKSPACE_TOO_SMALL
    assert L.arcq_mx_gemm_ws(*args, ctypes.c_void_p(0x10010), need, None) == B.BAD_ALIGN
    assert L.arcq_mx_gemm_ws(FAKE, FAKE, FAKE, FAKE, 256, 4096, 14592, FAKE, 7, 4096, FAKE, need, None) == B.INVALID_ARG
