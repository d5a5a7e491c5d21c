"""ARCQuant on the MXFP4 format, step by step, in numpy.  Test infrastructure only.

The paper's method is format-agnostic (Section 4.3 "Generalizability" and the appendix table on INT4 and
MXFP4): quantize, form the residual of the outlier channels, quantize it again, concatenate along K,
duplicate the weights' outlier blocks, one GEMM over K' = K + S.  Only the block format changes
(Section 3.1 "Block-scaled Quantization", Appendix A): MXFP4 has g = 32 E2M1 elements per block and one
E8M0 scale (a power of two, value 2^(byte - 127)), and no tensor scale.

Scale rule (the paper gives none for MXFP4; this is the rule of the OCP Microscaling specification the
paper cites for the format): shared exponent = floor(log2(max |v|)) - emax_elem with emax_elem = 2 for
E2M1, scale X = 2^shared; elements = round-to-nearest-even of v / X on the E2M1 grid, saturating at 6
(so a block maximum in (6X, 8X) clips).  Everything is exact except the element rounding: v / X is a
power-of-two scaling, and the residual v - X * Q is exact in fp32 (v has 11 significant bits).
Readings: an all-zero block gets scale byte 127 (X = 1) and zero codes; S is a multiple of 32.

Packed layout: codes uint8 [rows, K'/2] (element 2i in bits 0-3 of byte i), scales uint8 [rows, K'/32];
block b < K/32 primary, block K/32 + i the residual of primary block (K - S)/32 + i.

Two variants, both off by default, as for NVFP4:
  layout="interleaved"   Appendix D: blocks without compensation first, then every outlier block
                         immediately followed by its residual block (its copy, for weights);
  scale_rounding="up"    X is the smallest power of two with max |v| <= 6 X, so that no element clips
                         (the scale is never below the ideal max / q_max: alpha >= 1 in Section 3.4);
                         one more than the rule above exactly when max |v| / 2^floor(log2 max |v|) > 1.5.
"""
import numpy as np

from . import formats as F

G = 32            # MXFP4 block size
EMAX_ELEM = 2     # largest exponent of E2M1 (6 = 1.5 * 2^2)
E8M0_BIAS = 127


def e8m0_decode(b):
    """uint8 -> float64 2^(b - 127); 255 is NaN."""
    b = np.asarray(b, dtype=np.uint8)
    out = np.ldexp(1.0, b.astype(np.int32) - E8M0_BIAS)
    return np.where(b == 255, np.nan, out)


def interleaved_order(K, S):
    """Appendix D: physical block position -> block index in the concatenated layout."""
    nb, no = K // G, S // G
    order = list(range(nb - no))
    for i in range(no):
        order += [nb - no + i, nb + i]
    return np.array(order, dtype=np.int64)


def _lay_out(codes, sb, K, S, layout):
    if layout == "concat":
        return codes, sb
    if layout == "interleaved":
        order = interleaved_order(K, S)
        return codes[:, order], sb[:, order]
    raise ValueError("layout must be 'concat' or 'interleaved'")


def quantize_blocks(v, scale_rounding="nearest"):
    """v float32 [..., 32] finite -> (sbyte uint8 [...], codes uint8 [..., 32], X float64 [...]).
    scale_rounding "nearest" is the floor rule of the header (the name matches the NVFP4 oracle's default)."""
    if scale_rounding not in ("nearest", "up"):
        raise ValueError("scale_rounding must be 'nearest' or 'up'")
    v = np.asarray(v)
    assert v.dtype == np.float32 and v.shape[-1] == G
    if not np.all(np.isfinite(v)):
        raise ValueError("non-finite input")
    amax = np.abs(v).max(axis=-1).astype(np.float64)
    _, e = np.frexp(amax)                                   # amax = m * 2^e, m in [0.5, 1): floor(log2) = e - 1
    shared = np.where(amax > 0, e - 1 - EMAX_ELEM, 0)
    if scale_rounding == "up":
        # amax / 2^(e-1) in [1, 2), exact; above 1.5 the floor rule's 6 X falls short of amax
        shared = shared + ((amax > 0) & (np.ldexp(amax, -(e - 1)) > 1.5))
    if np.any(shared < -E8M0_BIAS) or np.any(shared > 127):
        raise ValueError("shared exponent outside E8M0")
    sbyte = (shared + E8M0_BIAS).astype(np.uint8)
    X = np.ldexp(1.0, shared)
    w = np.abs(v.astype(np.float64)) / X[..., None]        # exact
    idx = F.e2m1_encode_magnitude(np.minimum(w, 6.0))
    codes = (np.signbit(v).astype(np.uint8) << 3) | idx.astype(np.uint8)
    return sbyte, codes.astype(np.uint8), X


def residual_blocks(v, codes, X):
    """r = v - X * Q, exact, as float32."""
    r = v.astype(np.float64) - F.e2m1_decode(codes) * X[..., None]
    r32 = r.astype(np.float32)
    assert np.array_equal(r32.astype(np.float64), r)
    return r32


def pack_nibbles(codes):
    c = np.asarray(codes, dtype=np.uint8)
    return (c[..., 0::2] | (c[..., 1::2] << 4)).astype(np.uint8)


def unpack_nibbles(packed):
    p = np.asarray(packed, dtype=np.uint8)
    out = np.empty(p.shape[:-1] + (2 * p.shape[-1],), dtype=np.uint8)
    out[..., 0::2] = p & 0xF
    out[..., 1::2] = p >> 4
    return out


def _check_shape(K, S):
    if K <= 0 or K % G or S < 0 or S % G or S > K:
        raise ValueError("need K > 0, K % 32 == 0, 0 <= S <= K, S % 32 == 0")


def quantize_act(Xa, perm, S, layout="concat", scale_rounding="nearest"):
    """Online activation quantizer (Section 3.2 steps (1)-(3)) in MXFP4.  Xa fp16 [M, K]."""
    Xa = np.asarray(Xa)
    assert Xa.dtype == np.float16 and Xa.ndim == 2
    M, K = Xa.shape
    _check_shape(K, S)
    perm = np.asarray(perm)
    assert perm.shape == (K,)
    Xp = Xa[:, perm].astype(np.float32).reshape(M, K // G, G)
    sb, codes, X = quantize_blocks(Xp, scale_rounding)
    if S:
        o = (K - S) // G
        r = residual_blocks(Xp[:, o:], codes[:, o:], X[:, o:])
        sb_r, codes_r, _ = quantize_blocks(r, scale_rounding)
        codes = np.concatenate([codes, codes_r], axis=1)
        sb = np.concatenate([sb, sb_r], axis=1)
    codes, sb = _lay_out(codes, sb, K, S, layout)
    Kp = K + S
    return pack_nibbles(codes.reshape(M, Kp)), sb.reshape(M, Kp // G)


def pack_weight(W, perm, S, layout="concat", scale_rounding="nearest"):
    """Offline weight packer: reorder, quantize, append a verbatim copy of the outlier blocks."""
    W = np.asarray(W)
    assert W.dtype == np.float16 and W.ndim == 2
    N, K = W.shape
    _check_shape(K, S)
    Wp = W[:, np.asarray(perm)].astype(np.float32).reshape(N, K // G, G)
    sb, codes, _ = quantize_blocks(Wp, scale_rounding)
    if S:
        o = (K - S) // G
        codes = np.concatenate([codes, codes[:, o:]], axis=1)
        sb = np.concatenate([sb, sb[:, o:]], axis=1)
    codes, sb = _lay_out(codes, sb, K, S, layout)
    Kp = K + S
    return pack_nibbles(codes.reshape(N, Kp)), sb.reshape(N, Kp // G)


def dequantize(codes, scales):
    """Packed operand -> float64 [rows, K'] (exact)."""
    q = F.e2m1_decode(unpack_nibbles(codes))
    sc = e8m0_decode(scales)
    rows, Kp = q.shape
    return (q.reshape(rows, Kp // G, G) * sc[..., None]).reshape(rows, Kp)


def gemm(a_codes, a_scales, w_codes, w_scales):
    """Y = deq(A_aug) deq(W_aug)^T in float64 (Section 3.2 eq. (2)), [M, N]."""
    return dequantize(a_codes, a_scales) @ dequantize(w_codes, w_scales).T
