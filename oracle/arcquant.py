"""ARCQuant hot path, step by step, in numpy.  Test infrastructure only.

Notation follows the paper: X [M, K] activations, W [N, K] weights
(Y = X W^T, Section 3.1 "Problem Definition"), g = 16 the NVFP4 group size,
q_max = 6, S outlier channels, K' = K + S.

Arithmetic recipe (the paper gives eq. (1) in real numbers and is silent on
machine arithmetic; this is the frozen reading, every rounding listed):

  ginv  = fl32(1 / fl32(6 * s_T))                 once per tensor
  amax  = max_i |v_i|                             exact
  u     = fl32(amax * ginv)                       eq. (1): s = max|X| / q_max, in units of s_T
  sbyte = E4M3 nearest-even, saturating, of u     block scale (Appendix A)
  s     = fl32(E4M3_value(sbyte) * s_T)           effective scale of the block
  if s == 0: every magnitude is 0
  else:  inv = fl32(1 / s);  w_i = fl32(|v_i| * inv);  idx_i = E2M1 nearest-even of min(w_i, 6)
  code_i = signbit(v_i) << 3 | idx_i              eq. (1): Q = round(X / s)
  residual r_i = fl32(v_i - G[idx_i] * sign_i * s)     one rounding (fused multiply-add);
                                                  Section 3.2 step (2): R_o = X_o - s * Q_{X_o}

The residual block is quantized by the same routine with the same s_T
(eq. (2) has a single scale vector for the augmented operand, and a standard
block-scaled GEMM has one tensor scale per operand).

Packed layout (Section 3.2 step (3): plain concatenation along K):
  codes  uint8 [rows, K'/2]  byte i = element 2i in bits 0-3, element 2i+1 in bits 4-7
  scales uint8 [rows, K'/16] block b < K/16 primary; block K/16 + i is the residual
                             of primary block (K - S)/16 + i

Two variants, both off by default:
  layout="interleaved"   Appendix D "Interleaved Channel Layout": the same blocks in another physical
                         order -- the (K - S)/16 blocks without compensation first, then every outlier
                         block immediately followed by its residual block (by its copy, for weights);
  scale_rounding="up"    the block scale is the smallest E4M3 value not below u instead of the nearest
                         (Section 3.4 takes alpha = s / (max / q_max) in [1, 1.125], a scale never
                         rounded down); u > 448 still saturates, and a nonzero u below the smallest
                         subnormal 2^-9 goes to 2^-9 rather than to 0.
"""
import numpy as np

from . import formats as F

G = 16          # NVFP4 group size (Appendix A)
QMAX = 6.0      # largest E2M1 magnitude

_f32 = np.float32


def tensor_ginv(s_T):
    """fl32(1 / fl32(6 * s_T)) -- the per-tensor reciprocal used for block scales."""
    s_T = _f32(s_T)
    if not (np.isfinite(s_T) and s_T > 0):
        raise ValueError("tensor scale must be finite and > 0")
    return _f32(1.0) / (_f32(QMAX) * s_T)


def _scale_encoder(scale_rounding):
    if scale_rounding == "nearest":
        return F.e4m3_encode_rne_sat
    if scale_rounding == "up":
        return F.e4m3_encode_up_sat
    raise ValueError("scale_rounding must be 'nearest' or 'up'")


def interleaved_order(K, S):
    """Appendix D: physical block position -> block index in the concatenated layout."""
    nb, no = K // G, S // G
    order = list(range(nb - no))
    for i in range(no):
        order.append(nb - no + i)        # primary block of outlier group i
        order.append(nb + i)             # its residual (or, for weights, its copy)
    return np.array(order, dtype=np.int64)


def _lay_out(codes, sb, K, S, layout):
    """codes [rows, K'/16, 16], sb [rows, K'/16] in concatenated order -> the requested order."""
    if layout == "concat":
        return codes, sb
    if layout == "interleaved":
        order = interleaved_order(K, S)
        return codes[:, order], sb[:, order]
    raise ValueError("layout must be 'concat' or 'interleaved'")


def quantize_blocks(v, s_T, scale_rounding="nearest"):
    """NVFP4-quantize blocks of 16 (Section 3.1 eq. (1), Appendix A).

    v    float32 [..., 16], finite
    s_T  float32 tensor scale
    returns (sbyte uint8 [...], codes uint8 [..., 16] one 4-bit code per entry,
             s float32 [...] effective block scale)
    """
    v = np.asarray(v)
    assert v.dtype == np.float32 and v.shape[-1] == G
    if not np.all(np.isfinite(v)):
        raise ValueError("non-finite input")
    s_T = _f32(s_T)
    ginv = tensor_ginv(s_T)

    absv = np.abs(v)
    amax = absv.max(axis=-1)                                   # exact
    u = (amax * ginv).astype(np.float32)                       # one fp32 rounding
    sbyte = _scale_encoder(scale_rounding)(u)
    s = (F.e4m3_decode(sbyte).astype(np.float32) * s_T).astype(np.float32)

    nz = s != 0
    inv = np.zeros_like(s)
    inv[nz] = _f32(1.0) / s[nz]                                 # IEEE fp32 division
    w = (absv * inv[..., None]).astype(np.float32)             # one fp32 rounding
    idx = F.e2m1_encode_magnitude(np.minimum(w, _f32(QMAX)))
    idx = np.where(nz[..., None], idx, 0).astype(np.uint8)
    sign = np.signbit(v).astype(np.uint8)
    codes = (sign << 3) | idx
    return sbyte, codes.astype(np.uint8), s


def residual_blocks(v, codes, s):
    """r = fl32(v - deq) with deq = G[code] * s formed exactly (Section 3.2 step (2)).

    G[code] has at most 2 significant bits and s 24, so the product is exact in
    float64; v is within a factor of a few of it, so the difference is exact in
    float64 too, and the single cast to float32 is the only rounding: this is a
    fused multiply-add in fp32.
    """
    deq = F.e2m1_decode(codes) * s.astype(np.float64)[..., None]
    return (v.astype(np.float64) - deq).astype(np.float32)


def pack_nibbles(codes):
    """uint8 [..., n] of 4-bit codes -> uint8 [..., n/2], even element in the low nibble."""
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
        raise ValueError("need K > 0, K % 16 == 0, 0 <= S <= K, S % 16 == 0")


def quantize_act(X, perm, S, s_T, layout="concat", scale_rounding="nearest"):
    """Online activation quantizer (Section 3.2 "Online Activation Quantization").

    (1) reorder channels: Xp[:, j] = X[:, perm[j]]; quantize every block of 16;
    (2) on the last S reordered channels form the residual and quantize it;
    (3) concatenate [Q_X | Q_R] and [s_X | s_R] along K.
    X fp16 [M, K]; perm int [K]; returns (codes uint8 [M, K'/2], scales uint8 [M, K'/16]).
    """
    X = np.asarray(X)
    assert X.dtype == np.float16 and X.ndim == 2
    M, K = X.shape
    _check_shape(K, S)
    perm = np.asarray(perm)
    assert perm.shape == (K,)
    Xp = X[:, perm].astype(np.float32).reshape(M, K // G, G)

    sb, codes, s = quantize_blocks(Xp, s_T, scale_rounding)
    if S:
        o = (K - S) // G
        r = residual_blocks(Xp[:, o:], codes[:, o:], s[:, o:])
        sb_r, codes_r, _ = quantize_blocks(r, s_T, scale_rounding)
        codes = np.concatenate([codes, codes_r], axis=1)
        sb = np.concatenate([sb, sb_r], axis=1)
    codes, sb = _lay_out(codes, sb, K, S, layout)
    Kp = K + S
    return pack_nibbles(codes.reshape(M, Kp)), sb.reshape(M, Kp // G)


def rmsnorm(X, gamma, eps):
    """RMSNorm in front of the quantizer (Section 3.3 lists it as part of the fused kernel; the
    paper gives no formula, so this is the standard definition y = x / sqrt(mean(x^2) + eps) * gamma
    with the arithmetic of the reference Llama/Qwen layer, every rounding listed):

      ms   = fl32( fl64( fl64(sum_i x_i^2) / K ) )   the sum itself is EXACT (integer arithmetic: every
                                            fp16 value is a multiple of 2^-24), rounded once to float64,
                                            divided in float64, rounded to fp32 -- no summation order
      rstd = fl32( 1 / fl32( sqrt( fl32(ms + eps) ) ) )        IEEE fp32 add, sqrt, divide
      t_i  = fl16( fl32(x_i * rstd) )                           normalised value in the model dtype
      y_i  = fl16( t_i * gamma_i )                              product of two fp16, rounded once

    X fp16 [M, K], gamma fp16 [K], eps float; returns fp16 [M, K].
    """
    X = np.asarray(X)
    gamma = np.asarray(gamma)
    assert X.dtype == np.float16 and gamma.dtype == np.float16 and gamma.shape == (X.shape[1],)
    eps = _f32(eps)
    if not (np.isfinite(eps) and eps >= 0):
        raise ValueError("eps must be finite and >= 0")
    M, K = X.shape
    sumsq = np.empty(M, dtype=np.float64)
    for r0 in range(0, M, 256):                                # chunks only bound the memory of the big integers
        scaled = X[r0:r0 + 256].astype(np.float64) * 2.0 ** 24
        v = scaled.astype(np.int64)
        if not np.array_equal(v, scaled):
            raise ValueError("non-finite input")
        v = v.astype(object)
        n = (v * v).sum(axis=1)                                # Python integers: exact, any order
        sumsq[r0:r0 + 256] = [float(t) for t in n]             # int -> float64 is correctly rounded
    ms = (sumsq * 2.0 ** -48 / K).astype(np.float32)
    rstd = _f32(1.0) / np.sqrt((ms + eps).astype(np.float32)).astype(np.float32)
    t = (X.astype(np.float32) * rstd[:, None]).astype(np.float32).astype(np.float16)
    # fp16 x fp16 is exact in fp32 (22 significant bits); one rounding to fp16
    return (t.astype(np.float32) * gamma.astype(np.float32)[None, :]).astype(np.float16)


def rmsnorm_quantize_act(X, gamma, eps, perm, S, s_T, layout="concat", scale_rounding="nearest"):
    """The fused kernel of Section 3.3: RMSNorm, then the online activation quantizer."""
    return quantize_act(rmsnorm(X, gamma, eps), perm, S, s_T, layout, scale_rounding)


def pack_weight(W, perm, S, s_T, layout="concat", scale_rounding="nearest"):
    """Offline weight packer (Section 3.2 "Offline Weight Quantization").

    Reorder the K axis to match X, quantize (plain round-to-nearest), then append
    a verbatim copy of the quantized outlier columns: Q_Waug = [Q_W | Q_Wo].
    W fp16 [N, K]; returns (codes uint8 [N, K'/2], scales uint8 [N, K'/16]).
    """
    W = np.asarray(W)
    assert W.dtype == np.float16 and W.ndim == 2
    N, K = W.shape
    _check_shape(K, S)
    Wp = W[:, np.asarray(perm)].astype(np.float32).reshape(N, K // G, G)
    sb, codes, _ = quantize_blocks(Wp, s_T, scale_rounding)
    if S:
        o = (K - S) // G
        codes = np.concatenate([codes, codes[:, o:]], axis=1)
        sb = np.concatenate([sb, sb[:, o:]], axis=1)
    codes, sb = _lay_out(codes, sb, K, S, layout)
    Kp = K + S
    return pack_nibbles(codes.reshape(N, Kp)), sb.reshape(N, Kp // G)


def dequantize(codes, scales, s_T):
    """Packed operand -> float64 [rows, K'] = G[code] * E4M3(scale) * s_T (exact in fp64)."""
    q = F.e2m1_decode(unpack_nibbles(codes))                  # [rows, K']
    sc = F.e4m3_decode(scales) * np.float64(_f32(s_T))        # [rows, K'/16]
    rows, Kp = q.shape
    return (q.reshape(rows, Kp // G, G) * sc[..., None]).reshape(rows, Kp)


def gemm(a_codes, a_scales, a_sT, w_codes, w_scales, w_sT):
    """Y = deq(A_aug) deq(W_aug)^T in float64 (Section 3.2 eq. (2)), [M, N]."""
    A = dequantize(a_codes, a_scales, a_sT)
    Wd = dequantize(w_codes, w_scales, w_sT)
    return A @ Wd.T


def gemm_rows(a_codes, a_scales, a_sT, w_codes, w_scales, w_sT, rows):
    """Same product restricted to the given rows of A (for sampled parity at full sizes)."""
    rows = np.asarray(rows)
    return gemm(a_codes[rows], a_scales[rows], a_sT, w_codes, w_scales, w_sT)
