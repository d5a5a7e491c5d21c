"""Second, deliberately different implementation: exact rationals and loops.

Test infrastructure only; used on tiny inputs to pin oracle.formats and
oracle.arcquant.  Nothing is shared with them: the grids are rebuilt from
the bit-field definitions (Appendix A, Table "formats": E2M1 bias 1,
E4M3 bias 7), fp32 rounding is done by hand on fractions.Fraction values,
nearest-value searches are argmin loops, and the GEMM is a triple loop
over the sum in Section 3.2 eq. (2).
"""
from fractions import Fraction as Fr


def e2m1_value(code):
    s, e, m = (code >> 3) & 1, (code >> 1) & 3, code & 1
    mag = Fr(m, 2) if e == 0 else (1 + Fr(m, 2)) * Fr(2) ** (e - 1)
    return -mag if s else mag


def e4m3_value(byte):
    s, e, m = (byte >> 7) & 1, (byte >> 3) & 15, byte & 7
    if e == 15 and m == 7:
        raise ValueError("NaN pattern")
    mag = Fr(m, 8) * Fr(2) ** -6 if e == 0 else (1 + Fr(m, 8)) * Fr(2) ** (e - 7)
    return -mag if s else mag


def _nearest_even(x, candidates):
    """candidates: list of (code, value) with value >= 0; nearest to x, tie -> even code;
    x beyond the largest value goes to the largest value."""
    best = None
    for code, val in candidates:
        d = abs(x - val)
        if best is None or d < best[0] or (d == best[0] and code % 2 == 0):
            best = (d, code)
    return best[1]


_E2M1_POS = [(c, e2m1_value(c)) for c in range(8)]
_E4M3_POS = [(b, e4m3_value(b)) for b in range(0x7F)]


def e2m1_nearest(w):
    return _nearest_even(Fr(w), _E2M1_POS)


def e4m3_nearest_sat(u):
    return _nearest_even(Fr(u), _E4M3_POS)


def e4m3_up_sat(u):
    """Byte of the smallest E4M3 value >= u (a loop over all 127 values); beyond 448: 448."""
    u = Fr(u)
    best = None
    for byte, val in _E4M3_POS:
        if val >= u and (best is None or val < best[1]):
            best = (byte, val)
    return 0x7E if best is None else best[0]


def round_f32(q):
    """Round a rational to the nearest IEEE binary32 value (ties to even), as a Fraction.
    Subnormals are kept; overflow is not handled (never reached by the tests)."""
    q = Fr(q)
    if q == 0:
        return q
    a = abs(q)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fr(2) ** e > a:
        e -= 1
    assert Fr(2) ** e <= a < Fr(2) ** (e + 1)
    e = max(e, -126)
    quantum = Fr(2) ** (e - 23)
    n = round(a / quantum)          # Python rounds Fractions half-to-even
    r = n * quantum
    return -r if q < 0 else r


def round_f64(q):
    """Nearest IEEE binary64 value (ties to even) of a positive rational in the normal range, as a Fraction."""
    q = Fr(q)
    if q == 0:
        return q
    assert q > 0
    e = q.numerator.bit_length() - q.denominator.bit_length()
    if Fr(2) ** e > q:
        e -= 1
    quantum = Fr(2) ** (e - 52)
    return round(q / quantum) * quantum


def round_f16(q):
    """Nearest IEEE binary16 value (ties to even) of a rational, as a Fraction (no overflow handling)."""
    q = Fr(q)
    if q == 0:
        return q
    a = abs(q)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fr(2) ** e > a:
        e -= 1
    e = max(e, -14)
    quantum = Fr(2) ** (e - 10)
    r = round(a / quantum) * quantum
    return -r if q < 0 else r


def sqrt_f32(v):
    """Correctly rounded binary32 square root of a positive fp32-valued rational, decided exactly:
    lo = largest fp32 value <= sqrt(v); the upper neighbour is taken iff (lo + ulp/2)^2 <= v (a tie
    cannot occur: the square of a midpoint has too many bits to be an fp32 value)."""
    v = Fr(v)
    assert v > 0
    from math import isqrt
    shift = 400                                          # guard bits: floor(sqrt(v)) to 2^-200
    root = Fr(isqrt(int(v * Fr(2) ** shift)), 2 ** (shift // 2))
    lo = round_f32_down(root)
    e = lo.numerator.bit_length() - lo.denominator.bit_length()
    if Fr(2) ** e > lo:
        e -= 1
    ulp = Fr(2) ** (max(e, -126) - 23)
    mid = lo + ulp / 2
    return lo + ulp if mid * mid <= v else lo


def round_f32_down(q):
    """Largest binary32 value <= q (q > 0)."""
    q = Fr(q)
    e = q.numerator.bit_length() - q.denominator.bit_length()
    if Fr(2) ** e > q:
        e -= 1
    quantum = Fr(2) ** (max(e, -126) - 23)
    return (q // quantum) * quantum


def rmsnorm_row(x, gamma, eps):
    """One row of the RMSNorm recipe of oracle.arcquant.rmsnorm in exact rationals with hand-made
    roundings.  x, gamma: fp16-valued numbers; eps fp32-valued.  Returns a list of Fractions."""
    x = [Fr(v) for v in x]
    ms = round_f32(round_f64(round_f64(sum(v * v for v in x)) / len(x)))
    rstd = round_f32(1 / sqrt_f32(round_f32(ms + Fr(eps))))
    out = []
    for v, g in zip(x, gamma):
        t = round_f16(round_f32(v * rstd))
        out.append(round_f16(t * Fr(g)))
    return out


def quantize_block(v, s_T, scale_up=False):
    """v: 16 numbers exactly representable in fp32 (floats or Fractions), s_T fp32-valued.
    Returns (scale_byte, [16 codes], [16 residuals as Fractions]).
    Same recipe as oracle.arcquant's header, every fp32 rounding done by round_f32;
    scale_up: the block scale is rounded up instead of to nearest."""
    v = [Fr(x) for x in v]
    neg = [(x < 0) for x in v]
    s_T = Fr(s_T)
    ginv = round_f32(1 / round_f32(6 * s_T))
    amax = max(abs(x) for x in v)
    u = round_f32(amax * ginv)
    sb = e4m3_up_sat(u) if scale_up else e4m3_nearest_sat(u)
    s = round_f32(e4m3_value(sb) * s_T)
    codes, res = [], []
    for x, n in zip(v, neg):
        if s == 0:
            idx = 0
        else:
            inv = round_f32(1 / s)
            w = round_f32(abs(x) * inv)
            idx = e2m1_nearest(min(w, Fr(6)))
        code = (8 if n else 0) | idx
        codes.append(code)
        res.append(round_f32(x - e2m1_value(code) * s))
    return sb, codes, res


def quantize_block_real(v, s_T):
    """The same block under exact real arithmetic for the element division
    (codes = nearest-even of |v| / s with the true quotient).  Diagnostic only:
    shows how often the fp32 reciprocal-multiply recipe departs from eq. (1)
    evaluated in real numbers."""
    v = [Fr(x) for x in v]
    s_T = Fr(s_T)
    ginv = round_f32(1 / round_f32(6 * s_T))
    u = round_f32(max(abs(x) for x in v) * ginv)
    sb = e4m3_nearest_sat(u)
    s = round_f32(e4m3_value(sb) * s_T)
    codes = []
    for x in v:
        idx = 0 if s == 0 else e2m1_nearest(min(abs(x) / s, Fr(6)))
        codes.append((8 if x < 0 else 0) | idx)
    return sb, codes


def gemm_loops(a_codes, a_scales, a_sT, w_codes, w_scales, w_sT):
    """Y[m][n] = s_Ta s_Tw sum_b sx[m][b] sw[n][b] sum_i qx[m][16b+i] qw[n][16b+i]
    (Section 3.2 eq. (2)); a_codes / w_codes are UNPACKED 4-bit codes per element
    (lists of lists), scales are E4M3 bytes per block.  Exact, returns Fractions."""
    M, N = len(a_codes), len(w_codes)
    Kp = len(a_codes[0])
    Y = [[Fr(0)] * N for _ in range(M)]
    for m in range(M):
        for n in range(N):
            acc = Fr(0)
            for b in range(Kp // 16):
                dot = Fr(0)
                for i in range(16):
                    dot += e2m1_value(a_codes[m][16 * b + i]) * e2m1_value(w_codes[n][16 * b + i])
                acc += e4m3_value(a_scales[m][b]) * e4m3_value(w_scales[n][b]) * dot
            Y[m][n] = acc * Fr(a_sT) * Fr(w_sT)
    return Y
