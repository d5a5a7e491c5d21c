"""NVFP4 number formats, written as tables plus "nearest entry" searches.

Test infrastructure (see the package docstring).  Nothing here is tuned.

Appendix A / Table "formats" of the paper fix the formats:
  * element  : FP4 E2M1, exponent bias 1, largest magnitude 6
  * block scale : FP8 E4M3, exponent bias 7, largest normal 448, one per 16
  * tensor scale: one FP32 number per tensor
The paper only writes round(.) (Section 3.1 eq. (1)); the reading used here
is round-to-nearest with ties to the code whose last mantissa bit is 0, and
saturation at the largest finite magnitude (E2M1 has no Inf/NaN; the E4M3
flavour is the "finite" one whose only non-finite pattern, NaN, is never
produced).
"""
import numpy as np

# --- E2M1 -----------------------------------------------------------------
# code = sign<<3 | exponent(2 bits)<<1 | mantissa(1 bit); bias 1, exponent 0
# is subnormal: magnitudes m*0.5 for exponent 0, (1+m/2)*2^(e-1) otherwise.


def _e2m1_magnitude(idx):
    e, m = idx >> 1, idx & 1
    if e == 0:
        return 0.5 * m
    return (1.0 + 0.5 * m) * 2.0 ** (e - 1)


E2M1_GRID = np.array([_e2m1_magnitude(i) for i in range(8)], dtype=np.float64)


def e2m1_decode(code):
    """4-bit code(s) -> float64 value(s).  -0 decodes to -0.0."""
    code = np.asarray(code).astype(np.int64)
    mag = E2M1_GRID[code & 7]
    return np.where((code & 8) != 0, -mag, mag)


def e2m1_encode_magnitude(w):
    """Index (0..7) of the grid value nearest to w >= 0.

    Ties go to the even index (mantissa bit 0); anything above 6 maps to 6.
    Distances are formed in float64, where w - g is exact for every float32
    w within reach of a tie, so the comparison is the mathematical one.
    """
    w = np.asarray(w, dtype=np.float64)
    if np.any(~(w >= 0)):
        raise ValueError("e2m1_encode_magnitude expects finite w >= 0")
    w = np.minimum(w, E2M1_GRID[-1])                      # saturation: no code beyond 6
    dist = np.abs(w[..., None] - E2M1_GRID)             # [..., 8]
    best = dist.min(axis=-1, keepdims=True)
    is_best = dist == best                                # one or two True per row
    even_first = np.array([0, 2, 4, 6, 1, 3, 5, 7])
    # pick the even candidate when two entries are equally near
    pick = np.argmax(is_best[..., even_first], axis=-1)
    return even_first[pick].astype(np.uint8)


# --- E4M3 (finite flavour) -------------------------------------------------
# byte = sign<<7 | exponent(4)<<3 | mantissa(3); bias 7; exponent 0 subnormal;
# exponent 15 with mantissa 7 is NaN, every other pattern is finite (max 448).


def e4m3_decode(byte):
    """E4M3 byte(s) -> float64 value(s); the NaN patterns decode to NaN."""
    b = np.asarray(byte).astype(np.int64)
    s, e, m = (b >> 7) & 1, (b >> 3) & 15, b & 7
    val = np.where(e == 0, (m / 8.0) * 2.0 ** -6, (1.0 + m / 8.0) * 2.0 ** (e.astype(np.float64) - 7))
    val = np.where((e == 15) & (m == 7), np.nan, val)
    return np.where(s == 1, -val, val)


# the 127 finite non-negative values, ascending; the byte IS the table index
E4M3_POS = e4m3_decode(np.arange(0x7F))
assert np.all(np.diff(E4M3_POS) > 0) and E4M3_POS[-1] == 448.0


def e4m3_encode_rne_sat(u):
    """Byte (0x00..0x7E) of the finite E4M3 value nearest to u >= 0.

    Ties go to the even byte (= even mantissa); u above 448 saturates to 448.
    """
    u = np.asarray(u, dtype=np.float64)
    if np.any(~(u >= 0)):
        raise ValueError("e4m3_encode_rne_sat expects finite u >= 0")
    hi = np.searchsorted(E4M3_POS, u, side="left")       # first entry >= u
    hi = np.minimum(hi, len(E4M3_POS) - 1)
    lo = np.maximum(hi - 1, 0)
    d_lo = np.abs(u - E4M3_POS[lo])
    d_hi = np.abs(E4M3_POS[hi] - u)
    take_hi = (d_hi < d_lo) | ((d_hi == d_lo) & (hi % 2 == 0))
    out = np.where(take_hi, hi, lo)
    out = np.where(u >= 448.0, 0x7E, out)
    return out.astype(np.uint8)


def e4m3_encode_up_sat(u):
    """Byte (0x00..0x7E) of the smallest finite E4M3 value that is not below u >= 0 (rounding up);
    u above 448 saturates to 448.  The error analysis of Section 3.4 takes the ratio alpha of the
    stored scale to the ideal one in [1, 1.125]: a scale that is never rounded down."""
    u = np.asarray(u, dtype=np.float64)
    if np.any(~(u >= 0)):
        raise ValueError("e4m3_encode_up_sat expects finite u >= 0")
    hi = np.searchsorted(E4M3_POS, u, side="left")       # first entry >= u
    return np.minimum(hi, len(E4M3_POS) - 1).astype(np.uint8)
