"""Property tests (hypothesis) of the oracle's encoders and block recipe: monotonicity, symmetry, power-of-two
scale invariance, idempotence on grid values, and the interleaved layout as an involution-free permutation."""
import numpy as np
from hypothesis import given, settings, strategies as st

from oracle import arcquant as A
from oracle import formats as F
from oracle import mxfp4 as MX

f32 = st.floats(min_value=0.0, max_value=500.0, allow_nan=False, width=32)
fp16_vals = st.floats(min_value=-60000.0, max_value=60000.0, allow_nan=False, width=16)


@settings(max_examples=300, deadline=None, derandomize=True)
@given(st.lists(f32, min_size=2, max_size=40))
def test_scale_encoders_are_monotone_and_ordered(us):
    u = np.sort(np.array(us, dtype=np.float32))
    near, up = F.e4m3_encode_rne_sat(u).astype(int), F.e4m3_encode_up_sat(u).astype(int)
    assert np.all(np.diff(near) >= 0) and np.all(np.diff(up) >= 0)
    assert np.all(up >= near) and np.all(up - near <= 1)
    vals = F.e4m3_decode(np.arange(0x7F))
    ok = u <= 448
    assert np.all(np.abs(vals[near[ok]] - u[ok]) <= np.abs(vals[np.clip(near[ok] + 1, 0, 0x7E)] - u[ok]))
    assert np.all(np.abs(vals[near[ok]] - u[ok]) <= np.abs(vals[np.clip(near[ok] - 1, 0, 0x7E)] - u[ok]))


@settings(max_examples=300, deadline=None, derandomize=True)
@given(st.lists(st.floats(min_value=0.0, max_value=8.0, allow_nan=False, width=32), min_size=2, max_size=40))
def test_element_encoder_is_monotone_and_nearest(ws):
    w = np.sort(np.array(ws, dtype=np.float32))
    idx = F.e2m1_encode_magnitude(w).astype(int)
    assert np.all(np.diff(idx) >= 0)
    g = F.E2M1_GRID
    wc = np.minimum(w.astype(np.float64), 6.0)
    assert np.all(np.abs(g[idx] - wc) <= np.abs(g[np.clip(idx + 1, 0, 7)] - wc))
    assert np.all(np.abs(g[idx] - wc) <= np.abs(g[np.clip(idx - 1, 0, 7)] - wc))


@settings(max_examples=150, deadline=None, derandomize=True)
@given(st.lists(fp16_vals, min_size=16, max_size=16), st.integers(min_value=-6, max_value=6),
       st.sampled_from(["nearest", "up"]))
def test_block_recipe_symmetry_and_power_of_two_invariance(vals, e, rounding):
    v = np.array(vals, dtype=np.float16).astype(np.float32)[None, :]
    s_T = np.float32(0.37)
    sb, codes, s = A.quantize_blocks(v, s_T, rounding)
    # negating the block flips exactly the sign bits
    sb_n, codes_n, _ = A.quantize_blocks(-v, s_T, rounding)
    assert np.array_equal(sb, sb_n) and np.array_equal(codes ^ 8, codes_n)
    # scaling the block and the tensor scale by the same power of two changes nothing (all steps are exact or
    # scale with it), as long as nothing leaves the fp32 normal range
    k = np.float32(2.0 ** e)
    sb_k, codes_k, s_k = A.quantize_blocks(v * k, s_T * k, rounding)
    assert np.array_equal(sb, sb_k) and np.array_equal(codes, codes_k) and np.array_equal(s * k, s_k)
    # a dequantized block quantizes to itself when its scale byte is kept by the rounding (grid values are fixed points)
    deq = (F.e2m1_decode(codes) * s.astype(np.float64)[..., None]).astype(np.float32)
    if sb[0] > 0 and np.abs(deq).max() * 6 >= 6 * s[0] * 4:      # the block maximum still sits in the top binade
        sb2, codes2, _ = A.quantize_blocks(deq, s_T, rounding)
        if sb2[0] == sb[0]:
            assert np.array_equal(codes2 & 7, codes & 7)


@settings(max_examples=100, deadline=None, derandomize=True)
@given(st.integers(min_value=1, max_value=40), st.integers(min_value=0, max_value=40))
def test_interleaved_order_is_a_permutation_with_adjacent_partners(nb, no):
    no = min(no, nb)
    for mod, G in ((A, 16), (MX, 32)):
        o = mod.interleaved_order(nb * G, no * G)
        assert sorted(o.tolist()) == list(range(nb + no))
        assert o[: nb - no].tolist() == list(range(nb - no))
        for i in range(no):
            assert o[nb - no + 2 * i] == nb - no + i and o[nb - no + 2 * i + 1] == nb + i


@settings(max_examples=150, deadline=None, derandomize=True)
@given(st.lists(fp16_vals, min_size=32, max_size=32), st.sampled_from(["nearest", "up"]))
def test_mx_block_recipe_symmetry_and_exact_residual(vals, rounding):
    v = np.array(vals, dtype=np.float16).astype(np.float32)[None, :]
    sb, codes, X = MX.quantize_blocks(v, rounding)
    sb_n, codes_n, _ = MX.quantize_blocks(-v, rounding)
    assert np.array_equal(sb, sb_n) and np.array_equal(codes ^ 8, codes_n)
    r = MX.residual_blocks(v, codes, X)
    assert np.array_equal(r.astype(np.float64) + F.e2m1_decode(codes) * X[:, None], v.astype(np.float64))
    # doubling every value raises the scale byte by one and keeps the codes
    if np.abs(v).max() < 30000 and np.abs(v).max() > 0:
        sb2, codes2, _ = MX.quantize_blocks(v * np.float32(2), rounding)
        assert np.array_equal(sb2, sb + 1) and np.array_equal(codes2, codes)
