"""Pins for the two variants of the quantizer in oracle.arcquant: the interleaved channel layout
(Appendix D) and the block scale rounded up (the alpha >= 1 of Section 3.4)."""
from fractions import Fraction as Fr

import numpy as np
import pytest

from oracle import arcquant as A
from oracle import brute
from oracle import formats as F
from paper_2601_07475_amd import workloads as wk

from test_oracle_formats import golden
from test_oracle_arcquant import small_case, unpack_by_hand


# ---- scale rounded up -------------------------------------------------------------------
def test_e4m3_round_up_against_loop_over_all_values():
    vals = F.e4m3_decode(np.arange(0x7F))
    pts = [0.0, 2.0 ** -12, 2.0 ** -9, 447.9, 448.0, 449.0, 1e6]
    for b in range(0x7E):
        lo, hi = float(vals[b]), float(vals[b + 1])
        pts += [lo, np.nextafter(np.float32(lo), np.float32(np.inf)), 0.5 * (lo + hi),
                np.nextafter(np.float32(hi), np.float32(0))]
    rng = np.random.default_rng(3)
    pts += list(np.exp(rng.uniform(np.log(2.0 ** -11), np.log(500.0), 400)).astype(np.float32))
    u = np.array(pts, dtype=np.float32)
    got = F.e4m3_encode_up_sat(u)
    for x, g in zip(u, got):
        assert int(g) == brute.e4m3_up_sat(Fr(float(x))), float(x)
    # on a grid value both roundings agree; elsewhere up is the nearest one or the one above it
    near = F.e4m3_encode_rne_sat(u).astype(int)
    d = got.astype(int) - near
    assert set(d.tolist()) <= {0, 1}
    assert np.all(d[np.isin(u.astype(np.float64), vals)] == 0)
    # never below u (short of saturation), and the value before it is below u
    ok = u <= 448
    assert np.all(vals[got[ok]] >= u[ok].astype(np.float64))
    pos = ok & (got > 0)
    assert np.all(vals[got[pos] - 1] < u[pos].astype(np.float64))
    assert np.all(got[~ok] == 0x7E)


def test_round_up_block_recipe_against_exact_rational_brute_force():
    rng = np.random.default_rng(12)
    blocks = []
    for _ in range(40):
        b = rng.standard_normal(16).astype(np.float16)
        b[rng.integers(16)] *= np.float16(rng.choice([1, 30, 100]))
        blocks.append(b)
    sub = np.arange(1, 17, dtype=np.uint16).view(np.float16)
    blocks += [sub, np.zeros(16, np.float16), np.full(16, 60000, np.float16),
               np.float16([0.25 * i for i in range(16)])]
    V = np.stack(blocks).astype(np.float32)
    for s_T in (np.float32(1.0), np.float32(0.0123), np.float32(60000 / 2688.0), np.float32(2.0 ** -20)):
        sb, codes, s = A.quantize_blocks(V, s_T, "up")
        r = A.residual_blocks(V, codes, s)
        sb2, codes2, _ = A.quantize_blocks(r, s_T, "up")
        for i in range(len(V)):
            bsb, bcodes, bres = brute.quantize_block([float(x) for x in V[i]], float(s_T), scale_up=True)
            assert bsb == sb[i] and bcodes == codes[i].tolist(), (i, s_T)
            assert [float(x) for x in bres] == r[i].astype(np.float64).tolist()
            bsb2, bcodes2, _ = brute.quantize_block(bres, float(s_T), scale_up=True)
            assert bsb2 == sb2[i] and bcodes2 == codes2[i].tolist()


def test_round_up_meets_the_assumptions_of_the_error_analysis():
    """Section 3.4: alpha = s / (max / q_max) lies in [1, 1.125] and the bounds |e| <= alpha M eps4,
    |e_arc| <= alpha1 alpha2 M eps8 follow; with the scale rounded up the premise holds block by block
    (up to the one fp32 rounding of u, and away from scale underflow), which nearest rounding does not give."""
    g = golden()
    c = wk.make_case(wk.shrink(wk.WORKLOADS["c2_llama8b_q"], M=64, N=8))
    K, S, sT = c["wl"].K, c["S"], c["sT_x"]
    Xp = c["X"][:, c["perm"]].astype(np.float64)
    pc, ps = A.quantize_act(c["X"], c["perm"], S, sT, scale_rounding="up")
    pc_n, ps_n = A.quantize_act(c["X"], c["perm"], S, sT)
    deq = A.dequantize(pc, ps, sT)
    prim, res = deq[:, :K], deq[:, K:]
    s_blk = F.e4m3_decode(ps) * np.float64(sT)
    amax_blk = np.abs(Xp).reshape(-1, K // 16, 16).max(-1)
    normal = ps[:, :K // 16] >= 8                                # scale in E4M3's normal range
    alpha = s_blk[:, :K // 16][normal] / (amax_blk[normal] / 6)
    assert alpha.min() >= 1 - 2.0 ** -22 and alpha.max() <= 1.125 * (1 + 2.0 ** -22)
    assert alpha.max() > 1.11 and alpha.min() < 1.001            # the range is used, not vacuous
    alpha_n = (F.e4m3_decode(ps_n) * np.float64(sT))[:, :K // 16][normal] / (amax_blk[normal] / 6)
    assert alpha_n.min() < 0.95                                  # nearest rounding does go below 1
    # no element is clipped at 6 (beyond the fp32 rounding of u): the block maximum quantizes to code 7
    # with error at most half the top step
    s_el = np.repeat(s_blk[:, :K // 16], 16, axis=1)
    w = np.abs(Xp) / np.where(s_el > 0, s_el, 1)
    assert w[np.repeat(normal, 16, axis=1)].max() <= 6 * (1 + 2.0 ** -22)
    assert (np.abs(Xp) / np.where(s_el > 0, np.repeat(F.e4m3_decode(ps_n)[:, :K // 16] * np.float64(sT), 16, axis=1), 1)).max() > 6.2
    # the bounds
    err = np.abs(Xp - prim)
    amax = np.repeat(amax_blk, 16, axis=1)
    floor = 6 * 2.0 ** -9 * np.float64(sT)                       # blocks whose scale is a subnormal of E4M3
    assert np.all(err <= 1.125 * amax * g["eps4"] + floor)
    h = np.where(w <= 2, 0.25, np.where(w <= 4, 0.5, 1.0))
    assert np.all(err <= h * s_el * (1 + 2.0 ** -20))
    err2 = np.abs(Xp[:, K - S:] - prim[:, K - S:] - res)
    assert np.all(err2 <= g["sup_alpha1_alpha2"] * g["eps8"] * amax[:, K - S:] + floor)
    # a scale byte of the variant is the nearest one or the next
    d = ps.astype(int) - ps_n.astype(int)
    assert set(np.unique(d[:, :K // 16]).tolist()) == {0, 1}
    # tiny but nonzero blocks keep a nonzero scale
    tiny = np.full((1, 16), 2.0 ** -24, dtype=np.float16)
    sb_up, codes_up, _ = A.quantize_blocks(tiny.astype(np.float32), np.float32(1.0), "up")
    sb_ne, _, _ = A.quantize_blocks(tiny.astype(np.float32), np.float32(1.0))
    assert sb_up.tolist() == [1] and sb_ne.tolist() == [0]
    assert A.quantize_blocks(np.zeros((1, 16), np.float32), np.float32(1.0), "up")[0].tolist() == [0]


# ---- interleaved layout -----------------------------------------------------------------
def test_interleaved_order_worked_examples():
    # K = 32, S = 32: both blocks are outliers -> p0 r0 p1 r1 (concatenated numbering: 0 2 1 3)
    assert A.interleaved_order(32, 32).tolist() == [0, 2, 1, 3]
    # K = 64, S = 32: two plain blocks, then p2 r2 p3 r3
    assert A.interleaved_order(64, 32).tolist() == [0, 1, 2, 4, 3, 5]
    assert A.interleaved_order(48, 0).tolist() == [0, 1, 2]
    for K, S in ((256, 48), (512, 512), (1024, 16)):
        o = A.interleaved_order(K, S)
        assert sorted(o.tolist()) == list(range((K + S) // 16))


def test_interleaved_layout_is_a_block_permutation_of_the_concatenated_one():
    c = small_case(M=9, K=256, N=12, S=48)
    X, W, perm, S = c["X"], c["W"], c["perm"], c["S"]
    K = X.shape[1]
    nb, no = K // 16, S // 16
    for rounding in ("nearest", "up"):
        cc, cs = A.quantize_act(X, perm, S, c["sT_x"], scale_rounding=rounding)
        ic, isc = A.quantize_act(X, perm, S, c["sT_x"], layout="interleaved", scale_rounding=rounding)
        wc, wsc = A.pack_weight(W, perm, S, c["sT_w"], scale_rounding=rounding)
        iwc, iwsc = A.pack_weight(W, perm, S, c["sT_w"], layout="interleaved", scale_rounding=rounding)
        for (pc, ps, qc, qs) in ((cc, cs, ic, isc), (wc, wsc, iwc, iwsc)):
            assert qc.shape == pc.shape and qs.shape == ps.shape
            # explicit walk: plain blocks in place, then primary block and its partner side by side
            for b in range(nb - no):
                assert np.array_equal(qc[:, 8 * b:8 * b + 8], pc[:, 8 * b:8 * b + 8])
                assert np.array_equal(qs[:, b], ps[:, b])
            for i in range(no):
                p_src, r_src = nb - no + i, nb + i
                p_dst, r_dst = nb - no + 2 * i, nb - no + 2 * i + 1
                assert np.array_equal(qc[:, 8 * p_dst:8 * p_dst + 8], pc[:, 8 * p_src:8 * p_src + 8])
                assert np.array_equal(qc[:, 8 * r_dst:8 * r_dst + 8], pc[:, 8 * r_src:8 * r_src + 8])
                assert np.array_equal(qs[:, p_dst], ps[:, p_src]) and np.array_equal(qs[:, r_dst], ps[:, r_src])
        # weights: the partner of an outlier block is its verbatim copy, right behind it
        for i in range(no):
            p_dst = nb - no + 2 * i
            assert np.array_equal(iwc[:, 8 * p_dst:8 * p_dst + 8], iwc[:, 8 * p_dst + 8:8 * p_dst + 16])
            assert np.array_equal(iwsc[:, p_dst], iwsc[:, p_dst + 1])
        # the product does not see the order of the reduction axis (Appendix D: the standard GEMM
        # yields the same result): fp64 sums in another order
        Yc = A.gemm(cc, cs, c["sT_x"], wc, wsc, c["sT_w"])
        Yi = A.gemm(ic, isc, c["sT_x"], iwc, iwsc, c["sT_w"])
        assert np.allclose(Yc, Yi, rtol=0, atol=1e-12 * np.abs(Yc).max())
        # and exactly so in rational arithmetic, on a corner of it
        ua, uw = unpack_by_hand(ic[:2]), unpack_by_hand(iwc[:3])
        Yb = brute.gemm_loops(ua.tolist(), isc[:2].tolist(), float(c["sT_x"]), uw.tolist(), iwsc[:3].tolist(), float(c["sT_w"]))
        ua, uw = unpack_by_hand(cc[:2]), unpack_by_hand(wc[:3])
        Yb2 = brute.gemm_loops(ua.tolist(), cs[:2].tolist(), float(c["sT_x"]), uw.tolist(), wsc[:3].tolist(), float(c["sT_w"]))
        assert Yb == Yb2
    # mismatched layouts of the two operands do change the product: the layout is part of the contract
    Ybad = A.gemm(ic, isc, c["sT_x"], wc, wsc, c["sT_w"])
    assert not np.allclose(Ybad, Yc, rtol=1e-3, atol=1e-3 * np.abs(Yc).max())


def test_variants_reject_unknown_names_and_S0_is_unchanged():
    c = small_case(M=3, K=64, N=4, S=0)
    with pytest.raises(ValueError):
        A.quantize_act(c["X"], c["perm"], 0, c["sT_x"], layout="blocked")
    with pytest.raises(ValueError):
        A.quantize_act(c["X"], c["perm"], 0, c["sT_x"], scale_rounding="down")
    a = A.quantize_act(c["X"], c["perm"], 0, c["sT_x"])
    b = A.quantize_act(c["X"], c["perm"], 0, c["sT_x"], layout="interleaved")
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


# ---- the same two variants on MXFP4 -----------------------------------------------------
def test_mx_round_up_is_the_smallest_power_of_two_without_clipping():
    from oracle import mxfp4 as MX
    rng = np.random.default_rng(6)
    v = (rng.standard_normal((400, 32)) * np.exp(rng.standard_normal((400, 1)) * 3)).astype(np.float16)
    v[0] = 0
    v[1] = np.float16(2.0 ** -24)
    v[2, :] = np.float16(6.0)            # exactly 1.5 * 2^2: the floor rule already holds it
    v[3, :] = np.float16(6.004)          # just above
    v[4] = np.float16(65504.0)
    v = v.astype(np.float32)
    sb, codes, X = MX.quantize_blocks(v, "up")
    sb_f, _, X_f = MX.quantize_blocks(v)
    # the defining inequalities, in exact rationals, block by block
    for i in range(len(v)):
        amax = max(Fr(float(t)) for t in np.abs(v[i]))
        Xi = Fr(2) ** (int(sb[i]) - 127)
        if amax == 0:
            assert sb[i] == 127
            continue
        assert amax <= 6 * Xi and amax > 3 * Xi               # X / 2 would clip
        for t, c in zip(v[i], codes[i]):
            assert (c & 7) == brute.e2m1_nearest(abs(Fr(float(t))) / Xi) and (c >> 3) == int(np.signbit(t))
    assert sb[2] == sb_f[2] and sb[3] == sb_f[3] + 1
    d = sb.astype(int) - sb_f.astype(int)
    assert set(d.tolist()) == {0, 1} and 0.2 < d.mean() < 0.8
    # nothing clips: every element is within half a grid step
    deq = F.e2m1_decode(codes) * X[:, None]
    step = np.where(np.abs(deq) >= 4 * X[:, None], 2.0, np.where(np.abs(deq) >= 2 * X[:, None], 1.0, 0.5)) * X[:, None]
    assert np.all(np.abs(v - deq) <= step / 2)
    # the largest error of a block is at most amax / 6 (alpha <= 2: X < amax / 3), i.e. half the top step
    amax = np.abs(v).max(axis=1)
    assert np.all(np.abs(v - deq).max(axis=1) <= X)


def test_mx_interleaved_layout_is_a_block_permutation():
    from oracle import mxfp4 as MX
    assert MX.interleaved_order(64, 64).tolist() == [0, 2, 1, 3]
    assert MX.interleaved_order(128, 64).tolist() == [0, 1, 2, 4, 3, 5]
    wl = wk.Workload("t", 10, 256, 12, 96, 5, "const50", 0.02, 4)
    c = wk.make_case(wl)
    X, W, perm, S = c["X"], c["W"], c["perm"], 96
    nb, no = 256 // 32, 96 // 32
    for rounding in ("nearest", "up"):
        cc, cs = MX.quantize_act(X, perm, S, scale_rounding=rounding)
        ic, isc = MX.quantize_act(X, perm, S, layout="interleaved", scale_rounding=rounding)
        wc, wsc = MX.pack_weight(W, perm, S, scale_rounding=rounding)
        iwc, iwsc = MX.pack_weight(W, perm, S, layout="interleaved", scale_rounding=rounding)
        for (pc, ps, qc, qs) in ((cc, cs, ic, isc), (wc, wsc, iwc, iwsc)):
            for b in range(nb - no):
                assert np.array_equal(qc[:, 16 * b:16 * b + 16], pc[:, 16 * b:16 * b + 16]) and np.array_equal(qs[:, b], ps[:, b])
            for i in range(no):
                for src, dst in ((nb - no + i, nb - no + 2 * i), (nb + i, nb - no + 2 * i + 1)):
                    assert np.array_equal(qc[:, 16 * dst:16 * dst + 16], pc[:, 16 * src:16 * src + 16])
                    assert np.array_equal(qs[:, dst], ps[:, src])
        Yc, Yi = MX.gemm(cc, cs, wc, wsc), MX.gemm(ic, isc, iwc, iwsc)
        assert np.allclose(Yc, Yi, rtol=0, atol=1e-12 * np.abs(Yc).max())
    with pytest.raises(ValueError):
        MX.quantize_act(X, perm, S, layout="x")
    with pytest.raises(ValueError):
        MX.quantize_act(X, perm, S, scale_rounding="x")
