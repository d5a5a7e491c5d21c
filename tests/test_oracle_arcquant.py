"""Pins for oracle.arcquant: round trips, the paper's error bounds, S = 0, the eq. (2)
identity, residual benefit, layout, brute force with exact rationals, loop GEMM."""
import numpy as np
import pytest

from oracle import arcquant as A
from oracle import brute
from oracle import formats as F
from paper_2601_07475_amd import workloads as wk

from test_oracle_formats import golden

C1 = wk.WORKLOADS["c1_tiny"]


def small_case(M=24, K=256, N=40, S=48, seed=7, n_outlier=6):
    wl = wk.Workload("t", M, K, N, S, n_outlier, "loguniform20_100", 0.02, seed)
    return wk.make_case(wl)


def unpack_by_hand(packed):
    """byte i -> element 2i in bits 0-3, element 2i+1 in bits 4-7 (written independently)."""
    rows, nb = packed.shape
    out = np.zeros((rows, 2 * nb), dtype=np.uint8)
    for i in range(2 * nb):
        out[:, i] = (packed[:, i // 2] >> (4 * (i % 2))) & 0xF
    return out


# ---- P1: grid values round-trip exactly -----------------------------------------------
def test_grid_values_roundtrip_every_scale_byte():
    codes = np.arange(16)
    gvals = F.e2m1_decode(codes)
    for s_T in (1.0, 2.0 ** -7, 2.0 ** 5):
        for sb in range(1, 0x7F):
            sv = F.e4m3_decode(sb)
            v = (gvals * sv * s_T).astype(np.float32)
            assert np.array_equal(v.astype(np.float64), gvals * sv * s_T)      # representable
            got_sb, got_codes, s = A.quantize_blocks(v[None, :], np.float32(s_T))
            assert got_sb[0] == sb
            assert got_codes[0].tolist() == codes.tolist()                     # incl. -0 -> code 8
            assert s[0] == np.float32(sv * s_T)
    # and through the full packed path on fp16-representable inputs
    X = (gvals * 0.375 * 2.0 ** -3)[None, :].astype(np.float16)
    pc, ps = A.quantize_act(X, np.arange(16), 0, np.float32(2.0 ** -3))
    assert ps.tolist() == [[int(F.e4m3_encode_rne_sat(0.375))]]
    assert unpack_by_hand(pc)[0].tolist() == list(range(16))
    assert np.array_equal(A.dequantize(pc, ps, np.float32(2.0 ** -3)), X.astype(np.float64))


# ---- P4: error bounds ------------------------------------------------------------------
def test_error_bounds_single_and_dual_stage():
    g = golden()
    c = wk.make_case(wk.shrink(wk.WORKLOADS["c2_llama8b_q"], M=64, N=8))
    K, S, sT = c["wl"].K, c["S"], c["sT_x"]
    Xp = c["X"][:, c["perm"]].astype(np.float64)
    pc, ps = A.quantize_act(c["X"], c["perm"], S, sT)
    deq = A.dequantize(pc, ps, sT)
    prim, res = deq[:, :K], deq[:, K:]
    s = np.repeat(F.e4m3_decode(ps) * np.float64(sT), 16, axis=1)
    err = np.abs(Xp - prim)
    # half a grid step times the block scale, by magnitude range of the quantized value
    w = np.abs(Xp) / np.where(s[:, :K] > 0, s[:, :K], 1)
    h = np.where(w <= 2, 0.25, np.where(w <= 4, 0.5, 1.0))
    tol = 1 + 2.0 ** -20
    assert np.all(err <= h * s[:, :K] * tol)
    # single stage relative to the block maximum: <= (1.0625/6) amax with a nearest-even scale,
    # inside the paper's alpha*M*eps4 with alpha <= 1.125  (Section 3.4)
    amax = np.repeat(np.abs(Xp).reshape(-1, K // 16, 16).max(-1), 16, axis=1)
    floor = 6 * 2.0 ** -10 * np.float64(sT)                # block-scale underflow
    assert np.all(err <= (1.0625 / 6) * amax * tol + floor)
    assert np.all(err <= 1.125 * amax * g["eps4"])
    assert (err / np.maximum(amax, 1e-30)).max() > 0.12         # the bound is nearly met, not vacuous
    # dual stage on the outlier channels: paper's B_arc = alpha1 alpha2 M eps8  (Section 3.4 eq. (4))
    err2 = np.abs(Xp[:, K - S:] - prim[:, K - S:] - res)
    amax_o = amax[:, K - S:]
    assert np.all(err2 <= g["sup_alpha1_alpha2"] * g["eps8"] * amax_o + floor)
    assert np.all(err2 <= (1.0625 / 6) ** 2 * amax_o * tol + floor)
    assert g["eps4"] ** 2 == g["eps8"]


# ---- P5: S = 0 is plain NVFP4 ------------------------------------------------------------
def test_S0_is_plain_block_quantization_and_primary_part_is_unchanged():
    c = small_case()
    X, perm, sT = c["X"], c["perm"], c["sT_x"]
    M, K = X.shape
    pc0, ps0 = A.quantize_act(X, perm, 0, sT)
    assert pc0.shape == (M, K // 2) and ps0.shape == (M, K // 16)
    sb, codes, _ = A.quantize_blocks(X[:, perm].astype(np.float32).reshape(M, K // 16, 16), sT)
    assert np.array_equal(ps0, sb)
    assert np.array_equal(unpack_by_hand(pc0), codes.reshape(M, K))
    pc, ps = A.quantize_act(X, perm, c["S"], sT)
    assert pc.shape == (M, (K + c["S"]) // 2) and ps.shape == (M, (K + c["S"]) // 16)
    assert np.array_equal(pc[:, :K // 2], pc0) and np.array_equal(ps[:, :K // 16], ps0)
    wc0, ws0 = A.pack_weight(c["W"], perm, 0, c["sT_w"])
    Y0 = A.gemm(pc0, ps0, sT, wc0, ws0, c["sT_w"])
    plain = A.dequantize(pc0, ps0, sT) @ A.dequantize(wc0, ws0, c["sT_w"]).T
    assert np.array_equal(Y0, plain)


# ---- P6: eq. (2) identity ----------------------------------------------------------------
def test_augmented_product_equals_explicit_two_term_sum():
    c = small_case(M=20, K=320, N=36, S=64)
    X, W, perm, S, sTx, sTw = c["X"], c["W"], c["perm"], c["S"], c["sT_x"], c["sT_w"]
    M, K = X.shape
    pc, ps = A.quantize_act(X, perm, S, sTx)
    wc, ws = A.pack_weight(W, perm, S, sTw)
    Y = A.gemm(pc, ps, sTx, wc, ws, sTw)
    # the two terms, each built separately from its own quantization
    Xp = X[:, perm].astype(np.float32).reshape(M, K // 16, 16)
    sbx, cx, sx = A.quantize_blocks(Xp, sTx)
    # dequantized value = grid value * E4M3 byte value * tensor scale, all exact in fp64
    # (the fp32-rounded block scale s is what the quantizer divides by; it differs by <= 2^-24)
    def deq(c, sb, sT):
        return (F.e2m1_decode(c) * (F.e4m3_decode(sb) * np.float64(sT))[..., None]).reshape(c.shape[0], -1)
    QX = deq(cx, sbx, sTx)
    assert np.allclose(QX, (F.e2m1_decode(cx) * sx.astype(np.float64)[..., None]).reshape(M, K), rtol=2.0 ** -23, atol=0)
    o = (K - S) // 16
    R = A.residual_blocks(Xp[:, o:], cx[:, o:], sx[:, o:])
    assert np.allclose(R.reshape(M, S), Xp.astype(np.float64).reshape(M, K)[:, K - S:] - QX[:, K - S:],
                       rtol=0, atol=2.0 ** -20 * np.abs(Xp).max())
    sbr, cr, sr = A.quantize_blocks(R, sTx)
    QR = deq(cr, sbr, sTx)
    Wp = W[:, perm].astype(np.float32).reshape(-1, K // 16, 16)
    sbw, cw, sw = A.quantize_blocks(Wp, sTw)
    QW = deq(cw, sbw, sTw)
    two_terms = QX @ QW.T + QR @ QW[:, K - S:].T
    assert np.allclose(Y, two_terms, rtol=1e-12, atol=1e-12 * np.abs(two_terms).max())
    # weight augmentation is a verbatim copy of the outlier blocks (codes and scale bytes)
    assert np.array_equal(wc[:, K // 2:], wc[:, (K - S) // 2:K // 2])
    assert np.array_equal(ws[:, K // 16:], ws[:, (K - S) // 16:K // 16])
    # residual scale bytes sit after the K/16 primary ones, in outlier-block order
    assert np.array_equal(ps[:, K // 16:], sbr)


# ---- P7: the residual channels help --------------------------------------------------------
def test_residual_reduces_error():
    c = wk.make_case(C1)
    X, W, perm, S, sTx, sTw = c["X"], c["W"], c["perm"], c["S"], c["sT_x"], c["sT_w"]
    K = X.shape[1]
    pc, ps = A.quantize_act(X, perm, S, sTx)
    deq = A.dequantize(pc, ps, sTx)
    Xo = X[:, perm].astype(np.float64)[:, K - S:]
    e1 = (Xo - deq[:, K - S:K]).reshape(-1, 16)
    e2 = (Xo - deq[:, K - S:K] - deq[:, K:]).reshape(-1, 16)
    n1, n2 = np.linalg.norm(e1, axis=1), np.linalg.norm(e2, axis=1)
    assert np.all(n2[n1 > 0] < n1[n1 > 0])
    assert n2.sum() < 0.3 * n1.sum()
    wc, ws = A.pack_weight(W, perm, S, sTw)
    pc0, ps0 = A.quantize_act(X, perm, 0, sTx)
    wc0, ws0 = A.pack_weight(W, perm, 0, sTw)
    target = X.astype(np.float64) @ A.dequantize(wc0, ws0, sTw)[:, np.argsort(perm)].T    # X deq(W)^T
    Y = A.gemm(pc, ps, sTx, wc, ws, sTw)
    Y0 = A.gemm(pc0, ps0, sTx, wc0, ws0, sTw)
    assert np.linalg.norm(Y - target) < 0.8 * np.linalg.norm(Y0 - target)


# ---- P8: permutation convention --------------------------------------------------------------
def test_calibration_permutation_convention():
    c = wk.make_case(C1)
    X, perm, S = c["X"], c["perm"], c["S"]
    K = X.shape[1]
    assert sorted(perm.tolist()) == list(range(K)) and perm.dtype == np.int32
    colmax = np.abs(X).max(axis=0).astype(np.float64)
    assert np.all(np.diff(colmax[perm]) >= 0)                   # ascending: outliers last
    assert colmax[perm[K - S:]].min() >= colmax[perm[:K - S]].max()
    inv = np.empty(K, dtype=np.int64)
    inv[perm] = np.arange(K)
    assert np.array_equal(X[:, perm][:, inv], X)
    T = np.zeros((2, 32), dtype=np.float16)
    T[0] = [3, 1, 3, 2] * 8                                     # deliberate ties
    want = [i for v in (1, 2, 3) for i in range(32) if T[0, i] == v]
    assert wk.calibrate_perm(T).tolist() == want                # the harness's stand-in
    from oracle import calibration as CAL                        # and the oracle's calibration step (Section 3.2)
    sel = CAL.select_outliers(CAL.absmax_update(np.zeros(32, np.float32), T))
    assert sel["perm"].tolist() == want
    full = CAL.select_outliers(CAL.absmax_update(np.zeros(K, np.float32), X))
    assert np.array_equal(full["perm"], perm)
    cm = np.abs(X).max(axis=0).astype(np.float32)
    assert cm[full["perm"][K - full["S_raw"]:]].min() > full["tau"] >= cm[full["perm"][:K - full["S_raw"]]].max()
    # the quantizer gathers: reordered position j reads source channel perm[j]
    Xq = np.zeros((1, 32), dtype=np.float16)
    Xq[0, 5] = 6.0
    perm2 = np.roll(np.arange(32), 3)                            # perm2[8] == 5
    pc, ps = A.quantize_act(Xq, perm2, 0, np.float32(1.0))
    un = unpack_by_hand(pc)[0]
    assert perm2[8] == 5 and un[8] == 7 and un.sum() == 7


# ---- P2 / R5: brute force with exact rationals over whole blocks ------------------------------
def test_block_recipe_against_exact_rational_brute_force():
    rng = np.random.default_rng(11)
    blocks = []
    for _ in range(60):
        b = rng.standard_normal(16).astype(np.float16)
        b[rng.integers(16)] *= np.float16(rng.choice([1, 30, 100]))
        blocks.append(b)
    sub = np.arange(1, 17, dtype=np.uint16).view(np.float16)                    # fp16 subnormals
    blocks += [sub, sub * np.float16(-1), np.zeros(16, np.float16),
               np.full(16, 60000, np.float16), np.float16([0.25 * i for i in range(16)])]
    V = np.stack(blocks).astype(np.float32)
    for s_T in (np.float32(1.0), np.float32(0.0123), np.float32(60000 / 2688.0), np.float32(2.0 ** -20)):
        sb, codes, s = A.quantize_blocks(V, s_T)
        r = A.residual_blocks(V, codes, s)
        sb2, codes2, _ = A.quantize_blocks(r, s_T)
        for i in range(len(V)):
            bsb, bcodes, bres = brute.quantize_block([float(x) for x in V[i]], float(s_T))
            assert bsb == sb[i] and bcodes == codes[i].tolist(), (i, s_T)
            assert [float(x) for x in bres] == r[i].astype(np.float64).tolist()
            bsb2, bcodes2, _ = brute.quantize_block(bres, float(s_T))
            assert bsb2 == sb2[i]
            # sign of an exactly-zero residual is +0 in both; elsewhere codes must agree bit for bit
            assert bcodes2 == codes2[i].tolist()


def test_reciprocal_recipe_rarely_departs_from_real_division():
    c = wk.make_case(wk.shrink(wk.WORKLOADS["c2_llama8b_q"], M=2, N=8))
    X, sT = c["X"][:, c["perm"]].astype(np.float32), c["sT_x"]
    blocks = X.reshape(-1, 16)[:300]
    sb, codes, _ = A.quantize_blocks(blocks, sT)
    diff = 0
    for i in range(len(blocks)):
        rsb, rcodes = brute.quantize_block_real([float(x) for x in blocks[i]], float(sT))
        assert rsb == sb[i]
        diff += sum(a != b for a, b in zip(rcodes, codes[i].tolist()))
    assert diff <= 2          # a few per million expected; eq. (1) in real numbers otherwise reproduced


# ---- signs of zero, zero blocks, saturation -----------------------------------------------------
def test_zero_sign_underflow_and_saturation():
    v = np.zeros((1, 16), np.float32)
    v[0, 3] = -0.0
    sb, codes, s = A.quantize_blocks(v, np.float32(1.0))
    assert sb[0] == 0 and s[0] == 0 and codes[0].tolist() == [0, 0, 0, 8] + [0] * 12
    # block whose scale underflows E4M3: amax/(6 s_T) <= 2^-10 rounds to byte 0
    v = np.full((1, 16), -2.0 ** -10 * 6, np.float32)
    sb, codes, s = A.quantize_blocks(v, np.float32(1.0))
    assert sb[0] == 0 and np.all(codes == 8)
    # negative value that rounds to magnitude 0 keeps its sign bit
    v = np.float32([[6.0, -0.2] + [0.0] * 14])
    _, codes, _ = A.quantize_blocks(v, np.float32(1.0))
    assert codes[0, :2].tolist() == [7, 8]
    # tensor scale too small for the data: scale byte saturates at 448, elements at 6
    v = np.float32([[6.0 * 448 * 4, -6.0 * 448 * 4, 448.0 * 3] + [0.0] * 13])
    sb, codes, s = A.quantize_blocks(v, np.float32(1.0))
    assert sb[0] == 0x7E and codes[0, :3].tolist() == [7, 15, 5]
    # a nearest-even scale can round below amax/6, so the block maximum itself may exceed 6 and saturate
    v = np.float32([[6.375 * 1.0] + [0.0] * 15])             # u = 1.0625 -> ties to 1.0
    sb, codes, s = A.quantize_blocks(v, np.float32(1.0))
    assert F.e4m3_decode(sb[0]) == 1.0 and codes[0, 0] == 7
    for bad in (0.0, -1.0, np.inf, np.nan):
        with pytest.raises(ValueError):
            A.quantize_blocks(v, np.float32(bad))
    with pytest.raises(ValueError):
        A.quantize_blocks(np.float32([[np.inf] + [0.0] * 15]), np.float32(1.0))
    for K, S in ((24, 0), (32, 8), (32, 48), (32, -16)):
        with pytest.raises(ValueError):
            A.quantize_act(np.zeros((1, K), np.float16), np.arange(K), S, np.float32(1.0))


# ---- P9: loop GEMM with exact rationals -----------------------------------------------------------
def test_gemm_against_triple_loop():
    c = small_case(M=5, K=48, N=7, S=16, n_outlier=3)
    pc, ps = A.quantize_act(c["X"], c["perm"], c["S"], c["sT_x"])
    wc, ws = A.pack_weight(c["W"], c["perm"], c["S"], c["sT_w"])
    Y = A.gemm(pc, ps, c["sT_x"], wc, ws, c["sT_w"])
    assert Y.shape == (5, 7)
    Yb = brute.gemm_loops(unpack_by_hand(pc).tolist(), ps.tolist(), float(c["sT_x"]),
                          unpack_by_hand(wc).tolist(), ws.tolist(), float(c["sT_w"]))
    Yb = np.array([[float(v) for v in row] for row in Yb])
    assert np.allclose(Y, Yb, rtol=1e-13, atol=1e-13 * np.abs(Yb).max())
    rows = np.array([4, 1])
    assert np.allclose(A.gemm_rows(pc, ps, c["sT_x"], wc, ws, c["sT_w"], rows), Y[rows], rtol=1e-13, atol=1e-13)


def test_all_workloads_have_valid_shapes():
    for wl in wk.WORKLOADS.values():
        assert wl.K % 16 == 0 and wl.S % 16 == 0 and 0 < wl.S <= wl.K and wl.n_outlier < wl.S


# ---- RMSNorm in front of the quantizer (Section 3.3 fused kernel) ---------------------------------
def _norm_inputs(M=6, K=96, seed=21):
    rng = np.random.default_rng(seed)
    X = (rng.standard_normal((M, K)) * rng.uniform(0.05, 30, (M, 1))).astype(np.float16)
    X[:, 5] *= np.float16(40)
    gamma = (1 + 0.3 * rng.standard_normal(K)).astype(np.float16)
    return X, gamma


def test_rmsnorm_against_plain_torch_reference():
    import torch
    X, gamma = _norm_inputs(M=64, K=512)
    eps = 1e-5
    y = A.rmsnorm(X, gamma, eps)
    # the usual reference layer, written with library primitives (fp32 statistics, cast, then weight)
    xt = torch.from_numpy(X)
    var = xt.float().pow(2).mean(-1, keepdim=True)
    ref = (torch.from_numpy(gamma) * (xt.float() * torch.rsqrt(var + eps)).to(torch.float16)).numpy()
    # fp32 accumulation order and rsqrt rounding may move a value by one fp16 step, rarely
    same = (y == ref)
    assert same.mean() > 0.995
    ulp = np.abs(y.view(np.int16).astype(np.int32) - ref.view(np.int16).astype(np.int32))
    assert ulp.max() <= 1


def test_rmsnorm_closed_forms_and_invariants():
    K = 64
    gamma = np.ones(K, np.float16)
    # constant row: every entry becomes sign(c) (rms = |c|)
    for c in (0.5, -3.0, 120.0):
        y = A.rmsnorm(np.full((1, K), c, np.float16), gamma, 0.0)
        assert np.all(y == np.float16(np.sign(c)))
    # scaling a row by a power of two changes nothing when eps = 0 (every step scales exactly)
    X, g2 = _norm_inputs(M=8, K=K)
    X = (X / 64).astype(np.float16)                      # keep 4x inside the fp16 range, away from subnormals
    assert np.array_equal(A.rmsnorm(X, g2, 0.0), A.rmsnorm((X * np.float16(4)).astype(np.float16), g2, 0.0))
    # unit root-mean-square after normalisation (gamma = 1), up to fp16 rounding
    y = A.rmsnorm(X, gamma, 0.0).astype(np.float64)
    assert np.allclose(np.sqrt((y * y).mean(axis=1)), 1.0, rtol=2e-3)
    # gamma enters as a per-channel factor applied after the cast
    y1 = A.rmsnorm(X, gamma, 1e-6)
    yg = A.rmsnorm(X, g2, 1e-6)
    assert np.array_equal(yg, (y1.astype(np.float32) * g2.astype(np.float32)).astype(np.float16))
    # a large eps shrinks the output; zero row stays zero
    assert np.all(np.abs(A.rmsnorm(X, gamma, 100.0).astype(np.float32)) <= np.abs(y1.astype(np.float32)))
    assert np.all(A.rmsnorm(np.zeros((1, K), np.float16), gamma, 1e-6) == 0)
    with pytest.raises(ValueError):
        A.rmsnorm(X, gamma, -1.0)


def test_rmsnorm_against_exact_rational_brute_force():
    X, gamma = _norm_inputs(M=5, K=48, seed=22)
    # a row whose squares span 2^-48 .. 2^31: no floating-point order sums it exactly
    X[4, :] = np.float16(2.0 ** -24)
    X[4, 0], X[4, 1], X[4, 2] = np.float16(-60000.0), np.float16(0.3333), np.float16(6.1e-5)
    for eps in (0.0, 1e-6, 1e-5):
        y = A.rmsnorm(X, gamma, eps)
        for m in range(X.shape[0]):
            want = brute.rmsnorm_row([float(v) for v in X[m]], [float(g) for g in gamma], float(np.float32(eps)))
            assert [float(v) for v in want] == y[m].astype(np.float64).tolist(), (m, eps)


def test_fused_rmsnorm_quantizer_is_the_composition():
    X, gamma = _norm_inputs(M=10, K=128, seed=23)
    perm = wk.calibrate_perm(A.rmsnorm(X, gamma, 1e-5))
    sT = wk.tensor_scale(A.rmsnorm(X, gamma, 1e-5))
    c1, s1 = A.rmsnorm_quantize_act(X, gamma, 1e-5, perm, 32, sT)
    c2, s2 = A.quantize_act(A.rmsnorm(X, gamma, 1e-5), perm, 32, sT)
    assert np.array_equal(c1, c2) and np.array_equal(s1, s2)
    assert c1.shape == (10, 80) and s1.shape == (10, 10)
