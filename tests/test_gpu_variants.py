"""GPU parity of the layout and scale-rounding variants (the *_ex entry points) against the oracle:
packed bytes bit-exact, the product through the unchanged GEMM within the GEMM's tolerance."""
import numpy as np
import pytest
import torch

from oracle import arcquant as A
from oracle import mxfp4 as MX
from paper_2601_07475_amd import binding as B
from paper_2601_07475_amd import workloads as wk

from test_gpu_parity import (GEMM_TOL_F16, GEMM_TOL_F32, assert_same_bytes, dev, gpu_mx_quantize, gpu_quantize,
                             norm_case, norm_err, rand_case, say)

pytestmark = pytest.mark.gpu

VARIANTS = {  # flags -> the oracle's keyword arguments
    B.LAYOUT_INTERLEAVED: dict(layout="interleaved"),
    B.SCALE_ROUND_UP: dict(scale_rounding="up"),
    B.LAYOUT_INTERLEAVED | B.SCALE_ROUND_UP: dict(layout="interleaved", scale_rounding="up"),
}

SHAPES = [  # M, K, S: blocks per lane 1..4, lane tails, S = 0, S = K, one outlier block
    (3, 16, 16), (5, 48, 16), (16, 512, 32), (7, 1040, 0), (33, 1040, 1040), (67, 4096, 256), (9, 5120, 512),
    (5, 14336, 256), (4, 16400, 4800), (3, 28672, 1024), (2, 65536, 2048),
]


def with_flags(fn, flags):
    def call(x, perm, S, sT, codes, scales):
        return fn(x, perm, S, sT, flags, codes=codes, scales=scales)
    return call


@pytest.mark.parametrize("flags", sorted(VARIANTS))
@pytest.mark.parametrize("M,K,S", SHAPES)
def test_quantize_act_and_pack_weight_variants_bit_exact(M, K, S, flags):
    say(f"quantize_act_ex / pack_weight_ex parity M={M} K={K} S={S} flags={flags}")
    kw = VARIANTS[flags]
    c = rand_case(M, K, 8, S, seed=900 + K % 97)
    want_c, want_s = A.quantize_act(c["X"], c["perm"], S, c["sT_x"], **kw)
    got_c, got_s = gpu_quantize(with_flags(B.arcq_quantize_act_ex, flags), c["X"], c["perm"], S, c["sT_x"])
    assert_same_bytes(got_s, want_s, "scales")
    assert_same_bytes(got_c, want_c, "codes")
    want_c, want_s = A.pack_weight(c["X"], c["perm"], S, c["sT_x"], **kw)       # the packer on the same tensor
    got_c, got_s = gpu_quantize(with_flags(B.arcq_pack_weight_ex, flags), c["X"], c["perm"], S, c["sT_x"])
    assert_same_bytes(got_s, want_s, "weight scales")
    assert_same_bytes(got_c, want_c, "weight codes")


def test_flags_zero_is_the_plain_call():
    say("*_ex with flags = 0 against the plain entry points")
    c = rand_case(40, 2048, 24, 128, seed=5)
    X, W, perm = dev(c["X"]), dev(c["W"]), dev(c["perm"])
    for plain, ex, t, sT in ((B.arcq_quantize_act, B.arcq_quantize_act_ex, X, c["sT_x"]),
                             (B.arcq_pack_weight, B.arcq_pack_weight_ex, W, c["sT_w"])):
        a = plain(t, perm, 128, sT)
        b = ex(t, perm, 128, sT, 0)
        assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    a = B.arcq_mx_quantize_act(X, perm, 128)
    b = B.arcq_mx_quantize_act_ex(X, perm, 128, 0)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    with pytest.raises(B.ArcqError):
        B.arcq_quantize_act_ex(X, perm, 128, c["sT_x"], 4)


@pytest.mark.parametrize("flags", sorted(VARIANTS))
def test_round_up_over_every_fp16_value_and_edge_blocks(flags):
    say(f"quantize_act_ex over every finite fp16 value, flags={flags}")
    kw = VARIANTS[flags]
    bits = np.arange(0x10000, dtype=np.uint32)
    vals = bits[(bits & 0x7C00) != 0x7C00].astype(np.uint16).view(np.float16)
    rng = np.random.default_rng(8)
    K = 512
    rows = [vals[rng.permutation(len(vals))][: len(vals) // K * K].reshape(-1, K)]
    srt = np.sort(vals.astype(np.float32)).astype(np.float16)       # neighbours share a block: small spreads
    rows.append(srt[: len(srt) // K * K].reshape(-1, K))
    edge = np.zeros((3, K), np.float16)
    edge[1, ::3] = np.float16(-0.0)
    edge[2] = np.float16(2.0 ** -24)                                # nonzero, below every E4M3 subnormal step
    rows.append(edge)
    X = np.concatenate(rows).astype(np.float16)
    perm = rng.permutation(K).astype(np.int32)
    for sT in (wk.tensor_scale(X), np.float32(1.0), np.float32(2.0 ** -12)):
        want_c, want_s = A.quantize_act(X, perm, K, sT, **kw)
        got_c, got_s = gpu_quantize(with_flags(B.arcq_quantize_act_ex, flags), X, perm, K, sT)
        assert_same_bytes(got_s, want_s, f"scales sT={sT}")
        assert_same_bytes(got_c, want_c, f"codes sT={sT}")


@pytest.mark.parametrize("flags", sorted(VARIANTS))
@pytest.mark.parametrize("M,K,S", [(16, 512, 32), (67, 4096, 256), (5, 14336, 256), (3, 28672, 1024)])
def test_rmsnorm_quantize_act_variants_bit_exact(M, K, S, flags):
    say(f"rmsnorm_quantize_act_ex parity M={M} K={K} S={S} flags={flags}")
    X, gamma, perm, sT = norm_case(M, K, S, seed=340 + K % 89)
    g = dev(gamma)

    def fn(x, p, S_, t, codes, scales):
        return B.arcq_rmsnorm_quantize_act_ex(x, g, 1e-5, p, S_, t, flags, codes=codes, scales=scales)
    want_c, want_s = A.rmsnorm_quantize_act(X, gamma, 1e-5, perm, S, sT, **VARIANTS[flags])
    got_c, got_s = gpu_quantize(fn, X, perm, S, sT)
    assert_same_bytes(got_s, want_s, "scales")
    assert_same_bytes(got_c, want_c, "codes")


@pytest.mark.parametrize("flags", sorted(VARIANTS))
@pytest.mark.parametrize("M,N,K,S", [(16, 512, 512, 32), (70, 200, 1024, 1024), (16, 300, 4096, 256), (300, 260, 2048, 48)])
def test_variant_step_through_the_unchanged_gemm(M, N, K, S, flags):
    """Appendix D: with both operands in the same layout the standard GEMM needs no change."""
    say(f"variant step M={M} N={N} K={K} S={S} flags={flags}")
    kw = VARIANTS[flags]
    c = rand_case(M, K, N, S, seed=40 + M)
    X, W, perm = dev(c["X"]), dev(c["W"]), dev(c["perm"])
    ac, asc = B.arcq_quantize_act_ex(X, perm, S, c["sT_x"], flags)
    wc, wsc = B.arcq_pack_weight_ex(W, perm, S, c["sT_w"], flags)
    oac, oasc = A.quantize_act(c["X"], c["perm"], S, c["sT_x"], **kw)
    owc, owsc = A.pack_weight(c["W"], c["perm"], S, c["sT_w"], **kw)
    Yref = A.gemm(oac, oasc, c["sT_x"], owc, owsc, c["sT_w"])
    for dtype, tol in ((torch.float32, GEMM_TOL_F32), (torch.float16, GEMM_TOL_F16)):
        Y = B.arcq_gemm(ac, asc, c["sT_x"], wc, wsc, c["sT_w"], out_dtype=dtype).float().cpu().numpy()
        assert norm_err(Y, Yref) <= tol
    # the layout does not change the product beyond the order of the fp32 sums
    if flags == B.LAYOUT_INTERLEAVED:
        pac, pasc = B.arcq_quantize_act(X, perm, S, c["sT_x"])
        pwc, pwsc = B.arcq_pack_weight(W, perm, S, c["sT_w"])
        Yp = B.arcq_gemm(pac, pasc, c["sT_x"], pwc, pwsc, c["sT_w"], out_dtype=torch.float32).cpu().numpy()
        Yi = B.arcq_gemm(ac, asc, c["sT_x"], wc, wsc, c["sT_w"], out_dtype=torch.float32).cpu().numpy()
        assert norm_err(Yi, Yp.astype(np.float64)) <= GEMM_TOL_F32


def test_variants_full_size_llama8b_qproj():
    say("interleaved + round-up at full size 2048 x 4096 x 4096, S = 256")
    flags = B.LAYOUT_INTERLEAVED | B.SCALE_ROUND_UP
    kw = VARIANTS[flags]
    c = wk.make_case(wk.WORKLOADS["c2_llama8b_q"])
    X, W, perm, S = c["X"], c["W"], c["perm"], c["S"]
    want_c, want_s = A.quantize_act(X, perm, S, c["sT_x"], **kw)
    ac, asc = B.arcq_quantize_act_ex(dev(X), dev(perm), S, c["sT_x"], flags)
    assert_same_bytes(asc.cpu().numpy(), want_s, "scales")
    assert_same_bytes(ac.cpu().numpy(), want_c, "codes")
    wc, wsc = B.arcq_pack_weight_ex(dev(W), dev(perm), S, c["sT_w"], flags)
    owc, owsc = A.pack_weight(W, perm, S, c["sT_w"], **kw)
    assert_same_bytes(wc.cpu().numpy(), owc, "weight codes")
    assert_same_bytes(wsc.cpu().numpy(), owsc, "weight scales")
    Y = B.arcq_gemm(ac, asc, c["sT_x"], wc, wsc, c["sT_w"]).float().cpu().numpy()
    rows = np.random.default_rng(2).choice(X.shape[0], 48, replace=False)
    Yref = A.gemm(want_c[rows], want_s[rows], c["sT_x"], owc, owsc, c["sT_w"])
    assert norm_err(Y[rows], Yref) <= GEMM_TOL_F16


# ---- MXFP4 ---------------------------------------------------------------------------------
MX_SHAPES = [(3, 32, 32), (5, 96, 32), (16, 512, 64), (33, 1056, 1056), (67, 4096, 256), (9, 5120, 512),
             (5, 14336, 256), (3, 28672, 1024), (2, 40000, 32), (2, 65536, 2048)]


def mx_with_flags(fn, flags):
    def call(x, perm, S, codes, scales):
        return fn(x, perm, S, flags, codes=codes, scales=scales)
    return call


@pytest.mark.parametrize("flags", sorted(VARIANTS))
@pytest.mark.parametrize("M,K,S", MX_SHAPES)
def test_mx_variants_bit_exact(M, K, S, flags):
    say(f"mx_quantize_act_ex / mx_pack_weight_ex parity M={M} K={K} S={S} flags={flags}")
    kw = VARIANTS[flags]
    c = rand_case(M, K, 8, S, seed=1200 + K % 97)
    want_c, want_s = MX.quantize_act(c["X"], c["perm"], S, **kw)
    got_c, got_s = gpu_mx_quantize(mx_with_flags(B.arcq_mx_quantize_act_ex, flags), c["X"], c["perm"], S)
    assert_same_bytes(got_s, want_s, "scales")
    assert_same_bytes(got_c, want_c, "codes")
    want_c, want_s = MX.pack_weight(c["X"], c["perm"], S, **kw)
    got_c, got_s = gpu_mx_quantize(mx_with_flags(B.arcq_mx_pack_weight_ex, flags), c["X"], c["perm"], S)
    assert_same_bytes(got_s, want_s, "weight scales")
    assert_same_bytes(got_c, want_c, "weight codes")


def test_mx_round_up_over_every_fp16_value():
    say("mx_quantize_act_ex (round-up) over every finite fp16 value")
    bits = np.arange(0x10000, dtype=np.uint32)
    vals = bits[(bits & 0x7C00) != 0x7C00].astype(np.uint16).view(np.float16)
    rng = np.random.default_rng(9)
    K = 512
    rows = [vals[rng.permutation(len(vals))][: len(vals) // K * K].reshape(-1, K)]
    srt = np.sort(vals.astype(np.float32)).astype(np.float16)
    rows.append(srt[: len(srt) // K * K].reshape(-1, K))
    rows.append(np.zeros((2, K), np.float16))
    X = np.concatenate(rows).astype(np.float16)
    perm = rng.permutation(K).astype(np.int32)
    flags = B.LAYOUT_INTERLEAVED | B.SCALE_ROUND_UP
    want_c, want_s = MX.quantize_act(X, perm, K, **VARIANTS[flags])
    got_c, got_s = gpu_mx_quantize(mx_with_flags(B.arcq_mx_quantize_act_ex, flags), X, perm, K)
    assert_same_bytes(got_s, want_s, "scales")
    assert_same_bytes(got_c, want_c, "codes")


@pytest.mark.parametrize("flags", sorted(VARIANTS))
@pytest.mark.parametrize("M,N,K,S", [(16, 512, 512, 64), (70, 200, 1024, 1024), (16, 300, 4096, 256), (300, 260, 2048, 96)])
def test_mx_variant_step_through_the_unchanged_gemm(M, N, K, S, flags):
    say(f"mx variant step M={M} N={N} K={K} S={S} flags={flags}")
    kw = VARIANTS[flags]
    c = rand_case(M, K, N, S, seed=60 + M)
    X, W, perm = dev(c["X"]), dev(c["W"]), dev(c["perm"])
    ac, asc = B.arcq_mx_quantize_act_ex(X, perm, S, flags)
    wc, wsc = B.arcq_mx_pack_weight_ex(W, perm, S, flags)
    oac, oasc = MX.quantize_act(c["X"], c["perm"], S, **kw)
    owc, owsc = MX.pack_weight(c["W"], c["perm"], S, **kw)
    Yref = MX.gemm(oac, oasc, owc, owsc)
    for dtype, tol in ((torch.float32, GEMM_TOL_F32), (torch.float16, GEMM_TOL_F16)):
        Y = B.arcq_mx_gemm(ac, asc, wc, wsc, out_dtype=dtype).float().cpu().numpy()
        assert norm_err(Y, Yref) <= tol
