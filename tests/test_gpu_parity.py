"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element.

Bars: codes and scale bytes bit-exact; GEMM within 1e-3 of the fp64 oracle in the normalised
max error  max_ij |Y - Yref| / max(|Yref_ij|, rms(Yref))  (element-wise relative error is
unbounded at cancellation zeros), fp32 accumulate.
"""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

from oracle import arcquant as A
from oracle import calibration as CAL
from oracle import mxfp4 as MX
from paper_2601_07475_amd import binding as B
from paper_2601_07475_amd import workloads as wk

pytestmark = pytest.mark.gpu

GEMM_TOL_F16 = 1e-3      # fp16 output: half an ulp of fp16 is 2^-11 = 4.9e-4
GEMM_TOL_F32 = 2e-5      # fp32 output: only fp32 accumulation order differs from fp64


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def say(*a):
    print(*a, flush=True)


def norm_err(Y, Yref):
    Y = np.asarray(Y, dtype=np.float64)
    rms = np.sqrt(np.mean(Yref ** 2))
    return float(np.max(np.abs(Y - Yref) / np.maximum(np.abs(Yref), max(rms, 1e-300))))


def guarded_empty(shape, fill=0xA5):
    """uint8 buffer with 256 guard bytes on both sides, to catch out-of-bounds stores."""
    n = int(np.prod(shape))
    n_al = (n + 255) // 256 * 256
    raw = torch.full((n_al + 512,), fill, dtype=torch.uint8, device="cuda")
    return raw, raw[256:256 + n].view(*shape)


def guards_intact(raw, n, fill=0xA5):
    n_al = (n + 255) // 256 * 256
    r = raw.cpu().numpy()
    return bool(np.all(r[:256] == fill) and np.all(r[256 + n:] == fill)) and len(r) == n_al + 512


def gpu_quantize(fn, X, perm, S, sT):
    rows, K = X.shape
    Kp = K + S
    raw_c, codes = guarded_empty((rows, Kp // 2))
    raw_s, scales = guarded_empty((rows, Kp // 16))
    fn(dev(X), dev(perm.astype(np.int32)), S, sT, codes=codes, scales=scales)
    torch.cuda.synchronize()
    assert guards_intact(raw_c, rows * Kp // 2) and guards_intact(raw_s, rows * Kp // 16)
    return codes.cpu().numpy(), scales.cpu().numpy()


def assert_same_bytes(got, want, what):
    if not np.array_equal(got, want):
        bad = np.argwhere(got != want)
        raise AssertionError(f"{what}: {len(bad)} of {want.size} bytes differ; first at {bad[0].tolist()}: "
                             f"got {got[tuple(bad[0])]:#x} want {want[tuple(bad[0])]:#x}")


def rand_case(M, K, N, S, seed, kind="loguniform20_100"):
    wl = wk.Workload("t", M, K, N, S, max(1, K // 100), kind, 0.02, seed)
    return wk.make_case(wl)


# --------------------------------------------------------------------------------------
SHAPES = [  # M, K, S : several workgroup sizes, lanes-per-row tails, blocks-per-lane 1..4, S = 0 and S = K
    (1, 16, 0), (3, 16, 16), (5, 48, 16), (16, 512, 32), (7, 1040, 0), (33, 1040, 1040), (67, 4096, 256),
    (9, 5120, 512), (5, 14336, 256), (4, 16400, 4800), (3, 28672, 1024), (2, 40000, 16), (2, 65536, 2048),
]


@pytest.mark.parametrize("M,K,S", SHAPES)
def test_quantize_act_bit_exact(M, K, S):
    say(f"quantize_act parity M={M} K={K} S={S}")
    c = rand_case(M, K, 8, S, seed=100 + K % 97)
    want_c, want_s = A.quantize_act(c["X"], c["perm"], S, c["sT_x"])
    got_c, got_s = gpu_quantize(B.arcq_quantize_act, c["X"], c["perm"], S, c["sT_x"])
    assert_same_bytes(got_s, want_s, "scales")
    assert_same_bytes(got_c, want_c, "codes")


def norm_case(M, K, S, seed):
    """Pre-norm hidden states, RMSNorm weight, and a permutation / tensor scale calibrated on the
    normalised activations (the quantizer's input)."""
    wl = wk.Workload("t", M, K, 8, S, max(1, K // 100), "loguniform20_100", 0.02, seed)
    X = wk.activations(wl)
    gamma = wk.rmsnorm_gamma(wl)
    Yn = A.rmsnorm(X, gamma, 1e-5)
    return X, gamma, wk.calibrate_perm(Yn), wk.tensor_scale(Yn)


def norm_quantize_call(stats_path):
    """arcq_rmsnorm_quantize_act, or its _ex form with the flag that forces the integer sum."""
    if stats_path == "integer_sum":
        return lambda x, g, eps, p, S, t, **kw: B.arcq_rmsnorm_quantize_act_ex(x, g, eps, p, S, t, B.RMSNORM_EXACT_SUM, **kw)
    return B.arcq_rmsnorm_quantize_act


def gpu_norm_quantize(X, gamma, eps, perm, S, sT, stats_path="bracketed_sum"):
    g = dev(gamma)
    call = norm_quantize_call(stats_path)

    def fn(x, p, S_, t, codes, scales):
        return call(x, g, eps, p, S_, t, codes=codes, scales=scales)
    return gpu_quantize(fn, X, perm, S, sT)


NORM_SHAPES = [  # blocks per lane 1..4, one and two row buffers, lane tails, S = 0 and S = K
    (1, 16, 0), (5, 48, 48), (16, 512, 32), (33, 1040, 1040), (67, 4096, 256), (300, 5120, 512),
    (9, 8192, 0), (5, 14336, 256), (4, 16400, 4800), (3, 28672, 1024), (2, 40000, 16), (2, 65536, 2048),
]


@pytest.fixture(params=["bracketed_sum", "integer_sum"])
def stats_path(request):
    """The kernel sums the squares in fp64 and falls back to an exact integer sum for the rare row
    whose mean it cannot round with certainty; the ARCQ_RMSNORM_EXACT_SUM flag sends every row through the
    integer sum, so both paths are held to the same oracle."""
    return request.param


@pytest.mark.parametrize("M,K,S", NORM_SHAPES)
def test_rmsnorm_quantize_act_bit_exact(M, K, S, stats_path):
    say(f"rmsnorm_quantize_act parity M={M} K={K} S={S} {stats_path}")
    X, gamma, perm, sT = norm_case(M, K, S, seed=300 + K % 89)
    for eps in (1e-5, 0.0):
        want_c, want_s = A.rmsnorm_quantize_act(X, gamma, eps, perm, S, sT)
        got_c, got_s = gpu_norm_quantize(X, gamma, eps, perm, S, sT, stats_path)
        assert_same_bytes(got_s, want_s, f"scales eps={eps}")
        assert_same_bytes(got_c, want_c, f"codes eps={eps}")


def test_rmsnorm_quantize_edge_rows_and_strided_input(stats_path):
    """Rows that stress the statistics: all zero (eps decides), one huge value among subnormals
    (squares from 2^-48 to 2^31), constant rows, a row of fp16 maxima, rows whose mean square is an
    exact fp32 midpoint (the kernel's fp64 bracket cannot decide those); input with ldx > K."""
    say(f"rmsnorm_quantize_act edge rows {stats_path}")
    K, S = 1024, 64
    rng = np.random.default_rng(77)
    X = (rng.standard_normal((12, K)) * 2).astype(np.float16)
    X[0] = 0
    X[1] = np.float16(2.0 ** -24)
    X[1, 5], X[1, 700] = np.float16(-60000.0), np.float16(0.3333)
    X[2] = np.float16(-3.0)
    X[3] = np.float16(65504.0)
    X[4] = (rng.standard_normal(K) * 2.0 ** -20).astype(np.float16)      # subnormal inputs only
    X[5, ::2] = 0
    X[6] = 0
    X[6, 3], X[6, 900] = np.float16(32.0), np.float16(2.0 ** -7)         # mean square 1 + 2^-24: tie, rounds to even
    X[7] = 0
    X[7, 1000], X[7, 2], X[7, 77] = np.float16(-32.0), np.float16(2.0 ** -7), np.float16(2.0 ** -6.5)  # close to a midpoint
    assert ((X[6].astype(np.float64) ** 2).sum() / K) == 1.0 + 2.0 ** -24
    gamma = wk.rmsnorm_gamma(wk.Workload("t", 12, K, 8, S, 8, "const50", 0.02, 78))
    gamma[3] = np.float16(0.0)
    for eps in (1e-6, 1e-2):
        Yn = A.rmsnorm(X, gamma, eps)
        perm, sT = wk.calibrate_perm(Yn), wk.tensor_scale(Yn)
        want_c, want_s = A.quantize_act(Yn, perm, S, sT)
        wide = torch.full((12, K + 40), 3.0, dtype=torch.float16, device="cuda")
        wide[:, :K] = dev(X)
        cc, ss = norm_quantize_call(stats_path)(wide[:, :K], dev(gamma), eps, dev(perm), S, sT)
        assert_same_bytes(ss.cpu().numpy(), want_s, f"scales eps={eps}")
        assert_same_bytes(cc.cpu().numpy(), want_c, f"codes eps={eps}")


def test_rmsnorm_quantize_full_size_qproj(stats_path):
    """The layer input RMSNorm feeds in practice, at full size: 2048 tokens x 4096 hidden, S = 256."""
    say(f"rmsnorm_quantize_act full size 2048 x 4096 {stats_path}")
    X, gamma, perm, sT = norm_case(2048, 4096, 256, seed=41)
    want_c, want_s = A.rmsnorm_quantize_act(X, gamma, 1e-5, perm, 256, sT)
    got_c, got_s = gpu_norm_quantize(X, gamma, 1e-5, perm, 256, sT, stats_path)
    assert_same_bytes(got_s, want_s, "scales")
    assert_same_bytes(got_c, want_c, "codes")


@pytest.mark.parametrize("N,K,S", [(1, 16, 16), (40, 512, 32), (300, 4096, 256), (17, 14336, 256), (5, 28672, 1024)])
def test_pack_weight_bit_exact(N, K, S):
    say(f"pack_weight parity N={N} K={K} S={S}")
    wl = wk.Workload("t", 4, K, N, S, max(1, K // 100), "const50", 0.02, 200 + N)
    c = wk.make_case(wl)
    want_c, want_s = A.pack_weight(c["W"], c["perm"], S, c["sT_w"])
    got_c, got_s = gpu_quantize(B.arcq_pack_weight, c["W"], c["perm"], S, c["sT_w"])
    assert_same_bytes(got_s, want_s, "scales")
    assert_same_bytes(got_c, want_c, "codes")


def test_quantize_every_fp16_value_and_edge_blocks():
    """All 63488 finite fp16 bit patterns (incl. +-0 and subnormals), shuffled into blocks, under
    several tensor scales including ones that saturate the block scale; S = K so that every block
    also goes through the residual stage."""
    say("quantize_act parity over every finite fp16 value")
    bits = np.arange(0x10000, dtype=np.uint32)
    bits = bits[(bits & 0x7C00) != 0x7C00].astype(np.uint16)            # drop Inf/NaN
    rng = np.random.default_rng(5)
    vals = bits.view(np.float16)
    K = 512
    rows = []
    for rep in range(3):
        v = vals[rng.permutation(len(vals))]
        rows.append(v[: len(v) // K * K].reshape(-1, K))
    srt = np.sort(vals.astype(np.float32)).astype(np.float16)             # similar magnitudes share a block
    rows.append(srt[: len(srt) // K * K].reshape(-1, K))
    # exact grid midpoints times power-of-two scales: ties in the element rounding
    mids = np.float16([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, 6.0])
    tie = np.concatenate([mids * np.float16(2.0 ** e) * sgn for e in range(-8, 8) for sgn in (1, -1)])
    tie = np.resize(tie, (4, K)).astype(np.float16)
    tie[:, ::16] = (6.0 * 2.0 ** np.clip(np.arange(-8, 24), -8, 13)).astype(np.float16)[None, :]
    rows.append(tie)
    rows.append(np.zeros((2, K), np.float16))
    rows[-1][1, ::3] = np.float16(-0.0)
    X = np.concatenate(rows).astype(np.float16)
    perm = rng.permutation(K).astype(np.int32)
    for sT in (wk.tensor_scale(X), np.float32(1.0), np.float32(2.0 ** -12), np.float32(0.37), np.float32(3.1e-5)):
        want_c, want_s = A.quantize_act(X, perm, K, sT)
        got_c, got_s = gpu_quantize(B.arcq_quantize_act, X, perm, K, sT)
        assert_same_bytes(got_s, want_s, f"scales sT={sT}")
        assert_same_bytes(got_c, want_c, f"codes sT={sT}")


def test_quantize_strided_input_and_determinism():
    say("quantize_act with ldx > K, repeated")
    c = rand_case(37, 1024, 8, 64, seed=9)
    X, perm, S, sT = c["X"], c["perm"], c["S"], c["sT_x"]
    wide = torch.full((37, 1024 + 24), 7.0, dtype=torch.float16, device="cuda")
    wide[:, :1024] = dev(X)
    want_c, want_s = A.quantize_act(X, perm, S, sT)
    outs = []
    for _ in range(2):
        cc, ss = B.arcq_quantize_act(wide[:, :1024], dev(perm), S, sT)
        outs.append((cc.cpu().numpy(), ss.cpu().numpy()))
    assert_same_bytes(outs[0][0], want_c, "codes")
    assert_same_bytes(outs[0][1], want_s, "scales")
    assert np.array_equal(outs[0][0], outs[1][0]) and np.array_equal(outs[0][1], outs[1][1])


def test_empty_inputs_and_check_perm():
    say("empty inputs, perm check")
    perm = dev(np.arange(64, dtype=np.int32))
    cc, ss = B.arcq_quantize_act(torch.empty((0, 64), dtype=torch.float16, device="cuda"), perm, 16, 1.0)
    assert cc.shape == (0, 40) and ss.shape == (0, 5)
    y = B.arcq_gemm(cc, ss, 1.0, torch.zeros((8, 40), dtype=torch.uint8, device="cuda"),
                    torch.zeros((8, 5), dtype=torch.uint8, device="cuda"), 1.0)
    assert y.shape == (0, 8)
    assert B.arcq_check_perm(perm)
    bad = np.arange(64, dtype=np.int32)
    bad[5] = 6
    assert not B.arcq_check_perm(dev(bad))
    bad[5] = 64
    assert not B.arcq_check_perm(dev(bad))
    bad[5] = -1
    assert not B.arcq_check_perm(dev(bad))


# --------------------------------------------------------------------------------------
GEMM_SHAPES = [  # M, N, K, S : ragged tiles, K' with every residue mod 64, tiny and skinny cases
    (1, 1, 16, 0), (16, 512, 512, 32), (77, 200, 48, 16), (130, 129, 96, 16), (128, 256, 256, 0),
    (257, 131, 1040, 48), (16, 1000, 4096, 256), (300, 77, 2048, 2048),
    (7, 45, 160, 32), (16, 4097, 1008, 16), (3, 16, 14336, 256), (17, 40, 512, 0), (128, 384, 192, 0), (500, 260, 4160, 64),
    # rows shorter than one 128-k chunk on the weight-streaming kernel (K' = 32, 64, 96)
    (8, 40, 32, 0), (16, 33, 48, 16), (5, 17, 64, 32),
    # batched decode: 2, 4 and 8 tiles of 16 activation rows on the weight-streaming kernel, S from 0 to K
    (20, 300, 512, 32), (32, 1000, 1024, 0), (33, 77, 2048, 2048), (64, 4097, 256, 64), (100, 260, 4160, 64),
    (128, 45, 160, 32), (17, 14336, 512, 512), (48, 2048, 4096, 1024),
    # more than 128 rows but few tiles: the reduction dimension is split into 2 to 8 runs (the last run of the third
    # ends with a half stage) and the partial results are added by a second kernel; the fourth is too short to split
    (256, 512, 14336, 256), (300, 260, 4160, 64), (130, 129, 2048, 64), (200, 140, 576, 64), (384, 1000, 1024, 64),
    # ragged edges in every tile configuration of the staged kernel: 128 x 256 tiles (8 waves), 256 x 256 tiles
    (1990, 4070, 256, 64), (4000, 4100, 128, 64),
    # the same 128 x 256 tiles with K' a multiple of 128: the kernel whose wave pairs split every stage
    # (ragged edges, the shortest and a longer reduction, both output types)
    (1990, 4070, 192, 64), (2048, 3000, 1024, 128),
    # 65 to 128 rows with enough weights for the tiled kernels with split K instead of the weight-streaming kernel
    # (K' >= 4096 with 2 * 10^7 weights, K' >= 8192 with 1.2 * 10^7)
    (100, 4800, 4096, 256), (128, 1500, 8192, 512),
    # between 144 and 256 tiles of 64 x 64, 128 x 64 or 128 x 128 and K' a multiple of 256: the kernel whose waves split
    # every stage into k quarters inside the workgroup (ragged edges in both directions; two, five and 17 stages)
    (130, 3100, 512, 0), (192, 4096, 4096, 256), (300, 3500, 1024, 256), (700, 3900, 448, 64), (1024, 4096, 1024, 256),
    # ... K' a multiple of 64 but not of 256: the last stage holds one, two or three of the four k shares (every tile shape)
    (130, 3100, 512, 64), (192, 4096, 1024, 128), (300, 3500, 1024, 192), (1024, 4096, 512, 64), (512, 4000, 512, 192),
    (64, 6100, 512, 64), (700, 3900, 448, 128),
    # ... K' with an odd number of blocks, or K' % 64 = 32: the same tiles with stages through registers (every tile shape)
    (130, 3100, 512, 16), (192, 4096, 1024, 48), (300, 3500, 1024, 208), (1024, 4096, 512, 16), (512, 4000, 512, 176),
    (64, 6100, 512, 16),
    # ... 96 x 64 tiles (six fragments over four waves: two waves finish two, two finish one), exact and ragged; 128 x 64
    (384, 4096, 1024, 0), (290, 3500, 512, 256), (512, 4000, 512, 0),
    # four weight tiles per wave at up to 16 rows, left-over chunks behind the last group of four: 2 chunks (the last one
    # block), 1 chunk of two blocks, 4 chunks (the last six blocks), none
    (5, 12400, 656, 0), (16, 13000, 1040, 16), (9, 12320, 992, 0), (16, 12304, 1024, 0),
    # three weight tiles per wave on the weight-streaming kernel (513 to 768 tiles of 16 weight rows), 16 and 32 rows
    (16, 10240, 512, 32), (9, 8300, 1040, 16), (32, 9000, 256, 64), (20, 12288, 4096, 256), (32, 7000, 512, 0),
    (32, 12400, 528, 0),
    # 33 to 64 rows against many weight rows: the 64 x 64 k-split tiles instead of the weight-streaming kernel
    (50, 9300, 512, 0), (64, 14336, 256, 256), (33, 9216, 1024, 0),
    # 64 x 32 tiles (two fragments over four k-quarter waves: two of the waves finish none)
    (64, 6100, 512, 0), (100, 4000, 768, 256), (40, 5000, 4096, 256), (128, 500, 512, 0), (200, 1000, 4096, 256),
    # 192 x 128 tiles (more than 256 tiles of 128 x 128, too few for the 256-wide ones): ragged edges, a half stage at the end
    (500, 10200, 192, 64), (640, 8100, 256, 64),
    # 192 x 256 tiles (one round of them where 128-row tiles need two): ragged edges, whole stages and a half stage at the end;
    # 256 x 256 tiles that fill only part of the chip (fewer than 256 of them)
    (570, 14000, 192, 64), (1100, 8000, 256, 64), (1000, 14100, 128, 64),
    # K' with an odd number of blocks, or K' % 64 = 32 (S is any multiple of 16): rows that start 8 bytes off a 16-byte
    # boundary.  Weight-streaming kernel with 1, 2, 4 and 8 row tiles, one block per row, last chunk of 1, 3, 5, 7 blocks
    (8, 40, 16, 0), (1, 300, 1008, 0), (16, 1000, 4096, 272), (16, 4097, 1008, 48), (33, 77, 2048, 2000), (20, 300, 512, 48),
    (64, 4097, 240, 64), (100, 260, 4160, 80), (128, 45, 160, 16), (17, 14336, 512, 496),
    # the same on the tiled kernels, stages through registers: 128 x 128 tiles without and with split K' (the last stage
    # holds 2, 7, 1 and 4 blocks), 128 x 256 tiles, and a large output
    (257, 131, 1040, 16), (200, 140, 560, 64), (300, 260, 4160, 80), (256, 512, 4096, 320), (1990, 4070, 240, 64),
    (2048, 3000, 1024, 144), (4000, 4100, 112, 64), (128, 1500, 8192, 528),
    # ... 192 x 256 and 192 x 128 tiles with stages through registers
    (570, 14000, 192, 80), (500, 10200, 192, 48),
]


@pytest.mark.parametrize("M,N,K,S", GEMM_SHAPES)
@pytest.mark.parametrize("dtype", [torch.float32, torch.float16])
def test_gemm_parity(M, N, K, S, dtype):
    say(f"gemm parity M={M} N={N} K={K} S={S} {dtype}")
    c = rand_case(M, K, N, S, seed=300 + M + N)
    ac, asc = A.quantize_act(c["X"], c["perm"], S, c["sT_x"])
    wc, wsc = A.pack_weight(c["W"], c["perm"], S, c["sT_w"])
    Yref = A.gemm(ac, asc, c["sT_x"], wc, wsc, c["sT_w"])
    Y = B.arcq_gemm(dev(ac), dev(asc), c["sT_x"], dev(wc), dev(wsc), c["sT_w"], out_dtype=dtype)
    torch.cuda.synchronize()
    err = norm_err(Y.float().cpu().numpy(), Yref)
    say(f"   normalised max error {err:.3e}")
    assert err <= (GEMM_TOL_F16 if dtype == torch.float16 else GEMM_TOL_F32)


@pytest.mark.parametrize("M,N,Kp", [(16, 1000, 1024), (64, 300, 4352), (300, 260, 1024), (192, 4096, 1024), (2048, 3000, 256)])
@pytest.mark.parametrize("dtype", [torch.float32, torch.float16])
def test_gemm_operands_only_8_byte_aligned(M, N, Kp, dtype):
    """Codes 8 bytes off a 16-byte boundary and scale bytes at odd addresses: the least the interface asks for."""
    say(f"gemm with 8-byte aligned operands M={M} N={N} K'={Kp} {dtype}")
    rng = np.random.default_rng(M + N + Kp)
    ac = rng.integers(0, 256, (M, Kp // 2), dtype=np.uint8)
    wc = rng.integers(0, 256, (N, Kp // 2), dtype=np.uint8)
    asc = rng.integers(0x20, 0x50, (M, Kp // 16), dtype=np.uint8)
    wsc = rng.integers(0x20, 0x50, (N, Kp // 16), dtype=np.uint8)
    Yref = A.gemm(ac, asc, np.float32(0.5), wc, wsc, np.float32(0.25))

    def shifted(a, by):
        buf = torch.zeros(a.size + 256, dtype=torch.uint8, device="cuda")
        start = (-buf.data_ptr()) % 16 + by
        view = buf[start:start + a.size].view(a.shape)
        view.copy_(torch.from_numpy(a))
        assert view.data_ptr() % 16 == by % 16
        return view
    Y = B.arcq_gemm(shifted(ac, 8), shifted(asc, 3), 0.5, shifted(wc, 8), shifted(wsc, 1), 0.25, out_dtype=dtype)
    torch.cuda.synchronize()
    err = norm_err(Y.float().cpu().numpy(), Yref)
    say(f"   normalised max error {err:.3e}")
    assert err <= (GEMM_TOL_F16 if dtype == torch.float16 else GEMM_TOL_F32)


def test_gemm_extreme_scales_and_codes():
    """Largest and smallest scale bytes and every code value: the decode must be exact."""
    say("gemm with extreme scale bytes")
    rng = np.random.default_rng(17)
    M, N, Kp = 64, 96, 128
    ac = rng.integers(0, 256, (M, Kp // 2), dtype=np.uint8)
    wc = rng.integers(0, 256, (N, Kp // 2), dtype=np.uint8)
    asc = rng.choice(np.array([0, 1, 7, 8, 9, 0x38, 0x77, 0x7D, 0x7E], dtype=np.uint8), (M, Kp // 16))
    wsc = rng.choice(np.array([0, 1, 2, 8, 0x40, 0x7E], dtype=np.uint8), (N, Kp // 16))
    Yref = A.gemm(ac, asc, np.float32(1.0), wc, wsc, np.float32(1.0))
    Y = B.arcq_gemm(dev(ac), dev(asc), 1.0, dev(wc), dev(wsc), 1.0, out_dtype=torch.float32)
    assert norm_err(Y.cpu().numpy(), Yref) <= GEMM_TOL_F32
    # a single non-zero product per output: the result must be exact in fp32
    ac1 = np.zeros_like(ac); wc1 = np.zeros_like(wc)
    ac1[:, 0] = 0x0F & rng.integers(1, 16, M, dtype=np.uint8)
    wc1[:, 0] = 0x0F & rng.integers(1, 16, N, dtype=np.uint8)
    Yref = A.gemm(ac1, asc, np.float32(1.0), wc1, wsc, np.float32(1.0))
    Y = B.arcq_gemm(dev(ac1), dev(asc), 1.0, dev(wc1), dev(wsc), 1.0, out_dtype=torch.float32)
    assert np.array_equal(Y.cpu().numpy().astype(np.float64), Yref)


@pytest.mark.parametrize("M,N,Kp,dtype", [
    (300, 260, 256, torch.float32),       # 128 x 128 tiles
    (2048, 3072, 256, torch.float32),     # 128 x 256 tiles, eight waves of 64 x 64
    (2048, 3072, 256, torch.float16),     # 128 x 256 tiles, wave pairs splitting every stage
    (4096, 4096, 128, torch.float16),     # 256 x 256 tiles
])
def test_gemm_extreme_scales_tiled_kernels(M, N, Kp, dtype):
    """Every scale byte class (zero, subnormal, smallest and largest normal) and every code value through the
    decode of the tiled kernels; the weights' scales are kept small so that the fp16 output stays finite."""
    say(f"tiled gemm with extreme scale bytes M={M} N={N} K'={Kp} {dtype}")
    rng = np.random.default_rng(23)
    ac = rng.integers(0, 256, (M, Kp // 2), dtype=np.uint8)
    wc = rng.integers(0, 256, (N, Kp // 2), dtype=np.uint8)
    asc = rng.choice(np.array([0, 1, 7, 8, 9, 0x38, 0x77, 0x7D, 0x7E], dtype=np.uint8), (M, Kp // 16))
    wsc = rng.choice(np.array([0, 1, 2, 7, 8, 9, 0x10], dtype=np.uint8), (N, Kp // 16))
    Y = B.arcq_gemm(dev(ac), dev(asc), 1.0, dev(wc), dev(wsc), 1.0, out_dtype=dtype).float().cpu().numpy()
    assert np.all(np.isfinite(Y))
    rows = rng.choice(M, 64, replace=False)
    Yref = A.gemm(ac[rows], asc[rows], np.float32(1.0), wc, wsc, np.float32(1.0))
    assert norm_err(Y[rows], Yref) <= (GEMM_TOL_F32 if dtype == torch.float32 else GEMM_TOL_F16)


def test_gemm_strided_output_and_guard():
    say("gemm with ldy > N")
    c = rand_case(70, 256, 90, 32, seed=31)
    ac, asc = A.quantize_act(c["X"], c["perm"], 32, c["sT_x"])
    wc, wsc = A.pack_weight(c["W"], c["perm"], 32, c["sT_w"])
    Yref = A.gemm(ac, asc, c["sT_x"], wc, wsc, c["sT_w"])
    big = torch.full((70, 120), -77.0, dtype=torch.float32, device="cuda")
    B.arcq_gemm(dev(ac), dev(asc), c["sT_x"], dev(wc), dev(wsc), c["sT_w"], y=big[:, :90])
    out = big.cpu().numpy()
    assert np.all(out[:, 90:] == -77.0)
    assert norm_err(out[:, :90], Yref) <= GEMM_TOL_F32


# --------------------------------------------------------------------------------------
# Every configuration at its full size, launched as the benchmark launches it, and compared with the oracle in
# full: every code byte and scale byte of X and of W, and every element of Y (fp16 and fp32 output) against the
# fp64 product of the oracle's own packed operands.  The oracle works through the rows in chunks of about 2^18
# elements (its temporaries stay in the caches) on a pool of threads (numpy releases the interpreter lock
# inside its loops); chunking by rows changes nothing in what it computes, since every row is independent.
ORACLE_THREADS = min(16, os.cpu_count() or 1)
FULL_CONFIGS = ["c1_tiny", "c2_llama8b_q", "c3a_llama8b_up", "c3b_llama8b_down", "c4_qwen32b_mlp", "c5_llama70b_down"]


def oracle_by_rows(fn, T, chunk_elems=1 << 18):
    """fn(rows of T) -> tuple of arrays with one row per input row, evaluated chunk by chunk and concatenated."""
    step = max(1, chunk_elems // T.shape[1])
    with ThreadPoolExecutor(ORACLE_THREADS) as ex:
        parts = list(ex.map(lambda r0: fn(T[r0:r0 + step]), range(0, T.shape[0], step)))
    return tuple(np.concatenate([p[i] for p in parts]) for i in range(len(parts[0])))


class FullConfig:
    def __init__(self, name):
        wl = self.wl = wk.WORKLOADS[name]
        say(f"full config {name}: M={wl.M} K={wl.K} N={wl.N} S={wl.S}: inputs")
        self.c = wk.make_case(wl)
        self._act = self._wgt = self._yref = self._gpu = None

    def gpu(self):
        """The HIP path's packed operands (device tensors), computed once."""
        if self._gpu is None:
            c = self.c
            permd = dev(c["perm"])
            ac, asc = B.arcq_quantize_act(dev(c["X"]), permd, c["S"], c["sT_x"])
            wc, wsc = B.arcq_pack_weight(dev(c["W"]), permd, c["S"], c["sT_w"])
            torch.cuda.synchronize()
            self._gpu = (ac, asc, wc, wsc)
        return self._gpu

    def oracle_act(self):
        if self._act is None:
            c = self.c
            say("   oracle: quantize_act on every row")
            self._act = oracle_by_rows(lambda x: A.quantize_act(x, c["perm"], c["S"], c["sT_x"]), c["X"])
        return self._act

    def oracle_wgt(self):
        if self._wgt is None:
            c = self.c
            say("   oracle: pack_weight on every row")
            self._wgt = oracle_by_rows(lambda w: A.pack_weight(w, c["perm"], c["S"], c["sT_w"]), c["W"])
        return self._wgt

    def oracle_y(self):
        """eq. (2) in fp64 on the ORACLE's packed operands, all M x N entries."""
        if self._yref is None:
            c, wl = self.c, self.wl
            (oac, oasc), (owc, owsc) = self.oracle_act(), self.oracle_wgt()
            say("   oracle: fp64 dequantize + product, every entry")
            step = max(1, (1 << 18) // (wl.K + wl.S))
            with ThreadPoolExecutor(ORACLE_THREADS) as ex:
                Wd = np.concatenate(list(ex.map(
                    lambda r0: A.dequantize(owc[r0:r0 + step], owsc[r0:r0 + step], c["sT_w"]), range(0, wl.N, step))))
            Y = np.empty((wl.M, wl.N))
            for r0 in range(0, wl.M, 1024):
                Y[r0:r0 + 1024] = A.dequantize(oac[r0:r0 + 1024], oasc[r0:r0 + 1024], c["sT_x"]) @ Wd.T
            self._yref = Y
        return self._yref


@pytest.fixture(scope="module", params=FULL_CONFIGS)
def full(request):
    fc = FullConfig(request.param)
    yield fc
    fc.__dict__.clear()
    torch.cuda.empty_cache()


def test_full_size_activation_bytes(full):
    ac, asc, _, _ = full.gpu()
    oac, oasc = full.oracle_act()
    assert_same_bytes(asc.cpu().numpy(), oasc, "activation scales")
    assert_same_bytes(ac.cpu().numpy(), oac, "activation codes")


def test_full_size_weight_bytes(full):
    _, _, wc, wsc = full.gpu()
    owc, owsc = full.oracle_wgt()
    assert_same_bytes(wsc.cpu().numpy(), owsc, "weight scales")
    assert_same_bytes(wc.cpu().numpy(), owc, "weight codes")


@pytest.mark.parametrize("dtype", [torch.float16, torch.float32])
def test_full_size_gemm_every_entry(full, dtype):
    c = full.c
    ac, asc, wc, wsc = full.gpu()
    Y = B.arcq_gemm(ac, asc, c["sT_x"], wc, wsc, c["sT_w"], out_dtype=dtype)
    torch.cuda.synchronize()
    Yref = full.oracle_y()
    rms = max(float(np.sqrt(np.mean(Yref ** 2))), 1e-300)
    err, worst = 0.0, None
    for r0 in range(0, full.wl.M, 512):                       # row chunks only bound the temporaries
        ref = Yref[r0:r0 + 512]
        e = np.abs(Y[r0:r0 + 512].double().cpu().numpy() - ref) / np.maximum(np.abs(ref), rms)
        i = np.unravel_index(np.argmax(e), e.shape)
        if e[i] > err:
            err, worst = float(e[i]), (r0 + int(i[0]), int(i[1]))
    say(f"   {full.wl.name} {dtype}: normalised max error {err:.3e} at {worst} over {Yref.size} entries")
    assert err <= (GEMM_TOL_F16 if dtype == torch.float16 else GEMM_TOL_F32)


# --------------------------------------------------------------------------------------
# Offline calibration (Section 3.2 "Adaptive Outlier Identification"): exact integer / bit results
@pytest.mark.parametrize("M,K", [(1, 16), (7, 48), (33, 512), (100, 1040), (257, 4096), (2048, 4096), (64, 14336),
                                 (5, 65536), (1000, 8192)])
def test_calib_absmax_bit_exact(M, K):
    say(f"calib_absmax M={M} K={K}")
    wl = wk.Workload("t", M, K, 8, 0, max(1, K // 100), "loguniform20_100", 0.02, 500 + K % 61)
    X = wk.activations(wl)
    X[0, 0], X[M - 1, K - 1] = np.float16(-65504.0), np.float16(-0.0)
    if M > 2:
        X[:, 3] = (np.arange(M) % 7 * 2.0 ** -24).astype(np.float16)                 # a column of subnormals
    want = CAL.absmax_update(np.zeros(K, np.float32), X)
    got = B.arcq_calib_absmax(dev(X), torch.zeros(K, dtype=torch.float32, device="cuda"))
    assert np.array_equal(got.cpu().numpy().view(np.uint32), want.view(np.uint32))
    # batches in another order, one of them through a strided view, on top of a non-zero running statistic
    acc = torch.zeros(K, dtype=torch.float32, device="cuda")
    cut = M // 3
    wide = torch.full((M - cut, K + 24), 70000.0, dtype=torch.float32, device="cuda").to(torch.float16)
    wide[:, :K] = dev(X[cut:])
    B.arcq_calib_absmax(wide[:, :K], acc)
    B.arcq_calib_absmax(dev(X[:cut]) if cut else torch.empty((0, K), dtype=torch.float16, device="cuda"), acc)
    B.arcq_calib_absmax(dev(X[:1]), acc)
    assert np.array_equal(acc.cpu().numpy(), want)


@pytest.mark.parametrize("K,seed", [(16, 0), (48, 1), (512, 2), (4096, 3), (16400, 4), (65536, 5)])
def test_calib_select_exact(K, seed):
    say(f"calib_select K={K}")
    rng = np.random.default_rng(seed)
    cm = np.abs(rng.standard_normal(K) * np.exp(rng.standard_normal(K) * 2)).astype(np.float16).astype(np.float32)
    cm[rng.integers(0, K, K // 4)] = cm[rng.integers(0, K, K // 4)]                   # many ties
    cases = [cm, np.zeros(K, np.float32), np.full(K, 2.5, np.float32), np.arange(K, dtype=np.float32)[::-1].copy()]
    edge = np.ones(K, np.float32)
    edge[K // 2], edge[1] = 8.0, np.nextafter(np.float32(1.0), np.float32(2.0))       # one channel at tau, one just above
    cases.append(edge)
    for c in cases:
        want = CAL.select_outliers(c)
        perm, S, info = B.arcq_calib_select(dev(c))
        info = info.cpu().numpy()
        assert np.array_equal(perm.cpu().numpy(), want["perm"])
        assert S == want["S"] and info[0] == want["S"] and info[1] == want["S_raw"]
        assert info[2:].view(np.float32).tolist() == [want["layer_max"], want["tau"]]
        assert B.arcq_check_perm(perm)


def test_calibration_feeds_the_online_path():
    """abs-max over two batches -> perm, S -> packer, quantizer, GEMM: every stage equals the oracle fed the same way."""
    say("calibration end to end")
    wl = wk.Workload("t", 96, 1024, 200, 0, 12, "loguniform20_100", 0.02, 77)
    X, W = wk.activations(wl), wk.weights(wl)
    colmax = torch.zeros(wl.K, dtype=torch.float32, device="cuda")
    for part in (X[:40], X[40:]):
        B.arcq_calib_absmax(dev(part), colmax)
    perm, S, _ = B.arcq_calib_select(colmax)
    want = CAL.select_outliers(CAL.absmax_update(np.zeros(wl.K, np.float32), X))
    assert S == want["S"] and S > 0 and np.array_equal(perm.cpu().numpy(), want["perm"])
    sTx, sTw = wk.tensor_scale(X), wk.tensor_scale(W)
    ac, asc = B.arcq_quantize_act(dev(X), perm, S, sTx)
    wc, wsc = B.arcq_pack_weight(dev(W), perm, S, sTw)
    oac, oasc = A.quantize_act(X, want["perm"], S, sTx)
    owc, owsc = A.pack_weight(W, want["perm"], S, sTw)
    assert_same_bytes(ac.cpu().numpy(), oac, "activation codes")
    assert_same_bytes(asc.cpu().numpy(), oasc, "activation scales")
    assert_same_bytes(wc.cpu().numpy(), owc, "weight codes")
    assert_same_bytes(wsc.cpu().numpy(), owsc, "weight scales")
    Y = B.arcq_gemm(ac, asc, sTx, wc, wsc, sTw, out_dtype=torch.float32)
    assert norm_err(Y.cpu().numpy(), A.gemm(oac, oasc, sTx, owc, owsc, sTw)) <= GEMM_TOL_F32


# --------------------------------------------------------------------------------------
# MXFP4 variant of the path: codes and scale bytes bit-exact, GEMM on the scaled FP4 matrix instruction
def gpu_mx_quantize(fn, X, perm, S):
    rows, K = X.shape
    Kp = K + S
    raw_c, codes = guarded_empty((rows, Kp // 2))
    raw_s, scales = guarded_empty((rows, Kp // 32))
    fn(dev(X), dev(perm.astype(np.int32)), S, codes=codes, scales=scales)
    torch.cuda.synchronize()
    assert guards_intact(raw_c, rows * Kp // 2) and guards_intact(raw_s, rows * Kp // 32)
    return codes.cpu().numpy(), scales.cpu().numpy()


MX_SHAPES = [(1, 32, 0), (3, 32, 32), (5, 96, 32), (16, 512, 64), (33, 1056, 1056), (67, 4096, 256), (9, 5120, 512),
             (5, 14336, 256), (3, 28672, 1024), (2, 40000, 32), (2, 65536, 2048)]


@pytest.mark.parametrize("M,K,S", MX_SHAPES)
def test_mx_quantize_act_bit_exact(M, K, S):
    say(f"mx_quantize_act parity M={M} K={K} S={S}")
    c = rand_case(M, K, 8, S, seed=700 + K % 97)
    want_c, want_s = MX.quantize_act(c["X"], c["perm"], S)
    got_c, got_s = gpu_mx_quantize(B.arcq_mx_quantize_act, c["X"], c["perm"], S)
    assert_same_bytes(got_s, want_s, "scales")
    assert_same_bytes(got_c, want_c, "codes")
    want_c, want_s = MX.pack_weight(c["X"], c["perm"], S)            # the packer on the same tensor
    got_c, got_s = gpu_mx_quantize(B.arcq_mx_pack_weight, c["X"], c["perm"], S)
    assert_same_bytes(got_s, want_s, "weight scales")
    assert_same_bytes(got_c, want_c, "weight codes")


def test_mx_quantize_every_fp16_value():
    say("mx_quantize_act over every finite fp16 value")
    bits = np.arange(0x10000, dtype=np.uint32)
    vals = bits[(bits & 0x7C00) != 0x7C00].astype(np.uint16).view(np.float16)
    rng = np.random.default_rng(6)
    K = 512
    rows = [vals[rng.permutation(len(vals))][: len(vals) // K * K].reshape(-1, K) for _ in range(2)]
    srt = np.sort(vals.astype(np.float32)).astype(np.float16)
    rows.append(srt[: len(srt) // K * K].reshape(-1, K))
    rows.append(np.zeros((2, K), np.float16))
    rows[-1][1, ::3] = np.float16(-0.0)
    X = np.concatenate(rows).astype(np.float16)
    perm = rng.permutation(K).astype(np.int32)
    want_c, want_s = MX.quantize_act(X, perm, K)
    got_c, got_s = gpu_mx_quantize(B.arcq_mx_quantize_act, X, perm, K)
    assert_same_bytes(got_s, want_s, "scales")
    assert_same_bytes(got_c, want_c, "codes")


MX_GEMM_SHAPES = [  # M, N, K, S: fallback kernel (K' % 128 != 0), every staged tile configuration, ragged edges
    (1, 1, 32, 0), (77, 200, 64, 32), (130, 129, 96, 32), (16, 512, 512, 0), (128, 256, 256, 0), (257, 131, 1024, 0),
    (300, 77, 2048, 2048), (500, 260, 4096, 128), (16, 1000, 4096, 256), (1990, 4070, 256, 128), (4000, 4100, 96, 32),
    # weight-streaming kernel (up to 64 rows): 1, 2, 4 tiles of 16 rows, ragged N, one chunk, many chunks split over the waves
    (8, 40, 128, 0), (20, 300, 512, 128), (33, 77, 2048, 2048), (64, 4097, 256, 128), (100, 260, 4096, 128),
    (17, 14336, 512, 512), (48, 2048, 4096, 1024), (1, 4096, 14336, 256),
    # where the tiled kernels take over from the weight-streaming one: 33 to 64 rows with at least 8192 weight rows
    # (and just below), more than 64 rows
    (48, 8200, 480, 32), (48, 8100, 480, 32), (65, 300, 992, 32),
    # weight-streaming kernel with K' % 128 != 0: a last chunk of 1, 2 or 3 blocks, rows shorter than a chunk
    (8, 40, 96, 0), (3, 17, 32, 32), (20, 300, 512, 160), (33, 77, 2048, 2016), (64, 4097, 256, 96), (1, 4096, 14336, 288),
    (17, 14336, 512, 480),
    # three and four weight tiles per wave on the weight-streaming kernel
    (16, 10240, 512, 0), (32, 9000, 256, 64), (32, 12400, 512, 32),
    # 192 x 128 tiles (more than 256 tiles of 128 x 128, too few for the 256-wide ones): a whole unit, a half unit at the end
    (500, 10200, 256, 0), (640, 8100, 256, 128),
    # 192 x 256 tiles: whole units, a half unit at the end, units through registers
    (570, 14000, 512, 0), (1100, 8000, 256, 128), (570, 14000, 256, 96),
    # the same on the tiled kernels, units through registers: 128 x 128 tiles without and with split K' (the last unit
    # holds 1, 7 and 5 blocks), 128 x 256 and 256 x 256 tiles
    (257, 131, 1024, 32), (300, 77, 2048, 2016), (500, 260, 4096, 160), (1990, 4070, 256, 96), (4000, 4100, 288, 32),
    (96, 9000, 992, 96),
]


@pytest.mark.parametrize("M,N,K,S", MX_GEMM_SHAPES)
@pytest.mark.parametrize("dtype", [torch.float32, torch.float16])
def test_mx_gemm_parity(M, N, K, S, dtype):
    say(f"mx_gemm parity M={M} N={N} K={K} S={S} {dtype}")
    c = rand_case(M, K, N, S, seed=800 + M + N)
    ac, asc = MX.quantize_act(c["X"], c["perm"], S)
    wc, wsc = MX.pack_weight(c["W"], c["perm"], S)
    Yref = MX.gemm(ac, asc, wc, wsc)
    Y = B.arcq_mx_gemm(dev(ac), dev(asc), dev(wc), dev(wsc), out_dtype=dtype)
    torch.cuda.synchronize()
    err = norm_err(Y.float().cpu().numpy(), Yref)
    say(f"   normalised max error {err:.3e}")
    assert err <= (GEMM_TOL_F16 if dtype == torch.float16 else GEMM_TOL_F32)


@pytest.mark.parametrize("M,N,Kp", [(16, 1000, 1024), (64, 300, 4384), (300, 260, 1024), (2048, 3000, 256)])
def test_mx_gemm_operands_only_4_byte_aligned(M, N, Kp):
    """Codes 4 bytes off a 16-byte boundary and scale bytes at odd addresses: the least the interface asks for."""
    say(f"mx_gemm with 4-byte aligned operands M={M} N={N} K'={Kp}")
    rng = np.random.default_rng(M + N + Kp)
    ac = rng.integers(0, 256, (M, Kp // 2), dtype=np.uint8)
    wc = rng.integers(0, 256, (N, Kp // 2), dtype=np.uint8)
    asc = rng.integers(120, 134, (M, Kp // 32), dtype=np.uint8)
    wsc = rng.integers(120, 134, (N, Kp // 32), dtype=np.uint8)
    Yref = MX.gemm(ac, asc, wc, wsc)

    def shifted(a, by):
        buf = torch.zeros(a.size + 256, dtype=torch.uint8, device="cuda")
        start = (-buf.data_ptr()) % 16 + by
        view = buf[start:start + a.size].view(a.shape)
        view.copy_(torch.from_numpy(a))
        return view
    Y = B.arcq_mx_gemm(shifted(ac, 4), shifted(asc, 3), shifted(wc, 12), shifted(wsc, 1), out_dtype=torch.float32)
    torch.cuda.synchronize()
    err = norm_err(Y.cpu().numpy(), Yref)
    say(f"   normalised max error {err:.3e}")
    assert err <= GEMM_TOL_F32


def test_mx_gemm_extreme_scales():
    """Scale bytes from the ends of what fp16 data can produce, every code value, strided output with a guard."""
    say("mx_gemm extreme scales")
    rng = np.random.default_rng(3)
    M, N, Kp = 40, 72, 256
    ac = rng.integers(0, 256, (M, Kp // 2), dtype=np.uint8)
    wc = rng.integers(0, 256, (N, Kp // 2), dtype=np.uint8)
    asc = rng.choice(np.array([101, 102, 127, 139, 140], np.uint8), (M, Kp // 32))
    wsc = rng.choice(np.array([101, 110, 127, 130, 140], np.uint8), (N, Kp // 32))
    Yref = MX.gemm(ac, asc, wc, wsc)
    wide = torch.full((M, N + 8), 7.0, dtype=torch.float32, device="cuda")
    B.arcq_mx_gemm(dev(ac), dev(asc), dev(wc), dev(wsc), y=wide[:, :N])
    out = wide.cpu().numpy()
    assert norm_err(out[:, :N], Yref) <= GEMM_TOL_F32 and np.all(out[:, N:] == 7.0)


@pytest.mark.parametrize("M,N,Kp,dtype", [
    (300, 260, 512, torch.float32),       # 128 x 128 tiles
    (2048, 3072, 384, torch.float16),     # 128 x 256 tiles, a half unit at the end
    (4096, 4096, 256, torch.float16),     # 256 x 256 tiles
    (64, 4100, 1280, torch.float16),      # weight-streaming kernel: two groups of four chunks and two single chunks
])
def test_mx_gemm_extreme_scales_every_kernel(M, N, Kp, dtype):
    say(f"mx_gemm with extreme scale bytes M={M} N={N} K'={Kp} {dtype}")
    rng = np.random.default_rng(29)
    ac = rng.integers(0, 256, (M, Kp // 2), dtype=np.uint8)
    wc = rng.integers(0, 256, (N, Kp // 2), dtype=np.uint8)
    asc = rng.choice(np.array([101, 102, 127, 139, 140], np.uint8), (M, Kp // 32))
    wsc = rng.choice(np.array([101, 110, 118, 120], np.uint8), (N, Kp // 32))       # small, so fp16 outputs stay finite
    Y = B.arcq_mx_gemm(dev(ac), dev(asc), dev(wc), dev(wsc), out_dtype=dtype).float().cpu().numpy()
    assert np.all(np.isfinite(Y))
    rows = rng.choice(M, min(M, 64), replace=False)
    Yref = MX.gemm(ac[rows], asc[rows], wc, wsc)
    assert norm_err(Y[rows], Yref) <= (GEMM_TOL_F32 if dtype == torch.float32 else GEMM_TOL_F16)


def test_mx_full_size_llama8b_qproj():
    """The bench's MXFP4 workload at full size: quantizer bit-exact, GEMM on sampled rows."""
    say("mx path full size 2048 x 4096 x 4096, S = 256")
    c = wk.make_case(wk.WORKLOADS["c2_llama8b_q"])
    X, W, perm, S = c["X"], c["W"], c["perm"], c["S"]
    want_c, want_s = MX.quantize_act(X, perm, S)
    ac, asc = B.arcq_mx_quantize_act(dev(X), dev(perm), S)
    assert_same_bytes(asc.cpu().numpy(), want_s, "scales")
    assert_same_bytes(ac.cpu().numpy(), want_c, "codes")
    wc, wsc = B.arcq_mx_pack_weight(dev(W), dev(perm), S)
    owc, owsc = MX.pack_weight(W, perm, S)
    assert_same_bytes(wc.cpu().numpy(), owc, "weight codes")
    assert_same_bytes(wsc.cpu().numpy(), owsc, "weight scales")
    Y = B.arcq_mx_gemm(ac, asc, wc, wsc).float().cpu().numpy()
    rows = np.random.default_rng(1).choice(X.shape[0], 48, replace=False)
    Yref = MX.gemm(want_c[rows], want_s[rows], owc, owsc)
    assert norm_err(Y[rows], Yref) <= GEMM_TOL_F16


@pytest.mark.parametrize("name,k", [("arcq_probe_mfma_f16", 16), ("arcq_probe_mfma_fp4", 64)])
def test_matrix_rate_probe_runs_and_counts_its_work(name, k):
    say(name)
    sink = torch.full((B.PROBE_SINK_FLOATS,), float("nan"), dtype=torch.float32, device="cuda")
    flop = getattr(B, name)(3, sink)
    torch.cuda.synchronize()
    assert flop == 4096 * 3 * 4 * 2 * 32 * 32 * k
    out = sink.cpu().numpy()
    assert np.all(np.isfinite(out)) and np.any(out != 0)


@pytest.mark.parametrize("M,N,K", [(1, 8, 32), (77, 200, 96), (300, 260, 4096), (2048, 3072, 352), (4000, 4100, 128)])
def test_ref_gemm_bf16_against_fp64(M, N, K):
    """The bf16 comparison kernel (every tile configuration, ragged edges, a half unit at the end of K)."""
    say(f"ref_gemm_bf16 M={M} N={N} K={K}")
    g = torch.Generator().manual_seed(41 + M)
    x = torch.randn((M, K), generator=g).to(torch.bfloat16)
    w = (0.05 * torch.randn((N, K), generator=g)).to(torch.bfloat16)
    Y = B.arcq_ref_gemm_bf16(x.cuda(), w.cuda()).float().cpu().numpy()
    Yref = x.double().numpy() @ w.double().numpy().T
    assert norm_err(Y, Yref) <= GEMM_TOL_F16


@pytest.mark.parametrize("M,N,K,S", [(200, 260, 8192, 512), (130, 129, 4192, 32), (384, 1000, 6144, 0), (100, 300, 14336, 256),
                                     (200, 260, 8192, 544)])      # the last: an odd number of blocks, units through registers
@pytest.mark.parametrize("dtype", [torch.float32, torch.float16])
def test_mx_gemm_with_workspace_splits_the_reduction(M, N, K, S, dtype):
    """Few-tile problems with a long K' on arcq_mx_gemm_ws: 2 to 8 runs (the second ends with a half unit), against the
    oracle and against the plain entry point (same products, another order of the fp32 additions)."""
    say(f"mx_gemm_ws parity M={M} N={N} K={K} S={S} {dtype}")
    c = rand_case(M, K, N, S, seed=870 + M + N)
    ac, asc = MX.quantize_act(c["X"], c["perm"], S)
    wc, wsc = MX.pack_weight(c["W"], c["perm"], S)
    Yref = MX.gemm(ac, asc, wc, wsc)
    need = B.arcq_mx_gemm_workspace_size(M, N, K + S)
    assert need > 0 and need % (M * N * 4) == 0 and 2 <= need // (M * N * 4) <= 8
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    Y = B.arcq_mx_gemm(dev(ac), dev(asc), dev(wc), dev(wsc), out_dtype=dtype, workspace=ws)
    Y1 = B.arcq_mx_gemm(dev(ac), dev(asc), dev(wc), dev(wsc), out_dtype=dtype)
    torch.cuda.synchronize()
    tol = GEMM_TOL_F16 if dtype == torch.float16 else GEMM_TOL_F32
    assert norm_err(Y.float().cpu().numpy(), Yref) <= tol
    assert norm_err(Y.float().cpu().numpy(), Y1.float().cpu().numpy().astype(np.float64)) <= tol
    with pytest.raises(B.ArcqError):
        B.arcq_mx_gemm(dev(ac), dev(asc), dev(wc), dev(wsc), out_dtype=dtype, workspace=ws[: need - 256])


def test_mx_gemm_workspace_is_not_needed_where_nothing_splits():
    say("mx_gemm_ws where the plain kernels run")
    for M, N, Kp in ((16, 4096, 4352), (2048, 4096, 4352), (300, 260, 96), (64, 300, 8192)):
        assert B.arcq_mx_gemm_workspace_size(M, N, Kp) == 0
    c = rand_case(40, 256, 96, 32, seed=5)
    ac, asc = MX.quantize_act(c["X"], c["perm"], 32)
    wc, wsc = MX.pack_weight(c["W"], c["perm"], 32)
    a = B.arcq_mx_gemm(dev(ac), dev(asc), dev(wc), dev(wsc), workspace=torch.empty(0, dtype=torch.uint8, device="cuda"))
    b = B.arcq_mx_gemm(dev(ac), dev(asc), dev(wc), dev(wsc))
    assert torch.equal(a, b)
