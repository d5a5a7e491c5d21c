"""Pins of oracle.mxfp4 (the MXFP4 variant of the path): format tables against a library, the scale rule against its
defining inequalities and an exact-rational second implementation, and the identities of Section 3.2."""
from fractions import Fraction as Fr

import numpy as np
import pytest
import torch

from oracle import brute
from oracle import mxfp4 as MX
from paper_2601_07475_amd import workloads as wk


def test_e8m0_table_against_the_library_type():
    b = np.arange(256, dtype=np.uint8)
    lib = torch.from_numpy(b).view(torch.float8_e8m0fnu).to(torch.float32).numpy().astype(np.float64)
    mine = MX.e8m0_decode(b)
    assert np.isnan(mine[255]) and np.isnan(lib[255])
    assert np.array_equal(mine[1:255], lib[1:255])              # byte 0 is 2^-127: subnormal in the library's fp32
    assert mine[127] == 1.0 and mine[0] == 2.0 ** -127 and mine[254] == 2.0 ** 127


def brute_block(v):
    """Exact rationals: shared exponent from the integer bit length, nearest grid value by search, ties to even."""
    vals = [Fr(float(x)) for x in v]
    amax = max(abs(x) for x in vals)
    if amax == 0:
        return 127, [8 if np.signbit(x) else 0 for x in v], [Fr(0)] * len(vals)
    e = amax.numerator.bit_length() - amax.denominator.bit_length()
    if Fr(2) ** e > amax:
        e -= 1
    assert Fr(2) ** e <= amax < Fr(2) ** (e + 1)
    shared = e - 2
    X = Fr(2) ** shared
    codes, res = [], []
    for x, raw in zip(vals, v):
        idx = brute.e2m1_nearest(min(abs(x) / X, Fr(6)))
        code = (8 if np.signbit(raw) else 0) | idx
        codes.append(code)
        res.append(x - brute.e2m1_value(code) * X)
    return shared + 127, codes, res


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_block_recipe_against_exact_rationals(seed):
    rng = np.random.default_rng(seed)
    blocks = (rng.standard_normal((40, 32)) * np.exp(rng.standard_normal((40, 1)) * 3)).astype(np.float16)
    blocks[0] = 0
    blocks[1, ::2] = np.float16(-0.0)
    blocks[2] = np.float16(2.0 ** -24)                       # smallest subnormal
    blocks[3, :8] = np.float16([6, 7, 7.99, 5, -6.5, 4, 3.5, 2.5])   # clipping above 6 X and ties
    blocks[3, 8:] = 0
    blocks[4] = np.float16(65504.0)
    v = blocks.astype(np.float32)
    sb, codes, X = MX.quantize_blocks(v)
    r = MX.residual_blocks(v, codes, X)
    for i in range(len(v)):
        b_sb, b_codes, b_res = brute_block(v[i])
        assert sb[i] == b_sb and codes[i].tolist() == b_codes
        assert [Fr(float(t)) for t in r[i]] == b_res


def test_scale_rule_inequalities_and_error_bound():
    rng = np.random.default_rng(5)
    v = (rng.standard_normal((500, 32)) * np.exp(rng.standard_normal((500, 1)) * 3)).astype(np.float16).astype(np.float32)
    sb, codes, X = MX.quantize_blocks(v)
    amax = np.abs(v).max(axis=-1)
    assert np.all(amax / X >= 4) and np.all(amax / X < 8)       # floor(log2 amax) = shared + 2
    deq = MX.F.e2m1_decode(codes) * X[:, None]
    err = np.abs(v - deq)
    inside = np.abs(v) <= 6 * X[:, None]
    step = np.where(np.abs(deq) >= 4 * X[:, None], 2.0, np.where(np.abs(deq) >= 2 * X[:, None], 1.0, 0.5)) * X[:, None]
    assert np.all(err[inside] <= step[inside] / 2 + 1e-30)     # half a grid step where nothing clips
    assert np.all(err[~inside] < 2 * X.repeat(32).reshape(-1, 32)[~inside])   # clipped values lose less than 2 X
    # the second stage shrinks the error of every block
    r = MX.residual_blocks(v, codes, X)
    _, c2, X2 = MX.quantize_blocks(r)
    err2 = np.abs(r - MX.F.e2m1_decode(c2) * X2[:, None])
    assert np.all(err2.max(axis=1) <= err.max(axis=1)) and err2.max(axis=1).mean() < 0.3 * err.max(axis=1).mean()


def test_path_identities():
    wl = wk.Workload("t", 24, 256, 40, 64, 3, "const50", 0.02, 9)
    c = wk.make_case(wl)
    X, W, perm, S = c["X"], c["W"], c["perm"], 64
    ac, asc = MX.quantize_act(X, perm, S)
    wc, wsc = MX.pack_weight(W, perm, S)
    assert ac.shape == (24, 160) and asc.shape == (24, 10) and wc.shape == (40, 160) and wsc.shape == (40, 10)
    # S = 0 is plain per-block MXFP4 and equals the primary part
    a0, s0 = MX.quantize_act(X, perm, 0)
    assert np.array_equal(a0, ac[:, :128]) and np.array_equal(s0, asc[:, :8])
    # weights: verbatim copy of the outlier blocks
    assert np.array_equal(wc[:, 128:], wc[:, 96:128]) and np.array_equal(wsc[:, 8:], wsc[:, 6:8])
    # eq. (2): the K'-wide product is Q(X) Q(W)^T + Q(R_o) Q(W_o)^T
    Y = MX.gemm(ac, asc, wc, wsc)
    Y0 = MX.gemm(a0, s0, wc[:, :128], wsc[:, :8])
    Yr = MX.gemm(ac[:, 128:], asc[:, 8:], wc[:, 96:128], wsc[:, 6:8])
    assert np.allclose(Y, Y0 + Yr, rtol=1e-13, atol=1e-13)
    # and it is closer to X deq(W)^T than the product without the augmentation
    ref = X[:, perm].astype(np.float64) @ MX.dequantize(wc[:, :128], wsc[:, :8]).T
    assert np.abs(Y - ref).mean() < 0.5 * np.abs(Y0 - ref).mean()
    # primary + residual reconstruct the outlier channels better than the primary alone, exactly by the residual's own error
    A = MX.dequantize(ac, asc)
    Xo = X[:, perm][:, 192:].astype(np.float64)
    assert np.abs(A[:, 192:256] + A[:, 256:] - Xo).max() < np.abs(A[:, 192:256] - Xo).max()
    for bad_S in (16, 288):
        with pytest.raises(ValueError):
            MX.quantize_act(X, perm, bad_S)
