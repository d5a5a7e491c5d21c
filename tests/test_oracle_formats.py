"""Pins for oracle.formats: table definitions, ties, saturation, a library fp8 cast, brute force."""
import os
from fractions import Fraction as Fr

import numpy as np
import pytest
import torch

from oracle import brute
from oracle import formats as F

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "nvfp4_format_constants.txt")


def golden():
    out = {}
    with open(GOLDEN) as fh:
        for line in fh:
            line = line.split("#")[0].split()
            if len(line) == 2:
                out[line[0]] = float(line[1])
    return out


def test_e2m1_grid_is_the_printed_format():
    g = golden()
    # bias-1, 2 exponent bits, 1 mantissa bit: the eight magnitudes, typed here by hand
    assert F.E2M1_GRID.tolist() == [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]
    assert F.E2M1_GRID.max() == g["e2m1_max"]
    # bias: exponent field 1 with mantissa 0 is 2^(1-bias) = 1
    assert F.e2m1_decode(0b0010) == 2.0 ** (1 - g["e2m1_bias"])
    assert np.signbit(F.e2m1_decode(8)) and F.e2m1_decode(8) == 0.0
    assert F.e2m1_decode(np.arange(8, 16)).tolist() == [-0.0, -0.5, -1.0, -1.5, -2.0, -3.0, -4.0, -6.0]


def test_e2m1_roundtrip_and_monotone():
    idx = F.e2m1_encode_magnitude(F.E2M1_GRID)
    assert idx.tolist() == list(range(8))
    w = np.linspace(0, 8, 4001)
    assert np.all(np.diff(F.e2m1_encode_magnitude(w).astype(int)) >= 0)


def test_e2m1_ties_to_even_and_neighbours():
    mids = {0.25: 0, 0.75: 2, 1.25: 2, 1.75: 4, 2.5: 4, 3.5: 6, 5.0: 6}
    for w, want in mids.items():
        assert F.e2m1_encode_magnitude(np.float32(w)) == want, w
        lo = np.nextafter(np.float32(w), np.float32(0))
        hi = np.nextafter(np.float32(w), np.float32(10))
        below = max(i for i in range(8) if F.E2M1_GRID[i] < w)
        assert F.e2m1_encode_magnitude(lo) == below
        assert F.e2m1_encode_magnitude(hi) == below + 1


def test_e2m1_saturates():
    assert F.e2m1_encode_magnitude(np.float32([6.0, 6.0001, 6.375, 7.0, 1e30])).tolist() == [7] * 5
    with pytest.raises(ValueError):
        F.e2m1_encode_magnitude(np.float32([-1.0]))
    with pytest.raises(ValueError):
        F.e2m1_encode_magnitude(np.float32([np.nan]))


def test_e2m1_against_brute_force_over_all_fp16():
    # every non-negative finite fp16 value, scaled by a few reciprocal scales in fp32
    h = np.arange(0, 0x7C00, dtype=np.uint16).view(np.float16).astype(np.float32)
    for inv in (np.float32(1.0), np.float32(1 / 3.0), np.float32(7.3), np.float32(2.0 ** -9 * 1.1)):
        w = np.minimum(h * inv, np.float32(6.0))
        w = np.unique(w)
        got = F.e2m1_encode_magnitude(w)
        step = max(1, len(w) // 6000)       # Fractions are slow: a dense subsample plus all near-tie values
        near = np.abs(w[:, None] - np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0])).min(axis=1) < 1e-3
        sel = np.zeros(len(w), bool)
        sel[::step] = True
        sel |= near
        for wi, gi in zip(w[sel], got[sel]):
            assert brute.e2m1_nearest(Fr(float(wi))) == gi, wi


def test_e4m3_decode_all_bytes_against_library_cast():
    g = golden()
    b = torch.arange(256, dtype=torch.int32).to(torch.uint8)
    lib = b.view(torch.float8_e4m3fn).to(torch.float64).numpy()
    ours = F.e4m3_decode(b.numpy())
    assert np.array_equal(np.isnan(lib), np.isnan(ours))
    ok = ~np.isnan(lib)
    assert np.array_equal(lib[ok], ours[ok])
    assert np.array_equal(np.signbit(lib[ok]), np.signbit(ours[ok]))
    assert np.nanmax(ours) == g["e4m3_max"]
    assert F.e4m3_decode(0b0_0111_000) == 1.0            # exponent field == bias
    assert int(np.log2(F.e4m3_decode(0b0_0001_000))) == 1 - int(g["e4m3_bias"])
    assert F.e4m3_decode(1) == 2.0 ** -9                  # smallest subnormal


def test_e4m3_encode_roundtrip_ties_saturation():
    allb = np.arange(0x7F, dtype=np.uint8)
    vals = F.e4m3_decode(allb)
    assert np.array_equal(F.e4m3_encode_rne_sat(vals), allb)
    mids = (vals[:-1] + vals[1:]) / 2                      # exact in fp64
    want = np.where(allb[:-1] % 2 == 0, allb[:-1], allb[1:])
    assert np.array_equal(F.e4m3_encode_rne_sat(mids), want)
    assert np.array_equal(F.e4m3_encode_rne_sat(np.nextafter(mids, 0)), allb[:-1])
    assert np.array_equal(F.e4m3_encode_rne_sat(np.nextafter(mids, 1e9)), allb[1:])
    assert F.e4m3_encode_rne_sat(np.array([448.0, 449.0, 464.0, 465.0, 1e9, 3e38])).tolist() == [0x7E] * 6
    assert F.e4m3_encode_rne_sat(np.array([0.0, 2.0 ** -11, 2.0 ** -10, 2.0 ** -10 * 1.01])).tolist() == [0, 0, 0, 1]


def test_e4m3_encode_against_library_cast():
    rng = np.random.default_rng(3)
    u = np.concatenate([
        rng.uniform(0, 448, 20000), np.exp(rng.uniform(np.log(1e-4), np.log(448), 20000)),
        np.arange(0, 0x5F00, dtype=np.uint16).view(np.float16).astype(np.float64),   # every fp16 in [0, 448]
    ]).astype(np.float32)
    u = u[u <= 448]
    lib = torch.from_numpy(u).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(F.e4m3_encode_rne_sat(u), lib)


def test_e4m3_against_brute_force():
    rng = np.random.default_rng(4)
    u = np.exp(rng.uniform(np.log(2.0 ** -12), np.log(600.0), 1500)).astype(np.float32)
    got = F.e4m3_encode_rne_sat(u)
    for ui, gi in zip(u, got):
        assert brute.e4m3_nearest_sat(Fr(float(ui))) == gi


def test_brute_round_f32_matches_ieee():
    rng = np.random.default_rng(5)
    a = rng.standard_normal(400).astype(np.float32) * np.float32(1e-3)
    b = np.exp(rng.uniform(-60, 20, 400)).astype(np.float32)
    for x, y in zip(a, b):
        assert float(brute.round_f32(Fr(float(x)) * Fr(float(y)))) == float(np.float32(x) * np.float32(y))
        assert float(brute.round_f32(Fr(float(x)) / Fr(float(y)))) == float(np.float32(x) / np.float32(y))
    tiny = np.float32(2.0 ** -140)
    assert float(brute.round_f32(Fr(float(tiny)) * Fr(3, 8))) == float(tiny * np.float32(0.375))
