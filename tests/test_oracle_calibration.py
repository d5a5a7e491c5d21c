"""Pins of oracle.calibration (Section 3.2 "Adaptive Outlier Identification") against closed forms,
a second implementation built on Python's own sort, and the properties that define the result."""
import numpy as np
import pytest

from oracle import calibration as C
from paper_2601_07475_amd import workloads as wk


def brute_select(colmax):
    """Second implementation: Python's sort on (value, index) tuples, counting loop, exact fractions."""
    from fractions import Fraction as Fr
    vals = [Fr(float(v)) for v in colmax]
    order = [i for _, i in sorted((v, i) for i, v in enumerate(vals))]
    mx = max(vals)
    tau = mx / 8
    s_raw = sum(1 for v in vals if v > tau)
    K = len(vals)
    S = min(K, (s_raw + 15) // 16 * 16)
    return order, S, s_raw, mx, tau


def test_closed_forms():
    K = 64
    # distinct ascending statistics: identity permutation; threshold 63/8 = 7.875 -> channels 8..63 exceed it
    r = C.select_outliers(np.arange(K, dtype=np.float32))
    assert np.array_equal(r["perm"], np.arange(K)) and r["layer_max"] == 63 and r["tau"] == np.float32(7.875)
    assert r["S_raw"] == 56 and r["S"] == 64
    # descending: reversed
    r = C.select_outliers(np.arange(K, dtype=np.float32)[::-1].copy())
    assert np.array_equal(r["perm"], np.arange(K)[::-1])
    # one outlier channel far above the rest: S_raw = 1, S = one block
    cm = np.ones(K, np.float32)
    cm[37] = 100.0
    r = C.select_outliers(cm)
    assert r["S_raw"] == 1 and r["S"] == 16 and r["perm"][-1] == 37
    assert np.array_equal(r["perm"][:-1], [i for i in range(K) if i != 37])      # ties keep channel order
    # a channel exactly AT the threshold needs no compensation (|x| <= tau)
    cm = np.full(K, 1.0, np.float32)
    cm[5] = 8.0
    cm[9] = 1.0                                                                   # tau = 1: only channel 5 exceeds
    assert C.select_outliers(cm)["S_raw"] == 1
    cm[9] = np.nextafter(np.float32(1.0), np.float32(2.0))
    assert C.select_outliers(cm)["S_raw"] == 2
    # all equal (> 0): every channel exceeds max/8 -> S = K; all zero -> S = 0, identity order
    assert C.select_outliers(np.full(K, 3.0, np.float32))["S"] == K
    r = C.select_outliers(np.zeros(K, np.float32))
    assert r["S"] == 0 and r["S_raw"] == 0 and r["tau"] == 0 and np.array_equal(r["perm"], np.arange(K))
    for bad in (np.array([1.0] * 15, np.float32), np.array([-1.0] * 16, np.float32), np.array([np.inf] * 16, np.float32)):
        with pytest.raises(ValueError):
            C.select_outliers(bad)


@pytest.mark.parametrize("seed,K", [(0, 16), (1, 48), (2, 256), (3, 1040)])
def test_against_python_sort_and_defining_properties(seed, K):
    rng = np.random.default_rng(seed)
    # fp16-valued statistics with many ties and a heavy tail
    cm = np.abs(rng.standard_normal(K) * np.exp(rng.standard_normal(K) * 2)).astype(np.float16)
    cm[rng.integers(0, K, K // 4)] = cm[rng.integers(0, K, K // 4)]
    cm = cm.astype(np.float32)
    r = C.select_outliers(cm)
    order, S, s_raw, mx, tau = brute_select(cm)
    assert r["perm"].tolist() == order and r["S"] == S and r["S_raw"] == s_raw
    assert float(r["layer_max"]) == float(mx) and float(r["tau"]) == float(tau)
    p = r["perm"]
    assert sorted(p.tolist()) == list(range(K))                                   # a permutation
    keys = cm[p]
    assert np.all(keys[1:] >= keys[:-1])                                          # ascending
    same = keys[1:] == keys[:-1]
    assert np.all(p[1:][same] > p[:-1][same])                                     # ties by channel index
    assert r["S"] % 16 == 0 and r["S"] >= r["S_raw"] and r["S"] - r["S_raw"] < 16
    if r["S_raw"]:
        assert np.all(keys[K - r["S_raw"]:] > r["tau"])                           # exactly the last S_raw positions
    assert np.all(keys[:K - r["S_raw"]] <= r["tau"])


def test_absmax_update_is_a_running_maximum():
    rng = np.random.default_rng(7)
    X = (rng.standard_normal((100, 64)) * 5).astype(np.float16)
    X[17, 3] = np.float16(-60000.0)
    X[5, 9] = np.float16(-0.0)
    zero = np.zeros(64, np.float32)
    whole = C.absmax_update(zero, X)
    assert whole[3] == 60000.0 and whole.dtype == np.float32
    assert np.array_equal(whole, np.array([max(abs(float(v)) for v in X[:, k]) for k in range(64)], np.float32))
    # any split into batches, in any order, gives the same statistic
    parts = [X[60:], X[:10], X[10:60], X[:0]]
    acc = zero
    for part in parts:
        acc = C.absmax_update(acc, part)
    assert np.array_equal(acc, whole)
    assert np.array_equal(C.absmax_update(whole, X), whole)                       # idempotent
    with pytest.raises(ValueError):
        C.absmax_update(zero, np.full((2, 64), np.inf, np.float16))


def test_agrees_with_the_workload_generator_stand_in():
    """The synthetic workloads order their channels with the same rule; the oracle adds S."""
    wl = wk.shrink(wk.WORKLOADS["c2_llama8b_q"], M=64)
    X = wk.activations(wl)
    r = C.select_outliers(C.absmax_update(np.zeros(wl.K, np.float32), X))
    assert np.array_equal(r["perm"], wk.calibrate_perm(X))
