"""Seeded synthetic inputs shaped like the paper's workloads.

The paper measures on Llama-3.1 / Qwen2.5 linear layers with activations
calibrated on WikiText2 (Section 4 "Experimental Setup", Appendix B); neither
models nor data are used here.  These generators stand in for them: Gaussian
activations with a small set of heavy outlier channels, Gaussian weights, a
channel permutation from a stable ascending sort of per-channel abs-max (the
calibration stand-in; Section 3.2 "Adaptive Outlier Identification") and an
FP32 tensor scale amax/(6*448).

This module holds no quantization arithmetic.  It is the only code that both
the GPU library's tests and the CPU oracle's tests draw inputs from.
"""
from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    M: int            # rows of X (tokens)
    K: int            # input channels
    N: int            # output features
    S: int            # augmented (outlier) channels, multiple of 16
    n_outlier: int    # channels that get a heavy scale factor
    outlier: str      # "const50" | "loguniform20_100" | "lognormal2"
    sigma_w: float
    seed: int


# seed = 0 (the paper fixes seed 0, Appendix C) + index of the configuration
WORKLOADS = {
    "c1_tiny":        Workload("c1_tiny", 16, 512, 512, 32, 8, "const50", 0.02, 1),
    "c2_llama8b_q":   Workload("c2_llama8b_q", 2048, 4096, 4096, 256, 41, "loguniform20_100", 0.02, 2),
    "c3a_llama8b_up": Workload("c3a_llama8b_up", 16, 4096, 14336, 256, 41, "loguniform20_100", 0.02, 3),
    "c3b_llama8b_down": Workload("c3b_llama8b_down", 16, 14336, 4096, 256, 143, "loguniform20_100", 0.02, 3),
    "c4_qwen32b_mlp": Workload("c4_qwen32b_mlp", 4096, 5120, 27648, 512, 26, "const50", 0.02, 4),
    "c5_llama70b_down": Workload("c5_llama70b_down", 8192, 28672, 8192, 1024, 287, "lognormal2", 0.01, 5),
}


def shrink(wl, **kw):
    """Same distribution and seed, smaller extents (for tests the oracle finishes quickly)."""
    return replace(wl, **kw)


def _channel_factors(wl, rng):
    f = np.ones(wl.K, dtype=np.float32)
    ch = rng.choice(wl.K, size=min(wl.n_outlier, wl.K), replace=False)
    if wl.outlier == "const50":
        f[ch] = 50.0
    elif wl.outlier == "loguniform20_100":
        f[ch] = np.exp(rng.uniform(np.log(20.0), np.log(100.0), size=ch.size)).astype(np.float32)
    elif wl.outlier == "lognormal2":
        f[ch] = np.minimum(np.exp(2.0 * rng.standard_normal(ch.size)), 1000.0).astype(np.float32)
    else:
        raise ValueError(wl.outlier)
    return f


def activations(wl, chunk_rows=1024):
    """X fp16 [M, K]: N(0,1) times a per-channel factor, clipped to the fp16 range."""
    rng_f = np.random.default_rng([wl.seed, 11])
    rng_x = np.random.default_rng([wl.seed, 12])
    f = _channel_factors(wl, rng_f)
    X = np.empty((wl.M, wl.K), dtype=np.float16)
    for r0 in range(0, wl.M, chunk_rows):
        r1 = min(wl.M, r0 + chunk_rows)
        blk = rng_x.standard_normal((r1 - r0, wl.K), dtype=np.float32) * f
        X[r0:r1] = np.clip(blk, -60000.0, 60000.0).astype(np.float16)
    return X


def weights(wl, chunk_rows=2048):
    """W fp16 [N, K] (the nn.Linear layout; Y = X W^T), N(0, sigma_w)."""
    rng_w = np.random.default_rng([wl.seed, 13])
    W = np.empty((wl.N, wl.K), dtype=np.float16)
    for r0 in range(0, wl.N, chunk_rows):
        r1 = min(wl.N, r0 + chunk_rows)
        W[r0:r1] = (rng_w.standard_normal((r1 - r0, wl.K), dtype=np.float32)
                    * np.float32(wl.sigma_w)).astype(np.float16)
    return W


def rmsnorm_gamma(wl):
    """RMSNorm weight fp16 [K] for the fused norm + quantizer: near 1 with a 10 % spread, and the
    few channels of trained models that carry a much larger or much smaller weight."""
    rng = np.random.default_rng([wl.seed, 14])
    g = 1.0 + 0.1 * rng.standard_normal(wl.K)
    n_odd = max(1, wl.K // 128)
    odd = rng.choice(wl.K, size=n_odd, replace=False)
    g[odd] *= rng.choice([0.05, 0.25, 4.0, 12.0], size=n_odd)
    return g.astype(np.float16)


def calibrate_perm(X):
    """Calibration stand-in: perm[j] = source channel placed at reordered position j,
    channels in ascending order of abs-max, ties by lower channel index first, so the
    outliers occupy the last positions."""
    colmax = np.abs(X).max(axis=0).astype(np.float32)
    return np.argsort(colmax, kind="stable").astype(np.int32)


def tensor_scale(T):
    """FP32 tensor scale that maps the largest block scale onto the E4M3 maximum:
    amax / (6 * 448); 1 for an all-zero tensor."""
    amax = np.float32(np.abs(T).max()) if T.size else np.float32(0)
    if amax == 0:
        return np.float32(1.0)
    return np.float32(amax / np.float32(2688.0))


def make_case(wl, with_weights=True):
    """dict(X, W, perm, S, sT_x, sT_w) for a workload."""
    X = activations(wl)
    case = {"wl": wl, "X": X, "perm": calibrate_perm(X), "S": wl.S, "sT_x": tensor_scale(X)}
    if with_weights:
        W = weights(wl)
        case["W"] = W
        case["sT_w"] = tensor_scale(W)
    return case
