"""Offline calibration of ARCQuant, step by step, in numpy.  Test infrastructure only.

Section 3.2 "Adaptive Outlier Identification": from calibration activations the method fixes,
per layer, the channel reordering and the number S of outlier channels:

  1. statistic: the absolute maximum of every channel over all calibration tokens;
  2. reorder channels by that statistic (the sorting strategy of Atom): here ascending, so that the
     outliers are the LAST positions, which is where the quantizer expects them;
  3. layer maximum Mx = max over channels; threshold tau = 2^-3 * Mx (the three bits of exponent
     width between an E5M2 reference and E2M1);
  4. a channel needs compensation when its statistic EXCEEDS tau (values with |x| <= tau are the
     range where NVFP4 is as precise as the reference); S counts those channels.

Readings where the paper is silent (listed in the design notes too):
  * ties in the sort keep the lower channel index first (a stable sort), so the result is unique;
  * S is rounded up to a whole number of 16-channel blocks (the quantizer and the GEMM work on
    blocks of 16) and capped at K; the extra channels are the largest ones below the threshold;
  * an all-zero layer has tau = 0 and S = 0.

All arithmetic is exact: abs and max of fp16 values, one multiplication by a power of two.
"""
import numpy as np

G = 16


def absmax_update(colmax, X):
    """colmax float32 [K] (running statistic, zeros before the first batch), X fp16 [M, K]:
    returns max(colmax, max over rows of |X|).  Batches may come in any order and split."""
    X = np.asarray(X)
    colmax = np.asarray(colmax)
    assert X.dtype == np.float16 and X.ndim == 2 and colmax.dtype == np.float32 and colmax.shape == (X.shape[1],)
    if not np.all(np.isfinite(X)):
        raise ValueError("non-finite input")
    if X.shape[0] == 0:
        return colmax.copy()
    return np.maximum(colmax, np.abs(X).max(axis=0).astype(np.float32))


def select_outliers(colmax):
    """colmax float32 [K], all >= 0 -> dict(perm int32 [K], S, S_raw, layer_max float32, tau float32).

    perm[j] = source channel placed at reordered position j."""
    colmax = np.asarray(colmax)
    assert colmax.dtype == np.float32 and colmax.ndim == 1
    K = colmax.shape[0]
    if K <= 0 or K % G:
        raise ValueError("need K > 0, K % 16 == 0")
    if not (np.all(np.isfinite(colmax)) and np.all(colmax >= 0)):
        raise ValueError("statistics must be finite and >= 0")
    perm = np.argsort(colmax, kind="stable").astype(np.int32)
    layer_max = np.float32(colmax.max())
    tau = np.float32(layer_max * np.float32(0.125))              # exact: a power of two
    S_raw = int(np.count_nonzero(colmax > tau))
    S = min(K, -(-S_raw // G) * G)
    return {"perm": perm, "S": S, "S_raw": S_raw, "layer_max": layer_max, "tau": tau}
