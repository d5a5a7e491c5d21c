"""arcq_gemm_noalloc (the entry point for callers that cannot allocate a workspace) against arcq_gemm:
same kernels, so the same bits, on two calls in a row that both split K' and share the library's built-in
scratch, the second on a smaller problem; also against the oracle, and on a shape that needs no scratch."""
import numpy as np
import pytest
import torch

from oracle import arcquant as A
from paper_2601_07475_amd import binding as B
from paper_2601_07475_amd import workloads as wk

pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def packed_case(M, N, K, S, seed):
    c = wk.make_case(wk.Workload("t", M, K, N, S, max(1, K // 100), "loguniform20_100", 0.02, seed))
    ac, asc = A.quantize_act(c["X"], c["perm"], S, c["sT_x"])
    wc, wsc = A.pack_weight(c["W"], c["perm"], S, c["sT_w"])
    return (ac, asc, c["sT_x"], wc, wsc, c["sT_w"]), A.gemm(ac, asc, c["sT_x"], wc, wsc, c["sT_w"])


def norm_err(Y, Yref):
    rms = np.sqrt(np.mean(Yref ** 2))
    return float(np.max(np.abs(np.asarray(Y, dtype=np.float64) - Yref) / np.maximum(np.abs(Yref), max(rms, 1e-300))))


@pytest.mark.parametrize("dtype,tol", [(torch.float32, 2e-5), (torch.float16, 1e-3)])
def test_noalloc_gemm_equals_gemm_on_two_calls_in_a_row(dtype, tol):
    # (M, N, K, S): 8 runs of K', then a smaller problem with 2 runs, then one without a split (no scratch)
    shapes = [(256, 512, 14336, 256), (130, 129, 2048, 64), (16, 512, 512, 32)]
    cases = [packed_case(M, N, K, S, seed=40 + i) for i, (M, N, K, S) in enumerate(shapes)]
    needs = [B.arcq_gemm_workspace_size(M, N, K + S) for M, N, K, S in shapes]
    assert needs[0] > needs[1] > 0 and needs[2] == 0 and needs[0] <= B.NOALLOC_SCRATCH_BYTES
    ops = [[dev(t) if isinstance(t, np.ndarray) else t for t in ops] for ops, _ in cases]
    outs = [torch.full((M, N), float("nan"), dtype=dtype, device="cuda") for M, N, _, _ in shapes]
    want = [B.arcq_gemm(*o, out_dtype=dtype) for o in ops]          # the existing entry point, caller's workspace
    torch.cuda.synchronize()
    for o, y, (M, N, K, S) in zip(ops, outs, shapes):               # back to back on one stream, no sync between
        print(f"arcq_gemm_noalloc M={M} N={N} K'={K + S} {dtype}", flush=True)
        B.arcq_gemm_noalloc(*o, y)
    torch.cuda.synchronize()
    for y, w, (_, yref) in zip(outs, want, cases):
        assert torch.equal(y, w)
        assert norm_err(y.float().cpu().numpy(), yref) <= tol
    # and once more in the opposite order (the scratch now holds the small problem's partial results)
    for o, y in zip(ops[1::-1], outs[1::-1]):
        y.fill_(float("nan"))
        B.arcq_gemm_noalloc(*o, y)
    torch.cuda.synchronize()
    for y, w in zip(outs, want):
        assert torch.equal(y, w)
