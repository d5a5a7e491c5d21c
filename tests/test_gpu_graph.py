"""The library's launches under HIP graph capture: every entry point of the online path only enqueues kernels on
the caller's stream (no allocation, no synchronisation, no memset node), so a captured step must replay with the
same bytes an eager call produces, on every replay and with new input contents between replays."""
import numpy as np
import pytest
import torch

from paper_2601_07475_amd import binding as B

from test_gpu_parity import dev, norm_case, rand_case, say

pytestmark = pytest.mark.gpu


def _replays_match(capture, eager, outputs, refresh):
    """capture(): enqueues the step on the current (capturing) stream; eager(): the same step with plain calls;
    outputs: the tensors the step writes; refresh(i): new input contents before replay i."""
    eager()                                  # first-call set-up of every kernel happens outside the capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        capture()
    for i in range(4):
        refresh(i)
        for t in outputs:
            t.fill_(0x5A if t.dtype == torch.uint8 else 7.0)
        g.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in outputs]
        for t in outputs:
            t.fill_(0x5A if t.dtype == torch.uint8 else 7.0)
        eager()                              # the program's own eager work between the replays
        torch.cuda.synchronize()
        for a, b in zip(got, outputs):
            assert torch.equal(a, b), f"replay {i} differs from the eager result"


# M, K, N, S: the pair kernel's tile shape (ragged), the weight-streaming kernel, split K with a workspace
@pytest.mark.parametrize("M,K,N,S", [(1000, 896, 6100, 128), (16, 4096, 1024, 256), (200, 4096, 256, 256)])
def test_nvfp4_step_replays_bit_identically(M, K, N, S):
    say(f"graph capture of quantize_act + gemm M={M} K={K} N={N} S={S}")
    c = rand_case(M, K, N, S, seed=61)
    inputs = [dev(rand_case(M, K, N, S, seed=62 + i)["X"]) for i in range(4)]
    X, perm = dev(c["X"]), dev(c["perm"])
    sTx, sTw = float(c["sT_x"]), float(c["sT_w"])
    wc, wsc = B.arcq_pack_weight(dev(c["W"]), perm, S, sTw)
    Kp = K + S
    ac = torch.empty((M, Kp // 2), dtype=torch.uint8, device="cuda")
    asc = torch.empty((M, Kp // 16), dtype=torch.uint8, device="cuda")
    Y = torch.empty((M, N), dtype=torch.float16, device="cuda")
    ws = torch.empty(max(B.arcq_gemm_workspace_size(M, N, Kp), 1), dtype=torch.uint8, device="cuda")

    def eager():
        B.arcq_quantize_act(X, perm, S, sTx, codes=ac, scales=asc)
        B.arcq_gemm(ac, asc, sTx, wc, wsc, sTw, y=Y, workspace=ws)

    def capture():                           # prepared calls bind the stream that is current here: the capturing one
        B.prepare_quantize_act(X, perm, S, sTx, ac, asc)()
        B.prepare_gemm(ac, asc, sTx, wc, wsc, sTw, Y, ws)()

    _replays_match(capture, eager, [ac, asc, Y], lambda i: X.copy_(inputs[i]))


def test_rmsnorm_and_mxfp4_steps_replay_bit_identically():
    say("graph capture of rmsnorm_quantize_act + gemm and of the MXFP4 step")
    M, K, N, S = 130, 8192, 512, 128         # long enough for the MXFP4 GEMM to split K' when given a workspace
    Xn, gamma, perm_n, sT = norm_case(M, K, S, seed=71)
    c = rand_case(M, K, N, S, seed=72)
    inputs = [dev(norm_case(M, K, S, seed=73 + i)[0]) for i in range(4)]
    X, g_, perm = dev(Xn), dev(gamma), dev(perm_n)
    sT, sTw = float(sT), float(c["sT_w"])
    W = dev(c["W"])
    wc, wsc = B.arcq_pack_weight(W, perm, S, sTw)
    mwc, mwsc = B.arcq_mx_pack_weight(W, perm, S)
    Kp = K + S
    ac = torch.empty((M, Kp // 2), dtype=torch.uint8, device="cuda")
    asc = torch.empty((M, Kp // 16), dtype=torch.uint8, device="cuda")
    mac = torch.empty((M, Kp // 2), dtype=torch.uint8, device="cuda")
    masc = torch.empty((M, Kp // 32), dtype=torch.uint8, device="cuda")
    Y = torch.empty((M, N), dtype=torch.float16, device="cuda")
    Ym = torch.empty((M, N), dtype=torch.float32, device="cuda")
    ws = torch.empty(max(B.arcq_gemm_workspace_size(M, N, Kp), 1), dtype=torch.uint8, device="cuda")
    assert B.arcq_mx_gemm_workspace_size(M, N, Kp) > 0
    mws = torch.empty(B.arcq_mx_gemm_workspace_size(M, N, Kp), dtype=torch.uint8, device="cuda")

    def eager():
        B.arcq_rmsnorm_quantize_act(X, g_, 1e-5, perm, S, sT, codes=ac, scales=asc)
        B.arcq_gemm(ac, asc, sT, wc, wsc, sTw, y=Y, workspace=ws)
        B.arcq_mx_quantize_act(X, perm, S, codes=mac, scales=masc)
        B.arcq_mx_gemm(mac, masc, mwc, mwsc, y=Ym, workspace=mws)

    def capture():
        B.prepare_rmsnorm_quantize_act(X, g_, 1e-5, perm, S, sT, ac, asc)()
        B.prepare_gemm(ac, asc, sT, wc, wsc, sTw, Y, ws)()
        B.prepare_mx_quantize_act(X, perm, S, mac, masc)()
        B.prepare_mx_gemm(mac, masc, mwc, mwsc, Ym, mws)()

    _replays_match(capture, eager, [ac, asc, Y, mac, masc, Ym], lambda i: X.copy_(inputs[i]))
