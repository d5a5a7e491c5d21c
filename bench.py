#!/usr/bin/env python3
"""Benchmark of the ARCQuant hot path on one MI355X.

A step is one pass of the whole online path over one batch of synthetic input already resident
in HBM: arcq_quantize_act (fused reorder + NVFP4 + residual channels) followed by arcq_gemm over
K' = K + S.  Weights are packed once, offline, outside the timed region (Section 3.2 "Offline
Weight Quantization").  The default workload is the LLaMA-3-8B q_proj prefill shape
(M=2048, K=4096, N=4096, S=256).

The timed region holds exactly --steps steps and nothing else on the stream (two events bracket it).  The
per-kernel launch durations of the rooflines come from loops of the same launch, back to back, between two events
(`detail.gemm_loop_ms`, `detail.quant_loop_ms`); the steps are also repeated (at most 200 of them) with an event
after every launch (`detail.gemm_ms`, `detail.quant_ms`), which shows the kernels in the order of the step but adds
2-5 us of event overhead to each, so those figures are upper bounds and stay out of `value` and the rooflines.  The defaults (2000 steps after 300 untimed ones, 0.2 s in all) are long on purpose: for the first
fifty to a hundred steps after the matrix load sets in this GPU's clock management makes the same GEMM up
to 20 % slower than it runs from then on, and a 50-step region measures mostly that transient.  Every other
figure comes from a loop sized the same way (`sustained_ms`: some 20 ms untimed, then some 40 ms timed).
`detail.rmsnorm_quant_ms` (the quantizer with RMSNorm fused in front) and `detail.mxfp4` (the same step
in the MXFP4 variant of the format, whose GEMM runs on the scaled FP4 matrix instruction) are reported
beside the headline figures and do not enter `value`.

Prints ONE JSON line.  `value` = 2*M*N*K' / step time, in TFLOP/s.  `roofline` prices the dominant
kernel (the GEMM; fp16 MFMA peak because operands are decoded exactly to fp16).  `cpu_baseline`
is the numpy oracle timed on the host cores on the same workload.  `detail.vendor_bf16_gemm_ms` and
`detail.hand_bf16_gemm_ms` time the unquantized bf16 linear layer over K (the vendor library through torch.matmul, and
this library's own bf16 kernel arcq_ref_gemm_bf16): the 16-bit baselines of `linear_vs_*` (> 1: the quantized step is faster).  `also` holds the other
single-GPU workloads (loop lengths from their own step time): the HBM-streaming claim of the quantizer is made on
c5_llama70b_down, the decode shapes c3a/c3b are weight-streaming bound (their `gemm_rotating_ms` cycles
over enough weight copies to exceed the last-level cache, so every launch streams its weight from HBM).
`s_sweep` times quantizer and GEMM against S at the main workload's shape (Section 3.4: cost linear in
S/K); `machine` holds what the box itself reaches: the plain copy rate and the register-only fp16 matrix
instruction rates (arcq_probe_mfma_f16, arcq_probe_mfma_fp4).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
PEAK_MFMA_F16_TFLOPS = 2500.0  # MI355X dense fp16/bf16 MFMA
PEAK_MFMA_FP4_TFLOPS = 10100.0 # MI355X dense fp4 MFMA (the MXFP4 variant's GEMM)

# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this script (see
# profiles/), scaled by the factor the same counters read for a plain copy of known size.
# workload -> kernel -> bytes; None where not measured.
MEASURED_TRAFFIC = {
    "c2_llama8b_q": {"arcq_gemm": 57350812, "arcq_quantize_act": 22006789, "arcq_rmsnorm_quantize_act": 22096896, "arcq_mx_quantize_act": 21727232, "arcq_mx_gemm": 54907910},
    "c4_qwen32b_mlp": {"arcq_gemm": 779865347, "arcq_quantize_act": 55168145, "arcq_rmsnorm_quantize_act": 55242134, "arcq_mx_quantize_act": 54472568, "arcq_mx_gemm": 735300181},
    "c5_llama70b_down": {"arcq_gemm": 1782181517, "arcq_quantize_act": 621149182, "arcq_rmsnorm_quantize_act": 622470456, "arcq_mx_quantize_act": 612794081, "arcq_mx_gemm": 1694914656},
    "c3a_llama8b_up": {"arcq_gemm": 36275510, "arcq_quantize_act": 353792, "arcq_rmsnorm_quantize_act": 443904, "arcq_mx_quantize_act": 334336, "arcq_mx_gemm": 34061503},
    "c3b_llama8b_down": {"arcq_gemm": 35078642, "arcq_quantize_act": 1101312, "arcq_rmsnorm_quantize_act": 1355264, "arcq_mx_quantize_act": 1076736, "arcq_mx_gemm": 32992742},
}


def quantizer_bytes(M, K, S):
    """Algorithmic HBM bytes of one quantizer launch: fp16 row in, codes and scale bytes out
    (2K + 9K'/16 per row); the permutation (4K bytes) is read once and stays cached."""
    Kp = K + S
    return M * (2 * K + Kp // 2 + Kp // 16)


def gemm_flops(M, N, Kp):
    return 2.0 * M * N * Kp


def gemm_bytes(M, N, Kp, out_bytes=2):
    """Algorithmic bytes of one GEMM launch: both packed operands once, the output once."""
    return (M + N) * (Kp // 2 + Kp // 16) + M * N * out_bytes


def sustained_ms(torch, fn, n=None, warm=None, target_ms=40.0, warm_ms=20.0):
    """Average time of fn() in a loop of back-to-back launches bracketed by two events on the current stream.
    Without n / warm the loop lengths come from a three-call estimate: about warm_ms of untimed calls first,
    then about target_ms of timed ones.  Short loops measure the clock transient of this GPU instead of the
    kernel: for some tens of launches after a matrix-heavy load sets in the same GEMM runs up to 20 % slower
    than it does a few milliseconds later, and idle gaps of a few microseconds let it run faster than it
    can when launched back to back."""
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    if n is None or warm is None:
        fn()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(3):
            fn()
        e1.record()
        torch.cuda.synchronize()
        est = max(e0.elapsed_time(e1) / 3, 1e-3)
        n = int(min(max(target_ms / est, 10), 4000)) if n is None else n
        warm = int(min(max(warm_ms / est, 3), 2000)) if warm is None else warm
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    e0.record()
    for _ in range(n):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / n


def measure(torch, B, case, steps, warmup, vendor_ref=True):
    """Runs warmup + steps of (quantize_act, gemm) on the current stream; per-kernel times come
    from events recorded on that same stream around each launch inside the timed region."""
    import numpy as np
    wl = case["wl"]
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    X, W, perm = d(case["X"]), d(case["W"]), d(case["perm"])
    S, sTx, sTw = case["S"], float(case["sT_x"]), float(case["sT_w"])
    wc, wsc = B.arcq_pack_weight(W, perm, S, sTw)          # offline
    Kp = wl.K + S
    ac = torch.empty((wl.M, Kp // 2), dtype=torch.uint8, device="cuda")
    asc = torch.empty((wl.M, Kp // 16), dtype=torch.uint8, device="cuda")
    Y = torch.empty((wl.M, wl.N), dtype=torch.float16, device="cuda")
    need = B.arcq_gemm_workspace_size(wl.M, wl.N, Kp)
    ws = torch.empty(max(need, 1), dtype=torch.uint8, device="cuda")
    quant = B.prepare_quantize_act(X, perm, S, sTx, ac, asc)
    gemm = B.prepare_gemm(ac, asc, sTx, wc, wsc, sTw, Y, ws)

    def step():
        quant()
        gemm()
    if steps is None:                       # loop lengths from the step's own duration: about 60 ms timed
        est = sustained_ms(torch, step, 3, 2)
        steps = int(min(max(60.0 / est, 10), 4000))
        warmup = int(min(max(20.0 / est, 4), 2000))
    for _ in range(warmup):
        quant()
        gemm()
    torch.cuda.synchronize()
    # timed region: exactly `steps` steps, nothing but the two launches per step on the stream
    first, last = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    first.record()
    for _ in range(steps):
        quant()
        gemm()
    last.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    dev_ms = first.elapsed_time(last) / steps
    # the same steps again with an event after every launch: per-kernel launch durations for the
    # rooflines (the extra events cost a few microseconds per step, so they stay out of the region above)
    nev = min(steps, 200)
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(nev)]
    for e in evs:
        e[0].record()
        quant()
        e[1].record()
        gemm()
        e[2].record()
    torch.cuda.synchronize()
    out = {
        "wall_ms": wall_ms,
        "dev_ms": dev_ms,
        "steps": steps,
        "warmup": warmup,
        "quant_ms": sum(e[0].elapsed_time(e[1]) for e in evs) / nev,
        "gemm_ms": sum(e[1].elapsed_time(e[2]) for e in evs) / nev,
        # the same kernels launched back to back in loops of their own (no event between launches)
        "quant_loop_ms": sustained_ms(torch, quant),
        "gemm_loop_ms": sustained_ms(torch, gemm),
    }
    # the quantizer with RMSNorm fused in front (Section 3.3), on the same tensor taken as the
    # pre-norm hidden state: its own figure, not part of the step
    from paper_2601_07475_amd import workloads as wk
    gamma = d(wk.rmsnorm_gamma(wl))
    nq = B.prepare_rmsnorm_quantize_act(X, gamma, 1e-5, perm, S, sTx, ac, asc)
    out["rmsnorm_quant_ms"] = sustained_ms(torch, nq)
    # the MXFP4 variant of the same step (block 32, E8M0 scales; the GEMM runs on the scaled FP4 matrix
    # instruction): its own figures, not part of `value`
    if wl.K % 32 == 0 and S % 32 == 0:
        mwc, mwsc = B.arcq_mx_pack_weight(W, perm, S)
        mac = torch.empty((wl.M, Kp // 2), dtype=torch.uint8, device="cuda")
        masc = torch.empty((wl.M, Kp // 32), dtype=torch.uint8, device="cuda")

        mx_quant = B.prepare_mx_quantize_act(X, perm, S, mac, masc)
        mx_gemm = B.prepare_mx_gemm(mac, masc, mwc, mwsc, Y)

        def mx_step():
            mx_quant()
            mx_gemm()
        out["mx_step_ms"] = sustained_ms(torch, mx_step)
        out["mx_gemm_ms"] = sustained_ms(torch, mx_gemm)
    if wl.M <= 128:
        # decode shapes: the packed weight (tens of MB) stays in the 256 MB last-level cache between
        # launches above; rotating over enough copies to exceed it gives the figure with the weight
        # streamed from HBM on every launch, which is what a model with many layers sees
        wbytes = wc.numel() + wsc.numel()
        ncopy = max(2, -(-384 * 2**20 // wbytes))
        copies = [(wc.clone(), wsc.clone()) for _ in range(ncopy)]
        gemms = [B.prepare_gemm(ac, asc, sTx, c, sc, sTw, Y, ws) for c, sc in copies]
        def rotate():                       # one call = one launch on every copy
            for g in gemms:
                g()
        out["gemm_rotating_ms"] = sustained_ms(torch, rotate) / ncopy
        out["gemm_rotating_copies"] = ncopy
        del copies, gemms
    if vendor_ref:
        # context only: the vendor library's bf16 GEMM (hipBLASLt through torch.matmul) on the
        # unquantized operands, K columns (no augmentation); not part of the product path
        Xb, Wb = X.to(torch.bfloat16), W.to(torch.bfloat16)
        Wt = Wb.t()
        Yb = torch.empty((wl.M, wl.N), dtype=torch.bfloat16, device="cuda")
        out["vendor_bf16_gemm_ms"] = sustained_ms(torch, lambda: torch.matmul(Xb, Wt, out=Yb))
        # and this library's own bf16 kernel on the tiled skeleton of the MXFP4 GEMM (arcq_ref_gemm_bf16); prefill
        # shapes only: it has no weight-streaming variant, so on the decode shapes it would flatter the quantized path
        if wl.K % 32 == 0 and wl.M > 128:
            out["hand_bf16_gemm_ms"] = sustained_ms(torch, B.prepare_ref_gemm_bf16(Xb, Wb, Y))
    return out


def summarize(wl, S, t):
    Kp = wl.K + S
    fl = gemm_flops(wl.M, wl.N, Kp)
    qb = quantizer_bytes(wl.M, wl.K, S)
    gb = gemm_bytes(wl.M, wl.N, Kp)
    s = {
        "M": wl.M, "K": wl.K, "N": wl.N, "S": S,
        "steps": t["steps"], "warmup": t["warmup"],
        "step_ms": round(t["dev_ms"], 5), "quant_ms": round(t["quant_ms"], 5), "gemm_ms": round(t["gemm_ms"], 5),
        "quant_loop_ms": round(t["quant_loop_ms"], 5), "gemm_loop_ms": round(t["gemm_loop_ms"], 5),
        "step_tflops": round(fl / t["dev_ms"] / 1e9, 2),
        # per-kernel rates from the back-to-back loops: an event pair around a single launch adds 2-5 us to a
        # kernel of this length (the kernel trace of the timed steps agrees with the loops, not with the pairs)
        "gemm_tflops": round(fl / t["gemm_loop_ms"] / 1e9, 2),
        "gemm_frac_of_f16_mfma_peak": round(fl / t["gemm_loop_ms"] / 1e9 / PEAK_MFMA_F16_TFLOPS, 4),
        "gemm_operand_gbs": round(gb / t["gemm_loop_ms"] / 1e6, 1),
        "gemm_frac_of_hbm_peak": round(gb / t["gemm_loop_ms"] / 1e6 / PEAK_HBM_GBS, 4),
        "quant_gbs": round(qb / t["quant_loop_ms"] / 1e6, 1),
        "quant_frac_of_hbm_peak": round(qb / t["quant_loop_ms"] / 1e6 / PEAK_HBM_GBS, 4),
        "rmsnorm_quant_ms": round(t["rmsnorm_quant_ms"], 5),
        "rmsnorm_quant_gbs": round((qb + 2 * wl.K) / t["rmsnorm_quant_ms"] / 1e6, 1),
    }
    if "mx_step_ms" in t:
        s["mxfp4"] = {"step_ms": round(t["mx_step_ms"], 5), "gemm_ms": round(t["mx_gemm_ms"], 5),
                      "step_tflops": round(fl / t["mx_step_ms"] / 1e9, 2),
                      "gemm_tflops": round(fl / t["mx_gemm_ms"] / 1e9, 2),
                      "gemm_frac_of_fp4_mfma_peak": round(fl / t["mx_gemm_ms"] / 1e9 / PEAK_MFMA_FP4_TFLOPS, 4)}
    if "vendor_bf16_gemm_ms" in t:
        s["vendor_bf16_gemm_ms"] = round(t["vendor_bf16_gemm_ms"], 5)
        s["linear_vs_vendor_bf16"] = round(t["vendor_bf16_gemm_ms"] / t["dev_ms"], 3)   # > 1: quantized linear is faster
    if "hand_bf16_gemm_ms" in t:
        s["hand_bf16_gemm_ms"] = round(t["hand_bf16_gemm_ms"], 5)
        s["linear_vs_hand_bf16"] = round(t["hand_bf16_gemm_ms"] / t["dev_ms"], 3)
    if "gemm_rotating_ms" in t:
        s["gemm_rotating_ms"] = round(t["gemm_rotating_ms"], 5)
        s["gemm_rotating_copies"] = t["gemm_rotating_copies"]
        s["gemm_rotating_gbs"] = round(gb / t["gemm_rotating_ms"] / 1e6, 1)
        s["gemm_rotating_frac_of_hbm_peak"] = round(gb / t["gemm_rotating_ms"] / 1e6 / PEAK_HBM_GBS, 4)
    s["traffic_bytes"] = MEASURED_TRAFFIC.get(wl.name)
    return s


def s_sweep(torch, B, case, values):
    """GEMM and quantizer time against the number S of augmented channels at the workload's shape
    (Section 3.4: the cost of compensation is the extra S/K of the reduction dimension, so the GEMM
    time should rise linearly in S from the S = 0 point, which is plain NVFP4 W4A4)."""
    import numpy as np
    wl = case["wl"]
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    X, W, perm = d(case["X"]), d(case["W"]), d(case["perm"])
    sTx, sTw = float(case["sT_x"]), float(case["sT_w"])
    Y = torch.empty((wl.M, wl.N), dtype=torch.float16, device="cuda")
    rows = []
    for S in values:
        if S > wl.K:
            continue
        Kp = wl.K + S
        wc, wsc = B.arcq_pack_weight(W, perm, S, sTw)
        ac = torch.empty((wl.M, Kp // 2), dtype=torch.uint8, device="cuda")
        asc = torch.empty((wl.M, Kp // 16), dtype=torch.uint8, device="cuda")
        ws = torch.empty(max(B.arcq_gemm_workspace_size(wl.M, wl.N, Kp), 1), dtype=torch.uint8, device="cuda")
        quant = B.prepare_quantize_act(X, perm, S, sTx, ac, asc)
        gemm = B.prepare_gemm(ac, asc, sTx, wc, wsc, sTw, Y, ws)
        rows.append({"S": S, "quant_ms": round(sustained_ms(torch, quant, target_ms=10.0, warm_ms=5.0), 5),
                     "gemm_ms": round(sustained_ms(torch, gemm, target_ms=30.0, warm_ms=15.0), 5)})
    g0 = rows[0]["gemm_ms"] if rows and rows[0]["S"] == 0 else None
    for r in rows:
        r["gemm_vs_S0"] = round(r["gemm_ms"] / g0, 4) if g0 else None
        r["Kp_vs_K"] = round((wl.K + r["S"]) / wl.K, 4)
    return rows


def mfma_rate(torch, probe, B, iters=2000):
    """Matrix instructions on register operands, four waves per SIMD, no memory traffic: the matrix rate
    this box sustains (TFLOP/s), the practical ceiling of the GEMM's roofline.  `probe`: B.arcq_probe_mfma_f16
    (fp16 32x32x16) or B.arcq_probe_mfma_fp4 (scaled FP4 32x32x64)."""
    sink = torch.empty(B.PROBE_SINK_FLOATS, dtype=torch.float32, device="cuda")
    flop = [0.0]

    def launch():
        flop[0] = probe(iters, sink)
    ms = sustained_ms(torch, launch)
    return round(flop[0] / ms / 1e9, 1)


def copy_rate(torch, nbytes=1 << 30, iters=5):
    """Plain device-to-device copy of 1 GiB: the streaming rate this machine reaches (read + write bytes per second)."""
    src = torch.ones(nbytes, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    return round(2 * nbytes * iters / e0.elapsed_time(e1) / 1e6, 1)


def cpu_baseline(case):
    """The oracle, as it stands, on the host cores: one pass of the same step on the same workload."""
    import numpy as np
    from oracle import arcquant as A
    wl = case["wl"]
    S = case["S"]
    owc, owsc = [], []
    for i in range(0, wl.N, 512):                          # offline, untimed; chunked to bound memory
        c, s = A.pack_weight(case["W"][i:i + 512], case["perm"], S, case["sT_w"])
        owc.append(c)
        owsc.append(s)
    owc, owsc = np.concatenate(owc), np.concatenate(owsc)
    t0 = time.perf_counter()
    oac, oasc = A.quantize_act(case["X"], case["perm"], S, case["sT_x"])
    t1 = time.perf_counter()
    A.gemm(oac, oasc, case["sT_x"], owc, owsc, case["sT_w"])
    t2 = time.perf_counter()
    threads = int(os.environ.get("OMP_NUM_THREADS", 0)) or os.cpu_count()
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        pass
    fl = gemm_flops(wl.M, wl.N, wl.K + S)
    return {
        "value": round(fl / (t2 - t0) / 1e12, 6), "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
        "sample": f"whole {wl.name} workload, one step (numpy: quantize_act {t1 - t0:.2f} s single-threaded, "
                  f"fp64 dequantize + matmul {t2 - t1:.2f} s on {threads} BLAS threads)",
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=300)
    ap.add_argument("--workload", default="c2_llama8b_q")
    ap.add_argument("--also", default="c4_qwen32b_mlp,c5_llama70b_down,c3a_llama8b_up,c3b_llama8b_down",
                    help="comma-separated extra workloads reported under 'also' (loop lengths from their own step time); '' for none")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-vendor-ref", action="store_true")
    ap.add_argument("--s-sweep", default="0,128,256,512,1024,2048",
                    help="values of S timed at the main workload's shape, reported under 's_sweep'; '' for none")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="first run three plain 1 GiB device copies (a kernel of known traffic, for scaling "
                         "the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc pass)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; rows of X shard across GPUs with no exchange, "
              "but no multi-GPU path is part of it. Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2601_07475_amd import binding as B
    from paper_2601_07475_amd import workloads as wk

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    B.lib()                                              # fail loudly if the HIP library is missing
    torch.cuda.set_device(0)

    if args.calibrate_copy:
        src = torch.ones(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

    wl = wk.WORKLOADS[args.workload]
    case = wk.make_case(wl)
    t = measure(torch, B, case, args.steps, args.warmup, not args.no_vendor_ref)
    s = summarize(wl, case["S"], t)
    Kp = wl.K + case["S"]

    also = {}
    for name in [n for n in args.also.split(",") if n and n != args.workload]:
        w2 = wk.WORKLOADS[name]
        c2 = wk.make_case(w2)
        also[name] = summarize(w2, c2["S"], measure(torch, B, c2, None, None, not args.no_vendor_ref))
        del c2
        torch.cuda.empty_cache()

    mfma_tflops = mfma_rate(torch, B.arcq_probe_mfma_f16, B)
    mfma_fp4_tflops = mfma_rate(torch, B.arcq_probe_mfma_fp4, B)
    sweep = s_sweep(torch, B, case, [int(v) for v in args.s_sweep.split(",") if v]) if args.s_sweep else None
    stream_gbs = copy_rate(torch)

    traffic = MEASURED_TRAFFIC.get(args.workload, {})
    out = {
        "metric": "augmented NVFP4 GEMM TFLOPS (2*M*N*K') over the quantizer+GEMM step; quantizer GB/s and % of MI355X roofline alongside",
        "value": s["step_tflops"], "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(t["wall_ms"], 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16",
        "dtype_note": "NVFP4 (E2M1 x E4M3) operands decoded exactly to f16 for the MFMA, f32 accumulate; quantizer arithmetic in f32",
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: X fp16 [{wl.M},{wl.K}] -> W4A4 linear N={wl.N}, S={case['S']}, K'={Kp}",
                   "outliers": f"{wl.n_outlier} channels {wl.outlier}", "seed": wl.seed},
        "roofline": {"kernel": "arcq_gemm", "bound": "mfma", "achieved": s["gemm_tflops"], "peak": PEAK_MFMA_F16_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(s["gemm_tflops"] / PEAK_MFMA_F16_TFLOPS, 4), "launch_ms": s["gemm_loop_ms"],
                     "traffic": traffic.get("arcq_gemm")},
        "roofline_quantizer": {"kernel": "arcq_quantize_act", "bound": "hbm", "achieved": s["quant_gbs"],
                               "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": s["quant_frac_of_hbm_peak"],
                               "traffic": traffic.get("arcq_quantize_act"),
                               "note": "this workload (22 MB) is cache-resident: effective GB/s; the HBM-streaming figure is also.c5_llama70b_down.quant_gbs"},
        "detail": s, "also": also, "s_sweep": sweep,
        "machine": {"device_copy_gbs": stream_gbs, "mfma_f16_tflops": mfma_tflops, "mfma_fp4_tflops": mfma_fp4_tflops,
                    "note": "measured on this box: 1 GiB device-to-device copy (read + write bytes); fp16 32x32x16 and "
                            "scaled FP4 32x32x64 matrix instructions on register operands, four waves per SIMD"},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(case)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
