#!/usr/bin/env python3
"""Benchmark of the CCQ fused dequantize-and-multiply on one MI355X.

A step is one pass of the whole hot path (stream codes -> Code Cluster map -> window
extraction -> linear value map -> contraction -> K reduction) over one batch: one ccq_gemm
call with M = 1 on the dense decode configuration K = N = 8192 at 2.0 code bits/weight with fp16
group-64 scales.  Inputs are resident in HBM before the timed region.  The step rotates over
enough copies of the weights (distinct addresses) that the 256 MB Infinity Cache cannot hold
them, so the rate is an HBM rate.  Launches are captured in a HIP graph (one replay = one pass
over all copies) so that the host launch path is not what is timed.

Prints one JSON line: the headline metric (effective HBM GB/s at M = 1), the roofline object
for the dominant kernel (HIP events over the timed region), the oracle timed on the host cores
(cpu_baseline), and, as additional context, the M = 2048 prefill rate in TFLOP/s.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published
# HBM bytes per launch of the GEMV kernel from rocprofv3 --pmc (profiles/gemv_narrow_config2_hbm_traffic.txt):
# FETCH_SIZE 9407.26 KiB x 2.0 (a plain 64 MiB copy reads 32780 KiB on that counter) + WRITE_SIZE 16.0 KiB x 1.0
TRAFFIC_BYTES_PER_LAUNCH = int(9407.26 * 1024 * 2.0 + 16.0 * 1024)


def algorithmic_bytes(K: int, N: int, M: int, code_bytes: int, has_cluster: bool) -> int:
    """codes + fp16 group scales + per-row alpha/beta + activations + outputs."""
    return code_bytes + N * (K // 64) * 2 + (8 * N if has_cluster else 0) + 2 * M * K + 2 * M * N


def make_weight_copies(K, N, copies, device, compressed=False):
    """Random code bitstream (valid: every bit pattern decodes), log-uniform fp16 scales (or, with compressed scales,
    random 4-bit fields and log-uniform fp16 super scales), random Code Cluster parameters; packed once and cloned to
    `copies` distinct device buffers."""
    import numpy as np
    import torch
    from paper_2507_07145_amd import binding as b, synth
    codes = synth.random_codes(N, K // 4, synth.rng(2, 0))
    alpha, beta = synth.cluster_params(N, synth.rng(2, 2))
    if compressed:
        sq = synth.rng(2, 5).integers(0, 256, size=(N, K // 128), dtype=np.uint8)
        ssup = synth.scales_log_uniform_fp16(N, 1, synth.rng(2, 6), 1e-4, 1e-2).reshape(N)
        w0 = b.Weight.from_canonical_compressed(K, N, [b.NARROW], codes, sq, ssup, alpha, beta, device=device)
        canon = (codes, sq, ssup, alpha, beta)
    else:
        scales = synth.scales_log_uniform_fp16(N, K // 64, synth.rng(2, 1))
        w0 = b.Weight.from_canonical(K, N, [b.NARROW], codes, scales, alpha, beta, device=device)
        canon = (codes, scales, alpha, beta)
    ws = [w0]
    for _ in range(copies - 1):
        w = b.Weight()
        w.codes, w.scales, w.alpha, w.beta = w0.codes.clone(), w0.scales.clone(), w0.alpha.clone(), w0.beta.clone()
        d = b.descriptor(K, N, [b.NARROW], scale_mode=1 if compressed else 0)
        d.codes, d.scales, d.code_alpha, d.code_beta = w.codes.data_ptr(), w.scales.data_ptr(), w.alpha.data_ptr(), w.beta.data_ptr()
        if compressed:
            w.ssup = w0.ssup.clone()
            d.scale_super = w.ssup.data_ptr()
        w.desc, w.info, w.E = d, w0.info, 1
        ws.append(w)
    return ws, canon


def time_steps(step_fns, steps, warmup, device):
    """Run `warmup` untimed and exactly `steps` timed steps, cycling over step_fns; one graph replay
    covers len(step_fns) steps.  Returns (wall seconds, event seconds)."""
    import torch
    R = len(step_fns)
    for i in range(warmup):
        step_fns[i % R]()
    torch.cuda.synchronize()
    stream = torch.cuda.Stream(device=device)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        for f in step_fns:          # one eager pass on the capture stream first
            f()
        stream.synchronize()
        with torch.cuda.graph(graph, stream=stream):
            for f in step_fns:
                f()
        graph.replay()
        stream.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        full, rest = divmod(steps, R)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record(stream)
        for _ in range(full):
            graph.replay()
        for i in range(rest):
            step_fns[i]()
        e1.record(stream)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    return t1 - t0, e0.elapsed_time(e1) * 1e-3


def cpu_baseline(canon, K, N, x_bits, budget_s=12.0):
    """The oracle as it stands (decode + fp64 GEMV) on the host cores, repeated for about budget_s."""
    from oracle import ccq_oracle as o
    codes, scales, alpha, beta = canon
    reps, spent = 0, 0.0
    t_start = time.perf_counter()
    while spent < budget_s and reps < 2000:
        W = o.decode(K, N, o.F2, codes, scales, alpha, beta)
        o.matmul(x_bits, W)
        reps += 1
        spent = time.perf_counter() - t_start
    nbytes = algorithmic_bytes(K, N, 1, codes.size, True)
    return {"value": round(nbytes * reps / spent / 1e9, 4), "unit": "GB/s", "cores": o.num_threads(), "kind": "oracle",
            "sample": f"whole workload (decode + fp64 GEMV of the {N}x{K} matrix, M=1), {reps} repetitions, {spent:.1f} s"}


PAPER_TABLE4_MS = {(4096, 4096, 1): 0.034, (4096, 1024, 1): 0.017, (8192, 8192, 1): 0.090, (8192, 1024, 1): 0.022,
                   (4096, 4096, 4): 0.035, (4096, 1024, 4): 0.017, (8192, 8192, 4): 0.104, (8192, 1024, 4): 0.024}
PAPER_TABLE5_MS = {(7168, 512, 1): 0.021, (1024, 7168, 1): 0.058, (7168, 512, 4): 0.027, (1024, 7168, 4): 0.166,
                   (7168, 512, 16): 0.059, (1024, 7168, 16): 0.527, (7168, 512, 64): 0.161, (1024, 7168, 64): 1.386}


def paper_tables(dev) -> int:
    """Second workload: the shapes of the paper's operator benchmarks (Table 4 GEMV, Table 5 Grouped-GEMM) at 2.06 bits
    per weight (narrow format, compressed scales).  Table 5 is read as 256 experts of one shape, M tokens, each routed to
    8 distinct experts.  One JSON line; the paper's H20 times ride along as context, not as a target."""
    import numpy as np
    import torch
    from paper_2507_07145_amd import binding as b, synth

    def comp_weights(E, K, N, seed):
        rng = synth.rng(8, seed)
        codes = synth.random_codes(E * N, K // 4, rng).reshape(E, N, K // 4)
        sq = rng.integers(0, 256, size=(E, N, K // 128), dtype=np.uint8)
        ssup = synth.scales_log_uniform_fp16(E * N, 1, rng, 1e-4, 1e-2).reshape(E, N)
        alpha, beta = synth.cluster_params(E * N, rng)
        return b.Weight.from_canonical_compressed(K, N, [b.NARROW], codes, sq, ssup, alpha.reshape(E, N), beta.reshape(E, N), device=dev,
                                                  experts=None if E == 1 else E)

    def clone(w0, K, N):
        w = b.Weight()
        w.codes, w.scales, w.alpha, w.beta, w.ssup = w0.codes.clone(), w0.scales.clone(), w0.alpha.clone(), w0.beta.clone(), w0.ssup.clone()
        d = b.descriptor(K, N, [b.NARROW], scale_mode=1)
        d.codes, d.scales, d.code_alpha, d.code_beta, d.scale_super = (w.codes.data_ptr(), w.scales.data_ptr(), w.alpha.data_ptr(),
                                                                       w.beta.data_ptr(), w.ssup.data_ptr())
        w.desc, w.info, w.E = d, w0.info, w0.E
        return w

    out = {"workload": "paper Tables 4 and 5 at 2.06 bpw (narrow format + compressed scales)", "table4_gemv": [], "table5_grouped": []}
    for (K, N) in ((4096, 4096), (4096, 1024), (8192, 8192), (8192, 1024)):
        w0 = comp_weights(1, K, N, K + N)
        per_copy = w0.info.code_bytes + w0.info.scale_bytes + 10 * N
        copies = max(2, min(64, int(600e6 // per_copy) + 1))
        ws = [w0] + [clone(w0, K, N) for _ in range(copies - 1)]
        for M in (1, 4):
            x = b.bf16_tensor(synth.activations_bf16(M, K, synth.rng(8, 3)), dev)
            ys = [torch.empty((M, N), dtype=torch.bfloat16, device=dev) for _ in ws]
            wsp = torch.empty(max(b.pack_info(w0.desc, M).workspace_bytes, 16), dtype=torch.uint8, device=dev)
            fns = [(lambda w=w, y=y: b.gemm(w, x, out=y, workspace=wsp)) for w, y in zip(ws, ys)]
            steps = copies * 20
            _, ev = time_steps(fns, steps, copies, dev)
            nbytes = per_copy + 2 * M * K + 2 * M * N
            us = ev / steps * 1e6
            out["table4_gemv"].append({"K": K, "N": N, "M": M, "us": round(us, 2), "GBps": round(nbytes / us / 1e3, 1),
                                       "frac_of_hbm_peak": round(nbytes / us / 1e3 / HBM_PEAK_GBS, 4), "paper_h20_ms": PAPER_TABLE4_MS[(K, N, M)]})
        del ws
    E, topk = 256, 8
    for (N, K) in ((7168, 512), (1024, 7168)):
        w0 = comp_weights(E, K, N, 1000 + N)
        ws = [w0, clone(w0, K, N)]
        per_expert = (w0.info.code_bytes + w0.info.scale_bytes + 10 * N)
        for M in (1, 4, 16, 64):
            P = M * topk
            x = b.bf16_tensor(synth.activations_bf16(M, K, synth.rng(8, 4)), dev)
            routes, active = [], []
            for r in range(8):
                rows, offs = synth.routing_topk(M, E, topk, synth.rng(8, 100 * M + r))
                routes.append((torch.from_numpy(rows).to(dev), torch.from_numpy(offs).to(dev), offs))
                active.append(int(np.count_nonzero(np.diff(offs))))
            y = torch.empty((P, N), dtype=torch.bfloat16, device=dev)
            wsp = torch.empty(max(b.grouped_workspace_bytes(w0, P), 16), dtype=torch.uint8, device=dev)
            fns = [(lambda i=i: b.grouped_gemm(ws[i % 2], x, routes[i][0], routes[i][1], routes[i][2], out=y, workspace=wsp)) for i in range(8)]
            steps = 8 * 10
            _, ev = time_steps(fns, steps, 8, dev)
            nbytes = float(np.mean(active)) * per_expert + 2 * M * K + 2 * P * N
            us = ev / steps * 1e6
            out["table5_grouped"].append({"experts": E, "N": N, "K": K, "M": M, "rows": P, "active_experts_mean": round(float(np.mean(active)), 1),
                                          "us": round(us, 2), "GBps": round(nbytes / us / 1e3, 1),
                                          "frac_of_hbm_peak": round(nbytes / us / 1e3 / HBM_PEAK_GBS, 4), "paper_h20_ms": PAPER_TABLE5_MS[(N, K, M)]})
        del ws
    print(json.dumps(out))
    return 0


def hybrid_word(dev) -> int:
    """Third workload: the hybrid 16-bit word of Sec. 3.2 with its scale in the 13 spare bits (Sec. 3.4; 2.5 bits per
    weight in all) on the 8192 x 8192 shape, from one activation row to a prefill-sized batch.  One JSON line."""
    import numpy as np
    import torch
    from paper_2507_07145_amd import binding as b, synth
    K = N = 8192
    codes = synth.random_codes(N, (K // 64) * 20, synth.rng(9, 0))
    ssup = synth.scales_log_uniform_fp16(N, 1, synth.rng(9, 1), 1e-5, 1e-3).reshape(N)
    copies = 24
    ws = [b.Weight.from_canonical_compressed(K, N, b.H16, codes, None, ssup, device=dev) for _ in range(copies)]
    per_copy = ws[0].info.code_bytes + 2 * N
    out = {"workload": "hybrid word (3,3,2)+(3,4,2), scale in the 13 spare bits, 2.5 bpw, K=N=8192", "bytes_of_weights": per_copy, "rows": []}
    for M in (1, 4, 16, 64, 256, 2048):
        x = b.bf16_tensor(synth.activations_bf16(M, K, synth.rng(9, 3)), dev)
        ys = [torch.empty((M, N), dtype=torch.bfloat16, device=dev) for _ in ws]
        wsp = torch.empty(max(b.pack_info(ws[0].desc, M).workspace_bytes, 16), dtype=torch.uint8, device=dev)
        fns = [(lambda w=w, y=y: b.gemm(w, x, out=y, workspace=wsp)) for w, y in zip(ws, ys)]
        # enough launches before and inside the timed region for the clock to settle (about 20 ms of load)
        steps = copies * (20 if M <= 64 else (8 if M <= 256 else 2))
        _, ev = time_steps(fns, steps, copies * (4 if 64 < M <= 256 else 1), dev)
        nbytes = per_copy + 2 * M * K + 2 * M * N
        us = ev / steps * 1e6
        out["rows"].append({"M": M, "us": round(us, 2), "GBps": round(nbytes / us / 1e3, 1), "frac_of_hbm_peak": round(nbytes / us / 1e3 / HBM_PEAK_GBS, 4),
                            "TFLOPs": round(2.0 * M * K * N / us / 1e6, 1), "frac_of_mfma_peak": round(2.0 * M * K * N / us / 1e6 / MFMA_BF16_PEAK_TFLOPS, 4)})
        del ys, fns
    print(json.dumps(out))
    return 0


def quantize_workload(dev) -> int:
    """Fourth workload: the quantizer itself (Alg. 1 search + Eq. 4 + Code Cluster) on an 8192 x 8192 fp32 matrix of
    N(0, 0.02) weights, narrow and wide formats, next to the oracle's encoder timed on a sample of rows.  One JSON line."""
    import numpy as np
    import torch
    from paper_2507_07145_amd import binding as b, synth
    from oracle import ccq_oracle as o
    K = N = 8192
    Wh = synth.weights_normal(N, K, synth.rng(12, 0))
    W = torch.from_numpy(Wh).to(dev)
    out = {"workload": "quantize 8192 x 8192 fp32 weights ~ N(0, 0.02), group 64", "rows": []}
    for name, fmt, ofmt, mode in (("narrow (6,4,3) + Code Cluster, fp16 scales", b.NARROW, o.F2, 0), ("wide (4,3,2), fp16 scales", b.WIDE, o.F275, 0),
                                  ("narrow, compressed scales (2.06 bpw)", b.NARROW, o.F2, 1)):
        b.quantize(W, fmt, scale_mode=mode)
        torch.cuda.synchronize()
        reps = 3
        t0 = time.perf_counter()
        for _ in range(reps):
            b.quantize(W, fmt, scale_mode=mode)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / reps * 1e3
        rows = 32
        t0 = time.perf_counter()
        enc = o.quantize(Wh[:rows], ofmt)
        if mode == 1:
            o.compress_scales(Wh[:rows], ofmt, *enc)
        cpu_s = time.perf_counter() - t0
        out["rows"].append({"format": name, "ms": round(ms, 2), "Gweights_per_s": round(N * K / ms / 1e6, 2),
                            "cpu_oracle": {"Gweights_per_s": round(rows * K / cpu_s / 1e9, 5), "cores": o.num_threads(), "sample": f"{rows} rows"}})
    print(json.dumps(out))
    return 0


def calibrate_copy(dev) -> int:
    """A plain copy kernel of known size, rotating over buffers that together exceed the last-level cache."""
    import torch
    nbytes = 64 << 20
    srcs = [torch.full((nbytes,), i, dtype=torch.uint8, device=dev) for i in range(6)]
    dsts = [torch.empty_like(s) for s in srcs]
    launches = 24
    for i in range(launches):
        dsts[i % 6].copy_(srcs[i % 6])
    torch.cuda.synchronize()
    print(json.dumps({"calibration": "plain device copy", "bytes_read_per_launch": nbytes, "bytes_written_per_launch": nbytes, "launches": launches}))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=6400)
    ap.add_argument("--warmup", type=int, default=640)
    ap.add_argument("--copies", type=int, default=32, help="weight copies the step rotates over")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-prefill", action="store_true")
    ap.add_argument("--no-more-rows", action="store_true", help="skip the M = 8 and M = 16 rows of config 2")
    ap.add_argument("--no-compressed", action="store_true", help="skip the compressed-scale variant of the GEMV")
    ap.add_argument("--launch", type=str, default="", help="explicit decomposition RT,WR,WK,S for tuning (default: the library's choice)")
    ap.add_argument("--paper-tables", action="store_true",
                    help="run the second workload instead: the GEMV and Grouped-GEMM shapes of the paper's Tables 4 and 5 at 2.06 bpw")
    ap.add_argument("--hybrid-word", action="store_true",
                    help="run the third workload instead: the hybrid 16-bit word of Sec. 3.2 at 2.5 bpw on the 8192 x 8192 shape")
    ap.add_argument("--quantize", action="store_true", help="run the fourth workload instead: the GPU quantizer on an 8192 x 8192 matrix")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run only a plain device copy of known size (64 MiB read + 64 MiB written per launch): the reference that "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE readings are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2507_07145_amd import binding as b, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    b.load()

    if args.calibrate_copy:
        return calibrate_copy(dev)
    if args.paper_tables:
        return paper_tables(dev)
    if args.hybrid_word:
        return hybrid_word(dev)
    if args.quantize:
        return quantize_workload(dev)

    K = N = 8192
    M = 1
    weights, canon = make_weight_copies(K, N, args.copies, dev)
    x_bits = synth.activations_bf16(M, K, synth.rng(2, 3))
    x = b.bf16_tensor(x_bits, dev)
    ys = [torch.empty((M, N), dtype=torch.bfloat16, device=dev) for _ in weights]
    launch = b.ccq_launch(*[int(v) for v in args.launch.split(",")]) if args.launch else None
    ws_bytes = b.pack_info(weights[0].desc, M).workspace_bytes if launch is None else launch.splits_k * M * N * 4
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev)

    def make_step(w, y):
        return lambda: b.gemm(w, x, out=y, workspace=ws, launch=launch)

    steps_fns = [make_step(w, y) for w, y in zip(weights, ys)]
    wall, ev = time_steps(steps_fns, args.steps, args.warmup, dev)
    nbytes = algorithmic_bytes(K, N, M, weights[0].info.code_bytes, True)
    value = nbytes * args.steps / wall / 1e9
    per_launch_s = ev / args.steps
    achieved = nbytes / per_launch_s / 1e9
    out = {
        "metric": "CCQ decode-GEMM effective HBM GB/s (M=1) and TFLOP/s (M=2048), % of roofline",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(wall / args.steps * 1e3, 6), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic (seeded random code bitstream, log-uniform fp16 scales, N(0,1) bf16 activations)",
        "config": {"workload": "config 2: dense decode GEMV, M=1, K=8192, N=8192, 2.0 code bits/weight + fp16 group-64 scales",
                   "M": M, "K": K, "N": N, "weight_copies": args.copies, "bytes_per_step": nbytes, "launch": "HIP graph replay"},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": TRAFFIC_BYTES_PER_LAUNCH,
                     "kernel": "ccq_gemv_narrow_kernel", "us_per_launch": round(per_launch_s * 1e6, 3)},
    }

    if not args.no_more_rows:
        # the other row counts of config 2 (M = 8, 16), same weights, as context
        rows_out = []
        for Mr in (8, 16):
            xr = b.bf16_tensor(synth.activations_bf16(Mr, K, synth.rng(2, 30 + Mr)), dev)
            yr = [torch.empty((Mr, N), dtype=torch.bfloat16, device=dev) for _ in weights]
            wsr = torch.empty(max(b.pack_info(weights[0].desc, Mr).workspace_bytes, 16), dtype=torch.uint8, device=dev)
            fns = [(lambda w=w, y=y: b.gemm(w, xr, out=y, workspace=wsr)) for w, y in zip(weights, yr)]
            _, ev_r = time_steps(fns, 20 * len(fns), len(fns), dev)
            us = ev_r / (20 * len(fns)) * 1e6
            nb = algorithmic_bytes(K, N, Mr, weights[0].info.code_bytes, True)
            rows_out.append({"M": Mr, "us_per_launch": round(us, 2), "GBps": round(nb / us / 1e3, 1), "frac_of_hbm_peak": round(nb / us / 1e3 / HBM_PEAK_GBS, 4)})
        out["config2_more_rows"] = rows_out

    if not args.no_prefill:
        Kp, Np, Mp = 7168, 18432, 2048
        cp = synth.random_codes(Np, Kp // 4, synth.rng(5, 0))
        sp = synth.scales_log_uniform_fp16(Np, Kp // 64, synth.rng(5, 1))
        ap_, bp_ = synth.cluster_params(Np, synth.rng(5, 2))
        wp = b.Weight.from_canonical(Kp, Np, [b.NARROW], cp, sp, ap_, bp_, device=dev)
        xp = b.bf16_tensor(synth.activations_bf16(Mp, Kp, synth.rng(5, 3)), dev)
        yp = torch.empty((Mp, Np), dtype=torch.bfloat16, device=dev)
        wsp = torch.empty(max(b.pack_info(wp.desc, Mp).workspace_bytes, 16), dtype=torch.uint8, device=dev)
        # the clock takes some 20 ms of this load to settle (the first launches after the GEMV legs run about 20 %
        # slower than the sustained rate): 50 untimed launches, then 100 timed ones (about 50 ms)
        for _ in range(50):
            b.gemm(wp, xp, out=yp, workspace=wsp)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 100
        e0.record()
        for _ in range(reps):
            b.gemm(wp, xp, out=yp, workspace=wsp)
        e1.record()
        torch.cuda.synchronize()
        sec = e0.elapsed_time(e1) * 1e-3 / reps
        tf = 2.0 * Mp * Kp * Np / sec / 1e12
        out["prefill"] = {"workload": "config 5: M=2048, K=7168, N=18432, 2.0 code bits/weight", "ms": round(sec * 1e3, 4),
                          "value": round(tf, 2), "unit": "TFLOP/s",
                          "roofline": {"bound": "mfma", "achieved": round(tf, 2), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                       "frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 4)}}

    if not args.no_compressed:
        # the same GEMV with the compressed scales of Sec. 3.4 (2.0625 bits per weight all told)
        weights_c, _ = make_weight_copies(K, N, args.copies, dev, compressed=True)
        ys_c = [torch.empty((M, N), dtype=torch.bfloat16, device=dev) for _ in weights_c]
        fns_c = [(lambda w=w, y=y: b.gemm(w, x, out=y, workspace=ws)) for w, y in zip(weights_c, ys_c)]
        steps_c = max(args.copies * 8, (args.steps // 4) // args.copies * args.copies)
        _, ev_c = time_steps(fns_c, steps_c, args.copies, dev)
        nbytes_c = weights_c[0].info.code_bytes + weights_c[0].info.scale_bytes + 8 * N + 2 * N + 2 * M * K + 2 * M * N
        out["compressed_scales"] = {"workload": "config 2 shape with 4-bit group scales x fp16 super scale per row (Sec. 3.4), M=1",
                                    "bytes_per_step": nbytes_c, "us_per_launch": round(ev_c / steps_c * 1e6, 3),
                                    "value": round(nbytes_c / (ev_c / steps_c) / 1e9, 1), "unit": "GB/s",
                                    "frac_of_hbm_peak": round(nbytes_c / (ev_c / steps_c) / 1e9 / HBM_PEAK_GBS, 4)}
        del weights_c, ys_c, fns_c

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(canon, K, N, x_bits)
    out["context"] = {"paper": "CCQ GEMV 8192x8192 M=1 at 2.06 bpw: 0.090 ms on one NVIDIA H20 (Table 4); another machine, not a target"}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
