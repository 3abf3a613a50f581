#!/usr/bin/env python3
"""Benchmark of the CCQ fused dequantize-and-multiply on one MI355X.

A step is one pass of the whole hot path (stream codes -> Code Cluster map -> window
extraction -> linear value map -> contraction -> K reduction) over one batch: one ccq_gemm
call with M = 1 on the dense decode configuration K = N = 8192 at 2.0 code bits/weight with fp16
group-64 scales.  Inputs are resident in HBM before the timed region.  The step rotates over
enough copies of the weights (distinct addresses) that the 256 MB Infinity Cache cannot hold
them, so the rate is an HBM rate.

Every timed launch comes from a HIP graph, whatever --steps says: a graph of one pass over all
weight copies is replayed steps // copies times and a second graph holds the remaining
steps % copies launches, so exactly `steps` launches are timed.  Before the timed region the
first graph is replayed until the GPU has been under this load for about 20 ms (and at least
--warmup launches), because the clock needs that long to settle.  The timed region is repeated
(each repetition is exactly `steps` launches between two HIP events on the launch stream and a
synchronize on both sides) and the repetition with the median event time is the one reported.

Prints one JSON line: the headline metric (effective HBM GB/s at M = 1) with its roofline
object, and as further keys the other rows of config 2, configs 3, 4 and 5, the compressed-scale
variant, the measured ceilings (a read-only streaming kernel over the same bytes, a pure MFMA
loop) and the oracle timed on the host cores (cpu_baseline).  --legs selects a subset.
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
# HBM bytes per launch of the GEMV kernel, read from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE and scaled by a plain
# copy of known size; a constant taken from the named profile, not a measurement of the run that prints it
TRAFFIC_BYTES_PER_LAUNCH = int(9375.51 * 1024 * 2.0 + 16.0 * 1024)
TRAFFIC_SOURCE = "profiles/gemv_config2_hbm_traffic.txt (FETCH_SIZE 9375.51 KiB x 2.0 + WRITE_SIZE 16.0 KiB x 1.0)"
ALL_LEGS = ("headline", "more_rows", "compressed", "config3", "config4", "prefill", "ceilings", "cpu")
SETTLE_MS = 20.0                # load the clock needs before it has settled


def algorithmic_bytes(K: int, N: int, M: int, code_bytes: int, has_cluster: bool) -> int:
    """codes + fp16 group scales + per-row alpha/beta + activations + outputs."""
    return code_bytes + N * (K // 64) * 2 + (8 * N if has_cluster else 0) + 2 * M * K + 2 * M * N


def clone_weight(w0, fmts, scale_mode=0, group_fmt=None):
    """A second copy of a device-resident weight at distinct addresses (same descriptor fields)."""
    from paper_2507_07145_amd import binding as b
    w = b.Weight()
    d = b.descriptor(w0.desc.K, w0.desc.N, fmts, group_fmt if group_fmt is not None else w0._group_fmt, scale_mode=scale_mode)
    w._group_fmt = w0._group_fmt
    for name, field in (("codes", "codes"), ("scales", "scales"), ("alpha", "code_alpha"), ("beta", "code_beta"), ("meta", "meta"),
                        ("ssup", "scale_super")):
        t = getattr(w0, name)
        if t is not None:
            t = t.clone()
            setattr(w, name, t)
            setattr(d, field, t.data_ptr())
    w.desc, w.info, w.E = d, w0.info, w0.E
    return w


def make_weight_copies(K, N, copies, device, compressed=False):
    """Random code bitstream (valid: every bit pattern decodes), log-uniform fp16 scales (or, with compressed scales,
    random 4-bit fields and log-uniform fp16 super scales), random Code Cluster parameters; packed once and cloned to
    `copies` distinct device buffers."""
    import numpy as np
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
    return [w0] + [clone_weight(w0, [b.NARROW], 1 if compressed else 0) for _ in range(copies - 1)], canon


def time_steps(step_fns, steps, warmup, device, target_launches=3000, max_reps=51):
    """Times exactly `steps` launches, all replayed from HIP graphs, cycling over step_fns (see the module text).
    Returns a dict: event seconds and wall seconds of the median repetition, what ran, and how."""
    import torch
    R = len(step_fns)
    full, rest = divmod(steps, R)
    stream = torch.cuda.Stream(device=device)
    with torch.cuda.stream(stream):
        for f in step_fns:          # one eager pass first: modules load and kernel attributes are set outside the capture
            f()
        stream.synchronize()
        g_full = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g_full, stream=stream):
            for f in step_fns:
                f()
        g_rest = None
        if rest:
            g_rest = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g_rest, stream=stream):
                for f in step_fns[:rest]:
                    f()
        # untimed: at least `warmup` launches and about SETTLE_MS of this load
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        warm_launches, warm_ms = 0, 0.0
        while warm_launches < max(warmup, R) or warm_ms < SETTLE_MS:
            e0.record(stream)
            g_full.replay()
            e1.record(stream)
            stream.synchronize()
            warm_ms += e0.elapsed_time(e1)
            warm_launches += R
            if warm_launches > 200000:
                break
        reps = max(1, min(max_reps, -(-target_launches // max(steps, 1))))
        reps += 1 - reps % 2
        results = []
        for _ in range(reps):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            e0.record(stream)
            for _ in range(full):
                g_full.replay()
            if g_rest is not None:
                g_rest.replay()
            e1.record(stream)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            results.append((e0.elapsed_time(e1) * 1e-3, t1 - t0))
        results.sort()
        ev, wall = results[len(results) // 2]
    return {"event_s": ev, "wall_s": wall, "launches": steps, "repetitions": reps, "warm_launches": warm_launches, "warm_ms": round(warm_ms, 2),
            "launch": f"HIP graph replay: {full} x graph of {R} launches" + (f" + 1 x graph of {rest}" if rest else "")
                      + f"; median of {reps} repetitions after {warm_launches} untimed launches ({warm_ms:.1f} ms)"}


def timed_row(step_fns, device, nbytes, flop=None, min_ms=12.0, guess_us=20.0):
    """A context row: enough whole passes over the copies for about min_ms of timed load."""
    R = len(step_fns)
    steps = max(R, int(min_ms * 1e3 / guess_us) // R * R)
    t = time_steps(step_fns, steps, R, device, target_launches=steps)
    us = t["event_s"] / steps * 1e6
    row = {"us_per_launch": round(us, 2), "launches": steps, "GBps": round(nbytes / us / 1e3, 1),
           "frac_of_hbm_peak": round(nbytes / us / 1e3 / HBM_PEAK_GBS, 4), "bytes_per_launch": int(nbytes)}
    if flop is not None:
        row["TFLOPs"] = round(flop / us / 1e6, 1)
        row["frac_of_mfma_peak"] = round(flop / us / 1e6 / MFMA_BF16_PEAK_TFLOPS, 4)
    return row


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


def config3_leg(dev):
    """Config 3: K = 8192, N = 28672, every group in the 2.75-bit format, and the seeded 32-of-128 mix with the 2-bit
    format; M in {1, 16, 64}.  Bytes as stored; M = 64 is reported against both roofs."""
    import torch
    from paper_2507_07145_amd import binding as b, synth
    K, N, G = 8192, 28672, 128
    out = []
    for variant in ("all_wide", "mixed_32_of_128"):
        if variant == "all_wide":
            fmts, gf = [b.WIDE], None
            codes = synth.random_codes(N, G * 22, synth.rng(3, 0))
            alpha = beta = None
        else:
            fmts = [b.NARROW, b.WIDE]
            gf = synth.group_format_map(G, 32, synth.rng(3, 24))
            codes = synth.random_codes(N, 96 * 16 + 32 * 22, synth.rng(3, 20))
            alpha, beta = synth.cluster_params(N, synth.rng(3, 22))
        scales = synth.scales_log_uniform_fp16(N, G, synth.rng(3, 1))
        w0 = b.Weight.from_canonical(K, N, fmts, codes, scales, alpha, beta, gf, device=dev)
        ws = [w0] + [clone_weight(w0, fmts) for _ in range(7)]       # 8 copies: 570-700 MB
        stored = w0.info.code_bytes + w0.info.scale_bytes + (8 * N if alpha is not None else 0)
        rows = []
        for M in (1, 16, 64):
            x = b.bf16_tensor(synth.activations_bf16(M, K, synth.rng(3, 30 + M)), dev)
            ys = [torch.empty((M, N), dtype=torch.bfloat16, device=dev) for _ in ws]
            wsp = torch.empty(max(b.gemm_workspace_bytes(w0.desc, M), 16), dtype=torch.uint8, device=dev)
            fns = [(lambda w=w, y=y: b.gemm(w, x, out=y, workspace=wsp)) for w, y in zip(ws, ys)]
            row = {"M": M}
            row.update(timed_row(fns, dev, stored + 2 * M * K + 2 * M * N, flop=2.0 * M * K * N if M == 64 else None, guess_us=40.0))
            rows.append(row)
            del ys, fns
        out.append({"variant": variant, "code_bits_per_weight": w0.info.code_bpw, "rows": rows})
        del ws, w0
        torch.cuda.empty_cache()
    return {"workload": "config 3: K=8192, N=28672, 2.75-bit format / per-group mix with the 2-bit format, fp16 group scales", "variants": out}


def config4_leg(dev):
    """Config 4: 64 experts, up-projection K = 7168 -> N = 2048 and down-projection K = 2048 -> N = 7168 at 2.0 bits per
    weight, 64 tokens routed to 8 distinct experts each (seeded); two independent ccq_grouped_gemm calls.  Bytes count
    the experts that have rows."""
    import numpy as np
    import torch
    from paper_2507_07145_amd import binding as b, synth
    E, T, topk = 64, 64, 8
    out = []
    for proj, K, N, s0 in (("up", 7168, 2048, 0), ("down", 2048, 7168, 50)):
        G = K // 64
        codes = synth.random_codes(E * N, K // 4, synth.rng(4, s0)).reshape(E, N, K // 4)
        scales = synth.scales_log_uniform_fp16(E * N, G, synth.rng(4, s0 + 1)).reshape(E, N, G)
        alpha, beta = synth.cluster_params(E * N, synth.rng(4, s0 + 2))
        w0 = b.Weight.from_canonical(K, N, [b.NARROW], codes, scales, alpha.reshape(E, N), beta.reshape(E, N), device=dev, experts=E)
        ws = [w0, clone_weight(w0, [b.NARROW]), clone_weight(w0, [b.NARROW])]   # 3 x 268 MB
        per_expert = (w0.info.code_bytes + w0.info.scale_bytes + 8 * N)
        P = T * topk
        x = b.bf16_tensor(synth.activations_bf16(T, K, synth.rng(4, s0 + 4)), dev)
        routes, active = [], []
        for r in range(6):
            rows, offs = synth.routing_topk(T, E, topk, synth.rng(4, s0 + 3 + 100 * r))
            routes.append((torch.from_numpy(rows).to(dev), torch.from_numpy(offs).to(dev), offs))
            active.append(int(np.count_nonzero(np.diff(offs))))
        y = torch.empty((P, N), dtype=torch.bfloat16, device=dev)
        wsp = torch.empty(max(b.grouped_workspace_bytes(w0, P), 16), dtype=torch.uint8, device=dev)
        fns = [(lambda i=i: b.grouped_gemm(ws[i % 3], x, routes[i][0], routes[i][1], routes[i][2], out=y, workspace=wsp)) for i in range(6)]
        nbytes = float(np.mean(active)) * per_expert + 2 * T * K + 2 * P * N
        row = {"projection": proj, "K": K, "N": N, "experts": E, "tokens": T, "rows": P, "experts_with_rows_mean": round(float(np.mean(active)), 1)}
        row.update(timed_row(fns, dev, nbytes, flop=2.0 * P * K * N, guess_us=100.0))
        out.append(row)
        del ws, w0, fns
        torch.cuda.empty_cache()
    return {"workload": "config 4: MoE grouped decode GEMM, 64 experts, 64 tokens, top-8, 2.0 code bits/weight", "projections": out}


def ceilings_leg(dev, nbytes_config2):
    """What the machine delivers when nothing else is asked of it: a kernel that only reads the bytes of one config-2
    launch (same 16-byte nontemporal loads, rotating over 32 buffers), the same read over 1 GiB in one launch, and a
    loop of back-to-back bf16 MFMAs on N(0,1) register operands."""
    import numpy as np
    import torch
    from paper_2507_07145_amd import binding as b, synth
    n = nbytes_config2 // 16 * 16
    bufs = [torch.randint(0, 256, (n,), dtype=torch.uint8, device=dev) for _ in range(32)]
    sink = torch.zeros(1 << 20, dtype=torch.float32, device=dev)
    reads = []
    for lpt, bt in ((2, 256), (4, 256), (4, 512), (8, 256), (8, 512)):
        fns = [(lambda s=s: b.probe_stream_read(s, sink, lpt, bt)) for s in bufs]
        steps = 32 * 60
        t = time_steps(fns, steps, 32, dev, target_launches=steps)
        us = t["event_s"] / steps * 1e6
        reads.append({"loads_per_thread": lpt, "block_threads": bt, "us_per_launch": round(us, 3), "GBps": round(n / us / 1e3, 1),
                      "frac_of_hbm_peak": round(n / us / 1e3 / HBM_PEAK_GBS, 4)})
    best = min(reads, key=lambda r: r["us_per_launch"])
    del bufs
    # the same read over the bytes of one launch of config 3 (all wide, M = 1) and of config 4 (one projection)
    larger = []
    for label, nb in (("config3_all_wide_bytes", 88154112), ("config4_up_projection_bytes", 268304384)):
        nb = nb // 16 * 16
        copies = 8 if nb < (128 << 20) else 3
        bl = [torch.randint(0, 256, (nb,), dtype=torch.uint8, device=dev) for _ in range(copies)]
        fns = [(lambda s=s: b.probe_stream_read(s, sink, 2, 256)) for s in bl]
        steps = copies * 40
        t = time_steps(fns, steps, copies, dev, target_launches=steps)
        us = t["event_s"] / steps * 1e6
        larger.append({"what": label, "bytes_per_launch": nb, "loads_per_thread": 2, "block_threads": 256, "us_per_launch": round(us, 2),
                       "GBps": round(nb / us / 1e3, 1), "frac_of_hbm_peak": round(nb / us / 1e3 / HBM_PEAK_GBS, 4)})
        del bl
    big = [torch.randint(0, 256, (1 << 30,), dtype=torch.uint8, device=dev) for _ in range(2)]
    fns = [(lambda s=s: b.probe_stream_read(s, sink, 8, 256)) for s in big]
    t = time_steps(fns, 40, 2, dev, target_launches=40)
    us_big = t["event_s"] / 40 * 1e6
    del big
    torch.cuda.empty_cache()
    ops = b.bf16_tensor(synth.activations_bf16(8 * 64, 8, synth.rng(6, 0)), dev)
    mf = []
    for wgs in (256, 512, 1024):
        iters = 20000 * 256 // wgs
        flop = b.probe_mfma_bf16(ops, sink, wgs, iters)       # eager once (module load)
        torch.cuda.synchronize()
        fns = [lambda: b.probe_mfma_bf16(ops, sink, wgs, iters)]
        t = time_steps(fns, 30, 1, dev, target_launches=30)
        sec = t["event_s"] / 30
        mf.append({"workgroups": wgs, "wavefronts_per_simd": wgs // 256, "ms_per_launch": round(sec * 1e3, 4), "TFLOPs": round(flop / sec / 1e12, 1),
                   "frac_of_mfma_peak": round(flop / sec / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)})
    return {"stream_read_config2_bytes": {"bytes_per_launch": n, "variants": reads, "best": best},
            "stream_read_larger_launches": larger,
            "stream_read_1GiB": {"us_per_launch": round(us_big, 1), "GBps": round((1 << 30) / us_big / 1e3, 1),
                                 "frac_of_hbm_peak": round((1 << 30) / us_big / 1e3 / HBM_PEAK_GBS, 4)},
            "mfma_bf16_32x32x16_loop": mf}


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

    out = {"workload": "paper Tables 4 and 5 at 2.06 bpw (narrow format + compressed scales)", "table4_gemv": [], "table5_grouped": []}
    for (K, N) in ((4096, 4096), (4096, 1024), (8192, 8192), (8192, 1024)):
        w0 = comp_weights(1, K, N, K + N)
        per_copy = w0.info.code_bytes + w0.info.scale_bytes + 10 * N
        copies = max(2, min(64, int(600e6 // per_copy) + 1))
        ws = [w0] + [clone_weight(w0, [b.NARROW], 1) for _ in range(copies - 1)]
        for M in (1, 4):
            x = b.bf16_tensor(synth.activations_bf16(M, K, synth.rng(8, 3)), dev)
            ys = [torch.empty((M, N), dtype=torch.bfloat16, device=dev) for _ in ws]
            wsp = torch.empty(max(b.gemm_workspace_bytes(w0.desc, M), 16), dtype=torch.uint8, device=dev)
            fns = [(lambda w=w, y=y: b.gemm(w, x, out=y, workspace=wsp)) for w, y in zip(ws, ys)]
            row = {"K": K, "N": N, "M": M}
            row.update(timed_row(fns, dev, per_copy + 2 * M * K + 2 * M * N, guess_us=8.0))
            row["paper_h20_ms"] = PAPER_TABLE4_MS[(K, N, M)]
            out["table4_gemv"].append(row)
        del ws
    E, topk = 256, 8
    for (N, K) in ((7168, 512), (1024, 7168)):
        w0 = comp_weights(E, K, N, 1000 + N)
        ws = [w0, clone_weight(w0, [b.NARROW], 1)]
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
            row = {"experts": E, "N": N, "K": K, "M": M, "rows": P, "active_experts_mean": round(float(np.mean(active)), 1)}
            row.update(timed_row(fns, dev, float(np.mean(active)) * per_expert + 2 * M * K + 2 * P * N, guess_us=30.0))
            row["paper_h20_ms"] = PAPER_TABLE5_MS[(N, K, M)]
            out["table5_grouped"].append(row)
        del ws
    print(json.dumps(out))
    return 0


def hybrid_word(dev) -> int:
    """Third workload: the hybrid 16-bit word of Sec. 3.2 with its scale in the 13 spare bits (Sec. 3.4; 2.5 bits per
    weight in all) on the 8192 x 8192 shape, from one activation row to a prefill-sized batch.  One JSON line."""
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
        wsp = torch.empty(max(b.gemm_workspace_bytes(ws[0].desc, M), 16), dtype=torch.uint8, device=dev)
        fns = [(lambda w=w, y=y: b.gemm(w, x, out=y, workspace=wsp)) for w, y in zip(ws, ys)]
        row = {"M": M}
        row.update(timed_row(fns, dev, per_copy + 2 * M * K + 2 * M * N, flop=2.0 * M * K * N, guess_us=(20.0 if M <= 64 else (100.0 if M <= 256 else 600.0))))
        out["rows"].append(row)
        del ys, fns
    print(json.dumps(out))
    return 0


def quantize_workload(dev) -> int:
    """Fourth workload: the quantizer itself (Alg. 1 search + Eq. 4 + Code Cluster) on an 8192 x 8192 fp32 matrix of
    N(0, 0.02) weights, narrow and wide formats, next to the oracle's encoder timed on a sample of rows.  One JSON line."""
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
    ap.add_argument("--legs", type=str, default=",".join(ALL_LEGS),
                    help="comma-separated subset of " + ",".join(ALL_LEGS) + " (the headline is always run)")
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
    legs = set(s for s in args.legs.split(",") if s)
    unknown = legs - set(ALL_LEGS)
    if unknown or args.steps < 1 or args.warmup < 0 or args.copies < 1:
        print(f"bench.py: bad arguments (unknown legs {sorted(unknown)})" if unknown else "bench.py: bad --steps/--warmup/--copies", file=sys.stderr)
        return 2

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
    ws_bytes = b.gemm_workspace_bytes(weights[0].desc, M) if launch is None else launch.splits_k * M * N * 4
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev)

    def make_step(w, y):
        return lambda: b.gemm(w, x, out=y, workspace=ws, launch=launch)

    steps_fns = [make_step(w, y) for w, y in zip(weights, ys)]
    t = time_steps(steps_fns, args.steps, args.warmup, dev)
    nbytes = algorithmic_bytes(K, N, M, weights[0].info.code_bytes, True)
    value = nbytes * args.steps / t["wall_s"] / 1e9
    per_launch_s = t["event_s"] / args.steps
    achieved = nbytes / per_launch_s / 1e9
    out = {
        "metric": "CCQ decode-GEMM effective HBM GB/s (M=1) and TFLOP/s (M=2048), % of roofline",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(t["wall_s"] / args.steps * 1e3, 6), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic (seeded random code bitstream, log-uniform fp16 scales, N(0,1) bf16 activations)",
        "config": {"workload": "config 2: dense decode GEMV, M=1, K=8192, N=8192, 2.0 code bits/weight + fp16 group-64 scales",
                   "M": M, "K": K, "N": N, "weight_copies": args.copies, "bytes_per_step": nbytes, "launch": t["launch"],
                   "timed_repetitions": t["repetitions"], "untimed_launches": t["warm_launches"],
                   "value_is": "bytes_per_step x steps / wall clock of the median repetition (includes the host's graph launch and "
                               "synchronize, which weigh on a short timed region); roofline.achieved uses the HIP events of the same repetition"},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": TRAFFIC_BYTES_PER_LAUNCH, "traffic_source": TRAFFIC_SOURCE,
                     "kernel": "ccq::gemv::kernel<1, 2, 0>", "us_per_launch": round(per_launch_s * 1e6, 3)},
    }

    if "more_rows" in legs:
        # the other row counts of config 2 (M = 8, 16), same weights
        rows_out = []
        for Mr in (8, 16):
            xr = b.bf16_tensor(synth.activations_bf16(Mr, K, synth.rng(2, 30 + Mr)), dev)
            yr = [torch.empty((Mr, N), dtype=torch.bfloat16, device=dev) for _ in weights]
            wsr = torch.empty(max(b.gemm_workspace_bytes(weights[0].desc, Mr), 16), dtype=torch.uint8, device=dev)
            fns = [(lambda w=w, y=y: b.gemm(w, xr, out=y, workspace=wsr)) for w, y in zip(weights, yr)]
            row = {"M": Mr}
            row.update(timed_row(fns, dev, algorithmic_bytes(K, N, Mr, weights[0].info.code_bytes, True), guess_us=12.0))
            rows_out.append(row)
        out["config2_more_rows"] = rows_out

    if "compressed" in legs:
        # the same GEMV with the compressed scales of Sec. 3.4 (2.0625 bits per weight all told)
        weights_c, _ = make_weight_copies(K, N, args.copies, dev, compressed=True)
        ys_c = [torch.empty((M, N), dtype=torch.bfloat16, device=dev) for _ in weights_c]
        fns_c = [(lambda w=w, y=y: b.gemm(w, x, out=y, workspace=ws)) for w, y in zip(weights_c, ys_c)]
        nbytes_c = weights_c[0].info.code_bytes + weights_c[0].info.scale_bytes + 8 * N + 2 * N + 2 * M * K + 2 * M * N
        row = {"workload": "config 2 shape with 4-bit group scales x fp16 super scale per row (Sec. 3.4), M=1"}
        row.update(timed_row(fns_c, dev, nbytes_c, guess_us=8.0))
        out["compressed_scales"] = row
        del weights_c, ys_c, fns_c
    del weights, ys, steps_fns
    torch.cuda.empty_cache()

    if "config3" in legs:
        out["config3"] = config3_leg(dev)
    if "config4" in legs:
        out["config4"] = config4_leg(dev)

    if "prefill" in legs:
        Kp, Np, Mp = 7168, 18432, 2048
        cp = synth.random_codes(Np, Kp // 4, synth.rng(5, 0))
        sp = synth.scales_log_uniform_fp16(Np, Kp // 64, synth.rng(5, 1))
        ap_, bp_ = synth.cluster_params(Np, synth.rng(5, 2))
        wp = b.Weight.from_canonical(Kp, Np, [b.NARROW], cp, sp, ap_, bp_, device=dev)
        xp = b.bf16_tensor(synth.activations_bf16(Mp, Kp, synth.rng(5, 3)), dev)
        yp = torch.empty((Mp, Np), dtype=torch.bfloat16, device=dev)
        wsp = torch.empty(max(b.gemm_workspace_bytes(wp.desc, Mp), 16), dtype=torch.uint8, device=dev)
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
                          "value": round(tf, 2), "unit": "TFLOP/s", "launch": "100 eager launches after 50 untimed ones",
                          "roofline": {"bound": "mfma", "achieved": round(tf, 2), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                       "frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 4)}}
        del wp, xp, yp
        torch.cuda.empty_cache()

    if "ceilings" in legs:
        out["ceilings"] = ceilings_leg(dev, nbytes)
    if "cpu" in legs:
        out["cpu_baseline"] = cpu_baseline(canon, K, N, x_bits)
    out["context"] = {"paper": "CCQ GEMV 8192x8192 M=1 at 2.06 bpw: 0.090 ms on one NVIDIA H20 (Table 4); another machine, not a target"}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
