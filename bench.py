#!/usr/bin/env python3
"""Benchmark of the PrecisionBatching hot path on one MI355X.

A step is one pass of the whole path (activation conversion + bit transpose, 1-bit products,
plane and bitlayer accumulation) over one batch-1 activation vector for every
bits_used = 1..B of one FC layer (default: 4096 x 4096, B = 8): B calls of pb_matmul.
--layout mfma (default) runs the matrix-core kernel (one launch per call), --layout popc the
AND + popcount kernel (activation kernel + product kernel per call).
Weights are resident in HBM before the timed region; each call reads a different copy out of
a pool larger than the last-level cache, so the weight stream really comes from HBM ("cold").

Prints ONE JSON line: effective weight GB/s (bytes of the bitlayers a call must read / time),
matvecs/s, per-bits_used table, the roofline of the dominant kernel and the CPU oracle timed
on a bounded sample.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0                       # MI355X HBM3E, published
ALU_PEAK_GOPS = 256 * 4 * 16 * 2.4          # CUs x SIMDs x lanes x GHz = 39321.6 G int32 lane-ops/s
FP4_PEAK_TFLOPS = 10100.0                   # dense FP4 matrix-core peak, published
LLC_BYTES = 256 << 20                       # last-level (Infinity) cache
POOL_BYTES = 768 << 20                      # weight copies rotated through: 3x the last-level cache


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--min-timed-ms", type=float, default=20.0,
                    help="the K steps are timed repeatedly until at least this much time is measured (a sweep lasts "
                         "tens of microseconds: a region of K steps alone would be shorter than timer noise)")
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--size", type=int, default=4096, help="FC layer is size x size (4096 = the headline config)")
    ap.add_argument("--bits", type=int, default=8, help="stored bitlayers B; bits_used sweeps 1..B")
    ap.add_argument("--layout", choices=["mfma", "popc", "pair"], default="mfma",
                    help="packed layout = kernel: matrix cores (default), AND + popcount, or the matrix cores on the "
                         "layout that stores the digits of the bitlayer pairs")
    ap.add_argument("--warm", action="store_true", help="reuse one weight copy (cache-resident) instead of the pool")
    ap.add_argument("--eager", action="store_true", help="plain launches from Python instead of HIP graph replay")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-batch", action="store_true", help="skip the batched (8192 x 8192, batch 1..64) comparison")
    ap.add_argument("--no-sizes", action="store_true", help="skip the larger layers (8192, 16384: bandwidth asymptote)")
    ap.add_argument("--no-models", action="store_true", help="skip the MLP forward and the 35-step LSTM sequence")
    ap.add_argument("--sweep-only", action="store_true",
                    help="only the bits_used sweep of the headline workload (the run the profiler summaries are made "
                         "from: every launch of the product kernel then belongs to the sweep)")
    ap.add_argument("--batch-point", type=int, default=0, metavar="N",
                    help="only the batched workload at one point: --size x --size (use 8192), bits_used = --bits, N "
                         "vectors, --steps calls (the run the batched profiler summaries are made from; prints its own "
                         "small JSON line, not the headline one)")
    ap.add_argument("--models-only", action="store_true",
                    help="only the MLP forward and the LSTM sequence (the run the profiler summaries of the layer "
                         "sequences are made from; prints its own small JSON line)")
    ap.add_argument("--calib", action="store_true",
                    help="also launch a plain elementwise kernel that reads and writes 256 MiB (reference for the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run of this command)")
    ap.add_argument("--detail", default=None, help="also write the JSON (indented) to this file")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (across GPUs the path would shard by output rows); "
              "--gpus %d is not supported, use --gpus 1" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    from paper_2003_00822_amd import pb, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    pb.lib()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    n, B = args.size, args.bits
    if args.batch_point:
        print(json.dumps(batch_point(torch, pb, synth, dev, n, B, args.batch_point, args.steps, args.layout)),
              flush=True)
        return
    if args.models_only:
        print(json.dumps(model_sequences(torch, pb, synth, dev)), flush=True)
        return
    std = {4096: 0.02, 8192: 0.01}.get(n, 0.01)
    W, X = synth.fc_square(n, std, batch=1, cfg=2 if n == 4096 else 5)
    Wd = torch.from_numpy(W).to(dev)
    Xd = torch.from_numpy(X).to(dev)
    mfma = args.layout != "popc"
    d = pb.pb_desc_init_layout(n, n, B, {"mfma": pb.PB_LAYOUT_TILE16_V1, "popc": pb.PB_LAYOUT_ROWMAJOR_V1,
                                         "pair": pb.PB_LAYOUT_TILE16_PAIRS_V1}[args.layout])
    packed = pb.alloc_packed(d, dev)
    scales = torch.empty(max(B, 4), dtype=torch.float32, device=dev)
    pb.pb_quantize_pack_desc(Wd, d, packed, scales)
    torch.cuda.synchronize()
    del Wd
    pbytes = packed.numel()
    copies = 1 if args.warm else max(2, -(-POOL_BYTES // pbytes))
    pool = [packed] + [packed.clone() for _ in range(copies - 1)]
    ws = pb.alloc_workspace(d, 1, dev)
    Y = torch.empty((1, n), dtype=torch.float32, device=dev)
    layer_bytes = pbytes // B   # bytes of one packed bitlayer (padding included)

    # Work lists.  A "round" visits every weight copy once: G = copies // B steps of B calls (bits_used 1..B).
    # Rounds are captured into HIP graphs so that the Python launch overhead (several microseconds per call,
    # more than a kernel lasts) is outside the measurement; --eager times plain launches instead.
    G = max(1, copies // B) if not args.warm else 6

    def round_calls():
        i = 0
        for _ in range(G):
            for m in range(1, B + 1):
                pb.pb_matmul(pool[i % copies], scales, d, m, Xd, 1, Y, ws)
                i += 1

    def capture(fn):
        if args.eager:
            return fn
        fn()                                   # first call outside capture (lazy module load etc.)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn()
        return g.replay

    def timed(fn, iters):
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / iters   # seconds per iteration

    # ---- the timed region of the contract: W warmup steps, K timed steps (rounded up to whole rounds) ----
    # K steps = ceil(K / G) replays of a graph of G steps (a round visits every weight copy once, so the stream stays
    # cold); the region is repeated until it covers --min-timed-ms.  `steps` reports K as asked, `steps_timed` what ran.
    run_round = capture(round_calls)
    for _ in range(-(-args.warmup // G)):
        run_round()
    rounds = -(-args.steps // G)
    t_region = timed(run_round, rounds) * rounds                     # seconds for `rounds` replays
    repeats = max(1, int(-(-(args.min_timed_ms * 1e-3) // max(t_region, 1e-9))))
    total = t_region
    for _ in range(repeats - 1):
        total += timed(run_round, rounds) * rounds
    steps_timed = rounds * G * repeats
    sec_per_step = total / steps_timed
    step_bytes = layer_bytes * B * (B + 1) // 2
    value = step_bytes / sec_per_step / 1e9

    # plane statistics of this input (written by the activation kernel): planes the popcount kernel multiplies
    pb.pb_act_prep(d, Xd, 1, ws)
    meta = ws[:64].view(torch.int32).cpu().numpy()
    nplanes = int(meta[3]) if not mfma else 32

    # ---- per bits_used: whole call (prep + product) and the product kernel alone ----
    per_m = []
    kern_time_sum = 0.0
    reps = max(2, -(-max(50, args.steps) // max(copies, 48)))

    loop_calls = max(copies, 48)     # calls per captured graph (a graph launch costs several microseconds itself)

    def call_loop(m):
        def f():
            for i in range(loop_calls):
                pb.pb_matmul(pool[i % copies], scales, d, m, Xd, 1, Y, ws)
        return f

    def kern_loop(m):
        def f():
            for i in range(loop_calls):
                pb.pb_matmul_prepared(pool[i % copies], scales, d, m, 1, Y, ws)
        return f

    for m in range(1, B + 1):
        t_call = timed(capture(call_loop(m)), reps) / loop_calls
        # matrix-core layout: the call IS one kernel; popcount layout: the product kernel without the activation kernel
        t_kern = t_call if mfma else timed(capture(kern_loop(m)), reps) / loop_calls
        kern_time_sum += t_kern
        wbytes = layer_bytes * m
        row = {
            "bits_used": m,
            "us_per_call": round(t_call * 1e6, 3),
            "matvecs_per_s": round(1.0 / t_call, 1),
            "eff_weight_GBps": round(wbytes / t_call / 1e9, 1),
            "kernel_us": round(t_kern * 1e6, 3),
            "kernel_GBps": round(wbytes / t_kern / 1e9, 1),
            "kernel_hbm_frac": round(wbytes / t_kern / 1e9 / HBM_PEAK_GBS, 4),
        }
        if mfma:   # flops of the matrix instructions issued: 2 per (weight bit, digit row), 16 digit rows = 32 planes
            row["kernel_mfma_frac"] = round(2.0 * 16 * wbytes * 8 / t_kern / 1e12 / FP4_PEAK_TFLOPS, 4)
        else:      # one AND + one popcount-accumulate per (word, plane)
            row["kernel_alu_frac"] = round(2.0 * nplanes * (wbytes / 4) / t_kern / 1e9 / ALU_PEAK_GOPS, 4)
        per_m.append(row)

    t_prep = 0.0
    if not mfma:
        def prep_loop():
            for _ in range(loop_calls):
                pb.pb_act_prep(d, Xd, 1, ws)
        t_prep = timed(capture(prep_loop), reps) / loop_calls

    # ---- roofline of the dominant kernel over the sweep bits_used = 1..B (average launch) ----
    avg_kernel_s = kern_time_sum / B
    avg_bytes = step_bytes / B
    hbm_frac = avg_bytes / avg_kernel_s / 1e9 / HBM_PEAK_GBS
    roof_hbm = {"bound": "hbm", "achieved": round(avg_bytes / avg_kernel_s / 1e9, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(hbm_frac, 4), "traffic": None}
    if mfma:
        tflops = 2.0 * 16 * avg_bytes * 8 / avg_kernel_s / 1e12   # issued: 16 digit rows (two planes each)
        cmp_frac = tflops / FP4_PEAK_TFLOPS
        roof_cmp = {"bound": "mfma", "achieved": round(tflops, 1), "peak": FP4_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(cmp_frac, 4), "traffic": None}
    else:
        avg_lane_ops = 2.0 * nplanes * (avg_bytes / 4)
        cmp_frac = avg_lane_ops / avg_kernel_s / 1e9 / ALU_PEAK_GOPS
        roof_cmp = {"bound": "alu", "achieved": round(avg_lane_ops / avg_kernel_s / 1e9, 1),
                    "peak": round(ALU_PEAK_GOPS, 1), "unit": "Gop/s", "frac": round(cmp_frac, 4), "traffic": None}
    binding, other = (roof_cmp, roof_hbm) if cmp_frac > hbm_frac else (roof_hbm, roof_cmp)
    binding["kernel"] = other["kernel"] = "k_mfma" if mfma else "k_matvec"
    binding["avg_launch_us"] = other["avg_launch_us"] = round(avg_kernel_s * 1e6, 3)
    binding["active_planes"] = nplanes
    binding["algorithmic_bytes_per_launch"] = int(avg_bytes)
    # measured HBM traffic per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled by a copy kernel of known size):
    # taken from the committed counter summary of this kernel and workload, if there is one
    roof_hbm["traffic"] = measured_traffic("k_mfma" if mfma else "k_matvec", n, B)
    roof_hbm["traffic_source"] = ("profiles/%s_fc%d_b%d_pmc.txt (rocprofv3 --pmc runs of this command; not measured in "
                                  "this run)" % ("k_mfma" if mfma else "k_matvec", n, B))

    if args.calib:
        xc = torch.zeros(64 << 20, dtype=torch.float32, device=dev)
        yc = torch.empty_like(xc)
        for _ in range(4):
            torch.add(xc, 1.0, out=yc)      # one elementwise kernel: reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del xc, yc

    out = {
        "metric": "effective weight GB/s + matvecs/sec at bits_used=1..8 (batch 1); % HBM roofline",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "steps_timed": steps_timed,
        "timed_ms": round(total * 1e3, 3),
        "warmup": args.warmup,
        "ms_per_step": round(sec_per_step * 1e3, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "fp4 base-4 digit operands, fp32 exact sums, int64 accumulate" if mfma
                 else "u32 popcount / int64 accumulate",
        "data": "synthetic",
        "config": {"workload": "FC %dx%d, weight bitlayers B=%d, bits_used swept 1..%d (one call each per step), "
                               "batch 1, x~N(0,1) as 32-bit fixed point" % (n, n, B, B),
                   "weights": "cold: %d copies (%d MiB) rotated" % (copies, copies * pbytes >> 20) if not args.warm
                   else "warm: one copy, cache resident",
                   "kernel": "matrix cores (FP4 MFMA, two bit planes per operand row), one launch per call" if mfma
                   else "AND + popcount, activation kernel + product kernel per call",
                   "launch": "eager" if args.eager else "hip graph replay (%d steps per graph)" % G,
                   "active_planes": nplanes},
        "matvecs_per_s": round(B / sec_per_step, 1),
        "hbm_frac_whole_call": round(value / HBM_PEAK_GBS, 4),
        "prep_kernel_us": round(t_prep * 1e6, 3),
        "per_bits_used": per_m,
        "roofline": binding,
        "roofline_other": other,
    }

    if args.sweep_only:
        if args.detail:
            with open(args.detail, "w") as f:
                json.dump(out, f, indent=1)
        print(json.dumps(out), flush=True)
        return
    out["same_gpu_references"] = same_gpu_references(torch, dev, W, X, per_m)
    if mfma:
        out["same_gpu_references"]["fp4_matrix_calibration"] = mfma_calibration(torch, pb, dev)
        out["table1_analog"] = table1_analog(torch, pb, dev, W, X, out["same_gpu_references"]["fp32_matvec_us"])
    out["paper_reference"] = {
        "what": "Table 1 of the paper: kernel speedup over a Cutlass fp32 matrix-vector product at 4096 x 4096, "
                "batch 1, 32-bit activations; PBatch-n stores n + 1 bitlayers (bits_used = n + 1 here)",
        "hardware": "NVIDIA Tesla T4 (the paper's; another machine: context, not a target)",
        "speedup_vs_fp32": {"PBatch-1": 10.7, "PBatch-2": 8.3, "PBatch-4": 5.3, "PBatch-8": 3.1},
        "stated_bound": "32 / (n + 1)"}
    if not args.no_batch:
        del pool, packed
        torch.cuda.empty_cache()
        out["batch_sweep"] = batch_sweep(torch, pb, synth, dev)
    if not args.no_sizes:
        out["size_sweep"] = size_sweep(torch, pb, dev, args.layout)
    if not args.no_models:
        out["models"] = model_sequences(torch, pb, synth, dev)
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(W, X, B, layer_bytes)
        gpu = {}
        for r in out.get("batch_sweep", {}).get("rows", []):
            if r["kernel"] == "mfma" and r["act_bits"] == 32 and r["batch"] in (1, 4):
                gpu["fc8192_b%d_us" % r["batch"]] = r["us_per_call"]
        mdl = out.get("models", {})
        for r in mdl.get("mlp_784_4096_4096_10", {}).get("rows", []):
            if r["bits_used"] == 8:
                gpu["mlp_m8_us"] = r["us_per_forward"]
        for r in mdl.get("lstm_1500_35_steps", {}).get("rows", []):
            if r["bits_used"] == 8:
                gpu["lstm_m8_us"] = r["us_per_step"]
        out["cpu_baseline_workloads"] = cpu_workloads(synth, gpu)

    line = json.dumps(out)
    if args.detail:
        with open(args.detail, "w") as f:
            json.dump(out, f, indent=1)
    print(line, flush=True)


def table1_analog(torch, pb, dev, W, X, fp32_us):
    """The layout of the paper's Table 1 on this GPU: PBatch-n = n + 1 stored bitlayers, all used, with 8-, 16-
    and 32-bit fixed-point activations (frac_bits 4 / 12 / 16, so that x ~ N(0,1) keeps a few integer bits),
    4096 x 4096, batch 1, cold weights; speedup over the fp32 matrix-vector product measured in this run."""
    n = W.shape[0]
    Wd = torch.from_numpy(W).to(dev)
    Xd = torch.from_numpy(X).to(dev)
    Y = torch.empty((1, n), dtype=torch.float32, device=dev)
    rows = []
    for nbits in (1, 2, 4, 8):
        B = nbits + 1
        for (k, f) in ((8, 4), (16, 12), (32, 16)):
            lin = pb.PackedLinear(Wd, B, frac_bits=f, act_bits=k)
            copies = max(2, POOL_BYTES // lin.packed.numel())
            copies = min(copies, 96)
            pool = [lin.packed] + [lin.packed.clone() for _ in range(copies - 1)]

            def f_():
                for i in range(copies):
                    pb.pb_matmul(pool[i], lin.scales, lin.desc, B, Xd, 1, Y, lin.workspace)
            t = _graph_time(torch, f_, 1) / copies
            rows.append({"method": "PBatch-%d" % nbits, "bitlayers": B, "act_bits": k, "us_per_call": round(t * 1e6, 2),
                         "speedup_vs_fp32": round(fp32_us / (t * 1e6), 2), "bound": round(32.0 / B, 2)})
            del pool, lin
    torch.cuda.empty_cache()
    return {"workload": "FC %dx%d, batch 1, bits_used = bitlayers" % (n, n), "fp32_matvec_us": fp32_us, "rows": rows}


def same_gpu_references(torch, dev, W, X, per_m):
    """Two reference points measured in this run on this GPU: (1) the bandwidth a plain elementwise kernel reaches
    on 256 MiB (read + write), the practical ceiling next to the 8 TB/s of the data sheet; (2) the fp32
    matrix-vector product the quantized one replaces (torch.mv = the vendor BLAS), cold weights, in a HIP graph,
    and the speedup of every bits_used over it (the paper's Table 1 metric, here on one machine)."""
    xc = torch.zeros(64 << 20, dtype=torch.float32, device=dev)
    yc = torch.empty_like(xc)
    torch.add(xc, 1.0, out=yc)
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(10):
        torch.add(xc, 1.0, out=yc)
    e1.record()
    torch.cuda.synchronize()
    stream_gbps = 2 * xc.numel() * 4 * 10 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del xc, yc
    n = W.shape[0]
    Wd = torch.from_numpy(W).to(dev)
    copies = max(2, POOL_BYTES // (Wd.numel() * 4))
    pool = [Wd] + [Wd.clone() for _ in range(copies - 1)]
    xd = torch.from_numpy(X[0]).to(dev)
    y = torch.empty(n, dtype=torch.float32, device=dev)

    def f():
        for i in range(copies):
            torch.mv(pool[i], xd, out=y)
    t = _graph_time(torch, f, 1) / copies
    del pool, Wd
    torch.cuda.empty_cache()
    return {"stream_elementwise_GBps": round(stream_gbps, 1),
            "fp32_matvec_us": round(t * 1e6, 2), "fp32_matvec_GBps": round(n * n * 4 / t / 1e9, 1),
            "speedup_vs_fp32": {str(r["bits_used"]): round(t * 1e6 / r["us_per_call"], 2) for r in per_m},
            "bound_32_over_bits_used": {str(r["bits_used"]): round(32.0 / r["bits_used"], 2) for r in per_m}}


def mfma_calibration(torch, pb, dev):
    """The rate of the product kernel's FP4 matrix instruction on this GPU (the calibration loop of `paper_2003_00822_amd/csrc/calib`, a
    library of its own beside the product: constant operands, two waves per SIMD on every compute unit): alone, with the expansion of one packed weight word per four
    instructions, and with the kernel's epilogue per chain of four.  On a SIMD the matrix and the vector-ALU
    instructions take turns, so the third figure is the ceiling of the batched regime with this much ALU work."""
    from paper_2003_00822_amd import calib
    cus = torch.cuda.get_device_properties(dev).multi_processor_count
    buf = torch.empty(cus, dtype=torch.float32, device=dev)
    res = {}
    for mode, name in ((0, "instructions_alone"), (1, "with_weight_expansion"), (2, "with_expansion_and_epilogue")):
        ts = []
        for iters in (200, 2200):
            calib.pb_calib_mfma(mode, iters, cus, buf)
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            calib.pb_calib_mfma(mode, iters, cus, buf)
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1) * 1e-3)
        flops = 65536.0 * 16 * 2000 * 8 * cus
        tf = flops / (ts[1] - ts[0]) / 1e12
        res[name] = {"TFLOPs": round(tf, 1), "frac_of_peak": round(tf / FP4_PEAK_TFLOPS, 4)}
    return res


def measured_traffic(kernel, n, B):
    """HBM bytes per launch from profiles/<kernel>_fc<n>_b<B>_pmc.txt (line 'traffic_bytes_per_launch: N'), else None."""
    path = os.path.join(ROOT, "profiles", "%s_fc%d_b%d_pmc.txt" % (kernel, n, B))
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch:"):
                    return int(float(line.split(":")[1]))
    except OSError:
        pass
    return None


def model_sequences(torch, pb, synth, dev):
    """The layer sequences of the paper's models on the matrix-core kernel, each captured in one HIP graph:
    the 3-layer MLP 784-4096-4096-10 (one launch per layer, bias-free, ReLU fused into the store) and 35
    sequential steps of the LSTM cell (hidden = input = 1500, fused gate matrix 6000 x 3000, one launch per step:
    product and cell update together, hidden state ping-ponged between two buffers).  Batch 1, weights warm
    (a model's own weights, a few MiB, are what stays in cache between its steps)."""
    res = {}
    # ---- MLP
    Ws, X = synth.mlp()
    B = 8
    lins = [pb.PackedLinear(torch.from_numpy(W).to(dev), B) for W in Ws]
    acts = [torch.from_numpy(X).to(dev)] + [torch.empty((1, W.shape[0]), dtype=torch.float32, device=dev) for W in Ws]
    rows = []
    for m in (2, 4, 8):
        def fwd():
            for li, lin in enumerate(lins):
                pb.pb_matmul_bias_act(lin.packed, lin.scales, lin.desc, m, acts[li], 1, None,
                                      pb.PB_ACT_RELU if li < 2 else pb.PB_ACT_NONE, acts[li + 1], lin.workspace)
        rows.append({"bits_used": m, "us_per_forward": round(_graph_time(torch, fwd, 32) * 1e6, 2)})
    res["mlp_784_4096_4096_10"] = {"launches_per_forward": 3, "weight_bits_stored": B, "rows": rows}
    del lins
    # ---- LSTM
    H = I = 1500
    W, xs, bias = synth.lstm(H, I, steps=35)
    rows = []
    xs_d = [torch.from_numpy(x).to(dev) for x in xs]
    bias_d = torch.from_numpy(bias).to(dev)
    for B in (4, 8):
        lin = pb.PackedLinear(torch.from_numpy(W).to(dev), B, layout=pb.PB_LAYOUT_TILE16_GATES_V1)
        h = [torch.zeros((1, H), device=dev), torch.zeros((1, H), device=dev)]
        c = torch.zeros((1, H), device=dev)
        for m in sorted({2, B}):
            def seq():
                for t in range(35):
                    pb.pb_lstm_cell(lin.packed, lin.scales, lin.desc, m, xs_d[t], I, h[t & 1], c, bias_d,
                                    h[(t + 1) & 1], c, 1, lin.workspace)
            t35 = _graph_time(torch, seq, 1)
            rows.append({"weight_bits_stored": B, "bits_used": m, "us_per_step": round(t35 * 1e6 / 35, 2),
                         "us_per_35_steps": round(t35 * 1e6, 1)})
        del lin
    res["lstm_1500_35_steps"] = {"launches_per_step": 1, "rows": rows}
    return res


def _graph_time(torch, fn, per_graph):
    """Seconds per call of fn, captured `per_graph` times into one HIP graph and replayed."""
    def body():
        for _ in range(per_graph):
            fn()
    body()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        body()
    g.replay()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(20):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e-3 / (20 * per_graph)


def size_sweep(torch, pb, dev, layout):
    """Larger square layers (the north star's "4096 x 4096 +"): a 4096^2 bitlayer is 2 MiB, a fraction of a
    microsecond of HBM time, so the per-call figures of the headline workload are latency-bound; these show the
    bandwidth the same kernel reaches once a call streams tens of MiB.  Cold weights (copies rotated through
    768 MiB), HIP-graph replay, batch 1.  Weights and activations ~N(0, 0.01) / N(0, 1) from the device generator."""
    rows = []
    gen = torch.Generator(device=dev)
    gen.manual_seed(200300822 + 6000)
    lay = {"mfma": pb.PB_LAYOUT_TILE16_V1, "popc": pb.PB_LAYOUT_ROWMAJOR_V1, "pair": pb.PB_LAYOUT_TILE16_PAIRS_V1}[layout]
    for n in (8192, 16384):
        B = 8
        Wd = torch.randn((n, n), device=dev, generator=gen) * 0.01
        lin = pb.PackedLinear(Wd, B, layout=lay)
        del Wd
        X = torch.randn((1, n), device=dev, generator=gen)
        Y = torch.empty((1, n), dtype=torch.float32, device=dev)
        copies = max(3, POOL_BYTES // lin.packed.numel())
        pool = [lin.packed] + [lin.packed.clone() for _ in range(copies - 1)]
        layer_bytes = lin.packed.numel() // B
        calls = max(copies, 24)      # per captured graph (a graph launch costs several microseconds itself)
        for m in range(1, B + 1):
            def f():
                for i in range(calls):
                    pb.pb_matmul(pool[i % copies], lin.scales, lin.desc, m, X, 1, Y, lin.workspace)
            f()
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                f()
            reps = max(4, 192 // calls)
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            g.replay()
            torch.cuda.synchronize()
            e0.record()
            for _ in range(reps):
                g.replay()
            e1.record()
            torch.cuda.synchronize()
            t = e0.elapsed_time(e1) * 1e-3 / (reps * calls)
            rows.append({"size": n, "bits_used": m, "us_per_call": round(t * 1e6, 2),
                         "eff_weight_GBps": round(layer_bytes * m / t / 1e9, 1),
                         "hbm_frac": round(layer_bytes * m / t / 1e9 / HBM_PEAK_GBS, 4)})
        del pool, lin
        torch.cuda.empty_cache()
    return {"workload": "FC n x n, B=8, batch 1, cold weights, whole call (one launch)", "rows": rows}


def batch_sweep(torch, pb, synth, dev):
    """Large FC layer (8192 x 8192, B = 8, bits_used = 8) at batch 1 .. 1024: the regime where the product is a
    dense contraction.  Both kernels, weights warm (the 64 MiB stay in the last-level cache between the passes
    of one call anyway).  Nominal work = rows * cols * bits_used * 32 planes * batch 1-bit multiply-accumulates.
    Matrix-core rows: the FP4 instructions issued against the matrix peak.  Popcount rows: the vector-ALU lane
    operations the kernel executes (one AND + one popcount-accumulate per 32-bit weight word and ACTIVE plane: planes
    that are empty or copies of the sign plane are skipped, the count comes from the plane statistics the activation
    kernel leaves in the workspace) against the integer vector-ALU peak.  Narrower activations (Section 3.1, Table 1)
    at batch 16 and 64 on the matrix-core kernel."""
    n, B, m = 8192, 8, 8
    W, _ = synth.fc_square(n, 0.01, batch=1, cfg=5)
    Wd = torch.from_numpy(W).to(dev)
    del W
    rows = []
    gen = torch.Generator(device=dev)
    gen.manual_seed(200300822 + 5000)
    NMAX = 1024
    X = torch.randn((NMAX, n), device=dev, generator=gen)
    Y = torch.empty((NMAX, n), dtype=torch.float32, device=dev)

    def time_calls(f, N):
        """Seconds per call: the best of three trials of back-to-back eager calls (the first calls after a change of
        kernel run at other clocks; single trials of this sweep differed by up to 20 %)."""
        for _ in range(3):
            f()
        reps = 20 if N <= 16 else (8 if N <= 64 else 3)
        best = float("inf")
        for _ in range(3):
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(reps):
                f()
            e1.record()
            torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1) * 1e-3 / reps)
        return best

    for name, lay, batches in (("mfma", pb.PB_LAYOUT_TILE16_V1, (1, 4, 16, 64, 256, 1024)),
                               ("mfma, pairs layout", pb.PB_LAYOUT_TILE16_PAIRS_V1, (1, 4, 16, 64, 256, 1024)),
                               ("popc", pb.PB_LAYOUT_ROWMAJOR_V1, (1, 4, 16, 64, 256))):
        lin = pb.PackedLinear(Wd, B, max_batch=max(batches), layout=lay)
        for N in batches:
            def f():
                pb.pb_matmul(lin.packed, lin.scales, lin.desc, m, X[:N], N, Y[:N], lin.workspace)
            t = time_calls(f, N)
            macs = float(n) * n * m * 32 * N
            row = {"kernel": name, "batch": N, "act_bits": 32, "us_per_call": round(t * 1e6, 1),
                   "us_per_vector": round(t * 1e6 / N, 2), "Tbitmac_per_s": round(macs / t / 1e12, 1)}
            if name.startswith("mfma"):
                # matrix instructions issued: 16 digit rows (two planes each) per vector, and with more than one
                # vector (on the pairs layout: always) two bitlayers per instruction
                units = m if (N == 1 and name == "mfma") else (m + 1) // 2
                row["mfma_issued_TFLOPs"] = round(2.0 * 16 * n * n * units * N / t / 1e12, 1)
                row["mfma_frac"] = round(2.0 * 16 * n * n * units * N / t / 1e12 / FP4_PEAK_TFLOPS, 4)
            else:
                meta = lin.workspace[:N * 64].view(torch.int32).view(N, 16).cpu().numpy()
                planes = float(meta[:, 3].sum())                       # active planes, summed over the vectors
                lane_ops = 2.0 * planes * (n * (n // 32)) * m          # AND + popcount per (word, active plane)
                row["active_planes_per_vector"] = round(planes / N, 2)
                row["alu_lane_Gops"] = round(lane_ops / t / 1e9, 1)
                row["alu_frac"] = round(lane_ops / t / 1e9 / ALU_PEAK_GOPS, 4)
            rows.append(row)
        del lin
    # narrower activations on the matrix-core kernel (frac_bits as in table1_analog)
    for name, lay in (("mfma", pb.PB_LAYOUT_TILE16_V1), ("mfma, pairs layout", pb.PB_LAYOUT_TILE16_PAIRS_V1)):
        for (k, fb) in ((8, 4), (16, 12)):
            lin = pb.PackedLinear(Wd, B, max_batch=64, frac_bits=fb, act_bits=k, layout=lay)
            for N in (16, 64):
                def f():
                    pb.pb_matmul(lin.packed, lin.scales, lin.desc, m, X[:N], N, Y[:N], lin.workspace)
                t = time_calls(f, N)
                rows.append({"kernel": name, "batch": N, "act_bits": k, "us_per_call": round(t * 1e6, 1),
                             "us_per_vector": round(t * 1e6 / N, 2),
                             "Tbitmac_per_s": round(float(n) * n * m * k * N / t / 1e12, 1)})
            del lin
    # rows of 16384 columns: the kernels that take the columns in several passes (batch 16 and 64)
    del Wd, X, Y
    nw = 16384
    W, _ = synth.fc_square(nw, 0.01, batch=1, cfg=6)
    Wd = torch.from_numpy(W).to(dev)
    del W
    X = torch.randn((64, nw), device=dev, generator=gen)
    Y = torch.empty((64, nw), dtype=torch.float32, device=dev)
    wide = []
    for name, lay in (("mfma", pb.PB_LAYOUT_TILE16_V1), ("mfma, pairs layout", pb.PB_LAYOUT_TILE16_PAIRS_V1)):
        lin = pb.PackedLinear(Wd, B, max_batch=64, layout=lay)
        for N in (16, 64):
            def f():
                pb.pb_matmul(lin.packed, lin.scales, lin.desc, m, X[:N], N, Y[:N], lin.workspace)
            t = time_calls(f, N)
            issued = 2.0 * 16 * nw * nw * ((m + 1) // 2) * N / t / 1e12
            wide.append({"kernel": name, "batch": N, "act_bits": 32, "us_per_call": round(t * 1e6, 1),
                         "us_per_vector": round(t * 1e6 / N, 2),
                         "Tbitmac_per_s": round(float(nw) * nw * m * 32 * N / t / 1e12, 1),
                         "mfma_issued_TFLOPs": round(issued, 1), "mfma_frac": round(issued / FP4_PEAK_TFLOPS, 4)})
        del lin
    return {"workload": "FC 8192x8192, B=8, bits_used=8, x~N(0,1), batch 1..1024, weights warm",
            "alu_peak_Gops": round(ALU_PEAK_GOPS, 1), "fp4_peak_TFLOPs": FP4_PEAK_TFLOPS, "rows": rows,
            "wide_rows": {"workload": "FC 16384x16384, B=8, bits_used=8, x~N(0,1), batch 16 and 64, weights warm",
                          "rows": wide}}


def batch_point(torch, pb, synth, dev, n, B, N, steps, layout):
    """One point of the batched regime by itself (cfg 5 recipe: W ~N(0, 0.01), x ~N(0, 1)), eager launches."""
    W, _ = synth.fc_square(n, 0.01, batch=1, cfg=5)
    lay = {"mfma": pb.PB_LAYOUT_TILE16_V1, "popc": pb.PB_LAYOUT_ROWMAJOR_V1, "pair": pb.PB_LAYOUT_TILE16_PAIRS_V1}[layout]
    lin = pb.PackedLinear(torch.from_numpy(W).to(dev), B, max_batch=N, layout=lay)
    gen = torch.Generator(device=dev)
    gen.manual_seed(200300822 + 5000)
    X = torch.randn((N, n), device=dev, generator=gen)
    Y = torch.empty((N, n), dtype=torch.float32, device=dev)
    for _ in range(3):
        pb.pb_matmul(lin.packed, lin.scales, lin.desc, B, X, N, Y, lin.workspace)
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(steps):
        pb.pb_matmul(lin.packed, lin.scales, lin.desc, B, X, N, Y, lin.workspace)
    e1.record()
    torch.cuda.synchronize()
    t = e0.elapsed_time(e1) * 1e-3 / steps
    units = B if (N == 1 and layout == "mfma") else (B + 1) // 2
    return {"workload": "FC %dx%d, B=bits_used=%d, batch %d, x~N(0,1), weights warm, kernel %s" % (n, n, B, N, layout),
            "steps": steps, "us_per_call": round(t * 1e6, 1),
            "Tbitmac_per_s": round(float(n) * n * B * 32 * N / t / 1e12, 1),
            "mfma_issued_TFLOPs": round(2.0 * 16 * n * n * units * N / t / 1e12, 1) if layout != "popc" else None}


def _host_threads():
    return max(1, min(16, os.cpu_count() or 1))


def _oracle_call_time(call, budget_s=2.5, max_reps=200):
    """Median seconds of `call()` over as many repetitions as fit the budget (at least 3)."""
    ts = []
    t_end = time.perf_counter() + budget_s
    while len(ts) < 3 or (time.perf_counter() < t_end and len(ts) < max_reps):
        t0 = time.perf_counter()
        call()
        ts.append(time.perf_counter() - t0)
    ts.sort()
    return ts[len(ts) // 2], len(ts)


def cpu_baseline(W, X, B, layer_bytes):
    """The oracle's packed-word tier (plain C, uint64 AND + popcount), timed as it stands on the host cores:
    the same sweep bits_used = 1..B, rows split over threads, repeated for a bounded time."""
    from concurrent.futures import ThreadPoolExecutor

    from oracle import pb_oracle as po

    R, C = W.shape
    prep = po.prepare(W, B)
    lw = po.pack_words(prep["layers"])
    threads = _host_threads()
    bounds = [(R * t // threads, R * (t + 1) // threads) for t in range(threads)]

    def sweep(pool):
        for m in range(1, B + 1):
            list(pool.map(lambda b: po.matmul_words(lw, prep["scales"], m, C, X, r0=b[0], r1=b[1], want_A=False),
                          bounds))

    with ThreadPoolExecutor(threads) as pool:
        t0 = time.perf_counter()
        sweep(pool)
        one = time.perf_counter() - t0
        reps = int(min(1000, max(1, 12.0 / max(one, 1e-3))))    # about 12 s of host time
        t0 = time.perf_counter()
        for _ in range(reps):
            sweep(pool)
        dt = (time.perf_counter() - t0) / reps
    # the same sweep on one thread (best of three)
    dt1 = float("inf")
    for _ in range(3):
        t0 = time.perf_counter()
        for m in range(1, B + 1):
            po.matmul_words(lw, prep["scales"], m, C, X, want_A=False)
        dt1 = min(dt1, time.perf_counter() - t0)
    step_bytes = layer_bytes * B * (B + 1) // 2
    return {"value": round(step_bytes / dt / 1e9, 3), "unit": "GB/s", "cores": threads, "kind": "oracle",
            "value_one_thread": round(step_bytes / dt1 / 1e9, 3),
            "sample": "oracle packed-word tier (uint64 AND+popcount, gcc -O2), full %dx%d layer, bits_used 1..%d, "
                      "%d sweeps, %.2f s each" % (R, C, B, reps, dt),
            "matvecs_per_s": round(B / dt, 2)}


def cpu_workloads(synth, gpu):
    """The oracle timed on the other workloads, beside the GPU figures of the same run (`gpu`: microseconds per call
    where this run measured the workload): config 1 (1024 x 1024, B = 4; both tiers: Algorithm 2 bit by bit on byte
    arrays, and packed words), config 3 (MLP forward, three layers), config 4 (one LSTM step: gate product + cell
    update), config 5 (8192 x 8192, bits_used 8, batch 1 and 4).  Packed-word tier with the rows split over
    `cores` threads and on one thread; the definition-level tier has no row range and runs on one thread.
    Each leg is the median of at least 3 calls within about 2.5 s."""
    import numpy as np
    from concurrent.futures import ThreadPoolExecutor

    from oracle import pb_oracle as po

    threads = _host_threads()
    legs = []

    def words_leg(name, mats, X, m, pool, post=None, gpu_us=None):
        """mats: list of (lw, scales, R, C); a call applies them one after the other (ReLU between, like the MLP)."""
        def run(nthreads):
            def call():
                x = X
                for li, (lw, sc, R, C) in enumerate(mats):
                    if nthreads == 1:
                        _, y = po.matmul_words(lw, sc, m, C, x, want_A=False)
                    else:
                        bounds = [(R * t // nthreads, R * (t + 1) // nthreads) for t in range(nthreads)]
                        parts = list(pool.map(lambda b: po.matmul_words(lw, sc, m, C, x, r0=b[0], r1=b[1],
                                                                        want_A=False)[1][:, b[0]:b[1]], bounds))
                        y = np.concatenate(parts, axis=1)
                    x = np.maximum(y, 0.0) if li + 1 < len(mats) else y
                if post:
                    post(x)
            return _oracle_call_time(call)
        tN, nN = run(threads)
        t1, n1 = run(1)
        leg = {"workload": name, "tier": "packed words", "bits_used": m, "cores": threads,
               "ms_per_call": round(tN * 1e3, 3), "ms_per_call_one_thread": round(t1 * 1e3, 3), "calls_timed": [nN, n1]}
        if gpu_us:
            leg["gpu_us_per_call"] = gpu_us
            leg["gpu_over_oracle"] = round(tN * 1e6 / gpu_us, 1)
        legs.append(leg)

    def pack(W, bits):
        prep = po.prepare(W, bits)
        return (po.pack_words(prep["layers"]), prep["scales"], W.shape[0], W.shape[1]), prep

    with ThreadPoolExecutor(threads) as pool:
        # config 1
        W, X = synth.fc_small()
        mat, prep = pack(W, 4)
        t, nrep = _oracle_call_time(lambda: po.matmul_bitserial(prep["layers"], prep["scales"], prep["s"], 4, X))
        legs.append({"workload": "cfg1 FC 1024x1024 B=4", "tier": "definition level (Algorithm 2 bit by bit)",
                     "bits_used": 4, "cores": 1, "ms_per_call": round(t * 1e3, 3), "calls_timed": [nrep]})
        words_leg("cfg1 FC 1024x1024 B=4", [mat], X, 4, pool)
        # config 3
        Ws, X = synth.mlp()
        words_leg("cfg3 MLP 784-4096-4096-10 forward, B=8", [pack(Wl, 8)[0] for Wl in Ws], X, 8, pool,
                  gpu_us=gpu.get("mlp_m8_us"))
        # config 4: one step
        Wg, xs, bias = synth.lstm(1500, 1500, steps=1)
        mat, _ = pack(Wg, 8)
        xh = np.concatenate([xs[0], np.zeros((1, 1500), dtype=np.float32)], axis=1)
        c0 = np.zeros((1, 1500), dtype=np.float32)
        words_leg("cfg4 LSTM step 6000x3000 B=8 (+ cell update)", [mat], xh, 8, pool,
                  post=lambda g: po.lstm_pointwise(g, bias, c0), gpu_us=gpu.get("lstm_m8_us"))
        # config 5
        W, X = synth.fc_square(8192, 0.01, batch=4, cfg=5)
        mat, _ = pack(W, 8)
        del W
        words_leg("cfg5 FC 8192x8192 B=8 batch 1", [mat], X[:1], 8, pool, gpu_us=gpu.get("fc8192_b1_us"))
        words_leg("cfg5 FC 8192x8192 B=8 batch 4", [mat], X, 8, pool, gpu_us=gpu.get("fc8192_b4_us"))
    return {"kind": "oracle", "unit": "ms per call", "legs": legs}


if __name__ == "__main__":
    main()
