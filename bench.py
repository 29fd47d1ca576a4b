#!/usr/bin/env python3
"""Benchmark: one MoE FFN layer, index build + forward + backward, on one MI355X.

A step is one pass of the whole hot path (hexa_moe_index, hexa_moe_fwd, hexa_moe_bwd) over one
synthetic batch that is already resident in HBM.  Prints ONE JSON line.

  value     useful TFLOP/s = 12 * T*k * d_model * d_ff / step time   (2 GEMMs forward, 4 backward)
  roofline  the kernel with the largest share of the step (always a bf16 MFMA contraction launch;
            the backward of a linear layer is one launch of two contractions): its 2*A*d*f FLOP per
            contraction over its average launch duration, measured with HIP events that the library
            records on the launch stream, against the 2.5 PFLOP/s dense bf16 MFMA peak; the rates of
            all contraction launches are listed under contraction_tflops
            (sustained_mfma_peak: a register-only MFMA loop timed in the same run, i.e. the
            matrix rate at the clock the power limit allows)
  cpu_baseline  the CPU oracle, as it stands, timed on a bounded sample of the same workload
"""
import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

BF16_MFMA_PEAK_TFLOPS = 2500.0
METRIC = "MoE layer fwd+bwd useful TFLOP/s on 1 MI355X + % of bf16 MFMA peak"
# contraction launches: label -> number of 2*A*d*f contractions in the launch (the backward of each
# linear layer runs its input-gradient and weight-gradient contractions in one grid)
GEMM_LABELS = {"fc1": 1, "fc2": 1, "bwd_fc2": 2, "bwd_fc1": 2}
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "c5_gemm_pmc_counters.md")


def profiled_traffic():
    """HBM-side bytes per launch at C5 from the committed rocprofv3 summary (FETCH_SIZE and WRITE_SIZE,
    calibrated with a plain 1 GiB copy): {launch label: bytes}.  The counters cannot be read from
    inside a timed run, so this is the profile's figure, not this run's; {} if the table is missing."""
    out = {}
    try:
        for line in open(TRAFFIC_FILE):
            cells = [c.strip() for c in line.split("|")]
            if len(cells) > 6 and cells[1].startswith("gemm_bf16") and "(" in cells[1]:
                label = cells[1].rsplit("(", 1)[1].rstrip(")")
                out[label] = (float(cells[3]) + float(cells[5])) * 1e9
    except (OSError, ValueError):
        return {}
    return out


def cpu_baseline(w, data, sample_tokens=2048, col_frac=16):
    """Oracle (fp64 loop nest) timed on the first `sample_tokens` tokens of the batch with all
    experts resident; the per-expert gradients on f/col_frac of the hidden units (each hidden
    unit is an independent, equal share of that work).  Returns useful TFLOP/s per the same
    12*d*f FLOP per assignment."""
    from oracle import hexa_oracle as O
    O.build()
    S = min(sample_tokens, w.T)
    h = lambda t: t.detach().to("cpu").float().numpy()
    x, dY, gate = h(data["x"][:S]), h(data["dY"][:S]), h(data["gate"][:S])
    idx = data["topk_idx"][:S].cpu().numpy()
    W1, b1, W2, b2 = h(data["W1"]), h(data["b1"]), h(data["W2"]), h(data["b2"])
    ncols = max(1, w.d_ff // col_frac)
    cols = np.arange(ncols, dtype=np.int32)
    c0 = time.process_time()
    t0 = time.perf_counter()
    O.fwd(x, idx, gate, W1, b1, W2, b2)
    t1 = time.perf_counter()
    O.bwd_tokens(x, idx, gate, W1, b1, W2, b2, dY)
    t2 = time.perf_counter()
    O.bwd_experts(x, idx, gate, W1, b1, W2, dY, cols=cols)
    t3 = time.perf_counter()
    c1 = time.process_time()
    per_assign = ((t1 - t0) + (t2 - t1) + (t3 - t2) * (w.d_ff / ncols)) / (S * w.k)
    tflops = 12.0 * w.d_model * w.d_ff / per_assign / 1e12
    # threads the oracle's OpenMP regions ran with: the team size, capped by the CPUs this process
    # may run on; busy = CPU seconds per wall second over the timed calls (what the box really gave)
    threads = min(int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)), len(os.sched_getaffinity(0)))
    busy = (c1 - c0) / max(t3 - t0, 1e-9)
    return {
        "value": tflops, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
        "cpu_seconds_per_wall_second": round(busy, 2),
        "sample": (f"first {S} tokens ({S * w.k} assignments) of the same batch, all {w.E} experts "
                   f"resident; fwd {t1 - t0:.2f}s + dx/dgate {t2 - t1:.2f}s + weight/bias grads on "
                   f"{ncols}/{w.d_ff} hidden units {t3 - t2:.2f}s (scaled x{w.d_ff // ncols}); "
                   f"rate = 12*d*f / time per assignment; {threads} OpenMP threads on "
                   f"{len(os.sched_getaffinity(0))} schedulable CPUs, {busy:.1f} of them busy on average"),
    }


def hbm_steps(w, kernels, copy_gbps):
    es = 4 if w.dtype == "f32" else 2
    A, T, d, k = w.A, w.T, w.d_model, w.k
    algo = {
        # y_t = sum_j g o_a: o [A,d] and inv, gate in; y [T,d] out
        "combine_y": A * d * es + T * d * es + A * 8,
        # dY (gathered) and o in; dout out (+ perm, gate, dgate)
        "bwd_prologue": A * d * es * 3 + A * 12,
        "combine_dx": A * d * es + T * d * es + A * 4,
        "index_scatter": A * 4 + A * 8,
    }
    out = {"copy_GBps": round(copy_gbps, 1)}
    for name, nbytes in algo.items():
        if name in kernels and kernels[name]["ms"] > 0:
            gbps = nbytes / (kernels[name]["ms"] * 1e-3) / 1e9
            out[name] = {"ms": round(kernels[name]["ms"], 4), "bytes": int(nbytes), "GBps": round(gbps, 1),
                         "frac_of_hbm_peak": round(gbps / 8000.0, 3), "frac_of_copy": round(gbps / copy_gbps, 3)}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="C5")
    ap.add_argument("--routing", default=None, help="override the routing recipe (zipf, forced, ...)")
    ap.add_argument("--dtype", default=None, help="override the element type (bf16, f16, f32)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="time replays of the step captured into one HIP graph (launch-latency regime: "
                         "small workloads); per-kernel events are then taken from an eager pass")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (reference for rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build is single-GPU (all experts resident, no collectives); "
                 "run with --gpus 1")

    from paper_2411_01288_amd import binding as B
    from paper_2411_01288_amd.workloads import generate, workload

    ov = {"routing": args.routing} if args.routing else {}
    if args.dtype:
        ov["dtype"] = args.dtype
    w = workload(args.workload, **ov)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    data = generate(w, dev)
    shape = B.make_shape(w.T, w.d_model, w.d_ff, w.E, w.k, w.dtype)
    idx = B.alloc_idx(shape, dev)
    iscratch = torch.empty(max(B.index_scratch_bytes(shape), 256), dtype=torch.uint8, device=dev)
    ws = B.alloc_workspace(shape, dev)
    y = torch.empty((w.T, w.d_model), dtype=data["x"].dtype, device=dev)
    grads = None

    def step():
        nonlocal grads
        B.hexa_moe_index(shape, data["topk_idx"], idx, iscratch)
        B.hexa_moe_fwd(shape, data["x"], data["topk_idx"], data["gate"], data["W1"], data["b1"],
                       data["W2"], data["b2"], idx, ws, y)
        grads = B.hexa_moe_bwd(shape, data["dY"], data["x"], data["topk_idx"], data["gate"],
                               data["W1"], data["W2"], idx, ws, out=grads)

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.graph:
        B.profile_enable(True)      # per-kernel figures from eager steps, outside the timed region
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        prof = B.profile_read()
        B.profile_enable(False)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    else:
        B.profile_enable(True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        prof = B.profile_read()
        B.profile_enable(False)

    # the matrix rate the part sustains under its power limit: a register-only MFMA loop, ~50 ms
    sink = torch.zeros(1, dtype=torch.float32, device=dev)
    B.mfma_probe(1024, 2000, sink)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    probe_flop = B.mfma_probe(1024, 30000, sink)
    e1.record()
    torch.cuda.synchronize()
    sustained = probe_flop / (e0.elapsed_time(e1) * 1e-3) / 1e12
    probes = {"16x16x32_random": round(sustained, 1)}
    for name, variant in (("16x16x32_zero_operands", 1), ("32x32x16_random", 2)):
        B.mfma_probe(1024, 2000, sink, variant)
        e0.record()
        flop = B.mfma_probe(1024, 30000, sink, variant)
        e1.record()
        torch.cuda.synchronize()
        probes[name] = round(flop / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1)

    # the router front-end (the step before the path; not part of `value`): HBM-bound,
    # T*E*4 bytes of logits in, T*k*8 bytes out
    logits = torch.randn((w.T, w.E), dtype=torch.float32, device=dev)
    rt_idx, rt_gate = B.hexa_moe_route(shape, logits)
    e0.record()
    for _ in range(10):
        B.hexa_moe_route(shape, logits, B.GATE_SOFTMAX_SELECTED, rt_idx, rt_gate)
    e1.record()
    torch.cuda.synchronize()
    route_ms = e0.elapsed_time(e1) / 10
    route_bytes = w.T * w.E * 4 + w.T * w.k * 8

    # plain device copy (1 GiB read + 1 GiB written) as the yardstick for the bandwidth-bound steps
    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    dst.copy_(src)
    e0.record()
    for _ in range(5):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    copy_gbps = 5 * 2 * (1 << 30) / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del src, dst

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tflops = w.useful_flop / (ms_per_step * 1e-3) / 1e12
    kernels = {k: {"ms": v[0] / v[1], "launches": v[1]} for k, v in prof.items()}
    gemm_flop = 2.0 * w.A * w.d_model * w.d_ff
    # the dominant kernel: the contraction launch that takes the largest share of the step
    rates = {k: GEMM_LABELS[k] * gemm_flop / (kernels[k]["ms"] * 1e-3) / 1e12 for k in kernels if k in GEMM_LABELS}
    dom = max(rates, key=lambda k: kernels[k]["ms"])
    gemm_flop *= GEMM_LABELS[dom]
    achieved = rates[dom]
    counts = idx["counts"].cpu().numpy()
    ksum = lambda names: sum(kernels[k]["ms"] * kernels[k]["launches"] for k in names if k in kernels) / args.steps
    idx_ms = ksum(["index_count", "index_scan", "index_scatter"])
    fwd_ms = ksum(["fc1", "fc2", "combine_y"]) + 0.5 * ksum(["worklists"])
    all_ms = ksum(list(kernels))
    out = {
        "metric": METRIC, "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "pct_of_bf16_mfma_peak": 100.0 * tflops / BF16_MFMA_PEAK_TFLOPS,
        "launch": "hip_graph_replay" if args.graph else "eager",
        "config": {"workload": f"{w.name}: one MoE FFN layer fwd+bwd incl. index build, T={w.T} "
                               f"d_model={w.d_model} d_ff={w.d_ff} E={w.E} top-{w.k}, routing={w.routing}",
                   "T": w.T, "d_model": w.d_model, "d_ff": w.d_ff, "E": w.E, "k": w.k,
                   "routing": w.routing,
                   "tokens_per_expert": {"min": int(counts.min()), "max": int(counts.max())}},
        "roofline": {"bound": "mfma", "kernel": f"gemm_bf16<{dom}>", "achieved": achieved,
                     "peak": BF16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / BF16_MFMA_PEAK_TFLOPS,
                     "traffic": profiled_traffic().get(dom) if w.name == "C5" and not args.routing and not args.dtype else None,
                     "traffic_source": "profiles/c5_gemm_pmc_counters.md (rocprofv3 FETCH_SIZE + WRITE_SIZE per launch; not this run)",
                     "flop_per_launch": gemm_flop, "avg_ms": kernels[dom]["ms"],
                     "sustained_mfma_peak": sustained, "frac_of_sustained": achieved / sustained,
                     "mfma_probe_tflops": probes},
        # sums of kernel durations per step (HIP events); "fwd_incl_index" = index + fwd
        "phases_ms": {"index": round(idx_ms, 4), "fwd": round(fwd_ms, 4),
                      "fwd_incl_index": round(idx_ms + fwd_ms, 4),
                      "bwd": round(all_ms - idx_ms - fwd_ms, 4)},
        "kernels_ms": {k: round(v["ms"], 4) for k, v in kernels.items()},
        "contraction_tflops": {k: round(v, 1) for k, v in rates.items()},
        # bandwidth-bound steps: algorithmic bytes (each tensor once) over the kernel's duration
        "hbm_steps": hbm_steps(w, kernels, copy_gbps),
        "router": {"bound": "hbm", "ms": round(route_ms, 4), "achieved": route_bytes / (route_ms * 1e-3) / 1e9,
                   "peak": 8000.0, "unit": "GB/s", "frac": route_bytes / (route_ms * 1e-3) / 1e9 / 8000.0,
                   "bytes": route_bytes},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, data)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
