#!/usr/bin/env python3
"""Benchmark of the chunk-attention hot path on one MI355X.

One "step" is one pass of the whole hot path (schedule, forward, backward pre-pass, backward main
kernel, dQ conversion) over one batch of synthetic chunks:

  * the 64K-token skewed packed chunk (block-diagonal causal, 32 query / 8 KV heads, d = 128), and
  * the 128K-token sequence split into 8 slices of 16K (64 query / 8 KV heads, d = 128): forward of
    slices 0..7 in order, each attending to the keys/values of the slices before it, then backward
    of slices 7..0, accumulating dK/dV of the shared context rows.

Inputs are seeded N(0,1) bf16 tensors already resident in HBM.  The metric is causal TFLOP/s:
14 * head_dim * (unmasked query-key pairs) * query heads per forward+backward, divided by the step time.
Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6  # MI355X dense bf16 MFMA: 256 CU x 4096 flop/clk/CU x 2.4 GHz


def cpu_baseline():
    """The CPU oracle, as it stands, timed on a bounded sample of the packed workload."""
    import numpy as np
    import torch

    import oracle
    import synth
    oracle.build()
    case = synth.case_by_index(4)
    d, Hq, Hkv = case.head_dim, case.num_q_heads, case.num_kv_heads
    # sample: the shortest whole sequences of the packed chunk, all heads, up to a pair budget
    segs = sorted(case.segs, key=lambda s: s.q_len)
    chosen, pairs = [], 0
    for s in segs:
        p = s.q_len * (s.q_len + 1) // 2
        if chosen and (pairs + p) * Hq > 100_000_000:
            break
        chosen.append(s)
        pairs += p
    packed = synth.packed_chunk([s.q_len for s in chosen])
    tq = sum(s.q_len for s in chosen)
    q = synth.normal_bf16(case.seed, 0, (tq, Hq, d)); k = synth.normal_bf16(case.seed, 1, (tq, Hkv, d))
    v = synth.normal_bf16(case.seed, 2, (tq, Hkv, d)); do = synth.normal_bf16(case.seed, 3, (tq, Hq, d))
    orc = oracle.Oracle(packed, q, k, v, do, case.scale)
    t0 = time.perf_counter()
    orc.forward()
    orc.backward()
    dt = time.perf_counter() - t0
    flops = 14.0 * d * pairs * Hq
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count()
    omp = os.environ.get("OMP_NUM_THREADS")
    if omp:
        cores = min(cores, int(omp))
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "seconds": dt,
            "sample": f"full fp64 forward+backward of the {len(chosen)} shortest sequences of the packed chunk "
                      f"(lengths {[s.q_len for s in chosen]}, {Hq}/{Hkv} heads, d={d}, {pairs} pairs per head)"}


def recorded_traffic():
    """HBM-side bytes per launch of the dominant kernel, as measured by the two rocprofv3 counter runs that are
    summarised under profiles/ (this script cannot run the profiler on itself).  None if no summary is there."""
    path = os.path.join(ROOT, "profiles", "bwd_dkv_pipe_kernel_bench_workload_hbm_traffic.md")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":", 1)[1])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only", choices=["all", "packed", "split"], default="all",
                    help="restrict the step to one of the two chunk sets (for profiling)")
    ap.add_argument("--fast-inputs", action="store_true",
                    help="draw the N(0,1) inputs with torch.randn (one kernel per tensor) instead of the counter-based "
                         "generator (thousands of small kernels, slow under rocprofv3 counter collection)")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="before the steps, run one plain device copy of this many MiB (a kernel of known HBM "
                         "traffic against which rocprofv3's FETCH_SIZE / WRITE_SIZE counters are scaled)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (--gpus must be 1); the path shards by KV head or by "
              "segment without communication", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2509_21275_amd as ca
    import synth

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.fast_inputs:
        torch.manual_seed(synth.BASE_SEED)

        def normal_bf16(seed, tensor_id, shape, device):
            return torch.randn(shape, dtype=torch.float32, device=device).to(torch.bfloat16)
    else:
        normal_bf16 = synth.normal_bf16
    evpool = ca.HipEvents()

    # ---------------- workloads ----------------
    calls = []  # dicts: name, desc, tensors, flops

    def add_call(name, case, q, k, v, do, dk, dv, accumulate):
        desc = ca.make_desc(case.segs, case.num_q_heads, case.num_kv_heads, case.head_dim, case.total_q,
                            case.total_kv, case.scale)
        pairs = ca.chunk_attn_pair_count(desc)
        assert pairs == case.pairs
        calls.append(dict(name=name, desc=desc, q=q, k=k, v=v, do=do, o=torch.empty_like(q),
                          lse=torch.empty((case.num_q_heads, case.total_q), dtype=torch.float32, device=dev),
                          dq=torch.empty_like(q), dk=dk, dv=dv, accumulate=accumulate,
                          ws=ca.alloc_workspace(desc, dev), pairs=pairs,
                          fwd_flops=4.0 * case.head_dim * pairs * case.num_q_heads,
                          bwd_flops=10.0 * case.head_dim * pairs * case.num_q_heads,
                          fwd_ms=[], bwd_ms=[], bwd_call_ms=[]))

    if args.only in ("all", "packed"):
        c4 = synth.case_by_index(4)
        q = normal_bf16(c4.seed, 0, (c4.total_q, c4.num_q_heads, c4.head_dim), dev)
        k = normal_bf16(c4.seed, 1, (c4.total_kv, c4.num_kv_heads, c4.head_dim), dev)
        v = normal_bf16(c4.seed, 2, (c4.total_kv, c4.num_kv_heads, c4.head_dim), dev)
        do = normal_bf16(c4.seed, 3, (c4.total_q, c4.num_q_heads, c4.head_dim), dev)
        add_call("packed_64k", c4, q, k, v, do, torch.empty_like(k), torch.empty_like(v), 0)
    n_split = 0
    if args.only in ("all", "split"):
        c5 = synth.case_by_index(5, 0)
        k5 = normal_bf16(c5.seed, 1, (c5.total_kv, c5.num_kv_heads, c5.head_dim), dev)
        v5 = normal_bf16(c5.seed, 2, (c5.total_kv, c5.num_kv_heads, c5.head_dim), dev)
        dk5 = torch.empty_like(k5); dv5 = torch.empty_like(v5)
        for i in range(8):
            ci = synth.case_by_index(5, i)
            # tensor ids 10+i / 20+i: each slice has its own query and dO rows of the long sequence
            q = normal_bf16(ci.seed, 10 + i, (ci.total_q, ci.num_q_heads, ci.head_dim), dev)
            do = normal_bf16(ci.seed, 20 + i, (ci.total_q, ci.num_q_heads, ci.head_dim), dev)
            # the last slice's key range covers the whole sequence: it overwrites, the others accumulate
            add_call(f"split_128k_slice{i}", ci, q, k5, v5, do, dk5, dv5, 0 if i == 7 else 1)
        n_split = 8

    if args.copy_probe_mib > 0:
        src = torch.empty(args.copy_probe_mib << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)      # the probed kernel: reads and writes copy_probe_mib MiB
        torch.cuda.synchronize()
        del src, dst

    fwd_order = list(range(len(calls)))
    split_ids = [i for i, c in enumerate(calls) if c["name"].startswith("split")]
    bwd_order = [i for i in range(len(calls)) if i not in split_ids] + split_ids[::-1]

    def step(record):
        for i in fwd_order:
            c = calls[i]
            if record:
                ev = evpool.pair(); c["fwd_ms"].append(ev)
                ca.chunk_attn_profile_events(*ev)
            ca.chunk_attn_fwd(c["desc"], c["q"], c["k"], c["v"], c["o"], c["lse"], c["ws"])
        for i in bwd_order:
            c = calls[i]
            if record:
                ev = evpool.pair(); c["bwd_ms"].append(ev)
                ca.chunk_attn_profile_events(*ev)
            ca.chunk_attn_bwd(c["desc"], c["q"], c["k"], c["v"], c["o"], c["do"], c["lse"], c["dq"], c["dk"],
                              c["dv"], c["accumulate"], c["ws"])

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps

    # host side of one more step: the calls build their schedules, upload them and launch, and return while the GPU is
    # still working (the paper overlaps planning with GPU work, section 3 overview)
    t0 = time.perf_counter()
    step(False)
    host_ms = (time.perf_counter() - t0) * 1e3
    torch.cuda.synchronize()

    total_flops = sum(c["fwd_flops"] + c["bwd_flops"] for c in calls)
    value = total_flops / (ms_per_step * 1e-3) / 1e12

    # what the chip's clock allows under matrix load: a kernel of nothing but bf16 MFMAs, half a second of it, measured right
    # after the timed steps (include/chunk_attn.h: chunk_attn_measure_mfma_rate)
    measured_peak = ca.chunk_attn_measure_mfma_rate(500)

    # per chunk: whole forward and whole backward calls (all their kernels), one more step with events around every call
    call_ev = []
    for i in fwd_order:
        c = calls[i]
        e0 = evpool.pair()
        evpool.record(e0[0]); ca.chunk_attn_fwd(c["desc"], c["q"], c["k"], c["v"], c["o"], c["lse"], c["ws"]); evpool.record(e0[1])
        call_ev.append((i, "fwd", e0))
    for i in bwd_order:
        c = calls[i]
        e0 = evpool.pair()
        evpool.record(e0[0])
        ca.chunk_attn_bwd(c["desc"], c["q"], c["k"], c["v"], c["o"], c["do"], c["lse"], c["dq"], c["dk"], c["dv"], c["accumulate"], c["ws"])
        evpool.record(e0[1])
        call_ev.append((i, "bwd", e0))
    torch.cuda.synchronize()
    call_ms = {(i, kind): evpool.elapsed_ms(*ev) for i, kind, ev in call_ev}

    # the clock the three main kernels run at: one more step with the library's clock log switched on, every call read
    # back by itself (include/chunk_attn.h: chunk_attn_measure_set_clock_log); shader clocks / 100 MHz ticks, summed over
    # the workgroups of all calls
    clock_buf = torch.zeros(ca.CLOCK_LOG_BYTES // 8, dtype=torch.int64, device=dev)
    clock_sum = {k: [0, 0] for k in ca.CLOCK_LOG_KERNELS}
    ca.chunk_attn_measure_set_clock_log(clock_buf)
    try:
        for order, kind in ((fwd_order, "fwd"), (bwd_order, "bwd")):
            for i in order:
                c = calls[i]
                clock_buf.zero_()
                if kind == "fwd":
                    ca.chunk_attn_fwd(c["desc"], c["q"], c["k"], c["v"], c["o"], c["lse"], c["ws"])
                else:
                    ca.chunk_attn_bwd(c["desc"], c["q"], c["k"], c["v"], c["o"], c["do"], c["lse"], c["dq"], c["dk"], c["dv"],
                                      c["accumulate"], c["ws"])
                torch.cuda.synchronize()
                for k, v in ca.clock_log_sums(clock_buf).items():
                    clock_sum[k][0] += v["shader_clocks"]; clock_sum[k][1] += v["ticks_100mhz"]
    finally:
        ca.chunk_attn_measure_set_clock_log(None)
    kernel_clock_mhz = {k: round(100.0 * v[0] / v[1], 1) if v[1] else None for k, v in clock_sum.items()}

    # per-kernel durations from the HIP events recorded on the launch stream
    per_call = []
    fwd_k_ms = bwd_k_ms = 0.0
    for c in calls:
        f = sum(evpool.elapsed_ms(*e) for e in c["fwd_ms"]) / args.steps
        b = sum(evpool.elapsed_ms(*e) for e in c["bwd_ms"]) / args.steps
        fwd_k_ms += f; bwd_k_ms += b
        ci = calls.index(c)
        fw, bw = call_ms[(ci, "fwd")], call_ms[(ci, "bwd")]
        per_call.append({"call": c["name"], "pairs_per_head": c["pairs"], "fwd_kernel_ms": round(f, 4),
                         "bwd_dkv_kernel_ms": round(b, 4),
                         "fwd_tflops": round(c["fwd_flops"] / f / 1e9, 1),
                         "bwd_dkv_kernel_tflops": round(0.8 * c["bwd_flops"] / b / 1e9, 1),
                         "fwd_call_ms": round(fw, 4), "bwd_call_ms": round(bw, 4),
                         "fwd_bwd_tflops": round((c["fwd_flops"] + c["bwd_flops"]) / (fw + bw) / 1e9, 1)})
    evpool.close()
    bwd_flops = sum(c["bwd_flops"] for c in calls)
    fwd_flops = sum(c["fwd_flops"] for c in calls)
    n_launch = len(calls)
    # The dominant kernel is the dK/dV kernel of the backward.  It computes four contractions per unmasked
    # (query, key) pair and query head -- S, dP, dV, dK -- i.e. 8 * head_dim flops, 0.8 of the backward's 10 * head_dim.
    dkv_flops = 0.8 * bwd_flops
    achieved = dkv_flops / (bwd_k_ms * 1e-3) / 1e12

    # the two workloads the target names, each by itself (whole calls, all kernels)
    def shape_row(names):
        sel = [c for c in calls if c["name"] in names or any(c["name"].startswith(n) for n in names)]
        if not sel:
            return None
        fl = sum(c["fwd_flops"] + c["bwd_flops"] for c in sel)
        ms = sum(call_ms[(calls.index(c), "fwd")] + call_ms[(calls.index(c), "bwd")] for c in sel)
        tf = fl / ms / 1e9
        return {"tflops": round(tf, 1), "ms": round(ms, 3), "pct_of_bf16_mfma_peak": round(100.0 * tf / PEAK_BF16_TFLOPS, 2),
                "pct_of_measured_clock_peak": round(100.0 * tf / measured_peak, 2)}
    per_shape = {"packed_64k": shape_row(["packed_64k"]), "split_128k_x8": shape_row(["split_128k_slice"])}

    out = {
        "metric": "chunk attention fwd+bwd causal TFLOP/s, 1 MI355X",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3), "host_plan_and_enqueue_ms_per_step": round(host_ms, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic (torch.randn)" if args.fast_inputs else "synthetic",
        "config": {"workload": {"all": "packed_64k_skewed(32/8 heads,d128) + split_128k_x8(64/8 heads,d128), fwd+bwd",
                                "packed": "packed_64k_skewed(32/8 heads,d128), fwd+bwd",
                                "split": "split_128k_x8(64/8 heads,d128), fwd+bwd"}[args.only],
                   "calls_per_step": 2 * n_launch, "flops_per_step": total_flops,
                   "seed_base": synth.BASE_SEED},
        "pct_of_bf16_mfma_peak": round(100.0 * value / PEAK_BF16_TFLOPS, 2),
        "target": {"pct_of_bf16_mfma_peak": 50.0, "met": bool(value >= 0.5 * PEAK_BF16_TFLOPS)},
        "pct_of_measured_clock_peak": round(100.0 * value / measured_peak, 2),
        "per_shape": per_shape,
        "roofline": {"kernel": "bwd_dkv_pipe_kernel<128>", "bound": "mfma", "achieved": round(achieved, 2),
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                     "measured_clock_peak": round(measured_peak, 1),
                     "frac_of_measured_clock_peak": round(achieved / measured_peak, 4),
                     "kernel_clock_mhz": kernel_clock_mhz,
                     "frac_of_peak_at_kernel_clock": (round(achieved / (PEAK_BF16_TFLOPS * kernel_clock_mhz["dkv"] / 2400.0), 4)
                                                      if kernel_clock_mhz["dkv"] else None),
                     "traffic": recorded_traffic(), "launches_per_step": n_launch,
                     "avg_launch_ms": round(bwd_k_ms / n_launch, 4),
                     "flops_per_launch_avg": dkv_flops / n_launch,
                     "fwd_kernel": {"kernel": "fwd_pipe_kernel<128>", "achieved": round(fwd_flops / (fwd_k_ms * 1e-3) / 1e12, 2),
                                    "frac": round(fwd_flops / (fwd_k_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                                    "avg_launch_ms": round(fwd_k_ms / n_launch, 4)}},
        "per_call": per_call,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
