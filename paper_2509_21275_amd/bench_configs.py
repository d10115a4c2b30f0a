"""Forward and backward throughput of the five workload shapes, one after the other, on one GPU.

    python -m paper_2509_21275_amd.bench_configs [--markdown out.md] [--variants]

Inputs resident in HBM, median of 5 timed calls after 2 warm-up calls, causal flops (4 d per unmasked pair and query head
forward, 10 d backward).  The split sequence (shape 5) is reported for its first, middle and last slice.
--variants adds the packed 64K chunk and the middle slice of the split sequence at head dimensions 64, 96 and 256 (same
head counts) and with the one-pass backward of head dimension 128.
"""
from __future__ import annotations

import argparse
import dataclasses

import numpy as np
import torch

import paper_2509_21275_amd as ca
import synth

PEAK = 2516.6


def measure(case):
    dev = "cuda"
    qs = (case.total_q, case.num_q_heads, case.head_dim); ks = (case.total_kv, case.num_kv_heads, case.head_dim)
    q = torch.randn(qs, device=dev, dtype=torch.bfloat16); do = torch.randn_like(q)
    k = torch.randn(ks, device=dev, dtype=torch.bfloat16); v = torch.randn_like(k)
    desc = ca.make_desc(case.segs, case.num_q_heads, case.num_kv_heads, case.head_dim, case.total_q, case.total_kv, case.scale)
    ws = ca.alloc_workspace(desc)
    o = torch.empty_like(q); lse = torch.empty((case.num_q_heads, case.total_q), dtype=torch.float32, device=dev)
    dq = torch.empty_like(q); dk = torch.empty_like(k); dv = torch.empty_like(v)
    out = []
    for fn in (lambda: ca.chunk_attn_fwd(desc, q, k, v, o, lse, ws),
               lambda: ca.chunk_attn_bwd(desc, q, k, v, o, do, lse, dq, dk, dv, 0, ws)):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(5):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(); fn(); e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1))
        out.append(float(np.median(ts)))
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--markdown", default=None)
    ap.add_argument("--variants", action="store_true")
    args = ap.parse_args()
    cases = [synth.case_by_index(i) for i in (1, 2, 3, 4)] + [synth.case_by_index(5, s) for s in (0, 3, 7)]
    # bring the chip to its sustained clock before anything is timed
    measure(cases[1])
    lines = ["| shape | heads (q/kv), d | queries x keys | pairs per head | forward ms | backward ms | forward TFLOP/s | backward TFLOP/s | "
             "total TFLOP/s | % of 2516.6 |", "|---|---|---|---|---|---|---|---|---|---|"]
    def row(c, label=None):
        f, b = measure(c)
        fl = c.head_dim * c.pairs * c.num_q_heads / 1e9
        tot = 14 * fl / (f + b)
        lines.append(f"| {label or c.name} | {c.num_q_heads}/{c.num_kv_heads}, {c.head_dim} | {c.total_q} x {c.total_kv} | {c.pairs} | {f:.3f} | {b:.3f} | "
                     f"{4 * fl / f:.1f} | {10 * fl / b:.1f} | {tot:.1f} | {100 * tot / PEAK:.1f} |")
        print(lines[-1], flush=True)

    for c in cases:
        row(c)
    if args.variants:
        for base in (cases[3], cases[5]):
            for d in (64, 96, 256):
                row(dataclasses.replace(base, head_dim=d), f"{base.name}, head_dim {d}")
            ca.chunk_attn_test_set_bwd_mode(2)
            try:
                row(base, f"{base.name}, one-pass backward")
            finally:
                ca.chunk_attn_test_set_bwd_mode(0)
    # what this machine sustains on matrix instructions alone (boxes differ by several per cent): the yardstick for the rows above
    rate = ca.chunk_attn_measure_mfma_rate(500)
    lines += ["", f"MFMA-only rate of the box these rows were measured on (chunk_attn_measure_mfma_rate, right after them): {rate:.0f} TFLOP/s."]
    print(lines[-1], flush=True)
    text = "\n".join(lines) + "\n"
    if args.markdown:
        with open(args.markdown, "w") as fh:
            fh.write(text)


if __name__ == "__main__":
    main()
