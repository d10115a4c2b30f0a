"""Throughput of the fused in-place cross-entropy on one GPU against the HBM roofline.

    python -m paper_2509_21275_amd.bench_fused_ce [--rows 16384] [--vocab 131072] [--iters 20]

One call reads every logit once and writes its gradient once: 4 bytes per logit of algorithmic traffic.  Prints one
JSON line (GB/s = rows * vocab * 4 / kernel time, measured with events on the launch stream; the logits are refilled
outside the timed region so that every iteration sees realistic values)."""
from __future__ import annotations

import argparse
import json

import torch

from paper_2509_21275_amd.fused_ce import fused_ce_inplace

PEAK_HBM_GBS = 8000.0  # MI355X


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--rows", type=int, default=16384)
    ap.add_argument("--vocab", type=int, default=131072)
    ap.add_argument("--iters", type=int, default=20)
    a = ap.parse_args()
    g = torch.Generator(device="cuda").manual_seed(250921275)
    src = (torch.randn((a.rows, a.vocab), generator=g, device="cuda") * 2.0).to(torch.bfloat16)
    targets = torch.randint(0, a.vocab, (a.rows,), generator=g, device="cuda", dtype=torch.int32)
    logits = torch.empty_like(src)
    loss = torch.empty((a.rows,), device="cuda")
    times = []
    for it in range(a.iters + 3):
        logits.copy_(src)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fused_ce_inplace(logits, targets, loss, 1.0 / a.rows)
        e1.record()
        torch.cuda.synchronize()
        if it >= 3:
            times.append(e0.elapsed_time(e1))
    # reference: a plain device copy of the same tensor moves the same bytes (read once, write once)
    ctimes = []
    for it in range(8):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        logits.copy_(src)
        e1.record()
        torch.cuda.synchronize()
        if it >= 3:
            ctimes.append(e0.elapsed_time(e1))
    copy_gbs = a.rows * a.vocab * 4 / (sorted(ctimes)[len(ctimes) // 2] * 1e-3) / 1e9
    ms = sorted(times)[len(times) // 2]
    gbs = a.rows * a.vocab * 4 / (ms * 1e-3) / 1e9
    print(json.dumps({"op": "fused_ce_inplace", "rows": a.rows, "vocab": a.vocab, "dtype": "bf16 logits, fp32 reductions",
                      "ms": round(ms, 4), "algorithmic_bytes": a.rows * a.vocab * 4,
                      "roofline": {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                   "frac": round(gbs / PEAK_HBM_GBS, 4)},
                      "device_copy_same_bytes_gbs": round(copy_gbs, 1), "mean_loss": float(loss.mean())}))


if __name__ == "__main__":
    main()
