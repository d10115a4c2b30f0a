"""Attention throughput of one long sequence against the number of slices it is cut into (the paper's motivation for
workload-aware splitting, section 2.3 / Fig. 1(a): finer slices cost kernel efficiency).

    python -m paper_2509_21275_amd.split_scan [--tokens 32768] [--heads 32 8] [--markdown out.md]

For N_split in {1, 2, 4, 8, 16, 32} the sequence runs as N_split split chunks of equal length: forward slice 0 .. N - 1,
backward N - 1 .. 0 with dK/dV accumulated over the calls, all on one stream, inputs resident; the time of the whole
sequence (median of 5) gives TFLOP/s on the causal flops of the unsplit sequence, which do not depend on N_split.
"""
from __future__ import annotations

import argparse

import numpy as np
import torch

import paper_2509_21275_amd as ca


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--tokens", type=int, default=32768)
    ap.add_argument("--heads", type=int, nargs=2, default=[32, 8], metavar=("HQ", "HKV"))
    ap.add_argument("--head-dim", type=int, default=128)
    ap.add_argument("--markdown", default=None)
    args = ap.parse_args()
    n, (Hq, Hkv), d = args.tokens, args.heads, args.head_dim
    dev = "cuda"
    q = torch.randn((n, Hq, d), device=dev, dtype=torch.bfloat16); do = torch.randn_like(q)
    k = torch.randn((n, Hkv, d), device=dev, dtype=torch.bfloat16); v = torch.randn_like(k)
    o = torch.empty_like(q); dq = torch.empty_like(q)
    lse = torch.empty((Hq, n), dtype=torch.float32, device=dev)
    dk = torch.empty_like(k); dv = torch.empty_like(v)
    pairs = n * (n + 1) // 2
    flops = 14.0 * d * pairs * Hq
    lines = ["| N_split | slice tokens | forward ms | backward ms | TFLOP/s (fwd + bwd) | relative to unsplit |", "|---|---|---|---|---|---|"]
    base = None
    for ns in (1, 2, 4, 8, 16, 32):
        sl = n // ns
        descs = [ca.make_desc([(0, sl, 0, sl * (i + 1))], Hq, Hkv, d, sl, n, d ** -0.5) for i in range(ns)]
        ws = [ca.alloc_workspace(x) for x in descs]
        lse_s = [lse[:, i * sl:(i + 1) * sl].contiguous() for i in range(ns)]

        def fwd():
            for i in range(ns):
                ca.chunk_attn_fwd(descs[i], q[i * sl:(i + 1) * sl], k, v, o[i * sl:(i + 1) * sl], lse_s[i], ws[i])

        def bwd():
            dk.zero_(); dv.zero_()
            for i in range(ns - 1, -1, -1):
                ca.chunk_attn_bwd(descs[i], q[i * sl:(i + 1) * sl], k, v, o[i * sl:(i + 1) * sl], do[i * sl:(i + 1) * sl],
                                  lse_s[i], dq[i * sl:(i + 1) * sl], dk, dv, 1, ws[i])
        for _ in range(2):
            fwd(); bwd()
        torch.cuda.synchronize()
        tf, tb = [], []
        for _ in range(5):
            e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
            e[0].record(); fwd(); e[1].record(); bwd(); e[2].record()
            torch.cuda.synchronize()
            tf.append(e[0].elapsed_time(e[1])); tb.append(e[1].elapsed_time(e[2]))
        f, b = float(np.median(tf)), float(np.median(tb))
        rate = flops / (f + b) / 1e9
        base = base or rate
        lines.append(f"| {ns} | {sl} | {f:.3f} | {b:.3f} | {rate:.1f} | {rate / base:.3f} |")
        print(lines[-1], flush=True)
    text = (f"one sequence of {n} tokens, {Hq}/{Hkv} heads, head_dim {d}; {flops / 1e12:.2f} TFLOP per forward + backward\n\n"
            + "\n".join(lines) + "\n")
    print(text)
    if args.markdown:
        with open(args.markdown, "w") as fh:
            fh.write(text)


if __name__ == "__main__":
    main()
