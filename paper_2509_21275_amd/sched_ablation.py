"""Plans one long-tailed batch with the sequence processor (paper section 3.3) and the chunk scheduler (section 3.4)
and runs the plan, and the three ablated variants of the paper's section 5.4, through the 1F1B timeline:

    full method   workload-balanced chunks (K tuned in [1, d_p + 4]), sequence grouping, adaptive checkpointing
    w/o wbc       long sequences cut evenly, short ones packed to a fixed token count; same scheduler
    w/o ckpt      no checkpointing: K is raised until every chunk window fits without it
    full ckpt     the full method's chunks, every layer checkpointed

    python -m paper_2509_21275_amd.sched_ablation [--capacity-gb 80] [--markdown out.md]

Host only (no GPU is used).  Times come from the paper's cost model (Eq. 1) with the attention coefficients fitted to
this library's kernels on one MI355X (alpha1, beta1) and a linear term for the rest of a layer that is an assumption
(72 D^2 flop per token at 1.2 PFLOP/s); memory from the model of sections 3.2.2 / 3.2.3 for a 7B-class model
(D = 4096, 32 layers, 128K-token vocabulary) on d_p x d_s = 4 x 8 devices.  The output shows the shape of the paper's
ablation (who pays recomputation, who pays bubbles), not measured training time.
"""
from __future__ import annotations

import argparse
import math
import random
from typing import List, Sequence, Tuple

from paper_2509_21275_amd import chunk_plan as cp
from paper_2509_21275_amd import chunk_sched as cs

D_P, D_S, LAYERS, HIDDEN, KV_HIDDEN, VOCAB = 4, 8, 32, 4096.0, 4096.0, 128256
# fitted to the chunk-attention kernels (forward + backward, 32 query heads, head_dim 128), ms
ALPHA1, BETA1 = 2.9895e-08, 0.1869
ALPHA2 = 72.0 * HIDDEN * HIDDEN / 1.2e15 * 1e3  # assumed: linear layers of one transformer layer, ms per token
ALIGN = 128


def cost_model() -> cp.CostModel:
    # per layer; attention heads and tokens of the linear layers are spread over the d_s devices of a stage
    return cp.CostModel(ALPHA1, ALPHA2, BETA1, 0.0, 0.0, D_S, 1)


def mem_model(capacity: float) -> cs.MemModel:
    params = 7e9
    return cs.MemModel(d_p=D_P, d_s=D_S, layers=LAYERS, m_token=34.0 * HIDDEN * LAYERS, m_logits=4.0 * VOCAB, e=2.0,
                       hidden=HIDDEN, kv_hidden=KV_HIDDEN, capacity=capacity, m_ms=[16.0 * params / (D_P * D_S)] * D_P)


def batch(seed: int, n: int, longest: int) -> List[int]:
    rng = random.Random(seed)
    out = [longest]
    while len(out) < n:
        out.append(int(min(longest, max(128, round(math.exp(math.log(2048) + 1.3 * rng.gauss(0.0, 1.0)))))))
    return out


Unit = List[Tuple[int, int, float]]  # chunks of one sequence: (tokens, is_split, time of one layer, fwd + bwd)


def units_of(chunks: Sequence[cp.Chunk]) -> List[Unit]:
    """Sequences as the scheduler sees them: the split chunks of a long sequence followed by the chunk that holds its
    tail slice; every chunk without a tail slice is a sequence of its own."""
    by_seq, units = {}, []
    for c in chunks:
        if c.is_split:
            by_seq.setdefault(c.slices[0][0], []).append(c)
    for c in chunks:
        if c.is_split:
            continue
        head = sorted(by_seq.pop(c.slices[0][0], []), key=lambda x: x.context) if c.context > 0 else []
        units.append([(x.tokens, 1, x.time) for x in head] + [(c.tokens, 0, c.time)])
    assert not by_seq
    return units


def even_chunks(model: cp.CostModel, lengths: Sequence[int], slice_len: int) -> List[Unit]:
    """'w/o wbc': equal slices of slice_len tokens for long sequences, short ones packed first-fit to slice_len."""
    units, shorts = [], []
    for n in lengths:
        if n <= slice_len:
            shorts.append(n)
            continue
        u, pos = [], 0
        while pos < n:
            s = min(slice_len, n - pos)
            u.append((s, int(pos + s < n), cp.chunk_plan_time(model, pos, [s])))
            pos += s
        units.append(u)
    bins: List[List[int]] = []
    for s in sorted(shorts, reverse=True):
        for b in bins:
            if sum(b) + s <= slice_len:
                b.append(s)
                break
        else:
            bins.append([s])
    units += [[(sum(b), 0, cp.chunk_plan_time(model, 0, b))] for b in bins]
    return units


def run_plan(mm: cs.MemModel, units: List[Unit], mode: str, gap: float):
    """mode: 'adaptive' (grouping + Algorithm 2), 'none' (a grouping that fits with C = 0), 'full' (every layer).
    Returns None if the plan does not fit, else a dict of totals over the pipelines."""
    flat = [c for u in units for c in u]
    per_stage = LAYERS // D_P
    mean_t = sum(c[2] for c in flat) / len(flat) * per_stage
    f_hat = sum(c[2] for c in flat) / len(flat) / 3.0  # forward pass of one layer, average chunk
    delta = (D_P - 1) * mean_t
    plain = [[(t, s) for t, s, _ in u] for u in units]
    # 'none': recomputation priced so high that the grouping avoids it whenever some grouping fits without any
    res = cs.chunk_sched_group(mm, plain, 1e12 if mode == "none" else f_hat, delta, gap)
    if res is None:
        return None
    pipes = res[1]
    if mode == "none" and any(any(p.C) for p in pipes):
        return None
    tot = dict(time=0.0, busy=0.0, recomp=0.0, chunks=len(flat), pipelines=len(pipes), ckpt=0, peak=0.0)
    for p in pipes:
        ch = [flat[k] for k in p.order]
        uo = [j for j, u in enumerate(p.units) for _ in units[u]]
        fb = cs.chunk_sched_f2b(uo)
        n, ns = len(ch), max(len(units[u]) for u in p.units)
        C = p.C if mode != "full" else [per_stage] * len(p.C)
        ck = [[C[fb[k] + D_P - st] for k in range(n)] for st in range(1, D_P + 1)]
        t_f = [c[2] / 3.0 * per_stage for c in ch]
        t_b = [2.0 * c[2] / 3.0 * per_stage for c in ch]
        rec = [[ck[st][k] * ch[k][2] / 3.0 for k in range(n)] for st in range(D_P)]
        mem = [[cs.chunk_sched_act_bytes(mm, st + 1, ch[k][0], ch[k][1], ck[st][k]) for k in range(n)] for st in range(D_P)]
        ms, busy, peak, _ = cs.chunk_sched_simulate(D_P, ns, fb, t_f, t_b, rec, mem)
        tot["time"] += ms
        tot["busy"] += sum(busy) / D_P
        tot["recomp"] += sum(sum(r) for r in rec) / D_P
        tot["ckpt"] += sum(C)
        tot["peak"] = max(tot["peak"], max(pk + mm.m_ms[st] for st, pk in enumerate(peak)))
    return tot


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--capacity-gb", type=float, default=80.0)
    ap.add_argument("--sequences", type=int, default=128)
    ap.add_argument("--longest", type=int, default=65536)
    ap.add_argument("--seed", type=int, default=7)
    ap.add_argument("--gap", type=float, default=0.02)
    ap.add_argument("--markdown", default=None)
    args = ap.parse_args()
    model, mm = cost_model(), mem_model(args.capacity_gb * 1e9)
    lengths = batch(args.seed, args.sequences, args.longest)
    token_cap = 1 << 20

    rows = []
    best = None
    for K in range(1, D_P + 5):
        chunks, _, _ = cp.chunk_plan_build(model, token_cap, lengths, K, ALIGN)
        r = run_plan(mm, units_of(chunks), "adaptive", args.gap)
        if r is not None and (best is None or r["time"] < best[1]["time"]):
            best = (K, r, chunks)
    if best is None:
        raise SystemExit("the batch does not fit at any K in [1, d_p + 4]")
    K, full, chunks = best
    rows.append(("full method", K, full))
    mesh, _, _ = cp.chunk_plan_mesh(model, max(lengths), K, ALIGN, token_cap)
    even = run_plan(mm, even_chunks(model, lengths, -(-max(lengths) // K // ALIGN) * ALIGN), "adaptive", args.gap)
    rows.append(("w/o wbc", K, even))
    nock = None
    for K2 in range(1, 129):
        ch2, _, _ = cp.chunk_plan_build(model, token_cap, lengths, K2, ALIGN)
        nock = run_plan(mm, units_of(ch2), "none", args.gap)
        if nock is not None:
            rows.append(("w/o ckpt", K2, nock))
            break
    if nock is None:
        rows.append(("w/o ckpt", None, None))
    rows.append(("full ckpt", K, run_plan(mm, units_of(chunks), "full", args.gap)))

    lines = ["| variant | K | chunks | 1F1B pipelines | sum of C | end-to-end time (full method = 1) | recomputation share | bubble share | peak memory GB |",
             "|---|---|---|---|---|---|---|---|---|"]
    for name, k, r in rows:
        if r is None:
            lines.append(f"| {name} | - | does not fit | | | | | | |")
            continue
        lines.append(f"| {name} | {k} | {r['chunks']} | {r['pipelines']} | {r['ckpt']} | {r['time'] / full['time']:.3f} | "
                     f"{r['recomp'] / r['time']:.3f} | {1.0 - r['busy'] / r['time']:.3f} | {r['peak'] / 1e9:.1f} |")
    head = (f"batch: {len(lengths)} sequences, {sum(lengths)} tokens, longest {max(lengths)}; d_p x d_s = {D_P} x {D_S}, "
            f"{LAYERS} layers, capacity {args.capacity_gb:g} GB, mesh of the full method {mesh}")
    text = head + "\n\n" + "\n".join(lines) + "\n"
    print(text)
    if args.markdown:
        with open(args.markdown, "w") as f:
            f.write(text)


if __name__ == "__main__":
    main()
