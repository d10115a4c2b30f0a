"""Plain Python reference of the paper's chunk scheduler (section 3.4): the memory model of a chunk with layer-wise
checkpointing (section 3.2.2 and 3.2.3), the 1F1B order of chunks and its chunk windows, the stage-aware chunk-level
checkpointing problem (section 3.4.3, Algorithm 2) solved by exhaustive enumeration, the sequence grouping (section
3.4.2) solved by trying every grouping, and a 1F1B timeline.  Test infrastructure only: it checks the C++ scheduler of
the library and is never used by the product path.

Stages are numbered p = 1 .. d_p as in the paper; chunks are numbered 0 .. n - 1 in forward order.

Readings of points the paper leaves open:
  - N, the number of devices an activation is spread over, is d_p * d_s: only then do the activation footprint with
    l_ckpt checkpointed layers (section 3.2.3) and the coefficients of Algorithm 2 describe the same quantity;
  - forward order inside a 1F1B pipeline: sequences with more chunks first (ties: more tokens first, then input
    order), the chunks of a sequence in order; backward order: sequence by sequence in the same order, the chunks of
    a sequence last to first (section 3.4.1 and the dependency of a slice on the slices before it);
  - stage p runs min(n, d_p - p + N_split) forward passes, then alternates one backward and one forward pass, then the
    remaining backward passes; a chunk window is the set of chunks whose forward pass has run and whose backward pass
    has not finished, taken each time a forward pass has just finished;
  - delta = (d_p - 1) * mean over the batch's chunks of their forward + backward time;
  - a group S[k+1 : i+1] that holds no sequence costs nothing (no pipeline is run for it).
"""
from __future__ import annotations

import itertools
from dataclasses import dataclass
from typing import List, Sequence, Tuple


@dataclass
class MemModel:
    d_p: int
    d_s: int
    layers: int          # L, a multiple of d_p
    m_token: float       # activation bytes per token, all layers
    m_logits: float      # logits bytes per token
    e: float             # bytes per activation element
    hidden: float        # D
    kv_hidden: float     # D_kv
    capacity: float      # G
    m_ms: Sequence[float]  # model-state bytes of stage p at index p - 1


def act_bytes(m: MemModel, p: int, tokens: int, is_split: int, l_ckpt: int) -> float:
    """Activation footprint of one chunk at stage p with l_ckpt of the stage's layers checkpointed (section 3.2.3):
    dK/dV buffers of a split chunk + what the checkpointed layers keep (their input, and keys/values for a split
    chunk) + the activations of the layers that are not checkpointed + the logits on the last stage."""
    n_dev = m.d_p * m.d_s
    m_dkv = is_split * 2.0 * m.e * m.layers * m.kv_hidden / n_dev * tokens
    m_ckpt = m.e * (m.hidden + 2.0 * is_split * m.kv_hidden) * l_ckpt / m.d_s * tokens
    rest = ((m.layers - l_ckpt * m.d_p) / m.layers * m.m_token / n_dev + (m.m_logits / m.d_s if p == m.d_p else 0.0)) * tokens
    return m_dkv + m_ckpt + rest


def pipeline_order(units: Sequence[Sequence[Tuple[int, int]]]) -> List[int]:
    """Order in which the units (sequences: lists of (tokens, is_split) chunks) of one pipeline run: more chunks first,
    then more tokens, then input order."""
    return sorted(range(len(units)), key=lambda u: (-len(units[u]), -sum(c[0] for c in units[u]), u))


def f2b(unit_of_chunk: Sequence[int]) -> List[int]:
    """Backward position of every chunk (chunks in forward order, the chunks of a unit adjacent): units keep their
    order, the chunks of a unit are reversed."""
    n = len(unit_of_chunk)
    out = [0] * n
    start = 0
    while start < n:
        end = start
        while end < n and unit_of_chunk[end] == unit_of_chunk[start]:
            end += 1
        for k in range(start, end):
            out[k] = start + (end - 1 - k)
        start = end
    return out


def stage_ops(d_p: int, p: int, n: int, n_split: int, f2b_: Sequence[int]) -> List[Tuple[str, int]]:
    """Passes of stage p in order: ('F', chunk) / ('B', chunk)."""
    b2f = [0] * n
    for k, j in enumerate(f2b_):
        b2f[j] = k
    w = min(n, d_p - p + n_split)
    ops = [("F", k) for k in range(w)]
    nf, nb = w, 0
    while nb < n:
        ops.append(("B", b2f[nb]))
        nb += 1
        if nf < n:
            ops.append(("F", nf))
            nf += 1
    return ops


def windows(d_p: int, p: int, n: int, n_split: int, f2b_: Sequence[int]) -> List[List[int]]:
    """Chunk windows of stage p: after every forward pass, the chunks that are between forward and end of backward."""
    live, out = [], []
    for kind, k in stage_ops(d_p, p, n, n_split, f2b_):
        if kind == "F":
            live.append(k)
            out.append(sorted(live))
        else:
            live.remove(k)
    return out


def ckpt_of(d_p: int, p: int, k: int, f2b_: Sequence[int], C: Sequence[int]) -> int:
    """ckpt(p, k) = C[f2b[k] + d_p - p]  (section 3.4.3)."""
    return C[f2b_[k] + d_p - p]


def config_fits(m: MemModel, chunks: Sequence[Tuple[int, int]], n_split: int, f2b_: Sequence[int], C: Sequence[int]) -> bool:
    n = len(chunks)
    for p in range(1, m.d_p + 1):
        for w in windows(m.d_p, p, n, n_split, f2b_):
            tot = m.m_ms[p - 1] + sum(act_bytes(m, p, chunks[k][0], chunks[k][1], ckpt_of(m.d_p, p, k, f2b_, C)) for k in w)
            if tot > m.capacity:
                return False
    return True


def solve_ckpt(m: MemModel, chunks: Sequence[Tuple[int, int]], unit_of_chunk: Sequence[int], n_split: int):
    """Smallest sum of C over all C in {0 .. L / d_p}^(n + d_p - 1) whose every chunk window fits the capacity
    (section 3.4.3): plain enumeration, for small cases.  Returns (sum, C) or None."""
    n = len(chunks)
    fb = f2b(unit_of_chunk)
    hi = m.layers // m.d_p
    best = None
    for C in itertools.product(range(hi + 1), repeat=n + m.d_p - 1):
        s = sum(C)
        if best is not None and s >= best[0]:
            continue
        if config_fits(m, chunks, n_split, fb, C):
            best = (s, list(C))
    return best


def group(m: MemModel, units: Sequence[Sequence[Tuple[int, int]]], layer_fwd_time: float, delta: float):
    """Sequence grouping (section 3.4.2): units sorted by their number of chunks are cut into groups of adjacent chunk
    counts, each group one 1F1B pipeline costing delta + layer_fwd_time * (smallest sum of C); every way of cutting
    is tried.  Returns (cost, [list of unit indices per group]) or None if no grouping fits."""
    counts = sorted({len(u) for u in units})
    best = None
    for cuts in itertools.product([0, 1], repeat=len(counts) - 1):
        groups, cur = [], [counts[0]]
        for c, cut in zip(counts[1:], cuts):
            if cut:
                groups.append(cur)
                cur = [c]
            else:
                cur.append(c)
        groups.append(cur)
        cost, members, ok = 0.0, [], True
        for g in groups:
            idx = [u for u in range(len(units)) if len(units[u]) in g]
            sub = [units[u] for u in idx]
            order = pipeline_order(sub)
            chunks = [c for o in order for c in sub[o]]
            unit_of = [j for j, o in enumerate(order) for _ in sub[o]]
            r = solve_ckpt(m, chunks, unit_of, max(len(u) for u in sub))
            if r is None:
                ok = False
                break
            cost += delta + layer_fwd_time * r[0]
            members.append([idx[o] for o in order])
        if ok and (best is None or cost < best[0] - 1e-12):
            best = (cost, members)
    return best


def simulate(d_p: int, n_split: int, f2b_: Sequence[int], t_fwd: Sequence[float], t_bwd: Sequence[float],
             t_recomp=None, mem=None, p2p: float = 0.0):
    """Timeline of one 1F1B pipeline: every stage runs its passes in order (stage_ops); the forward pass of chunk k at
    stage p starts once stage p - 1 has finished it (+ p2p), the backward pass once stage p + 1 has finished it
    (+ p2p); t_recomp[p - 1][k] is added to the backward pass of chunk k at stage p.  mem[p - 1][k] is held from the
    start of the forward pass to the end of the backward pass.  Returns (makespan, busy time per stage, peak bytes
    per stage, largest number of chunks held per stage)."""
    n = len(t_fwd)
    ops = {p: stage_ops(d_p, p, n, n_split, f2b_) for p in range(1, d_p + 1)}
    pos = {p: {op: i for i, op in enumerate(ops[p])} for p in ops}
    memo = {}

    def end(p: int, i: int) -> float:
        key = (p, i)
        if key in memo:
            return memo[key]
        kind, k = ops[p][i]
        ready = end(p, i - 1) if i > 0 else 0.0
        if kind == "F":
            if p > 1:
                ready = max(ready, end(p - 1, pos[p - 1][("F", k)]) + p2p)
            dur = t_fwd[k]
        else:
            if p < d_p:
                ready = max(ready, end(p + 1, pos[p + 1][("B", k)]) + p2p)
            dur = t_bwd[k] + (t_recomp[p - 1][k] if t_recomp is not None else 0.0)
        memo[key] = ready + dur
        return memo[key]

    import sys
    sys.setrecursionlimit(max(10000, 8 * n * d_p + 1000))
    makespan = max(end(p, len(ops[p]) - 1) for p in ops)
    busy, peak, held = [], [], []
    for p in range(1, d_p + 1):
        busy.append(sum(t_fwd[k] if kind == "F" else t_bwd[k] + (t_recomp[p - 1][k] if t_recomp is not None else 0.0)
                        for kind, k in ops[p]))
        cur_m, cur_n, pk_m, pk_n = 0.0, 0, 0.0, 0
        for kind, k in ops[p]:
            if kind == "F":
                cur_m += mem[p - 1][k] if mem is not None else 0.0
                cur_n += 1
                pk_m, pk_n = max(pk_m, cur_m), max(pk_n, cur_n)
            else:
                cur_m -= mem[p - 1][k] if mem is not None else 0.0
                cur_n -= 1
        peak.append(pk_m)
        held.append(pk_n)
    return makespan, busy, peak, held


def units_of_chunks(chunks):
    """Sequences as the scheduler sees them, from the chunks (C, slices, I) of the sequence processor: the split
    chunks of one long sequence in order followed by the chunk that holds its tail slice; every other chunk alone.
    Returns lists of chunk indices."""
    units = []
    for c, (ctx, slices, is_split) in enumerate(chunks):
        if is_split:
            continue
        head = []
        if ctx > 0:
            seq = slices[0][0]
            head = sorted((j for j, (cj, sj, ij) in enumerate(chunks) if ij and sj[0][0] == seq), key=lambda j: chunks[j][0])
        units.append(head + [c])
    return units


def plan_batch(plan_oracle, cost, mem: MemModel, lengths, ks, fwd_fraction: float, mesh_of):
    """The whole solve (sections 3.3 and 3.4): for every K, chunks from the sequence processor's reference
    (plan_oracle.process on the mesh and thresholds mesh_of(K) supplies), grouping and checkpointing by trying
    everything; estimated time = sum of chunk times * layers / d_p + sum over pipelines of (delta + F_hat * sum C),
    delta = (d_p - 1) * mean chunk time * layers / d_p, F_hat = fwd_fraction * mean chunk time.  Returns
    (K, time, chunks, groups) of the best K (ties: the smaller K) or None."""
    best = None
    per_stage = mem.layers / mem.d_p
    for K in ks:
        mesh, t_t, t_m = mesh_of(K)
        chunks, _ = plan_oracle.process(cost, 10 ** 12, lengths, mesh, t_t, t_m)
        times = [plan_oracle.t_tot(cost, ctx, [s[2] for s in sl]) for ctx, sl, _ in chunks]
        units = units_of_chunks(chunks)
        mean_t = sum(times) / len(times)
        sched_units = [[(sum(s[2] for s in chunks[c][1]), chunks[c][2]) for c in u] for u in units]
        r = group(mem, sched_units, fwd_fraction * mean_t, (mem.d_p - 1) * mean_t * per_stage)
        if r is None:
            continue
        total = sum(times) * per_stage + r[0]
        if best is None or total < best[1] * (1.0 - 1e-12):
            best = (K, total, chunks, [[units[u] for u in g] for g in r[1]])
    return best
