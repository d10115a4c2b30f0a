"""Plain Python reference of the paper's sequence processor (section 3.3, Algorithm 1) and of the chunk cost model
(section 3.2.1, Eq. 1, Eq. 3, Eq. 4).  Test infrastructure only: it checks the C++ planner of the library and is never
used by the product path.

The steps are taken in the order of Algorithm 1.  Where the paper leaves a step open, the reading is the one
stated in the function's docstring.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple


@dataclass
class Model:
    alpha1: float
    alpha2: float
    beta1: float
    a2a_per_token: float = 0.0
    a2a_const: float = 0.0
    n_devices: int = 1
    dp: int = 1


def t_tot(m: Model, context: int, slices: List[int]) -> float:
    """T_tot(C, S) = T_comp(C, S) + T_all2all(S)  (Eq. 4): the first slice s0 pays alpha1 ((C + s0)^2 - C^2) + alpha2 s0,
    every other slice alpha1 s^2 + alpha2 s, all divided by N, plus beta1 / d_p (Eq. 1); the all-to-all term of Eq. 3 is
    linear in the chunk's tokens plus a constant."""
    s0 = slices[0]
    comp = m.alpha1 * ((context + s0) ** 2 - context ** 2) + m.alpha2 * s0
    for s in slices[1:]:
        comp += m.alpha1 * s ** 2 + m.alpha2 * s
    return comp / m.n_devices + m.beta1 / m.dp + m.a2a_per_token * sum(slices) + m.a2a_const


def balanced_mesh_time(m: Model, max_len: int, K: int, align: int) -> float:
    """The smallest possible value of the largest slice time when max_len tokens are cut into K consecutive slices, each
    a positive multiple of `align` except the last one (which takes what is left, at least one token), slice k having the
    slices before it as context: exhaustive dynamic programme over the cut positions.  ("K workload-balanced slices",
    the mesh step of Algorithm 1: the reading is that balanced means the largest T_tot is as small as it can be.)"""
    K = max(1, min(K, max_len // align))
    n_full = (max_len - 1) // align   # cut positions are align * 1 .. align * n_full (the last slice keeps >= 1 token)
    INF = float("inf")
    # best[k][p]: smallest possible largest time of k slices that end exactly at position p * align
    best = [[INF] * (n_full + 1) for _ in range(K)]
    best[0][0] = 0.0
    for k in range(1, K):
        for p in range(k, n_full + 1):
            for q in range(k - 1, p):
                if best[k - 1][q] == INF:
                    continue
                t = t_tot(m, q * align, [(p - q) * align])
                best[k][p] = min(best[k][p], max(best[k - 1][q], t))
    out = INF
    for q in range(K - 1, n_full + 1):
        if best[K - 1][q] == INF:
            continue
        out = min(out, max(best[K - 1][q], t_tot(m, q * align, [max_len - q * align])))
    return out


@dataclass
class Bucket:
    context: int = 0
    slices: List[Tuple[int, int, int]] = field(default_factory=list)  # (sequence, start, length), tail slice first

    def tokens(self) -> int:
        return sum(s[2] for s in self.slices)

    def time(self, m: Model) -> float:
        return t_tot(m, self.context, [s[2] for s in self.slices])


def process(m: Model, capacity: int, lengths: List[int], mesh: List[int], time_threshold: float, token_threshold: int):
    """Algorithm 1 after its mesh step, for a given mesh and thresholds (the mesh is checked separately, see
    balanced_mesh_time).  Returns (chunks, final time threshold); a chunk is (C, [(sequence, start, length), ...], I).

    Readings: a sequence longer than the first j mesh slices together yields j split chunks and a tail slice; the time
    of a bucket with one more sequence is T_tot of the combined chunk (the constants of Eq. 1 / Eq. 3 are paid once per
    chunk); buckets are tried in ascending order of tot_time / tot_tokens, ties in order of creation; when nothing fits,
    the time threshold becomes the smallest combined time among the buckets that have room for the tokens (the paper
    takes the minimum over all buckets, which need not terminate when the cheapest bucket is full).
    """
    split_chunks, tails, shorts = [], [], []
    for i, n in enumerate(lengths):                      # cut long sequences along the mesh
        pos, k = 0, 0
        while k < len(mesh) and pos + mesh[k] < n:
            split_chunks.append((pos, [(i, pos, mesh[k])], 1))
            pos += mesh[k]
            k += 1
        (tails if pos > 0 else shorts).append((i, pos, n - pos))
    buckets = [Bucket(context=t[1], slices=[t]) for t in tails]                      # one bucket per tail slice
    shorts.sort(key=lambda s: -t_tot(m, 0, [s[2]]))                                   # by decreasing time (stable)
    T_t, T_m = time_threshold, token_threshold
    for s in shorts:                                                                  # packing loop
        if not buckets or min(b.tokens() for b in buckets) + s[2] > T_m:            # no room anywhere
            buckets.append(Bucket(context=0, slices=[s]))
            continue
        while True:
            order = sorted(range(len(buckets)), key=lambda j: buckets[j].time(m) / buckets[j].tokens())
            placed = False
            for j in order:                                                           # first bucket that fits
                b = buckets[j]
                combined = t_tot(m, b.context, [x[2] for x in b.slices] + [s[2]])
                if combined <= T_t and b.tokens() + s[2] <= T_m:
                    b.slices.append(s)
                    placed = True
                    break
            if placed:
                break
            T_t = min(t_tot(m, b.context, [x[2] for x in b.slices] + [s[2]])          # relax T_t
                      for b in buckets if b.tokens() + s[2] <= T_m)
    chunks = split_chunks + [(b.context, b.slices, 0) for b in buckets]              # buckets become chunks
    return chunks, T_t


def segments(context: int, slice_lens: List[int]):
    """Rows of the chunk's Q and K/V tensors: the first slice attends to [context rows | own rows], every other slice to
    itself (section 3.1)."""
    segs, q, kv = [], 0, 0
    for i, s in enumerate(slice_lens):
        c = context if i == 0 else 0
        segs.append((q, s, kv, c + s))
        q += s
        kv += c + s
    return segs, q, kv
