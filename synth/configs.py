"""Segment tables of the synthetic chunk workloads.

A chunk is a list of segments.  Segment t holds q_len query rows starting at q_start and
kv_len >= q_len key/value rows starting at kv_start; its context length is
C = kv_len - q_len (0 for a whole short sequence, > 0 for a slice of a long sequence that
comes with the keys and values of the slices before it).

  packed chunk : several whole sequences, C = 0 each
  split chunk  : one slice with C > 0 (or C = 0 for the first slice)
  hybrid chunk : a tail slice with C > 0 followed by whole short sequences

Length draws are log-normal, clipped, appended until the token budget is full, the last
one truncated to fit.  They stand in for the long-tailed length distributions of the
CommonCrawl and GitHub corpora the paper trains on, which are not available here.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, NamedTuple

import torch

from .tensors import uniform_u32

BASE_SEED = 250921275


class Seg(NamedTuple):
    q_start: int
    q_len: int
    kv_start: int
    kv_len: int


@dataclass
class ChunkCase:
    name: str
    segs: List[Seg]
    total_q: int
    total_kv: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    seed: int
    note: str = ""
    extra: dict = field(default_factory=dict)

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.head_dim)

    @property
    def pairs(self) -> int:
        """Unmasked (query, key) pairs per query head (bookkeeping, integer)."""
        return sum(s.q_len * (s.kv_len - s.q_len) + s.q_len * (s.q_len + 1) // 2 for s in self.segs)


def lognormal_lengths(seed: int, stream_id: int, budget: int, median: float, sigma: float,
                      lo: int, hi: int) -> List[int]:
    """Lengths round(exp(ln(median) + sigma z)) clipped to [lo, hi] until they fill `budget`."""
    out, tot, i = [], 0, 0
    while tot < budget:
        u1 = (float(uniform_u32(seed, 1000 + stream_id, 0, i, 1)[0]) + 0.5) / 4294967296.0
        u2 = (float(uniform_u32(seed, 1000 + stream_id, 1, i, 1)[0]) + 0.5) / 4294967296.0
        z = math.sqrt(-2.0 * math.log(u1)) * math.cos(2.0 * math.pi * u2)
        n = int(round(math.exp(math.log(median) + sigma * z)))
        n = max(lo, min(hi, n))
        n = min(n, budget - tot)
        out.append(n)
        tot += n
        i += 1
    return out


def packed_chunk(lengths) -> List[Seg]:
    segs, cum = [], 0
    for n in lengths:
        segs.append(Seg(cum, n, cum, n))
        cum += n
    return segs


def split_slice(q_len: int, context: int) -> List[Seg]:
    return [Seg(0, q_len, 0, context + q_len)]


def hybrid_chunk(tail_len: int, context: int, short_lengths) -> List[Seg]:
    segs = [Seg(0, tail_len, 0, context + tail_len)]
    cq, ckv = tail_len, context + tail_len
    for n in short_lengths:
        segs.append(Seg(cq, n, ckv, n))
        cq += n
        ckv += n
    return segs


def _totals(segs):
    return (max(s.q_start + s.q_len for s in segs), max(s.kv_start + s.kv_len for s in segs))


def case_by_index(idx: int, slice_index: int | None = None) -> ChunkCase:
    """The five benchmark workloads (1-based).  Case 5 is a per-slice call; pass slice_index 0..7."""
    seed = BASE_SEED + idx
    if idx == 1:
        segs = packed_chunk([256, 512, 128, 128])
        return ChunkCase("packed_1k", segs, 1024, 1024, 8, 8, 64, seed)
    if idx == 2:
        segs = split_slice(8192, 24576)
        return ChunkCase("split_32k_last_of_4", segs, 8192, 32768, 32, 8, 128, seed)
    if idx == 3:
        short = lognormal_lengths(seed, 0, 8192, 1024.0, 1.0, 128, 4096)
        segs = hybrid_chunk(8192, 57344, short)
        tq, tkv = _totals(segs)
        return ChunkCase("hybrid_64k_tail_plus_short", segs, tq, tkv, 32, 8, 128, seed,
                         extra={"short_lengths": short})
    if idx == 4:
        lens = lognormal_lengths(seed, 0, 65536, 2048.0, 1.2, 128, 16384)
        segs = packed_chunk(lens)
        return ChunkCase("packed_64k_skewed", segs, 65536, 65536, 32, 8, 128, seed,
                         extra={"lengths": lens})
    if idx == 5:
        i = 7 if slice_index is None else int(slice_index)
        assert 0 <= i < 8
        segs = split_slice(16384, 16384 * i)
        return ChunkCase(f"split_128k_slice{i}_of_8", segs, 16384, 131072, 64, 8, 128, seed,
                         extra={"slice": i, "num_slices": 8, "slice_len": 16384})
    raise ValueError("case index must be 1..5")


def scaled_case(idx: int, divisor: int = 16, slice_index: int | None = None) -> ChunkCase:
    """Same segment structure with every length divided by `divisor` and 8 query / 2 KV heads.

    Small enough for the CPU oracle to compute in full.
    """
    c = case_by_index(idx, slice_index)
    segs, cq, ckv = [], 0, 0
    for s in c.segs:
        ql = max(1, s.q_len // divisor)
        ctx = (s.kv_len - s.q_len) // divisor
        segs.append(Seg(cq, ql, ckv, ctx + ql))
        cq += ql
        ckv += ctx + ql
    tkv = ckv
    if idx == 5:
        tkv = 131072 // divisor
    return ChunkCase(c.name + f"_div{divisor}", segs, cq, tkv, 8, 2, c.head_dim, c.seed,
                     extra=dict(c.extra))
