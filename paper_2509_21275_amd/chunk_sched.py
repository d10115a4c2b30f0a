"""Python binding of the host-side chunk scheduler (include/chunk_sched.h): sequence grouping (paper section
3.4.2), stage-aware chunk-level checkpointing (section 3.4.3, Algorithm 2) and a 1F1B timeline.  Argument
marshalling only; the work is done by the C++ code in libchunk_attn.so.
"""
from __future__ import annotations

import ctypes
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

from . import _lib, ChunkAttnError


class _MemModel(ctypes.Structure):
    _fields_ = [("d_p", ctypes.c_int32), ("d_s", ctypes.c_int32), ("layers", ctypes.c_int32),
                ("m_token", ctypes.c_double), ("m_logits", ctypes.c_double), ("e", ctypes.c_double),
                ("hidden", ctypes.c_double), ("kv_hidden", ctypes.c_double), ("capacity", ctypes.c_double),
                ("m_ms", ctypes.POINTER(ctypes.c_double))]


class _Chunk(ctypes.Structure):
    _fields_ = [("tokens", ctypes.c_int32), ("is_split", ctypes.c_int32)]


@dataclass
class MemModel:
    """Memory model of sections 3.2.2 / 3.2.3 (bytes): m_ms[p - 1] is the model-state footprint of stage p."""
    d_p: int
    d_s: int
    layers: int
    m_token: float
    m_logits: float
    e: float
    hidden: float
    kv_hidden: float
    capacity: float
    m_ms: Sequence[float]

    def _c(self):
        arr = (ctypes.c_double * max(1, len(self.m_ms)))(*self.m_ms)
        m = _MemModel(self.d_p, self.d_s, self.layers, self.m_token, self.m_logits, self.e, self.hidden, self.kv_hidden,
                      self.capacity, ctypes.cast(arr, ctypes.POINTER(ctypes.c_double)))
        m._keep = arr
        if len(self.m_ms) != self.d_p:
            raise ChunkAttnError(-1)
        return m


_bound = False


def _bind():
    global _bound
    if _bound:
        return
    mm, ck = ctypes.POINTER(_MemModel), ctypes.POINTER(_Chunk)
    i32, i32p, i64p, dbl, dblp = ctypes.c_int32, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int64), \
        ctypes.c_double, ctypes.POINTER(ctypes.c_double)
    _lib.chunk_sched_act_bytes.argtypes = [mm, i32, i32, i32, i32]
    _lib.chunk_sched_act_bytes.restype = dbl
    _lib.chunk_sched_f2b.argtypes = [i32p, i32, i32p]
    _lib.chunk_sched_f2b.restype = ctypes.c_int
    _lib.chunk_sched_windows.argtypes = [i32, i32, i32, i32, i32p, i32p, i32p, i32p]
    _lib.chunk_sched_windows.restype = ctypes.c_int
    _lib.chunk_sched_solve_ckpt.argtypes = [mm, ck, i32p, i32, i32, dbl, i32p, i64p, i32p, i64p, i64p]
    _lib.chunk_sched_solve_ckpt.restype = ctypes.c_int
    _lib.chunk_sched_group.argtypes = [mm, ck, i32p, i32, dbl, dbl, dbl, i32p, i32p, dblp, i32p, i32p, i32p, i32p, i32p]
    _lib.chunk_sched_group.restype = ctypes.c_int
    _lib.chunk_sched_simulate.argtypes = [i32, i32, i32, i32p, dblp, dblp, dblp, dblp, dbl, dblp, dblp, dblp, i32p]
    _lib.chunk_sched_simulate.restype = ctypes.c_int
    _bound = True


def _check(rc: int, what: str):
    if rc != 0:
        raise ChunkAttnError(rc)


def _i32(xs):
    return (ctypes.c_int32 * max(1, len(xs)))(*xs)


def _dbl(xs):
    return (ctypes.c_double * max(1, len(xs)))(*xs)


def _chunks(chunks: Sequence[Tuple[int, int]]):
    arr = (_Chunk * max(1, len(chunks)))()
    for i, (t, s) in enumerate(chunks):
        arr[i].tokens, arr[i].is_split = int(t), int(s)
    return arr


def chunk_sched_act_bytes(model: MemModel, p: int, tokens: int, is_split: int, l_ckpt: int) -> float:
    _bind()
    v = _lib.chunk_sched_act_bytes(ctypes.byref(model._c()), p, tokens, is_split, l_ckpt)
    if v < 0:
        raise ChunkAttnError(-1)
    return v


def chunk_sched_f2b(unit_of_chunk: Sequence[int]) -> List[int]:
    _bind()
    n = len(unit_of_chunk)
    out = _i32([0] * n)
    _check(_lib.chunk_sched_f2b(_i32(unit_of_chunk), n, out), "chunk_sched_f2b")
    return list(out)[:n]


def chunk_sched_windows(d_p: int, p: int, n: int, n_split: int, f2b: Sequence[int]) -> List[List[int]]:
    _bind()
    out = _i32([0] * (n * n))
    nw, w = ctypes.c_int32(), ctypes.c_int32()
    _check(_lib.chunk_sched_windows(d_p, p, n, n_split, _i32(f2b), out, ctypes.byref(nw), ctypes.byref(w)),
           "chunk_sched_windows")
    return [list(out[i * w.value:(i + 1) * w.value]) for i in range(nw.value)]


def chunk_sched_solve_ckpt(model: MemModel, chunks: Sequence[Tuple[int, int]], unit_of_chunk: Sequence[int],
                           n_split: int, gap: float = 0.0) -> Optional[Tuple[int, List[int], int, int]]:
    """Returns (sum of C, C, branch-and-bound nodes, proven lower bound of the sum) or None if even full checkpointing
    does not fit.  gap: relative optimality gap at which the search stops (0: smallest sum; nodes < 0: the search hit
    its node limit first)."""
    _bind()
    n = len(chunks)
    C = _i32([0] * (n + model.d_p - 1))
    s, nodes, ok, lb = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int32(), ctypes.c_int64()
    _check(_lib.chunk_sched_solve_ckpt(ctypes.byref(model._c()), _chunks(chunks), _i32(unit_of_chunk), n, n_split, gap, C,
                                       ctypes.byref(s), ctypes.byref(ok), ctypes.byref(nodes), ctypes.byref(lb)),
           "chunk_sched_solve_ckpt")
    if not ok.value:
        return None
    return s.value, list(C)[:n + model.d_p - 1], nodes.value, lb.value


@dataclass
class Pipeline:
    units: List[int]      # sequences in the order they run
    order: List[int]      # chunk indices in forward order
    C: List[int]          # the n + d_p - 1 checkpointing variables; ckpt(p, k) = C[f2b[k] + d_p - p]


def chunk_sched_group(model: MemModel, units: Sequence[Sequence[Tuple[int, int]]], layer_fwd_time: float,
                      delta: float, gap: float = 0.0) -> Optional[Tuple[float, List[Pipeline]]]:
    """units[u]: the (tokens, is_split) chunks of sequence u in order.  Returns (cost, pipelines) or None."""
    _bind()
    flat = [c for u in units for c in u]
    first = [0]
    for u in units:
        first.append(first[-1] + len(u))
    n_units, n_chunks = len(units), len(flat)
    gou, order = _i32([0] * n_units), _i32([0] * n_chunks)
    of, cf = _i32([0] * (n_units + 1)), _i32([0] * (n_units + 1))
    C = _i32([0] * (n_chunks + n_units * (model.d_p - 1)))
    ng, ok, cost = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_double()
    _check(_lib.chunk_sched_group(ctypes.byref(model._c()), _chunks(flat), _i32(first), n_units, layer_fwd_time, delta, gap,
                                  gou, ctypes.byref(ng), ctypes.byref(cost), order, of, C, cf, ctypes.byref(ok)),
           "chunk_sched_group")
    if not ok.value:
        return None
    pipes = []
    for g in range(ng.value):
        od = list(order[of[g]:of[g + 1]])
        us = []
        for k in od:
            u = max(i for i in range(n_units) if first[i] <= k)
            if not us or us[-1] != u:
                us.append(u)
        pipes.append(Pipeline(units=us, order=od, C=list(C[cf[g]:cf[g + 1]])))
    return cost.value, pipes


def chunk_sched_simulate(d_p: int, n_split: int, f2b: Sequence[int], t_fwd: Sequence[float], t_bwd: Sequence[float],
                         t_recomp=None, mem=None, p2p: float = 0.0):
    """Returns (makespan, busy[d_p], peak_mem[d_p], peak_held[d_p]); t_recomp / mem are [d_p][n] or None."""
    _bind()
    n = len(t_fwd)
    flat = lambda a: _dbl([x for row in a for x in row]) if a is not None else None
    ms = ctypes.c_double()
    busy, peak, held = _dbl([0.0] * d_p), _dbl([0.0] * d_p), _i32([0] * d_p)
    _check(_lib.chunk_sched_simulate(d_p, n, n_split, _i32(f2b), _dbl(t_fwd), _dbl(t_bwd), flat(t_recomp), flat(mem), p2p,
                                     ctypes.byref(ms), busy, peak, held), "chunk_sched_simulate")
    return ms.value, list(busy)[:d_p], list(peak)[:d_p], list(held)[:d_p]


@dataclass
class BatchPlan:
    k: int                          # the slice number K that won
    est_time: float                 # estimated time of the batch (see include/chunk_sched.h)
    chunks: list                    # chunk_plan.Chunk, as chunk_plan_build returns them
    pipeline_of_chunk: List[int]
    fwd_pos_of_chunk: List[int]     # position in its pipeline's forward order
    C: List[List[int]]              # per pipeline: the n + d_p - 1 checkpointing variables


def chunk_sched_plan_batch(cost, model: MemModel, token_capacity: int, lengths: Sequence[int], k_min: int, k_max: int,
                           align: int, fwd_fraction: float = 1.0 / 3.0, gap: float = 0.0) -> Optional[BatchPlan]:
    """The whole solve for one batch: K tuned in [k_min, k_max], sequence processor, grouping, checkpointing.
    cost: chunk_plan.CostModel.  Returns None if no K gives a plan that fits."""
    from . import chunk_plan as cp
    _bind()
    cp._bind()
    if not getattr(_lib, "_plan_batch_bound", False):
        i32, i32p, i64, dbl, dblp = ctypes.c_int32, ctypes.POINTER(ctypes.c_int32), ctypes.c_int64, ctypes.c_double, \
            ctypes.POINTER(ctypes.c_double)
        _lib.chunk_sched_plan_batch.argtypes = [ctypes.POINTER(cp.CostModel), ctypes.POINTER(_MemModel), i64, i32p, i32, i32, i32,
                                                i32, dbl, dbl, i32p, dblp, ctypes.POINTER(cp._Chunk), i32, i32p,
                                                ctypes.POINTER(cp._Slice), i32, i32p, i32p, i32p, i32p, i32p, i32p, i32p]
        _lib.chunk_sched_plan_batch.restype = ctypes.c_int
        _lib._plan_batch_bound = True
    n = len(lengths)
    cap = max(1, n * (k_max + 1))
    chunks, slices = (cp._Chunk * cap)(), (cp._Slice * cap)()
    pipe, pos, cf = _i32([0] * cap), _i32([0] * cap), _i32([0] * (cap + 1))
    C = _i32([0] * (cap * model.d_p))
    bk, nc, ns, npipe, ok, et = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32(), \
        ctypes.c_double()
    _check(_lib.chunk_sched_plan_batch(ctypes.byref(cost), ctypes.byref(model._c()), token_capacity, _i32(lengths), n, k_min,
                                       k_max, align, fwd_fraction, gap, ctypes.byref(bk), ctypes.byref(et), chunks, cap,
                                       ctypes.byref(nc), slices, cap, ctypes.byref(ns), pipe, pos, ctypes.byref(npipe), C, cf,
                                       ctypes.byref(ok)), "chunk_sched_plan_batch")
    if not ok.value:
        return None
    out = []
    for c in chunks[:nc.value]:
        sl = [(s.seq, s.start, s.len) for s in slices[c.first_slice:c.first_slice + c.num_slices]]
        out.append(cp.Chunk(c.context, sl, bool(c.is_split), c.tokens, c.time))
    return BatchPlan(bk.value, et.value, out, list(pipe[:nc.value]), list(pos[:nc.value]),
                     [list(C[cf[g]:cf[g + 1]]) for g in range(npipe.value)])
