"""Python binding of the host-side sequence processor (include/chunk_plan.h): the paper's Algorithm 1
("Workload-Balanced Sequence Processing for Heterogeneous Chunks", section 3.3) with the cost model of
section 3.2.1.  Argument marshalling only; the work is done by the C++ code in libchunk_attn.so.
"""
from __future__ import annotations

import ctypes
from dataclasses import dataclass
from typing import List, Sequence, Tuple

from . import Seg, _lib, ChunkAttnError


class CostModel(ctypes.Structure):
    """T_tot(C, S) = (alpha1 ((C + s0)^2 - C^2) + alpha2 s0 + sum_{s != s0} (alpha1 s^2 + alpha2 s)) / n_devices
    + beta1 / dp + a2a_per_token * sum(S) + a2a_const   (Eq. 1, Eq. 3, Eq. 4)."""
    _fields_ = [("alpha1", ctypes.c_double), ("alpha2", ctypes.c_double), ("beta1", ctypes.c_double),
                ("a2a_per_token", ctypes.c_double), ("a2a_const", ctypes.c_double),
                ("n_devices", ctypes.c_int32), ("dp", ctypes.c_int32)]


class _Slice(ctypes.Structure):
    _fields_ = [("seq", ctypes.c_int32), ("start", ctypes.c_int32), ("len", ctypes.c_int32)]


class _Chunk(ctypes.Structure):
    _fields_ = [("context", ctypes.c_int64), ("first_slice", ctypes.c_int32), ("num_slices", ctypes.c_int32),
                ("is_split", ctypes.c_int32), ("tokens", ctypes.c_int32), ("time", ctypes.c_double)]


@dataclass
class Chunk:
    context: int                          # C
    slices: List[Tuple[int, int, int]]    # (sequence, start, length); the first one is s0
    is_split: bool                        # the paper's indicator I
    tokens: int
    time: float                           # T_tot(C, S)


_bound = False


def _bind():
    global _bound
    if _bound:
        return
    cm, i32p, i64p, dblp = ctypes.POINTER(CostModel), ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int64), \
        ctypes.POINTER(ctypes.c_double)
    _lib.chunk_plan_time.argtypes = [cm, ctypes.c_int64, i32p, ctypes.c_int32]
    _lib.chunk_plan_time.restype = ctypes.c_double
    _lib.chunk_plan_mesh.argtypes = [cm, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, i32p, i32p, dblp, i64p]
    _lib.chunk_plan_mesh.restype = ctypes.c_int
    _lib.chunk_plan_build.argtypes = [cm, ctypes.c_int64, i32p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                      ctypes.POINTER(_Chunk), ctypes.c_int32, i32p, ctypes.POINTER(_Slice), ctypes.c_int32,
                                      i32p, dblp, i64p]
    _lib.chunk_plan_build.restype = ctypes.c_int
    _lib.chunk_plan_segments.argtypes = [ctypes.POINTER(_Chunk), ctypes.POINTER(_Slice), ctypes.POINTER(Seg), i32p, i32p]
    _lib.chunk_plan_segments.restype = ctypes.c_int
    _bound = True


def _i32(values: Sequence[int]):
    return (ctypes.c_int32 * max(1, len(values)))(*[int(v) for v in values])


def chunk_plan_time(model: CostModel, context: int, slice_lens: Sequence[int]) -> float:
    _bind()
    return _lib.chunk_plan_time(ctypes.byref(model), int(context), _i32(slice_lens), len(slice_lens))


def chunk_plan_mesh(model: CostModel, max_len: int, K: int, align: int, capacity: int):
    """Returns (mesh, time_threshold, token_threshold)."""
    _bind()
    mesh = (ctypes.c_int32 * max(1, K))()
    k_out, tt, tm = ctypes.c_int32(), ctypes.c_double(), ctypes.c_int64()
    rc = _lib.chunk_plan_mesh(ctypes.byref(model), max_len, K, align, capacity, mesh, ctypes.byref(k_out),
                              ctypes.byref(tt), ctypes.byref(tm))
    if rc != 0:
        raise ChunkAttnError(rc)
    return list(mesh[:k_out.value]), tt.value, tm.value


def chunk_plan_build(model: CostModel, capacity: int, lengths: Sequence[int], K: int, align: int):
    """Algorithm 1.  Returns (chunks, time_threshold, token_threshold)."""
    _bind()
    n = len(lengths)
    cap = max(1, n * (K + 1))
    chunks, slices = (_Chunk * cap)(), (_Slice * cap)()
    nc, ns, tt, tm = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_double(), ctypes.c_int64()
    rc = _lib.chunk_plan_build(ctypes.byref(model), capacity, _i32(lengths), n, K, align, chunks, cap, ctypes.byref(nc),
                               slices, cap, ctypes.byref(ns), ctypes.byref(tt), ctypes.byref(tm))
    if rc != 0:
        raise ChunkAttnError(rc)
    out = []
    for c in chunks[:nc.value]:
        sl = [(s.seq, s.start, s.len) for s in slices[c.first_slice:c.first_slice + c.num_slices]]
        out.append(Chunk(c.context, sl, bool(c.is_split), c.tokens, c.time))
    return out, tt.value, tm.value


def chunk_plan_segments(chunk: Chunk):
    """Segment table of a chunk for chunk_attn_fwd / chunk_attn_bwd: (segments, total_q, total_kv)."""
    _bind()
    n = len(chunk.slices)
    sl = (_Slice * n)(*[_Slice(*s) for s in chunk.slices])
    c = _Chunk(chunk.context, 0, n, int(chunk.is_split), chunk.tokens, chunk.time)
    segs = (Seg * n)()
    tq, tkv = ctypes.c_int32(), ctypes.c_int32()
    rc = _lib.chunk_plan_segments(ctypes.byref(c), sl, segs, ctypes.byref(tq), ctypes.byref(tkv))
    if rc != 0:
        raise ChunkAttnError(rc)
    return [(s.q_start, s.q_len, s.kv_start, s.kv_len) for s in segs], tq.value, tkv.value
