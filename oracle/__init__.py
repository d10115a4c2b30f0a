"""Python face of the CPU fp64 oracle (oracle/chunk_attn_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may use this package; the
GPU library never does, and this package imports nothing from it.

Arrays in, arrays out: Q, dO as [Tq, Hq, d]; K, V as [Tkv, Hkv, d]; either float64 numpy
arrays or bf16 torch CPU tensors (passed to C as bit patterns and widened exactly).
Segments are (q_start, q_len, kv_start, kv_len) tuples; see the C file's header for the
definition that is computed and the paper passages it follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "chunk_attn_oracle.c")
_LIB = os.path.join(_HERE, "libchunk_attn_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, no fast-math, OpenMP).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-o", tmp,
                               _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class _Seg(ctypes.Structure):
    _fields_ = [("q_start", ctypes.c_int32), ("q_len", ctypes.c_int32),
                ("kv_start", ctypes.c_int32), ("kv_len", ctypes.c_int32)]


class _Problem(ctypes.Structure):
    _fields_ = [("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("num_segments", ctypes.c_int32), ("segments", ctypes.POINTER(_Seg)),
                ("scale", ctypes.c_double), ("is_bf16", ctypes.c_int32)]


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_pair_count.restype = ctypes.c_int64
        for f in (_lib.oracle_fwd_rows, _lib.oracle_dq_rows, _lib.oracle_dkv_rows):
            f.restype = ctypes.c_int
    return _lib


def _as_input(x):
    """-> (numpy array kept alive, is_bf16)."""
    if isinstance(x, np.ndarray):
        return np.ascontiguousarray(x, dtype=np.float64), 0
    import torch
    assert isinstance(x, torch.Tensor) and x.dtype == torch.bfloat16, "inputs: float64 numpy or bf16 torch"
    return x.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16), 1


class Oracle:
    """One chunk-attention problem: segment table, head counts, scale and the input tensors."""

    def __init__(self, segs, q, k, v, d_o=None, scale=None):
        self.q, b0 = _as_input(q)
        self.k, b1 = _as_input(k)
        self.v, b2 = _as_input(v)
        kinds = {b0, b1, b2}
        self.d_o = None
        if d_o is not None:
            self.d_o, b3 = _as_input(d_o)
            kinds.add(b3)
        assert len(kinds) == 1, "all inputs must share one dtype"
        self.total_q, self.Hq, self.d = self.q.shape
        self.total_kv, self.Hkv, d2 = self.k.shape
        assert d2 == self.d and self.v.shape == self.k.shape and self.Hq % self.Hkv == 0
        assert self.d_o is None or self.d_o.shape == self.q.shape
        self.segs = [tuple(int(a) for a in s) for s in segs]
        for (qs, ql, ks, kl) in self.segs:
            assert ql >= 1 and kl >= ql and qs >= 0 and ks >= 0
            assert qs + ql <= self.total_q and ks + kl <= self.total_kv
        self._segarr = (_Seg * len(self.segs))(*[_Seg(*s) for s in self.segs])
        self.scale = float(scale) if scale is not None else 1.0 / np.sqrt(self.d)
        self._p = _Problem(self.Hq, self.Hkv, self.d, len(self.segs), self._segarr, self.scale, kinds.pop())

    @staticmethod
    def _ptr(a):
        return a.ctypes.data_as(ctypes.c_void_p)

    def _pairs(self, heads, rows):
        heads = np.ascontiguousarray(heads, dtype=np.int32).ravel()
        rows = np.ascontiguousarray(rows, dtype=np.int32).ravel()
        assert heads.shape == rows.shape
        return heads, rows

    def covered_rows(self):
        return np.concatenate([np.arange(qs, qs + ql) for (qs, ql, _, _) in self.segs])

    def pair_count(self) -> int:
        return int(_load().oracle_pair_count(ctypes.byref(self._p)))

    def fwd_rows(self, heads, rows):
        """O [n, d] and LSE [n] (natural log) for the listed (head, query row) pairs."""
        heads, rows = self._pairs(heads, rows)
        n = heads.size
        o = np.zeros((n, self.d)); lse = np.zeros(n)
        rc = _load().oracle_fwd_rows(ctypes.byref(self._p), self._ptr(self.q), self._ptr(self.k), self._ptr(self.v),
                                     ctypes.c_int64(n), self._ptr(heads), self._ptr(rows), self._ptr(o),
                                     self._ptr(lse))
        if rc != 0:
            raise ValueError("row outside every segment or bad head index")
        return o, lse

    def dq_rows(self, heads, rows):
        """dQ [n, d], LSE [n], D [n] for the listed (head, query row) pairs."""
        assert self.d_o is not None
        heads, rows = self._pairs(heads, rows)
        n = heads.size
        dq = np.zeros((n, self.d)); lse = np.zeros(n); dsum = np.zeros(n)
        rc = _load().oracle_dq_rows(ctypes.byref(self._p), self._ptr(self.q), self._ptr(self.k), self._ptr(self.v),
                                    self._ptr(self.d_o), ctypes.c_int64(n), self._ptr(heads), self._ptr(rows),
                                    self._ptr(dq), self._ptr(lse), self._ptr(dsum))
        if rc != 0:
            raise ValueError("row outside every segment or bad head index")
        return dq, lse, dsum

    def dkv_rows(self, kv_heads, kv_rows, lse_table, dsum_table):
        """dK [n, d], dV [n, d] for the listed (kv head, key row) pairs.

        lse_table, dsum_table: [Hq, total_q] float64, valid for every query that sees a listed key.
        """
        assert self.d_o is not None
        kv_heads, kv_rows = self._pairs(kv_heads, kv_rows)
        n = kv_heads.size
        lse_table = np.ascontiguousarray(lse_table, dtype=np.float64)
        dsum_table = np.ascontiguousarray(dsum_table, dtype=np.float64)
        assert lse_table.shape == (self.Hq, self.total_q) == dsum_table.shape
        dk = np.zeros((n, self.d)); dv = np.zeros((n, self.d))
        _load().oracle_dkv_rows(ctypes.byref(self._p), self._ptr(self.q), self._ptr(self.k), self._ptr(self.v),
                                self._ptr(self.d_o), ctypes.c_int64(self.total_q), self._ptr(lse_table),
                                self._ptr(dsum_table), ctypes.c_int64(n), self._ptr(kv_heads), self._ptr(kv_rows),
                                self._ptr(dk), self._ptr(dv))
        return dk, dv

    # ---- whole-tensor conveniences (small problems) -------------------------------------
    def _all_pairs(self, head_list=None):
        rows = self.covered_rows()
        hl = np.arange(self.Hq) if head_list is None else np.asarray(head_list)
        return np.repeat(hl, rows.size).astype(np.int32), np.tile(rows, hl.size).astype(np.int32)

    def forward(self):
        """O [Tq, Hq, d], LSE [Hq, Tq]; rows outside every segment are left at zero."""
        heads, rows = self._all_pairs()
        o, lse = self.fwd_rows(heads, rows)
        O = np.zeros((self.total_q, self.Hq, self.d)); L = np.zeros((self.Hq, self.total_q))
        O[rows, heads] = o
        L[heads, rows] = lse
        return O, L

    def lse_d_tables(self, head_list=None):
        """(dQ rows, LSE table, D table) for all covered rows of the listed heads (all by default)."""
        heads, rows = self._all_pairs(head_list)
        dq, lse, dsum = self.dq_rows(heads, rows)
        L = np.zeros((self.Hq, self.total_q)); D = np.zeros((self.Hq, self.total_q))
        L[heads, rows] = lse
        D[heads, rows] = dsum
        return (heads, rows, dq), L, D

    def backward(self):
        """dQ [Tq, Hq, d], dK [Tkv, Hkv, d], dV [Tkv, Hkv, d] (rows nobody touches stay zero)."""
        (heads, rows, dq), L, D = self.lse_d_tables()
        dQ = np.zeros((self.total_q, self.Hq, self.d))
        dQ[rows, heads] = dq
        kvrows = np.unique(np.concatenate([np.arange(ks, ks + kl) for (_, _, ks, kl) in self.segs]))
        kh = np.repeat(np.arange(self.Hkv), kvrows.size).astype(np.int32)
        kr = np.tile(kvrows, self.Hkv).astype(np.int32)
        dk, dv = self.dkv_rows(kh, kr, L, D)
        dK = np.zeros((self.total_kv, self.Hkv, self.d)); dV = np.zeros_like(dK)
        dK[kr, kh] = dk
        dV[kr, kh] = dv
        return dQ, dK, dV
