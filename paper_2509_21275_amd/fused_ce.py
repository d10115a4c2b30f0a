"""Python binding of the fused in-place cross-entropy (include/fused_ce.h).  Argument marshalling only."""
from __future__ import annotations

import ctypes

from . import ChunkAttnError, _lib, _ptr, _stream

_bound = False


def fused_ce_inplace(logits, targets, loss, grad_scale: float = 1.0, stream=None) -> None:
    """logits: bf16 GPU tensor [rows, vocab] (rows may be strided by a multiple of 8 elements), overwritten with
    grad_scale * d loss_i / d logits; targets: int32 GPU tensor [rows] (negative: ignored row); loss: fp32 GPU tensor [rows]."""
    import torch
    global _bound
    if not _bound:
        _lib.fused_ce_inplace.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32,
                                          ctypes.c_int64, ctypes.c_float, ctypes.c_void_p]
        _lib.fused_ce_inplace.restype = ctypes.c_int
        _bound = True
    if not (logits.is_cuda and logits.dtype == torch.bfloat16 and logits.dim() == 2 and logits.stride(1) == 1):
        raise ValueError("logits: expected a bf16 GPU tensor [rows, vocab] with unit stride along the vocabulary")
    rows, vocab = logits.shape
    if not (targets.is_cuda and targets.dtype == torch.int32 and targets.is_contiguous() and tuple(targets.shape) == (rows,)):
        raise ValueError("targets: expected a contiguous int32 GPU tensor [rows]")
    if not (loss.is_cuda and loss.dtype == torch.float32 and loss.is_contiguous() and tuple(loss.shape) == (rows,)):
        raise ValueError("loss: expected a contiguous fp32 GPU tensor [rows]")
    rc = _lib.fused_ce_inplace(_ptr(logits), _ptr(targets), _ptr(loss), rows, vocab, logits.stride(0) if rows > 1 else vocab,
                               float(grad_scale), _stream(stream))
    if rc != 0:
        raise ChunkAttnError(rc)
