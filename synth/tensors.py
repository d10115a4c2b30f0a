"""Counter-based random tensors: element i of tensor t under seed s depends only on (s, t, i).

uniform_u32 hashes the element index with a 32-bit integer mixer (two multiply-xorshift
rounds) keyed by (seed, tensor id, stream).  normal_bf16 turns two such streams into a
standard normal by the Box-Muller transform in float64 and rounds to bfloat16
(round-to-nearest-even, torch's conversion).  The integer part is bit-identical on every
device; generation runs in blocks so a 2^30-element tensor needs no large temporaries.
"""
from __future__ import annotations

import math

import torch

_M32 = 0xFFFFFFFF


def _mix32(x: torch.Tensor) -> torch.Tensor:
    """32-bit avalanche mixer on int64 containers holding values < 2**32."""
    x = x ^ (x >> 16)
    x = (x * 0x7FEB352D) & _M32
    x = x ^ (x >> 15)
    x = (x * 0x846CA68B) & _M32
    x = x ^ (x >> 16)
    return x


def _key(seed: int, tensor_id: int, stream: int) -> int:
    k = (seed * 0x9E3779B1 + tensor_id * 0x85EBCA77 + stream * 0xC2B2AE3D + 0x27D4EB2F) & _M32
    # scalar version of the same mixer
    k ^= k >> 16
    k = (k * 0x7FEB352D) & _M32
    k ^= k >> 15
    k = (k * 0x846CA68B) & _M32
    k ^= k >> 16
    return k


def uniform_u32(seed: int, tensor_id: int, stream: int, start: int, count: int,
                device: torch.device | str = "cpu") -> torch.Tensor:
    """int64 tensor of `count` values in [0, 2**32) for element indices start..start+count-1."""
    idx = torch.arange(start, start + count, dtype=torch.int64, device=device)
    lo = idx & _M32
    hi = (idx >> 32) & _M32
    x = _mix32(lo ^ _key(seed, tensor_id, stream))
    x = _mix32((x + hi * 0x632BE5AB + _key(seed, tensor_id, stream + 101)) & _M32)
    return x


def normal_bf16(seed: int, tensor_id: int, shape, device: torch.device | str = "cpu",
                block: int = 1 << 24) -> torch.Tensor:
    """bf16 tensor of `shape`, entries i.i.d. N(0,1) rounded to bf16, in row-major element order."""
    n = 1
    for s in shape:
        n *= int(s)
    out = torch.empty(n, dtype=torch.bfloat16, device=device)
    for start in range(0, n, block):
        cnt = min(block, n - start)
        u1 = (uniform_u32(seed, tensor_id, 0, start, cnt, device).double() + 0.5) * (1.0 / 4294967296.0)
        u2 = (uniform_u32(seed, tensor_id, 1, start, cnt, device).double() + 0.5) * (1.0 / 4294967296.0)
        z = torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)
        out[start:start + cnt] = z.to(torch.bfloat16)
    return out.reshape(*shape)


def to_f64(t: torch.Tensor):
    """Host float64 numpy copy of a tensor (exact widening for bf16)."""
    return t.detach().to("cpu").double().numpy()
