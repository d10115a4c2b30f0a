"""Python binding of libchunk_attn.so, the MI355X chunk-attention library.

Argument marshalling only: every step of the computation runs in the library's HIP kernels.
The functions mirror the C ABI in include/chunk_attn.h (same names).  PyTorch is used for
device memory and streams; tensors must be contiguous bf16 (float32 for lse) on the GPU.
There is no CPU fallback: if the library is missing, importing fails loudly.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libchunk_attn.so")

OK, INVALID_ARG, UNSUPPORTED, BAD_SEGMENT, WORKSPACE_TOO_SMALL, HIP_ERROR, TOO_LARGE = 0, -1, -2, -3, -4, -5, -6


class Seg(ctypes.Structure):
    _fields_ = [("q_start", ctypes.c_int32), ("q_len", ctypes.c_int32),
                ("kv_start", ctypes.c_int32), ("kv_len", ctypes.c_int32)]


class Desc(ctypes.Structure):
    _fields_ = [("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("total_q", ctypes.c_int32), ("total_kv", ctypes.c_int32), ("num_segments", ctypes.c_int32),
                ("segments", ctypes.POINTER(Seg)), ("softmax_scale", ctypes.c_float)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2509_21275_amd.build` "
                          "(there is no fallback path)")
    # PyTorch first: it brings its own HIP runtime, and a process must not end up with the system's runtime loaded
    # by this library and PyTorch's tensors living in another one (both have the same soname; the first one loaded wins)
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = ctypes.CDLL(LIB_PATH)
    vp, sz = ctypes.c_void_p, ctypes.c_size_t
    dp = ctypes.POINTER(Desc)
    lib.chunk_attn_validate.argtypes = [dp]
    lib.chunk_attn_validate.restype = ctypes.c_int
    lib.chunk_attn_pair_count.argtypes = [dp]
    lib.chunk_attn_pair_count.restype = ctypes.c_int64
    lib.chunk_attn_strerror.argtypes = [ctypes.c_int]
    lib.chunk_attn_strerror.restype = ctypes.c_char_p
    lib.chunk_attn_workspace_bytes.argtypes = [dp, ctypes.POINTER(sz), ctypes.POINTER(sz)]
    lib.chunk_attn_workspace_bytes.restype = ctypes.c_int
    lib.chunk_attn_fwd.argtypes = [dp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.chunk_attn_fwd.restype = ctypes.c_int
    lib.chunk_attn_fwd_static.argtypes = [dp, vp, vp, vp, vp, vp, vp]
    lib.chunk_attn_fwd_static.restype = ctypes.c_int
    lib.chunk_attn_shutdown.restype = ctypes.c_int
    lib.chunk_attn_test_set_fwd_rescale_limit.argtypes = [ctypes.c_float]
    lib.chunk_attn_bwd.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_int, vp, sz, vp]
    lib.chunk_attn_bwd.restype = ctypes.c_int
    lib.chunk_attn_bwd_f32kv.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_int, vp, sz, vp]
    lib.chunk_attn_bwd_f32kv.restype = ctypes.c_int
    lib.chunk_attn_profile_events.argtypes = [vp, vp]
    lib.chunk_attn_profile_events.restype = ctypes.c_int
    lib.chunk_attn_measure_set_clock_log.argtypes = [vp, sz]
    lib.chunk_attn_measure_set_clock_log.restype = ctypes.c_int
    return lib


class _Lazy:
    """Loads the library on first use so that `python -m paper_2509_21275_amd.build` can run before it exists."""
    _real = None

    def __getattr__(self, name):
        if _Lazy._real is None:
            _Lazy._real = _load()
        return getattr(_Lazy._real, name)


_lib = _Lazy()


class ChunkAttnError(RuntimeError):
    def __init__(self, code):
        self.code = code
        super().__init__(f"chunk_attn error {code}: {_lib.chunk_attn_strerror(code).decode()}")


def make_desc(segs, num_q_heads, num_kv_heads, head_dim, total_q, total_kv, softmax_scale):
    """Builds a chunk_attn_desc; keep the returned object alive for the duration of the call."""
    arr = (Seg * max(1, len(segs)))(*[Seg(*[int(x) for x in s]) for s in segs])
    d = Desc(num_q_heads, num_kv_heads, head_dim, total_q, total_kv, len(segs), arr, float(softmax_scale))
    d._keepalive = arr
    return d


def chunk_attn_validate(desc) -> int:
    return _lib.chunk_attn_validate(ctypes.byref(desc))


def chunk_attn_strerror(code: int) -> str:
    return _lib.chunk_attn_strerror(code).decode()


def chunk_attn_pair_count(desc) -> int:
    n = _lib.chunk_attn_pair_count(ctypes.byref(desc))
    if n < 0:
        raise ChunkAttnError(int(n))
    return int(n)


def chunk_attn_workspace_bytes(desc):
    f, b = ctypes.c_size_t(0), ctypes.c_size_t(0)
    rc = _lib.chunk_attn_workspace_bytes(ctypes.byref(desc), ctypes.byref(f), ctypes.byref(b))
    if rc != OK:
        raise ChunkAttnError(rc)
    return f.value, b.value


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr())


def _check(t, dtype, shape, name):
    import torch
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous() and t.dtype == dtype
            and tuple(t.shape) == tuple(shape)):
        raise ValueError(f"{name}: expected contiguous {dtype} GPU tensor of shape {tuple(shape)}")


def _stream(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def chunk_attn_fwd(desc, q, k, v, o, lse, workspace, stream=None) -> None:
    """Enqueues the forward on `stream` (default: torch's current stream).  Writes o and lse."""
    import torch
    qs = (desc.total_q, desc.num_q_heads, desc.head_dim)
    ks = (desc.total_kv, desc.num_kv_heads, desc.head_dim)
    _check(q, torch.bfloat16, qs, "q"); _check(k, torch.bfloat16, ks, "k"); _check(v, torch.bfloat16, ks, "v")
    _check(o, torch.bfloat16, qs, "o"); _check(lse, torch.float32, (desc.num_q_heads, desc.total_q), "lse")
    rc = _lib.chunk_attn_fwd(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(workspace),
                             workspace.numel() * workspace.element_size(), _stream(stream))
    if rc != OK:
        raise ChunkAttnError(rc)


def chunk_attn_fwd_static(desc, q, k, v, o, lse, stream=None) -> None:
    """chunk_attn_fwd without a workspace: the library's fixed per-GPU scratch array is used (small chunks only)."""
    import torch
    qs = (desc.total_q, desc.num_q_heads, desc.head_dim)
    ks = (desc.total_kv, desc.num_kv_heads, desc.head_dim)
    _check(q, torch.bfloat16, qs, "q"); _check(k, torch.bfloat16, ks, "k"); _check(v, torch.bfloat16, ks, "v")
    _check(o, torch.bfloat16, qs, "o"); _check(lse, torch.float32, (desc.num_q_heads, desc.total_q), "lse")
    rc = _lib.chunk_attn_fwd_static(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _stream(stream))
    if rc != OK:
        raise ChunkAttnError(rc)


def chunk_attn_bwd(desc, q, k, v, o, d_o, lse, dq, dk, dv, accumulate_dkv, workspace, stream=None) -> None:
    """Enqueues the backward on `stream`.  Writes dq; writes or accumulates into dk, dv."""
    import torch
    qs = (desc.total_q, desc.num_q_heads, desc.head_dim)
    ks = (desc.total_kv, desc.num_kv_heads, desc.head_dim)
    for t, n in ((q, "q"), (o, "o"), (d_o, "d_o"), (dq, "dq")):
        _check(t, torch.bfloat16, qs, n)
    for t, n in ((k, "k"), (v, "v"), (dk, "dk"), (dv, "dv")):
        _check(t, torch.bfloat16, ks, n)
    _check(lse, torch.float32, (desc.num_q_heads, desc.total_q), "lse")
    rc = _lib.chunk_attn_bwd(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(d_o), _ptr(lse), _ptr(dq),
                             _ptr(dk), _ptr(dv), int(bool(accumulate_dkv)), _ptr(workspace),
                             workspace.numel() * workspace.element_size(), _stream(stream))
    if rc != OK:
        raise ChunkAttnError(rc)


def chunk_attn_bwd_f32kv(desc, q, k, v, o, d_o, lse, dq, dk, dv, accumulate_dkv, workspace, stream=None) -> None:
    """chunk_attn_bwd with float32 dk, dv (written, or added to in fp32)."""
    import torch
    qs = (desc.total_q, desc.num_q_heads, desc.head_dim)
    ks = (desc.total_kv, desc.num_kv_heads, desc.head_dim)
    for t, n in ((q, "q"), (o, "o"), (d_o, "d_o"), (dq, "dq")):
        _check(t, torch.bfloat16, qs, n)
    for t, n in ((k, "k"), (v, "v")):
        _check(t, torch.bfloat16, ks, n)
    for t, n in ((dk, "dk"), (dv, "dv")):
        _check(t, torch.float32, ks, n)
    _check(lse, torch.float32, (desc.num_q_heads, desc.total_q), "lse")
    rc = _lib.chunk_attn_bwd_f32kv(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(d_o), _ptr(lse), _ptr(dq),
                                   _ptr(dk), _ptr(dv), int(bool(accumulate_dkv)), _ptr(workspace),
                                   workspace.numel() * workspace.element_size(), _stream(stream))
    if rc != OK:
        raise ChunkAttnError(rc)


def chunk_attn_shutdown() -> None:
    """Releases the pinned staging buffers of the library (they are allocated again on demand)."""
    rc = _lib.chunk_attn_shutdown()
    if rc != 0:
        raise ChunkAttnError(rc)


def chunk_attn_test_set_fwd_rescale_limit(log2_growth: float) -> None:
    """Test hook: growth of a row's maximum (log2) past which the head_dim 128 forward takes its second pass."""
    _lib.chunk_attn_test_set_fwd_rescale_limit(ctypes.c_float(log2_growth))


def chunk_attn_measure_mfma_rate(milliseconds: int = 500, stream=None) -> float:
    """Measurement hook: TFLOP/s this GPU sustains on bf16 matrix instructions alone (its clock under matrix load)."""
    import torch
    scratch = torch.empty(1052672, dtype=torch.uint8, device="cuda")
    out = ctypes.c_double(0.0)
    rc = _lib.chunk_attn_measure_mfma_rate(ctypes.c_int(milliseconds), _ptr(scratch), ctypes.c_size_t(scratch.numel()),
                                           _stream(stream), ctypes.byref(out))
    if rc != 0:
        raise ChunkAttnError(rc)
    return out.value


def chunk_attn_measure_mfma_rate_on(workgroups: int, milliseconds: int = 500, stream=None) -> float:
    """The same with `workgroups` workgroups instead of one per CU (part of the chip busy)."""
    import torch
    scratch = torch.empty(1052672, dtype=torch.uint8, device="cuda")
    out = ctypes.c_double(0.0)
    rc = _lib.chunk_attn_measure_mfma_rate_on(ctypes.c_int(milliseconds), ctypes.c_int(workgroups), _ptr(scratch),
                                              ctypes.c_size_t(scratch.numel()), _stream(stream), ctypes.byref(out))
    if rc != 0:
        raise ChunkAttnError(rc)
    return out.value


CLOCK_LOG_BYTES = 3 * 4096 * 8
CLOCK_LOG_KERNELS = ("fwd", "dq", "dkv")


def chunk_attn_measure_set_clock_log(buffer) -> None:
    """Measurement hook: while `buffer` (a CUDA tensor of at least CLOCK_LOG_BYTES bytes, kept alive by the caller) is
    set, the workgroups of the pipelined forward, dQ and dK/dV kernels log their start and end counters there; None
    switches it off."""
    if buffer is None:
        rc = _lib.chunk_attn_measure_set_clock_log(None, 0)
    else:
        rc = _lib.chunk_attn_measure_set_clock_log(_ptr(buffer), ctypes.c_size_t(buffer.numel() * buffer.element_size()))
    if rc != 0:
        raise ChunkAttnError(rc)


def clock_log_sums(buffer) -> dict:
    """Decodes a clock log (after a synchronisation): per kernel {"workgroups", "ticks_100mhz", "shader_clocks"}, the
    last two summed over the workgroups that logged both a start and an end."""
    log = buffer.view(-1).cpu().numpy().view("uint64")[:3 * 4096].reshape(3, 1024, 4).astype("int64")
    out = {}
    for name, sec in zip(CLOCK_LOG_KERNELS, log):
        ok = (sec[:, 0] > 0) & (sec[:, 1] > sec[:, 0]) & (sec[:, 3] > sec[:, 2])
        out[name] = {"workgroups": int(ok.sum()), "ticks_100mhz": int((sec[ok, 1] - sec[ok, 0]).sum()),
                     "shader_clocks": int((sec[ok, 3] - sec[ok, 2]).sum())}
    return out


def chunk_attn_test_set_bwd_mode(mode: int) -> None:
    """Test hook: 0 = library's choice, 1 = two-kernel backward, 2 = one-pass backward (head_dim 128)."""
    rc = _lib.chunk_attn_test_set_bwd_mode(ctypes.c_int(mode))
    if rc != 0:
        raise ChunkAttnError(rc)


def chunk_attn_test_bwd_status(desc, workspace) -> int:
    """Test hook: the status word the one-pass backward left in `workspace` (synchronises the device)."""
    import torch
    off = ctypes.c_size_t(0)
    rc = _lib.chunk_attn_test_bwd_status_offset(ctypes.byref(desc), ctypes.byref(off))
    if rc != 0:
        raise ChunkAttnError(rc)
    torch.cuda.synchronize()
    return int(workspace[off.value:off.value + 4].view(torch.int32).item())


def chunk_attn_profile_events(start_event, stop_event) -> None:
    """Arms raw hipEvent_t handles (ints or None) for the next forward/backward call of this thread."""
    _lib.chunk_attn_profile_events(ctypes.c_void_p(start_event), ctypes.c_void_p(stop_event))


class HipEvents:
    """A pool of raw hipEvent_t pairs (timing enabled) created through the HIP runtime, for kernel timing."""

    def __init__(self):
        self._hip = ctypes.CDLL("libamdhip64.so")
        self._hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self._hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self._hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self._hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        self._all = []

    def record(self, event, stream=None) -> None:
        """Records `event` on `stream` (default: torch's current stream)."""
        rc = self._hip.hipEventRecord(ctypes.c_void_p(event), _stream(stream))
        if rc != 0:
            raise RuntimeError(f"hipEventRecord failed: {rc}")

    def pair(self):
        evs = []
        for _ in range(2):
            e = ctypes.c_void_p()
            rc = self._hip.hipEventCreate(ctypes.byref(e))
            if rc != 0:
                raise RuntimeError(f"hipEventCreate failed: {rc}")
            evs.append(e.value)
        self._all.extend(evs)
        return tuple(evs)

    def elapsed_ms(self, start, stop) -> float:
        ms = ctypes.c_float()
        rc = self._hip.hipEventElapsedTime(ctypes.byref(ms), ctypes.c_void_p(start), ctypes.c_void_p(stop))
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed: {rc}")
        return ms.value

    def close(self):
        for e in self._all:
            self._hip.hipEventDestroy(ctypes.c_void_p(e))
        self._all = []


def alloc_workspace(desc, device="cuda"):
    """A uint8 tensor large enough for both chunk_attn_fwd and chunk_attn_bwd on this descriptor."""
    import torch
    f, b = chunk_attn_workspace_bytes(desc)
    return torch.empty(max(f, b, 256), dtype=torch.uint8, device=device)
