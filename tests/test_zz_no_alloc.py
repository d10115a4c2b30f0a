"""chunk_attn_fwd_static, the forward that allocates nothing (its scratch memory is a fixed array inside the library),
against chunk_attn_fwd on the same inputs: identical bits, on two calls in a row, the second on a smaller chunk (the
array keeps the first call's contents), for every head dimension; chunks beyond its limits are refused on the host."""
import ctypes

import pytest
import torch

import synth
from gpu_util import make_inputs

pytestmark = pytest.mark.gpu


def _both(ca, lib, case):
    q, k, v, _ = make_inputs(case)
    desc = ca.make_desc(case.segs, case.num_q_heads, case.num_kv_heads, case.head_dim, case.total_q, case.total_kv,
                        case.scale)
    ws = ca.alloc_workspace(desc)
    o_ref = torch.full_like(q, float("nan"))
    lse_ref = torch.full((case.num_q_heads, case.total_q), float("nan"), dtype=torch.float32, device="cuda")
    ca.chunk_attn_fwd(desc, q, k, v, o_ref, lse_ref, ws)
    o = torch.full_like(q, float("nan")); lse = torch.full_like(lse_ref, float("nan"))
    torch.cuda.synchronize()
    print("chunk_attn_fwd_static", case.name, case.total_q, case.total_kv, case.head_dim, flush=True)
    P = lambda t: ctypes.c_void_p(t.data_ptr())
    rc = lib.chunk_attn_fwd_static(ctypes.byref(desc), P(q), P(k), P(v), P(o), P(lse),
                                   ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == ca.OK, ca.chunk_attn_strerror(rc)
    torch.cuda.synchronize()
    assert torch.equal(o, o_ref) and torch.equal(lse, lse_ref)


@pytest.mark.parametrize("d", [128, 64, 96, 256])
def test_static_forward_matches_the_workspace_forward_twice(d):
    import paper_2509_21275_amd as ca
    lib = ctypes.CDLL(ca.LIB_PATH)
    lib.chunk_attn_fwd_static.restype = ctypes.c_int
    big = synth.ChunkCase("hybrid_big", synth.hybrid_chunk(700, 1500, [300, 129, 64, 1, 257]), 1451, 2951, 8, 2, d, 71)
    small = synth.ChunkCase("packed_small", synth.packed_chunk([130, 33]), 163, 163, 8, 2, d, 72)
    _both(ca, lib, big)
    _both(ca, lib, small)   # fewer items, tiles and flags than the call before: nothing stale may be picked up
    _both(ca, lib, big)


def test_static_forward_second_pass():
    """Rows sent to the head_dim 128 forward's second pass read the transposed V images from the static array."""
    import paper_2509_21275_amd as ca
    lib = ctypes.CDLL(ca.LIB_PATH)
    lib.chunk_attn_fwd_static.restype = ctypes.c_int
    case = synth.ChunkCase("redo_forced", synth.hybrid_chunk(200, 500, [130, 70]), 400, 900, 8, 2, 128, 31)
    ca.chunk_attn_test_set_fwd_rescale_limit(-1e30)
    try:
        _both(ca, lib, case)
    finally:
        ca.chunk_attn_test_set_fwd_rescale_limit(60.0)


def test_static_forward_refuses_what_does_not_fit():
    import paper_2509_21275_amd as ca
    lib = ctypes.CDLL(ca.LIB_PATH)
    lib.chunk_attn_fwd_static.restype = ctypes.c_int
    P = lambda t: ctypes.c_void_p(t.data_ptr())
    # 65 segments
    case = synth.ChunkCase("many", synth.packed_chunk([4] * 65), 260, 260, 4, 2, 64, 73)
    q, k, v, _ = make_inputs(case)
    desc = ca.make_desc(case.segs, 4, 2, 64, 260, 260, case.scale)
    o = torch.empty_like(q); lse = torch.empty((4, 260), dtype=torch.float32, device="cuda")
    assert lib.chunk_attn_fwd_static(ctypes.byref(desc), P(q), P(k), P(v), P(o), P(lse), None) == ca.TOO_LARGE
    # a transposed copy of V beyond 16 MiB: 40000 keys x 2 heads x 128 x 2 bytes = 20 MB
    n = 40000
    desc = ca.make_desc([(0, 64, 0, n)], 8, 2, 128, 64, n, 0.1)
    f, _ = ca.chunk_attn_workspace_bytes(desc)
    assert f > (16 << 20)
    q = torch.zeros((64, 8, 128), dtype=torch.bfloat16, device="cuda"); kv = torch.zeros((n, 2, 128), dtype=torch.bfloat16, device="cuda")
    o = torch.empty_like(q); lse = torch.empty((8, 64), dtype=torch.float32, device="cuda")
    assert lib.chunk_attn_fwd_static(ctypes.byref(desc), P(q), P(kv), P(kv), P(o), P(lse), None) == ca.TOO_LARGE
    assert "16 MiB" in ca.chunk_attn_strerror(ca.TOO_LARGE)
    torch.cuda.synchronize()


def test_static_forward_under_graph_capture():
    """The callers the entry point is for: captured into a HIP graph (after one eager call, which takes the scratch
    array's address) and replayed several times with eager work in between, every replay gives the eager bits."""
    import paper_2509_21275_amd as ca
    case = synth.ChunkCase("hybrid_big", synth.hybrid_chunk(700, 1500, [300, 129, 64, 1, 257]), 1451, 2951, 8, 2, 128, 71)
    q, k, v, _ = make_inputs(case)
    desc = ca.make_desc(case.segs, 8, 2, 128, case.total_q, case.total_kv, case.scale)
    o_ref = torch.empty_like(q); lse_ref = torch.empty((8, case.total_q), dtype=torch.float32, device="cuda")
    ca.chunk_attn_fwd_static(desc, q, k, v, o_ref, lse_ref)
    torch.cuda.synchronize()
    o = torch.zeros_like(q); lse = torch.zeros_like(lse_ref)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    print("capturing chunk_attn_fwd_static", flush=True)
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            ca.chunk_attn_fwd_static(desc, q, k, v, o, lse, stream=side)
    torch.cuda.synchronize()
    for rep in range(4):
        o.fill_(float("nan")); lse.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(o, o_ref) and torch.equal(lse, lse_ref), rep
        other = synth.ChunkCase("packed_small", synth.packed_chunk([130, 33]), 163, 163, 8, 2, 128, 72)   # eager work
        q2, k2, v2, _ = make_inputs(other)
        d2 = ca.make_desc(other.segs, 8, 2, 128, 163, 163, other.scale)
        ca.chunk_attn_fwd_static(d2, q2, k2, v2, torch.empty_like(q2), torch.empty((8, 163), dtype=torch.float32, device="cuda"))
        torch.cuda.synchronize()
