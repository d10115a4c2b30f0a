"""CPU-only tests of the C ABI: the library loads, exports every symbol the header declares, and rejects bad
descriptors on the host with the documented codes (no GPU is touched)."""
import ctypes
import os
import re

import pytest

import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def ca():
    import paper_2509_21275_amd as ca
    if not os.path.exists(ca.LIB_PATH):
        from paper_2509_21275_amd.build import build_library
        build_library()
    return ca


def test_library_exports_every_declared_symbol(ca):
    names = set()
    for h in sorted(os.listdir(os.path.join(ROOT, "include"))):
        header = open(os.path.join(ROOT, "include", h)).read()
        header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
        names |= set(re.findall(r"\b((?:chunk_attn|chunk_plan|chunk_sched|fused_ce)_[a-z0-9_]+)\s*\(", header))
    assert {"chunk_attn_fwd", "chunk_attn_bwd", "chunk_attn_bwd_f32kv", "chunk_attn_workspace_bytes", "chunk_attn_validate",
            "chunk_attn_pair_count", "chunk_attn_strerror", "chunk_attn_profile_events", "chunk_attn_shutdown",
            "chunk_attn_test_set_fwd_rescale_limit",
            "chunk_plan_time", "chunk_plan_mesh", "chunk_plan_build", "chunk_plan_segments", "fused_ce_inplace",
            "chunk_sched_act_bytes", "chunk_sched_f2b", "chunk_sched_windows", "chunk_sched_solve_ckpt", "chunk_sched_group",
            "chunk_sched_simulate", "chunk_sched_plan_batch"} <= names
    lib = ctypes.CDLL(ca.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in the header but not exported"


def desc(ca, segs, Hq=8, Hkv=2, d=128, tq=None, tkv=None, scale=0.1):
    tq = tq if tq is not None else max(s[0] + s[1] for s in segs)
    tkv = tkv if tkv is not None else max(s[2] + s[3] for s in segs)
    return ca.make_desc(segs, Hq, Hkv, d, tq, tkv, scale)


def test_valid_descriptors(ca):
    for idx in range(1, 6):
        c = synth.case_by_index(idx)
        d = ca.make_desc(c.segs, c.num_q_heads, c.num_kv_heads, c.head_dim, c.total_q, c.total_kv, c.scale)
        assert ca.chunk_attn_validate(d) == ca.OK
        assert ca.chunk_attn_pair_count(d) == c.pairs
        f, b = ca.chunk_attn_workspace_bytes(d)
        assert f > 0 and b > 0 and f % 256 == 0 and b % 256 == 0
    # key ranges may leave gaps; a hybrid chunk is legal; so are several segments with context
    assert ca.chunk_attn_validate(desc(ca, [(0, 4, 3, 10), (4, 6, 20, 9)], tkv=40)) == ca.OK


def test_head_dimensions(ca):
    """64, 96, 128 and 256 are accepted; 96 runs as 128 on zero-padded copies kept in the workspace, so its workspace
    is that of 128 plus the copies (Q, K, V, O for the forward; Q, K, V, O, dO, dQ and float32-sized dK, dV for the
    backward)."""
    segs = [(0, 300, 0, 500), (300, 212, 500, 212)]
    sizes = {}
    for d in (64, 96, 128, 256):
        dd = desc(ca, segs, Hq=8, Hkv=2, d=d)
        assert ca.chunk_attn_validate(dd) == ca.OK
        assert ca.chunk_attn_pair_count(dd) == 300 * 200 + 300 * 301 // 2 + 212 * 213 // 2
        sizes[d] = ca.chunk_attn_workspace_bytes(dd)
    up = lambda x: (x + 255) // 256 * 256
    qb, kb, gb = up(512 * 8 * 128 * 2), up(712 * 2 * 128 * 2), up(712 * 2 * 128 * 4)
    assert sizes[96][0] == sizes[128][0] + 2 * qb + 2 * kb
    assert sizes[96][1] == sizes[128][1] + 4 * qb + 2 * kb + 2 * gb
    for d in (32, 80, 192, 512):
        assert ca.chunk_attn_validate(desc(ca, segs, d=d)) == ca.UNSUPPORTED
    assert "64, 96, 128 or 256" in ca.chunk_attn_strerror(ca.UNSUPPORTED)


@pytest.mark.parametrize("segs,kw,code", [
    ([(0, 0, 0, 4)], {"tq": 4}, "BAD_SEGMENT"),                        # empty query range
    ([(0, 8, 0, 4)], {}, "BAD_SEGMENT"),                          # fewer keys than queries
    ([(1, 4, 0, 4)], {"tq": 5}, "BAD_SEGMENT"),                   # queries must start at row 0
    ([(0, 4, 0, 4), (5, 4, 4, 4)], {}, "BAD_SEGMENT"),            # hole in the query rows
    ([(0, 4, 0, 4), (4, 4, 2, 4)], {}, "BAD_SEGMENT"),            # overlapping key ranges
    ([(0, 4, 0, 4)], {"tq": 6}, "BAD_SEGMENT"),                   # queries do not cover total_q
    ([(0, 4, 0, 8)], {"tkv": 6}, "BAD_SEGMENT"),                  # key range past total_kv
    ([(0, 4, 0, 4)], {"d": 80}, "UNSUPPORTED"),
    ([(0, 4, 0, 4)], {"Hq": 6, "Hkv": 4}, "UNSUPPORTED"),
    ([(0, 4, 0, 4)], {"scale": 0.0}, "INVALID_ARG"),
    ([(0, 4, 0, 4)], {"scale": float("nan")}, "INVALID_ARG"),
    ([(0, 4, 0, 4)], {"Hq": 0}, "INVALID_ARG"),
])
def test_bad_descriptors(ca, segs, kw, code):
    d = desc(ca, segs, **kw)
    rc = ca.chunk_attn_validate(d)
    assert rc == getattr(ca, code), ca.chunk_attn_strerror(rc)
    with pytest.raises(ca.ChunkAttnError):
        ca.chunk_attn_workspace_bytes(d)
    with pytest.raises(ca.ChunkAttnError):
        ca.chunk_attn_pair_count(d)


def test_null_descriptor_and_messages(ca):
    lib = ctypes.CDLL(ca.LIB_PATH)
    lib.chunk_attn_validate.restype = ctypes.c_int
    assert lib.chunk_attn_validate(None) == ca.INVALID_ARG
    for code in (0, -1, -2, -3, -4, -5, -99):
        assert isinstance(ca.chunk_attn_strerror(code), str) and ca.chunk_attn_strerror(code)


def test_clock_log_hook_checks_its_buffer(ca):
    """The hook only stores the pointer: size and alignment are checked on the host, null switches it off."""
    import ctypes
    lib = ctypes.CDLL(ca.LIB_PATH)
    lib.chunk_attn_measure_set_clock_log.argtypes = [ctypes.c_void_p, ctypes.c_size_t]
    lib.chunk_attn_measure_set_clock_log.restype = ctypes.c_int
    assert ca.CLOCK_LOG_BYTES == 3 * 4096 * 8
    assert lib.chunk_attn_measure_set_clock_log(None, 0) == ca.OK
    assert lib.chunk_attn_measure_set_clock_log(ctypes.c_void_p(4096), ca.CLOCK_LOG_BYTES - 1) == ca.WORKSPACE_TOO_SMALL
    assert lib.chunk_attn_measure_set_clock_log(ctypes.c_void_p(4100), ca.CLOCK_LOG_BYTES) == ca.INVALID_ARG
    assert lib.chunk_attn_measure_set_clock_log(None, 0) == ca.OK


def test_shutdown_without_any_upload_is_a_no_op(ca):
    # nothing has been uploaded in this process: there is nothing to release, and no GPU call is made
    lib = ctypes.CDLL(ca.LIB_PATH)
    assert lib.chunk_attn_shutdown() == ca.OK
    assert lib.chunk_attn_shutdown() == ca.OK
    ca.chunk_attn_shutdown()


def test_synthetic_workloads_have_the_documented_shapes():
    c3 = synth.case_by_index(3); c4 = synth.case_by_index(4)
    assert c3.segs[0] == synth.Seg(0, 8192, 0, 65536) and c3.total_q == 16384 and c3.total_kv == 73728
    assert all(s.kv_len == s.q_len and 1 <= s.q_len <= 4096 for s in c3.segs[1:])
    assert sum(s.q_len for s in c4.segs) == 65536 and all(s.q_len <= 16384 for s in c4.segs)
    assert all(s.q_len >= 128 for s in c4.segs[:-1])
    for i in range(8):
        c5 = synth.case_by_index(5, i)
        assert c5.segs == [synth.Seg(0, 16384, 0, 16384 * (i + 1))]
    # determinism of the tensor generator: same (seed, id, index) -> same value, independent of blocking
    import torch
    a = synth.normal_bf16(7, 3, (5000,)); b = synth.normal_bf16(7, 3, (5000,), block=777)
    assert torch.equal(a, b)
