"""GPU tests of the C ABI's call semantics: accumulation of dK/dV across the slices of a split sequence (in both
orders), determinism, re-callability of the forward, and error codes that need a device pointer."""
import numpy as np
import pytest
import torch

import synth
from gpu_util import TOL_GRAD, TOL_O, make_inputs, rel_err, run_gpu

pytestmark = pytest.mark.gpu


def _split_sequence(n_slices, slice_len, Hq, Hkv, d, seed):
    n = n_slices * slice_len
    q = synth.normal_bf16(seed, 0, (n, Hq, d), "cuda"); k = synth.normal_bf16(seed, 1, (n, Hkv, d), "cuda")
    v = synth.normal_bf16(seed, 2, (n, Hkv, d), "cuda"); do = synth.normal_bf16(seed, 3, (n, Hq, d), "cuda")
    return n, q, k, v, do


@pytest.mark.parametrize("order", ["reverse", "forward"])
def test_split_sequence_driver_matches_unsplit_oracle(oracle_mod, order):
    """8 slices of a 2048-token sequence (the 128K workload divided by 64): slice i attends to the keys/values of
    slices 0..i; the backward accumulates dK/dV over the slices.  The sum must equal the unsplit gradient."""
    n_slices, sl, Hq, Hkv, d = 8, 256, 8, 2, 128
    n, q, k, v, do = _split_sequence(n_slices, sl, Hq, Hkv, d, 555)
    dk = torch.zeros_like(k); dv = torch.zeros_like(v)
    o_all = torch.empty_like(q); dq_all = torch.empty_like(q)
    idx = range(n_slices - 1, -1, -1) if order == "reverse" else range(n_slices)
    for i in idx:
        case = synth.ChunkCase(f"slice{i}", synth.split_slice(sl, sl * i), sl, n, Hq, Hkv, d, 0)
        qi = q[i * sl:(i + 1) * sl].contiguous(); doi = do[i * sl:(i + 1) * sl].contiguous()
        o, lse, dq, dk, dv = run_gpu(case, qi, k, v, doi, accumulate=True, dk_init=dk, dv_init=dv)
        o_all[i * sl:(i + 1) * sl] = o; dq_all[i * sl:(i + 1) * sl] = dq
    whole = oracle_mod.Oracle([(0, n, 0, n)], q.cpu(), k.cpu(), v.cpu(), do.cpu())
    O, _ = whole.forward(); dQ, dK, dV = whole.backward()
    errs = (rel_err(o_all, O), rel_err(dq_all, dQ), rel_err(dk, dK), rel_err(dv, dV))
    print(order, errs, flush=True)
    assert errs[0] <= TOL_O and max(errs[1:]) <= TOL_GRAD


def test_accumulate_leaves_uncovered_rows_untouched_and_overwrite_zeroes_them(oracle_mod):
    segs = [(0, 100, 10, 150), (100, 60, 200, 60)]
    case = synth.ChunkCase("gaps", [synth.Seg(*s) for s in segs], 160, 300, 4, 2, 64, 31)
    q, k, v, do = make_inputs(case)
    init_k = torch.full_like(k, 3.0); init_v = torch.full_like(v, -2.0)
    _, _, _, dk_acc, dv_acc = run_gpu(case, q, k, v, do, accumulate=True, dk_init=init_k, dv_init=init_v)
    _, _, _, dk_ow, dv_ow = run_gpu(case, q, k, v, do)
    cov = torch.zeros(300, dtype=torch.bool)
    for s in segs:
        cov[s[2]:s[2] + s[3]] = True
    assert torch.all(dk_acc.cpu()[~cov] == 3.0) and torch.all(dv_acc.cpu()[~cov] == -2.0)
    assert torch.all(dk_ow.cpu()[~cov] == 0) and torch.all(dv_ow.cpu()[~cov] == 0)
    # covered rows: accumulate = bf16(init + fp32 sum); compare with the oracle plus the initial value
    orc = oracle_mod.Oracle(case.segs, q.cpu(), k.cpu(), v.cpu(), do.cpu(), case.scale)
    _, dK, dV = orc.backward()
    c = cov.numpy()
    assert rel_err(dk_acc.cpu()[cov], dK[c] + 3.0) <= TOL_GRAD
    assert rel_err(dv_acc.cpu()[cov], dV[c] - 2.0) <= TOL_GRAD


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5])
def test_results_are_bit_reproducible_and_forward_is_recallable(idx):
    """Every kernel writes each output once, in a fixed order of accumulation (no atomics): repeated calls agree bit for
    bit, for every chunk type and both head dimensions, whatever else the GPU was doing in between."""
    case = synth.scaled_case(idx, 16, 5 if idx == 5 else None)
    q, k, v, do = make_inputs(case)
    a = run_gpu(case, q, k, v, do)
    other = synth.scaled_case(4 if idx != 4 else 3, 16)   # unrelated work between the two calls
    run_gpu(other, *make_inputs(other))
    for _ in range(3):
        b = run_gpu(case, q, k, v, do)
        for x, y in zip(a, b):
            assert torch.equal(x, y)


def test_workspace_too_small_and_null_pointers_are_reported():
    import ctypes
    import paper_2509_21275_amd as ca
    case = synth.scaled_case(2, 16)
    q, k, v, do = make_inputs(case)
    desc = ca.make_desc(case.segs, case.num_q_heads, case.num_kv_heads, case.head_dim, case.total_q, case.total_kv,
                        case.scale)
    o = torch.empty_like(q); lse = torch.empty((case.num_q_heads, case.total_q), dtype=torch.float32, device="cuda")
    tiny = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(ca.ChunkAttnError) as e:
        ca.chunk_attn_fwd(desc, q, k, v, o, lse, tiny)
    assert e.value.code == ca.WORKSPACE_TOO_SMALL
    dq = torch.empty_like(q); dk = torch.empty_like(k); dv = torch.empty_like(v)
    with pytest.raises(ca.ChunkAttnError) as e:
        ca.chunk_attn_bwd(desc, q, k, v, o, do, lse, dq, dk, dv, 0, tiny)
    assert e.value.code == ca.WORKSPACE_TOO_SMALL
    lib = ctypes.CDLL(ca.LIB_PATH)
    lib.chunk_attn_fwd.restype = ctypes.c_int
    ws = ca.alloc_workspace(desc)
    rc = lib.chunk_attn_fwd(ctypes.byref(desc), None, ctypes.c_void_p(k.data_ptr()), ctypes.c_void_p(v.data_ptr()),
                            ctypes.c_void_p(o.data_ptr()), ctypes.c_void_p(lse.data_ptr()),
                            ctypes.c_void_p(ws.data_ptr()), ctypes.c_size_t(ws.numel()), None)
    assert rc == ca.INVALID_ARG


def test_shutdown_releases_the_staging_buffers_and_later_calls_start_over():
    """chunk_attn_shutdown frees the pinned upload buffers (waiting for uploads in flight); the next call allocates
    again and gives the same bits."""
    import paper_2509_21275_amd as ca
    case = synth.scaled_case(3, 16)
    q, k, v, do = make_inputs(case)
    a = run_gpu(case, q, k, v, do)
    ca.chunk_attn_shutdown()
    ca.chunk_attn_shutdown()          # nothing left to free
    b = run_gpu(case, q, k, v, do)
    # shut down while a call's upload may still be in flight: the release waits for it
    desc = ca.make_desc(case.segs, case.num_q_heads, case.num_kv_heads, case.head_dim, case.total_q, case.total_kv,
                        case.scale)
    ws = ca.alloc_workspace(desc)
    o = torch.empty_like(q); lse = torch.empty((case.num_q_heads, case.total_q), dtype=torch.float32, device="cuda")
    ca.chunk_attn_fwd(desc, q, k, v, o, lse, ws)
    ca.chunk_attn_shutdown()
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        assert torch.equal(x, y)
    assert torch.equal(o, a[0]) and torch.equal(lse, a[1])


def test_misaligned_tensor_pointers_are_rejected_on_the_host():
    """Rows are moved in 16-byte pieces: a tensor pointer that is not 16-byte aligned is an argument error, found
    before anything is launched."""
    import ctypes
    import paper_2509_21275_amd as ca
    case = synth.scaled_case(2, 16)
    q, k, v, do = make_inputs(case)
    desc = ca.make_desc(case.segs, case.num_q_heads, case.num_kv_heads, case.head_dim, case.total_q, case.total_kv,
                        case.scale)
    o = torch.empty_like(q); lse = torch.empty((case.num_q_heads, case.total_q), dtype=torch.float32, device="cuda")
    dq = torch.empty_like(q); dk = torch.empty_like(k); dv = torch.empty_like(v)
    ws = ca.alloc_workspace(desc)
    lib = ctypes.CDLL(ca.LIB_PATH)
    lib.chunk_attn_fwd.restype = ctypes.c_int
    lib.chunk_attn_bwd.restype = ctypes.c_int
    P = lambda t, off=0: ctypes.c_void_p(t.data_ptr() + off)
    wsz = ctypes.c_size_t(ws.numel())
    for bad in range(4):   # q, k, v, o each 2 bytes off
        args = [P(q), P(k), P(v), P(o)]
        args[bad] = P([q, k, v, o][bad], 2)
        assert lib.chunk_attn_fwd(ctypes.byref(desc), *args, P(lse), P(ws), wsz, None) == ca.INVALID_ARG
    for bad in range(8):   # q, k, v, o, d_o, dq, dk, dv
        ts = [q, k, v, o, do, None, dq, dk, dv]
        args = [P(t) if t is not None else P(lse) for t in ts]
        i = bad if bad < 5 else bad + 1
        args[i] = P(ts[i], 8)
        assert lib.chunk_attn_bwd(ctypes.byref(desc), *args, ctypes.c_int(0), P(ws), wsz, None) == ca.INVALID_ARG
    torch.cuda.synchronize()


def test_two_streams_with_a_workspace_each_do_not_disturb_each_other():
    """The head_dim 128 kernels launch one persistent workgroup per CU and hand out their blocks through counters in
    the workspace: two calls in flight at once, on two streams of the default priority with a workspace each, share the
    CUs without sharing anything else and give the bits of the same calls run one after the other."""
    import paper_2509_21275_amd as ca
    cases = [synth.scaled_case(4, 8), synth.scaled_case(3, 8)]
    ref, work = [], []
    for case in cases:
        q, k, v, do = make_inputs(case)
        ref.append(run_gpu(case, q, k, v, do))
        desc = ca.make_desc(case.segs, case.num_q_heads, case.num_kv_heads, case.head_dim, case.total_q, case.total_kv,
                            case.scale)
        o = torch.full_like(q, float("nan")); dq = torch.full_like(q, float("nan"))
        dk = torch.full_like(k, float("nan")); dv = torch.full_like(v, float("nan"))
        lse = torch.full((case.num_q_heads, case.total_q), float("nan"), dtype=torch.float32, device="cuda")
        work.append((desc, ca.alloc_workspace(desc), q, k, v, do, o, lse, dq, dk, dv, torch.cuda.Stream()))
    torch.cuda.synchronize()
    for rep in range(3):
        for desc, ws, q, k, v, do, o, lse, dq, dk, dv, st in work:
            ca.chunk_attn_fwd(desc, q, k, v, o, lse, ws, stream=st)
        for desc, ws, q, k, v, do, o, lse, dq, dk, dv, st in work:
            ca.chunk_attn_bwd(desc, q, k, v, o, do, lse, dq, dk, dv, 0, ws, stream=st)
    torch.cuda.synchronize()
    for (desc, ws, q, k, v, do, o, lse, dq, dk, dv, st), r in zip(work, ref):
        for x, y in zip((o, lse, dq, dk, dv), r):
            assert torch.equal(x, y)


def test_clock_log_reports_a_plausible_clock_and_changes_no_result():
    """The measurement hook: with the log switched on the three pipelined kernels give the same bits, every workgroup
    leaves a start and an end, and the clock they imply lies between 0.5 and 2.6 GHz (the chip's peak is 2.4)."""
    import paper_2509_21275_amd as ca
    case = synth.scaled_case(4, 8)
    q, k, v, do = make_inputs(case)
    ref = run_gpu(case, q, k, v, do)
    buf = torch.zeros(ca.CLOCK_LOG_BYTES // 8, dtype=torch.int64, device="cuda")
    ca.chunk_attn_measure_set_clock_log(buf)
    try:
        got = run_gpu(case, q, k, v, do)
        torch.cuda.synchronize()
    finally:
        ca.chunk_attn_measure_set_clock_log(None)
    for x, y in zip(ref, got):
        assert torch.equal(x, y)
    sums = ca.clock_log_sums(buf)
    print(sums, flush=True)
    for name in ca.CLOCK_LOG_KERNELS:
        s = sums[name]
        assert 1 <= s["workgroups"] <= 1024
        mhz = 100.0 * s["shader_clocks"] / s["ticks_100mhz"]
        assert 500.0 < mhz < 2600.0, (name, mhz)
    # switched off again: a later call leaves the buffer alone
    buf.zero_()
    run_gpu(case, q, k, v, do)
    torch.cuda.synchronize()
    assert int(buf.abs().sum()) == 0
