"""The one-pass backward for head_dim 128 (mode 2 of chunk_attn_test_set_bwd_mode): dK, dV and dQ from one walk over
the keys, dQ added into float32 tiles in a fixed order along chains of key blocks (paper section 2.1: the gradient of a
query sums over all keys it sees, that of a key over all queries that see it).  Against the oracle on the edge cases and
on the scaled replicas of the workloads (one, two and four sub-chains per chain), dK / dV against the two-kernel
backward (the same products, summed over the query tiles in another order: the two-kernel backward walks some key
blocks downwards), bit-reproducibility, the accumulate and float32 variants, a clean status word, and sampled rows at
full size."""
import numpy as np
import pytest
import torch

import synth
import paper_2509_21275_amd as ca

# dK / dV of the two backwards: float32 sums of the same terms in two orders, then one rounding to bf16 (2^-8 relative)
TOL_ORDER = 1e-2


def same_up_to_order(a, b):
    return rel_err(a, b.double().cpu().numpy()) <= TOL_ORDER
from gpu_util import TOL_GRAD, make_inputs, rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _restore_mode():
    yield
    ca.chunk_attn_test_set_bwd_mode(0)


def run_bwd(case, mode, q, k, v, do, accumulate=False, init=None, f32kv=False):
    ca.chunk_attn_test_set_bwd_mode(mode)
    desc = ca.make_desc(case.segs, case.num_q_heads, case.num_kv_heads, case.head_dim, case.total_q, case.total_kv,
                        case.scale)
    ws = ca.alloc_workspace(desc)
    o = torch.empty_like(q); lse = torch.empty((case.num_q_heads, case.total_q), dtype=torch.float32, device="cuda")
    ca.chunk_attn_fwd(desc, q, k, v, o, lse, ws)
    dq = torch.full_like(q, float("nan"))
    kv_dtype = torch.float32 if f32kv else torch.bfloat16
    if accumulate:
        dk = init[0].clone().to(kv_dtype); dv = init[1].clone().to(kv_dtype)
    else:
        dk = torch.full(k.shape, float("nan"), dtype=kv_dtype, device="cuda"); dv = torch.full_like(dk, float("nan"))
    (ca.chunk_attn_bwd_f32kv if f32kv else ca.chunk_attn_bwd)(desc, q, k, v, o, do, lse, dq, dk, dv, int(accumulate), ws)
    torch.cuda.synchronize()
    status = ca.chunk_attn_test_bwd_status(desc, ws) if mode == 2 else 0
    return dq, dk, dv, status


EDGE = [
    ("one_query_long_context", [(0, 1, 0, 700)], 8, 2),
    ("ragged_single", [(0, 77, 0, 77)], 4, 1),
    ("ragged_tail_slice", [(0, 130, 0, 1000)], 8, 2),
    ("hybrid_with_gaps", [(0, 150, 5, 400), (150, 70, 420, 70), (220, 1, 500, 1), (221, 300, 512, 300)], 8, 2),
    ("mha_g1", [(0, 300, 0, 300), (300, 260, 300, 260)], 3, 3),
    ("gqa8", [(0, 96, 0, 640), (96, 160, 640, 160)], 16, 2),
    ("tiny_walks", [(0, 32, 0, 32), (32, 33, 32, 33), (65, 64, 65, 64), (129, 1, 129, 129), (130, 95, 258, 95)], 2, 2),
    ("many_contexts", [(0, 40, 0, 127), (40, 40, 127, 128), (80, 40, 255, 129), (120, 200, 384, 513)], 8, 2),
    # 17 and 65 key blocks in one chain: two and four sub-chains, the last ones ragged
    ("two_sub_chains", [(0, 64, 0, 2100)], 4, 2),
    ("four_sub_chains", [(0, 50, 0, 8200), (50, 300, 8200, 300)], 4, 1),
]


@pytest.mark.parametrize("name,segs,Hq,Hkv", EDGE, ids=[e[0] for e in EDGE])
def test_edge_cases_against_oracle_and_two_kernel_backward(oracle_mod, name, segs, Hq, Hkv):
    tq = max(s[0] + s[1] for s in segs); tkv = max(s[2] + s[3] for s in segs) + 3
    case = synth.ChunkCase(name, [synth.Seg(*s) for s in segs], tq, tkv, Hq, Hkv, 128, 9100 + len(name))
    q, k, v, do = make_inputs(case)
    dq2, dk2, dv2, st = run_bwd(case, 2, q, k, v, do)
    dq1, dk1, dv1, _ = run_bwd(case, 1, q, k, v, do)
    assert st == 0
    assert same_up_to_order(dk1, dk2) and same_up_to_order(dv1, dv2)
    orc = oracle_mod.Oracle(case.segs, q.cpu(), k.cpu(), v.cpu(), do.cpu(), case.scale)
    dQ, dK, dV = orc.backward()
    errs = (rel_err(dq2, dQ), rel_err(dk2, dK), rel_err(dv2, dV))
    print(name, errs, flush=True)
    assert max(errs) <= TOL_GRAD
    again = run_bwd(case, 2, q, k, v, do)
    assert torch.equal(dq2, again[0]) and torch.equal(dk2, again[1]) and torch.equal(dv2, again[2]) and again[3] == 0


@pytest.mark.parametrize("idx", [2, 3, 4, 5])
def test_scaled_replicas(oracle_mod, idx):
    case = synth.scaled_case(idx, 16)
    q, k, v, do = make_inputs(case)
    dq, dk, dv, st = run_bwd(case, 2, q, k, v, do)
    orc = oracle_mod.Oracle(case.segs, q.cpu(), k.cpu(), v.cpu(), do.cpu(), case.scale)
    dQ, dK, dV = orc.backward()
    errs = (rel_err(dq, dQ), rel_err(dk, dK), rel_err(dv, dV))
    print(case.name, errs, "status", st, flush=True)
    assert st == 0 and max(errs) <= TOL_GRAD


def test_accumulate_and_float32_buffers():
    case = synth.scaled_case(3, 16)
    q, k, v, do = make_inputs(case)
    init = (torch.full_like(k, 0.5), torch.full_like(v, -0.25))
    for f32 in (False, True):
        a = run_bwd(case, 2, q, k, v, do, accumulate=True, init=init, f32kv=f32)
        b = run_bwd(case, 1, q, k, v, do, accumulate=True, init=init, f32kv=f32)
        assert a[3] == 0 and same_up_to_order(a[1], b[1]) and same_up_to_order(a[2], b[2])
        assert rel_err(a[0], b[0].double().cpu().numpy()) <= 2e-2   # dQ: two float32 summation orders, rounded to bf16


def test_full_size_split_slice_sampled(oracle_mod):
    """The 32K split chunk at full size: 256 key blocks per chain (four sub-chains of 64), dQ on sampled rows against the
    oracle, dK / dV equal to the two-kernel backward's up to the order of the sums, twice the same bits."""
    case = synth.case_by_index(2)
    q, k, v, do = make_inputs(case)
    dq2, dk2, dv2, st = run_bwd(case, 2, q, k, v, do)
    dq1, dk1, dv1, _ = run_bwd(case, 1, q, k, v, do)
    assert st == 0 and same_up_to_order(dk1, dk2) and same_up_to_order(dv1, dv2)
    rng = np.random.default_rng(case.seed + 3)
    rows = np.array(sorted({0, 1, 31, 32, 33, 127, 128, 4095, 4096, case.total_q - 1} | {int(x) for x in rng.integers(0, case.total_q, 20)}),
                    dtype=np.int32)
    heads = np.array([0, 13, case.num_q_heads - 1], dtype=np.int32)
    hh = np.repeat(heads, rows.size); rr = np.tile(rows, heads.size)
    orc = oracle_mod.Oracle(case.segs, q.cpu(), k.cpu(), v.cpu(), do.cpu(), case.scale)
    dQ, _, _ = orc.dq_rows(hh, rr)
    rt = torch.as_tensor(rr.astype(np.int64)); ht = torch.as_tensor(hh.astype(np.int64))
    e = rel_err(dq2.cpu()[rt, ht], dQ)
    print(case.name, "one-pass dq on", hh.size, "sampled rows", e, "max |one-pass - two-kernel| / max",
          ((dq2.float() - dq1.float()).abs().max() / dq1.float().abs().max()).item(), flush=True)
    assert e <= TOL_GRAD
    again = run_bwd(case, 2, q, k, v, do)
    assert torch.equal(dq2, again[0]) and again[3] == 0
