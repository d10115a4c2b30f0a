"""GPU parity: the HIP library, called through its C ABI, against the CPU fp64 oracle, element by element.

Tolerances (max-abs error relative to the tensor's max magnitude): 2e-2 for O, 5e-2 for dQ, dK, dV.
"""
import numpy as np
import pytest
import torch

import synth
import paper_2509_21275_amd as ca
from gpu_util import TOL_GRAD, TOL_O, make_inputs, rel_err, run_gpu

pytestmark = pytest.mark.gpu


def full_compare(oracle_mod, case, scale=None):
    q, k, v, do = make_inputs(case)
    o, lse, dq, dk, dv = run_gpu(case, q, k, v, do, scale=scale)
    orc = oracle_mod.Oracle(case.segs, q.cpu(), k.cpu(), v.cpu(), do.cpu(), scale if scale is not None else case.scale)
    O, LSE = orc.forward()
    dQ, dK, dV = orc.backward()
    errs = {"o": rel_err(o, O), "dq": rel_err(dq, dQ), "dk": rel_err(dk, dK), "dv": rel_err(dv, dV),
            "lse_abs": float(np.abs(lse.double().cpu().numpy() - LSE).max())}
    print(case.name, errs, flush=True)
    assert errs["o"] <= TOL_O and errs["lse_abs"] <= 2e-2
    assert errs["dq"] <= TOL_GRAD and errs["dk"] <= TOL_GRAD and errs["dv"] <= TOL_GRAD
    return errs


def test_config1_packed_full(oracle_mod):
    full_compare(oracle_mod, synth.case_by_index(1))


@pytest.mark.parametrize("idx", [2, 3, 4, 5])
def test_scaled_replicas_full(oracle_mod, idx):
    full_compare(oracle_mod, synth.scaled_case(idx, 16))      # 5: the last slice of the long split sequence


EDGE = [
    # name, segs, Hq, Hkv, d
    ("one_token", [(0, 1, 0, 1)], 4, 4, 64),
    ("one_query_long_context", [(0, 1, 0, 700)], 8, 2, 128),
    ("ragged_single", [(0, 77, 0, 77)], 4, 1, 128),
    ("ragged_tail_slice", [(0, 130, 0, 1000)], 8, 2, 128),
    ("context_not_tile_aligned", [(0, 200, 0, 200 + 333)], 8, 8, 64),
    ("many_tiny", [(i, 1, 3 * i, 1) for i in range(40)], 4, 2, 64),
    ("hybrid_with_gaps", [(0, 150, 5, 400), (150, 70, 420, 70), (220, 1, 500, 1), (221, 300, 512, 300)], 8, 2, 128),
    ("mha_g1_d128", [(0, 300, 0, 300), (300, 260, 300, 260)], 3, 3, 128),
    ("gqa2", [(0, 129, 0, 257)], 4, 2, 128),
    ("gqa8", [(0, 96, 0, 640), (96, 160, 640, 160)], 16, 2, 128),
    ("gqa3_odd_group", [(0, 65, 0, 193)], 6, 2, 64),
    # walks of one, two and three pipeline stages (the pipelined kernels run their prologue / epilogue steps only)
    ("d128_tiny_walks", [(0, 32, 0, 32), (32, 33, 32, 33), (65, 64, 65, 64), (129, 1, 129, 129), (130, 95, 258, 95)], 2, 2, 128),
    # several segments with a context each, key ranges of 127 / 128 / 129 rows around a workgroup's 128 keys
    ("d128_many_contexts", [(0, 40, 0, 127), (40, 40, 127, 128), (80, 40, 255, 129), (120, 200, 384, 513)], 8, 2, 128),
    # 64 key/value heads: four key blocks of a head run side by side, so the 12 + 2 key blocks of the long sequence go
    # through every branch of the host's ordering (context blocks upwards, groups walking down with partners walking up,
    # the leftover split in two, the shortest quarter last), next to a sequence with a single block
    ("d128_two_way_walks", [(0, 1500, 0, 1500 + 200), (1500, 90, 1700, 90)], 64, 64, 128),
    # 65 key blocks of context per key/value head: the equal walks of a queue start in three groups, one after the other
    ("d128_context_in_groups", [(0, 200, 0, 200 + 65 * 128)], 8, 8, 128),
    # head_dim 256 (a variant of the path: other head dimensions)
    ("d256_one_token", [(0, 1, 0, 1)], 2, 2, 256),
    ("d256_ragged_tail_slice", [(0, 130, 0, 1000)], 8, 2, 256),
    ("d256_hybrid_with_gaps", [(0, 150, 5, 400), (150, 70, 420, 70), (220, 1, 500, 1), (221, 300, 512, 300)], 8, 2, 256),
    ("d256_mha_packed", [(0, 300, 0, 300), (300, 260, 300, 260), (560, 33, 560, 33)], 3, 3, 256),
    ("d256_many_contexts", [(0, 40, 0, 63), (40, 40, 63, 64), (80, 40, 127, 65), (120, 200, 192, 513)], 8, 1, 256),
    # head_dim 96
    ("d96_one_token", [(0, 1, 0, 1)], 2, 2, 96),
    ("d96_ragged_tail_slice", [(0, 130, 0, 1000)], 8, 2, 96),
    ("d96_hybrid_with_gaps", [(0, 150, 5, 400), (150, 70, 420, 70), (220, 1, 500, 1), (221, 300, 512, 300)], 8, 2, 96),
    ("d96_mha_packed", [(0, 300, 0, 300), (300, 260, 300, 260), (560, 33, 560, 33)], 3, 3, 96),
]


@pytest.mark.parametrize("name,segs,Hq,Hkv,d", EDGE, ids=[e[0] for e in EDGE])
def test_edge_cases(oracle_mod, name, segs, Hq, Hkv, d):
    tq = max(s[0] + s[1] for s in segs)
    tkv = max(s[2] + s[3] for s in segs) + 3          # trailing key rows that no segment covers
    case = synth.ChunkCase(name, [synth.Seg(*s) for s in segs], tq, tkv, Hq, Hkv, d, 4242 + len(name))
    q, k, v, do = make_inputs(case)
    o, lse, dq, dk, dv = run_gpu(case, q, k, v, do)
    orc = oracle_mod.Oracle(case.segs, q.cpu(), k.cpu(), v.cpu(), do.cpu(), case.scale)
    O, LSE = orc.forward(); dQ, dK, dV = orc.backward()
    errs = (rel_err(o, O), rel_err(dq, dQ), rel_err(dk, dK), rel_err(dv, dV))
    print(name, errs, flush=True)
    assert errs[0] <= TOL_O and max(errs[1:]) <= TOL_GRAD
    # rows outside every key range get exactly zero
    cov = np.zeros(tkv, dtype=bool)
    for s in segs:
        cov[s[2]:s[2] + s[3]] = True
    assert torch.all(dk.cpu()[~cov] == 0) and torch.all(dv.cpu()[~cov] == 0)


def test_nonstandard_scale(oracle_mod):
    case = synth.ChunkCase("scale", synth.hybrid_chunk(100, 300, [50, 90]), 240, 540, 8, 2, 128, 99)
    full_compare(oracle_mod, case, scale=0.05)


def _forward_only(oracle_mod, case, q, k, v):
    o, lse = run_gpu(case, q, k, v, backward=False)
    orc = oracle_mod.Oracle(case.segs, q.cpu(), k.cpu(), v.cpu(), None, case.scale)
    O, LSE = orc.forward()
    return rel_err(o, O), float(np.abs(lse.double().cpu().numpy() - LSE).max())


def test_forward_second_pass_forced(oracle_mod):
    """The head_dim-128 forward keeps one reference maximum per row and hands rows whose scores outgrow it to a
    second, rescaling pass.  With the growth limit set below any score every item takes the second pass."""
    case = synth.ChunkCase("redo_forced", synth.hybrid_chunk(200, 500, [130, 70]), 400, 900, 8, 2, 128, 31)
    q, k, v, _ = make_inputs(case)
    ca.chunk_attn_test_set_fwd_rescale_limit(-1e30)
    try:
        eo, el = _forward_only(oracle_mod, case, q, k, v)
    finally:
        ca.chunk_attn_test_set_fwd_rescale_limit(60.0)
    print("forced second pass", eo, el, flush=True)
    assert eo <= TOL_O and el <= 2e-2


def test_forward_scores_outgrow_first_tile(oracle_mod):
    """Scores that grow by hundreds of nats along the keys: the first tile's maximum is useless as a reference
    for the later ones (exp2 would overflow), so the second pass must take over, on its own."""
    n, Hq, Hkv, d = 700, 8, 2, 128
    case = synth.ChunkCase("growing_scores", [synth.Seg(0, n, 0, n)], n, n, Hq, Hkv, d, 32)
    q, k, v, _ = make_inputs(case)
    ramp = torch.linspace(0.0, 3.0, n, device=q.device).view(n, 1, 1)
    q = (torch.ones_like(q) * 4.0).to(torch.bfloat16)                       # q . k_j = 4 * 128 * ramp_j * scale
    k = (k.float() * 0.05 + ramp).to(torch.bfloat16)                        # up to ~136 nats at the last key
    eo, el = _forward_only(oracle_mod, case, q, k, v)
    print("growing scores", eo, el, flush=True)
    assert eo <= TOL_O and el <= 5e-2
