"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

The fp64 oracle cannot compute these chunks whole, so each test compares
  * O, LSE and dQ on sampled (head, query row) pairs, which the oracle computes one by one: first and last
    row of every segment, rows around tile boundaries, and seeded random rows;
  * dK and dV on sampled key rows near the end of segments (few queries see them, so the oracle can afford
    the log-sum-exp of every query that does);
and checks properties that hold at any size over ALL rows:
  * with K = 0 the attention is uniform: O_i is the running mean of V over the visible keys and
    LSE_i = ln(n_i), a complete test of the mask;
  * sum_j dV_j = sum_{h in group} sum_i dO_i and sum_j dK_j = 0 per segment and key/value head (rows of P sum
    to one; softmax is shift invariant).
"""
import numpy as np
import pytest
import torch

import synth
from gpu_util import TOL_GRAD, TOL_O, make_inputs, rel_err, run_gpu

pytestmark = pytest.mark.gpu


def sample_rows(case, rng, n_random=48):
    rows = set()
    for s in case.segs:
        rows.update([s.q_start, s.q_start + s.q_len - 1])
    for s in sorted(case.segs, key=lambda s: -s.q_len)[:3]:
        for m in (32, 64, 128, 256):
            for b in range(m, s.q_len, max(m, (s.q_len // 3) // m * m or m)):
                for dlt in (-1, 0, 1):
                    if 0 <= b + dlt < s.q_len:
                        rows.add(s.q_start + b + dlt)
    rows.update(int(r) for r in rng.integers(0, case.total_q, n_random))
    return np.array(sorted(rows), dtype=np.int32)


def sample_heads(case, rng):
    hs = {0, case.num_q_heads - 1}
    hs.update(int(h) for h in rng.integers(0, case.num_q_heads, 2))
    return np.array(sorted(hs), dtype=np.int32)


def check_sampled(oracle_mod, case, q, k, v, do, o, lse, dq, dk, dv, kv_rows_from_end=(1, 2, 33, 64)):
    rng = np.random.default_rng(case.seed)
    orc = oracle_mod.Oracle(case.segs, q.cpu(), k.cpu(), v.cpu(), do.cpu(), case.scale)
    rows = sample_rows(case, rng)
    heads = sample_heads(case, rng)
    hh = np.repeat(heads, rows.size); rr = np.tile(rows, heads.size)
    O, LSE = orc.fwd_rows(hh, rr)
    dQ, _, _ = orc.dq_rows(hh, rr)
    rt = torch.as_tensor(rr.astype(np.int64)); ht = torch.as_tensor(hh.astype(np.int64))
    errs = {"o": rel_err(o.cpu()[rt, ht], O), "dq": rel_err(dq.cpu()[rt, ht], dQ),
            "lse_abs": float(np.abs(lse.cpu().double().numpy()[hh, rr] - LSE).max())}
    # key rows close to the end of the longest and the shortest segment, one key/value head
    G = case.num_q_heads // case.num_kv_heads
    g = int(rng.integers(0, case.num_kv_heads))
    segs = sorted(case.segs, key=lambda s: s.q_len)
    picked = [segs[-1]] + ([segs[0]] if len(segs) > 1 else [])
    kv_rows, need = [], set()
    for s in picked:
        C = s.kv_len - s.q_len
        for back in kv_rows_from_end:
            j = s.kv_len - back
            if j < 0:
                continue
            kv_rows.append(s.kv_start + j)
            for i in range(max(0, j - C), s.q_len):          # the queries that see key j
                need.add(s.q_start + i)
    need = np.array(sorted(need), dtype=np.int32)
    gh = np.arange(g * G, (g + 1) * G, dtype=np.int32)
    nh = np.repeat(gh, need.size); nr = np.tile(need, gh.size)
    _, l_rows, d_rows = orc.dq_rows(nh, nr)
    L = np.zeros((case.num_q_heads, case.total_q)); Dm = np.zeros_like(L)
    L[nh, nr] = l_rows; Dm[nh, nr] = d_rows
    kv_rows = np.array(kv_rows, dtype=np.int32)
    dK, dV = orc.dkv_rows(np.full(kv_rows.size, g, dtype=np.int32), kv_rows, L, Dm)
    kt = torch.as_tensor(kv_rows.astype(np.int64))
    errs["dk"] = rel_err(dk.cpu()[kt, g], dK)
    errs["dv"] = rel_err(dv.cpu()[kt, g], dV)
    errs["n_pairs"] = int(hh.size); errs["n_kv_rows"] = int(kv_rows.size)
    return errs


def check_sum_rules(case, do, dk, dv):
    """sum_j dV_j = sum_{h in g} sum_i dO_i and sum_j dK_j = 0, per segment and key/value head."""
    G = case.num_q_heads // case.num_kv_heads
    worst_v = worst_k = 0.0
    for s in case.segs:
        dv_sum = dv[s.kv_start:s.kv_start + s.kv_len].double().sum(0)                       # [Hkv, d]
        do_sum = do[s.q_start:s.q_start + s.q_len].double().sum(0).reshape(case.num_kv_heads, G, -1).sum(1)
        # every stored dV_j carries one bf16 rounding of relative size 2^-9: the sums agree to ~sqrt(n) ulps
        scale_v = dv[s.kv_start:s.kv_start + s.kv_len].double().abs().max().item() * max(1.0, s.kv_len ** 0.5)
        worst_v = max(worst_v, (dv_sum - do_sum).abs().max().item() / scale_v)
        dk_sum = dk[s.kv_start:s.kv_start + s.kv_len].double().sum(0)
        scale_k = dk[s.kv_start:s.kv_start + s.kv_len].double().abs().max().item() * max(1.0, s.kv_len ** 0.5)
        worst_k = max(worst_k, dk_sum.abs().max().item() / scale_k)
    return worst_v, worst_k


def check_uniform_attention(case, q, v):
    """K = 0: O_i = mean of V over the visible keys, LSE_i = ln n_i, for every row and head."""
    k0 = torch.zeros((case.total_kv, case.num_kv_heads, case.head_dim), dtype=torch.bfloat16, device=q.device)
    o, lse = run_gpu(case, q, k0, v, None, backward=False)
    G = case.num_q_heads // case.num_kv_heads
    worst_o = worst_l = 0.0
    for s in case.segs:
        C = s.kv_len - s.q_len
        csum = torch.cumsum(v[s.kv_start:s.kv_start + s.kv_len].double(), dim=0)           # [kv_len, Hkv, d]
        n = torch.arange(C + 1, C + s.q_len + 1, device=q.device, dtype=torch.float64)
        ref = (csum[C:C + s.q_len] / n[:, None, None]).repeat_interleave(G, dim=1)           # [q_len, Hq, d]
        got = o[s.q_start:s.q_start + s.q_len].double()
        worst_o = max(worst_o, ((got - ref).abs().max() / ref.abs().max()).item())
        worst_l = max(worst_l, (lse[:, s.q_start:s.q_start + s.q_len].double() - torch.log(n)[None, :]).abs().max().item())
    return worst_o, worst_l


def full_scale(oracle_mod, case):
    q, k, v, do = make_inputs(case)
    o, lse, dq, dk, dv = run_gpu(case, q, k, v, do)
    errs = check_sampled(oracle_mod, case, q, k, v, do, o, lse, dq, dk, dv)
    sv, sk = check_sum_rules(case, do, dk, dv)
    uo, ul = check_uniform_attention(case, q, v)
    print(case.name, errs, {"sum_dv": sv, "sum_dk": sk, "uniform_o": uo, "uniform_lse": ul}, flush=True)
    assert errs["o"] <= TOL_O and errs["lse_abs"] <= 2e-2
    assert errs["dq"] <= TOL_GRAD and errs["dk"] <= TOL_GRAD and errs["dv"] <= TOL_GRAD
    assert sv <= 1e-2 and sk <= 1e-2
    assert uo <= 1e-2 and ul <= 1e-2
    # first row of a whole sequence sees one key: O = V exactly (bf16), dQ = 0 up to the rounding of dP - D
    G = case.num_q_heads // case.num_kv_heads
    for s in case.segs:
        if s.kv_len == s.q_len:
            assert torch.equal(o[s.q_start], v[s.kv_start].repeat_interleave(G, dim=0))
            assert dq[s.q_start].float().abs().max().item() <= 1e-4 * dq.float().abs().max().item()


def test_config2_split_slice(oracle_mod):
    full_scale(oracle_mod, synth.case_by_index(2))


def test_config3_hybrid(oracle_mod):
    full_scale(oracle_mod, synth.case_by_index(3))


def test_config4_packed_skewed(oracle_mod):
    full_scale(oracle_mod, synth.case_by_index(4))


@pytest.mark.parametrize("slice_index", [0, 3, 7])
def test_config5_long_split_slices(oracle_mod, slice_index):
    full_scale(oracle_mod, synth.case_by_index(5, slice_index))
