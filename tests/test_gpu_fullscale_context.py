"""GPU parity at the full benchmark sizes where the key/value gradients are hardest to see: the CONTEXT rows of a split
chunk (paper section 2.1: the gradient of a token's key and value comes from every later token; section 3.2.2: the
key/value gradients of a split sequence are built up over all its slices), which thousands of queries of up to eight
heads add into, and the 8-call chain over the slices of the 128K-token sequence with `accumulate_dkv`.

Three kinds of evidence:
  * the fp64 oracle on sampled context and own key rows of the 32K split chunk, one key/value head (it needs the
    log-sum-exp of every query of that head group: about half a minute on the machine's host cores);
  * closed forms that hold at any size, over ALL key rows: with K = 0 attention is uniform, P_ij = 1 / n_i with
    n_i = C + i + 1 visible keys, so with W_i = dO_i / n_i
        dV_j = sum_{h in group} sum_{i >= i_j} W_hi                       (i_j = max(0, j - C): first query seeing j)
        dK_j = scale * sum_h [ (sum_{i >= i_j} Q_hi dO_hi^T / n_i) V_j - sum_{i >= i_j} D_hi Q_hi / n_i ],  dQ = 0
    (D_hi = <dO_hi, O_hi> with the O the forward wrote); every context row shares one suffix sum, own rows have one each;
  * invariants of the true gradients: sum_j dV_j = sum dO, sum_j dK_j = 0 over the whole sequence, and the bf16
    accumulation chain against the float32 one.
"""
import numpy as np
import pytest
import torch

import synth
import paper_2509_21275_amd as ca
from gpu_util import TOL_GRAD, TOL_O, make_inputs, rel_err, run_gpu

pytestmark = pytest.mark.gpu


def _rel(got, ref):
    assert torch.isfinite(got).all()
    return ((got.double() - ref).abs().max() / ref.abs().max().clamp_min(1e-300)).item()


def uniform_attention_grads(seg, q, do, o, v, Hq, Hkv, scale, own_samples):
    """Closed-form dV (all key rows of the segment) and dK (all context rows + the sampled own rows) of one segment
    when K = 0, as float64: returns dV [kv_len, Hkv, d], dK_ctx [C, Hkv, d], {own key index: dK row [Hkv, d]}."""
    G = Hq // Hkv
    s, C = seg.q_len, seg.kv_len - seg.q_len
    d = q.shape[-1]
    n = torch.arange(C + 1, C + s + 1, device=q.device, dtype=torch.float64)
    dV = torch.empty((seg.kv_len, Hkv, d), dtype=torch.float64, device=q.device)
    dK_ctx = torch.empty((C, Hkv, d), dtype=torch.float64, device=q.device)
    dK_own = {r: torch.empty((Hkv, d), dtype=torch.float64, device=q.device) for r in own_samples}
    rows = slice(seg.q_start, seg.q_start + s)
    for g in range(Hkv):
        hs = slice(g * G, (g + 1) * G)
        Q = q[rows, hs].double(); dO = do[rows, hs].double(); O = o[rows, hs].double()          # [s, G, d]
        W = dO / n[:, None, None]
        sfx = torch.flip(torch.cumsum(torch.flip(W.sum(1), [0]), 0), [0])                       # [s, d]: sum over i' >= i
        dV[:C, g] = sfx[0]
        dV[C:, g] = sfx
        Dn = (dO * O).sum(-1) / n[:, None]                                                        # D_hi / n_i   [s, G]
        Vg = v[seg.kv_start:seg.kv_start + seg.kv_len, g].double()                                # [kv_len, d]

        def dk_rows(i0, Vrows):
            M = torch.einsum("ihc,ihe->ce", Q[i0:], W[i0:])                                       # sum Q dO^T / n
            c0 = torch.einsum("ih,ihc->c", Dn[i0:], Q[i0:])
            return scale * (Vrows @ M.T - c0)

        if C > 0:
            dK_ctx[:, g] = dk_rows(0, Vg[:C])
        for r in own_samples:
            dK_own[r][g] = dk_rows(r, Vg[C + r:C + r + 1])[0]
    return dV, dK_ctx, dK_own


def test_config2_context_rows_against_the_oracle(oracle_mod):
    """dK and dV of sampled context rows (first row, rows around multiples of 128, random ones) and own rows of the
    32K split chunk, one key/value head, element by element against the oracle; then a second run must agree bit for bit."""
    case = synth.case_by_index(2)
    q, k, v, do = make_inputs(case)
    o, lse, dq, dk, dv = run_gpu(case, q, k, v, do)
    s = case.segs[0]
    C, G = s.kv_len - s.q_len, case.num_q_heads // case.num_kv_heads
    rng = np.random.default_rng(case.seed + 99)
    g = int(rng.integers(0, case.num_kv_heads))
    print("oracle: log-sum-exp of all", s.q_len, "queries x", G, "heads of key/value head", g, flush=True)
    orc = oracle_mod.Oracle(case.segs, q.cpu(), k.cpu(), v.cpu(), do.cpu(), case.scale)
    heads = np.arange(g * G, (g + 1) * G, dtype=np.int32)
    hh = np.repeat(heads, s.q_len); rr = np.tile(np.arange(s.q_len, dtype=np.int32), G)
    O, LSE = orc.fwd_rows(hh, rr)
    D = (O * do.cpu().double().numpy()[rr, hh]).sum(-1)          # D_i = <dO_i, O_i> with the oracle's own O
    L = np.zeros((case.num_q_heads, case.total_q)); Dm = np.zeros_like(L)
    L[hh, rr] = LSE; Dm[hh, rr] = D
    ctx_rows = [0, 1, 127, 128, 129, 4095, 4096, 12287, 12288, C - 129, C - 128, C - 1] + [int(x) for x in rng.integers(0, C, 6)]
    own_rows = [C, C + 1, C + 127, C + 128, C + 4095, C + s.q_len - 65, C + s.q_len - 1] + [int(x) for x in rng.integers(C, s.kv_len, 3)]
    kv_rows = np.array(sorted(set(ctx_rows + own_rows)), dtype=np.int32)
    dK, dV = orc.dkv_rows(np.full(kv_rows.size, g, dtype=np.int32), kv_rows, L, Dm)
    kt = torch.as_tensor(kv_rows.astype(np.int64))
    is_ctx = kv_rows < C
    errs = {"dk_ctx": rel_err(dk.cpu()[kt[is_ctx], g], dK[is_ctx]), "dv_ctx": rel_err(dv.cpu()[kt[is_ctx], g], dV[is_ctx]),
            "dk_own": rel_err(dk.cpu()[kt[~is_ctx], g], dK[~is_ctx]), "dv_own": rel_err(dv.cpu()[kt[~is_ctx], g], dV[~is_ctx]),
            # the forward of the same head group, every row (the oracle computed them on the way)
            "o": rel_err(o.cpu()[rr.astype(np.int64), hh.astype(np.int64)], O),
            "lse_abs": float(np.abs(lse.cpu().double().numpy()[hh, rr] - LSE).max())}
    print(case.name, "kv head", g, int(is_ctx.sum()), "context rows,", int((~is_ctx).sum()), "own rows", errs, flush=True)
    assert max(errs["dk_ctx"], errs["dv_ctx"], errs["dk_own"], errs["dv_own"]) <= TOL_GRAD
    assert errs["o"] <= TOL_O and errs["lse_abs"] <= 2e-2
    # bit-reproducibility at full size (the same launch configuration as the benchmark)
    again = run_gpu(case, q, k, v, do)
    for x, y in zip((o, lse, dq, dk, dv), again):
        assert torch.equal(x, y)


def _config5_inputs(zero_k=False):
    c0 = synth.case_by_index(5, 0)
    ks = (c0.total_kv, c0.num_kv_heads, c0.head_dim)
    k = torch.zeros(ks, dtype=torch.bfloat16, device="cuda") if zero_k else synth.normal_bf16(c0.seed, 1, ks, "cuda")
    v = synth.normal_bf16(c0.seed, 2, ks, "cuda")
    qs, dos = [], []
    for i in range(8):
        qs.append(synth.normal_bf16(c0.seed, 10 + i, (c0.total_q, c0.num_q_heads, c0.head_dim), "cuda"))
        dos.append(synth.normal_bf16(c0.seed, 20 + i, (c0.total_q, c0.num_q_heads, c0.head_dim), "cuda"))
    return k, v, qs, dos


def _run_chain(k, v, qs, dos, f32kv):
    """Forward of slices 0..7, backward of slices 7..0 accumulating into dK/dV that start at zero (the benchmark's
    split workload; paper section 2.1 / 3.2.2).  Returns per-slice (o, lse, dq) and the accumulated dk, dv."""
    kv_dtype = torch.float32 if f32kv else torch.bfloat16
    dk = torch.zeros(k.shape, dtype=kv_dtype, device="cuda"); dv = torch.zeros_like(dk)
    outs = [None] * 8
    descs = []
    for i in range(8):
        c = synth.case_by_index(5, i)
        desc = ca.make_desc(c.segs, c.num_q_heads, c.num_kv_heads, c.head_dim, c.total_q, c.total_kv, c.scale)
        ws = ca.alloc_workspace(desc)
        o = torch.full_like(qs[i], float("nan"))
        lse = torch.full((c.num_q_heads, c.total_q), float("nan"), dtype=torch.float32, device="cuda")
        ca.chunk_attn_fwd(desc, qs[i], k, v, o, lse, ws)
        descs.append((desc, ws))
        outs[i] = [o, lse, None]
    bwd = ca.chunk_attn_bwd_f32kv if f32kv else ca.chunk_attn_bwd
    for i in range(7, -1, -1):
        desc, ws = descs[i]
        dq = torch.full_like(qs[i], float("nan"))
        bwd(desc, qs[i], k, v, outs[i][0], dos[i], outs[i][1], dq, dk, dv, 1, ws)
        outs[i][2] = dq
    torch.cuda.synchronize()
    return outs, dk, dv


def test_config5_accumulate_chain_at_full_size(oracle_mod):
    """All 8 slices of the 128K sequence, 7 -> 0, with bf16 and with float32 dK/dV buffers: sum rules over the whole
    sequence, the two chains against each other, the last 64 key rows (seen by the last slice only) and sampled
    O / LSE / dQ rows of EVERY slice against the oracle."""
    k, v, qs, dos = _config5_inputs()
    outs, dk16, dv16 = _run_chain(k, v, qs, dos, f32kv=False)
    _, dk32, dv32 = _run_chain(k, v, qs, dos, f32kv=True)
    c7 = synth.case_by_index(5, 7)
    G = c7.num_q_heads // c7.num_kv_heads
    # sum rules (rows of P sum to one; softmax is invariant to a shift of the scores), on the float32 buffers
    do_sum = sum(x.double().sum(0) for x in dos).reshape(c7.num_kv_heads, G, -1).sum(1)               # [Hkv, d]
    dv_sum = dv32.double().sum(0); dk_sum = dk32.double().sum(0)
    scale_v = dv32.abs().max().item() * c7.total_kv ** 0.5
    scale_k = dk32.abs().max().item() * c7.total_kv ** 0.5
    sum_v = ((dv_sum - do_sum).abs().max() / scale_v).item(); sum_k = (dk_sum.abs().max() / scale_k).item()
    # bf16 chain against the float32 chain: up to 8 roundings of relative size 2^-9 each (reading: one rounding per call)
    chain_k = _rel(dk16, dk32.double()); chain_v = _rel(dv16, dv32.double())
    print("chain: sum_dv", sum_v, "sum_dk", sum_k, "bf16 vs f32 dk", chain_k, "dv", chain_v, flush=True)
    assert sum_v <= 1e-2 and sum_k <= 1e-2
    assert chain_k <= 8 * 2.0 ** -8 and chain_v <= 8 * 2.0 ** -8
    # the last 64 key rows: only the last queries of the last slice see them
    rng = np.random.default_rng(c7.seed + 5)
    g = int(rng.integers(0, c7.num_kv_heads))
    orc = oracle_mod.Oracle(c7.segs, qs[7].cpu(), k.cpu(), v.cpu(), dos[7].cpu(), c7.scale)
    need = np.arange(c7.total_q - 64, c7.total_q, dtype=np.int32)
    gh = np.arange(g * G, (g + 1) * G, dtype=np.int32)
    nh = np.repeat(gh, need.size); nr = np.tile(need, gh.size)
    _, l_rows, d_rows = orc.dq_rows(nh, nr)
    L = np.zeros((c7.num_q_heads, c7.total_q)); Dm = np.zeros_like(L)
    L[nh, nr] = l_rows; Dm[nh, nr] = d_rows
    kv_rows = np.arange(c7.total_kv - 64, c7.total_kv, dtype=np.int32)
    dK, dV = orc.dkv_rows(np.full(64, g, dtype=np.int32), kv_rows, L, Dm)
    kt = torch.as_tensor(kv_rows.astype(np.int64))
    last = {"dk16": rel_err(dk16.cpu()[kt, g], dK), "dv16": rel_err(dv16.cpu()[kt, g], dV),
            "dk32": rel_err(dk32.cpu()[kt, g], dK), "dv32": rel_err(dv32.cpu()[kt, g], dV)}
    print("last 64 key rows, kv head", g, last, flush=True)
    assert max(last.values()) <= TOL_GRAD
    # sampled rows of every slice: O, LSE, dQ
    for i in range(8):
        c = synth.case_by_index(5, i)
        o, lse, dq = outs[i]
        orc = oracle_mod.Oracle(c.segs, qs[i].cpu(), k.cpu(), v.cpu(), dos[i].cpu(), c.scale)
        rows = np.array(sorted({0, 1, 31, 32, 33, 127, 128, 8191, 8192, c.total_q - 2, c.total_q - 1} |
                               {int(x) for x in rng.integers(0, c.total_q, 12)}), dtype=np.int32)
        heads = np.array(sorted({0, c.num_q_heads - 1, int(rng.integers(0, c.num_q_heads))}), dtype=np.int32)
        hh = np.repeat(heads, rows.size); rr = np.tile(rows, heads.size)
        O, LSE = orc.fwd_rows(hh, rr)
        dQ, _, _ = orc.dq_rows(hh, rr)
        rt = torch.as_tensor(rr.astype(np.int64)); ht = torch.as_tensor(hh.astype(np.int64))
        e = (rel_err(o.cpu()[rt, ht], O), float(np.abs(lse.cpu().double().numpy()[hh, rr] - LSE).max()),
             rel_err(dq.cpu()[rt, ht], dQ))
        print("slice", i, "sampled o / lse / dq", e, flush=True)
        assert e[0] <= TOL_O and e[1] <= 2e-2 and e[2] <= TOL_GRAD


def test_config5_chain_uniform_attention_closed_form():
    """The same 8-call chain with K = 0: dV of ALL 131072 key rows and dK of all rows below the last slice plus sampled
    rows of every slice against the closed form (see the module docstring), dQ = 0; and the forward of every slice (O =
    running mean of V, LSE = ln n) on all rows."""
    k, v, qs, dos = _config5_inputs(zero_k=True)
    outs, dk, dv = _run_chain(k, v, qs, dos, f32kv=False)
    c0 = synth.case_by_index(5, 0)
    Hq, Hkv, d, sl = c0.num_q_heads, c0.num_kv_heads, c0.head_dim, c0.total_q
    G = Hq // Hkv
    want_dv = torch.zeros((c0.total_kv, Hkv, d), dtype=torch.float64, device="cuda")
    want_dk = torch.zeros_like(want_dv)
    rng = np.random.default_rng(c0.seed + 7)
    own = sorted({0, 1, 31, 32, 127, 128, 129, sl - 129, sl - 128, sl - 1} | {int(x) for x in rng.integers(0, sl, 6)})
    worst_o = worst_l = 0.0
    for i in range(8):
        c = synth.case_by_index(5, i)
        seg = c.segs[0]
        o, lse, dq = outs[i]
        assert torch.count_nonzero(dq).item() == 0                       # dQ = scale * dS K = 0
        dV, dK_ctx, dK_own = uniform_attention_grads(seg, qs[i], dos[i], o, v, Hq, Hkv, c.scale, own)
        want_dv[:seg.kv_len] += dV
        C = seg.kv_len - seg.q_len
        want_dk[:C] += dK_ctx
        for r, row in dK_own.items():
            want_dk[C + r] += row
        # forward: running mean of V and ln n over all rows, in blocks of rows
        csum = torch.cumsum(v[:seg.kv_len].double(), dim=0)
        for r0 in range(0, sl, 2048):
            n = torch.arange(C + r0 + 1, C + r0 + 2049, device="cuda", dtype=torch.float64)
            ref = (csum[C + r0:C + r0 + 2048] / n[:, None, None]).repeat_interleave(G, dim=1)
            worst_o = max(worst_o, _rel(o[r0:r0 + 2048], ref))
            worst_l = max(worst_l, (lse[:, r0:r0 + 2048].double() - torch.log(n)[None, :]).abs().max().item())
    e_dv = _rel(dv, want_dv)
    # dK: rows of slices 0 .. 6 got their own-slice part only on the sampled rows; compare context-complete rows, i.e.
    # the sampled rows of every slice (all parts present)
    rows = torch.as_tensor([b * sl + r for b in range(8) for r in own], device="cuda")
    e_dk = _rel(dk[rows], want_dk[rows])
    print("uniform chain: dv all rows", e_dv, "dk sampled rows", e_dk, "o", worst_o, "lse", worst_l, flush=True)
    assert e_dv <= TOL_GRAD and e_dk <= TOL_GRAD
    assert worst_o <= 1e-2 and worst_l <= 1e-2


def test_config3_uniform_attention_gradients_all_rows():
    """Hybrid chunk with K = 0: dV of every key row, dK of every context row of the tail slice and of sampled own rows of
    every segment, in one non-accumulating call (rows outside every key range must come out zero)."""
    case = synth.case_by_index(3)
    q, _, v, do = make_inputs(case)
    k0 = torch.zeros((case.total_kv, case.num_kv_heads, case.head_dim), dtype=torch.bfloat16, device="cuda")
    o, lse, dq, dk, dv = run_gpu(case, q, k0, v, do)
    assert torch.count_nonzero(dq).item() == 0
    worst = {"dv": 0.0, "dk_ctx": 0.0, "dk_own": 0.0}
    for seg in case.segs:
        own = sorted({0, seg.q_len // 2, seg.q_len - 1, min(seg.q_len - 1, 128), min(seg.q_len - 1, 31)})
        dV, dK_ctx, dK_own = uniform_attention_grads(seg, q, do, o, v, case.num_q_heads, case.num_kv_heads, case.scale, own)
        C = seg.kv_len - seg.q_len
        worst["dv"] = max(worst["dv"], _rel(dv[seg.kv_start:seg.kv_start + seg.kv_len], dV))
        if C > 0:
            worst["dk_ctx"] = max(worst["dk_ctx"], _rel(dk[seg.kv_start:seg.kv_start + C], dK_ctx))
        got = torch.stack([dk[seg.kv_start + C + r] for r in own]); ref = torch.stack([dK_own[r] for r in own])
        worst["dk_own"] = max(worst["dk_own"], _rel(got, ref))
    print(case.name, "uniform attention gradients", worst, flush=True)
    assert max(worst.values()) <= TOL_GRAD


def test_unsplit_128k_sequence_64_heads_addresses_past_2_gib():
    """One unsplit 131072-token sequence with 64 query heads: Q and O are exactly 2 GiB each, so row offsets pass 2^31
    bytes.  K = 0 makes every output row a closed form (running mean of V, ln n): all rows and heads are checked."""
    n, Hq, Hkv, d = 131072, 64, 8, 128
    case = synth.ChunkCase("unsplit_128k", [synth.Seg(0, n, 0, n)], n, n, Hq, Hkv, d, synth.BASE_SEED + 50)
    q = synth.normal_bf16(case.seed, 0, (n, Hq, d), "cuda")
    v = synth.normal_bf16(case.seed, 2, (n, Hkv, d), "cuda")
    k0 = torch.zeros((n, Hkv, d), dtype=torch.bfloat16, device="cuda")
    assert q.numel() * 2 == 1 << 31
    print("forward of the unsplit 128K x 64-head call", flush=True)
    o, lse = run_gpu(case, q, k0, v, None, backward=False)
    G = Hq // Hkv
    csum = torch.cumsum(v.double(), dim=0)
    worst_o = worst_l = 0.0
    for r0 in range(0, n, 4096):
        nn = torch.arange(r0 + 1, r0 + 4097, device="cuda", dtype=torch.float64)
        ref = (csum[r0:r0 + 4096] / nn[:, None, None]).repeat_interleave(G, dim=1)
        worst_o = max(worst_o, _rel(o[r0:r0 + 4096], ref))
        worst_l = max(worst_l, (lse[:, r0:r0 + 4096].double() - torch.log(nn)[None, :]).abs().max().item())
    print(case.name, "uniform o", worst_o, "lse", worst_l, flush=True)
    assert worst_o <= 1e-2 and worst_l <= 1e-2
