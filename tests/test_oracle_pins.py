"""Pins for the CPU oracle: it is checked against things other than itself.

  * a dense brute force (explicit boolean mask, whole-matrix softmax) in numpy,
  * central finite differences of L = sum(O * dO),
  * torch's scaled_dot_product_attention + autograd in float64 (library routine) on the
    special cases that reduce to textbook causal attention,
  * closed forms (first row, K = 0 running mean, gradient sum rules),
  * the two invariants the chunk definition implies (section 3.1 of the paper): a packed
    chunk equals its sequences attended one by one, and the slices of a split sequence,
    each with the keys/values of the slices before it, reproduce the unsplit sequence,
  * the pair count behind the quadratic cost term of the paper's Eq. (1) (T_comp).
"""
import json
import math
import os

import numpy as np
import pytest
import torch

import synth

RNG = np.random.default_rng(20250921)


def visible(segs, qrow, kvrow):
    """Mask predicate written independently of the oracle: may query row see key row?"""
    for (qs, ql, ks, kl) in segs:
        if qs <= qrow < qs + ql:
            if not (ks <= kvrow < ks + kl):
                return False
            pos_q = (kl - ql) + (qrow - qs)      # absolute position of the query in its sequence
            pos_k = kvrow - ks
            return pos_k <= pos_q
    return False


def dense_reference(segs, q, k, v, scale, d_o=None):
    """softmax(Q K^T scale + mask) V per head with whole matrices; gradients by the matrix calculus."""
    Tq, Hq, d = q.shape
    Tkv, Hkv, _ = k.shape
    G = Hq // Hkv
    mask = np.array([[visible(segs, i, j) for j in range(Tkv)] for i in range(Tq)])
    O = np.zeros_like(q); LSE = np.full((Hq, Tq), np.nan)
    dQ = np.zeros_like(q); dK = np.zeros_like(k); dV = np.zeros_like(v)
    rows = mask.any(axis=1)
    for h in range(Hq):
        g = h // G
        S = (q[:, h] @ k[:, g].T) * scale
        S = np.where(mask, S, -np.inf)
        m = np.max(S[rows], axis=1, keepdims=True)
        E = np.exp(S[rows] - m)
        Z = E.sum(axis=1, keepdims=True)
        P = np.zeros((Tq, Tkv)); P[rows] = E / Z
        O[:, h] = P @ v[:, g]
        LSE[h, rows] = (m + np.log(Z))[:, 0]
        if d_o is not None:
            dP = d_o[:, h] @ v[:, g].T
            D = (d_o[:, h] * O[:, h]).sum(axis=1, keepdims=True)
            dS = P * (dP - D)
            dQ[:, h] = scale * dS @ k[:, g]
            dK[:, g] += scale * dS.T @ q[:, h]
            dV[:, g] += P.T @ d_o[:, h]
    return O, LSE, dQ, dK, dV


def random_problem(segs, Hq, Hkv, d, tq=None, tkv=None):
    tq = tq or max(s[0] + s[1] for s in segs)
    tkv = tkv or max(s[2] + s[3] for s in segs)
    q = RNG.standard_normal((tq, Hq, d)); k = RNG.standard_normal((tkv, Hkv, d))
    v = RNG.standard_normal((tkv, Hkv, d)); do = RNG.standard_normal((tq, Hq, d))
    return q, k, v, do


TINY_CASES = [
    # (segments, Hq, Hkv, d)
    ([(0, 7, 0, 7)], 1, 1, 4),
    ([(0, 1, 0, 1)], 1, 1, 4),
    ([(0, 1, 0, 33)], 4, 2, 8),                                   # one query, long context
    ([(0, 5, 0, 29)], 4, 1, 8),                                   # C >> s
    ([(0, 6, 0, 6), (6, 1, 6, 1), (7, 9, 7, 9)], 4, 2, 4),        # packed, includes s = 1
    ([(0, 8, 0, 20), (8, 5, 20, 5), (13, 3, 25, 3)], 4, 2, 8),    # hybrid: tail slice + shorts
    ([(0, 4, 3, 10), (4, 6, 20, 6)], 2, 2, 4),                    # kv ranges with gaps
]


@pytest.mark.parametrize("segs,Hq,Hkv,d", TINY_CASES)
def test_brute_force_forward_and_backward(oracle_mod, segs, Hq, Hkv, d):
    q, k, v, do = random_problem(segs, Hq, Hkv, d, tkv=max(s[2] + s[3] for s in segs) + 2)
    scale = 1.0 / math.sqrt(d)
    orc = oracle_mod.Oracle(segs, q, k, v, do, scale)
    O, LSE = orc.forward()
    dQ, dK, dV = orc.backward()
    rO, rL, rdQ, rdK, rdV = dense_reference(segs, q, k, v, scale, do)
    cov = orc.covered_rows()
    np.testing.assert_allclose(O, rO, rtol=0, atol=1e-12)
    np.testing.assert_allclose(LSE[:, cov], rL[:, cov], rtol=0, atol=1e-12)
    np.testing.assert_allclose(dQ, rdQ, rtol=0, atol=1e-12)
    np.testing.assert_allclose(dK, rdK, rtol=0, atol=1e-12)
    np.testing.assert_allclose(dV, rdV, rtol=0, atol=1e-12)
    # the trailing key rows belong to no segment: nobody sees them
    assert np.all(dK[-2:] == 0) and np.all(dV[-2:] == 0)


@pytest.mark.parametrize("segs,Hq,Hkv,d", TINY_CASES[3:6])
def test_finite_differences(oracle_mod, segs, Hq, Hkv, d):
    q, k, v, do = random_problem(segs, Hq, Hkv, d)
    scale = 0.37  # not 1/sqrt(d): a dropped or doubled scale factor must show
    dQ, dK, dV = oracle_mod.Oracle(segs, q, k, v, do, scale).backward()

    def loss(q_, k_, v_):
        O, _, *_ = dense_reference(segs, q_, k_, v_, scale)   # forward of the brute force, not the oracle
        return float((O * do).sum())

    def loss_oracle(q_, k_, v_):
        O, _ = oracle_mod.Oracle(segs, q_, k_, v_, None, scale).forward()
        return float((O * do).sum())

    eps = 1e-5
    for name, x, g in (("q", q, dQ), ("k", k, dK), ("v", v, dV)):
        idxs = [tuple(RNG.integers(0, n) for n in x.shape) for _ in range(25)]
        for idx in idxs:
            for lf in (loss, loss_oracle):
                xp = x.copy(); xm = x.copy()
                xp[idx] += eps; xm[idx] -= eps
                args_p = {"q": (xp, k, v), "k": (q, xp, v), "v": (q, k, xp)}[name]
                args_m = {"q": (xm, k, v), "k": (q, xm, v), "v": (q, k, xm)}[name]
                fd = (lf(*args_p) - lf(*args_m)) / (2 * eps)
                assert abs(fd - g[idx]) <= 1e-6 * max(1.0, abs(fd)), (name, idx, fd, g[idx])


def test_textbook_causal_attention_via_torch_autograd(oracle_mod):
    """One segment with C = 0 is ordinary causal self-attention; Hq = Hkv is plain multi-head."""
    n, H, d = 19, 3, 8
    segs = [(0, n, 0, n)]
    q, k, v, do = random_problem(segs, H, H, d)
    tq, tk, tv = (torch.tensor(x.transpose(1, 0, 2), dtype=torch.float64, requires_grad=True) for x in (q, k, v))
    out = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)     # [H, n, d]
    (out * torch.tensor(do.transpose(1, 0, 2))).sum().backward()
    orc = oracle_mod.Oracle(segs, q, k, v, do)             # default scale 1/sqrt(d), as torch's
    O, _ = orc.forward(); dQ, dK, dV = orc.backward()
    np.testing.assert_allclose(O, out.detach().numpy().transpose(1, 0, 2), atol=1e-12)
    np.testing.assert_allclose(dQ, tq.grad.numpy().transpose(1, 0, 2), atol=1e-12)
    np.testing.assert_allclose(dK, tk.grad.numpy().transpose(1, 0, 2), atol=1e-12)
    np.testing.assert_allclose(dV, tv.grad.numpy().transpose(1, 0, 2), atol=1e-12)


def test_gqa_and_prefix_via_torch_autograd(oracle_mod):
    """A slice with context C and grouped heads against a dense masked softmax built from torch ops."""
    s, C, Hq, Hkv, d = 6, 11, 4, 2, 8
    segs = [(0, s, 0, C + s)]
    q, k, v, do = random_problem(segs, Hq, Hkv, d)
    tq, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, k, v))
    kk = tk.repeat_interleave(Hq // Hkv, dim=1); vv = tv.repeat_interleave(Hq // Hkv, dim=1)
    sc = torch.einsum("ihc,jhc->hij", tq, kk) / math.sqrt(d)
    i = torch.arange(s)[:, None]; j = torch.arange(C + s)[None, :]
    sc = sc.masked_fill(~(j <= C + i), float("-inf"))
    out = torch.einsum("hij,jhc->ihc", torch.softmax(sc, dim=-1), vv)
    (out * torch.tensor(do)).sum().backward()
    orc = oracle_mod.Oracle(segs, q, k, v, do)
    O, LSE = orc.forward(); dQ, dK, dV = orc.backward()
    np.testing.assert_allclose(O, out.detach().numpy(), atol=1e-12)
    np.testing.assert_allclose(LSE, torch.logsumexp(sc, dim=-1).detach().numpy(), atol=1e-12)
    np.testing.assert_allclose(dQ, tq.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dK, tk.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dV, tv.grad.numpy(), atol=1e-12)


def test_single_query_is_unmasked_attention(oracle_mod):
    C, d = 40, 8
    segs = [(0, 1, 0, C + 1)]
    q, k, v, do = random_problem(segs, 2, 1, d)
    O, LSE = oracle_mod.Oracle(segs, q, k, v).forward()
    for h in range(2):
        sc = (k[:, 0] @ q[0, h]) / math.sqrt(d)
        p = np.exp(sc - sc.max()); p /= p.sum()
        np.testing.assert_allclose(O[0, h], p @ v[:, 0], atol=1e-13)
        np.testing.assert_allclose(LSE[h, 0], np.log(np.exp(sc).sum()), atol=1e-13)


def test_packing_invariant(oracle_mod):
    """Packed chunk == each sequence on its own (outputs and all gradients), section 3.1 / 2.2."""
    lens = [5, 12, 1, 7]
    segs = synth.packed_chunk(lens)
    q, k, v, do = random_problem(segs, 4, 2, 8)
    O, LSE = oracle_mod.Oracle(segs, q, k, v, do).forward()
    dQ, dK, dV = oracle_mod.Oracle(segs, q, k, v, do).backward()
    for (qs, ql, ks, kl) in segs:
        one = oracle_mod.Oracle([(0, ql, 0, kl)], q[qs:qs + ql], k[ks:ks + kl], v[ks:ks + kl], do[qs:qs + ql])
        o1, l1 = one.forward(); dq1, dk1, dv1 = one.backward()
        assert np.array_equal(O[qs:qs + ql], o1) and np.array_equal(LSE[:, qs:qs + ql], l1)
        assert np.array_equal(dQ[qs:qs + ql], dq1)
        assert np.array_equal(dK[ks:ks + kl], dk1) and np.array_equal(dV[ks:ks + kl], dv1)


@pytest.mark.parametrize("slices", [[8, 8, 8, 8], [14, 9, 6, 3], [1, 30, 1]])
def test_splitting_invariant(oracle_mod, slices):
    """Slices with prefix KV reproduce the unsplit sequence; dK/dV contributions add up (section 2.1, 3.2.2)."""
    n = sum(slices)
    q, k, v, do = random_problem([(0, n, 0, n)], 4, 2, 8)
    whole = oracle_mod.Oracle([(0, n, 0, n)], q, k, v, do)
    O, LSE = whole.forward(); dQ, dK, dV = whole.backward()
    dK_acc = np.zeros_like(dK); dV_acc = np.zeros_like(dV)
    start = 0
    for s in slices:
        part = oracle_mod.Oracle([(0, s, 0, start + s)], q[start:start + s], k, v, do[start:start + s])
        o, l = part.forward(); dq, dk, dv = part.backward()
        np.testing.assert_allclose(o, O[start:start + s], atol=1e-13)
        np.testing.assert_allclose(l, LSE[:, start:start + s], atol=1e-13)
        np.testing.assert_allclose(dq, dQ[start:start + s], atol=1e-13)
        assert np.all(dk[start + s:] == 0) and np.all(dv[start + s:] == 0)   # later keys are invisible
        dK_acc += dk; dV_acc += dv
        start += s
    np.testing.assert_allclose(dK_acc, dK, atol=1e-12)
    np.testing.assert_allclose(dV_acc, dV, atol=1e-12)


def test_hybrid_is_split_plus_packed(oracle_mod):
    segs = synth.hybrid_chunk(6, 10, [4, 9])
    q, k, v, do = random_problem(segs, 2, 2, 4)
    O, _ = oracle_mod.Oracle(segs, q, k, v, do).forward()
    dQ, dK, dV = oracle_mod.Oracle(segs, q, k, v, do).backward()
    for (qs, ql, ks, kl) in segs:
        one = oracle_mod.Oracle([(0, ql, 0, kl)], q[qs:qs + ql], k[ks:ks + kl], v[ks:ks + kl], do[qs:qs + ql])
        o1, _ = one.forward(); dq1, dk1, dv1 = one.backward()
        assert np.array_equal(O[qs:qs + ql], o1) and np.array_equal(dQ[qs:qs + ql], dq1)
        assert np.array_equal(dK[ks:ks + kl], dk1) and np.array_equal(dV[ks:ks + kl], dv1)


def test_closed_forms(oracle_mod):
    segs = synth.hybrid_chunk(7, 13, [5, 1, 8])
    Hq, Hkv, d = 4, 2, 8
    q, k, v, do = random_problem(segs, Hq, Hkv, d)
    G = Hq // Hkv
    orc = oracle_mod.Oracle(segs, q, k, v, do)
    O, LSE = orc.forward(); dQ, dK, dV = orc.backward()
    for (qs, ql, ks, kl) in segs:
        if kl == ql:   # first row of a whole sequence sees one key: O = V, LSE = its score, dQ = 0
            for h in range(Hq):
                np.testing.assert_allclose(O[qs, h], v[ks, h // G], atol=1e-14)
                np.testing.assert_allclose(LSE[h, qs], (q[qs, h] @ k[ks, h // G]) / math.sqrt(d), atol=1e-13)
                np.testing.assert_allclose(dQ[qs, h], 0, atol=1e-14)
        # softmax shift invariance: sum_j dS_ij = 0  =>  sum over keys of ... per segment and kv head:
        #   sum_j dV_j = sum_{h in g} sum_i dO_i (rows of P sum to one)
        for g in range(Hkv):
            np.testing.assert_allclose(dV[ks:ks + kl, g].sum(0), do[qs:qs + ql, g * G:(g + 1) * G].sum((0, 1)),
                                       atol=1e-12)
    # K = 0: uniform attention -> O_i is the running mean of V, LSE_i = ln n_i, and dK = sum_i dS_ij Q_i with
    # sum_j dS_ij = 0 still; dQ = 0 because K = 0.
    k0 = np.zeros_like(k)
    orc0 = oracle_mod.Oracle(segs, q, k0, v, do)
    O0, L0 = orc0.forward(); dQ0, dK0, _ = orc0.backward()
    for (qs, ql, ks, kl) in segs:
        C = kl - ql
        for g in range(Hkv):
            csum = np.cumsum(v[ks:ks + kl, g], axis=0)
            for i in range(ql):
                n_i = C + i + 1
                for h in range(g * G, (g + 1) * G):
                    np.testing.assert_allclose(O0[qs + i, h], csum[n_i - 1] / n_i, atol=1e-13)
                    np.testing.assert_allclose(L0[h, qs + i], math.log(n_i), atol=1e-13)
    np.testing.assert_allclose(dQ0, 0, atol=1e-14)


def test_dk_sum_rule_with_shared_query(oracle_mod):
    """If every query of a head is the same vector u, dK_j = scale * u * sum_i dS_ij and sum_j dK_j = 0."""
    n, d = 12, 4
    segs = [(0, n, 0, n + 5)]
    q, k, v, do = random_problem(segs, 1, 1, d)
    q[:] = q[0]
    _, dK, _ = oracle_mod.Oracle(segs, q, k, v, do).backward()
    np.testing.assert_allclose(dK.sum(axis=0), 0, atol=1e-12)
    assert np.abs(dK).max() > 1e-3


def test_bf16_inputs_equal_widened_inputs(oracle_mod):
    c = synth.ChunkCase("t", synth.hybrid_chunk(9, 17, [6, 3]), 18, 35, 4, 2, 8, 77)
    q = synth.normal_bf16(c.seed, 0, (c.total_q, 4, 8)); k = synth.normal_bf16(c.seed, 1, (c.total_kv, 2, 8))
    v = synth.normal_bf16(c.seed, 2, (c.total_kv, 2, 8)); do = synth.normal_bf16(c.seed, 3, (c.total_q, 4, 8))
    a = oracle_mod.Oracle(c.segs, q, k, v, do)
    b = oracle_mod.Oracle(c.segs, *(synth.to_f64(x) for x in (q, k, v, do)))
    for x, y in zip(a.forward() + a.backward(), b.forward() + b.backward()):
        assert np.array_equal(x, y)


def test_pair_counts_match_closed_form_and_golden(oracle_mod):
    """Pairs visited = sum_t (s C + s (s + 1) / 2); twice that is (C+s)^2 - C^2 + s, the paper's quadratic term."""
    golden = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "pair_counts.json")))
    for idx in range(1, 6):
        for sl in (range(8) if idx == 5 else [None]):
            c = synth.case_by_index(idx, sl)
            dummy = np.zeros((c.total_q, 1, 1)); dk = np.zeros((c.total_kv, 1, 1))
            n = oracle_mod.Oracle(c.segs, dummy, dk, dk).pair_count()
            closed = sum(s.q_len * (s.kv_len - s.q_len) + s.q_len * (s.q_len + 1) // 2 for s in c.segs)
            quad = sum((s.kv_len) ** 2 - (s.kv_len - s.q_len) ** 2 + s.q_len for s in c.segs)
            assert n == closed == c.pairs and 2 * n == quad
            key = c.name
            assert golden[key] == n
    # values printed in the workload description: 4 x {256,512,128,128} and the split slices
    assert golden["packed_1k"] == 180736
    assert golden["split_32k_last_of_4"] == 234885120
    assert golden["split_128k_slice0_of_8"] == 134225920
    assert golden["split_128k_slice7_of_8"] - golden["split_128k_slice6_of_8"] == 268435456


def test_rows_outside_segments_rejected(oracle_mod):
    segs = [(2, 3, 0, 3)]
    q, k, v, do = random_problem(segs, 1, 1, 4, tq=6)
    with pytest.raises(ValueError):
        oracle_mod.Oracle(segs, q, k, v).fwd_rows([0], [0])
