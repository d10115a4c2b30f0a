"""Host-side sequence processor (paper section 3.3, Algorithm 1; cost model section 3.2.1).

First the Python oracle is pinned to what the paper and the mathematics fix (closed forms of the cost model, the worked
mesh example of section 3.3, exhaustive enumeration of tiny meshes, the structural guarantees of the algorithm); then the
C++ planner of the library is compared with the oracle, bit for bit, on seeded random batches.  Cost models with
integer coefficients keep every time an exactly representable integer, so that equal times compare equal on both sides.
"""
import itertools
import random

import pytest

from oracle import chunk_plan_oracle as orc


# ------------------------------------------------------------------ oracle pins
def test_time_closed_forms():
    m = orc.Model(alpha1=3.0, alpha2=5.0, beta1=7.0, a2a_per_token=2.0, a2a_const=11.0, n_devices=1, dp=1)
    # one sequence, no context: alpha1 s^2 + alpha2 s + beta1 + a2a (Eq. 1 with C = 0, Eq. 3)
    assert orc.t_tot(m, 0, [10]) == 3 * 100 + 5 * 10 + 7 + 2 * 10 + 11
    # a slice behind a context pays the rectangle plus its own triangle: (C + s)^2 - C^2 = 2 C s + s^2
    assert orc.t_tot(m, 6, [4]) == 3 * (2 * 6 * 4 + 16) + 5 * 4 + 7 + 2 * 4 + 11
    # packed short sequences do not see the context nor each other
    assert orc.t_tot(m, 6, [4, 3, 2]) == orc.t_tot(m, 6, [4]) + 3 * (9 + 4) + 5 * 5 + 2 * 5
    # N devices divide the computation, d_p the constant (Eq. 1)
    m2 = orc.Model(alpha1=4.0, alpha2=8.0, beta1=12.0, n_devices=4, dp=3)
    assert orc.t_tot(m2, 0, [2]) == (4 * 4 + 8 * 2) / 4 + 12 / 3


def test_split_slices_add_up_to_the_whole_sequence():
    # sum over consecutive slices of ((C + s)^2 - C^2) telescopes to L^2: splitting changes no computation (section 3.1)
    m = orc.Model(alpha1=1.0, alpha2=0.0, beta1=0.0)
    cuts = [0, 5, 12, 13, 40]
    total = sum(orc.t_tot(m, a, [b - a]) for a, b in zip(cuts, cuts[1:]))
    assert total == orc.t_tot(m, 0, [40]) == 1600


def test_mesh_example_of_the_paper():
    # Section 3.3: with a mesh {8K, 4K, 2K}, sequences with more than 12K tokens are split into an 8K and a 4K slice
    # followed by a variable-length remainder.
    m = orc.Model(alpha1=1.0, alpha2=0.0, beta1=0.0)
    K1 = 1024
    mesh = [8 * K1, 4 * K1, 2 * K1]
    chunks, _ = orc.process(m, 10 ** 9, [13 * K1, 9 * K1, 3 * K1, 14 * K1], mesh, 1e30, 10 ** 9)
    by_seq = {}
    for C, sl, I in chunks:
        for s in sl:
            by_seq.setdefault(s[0], []).append((s[1], s[2], I))
    assert sorted(by_seq[0]) == [(0, 8 * K1, 1), (8 * K1, 4 * K1, 1), (12 * K1, K1, 0)]
    assert sorted(by_seq[1]) == [(0, 8 * K1, 1), (8 * K1, K1, 0)]
    assert sorted(by_seq[2]) == [(0, 3 * K1, 0)]                       # not sharded by the mesh: a short sequence
    assert sorted(by_seq[3]) == [(0, 8 * K1, 1), (8 * K1, 4 * K1, 1), (12 * K1, 2 * K1, 0)]  # the whole mesh: last slice is the tail


def brute_mesh_time(m, max_len, K, align):
    best = float("inf")
    n_full = (max_len - 1) // align
    for cuts in itertools.combinations(range(1, n_full + 1), K - 1):
        pos = [0] + [c * align for c in cuts] + [max_len]
        best = min(best, max(orc.t_tot(m, a, [b - a]) for a, b in zip(pos, pos[1:])))
    return best


@pytest.mark.parametrize("max_len,K,align", [(37, 3, 4), (64, 4, 8), (50, 2, 1), (45, 5, 5), (9, 4, 2)])
def test_mesh_dynamic_programme_against_enumeration(max_len, K, align):
    m = orc.Model(alpha1=2.0, alpha2=3.0, beta1=1.0)
    K_eff = max(1, min(K, max_len // align))
    assert orc.balanced_mesh_time(m, max_len, K, align) == brute_mesh_time(m, max_len, K_eff, align)


def check_structure(chunks, lengths, mesh, T_t, T_m, m):
    covered = {i: [] for i in range(len(lengths))}
    for C, sl, I in chunks:
        assert len(sl) >= 1
        if I:
            assert len(sl) == 1 and sl[0][2] in mesh          # a split chunk is one mesh slice
        assert C == sl[0][1]                                  # context = tokens of that sequence before the first slice
        for k, s in enumerate(sl):
            covered[s[0]].append((s[1], s[2]))
            if k > 0:
                assert s[1] == 0                              # only the first slice may have a context: no two tail slices
        if not I and len(sl) > 1:
            assert orc.t_tot(m, C, [s[2] for s in sl]) <= T_t
            assert sum(s[2] for s in sl) <= T_m
    for i, n in enumerate(lengths):                           # every token exactly once, in order
        pos = 0
        for start, ln in sorted(covered[i]):
            assert start == pos and ln >= 1
            pos += ln
        assert pos == n


def random_batch(rng, n):
    # long-tailed lengths like the paper's corpora (section 1: most sequences short, a few very long)
    return [max(1, min(4096, int(rng.lognormvariate(5.5, 1.2)))) for _ in range(n)]


@pytest.mark.parametrize("seed", range(6))
def test_oracle_structure(seed):
    rng = random.Random(seed)
    lengths = random_batch(rng, 40)
    m = orc.Model(alpha1=1.0, alpha2=64.0, beta1=4096.0)
    mesh_like = sorted({max(lengths) // 2, max(lengths) // 4, max(lengths) // 8 or 1}, reverse=True)
    mesh = mesh_like + [max(1, max(lengths) - sum(mesh_like))]
    T_t0 = max(orc.t_tot(m, sum(mesh[:k]), [mesh[k]]) for k in range(len(mesh)))
    T_m = mesh[0]
    chunks, T_t = orc.process(m, 10 ** 9, lengths, mesh, T_t0, T_m)
    assert T_t >= T_t0
    check_structure(chunks, lengths, mesh, T_t, T_m, m)


# The packing loop of Algorithm 1 (section 3.3) on a batch small enough to follow with pencil and paper.  Cost model
# T = (C + s0)^2 - C^2 + sum of s^2 over the other slices (alpha1 = 1, nothing else), mesh {8, 4}, T_t = 45, T_m = 7.
#   lengths 14, 11, 9 are cut by the mesh: split chunks (0, 8), (8, 4) | (0, 8) | (0, 8) and the tail slices
#     A = (C 12, 2 tokens): 14^2 - 12^2 = 52, ratio 26;  B = (C 8, 3 tokens): 11^2 - 8^2 = 57, ratio 19;
#     C = (C 8, 1 token): 9^2 - 8^2 = 17, ratio 17;      one bucket each.
#   short sequences by decreasing time: 7 (49), 5 (25), 4 (16), 3 (9), 1 (1).
#   7: the emptiest bucket has 1 token, 1 + 7 > T_m: a new bucket D = [7] (time 49, ratio 7).
#   5: buckets by ascending ratio D 7, C 17, B 19, A 26.  D: 49 + 25 > 45.  C: 17 + 25 = 42 <= 45, 6 tokens: placed.
#      C is now [1, 5]: time 42, 6 tokens, ratio 7.
#   4: C (7; created before D): 10 tokens > 7.  D: 11 tokens.  B: 57 + 16 = 73 > 45.  A: 52 + 16 = 68 > 45.  Nothing
#      fits: T_t becomes the cheapest combined time among the buckets with room for 4 tokens, min(73, 68) = 68 (the
#      cheapest of all, C with 58, is full: taking it would never end).  Again: C, D full, B 73 > 68, A 68 <= 68:
#      placed.  A is now [2, 4]: time 68, 6 tokens, ratio 11.33.
#   3: C, D full.  A (11.33): 68 + 9 > 68.  B (19): 57 + 9 = 66 <= 68, 6 tokens: placed.  B: ratio 11.
#   1: C (7): 42 + 1 = 43 <= 68, 7 tokens: placed.  (Descending ratio order would take B: A 69 > 68, B 67 fits;
#      so would a best fit by time, B leaving 1 and C 25.)
def test_packing_loop_worked_example():
    m = orc.Model(alpha1=1.0, alpha2=0.0, beta1=0.0)
    lengths = [14, 11, 9, 7, 5, 4, 3, 1]
    # given in an order that is not the sorted one: the loop has to sort the short sequences itself
    perm = [4, 0, 7, 2, 6, 1, 3, 5]
    chunks, T_t = orc.process(m, 10 ** 9, [lengths[i] for i in perm], [8, 4], 45.0, 7)
    seq = {length: i for i, length in enumerate(lengths[j] for j in perm)}   # lengths are distinct: name sequences by length
    want = [
        (0, [(seq[14], 0, 8)], 1), (8, [(seq[14], 8, 4)], 1), (0, [(seq[11], 0, 8)], 1), (0, [(seq[9], 0, 8)], 1),
        (12, [(seq[14], 12, 2), (seq[4], 0, 4)], 0),
        (8, [(seq[11], 8, 3), (seq[3], 0, 3)], 0),
        (8, [(seq[9], 8, 1), (seq[5], 0, 5), (seq[1], 0, 1)], 0),
        (0, [(seq[7], 0, 7)], 0),
    ]
    assert T_t == 68.0
    key = lambda c: (c[1][0][0], c[1][0][1])       # chunks compared as a set: by (sequence, start) of the first slice
    assert sorted(chunks, key=key) == sorted(want, key=key)


# ------------------------------------------------------------------ C++ planner against the oracle
ca_plan = pytest.importorskip("paper_2509_21275_amd.chunk_plan")


def models():
    yield orc.Model(alpha1=1.0, alpha2=64.0, beta1=4096.0)
    yield orc.Model(alpha1=2.0, alpha2=0.0, beta1=0.0, a2a_per_token=16.0, a2a_const=1024.0)
    yield orc.Model(alpha1=4.0, alpha2=32.0, beta1=8192.0, n_devices=4, dp=2)


def to_c(m):
    return ca_plan.CostModel(m.alpha1, m.alpha2, m.beta1, m.a2a_per_token, m.a2a_const, m.n_devices, m.dp)


def test_time_matches():
    rng = random.Random(1)
    for m in models():
        for _ in range(50):
            C = rng.randrange(0, 5000)
            sl = [rng.randrange(1, 3000) for _ in range(rng.randrange(1, 6))]
            assert ca_plan.chunk_plan_time(to_c(m), C, sl) == orc.t_tot(m, C, sl)


@pytest.mark.parametrize("max_len,K,align", [(4096, 4, 64), (1000, 3, 8), (777, 5, 1), (130, 8, 64), (64, 1, 64), (5, 3, 64)])
def test_mesh_is_balanced(max_len, K, align):
    for m in models():
        mesh, T_t, T_m = ca_plan.chunk_plan_mesh(to_c(m), max_len, K, align, 10 ** 9)
        assert sum(mesh) == max_len and all(s >= 1 for s in mesh)
        assert all(s % align == 0 for s in mesh[:-1])
        assert len(mesh) == max(1, min(K, max_len // align))
        times = [orc.t_tot(m, sum(mesh[:k]), [mesh[k]]) for k in range(len(mesh))]
        assert T_t == max(times)
        assert T_m == mesh[0]
        if max_len <= 1000:  # the largest slice time is the smallest possible one (what is unique about a balanced mesh)
            assert T_t == orc.balanced_mesh_time(m, max_len, K, align)
    assert ca_plan.chunk_plan_mesh(to_c(next(models())), 4096, 4, 64, 100)[2] == 100   # capacity caps the token threshold


@pytest.mark.parametrize("seed", range(8))
def test_build_matches_oracle(seed):
    rng = random.Random(100 + seed)
    lengths = random_batch(rng, rng.choice([1, 7, 40, 120]))
    K, align = rng.choice([1, 2, 4, 6]), rng.choice([1, 16, 64])
    for m in models():
        cap = rng.choice([10 ** 9, 2048, 300])
        mesh, T_t0, T_m = ca_plan.chunk_plan_mesh(to_c(m), max(lengths), K, align, cap)
        want, want_T = orc.process(m, cap, lengths, mesh, T_t0, T_m)
        got, got_T, got_Tm = ca_plan.chunk_plan_build(to_c(m), cap, lengths, K, align)
        assert got_Tm == T_m and got_T == want_T
        assert [(c.context, c.slices, int(c.is_split)) for c in got] == [(C, sl, I) for C, sl, I in want]
        for c in got:
            assert c.time == orc.t_tot(m, c.context, [s[2] for s in c.slices])
            assert c.tokens == sum(s[2] for s in c.slices)
        check_structure(want, lengths, mesh, want_T, T_m, m)


def test_build_worked_example():
    # the planner of the library on the batch of test_packing_loop_worked_example, thresholds from its own mesh step:
    # alpha1 = 1 and a longest sequence of 14 cut into slices of 10 and 4 (10^2 = 100 >= 14^2 - 10^2 = 96; 9 and 5
    # give 115) make T_t = 100, T_m = 10.  Sequences 14 and 11 lose a 10-token slice: tails (C 10, 4 tokens; 96,
    # ratio 24) and (C 10, 1 token; 21, ratio 21).  Shorts 9, 7, 5, 4, 3, 1: 9 -> the 1-token bucket (21 + 81 > 100 but
    # the 4-token bucket has 13 tokens; nothing fits, T_t = 102 (the only bucket with room), placed there, 10 tokens,
    # full).  7: 4 + 7 > 10: new bucket [7] (49, ratio 7).  5 (ratios 7, 10.2, 24): [7] has no room, the full one
    # neither, A: 96 + 25 = 121 > 102, 9 tokens: T_t = 121, placed (ratio 13.4).  4: [7] 11 tokens, full, A 13 tokens:
    # the emptiest bucket has 7 tokens, 7 + 4 > 10: new bucket [4] (16, ratio 4).  3: [4] first: 25 <= 121, 7 tokens.
    # 1: [4, 3] (25 / 7 = 3.6): 26, 8 tokens: placed.
    m = orc.Model(alpha1=1.0, alpha2=0.0, beta1=0.0)
    lengths = [14, 11, 9, 7, 5, 4, 3, 1]
    got, got_T, got_Tm = ca_plan.chunk_plan_build(to_c(m), 10 ** 9, lengths, 2, 1)
    assert (got_T, got_Tm) == (121.0, 10)
    want = [(0, [(0, 0, 10)], 1), (0, [(1, 0, 10)], 1),
            (10, [(0, 10, 4), (4, 0, 5)], 0), (10, [(1, 10, 1), (2, 0, 9)], 0),
            (0, [(3, 0, 7)], 0), (0, [(5, 0, 4), (6, 0, 3), (7, 0, 1)], 0)]
    key = lambda c: (c[1][0][0], c[1][0][1])
    assert sorted(((c.context, c.slices, int(c.is_split)) for c in got), key=key) == sorted(want, key=key)


def test_segments_match():
    c = ca_plan.Chunk(context=300, slices=[(4, 300, 200), (7, 0, 50), (9, 0, 70)], is_split=False, tokens=320, time=0.0)
    assert ca_plan.chunk_plan_segments(c) == orc.segments(300, [200, 50, 70])
    assert orc.segments(300, [200, 50, 70]) == ([(0, 200, 0, 500), (200, 50, 500, 50), (250, 70, 550, 70)], 320, 620)


def test_bad_arguments():
    m = to_c(next(models()))
    with pytest.raises(Exception):
        ca_plan.chunk_plan_build(m, 100, [5, 0, 3], 2, 1)       # a sequence without tokens
    with pytest.raises(Exception):
        ca_plan.chunk_plan_mesh(m, 0, 2, 1, 100)
    bad = ca_plan.CostModel(0.0, 1.0, 1.0, 0.0, 0.0, 1, 1)       # alpha1 must be positive
    with pytest.raises(Exception):
        ca_plan.chunk_plan_mesh(bad, 100, 2, 1, 100)
