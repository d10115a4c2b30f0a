"""The C++ chunk scheduler (include/chunk_sched.h, through its Python binding) against the plain reference in
oracle/chunk_sched_oracle.py on seeded cases: orders and windows element by element, the checkpointing problem by
its optimal value (several configurations can reach it) plus feasibility of the returned one, the grouping by its
cost, the timeline by its numbers.  No GPU is needed."""
import os
import random
import sys

import pytest

sys.path.insert(0, os.path.join(os.path.dirname(__file__), "..", "oracle"))
import chunk_sched_oracle as o  # noqa: E402

from paper_2509_21275_amd import ChunkAttnError  # noqa: E402
from paper_2509_21275_amd import chunk_sched as cs  # noqa: E402


def models(d_p=2, d_s=2, layers=8, capacity=1e18, m_ms=None):
    kw = dict(d_p=d_p, d_s=d_s, layers=layers, m_token=34.0 * 4096 * 2 * layers, m_logits=4.0 * 128256, e=2.0,
              hidden=4096.0, kv_hidden=1024.0, capacity=capacity, m_ms=m_ms or [0.0] * d_p)
    return cs.MemModel(**kw), o.MemModel(**kw)


def random_units(rng, max_units=5, max_chunks=4):
    counts = sorted((rng.randint(1, max_chunks) for _ in range(rng.randint(1, max_units))), reverse=True)
    return counts, [u for u, c in enumerate(counts) for _ in range(c)]


def random_chunks(rng, unit_of):
    # every chunk of a sequence but its last is a split chunk
    return [(rng.choice([512, 1024, 1536, 2048, 4096]), int(k + 1 < len(unit_of) and unit_of[k + 1] == u))
            for k, u in enumerate(unit_of)]


def no_ckpt_peak(om, chunks, n_split, fb):
    n = len(chunks)
    return max(om.m_ms[p - 1] + sum(o.act_bytes(om, p, chunks[k][0], chunks[k][1], 0) for k in w)
               for p in range(1, om.d_p + 1) for w in o.windows(om.d_p, p, n, n_split, fb))


def test_act_bytes_match():
    m, om = models(d_p=4, d_s=2, layers=16)
    for p in range(1, 5):
        for split in (0, 1):
            for l in range(0, 5):
                assert cs.chunk_sched_act_bytes(m, p, 3000, split, l) == pytest.approx(o.act_bytes(om, p, 3000, split, l), rel=1e-12)
    with pytest.raises(ChunkAttnError):
        cs.chunk_sched_act_bytes(m, 5, 3000, 0, 0)
    with pytest.raises(ChunkAttnError):
        cs.chunk_sched_act_bytes(m, 1, 3000, 0, 5)


def test_f2b_and_windows_match():
    rng = random.Random(101)
    for _ in range(200):
        d_p = rng.randint(1, 6)
        counts, unit_of = random_units(rng)
        n = len(unit_of)
        fb = cs.chunk_sched_f2b(unit_of)
        assert fb == o.f2b(unit_of)
        for p in range(1, d_p + 1):
            w = min(n, d_p - p + counts[0])
            assert cs.chunk_sched_windows(d_p, p, n, counts[0], fb) == o.windows(d_p, p, n, counts[0], fb)[w - 1:]


def test_f2b_rejects_a_sequence_in_two_pieces():
    with pytest.raises(ChunkAttnError):
        cs.chunk_sched_f2b([0, 1, 0])


def test_solve_ckpt_matches_enumeration():
    rng = random.Random(103)
    solved = infeasible = 0
    for _ in range(40):
        d_p = rng.randint(1, 3)
        lay = rng.choice([1, 2, 3])
        m, om = models(d_p=d_p, d_s=rng.choice([1, 2]), layers=lay * d_p, m_ms=[rng.uniform(0, 1e8) for _ in range(d_p)])
        counts, unit_of = random_units(rng, max_units=3, max_chunks=2)
        if len(unit_of) + d_p - 1 > 6:
            continue
        chunks = random_chunks(rng, unit_of)
        fb = o.f2b(unit_of)
        cap = rng.uniform(0.35, 1.05) * no_ckpt_peak(om, chunks, counts[0], fb)
        m.capacity = om.capacity = cap
        want = o.solve_ckpt(om, chunks, unit_of, counts[0])
        got = cs.chunk_sched_solve_ckpt(m, chunks, unit_of, counts[0])
        if want is None:
            assert got is None
            infeasible += 1
            continue
        assert got is not None and got[0] == want[0] == sum(got[1])
        assert o.config_fits(om, chunks, counts[0], fb, got[1])
        assert got[2] >= 0 and got[3] == got[0]  # ran to the end: the bound is the optimum
        solved += 1
    assert solved >= 10 and infeasible >= 1


def test_solve_ckpt_mid_size_is_feasible_and_locally_minimal():
    rng = random.Random(107)
    d_p = 4
    m, om = models(d_p=d_p, d_s=2, layers=32, m_ms=[2e9, 1.5e9, 1.5e9, 2.5e9])
    counts = [5, 3, 2, 1, 1, 1, 1]
    unit_of = [u for u, c in enumerate(counts) for _ in range(c)]
    chunks = random_chunks(rng, unit_of)
    fb = o.f2b(unit_of)
    m.capacity = om.capacity = 0.6 * no_ckpt_peak(om, chunks, counts[0], fb)
    s, C, nodes, lb = cs.chunk_sched_solve_ckpt(m, chunks, unit_of, counts[0], gap=0.02)
    assert nodes != 0 and s == sum(C) and 0 < s < len(C) * 8 and 0 < lb <= s
    assert nodes < 0 or s - lb <= 0.02 * s
    assert o.config_fits(om, chunks, counts[0], fb, C)
    for j in range(len(C)):
        if C[j] > 0:
            C2 = list(C)
            C2[j] -= 1
            assert not o.config_fits(om, chunks, counts[0], fb, C2)
    # with room for everything nothing is checkpointed; with room for nothing the answer is "does not fit"
    m.capacity = 1e18
    assert cs.chunk_sched_solve_ckpt(m, chunks, unit_of, counts[0])[0] == 0
    m.capacity = 3e9
    assert cs.chunk_sched_solve_ckpt(m, chunks, unit_of, counts[0]) is None


def test_group_matches_trying_every_grouping():
    rng = random.Random(109)
    done = 0
    for _ in range(25):
        d_p = rng.randint(1, 2)
        m, om = models(d_p=d_p, d_s=1, layers=2 * d_p)
        n_units = rng.randint(1, 3)
        units = []
        for _u in range(n_units):
            c = rng.randint(1, 2)
            units.append([(rng.choice([512, 1024, 2048]), int(i + 1 < c)) for i in range(c)])
        if sum(len(u) for u in units) + d_p - 1 > 6:
            continue
        order = o.pipeline_order(units)
        chunks = [c for u in order for c in units[u]]
        unit_of = [j for j, u in enumerate(order) for _ in units[u]]
        peak = no_ckpt_peak(om, chunks, max(len(u) for u in units), o.f2b(unit_of))
        m.capacity = om.capacity = rng.uniform(0.5, 1.0) * peak
        f_hat, delta = rng.uniform(0.5, 2.0), rng.choice([0.0, 0.7, 5.0])
        want = o.group(om, units, f_hat, delta)
        got = cs.chunk_sched_group(m, units, f_hat, delta)
        if want is None:
            assert got is None
            continue
        assert got is not None and got[0] == pytest.approx(want[0], rel=1e-12)
        assert sorted(u for p in got[1] for u in p.units) == list(range(n_units))
        total = 0.0
        first = [0]
        for u in units:
            first.append(first[-1] + len(u))
        for p in got[1]:  # every pipeline's C fits its own windows and adds up to the reported cost
            sub = [units[u] for u in p.units]
            assert p.order == [first[u] + i for u in p.units for i in range(len(units[u]))]
            assert o.pipeline_order(sub) == list(range(len(sub)))
            ch = [c for u in sub for c in u]
            uo = [j for j, u in enumerate(sub) for _ in u]
            assert o.config_fits(om, ch, max(len(u) for u in sub), o.f2b(uo), p.C)
            total += delta + f_hat * sum(p.C)
        assert total == pytest.approx(got[0], rel=1e-12)
        done += 1
    assert done >= 8


def test_simulate_matches():
    rng = random.Random(113)
    for _ in range(100):
        d_p = rng.randint(1, 5)
        counts, unit_of = random_units(rng)
        n = len(unit_of)
        fb = o.f2b(unit_of)
        tf = [rng.uniform(0.5, 2.0) for _ in range(n)]
        tb = [rng.uniform(1.0, 4.0) for _ in range(n)]
        rec = [[rng.uniform(0.0, 1.0) for _ in range(n)] for _ in range(d_p)] if rng.random() < 0.7 else None
        mem = [[rng.uniform(1.0, 9.0) for _ in range(n)] for _ in range(d_p)] if rng.random() < 0.7 else None
        p2p = rng.choice([0.0, 0.05])
        want = o.simulate(d_p, counts[0], fb, tf, tb, rec, mem, p2p)
        got = cs.chunk_sched_simulate(d_p, counts[0], fb, tf, tb, rec, mem, p2p)
        assert got[0] == pytest.approx(want[0], rel=1e-12)
        assert got[1] == pytest.approx(want[1], rel=1e-12)
        assert got[2] == pytest.approx(want[2], rel=1e-12)
        assert got[3] == want[3]


def test_plan_of_the_scheduler_fits_in_the_timeline():
    # end to end: group, then run every pipeline through the timeline with the footprints its C implies
    rng = random.Random(127)
    d_p = 4
    m, om = models(d_p=d_p, d_s=2, layers=16, m_ms=[1e9] * 4)
    units = [[(4096, 1), (3072, 1), (2048, 1), (3000, 0)], [(4096, 1), (2500, 0)], [(3500, 0)], [(2800, 0)], [(3900, 0)]]
    flat = [c for u in units for c in u]
    m.capacity = om.capacity = 1e9 + 3.2 * max(o.act_bytes(om, 4, t, s, 0) for t, s in flat)
    cost, pipes = cs.chunk_sched_group(m, units, layer_fwd_time=0.01, delta=0.5)
    assert sorted(u for p in pipes for u in p.units) == list(range(len(units)))
    for p in pipes:
        ch = [flat[k] for k in p.order]
        uo = [j for j, u in enumerate(p.units) for _ in units[u]]
        fb = cs.chunk_sched_f2b(uo)
        n, ns = len(ch), max(len(units[u]) for u in p.units)
        mem = [[cs.chunk_sched_act_bytes(m, st, ch[k][0], ch[k][1], p.C[fb[k] + d_p - st]) for k in range(n)]
               for st in range(1, d_p + 1)]
        rec = [[0.01 * p.C[fb[k] + d_p - st] for k in range(n)] for st in range(1, d_p + 1)]
        ms, busy, peak, held = cs.chunk_sched_simulate(d_p, ns, fb, [1.0] * n, [2.0] * n, rec, mem)
        assert all(1e9 + pk <= m.capacity * (1 + 1e-12) for pk in peak)
        assert ms == pytest.approx((n + d_p - 1) * 3.0 + 0.01 * sum(p.C))  # recomputation is paid once per variable


def test_invalid_arguments():
    m, _ = models()
    with pytest.raises(ChunkAttnError):
        cs.chunk_sched_solve_ckpt(m, [(0, 0)], [0], 1)
    with pytest.raises(ChunkAttnError):
        cs.chunk_sched_solve_ckpt(m, [(10, 0)], [0], 2)
    with pytest.raises(ChunkAttnError):
        cs.chunk_sched_windows(2, 3, 4, 1, [0, 1, 2, 3])
    with pytest.raises(ChunkAttnError):
        cs.chunk_sched_windows(2, 1, 4, 1, [0, 1, 1, 3])
    with pytest.raises(ChunkAttnError):
        cs.chunk_sched_simulate(2, 1, [0, 0], [1.0, 1.0], [1.0, 1.0])
    bad = cs.MemModel(d_p=2, d_s=1, layers=3, m_token=1e6, m_logits=0.0, e=2.0, hidden=64.0, kv_hidden=64.0, capacity=1e9,
                      m_ms=[0.0, 0.0])
    with pytest.raises(ChunkAttnError):
        cs.chunk_sched_solve_ckpt(bad, [(10, 0)], [0], 1)


def test_plan_batch_matches_the_composed_reference():
    """The whole solve (K tuning, sequence processor, grouping, checkpointing) on batches small enough for the
    reference to try everything: same K, same estimated time, same chunks; every chunk in one pipeline."""
    import chunk_plan_oracle as po
    from paper_2509_21275_amd import chunk_plan as cp
    rng = random.Random(131)
    done = 0
    for _ in range(30):
        d_p = rng.randint(1, 2)
        m, om = models(d_p=d_p, d_s=1, layers=2 * d_p)
        pm = po.Model(alpha1=1.0, alpha2=64.0, beta1=float(rng.choice([0, 4096])))
        cm = cp.CostModel(pm.alpha1, pm.alpha2, pm.beta1, 0.0, 0.0, 1, 1)
        lengths = [rng.choice([256, 384, 512, 1024, 2048]) for _ in range(rng.randint(1, 3))]
        align, ks = 128, [1, 2]

        def mesh_of(K):
            return cp.chunk_plan_mesh(cm, max(lengths), K, align, 1 << 20)

        # keep only batches the reference can enumerate (at most 4 chunks per K)
        sizes = [len(po.process(pm, 10 ** 12, lengths, *mesh_of(K))[0]) for K in ks]
        if max(sizes) + d_p - 1 > 5:
            continue
        biggest = max(o.act_bytes(om, d_p, n, 1, 0) for n in lengths)
        m.capacity = om.capacity = rng.uniform(0.6, 2.5) * biggest
        want = o.plan_batch(po, pm, om, lengths, ks, 1.0 / 3.0, mesh_of)
        got = cs.chunk_sched_plan_batch(cm, m, 1 << 20, lengths, ks[0], ks[-1], align, 1.0 / 3.0, 0.0)
        if want is None:
            assert got is None
            continue
        assert got is not None and got.k == want[0]
        assert got.est_time == pytest.approx(want[1], rel=1e-9)
        assert [(c.context, c.slices, int(c.is_split)) for c in got.chunks] == [(ctx, sl, i) for ctx, sl, i in want[2]]
        assert all(0 <= p < len(got.C) for p in got.pipeline_of_chunk)
        for g in range(len(got.C)):  # positions inside a pipeline are a permutation, C has n + d_p - 1 entries
            pos = sorted(got.fwd_pos_of_chunk[c] for c in range(len(got.chunks)) if got.pipeline_of_chunk[c] == g)
            assert pos == list(range(len(pos))) and len(got.C[g]) == len(pos) + d_p - 1
        done += 1
    assert done >= 8


def test_plan_batch_worked_example():
    """The batch of tests/test_chunk_sched_oracle.py::test_plan_batch_worked_example, whose answer is derived by hand
    there (K = 2, estimated time 128, one pipeline), through the library."""
    from paper_2509_21275_amd import chunk_plan as cp
    m, _ = models(d_p=2, d_s=1, layers=2)
    cm = cp.CostModel(1.0, 0.0, 0.0, 0.0, 0.0, 1, 1)
    got = cs.chunk_sched_plan_batch(cm, m, 1 << 20, [8, 4, 4], 1, 2, 1, 1.0 / 3.0, 0.0)
    assert got is not None and got.k == 2 and got.est_time == 128.0
    assert [(c.context, c.slices, int(c.is_split)) for c in got.chunks] == \
        [(0, [(0, 0, 6)], 1), (6, [(0, 6, 2), (1, 0, 4)], 0), (0, [(2, 0, 4)], 0)]
    assert got.pipeline_of_chunk == [0, 0, 0] and got.fwd_pos_of_chunk == [0, 1, 2]
    assert got.C == [[0, 0, 0, 0]]
    only1 = cs.chunk_sched_plan_batch(cm, m, 1 << 20, [8, 4, 4], 1, 1, 1, 1.0 / 3.0, 0.0)
    assert only1.k == 1 and only1.est_time == 144.0
