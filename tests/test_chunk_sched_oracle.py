"""Pins of the chunk scheduler's reference (oracle/chunk_sched_oracle.py) against what the paper and the textbook fix:
the 1F1B makespan, the size of a chunk window (section 3.2.2), the rule that checkpointing along a diagonal of the
(stage, backward position) grid costs its recomputation exactly once (section 3.4.3), the two statements of the
activation footprint under checkpointing (section 3.2.3 and Algorithm 2), and closed forms of the checkpointing
problem and of the grouping."""
import math
import os
import random
import sys

import pytest

sys.path.insert(0, os.path.join(os.path.dirname(__file__), "..", "oracle"))
import chunk_sched_oracle as o  # noqa: E402


def model(d_p=2, d_s=2, layers=8, capacity=1e18, m_ms=None):
    return o.MemModel(d_p=d_p, d_s=d_s, layers=layers, m_token=34.0 * 4096 * 2 * layers, m_logits=4.0 * 128256, e=2.0,
                      hidden=4096.0, kv_hidden=1024.0, capacity=capacity, m_ms=m_ms or [0.0] * d_p)


def random_units(rng, max_units=5, max_chunks=4):
    counts = sorted((rng.randint(1, max_chunks) for _ in range(rng.randint(1, max_units))), reverse=True)
    return counts, [u for u, c in enumerate(counts) for _ in range(c)]


# ---- order and windows ----

def test_f2b_reverses_inside_a_sequence_only():
    assert o.f2b([0, 0, 0, 1, 1, 2]) == [2, 1, 0, 4, 3, 5]
    assert o.f2b([0, 1, 2, 3]) == [0, 1, 2, 3]
    assert o.f2b([0] * 5) == [4, 3, 2, 1, 0]


def test_pipeline_order_longest_first():
    units = [[(100, 0)], [(50, 1), (50, 1), (10, 0)], [(300, 0)], [(80, 1), (20, 0)]]
    assert o.pipeline_order(units) == [1, 3, 2, 0]


def test_window_size_is_dp_minus_p_plus_nsplit():
    # section 3.2.2: |W_p(t)| = d_p - p + N_split in the steady phase (never more, and that many once enough chunks ran)
    rng = random.Random(3)
    for _ in range(200):
        d_p = rng.randint(1, 6)
        counts, unit_of = random_units(rng)
        n, ns = len(unit_of), counts[0]
        fb = o.f2b(unit_of)
        for p in range(1, d_p + 1):
            ws = o.windows(d_p, p, n, ns, fb)
            w = min(n, d_p - p + ns)
            assert max(len(x) for x in ws) == w
            assert all(len(x) == w for x in ws[w - 1:])
            assert len(ws) == n


def test_windows_of_plain_1f1b_are_runs_of_microbatches():
    # every sequence one chunk: stage p holds d_p - p + 1 consecutive micro-batches
    d_p, n = 4, 9
    fb = list(range(n))
    for p in range(1, d_p + 1):
        w = d_p - p + 1
        ws = o.windows(d_p, p, n, 1, fb)
        assert ws[w - 1:] == [list(range(m - w, m)) for m in range(w, n + 1)]


def test_backward_never_precedes_forward_and_slices_run_backward_last_to_first():
    rng = random.Random(5)
    for _ in range(100):
        d_p = rng.randint(1, 5)
        counts, unit_of = random_units(rng)
        n, ns = len(unit_of), counts[0]
        fb = o.f2b(unit_of)
        for p in range(1, d_p + 1):
            ops = o.stage_ops(d_p, p, n, ns, fb)
            assert sorted(ops) == sorted([("F", k) for k in range(n)] + [("B", k) for k in range(n)])
            at = {op: i for i, op in enumerate(ops)}
            for k in range(n):
                assert at[("F", k)] < at[("B", k)]
                if k + 1 < n and unit_of[k + 1] == unit_of[k]:
                    assert at[("B", k + 1)] < at[("B", k)] and at[("F", k)] < at[("F", k + 1)]


# ---- timeline ----

def test_makespan_of_uniform_1f1b_is_textbook():
    # n micro-batches on d_p stages: (n + d_p - 1) (t_f + t_b), whatever the split of the sequences into chunks
    rng = random.Random(7)
    for _ in range(200):
        d_p = rng.randint(1, 6)
        counts, unit_of = random_units(rng)
        n = len(unit_of)
        tf, tb = rng.uniform(0.5, 2.0), rng.uniform(1.0, 4.0)
        ms, busy, _, held = o.simulate(d_p, counts[0], o.f2b(unit_of), [tf] * n, [tb] * n)
        assert ms == pytest.approx((n + d_p - 1) * (tf + tb), rel=1e-12)
        assert busy == pytest.approx([n * (tf + tb)] * d_p)
        assert held == [min(n, d_p - p + counts[0]) for p in range(1, d_p + 1)]
        # warm-up and cool-down cost delta = (d_p - 1) avg(T_tot)  (section 3.4.1)
        assert ms - busy[0] == pytest.approx((d_p - 1) * (tf + tb))


def test_p2p_delay_adds_two_traversals():
    d_p, n, tf, tb, c = 4, 6, 1.0, 2.0, 0.125
    ms = o.simulate(d_p, 1, list(range(n)), [tf] * n, [tb] * n, p2p=c)[0]
    assert ms >= (n + d_p - 1) * (tf + tb) + 2 * (d_p - 1) * c - 1e-12


def test_diagonal_checkpointing_costs_its_recomputation_once():
    # section 3.4.3: with ckpt'(p, k) = C[k + d_p - p] the propagated bubbles are filled, so the pipeline gets longer by
    # F_hat * sum(C) and no more
    rng = random.Random(11)
    for _ in range(300):
        d_p = rng.randint(1, 5)
        counts, unit_of = random_units(rng)
        n = len(unit_of)
        fb = o.f2b(unit_of)
        C = [rng.randint(0, 3) for _ in range(n + d_p - 1)]
        f_hat = 0.25
        rec = [[o.ckpt_of(d_p, p, k, fb, C) * f_hat for k in range(n)] for p in range(1, d_p + 1)]
        base = o.simulate(d_p, counts[0], fb, [1.0] * n, [2.0] * n)[0]
        with_ckpt = o.simulate(d_p, counts[0], fb, [1.0] * n, [2.0] * n, rec)[0]
        assert with_ckpt - base == pytest.approx(f_hat * sum(C), abs=1e-9)


def test_peak_memory_is_the_heaviest_window():
    rng = random.Random(13)
    for _ in range(50):
        d_p = rng.randint(1, 4)
        counts, unit_of = random_units(rng)
        n = len(unit_of)
        fb = o.f2b(unit_of)
        mem = [[rng.uniform(1, 10) for _ in range(n)] for _ in range(d_p)]
        peak = o.simulate(d_p, counts[0], fb, [1.0] * n, [2.0] * n, mem=mem)[2]
        for p in range(1, d_p + 1):
            assert peak[p - 1] == pytest.approx(max(sum(mem[p - 1][k] for k in w) for w in o.windows(d_p, p, n, counts[0], fb)))


# ---- activation footprint ----

def test_full_checkpointing_keeps_only_layer_inputs():
    # section 3.2.3: a checkpointed layer keeps its input (e D bytes per token, over d_s devices); a chunk that is not
    # split, on a stage without logits, with all L / d_p layers checkpointed holds nothing else
    m = model(d_p=4, d_s=2, layers=16)
    lay = m.layers // m.d_p
    assert o.act_bytes(m, 1, 1000, 0, lay) == pytest.approx(m.e * m.hidden * lay / m.d_s * 1000)


def test_no_checkpointing_is_the_plain_footprint():
    # section 3.2.2: M_token / N per token, + logits / d_s on the last stage, + dK/dV (2 e L D_kv / N) for a split chunk
    m = model(d_p=4, d_s=2, layers=16)
    n_dev = 8
    assert o.act_bytes(m, 2, 512, 0, 0) == pytest.approx(m.m_token / n_dev * 512)
    assert o.act_bytes(m, 4, 512, 0, 0) - o.act_bytes(m, 2, 512, 0, 0) == pytest.approx(m.m_logits / m.d_s * 512)
    assert o.act_bytes(m, 2, 512, 1, 0) - o.act_bytes(m, 2, 512, 0, 0) == pytest.approx(2 * m.e * m.layers * m.kv_hidden / n_dev * 512)


def test_footprint_is_linear_in_ckpt_with_the_slope_of_algorithm_2():
    # Algorithm 2: M_act = I_p[k] - F[k] c with F[k] = (M_token / (L d_s) - e (D + 2 I D_kv) / d_s) * tokens
    m = model(d_p=2, d_s=4, layers=12)
    for split in (0, 1):
        for p in (1, 2):
            f = (m.m_token / (m.layers * m.d_s) - m.e * (m.hidden + 2 * split * m.kv_hidden) / m.d_s) * 777
            a = [o.act_bytes(m, p, 777, split, l) for l in range(m.layers // m.d_p + 1)]
            for l in range(1, len(a)):
                assert a[l - 1] - a[l] == pytest.approx(f, rel=1e-12)
    # a split chunk gains less from a checkpointed layer: its keys and values stay
    assert o.act_bytes(m, 1, 777, 1, 0) - o.act_bytes(m, 1, 777, 1, 1) < o.act_bytes(m, 1, 777, 0, 0) - o.act_bytes(m, 1, 777, 0, 1)


# ---- checkpointing problem ----

def test_no_checkpointing_needed_when_everything_fits():
    m = model(d_p=2, layers=4)
    s, C = o.solve_ckpt(m, [(1000, 1), (1000, 0), (500, 0)], [0, 0, 1], 2)
    assert s == 0 and C == [0] * 4


def test_one_chunk_one_stage_closed_form():
    # a single chunk on a single stage: c = ceil((I - (G - M_ms)) / F)
    for cap_frac in (0.95, 0.7, 0.5, 0.3):
        m = model(d_p=1, d_s=1, layers=8, m_ms=[1e9])
        full = o.act_bytes(m, 1, 4096, 0, 0)
        m.capacity = 1e9 + cap_frac * full
        slope = full - o.act_bytes(m, 1, 4096, 0, 1)
        r = o.solve_ckpt(m, [(4096, 0)], [0], 1)
        need = math.ceil((full - cap_frac * full) / slope - 1e-12)
        if need > m.layers:
            assert r is None
        else:
            assert r is not None and r[0] == need


def test_infeasible_when_full_checkpointing_does_not_fit():
    m = model(d_p=2, layers=4)
    m.capacity = 0.5 * o.act_bytes(m, 1, 1000, 0, 2)
    assert o.solve_ckpt(m, [(1000, 0), (1000, 0)], [0, 1], 1) is None


def test_solution_fits_and_one_less_does_not():
    rng = random.Random(17)
    for _ in range(12):
        d_p = rng.randint(1, 2)
        m = model(d_p=d_p, d_s=1, layers=2 * d_p)
        counts, unit_of = random_units(rng, max_units=2, max_chunks=2)
        chunks = [(rng.choice([512, 1024, 2048]), int(counts[u] > 1 and k + 1 < len(unit_of) and unit_of[k + 1] == u))
                  for k, u in enumerate(unit_of)]
        n = len(chunks)
        fb = o.f2b(unit_of)
        no_ckpt = max(sum(o.act_bytes(m, p, chunks[k][0], chunks[k][1], 0) for k in w)
                      for p in range(1, d_p + 1) for w in o.windows(d_p, p, n, counts[0], fb))
        m.capacity = rng.uniform(0.55, 1.05) * no_ckpt
        r = o.solve_ckpt(m, chunks, unit_of, counts[0])
        if r is None:
            assert not o.config_fits(m, chunks, counts[0], fb, [m.layers // d_p] * (n + d_p - 1))
            continue
        assert o.config_fits(m, chunks, counts[0], fb, r[1])
        for j in range(len(r[1])):  # optimal: lowering any single variable breaks a window
            if r[1][j] > 0:
                C2 = list(r[1])
                C2[j] -= 1
                assert not o.config_fits(m, chunks, counts[0], fb, C2)
        tight = o.MemModel(**{**m.__dict__, "capacity": m.capacity * 0.9})
        r2 = o.solve_ckpt(tight, chunks, unit_of, counts[0])
        assert r2 is None or r2[0] >= r[0]  # less memory never needs less recomputation


def test_checkpointing_goes_to_the_longer_chunk():
    # section 3.4.1: at equal recomputation cost a longer chunk frees more memory
    m = model(d_p=1, d_s=1, layers=4)
    chunks, unit_of = [(4096, 0), (512, 0)], [0, 1]
    both = o.act_bytes(m, 1, 4096, 0, 0)  # the window of a single stage holds one chunk at a time
    m.capacity = both - 0.5 * (both - o.act_bytes(m, 1, 4096, 0, 1))
    s, C = o.solve_ckpt(m, chunks, unit_of, 1)
    assert s == 1 and C[o.f2b(unit_of)[0]] == 1


# ---- grouping ----

def test_grouping_one_pipeline_when_warmup_is_expensive_and_many_when_it_is_free():
    m = model(d_p=2, d_s=1, layers=4)
    units = [[(2048, 1), (2048, 0)], [(1024, 0)], [(1024, 0)]]
    order = o.pipeline_order(units)
    chunks = [c for u in order for c in units[u]]
    unit_of = [j for j, u in enumerate(order) for _ in units[u]]
    fb = o.f2b(unit_of)
    no_ckpt = max(sum(o.act_bytes(m, p, chunks[k][0], chunks[k][1], 0) for k in w)
                  for p in (1, 2) for w in o.windows(2, p, len(chunks), 2, fb))
    m.capacity = 0.8 * no_ckpt
    together = o.solve_ckpt(m, chunks, unit_of, 2)
    assert together is not None and together[0] > 0
    cost, groups = o.group(m, units, layer_fwd_time=1.0, delta=1e6)
    assert len(groups) == 1 and cost == pytest.approx(1e6 + together[0])
    cost0, groups0 = o.group(m, units, layer_fwd_time=1.0, delta=0.0)
    assert cost0 <= together[0] and sorted(sum(groups0, [])) == [0, 1, 2]


def test_grouping_is_none_when_a_sequence_can_never_fit():
    m = model(d_p=1, d_s=1, layers=2)
    m.capacity = 0.5 * o.act_bytes(m, 1, 4096, 0, 2)
    assert o.group(m, [[(4096, 0)], [(16, 0)]], 1.0, 1.0) is None


# ---- the whole solve of a batch (sections 3.3 and 3.4.2) and the sequences the scheduler sees ----

def test_units_of_chunks_on_the_mesh_example():
    # Section 3.3's example, mesh {8K, 4K, 2K}: a 13K sequence is an 8K and a 4K split chunk plus a 1K tail slice, a 9K
    # one an 8K split chunk plus a 1K tail, a 14K one 8K + 4K + a 2K tail; a 3K sequence is not cut.  The scheduler
    # sees one sequence per tail-holding chunk, its split chunks first, in order of their context.
    K = 1024
    chunks = [(0, [(0, 0, 8 * K)], 1), (8 * K, [(3, 8 * K, 4 * K)], 1), (0, [(1, 0, 8 * K)], 1), (0, [(3, 0, 8 * K)], 1),
              (8 * K, [(0, 8 * K, 4 * K)], 1),
              (12 * K, [(0, 12 * K, K)], 0), (8 * K, [(1, 8 * K, K), (2, 0, 3 * K)], 0), (12 * K, [(3, 12 * K, 2 * K)], 0)]
    assert o.units_of_chunks(chunks) == [[0, 4, 5], [2, 6], [3, 1, 7]]
    assert o.units_of_chunks([(0, [(0, 0, 5)], 0), (0, [(1, 0, 7), (2, 0, 1)], 0)]) == [[0], [1]]


def test_plan_batch_worked_example():
    # Lengths 8, 4, 4; cost T = (C + s0)^2 - C^2 + sum of the other s^2; two stages, two layers (one per stage), memory
    # to spare, so nothing is checkpointed and a pipeline costs delta = (d_p - 1) * mean chunk time.
    #   K = 1: mesh {8}, T_t = 64, T_m = 8.  Nothing is cut.  8 opens a bucket (64); 4: 8 + 4 > T_m, a second bucket
    #     (16); 4: 4 + 4 <= 8, ratios 64 / 8 = 8 and 16 / 4 = 4: the second bucket first, 16 + 16 <= 64: placed.
    #     Chunks [8], [4, 4]: times 64, 32, sum 96, mean 48; every sequence has one chunk: one pipeline.  96 + 48 = 144.
    #   K = 2: 8 = 6 + 2 (36 and 64 - 36 = 28; 5 + 3 gives 39), T_t = 36, T_m = 6.  The 8 leaves a split chunk (0, 6)
    #     and a tail (C 6, 2 tokens, 28).  4: 2 + 4 <= 6 but 28 + 16 = 44 > 36: T_t becomes 44, placed.  4: 6 + 4 > 6: a
    #     new bucket.  Chunks: split [6] 36, hybrid (C 6) [2, 4] 44, batched [4] 16: sum 96, mean 32.  Sequences: one
    #     of two chunks, one of one chunk.  One pipeline for both: 96 + 32 = 128; one each: 96 + 64 = 160.
    #   K = 2 wins with 128, one pipeline, the longer sequence first.
    import chunk_plan_oracle as po
    cost = po.Model(alpha1=1.0, alpha2=0.0, beta1=0.0)
    mem = model(d_p=2, d_s=1, layers=2)
    meshes = {1: ([8], 64.0, 8), 2: ([6, 2], 36.0, 6)}
    assert po.balanced_mesh_time(cost, 8, 2, 1) == 36.0 and po.balanced_mesh_time(cost, 8, 1, 1) == 64.0
    K, t, chunks, groups = o.plan_batch(po, cost, mem, [8, 4, 4], [1, 2], 1.0 / 3.0, lambda k: meshes[k])
    assert (K, t) == (2, 128.0)
    assert chunks == [(0, [(0, 0, 6)], 1), (6, [(0, 6, 2), (1, 0, 4)], 0), (0, [(2, 0, 4)], 0)]
    assert groups == [[[0, 1], [2]]]
    # each K alone
    assert o.plan_batch(po, cost, mem, [8, 4, 4], [1], 1.0 / 3.0, lambda k: meshes[k])[:2] == (1, 144.0)
    assert o.plan_batch(po, cost, mem, [8, 4, 4], [2], 1.0 / 3.0, lambda k: meshes[k])[1] == 128.0
