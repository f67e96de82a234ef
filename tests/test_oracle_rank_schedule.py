"""Pins for the oracle's rank-block schedule (the paper's own eviction order)."""
import itertools
import os

import numpy as np
import pytest

from oracle import kvc_oracle as O
from paper_2410_00161_amd import workloads as W
from helpers import oracle_state, check_allocator_invariants
from test_oracle_worked_example import load_fixture, build


def small_state(seed, **kw):
    shape, ctx, seed = W.small_mixed(seed, **kw)
    cache = W.make_cache(shape, ctx, seed, placement="fragmented")
    st = oracle_state(cache)
    rng = np.random.default_rng(seed)
    st.metric = rng.random(st.metric.shape).astype(np.float32).astype(np.float64)
    return shape, st


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_evicted_set_is_the_smallest_metrics_and_heads_end_on_block_boundaries(seed):
    """Per head the evicted KVs are exactly its e*b - z smallest metrics (z = empty slots of
    the last block): what an unconstrained eviction of that many KVs would take."""
    shape, st = small_state(seed, S=2, Lyr=2, Hk=3, r=2, d=64, L=260, b=16 if seed != 3 else 4)
    nb = -(-st.lens() // st.b)
    budget = [int(0.4 * nb.reshape(st.S, -1).sum(1)[s]) for s in range(st.S)]
    rows, masks, sel = O.rank_schedule(st, budget)
    assert list(sel) == budget
    for g in range(st.G):
        C = int(st.lens()[g]); z = nb[g] * st.b - C
        n, o = O.slots_of(st, g)
        vals = st.metric[n, o]
        want_n = max(0, rows[g] * st.b - z) if rows[g] else 0
        assert masks[g].sum() == want_n
        assert rows[g] <= nb[g] - 1
        if want_n:
            assert vals[masks[g]].max() <= vals[~masks[g]].min()
            # unconstrained optimum for that count
            assert np.isclose(vals[masks[g]].sum(), np.sort(vals)[:want_n].sum())
    before = st.copy()
    freed = O.compact_slots(st, masks)
    assert freed == sum(budget) == int(rows.sum())
    check_allocator_invariants(st)
    for g in range(st.G):
        if rows[g]:
            assert st.lens()[g] % st.b == 0                      # whole blocks left
        assert -(-st.lens()[g] // st.b) == nb[g] - rows[g]
        n0, o0 = O.slots_of(before, g); n1, o1 = O.slots_of(st, g)
        keep = np.sort(before.metric[n0, o0][~masks[g]]); got = np.sort(st.metric[n1, o1])
        np.testing.assert_array_equal(keep, got)


def test_cross_head_order_is_by_row_maximum_brute_force():
    """Tiny case: the marked rows are the E smallest of {m(h, e)} over all heads, where m(h, e)
    is the (e*b)-th smallest entry of the head counting its empty slots as zeros."""
    rng = np.random.default_rng(5)
    S, Lyr, Hk, b = 1, 2, 2, 3
    G = S * Lyr * Hk
    lens = np.array([7, 3, 10, 4])
    nb = -(-lens // b)
    N = int(nb.sum()); maxb = int(nb.max())
    table = -np.ones((G, maxb), dtype=np.int64); p = 0
    for g in range(G):
        table[g, :nb[g]] = np.arange(p, p + nb[g]); p += nb[g]
    M = rng.permutation(N * b).astype(np.float64).reshape(N, b) + 1.0   # distinct
    st = O.State(S, Lyr, Hk, 1, 1, b, N, maxb, np.zeros((N, b, 1)), np.zeros((N, b, 1)), M,
                 np.zeros((N, b)), table, lens, np.zeros(N, dtype=np.uint8))
    def m_of(g, e):
        n, o = O.slots_of(st, g)
        vals = sorted([0.0] * (nb[g] * b - lens[g]) + list(M[n, o]))
        return vals[e * b - 1]
    all_rows = sorted((m_of(g, e), g, e) for g in range(G) for e in range(1, nb[g]))
    for E in range(0, len(all_rows) + 2):
        rows, masks, sel = O.rank_schedule(st, [E])
        take = min(E, len(all_rows))
        assert sel[0] == take
        want = np.zeros(G, dtype=int)
        for _, g, e in all_rows[:take]:
            want[g] += 1
        np.testing.assert_array_equal(rows, want)


def test_b1_rank_mode_equals_physical_mode_and_flat_sort():
    rng = np.random.default_rng(7)
    S, Lyr, Hk, b = 2, 1, 3, 1
    G = S * Lyr * Hk
    lens = rng.integers(2, 9, size=G)
    N = int(lens.sum()); maxb = int(lens.max())
    table = -np.ones((G, maxb), dtype=np.int64); p = 0
    for g in range(G):
        table[g, :lens[g]] = np.arange(p, p + lens[g]); p += lens[g]
    M = rng.random((N, 1)).astype(np.float32).astype(np.float64)
    st = O.State(S, Lyr, Hk, 1, 1, b, N, maxb, np.zeros((N, 1, 1)), np.zeros((N, 1, 1)), M,
                 np.zeros((N, 1)), table, lens, np.zeros(N, dtype=np.uint8))
    key, _ = O.block_keys(st)
    for protect in (0, 1):
        budget = [3, 4]
        rows, masks, sel = O.rank_schedule(st, budget, protect_tail_blocks=protect)
        flag, count, sel2 = O.evict_select(st, key, budget, protect_tail_blocks=protect)
        np.testing.assert_array_equal(sel, sel2)
        if protect == 0:  # the same KVs: the E lowest metrics of each sequence's flattened heads
            np.testing.assert_array_equal(rows, count)
            for g in range(G):
                np.testing.assert_array_equal(masks[g], flag[g][:lens[g]].astype(bool))
            for s in range(S):
                gs = range(s * Lyr * Hk, (s + 1) * Lyr * Hk)
                allv = np.sort(np.concatenate([M[table[g, :lens[g]], 0] for g in gs]))
                ev = np.sort(np.concatenate([M[table[g, :lens[g]], 0][masks[g]] for g in gs]))
                np.testing.assert_array_equal(ev, allv[:budget[s]])


def test_worked_example_in_rank_mode():
    """Two heads, b = 2, 5 and 2 KVs, two blocks to evict: both from head 0, which is left
    with exactly 2 KVs in one block; a third eviction takes head 1's lone block."""
    st = build(load_fixture())
    rows, masks, sel = O.rank_schedule(st, [2], protect_tail_blocks=0)
    assert list(rows) == [2, 0] and sel[0] == 2
    assert masks[0].sum() == 3                        # 2 * b minus the one empty slot
    rows3, _, sel3 = O.rank_schedule(st, [3], protect_tail_blocks=0)
    assert list(rows3) == [2, 1] and sel3[0] == 3
    freed = O.compact_slots(st, masks)
    assert freed == 2 and st.lens()[0] == 2 and st.lens()[1] == 2
    n, o = O.slots_of(st, 0)
    assert sorted(st.metric[n, o]) == [0.20, 1.90]    # the two largest of head 0 survive


def test_ties_and_errors():
    shape, st = small_state(9, S=2, Lyr=1, Hk=2, r=1, d=32, L=80, b=4)
    rng = np.random.default_rng(0)
    st.metric = rng.integers(0, 3, st.metric.shape).astype(np.float64)     # heavy ties
    nb = -(-st.lens() // st.b)
    budget = [int(nb.reshape(st.S, -1).sum(1)[s] // 2) for s in range(st.S)]
    rows, masks, sel = O.rank_schedule(st, budget)
    for g in range(st.G):   # among equal metrics the lower logical index goes first
        n, o = O.slots_of(st, g); vals = st.metric[n, o]
        if masks[g].any():
            thr = vals[masks[g]].max()
            tied = np.flatnonzero(vals == thr)
            k = int(masks[g][tied].sum())
            assert masks[g][tied[:k]].all() and not masks[g][tied[k:]].any()
    bad = st.metric.copy(); n, o = O.slots_of(st, 0); bad[n[0], o[0]] = np.nan
    with pytest.raises(O.OracleError) as e:
        O.rank_schedule(st, budget, metric=bad)
    assert e.value.code == O.ERR_NUMERIC
