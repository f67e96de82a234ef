"""Pins for the CPU oracle: each test ties one oracle function to something the
paper or the mathematics fixes independently of the oracle's own code — a
library routine, a closed form, brute force, or an invariant."""
import itertools
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import kvc_oracle as O
from paper_2410_00161_amd import workloads as W
from helpers import oracle_state, check_allocator_invariants


def small_state(seed=3, **kw):
    shape, ctx, seed = W.small_mixed(seed, **kw)
    cache = W.make_cache(shape, ctx, seed, placement="fragmented")
    return shape, cache, oracle_state(cache)


# --- decode: paged lookup, softmax, GQA mapping -----------------------------

def test_paged_equals_library_sdpa_on_dense_kv():
    """Paged layout + per-head tables give the same output as a library SDPA run
    on dense K, V laid out before paging, with KV heads interleave-repeated r
    times (Preliminaries: Paged Attention, Grouped-Query Attention)."""
    rng = np.random.default_rng(11)
    S, Lyr, Hk, r, d, b = 2, 2, 3, 4, 32, 4
    G = S * Lyr * Hk
    lens = rng.integers(1, 40, size=G)
    nb = -(-lens // b)
    N = int(nb.sum()) + 5
    maxb = int(nb.max()) + 1
    perm = rng.permutation(N)
    dense_k = [rng.standard_normal((c, d)) for c in lens]
    dense_v = [rng.standard_normal((c, d)) for c in lens]
    kc = rng.standard_normal((N, b, d)) * 100  # garbage everywhere else
    vc = rng.standard_normal((N, b, d)) * 100
    table = -np.ones((G, maxb), dtype=np.int64)
    free = np.ones(N, dtype=np.uint8)
    p = 0
    for g in range(G):
        for u in range(nb[g]):
            table[g, u] = perm[p]; free[perm[p]] = 0; p += 1
        for j in range(lens[g]):
            kc[table[g, j // b], j % b] = dense_k[g][j]
            vc[table[g, j // b], j % b] = dense_v[g][j]
    st = O.State(S, Lyr, Hk, r, d, b, N, maxb, kc, vc, np.zeros((N, b)), np.zeros((N, b)),
                 table, lens, free)
    q = rng.standard_normal((S, Lyr, Hk * r, d))
    out = O.paged_decode(st, q, accumulate_metric=False)
    for g in range(G):
        s, l, h = g // (Lyr * Hk), (g // Hk) % Lyr, g % Hk
        K = torch.from_numpy(dense_k[g]).unsqueeze(0).repeat_interleave(r, 0)  # [r, C, d]
        V = torch.from_numpy(dense_v[g]).unsqueeze(0).repeat_interleave(r, 0)
        Q = torch.from_numpy(q[s, l, r * h:r * (h + 1)]).unsqueeze(1)          # [r, 1, d]
        ref = F.scaled_dot_product_attention(Q, K, V).squeeze(1).numpy()
        np.testing.assert_allclose(out[s, l, r * h:r * (h + 1)], ref, rtol=1e-10, atol=1e-12)


def test_uniform_heads_reduce_to_vanilla_paged_attention():
    """Equal lengths and one shared table per sequence: the per-head tables
    collapse to PagedAttention's [B, Lmax/b] table and the result equals
    ordinary attention over each sequence's tokens."""
    rng = np.random.default_rng(5)
    S, Lyr, Hk, r, d, b, L = 2, 1, 2, 2, 16, 4, 10
    nb = -(-L // b)
    # vanilla layout: one table per sequence, cache [Nv, Hk, b, d]
    Nv = S * nb + 2
    Tv = rng.permutation(Nv)[:S * nb].reshape(S, nb)
    Kv = rng.standard_normal((Nv, Hk, b, d)); Vv = rng.standard_normal((Nv, Hk, b, d))
    # the same data in the unified [N, b, d] layout: block id = vanilla id * Hk + h
    N = Nv * Hk
    kc = Kv.reshape(N, b, d).copy(); vc = Vv.reshape(N, b, d).copy()
    table = -np.ones((S, Lyr, Hk, nb), dtype=np.int64)
    for s in range(S):
        for h in range(Hk):
            table[s, 0, h] = Tv[s] * Hk + h
    free = np.ones(N, dtype=np.uint8); free[table.reshape(-1)] = 0
    st = O.State(S, Lyr, Hk, r, d, b, N, nb, kc, vc, np.zeros((N, b)), np.zeros((N, b)),
                 table, np.full((S, Lyr, Hk), L), free)
    q = rng.standard_normal((S, Lyr, Hk * r, d))
    out = O.paged_decode(st, q, accumulate_metric=False)
    for s in range(S):
        for hq in range(Hk * r):
            h = hq // r
            K = np.stack([Kv[Tv[s, i // b], h, i % b] for i in range(L)])
            V = np.stack([Vv[Tv[s, i // b], h, i % b] for i in range(L)])
            a = torch.softmax(torch.from_numpy(K @ q[s, 0, hq]) / math.sqrt(d), 0).numpy()
            np.testing.assert_allclose(out[s, 0, hq], a @ V, rtol=1e-10, atol=1e-12)


def _one_head_state(K, V, r, b, M0=None):
    C, d = K.shape
    nb = -(-C // b)
    kc = np.full((nb + 1, b, d), 7.0); vc = np.full((nb + 1, b, d), -7.0)
    table = np.arange(nb)[::-1].copy()  # reversed physical order
    for j in range(C):
        kc[table[j // b], j % b] = K[j]; vc[table[j // b], j % b] = V[j]
    free = np.ones(nb + 1, dtype=np.uint8); free[table] = 0
    M = np.zeros((nb + 1, b)) if M0 is None else M0
    return O.State(1, 1, 1, r, d, b, nb + 1, nb, kc, vc, M, np.zeros((nb + 1, b)),
                   table.reshape(1, 1, 1, nb), np.array([C]), free)


def _metric_of(st, g=0):
    n, o = O.slots_of(st, g)
    return st.metric[n, o]


def test_closed_forms():
    rng = np.random.default_rng(0)
    r, d, b, C = 4, 8, 4, 11
    # identical keys: p = 1/C, out = mean(V), increment r / C^2 (L2), r / C (L1)
    K = np.tile(rng.standard_normal(d), (C, 1)); V = rng.standard_normal((C, d))
    q = rng.standard_normal((1, 1, r, d))
    st = _one_head_state(K, V, r, b)
    out = O.paged_decode(st, q)
    np.testing.assert_allclose(out[0, 0], np.tile(V.mean(0), (r, 1)), atol=1e-12)
    np.testing.assert_allclose(_metric_of(st), r / C ** 2, atol=1e-14)
    st = _one_head_state(K, V, r, b)
    O.paged_decode(st, q, metric_mode="L1")
    np.testing.assert_allclose(_metric_of(st), r / C, atol=1e-14)
    # one dominant key: out -> its v, increment -> r on it and 0 elsewhere
    K = np.zeros((C, d)); qv = np.ones(d); K[6] = 60 * math.sqrt(d) * qv / d
    st = _one_head_state(K, V, r, b)
    out = O.paged_decode(st, np.tile(qv, (1, 1, r, 1)))
    np.testing.assert_allclose(out[0, 0], np.tile(V[6], (r, 1)), atol=1e-20 + 1e-12)
    want = np.zeros(C); want[6] = r
    np.testing.assert_allclose(_metric_of(st), want, atol=1e-12)
    # a single KV: out = v_0, increment r
    st = _one_head_state(K[:1], V[:1], r, b)
    out = O.paged_decode(st, q)
    np.testing.assert_allclose(out[0, 0], np.tile(V[0], (r, 1)), atol=1e-14)
    np.testing.assert_allclose(_metric_of(st), [r], atol=1e-14)
    # two keys with a known logit gap: p = sigmoid(gap)
    gap = 1.25
    K2 = np.zeros((2, d)); K2[0, 0] = gap * math.sqrt(d)
    q2 = np.zeros((1, 1, r, d)); q2[..., 0] = 1.0
    st = _one_head_state(K2, V[:2], r, b)
    O.paged_decode(st, q2)
    p0 = 1 / (1 + math.exp(-gap))
    np.testing.assert_allclose(_metric_of(st), [r * p0 ** 2, r * (1 - p0) ** 2], atol=1e-14)


def test_metric_sums_and_group_mapping():
    shape, cache, st = small_state(seed=21, r=4, d=64, L=200)
    q = W.make_query(shape, 21).double().numpy()
    m0 = st.metric.copy()
    O.paged_decode(st, q, metric_mode="L1")
    d = st.metric - m0
    for g in range(st.G):
        n, o = O.slots_of(st, g)
        assert abs(d[n, o].sum() - st.r) < 1e-9          # probabilities of r heads
    # nothing outside the attended slots moved
    mask = np.zeros_like(d, dtype=bool)
    for g in range(st.G):
        n, o = O.slots_of(st, g); mask[n, o] = True
    assert (d[~mask] == 0).all()
    st2 = oracle_state(cache)
    O.paged_decode(st2, q, metric_mode="L2")
    d2 = st2.metric - m0
    for g in range(st.G):
        n, o = O.slots_of(st2, g); C = len(n)
        assert st.r / C - 1e-12 <= d2[n, o].sum() <= st.r + 1e-12
    # the increment of KV head h uses exactly query heads r*h .. r*h+r-1:
    # zeroing any other query head's vector leaves that head's increments unchanged
    q3 = q.copy(); q3[:, :, 0:st.r] = 0.0          # group of KV head 0
    st3 = oracle_state(cache)
    O.paged_decode(st3, q3, metric_mode="L2")
    d3 = st3.metric - m0
    for g in range(st.G):
        n, o = O.slots_of(st, g)
        same = np.allclose(d3[n, o], d2[n, o], atol=0, rtol=0)
        assert same == (g % st.Hk != 0)


def test_continual_accumulation_equals_dense_column_sums():
    """T decode steps, no eviction: the metric of every KV equals the column sum
    of the squared attention matrix of those T queries (Continual Compression)."""
    rng = np.random.default_rng(9)
    r, d, b, C0, T = 2, 16, 4, 9, 6
    K = rng.standard_normal((C0 + T, d)); V = rng.standard_normal((C0 + T, d))
    Q = rng.standard_normal((T, r, d))
    M0 = None
    nb = -(-(C0 + T) // b)
    st = _one_head_state(K[:C0], V[:C0], r, b)
    # room to grow: rebuild with a bigger table
    st = O.State(1, 1, 1, r, d, b, nb + 2, nb + 1,
                 np.concatenate([st.k_cache, np.zeros((nb + 2 - st.N, b, d))]),
                 np.concatenate([st.v_cache, np.zeros((nb + 2 - st.N, b, d))]),
                 np.zeros((nb + 2, b)), np.zeros((nb + 2, b)),
                 np.concatenate([st.block_table.reshape(-1), -np.ones(nb + 1 - st.max_blocks)]).reshape(1, 1, 1, -1),
                 st.ctx_len, np.concatenate([st.free_map, np.ones(nb + 2 - st.N, dtype=np.uint8)]))
    prior = rng.random(C0)
    n, o = O.slots_of(st, 0); st.metric[n, o] = prior
    for t in range(T):
        O.append(st, K[C0 + t].reshape(1, 1, 1, d), V[C0 + t].reshape(1, 1, 1, d))
        O.paged_decode(st, Q[t].reshape(1, 1, r, d))
    # dense: query t sees keys 0 .. C0+t (its own token included)
    want = np.zeros(C0 + T); want[:C0] = prior
    for t in range(T):
        for h in range(r):
            L = C0 + t + 1
            a = torch.softmax(torch.from_numpy(K[:L] @ Q[t, h]) / math.sqrt(d), 0).numpy()
            want[:L] += a ** 2
    np.testing.assert_allclose(_metric_of(st), want, rtol=1e-12, atol=1e-14)
    n, o = O.slots_of(st, 0)
    np.testing.assert_array_equal(st.pos[n, o][C0:], np.arange(C0, C0 + T))
    check_allocator_invariants(st)


# --- allocator ---------------------------------------------------------------

def test_alloc_order_free_and_errors():
    shape, cache, st = small_state(seed=4, L=120)
    check_allocator_invariants(st)
    free_before = np.flatnonzero(st.free_map == 1)
    want = np.zeros(st.G, dtype=np.int64); want[[1, 4, 5]] = [2, 1, 3]
    held = [O.num_blocks_held(st, g) for g in range(st.G)]
    O.block_alloc(st, want)
    check_allocator_invariants(st)
    got = np.concatenate([st.table()[g, held[g]:held[g] + want[g]] for g in (1, 4, 5)])
    np.testing.assert_array_equal(got, free_before[:6])   # lowest ids, ascending g
    # free gives them back and clamps nothing it should not
    lens0 = st.lens().copy()
    assert O.block_free(st, want) == 6
    check_allocator_invariants(st)
    np.testing.assert_array_equal(st.lens(), lens0)
    np.testing.assert_array_equal(np.flatnonzero(st.free_map == 1), free_before)
    # dropping a block that holds tokens shortens the head
    drop = np.zeros(st.G, dtype=np.int64); drop[2] = 1
    O.block_free(st, drop)
    assert st.lens()[2] == (held[2] - 1) * st.b
    # errors leave the state untouched
    snap = st.copy()
    big = np.zeros(st.G, dtype=np.int64); big[0] = int((st.free_map == 1).sum()) + 1
    with pytest.raises(O.OracleError) as e:
        O.block_alloc(st, big)
    assert e.value.code in (O.ERR_OOM, O.ERR_TABLE_FULL)
    full = np.zeros(st.G, dtype=np.int64); full[0] = st.max_blocks - held[0] + 1
    with pytest.raises(O.OracleError) as e:
        O.block_alloc(st, full)
    assert e.value.code == O.ERR_TABLE_FULL
    for a, c in zip((st.block_table, st.free_map, st.ctx_len),
                    (snap.block_table, snap.free_map, snap.ctx_len)):
        np.testing.assert_array_equal(a, c)


def test_append_allocates_only_on_block_boundaries():
    shape, cache, st = small_state(seed=8, L=90, b=16)
    lens0 = st.lens().copy()
    free0 = int((st.free_map == 1).sum())
    k, v = W.make_new_kv(shape, 8)
    O.append(st, k.double().numpy(), v.double().numpy())
    check_allocator_invariants(st)
    crossed = int((lens0 % st.b == 0).sum())
    assert free0 - int((st.free_map == 1).sum()) == crossed
    np.testing.assert_array_equal(st.lens(), lens0 + 1)
    kk = k.double().numpy().reshape(st.G, -1)
    for g in range(st.G):
        n, o = O.slots_of(st, g)
        np.testing.assert_array_equal(st.k_cache[n[-1], o[-1]], kk[g])
        assert st.metric[n[-1], o[-1]] == 0.0


# --- block keys ---------------------------------------------------------------

def test_block_keys_fill_rule_and_fp32_order():
    shape, cache, st = small_state(seed=6, L=150)
    rng = np.random.default_rng(1)
    st.metric = rng.random(st.metric.shape)
    # poison every slot that is not a real KV: it must not matter
    real = np.zeros_like(st.metric, dtype=bool)
    for g in range(st.G):
        n, o = O.slots_of(st, g); real[n, o] = True
    st.metric[~real] = np.nan
    key, key64 = O.block_keys(st)
    assert np.isfinite(key).all()
    for g in range(st.G):
        n, o = O.slots_of(st, g)
        vals = st.metric[n, o]
        for u in range(-(-len(vals) // st.b)):
            chunk = vals[u * st.b:(u + 1) * st.b]
            assert abs(key[g, u] - math.fsum(chunk)) <= 4e-6 * max(1.0, math.fsum(chunk))
            assert abs(key64[g, u] - math.fsum(chunk)) < 1e-12
        assert (key[g, -(-len(vals) // st.b):] == 0).all()
    # integer-valued metrics sum exactly in any precision
    st.metric = np.where(real, rng.integers(0, 1000, st.metric.shape), 0).astype(np.float64)
    key, key64 = O.block_keys(st)
    np.testing.assert_array_equal(key.astype(np.float64), key64)
    # left-to-right fp32: 2^24 + 1 + 1 stays 2^24, while 1 + 1 + 2^24 gains 2
    C, b = 3, 4
    for order, want in (([2.0 ** 24, 1.0, 1.0], 2.0 ** 24), ([1.0, 1.0, 2.0 ** 24], 2.0 ** 24 + 2)):
        s1 = _one_head_state(np.zeros((C, 2)), np.zeros((C, 2)), 1, b)
        n, o = O.slots_of(s1, 0); s1.metric[n, o] = order
        assert O.block_keys(s1)[0][0, 0] == np.float32(want)


def test_block_keys_maximum_mode():
    """Max keys: the largest metric among a block's real slots; and the bridge to the paper's
    own schedule: when a head stores its KVs in ascending metric order (equal values aside),
    block u IS row u of the sorted metric matrix, so its max key is that row's last column and
    selecting blocks by max key evicts, head by head, as many blocks as the rank schedule
    evicts rows."""
    shape, cache, st = small_state(seed=9, L=150)
    rng = np.random.default_rng(4)
    real = np.zeros_like(st.metric, dtype=bool)
    for g in range(st.G):
        n, o = O.slots_of(st, g); real[n, o] = True
    st.metric = rng.random(st.metric.shape)
    st.metric[~real] = np.nan
    key, key64 = O.block_keys(st, key="max")
    for g in range(st.G):
        n, o = O.slots_of(st, g)
        vals = st.metric[n, o]
        nb = -(-len(vals) // st.b)
        for u in range(nb):
            chunk = vals[u * st.b:(u + 1) * st.b]
            assert key[g, u] == np.float32(max(chunk)) and key64[g, u] == max(chunk)
        assert (key[g, nb:] == 0).all()
    with pytest.raises(O.OracleError):
        O.block_keys(st, key="mean")
    # sorted heads of whole blocks: physical blocks by max key == rank rows
    for g in range(st.G):
        n, o = O.slots_of(st, g)
        keep = (len(n) // st.b) * st.b          # whole blocks only, so no empty slots enter the rows
        st.ctx_len.reshape(-1)[g] = keep
        n, o = n[:keep], o[:keep]
        st.metric[n, o] = np.sort(rng.random(keep))
    key, _ = O.block_keys(st, key="max")
    nb = st.lens() // st.b
    budget = (nb.reshape(st.S, -1).sum(1) * 0.4).astype(np.int64)
    flag, count, sel = O.evict_select(st, key, budget, None, 1)
    rows, _, sel_r = O.rank_schedule(st, budget, None, 1)
    np.testing.assert_array_equal(count, rows)
    np.testing.assert_array_equal(sel, sel_r)
    for g in range(st.G):                       # and they are each head's first blocks
        assert flag[g, :count[g]].all() and not flag[g, count[g]:].any()


# --- selection ----------------------------------------------------------------

def _brute_force_select(cands, E):
    """Minimum-total-key subset of size E; ties resolved towards the
    lexicographically smallest sorted index list."""
    best = None
    for sub in itertools.combinations(range(len(cands)), E):
        tot = math.fsum(cands[i][0] for i in sub)
        keyt = (tot, sub)
        if best is None or keyt < best:
            best = keyt
    return set(best[1]) if best else set()


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_selection_is_the_minimum_cost_subset(seed):
    rng = np.random.default_rng(seed)
    S, Lyr, Hk, b = 2, 2, 2, 2
    G = S * Lyr * Hk
    lens = rng.integers(1, 6, size=G)
    nb = -(-lens // b)
    maxb = int(nb.max())
    N = int(nb.sum())
    table = -np.ones((G, maxb), dtype=np.int64); p = 0
    for g in range(G):
        for u in range(nb[g]):
            table[g, u] = p; p += 1
    st = O.State(S, Lyr, Hk, 1, 2, b, N, maxb, np.zeros((N, b, 2)), np.zeros((N, b, 2)),
                 np.zeros((N, b)), np.zeros((N, b)), table, lens, np.zeros(N, dtype=np.uint8))
    key = np.zeros((G, maxb), dtype=np.float32)
    # distinct powers of two (subset sums are then unique), plus a few exact ties
    vals = (2.0 ** rng.permutation(np.arange(-10, 14)))[:N]
    key[table >= 0] = vals
    if seed == 2:
        key[table >= 0] = rng.integers(0, 3, size=N).astype(np.float32)  # heavy ties
    for protect in (0, 1):
        for E in (0, 1, 2, 3):
            flag, count, sel = O.evict_select(st, key, [E, E], protect_tail_blocks=protect)
            for s in range(S):
                cands = [(float(key[g, u]), g, u) for g in range(s * Lyr * Hk, (s + 1) * Lyr * Hk)
                         for u in range(max(0, nb[g] - protect))]
                take = min(E, len(cands))
                assert sel[s] == take
                got = {i for i, (_, g, u) in enumerate(cands) if flag[g, u]}
                assert len(got) == take
                if seed != 2:
                    assert got == _brute_force_select(cands, take)
                else:  # ties: cost is minimal and the tie-break is index order
                    order = sorted(range(len(cands)), key=lambda i: cands[i])
                    assert got == set(order[:take])
                    bf = _brute_force_select(cands, take)
                    assert math.fsum(cands[i][0] for i in got) == math.fsum(cands[i][0] for i in bf)
            np.testing.assert_array_equal(count, flag.sum(1))
            # protected tails are never flagged
            for g in range(G):
                assert not flag[g, max(0, nb[g] - protect):].any()


def test_pooled_segment_and_b1_reduce_to_flat_sort():
    """b = 1 and one segment over the batch: selection is 'drop the E lowest
    metrics of the flattened heads' (Ada-SnapKV style flattened sort)."""
    rng = np.random.default_rng(3)
    S, Lyr, Hk, b = 3, 1, 2, 1
    G = S * Lyr * Hk
    lens = rng.integers(2, 9, size=G)
    N = int(lens.sum()); maxb = int(lens.max())
    table = -np.ones((G, maxb), dtype=np.int64); p = 0
    for g in range(G):
        table[g, :lens[g]] = np.arange(p, p + lens[g]); p += lens[g]
    M = rng.random((N, 1))
    st = O.State(S, Lyr, Hk, 1, 2, b, N, maxb, np.zeros((N, 1, 2)), np.zeros((N, 1, 2)),
                 M, np.zeros((N, 1)), table, lens, np.zeros(N, dtype=np.uint8))
    key, _ = O.block_keys(st)
    E = 7
    flag, count, sel = O.evict_select(st, key, [E], seg_offsets=[0, S], protect_tail_blocks=0)
    assert sel[0] == E
    flat = np.sort(M.astype(np.float32).reshape(-1))
    chosen = np.sort(key[flag.astype(bool)])
    np.testing.assert_array_equal(chosen, flat[:E])


def test_select_errors_and_clamp():
    shape, cache, st = small_state(seed=2, L=100)
    key, _ = O.block_keys(st)
    bad = key.copy(); bad[0, 0] = np.nan
    with pytest.raises(O.OracleError) as e:
        O.evict_select(st, bad, [1] * st.S)
    assert e.value.code == O.ERR_NUMERIC
    bad = key.copy(); bad[0, 0] = -1.0
    with pytest.raises(O.OracleError):
        O.evict_select(st, bad, [1] * st.S)
    flag, count, sel = O.evict_select(st, key, [10 ** 6] * st.S)
    nb = -(-st.lens() // st.b)
    per_seq = (np.maximum(nb - 1, 0)).reshape(st.S, -1).sum(1)
    np.testing.assert_array_equal(sel, per_seq)


# --- compaction ---------------------------------------------------------------

def one_head_state(C, b, rng, spare=3):
    """One head instance of C KVs over a shuffled pool; the K row, V row, metric and pos of
    logical slot j all carry j, so that after a compaction every slot says where its KV came
    from.  Slots past C (the rest of the last block) carry -7."""
    nb = -(-C // b)
    N = nb + spare
    ids = rng.permutation(N)[:nb]
    kc = np.full((N, b, 2), -7.0); vc = np.full((N, b, 2), -7.0)
    M = np.full((N, b), -7.0); pos = np.full((N, b), -7)
    for j in range(C):
        n, o = ids[j // b], j % b
        kc[n, o] = (j, 1000 + j); vc[n, o] = (2000 + j, 3000 + j); M[n, o] = j; pos[n, o] = j
    table = -np.ones((1, nb + 1), dtype=np.int64); table[0, :nb] = ids
    free = np.ones(N, dtype=np.uint8); free[ids] = 0
    return O.State(1, 1, 1, 1, 2, b, N, nb + 1, kc, vc, M, pos, table, [C], free), ids


def logical_sources(st):
    """The original logical index of the KV that sits in each logical slot now; checks that
    key, value, metric and pos of a slot all moved together."""
    n, o = O.slots_of(st, 0)
    src = st.pos[n, o]
    np.testing.assert_array_equal(st.k_cache[n, o][:, 0], src)
    np.testing.assert_array_equal(st.k_cache[n, o][:, 1], 1000 + src)
    np.testing.assert_array_equal(st.v_cache[n, o][:, 0], 2000 + src)
    np.testing.assert_array_equal(st.v_cache[n, o][:, 1], 3000 + src)
    np.testing.assert_array_equal(st.metric[n, o], src)
    return [int(x) for x in src]


def two_pointer_by_hand(w):
    """Algorithm 1 restated inside the test, independently of the oracle: j walks down from the
    last KV through the eviction range (the last n_ev slots); every kept KV met there goes to
    the evicted slot that i, walking up from slot 0, finds next.  Returns the logical order
    after the moves (content of slots 0 .. T-1)."""
    C = len(w); n_ev = int(np.sum(w)); T = C - n_ev
    content = list(range(C))
    i = 0
    for j in range(C - 1, T - 1, -1):
        if w[j]:
            continue
        while not w[i]:
            i += 1
        assert i < T
        content[i] = j
        i += 1
    return content[:T]


def test_movecache_pairing_order_by_hand():
    """Algorithm 1 on a case worked by hand.  b = 2, C = 6, the head's first block (slots 0, 1)
    is evicted: the eviction range is slots 4, 5; j starts at 5, so slot 5 moves first and lands
    in the first hole i finds, slot 0; then slot 4 goes to slot 1.  Logical order afterwards:
    5, 4, 2, 3.  (The reversed pairing, movers ascending, would give 4, 5, 2, 3.)"""
    rng = np.random.default_rng(0)
    for via in ("flags", "slots"):
        st, ids = one_head_state(6, 2, rng)
        if via == "flags":
            flag = np.zeros((1, st.max_blocks), dtype=np.uint8); flag[0, 0] = 1
            freed = O.compact(st, flag, [1])
        else:
            freed = O.compact_slots(st, [np.array([1, 1, 0, 0, 0, 0], dtype=bool)])
        assert freed == 1 and int(st.lens()[0]) == 4
        assert logical_sources(st) == [5, 4, 2, 3]
        # the freed block is the LAST one of the row (the eviction range), not the flagged one
        assert st.table()[0].tolist() == [ids[0], ids[1], -1, -1]
        assert st.free_map[ids[2]] == 1 and st.free_map[ids[0]] == 0
    # a mask that is not block-aligned: slots 1 and 2 evicted of 7 (b = 4).  Range = slots 5, 6;
    # 6 -> hole 1, 5 -> hole 2: order 0, 6, 5, 3, 4; T = 5 still needs both blocks.
    st, ids = one_head_state(7, 4, rng)
    assert O.compact_slots(st, [np.array([0, 1, 1, 0, 0, 0, 0], dtype=bool)]) == 0
    assert logical_sources(st) == [0, 6, 5, 3, 4]
    assert st.table()[0, :2].tolist() == [ids[0], ids[1]]
    # kept KVs inside the range that are themselves evicted are skipped: evict 0 and 5 of 6:
    # range = slots 4, 5; 5 is evicted, 4 -> hole 0: order 4, 1, 2, 3
    st, ids = one_head_state(6, 2, rng)
    O.compact_slots(st, [np.array([1, 0, 0, 0, 0, 1], dtype=bool)])
    assert logical_sources(st) == [4, 1, 2, 3]


@pytest.mark.parametrize("seed", range(6))
def test_compact_moves_match_the_two_pointer_loop(seed):
    """The oracle's compaction (the closed form: k-th kept KV from the top of the range into
    the k-th evicted slot from the bottom), run on real states through O.compact_slots and
    O.compact, leaves in every slot what Algorithm 1's two-pointer walk leaves there - checked
    slot by slot against the walk restated in this test and against
    O.movecache_sequential's (src, dst) pairs, for masks that are block-aligned and masks that
    are not."""
    rng = np.random.default_rng(seed)
    for trial in range(40):
        b = int(rng.choice([1, 2, 4, 8]))
        C = int(rng.integers(1, 60))
        nb = -(-C // b)
        if trial % 2 == 0:      # any slot mask
            w = rng.random(C) < rng.random()
            st, ids = one_head_state(C, b, rng)
            O.compact_slots(st, [w])
        else:                   # whole blocks, as the block selection flags them
            fl = rng.random(nb) < rng.random()
            w = fl[np.arange(C) // b]
            st, ids = one_head_state(C, b, rng)
            flag = np.zeros((1, st.max_blocks), dtype=np.uint8); flag[0, :nb] = fl
            O.compact(st, flag, [int(fl.sum())])
        n_ev = int(w.sum()); T = C - n_ev
        assert int(st.lens()[0]) == T
        got = logical_sources(st)
        assert got == two_pointer_by_hand(w)
        want = list(range(C))
        for src, dst in O.movecache_sequential(w, C, n_ev):
            want[dst] = src
        assert got == want[:T]
        # the blocks freed are the row's last ones
        nb2 = -(-T // b)
        assert st.table()[0, :nb2].tolist() == list(ids[:nb2]) and (st.table()[0, nb2:] == -1).all()
        assert sorted(np.flatnonzero(st.free_map == 0)) == sorted(ids[:nb2])


@pytest.mark.parametrize("protect", [0, 1])
def test_compact_preserves_retained_set_and_frees_whole_blocks(protect):
    shape, cache, st = small_state(seed=12, L=300, r=2, d=64)
    rng = np.random.default_rng(0)
    st.metric = rng.random(st.metric.shape)
    key, _ = O.block_keys(st)
    nb = -(-st.lens() // st.b)
    budget = [int(0.5 * nb.reshape(st.S, -1).sum(1)[s]) for s in range(st.S)]
    flag, count, sel = O.evict_select(st, key, budget, protect_tail_blocks=protect)
    before = st.copy()
    q = W.make_query(shape, 1).double().numpy()
    freed = O.compact(st, flag, count)
    check_allocator_invariants(st)
    assert freed == int(sel.sum()) == int((st.free_map == 1).sum()) - int((before.free_map == 1).sum())
    # bytes freed = evicted blocks x block bytes (K and V)
    assert freed * 2 * st.b * st.d * shape.kv_bytes == int(sel.sum()) * 2 * st.b * st.d * shape.kv_bytes
    for g in range(st.G):
        n0, o0 = O.slots_of(before, g)
        w = flag[g][np.arange(len(n0)) // st.b].astype(bool)
        n1, o1 = O.slots_of(st, g)
        assert len(n1) == len(n0) - int(w.sum())
        rows0 = np.concatenate([before.k_cache[n0, o0], before.v_cache[n0, o0],
                                before.metric[n0, o0][:, None], before.pos[n0, o0][:, None]], 1)[~w]
        rows1 = np.concatenate([st.k_cache[n1, o1], st.v_cache[n1, o1],
                                st.metric[n1, o1][:, None], st.pos[n1, o1][:, None]], 1)
        key0 = np.lexsort(rows0.T[::-1]); key1 = np.lexsort(rows1.T[::-1])
        np.testing.assert_array_equal(rows0[key0], rows1[key1])
        # slots below the new length that were kept did not move
        keep_low = ~w[:len(n1)]
        np.testing.assert_array_equal(before.pos[n0, o0][:len(n1)][keep_low], st.pos[n1, o1][keep_low])
    # attention over the compacted head == dense attention over the retained set
    out = O.paged_decode(st, q, accumulate_metric=False)
    for g in range(st.G):
        s, l, h = g // (st.Lyr * st.Hk), (g // st.Hk) % st.Lyr, g % st.Hk
        n0, o0 = O.slots_of(before, g)
        w = flag[g][np.arange(len(n0)) // st.b].astype(bool)
        if (~w).sum() == 0:
            continue
        K = torch.from_numpy(before.k_cache[n0, o0][~w]); V = torch.from_numpy(before.v_cache[n0, o0][~w])
        for hq in range(st.r * h, st.r * (h + 1)):
            ref = F.scaled_dot_product_attention(torch.from_numpy(q[s, l, hq]).view(1, 1, -1),
                                                 K.unsqueeze(0), V.unsqueeze(0)).view(-1).numpy()
            np.testing.assert_allclose(out[s, l, hq], ref, rtol=1e-9, atol=1e-12)


def test_compact_rejects_bad_flags_without_touching_state():
    shape, cache, st = small_state(seed=2, L=100)
    flag = np.zeros((st.G, st.max_blocks), dtype=np.uint8)
    flag[0, st.max_blocks - 1] = 1
    snap = st.copy()
    with pytest.raises(O.OracleError):
        O.compact(st, flag)
    np.testing.assert_array_equal(st.block_table, snap.block_table)
    np.testing.assert_array_equal(st.ctx_len, snap.ctx_len)


def test_scheduling_helpers_by_hand():
    """Two sequences, one layer, two heads, b = 4: counts, prefill allocation and preemption
    worked out by hand."""
    S, Lyr, Hk, b, N, maxb = 2, 1, 2, 4, 16, 4
    table = -np.ones((S * Lyr * Hk, maxb), dtype=np.int64)
    table[0, :2] = [3, 9]      # seq 0 head 0: 8 KVs, both blocks full
    table[1, :1] = [5]         # seq 0 head 1: 2 KVs
    lens = np.array([8, 2, 0, 0])
    free = np.ones(N, dtype=np.uint8); free[[3, 9, 5]] = 0
    st = O.State(S, Lyr, Hk, 1, 2, b, N, maxb, np.zeros((N, b, 2)), np.zeros((N, b, 2)), np.zeros((N, b)),
                 np.zeros((N, b)), table, lens, free)
    needed, held = O.count_blocks(st)
    assert list(needed) == [1, 2] and list(held) == [3, 0]     # empty heads need their first block too
    O.prefill_alloc(st, [0, 9])                                # seq 1: ceil(9/4) = 3 blocks per head
    assert list(st.lens()) == [8, 2, 9, 9]
    np.testing.assert_array_equal(st.table()[2, :3], [0, 1, 2])   # lowest free ids, ascending g
    np.testing.assert_array_equal(st.table()[3, :3], [4, 6, 7])
    check_allocator_invariants(st)
    needed, held = O.count_blocks(st)
    assert list(needed) == [1, 0] and list(held) == [3, 6]
    assert O.preempt(st, [1, 0]) == 3
    assert list(st.lens()) == [0, 0, 9, 9] and (st.table()[:2] == -1).all()
    assert sorted(np.flatnonzero(st.free_map == 0)) == [0, 1, 2, 4, 6, 7]
    check_allocator_invariants(st)
    with pytest.raises(O.OracleError):
        O.prefill_alloc(st, [1000, 0])                         # row too short / pool too small


def test_count_blocks_over_a_layer_range_by_hand():
    """One sequence of three layers, two heads each, b = 4.  Lengths 4, 3 | 8, 0 | 5, 12 with
    1, 1 | 2, 0 | 2, 3 blocks held: the heads whose blocks are all full (a head with no block
    counts as full) are layer 0 head 0, layer 1 both heads, layer 2 head 1.  'needed' counts
    those of the chosen layers only; 'held' is over all layers whatever the range."""
    S, Lyr, Hk, b, N, maxb = 1, 3, 2, 4, 12, 3
    table = -np.ones((6, maxb), dtype=np.int64)
    table[0, :1] = [0]; table[1, :1] = [1]; table[2, :2] = [2, 3]
    table[4, :2] = [4, 5]; table[5, :3] = [6, 7, 8]
    lens = np.array([4, 3, 8, 0, 5, 12])
    free = np.ones(N, dtype=np.uint8); free[:9] = 0
    st = O.State(S, Lyr, Hk, 1, 2, b, N, maxb, np.zeros((N, b, 2)), np.zeros((N, b, 2)), np.zeros((N, b)),
                 np.zeros((N, b)), table, lens, free)
    for (l0, l1), want in {(0, 3): 4, (0, 1): 1, (1, 2): 2, (2, 3): 1, (1, 3): 3, (0, 2): 3}.items():
        needed, held = O.count_blocks(st, l0, l1)
        assert list(needed) == [want], (l0, l1)
        assert list(held) == [9]


def test_append_with_caller_positions_by_hand():
    """Two sequences, one layer, one head each, b = 2.  Sequence 0 holds 2 KVs (its block is
    full), sequence 1 holds 3 (blocks 4 and 1, second half-empty).  Appending with
    new_pos = [40, 7]: sequence 0 takes the lowest free block (0) and writes slot (0, 0);
    sequence 1 writes slot (1, 1); the new slots carry the caller's positions, not the heads'
    old lengths, and nothing else of pos changes.  With new_pos = None the old lengths go in."""
    S, Lyr, Hk, b, N, maxb, d = 2, 1, 1, 2, 6, 3, 2
    def fresh():
        table = -np.ones((2, maxb), dtype=np.int64)
        table[0, :1] = [2]; table[1, :2] = [4, 1]
        free = np.ones(N, dtype=np.uint8); free[[2, 4, 1]] = 0
        pos = np.arange(N * b).reshape(N, b) + 100
        return O.State(S, Lyr, Hk, 1, d, b, N, maxb, np.zeros((N, b, d)), np.zeros((N, b, d)),
                       np.ones((N, b)), pos, table, [2, 3], free)
    k = np.array([[1.0, 2.0], [3.0, 4.0]]).reshape(S, Lyr, Hk, d)
    v = -k
    st = fresh()
    pos0 = st.pos.copy()
    O.append(st, k, v, new_pos=[40, 7])
    assert st.table()[0].tolist() == [2, 0, -1] and st.table()[1].tolist() == [4, 1, -1]
    assert list(st.lens()) == [3, 4] and st.free_map.tolist() == [0, 0, 0, 1, 0, 1]
    assert st.pos[0, 0] == 40 and st.pos[1, 1] == 7
    changed = st.pos != pos0
    assert int(changed.sum()) == 2 and changed[0, 0] and changed[1, 1]
    np.testing.assert_array_equal(st.k_cache[0, 0], [1.0, 2.0]); np.testing.assert_array_equal(st.v_cache[1, 1], [-3.0, -4.0])
    assert st.metric[0, 0] == 0.0 and st.metric[1, 1] == 0.0 and st.metric[1, 0] == 1.0
    st = fresh()
    O.append(st, k, v)
    assert st.pos[0, 0] == 2 and st.pos[1, 1] == 3


def test_compression_batch_by_hand_and_against_a_prefix_search():
    """Five sequences, one head each, b = 4, holding 2, 5, 1, 3, 4 blocks (8, 20, 4, 12, 16 KV
    slots).  Never-compressed sequences come first, then older compressions first; the batch is
    the longest prefix of that order whose allocated KVs stay within the limit, and a sequence
    that does not fit ends it even if a later one would."""
    S, b, N, maxb = 5, 4, 32, 8
    blocks = [2, 5, 1, 3, 4]
    table = -np.ones((S, maxb), dtype=np.int64)
    nxt = 0
    for s_, nb in enumerate(blocks):
        table[s_, :nb] = range(nxt, nxt + nb); nxt += nb
    lens = np.array([nb * b - 1 for nb in blocks])            # last block partly filled: slots count, not KVs
    free = np.ones(N, dtype=np.uint8); free[:nxt] = 0
    st = O.State(S, 1, 1, 1, 2, b, N, maxb, np.zeros((N, b, 2)), np.zeros((N, b, 2)), np.zeros((N, b)),
                 np.zeros((N, b)), table, lens, free)
    last = [7, -1, 3, -5, 3]                                   # order: 1, 3 (never), then 2, 4 (time 3), then 0
    got, total = O.compression_batch(st, last, 40)
    assert list(got) == [False, True, True, True, False] and total == 36     # 20 + 12 + 4; 16 more would be 52
    got, total = O.compression_batch(st, last, 35)
    assert list(got) == [False, True, False, True, False] and total == 32    # seq 2 (4 more slots) is over the limit and closes the batch
    got, total = O.compression_batch(st, last, 19)
    assert not got.any() and total == 0                        # the first in line does not fit: nothing is compressed
    got, total = O.compression_batch(st, last, 10 ** 9)
    assert got.all() and total == 60
    got, total = O.compression_batch(st, last, 40, running=[1, 0, 1, 0, 1])  # order: 2, 4, 0
    assert list(got) == [True, False, True, False, True] and total == 28
    with pytest.raises(O.OracleError):
        O.compression_batch(st, last, -1)
    # against a search over prefixes of the explicitly sorted order, random cases
    rng = np.random.default_rng(3)
    alloc = np.array(blocks) * b
    for _ in range(200):
        last = rng.integers(-2, 4, S)
        run = rng.integers(0, 2, S).astype(bool)
        limit = int(rng.integers(0, 70))
        order = sorted(np.flatnonzero(run), key=lambda s_: (max(int(last[s_]), -1), s_))
        best = 0
        while best < len(order) and alloc[order[:best + 1]].sum() <= limit:
            best += 1
        want = np.zeros(S, dtype=bool); want[order[:best]] = True
        got, total = O.compression_batch(st, last, limit, running=run)
        np.testing.assert_array_equal(got, want)
        assert total == alloc[want].sum()


# --- 8-bit inputs -----------------------------------------------------------------

def test_e4m3_bytes_decode_as_the_format_defines():
    """The tests hand 8-bit caches to the oracle through torch's float8_e4m3fn conversion; this
    pins that conversion to the format itself: 1 sign, 4 exponent (bias 7), 3 mantissa bits,
    subnormals at exponent 0, no infinities, 0x7f and 0xff the only NaNs, largest value 448."""
    got = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    for byte in range(256):
        s, e, m = byte >> 7, (byte >> 3) & 15, byte & 7
        if e == 15 and m == 7:
            assert math.isnan(got[byte])
            continue
        mag = (m / 8.0) * 2.0 ** -6 if e == 0 else (1.0 + m / 8.0) * 2.0 ** (e - 7)
        assert got[byte] == (-mag if s else mag), byte
    assert got[0x7E] == 448.0 and math.copysign(1.0, got[0x80]) == -1.0
