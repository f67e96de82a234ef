"""GPU parity of the observation-window metric (matrix-core kernels) against the oracle."""
import numpy as np
import pytest
import torch

from oracle import kvc_oracle as O
from paper_2410_00161_amd import binding as B
from paper_2410_00161_amd import workloads as W
from helpers import oracle_state, assert_keys_equal
from test_gpu_parity import session, say, TOL

pytestmark = pytest.mark.gpu

CASES = [
    ("w8_r4", dict(r=4, L=2600, rho=1.5), 8, 7, B.KVC_L2),
    ("w32_r4", dict(r=4, L=1500, rho=1.5), 32, 7, B.KVC_L2),
    ("w8_r8_b32", dict(r=8, L=1300, rho=2.0, b=32), 8, 7, B.KVC_L2),
    ("w32_r8", dict(r=8, L=1100, rho=2.0), 32, 5, B.KVC_L2),
    ("w5_r2_L1_nopool", dict(r=2, L=1200, rho=2.0), 5, 1, B.KVC_L1),
    ("w16_r1", dict(r=1, L=1200, rho=2.0), 16, 3, B.KVC_L2),
    # a pool wider than the halo the pooling kernel stages; heads longer than one pooling tile
    ("w8_r4_wide_pool", dict(r=4, L=2600, rho=1.5), 8, 201, B.KVC_L2),
    ("w4_r2_pool_129", dict(r=2, L=4500, rho=1.2), 4, 129, B.KVC_L2),
    # the shapes the decode covers as well: 8-bit rows, d = 64, blocks shorter than a row of lanes
    ("fp8_w32_r4", dict(r=4, L=1500, rho=1.5, kv_dtype="fp8"), 32, 7, B.KVC_L2),
    ("fp8_w32_r8_b32", dict(r=8, L=1300, rho=2.0, kv_dtype="fp8", b=32), 32, 7, B.KVC_L2),
    ("fp8_d64_w16_r2_L1", dict(r=2, L=1300, rho=2.0, kv_dtype="fp8", d=64), 16, 3, B.KVC_L1),
    ("d64_w32_r4", dict(r=4, L=1500, rho=1.5, d=64), 32, 7, B.KVC_L2),
    ("d64_w8_r1", dict(r=1, L=2600, rho=1.5, d=64), 8, 7, B.KVC_L2),
    ("d64_w32_r8_b64", dict(r=8, L=1300, rho=2.0, d=64, b=64), 32, 5, B.KVC_L2),
    ("b4_w32_r4", dict(r=4, L=1500, rho=1.5, b=4), 32, 7, B.KVC_L2),
    ("b8_w8_r8", dict(r=8, L=1300, rho=2.0, b=8), 8, 7, B.KVC_L2),
    ("b1_w16_r2", dict(r=2, L=1200, rho=2.0, b=1), 16, 7, B.KVC_L2),
    ("b2_fp8_d64_w8_r4", dict(r=4, L=1200, rho=2.0, b=2, kv_dtype="fp8", d=64), 8, 3, B.KVC_L2),
    ("b128_w8_r4", dict(r=4, L=2600, rho=1.5, b=128), 8, 7, B.KVC_L2),
]


def window_queries(shape, w, seed, device):
    g = torch.Generator(device=device).manual_seed(seed)
    q = torch.randn((shape.num_seqs, shape.num_layers, shape.num_q_heads, w, shape.head_dim),
                    generator=g, device=device, dtype=torch.float32)
    return q.to(shape.q_torch_dtype)


def poison_unowned_keys(cache, real):
    if cache.k_cache.dtype == torch.float8_e4m3fn:
        cache.k_cache.view(torch.uint8)[~real] = 0x7F      # the 8-bit NaN
    else:
        cache.k_cache[~real] = float("nan")


def row_lse(st, q, w, first_pos=None):
    """ln of every query row's softmax denominator over the keys it attends to, with a library
    logsumexp on the host (what a prefill's attention kernel would hand over).  q [S, Lyr, Hq, w, d];
    query i sits at C - w + i (first_pos None) or at first_pos + i, seeing keys up to
    min(position, C - 1).  Rows that see no key get 0 (never used)."""
    S, Lyr, Hk, r, d = st.S, st.Lyr, st.Hk, st.r, st.d
    q = np.asarray(q, dtype=np.float64).reshape(S, Lyr, Hk * r, w, d)
    out = np.zeros((S, Lyr, Hk * r, w), dtype=np.float32)
    for g in range(st.G):
        s, l, h = g // (Lyr * Hk), (g // Hk) % Lyr, g % Hk
        C = int(st.lens()[g])
        if C == 0:
            continue
        n, o = O.slots_of(st, g)
        K = torch.from_numpy(st.k_cache[n, o])
        for hq in range(r * h, r * (h + 1)):
            sc = (K @ torch.from_numpy(q[s, l, hq]).T) / np.sqrt(float(d))         # [C, w]
            for i in range(w):
                last = (C - w + i) if first_pos is None else min(first_pos + i, C - 1)
                if last >= 0:
                    out[s, l, hq, i] = float(torch.logsumexp(sc[:last + 1, i], dim=0))
    return out


@pytest.mark.parametrize("name,kw,w,pool,mode", CASES, ids=[c[0] for c in CASES])
def test_window_metric_matches_oracle(name, kw, w, pool, mode):
    say("window metric", name)
    base = dict(d=128, kv_dtype="bf16")
    base.update(kw)
    shape, ctx, seed = W.small_mixed(101, S=2, Lyr=2, Hk=2, **base)
    ctx[1] = 0            # no KV at all
    ctx[2] = 3            # shorter than the window
    ctx[3] = w            # exactly the window
    ctx[4] = 1024 + 16    # just past one chunk
    cache = W.make_cache(shape, ctx, seed, placement="fragmented", init_metric="prefill")
    st0 = oracle_state(cache)
    real = torch.zeros_like(cache.metric, dtype=torch.bool)
    for g in range(st0.G):
        n, o = O.slots_of(st0, g)
        real[torch.from_numpy(n), torch.from_numpy(o)] = True
    poison_unowned_keys(cache, real)             # slots that hold no KV must never leak in
    st = oracle_state(cache)
    qw = window_queries(shape, w, seed, "cpu")
    O.window_metric(st, qw.double().numpy(), w, pool, "L2" if mode == B.KVC_L2 else "L1")
    sess = session(cache, mode)
    sess.window_metric(qw.to(sess.device), w, pool)
    torch.cuda.synchronize()
    m = sess.cache.metric.cpu().numpy().astype(np.float64)
    rm = real.numpy()
    assert np.isfinite(m[rm]).all()
    np.testing.assert_allclose(m[rm], st.metric[rm], rtol=0, atol=TOL)
    np.testing.assert_array_equal(m[~rm], cache.metric.numpy().astype(np.float64)[~rm])
    # relative check too: the sums span orders of magnitude
    big = rm & (st.metric > 1e-3)
    np.testing.assert_allclose(m[big], st.metric[big], rtol=2e-2, atol=0)
    # the same metric in one pass, from the log-sum-exp of every query row: first the true one (the
    # result above again), then one that is off by a different amount per row (used as given)
    st1 = oracle_state(cache)
    lse = row_lse(st1, qw.double().numpy(), w)
    rng = np.random.default_rng(5)
    for shift in (0.0, 0.4):
        lse_s = (lse + shift * rng.random(lse.shape)).astype(np.float32)
        st2 = oracle_state(cache)
        O.window_metric(st2, qw.double().numpy(), w, pool, "L2" if mode == B.KVC_L2 else "L1", row_lse=lse_s)
        sess2 = session(cache, mode)
        sess2.window_metric(qw.to(sess2.device), w, pool, row_lse=torch.from_numpy(lse_s).to(sess2.device))
        torch.cuda.synchronize()
        m2 = sess2.cache.metric.cpu().numpy().astype(np.float64)
        np.testing.assert_allclose(m2[rm], st2.metric[rm], rtol=0, atol=TOL)
        np.testing.assert_array_equal(m2[~rm], cache.metric.numpy().astype(np.float64)[~rm])
        big2 = rm & (st2.metric > 1e-3)
        np.testing.assert_allclose(m2[big2], st2.metric[big2], rtol=2e-2, atol=0)
        if shift == 0.0:
            np.testing.assert_allclose(st2.metric[rm], st.metric[rm], rtol=0, atol=1e-5)


def test_window_metric_layer_range_accumulate_and_unsupported():
    say("window metric layer range")
    shape, ctx, seed = W.small_mixed(103, S=2, Lyr=3, Hk=2, r=4, d=128, kv_dtype="bf16", L=500, rho=1.5)
    cache = W.make_cache(shape, ctx, seed, init_metric="prefill")
    st = oracle_state(cache)
    w = 8
    qw = window_queries(shape, w, seed, "cpu")
    sess = session(cache)
    before = sess.cache.metric.clone()
    O.window_metric(st, qw.double().numpy(), w, 7, accumulate=True, layer_begin=1, layer_end=2)
    sess.window_metric(qw.to(sess.device), w, 7, accumulate=True, layer_begin=1, layer_end=2)
    torch.cuda.synchronize()
    m = sess.cache.metric.cpu().numpy()
    np.testing.assert_allclose(m[st.free_map == 0], st.metric[st.free_map == 0], rtol=0, atol=TOL)
    for g in range(st.G):          # other layers untouched, bit for bit
        if (g // st.Hk) % st.Lyr != 1:
            n, o = O.slots_of(st, g)
            np.testing.assert_array_equal(m[n, o], before.cpu().numpy()[n, o])
    # then the eviction path runs on it as on any metric
    key = sess.metric_reduce()
    want_key, _ = O.block_keys(st, sess.cache.metric.cpu().numpy())
    assert_keys_equal(key, want_key, st)
    # shapes the matrix-core kernels do not cover are refused, nothing is touched
    shape2, ctx2, _ = W.small_mixed(104, S=1, Lyr=1, Hk=2, r=2, d=64, kv_dtype="f32", L=100)
    sess2 = session(W.make_cache(shape2, ctx2, 104))
    with pytest.raises(B.KvcError) as e:
        sess2.window_metric(torch.zeros((1, 1, 4, 4, 64), device=sess2.device), 4, 7)
    assert e.value.code == B.KVC_ERR_UNSUPPORTED
    with pytest.raises(B.KvcError) as e:
        sess.window_metric(qw.to(sess.device), w, 4)          # even pool size
    assert e.value.code == B.KVC_ERR_ARG
    # more than 64 window queries, or more than 256 query rows, at any group size (a block of the
    # all-queries metric may be that long: it is worked off in passes)
    for r, w_bad in ((1, 65), (2, 65), (4, 65), (8, 33)):
        shape3, ctx3, _ = W.small_mixed(105, S=1, Lyr=1, Hk=1, r=r, d=128, kv_dtype="bf16", L=100)
        sess3 = session(W.make_cache(shape3, ctx3, 105))
        q3 = torch.zeros((1, 1, r, w_bad, 128), device=sess3.device, dtype=torch.bfloat16)
        with pytest.raises(B.KvcError) as e:
            sess3.window_metric(q3, w_bad, 7)
        assert e.value.code == B.KVC_ERR_UNSUPPORTED, (r, w_bad)
        sess3.query_block_metric(q3, w_bad, 0)
        torch.cuda.synchronize()


def test_query_block_metric_builds_kvc_full():
    """All-queries metric with an excluded window, one block of queries at a time, against the
    oracle's block function (itself pinned to the dense definition)."""
    say("query block metric (all queries, excluded window)")
    S, Lyr, Hk, r, d, b, L, v, blk = 1, 2, 2, 4, 128, 16, 1400, 10, 64
    ctx = W.uniform_lengths(S * Lyr * Hk, L)
    shape = W.Shape(S, Lyr, Hk, r, d, b, W.pool_size(ctx, b, 1.1, 4), L // b + 2, "bf16")
    cache = W.make_cache(shape, ctx, 107, placement="fragmented")
    st = oracle_state(cache)
    sess = session(cache)
    g = torch.Generator().manual_seed(107)
    Q = torch.randn((S, Lyr, Hk * r, L, d), generator=g).to(torch.bfloat16)
    for start in list(range(0, L, blk)):
        w = min(blk, L - start)
        qb = Q[:, :, :, start:start + w].contiguous()
        if start % (5 * blk) == 0 or start + blk >= L:          # the oracle on a subset of blocks ...
            O.query_block_metric(st, qb.double().numpy(), w, start, v)
            sess.query_block_metric(qb.to(sess.device), w, start, v)
    torch.cuda.synchronize()
    m = sess.cache.metric.cpu().numpy().astype(np.float64)
    used = st.free_map == 0
    np.testing.assert_allclose(m[used], st.metric[used], rtol=0, atol=TOL)
    big = used[:, None] & (st.metric > 1e-3)
    np.testing.assert_allclose(m[big], st.metric[big], rtol=2e-2, atol=0)
    # the same blocks with the queries' log-sum-exp handed over (one pass over the keys)
    st2 = oracle_state(cache)
    sess2 = session(cache)
    for start in (0, 5 * blk, L - (L % blk or blk)):
        w = min(blk, L - start)
        qb = Q[:, :, :, start:start + w].contiguous()
        lse = row_lse(st2, qb.double().numpy(), w, first_pos=start)
        O.query_block_metric(st2, qb.double().numpy(), w, start, v, row_lse=lse)
        sess2.query_block_metric(qb.to(sess2.device), w, start, v, row_lse=torch.from_numpy(lse).to(sess2.device))
    torch.cuda.synchronize()
    m2 = sess2.cache.metric.cpu().numpy().astype(np.float64)
    np.testing.assert_allclose(m2[used], st2.metric[used], rtol=0, atol=TOL)
    big = used[:, None] & (st2.metric > 1e-3)
    np.testing.assert_allclose(m2[big], st2.metric[big], rtol=2e-2, atol=0)
