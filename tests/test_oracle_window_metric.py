"""Pins for the oracle's observation-window metric."""
import math

import numpy as np
import torch
import torch.nn.functional as F

from oracle import kvc_oracle as O
from paper_2410_00161_amd import workloads as W
from helpers import oracle_state
from test_oracle_pins import _one_head_state, _metric_of


def test_window_metric_equals_library_softmax_and_max_pool():
    rng = np.random.default_rng(2)
    r, d, b, C, w, pool = 2, 16, 4, 37, 5, 7
    K = rng.standard_normal((C, d)); V = np.zeros((C, d))
    Q = rng.standard_normal((r, w, d))
    st = _one_head_state(K, V, r, b)
    n, o = O.slots_of(st, 0)
    st.metric[n, o] = 123.0                                  # replaced, not added to
    O.window_metric(st, Q.reshape(1, 1, r, w, d), w, pool)
    # library route: masked scores -> softmax -> square -> sum over queries and heads -> max_pool1d
    scores = torch.from_numpy(np.einsum("hwd,cd->hwc", Q, K)) / math.sqrt(d)
    pos = torch.arange(C).view(1, 1, C)
    qpos = (C - w + torch.arange(w)).view(1, w, 1)
    scores = scores.masked_fill(pos > qpos, float("-inf"))
    A = torch.softmax(scores, dim=-1)
    raw = (A ** 2).sum(dim=(0, 1))
    prefix = raw[:C - w].view(1, 1, -1)
    pooled = F.max_pool1d(prefix, kernel_size=pool, stride=1, padding=pool // 2).view(-1)
    want = torch.cat([pooled, raw[C - w:]]).numpy()
    np.testing.assert_allclose(_metric_of(st), want, rtol=1e-12, atol=1e-15)
    # pool = 1 leaves the raw sums; L1 sums probabilities: every window query's row sums to 1
    st = _one_head_state(K, V, r, b)
    O.window_metric(st, Q.reshape(1, 1, r, w, d), w, 1, metric_mode="L1")
    np.testing.assert_allclose(_metric_of(st), A.sum(dim=(0, 1)).numpy(), rtol=1e-12)
    assert abs(_metric_of(st).sum() - r * w) < 1e-9
    # accumulate adds to what is there
    st2 = _one_head_state(K, V, r, b)
    n, o = O.slots_of(st2, 0); st2.metric[n, o] = 1.0
    O.window_metric(st2, Q.reshape(1, 1, r, w, d), w, 1, metric_mode="L1", accumulate=True)
    np.testing.assert_allclose(_metric_of(st2), 1.0 + A.sum(dim=(0, 1)).numpy(), rtol=1e-12)


def test_window_metric_closed_form_and_short_heads():
    r, d, b, C, w = 3, 8, 4, 10, 4
    K = np.tile(np.random.default_rng(0).standard_normal(d), (C, 1))     # identical keys: uniform rows
    st = _one_head_state(K, np.zeros((C, d)), r, b)
    O.window_metric(st, np.ones((1, 1, r, w, d)), w, 1)
    want = np.zeros(C)
    for i in range(w):
        vis = C - w + i + 1
        want[:vis] += r / vis ** 2
    np.testing.assert_allclose(_metric_of(st), want, rtol=1e-12)
    # a head shorter than the window: queries that would sit before position 0 do not exist
    C2 = 3
    st = _one_head_state(K[:C2], np.zeros((C2, d)), r, b)
    O.window_metric(st, np.ones((1, 1, r, w, d)), w, 7)
    want = np.zeros(C2)
    for i in range(w):
        last = C2 - w + i
        if last >= 0:
            want[:last + 1] += r / (last + 1) ** 2
    np.testing.assert_allclose(_metric_of(st), want, rtol=1e-12)


def test_window_metric_equals_one_decode_per_window_query():
    """The same numbers as running the decode once per window query with the context length
    that query sees (how a caller without the window kernel gathers the metric)."""
    shape, ctx, seed = W.small_mixed(5, S=2, Lyr=1, Hk=2, r=2, d=32, L=90, b=4)
    cache = W.make_cache(shape, ctx, seed)
    st = oracle_state(cache); st2 = oracle_state(cache)
    w = 6
    rng = np.random.default_rng(1)
    qw = rng.standard_normal((shape.num_seqs, shape.num_layers, shape.num_q_heads, w, shape.head_dim))
    O.window_metric(st, qw, w, 1)
    lens = st2.lens().copy()
    st2.metric[...] = 0.0
    for i in range(w):
        st2.ctx_len[...] = np.maximum(lens - w + i + 1, 0).reshape(st2.ctx_len.shape)
        O.paged_decode(st2, qw[:, :, :, i, :])
    st2.ctx_len[...] = lens.reshape(st2.ctx_len.shape)
    for g in range(st.G):
        n, o = O.slots_of(st, g)
        np.testing.assert_allclose(st.metric[n, o], st2.metric[n, o], rtol=1e-10, atol=1e-14)


def test_query_blocks_build_the_all_queries_metric_with_excluded_window():
    """Calling the block function over a prompt's queries in blocks gives
    M_full[j] = sum over i >= j + v of A_ij^2 (summed over the group), A the causal attention
    matrix of the prompt, computed here with a library softmax."""
    rng = np.random.default_rng(4)
    r, d, b, L, v, blk = 2, 16, 4, 29, 3, 8
    K = rng.standard_normal((L, d)); Q = rng.standard_normal((r, L, d))
    st = _one_head_state(K, np.zeros((L, d)), r, b)
    for start in range(0, L, blk):
        w = min(blk, L - start)
        O.query_block_metric(st, Q[:, start:start + w].reshape(1, 1, r, w, d), w, start, v)
    scores = torch.from_numpy(np.einsum("hid,jd->hij", Q, K)) / math.sqrt(d)
    i = torch.arange(L).view(1, L, 1); j = torch.arange(L).view(1, 1, L)
    A = torch.softmax(scores.masked_fill(j > i, float("-inf")), dim=-1)
    want = ((A ** 2) * (i >= j + v)).sum(dim=(0, 1)).numpy()
    np.testing.assert_allclose(_metric_of(st), want, rtol=1e-12, atol=1e-15)
    assert (want[L - v:] == 0).all()              # the last v keys have no query far enough away


def test_query_block_past_the_end_of_a_head():
    """Queries that sit at or behind a head's last key (the head kept fewer KVs than the prompt is
    long): each attends to all C keys and adds to key j only when its own position is at least v
    past j — the excluded window is counted from the query, not from the head's end.  Against a
    dense softmax over the C keys, query by query."""
    rng = np.random.default_rng(9)
    r, d, b, C, v, w, start = 2, 16, 4, 21, 5, 6, 18       # positions 18 .. 23, keys 0 .. 20
    K = rng.standard_normal((C, d)); Q = rng.standard_normal((r, w, d))
    st = _one_head_state(K, np.zeros((C, d)), r, b)
    O.query_block_metric(st, Q.reshape(1, 1, r, w, d), w, start, v)
    want = np.zeros(C)
    for h in range(r):
        for i in range(w):
            x = start + i
            seen = min(x, C - 1) + 1
            a = torch.softmax(torch.from_numpy(K[:seen] @ Q[h, i]) / math.sqrt(d), dim=0).numpy()
            for j in range(seen):
                if x - j >= v:
                    want[j] += a[j] ** 2
    np.testing.assert_allclose(_metric_of(st), want, rtol=1e-12, atol=1e-15)
    assert want[C - 1 - (v - (start + w - 1 - (C - 1))) + 1:].sum() == 0     # keys too close to every query
    assert want[C - 3] > 0      # key 18 is 5 behind the last query (position 23): it does get its share


def test_metrics_from_a_given_log_sum_exp():
    """With the log-sum-exp of every query row handed over (what a prefill's attention kernel
    leaves behind), both prefill-end metrics take A_ij = exp(s_ij - lse_i).  Pinned three ways:
    a library logsumexp over the keys each query sees gives back the self-normalised result;
    identical keys give the closed form 1 / (keys seen); and a log-sum-exp that is too large by
    ln 2 halves every probability (the value is used as given, nothing is renormalised)."""
    rng = np.random.default_rng(12)
    r, d, b, C, w, pool = 2, 16, 4, 41, 6, 7
    K = rng.standard_normal((C, d)); Q = rng.standard_normal((r, w, d))
    scores = torch.from_numpy(np.einsum("hwd,cd->hwc", Q, K)) / math.sqrt(d)
    pos = torch.arange(C).view(1, 1, C)
    qpos = (C - w + torch.arange(w)).view(1, w, 1)
    lse = torch.logsumexp(scores.masked_fill(pos > qpos, float("-inf")), dim=-1).numpy()     # [r, w]
    for mode in ("L2", "L1"):
        a = _one_head_state(K, np.zeros((C, d)), r, b)
        c = _one_head_state(K, np.zeros((C, d)), r, b)
        O.window_metric(a, Q.reshape(1, 1, r, w, d), w, pool, metric_mode=mode)
        O.window_metric(c, Q.reshape(1, 1, r, w, d), w, pool, metric_mode=mode, row_lse=lse.reshape(1, 1, r, w))
        np.testing.assert_allclose(_metric_of(c), _metric_of(a), rtol=1e-12, atol=1e-15)
        h = _one_head_state(K, np.zeros((C, d)), r, b)
        O.window_metric(h, Q.reshape(1, 1, r, w, d), w, pool, metric_mode=mode,
                        row_lse=(lse + math.log(2.0)).reshape(1, 1, r, w))
        np.testing.assert_allclose(_metric_of(h), _metric_of(a) * (0.25 if mode == "L2" else 0.5), rtol=1e-12)
    # identical keys: every score of a row is the same number c, lse = c + ln(keys seen), p = 1 / keys seen
    k0 = rng.standard_normal(d)
    Ku = np.tile(k0, (C, 1))
    qv = rng.standard_normal(d)
    c0 = float(k0 @ qv) / math.sqrt(d)
    seen = np.array([C - w + i + 1 for i in range(w)], dtype=np.float64)
    st = _one_head_state(Ku, np.zeros((C, d)), r, b)
    O.window_metric(st, np.tile(qv, (1, 1, r, w, 1)), w, 1, row_lse=np.tile(c0 + np.log(seen), (1, 1, r, 1)))
    want = np.zeros(C)
    for i in range(w):
        want[:int(seen[i])] += r / seen[i] ** 2
    np.testing.assert_allclose(_metric_of(st), want, rtol=1e-12)
    # the block form of the all-queries metric, blocks of 8 queries with an excluded window of 3
    L, v, blk = 29, 3, 8
    K = rng.standard_normal((L, d)); Q = rng.standard_normal((r, L, d))
    sc = torch.from_numpy(np.einsum("hid,jd->hij", Q, K)) / math.sqrt(d)
    i_ = torch.arange(L).view(1, L, 1); j_ = torch.arange(L).view(1, 1, L)
    lse_all = torch.logsumexp(sc.masked_fill(j_ > i_, float("-inf")), dim=-1).numpy()      # [r, L]
    a = _one_head_state(K, np.zeros((L, d)), r, b)
    c = _one_head_state(K, np.zeros((L, d)), r, b)
    for start in range(0, L, blk):
        wq = min(blk, L - start)
        O.query_block_metric(a, Q[:, start:start + wq].reshape(1, 1, r, wq, d), wq, start, v)
        O.query_block_metric(c, Q[:, start:start + wq].reshape(1, 1, r, wq, d), wq, start, v,
                             row_lse=lse_all[:, start:start + wq].reshape(1, 1, r, wq))
    np.testing.assert_allclose(_metric_of(c), _metric_of(a), rtol=1e-12, atol=1e-15)
    assert _metric_of(a).sum() > 0
