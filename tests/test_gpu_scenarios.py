"""Scaled-down versions of the other benchmark configurations, every step compared with the
oracle: periodic eviction inside a decode loop at high compression, prefill-end compression
from an observation window, and the group-of-8 shape."""
import numpy as np
import pytest
import torch

from oracle import kvc_oracle as O
from paper_2410_00161_amd import binding as B
from paper_2410_00161_amd import workloads as W
from helpers import oracle_state, check_allocator_invariants, assert_keys_equal
from test_gpu_parity import session, say, assert_state_equal, TOL

pytestmark = pytest.mark.gpu


def evict_round(sess, st, frac, mode):
    """One compression round on both sides, the oracle ranking the device's metric."""
    torch.cuda.synchronize()
    st.metric = sess.cache.metric.cpu().numpy().astype(np.float64)   # identical metric inputs
    nb = -(-st.lens() // st.b)
    budget = torch.tensor((nb.reshape(st.S, -1).sum(1) * frac).astype(np.int64), dtype=torch.int32)
    if mode == "block":
        key = sess.metric_reduce()
        want_key, _ = O.block_keys(st)
        assert_keys_equal(key, want_key, st)
        flag_w, count_w, sel_w = O.evict_select(st, want_key, budget.numpy())
        flag, count, sel = sess.evict_select(budget)
        np.testing.assert_array_equal(flag.cpu().numpy(), flag_w)
        freed_w = O.compact(st, flag_w, count_w)
        freed = int(sess.compact().item())
    else:
        rows_w, masks_w, sel_w = O.rank_schedule(st, budget.numpy())
        rows, sel = sess.evict_rank_select(budget)
        np.testing.assert_array_equal(rows.cpu().numpy(), rows_w)
        freed_w = O.compact_slots(st, masks_w)
        freed = int(sess.compact_rank().item())
    np.testing.assert_array_equal(sel.cpu().numpy(), sel_w)
    assert freed == freed_w
    return freed


@pytest.mark.parametrize("mode", ["block", "rank"])
def test_periodic_eviction_in_a_decode_loop_at_high_compression(mode):
    """Many short, unevenly compressed heads; every 4th step the cheapest 10 % of each
    sequence's blocks go and the cache is compacted into the freed blocks."""
    say("periodic eviction", mode)
    shape, ctx, seed = W.small_mixed(91, S=6, Lyr=2, Hk=4, r=4, d=128, L=2048, rho=32.0, extra_blocks=3)
    cache = W.make_cache(shape, ctx, seed, placement="fragmented", init_metric="prefill")
    st = oracle_state(cache)
    sess = session(cache)
    total_freed = 0
    for step in range(12):
        k, v = W.make_new_kv(shape, seed, step)
        q = W.make_query(shape, seed, step)
        O.append(st, k.double().numpy(), v.double().numpy())
        want = O.paged_decode(st, q.double().numpy())
        sess.append(k.to(sess.device), v.to(sess.device))
        out = sess.paged_decode(q.to(sess.device))
        torch.cuda.synchronize()
        np.testing.assert_allclose(out.cpu().numpy(), want, rtol=0, atol=TOL)
        np.testing.assert_allclose(sess.cache.metric.cpu().numpy()[st.free_map == 0],
                                   st.metric[st.free_map == 0], rtol=0, atol=TOL)
        if (step + 1) % 4 == 0:
            total_freed += evict_round(sess, st, 0.10, mode)
            assert_state_equal(sess, st)
            check_allocator_invariants(st)
    assert total_freed > 0


def test_prefill_end_compression_from_an_observation_window():
    """A full-length prompt; the metric is the squared attention of the last w prompt queries
    (query i sees keys 0 .. L-w+i), gathered by running the decode once per window query with
    the context lengths set accordingly; then eviction to 8x and a few decode steps."""
    say("observation window -> 8x")
    S, Lyr, Hk, r, d, b, L, w = 1, 4, 2, 4, 128, 16, 768, 8
    ctx = W.uniform_lengths(S * Lyr * Hk, L)
    N = W.pool_size(ctx, b, 1.2, 16)
    shape = W.Shape(S, Lyr, Hk, r, d, b, N, L // b + 2, "bf16")
    cache = W.make_cache(shape, ctx, 95)
    st = oracle_state(cache)
    sess = session(cache)
    for i in range(w):
        seen = L - w + i + 1
        st.ctx_len[...] = seen
        sess.cache.ctx_len.fill_(seen)
        q = W.make_query(shape, 95, i)
        want = O.paged_decode(st, q.double().numpy())
        out = sess.paged_decode(q.to(sess.device))
        torch.cuda.synchronize()
        np.testing.assert_allclose(out.cpu().numpy(), want, rtol=0, atol=TOL)
    # the window metric equals the column sums of the w x L squared attention matrix
    np.testing.assert_allclose(sess.cache.metric.cpu().numpy(), st.metric, rtol=0, atol=TOL)
    g0 = 3
    n, o = O.slots_of(st, g0)
    assert (st.metric[n, o][-1] > 0) and st.metric[n, o][: L - w].min() >= 0
    for mode in ("block",):
        freed = evict_round(sess, st, 7.0 / 8.0, mode)
        assert freed > 0
    assert_state_equal(sess, st)
    kept = st.lens().sum()
    assert kept <= L * S * Lyr * Hk / 8 + S * Lyr * Hk * b * 2     # about 8x, up to block rounding
    assert len(set(st.lens().tolist())) > 1                         # rates differ per head
    for step in range(6):
        k, v = W.make_new_kv(shape, 95, 100 + step)
        q = W.make_query(shape, 95, 100 + step)
        O.append(st, k.double().numpy(), v.double().numpy())
        want = O.paged_decode(st, q.double().numpy())
        sess.append(k.to(sess.device), v.to(sess.device))
        out = sess.paged_decode(q.to(sess.device))
        torch.cuda.synchronize()
        np.testing.assert_allclose(out.cpu().numpy(), want, rtol=0, atol=TOL)
    assert_state_equal(sess, st)


def test_state_check_passes_what_the_library_leaves_and_names_what_is_broken():
    """kvc_check_state after appends and a compression round of each kind (the library's own
    calls keep a state consistent), then one planted inconsistency at a time: each is refused
    with KVC_ERR_ARG, nothing is modified, and the repaired state passes again."""
    say("state check")
    shape, ctx, seed = W.small_mixed(97, S=2, Lyr=2, Hk=2, r=2, d=64, b=16, L=300, rho=2.0, kv_dtype="bf16")
    ctx[1] = 0
    cache = W.make_cache(shape, ctx, seed, placement="fragmented", init_metric="prefill")
    st = oracle_state(cache)
    sess = session(cache)
    sess.check_state()
    for step in range(3):
        k, v = W.make_new_kv(shape, seed, step)
        O.append(st, k.double().numpy(), v.double().numpy())
        sess.append(k.to(sess.device), v.to(sess.device))
        sess.paged_decode(W.make_query(shape, seed, step).to(sess.device))
    sess.check_state()
    for mode in ("block", "rank"):
        evict_round(sess, st, 0.3, mode)
        sess.check_state()
    c = sess.cache
    table, lens, fmap = c.block_table.view(shape.G, -1), c.ctx_len.view(-1), c.free_map
    g = 3                                            # a head with several blocks
    held = int((table[g] >= 0).sum())
    assert held >= 3
    free_id = int(torch.nonzero(fmap == 1)[0])
    plants = {
        "length past the blocks held": lambda: lens.__setitem__(g, held * shape.block_size + 1),
        "negative length": lambda: lens.__setitem__(g, -1),
        "block id past the pool": lambda: table.__setitem__((g, 1), shape.num_blocks),
        "negative block id": lambda: table.__setitem__((g, 1), -7),
        "a hole in the row": lambda: table.__setitem__((g, 0), -1),
        "a block held by two heads": lambda: table.__setitem__((g, 1), int(table[g + 1, 0])),
        "a held block marked free": lambda: fmap.__setitem__(int(table[g, 2]), 1),
        "an id behind the end of the row": lambda: table.__setitem__((g, shape.max_blocks_per_head - 1), free_id),
    }
    for what, plant in plants.items():
        keep = (table.clone(), lens.clone(), fmap.clone())
        plant()
        broken = (table.clone(), lens.clone(), fmap.clone())
        with pytest.raises(B.KvcError) as e:
            sess.check_state()
        assert e.value.code == B.KVC_ERR_ARG, what
        for now, was in zip((table, lens, fmap), broken):     # the check reads only
            assert torch.equal(now, was), what
        table.copy_(keep[0]); lens.copy_(keep[1]); fmap.copy_(keep[2])
        sess.check_state()
    assert_state_equal(sess, st)
    # the asynchronous form leaves its verdict in the status word
    lens[g] = -1
    sess.check_state(flags=B.KVC_ASYNC)
    assert B.kvc_poll_status(sess.cfg, sess.ws) == B.KVC_ERR_ARG
    lens[g] = int(st.ctx_len.reshape(-1)[g])
    B.kvc_workspace_reset(sess.cfg, sess.ws)
    sess.check_state()


def _round_matrix():
    cases, i = [], 0
    for b in (1, 2, 4, 8, 16, 32, 64):
        for dt in ("bf16", "f32", "fp8"):
            d, r = ((64, 2), (128, 4), (128, 8), (64, 1))[i % 4]
            i += 1
            cases.append((f"b{b}_{dt}_d{d}_r{r}", dict(b=b, kv_dtype=dt, d=d, r=r)))
    return cases


ROUND_MATRIX = _round_matrix()


@pytest.mark.parametrize("name,kw", ROUND_MATRIX, ids=[c[0] for c in ROUND_MATRIX])
def test_compression_rounds_over_block_sizes_and_row_types(name, kw):
    """Append + decode, a physical-block round, append + decode, a rank-block round, decode:
    every block size from 1 to 64 tokens with every row type."""
    say("rounds over shapes", name)
    L = 40 * max(kw["b"], 4)
    shape, ctx, seed = W.small_mixed(131, S=3, Lyr=2, Hk=2, L=L, rho=2.0, extra_blocks=3, **kw)
    cache = W.make_cache(shape, ctx, seed, placement="fragmented", init_metric="prefill")
    st = oracle_state(cache)
    sess = session(cache)
    for step, mode in enumerate(("block", "rank", None)):
        k, v = W.make_new_kv(shape, seed, step)
        q = W.make_query(shape, seed, step)
        O.append(st, k.double().numpy(), v.double().numpy())
        want = O.paged_decode(st, q.double().numpy())
        sess.append(k.to(sess.device), v.to(sess.device))
        out = sess.paged_decode(q.to(sess.device))
        torch.cuda.synchronize()
        np.testing.assert_allclose(out.cpu().numpy(), want, rtol=0, atol=TOL)
        if mode:
            freed = evict_round(sess, st, 0.3, mode)
            assert freed > 0
            assert_state_equal(sess, st)
            check_allocator_invariants(st)


def test_group_of_eight_shape_with_long_heads():
    """70B-like grouping (8 query heads per KV head) with heads long enough to be split into
    several chunks at the default chunk length, then a rank-block round."""
    say("r = 8, long heads")
    shape, ctx, seed = W.small_mixed(97, S=2, Lyr=2, Hk=2, r=8, d=128, L=6000, rho=2.0, extra_blocks=2)
    cache = W.make_cache(shape, ctx, seed, placement="fragmented", init_metric="prefill")
    st = oracle_state(cache)
    sess = session(cache)
    assert int(ctx.max()) > B.kvc_get_decode_chunk(sess.cfg) > 0
    for step in range(2):
        k, v = W.make_new_kv(shape, seed, step)
        q = W.make_query(shape, seed, step)
        O.append(st, k.double().numpy(), v.double().numpy())
        want = O.paged_decode(st, q.double().numpy())
        sess.append(k.to(sess.device), v.to(sess.device))
        out = sess.paged_decode(q.to(sess.device))
        torch.cuda.synchronize()
        np.testing.assert_allclose(out.cpu().numpy(), want, rtol=0, atol=TOL)
    np.testing.assert_allclose(sess.cache.metric.cpu().numpy()[st.free_map == 0],
                               st.metric[st.free_map == 0], rtol=0, atol=TOL)
    evict_round(sess, st, 0.25, "rank")
    assert_state_equal(sess, st)


def test_append_and_decode_replay_from_a_hip_graph():
    """The asynchronous entry points hold no host synchronisation and no memset nodes, so a
    caller can capture append + decode into a HIP graph; every replay is checked against the
    oracle taking the same step, with eager work and synchronisations between replays."""
    say("graph capture of append + decode")
    shape, ctx, seed = W.small_mixed(111, S=2, Lyr=2, Hk=2, r=4, d=128, L=5000, rho=3.0, extra_blocks=3)
    cache = W.make_cache(shape, ctx, seed, placement="fragmented", init_metric="prefill")
    st = oracle_state(cache)
    sess = session(cache)
    k, v = W.make_new_kv(shape, seed, 0)
    q = W.make_query(shape, seed, 0)
    kd, vd, qd = k.to(sess.device), v.to(sess.device), q.to(sess.device)

    def oracle_step():
        O.append(st, k.double().numpy(), v.double().numpy())
        return O.paged_decode(st, q.double().numpy())

    # one eager step first (also warms up everything the capture must not do for the first time)
    want = oracle_step()
    sess.append(kd, vd, flags=B.KVC_ASYNC)
    sess.paged_decode(qd)
    torch.cuda.synchronize()
    np.testing.assert_allclose(sess.out.cpu().numpy(), want, rtol=0, atol=TOL)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        sess.append(kd, vd, flags=B.KVC_ASYNC)
        sess.paged_decode(qd)
    torch.cuda.synchronize()
    for rep in range(4):
        want = oracle_step()
        graph.replay()
        torch.cuda.synchronize()
        np.testing.assert_allclose(sess.out.cpu().numpy(), want, rtol=0, atol=TOL)
        scratch = torch.randn(1 << 16, device=sess.device).sum().item()   # eager work in between
        assert np.isfinite(scratch)
    assert B.kvc_poll_status(sess.cfg, sess.ws) == B.KVC_OK
    assert_state_equal(sess, st)


def test_compression_round_replays_from_a_hip_graph():
    """A compression round (block keys, selection, compaction) issued with KVC_ASYNC holds no host
    synchronisation either: captured once, replayed after further decode steps, every replay checked
    against the oracle's round on the same metrics."""
    say("graph capture of a compression round")
    shape, ctx, seed = W.small_mixed(131, S=3, Lyr=2, Hk=2, r=4, d=128, L=1500, rho=2.0, extra_blocks=6)
    cache = W.make_cache(shape, ctx, seed, placement="fragmented", init_metric="prefill")
    st = oracle_state(cache)
    sess = session(cache)
    budget = torch.tensor([5, 0, 9], dtype=torch.int32)
    budget_dev = budget.to(sess.device)

    def decode_steps(first, n):
        for i in range(first, first + n):
            k, v = W.make_new_kv(shape, seed, i)
            q = W.make_query(shape, seed, i)
            O.append(st, k.double().numpy(), v.double().numpy())
            want = O.paged_decode(st, q.double().numpy())
            sess.append(k.to(sess.device), v.to(sess.device))
            out = sess.paged_decode(q.to(sess.device))
            torch.cuda.synchronize()
            np.testing.assert_allclose(out.cpu().numpy(), want, rtol=0, atol=TOL)

    def oracle_round():
        torch.cuda.synchronize()
        st.metric = sess.cache.metric.cpu().numpy().astype(np.float64)   # identical metric inputs
        want_key, _ = O.block_keys(st)
        flag_w, count_w, sel_w = O.evict_select(st, want_key, budget.numpy())
        return flag_w, count_w, sel_w, O.compact(st, flag_w, count_w)

    def device_round():
        sess.metric_reduce()
        _, _, sel = sess.evict_select(budget_dev, flags=B.KVC_ASYNC)
        return sel, sess.compact(flags=B.KVC_ASYNC)

    decode_steps(0, 2)
    flag_w, count_w, sel_w, freed_w = oracle_round()
    sel, freed = device_round()          # eager once: whatever a first call sets up happens outside the capture
    torch.cuda.synchronize()
    np.testing.assert_array_equal(sel.cpu().numpy(), sel_w)
    assert int(freed.item()) == freed_w
    assert_state_equal(sess, st)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        sel, freed = device_round()
    torch.cuda.synchronize()
    for rep in range(3):
        decode_steps(2 + 3 * rep, 3)
        flag_w, count_w, sel_w, freed_w = oracle_round()
        graph.replay()
        torch.cuda.synchronize()
        np.testing.assert_array_equal(sess.evict_flag.cpu().numpy(), flag_w)
        np.testing.assert_array_equal(sess.evict_count.cpu().numpy(), count_w)
        np.testing.assert_array_equal(sel.cpu().numpy(), sel_w)
        assert int(freed.item()) == freed_w == int(sel_w.sum())
        assert_state_equal(sess, st)
        scratch = torch.randn(1 << 16, device=sess.device).sum().item()   # eager work in between
        assert np.isfinite(scratch)
    assert B.kvc_poll_status(sess.cfg, sess.ws) == B.KVC_OK
    check_allocator_invariants(st)


def test_snapshot_of_the_six_buffers_resumes_bit_for_bit():
    """The whole state of a cache is its plain buffers (keys, values, metrics, logical indices,
    tables, lengths, free map); the workspace holds nothing between calls.  A copy of them taken in
    the middle of a run, put into a new session with a new workspace, continues exactly as the
    original does: same outputs, same metrics, same tables after decode steps and both kinds of round."""
    from paper_2410_00161_amd.session import KvcSession
    print("[case] snapshot / resume", flush=True)
    shape, ctx, seed = W.small_mixed(311, S=3, Lyr=2, Hk=2, r=4, d=128, L=900, rho=2.0, extra_blocks=4)
    a = KvcSession(W.make_cache(shape, ctx, seed, placement="fragmented", init_metric="prefill"))

    def steps(sess, first, n, outs):
        for i in range(first, first + n):
            k, v = W.make_new_kv(shape, seed, i, sess.device)
            sess.append(k, v)
            outs.append(sess.paged_decode(W.make_query(shape, seed, i, sess.device)).clone())

    def round_(sess, rank):
        nb = (sess.cache.ctx_len.reshape(shape.num_seqs, -1).long() + shape.block_size - 1) // shape.block_size
        bud = (nb.sum(1) // 5).to(torch.int32)
        if rank:
            sess.evict_rank_select(bud)
            return int(sess.compact_rank().item())
        sess.metric_reduce()
        sess.evict_select(bud)
        return int(sess.compact().item())

    warm = []
    steps(a, 0, 5, warm)
    assert round_(a, False) > 0
    snap = a.cache.clone().to("cpu")                     # the snapshot: six buffers (and pos), nothing else
    b = KvcSession(snap)                                 # new tensors, new workspace
    out_a, out_b = [], []
    for sess, outs in ((a, out_a), (b, out_b)):
        steps(sess, 5, 7, outs)
        outs.append(torch.tensor(round_(sess, True)))
        steps(sess, 12, 3, outs)
        outs.append(torch.tensor(round_(sess, False)))
    torch.cuda.synchronize()
    for x, y in zip(out_a, out_b):
        assert torch.equal(x.cpu(), y.cpu())
    for name in ("k_cache", "v_cache", "metric", "pos", "block_table", "ctx_len", "free_map"):
        ta, tb = getattr(a.cache, name), getattr(b.cache, name)
        if ta.dtype == torch.float8_e4m3fn:
            ta, tb = ta.view(torch.uint8), tb.view(torch.uint8)
        assert torch.equal(ta.cpu(), tb.cpu()), name
    a.check_state()


def test_read_probes_read_and_add_what_they_say():
    """The bench's bandwidth probes: the checksum of the bytes read is the XOR of all of them (so every
    byte was read once), and the adds land once per 512 bytes read, nowhere else."""
    say("read probes")
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev).manual_seed(3)
    nbytes, item = 9 << 20, 1 << 20
    src = torch.randint(0, 2 ** 31 - 1, (nbytes // 4,), generator=g, device=dev, dtype=torch.int32)
    want = 0
    for w in src.cpu().numpy().view(np.uint32).reshape(-1, 1 << 16):
        want ^= int(np.bitwise_xor.reduce(w))
    for wgs in (7, 512):
        sink = torch.zeros(wgs, dtype=torch.int32, device=dev)
        B.kvc_stream_read_probe(src, nbytes, sink, wgs)
        got = int(np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint32)))
        assert got == want
        for adds in (0, 1):
            dst = torch.zeros(nbytes // 512 + 100, dtype=torch.float32, device=dev)
            sink.zero_()
            B.kvc_stream_read_add_probe(src, nbytes, item, adds, dst, sink, wgs)
            torch.cuda.synchronize()
            assert int(np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint32))) == want
            d = dst.cpu().numpy()
            assert (d[: nbytes // 512] == float(adds)).all() and (d[nbytes // 512:] == 0).all()
