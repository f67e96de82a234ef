"""Parity at the benchmark's full size (Llama-3.1-8B-shaped decode, 64 x 8192 prompt tokens,
mean 8x compression) in the launch configuration bench.py times: sampled head instances are
copied back and recomputed by the oracle one by one; whole-tensor properties are checked on
the device."""
import numpy as np
import pytest
import torch

from oracle import kvc_oracle as O
from paper_2410_00161_amd import binding as B
from paper_2410_00161_amd import workloads as W
from helpers import oracle_state, assert_keys_equal

pytestmark = pytest.mark.gpu
TOL = 2e-3


def pick_heads(ctx, chunk, n_random, seed):
    """Longest, shortest, the ones around the chunk boundary, and a random draw."""
    c = ctx.reshape(-1).cpu()
    order = torch.argsort(c)
    picks = set(order[:4].tolist()) | set(order[-4:].tolist())
    near = torch.argsort((c - chunk).abs())[:6].tolist()
    picks |= set(near)
    g = torch.Generator().manual_seed(seed)
    picks |= set(torch.randperm(c.numel(), generator=g)[:n_random].tolist())
    return sorted(picks)


@pytest.fixture
def forced_chunk(request):
    """0 = the library's own choice (what bench.py times); otherwise a shorter chunk so that long
    heads are split over several workgroups and finished by the combine kernel."""
    B.kvc_set_decode_chunk(request.param)
    yield request.param
    B.kvc_set_decode_chunk(0)


# (sequences, prompt tokens, mean compression): the benchmark's configuration, and the high
# compression one (256 long prompts kept at 1/64: mostly short heads, 17 GB of K and V)
FULL_SIZES = [(64, 8192, 8.0, 0), (64, 8192, 8.0, 2048), (256, 32768, 64.0, 0)]


@pytest.mark.parametrize("num_seqs,prompt,rho,forced_chunk", FULL_SIZES, indirect=["forced_chunk"],
                         ids=["8x", "8x_chunk2048", "64x"])
def test_llama8b_shape_sampled_parity_and_invariants(num_seqs, prompt, rho, forced_chunk):
    from paper_2410_00161_amd.session import KvcSession
    print(f"[case] full-size llama8b decode + eviction, {num_seqs} x {prompt} at {rho:g}x, "
          f"chunk setting {forced_chunk}", flush=True)
    shape, ctx, seed = W.llama8b_decode(num_seqs=num_seqs, prompt=prompt, rho=rho, extra_tokens=64)
    dev = torch.device("cuda:0")
    cache = W.make_cache(shape, ctx, seed, device=dev, placement="fragmented", init_metric="prefill")
    sess = KvcSession(cache, device=dev)
    del cache
    chunk = B.kvc_get_decode_chunk(sess.cfg)
    assert chunk > 0
    G, r, d, b = shape.G, shape.group_size, shape.head_dim, shape.block_size
    k, v = W.make_new_kv(shape, seed, 0, dev)
    q = W.make_query(shape, seed, 0, dev)
    free0 = int(sess.cache.free_map.sum())
    crossing = int((sess.cache.ctx_len.reshape(-1) % b == 0).sum())
    sess.append(k, v)
    assert free0 - int(sess.cache.free_map.sum()) == crossing
    heads = pick_heads(sess.cache.ctx_len, chunk, 40, seed)
    if int(sess.cache.ctx_len.max()) > chunk:      # then a split head is in the sample
        assert any(int(sess.cache.ctx_len.reshape(-1)[g]) > chunk for g in heads)
    assert forced_chunk == 0 or int(sess.cache.ctx_len.max()) > 2 * chunk
    small, q_small = W.gather_heads(sess.cache, heads, q)
    st = oracle_state(small)
    m_before = sess.cache.metric.clone()
    out = sess.paged_decode(q)
    torch.cuda.synchronize()
    want = O.paged_decode(st, q_small.double().numpy())
    got = out.reshape(G, r, d)[torch.tensor(heads, device=dev)].cpu().numpy()
    np.testing.assert_allclose(got, want.reshape(len(heads), r, d), rtol=0, atol=TOL)
    after, _ = W.gather_heads(sess.cache, heads)
    for i in range(len(heads)):
        n, o = O.slots_of(st, i)
        np.testing.assert_allclose(after.metric.numpy()[n, o], st.metric[n, o], rtol=0, atol=TOL)
    # properties over the whole tensor: every head's increments sum to between r / C and r,
    # no slot lost metric, slots that hold no KV did not change
    delta = (sess.cache.metric - m_before).double()
    assert float(delta.min()) >= 0.0
    table = sess.cache.block_table.reshape(G, -1).long()
    ctx_now = sess.cache.ctx_len.reshape(G).long()
    owner = torch.full((shape.num_blocks,), G, dtype=torch.long, device=dev)
    valid = table >= 0
    owner[table[valid]] = torch.arange(G, device=dev).unsqueeze(1).expand_as(table)[valid]
    per_head = torch.zeros(G + 1, dtype=torch.float64, device=dev)
    per_head.index_add_(0, owner, delta.sum(1))
    ph = per_head[:G]
    assert bool((ph <= r + 1e-3).all()) and bool((ph >= r / ctx_now.double() - 1e-3).all())
    assert float(per_head[G]) == 0.0                       # blocks nobody owns were not touched
    assert bool(torch.isfinite(out).all())

    # compression round: 10 % of every sequence's blocks
    key = sess.metric_reduce()
    nb = (ctx_now + b - 1) // b
    per_seq = nb.reshape(shape.num_seqs, -1).sum(1)
    budget = (per_seq // 10).to(torch.int32)
    flag, count, sel = sess.evict_select(budget)
    torch.cuda.synchronize()
    assert torch.equal(sel.cpu(), budget.cpu())
    assert int(count.sum()) == int(budget.sum()) == int(flag.sum())
    # selection parity on sampled sequences: the oracle ranks the same keys
    key_h = key.cpu().numpy()
    for s in (0, 17, shape.num_seqs - 1):
        lo, hi = s * shape.num_layers * shape.num_kv_heads, (s + 1) * shape.num_layers * shape.num_kv_heads
        mini = O.State(1, shape.num_layers, shape.num_kv_heads, 1, 1, b, 1, shape.max_blocks_per_head,
                       np.zeros((1, b, 1)), np.zeros((1, b, 1)), np.zeros((1, b)), np.zeros((1, b)),
                       np.zeros((hi - lo, shape.max_blocks_per_head)), ctx_now[lo:hi].cpu().numpy(),
                       np.zeros(1, dtype=np.uint8))
        fw, cw, sw = O.evict_select(mini, key_h[lo:hi], [int(budget[s])])
        np.testing.assert_array_equal(flag[lo:hi].cpu().numpy(), fw)
        np.testing.assert_array_equal(count[lo:hi].cpu().numpy(), cw)
    # block keys of the sampled heads, bit for bit
    st_after = oracle_state(after)
    kw, _ = O.block_keys(st_after)
    assert_keys_equal(key_h[heads], kw, st_after)
    # compaction parity on the sampled heads, given the device's flags
    st2 = oracle_state(after)
    f_small = flag[torch.tensor(heads, device=dev)].cpu().numpy()
    free_before = int(sess.cache.free_map.sum())
    freed = int(sess.compact().item())
    assert freed == int(budget.sum())
    assert int(sess.cache.free_map.sum()) - free_before == freed       # whole blocks returned
    O.compact(st2, f_small)
    post, _ = W.gather_heads(sess.cache, heads)
    np.testing.assert_array_equal(post.ctx_len.reshape(-1).numpy(), st2.lens())
    stp = oracle_state(post)   # blocks renumbered: compare head by head in logical order
    for i in range(len(heads)):
        n, o = O.slots_of(st2, i)
        n2, o2 = O.slots_of(stp, i)
        np.testing.assert_array_equal(stp.k_cache[n2, o2], st2.k_cache[n, o])
        np.testing.assert_array_equal(stp.v_cache[n2, o2], st2.v_cache[n, o])
        np.testing.assert_array_equal(stp.metric[n2, o2], st2.metric[n, o])
        np.testing.assert_array_equal(stp.pos[n2, o2], st2.pos[n, o])
    # allocator invariants over the whole pool
    table = sess.cache.block_table.reshape(G, -1).long()
    ctx_now = sess.cache.ctx_len.reshape(G).long()
    held = (table >= 0).sum(1)
    assert torch.equal(held, (ctx_now + b - 1) // b)
    ids = table[table >= 0]
    assert ids.numel() == torch.unique(ids).numel()
    assert int((sess.cache.free_map == 0).sum()) == ids.numel()
    assert int(sess.cache.free_map[ids].sum()) == 0


def test_llama8b_shape_rank_schedule_on_one_sequence():
    """The rank-block schedule at full size; one whole sequence (256 head instances) is copied
    back and scheduled by the oracle from the same metrics."""
    from paper_2410_00161_amd.session import KvcSession
    print("[case] full-size llama8b rank-block eviction", flush=True)
    shape, ctx, seed = W.llama8b_decode(extra_tokens=64)
    dev = torch.device("cuda:0")
    cache = W.make_cache(shape, ctx, seed, device=dev, placement="fragmented", init_metric="prefill")
    sess = KvcSession(cache, device=dev)
    del cache
    G, b = shape.G, shape.block_size
    per = shape.num_layers * shape.num_kv_heads
    q = W.make_query(shape, seed, 0, dev)
    sess.paged_decode(q)                                   # metrics as a decode step leaves them
    ctx_now = sess.cache.ctx_len.reshape(G).long()
    nb = (ctx_now + b - 1) // b
    budget = (nb.reshape(shape.num_seqs, -1).sum(1) // 8).to(torch.int32)
    s = 11
    heads = list(range(s * per, (s + 1) * per))
    small, _ = W.gather_heads(sess.cache, heads)
    one = oracle_state(small)
    st = O.State(1, shape.num_layers, shape.num_kv_heads, shape.group_size, shape.head_dim, b, one.N,
                 one.max_blocks, one.k_cache, one.v_cache, one.metric, one.pos, one.block_table, one.ctx_len,
                 one.free_map)
    rows, sel = sess.evict_rank_select(budget)
    torch.cuda.synchronize()
    assert torch.equal(sel.cpu(), budget.cpu()) and int(rows.sum()) == int(budget.sum())
    rows_w, masks_w, sel_w = O.rank_schedule(st, [int(budget[s])], metric=small.metric.numpy())
    np.testing.assert_array_equal(rows[s * per:(s + 1) * per].cpu().numpy(), rows_w)
    free_before = int(sess.cache.free_map.sum())
    freed = int(sess.compact_rank().item())
    assert freed == int(budget.sum()) == int(sess.cache.free_map.sum()) - free_before
    O.compact_slots(st, masks_w)
    post, _ = W.gather_heads(sess.cache, heads)
    stp = oracle_state(post)
    np.testing.assert_array_equal(stp.lens(), st.lens())
    for i in range(len(heads)):
        n, o = O.slots_of(st, i)
        n2, o2 = O.slots_of(stp, i)
        np.testing.assert_array_equal(stp.k_cache[n2, o2], st.k_cache[n, o])
        np.testing.assert_array_equal(stp.metric[n2, o2], st.metric[n, o])
        np.testing.assert_array_equal(stp.pos[n2, o2], st.pos[n, o])
    ctx_after = sess.cache.ctx_len.reshape(G).long()
    changed = rows.long() > 0
    assert bool((ctx_after[changed] % b == 0).all())        # heads that lost rows end on whole blocks
    assert torch.equal((ctx_after + b - 1) // b, nb - rows.long())


@pytest.mark.parametrize("forced_chunk", [0, 1024], indirect=True)
def test_llama70b_shape_long_heads_sampled(forced_chunk):
    """One sequence of the 70B shape (80 layers x 8 KV heads, groups of 8 query heads, 131072
    prompt tokens, mean 8x): heads of up to 131 K tokens are split into 52 chunks at the default
    chunk length and into 128 with the forced one, past what the combine kernel keeps in LDS.
    The longest, the shortest and a few random head instances are recomputed by the oracle."""
    from paper_2410_00161_amd.session import KvcSession
    print(f"[case] llama70b shape, one sequence, chunk setting {forced_chunk}", flush=True)
    shape, ctx, seed = W.llama70b_decode(num_seqs=1, extra_tokens=32)
    ctx[5] = 131072                         # a head that kept everything
    dev = torch.device("cuda:0")
    cache = W.make_cache(shape, ctx, seed, device=dev, placement="fragmented", init_metric="prefill")
    sess = KvcSession(cache, device=dev)
    del cache
    chunk = B.kvc_get_decode_chunk(sess.cfg)
    G, r, d = shape.G, shape.group_size, shape.head_dim
    assert int(sess.cache.ctx_len.max()) >= 32 * chunk    # dozens of chunks per head either way
    c = sess.cache.ctx_len.reshape(-1).cpu()
    order = torch.argsort(c)
    g0 = torch.Generator().manual_seed(seed)
    heads = sorted(set([5] + order[:2].tolist() + order[-2:].tolist() +
                       torch.randperm(G, generator=g0)[:6].tolist()))
    q = W.make_query(shape, seed, 0, dev)
    small, q_small = W.gather_heads(sess.cache, heads, q)
    st = oracle_state(small)
    m_before = sess.cache.metric.clone()
    out = sess.paged_decode(q)
    torch.cuda.synchronize()
    want = O.paged_decode(st, q_small.double().numpy())
    got = out.reshape(G, r, d)[torch.tensor(heads, device=dev)].cpu().numpy()
    np.testing.assert_allclose(got, want.reshape(len(heads), r, d), rtol=0, atol=TOL)
    after, _ = W.gather_heads(sess.cache, heads)
    for i in range(len(heads)):
        n, o = O.slots_of(st, i)
        np.testing.assert_allclose(after.metric.numpy()[n, o], st.metric[n, o], rtol=0, atol=TOL)
    # every head's increments sum to between r / C and r; nothing lost metric
    delta = (sess.cache.metric - m_before).double()
    assert float(delta.min()) >= 0.0
    table = sess.cache.block_table.reshape(G, -1).long()
    owner = torch.full((shape.num_blocks,), G, dtype=torch.long, device=dev)
    valid = table >= 0
    owner[table[valid]] = torch.arange(G, device=dev).unsqueeze(1).expand_as(table)[valid]
    per_head = torch.zeros(G + 1, dtype=torch.float64, device=dev)
    per_head.index_add_(0, owner, delta.sum(1))
    ctx_now = sess.cache.ctx_len.reshape(G).double()
    assert bool((per_head[:G] <= r + 1e-3).all()) and bool((per_head[:G] >= r / ctx_now - 1e-3).all())
    assert float(per_head[G]) == 0.0
    assert bool(torch.isfinite(out).all())


def test_llama70b_full_batch_sampled_with_both_kinds_of_round():
    """The whole 70B-shaped batch the benchmark runs (16 sequences x 131072 prompt tokens, mean 8x:
    10240 head instances, 86 GB of keys and values): append + decode checked on sampled head
    instances and by per-head properties over the whole cache; then a rank-block round and a block
    round of a tenth of every sequence's blocks, each with its selection recomputed by the oracle
    for the head instances of one layer of one sequence (given the device's metrics / keys) and
    the compacted heads compared slot by slot; allocator invariants on the device after each."""
    from paper_2410_00161_amd.session import KvcSession
    print("[case] llama70b shape, full batch of 16 x 131072", flush=True)
    shape, ctx, seed = W.llama70b_decode(extra_tokens=48)
    dev = torch.device("cuda:0")
    free_b, _ = torch.cuda.mem_get_info()
    if free_b < 150 * (1 << 30):
        pytest.skip("needs 150 GB of free device memory")
    cache = W.make_cache(shape, ctx, seed, device=dev, placement="fragmented", init_metric="prefill")
    sess = KvcSession(cache, device=dev)
    del cache
    G, r, d, b = shape.G, shape.group_size, shape.head_dim, shape.block_size
    chunk = B.kvc_get_decode_chunk(sess.cfg)
    k, v = W.make_new_kv(shape, seed, 0, dev)
    q = W.make_query(shape, seed, 0, dev)
    sess.append(k, v)
    heads = pick_heads(sess.cache.ctx_len, chunk, 8, seed)
    small, q_small = W.gather_heads(sess.cache, heads, q)
    st = oracle_state(small)
    m_before = sess.cache.metric.clone()
    out = sess.paged_decode(q)
    torch.cuda.synchronize()
    want = O.paged_decode(st, q_small.double().numpy())
    got = out.reshape(G, r, d)[torch.tensor(heads, device=dev)].cpu().numpy()
    np.testing.assert_allclose(got, want.reshape(len(heads), r, d), rtol=0, atol=TOL)
    after, _ = W.gather_heads(sess.cache, heads)
    for i in range(len(heads)):
        n, o = O.slots_of(st, i)
        np.testing.assert_allclose(after.metric.numpy()[n, o], st.metric[n, o], rtol=0, atol=TOL)
    del st, small, after
    delta = sess.cache.metric - m_before
    del m_before
    assert float(delta.min()) >= 0.0
    table = sess.cache.block_table.reshape(G, -1).long()
    owner = torch.full((shape.num_blocks,), G, dtype=torch.long, device=dev)
    valid = table >= 0
    owner[table[valid]] = torch.arange(G, device=dev).unsqueeze(1).expand_as(table)[valid]
    per_head = torch.zeros(G + 1, dtype=torch.float64, device=dev)
    per_head.index_add_(0, owner, delta.double().sum(1))
    del delta, owner, valid, table
    ctx_now = sess.cache.ctx_len.reshape(G).double()
    assert bool((per_head[:G] <= r + 1e-3).all()) and bool((per_head[:G] >= r / ctx_now - 1e-3).all())
    assert float(per_head[G]) == 0.0 and bool(torch.isfinite(out).all())

    per = shape.num_layers * shape.num_kv_heads
    s, layer = 7, 33
    heads = list(range(s * per + layer * shape.num_kv_heads, s * per + (layer + 1) * shape.num_kv_heads))

    def budgets():
        nb = (sess.cache.ctx_len.reshape(shape.num_seqs, -1).long() + b - 1) // b
        return (nb.sum(1) // 10).to(torch.int32)

    def held_blocks():
        return int(((sess.cache.ctx_len.reshape(-1).long() + b - 1) // b).sum())

    # rank-block round: the rows of the sampled heads follow from the schedule's threshold, which the
    # oracle cannot recompute without the whole sequence; what it can check is each sampled head by
    # itself: given the rows the device took from it, the head must have lost exactly its smallest
    # metrics (ties in logical order) and be compacted as Algorithm 1 says
    bud = budgets()
    small, _ = W.gather_heads(sess.cache, heads)
    st = oracle_state(small)
    held0 = held_blocks()
    rows, sel = sess.evict_rank_select(bud)
    assert torch.equal(sel.cpu(), bud.cpu()) and int(rows.sum()) == int(bud.sum())
    rows_s = rows[torch.tensor(heads, device=dev)].cpu().numpy()
    masks = []
    for i in range(len(heads)):     # the oracle's schedule of that head alone, asked for the rows the device took from it
        one = oracle_state(W.gather_heads(sess.cache, [heads[i]])[0])
        rows_w, masks_w, sel_w = O.rank_schedule(one, [int(rows_s[i])], protect_tail_blocks=0)
        assert int(rows_w[0]) == int(rows_s[i]) == int(sel_w[0])
        masks.append(masks_w[0])
    freed = int(sess.compact_rank().item())
    assert freed == int(bud.sum()) and held_blocks() == held0 - freed
    sess.check_state()
    O.compact_slots(st, masks)
    post = oracle_state(W.gather_heads(sess.cache, heads)[0])
    np.testing.assert_array_equal(post.lens(), st.lens())
    for i in range(len(heads)):
        n, o = O.slots_of(st, i)
        n2, o2 = O.slots_of(post, i)
        np.testing.assert_array_equal(post.k_cache[n2, o2], st.k_cache[n, o])
        np.testing.assert_array_equal(post.v_cache[n2, o2], st.v_cache[n, o])
        np.testing.assert_array_equal(post.metric[n2, o2], st.metric[n, o])
        np.testing.assert_array_equal(post.pos[n2, o2], st.pos[n, o])
    del st, post, small

    # block round (the long tables take the sliced compaction): flags of the sampled heads given, the
    # oracle moves them; keys of the sampled heads against the oracle's bit for bit
    bud = budgets()
    small, _ = W.gather_heads(sess.cache, heads)
    st = oracle_state(small)
    key = sess.metric_reduce()
    want_key, _ = O.block_keys(st, small.metric.numpy())
    hsel = torch.tensor(heads, device=dev)
    nbs = -(-st.lens() // b)
    for i in range(len(heads)):
        np.testing.assert_array_equal(key[hsel[i], :nbs[i]].cpu().numpy().view(np.uint32), want_key[i, :nbs[i]].view(np.uint32))
    held0 = held_blocks()
    flag, count, sel = sess.evict_select(bud)
    assert torch.equal(sel.cpu(), bud.cpu()) and int(count.sum()) == int(bud.sum())
    flag_s = flag[hsel].cpu().numpy()
    assert (flag_s.sum(1) == count[hsel].cpu().numpy()).all()
    freed = int(sess.compact().item())
    assert freed == int(bud.sum()) and held_blocks() == held0 - freed
    sess.check_state()
    O.compact(st, flag_s, flag_s.sum(1))
    post = oracle_state(W.gather_heads(sess.cache, heads)[0])
    np.testing.assert_array_equal(post.lens(), st.lens())
    for i in range(len(heads)):
        n, o = O.slots_of(st, i)
        n2, o2 = O.slots_of(post, i)
        np.testing.assert_array_equal(post.k_cache[n2, o2], st.k_cache[n, o])
        np.testing.assert_array_equal(post.v_cache[n2, o2], st.v_cache[n, o])
        np.testing.assert_array_equal(post.metric[n2, o2], st.metric[n, o])
        np.testing.assert_array_equal(post.pos[n2, o2], st.pos[n, o])
    assert held_blocks() + int(sess.cache.free_map.sum()) == shape.num_blocks
