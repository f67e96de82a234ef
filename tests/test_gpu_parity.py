"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs.  Floating point within 2e-3 max-abs (outputs and
metrics, fp32 accumulation on the GPU, fp64 in the oracle); tables, free maps,
context lengths, block keys, selections and compacted caches bit-exact."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import kvc_oracle as O
from paper_2410_00161_amd import binding as B
from paper_2410_00161_amd import workloads as W
from helpers import oracle_state, check_allocator_invariants, assert_keys_equal

pytestmark = pytest.mark.gpu
TOL = 2e-3


def session(cache, mode=B.KVC_L2):
    from paper_2410_00161_amd.session import KvcSession
    return KvcSession(cache, metric_mode=mode)


def say(*a):
    print("[case]", *a, flush=True)


def assert_state_equal(sess, st: O.State, kv_exact=True, check_pos=True):
    c = sess.cache
    torch.cuda.synchronize()
    np.testing.assert_array_equal(c.block_table.cpu().numpy().astype(np.int64), st.block_table)
    np.testing.assert_array_equal(c.ctx_len.cpu().numpy().astype(np.int64), st.ctx_len)
    np.testing.assert_array_equal(c.free_map.cpu().numpy(), st.free_map)
    if kv_exact:  # compare only slots that hold a KV: the rest is unspecified
        k = c.k_cache.float().cpu().numpy().astype(np.float64)
        v = c.v_cache.float().cpu().numpy().astype(np.float64)
        m = c.metric.cpu().numpy().astype(np.float64)
        p = c.pos.cpu().numpy().astype(np.int64)
        for g in range(st.G):
            n, o = O.slots_of(st, g)
            np.testing.assert_array_equal(k[n, o], st.k_cache[n, o])
            np.testing.assert_array_equal(v[n, o], st.v_cache[n, o])
            if check_pos:
                np.testing.assert_array_equal(p[n, o], st.pos[n, o])
            np.testing.assert_allclose(m[n, o], st.metric[n, o], rtol=0, atol=TOL)


# ---------------------------------------------------------------------------
# decode + metric
# ---------------------------------------------------------------------------

DECODE_CASES = [
    # name, small_mixed kwargs, chunk tokens (0 = default), mode
    ("bf16_d128_r4", dict(r=4, d=128, kv_dtype="bf16", L=700), 0, B.KVC_L2),
    ("bf16_d128_r4_split", dict(r=4, d=128, kv_dtype="bf16", L=700), 128, B.KVC_L2),
    ("bf16_d128_r8_split", dict(r=8, d=128, kv_dtype="bf16", L=500), 64, B.KVC_L2),
    ("bf16_odd_chunk", dict(r=4, d=128, kv_dtype="bf16", L=1500, rho=2.0, S=2), 1088, B.KVC_L2),
    # few head instances: the library shortens its chunks by itself; blocks of 64 tokens and
    # r = 8 are the cases in which a halved chunk must still start on a block boundary
    ("bf16_b64_default_chunk", dict(r=4, d=128, kv_dtype="bf16", L=1500, rho=2.0, S=2, b=64), 0, B.KVC_L2),
    ("bf16_r8_default_chunk", dict(r=8, d=128, kv_dtype="bf16", L=1500, rho=2.0, S=2), 0, B.KVC_L2),
    ("fp8_r8_b32_default_chunk", dict(r=8, d=128, kv_dtype="fp8", L=1500, rho=2.0, S=2, b=32), 0, B.KVC_L2),
    ("bf16_d128_r1", dict(r=1, d=128, kv_dtype="bf16", L=300), 0, B.KVC_L2),
    ("bf16_d128_r2_L1", dict(r=2, d=128, kv_dtype="bf16", L=300), 64, B.KVC_L1),
    ("bf16_d64_r4", dict(r=4, d=64, kv_dtype="bf16", L=400), 128, B.KVC_L2),
    ("f32_d64_r2", dict(r=2, d=64, kv_dtype="f32", L=512), 0, B.KVC_L2),
    ("f32_d128_r4_split", dict(r=4, d=128, kv_dtype="f32", L=400), 64, B.KVC_L2),
    ("bf16_b32", dict(r=4, d=128, kv_dtype="bf16", L=400, b=32), 128, B.KVC_L2),
    ("bf16_b4", dict(r=4, d=128, kv_dtype="bf16", L=200, b=4), 64, B.KVC_L2),
    ("bf16_b2", dict(r=4, d=128, kv_dtype="bf16", L=120, b=2), 0, B.KVC_L2),
    ("bf16_b1_split", dict(r=4, d=128, kv_dtype="bf16", L=700, b=1), 128, B.KVC_L2),
    ("bf16_b2_r8_split", dict(r=8, d=128, kv_dtype="bf16", L=500, b=2), 64, B.KVC_L1),
    ("f32_b1_d64", dict(r=2, d=64, kv_dtype="f32", L=300, b=1), 0, B.KVC_L2),
    ("fp8_b1_r8", dict(r=8, d=128, kv_dtype="fp8", L=400, b=1), 64, B.KVC_L2),
    ("generic_b128", dict(r=4, d=128, kv_dtype="bf16", L=600, b=128), 0, B.KVC_L2),
    ("generic_r3", dict(r=3, d=64, kv_dtype="f32", L=200), 0, B.KVC_L1),
    ("generic_d32", dict(r=2, d=32, kv_dtype="bf16", L=200), 0, B.KVC_L2),
    ("fp8_d128_r4", dict(r=4, d=128, kv_dtype="fp8", L=700), 0, B.KVC_L2),
    ("fp8_d128_r4_split", dict(r=4, d=128, kv_dtype="fp8", L=700), 128, B.KVC_L2),
    ("fp8_d128_r8", dict(r=8, d=128, kv_dtype="fp8", L=300), 64, B.KVC_L2),
    ("fp8_d128_r1_L1", dict(r=1, d=128, kv_dtype="fp8", L=300), 0, B.KVC_L1),
    ("fp8_d64_r2", dict(r=2, d=64, kv_dtype="fp8", L=400), 64, B.KVC_L2),
    ("fp8_b8", dict(r=4, d=128, kv_dtype="fp8", L=200, b=8), 64, B.KVC_L2),
    ("fp8_b2", dict(r=4, d=128, kv_dtype="fp8", L=120, b=2), 0, B.KVC_L2),
    ("fp8_generic_b128", dict(r=4, d=128, kv_dtype="fp8", L=600, b=128), 0, B.KVC_L2),
]


def poison(t, mask):
    """NaN into the masked rows; 8-bit floats are written as the byte 0x7f, their NaN."""
    if t.dtype == torch.float8_e4m3fn:
        t.view(torch.uint8)[mask] = 0x7F
    else:
        t[mask] = float("nan")


@pytest.mark.parametrize("name,kw,chunk,mode", DECODE_CASES, ids=[c[0] for c in DECODE_CASES])
def test_decode_matches_oracle(name, kw, chunk, mode):
    say("decode", name, kw, "chunk", chunk)
    shape, ctx, seed = W.small_mixed(41, **kw)
    ctx[1] = 0                       # a head with no KV at all
    ctx[2] = 1                       # a single KV
    ctx[3] = shape.block_size * 3    # ends exactly on a block boundary
    cache = W.make_cache(shape, ctx, seed, placement="fragmented", init_metric="prefill")
    # poison every slot that holds no KV: the kernels must never let it through
    owner_real = torch.zeros_like(cache.metric, dtype=torch.bool)
    st0 = oracle_state(cache)
    for g in range(st0.G):
        n, o = O.slots_of(st0, g)
        owner_real[torch.from_numpy(n), torch.from_numpy(o)] = True
    poison(cache.v_cache, ~owner_real)
    poison(cache.k_cache, ~owner_real)
    st = oracle_state(cache)
    q = W.make_query(shape, seed)
    want = O.paged_decode(st, q.double().numpy(), metric_mode="L2" if mode == B.KVC_L2 else "L1")
    B.kvc_set_decode_chunk(chunk)
    try:
        sess = session(cache, mode)
        sess.out.fill_(7.0)
        out = sess.paged_decode(q.to(sess.device))
        torch.cuda.synchronize()
    finally:
        B.kvc_set_decode_chunk(0)
    got = out.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    np.testing.assert_allclose(got, want, rtol=0, atol=TOL)
    m = sess.cache.metric.cpu().numpy().astype(np.float64)
    real = owner_real.numpy()
    np.testing.assert_allclose(m[real], st.metric[real], rtol=0, atol=TOL)
    # slots that hold no KV keep their old metric bit for bit
    np.testing.assert_array_equal(m[~real], cache.metric.numpy().astype(np.float64)[~real])


def _shape_matrix():
    """Every query-group size x row type x head dimension, each with a block size and a chunk
    setting taken in rotation (0 = the library's own choice for a call over few heads)."""
    cases, i = [], 0
    blocks = (16, 64, 8, 32, 4, 2, 1)
    chunks = (0, 64, 0, 192, 0, 1088)
    for r in (1, 2, 4, 8):
        for dt in ("bf16", "f32", "fp8"):
            for d in (64, 128):
                for rep in range(2):
                    b, chunk = blocks[i % len(blocks)], chunks[i % len(chunks)]
                    i += 1
                    cases.append((f"r{r}_{dt}_d{d}_b{b}_c{chunk}", dict(r=r, d=d, kv_dtype=dt, b=b), chunk))
    return cases


SHAPE_MATRIX = _shape_matrix()


@pytest.mark.parametrize("name,kw,chunk", SHAPE_MATRIX, ids=[c[0] for c in SHAPE_MATRIX])
def test_decode_over_the_matrix_of_shapes(name, kw, chunk):
    say("decode shape matrix", name)
    shape, ctx, seed = W.small_mixed(59, S=2, Lyr=1, Hk=2, L=1300, rho=2.0, **kw)
    ctx[0] = 1300                    # one head at the full length: several chunks at every setting
    cache = W.make_cache(shape, ctx, seed, placement="fragmented", init_metric="prefill")
    st = oracle_state(cache)
    q = W.make_query(shape, seed)
    want = O.paged_decode(st, q.double().numpy())
    B.kvc_set_decode_chunk(chunk)
    try:
        sess = session(cache)
        out = sess.paged_decode(q.to(sess.device))
        torch.cuda.synchronize()
    finally:
        B.kvc_set_decode_chunk(0)
    np.testing.assert_allclose(out.cpu().numpy().astype(np.float64), want, rtol=0, atol=TOL)
    live = st.free_map == 0
    np.testing.assert_allclose(sess.cache.metric.cpu().numpy().astype(np.float64)[live], st.metric[live], rtol=0, atol=TOL)


# Calls over at most 1024 head instances with the library's own chunk setting: the chunk length
# is picked on the device from the lengths (1.25 / 256 of all tokens up to 256 heads, / 512 from
# 512 on, at least 256, at most the default).  Few long heads (chunks of ~800 tokens, every head
# split many times), many short ones (nothing split), one head far longer than the rest.
DEVICE_CHUNK_CASES = [
    ("few_long_heads", dict(S=1, Lyr=1, Hk=8, r=4, d=128, kv_dtype="bf16", L=20000, rho=1.3), None),
    ("many_short_heads", dict(S=6, Lyr=5, Hk=8, r=4, d=128, kv_dtype="bf16", L=700, rho=1.5), None),
    ("one_long_head_r8_fp8", dict(S=2, Lyr=2, Hk=8, r=8, d=128, kv_dtype="fp8", L=1200, rho=2.0, b=32), 30000),
]


@pytest.mark.parametrize("name,kw,long_head", DEVICE_CHUNK_CASES, ids=[c[0] for c in DEVICE_CHUNK_CASES])
def test_decode_with_the_chunk_length_picked_on_the_device(name, kw, long_head):
    say("decode, chunk length picked on the device", name)
    shape, ctx, seed = W.small_mixed(71, **kw)
    if long_head:
        import dataclasses
        ctx[5] = long_head
        shape = dataclasses.replace(shape, num_blocks=shape.num_blocks + long_head // shape.block_size + 8,
                                    max_blocks_per_head=long_head // shape.block_size + 8)
    cache = W.make_cache(shape, ctx, seed, placement="fragmented", init_metric="prefill")
    st = oracle_state(cache)
    q = W.make_query(shape, seed)
    want = O.paged_decode(st, q.double().numpy())
    sess = session(cache)
    out = sess.paged_decode(q.to(sess.device))
    torch.cuda.synchronize()
    np.testing.assert_allclose(out.cpu().numpy().astype(np.float64), want, rtol=0, atol=TOL)
    live = st.free_map == 0
    np.testing.assert_allclose(sess.cache.metric.cpu().numpy().astype(np.float64)[live], st.metric[live], rtol=0, atol=TOL)
    # one layer of it alone (fewer heads, another length)
    out2 = sess.paged_decode(q.to(sess.device), accumulate_metric=False, layer_begin=shape.num_layers - 1,
                             layer_end=shape.num_layers)
    torch.cuda.synchronize()
    lsel = shape.num_layers - 1
    np.testing.assert_allclose(out2.cpu().numpy().astype(np.float64)[:, lsel], want[:, lsel], rtol=0, atol=TOL)


DOMINANT_CASES = [
    ("bf16_r8", dict(r=8, d=128, kv_dtype="bf16", L=600), 128),
    ("fp8_r8", dict(r=8, d=128, kv_dtype="fp8", L=600), 128),
    ("bf16_r4", dict(r=4, d=128, kv_dtype="bf16", L=600), 0),
    ("fp8_r4", dict(r=4, d=128, kv_dtype="fp8", L=600), 0),
    ("f32_r2_d64", dict(r=2, d=64, kv_dtype="f32", L=400), 64),
]


@pytest.mark.parametrize("name,kw,chunk", DOMINANT_CASES, ids=[c[0] for c in DOMINANT_CASES])
def test_decode_with_a_dominant_key(name, kw, chunk):
    """One key per head instance is aligned with a query head of its group (probability close to
    one for that head) and carries a large value row: the regime in which a probability that
    entered the P V product with fewer than 16 bits would miss the tolerance."""
    say("decode dominant key", name, kw, "chunk", chunk)
    shape, ctx, seed = W.small_mixed(47, **kw)
    cache = W.make_cache(shape, ctx, seed, placement="fragmented", init_metric="prefill")
    q = W.make_query(shape, seed)
    st0 = oracle_state(cache)
    r = shape.num_q_heads // shape.num_kv_heads
    kdt = cache.k_cache.dtype

    def put(t, n, o, row):   # 8-bit tensors take no indexed assignment: move the bytes
        if kdt == torch.float8_e4m3fn:
            t.view(torch.uint8)[n, o] = row.to(kdt).view(torch.uint8)
        else:
            t[n, o] = row.to(kdt)

    for g in range(st0.G):
        n, o = O.slots_of(st0, g)
        if len(n) < 3:
            continue
        s_, l_, h_ = np.unravel_index(g, (shape.num_seqs, shape.num_layers, shape.num_kv_heads))
        j = (7 * g + 3) % len(n)                    # anywhere in the head, also in later chunks
        hq = r * h_ + (g % r)                       # the query head it is aligned with
        qrow = q[s_, l_, hq].float()
        put(cache.k_cache, int(n[j]), int(o[j]), 2.0 * qrow)
        vrow = cache.v_cache[int(n[j]), int(o[j])].float() if kdt != torch.float8_e4m3fn else \
            cache.v_cache.view(torch.uint8)[int(n[j]), int(o[j])].view(kdt).float()
        put(cache.v_cache, int(n[j]), int(o[j]), 3.0 * vrow + 1.0)
    st = oracle_state(cache)
    want = O.paged_decode(st, q.double().numpy())
    B.kvc_set_decode_chunk(chunk)
    try:
        sess = session(cache)
        out = sess.paged_decode(q.to(sess.device))
        torch.cuda.synchronize()
    finally:
        B.kvc_set_decode_chunk(0)
    # the setup did what it was meant to: some metric increment is close to its maximum of one per head
    inc = st.metric - st0.metric
    assert inc.max() > 0.9
    np.testing.assert_allclose(out.cpu().numpy().astype(np.float64), want, rtol=0, atol=TOL)
    np.testing.assert_allclose(sess.cache.metric.cpu().numpy().astype(np.float64), st.metric, rtol=0, atol=TOL)


def test_decode_layer_range_and_no_metric():
    say("decode layer range")
    shape, ctx, seed = W.small_mixed(43, S=2, Lyr=3, Hk=2, r=4, d=128, L=300)
    cache = W.make_cache(shape, ctx, seed, init_metric="prefill")
    st = oracle_state(cache)
    q = W.make_query(shape, seed)
    sess = session(cache)
    sess.out.fill_(-5.0)
    m_before = sess.cache.metric.clone()
    out = sess.paged_decode(q.to(sess.device), accumulate_metric=False, layer_begin=1, layer_end=2)
    torch.cuda.synchronize()
    want = O.paged_decode(st, q.double().numpy(), accumulate_metric=False, layer_begin=1, layer_end=2)
    got = out.cpu().numpy()
    np.testing.assert_allclose(got[:, 1], want[:, 1], rtol=0, atol=TOL)
    assert (got[:, 0] == -5.0).all() and (got[:, 2] == -5.0).all()   # other layers untouched
    assert torch.equal(sess.cache.metric, m_before)
    # per-layer calls with accumulation == one call over all layers
    for l in range(shape.num_layers):
        sess.paged_decode(q.to(sess.device), accumulate_metric=True, layer_begin=l, layer_end=l + 1)
    torch.cuda.synchronize()
    want = O.paged_decode(st, q.double().numpy())
    np.testing.assert_allclose(sess.out.cpu().numpy(), want, rtol=0, atol=TOL)
    np.testing.assert_allclose(sess.cache.metric.cpu().numpy(), st.metric, rtol=0, atol=TOL)


@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8"])
def test_decode_steps_accumulate_with_append(kv_dtype):
    say("append + decode x 20", kv_dtype)
    shape, ctx, seed = W.small_mixed(47, S=2, Lyr=2, Hk=2, r=4, d=128, L=100, extra_blocks=3, kv_dtype=kv_dtype)
    cache = W.make_cache(shape, ctx, seed)
    st = oracle_state(cache)
    sess = session(cache)
    for step in range(20):
        k, v = W.make_new_kv(shape, seed, step)
        q = W.make_query(shape, seed, step)
        O.append(st, k.double().numpy(), v.double().numpy())
        want = O.paged_decode(st, q.double().numpy())
        sess.append(k.to(sess.device), v.to(sess.device))
        out = sess.paged_decode(q.to(sess.device))
        torch.cuda.synchronize()
        np.testing.assert_allclose(out.cpu().numpy(), want, rtol=0, atol=TOL)
    assert_state_equal(sess, st)
    check_allocator_invariants(st)


# ---------------------------------------------------------------------------
# allocator
# ---------------------------------------------------------------------------

def test_alloc_free_match_oracle_bit_exactly():
    say("alloc/free")
    shape, ctx, seed = W.small_mixed(51, S=4, Lyr=3, Hk=4, L=260, slack=2.0)
    cache = W.make_cache(shape, ctx, seed, placement="fragmented")
    st = oracle_state(cache)
    sess = session(cache)
    rng = np.random.default_rng(0)
    for it in range(4):
        n_new = torch.from_numpy(rng.integers(0, 3, size=shape.G).astype(np.int32))
        O.block_alloc(st, n_new.numpy())
        sess.block_alloc(n_new)
        assert_state_equal(sess, st, kv_exact=False)
        held = np.array([O.num_blocks_held(st, g) for g in range(st.G)])
        n_drop = torch.from_numpy(np.minimum(rng.integers(0, 3, size=shape.G), held).astype(np.int32))
        freed_want = O.block_free(st, n_drop.numpy())
        assert sess.block_free(n_drop) == freed_want
        assert_state_equal(sess, st, kv_exact=False)
    check_allocator_invariants(st)
    # prefill from an empty pool: every head takes its blocks in one call
    shape2, ctx2, _ = W.small_mixed(52, S=3, Lyr=2, Hk=2, L=5000, rho=6.0)
    cache2 = W.make_cache(shape2, torch.zeros_like(ctx2), 52)
    st2 = oracle_state(cache2)
    sess2 = session(cache2)
    nb = W.blocks_needed(ctx2, shape2.block_size).to(torch.int32)
    O.block_alloc(st2, nb.numpy())
    sess2.block_alloc(nb)
    assert_state_equal(sess2, st2, kv_exact=False)


def test_alloc_errors_leave_state_untouched():
    say("alloc errors")
    shape, ctx, seed = W.small_mixed(53, S=2, Lyr=2, Hk=2, L=200, extra_blocks=2)
    total = int(W.blocks_needed(ctx, shape.block_size).sum())
    shape = W.Shape(**{**shape.__dict__, "num_blocks": total + 5})       # five free blocks
    cache = W.make_cache(shape, ctx, seed)
    st = oracle_state(cache)
    sess = session(cache)
    big = torch.ones(shape.G, dtype=torch.int32)                          # 8 wanted, 5 free
    cases = [(big, B.KVC_ERR_OOM)]
    full = torch.zeros(shape.G, dtype=torch.int32); full[3] = shape.max_blocks_per_head
    cases.append((full, B.KVC_ERR_TABLE_FULL))
    neg = torch.zeros(shape.G, dtype=torch.int32); neg[1] = -1
    cases.append((neg, B.KVC_ERR_ARG))
    for req, code in cases:
        with pytest.raises(O.OracleError) as eo:
            O.block_alloc(st, req.numpy())
        assert eo.value.code == code
        with pytest.raises(B.KvcError) as e:
            sess.block_alloc(req)
        assert e.value.code == code
        assert_state_equal(sess, st, kv_exact=False)
    # asynchronous form: the error waits in the status word and later steps are no-ops
    sess.block_alloc(big, flags=B.KVC_ASYNC)
    assert B.kvc_poll_status(sess.cfg, sess.ws) == B.KVC_ERR_OOM
    ok = torch.zeros(shape.G, dtype=torch.int32); ok[0] = 1
    sess.block_alloc(ok, flags=B.KVC_ASYNC)
    assert_state_equal(sess, st, kv_exact=False)       # still untouched: the error is sticky
    B.kvc_workspace_reset(sess.cfg, sess.ws)
    sess.block_alloc(ok)
    O.block_alloc(st, ok.numpy())
    assert_state_equal(sess, st, kv_exact=False)
    # drop more than held
    over = torch.zeros(shape.G, dtype=torch.int32); over[2] = 10 ** 6
    with pytest.raises(B.KvcError) as e:
        sess.block_free(over)
    assert e.value.code == B.KVC_ERR_ARG
    assert_state_equal(sess, st, kv_exact=False)
    # append with the table row full
    shape3, ctx3, _ = W.small_mixed(54, S=1, Lyr=1, Hk=2, L=64, rho=1.0, extra_blocks=0)
    shape3 = W.Shape(**{**shape3.__dict__, "max_blocks_per_head": 4})
    ctx3[:] = 64
    cache3 = W.make_cache(shape3, ctx3, 54)
    st3 = oracle_state(cache3); sess3 = session(cache3)
    k, v = W.make_new_kv(shape3, 54)
    with pytest.raises(O.OracleError):
        O.append(st3, k.double().numpy(), v.double().numpy())
    with pytest.raises(B.KvcError) as e:
        sess3.append(k.to(sess3.device), v.to(sess3.device))
    assert e.value.code == B.KVC_ERR_TABLE_FULL
    assert_state_equal(sess3, st3)


# ---------------------------------------------------------------------------
# block keys, selection, compaction
# ---------------------------------------------------------------------------

def test_block_keys_bit_exact():
    say("block keys")
    shape, ctx, seed = W.small_mixed(61, S=3, Lyr=2, Hk=3, L=900)
    cache = W.make_cache(shape, ctx, seed, placement="fragmented", init_metric="prefill")
    st0 = oracle_state(cache)
    real = np.zeros((shape.num_blocks, shape.block_size), dtype=bool)
    for g in range(st0.G):
        n, o = O.slots_of(st0, g); real[n, o] = True
    cache.metric[torch.from_numpy(~real)] = float("nan")
    st = oracle_state(cache)
    want, _ = O.block_keys(st, cache.metric.numpy())
    sess = session(cache)
    sess.block_key.fill_(123.0)
    got = sess.metric_reduce().cpu().numpy()
    held = assert_keys_equal(got, want, st)
    assert (got[~held] == 123.0).all()   # cells of blocks a head does not hold are not written
    want_max, _ = O.block_keys(st, cache.metric.numpy(), key="max")
    got = sess.metric_reduce(key_mode=B.KVC_KEY_MAX).cpu().numpy()
    assert_keys_equal(got, want_max, st)


SELECT_CASES = [
    ("per_seq_protect1", dict(pooled=False, protect=1, ties=False, frac=0.5)),
    ("per_seq_protect0", dict(pooled=False, protect=0, ties=False, frac=0.3)),
    ("pooled", dict(pooled=True, protect=1, ties=False, frac=0.4)),
    ("heavy_ties", dict(pooled=False, protect=1, ties=True, frac=0.5)),
    ("pooled_ties_protect0", dict(pooled=True, protect=0, ties=True, frac=0.6)),
    ("budget_zero_and_huge", dict(pooled=False, protect=1, ties=False, frac=None)),
    ("max_keys", dict(pooled=False, protect=1, ties=False, frac=0.5, key="max")),
]


@pytest.mark.parametrize("name,kw", SELECT_CASES, ids=[c[0] for c in SELECT_CASES])
def test_select_and_compact_bit_exact(name, kw):
    say("select+compact", name)
    shape, ctx, seed = W.small_mixed(71, S=4, Lyr=3, Hk=2, r=2, d=64, L=1200, rho=2.0)
    cache = W.make_cache(shape, ctx, seed, placement="fragmented", init_metric="prefill")
    if kw["ties"]:
        g = torch.Generator().manual_seed(5)
        cache.metric = torch.randint(0, 2, cache.metric.shape, generator=g).float()
    st = oracle_state(cache)
    sess = session(cache)
    key = sess.metric_reduce(key_mode=B.KVC_KEY_MAX if kw.get("key") == "max" else B.KVC_KEY_SUM)
    want_key, _ = O.block_keys(st, cache.metric.numpy(), key=kw.get("key", "sum"))
    nb = -(-st.lens() // st.b)
    per_seq = nb.reshape(st.S, -1).sum(1)
    if kw["pooled"]:
        seg = torch.tensor([0, 1, 1, st.S], dtype=torch.int32)  # one empty segment in the middle
        tot = [int(per_seq[:1].sum()), 0, int(per_seq[1:].sum())]
        budget = torch.tensor([int(kw["frac"] * t) for t in tot], dtype=torch.int32)
        if budget[1] == 0:
            budget[1] = 3  # asks for blocks from a segment that has none
    else:
        seg = None
        if kw["frac"] is None:
            budget = torch.tensor([0, 10 ** 6, 1, int(per_seq[3])], dtype=torch.int32)
        else:
            budget = torch.tensor([int(kw["frac"] * t) for t in per_seq], dtype=torch.int32)
    flag_w, count_w, sel_w = O.evict_select(st, want_key, budget.numpy(),
                                            None if seg is None else seg.numpy(), kw["protect"])
    flag, count, sel = sess.evict_select(budget, seg, kw["protect"])
    torch.cuda.synchronize()
    assert_keys_equal(key, want_key, st)
    np.testing.assert_array_equal(sel.cpu().numpy(), sel_w)
    np.testing.assert_array_equal(count.cpu().numpy(), count_w)
    np.testing.assert_array_equal(flag.cpu().numpy(), flag_w)
    freed_w = O.compact(st, flag_w, count_w)
    freed = sess.compact()
    torch.cuda.synchronize()
    assert int(freed.item()) == freed_w == int(sel_w.sum())
    assert_state_equal(sess, st)
    check_allocator_invariants(st)
    # the compacted cache still decodes to the oracle's result
    q = W.make_query(shape, seed, 9)
    want = O.paged_decode(st, q.double().numpy())
    out = sess.paged_decode(q.to(sess.device))
    torch.cuda.synchronize()
    np.testing.assert_allclose(out.cpu().numpy(), want, rtol=0, atol=TOL)


SEGMENT_CASES = [
    # one workgroup per sequence walks that sequence's candidate blocks: more of them than the
    # copy it keeps on chip holds (blocks of one token), and keys that tie at the threshold
    ("more_keys_than_the_on_chip_copy", dict(b=1, L=6800, protect=1, ties=True, empty=False)),
    ("more_keys_protect0_distinct", dict(b=1, L=6800, protect=0, ties=False, empty=False)),
    # sequences whose first head instances have no candidate at all, with ties to rank behind them
    ("first_heads_without_candidates", dict(b=16, L=900, protect=1, ties=True, empty=True)),
    ("first_heads_without_candidates_protect2", dict(b=4, L=300, protect=2, ties=True, empty=True)),
]


@pytest.mark.parametrize("name,kw", SEGMENT_CASES, ids=[c[0] for c in SEGMENT_CASES])
def test_select_one_sequence_per_segment_edges(name, kw):
    say("select by sequence", name)
    shape, ctx, seed = W.small_mixed(83, S=2, Lyr=3, Hk=2, r=2, d=64, b=kw["b"], L=kw["L"], rho=1.2)
    ctx = ctx.clone()
    if kw["b"] == 1:
        # the library picks this path by the pool's blocks per sequence: one long sequence next to
        # a short one keeps that average low while the long one overflows the on-chip copy
        ctx.reshape(2, -1)[1] //= 16
        total = int(ctx.sum())
        shape = dataclasses.replace(shape, num_blocks=int(1.3 * total) + 64)
        assert shape.num_blocks <= 28672 * shape.num_seqs
    if kw["empty"]:
        flat = ctx.reshape(2, -1)
        flat[0, 0] = 0                                  # no KV at all
        flat[0, 1] = kw["b"] * kw["protect"]            # only protected blocks
        flat[1, 0] = 1
        flat[1, 2] = 0
    cache = W.make_cache(shape, ctx, seed, placement="fragmented", init_metric="prefill")
    if kw["ties"]:
        g = torch.Generator().manual_seed(11)
        cache.metric = torch.randint(0, 2, cache.metric.shape, generator=g).float()
    st = oracle_state(cache)
    sess = session(cache)
    key = sess.metric_reduce()
    want_key, _ = O.block_keys(st, cache.metric.numpy())
    nb = -(-st.lens() // st.b)
    cand = np.maximum(nb - kw["protect"], 0).reshape(st.S, -1).sum(1)
    if kw["b"] == 1:
        assert cand[0] > 28672, "the case is about a sequence with more candidates than are kept on chip"
    for frac in (0.37, 0.9):
        budget = torch.tensor([int(frac * c) for c in cand], dtype=torch.int32)
        flag_w, count_w, sel_w = O.evict_select(st, want_key, budget.numpy(), None, kw["protect"])
        flag, count, sel = sess.evict_select(budget, None, kw["protect"])
        torch.cuda.synchronize()
        np.testing.assert_array_equal(sel.cpu().numpy(), sel_w)
        np.testing.assert_array_equal(count.cpu().numpy(), count_w)
        np.testing.assert_array_equal(flag.cpu().numpy(), flag_w)
    freed_w = O.compact(st, flag_w, count_w)
    freed = sess.compact()
    torch.cuda.synchronize()
    assert int(freed.item()) == freed_w == int(sel_w.sum())
    assert_state_equal(sess, st)


@pytest.mark.parametrize("kv_dtype,b", [("bf16", 16), ("fp8", 64), ("f32", 4)])
def test_compaction_of_long_heads_in_slices(kv_dtype, b):
    """Tables sized for more than 65536 tokens a head: the compaction spreads a head's movers over
    several workgroups and frees the tail blocks in a launch of its own.  Heads of up to 20000 KVs
    (movers in several slices), one that loses nearly everything, one that loses nothing, one empty."""
    import dataclasses
    say("sliced compaction", kv_dtype, b)
    shape, ctx, seed = W.small_mixed(77, S=2, Lyr=1, Hk=3, r=1, d=64, L=20000, rho=1.3, b=b, kv_dtype=kv_dtype)
    shape = dataclasses.replace(shape, max_blocks_per_head=70000 // b)
    assert shape.max_blocks_per_head * b > 65536
    ctx[4] = 0
    cache = W.make_cache(shape, ctx, seed, placement="fragmented", init_metric="prefill")
    g = torch.Generator().manual_seed(9)
    cache.metric = torch.rand(cache.metric.shape, generator=g)
    t = cache.block_table.reshape(shape.G, -1)
    cache.metric[t[1][t[1] >= 0].long()] += 10.0      # head 1 keeps everything
    cache.metric[t[2][t[2] >= 0].long()] *= 1e-3      # head 2 is the cheapest by far
    st = oracle_state(cache)
    sess = session(cache)
    key = sess.metric_reduce()
    want_key, _ = O.block_keys(st, cache.metric.numpy())
    nb = -(-st.lens() // st.b)
    budget = torch.tensor([int(0.45 * x) for x in nb.reshape(st.S, -1).sum(1)], dtype=torch.int32)
    flag_w, count_w, sel_w = O.evict_select(st, want_key, budget.numpy())
    flag, count, sel = sess.evict_select(budget)
    np.testing.assert_array_equal(flag.cpu().numpy(), flag_w)
    assert count_w[1] == 0 and count_w[2] == nb[2] - 1
    freed_w = O.compact(st, flag_w, count_w)
    assert int(sess.compact().item()) == freed_w
    assert_state_equal(sess, st)
    check_allocator_invariants(st)


def test_select_numeric_error_and_compact_argument_error():
    say("select/compact errors")
    shape, ctx, seed = W.small_mixed(73, S=2, Lyr=2, Hk=2, r=2, d=64, L=300)
    cache = W.make_cache(shape, ctx, seed, init_metric="prefill")
    st = oracle_state(cache)
    sess = session(cache)
    key = sess.metric_reduce().clone()
    budget = torch.tensor([3, 3], dtype=torch.int32)
    for bad in (float("nan"), -1.0, float("inf")):
        k2 = key.clone(); k2[0, 0] = bad
        with pytest.raises(B.KvcError) as e:
            sess.evict_select(budget, block_key=k2)
        assert e.value.code == B.KVC_ERR_NUMERIC
        assert int(sess.evict_flag.sum()) == 0 and int(sess.evict_count.sum()) == 0
    k2 = key.clone(); k2[0, 0] = -0.0     # minus zero is a valid key equal to zero
    sess.evict_select(budget, block_key=k2)
    neg = torch.tensor([3, -1], dtype=torch.int32)
    with pytest.raises(B.KvcError) as e:
        sess.evict_select(neg)
    assert e.value.code == B.KVC_ERR_ARG
    # compact: a flag beyond the head's blocks, and a count that disagrees
    flag, count, sel = sess.evict_select(budget)
    nb0 = -(-int(st.lens()[0]) // shape.block_size)
    maxb = shape.max_blocks_per_head
    for g_bad, u_bad in ((0, maxb - 1), (0, nb0), (0, nb0 + 1), (0, (nb0 + maxb) // 2), (1, maxb - 2), (2, maxb - 17)):
        nb_g = -(-int(st.lens()[g_bad]) // shape.block_size)
        assert nb_g <= u_bad < maxb
        f2 = flag.clone(); f2[g_bad, u_bad] = 1      # a block the head does not hold
        with pytest.raises(B.KvcError) as e:
            sess.compact(f2, count)
        assert e.value.code == B.KVC_ERR_ARG
    c2 = count.clone(); c2[1] += 1
    with pytest.raises(B.KvcError) as e:
        sess.compact(flag, c2)
    assert e.value.code == B.KVC_ERR_ARG
    assert_state_equal(sess, st)


def test_tiny_reference_config_end_to_end():
    """Configuration 1: one decode step from zero metrics, evict half the blocks
    (per sequence, then pooled), compact; everything compared."""
    for pooled in (False, True):
        say("tiny ref pooled=", pooled)
        shape, ctx, seed = W.tiny_ref()
        cache = W.make_cache(shape, ctx, seed)
        st = oracle_state(cache)
        sess = session(cache)
        q = W.make_query(shape, seed)
        want = O.paged_decode(st, q.double().numpy())
        out = sess.paged_decode(q.to(sess.device))
        torch.cuda.synchronize()
        np.testing.assert_allclose(out.cpu().numpy(), want, rtol=0, atol=TOL)
        key = sess.metric_reduce()
        torch.cuda.synchronize()
        # selection parity is defined on identical metric inputs: the oracle ranks the GPU's keys
        want_key, want_key64 = O.block_keys(st, sess.cache.metric.cpu().numpy())
        assert_keys_equal(key, want_key, st)
        np.testing.assert_allclose(want_key, O.block_keys(st)[1], rtol=0, atol=TOL * 16)
        nb_seq = (-(-st.lens() // st.b)).reshape(st.S, -1).sum(1)
        if pooled:
            seg = torch.tensor([0, st.S], dtype=torch.int32)
            budget = torch.tensor([int(nb_seq.sum()) // 2], dtype=torch.int32)
        else:
            seg, budget = None, torch.tensor(nb_seq // 2, dtype=torch.int32)
        flag_w, count_w, sel_w = O.evict_select(st, want_key, budget.numpy(),
                                                None if seg is None else seg.numpy(), 1)
        flag, count, sel = sess.evict_select(budget, seg, 1)
        np.testing.assert_array_equal(flag.cpu().numpy(), flag_w)
        np.testing.assert_array_equal(sel.cpu().numpy(), sel_w)
        st.metric = sess.cache.metric.cpu().numpy().astype(np.float64)   # same metric inputs
        free_before = int(sess.cache.free_map.sum())
        freed_w = O.compact(st, flag_w, count_w)
        freed = int(sess.compact().item())
        assert freed == freed_w == int(budget.sum())
        # memory freed = evicted blocks x block bytes
        assert (int(sess.cache.free_map.sum()) - free_before) * shape.block_size * shape.head_dim * 4 * 2 \
            == freed * 2 * shape.block_size * shape.head_dim * shape.kv_bytes
        assert_state_equal(sess, st)


def test_scheduling_helpers_match_oracle():
    say("count / prefill alloc / preempt")
    shape, ctx, seed = W.small_mixed(57, S=5, Lyr=3, Hk=2, L=300, slack=3.0, extra_blocks=6)
    ctx[6:12] = 0                        # sequence 1 not yet prefetched
    ctx[0] = 3 * shape.block_size        # a head exactly on a block boundary
    cache = W.make_cache(shape, ctx, seed, placement="fragmented")
    st = oracle_state(cache)
    sess = session(cache)
    dev = sess.device
    needed = torch.full((shape.num_seqs,), -7, dtype=torch.int32, device=dev)
    held = torch.full((shape.num_seqs,), -7, dtype=torch.int32, device=dev)
    for l0, l1 in ((0, shape.num_layers), (1, 2)):
        B.kvc_count_blocks(sess.cfg, sess.st, l0, l1, needed, held, sess.ws)
        torch.cuda.synchronize()
        nw, hw = O.count_blocks(st, l0, l1)
        np.testing.assert_array_equal(needed.cpu().numpy(), nw)
        np.testing.assert_array_equal(held.cpu().numpy(), hw)
    tokens = torch.tensor([0, 137, 0, 0, 0], dtype=torch.int32)
    O.prefill_alloc(st, tokens.numpy())
    B.kvc_prefill_alloc(sess.cfg, sess.st, tokens.to(dev), sess.ws)
    assert_state_equal(sess, st, kv_exact=False)
    mask = torch.tensor([1, 0, 0, 1, 0], dtype=torch.uint8)
    freed_w = O.preempt(st, mask.numpy())
    assert B.kvc_preempt(sess.cfg, sess.st, mask.to(dev), sess.ws) == freed_w > 0
    assert_state_equal(sess, st, kv_exact=False)
    check_allocator_invariants(st)
    # a prefill that cannot fit leaves everything as it was
    huge = torch.tensor([0, 0, 0, 10 ** 6, 0], dtype=torch.int32)
    with pytest.raises(O.OracleError):
        O.prefill_alloc(st, huge.numpy())
    with pytest.raises(B.KvcError):
        B.kvc_prefill_alloc(sess.cfg, sess.st, huge.to(dev), sess.ws)
    assert_state_equal(sess, st, kv_exact=False)


# ---------------------------------------------------------------------------
# degenerate: nothing cached at all
# ---------------------------------------------------------------------------

def test_empty_cache_every_call_then_first_tokens():
    """No head holds a KV: decode writes zero rows and leaves the metric alone, block keys are
    zero, selection and both compactions take and free nothing; then the first tokens arrive
    (every head allocates its first block) and a decode over one KV per head returns that V."""
    say("all heads empty")
    shape, ctx, seed = W.small_mixed(83, S=2, Lyr=2, Hk=3, r=4, d=128, L=100)
    cache = W.make_cache(shape, torch.zeros_like(ctx), seed, init_metric="prefill")
    st = oracle_state(cache)
    sess = session(cache)
    q = W.make_query(shape, seed)
    sess.out.fill_(3.0)
    m0 = sess.cache.metric.clone()
    out = sess.paged_decode(q.to(sess.device))
    torch.cuda.synchronize()
    assert float(out.abs().max()) == 0.0 and torch.equal(sess.cache.metric, m0)
    np.testing.assert_array_equal(out.cpu().numpy(), O.paged_decode(st, q.double().numpy()))
    assert float(sess.metric_reduce().abs().max()) == 0.0
    budget = torch.full((shape.num_seqs,), 5, dtype=torch.int32)
    flag, count, sel = sess.evict_select(budget)
    assert int(flag.sum()) == 0 and int(count.sum()) == 0 and int(sel.sum()) == 0
    assert int(sess.compact().item()) == 0
    rows, sel = sess.evict_rank_select(budget)
    assert int(rows.sum()) == 0 and int(sel.sum()) == 0
    assert int(sess.compact_rank().item()) == 0
    assert_state_equal(sess, st)
    for step in range(2):
        k, v = W.make_new_kv(shape, seed, step)
        O.append(st, k.double().numpy(), v.double().numpy())
        sess.append(k.to(sess.device), v.to(sess.device))
        want = O.paged_decode(st, q.double().numpy())
        out = sess.paged_decode(q.to(sess.device))
        torch.cuda.synchronize()
        np.testing.assert_allclose(out.cpu().numpy(), want, rtol=0, atol=TOL)
        if step == 0:   # one KV per head: the output is that V row, whatever q is
            r = shape.group_size
            vv = v.float().unsqueeze(3).expand(-1, -1, -1, r, -1).reshape(out.shape)
            np.testing.assert_allclose(out.cpu().numpy(), vv.numpy(), rtol=0, atol=1e-6)
    assert_state_equal(sess, st)
    check_allocator_invariants(st)


@pytest.mark.parametrize("skw", [dict(S=37, Lyr=2, Hk=2, L=300), dict(S=2500, Lyr=1, Hk=1, L=48)],
                         ids=["37_seqs", "2500_seqs"])
def test_compression_batch_matches_oracle(skw):
    say("compression batch", skw)
    shape, ctx, seed = W.small_mixed(91, r=1, d=64, rho=2.0, **skw)
    ctx[4:8] = 0                                  # a sequence (or a few) that holds nothing
    cache = W.make_cache(shape, ctx, seed, placement="fragmented")
    st = oracle_state(cache)
    sess = session(cache)
    rng = np.random.default_rng(5)
    per = shape.num_layers * shape.num_kv_heads
    held = [sum(O.num_blocks_held(st, g) for g in range(s * per, (s + 1) * per)) for s in range(shape.num_seqs)]
    total = sum(held) * shape.block_size
    in_batch = torch.zeros(shape.num_seqs, dtype=torch.uint8, device=sess.device)
    kvs = torch.zeros(1, dtype=torch.int64, device=sess.device)
    for case in range(14):
        last = rng.integers(-3, 6, shape.num_seqs)
        run = None if case % 3 == 0 else rng.integers(0, 2, shape.num_seqs).astype(np.uint8)
        limit = [0, total, total // 2, total // 5, 10 ** 15, 1, (total * 9) // 10][case % 7]
        want, want_kvs = O.compression_batch(st, last, limit, running=run)
        in_batch.fill_(9)
        B.kvc_compression_batch(sess.cfg, sess.st, torch.from_numpy(last).to(sess.device),
                                None if run is None else torch.from_numpy(run).to(sess.device),
                                limit, in_batch, kvs, sess.ws)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(in_batch.cpu().numpy().astype(bool), want)
        assert int(kvs.item()) == want_kvs
    with pytest.raises(B.KvcError):
        B.kvc_compression_batch(sess.cfg, sess.st, torch.zeros(shape.num_seqs, dtype=torch.int64, device=sess.device),
                                None, -1, in_batch, kvs, sess.ws)


# ---------------------------------------------------------------------------
# work lists of all layers kept from one launch (kvc_decode_plan / kvc_paged_decode_planned)
# ---------------------------------------------------------------------------

PLAN_CASES = [
    ("many_short_heads", dict(S=6, Lyr=5, Hk=8, r=4, d=128, kv_dtype="bf16", L=700, rho=1.5)),
    ("few_long_heads_r8_fp8", dict(S=1, Lyr=3, Hk=8, r=8, d=128, kv_dtype="fp8", L=9000, rho=1.3, b=32)),
    ("b4_d64", dict(S=3, Lyr=2, Hk=4, r=2, d=64, kv_dtype="bf16", L=2000, rho=2.0, b=4)),
]


@pytest.mark.parametrize("name,kw", PLAN_CASES, ids=[c[0] for c in PLAN_CASES])
def test_decode_layer_by_layer_from_kept_work_lists(name, kw):
    say("planned decode", name)
    shape, ctx, seed = W.small_mixed(83, extra_blocks=3, **kw)
    ctx[2] = 0
    cache = W.make_cache(shape, ctx, seed, placement="fragmented", init_metric="prefill")
    st = oracle_state(cache)
    sess = session(cache)
    q = W.make_query(shape, seed)
    want = O.paged_decode(st, q.double().numpy())
    sess.out.fill_(5.0)
    sess.decode_plan()
    for l in reversed(range(shape.num_layers)):          # any order of layers
        sess.paged_decode_planned(q.to(sess.device), l)
    torch.cuda.synchronize()
    assert B.kvc_poll_status(sess.cfg, sess.ws) == B.KVC_OK
    np.testing.assert_allclose(sess.out.cpu().numpy().astype(np.float64), want, rtol=0, atol=TOL)
    live = st.free_map == 0
    np.testing.assert_allclose(sess.cache.metric.cpu().numpy().astype(np.float64)[live], st.metric[live], rtol=0, atol=TOL)
    # the same numbers as the ordinary call over that layer, bit for bit (same kernels, same cuts)
    ref = session(cache)
    for l in range(shape.num_layers):
        ref.paged_decode(q.to(ref.device), layer_begin=l, layer_end=l + 1)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(sess.out.cpu().numpy(), ref.out.cpu().numpy())
    np.testing.assert_array_equal(sess.cache.metric.cpu().numpy(), ref.cache.metric.cpu().numpy())
    # a step as a model runs it: the lists are made for heads one token longer, then every layer
    # appends its token and decodes from its list
    k, v = W.make_new_kv(shape, seed, 1)
    q2 = W.make_query(shape, seed, 1)
    for l in range(shape.num_layers):     # (the allocation order follows the order of the appends)
        O.append(st, k.double().numpy(), v.double().numpy(), layer_begin=l, layer_end=l + 1)
    want2 = O.paged_decode(st, q2.double().numpy())
    sess.decode_plan(ctx_plus=1)
    for l in range(shape.num_layers):
        sess.append(k.to(sess.device), v.to(sess.device), None, l, l + 1)
        sess.paged_decode_planned(q2.to(sess.device), l)
    torch.cuda.synchronize()
    assert B.kvc_poll_status(sess.cfg, sess.ws) == B.KVC_OK
    np.testing.assert_allclose(sess.out.cpu().numpy().astype(np.float64), want2, rtol=0, atol=TOL)
    assert_state_equal(sess, st)
    # a stale list: the heads have grown since it was made.  Nothing of the cache changes, and the
    # status word says so
    m0 = sess.cache.metric.clone()
    sess.append(k.to(sess.device), v.to(sess.device))
    m1 = sess.cache.metric.clone()
    sess.paged_decode_planned(q2.to(sess.device), 0)
    torch.cuda.synchronize()
    assert torch.equal(sess.cache.metric, m1)
    assert B.kvc_poll_status(sess.cfg, sess.ws) == B.KVC_ERR_ARG
    B.kvc_workspace_reset(sess.cfg, sess.ws)
    del m0


def test_kept_work_lists_refuse_what_they_do_not_cover():
    say("planned decode, unsupported shapes")
    # more than 1024 head instances per layer
    shape, ctx, seed = W.small_mixed(85, S=140, Lyr=1, Hk=8, r=1, d=64, L=64, rho=1.0)
    sess = session(W.make_cache(shape, ctx, seed))
    with pytest.raises(B.KvcError) as e:
        sess.decode_plan()
    assert e.value.code == B.KVC_ERR_UNSUPPORTED
    # a shape of the fallback kernel; a forced chunk length
    shape, ctx, seed = W.small_mixed(86, S=2, Lyr=2, Hk=2, r=3, d=64, kv_dtype="f32", L=100)
    sess = session(W.make_cache(shape, ctx, seed))
    with pytest.raises(B.KvcError) as e:
        sess.decode_plan()
    assert e.value.code == B.KVC_ERR_UNSUPPORTED
    shape, ctx, seed = W.small_mixed(87, S=2, Lyr=2, Hk=2, r=4, d=128, L=300)
    sess = session(W.make_cache(shape, ctx, seed))
    B.kvc_set_decode_chunk(128)
    try:
        with pytest.raises(B.KvcError) as e:
            sess.decode_plan()
        assert e.value.code == B.KVC_ERR_UNSUPPORTED
    finally:
        B.kvc_set_decode_chunk(0)
    with pytest.raises(B.KvcError) as e:
        B.kvc_decode_plan(sess.cfg, sess.st, 2, sess.ws)
    assert e.value.code == B.KVC_ERR_ARG
