"""Seeded random sweep over valid shapes: append, decode with metric accumulation, a
physical-block round, a rank-block round, and the window metric, each step against the oracle.
Shapes, lengths, chunk settings and placements are drawn at random; every draw is printed first."""
import numpy as np
import pytest
import torch

from oracle import kvc_oracle as O
from paper_2410_00161_amd import binding as B
from paper_2410_00161_amd import workloads as W
from helpers import oracle_state, check_allocator_invariants
from test_gpu_parity import session, say, assert_state_equal, TOL
from test_gpu_scenarios import evict_round

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed0", [11, 12, 13, 14])
def test_decode_and_rounds_on_random_shapes(seed0):
    rng = np.random.default_rng(seed0)
    for case in range(30):
        r = int(rng.choice([1, 2, 4, 8])); d = int(rng.choice([64, 128]))
        dt = str(rng.choice(["bf16", "f32", "fp8"])); b = int(rng.choice([1, 2, 4, 8, 16, 32, 64]))
        S, Lyr, Hk = int(rng.integers(1, 5)), int(rng.integers(1, 4)), int(rng.integers(1, 4))
        L = int(rng.integers(max(3 * b, 40), 2600 if b >= 8 else 500))
        rho = float(rng.uniform(1.0, 4.0))
        chunk = int(rng.choice([0, 0, 64, 128, 192, 1088]))
        placement = str(rng.choice(["fresh", "fragmented"]))
        mode = int(rng.choice([B.KVC_L2, B.KVC_L1]))
        say("random shape", dict(seed0=seed0, case=case, r=r, d=d, dt=dt, b=b, S=S, Lyr=Lyr, Hk=Hk, L=L,
                                 rho=round(rho, 2), chunk=chunk, placement=placement, mode=mode))
        shape, ctx, seed = W.small_mixed(1000 + seed0 * 1000 + case, S=S, Lyr=Lyr, Hk=Hk, r=r, d=d, b=b, L=L,
                                         rho=rho, kv_dtype=dt, extra_blocks=3)
        if rng.random() < 0.3:
            ctx[int(rng.integers(0, len(ctx)))] = 0
        if rng.random() < 0.3:
            ctx[int(rng.integers(0, len(ctx)))] = 1
        cache = W.make_cache(shape, ctx, seed, placement=placement, init_metric="prefill")
        st = oracle_state(cache)
        sess = session(cache, mode)
        B.kvc_set_decode_chunk(chunk)
        try:
            for step, ev in enumerate(("block", "rank", None)):
                k, v = W.make_new_kv(shape, seed, step)
                q = W.make_query(shape, seed, step)
                O.append(st, k.double().numpy(), v.double().numpy())
                want = O.paged_decode(st, q.double().numpy(), metric_mode="L2" if mode == B.KVC_L2 else "L1")
                sess.append(k.to(sess.device), v.to(sess.device))
                out = sess.paged_decode(q.to(sess.device))
                torch.cuda.synchronize()
                np.testing.assert_allclose(out.cpu().numpy(), want, rtol=0, atol=TOL)
                live = st.free_map == 0
                np.testing.assert_allclose(sess.cache.metric.cpu().numpy()[live], st.metric[live], rtol=0, atol=TOL)
                if ev:
                    evict_round(sess, st, float(rng.uniform(0.05, 0.6)), ev)
                    assert_state_equal(sess, st)
                    check_allocator_invariants(st)
        finally:
            B.kvc_set_decode_chunk(0)


@pytest.mark.parametrize("seed0", [21, 22])
def test_window_metric_on_random_shapes(seed0):
    rng = np.random.default_rng(seed0)
    for case in range(30):
        r = int(rng.choice([1, 2, 4, 8]))
        w = int(rng.integers(1, min(32, 256 // r) + 1))
        b = int(rng.choice([16, 32, 64, 4, 8, 1]))
        d = int(rng.choice([128, 128, 64]))
        dt = str(rng.choice(["bf16", "bf16", "fp8"]))
        pool = int(rng.choice([1, 3, 5, 7, 9, 131]))
        S, Lyr, Hk = int(rng.integers(1, 4)), int(rng.integers(1, 3)), int(rng.integers(1, 3))
        L = int(rng.integers(64, 4200))
        rho = float(rng.uniform(1.0, 3.0))
        mode = int(rng.choice([B.KVC_L2, B.KVC_L1]))
        acc = bool(rng.random() < 0.3)
        say("random window", dict(seed0=seed0, case=case, r=r, w=w, b=b, d=d, dt=dt, pool=pool, S=S, Lyr=Lyr, Hk=Hk, L=L,
                                  rho=round(rho, 2), mode=mode, acc=acc))
        shape, ctx, seed = W.small_mixed(5000 + seed0 * 1000 + case, S=S, Lyr=Lyr, Hk=Hk, r=r, d=d, b=b, L=L,
                                         rho=rho, kv_dtype=dt)
        if rng.random() < 0.3:
            ctx[int(rng.integers(0, len(ctx)))] = 0
        if rng.random() < 0.3:
            ctx[int(rng.integers(0, len(ctx)))] = int(rng.integers(1, w + 1))
        cache = W.make_cache(shape, ctx, seed, placement=str(rng.choice(["fresh", "fragmented"])),
                             init_metric="prefill")
        st = oracle_state(cache)
        g = torch.Generator().manual_seed(seed + 3)
        qw = torch.randn((S, Lyr, Hk * r, w, d), generator=g).to(torch.bfloat16)
        O.window_metric(st, qw.double().numpy(), w, pool, "L2" if mode == B.KVC_L2 else "L1", accumulate=acc)
        sess = session(cache, mode)
        sess.window_metric(qw.to(sess.device), w, pool, accumulate=acc)
        torch.cuda.synchronize()
        m = sess.cache.metric.cpu().numpy().astype(np.float64)
        real = np.zeros(m.shape, dtype=bool)
        for gi in range(st.G):
            n, o = O.slots_of(st, gi)
            real[n, o] = True
        np.testing.assert_allclose(m[real], st.metric[real], rtol=0, atol=TOL)


@pytest.mark.parametrize("seed0", [41, 42])
def test_query_block_metric_on_random_shapes(seed0):
    """Blocks of queries at random positions of ragged heads: in front of, inside and past the end
    of a head, chunks with and without visible keys, heads of a multiple of eight chunks, excluded
    windows longer than the block, blocks longer than one pass of the kernels takes; several blocks
    accumulate into one metric."""
    rng = np.random.default_rng(seed0)
    for case in range(24):
        r = int(rng.choice([1, 2, 4, 8]))
        w = int(rng.integers(1, min(64, 256 // r) + 1))
        if case % 4 == 3:
            w = int(rng.integers(65, 300))       # a long block: several passes of the kernels
        b = int(rng.choice([16, 32, 64, 8, 2]))
        d = int(rng.choice([128, 128, 64]))
        dt = str(rng.choice(["bf16", "bf16", "fp8"]))
        S, Lyr, Hk = int(rng.integers(1, 3)), int(rng.integers(1, 3)), int(rng.integers(1, 4))
        L = int(rng.choice([int(rng.integers(64, 3000)), 2048, 8192]))
        rho = float(rng.choice([1.0, rng.uniform(1.0, 3.0)]))
        mode = int(rng.choice([B.KVC_L2, B.KVC_L1]))
        excl = int(rng.choice([0, 1, 10, w + 5]))
        say("random query blocks", dict(seed0=seed0, case=case, r=r, w=w, b=b, d=d, dt=dt, S=S, Lyr=Lyr, Hk=Hk, L=L,
                                        rho=round(rho, 2), mode=mode, excl=excl))
        shape, ctx, seed = W.small_mixed(7000 + seed0 * 1000 + case, S=S, Lyr=Lyr, Hk=Hk, r=r, d=d, b=b, L=L,
                                         rho=rho, kv_dtype=dt)
        if rng.random() < 0.3:
            ctx[int(rng.integers(0, len(ctx)))] = 0
        cache = W.make_cache(shape, ctx, seed, placement=str(rng.choice(["fresh", "fragmented"])),
                             init_metric="prefill")
        st = oracle_state(cache)
        sess = session(cache, mode)
        g = torch.Generator().manual_seed(seed + 5)
        starts = [0, int(rng.integers(0, L)), max(0, L - w), int(rng.integers(0, L))]
        for start in starts[: 2 if L > 4096 else 4]:
            qb = torch.randn((S, Lyr, Hk * r, w, d), generator=g).to(torch.bfloat16)
            O.query_block_metric(st, qb.double().numpy(), w, start, excl, "L2" if mode == B.KVC_L2 else "L1")
            sess.query_block_metric(qb.to(sess.device), w, start, excl)
        torch.cuda.synchronize()
        m = sess.cache.metric.cpu().numpy().astype(np.float64)
        real = np.zeros(m.shape, dtype=bool)
        for gi in range(st.G):
            n, o = O.slots_of(st, gi)
            real[n, o] = True
        np.testing.assert_allclose(m[real], st.metric[real], rtol=0, atol=TOL)
        np.testing.assert_array_equal(m[~real], cache.metric.numpy().astype(np.float64)[~real])


@pytest.mark.parametrize("seed0", [31, 32])
def test_allocator_operations_in_random_order(seed0):
    """Random sequences of alloc / free / append / preempt / prefill / count, some of them requests
    that must be refused: both sides accept and refuse alike (same code), and the state matches
    after every operation."""
    rng = np.random.default_rng(seed0)
    refused = 0
    for case in range(60):
        b = int(rng.choice([1, 4, 16, 64]))
        S, Lyr, Hk = int(rng.integers(1, 6)), int(rng.integers(1, 4)), int(rng.integers(1, 4))
        L = int(rng.integers(4 * b, 40 * b))
        slack = float(rng.uniform(1.05, 2.5))
        say("random allocator sequence", dict(seed0=seed0, case=case, b=b, S=S, Lyr=Lyr, Hk=Hk, L=L, slack=round(slack, 2)))
        shape, ctx, seed = W.small_mixed(3000 + seed0 * 1000 + case, S=S, Lyr=Lyr, Hk=Hk, r=2, d=64, b=b, L=L,
                                         rho=2.0, slack=slack, extra_blocks=int(rng.integers(0, 4)))
        cache = W.make_cache(shape, ctx, seed, placement=str(rng.choice(["fresh", "fragmented"])))
        st = oracle_state(cache)
        sess = session(cache)
        dev, G = sess.device, shape.G

        def both(on_oracle, on_gpu):
            eo = eg = ro = rg = None
            try:
                ro = on_oracle()
            except O.OracleError as e:
                eo = e
            try:
                rg = on_gpu()
            except B.KvcError as e:
                eg = e
            assert (eo is None) == (eg is None), (eo, eg)
            if eo is not None:
                assert eo.code == eg.code
            return ro, rg, eo is not None

        for op_i in range(10):
            op = str(rng.choice(["alloc", "free", "append", "preempt", "prefill", "count"]))
            bad = False
            if op == "alloc":
                n = torch.from_numpy((rng.integers(0, 3, size=G) * (rng.random(G) < 0.5)).astype(np.int32))
                _, _, bad = both(lambda: O.block_alloc(st, n.numpy()), lambda: sess.block_alloc(n))
            elif op == "free":
                held = np.array([O.num_blocks_held(st, g) for g in range(G)])
                n = np.minimum(held, rng.integers(0, 3, size=G)) * (rng.random(G) < 0.5)
                if rng.random() < 0.1:
                    n[int(rng.integers(0, G))] += 1000   # more than the head holds
                n = torch.from_numpy(n.astype(np.int32))
                ro, rg, bad = both(lambda: O.block_free(st, n.numpy()), lambda: sess.block_free(n))
                assert ro == rg
            elif op == "append":
                k, v = W.make_new_kv(shape, seed, op_i)
                l0 = int(rng.integers(0, Lyr))
                l1 = int(rng.integers(l0 + 1, Lyr + 1))
                _, _, bad = both(lambda: O.append(st, k.double().numpy(), v.double().numpy(), None, l0, l1),
                                 lambda: sess.append(k.to(dev), v.to(dev), None, l0, l1))
            elif op == "preempt":
                m = torch.from_numpy((rng.random(S) < 0.3).astype(np.uint8))
                ro, rg, bad = both(lambda: O.preempt(st, m.numpy()),
                                   lambda: B.kvc_preempt(sess.cfg, sess.st, m.to(dev), sess.ws))
                assert ro == rg
            elif op == "prefill":
                t = torch.from_numpy((rng.integers(0, L, size=S) * (rng.random(S) < 0.4)).astype(np.int32))
                _, _, bad = both(lambda: O.prefill_alloc(st, t.numpy()),
                                 lambda: B.kvc_prefill_alloc(sess.cfg, sess.st, t.to(dev), sess.ws))
            else:
                needed = torch.zeros(S, dtype=torch.int32, device=dev)
                held_t = torch.zeros(S, dtype=torch.int32, device=dev)
                B.kvc_count_blocks(sess.cfg, sess.st, 0, Lyr, needed, held_t, sess.ws)
                torch.cuda.synchronize()
                nw, hw = O.count_blocks(st, 0, Lyr)
                np.testing.assert_array_equal(needed.cpu().numpy(), nw)
                np.testing.assert_array_equal(held_t.cpu().numpy(), hw)
            refused += bad
            assert_state_equal(sess, st, kv_exact=False)
            check_allocator_invariants(st)
    assert refused > 0   # the sweep did exercise refusals
