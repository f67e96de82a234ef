"""GPU parity of the rank-block (paper-exact) eviction schedule against the oracle: rows per
head, selected counts and the compacted cache, bit for bit, on identical metric inputs."""
import numpy as np
import pytest
import torch

from oracle import kvc_oracle as O
from paper_2410_00161_amd import binding as B
from paper_2410_00161_amd import workloads as W
from helpers import oracle_state, check_allocator_invariants
from test_gpu_parity import session, say, assert_state_equal, TOL

pytestmark = pytest.mark.gpu

CASES = [
    ("per_seq", dict(b=16), dict(pooled=False, protect=1, ties=False, frac=0.4)),
    ("per_seq_protect0_b4", dict(b=4, L=300), dict(pooled=False, protect=0, ties=False, frac=0.7)),
    ("pooled_ties", dict(b=16), dict(pooled=True, protect=1, ties=True, frac=0.5)),
    ("ties_protect0_b2", dict(b=2, L=150), dict(pooled=False, protect=0, ties=True, frac=0.6)),
    ("budget_zero_and_huge", dict(b=16), dict(pooled=False, protect=1, ties=False, frac=None)),
    ("f32_d64", dict(b=16, kv_dtype="f32", d=64), dict(pooled=False, protect=1, ties=False, frac=0.3)),
    ("fp8_d128", dict(b=16, kv_dtype="fp8"), dict(pooled=False, protect=1, ties=False, frac=0.4)),
    # more than 1024 head instances: the kernels run in their 256-thread form (below that, with few
    # and possibly long heads, a workgroup has 1024 threads)
    ("many_heads", dict(S=24, Lyr=7, Hk=8, L=150, b=16), dict(pooled=False, protect=1, ties=False, frac=0.4)),
    ("many_heads_ties_b4", dict(S=24, Lyr=7, Hk=8, L=60, b=4), dict(pooled=True, protect=0, ties=True, frac=0.5)),
    # tables sized for more than 16 384 KVs a head: the histogram passes give a head a workgroup
    # (of 1024 threads with few heads, of 256 with many) instead of a wavefront
    ("long_tables_few_heads", dict(L=17000, rho=8.0, b=16), dict(pooled=False, protect=1, ties=False, frac=0.4)),
    ("long_tables_many_heads", dict(S=24, Lyr=7, Hk=8, L=17000, rho=64.0, b=16), dict(pooled=True, protect=1, ties=True, frac=0.5)),
]


@pytest.mark.parametrize("name,skw,kw", CASES, ids=[c[0] for c in CASES])
def test_rank_select_and_compact_bit_exact(name, skw, kw):
    say("rank mode", name)
    base = dict(S=4, Lyr=3, Hk=2, r=2, d=64, L=1200, rho=2.0)
    base.update(skw)
    shape, ctx, seed = W.small_mixed(81, **base)
    ctx[5] = 0
    ctx[6] = 1
    cache = W.make_cache(shape, ctx, seed, placement="fragmented", init_metric="prefill")
    if kw["ties"]:
        g = torch.Generator().manual_seed(5)
        cache.metric = torch.randint(0, 3, cache.metric.shape, generator=g).float()
    st = oracle_state(cache)
    sess = session(cache)
    nb = -(-st.lens() // st.b)
    per_seq = nb.reshape(st.S, -1).sum(1)
    if kw["pooled"]:
        seg = torch.tensor([0, 1, 1, st.S], dtype=torch.int32)
        tot = [int(per_seq[:1].sum()), 0, int(per_seq[1:].sum())]
        budget = torch.tensor([int(kw["frac"] * t) for t in tot], dtype=torch.int32)
        budget[1] = 3
    else:
        seg = None
        if kw["frac"] is None:
            budget = torch.tensor([0, 10 ** 6, 1, int(per_seq[3])], dtype=torch.int32)
        else:
            budget = torch.tensor([int(kw["frac"] * t) for t in per_seq], dtype=torch.int32)
    rows_w, masks_w, sel_w = O.rank_schedule(st, budget.numpy(), None if seg is None else seg.numpy(),
                                             kw["protect"], metric=cache.metric.numpy())
    rows, sel = sess.evict_rank_select(budget, seg, kw["protect"])
    torch.cuda.synchronize()
    np.testing.assert_array_equal(sel.cpu().numpy(), sel_w)
    np.testing.assert_array_equal(rows.cpu().numpy(), rows_w)
    freed_w = O.compact_slots(st, masks_w)
    freed = int(sess.compact_rank().item())
    assert freed == freed_w == int(sel_w.sum())
    assert_state_equal(sess, st)
    check_allocator_invariants(st)
    for g in range(st.G):
        if rows_w[g]:
            assert st.lens()[g] % st.b == 0
    q = W.make_query(shape, seed, 3)
    want = O.paged_decode(st, q.double().numpy())
    out = sess.paged_decode(q.to(sess.device))
    torch.cuda.synchronize()
    np.testing.assert_allclose(out.cpu().numpy(), want, rtol=0, atol=TOL)


def test_rank_errors_leave_state_untouched():
    say("rank mode errors")
    shape, ctx, seed = W.small_mixed(83, S=2, Lyr=2, Hk=2, r=2, d=64, L=300)
    cache = W.make_cache(shape, ctx, seed, init_metric="prefill")
    st0 = oracle_state(cache)
    n, o = O.slots_of(st0, 1)
    budget = torch.tensor([3, 3], dtype=torch.int32)
    for bad in (float("nan"), -1.0, float("inf")):
        c2 = cache.clone()
        c2.metric[int(n[0]), int(o[0])] = bad
        sess = session(c2)
        with pytest.raises(B.KvcError) as e:
            sess.evict_rank_select(budget)
        assert e.value.code == B.KVC_ERR_NUMERIC
        assert int(sess.evict_count.sum()) == 0
    sess = session(cache)
    st = oracle_state(cache)
    rows, sel = sess.evict_rank_select(budget)
    r2 = rows.clone(); r2[0] = 10 ** 6
    with pytest.raises(B.KvcError) as e:
        sess.compact_rank(r2)
    assert e.value.code == B.KVC_ERR_ARG
    r2 = rows.clone(); r2[1] = -1
    with pytest.raises(B.KvcError) as e:
        sess.compact_rank(r2)
    assert e.value.code == B.KVC_ERR_ARG
    assert_state_equal(sess, st)
