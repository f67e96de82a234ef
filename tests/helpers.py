"""Glue used by the tests only: turns a workloads.Cache into an oracle State and
compares states.  No arithmetic of the method lives here."""
import numpy as np
import torch

from oracle import kvc_oracle as O


def oracle_state(cache) -> O.State:
    sh = cache.shape
    f = lambda t: t.detach().to("cpu").to(torch.float64).numpy()
    i = lambda t: t.detach().to("cpu").to(torch.int64).numpy()
    return O.State(sh.num_seqs, sh.num_layers, sh.num_kv_heads, sh.group_size, sh.head_dim,
                   sh.block_size, sh.num_blocks, sh.max_blocks_per_head,
                   f(cache.k_cache), f(cache.v_cache), f(cache.metric), i(cache.pos),
                   i(cache.block_table), i(cache.ctx_len), i(cache.free_map))


def check_allocator_invariants(st: O.State):
    """Every held block is owned once, rows are prefix-filled, and the free map
    is exactly the complement of the tables."""
    tab, lens = st.table(), st.lens()
    held = tab[tab >= 0]
    assert held.size == np.unique(held).size, "a block id sits in two table cells"
    assert (st.free_map[held] == 0).all(), "held block marked free"
    assert int((st.free_map == 0).sum()) == held.size, "leaked block"
    for g in range(st.G):
        n = O.num_blocks_held(st, g)
        assert (tab[g, n:] == -1).all(), "row not prefix-filled"
        assert n * st.b >= lens[g], "context longer than the blocks held"


def assert_keys_equal(key, want_key, st: O.State):
    """Block keys bit for bit over the blocks every head holds; the library leaves the cells of
    blocks a head does not hold as they were."""
    key = np.asarray(key.detach().cpu().numpy() if hasattr(key, "detach") else key)
    nb = -(-st.lens() // st.b)
    held = np.arange(st.max_blocks)[None, :] < nb[:, None]
    np.testing.assert_array_equal(key.reshape(st.G, -1).view(np.uint32)[held],
                                  np.asarray(want_key).reshape(st.G, -1).view(np.uint32)[held])
    return held
