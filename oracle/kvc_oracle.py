"""CPU oracle for the head-variable paged KV cache (KV-Compress hot path).

TEST INFRASTRUCTURE ONLY.  This file is a plain, slow, obviously-correct
statement of what the path computes, written from the paper.  It shares no code
with the HIP library and is imported only by tests, the smoke check and the
benchmark's cpu_baseline leg.  Floating point is fp64 unless a step fixes fp32
(the block-key sum, which the selection must reproduce bit for bit).

Where each function comes from (sections of the KV-Compress paper):
  gather / paged lookup ...... Preliminaries "Paged Attention" (n = T[s, i//b],
                               o = i mod b), generalised to one table per
                               (sequence, layer, KV head): Method "Block Layout
                               and Parallel Allocation"
  decode ..................... Preliminaries "Multi-head Attention"
                               (A = softmax(Q K^T / sqrt d), out = A V)
  metric accumulation ........ Method "Query Group Compression" (sum over the
                               query heads of the KV head's group), "Squared
                               Attention Metric" (sum of A^2; L1 = sum of A),
                               "Continual Compression" (decode queries add
                               into the metrics already held)
  window_metric .............. Preliminaries "KV Cache Compression" (observation
                               window, max-pooling), Method "Metric Calculation"
                               (KVC-w: squared before summation)
  alloc / free / append ...... "Block Layout and Parallel Allocation" (flat
                               length-N allocation tensor, per-head context
                               lengths)
  block_keys / select ........ "Evicting from a Paged KV Cache": blocks ordered
                               by summed metric; per-sequence budget E_s of
                               blocks; domain 1 <= e < ceil(C_h / b)
  compact .................... Algorithm 1 (MoveCache) in closed form, and
                               movecache_sequential = the two-pointer loop
  rank_schedule .............. the same section's schedule as printed: per-head
                               sort, rows of b, m(h, e) = last column, rows
                               ordered across heads, first E_s marked

Readings taken where the paper is silent or inconsistent:
  * a "block" in block_keys/select is a physical block as it lies in a head's
    table (block-level reduction of the metric), not a rank-sorted group of b
    KVs; the two agree when b = 1.
  * the cross-head ordering key is the block's metric SUM.
  * allocation order: requesters in ascending head-instance index, the k-th
    requested block gets the k-th lowest free id.
  * a newly appended KV starts with metric 0 and attends to itself in the same
    step.
  * Algorithm 1 as printed never advances i after a move and does not bound
    the inner search; both are treated as typos.
  * the last `protect` logical blocks of a head are never candidates
    (protect = 1 keeps e < ceil(C_h / b); protect = 0 lets a head lose its
    only block, as the paper's worked example mentions).
"""
from __future__ import annotations

import numpy as np

KVC_OK = 0
ERR_ARG, ERR_OOM, ERR_TABLE_FULL, ERR_BUDGET, ERR_NUMERIC = 1, 2, 3, 4, 5


class OracleError(Exception):
    def __init__(self, code: int, msg: str = ""):
        super().__init__(f"oracle error {code}: {msg}")
        self.code = code


class State:
    """All arrays are numpy, owned here.  Layouts as in the paper:
    k_cache, v_cache [N, b, d]; metric, pos [N, b]; block_table
    [S, Lyr, Hk, max_blocks] (-1 = none); ctx_len [S, Lyr, Hk]; free_map [N]."""

    def __init__(self, S, Lyr, Hk, r, d, b, N, max_blocks, k_cache, v_cache, metric,
                 pos, block_table, ctx_len, free_map):
        self.S, self.Lyr, self.Hk, self.r, self.d, self.b = S, Lyr, Hk, r, d, b
        self.N, self.max_blocks = N, max_blocks
        self.k_cache = np.array(k_cache, dtype=np.float64).reshape(N, b, d)
        self.v_cache = np.array(v_cache, dtype=np.float64).reshape(N, b, d)
        self.metric = np.array(metric, dtype=np.float64).reshape(N, b)
        self.pos = np.array(pos, dtype=np.int64).reshape(N, b)
        self.block_table = np.array(block_table, dtype=np.int64).reshape(S, Lyr, Hk, max_blocks)
        self.ctx_len = np.array(ctx_len, dtype=np.int64).reshape(S, Lyr, Hk)
        self.free_map = np.array(free_map, dtype=np.uint8).reshape(N)

    @property
    def G(self):
        return self.S * self.Lyr * self.Hk

    def copy(self):
        return State(self.S, self.Lyr, self.Hk, self.r, self.d, self.b, self.N,
                     self.max_blocks, self.k_cache, self.v_cache, self.metric, self.pos,
                     self.block_table, self.ctx_len, self.free_map)

    # flat views over head instances g = (s*Lyr + l)*Hk + h
    def table(self):
        return self.block_table.reshape(self.G, self.max_blocks)

    def lens(self):
        return self.ctx_len.reshape(self.G)


def num_blocks_held(st: State, g: int) -> int:
    """Blocks a head instance holds = length of the non-negative prefix of its row."""
    row = st.table()[g]
    n = 0
    while n < st.max_blocks and row[n] >= 0:
        n += 1
    return n


def slots_of(st: State, g: int):
    """Physical (block, offset) of logical slots 0..C_g-1 of head instance g."""
    C = int(st.lens()[g])
    j = np.arange(C)
    n = st.table()[g][j // st.b]
    o = j % st.b
    return n, o


# --------------------------------------------------------------------------
# allocation
# --------------------------------------------------------------------------

def block_alloc(st: State, n_new) -> None:
    n_new = np.asarray(n_new, dtype=np.int64).reshape(st.G)
    if (n_new < 0).any():
        raise OracleError(ERR_ARG, "negative request")
    held = np.array([num_blocks_held(st, g) for g in range(st.G)])
    if ((held + n_new) > st.max_blocks).any():
        raise OracleError(ERR_TABLE_FULL)
    free_ids = np.flatnonzero(st.free_map == 1)  # ascending
    if n_new.sum() > free_ids.size:
        raise OracleError(ERR_OOM)
    k = 0
    tab = st.table()
    for g in range(st.G):
        for i in range(int(n_new[g])):
            tab[g, held[g] + i] = free_ids[k]
            st.free_map[free_ids[k]] = 0
            k += 1


def block_free(st: State, n_drop) -> int:
    """Drop the last n_drop[g] blocks of every head instance; returns blocks freed."""
    n_drop = np.asarray(n_drop, dtype=np.int64).reshape(st.G)
    held = np.array([num_blocks_held(st, g) for g in range(st.G)])
    if (n_drop < 0).any() or (n_drop > held).any():
        raise OracleError(ERR_ARG, "drop count out of range")
    tab, lens = st.table(), st.lens()
    for g in range(st.G):
        for u in range(held[g] - n_drop[g], held[g]):
            st.free_map[tab[g, u]] = 1
            tab[g, u] = -1
        lens[g] = min(lens[g], (held[g] - n_drop[g]) * st.b)
    return int(n_drop.sum())


def count_blocks(st: State, layer_begin=0, layer_end=None):
    """Per sequence: blocks needed before the next decode step over the chosen
    layers (one per head instance whose blocks are all full) and blocks held."""
    layer_end = st.Lyr if layer_end is None else layer_end
    needed = np.zeros(st.S, dtype=np.int64); held = np.zeros(st.S, dtype=np.int64)
    for g in range(st.G):
        s, l = g // (st.Lyr * st.Hk), (g // st.Hk) % st.Lyr
        h = num_blocks_held(st, g)
        held[s] += h
        if layer_begin <= l < layer_end and st.lens()[g] == h * st.b:
            needed[s] += 1
    return needed, held


def prefill_alloc(st: State, seq_tokens) -> None:
    """Every head of a sequence with tokens > 0 is brought up to ceil(tokens / b)
    blocks and its length set to tokens."""
    seq_tokens = np.asarray(seq_tokens, dtype=np.int64).reshape(st.S)
    if (seq_tokens < 0).any():
        raise OracleError(ERR_ARG)
    want = np.zeros(st.G, dtype=np.int64)
    for g in range(st.G):
        t = seq_tokens[g // (st.Lyr * st.Hk)]
        if t > 0:
            want[g] = max(0, -(-t // st.b) - num_blocks_held(st, g))
    block_alloc(st, want)
    for g in range(st.G):
        t = seq_tokens[g // (st.Lyr * st.Hk)]
        if t > 0:
            st.lens()[g] = t


def preempt(st: State, seq_mask) -> int:
    """Frees every block of the masked sequences; returns blocks freed."""
    seq_mask = np.asarray(seq_mask).reshape(st.S)
    drop = np.zeros(st.G, dtype=np.int64)
    for g in range(st.G):
        if seq_mask[g // (st.Lyr * st.Hk)]:
            drop[g] = num_blocks_held(st, g)
    return block_free(st, drop)


def compression_batch(st: State, last_compressed, kv_limit, running=None):
    """The sequences one round of compression takes ("Experiments", scheduling of compression).

    The running sequences are visited in order of the time of their last
    compression, those never compressed (negative time) first, equal times by
    sequence index.  A running total of the KVs allocated to the batch
    (blocks held x block size, summed over the sequence's head instances) is
    kept; the first sequence that would push it past kv_limit is discarded and
    the batch is closed there.  Returns (in_batch [S] bool, allocated KVs of the
    batch)."""
    last = np.asarray(last_compressed, dtype=np.int64).reshape(st.S)
    run = np.ones(st.S, dtype=bool) if running is None else np.asarray(running).reshape(st.S).astype(bool)
    if kv_limit < 0:
        raise OracleError(ERR_ARG, "negative limit")
    per = st.Lyr * st.Hk
    alloc = [sum(num_blocks_held(st, g) for g in range(s * per, (s + 1) * per)) * st.b for s in range(st.S)]
    order = sorted((s for s in range(st.S) if run[s]), key=lambda s: (-1 if last[s] < 0 else int(last[s]), s))
    in_batch = np.zeros(st.S, dtype=bool)
    total = 0
    for s in order:
        if total + alloc[s] > kv_limit:
            break
        in_batch[s] = True
        total += alloc[s]
    return in_batch, total


def append(st: State, k_new, v_new, new_pos=None, layer_begin=0, layer_end=None) -> None:
    """Store one new token's k, v for every head instance of the chosen layers."""
    layer_end = st.Lyr if layer_end is None else layer_end
    k_new = np.asarray(k_new, dtype=np.float64).reshape(st.S, st.Lyr, st.Hk, st.d)
    v_new = np.asarray(v_new, dtype=np.float64).reshape(st.S, st.Lyr, st.Hk, st.d)
    sel = [(s * st.Lyr + l) * st.Hk + h for s in range(st.S)
           for l in range(layer_begin, layer_end) for h in range(st.Hk)]
    lens = st.lens()
    want = np.zeros(st.G, dtype=np.int64)
    for g in sel:
        held = num_blocks_held(st, g)
        if lens[g] == held * st.b:
            want[g] = 1
    block_alloc(st, want)  # raises with the state untouched
    tab = st.table()
    for g in sel:
        s, l, h = g // (st.Lyr * st.Hk), (g // st.Hk) % st.Lyr, g % st.Hk
        C = int(lens[g])
        n, o = tab[g, C // st.b], C % st.b
        st.k_cache[n, o] = k_new[s, l, h]
        st.v_cache[n, o] = v_new[s, l, h]
        st.metric[n, o] = 0.0
        st.pos[n, o] = C if new_pos is None else int(np.asarray(new_pos).reshape(st.S)[s])
        lens[g] = C + 1


# --------------------------------------------------------------------------
# decode + metric
# --------------------------------------------------------------------------

def attend_dense(q, K, V):
    """Single-query softmax attention, fp64.  q [d], K, V [C, d] -> (out [d], p [C])."""
    d = q.shape[0]
    s = (K @ q) / np.sqrt(float(d))
    s = s - s.max()
    e = np.exp(s)
    p = e / e.sum()
    return p @ V, p


def paged_decode(st: State, q, accumulate_metric=True, metric_mode="L2",
                 layer_begin=0, layer_end=None):
    """One decode step over every head instance of the chosen layers.

    q [S, Lyr, Hq, d].  Returns out [S, Lyr, Hq, d] fp64 (zeros outside the
    chosen layers).  Query head hq belongs to KV head hq // r.  The metric of
    every attended slot grows by the group-sum of p^2 (L2) or p (L1)."""
    layer_end = st.Lyr if layer_end is None else layer_end
    Hq = st.Hk * st.r
    q = np.asarray(q, dtype=np.float64).reshape(st.S, st.Lyr, Hq, st.d)
    out = np.zeros((st.S, st.Lyr, Hq, st.d))
    for s in range(st.S):
        for l in range(layer_begin, layer_end):
            for h in range(st.Hk):
                g = (s * st.Lyr + l) * st.Hk + h
                C = int(st.lens()[g])
                if C == 0:
                    continue
                n, o = slots_of(st, g)
                K = st.k_cache[n, o]
                V = st.v_cache[n, o]
                inc = np.zeros(C)
                for hq in range(st.r * h, st.r * (h + 1)):
                    out[s, l, hq], p = attend_dense(q[s, l, hq], K, V)
                    inc += p * p if metric_mode == "L2" else p
                if accumulate_metric:
                    st.metric[n, o] += inc
    return out


def window_metric(st: State, q_win, w, pool=7, metric_mode="L2", accumulate=False,
                  layer_begin=0, layer_end=None, row_lse=None):
    """Prefill-end metric from an observation window (Preliminaries, "KV Cache
    Compression": sum over the last w prompt queries; Method, "Query Group
    Compression": also over the query heads of the group; "Metric Calculation":
    squared attention, KVC-w; max-pooling over the sequence with size `pool`).

    q_win [S, Lyr, Hq, w, d]: window query i of a head with C KVs sits at
    position C - w + i and attends to keys 0 .. C - w + i (causal).  raw[j] =
    sum over the group's heads and the window queries of p^2 (p with "L1").
    Keys before the window get the maximum of raw over the pool//2 neighbours
    on either side, the neighbourhood cut at the ends of that prefix; keys
    inside the window keep raw.  The result replaces the metric of the head's
    slots (or is added when accumulate).

    row_lse [S, Lyr, Hq, w] (optional): the natural logarithm of every window
    query's softmax denominator, ln sum_j exp(q.k_j / sqrt d) over the keys it
    attends to, as the attention kernel of a prefill leaves it.  A = softmax
    means A_ij = exp(s_ij - lse_i) (Preliminaries, "Multi-head Attention"), so
    when it is given the probabilities are taken as exactly that, without
    forming the denominator again."""
    layer_end = st.Lyr if layer_end is None else layer_end
    Hq = st.Hk * st.r
    q_win = np.asarray(q_win, dtype=np.float64).reshape(st.S, st.Lyr, Hq, w, st.d)
    if row_lse is not None:
        row_lse = np.asarray(row_lse, dtype=np.float64).reshape(st.S, st.Lyr, Hq, w)
    half = pool // 2
    for s in range(st.S):
        for l in range(layer_begin, layer_end):
            for h in range(st.Hk):
                g = (s * st.Lyr + l) * st.Hk + h
                C = int(st.lens()[g])
                if C == 0:
                    continue
                n, o = slots_of(st, g)
                K = st.k_cache[n, o]
                raw = np.zeros(C)
                for hq in range(st.r * h, st.r * (h + 1)):
                    for i in range(w):
                        last = C - w + i
                        if last < 0:
                            continue
                        sc = (K[:last + 1] @ q_win[s, l, hq, i]) / np.sqrt(float(st.d))
                        if row_lse is None:
                            e = np.exp(sc - sc.max())
                            p = e / e.sum()
                        else:
                            p = np.exp(sc - row_lse[s, l, hq, i])
                        raw[:last + 1] += p * p if metric_mode == "L2" else p
                P = max(0, C - w)
                pooled = raw.copy()
                for j in range(P):
                    pooled[j] = raw[max(0, j - half):min(P, j + half + 1)].max()
                if accumulate:
                    st.metric[n, o] += pooled
                else:
                    st.metric[n, o] = pooled


def query_block_metric(st: State, q_blk, w, first_pos, exclude=0, metric_mode="L2",
                       layer_begin=0, layer_end=None, row_lse=None):
    """One block of the all-queries metric ("Metric Calculation", KVC-full):
    query i of the block sits at position first_pos + i, attends causally to
    keys 0 .. min(position, C - 1), and adds p^2 to the metric of key j only
    when position - j >= exclude (the first `exclude` queries after a key are
    left out).  Always accumulates.  row_lse [S, Lyr, Hq, w] (optional) as in
    window_metric: p = exp(score - lse) with the caller's log-sum-exp."""
    layer_end = st.Lyr if layer_end is None else layer_end
    Hq = st.Hk * st.r
    q_blk = np.asarray(q_blk, dtype=np.float64).reshape(st.S, st.Lyr, Hq, w, st.d)
    if row_lse is not None:
        row_lse = np.asarray(row_lse, dtype=np.float64).reshape(st.S, st.Lyr, Hq, w)
    for s in range(st.S):
        for l in range(layer_begin, layer_end):
            for h in range(st.Hk):
                g = (s * st.Lyr + l) * st.Hk + h
                C = int(st.lens()[g])
                if C == 0:
                    continue
                n, o = slots_of(st, g)
                K = st.k_cache[n, o]
                inc = np.zeros(C)
                for hq in range(st.r * h, st.r * (h + 1)):
                    for i in range(w):
                        pos = first_pos + i
                        last = min(pos, C - 1)
                        sc = (K[:last + 1] @ q_blk[s, l, hq, i]) / np.sqrt(float(st.d))
                        if row_lse is None:
                            e = np.exp(sc - sc.max())
                            p = e / e.sum()
                        else:
                            p = np.exp(sc - row_lse[s, l, hq, i])
                        cnt = min(last, pos - exclude) + 1
                        if cnt > 0:
                            inc[:cnt] += (p * p if metric_mode == "L2" else p)[:cnt]
                st.metric[n, o] += inc


# --------------------------------------------------------------------------
# block keys and selection
# --------------------------------------------------------------------------

def block_keys(st: State, metric=None, key="sum"):
    """key[g, u] = sum (or, with key="max", maximum) of the metrics held in
    logical block u of head instance g.  "Evicting from a Paged KV Cache" asks
    for the order by sum; the matrix it builds reads a row's last column, its
    maximum.

    fp32, added left to right over the filled slots only (a partial last block
    contributes its C_g - u*b real slots; whatever sits in empty slots is
    ignored).  Entries with u >= ceil(C_g / b) are 0.  Also returns the same
    keys in fp64."""
    if key not in ("sum", "max"):
        raise OracleError(ERR_ARG, "key is 'sum' or 'max'")
    M = st.metric if metric is None else np.asarray(metric).reshape(st.N, st.b)
    M32 = M.astype(np.float32)
    key_arr = np.zeros((st.G, st.max_blocks), dtype=np.float32)
    key64 = np.zeros((st.G, st.max_blocks), dtype=np.float64)
    tab, lens = st.table(), st.lens()
    for g in range(st.G):
        C = int(lens[g])
        nb = -(-C // st.b)
        for u in range(nb):
            fill = min(st.b, C - u * st.b)
            if key == "max":
                key_arr[g, u] = M32[tab[g, u], :fill].max()
                key64[g, u] = M[tab[g, u], :fill].astype(np.float64).max()
                continue
            acc = np.float32(0.0)
            for o in range(fill):
                acc = np.float32(acc + M32[tab[g, u], o])
            key_arr[g, u] = acc
            key64[g, u] = M[tab[g, u], :fill].astype(np.float64).sum()
    return key_arr, key64


def evict_select(st: State, key, budget, seg_offsets=None, protect_tail_blocks=1):
    """Per segment, the blocks with the smallest (key, s, l, h, u).

    A segment is a run of consecutive sequences (default: each sequence its
    own).  Candidates of head instance g: logical blocks u < nb_g - protect.
    Takes min(budget, candidates) per segment.  Returns (flag [G, max_blocks]
    u8, count [G] i32, selected [nseg] i32)."""
    key = np.asarray(key, dtype=np.float32).reshape(st.G, st.max_blocks)
    if seg_offsets is None:
        seg_offsets = np.arange(st.S + 1)
    seg_offsets = np.asarray(seg_offsets, dtype=np.int64)
    nseg = seg_offsets.size - 1
    budget = np.asarray(budget, dtype=np.int64).reshape(nseg)
    if seg_offsets[0] != 0 or seg_offsets[-1] != st.S or (np.diff(seg_offsets) < 0).any():
        raise OracleError(ERR_ARG, "bad segment offsets")
    if (budget < 0).any() or protect_tail_blocks < 0:
        raise OracleError(ERR_ARG)
    flag = np.zeros((st.G, st.max_blocks), dtype=np.uint8)
    count = np.zeros(st.G, dtype=np.int32)
    selected = np.zeros(nseg, dtype=np.int32)
    lens = st.lens()
    per_seq = st.Lyr * st.Hk
    all_cands = []
    for sg in range(nseg):
        cands = []
        for g in range(seg_offsets[sg] * per_seq, seg_offsets[sg + 1] * per_seq):
            nb = -(-int(lens[g]) // st.b)
            for u in range(max(0, nb - protect_tail_blocks)):
                kv = key[g, u]
                if not (kv >= 0.0) or not np.isfinite(kv):
                    raise OracleError(ERR_NUMERIC, "negative, NaN or infinite block key")
                cands.append((float(kv), g, u))
        all_cands.append(cands)
    for sg, cands in enumerate(all_cands):
        cands.sort()  # (key, g, u): g ascending is (s, l, h) ascending
        take = min(int(budget[sg]), len(cands))
        for _, g, u in cands[:take]:
            flag[g, u] = 1
            count[g] += 1
        selected[sg] = take
    return flag, count, selected


# --------------------------------------------------------------------------
# compaction
# --------------------------------------------------------------------------

def _evicted_slots(st: State, g: int, flag_row):
    C = int(st.lens()[g])
    j = np.arange(C)
    return flag_row[j // st.b].astype(bool)


def compact(st: State, flag, count=None) -> int:
    """Move kept KVs out of each head's tail range into its evicted slots, shrink
    the head, free the tail blocks.  Returns the number of blocks freed.

    Per head: w = eviction mask over logical slots, n_ev = evicted real slots,
    T = C - n_ev.  holes = evicted slots below T, ascending; movers = kept slots
    at or above T, descending; the k-th mover goes to the k-th hole."""
    flag = np.asarray(flag, dtype=np.uint8).reshape(st.G, st.max_blocks)
    tab, lens = st.table(), st.lens()
    for g in range(st.G):
        nb = -(-int(lens[g]) // st.b)
        if flag[g, nb:].any():
            raise OracleError(ERR_ARG, "flag set beyond the head's blocks")
        if count is not None and int(np.asarray(count).reshape(-1)[g]) != int(flag[g].sum()):
            raise OracleError(ERR_ARG, "count does not match flags")
    freed = 0
    for g in range(st.G):
        C = int(lens[g])
        if C == 0 or not flag[g].any():
            continue
        freed += _move_and_free(st, g, _evicted_slots(st, g, flag[g]))
    return freed


def _move_and_free(st: State, g: int, w) -> int:
    """MoveCache on head g for the slot mask w (True = evicted), then the free step."""
    tab, lens = st.table(), st.lens()
    C = int(lens[g])
    T = C - int(np.sum(w))
    holes = [i for i in range(T) if w[i]]
    movers = [j for j in range(C - 1, T - 1, -1) if not w[j]]
    assert len(holes) == len(movers)
    for i, j in zip(holes, movers):
        ns, os_ = tab[g, j // st.b], j % st.b
        nd, od = tab[g, i // st.b], i % st.b
        st.k_cache[nd, od] = st.k_cache[ns, os_]
        st.v_cache[nd, od] = st.v_cache[ns, os_]
        st.metric[nd, od] = st.metric[ns, os_]
        st.pos[nd, od] = st.pos[ns, os_]
    nb, nb2 = -(-C // st.b), -(-T // st.b)
    for u in range(nb2, nb):
        st.free_map[tab[g, u]] = 1
        tab[g, u] = -1
    lens[g] = T
    return nb - nb2


# --------------------------------------------------------------------------
# the paper's own eviction schedule (rank blocks)
# --------------------------------------------------------------------------

def rank_schedule(st: State, budget, seg_offsets=None, protect_tail_blocks=1, metric=None):
    """The schedule of "Evicting from a Paged KV Cache", step by step.

    Per head: its metrics sorted ascending, the empty slots of its last block
    first (they count as zero and come before every real metric); the sorted
    list cut into rows of b; row e-1 holds what evicting the e-th block would
    remove, and its last column is m(h, e), the largest metric evicted with
    it.  Candidate rows of a head: e < ceil(C_h / b) (protect_tail_blocks = 1;
    0 lets a head lose every block).  Per segment the candidate rows of all its
    heads are ordered by that last column (ties: sequence, layer, head, row)
    and the first E rows are marked; the KVs of a marked row are evicted.
    Metrics are compared as f32; equal metrics of one head go in logical order.

    Returns (rows [G] i32 = blocks each head loses, masks = list of G boolean
    arrays over logical slots, selected [nseg] i32)."""
    M = st.metric if metric is None else np.asarray(metric).reshape(st.N, st.b)
    M32 = M.astype(np.float32)
    if seg_offsets is None:
        seg_offsets = np.arange(st.S + 1)
    seg_offsets = np.asarray(seg_offsets, dtype=np.int64)
    nseg = seg_offsets.size - 1
    budget = np.asarray(budget, dtype=np.int64).reshape(nseg)
    if seg_offsets[0] != 0 or seg_offsets[-1] != st.S or (np.diff(seg_offsets) < 0).any():
        raise OracleError(ERR_ARG, "bad segment offsets")
    if (budget < 0).any() or protect_tail_blocks < 0:
        raise OracleError(ERR_ARG)
    lens = st.lens()
    per_seq = st.Lyr * st.Hk
    rows = np.zeros(st.G, dtype=np.int32)
    masks = [np.zeros(int(lens[g]), dtype=bool) for g in range(st.G)]
    selected = np.zeros(nseg, dtype=np.int32)
    sorted_rows = {}   # g -> list of rows, each a list of (is_real, metric, logical index)
    for g in range(st.G):
        C = int(lens[g])
        if C == 0:
            sorted_rows[g] = []
            continue
        n, o = slots_of(st, g)
        vals = M32[n, o]
        if not (vals >= 0).all() or not np.isfinite(vals).all():
            raise OracleError(ERR_NUMERIC, "negative, NaN or infinite metric")
        nb = -(-C // st.b)
        entries = [(0, np.float32(0.0), -1)] * (nb * st.b - C) + \
                  sorted((1, vals[j], j) for j in range(C))
        sorted_rows[g] = [entries[e * st.b:(e + 1) * st.b] for e in range(nb)]
    for sg in range(nseg):
        cands = []
        for g in range(seg_offsets[sg] * per_seq, seg_offsets[sg + 1] * per_seq):
            r = sorted_rows[g]
            for e in range(max(0, len(r) - protect_tail_blocks)):
                cands.append((float(r[e][-1][1]), g, e))
        cands.sort()
        take = min(int(budget[sg]), len(cands))
        for _, g, e in cands[:take]:
            rows[g] += 1
            for is_real, _, j in sorted_rows[g][e]:
                if is_real:
                    masks[g][j] = True
        selected[sg] = take
    return rows, masks, selected


def compact_slots(st: State, masks) -> int:
    """MoveCache + free for an eviction mask over logical slots (one boolean array per head)."""
    freed = 0
    for g in range(st.G):
        w = np.asarray(masks[g], dtype=bool)
        if w.size != int(st.lens()[g]):
            raise OracleError(ERR_ARG, "mask length")
        if w.any():
            freed += _move_and_free(st, g, w)
    return freed


def movecache_sequential(w, C, n_ev):
    """The two-pointer loop of Algorithm 1 on one head, returning the (src, dst)
    logical-slot pairs in the order they are made.  w[j] = 1 when slot j is
    evicted; the eviction range is the last n_ev slots.  i advances after each
    move and stays below the range (the printed listing omits both)."""
    moves = []
    i = 0
    j = C - 1
    end = j - n_ev
    while j > end:
        if not w[j]:
            while i <= end and not w[i]:
                i += 1
            if i > end:
                raise AssertionError("no hole left for a kept KV")
            moves.append((j, i))
            i += 1
        j -= 1
    return moves
