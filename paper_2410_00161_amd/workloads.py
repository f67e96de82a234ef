"""Seeded synthetic inputs for the head-variable paged KV cache.

This module only lays out data: shapes, random values, retained lengths and
block placements.  It holds none of the method's arithmetic (no attention, no
metric, no selection, no compaction) so that both the CPU oracle's tests and
the HIP path's tests can draw the same inputs from it without sharing any of
the computation under test.

Notation follows the paper (Method, "Block Layout and Parallel Allocation"):
S sequences, Lyr layers, Hk KV heads, r query heads per KV head, d head
dimension, b block size, N physical blocks.  A head instance is g = (s, l, h),
flat index (s*Lyr + l)*Hk + h; it owns ceil(C_g / b) blocks of the unified
[N, b, d] cache.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import torch


@dataclass(frozen=True)
class Shape:
    """Immutable description of one cache; mirrors the C struct kvc_config."""

    num_seqs: int
    num_layers: int
    num_kv_heads: int
    group_size: int
    head_dim: int
    block_size: int
    num_blocks: int
    max_blocks_per_head: int
    kv_dtype: str = "bf16"  # "bf16" | "f32" | "fp8" (OCP e4m3 K and V, bf16 queries)

    @property
    def G(self) -> int:
        return self.num_seqs * self.num_layers * self.num_kv_heads

    @property
    def num_q_heads(self) -> int:
        return self.num_kv_heads * self.group_size

    @property
    def torch_dtype(self) -> torch.dtype:
        return {"bf16": torch.bfloat16, "f32": torch.float32, "fp8": torch.float8_e4m3fn}[self.kv_dtype]

    @property
    def q_torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.kv_dtype == "f32" else torch.bfloat16

    @property
    def kv_bytes(self) -> int:
        return {"bf16": 2, "f32": 4, "fp8": 1}[self.kv_dtype]


@dataclass
class Cache:
    """Mutable cache state as plain tensors (device chosen by the caller)."""

    shape: Shape
    k_cache: torch.Tensor      # [N, b, d] kv dtype
    v_cache: torch.Tensor      # [N, b, d] kv dtype
    metric: torch.Tensor       # [N, b] f32
    pos: torch.Tensor          # [N, b] i32, logical index of the KV in a slot
    block_table: torch.Tensor  # [S, Lyr, Hk, max_blocks] i32, -1 = none
    ctx_len: torch.Tensor      # [S, Lyr, Hk] i32
    free_map: torch.Tensor     # [N] u8, 1 = free
    heavy: torch.Tensor | None = field(default=None)  # [N, b] bool, heavy-hitter slots

    def clone(self) -> "Cache":
        return Cache(self.shape, self.k_cache.clone(), self.v_cache.clone(),
                     self.metric.clone(), self.pos.clone(), self.block_table.clone(),
                     self.ctx_len.clone(), self.free_map.clone(),
                     None if self.heavy is None else self.heavy.clone())

    def to(self, device) -> "Cache":
        mv = lambda t: None if t is None else t.to(device)
        return Cache(self.shape, mv(self.k_cache), mv(self.v_cache), mv(self.metric),
                     mv(self.pos), mv(self.block_table), mv(self.ctx_len),
                     mv(self.free_map), mv(self.heavy))


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def loguniform_bounds(L: int, rho: float, b: int) -> tuple[float, float]:
    """Bounds [lo, hi] of a log-uniform law on token counts with mean L / rho.

    The mean of a log-uniform law on [lo, hi] is (hi - lo) / ln(hi / lo).
    Rule: keep lo = b and bisect hi <= L; if even hi = L falls short of the
    target mean, keep hi = L and bisect lo >= b instead.
    """
    target = L / rho
    mean = lambda lo, hi: (hi - lo) / math.log(hi / lo) if hi > lo * (1 + 1e-12) else lo
    if target <= b:
        return float(b), float(b)
    if mean(b, L) >= target:
        a, c = float(b), float(L)
        for _ in range(200):
            m = 0.5 * (a + c)
            if mean(b, m) < target:
                a = m
            else:
                c = m
        return float(b), 0.5 * (a + c)
    a, c = float(b), float(L)
    for _ in range(200):
        m = 0.5 * (a + c)
        if mean(m, L) < target:
            a = m
        else:
            c = m
    return 0.5 * (a + c), float(L)


def loguniform_lengths(G: int, L: int, rho: float, b: int, seed: int) -> torch.Tensor:
    """Retained KV count per head instance, in tokens (partial tail blocks occur).

    Stands in for the state a long-running, previously compressed batch reaches
    under variable-head-rate eviction: lengths spread over orders of magnitude,
    mean L / rho, never below one block.
    """
    lo, hi = loguniform_bounds(L, rho, b)
    u = torch.rand(G, generator=_gen(seed, "cpu"), dtype=torch.float64)
    c = torch.floor(torch.exp(math.log(lo) + u * (math.log(hi) - math.log(lo))))
    return c.clamp_(min=b, max=L).to(torch.int32)


def uniform_lengths(G: int, L: int) -> torch.Tensor:
    return torch.full((G,), L, dtype=torch.int32)


def blocks_needed(ctx_len: torch.Tensor, b: int) -> torch.Tensor:
    return (ctx_len.to(torch.int64) + b - 1) // b


def pool_size(ctx_len: torch.Tensor, b: int, slack: float = 1.25, extra: int = 0) -> int:
    return int(math.ceil(float(blocks_needed(ctx_len, b).sum()) * slack)) + int(extra)


def place_blocks(shape: Shape, ctx_len: torch.Tensor, seed: int,
                 placement: str = "fresh") -> tuple[torch.Tensor, torch.Tensor]:
    """Block tables and free map for the given per-head lengths.

    "fresh": head instances in ascending g take consecutive block ids from 0,
    the picture right after a prefill into an empty pool.  "fragmented": the
    same number of blocks but drawn from a seeded permutation of the whole
    pool, the picture after many rounds of freeing and re-allocating.
    """
    G, maxb, N = shape.G, shape.max_blocks_per_head, shape.num_blocks
    nb = blocks_needed(ctx_len.reshape(-1), shape.block_size)
    total = int(nb.sum())
    if total > N:
        raise ValueError(f"pool too small: need {total} blocks, have {N}")
    if int(nb.max()) > maxb:
        raise ValueError("max_blocks_per_head too small")
    if placement == "fresh":
        ids = torch.arange(total, dtype=torch.int32)
    elif placement == "fragmented":
        ids = torch.randperm(N, generator=_gen(seed + 7919, "cpu"))[:total].to(torch.int32)
    else:
        raise ValueError(placement)
    table = torch.full((G, maxb), -1, dtype=torch.int32)
    col = torch.arange(maxb, dtype=torch.int64).unsqueeze(0).expand(G, maxb)
    mask = col < nb.unsqueeze(1)
    table[mask] = ids  # row-major fill: ascending g, then ascending logical block
    free_map = torch.ones(N, dtype=torch.uint8)
    free_map[ids.long()] = 0
    return (table.reshape(shape.num_seqs, shape.num_layers, shape.num_kv_heads, maxb),
            free_map)


def _owner_of_block(shape: Shape, block_table: torch.Tensor) -> torch.Tensor:
    """[N] int64: head instance that holds each block, -1 when free."""
    G, maxb = shape.G, shape.max_blocks_per_head
    t = block_table.reshape(G, maxb).long()
    g = torch.arange(G, device=t.device).unsqueeze(1).expand(G, maxb)
    owner = torch.full((shape.num_blocks,), -1, dtype=torch.int64, device=t.device)
    m = t >= 0
    owner[t[m]] = g[m]
    return owner


def make_cache(shape: Shape, ctx_len: torch.Tensor, seed: int, device="cpu",
               placement: str = "fresh", heavy_frac: float = 0.02,
               heavy_scale: float = 3.0, init_metric: str = "zero") -> Cache:
    """A populated cache: q-independent part of a workload.

    K, V ~ N(0, 1) rounded to the cache dtype.  A fraction `heavy_frac` of the
    slots (Bernoulli per slot) hold keys equal to `heavy_scale` times a random
    unit direction drawn once per head instance ("heavy hitters").  The whole
    pool is filled, so unowned and empty slots hold finite garbage as a real
    pool would.  init_metric: "zero", or "prefill" = |N(0,1)| * 1e-2 per slot
    plus 1 on heavy-hitter slots, standing for metrics left by a prefill.
    """
    dev = torch.device(device)
    N, b, d = shape.num_blocks, shape.block_size, shape.head_dim
    table, free_map = place_blocks(shape, ctx_len, seed, placement)
    table, free_map = table.to(dev), free_map.to(dev)
    g = _gen(seed, dev)
    dt = shape.torch_dtype
    # filled in slabs so that the f32 draw of a very large pool never exists whole
    k = torch.empty((N, b, d), device=dev, dtype=dt)
    v = torch.empty((N, b, d), device=dev, dtype=dt)
    slab = 1 << 17
    for t in (k, v):
        for lo in range(0, N, slab):
            hi = min(N, lo + slab)
            t[lo:hi] = torch.randn((hi - lo, b, d), generator=g, device=dev, dtype=torch.float32).to(dt)
    heavy = torch.rand((N, b), generator=g, device=dev) < heavy_frac
    u = torch.randn((shape.G, d), generator=g, device=dev, dtype=torch.float32)
    u = u / u.norm(dim=1, keepdim=True)
    owner = _owner_of_block(shape, table)
    rows = heavy & (owner >= 0).unsqueeze(1)
    if bool(rows.any()):
        own = owner.unsqueeze(1).expand(N, b)[rows]
        vals = (heavy_scale * u[own]).to(dt)
        if shape.kv_dtype == "fp8":   # 8-bit floats are moved as bytes: indexing knows no such type
            k.view(torch.uint8)[rows] = vals.view(torch.uint8)
        else:
            k[rows] = vals
    if init_metric == "zero":
        metric = torch.zeros((N, b), device=dev, dtype=torch.float32)
    elif init_metric == "prefill":
        metric = torch.randn((N, b), generator=g, device=dev, dtype=torch.float32).abs_() * 1e-2
        metric += heavy.to(torch.float32)
    else:
        raise ValueError(init_metric)
    # logical index = position of the slot in its head's ordering
    pos = torch.full((N, b), -1, dtype=torch.int32, device=dev)
    t = table.reshape(shape.G, -1).long()
    m = t >= 0
    u_idx = torch.arange(t.shape[1], device=dev).unsqueeze(0).expand_as(t)[m]
    base = (u_idx * b).unsqueeze(1) + torch.arange(b, device=dev).unsqueeze(0)
    pos[t[m]] = base.to(torch.int32)
    ctx = ctx_len.reshape(shape.num_seqs, shape.num_layers, shape.num_kv_heads).to(torch.int32).to(dev)
    return Cache(shape, k, v, metric, pos, table, ctx.contiguous(), free_map, heavy)


def make_query(shape: Shape, seed: int, step: int = 0, device="cpu") -> torch.Tensor:
    """Decode-step queries [S, Lyr, Hq, d] ~ N(0, 1) in the query dtype of the cache."""
    dev = torch.device(device)
    g = _gen(seed * 1_000_003 + 17 * step + 1, dev)
    q = torch.randn((shape.num_seqs, shape.num_layers, shape.num_q_heads, shape.head_dim),
                    generator=g, device=dev, dtype=torch.float32)
    return q.to(shape.q_torch_dtype)


def make_new_kv(shape: Shape, seed: int, step: int = 0, device="cpu"):
    """The new token's k, v for every head instance: two [S, Lyr, Hk, d] tensors."""
    dev = torch.device(device)
    g = _gen(seed * 1_000_003 + 17 * step + 2, dev)
    sz = (shape.num_seqs, shape.num_layers, shape.num_kv_heads, shape.head_dim)
    k = torch.randn(sz, generator=g, device=dev, dtype=torch.float32).to(shape.torch_dtype)
    v = torch.randn(sz, generator=g, device=dev, dtype=torch.float32).to(shape.torch_dtype)
    return k, v


# ---------------------------------------------------------------------------
# Named workloads (shapes of the benchmark configurations)
# ---------------------------------------------------------------------------

def tiny_ref(seed: int = 1001):
    """1 layer, 4 q / 2 KV heads, d = 64, f32 KV, b = 16, 2 sequences x 512 tokens."""
    S, Lyr, Hk, r, d, b, L = 2, 1, 2, 2, 64, 16, 512
    ctx = uniform_lengths(S * Lyr * Hk, L)
    N = pool_size(ctx, b, 1.25, 8)
    shape = Shape(S, Lyr, Hk, r, d, b, N, L // b + 4, "f32")
    return shape, ctx, seed


def llama8b_decode(seed: int = 1002, num_seqs: int = 64, prompt: int = 8192,
                   rho: float = 8.0, extra_tokens: int = 160, block_size: int = 16):
    """32 layers, 32 q / 8 KV heads, d = 128, bf16, b = 16 (or block_size); log-uniform retention."""
    S, Lyr, Hk, r, d, b = num_seqs, 32, 8, 4, 128, block_size
    ctx = loguniform_lengths(S * Lyr * Hk, prompt, rho, b, seed)
    maxb = (prompt + extra_tokens + b - 1) // b + 1
    N = pool_size(ctx, b, 1.25, S * Lyr * Hk * ((extra_tokens + b - 1) // b))
    shape = Shape(S, Lyr, Hk, r, d, b, N, maxb, "bf16")
    return shape, ctx, seed


def llama70b_decode(seed: int = 1005, num_seqs: int = 16, prompt: int = 131072,
                    rho: float = 8.0, extra_tokens: int = 96):
    """80 layers, 64 q / 8 KV heads (group of 8), d = 128, bf16, b = 16."""
    S, Lyr, Hk, r, d, b = num_seqs, 80, 8, 8, 128, 16
    ctx = loguniform_lengths(S * Lyr * Hk, prompt, rho, b, seed)
    maxb = (prompt + extra_tokens + b - 1) // b + 1
    N = pool_size(ctx, b, 1.1, S * Lyr * Hk * ((extra_tokens + b - 1) // b))
    shape = Shape(S, Lyr, Hk, r, d, b, N, maxb, "bf16")
    return shape, ctx, seed


def small_mixed(seed: int, S=3, Lyr=2, Hk=2, r=4, d=128, b=16, L=700, rho=3.0,
                kv_dtype="bf16", slack=1.5, extra_blocks=4):
    """A small ragged case: several tiles, partial tail blocks, sizes the oracle
    finishes in seconds."""
    ctx = loguniform_lengths(S * Lyr * Hk, L, rho, b, seed)
    N = pool_size(ctx, b, slack, S * Lyr * Hk * extra_blocks)
    maxb = (L + b - 1) // b + extra_blocks
    shape = Shape(S, Lyr, Hk, r, d, b, N, maxb, kv_dtype)
    return shape, ctx, seed


def gather_heads(cache: Cache, heads, q: torch.Tensor | None = None):
    """Copies the chosen head instances into a small CPU cache of its own.

    The result has S' = len(heads), one layer, one KV head; its blocks are
    renumbered 0, 1, 2, ... in table order.  Returns (small_cache, q_small)
    where q_small [S', 1, r, d] holds the query rows of those heads.  Pure data
    movement: lets a CPU check run on a sample of a cache too large for the host.
    """
    sh = cache.shape
    heads = [int(g) for g in heads]
    G, maxb, b = sh.G, sh.max_blocks_per_head, sh.block_size
    table = cache.block_table.reshape(G, maxb)
    ctx = cache.ctx_len.reshape(G)
    idx = torch.tensor(heads, dtype=torch.long, device=table.device)
    rows = table[idx].cpu()
    lens = ctx[idx].cpu()
    held = (rows >= 0).sum(1)
    total = int(held.sum())
    new_table = torch.full((len(heads), maxb), -1, dtype=torch.int32)
    src_ids = rows[rows >= 0].long()
    new_table[rows >= 0] = torch.arange(total, dtype=torch.int32)
    small_shape = Shape(len(heads), 1, 1, sh.group_size, sh.head_dim, b, max(total, 1), maxb, sh.kv_dtype)
    dev_ids = src_ids.to(cache.k_cache.device)
    def take(t):
        if t.dtype == torch.float8_e4m3fn:   # moved as bytes
            return take(t.view(torch.uint8)).view(torch.float8_e4m3fn)
        return t[dev_ids].cpu() if total else t[:1].cpu()
    small = Cache(small_shape, take(cache.k_cache), take(cache.v_cache), take(cache.metric),
                  take(cache.pos), new_table.reshape(len(heads), 1, 1, maxb),
                  lens.to(torch.int32).reshape(len(heads), 1, 1),
                  torch.zeros(max(total, 1), dtype=torch.uint8) if total else torch.ones(1, dtype=torch.uint8),
                  None)
    q_small = None
    if q is not None:
        r, d = sh.group_size, sh.head_dim
        q_small = q.reshape(G, r, d)[idx.to(q.device)].cpu().reshape(len(heads), 1, r, d)
    return small, q_small
