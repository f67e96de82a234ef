"""A cache on one GPU plus its workspace: holds the tensors alive and forwards
to the C entry points.  No computation happens here."""
from __future__ import annotations

import torch

from . import binding as B


class KvcSession:
    def __init__(self, cache, metric_mode=B.KVC_L2, device="cuda:0", with_pos=True):
        """cache: workloads.Cache (any device); tensors are moved to `device`.  with_pos=False
        hands the library a state whose `pos` is NULL (logical indices not tracked)."""
        self.device = torch.device(device)
        sh = cache.shape
        self.shape = sh
        self.cache = cache.to(self.device)
        c = self.cache
        self.cfg = B.make_config(sh.num_seqs, sh.num_layers, sh.num_kv_heads, sh.group_size,
                                 sh.head_dim, sh.block_size, sh.num_blocks, sh.max_blocks_per_head,
                                 sh.kv_dtype, metric_mode)
        for name in ("k_cache", "v_cache", "metric", "pos", "block_table", "ctx_len", "free_map"):
            setattr(c, name, getattr(c, name).contiguous())
        self.st = B.make_state(c.k_cache, c.v_cache, c.metric, c.pos if with_pos else None, c.block_table,
                               c.ctx_len, c.free_map)
        torch.cuda.set_device(self.device)
        self.ws = B.new_workspace(self.cfg, self.device)
        G, maxb = sh.G, sh.max_blocks_per_head
        self.out = torch.zeros((sh.num_seqs, sh.num_layers, sh.num_q_heads, sh.head_dim),
                               dtype=torch.float32, device=self.device)
        self.block_key = torch.zeros((G, maxb), dtype=torch.float32, device=self.device)
        self.evict_flag = torch.zeros((G, maxb), dtype=torch.uint8, device=self.device)
        self.evict_count = torch.zeros((G,), dtype=torch.int32, device=self.device)
        self.blocks_freed = torch.zeros((1,), dtype=torch.int64, device=self.device)

    # one method per entry point, same names
    def block_alloc(self, n_new, flags=0):
        B.kvc_block_alloc(self.cfg, self.st, n_new.to(self.device, torch.int32).contiguous(), self.ws,
                          flags=flags)

    def block_free(self, n_drop, flags=0) -> int:
        return B.kvc_block_free(self.cfg, self.st, n_drop.to(self.device, torch.int32).contiguous(),
                                self.ws, flags=flags)

    def check_state(self, flags=0):
        """Raises KvcError(KVC_ERR_ARG) when the tables, lengths and free map contradict each other."""
        B.kvc_check_state(self.cfg, self.st, self.ws, flags=flags)

    def append(self, k_new, v_new, new_pos=None, layer_begin=0, layer_end=None, flags=0):
        layer_end = self.shape.num_layers if layer_end is None else layer_end
        B.kvc_append(self.cfg, self.st, k_new, v_new, new_pos, layer_begin, layer_end, self.ws,
                     flags=flags)

    def paged_decode(self, q, accumulate_metric=True, layer_begin=0, layer_end=None, out=None):
        layer_end = self.shape.num_layers if layer_end is None else layer_end
        out = self.out if out is None else out
        B.kvc_paged_decode(self.cfg, self.st, q, out, layer_begin, layer_end, accumulate_metric, self.ws)
        return out

    def decode_plan(self, ctx_plus=0):
        B.kvc_decode_plan(self.cfg, self.st, ctx_plus, self.ws)

    def paged_decode_planned(self, q, layer, accumulate_metric=True, out=None):
        out = self.out if out is None else out
        B.kvc_paged_decode_planned(self.cfg, self.st, q, out, layer, accumulate_metric, self.ws)
        return out

    def metric_reduce(self, key_mode=B.KVC_KEY_SUM):
        B.kvc_metric_reduce(self.cfg, self.st, self.block_key, self.ws, key_mode=key_mode)
        return self.block_key

    def evict_select(self, budget, seg_offsets=None, protect_tail_blocks=1, block_key=None, flags=0):
        budget = budget.to(self.device, torch.int32).contiguous()
        nseg = budget.numel()
        if seg_offsets is not None:
            seg_offsets = seg_offsets.to(self.device, torch.int32).contiguous()
        selected = torch.zeros((nseg,), dtype=torch.int32, device=self.device)
        key = self.block_key if block_key is None else block_key
        B.kvc_evict_select(self.cfg, self.st, key, seg_offsets, budget, nseg, protect_tail_blocks,
                           self.evict_flag, self.evict_count, selected, self.ws, flags=flags)
        return self.evict_flag, self.evict_count, selected

    def compact(self, evict_flag=None, evict_count=None, flags=0):
        B.kvc_compact(self.cfg, self.st, self.evict_flag if evict_flag is None else evict_flag,
                      self.evict_count if evict_count is None else evict_count, self.blocks_freed,
                      self.ws, flags=flags)
        return self.blocks_freed

    def evict_rank_select(self, budget, seg_offsets=None, protect_tail_blocks=1, flags=0):
        budget = budget.to(self.device, torch.int32).contiguous()
        nseg = budget.numel()
        if seg_offsets is not None:
            seg_offsets = seg_offsets.to(self.device, torch.int32).contiguous()
        selected = torch.zeros((nseg,), dtype=torch.int32, device=self.device)
        B.kvc_evict_rank_select(self.cfg, self.st, seg_offsets, budget, nseg, protect_tail_blocks,
                                self.evict_count, selected, self.ws, flags=flags)
        return self.evict_count, selected

    def compact_rank(self, evict_rows=None, flags=0):
        B.kvc_compact_rank(self.cfg, self.st, self.evict_count if evict_rows is None else evict_rows,
                           self.blocks_freed, self.ws, flags=flags)
        return self.blocks_freed

    def compression_batch(self, last_compressed, kv_limit, running=None):
        S = self.shape.num_seqs
        in_batch = torch.zeros(S, dtype=torch.uint8, device=self.device)
        kvs = torch.zeros(1, dtype=torch.int64, device=self.device)
        B.kvc_compression_batch(self.cfg, self.st, last_compressed.to(self.device, torch.int64).contiguous(),
                                None if running is None else running.to(self.device, torch.uint8).contiguous(),
                                kv_limit, in_batch, kvs, self.ws)
        return in_batch, kvs

    def window_metric(self, q_win, w, pool=7, accumulate=False, layer_begin=0, layer_end=None, row_lse=None):
        layer_end = self.shape.num_layers if layer_end is None else layer_end
        B.kvc_window_metric(self.cfg, self.st, q_win, row_lse, w, pool, accumulate, layer_begin, layer_end, self.ws)
        return self.cache.metric

    def query_block_metric(self, q_blk, w, first_pos, exclude=0, layer_begin=0, layer_end=None, row_lse=None):
        layer_end = self.shape.num_layers if layer_end is None else layer_end
        B.kvc_query_block_metric(self.cfg, self.st, q_blk, row_lse, w, first_pos, exclude, layer_begin, layer_end,
                                 self.ws)
        return self.cache.metric
