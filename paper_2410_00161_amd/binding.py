"""ctypes binding of libkvc.so: argument marshalling only.

Every function here has the name and the argument order of the C entry point
it calls (include/kvc.h).  Tensors are torch tensors used as device memory;
the stream is torch's current stream unless one is given.  Nothing is computed
in Python and there is no fallback: a missing library raises at first use.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libkvc.so")

KVC_OK, KVC_ERR_ARG, KVC_ERR_OOM, KVC_ERR_TABLE_FULL = 0, 1, 2, 3
KVC_ERR_NUMERIC, KVC_ERR_HIP, KVC_ERR_UNSUPPORTED = 5, 6, 7
KVC_F32, KVC_BF16, KVC_FP8_E4M3 = 0, 1, 2
KVC_L2, KVC_L1 = 0, 1
KVC_KEY_SUM, KVC_KEY_MAX = 0, 1
KVC_ASYNC = 1

EXPORTS = [
    "kvc_workspace_bytes", "kvc_validate", "kvc_status_string", "kvc_workspace_reset",
    "kvc_poll_status", "kvc_check_state", "kvc_block_alloc", "kvc_block_free", "kvc_append", "kvc_paged_decode", "kvc_paged_decode_static", "kvc_decode_plan", "kvc_paged_decode_planned",
    "kvc_metric_reduce", "kvc_evict_select", "kvc_compact", "kvc_set_decode_chunk",
    "kvc_get_decode_chunk", "kvc_get_decode_short", "kvc_evict_rank_select", "kvc_compact_rank", "kvc_window_metric", "kvc_query_block_metric", "kvc_count_blocks", "kvc_prefill_alloc", "kvc_preempt", "kvc_compression_batch",
    "kvc_profile_begin", "kvc_profile_enable", "kvc_profile_collect", "kvc_stream_read_probe",
    "kvc_stream_read_add_probe",
]


class kvc_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "num_seqs", "num_layers", "num_kv_heads", "group_size", "head_dim", "block_size",
        "num_blocks", "max_blocks_per_head", "kv_dtype", "metric_mode")]


class kvc_state(C.Structure):
    _fields_ = [("k_cache", C.c_void_p), ("v_cache", C.c_void_p), ("metric", C.c_void_p),
                ("pos", C.c_void_p), ("block_table", C.c_void_p), ("ctx_len", C.c_void_p),
                ("free_map", C.c_void_p)]


class KvcError(RuntimeError):
    def __init__(self, code: int, where: str):
        super().__init__(f"{where}: {status_string(code)} ({code})")
        self.code = code


_lib = None


def lib() -> C.CDLL:
    """Loads libkvc.so (built by paper_2410_00161_amd.build).  No fallback."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2410_00161_amd.build`")
        L = C.CDLL(LIB_PATH)
        P, I = C.c_void_p, C.c_int
        cfgp, stp = C.POINTER(kvc_config), C.POINTER(kvc_state)
        L.kvc_workspace_bytes.restype = C.c_size_t
        L.kvc_workspace_bytes.argtypes = [cfgp]
        L.kvc_validate.argtypes = [cfgp, stp]
        L.kvc_status_string.restype = C.c_char_p
        L.kvc_status_string.argtypes = [I]
        L.kvc_workspace_reset.argtypes = [cfgp, P, P]
        L.kvc_poll_status.argtypes = [cfgp, P, P, C.POINTER(C.c_int)]
        L.kvc_block_alloc.argtypes = [cfgp, stp, P, P, P, I]
        L.kvc_block_free.argtypes = [cfgp, stp, P, C.POINTER(C.c_int64), P, P, I]
        L.kvc_append.argtypes = [cfgp, stp, P, P, P, I, I, P, P, I]
        L.kvc_paged_decode.argtypes = [cfgp, stp, P, P, I, I, I, P, P]
        L.kvc_paged_decode_static.argtypes = [cfgp, stp, P, P, I, I, I, P]
        L.kvc_decode_plan.argtypes = [cfgp, stp, I, P, P]
        L.kvc_paged_decode_planned.argtypes = [cfgp, stp, P, P, I, I, P, P]
        L.kvc_metric_reduce.argtypes = [cfgp, stp, P, I, P, P]
        L.kvc_evict_select.argtypes = [cfgp, stp, P, P, P, I, I, P, P, P, P, P, I]
        L.kvc_compact.argtypes = [cfgp, stp, P, P, P, P, P, I]
        L.kvc_set_decode_chunk.argtypes = [I]
        L.kvc_evict_rank_select.argtypes = [cfgp, stp, P, P, I, I, P, P, P, P, I]
        L.kvc_compact_rank.argtypes = [cfgp, stp, P, P, P, P, I]
        L.kvc_count_blocks.argtypes = [cfgp, stp, I, I, P, P, P, P]
        L.kvc_prefill_alloc.argtypes = [cfgp, stp, P, P, P, I]
        L.kvc_preempt.argtypes = [cfgp, stp, P, C.POINTER(C.c_int64), P, P, I]
        L.kvc_check_state.argtypes = [cfgp, stp, P, P, I]
        L.kvc_compression_batch.argtypes = [cfgp, stp, P, P, C.c_int64, P, P, P, P]
        L.kvc_window_metric.argtypes = [cfgp, stp, P, P, I, I, I, I, I, P, P]
        L.kvc_query_block_metric.argtypes = [cfgp, stp, P, P, I, I, I, I, I, P, P]
        L.kvc_get_decode_chunk.argtypes = [cfgp, C.POINTER(C.c_int)]
        L.kvc_get_decode_short.argtypes = [cfgp, C.POINTER(C.c_int)]
        L.kvc_profile_begin.argtypes = [I]
        L.kvc_profile_enable.argtypes = [I]
        L.kvc_stream_read_probe.argtypes = [P, C.c_size_t, P, I, P]
        L.kvc_stream_read_add_probe.argtypes = [P, C.c_size_t, C.c_size_t, I, P, C.c_size_t, P, I, P]
        L.kvc_profile_collect.argtypes = [P, P, P, I, C.POINTER(C.c_int)]
        for n in EXPORTS:
            if n not in ("kvc_workspace_bytes", "kvc_status_string"):
                getattr(L, n).restype = I
        _lib = L
    return _lib


def status_string(code: int) -> str:
    return lib().kvc_status_string(int(code)).decode()


def _ptr(t, dtype=None):
    if t is None:
        return None
    if not isinstance(t, torch.Tensor):
        raise TypeError("expected a torch tensor")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        return C.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, torch.cuda.Stream):
        return C.c_void_p(stream.cuda_stream)
    return C.c_void_p(int(stream))


def _check(rc: int, where: str):
    if rc != KVC_OK:
        raise KvcError(rc, where)


def make_config(num_seqs, num_layers, num_kv_heads, group_size, head_dim, block_size,
                num_blocks, max_blocks_per_head, kv_dtype, metric_mode=KVC_L2) -> kvc_config:
    if isinstance(kv_dtype, str):
        kv_dtype = {"bf16": KVC_BF16, "f32": KVC_F32, "fp8": KVC_FP8_E4M3}[kv_dtype]
    return kvc_config(num_seqs, num_layers, num_kv_heads, group_size, head_dim, block_size,
                      num_blocks, max_blocks_per_head, kv_dtype, metric_mode)


def make_state(k_cache, v_cache, metric, pos, block_table, ctx_len, free_map) -> kvc_state:
    """Wraps device tensors; the caller keeps them alive."""
    st = kvc_state(_ptr(k_cache), _ptr(v_cache), _ptr(metric, torch.float32),
                   _ptr(pos, torch.int32) if pos is not None else None,
                   _ptr(block_table, torch.int32), _ptr(ctx_len, torch.int32),
                   _ptr(free_map, torch.uint8))
    return st


def kvc_workspace_bytes(cfg) -> int:
    return int(lib().kvc_workspace_bytes(C.byref(cfg)))


def kvc_validate(cfg, st=None) -> int:
    return int(lib().kvc_validate(C.byref(cfg), C.byref(st) if st is not None else None))


def new_workspace(cfg, device) -> torch.Tensor:
    n = kvc_workspace_bytes(cfg)
    if n == 0:
        raise KvcError(KVC_ERR_ARG, "kvc_workspace_bytes")
    ws = torch.empty(n + 256, dtype=torch.uint8, device=device)
    off = (-ws.data_ptr()) % 256
    ws = ws[off:off + n]
    with torch.cuda.device(device):
        kvc_workspace_reset(cfg, ws)
    return ws


def kvc_workspace_reset(cfg, ws, stream=None):
    _check(lib().kvc_workspace_reset(C.byref(cfg), _ptr(ws), _stream(stream)), "kvc_workspace_reset")


def kvc_poll_status(cfg, ws, stream=None) -> int:
    out = C.c_int(0)
    _check(lib().kvc_poll_status(C.byref(cfg), _ptr(ws), _stream(stream), C.byref(out)), "kvc_poll_status")
    return out.value


def kvc_check_state(cfg, st, ws, stream=None, flags=0):
    _check(lib().kvc_check_state(C.byref(cfg), C.byref(st), _ptr(ws), _stream(stream), flags), "kvc_check_state")


def kvc_block_alloc(cfg, st, n_new, ws, stream=None, flags=0):
    _check(lib().kvc_block_alloc(C.byref(cfg), C.byref(st), _ptr(n_new, torch.int32), _ptr(ws),
                                 _stream(stream), flags), "kvc_block_alloc")


def kvc_block_free(cfg, st, n_drop, ws, stream=None, flags=0) -> int:
    freed = C.c_int64(0)
    _check(lib().kvc_block_free(C.byref(cfg), C.byref(st), _ptr(n_drop, torch.int32), C.byref(freed),
                                _ptr(ws), _stream(stream), flags), "kvc_block_free")
    return freed.value


def kvc_append(cfg, st, k_new, v_new, new_pos, layer_begin, layer_end, ws, stream=None, flags=0):
    _check(lib().kvc_append(C.byref(cfg), C.byref(st), _ptr(k_new), _ptr(v_new),
                            _ptr(new_pos, torch.int32) if new_pos is not None else None,
                            layer_begin, layer_end, _ptr(ws), _stream(stream), flags), "kvc_append")


def kvc_paged_decode(cfg, st, q, out, layer_begin, layer_end, accumulate_metric, ws, stream=None):
    _check(lib().kvc_paged_decode(C.byref(cfg), C.byref(st), _ptr(q), _ptr(out, torch.float32),
                                  layer_begin, layer_end, int(accumulate_metric), _ptr(ws),
                                  _stream(stream)), "kvc_paged_decode")


def kvc_decode_plan(cfg, st, ctx_plus, ws, stream=None):
    _check(lib().kvc_decode_plan(C.byref(cfg), C.byref(st), int(ctx_plus), _ptr(ws), _stream(stream)), "kvc_decode_plan")


def kvc_paged_decode_planned(cfg, st, q, out, layer, accumulate_metric, ws, stream=None):
    _check(lib().kvc_paged_decode_planned(C.byref(cfg), C.byref(st), _ptr(q), _ptr(out, torch.float32), int(layer),
                                          int(accumulate_metric), _ptr(ws), _stream(stream)), "kvc_paged_decode_planned")


KVC_STATIC_SCRATCH_BYTES = 32 << 20


def kvc_paged_decode_static(cfg, st, q, out, layer_begin, layer_end, accumulate_metric, stream=None):
    _check(lib().kvc_paged_decode_static(C.byref(cfg), C.byref(st), _ptr(q), _ptr(out, torch.float32),
                                         layer_begin, layer_end, int(accumulate_metric), _stream(stream)),
           "kvc_paged_decode_static")


def kvc_metric_reduce(cfg, st, block_key, ws, stream=None, key_mode=KVC_KEY_SUM):
    _check(lib().kvc_metric_reduce(C.byref(cfg), C.byref(st), _ptr(block_key, torch.float32), int(key_mode),
                                   _ptr(ws), _stream(stream)), "kvc_metric_reduce")


def kvc_evict_select(cfg, st, block_key, seg_offsets, budget, nseg, protect_tail_blocks, evict_flag,
                     evict_count, selected, ws, stream=None, flags=0):
    _check(lib().kvc_evict_select(C.byref(cfg), C.byref(st), _ptr(block_key, torch.float32),
                                  _ptr(seg_offsets, torch.int32) if seg_offsets is not None else None,
                                  _ptr(budget, torch.int32), nseg, protect_tail_blocks,
                                  _ptr(evict_flag, torch.uint8), _ptr(evict_count, torch.int32),
                                  _ptr(selected, torch.int32), _ptr(ws), _stream(stream), flags),
           "kvc_evict_select")


def kvc_compact(cfg, st, evict_flag, evict_count, blocks_freed, ws, stream=None, flags=0):
    _check(lib().kvc_compact(C.byref(cfg), C.byref(st), _ptr(evict_flag, torch.uint8),
                             _ptr(evict_count, torch.int32),
                             _ptr(blocks_freed, torch.int64) if blocks_freed is not None else None,
                             _ptr(ws), _stream(stream), flags), "kvc_compact")


def kvc_set_decode_chunk(tokens: int):
    _check(lib().kvc_set_decode_chunk(int(tokens)), "kvc_set_decode_chunk")


def kvc_profile_begin(n: int):
    _check(lib().kvc_profile_begin(int(n)), "kvc_profile_begin")


def kvc_profile_collect(cap: int = 4096):
    """Returns (chunk_ms, short_ms, combine_ms) lists of the recorded decode calls."""
    a = (C.c_float * cap)()
    sh = (C.c_float * cap)()
    b = (C.c_float * cap)()
    n = C.c_int(0)
    _check(lib().kvc_profile_collect(a, sh, b, cap, C.byref(n)), "kvc_profile_collect")
    k = min(n.value, cap)
    return list(a[:k]), list(sh[:k]), list(b[:k])


def kvc_stream_read_add_probe(src, nbytes, item_bytes, adds, dst, sink, workgroups, stream=None):
    _check(lib().kvc_stream_read_add_probe(_ptr(src), int(nbytes), int(item_bytes), int(bool(adds)), _ptr(dst, torch.float32), int(dst.numel()),
                                           _ptr(sink, torch.int32), int(workgroups), _stream(stream)),
           "kvc_stream_read_add_probe")


def kvc_stream_read_probe(src, nbytes, sink, workgroups, stream=None):
    _check(lib().kvc_stream_read_probe(_ptr(src), int(nbytes), _ptr(sink, torch.int32), int(workgroups),
                                       _stream(stream)), "kvc_stream_read_probe")


def kvc_profile_enable(on: bool):
    _check(lib().kvc_profile_enable(int(bool(on))), "kvc_profile_enable")


def kvc_get_decode_chunk(cfg) -> int:
    out = C.c_int(0)
    _check(lib().kvc_get_decode_chunk(C.byref(cfg), C.byref(out)), "kvc_get_decode_chunk")
    return out.value


def kvc_get_decode_short(cfg) -> int:
    out = C.c_int(0)
    _check(lib().kvc_get_decode_short(C.byref(cfg), C.byref(out)), "kvc_get_decode_short")
    return out.value


def kvc_evict_rank_select(cfg, st, seg_offsets, budget, nseg, protect_tail_blocks, evict_rows, selected, ws,
                          stream=None, flags=0):
    _check(lib().kvc_evict_rank_select(C.byref(cfg), C.byref(st),
                                       _ptr(seg_offsets, torch.int32) if seg_offsets is not None else None,
                                       _ptr(budget, torch.int32), nseg, protect_tail_blocks,
                                       _ptr(evict_rows, torch.int32), _ptr(selected, torch.int32), _ptr(ws),
                                       _stream(stream), flags), "kvc_evict_rank_select")


def kvc_compact_rank(cfg, st, evict_rows, blocks_freed, ws, stream=None, flags=0):
    _check(lib().kvc_compact_rank(C.byref(cfg), C.byref(st), _ptr(evict_rows, torch.int32),
                                  _ptr(blocks_freed, torch.int64) if blocks_freed is not None else None,
                                  _ptr(ws), _stream(stream), flags), "kvc_compact_rank")


def kvc_window_metric(cfg, st, q_win, row_lse, w, pool, accumulate, layer_begin, layer_end, ws, stream=None):
    _check(lib().kvc_window_metric(C.byref(cfg), C.byref(st), _ptr(q_win),
                                   _ptr(row_lse, torch.float32) if row_lse is not None else None, int(w), int(pool),
                                   int(accumulate), layer_begin, layer_end, _ptr(ws), _stream(stream)), "kvc_window_metric")


def kvc_query_block_metric(cfg, st, q_blk, row_lse, w, first_pos, exclude, layer_begin, layer_end, ws, stream=None):
    _check(lib().kvc_query_block_metric(C.byref(cfg), C.byref(st), _ptr(q_blk),
                                        _ptr(row_lse, torch.float32) if row_lse is not None else None, int(w),
                                        int(first_pos), int(exclude), layer_begin, layer_end, _ptr(ws), _stream(stream)),
           "kvc_query_block_metric")


def kvc_count_blocks(cfg, st, layer_begin, layer_end, needed, held, ws, stream=None):
    _check(lib().kvc_count_blocks(C.byref(cfg), C.byref(st), layer_begin, layer_end,
                                  _ptr(needed, torch.int32) if needed is not None else None,
                                  _ptr(held, torch.int32) if held is not None else None, _ptr(ws),
                                  _stream(stream)), "kvc_count_blocks")


def kvc_prefill_alloc(cfg, st, seq_tokens, ws, stream=None, flags=0):
    _check(lib().kvc_prefill_alloc(C.byref(cfg), C.byref(st), _ptr(seq_tokens, torch.int32), _ptr(ws),
                                   _stream(stream), flags), "kvc_prefill_alloc")


def kvc_compression_batch(cfg, st, last_compressed, running, kv_limit, in_batch, batch_kvs, ws, stream=None):
    _check(lib().kvc_compression_batch(C.byref(cfg), C.byref(st), _ptr(last_compressed, torch.int64),
                                       _ptr(running, torch.uint8) if running is not None else None,
                                       int(kv_limit), _ptr(in_batch, torch.uint8),
                                       _ptr(batch_kvs, torch.int64) if batch_kvs is not None else None,
                                       _ptr(ws), _stream(stream)), "kvc_compression_batch")


def kvc_preempt(cfg, st, seq_mask, ws, stream=None, flags=0) -> int:
    freed = C.c_int64(0)
    _check(lib().kvc_preempt(C.byref(cfg), C.byref(st), _ptr(seq_mask, torch.uint8), C.byref(freed), _ptr(ws),
                             _stream(stream), flags), "kvc_preempt")
    return freed.value
