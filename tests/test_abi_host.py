"""CPU-side checks of the C ABI: the library loads without a GPU, exports every
symbol include/kvc.h declares, and rejects bad arguments on the host before any
HIP call."""
import ctypes as C
import os
import re

import pytest
import torch

from paper_2410_00161_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    src = "".join(open(os.path.join(ROOT, "include", h)).read() for h in sorted(os.listdir(os.path.join(ROOT, "include"))))
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(kvc_[a-z_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    L = B.lib()
    names = declared_functions()
    assert len(names) >= 12
    for n in names:
        assert hasattr(L, n), f"{n} declared in kvc.h but not exported"
    assert sorted(B.EXPORTS) == names


def good_cfg(**kw):
    base = dict(num_seqs=2, num_layers=2, num_kv_heads=2, group_size=4, head_dim=128, block_size=16,
                num_blocks=64, max_blocks_per_head=8, kv_dtype="bf16")
    base.update(kw)
    return B.make_config(**base)


def test_validate_and_workspace_size():
    cfg = good_cfg()
    assert B.kvc_validate(cfg) == B.KVC_OK
    n = B.kvc_workspace_bytes(cfg)
    assert n > 0 and n % 256 == 0
    assert B.kvc_workspace_bytes(good_cfg(num_blocks=128)) > n
    for bad in (dict(num_seqs=0), dict(head_dim=-1), dict(kv_dtype=7), dict(block_size=0),
                dict(metric_mode=3)):
        c = good_cfg(**bad)
        assert B.kvc_validate(c) == B.KVC_ERR_ARG
        assert B.kvc_workspace_bytes(c) == 0
    assert B.kvc_validate(good_cfg(group_size=32)) == B.KVC_ERR_UNSUPPORTED
    assert B.kvc_validate(good_cfg(head_dim=100, kv_dtype="bf16")) == B.KVC_ERR_UNSUPPORTED
    # block sizes are powers of two: the compaction, rank-schedule and window kernels index a slot
    # as (block id << log2 b) + (j & (b - 1)), so anything else is refused at the boundary
    for b in (3, 24, 48, 2048):
        c = good_cfg(block_size=b)
        assert B.kvc_validate(c) == B.KVC_ERR_UNSUPPORTED, b
        assert B.kvc_workspace_bytes(c) == 0
    for b in (1, 2, 4, 8, 16, 32, 64, 128):
        assert B.kvc_validate(good_cfg(block_size=b)) == B.KVC_OK, b


def test_status_strings_and_chunk_knob():
    seen = {B.status_string(c) for c in (0, 1, 2, 3, 5, 6, 7)}
    assert len(seen) == 7 and "ok" in seen and "unknown status" not in seen
    assert B.status_string(4) == "unknown status"   # no such code
    assert B.status_string(99) == "unknown status"
    L = B.lib()
    assert L.kvc_set_decode_chunk(100) == B.KVC_ERR_ARG
    assert L.kvc_set_decode_chunk(16384) == B.KVC_ERR_ARG
    assert L.kvc_set_decode_chunk(512) == B.KVC_OK
    assert L.kvc_set_decode_chunk(0) == B.KVC_OK


def test_chunk_length_is_whole_strips_for_every_shape():
    """The chunk length the library picks (shortened for calls over few head instances, capped by
    the LDS) is a whole number of 64-token strips, so that a chunk starts on a block boundary."""
    for r in (1, 2, 4, 8):
        for d in (64, 128):
            for dt in ("bf16", "f32", "fp8"):
                for b in (4, 16, 64):
                    for seqs, layers, maxb in ((1, 1, 8), (2, 2, 400), (3, 1, 2000), (64, 32, 512), (16, 80, 8192 // b * 16)):
                        cfg = B.make_config(seqs, layers, 2, r, d, b, 64, maxb, dt)
                        if B.kvc_validate(cfg) != B.KVC_OK:
                            continue
                        t = B.kvc_get_decode_chunk(cfg)
                        s_ = B.kvc_get_decode_short(cfg)
                        assert t % 64 == 0 and t >= 0, (r, d, dt, b, seqs, layers, maxb, t)
                        if t:
                            assert 0 < s_ <= min(t, 512)


def test_entry_points_reject_bad_arguments_on_the_host():
    """Null state pointers, a misaligned workspace and a bad layer range are
    refused before anything is launched (so this runs without a GPU)."""
    L = B.lib()
    cfg = good_cfg()
    st = B.kvc_state()  # all NULL
    one = C.c_void_p(4096)
    assert L.kvc_block_alloc(C.byref(cfg), C.byref(st), one, one, None, 0) == B.KVC_ERR_ARG
    assert L.kvc_paged_decode(C.byref(cfg), C.byref(st), one, one, 0, 1, 1, one, None) == B.KVC_ERR_ARG
    assert L.kvc_compact(C.byref(cfg), C.byref(st), one, one, None, one, None, 0) == B.KVC_ERR_ARG
    # a plausible state (never dereferenced: the calls fail on later checks)
    st = B.kvc_state(4096, 8192, 4096, None, 4096, 4096, 4096)
    assert B.kvc_validate(cfg, st) == B.KVC_OK
    assert L.kvc_paged_decode(C.byref(cfg), C.byref(st), one, one, 0, 3, 1, one, None) == B.KVC_ERR_ARG  # layers
    assert L.kvc_paged_decode(C.byref(cfg), C.byref(st), one, one, 1, 1, 1, one, None) == B.KVC_ERR_ARG
    assert L.kvc_paged_decode(C.byref(cfg), C.byref(st), None, one, 0, 1, 1, one, None) == B.KVC_ERR_ARG
    assert L.kvc_paged_decode(C.byref(cfg), C.byref(st), one, one, 0, 1, 1, C.c_void_p(4100), None) == B.KVC_ERR_ARG
    assert L.kvc_append(C.byref(cfg), C.byref(st), one, C.c_void_p(4104), None, 0, 1, one, None, 0) == B.KVC_ERR_ARG
    assert L.kvc_evict_select(C.byref(cfg), C.byref(st), one, None, one, 1, 1, one, one, one, one, None, 0) == B.KVC_ERR_ARG  # nseg != S
    assert L.kvc_evict_select(C.byref(cfg), C.byref(st), one, one, one, 3, 1, one, one, one, one, None, 0) == B.KVC_ERR_ARG  # nseg > S
    assert L.kvc_metric_reduce(C.byref(cfg), C.byref(st), None, B.KVC_KEY_SUM, one, None) == B.KVC_ERR_ARG
    assert L.kvc_metric_reduce(C.byref(cfg), C.byref(st), one, 7, one, None) == B.KVC_ERR_ARG
    st_bad = B.kvc_state(4097, 8192, 4096, None, 4096, 4096, 4096)
    assert B.kvc_validate(cfg, st_bad) == B.KVC_ERR_ARG
    # the measurement hooks check their arguments the same way
    mib = 1 << 20
    probe = L.kvc_stream_read_add_probe
    assert probe(None, 64 * mib, mib, 1, one, 1 << 20, one, 512, None) == B.KVC_ERR_ARG            # no source
    assert probe(C.c_void_p(4104), 64 * mib, mib, 1, one, 1 << 20, one, 512, None) == B.KVC_ERR_ARG  # source not 16-byte aligned
    assert probe(one, 64 * mib, 1000, 1, one, 1 << 20, one, 512, None) == B.KVC_ERR_ARG            # item not a multiple of 512
    assert probe(one, 64 * mib, mib, 1, one, 64 * 2048 - 1, one, 512, None) == B.KVC_ERR_ARG       # too few floats to add to
    assert probe(one, mib // 2, mib, 1, one, 1 << 20, one, 512, None) == B.KVC_ERR_ARG             # not one whole item
    assert probe(one, 64 * mib, mib, 1, one, 1 << 20, one, 0, None) == B.KVC_ERR_ARG               # no workgroups
    assert L.kvc_stream_read_probe(one, 100, one, 512, None) == B.KVC_ERR_ARG                      # bytes not a multiple of 16


def test_binding_refuses_wrong_dtypes_and_strides():
    t = torch.zeros(4, 4)
    with pytest.raises(TypeError):
        B._ptr(t, torch.int32)
    with pytest.raises(ValueError):
        B._ptr(t.t())
