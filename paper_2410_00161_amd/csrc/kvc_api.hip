// Host-side entry points that launch little or nothing: validation, workspace
// sizing, status words.  Also the one kernel the device-wide scan shares.
#include "kvc_common.h"

namespace kvc {

int validate(const kvc_config* c, const kvc_state* st) {
  if (!c) return KVC_ERR_ARG;
  if (c->num_seqs <= 0 || c->num_layers <= 0 || c->num_kv_heads <= 0 || c->group_size <= 0 ||
      c->head_dim <= 0 || c->block_size <= 0 || c->num_blocks <= 0 || c->max_blocks_per_head <= 0)
    return KVC_ERR_ARG;
  if (c->kv_dtype != KVC_F32 && c->kv_dtype != KVC_BF16 && c->kv_dtype != KVC_FP8_E4M3) return KVC_ERR_ARG;
  if (c->metric_mode != KVC_L2 && c->metric_mode != KVC_L1) return KVC_ERR_ARG;
  // index arithmetic is 32-bit for head instances and table cells, 64-bit for slots
  const int64_t G = (int64_t)c->num_seqs * c->num_layers * c->num_kv_heads;
  if (G > (1ll << 28)) return KVC_ERR_UNSUPPORTED;
  if (G * c->max_blocks_per_head > (1ll << 40)) return KVC_ERR_UNSUPPORTED;
  if ((int64_t)c->num_blocks * c->block_size > (1ll << 40)) return KVC_ERR_UNSUPPORTED;
  if (c->group_size > 16 || c->head_dim > 512) return KVC_ERR_UNSUPPORTED;
  // slots are indexed as (block id << log2 b) + (j & (b - 1)) by the compaction, rank-schedule and
  // window kernels: a block size that is not a power of two would send rows to wrong slots
  if ((c->block_size & (c->block_size - 1)) != 0 || c->block_size > 1024) return KVC_ERR_UNSUPPORTED;
  const int esz = kv_esz(c->kv_dtype);
  if ((c->head_dim * esz) % 16 != 0) return KVC_ERR_UNSUPPORTED;  // rows are read 16 bytes at a time
  if (st) {
    if (!st->k_cache || !st->v_cache || !st->metric || !st->block_table || !st->ctx_len ||
        !st->free_map)
      return KVC_ERR_ARG;
    if (((uintptr_t)st->k_cache | (uintptr_t)st->v_cache) & 15) return KVC_ERR_ARG;
    if (((uintptr_t)st->metric | (uintptr_t)st->block_table | (uintptr_t)st->ctx_len) & 3)
      return KVC_ERR_ARG;
    if (st->pos && ((uintptr_t)st->pos & 3)) return KVC_ERR_ARG;
  }
  return KVC_OK;
}

__global__ void __launch_bounds__(256) stream_read_kernel(const uint4* __restrict__ src, size_t n16,
                                                          uint32_t* __restrict__ sink) {
  uint32_t acc = 0;
  const size_t stride = (size_t)gridDim.x * 256;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {  // four independent loads in flight per lane
    const uint4 a = load_stream16(src + i), b = load_stream16(src + i + stride);
    const uint4 c = load_stream16(src + i + 2 * stride), d = load_stream16(src + i + 3 * stride);
    acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
  }
  for (; i < n16; i += stride) { const uint4 a = load_stream16(src + i); acc ^= a.x ^ a.y ^ a.z ^ a.w; }
  for (int m = 32; m >= 1; m >>= 1) acc ^= __shfl_xor(acc, m);
  if ((threadIdx.x & 63) == 0) atomicXor(&sink[blockIdx.x], acc);
}

// A read stream shaped like the decode's, with the decode's share of writes if asked for: a
// workgroup reads items of `item16` 16-byte pieces at a stretch (what a chunk's workgroup does with
// a chunk's K and V rows) and after each item adds one float per 512 bytes read to `dst`, with the
// hardware add the decode uses for the metric (`adds`; 512 bytes are the K and V rows of one KV of
// 16-bit elements, d = 128).
__global__ void __launch_bounds__(256) stream_read_add_kernel(const uint4* __restrict__ src, size_t item16, int n_items,
                                                              int adds, float* __restrict__ dst,
                                                              uint32_t* __restrict__ sink) {
  uint32_t acc = 0;
  const int per_item = (int)(item16 / 32);   // floats added per item
  for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
    const uint4* p = src + (size_t)item * item16;
    size_t i = threadIdx.x;
    for (; i + 3 * 256 < item16; i += 4 * 256) {
      const uint4 a = load_stream16(p + i), b = load_stream16(p + i + 256);
      const uint4 c = load_stream16(p + i + 512), d = load_stream16(p + i + 768);
      acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
    }
    for (; i < item16; i += 256) { const uint4 a = load_stream16(p + i); acc ^= a.x ^ a.y ^ a.z ^ a.w; }
    if (adds) {
      float* m = dst + (size_t)item * per_item;
      for (int k = threadIdx.x; k < per_item; k += 256) unsafeAtomicAdd(&m[k], 1.0f);
    }
  }
  for (int m = 32; m >= 1; m >>= 1) acc ^= __shfl_xor(acc, m);
  if ((threadIdx.x & 63) == 0) atomicXor(&sink[blockIdx.x], acc);
}

}  // namespace kvc

using namespace kvc;

extern "C" {

size_t kvc_workspace_bytes(const kvc_config* cfg) {
  if (validate(cfg, nullptr) != KVC_OK) return 0;
  Dims D = dims_of(cfg);
  return carve(D, nullptr).bytes;
}

int kvc_validate(const kvc_config* cfg, const kvc_state* st) { return validate(cfg, st); }

const char* kvc_status_string(int status) {
  switch (status) {
    case KVC_OK: return "ok";
    case KVC_ERR_ARG: return "invalid argument";
    case KVC_ERR_OOM: return "not enough free blocks";
    case KVC_ERR_TABLE_FULL: return "block table row full";
    case KVC_ERR_NUMERIC: return "NaN, infinite or negative block key";
    case KVC_ERR_HIP: return "HIP runtime error";
    case KVC_ERR_UNSUPPORTED: return "shape not supported";
    default: return "unknown status";
  }
}

int kvc_workspace_reset(const kvc_config* cfg, void* ws, void* stream) {
  int rc = validate(cfg, nullptr);
  if (rc != KVC_OK) return rc;
  if (!ws || ((uintptr_t)ws & 255)) return KVC_ERR_ARG;
  Workspace W = carve(dims_of(cfg), ws);
  // a fill kernel rather than a memset node: safe to record into a HIP graph
  const int words = HW_WORDS * (1 + dims_of(cfg).Lyr);   // the header, then the layers' plan headers, back to back
  hipLaunchKernelGGL(zero_words_kernel, dim3((words + 255) / 256), dim3(256), 0, (hipStream_t)stream, W.header, words);
  KVC_LAUNCH_CHECK();
  return KVC_OK;
}

int kvc_stream_read_probe(const void* src, size_t bytes, uint32_t* sink, int workgroups, void* stream) {
  if (!src || !sink || workgroups <= 0 || (bytes & 15) || ((uintptr_t)src & 15)) return KVC_ERR_ARG;
  hipLaunchKernelGGL(stream_read_kernel, dim3(workgroups), dim3(256), 0, (hipStream_t)stream,
                     (const uint4*)src, bytes / 16, sink);
  KVC_LAUNCH_CHECK();
  return KVC_OK;
}

int kvc_stream_read_add_probe(const void* src, size_t bytes, size_t item_bytes, int adds, float* dst,
                              size_t dst_floats, uint32_t* sink, int workgroups, void* stream) {
  if (!src || !dst || !sink || workgroups <= 0 || ((uintptr_t)src & 15) || ((uintptr_t)dst & 3)) return KVC_ERR_ARG;
  if (item_bytes < 4096 || (item_bytes & 511)) return KVC_ERR_ARG;
  const size_t n_items = bytes / item_bytes;
  if (n_items == 0 || n_items > 0x7fffffffull || dst_floats < n_items * (item_bytes / 512)) return KVC_ERR_ARG;
  hipLaunchKernelGGL(stream_read_add_kernel, dim3(workgroups), dim3(256), 0, (hipStream_t)stream,
                     (const uint4*)src, item_bytes / 16, (int)n_items, adds ? 1 : 0, dst, sink);
  KVC_LAUNCH_CHECK();
  return KVC_OK;
}

int kvc_poll_status(const kvc_config* cfg, void* ws, void* stream, int* status) {
  int rc = validate(cfg, nullptr);
  if (rc != KVC_OK) return rc;
  if (!ws || !status || ((uintptr_t)ws & 255)) return KVC_ERR_ARG;
  Workspace W = carve(dims_of(cfg), ws);
  int32_t w = 0;
  rc = read_words(W.header + HW_STATUS, &w, 1, (hipStream_t)stream);
  if (rc != KVC_OK) return rc;
  *status = w;
  return KVC_OK;
}

}  // extern "C"
