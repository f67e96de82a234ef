// On-device block manager: parallel counting and allocation over all
// (sequence, layer, head) instances against a flat length-N free map
// (KV-Compress, Method, "Block Layout and Parallel Allocation"), plus the
// append that stores a new token's key and value.
//
// Order rule (the paper leaves it open): requesters in ascending head-instance
// index; the k-th requested block is the k-th lowest-numbered free block.
// Every launch that writes cache state first reads the workspace status word
// and does nothing when an earlier step of the same call has failed.
#include "kvc_common.h"

namespace kvc {

// blocks held = non-negative prefix of the row; rows are prefix-filled and
// cover at least ceil(ctx_len / b) cells, so the search starts there.
__device__ __forceinline__ int held_blocks(const int32_t* row, int C, int b, int maxb) {
  int u = (C + b - 1) / b;
  while (u < maxb && row[u] >= 0) ++u;
  return u;
}

// mode 0: explicit request counts n[g]; mode 1: append (one block when full and
// the layer is in range); mode 2: drop counts n[g] (must be <= held).
__global__ void __launch_bounds__(256) count_kernel(Dims D, const int32_t* __restrict__ table,
                                                    const int32_t* __restrict__ ctx,
                                                    const int32_t* __restrict__ n, int mode, int l0,
                                                    int l1, int32_t* __restrict__ held,
                                                    int32_t* __restrict__ req,
                                                    int32_t* __restrict__ header) {
  int g = blockIdx.x * 256 + threadIdx.x;
  if (g >= D.G) return;
  const int C = ctx[g];
  const int h = held_blocks(table + (size_t)g * D.maxb, C, D.b, D.maxb);
  held[g] = h;
  int want = 0, bits = 0;
  if (mode == 0) {
    want = n[g];
    if (want < 0) { bits |= EB_ARG; want = 0; }
    else if (h + want > D.maxb) bits |= EB_TABLE;
  } else if (mode == 1) {
    int l = (g / D.Hk) % D.Lyr;
    if (l >= l0 && l < l1 && C == h * D.b) {
      want = 1;
      if (h + 1 > D.maxb) bits |= EB_TABLE;
    }
  } else {
    want = n[g];
    if (want < 0 || want > h) { bits |= EB_ARG; want = 0; }
  }
  req[g] = want;
  if (bits) atomicOr(&header[HW_SCRATCH0], bits);
}

struct ReqFn {
  const int32_t* req;
  __device__ int operator()(int i) const { return req[i]; }
};
struct FreeFn {
  const uint8_t* free_map;
  __device__ int operator()(int i) const { return free_map[i] != 0; }
};

// Third phase of the scan over the free map: rank of every free block; the
// first `total_req` of them are written to picked[] in ascending id.
__global__ void __launch_bounds__(kScanThreads) pick_free_kernel(const uint8_t* __restrict__ free_map,
                                                                 int N,
                                                                 const int32_t* __restrict__ tile_sums,
                                                                 const int32_t* __restrict__ header,
                                                                 int32_t* __restrict__ picked) {
  __shared__ int smem[kScanThreads / 64 + 1];
  const int total_req = header[HW_TOTAL_REQ];
  int base = blockIdx.x * kScanTile + threadIdx.x * kScanItems;
  int v[kScanItems];
  int s = 0;
#pragma unroll
  for (int k = 0; k < kScanItems; ++k) { v[k] = (base + k < N) ? (free_map[base + k] != 0) : 0; s += v[k]; }
  int ex = block_exclusive_scan<kScanThreads>(s, smem, nullptr) + tile_sums[blockIdx.x];
#pragma unroll
  for (int k = 0; k < kScanItems; ++k) {
    if (v[k]) { if (ex < total_req) picked[ex] = base + k; ++ex; }
  }
}

__global__ void __launch_bounds__(256) scatter_alloc_kernel(Dims D, int32_t* __restrict__ table,
                                                            uint8_t* __restrict__ free_map,
                                                            const int32_t* __restrict__ held,
                                                            const int32_t* __restrict__ req,
                                                            const int32_t* __restrict__ off,
                                                            const int32_t* __restrict__ picked,
                                                            const int32_t* __restrict__ header) {
  if (header[HW_STATUS] != KVC_OK) return;
  int g = blockIdx.x * 256 + threadIdx.x;
  if (g >= D.G) return;
  int n = req[g];
  if (n <= 0) return;
  int32_t* row = table + (size_t)g * D.maxb + held[g];
  const int32_t* src = picked + off[g];
  for (int i = 0; i < n; ++i) {
    int id = src[i];
    row[i] = id;
    free_map[id] = 0;
  }
}

__global__ void __launch_bounds__(256) drop_kernel(Dims D, int32_t* __restrict__ table,
                                                   int32_t* __restrict__ ctx,
                                                   uint8_t* __restrict__ free_map,
                                                   const int32_t* __restrict__ held,
                                                   const int32_t* __restrict__ req,
                                                   int32_t* __restrict__ header) {
  if (header[HW_STATUS] != KVC_OK) return;
  int g = blockIdx.x * 256 + threadIdx.x;
  int n = 0;
  if (g < D.G) {
    n = req[g];
    if (n > 0) {
      int h = held[g];
      int32_t* row = table + (size_t)g * D.maxb;
      for (int u = h - n; u < h; ++u) { free_map[row[u]] = 1; row[u] = -1; }
      int cap = (h - n) * D.b;
      if (ctx[g] > cap) ctx[g] = cap;
    }
  }
  int tot = wave_sum_i(n);
  if ((threadIdx.x & 63) == 0 && tot) atomicAdd(&header[HW_FREED], tot);
}

// One workgroup of 64 threads per head instance: copy the new key and value in
// 16-byte pieces, zero the metric, set the logical index, bump the length.
__global__ void __launch_bounds__(64) append_write_kernel(Dims D, int l0, int l1, char* __restrict__ kc,
                                                          char* __restrict__ vc,
                                                          float* __restrict__ metric,
                                                          int32_t* __restrict__ pos,
                                                          const int32_t* __restrict__ table,
                                                          int32_t* __restrict__ ctx,
                                                          const char* __restrict__ k_new,
                                                          const char* __restrict__ v_new,
                                                          const int32_t* __restrict__ new_pos,
                                                          const int32_t* __restrict__ header) {
  if (header[HW_STATUS] != KVC_OK) return;
  const int nl = l1 - l0;
  const int idx = blockIdx.x;                 // over S * nl * Hk
  const int s = idx / (nl * D.Hk);
  const int l = l0 + (idx / D.Hk) % nl;
  const int h = idx % D.Hk;
  const int g = (s * D.Lyr + l) * D.Hk + h;
  const int C = ctx[g];
  const int blk = table[(size_t)g * D.maxb + C / D.b];
  const int o = C % D.b;
  const size_t row_bytes = (size_t)D.d * (D.dtype == KVC_BF16 ? 2 : 4);
  const size_t slot = (size_t)blk * D.b + o;
  const int pieces = (int)(row_bytes / 16);
  for (int c = threadIdx.x; c < 2 * pieces; c += 64) {
    const bool is_v = c >= pieces;
    const int cc = is_v ? c - pieces : c;
    const uint4* src = (const uint4*)((is_v ? v_new : k_new) + (size_t)g * row_bytes) + cc;
    uint4* dst = (uint4*)((is_v ? vc : kc) + slot * row_bytes) + cc;
    *dst = *src;
  }
  __syncthreads();  // every thread has read ctx[g]
  if (threadIdx.x == 0) {
    metric[slot] = 0.0f;
    if (pos) pos[slot] = new_pos ? new_pos[s] : C;
    ctx[g] = C + 1;
  }
}

// Count (mode as in count_kernel), rank the free map, resolve errors, scatter.
static int alloc_common(const Dims& D, const kvc_state* st, const Workspace& W, const int32_t* n,
                        int mode, int l0, int l1, hipStream_t s) {
  const int gb = (D.G + 255) / 256;
  hipLaunchKernelGGL(count_kernel, dim3(gb), dim3(256), 0, s, D, st->block_table, st->ctx_len, n, mode,
                     l0, l1, W.held, W.off_b, W.header);
  KVC_LAUNCH_CHECK();
  int rc = device_exclusive_scan(ReqFn{W.off_b}, D.G, W.tile_sums, W.off_a, W.header + HW_TOTAL_REQ, s);
  if (rc != KVC_OK) return rc;
  // scan of the free map: tile sums, their scan (total -> HW_TOTAL_FREE), then the pick pass
  const int ntiles = (D.N + kScanTile - 1) / kScanTile;
  hipLaunchKernelGGL(scan_tile_reduce<FreeFn>, dim3(ntiles), dim3(kScanThreads), 0, s,
                     FreeFn{st->free_map}, D.N, W.tile_sums);
  KVC_LAUNCH_CHECK();
  hipLaunchKernelGGL(scan_tile_sums, dim3(1), dim3(1024), 0, s, W.tile_sums, ntiles,
                     W.header + HW_TOTAL_FREE);
  KVC_LAUNCH_CHECK();
  hipLaunchKernelGGL(resolve_kernel, dim3(1), dim3(64), 0, s, W.header, 1);
  KVC_LAUNCH_CHECK();
  hipLaunchKernelGGL(pick_free_kernel, dim3(ntiles), dim3(kScanThreads), 0, s, st->free_map, D.N,
                     W.tile_sums, W.header, W.picked);
  KVC_LAUNCH_CHECK();
  hipLaunchKernelGGL(scatter_alloc_kernel, dim3(gb), dim3(256), 0, s, D, st->block_table, st->free_map,
                     W.held, W.off_b, W.off_a, W.picked, W.header);
  KVC_LAUNCH_CHECK();
  return KVC_OK;
}

}  // namespace kvc

using namespace kvc;

extern "C" {

int kvc_block_alloc(const kvc_config* cfg, const kvc_state* st, const int32_t* n_new, void* ws,
                    void* stream, int flags) {
  int rc = validate(cfg, st);
  if (rc != KVC_OK) return rc;
  if (!n_new || !ws || ((uintptr_t)ws & 255)) return KVC_ERR_ARG;
  Dims D = dims_of(cfg);
  Workspace W = carve(D, ws);
  hipStream_t s = (hipStream_t)stream;
  rc = alloc_common(D, st, W, n_new, 0, 0, D.Lyr, s);
  if (rc != KVC_OK) return rc;
  return (flags & KVC_ASYNC) ? KVC_OK : finish_sync(W, s);
}

int kvc_block_free(const kvc_config* cfg, const kvc_state* st, const int32_t* n_drop,
                   int64_t* blocks_freed, void* ws, void* stream, int flags) {
  int rc = validate(cfg, st);
  if (rc != KVC_OK) return rc;
  if (!n_drop || !ws || ((uintptr_t)ws & 255)) return KVC_ERR_ARG;
  Dims D = dims_of(cfg);
  Workspace W = carve(D, ws);
  hipStream_t s = (hipStream_t)stream;
  const int gb = (D.G + 255) / 256;
  hipLaunchKernelGGL(zero_words_kernel, dim3(1), dim3(64), 0, s, W.header + HW_FREED, 1);
  KVC_LAUNCH_CHECK();
  hipLaunchKernelGGL(count_kernel, dim3(gb), dim3(256), 0, s, D, st->block_table, st->ctx_len, n_drop, 2,
                     0, D.Lyr, W.held, W.off_b, W.header);
  KVC_LAUNCH_CHECK();
  hipLaunchKernelGGL(resolve_kernel, dim3(1), dim3(64), 0, s, W.header, 0);
  KVC_LAUNCH_CHECK();
  hipLaunchKernelGGL(drop_kernel, dim3(gb), dim3(256), 0, s, D, st->block_table, st->ctx_len,
                     st->free_map, W.held, W.off_b, W.header);
  KVC_LAUNCH_CHECK();
  if (flags & KVC_ASYNC) return KVC_OK;
  rc = finish_sync(W, s);
  if (rc != KVC_OK) return rc;
  if (blocks_freed) {
    int32_t f = 0;
    rc = read_words(W.header + HW_FREED, &f, 1, s);
    if (rc != KVC_OK) return rc;
    *blocks_freed = f;
  }
  return KVC_OK;
}

int kvc_append(const kvc_config* cfg, const kvc_state* st, const void* k_new, const void* v_new,
               const int32_t* new_pos, int layer_begin, int layer_end, void* ws, void* stream,
               int flags) {
  int rc = validate(cfg, st);
  if (rc != KVC_OK) return rc;
  if (!k_new || !v_new || !ws || ((uintptr_t)ws & 255)) return KVC_ERR_ARG;
  if (((uintptr_t)k_new | (uintptr_t)v_new) & 15) return KVC_ERR_ARG;
  Dims D = dims_of(cfg);
  if (layer_begin < 0 || layer_end > D.Lyr || layer_begin >= layer_end) return KVC_ERR_ARG;
  Workspace W = carve(D, ws);
  hipStream_t s = (hipStream_t)stream;
  rc = alloc_common(D, st, W, nullptr, 1, layer_begin, layer_end, s);
  if (rc != KVC_OK) return rc;
  const int nsel = D.S * (layer_end - layer_begin) * D.Hk;
  hipLaunchKernelGGL(append_write_kernel, dim3(nsel), dim3(64), 0, s, D, layer_begin, layer_end,
                     (char*)st->k_cache, (char*)st->v_cache, st->metric, st->pos, st->block_table,
                     st->ctx_len, (const char*)k_new, (const char*)v_new, new_pos, W.header);
  KVC_LAUNCH_CHECK();
  return (flags & KVC_ASYNC) ? KVC_OK : finish_sync(W, s);
}

}  // extern "C"
