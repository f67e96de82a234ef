// Shared host/device plumbing of libkvc: workspace layout, launch checks, a
// device-wide exclusive scan, and small wavefront helpers.  gfx950 only.
#pragma once

#include <hip/hip_runtime.h>
#include <atomic>
#include <stdint.h>
#include <stddef.h>

#include "kvc.h"

namespace kvc {

constexpr int kWave = 64;
constexpr int kScanThreads = 256;
constexpr int kScanItems = 8;                       // per thread
constexpr int kScanTile = kScanThreads * kScanItems; // 2048 elements per workgroup

// ---- workspace header: one int32 per field, zeroed by kvc_workspace_reset ----
enum HeaderWord {
  HW_STATUS = 0,      // sticky error word written by device-side guards
  HW_TOTAL_REQ = 1,   // blocks requested by the call in flight
  HW_TOTAL_FREE = 2,  // free blocks counted by the call in flight
  HW_TOTAL_ITEMS = 3, // decode work items
  HW_FREED = 4,       // blocks freed by the call in flight
  HW_SCRATCH0 = 5,
  HW_SCRATCH1 = 6,
  HW_SHORT_ITEMS = 8,  // decode work items short enough for the one-wavefront launch
  HW_TOTAL_PARTIALS = 9,  // per-chunk partial-result slots in use = chunks of heads of more than one chunk
  HW_CHUNK_T = 10,     // chunk length the work list in place was cut with (tokens)
  // decode work-list block: item counts per size class, per-class cursors, cursor of the
  // per-chunk partial results.  All zero between calls (the chunk kernel clears it).
  HW_DEC_BINS = 32,    // [16]
  HW_DEC_CUR = 48,     // [16]
  HW_DEC_PCUR = 64,    // [1]
  HW_DEC_PTOT = 65,    // [1] partial-result slots wanted, counted in pass 1
  HW_DEC_END = 66,
  HW_WORDS = 128
};

struct Dims {
  int S, Lyr, Hk, r, d, b, N, maxb, G;
  int dtype, mode;
};

inline Dims dims_of(const kvc_config* c) {
  Dims D;
  D.S = c->num_seqs; D.Lyr = c->num_layers; D.Hk = c->num_kv_heads; D.r = c->group_size;
  D.d = c->head_dim; D.b = c->block_size; D.N = c->num_blocks; D.maxb = c->max_blocks_per_head;
  D.G = D.S * D.Lyr * D.Hk; D.dtype = c->kv_dtype; D.mode = c->metric_mode;
  return D;
}

constexpr int kMinChunk = 64;      // smallest decode chunk (tokens per workgroup)
constexpr int kMaxChunk = 8192;

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Carves the caller's workspace.  All offsets are multiples of 256 bytes.
struct Workspace {
  int32_t* header;     // [HW_WORDS]
  int32_t* plan_hdr;   // [Lyr][HW_WORDS]     header block of every layer's kept work list (kvc_decode_plan)
  int32_t* tile_sums;  // [ntile_max + 1]
  int32_t* off_a;      // [G + 1]  scan over head instances (requests / chunks / ties)
  int32_t* off_b;      // [G + 1]
  int32_t* held;       // [G]      blocks held per head instance
  int32_t* picked;     // [N]      k-th lowest free block id
  int32_t* items;      // [max_items][8]      decode work items (see DecodeItem)
  int32_t* slot_item;  // [max_items]         work item of every partial-result slot in use
  float*   part_ml;    // [max_items][r][2]   chunk max and sum per query head
  float*   part_acc;   // [max_items][r][d]   chunk un-normalised output
  float*   stash;      // [N*b][r]            chunk-relative exp of every logit
  int32_t* seg_hist;   // [S][256]            radix histograms per segment
  int32_t* seg_state;  // [S][8]              prefix, remaining, ties wanted, ...
  int32_t* flag_scan;  // [G][maxb]           per-head prefix count of flagged blocks
  size_t bytes;
};

inline size_t max_items_of(const Dims& D) {
  // every chunk but a head's last is full, so items <= slots / min_chunk + G
  return (size_t)D.N * (size_t)D.b / kMinChunk + (size_t)D.G + 1;
}

inline Workspace carve(const Dims& D, void* base) {
  Workspace w;
  char* p = (char*)base;
  size_t o = 0;
  // (sized with a null base by kvc_workspace_bytes: then only the offsets are formed)
  auto take = [&](size_t bytes) { char* q = p ? p + o : nullptr; o += align_up(bytes, 256); return q; };
  size_t nmax = (size_t)(D.N > D.G ? D.N : D.G) + 1;
  size_t ntile = nmax / kScanTile + 2;
  w.header = (int32_t*)take(HW_WORDS * 4);
  w.plan_hdr = (int32_t*)take((size_t)D.Lyr * HW_WORDS * 4);
  w.tile_sums = (int32_t*)take(ntile * 4);
  w.off_a = (int32_t*)take(((size_t)D.G + 1) * 4);
  w.off_b = (int32_t*)take(((size_t)D.G + 1) * 4);
  w.held = (int32_t*)take((size_t)D.G * 4);
  w.picked = (int32_t*)take((size_t)D.N * 4);
  size_t items = max_items_of(D);
  w.items = (int32_t*)take(items * 32);
  w.slot_item = (int32_t*)take(items * 4);
  w.part_ml = (float*)take(items * D.r * 2 * 4);
  w.part_acc = (float*)take(items * D.r * D.d * 4);
  w.stash = (float*)take((size_t)D.N * D.b * D.r * 4);
  w.seg_hist = (int32_t*)take((size_t)D.S * 256 * 4);
  w.seg_state = (int32_t*)take((size_t)D.S * 8 * 4);
  w.flag_scan = (int32_t*)take((size_t)D.G * D.maxb * 4);
  w.bytes = o;
  return w;
}

int validate(const kvc_config* cfg, const kvc_state* st);  // kvc_api.hip

#define KVC_HIP(expr)                                   \
  do {                                                  \
    hipError_t e__ = (expr);                            \
    if (e__ != hipSuccess) return KVC_ERR_HIP;          \
  } while (0)

#define KVC_LAUNCH_CHECK() KVC_HIP(hipGetLastError())

inline int read_words(const int32_t* dev, int32_t* host, int n, hipStream_t s) {
  KVC_HIP(hipMemcpyAsync(host, dev, (size_t)n * 4, hipMemcpyDeviceToHost, s));
  KVC_HIP(hipStreamSynchronize(s));
  return KVC_OK;
}

// ---------------------------------------------------------------------------
// device helpers
// ---------------------------------------------------------------------------

// 16-byte load of data that is read once per launch (K and V rows): marked non-temporal so that
// it does not displace what the caches should keep; a plain read stream measures 6.0-6.3 TB/s on
// this chip, the same stream with this hint 6.4-7.1 TB/s.
__device__ __forceinline__ uint4 load_stream16(const void* p) {
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 t = __builtin_nontemporal_load((const u32x4*)p);
  return make_uint4(t.x, t.y, t.z, t.w);
}
__device__ __forceinline__ uint2 load_stream8(const void* p) {
  typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
  const u32x2 t = __builtin_nontemporal_load((const u32x2*)p);
  return make_uint2(t.x, t.y);
}

// bytes of one K/V element, and of one query element (queries of an 8-bit cache are bf16)
__host__ __device__ inline int kv_esz(int dtype) { return dtype == KVC_F32 ? 4 : dtype == KVC_BF16 ? 2 : 1; }
__host__ __device__ inline int q_esz(int dtype) { return dtype == KVC_F32 ? 4 : 2; }

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

__device__ __forceinline__ int wave_sum_i(int v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m);
  return v;
}
__device__ __forceinline__ float wave_sum_f(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m);
  return v;
}
__device__ __forceinline__ float wave_max_f(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m));
  return v;
}

// Exclusive scan of one int per thread over a workgroup of NT threads.
// `total` (if non-null) receives the workgroup sum.  smem: NT/64 + 1 ints.
template <int NT>
__device__ __forceinline__ int block_exclusive_scan(int v, int* smem, int* total) {
  const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
  int inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    int t = __shfl_up(inc, o);
    if (lane >= o) inc += t;
  }
  if (lane == 63) smem[wid] = inc;
  __syncthreads();
  if (threadIdx.x == 0) {
    int run = 0;
    for (int w = 0; w < NT / 64; ++w) { int t = smem[w]; smem[w] = run; run += t; }
    smem[NT / 64] = run;
  }
  __syncthreads();
  int base = smem[wid];
  if (total) *total = smem[NT / 64];
  __syncthreads();
  return base + inc - v;
}

// Error bits a kernel leaves in the header's scratch word for the launch that settles the status.
enum ErrBit { EB_ARG = 1, EB_TABLE = 2, EB_NUMERIC = 4 };

// Blocks a compaction freed = the sum of the per-head counts it was given (each head gives back
// exactly the blocks it loses), or 0 when the call failed.  One workgroup adds the counts up:
// a counter bumped by every head would see thousands of adds to one word, which the chip runs
// one after the other (that counter alone took 0.13 ms per round at 16 384 heads).
// With `resolve` set the launch also does what resolve_kernel(header, 0) does, first: a compaction
// that reports its count settles its status and publishes in one launch, ahead of the moves.
static __global__ void __launch_bounds__(1024) publish_freed_kernel(int32_t* __restrict__ header,
                                                                    const int32_t* __restrict__ counts, int G,
                                                                    int64_t* __restrict__ out, int resolve) {
  __shared__ long long part[1024 / 64];
  __shared__ int status_s;
  if (threadIdx.x == 0) {
    if (resolve) {
      const int bits = header[HW_SCRATCH0];
      int st = KVC_OK;
      if (bits & EB_ARG) st = KVC_ERR_ARG;
      else if (bits & EB_TABLE) st = KVC_ERR_TABLE_FULL;
      else if (bits & EB_NUMERIC) st = KVC_ERR_NUMERIC;
      if (st != KVC_OK && header[HW_STATUS] == KVC_OK) header[HW_STATUS] = st;
      header[HW_SCRATCH0] = 0;
    }
    status_s = header[HW_STATUS];
  }
  long long s = 0;
  // One workgroup reads all the counts: 32 of them per thread asked for at a time (eight 16-byte
  // loads) when the array is 16-byte aligned, else eight.
  if (((uintptr_t)counts & 15) == 0) {
    const int4* c4 = (const int4*)counts;
    const int n4 = G >> 2;
    for (int i0 = threadIdx.x; i0 < n4; i0 += 8 * 1024) {
      int4 v[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) v[k] = i0 + k * 1024 < n4 ? c4[i0 + k * 1024] : make_int4(0, 0, 0, 0);
#pragma unroll
      for (int k = 0; k < 8; ++k) s += (long long)max(v[k].x, 0) + max(v[k].y, 0) + max(v[k].z, 0) + max(v[k].w, 0);
    }
    for (int g = (n4 << 2) + threadIdx.x; g < G; g += 1024) s += max(counts[g], 0);
  } else {
    for (int g0 = threadIdx.x; g0 < G; g0 += 8 * 1024) {
      int v[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) v[k] = g0 + k * 1024 < G ? counts[g0 + k * 1024] : 0;
#pragma unroll
      for (int k = 0; k < 8; ++k) s += max(v[k], 0);
    }
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) s += __shfl_xor(s, o);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    long long t = 0;
    for (int w = 0; w < 1024 / 64; ++w) t += part[w];
    out[0] = status_s == KVC_OK ? t : 0;
  }
}

// ---- device-wide exclusive scan in three launches -------------------------
// F: __device__ int operator()(int i) giving element i.  Results go to
// out[0..n) and out[n] = total; `total_word` (may be null) also receives it.
template <class F>
__global__ void __launch_bounds__(kScanThreads) scan_tile_reduce(F f, int n, int32_t* tile_sums) {
  __shared__ int red[kScanThreads / 64];
  int base = blockIdx.x * kScanTile + threadIdx.x * kScanItems;
  int s = 0;
#pragma unroll
  for (int k = 0; k < kScanItems; ++k) if (base + k < n) s += f(base + k);
  s = wave_sum_i(s);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    int t = 0;
    for (int w = 0; w < kScanThreads / 64; ++w) t += red[w];
    tile_sums[blockIdx.x] = t;
  }
}

static __global__ void __launch_bounds__(1024) scan_tile_sums(int32_t* tile_sums, int ntiles,
                                                              int32_t* total_word) {
  __shared__ int smem[1024 / 64 + 1];
  __shared__ int carry_s;
  if (threadIdx.x == 0) carry_s = 0;
  __syncthreads();
  for (int base = 0; base < ntiles; base += 1024) {
    int i = base + threadIdx.x;
    int v = (i < ntiles) ? tile_sums[i] : 0;
    int tot;
    int ex = block_exclusive_scan<1024>(v, smem, &tot);
    int carry = carry_s;
    if (i < ntiles) tile_sums[i] = ex + carry;
    __syncthreads();
    if (threadIdx.x == 0) carry_s = carry + tot;
    __syncthreads();
  }
  if (threadIdx.x == 0 && total_word) *total_word = carry_s;
}

template <class F>
__global__ void __launch_bounds__(kScanThreads) scan_tile_apply(F f, int n, const int32_t* tile_sums,
                                                                int32_t* out) {
  __shared__ int smem[kScanThreads / 64 + 1];
  int base = blockIdx.x * kScanTile + threadIdx.x * kScanItems;
  int v[kScanItems];
  int s = 0;
#pragma unroll
  for (int k = 0; k < kScanItems; ++k) { v[k] = (base + k < n) ? f(base + k) : 0; s += v[k]; }
  int ex = block_exclusive_scan<kScanThreads>(s, smem, nullptr) + tile_sums[blockIdx.x];
#pragma unroll
  for (int k = 0; k < kScanItems; ++k) {
    if (base + k < n) out[base + k] = ex;
    ex += v[k];
  }
  if (blockIdx.x == gridDim.x - 1 && threadIdx.x == kScanThreads - 1) out[n] = ex;
}

template <class F>
inline int device_exclusive_scan(F f, int n, int32_t* tile_sums, int32_t* out, int32_t* total_word,
                                 hipStream_t s) {
  int ntiles = (n + kScanTile - 1) / kScanTile;
  if (ntiles < 1) ntiles = 1;
  hipLaunchKernelGGL(scan_tile_reduce<F>, dim3(ntiles), dim3(kScanThreads), 0, s, f, n, tile_sums);
  KVC_LAUNCH_CHECK();
  hipLaunchKernelGGL(scan_tile_sums, dim3(1), dim3(1024), 0, s, tile_sums, ntiles, total_word);
  KVC_LAUNCH_CHECK();
  hipLaunchKernelGGL(scan_tile_apply<F>, dim3(ntiles), dim3(kScanThreads), 0, s, f, n, tile_sums, out);
  KVC_LAUNCH_CHECK();
  return KVC_OK;
}

// ---- status word plumbing shared by the entry points ------------------------

static __global__ void zero_words_kernel(int32_t* p, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

// Turns the error bits and the two totals into the status word, in a fixed
// priority: argument, table full, numeric, out of blocks (check_oom == 1 only).
static __global__ void resolve_kernel(int32_t* header, int check_oom) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  int bits = header[HW_SCRATCH0];
  int st = KVC_OK;
  if (bits & EB_ARG) st = KVC_ERR_ARG;
  else if (bits & EB_TABLE) st = KVC_ERR_TABLE_FULL;
  else if (bits & EB_NUMERIC) st = KVC_ERR_NUMERIC;
  else if (check_oom == 1 && header[HW_TOTAL_REQ] > header[HW_TOTAL_FREE]) st = KVC_ERR_OOM;
  if (st != KVC_OK && header[HW_STATUS] == KVC_OK) header[HW_STATUS] = st;
  header[HW_SCRATCH0] = 0;
}

// Per-segment state of a selection (block mode and rank-block mode share it): eight words.
enum SegWord { SEG_PREFIX = 0, SEG_REMAIN = 1, SEG_CAND = 2, SEG_TAKE = 3, SEG_FIRSTG = 4, SEG_ALLTIES = 5 };

// First launch of either selection: the segment of every sequence (segments are runs of
// consecutive sequences; seg_offsets NULL = one per sequence), cleared histograms and segment
// state with the segment's first head instance, cleared per-head counts and per-segment results,
// and the check of the offsets (first 0, last S, non-decreasing).
static __global__ void __launch_bounds__(256) segments_init_kernel(Dims D, const int32_t* __restrict__ seg_offsets,
                                                                   int nseg, int32_t* __restrict__ seq_seg,
                                                                   int32_t* __restrict__ seg_hist,
                                                                   int32_t* __restrict__ seg_state,
                                                                   int32_t* __restrict__ per_head,
                                                                   int32_t* __restrict__ selected,
                                                                   int32_t* __restrict__ header) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < D.S) {
    int sg = i;
    if (seg_offsets) {  // last segment whose first sequence is <= i
      int lo = 0, hi = nseg;
      while (hi - lo > 1) { const int mid = (lo + hi) >> 1; if (seg_offsets[mid] <= i) lo = mid; else hi = mid; }
      sg = lo;
    }
    seq_seg[i] = sg;
  }
  if (i < nseg * 256) seg_hist[i] = 0;
  if (i < nseg) {
    selected[i] = 0;
    for (int k = 0; k < 8; ++k) seg_state[i * 8 + k] = 0;
    const int first_seq = seg_offsets ? seg_offsets[i] : i;
    seg_state[i * 8 + SEG_FIRSTG] = first_seq * D.Lyr * D.Hk;
    if (seg_offsets) {
      const int a = seg_offsets[i], b2 = seg_offsets[i + 1];
      if (a > b2 || (i == 0 && a != 0) || (i == nseg - 1 && b2 != D.S)) atomicOr(&header[HW_SCRATCH0], EB_ARG);
    }
  }
  if (i < D.G) per_head[i] = 0;
}

// How much dynamic LDS a kernel may take above the default 64 KB is an attribute of the kernel on
// a device: remembered per device (the first 64 of a process), raised when a call needs more.
// Host threads may race here; telling the runtime twice is harmless.
struct LdsLimit {
  std::atomic<size_t> allowed[64] = {};
  template <class... Kernels>
  int need(size_t bytes, Kernels... kernels) {
    if (bytes <= 64 * 1024) return KVC_OK;
    int dev = -1;
    KVC_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) return KVC_ERR_UNSUPPORTED;
    if (bytes <= allowed[dev].load(std::memory_order_acquire)) return KVC_OK;
    const void* ks[] = {(const void*)kernels...};
    for (const void* k : ks) KVC_HIP(hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
    size_t seen = allowed[dev].load(std::memory_order_relaxed);
    while (seen < bytes && !allowed[dev].compare_exchange_weak(seen, bytes, std::memory_order_release)) {}
    return KVC_OK;
  }
};

// Reads the status word; a non-zero word is cleared so that the next call starts clean.
inline int finish_sync(const Workspace& W, hipStream_t s) {
  int32_t w = 0;
  int rc = read_words(W.header + HW_STATUS, &w, 1, s);
  if (rc != KVC_OK) return rc;
  if (w != KVC_OK) {
    hipLaunchKernelGGL(zero_words_kernel, dim3(1), dim3(64), 0, s, W.header + HW_STATUS, 1);
    KVC_LAUNCH_CHECK();
    KVC_HIP(hipStreamSynchronize(s));
  }
  return w;
}

}  // namespace kvc
