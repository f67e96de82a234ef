// Prefill-end eviction metric from an observation window (KV-Compress:
// Preliminaries "KV Cache Compression" - sum of attention over the last w
// prompt queries, max-pooling over the sequence; Method "Query Group
// Compression" - also over the query heads of the KV head's group; "Metric
// Calculation", KVC-w - squared before summation).
//
// Unlike the decode this is a dense contraction: w * r query rows (32 .. 256)
// against every key of the head, so it runs on the matrix cores.  Per
// 16-token block: S^T[16 tokens x 16 query rows] += K[16 x 32] * Q^T[32 x 16]
// with v_mfma_f32_16x16x32_bf16, four k-slices for d = 128.  A lane holds 64
// contiguous bytes of one token (its four 16-byte loads are the four k-slices),
// and Q is staged in LDS in exactly the register order of the B operand, so no
// transposes and no bank conflicts.  The contraction over d does not care in
// which order dimensions are assigned to k-slices as long as K and Q agree.
//
// Two passes over K: (1) per query row, max and sum of exp over its visible
// keys (online, then merged over lanes, wavefronts and chunks); (2) normalised
// probabilities, squared, summed over the query rows per key.  V is never
// read.  A last light pass max-pools over the logical sequence.
#include <type_traits>

#include "kvc_common.h"
#include "kvc_worklist.h"

namespace kvc {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int kWinChunk = 1024;   // tokens per workgroup
constexpr int kWinThreads = 256;
constexpr int kWinWaves = 4;

struct WindowArgs {
  DecodeArgs A;        // cache, tables, work list (A.T = kWinChunk, A.q = window queries)
  int w, rows;         // window queries; query rows = w * r
  int pool;            // max-pool size over the sequence
  int add;             // add to the metric instead of replacing it
  int first_pos;       // position of query 0, the same for every head; -1 = the head's C - w
  int exclude;         // a query at position x adds to key j only when j <= x - exclude
  float* part;         // [partial slot][rows_pad][2]
  float* raw;          // [N * b] un-pooled sums, by physical slot
};

__device__ __forceinline__ f32x4_t mfma16(const uint4& a, const uint4& b, f32x4_t c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c,
                                                 0, 0, 0);
}

// Q of one head instance into LDS, in B-operand order: entry ((ct * 4 + kk) * 64 + lane) holds,
// for query row ct * 16 + lane % 16, the 8 dimensions 32 * (lane / 16) + 8 * kk .. + 8.
// Query row rho = i * r + hh (window query i, query head hh); rows past w * r are zero.
template <int NT>
__device__ __forceinline__ void stage_queries(const WindowArgs& W, int g, uint4* s_q) {
  const int r = W.A.D.r, w = W.w;
  const char* qbase = W.A.q + (size_t)g * r * w * 256;  // [r][w][128] bf16
  for (int e = threadIdx.x; e < NT * 4 * 64; e += kWinThreads) {
    const int lane = e & 63, kk = (e >> 6) & 3, ct = e >> 8;
    const int rho = ct * 16 + (lane & 15);
    uint4 v = make_uint4(0, 0, 0, 0);
    if (rho < W.rows) {
      const int i = rho / r, hh = rho % r;
      v = *(const uint4*)(qbase + ((size_t)hh * w + i) * 256 + 64 * (lane >> 4) + 16 * kk);
    }
    s_q[e] = v;
  }
}

// Loads the 64-token tile starting at chunk token `tt`: four blocks, four k-slices each.
// Blocks past the end of the chunk are not touched.
__device__ __forceinline__ void load_tile(const WindowArgs& W, const int* s_tab, int tt, int n_tok, int lane,
                                          uint4 (&k)[4][4]) {
  const int lb = W.A.log2b, b = W.A.D.b;
#pragma unroll
  for (int tg = 0; tg < 4; ++tg) {
    const int t = tt + tg * 16;
    if (t < n_tok) {
      const size_t slot = ((size_t)s_tab[t >> lb] << lb) + (t & (b - 1)) + (lane & 15);
      const char* p = W.A.kc + slot * 256 + 64 * (lane >> 4);
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) k[tg][kk] = *(const uint4*)(p + 16 * kk);
    } else {
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) k[tg][kk] = make_uint4(0, 0, 0, 0);
    }
  }
}

// Running (max, sum) pairs a wavefront keeps per column tile in pass 1.  One per lane (a lane
// covers 16 of a tile's 64 tokens for its query row) up to 128 query rows; at 256 rows the four
// lanes of a row merge theirs after every tile instead, four cross-lane moves per tile, which
// brings the workgroup from 96 KB of LDS to 72 and a second workgroup onto the CU.
__host__ __device__ constexpr int window_pairs_per_tile(int nt) { return nt >= 16 ? 16 : 64; }

// Pass 1: per chunk and query row, max and sum of exp2 over the visible keys.
template <int NT>
__global__ void __launch_bounds__(kWinThreads) window_stats_kernel(WindowArgs W) {
  constexpr int PPT = window_pairs_per_tile(NT);
  constexpr bool kRowMerged = PPT == 16;
  const DecodeArgs& A = W.A;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int total_items = A.header[HW_TOTAL_ITEMS];
  if ((int)blockIdx.x >= total_items || total_items > A.cap) return;
  const DecodeItem it = A.items[blockIdx.x];
  const int g = it.g, t0 = it.t0, n_tok = it.n_tok;
  if ((unsigned)g >= (unsigned)A.D.G || n_tok <= 0 || n_tok > A.T || t0 < 0 || it.nch <= 0 || it.pbase < 0 ||
      it.pbase + it.nch > A.cap)
    return;
  extern __shared__ __align__(16) char smem_raw[];
  uint4* s_q = (uint4*)smem_raw;                        // [NT * 4 * 64]
  float* s_ml = (float*)s_q;                            // [waves][NT * 16][2], once the main loops are over
  float2* s_st = (float2*)(s_q + NT * 4 * 64);          // [waves][NT][PPT]
  int* s_tab = (int*)(s_st + kWinWaves * NT * PPT);     // [T / b + 1]
  const int b = A.D.b, lb = A.log2b;
  const int C = A.ctx[g];
  {
    const int nblk = (n_tok + b - 1) >> lb;
    const int32_t* row = A.table + (size_t)g * A.D.maxb + (t0 >> lb);
    for (int i = tid; i < nblk; i += kWinThreads) s_tab[i] = row[i];
  }
  stage_queries<NT>(W, g, s_q);
  __syncthreads();
  // running (max, sum) of this lane's query row per column tile: kept in LDS so that the loop
  // over column tiles stays a loop (registers: one K tile and one Q tile at a time)
  float2* my_st = s_st + (size_t)wv * NT * PPT + (lane & (PPT - 1));
  for (int ct = 0; ct < NT; ++ct) my_st[ct * PPT] = make_float2(-INFINITY, 0.0f);
  const int first_free = W.first_pos >= 0 ? W.first_pos : C - W.w;  // query i sits at first_free + i
  const int free_lim = min(first_free, C - 1);   // keys up to here are visible to every query
  const bool dead = t0 > min(first_free + W.w - 1, C - 1);  // no query of the block sees this chunk
  for (int tt = wv * 64; tt < n_tok && !dead; tt += 64 * kWinWaves) {
    uint4 k[4][4];
    load_tile(W, s_tab, tt, n_tok, lane, k);
    // most tiles lie wholly in front of the window: they run the loop without the causal mask
    auto column_tiles = [&](auto masked_c) {
      constexpr bool kMasked = decltype(masked_c)::value;
#pragma unroll 1
      for (int ct = 0; ct < NT; ++ct) {
        uint4 q[4];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) q[kk] = s_q[(ct * 4 + kk) * 64 + lane];
        int last_vis = 0;
        if constexpr (kMasked) {
          const int rho = ct * 16 + (lane & 15);
          last_vis = min(first_free + rho / A.D.r, C - 1);  // query i sees keys 0 .. its position
        }
        // the running max stays in raw dot-product units inside the loop: the scale goes into one
        // multiply-add per logit (max, fma, exp2, add)
        const float2 old = my_st[ct * PPT];
        float s[16];
        float mx = old.x;
#pragma unroll
        for (int tg = 0; tg < 4; ++tg) {
          f32x4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
          for (int kk = 0; kk < 4; ++kk) acc = mfma16(k[tg][kk], q[kk], acc);
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            float x = acc[v];
            if constexpr (kMasked) {
              const int j = t0 + tt + tg * 16 + 4 * (lane >> 4) + v;
              if (j > last_vis) x = -INFINITY;
            }
            s[tg * 4 + v] = x;
            mx = fmaxf(mx, x);
          }
        }
        if constexpr (kRowMerged) {   // the row's max over the tile's 64 tokens
          mx = fmaxf(mx, __shfl_xor(mx, 16));
          mx = fmaxf(mx, __shfl_xor(mx, 32));
        }
        if (mx > -INFINITY) {   // (the same in the four lanes of a row when they merge)
          const float off = -mx * A.scale_log2;
          float sum = 0.0f;
#pragma unroll
          for (int e = 0; e < 16; ++e) sum += __builtin_amdgcn_exp2f(fmaf(s[e], A.scale_log2, off));
          if constexpr (kRowMerged) {
            sum += __shfl_xor(sum, 16);
            sum += __shfl_xor(sum, 32);
          }
          sum += old.y * __builtin_amdgcn_exp2f(fmaf(old.x, A.scale_log2, off));
          if (!kRowMerged || lane < 16) my_st[ct * PPT] = make_float2(mx, sum);
        }
      }
    };
    if (t0 + tt + 63 > free_lim) column_tiles(std::true_type{});
    else column_tiles(std::false_type{});
  }
  __syncthreads();   // every wavefront is done with Q: its bytes now take the per-wavefront pairs
  // merge the four lanes that share a query row, then the wavefronts, then write the chunk's pair
  for (int ct = 0; ct < NT; ++ct) {
    float2 st = my_st[ct * PPT];
    st.x *= A.scale_log2;   // from here on maxima are in scaled log2 units
#pragma unroll
    for (int msk = 16; msk <= (kRowMerged ? 0 : 32); msk <<= 1) {
      const float om = __shfl_xor(st.x, msk), ol = __shfl_xor(st.y, msk);
      const float nm = fmaxf(st.x, om);
      if (nm > -INFINITY) st.y = st.y * __builtin_amdgcn_exp2f(st.x - nm) + ol * __builtin_amdgcn_exp2f(om - nm);
      st.x = nm;
    }
    if (lane < 16) {
      s_ml[((wv * NT + ct) * 16 + lane) * 2 + 0] = st.x;
      s_ml[((wv * NT + ct) * 16 + lane) * 2 + 1] = st.y;
    }
  }
  __syncthreads();
  const size_t pslot = (size_t)it.pbase + (size_t)(t0 / A.T);
  for (int rho = tid; rho < NT * 16; rho += kWinThreads) {
    float mm = -INFINITY, ll = 0.0f;
    for (int ww = 0; ww < kWinWaves; ++ww) {
      const float om = s_ml[((ww * NT * 16) + rho) * 2], ol = s_ml[((ww * NT * 16) + rho) * 2 + 1];
      const float nm = fmaxf(mm, om);
      if (nm > -INFINITY) ll = ll * __builtin_amdgcn_exp2f(mm - nm) + ol * __builtin_amdgcn_exp2f(om - nm);
      mm = nm;
    }
    W.part[(pslot * NT * 16 + rho) * 2 + 0] = mm;
    W.part[(pslot * NT * 16 + rho) * 2 + 1] = ll;
  }
}

// Between the passes, once per head instance (the workgroup of its first chunk): the head's max
// and sum per query row from the per-chunk pairs, left as max + log2(sum) in the first chunk's
// slot, so that p = exp2(logit - that).  Padded rows and rows that see no key get +inf there:
// their p is exactly 0.  (Done here, not by every chunk's workgroup in pass 2: there the walk
// over the chunks' pairs, one dependent load after the other, was most of a workgroup's life.)
__global__ void __launch_bounds__(256) window_rows_kernel(WindowArgs W, int rows_pad) {
  const DecodeArgs& A = W.A;
  const int total_items = A.header[HW_TOTAL_ITEMS];
  if ((int)blockIdx.x >= total_items || total_items > A.cap) return;
  const DecodeItem it = A.items[blockIdx.x];
  if (it.t0 != 0 || (unsigned)it.g >= (unsigned)A.D.G || it.nch <= 0 || it.pbase < 0 || it.pbase + it.nch > A.cap) return;
  for (int rho = threadIdx.x; rho < rows_pad; rho += 256) {
    float mm = -INFINITY, ll = 0.0f;
    for (int cc = 0; cc < it.nch; ++cc) {
      const float2 ml = *(const float2*)(W.part + (((size_t)it.pbase + cc) * rows_pad + rho) * 2);
      const float nm = fmaxf(mm, ml.x);
      if (nm > -INFINITY) ll = ll * __builtin_amdgcn_exp2f(mm - nm) + ml.y * __builtin_amdgcn_exp2f(ml.x - nm);
      mm = nm;
    }
    W.part[((size_t)it.pbase * rows_pad + rho) * 2] = (rho < W.rows && ll > 0.0f) ? mm + __builtin_amdgcn_logf(ll) : INFINITY;
  }
}

// Pass 2: raw[j] = sum over query rows of p^2 (or p), p normalised with the head's max and sum.
template <int NT, bool L2>
__global__ void __launch_bounds__(kWinThreads) window_sum_kernel(WindowArgs W) {
  const DecodeArgs& A = W.A;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int total_items = A.header[HW_TOTAL_ITEMS];
  if (blockIdx.x == 0 && tid < HW_DEC_END - HW_DEC_BINS) A.header[HW_DEC_BINS + tid] = 0;  // work-list block back to zero
  if ((int)blockIdx.x >= total_items || total_items > A.cap) return;
  const DecodeItem it = A.items[blockIdx.x];
  const int g = it.g, t0 = it.t0, n_tok = it.n_tok, nch = it.nch;
  if ((unsigned)g >= (unsigned)A.D.G || n_tok <= 0 || n_tok > A.T || t0 < 0 || nch <= 0 || it.pbase < 0 ||
      it.pbase + nch > A.cap)
    return;
  extern __shared__ __align__(16) char smem_raw[];
  uint4* s_q = (uint4*)smem_raw;                        // [NT * 4 * 64]
  float* s_ml = (float*)(s_q + NT * 4 * 64);            // [NT * 16]: max + log2(sum) per query row (inf: the row adds nothing)
  int* s_tab = (int*)(s_ml + NT * 16);                  // [T / b + 1]
  const int b = A.D.b, lb = A.log2b;
  const int C = A.ctx[g];
  {
    const int nblk = (n_tok + b - 1) >> lb;
    const int32_t* row = A.table + (size_t)g * A.D.maxb + (t0 >> lb);
    for (int i = tid; i < nblk; i += kWinThreads) s_tab[i] = row[i];
  }
  stage_queries<NT>(W, g, s_q);
  for (int rho = tid; rho < NT * 16; rho += kWinThreads) s_ml[rho] = W.part[((size_t)it.pbase * NT * 16 + rho) * 2];
  __syncthreads();
  const int first_free = W.first_pos >= 0 ? W.first_pos : C - W.w;
  const int free_lim = min(first_free, C - 1) - W.exclude;   // keys up to here count for every query
  const bool dead = t0 > min(first_free + W.w - 1, C - 1) - W.exclude;  // the chunk gets nothing
  if (dead) {
    for (int t = tid; t < n_tok; t += kWinThreads)
      if (t0 + t < C) W.raw[((size_t)s_tab[t >> lb] << lb) + (t & (b - 1))] = 0.0f;
    return;
  }
  for (int tt = wv * 64; tt < n_tok; tt += 64 * kWinWaves) {
    uint4 k[4][4];
    load_tile(W, s_tab, tt, n_tok, lane, k);
    float tok[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) tok[e] = 0.0f;
    auto column_tiles = [&](auto masked_c) {
      constexpr bool kMasked = decltype(masked_c)::value;
#pragma unroll 1
      for (int ct = 0; ct < NT; ++ct) {
        uint4 q[4];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) q[kk] = s_q[(ct * 4 + kk) * 64 + lane];
        const int rho = ct * 16 + (lane & 15);
        int last_vis = 0;
        if constexpr (kMasked) last_vis = min(first_free + rho / A.D.r, C - 1) - W.exclude;
        const float c_row = s_ml[rho];
#pragma unroll
        for (int tg = 0; tg < 4; ++tg) {
          f32x4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
          for (int kk = 0; kk < 4; ++kk) acc = mfma16(k[tg][kk], q[kk], acc);
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            float p = __builtin_amdgcn_exp2f(fmaf(acc[v], A.scale_log2, -c_row));
            if constexpr (kMasked) {
              const int j = t0 + tt + tg * 16 + 4 * (lane >> 4) + v;
              if (j > last_vis) p = 0.0f;
            }
            tok[tg * 4 + v] = L2 ? fmaf(p, p, tok[tg * 4 + v]) : tok[tg * 4 + v] + p;
          }
        }
      }
    };
    if (t0 + tt + 63 > free_lim) column_tiles(std::true_type{});
    else column_tiles(std::false_type{});
    // sum over the 16 lanes of a row group: lane % 16 == e ends up with value e
    Butterfly<16, 8>::run(tok, lane);
    const int e = lane & 15;
    const int t = tt + (e >> 2) * 16 + 4 * (lane >> 4) + (e & 3);
    if (t < n_tok && t0 + t < C) {
      const size_t slot = ((size_t)s_tab[t >> lb] << lb) + (t & (b - 1));
      W.raw[slot] = tok[0];
    }
  }
}

// Max-pool over the logical sequence and the write into the metric.  One workgroup per head
// instance and tile of 2048 logical positions: the tile's un-pooled sums and a halo of pool / 2
// on either side are gathered into LDS once (a pool wider than the halo the LDS array has room
// for reads its neighbours from global memory instead).
constexpr int kPoolTile = 2048;
constexpr int kPoolHalo = 64;
__global__ void __launch_bounds__(256) window_pool_kernel(WindowArgs W) {
  const DecodeArgs& A = W.A;
  const int gi = blockIdx.x;
  const int g = sel_to_g(A.D, A.l0, A.nl, gi);
  const int C = A.ctx[g];
  const int j0 = blockIdx.y * kPoolTile;
  if (j0 >= C) return;
  const int j1 = min(C, j0 + kPoolTile);
  const int b = A.D.b, lb = A.log2b;
  const int32_t* row = A.table + (size_t)g * A.D.maxb;
  const int P = W.first_pos >= 0 ? 0 : max(0, C - W.w), half = W.pool / 2;
  __shared__ float s_raw[kPoolTile + 2 * kPoolHalo];
  const bool staged = half <= kPoolHalo;
  const int lo0 = staged ? max(0, j0 - half) : j0, hi0 = staged ? min(C, j1 + half) : j1;
  for (int j = lo0 + threadIdx.x; j < hi0; j += 256)
    s_raw[j - lo0] = W.raw[((size_t)row[j >> lb] << lb) + (j & (b - 1))];
  __syncthreads();
  for (int j = j0 + threadIdx.x; j < j1; j += 256) {
    const size_t slot = ((size_t)row[j >> lb] << lb) + (j & (b - 1));
    float v = s_raw[j - lo0];
    if (j < P) {
      const int lo = max(0, j - half), hi = min(P - 1, j + half);
      if (staged) {
        for (int t = lo; t <= hi; ++t) v = fmaxf(v, s_raw[t - lo0]);
      } else {
        for (int t = lo; t <= hi; ++t) v = fmaxf(v, W.raw[((size_t)row[t >> lb] << lb) + (t & (b - 1))]);
      }
    }
    A.metric[slot] = W.add ? A.metric[slot] + v : v;
  }
}

template <int NT>
static int launch_window(const WindowArgs& W, int grid, hipStream_t s) {
  // pass 1: Q (later the per-wavefront pairs), running pairs per column tile, block ids;
  // pass 2: Q, one float per query row, block ids.  Three and four workgroups per CU at 128 rows,
  // two and two at 256.
  const size_t tab = ((size_t)kWinChunk / W.A.D.b + 1) * 4;
  const size_t lds = (size_t)NT * 4 * 64 * 16 + (size_t)kWinWaves * NT * window_pairs_per_tile(NT) * 8 + tab;
  const size_t lds2 = (size_t)NT * 4 * 64 * 16 + (size_t)NT * 16 * 4 + tab;
  static_assert((size_t)kWinWaves * NT * 16 * 2 * 4 <= (size_t)NT * 4 * 64 * 16, "pairs fit where Q was");
  static size_t allowed = 0;   // above the default cap a kernel must be told how much it may take
  if (lds > 64 * 1024 && lds > allowed) {   // (lds >= lds2; the block-id array grows as blocks shrink)
    KVC_HIP(hipFuncSetAttribute((const void*)window_stats_kernel<NT>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    KVC_HIP(hipFuncSetAttribute((const void*)window_sum_kernel<NT, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    KVC_HIP(hipFuncSetAttribute((const void*)window_sum_kernel<NT, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    allowed = lds;
  }
  hipLaunchKernelGGL(window_stats_kernel<NT>, dim3(grid), dim3(kWinThreads), lds, s, W);
  KVC_LAUNCH_CHECK();
  hipLaunchKernelGGL(window_rows_kernel, dim3(grid), dim3(256), 0, s, W, NT * 16);
  KVC_LAUNCH_CHECK();
  if (W.A.D.mode == KVC_L2) hipLaunchKernelGGL((window_sum_kernel<NT, true>), dim3(grid), dim3(kWinThreads), lds2, s, W);
  else hipLaunchKernelGGL((window_sum_kernel<NT, false>), dim3(grid), dim3(kWinThreads), lds2, s, W);
  KVC_LAUNCH_CHECK();
  return KVC_OK;
}

}  // namespace kvc

using namespace kvc;

extern "C" {

static int window_common(const kvc_config* cfg, const kvc_state* st, const void* q_win, int w, int pool,
                         int accumulate, int first_pos, int exclude, int layer_begin, int layer_end, void* ws,
                         void* stream) {
  int rc = validate(cfg, st);
  if (rc != KVC_OK) return rc;
  if (!q_win || !ws || ((uintptr_t)ws & 255) || ((uintptr_t)q_win & 15)) return KVC_ERR_ARG;
  Dims D = dims_of(cfg);
  if (layer_begin < 0 || layer_end > D.Lyr || layer_begin >= layer_end) return KVC_ERR_ARG;
  if (w <= 0 || pool <= 0 || (pool & 1) == 0 || exclude < 0) return KVC_ERR_ARG;
  // the matrix-core kernels cover bf16, d = 128, blocks of a multiple of 16 tokens, up to 256 query rows
  if (D.dtype != KVC_BF16 || D.d != 128 || D.b % 16 != 0 || 64 % D.b != 0) return KVC_ERR_UNSUPPORTED;
  const int rows = w * D.r;
  // (w <= 64: a chunk's pairs, 8 bytes per padded query row, live in the decode's slot of r * d floats)
  if (rows > 256 || w > 64) return KVC_ERR_UNSUPPORTED;
  const int nt = rows <= 32 ? 2 : rows <= 64 ? 4 : rows <= 128 ? 8 : 16;
  if ((size_t)nt * 16 * 8 > (size_t)D.r * D.d * 4) return KVC_ERR_UNSUPPORTED;
  Workspace Wk = carve(D, ws);
  hipStream_t s = (hipStream_t)stream;
  WindowArgs W;
  DecodeArgs& A = W.A;
  A.D = D;
  A.kc = (const char*)st->k_cache; A.vc = (const char*)st->v_cache;
  A.metric = st->metric; A.table = st->block_table; A.ctx = st->ctx_len;
  A.q = (const char*)q_win; A.out = nullptr;
  A.l0 = layer_begin; A.nl = layer_end - layer_begin; A.gsel = D.S * A.nl * D.Hk;
  A.accumulate = 1; A.T = kWinChunk;
  A.log2b = 0;
  while ((1 << A.log2b) < D.b) ++A.log2b;
  A.all_partials = 1;
  A.short_class = 16;  // no separate launch for short items here
  A.Ts = 0;
  A.cap = (int)(max_items_of(D) < 0x7fffffffull ? max_items_of(D) : 0x7fffffffull);
  A.items = (DecodeItem*)Wk.items; A.slot_item = Wk.slot_item; A.part_ml = Wk.part_ml; A.part_acc = Wk.part_acc; A.stash = Wk.stash;
  A.header = Wk.header;
  A.scale_log2 = (float)(1.4426950408889634 / 11.313708498984761);  // log2(e) / sqrt(128)
  W.w = w; W.rows = rows; W.pool = pool; W.add = accumulate != 0;
  W.first_pos = first_pos; W.exclude = exclude;
  W.part = Wk.part_acc; W.raw = Wk.stash;
  // a head that holds no KV has no output here: the item kernel's zero rows must not be written
  if (A.gsel <= kSmallWorklistHeads) {
    hipLaunchKernelGGL(decode_worklist_small_kernel, dim3(1), dim3(1024), 0, s, A);
    KVC_LAUNCH_CHECK();
  } else {
    hipLaunchKernelGGL(decode_count_kernel, dim3((A.gsel + 255) / 256), dim3(256), 0, s, A);
    KVC_LAUNCH_CHECK();
    hipLaunchKernelGGL(decode_items_kernel, dim3((A.gsel + 255) / 256), dim3(256), 0, s, A);
    KVC_LAUNCH_CHECK();
  }
  const size_t bound_pool = (size_t)D.N * D.b / A.T + (size_t)A.gsel;
  const size_t bound_row = (size_t)A.gsel * (((size_t)D.maxb * D.b + A.T - 1) / A.T);
  const size_t grid = bound_pool < bound_row ? bound_pool : bound_row;
  if (grid > 0x7fffffffull) return KVC_ERR_UNSUPPORTED;
  switch (nt) {
    case 2: rc = launch_window<2>(W, (int)grid, s); break;
    case 4: rc = launch_window<4>(W, (int)grid, s); break;
    case 8: rc = launch_window<8>(W, (int)grid, s); break;
    default: rc = launch_window<16>(W, (int)grid, s); break;
  }
  if (rc != KVC_OK) return rc;
  const int pool_tiles = (int)(((size_t)D.maxb * D.b + kPoolTile - 1) / kPoolTile);
  if (pool_tiles > 65535) return KVC_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(window_pool_kernel, dim3(A.gsel, pool_tiles), dim3(256), 0, s, W);
  KVC_LAUNCH_CHECK();
  return KVC_OK;
}

int kvc_window_metric(const kvc_config* cfg, const kvc_state* st, const void* q_win, int w, int pool,
                      int accumulate, int layer_begin, int layer_end, void* ws, void* stream) {
  return window_common(cfg, st, q_win, w, pool, accumulate, -1, 0, layer_begin, layer_end, ws, stream);
}

int kvc_query_block_metric(const kvc_config* cfg, const kvc_state* st, const void* q_blk, int w, int first_pos,
                           int exclude, int layer_begin, int layer_end, void* ws, void* stream) {
  if (first_pos < 0) return KVC_ERR_ARG;
  return window_common(cfg, st, q_blk, w, 1, 1, first_pos, exclude, layer_begin, layer_end, ws, stream);
}

}  // extern "C"
