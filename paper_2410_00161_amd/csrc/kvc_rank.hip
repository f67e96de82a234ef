// The paper's own eviction schedule ("Evicting from a Paged KV Cache", steps
// M1..W7) without any sort.
//
// In the paper each head's metrics are sorted, cut into rows of b (the empty
// slots of its last block first, as zeros), row e-1 is what evicting the head's
// e-th block removes and its last column m(h, e) orders the rows of all heads.
// Two facts make sorting unnecessary:
//   * row k of a head has m <= x exactly when the head has at least (k+1)*b
//     entries <= x, so the number of candidate rows of a head with m <= x is
//     min(candidates, floor(count(<= x) / b)).  Summed over the heads of a
//     segment this is monotone in x, and an 8-bit-per-pass radix descent on the
//     f32 bit pattern finds the E-th smallest m and how many rows tie with it;
//   * once a head knows how many rows e it loses, the KVs it loses are its
//     e*b - (empty slots) smallest by (metric, logical index): a per-head
//     radix select gives the threshold metric and the number of ties to take.
// The compaction is MoveCache (Algorithm 1) for a slot-granular mask: holes and
// movers are ranked with ordered prefix counts and paired k-th to k-th.
#include "kvc_common.h"

namespace kvc {

enum { RS_PREFIX = SEG_PREFIX, RS_REMAIN = SEG_REMAIN, RS_CAND = SEG_CAND, RS_TAKE = SEG_TAKE, RS_FIRSTG = SEG_FIRSTG };

// Heads of at most this many KVs (by the table's row length) get a wavefront each in the histogram
// passes of the rank schedule; longer ones a workgroup.
constexpr size_t kRankWaveTokens = 16384;

__device__ __forceinline__ uint32_t metric_bits(float f) {
  const uint32_t k = __float_as_uint(f);
  return k == 0x80000000u ? 0u : k;  // -0 orders as +0
}

// A head's metrics as ordered bit patterns, four strided elements per thread at a time: the four
// block ids are requested together, then the four metrics, so that a pass over a head waits for
// two rounds of loads per four elements instead of two per element.  visit(j, bits) sees every
// logical slot j < C once.
template <int NTH, class Visit>
__device__ __forceinline__ void for_each_metric(const float* __restrict__ metric, const int32_t* __restrict__ row,
                                                int C, int lb, int bmask, Visit visit) {
  if (bmask >= 3) {
    // blocks of at least four slots: four consecutive slots (one block) per load, so a round of
    // loads covers 16 slots per thread
    const int nq = (C + 3) >> 2;
    for (int q0 = threadIdx.x; q0 < nq; q0 += 4 * NTH) {
      int id[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) id[i] = row[(4 * min(q0 + i * NTH, nq - 1)) >> lb];
      float4 m[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int j = 4 * min(q0 + i * NTH, nq - 1);
        m[i] = *(const float4*)&metric[((size_t)id[i] << lb) + (j & bmask)];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int j = 4 * (q0 + i * NTH);
        if (j < C) visit(j, metric_bits(m[i].x));
        if (j + 1 < C) visit(j + 1, metric_bits(m[i].y));
        if (j + 2 < C) visit(j + 2, metric_bits(m[i].z));
        if (j + 3 < C) visit(j + 3, metric_bits(m[i].w));
      }
    }
    return;
  }
  for (int j0 = threadIdx.x; j0 < C; j0 += 4 * NTH) {
    int id[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) id[i] = row[min(j0 + i * NTH, C - 1) >> lb];
    float m[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int j = min(j0 + i * NTH, C - 1);
      m[i] = metric[((size_t)id[i] << lb) + (j & bmask)];
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (j0 + i * NTH < C) visit(j0 + i * NTH, metric_bits(m[i]));
  }
}


// One workgroup (NTH threads: 256, or 1024 when there are few, long heads) per heads_per_wg
// consecutive head instances, one after the other.  Counts a
// head's entries below the prefix found so far and histograms the next digit of those that
// match it; turns the running counts into rows per digit; the rows of all its heads go to the
// segment's histogram together (thread = digit), so that one address sees G / heads_per_wg
// adds per pass instead of G: adds to one word from all over the chip run one after the other,
// and in the first pass (the exponent byte) nearly every head lands on the same digit.
template <int NTH>
__global__ void __launch_bounds__(NTH) rank_hist_kernel(Dims D, int pass, int protect, int heads_per_wg,
                                                        const float* __restrict__ metric,
                                                        const int32_t* __restrict__ table,
                                                        const int32_t* __restrict__ ctx,
                                                        const int32_t* __restrict__ seq_seg,
                                                        int32_t* __restrict__ seg_hist,
                                                        int32_t* __restrict__ seg_state,
                                                        int32_t* __restrict__ header) {
  __shared__ int hist[256];
  __shared__ int below_s;
  __shared__ int smem[NTH / 64 + 1];
  const int tid = threadIdx.x;
  const int g_first = blockIdx.x * heads_per_wg;
  const int g_end = min(D.G, g_first + heads_per_wg);
  const int shift = 24 - 8 * pass;
  int lb = 0;
  while ((1 << lb) < D.b) ++lb;   // block sizes are powers of two
  int cur_sg = -1, rows_acc = 0, cand_acc = 0;
  auto flush = [&]() {
    if (cur_sg < 0) return;
    if (tid < 256 && rows_acc) atomicAdd(&seg_hist[cur_sg * 256 + tid], rows_acc);
    if (pass == 0 && tid == 0 && cand_acc) atomicAdd(&seg_state[cur_sg * 8 + RS_CAND], cand_acc);
    rows_acc = 0;
    cand_acc = 0;
  };
  for (int g = g_first; g < g_end; ++g) {
    const int sg = seq_seg[g / (D.Lyr * D.Hk)];
    if (sg != cur_sg) { flush(); cur_sg = sg; }
    const int C = ctx[g];
    const int nb = (C + D.b - 1) / D.b;
    const int ncand = max(0, nb - protect);
    cand_acc += ncand;
    if (ncand == 0) continue;
    if (pass > 0 && seg_state[sg * 8 + RS_TAKE] <= 0) continue;
    if (tid < 256) hist[tid] = 0;
    if (tid == 0) below_s = 0;
    __syncthreads();
    const uint32_t prefix = (uint32_t)seg_state[sg * 8 + RS_PREFIX];
    const int32_t* row = table + (size_t)g * D.maxb;
    int below = 0;
    bool bad = false;
    for_each_metric<NTH>(metric, row, C, lb, D.b - 1, [&](int, uint32_t k) {
      if (pass == 0) bad |= k >= 0x7f800000u;
      const uint32_t top = pass == 0 ? 0u : (k >> (shift + 8));
      if (top < prefix) ++below;
      else if (top == prefix) atomicAdd(&hist[(k >> shift) & 255], 1);
    });
    const int z = nb * D.b - C;  // the empty slots count as zeros, ahead of every real metric
    if (tid == 0 && z) {
      if (prefix == 0) atomicAdd(&hist[0], z); else below += z;
    }
    below = wave_sum_i(below);
    if ((tid & 63) == 0 && below) atomicAdd(&below_s, below);
    if (bad) atomicOr(&header[HW_SCRATCH0], EB_NUMERIC);
    __syncthreads();
    const int c = tid < 256 ? hist[tid] : 0;
    const int ex = block_exclusive_scan<NTH>(c, smem, nullptr) + below_s;
    if (tid < 256) rows_acc += min(ncand, (ex + c) >> lb) - min(ncand, ex >> lb);
    __syncthreads();   // hist and below_s are reused by the next head
  }
  flush();
}

// The same step with one wavefront per head instance (four per workgroup, each taking
// heads_per_wave consecutive heads), for caches of many heads of a few thousand KVs at most:
// nothing in it waits at a barrier, the 256 counters of a head are four per lane, and a CU holds
// four times as many heads in flight as with a workgroup per head (16 384 heads of ~1000 KVs:
// a pass took 50 us that way).
__global__ void __launch_bounds__(256) rank_hist_wave_kernel(Dims D, int pass, int protect, int heads_per_wave,
                                                             const float* __restrict__ metric,
                                                             const int32_t* __restrict__ table,
                                                             const int32_t* __restrict__ ctx,
                                                             const int32_t* __restrict__ seq_seg,
                                                             int32_t* __restrict__ seg_hist,
                                                             int32_t* __restrict__ seg_state,
                                                             int32_t* __restrict__ header) {
  __shared__ __align__(16) int hist_all[4][256];
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  int* hist = hist_all[wv];   // this wavefront's own: its LDS accesses happen in program order
  const int g_first = (blockIdx.x * 4 + wv) * heads_per_wave;
  const int g_end = min(D.G, g_first + heads_per_wave);
  const int shift = 24 - 8 * pass;
  int lb = 0;
  while ((1 << lb) < D.b) ++lb;   // block sizes are powers of two
  const int bmask = D.b - 1;
  int cur_sg = -1, cand_acc = 0;
  int rows_acc[4] = {0, 0, 0, 0};   // digits 4 lane .. 4 lane + 3
  bool bad = false;
  auto flush = [&]() {
    if (cur_sg < 0) return;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      if (rows_acc[k]) atomicAdd(&seg_hist[cur_sg * 256 + 4 * lane + k], rows_acc[k]);
      rows_acc[k] = 0;
    }
    if (pass == 0 && lane == 0 && cand_acc) atomicAdd(&seg_state[cur_sg * 8 + RS_CAND], cand_acc);
    cand_acc = 0;
  };
  for (int g = g_first; g < g_end; ++g) {
    const int sg = seq_seg[g / (D.Lyr * D.Hk)];
    if (sg != cur_sg) { flush(); cur_sg = sg; }
    const int C = ctx[g];
    const int nb = (C + D.b - 1) / D.b;
    const int ncand = max(0, nb - protect);
    cand_acc += ncand;
    if (ncand == 0) continue;
    if (pass > 0 && seg_state[sg * 8 + RS_TAKE] <= 0) continue;
    *(int4*)(hist + 4 * lane) = make_int4(0, 0, 0, 0);
    const uint32_t prefix = (uint32_t)seg_state[sg * 8 + RS_PREFIX];
    const int32_t* row = table + (size_t)g * D.maxb;
    int below = 0;
    auto count = [&](uint32_t k) {
      if (pass == 0) bad |= k >= 0x7f800000u;
      const uint32_t top = pass == 0 ? 0u : (k >> (shift + 8));
      if (top < prefix) ++below;
      else if (top == prefix) atomicAdd(&hist[(k >> shift) & 255], 1);
    };
    if (D.b >= 4) {
      // four consecutive slots (one block: b is a power of two >= 4) per lane and load: a head of
      // 1000 KVs is four block ids and four 16-byte loads per lane, all asked for together
      const int nq = (C + 3) >> 2;
      for (int q0 = lane; q0 < nq; q0 += 4 * 64) {
        int id[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) id[i] = row[(4 * min(q0 + i * 64, nq - 1)) >> lb];
        float4 m[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int j = 4 * min(q0 + i * 64, nq - 1);
          m[i] = *(const float4*)&metric[((size_t)id[i] << lb) + (j & bmask)];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int j = 4 * (q0 + i * 64);
          if (j < C) count(metric_bits(m[i].x));
          if (j + 1 < C) count(metric_bits(m[i].y));
          if (j + 2 < C) count(metric_bits(m[i].z));
          if (j + 3 < C) count(metric_bits(m[i].w));
        }
      }
    } else {
      for (int j0 = lane; j0 < C; j0 += 4 * 64) {   // four block ids, then four metrics, asked for together
        int id[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) id[i] = row[min(j0 + i * 64, C - 1) >> lb];
        float m[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int j = min(j0 + i * 64, C - 1);
          m[i] = metric[((size_t)id[i] << lb) + (j & bmask)];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (j0 + i * 64 < C) count(metric_bits(m[i]));
      }
    }
    const int z = nb * D.b - C;  // the empty slots count as zeros, ahead of every real metric
    if (lane == 0 && z) {
      if (prefix == 0) atomicAdd(&hist[0], z); else below += z;
    }
    below = wave_sum_i(below);
    // running counts over the digits in order: four per lane, then over the lanes
    const int4 c = *(const int4*)(hist + 4 * lane);
    const int mine = c.x + c.y + c.z + c.w;
    int inc = mine;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int t = __shfl_up(inc, o);
      if (lane >= o) inc += t;
    }
    int ex = below + inc - mine;
    const int cc[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      rows_acc[k] += min(ncand, (ex + cc[k]) >> lb) - min(ncand, ex >> lb);
      ex += cc[k];
    }
  }
  flush();
  if (__any(bad) && lane == 0) atomicOr(&header[HW_SCRATCH0], EB_NUMERIC);
}

// One workgroup per segment: the digit that holds the E-th smallest row key (same rule as the
// block-key selection).
__global__ void __launch_bounds__(256) rank_pick_kernel(int pass, const int32_t* __restrict__ budget,
                                                        int32_t* __restrict__ seg_hist,
                                                        int32_t* __restrict__ seg_state,
                                                        int32_t* __restrict__ header) {
  __shared__ int smem[256 / 64 + 1];
  __shared__ int chosen;
  const int sg = blockIdx.x;
  int32_t* stt = seg_state + sg * 8;
  if (pass == 0 && threadIdx.x == 0) {
    int bud = budget[sg];
    if (bud < 0) { atomicOr(&header[HW_SCRATCH0], EB_ARG); bud = 0; }
    const int take = min(bud, stt[RS_CAND]);
    stt[RS_TAKE] = take;
    stt[RS_REMAIN] = take;
  }
  __syncthreads();
  const int take = stt[RS_TAKE];
  const int remain = stt[RS_REMAIN];
  const int c = seg_hist[sg * 256 + threadIdx.x];
  const int ex = block_exclusive_scan<256>(c, smem, nullptr);
  if (threadIdx.x == 0) chosen = -1;
  __syncthreads();
  if (take > 0 && ex < remain && remain <= ex + c) chosen = threadIdx.x;
  __syncthreads();
  if (take > 0 && (int)threadIdx.x == chosen) {
    stt[RS_PREFIX] = (int32_t)(((uint32_t)stt[RS_PREFIX] << 8) | (uint32_t)chosen);
    stt[RS_REMAIN] = remain - ex;
  }
  seg_hist[sg * 256 + threadIdx.x] = 0;
}

// Rows strictly below the threshold key, and rows that tie with it, per head.
__global__ void __launch_bounds__(256) rank_tie_kernel(Dims D, int protect, const float* __restrict__ metric,
                                                       const int32_t* __restrict__ table,
                                                       const int32_t* __restrict__ ctx,
                                                       const int32_t* __restrict__ seq_seg,
                                                       const int32_t* __restrict__ seg_state,
                                                       int32_t* __restrict__ rows_lt,
                                                       int32_t* __restrict__ rows_tie) {
  __shared__ int lt_s, le_s;
  const int g = blockIdx.x, tid = threadIdx.x;
  const int sg = seq_seg[g / (D.Lyr * D.Hk)];
  const int C = ctx[g];
  const int nb = (C + D.b - 1) / D.b;
  const int ncand = max(0, nb - protect);
  if (ncand == 0 || seg_state[sg * 8 + RS_TAKE] <= 0) {
    if (tid == 0) { rows_lt[g] = 0; rows_tie[g] = 0; }
    return;
  }
  if (tid == 0) { lt_s = 0; le_s = 0; }
  __syncthreads();
  const uint32_t thr = (uint32_t)seg_state[sg * 8 + RS_PREFIX];
  const int32_t* row = table + (size_t)g * D.maxb;
  int lt = 0, le = 0;
  int lb = 0;
  while ((1 << lb) < D.b) ++lb;   // block sizes are powers of two
  for_each_metric<256>(metric, row, C, lb, D.b - 1, [&](int, uint32_t k) {
    lt += k < thr;
    le += k <= thr;
  });
  if (tid == 0) {
    const int z = nb * D.b - C;
    le += z;
    if (thr > 0) lt += z;
  }
  lt = wave_sum_i(lt);
  le = wave_sum_i(le);
  if ((tid & 63) == 0) { atomicAdd(&lt_s, lt); atomicAdd(&le_s, le); }
  __syncthreads();
  if (tid == 0) {
    const int a = min(ncand, lt_s / D.b), c = min(ncand, le_s / D.b);
    rows_lt[g] = a;
    rows_tie[g] = c - a;
  }
}

// The same with one wavefront per head instance (heads of a few thousand KVs at most), four
// consecutive slots per lane and load when a block holds at least four.
__global__ void __launch_bounds__(256) rank_tie_wave_kernel(Dims D, int protect, const float* __restrict__ metric,
                                                            const int32_t* __restrict__ table,
                                                            const int32_t* __restrict__ ctx,
                                                            const int32_t* __restrict__ seq_seg,
                                                            const int32_t* __restrict__ seg_state,
                                                            int32_t* __restrict__ rows_lt,
                                                            int32_t* __restrict__ rows_tie) {
  const int lane = threadIdx.x & 63;
  const int g = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (g >= D.G) return;
  const int sg = seq_seg[g / (D.Lyr * D.Hk)];
  const int C = ctx[g];
  const int nb = (C + D.b - 1) / D.b;
  const int ncand = max(0, nb - protect);
  if (ncand == 0 || seg_state[sg * 8 + RS_TAKE] <= 0) {
    if (lane == 0) { rows_lt[g] = 0; rows_tie[g] = 0; }
    return;
  }
  const uint32_t thr = (uint32_t)seg_state[sg * 8 + RS_PREFIX];
  const int32_t* row = table + (size_t)g * D.maxb;
  int lt = 0, le = 0;
  int lb = 0;
  while ((1 << lb) < D.b) ++lb;   // block sizes are powers of two
  const int bmask = D.b - 1;
  auto count = [&](uint32_t k) { lt += k < thr; le += k <= thr; };
  if (D.b >= 4) {
    const int nq = (C + 3) >> 2;
    for (int q0 = lane; q0 < nq; q0 += 4 * 64) {
      int id[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) id[i] = row[(4 * min(q0 + i * 64, nq - 1)) >> lb];
      float4 m[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int j = 4 * min(q0 + i * 64, nq - 1);
        m[i] = *(const float4*)&metric[((size_t)id[i] << lb) + (j & bmask)];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int j = 4 * (q0 + i * 64);
        if (j < C) count(metric_bits(m[i].x));
        if (j + 1 < C) count(metric_bits(m[i].y));
        if (j + 2 < C) count(metric_bits(m[i].z));
        if (j + 3 < C) count(metric_bits(m[i].w));
      }
    }
  } else {
    for (int j0 = lane; j0 < C; j0 += 4 * 64) {
      int id[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) id[i] = row[min(j0 + i * 64, C - 1) >> lb];
      float m[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int j = min(j0 + i * 64, C - 1);
        m[i] = metric[((size_t)id[i] << lb) + (j & bmask)];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (j0 + i * 64 < C) count(metric_bits(m[i]));
    }
  }
  if (lane == 0) {
    const int z = nb * D.b - C;
    le += z;
    if (thr > 0) lt += z;
  }
  lt = wave_sum_i(lt);
  le = wave_sum_i(le);
  if (lane == 0) {
    const int a = min(ncand, lt / D.b), c = min(ncand, le / D.b);
    rows_lt[g] = a;
    rows_tie[g] = c - a;
  }
}

struct RowTieFn {
  const int32_t* cnt;
  __device__ int operator()(int i) const { return cnt[i]; }
};

__global__ void __launch_bounds__(256) rank_grant_kernel(Dims D, const int32_t* __restrict__ seq_seg,
                                                         const int32_t* __restrict__ seg_state,
                                                         const int32_t* __restrict__ rows_tie,
                                                         const int32_t* __restrict__ tie_off,
                                                         int32_t* __restrict__ evict_rows,
                                                         int32_t* __restrict__ selected,
                                                         const int32_t* __restrict__ header) {
  const int g = blockIdx.x * 256 + threadIdx.x;
  if (g >= D.G) return;
  if (header[HW_STATUS] != KVC_OK) { evict_rows[g] = 0; return; }
  const int sg = seq_seg[g / (D.Lyr * D.Hk)];
  const int32_t* stt = seg_state + sg * 8;
  const int take = stt[RS_TAKE];
  if (g == stt[RS_FIRSTG]) selected[sg] = take;
  if (take <= 0) { evict_rows[g] = 0; return; }
  const int before = tie_off[g] - tie_off[stt[RS_FIRSTG]];
  const int granted = max(0, min(rows_tie[g], stt[RS_REMAIN] - before));
  evict_rows[g] += granted;  // evict_rows holds the rows strictly below the threshold
}

// ---------------------------------------------------------------------------
// compaction for a head that loses e rows
// ---------------------------------------------------------------------------

__global__ void __launch_bounds__(256) rank_check_kernel(Dims D, const int32_t* __restrict__ ctx,
                                                         const int32_t* __restrict__ evict_rows,
                                                         int32_t* __restrict__ header) {
  const int g = blockIdx.x * 256 + threadIdx.x;
  if (g >= D.G) return;
  const int nb = (ctx[g] + D.b - 1) / D.b;
  const int e = evict_rows[g];
  if (e < 0 || e > nb) atomicOr(&header[HW_SCRATCH0], EB_ARG);
}

// One workgroup per head.  scratch is an int array shaped like the metric ([N, b]); the head
// uses the cells of its own blocks: hole k at logical cell k, mover k at logical cell C-1-k.
// NTH threads: 256 when there are many head instances, 1024 when there are few (a prompt's
// worth of long heads), so that a head's passes over its metrics run four times as wide.
template <int NTH>
__global__ void __launch_bounds__(NTH) rank_compact_kernel(Dims D, char* __restrict__ kc, char* __restrict__ vc,
                                                           float* __restrict__ metric,
                                                           int32_t* __restrict__ pos,
                                                           int32_t* __restrict__ table,
                                                           int32_t* __restrict__ ctx,
                                                           uint8_t* __restrict__ free_map,
                                                           const int32_t* __restrict__ evict_rows,
                                                           int32_t* __restrict__ scratch,
                                                           int32_t* __restrict__ header, int lds_tokens) {
  if (header[HW_STATUS] != KVC_OK) return;
  const int g = blockIdx.x, tid = threadIdx.x;
  const int e = evict_rows[g];
  if (e <= 0) return;
  __shared__ int hist[256];
  __shared__ int prefix_s, remain_s;
  // the head's metrics as ordered bit patterns, kept from the first radix pass on when the head
  // fits the lds_tokens words this launch has: the three passes and the ordered pass after it
  // then read LDS instead of gathering through the table again
  extern __shared__ uint32_t s_bits[];
  const int b = D.b;
  int lb = 0;
  while ((1 << lb) < b) ++lb;   // block sizes are powers of two
  const int C = ctx[g];
  const int nb = (C + b - 1) / b;
  const int n_ev = e * b - (nb * b - C);  // real KVs in the first e rows
  const int T = C - n_ev;                 // = (nb - e) * b
  int32_t* row = table + (size_t)g * D.maxb;
  auto phys = [&](int j) -> size_t { return ((size_t)row[j >> lb] << lb) + (j & (b - 1)); };
  const bool kept = C <= lds_tokens;

  // ---- threshold metric: the n_ev-th smallest by (metric, logical index) ----
  // Three barriers per pass: the 256 counters are walked by the first wavefront alone, four per
  // lane (a scan over the whole workgroup would wait at six more).
  const int lane = tid & 63, wv = tid >> 6;
  if (tid == 0) { prefix_s = 0; remain_s = n_ev; }
  for (int pass = 0; pass < 4; ++pass) {
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    const int shift = 24 - 8 * pass;
    const uint32_t prefix = (uint32_t)prefix_s;
    if (pass == 0 || !kept) {
      for_each_metric<NTH>(metric, row, C, lb, b - 1, [&](int j, uint32_t k) {
        if (pass == 0 && kept) s_bits[j] = k;
        if (pass == 0 || (k >> (shift + 8)) == prefix) atomicAdd(&hist[(k >> shift) & 255], 1);
      });
    } else {
      for (int j = tid; j < C; j += NTH) {
        const uint32_t k = s_bits[j];
        if ((k >> (shift + 8)) == prefix) atomicAdd(&hist[(k >> shift) & 255], 1);
      }
    }
    __syncthreads();
    if (wv == 0) {
      const int c4[4] = {hist[4 * lane], hist[4 * lane + 1], hist[4 * lane + 2], hist[4 * lane + 3]};
      const int mine = c4[0] + c4[1] + c4[2] + c4[3];
      int inc = mine;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_up(inc, o);
        if (lane >= o) inc += t;
      }
      int ex = inc - mine;
      const int remain = remain_s;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (ex < remain && remain <= ex + c4[q]) {   // exactly one lane and digit
          prefix_s = (int)((prefix << 8) | (uint32_t)(4 * lane + q));
          remain_s = remain - ex;
        }
        ex += c4[q];
      }
    }
    __syncthreads();
  }
  const uint32_t thr = (uint32_t)prefix_s;
  const int ties_take = remain_s;

  // ---- ordered pass: who is evicted, hole and mover ranks ----
  // Ranks inside a wavefront come from ballots; the wavefronts exchange their counts through LDS,
  // two barriers per round of NTH slots (counts double-buffered by the round's parity), and every
  // thread keeps the running totals itself.
  __shared__ int cnt_s[2][3][NTH / 64];
  const unsigned long long lower = (1ull << lane) - 1ull;
  int carry_tie = 0, carry_ev = 0, n_moves = 0;
  auto ordered_round = [&](int base, int par, uint32_t k) {
    const int j = base + tid;
    const bool is_tie = (j < C) && k == thr;
    const unsigned long long tm = __ballot(is_tie);
    if (lane == 0) cnt_s[par][0][wv] = __popcll(tm);
    __syncthreads();
    int tie_rank = carry_tie + __popcll(tm & lower), tot_tie = 0;
#pragma unroll
    for (int w2 = 0; w2 < NTH / 64; ++w2) {
      const int c = cnt_s[par][0][w2];
      if (w2 < wv) tie_rank += c;
      tot_tie += c;
    }
    const bool ev = (j < C) && (k < thr || (is_tie && tie_rank < ties_take));
    const unsigned long long em = __ballot(ev);
    const unsigned long long hm = __ballot(ev && j < T);
    if (lane == 0) { cnt_s[par][1][wv] = __popcll(em); cnt_s[par][2][wv] = __popcll(hm); }
    __syncthreads();
    int ev_before = carry_ev + __popcll(em & lower), tot_ev = 0;
#pragma unroll
    for (int w2 = 0; w2 < NTH / 64; ++w2) {
      const int c = cnt_s[par][1][w2];
      if (w2 < wv) ev_before += c;
      tot_ev += c;
      n_moves += cnt_s[par][2][w2];
    }
    if (j < C) {
      if (ev) {
        if (j < T) scratch[phys(ev_before)] = j;
      } else if (j >= T) {
        const int kk = (C - 1 - j) - (n_ev - ev_before);  // kept slots above j
        scratch[phys(C - 1 - kk)] = j;
      }
    }
    carry_tie += tot_tie;
    carry_ev += tot_ev;
  };
  {
    for (int base = 0, par = 0; base < C; base += NTH, par ^= 1) {
      const int j = base + tid;
      uint32_t k = 0xffffffffu;
      if (j < C) k = kept ? s_bits[j] : metric_bits(metric[phys(j)]);
      ordered_round(base, par, k);
    }
  }
  __syncthreads();   // the lists are complete (and in memory) before anyone reads them back

  const size_t row_bytes = (size_t)D.d * kv_esz(D.dtype);
  const int pieces = (int)(row_bytes / 16);
  const int grp = tid >> 4, gl = tid & 15;
  for (int kk = grp; kk < n_moves; kk += NTH / 16) {
    const size_t dst = phys(scratch[phys(kk)]);
    const size_t src = phys(scratch[phys(C - 1 - kk)]);
    for (int c = gl; c < pieces; c += 16) {
      ((uint4*)(kc + dst * row_bytes))[c] = ((const uint4*)(kc + src * row_bytes))[c];
      ((uint4*)(vc + dst * row_bytes))[c] = ((const uint4*)(vc + src * row_bytes))[c];
    }
    if (gl == 0) {
      metric[dst] = metric[src];
      if (pos) pos[dst] = pos[src];
    }
  }
  __syncthreads();
  const int nb2 = nb - e;
  for (int u = nb2 + tid; u < nb; u += NTH) {
    free_map[row[u]] = 1;
    row[u] = -1;
  }
  if (tid == 0) ctx[g] = T;
}

}  // namespace kvc

using namespace kvc;

extern "C" {

int kvc_evict_rank_select(const kvc_config* cfg, const kvc_state* st, const int32_t* seg_offsets,
                          const int32_t* budget, int nseg, int protect_tail_blocks, int32_t* evict_rows,
                          int32_t* selected, void* ws, void* stream, int flags) {
  int rc = validate(cfg, st);
  if (rc != KVC_OK) return rc;
  if (!budget || !evict_rows || !selected || !ws || ((uintptr_t)ws & 255)) return KVC_ERR_ARG;
  Dims D = dims_of(cfg);
  if (nseg <= 0 || nseg > D.S || protect_tail_blocks < 0) return KVC_ERR_ARG;
  if (!seg_offsets && nseg != D.S) return KVC_ERR_ARG;
  Workspace W = carve(D, ws);
  hipStream_t s = (hipStream_t)stream;
  int32_t* seq_seg = W.held;
  const int n_init = D.G > nseg * 256 ? D.G : nseg * 256;
  hipLaunchKernelGGL(segments_init_kernel, dim3((n_init + 255) / 256), dim3(256), 0, s, D, seg_offsets, nseg, seq_seg,
                     W.seg_hist, W.seg_state, evict_rows, selected, W.header);
  KVC_LAUNCH_CHECK();
  for (int pass = 0; pass < 4; ++pass) {
    // first pass (the exponent byte): nearly every head lands on the same digit of its segment's
    // histogram, and four heads per workgroup (a quarter of the adds) measured fastest
    const int hpw = pass == 0 ? 4 : 1;
    if ((size_t)D.maxb * D.b <= kRankWaveTokens)
      hipLaunchKernelGGL(rank_hist_wave_kernel, dim3((D.G + 4 * hpw - 1) / (4 * hpw)), dim3(256), 0, s, D, pass,
                         protect_tail_blocks, hpw, st->metric,
                         st->block_table, st->ctx_len, seq_seg, W.seg_hist, W.seg_state, W.header);
    else if (D.G <= 1024)
      hipLaunchKernelGGL(rank_hist_kernel<1024>, dim3(D.G), dim3(1024), 0, s, D, pass, protect_tail_blocks, 1,
                         st->metric, st->block_table, st->ctx_len, seq_seg, W.seg_hist, W.seg_state, W.header);
    else
      hipLaunchKernelGGL(rank_hist_kernel<256>, dim3((D.G + hpw - 1) / hpw), dim3(256), 0, s, D, pass,
                         protect_tail_blocks, hpw, st->metric,
                         st->block_table, st->ctx_len, seq_seg, W.seg_hist, W.seg_state, W.header);
    KVC_LAUNCH_CHECK();
    hipLaunchKernelGGL(rank_pick_kernel, dim3(nseg), dim3(256), 0, s, pass, budget, W.seg_hist, W.seg_state,
                       W.header);
    KVC_LAUNCH_CHECK();
    if (pass == 0) {
      hipLaunchKernelGGL(resolve_kernel, dim3(1), dim3(64), 0, s, W.header, 0);
      KVC_LAUNCH_CHECK();
    }
  }
  if ((size_t)D.maxb * D.b <= kRankWaveTokens)
    hipLaunchKernelGGL(rank_tie_wave_kernel, dim3((D.G + 3) / 4), dim3(256), 0, s, D, protect_tail_blocks, st->metric,
                       st->block_table, st->ctx_len, seq_seg, W.seg_state, evict_rows, W.off_b);
  else
    hipLaunchKernelGGL(rank_tie_kernel, dim3(D.G), dim3(256), 0, s, D, protect_tail_blocks, st->metric,
                       st->block_table, st->ctx_len, seq_seg, W.seg_state, evict_rows, W.off_b);
  KVC_LAUNCH_CHECK();
  rc = device_exclusive_scan(RowTieFn{W.off_b}, D.G, W.tile_sums, W.off_a, nullptr, s);
  if (rc != KVC_OK) return rc;
  hipLaunchKernelGGL(rank_grant_kernel, dim3((D.G + 255) / 256), dim3(256), 0, s, D, seq_seg, W.seg_state,
                     W.off_b, W.off_a, evict_rows, selected, W.header);
  KVC_LAUNCH_CHECK();
  return (flags & KVC_ASYNC) ? KVC_OK : finish_sync(W, s);
}

int kvc_compact_rank(const kvc_config* cfg, const kvc_state* st, const int32_t* evict_rows,
                     int64_t* blocks_freed, void* ws, void* stream, int flags) {
  int rc = validate(cfg, st);
  if (rc != KVC_OK) return rc;
  if (!evict_rows || !ws || ((uintptr_t)ws & 255)) return KVC_ERR_ARG;
  if (blocks_freed && ((uintptr_t)blocks_freed & 7)) return KVC_ERR_ARG;
  Dims D = dims_of(cfg);
  Workspace W = carve(D, ws);
  hipStream_t s = (hipStream_t)stream;
  hipLaunchKernelGGL(rank_check_kernel, dim3((D.G + 255) / 256), dim3(256), 0, s, D, st->ctx_len, evict_rows,
                     W.header);
  KVC_LAUNCH_CHECK();
  // the status is settled before anything moves; a caller that wants the count gets it from the
  // same launch (the counts are this call's input, the moves do not change them)
  if (blocks_freed) hipLaunchKernelGGL(publish_freed_kernel, dim3(1), dim3(1024), 0, s, W.header, evict_rows, D.G, blocks_freed, 1);
  else hipLaunchKernelGGL(resolve_kernel, dim3(1), dim3(64), 0, s, W.header, 0);
  KVC_LAUNCH_CHECK();
  if (D.G <= 1024) {
    // few, possibly long heads: a workgroup of 1024 threads per head, the head's metrics kept in
    // LDS (up to 36864 tokens; one such workgroup per CU is all there is to run anyway)
    const size_t head_tokens = (size_t)D.maxb * D.b;
    const int lds_tokens = (int)(head_tokens < 36864 ? head_tokens : 36864);
    static LdsLimit limit;
    const int rc2 = limit.need((size_t)36864 * 4, rank_compact_kernel<1024>);
    if (rc2 != KVC_OK) return rc2;
    hipLaunchKernelGGL(rank_compact_kernel<1024>, dim3(D.G), dim3(1024), (size_t)lds_tokens * 4, s, D, (char*)st->k_cache,
                       (char*)st->v_cache, st->metric, st->pos, st->block_table, st->ctx_len, st->free_map, evict_rows,
                       (int32_t*)W.stash, W.header, lds_tokens);
  } else {
    // many heads: what hides the load latencies is workgroups per CU, and LDS for the metrics would
    // cost more of those than the second reads through the table do (measured: 0.19 -> 0.24 ms)
    // many heads: what hides the load latencies is workgroups per CU.  16 KB of LDS for the metrics
    // of heads of up to 4096 KVs leaves a CU its eight workgroups (0.18 -> 0.16 ms per round of
    // 16 384 heads); 32 KB for up to 8192 costs three of them (0.19 ms).
    // (A wavefront per head of up to 2048 KVs, its metrics in registers and ranks by ballots, took
    // 0.08 ms for the four fifths of the heads it covers, and the workgroups left with the long
    // heads still 0.16: no gain.)
    const size_t head_tokens = (size_t)D.maxb * D.b;
    const int lds_tokens = (int)(head_tokens < 4096 ? head_tokens : 4096);
    hipLaunchKernelGGL(rank_compact_kernel<256>, dim3(D.G), dim3(256), (size_t)lds_tokens * 4, s, D, (char*)st->k_cache,
                       (char*)st->v_cache, st->metric, st->pos, st->block_table, st->ctx_len, st->free_map, evict_rows,
                       (int32_t*)W.stash, W.header, lds_tokens);
  }
  KVC_LAUNCH_CHECK();
  return (flags & KVC_ASYNC) ? KVC_OK : finish_sync(W, s);
}

}  // extern "C"
