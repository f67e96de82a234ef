// Eviction path: block-level metric reduction, lowest-metric block selection
// across layers and heads, and MoveCache compaction with the free step
// (KV-Compress, Method, "Evicting from a Paged KV Cache" and Algorithm 1).
//
// Selection never sorts: per segment an 8-bit-per-pass radix select over the
// f32 keys (non-negative, so their bit patterns order like the values) finds
// the threshold key and how many ties at the threshold are still wanted; ties
// are then granted in ascending (s, l, h, u).  All counting is integer, so the
// result is the one a stable sort by (key, s, l, h, u) would give.
#include "kvc_common.h"
#include <atomic>

namespace kvc {

enum { SS_PREFIX = SEG_PREFIX, SS_REMAIN = SEG_REMAIN, SS_CAND = SEG_CAND, SS_TAKE = SEG_TAKE, SS_FIRSTG = SEG_FIRSTG, SS_ALLTIES = SEG_ALLTIES };

// ---------------------------------------------------------------------------
// block keys
// ---------------------------------------------------------------------------
// One wavefront per head instance; lane -> logical block.  The b metrics of a
// block are contiguous (64 bytes at b = 16) and are added left to right in f32
// (key_mode KVC_KEY_SUM) or reduced to their maximum (KVC_KEY_MAX).
__global__ void __launch_bounds__(256) block_key_kernel(Dims D, int key_mode, const float* __restrict__ metric,
                                                        const int32_t* __restrict__ table,
                                                        const int32_t* __restrict__ ctx,
                                                        float* __restrict__ key) {
  const int g = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (g >= D.G) return;
  const int lane = threadIdx.x & 63;
  const int C = ctx[g];
  const int nb = (C + D.b - 1) / D.b;
  const int32_t* row = table + (size_t)g * D.maxb;
  float* krow = key + (size_t)g * D.maxb;
  for (int u = lane; u < nb; u += 64) {   // cells of blocks the head does not hold are left alone
    float acc = 0.0f;
    {
      const float* m = metric + (size_t)row[u] * D.b;
      const int fill = min(D.b, C - u * D.b);
      if (fill == D.b && (D.b & 3) == 0) {   // a full block: 16-byte loads, the same order of additions
        const bool sum = key_mode == KVC_KEY_SUM;
        acc = sum ? 0.0f : m[0];
        for (int o = 0; o < fill; o += 4) {
          const float4 v = *(const float4*)(m + o);
          if (sum) acc = (((acc + v.x) + v.y) + v.z) + v.w;
          else acc = fmaxf(fmaxf(acc, v.x), fmaxf(v.y, fmaxf(v.z, v.w)));
        }
      } else if (key_mode == KVC_KEY_SUM) {
        for (int o = 0; o < fill; ++o) acc = acc + m[o];
      } else {
        acc = m[0];
        for (int o = 1; o < fill; ++o) acc = fmaxf(acc, m[o]);
      }
    }
    krow[u] = acc;
  }
}

// ---------------------------------------------------------------------------
// selection
// ---------------------------------------------------------------------------

__global__ void __launch_bounds__(256) zero_bytes_kernel(uint8_t* p, size_t n) {
  size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 16;
  if (i + 16 <= n) {
    if (((uintptr_t)(p + i) & 15) == 0) { *(uint4*)(p + i) = make_uint4(0, 0, 0, 0); return; }
  }
  for (size_t k = i; k < n && k < i + 16; ++k) p[k] = 0;
}

__device__ __forceinline__ uint32_t key_bits(float f) {
  uint32_t k = __float_as_uint(f);
  return k == 0x80000000u ? 0u : k;  // -0 orders as +0
}

// Histogram of the current 8-bit digit over the candidates that still match the
// prefix found so far.  A wavefront takes heads_per_wave consecutive head instances (four
// wavefronts per workgroup) and adds their digits to the segment's histogram together; pass 0
// also counts candidates and checks the keys.  In pass 0 (the exponent byte) nearly all keys of
// a segment share one digit, and adds to one global word from all over the chip run one after
// the other: there a wavefront takes several heads, later passes one.
__global__ void __launch_bounds__(256) select_hist_kernel(Dims D, int pass, int protect, int heads_per_wave,
                                                          const float* __restrict__ key,
                                                          const int32_t* __restrict__ ctx,
                                                          const int32_t* __restrict__ seq_seg,
                                                          int32_t* __restrict__ seg_hist,
                                                          int32_t* __restrict__ seg_state,
                                                          int32_t* __restrict__ header) {
  __shared__ int hist[4][256];
  const int wid = threadIdx.x >> 6, lane = threadIdx.x & 63;
  int* my = hist[wid];   // written and read by this wavefront only
  for (int i = lane; i < 256; i += 64) my[i] = 0;
  const int g_first = (blockIdx.x * 4 + wid) * heads_per_wave;
  const int g_end = min(D.G, g_first + heads_per_wave);
  const int shift = 24 - 8 * pass;
  int cur_sg = -1, cand_acc = 0;
  bool bad = false;
  auto flush = [&]() {
    if (cur_sg < 0) return;
    for (int i = lane; i < 256; i += 64) {
      const int c = my[i];
      if (c) { atomicAdd(&seg_hist[cur_sg * 256 + i], c); my[i] = 0; }
    }
    if (pass == 0 && lane == 0 && cand_acc) atomicAdd(&seg_state[cur_sg * 8 + SS_CAND], cand_acc);
    cand_acc = 0;
  };
  for (int g = g_first; g < g_end; ++g) {
    const int sg = seq_seg[g / (D.Lyr * D.Hk)];
    if (sg != cur_sg) { flush(); cur_sg = sg; }
    const int C = ctx[g];
    const int ncand = max(0, (C + D.b - 1) / D.b - protect);
    cand_acc += ncand;
    const uint32_t prefix = (uint32_t)seg_state[sg * 8 + SS_PREFIX];
    const bool live = pass == 0 || seg_state[sg * 8 + SS_TAKE] > 0;
    const float* krow = key + (size_t)g * D.maxb;
    if (live) {
      for (int u = lane; u < ncand; u += 64) {
        const uint32_t k = key_bits(krow[u]);
        if (pass == 0) bad |= k >= 0x7f800000u;
        if (pass == 0 || (k >> (shift + 8)) == prefix) atomicAdd(&my[(k >> shift) & 255], 1);
      }
    }
  }
  flush();
  if (pass == 0 && __any(bad) && lane == 0) atomicOr(&header[HW_SCRATCH0], EB_NUMERIC);
}

// One workgroup per segment: choose the digit that holds the E-th smallest key.
__global__ void __launch_bounds__(256) select_pick_kernel(int pass, const int32_t* __restrict__ budget,
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
    const int take = min(bud, stt[SS_CAND]);
    stt[SS_TAKE] = take;
    stt[SS_REMAIN] = take;
  }
  __syncthreads();
  const int take = stt[SS_TAKE];
  const int remain = stt[SS_REMAIN];
  const int c = seg_hist[sg * 256 + threadIdx.x];
  int tot;
  const int ex = block_exclusive_scan<256>(c, smem, &tot);
  if (threadIdx.x == 0) chosen = -1;
  __syncthreads();
  if (take > 0 && ex < remain && remain <= ex + c) chosen = threadIdx.x;  // exactly one thread
  __syncthreads();
  if (take > 0 && threadIdx.x == chosen) {
    stt[SS_PREFIX] = (int32_t)(((uint32_t)stt[SS_PREFIX] << 8) | (uint32_t)chosen);
    stt[SS_REMAIN] = remain - ex;  // still wanted among keys equal on all digits so far
  }
  seg_hist[sg * 256 + threadIdx.x] = 0;
}

// Ties at the threshold key, per head instance.
__global__ void __launch_bounds__(256) select_tie_count_kernel(Dims D, int protect,
                                                               const float* __restrict__ key,
                                                               const int32_t* __restrict__ ctx,
                                                               const int32_t* __restrict__ seq_seg,
                                                               const int32_t* __restrict__ seg_state,
                                                               int32_t* __restrict__ tie_cnt) {
  const int g = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (g >= D.G) return;
  const int lane = threadIdx.x & 63;
  const int sg = seq_seg[g / (D.Lyr * D.Hk)];
  int n = 0;
  if (seg_state[sg * 8 + SS_TAKE] > 0) {
    const uint32_t thr = (uint32_t)seg_state[sg * 8 + SS_PREFIX];
    const int ncand = max(0, (ctx[g] + D.b - 1) / D.b - protect);
    const float* krow = key + (size_t)g * D.maxb;
    for (int u = lane; u < ncand; u += 64) n += key_bits(krow[u]) == thr;
  }
  n = wave_sum_i(n);
  if (lane == 0) tie_cnt[g] = n;
}

struct TieFn {
  const int32_t* cnt;
  __device__ int operator()(int i) const { return cnt[i]; }
};

__global__ void __launch_bounds__(256) select_mark_kernel(Dims D, int protect, const float* __restrict__ key,
                                                          const int32_t* __restrict__ ctx,
                                                          const int32_t* __restrict__ seq_seg,
                                                          const int32_t* __restrict__ seg_state,
                                                          const int32_t* __restrict__ tie_off,
                                                          uint8_t* __restrict__ flag,
                                                          int32_t* __restrict__ evict_count,
                                                          int32_t* __restrict__ selected,
                                                          const int32_t* __restrict__ header) {
  if (header[HW_STATUS] != KVC_OK) return;
  const int g = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (g >= D.G) return;
  const int lane = threadIdx.x & 63;
  const int sg = seq_seg ? seq_seg[g / (D.Lyr * D.Hk)] : g / (D.Lyr * D.Hk);   // no map: one segment per sequence
  const int32_t* stt = seg_state + sg * 8;
  const int take = stt[SS_TAKE];
  if (g == stt[SS_FIRSTG] && lane == 0) selected[sg] = take;
  if (take <= 0) return;
  const uint32_t thr = (uint32_t)stt[SS_PREFIX];
  // ties granted to this head: those whose rank inside the segment is below SS_REMAIN (a segment
  // that takes every key at its threshold has no ranks to look up)
  const bool all_ties = stt[SS_ALLTIES] != 0;
  int ties_before = all_ties ? 0 : tie_off[g] - tie_off[stt[SS_FIRSTG]];
  const int want = all_ties ? 0x7fffffff : stt[SS_REMAIN];
  const int ncand = max(0, (ctx[g] + D.b - 1) / D.b - protect);
  const float* krow = key + (size_t)g * D.maxb;
  uint8_t* frow = flag + (size_t)g * D.maxb;
  int cnt = 0;
  for (int base = 0; base < ncand; base += 64) {
    const int u = base + lane;
    uint32_t k = 0xffffffffu;
    if (u < ncand) k = key_bits(krow[u]);
    const bool tie = k == thr;
    const unsigned long long tm = __ballot(tie);
    const int my_rank = ties_before + __popcll(tm & ((1ull << lane) - 1ull));
    const bool ev = (u < ncand) && (k < thr || (tie && my_rank < want));
    if (ev) frow[u] = 1;
    cnt += __popcll(__ballot(ev));
    ties_before += __popcll(tm);
  }
  if (lane == 0) evict_count[g] = cnt;
}

// The whole selection of one segment in one workgroup, for segments that are single sequences
// (the case of every decode-time round): instead of four histogram launches over all heads with a
// pick launch after each, a tie count, a scan and the marking, the segment's workgroup walks its
// own candidates -- head instances (s, *, *), blocks 0 .. nb - protect - 1 of each, numbered
// j = 0, 1, ... in (g, u) order -- four times, the last three over a copy of the keys in LDS when
// they fit (lds_keys words; else over the keys again), and leaves threshold, ties wanted and, only
// when some but not all keys at the threshold are taken, every head's count of such keys in front
// of it.  It also clears its share of the outputs; the marking launch fills them once the status
// is settled.  heads_lds: per-head first candidate numbers, kept in LDS (Lyr Hk + 1 words).
constexpr int kSegThreads = 1024;
constexpr int kSegWaves = kSegThreads / 64;
constexpr int kSegMaxHeads = 4096;     // head instances of a sequence whose first candidate numbers fit the LDS
constexpr int kSegLdsKeys = 28672;     // keys of a segment kept in LDS between the passes (112 KB)

__global__ void __launch_bounds__(kSegThreads) select_segment_kernel(Dims D, int protect, int lds_keys,
                                                                      const float* __restrict__ key,
                                                                      const int32_t* __restrict__ ctx,
                                                                      const int32_t* __restrict__ budget,
                                                                      uint8_t* __restrict__ flag,
                                                                      int32_t* __restrict__ evict_count,
                                                                      int32_t* __restrict__ selected,
                                                                      int32_t* __restrict__ seg_state,
                                                                      int32_t* __restrict__ tie_before,
                                                                      int32_t* __restrict__ header) {
  extern __shared__ __align__(16) uint32_t seg_smem[];
  const int nh = D.Lyr * D.Hk;
  int* s_base = (int*)seg_smem;                        // [nh + 1]
  int* s_whist = s_base + ((nh + 1 + 3) & ~3);         // [waves][256]
  uint32_t* s_key = (uint32_t*)(s_whist + kSegWaves * 256);   // [lds_keys]
  __shared__ int smem[kSegThreads / 64 + 1];
  __shared__ int hist[256];
  __shared__ int carry_s, chosen_s, prefix_s, remain_s, clast_s, bad_s;
  const int sg = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
  const int g0 = sg * nh;

  // this workgroup's share of the outputs starts from zero
  {
    const size_t nflag = (size_t)D.G * D.maxb;
    const size_t per = ((nflag + gridDim.x - 1) / gridDim.x + 15) & ~(size_t)15;
    const size_t lo = (size_t)sg * per, hi = lo + per < nflag ? lo + per : nflag;
    if (lo < hi) {
      size_t i = lo + (size_t)tid * 16;
      const bool wide = ((uintptr_t)flag & 15) == 0;
      for (; i < hi; i += (size_t)kSegThreads * 16) {
        if (wide && i + 16 <= hi) *(uint4*)(flag + i) = make_uint4(0, 0, 0, 0);
        else for (size_t k = i; k < hi && k < i + 16; ++k) flag[k] = 0;
      }
    }
    for (int i = g0 + tid; i < g0 + nh; i += kSegThreads) evict_count[i] = 0;
    if (tid == 0) selected[sg] = 0;
  }

  // candidates per head and their first numbers
  if (tid == 0) { carry_s = 0; bad_s = 0; }
  __syncthreads();
  for (int h0 = 0; h0 < nh; h0 += kSegThreads) {
    const int h = h0 + tid;
    const int n = h < nh ? max(0, (ctx[g0 + h] + D.b - 1) / D.b - protect) : 0;
    int tot;
    const int ex = block_exclusive_scan<kSegThreads>(n, smem, &tot);
    const int carry = carry_s;
    if (h < nh) s_base[h] = carry + ex;
    __syncthreads();
    if (tid == 0) carry_s = carry + tot;
    __syncthreads();
  }
  const int K = carry_s;
  if (tid == 0) s_base[nh] = K;
  int bud = budget[sg];
  if (bud < 0) { if (tid == 0) atomicOr(&header[HW_SCRATCH0], EB_ARG); bud = 0; }
  const int take = min(bud, K);
  if (tid == 0) { prefix_s = 0; remain_s = take; clast_s = 0; }
  __syncthreads();
  const bool kept = K <= lds_keys;
  // key number j -> (head, block): the last head whose first number is <= j.  The searches of the
  // UQ keys a thread asks for at a time run side by side, a fixed number of halvings each, so that
  // their LDS reads overlap.
  constexpr int UQ = 8;
  int halvings = 0;
  while ((1 << halvings) < nh) ++halvings;
  auto keys_from_memory = [&](int jfirst, uint32_t (&out)[UQ]) {
    int lo[UQ], hi[UQ];
#pragma unroll
    for (int q = 0; q < UQ; ++q) { lo[q] = 0; hi[q] = nh; }
    for (int step = 0; step < halvings; ++step) {
#pragma unroll
      for (int q = 0; q < UQ; ++q) {
        const int mid = (lo[q] + hi[q]) >> 1;      // == lo once hi - lo <= 1: then nothing moves
        const bool le = s_base[mid] <= jfirst + q * kSegThreads;
        lo[q] = le ? mid : lo[q];
        hi[q] = le ? hi[q] : mid;
      }
    }
#pragma unroll
    for (int q = 0; q < UQ; ++q) {
      const int j = jfirst + q * kSegThreads;
      out[q] = j < K ? key_bits(key[(size_t)(g0 + lo[q]) * D.maxb + (j - s_base[lo[q]])]) : 0u;
    }
  };

  for (int pass = 0; pass < 4; ++pass) {
    if (pass > 0 && take == 0) break;   // (the first pass also checks the keys, so it always runs)
    for (int i = tid; i < kSegWaves * 256; i += kSegThreads) s_whist[i] = 0;
    __syncthreads();
    const int shift = 24 - 8 * pass;
    const uint32_t prefix = (uint32_t)prefix_s;
    int* my = s_whist + wid * 256;
    bool bad = false;
    for (int j0 = 0; j0 < K; j0 += UQ * kSegThreads) {
      uint32_t kq[UQ];   // eight keys asked for before the first is used
      if (pass == 0 || !kept) {
        keys_from_memory(j0 + tid, kq);
      } else {
#pragma unroll
        for (int q = 0; q < UQ; ++q) {
          const int j = j0 + q * kSegThreads + tid;
          kq[q] = j < K ? s_key[j] : 0u;
        }
      }
#pragma unroll
      for (int q = 0; q < UQ; ++q) {
        const int j = j0 + q * kSegThreads + tid;
        const bool in = j < K;
        const uint32_t k = kq[q];
        if (pass == 0) {
          bad |= in && k >= 0x7f800000u;
          if (in && kept) s_key[j] = k;
        }
        const bool counts = in && (pass == 0 || (k >> (shift + 8)) == prefix);
        const int digit = (int)((k >> shift) & 255u);
        // nearly all keys of a segment share their exponent byte: a wavefront whose lanes agree adds once
        const unsigned long long m = __ballot(counts);
        if (m) {
          const int first = __builtin_amdgcn_readlane(digit, __builtin_ctzll(m));
          if (__ballot(counts && digit != first) == 0ull) {
            if (lane == 0) my[first] += __popcll(m);
          } else if (counts) {
            atomicAdd(&my[digit], 1);
          }
        }
      }
    }
    if (pass == 0 && __any(bad) && lane == 0) bad_s = 1;
    __syncthreads();
    if (tid < 256) {
      int c = 0;
#pragma unroll
      for (int w2 = 0; w2 < kSegWaves; ++w2) c += s_whist[w2 * 256 + tid];
      hist[tid] = c;
    }
    __syncthreads();
    const int c = tid < 256 ? hist[tid] : 0;
    const int ex = block_exclusive_scan<kSegThreads>(c, smem, nullptr);
    const int remain = remain_s;
    if (tid == 0) chosen_s = -1;
    __syncthreads();
    if (take > 0 && tid < 256 && ex < remain && remain <= ex + c) chosen_s = tid;   // exactly one thread
    __syncthreads();
    if (take > 0 && tid == chosen_s) {
      prefix_s = (int)((prefix << 8) | (uint32_t)tid);
      remain_s = remain - ex;    // still wanted among keys equal on all digits so far
      clast_s = c;               // keys equal on all digits so far
    }
    __syncthreads();
  }
  if (tid == 0 && bad_s) atomicOr(&header[HW_SCRATCH0], EB_NUMERIC);
  const uint32_t thr = (uint32_t)prefix_s;
  const int want = remain_s;
  const bool all_ties = take == 0 || want == clast_s;
  if (tid == 0) {
    int32_t* stt = seg_state + sg * 8;
    stt[SS_PREFIX] = (int32_t)thr;
    stt[SS_REMAIN] = want;
    stt[SS_CAND] = K;
    stt[SS_TAKE] = take;
    stt[SS_FIRSTG] = g0;
    stt[SS_ALLTIES] = all_ties ? 1 : 0;
    stt[6] = stt[7] = 0;
  }
  if (all_ties) return;
  // some of the keys at the threshold stay: the first `want` in (g, u) order go.  Every head
  // with candidates learns how many such keys lie in front of its first one.
  if (tid == 0) carry_s = 0;
  __syncthreads();
  for (int j0 = 0; j0 < K; j0 += kSegThreads) {
    const int j = j0 + tid;
    uint32_t k = 0xffffffffu;
    int h = 0;
    if (j < K) {
      int lo = 0, hi = nh;
      while (hi - lo > 1) { const int mid = (lo + hi) >> 1; if (s_base[mid] <= j) lo = mid; else hi = mid; }
      h = lo;
      k = kept ? s_key[j] : key_bits(key[(size_t)(g0 + lo) * D.maxb + (j - s_base[lo])]);
    }
    const int is_tie = (j < K) && k == thr;
    int tot;
    const int rank = block_exclusive_scan<kSegThreads>(is_tie, smem, &tot) + carry_s;
    if (j < K && j == s_base[h]) tie_before[g0 + h] = rank;
    if (j0 == 0 && tid == 0 && s_base[1] == 0) tie_before[g0] = 0;   // (the marking launch subtracts the first head's count)
    __syncthreads();
    if (tid == 0) carry_s += tot;
    __syncthreads();
  }
}

// ---------------------------------------------------------------------------
// compaction
// ---------------------------------------------------------------------------

// Per head: inclusive prefix count of flagged blocks; checks flags against the
// head's block count and against evict_count.
__global__ void __launch_bounds__(256) compact_scan_kernel(Dims D, const uint8_t* __restrict__ flag,
                                                           const int32_t* __restrict__ evict_count,
                                                           const int32_t* __restrict__ ctx,
                                                           int32_t* __restrict__ flag_scan,
                                                           int32_t* __restrict__ header) {
  const int g = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (g >= D.G) return;
  const int lane = threadIdx.x & 63;
  const int nb = (ctx[g] + D.b - 1) / D.b;
  const uint8_t* frow = flag + (size_t)g * D.maxb;
  int32_t* srow = flag_scan + (size_t)g * D.maxb;
  int run = 0;
  bool bad = false;
  for (int base = 0; base < nb; base += 64) {
    const int u = base + lane;
    const bool f = (u < nb) && frow[u] != 0;
    const unsigned long long m = __ballot(f);
    const int inc = run + __popcll(m & ((2ull << lane) - 1ull));
    if (u < nb) srow[u] = inc;
    run += __popcll(m);
  }
  // no flag may be set past the blocks the head holds: that stretch (most of the row when heads
  // are compressed far below the length the table is sized for) is only looked at, 16 bytes a
  // lane where the row is aligned, bytes at its two ends
  {
    const uint8_t* p = frow + nb;
    const uint8_t* end = frow + D.maxb;
    const uint8_t* body = (const uint8_t*)(((uintptr_t)p + 15) & ~(uintptr_t)15);
    if (body > end) body = end;
    const uint8_t* body_end = body + ((end - body) & ~(ptrdiff_t)15);
    for (const uint8_t* q = p + lane; q < body; q += 64) bad |= *q != 0;
    for (const uint8_t* q = body + (size_t)lane * 16; q < body_end; q += 1024) {
      const uint4 v = *(const uint4*)q;
      bad |= (v.x | v.y | v.z | v.w) != 0;
    }
    for (const uint8_t* q = body_end + lane; q < end; q += 64) bad |= *q != 0;
  }
  bad |= run != evict_count[g];
  if (__any(bad) && lane == 0) atomicOr(&header[HW_SCRATCH0], EB_ARG);
}

// One workgroup per head instance.  A 16-lane group moves one KV: its key row, value row, metric
// and logical index.  Sources lie in [T, C), destinations in [0, T), so moves of one head never
// overlap; heads own disjoint blocks.
// STAGED: the head's prefix counts of flags and its block ids are copied into LDS first (one
// round of loads), so that a mover's walk - its block's flag, the flags before it, a binary
// search for its hole - no longer is a chain of a dozen dependent global loads.
template <bool STAGED>
__global__ void __launch_bounds__(256) compact_move_kernel(Dims D, char* __restrict__ kc,
                                                           char* __restrict__ vc,
                                                           float* __restrict__ metric,
                                                           int32_t* __restrict__ pos,
                                                           int32_t* __restrict__ table,
                                                           int32_t* __restrict__ ctx,
                                                           uint8_t* __restrict__ free_map,
                                                           const int32_t* __restrict__ evict_count,
                                                           const int32_t* __restrict__ flag_scan,
                                                           int32_t* __restrict__ header) {
  if (header[HW_STATUS] != KVC_OK) return;
  const int g = blockIdx.x;
  const int e = evict_count[g];
  if (e <= 0) return;
  const int b = D.b;
  int lb = 0;
  while ((1 << lb) < b) ++lb;   // block sizes are powers of two
  const int C = ctx[g];
  const int nb = (C + b - 1) >> lb;
  int32_t* row = table + (size_t)g * D.maxb;
  extern __shared__ int32_t s_stage[];   // STAGED: [nb] inclusive prefix of flags, [nb] block ids
  const int32_t* pi = flag_scan + (size_t)g * D.maxb;  // inclusive prefix of flags: block u is flagged when it steps there
  const int32_t* ids = row;
  if constexpr (STAGED) {
    for (int u = threadIdx.x; u < nb; u += 256) {
      s_stage[u] = pi[u];
      s_stage[D.maxb + u] = row[u];
    }
    __syncthreads();
    pi = s_stage;
    ids = s_stage + D.maxb;
  }
  const int last_flag = pi[nb - 1] - (nb > 1 ? pi[nb - 2] : 0);
  // evicted real KVs: flagged blocks are full except possibly the last one
  const int n_ev = e * b - (last_flag ? nb * b - C : 0);
  const int T = C - n_ev;
  const size_t row_bytes = (size_t)D.d * kv_esz(D.dtype);
  const int pieces = (int)(row_bytes / 16);
  const int grp = threadIdx.x >> 4, gl = threadIdx.x & 15;
  for (int j = T + grp; j < C; j += 16) {
    const int uj = j >> lb;
    const int before = uj ? pi[uj - 1] : 0;
    if (pi[uj] != before) continue;  // its block is flagged: evicted, nothing to keep
    // evicted real slots in [0, j+1): whole flagged blocks before block uj (uj itself is kept)
    const int ev_below = before << lb;
    const int k = (C - 1 - j) - (n_ev - ev_below);  // kept slots above j = rank among movers
    // k-th hole: offset k % b of the (k / b)-th flagged block
    const int want = (k >> lb) + 1;
    int lo = 0, hi = nb - 1;  // smallest u with pi[u] >= want
    while (lo < hi) { int mid = (lo + hi) >> 1; if (pi[mid] >= want) hi = mid; else lo = mid + 1; }
    const size_t src = ((size_t)ids[uj] << lb) + (j & (b - 1));
    const size_t dst = ((size_t)ids[lo] << lb) + (k & (b - 1));
    for (int c = gl; c < pieces; c += 16) {
      ((uint4*)(kc + dst * row_bytes))[c] = ((const uint4*)(kc + src * row_bytes))[c];
      ((uint4*)(vc + dst * row_bytes))[c] = ((const uint4*)(vc + src * row_bytes))[c];
    }
    if (gl == 0) {
      metric[dst] = metric[src];
      if (pos) pos[dst] = pos[src];
    }
  }
  __syncthreads();  // all moves of this head read the table before it shrinks
  const int nb2 = (T + b - 1) >> lb;
  for (int u = nb2 + threadIdx.x; u < nb; u += 256) {
    free_map[ids[u]] = 1;
    row[u] = -1;
  }
  if (threadIdx.x == 0) ctx[g] = T;   // nb - nb2 = e blocks went back
}

// Tables sized for long prompts: workgroup (g, y) moves the kept KVs of logical slots
// T + y * kSlice .. + kSlice - 1 of head g, and the tables are left to compact_free_kernel.
// (One workgroup per head with the head's whole table in LDS: a 131072-token head that loses a
// tenth of its blocks is 12 MB of moves behind one workgroup, two such workgroups fit a CU, and
// a round of a million blocks took 7.4 ms.)  The movers of a slice are consecutive in rank, so
// their holes are consecutive flagged blocks: the workgroup finds the first of them with a
// 256-way search over the prefix counts, walks on from there gathering block ids, and keeps only
// its own stretch of the table in LDS (a few KB).
constexpr int kSlice = 2048;
__global__ void __launch_bounds__(256) compact_move_sliced_kernel(Dims D, char* __restrict__ kc, char* __restrict__ vc,
                                                                  float* __restrict__ metric, int32_t* __restrict__ pos,
                                                                  const int32_t* __restrict__ table,
                                                                  const int32_t* __restrict__ ctx,
                                                                  const int32_t* __restrict__ evict_count,
                                                                  const int32_t* __restrict__ flag_scan,
                                                                  const int32_t* __restrict__ header) {
  if (header[HW_STATUS] != KVC_OK) return;
  const int g = blockIdx.x;
  const int e = evict_count[g];
  if (e <= 0) return;
  const int b = D.b;
  if ((long long)blockIdx.y * kSlice >= (long long)e * b) return;   // the range of movers is at most e * b slots long
  int lb = 0;
  while ((1 << lb) < b) ++lb;   // block sizes are powers of two
  const int C = ctx[g];
  const int nb = (C + b - 1) >> lb;
  const int32_t* row = table + (size_t)g * D.maxb;
  const int32_t* pi = flag_scan + (size_t)g * D.maxb;  // inclusive prefix of flags
  const int last_flag = pi[nb - 1] - (nb > 1 ? pi[nb - 2] : 0);
  const int n_ev = e * b - (last_flag ? nb * b - C : 0);
  const int T = C - n_ev;
  const int j_lo = T + (int)blockIdx.y * kSlice;
  if (j_lo >= C) return;
  const int j_hi = min(C, j_lo + kSlice);
  const int tid = threadIdx.x;
  constexpr int kMaxBlk = kSlice + 2;                 // blocks of a slice at b = 1, and one before
  __shared__ int s_pi[kMaxBlk], s_id[kMaxBlk], s_hole[kMaxBlk];
  __shared__ int s_first;
  // this slice's stretch of the table: blocks ub0 .. ub1 and the prefix count before ub0
  const int ub0 = j_lo >> lb, ub1 = (j_hi - 1) >> lb;
  for (int i = tid; i <= ub1 - ub0 + 1; i += 256) {
    const int u = ub0 - 1 + i;                        // s_pi[i] = pi[ub0 - 1 + i], 0 before the row
    s_pi[i] = u >= 0 ? pi[u] : 0;
    if (i > 0) s_id[i] = row[u];
  }
  __syncthreads();
  // kept slots above j (= rank of mover j when j itself is kept), for any slot j of the slice
  auto kept_above = [&](int j) {
    const int uj = j >> lb;
    const int before = s_pi[uj - ub0], here = s_pi[uj - ub0 + 1];
    const int ev_upto = (before << lb) + (here != before ? (j & (b - 1)) + 1 : 0);   // evicted slots in [0, j]
    return (C - 1 - j) - (n_ev - ev_upto);
  };
  const int r_lo = kept_above(j_hi - 1) >> lb, r_hi = kept_above(j_lo) >> lb;   // flagged blocks (by rank) that hold the holes
  // first block u with pi[u] >= r_lo + 1: a 256-way search, twice
  {
    const int want = r_lo + 1;
    int lo = 0, hi = nb - 1;      // the answer lies in [lo, hi]: pi[nb - 1] = e > r_hi >= r_lo
    while (hi - lo >= 256) {
      const int step = (hi - lo + 256) / 256;
      if (tid == 0) s_first = 256;
      __syncthreads();
      const int u = min(hi, lo + tid * step);
      if (pi[u] >= want) atomicMin(&s_first, tid);
      __syncthreads();
      const int t = s_first;      // < 256: the probe at hi always succeeds
      const int nhi = min(hi, lo + t * step), nlo = t == 0 ? lo : min(hi, lo + (t - 1) * step) + 1;
      __syncthreads();
      lo = nlo; hi = nhi;
    }
    if (tid == 0) s_first = hi;
    __syncthreads();
    if (lo + tid <= hi && pi[lo + tid] >= want) atomicMin(&s_first, lo + tid);
    __syncthreads();
  }
  // walk on from there: the flagged blocks of ranks r_lo .. r_hi, their ids into s_hole
  for (int base = s_first; base < nb; base += 256) {
    const int u = base + tid;
    int here = 0, before = 0;
    if (u < nb) { here = pi[u]; before = u ? pi[u - 1] : 0; }
    if (u < nb && here != before && here - 1 >= r_lo && here - 1 <= r_hi) s_hole[here - 1 - r_lo] = row[u];
    const int last = pi[min(nb - 1, base + 255)];
    if (last > r_hi) break;       // the same for every thread
  }
  __syncthreads();
  const size_t row_bytes = (size_t)D.d * kv_esz(D.dtype);
  const int pieces = (int)(row_bytes / 16);
  const int grp = tid >> 4, gl = tid & 15;
  auto route = [&](int j, size_t& src, size_t& dst) {
    if (j >= j_hi) return false;
    const int uj = j >> lb;
    if (s_pi[uj - ub0 + 1] != s_pi[uj - ub0]) return false;   // its block is flagged: evicted, nothing to keep
    const int k = kept_above(j);                               // rank among the movers, from the top
    src = ((size_t)s_id[uj - ub0 + 1] << lb) + (j & (b - 1));
    dst = ((size_t)s_hole[(k >> lb) - r_lo] << lb) + (k & (b - 1));   // k-th hole: offset k % b of the (k / b)-th flagged block
    return true;
  };
  for (int j = j_lo + grp; j < j_hi; j += 16) {
    size_t src = 0, dst = 0;
    if (!route(j, src, dst)) continue;
    for (int c = gl; c < pieces; c += 16) {
      ((uint4*)(kc + dst * row_bytes))[c] = ((const uint4*)(kc + src * row_bytes))[c];
      ((uint4*)(vc + dst * row_bytes))[c] = ((const uint4*)(vc + src * row_bytes))[c];
    }
    if (gl == 0) {
      metric[dst] = metric[src];
      if (pos) pos[dst] = pos[src];
    }
  }
}

// The free step after a sliced move: one wavefront per head instance gives the tail blocks back
// and shortens the head.
__global__ void __launch_bounds__(256) compact_free_kernel(Dims D, int32_t* __restrict__ table,
                                                           int32_t* __restrict__ ctx,
                                                           uint8_t* __restrict__ free_map,
                                                           const int32_t* __restrict__ evict_count,
                                                           const int32_t* __restrict__ flag_scan,
                                                           const int32_t* __restrict__ header) {
  if (header[HW_STATUS] != KVC_OK) return;
  const int g = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (g >= D.G) return;
  const int lane = threadIdx.x & 63;
  const int e = evict_count[g];
  if (e <= 0) return;
  const int b = D.b;
  const int C = ctx[g];
  const int nb = (C + b - 1) / b;
  const int32_t* pi = flag_scan + (size_t)g * D.maxb;
  const int last_flag = pi[nb - 1] - (nb > 1 ? pi[nb - 2] : 0);
  const int n_ev = e * b - (last_flag ? nb * b - C : 0);
  const int T = C - n_ev;
  int32_t* row = table + (size_t)g * D.maxb;
  const int nb2 = (T + b - 1) / b;
  for (int u = nb2 + lane; u < nb; u += 64) {
    free_map[row[u]] = 1;
    row[u] = -1;
  }
  if (lane == 0) ctx[g] = T;
}

}  // namespace kvc

using namespace kvc;

extern "C" {

int kvc_metric_reduce(const kvc_config* cfg, const kvc_state* st, float* block_key, int key_mode,
                      void* ws, void* stream) {
  int rc = validate(cfg, st);
  if (rc != KVC_OK) return rc;
  if (!block_key || ((uintptr_t)block_key & 3)) return KVC_ERR_ARG;
  if (key_mode != KVC_KEY_SUM && key_mode != KVC_KEY_MAX) return KVC_ERR_ARG;
  (void)ws;
  Dims D = dims_of(cfg);
  hipLaunchKernelGGL(block_key_kernel, dim3((D.G + 3) / 4), dim3(256), 0, (hipStream_t)stream, D, key_mode,
                     st->metric, st->block_table, st->ctx_len, block_key);
  KVC_LAUNCH_CHECK();
  return KVC_OK;
}

int kvc_evict_select(const kvc_config* cfg, const kvc_state* st, const float* block_key,
                     const int32_t* seg_offsets, const int32_t* budget, int nseg,
                     int protect_tail_blocks, uint8_t* evict_flag, int32_t* evict_count,
                     int32_t* selected, void* ws, void* stream, int flags) {
  int rc = validate(cfg, st);
  if (rc != KVC_OK) return rc;
  if (!block_key || !budget || !evict_flag || !evict_count || !selected || !ws ||
      ((uintptr_t)ws & 255))
    return KVC_ERR_ARG;
  Dims D = dims_of(cfg);
  if (nseg <= 0 || nseg > D.S || protect_tail_blocks < 0) return KVC_ERR_ARG;
  if (!seg_offsets && nseg != D.S) return KVC_ERR_ARG;
  Workspace W = carve(D, ws);
  hipStream_t s = (hipStream_t)stream;
  int32_t* seq_seg = W.held;  // [S] fits in the [G] array
  const int gw = (D.G + 3) / 4;
  // One segment per sequence, and a pool that gives the average sequence no more blocks than a
  // workgroup keeps on chip: every segment's selection in its own workgroup, three launches in
  // all.  (A sequence with more candidates than that is still served, its keys re-read in every
  // pass; with sequences of 650 000 blocks each that took 3.2 ms against 0.5 for the launches
  // over all heads below, which is why the pool size decides.)
  const int heads_per_seq = D.Lyr * D.Hk;
  if (!seg_offsets && heads_per_seq <= kSegMaxHeads && (size_t)D.N <= (size_t)kSegLdsKeys * D.S) {
    const size_t lds = ((size_t)((heads_per_seq + 1 + 3) & ~3) + kSegWaves * 256 + kSegLdsKeys) * 4;
    static LdsLimit limit;
    rc = limit.need(((size_t)kSegMaxHeads + 4 + kSegWaves * 256 + kSegLdsKeys) * 4, select_segment_kernel);
    if (rc != KVC_OK) return rc;
    hipLaunchKernelGGL(select_segment_kernel, dim3(D.S), dim3(kSegThreads), lds, s, D, protect_tail_blocks, kSegLdsKeys,
                       block_key, st->ctx_len, budget, evict_flag, evict_count, selected, W.seg_state, W.off_a, W.header);
    KVC_LAUNCH_CHECK();
    hipLaunchKernelGGL(resolve_kernel, dim3(1), dim3(64), 0, s, W.header, 0);
    KVC_LAUNCH_CHECK();
    hipLaunchKernelGGL(select_mark_kernel, dim3(gw), dim3(256), 0, s, D, protect_tail_blocks, block_key,
                       st->ctx_len, (const int32_t*)nullptr, W.seg_state, W.off_a, evict_flag, evict_count, selected,
                       W.header);
    KVC_LAUNCH_CHECK();
    return (flags & KVC_ASYNC) ? KVC_OK : finish_sync(W, s);
  }
  int n_init = D.G > nseg * 256 ? D.G : nseg * 256;
  hipLaunchKernelGGL(segments_init_kernel, dim3((n_init + 255) / 256), dim3(256), 0, s, D, seg_offsets, nseg,
                     seq_seg, W.seg_hist, W.seg_state, evict_count, selected, W.header);
  KVC_LAUNCH_CHECK();
  const size_t nflag = (size_t)D.G * D.maxb;
  hipLaunchKernelGGL(zero_bytes_kernel, dim3((unsigned)((nflag / 16 + 256) / 256)), dim3(256), 0, s,
                     evict_flag, nflag);
  KVC_LAUNCH_CHECK();
  for (int pass = 0; pass < 4; ++pass) {
    const int hpw = pass == 0 ? 8 : 1;
    hipLaunchKernelGGL(select_hist_kernel, dim3((D.G + 4 * hpw - 1) / (4 * hpw)), dim3(256), 0, s, D, pass,
                       protect_tail_blocks, hpw, block_key, st->ctx_len, seq_seg, W.seg_hist, W.seg_state, W.header);
    KVC_LAUNCH_CHECK();
    hipLaunchKernelGGL(select_pick_kernel, dim3(nseg), dim3(256), 0, s, pass, budget, W.seg_hist,
                       W.seg_state, W.header);
    KVC_LAUNCH_CHECK();
    if (pass == 0) {  // keys checked, budgets checked: settle the status before any output is written
      hipLaunchKernelGGL(resolve_kernel, dim3(1), dim3(64), 0, s, W.header, 0);
      KVC_LAUNCH_CHECK();
    }
  }
  hipLaunchKernelGGL(select_tie_count_kernel, dim3(gw), dim3(256), 0, s, D, protect_tail_blocks, block_key,
                     st->ctx_len, seq_seg, W.seg_state, W.off_b);
  KVC_LAUNCH_CHECK();
  rc = device_exclusive_scan(TieFn{W.off_b}, D.G, W.tile_sums, W.off_a, nullptr, s);
  if (rc != KVC_OK) return rc;
  hipLaunchKernelGGL(select_mark_kernel, dim3(gw), dim3(256), 0, s, D, protect_tail_blocks, block_key,
                     st->ctx_len, seq_seg, W.seg_state, W.off_a, evict_flag, evict_count, selected,
                     W.header);
  KVC_LAUNCH_CHECK();
  return (flags & KVC_ASYNC) ? KVC_OK : finish_sync(W, s);
}

int kvc_compact(const kvc_config* cfg, const kvc_state* st, const uint8_t* evict_flag,
                const int32_t* evict_count, int64_t* blocks_freed, void* ws, void* stream, int flags) {
  int rc = validate(cfg, st);
  if (rc != KVC_OK) return rc;
  if (!evict_flag || !evict_count || !ws || ((uintptr_t)ws & 255)) return KVC_ERR_ARG;
  if (blocks_freed && ((uintptr_t)blocks_freed & 7)) return KVC_ERR_ARG;
  Dims D = dims_of(cfg);
  Workspace W = carve(D, ws);
  hipStream_t s = (hipStream_t)stream;
  hipLaunchKernelGGL(compact_scan_kernel, dim3((D.G + 3) / 4), dim3(256), 0, s, D, evict_flag, evict_count,
                     st->ctx_len, W.flag_scan, W.header);
  KVC_LAUNCH_CHECK();
  // the status is settled before anything moves; a caller that wants the count gets it from the
  // same launch (the counts are this call's input, the moves do not change them)
  if (blocks_freed) hipLaunchKernelGGL(publish_freed_kernel, dim3(1), dim3(1024), 0, s, W.header, evict_count, D.G, blocks_freed, 1);
  else hipLaunchKernelGGL(resolve_kernel, dim3(1), dim3(64), 0, s, W.header, 0);
  KVC_LAUNCH_CHECK();
  const size_t stage_bytes = (size_t)D.maxb * 8;   // prefix counts and block ids of one head
  char* kcp = (char*)st->k_cache;
  char* vcp = (char*)st->v_cache;
  // Tables sized for long prompts (more than 65536 tokens a head, where a head's table no longer
  // fits the LDS several times over): a head's movers are spread over workgroups of kSlice logical
  // slots each, and the tables change in a launch of their own.  (Below that the empty workgroups
  // of the slice grid cost more than the slices gain: 65536 heads with tables for 32768 tokens,
  // 0.70 ms per head-sized workgroup against 1.36 ms sliced.)
  const size_t row_tokens = (size_t)D.maxb * D.b;
  const size_t slices = (row_tokens + kSlice - 1) / kSlice;
  if (row_tokens > 65536 && slices <= 65535) {
    hipLaunchKernelGGL(compact_move_sliced_kernel, dim3(D.G, (unsigned)slices), dim3(256), 0, s, D, kcp, vcp, st->metric,
                       st->pos, st->block_table, st->ctx_len, evict_count, W.flag_scan, W.header);
    KVC_LAUNCH_CHECK();
    hipLaunchKernelGGL(compact_free_kernel, dim3((D.G + 3) / 4), dim3(256), 0, s, D, st->block_table, st->ctx_len,
                       st->free_map, evict_count, W.flag_scan, W.header);
  } else if (stage_bytes <= 64 * 1024) {
    hipLaunchKernelGGL(compact_move_kernel<true>, dim3(D.G), dim3(256), stage_bytes, s, D, kcp, vcp, st->metric,
                       st->pos, st->block_table, st->ctx_len, st->free_map, evict_count, W.flag_scan, W.header);
  } else {
    hipLaunchKernelGGL(compact_move_kernel<false>, dim3(D.G), dim3(256), 0, s, D, kcp, vcp, st->metric, st->pos,
                       st->block_table, st->ctx_len, st->free_map, evict_count, W.flag_scan, W.header);
  }
  KVC_LAUNCH_CHECK();
  return (flags & KVC_ASYNC) ? KVC_OK : finish_sync(W, s);
}

}  // extern "C"
