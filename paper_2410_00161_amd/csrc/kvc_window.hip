// Prefill-end eviction metric from an observation window (KV-Compress:
// Preliminaries "KV Cache Compression" - sum of attention over the last w
// prompt queries, max-pooling over the sequence; Method "Query Group
// Compression" - also over the query heads of the KV head's group; "Metric
// Calculation", KVC-w - squared before summation).
//
// Unlike the decode this is a dense contraction: w * r query rows (32 .. 256)
// against every key of the head, so it runs on the matrix cores.  Up to 128
// rows, per 16 tokens and 16 rows: S^T[16 x 16] += K[16 x 32] * Q^T[32 x 16]
// with v_mfma_f32_16x16x32_bf16, four k-slices for d = 128; above, per 32
// tokens and 32 rows, v_mfma_f32_32x32x16_bf16 with eight k-slices (that shape
// issues at the full bf16 rate of this chip and the smaller one at half of it,
// but its kernel needs more registers than three or four wavefronts per SIMD
// leave; at 256 rows the LDS holds the CU to two per SIMD anyway).  A lane holds
// 64 (128) contiguous bytes of one token, its 16-byte loads being the k-slices,
// and Q is staged in LDS in exactly the register order of the B operand, so no
// transposes and no bank conflicts.  The contraction over d does not care in
// which order dimensions are assigned to k-slices as long as K and Q agree.
//
// Two passes over K: (1) per query row, max and sum of exp over its visible
// keys (online, then merged over lanes, wavefronts and chunks); (2) normalised
// probabilities, squared, summed over the query rows per key.  V is never
// read.  A last light pass max-pools over the logical sequence.
#include <cmath>
#include <type_traits>

#include "kvc_common.h"
#include "kvc_worklist.h"

namespace kvc {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kWinChunk = 1024;   // tokens per workgroup
constexpr int kWinThreads = 256;
constexpr int kWinWaves = 4;

struct WindowArgs {
  DecodeArgs A;        // cache, tables, work list (A.T = kWinChunk, A.q = window queries)
  int w, rows;         // queries this pass handles; query rows = w * r
  int q_first, q_count; // they are queries q_first .. q_first + w - 1 of the q_count the caller's tensor holds per head
  int pool;            // max-pool size over the sequence
  int add;             // add to the metric instead of replacing it
  int first_pos;       // position of query 0, the same for every head; -1 = the head's C - w
  int exclude;         // a query at position x adds to key j only when j <= x - exclude
  float* part;         // [partial slot][rows_pad][2]
  float* raw;          // [N * b] un-pooled sums, by physical slot
  const float* lse;    // [S, Lyr, Hq, q_count] natural-log softmax denominators from the caller, or NULL
  int reverse;         // pass 2 walks the work list backwards (what pass 1 read last is read first)
};

// Last key, in a head of C KVs, that any query of the call sees (lag = 0; query i sits at
// first + i and sees keys 0 .. its position) or adds to (lag = the excluded window: only keys at
// least that far behind the query).  Chunks that start behind it have no work in that pass, and
// nothing reads what they would have left.
__device__ __forceinline__ int last_key(const WindowArgs& W, int C, int lag) {
  const int first = W.first_pos >= 0 ? W.first_pos : C - W.w;
  return min(first + W.w - 1 - lag, C - 1);
}

// One matrix-core product: M tokens x M query rows.  Lane l holds query row l % M; `token` is
// the token, among the product's M, of element i of that lane's result.
template <int M> struct Mma;
template <> struct Mma<16> {
  typedef f32x4_t Acc;
  static constexpr int NV = 4;
  static __device__ __forceinline__ Acc run(const uint4& a, const uint4& b, Acc c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b),
                                                   c, 0, 0, 0);
  }
  static __device__ __forceinline__ int token(int i, int lane) { return 4 * (lane >> 4) + i; }
};
template <> struct Mma<32> {
  typedef f32x16_t Acc;
  static constexpr int NV = 16;
  static __device__ __forceinline__ Acc run(const uint4& a, const uint4& b, Acc c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b),
                                                   c, 0, 0, 0);
  }
  static __device__ __forceinline__ int token(int i, int lane) { return (i & 3) + 8 * (i >> 2) + 4 * (lane >> 5); }
};
// lanes that share a query row; k-slices (8 elements: 16 bytes of a query row, 16 or 8 bytes of a
// key row) of a lane's part of a row of HD elements; products per 64-token tile
template <int M> constexpr int kLanesPerRow = 64 / M;
template <int M, int HD> constexpr int kSlices = (HD / 8) / kLanesPerRow<M>;
template <int M> constexpr int kProducts = 64 / M;

// The piece of a key row a lane loads per k-slice, and its eight elements as packed bf16 (8-bit
// rows are widened exactly: 3 mantissa bits fit in 7).
template <int ESZ> struct KPiece;
template <> struct KPiece<2> {
  typedef uint4 Raw;
  static __device__ __forceinline__ Raw zero() { return make_uint4(0, 0, 0, 0); }
  static __device__ __forceinline__ uint4 widen(const uint4& a) { return a; }
};
template <> struct KPiece<1> {
  typedef uint2 Raw;
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  static __device__ __forceinline__ Raw zero() { return make_uint2(0, 0); }
  static __device__ __forceinline__ uint4 widen(const uint2& a) {
    return make_uint4(__builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(a.x, 1.0f, false)),
                      __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(a.x, 1.0f, true)),
                      __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(a.y, 1.0f, false)),
                      __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(a.y, 1.0f, true)));
  }
};

// Q of one head instance into LDS, in B-operand order: entry ((ct * KS + s) * 64 + lane) holds,
// for query row ct * M + lane % M, the 8 dimensions at byte 16 KS (lane / M) + 16 s of the row.
// Query row rho = i * r + hh (window query i, query head hh); rows past w * r are zero.
// Read in runs of 64 bytes, four lanes to a run and 16 consecutive rows to a wavefront, all of a
// thread's loads before its stores; the LDS writes then meet a 4-way bank conflict, well under
// a microsecond per workgroup.  (One lane per LDS entry in entry order, every 16-byte read on
// a line of its own, measured the same.)
template <int HD, int M, int NT>
__device__ __forceinline__ void stage_queries(const WindowArgs& W, int g, uint4* s_q) {
  constexpr int KS = kSlices<M, HD>, ROWS = NT * M;
  constexpr int QP = HD / 8;                      // 16-byte pieces of a query row
  constexpr int QROWB = HD * 2;
  constexpr int PER = ROWS * QP / kWinThreads;    // pieces per thread
  static_assert(PER * kWinThreads == ROWS * QP && PER >= 1 && PER <= 16, "whole rounds of the workgroup");
  const int r = W.A.D.r, w = W.q_count;
  const char* qbase = W.A.q + ((size_t)g * r * w + W.q_first) * QROWB;  // [r][q_count][HD] bf16, from query q_first
  // all of a thread's loads first, then its stores: one trip to memory, not PER of them
  uint4 v[PER];
#pragma unroll
  for (int it = 0; it < PER; ++it) {
    const int e = threadIdx.x + it * kWinThreads;
    const int rho = (e >> 2) % ROWS;
    const int c = 4 * ((e >> 2) / ROWS) + (e & 3);   // 16-byte piece of the row
    const int i = rho / r, hh = rho % r;
    // (rows past w * r read row 0 and are zeroed: a select between values, no branch around a load)
    const uint4 t = *(const uint4*)(qbase + (rho < W.rows ? (size_t)hh * w + i : 0) * QROWB + 16 * c);
    v[it] = rho < W.rows ? t : make_uint4(0, 0, 0, 0);
  }
#pragma unroll
  for (int it = 0; it < PER; ++it) {
    const int e = threadIdx.x + it * kWinThreads;
    const int rho = (e >> 2) % ROWS;
    const int c = 4 * ((e >> 2) / ROWS) + (e & 3);
    s_q[((rho / M) * KS + c % KS) * 64 + (c / KS) * M + rho % M] = v[it];
  }
}

// Loads the 64-token tile starting at chunk token `tt` as A operands of M tokens each: lane
// (token lane % M, part lane / M of its row) holds that part's k-slices.  Every lane looks its own
// token's block up (blocks may be shorter than the 16 tokens that share a row of lanes); tokens
// past the end of the chunk are not touched and read as zero.
template <int ESZ, int HD, int M>
__device__ __forceinline__ void load_tile(const WindowArgs& W, const int* s_tab, int tt, int n_tok, int lane,
                                          typename KPiece<ESZ>::Raw (&k)[kProducts<M>][kSlices<M, HD>]) {
  constexpr int KS = kSlices<M, HD>;
  constexpr int PB = 8 * ESZ;                     // bytes of one k-slice of a key row
  typedef typename KPiece<ESZ>::Raw Raw;
  const int lb = W.A.log2b, b = W.A.D.b;
#pragma unroll
  for (int pr = 0; pr < kProducts<M>; ++pr) {
    const int t = tt + pr * M + (lane & (M - 1));
    const bool live = t < n_tok;
    const size_t slot = live ? ((size_t)s_tab[t >> lb] << lb) + (t & (b - 1)) : 0;
    const char* p = W.A.kc + slot * (size_t)(HD * ESZ) + PB * KS * (lane / M);
#pragma unroll
    for (int sl = 0; sl < KS; ++sl) k[pr][sl] = live ? *(const Raw*)(p + PB * sl) : KPiece<ESZ>::zero();
  }
}

// Running (max, sum) pairs a wavefront keeps per column tile in pass 1.  One per lane (a lane
// covers 64 / kLanesPerRow tokens of a tile for its query row) up to 128 query rows; at 256 the
// lanes of a row merge theirs after every tile instead, a few cross-lane moves per tile, which
// brings the workgroup from 96 KB of LDS to 72 and a second workgroup onto the CU.
__host__ __device__ constexpr int window_pairs_per_tile(int m, int nt) { return nt * m >= 256 ? m : 64; }

// Pass 1: per chunk and query row, max and sum of exp2 over the visible keys.
template <int ESZ, int HD, int M, int NT>
__global__ void __launch_bounds__(kWinThreads) window_stats_kernel(WindowArgs W) {
  typedef Mma<M> MM;
  typedef typename KPiece<ESZ>::Raw Raw;
  constexpr int KS = kSlices<M, HD>, NP = kProducts<M>, ROWS = NT * M;
  constexpr int PPT = window_pairs_per_tile(M, NT);
  constexpr bool kRowMerged = PPT == M;
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
  uint4* s_q = (uint4*)smem_raw;                        // [NT * KS * 64]
  float* s_ml = (float*)s_q;                            // [waves][ROWS][2], once the main loops are over
  float2* s_st = (float2*)(s_q + NT * KS * 64);         // [waves][NT][PPT]
  int* s_tab = (int*)(s_st + kWinWaves * NT * PPT);     // [T / b + 1]
  const int b = A.D.b, lb = A.log2b;
  const int C = A.ctx[g];
  const size_t pslot = (size_t)it.pbase + (size_t)(t0 / A.T);
  const int first_free = W.first_pos >= 0 ? W.first_pos : C - W.w;  // query i sits at first_free + i
  const int free_lim = min(first_free, C - 1);   // keys up to here are visible to every query
  const int n_seen = last_key(W, C, 0) - t0 + 1;   // tokens of the chunk that some query sees
  if (n_seen <= 0) return;
  {
    const int nblk = (n_tok + b - 1) >> lb;
    const int32_t* row = A.table + (size_t)g * A.D.maxb + (t0 >> lb);
    for (int i = tid; i < nblk; i += kWinThreads) s_tab[i] = row[i];
  }
  stage_queries<HD, M, NT>(W, g, s_q);
  __syncthreads();
  // running (max, sum) per column tile: kept in LDS so that the loop over column tiles stays a
  // loop (registers: one K tile and one Q tile at a time)
  float2* my_st = s_st + (size_t)wv * NT * PPT + (lane & (PPT - 1));
  for (int ct = 0; ct < NT; ++ct) my_st[ct * PPT] = make_float2(-INFINITY, 0.0f);
  auto tile = [&](Raw (&kraw)[NP][KS], int tt) {
    uint4 k[NP][KS];
#pragma unroll
    for (int pr = 0; pr < NP; ++pr)
#pragma unroll
      for (int sl = 0; sl < KS; ++sl) k[pr][sl] = KPiece<ESZ>::widen(kraw[pr][sl]);
    // most tiles lie wholly in front of the window: they run the loop without the causal mask
    auto column_tiles = [&](auto masked_c) {
      constexpr bool kMasked = decltype(masked_c)::value;
#pragma unroll 1
      for (int ct = 0; ct < NT; ++ct) {
        uint4 q[KS];
#pragma unroll
        for (int sl = 0; sl < KS; ++sl) q[sl] = s_q[(ct * KS + sl) * 64 + lane];
        int last_vis = 0;
        if constexpr (kMasked) {
          const int rho = ct * M + (lane & (M - 1));
          last_vis = min(first_free + rho / A.D.r, C - 1);  // query i sees keys 0 .. its position
        }
        typename MM::Acc acc[NP];
#pragma unroll
        for (int pr = 0; pr < NP; ++pr)
#pragma unroll
          for (int i = 0; i < MM::NV; ++i) acc[pr][i] = 0.0f;
#pragma unroll
        for (int sl = 0; sl < KS; ++sl)   // NP independent accumulation chains
#pragma unroll
          for (int pr = 0; pr < NP; ++pr) acc[pr] = MM::run(k[pr][sl], q[sl], acc[pr]);
        // the running max stays in raw dot-product units inside the loop: the scale goes into one
        // multiply-add per logit (max, fma, exp2, add)
        const float2 old = my_st[ct * PPT];
        float mx = old.x;
#pragma unroll
        for (int pr = 0; pr < NP; ++pr)
#pragma unroll
          for (int i = 0; i < MM::NV; ++i) {
            if constexpr (kMasked) {
              const int j = t0 + tt + pr * M + MM::token(i, lane);
              if (j > last_vis) acc[pr][i] = -INFINITY;
            }
            mx = fmaxf(mx, acc[pr][i]);
          }
        if constexpr (kRowMerged) {   // the row's max over the tile's 64 tokens
#pragma unroll
          for (int msk = M; msk < 64; msk <<= 1) mx = fmaxf(mx, __shfl_xor(mx, msk));
        }
        if (mx > -INFINITY) {   // (the same in the lanes of a row when they merge)
          const float off = -mx * A.scale_log2;
          float sum = 0.0f;
#pragma unroll
          for (int pr = 0; pr < NP; ++pr)
#pragma unroll
            for (int i = 0; i < MM::NV; ++i) sum += __builtin_amdgcn_exp2f(fmaf(acc[pr][i], A.scale_log2, off));
          if constexpr (kRowMerged) {
#pragma unroll
            for (int msk = M; msk < 64; msk <<= 1) sum += __shfl_xor(sum, msk);
          }
          sum += old.y * __builtin_amdgcn_exp2f(fmaf(old.x, A.scale_log2, off));
          if (!kRowMerged || lane < M) my_st[ct * PPT] = make_float2(mx, sum);
        }
      }
    };
    if (t0 + tt + 63 > free_lim) column_tiles(std::true_type{});
    else column_tiles(std::false_type{});
  };
  for (int tt = wv * 64; tt < min(n_tok, n_seen); tt += 64 * kWinWaves) {
    Raw k[NP][KS];
    load_tile<ESZ, HD, M>(W, s_tab, tt, n_tok, lane, k);
    tile(k, tt);
  }
  __syncthreads();   // every wavefront is done with Q: its bytes now take the per-wavefront pairs
  // merge the lanes that share a query row (if not done yet), then the wavefronts, then write
  // the chunk's pair
  for (int ct = 0; ct < NT; ++ct) {
    float2 st = my_st[ct * PPT];
    st.x *= A.scale_log2;   // from here on maxima are in scaled log2 units
#pragma unroll
    for (int msk = M; msk < (kRowMerged ? 0 : 64); msk <<= 1) {
      const float om = __shfl_xor(st.x, msk), ol = __shfl_xor(st.y, msk);
      const float nm = fmaxf(st.x, om);
      if (nm > -INFINITY) st.y = st.y * __builtin_amdgcn_exp2f(st.x - nm) + ol * __builtin_amdgcn_exp2f(om - nm);
      st.x = nm;
    }
    if (lane < M) {
      s_ml[((wv * NT + ct) * M + lane) * 2 + 0] = st.x;
      s_ml[((wv * NT + ct) * M + lane) * 2 + 1] = st.y;
    }
  }
  __syncthreads();
  for (int rho = tid; rho < ROWS; rho += kWinThreads) {
    float mm = -INFINITY, ll = 0.0f;
    for (int ww = 0; ww < kWinWaves; ++ww) {
      const float om = s_ml[((ww * ROWS) + rho) * 2], ol = s_ml[((ww * ROWS) + rho) * 2 + 1];
      const float nm = fmaxf(mm, om);
      if (nm > -INFINITY) ll = ll * __builtin_amdgcn_exp2f(mm - nm) + ol * __builtin_amdgcn_exp2f(om - nm);
      mm = nm;
    }
    W.part[(pslot * ROWS + rho) * 2 + 0] = mm;
    W.part[(pslot * ROWS + rho) * 2 + 1] = ll;
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
  const int seen = last_key(W, A.ctx[it.g], 0);
  const int nch = seen < 0 ? 0 : min(it.nch, seen / A.T + 1);   // chunks that pass 1 worked on
  for (int rho = threadIdx.x; rho < rows_pad; rho += 256) {
    float mm = -INFINITY, ll = 0.0f;
    for (int cc = 0; cc < nch; ++cc) {
      const float2 ml = *(const float2*)(W.part + (((size_t)it.pbase + cc) * rows_pad + rho) * 2);
      const float nm = fmaxf(mm, ml.x);
      if (nm > -INFINITY) ll = ll * __builtin_amdgcn_exp2f(mm - nm) + ml.y * __builtin_amdgcn_exp2f(ml.x - nm);
      mm = nm;
    }
    W.part[((size_t)it.pbase * rows_pad + rho) * 2] = (rho < W.rows && ll > 0.0f) ? mm + __builtin_amdgcn_logf(ll) : INFINITY;
  }
}

// Pass 2: raw[j] = sum over query rows of p^2 (or p), p normalised with the head's max and sum.
template <int ESZ, int HD, int M, int NT, bool L2>
__global__ void __launch_bounds__(kWinThreads) window_sum_kernel(WindowArgs W) {
  typedef Mma<M> MM;
  typedef typename KPiece<ESZ>::Raw Raw;
  constexpr int KS = kSlices<M, HD>, NP = kProducts<M>, ROWS = NT * M;
  const DecodeArgs& A = W.A;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int total_items = A.header[HW_TOTAL_ITEMS];
  if (blockIdx.x == 0 && tid < HW_DEC_END - HW_DEC_BINS) A.header[HW_DEC_BINS + tid] = 0;  // work-list block back to zero
  if ((int)blockIdx.x >= total_items || total_items > A.cap) return;
  // Backwards through the list when this pass follows pass 1: the keys that pass read last are the
  // ones still held by the memory-side cache, and this pass reads them first.
  const DecodeItem it = A.items[W.reverse ? total_items - 1 - (int)blockIdx.x : (int)blockIdx.x];
  const int g = it.g, t0 = it.t0, n_tok = it.n_tok, nch = it.nch;
  if ((unsigned)g >= (unsigned)A.D.G || n_tok <= 0 || n_tok > A.T || t0 < 0 || nch <= 0 || it.pbase < 0 ||
      it.pbase + nch > A.cap)
    return;
  extern __shared__ __align__(16) char smem_raw[];
  uint4* s_q = (uint4*)smem_raw;                        // [NT * KS * 64]
  float* s_ml = (float*)(s_q + NT * KS * 64);           // [ROWS]: max + log2(sum) per query row (inf: the row adds nothing)
  int* s_tab = (int*)(s_ml + ROWS);                     // [T / b + 1]
  const int b = A.D.b, lb = A.log2b;
  const int C = A.ctx[g];
  const int n_fed = last_key(W, C, W.exclude) - t0 + 1;   // tokens of the chunk that some query adds to
  if (n_fed <= 0) return;
  {
    const int nblk = (n_tok + b - 1) >> lb;
    const int32_t* row = A.table + (size_t)g * A.D.maxb + (t0 >> lb);
    for (int i = tid; i < nblk; i += kWinThreads) s_tab[i] = row[i];
  }
  const int first_free = W.first_pos >= 0 ? W.first_pos : C - W.w;
  const int free_lim = min(first_free - W.exclude, C - 1);   // keys up to here count for every query
  stage_queries<HD, M, NT>(W, g, s_q);
  for (int rho = tid; rho < ROWS; rho += kWinThreads) {
    if (W.lse) {   // the caller's ln(sum of exp) per query row, to log2 units; padded rows add nothing
      const int i = rho / A.D.r, hh = rho % A.D.r;
      s_ml[rho] = rho < W.rows ? W.lse[((size_t)g * A.D.r + hh) * W.q_count + W.q_first + i] * 1.4426950408889634f : INFINITY;
    } else {
      s_ml[rho] = W.part[((size_t)it.pbase * ROWS + rho) * 2];
    }
  }
  __syncthreads();
  auto tile = [&](Raw (&kraw)[NP][KS], int tt) {
    uint4 k[NP][KS];
#pragma unroll
    for (int pr = 0; pr < NP; ++pr)
#pragma unroll
      for (int sl = 0; sl < KS; ++sl) k[pr][sl] = KPiece<ESZ>::widen(kraw[pr][sl]);
    float tok[M];   // [product][element]
#pragma unroll
    for (int e = 0; e < M; ++e) tok[e] = 0.0f;
    auto column_tiles = [&](auto masked_c) {
      constexpr bool kMasked = decltype(masked_c)::value;
#pragma unroll 1
      for (int ct = 0; ct < NT; ++ct) {
        uint4 q[KS];
#pragma unroll
        for (int sl = 0; sl < KS; ++sl) q[sl] = s_q[(ct * KS + sl) * 64 + lane];
        const int rho = ct * M + (lane & (M - 1));
        int last_vis = 0;
        if constexpr (kMasked) last_vis = min(first_free + rho / A.D.r - W.exclude, C - 1);   // seen, and far enough behind
        const float c_row = s_ml[rho];
        typename MM::Acc acc[NP];
#pragma unroll
        for (int pr = 0; pr < NP; ++pr)
#pragma unroll
          for (int i = 0; i < MM::NV; ++i) acc[pr][i] = 0.0f;
#pragma unroll
        for (int sl = 0; sl < KS; ++sl)
#pragma unroll
          for (int pr = 0; pr < NP; ++pr) acc[pr] = MM::run(k[pr][sl], q[sl], acc[pr]);
#pragma unroll
        for (int pr = 0; pr < NP; ++pr)
#pragma unroll
          for (int i = 0; i < MM::NV; ++i) {
            float p = __builtin_amdgcn_exp2f(fmaf(acc[pr][i], A.scale_log2, -c_row));
            if constexpr (kMasked) {
              const int j = t0 + tt + pr * M + MM::token(i, lane);
              if (j > last_vis) p = 0.0f;
            }
            tok[pr * MM::NV + i] = L2 ? fmaf(p, p, tok[pr * MM::NV + i]) : tok[pr * MM::NV + i] + p;
          }
      }
    };
    if (t0 + tt + 63 > free_lim) column_tiles(std::true_type{});
    else column_tiles(std::false_type{});
    // sum over the M lanes (query rows) of a row group: lane % M == e ends up with value e
    Butterfly<M, M / 2>::run(tok, lane);
    const int e = lane & (M - 1);
    const int t = tt + (e / MM::NV) * M + MM::token(e % MM::NV, lane);
    if (t < n_tok && t0 + t < C) {
      const size_t slot = ((size_t)s_tab[t >> lb] << lb) + (t & (b - 1));
      if (W.pool > 1) W.raw[slot] = tok[0];          // pooled over the sequence by window_pool_kernel
      else if (t < n_fed) A.metric[slot] = W.add ? A.metric[slot] + tok[0] : tok[0];   // no pooling: straight into the metric (one writer per slot)
    }
  };
  for (int tt = wv * 64; tt < min(n_tok, n_fed); tt += 64 * kWinWaves) {
    Raw k[NP][KS];
    load_tile<ESZ, HD, M>(W, s_tab, tt, n_tok, lane, k);
    tile(k, tt);
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
  // positions behind the last key that pass 2 added to get nothing (and hold nothing to read)
  const int live = max(0, last_key(W, C, W.exclude) + 1);
  if (j0 >= live) return;
  const int j1 = min(live, j0 + kPoolTile);
  const int b = A.D.b, lb = A.log2b;
  const int32_t* row = A.table + (size_t)g * A.D.maxb;
  const int P = W.first_pos >= 0 ? 0 : max(0, C - W.w), half = W.pool / 2;
  __shared__ float s_raw[kPoolTile + 2 * kPoolHalo];
  const bool staged = half <= kPoolHalo;
  const int lo0 = staged ? max(0, j0 - half) : j0, hi0 = staged ? min(live, j1 + half) : j1;
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

template <int ESZ, int HD, int M, int NT>
static int launch_window(const WindowArgs& W, int grid, hipStream_t s) {
  // pass 1: Q (later the per-wavefront pairs), running pairs per column tile, block ids;
  // pass 2: Q, one float per query row, block ids.  Three and four workgroups per CU at 128 rows
  // of d = 128, two and two at 256.
  constexpr size_t q_bytes = (size_t)NT * M * HD * 2, rows = (size_t)NT * M;
  const size_t tab = ((size_t)kWinChunk / W.A.D.b + 1) * 4;
  static_assert((size_t)kWinWaves * rows * 2 * 4 <= q_bytes, "the per-wavefront pairs of pass 1 fit where Q was");
  const size_t lds = q_bytes + (size_t)kWinWaves * NT * window_pairs_per_tile(M, NT) * 8 + tab;
  const size_t lds2 = q_bytes + rows * 4 + tab;
  {  // above the default cap a kernel must be told how much it may take (the block-id array grows as blocks shrink)
    static LdsLimit limit;
    const int rc = limit.need(lds > lds2 ? lds : lds2, window_stats_kernel<ESZ, HD, M, NT>,
                              window_sum_kernel<ESZ, HD, M, NT, true>, window_sum_kernel<ESZ, HD, M, NT, false>);
    if (rc != KVC_OK) return rc;
  }
  if (!W.lse) {   // with the caller's log-sum-exp there is nothing for pass 1 to find
    hipLaunchKernelGGL((window_stats_kernel<ESZ, HD, M, NT>), dim3(grid), dim3(kWinThreads), lds, s, W);
    KVC_LAUNCH_CHECK();
    hipLaunchKernelGGL(window_rows_kernel, dim3(grid), dim3(256), 0, s, W, (int)rows);
    KVC_LAUNCH_CHECK();
  }
  if (W.A.D.mode == KVC_L2) hipLaunchKernelGGL((window_sum_kernel<ESZ, HD, M, NT, true>), dim3(grid), dim3(kWinThreads), lds2, s, W);
  else hipLaunchKernelGGL((window_sum_kernel<ESZ, HD, M, NT, false>), dim3(grid), dim3(kWinThreads), lds2, s, W);
  KVC_LAUNCH_CHECK();
  return KVC_OK;
}

template <int ESZ, int HD>
static int launch_window_rows(const WindowArgs& W, int padded_rows, int grid, hipStream_t s) {
  switch (padded_rows) {
    case 32: return launch_window<ESZ, HD, 16, 2>(W, grid, s);
    case 64: return launch_window<ESZ, HD, 16, 4>(W, grid, s);
    case 128: return launch_window<ESZ, HD, 16, 8>(W, grid, s);
    default: return launch_window<ESZ, HD, 32, 8>(W, grid, s);
  }
}

}  // namespace kvc

using namespace kvc;

extern "C" {

static int window_common(const kvc_config* cfg, const kvc_state* st, const void* q_win, int w, int pool,
                         int accumulate, int first_pos, int exclude, const float* row_lse, int layer_begin,
                         int layer_end, void* ws, void* stream) {
  int rc = validate(cfg, st);
  if (rc != KVC_OK) return rc;
  if (!q_win || !ws || ((uintptr_t)ws & 255) || ((uintptr_t)q_win & 15) || ((uintptr_t)row_lse & 3)) return KVC_ERR_ARG;
  Dims D = dims_of(cfg);
  if (layer_begin < 0 || layer_end > D.Lyr || layer_begin >= layer_end) return KVC_ERR_ARG;
  if (w <= 0 || pool <= 0 || (pool & 1) == 0 || exclude < 0) return KVC_ERR_ARG;
  // the matrix-core kernels cover 16-bit and 8-bit rows (bf16 queries), d = 64 or 128, any block
  // size that divides a chunk, up to 256 query rows
  if ((D.dtype != KVC_BF16 && D.dtype != KVC_FP8_E4M3) || (D.d != 128 && D.d != 64) || kWinChunk % D.b != 0)
    return KVC_ERR_UNSUPPORTED;
  // One pass of the kernels takes at most 64 queries and 256 query rows (a chunk's pairs, 8 bytes
  // per padded query row, live in the decode's slot of r * d floats).  A block of queries at a
  // given position may be longer: it is worked off in such passes over one work list.
  auto padded = [](int rows) { return rows <= 32 ? 32 : rows <= 64 ? 64 : rows <= 128 ? 128 : 256; };
  int w_pass = w < 64 ? w : 64;
  while (w_pass >= 1 && (w_pass * D.r > 256 || (size_t)padded(w_pass * D.r) * 8 > (size_t)D.r * D.d * 4)) --w_pass;
  if (w_pass < 1 || (w > w_pass && first_pos < 0)) return KVC_ERR_UNSUPPORTED;
  Workspace Wk = carve(D, ws);
  hipStream_t s = (hipStream_t)stream;
  WindowArgs W;
  DecodeArgs& A = W.A;
  A.D = D;
  A.kc = (const char*)st->k_cache; A.vc = (const char*)st->v_cache;
  A.metric = st->metric; A.table = st->block_table; A.ctx = st->ctx_len;
  A.q = (const char*)q_win; A.out = nullptr;
  A.l0 = layer_begin; A.nl = layer_end - layer_begin; A.gsel = D.S * A.nl * D.Hk;
  A.accumulate = 1; A.T = kWinChunk; A.adapt_T = 0;
  A.log2b = 0;
  while ((1 << A.log2b) < D.b) ++A.log2b;
  A.all_partials = 1;
  A.rotate_chunks = 1;
  A.short_class = 16;  // no separate launch for short items here
  A.Ts = 0;
  A.cap = (int)(max_items_of(D) < 0x7fffffffull ? max_items_of(D) : 0x7fffffffull);
  A.items = (DecodeItem*)Wk.items; A.slot_item = Wk.slot_item; A.part_ml = Wk.part_ml; A.part_acc = Wk.part_acc; A.stash = Wk.stash;
  A.header = Wk.header;
  A.status = Wk.header;
  A.plan = 0; A.plan_stride = 0; A.ctx_plus = 0;
  A.scale_log2 = (float)(1.4426950408889634 / sqrt((double)D.d));
  W.pool = pool; W.add = accumulate != 0; W.exclude = exclude;
  W.q_count = w;
  W.part = Wk.part_acc; W.raw = Wk.stash;
  W.lse = row_lse;
  W.reverse = row_lse == nullptr;
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
  const int pool_tiles = (int)(((size_t)D.maxb * D.b + kPoolTile - 1) / kPoolTile);
  if (pool_tiles > 65535) return KVC_ERR_UNSUPPORTED;
  for (int q0 = 0; q0 < w; q0 += w_pass) {
    W.q_first = q0;
    W.w = w - q0 < w_pass ? w - q0 : w_pass;
    W.rows = W.w * D.r;
    W.first_pos = first_pos < 0 ? first_pos : first_pos + q0;
    const int pr = padded(W.rows);
    if (D.dtype == KVC_BF16) rc = D.d == 128 ? launch_window_rows<2, 128>(W, pr, (int)grid, s) : launch_window_rows<2, 64>(W, pr, (int)grid, s);
    else rc = D.d == 128 ? launch_window_rows<1, 128>(W, pr, (int)grid, s) : launch_window_rows<1, 64>(W, pr, (int)grid, s);
    if (rc != KVC_OK) return rc;
    if (pool > 1) {   // without pooling the sums went into the metric as they were formed
      hipLaunchKernelGGL(window_pool_kernel, dim3(A.gsel, pool_tiles), dim3(256), 0, s, W);
      KVC_LAUNCH_CHECK();
    }
  }
  return KVC_OK;
}

int kvc_window_metric(const kvc_config* cfg, const kvc_state* st, const void* q_win, const float* row_lse, int w,
                      int pool, int accumulate, int layer_begin, int layer_end, void* ws, void* stream) {
  return window_common(cfg, st, q_win, w, pool, accumulate, -1, 0, row_lse, layer_begin, layer_end, ws, stream);
}

int kvc_query_block_metric(const kvc_config* cfg, const kvc_state* st, const void* q_blk, const float* row_lse, int w,
                           int first_pos, int exclude, int layer_begin, int layer_end, void* ws, void* stream) {
  if (first_pos < 0) return KVC_ERR_ARG;
  return window_common(cfg, st, q_blk, w, 1, 1, first_pos, exclude, row_lse, layer_begin, layer_end, ws, stream);
}

}  // extern "C"
