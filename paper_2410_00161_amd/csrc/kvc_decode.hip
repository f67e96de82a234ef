// Paged decode attention with one block table and one context length per
// (sequence, layer, KV head), accumulating the per-KV eviction metric in the
// same pass (KV-Compress: Preliminaries "Multi-head Attention" and "Paged
// Attention"; Method "Query Group Compression", "Block Layout and Parallel
// Allocation", "Squared Attention Metric", "Continual Compression").
//
// Work decomposition.  The metric needs the NORMALISED probability of every KV,
// which is known only once a head's max and sum are.  A head instance is cut
// into chunks of T tokens; one workgroup owns one chunk, keeps the chunk's r x T
// logits in LDS between its pass over K and its pass over V, and therefore
// reads every key and value exactly once.  A head that fits one chunk is
// finished inside that workgroup (output and metric written directly).  A longer
// head leaves per-chunk (max, sum, un-normalised output) and the chunk-relative
// exp of every logit in the workspace; a second, light kernel combines them.
//
// Data movement.  A KV row (d elements) is 256 bytes at d = 128 / bf16; a lane
// reads 16 bytes, so LPT = row_bytes / 16 lanes cover one token and a wavefront
// load covers 64 / LPT whole tokens: 1 KiB contiguous per load at b >= TPI.
// The r dot products of a token are finished with a halving butterfly over the
// LPT lanes, which leaves each lane with distinct (token, head) logits instead
// of every lane with all of them.
#include <cmath>

#include "kvc_common.h"

namespace kvc {

static int g_chunk_tokens = 0;  // 0 = default; set by kvc_set_decode_chunk

// optional event pairs around the two decode kernels (kvc_profile_begin / _collect)
struct ProfilePair { hipEvent_t a0, a1, b0, b1; };
static ProfilePair* g_prof = nullptr;
static int g_prof_cap = 0, g_prof_used = 0;

struct DecodeArgs {
  Dims D;
  const char* kc;
  const char* vc;
  float* metric;
  const int32_t* table;
  const int32_t* ctx;
  const char* q;
  float* out;
  int l0, nl, gsel;       // first layer, layer count, head instances selected
  int accumulate, T;      // metric on/off, chunk tokens
  const int32_t* chunk_off;  // [gsel + 1]
  float* part_ml;
  float* part_acc;
  float* stash;
  const int32_t* header;
  float scale_log2;       // log2(e) / sqrt(d)
};

__device__ __forceinline__ int sel_to_g(const Dims& D, int l0, int nl, int gi) {
  const int s = gi / (nl * D.Hk);
  const int l = l0 + (gi / D.Hk) % nl;
  const int h = gi % D.Hk;
  return (s * D.Lyr + l) * D.Hk + h;
}

struct ChunkFn {
  const int32_t* ctx;
  Dims D;
  int l0, nl, T;
  __device__ int operator()(int gi) const {
    const int C = ctx[sel_to_g(D, l0, nl, gi)];
    return (C + T - 1) / T;
  }
};

// A head instance with no KV gets a zero output row for each of its query heads.
__global__ void __launch_bounds__(256) zero_empty_kernel(DecodeArgs A) {
  const int gi = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (gi >= A.gsel) return;
  const int g = sel_to_g(A.D, A.l0, A.nl, gi);
  if (A.ctx[g] != 0) return;
  float* o = A.out + (size_t)g * A.D.r * A.D.d;
  for (int i = threadIdx.x & 63; i < A.D.r * A.D.d; i += 64) o[i] = 0.0f;
}

// largest i in [0, n) with off[i] <= item, given off[n] > item
__device__ __forceinline__ int find_owner(const int32_t* __restrict__ off, int n, int item) {
  int lo = 0, hi = n;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (off[mid] <= item) lo = mid; else hi = mid;
  }
  return lo;
}

template <int N, int MASK>
struct Butterfly {
  // Sums v[0..N) across the lanes that differ in the bits at and below MASK, halving the
  // number of live values at each step while more than one is left.
  static __device__ __forceinline__ void run(float* v, int lane) {
    if constexpr (MASK >= 1) {
      if constexpr (N > 1) {
        constexpr int H = N / 2;
        const bool up = (lane & MASK) != 0;
#pragma unroll
        for (int i = 0; i < H; ++i) {
          const float keep = up ? v[H + i] : v[i];
          const float send = up ? v[i] : v[H + i];
          v[i] = keep + __shfl_xor(send, MASK);
        }
        Butterfly<H, MASK / 2>::run(v, lane);
      } else {
        v[0] += __shfl_xor(v[0], MASK);
        Butterfly<1, MASK / 2>::run(v, lane);
      }
    }
  }
};

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

template <int ESZ> struct Row;
template <> struct Row<2> {  // bf16: 8 elements in 16 bytes
  static constexpr int EPL = 8;
  static __device__ __forceinline__ float dot(const uint4& a, const uint4& b) {
    float s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.x), __builtin_bit_cast(bf16x2_t, b.x), 0.0f, false);
    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.y), __builtin_bit_cast(bf16x2_t, b.y), s, false);
    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.z), __builtin_bit_cast(bf16x2_t, b.z), s, false);
    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.w), __builtin_bit_cast(bf16x2_t, b.w), s, false);
    return s;
  }
  static __device__ __forceinline__ void widen(const uint4& a, float* f) {
    f[0] = bf16_lo(a.x); f[1] = bf16_hi(a.x); f[2] = bf16_lo(a.y); f[3] = bf16_hi(a.y);
    f[4] = bf16_lo(a.z); f[5] = bf16_hi(a.z); f[6] = bf16_lo(a.w); f[7] = bf16_hi(a.w);
  }
};
template <> struct Row<4> {  // f32: 4 elements in 16 bytes
  static constexpr int EPL = 4;
  static __device__ __forceinline__ float dot(const uint4& a, const uint4& b) {
    float s = __uint_as_float(a.x) * __uint_as_float(b.x);
    s = fmaf(__uint_as_float(a.y), __uint_as_float(b.y), s);
    s = fmaf(__uint_as_float(a.z), __uint_as_float(b.z), s);
    s = fmaf(__uint_as_float(a.w), __uint_as_float(b.w), s);
    return s;
  }
  static __device__ __forceinline__ void widen(const uint4& a, float* f) {
    f[0] = __uint_as_float(a.x); f[1] = __uint_as_float(a.y);
    f[2] = __uint_as_float(a.z); f[3] = __uint_as_float(a.w);
  }
};

constexpr int kDecodeThreads = 256;
constexpr int kDecodeWaves = kDecodeThreads / 64;

__host__ __device__ inline size_t decode_lds_bytes(int T, int R, int HD, int b) {
  return (size_t)T * R * 4 + (size_t)kDecodeWaves * R * HD * 4 + 2 * kDecodeWaves * R * 4 +
         ((size_t)T / b + 1) * 4;
}

template <int ESZ, int HD, int R>
__global__ void __launch_bounds__(kDecodeThreads) decode_chunk_kernel(DecodeArgs A) {
  constexpr int EPL = Row<ESZ>::EPL;
  constexpr int LPT = HD / EPL;        // lanes per token
  constexpr int TPI = 64 / LPT;        // tokens per wavefront load
  constexpr int U = 16 / TPI;          // loads per 16-token group
  constexpr int NV = R * U;            // partial logits per lane before the butterfly
  constexpr int PER = NV >= LPT ? NV / LPT : 1;  // logits per lane after it
  constexpr size_t ROWB = (size_t)HD * ESZ;
  static_assert(LPT >= 2 && LPT <= 64 && (16 % TPI) == 0, "row geometry");

  const int item = blockIdx.x;
  if (item >= A.header[HW_TOTAL_ITEMS]) return;
  const int gi = find_owner(A.chunk_off, A.gsel, item);
  const int first = A.chunk_off[gi];
  const int c = item - first;
  const int nch = A.chunk_off[gi + 1] - first;
  const int g = sel_to_g(A.D, A.l0, A.nl, gi);
  const int b = A.D.b, T = A.T;
  const int C = A.ctx[g];
  const int t0 = c * T;
  const int n_tok = min(T, C - t0);

  extern __shared__ __align__(16) char smem_raw[];
  float* s_log = (float*)smem_raw;                     // [T][R]
  float* s_acc = s_log + (size_t)T * R;                // [waves][R][HD]
  float* s_red = s_acc + kDecodeWaves * R * HD;        // [2][waves][R]
  int* s_tab = (int*)(s_red + 2 * kDecodeWaves * R);   // [T / b + 1]

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int sub = lane / LPT, seg = lane % LPT;

  {
    const int nblk = (n_tok + b - 1) / b;
    const int32_t* row = A.table + (size_t)g * A.D.maxb + t0 / b;
    for (int i = tid; i < nblk; i += kDecodeThreads) s_tab[i] = row[i];
  }
  uint4 qv[R];
#pragma unroll
  for (int hh = 0; hh < R; ++hh)
    qv[hh] = *(const uint4*)(A.q + ((size_t)g * R + hh) * ROWB + (size_t)seg * 16);
  __syncthreads();

  // ---- pass over K: logits (scaled for exp2) into LDS ----
  for (int base = w * 16; base < n_tok; base += 16 * kDecodeWaves) {
    uint4 kv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int tok = base + u * TPI + sub;
      if (base + u * TPI < n_tok) {
        const size_t slot = (size_t)s_tab[tok / b] * b + (tok % b);
        kv[u] = *(const uint4*)(A.kc + slot * ROWB + (size_t)seg * 16);
      } else {
        kv[u] = make_uint4(0, 0, 0, 0);
      }
    }
    float part[NV];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int hh = 0; hh < R; ++hh) part[u * R + hh] = Row<ESZ>::dot(kv[u], qv[hh]);
    Butterfly<NV, LPT / 2>::run(part, lane);
    const int idx0 = (seg * NV) / LPT;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int idx = idx0 + i;
      const int u = idx / R, hh = idx % R;
      const int tok = base + u * TPI + sub;
      s_log[tok * R + hh] = tok < n_tok ? part[i] * A.scale_log2 : -INFINITY;
    }
  }
  __syncthreads();

  // ---- chunk max and sum per query head; logits become exp2(s - max) ----
  float mx[R], sm[R];
#pragma unroll
  for (int hh = 0; hh < R; ++hh) mx[hh] = -INFINITY;
  for (int tok = tid; tok < n_tok; tok += kDecodeThreads)
#pragma unroll
    for (int hh = 0; hh < R; ++hh) mx[hh] = fmaxf(mx[hh], s_log[tok * R + hh]);
#pragma unroll
  for (int hh = 0; hh < R; ++hh) {
    mx[hh] = wave_max_f(mx[hh]);
    if (lane == 0) s_red[w * R + hh] = mx[hh];
  }
  __syncthreads();
#pragma unroll
  for (int hh = 0; hh < R; ++hh) {
    float m = s_red[hh];
#pragma unroll
    for (int ww = 1; ww < kDecodeWaves; ++ww) m = fmaxf(m, s_red[ww * R + hh]);
    mx[hh] = m;
    sm[hh] = 0.0f;
  }
  for (int tok = tid; tok < n_tok; tok += kDecodeThreads)
#pragma unroll
    for (int hh = 0; hh < R; ++hh) {
      const float e = __builtin_amdgcn_exp2f(s_log[tok * R + hh] - mx[hh]);
      s_log[tok * R + hh] = e;
      sm[hh] += e;
    }
#pragma unroll
  for (int hh = 0; hh < R; ++hh) {
    sm[hh] = wave_sum_f(sm[hh]);
    if (lane == 0) s_red[(kDecodeWaves + w) * R + hh] = sm[hh];
  }
  __syncthreads();
#pragma unroll
  for (int hh = 0; hh < R; ++hh) {
    float l = 0.0f;
#pragma unroll
    for (int ww = 0; ww < kDecodeWaves; ++ww) l += s_red[(kDecodeWaves + ww) * R + hh];
    sm[hh] = l;
  }

  // ---- pass over V ----
  float acc[R][EPL];
#pragma unroll
  for (int hh = 0; hh < R; ++hh)
#pragma unroll
    for (int k = 0; k < EPL; ++k) acc[hh][k] = 0.0f;
  for (int base = w * 16; base < n_tok; base += 16 * kDecodeWaves) {
    uint4 vv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int tok = base + u * TPI + sub;
      if (tok < n_tok) {  // an empty slot may hold anything, NaN included: never touch it
        const size_t slot = (size_t)s_tab[tok / b] * b + (tok % b);
        vv[u] = *(const uint4*)(A.vc + slot * ROWB + (size_t)seg * 16);
      } else {
        vv[u] = make_uint4(0, 0, 0, 0);
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int tok = base + u * TPI + sub;
      float vf[EPL];
      Row<ESZ>::widen(vv[u], vf);
#pragma unroll
      for (int hh = 0; hh < R; ++hh) {
        const float p = tok < n_tok ? s_log[tok * R + hh] : 0.0f;
#pragma unroll
        for (int k = 0; k < EPL; ++k) acc[hh][k] = fmaf(p, vf[k], acc[hh][k]);
      }
    }
  }
  // token groups of one wavefront, then the wavefronts
#pragma unroll
  for (int m = LPT; m < 64; m <<= 1)
#pragma unroll
    for (int hh = 0; hh < R; ++hh)
#pragma unroll
      for (int k = 0; k < EPL; ++k) acc[hh][k] += __shfl_xor(acc[hh][k], m);
  if (sub == 0) {
#pragma unroll
    for (int hh = 0; hh < R; ++hh)
#pragma unroll
      for (int k = 0; k < EPL; ++k) s_acc[(w * R + hh) * HD + seg * EPL + k] = acc[hh][k];
  }
  __syncthreads();

  const bool single = nch == 1;
  for (int i = tid; i < R * HD; i += kDecodeThreads) {
    float s = 0.0f;
#pragma unroll
    for (int ww = 0; ww < kDecodeWaves; ++ww) s += s_acc[ww * R * HD + i];
    if (single) {
      const int hh = i / HD;
      float l = 0.0f;
#pragma unroll
      for (int ww = 0; ww < kDecodeWaves; ++ww) l += s_red[(kDecodeWaves + ww) * R + hh];
      A.out[(size_t)g * R * HD + i] = s / l;
    } else {
      A.part_acc[(size_t)item * R * HD + i] = s;
    }
  }
  if (!single && tid < R) {
    float m = s_red[tid];
#pragma unroll
    for (int ww = 1; ww < kDecodeWaves; ++ww) m = fmaxf(m, s_red[ww * R + tid]);
    float l = 0.0f;
#pragma unroll
    for (int ww = 0; ww < kDecodeWaves; ++ww) l += s_red[(kDecodeWaves + ww) * R + tid];
    A.part_ml[((size_t)item * R + tid) * 2 + 0] = m;
    A.part_ml[((size_t)item * R + tid) * 2 + 1] = l;
  }
  if (!A.accumulate) return;
  if (single) {
    float inv[R];
#pragma unroll
    for (int hh = 0; hh < R; ++hh) inv[hh] = 1.0f / sm[hh];
    for (int tok = tid; tok < n_tok; tok += kDecodeThreads) {
      const size_t slot = (size_t)s_tab[tok / b] * b + (tok % b);
      float inc = 0.0f;
#pragma unroll
      for (int hh = 0; hh < R; ++hh) {
        const float p = s_log[tok * R + hh] * inv[hh];
        inc += A.D.mode == KVC_L2 ? p * p : p;
      }
      A.metric[slot] += inc;
    }
  } else {
    for (int i = tid; i < n_tok * R; i += kDecodeThreads) {
      const int tok = i / R, hh = i % R;
      const size_t slot = (size_t)s_tab[tok / b] * b + (tok % b);
      A.stash[slot * R + hh] = s_log[i];
    }
  }
}

// Second kernel, heads of more than one chunk only.  Every chunk's workgroup
// rebuilds the head's max and sum from the per-chunk pairs, then adds the
// metric increments of its own tokens; the first chunk's workgroup also writes
// the combined output.
template <int R>
__global__ void __launch_bounds__(256) decode_combine_kernel(DecodeArgs A) {
  const int item = blockIdx.x;
  if (item >= A.header[HW_TOTAL_ITEMS]) return;
  const int gi = find_owner(A.chunk_off, A.gsel, item);
  const int first = A.chunk_off[gi];
  const int nch = A.chunk_off[gi + 1] - first;
  if (nch == 1) return;
  const int c = item - first;
  const int g = sel_to_g(A.D, A.l0, A.nl, gi);
  const int b = A.D.b, T = A.T, HD = A.D.d;
  const int C = A.ctx[g];
  const int t0 = c * T;
  const int n_tok = min(T, C - t0);
  __shared__ float s_m[R], s_il[R], s_w[R];
  const int tid = threadIdx.x;
  if (tid < R) {
    float m = -INFINITY;
    for (int cc = 0; cc < nch; ++cc) m = fmaxf(m, A.part_ml[((size_t)(first + cc) * R + tid) * 2]);
    float l = 0.0f;
    for (int cc = 0; cc < nch; ++cc) {
      const float* ml = A.part_ml + ((size_t)(first + cc) * R + tid) * 2;
      l += ml[1] * __builtin_amdgcn_exp2f(ml[0] - m);
    }
    s_m[tid] = m;
    s_il[tid] = 1.0f / l;
    s_w[tid] = __builtin_amdgcn_exp2f(A.part_ml[((size_t)item * R + tid) * 2] - m) / l;
  }
  __syncthreads();
  if (A.accumulate) {
    const int32_t* row = A.table + (size_t)g * A.D.maxb;
    for (int tok = tid; tok < n_tok; tok += 256) {
      const int j = t0 + tok;
      const size_t slot = (size_t)row[j / b] * b + (j % b);
      float inc = 0.0f;
#pragma unroll
      for (int hh = 0; hh < R; ++hh) {
        const float p = A.stash[slot * R + hh] * s_w[hh];
        inc += A.D.mode == KVC_L2 ? p * p : p;
      }
      A.metric[slot] += inc;
    }
  }
  if (c == 0) {
    for (int i = tid; i < R * HD; i += 256) {
      const int hh = i / HD;
      float s = 0.0f;
      for (int cc = 0; cc < nch; ++cc) {
        const float wgt = __builtin_amdgcn_exp2f(A.part_ml[((size_t)(first + cc) * R + hh) * 2] - s_m[hh]);
        s += A.part_acc[(size_t)(first + cc) * R * HD + i] * wgt;
      }
      A.out[(size_t)g * R * HD + i] = s * s_il[hh];
    }
  }
}

// Fallback for shapes the tiled kernel does not cover (any b, any d that is a
// multiple of 16 bytes, any r <= 16): one workgroup per head instance, logits
// kept in the workspace.  Correct, not fast.
__global__ void __launch_bounds__(256) decode_generic_kernel(DecodeArgs A) {
  const int gi = blockIdx.x;
  const int g = sel_to_g(A.D, A.l0, A.nl, gi);
  const int R = A.D.r, HD = A.D.d, b = A.D.b;
  const int C = A.ctx[g];
  if (C == 0) return;  // zero_empty_kernel wrote the zeros
  extern __shared__ __align__(16) char smem_raw[];
  float* s_q = (float*)smem_raw;      // [R][HD]
  float* s_red = s_q + R * HD;        // [4][16]
  float* s_ml = s_red + 4 * 16;       // [2][16]
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const bool bf = A.D.dtype == KVC_BF16;
  const size_t rowb = (size_t)HD * (bf ? 2 : 4);
  auto elem = [&](const char* base, size_t row_off, int k) -> float {
    return bf ? bf16_to_f32(((const uint16_t*)(base + row_off))[k]) : ((const float*)(base + row_off))[k];
  };
  for (int i = tid; i < R * HD; i += 256) s_q[i] = elem(A.q, ((size_t)g * R + i / HD) * rowb, i % HD);
  __syncthreads();
  const int32_t* row = A.table + (size_t)g * A.D.maxb;
  float mx[16];
  for (int hh = 0; hh < R; ++hh) mx[hh] = -INFINITY;
  for (int j = tid; j < C; j += 256) {
    const size_t slot = (size_t)row[j / b] * b + (j % b);
    for (int hh = 0; hh < R; ++hh) {
      float s = 0.0f;
      for (int k = 0; k < HD; ++k) s = fmaf(s_q[hh * HD + k], elem(A.kc, slot * rowb, k), s);
      s *= A.scale_log2;
      A.stash[slot * R + hh] = s;
      mx[hh] = fmaxf(mx[hh], s);
    }
  }
  for (int hh = 0; hh < R; ++hh) {
    const float m = wave_max_f(mx[hh]);
    if (lane == 0) s_red[w * 16 + hh] = m;
  }
  __syncthreads();
  if (tid < R) s_ml[tid] = fmaxf(fmaxf(s_red[tid], s_red[16 + tid]), fmaxf(s_red[32 + tid], s_red[48 + tid]));
  __syncthreads();
  float sm[16];
  for (int hh = 0; hh < R; ++hh) sm[hh] = 0.0f;
  for (int j = tid; j < C; j += 256) {
    const size_t slot = (size_t)row[j / b] * b + (j % b);
    for (int hh = 0; hh < R; ++hh) {
      const float e = __builtin_amdgcn_exp2f(A.stash[slot * R + hh] - s_ml[hh]);
      A.stash[slot * R + hh] = e;
      sm[hh] += e;
    }
  }
  for (int hh = 0; hh < R; ++hh) {
    const float t = wave_sum_f(sm[hh]);
    if (lane == 0) s_red[w * 16 + hh] = t;
  }
  __syncthreads();
  if (tid < R) s_ml[16 + tid] = 1.0f / (s_red[tid] + s_red[16 + tid] + s_red[32 + tid] + s_red[48 + tid]);
  __syncthreads();  // also orders the stash writes above before the reads below
  for (int i = tid; i < R * HD; i += 256) {
    const int hh = i / HD, k = i % HD;
    float s = 0.0f;
    for (int j = 0; j < C; ++j) {
      const size_t slot = (size_t)row[j / b] * b + (j % b);
      s = fmaf(A.stash[slot * R + hh], elem(A.vc, slot * rowb, k), s);
    }
    A.out[(size_t)g * R * HD + i] = s * s_ml[16 + hh];
  }
  if (A.accumulate) {
    for (int j = tid; j < C; j += 256) {
      const size_t slot = (size_t)row[j / b] * b + (j % b);
      float inc = 0.0f;
      for (int hh = 0; hh < R; ++hh) {
        const float p = A.stash[slot * R + hh] * s_ml[16 + hh];
        inc += A.D.mode == KVC_L2 ? p * p : p;
      }
      A.metric[slot] += inc;
    }
  }
}

template <int ESZ, int HD, int R>
static int launch_tiled(const DecodeArgs& A, int grid, size_t lds, hipStream_t s) {
  auto kern = decode_chunk_kernel<ESZ, HD, R>;
  ProfilePair* pp = (g_prof && g_prof_used < g_prof_cap) ? &g_prof[g_prof_used++] : nullptr;
  if (pp) KVC_HIP(hipEventRecord(pp->a0, s));
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kDecodeThreads), lds, s, A);
  KVC_LAUNCH_CHECK();
  if (pp) { KVC_HIP(hipEventRecord(pp->a1, s)); KVC_HIP(hipEventRecord(pp->b0, s)); }
  hipLaunchKernelGGL(decode_combine_kernel<R>, dim3(grid), dim3(256), 0, s, A);
  KVC_LAUNCH_CHECK();
  if (pp) KVC_HIP(hipEventRecord(pp->b1, s));
  return KVC_OK;
}

template <int ESZ, int HD>
static int launch_tiled_r(const DecodeArgs& A, int grid, size_t lds, hipStream_t s) {
  switch (A.D.r) {
    case 1: return launch_tiled<ESZ, HD, 1>(A, grid, lds, s);
    case 2: return launch_tiled<ESZ, HD, 2>(A, grid, lds, s);
    case 4: return launch_tiled<ESZ, HD, 4>(A, grid, lds, s);
    case 8: return launch_tiled<ESZ, HD, 8>(A, grid, lds, s);
  }
  return KVC_ERR_UNSUPPORTED;
}

constexpr size_t kLdsLimit = 64 * 1024;

}  // namespace kvc

using namespace kvc;

extern "C" {

int kvc_profile_begin(int n) {
  if (n < 0 || n > 4096) return KVC_ERR_ARG;
  if (g_prof) {
    for (int i = 0; i < g_prof_cap; ++i) {
      hipEventDestroy(g_prof[i].a0); hipEventDestroy(g_prof[i].a1);
      hipEventDestroy(g_prof[i].b0); hipEventDestroy(g_prof[i].b1);
    }
    delete[] g_prof;
    g_prof = nullptr;
  }
  g_prof_cap = g_prof_used = 0;
  if (n == 0) return KVC_OK;
  g_prof = new ProfilePair[n];
  for (int i = 0; i < n; ++i) {
    KVC_HIP(hipEventCreate(&g_prof[i].a0)); KVC_HIP(hipEventCreate(&g_prof[i].a1));
    KVC_HIP(hipEventCreate(&g_prof[i].b0)); KVC_HIP(hipEventCreate(&g_prof[i].b1));
  }
  g_prof_cap = n;
  return KVC_OK;
}

int kvc_profile_collect(float* chunk_ms, float* combine_ms, int cap, int* count) {
  if (!count || cap < 0) return KVC_ERR_ARG;
  *count = g_prof_used;
  for (int i = 0; i < g_prof_used && i < cap; ++i) {
    KVC_HIP(hipEventSynchronize(g_prof[i].b1));
    float ms = 0.0f;
    if (chunk_ms) { KVC_HIP(hipEventElapsedTime(&ms, g_prof[i].a0, g_prof[i].a1)); chunk_ms[i] = ms; }
    if (combine_ms) { KVC_HIP(hipEventElapsedTime(&ms, g_prof[i].b0, g_prof[i].b1)); combine_ms[i] = ms; }
  }
  return KVC_OK;
}

int kvc_set_decode_chunk(int tokens) {
  if (tokens != 0 && (tokens < kMinChunk || tokens > kMaxChunk || tokens % 64 != 0)) return KVC_ERR_ARG;
  g_chunk_tokens = tokens;
  return KVC_OK;
}

int kvc_paged_decode(const kvc_config* cfg, const kvc_state* st, const void* q, float* out,
                     int layer_begin, int layer_end, int accumulate_metric, void* ws, void* stream) {
  int rc = validate(cfg, st);
  if (rc != KVC_OK) return rc;
  if (!q || !out || !ws || ((uintptr_t)ws & 255)) return KVC_ERR_ARG;
  if (((uintptr_t)q & 15) || ((uintptr_t)out & 15)) return KVC_ERR_ARG;
  Dims D = dims_of(cfg);
  if (layer_begin < 0 || layer_end > D.Lyr || layer_begin >= layer_end) return KVC_ERR_ARG;
  Workspace W = carve(D, ws);
  hipStream_t s = (hipStream_t)stream;

  DecodeArgs A;
  A.D = D;
  A.kc = (const char*)st->k_cache; A.vc = (const char*)st->v_cache;
  A.metric = st->metric; A.table = st->block_table; A.ctx = st->ctx_len;
  A.q = (const char*)q; A.out = out;
  A.l0 = layer_begin; A.nl = layer_end - layer_begin; A.gsel = D.S * A.nl * D.Hk;
  A.accumulate = accumulate_metric != 0;
  A.chunk_off = W.off_a; A.part_ml = W.part_ml; A.part_acc = W.part_acc; A.stash = W.stash;
  A.header = W.header;
  A.scale_log2 = (float)(1.4426950408889634 / sqrt((double)D.d));

  const int esz = D.dtype == KVC_BF16 ? 2 : 4;
  const int lpt = D.d * esz / 16;
  const int tpi = lpt <= 64 ? 64 / lpt : 0;
  bool tiled = (D.r == 1 || D.r == 2 || D.r == 4 || D.r == 8) && (D.d == 64 || D.d == 128) &&
               tpi >= 1 && D.b % tpi == 0 && 64 % D.b == 0;
  int T = 0;
  size_t lds = 0;
  if (tiled) {
    T = g_chunk_tokens ? g_chunk_tokens : (D.r >= 8 ? 1024 : 2048);
    while (T > kMinChunk && decode_lds_bytes(T, D.r, D.d, D.b) > kLdsLimit) T /= 2;
    lds = decode_lds_bytes(T, D.r, D.d, D.b);
    if (lds > kLdsLimit) tiled = false;
  }
  A.T = tiled ? T : (1 << 30);  // generic path: one "chunk" per head

  hipLaunchKernelGGL(zero_empty_kernel, dim3((A.gsel + 3) / 4), dim3(256), 0, s, A);
  KVC_LAUNCH_CHECK();
  if (!tiled) {
    const size_t gl = ((size_t)D.r * D.d + 4 * 16 + 2 * 16) * 4;
    hipLaunchKernelGGL(decode_generic_kernel, dim3(A.gsel), dim3(256), gl, s, A);
    KVC_LAUNCH_CHECK();
    return KVC_OK;
  }
  rc = device_exclusive_scan(ChunkFn{st->ctx_len, D, A.l0, A.nl, T}, A.gsel, W.tile_sums, W.off_a,
                             W.header + HW_TOTAL_ITEMS, s);
  if (rc != KVC_OK) return rc;
  // items <= (slots in the pool) / T + heads, and <= heads * chunks a full row can hold
  const size_t bound_pool = (size_t)D.N * D.b / T + (size_t)A.gsel;
  const size_t bound_row = (size_t)A.gsel * (((size_t)D.maxb * D.b + T - 1) / T);
  const size_t grid = bound_pool < bound_row ? bound_pool : bound_row;
  if (grid > 0x7fffffffull) return KVC_ERR_UNSUPPORTED;
  if (esz == 2) return D.d == 64 ? launch_tiled_r<2, 64>(A, (int)grid, lds, s) : launch_tiled_r<2, 128>(A, (int)grid, lds, s);
  return D.d == 64 ? launch_tiled_r<4, 64>(A, (int)grid, lds, s) : launch_tiled_r<4, 128>(A, (int)grid, lds, s);
}

}  // extern "C"
