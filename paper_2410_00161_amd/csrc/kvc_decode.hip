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
#include <algorithm>
#include <atomic>
#include <cmath>
#include <mutex>

#include "kvc_common.h"
#include "kvc_worklist.h"

namespace kvc {

// Host-side state of the process: the chunk-length knob (read once per call), what the runtime
// has been told about the chunk kernels' LDS, and the benchmark's event recording behind one lock.
static std::atomic<int> g_chunk_tokens{0};  // 0 = default; set by kvc_set_decode_chunk

// optional event pairs around the decode kernels (kvc_profile_begin / _collect)
struct ProfilePair { hipEvent_t a0, a1, s0, s1, b0, b1; };  // long-item, short-item, combine launches
static std::mutex g_prof_lock;
static ProfilePair* g_prof = nullptr;
static int g_prof_cap = 0, g_prof_used = 0, g_prof_on = 1;
static std::atomic<bool> g_prof_any{false};   // recording asked for: only then a call takes the lock

static ProfilePair* claim_profile_pair() {
  if (!g_prof_any.load(std::memory_order_acquire)) return nullptr;
  std::lock_guard<std::mutex> hold(g_prof_lock);
  return (g_prof && g_prof_on && g_prof_used < g_prof_cap) ? &g_prof[g_prof_used++] : nullptr;
}

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef short i16x4_t __attribute__((ext_vector_type(4)));

template <int ESZ> struct Row;
// P: the piece of a K or V row one lane loads (PB bytes, EPL elements); Q: the query elements
// that face it; QSZ: bytes of a query element.
template <> struct Row<2> {  // bf16: 8 elements in 16 bytes
  static constexpr int EPL = 8;
  static constexpr int QSZ = 2;
  static constexpr int PB = 16;
  typedef uint4 P;
  typedef uint4 Q;
  static __device__ __forceinline__ P load(const void* p) { return load_stream16(p); }
  static __device__ __forceinline__ P zero() { return make_uint4(0, 0, 0, 0); }
  static __device__ __forceinline__ Q load_q(const char* qrow, int seg) { return *(const uint4*)(qrow + (size_t)seg * 16); }
  static __device__ __forceinline__ float dot(const uint4& a, const uint4& b) {
    float s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.x), __builtin_bit_cast(bf16x2_t, b.x), 0.0f, false);
    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.y), __builtin_bit_cast(bf16x2_t, b.y), s, false);
    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.z), __builtin_bit_cast(bf16x2_t, b.z), s, false);
    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.w), __builtin_bit_cast(bf16x2_t, b.w), s, false);
    return s;
  }
  static __device__ __forceinline__ uint4 as_bf16x8(const uint4& a) { return a; }
  static __device__ __forceinline__ void widen(const uint4& a, float* f) {
    f[0] = bf16_lo(a.x); f[1] = bf16_hi(a.x); f[2] = bf16_lo(a.y); f[3] = bf16_hi(a.y);
    f[4] = bf16_lo(a.z); f[5] = bf16_hi(a.z); f[6] = bf16_lo(a.w); f[7] = bf16_hi(a.w);
  }
};
template <> struct Row<4> {  // f32: 4 elements in 16 bytes
  static constexpr int EPL = 4;
  static constexpr int QSZ = 4;
  static constexpr int PB = 16;
  typedef uint4 P;
  typedef uint4 Q;
  static __device__ __forceinline__ P load(const void* p) { return load_stream16(p); }
  static __device__ __forceinline__ P zero() { return make_uint4(0, 0, 0, 0); }
  static __device__ __forceinline__ Q load_q(const char* qrow, int seg) { return *(const uint4*)(qrow + (size_t)seg * 16); }
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

typedef float f32x2_t __attribute__((ext_vector_type(2)));
template <> struct Row<1> {  // OCP e4m3: 8 elements in 8 bytes, facing 8 bf16 query elements
  // Pieces of 8 bytes, not 16: a d = 128 row is then spread over 16 lanes as for bf16, and the
  // output accumulator of a lane (r x EPL floats) stays at the size the registers hold.
  static constexpr int EPL = 8;
  static constexpr int QSZ = 2;
  static constexpr int PB = 8;
  typedef uint2 P;
  typedef uint4 Q;
  static __device__ __forceinline__ P load(const void* p) { return load_stream8(p); }
  static __device__ __forceinline__ P zero() { return make_uint2(0, 0); }
  static __device__ __forceinline__ Q load_q(const char* qrow, int seg) { return *(const uint4*)(qrow + (size_t)seg * 16); }
  // four 8-bit floats -> two packed bf16 pairs (exact: 3 mantissa bits fit in 7; one instruction
  // per pair, scale 1), then the same packed dot product as for a bf16 cache
  static __device__ __forceinline__ float dot4(uint32_t k, uint32_t q01, uint32_t q23, float s) {
    const bf16x2_t p01 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(k, 1.0f, false);
    const bf16x2_t p23 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(k, 1.0f, true);
    s = __builtin_amdgcn_fdot2_f32_bf16(p01, __builtin_bit_cast(bf16x2_t, q01), s, false);
    return __builtin_amdgcn_fdot2_f32_bf16(p23, __builtin_bit_cast(bf16x2_t, q23), s, false);
  }
  static __device__ __forceinline__ uint4 as_bf16x8(const uint2& a) {
    return make_uint4(__builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(a.x, 1.0f, false)),
                      __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(a.x, 1.0f, true)),
                      __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(a.y, 1.0f, false)),
                      __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(a.y, 1.0f, true)));
  }
  static __device__ __forceinline__ float dot(const uint2& a, const Q& q) {
    return dot4(a.y, q.z, q.w, dot4(a.x, q.x, q.y, 0.0f));
  }
  static __device__ __forceinline__ void widen(const uint2& a, float* f) {
    const uint32_t w[2] = {a.x, a.y};
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const f32x2_t lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[i], false);
      const f32x2_t hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[i], true);
      f[4 * i] = lo.x; f[4 * i + 1] = lo.y; f[4 * i + 2] = hi.x; f[4 * i + 3] = hi.y;
    }
  }
};

// A head of more than one chunk leaves, for every KV and query head, e = exp2(logit - chunk
// max) in [0, 1] for the combine kernel.  It is kept as 16-bit fixed point: the error of e, and
// so of the probability it turns into (p = e * weight, weight <= 1), is at most 2^-17, which
// moves a metric increment (sum over r heads of p^2 or p) by at most r * 2^-16.
__device__ __forceinline__ uint32_t q16(float e) { return (uint32_t)(e * 65535.0f + 0.5f); }
__device__ __forceinline__ float unq16(uint32_t q) { return (float)q * (1.0f / 65535.0f); }

template <int R>
__device__ __forceinline__ void stash_store(float* stash, size_t slot, const float* e) {
  uint16_t* base = (uint16_t*)stash + slot * R;
  if constexpr (R == 1) {
    *base = (uint16_t)q16(e[0]);
  } else {
    uint32_t wds[R / 2];
#pragma unroll
    for (int i = 0; i < R / 2; ++i) wds[i] = q16(e[2 * i]) | (q16(e[2 * i + 1]) << 16);
    if constexpr (R == 2) __builtin_nontemporal_store(wds[0], (uint32_t*)base);
    else if constexpr (R == 4) { typedef unsigned int u2 __attribute__((ext_vector_type(2))); u2 t = {wds[0], wds[1]}; __builtin_nontemporal_store(t, (u2*)base); }
    else { typedef unsigned int u4 __attribute__((ext_vector_type(4))); u4 t = {wds[0], wds[1], wds[2], wds[3]}; __builtin_nontemporal_store(t, (u4*)base); }
  }
}
template <int R>
__device__ __forceinline__ void stash_load(const float* stash, size_t slot, float* e) {
  const uint16_t* base = (const uint16_t*)stash + slot * R;
  if constexpr (R == 1) {
    e[0] = unq16(*base);
  } else {
    uint32_t wds[R / 2];
    if constexpr (R == 2) wds[0] = __builtin_nontemporal_load((const uint32_t*)base);
    else if constexpr (R == 4) { typedef unsigned int u2 __attribute__((ext_vector_type(2))); const u2 t = __builtin_nontemporal_load((const u2*)base); wds[0] = t.x; wds[1] = t.y; }
    else { const uint4 t = load_stream16(base); wds[0] = t.x; wds[1] = t.y; wds[2] = t.z; wds[3] = t.w; }
#pragma unroll
    for (int i = 0; i < R / 2; ++i) { e[2 * i] = unq16(wds[i] & 0xffffu); e[2 * i + 1] = unq16(wds[i] >> 16); }
  }
}

constexpr int kDecodeThreads = 256;
constexpr int kDecodeWaves = kDecodeThreads / 64;

// A shape takes Q K^T to the matrix cores where the plain ALUs are the bound: 16-bit or 8-bit
// rows (the latter widened to bf16 on their way into the operand tile) with eight query heads per
// KV head, 8-bit rows with four (half the bytes per logit: with the dot products on the plain ALUs
// that launch ran 8 % longer), d = 128, blocks of a multiple of 16 tokens.
__host__ __device__ constexpr bool decode_uses_mfma(int esz, int R, int HD, int b) {
  return esz <= 2 && (R == 8 || (R == 4 && esz == 1)) && HD == 128 && b % 16 == 0;
}

// P V goes to the matrix cores wherever Q K^T does.
__host__ __device__ constexpr bool decode_pv_mfma(int esz, int R, int HD, int b) {
  return decode_uses_mfma(esz, R, HD, b);
}

// Register buffers of K and V groups a wavefront rotates through (one less is in flight behind
// the group being worked on): three for rows of at most 16 bits when four wavefronts share a
// long chunk (up to four query heads, or the matrix-core shapes), else two.
__host__ __device__ constexpr int decode_depth(int esz, int R, int HD, bool b16, int nw) {
  if (nw != 4 || esz > 2) return 2;
  return (R <= 4 || (b16 && decode_uses_mfma(esz, R, HD, 16))) ? 3 : 2;
}

__host__ __device__ inline size_t decode_lds_bytes(int T, int R, int HD, int b, int waves = kDecodeWaves,
                                                   bool mfma = false) {
  // per-wavefront un-normalised output; on the matrix-core path the same bytes serve, while
  // the main loop runs, as the wavefront's operand tile (16 tokens of d 16-bit elements)
  const size_t per_wave_out = mfma ? (size_t)16 * HD * 2 : (size_t)R * HD * 4;
  return (size_t)T * R * 2                       // exp of every logit against its group's running max, 16-bit
         + (size_t)(T / 16) * R * 4              // that running max, per 16-token group and head
         + (size_t)waves * per_wave_out
         + (size_t)waves * 16 * R * 4            // per-wavefront exp of the current group, f32
         + 2 * waves * R * 4                     // per-wavefront max and sum
         + ((size_t)T / b + 1) * 4;              // block ids of the chunk
}

// One workgroup = one chunk of up to T tokens of one head instance; one pass.
//
// Each wavefront walks its 16-token groups with the next group's K and V rows
// already in flight.  Per group: r dot products per token (butterfly over the
// lanes of a token), running max per query head (online softmax), exp of the
// group against the running max, rescale of the output accumulator when a max
// moved, then acc += p * v.  What the metric needs later, the exp of every
// logit, stays in LDS as 16-bit fixed point next to the running max it was
// taken against (one f32 per group and head): once the wavefronts have been
// merged, the normalised probability of every KV follows without touching K
// again.  The quantisation moves a probability by at most 2^-17.
//
// NW = 4 wavefronts share a chunk.  The short items at the end of the work list (at most
// A.Ts tokens) are latency-bound, a chain of dependent loads (item, block table, K and V) in
// front of a few groups of arithmetic: they get a launch of their own with NW = 1, small LDS
// and fewer registers, so that a CU holds many of those chains at once.
template <int ESZ, int HD, int R, bool B16, int NW>
__global__ void __launch_bounds__(NW * 64) decode_chunk_kernel(DecodeArgs A) {
  constexpr int NT = NW * 64;
  constexpr int DEPTH = decode_depth(ESZ, R, HD, B16, NW);
  constexpr int EPL = Row<ESZ>::EPL;
  constexpr int PB = Row<ESZ>::PB;     // bytes a lane loads at once
  typedef typename Row<ESZ>::P Piece;
  constexpr int LPT = HD / EPL;        // lanes per token
  constexpr int TPI = 64 / LPT;        // tokens per wavefront load
  constexpr int U = 16 / TPI;          // loads per 16-token group
  constexpr int NV = R * U;            // partial logits per lane before the butterfly
  constexpr int PER = NV >= LPT ? NV / LPT : 1;  // logits per lane after it
  constexpr size_t ROWB = (size_t)HD * ESZ;
  constexpr size_t QROWB = (size_t)HD * Row<ESZ>::QSZ;
  static_assert(LPT >= 4 && LPT <= 32 && (16 % TPI) == 0, "row geometry");
  // Q K^T of a 16-token group on the matrix cores (v_mfma_f32_16x16x32_bf16: rows = query heads,
  // columns = tokens, four steps of 32 dimensions).  K still arrives by contiguous 1 KiB loads
  // (a load shaped like the operand is 12 % slower); a wavefront turns its tile into operand
  // order through 4 KiB of LDS, cells XOR-swizzled so that neither side has a bank conflict.
  // Head h sits in operand row 4 (h % 4) + h / 4, which leaves lane 16 a + t with the logits of
  // token t against heads a and a + 4.
  constexpr bool MF = B16 && decode_uses_mfma(ESZ, R, HD, 16);
  constexpr bool PVM = B16 && decode_pv_mfma(ESZ, R, HD, 16);   // P V on the matrix cores (with or without Q K^T)
  constexpr int RW = PVM ? 8 : R;      // output rows a wavefront's LDS region has room for
  constexpr int NVH = (R + 3) / 4;     // MF: logits per lane
  constexpr int OWN = MF ? NVH : PER;

  const int tid = threadIdx.x, lane = tid & 63, w = NW == 1 ? 0 : tid >> 6;
  const int total_items = A.header[HW_TOTAL_ITEMS];
  const int short_items = A.header[HW_SHORT_ITEMS];
  if (NW == 4 && blockIdx.x == 0 && tid < HW_DEC_END - HW_DEC_BINS) A.header[HW_DEC_BINS + tid] = 0;  // work-list block back to zero
  if (NW == 4 && A.plan && (int)blockIdx.x < A.gsel) {
    // a list kept from kvc_decode_plan was made without the output at hand: the zero rows of a
    // head that holds no KV are written here, by the workgroup with the head's index
    const int ge = sel_to_g(A.D, A.l0, A.nl, blockIdx.x);
    if (A.ctx[ge] == 0)
      for (int i = tid; i < R * HD; i += NT) A.out[(size_t)ge * R * HD + i] = 0.0f;
  }
  if (total_items > A.cap || short_items < 0 || short_items > total_items) return;
  const int n_long = total_items - short_items;
  if ((int)blockIdx.x >= (NW == 4 ? n_long : short_items)) return;
  const int item = NW == 4 ? blockIdx.x : n_long + blockIdx.x;   // the short items end the list
  const DecodeItem it = A.items[item];
  const int g = it.g, t0 = it.t0, n_tok = it.n_tok, nch = it.nch;
  const int T = NW == 4 ? A.T : A.Ts;    // tokens this launch sizes its LDS arrays for
  const int Tc = A.header[HW_CHUNK_T];   // tokens the work list was cut at (<= A.T)
  if ((unsigned)g >= (unsigned)A.D.G || n_tok <= 0 || n_tok > T || t0 < 0 || nch <= 0 || Tc < 64 || Tc > A.T ||
      (nch > 1 && (it.pbase < 0 || it.pbase + nch > A.cap)))
    return;  // not a record this call wrote
  if (A.plan) {
    // the head must still be as long as the plan took it to be (the record carries that length).
    // A stale plan is an argument error, found here and left in the status word.
    if (A.ctx[g] != it.pad[0]) {
      if (tid == 0 && A.status[HW_STATUS] == KVC_OK) A.status[HW_STATUS] = KVC_ERR_ARG;
      return;
    }
  }
  const int b = A.D.b, lb = A.log2b;

  extern __shared__ __align__(16) char smem_raw[];
  uint4* s_kt = (uint4*)smem_raw;                      // MF: [waves][16 tokens][16 cells of 16 bytes]
  // [waves][R][HD]; on the matrix-core path a wavefront's 4 KiB of it are its operand tile until
  // its main loop ends (R * HD * 4 = 16 * HD * 2 there, so no wavefront touches another's tile)
  float* s_acc = (float*)smem_raw;
  static_assert(!PVM || (size_t)RW * HD * 4 == (size_t)16 * HD * 2, "output rows alias the operand tile wavefront by wavefront");
  float* s_e = s_acc + NW * RW * HD;         // [waves][16][R]
  float* s_red = s_e + NW * 16 * R;          // [2][waves][R]
  float* s_gm = s_red + 2 * NW * R;          // [T / 16][R]
  uint16_t* s_q = (uint16_t*)(s_gm + (T / 16) * R);    // [T][R]
  int* s_tab = (int*)(s_q + (size_t)T * R);            // [T / b + 1]

  const int sub = lane / LPT, seg = lane % LPT;

  {
    const int nblk = (n_tok + b - 1) >> lb;
    const int32_t* row = A.table + (size_t)g * A.D.maxb + (t0 >> lb);
    for (int i = tid; i < nblk; i += NT) s_tab[i] = row[i];
  }
  // VALU path: every head's q at this lane's dimensions.  MFMA path: A operand of step st: lane =
  // (row lane % 16, dimensions 32 st + 8 (lane / 16) .. + 8); rows without a head are zero.
  typename Row<ESZ>::Q qv[MF ? U : R];
  if constexpr (MF) {
    const int arow = lane & 15, ahead = (arow >> 2) + 4 * (arow & 3);
#pragma unroll
    for (int st = 0; st < U; ++st) {
      // (rows without a head read the last head and are zeroed: a select between values)
      const uint4 t = *(const uint4*)(A.q + ((size_t)g * R + min(ahead, R - 1)) * QROWB + (size_t)st * 64 + (size_t)(lane >> 4) * 16);
      qv[st] = ahead < R ? t : make_uint4(0, 0, 0, 0);
    }
  } else {
#pragma unroll
    for (int hh = 0; hh < R; ++hh) qv[hh] = Row<ESZ>::load_q(A.q + ((size_t)g * R + hh) * QROWB, seg);
  }
  __syncthreads();

  // One 16-token group = U wavefront loads of 64 pieces each (1 KiB; 512 bytes for 8-bit
  // rows).  With b a multiple of 16 a group lies in one block, so one table lookup serves it
  // and the slots past the end of the head (still inside the block) are masked later, read or not.
  // Otherwise every load looks its block up and tokens past the end re-read the last token.
  const int last = n_tok - 1;
  auto load_group = [&](const char* __restrict__ basep, int grp, Piece (&buf)[U]) {
    if constexpr (B16) {
      const int tk = grp * 16;
      const size_t slot = ((size_t)s_tab[tk >> lb] << lb) + (tk & (b - 1));
      const char* p = basep + slot * ROWB + (size_t)lane * PB;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        // A short item's last block is half empty on average, 7 % of what the item reads: the
        // one-wavefront launch leaves the slots past the head's end unread.  (In the long items'
        // loop the test costs more than the few rows it saves.)
        if (NW == 1 && tk + u * TPI + sub >= n_tok) buf[u] = Row<ESZ>::zero();
        else buf[u] = Row<ESZ>::load(p + (size_t)u * (64 * PB));
      }
    } else {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int tok = min(grp * 16 + u * TPI + sub, last);
        const size_t slot = ((size_t)s_tab[tok >> lb] << lb) + (tok & (b - 1));
        buf[u] = Row<ESZ>::load(basep + slot * ROWB + (size_t)seg * PB);
      }
    }
  };
  const int ngroups = (n_tok + 15) >> 4;

  float acc[R][EPL];         // VALU path: un-normalised output, this lane's dimensions and tokens
#pragma unroll
  for (int hh = 0; hh < R; ++hh)
#pragma unroll
    for (int k = 0; k < EPL; ++k) acc[hh][k] = 0.0f;
  // MFMA path: P V as v_mfma_f32_16x16x16_bf16 per 16 dimensions (rows = heads, columns =
  // dimensions, k = the 16 tokens of a group).  A probability goes in as two bf16 halves,
  // hi = its upper 16 bits in row h, lo = (p - hi) in row h + 8, so that the product carries
  // 16 bits of p (one half alone misses the output tolerance when one key dominates).
  constexpr int NDT = HD / 16;
  static_assert(!PVM || R == 8 || R == 4, "operand rows: heads 0..7 as upper halves, then as remainders");
  f32x4_t pacc[PVM ? NDT : 1];
#pragma unroll
  for (int i = 0; i < (PVM ? NDT : 1); ++i) pacc[i] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
  float m_run[R];            // running max per query head, the same in every lane
  float m_own[OWN], l_own[OWN];  // this lane's head(s): running max and partial sum
#pragma unroll
  for (int hh = 0; hh < R; ++hh) m_run[hh] = -INFINITY;
#pragma unroll
  for (int i = 0; i < OWN; ++i) { m_own[i] = -INFINITY; l_own[i] = 0.0f; }
  const int idx0 = (seg * NV) / LPT;
  float* my_e = s_e + w * 16 * R;
  const bool gm_writer = (lane & 60) == 0;  // lanes 0..3 hold every head between them

  auto process = [&](Piece (&kcur)[U], Piece (&vcur)[U], int grp) {
      float m_new[R];
      bool moved = false;
      if constexpr (MF) {
        // this wavefront's K tile into operand order: cell (token, 16-byte piece c) sits at
        // position c ^ token of the token's row
        uint4* kt = s_kt + w * 256;
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int t = u * TPI + sub;
          kt[t * 16 + (seg ^ t)] = Row<ESZ>::as_bf16x8(kcur[u]);
        }
        const int tl = lane & 15, hrow = lane >> 4;
        f32x4_t sacc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int st = 0; st < U; ++st) {
          const uint4 kb = kt[tl * 16 + ((4 * st + hrow) ^ tl)];
          sacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, qv[st]),
                                                         __builtin_bit_cast(bf16x8_t, kb), sacc, 0, 0, 0);
        }
        const bool live = grp * 16 + tl < n_tok;
        float x[NVH], gm[NVH], e[NVH];
#pragma unroll
        for (int v = 0; v < NVH; ++v) {
          x[v] = live ? sacc[v] * A.scale_log2 : -INFINITY;
          float m = x[v];   // max over the 16 tokens = over the 16 lanes of this row of lanes
          m = fmaxf(m, lane_xor<1>(m));
          m = fmaxf(m, lane_xor<2>(m));
          m = fmaxf(m, lane_xor<4>(m));
          m = fmaxf(m, lane_xor<8>(m));
          gm[v] = fmaxf(m, m_own[v]);
        }
#pragma unroll
        for (int v = 0; v < NVH; ++v) {
          e[v] = __builtin_amdgcn_exp2f(x[v] - gm[v]);
          l_own[v] = l_own[v] * __builtin_amdgcn_exp2f(m_own[v] - gm[v]) + e[v];
          m_own[v] = gm[v];
        }
#pragma unroll
        for (int v = 0; v < NVH; ++v) {
          const int hh = hrow + 4 * v;
          if (hh < R) {
            my_e[hh * 16 + tl] = e[v];      // [head][token] here: the P V operand reads four tokens of a head
            s_q[(grp * 16 + tl) * R + hh] = (uint16_t)q16(e[v]);
            if (tl == 0) s_gm[grp * R + hh] = gm[v];
          }
        }
#pragma unroll
        for (int hh = 0; hh < R; ++hh) {
          m_new[hh] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, gm[hh / 4]), 16 * (hh % 4)));
          moved |= m_new[hh] > m_run[hh];
        }
      } else {
        // logits of the group
        float part[NV];
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
          for (int hh = 0; hh < R; ++hh) part[u * R + hh] = Row<ESZ>::dot(kcur[u], qv[hh]);
        Butterfly<NV, LPT / 2>::run(part, lane);
        float gm[PER];
#pragma unroll
        for (int i = 0; i < PER; ++i) {
          const int u = (idx0 + i) / R;
          const int tok = grp * 16 + u * TPI + sub;
          part[i] = tok < n_tok ? part[i] * A.scale_log2 : -INFINITY;
          // max over the group's tokens: the lanes that hold one head differ in lane bits 2..5
          float m = part[i];
          m = fmaxf(m, lane_xor<4>(m));
          m = fmaxf(m, lane_xor<8>(m));
          m = fmaxf(m, __shfl_xor(m, 16));
          m = fmaxf(m, __shfl_xor(m, 32));
          gm[i] = fmaxf(m, m_own[i]);
        }
        // exp of the group against the new running max; partial sums rescaled
#pragma unroll
        for (int i = 0; i < PER; ++i) {
          const int idx = idx0 + i;
          const int u = idx / R, hh = idx % R;
          const int tl = u * TPI + sub;
          const float e = __builtin_amdgcn_exp2f(part[i] - gm[i]);
          l_own[i] = l_own[i] * __builtin_amdgcn_exp2f(m_own[i] - gm[i]) + e;
          m_own[i] = gm[i];
          my_e[PVM ? hh * 16 + tl : tl * R + hh] = e;   // [head][token] for the matrix-core P V
          s_q[(grp * 16 + tl) * R + hh] = (uint16_t)q16(e);
          if (gm_writer) s_gm[grp * R + hh] = gm[i];
        }
        // new running max of every head, read from the lane that owns it
#pragma unroll
        for (int hh = 0; hh < R; ++hh) {
          m_new[hh] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, gm[hh % PER]), (hh * 4) / R));
          moved |= m_new[hh] > m_run[hh];
        }
      }
      const bool tail = B16 && grp * 16 + 16 > n_tok;
      if constexpr (PVM) {
        if (moved) {
          // this lane's product rows 4 (lane / 16) + v belong to heads 4 ((lane / 16) % 2) + v
          const bool upper = (lane & 16) != 0;
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const float a_lo = __builtin_amdgcn_exp2f(m_run[v] - m_new[v]);
            const float a_hi = R > 4 ? __builtin_amdgcn_exp2f(m_run[(4 + v) % R] - m_new[(4 + v) % R]) : 1.0f;
            const float a = upper ? a_hi : a_lo;
#pragma unroll
            for (int dt = 0; dt < NDT; ++dt) pacc[dt][v] *= a;
          }
#pragma unroll
          for (int hh = 0; hh < R; ++hh) m_run[hh] = m_new[hh];
        }
        // The K tile (if Q K^T went through it) has been consumed: its 4 KiB take the V tile, row-major [token][d] in
        // bf16, the 16-byte cell c of token t at position c ^ 2 (t % 8) of the row, which keeps
        // the transposing reads below (8 tokens x 32 bytes per half wavefront) off each other's banks.
        uint4* vt = s_kt + w * 256;
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int t = u * TPI + sub;
          const bool dead = tail && grp * 16 + t >= n_tok;   // empty slot: may hold anything
          vt[t * 16 + (seg ^ (2 * (t & 7)))] = Row<ESZ>::as_bf16x8(dead ? Row<ESZ>::zero() : vcur[u]);
        }
        // A operand: lane = (row lane % 16, tokens 4 (lane / 16) .. + 3)
        const int rho = lane & 15, kap = lane >> 4;
        float4 pe = *(const float4*)(my_e + (rho & (R - 1)) * 16 + 4 * kap);
        if (R < 8 && (rho & 7) >= R) pe = make_float4(0.0f, 0.0f, 0.0f, 0.0f);   // operand rows without a head
        const bool hi_row = rho < 8;
        auto half_of = [&](float p) {   // the float whose upper 16 bits are this row's half of p
          const uint32_t bits = __float_as_uint(p);
          const float lo = p - __uint_as_float(bits & 0xffff0000u);   // exact
          return hi_row ? bits : __float_as_uint(lo);
        };
        const uint32_t hb0 = half_of(pe.x), hb1 = half_of(pe.y), hb2 = half_of(pe.z), hb3 = half_of(pe.w);
        const uint2 apack = make_uint2(__builtin_amdgcn_perm(hb1, hb0, 0x07060302u),
                                       __builtin_amdgcn_perm(hb3, hb2, 0x07060302u));
        const i16x4_t aop = __builtin_bit_cast(i16x4_t, apack);
        // B operand of dimension tile dt: lane = (column lane % 16, tokens 4 (lane / 16) .. + 3).
        // The transposing read delivers it when lane j of a group of 16 points at token
        // 4 (lane / 16) + j / 4, dimensions 16 dt + 4 (j % 4) .. + 3.
        const int tt = 4 * kap + (rho >> 2);
        const char* vrow = (const char*)vt + tt * 256 + 8 * (rho & 1);
        const int csw = 2 * (tt & 7), chalf = (rho & 3) >> 1;
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt) {
          const int c = (2 * dt + chalf) ^ csw;
          const i16x4_t bop = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (i16x4_t __attribute__((address_space(3)))*)(vrow + c * 16));
          pacc[dt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(aop, bop, pacc[dt], 0, 0, 0);
        }
      } else {
        if (moved) {
#pragma unroll
          for (int hh = 0; hh < R; ++hh) {
            const float alpha = __builtin_amdgcn_exp2f(m_run[hh] - m_new[hh]);
#pragma unroll
            for (int k = 0; k < EPL; ++k) acc[hh][k] *= alpha;
            m_run[hh] = m_new[hh];
          }
        }
        // acc += p * v
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int tl = u * TPI + sub;
          if (tail && grp * 16 + tl >= n_tok) vcur[u] = Row<ESZ>::zero();  // empty slot: may hold anything
          float vf[EPL];
          Row<ESZ>::widen(vcur[u], vf);
#pragma unroll
          for (int hh = 0; hh < R; ++hh) {
            const float p = my_e[tl * R + hh];
#pragma unroll
            for (int k = 0; k < EPL; ++k) acc[hh][k] = fmaf(p, vf[k], acc[hh][k]);
          }
        }
      }
  };
  {
    // DEPTH register buffers used in rotation (the loop is unrolled DEPTH times so that no
    // buffer is ever copied): DEPTH - 1 groups in flight behind the one being worked on
    Piece kb[DEPTH][U], vb[DEPTH][U];
#pragma unroll
    for (int st = 0; st < DEPTH - 1; ++st) {
      const int g2 = w + st * NW;
      if (g2 < ngroups) { load_group(A.kc, g2, kb[st]); load_group(A.vc, g2, vb[st]); }
    }
    for (int base = w; base < ngroups; base += DEPTH * NW) {
#pragma unroll
      for (int st = 0; st < DEPTH; ++st) {
        const int grp = base + st * NW;
        if (grp >= ngroups) break;
        const int gp = grp + (DEPTH - 1) * NW;
        if (gp < ngroups) {
          load_group(A.kc, gp, kb[(st + DEPTH - 1) % DEPTH]);
          load_group(A.vc, gp, vb[(st + DEPTH - 1) % DEPTH]);
        }
        process(kb[st], vb[st], grp);
      }
    }
  }
  // ---- merge: token groups of one wavefront, then the wavefronts ----
  if constexpr (MF) {
#pragma unroll
    for (int v = 0; v < NVH; ++v) {   // sums over the 16 token lanes of a row of lanes
      float l = l_own[v];
      l += lane_xor<1>(l);
      l += lane_xor<2>(l);
      l += lane_xor<4>(l);
      l += lane_xor<8>(l);
      l_own[v] = l;
    }
    if ((lane & 15) == 0) {
#pragma unroll
      for (int v = 0; v < NVH; ++v) {
        const int hh = (lane >> 4) + 4 * v;
        if (hh < R) {
          s_red[w * R + hh] = m_own[v];
          s_red[(NW + w) * R + hh] = l_own[v];
        }
      }
    }
  } else {
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      float l = l_own[i];
      l += lane_xor<4>(l);
      l += lane_xor<8>(l);
      l += __shfl_xor(l, 16);
      l += __shfl_xor(l, 32);
      l_own[i] = l;
    }
    if (lane < 4) {
#pragma unroll
      for (int i = 0; i < PER; ++i) {
        const int hh = (idx0 + i) % R;
        if ((hh * 4) / R == lane) {
          s_red[w * R + hh] = m_own[i];
          s_red[(NW + w) * R + hh] = l_own[i];
        }
      }
    }
  }
  if constexpr (PVM) {
    // rows h and h + 8 of the product (lanes 32 apart) are the two halves of head h
#pragma unroll
    for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const float a = pacc[dt][v] + __shfl_xor(pacc[dt][v], 32);
        if (lane < (R > 4 ? 32 : 16)) s_acc[(w * RW + 4 * (lane >> 4) + v) * HD + 16 * dt + (lane & 15)] = a;
      }
  } else {
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
        for (int k = 0; k < EPL; ++k) s_acc[(w * RW + hh) * HD + seg * EPL + k] = acc[hh][k];
    }
  }
  __syncthreads();

  // chunk max and sum per head from the wavefronts' pairs
  const bool single = nch == 1;
  float cm[R], cl[R], wsc[NW][R];
#pragma unroll
  for (int hh = 0; hh < R; ++hh) {
    float m = s_red[hh];
#pragma unroll
    for (int ww = 1; ww < NW; ++ww) m = fmaxf(m, s_red[ww * R + hh]);
    float l = 0.0f;
#pragma unroll
    for (int ww = 0; ww < NW; ++ww) {
      wsc[ww][hh] = __builtin_amdgcn_exp2f(s_red[ww * R + hh] - m);
      l += s_red[(NW + ww) * R + hh] * wsc[ww][hh];
    }
    cm[hh] = m;
    cl[hh] = l;
  }
  const size_t pslot = (size_t)it.pbase + (size_t)(t0 / Tc);  // partial-result slot of this chunk
#pragma unroll
  for (int hh = 0; hh < R; ++hh) {
    for (int k = tid; k < HD; k += NT) {
      float s = 0.0f;
#pragma unroll
      for (int ww = 0; ww < NW; ++ww) s += s_acc[(ww * RW + hh) * HD + k] * wsc[ww][hh];
      if (single) __builtin_nontemporal_store(s / cl[hh], &A.out[((size_t)g * R + hh) * HD + k]);
      else __builtin_nontemporal_store(s, &A.part_acc[(pslot * R + hh) * HD + k]);
    }
  }
  if (!single && tid == 0) {
#pragma unroll
    for (int hh = 0; hh < R; ++hh) {
      A.part_ml[(pslot * R + hh) * 2 + 0] = cm[hh];
      A.part_ml[(pslot * R + hh) * 2 + 1] = cl[hh];
    }
  }
  if (!A.accumulate) return;
  // The stored 16-bit value of a KV times 2^(its group's running max - chunk max) is the exp of
  // its logit against the chunk max; for a head of one chunk, divided by the sum, its
  // probability.  That factor is the same for the 16 tokens of a group: formed once, in place.
  for (int i = tid; i < ngroups * R; i += NT) {
    const int hh = i % R;
    float f = 0.0f;
#pragma unroll
    for (int h2 = 0; h2 < R; ++h2)
      if (h2 == hh) f = __builtin_amdgcn_exp2f(s_gm[i] - cm[h2]) * (single ? 1.0f / cl[h2] : 1.0f) * (1.0f / 65535.0f);
    s_gm[i] = f;
  }
  __syncthreads();
  for (int tok = tid; tok < n_tok; tok += NT) {
    const size_t slot = ((size_t)s_tab[tok >> lb] << lb) + (tok & (b - 1));
    float e[R];
#pragma unroll
    for (int hh = 0; hh < R; ++hh) e[hh] = (float)s_q[tok * R + hh] * s_gm[(tok >> 4) * R + hh];
    if (single) {
      float inc = 0.0f;
#pragma unroll
      for (int hh = 0; hh < R; ++hh) inc += A.D.mode == KVC_L2 ? e[hh] * e[hh] : e[hh];
      // one writer per slot in a launch, so the hardware add gives the same bits as load-add-store
      unsafeAtomicAdd(&A.metric[slot], inc);
    } else {
      stash_store<R>(A.stash, slot, e);
    }
  }
}

// Second kernel, heads of more than one chunk only.  Every chunk's workgroup
// rebuilds the head's max and sum from the per-chunk pairs, then adds the
// metric increments of its own tokens; the first chunk's workgroup also writes
// the combined output.
template <int R>
__global__ void __launch_bounds__(256) decode_combine_kernel(DecodeArgs A) {
  // one workgroup per partial-result slot in use, i.e. per chunk of a head of more than one chunk
  const int p = blockIdx.x;
  if (p >= A.header[HW_TOTAL_PARTIALS] || p >= A.cap) return;
  const int item = A.slot_item[p];
  if (item < 0 || item >= A.header[HW_TOTAL_ITEMS] || item >= A.cap) return;
  const DecodeItem it = A.items[item];
  const int nch = it.nch;
  if (nch <= 1) return;
  if ((unsigned)it.g >= (unsigned)A.D.G || it.n_tok <= 0 || it.n_tok > A.T || it.t0 < 0 || it.pbase < 0 ||
      it.pbase + nch > A.cap)
    return;  // not a record this call wrote
  const int g = it.g, t0 = it.t0, n_tok = it.n_tok;
  const int Tc = A.header[HW_CHUNK_T];       // tokens the work list was cut at
  if (Tc < 64 || Tc > A.T) return;
  if (A.plan && A.ctx[g] != it.pad[0]) return;   // a kept list that no longer fits the head: its chunks did nothing either
  const int c = t0 / Tc;
  if (c >= nch) return;
  const int first = it.pbase;                // partial-result slots first .. first + nch - 1
  const int b = A.D.b, lb = A.log2b, HD = A.D.d;
  constexpr int kMaxCh = 64;                 // chunk weights kept in LDS; longer heads recompute
  __shared__ float s_m[R], s_il[R], s_w[R], s_wc[kMaxCh][R];
  const int tid = threadIdx.x;
  // one thread per (chunk, head) pair fetches its max and sum; the head's max and sum follow
  __shared__ float s_pm[kMaxCh][R], s_pl[kMaxCh][R];
  const int ncl = min(nch, kMaxCh);
  for (int i = tid; i < ncl * R; i += 256) {
    const float2 ml = *(const float2*)(A.part_ml + ((size_t)first * R + i) * 2);
    s_pm[i / R][i % R] = ml.x;
    s_pl[i / R][i % R] = ml.y;
  }
  __syncthreads();
  if (tid < R) {
    float m = -INFINITY;
    for (int cc = 0; cc < nch; ++cc)
      m = fmaxf(m, cc < kMaxCh ? s_pm[cc][tid] : A.part_ml[((size_t)(first + cc) * R + tid) * 2]);
    float l = 0.0f;
    for (int cc = 0; cc < nch; ++cc) {
      const float pm = cc < kMaxCh ? s_pm[cc][tid] : A.part_ml[((size_t)(first + cc) * R + tid) * 2];
      const float pl = cc < kMaxCh ? s_pl[cc][tid] : A.part_ml[((size_t)(first + cc) * R + tid) * 2 + 1];
      const float wgt = __builtin_amdgcn_exp2f(pm - m);
      if (cc < kMaxCh) s_wc[cc][tid] = wgt;
      l += pl * wgt;
    }
    s_m[tid] = m;
    s_il[tid] = 1.0f / l;
    s_w[tid] = __builtin_amdgcn_exp2f((c < kMaxCh ? s_pm[c][tid] : A.part_ml[((size_t)(first + c) * R + tid) * 2]) - m) / l;
  }
  __syncthreads();
  if (A.accumulate) {
    const int32_t* row = A.table + (size_t)g * A.D.maxb;
    float wv[R];
#pragma unroll
    for (int hh = 0; hh < R; ++hh) wv[hh] = s_w[hh];
    // four tokens per thread at a time, their block ids asked for together and then their exps:
    // a token by itself is a chain of two dependent loads in front of one add, and a chunk of
    // 3456 tokens a dozen such chains per thread one after the other
    for (int tok0 = tid; tok0 < n_tok; tok0 += 4 * 256) {
      int id[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) id[u] = row[(t0 + min(tok0 + u * 256, n_tok - 1)) >> lb];
      size_t slot[4];
      float e[4][R];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int j = t0 + min(tok0 + u * 256, n_tok - 1);
        slot[u] = ((size_t)id[u] << lb) + (j & (b - 1));
        stash_load<R>(A.stash, slot[u], e[u]);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (tok0 + u * 256 >= n_tok) break;
        float inc = 0.0f;
#pragma unroll
        for (int hh = 0; hh < R; ++hh) {
          const float p = e[u][hh] * wv[hh];
          inc += A.D.mode == KVC_L2 ? p * p : p;
        }
        unsafeAtomicAdd(&A.metric[slot[u]], inc);
      }
    }
  }
  if (c == 0) {
    for (int i = tid; i < R * HD; i += 256) {
      const int hh = i / HD;
      float s = 0.0f;
#pragma unroll 4
      for (int cc = 0; cc < ncl; ++cc) s += A.part_acc[(size_t)(first + cc) * R * HD + i] * s_wc[cc][hh];
      for (int cc = kMaxCh; cc < nch; ++cc) {
        const float wgt = __builtin_amdgcn_exp2f(A.part_ml[((size_t)(first + cc) * R + hh) * 2] - s_m[hh]);
        s += A.part_acc[(size_t)(first + cc) * R * HD + i] * wgt;
      }
      A.out[(size_t)g * R * HD + i] = s * s_il[hh];
    }
  }
}

// Fallback for shapes the tiled kernel does not cover (blocks of more than 64 tokens, any d that
// is a multiple of 16 bytes, any r <= 16): one workgroup per head instance, logits
// kept in the workspace.  Correct, not fast.
__global__ void __launch_bounds__(256) decode_generic_kernel(DecodeArgs A) {
  const int gi = blockIdx.x;
  const int g = sel_to_g(A.D, A.l0, A.nl, gi);
  const int R = A.D.r, HD = A.D.d, b = A.D.b;
  const int C = A.ctx[g];
  if (C == 0) {  // a head with no KV: zero output rows
    float* o = A.out + (size_t)g * R * HD;
    for (int i = threadIdx.x; i < R * HD; i += 256) o[i] = 0.0f;
    return;
  }
  extern __shared__ __align__(16) char smem_raw[];
  float* s_q = (float*)smem_raw;      // [R][HD]
  float* s_red = s_q + R * HD;        // [4][16]
  float* s_ml = s_red + 4 * 16;       // [2][16]
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int dt = A.D.dtype;
  const size_t rowb = (size_t)HD * kv_esz(dt), qrowb = (size_t)HD * q_esz(dt);
  auto elem = [&](const char* base, size_t row_off, int k) -> float {
    if (dt == KVC_BF16) return bf16_to_f32(((const uint16_t*)(base + row_off))[k]);
    if (dt == KVC_F32) return ((const float*)(base + row_off))[k];
    return __builtin_amdgcn_cvt_pk_f32_fp8((int)((const uint8_t*)(base + row_off))[k], false)[0];
  };
  for (int i = tid; i < R * HD; i += 256) {
    const char* qr = A.q + ((size_t)g * R + i / HD) * qrowb;
    s_q[i] = dt == KVC_F32 ? ((const float*)qr)[i % HD] : bf16_to_f32(((const uint16_t*)qr)[i % HD]);
  }
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
static int launch_tiled(const DecodeArgs& A, int grid, size_t lds, int grid_short, hipStream_t s) {
  auto kern = (A.D.b % 16 == 0) ? decode_chunk_kernel<ESZ, HD, R, true, 4> : decode_chunk_kernel<ESZ, HD, R, false, 4>;
  auto kern_short = (A.D.b % 16 == 0) ? decode_chunk_kernel<ESZ, HD, R, true, 1> : decode_chunk_kernel<ESZ, HD, R, false, 1>;
  ProfilePair* pp = claim_profile_pair();
  if (pp) KVC_HIP(hipEventRecord(pp->a0, s));
  {  // above the default cap the kernel must be told how much it may take (per instantiation and device)
    static LdsLimit limit[2];
    const int rc = limit[A.D.b % 16 == 0].need(lds, kern);
    if (rc != KVC_OK) return rc;
  }
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kDecodeThreads), lds, s, A);
  KVC_LAUNCH_CHECK();
  if (pp) { KVC_HIP(hipEventRecord(pp->a1, s)); KVC_HIP(hipEventRecord(pp->s0, s)); }
  if (A.short_class < 16) {
    hipLaunchKernelGGL(kern_short, dim3(grid_short), dim3(64),
                       decode_lds_bytes(A.Ts, R, HD, A.D.b, 1, decode_pv_mfma(ESZ, R, HD, A.D.b)), s, A);
    KVC_LAUNCH_CHECK();
  }
  if (pp) { KVC_HIP(hipEventRecord(pp->s1, s)); KVC_HIP(hipEventRecord(pp->b0, s)); }
  // heads of more than one chunk hold more than T tokens each: at most N b / T of them, and their
  // chunks number at most tokens / T plus one per head (a chunk length picked on the device: the
  // bound on the work items serves)
  const size_t split_bound = A.adapt_T ? (size_t)grid : 2 * ((size_t)A.D.N * A.D.b / A.T) + 1;
  const int grid_combine = (size_t)grid < split_bound ? grid : (int)split_bound;
  hipLaunchKernelGGL(decode_combine_kernel<R>, dim3(grid_combine), dim3(256), 0, s, A);
  KVC_LAUNCH_CHECK();
  if (pp) KVC_HIP(hipEventRecord(pp->b1, s));
  return KVC_OK;
}

template <int ESZ, int HD>
static int launch_tiled_r(const DecodeArgs& A, int grid, size_t lds, int grid_short, hipStream_t s) {
  switch (A.D.r) {
    case 1: return launch_tiled<ESZ, HD, 1>(A, grid, lds, grid_short, s);
    case 2: return launch_tiled<ESZ, HD, 2>(A, grid, lds, grid_short, s);
    case 4: return launch_tiled<ESZ, HD, 4>(A, grid, lds, grid_short, s);
    case 8: return launch_tiled<ESZ, HD, 8>(A, grid, lds, grid_short, s);
  }
  return KVC_ERR_UNSUPPORTED;
}

constexpr size_t kLdsLimit = 160 * 1024;  // gfx950: 160 KiB of LDS per workgroup

// Whether the tiled kernels cover this shape, and with which chunk length and LDS size.
static bool choose_chunk(const Dims& D, int gsel, int* T_out, size_t* lds_out, bool* small_call = nullptr,
                         bool* on_device = nullptr) {
  const int esz = kv_esz(D.dtype);
  const int lpt = D.d * esz / 16;
  const int tpi = (lpt >= 1 && lpt <= 64) ? 64 / lpt : 0;
  // (blocks shorter than the tokens one wavefront load covers are fine: off the 16-token-block
  // fast path every token of a load looks its own block up)
  bool tiled = (D.r == 1 || D.r == 2 || D.r == 4 || D.r == 8) && (D.d == 64 || D.d == 128) &&
               tpi >= 1 && 64 % D.b == 0;
  if (!tiled) return false;
  // default: a chunk that lets two workgroups share a CU (at r = 8, d = 128, 16-bit rows: 3456
  // tokens x 16 bytes of exps + the rest = 81 764 of the 81 920 bytes a half CU has)
  const int knob = g_chunk_tokens.load(std::memory_order_relaxed);
  int T = knob ? knob : (D.r >= 8 ? 3456 : 6144);
  const int T_default = T;
  bool shrunk = false, device_side = false;
  if (!knob) {
    // a call over few head instances (one layer at a time) has too few long chunks to fill the
    // chip: shorten them until full rows would give a few thousand work items
    const long long want_items = 6144;
    // (halved and rounded up to whole 64-token strips: a chunk starts on a block boundary)
    while (T > 256 && (long long)gsel * (((long long)D.maxb * D.b + T - 1) / T) < want_items)
      T = ((T / 2) + 63) & ~63;
    shrunk = T < T_default;
    // ... unless the one-launch work list serves the call: it sees the lengths themselves, not
    // just what the tables have room for, and picks the length (at most the default) on the device
    if (shrunk && gsel <= kSmallWorklistHeads) { T = T_default; device_side = true; }
  }
  const bool mf = decode_pv_mfma(esz, D.r, D.d, D.b);   // a per-wavefront operand tile in LDS
  // the default is sized so that two workgroups share a CU's LDS with blocks of 16 tokens; blocks
  // of one or two tokens put a block id per token or two next to the exps: a shorter chunk keeps
  // the second workgroup on the CU
  if (!g_chunk_tokens.load(std::memory_order_relaxed) && D.b < 4 &&
      decode_lds_bytes(T, D.r, D.d, 16, kDecodeWaves, mf) <= kLdsLimit / 2)
    while (T > 1024 && decode_lds_bytes(T, D.r, D.d, D.b, kDecodeWaves, mf) > kLdsLimit / 2) T -= 64;
  while (T > kMinChunk && decode_lds_bytes(T, D.r, D.d, D.b, kDecodeWaves, mf) > kLdsLimit) T -= 64;
  const size_t lds = decode_lds_bytes(T, D.r, D.d, D.b, kDecodeWaves, mf);
  if (lds > kLdsLimit || T % 64 != 0) return false;
  *T_out = T;
  *lds_out = lds;
  if (small_call) *small_call = shrunk;
  if (on_device) *on_device = device_side;
  return true;
}

// Items of at most 512 tokens go to the one-wavefront launch: the size classes from *cls up,
// whose items hold at most *max_tokens tokens; *lds_tokens is that bound in whole 64-token strips.
static void short_split(int T, int* cls, int* max_tokens, int* lds_tokens) {
  int k = 1;
  while (k < 15 && (T >> (k - 1)) > 512) ++k;
  *cls = k;
  *max_tokens = T >> (k - 1);
  *lds_tokens = (*max_tokens + 63) & ~63;
}

}  // namespace kvc

using namespace kvc;

extern "C" {

int kvc_profile_begin(int n) {
  if (n < 0 || n > 4096) return KVC_ERR_ARG;
  std::lock_guard<std::mutex> hold(g_prof_lock);
  g_prof_any.store(n > 0, std::memory_order_release);
  if (g_prof) {
    for (int i = 0; i < g_prof_cap; ++i) {
      hipEventDestroy(g_prof[i].a0); hipEventDestroy(g_prof[i].a1);
      hipEventDestroy(g_prof[i].s0); hipEventDestroy(g_prof[i].s1);
      hipEventDestroy(g_prof[i].b0); hipEventDestroy(g_prof[i].b1);
    }
    delete[] g_prof;
    g_prof = nullptr;
  }
  g_prof_cap = g_prof_used = 0;
  g_prof_on = 1;
  if (n == 0) return KVC_OK;
  g_prof = new ProfilePair[n];
  for (int i = 0; i < n; ++i) {
    KVC_HIP(hipEventCreate(&g_prof[i].a0)); KVC_HIP(hipEventCreate(&g_prof[i].a1));
    KVC_HIP(hipEventCreate(&g_prof[i].s0)); KVC_HIP(hipEventCreate(&g_prof[i].s1));
    KVC_HIP(hipEventCreate(&g_prof[i].b0)); KVC_HIP(hipEventCreate(&g_prof[i].b1));
  }
  g_prof_cap = n;
  return KVC_OK;
}

int kvc_profile_enable(int on) {
  std::lock_guard<std::mutex> hold(g_prof_lock);
  g_prof_on = on != 0;
  return KVC_OK;
}

int kvc_profile_collect(float* chunk_ms, float* short_ms, float* combine_ms, int cap, int* count) {
  if (!count || cap < 0) return KVC_ERR_ARG;
  std::lock_guard<std::mutex> hold(g_prof_lock);
  *count = g_prof_used;
  for (int i = 0; i < g_prof_used && i < cap; ++i) {
    KVC_HIP(hipEventSynchronize(g_prof[i].b1));
    float ms = 0.0f;
    if (chunk_ms) { KVC_HIP(hipEventElapsedTime(&ms, g_prof[i].a0, g_prof[i].a1)); chunk_ms[i] = ms; }
    if (short_ms) { KVC_HIP(hipEventElapsedTime(&ms, g_prof[i].s0, g_prof[i].s1)); short_ms[i] = ms; }
    if (combine_ms) { KVC_HIP(hipEventElapsedTime(&ms, g_prof[i].b0, g_prof[i].b1)); combine_ms[i] = ms; }
  }
  return KVC_OK;
}

int kvc_get_decode_chunk(const kvc_config* cfg, int* tokens) {
  int rc = validate(cfg, nullptr);
  if (rc != KVC_OK) return rc;
  if (!tokens) return KVC_ERR_ARG;
  int T = 0;
  size_t lds = 0;
  const Dims D = dims_of(cfg);
  *tokens = choose_chunk(D, D.G, &T, &lds) ? T : 0;
  return KVC_OK;
}

int kvc_get_decode_short(const kvc_config* cfg, int* tokens) {
  int rc = validate(cfg, nullptr);
  if (rc != KVC_OK) return rc;
  if (!tokens) return KVC_ERR_ARG;
  int T = 0;
  size_t lds = 0;
  const Dims D = dims_of(cfg);
  *tokens = 0;
  if (choose_chunk(D, D.G, &T, &lds)) {
    int cls = 0, lds_tokens = 0;
    short_split(T, &cls, tokens, &lds_tokens);
  }
  return KVC_OK;
}

int kvc_set_decode_chunk(int tokens) {
  if (tokens != 0 && (tokens < kMinChunk || tokens > kMaxChunk || tokens % 64 != 0)) return KVC_ERR_ARG;
  g_chunk_tokens.store(tokens, std::memory_order_relaxed);
  return KVC_OK;
}

}  // extern "C"

// What both decode entry points check on the host before anything is launched.
static int decode_args_check(const kvc_config* cfg, const kvc_state* st, const void* q, const float* out,
                             int layer_begin, int layer_end) {
  const int rc = validate(cfg, st);
  if (rc != KVC_OK) return rc;
  if (!q || !out || ((uintptr_t)q & 15) || ((uintptr_t)out & 15)) return KVC_ERR_ARG;
  if (layer_begin < 0 || layer_end > cfg->num_layers || layer_begin >= layer_end) return KVC_ERR_ARG;
  return KVC_OK;
}

// plan_mode 0: an ordinary call (work list, chunks, combine).  1: only the work lists, one per
// layer, kept in the workspace (q and out are not looked at).  2: layer `layer_begin` from its kept list.
enum { PLAN_NONE = 0, PLAN_BUILD = 1, PLAN_USE = 2 };
static int paged_decode_impl(const kvc_config* cfg, const kvc_state* st, const void* q, float* out,
                             int layer_begin, int layer_end, int accumulate_metric, void* ws, void* stream,
                             int plan_mode = PLAN_NONE, int ctx_plus = 0) {
  int rc = plan_mode == PLAN_BUILD ? validate(cfg, st) : decode_args_check(cfg, st, q, out, layer_begin, layer_end);
  if (rc != KVC_OK) return rc;
  if (!ws || ((uintptr_t)ws & 255)) return KVC_ERR_ARG;
  Dims D = dims_of(cfg);
  if (plan_mode == PLAN_BUILD) { layer_begin = 0; layer_end = 1; }   // lists are per layer: sized as a one-layer call
  Workspace W = carve(D, ws);
  hipStream_t s = (hipStream_t)stream;

  DecodeArgs A;
  A.D = D;
  A.kc = (const char*)st->k_cache; A.vc = (const char*)st->v_cache;
  A.metric = st->metric; A.table = st->block_table; A.ctx = st->ctx_len;
  A.q = (const char*)q; A.out = out;
  A.l0 = layer_begin; A.nl = layer_end - layer_begin; A.gsel = D.S * A.nl * D.Hk;
  A.accumulate = accumulate_metric != 0;
  A.all_partials = 0;
  A.rotate_chunks = 0;
  A.cap = (int)(max_items_of(D) < 0x7fffffffull ? max_items_of(D) : 0x7fffffffull);
  A.items = (DecodeItem*)W.items; A.slot_item = W.slot_item; A.part_ml = W.part_ml; A.part_acc = W.part_acc; A.stash = W.stash;
  A.header = W.header;
  A.status = W.header;
  A.plan = 0; A.plan_stride = 0; A.ctx_plus = 0;
  A.scale_log2 = (float)(1.4426950408889634 / sqrt((double)D.d));

  int T = 0;
  size_t lds = 0;
  bool small_call = false, on_device = false;
  bool tiled = choose_chunk(D, D.S * (layer_end - layer_begin) * D.Hk, &T, &lds, &small_call, &on_device);
  A.adapt_T = tiled && on_device;
  const int esz = kv_esz(D.dtype);
  A.T = tiled ? T : (1 << 30);  // generic path: one "chunk" per head
  A.short_class = 16;
  A.Ts = 0;
  // A small call (one layer of a model) is bound by the time of its slowest item, not by
  // throughput: there every item gets four wavefronts and the short-item launch is left out.
  if (tiled && !small_call) {
    int short_max = 0;
    short_split(T, &A.short_class, &short_max, &A.Ts);
  }
  A.log2b = 0;
  while ((1 << A.log2b) < D.b) ++A.log2b;

  // kept lists exist for what a model's layer-by-layer calls look like: the tiled kernels, few heads
  // per layer, the chunk length picked on the device
  if (plan_mode != PLAN_NONE && !(tiled && small_call && on_device && A.gsel <= kSmallWorklistHeads)) return KVC_ERR_UNSUPPORTED;
  if (!tiled) {
    const size_t gl = ((size_t)D.r * D.d + 4 * 16 + 2 * 16) * 4;
    hipLaunchKernelGGL(decode_generic_kernel, dim3(A.gsel), dim3(256), gl, s, A);
    KVC_LAUNCH_CHECK();
    return KVC_OK;
  }
  // items <= (slots in the pool) / T + heads, and <= heads * chunks a full row can hold.  A chunk
  // length picked on the device is T (then the first bound holds), or at least 1.25 / 512 of all
  // tokens, or the 256-token floor with under 256 * 512 / 1.25 tokens in all: at most 512 / 1.25
  // full chunks either way, and one shorter item per head.
  const size_t most_tokens = std::min((size_t)D.N * D.b, (size_t)A.gsel * D.maxb * D.b);   // pool, or the rows of the heads called for
  const size_t bound_pool = (A.adapt_T ? std::max(most_tokens / T, (size_t)410) : most_tokens / T) + (size_t)A.gsel;
  const size_t Tmin = A.adapt_T ? 256 : (size_t)T;
  const size_t bound_row = (size_t)A.gsel * (((size_t)D.maxb * D.b + Tmin - 1) / Tmin);
  const size_t grid = bound_pool < bound_row ? bound_pool : bound_row;
  if (grid > 0x7fffffffull) return KVC_ERR_UNSUPPORTED;   // before anything is launched: the work list stays clean
  if (plan_mode != PLAN_NONE) {
    // every layer's list has `grid` records of its own (the most its call could need)
    if (grid * (size_t)D.Lyr > (size_t)A.cap) return KVC_ERR_UNSUPPORTED;
    A.plan = 1;
    A.plan_stride = (int)grid;
    A.ctx_plus = ctx_plus;
    A.header = W.plan_hdr;
    if (plan_mode == PLAN_BUILD) {
      A.out = nullptr;    // (the zero rows of heads without a KV are written when the layer is decoded)
      hipLaunchKernelGGL(decode_worklist_small_kernel, dim3(D.Lyr), dim3(1024), 0, s, A);
      KVC_LAUNCH_CHECK();
      return KVC_OK;
    }
    A.header += (size_t)layer_begin * HW_WORDS;
    A.items += (size_t)layer_begin * grid;
    A.slot_item += (size_t)layer_begin * grid;
    A.cap = (int)grid;
  } else if (A.gsel <= kSmallWorklistHeads) {
    hipLaunchKernelGGL(decode_worklist_small_kernel, dim3(1), dim3(1024), 0, s, A);
    KVC_LAUNCH_CHECK();
  } else {
    hipLaunchKernelGGL(decode_count_kernel, dim3((A.gsel + 255) / 256), dim3(256), 0, s, A);
    KVC_LAUNCH_CHECK();
    hipLaunchKernelGGL(decode_items_kernel, dim3((A.gsel + 255) / 256), dim3(256), 0, s, A);
    KVC_LAUNCH_CHECK();
  }
  const int gs = A.gsel;   // a head ends in at most one item shorter than a chunk
  if (esz == 1) return D.d == 64 ? launch_tiled_r<1, 64>(A, (int)grid, lds, gs, s) : launch_tiled_r<1, 128>(A, (int)grid, lds, gs, s);
  if (esz == 2) return D.d == 64 ? launch_tiled_r<2, 64>(A, (int)grid, lds, gs, s) : launch_tiled_r<2, 128>(A, (int)grid, lds, gs, s);
  return D.d == 64 ? launch_tiled_r<4, 64>(A, (int)grid, lds, gs, s) : launch_tiled_r<4, 128>(A, (int)grid, lds, gs, s);
}

// ---- the decode for callers that cannot allocate --------------------------------------------
// The temporaries of kvc_paged_decode (work items, per-chunk partial results, the 16-bit exps of
// split heads) in a fixed array of this library's own instead of a caller's workspace.  Every
// GPU holds its own copy of the array at its own address; host code never uses the array's name
// as an address, only what hipGetSymbolAddress returned for the device that is current.
static __device__ __align__(256) unsigned char scratch[KVC_STATIC_SCRATCH_BYTES];

static constexpr int kMaxDevices = 64;
static std::mutex g_scratch_lock;
static void* g_scratch_ptr[kMaxDevices] = {};   // per device, filled on the first call there

static int scratch_of_current_device(void** out) {
  int dev = -1;
  KVC_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return KVC_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> hold(g_scratch_lock);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    KVC_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p || ((uintptr_t)p & 255)) return KVC_ERR_HIP;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return KVC_OK;
}

extern "C" {

int kvc_paged_decode(const kvc_config* cfg, const kvc_state* st, const void* q, float* out,
                     int layer_begin, int layer_end, int accumulate_metric, void* ws, void* stream) {
  return paged_decode_impl(cfg, st, q, out, layer_begin, layer_end, accumulate_metric, ws, stream);
}

int kvc_decode_plan(const kvc_config* cfg, const kvc_state* st, int ctx_plus, void* ws, void* stream) {
  if (ctx_plus < 0 || ctx_plus > 1) return KVC_ERR_ARG;
  return paged_decode_impl(cfg, st, nullptr, nullptr, 0, 1, 0, ws, stream, PLAN_BUILD, ctx_plus);
}

int kvc_paged_decode_planned(const kvc_config* cfg, const kvc_state* st, const void* q, float* out, int layer,
                             int accumulate_metric, void* ws, void* stream) {
  return paged_decode_impl(cfg, st, q, out, layer, layer + 1, accumulate_metric, ws, stream, PLAN_USE, 0);
}

int kvc_paged_decode_static(const kvc_config* cfg, const kvc_state* st, const void* q, float* out,
                            int layer_begin, int layer_end, int accumulate_metric, void* stream) {
  int rc = decode_args_check(cfg, st, q, out, layer_begin, layer_end);
  if (rc != KVC_OK) return rc;
  if (carve(dims_of(cfg), nullptr).bytes > (size_t)KVC_STATIC_SCRATCH_BYTES) return KVC_ERR_UNSUPPORTED;
  void* ws = nullptr;
  rc = scratch_of_current_device(&ws);
  if (rc != KVC_OK) return rc;
  // The array keeps what the last call left, possibly a call with another config: the header words
  // (item counts, work-list cursors) start from zero again.  A fill kernel, not a memset, so that
  // the call may be recorded into a HIP graph.
  hipLaunchKernelGGL(zero_words_kernel, dim3((HW_WORDS + 63) / 64), dim3(64), 0, (hipStream_t)stream, (int32_t*)ws, HW_WORDS);
  KVC_LAUNCH_CHECK();
  return paged_decode_impl(cfg, st, q, out, layer_begin, layer_end, accumulate_metric, ws, stream);
}

}  // extern "C"
