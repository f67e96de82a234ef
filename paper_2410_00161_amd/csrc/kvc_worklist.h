// Work list shared by the kernels that walk every head instance in chunks of T tokens (the
// decode and the observation-window metric): item records built on the device from the
// context lengths, ordered by size class, plus the cross-lane helpers those kernels use.
#pragma once

#include "kvc_common.h"

namespace kvc {

struct DecodeItem {   // 32 bytes
  int g;        // head instance
  int t0;       // first token of the chunk
  int n_tok;    // tokens in the chunk
  int nch;      // chunks of the head
  int pbase;    // first partial-result slot of the head (heads of more than one chunk)
  int pad[3];   // [0]: the head's length the list was made for (lists kept by kvc_decode_plan)
};

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
  int accumulate, T;      // metric on/off, chunk tokens (the most a chunk may hold when adapt_T is set)
  int adapt_T;            // the one-launch work list picks the chunk length from the lengths it sees (see there)
  int log2b;              // block size is a power of two on the tiled path
  int cap;                // item records and partial-result slots the workspace holds
  int all_partials;       // give every head a partial-result slot range, not only split heads
  int rotate_chunks;      // a head's full chunks take their places rotated by the head's index (see decode_items_kernel)
  int short_class, Ts;    // size classes from short_class up (at most Ts tokens) are "short" items; 16 = none
  DecodeItem* items;
  int32_t* slot_item;     // work item of partial-result slot p (heads of more than one chunk): what the combine kernel runs over
  float* part_ml;
  float* part_acc;
  float* stash;
  int32_t* header;
  // Work lists kept from one launch for every layer (kvc_decode_plan): layer l has its own header
  // block at header + l * HW_WORDS and its own stretch of plan_stride records of items / slot_item.
  int plan, plan_stride;  // plan: the work-list kernel runs one workgroup per layer; a decode reads one layer's list
  int ctx_plus;           // the plan is made for heads ctx_plus tokens longer than they are now
  int32_t* status;        // the workspace's own header (status word), whatever `header` points at
  float scale_log2;       // log2(e) / sqrt(d)
};

__device__ __forceinline__ int sel_to_g(const Dims& D, int l0, int nl, int gi) {
  const int s = gi / (nl * D.Hk);
  const int l = l0 + (gi / D.Hk) % nl;
  const int h = gi % D.Hk;
  return (s * D.Lyr + l) * D.Hk + h;
}

// Work items are ordered by size class, largest first, so that the short ones fill the end
// of the launch.  Class 0 = a full chunk of T tokens; class k >= 1 = (T / 2^k, T / 2^(k-1)).
__device__ __forceinline__ int size_class(int n, int T) {
  if (n >= T) return 0;
  int cls = 1, t = T >> 1;
  while (n <= t && cls < 15) { ++cls; t >>= 1; }
  return cls;
}

// Pass 1 of the work list: number of items per size class.
static __global__ void __launch_bounds__(256) decode_count_kernel(DecodeArgs A) {
  __shared__ int bins[17];   // [16] = partial-result slots wanted
  if (threadIdx.x < 17) bins[threadIdx.x] = 0;
  __syncthreads();
  const int gi = blockIdx.x * 256 + threadIdx.x;
  if (gi < A.gsel) {
    const int C = A.ctx[sel_to_g(A.D, A.l0, A.nl, gi)];
    const int nfull = C / A.T, rem = C - nfull * A.T;
    const int nch = nfull + (rem ? 1 : 0);
    if (nfull) atomicAdd(&bins[0], nfull);
    if (rem) atomicAdd(&bins[size_class(rem, A.T)], 1);
    if (nch > 1 || (A.all_partials && nch > 0)) atomicAdd(&bins[16], nch);
  }
  __syncthreads();
  if (threadIdx.x < 16 && bins[threadIdx.x]) atomicAdd(&A.header[HW_DEC_BINS + threadIdx.x], bins[threadIdx.x]);
  if (threadIdx.x == 16 && bins[16]) atomicAdd(&A.header[HW_DEC_PTOT], bins[16]);
}

// Pass 2: every head instance claims its places and writes its items; a head that holds no
// KV gets its zero output rows here.  Workgroup x of a launch runs on XCD x % 8, so with
// rotate_chunks a head's chunks are dealt to the XCDs starting from a different one for every
// head: where only the first few chunks of every head have work (a block of queries early in a
// prompt) and heads hold a multiple of eight chunks, that work would otherwise all land on the
// same few XCDs.  Places are claimed per workgroup (one global atomic
// per class) and handed out inside it through LDS, so the global counters see few updates.
static __global__ void __launch_bounds__(256) decode_items_kernel(DecodeArgs A) {
  __shared__ int base[16], want[17], got[17];
  const int tid = threadIdx.x;
  if (tid < 17) want[tid] = 0;
  if (tid == 0) {
    int run = 0;
    int shorts = 0;
    for (int k = 0; k < 16; ++k) {
      const int c = A.header[HW_DEC_BINS + k];
      base[k] = run;
      run += c;
      if (k >= A.short_class) shorts += c;
    }
    if (blockIdx.x == 0) {
      A.header[HW_TOTAL_ITEMS] = run;
      A.header[HW_SHORT_ITEMS] = shorts;
      A.header[HW_TOTAL_PARTIALS] = A.header[HW_DEC_PTOT];
      A.header[HW_CHUNK_T] = A.T;
    }
  }
  __syncthreads();
  const int gi = blockIdx.x * 256 + tid;
  const int T = A.T;
  int g = 0, C = 0, nfull = 0, rem = 0, nch = 0, cls = 0;
  int my_full = 0, my_rem = 0, my_p = 0;  // offsets inside this workgroup's claims
  if (gi < A.gsel) {
    g = sel_to_g(A.D, A.l0, A.nl, gi);
    C = A.ctx[g];
    nfull = C / T;
    rem = C - nfull * T;
    nch = nfull + (rem ? 1 : 0);
    cls = rem ? size_class(rem, T) : 0;
    if (nfull) my_full = atomicAdd(&want[0], nfull);
    if (rem) my_rem = atomicAdd(&want[cls], 1);       // class 0 never holds a remainder
    if (nch > 1 || (A.all_partials && nch > 0)) my_p = atomicAdd(&want[16], nch);
  }
  __syncthreads();
  if (tid < 17 && want[tid])
    got[tid] = atomicAdd(&A.header[tid < 16 ? HW_DEC_CUR + tid : HW_DEC_PCUR], want[tid]);
  __syncthreads();
  if (gi >= A.gsel) return;
  if (C == 0) {
    if (A.out) {
      float* o = A.out + (size_t)g * A.D.r * A.D.d;
      for (int i = 0; i < A.D.r * A.D.d; ++i) o[i] = 0.0f;
    }
    return;
  }
  const bool slotted = nch > 1 || A.all_partials;
  const int pbase = slotted ? got[16] + my_p : 0;
  // the counters start from zero, so these bounds hold by construction; a workspace that was
  // never reset is the one way to break them, and then nothing is written
  if (pbase < 0 || pbase + nch > A.cap) return;
  if (nfull) {
    const int at = base[0] + got[0] + my_full;
    if (at < 0 || at + nfull > A.cap) return;
    for (int c = 0; c < nfull; ++c) {
      DecodeItem it = {g, c * T, T, nch, pbase, {0, 0, 0}};
      const int place = at + (A.rotate_chunks ? (c + g) % nfull : c);
      A.items[place] = it;
      if (slotted) A.slot_item[pbase + c] = place;
    }
  }
  if (rem) {
    const int at = base[cls] + got[cls] + my_rem;
    if (at < 0 || at >= A.cap) return;
    DecodeItem it = {g, nfull * T, rem, nch, pbase, {0, 0, 0}};
    A.items[at] = it;
    if (slotted) A.slot_item[pbase + nfull] = at;
  }
}

// Both passes in one workgroup, for calls over at most kSmallWorklistHeads head instances (one
// layer of a model, one prompt): one launch instead of two.  Leaves the header words as the
// two-pass pair does.  (Measured with two heads per thread, 2048 heads: no faster than the pair.)
constexpr int kSmallWorklistHeads = 1024;
static __global__ void __launch_bounds__(1024) decode_worklist_small_kernel(DecodeArgs A) {
  __shared__ int bins[16], base[16], cur[17], ptot;
  __shared__ unsigned long long tokens;
  __shared__ int live;
  const int tid = threadIdx.x;
  // a plan: workgroup l lists layer A.l0 + l into that layer's header block and stretch of records
  const int layer = A.plan ? (int)blockIdx.x : 0;
  int32_t* header = A.header + (size_t)layer * (A.plan ? HW_WORDS : 0);
  DecodeItem* items = A.items + (size_t)layer * A.plan_stride;
  int32_t* slot_item = A.slot_item + (size_t)layer * A.plan_stride;
  const int cap = A.plan ? A.plan_stride : A.cap;
  if (tid == 0) { ptot = 0; tokens = 0; live = 0; }
  if (tid < 16) bins[tid] = 0;
  if (tid < 17) cur[tid] = 0;
  __syncthreads();
  int g = 0, C = 0, nfull = 0, rem = 0, nch = 0, cls = 0;
  if (tid < A.gsel) {
    g = sel_to_g(A.D, A.l0 + layer, A.nl, tid);
    C = A.ctx[g] + A.ctx_plus;
  }
  // Chunk length of a call over few heads.  Such a call is over when its slowest item is.  One
  // workgroup alone on its CU streams ~25 GB/s, two that share one ~12 each, the chip ~6 TB/s:
  // the slowest item and the whole call end together when a chunk is 1/256 of all the tokens
  // with up to 256 heads, 1/512 from 512 heads on.  A quarter on top, so that heads of one
  // length (each an item of that length then) are not cut just behind their first chunk;
  // cutting costs (the exps of a split head go through the workspace), so nothing shorter than
  // 256 tokens.
  int T = A.T;
  if (A.adapt_T) {
    unsigned long long t = (unsigned long long)max(C, 0);
    for (int m = 32; m >= 1; m >>= 1) t += __shfl_xor(t, m);
    if ((tid & 63) == 0 && t) atomicAdd(&tokens, t);
    if (C > 0) atomicAdd(&live, 1);
    __syncthreads();
    const int den = min(512, max(256, live));
    const unsigned long long want = (tokens + tokens / 4) / den;
    const int t64 = (int)((want < (unsigned long long)A.T ? want : (unsigned long long)A.T) + 63) & ~63;
    T = min(A.T, max(256, t64));
  }
  if (tid == 0) header[HW_CHUNK_T] = T;
  if (tid < A.gsel) {
    nfull = C / T;
    rem = C - nfull * T;
    nch = nfull + (rem ? 1 : 0);
    cls = rem ? size_class(rem, T) : 0;
    if (nfull) atomicAdd(&bins[0], nfull);
    if (rem) atomicAdd(&bins[cls], 1);
    if (nch > 1 || (A.all_partials && nch > 0)) atomicAdd(&ptot, nch);
  }
  __syncthreads();
  if (tid == 0) {
    header[HW_TOTAL_PARTIALS] = ptot;
    int run = 0, shorts = 0;
    for (int k = 0; k < 16; ++k) {
      base[k] = run;
      run += bins[k];
      if (k >= A.short_class) shorts += bins[k];
    }
    header[HW_TOTAL_ITEMS] = run;
    header[HW_SHORT_ITEMS] = shorts;
  }
  __syncthreads();
  if (tid >= A.gsel) return;
  if (C == 0) {
    if (A.out) {
      float* o = A.out + (size_t)g * A.D.r * A.D.d;
      for (int i = 0; i < A.D.r * A.D.d; ++i) o[i] = 0.0f;
    }
    return;
  }
  const bool slotted = nch > 1 || A.all_partials;
  const int pbase = slotted ? atomicAdd(&cur[16], nch) : 0;
  if (pbase < 0 || pbase + nch > cap) return;
  if (nfull) {
    const int at = base[0] + atomicAdd(&cur[0], nfull);
    if (at < 0 || at + nfull > cap) return;
    for (int c = 0; c < nfull; ++c) {
      DecodeItem it = {g, c * T, T, nch, pbase, {C, 0, 0}};
      const int place = at + (A.rotate_chunks ? (c + g) % nfull : c);
      items[place] = it;
      if (slotted) slot_item[pbase + c] = place;
    }
  }
  if (rem) {
    const int at = base[cls] + atomicAdd(&cur[cls], 1);
    if (at < 0 || at >= cap) return;
    DecodeItem it = {g, nfull * T, rem, nch, pbase, {C, 0, 0}};
    items[at] = it;
    if (slotted) slot_item[pbase + nfull] = at;
  }
}

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
// Value held by lane (l ^ MASK).  Masks below 16 stay inside a row of 16 lanes and use
// data-parallel primitives: quad permutes for 1 and 2, a quad reverse followed by a half-row
// mirror for 4 (i ^ 3 ^ 7 = i ^ 4), a rotation by 8 for 8.
template <int MASK>
__device__ __forceinline__ float lane_xor(float v) {
  if constexpr (MASK == 1) return dpp_move<0xB1>(v);
  else if constexpr (MASK == 2) return dpp_move<0x4E>(v);
  else if constexpr (MASK == 4) return dpp_move<0x141>(dpp_move<0x1B>(v));
  else if constexpr (MASK == 8) return dpp_move<0x128>(v);
  else return __shfl_xor(v, MASK);
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
          v[i] = keep + lane_xor<MASK>(send);
        }
        Butterfly<H, MASK / 2>::run(v, lane);
      } else {
        v[0] += lane_xor<MASK>(v[0]);
        Butterfly<1, MASK / 2>::run(v, lane);
      }
    }
  }
};

}  // namespace kvc
