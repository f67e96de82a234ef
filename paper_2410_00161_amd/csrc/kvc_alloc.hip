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

// Drop counts n[g] of kvc_block_free: blocks held per head instance, checked request.
__global__ void __launch_bounds__(256) count_drop_kernel(Dims D, const int32_t* __restrict__ table,
                                                         const int32_t* __restrict__ ctx,
                                                         const int32_t* __restrict__ n,
                                                         int32_t* __restrict__ held,
                                                         int32_t* __restrict__ req,
                                                         int32_t* __restrict__ header) {
  const int g = blockIdx.x * 256 + threadIdx.x;
  if (g >= D.G) return;
  const int h = held_blocks(table + (size_t)g * D.maxb, ctx[g], D.b, D.maxb);
  held[g] = h;
  int want = n[g];
  if (want < 0 || want > h) { atomicOr(&header[HW_SCRATCH0], EB_ARG); want = 0; }
  req[g] = want;
}

// Launch 1 of an allocation: workgroups [0, gb) count requests per head instance (mode 0:
// the caller's counts n[g]; mode 1: append, one block when the head's blocks are full and its
// layer is in range), workgroups [gb, gb + ntiles) count the free blocks of one tile of the map.
__global__ void __launch_bounds__(256) count_and_free_tiles_kernel(Dims D, const int32_t* __restrict__ table,
                                                                   const int32_t* __restrict__ ctx,
                                                                   const int32_t* __restrict__ n, int mode,
                                                                   int l0, int l1, int gb,
                                                                   const uint8_t* __restrict__ free_map,
                                                                   int32_t* __restrict__ held,
                                                                   int32_t* __restrict__ req,
                                                                   int32_t* __restrict__ tile_sums,
                                                                   int32_t* __restrict__ header) {
  if ((int)blockIdx.x < gb) {
    const int g = blockIdx.x * 256 + threadIdx.x;
    if (g >= D.G) return;
    const int C = ctx[g];
    const int h = held_blocks(table + (size_t)g * D.maxb, C, D.b, D.maxb);
    held[g] = h;
    int want = 0, bits = 0;
    if (mode == 0) {
      want = n[g];
      if (want < 0) { bits |= EB_ARG; want = 0; }
      else if (h + want > D.maxb) bits |= EB_TABLE;
    } else {
      const int l = (g / D.Hk) % D.Lyr;
      if (l >= l0 && l < l1 && C == h * D.b) {
        want = 1;
        if (h + 1 > D.maxb) bits |= EB_TABLE;
      }
    }
    req[g] = want;
    if (bits) atomicOr(&header[HW_SCRATCH0], bits);
    return;
  }
  __shared__ int red[kScanThreads / 64];
  const int tile = blockIdx.x - gb;
  const int base = tile * kScanTile + threadIdx.x * kScanItems;
  int s = 0;
#pragma unroll
  for (int k = 0; k < kScanItems; ++k) if (base + k < D.N) s += free_map[base + k] != 0;
  s = wave_sum_i(s);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) tile_sums[tile] = red[0] + red[1] + red[2] + red[3];
}

constexpr int kScanRun = 16;                   // elements per thread and tile in alloc_scan_kernel
constexpr int kScanWide = 1024 * kScanRun;     // elements per tile

// Exclusive scan of n ints over one workgroup of 1024 threads: every thread takes a run of 16
// consecutive elements (four 16-byte loads and, for the results, four 16-byte stores when the
// arrays are 16-byte aligned, which workspace arrays are: a thread's run is 64 bytes, so with
// 4-byte accesses every instruction of a wavefront touched 64 different lines), one workgroup
// scan joins the runs.  out[i] = exclusive prefix (out may be `in`); `visit(i, value,
// exclusive)` sees every element with a non-zero value.
template <class Visit>
__device__ __forceinline__ int wide_exclusive_scan(const int32_t* in, int n, int32_t* out, int* smem, Visit visit) {
  __shared__ int carry_s;
  if (threadIdx.x == 0) carry_s = 0;
  __syncthreads();
  const bool aligned = (((uintptr_t)in | (uintptr_t)out) & 15) == 0;
  for (int base = 0; base < n; base += kScanWide) {
    const int first = base + threadIdx.x * kScanRun;
    const bool whole = aligned && first + kScanRun <= n;
    int v[kScanRun], sum = 0;
    if (whole) {
#pragma unroll
      for (int k = 0; k < kScanRun; k += 4) {
        const int4 t = *(const int4*)(in + first + k);
        v[k] = t.x; v[k + 1] = t.y; v[k + 2] = t.z; v[k + 3] = t.w;
      }
    } else {
#pragma unroll
      for (int k = 0; k < kScanRun; ++k) v[k] = first + k < n ? in[first + k] : 0;
    }
#pragma unroll
    for (int k = 0; k < kScanRun; ++k) sum += v[k];
    int tot;
    int ex = block_exclusive_scan<1024>(sum, smem, &tot) + carry_s;
    int o[kScanRun];
#pragma unroll
    for (int k = 0; k < kScanRun; ++k) {
      o[k] = ex;
      if (v[k] && first + k < n) visit(first + k, v[k], ex);
      ex += v[k];
    }
    if (whole) {
#pragma unroll
      for (int k = 0; k < kScanRun; k += 4) *(int4*)(out + first + k) = make_int4(o[k], o[k + 1], o[k + 2], o[k + 3]);
    } else {
#pragma unroll
      for (int k = 0; k < kScanRun; ++k) if (first + k < n) out[first + k] = o[k];
    }
    __syncthreads();
    if (threadIdx.x == 0) carry_s += tot;
    __syncthreads();
  }
  return carry_s;
}

// Launch 2, one workgroup: exclusive scan of the requests (off[g], off[G] = total), the owner
// of every request (owner[k] = head instance that gets the k-th block), exclusive scan of the
// free-tile counts, and the status word.
__global__ void __launch_bounds__(1024) alloc_scan_kernel(Dims D, const int32_t* __restrict__ req,
                                                          int32_t* __restrict__ off,
                                                          int32_t* __restrict__ owner,
                                                          int32_t* __restrict__ tile_sums, int ntiles,
                                                          int32_t* __restrict__ header) {
  __shared__ int smem[1024 / 64 + 1];
  const int N = D.N;
  const int total_req = wide_exclusive_scan(req, D.G, off, smem, [&](int g, int v, int ex) {
    if (ex + v <= N)  // more requests than blocks exist is an error found below
      for (int i = 0; i < v; ++i) owner[ex + i] = g;
  });
  const int total_free = wide_exclusive_scan(tile_sums, ntiles, tile_sums, smem, [](int, int, int) {});
  if (threadIdx.x == 0) {
    off[D.G] = total_req;
    header[HW_TOTAL_REQ] = total_req;
    header[HW_TOTAL_FREE] = total_free;
    const int bits = header[HW_SCRATCH0];
    int st = KVC_OK;
    if (bits & EB_ARG) st = KVC_ERR_ARG;
    else if (bits & EB_TABLE) st = KVC_ERR_TABLE_FULL;
    else if (total_req > total_free) st = KVC_ERR_OOM;
    if (st != KVC_OK && header[HW_STATUS] == KVC_OK) header[HW_STATUS] = st;
    header[HW_SCRATCH0] = 0;
  }
}

// Third phase of the scan over the free map, fused with the hand-out: the free block of
// rank k (ascending id) goes to owner[k], the head instance g with off[g] <= k < off[g + 1],
// as its (k - off[g])-th new block.
__global__ void __launch_bounds__(kScanThreads) pick_scatter_kernel(Dims D, int32_t* __restrict__ table,
                                                                    uint8_t* __restrict__ free_map,
                                                                    const int32_t* __restrict__ tile_sums,
                                                                    const int32_t* __restrict__ held,
                                                                    const int32_t* __restrict__ off,
                                                                    const int32_t* __restrict__ owner,
                                                                    const int32_t* __restrict__ header) {
  __shared__ int smem[kScanThreads / 64 + 1];
  const int total_req = header[HW_TOTAL_REQ];
  const bool ok = header[HW_STATUS] == KVC_OK;
  const int tile0 = tile_sums[blockIdx.x];
  if (!ok || tile0 >= total_req) return;  // uniform over the workgroup
  const int base = blockIdx.x * kScanTile + threadIdx.x * kScanItems;
  int v[kScanItems];
  int s = 0;
#pragma unroll
  for (int k = 0; k < kScanItems; ++k) { v[k] = (base + k < D.N) ? (free_map[base + k] != 0) : 0; s += v[k]; }
  int ex = block_exclusive_scan<kScanThreads>(s, smem, nullptr) + tile0;
#pragma unroll
  for (int k = 0; k < kScanItems; ++k) {
    if (v[k]) {
      if (ex < total_req) {
        const int lo = owner[ex];
        table[(size_t)lo * D.maxb + held[lo] + (ex - off[lo])] = base + k;
        free_map[base + k] = 0;
      }
      ++ex;
    }
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

// A group of lanes per head instance, as many as the new key and value have 16-byte pieces
// (rounded up to a power of two, at most a wavefront; 32 lanes for 256-byte rows, so two heads
// per wavefront): copy the rows, zero the metric, set the logical index, bump the length.  The
// kernel is a chain of three dependent loads per head, so heads in flight are what counts.
__global__ void __launch_bounds__(256) append_write_kernel(Dims D, int l0, int l1, int lanes_per_head,
                                                          char* __restrict__ kc,
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
  const int heads_per_wg = 256 / lanes_per_head;
  const int idx = blockIdx.x * heads_per_wg + threadIdx.x / lanes_per_head;   // over S * nl * Hk
  const int gl = threadIdx.x % lanes_per_head;
  if (idx >= D.S * nl * D.Hk) return;   // no barrier below
  const int s = idx / (nl * D.Hk);
  const int l = l0 + (idx / D.Hk) % nl;
  const int h = idx % D.Hk;
  const int g = (s * D.Lyr + l) * D.Hk + h;
  const int C = ctx[g];
  const int blk = table[(size_t)g * D.maxb + C / D.b];
  const int o = C % D.b;
  const size_t row_bytes = (size_t)D.d * kv_esz(D.dtype);
  const size_t slot = (size_t)blk * D.b + o;
  const int pieces = (int)(row_bytes / 16);
  for (int c = gl; c < 2 * pieces; c += lanes_per_head) {
    const bool is_v = c >= pieces;
    const int cc = is_v ? c - pieces : c;
    const uint4* src = (const uint4*)((is_v ? v_new : k_new) + (size_t)g * row_bytes) + cc;
    uint4* dst = (uint4*)((is_v ? vc : kc) + slot * row_bytes) + cc;
    *dst = *src;
  }
  // the lanes of a group belong to one wavefront (one instruction stream): all of them have read
  // ctx[g] by the time one of them writes it
  if (gl == 0) {
    metric[slot] = 0.0f;
    if (pos) pos[slot] = new_pos ? new_pos[s] : C;
    ctx[g] = C + 1;
  }
}

// Count (mode as in count_kernel), rank the free map, resolve errors, scatter.
static int alloc_common(const Dims& D, const kvc_state* st, const Workspace& W, const int32_t* n,
                        int mode, int l0, int l1, hipStream_t s) {
  const int gb = (D.G + 255) / 256;
  const int ntiles = (D.N + kScanTile - 1) / kScanTile;
  hipLaunchKernelGGL(count_and_free_tiles_kernel, dim3(gb + ntiles), dim3(256), 0, s, D, st->block_table,
                     st->ctx_len, n, mode, l0, l1, gb, st->free_map, W.held, W.off_b, W.tile_sums, W.header);
  KVC_LAUNCH_CHECK();
  hipLaunchKernelGGL(alloc_scan_kernel, dim3(1), dim3(1024), 0, s, D, W.off_b, W.off_a, W.picked, W.tile_sums,
                     ntiles, W.header);
  KVC_LAUNCH_CHECK();
  hipLaunchKernelGGL(pick_scatter_kernel, dim3(ntiles), dim3(kScanThreads), 0, s, D, st->block_table,
                     st->free_map, W.tile_sums, W.held, W.off_a, W.picked, W.header);
  KVC_LAUNCH_CHECK();
  return KVC_OK;
}

// ---- scheduling helpers: counts per sequence, prefill allocation, preemption --------------

// needed[s] = blocks sequence s must get before its next decode step (head instances of the
// chosen layers whose blocks are all full); held[s] = blocks it holds over all layers.
__global__ void __launch_bounds__(256) count_blocks_kernel(Dims D, const int32_t* __restrict__ table,
                                                           const int32_t* __restrict__ ctx, int l0, int l1,
                                                           int32_t* __restrict__ needed,
                                                           int32_t* __restrict__ held_out) {
  const int g = blockIdx.x * 256 + threadIdx.x;
  const bool in = g < D.G;
  const int gg = in ? g : D.G - 1;
  const int s = gg / (D.Lyr * D.Hk), l = (gg / D.Hk) % D.Lyr;
  const int C = ctx[gg];
  const int h = held_blocks(table + (size_t)gg * D.maxb, C, D.b, D.maxb);
  int need = in && l >= l0 && l < l1 && C == h * D.b;
  int hh = in ? h : 0;
  // one atomic per wavefront when all its lanes belong to one sequence
  const int s0 = __builtin_amdgcn_readfirstlane(s);
  if (__all(s == s0)) {
    need = wave_sum_i(need);
    hh = wave_sum_i(hh);
    if ((threadIdx.x & 63) == 0) {
      if (needed && need) atomicAdd(&needed[s0], need);
      if (held_out && hh) atomicAdd(&held_out[s0], hh);
    }
  } else if (in) {
    if (needed && need) atomicAdd(&needed[s], need);
    if (held_out && hh) atomicAdd(&held_out[s], hh);
  }
}

// The batch of a compression round, one workgroup.  Rank of every running sequence in the order
// (time of last compression, never = first; then index) by counting, the order written out,
// a 64-bit running total of allocated KVs along it, and the cut at the first sequence that does
// not fit.  held[s] = blocks the sequence holds (from count_blocks_kernel); order: S ints.
__global__ void __launch_bounds__(1024) compression_batch_kernel(int S, int b, const int32_t* __restrict__ held,
                                                                 const int64_t* __restrict__ last,
                                                                 const uint8_t* __restrict__ running,
                                                                 long long limit, int32_t* __restrict__ order,
                                                                 uint8_t* __restrict__ in_batch,
                                                                 int64_t* __restrict__ batch_kvs) {
  __shared__ long long wave_tot[1024 / 64];
  __shared__ long long carry_s, total_s;
  __shared__ int cut_s, nrun_s;
  const int tid = threadIdx.x;
  if (tid == 0) { carry_s = 0; total_s = 0; cut_s = 0x7fffffff; nrun_s = 0; }
  __syncthreads();
  auto key = [&](int s) -> long long { const long long t = last[s]; return t < 0 ? -1 : t; };
  auto runs = [&](int s) -> bool { return running == nullptr || running[s] != 0; };
  for (int s = tid; s < S; s += 1024) {
    in_batch[s] = 0;
    if (!runs(s)) continue;
    const long long ks = key(s);
    int rank = 0;
    for (int t = 0; t < S; ++t) {
      if (!runs(t)) continue;
      const long long kt = key(t);
      rank += (kt < ks) || (kt == ks && t < s);
    }
    order[rank] = s;
    atomicAdd(&nrun_s, 1);
  }
  __syncthreads();   // the order is complete (global writes of this workgroup are visible to it)
  const int nrun = nrun_s;
  for (int base = 0; base < nrun; base += 1024) {
    const int p = base + tid;
    const int s = p < nrun ? order[p] : -1;
    const long long v = s >= 0 ? (long long)held[s] * b : 0;
    long long inc = v;   // inclusive scan over the wavefront
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const long long t = __shfl_up(inc, o);
      if ((tid & 63) >= o) inc += t;
    }
    if ((tid & 63) == 63) wave_tot[tid >> 6] = inc;
    __syncthreads();
    long long before = carry_s;
    for (int w = 0; w < (tid >> 6); ++w) before += wave_tot[w];
    const long long cum = before + inc;
    if (s >= 0 && cum > limit) atomicMin(&cut_s, p);
    __syncthreads();
    if (tid == 1023) carry_s = cum;
    __syncthreads();
    // positions before the cut of this or an earlier tile are in; a cut found in this tile is final
    const int cut = cut_s;
    if (s >= 0 && p < cut) in_batch[s] = 1;
    // the last position taken so far, if it lies in this tile, knows the batch's total
    const int last_in = min(min(cut, nrun), base + 1024) - 1;
    if (p == last_in && last_in >= base) total_s = cum;
    __syncthreads();
    if (cut != 0x7fffffff) break;
  }
  __syncthreads();
  if (tid == 0 && batch_kvs) *batch_kvs = total_s;
}

// Requests of a prefill: every head of sequence s wants ceil(tokens[s] / b) blocks in all.
__global__ void __launch_bounds__(256) prefill_want_kernel(Dims D, const int32_t* __restrict__ table,
                                                           const int32_t* __restrict__ ctx,
                                                           const int32_t* __restrict__ seq_tokens,
                                                           int32_t* __restrict__ n_new,
                                                           int32_t* __restrict__ header) {
  const int g = blockIdx.x * 256 + threadIdx.x;
  if (g >= D.G) return;
  const int t = seq_tokens[g / (D.Lyr * D.Hk)];
  int want = 0;
  if (t < 0) atomicOr(&header[HW_SCRATCH0], EB_ARG);
  else if (t > 0) {
    const int h = held_blocks(table + (size_t)g * D.maxb, ctx[g], D.b, D.maxb);
    want = max(0, (t + D.b - 1) / D.b - h);
  }
  n_new[g] = want;
}

__global__ void __launch_bounds__(256) prefill_len_kernel(Dims D, const int32_t* __restrict__ seq_tokens,
                                                          int32_t* __restrict__ ctx,
                                                          const int32_t* __restrict__ header) {
  if (header[HW_STATUS] != KVC_OK) return;
  const int g = blockIdx.x * 256 + threadIdx.x;
  if (g >= D.G) return;
  const int t = seq_tokens[g / (D.Lyr * D.Hk)];
  if (t > 0) ctx[g] = t;
}

__global__ void __launch_bounds__(256) preempt_kernel(Dims D, int32_t* __restrict__ table,
                                                      int32_t* __restrict__ ctx, uint8_t* __restrict__ free_map,
                                                      const uint8_t* __restrict__ seq_mask,
                                                      int32_t* __restrict__ header) {
  const int g = blockIdx.x * 256 + threadIdx.x;
  int n = 0;
  if (g < D.G && seq_mask[g / (D.Lyr * D.Hk)]) {
    int32_t* row = table + (size_t)g * D.maxb;
    n = held_blocks(row, ctx[g], D.b, D.maxb);
    for (int u = 0; u < n; ++u) { free_map[row[u]] = 1; row[u] = -1; }
    ctx[g] = 0;
  }
  n = wave_sum_i(n);
  if ((threadIdx.x & 63) == 0 && n) atomicAdd(&header[HW_FREED], n);
}

// State check.  One wavefront per head instance walks its table row: ids in [0, N) as a prefix,
// -1 after it, the length within what the prefix holds; every held block counted once in
// `owner` (zeroed before the launch) and not marked free.
__global__ void __launch_bounds__(256) check_state_kernel(Dims D, const int32_t* __restrict__ table,
                                                          const int32_t* __restrict__ ctx,
                                                          const uint8_t* __restrict__ free_map,
                                                          int32_t* __restrict__ owner,
                                                          int32_t* __restrict__ header) {
  const int g = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (g >= D.G) return;
  const int lane = threadIdx.x & 63;
  const int32_t* row = table + (size_t)g * D.maxb;
  bool bad = false;
  int held = 0;
  bool ended = false;   // a -1 has been seen (the same in every lane)
  for (int base = 0; base < D.maxb; base += 64) {
    const int u = base + lane;
    const int id = u < D.maxb ? row[u] : -1;
    const bool holds = id != -1;
    if (holds) {
      if (id < 0 || id >= D.N) bad = true;
      else {
        if (atomicAdd(&owner[id], 1) != 0) bad = true;   // held twice
        if (free_map[id] != 0) bad = true;               // held and marked free
      }
    }
    const unsigned long long m = __ballot(holds);
    const int run = m == ~0ull ? 64 : __ffsll((long long)~m) - 1;   // ids at the front of these 64 cells
    if (ended ? m != 0 : (run < 64 && (m >> run) != 0)) bad = true;   // an id behind a -1
    if (!ended) held += run;
    if (run < 64) ended = true;
  }
  const int C = ctx[g];
  if (C < 0 || (long long)C > (long long)held * D.b) bad = true;
  if (__any(bad) && lane == 0) atomicOr(&header[HW_SCRATCH0], EB_ARG);
}

}  // namespace kvc

using namespace kvc;

extern "C" {

int kvc_check_state(const kvc_config* cfg, const kvc_state* st, void* ws, void* stream, int flags) {
  int rc = validate(cfg, st);
  if (rc != KVC_OK) return rc;
  if (!ws || ((uintptr_t)ws & 255)) return KVC_ERR_ARG;
  Dims D = dims_of(cfg);
  Workspace W = carve(D, ws);
  hipStream_t s = (hipStream_t)stream;
  int32_t* owner = (int32_t*)W.stash;   // [N] fits where the decode keeps N * b * r floats
  hipLaunchKernelGGL(zero_words_kernel, dim3((D.N + 255) / 256), dim3(256), 0, s, owner, D.N);
  KVC_LAUNCH_CHECK();
  hipLaunchKernelGGL(check_state_kernel, dim3((D.G + 3) / 4), dim3(256), 0, s, D, st->block_table, st->ctx_len,
                     st->free_map, owner, W.header);
  KVC_LAUNCH_CHECK();
  hipLaunchKernelGGL(resolve_kernel, dim3(1), dim3(64), 0, s, W.header, 0);
  KVC_LAUNCH_CHECK();
  return (flags & KVC_ASYNC) ? KVC_OK : finish_sync(W, s);
}

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
  hipLaunchKernelGGL(count_drop_kernel, dim3(gb), dim3(256), 0, s, D, st->block_table, st->ctx_len, n_drop,
                     W.held, W.off_b, W.header);
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
  int lanes_per_head = 8;   // 2 * pieces rounded up to a power of two, within [8, 64]
  while (lanes_per_head < 64 && lanes_per_head < 2 * (D.d * kv_esz(D.dtype) / 16)) lanes_per_head *= 2;
  const int heads_per_wg = 256 / lanes_per_head;
  hipLaunchKernelGGL(append_write_kernel, dim3((nsel + heads_per_wg - 1) / heads_per_wg), dim3(256), 0, s, D,
                     layer_begin, layer_end, lanes_per_head,
                     (char*)st->k_cache, (char*)st->v_cache, st->metric, st->pos, st->block_table,
                     st->ctx_len, (const char*)k_new, (const char*)v_new, new_pos, W.header);
  KVC_LAUNCH_CHECK();
  return (flags & KVC_ASYNC) ? KVC_OK : finish_sync(W, s);
}

int kvc_count_blocks(const kvc_config* cfg, const kvc_state* st, int layer_begin, int layer_end,
                     int32_t* needed, int32_t* held, void* ws, void* stream) {
  int rc = validate(cfg, st);
  if (rc != KVC_OK) return rc;
  (void)ws;
  Dims D = dims_of(cfg);
  if (layer_begin < 0 || layer_end > D.Lyr || layer_begin >= layer_end) return KVC_ERR_ARG;
  if (!needed && !held) return KVC_ERR_ARG;
  hipStream_t s = (hipStream_t)stream;
  if (needed) { hipLaunchKernelGGL(zero_words_kernel, dim3((D.S + 63) / 64), dim3(64), 0, s, needed, D.S); KVC_LAUNCH_CHECK(); }
  if (held) { hipLaunchKernelGGL(zero_words_kernel, dim3((D.S + 63) / 64), dim3(64), 0, s, held, D.S); KVC_LAUNCH_CHECK(); }
  hipLaunchKernelGGL(count_blocks_kernel, dim3((D.G + 255) / 256), dim3(256), 0, s, D, st->block_table, st->ctx_len,
                     layer_begin, layer_end, needed, held);
  KVC_LAUNCH_CHECK();
  return KVC_OK;
}

int kvc_compression_batch(const kvc_config* cfg, const kvc_state* st, const int64_t* last_compressed,
                          const uint8_t* running, int64_t kv_limit, uint8_t* in_batch, int64_t* batch_kvs,
                          void* ws, void* stream) {
  int rc = validate(cfg, st);
  if (rc != KVC_OK) return rc;
  if (!last_compressed || !in_batch || !ws || ((uintptr_t)ws & 255) || kv_limit < 0) return KVC_ERR_ARG;
  if (((uintptr_t)last_compressed & 7) || (batch_kvs && ((uintptr_t)batch_kvs & 7))) return KVC_ERR_ARG;
  Dims D = dims_of(cfg);
  if (D.S > 8192) return KVC_ERR_UNSUPPORTED;   // ranks are found by counting, S^2 comparisons in one workgroup
  Workspace W = carve(D, ws);
  hipStream_t s = (hipStream_t)stream;
  int32_t* held = W.off_b;    // [S] fits in the [G + 1] array
  int32_t* order = W.off_a;
  hipLaunchKernelGGL(zero_words_kernel, dim3((D.S + 63) / 64), dim3(64), 0, s, held, D.S);
  KVC_LAUNCH_CHECK();
  hipLaunchKernelGGL(count_blocks_kernel, dim3((D.G + 255) / 256), dim3(256), 0, s, D, st->block_table, st->ctx_len,
                     0, D.Lyr, (int32_t*)nullptr, held);
  KVC_LAUNCH_CHECK();
  hipLaunchKernelGGL(compression_batch_kernel, dim3(1), dim3(1024), 0, s, D.S, D.b, held, last_compressed, running,
                     (long long)kv_limit, order, in_batch, batch_kvs);
  KVC_LAUNCH_CHECK();
  return KVC_OK;
}

int kvc_prefill_alloc(const kvc_config* cfg, const kvc_state* st, const int32_t* seq_tokens, void* ws,
                      void* stream, int flags) {
  int rc = validate(cfg, st);
  if (rc != KVC_OK) return rc;
  if (!seq_tokens || !ws || ((uintptr_t)ws & 255)) return KVC_ERR_ARG;
  Dims D = dims_of(cfg);
  Workspace W = carve(D, ws);
  hipStream_t s = (hipStream_t)stream;
  const int gb = (D.G + 255) / 256;
  int32_t* n_new = W.flag_scan;  // [G] fits in the [G][maxb] array
  hipLaunchKernelGGL(prefill_want_kernel, dim3(gb), dim3(256), 0, s, D, st->block_table, st->ctx_len, seq_tokens,
                     n_new, W.header);
  KVC_LAUNCH_CHECK();
  rc = alloc_common(D, st, W, n_new, 0, 0, D.Lyr, s);
  if (rc != KVC_OK) return rc;
  hipLaunchKernelGGL(prefill_len_kernel, dim3(gb), dim3(256), 0, s, D, seq_tokens, st->ctx_len, W.header);
  KVC_LAUNCH_CHECK();
  return (flags & KVC_ASYNC) ? KVC_OK : finish_sync(W, s);
}

int kvc_preempt(const kvc_config* cfg, const kvc_state* st, const uint8_t* seq_mask, int64_t* blocks_freed,
                void* ws, void* stream, int flags) {
  int rc = validate(cfg, st);
  if (rc != KVC_OK) return rc;
  if (!seq_mask || !ws || ((uintptr_t)ws & 255)) return KVC_ERR_ARG;
  Dims D = dims_of(cfg);
  Workspace W = carve(D, ws);
  hipStream_t s = (hipStream_t)stream;
  hipLaunchKernelGGL(zero_words_kernel, dim3(1), dim3(64), 0, s, W.header + HW_FREED, 1);
  KVC_LAUNCH_CHECK();
  hipLaunchKernelGGL(preempt_kernel, dim3((D.G + 255) / 256), dim3(256), 0, s, D, st->block_table, st->ctx_len,
                     st->free_map, seq_mask, W.header);
  KVC_LAUNCH_CHECK();
  if ((flags & KVC_ASYNC) || !blocks_freed) return KVC_OK;
  int32_t f = 0;
  rc = read_words(W.header + HW_FREED, &f, 1, s);
  if (rc != KVC_OK) return rc;
  *blocks_freed = f;
  return KVC_OK;
}

}  // extern "C"
