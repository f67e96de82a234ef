/*
 * kvc.h - C ABI of libkvc: head-variable paged KV cache for MI355X (gfx950).
 *
 * The library implements the data-parallel hot path of KV-Compress
 * (arXiv 2410.00161): a paged decode attention in which every
 * (sequence, layer, KV head) owns its own block table and context length over
 * one unified [N, b, d] cache, the per-KV eviction metric accumulated in the
 * same pass, a block-level reduction of that metric, a lowest-metric block
 * selection across layers and heads, and a MoveCache compaction that returns
 * whole blocks to an on-device allocator.
 *
 * Conventions common to every call
 *   - Plain C ABI.  Every function returns a kvc_status (KVC_OK = 0).
 *   - Every pointer named below is DEVICE memory on the current HIP device and
 *     is owned by the caller, unless its comment says "host".  The library
 *     allocates nothing; its temporaries live in the caller's workspace `ws`
 *     of at least kvc_workspace_bytes(cfg) bytes, 256-byte aligned.  Two calls
 *     that share a workspace must be ordered on one stream.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     All work is enqueued on it.
 *   - Argument errors are found on the host before anything is launched.
 *     Capacity and numeric errors are found on the device before any state is
 *     written: on ANY error the cache state is left exactly as it was.
 *   - Calls documented as "synchronises" wait for the stream before returning
 *     because they return a count or an error found on the device.  Passing
 *     KVC_ASYNC in `flags` skips that wait: the call returns KVC_OK at once,
 *     later launches that depend on a failed step become no-ops, and the code
 *     is read later with kvc_poll_status().
 *   - Host side, the library keeps no state of a cache: what a call needs is in
 *     its arguments, so calls on different workspaces may come from different
 *     host threads.  Process-wide are only the tuning knob kvc_set_decode_chunk
 *     (read once per call) and what the library has told the runtime about its
 *     kernels (set once, under atomics).
 *   - Head instance g = (s * num_layers + l) * num_kv_heads + h; G = S*Lyr*Hk.
 *     Query head hq of a layer belongs to KV head hq / group_size.
 *   - A head instance holds the blocks block_table[g][0 .. held), held = the
 *     length of the non-negative prefix of its row; its ctx_len[g] KVs occupy
 *     logical slots 0 .. ctx_len-1, slot j at (block_table[g][j / b], j % b).
 */
#ifndef KVC_H_
#define KVC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  KVC_OK = 0,
  KVC_ERR_ARG = 1,        /* null / misaligned pointer, bad enum, bad range     */
  KVC_ERR_OOM = 2,        /* fewer free blocks than requested                    */
  KVC_ERR_TABLE_FULL = 3, /* a head would exceed max_blocks_per_head             */
  /* 4 is not used */
  KVC_ERR_NUMERIC = 5,    /* NaN, infinite or negative block key                 */
  KVC_ERR_HIP = 6,        /* a HIP runtime call failed                           */
  KVC_ERR_UNSUPPORTED = 7 /* shape outside what the kernels cover                */
} kvc_status;

/* kv_dtype.  KVC_FP8_E4M3: K and V (cache rows and appended rows) are OCP 8-bit floats,
 * 4 exponent bits (bias 7), 3 mantissa bits, no infinities, 0x7f / 0xff = NaN, taken at
 * face value (a caller with scale factors folds them into q and out); queries are bf16.  */
enum { KVC_F32 = 0, KVC_BF16 = 1, KVC_FP8_E4M3 = 2 };
enum { KVC_L2 = 0, KVC_L1 = 1 };     /* metric_mode: sum of p^2 (default) or of p */
enum { KVC_KEY_SUM = 0, KVC_KEY_MAX = 1 };  /* key_mode of kvc_metric_reduce               */
enum { KVC_ASYNC = 1 };              /* flags                                     */

/* Immutable description of the cache (paper: Method, "Block Layout and Parallel
 * Allocation": block tables B x l x H x Lmax/b, one cache N x b x d).           */
typedef struct kvc_config {
  int32_t num_seqs;            /* S (paper B)                                   */
  int32_t num_layers;          /* Lyr (paper l)                                 */
  int32_t num_kv_heads;        /* Hk (paper H)                                  */
  int32_t group_size;          /* r = query heads per KV head                   */
  int32_t head_dim;            /* d                                             */
  int32_t block_size;          /* b: a power of two, 1 .. 1024 (else KVC_ERR_UNSUPPORTED) */
  int32_t num_blocks;          /* N                                             */
  int32_t max_blocks_per_head; /* Lmax / b                                      */
  int32_t kv_dtype;            /* KVC_F32 | KVC_BF16 (q has the same type) | KVC_FP8_E4M3 (q is bf16) */
  int32_t metric_mode;         /* KVC_L2 | KVC_L1                               */
} kvc_config;

/* Mutable state, all device memory ("Evicting from a Paged KV Cache": K_u, V_u
 * of shape N x b x d, metrics M of shape N x b in the same layout, the logical
 * index of every slot; "Block Layout and Parallel Allocation": tables, context
 * lengths and the flat length-N allocation tensor).                            */
typedef struct kvc_state {
  void*    k_cache;     /* [N, b, d] kv_dtype, 16-byte aligned                  */
  void*    v_cache;     /* [N, b, d] kv_dtype, 16-byte aligned                  */
  float*   metric;      /* [N, b] f32                                           */
  int32_t* pos;         /* [N, b] logical index, may be NULL                    */
  int32_t* block_table; /* [S, Lyr, Hk, max_blocks_per_head], -1 = none         */
  int32_t* ctx_len;     /* [S, Lyr, Hk]                                         */
  uint8_t* free_map;    /* [N], 1 = free                                        */
} kvc_state;

/* Bytes of workspace any call with this config may need.  Host only, no HIP
 * call.  Returns 0 when cfg is invalid.                                        */
size_t kvc_workspace_bytes(const kvc_config* cfg);

/* Checks cfg (and st when non-NULL) the way every entry point does.  Host
 * only.  KVC_OK, KVC_ERR_ARG or KVC_ERR_UNSUPPORTED.                           */
int kvc_validate(const kvc_config* cfg, const kvc_state* st);

/* Host string for a status code; never NULL.                                   */
const char* kvc_status_string(int status);

/* Zeroes the workspace header.  Call once after allocating `ws`, and again to
 * clear an error left by an asynchronous call.                                 */
int kvc_workspace_reset(const kvc_config* cfg, void* ws, void* stream);

/* Reads the error word the device-side guards write (host out-param `status`).
 * Synchronises the stream.                                                     */
int kvc_poll_status(const kvc_config* cfg, void* ws, void* stream, int* status);

/* Checks what every other call takes for granted of a state (a caller that fills the tables
 * itself can ask before it trusts them; the library's own calls keep all of it): every row of
 * block_table is a run of ids in [0, N) followed by -1s; 0 <= ctx_len[g] <= (ids in row g) * b;
 * no block is held twice; free_map is 0 for every held block.  Reads only.  KVC_OK, or
 * KVC_ERR_ARG when any of it fails.  Synchronises unless KVC_ASYNC.                  */
int kvc_check_state(const kvc_config* cfg, const kvc_state* st, void* ws, void* stream, int flags);

/* On-device block allocator ("Block Layout and Parallel Allocation": a flat
 * tensor of length N tracks allocation; counting and allocation run in
 * parallel over all sequences, layers and heads).
 * n_new [G] i32: blocks wanted per head instance, appended to its row after the
 * blocks it holds.  Requesters are served in ascending g and the k-th requested
 * block overall is the k-th lowest-numbered free block.  ctx_len is not
 * changed.  Errors: KVC_ERR_OOM, KVC_ERR_TABLE_FULL, KVC_ERR_ARG (negative
 * request).  Synchronises unless KVC_ASYNC.                                    */
int kvc_block_alloc(const kvc_config* cfg, const kvc_state* st, const int32_t* n_new,
                    void* ws, void* stream, int flags);

/* Drops the last n_drop[g] blocks of every head instance (a preemption drops
 * them all): their ids go back to free_map, their table cells become -1 and
 * ctx_len[g] is clamped to the slots that remain.  blocks_freed: host int64
 * out-param, may be NULL (then nothing is read back).  KVC_ERR_ARG when a count
 * is negative or exceeds the blocks held.  Synchronises unless KVC_ASYNC.      */
int kvc_block_free(const kvc_config* cfg, const kvc_state* st, const int32_t* n_drop,
                   int64_t* blocks_freed, void* ws, void* stream, int flags);

/* Which sequences a round of compression takes (Experiments, where the scheduling of
 * compression is described): the running sequences are taken in order of the time of their last
 * compression, never-compressed ones first, equal times by sequence index, while the KVs
 * allocated to the batch (blocks held x block_size per sequence) stay within kv_limit; the
 * first sequence that would exceed it is left out and closes the batch.  last_compressed [S]
 * i64 (device): any clock that grows, negative = never.  running [S] u8 (device) or NULL = all.
 * in_batch [S] u8 (device, out); batch_kvs: device i64 scalar (out, may be NULL), the KVs
 * allocated to the batch.  A caller turns in_batch into per-sequence budgets for
 * kvc_evict_select / kvc_evict_rank_select (0 for the sequences left out).  KVC_ERR_ARG for a
 * negative limit, KVC_ERR_UNSUPPORTED above 8192 sequences.  Asynchronous.            */
int kvc_compression_batch(const kvc_config* cfg, const kvc_state* st, const int64_t* last_compressed,
                          const uint8_t* running, int64_t kv_limit, uint8_t* in_batch, int64_t* batch_kvs,
                          void* ws, void* stream);

/* Scheduling counts, computed in parallel on the device ("Block Layout and Parallel
 * Allocation": required additional blocks of running sequences from the context lengths;
 * blocks a preemption would free, per sequence).  needed [S] i32 (device, may be NULL): blocks
 * sequence s must get before the next decode step over layers [layer_begin, layer_end) - one
 * per head instance whose blocks are all full.  held [S] i32 (device, may be NULL): blocks it
 * holds over all layers.  Asynchronous.                                           */
int kvc_count_blocks(const kvc_config* cfg, const kvc_state* st, int layer_begin, int layer_end,
                     int32_t* needed, int32_t* held, void* ws, void* stream);

/* Prefill scheduling (same section: blocks follow from the token length alone, every head of
 * a sequence starts with the same number).  seq_tokens [S] i32 (device): every head instance
 * of a sequence with tokens > 0 is brought up to ceil(tokens / b) blocks and its ctx_len set
 * to tokens (the caller then writes the keys and values); sequences with 0 are left alone.
 * Errors and order rule as kvc_block_alloc.  Synchronises unless KVC_ASYNC.       */
int kvc_prefill_alloc(const kvc_config* cfg, const kvc_state* st, const int32_t* seq_tokens,
                      void* ws, void* stream, int flags);

/* Preemption: every block of the sequences with seq_mask[s] != 0 (device [S] u8) goes back to
 * free_map, their table rows become -1 and their ctx_len 0.  blocks_freed: host int64
 * out-param, may be NULL.  Synchronises unless KVC_ASYNC or blocks_freed is NULL.  */
int kvc_preempt(const kvc_config* cfg, const kvc_state* st, const uint8_t* seq_mask,
                int64_t* blocks_freed, void* ws, void* stream, int flags);

/* Appends one new token's key and value to every head instance of layers
 * [layer_begin, layer_end).  k_new, v_new [S, Lyr, Hk, d] kv_dtype.  A head
 * whose blocks are all full first takes one block (same order rule as
 * kvc_block_alloc).  The new slot's metric starts at 0 ("Continual
 * Compression": later queries add into it) and its logical index is
 * new_pos[s] (device [S] i32) or, when new_pos is NULL, the head's old length.
 * Errors as kvc_block_alloc.  Synchronises unless KVC_ASYNC.                   */
int kvc_append(const kvc_config* cfg, const kvc_state* st, const void* k_new,
               const void* v_new, const int32_t* new_pos, int layer_begin, int layer_end,
               void* ws, void* stream, int flags);

/* One decode step of paged attention with per-head tables (Preliminaries:
 * A = softmax(q K^T / sqrt d), out = A V; Method: "Block Layout and Parallel
 * Allocation") over layers [layer_begin, layer_end).
 * q [S, Lyr, Hq, d] kv_dtype (bf16 for an 8-bit cache), out [S, Lyr, Hq, d] f32; rows of other layers are
 * neither read nor written.  Head instance g attends to its own ctx_len[g]
 * KVs; a head with no KV gets zeros.  When accumulate_metric != 0 every
 * attended slot's metric grows by the sum over the r query heads of its group
 * ("Query Group Compression") of p^2 ("Squared Attention Metric"; p with
 * KVC_L1), p being the normalised probability ("Continual Compression").
 * Asynchronous; no device-side error exists for this call.                     */
int kvc_paged_decode(const kvc_config* cfg, const kvc_state* st, const void* q, float* out,
                     int layer_begin, int layer_end, int accumulate_metric,
                     void* ws, void* stream);

/* A model decodes one layer at a time (the query of a layer follows from the layer before), and
 * a call over one layer's few heads spends a fair part of its time on its work list.  This call
 * builds the work lists of ALL layers in one launch and keeps them in the workspace;
 * kvc_paged_decode_planned then decodes one layer from its kept list (same kernels, same
 * results as kvc_paged_decode over that layer).  ctx_plus = 0: the lists are for the heads as
 * they are now; 1: for every head one token longer than now, i.e. planned before the step's
 * kvc_append calls (layer by layer, each before its layer's decode).  The lists stay valid
 * until a context length changes in any other way (compaction, free, preemption, a second
 * append): a layer decoded from a stale list does nothing for the heads that changed and leaves
 * KVC_ERR_ARG in the status word (kvc_poll_status; the cache state is not touched).
 * Covers what kvc_paged_decode runs on its tiled kernels with at most 1024 head instances per
 * layer and the library's own chunk length, else KVC_ERR_UNSUPPORTED.  Asynchronous.     */
int kvc_decode_plan(const kvc_config* cfg, const kvc_state* st, int ctx_plus, void* ws, void* stream);
int kvc_paged_decode_planned(const kvc_config* cfg, const kvc_state* st, const void* q, float* out, int layer,
                             int accumulate_metric, void* ws, void* stream);

/* kvc_paged_decode for callers that cannot allocate device memory or bring a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, kernels and results as kvc_paged_decode, without `ws`: the temporaries live in a
 * fixed array of KVC_STATIC_SCRATCH_BYTES inside the library (every GPU the library runs on
 * holds one until the process ends).  KVC_ERR_UNSUPPORTED when kvc_workspace_bytes(cfg) exceeds
 * that size - such caches go through kvc_paged_decode with a caller's workspace.  Allocates
 * nothing and calls no allocating routine.  All calls on one GPU share the array: two calls
 * that overlap there (different streams, different threads) race; order them.  Asynchronous. */
#define KVC_STATIC_SCRATCH_BYTES (32u << 20)
int kvc_paged_decode_static(const kvc_config* cfg, const kvc_state* st, const void* q, float* out,
                            int layer_begin, int layer_end, int accumulate_metric, void* stream);

/* Block-level reduction of the metric ("Evicting from a Paged KV Cache": the
 * requirement orders blocks by the SUM of their KVs' metrics; the matrix the
 * same section builds takes the last column of a row, its MAX).  block_key
 * [G, max_blocks] f32.  KVC_KEY_SUM: block_key[g][u] = M[n][0] + M[n][1] + ...
 * over the filled slots of logical block u (n = block_table[g][u]), added left
 * to right in f32.  KVC_KEY_MAX: the largest of those metrics.  A partial last
 * block contributes only its real slots.  Cells with u >= ceil(ctx_len/b) are
 * not written (tables are sized for the longest prompt, compressed heads use a
 * fraction of their row, and nothing reads the keys of blocks a head does not
 * hold).  KVC_ERR_ARG for any other key_mode.  Asynchronous.                    */
int kvc_metric_reduce(const kvc_config* cfg, const kvc_state* st, float* block_key, int key_mode,
                      void* ws, void* stream);

/* Lowest-metric block selection across layers and heads (same section: each
 * sequence s evicts its budget E_s of blocks, the cheapest first).
 * A segment is a run of consecutive sequences: seg_offsets [nseg + 1] i32
 * (device) in sequence units, seg_offsets[0] = 0, last = S; NULL = one segment
 * per sequence (then nseg must equal S).  1 <= nseg <= S (segments may be
 * empty, but the workspace holds S of them).  budget [nseg] i32 (device).
 * Candidates of head g are its logical blocks u < ceil(ctx_len/b) -
 * protect_tail_blocks (1 keeps every head's last block, matching the domain
 * 1 <= e < ceil(C_h/b); 0 lets a head lose everything).  Per segment the
 * min(budget, candidates) candidates smallest in (key, s, l, h, u) are chosen.
 * Outputs: evict_flag [G, max_blocks] u8 (fully rewritten), evict_count [G]
 * i32, selected [nseg] i32 = blocks actually chosen.
 * KVC_ERR_NUMERIC when a candidate key is NaN, infinite or negative (outputs
 * are then all zero).  Synchronises unless KVC_ASYNC.                          */
int kvc_evict_select(const kvc_config* cfg, const kvc_state* st, const float* block_key,
                     const int32_t* seg_offsets, const int32_t* budget, int nseg,
                     int protect_tail_blocks, uint8_t* evict_flag, int32_t* evict_count,
                     int32_t* selected, void* ws, void* stream, int flags);

/* MoveCache (Algorithm 1) for every head at once, then the free step.  Per head
 * with flagged blocks: n_ev = KVs in flagged blocks, T = ctx_len - n_ev; kept
 * KVs in slots >= T move, highest first, into the evicted slots below T, lowest
 * first (key, value, metric and pos together); ctx_len becomes T and the table
 * cells from ceil(T/b) on are freed.  evict_flag / evict_count as produced by
 * kvc_evict_select.  blocks_freed: device int64, set to the number of blocks
 * returned to free_map; may be NULL.  KVC_ERR_ARG (nothing modified) when a flag
 * is set at or beyond ceil(ctx_len/b) or a count disagrees with its flags.
 * Synchronises unless KVC_ASYNC.                                               */
int kvc_compact(const kvc_config* cfg, const kvc_state* st, const uint8_t* evict_flag,
                const int32_t* evict_count, int64_t* blocks_freed, void* ws, void* stream,
                int flags);

/* The paper's own eviction schedule ("Evicting from a Paged KV Cache": metrics sorted per
 * head, rows of b with the empty slots of the last block first as zeros, m(h, e) = last
 * column of row e-1, rows of all heads of a sequence ordered by it, first E_s rows marked),
 * computed without sorting.  Candidate rows of head g: e <= ceil(ctx_len/b) -
 * protect_tail_blocks.  Per segment the min(budget, candidates) rows smallest in
 * (m, s, l, h, e) are chosen.  seg_offsets / budget / nseg / selected as kvc_evict_select.
 * Output evict_rows [G] i32: blocks each head loses.  KVC_ERR_NUMERIC when a metric of a
 * candidate head is NaN, infinite or negative (outputs all zero).  Reads metric, block_table
 * and ctx_len; changes no state.  Synchronises unless KVC_ASYNC.                  */
int kvc_evict_rank_select(const kvc_config* cfg, const kvc_state* st, const int32_t* seg_offsets,
                          const int32_t* budget, int nseg, int protect_tail_blocks,
                          int32_t* evict_rows, int32_t* selected, void* ws, void* stream, int flags);

/* Carries a rank schedule out: head g loses its evict_rows[g]*b - (empty slots of its last
 * block) KVs of smallest (metric, logical index) — the KVs of its first evict_rows[g] rows —
 * then MoveCache (Algorithm 1) closes the holes below the new length with the kept KVs above
 * it, ctx_len becomes (ceil(ctx_len/b) - evict_rows[g]) * b and the tail blocks are freed.
 * blocks_freed: device int64, may be NULL.  KVC_ERR_ARG (nothing modified) when a count is
 * negative or exceeds the head's blocks.  Synchronises unless KVC_ASYNC.          */
int kvc_compact_rank(const kvc_config* cfg, const kvc_state* st, const int32_t* evict_rows,
                     int64_t* blocks_freed, void* ws, void* stream, int flags);

/* Prefill-end metric from an observation window (Preliminaries "KV Cache Compression":
 * attention summed over the last w prompt queries, max-pooled over the sequence; "Query Group
 * Compression": and over the query heads of the group; "Metric Calculation", KVC-w: squared
 * before summation, p itself with KVC_L1) over layers [layer_begin, layer_end).
 * q_win [S, Lyr, Hq, w, d] bf16: window query i of a head with C = ctx_len KVs sits at
 * position C - w + i and attends to keys 0 .. C - w + i; queries that would sit before
 * position 0 are ignored.  raw[j] = sum over the r heads and w queries of p^2.  Keys before
 * the window get max(raw[j - pool/2 .. j + pool/2]) with the range cut at the ends of that
 * prefix (pool odd; 1 = no pooling); keys inside the window keep raw.  The result replaces
 * metric[slot] of every KV of those layers, or is added to it when accumulate != 0.
 * row_lse [S, Lyr, Hq, w] f32 (device) or NULL: ln of every window query's softmax
 * denominator over the keys it attends to (what a prefill's attention kernel leaves per query
 * row).  With it p = exp(q.k / sqrt d - row_lse) is formed in ONE pass over the keys; without
 * it the kernels first pass over the keys once more to find the denominators themselves.
 * Runs on the matrix cores; covers kv_dtype = KVC_BF16 and KVC_FP8_E4M3, head_dim 64 and 128,
 * every block size, w <= 64 and w * group_size <= 256, else KVC_ERR_UNSUPPORTED (such callers
 * can gather the same sums with one kvc_paged_decode per window query).  Asynchronous. */
int kvc_window_metric(const kvc_config* cfg, const kvc_state* st, const void* q_win, const float* row_lse,
                      int w, int pool, int accumulate, int layer_begin, int layer_end, void* ws, void* stream);

/* Building block of the all-queries metric ("Metric Calculation", KVC-full: squared attention
 * aggregated over all observed queries, one block of queries at a time, leaving out the first v
 * queries after each key).  q_blk [S, Lyr, Hq, w, d]: query i sits at position first_pos + i
 * (the same for every head; a prefill), attends to keys 0 .. min(position, ctx_len - 1), and
 * adds p^2 (p with KVC_L1) to metric[slot of key j] only when j <= position - exclude.
 * Always accumulates; no pooling.  Calling it for consecutive blocks of a prompt's queries
 * builds M_full[j] = sum over i >= j + v and the group's heads of A_ij^2.  row_lse
 * [S, Lyr, Hq, w] or NULL, shapes and errors as kvc_window_metric, except that w may be any
 * length (the paper aggregates 1024 queries at a time): a longer block is worked off 64
 * queries, or 256 query rows, at a time.  Asynchronous.                            */
int kvc_query_block_metric(const kvc_config* cfg, const kvc_state* st, const void* q_blk, const float* row_lse,
                           int w, int first_pos, int exclude, int layer_begin, int layer_end, void* ws,
                           void* stream);

/* Tuning knob of kvc_paged_decode: tokens handled by one workgroup before a
 * head is split across workgroups.  0 restores the default.  Process-wide,
 * host only.  KVC_ERR_ARG unless 0 or a multiple of 64 in [64, 8192].          */
int kvc_set_decode_chunk(int tokens);

/* The chunk length kvc_paged_decode uses for this config when called over all layers (host
 * out-param), 0 when the shape takes the general fallback kernel, which does not split heads.
 * It is the most a chunk holds: a call over few head instances (fewer layers, few sequences)
 * may use shorter chunks, and one over at most 1024 picks the length on the device from the
 * lengths of the heads.  Host only.                                              */
int kvc_get_decode_chunk(const kvc_config* cfg, int* tokens);

/* kvc_paged_decode runs the last chunk of a head (or a whole short head) in a second launch,
 * one wavefront per item, when it holds at most this many tokens (host out-param; for a call
 * over all layers; 0 on the fallback path).  Host only.                          */
int kvc_get_decode_short(const kvc_config* cfg, int* tokens);

#ifdef __cplusplus
}
#endif
#endif /* KVC_H_ */
