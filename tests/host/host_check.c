/* Host-only exercise of libkvc's C ABI, meant to be built with AddressSanitizer and
 * UndefinedBehaviorSanitizer on the host side (tests/test_host_sanitizers.py does that): every
 * entry point is driven down its argument checks, none of which touches a GPU.  Plain C: also a
 * check that include/kvc.h is a C header. */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "kvc.h"
#include "kvc_bench.h"

static int failures = 0;
#define EXPECT(cond)                                                        \
  do {                                                                      \
    if (!(cond)) { fprintf(stderr, "FAILED line %d: %s\n", __LINE__, #cond); ++failures; } \
  } while (0)

static kvc_config good(void) {
  kvc_config c;
  memset(&c, 0, sizeof c);
  c.num_seqs = 2; c.num_layers = 3; c.num_kv_heads = 2; c.group_size = 4; c.head_dim = 128;
  c.block_size = 16; c.num_blocks = 64; c.max_blocks_per_head = 8; c.kv_dtype = KVC_BF16; c.metric_mode = KVC_L2;
  return c;
}

int main(void) {
  kvc_config c = good();
  EXPECT(kvc_validate(&c, NULL) == KVC_OK);
  EXPECT(kvc_validate(NULL, NULL) == KVC_ERR_ARG);
  size_t n0 = kvc_workspace_bytes(&c);
  EXPECT(n0 > 0 && n0 % 256 == 0);
  /* sizes grow with every dimension, and stay exact for sizes past 32 bits */
  for (int f = 0; f < 4; ++f) {
    kvc_config d = good();
    if (f == 0) d.num_blocks = 1 << 22;
    if (f == 1) d.num_seqs = 4096;
    if (f == 2) d.max_blocks_per_head = 1 << 14;
    if (f == 3) d.group_size = 8;
    EXPECT(kvc_workspace_bytes(&d) > n0);
  }
  {
    kvc_config d = good();
    d.num_seqs = 16; d.num_layers = 80; d.num_kv_heads = 8; d.group_size = 8; d.num_blocks = 11532651; d.max_blocks_per_head = 8200;
    EXPECT(kvc_workspace_bytes(&d) > ((size_t)1 << 32));
  }
  /* what validate refuses */
  {
    int bad_b[] = {0, -16, 3, 24, 48, 2048};
    for (unsigned i = 0; i < sizeof bad_b / sizeof *bad_b; ++i) {
      kvc_config d = good(); d.block_size = bad_b[i];
      EXPECT(kvc_validate(&d, NULL) != KVC_OK && kvc_workspace_bytes(&d) == 0);
    }
    kvc_config d = good(); d.kv_dtype = 9; EXPECT(kvc_validate(&d, NULL) == KVC_ERR_ARG);
    d = good(); d.metric_mode = -1; EXPECT(kvc_validate(&d, NULL) == KVC_ERR_ARG);
    d = good(); d.head_dim = 100; EXPECT(kvc_validate(&d, NULL) == KVC_ERR_UNSUPPORTED);
    d = good(); d.group_size = 17; EXPECT(kvc_validate(&d, NULL) == KVC_ERR_UNSUPPORTED);
    d = good(); d.num_seqs = 1 << 20; d.num_layers = 1 << 10; EXPECT(kvc_validate(&d, NULL) == KVC_ERR_UNSUPPORTED);
  }
  for (int s = -2; s < 12; ++s) EXPECT(kvc_status_string(s) != NULL && strlen(kvc_status_string(s)) > 0);
  /* the tuning knob */
  int t = -1;
  EXPECT(kvc_set_decode_chunk(100) == KVC_ERR_ARG && kvc_set_decode_chunk(1 << 20) == KVC_ERR_ARG);
  EXPECT(kvc_set_decode_chunk(512) == KVC_OK && kvc_get_decode_chunk(&c, &t) == KVC_OK && t == 512);
  EXPECT(kvc_set_decode_chunk(0) == KVC_OK && kvc_get_decode_chunk(&c, &t) == KVC_OK && t > 0 && t % 64 == 0);
  EXPECT(kvc_get_decode_short(&c, &t) == KVC_OK && t > 0 && t <= 512);
  EXPECT(kvc_get_decode_chunk(&c, NULL) == KVC_ERR_ARG);
  /* every entry point refuses a state of null pointers, a misaligned workspace, bad ranges -
   * before anything is launched (the addresses below are never dereferenced) */
  kvc_state nul;
  memset(&nul, 0, sizeof nul);
  kvc_state st;
  st.k_cache = (void*)4096; st.v_cache = (void*)8192; st.metric = (float*)4096; st.pos = NULL;
  st.block_table = (int32_t*)4096; st.ctx_len = (int32_t*)4096; st.free_map = (uint8_t*)4096;
  EXPECT(kvc_validate(&c, &st) == KVC_OK && kvc_validate(&c, &nul) == KVC_ERR_ARG);
  void* p = (void*)4096;
  void* odd = (void*)4100;
  EXPECT(kvc_workspace_reset(&c, NULL, NULL) == KVC_ERR_ARG && kvc_workspace_reset(&c, odd, NULL) == KVC_ERR_ARG);
  EXPECT(kvc_poll_status(&c, p, NULL, NULL) == KVC_ERR_ARG);
  EXPECT(kvc_check_state(&c, &nul, p, NULL, 0) == KVC_ERR_ARG);
  EXPECT(kvc_block_alloc(&c, &nul, p, p, NULL, 0) == KVC_ERR_ARG && kvc_block_alloc(&c, &st, NULL, p, NULL, 0) == KVC_ERR_ARG);
  EXPECT(kvc_block_free(&c, &st, NULL, NULL, p, NULL, 0) == KVC_ERR_ARG);
  EXPECT(kvc_append(&c, &st, p, p, NULL, 0, 4, p, NULL, 0) == KVC_ERR_ARG);      /* layers */
  EXPECT(kvc_append(&c, &st, p, odd, NULL, 0, 1, p, NULL, 0) == KVC_ERR_ARG);    /* alignment */
  EXPECT(kvc_paged_decode(&c, &st, p, p, 2, 2, 1, p, NULL) == KVC_ERR_ARG);
  EXPECT(kvc_paged_decode(&c, &st, p, p, 0, 1, 1, odd, NULL) == KVC_ERR_ARG);
  EXPECT(kvc_paged_decode(&c, &st, NULL, p, 0, 1, 1, p, NULL) == KVC_ERR_ARG);
  EXPECT(kvc_paged_decode_static(&c, &st, p, NULL, 0, 1, 1, NULL) == KVC_ERR_ARG);
  EXPECT(kvc_paged_decode_planned(&c, &st, p, p, 3, 1, p, NULL) == KVC_ERR_ARG);
  EXPECT(kvc_decode_plan(&c, &st, 2, p, NULL) == KVC_ERR_ARG && kvc_decode_plan(&c, &nul, 0, p, NULL) == KVC_ERR_ARG);
  EXPECT(kvc_metric_reduce(&c, &st, NULL, KVC_KEY_SUM, p, NULL) == KVC_ERR_ARG);
  EXPECT(kvc_metric_reduce(&c, &st, p, 5, p, NULL) == KVC_ERR_ARG);
  EXPECT(kvc_evict_select(&c, &st, p, NULL, p, 1, 1, p, p, p, p, NULL, 0) == KVC_ERR_ARG);   /* nseg != S without offsets */
  EXPECT(kvc_evict_select(&c, &st, p, p, p, 3, 1, p, p, p, p, NULL, 0) == KVC_ERR_ARG);      /* nseg > S */
  EXPECT(kvc_evict_select(&c, &st, p, NULL, p, 2, -1, p, p, p, p, NULL, 0) == KVC_ERR_ARG);
  EXPECT(kvc_compact(&c, &st, NULL, p, NULL, p, NULL, 0) == KVC_ERR_ARG);
  EXPECT(kvc_compact(&c, &st, p, p, (int64_t*)4100, p, NULL, 0) == KVC_ERR_ARG);
  EXPECT(kvc_evict_rank_select(&c, &st, NULL, NULL, 2, 1, p, p, p, NULL, 0) == KVC_ERR_ARG);
  EXPECT(kvc_compact_rank(&c, &st, NULL, NULL, p, NULL, 0) == KVC_ERR_ARG);
  EXPECT(kvc_window_metric(&c, &st, p, NULL, 8, 4, 0, 0, 1, p, NULL) == KVC_ERR_ARG);          /* even pool */
  EXPECT(kvc_window_metric(&c, &st, p, NULL, 0, 7, 0, 0, 1, p, NULL) == KVC_ERR_ARG);
  EXPECT(kvc_window_metric(&c, &st, p, NULL, 65, 7, 0, 0, 1, p, NULL) == KVC_ERR_UNSUPPORTED);  /* too many window queries */
  EXPECT(kvc_query_block_metric(&c, &st, p, NULL, 8, -1, 0, 0, 1, p, NULL) == KVC_ERR_ARG);
  {
    kvc_config d = good(); d.kv_dtype = KVC_F32;
    EXPECT(kvc_window_metric(&d, &st, p, NULL, 8, 7, 0, 0, 1, p, NULL) == KVC_ERR_UNSUPPORTED);
  }
  EXPECT(kvc_count_blocks(&c, &st, 1, 1, p, p, p, NULL) == KVC_ERR_ARG);
  EXPECT(kvc_prefill_alloc(&c, &st, NULL, p, NULL, 0) == KVC_ERR_ARG);
  EXPECT(kvc_preempt(&c, &st, NULL, NULL, p, NULL, 0) == KVC_ERR_ARG);
  EXPECT(kvc_compression_batch(&c, &st, p, NULL, -1, p, NULL, p, NULL) == KVC_ERR_ARG);
  /* measurement hooks */
  int cnt = -1;
  EXPECT(kvc_profile_begin(-1) == KVC_ERR_ARG && kvc_profile_begin(0) == KVC_OK);
  EXPECT(kvc_profile_enable(1) == KVC_OK && kvc_profile_collect(NULL, NULL, NULL, 0, &cnt) == KVC_OK && cnt == 0);
  EXPECT(kvc_profile_collect(NULL, NULL, NULL, 0, NULL) == KVC_ERR_ARG);
  EXPECT(kvc_stream_read_probe(p, 24, (uint32_t*)p, 4, NULL) == KVC_ERR_ARG);
  EXPECT(kvc_stream_read_add_probe(p, (size_t)64 << 20, 1000, 1, (float*)p, 1 << 20, (uint32_t*)p, 4, NULL) == KVC_ERR_ARG);
  EXPECT(kvc_stream_read_add_probe(p, (size_t)64 << 20, (size_t)1 << 20, 1, (float*)p, 100, (uint32_t*)p, 4, NULL) == KVC_ERR_ARG);
  if (failures) { fprintf(stderr, "%d host checks failed\n", failures); return 1; }
  printf("host checks passed\n");
  return 0;
}
