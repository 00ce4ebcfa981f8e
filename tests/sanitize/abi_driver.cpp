// Calls every entry point of the C ABI with arguments that its host-side validation
// must turn away before anything is launched, and checks the status codes.  Built by
// tests/test_sanitizers.py against the library's entry-point file compiled with
// -fsanitize=address,undefined on the host side: a validation path that reads past a
// struct, overflows a size computation or dereferences what it should only test aborts
// the run.  No GPU is needed: nothing gets as far as the device.
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "tinyserve.h"

static int failures = 0;
#define EXPECT(call, want)                                                       \
  do {                                                                           \
    const long got_ = (long)(call);                                              \
    if (got_ != (long)(want)) {                                                  \
      printf("FAIL line %d: %s -> %ld, expected %ld\n", __LINE__, #call, got_, (long)(want)); \
      ++failures;                                                                \
    }                                                                            \
  } while (0)

static ts_layout good() {
  ts_layout l;
  memset(&l, 0, sizeof(l));
  l.num_seqs = 2; l.num_q_heads = 8; l.num_kv_heads = 2; l.head_dim = 64; l.page_size = 16;
  l.max_pages_per_seq = 64; l.num_phys_pages = 128;
  void* p = (void*)0x1000;
  l.k_pool = p; l.v_pool = p; l.block_table = (const int32_t*)p; l.seq_lens = (int32_t*)p;
  l.page_min = p; l.page_max = p;
  return l;
}

int main() {
  void* p = (void*)0x1000;
  float* pf = (float*)p;
  int32_t* pi = (int32_t*)p;
  const size_t big = (size_t)1 << 30;
  ts_layout l = good();
  EXPECT(ts_version() >= 1, 1);
  EXPECT(ts_strerror(TS_ERR_WORKSPACE) != NULL, 1);
  EXPECT(ts_strerror(12345) != NULL, 1);
  EXPECT(ts_workspace_bytes(&l, 8) > 0, 1);
  EXPECT(ts_workspace_bytes(&l, 0), 0);
  EXPECT(ts_workspace_bytes(NULL, 8), 0);
  EXPECT(ts_dense_workspace_bytes(&l) > 0, 1);
  EXPECT(ts_score_pages(NULL, p, pf, NULL), TS_ERR_NULL);
  EXPECT(ts_score_pages(&l, NULL, pf, NULL), TS_ERR_NULL);
  EXPECT(ts_build_page_meta(NULL, NULL), TS_ERR_NULL);
  EXPECT(ts_append_token_meta(&l, NULL, NULL, 1, NULL), TS_ERR_NULL);
  EXPECT(ts_select_topk_pages(&l, pf, 0, NULL, 8, pi, pi, NULL), TS_ERR_SHAPE);
  EXPECT(ts_select_topk_pages(&l, pf, 9, NULL, 8, pi, pi, NULL), TS_ERR_SHAPE);
  EXPECT(ts_select_topk_pages(&l, pf, 4, NULL, 8, NULL, pi, NULL), TS_ERR_NULL);
  EXPECT(ts_sparse_decode_attention(&l, p, pi, pi, 8, 1.0f, p, NULL, p, 16, NULL), TS_ERR_WORKSPACE);
  EXPECT(ts_sparse_decode_attention(&l, p, pi, pi, 8, 1.0f, NULL, NULL, p, big, NULL), TS_ERR_NULL);
  EXPECT(ts_query_aware_decode(&l, p, 4, NULL, 8, 1.0f, p, NULL, NULL, NULL, p, 16, NULL), TS_ERR_WORKSPACE);
  EXPECT(ts_query_aware_decode(&l, p, 0, NULL, 8, 1.0f, p, NULL, NULL, NULL, p, big, NULL), TS_ERR_SHAPE);
  EXPECT(ts_query_aware_decode(&l, p, 9, NULL, 8, 1.0f, p, NULL, NULL, NULL, p, big, NULL), TS_ERR_SHAPE);
  EXPECT(ts_query_aware_decode_static(NULL, p, 4, NULL, 8, 1.0f, p, NULL, NULL, NULL, NULL), TS_ERR_NULL);
  EXPECT(ts_append_and_decode(&l, NULL, p, p, 4, NULL, 8, 1.0f, p, NULL, NULL, NULL, p, big, NULL), TS_ERR_NULL);
  EXPECT(ts_append_and_decode(&l, p, p, p, 4, NULL, 8, 1.0f, p, NULL, NULL, NULL, p, 16, NULL), TS_ERR_WORKSPACE);
  EXPECT(ts_append_and_decode_launches(&l, 0), TS_ERR_SHAPE);
  EXPECT(ts_dense_decode_attention(&l, p, 1.0f, p, NULL, p, 16, NULL), TS_ERR_WORKSPACE);
  EXPECT(ts_dense_decode_attention(&l, NULL, 1.0f, p, NULL, p, big, NULL), TS_ERR_NULL);
  EXPECT(ts_workspace_init(NULL, 1024, NULL), TS_ERR_NULL);
  EXPECT(ts_workspace_init(p, 8, NULL), TS_ERR_WORKSPACE);
  EXPECT(ts_workspace_status(NULL, NULL), TS_ERR_NULL);
  EXPECT(ts_debug_xcc_ids(NULL, 8, NULL), TS_ERR_NULL);
  EXPECT(ts_debug_xcc_ids(pi, 0, NULL), TS_ERR_SHAPE);
  EXPECT(ts_set_tuning(1, 0, 0), TS_ERR_SHAPE);
  EXPECT(ts_set_tuning(0, -1, 0), TS_ERR_SHAPE);
  EXPECT(ts_set_tuning(0, 3, 0), TS_OK);
  EXPECT(ts_workspace_bytes(&l, 8) > 0, 1);
  EXPECT(ts_set_tuning(0, 0, 0), TS_OK);
  // every field that the validation looks at, pushed out of range in turn
  { ts_layout x = good(); x.num_seqs = 0; EXPECT(ts_score_pages(&x, p, pf, NULL), TS_ERR_SHAPE); }
  { ts_layout x = good(); x.num_q_heads = 7; EXPECT(ts_build_page_meta(&x, NULL), TS_ERR_SHAPE); }
  { ts_layout x = good(); x.head_dim = 96; EXPECT(ts_workspace_bytes(&x, 8), 0); }
  { ts_layout x = good(); x.page_size = 12; EXPECT(ts_score_pages(&x, p, pf, NULL), TS_ERR_UNSUPPORTED); }
  { ts_layout x = good(); x.num_q_heads = 64; EXPECT(ts_score_pages(&x, p, pf, NULL), TS_ERR_UNSUPPORTED); }
  { ts_layout x = good(); x.max_pages_per_seq = 1 << 20; EXPECT(ts_score_pages(&x, p, pf, NULL), TS_ERR_UNSUPPORTED); }
  { ts_layout x = good(); x.max_pages_per_seq = TS_MAX_PAGES_PER_SEQ; x.num_seqs = 16;
    EXPECT(ts_workspace_bytes(&x, 16384) > 0, 1); EXPECT(ts_dense_workspace_bytes(&x) > 0, 1); }
  { ts_layout x = good(); x.num_seqs = 65535; x.num_kv_heads = 8; EXPECT(ts_score_pages(&x, p, pf, NULL), TS_ERR_UNSUPPORTED); }
  { ts_layout x = good(); x.kv_tile_stride = 512; EXPECT(ts_score_pages(&x, p, pf, NULL), TS_ERR_SHAPE); }
  { ts_layout x = good(); x.kv_tile_stride = 2052; EXPECT(ts_score_pages(&x, p, pf, NULL), TS_ERR_SHAPE); }
  { ts_layout x = good(); x.keep_first_pages = -1; EXPECT(ts_score_pages(&x, p, pf, NULL), TS_ERR_SHAPE); }
  { ts_layout x = good(); x.cluster_size = -1; EXPECT(ts_score_pages(&x, p, pf, NULL), TS_ERR_SHAPE); }
  { ts_layout x = good(); x.wait_limit = -1; EXPECT(ts_score_pages(&x, p, pf, NULL), TS_ERR_SHAPE); }
  { ts_layout x = good(); x.out_format = 7; EXPECT(ts_score_pages(&x, p, pf, NULL), TS_ERR_UNSUPPORTED); }
  { ts_layout x = good(); x.kv_format = 9; EXPECT(ts_score_pages(&x, p, pf, NULL), TS_ERR_UNSUPPORTED); }
  { ts_layout x = good(); x.kv_format = TS_KV_INT8; x.kv_tile_stride = 1024;
    EXPECT(ts_query_aware_decode(&x, p, 4, NULL, 8, 1.0f, p, NULL, NULL, NULL, p, big, NULL), TS_ERR_NULL);
    EXPECT(ts_dense_decode_attention(&x, p, 1.0f, p, NULL, p, big, NULL), TS_ERR_NULL);
    EXPECT(ts_build_page_meta(&x, NULL), TS_ERR_NULL); }
  { ts_layout x = good(); x.page_min = NULL; EXPECT(ts_score_pages(&x, p, pf, NULL), TS_ERR_NULL); }
  { ts_layout x = good(); x.num_seqs = 8; x.num_kv_heads = 4; x.num_q_heads = 16; x.max_pages_per_seq = 16384;
    EXPECT(ts_query_aware_decode_static(&x, p, 512, NULL, 512, 1.0f, p, NULL, NULL, NULL, NULL), TS_ERR_WORKSPACE); }
  if (failures == 0) puts("ok");
  return failures != 0;
}
