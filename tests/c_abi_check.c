/* Compiled as plain C99 by tests/test_abi_host.py (and again with -fsanitize=address,undefined by
 * tests/test_sanitizers.py): the header must be valid C, and every entry point must turn bad arguments into its
 * documented status on the host, before anything is launched -- no GPU is needed to run this program. */
#include <stdio.h>
#include <string.h>
#include "tokenselect.h"

#define EXPECT(call, status) do { const int32_t got_ = (call); if (got_ != (status)) { \
  printf("line %d: %s returned %d, expected %d\n", __LINE__, #call, (int)got_, (int)(status)); return 1; } } while (0)

int main(void) {
  ts_problem p, c;
  size_t bytes = 0;
  int32_t dummy[64];
  void* x = dummy;                    /* stands for any non-NULL device pointer: nothing dereferences it on the host */
  void* ws = (void*)(uintptr_t)0x100000;   /* 256-byte aligned */
  const size_t big = (size_t)1 << 34;
  memset(dummy, 0, sizeof dummy);
  memset(&p, 0, sizeof p);
  p.batch = 2; p.chunk = 1; p.num_q_heads = 32; p.num_kv_heads = 8; p.head_dim = 128; p.page_size = 16;
  p.max_seq_len = 131072; p.dtype = TS_BF16;
  p.k_pool = x; p.v_pool = x; p.page_indptr = x; p.page_indices = x; p.seq_lens = x;
  p.num_initial = 128; p.num_local = 512;
  if (ts_version() < 100) return 1;
  if (strcmp(ts_strerror(TS_OK), "ok") != 0 || strcmp(ts_strerror(-99), "unknown status") != 0) return 2;
  EXPECT(ts_workspace_bytes(&p, 2048, &bytes), TS_OK);
  if (bytes == 0) return 3;
  EXPECT(ts_workspace_bytes(&p, 2048, NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_workspace_bytes(&p, 0, &bytes), TS_ERR_INVALID_ARG);
  EXPECT(ts_workspace_bytes(NULL, 16, &bytes), TS_ERR_INVALID_ARG);
  EXPECT(ts_workspace_bytes(&p, 40000, &bytes), TS_ERR_UNSUPPORTED);        /* more tokens than the decode attention merges */
  c = p; c.head_dim = 96;      EXPECT(ts_workspace_bytes(&c, 2048, &bytes), TS_ERR_UNSUPPORTED);
  c = p; c.num_local = -1;     EXPECT(ts_workspace_bytes(&c, 2048, &bytes), TS_ERR_INVALID_ARG);
  c = p; c.num_q_heads = 30;   EXPECT(ts_workspace_bytes(&c, 2048, &bytes), TS_ERR_INVALID_ARG);
  c = p; c.dtype = 7;          EXPECT(ts_workspace_bytes(&c, 2048, &bytes), TS_ERR_INVALID_ARG);
  c = p; c.seq_lens = NULL;    EXPECT(ts_workspace_bytes(&c, 2048, &bytes), TS_ERR_INVALID_ARG);
  c = p; c.page_size = 12;     EXPECT(ts_workspace_bytes(&c, 2048, &bytes), TS_ERR_UNSUPPORTED);
  c = p; c.num_kv_heads = 2;   EXPECT(ts_workspace_bytes(&c, 2048, &bytes), TS_ERR_UNSUPPORTED);   /* 16 query heads per KV head */
  EXPECT(ts_workspace_init(NULL, 1024, NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_workspace_init(ws, 0, NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_workspace_init(ws, 1022, NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_workspace_init((char*)ws + 4, 1024, NULL), TS_ERR_INVALID_ARG);

  /* score pass, both forms */
  EXPECT(ts_paged_qk_scores(&p, NULL, x, 1.f, NULL, ws, big, NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_paged_qk_scores(&p, x, NULL, 1.f, NULL, ws, big, NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_paged_qk_scores(&p, x, x, -1.f, NULL, ws, big, NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_paged_qk_scores(&p, x, x, 1.f, NULL, NULL, big, NULL), TS_ERR_WORKSPACE);
  EXPECT(ts_paged_qk_scores(&p, x, x, 1.f, NULL, ws, 64, NULL), TS_ERR_WORKSPACE);
  EXPECT(ts_paged_qk_scores(&p, x, x, 1.f, NULL, (char*)ws + 8, big, NULL), TS_ERR_WORKSPACE);
  c = p; c.chunk = 8;          EXPECT(ts_paged_qk_scores(&c, x, x, 1.f, NULL, ws, big, NULL), TS_ERR_UNSUPPORTED);
  c = p; c.k_pool = NULL;      EXPECT(ts_paged_qk_scores(&c, x, x, 1.f, NULL, ws, big, NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_paged_qk_codes(&p, NULL, x, 1.f, NULL, ws, big, NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_paged_qk_codes(&p, x, NULL, 1.f, NULL, ws, big, NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_paged_qk_codes(&p, x, x, 2e30f, NULL, ws, big, NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_paged_qk_codes(&p, x, x, 1.f, NULL, ws, 4096, NULL), TS_ERR_WORKSPACE);
  c = p; c.chunk = 8;          EXPECT(ts_paged_qk_codes(&c, x, x, 1.f, NULL, ws, big, NULL), TS_ERR_UNSUPPORTED);

  {
    /* the score calls that run Algorithm 1's test themselves: a complete, non-overlapping state or an error */
    static char dev[4][65536];          /* stand-ins for four 16-byte aligned device buffers (never dereferenced) */
    void* qa = (void*)(((uintptr_t)dev[0] + 15) & ~(uintptr_t)15);
    void* ca = (void*)(((uintptr_t)dev[1] + 15) & ~(uintptr_t)15);
    void* cb = (void*)(((uintptr_t)dev[2] + 15) & ~(uintptr_t)15);
    uint8_t* fl = (uint8_t*)dev[3];
    ts_selcache sc, bad;
    sc.cached_q = ca; sc.cached_q_next = cb; sc.first = fl; sc.first_next = fl + 64; sc.reuse = fl + 128; sc.theta = 0.9f;
    EXPECT(ts_paged_qk_scores_checked(&p, qa, NULL, x, 1.f, ws, big, NULL), TS_ERR_INVALID_ARG);
    EXPECT(ts_paged_qk_codes_checked(&p, qa, NULL, x, 1.f, ws, big, NULL), TS_ERR_INVALID_ARG);
    EXPECT(ts_paged_qk_scores_checked(&p, qa, &sc, NULL, 1.f, ws, big, NULL), TS_ERR_INVALID_ARG);
    EXPECT(ts_paged_qk_codes_checked(&p, qa, &sc, x, 1.f, ws, 4096, NULL), TS_ERR_WORKSPACE);
    bad = sc; bad.cached_q_next = NULL;             EXPECT(ts_paged_qk_scores_checked(&p, qa, &bad, x, 1.f, ws, big, NULL), TS_ERR_INVALID_ARG);
    bad = sc; bad.reuse = NULL;                     EXPECT(ts_paged_qk_codes_checked(&p, qa, &bad, x, 1.f, ws, big, NULL), TS_ERR_INVALID_ARG);
    bad = sc; bad.cached_q_next = ca;               EXPECT(ts_paged_qk_codes_checked(&p, qa, &bad, x, 1.f, ws, big, NULL), TS_ERR_INVALID_ARG);   /* one buffer for both states */
    bad = sc; bad.cached_q_next = (char*)ca + 4096; EXPECT(ts_paged_qk_scores_checked(&p, qa, &bad, x, 1.f, ws, big, NULL), TS_ERR_INVALID_ARG);  /* overlapping */
    bad = sc; bad.cached_q_next = qa;               EXPECT(ts_paged_qk_scores_checked(&p, qa, &bad, x, 1.f, ws, big, NULL), TS_ERR_INVALID_ARG);  /* would overwrite the query */
    bad = sc; bad.cached_q = (char*)ca + 2;         EXPECT(ts_paged_qk_codes_checked(&p, qa, &bad, x, 1.f, ws, big, NULL), TS_ERR_INVALID_ARG);   /* not 16-byte aligned */
    bad = sc; bad.first_next = fl + 1;              EXPECT(ts_paged_qk_codes_checked(&p, qa, &bad, x, 1.f, ws, big, NULL), TS_ERR_INVALID_ARG);   /* flags overlap (B = 2) */
  }

  /* votes */
  EXPECT(ts_soft_vote(&p, NULL, 1.f, x, x, NULL, ws, big, NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_soft_vote(&p, x, 1.f, NULL, x, NULL, ws, big, NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_soft_vote(&p, x, 1.f, x, NULL, NULL, ws, big, NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_soft_vote(&p, x, -2.f, x, x, NULL, ws, big, NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_soft_vote(&p, x, 1.f, x, x, NULL, ws, 8, NULL), TS_ERR_WORKSPACE);
  EXPECT(ts_soft_vote_bounds(&p, NULL, 1.f, x, x, x, NULL, ws, big, NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_soft_vote_bounds(&p, x, 1.f, x, NULL, x, NULL, ws, big, NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_soft_vote_bounds(&p, x, 1.f, x, x, x, NULL, NULL, 0, NULL), TS_ERR_WORKSPACE);
  c = p; c.chunk = 2;          EXPECT(ts_soft_vote_bounds(&c, x, 1.f, x, x, x, NULL, ws, big, NULL), TS_ERR_UNSUPPORTED);
  EXPECT(ts_sum_vote(&p, NULL, x, NULL, NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_head_vote_scratch_bytes(&p, NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_head_vote_scratch_bytes(&p, &bytes), TS_OK);
  EXPECT(ts_head_vote(&p, x, 0, x, NULL, ws, big, NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_head_vote(&p, x, 16, x, NULL, ws, 1024, NULL), TS_ERR_WORKSPACE);

  /* top-k, all three entry points */
  EXPECT(ts_topk(&p, NULL, 1, NULL, NULL, NULL, TS_TOPK_FLAT_VOTES, NULL, 0, NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_topk(&p, x, 0, (int32_t*)x, (int32_t*)x, NULL, 0, ws, big, NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_topk(&p, x, 16, (int32_t*)x, (int32_t*)x, NULL, 4, ws, big, NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_topk(&p, x, 16, (int32_t*)x, (int32_t*)x, NULL, 0, ws, 1024, NULL), TS_ERR_WORKSPACE);
  EXPECT(ts_topk_exact(&p, NULL, x, x, 1.f, 16, (int32_t*)x, (int32_t*)x, NULL, NULL, ws, big, NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_topk_exact(&p, x, x, x, 1.f, 0, (int32_t*)x, (int32_t*)x, NULL, NULL, ws, big, NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_topk_exact(&p, x, x, x, 1.f, 16, (int32_t*)x, (int32_t*)x, NULL, NULL, ws, 1024, NULL), TS_ERR_WORKSPACE);
  c = p; c.k_pool = NULL;      EXPECT(ts_topk_exact(&c, x, x, x, 1.f, 16, (int32_t*)x, (int32_t*)x, NULL, NULL, ws, big, NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_topk_noalloc(&p, NULL, 16, (int32_t*)x, (int32_t*)x, NULL, 0, NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_topk_noalloc(&p, x, 16, (int32_t*)x, (int32_t*)x, NULL, 8, NULL), TS_ERR_INVALID_ARG);
  c = p; c.batch = 17; c.max_seq_len = 1000; EXPECT(ts_topk_noalloc(&c, x, 16, (int32_t*)x, (int32_t*)x, NULL, 0, NULL), TS_ERR_UNSUPPORTED);
  c = p; c.batch = 8;          EXPECT(ts_topk_noalloc(&c, x, 16, (int32_t*)x, (int32_t*)x, NULL, 0, NULL), TS_ERR_UNSUPPORTED);   /* 8 x 64 chunks */

  /* Selection Cache, attention, chunk calls */
  EXPECT(ts_selcache_check(&p, x, x, NULL, 0.9f, (uint8_t*)x, NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_selcache_check(&p, x, NULL, (uint8_t*)x, 0.9f, (uint8_t*)x, NULL), TS_ERR_INVALID_ARG);
  c = p; c.chunk = 4;          EXPECT(ts_selcache_check(&c, x, x, (uint8_t*)x, 0.9f, (uint8_t*)x, NULL), TS_ERR_UNSUPPORTED);
  EXPECT(ts_sparse_paged_attn(&p, x, (int32_t*)x, 0, (int32_t*)x, 0.1f, x, NULL, ws, big, NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_sparse_paged_attn(&p, x, NULL, 16, (int32_t*)x, 0.1f, x, NULL, ws, big, NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_sparse_paged_attn(&p, x, (int32_t*)x, 16, (int32_t*)x, 0.1f, x, NULL, ws, 64, NULL), TS_ERR_WORKSPACE);
  EXPECT(ts_sparse_paged_attn(&p, x, (int32_t*)x, 40000, (int32_t*)x, 0.1f, x, NULL, ws, big, NULL), TS_ERR_UNSUPPORTED);
  c = p; c.v_pool = NULL;      EXPECT(ts_sparse_paged_attn(&c, x, (int32_t*)x, 16, (int32_t*)x, 0.1f, x, NULL, ws, big, NULL), TS_ERR_INVALID_ARG);
  c = p; c.chunk = 64;
  EXPECT(ts_chunk_row_stats(&c, NULL, 1.f, x, ws, big, NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_chunk_row_stats(&c, x, 1.f, NULL, ws, big, NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_chunk_row_stats(&c, x, 1.f, x, ws, 64, NULL), TS_ERR_WORKSPACE);
  EXPECT(ts_chunk_row_stats(&p, x, 1.f, x, ws, big, NULL), TS_ERR_UNSUPPORTED);     /* a decode problem */
  EXPECT(ts_chunk_soft_vote(&c, x, NULL, 1.f, x, ws, big, NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_chunk_soft_vote(&c, x, x, 1.f, NULL, ws, big, NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_chunk_mean_query(&c, NULL, x, NULL), TS_ERR_INVALID_ARG);
  c.dtype = TS_F32;            EXPECT(ts_chunk_mean_query(&c, x, x, NULL), TS_ERR_UNSUPPORTED);

  /* tuning knobs */
  EXPECT(ts_debug_set_score_variant(7, 0, 0), TS_ERR_INVALID_ARG);
  EXPECT(ts_debug_set_score_variant(1, 0, 3), TS_ERR_INVALID_ARG);
  EXPECT(ts_debug_set_score_variant(1, 0, 0), TS_OK);
  EXPECT(ts_debug_set_score_variant(2, 0, 0), TS_OK);
  EXPECT(ts_debug_set_codes_path(2, 0), TS_ERR_INVALID_ARG);
  EXPECT(ts_debug_set_codes_path(1, 9), TS_ERR_INVALID_ARG);
  EXPECT(ts_debug_set_codes_path(1, 0), TS_OK);
  EXPECT(ts_debug_set_topk_path(2), TS_ERR_INVALID_ARG);
  EXPECT(ts_debug_set_topk_path(0), TS_OK);
  EXPECT(ts_debug_event_create(NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_debug_event_destroy(NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_debug_event_elapsed_ms(NULL, NULL, NULL), TS_ERR_INVALID_ARG);
  EXPECT(ts_debug_set_score_timing_events(x, NULL), TS_ERR_INVALID_ARG);
  printf("c abi ok, workspace %zu bytes\n", bytes);
  return 0;
}
