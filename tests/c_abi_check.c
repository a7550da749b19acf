/* Compiled as plain C99 by tests/test_abi_host.py: the header must be valid C, and the host-only entry points
 * must link and behave without a GPU. */
#include <stdio.h>
#include <string.h>
#include "tokenselect.h"

int main(void) {
  ts_problem p;
  size_t bytes = 0;
  int32_t dummy = 0;
  memset(&p, 0, sizeof p);
  p.batch = 2; p.chunk = 1; p.num_q_heads = 32; p.num_kv_heads = 8; p.head_dim = 128; p.page_size = 16;
  p.max_seq_len = 131072; p.dtype = TS_BF16;
  p.k_pool = &dummy; p.v_pool = &dummy; p.page_indptr = &dummy; p.page_indices = &dummy; p.seq_lens = &dummy;
  p.num_initial = 128; p.num_local = 512;
  if (ts_version() < 100) return 1;
  if (strcmp(ts_strerror(TS_OK), "ok") != 0) return 2;
  if (ts_workspace_bytes(&p, 2048, &bytes) != TS_OK || bytes == 0) return 3;
  p.head_dim = 96;
  if (ts_workspace_bytes(&p, 2048, &bytes) != TS_ERR_UNSUPPORTED) return 4;
  p.head_dim = 128; p.num_local = -1;
  if (ts_workspace_bytes(&p, 2048, &bytes) != TS_ERR_INVALID_ARG) return 5;
  if (ts_topk(&p, NULL, 1, NULL, NULL, NULL, TS_TOPK_FLAT_VOTES, NULL, 0, NULL) != TS_ERR_INVALID_ARG) return 6;
  printf("c abi ok, workspace %zu bytes\n", bytes);
  return 0;
}
