/* Built by tests/test_sanitizers.py with -fsanitize=address,undefined: every C entry point of the oracle runs on small
 * inputs held in heap buffers of exactly the size the call may touch, so that a read or write past a documented
 * extent, a signed overflow or a misaligned access stops the program.  A few closed forms are checked on the way
 * (the arithmetic itself is pinned by tests/test_oracle_pins.py). */
#include <stdio.h>
#include "../oracle/tokenselect_oracle.c"

static uint32_t lcg_state = 12345u;
static float rnd(void) { lcg_state = lcg_state * 1664525u + 1013904223u; return ((lcg_state >> 8) & 0xffff) / 32768.0f - 1.0f; }
static uint16_t bf16_of(float f) { uint32_t u; memcpy(&u, &f, 4); u += 0x7fffu + ((u >> 16) & 1u); return (uint16_t)(u >> 16); }
#define CHECK(c) do { if (!(c)) { printf("check failed at line %d: %s\n", __LINE__, #c); return 1; } } while (0)

static int run(int dtype, int H, int H_kv, int D, int P, int64_t N, int k) {
  const int es = dtype == 1 ? 2 : 4;
  const int64_t npages = (N + P - 1) / P > 0 ? (N + P - 1) / P : 1;
  const int64_t rows = npages * P * H_kv;
  void* kp = malloc((size_t)(rows * D * es)); void* vp = malloc((size_t)(rows * D * es));
  void* q = malloc((size_t)(H * D * es)); void* cq = malloc((size_t)(H * D * es));
  int32_t* pages = (int32_t*)malloc(sizeof(int32_t) * (size_t)npages);
  for (int64_t i = 0; i < npages; ++i) pages[i] = (int32_t)(npages - 1 - i);        /* reversed page order */
  for (int64_t i = 0; i < rows * D; ++i) {
    const float a = rnd(), b = rnd();
    if (dtype == 1) { ((uint16_t*)kp)[i] = bf16_of(a); ((uint16_t*)vp)[i] = bf16_of(b); } else { ((float*)kp)[i] = a; ((float*)vp)[i] = b; }
  }
  for (int i = 0; i < H * D; ++i) {
    const float a = rnd();
    if (dtype == 1) { ((uint16_t*)q)[i] = bf16_of(a); ((uint16_t*)cq)[i] = 0; } else { ((float*)q)[i] = a; ((float*)cq)[i] = 0.f; }
  }
  double* S = (double*)malloc(sizeof(double) * (size_t)(H * (N > 0 ? N : 1)));
  oracle_paged_qk_scores(q, kp, dtype, H, H_kv, D, P, pages, N, S);
  double* votes = (double*)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
  double* rmax = (double*)malloc(sizeof(double) * (size_t)H); double* rsum = (double*)malloc(sizeof(double) * (size_t)H);
  if (N > 0) {
    oracle_soft_vote(S, H, N, 0.25, votes, rmax, rsum);
    double tot = 0.0;
    for (int64_t t = 0; t < N; ++t) tot += votes[t];
    CHECK(fabs(tot - H) < 1e-9 * H);                                                /* Eq. 5: the votes sum to H */
  }
  int32_t* idx = (int32_t*)malloc(sizeof(int32_t) * (size_t)k); int32_t count = -1;
  oracle_topk(votes, N, k, idx, &count);
  CHECK(count == (k < N ? k : (int)N));
  for (int j = 1; j < count; ++j) CHECK(idx[j] > idx[j - 1]);
  for (int j = count; j < k; ++j) CHECK(idx[j] == -1);
  uint8_t first = 1;
  CHECK(oracle_selcache_check(q, cq, dtype, (int64_t)H * D, &first, 0.9) == 0 && first == 0);   /* first step: miss */
  CHECK(oracle_selcache_check(q, cq, dtype, (int64_t)H * D, &first, 0.9) == 1);                  /* same query: hit */
  CHECK(fabs(oracle_cosine(q, cq, dtype, (int64_t)H * D) - 1.0) < 1e-12);
  double* out = (double*)malloc(sizeof(double) * (size_t)(H * D)); double* full = (double*)malloc(sizeof(double) * (size_t)(H * D));
  double* lse = (double*)malloc(sizeof(double) * (size_t)H);
  oracle_sparse_attn(q, kp, vp, dtype, H, H_kv, D, P, pages, idx, count, 0, 0, 0.125, out, lse);
  oracle_sparse_attn(q, kp, vp, dtype, H, H_kv, D, P, pages, idx, 0, 0, 0, 0.125, out, NULL);    /* empty selection */
  if (N > 0) {
    int32_t* all = (int32_t*)malloc(sizeof(int32_t) * (size_t)N);
    for (int64_t t = 0; t < N; ++t) all[t] = (int32_t)t;
    oracle_sparse_attn(q, kp, vp, dtype, H, H_kv, D, P, pages, all, (int)N, 0, 0, 0.125, out, lse);
    oracle_full_attn(q, kp, vp, dtype, H, H_kv, D, P, pages, N, 0.125, full);
    for (int i = 0; i < H * D; ++i) CHECK(out[i] == full[i]);                     /* k >= N: Eq. 2 is Eq. 1, bit for bit */
    if (N > 2) {                                                                   /* selected tokens plus "current" ones */
      oracle_sparse_attn(q, kp, vp, dtype, H, H_kv, D, P, pages, all, (int)N - 2, N - 2, 2, 0.125, out, lse);
      for (int i = 0; i < H * D; ++i) CHECK(fabs(out[i] - full[i]) < 1e-12);
    }
    free(all);
  }
  void* qm = malloc((size_t)(H * D * es));
  oracle_mean_query(q, dtype, 1, (int64_t)H * D, qm);                              /* a chunk of one query is that query */
  CHECK(memcmp(qm, q, (size_t)(H * D * es)) == 0);
  free(kp); free(vp); free(q); free(cq); free(pages); free(S); free(votes); free(rmax); free(rsum); free(idx);
  free(out); free(full); free(lse); free(qm);
  return 0;
}

int main(void) {
  int rc = 0;
  rc |= run(0, 8, 2, 64, 16, 100, 7);       /* ragged last page */
  rc |= run(1, 32, 8, 128, 16, 48, 48);     /* bf16, k == N */
  rc |= run(1, 28, 4, 128, 1, 33, 64);      /* page size 1, k > N */
  rc |= run(0, 4, 4, 64, 4, 1, 3);          /* a single token */
  rc |= run(0, 6, 2, 64, 2, 0, 5);          /* an empty sequence */
  if (rc == 0) printf("oracle entry points ran clean under the sanitizers, %d thread(s)\n", oracle_num_threads());
  return rc;
}
