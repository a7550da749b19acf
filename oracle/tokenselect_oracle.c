/*
 * CPU oracle for the TokenSelect decode / chunked-prefill hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, double-precision statement of what
 * the GPU library must compute.  It shares no code with the HIP path; only tests, the smoke
 * check and the benchmark's cpu_baseline leg may call it.  Every function takes host pointers.
 *
 * Element types: dtype 0 = float32, dtype 1 = bfloat16 stored as uint16 bit patterns; both are
 * widened exactly to double before any arithmetic.
 *
 * Paged layout: pool[page][P][H_kv][D]; logical token t of a sequence lives in physical slot
 * page_indices[t / P] * P + t % P  (the index list I of Algorithm 2, grouped in pages).
 * GQA reading: query head h uses KV head h / (H / H_kv) (contiguous groups).
 *
 * Pins (tests/test_oracle_pins.py): numpy einsum on un-paged arrays, paging invariance, softmax
 * rows summing to one / votes summing to H, H = 1 reducing to an argsort of raw logits, brute
 * force top-k on tiny inputs, constructed ties, k >= N equal to brute-force full attention,
 * Algorithm 1 traced by hand, scipy's softmax, planted tokens recovered; the chunk's mean query against numpy
 * and constructed halfway cases of the bfloat16 rounding.  The paper prints no worked numerical example of
 * this path, so absolute values are pinned by these only.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static double elt(const void* base, int dtype, int64_t i) {
  if (dtype == 1) {
    uint32_t u = ((uint32_t)((const uint16_t*)base)[i]) << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
  }
  return (double)((const float*)base)[i];
}

static int64_t slot_of(const int32_t* page_indices, int P, int64_t t) {
  return (int64_t)page_indices[t / P] * P + t % P;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
  extern int omp_get_max_threads(void);
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Algorithm 2 (Paged Dot Product Kernel): S[h][t] = <Q[h,:], K[I[t], kv(h), :]>, raw, unscaled.
 * q: [H][D]; S: [H][N] doubles. */
void oracle_paged_qk_scores(const void* q, const void* k_pool, int dtype, int H, int H_kv, int D, int P,
                            const int32_t* page_indices, int64_t N, double* S) {
  const int G = H / H_kv;
  for (int h = 0; h < H; ++h) {
    const int hkv = h / G;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < N; ++t) {
      const int64_t row = (slot_of(page_indices, P, t) * H_kv + hkv) * D;
      double s = 0.0;
      for (int d = 0; d < D; ++d) s += elt(q, dtype, (int64_t)h * D + d) * elt(k_pool, dtype, row + d);
      S[(int64_t)h * N + t] = s;
    }
  }
}

/* Eq. 5 (head soft vote): votes[t] = sum_h softmax_t(c * S[h][:])[t].
 * S: [H][N]; votes: [N]; row_max/row_sum (optional, [H]) receive max_t c*S and sum_t exp(c*S - max). */
void oracle_soft_vote(const double* S, int H, int64_t N, double c, double* votes, double* row_max, double* row_sum) {
  for (int64_t t = 0; t < N; ++t) votes[t] = 0.0;
  for (int h = 0; h < H; ++h) {
    const double* s = S + (int64_t)h * N;
    double m = -INFINITY;
    for (int64_t t = 0; t < N; ++t) if (c * s[t] > m) m = c * s[t];
    double z = 0.0;
    for (int64_t t = 0; t < N; ++t) z += exp(c * s[t] - m);
    for (int64_t t = 0; t < N; ++t) votes[t] += exp(c * s[t] - m) / z;
    if (row_max) row_max[h] = m;
    if (row_sum) row_sum[h] = z;
  }
}

/* TopK of Eq. 3-5: the k largest values; equal values are ordered by lower token index first; the
 * chosen indices are returned in ascending order.  count = min(k, N); unused idx slots get -1. */
typedef struct { double v; int32_t i; } vi_t;
static int cmp_desc_then_index(const void* a, const void* b) {
  const vi_t* x = (const vi_t*)a; const vi_t* y = (const vi_t*)b;
  if (x->v > y->v) return -1;
  if (x->v < y->v) return 1;
  return (x->i > y->i) - (x->i < y->i);
}
static int cmp_int(const void* a, const void* b) {
  int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
  return (x > y) - (x < y);
}
void oracle_topk(const double* values, int64_t N, int k, int32_t* idx, int32_t* count) {
  vi_t* a = (vi_t*)malloc(sizeof(vi_t) * (size_t)(N > 0 ? N : 1));
  for (int64_t t = 0; t < N; ++t) { a[t].v = values[t]; a[t].i = (int32_t)t; }
  qsort(a, (size_t)N, sizeof(vi_t), cmp_desc_then_index);
  int n = (int64_t)k < N ? k : (int)N;
  if (n < 0) n = 0;
  for (int j = 0; j < n; ++j) idx[j] = a[j].i;
  qsort(idx, (size_t)n, sizeof(int32_t), cmp_int);
  for (int j = n; j < k; ++j) idx[j] = -1;
  *count = n;
  free(a);
}

/* cos(Q, C_Q) over the flattened H*D vector (the single test of Algorithm 1's condition).
 * A zero-norm operand gives 0. */
double oracle_cosine(const void* a, const void* b, int dtype, int64_t n) {
  double ab = 0.0, aa = 0.0, bb = 0.0;
  for (int64_t i = 0; i < n; ++i) {
    double x = elt(a, dtype, i), y = elt(b, dtype, i);
    ab += x * y; aa += x * x; bb += y * y;
  }
  if (aa == 0.0 || bb == 0.0) return 0.0;
  return ab / (sqrt(aa) * sqrt(bb));
}

/* The condition and the state update of Algorithm 1 without the call of S: returns 1 when the
 * cached selection is reused (not first and cos >= theta); on a miss copies Q into C_Q and clears
 * the first flag.  The caller runs the selection on a miss and stores C_I. */
int oracle_selcache_check(const void* q, void* cached_q, int dtype, int64_t n, uint8_t* first, double theta) {
  int reselect = (*first != 0) || (oracle_cosine(q, cached_q, dtype, n) < theta);
  if (reselect) {
    memcpy(cached_q, q, (size_t)n * (dtype == 1 ? 2 : 4));
    *first = 0;
    return 0;
  }
  return 1;
}

/* Eq. 2 (selective sparse attention) for one query position: for every head
 *   w_j = softmax_j(<Q[h], K[slot(idx[j]), kv(h)]> * sm_scale),  out[h] = sum_j w_j V[slot(idx[j]), kv(h)],
 * j running over idx[0..count) in the order given, followed by the n_extra logical tokens
 * extra_first .. extra_first + n_extra - 1 (the in-chunk "current" tokens of Eq. 2; n_extra = 0 in
 * decode, where the cached tokens already include the current one).
 * q: [H][D]; out: [H][D] doubles; lse (optional): [H] log-sum-exp of the scaled logits. */
void oracle_sparse_attn(const void* q, const void* k_pool, const void* v_pool, int dtype, int H, int H_kv, int D,
                        int P, const int32_t* page_indices, const int32_t* idx, int count,
                        int64_t extra_first, int n_extra, double sm_scale, double* out, double* lse) {
  const int G = H / H_kv;
  const int n = count + n_extra;
  double* logit = (double*)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
  for (int h = 0; h < H; ++h) {
    const int hkv = h / G;
    double m = -INFINITY;
    for (int j = 0; j < n; ++j) {
      const int64_t t = j < count ? (int64_t)idx[j] : extra_first + (j - count);
      const int64_t row = (slot_of(page_indices, P, t) * H_kv + hkv) * D;
      double s = 0.0;
      for (int d = 0; d < D; ++d) s += elt(q, dtype, (int64_t)h * D + d) * elt(k_pool, dtype, row + d);
      logit[j] = s * sm_scale;
      if (logit[j] > m) m = logit[j];
    }
    double z = 0.0;
    for (int j = 0; j < n; ++j) z += exp(logit[j] - m);
    for (int d = 0; d < D; ++d) out[(int64_t)h * D + d] = 0.0;
    for (int j = 0; j < n; ++j) {
      const int64_t t = j < count ? (int64_t)idx[j] : extra_first + (j - count);
      const int64_t row = (slot_of(page_indices, P, t) * H_kv + hkv) * D;
      const double w = exp(logit[j] - m) / z;
      for (int d = 0; d < D; ++d) out[(int64_t)h * D + d] += w * elt(v_pool, dtype, row + d);
    }
    if (lse) lse[h] = n > 0 ? m + log(z) : -INFINITY;
  }
  free(logit);
}

/* Eq. 1 (full SDPA over the N cached tokens) written out on its own: brute force, used only as a pin. */
void oracle_full_attn(const void* q, const void* k_pool, const void* v_pool, int dtype, int H, int H_kv, int D,
                      int P, const int32_t* page_indices, int64_t N, double sm_scale, double* out) {
  const int G = H / H_kv;
  double* p = (double*)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
  for (int h = 0; h < H; ++h) {
    const int hkv = h / G;
    double m = -INFINITY;
    for (int64_t t = 0; t < N; ++t) {
      const int64_t row = (slot_of(page_indices, P, t) * H_kv + hkv) * D;
      double s = 0.0;
      for (int d = 0; d < D; ++d) s += elt(q, dtype, (int64_t)h * D + d) * elt(k_pool, dtype, row + d);
      p[t] = s * sm_scale;
      if (p[t] > m) m = p[t];
    }
    double z = 0.0;
    for (int64_t t = 0; t < N; ++t) z += exp(p[t] - m);
    for (int d = 0; d < D; ++d) out[(int64_t)h * D + d] = 0.0;
    for (int64_t t = 0; t < N; ++t) {
      const int64_t row = (slot_of(page_indices, P, t) * H_kv + hkv) * D;
      const double w = exp(p[t] - m) / z;
      for (int d = 0; d < D; ++d) out[(int64_t)h * D + d] += w * elt(v_pool, dtype, row + d);
    }
  }
  free(p);
}

/* Sec. 5.2 (chunk-wise selection during prefill): the query handed to the selection function is the
 * mean of the chunk's C queries.  q: [C][n] stored elements (n = H * D); out: [n] in the same element
 * type.  The mean is formed in double, rounded to float (nearest-even) and, for bfloat16 storage,
 * rounded once more to bfloat16 (nearest-even): the selection function takes queries in the model's
 * element type. */
void oracle_mean_query(const void* q, int dtype, int C, int64_t n, void* out) {
  for (int64_t i = 0; i < n; ++i) {
    double s = 0.0;
    for (int c = 0; c < C; ++c) s += elt(q, dtype, (int64_t)c * n + i);
    const float f = (float)(s / (double)C);
    if (dtype == 1) {
      uint32_t u;
      memcpy(&u, &f, 4);
      const uint32_t lower_half = u & 0xffffu;
      uint32_t top = u >> 16;
      /* nearest-even: up when the dropped half exceeds one half, or equals it and the kept part is odd */
      if (lower_half > 0x8000u || (lower_half == 0x8000u && (top & 1u))) top += 1u;
      ((uint16_t*)out)[i] = (uint16_t)top;
    } else {
      ((float*)out)[i] = f;
    }
  }
}
