// Eq. 5 (head soft vote): votes[t] = sum_h exp(c * (S[h][t] - max_h)) / sumexp_h.
//
// One thread per token; the H scores of a token are read with loads that are coalesced across the
// wave (consecutive lanes = consecutive tokens of one head row).  All arithmetic after the load is
// double precision (the subtraction of the row maximum is then exact and the exponential is good to
// ~1e-11), so the float scores are the only source of error in a vote; the sum over heads is rounded
// to float once.
#include "ts_kernels.h"

namespace ts {


__global__ __launch_bounds__(256) void soft_vote_kernel(VoteArgs a) {
  __shared__ double s_m[128];
  __shared__ double s_inv[128];
  const int b = blockIdx.y;
  if (a.skip != nullptr && a.skip[b] != 0) return;
  const int N = min(max(a.seq_lens[b], 0), a.max_seq_len);
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (blockIdx.x * 256 >= N) return;
  for (int h = threadIdx.x; h < a.H; h += 256) {
    s_m[h] = (double)a.row_stats[((size_t)b * a.H + h) * 2];
    s_inv[h] = 1.0 / (double)a.row_stats[((size_t)b * a.H + h) * 2 + 1];
  }
  __syncthreads();
  if (t >= N) return;
  const double c = (double)a.scale;
  const float* sp = a.scores + (size_t)b * a.H * a.max_seq_len + t;
  double vote = 0.0;
  int h = 0;
  for (; h + 8 <= a.H; h += 8) {
    float s[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) s[e] = sp[(size_t)(h + e) * a.max_seq_len];
#pragma unroll
    for (int e = 0; e < 8; ++e) vote = fma(exp_f64(c * ((double)s[e] - s_m[h + e])), s_inv[h + e], vote);
  }
  for (; h < a.H; ++h) vote = fma(exp_f64(c * ((double)sp[(size_t)h * a.max_seq_len] - s_m[h])), s_inv[h], vote);
  a.votes[(size_t)b * a.max_seq_len + t] = (float)vote;
}

hipError_t launch_soft_vote(const VoteArgs& a, int B, hipStream_t s) {
  dim3 grid((a.max_seq_len + 255) / 256, B);
  hipLaunchKernelGGL(soft_vote_kernel, grid, dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace ts
