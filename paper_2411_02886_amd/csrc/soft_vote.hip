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
  if (blockIdx.x * 256 >= N) return;
  const int t = blockIdx.x * 256 + threadIdx.x;
  const int tc = min(t, N - 1);                     // out-of-range threads shadow the last token
  const double c = (double)a.scale;
  const float* sp = a.scores + (size_t)b * a.H * a.max_seq_len + tc;
  // statistics of every head: issued together with the first batch of score loads
  const float2 stv = *reinterpret_cast<const float2*>(a.row_stats + ((size_t)b * a.H + min((int)threadIdx.x, a.H - 1)) * 2);
  const float st_m = stv.x, st_l = stv.y;
  double vote = 0.0;
  for (int h0 = 0; h0 < a.H; h0 += 32) {
    float s[32];
#pragma unroll
    for (int e = 0; e < 32; ++e) s[e] = sp[(size_t)min(h0 + e, a.H - 1) * a.max_seq_len];   // clamped: no branch between loads
    if (h0 == 0) {
      if (threadIdx.x < a.H) { s_m[threadIdx.x] = (double)st_m; s_inv[threadIdx.x] = 1.0 / (double)st_l; }
      __syncthreads();
    }
#pragma unroll
    for (int e = 0; e < 32; ++e) {
      const int hh = min(h0 + e, a.H - 1);
      const double w = (h0 + e < a.H) ? s_inv[hh] : 0.0;
      vote = fma(exp_f64(c * ((double)s[e] - s_m[hh])), w, vote);
    }
  }
  if (t < N) a.votes[(size_t)b * a.max_seq_len + t] = (float)vote;
}

hipError_t launch_soft_vote(const VoteArgs& a, int B, hipStream_t s) {
  dim3 grid((a.max_seq_len + 255) / 256, B);
  hipLaunchKernelGGL(soft_vote_kernel, grid, dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace ts
