// Eq. 5 (head soft vote): votes[t] = sum_h exp(c * (S[h][t] - max_h)) / sumexp_h.
//
// Up to eight lanes share one token; its H scores are one contiguous row, read as 16-byte pieces
// (a wave load covers whole consecutive rows).  All arithmetic after the load is
// double precision (the subtraction of the row maximum is then exact and the exponential is good to
// ~1e-11), so the float scores are the only source of error in a vote; the sum over heads is rounded
// to float once.
#include "ts_kernels.h"

namespace ts {


// LPT lanes share one token row of H scores (stored [token][head]); a lane owns CPL 16-byte chunks.
template <int CPL, bool VEC>
__global__ __launch_bounds__(256) void soft_vote_kernel(VoteArgs a, int lpt_shift) {
  __shared__ double s_m[128];
  __shared__ double s_inv[128];
  const int b = blockIdx.y;
  if (a.skip != nullptr && a.skip[b] != 0) return;
  const int N = min(max(a.seq_lens[b], 0), a.max_seq_len);
  const int LPT = 1 << lpt_shift;
  const int tpb = 256 >> lpt_shift;                 // tokens per workgroup
  if (blockIdx.x * tpb >= N) return;
  const int jv = threadIdx.x & (LPT - 1);
  const int t = blockIdx.x * tpb + (threadIdx.x >> lpt_shift);
  const int tc = min(t, N - 1);                     // out-of-range threads shadow the last token
  const double c = (double)a.scale;
  const int H = a.H;
  const float* sp = a.scores + ((size_t)b * a.max_seq_len + tc) * H;
  // statistics of every head: issued together with the score loads
  const float2 stv = *reinterpret_cast<const float2*>(a.row_stats + ((size_t)b * H + min((int)threadIdx.x, H - 1)) * 2);
  float s[CPL][4];
#pragma unroll
  for (int i = 0; i < CPL; ++i) {
    const int h0 = (jv + i * LPT) * 4;
    if (VEC) {
      const float4 v = *reinterpret_cast<const float4*>(sp + min(h0, H - 4));   // clamped: no branch between loads
      s[i][0] = v.x; s[i][1] = v.y; s[i][2] = v.z; s[i][3] = v.w;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) s[i][e] = sp[min(h0 + e, H - 1)];
    }
  }
  if (threadIdx.x < H) { s_m[threadIdx.x] = (double)stv.x; s_inv[threadIdx.x] = 1.0 / (double)stv.y; }
  __syncthreads();
  double vote = 0.0;
#pragma unroll
  for (int i = 0; i < CPL; ++i) {
    const int h0 = (jv + i * LPT) * 4;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int hh = min(h0 + e, H - 1);
      const double w = (h0 + e < H) ? s_inv[hh] : 0.0;
      vote = fma(exp_f64(c * ((double)s[i][e] - s_m[hh])), w, vote);
    }
  }
  for (int off = 1; off < LPT; off <<= 1) vote += __shfl_xor(vote, off);
  if (t < N && jv == 0) a.votes[(size_t)b * a.max_seq_len + t] = (float)vote;
}

hipError_t launch_soft_vote(const VoteArgs& a, int B, hipStream_t s) {
  const int hq = (a.H + 3) / 4;                     // 16-byte chunks per token row
  int lpt_shift = 0;
  while ((1 << lpt_shift) < hq && lpt_shift < 3) ++lpt_shift;
  const int cpl = (hq + (1 << lpt_shift) - 1) >> lpt_shift;   // 1, 2 or 4 for H <= 128
  const bool vec = (a.H % 4 == 0) && (((uintptr_t)a.scores & 15) == 0);
  dim3 grid((a.max_seq_len + (256 >> lpt_shift) - 1) / (256 >> lpt_shift), B);
#define TS_VOTE(C, V) hipLaunchKernelGGL((soft_vote_kernel<C, V>), grid, dim3(256), 0, s, a, lpt_shift)
  if (cpl <= 1) { if (vec) TS_VOTE(1, true); else TS_VOTE(1, false); }
  else if (cpl <= 2) { if (vec) TS_VOTE(2, true); else TS_VOTE(2, false); }
  else { if (vec) TS_VOTE(4, true); else TS_VOTE(4, false); }
#undef TS_VOTE
  return hipGetLastError();
}

}  // namespace ts
