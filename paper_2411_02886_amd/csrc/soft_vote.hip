// Eq. 5 (head soft vote): votes[t] = sum_h exp(c * (S[h][t] - max_h)) / sumexp_h.
//
// Up to eight lanes share one token; its H scores are one contiguous row, read as 16-byte pieces
// (a wave load covers whole consecutive rows).  The subtraction of the row maximum, the scaling and the
// argument reduction are double precision (exact difference, no loss to a large argument), the fractional
// power of two is the hardware float exponential, the weighted sum over heads is double again and is rounded
// to float once: a vote carries about 1e-7 relative error on top of what the float scores' own rounding gives.
#include "ts_kernels.h"

namespace ts {


// Merges the per-workgroup (max, sum-exp) partials of one (sequence, head) into row_stats.
// One workgroup per (head, sequence); every partial is loaded at once (one memory round trip), the
// rescaling exponentials and the sum are double precision.
__global__ __launch_bounds__(256) void score_stats_merge_kernel(VoteArgs a) {
  __shared__ float s_m[4];
  __shared__ double s_l[4];
  const int h = blockIdx.x, b = blockIdx.y;
  const int skip_flag = a.skip != nullptr ? (int)a.skip[b] : 0;   // checked after the partials' loads have been issued
  // the partial count is what the score launch recorded in the workspace, whatever the host believes now; every
  // slot is loaded at once (one memory round trip, the slots all exist) and the unused ones are masked afterwards
  const int nparts = min((int)a.hdr[b * 8 + 0], kScoreMaxWg);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  constexpr int PER = kScoreMaxWg / 256;
  float mp[PER], lp[PER];
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int p = threadIdx.x + 256 * i;
    const float2 v = *reinterpret_cast<const float2*>(a.partials + (((size_t)b * kScoreMaxWg + p) * a.H + h) * 2);
    mp[i] = v.x; lp[i] = v.y;
  }
#pragma unroll
  for (int i = 0; i < PER; ++i)
    if (threadIdx.x + 256 * i >= nparts) { mp[i] = -INFINITY; lp[i] = 0.f; }
  if (skip_flag != 0) return;
  float m = mp[0];
#pragma unroll
  for (int i = 1; i < PER; ++i) m = fmaxf(m, mp[i]);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
  if (lane == 0) s_m[wave] = m;
  __syncthreads();
  m = fmaxf(fmaxf(s_m[0], s_m[1]), fmaxf(s_m[2], s_m[3]));
  const double sc = (double)a.scale;
  double l = 0.0;
#pragma unroll
  for (int i = 0; i < PER; ++i)
    if (mp[i] != -INFINITY) l += (double)lp[i] * exp_f64(sc * ((double)mp[i] - (double)m));
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) l += __shfl_xor(l, off);
  if (lane == 0) s_l[wave] = l;
  __syncthreads();
  if (threadIdx.x == 0) {
    a.row_stats_out[((size_t)b * a.H + h) * 2] = m;
    a.row_stats_out[((size_t)b * a.H + h) * 2 + 1] = (float)(s_l[0] + s_l[1] + s_l[2] + s_l[3]);
  }
}

// exp(c * d) for the vote, d = score - row maximum (exact in double), c2 = c * log2(e): the argument is reduced in
// double (t = n + f, |f| <= 1/2, so nothing of the float scores' precision is lost to a large argument), 2^f comes
// from the hardware float exponential (1 ulp) and is scaled by 2^n.  Relative error about 1e-7, the size of the
// rounding of the float vote itself and well below what the float scores' own rounding does to a vote.
__device__ __forceinline__ float vote_exp(double d, double c2) {
  const double t = fmax(d * c2, -1000.0);
  const double n = rint(t);
  const float f = (float)(t - n);
  return ldexpf(__builtin_amdgcn_exp2f(f), (int)n);
}

// LPT lanes share one token row of H scores (stored [token][head]); a lane owns CPL 16-byte chunks.
// A workgroup takes NP passes of 256 / LPT tokens, all score loads issued up front (NP > 1 for long sequences:
// fewer, fatter workgroups, as the dispatch rate of tiny workgroups is what limits the kernel there).
template <int CPL, bool VEC, int NP>
__global__ __launch_bounds__(256) void soft_vote_kernel(VoteArgs a, int lpt_shift) {
  __shared__ double s_m[128];
  __shared__ double s_inv[128];
  const int b = blockIdx.y;
  const int skip_flag = a.skip != nullptr ? (int)a.skip[b] : 0;   // issued together with the length
  const int N = min(max(a.seq_lens[b], 0), a.max_seq_len);
  if (skip_flag != 0) return;
  const int LPT = 1 << lpt_shift;
  const int tpp = 256 >> lpt_shift;                 // tokens per pass
  const int tok0 = blockIdx.x * (tpp * NP);
  if (tok0 >= N) return;
  const int jv = threadIdx.x & (LPT - 1);
  const double c2 = (double)a.scale * 1.44269504088896340736;
  const int H = a.H;
  // statistics of every head: issued together with the score loads
  const float2 stv = *reinterpret_cast<const float2*>(a.row_stats + ((size_t)b * H + min((int)threadIdx.x, H - 1)) * 2);
  float s[NP][CPL][4];
#pragma unroll
  for (int p = 0; p < NP; ++p) {
    const int tc = min(tok0 + p * tpp + (int)(threadIdx.x >> lpt_shift), N - 1);   // out-of-range threads shadow the last token
    const float* sp = a.scores + ((size_t)b * a.max_seq_len + tc) * H;
#pragma unroll
    for (int i = 0; i < CPL; ++i) {
      const int h0 = (jv + i * LPT) * 4;
      if (VEC) {
        const float4 v = *reinterpret_cast<const float4*>(sp + min(h0, H - 4));   // clamped: no branch between loads
        s[p][i][0] = v.x; s[p][i][1] = v.y; s[p][i][2] = v.z; s[p][i][3] = v.w;
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) s[p][i][e] = sp[min(h0 + e, H - 1)];
      }
    }
  }
  if (threadIdx.x < H) { s_m[threadIdx.x] = (double)stv.x; s_inv[threadIdx.x] = 1.0 / (double)stv.y; }
  __syncthreads();
  const int r_lo = min(a.n_init, N), r_hi = max(r_lo, N - a.n_local);
#pragma unroll
  for (int p = 0; p < NP; ++p) {
    const int t = tok0 + p * tpp + (int)(threadIdx.x >> lpt_shift);
    double vote = 0.0;
#pragma unroll
    for (int i = 0; i < CPL; ++i) {
      const int h0 = (jv + i * LPT) * 4;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        // lanes past the last head hold a shadow of heads H-4..H-1: they are skipped, not weighted by zero
        // (a shadowed score can lie far above the maximum of the head it would be compared with: inf * 0)
        if (h0 + e < H) vote = fma((double)vote_exp((double)s[p][i][e] - s_m[h0 + e], c2), s_inv[h0 + e], vote);
      }
    }
    for (int off = 1; off < LPT; off <<= 1) vote += __shfl_xor(vote, off);
    if (t < N && jv == 0) a.votes[(size_t)b * a.max_seq_len + t] = (t >= r_lo && t < r_hi) ? (float)vote : 0.f;
  }
}

// Eq. 5 and the start of the TopK in one launch.  A workgroup of 1024 threads owns kRankTokens consecutive tokens:
// it computes their votes as soft_vote_kernel does (same arithmetic, LPT lanes per token row, four passes of loads in
// flight), counts the top 11 key bits of the ranked tokens' votes in an LDS histogram and adds the non-empty bins to
// one of the replicated global histograms -- one flush per workgroup, spread over kBoundHistCopies copies, so the
// same-address atomics stay few.  (Measured and dropped: merging the score pass's statistics partials inside this
// kernel as well, every workgroup for itself.  At 128K tokens that is 128 KiB of partials per workgroup, 32 MiB of
// L2 reads per launch, and costs the kernel 4.7 us -- what the merge launch costs.)
constexpr int kRankTokens = 512;     // per workgroup: one round of four passes for H = 32, and a workgroup for every CU at 128K tokens

template <int CPL, bool VEC>
__global__ __launch_bounds__(1024) void soft_vote_ranked_kernel(VoteArgs a, int lpt_shift) {
  __shared__ double s_m[128];
  __shared__ double s_inv[128];
  __shared__ uint32_t hist[kTopkBins];
  constexpr int NP = 4;
  const int b = blockIdx.y;
  const int skip_flag = a.skip != nullptr ? (int)a.skip[b] : 0;   // issued together with the length
  const int N = min(max(a.seq_lens[b], 0), a.max_seq_len);
  if (skip_flag != 0) return;
  const int tok0 = blockIdx.x * kRankTokens;
  if (tok0 >= N) return;
  const int H = a.H;
  const double c2 = (double)a.scale * 1.44269504088896340736;
  const int LPT = 1 << lpt_shift;
  const int tpp = 1024 >> lpt_shift;                 // tokens per pass
  const int jv = threadIdx.x & (LPT - 1);
  const int npass = (kRankTokens + tpp - 1) / tpp;   // LPT / 2 passes, one for the narrowest rows
  float s[NP][CPL][4];
  // the scores of a round of NP passes: all loads issued up front
  auto load_round = [&](int p0) {
#pragma unroll
    for (int p = 0; p < NP; ++p) {
      const int tc = min(tok0 + (p0 + p) * tpp + (int)(threadIdx.x >> lpt_shift), N - 1);   // out-of-range threads shadow the last token
      const float* sp = a.scores + ((size_t)b * a.max_seq_len + tc) * H;
#pragma unroll
      for (int i = 0; i < CPL; ++i) {
        const int h0 = (jv + i * LPT) * 4;
        if (VEC) {
          const float4 v = *reinterpret_cast<const float4*>(sp + min(h0, H - 4));   // clamped: no branch between loads
          s[p][i][0] = v.x; s[p][i][1] = v.y; s[p][i][2] = v.z; s[p][i][3] = v.w;
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) s[p][i][e] = sp[min(h0 + e, H - 1)];
        }
      }
    }
  };
  load_round(0);
  for (int i = threadIdx.x; i < kTopkBins; i += 1024) hist[i] = 0u;
  if (threadIdx.x < H) {
    const float2 stv = *reinterpret_cast<const float2*>(a.row_stats + ((size_t)b * H + threadIdx.x) * 2);
    s_m[threadIdx.x] = (double)stv.x; s_inv[threadIdx.x] = 1.0 / (double)stv.y;
  }
  __syncthreads();
  const int r_lo = min(a.n_init, N), r_hi = max(r_lo, N - a.n_local);
  for (int p0 = 0; p0 < npass; p0 += NP) {
    if (tok0 + p0 * tpp >= N) break;
    if (p0 != 0) load_round(p0);
#pragma unroll
    for (int p = 0; p < NP; ++p) {
      if (p0 + p >= npass) break;
      const int tl = (p0 + p) * tpp + (int)(threadIdx.x >> lpt_shift);   // token inside the workgroup's range
      const int t = tl < kRankTokens ? tok0 + tl : N;                     // (a pass of the narrowest rows is wider than the range)
      double vote = 0.0;
#pragma unroll
      for (int i = 0; i < CPL; ++i) {
        const int h0 = (jv + i * LPT) * 4;
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (h0 + e < H) vote = fma((double)vote_exp((double)s[p][i][e] - s_m[h0 + e], c2), s_inv[h0 + e], vote);
      }
      for (int off = 1; off < LPT; off <<= 1) vote += __shfl_xor(vote, off);
      if (t < N && jv == 0) {
        const bool ranked = t >= r_lo && t < r_hi;
        const float vf = ranked ? (float)vote : 0.f;
        a.votes[(size_t)b * a.max_seq_len + t] = vf;
        if (ranked) atomicAdd(&hist[float_key(vf) >> 21], 1u);
      }
    }
  }
  __syncthreads();
  uint32_t* gh = a.rank_hist + ((size_t)b * kBoundHistCopies + (blockIdx.x & (kBoundHistCopies - 1))) * kTopkBins;
  for (int i = threadIdx.x; i < kTopkBins; i += 1024)
    if (hist[i] != 0u) atomicAdd(&gh[i], hist[i]);
}

hipError_t launch_soft_vote_ranked(const VoteArgs& a, int B, hipStream_t s) {
  const int hq = (a.H + 3) / 4;                     // 16-byte chunks per token row
  int lpt_shift = 0;
  while ((1 << lpt_shift) < hq && lpt_shift < 3) ++lpt_shift;
  const int cpl = (hq + (1 << lpt_shift) - 1) >> lpt_shift;   // 1, 2 or 4 for H <= 128
  const bool vec = (a.H % 4 == 0) && (((uintptr_t)a.scores & 15) == 0);
  hipLaunchKernelGGL(score_stats_merge_kernel, dim3(a.H, B), dim3(256), 0, s, a);
  dim3 grid((a.max_seq_len + kRankTokens - 1) / kRankTokens, B);
#define TS_RV(C, V) hipLaunchKernelGGL((soft_vote_ranked_kernel<C, V>), grid, dim3(1024), 0, s, a, lpt_shift)
  if (cpl <= 1) { if (vec) TS_RV(1, true); else TS_RV(1, false); }
  else if (cpl <= 2) { if (vec) TS_RV(2, true); else TS_RV(2, false); }
  else { if (vec) TS_RV(4, true); else TS_RV(4, false); }
#undef TS_RV
  return hipGetLastError();
}

hipError_t launch_stats_merge(const VoteArgs& a, int B, hipStream_t s) {
  hipLaunchKernelGGL(score_stats_merge_kernel, dim3(a.H, B), dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_soft_vote(const VoteArgs& a, int B, hipStream_t s) {
  const int hq = (a.H + 3) / 4;                     // 16-byte chunks per token row
  int lpt_shift = 0;
  while ((1 << lpt_shift) < hq && lpt_shift < 3) ++lpt_shift;
  const int cpl = (hq + (1 << lpt_shift) - 1) >> lpt_shift;   // 1, 2 or 4 for H <= 128
  const bool vec = (a.H % 4 == 0) && (((uintptr_t)a.scores & 15) == 0);
  hipLaunchKernelGGL(score_stats_merge_kernel, dim3(a.H, B), dim3(256), 0, s, a);
  const int tpp = 256 >> lpt_shift;
  const long nwg1 = ((long)a.max_seq_len * B + tpp - 1) / tpp;
  const int np = nwg1 >= 16384 ? 4 : (nwg1 >= 2048 ? 2 : 1);   // passes per workgroup (measured: 1 M tokens 42 -> 32 us with 4)
  dim3 grid((a.max_seq_len + tpp * np - 1) / (tpp * np), B);
#define TS_VOTE(C, V) do { if (np == 4) hipLaunchKernelGGL((soft_vote_kernel<C, V, 4>), grid, dim3(256), 0, s, a, lpt_shift); \
    else if (np == 2) hipLaunchKernelGGL((soft_vote_kernel<C, V, 2>), grid, dim3(256), 0, s, a, lpt_shift); \
    else hipLaunchKernelGGL((soft_vote_kernel<C, V, 1>), grid, dim3(256), 0, s, a, lpt_shift); } while (0)
  if (cpl <= 1) { if (vec) TS_VOTE(1, true); else TS_VOTE(1, false); }
  else if (cpl <= 2) { if (vec) TS_VOTE(2, true); else TS_VOTE(2, false); }
  else { if (vec) TS_VOTE(4, true); else TS_VOTE(4, false); }
#undef TS_VOTE
  return hipGetLastError();
}

}  // namespace ts
