// The two selection functions that the paper ablates against the head soft vote (Sec. 5.1), producing the
// same `votes` vector that ts_topk ranks:
//   Eq. 3 (I_topk)       votes[t] = sum_h S[t][h]                 raw dot products summed over heads
//   Eq. 4 (I_head-vote)  votes[t] = #{h : t in TopK_k(S[:, h])}   every head takes its own top-k
// Eq. 4 runs the radix select of topk.hip once per (sequence, head) over a transposed copy of the score
// matrix (contiguous per head, so that the five passes stream it), and its emit pass counts winners per token
// with float atomics (integers up to H: exact and order-independent) instead of listing them.
#include "ts_kernels.h"

namespace ts {

// Eq. 3: one thread per token, the H scores of its row summed in double in head order, rounded once
__global__ __launch_bounds__(256) void sum_vote_kernel(VoteArgs a) {
  const int b = blockIdx.y;
  const int skip_flag = a.skip != nullptr ? (int)a.skip[b] : 0;   // issued together with the length
  const int N = min(max(a.seq_lens[b], 0), a.max_seq_len);
  if (skip_flag != 0) return;
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t >= N) return;
  const int r_lo = min(a.n_init, N), r_hi = max(r_lo, N - a.n_local);
  const float* sp = a.scores + ((size_t)b * a.max_seq_len + t) * a.H;
  double v = 0.0;
  for (int h = 0; h < a.H; ++h) v += (double)sp[h];
  a.votes[(size_t)b * a.max_seq_len + t] = (t >= r_lo && t < r_hi) ? (float)v : 0.f;
}

// S [b][t][h] -> ST [b * H + h][t] for t < N_b, 64 tokens per workgroup through LDS
__global__ __launch_bounds__(256) void transpose_scores_kernel(VoteArgs a, float* __restrict__ st) {
  __shared__ float tile[64][129];
  const int b = blockIdx.y;
  const int skip_flag = a.skip != nullptr ? (int)a.skip[b] : 0;   // issued together with the length
  const int N = min(max(a.seq_lens[b], 0), a.max_seq_len);
  if (skip_flag != 0) return;
  const int t0 = blockIdx.x * 64;
  if (t0 >= N) return;
  const int H = a.H, nt = min(64, N - t0);
  const float* src = a.scores + ((size_t)b * a.max_seq_len + t0) * H;
  for (int i = threadIdx.x; i < nt * H; i += 256) tile[i / H][i % H] = src[i];   // contiguous rows
  __syncthreads();
  const int tl = threadIdx.x & 63;
  for (int h = threadIdx.x >> 6; h < H; h += 4)
    if (tl < nt) st[((size_t)b * H + h) * a.max_seq_len + t0 + tl] = tile[tl][h];
}

__global__ __launch_bounds__(256) void fill_u32_kernel(uint32_t* p, size_t n, uint32_t v) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) p[i] = v;
}

// votes[b][0..N_b) = 0 for the sequences that are not skipped
__global__ __launch_bounds__(256) void zero_votes_kernel(VoteArgs a) {
  const int b = blockIdx.y;
  const int skip_flag = a.skip != nullptr ? (int)a.skip[b] : 0;   // issued together with the length
  const int N = min(max(a.seq_lens[b], 0), a.max_seq_len);
  if (skip_flag != 0) return;
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t < N) a.votes[(size_t)b * a.max_seq_len + t] = 0.f;
}

hipError_t launch_zero_votes(const VoteArgs& a, int B, hipStream_t s) {
  hipLaunchKernelGGL(zero_votes_kernel, dim3((a.max_seq_len + 255) / 256, B), dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_sum_vote(const VoteArgs& a, int B, hipStream_t s) {
  hipLaunchKernelGGL(sum_vote_kernel, dim3((a.max_seq_len + 255) / 256, B), dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_transpose_scores(const VoteArgs& a, float* st, int B, hipStream_t s) {
  hipLaunchKernelGGL(transpose_scores_kernel, dim3((a.max_seq_len + 63) / 64, B), dim3(256), 0, s, a, st);
  return hipGetLastError();
}

hipError_t launch_fill_u32(uint32_t* p, size_t n, uint32_t v, hipStream_t s) {
  if (n == 0) return hipSuccess;
  size_t blocks = (n + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)blocks), dim3(256), 0, s, p, n, v);
  return hipGetLastError();
}

}  // namespace ts
