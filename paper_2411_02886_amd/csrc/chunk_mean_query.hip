// Sec. 5.2 (chunk-wise selection during prefill): the query handed to the selection function is the mean
// of the chunk's C queries.  q [B][C][H][D] bf16 -> q_mean [B][1][H][D] bf16.  The sum of up to a few
// thousand bf16 values is exact in double, so the split of the C queries over lane groups does not change
// the result; the mean is rounded to float and then to bf16 (both nearest-even).
#include "ts_kernels.h"

namespace ts {

// A workgroup owns 64 consecutive elements (one 128-byte line of every query row): eight lanes read the line as
// 16-byte pieces, 32 lane groups take the rows c = slice, slice + 32, ... with eight loads in flight each; the 32
// partial sums per element meet in LDS.
__global__ __launch_bounds__(256) void chunk_mean_query_kernel(const uint16_t* __restrict__ q, uint16_t* __restrict__ out,
                                                               int C, int n) {
  __shared__ double part[32][65];
  const int b = blockIdx.y;
  const int piece = threadIdx.x & 7, slice = threadIdx.x >> 3;
  const int i0 = blockIdx.x * 64 + piece * 8;           // n is a multiple of 64
  const uint16_t* src = q + (size_t)b * C * n + i0;
  double s[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) s[e] = 0.0;
  for (int c0 = slice; c0 < C; c0 += 32 * 8) {
    uint4 w[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int c = c0 + u * 32;
      w[u] = c < C ? *reinterpret_cast<const uint4*>(src + (size_t)c * n) : make_uint4(0u, 0u, 0u, 0u);
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      s[0] += (double)bf16_lo(w[u].x); s[1] += (double)bf16_hi(w[u].x);
      s[2] += (double)bf16_lo(w[u].y); s[3] += (double)bf16_hi(w[u].y);
      s[4] += (double)bf16_lo(w[u].z); s[5] += (double)bf16_hi(w[u].z);
      s[6] += (double)bf16_lo(w[u].w); s[7] += (double)bf16_hi(w[u].w);
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) part[slice][piece * 8 + e] = s[e];
  __syncthreads();
  if (threadIdx.x < 64) {
    double tot = 0.0;
#pragma unroll
    for (int r = 0; r < 32; ++r) tot += part[r][threadIdx.x];
    out[(size_t)b * n + blockIdx.x * 64 + threadIdx.x] = (uint16_t)f32_to_bf16_bits((float)(tot / (double)C));
  }
}

hipError_t launch_chunk_mean_query(const void* q, void* out, int B, int C, int n, hipStream_t s) {
  if (n % 64 != 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(chunk_mean_query_kernel, dim3(n / 64, B), dim3(256), 0, s, (const uint16_t*)q, (uint16_t*)out, C, n);
  return hipGetLastError();
}

}  // namespace ts
