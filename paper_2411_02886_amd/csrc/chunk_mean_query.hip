// Sec. 5.2 (chunk-wise selection during prefill): the query handed to the selection function is the mean
// of the chunk's C queries.  q [B][C][H][D] bf16 -> q_mean [B][1][H][D] bf16.  The sum of up to a few
// thousand bf16 values is exact in double, so the split of the C queries over four slices does not change
// the result; the mean is rounded to float and then to bf16 (both nearest-even).
#include "ts_kernels.h"

namespace ts {

__global__ __launch_bounds__(256) void chunk_mean_query_kernel(const uint16_t* __restrict__ q, uint16_t* __restrict__ out,
                                                               int C, int n) {
  __shared__ double part[4][64];
  const int b = blockIdx.y;
  const int e = threadIdx.x & 63, slice = threadIdx.x >> 6;
  const int i = blockIdx.x * 64 + e;
  const int per = (C + 3) / 4;
  const int c0 = slice * per, c1 = min(C, c0 + per);
  double s = 0.0;
  if (i < n) {
    const uint16_t* src = q + (size_t)b * C * n + i;
    for (int c = c0; c < c1; ++c) s += (double)__uint_as_float((uint32_t)src[(size_t)c * n] << 16);
  }
  part[slice][e] = s;
  __syncthreads();
  if (slice == 0 && i < n) {
    const double tot = ((part[0][e] + part[1][e]) + part[2][e]) + part[3][e];
    out[(size_t)b * n + i] = (uint16_t)f32_to_bf16_bits((float)(tot / (double)C));
  }
}

hipError_t launch_chunk_mean_query(const void* q, void* out, int B, int C, int n, hipStream_t s) {
  hipLaunchKernelGGL(chunk_mean_query_kernel, dim3((n + 63) / 64, B), dim3(256), 0, s, (const uint16_t*)q, (uint16_t*)out, C, n);
  return hipGetLastError();
}

}  // namespace ts
