// Algorithm 1 (Selection Cache): the cosine test and the C_Q / first-flag update, one workgroup per
// sequence.  The three sums (Q.C_Q, |Q|^2, |C_Q|^2) are accumulated in double precision so that the
// reuse decision is taken on the same value as a plain double-precision evaluation.
#include "ts_kernels.h"

namespace ts {


__device__ __forceinline__ double elt_f64(const uint8_t* p, int dtype, int i) {
  if (dtype == TS_BF16) return (double)__uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(p)[i] << 16);
  return (double)reinterpret_cast<const float*>(p)[i];
}

__global__ __launch_bounds__(256) void selcache_kernel(SelcacheArgs a) {
  __shared__ double red[3][4];
  __shared__ int s_reuse;
  const int b = blockIdx.x;
  const size_t esz = a.dtype == TS_BF16 ? 2 : 4;
  const uint8_t* q = a.q + (size_t)b * a.n * esz;
  uint8_t* cq = a.cached_q + (size_t)b * a.n * esz;
  double ab = 0.0, aa = 0.0, bb = 0.0;
  for (int i = threadIdx.x; i < a.n; i += 256) {
    const double x = elt_f64(q, a.dtype, i), y = elt_f64(cq, a.dtype, i);
    ab = fma(x, y, ab); aa = fma(x, x, aa); bb = fma(y, y, bb);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    ab += __shfl_xor(ab, off); aa += __shfl_xor(aa, off); bb += __shfl_xor(bb, off);
  }
  if ((threadIdx.x & 63) == 0) {
    red[0][threadIdx.x >> 6] = ab; red[1][threadIdx.x >> 6] = aa; red[2][threadIdx.x >> 6] = bb;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    ab = red[0][0] + red[0][1] + red[0][2] + red[0][3];
    aa = red[1][0] + red[1][1] + red[1][2] + red[1][3];
    bb = red[2][0] + red[2][1] + red[2][2] + red[2][3];
    const double c = (aa == 0.0 || bb == 0.0) ? 0.0 : ab / (sqrt(aa) * sqrt(bb));
    const int reselect = (a.first[b] != 0) || (c < (double)a.theta);
    s_reuse = !reselect;
    a.reuse[b] = (uint8_t)(!reselect);
    if (reselect) a.first[b] = 0;
  }
  __syncthreads();
  if (s_reuse) return;
  if (a.dtype == TS_BF16) {
    for (int i = threadIdx.x; i < a.n; i += 256)
      reinterpret_cast<uint16_t*>(cq)[i] = reinterpret_cast<const uint16_t*>(q)[i];
  } else {
    for (int i = threadIdx.x; i < a.n; i += 256)
      reinterpret_cast<uint32_t*>(cq)[i] = reinterpret_cast<const uint32_t*>(q)[i];
  }
}

hipError_t launch_selcache(const SelcacheArgs& a, int B, hipStream_t s) {
  hipLaunchKernelGGL(selcache_kernel, dim3(B), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace ts
