// Algorithm 1 (Selection Cache): the cosine test and the C_Q / first-flag update, one workgroup per
// sequence.  The three sums (Q.C_Q, |Q|^2, |C_Q|^2) are accumulated in double precision so that the
// reuse decision is taken on the same value as a plain double-precision evaluation.
#include "ts_kernels.h"
#include "selcache_device.h"

namespace ts {


// One workgroup per sequence.
template <int DT>
__global__ __launch_bounds__(256) void selcache_kernel(SelcacheArgs a) {
  __shared__ double red[3][4];
  __shared__ int s_flag;
  constexpr int ES = DT == TS_BF16 ? 2 : 4;
  constexpr int KEEP = kSelcacheKeep;
  const int b = blockIdx.x;
  const uint4* q = reinterpret_cast<const uint4*>(a.q + (size_t)b * a.n * ES);
  uint4* cq = reinterpret_cast<uint4*>(a.cached_q + (size_t)b * a.n * ES);
  const int npieces = a.n * ES / 16;            // H * D is a multiple of 64, so this is exact
  const int first0 = a.first[b];                // read with the vectors, not after the reduction
  uint4 qkeep[KEEP];
  const int reselect = selcache_reselect<DT>(q, cq, npieces, first0, a.theta, red, &s_flag, qkeep);
  if (threadIdx.x == 0) {
    a.reuse[b] = (uint8_t)(!reselect);
    if (reselect) a.first[b] = 0;
  }
  if (!reselect) return;
  // miss: C_Q <- Q (the first pieces are still in registers)
#pragma unroll
  for (int e = 0; e < KEEP; ++e) {
    const int p = e * 256 + threadIdx.x;
    if (p < npieces) cq[p] = qkeep[e];
  }
  for (int p = 256 * KEEP + threadIdx.x; p < npieces; p += 256) cq[p] = q[p];
}

hipError_t launch_selcache(const SelcacheArgs& a, int B, hipStream_t s) {
  if (a.dtype == TS_BF16) hipLaunchKernelGGL(selcache_kernel<TS_BF16>, dim3(B), dim3(256), 0, s, a);
  else hipLaunchKernelGGL(selcache_kernel<TS_F32>, dim3(B), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace ts
