// Algorithm 1's cosine test as a device function of one 256-thread workgroup, shared by the stand-alone check and
// by the score kernels that run the check in their prologue.  The order of every sum is fixed by the thread layout,
// so all workgroups that evaluate the same two vectors take the same decision bit for bit.
#pragma once
#include "ts_common.h"

namespace ts {

// accumulates the dot product and the two squared norms of one 16-byte piece pair
template <int DT>
__device__ __forceinline__ void acc16(uint4 x, uint4 y, double& ab, double& aa, double& bb) {
  if (DT == TS_BF16) {
    const uint32_t xs[4] = {x.x, x.y, x.z, x.w}, ys[4] = {y.x, y.y, y.z, y.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const double x0 = (double)bf16_lo(xs[e]), x1 = (double)bf16_hi(xs[e]);
      const double y0 = (double)bf16_lo(ys[e]), y1 = (double)bf16_hi(ys[e]);
      ab = fma(x0, y0, ab); aa = fma(x0, x0, aa); bb = fma(y0, y0, bb);
      ab = fma(x1, y1, ab); aa = fma(x1, x1, aa); bb = fma(y1, y1, bb);
    }
  } else {
    const uint32_t xs[4] = {x.x, x.y, x.z, x.w}, ys[4] = {y.x, y.y, y.z, y.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const double x0 = (double)__uint_as_float(xs[e]), y0 = (double)__uint_as_float(ys[e]);
      ab = fma(x0, y0, ab); aa = fma(x0, x0, aa); bb = fma(y0, y0, bb);
    }
  }
}

constexpr int kSelcacheKeep = 4;   // 16-byte pieces of Q a thread still holds after the test

// The test in two halves, so that a caller can put other work between the loads and the decision.
// selcache_sums: the vectors are read as 16-byte pieces, four per thread in flight (about one memory round trip);
// the three sums (Q.C_Q, |Q|^2, |C_Q|^2) are accumulated in double precision and left per wave in red.  qkeep
// receives the thread's first pieces of Q.
// selcache_decide: 1 = reselect (first query, or cos(Q, C_Q) < theta; a zero vector gives cos = 0), the same value in
// every thread.  blockDim.x == 256; every thread of the workgroup must call both; red = 12 doubles and flag = one int
// of LDS that nothing else touches in between, free for other use afterwards (selcache_decide ends with a barrier).
template <int DT>
__device__ __forceinline__ void selcache_sums(const uint4* q, const uint4* cq, int npieces, double (*red)[4],
                                              uint4 (&qkeep)[kSelcacheKeep]) {
  constexpr int KEEP = kSelcacheKeep;
  double ab = 0.0, aa = 0.0, bb = 0.0;
  for (int p0 = 0; p0 < npieces; p0 += 256 * KEEP) {
    uint4 x[KEEP], y[KEEP];
#pragma unroll
    for (int e = 0; e < KEEP; ++e) {
      const int p = p0 + e * 256 + threadIdx.x;
      x[e] = make_uint4(0, 0, 0, 0); y[e] = make_uint4(0, 0, 0, 0);
      if (p < npieces) { x[e] = q[p]; y[e] = cq[p]; }
    }
#pragma unroll
    for (int e = 0; e < KEEP; ++e) { acc16<DT>(x[e], y[e], ab, aa, bb); if (p0 == 0) qkeep[e] = x[e]; }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    ab += __shfl_xor(ab, off); aa += __shfl_xor(aa, off); bb += __shfl_xor(bb, off);
  }
  if ((threadIdx.x & 63) == 0) {
    red[0][threadIdx.x >> 6] = ab; red[1][threadIdx.x >> 6] = aa; red[2][threadIdx.x >> 6] = bb;
  }
}

__device__ __forceinline__ int selcache_decide(double (*red)[4], int* flag, int first0, float theta) {
  __syncthreads();
  if (threadIdx.x == 0) {
    const double ab = red[0][0] + red[0][1] + red[0][2] + red[0][3];
    const double aa = red[1][0] + red[1][1] + red[1][2] + red[1][3];
    const double bb = red[2][0] + red[2][1] + red[2][2] + red[2][3];
    const double c = (aa == 0.0 || bb == 0.0) ? 0.0 : ab / (sqrt(aa) * sqrt(bb));
    *flag = ((first0 != 0) || (c < (double)theta)) ? 1 : 0;
  }
  __syncthreads();
  const int reselect = *flag;
  __syncthreads();
  return reselect;
}

template <int DT>
__device__ __forceinline__ int selcache_reselect(const uint4* q, const uint4* cq, int npieces, int first0, float theta,
                                                 double (*red)[4], int* flag, uint4 (&qkeep)[kSelcacheKeep]) {
  selcache_sums<DT>(q, cq, npieces, red, qkeep);
  return selcache_decide(red, flag, first0, theta);
}

}  // namespace ts
