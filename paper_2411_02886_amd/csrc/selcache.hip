// Algorithm 1 (Selection Cache): the cosine test and the C_Q / first-flag update, one workgroup per
// sequence.  The three sums (Q.C_Q, |Q|^2, |C_Q|^2) are accumulated in double precision so that the
// reuse decision is taken on the same value as a plain double-precision evaluation.
#include "ts_kernels.h"

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

// One workgroup per sequence.  The vectors are read as 16-byte pieces, four per thread in flight,
// so that the whole test costs about one memory round trip.
template <int DT>
__global__ __launch_bounds__(256) void selcache_kernel(SelcacheArgs a) {
  __shared__ double red[3][4];
  __shared__ int s_reuse;
  constexpr int ES = DT == TS_BF16 ? 2 : 4;
  constexpr int KEEP = 4;
  const int b = blockIdx.x;
  const uint4* q = reinterpret_cast<const uint4*>(a.q + (size_t)b * a.n * ES);
  uint4* cq = reinterpret_cast<uint4*>(a.cached_q + (size_t)b * a.n * ES);
  const int npieces = a.n * ES / 16;            // H * D is a multiple of 64, so this is exact
  const int first0 = a.first[b];                // read with the vectors, not after the reduction
  double ab = 0.0, aa = 0.0, bb = 0.0;
  uint4 qkeep[KEEP];
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
  __syncthreads();
  if (threadIdx.x == 0) {
    ab = red[0][0] + red[0][1] + red[0][2] + red[0][3];
    aa = red[1][0] + red[1][1] + red[1][2] + red[1][3];
    bb = red[2][0] + red[2][1] + red[2][2] + red[2][3];
    const double c = (aa == 0.0 || bb == 0.0) ? 0.0 : ab / (sqrt(aa) * sqrt(bb));
    const int reselect = (first0 != 0) || (c < (double)a.theta);
    s_reuse = !reselect;
    a.reuse[b] = (uint8_t)(!reselect);
    if (reselect) a.first[b] = 0;
  }
  __syncthreads();
  if (s_reuse) return;
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
