// TopK of Eq. 3-5 as an exact radix select over 32-bit order-preserving keys.
//
// Three histogram passes (11 + 11 + 10 bits) find the key of the k-th largest value: every
// workgroup histograms its 2048-key chunk in LDS, adds the non-empty bins to a global histogram,
// and the last workgroup to finish walks the histogram from the top and fixes the next digit.
// A counting pass then gives every chunk the number of keys above / equal to that key before it,
// and the emit pass writes the winners in token order: all keys above the threshold plus the
// first (k - #above) keys equal to it.  That is the "lower token index wins ties" rule and yields
// ascending indices without a sort.
#include "ts_kernels.h"

namespace ts {


// exclusive prefix sum over the 256 threads of a workgroup; *total receives the sum
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* total, uint32_t* lds /* >= 5 words */) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t incl = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t o = __shfl_up(incl, off);
    if (lane >= off) incl += o;
  }
  __syncthreads();
  if (lane == 63) lds[wave] = incl;
  __syncthreads();
  uint32_t base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const uint32_t x = lds[w];
    if (w < wave) base += x;
    tot += x;
  }
  *total = tot;
  return base + incl - v;
}

__device__ __forceinline__ bool arrive_last(uint32_t* counter, uint32_t nblocks) {
  __shared__ int s_last;
  fence_device();
  __syncthreads();
  if (threadIdx.x == 0) s_last = (atomicAdd(counter, 1u) == nblocks - 1);
  __syncthreads();
  const bool last = s_last != 0;
  if (last) fence_device();
  return last;
}

template <int PASS>
__global__ __launch_bounds__(256) void topk_hist_kernel(TopkArgs a) {
  constexpr int SHIFT = PASS == 0 ? 21 : (PASS == 1 ? 10 : 0);
  constexpr int NB = PASS == 2 ? 1024 : 2048;
  constexpr int HI_SHIFT = PASS == 1 ? 21 : 10;   // bits above this pass's digit (PASS > 0)
  __shared__ uint32_t h[kTopkBins];
  __shared__ uint32_t scan_lds[8];
  const int b = blockIdx.y;
  if (a.skip != nullptr && a.skip[b] != 0) return;
  const int N = min(max(a.seq_lens[b], 0), a.max_seq_len);
  for (int i = threadIdx.x; i < NB; i += 256) h[i] = 0;
  __syncthreads();
  const uint32_t prefix = PASS > 0 ? a.state[b * 4 + 0] : 0u;
  const float* v = a.votes + (size_t)b * a.max_seq_len;
  const int base = blockIdx.x * kTopkChunk;
#pragma unroll
  for (int i = 0; i < kTopkChunk / 256; ++i) {
    const int t = base + i * 256 + threadIdx.x;
    if (t < N) {
      const uint32_t key = float_key(v[t]);
      if (PASS == 0 || (key >> HI_SHIFT) == (prefix >> HI_SHIFT)) atomicAdd(&h[(key >> SHIFT) & (NB - 1)], 1u);
    }
  }
  __syncthreads();
  uint32_t* gh = a.hist + (size_t)b * kTopkBins;
  for (int i = threadIdx.x; i < NB; i += 256)
    if (h[i] != 0) atomicAdd(&gh[i], h[i]);
  if (!arrive_last(&a.counters[b * 2], gridDim.x)) return;

  // last workgroup: walk the global histogram from the top bin down
  uint32_t k_rem;
  if (PASS == 0) k_rem = (uint32_t)min(a.k, N); else k_rem = a.state[b * 4 + 1];
  constexpr int PER = NB / 256;
  uint32_t c[PER];
  uint32_t sum = 0;
#pragma unroll
  for (int e = 0; e < PER; ++e) {   // thread 0 owns the top PER bins, in descending order
    const int bin = NB - 1 - (threadIdx.x * PER + e);
    c[e] = __hip_atomic_load(&gh[bin], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    sum += c[e];
  }
  uint32_t total;
  uint32_t above = block_exclusive_scan(sum, &total, scan_lds);
  if (k_rem == 0) {
    if (threadIdx.x == 0) {
      a.state[b * 4 + 0] = 0xffffffffu; a.state[b * 4 + 1] = 0u;
      if (PASS == 0) a.state[b * 4 + 2] = 0u;
    }
  } else {
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      if (above < k_rem && k_rem <= above + c[e]) {
        const uint32_t bin = NB - 1 - (threadIdx.x * PER + e);
        a.state[b * 4 + 0] = prefix | (bin << SHIFT);
        a.state[b * 4 + 1] = k_rem - above;
        if (PASS == 0) a.state[b * 4 + 2] = k_rem;
      }
      above += c[e];
    }
  }
#pragma unroll
  for (int e = 0; e < PER; ++e) gh[NB - 1 - (threadIdx.x * PER + e)] = 0u;
  if (threadIdx.x == 0) a.counters[b * 2] = 0u;
}

// per chunk: how many keys are above / equal to the threshold; last workgroup turns the per-chunk
// counts into exclusive offsets and publishes count[b]
__global__ __launch_bounds__(256) void topk_count_kernel(TopkArgs a) {
  __shared__ uint32_t scan_lds[8];
  __shared__ uint32_t red[8];
  const int b = blockIdx.y;
  if (a.skip != nullptr && a.skip[b] != 0) return;
  const int N = min(max(a.seq_lens[b], 0), a.max_seq_len);
  const uint32_t thr = a.state[b * 4 + 0];
  const float* v = a.votes + (size_t)b * a.max_seq_len;
  const int base = blockIdx.x * kTopkChunk;
  uint32_t gt = 0, eq = 0;
#pragma unroll
  for (int i = 0; i < kTopkChunk / 256; ++i) {
    const int t = base + i * 256 + threadIdx.x;
    if (t < N) {
      const uint32_t key = float_key(v[t]);
      gt += key > thr;
      eq += key == thr;
    }
  }
  uint32_t packed = gt | (eq << 16);   // a chunk holds 2048 keys: both counts fit in 16 bits
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) packed += __shfl_xor(packed, off);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = packed;
  __syncthreads();
  uint32_t* blk = a.blk + (size_t)b * a.nblk * 2;
  if (threadIdx.x == 0) {
    const uint32_t s = red[0] + red[1] + red[2] + red[3];
    blk[blockIdx.x * 2 + 0] = s & 0xffffu;
    blk[blockIdx.x * 2 + 1] = s >> 16;
  }
  if (!arrive_last(&a.counters[b * 2 + 1], gridDim.x)) return;
  uint32_t carry_gt = 0, carry_eq = 0;
  for (int i0 = 0; i0 < (int)gridDim.x; i0 += 256) {
    const int i = i0 + threadIdx.x;
    uint32_t g = 0, e = 0;
    if (i < (int)gridDim.x) {
      g = __hip_atomic_load(&blk[i * 2 + 0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      e = __hip_atomic_load(&blk[i * 2 + 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    uint32_t tg, te;
    const uint32_t xg = block_exclusive_scan(g, &tg, scan_lds);
    const uint32_t xe = block_exclusive_scan(e, &te, scan_lds);
    if (i < (int)gridDim.x) { blk[i * 2 + 0] = carry_gt + xg; blk[i * 2 + 1] = carry_eq + xe; }
    carry_gt += tg; carry_eq += te;
  }
  if (threadIdx.x == 0) {
    a.count[b] = (int32_t)a.state[b * 4 + 2];
    a.counters[b * 2 + 1] = 0u;
  }
}

// winners of a chunk, in token order
__global__ __launch_bounds__(256) void topk_emit_kernel(TopkArgs a) {
  __shared__ uint32_t scan_lds[8];
  const int b = blockIdx.y;
  if (a.skip != nullptr && a.skip[b] != 0) return;
  const int N = min(max(a.seq_lens[b], 0), a.max_seq_len);
  const uint32_t thr = a.state[b * 4 + 0];
  const uint32_t need_eq = a.state[b * 4 + 1];
  const int k_eff = (int)a.state[b * 4 + 2];
  int32_t* out = a.idx + (size_t)b * a.k;
  if (blockIdx.x == 0)
    for (int i = k_eff + threadIdx.x; i < a.k; i += 256) out[i] = -1;
  const int base = blockIdx.x * kTopkChunk;
  if (base >= N) return;
  const float* v = a.votes + (size_t)b * a.max_seq_len;
  constexpr int PER = kTopkChunk / 256;
  const int t0 = base + threadIdx.x * PER;   // PER consecutive tokens per thread: order is preserved
  uint32_t key[PER];
  uint32_t gt = 0, eq = 0;
#pragma unroll
  for (int e = 0; e < PER; ++e) {
    const int t = t0 + e;
    key[e] = t < N ? float_key(v[t]) : 0u;
    const bool valid = t < N;
    gt += valid && key[e] > thr;
    eq += valid && key[e] == thr;
  }
  uint32_t total;
  const uint32_t ex = block_exclusive_scan(gt | (eq << 16), &total, scan_lds);
  const uint32_t* blk = a.blk + ((size_t)b * a.nblk + blockIdx.x) * 2;
  uint32_t gt_before = blk[0] + (ex & 0xffffu);
  uint32_t eq_before = blk[1] + (ex >> 16);
#pragma unroll
  for (int e = 0; e < PER; ++e) {
    const int t = t0 + e;
    if (t < N) {
      if (key[e] > thr) {
        out[gt_before + min(eq_before, need_eq)] = t;
        ++gt_before;
      } else if (key[e] == thr) {
        if (eq_before < need_eq) out[gt_before + eq_before] = t;
        ++eq_before;
      }
    }
  }
}

hipError_t launch_topk(const TopkArgs& a, int B, hipStream_t s) {
  dim3 grid(a.nblk, B);
  hipLaunchKernelGGL(topk_hist_kernel<0>, grid, dim3(256), 0, s, a);
  hipLaunchKernelGGL(topk_hist_kernel<1>, grid, dim3(256), 0, s, a);
  hipLaunchKernelGGL(topk_hist_kernel<2>, grid, dim3(256), 0, s, a);
  hipLaunchKernelGGL(topk_count_kernel, grid, dim3(256), 0, s, a);
  hipLaunchKernelGGL(topk_emit_kernel, grid, dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace ts
