// Eq. 2 (selective sparse attention), decode form: attention of one query per sequence over the
// selected tokens, gathered row by row through the page table (the selection is handed over as k
// indices, never as gathered K/V copies).
//
// Split-k: a workgroup takes 64 selected tokens of one KV head (all G query heads of the group share
// the gathered K and V rows), computes logits with eight lanes per K row, a local softmax in LDS,
// then the P.V product with 16-byte V pieces per lane; the (max, sum, partial output) triples of the
// splits are merged by the last workgroup of a (sequence, KV head) to finish.
#include "ts_kernels.h"

namespace ts {


template <int DT> struct AElt;
template <> struct AElt<TS_F32> { static constexpr int size = 4; };
template <> struct AElt<TS_BF16> { static constexpr int size = 2; };

template <int DT> __device__ __forceinline__ void unpack16(uint4 w, float* f);
template <> __device__ __forceinline__ void unpack16<TS_F32>(uint4 w, float* f) {
  f[0] = __uint_as_float(w.x); f[1] = __uint_as_float(w.y); f[2] = __uint_as_float(w.z); f[3] = __uint_as_float(w.w);
}
template <> __device__ __forceinline__ void unpack16<TS_BF16>(uint4 w, float* f) {
  f[0] = bf16_lo(w.x); f[1] = bf16_hi(w.x); f[2] = bf16_lo(w.y); f[3] = bf16_hi(w.y);
  f[4] = bf16_lo(w.z); f[5] = bf16_hi(w.z); f[6] = bf16_lo(w.w); f[7] = bf16_hi(w.w);
}

template <int DT, int D, int G>
__global__ __launch_bounds__(256) void sparse_attn_decode_kernel(AttnArgs a) {
  constexpr int ES = AElt<DT>::size;
  constexpr int RB = D * ES;
  constexpr int L = RB / 128;          // 16-byte K loads per lane per row (eight lanes per row)
  constexpr int EPL = 16 / ES;         // elements per 16-byte piece
  constexpr int LPR = RB / 16;         // lanes per V row
  constexpr int RPL = 64 / LPR;        // V rows per wave load
  constexpr int CH = kAttnChunk;       // 64 selected tokens per workgroup
  __shared__ long long s_slot[CH];
  __shared__ float s_p[G][CH];
  __shared__ float s_red[4][G][D];
  __shared__ float s_ml[G][2];
  __shared__ int s_last;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int split = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
  const int H = a.H;
  const int cnt = min(max(a.count[b], 0), a.idx_stride);
  const int j0 = split * CH;
  const int nj = min(max(cnt - j0, 0), CH);

  if (nj > 0) {
    if (threadIdx.x < CH) {
      long long slot = -1;
      const int jj = j0 + threadIdx.x;
      if (jj < cnt) {
        int t = a.idx[(size_t)b * a.idx_stride + jj];
        const int nb = min(max(a.seq_lens[b], 1), a.max_seq_len);
        t = min(max(t, 0), nb - 1);                 // a stale or corrupt index must not leave the page table
        const int page = a.page_indices[a.page_indptr[b] + (t >> a.p_shift)];
        slot = ((long long)page << a.p_shift) + (t & (a.P - 1));
      }
      s_slot[threadIdx.x] = slot;
    }
    __syncthreads();

    // ---- logits: eight lanes per K row, eight rows per wave step, two steps per wave
    {
      const int j = lane & 7, r = lane >> 3;
      float qf[G][L][EPL];
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int i = 0; i < L; ++i) {
          const uint8_t* qp = a.q + ((size_t)b * H + (size_t)kvh * G + g) * RB + i * 128 + j * 16;
          unpack16<DT>(*reinterpret_cast<const uint4*>(qp), qf[g][i]);
        }
#pragma unroll
      for (int s = 0; s < CH / 32; ++s) {
        const int jl = (wave * (CH / 32) + s) * 8 + r;
        const long long slot = s_slot[jl];
        float acc[G];
#pragma unroll
        for (int g = 0; g < G; ++g) acc[g] = 0.f;
        if (slot >= 0) {
          const uint8_t* kp = a.k_pool + ((size_t)slot * a.H_kv + kvh) * RB + j * 16;
#pragma unroll
          for (int i = 0; i < L; ++i) {
            float kf[EPL];
            unpack16<DT>(*reinterpret_cast<const uint4*>(kp + i * 128), kf);
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
              for (int e = 0; e < EPL; ++e) acc[g] = fmaf(kf[e], qf[g][i][e], acc[g]);
          }
        }
#pragma unroll
        for (int g = 0; g < G; ++g) acc[g] = group8_sum(acc[g]);
        float v = acc[0];
#pragma unroll
        for (int g = 1; g < G; ++g) v = (j == g) ? acc[g] : v;
        if (j < G) s_p[j][jl] = slot >= 0 ? v * a.sm_scale : -INFINITY;
      }
    }
    __syncthreads();

    // ---- local softmax: wave w normalises heads w, w+4, ...; one lane per token
    for (int g = wave; g < G; g += 4) {
      const float x = s_p[g][lane];
      float m = x;
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
      const float p = (x == -INFINITY) ? 0.f : expf(x - m);
      float l = p;
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) l += __shfl_xor(l, off);
      s_p[g][lane] = p;
      if (lane == 0) { s_ml[g][0] = m; s_ml[g][1] = l; }
    }
    __syncthreads();

    // ---- P.V: wave w takes tokens 16w .. 16w+15; a lane owns one 16-byte piece of the V row
    {
      const int piece = lane % LPR, rsub = lane / LPR;
      float acc[G][EPL];
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
#pragma unroll
      for (int it = 0; it < 16 / RPL; ++it) {
        const int jl = wave * 16 + it * RPL + rsub;
        const long long slot = s_slot[jl];
        if (slot >= 0) {
          float vf[EPL];
          unpack16<DT>(*reinterpret_cast<const uint4*>(a.v_pool + ((size_t)slot * a.H_kv + kvh) * RB + piece * 16), vf);
#pragma unroll
          for (int g = 0; g < G; ++g) {
            const float p = s_p[g][jl];
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(p, vf[e], acc[g][e]);
          }
        }
      }
      // lanes with the same piece but different rsub hold partial sums of the same outputs
#pragma unroll
      for (int off = LPR; off < 64; off <<= 1)
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
          for (int e = 0; e < EPL; ++e) acc[g][e] += __shfl_xor(acc[g][e], off);
      if (rsub == 0) {
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
          for (int e = 0; e < EPL; ++e) s_red[wave][g][piece * EPL + e] = acc[g][e];
      }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < G * D; i += 256) {
      const int g = i / D, d = i % D;
      const float o = s_red[0][g][d] + s_red[1][g][d] + s_red[2][g][d] + s_red[3][g][d];
      a.part_out[(((size_t)b * H + kvh * G + g) * a.nsplit + split) * D + d] = o;
    }
    if (threadIdx.x < G) {
      float* ml = a.part_ml + (((size_t)b * H + kvh * G + threadIdx.x) * a.nsplit + split) * 2;
      ml[0] = s_ml[threadIdx.x][0]; ml[1] = s_ml[threadIdx.x][1];
    }
  } else if (threadIdx.x < G) {
    float* ml = a.part_ml + (((size_t)b * H + kvh * G + threadIdx.x) * a.nsplit + split) * 2;
    ml[0] = -INFINITY; ml[1] = 0.f;
  }

  // ---- last workgroup of this (sequence, KV head): merge the splits
  fence_device();
  __syncthreads();
  if (threadIdx.x == 0) s_last = (atomicAdd(&a.counters[b * a.H_kv + kvh], 1u) == gridDim.x - 1);
  __syncthreads();
  if (!s_last) return;
  fence_device();
  for (int i = threadIdx.x; i < G * D; i += 256) {
    const int g = i / D, d = i % D;
    const size_t hb = (size_t)b * H + kvh * G + g;
    const float* ml = a.part_ml + hb * a.nsplit * 2;
    float M = -INFINITY;
    for (int s = 0; s < a.nsplit; ++s) M = fmaxf(M, __hip_atomic_load(ml + 2 * s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    float Lsum = 0.f, o = 0.f;
    for (int s = 0; s < a.nsplit; ++s) {
      const float ms = __hip_atomic_load(ml + 2 * s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (ms == -INFINITY) continue;
      const float w = expf(ms - M);
      Lsum += w * __hip_atomic_load(ml + 2 * s + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      o += w * __hip_atomic_load(a.part_out + (hb * a.nsplit + s) * D + d, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    const float res = Lsum > 0.f ? o / Lsum : 0.f;
    if (DT == TS_BF16) reinterpret_cast<uint16_t*>(a.out)[hb * D + d] = (uint16_t)f32_to_bf16_bits(res);
    else reinterpret_cast<float*>(a.out)[hb * D + d] = res;
    if (d == 0 && a.lse != nullptr) a.lse[hb] = Lsum > 0.f ? M + logf(Lsum) : -INFINITY;
  }
  if (threadIdx.x == 0) a.counters[b * a.H_kv + kvh] = 0u;
}

template <int DT, int D>
static hipError_t attn_launch_g(int G, const AttnArgs& a, dim3 grid, hipStream_t s) {
#define TS_CASE(g) case g: hipLaunchKernelGGL((sparse_attn_decode_kernel<DT, D, g>), grid, dim3(256), 0, s, a); break;
  switch (G) {
    TS_CASE(1) TS_CASE(2) TS_CASE(3) TS_CASE(4) TS_CASE(5) TS_CASE(6) TS_CASE(7) TS_CASE(8)
    default: return hipErrorInvalidValue;
  }
#undef TS_CASE
  return hipGetLastError();
}

hipError_t launch_sparse_attn_decode(int dtype, int D, int G, const AttnArgs& a, int B, hipStream_t s) {
  dim3 grid(a.nsplit, a.H_kv, B);
  if (dtype == TS_F32) return D == 64 ? attn_launch_g<TS_F32, 64>(G, a, grid, s) : attn_launch_g<TS_F32, 128>(G, a, grid, s);
  return D == 64 ? attn_launch_g<TS_BF16, 64>(G, a, grid, s) : attn_launch_g<TS_BF16, 128>(G, a, grid, s);
}

}  // namespace ts
