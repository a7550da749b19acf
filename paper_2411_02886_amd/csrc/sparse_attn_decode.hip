// Eq. 2 (selective sparse attention), decode form: attention of one query per sequence over the
// selected tokens, gathered row by row through the page table (the selection is handed over as k
// indices, never as gathered K/V copies).
//
// Split-k: a workgroup takes 64 selected tokens (kAttnChunk) of one KV head (all G query heads of the group share
// the gathered K and V rows).  For one sequence memory latency, not bandwidth, bounds this step (a few MiB are
// gathered), so every K and V load of a wave is issued before the first multiply; logits use eight
// lanes per K row, a local softmax sits in LDS, the P.V product uses 16-byte V pieces per lane.  With
// thousands of such workgroups (large batches) a workgroup takes several chunks in a row instead (MULTI).  A
// second small kernel merges the (max, sum, partial output) triples of the splits.
#include "ts_kernels.h"
#include "ts_score_math.h"

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

// MULTI: a workgroup takes up to kAttnMaxRun consecutive chunks of 64 tokens (a.nch of them) and folds them into one
// partial with a running (max, sum): the next chunk's K and V rows are in flight while the current chunk is worked
// on.  For batches whose splits alone give thousands of workgroups the step is a throughput problem, and a workgroup
// that loads, then computes, then leaves keeps the memory system busy about half of its life; a plain random gather
// of 256-byte pieces from the same pools runs at 5.9 TB/s.  With few workgroups (one sequence) the single-chunk form
// stays: there the chain of one workgroup is the latency that counts.
template <int DT, int D, int G, bool MULTI>
__global__ __launch_bounds__(256) void sparse_attn_decode_kernel(AttnArgs a) {
  constexpr int ES = AElt<DT>::size;
  constexpr int RB = D * ES;
  constexpr int L = RB / 128;          // 16-byte K loads per lane per row (eight lanes per row)
  constexpr int EPL = 16 / ES;         // elements per 16-byte piece
  constexpr int LPR = RB / 16;         // lanes per V row
  constexpr int RPL = 64 / LPR;        // V rows per wave load
  constexpr int CH = kAttnChunk;       // selected tokens per chunk
  constexpr int WT = CH / 4;           // tokens per wave and chunk
  constexpr int KS = WT / 8;           // K steps per wave (eight rows each)
  constexpr int VS = WT / RPL;         // V loads per lane
  constexpr int NSL = MULTI ? kAttnMaxRun * CH : CH;
  __shared__ long long s_slot[NSL];
  __shared__ float s_p[G][CH];
  __shared__ __attribute__((aligned(16))) float s_red[4 * (64 / (D * AElt<DT>::size / 16))][G][D];   // [wave x row group][head][d]
  __shared__ float s_ml[G][3];         // running max, running sum, factor that rescales what was summed before this chunk

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int split = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
  const int H = a.H;
  // attended list = forced initial tokens [0, f_lo), the cnt selected tokens, forced recent tokens [f_hi, nb)
  const int nb = min(max(a.seq_lens[b], 0), a.max_seq_len);
  const int f_lo = min(a.n_init, nb), f_hi = max(f_lo, nb - a.n_local);
  const int cnt = nb > 0 ? min(max(a.count[b], 0), a.idx_stride) : 0;   // an empty sequence attends nothing, whatever count says: its page table may be empty
  const int total = f_lo + cnt + (nb - f_hi);
  const int span = MULTI ? CH * a.nch : CH;     // a.nch <= kAttnMaxRun
  const int j0 = split * span;
  const int nj = min(max(total - j0, 0), span);
  if (nj <= 0) {                       // nothing attended in this split: publish an empty partial
    if (threadIdx.x < G) {
      float* ml = a.part_ml + (((size_t)b * H + kvh * G + threadIdx.x) * a.nsplit + split) * 2;
      ml[0] = -INFINITY; ml[1] = 0.f;
    }
    return;
  }
  const int nchunk = MULTI ? (nj + CH - 1) / CH : 1;
  if (threadIdx.x < NSL) {             // one thread per list entry of the workgroup's span
    long long slot = -1;
    const int jj = j0 + threadIdx.x;
    if ((int)threadIdx.x < span && jj < total) {
      int t;
      if (jj < f_lo) t = jj;
      else if (jj < f_lo + cnt) t = a.idx[(size_t)b * a.idx_stride + (jj - f_lo)];
      else t = f_hi + (jj - f_lo - cnt);
      t = min(max(t, 0), max(nb, 1) - 1);         // a stale or corrupt index must not leave the page table
      const int page = a.page_indices[a.page_indptr[b] + (t >> a.p_shift)];
      slot = ((long long)page << a.p_shift) + (t & (a.P - 1));
    }
    s_slot[threadIdx.x] = slot;
  }
  // the query pieces of this lane (eight lanes per row, as in the score pass)
  const int j = lane & 7, r = lane >> 3;
  uint4 qraw[G][L];
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int i = 0; i < L; ++i)
      qraw[g][i] = *reinterpret_cast<const uint4*>(a.q + ((size_t)b * H + (size_t)kvh * G + g) * RB + i * 128 + j * 16);
  __syncthreads();

  // ---- every K and V load of a wave and chunk is issued before any arithmetic on it: one memory round trip
  const int piece = lane % LPR, rsub = lane / LPR;
  struct Raw { uint4 k[KS][L]; uint4 v[VS]; bool kvalid[KS]; };
  auto issue = [&](int c, Raw& x) {
    const long long* sl = s_slot + c * CH;
    const long long slot0 = sl[0];     // valid: every chunk of the span holds a token; stands in for the padding rows
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const long long slot = sl[wave * WT + s * 8 + r];
      x.kvalid[s] = slot >= 0;
      const uint8_t* kp = a.k_pool + ((size_t)(x.kvalid[s] ? slot : slot0) * a.H_kv + kvh) * RB + j * 16;
#pragma unroll
      for (int i = 0; i < L; ++i) x.k[s][i] = *reinterpret_cast<const uint4*>(kp + i * 128);
    }
#pragma unroll
    for (int it = 0; it < VS; ++it) {
      const long long slot = sl[wave * WT + it * RPL + rsub];
      x.v[it] = *reinterpret_cast<const uint4*>(a.v_pool + ((size_t)(slot >= 0 ? slot : slot0) * a.H_kv + kvh) * RB + piece * 16);
    }
  };
  Raw cur, nxt;
  issue(0, cur);
  float acc[G][EPL];
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;          // of head threadIdx.x / 8, in the threads of the softmax stage

  for (int c = 0; c < nchunk; ++c) {
    if (MULTI) {
      if (c > 0) __syncthreads();                // the previous chunk's weights have been read by every wave
      if (c + 1 < nchunk) issue(c + 1, nxt);
    }
    // ---- logits
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      float lg[G];
#pragma unroll
      for (int g = 0; g < G; ++g) lg[g] = 0.f;
#pragma unroll
      for (int i = 0; i < L; ++i) {
        if (DT == TS_BF16) {
          // packed bf16 dot products (exact products, float accumulation): a quarter of the instructions of
          // unpacking both operands and multiplying element by element
#pragma unroll
          for (int g = 0; g < G; ++g) {
            Piece<TS_BF16, true>::Q qq; qq.w = qraw[g][i];
            lg[g] = Piece<TS_BF16, true>::dot(cur.k[s][i], qq, lg[g]);
          }
        } else {
          float kf[EPL];
          unpack16<DT>(cur.k[s][i], kf);
#pragma unroll
          for (int g = 0; g < G; ++g) {
            float qf[EPL];
            unpack16<DT>(qraw[g][i], qf);
#pragma unroll
            for (int e = 0; e < EPL; ++e) lg[g] = fmaf(kf[e], qf[e], lg[g]);
          }
        }
      }
#pragma unroll
      for (int g = 0; g < G; ++g) lg[g] = group8_sum(lg[g]);
      float v = lg[0];
#pragma unroll
      for (int g = 1; g < G; ++g) v = (j == g) ? lg[g] : v;
      if (j < G) s_p[j][wave * WT + s * 8 + r] = cur.kvalid[s] ? v * a.sm_scale : -INFINITY;
    }
    __syncthreads();

    // ---- softmax of the chunk against the running maximum: eight lanes per head, eight tokens per lane, the lanes of
    // a head meet through DPP
    if (threadIdx.x < G * 8) {
      constexpr int TPL = CH / 8;                  // tokens per lane
      const int g = threadIdx.x >> 3, part = threadIdx.x & 7;
      float x[TPL];
      float m = -INFINITY;
#pragma unroll
      for (int e = 0; e < TPL; ++e) { x[e] = s_p[g][part + 8 * e]; m = fmaxf(m, x[e]); }
      m = fmaxf(group8_max(m), m_run);             // a chunk holds a token, so m is finite unless every logit is -inf / NaN
      float l = 0.f;
#pragma unroll
      for (int e = 0; e < TPL; ++e) {
        const float p = (x[e] == -INFINITY) ? 0.f : expf(x[e] - m);
        s_p[g][part + 8 * e] = p;
        l += p;
      }
      l = group8_sum(l);
      const float f = (MULTI && m_run != -INFINITY) ? expf(m_run - m) : 0.f;   // nothing summed before the first chunk
      l_run = fmaf(l_run, f, l);
      m_run = m;
      if (part == 0) { s_ml[g][0] = m_run; s_ml[g][1] = l_run; s_ml[g][2] = f; }
    }
    __syncthreads();

    // ---- P.V from the V pieces already in registers
    if (MULTI && c > 0) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float f = s_ml[g][2];
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] *= f;
      }
    }
#pragma unroll
    for (int it = 0; it < VS; ++it) {
      const int jl = wave * WT + it * RPL + rsub;
      float vf[EPL];
      unpack16<DT>(cur.v[it], vf);
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float p = s_p[g][jl];        // 0 for padding rows
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(p, vf[e], acc[g][e]);
      }
    }
    if (MULTI) cur = nxt;
  }
  // lanes with the same piece but different rsub hold partial sums of the same outputs: all of them go to LDS (16-byte
  // stores) and meet there -- a cross-lane exchange of the G * EPL accumulators costs more LDS operations than that,
  // and one strip per wave filled by the row groups in turn (a quarter of the LDS) costs 1-2 us of latency
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int e4 = 0; e4 < EPL / 4; ++e4)
      *reinterpret_cast<float4*>(&s_red[wave * RPL + rsub][g][piece * EPL + e4 * 4]) =
          make_float4(acc[g][e4 * 4], acc[g][e4 * 4 + 1], acc[g][e4 * 4 + 2], acc[g][e4 * 4 + 3]);
  __syncthreads();
  for (int i = threadIdx.x; i < G * D; i += 256) {
    const int g = i / D, d = i % D;
    float o = 0.f;
#pragma unroll
    for (int r4 = 0; r4 < 4 * RPL; ++r4) o += s_red[r4][g][d];
    a.part_out[(((size_t)b * H + kvh * G + g) * a.nsplit + split) * D + d] = o;
  }
  if (threadIdx.x < G) {
    float* ml = a.part_ml + (((size_t)b * H + kvh * G + threadIdx.x) * a.nsplit + split) * 2;
    ml[0] = s_ml[threadIdx.x][0]; ml[1] = s_ml[threadIdx.x][1];
  }
}

// Merges the split partials of one (sequence, head): out = sum_s e^{m_s - M} o_s / sum_s e^{m_s - M} l_s.
// One workgroup of D x kMergeGroups threads per head: thread (d, g) takes the splits g, g + kMergeGroups, ... (eight at a
// time, all loads of a thread in flight together: the step is a chain of memory round trips, not bandwidth), the
// groups' sums meet in LDS.
constexpr int kMergeGroups = 8;
template <int DT, int D>
__global__ __launch_bounds__(D * kMergeGroups) void sparse_attn_merge_kernel(AttnArgs a) {
  __shared__ float s_w[kAttnMaxSplit];
  __shared__ float s_red[2 * D * kMergeGroups / 64];
  __shared__ float s_o[kMergeGroups][D];
  const int h = blockIdx.x, b = blockIdx.y, d = threadIdx.x % D, g = threadIdx.x / D;
  const size_t hb = (size_t)b * a.H + h;
  const float* ml = a.part_ml + hb * a.nsplit * 2;
  const int nb = min(max(a.seq_lens[b], 0), a.max_seq_len);
  const int f_lo = min(a.n_init, nb), f_hi = max(f_lo, nb - a.n_local);
  const int total = f_lo + (nb > 0 ? min(max(a.count[b], 0), a.idx_stride) : 0) + (nb - f_hi);
  const int span = kAttnChunk * a.nch;
  const int ns = min(a.nsplit, (total + span - 1) / span);   // splits that hold tokens
  // the partial outputs do not depend on the weights: their loads go out first
  const float* po = a.part_out + hb * a.nsplit * D + d;
  float v[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) { const int s = g + e * kMergeGroups; v[e] = s < ns ? po[(size_t)s * D] : 0.f; }
  // thread s owns split s (ns <= kAttnMaxSplit <= threads): block maximum, then the weights and their sum
  constexpr int NT = D * kMergeGroups, NW = NT / 64;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float2 mine = make_float2(-INFINITY, 0.f);
  if ((int)threadIdx.x < ns) mine = *reinterpret_cast<const float2*>(ml + 2 * threadIdx.x);
  float M = mine.x;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) M = fmaxf(M, __shfl_xor(M, off));
  if (lane == 0) s_red[wave] = M;
  __syncthreads();
  M = s_red[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) M = fmaxf(M, s_red[w]);
  const float wgt = (int)threadIdx.x < ns ? expf(mine.x - M) : 0.f;
  if ((int)threadIdx.x < ns) s_w[threadIdx.x] = wgt;
  float Lsum = wgt * mine.y;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) Lsum += __shfl_xor(Lsum, off);
  if (lane == 0) s_red[NW + wave] = Lsum;
  __syncthreads();
  Lsum = 0.f;
#pragma unroll
  for (int w = 0; w < NW; ++w) Lsum += s_red[NW + w];
  float o = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) { const int s = g + e * kMergeGroups; if (s < ns) o = fmaf(s_w[s], v[e], o); }
  for (int s0 = 8 * kMergeGroups; s0 < ns; s0 += 8 * kMergeGroups) {      // more than 64 splits (k > 4096)
#pragma unroll
    for (int e = 0; e < 8; ++e) { const int s = s0 + g + e * kMergeGroups; v[e] = s < ns ? po[(size_t)s * D] : 0.f; }
#pragma unroll
    for (int e = 0; e < 8; ++e) { const int s = s0 + g + e * kMergeGroups; if (s < ns) o = fmaf(s_w[s], v[e], o); }
  }
  s_o[g][d] = o;
  __syncthreads();
  if (g != 0) return;
  o = 0.f;
#pragma unroll
  for (int gg = 0; gg < kMergeGroups; ++gg) o += s_o[gg][d];
  const float res = Lsum > 0.f ? o / Lsum : 0.f;
  if (DT == TS_BF16) reinterpret_cast<uint16_t*>(a.out)[hb * D + d] = (uint16_t)f32_to_bf16_bits(res);
  else reinterpret_cast<float*>(a.out)[hb * D + d] = res;
  if (d == 0 && a.lse != nullptr) a.lse[hb] = Lsum > 0.f ? M + logf(Lsum) : -INFINITY;
}

template <int DT, int D>
static hipError_t attn_launch_g(int G, const AttnArgs& a, dim3 grid, hipStream_t s) {
#define TS_CASE(g) case g: if (a.nch > 1) hipLaunchKernelGGL((sparse_attn_decode_kernel<DT, D, g, true>), grid, dim3(256), 0, s, a); \
                   else hipLaunchKernelGGL((sparse_attn_decode_kernel<DT, D, g, false>), grid, dim3(256), 0, s, a); break;
  switch (G) {
    TS_CASE(1) TS_CASE(2) TS_CASE(3) TS_CASE(4) TS_CASE(5) TS_CASE(6) TS_CASE(7) TS_CASE(8)
    default: return hipErrorInvalidValue;
  }
#undef TS_CASE
  hipLaunchKernelGGL((sparse_attn_merge_kernel<DT, D>), dim3(a.H, grid.z), dim3(D * kMergeGroups), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_sparse_attn_decode(int dtype, int D, int G, const AttnArgs& a, int B, hipStream_t s) {
  if (a.nch < 1 || a.nch > kAttnMaxRun) return hipErrorInvalidValue;
  dim3 grid(a.nsplit, a.H_kv, B);
  if (dtype == TS_F32) return D == 64 ? attn_launch_g<TS_F32, 64>(G, a, grid, s) : attn_launch_g<TS_F32, 128>(G, a, grid, s);
  return D == 64 ? attn_launch_g<TS_BF16, 64>(G, a, grid, s) : attn_launch_g<TS_BF16, 128>(G, a, grid, s);
}

}  // namespace ts
