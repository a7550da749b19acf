// Compact form of the decode selection (Algorithm 2 + Eq. 5 + TopK without the score matrix in memory).
//
// The score pass leaves one byte per score -- its distance below the head's maximum inside a block of
// tokens, in quarter octaves of softmax weight, rounded towards the maximum -- the block maxima, and the
// usual per-workgroup softmax statistics.  After the statistics merge (soft_vote.hip):
//   vote_bounds_kernel   turns the bytes into an upper and a lower bound of every token's vote (they differ
//                        by 2^(1/4) plus guards) and histograms the lower bounds;
//   topk_refine_kernel   takes every token whose upper bound reaches the histogram bin of the k-th largest
//                        lower bound -- a superset of the top-k, usually 1.05-1.5 k tokens -- recomputes its
//                        scores from K (exact products, double accumulation) and its vote as Eq. 5 defines
//                        it, and lists (vote key, token) in token order.
// The finishing workgroup of the radix select (topk.hip) then picks the k largest of those votes.  Why the
// candidates are a superset: k tokens have votes >= their lower bounds >= the k-th largest lower bound L_k,
// so the k-th largest vote is >= L_k, and a token of the top-k has upper bound >= its vote >= L_k.
#include "ts_kernels.h"
#include "ts_score_math.h"

namespace ts {

// Guards that keep the bounds valid under rounding.  The byte was formed from the float score of the score pass
// (a few ulp of the largest score away from the exact one that the candidates are re-evaluated with) through a
// float product; the exponent offset of a block is rounded to float; the hardware exponential has 1 ulp; the
// sum over heads rounds H times.
constexpr float kCodeGuard = 1e-3f;               // octaves added to the decoded upper end of a byte ...
constexpr float kScoreGuard = 1.0f / 262144.0f;   // ... plus c2 * |largest maximum| * 2^-18 for the score's own rounding
constexpr float kBoundUp = 1.0002f;               // factor on the summed upper bound
constexpr float kBoundDown = 0.9998f;             // factor on the summed lower bound

// One lane per token: a lane reads its token's H bytes (a wave reads 64 consecutive rows) and sums, head by head,
// weight(block, head) * 2^((byte - 255) / 4): the weight of a byte-255 score of each 32-token block this workgroup
// meets (2^(c2 * (block max - max_h)) / sumexp_h, exponent formed in double) from an LDS table, the power from the
// hardware exponential.  The next 256 tokens' bytes are in flight while the current ones are summed.  The
// workgroup's histogram of the lower bounds is flushed once.
template <int HW>                                // dwords per token row (H / 4); 0 = any H, byte loads
__global__ __launch_bounds__(256) void vote_bounds_kernel(BoundArgs a, int tokens_per_wg) {
  constexpr int BT = kScoreTileTokens;          // tokens per block of the byte form
  constexpr int NW = HW > 0 ? HW : 1;
  __shared__ double s_km[128];                  // c2 * max_h + log2(sumexp_h)
  __shared__ float s_absmax[4];
  __shared__ uint32_t hist[kTopkBins];
  extern __shared__ float s_off[];              // [blocks of this workgroup][H]
  const int b = blockIdx.y;
  const int H = a.H;
  const int tbeg = blockIdx.x * tokens_per_wg;
  uint32_t qn[NW];
  auto load_codes = [&](int t0) {               // rows past the sequence are read too (they exist) and ignored
    if (HW > 0) {
      const int tc = min(t0 + (int)threadIdx.x, a.max_seq_len - 1);
      const uint32_t* cp = reinterpret_cast<const uint32_t*>(a.codes + ((size_t)b * a.max_seq_len + tc) * H);
#pragma unroll
      for (int w = 0; w < NW; ++w) qn[w] = cp[w];
    }
  };
  if (tbeg < a.max_seq_len) load_codes(tbeg);
  const int skip_flag = a.skip != nullptr ? (int)a.skip[b] : 0;
  const int N = min(max(a.seq_lens[b], 0), a.max_seq_len);
  if (skip_flag != 0) return;
  if (tbeg >= N) return;
  const int tend = min(N, tbeg + tokens_per_wg);
  const double c2d = (double)a.scale * 1.44269504088896340736;
  float am = 0.f;
  if (threadIdx.x < H) {
    const float2 st = *reinterpret_cast<const float2*>(a.row_stats + ((size_t)b * H + threadIdx.x) * 2);
    s_km[threadIdx.x] = c2d * (double)st.x + log2((double)st.y);
    am = fabsf(st.x);
  }
  const int blk0 = tbeg / BT, nblk_wg = (tend - 1) / BT - blk0 + 1;
  // block maxima of this workgroup's tokens: loaded before the barrier, turned into weights after it
  float mxb[4];
#pragma unroll
  for (int i4 = 0; i4 < 4; ++i4) {
    const int i = threadIdx.x + i4 * 256;
    mxb[i4] = i < nblk_wg * H ? a.blk_max[((size_t)b * a.nblk + min(blk0 + i / H, a.nblk - 1)) * H + i % H] : 0.f;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) am = fmaxf(am, __shfl_xor(am, off));
  if ((threadIdx.x & 63) == 0) s_absmax[threadIdx.x >> 6] = am;
  for (int i = threadIdx.x; i < kTopkBins; i += 256) hist[i] = 0u;
  __syncthreads();
  am = fmaxf(fmaxf(s_absmax[0], s_absmax[1]), fmaxf(s_absmax[2], s_absmax[3]));
  const float guard = kCodeGuard + (float)c2d * am * kScoreGuard;
  const float lo_scale = kBoundDown * __builtin_amdgcn_exp2f(-0.25f - 2.f * guard);
  for (int i = threadIdx.x; i < nblk_wg * H; i += 256) {
    const int i4 = i >> 8;                      // the first 1024 entries were loaded above
    float m;
    if (i4 < 4) m = i4 == 0 ? mxb[0] : i4 == 1 ? mxb[1] : i4 == 2 ? mxb[2] : mxb[3];
    else m = a.blk_max[((size_t)b * a.nblk + min(blk0 + i / H, a.nblk - 1)) * H + i % H];
    s_off[i] = __builtin_amdgcn_exp2f((float)(c2d * (double)m - s_km[i % H]) + guard);   // exponent <= guard; 0 for an empty block
  }
  __syncthreads();
  // Byte 0 is open towards minus infinity: a head with byte 0 gives no lower bound.  Instead of leaving such heads out
  // of the sum one by one (a compare, a select and an add per score), the most they can have put into the upper sum
  // is taken off once per token: 2^(-255/4) times the sum of the block's weights over the heads, and a weight is at
  // most 2^guard / sumexp_h <= 2^guard.
  const float zero_byte_total = __builtin_amdgcn_exp2f(-63.75f) * (float)H * __builtin_amdgcn_exp2f(guard) * 1.00001f;
  const int r_lo = min(a.n_init, N), r_hi = max(r_lo, N - a.n_local);
  for (int t0 = tbeg; t0 < tend; t0 += 256) {
    uint32_t qc[NW];
#pragma unroll
    for (int w = 0; w < NW; ++w) qc[w] = qn[w];
    if (t0 + 256 < tend) load_codes(t0 + 256);
    const int t = t0 + (int)threadIdx.x;
    const int tblk = min(t, tend - 1) / BT - blk0;
    const float* offp = s_off + tblk * H;
    float up = 0.f;
    if (HW > 0) {
#pragma unroll
      for (int w = 0; w < NW; ++w) {
        const float4 o4 = *reinterpret_cast<const float4*>(offp + w * 4);
        const uint32_t c0 = qc[w] & 255u, c1 = (qc[w] >> 8) & 255u, c2b = (qc[w] >> 16) & 255u, c3 = qc[w] >> 24;
        // 2^((byte - 255) / 4) from the hardware exponential: a 256-entry LDS table read at random addresses by 64 lanes
        // conflicts on its banks and was what bounded the kernel (1M tokens: 15.2 us with the table, 14.2 us without)
        const float p2 = __builtin_amdgcn_exp2f(fmaf((float)c2b, 0.25f, -63.75f));
        const float p3 = __builtin_amdgcn_exp2f(fmaf((float)c3, 0.25f, -63.75f));
        const float p1 = __builtin_amdgcn_exp2f(fmaf((float)c1, 0.25f, -63.75f));
        const float p0 = __builtin_amdgcn_exp2f(fmaf((float)c0, 0.25f, -63.75f));
        up = fmaf(o4.x, p0, up); up = fmaf(o4.y, p1, up);
        up = fmaf(o4.z, p2, up); up = fmaf(o4.w, p3, up);
      }
    } else {
      const uint8_t* cp = a.codes + ((size_t)b * a.max_seq_len + min(t, N - 1)) * H;
      for (int h = 0; h < H; ++h) {
        const uint32_t c = cp[h];
        up = fmaf(offp[h], __builtin_amdgcn_exp2f(fmaf((float)c, 0.25f, -63.75f)), up);
      }
    }
    float lo = fmaxf(up - zero_byte_total, 0.f) * lo_scale;
    up *= kBoundUp;
    if (t < tend) {
      const bool ranked = t >= r_lo && t < r_hi;
      a.vote_hi[(size_t)b * a.max_seq_len + t] = ranked ? up : 0.f;
      if (a.vote_lo != nullptr) a.vote_lo[(size_t)b * a.max_seq_len + t] = ranked ? lo : 0.f;
      if (ranked) atomicAdd(&hist[float_key(lo) >> 21], 1u);
    }
  }
  __syncthreads();
  uint32_t* gh = a.hist + ((size_t)b * kBoundHistCopies + (blockIdx.x % kBoundHistCopies)) * kTopkBins;
  for (int i = threadIdx.x; i < kTopkBins; i += 256)
    if (hist[i] != 0u) atomicAdd(&gh[i], hist[i]);
}

hipError_t launch_vote_bounds(const BoundArgs& a, int B, hipStream_t s) {
  // a workgroup flushes one histogram: 256 tokens each for short sequences, at most about 1024 workgroups per
  // sequence for long ones
  int tpw = (a.max_seq_len + 1023) / 1024;
  if (tpw < 256) tpw = 256;
  tpw = (tpw + 255) / 256 * 256;
  // the table of block factors has to fit beside 11 KiB of static LDS without asking for more than the default 64 KiB
  while (tpw > 256 && (size_t)(tpw / kScoreTileTokens + 1) * a.H * sizeof(float) > 49152) tpw -= 256;
  const int nwg = (a.max_seq_len + tpw - 1) / tpw;
  const size_t lds = (size_t)(tpw / kScoreTileTokens + 1) * a.H * sizeof(float);
  const dim3 grid(nwg, B);
  const int hw = a.vec ? a.H / 4 : 0;
#define TS_VB(W) case W: hipLaunchKernelGGL((vote_bounds_kernel<W>), grid, dim3(256), lds, s, a, tpw); break;
  switch (hw) {
    TS_VB(1) TS_VB(2) TS_VB(3) TS_VB(4) TS_VB(5) TS_VB(6) TS_VB(7) TS_VB(8) TS_VB(10) TS_VB(12) TS_VB(14) TS_VB(16) TS_VB(24) TS_VB(32)
    default: hipLaunchKernelGGL((vote_bounds_kernel<0>), grid, dim3(256), lds, s, a, tpw); break;
  }
#undef TS_VB
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// The refine workgroup has 256 threads, or 1024 when a sequence has few chunks: the candidates of a chunk are few,
// their evaluation is a chain of dependent loads, so every candidate should get a wave step of its own in the
// first round; with many chunks small workgroups keep every chunk resident at once.
// exclusive prefix sum over the threads of the refine workgroup; *total receives the sum
template <int kRefineWaves>
__device__ __forceinline__ uint32_t refine_block_scan(uint32_t v, uint32_t* total, uint32_t* lds /* >= kRefineWaves words */) {
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
  for (int w = 0; w < kRefineWaves; ++w) {
    const uint32_t x = lds[w];
    if (w < wave) base += x;
    tot += x;
  }
  *total = tot;
  return base + incl - v;
}

// bin of the k_rem-th largest key in the replicated 2048-bin histogram (kTopkBins if k_rem == 0); all threads get it
template <int kRefineWaves>
__device__ __forceinline__ uint32_t refine_find_bin(const uint32_t* gh, uint32_t k_rem, uint32_t* lds /* >= kRefineWaves + 1 words */) {
  constexpr int kRefineThreads = kRefineWaves * 64;
  constexpr int PER = kTopkBins / kRefineThreads;
  uint32_t c[PER];
  uint32_t sum = 0;
  // the thread's PER bins are consecutive in memory (descending bin order = ascending address from `lowest`): vector loads
  const int lowest = kTopkBins - PER - (int)threadIdx.x * PER;
#pragma unroll
  for (int e = 0; e < PER; ++e) c[e] = 0u;
#pragma unroll
  for (int r = 0; r < kBoundHistCopies; ++r) {
    uint32_t v[PER];
    if (PER % 4 == 0) {
#pragma unroll
      for (int q4 = 0; q4 < PER / 4; ++q4) {
        const uint4 w = *reinterpret_cast<const uint4*>(gh + r * kTopkBins + lowest + q4 * 4);
        v[q4 * 4] = w.x; v[q4 * 4 + 1] = w.y; v[q4 * 4 + 2] = w.z; v[q4 * 4 + 3] = w.w;
      }
    } else {
#pragma unroll
      for (int q2 = 0; q2 < PER / 2; ++q2) {
        const uint2 w = *reinterpret_cast<const uint2*>(gh + r * kTopkBins + lowest + q2 * 2);
        v[q2 * 2] = w.x; v[q2 * 2 + 1] = w.y;
      }
    }
#pragma unroll
    for (int e = 0; e < PER; ++e) c[e] += v[PER - 1 - e];     // c[e] is bin kTopkBins - 1 - (threadIdx.x * PER + e)
  }
#pragma unroll
  for (int e = 0; e < PER; ++e) sum += c[e];
  uint32_t total;
  uint32_t above = refine_block_scan<kRefineWaves>(sum, &total, lds);
  __syncthreads();
  if (threadIdx.x == 0) lds[kRefineWaves] = kTopkBins;
  __syncthreads();
  if (k_rem != 0) {
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      if (above < k_rem && k_rem <= above + c[e]) lds[kRefineWaves] = kTopkBins - 1 - (threadIdx.x * PER + e);
      above += c[e];
    }
  }
  __syncthreads();
  const uint32_t d = lds[kRefineWaves];
  __syncthreads();
  return d;
}

// exp(c * d) as ts_soft_vote forms it: argument reduced in double, 2^fraction from the float hardware exponential
__device__ __forceinline__ float refine_vote_exp(double d, double c2) {
  const double t = fmax(d * c2, -1000.0);
  const double n = rint(t);
  const float f = (float)(t - n);
  return ldexpf(__builtin_amdgcn_exp2f(f), (int)n);
}

constexpr int ST_KEFF_WORD = 2;   // state word that carries min(k, ranked tokens) to the finishing workgroup

// sum of a double over the 8 lanes of an aligned lane group (both halves through the DPP network)
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v) {
  const long long u = __double_as_longlong(v);
  const int lo = __builtin_amdgcn_update_dpp(0, (int)(u & 0xffffffffLL), CTRL, 0xf, 0xf, true);
  const int hi = __builtin_amdgcn_update_dpp(0, (int)(u >> 32), CTRL, 0xf, 0xf, true);
  return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}
__device__ __forceinline__ double group8_sum_f64(double v) {
  v += dpp_f64<0xB1>(v);    // quad_perm [1,0,3,2]
  v += dpp_f64<0x4E>(v);    // quad_perm [2,3,0,1]
  v += dpp_f64<0x141>(v);   // row_half_mirror
  return v;
}

// exact products of one 16-byte piece of a K row with the matching piece of a query head, accumulated in double
template <int DT>
__device__ __forceinline__ double piece_dot_f64(uint4 k, uint4 q, double acc);
template <>
__device__ __forceinline__ double piece_dot_f64<TS_BF16>(uint4 k, uint4 q, double acc) {
  // a product of two bf16 values is exact in float; the sum runs in double
  acc += (double)(bf16_lo(k.x) * bf16_lo(q.x)); acc += (double)(bf16_hi(k.x) * bf16_hi(q.x));
  acc += (double)(bf16_lo(k.y) * bf16_lo(q.y)); acc += (double)(bf16_hi(k.y) * bf16_hi(q.y));
  acc += (double)(bf16_lo(k.z) * bf16_lo(q.z)); acc += (double)(bf16_hi(k.z) * bf16_hi(q.z));
  acc += (double)(bf16_lo(k.w) * bf16_lo(q.w)); acc += (double)(bf16_hi(k.w) * bf16_hi(q.w));
  return acc;
}
template <>
__device__ __forceinline__ double piece_dot_f64<TS_F32>(uint4 k, uint4 q, double acc) {
  acc = fma((double)__uint_as_float(k.x), (double)__uint_as_float(q.x), acc);
  acc = fma((double)__uint_as_float(k.y), (double)__uint_as_float(q.y), acc);
  acc = fma((double)__uint_as_float(k.z), (double)__uint_as_float(q.z), acc);
  acc = fma((double)__uint_as_float(k.w), (double)__uint_as_float(q.w), acc);
  return acc;
}

template <int DT, int D, int G, int kRefineThreads>
__global__ __launch_bounds__(kRefineThreads) void topk_refine_kernel(RefineArgs a) {
  constexpr int kRefineWaves = kRefineThreads / 64;
  constexpr int ES = Elt<DT>::size;
  constexpr int RB = D * ES;
  constexpr int L = RB / 128;
  constexpr int PER = kTopkChunk / kRefineThreads;
  constexpr int UB = DT == TS_F32 ? 2 : 4;      // wave steps whose K rows are in flight together
  __shared__ uint32_t lds[kRefineWaves + 2];
  __shared__ uint32_t scan_lds[kRefineWaves];
  __shared__ int ctok[kTopkChunk];
  __shared__ int cpid[kTopkChunk];
  __shared__ double s_m[128];
  __shared__ double s_inv[128];
  extern __shared__ uint4 q_lds[];              // the sequence's query, [H][row bytes]
  const TopkArgs& ta = a.t;
  const int b = blockIdx.y;
  const int skip_flag = ta.skip != nullptr ? (int)ta.skip[b] : 0;
  const int Nb = min(max(ta.seq_lens[b], 0), ta.max_seq_len);
  const int indptr = a.page_indptr[b];
  if (skip_flag != 0) return;
  const int LO = min(ta.head, Nb), N = max(LO, Nb - ta.tail);      // ranked range [LO, N)
  const uint32_t k_eff = (uint32_t)min(ta.k, N - LO);
  const int H = a.H;
  // a.parts workgroups share a chunk: each finds the threshold and compacts the chunk for itself (cheap, and the same
  // in all of them), then re-evaluates its share of the candidates -- few chunks then still fill the machine
  const int chunk = blockIdx.x / a.parts, part = blockIdx.x - chunk * a.parts;
  const int base = chunk * kTopkChunk;
  const int t0 = base + threadIdx.x * PER;      // PER consecutive tokens per thread: order is preserved
  const float* v = ta.votes + (size_t)b * ta.max_seq_len;
  uint32_t key[PER];
  bool valid[PER];
  if (PER % 4 == 0 && ((reinterpret_cast<uintptr_t>(v) & 15) == 0) && base + kTopkChunk <= ta.max_seq_len) {
    // the usual case: the chunk's upper bounds as 16-byte loads (the row exists up to max_seq_len)
#pragma unroll
    for (int q4 = 0; q4 < PER / 4; ++q4) {
      const float4 w = *reinterpret_cast<const float4*>(v + t0 + q4 * 4);
      const float x[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int e = q4 * 4 + i;
        valid[e] = (t0 + e) >= LO && (t0 + e) < N;
        key[e] = valid[e] ? float_key(x[i]) : 0u;
      }
    }
  } else {
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      valid[e] = (t0 + e) >= LO && (t0 + e) < N;
      key[e] = valid[e] ? float_key(v[t0 + e]) : 0u;
    }
  }
  if (threadIdx.x < H) {
    const float2 st = *reinterpret_cast<const float2*>(a.row_stats + ((size_t)b * H + threadIdx.x) * 2);
    s_m[threadIdx.x] = (double)st.x; s_inv[threadIdx.x] = 1.0 / (double)st.y;
  }
  // the sequence's query goes to LDS as floats ([H][D]): a product then costs one conversion and one double fma
  for (int i = threadIdx.x; i < H * (RB / 16); i += kRefineThreads) {
    const uint4 w = reinterpret_cast<const uint4*>(a.q + (size_t)b * H * RB)[i];
    if (DT == TS_BF16) {
      q_lds[2 * i] = make_uint4(w.x << 16, w.x & 0xffff0000u, w.y << 16, w.y & 0xffff0000u);
      q_lds[2 * i + 1] = make_uint4(w.z << 16, w.z & 0xffff0000u, w.w << 16, w.w & 0xffff0000u);
    } else {
      q_lds[i] = w;
    }
  }
  const uint32_t d0 = refine_find_bin<kRefineWaves>(ta.bound_hist + (size_t)b * kBoundHistCopies * kTopkBins, k_eff, lds);

  if (blockIdx.x == 0 && threadIdx.x == 0) ta.state[b * 8 + ST_KEFF_WORD] = k_eff;
  uint32_t n = 0;
#pragma unroll
  for (int e = 0; e < PER; ++e) n += valid[e] && (key[e] >> 21) >= d0;      // d0 == kTopkBins (empty selection) matches nothing
  uint32_t total;
  uint32_t pos = refine_block_scan<kRefineWaves>(n, &total, scan_lds);
  const int npages = (Nb + a.P - 1) >> a.p_shift;
#pragma unroll
  for (int e = 0; e < PER; ++e)
    if (valid[e] && (key[e] >> 21) >= d0) {
      ctok[pos] = t0 + e;
      cpid[pos] = a.page_indices[indptr + min((t0 + e) >> a.p_shift, npages - 1)];
      ++pos;
    }
  if (threadIdx.x == 0 && part == 0) ta.blk[(size_t)b * ta.nblk + chunk] = total;
  __syncthreads();
  if (total == 0) return;

  // ---- votes of the candidates from exact scores: a wave step covers 8 K rows = HB KV heads of 8 / HB candidates
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j = lane & 7, r = lane >> 3;
  const int HB = a.HB;
  const int kvh_l = r & (HB - 1);
  const int tis = r >> a.hb_shift;
  const int tps_shift = 3 - a.hb_shift;
  const int ngroups = ((int)total + (1 << tps_shift) - 1) >> tps_shift;
  const double c2d = (double)a.scale * 1.44269504088896340736;
  uint2* list = ta.list + ((size_t)b * ta.nblk + chunk) * kTopkChunk;
  const int g_begin = (int)((long)part * ngroups / a.parts), g_end = (int)((long)(part + 1) * ngroups / a.parts);   // this workgroup's groups
  for (int g0 = g_begin + wave; g0 < g_end; g0 += kRefineWaves * UB) {   // group uu of this round: g0 + uu * kRefineWaves
    // groups of this round that exist (the same for the whole wave): the others cost neither loads nor arithmetic
    const int nact = min(UB, (g_end - g0 + kRefineWaves - 1) / kRefineWaves);
    double vote[UB];
#pragma unroll
    for (int uu = 0; uu < UB; ++uu) vote[uu] = 0.0;
    for (int u = 0; u < a.NU; ++u) {
      const int kvh = u * HB + kvh_l;
      uint4 kr[UB][L];
#pragma unroll
      for (int uu = 0; uu < UB; ++uu) {
        if (uu >= nact) continue;
        const int ci = min(((g0 + uu * kRefineWaves) << tps_shift) + tis, (int)total - 1);
        const int t = ctok[ci], pid = cpid[ci];
        const uint8_t* kp = a.k_pool + (((size_t)pid << a.p_shift) + (size_t)(t & (a.P - 1))) * ((size_t)a.H_kv * RB) +
                            (size_t)kvh * RB + j * 16;
#pragma unroll
        for (int i = 0; i < L; ++i) kr[uu][i] = *reinterpret_cast<const uint4*>(kp + i * 128);
      }
      double svv[UB];
#pragma unroll
      for (int uu = 0; uu < UB; ++uu) svv[uu] = 0.0;
      constexpr int EPP = 16 / ES;               // elements per 16-byte piece of K
#pragma unroll
      for (int uu = 0; uu < UB; ++uu) {
        if (uu >= nact) continue;
        // the candidate's K pieces as doubles, once for all G query heads of the row's KV head
        double kd[L][EPP];
#pragma unroll
        for (int i = 0; i < L; ++i) {
          const uint4 k4 = kr[uu][i];
          if (DT == TS_BF16) {
            kd[i][0] = (double)bf16_lo(k4.x); kd[i][1] = (double)bf16_hi(k4.x); kd[i][2] = (double)bf16_lo(k4.y); kd[i][3] = (double)bf16_hi(k4.y);
            kd[i][4 % EPP] = (double)bf16_lo(k4.z); kd[i][5 % EPP] = (double)bf16_hi(k4.z); kd[i][6 % EPP] = (double)bf16_lo(k4.w); kd[i][7 % EPP] = (double)bf16_hi(k4.w);
          } else {
            kd[i][0] = (double)__uint_as_float(k4.x); kd[i][1] = (double)__uint_as_float(k4.y);
            kd[i][2] = (double)__uint_as_float(k4.z); kd[i][3] = (double)__uint_as_float(k4.w);
          }
        }
#pragma unroll 1
        for (int g = 0; g < G; ++g) {           // one query head at a time: its elements come from LDS as floats
          const float* qf = reinterpret_cast<const float*>(q_lds) + (size_t)(kvh * G + g) * D + j * EPP;
          double pc[L];                          // independent chains (products of two floats are exact in double)
#pragma unroll
          for (int i = 0; i < L; ++i) {
            double acc = 0.0;
#pragma unroll
            for (int e4 = 0; e4 < EPP / 4; ++e4) {
              const float4 q4 = *reinterpret_cast<const float4*>(qf + i * (128 / ES) + e4 * 4);
              acc = fma(kd[i][e4 * 4], (double)q4.x, acc); acc = fma(kd[i][e4 * 4 + 1], (double)q4.y, acc);
              acc = fma(kd[i][e4 * 4 + 2], (double)q4.z, acc); acc = fma(kd[i][e4 * 4 + 3], (double)q4.w, acc);
            }
            pc[i] = acc;
          }
          double sc = pc[0];
#pragma unroll
          for (int i = 1; i < L; ++i) sc += pc[i];
          sc = group8_sum_f64(sc);                // the eight lanes of the row
          svv[uu] = (j == g) ? sc : svv[uu];
        }
      }
#pragma unroll
      for (int uu = 0; uu < UB; ++uu) {
        if (uu >= nact) continue;
        const double sv = svv[uu];
        const int hh = min(kvh * G + j, H - 1);
        double term = (j < G) ? (double)refine_vote_exp(sv - s_m[hh], c2d) * s_inv[hh] : 0.0;
        // sum over the lanes of this candidate: the eight lanes of a row, then the HB rows
        term = group8_sum_f64(term);
        for (int off = 8; off < (8 << a.hb_shift); off <<= 1) term += __shfl_xor(term, off);
        vote[uu] += term;
      }
    }
#pragma unroll
    for (int uu = 0; uu < UB; ++uu) {
      const int ci = ((g0 + uu * kRefineWaves) << tps_shift) + tis;
      if (uu < nact && ci < (int)total && kvh_l == 0 && j == 0) list[ci] = make_uint2(float_key((float)vote[uu]), (uint32_t)ctok[ci]);
    }
  }
}

template <int DT, int D, int GG, int NT>
static hipError_t refine_launch(const RefineArgs& a, dim3 grid, hipStream_t s) {
  const size_t lds = (size_t)a.H * D * sizeof(float);     // the query as floats in LDS (next to about 19 KiB of static LDS)
  if (lds > 40960) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&topk_refine_kernel<DT, D, GG, NT>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL((topk_refine_kernel<DT, D, GG, NT>), grid, dim3(NT), lds, s, a);
  return hipGetLastError();
}

template <int DT, int D, int GG>
static hipError_t refine_one(const RefineArgs& a, dim3 grid, hipStream_t s) {
  // few chunks: one fat workgroup per CU at most anyway, so take 16 waves per chunk (bf16; the fp32 form needs the
  // registers); many chunks: small workgroups, so that all of them are resident at once (a workgroup's run is one
  // chain of dependent loads, about 10 us, whatever its size)
  if (DT == TS_BF16 && (long)grid.x * grid.y <= 256) return refine_launch<DT, D, GG, 1024>(a, grid, s);
  return refine_launch<DT, D, GG, 256>(a, grid, s);
}

template <int DT, int D>
static hipError_t refine_g(int G, const RefineArgs& a, dim3 grid, hipStream_t s) {
  switch (G) {
#define TS_CASE(GG) case GG: return refine_one<DT, D, GG>(a, grid, s);
    TS_CASE(1) TS_CASE(2) TS_CASE(3) TS_CASE(4) TS_CASE(5) TS_CASE(6) TS_CASE(7) TS_CASE(8)
#undef TS_CASE
  }
  return hipErrorInvalidValue;
}

hipError_t launch_topk_refine(int dtype, int D, int G, const RefineArgs& a, int B, hipStream_t s) {
  const dim3 grid(a.t.nblk * a.parts, B);
  if (dtype == TS_F32) return D == 64 ? refine_g<TS_F32, 64>(G, a, grid, s) : refine_g<TS_F32, 128>(G, a, grid, s);
  return D == 64 ? refine_g<TS_BF16, 64>(G, a, grid, s) : refine_g<TS_BF16, 128>(G, a, grid, s);
}

}  // namespace ts
