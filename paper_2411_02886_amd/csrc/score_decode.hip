// Decode score pass: Algorithm 2 (Paged Dot Product Kernel) re-designed for gfx950, fused with the
// per-head softmax statistics that Eq. 5 needs.
//
// HBM-bound streaming design.  A wave owns a tile of 32 logical tokens x HB = min(H_kv, 8) KV heads.
// Eight lanes share one K row (one token, one KV head): each lane loads 16-byte pieces of the row
// (a load instruction of the wave covers eight rows x 128 contiguous bytes, i.e. whole cache lines),
// multiplies them with the G query heads of that KV head kept in registers (the GQA group shares
// every K byte that is loaded), and the eight partial sums are combined with three DPP steps.
// The 32 x HB x G scores of the tile are staged in LDS token-major and leave as one contiguous run
// (scores are stored [token][head], so a tile is a single 4 KiB burst for 32 heads); the same staged
// values update running (max, sum-exp) statistics that a lane keeps in registers for its four heads.
#include "ts_kernels.h"

namespace ts {


template <int DT> struct Elt;
template <> struct Elt<TS_F32> { static constexpr int size = 4; };
template <> struct Elt<TS_BF16> { static constexpr int size = 2; };

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;

// One 16-byte piece of a K row times the matching piece of one query head.
template <int DT, bool DOT2> struct Piece;
template <> struct Piece<TS_F32, false> {
  struct Q { float v[4]; };
  static __device__ __forceinline__ Q prep(uint4 w) {
    Q q; q.v[0] = __uint_as_float(w.x); q.v[1] = __uint_as_float(w.y); q.v[2] = __uint_as_float(w.z); q.v[3] = __uint_as_float(w.w);
    return q;
  }
  static __device__ __forceinline__ float dot(uint4 k, const Q& q, float acc) {
    acc = fmaf(__uint_as_float(k.x), q.v[0], acc);
    acc = fmaf(__uint_as_float(k.y), q.v[1], acc);
    acc = fmaf(__uint_as_float(k.z), q.v[2], acc);
    acc = fmaf(__uint_as_float(k.w), q.v[3], acc);
    return acc;
  }
};
template <> struct Piece<TS_BF16, false> {
  struct Q { float v[8]; };
  static __device__ __forceinline__ Q prep(uint4 w) {
    Q q;
    q.v[0] = bf16_lo(w.x); q.v[1] = bf16_hi(w.x); q.v[2] = bf16_lo(w.y); q.v[3] = bf16_hi(w.y);
    q.v[4] = bf16_lo(w.z); q.v[5] = bf16_hi(w.z); q.v[6] = bf16_lo(w.w); q.v[7] = bf16_hi(w.w);
    return q;
  }
  static __device__ __forceinline__ float dot(uint4 k, const Q& q, float acc) {
    // bf16 x bf16 products are exact in float; each fma rounds once
    acc = fmaf(bf16_lo(k.x), q.v[0], acc); acc = fmaf(bf16_hi(k.x), q.v[1], acc);
    acc = fmaf(bf16_lo(k.y), q.v[2], acc); acc = fmaf(bf16_hi(k.y), q.v[3], acc);
    acc = fmaf(bf16_lo(k.z), q.v[4], acc); acc = fmaf(bf16_hi(k.z), q.v[5], acc);
    acc = fmaf(bf16_lo(k.w), q.v[6], acc); acc = fmaf(bf16_hi(k.w), q.v[7], acc);
    return acc;
  }
};
template <> struct Piece<TS_BF16, true> {
  struct Q { uint4 w; };
  static __device__ __forceinline__ Q prep(uint4 w) { Q q; q.w = w; return q; }
  static __device__ __forceinline__ float d2(uint32_t a, uint32_t b, float acc) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), acc, false);
  }
  static __device__ __forceinline__ float dot(uint4 k, const Q& q, float acc) {
    acc = d2(k.x, q.w.x, acc); acc = d2(k.y, q.w.y, acc); acc = d2(k.z, q.w.z, acc); acc = d2(k.w, q.w.w, acc);
    return acc;
  }
};

__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int DT, int D, int G, bool DOT2>
__global__ __launch_bounds__(256) void score_decode_kernel(ScoreArgs a) {
  constexpr int ES = Elt<DT>::size;
  constexpr int RB = D * ES;          // bytes per K row
  constexpr int L = RB / 128;         // 16-byte loads per lane per row
  constexpr int TT = kScoreTileTokens;
  constexpr int U = 4;                // wave steps (8 K rows each) per block of loads
  using P_ = Piece<DT, DOT2>;
  typedef unsigned v4u __attribute__((ext_vector_type(4)));
  extern __shared__ float smem[];

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j = lane & 7, r = lane >> 3;
  const int b = blockIdx.y;
  if (a.skip != nullptr && a.skip[b] != 0) return;
  const int N = min(max(a.seq_lens[b], 0), a.max_seq_len);
  const int H = a.H, HB = a.HB, HBG = HB * G;
  const int HS = (HBG + 3) & ~3;             // floats per token row of the staged tile
  float* tile = smem + wave * (TT * HS);     // [TT][HS] scores of the current tile, token-major

  const int tps_shift = 3 - a.hb_shift;      // log2(tokens per wave step)
  const int STEPS = TT >> tps_shift;
  const int kvh_l = r & (HB - 1);
  const int tok_in_step = r >> a.hb_shift;
  const int u = wave & (a.NU - 1);           // block of HB KV heads this wave stays with
  const int kvh = u * HB + kvh_l;
  const int h_base = u * HBG;
  const int ntt = (N + TT - 1) / TT;
  const int tt_step = (gridDim.x * 4) / a.NU;
  const int indptr = a.page_indptr[b];
  const int npages = (N + a.P - 1) >> a.p_shift;
  const float c2 = a.c2;

  // epilogue mapping: a lane owns one 16-byte chunk (four heads) of a token row, always the same heads
  const int CPT = HS >> 2;                   // chunks per token row
  const int TPP = 64 / CPT;                  // token rows per epilogue pass
  const int e_sub = lane / CPT, e_hq = lane - e_sub * CPT;
  const bool e_active = e_sub < TPP;
  const int e_nvh = min(4, HBG - e_hq * 4);  // heads of this chunk that exist
  float rm[4], rl[4];                        // running (max, sum-exp) of the lane's four heads
#pragma unroll
  for (int c = 0; c < 4; ++c) { rm[c] = -INFINITY; rl[c] = 0.f; }

  typename P_::Q qreg[G][L];
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int i = 0; i < L; ++i) {
      const uint8_t* qp = a.q + ((size_t)b * H + (size_t)kvh * G + g) * RB + i * 128 + j * 16;
      qreg[g][i] = P_::prep(*reinterpret_cast<const uint4*>(qp));
    }

  // ---- the wave's work as one stream of blocks (U wave steps = U x 8 K rows = 8 KiB each) that runs
  // across tile boundaries; page ids are fetched one tile ahead.  Measured on MI355X: keeping a second
  // block in flight per wave (register double buffering) or a larger U changes nothing -- occupancy
  // already covers the latency -- so the simple form with the fewest registers is kept.
  const int NBLK = STEPS / U;                // blocks per tile (STEPS is 4, 8, 16 or 32)
  const int tt_first = (blockIdx.x * 4 + wave) / a.NU;
  const int my_tiles = tt_first < ntt ? (ntt - tt_first + tt_step - 1) / tt_step : 0;
  const int total_blocks = my_tiles * NBLK;

  // physical page of each of a tile's 32 tokens, one per lane (lanes 32..63 mirror 0..31)
  auto load_pids = [&](int tt) -> int {
    const int pg = (tt * TT + (lane & 31)) >> a.p_shift;
    return a.page_indices[indptr + min(pg, npages - 1)];
  };
  auto issue = [&](uint4 (&kr)[U][L], int tt, int blk, int pidv) {
    const int t0 = tt * TT, s0 = blk * U;
#pragma unroll
    for (int uu = 0; uu < U; ++uu) {
      const int tl = ((s0 + uu) << tps_shift) + tok_in_step;
      int pid;
      if (a.uniform_page) pid = __builtin_amdgcn_readlane(pidv, (s0 + uu) << tps_shift);
      else pid = __shfl(pidv, tl);
      const int t = t0 + tl;
      const uint8_t* kp = a.k_pool + (((size_t)pid << a.p_shift) + (size_t)(t & (a.P - 1))) * ((size_t)a.H_kv * RB) +
                          (size_t)kvh * RB + j * 16;
#pragma unroll
      for (int i = 0; i < L; ++i) {
        // K is read once per call: a non-temporal load keeps it from displacing the staged scores
        const v4u w = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(kp + i * 128));
        kr[uu][i] = make_uint4(w.x, w.y, w.z, w.w);
      }
    }
  };
  auto compute = [&](const uint4 (&kr)[U][L], int blk) {
    const int s0 = blk * U;
#pragma unroll
    for (int uu = 0; uu < U; ++uu) {
      const int tl = ((s0 + uu) << tps_shift) + tok_in_step;
      float acc[G];
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float sc = 0.f;
#pragma unroll
        for (int i = 0; i < L; ++i) sc = P_::dot(kr[uu][i], qreg[g][i], sc);
        acc[g] = group8_sum(sc);
      }
      float v = acc[0];
#pragma unroll
      for (int g = 1; g < G; ++g) v = (j == g) ? acc[g] : v;
      if (j < G) tile[tl * HS + kvh_l * G + j] = v;
    }
  };
  // the tile leaves as one contiguous run of token rows; the same values feed the statistics
  auto epilogue = [&](int tt) {
    const int t0 = tt * TT;
    wave_lds_sync();
    for (int tok0 = 0; tok0 < TT; tok0 += TPP) {
      const int tok = tok0 + e_sub;
      const int t = t0 + tok;
      if (e_active && tok < TT && t < N) {
        const float4 v4 = *reinterpret_cast<const float4*>(&tile[tok * HS + e_hq * 4]);
        const float x[4] = {v4.x, v4.y, v4.z, v4.w};
        float* dst = a.scores + ((size_t)b * a.max_seq_len + t) * H + h_base + e_hq * 4;
        if (a.vec_store) {
          typedef float v4f __attribute__((ext_vector_type(4)));
          const v4f sv = {v4.x, v4.y, v4.z, v4.w};
          __builtin_nontemporal_store(sv, reinterpret_cast<v4f*>(dst));   // streamed out; the vote kernel reads it from HBM anyway
        } else {
#pragma unroll
          for (int c = 0; c < 4; ++c)
            if (c < e_nvh) dst[c] = x[c];
        }
        bool grow = false;
#pragma unroll
        for (int c = 0; c < 4; ++c) grow |= (c < e_nvh) && (x[c] > rm[c]);
        if (__builtin_amdgcn_ballot_w64(grow) != 0) {     // rare after the first tiles: rescale to the new maxima
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            if (c < e_nvh) {
              const float mn = fmaxf(rm[c], x[c]);
              rl[c] = (rm[c] == -INFINITY) ? 0.f : rl[c] * __builtin_amdgcn_exp2f(c2 * (rm[c] - mn));
              rm[c] = mn;
            }
          }
        }
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if (c < e_nvh) rl[c] += __builtin_amdgcn_exp2f(c2 * (x[c] - rm[c]));
      }
    }
    wave_lds_sync();
  };

  uint4 buf[U][L];
  int i_tt = tt_first, i_blk = 0, c_tt = tt_first, c_blk = 0;
  int i_pid = 0, i_pid_next = 0;
  auto advance_issue = [&]() {
    if (++i_blk == NBLK) {
      i_blk = 0; i_tt += tt_step;
      i_pid = i_pid_next;
      i_pid_next = load_pids(min(i_tt + tt_step, ntt - 1));   // one tile ahead: never on the critical path
    }
  };
  auto advance_compute = [&]() {
    if (++c_blk == NBLK) { epilogue(c_tt); c_blk = 0; c_tt += tt_step; }
  };
  if (total_blocks > 0) {
    i_pid = load_pids(i_tt);
    i_pid_next = load_pids(min(i_tt + tt_step, ntt - 1));
    issue(buf, i_tt, i_blk, i_pid);
    advance_issue();
  }
  for (int gb = 0; gb < total_blocks; ++gb) {
    compute(buf, c_blk);
    advance_compute();
    if (gb + 1 < total_blocks) { issue(buf, i_tt, i_blk, i_pid); advance_issue(); }
  }

  // ---- merge the lanes' statistics of this workgroup per head, publish the partial
  __syncthreads();
  float* st = smem;                          // [4 waves][64 lanes][4 heads][2]
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    st[((wave * 64 + lane) * 4 + c) * 2] = rm[c];
    st[((wave * 64 + lane) * 4 + c) * 2 + 1] = rl[c];
  }
  __syncthreads();
  for (int h = threadIdx.x; h < H; h += 256) {
    const int uh = h / HBG, hl = h - uh * HBG, hq = hl >> 2, c = hl & 3;
    float m = -INFINITY;
    for (int w = 0; w < 4; ++w)
      if ((w & (a.NU - 1)) == uh)
        for (int sub = 0; sub < TPP; ++sub) m = fmaxf(m, st[((w * 64 + sub * CPT + hq) * 4 + c) * 2]);
    float l = 0.f;
    for (int w = 0; w < 4; ++w)
      if ((w & (a.NU - 1)) == uh)
        for (int sub = 0; sub < TPP; ++sub) {
          const float mi = st[((w * 64 + sub * CPT + hq) * 4 + c) * 2];
          const float li = st[((w * 64 + sub * CPT + hq) * 4 + c) * 2 + 1];
          if (mi != -INFINITY) l += li * __builtin_amdgcn_exp2f(c2 * (mi - m));
        }
    float* pp = a.partials + (((size_t)b * kScoreMaxWg + blockIdx.x) * H + h) * 2;
    pp[0] = m; pp[1] = l;
  }
}

// ------------------------------------------------------------------------------------------------
template <int DT, int D, int G, bool DOT2>
static hipError_t launch_one(const ScoreArgs& a, dim3 grid, size_t lds, hipStream_t s) {
  hipLaunchKernelGGL((score_decode_kernel<DT, D, G, DOT2>), grid, dim3(256), lds, s, a);
  return hipGetLastError();
}

template <int DT, int D, bool DOT2>
static hipError_t launch_g(int G, const ScoreArgs& a, dim3 grid, size_t lds, hipStream_t s) {
  switch (G) {
    case 1: return launch_one<DT, D, 1, DOT2>(a, grid, lds, s);
    case 2: return launch_one<DT, D, 2, DOT2>(a, grid, lds, s);
    case 3: return launch_one<DT, D, 3, DOT2>(a, grid, lds, s);
    case 4: return launch_one<DT, D, 4, DOT2>(a, grid, lds, s);
    case 5: return launch_one<DT, D, 5, DOT2>(a, grid, lds, s);
    case 6: return launch_one<DT, D, 6, DOT2>(a, grid, lds, s);
    case 7: return launch_one<DT, D, 7, DOT2>(a, grid, lds, s);
    case 8: return launch_one<DT, D, 8, DOT2>(a, grid, lds, s);
  }
  return hipErrorInvalidValue;
}

// variant: 0 = fma arithmetic, 1 = packed bf16 dot2 (bf16 only)
hipError_t launch_score_decode(int dtype, int D, int G, int variant, const ScoreArgs& a, dim3 grid, size_t lds,
                               hipStream_t s) {
  if (dtype == TS_F32) {
    if (D == 64) return launch_g<TS_F32, 64, false>(G, a, grid, lds, s);
    return launch_g<TS_F32, 128, false>(G, a, grid, lds, s);
  }
  if (variant == 1) {
    if (D == 64) return launch_g<TS_BF16, 64, true>(G, a, grid, lds, s);
    return launch_g<TS_BF16, 128, true>(G, a, grid, lds, s);
  }
  if (D == 64) return launch_g<TS_BF16, 64, false>(G, a, grid, lds, s);
  return launch_g<TS_BF16, 128, false>(G, a, grid, lds, s);
}

}  // namespace ts
