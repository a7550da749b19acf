// Decode score pass: Algorithm 2 (Paged Dot Product Kernel) re-designed for gfx950, fused with the
// per-head softmax statistics that Eq. 5 needs.
//
// HBM-bound streaming design.  A wave owns tiles of 32 logical tokens x HB = min(H_kv, 8) KV heads.
// Eight lanes share one K row (one token, one KV head): each lane loads 16-byte pieces of the row
// (a load instruction of the wave covers eight rows x 128 contiguous bytes, i.e. whole cache lines),
// multiplies them with the G query heads of that KV head kept in registers (the GQA group shares
// every K byte that is loaded), and the eight partial sums are combined with three DPP steps.
// The 32 x HB x G scores of a tile are staged in LDS token-major; a run of 1, 2 or 4 consecutive tiles
// leaves as one contiguous burst (scores are stored [token][head]; 4-16 KiB for 32 heads) while the
// loads of the next tile are already in flight, and the same staged values update running
// (max, sum-exp) statistics that a lane keeps in registers for its four heads.  Longer runs are used for
// longer sequences: on this memory system a write stream mixed into the read stream costs about three
// times its bytes, and fewer, larger bursts reduce that.
#include "ts_kernels.h"
#include "selcache_device.h"
#include "ts_score_math.h"
#include <hip/hip_ext.h>

namespace ts {


// Both modes keep running softmax statistics in the lanes that end as one partial per workgroup.
// MODE 0: Algorithm 2's S leaves as fp32 rows.  MODE 1 (compact form): nothing but one byte per score leaves --
// the score's distance below the maximum of its head inside its 32-token tile (a "block"), in quarter
// octaves of the softmax weight, rounded towards the maximum -- next to the block's per-head maximum; S itself
// never reaches memory.  The bytes bound every softmax weight from both sides, which is enough to find the few
// tokens whose votes have to be evaluated exactly.  (The matrix-core kernel in score_codes_mfma.hip is the fast
// form of MODE 1 for bf16; this one serves fp32 and the shapes that one does not take.)
template <int DT, int D, int G, bool DOT2, int MODE>
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
  const int N = min(max(a.seq_lens[b], 0), a.max_seq_len);
  const int indptr = a.page_indptr[b];
  // Algorithm 1's test inside this launch: the vectors' loads and partial sums go first, the decision is taken below,
  // once the first page ids are on their way (the same sums in the same order in every workgroup of the sequence).
  // The reduction uses the head of the dynamic LDS, which nothing else touches before the decision.
  const bool sc_on = a.sc_cached_q != nullptr;
  double (*sc_red)[4] = reinterpret_cast<double (*)[4]>(smem);
  int sc_first0 = 0;
  if (sc_on) {
    uint4 qkeep[kSelcacheKeep];
    sc_first0 = a.sc_first[b];
    selcache_sums<DT>(reinterpret_cast<const uint4*>(a.q + (size_t)b * a.H * RB),
                      reinterpret_cast<const uint4*>(a.sc_cached_q + (size_t)b * a.H * RB), a.H * RB / 16, sc_red, qkeep);
  } else if (a.skip != nullptr && a.skip[b] != 0) {
    return;
  }
  const int H = a.H, HB = a.HB, HBG = HB * G;
  const int HS = (HBG + 3) & ~3;             // floats per token row of the staged tile
  const int RR = a.RR;                        // tiles a wave stages before it writes them out as one run
  const int stage_floats = max(RR * TT * HS, 512) + 64;  // [RR][TT][HS] staged scores, token-major (>= 512 floats: reused below) + 64 block maxima
  float* stage = smem + wave * stage_floats;

  const int tps_shift = 3 - a.hb_shift;      // log2(tokens per wave step)
  const int STEPS = TT >> tps_shift;
  const int kvh_l = r & (HB - 1);
  const int tok_in_step = r >> a.hb_shift;
  const int u = wave & (a.NU - 1);           // block of HB KV heads this wave stays with
  const int kvh = u * HB + kvh_l;
  const int h_base = u * HBG;
  const int ntt = (N + TT - 1) / TT;
  const int tt_step = (gridDim.x * 4) / a.NU;
  const int npages = (N + a.P - 1) >> a.p_shift;
  const float c2 = a.c2;
  const int r_lo = min(a.n_init, N), r_hi = max(r_lo, N - a.n_local);   // ranked range: the statistics cover it only

  // epilogue mapping: a lane owns one 16-byte chunk (four heads) of a token row, always the same heads
  const int CPT = HS >> 2;                   // chunks per token row
  const int TPP = 64 / CPT;                  // token rows per epilogue pass
  const int e_sub = lane / CPT, e_hq = lane - e_sub * CPT;
  const bool e_active = e_sub < TPP;
  const int e_nvh = min(4, HBG - e_hq * 4);  // heads of this chunk that exist
  // A lane with j < G always produces the score of the same head (KV head kvh_l, group member j), so it
  // keeps that head's running (max, sum-exp) over the tokens it sees; the updates sit in the load shadow.
  float rm = -INFINITY, rl = 0.f;

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
  // A wave owns runs of RR consecutive tiles: run n of the wave is run_first + n * run_step; its i-th tile
  // overall (i = n * RR + r) is tile (run_first + n * run_step) * RR + r.  The tiles that exist form a prefix.
  const int nrun = (ntt + RR - 1) / RR;
  const int run_first = (blockIdx.x * 4 + wave) / a.NU, run_step = tt_step;
  int my_tiles = 0;
  if (run_first < nrun) {
    const int my_runs = (nrun - run_first + run_step - 1) / run_step;
    const int last_run = run_first + (my_runs - 1) * run_step;
    my_tiles = (my_runs - 1) * RR + min(RR, ntt - last_run * RR);
  }
  const int total_blocks = my_tiles * NBLK;
  auto tile_of = [&](int n, int r) -> int { return (run_first + n * run_step) * RR + r; };

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
  auto compute = [&](const uint4 (&kr)[U][L], int blk, float* tile, int t0) {
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
      const bool act = (j < G) && (t0 + tl >= r_lo) && (t0 + tl < r_hi);
      if (__builtin_amdgcn_ballot_w64(act && v > rm) != 0) {   // rare after the first tiles: rescale to the new maximum
        const float mn = act ? fmaxf(rm, v) : rm;
        rl = (rm == -INFINITY) ? 0.f : rl * __builtin_amdgcn_exp2f(c2 * (rm - mn));
        rm = mn;
      }
      if (act) rl += __builtin_amdgcn_exp2f(c2 * (v - rm));
    }
  };
  // compact form: the run's per-head maximum over its ranked tokens, then one byte per score
  const int ncp_shift = a.ncp_shift;          // lanes per token subset: the power of two >= HBG (<= 64)
  auto epilogue_codes = [&](int run_t0, int run_ntok) {
    wave_lds_sync();
    const int NCP = 1 << ncp_shift;
    const int c = lane & (NCP - 1), sub = lane >> ncp_shift, groups = 64 >> ncp_shift;
    float* bmx = stage + (stage_floats - 64);
    for (int f0 = 0; f0 < run_ntok; f0 += TT) {            // a block of the byte form is one 32-token tile
      const int t0 = run_t0 + f0;
      const float* tile = stage + f0 * HS;
      const int tmin = max(0, r_lo - t0), tmax = min(TT, r_hi - t0);   // tokens of the tile that take part in the softmax
      float mx = -INFINITY;
      if (c < HBG)
        for (int tok = tmin + sub; tok < tmax; tok += groups) mx = fmaxf(mx, tile[tok * HS + c]);
      for (int off = NCP; off < 64; off <<= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
      if (sub == 0) {
        bmx[c] = (c < HBG) ? mx : -INFINITY;
        if (c < HBG) a.blk_max[((size_t)b * a.nblk + (size_t)(t0 / TT)) * H + h_base + c] = mx;
      }
      wave_lds_sync();
      for (int tok0 = 0; tok0 < TT; tok0 += TPP) {
        const int tok = tok0 + e_sub;
        const int t = t0 + tok;
        if (e_active && tok < TT && t < N) {
          const float4 v4 = *reinterpret_cast<const float4*>(&tile[tok * HS + e_hq * 4]);
          const float4 m4 = *reinterpret_cast<const float4*>(&bmx[e_hq * 4]);
          // 255 = at the maximum, one step = a quarter octave of softmax weight, rounded towards the maximum;
          // 0 = 63.75 octaves or more below it (fmaxf drops the NaN of an empty block)
          const uint32_t q0 = (uint32_t)fminf(fmaxf(255.f + ceilf(4.f * c2 * (v4.x - m4.x)), 0.f), 255.f);
          const uint32_t q1 = (uint32_t)fminf(fmaxf(255.f + ceilf(4.f * c2 * (v4.y - m4.y)), 0.f), 255.f);
          const uint32_t q2 = (uint32_t)fminf(fmaxf(255.f + ceilf(4.f * c2 * (v4.z - m4.z)), 0.f), 255.f);
          const uint32_t q3 = (uint32_t)fminf(fmaxf(255.f + ceilf(4.f * c2 * (v4.w - m4.w)), 0.f), 255.f);
          uint8_t* dst = a.codes + ((size_t)b * a.max_seq_len + t) * H + h_base + e_hq * 4;
          if (a.vec_store) {
            *reinterpret_cast<uint32_t*>(dst) = q0 | (q1 << 8) | (q2 << 16) | (q3 << 24);
          } else {
            const uint32_t qq[4] = {q0, q1, q2, q3};
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (e < e_nvh) dst[e] = (uint8_t)qq[e];
          }
        }
      }
      wave_lds_sync();
    }
  };
  // the staged tiles leave as one contiguous run of token rows
  auto epilogue = [&](int t0, int ntok) {
    wave_lds_sync();
    for (int tok0 = 0; tok0 < ntok; tok0 += TPP) {
      const int tok = tok0 + e_sub;
      const int t = t0 + tok;
      if (e_active && tok < ntok && t < N) {
        const float4 v4 = *reinterpret_cast<const float4*>(&stage[tok * HS + e_hq * 4]);
        float* dst = a.scores + ((size_t)b * a.max_seq_len + t) * H + h_base + e_hq * 4;
        if (a.vec_store) {
          typedef float v4f __attribute__((ext_vector_type(4)));
          const v4f sv = {v4.x, v4.y, v4.z, v4.w};
          __builtin_nontemporal_store(sv, reinterpret_cast<v4f*>(dst));   // streamed out; the vote kernel reads it from HBM anyway
        } else {
#pragma unroll
          for (int c = 0; c < 4; ++c)
            if (c < e_nvh) dst[c] = stage[tok * HS + e_hq * 4 + c];
        }
      }
    }
    wave_lds_sync();
  };

  uint4 buf[U][L];
  int i_n = 0, i_r = 0, i_blk = 0;           // issue cursor: run, tile in run, block in tile
  int c_n = 0, c_r = 0, c_blk = 0;           // compute cursor
  int i_pid = 0, i_pid_next = 0;
  auto next_tile = [&](int n, int r) -> int {  // tile after (n, r) in this wave's order, clamped to an existing one
    const int t = (r + 1 == RR) ? tile_of(n + 1, 0) : tile_of(n, r + 1);
    return min(t, ntt - 1);
  };
  auto advance_issue = [&]() {
    if (++i_blk == NBLK) {
      i_blk = 0;
      if (++i_r == RR) { i_r = 0; ++i_n; }
      i_pid = i_pid_next;
      i_pid_next = load_pids(next_tile(i_n, i_r));   // one tile ahead: never on the critical path
    }
  };
  if (total_blocks > 0) {
    i_pid = load_pids(tile_of(0, 0));
    i_pid_next = load_pids(next_tile(0, 0));
  }
  if (sc_on) {
    const int reselect = selcache_decide(sc_red, reinterpret_cast<int*>(sc_red + 3), sc_first0, a.sc_theta);
    if (blockIdx.x == 0) {                                // the state after the step: C_Q <- Q on a miss, kept on a hit
      const int npieces = a.H * RB / 16;
      const uint4* qv = reinterpret_cast<const uint4*>(a.q + (size_t)b * a.H * RB);
      const uint4* cv = reinterpret_cast<const uint4*>(a.sc_cached_q + (size_t)b * a.H * RB);
      uint4* nv = reinterpret_cast<uint4*>(a.sc_cached_q_next + (size_t)b * a.H * RB);
      for (int p = threadIdx.x; p < npieces; p += 256) nv[p] = reselect ? qv[p] : cv[p];
      if (threadIdx.x == 0) { a.sc_reuse[b] = (uint8_t)(!reselect); a.sc_first_next[b] = (uint8_t)(reselect ? 0 : sc_first0); }
    }
    if (!reselect) return;
  }
  if (total_blocks > 0) {
    issue(buf, tile_of(0, 0), 0, i_pid);
    advance_issue();
  }
  int done_tiles = 0;
  for (int gb = 0; gb < total_blocks; ++gb) {
    compute(buf, c_blk, stage + c_r * (TT * HS), tile_of(c_n, c_r) * TT);
    // the next block's loads go out before the epilogue, which then runs in their shadow
    if (gb + 1 < total_blocks) { issue(buf, tile_of(i_n, i_r), i_blk, i_pid); advance_issue(); }
    if (++c_blk == NBLK) {
      c_blk = 0; ++done_tiles;
      if (c_r + 1 == RR || done_tiles == my_tiles) {
        if (MODE == 0) epilogue(tile_of(c_n, 0) * TT, (c_r + 1) * TT);
        else epilogue_codes(tile_of(c_n, 0) * TT, (c_r + 1) * TT);
        c_r = 0; ++c_n;
      } else {
        ++c_r;
      }
    }
  }

  // what the following calls need to know about this launch (they read it from the workspace, not from the host)
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    a.hdr[b * 8 + 0] = gridDim.x;                          // statistics partials of this launch
    a.hdr[b * 8 + 2] = __float_as_uint(a.scale);
  }
  // ---- merge the lanes' statistics per head: first inside the wave (its own LDS region, no workgroup
  // barrier), then over the waves of the workgroup that share a head block; publish the partial
  {
    float2* st = reinterpret_cast<float2*>(stage);   // [64 lanes]; the wave's own staging region is free now
    wave_lds_sync();
    st[lane] = make_float2(rm, rl);
    wave_lds_sync();
    float m = -INFINITY, l = 0.f;
    if (lane < HBG) {                         // head (kv, jj) of the wave's block: rows kv, kv + HB, ... produced it
      const int kv = lane / G, jj = lane - kv * G;
      for (int rr = kv; rr < 8; rr += HB) m = fmaxf(m, st[rr * 8 + jj].x);
      for (int rr = kv; rr < 8; rr += HB) {
        const float2 e = st[rr * 8 + jj];
        l += (e.x == -INFINITY) ? 0.f : e.y * __builtin_amdgcn_exp2f(c2 * (e.x - m));
      }
    }
    __syncthreads();                          // every wave has read its lane statistics
    float2* wv = reinterpret_cast<float2*>(smem);   // [4 waves][HBG]
    if (lane < HBG) wv[wave * HBG + lane] = make_float2(m, l);
    __syncthreads();
  }
  for (int h = threadIdx.x; h < H; h += 256) {
    const int uh = h / HBG, hl = h - uh * HBG;
    const float2* wv = reinterpret_cast<const float2*>(smem);
    float m = -INFINITY;
    for (int w = uh; w < 4; w += a.NU) m = fmaxf(m, wv[w * HBG + hl].x);
    float l = 0.f;
    for (int w = uh; w < 4; w += a.NU) {
      const float2 e = wv[w * HBG + hl];
      l += (e.x == -INFINITY) ? 0.f : e.y * __builtin_amdgcn_exp2f(c2 * (e.x - m));
    }
    float* pp = a.partials + (((size_t)b * kScoreMaxWg + blockIdx.x) * H + h) * 2;
    pp[0] = m; pp[1] = l;
  }
}

// ------------------------------------------------------------------------------------------------
// Optional pair of events that the next launches bind to the kernel's own start and end (benchmarks: the
// duration then excludes what stream-ordered event records add around a launch).
static hipEvent_t g_time_start = nullptr, g_time_stop = nullptr;
void set_score_timing_events(hipEvent_t start, hipEvent_t stop) { g_time_start = start; g_time_stop = stop; }

template <int DT, int D, int G, bool DOT2>
static hipError_t launch_one(const ScoreArgs& a, dim3 grid, size_t lds, hipStream_t s) {
  if (a.codes != nullptr) {
    if (g_time_start != nullptr && g_time_stop != nullptr)
      hipExtLaunchKernelGGL((score_decode_kernel<DT, D, G, DOT2, 1>), grid, dim3(256), (uint32_t)lds, s, g_time_start, g_time_stop, 0u, a);
    else
      hipLaunchKernelGGL((score_decode_kernel<DT, D, G, DOT2, 1>), grid, dim3(256), lds, s, a);
    return hipGetLastError();
  }
  if (g_time_start != nullptr && g_time_stop != nullptr)
    hipExtLaunchKernelGGL((score_decode_kernel<DT, D, G, DOT2, 0>), grid, dim3(256), (uint32_t)lds, s, g_time_start, g_time_stop, 0u, a);
  else
    hipLaunchKernelGGL((score_decode_kernel<DT, D, G, DOT2, 0>), grid, dim3(256), lds, s, a);
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
