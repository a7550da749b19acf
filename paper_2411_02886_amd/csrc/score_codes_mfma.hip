// Compact score pass on the matrix cores (bf16): Algorithm 2 with one byte per score leaving the chip.
//
// Why matrix cores in an HBM-bound kernel: with G query heads per KV head the dot products are a dense
// [rows x D] x [D x G] contraction, and on the vector ALU they cost about 110 instructions per 2 KiB of K --
// enough that everything else a wave does (softmax statistics, coding, stores) delays its next loads.  On MFMA
// the same 2 KiB cost a few instructions, and the kernel runs at the speed of its loads.
//
// Data path.  Global loads keep the streaming layout of the vector kernel: eight lanes share a K row, a wave
// load covers eight rows x 128 contiguous bytes (whole cache lines), non-temporal.  A block of 32 rows (8 KiB)
// goes through a wave-private LDS tile with padded rows (conflict-free 16-byte reads) and comes back as A
// fragments of v_mfma_f32_16x16x32_bf16: 16 rows of one column block (KB = 2 or 4 KV heads) x 32 of D.  The B
// fragments are the query heads of those KV heads, CP = 4 or 8 columns per KV head, kept in registers for the
// whole kernel.  A row meets the columns of all KB KV heads of its column block; only the ones of its own KV
// head are scores (the matrix cores have the time).
//
// A lane always owns the same two query heads (one per column block), and the 16 scores of a 32-token tile
// that fall to it stay in registers until the tile is complete.  Then the tile's exact per-head maximum and
// sum of exponentials are formed with two cross-lane steps (they feed the wave's running softmax statistics,
// which end as one partial per workgroup), and every score becomes one byte: its distance
// below that maximum in quarter octaves of softmax weight, rounded towards the maximum (see
// ts_paged_qk_codes).  Bytes and statistics are collected in LDS for a run of consecutive tiles and leave as
// one contiguous burst at the end of the run: on this memory system small writes sprinkled into the read
// stream cost many times their bytes, a burst at the end of a wave's life costs about its own time.
#include "ts_kernels.h"
#include "selcache_device.h"
#include "ts_score_math.h"
#include <hip/hip_ext.h>

namespace ts {

typedef __attribute__((ext_vector_type(8))) __bf16 mfma_bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float mfma_f32x4_t;

// G in 3..4: CP = 4, column block = 4 KV heads, wave tile = 8 KV heads.  G in 5..8: CP = 8, 2 and 4.
// DENSE: Algorithm 2's score matrix itself leaves the chip (fp32 rows, ts_paged_qk_scores) instead of the bytes.
template <int D, int G, bool DENSE>
__global__ __launch_bounds__(256) void score_codes_mfma_kernel(ScoreArgs a) {
  constexpr int RB = D * 2;            // bytes per K row
  constexpr int L = RB / 128;          // 16-byte loads per lane per row
  constexpr int KS = D / 32;           // MFMA steps along D
  constexpr int CP = G <= 4 ? 4 : 8;   // columns per KV head
  constexpr int KB = 16 / CP;          // KV heads per column block
  constexpr int HB = 2 * KB;           // KV heads per wave tile (two column blocks)
  constexpr int HBG = HB * G;          // score columns of the wave
  constexpr int TPS = 8 / HB;          // tokens per wave step of 8 rows
  constexpr int TPS_SHIFT = TPS == 2 ? 1 : 0;
  constexpr int HB_SHIFT = HB == 8 ? 3 : 2;
  constexpr int TT = kScoreTileTokens;
  constexpr int STEPS = TT / TPS;
  constexpr int U = 4;                 // wave steps per block: 32 rows = 8 KiB (D = 128)
  constexpr int NBLK = STEPS / U;      // blocks per tile: 4 or 8
  constexpr int TB = U * TPS;          // tokens per block: 8 or 4
  constexpr int UPL = 4 / KB;          // scores per lane and MFMA: 2 or 1
  constexpr int ROWP = RB + 16;        // LDS row pitch: 16 rows land in 16 different bank groups
  typedef unsigned v4u __attribute__((ext_vector_type(4)));
  extern __shared__ uint8_t smem8[];

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j = lane & 7, r = lane >> 3;
  const int mrow = lane & 15, kg = lane >> 4;            // MFMA row / column and k-group of this lane
  const int b = blockIdx.y;
  const int N = min(max(a.seq_lens[b], 0), a.max_seq_len);
  const int indptr = a.page_indptr[b];
  // Algorithm 1's test inside this launch: the vectors' loads and partial sums go first, the decision is taken below,
  // once the first page ids are on their way (the same sums in the same order in every workgroup of the sequence).
  // The reduction uses the head of the dynamic LDS, which nothing else touches before the decision.
  const bool sc_on = a.sc_cached_q != nullptr;
  double (*sc_red)[4] = reinterpret_cast<double (*)[4]>(smem8);
  int sc_first0 = 0;
  if (sc_on) {
    uint4 qkeep[kSelcacheKeep];
    sc_first0 = a.sc_first[b];
    selcache_sums<TS_BF16>(reinterpret_cast<const uint4*>(a.q + (size_t)b * a.H * RB),
                      reinterpret_cast<const uint4*>(a.sc_cached_q + (size_t)b * a.H * RB), a.H * RB / 16, sc_red, qkeep);
  } else if (a.skip != nullptr && a.skip[b] != 0) {
    return;
  }
  const int H = a.H;
  const int RR = a.RR;                                    // tiles per run: bytes and statistics leave once per run
  // wave-private LDS: K tile, code bytes of the run, statistics of the run
  const int code_bytes = RR * TT * HBG * (DENSE ? 4 : 1);
  const int wave_bytes = 32 * ROWP + code_bytes + RR * HBG * 4;
  uint8_t* ktile = smem8 + (size_t)wave * wave_bytes;
  uint8_t* cbuf = ktile + 32 * ROWP;
  float* smax = reinterpret_cast<float*>(cbuf + code_bytes);
  float wm[2] = {-INFINITY, -INFINITY}, wl[2] = {0.f, 0.f};   // the wave's running (max, sum-exp) of this lane's two heads

  const int kvh_l = r & (HB - 1);
  const int tok_in_step = r >> HB_SHIFT;
  const int u = wave & (a.NU - 1);
  const int kvh = u * HB + kvh_l;
  const int h_base = u * HBG;
  const int ntt = (N + TT - 1) / TT;
  const int tt_step = (gridDim.x * 4) / a.NU;
  const int npages = (N + a.P - 1) >> a.p_shift;
  const float c2 = a.c2;
  const int r_lo = min(a.n_init, N), r_hi = max(r_lo, N - a.n_local);

  // B fragments: column c of column block cb is query head (cb * KB + c / CP) * G + c % CP of the wave's heads
  const int kvo = mrow / CP, gq = mrow % CP;             // as a column: KV head inside the block, group member
  const bool col_ok = gq < G;
  uint4 bq[2][KS];
#pragma unroll
  for (int cb = 0; cb < 2; ++cb)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      uint4 v = make_uint4(0u, 0u, 0u, 0u);
      if (col_ok) v = *reinterpret_cast<const uint4*>(a.q + ((size_t)b * H + (size_t)(u * HB + cb * KB + kvo) * G + gq) * RB + ks * 64 + kg * 16);
      bq[cb][ks] = v;
    }
  // A fragments: MFMA row m of column block cb is token m / KB of the block, KV head cb * KB + m % KB
  int arow[2];
#pragma unroll
  for (int cb = 0; cb < 2; ++cb) {
    const int tb = mrow / KB, kv = cb * KB + mrow % KB;
    arow[cb] = ((tb >> TPS_SHIFT) * 8 + (tb & (TPS - 1)) * HB + kv) * ROWP + kg * 16;
  }

  const int nrun = (ntt + RR - 1) / RR;
  const int run_first = (blockIdx.x * 4 + wave) / a.NU, run_step = tt_step;
  int my_tiles = 0;
  if (run_first < nrun) {
    const int my_runs = (nrun - run_first + run_step - 1) / run_step;
    const int last_run = run_first + (my_runs - 1) * run_step;
    my_tiles = (my_runs - 1) * RR + min(RR, ntt - last_run * RR);
  }
  const int total_blocks = my_tiles * NBLK;
  auto tile_of = [&](int n, int rr) -> int { return (run_first + n * run_step) * RR + rr; };
  auto load_pids = [&](int tt) -> int {
    const int pg = (tt * TT + (lane & 31)) >> a.p_shift;
    return a.page_indices[indptr + min(pg, npages - 1)];
  };
  auto issue = [&](uint4 (&kr)[U][L], int tt, int blk, int pidv) {
    const int t0 = tt * TT, s0 = blk * U;
#pragma unroll
    for (int uu = 0; uu < U; ++uu) {
      const int tl = ((s0 + uu) << TPS_SHIFT) + tok_in_step;
      int pid;
      if (a.uniform_page) pid = __builtin_amdgcn_readlane(pidv, (s0 + uu) << TPS_SHIFT);
      else pid = __shfl(pidv, tl);
      const int t = t0 + tl;
      const uint8_t* kp = a.k_pool + (((size_t)pid << a.p_shift) + (size_t)(t & (a.P - 1))) * ((size_t)a.H_kv * RB) +
                          (size_t)kvh * RB + j * 16;
#pragma unroll
      for (int i = 0; i < L; ++i) {
        const v4u w = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(kp + i * 128));
        kr[uu][i] = make_uint4(w.x, w.y, w.z, w.w);
      }
    }
  };
  // scores of the current tile that belong to this lane: [block][column block][e], token blk * TB + kg * UPL + e
  float sv[NBLK][2][UPL];
  auto to_lds = [&](const uint4 (&kr)[U][L]) {
#pragma unroll
    for (int uu = 0; uu < U; ++uu)
#pragma unroll
      for (int i = 0; i < L; ++i) *reinterpret_cast<uint4*>(ktile + (uu * 8 + r) * ROWP + i * 128 + j * 16) = kr[uu][i];
  };
  auto multiply = [&](float (&res)[2][UPL]) {
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
      mfma_f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const uint4 av = *reinterpret_cast<const uint4*>(ktile + arow[cb] + ks * 64);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(mfma_bf16x8_t, av),
                                                      __builtin_bit_cast(mfma_bf16x8_t, bq[cb][ks]), acc, 0, 0, 0);
      }
      // result rows of this lane: kg * 4 + ii; the row's KV head inside the block is (kg * 4 + ii) % KB = ii % KB
      if (KB == 2) {
        res[cb][0] = kvo ? acc[1] : acc[0];
        res[cb][UPL - 1] = kvo ? acc[3] : acc[2];
      } else {
        res[cb][0] = kvo == 0 ? acc[0] : kvo == 1 ? acc[1] : kvo == 2 ? acc[2] : acc[3];
      }
    }
  };
  // tile `f` of the run is complete: statistics and bytes into the run's LDS buffers
  auto finish_tile = [&](int f, int t0) {
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
      float mx = -INFINITY;
#pragma unroll
      for (int bb = 0; bb < NBLK; ++bb)
#pragma unroll
        for (int e = 0; e < UPL; ++e) {
          const int t = t0 + bb * TB + kg * UPL + e;
          if (t >= r_lo && t < r_hi) mx = fmaxf(mx, sv[bb][cb][e]);
        }
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      float sm = 0.f;
#pragma unroll
      for (int bb = 0; bb < NBLK; ++bb)
#pragma unroll
        for (int e = 0; e < UPL; ++e) {
          const int t = t0 + bb * TB + kg * UPL + e;
          if (t >= r_lo && t < r_hi) sm += __builtin_amdgcn_exp2f(c2 * (sv[bb][cb][e] - mx));
        }
      sm += __shfl_xor(sm, 16);
      sm += __shfl_xor(sm, 32);
      if (mx > wm[cb]) {                                   // same value in the four lanes of a column
        wl[cb] = (wm[cb] == -INFINITY) ? 0.f : wl[cb] * __builtin_amdgcn_exp2f(c2 * (wm[cb] - mx));
        wm[cb] = mx;
      }
      if (mx != -INFINITY) wl[cb] += sm * __builtin_amdgcn_exp2f(c2 * (mx - wm[cb]));
      const int hc = (cb * KB + kvo) * G + gq;             // column among the wave's HBG
      if (col_ok) {
        if (DENSE) {
          float* sbuf = reinterpret_cast<float*>(cbuf);
#pragma unroll
          for (int bb = 0; bb < NBLK; ++bb)
#pragma unroll
            for (int e = 0; e < UPL; ++e) sbuf[(f * TT + bb * TB + kg * UPL + e) * HBG + hc] = sv[bb][cb][e];
        } else {
          if (kg == 0) smax[f * HBG + hc] = mx;
#pragma unroll
          for (int bb = 0; bb < NBLK; ++bb)
#pragma unroll
            for (int e = 0; e < UPL; ++e) {
              const int tl = bb * TB + kg * UPL + e;
              const float qf = fminf(fmaxf(255.f + ceilf(4.f * c2 * (sv[bb][cb][e] - mx)), 0.f), 255.f);
              cbuf[(f * TT + tl) * HBG + hc] = (uint8_t)(uint32_t)qf;
            }
        }
      }
    }
  };
  // the run's bytes and statistics leave as contiguous bursts
  auto flush_run = [&](int tile0, int ntiles) {
    wave_lds_sync();
    const int t0 = tile0 * TT;
    const int ntok = min(ntiles * TT, N - t0);
    if (DENSE) {
      // fp32 rows, token-major; streamed out (the vote kernel reads them from memory anyway)
      typedef float v4f __attribute__((ext_vector_type(4)));
      const float* sbuf = reinterpret_cast<const float*>(cbuf);
      if (a.NU == 1) {
        float* dst = a.scores + ((size_t)b * a.max_seq_len + t0) * H;
        const int nf = ntok * H;                          // H is a multiple of 4
        if ((reinterpret_cast<uintptr_t>(dst) & 15) == 0) {
          for (int i = lane; i < (nf >> 2); i += 64)
            __builtin_nontemporal_store(reinterpret_cast<const v4f*>(sbuf)[i], reinterpret_cast<v4f*>(dst) + i);
        } else {
          for (int i = lane; i < nf; i += 64) __builtin_nontemporal_store(sbuf[i], dst + i);
        }
      } else {
        for (int i = lane; i < ntok * HBG; i += 64) {
          const int tok = i / HBG, c = i - tok * HBG;
          __builtin_nontemporal_store(sbuf[i], a.scores + ((size_t)b * a.max_seq_len + t0 + tok) * H + h_base + c);
        }
      }
      wave_lds_sync();
      return;
    }
    if (a.NU == 1) {
      uint8_t* dst = a.codes + ((size_t)b * a.max_seq_len + t0) * H;
      const int nbytes = ntok * H;
      if ((reinterpret_cast<uintptr_t>(dst) & 15) == 0) {
        const int n16 = nbytes >> 4;
        if (a.nt_codes) {
          for (int i = lane; i < n16; i += 64) { const v4u w = reinterpret_cast<const v4u*>(cbuf)[i]; __builtin_nontemporal_store(w, reinterpret_cast<v4u*>(dst) + i); }
        } else {
          for (int i = lane; i < n16; i += 64) reinterpret_cast<uint4*>(dst)[i] = reinterpret_cast<const uint4*>(cbuf)[i];
        }
        for (int i = (n16 << 2) + lane; i < (nbytes >> 2); i += 64) reinterpret_cast<uint32_t*>(dst)[i] = reinterpret_cast<const uint32_t*>(cbuf)[i];
      } else {
        for (int i = lane; i < (nbytes >> 2); i += 64) reinterpret_cast<uint32_t*>(dst)[i] = reinterpret_cast<const uint32_t*>(cbuf)[i];
      }
      float* dm = a.blk_max + ((size_t)b * a.nblk + tile0) * H;
      if (a.nt_codes) { for (int i = lane; i < ntiles * H; i += 64) __builtin_nontemporal_store(smax[i], dm + i); }
      else { for (int i = lane; i < ntiles * H; i += 64) dm[i] = smax[i]; }
    } else {
      constexpr int WPT = HBG / 4;                         // dwords per token row piece
      for (int i = lane; i < ntok * WPT; i += 64) {
        const int tok = i / WPT, wq = i - tok * WPT;
        reinterpret_cast<uint32_t*>(a.codes + ((size_t)b * a.max_seq_len + t0 + tok) * H + h_base)[wq] =
            reinterpret_cast<const uint32_t*>(cbuf + tok * HBG)[wq];
      }
      for (int i = lane; i < ntiles * HBG; i += 64) {
        const int f = i / HBG, c = i - f * HBG;
        a.blk_max[((size_t)b * a.nblk + tile0 + f) * H + h_base + c] = smax[i];
      }
    }
    wave_lds_sync();
  };

  uint4 buf[U][L];
  int i_n = 0, i_r = 0, i_blk = 0;           // issue cursor: run, tile in run, block in tile
  int c_n = 0, c_r = 0;                      // compute cursor: run, tile in run
  int i_pid = 0, i_pid_next = 0;
  auto next_tile = [&](int n, int rr) -> int {
    const int t = (rr + 1 == RR) ? tile_of(n + 1, 0) : tile_of(n, rr + 1);
    return min(t, ntt - 1);
  };
  auto advance_issue = [&]() {
    if (++i_blk == NBLK) {
      i_blk = 0;
      if (++i_r == RR) { i_r = 0; ++i_n; }
      i_pid = i_pid_next;
      i_pid_next = load_pids(next_tile(i_n, i_r));
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
  // One register buffer is enough: once a block sits in LDS its registers are free, and the next block's loads go
  // out before the matrix cores touch the current one.
  int issued = 1;
  for (int tile = 0; tile < my_tiles; ++tile) {
#pragma unroll
    for (int bb = 0; bb < NBLK; ++bb) {
      to_lds(buf);
      if (issued < total_blocks) { issue(buf, tile_of(i_n, i_r), i_blk, i_pid); advance_issue(); ++issued; }
      wave_lds_sync();
      multiply(sv[bb]);
      wave_lds_sync();
    }
    finish_tile(c_r, tile_of(c_n, c_r) * TT);
    if (c_r + 1 == RR || tile + 1 == my_tiles) {
      flush_run(tile_of(c_n, 0), c_r + 1);
      c_r = 0; ++c_n;
    } else {
      ++c_r;
    }
  }
  // ---- one (max, sum-exp) partial per workgroup and head, as the vector kernels leave it
  __syncthreads();                                        // every wave is done with its LDS region
  float2* wv = reinterpret_cast<float2*>(smem8);          // [4 waves][HBG]
  if (kg == 0 && col_ok) {
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) wv[wave * HBG + (cb * KB + kvo) * G + gq] = make_float2(wm[cb], wl[cb]);
  }
  __syncthreads();
  for (int h = threadIdx.x; h < H; h += 256) {
    const int uh = h / HBG, hl = h - uh * HBG;
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
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    a.hdr[b * 8 + 0] = gridDim.x;                          // statistics partials of this launch
    a.hdr[b * 8 + 2] = __float_as_uint(a.scale);
  }
}

static hipEvent_t g_codes_time_start = nullptr, g_codes_time_stop = nullptr;
void set_codes_timing_events(hipEvent_t start, hipEvent_t stop) { g_codes_time_start = start; g_codes_time_stop = stop; }

// shapes the matrix-core form covers: bf16, two column blocks per wave tile
bool score_codes_mfma_supported(int dtype, int D, int G, int H_kv) {
  if (dtype != TS_BF16 || (D != 64 && D != 128)) return false;
  if (G >= 3 && G <= 4) return H_kv >= 8;                 // wave tile of 8 KV heads
  if (G >= 5 && G <= 8) return H_kv == 4;                 // wave tile of 4 KV heads
  return false;
}

// dense: the run's fp32 rows are staged instead of its bytes
size_t score_codes_mfma_lds_bytes(int D, int G, int RR, bool dense) {
  const int HB = G <= 4 ? 8 : 4;
  const size_t per_wave = (size_t)32 * (D * 2 + 16) + (size_t)RR * kScoreTileTokens * HB * G * (dense ? 4 : 1) +
                          (size_t)RR * HB * G * 4;
  return 4 * per_wave;
}

template <int D, int G, bool DENSE>
static hipError_t launch_cm(const ScoreArgs& a, dim3 grid, size_t lds, hipStream_t s) {
  if (lds > 65536) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&score_codes_mfma_kernel<D, G, DENSE>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  if (g_codes_time_start != nullptr && g_codes_time_stop != nullptr)
    hipExtLaunchKernelGGL((score_codes_mfma_kernel<D, G, DENSE>), grid, dim3(256), (uint32_t)lds, s, g_codes_time_start, g_codes_time_stop, 0u, a);
  else
    hipLaunchKernelGGL((score_codes_mfma_kernel<D, G, DENSE>), grid, dim3(256), lds, s, a);
  return hipGetLastError();
}

// a.codes != nullptr: the compact form; else a.scores receives the fp32 score matrix
hipError_t launch_score_codes_mfma(int D, int G, const ScoreArgs& a, dim3 grid, size_t lds, hipStream_t s) {
  const bool dense = a.codes == nullptr;
#define TS_CM(GG) case GG: \
    if (dense) return D == 64 ? launch_cm<64, GG, true>(a, grid, lds, s) : launch_cm<128, GG, true>(a, grid, lds, s); \
    return D == 64 ? launch_cm<64, GG, false>(a, grid, lds, s) : launch_cm<128, GG, false>(a, grid, lds, s);
  switch (G) { TS_CM(3) TS_CM(4) TS_CM(5) TS_CM(6) TS_CM(7) TS_CM(8) }
#undef TS_CM
  return hipErrorInvalidValue;
}

}  // namespace ts
