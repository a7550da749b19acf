// Chunked-prefill selection (Sec. 5.2 with per-query votes): for the C queries of a chunk,
//   votes[t] = sum_{c < C} sum_h softmax_t(scale * S[c][h][:])[t]    over the cached tokens t,
// with S = Q K^T computed on the matrix cores and never written to memory.  Two sweeps over K:
//   sweep 1  per-row (query, head) log-sum-exp of scale * s over the cached tokens   -> row_stats
//   sweep 2  e = exp(scale * s - lse_row) summed over the rows of a tile column          -> votes
// Both sweeps form S from the same fragments with the same MFMA instruction (sweep 1 with the operands exchanged, which
// transposes the result and leaves the products and their order of summation alone).
//
// Work split.  For one KV head the G query heads x C queries are 'rows' that all meet the same K
// rows.  A workgroup (4 waves) owns 256 rows (64 per wave = two 32-row MFMA blocks, query fragments
// pinned in registers) and walks a range of 64-token tiles: the K tile is staged once in LDS (16-byte
// coalesced global loads, row stride padded to 272 B so that the 16-byte fragment reads are
// conflict-free), every wave reads its B fragments from there and issues 2 x 2 x (D/16)
// v_mfma_f32_32x32x16_bf16.  The next tile's K rows are in flight in registers while the current one
// is multiplied.  Workgroups that share a K range are placed on the same XCD and adjacent in launch
// order, so that one of them pulls a tile from HBM and the others find it in that XCD's L2.
#include "ts_kernels.h"
#include <type_traits>

namespace ts {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

constexpr int kPfRowsPerWg = 256;
constexpr int kPfTile = 64;            // tokens per tile
constexpr float kRefHead = 32.f;       // head room (log2 units) a raised reference exponent gets in sweep 1

// XCD-aware decode of the linear workgroup id: (row block, group) with group = (sequence, KV head, split)
__device__ __forceinline__ bool pf_decode_block(const PrefillArgs& a, int* rb, int* b, int* kvh, int* split) {
  const int L = blockIdx.x;
  const int xcd = L & 7, jq = L >> 3;
  *rb = jq % a.RB;
  const int group = (jq / a.RB) * 8 + xcd;
  if (group >= a.B * a.H_kv * a.TS) return false;
  *split = group % a.TS;
  const int r = group / a.TS;
  *kvh = r % a.H_kv;
  *b = r / a.H_kv;
  return true;
}

template <int D, int SWEEP>
// two workgroups per CU (256 registers per lane): with one the pipeline below has no second wave to hide behind
__global__ __launch_bounds__(256, 2) void prefill_qk_kernel(PrefillArgs a) {
  constexpr int KS = D / 16;                    // MFMA k-steps
  constexpr int RBYTES = D * 2;                 // bytes per K row
  constexpr int PPR = RBYTES / 16;              // 16-byte pieces per row
  constexpr int LROW = RBYTES + 16;             // padded LDS row
  __shared__ __attribute__((aligned(16))) uint8_t s_k[2][kPfTile * LROW];
  __shared__ float s_col[3][4][kPfTile];

  int rb, b, kvh, split;
  if (!pf_decode_block(a, &rb, &b, &kvh, &split)) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int C = a.C, G = a.G, H = a.H;
  const int Nc = min(max(a.seq_lens[b] - C, 0), a.max_seq_len);     // cached tokens the selection looks at
  // forced tokens: only the cached tokens [r_lo, r_hi) are ranked; the tiles that hold them are split over TS
  const int r_lo = min(a.n_init, Nc), r_hi = max(r_lo, Nc - a.n_local);
  const int tile_lo = r_lo / kPfTile, tile_hi = (r_hi > r_lo) ? (r_hi + kPfTile - 1) / kPfTile : tile_lo;
  const int tps = (tile_hi - tile_lo + a.TS - 1) / a.TS;
  const int tile_begin = min(tile_hi, tile_lo + split * tps), tile_end = min(tile_hi, tile_begin + tps);
  const int indptr = a.page_indptr[b];
  const int nrows = C * G;
  const float c2 = a.c2;

  // ---- query fragments: A[m][k], lane holds row m = lane % 32, k = 8 * (lane / 32) .. + 8 of each k-step
  const int half = lane >> 5, col = lane & 31;
  bf16x8_t afrag[2][KS];
  int row_of[2];                                 // global row of this lane's A row per block (for loads only)
#pragma unroll
  for (int mb = 0; mb < 2; ++mb) {
    const int row = rb * kPfRowsPerWg + wave * 64 + mb * 32 + col;
    row_of[mb] = row;
    const bool valid = row < nrows;
    const int c = valid ? row / G : 0, g = valid ? row % G : 0;
    const uint8_t* qp = a.q + ((((size_t)b * C + c) * H + (size_t)kvh * G + g) * D + 8 * half) * 2;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (valid) v = *reinterpret_cast<const uint4*>(qp + ks * 32);
      afrag[mb][ks] = __builtin_bit_cast(bf16x8_t, v);
    }
  }
  (void)row_of;

  // ---- per-row state.
  // Sweep 2 multiplies Q (A operand) with the K tile (B operand): in the result a lane holds, for token `col`, the 16
  // query rows 8 * i + 4 * half + j (i, j < 4) of each 32-row block, so the sum over the rows of a column is a sum inside
  // the lane; per lane and row it holds the row's log2-sum-exp: the high float as the exponent offset, 2^-low as a weight.
  // Sweep 1 multiplies the same fragments the other way round (K tile as A, Q as B: the same products summed in the same
  // order, S transposed): a lane then holds 16 tokens of ONE query row per block, so the row's running statistics are two
  // registers per block instead of 32 -- a reference exponent `off1` (log2 units) and the sum of exp2(c2 * s - off1) over
  // the lane's tokens.  The reference is raised only when an argument would exceed 2^64 (rare: a raised reference gets
  // 2^32 of head room), so the common path is one fma, one exp2 and one add per score plus half a max.
  float off[2][16], aux[2][16];                  // sweep 2 only
  float off1[2] = {-INFINITY, -INFINITY}, aux1[2] = {0.f, 0.f};   // sweep 1 only (see below)
  if (SWEEP == 2) {
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int row = rb * kPfRowsPerWg + wave * 64 + mb * 32 + 8 * (e >> 2) + 4 * half + (e & 3);
        float hi = INFINITY, lo = 0.f;           // rows past the end never vote: exp2(-inf) = 0
        if (row < nrows) {
          const int c = row / G, g = row % G;
          const float2 st = *reinterpret_cast<const float2*>(a.row_stats + (((size_t)b * C + c) * H + kvh * G + g) * 2);
          hi = st.x; lo = st.y;
        }
        off[mb][e] = hi; aux[mb][e] = __builtin_amdgcn_exp2f(-lo);   // |lo| < 2^-17: the factor 2^-lo, exact to an ulp
      }
  }

  // ---- K staging: a wave stages 16 consecutive tokens of the tile (lane -> row within a pass of 64 / PPR rows,
  // 16-byte piece).  With pages of 16 tokens or more those 16 tokens lie in one page: the page id is one scalar
  // load per wave and tile, and the lanes' addresses are a scalar base plus a constant lane offset (the address
  // arithmetic of a per-lane page lookup, with its integer multiplies, was a quarter of the vector instructions
  // of the loop).
  constexpr int RPW = 64 / PPR;                  // rows per pass of a wave
  constexpr int NLD = 16 / RPW;                  // staging loads per lane per tile
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const int st_row = lane / PPR, st_piece = lane % PPR;
  const size_t tok_stride = (size_t)a.H_kv * RBYTES;
  const uint32_t lane_off = (uint32_t)(st_row * (int)tok_stride + st_piece * 16);
  struct KRows { uint4 v[NLD]; };
  auto fetch = [&](int tile) __attribute__((always_inline)) -> KRows {
    KRows r;
    const int tbase = tile * kPfTile + wave_u * 16;
    if (a.P >= 16 && tbase + 16 <= Nc) {                      // uniform per wave
      const int page = a.page_indices[indptr + (tbase >> a.p_shift)];
      const uint8_t* base = a.k_pool + ((((size_t)page << a.p_shift) + (size_t)(tbase & (a.P - 1))) * a.H_kv + kvh) * RBYTES;
#pragma unroll
      for (int it = 0; it < NLD; ++it)
        r.v[it] = *reinterpret_cast<const uint4*>(base + (size_t)it * RPW * tok_stride + lane_off);
    } else {
#pragma unroll
      for (int it = 0; it < NLD; ++it) {
        int t = tbase + st_row + it * RPW;
        t = max(min(t, Nc - 1), 0);                           // the last tile may be ragged: shadow the last token
        const int page = a.page_indices[indptr + (t >> a.p_shift)];
        const uint8_t* kp = a.k_pool + ((((size_t)page << a.p_shift) + (t & (a.P - 1))) * a.H_kv + kvh) * RBYTES + st_piece * 16;
        r.v[it] = *reinterpret_cast<const uint4*>(kp);
      }
    }
    return r;
  };
  auto stage = [&](int buf, const KRows& r) {
#pragma unroll
    for (int it = 0; it < NLD; ++it)
      *reinterpret_cast<uint4*>(&s_k[buf][(wave_u * 16 + st_row + it * RPW) * LROW + st_piece * 16]) = r.v[it];
  };

  KRows kreg;
#pragma unroll
  for (int it = 0; it < NLD; ++it) kreg.v[it] = make_uint4(0, 0, 0, 0);
  if (tile_begin < tile_end) {
    stage(0, fetch(tile_begin));
    if (tile_begin + 1 < tile_end) kreg = fetch(tile_begin + 1);
  }
  __syncthreads();

  float* vout = (SWEEP == 2) ? a.vote_part + ((size_t)b * a.RB * a.H_kv + (size_t)rb * a.H_kv + kvh) * a.max_seq_len : nullptr;

  // one 64-row x 32-token block on the matrix cores; k-steps [ks0, ks1) (the first clears the accumulators)
  auto mfma_part = [&](int buf, int nb, f32x16_t (&acc)[2], auto ks0_c, auto ks1_c) __attribute__((always_inline)) {
    constexpr int ks0 = decltype(ks0_c)::value, ks1 = decltype(ks1_c)::value;
    if (ks0 == 0) {
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[mb][e] = 0.f;
    }
#pragma unroll
    for (int ks = ks0; ks < ks1; ++ks) {
      // B[k][n] = K[token n][d k]: lane holds token n = col, d = 16 * ks + 8 * half .. + 8
      const uint4 bv = *reinterpret_cast<const uint4*>(&s_k[buf][(nb * 32 + col) * LROW + (ks * 2 + half) * 16]);
      const bf16x8_t bfrag = __builtin_bit_cast(bf16x8_t, bv);
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
        acc[mb] = SWEEP == 1 ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfrag, afrag[mb][ks], acc[mb], 0, 0, 0)
                             : __builtin_amdgcn_mfma_f32_32x32x16_bf16(afrag[mb][ks], bfrag, acc[mb], 0, 0, 0);
    }
  };
  using K0 = std::integral_constant<int, 0>;
  using KH = std::integral_constant<int, KS / 2>;
  using KE = std::integral_constant<int, KS>;
  auto mfma_block = [&](int buf, int nb, f32x16_t (&acc)[2]) { mfma_part(buf, nb, acc, K0{}, KE{}); };

  // Softmax arithmetic of one block on the vector ALU, overlapped with the MFMAs of the next block `nacc`.
  // Sweep 1 has a (rare) branch in the middle -- a reference has to be raised -- and the scheduler cannot move MFMAs
  // across it, so half of the next block's k-steps are issued before it and half after it.  RAGGED: the tile holds
  // columns outside the ranked range; they get weight 0 in the sum (a full tile needs neither mask nor weight).
  auto step = [&](auto ragged, const f32x16_t (&acc)[2], int tile, int nb, int cbuf, int nbuf, int nnb, f32x16_t (&nacc)[2]) __attribute__((always_inline)) {
    constexpr bool RAGGED = decltype(ragged)::value;
    if (SWEEP == 1) {
      // acc[mb][e]: token 8 * (e / 4) + 4 * half + e % 4 of the block, query row mb * 32 + col
      mfma_part(nbuf, nnb, nacc, K0{}, KH{});
      float mraw[2], xm[2];
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) {
        float m = acc[mb][0];
#pragma unroll
        for (int e = 1; e < 16; ++e) m = fmaxf(m, acc[mb][e]);
        mraw[mb] = m;
        xm[mb] = fmaf(c2, m, -off1[mb]);          // the largest argument (c2 >= 0); +inf while off1 is unset
      }
      // first block of a lane, or a score far above the reference (tokens outside the ranked range shadow a real
      // token or are real tokens: a reference they raise is as good as any other)
      if (__builtin_amdgcn_ballot_w64(fmaxf(xm[0], xm[1]) > 64.f) != 0) {
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
          if (xm[mb] > 64.f) {
            // the new reference sits kRefHead above the value that forced it: without head room the next larger
            // score would raise it again
            const float noff = c2 * mraw[mb] + kRefHead;
            aux1[mb] = (off1[mb] == -INFINITY) ? 0.f : aux1[mb] * __builtin_amdgcn_exp2f(off1[mb] - noff);
            off1[mb] = noff;
          }
      }
      mfma_part(nbuf, nnb, nacc, KH{}, KE{});
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) {
        float s0 = 0.f, s1 = 0.f;
#pragma unroll
        for (int e = 0; e < 16; e += 2) {
          float e0 = __builtin_amdgcn_exp2f(fmaf(c2, acc[mb][e], -off1[mb]));        // arguments are <= 64: finite
          float e1 = __builtin_amdgcn_exp2f(fmaf(c2, acc[mb][e + 1], -off1[mb]));
          if (RAGGED) {
            const int t0 = tile * kPfTile + nb * 32 + 8 * (e >> 2) + 4 * half + (e & 3);
            e0 = (t0 >= r_lo && t0 < r_hi) ? e0 : 0.f;
            e1 = (t0 + 1 >= r_lo && t0 + 1 < r_hi) ? e1 : 0.f;
          }
          s0 += e0; s1 += e1;
        }
        aux1[mb] += s0 + s1;
      }
    } else {
      mfma_part(nbuf, nnb, nacc, K0{}, KE{});
      float cs = 0.f;
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int e = 0; e < 16; ++e) cs = fmaf(__builtin_amdgcn_exp2f(fmaf(c2, acc[mb][e], -off[mb][e])), aux[mb][e], cs);
      cs += __shfl_xor(cs, 32);                              // the other 16 rows of each block
      if (half == 0) s_col[cbuf][wave][nb * 32 + col] = cs;  // columns outside the range are dropped by write_votes
    }
  };
  auto write_votes = [&](int tile, int cbuf) {
    if (SWEEP == 2 && threadIdx.x < kPfTile) {
      const int t = tile * kPfTile + threadIdx.x;
      if (t >= r_lo && t < r_hi) vout[t] = (s_col[cbuf][0][threadIdx.x] + s_col[cbuf][1][threadIdx.x]) + (s_col[cbuf][2][threadIdx.x] + s_col[cbuf][3][threadIdx.x]);
    }
  };

  // Software pipeline over the blocks (tile, first half) (tile, second half) ...: the MFMAs of the next
  // block are issued with the softmax of the current one, so the matrix cores work while the vector
  // ALU exponentiates.  One barrier per tile publishes the staged K rows of the next tile.
  // The loop body is straight-line code (staging, fetching and the look-ahead MFMAs also run on the last tiles,
  // where their results are not used): only then can the compiler's scheduler mix MFMAs and vector instructions.
  f32x16_t acc0[2], acc1[2];
  if (tile_begin < tile_end) mfma_block(0, 0, acc0);
  auto body = [&](auto ragged, int tile) __attribute__((always_inline)) {
    const int it = tile - tile_begin;
    const int buf = it & 1, cbuf = it % 3;
    stage(buf ^ 1, kreg);                                    // rows fetched during the previous iteration
    kreg = fetch(min(tile + 2, tile_end - 1));
    step(ragged, acc0, tile, 0, cbuf, buf, 1, acc1);
    __syncthreads();                                         // next tile's rows are staged; all waves are done with tile - 1
    if (it > 0) write_votes(tile - 1, (it - 1) % 3);
    step(ragged, acc1, tile, 1, cbuf, buf ^ 1, 0, acc0);
  };
  // only the first and the last tile of the ranked range can be ragged: they are peeled off, so that the loop over
  // the full tiles holds one variant of the body
  int tile = tile_begin;
  if (SWEEP == 1 && tile < tile_end && tile * kPfTile < r_lo) { body(std::true_type{}, tile); ++tile; }
  const int full_end = (SWEEP == 1 && tile_end * kPfTile > r_hi) ? max(tile, tile_end - 1) : tile_end;
  for (; tile < full_end; ++tile) body(std::false_type{}, tile);
  for (; tile < tile_end; ++tile) body(std::true_type{}, tile);
  if (tile_begin < tile_end) {
    __syncthreads();
    write_votes(tile_end - 1, (tile_end - 1 - tile_begin) % 3);
  }

  if (SWEEP == 1) {
    // a query row's sums sit in the two lanes col and col + 32 (disjoint tokens): merge them
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) {
      const float m = off1[mb], l = aux1[mb];
      const float mo = __shfl_xor(m, 32), lo = __shfl_xor(l, 32);
      const float mn = fmaxf(m, mo);
      const float la = (m == -INFINITY) ? 0.f : l * __builtin_amdgcn_exp2f(m - mn);
      const float lb = (mo == -INFINITY) ? 0.f : lo * __builtin_amdgcn_exp2f(mo - mn);
      const int row = rb * kPfRowsPerWg + wave * 64 + mb * 32 + col;
      if (half == 0 && row < nrows) {
        const int c = row / G, g = row % G;
        float* pp = a.stat_part + ((((size_t)b * a.TS + split) * C + c) * H + kvh * G + g) * 2;
        pp[0] = mn; pp[1] = la + lb;                             // (reference exponent, sum of exp2(arg - reference))
      }
    }
  }
}

// row_stats[b][c][h] = log2 sum_t exp2(c2 * s_t) as a (high, low) float pair, from the splits' partials.
// 32 lanes per row, one split each (two when there are more than 32 splits): the partials of a row are a
// strided gather, so they should all be in flight at once.
__global__ __launch_bounds__(256) void prefill_stats_merge_kernel(PrefillArgs a) {
  const int lane32 = threadIdx.x & 31;
  const int i = blockIdx.x * 8 + (threadIdx.x >> 5);     // (b, c, h) flattened; eight rows per workgroup
  const int n = a.B * a.C * a.H;
  const bool row_ok = i < n;
  const int ic = row_ok ? i : n - 1;
  const int b = ic / (a.C * a.H), ch = ic % (a.C * a.H);
  float2 v[2];
#pragma unroll
  for (int e = 0; e < 2; ++e) {
    const int sp = lane32 + 32 * e;
    v[e] = make_float2(-INFINITY, 0.f);
    if (sp < a.TS) v[e] = *reinterpret_cast<const float2*>(a.stat_part + (((size_t)b * a.TS + sp) * a.C * a.H + ch) * 2);
  }
  float m = fmaxf(v[0].x, v[1].x);
#pragma unroll
  for (int o = 1; o < 32; o <<= 1) m = fmaxf(m, __shfl_xor(m, o));
  double l = 0.0;
#pragma unroll
  for (int e = 0; e < 2; ++e)
    if (v[e].x != -INFINITY) l += (double)v[e].y * exp_f64(0.69314718055994530942 * ((double)v[e].x - (double)m));
#pragma unroll
  for (int o = 1; o < 32; o <<= 1) l += __shfl_xor(l, o);
  if (!row_ok || lane32 != 0) return;
  const double lse2 = (m == -INFINITY) ? -INFINITY : (double)m + log2(l);
  const float hi = (float)lse2;
  a.row_stats_out[(size_t)i * 2] = hi;
  a.row_stats_out[(size_t)i * 2 + 1] = (m == -INFINITY) ? 0.f : (float)(lse2 - (double)hi);
}

// votes[b][t] = sum over the (row block, KV head) partial vote vectors, double accumulation
__global__ __launch_bounds__(256) void prefill_vote_reduce_kernel(PrefillArgs a) {
  const int b = blockIdx.y;
  const int t = blockIdx.x * 256 + threadIdx.x;
  const int Nc = min(max(a.seq_lens[b] - a.C, 0), a.max_seq_len);
  if (t >= Nc) return;
  const int r_lo = min(a.n_init, Nc), r_hi = max(r_lo, Nc - a.n_local);
  if (t < r_lo || t >= r_hi) { a.votes[(size_t)b * a.max_seq_len + t] = 0.f; return; }   // forced tokens are not ranked
  const int np = a.RB * a.H_kv;
  const float* p = a.vote_part + (size_t)b * np * a.max_seq_len + t;
  double v = 0.0;
  int i = 0;
  for (; i + 8 <= np; i += 8) {
    float x[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = p[(size_t)(i + e) * a.max_seq_len];
#pragma unroll
    for (int e = 0; e < 8; ++e) v += (double)x[e];
  }
  for (; i < np; ++i) v += (double)p[(size_t)i * a.max_seq_len];
  a.votes[(size_t)b * a.max_seq_len + t] = (float)v;
}

hipError_t launch_prefill_stats(const PrefillArgs& a, hipStream_t s) {
  const int groups = a.B * a.H_kv * a.TS;
  const int grid = (groups + 7) / 8 * 8 * a.RB;
  if (a.D == 128) hipLaunchKernelGGL((prefill_qk_kernel<128, 1>), dim3(grid), dim3(256), 0, s, a);
  else hipLaunchKernelGGL((prefill_qk_kernel<64, 1>), dim3(grid), dim3(256), 0, s, a);
  hipLaunchKernelGGL(prefill_stats_merge_kernel, dim3((a.B * a.C * a.H + 7) / 8), dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_prefill_votes(const PrefillArgs& a, hipStream_t s) {
  const int groups = a.B * a.H_kv * a.TS;
  const int grid = (groups + 7) / 8 * 8 * a.RB;
  if (a.D == 128) hipLaunchKernelGGL((prefill_qk_kernel<128, 2>), dim3(grid), dim3(256), 0, s, a);
  else hipLaunchKernelGGL((prefill_qk_kernel<64, 2>), dim3(grid), dim3(256), 0, s, a);
  hipLaunchKernelGGL(prefill_vote_reduce_kernel, dim3((a.max_seq_len + 255) / 256, a.B), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace ts
