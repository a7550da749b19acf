// Eq. 2 (selective sparse attention), chunk form: each of the C queries of a prefill chunk attends
// over the shared selected tokens plus the chunk's own tokens up to and including itself, in one
// joint softmax ([K_select, K_current] of Eq. 2 with a causal mask inside the chunk).
//
// Matrix-core flash attention over a gathered key list.  A small kernel first resolves the key list
// of a sequence (selected tokens, then the chunk's tokens) to physical slots.  In the main kernel a
// workgroup owns 128 rows (query x head pairs of one KV head; 32 per wave, fragments pinned in
// registers) and walks the key list in tiles of 32: K rows and V rows of the tile are gathered once
// into LDS (row-major both; the V operand of P V is read as eight 2-byte pieces down a column), S = Q K^T and O += P V run
// on v_mfma_f32_32x32x16_bf16, P goes through a wave-private LDS tile to change from the result
// layout to the operand layout.  The softmax uses a per-row reference exponent that is raised only
// when a logit would exceed it by 2^16, so the common tile needs no cross-lane traffic; row sums
// are merged once at the end.  The next tile's rows are in flight while the current one is used.
#include "ts_kernels.h"

namespace ts {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

constexpr int kCaRows = 128;   // rows per workgroup
constexpr int kCaTile = 32;    // keys per tile

// slots[b][j]: physical slot of the j-th key of sequence b: the count[b] selected tokens, then the
// chunk's C tokens (logical positions N_b - C ...); with forced tokens the selected ones are preceded by the initial
// block and followed by the cached tokens just before the chunk
__global__ __launch_bounds__(256) void chunk_slots_kernel(ChunkAttnArgs a) {
  const int b = blockIdx.y;
  const int j = blockIdx.x * 256 + threadIdx.x;
  const int cnt = min(max(a.count[b], 0), a.idx_stride);
  const int N = min(max(a.seq_lens[b], 0), a.max_seq_len);
  if (N < a.C) return;                                          // shorter than a chunk: holds none, nothing is attended
  const int Nc = max(N - a.C, 0);                               // cached tokens before the chunk
  const int f_lo = min(a.n_init, Nc), f_hi = max(f_lo, Nc - a.n_local);   // forced blocks [0, f_lo) and [f_hi, Nc)
  const int nsel = f_lo + cnt + (Nc - f_hi);                    // keys every query of the chunk sees
  if (j >= nsel + a.C) return;
  int t;
  if (j < f_lo) t = j;
  else if (j < f_lo + cnt) t = a.idx[(size_t)b * a.idx_stride + (j - f_lo)];
  else if (j < nsel) t = f_hi + (j - f_lo - cnt);
  else t = N - a.C + (j - nsel);
  t = min(max(t, 0), max(N, 1) - 1);             // a stale or corrupt index must not leave the page table
  const int page = a.page_indices[a.page_indptr[b] + (t >> a.p_shift)];
  a.slots[(size_t)b * a.slot_stride + j] = (page << a.p_shift) + (t & (a.P - 1));
}

template <int D>
__global__ __launch_bounds__(256) void chunk_attn_kernel(ChunkAttnArgs a) {
  constexpr int KS = D / 16;                     // k-steps of Q K^T
  constexpr int NBO = D / 32;                    // 32-column blocks of the output
  constexpr int RBYTES = D * 2;
  constexpr int PPR = RBYTES / 16;               // 16-byte pieces per K/V row
  constexpr int NLD = kCaTile * PPR / 256;       // gather loads per thread per tile and per pool (2 for D = 128)
  constexpr int LROW = RBYTES + 16;              // padded K row in LDS
  constexpr int VROW = kCaTile * 2 + 16;         // padded V^T row in LDS: 32 keys of bf16
  constexpr float TH = 16.f;
  static_assert(NLD >= 1, "tile too small for the workgroup");
  __shared__ __attribute__((aligned(16))) uint8_t s_k[2][kCaTile * LROW];
  __shared__ __attribute__((aligned(16))) uint8_t s_v[2][kCaTile * LROW];    // V rows as gathered ([key][d]); transposed on the way out
  __shared__ __attribute__((aligned(16))) uint8_t s_p[4][32 * VROW];

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int half = lane >> 5, col = lane & 31;
  const int rb = blockIdx.x / a.nsplit, split = blockIdx.x % a.nsplit, kvh = blockIdx.y, b = blockIdx.z;
  const int C = a.C, G = a.G, H = a.H;
  const int nrows = C * G;
  // keys every query sees: forced initial block, selected tokens, forced block before the chunk (see chunk_slots_kernel)
  const int Nc_ = max(min(max(a.seq_lens[b], 0), a.max_seq_len) - C, 0);
  const int f_lo_ = min(a.n_init, Nc_), f_hi_ = max(f_lo_, Nc_ - a.n_local);
  const int cnt = f_lo_ + min(max(a.count[b], 0), a.idx_stride) + (Nc_ - f_hi_);
  const int r0 = rb * kCaRows;
  if (r0 >= nrows) return;
  if (min(max(a.seq_lens[b], 0), a.max_seq_len) < C) {
    // a sequence shorter than the chunk holds no chunk (an idle slot of the batch): its rows are zero, and nothing is
    // read through its page table, which may be empty
    for (int i = threadIdx.x; i < kCaRows * D; i += 256) {
      const int row = r0 + i / D, d = i % D;
      if (row >= nrows) break;
      const size_t hb = ((size_t)b * C + row / G) * H + kvh * G + row % G;
      if (a.nsplit == 1) {
        reinterpret_cast<uint16_t*>(a.out)[hb * D + d] = 0;
        if (d == 0 && a.lse != nullptr) a.lse[hb] = -INFINITY;
      } else {
        a.part_o[(hb * a.nsplit + split) * D + d] = 0.f;
        if (d == 0) { float* pm = a.part_ml + (hb * a.nsplit + split) * 2; pm[0] = -INFINITY; pm[1] = 0.f; }
      }
    }
    return;
  }
  const int c_last = min(C - 1, (r0 + kCaRows - 1) / G);      // last query of this row block
  const int nkeys = cnt + c_last + 1;                          // keys any row of the block may see
  const int ntile_all = (nkeys + kCaTile - 1) / kCaTile;
  // this workgroup's share of the key list (tiles [tile0, tile0 + ntile)); may be empty
  const int tps = (ntile_all + a.nsplit - 1) / a.nsplit;
  const int tile0 = min(split * tps, ntile_all);
  const int ntile = min(tps, ntile_all - tile0);
  const int* slots = a.slots + (size_t)b * a.slot_stride;
  const float c2 = a.sm_scale * 1.44269504088896340736f;

  // ---- query fragments (A operand of Q K^T): lane holds row = col, k = 16 * ks + 8 * half .. + 8
  bf16x8_t qfrag[KS];
  {
    const int row = r0 + wave * 32 + col;
    const bool valid = row < nrows;
    const int c = valid ? row / G : 0, g = valid ? row % G : 0;
    const uint8_t* qp = a.q + ((((size_t)b * C + c) * H + (size_t)kvh * G + g) * D + 8 * half) * 2;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (valid) v = *reinterpret_cast<const uint4*>(qp + ks * 32);
      qfrag[ks] = __builtin_bit_cast(bf16x8_t, v);
    }
  }
  // rows of the result layout held by this lane: 8 * i + 4 * half + j; the query index decides causality
  int qidx[16];
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    const int row = r0 + wave * 32 + 8 * (e >> 2) + 4 * half + (e & 3);
    qidx[e] = row / G;
  }
  float ref[16], lsum[16];
#pragma unroll
  for (int e = 0; e < 16; ++e) { ref[e] = -INFINITY; lsum[e] = 0.f; }
  f32x16_t oacc[NBO];
#pragma unroll
  for (int nb = 0; nb < NBO; ++nb)
#pragma unroll
    for (int e = 0; e < 16; ++e) oacc[nb][e] = 0.f;

  // ---- gather staging: thread -> (key within pass, 16-byte piece)
  const int st_key = threadIdx.x / PPR, st_piece = threadIdx.x % PPR;
  constexpr int KPP = 256 / PPR;                 // keys per pass
  struct Rows { uint4 k[NLD]; uint4 v[NLD]; };
  struct Slots { int v[NLD]; };
  // the slots of a tile are read one tile earlier than its rows: the slot list and the pools are two dependent
  // round trips, and a tile's arithmetic is too short to hide both
  auto fetch_slots = [&](int tile) -> Slots {
    Slots r;
#pragma unroll
    for (int it = 0; it < NLD; ++it) r.v[it] = slots[min((tile0 + tile) * kCaTile + st_key + it * KPP, nkeys - 1)];   // ragged last tile: shadow the last key
    return r;
  };
  auto fetch = [&](const Slots& sl) -> Rows {
    Rows r;
#pragma unroll
    for (int it = 0; it < NLD; ++it) {
      const size_t o = ((size_t)sl.v[it] * a.H_kv + kvh) * RBYTES + st_piece * 16;
      r.k[it] = *reinterpret_cast<const uint4*>(a.k_pool + o);
      r.v[it] = *reinterpret_cast<const uint4*>(a.v_pool + o);
    }
    return r;
  };
  auto stage = [&](int buf, const Rows& r) {
#pragma unroll
    for (int it = 0; it < NLD; ++it) {
      const int key = st_key + it * KPP;
      *reinterpret_cast<uint4*>(&s_k[buf][key * LROW + st_piece * 16]) = r.k[it];
      *reinterpret_cast<uint4*>(&s_v[buf][key * LROW + st_piece * 16]) = r.v[it];
    }
  };

  Rows pre;
#pragma unroll
  for (int it = 0; it < NLD; ++it) { pre.k[it] = make_uint4(0, 0, 0, 0); pre.v[it] = make_uint4(0, 0, 0, 0); }
  Slots spre;
#pragma unroll
  for (int it = 0; it < NLD; ++it) spre.v[it] = 0;
  stage(0, fetch(fetch_slots(0)));
  if (ntile > 1) pre = fetch(fetch_slots(1));
  if (ntile > 2) spre = fetch_slots(2);
  __syncthreads();

  for (int tile = 0; tile < ntile; ++tile) {
    const int buf = tile & 1;
    if (tile + 1 < ntile) stage(buf ^ 1, pre);
    if (tile + 2 < ntile) pre = fetch(spre);
    if (tile + 3 < ntile) spre = fetch_slots(tile + 3);

    // ---- S = Q K^T for 32 rows x 32 keys
    f32x16_t sacc;
#pragma unroll
    for (int e = 0; e < 16; ++e) sacc[e] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const uint4 bv = *reinterpret_cast<const uint4*>(&s_k[buf][col * LROW + (ks * 2 + half) * 16]);
      sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qfrag[ks], __builtin_bit_cast(bf16x8_t, bv), sacc, 0, 0, 0);
    }
    // ---- mask and exponent arguments; key j of this lane's column
    const int j = (tile0 + tile) * kCaTile + col;
    const int cq = j - cnt;                                    // >= 0: the chunk's token cq
    float raw[16], ar[16];
    float amax = -INFINITY;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const bool vis = (j < cnt) || (j < nkeys && cq <= qidx[e]);
      raw[e] = vis ? c2 * sacc[e] : -INFINITY;
      ar[e] = raw[e] - ref[e];                                 // +inf while the reference is unset and the key visible
      ar[e] = (raw[e] == -INFINITY) ? -INFINITY : ar[e];
      amax = fmaxf(amax, ar[e]);
    }
    if (__builtin_amdgcn_ballot_w64(amax > TH) != 0) {         // first visible key of a row, or a logit far above the reference
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        float rmax = raw[e];
#pragma unroll
        for (int o = 1; o < 32; o <<= 1) rmax = fmaxf(rmax, __shfl_xor(rmax, o));   // over the row's 32 columns
        if (rmax - ref[e] > TH) {                              // same decision in all lanes of the row
          const float f = (ref[e] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(ref[e] - rmax);
          lsum[e] *= f;
#pragma unroll
          for (int nb = 0; nb < NBO; ++nb) oacc[nb][e] *= f;
          ref[e] = rmax;
          ar[e] = (raw[e] == -INFINITY) ? -INFINITY : raw[e] - rmax;
        }
      }
    }
    // ---- P (bf16) into the wave's LDS tile, row-major [row][key], and the row sums
    uint8_t* pw = s_p[wave];
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const float p = __builtin_amdgcn_exp2f(ar[e]);           // exp2(-inf) = 0 for masked keys
      const uint32_t pb = f32_to_bf16_bits(p);
      lsum[e] += __uint_as_float(pb << 16);                    // the sum uses the rounded weights that multiply V
      const int row = 8 * (e >> 2) + 4 * half + (e & 3);
      *reinterpret_cast<uint16_t*>(&pw[row * VROW + col * 2]) = (uint16_t)pb;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // ---- O += P V: A = P[row = col][keys 16 * ks + 8 * half ..], B = V^T[d = 32 * nb + col][same keys]
#pragma unroll
    for (int ks = 0; ks < kCaTile / 16; ++ks) {
      const uint4 pa = *reinterpret_cast<const uint4*>(&pw[col * VROW + (ks * 16 + 8 * half) * 2]);
#pragma unroll
      for (int nb = 0; nb < NBO; ++nb) {
        // B operand: column d = 32 * nb + col of eight consecutive keys -- eight 2-byte reads down a column of the
        // row-major V tile (a wave's 32 columns of one key are 64 contiguous bytes: no bank conflicts; writing V
        // transposed instead cost 16-way conflicts on 2-byte stores)
        const uint8_t* vcol = &s_v[buf][(ks * 16 + 8 * half) * LROW + (nb * 32 + col) * 2];
        uint32_t vw[4];
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          const uint32_t lo16 = *reinterpret_cast<const uint16_t*>(vcol + (2 * jj) * LROW);
          const uint32_t hi16 = *reinterpret_cast<const uint16_t*>(vcol + (2 * jj + 1) * LROW);
          vw[jj] = lo16 | (hi16 << 16);
        }
        const uint4 vb = make_uint4(vw[0], vw[1], vw[2], vw[3]);
        oacc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, pa), __builtin_bit_cast(bf16x8_t, vb),
                                                            oacc[nb], 0, 0, 0);
      }
    }
    __syncthreads();
  }

  // ---- finish: row sums over the 32 columns; normalise and write, or hand the partial to the merge kernel
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    float l = lsum[e];
#pragma unroll
    for (int o = 1; o < 32; o <<= 1) l += __shfl_xor(l, o);
    const int row = r0 + wave * 32 + 8 * (e >> 2) + 4 * half + (e & 3);
    if (row < nrows) {
      const int c = row / G, g = row % G;
      const size_t hb = ((size_t)b * C + c) * H + kvh * G + g;
      if (a.nsplit == 1) {
        const float inv = l > 0.f ? 1.f / l : 0.f;
#pragma unroll
        for (int nb = 0; nb < NBO; ++nb)
          reinterpret_cast<uint16_t*>(a.out)[hb * D + nb * 32 + col] = (uint16_t)f32_to_bf16_bits(oacc[nb][e] * inv);
        if (a.lse != nullptr && col == 0) a.lse[hb] = l > 0.f ? (ref[e] + __builtin_amdgcn_logf(l)) * 0.69314718055994530942f : -INFINITY;
      } else {
        float* po = a.part_o + (hb * a.nsplit + split) * D;
#pragma unroll
        for (int nb = 0; nb < NBO; ++nb) po[nb * 32 + col] = oacc[nb][e];
        if (col == 0) { float* pm = a.part_ml + (hb * a.nsplit + split) * 2; pm[0] = ref[e]; pm[1] = l; }
      }
    }
  }
}

// Merges the key-list splits of one row: with M = max_s ref_s (base-2 exponents),
// out = sum_s 2^(ref_s - M) O_s / sum_s 2^(ref_s - M) l_s.  One workgroup of D threads per row.
template <int D>
__global__ __launch_bounds__(D) void chunk_attn_merge_kernel(ChunkAttnArgs a) {
  const size_t hb = blockIdx.x;
  const int d = threadIdx.x;
  const float* pm = a.part_ml + hb * a.nsplit * 2;
  float M = -INFINITY;
  for (int s = 0; s < a.nsplit; ++s) M = fmaxf(M, pm[2 * s]);
  float L = 0.f, o = 0.f;
  for (int s = 0; s < a.nsplit; ++s) {
    const float r = pm[2 * s];
    const float w = (r == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(r - M);
    L = fmaf(w, pm[2 * s + 1], L);
    o = fmaf(w, a.part_o[(hb * a.nsplit + s) * D + d], o);
  }
  reinterpret_cast<uint16_t*>(a.out)[hb * D + d] = (uint16_t)f32_to_bf16_bits(L > 0.f ? o / L : 0.f);
  if (a.lse != nullptr && d == 0) a.lse[hb] = L > 0.f ? (M + __builtin_amdgcn_logf(L)) * 0.69314718055994530942f : -INFINITY;
}

hipError_t launch_sparse_attn_chunk(const ChunkAttnArgs& a, int B, hipStream_t s) {
  hipLaunchKernelGGL(chunk_slots_kernel, dim3((a.slot_stride + 255) / 256, B), dim3(256), 0, s, a);
  const int nrb = (a.C * a.G + kCaRows - 1) / kCaRows;
  const dim3 grid(nrb * a.nsplit, a.H_kv, B);
  if (a.D == 128) hipLaunchKernelGGL(chunk_attn_kernel<128>, grid, dim3(256), 0, s, a);
  else hipLaunchKernelGGL(chunk_attn_kernel<64>, grid, dim3(256), 0, s, a);
  if (a.nsplit > 1) {
    const int rows = B * a.C * a.H;
    if (a.D == 128) hipLaunchKernelGGL(chunk_attn_merge_kernel<128>, dim3(rows), dim3(128), 0, s, a);
    else hipLaunchKernelGGL(chunk_attn_merge_kernel<64>, dim3(rows), dim3(64), 0, s, a);
  }
  return hipGetLastError();
}

}  // namespace ts
