// Shared device helpers and workspace layout for the TokenSelect gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "tokenselect.h"

namespace ts {

constexpr int kWave = 64;
constexpr int kScoreTileTokens = 32;   // tokens per wave tile in the score pass
constexpr int kScoreLdsStride = 36;    // floats per head row of the staged score tile (16 B aligned)
constexpr int kScoreMaxWg = 1024;      // upper bound on workgroups per sequence in the score pass
constexpr int kTopkBins = 2048;        // 11-bit radix digit
constexpr int kTopkChunk = 2048;       // keys per workgroup in the top-k passes
constexpr int kBoundHistCopies = 8;    // replicas of the lower-bound histogram (same-address atomics are what its flush costs)
constexpr int kAttnChunk = 64;         // selected tokens per workgroup in sparse attention
constexpr int kAttnMaxRun = 4;        // chunks one attention workgroup folds into its partial, at most (256 list entries: one per thread)
constexpr int kAttnMaxSplit = 512;     // splits the merge kernel can stage (k <= 32768)

// ---------------------------------------------------------------- workspace layout (host + device)
struct WsLayout {
  size_t topk_hist;        // uint32 [B][3][kTopkBins] : one histogram per radix pass (must start zeroed)
  size_t bound_hist;       // uint32 [B][kBoundHistCopies][kTopkBins] : compact selection, histogram of the vote lower bounds
                           // (must start zeroed too; decode only)
  size_t topk_state;       // uint32 [B][8] : digits and remaining ranks fixed so far
  size_t hdr;              // uint32 [B][8] : left by the score pass for the calls that follow it
  size_t score_partials;   // float [B][kScoreMaxWg][H][2]
  size_t topk_blk;         // uint32 [B][nblk] : per-chunk counts
  size_t topk_list;        // uint2 [B][nblk][kTopkChunk] : compacted (key, token) entries of the short top-k path
  size_t blk_max;          // float [B][score_nblk][H] : compact score pass, per-block head maxima (decode only)
  int score_nblk;          // ceil(max_seq_len / kScoreTileTokens)
  size_t attn_out;         // float [B][H][nsplit][D]
  size_t attn_ml;          // float [B][H][nsplit][2]
  size_t pf_stat_part;     // float [B][TS][C][H][2]            (chunk > 1 only)
  size_t pf_vote_part;     // float [B][RB * H_kv][max_seq_len] (chunk > 1 only)
  size_t attn_slots;       // int32 [B][k + C]                  (chunk > 1 only)
  size_t attn_chunk_o;     // float [B][C][H][nsplit][D]        (chunk > 1 with key-list splits)
  size_t attn_chunk_ml;    // float [B][C][H][nsplit][2]
  int attn_chunk_nsplit;
  size_t total;
  int pf_rb, pf_ts;
  int topk_nblk;
  int attn_nsplit;
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Key-list splits of the chunk-form attention: its rows alone give few waves (config 5: 512 on 1024 SIMDs), so the
// key list is split until about two waves per SIMD are in flight; every split keeps at least four 32-key tiles.
inline int chunk_attn_splits(const ts_problem* p, int k) {
  const int G = p->num_q_heads / p->num_kv_heads;
  const long waves = (long)((p->chunk * G + 127) / 128) * 4 * p->num_kv_heads * p->batch;
  const int ntile = (k + p->num_initial + p->num_local + p->chunk + 31) / 32;
  int s = (int)((2048 + waves - 1) / waves);
  if (s > 8) s = 8;
  if (s > ntile / 4) s = ntile / 4;
  if (s < 1) s = 1;
  return s;
}

inline WsLayout ws_layout(const ts_problem* p, int k) {
  WsLayout w{};
  const size_t B = (size_t)p->batch, H = (size_t)p->num_q_heads, D = (size_t)p->head_dim;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
  w.topk_nblk = (p->max_seq_len + kTopkChunk - 1) / kTopkChunk;
  if (w.topk_nblk < 1) w.topk_nblk = 1;
  w.attn_nsplit = (k + p->num_initial + p->num_local + kAttnChunk - 1) / kAttnChunk;   // forced tokens join the list
  if (w.attn_nsplit < 1) w.attn_nsplit = 1;
  // the histograms come first: they are the part that must start (and is left) zeroed
  w.topk_hist = take(B * 3 * kTopkBins * 4);
  if (p->chunk == 1) w.bound_hist = take(B * kBoundHistCopies * kTopkBins * 4);
  w.topk_state = take(B * 8 * 4);
  w.hdr = take(B * 8 * 4);
  w.score_partials = take(B * kScoreMaxWg * H * 2 * 4);
  w.topk_blk = take(B * (size_t)w.topk_nblk * 4);
  w.topk_list = take(B * (size_t)w.topk_nblk * kTopkChunk * 8);
  w.score_nblk = (p->max_seq_len + kScoreTileTokens - 1) / kScoreTileTokens;
  if (p->chunk == 1) {
    w.blk_max = take(B * (size_t)w.score_nblk * H * 4);
  }
  if (p->chunk > 1) {
    const int G = p->num_q_heads / p->num_kv_heads;
    w.pf_rb = (p->chunk * G + 255) / 256;
    const int ntile = (p->max_seq_len + 63) / 64;
    int ts = 2048 / (p->batch * p->num_kv_heads * w.pf_rb);
    if (ts > 64) ts = 64;
    if (ts > ntile) ts = ntile;
    if (ts < 1) ts = 1;
    w.pf_ts = ts;
    w.pf_stat_part = take(B * (size_t)ts * p->chunk * H * 2 * 4);
    w.pf_vote_part = take(B * (size_t)w.pf_rb * p->num_kv_heads * (size_t)p->max_seq_len * 4);
  }
  // the sections that depend on k come last, so that every other offset is the same for any k
  w.attn_out = take(B * H * (size_t)w.attn_nsplit * D * 4);
  w.attn_ml = take(B * H * (size_t)w.attn_nsplit * 2 * 4);
  if (p->chunk > 1) {
    w.attn_slots = take(B * ((size_t)k + p->num_initial + p->num_local + p->chunk) * 4);
    w.attn_chunk_nsplit = chunk_attn_splits(p, k);
    if (w.attn_chunk_nsplit > 1) {
      w.attn_chunk_o = take(B * p->chunk * H * (size_t)w.attn_chunk_nsplit * D * 4);
      w.attn_chunk_ml = take(B * p->chunk * H * (size_t)w.attn_chunk_nsplit * 2 * 4);
    }
  }
  w.total = off;
  return w;
}

#ifdef __HIPCC__
// ---------------------------------------------------------------- device helpers
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// round-to-nearest-even float -> bf16 bits (finite inputs)
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}
// sum over the 8 lanes of an aligned lane group; every lane of the group gets the total
__device__ __forceinline__ float group8_sum(float v) {
  v += dpp_f32<0xB1>(v);    // quad_perm [1,0,3,2]
  v += dpp_f32<0x4E>(v);    // quad_perm [2,3,0,1]
  v += dpp_f32<0x141>(v);   // row_half_mirror
  return v;
}
__device__ __forceinline__ float group16_sum(float v) {
  v = group8_sum(v);
  v += dpp_f32<0x140>(v);   // row_mirror
  return v;
}
__device__ __forceinline__ float group8_max(float v) {
  v = fmaxf(v, dpp_f32<0xB1>(v));
  v = fmaxf(v, dpp_f32<0x4E>(v));
  v = fmaxf(v, dpp_f32<0x141>(v));
  return v;
}

// order-preserving key of a float: larger float <=> larger unsigned key; -0.0 maps onto +0.0
__device__ __forceinline__ uint32_t float_key(float v) {
  uint32_t u = __float_as_uint(v);
  if (u == 0x80000000u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// inverse of float_key
__device__ __forceinline__ float key_float(uint32_t k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

// exp(x) for x <= 0 (larger x also fine up to ~700); result below 1e-300 flushes to 0
__device__ __forceinline__ double exp_f64(double x) {
  const bool tiny = x < -690.0;
  x = tiny ? -690.0 : x;
  const double n = rint(x * 1.44269504088896340736);
  double r = fma(n, -6.93147180369123816490e-01, x);
  r = fma(n, -1.90821492927058770002e-10, r);
  // Taylor series on |r| <= 0.347, degree 11: truncation below 3e-14 relative
  double p = 1.0 / 39916800.0;
  p = fma(p, r, 1.0 / 3628800.0);
  p = fma(p, r, 1.0 / 362880.0);
  p = fma(p, r, 1.0 / 40320.0);
  p = fma(p, r, 1.0 / 5040.0);
  p = fma(p, r, 1.0 / 720.0);
  p = fma(p, r, 1.0 / 120.0);
  p = fma(p, r, 1.0 / 24.0);
  p = fma(p, r, 1.0 / 6.0);
  p = fma(p, r, 0.5);
  p = fma(p, r, 1.0);
  p = fma(p, r, 1.0);
  const long long bits = ((long long)n + 1023LL) << 52;   // 2^n, n >= -996 here
  return tiny ? 0.0 : p * __longlong_as_double(bits);
}

#endif  // __HIPCC__

}  // namespace ts
