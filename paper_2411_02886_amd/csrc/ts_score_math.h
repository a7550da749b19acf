// Element types and the dot-product arithmetic of the decode score pass, shared by the kernels that must
// produce bit-identical scores (the streaming pass and the exact re-evaluation of top-k candidates).
#pragma once
#include "ts_common.h"

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

}  // namespace ts
