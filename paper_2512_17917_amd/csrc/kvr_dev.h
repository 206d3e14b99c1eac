// Device-side building blocks shared by the kvr kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/kvr.h"

namespace kvr {

constexpr int D = KVR_HEAD_DIM;   // channels per head
constexpr int WAVE = 64;

// Problem constants handed to every kernel by value.
struct DevDesc {
  int B, Hq, Hkv, G;
  int r, w;
  int sign_mask, median_mode;
  float scale;
  uint64_t hp[KVR_MAX_ROWS][4];   // a, b, c, d per row
};

// ---- storage types -------------------------------------------------------
struct bf16_t { uint16_t bits; };

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b16) { return __uint_as_float(b16 << 16); }

// round-to-nearest-even float32 -> bf16 bit pattern (NaN -> quiet NaN)
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float x) {
  uint32_t b = __float_as_uint(x);
  if ((b & 0x7fffffffu) > 0x7f800000u) return 0x7fc0u;
  return (b + 0x7fffu + ((b >> 16) & 1u)) >> 16;
}

template <typename T> struct Store;
template <> struct Store<float> {
  static constexpr int VEC = 4;                    // channels per 16-byte load
  __device__ static __forceinline__ void load16(const float* p, float (&o)[4]) {
    float4 v = *reinterpret_cast<const float4*>(p);
    o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
  }
  __device__ static __forceinline__ void store16(float* p, const float (&o)[4]) {
    *reinterpret_cast<float4*>(p) = make_float4(o[0], o[1], o[2], o[3]);
  }
  __device__ static __forceinline__ float round(float x) { return x; }
  __device__ static __forceinline__ float load1(const float* p) { return *p; }
  __device__ static __forceinline__ void store1(float* p, float x) { *p = x; }
};
template <> struct Store<bf16_t> {
  static constexpr int VEC = 8;
  __device__ static __forceinline__ void load16(const bf16_t* p, float (&o)[8]) {
    uint4 v = *reinterpret_cast<const uint4*>(p);
    o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xffff0000u);
    o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xffff0000u);
    o[4] = __uint_as_float(v.z << 16); o[5] = __uint_as_float(v.z & 0xffff0000u);
    o[6] = __uint_as_float(v.w << 16); o[7] = __uint_as_float(v.w & 0xffff0000u);
  }
  __device__ static __forceinline__ void store16(bf16_t* p, const float (&o)[8]) {
    uint4 v;
    v.x = f32_to_bf16_bits(o[0]) | (f32_to_bf16_bits(o[1]) << 16);
    v.y = f32_to_bf16_bits(o[2]) | (f32_to_bf16_bits(o[3]) << 16);
    v.z = f32_to_bf16_bits(o[4]) | (f32_to_bf16_bits(o[5]) << 16);
    v.w = f32_to_bf16_bits(o[6]) | (f32_to_bf16_bits(o[7]) << 16);
    *reinterpret_cast<uint4*>(p) = v;
  }
  __device__ static __forceinline__ float round(float x) { return bf16_bits_to_f32(f32_to_bf16_bits(x)); }
  __device__ static __forceinline__ float load1(const bf16_t* p) { return bf16_bits_to_f32(p->bits); }
  __device__ static __forceinline__ void store1(bf16_t* p, float x) { p->bits = (uint16_t)f32_to_bf16_bits(x); }
};

// ---- hash and sign of a token position -------------------------------------
// h_i(J) = (((a*J + b) mod 2^64) >> 32) * w >> 32 ;  g_i(J) < 0 iff top bit of c*J + d
__device__ __forceinline__ int bucket_of(const DevDesc& d, int i, int J) {
  uint64_t u = d.hp[i][0] * (uint64_t)(uint32_t)J + d.hp[i][1];
  return (int)__umulhi((uint32_t)(u >> 32), (uint32_t)d.w);
}
__device__ __forceinline__ bool sign_neg(const DevDesc& d, int i, int J) {
  uint64_t s = d.hp[i][2] * (uint64_t)(uint32_t)J + d.hp[i][3];
  return (s >> 63) != 0;
}

// ---- element-wise median over the sketch rows -------------------------------
__device__ __forceinline__ void cswap(float& a, float& b) {
  float lo = fminf(a, b), hi = fmaxf(a, b);
  a = lo; b = hi;
}

// R > 0: compile-time row count.  R == 0: run-time count r in 1..8.
template <int R, typename T>
__device__ __forceinline__ float median_rows(float (&v)[R == 0 ? KVR_MAX_ROWS : R], int r, int mode) {
  if constexpr (R == 1) {
    return v[0];
  } else if constexpr (R == 2) {
    float lo = fminf(v[0], v[1]), hi = fmaxf(v[0], v[1]);
    return mode == KVR_MEDIAN_LOWER ? lo : Store<T>::round(0.5f * (lo + hi));
  } else if constexpr (R == 3) {
    return __builtin_amdgcn_fmed3f(v[0], v[1], v[2]);
  } else if constexpr (R == 4) {
    float mn1 = fminf(v[0], v[1]), mx1 = fmaxf(v[0], v[1]);
    float mn2 = fminf(v[2], v[3]), mx2 = fmaxf(v[2], v[3]);
    float m1 = fmaxf(mn1, mn2), m2 = fminf(mx1, mx2);
    float lo = fminf(m1, m2), hi = fmaxf(m1, m2);
    return mode == KVR_MEDIAN_LOWER ? lo : Store<T>::round(0.5f * (lo + hi));
  } else {
    // pad to 8 with +inf, sort with a 19-exchange network, pick by index
    float s[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) s[i] = (i < r) ? v[i] : __builtin_inff();
    cswap(s[0], s[1]); cswap(s[2], s[3]); cswap(s[4], s[5]); cswap(s[6], s[7]);
    cswap(s[0], s[2]); cswap(s[1], s[3]); cswap(s[4], s[6]); cswap(s[5], s[7]);
    cswap(s[1], s[2]); cswap(s[5], s[6]); cswap(s[0], s[4]); cswap(s[3], s[7]);
    cswap(s[1], s[5]); cswap(s[2], s[6]);
    cswap(s[1], s[4]); cswap(s[3], s[6]);
    cswap(s[2], s[4]); cswap(s[3], s[5]);
    cswap(s[3], s[4]);
    int il = (r - 1) >> 1, ih = r >> 1;
    float lo = s[0], hi = s[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) { lo = (i == il) ? s[i] : lo; hi = (i == ih) ? s[i] : hi; }
    if (il == ih) return lo;
    return mode == KVR_MEDIAN_LOWER ? lo : Store<T>::round(0.5f * (lo + hi));
  }
}

// Gather the r sketch rows of token J (one 16-byte chunk starting at channel c0)
// and reduce them to the per-channel median.  `sk` points at the unit's sketch
// [r, w, D]; `flip` says whether this tensor is signed.
template <typename T, int R>
__device__ __forceinline__ void query_chunk(const DevDesc& d, const T* __restrict__ sk, int J, int c0,
                                            bool flip, float (&out)[Store<T>::VEC]) {
  constexpr int VEC = Store<T>::VEC;
  constexpr int RR = (R == 0) ? KVR_MAX_ROWS : R;
  float rows[RR][VEC];
  const int r = (R == 0) ? d.r : R;
#pragma unroll
  for (int i = 0; i < RR; ++i) {
    if (i < r) {
      int h = bucket_of(d, i, J);
      Store<T>::load16(sk + ((size_t)i * d.w + h) * D + c0, rows[i]);
      if (flip && sign_neg(d, i, J)) {
#pragma unroll
        for (int c = 0; c < VEC; ++c) rows[i][c] = -rows[i][c];
      }
    } else {
#pragma unroll
      for (int c = 0; c < VEC; ++c) rows[i][c] = 0.f;
    }
  }
#pragma unroll
  for (int c = 0; c < VEC; ++c) {
    float col[RR];
#pragma unroll
    for (int i = 0; i < RR; ++i) col[i] = rows[i][c];
    out[c] = median_rows<R, T>(col, r, d.median_mode);
  }
}

// bf16 storage, three rows: the median of three is one of its inputs, so nothing
// has to be rounded; rows are flipped on their packed bits, widened to float32
// for the comparison (exact) and the winner's upper half is stored.
__device__ __forceinline__ uint32_t med3_pair_bf16(uint32_t a, uint32_t b, uint32_t c) {
  const float lo = __builtin_amdgcn_fmed3f(__uint_as_float(a << 16), __uint_as_float(b << 16), __uint_as_float(c << 16));
  const float hi = __builtin_amdgcn_fmed3f(__uint_as_float(a & 0xffff0000u), __uint_as_float(b & 0xffff0000u),
                                           __uint_as_float(c & 0xffff0000u));
  return __builtin_amdgcn_perm(__float_as_uint(hi), __float_as_uint(lo), 0x07060302u);
}

__device__ __forceinline__ uint4 query_piece3(const DevDesc& d, const bf16_t* __restrict__ sx, const int (&h)[3],
                                              const uint32_t (&flip)[3], int c0) {
  uint4 r[3];
#pragma unroll
  for (int i = 0; i < 3; ++i) {
    r[i] = *reinterpret_cast<const uint4*>(sx + ((size_t)i * d.w + h[i]) * D + c0);
    r[i].x ^= flip[i]; r[i].y ^= flip[i]; r[i].z ^= flip[i]; r[i].w ^= flip[i];
  }
  return make_uint4(med3_pair_bf16(r[0].x, r[1].x, r[2].x), med3_pair_bf16(r[0].y, r[1].y, r[2].y),
                    med3_pair_bf16(r[0].z, r[1].z, r[2].z), med3_pair_bf16(r[0].w, r[1].w, r[2].w));
}

__device__ __forceinline__ int clampi(int x, int lo, int hi) { return x < lo ? lo : (x > hi ? hi : x); }

}  // namespace kvr
