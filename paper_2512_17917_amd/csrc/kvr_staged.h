// Device helpers shared by the LDS-staged attention kernels over the Vague list.
#pragma once
#include "kvr_launch.h"

namespace kvr {

constexpr int ST_THREADS = 512;
constexpr int ST_WAVES = 8;
constexpr int ST_KMAX = 6;

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

// Per-channel median of three on packed bf16, taken on the raw bit patterns with
// v_med3_f16 (bf16 and f16 are both sign-magnitude with the exponent above the
// mantissa, so finite values order the same way; zeros of either sign compare
// equal).  The low and the high halves are two instructions: the first writes the
// low 16 bits of the destination, the second (op_sel) the high 16 bits and leaves
// the low half as it is.
//
// These are inline assembly, and the compiler's hazard bookkeeping does not see
// the register writes of inline assembly as vector-ALU writes: it would place a
// matrix instruction that reads the result directly behind it, which needs two
// wait states after a vector-ALU write on this target.  The wait states are
// therefore part of the primitive (s_nop 1 = two wait states behind the write
// that completes the dword), and the result may be consumed by any instruction
// right away: nothing depends on how the surrounding code is scheduled.  (Forms
// with one s_nop per 16-byte piece were measured: they tie up more registers at
// once, which costs the widest kernel more than the three s_nop they save.)
__device__ __forceinline__ uint32_t med3_dword(uint32_t a, uint32_t b, uint32_t c) {
  uint32_t dst;
  asm("v_med3_f16 %0, %1, %2, %3" : "=v"(dst) : "v"(a), "v"(b), "v"(c));
  asm("v_med3_f16 %0, %1, %2, %3 op_sel:[1,1,1,1]\n\ts_nop 1" : "+v"(dst) : "v"(a), "v"(b), "v"(c));
  return dst;
}
// 8 bytes (4 channels)
__device__ __forceinline__ uint2 med3_half_piece(uint2 a, uint2 b, uint2 c) {
  return make_uint2(med3_dword(a.x, b.x, c.x), med3_dword(a.y, b.y, c.y));
}
// 16 bytes (8 channels)
__device__ __forceinline__ uint4 med3_piece(uint4 a, uint4 b, uint4 c) {
  return make_uint4(med3_dword(a.x, b.x, c.x), med3_dword(a.y, b.y, c.y), med3_dword(a.z, b.z, c.z),
                    med3_dword(a.w, b.w, c.w));
}

__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), c,
                                         false);
}

__device__ __forceinline__ float bf_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
// two floats that are exactly representable in bf16 -> packed pair
__device__ __forceinline__ uint32_t pack_bf16_exact(float lo, float hi) {
  return (__float_as_uint(hi) & 0xffff0000u) | (__float_as_uint(lo) >> 16);
}

// (low half of a, low half of b) and (high half of a, high half of b) as one dword
__device__ __forceinline__ uint32_t pair_lo(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x05040100u); }
__device__ __forceinline__ uint32_t pair_hi(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x07060302u); }

// Packed minimum / maximum of two bf16 pairs on their raw bits (same argument as
// for v_med3_f16: the order of finite values is the same in both formats).
// Inline assembly again: results of these two may only feed ordinary vector-ALU
// instructions (which need no wait states); pk_min_bits_last carries the wait
// states for any consumer.
__device__ __forceinline__ uint32_t pk_min_bits(uint32_t a, uint32_t b) {
  uint32_t dst;
  asm("v_pk_min_f16 %0, %1, %2" : "=v"(dst) : "v"(a), "v"(b));
  return dst;
}
__device__ __forceinline__ uint32_t pk_max_bits(uint32_t a, uint32_t b) {
  uint32_t dst;
  asm("v_pk_max_f16 %0, %1, %2" : "=v"(dst) : "v"(a), "v"(b));
  return dst;
}
__device__ __forceinline__ uint32_t pk_min_bits_last(uint32_t a, uint32_t b) {
  uint32_t dst;
  asm("v_pk_min_f16 %0, %1, %2\n\ts_nop 1" : "=v"(dst) : "v"(a), "v"(b));
  return dst;
}
// two float32 -> packed bf16, round to nearest even (v_cvt_pk_bf16_f32, emitted by the compiler itself)
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t cvt_pk_bf16(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// Median over R rows of one dword (two packed bf16 channels), R != 3.
template <int R>
__device__ __forceinline__ uint32_t median_dword(const uint32_t (&x)[R], int mode) {
  static_assert(R != 3, "three rows go through med3_piece");
  if constexpr (R == 4) {
    // the two middle values of four: max of the pair minima, min of the pair maxima
    const uint32_t m1 = pk_max_bits(pk_min_bits(x[0], x[1]), pk_min_bits(x[2], x[3]));
    const uint32_t m2 = pk_min_bits(pk_max_bits(x[0], x[1]), pk_max_bits(x[2], x[3]));
    if (mode == KVR_MEDIAN_LOWER) return pk_min_bits_last(m1, m2);
    // Their mean in float32, rounded once to bf16.  0.5 m1 + 0.5 m2 per channel is one v_dot2_f32_bf16 on
    // the pair (m1, m2) against (0.5, 0.5): both products are exact, so the result is the float32 sum of two
    // exactly known terms, the same value as 0.5f * (m1 + m2) formed with separate instructions (the halving
    // only changes the exponent), in 5 instructions per dword instead of 9.
    const uint32_t halves = 0x3f003f00u;
    return cvt_pk_bf16(dot2_bf16(pair_lo(m1, m2), halves, 0.f), dot2_bf16(pair_hi(m1, m2), halves, 0.f));
  } else {
    float lo[R], hi[R];
#pragma unroll
    for (int i = 0; i < R; ++i) { lo[i] = bf_lo(x[i]); hi[i] = bf_hi(x[i]); }
    return pack_bf16_exact(median_rows<R, bf16_t>(lo, R, mode), median_rows<R, bf16_t>(hi, R, mode));
  }
}

// Median over R rows of a 16-byte piece (8 packed bf16 channels).
template <int R>
__device__ __forceinline__ uint4 median_piece(const uint4 (&row)[R], int mode) {
  if constexpr (R == 3) {
    return med3_piece(row[0], row[1], row[2]);
  } else {
    uint32_t x[R], y[R], z[R], w_[R];
#pragma unroll
    for (int i = 0; i < R; ++i) { x[i] = row[i].x; y[i] = row[i].y; z[i] = row[i].z; w_[i] = row[i].w; }
    return make_uint4(median_dword<R>(x, mode), median_dword<R>(y, mode), median_dword<R>(z, mode),
                      median_dword<R>(w_, mode));
  }
}

__device__ __forceinline__ uint4 xor4(uint4 v, uint32_t mask) {
  return make_uint4(v.x ^ mask, v.y ^ mask, v.z ^ mask, v.w ^ mask);
}

typedef short short4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ short4_t pack_k4(uint32_t k01, uint32_t k23) {
  return __builtin_bit_cast(short4_t, make_uint2(k01, k23));
}
template <int DW>
__device__ __forceinline__ uint32_t dword_of(const uint4& v) {
  return DW == 0 ? v.x : DW == 1 ? v.y : DW == 2 ? v.z : v.w;
}

// One dword position (two channels) of a piece, for the 4 tokens of a block:
// acc[2 DW] and acc[2 DW + 1] (4 head sums each) += weights x values.
template <int DW>
__device__ __forceinline__ void pv_mfma(const uint4 (&med)[4], short4_t a_hi, short4_t a_lo, f32x4_t (&acc)[8]) {
  const uint32_t t0 = dword_of<DW>(med[0]), t1 = dword_of<DW>(med[1]);
  const uint32_t t2 = dword_of<DW>(med[2]), t3 = dword_of<DW>(med[3]);
  const short4_t b_even = pack_k4(pair_lo(t0, t1), pair_lo(t2, t3));
  const short4_t b_odd = pack_k4(pair_hi(t0, t1), pair_hi(t2, t3));
  acc[2 * DW] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(a_hi, b_even, acc[2 * DW], 0, 0, 0);
  acc[2 * DW] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(a_lo, b_even, acc[2 * DW], 0, 0, 0);
  acc[2 * DW + 1] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(a_hi, b_odd, acc[2 * DW + 1], 0, 0, 0);
  acc[2 * DW + 1] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(a_lo, b_odd, acc[2 * DW + 1], 0, 0, 0);
}

// Workgroup barrier for data exchanged through LDS only: waits for this wave's
// LDS traffic, not for its outstanding global stores (which __syncthreads would).
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

template <int CTRL>
__device__ __forceinline__ float dpp_add(float x) {
  return x + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true));
}
// Sum over the lanes of a 16-lane row whose lane numbers are equal modulo LPT
// (row rotations by LPT, 2 LPT, ..., 8); every lane ends up with its class's sum.
template <int LPT>
__device__ __forceinline__ float row_sum(float x) {
  if constexpr (LPT <= 1) x = dpp_add<0x121>(x);
  if constexpr (LPT <= 2) x = dpp_add<0x122>(x);
  if constexpr (LPT <= 4) x = dpp_add<0x124>(x);
  return dpp_add<0x128>(x);
}

template <int CTRL>
__device__ __forceinline__ float dpp_max(float x) {
  return fmaxf(x, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true)));
}
// maximum over the 16 lanes of a row, in every lane
__device__ __forceinline__ float row_max(float x) {
  x = dpp_max<0x121>(x);
  x = dpp_max<0x122>(x);
  x = dpp_max<0x124>(x);
  return dpp_max<0x128>(x);
}

// token info: 4 x 16 bits; bits 0..14 = LDS row index (i * w + h_i(J)), bit 15 = 1 iff g_i(J) = -1
template <int I>
__device__ __forceinline__ uint32_t info_row(uint2 inf) {
  const uint32_t wd = (I < 2) ? inf.x : inf.y;
  return (I & 1) ? __builtin_amdgcn_ubfe(wd, 16, 15) : (wd & 0x7fffu);
}
template <int I>
__device__ __forceinline__ uint32_t info_neg(uint2 inf) {
  const uint32_t wd = (I < 2) ? inf.x : inf.y;
  return __builtin_amdgcn_ubfe(wd, (I & 1) * 16 + 15, 1);
}
// 0x80008000 if the signs of rows I and 0 differ, else 0
template <int I>
__device__ __forceinline__ uint32_t info_flipmask(uint2 inf) {
  const uint32_t wd = (I < 2) ? inf.x : inf.y;
  const uint32_t x = wd ^ (inf.x << ((I & 1) * 16));      // bit (I&1)*16+15 = sign_I ^ sign_0
  return (uint32_t)__builtin_amdgcn_sbfe(x, (I & 1) * 16 + 15, 1) & 0x80008000u;
}

template <int R>
__device__ __forceinline__ void row_offsets(uint2 inf, int (&rb)[R], int rowb_log2) {
  rb[0] = (int)(info_row<0>(inf) << rowb_log2);
  if constexpr (R > 1) rb[1] = (int)(info_row<1>(inf) << rowb_log2);
  if constexpr (R > 2) rb[2] = (int)(info_row<2>(inf) << rowb_log2);
  if constexpr (R > 3) rb[3] = (int)(info_row<3>(inf) << rowb_log2);
}

// Copy channel chunk `cc` of a sketch tensor [rows][128] (bf16, global) into LDS
// rows of ROWB bytes with global->LDS loads that bypass the registers
// (global_load_lds_dwordx4: lane i's 16 bytes land at the wave's LDS base +
// 16 i).  Piece p of the chunk lives at LDS offset 16 p, so a wave that takes 64
// consecutive pieces fills 1 KB of consecutive LDS.  All copies of a wave are
// in flight together; the caller's barrier must follow the vmcnt wait done here.
// Tail lanes re-read the last piece into the padding behind the chunk (the
// buffer is sized to a multiple of 1 KB).
template <int NC, int ROWB>
__device__ __forceinline__ void stage_chunk(const unsigned char* __restrict__ g, unsigned char* s_sk,
                                            int n_pieces, int cc, int tid) {
  const int lane = tid & 63, wave = tid >> 6;
  for (int p0 = wave * 64; p0 < n_pieces; p0 += ST_THREADS) {
    const int idx = min(p0 + lane, n_pieces - 1);
    const int row = idx / NC, c = idx % NC;
    __builtin_amdgcn_global_load_lds(
        (const __attribute__((address_space(1))) void*)(g + (size_t)row * (D * 2) + cc * ROWB + c * 16),
        (__attribute__((address_space(3))) void*)(s_sk + p0 * 16), 16, 0, 0);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}


// Issue half of stage_chunk: start the copies and return; stage_wait() before
// the barrier that publishes the chunk.
template <int NC, int ROWB>
__device__ __forceinline__ void stage_issue(const unsigned char* __restrict__ g, unsigned char* s_sk,
                                            int n_pieces, int cc, int tid) {
  const int lane = tid & 63, wave = tid >> 6;
  for (int p0 = wave * 64; p0 < n_pieces; p0 += ST_THREADS) {
    const int idx = min(p0 + lane, n_pieces - 1);
    const int row = idx / NC, c = idx % NC;
    __builtin_amdgcn_global_load_lds(
        (const __attribute__((address_space(1))) void*)(g + (size_t)row * (D * 2) + cc * ROWB + c * 16),
        (__attribute__((address_space(3))) void*)(s_sk + p0 * 16), 16, 0, 0);
  }
}
__device__ __forceinline__ void stage_wait() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

}  // namespace kvr
