// Staged attention kernel for the Vague index list (bf16 storage, values signed
// only, G <= 4 query heads per kv head, r = 3 or 4 sketch rows).
//
// Rebuilding a Vague token needs r rows of the K sketch and r rows of the V
// sketch (Algorithm 2); with tens of thousands of Vague tokens per unit the
// gather volume is far beyond what L2 can serve, so the sketch is staged through
// LDS.  One kv head's sketch does not fit (r*w*256 B per tensor), so it is cut
// into channel chunks of CH channels: for each chunk of the K sketch the
// workgroup adds that chunk's share of q.k for all of its tokens (logits stay in
// registers), then softmax weights are formed against the workgroup's own
// maximum, then for each chunk of the V sketch it accumulates p * v for the
// chunk's channels.  The merge kernel rescales the partials as for any slice.
//
// Token -> lane mapping.  A workgroup has 8 waves; wave gw (global over the
// unit's workgroups) owns the 64-token rounds gw, gw + NWT, gw + 2 NWT, ...
//   K phases: one lane = one token; the lane walks the CH/8 16-byte pieces of
//     each of its r rows starting at piece (lane mod CH/8), so that at any
//     moment 8 neighbouring lanes read 8 different 16-byte bank groups; q is
//     kept in registers in the same rotated order.  No cross-lane reduction.
//   V phases: CH/16 lanes share one token (two pieces = 16 channels each) and
//     accumulate p * v in registers across all of the wave's tokens; the
//     token's weights come from their owner lane by a lane permute.  Lanes of
//     odd token groups take their two pieces in the opposite order, so that 8
//     neighbouring lanes (two tokens) again cover 8 different bank groups.
// Per-channel median of three on packed bf16: v_med3_f16 on the raw bit
// patterns (both formats are sign-magnitude with the exponent above the
// mantissa, so the order of finite values is the same; zeros of either sign
// compare equal).  The sign g_0 of row 0 is moved onto the weight, so only
// rows 1.. need their sign bits flipped (the median is an odd function).
#include "kvr_launch.h"

namespace kvr {

constexpr int ST_THREADS = 512;
constexpr int ST_WAVES = 8;
constexpr int ST_KMAX = 6;

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

// Development aid, compiled out unless KVR_PHASE_TIMING is defined: thread 0 of
// every workgroup stamps the cycle counter at phase boundaries.
#ifdef KVR_PHASE_TIMING
__device__ unsigned long long g_phase_t[8192 * 16];
#define KVR_STAMP(i)                                                              \
  do {                                                                            \
    if (threadIdx.x == 0 && blockIdx.x < 8192) g_phase_t[blockIdx.x * 16 + (i)] = clock64(); \
  } while (0)
#else
#define KVR_STAMP(i) \
  do {               \
  } while (0)
#endif

__device__ __forceinline__ uint32_t med3_bf16x2(uint32_t a, uint32_t b, uint32_t c) {
  uint32_t dst;
  asm("v_med3_f16 %0, %1, %2, %3" : "=v"(dst) : "v"(a), "v"(b), "v"(c));
  asm("v_med3_f16 %0, %1, %2, %3 op_sel:[1,1,1,1]" : "+v"(dst) : "v"(a), "v"(b), "v"(c));
  return dst;
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

template <int R>
__device__ __forceinline__ uint32_t median_dword(const uint32_t (&x)[R], int mode) {
  if constexpr (R == 3) {
    return med3_bf16x2(x[0], x[1], x[2]);
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
  uint32_t x[R], y[R], z[R], w_[R];
#pragma unroll
  for (int i = 0; i < R; ++i) { x[i] = row[i].x; y[i] = row[i].y; z[i] = row[i].z; w_[i] = row[i].w; }
  return make_uint4(median_dword<R>(x, mode), median_dword<R>(y, mode), median_dword<R>(z, mode),
                    median_dword<R>(w_, mode));
}

__device__ __forceinline__ uint4 xor4(uint4 v, uint32_t mask) {
  return make_uint4(v.x ^ mask, v.y ^ mask, v.z ^ mask, v.w ^ mask);
}

typedef short short4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

// (low half of a, low half of b) and (high half of a, high half of b) as one dword
__device__ __forceinline__ uint32_t pair_lo(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x05040100u); }
__device__ __forceinline__ uint32_t pair_hi(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x07060302u); }
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
  return x + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, false));
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
  return fmaxf(x, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, false)));
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

template <int G, int R, int CH>
__global__ __launch_bounds__(ST_THREADS) void attend_vague_staged_kernel(DevDesc d, AttendArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  constexpr int NC = CH / 8;                 // 16-byte pieces per LDS row
  constexpr int NPH = D / CH;                // phases per tensor
  constexpr int ROWB = CH * 2;               // bytes per LDS row
  constexpr int ROWB_LOG2 = (CH == 64) ? 7 : (CH == 32) ? 6 : (CH == 16) ? 5 : 4;
  constexpr int PPL = (NC >= 2) ? 2 : 1;     // V phase: pieces per lane
  constexpr int LPT = NC / PPL;              // V phase: lanes per token
  constexpr int TPW = WAVE / LPT;            // V phase: tokens per wave-iteration
  constexpr int VCH = PPL * 8;               // V phase: channels per lane

  // XCD-aware mapping: workgroup ids are dealt round-robin to the 8 XCDs, so all
  // workgroups of a unit get ids that are equal modulo 8 (they share one L2).
  const int lin = blockIdx.x;
  const int xcd = lin & 7, jj = lin >> 3;
  const int unit = (jj / a.n_vslices) * 8 + xcd;
  const int vs = jj % a.n_vslices;
  const int units = d.B * d.Hkv;
  if (unit >= units) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = unit / d.Hkv, hk = unit % d.Hkv;
  const int w = d.w;
  // chunk buffer; it doubles as reduction scratch [32 rows][G][CH] floats
  const int sk_bytes = max((R * w * ROWB + 1023) & ~1023, 32 * G * CH * 4);
  unsigned char* s_sk = smem;
  uint2* s_info = reinterpret_cast<uint2*>(smem + sk_bytes);
  float* s_red = reinterpret_cast<float*>(smem + sk_bytes + ST_KMAX * ST_THREADS * 8);   // [8][G][CH]
  float* s_stat = s_red + ST_WAVES * G * 64;                                               // [8][G] x 2
  uint4* s_q = reinterpret_cast<uint4*>(smem + sk_bytes + ST_KMAX * ST_THREADS * 8 + ST_WAVES * G * 64 * 4 + 1024);

  const int nv = clampi(a.n_vague[unit], 0, a.vague_cap);
  const int rounds_total = (nv + 63) >> 6;
  const int NWT = a.n_vslices * ST_WAVES;
  const int gw = vs * ST_WAVES + wave;
  int n_k = gw < rounds_total ? (rounds_total - gw + NWT - 1) / NWT : 0;
  if (n_k > ST_KMAX) n_k = ST_KMAX;       // cannot happen when the plan was made for vague_cap

  // ---- touch this workgroup's share of the unit's two sketches so that the
  //      lines are on their way into L2 while the hashes are computed ----------
  uint32_t touched = 0;
  {
    const int n_lines = 2 * R * w;                     // 128-byte lines per tensor
    const int per_wg = (2 * n_lines + a.n_vslices - 1) / a.n_vslices;
    const int li = vs * per_wg + tid;
    if (tid < per_wg && li < 2 * n_lines) {
      const bf16_t* base = (li < n_lines) ? (const bf16_t*)a.sk : (const bf16_t*)a.sv;
      const int l2 = (li < n_lines) ? li : li - n_lines;
      touched = *reinterpret_cast<const uint32_t*>(base + (size_t)unit * R * w * D + (size_t)l2 * 64);
    }
  }

  // ---- hash every token once; q to LDS ---------------------------------------
  KVR_STAMP(0);
  uint2 info[ST_KMAX];
  uint32_t vmask = 0;
  const int32_t* vpos = a.vague_pos + (size_t)unit * a.vague_cap;
#pragma unroll
  for (int k = 0; k < ST_KMAX; ++k) {
    const int tok = (gw + k * NWT) * 64 + lane;
    uint2 pk = make_uint2(0u, 0u);
    if (k < n_k && tok < nv) {
      const int J = vpos[tok];
      uint32_t f[4] = {0u, 0u, 0u, 0u};
#pragma unroll
      for (int i = 0; i < R; ++i)
        f[i] = (uint32_t)(i * w + bucket_of(d, i, J)) | (sign_neg(d, i, J) ? 0x8000u : 0u);
      pk = make_uint2(f[0] | (f[1] << 16), f[2] | (f[3] << 16));
      vmask |= 1u << k;
    }
    info[k] = pk;
    s_info[(k * ST_WAVES + wave) * 64 + lane] = pk;
  }
  if (touched == 0x7fc1u && nv < 0) vmask = 0;       // never true; keeps the touch load alive
  if (tid < G * 16) {
    const uint4* qg = reinterpret_cast<const uint4*>((const bf16_t*)a.q + ((size_t)b * d.Hq + (size_t)hk * G) * D);
    s_q[tid] = qg[tid];
  }

  const size_t sk_unit = (size_t)unit * R * w * D;      // elements
  const unsigned char* skg = reinterpret_cast<const unsigned char*>((const bf16_t*)a.sk + sk_unit);
  const unsigned char* svg = reinterpret_cast<const unsigned char*>((const bf16_t*)a.sv + sk_unit);
  const int n_pieces = R * w * NC;

  // ---- K phases: logits -----------------------------------------------------
  KVR_STAMP(1);
  float s[ST_KMAX][G];
#pragma unroll
  for (int k = 0; k < ST_KMAX; ++k)
#pragma unroll
    for (int g = 0; g < G; ++g) s[k][g] = 0.f;

  for (int cc = 0; cc < NPH; ++cc) {
    lds_barrier();
    stage_chunk<NC, ROWB>(skg, s_sk, n_pieces, cc, tid);
    lds_barrier();
    KVR_STAMP(2 + 2 * cc);
    // the pieces of a row are taken in two halves so that only half of q (in
    // this lane's rotated order) has to sit in registers at a time
    constexpr int JH = (NC >= 8) ? NC / 2 : NC;
#pragma unroll
    for (int j0 = 0; j0 < NC; j0 += JH) {
      uint4 qreg[JH][G];
#pragma unroll
      for (int j = 0; j < JH; ++j)
#pragma unroll
        for (int g = 0; g < G; ++g) qreg[j][g] = s_q[g * 16 + cc * NC + ((lane + j0 + j) & (NC - 1))];
#pragma unroll
      for (int k = 0; k < ST_KMAX; ++k) {
        if (k < n_k) {
          int rb[R];
          row_offsets<R>(info[k], rb, ROWB_LOG2);
#pragma unroll
          for (int j = 0; j < JH; ++j) {
            const int co = ((lane + j0 + j) & (NC - 1)) * 16;
            uint4 row[R];
#pragma unroll
            for (int i = 0; i < R; ++i) row[i] = *reinterpret_cast<const uint4*>(s_sk + rb[i] + co);
            const uint4 m = median_piece<R>(row, d.median_mode);
#pragma unroll
            for (int g = 0; g < G; ++g) {
              float x = s[k][g];
              x = dot2_bf16(m.x, qreg[j][g].x, x);
              x = dot2_bf16(m.y, qreg[j][g].y, x);
              x = dot2_bf16(m.z, qreg[j][g].z, x);
              x = dot2_bf16(m.w, qreg[j][g].w, x);
              s[k][g] = x;
            }
          }
        }
      }
    }
    KVR_STAMP(3 + 2 * cc);
  }

  // ---- softmax weights against the workgroup's own maximum -------------------
  const int tot_cap = a.ret_cap + a.vague_cap;
  float mx[G];
#pragma unroll
  for (int g = 0; g < G; ++g) mx[g] = -__builtin_inff();
#pragma unroll
  for (int k = 0; k < ST_KMAX; ++k) {
    const bool valid = (vmask >> k) & 1u;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      s[k][g] = valid ? s[k][g] * d.scale : -__builtin_inff();
      mx[g] = fmaxf(mx[g], s[k][g]);
    }
    if (a.logits != nullptr && valid) {
      const int tok = (gw + k * NWT) * 64 + lane;
      float* lg = a.logits + ((size_t)unit * tot_cap + a.ret_cap + tok) * G;
      if constexpr (G == 4) {
        *reinterpret_cast<float4*>(lg) = make_float4(s[k][0], s[k][1], s[k][2], s[k][3]);
      } else {
#pragma unroll
        for (int g = 0; g < G; ++g) lg[g] = s[k][g];
      }
    }
  }
  // maxima and sums: DPP inside each 16-lane row, then the 32 rows of the
  // workgroup meet in LDS (s_stat: [32][G] maxima, [32][G] sums)
  constexpr int NROW = ST_WAVES * 4;
  const int prow = wave * 4 + (lane >> 4);
#pragma unroll
  for (int g = 0; g < G; ++g) {
    mx[g] = row_max(mx[g]);
    if ((lane & 15) == 0) s_stat[prow * G + g] = mx[g];
  }
  lds_barrier();
  float lsum[G];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float M = s_stat[g];
#pragma unroll
    for (int pr = 1; pr < NROW; ++pr) M = fmaxf(M, s_stat[pr * G + g]);
    lsum[g] = 0.f;
#pragma unroll
    for (int k = 0; k < ST_KMAX; ++k) {
      const float p = (s[k][g] == -__builtin_inff()) ? 0.f : __expf(s[k][g] - M);
      s[k][g] = p;                 // from here on s holds the weights
      lsum[g] += p;
    }
  }
#pragma unroll
  for (int g = 0; g < G; ++g) {
    lsum[g] = row_sum<1>(lsum[g]);
    if ((lane & 15) == 0) s_stat[NROW * G + prow * G + g] = lsum[g];
  }
  lds_barrier();
  const size_t part = (size_t)unit * a.n_slices + a.n_rslices + vs;
  if (tid < G) {
    float L = 0.f, Mg = s_stat[tid];
#pragma unroll
    for (int pr = 0; pr < NROW; ++pr) {
      L += s_stat[NROW * G + pr * G + tid];
      Mg = fmaxf(Mg, s_stat[pr * G + tid]);
    }
    a.part_ml[(part * G + tid) * 2] = Mg;
    a.part_ml[(part * G + tid) * 2 + 1] = L;
  }

  // ---- V phases: weighted values ------------------------------------------------
  KVR_STAMP(6);
  const int sub = lane % LPT, tl = lane / LPT;
  // the two pieces of this lane: odd token groups take them in the opposite order
  const int pa = (PPL == 2) ? sub + ((tl & 1) ? LPT : 0) : sub;
  const int pb = (PPL == 2) ? sub + ((tl & 1) ? 0 : LPT) : sub;
  for (int cc = 0; cc < NPH; ++cc) {
    lds_barrier();
    stage_chunk<NC, ROWB>(svg, s_sk, n_pieces, cc, tid);
    lds_barrier();
    KVR_STAMP(7 + 2 * cc);
    float acc[G][VCH];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int c = 0; c < VCH; ++c) acc[g][c] = 0.f;
    // With 4 lanes per token (CH = 64) the 4 lanes of a token group are one block
    // of v_mfma_f32_4x4x4 (16 blocks): the group's 4 tokens of a round are the
    // contraction index, lane `sub` supplies the weights of head `sub` (A) and
    // one channel of the rebuilt values (B), and keeps that channel's 4 head
    // sums (D).  The weights go in as bf16 hi + lo (two MFMAs), which carries 16
    // mantissa bits; the values are bf16 already.  This replaces the float32
    // multiply-adds of the vector ALUs, which are this kernel's bottleneck.
    constexpr bool V_MFMA = (LPT == 4 && PPL == 2);
    f32x4_t accm[V_MFMA ? 2 : 1][V_MFMA ? 8 : 1];
    if constexpr (V_MFMA) {
#pragma unroll
      for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int c = 0; c < 8; ++c) accm[h][c] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int k = 0; k < ST_KMAX; ++k) {
      if (k < n_k) {
        uint4 med[V_MFMA ? 2 : 1][V_MFMA ? 4 : 1];
        float psel[V_MFMA ? 4 : 1];
#pragma unroll
        for (int j8 = 0; j8 < LPT; ++j8) {
          const int owner = j8 * TPW + tl;
          const uint2 inf = s_info[(k * ST_WAVES + wave) * 64 + owner];
          float pg[G];
#pragma unroll
          for (int g = 0; g < G; ++g) pg[g] = __shfl(s[k][g], owner);
          int rb[R];
          row_offsets<R>(inf, rb, ROWB_LOG2);
          uint32_t fm[R];
          if constexpr (R == 3) {
            // g_0 goes onto the weight; rows 1, 2 are flipped relative to row 0
            fm[0] = 0u;
            fm[1] = info_flipmask<1>(inf);
            fm[2] = info_flipmask<2>(inf);
            const uint32_t sgn = inf.x << 16 & 0x80000000u;
#pragma unroll
            for (int g = 0; g < G; ++g) pg[g] = __uint_as_float(__float_as_uint(pg[g]) ^ sgn);
          } else {
            fm[0] = info_neg<0>(inf) ? 0x80008000u : 0u;
            fm[1] = info_neg<1>(inf) ? 0x80008000u : 0u;
            fm[2] = info_neg<2>(inf) ? 0x80008000u : 0u;
            if constexpr (R > 3) fm[3] = info_neg<3>(inf) ? 0x80008000u : 0u;
          }
          if constexpr (V_MFMA) {
            float ph = pg[0];
            if constexpr (G > 1) ph = (sub == 1) ? pg[1] : ph;
            if constexpr (G > 2) ph = (sub == 2) ? pg[2] : ph;
            if constexpr (G > 3) ph = (sub == 3) ? pg[3] : ph;
            psel[j8] = (sub < G) ? ph : 0.f;
          }
#pragma unroll
          for (int h = 0; h < PPL; ++h) {
            const int co = (h == 0 ? pa : pb) * 16;
            uint4 row[R];
#pragma unroll
            for (int i = 0; i < R; ++i) {
              row[i] = *reinterpret_cast<const uint4*>(s_sk + rb[i] + co);
              if (!(R == 3 && i == 0)) row[i] = xor4(row[i], fm[i]);
            }
            const uint4 m = median_piece<R>(row, d.median_mode);
            if constexpr (V_MFMA) {
              med[h][j8] = m;
            } else {
              const float v[8] = {bf_lo(m.x), bf_hi(m.x), bf_lo(m.y), bf_hi(m.y),
                                  bf_lo(m.z), bf_hi(m.z), bf_lo(m.w), bf_hi(m.w)};
#pragma unroll
              for (int g = 0; g < G; ++g)
#pragma unroll
                for (int c = 0; c < 8; ++c) acc[g][h * 8 + c] = fmaf(pg[g], v[c], acc[g][h * 8 + c]);
            }
          }
        }
        if constexpr (V_MFMA) {
          // A: this lane's head, 4 tokens, as bf16 hi and lo parts
          uint32_t hb[4], lb[4];
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            const uint32_t pb_ = __float_as_uint(psel[t]);
            hb[t] = pb_ & 0xffff0000u;
            lb[t] = __float_as_uint(psel[t] - __uint_as_float(hb[t]));
          }
          const short4_t a_hi = pack_k4(pair_hi(hb[0], hb[1]), pair_hi(hb[2], hb[3]));
          const short4_t a_lo = pack_k4(pair_hi(lb[0], lb[1]), pair_hi(lb[2], lb[3]));
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            pv_mfma<0>(med[h], a_hi, a_lo, accm[h]);
            pv_mfma<1>(med[h], a_hi, a_lo, accm[h]);
            pv_mfma<2>(med[h], a_hi, a_lo, accm[h]);
            pv_mfma<3>(med[h], a_hi, a_lo, accm[h]);
          }
        }
      }
    }
    if constexpr (V_MFMA) {
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
          for (int c = 0; c < 8; ++c) acc[g][h * 8 + c] = accm[h][c][g];
    }
    KVR_STAMP(8 + 2 * cc);
    // odd token groups hold their two pieces swapped: put them in piece order
    if constexpr (PPL == 2) {
      const bool odd = (tl & 1) != 0;
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int c = 0; c < 8; ++c) {
          const float lo = acc[g][c], hi = acc[g][8 + c];
          acc[g][c] = odd ? hi : lo;
          acc[g][8 + c] = odd ? lo : hi;
        }
    }
    // lanes with equal `sub` hold the same channels.  Inside a row of 16 lanes
    // they are added with DPP rotations (no LDS traffic); the 4 rows of the 8
    // waves then meet in LDS, in the space of the sketch chunk, which nobody
    // reads any more after the barrier.
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int c = 0; c < VCH; ++c) acc[g][c] = row_sum<LPT>(acc[g][c]);
    lds_barrier();
    float* s_part = reinterpret_cast<float*>(s_sk);          // [8 waves * 4 rows][G][CH]
    if ((lane & 15) < LPT) {
      const int prow = wave * 4 + (lane >> 4);
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int h = 0; h < PPL; ++h) {
          float* dst = s_part + (prow * G + g) * CH + (sub + h * LPT) * 8;
          *reinterpret_cast<float4*>(dst) = make_float4(acc[g][h * 8], acc[g][h * 8 + 1], acc[g][h * 8 + 2], acc[g][h * 8 + 3]);
          *reinterpret_cast<float4*>(dst + 4) = make_float4(acc[g][h * 8 + 4], acc[g][h * 8 + 5], acc[g][h * 8 + 6], acc[g][h * 8 + 7]);
        }
    }
    lds_barrier();
    for (int idx = tid; idx < G * CH; idx += ST_THREADS) {
      float o = 0.f;
#pragma unroll
      for (int pr = 0; pr < ST_WAVES * 4; ++pr) o += s_part[pr * G * CH + idx];
      a.part_o[part * G * D + (idx / CH) * D + cc * CH + (idx % CH)] = o;
    }
  }
  KVR_STAMP(11);
}

#ifdef KVR_PHASE_TIMING
extern "C" int kvr_debug_phase_times(unsigned long long* host_out, int n_words) {
  return (int)hipMemcpyFromSymbol(host_out, HIP_SYMBOL(g_phase_t), (size_t)n_words * 8, 0, hipMemcpyDeviceToHost);
}
#endif

template <int G, int R, int CH>
static hipError_t launch_one(const DevDesc& d, const AttendArgs& a, const AttendPlan& plan, hipStream_t st) {
  static bool attr_set = false;
  auto kern = attend_vague_staged_kernel<G, R, CH>;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int units = d.B * d.Hkv;
  const int units_pad = (units + 7) / 8 * 8;
  hipLaunchKernelGGL(kern, dim3(units_pad * plan.n_vslices), dim3(ST_THREADS), plan.lds_bytes, st, d, a);
  return hipGetLastError();
}

template <int G, int R>
static hipError_t launch_ch(const DevDesc& d, const AttendArgs& a, const AttendPlan& plan, hipStream_t st) {
  switch (plan.ch) {
    case 64: return launch_one<G, R, 64>(d, a, plan, st);
    case 32: return launch_one<G, R, 32>(d, a, plan, st);
    case 16: return launch_one<G, R, 16>(d, a, plan, st);
    case 8: return launch_one<G, R, 8>(d, a, plan, st);
    default: return hipErrorInvalidValue;
  }
}

template <int G>
static hipError_t launch_r(const DevDesc& d, const AttendArgs& a, const AttendPlan& plan, hipStream_t st) {
  if (d.r == 3) return launch_ch<G, 3>(d, a, plan, st);
  if (d.r == 4) return launch_ch<G, 4>(d, a, plan, st);
  return hipErrorInvalidValue;
}

hipError_t launch_attend_vague_staged(const DevDesc& d, const AttendArgs& a, const AttendPlan& plan,
                                      hipStream_t st) {
  switch (d.G) {
    case 1: return launch_r<1>(d, a, plan, st);
    case 2: return launch_r<2>(d, a, plan, st);
    case 4: return launch_r<4>(d, a, plan, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace kvr
