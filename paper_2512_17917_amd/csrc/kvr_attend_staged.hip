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
//   V phases: CH/8 lanes share one token (8 channels each) and accumulate
//     p * v in registers across all of the wave's tokens; the token's weights
//     come from their owner lane by a lane permute.
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

// Median over R rows of a 16-byte piece (8 packed bf16 channels).
template <int R>
__device__ __forceinline__ uint4 median_piece(const uint4 (&row)[R], int mode) {
  uint4 m;
  if constexpr (R == 3) {
    m.x = med3_bf16x2(row[0].x, row[1].x, row[2].x);
    m.y = med3_bf16x2(row[0].y, row[1].y, row[2].y);
    m.z = med3_bf16x2(row[0].z, row[1].z, row[2].z);
    m.w = med3_bf16x2(row[0].w, row[1].w, row[2].w);
  } else {
    const uint32_t* rw[R];
#pragma unroll
    for (int i = 0; i < R; ++i) rw[i] = reinterpret_cast<const uint32_t*>(&row[i]);
    uint32_t o[4];
#pragma unroll
    for (int dw = 0; dw < 4; ++dw) {
      float lo[R], hi[R];
#pragma unroll
      for (int i = 0; i < R; ++i) { lo[i] = bf_lo(rw[i][dw]); hi[i] = bf_hi(rw[i][dw]); }
      o[dw] = pack_bf16_exact(median_rows<R, bf16_t>(lo, R, mode), median_rows<R, bf16_t>(hi, R, mode));
    }
    m = make_uint4(o[0], o[1], o[2], o[3]);
  }
  return m;
}

__device__ __forceinline__ uint4 xor4(uint4 v, uint32_t mask) {
  return make_uint4(v.x ^ mask, v.y ^ mask, v.z ^ mask, v.w ^ mask);
}

// token info: 4 x 16 bits; bits 0..14 bucket, bit 15 sign (1 = negative)
__device__ __forceinline__ int info_bucket(uint2 inf, int i) {
  const uint32_t wd = (i < 2) ? inf.x : inf.y;
  return (int)((wd >> ((i & 1) * 16)) & 0x7fffu);
}
__device__ __forceinline__ uint32_t info_neg(uint2 inf, int i) {
  const uint32_t wd = (i < 2) ? inf.x : inf.y;
  return (wd >> ((i & 1) * 16 + 15)) & 1u;
}

template <int G, int R, int CH>
__global__ __launch_bounds__(ST_THREADS) void attend_vague_staged_kernel(DevDesc d, AttendArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  constexpr int NC = CH / 8;          // 16-byte pieces per LDS row
  constexpr int NPH = D / CH;         // phases per tensor
  constexpr int ROWB = CH * 2;        // bytes per LDS row
  constexpr int TPW = WAVE / NC;      // V phase: tokens per wave-iteration

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
  const int sk_bytes = (R * w * ROWB + 15) & ~15;
  unsigned char* s_sk = smem;
  uint2* s_info = reinterpret_cast<uint2*>(smem + sk_bytes);
  float* s_red = reinterpret_cast<float*>(smem + sk_bytes + ST_KMAX * ST_THREADS * 8);   // [8][G][CH]
  float* s_stat = s_red + ST_WAVES * G * 64;                                               // [8][G] x 2, [G] x 2
  uint4* s_q = reinterpret_cast<uint4*>(smem + sk_bytes + ST_KMAX * ST_THREADS * 8 + ST_WAVES * G * 64 * 4 + 1024);

  const int nv = clampi(a.n_vague[unit], 0, a.vague_cap);
  const int rounds_total = (nv + 63) >> 6;
  const int NWT = a.n_vslices * ST_WAVES;
  const int gw = vs * ST_WAVES + wave;
  int n_k = gw < rounds_total ? (rounds_total - gw + NWT - 1) / NWT : 0;
  if (n_k > ST_KMAX) n_k = ST_KMAX;       // cannot happen when the plan was made for vague_cap

  // ---- hash every token once; q to LDS ---------------------------------------
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
      for (int i = 0; i < R; ++i) f[i] = (uint32_t)bucket_of(d, i, J) | (sign_neg(d, i, J) ? 0x8000u : 0u);
      pk = make_uint2(f[0] | (f[1] << 16), f[2] | (f[3] << 16));
      vmask |= 1u << k;
    }
    info[k] = pk;
    s_info[(k * ST_WAVES + wave) * 64 + lane] = pk;
  }
  if (tid < G * 16) {
    const uint4* qg = reinterpret_cast<const uint4*>((const bf16_t*)a.q + ((size_t)b * d.Hq + (size_t)hk * G) * D);
    s_q[tid] = qg[tid];
  }

  const size_t sk_unit = (size_t)unit * R * w * D;      // elements
  const unsigned char* skg = reinterpret_cast<const unsigned char*>((const bf16_t*)a.sk + sk_unit);
  const unsigned char* svg = reinterpret_cast<const unsigned char*>((const bf16_t*)a.sv + sk_unit);
  const int n_pieces = R * w * NC;

  // ---- K phases: logits -----------------------------------------------------
  float s[ST_KMAX][G];
#pragma unroll
  for (int k = 0; k < ST_KMAX; ++k)
#pragma unroll
    for (int g = 0; g < G; ++g) s[k][g] = 0.f;

  for (int cc = 0; cc < NPH; ++cc) {
    __syncthreads();
    for (int idx = tid; idx < n_pieces; idx += ST_THREADS) {
      const int row = idx / NC, c = idx % NC;
      const uint4 v = *reinterpret_cast<const uint4*>(skg + (size_t)row * (D * 2) + cc * ROWB + c * 16);
      *reinterpret_cast<uint4*>(s_sk + row * ROWB + c * 16) = v;
    }
    __syncthreads();
    uint4 qreg[NC][G];
#pragma unroll
    for (int j = 0; j < NC; ++j)
#pragma unroll
      for (int g = 0; g < G; ++g) qreg[j][g] = s_q[g * 16 + cc * NC + ((lane + j) & (NC - 1))];
#pragma unroll
    for (int k = 0; k < ST_KMAX; ++k) {
      if (k < n_k) {
        int rb[R];
#pragma unroll
        for (int i = 0; i < R; ++i) rb[i] = (i * w + info_bucket(info[k], i)) * ROWB;
#pragma unroll
        for (int j = 0; j < NC; ++j) {
          const int co = ((lane + j) & (NC - 1)) * 16;
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
#pragma unroll
  for (int g = 0; g < G; ++g) {
#pragma unroll
    for (int off = 1; off < WAVE; off <<= 1) mx[g] = fmaxf(mx[g], __shfl_xor(mx[g], off));
    if (lane == 0) s_stat[wave * G + g] = mx[g];
  }
  __syncthreads();
  float M[G], lsum[G];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float v = s_stat[g];
#pragma unroll
    for (int w_ = 1; w_ < ST_WAVES; ++w_) v = fmaxf(v, s_stat[w_ * G + g]);
    M[g] = v;
    lsum[g] = 0.f;
  }
#pragma unroll
  for (int k = 0; k < ST_KMAX; ++k)
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float p = (s[k][g] == -__builtin_inff()) ? 0.f : expf(s[k][g] - M[g]);
      s[k][g] = p;                 // from here on s holds the weights
      lsum[g] += p;
    }
#pragma unroll
  for (int g = 0; g < G; ++g) {
#pragma unroll
    for (int off = 1; off < WAVE; off <<= 1) lsum[g] += __shfl_xor(lsum[g], off);
    if (lane == 0) s_stat[ST_WAVES * G + wave * G + g] = lsum[g];
  }
  __syncthreads();
  const size_t part = (size_t)unit * a.n_slices + a.n_rslices + vs;
  if (tid < G) {
    float L = 0.f, Mg = s_stat[tid];
#pragma unroll
    for (int w_ = 0; w_ < ST_WAVES; ++w_) {
      L += s_stat[ST_WAVES * G + w_ * G + tid];
      Mg = fmaxf(Mg, s_stat[w_ * G + tid]);
    }
    a.part_ml[(part * G + tid) * 2] = Mg;
    a.part_ml[(part * G + tid) * 2 + 1] = L;
  }

  // ---- V phases: weighted values ------------------------------------------------
  const int sub = lane % NC, tl = lane / NC;
  for (int cc = 0; cc < NPH; ++cc) {
    __syncthreads();
    for (int idx = tid; idx < n_pieces; idx += ST_THREADS) {
      const int row = idx / NC, c = idx % NC;
      const uint4 v = *reinterpret_cast<const uint4*>(svg + (size_t)row * (D * 2) + cc * ROWB + c * 16);
      *reinterpret_cast<uint4*>(s_sk + row * ROWB + c * 16) = v;
    }
    __syncthreads();
    float acc[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int c = 0; c < 8; ++c) acc[g][c] = 0.f;
#pragma unroll
    for (int k = 0; k < ST_KMAX; ++k) {
      if (k < n_k) {
        for (int j8 = 0; j8 < NC; ++j8) {
          const int owner = j8 * TPW + tl;
          const uint2 inf = s_info[(k * ST_WAVES + wave) * 64 + owner];
          float pg[G];
#pragma unroll
          for (int g = 0; g < G; ++g) pg[g] = __shfl(s[k][g], owner);
          uint4 row[R];
#pragma unroll
          for (int i = 0; i < R; ++i)
            row[i] = *reinterpret_cast<const uint4*>(s_sk + (i * w + info_bucket(inf, i)) * ROWB + sub * 16);
          if constexpr (R == 3) {
            // g_0 goes onto the weight; rows 1, 2 are flipped relative to row 0
            const uint32_t n0 = info_neg(inf, 0);
            row[1] = xor4(row[1], (info_neg(inf, 1) ^ n0) ? 0x80008000u : 0u);
            row[2] = xor4(row[2], (info_neg(inf, 2) ^ n0) ? 0x80008000u : 0u);
            const uint32_t sgn = n0 << 31;
#pragma unroll
            for (int g = 0; g < G; ++g) pg[g] = __uint_as_float(__float_as_uint(pg[g]) ^ sgn);
          } else {
#pragma unroll
            for (int i = 0; i < R; ++i) row[i] = xor4(row[i], info_neg(inf, i) ? 0x80008000u : 0u);
          }
          const uint4 m = median_piece<R>(row, d.median_mode);
          const float v[8] = {bf_lo(m.x), bf_hi(m.x), bf_lo(m.y), bf_hi(m.y),
                              bf_lo(m.z), bf_hi(m.z), bf_lo(m.w), bf_hi(m.w)};
#pragma unroll
          for (int g = 0; g < G; ++g)
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[g][c] = fmaf(pg[g], v[c], acc[g][c]);
        }
      }
    }
    // lanes with equal `sub` hold the same channels: add them up, then the waves
#pragma unroll
    for (int off = NC; off < WAVE; off <<= 1)
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[g][c] += __shfl_xor(acc[g][c], off);
    if (tl == 0) {
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int c = 0; c < 8; ++c) s_red[(wave * G + g) * CH + sub * 8 + c] = acc[g][c];
    }
    __syncthreads();
    for (int idx = tid; idx < G * CH; idx += ST_THREADS) {
      const int g = idx / CH, c = idx % CH;
      float o = 0.f;
#pragma unroll
      for (int w_ = 0; w_ < ST_WAVES; ++w_) o += s_red[(w_ * G + g) * CH + c];
      a.part_o[(part * G + g) * D + cc * CH + c] = o;
    }
  }
}

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
