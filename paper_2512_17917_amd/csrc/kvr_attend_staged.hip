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
#include "kvr_staged.h"

namespace kvr {

// MODE: the median rule for an even row count, fixed at compile time so that the
// inner loops carry no branch on it (it plays no part when R is odd).
template <int G, int R, int CH, int MODE>
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
  asm volatile("" ::"v"(touched));       // the touch load has no other use: keep it
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
    lds_barrier();
    stage_chunk<NC, ROWB>(skg, s_sk, n_pieces, cc, tid);
    lds_barrier();
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
            const uint4 m = median_piece<R>(row, MODE);
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
  const int sub = lane % LPT, tl = lane / LPT;
  // the two pieces of this lane: odd token groups take them in the opposite order
  const int pa = (PPL == 2) ? sub + ((tl & 1) ? LPT : 0) : sub;
  const int pb = (PPL == 2) ? sub + ((tl & 1) ? 0 : LPT) : sub;
  for (int cc = 0; cc < NPH; ++cc) {
    lds_barrier();
    stage_chunk<NC, ROWB>(svg, s_sk, n_pieces, cc, tid);
    lds_barrier();
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
          // one lane per token: the lane is its own owner
          const uint2 inf = (LPT == 1) ? info[k] : s_info[(k * ST_WAVES + wave) * 64 + owner];
          float pg[G];
#pragma unroll
          for (int g = 0; g < G; ++g) pg[g] = (LPT == 1) ? s[k][g] : __shfl(s[k][g], owner);
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
            const uint4 m = median_piece<R>(row, MODE);
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
}


template <int G, int R, int CH, int MODE>
static hipError_t launch_one(const DevDesc& d, const AttendArgs& a, const AttendPlan& plan, hipStream_t st) {
  auto kern = attend_vague_staged_kernel<G, R, CH, MODE>;
  static std::once_flag once;
  static hipError_t attr_rc = hipSuccess;
  std::call_once(once, [&]() {
    attr_rc = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  160 * 1024);
  });
  if (attr_rc != hipSuccess) return attr_rc;
  const int units = d.B * d.Hkv;
  const int units_pad = (units + 7) / 8 * 8;
  hipLaunchKernelGGL(kern, dim3(units_pad * plan.n_vslices), dim3(ST_THREADS), plan.lds_bytes, st, d, a);
  return hipGetLastError();
}

template <int G, int R, int MODE>
static hipError_t launch_ch(const DevDesc& d, const AttendArgs& a, const AttendPlan& plan, hipStream_t st) {
  switch (plan.ch) {
    case 64: return launch_one<G, R, 64, MODE>(d, a, plan, st);
    case 32: return launch_one<G, R, 32, MODE>(d, a, plan, st);
    case 16: return launch_one<G, R, 16, MODE>(d, a, plan, st);
    case 8: return launch_one<G, R, 8, MODE>(d, a, plan, st);
    default: return hipErrorInvalidValue;
  }
}

template <int G>
static hipError_t launch_r(const DevDesc& d, const AttendArgs& a, const AttendPlan& plan, hipStream_t st) {
  if (d.r == 3) return launch_ch<G, 3, KVR_MEDIAN_MIDMEAN>(d, a, plan, st);
  if (d.r == 4)
    return d.median_mode == KVR_MEDIAN_LOWER ? launch_ch<G, 4, KVR_MEDIAN_LOWER>(d, a, plan, st)
                                             : launch_ch<G, 4, KVR_MEDIAN_MIDMEAN>(d, a, plan, st);
  return hipErrorInvalidValue;
}

hipError_t launch_attend_vague_staged(const DevDesc& d, const AttendArgs& a, const AttendPlan& plan,
                                      hipStream_t st) {
  if (d.r == 3 && plan.ch == 64 && 3 * d.w <= 1024) return launch_attend_vague_staged64(d, a, plan, st);
  if (staged_r4_applies(d)) return launch_attend_vague_staged_r4(d, a, plan, st);
  switch (d.G) {
    case 1: return launch_r<1>(d, a, plan, st);
    case 2: return launch_r<2>(d, a, plan, st);
    case 4: return launch_r<4>(d, a, plan, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace kvr
