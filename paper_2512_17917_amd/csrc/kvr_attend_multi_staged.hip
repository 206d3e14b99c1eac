// kvr_attend_multi, Vague index list, LDS-staged (bf16, three sketch rows, values
// signed only, 3 w <= 1024 so that a 64-channel chunk of a sketch fits LDS).
//
// Rebuilding a Vague token (Algorithm 2) needs three rows of the K sketch and three
// of the V sketch; gathered out of L2 that is 5 GB per layer of the 32k workload.
// Here a workgroup copies one 64-channel chunk of a unit's sketch into LDS and
// walks ALL of its tokens against it, four times (K chunk 0, K chunk 1, V chunk 0,
// V chunk 1).  Nothing about a token stays in registers between the phases: the
// token's record (slots and signs), its partial logits after the first K chunk and
// its final logits go through scratch memory, 16-token tile by tile, so a
// workgroup's share of the list is not limited by registers and a unit's sketch is
// staged by as few workgroups as fill the chip.
//
// Per 16-token tile, with lane = (r16, col) = (lane / 16, lane mod 16):
//   K phases: token t0 + col, 16-byte piece 4 kx + r16 of the chunk (kx = 0, 1) is
//     rebuilt from LDS and is directly the A operand of v_mfma_f32_16x16x32_bf16;
//     the NCOL query vectors are the B operand (column c = query t * G + head g).
//     The lane receives the logits of tokens t0 + 4 r16 + {0..3} for column col.
//   V phases: the weights of those same four tokens for column col are the A operand
//     of v_mfma_f32_16x16x16_bf16 (bf16 hi + lo); the lane rebuilds channels
//     4 col .. 4 col + 3 of the chunk for the four tokens (8 bytes per row) and a
//     register transpose gives the four B operands; instruction c leaves the lane
//     with the sums of columns 4 r16 + {0..3} for channel 4 col + c.
// Softmax: the K-chunk-1 phase knows the final logits, so each wave takes the
// maximum of its tiles per column there; the V phases form the weights against
// the workgroup's maximum (the waves' maxima meet in LDS in between).
// Tiles are handed to the waves through a counter in LDS, phase by phase.
//
// LDS layout: row-major, 128 bytes per sketch slot, but piece p of slot s is kept
// at piece position p xor (s mod 8): the 16 lanes that read the same piece of 16
// random slots then spread over all bank groups instead of two.
#include "kvr_staged.h"

namespace kvr {

typedef __bf16 bf16x8ms_t __attribute__((ext_vector_type(8)));

constexpr int MS_THREADS = 1024;          // 16 waves: four per SIMD cover each other's memory round trips
constexpr int MS_WAVES = MS_THREADS / 64;
// The tile loops read the scratch arrays up to four tiles per wave past the end of a workgroup's share
// (look-ahead, loop rounding, the ragged last round of tiles) without clamping: the arrays are padded.
constexpr int MS_PAD_TOKENS = 4 * MS_WAVES * 16;

struct MultiStagedArgs {
  const bf16_t* q;          // [B, n_q, Hq, D]
  const int32_t* n_ctx;     // [B], or null: every listed token is visible to every query
  int n_q;
  const bf16_t* sk;         // [units, 3, w, D]
  const bf16_t* sv;
  const int32_t* pos;       // Vague index list [units, cap]
  const int32_t* n_valid;   // [units]
  int cap;
  int part_tokens, n_parts; // tokens per workgroup (a multiple of 16), workgroups per unit
  int slice0, n_slices;     // partial index of part 0 / partials per unit
  int tok0, tot_cap;        // logits index of list entry 0 / logits rows per unit
  float* part_o;            // [units, n_slices, NCOL, D]
  float* part_ml;           // [units, n_slices, NCOL, 2]
  float* logits;            // [units, tot_cap, NCOL] final logits (also the merge kernel's input)
  float* partial;           // scratch [units, cap, NCOL]: logits after the first K chunk
  uint2* rec;               // scratch [units, cap]: token records
};

// Token record, the layout of the decode kernel's: LDS row indices (i * w + h_i < 1024) at bit 7 of x
// (first listed row), bit 17 of x (second) and bit 7 of y (third); bit 0 of x = the sign two of the three
// rows agree on (1 = minus, folded into the token's weight); bit 31 of y = the third listed row has the
// other sign.  The row whose sign differs from the other two, if any, is listed third.
__device__ __forceinline__ uint2 make_record3(const DevDesc& d, int w, int J) {
  const uint32_t r0 = (uint32_t)bucket_of(d, 0, J), r1 = (uint32_t)(w + bucket_of(d, 1, J)),
                 r2 = (uint32_t)(2 * w + bucket_of(d, 2, J));
  const uint32_t s0 = sign_neg(d, 0, J) ? 1u : 0u, s1 = sign_neg(d, 1, J) ? 1u : 0u, s2 = sign_neg(d, 2, J) ? 1u : 0u;
  const uint32_t maj = (s0 & s1) | (s0 & s2) | (s1 & s2);
  const bool odd0 = s0 != maj, odd1 = s1 != maj;
  const uint32_t ra = odd0 ? r2 : r0, rbk = odd1 ? r2 : r1, rc = odd0 ? r0 : (odd1 ? r1 : r2);
  const uint32_t flip = (s0 ^ s1) | (s0 ^ s2);
  return make_uint2((ra << 7) | (rbk << 17) | maj, (rc << 7) | (flip << 31));
}
// byte offsets of the three listed rows in the LDS chunk
__device__ __forceinline__ void record_rows(uint2 rec, int (&rb)[3]) {
  rb[0] = (int)(rec.x & 0x1ff80u);
  rb[1] = (int)(__builtin_amdgcn_ubfe(rec.x, 17, 10) << 7);
  rb[2] = (int)(rec.y & 0x1ff80u);
}
// byte offset of piece p inside the LDS row that starts at byte rb (rows are 128 bytes)
__device__ __forceinline__ int swz_piece(int rb, int p) { return rb + (((rb >> 3) ^ (p << 4)) & 0x70); }

// Copy chunk cc (64 channels) of a sketch tensor [rows][128] into LDS, in the swizzled layout (K chunks) or
// plainly (V chunks: their readers take a whole row at a time, 16 lanes x 8 bytes).
template <bool SWZ>
__device__ __forceinline__ void stage_issue_swz(const unsigned char* __restrict__ g, unsigned char* s_sk,
                                                int n_pieces, int cc, int tid) {
  const int lane = tid & 63, wave = tid >> 6;
  for (int p0 = wave * 64; p0 < n_pieces; p0 += MS_THREADS) {
    const int idx = min(p0 + lane, n_pieces - 1);
    const int row = idx >> 3, c = SWZ ? ((idx ^ row) & 7) : (idx & 7);   // LDS piece position idx & 7 holds piece c
    __builtin_amdgcn_global_load_lds(
        (const __attribute__((address_space(1))) void*)(g + (size_t)row * (D * 2) + cc * 128 + c * 16),
        (__attribute__((address_space(3))) void*)(s_sk + p0 * 16), 16, 0, 0);
  }
}

template <int NCOL>
__global__ __launch_bounds__(MS_THREADS) void attend_multi_staged_kernel(DevDesc d, MultiStagedArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  constexpr int CH = 64;
  const float NEG_INF = -__builtin_inff();
  const int units = d.B * d.Hkv;
  // workgroup ids go round-robin to the 8 XCDs: all parts of a unit get ids that are equal modulo 8
  const int lin = blockIdx.x;
  const int unit = ((lin >> 3) / a.n_parts) * 8 + (lin & 7);
  const int part_i = (lin >> 3) % a.n_parts;
  if (unit >= units) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r16 = lane >> 4, col = lane & 15;
  const int w = d.w;
  const int sk_bytes = max((3 * w * 128 + 1023) & ~1023, MS_WAVES * NCOL * CH * 4);
  unsigned char* s_sk = smem;                                        // chunk; later [waves][NCOL][64] floats
  float* s_max = reinterpret_cast<float*>(smem + sk_bytes);          // [waves][16]
  float* s_sum = s_max + MS_WAVES * 16;                              // [waves][16]
  int* s_ctr = reinterpret_cast<int*>(s_sum + MS_WAVES * 16);        // next tile of the running phase

  const int b = unit / d.Hkv, hk = unit % d.Hkv;
  const int rows = clampi(a.n_valid[unit], 0, a.cap);
  const int t_begin = min(part_i * a.part_tokens, rows);
  const int t_end = min(t_begin + a.part_tokens, rows);
  const int n_tiles = (t_end - t_begin + 15) >> 4;
  const int32_t* pp = a.pos + (size_t)unit * a.cap;
  uint2* recs = a.rec + (size_t)unit * a.cap;
  float* partial = a.partial + (size_t)unit * a.cap * NCOL;
  float* logits = a.logits + ((size_t)unit * a.tot_cap + a.tok0) * NCOL;
  const size_t sk_unit = (size_t)unit * 3 * w * D;
  const unsigned char* skg = reinterpret_cast<const unsigned char*>(a.sk + sk_unit);
  const unsigned char* svg = reinterpret_cast<const unsigned char*>(a.sv + sk_unit);
  const int n_pieces = 3 * w * 8;

  // this lane's column: query tq, head g
  const int tq = col / d.G, g = col % d.G;
  const bool col_live = col < NCOL;
  const int qpos = a.n_ctx ? a.n_ctx[b] - a.n_q + tq : 0x7fffffff;   // no n_ctx: no causal mask (decode call)

  // Tiles are handed out through a counter in LDS, phase by phase: of the four waves that share a SIMD the
  // ones started first win the issue arbitration, and with a fixed share each the workgroup would wait for
  // its slowest wave at the end of every phase.
  auto next_tile = [&]() {
    int t = 0;
    if (lane == 0) t = atomicAdd(s_ctr, 1);
    return __builtin_amdgcn_readfirstlane(t);
  };

  // ---- K phases -----------------------------------------------------------------------------------
  float m_run = NEG_INF;
  for (int cc = 0; cc < 2; ++cc) {
    if (cc > 0) lds_barrier();                                // every wave is done with the previous chunk
    stage_issue_swz<true>(skg, s_sk, n_pieces, cc, tid);
    if (cc == 0) {
      // under the first chunk copy: the record of every token of this workgroup, one token per thread
      // (hashed once, not once per lane group that needs it); published by the barrier below
      for (int t = t_begin + tid; t < t_end; t += MS_THREADS) recs[t] = make_record3(d, w, pp[t]);
    }
    // q of this lane's column, channels 64 cc + 32 kx + 8 r16 .. + 7
    uint4 qb[2];
    {
      const bf16_t* q = a.q + (((size_t)b * a.n_q + (col_live ? tq : 0)) * d.Hq + (size_t)hk * d.G + (col_live ? g : 0)) * D +
                        64 * cc + 8 * r16;
#pragma unroll
      for (int kx = 0; kx < 2; ++kx) {
        qb[kx] = *reinterpret_cast<const uint4*>(q + 32 * kx);
        if (!col_live) qb[kx] = make_uint4(0u, 0u, 0u, 0u);
      }
    }
    if (tid == 0) *s_ctr = 0;
    stage_wait();
    lds_barrier();
    // What a tile needs from memory is requested one tile ahead with unconditional loads (indices clamped
    // into the list, results masked afterwards), and what a tile leaves in memory is stored one tile late.
    // Vector memory returns reads in order and writes in order, but not the two against each other, so a
    // wait for any read with a write outstanding drains everything: arranged like this, every such wait
    // only covers requests that are a whole tile old.
    struct KIn {
      uint2 rec;          // record of token t0 + col
      float prev[4];      // second chunk: partial logits of tokens t0 + 4 r16 + i, this lane's column
      int tpos[4];        //               and their positions
    };
    const int t_last = max(t_end - 1, 0);
    const int col_c = col_live ? col : 0;
    auto k_loads = [&](int ti, KIn& in) {
      const int t0 = t_begin + ti * 16;
      in.rec = make_uint2(0u, 0u);
#pragma unroll
      for (int i = 0; i < 4; ++i) { in.prev[i] = 0.f; in.tpos[i] = -1; }
      // the scratch arrays are padded: reads past the end of the list need no clamp (masked later)
      in.rec = recs[t0 + col];
      if (cc == 1) {
        const float* pv = partial + (size_t)(t0 + 4 * r16) * NCOL + col_c;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          in.tpos[i] = pp[min(t0 + 4 * r16 + i, t_last)];
          in.prev[i] = pv[i * NCOL];
        }
      }
    };
    // results of the previous tile, not yet stored
    int st_t0 = -1;
    float st_v[4] = {0.f, 0.f, 0.f, 0.f};
    auto k_stores = [&]() {
      if (st_t0 < 0) return;
      if (col_live) {
        float* dst = (cc == 0) ? partial : logits;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int tt = st_t0 + 4 * r16 + i;
          if (tt < t_end) dst[(size_t)tt * NCOL + col] = st_v[i];
        }
      }
    };
    // Two input buffers take the tiles in turn (copying a buffer would wait for its loads).  A tile past
    // the end of this wave's share computes on clamped inputs and leaves nothing behind.
    auto k_tile = [&](const KIn& cur, KIn& nxt, int ti, int ti_next) {
      const int t0 = t_begin + ti * 16;
      // the tile's inputs must have arrived here (empty statement that reads them), before the
      // previous tile's stores and the next tile's loads are issued
      if (cc == 0) asm volatile("" ::"v"(cur.rec.x), "v"(cur.rec.y));
      else asm volatile("" ::"v"(cur.rec.x), "v"(cur.rec.y), "v"(cur.prev[0]), "v"(cur.prev[1]), "v"(cur.prev[2]),
                        "v"(cur.prev[3]), "v"(cur.tpos[0]), "v"(cur.tpos[1]), "v"(cur.tpos[2]), "v"(cur.tpos[3]));
      __builtin_amdgcn_sched_barrier(0);
      k_stores();
      __builtin_amdgcn_sched_barrier(0);
      k_loads(ti_next, nxt);
      __builtin_amdgcn_sched_barrier(0);
      const bool tk_ok = t0 + col < t_end;
      uint2 rec = cur.rec;
      if (!tk_ok) rec = make_uint2(0u, 0u);
      int rb[3];
      record_rows(rec, rb);
      uint4 ka[2];
#pragma unroll
      for (int kx = 0; kx < 2; ++kx) {
        const int p = 4 * kx + r16;
        const uint4 x0 = *reinterpret_cast<const uint4*>(s_sk + swz_piece(rb[0], p));
        const uint4 x1 = *reinterpret_cast<const uint4*>(s_sk + swz_piece(rb[1], p));
        const uint4 x2 = *reinterpret_cast<const uint4*>(s_sk + swz_piece(rb[2], p));
        ka[kx] = med3_piece(x0, x1, x2);
      }
      f32x4_t S = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kx = 0; kx < 2; ++kx)
        S = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8ms_t, ka[kx]),
                                                    __builtin_bit_cast(bf16x8ms_t, qb[kx]), S, 0, 0, 0);
      st_t0 = t0;
      if (cc == 0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) st_v[i] = S[i];
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int tt = t0 + 4 * r16 + i;
          const bool ok = tt < t_end && cur.tpos[i] >= 0 && cur.tpos[i] <= qpos && col_live;
          st_v[i] = ok ? (S[i] + cur.prev[i]) * d.scale : NEG_INF;
          m_run = fmaxf(m_run, st_v[i]);
        }
      }
    };
    KIn in_a, in_b;
    int ti = next_tile();
    k_loads(ti, in_a);
    while (ti < n_tiles) {
      const int t1 = next_tile();
      k_tile(in_a, in_b, ti, t1);
      const int t2 = next_tile();
      k_tile(in_b, in_a, t1, t2);
      ti = t2;
    }
    k_stores();
  }
  // the wave's maximum per column (the four 16-lane rows hold different tokens of the same column)
  m_run = fmaxf(m_run, __shfl_xor(m_run, 16));
  m_run = fmaxf(m_run, __shfl_xor(m_run, 32));
  if (r16 == 0) s_max[wave * 16 + col] = m_run;

  // ---- V phases -----------------------------------------------------------------------------------
  const size_t part = (size_t)unit * a.n_slices + a.slice0 + part_i;
  float l_run = 0.f;
  for (int cc = 0; cc < 2; ++cc) {
    lds_barrier();                                            // every wave is done with the previous chunk
    stage_issue_swz<false>(svg, s_sk, n_pieces, cc, tid);
    if (tid == 0) *s_ctr = 0;
    if (cc == 0) {
      // a wave meets other tiles here than in the K phases: weights against the workgroup's maximum
      float M = s_max[col];
#pragma unroll
      for (int w_ = 1; w_ < MS_WAVES; ++w_) M = fmaxf(M, s_max[w_ * 16 + col]);
      m_run = M;
    }
    stage_wait();                                             // also: this wave's logits stores have landed
    lds_barrier();
    f32x4_t acc[4];                                           // acc[c][i]: column 4 r16 + i, channel 64 cc + 4 col + c
#pragma unroll
    for (int c = 0; c < 4; ++c) acc[c] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    // this lane's four tokens of a tile: records, and their logits for this lane's column; requested one
    // tile ahead with unconditional loads (no stores in these phases: the waits are exact)
    struct VIn {
      uint2 rj[4];
      float s[4];
    };
    const int col_c = col_live ? col : 0;
    const unsigned char* s_vcol = s_sk + 8 * col;
    const float m_safe = (m_run == NEG_INF) ? 0.f : m_run;    // a column without any visible token: all weights 0
    auto v_loads = [&](int ti, VIn& in) {
      // padded scratch arrays: no clamp (what lies past the end of the list is masked later)
      const int tt0 = t_begin + ti * 16 + 4 * r16;
      const uint2* rp = recs + tt0;
      const float* lp = logits + (size_t)tt0 * NCOL + col_c;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        in.rj[j] = rp[j];
        in.s[j] = lp[j * NCOL];
      }
    };
    auto v_tile = [&](const VIn& cur, VIn& nxt, int ti, int ti_next) {
      const int t0 = t_begin + ti * 16;
      v_loads(ti_next, nxt);
      uint2 rj[4];
      float p[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const bool ok = t0 + 4 * r16 + j < t_end;
        rj[j] = ok ? cur.rj[j] : make_uint2(0u, 0u);
        const float sl = (ok && col_live) ? cur.s[j] : NEG_INF;
        p[j] = __expf(sl - m_safe);                       // -inf (masked, or past the end) gives 0
        if (cc == 0) l_run += p[j];
        // the sign two of the token's three rows agree on goes onto the weight
        p[j] = __uint_as_float(__float_as_uint(p[j]) ^ (rj[j].x << 31));
      }
      uint32_t hb[4], lb[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        hb[i] = __float_as_uint(p[i]) & 0xffff0000u;
        lb[i] = __float_as_uint(p[i] - __uint_as_float(hb[i]));
      }
      const short4_t a_hi = pack_k4(pair_hi(hb[0], hb[1]), pair_hi(hb[2], hb[3]));
      const short4_t a_lo = pack_k4(pair_hi(lb[0], lb[1]), pair_hi(lb[2], lb[3]));
      // channels 4 col .. + 3 of the chunk for the four tokens: 8 bytes at offset 8 col of each row
      uint2 vt[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        int rb[3];
        record_rows(rj[j], rb);
        const uint2 x0 = *reinterpret_cast<const uint2*>(s_vcol + rb[0]);
        const uint2 x1 = *reinterpret_cast<const uint2*>(s_vcol + rb[1]);
        uint2 x2 = *reinterpret_cast<const uint2*>(s_vcol + rb[2]);
        const uint32_t fm = (uint32_t)((int)rj[j].y >> 31) & 0x80008000u;
        x2.x ^= fm;
        x2.y ^= fm;
        vt[j] = med3_half_piece(x0, x1, x2);
      }
      short4_t bop[4];
      bop[0] = pack_k4(pair_lo(vt[0].x, vt[1].x), pair_lo(vt[2].x, vt[3].x));
      bop[1] = pack_k4(pair_hi(vt[0].x, vt[1].x), pair_hi(vt[2].x, vt[3].x));
      bop[2] = pack_k4(pair_lo(vt[0].y, vt[1].y), pair_lo(vt[2].y, vt[3].y));
      bop[3] = pack_k4(pair_hi(vt[0].y, vt[1].y), pair_hi(vt[2].y, vt[3].y));
#pragma unroll
      for (int c = 0; c < 4; ++c) acc[c] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a_hi, bop[c], acc[c], 0, 0, 0);
#pragma unroll
      for (int c = 0; c < 4; ++c) acc[c] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a_lo, bop[c], acc[c], 0, 0, 0);
    };
    VIn in_a, in_b;
    int ti = next_tile();
    v_loads(ti, in_a);
    while (ti < n_tiles) {
      const int t1 = next_tile();
      v_tile(in_a, in_b, ti, t1);
      const int t2 = next_tile();
      v_tile(in_b, in_a, t1, t2);
      ti = t2;
    }
    if (cc == 0) {
      // a lane's sum of weights covers its own four tokens of every tile: add the four 16-lane rows
      float l = l_run + __shfl_xor(l_run, 16);
      l += __shfl_xor(l, 32);
      if (r16 == 0) s_sum[wave * 16 + col] = l;
    }
    lds_barrier();                                            // the chunk is free: the waves' sums meet in it
    float* s_acc = reinterpret_cast<float*>(s_sk);            // [waves][NCOL][64]
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int c_ = 4 * r16 + i;
      if (c_ < NCOL) {
        *reinterpret_cast<float4*>(s_acc + ((size_t)wave * NCOL + c_) * CH + 4 * col) =
            make_float4(acc[0][i], acc[1][i], acc[2][i], acc[3][i]);
      }
    }
    lds_barrier();
    for (int idx = tid; idx < NCOL * CH; idx += MS_THREADS) {
      const int c_ = idx / CH, ch = idx % CH;
      float M = s_max[c_];
#pragma unroll
      for (int w_ = 1; w_ < MS_WAVES; ++w_) M = fmaxf(M, s_max[w_ * 16 + c_]);
      float L = 0.f, O = 0.f;
#pragma unroll
      for (int w_ = 0; w_ < MS_WAVES; ++w_) {
        L += s_sum[w_ * 16 + c_];
        O += s_acc[((size_t)w_ * NCOL + c_) * CH + ch];
      }
      a.part_o[(part * NCOL + c_) * D + cc * CH + ch] = O;
      if (cc == 0 && ch == 0) {
        a.part_ml[(part * NCOL + c_) * 2] = M;
        a.part_ml[(part * NCOL + c_) * 2 + 1] = L;
      }
    }
  }
}

// ---- host side ----------------------------------------------------------------------------------------
bool multi_staged_applies(const DevDesc& d, long long vague_cap) {
  return d.r == 3 && d.sign_mask == 2 && 3 * d.w <= 1024 && vague_cap >= 64;
}

int multi_staged_pad_tokens() { return MS_PAD_TOKENS; }

// tokens per workgroup: a unit's list is cut for about one workgroup per CU in all, at least 256 tokens each
int multi_staged_part_tokens(long long vague_cap, long long units) {
  long long parts = (256 + units - 1) / units;
  if (parts < 1) parts = 1;
  long long t = (vague_cap + parts - 1) / parts;
  if (t < 256) t = 256;
  return (int)((t + 15) / 16 * 16);
}

template <int NCOL>
static hipError_t launch_n(const DevDesc& d, const MultiStagedArgs& a, hipStream_t st) {
  auto kern = attend_multi_staged_kernel<NCOL>;
  static std::once_flag once;
  static hipError_t attr_rc = hipSuccess;
  std::call_once(once, [&]() {
    attr_rc = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  160 * 1024);
  });
  if (attr_rc != hipSuccess) return attr_rc;
  size_t chunk = ((size_t)3 * d.w * 128 + 1023) & ~(size_t)1023;
  const size_t merge = (size_t)MS_WAVES * NCOL * 64 * 4;
  if (chunk < merge) chunk = merge;
  const size_t lds = chunk + 2 * MS_WAVES * 16 * sizeof(float) + 16;
  if (lds > 160 * 1024) return hipErrorInvalidValue;
  const int units = d.B * d.Hkv;
  const int units_pad = (units + 7) / 8 * 8;
  hipLaunchKernelGGL(kern, dim3(units_pad * a.n_parts), dim3(MS_THREADS), lds, st, d, a);
  return hipGetLastError();
}

hipError_t launch_attend_multi_staged(const DevDesc& d, const AttendArgs& a0, const int32_t* n_ctx, int n_q,
                                      int part_tokens, int n_parts, int slice0, int n_slices, float* part_o,
                                      float* part_ml, float* logits, void* scratch_rec, void* scratch_partial,
                                      hipStream_t st) {
  if (!multi_staged_applies(d, a0.vague_cap) || n_parts < 1 || (part_tokens & 15) != 0) return hipErrorInvalidValue;
  MultiStagedArgs a;
  a.q = (const bf16_t*)a0.q;
  a.n_ctx = n_ctx;
  a.n_q = n_q;
  a.sk = (const bf16_t*)a0.sk;
  a.sv = (const bf16_t*)a0.sv;
  a.pos = a0.vague_pos;
  a.n_valid = a0.n_vague;
  a.cap = a0.vague_cap;
  a.part_tokens = part_tokens;
  a.n_parts = n_parts;
  a.slice0 = slice0;
  a.n_slices = n_slices;
  a.tok0 = a0.ret_cap;
  a.tot_cap = a0.ret_cap + a0.vague_cap;
  a.part_o = part_o;
  a.part_ml = part_ml;
  a.logits = logits;
  a.partial = (float*)scratch_partial;
  a.rec = (uint2*)scratch_rec;
  switch (n_q * d.G) {
    case 1: return launch_n<1>(d, a, st);
    case 2: return launch_n<2>(d, a, st);
    case 4: return launch_n<4>(d, a, st);
    case 8: return launch_n<8>(d, a, st);
    case 16: return launch_n<16>(d, a, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace kvr
