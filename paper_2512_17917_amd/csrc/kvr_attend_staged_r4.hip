// Staged attention kernel over the Vague list for r = 4 sketch rows (bf16 storage,
// values signed only, G <= 4 query heads per kv head).  Same contract and the
// same token -> wave mapping as the general staged kernel (kvr_attend_staged.hip),
// which it replaces for four rows.
//
// With four rows a kv head's sketch is large (the 131k-token workload: 4 x 819
// slots of 256 bytes per tensor), so it goes through LDS in chunks of 16 channels
// (32 bytes per slot; eight chunks of the K sketch, then eight of the V sketch).
// Inside a chunk the unit of work is a *half piece*: 4 channels = 8 bytes, which
// is exactly the contraction length of v_mfma_f32_4x4x4.
//
//  * K phases: one lane = one token.  The 4 lanes of a block read the same half
//    piece of their tokens' rows (neighbouring blocks take different half pieces,
//    so the 16 lanes served together spread over the banks), the four-row median
//    is taken on packed bf16 bits (median_dword<4>), and one matrix instruction per
//    half piece multiplies the block's 4 rebuilt tokens (A, one row per lane) with
//    q (B, column j = head j): lane j receives the logits of the block's 4 tokens
//    for head j -- already the layout the V phases want for their A operand, so the
//    softmax needs no transposition afterwards.
//  * V phases: a quad rebuilds the 4 tokens its own lanes own, lane `sub` taking
//    half piece `sub` of every row; a token's row offsets and flip masks reach the
//    quad by DPP quad broadcasts.  With the mean-of-the-middle-two rule (an odd
//    function of the four values) g_0 is folded into the token's weight and the
//    other rows are flipped relative to row 0; with the lower-middle rule every row
//    is flipped by its own sign.  p.v on the same matrix instruction with the 4
//    tokens as the contraction index; weights as bf16 hi + lo.
//  * Every loop over LDS reads is a pinned software pipeline (rows of the step
//    after next requested, medians of the next step formed, matrix instruction of
//    this step issued): two waves per SIMD cannot hide LDS latency for each other.
//  * The copy of the next chunk is started as soon as every wave is done with the
//    current one and overlaps the reduction of the V partial sums, which have LDS
//    of their own (two sets that take turns, so that a chunk needs two barriers).
#include "kvr_staged.h"

namespace kvr {
namespace {

constexpr int R4_CH = 16;                 // channels per chunk
constexpr int R4_ROWB = 32;               // bytes per LDS row
constexpr int R4_NHP = 4;                 // 8-byte half pieces per LDS row
constexpr int R4_NCHUNK = D / R4_CH;      // chunks per tensor
constexpr int R4_NROW = ST_WAVES * 4;     // 16-lane rows per workgroup
constexpr int R4_KMAX = STAGED_R4_KMAX;   // wave-rounds (64 tokens) per wave

struct Rows4 {
  uint2 r0, r1, r2, r3;
};

__device__ __forceinline__ void load_rows4(Rows4& o, const unsigned char* s_sk, const int (&rb)[4], int co) {
  o.r0 = *reinterpret_cast<const uint2*>(s_sk + rb[0] + co);
  o.r1 = *reinterpret_cast<const uint2*>(s_sk + rb[1] + co);
  o.r2 = *reinterpret_cast<const uint2*>(s_sk + rb[2] + co);
  o.r3 = *reinterpret_cast<const uint2*>(s_sk + rb[3] + co);
}

template <int MODE>
__device__ __forceinline__ uint2 median4(const Rows4& v) {
  const uint32_t x[4] = {v.r0.x, v.r1.x, v.r2.x, v.r3.x};
  const uint32_t y[4] = {v.r0.y, v.r1.y, v.r2.y, v.r3.y};
  return make_uint2(median_dword<4>(x, MODE), median_dword<4>(y, MODE));
}

// value of lane J of this lane's quad
template <int J>
__device__ __forceinline__ uint32_t quad_bcast(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, J | (J << 2) | (J << 4) | (J << 6), 0xf, 0xf, true);
}

// Token record (2 dwords).  LDS row indices (i * w + h_i(J) < 4096) are stored
// pre-multiplied by the 32-byte row pitch: row 0 in x[5..16], row 1 in x[17..28],
// row 2 in y[5..16], row 3 in y[17..28].  Bit 0 of x is a sign that is folded into
// the token's weight; bit 30 of x, bit 31 of x, bit 31 of y and bit 30 of y say
// whether rows 0, 1, 2, 3 are flipped before the median.  The mean of the two middle
// values is an odd function of the four values, so there g_0 goes onto the weight
// and the rows are flipped relative to row 0 (row 0 never is); the lower of the two
// middle values is not odd, so there nothing is folded and every row is flipped by
// its own sign.
template <int MODE>
__device__ __forceinline__ uint2 make_record(const DevDesc& d, int w, int J) {
  const uint32_t r0 = (uint32_t)bucket_of(d, 0, J), r1 = (uint32_t)(w + bucket_of(d, 1, J)),
                 r2 = (uint32_t)(2 * w + bucket_of(d, 2, J)), r3 = (uint32_t)(3 * w + bucket_of(d, 3, J));
  const uint32_t s0 = sign_neg(d, 0, J) ? 1u : 0u, s1 = sign_neg(d, 1, J) ? 1u : 0u,
                 s2 = sign_neg(d, 2, J) ? 1u : 0u, s3 = sign_neg(d, 3, J) ? 1u : 0u;
  const uint32_t fold = (MODE == KVR_MEDIAN_MIDMEAN) ? s0 : 0u;
  return make_uint2((r0 << 5) | (r1 << 17) | fold | ((s0 ^ fold) << 30) | ((s1 ^ fold) << 31),
                    (r2 << 5) | (r3 << 17) | ((s2 ^ fold) << 31) | ((s3 ^ fold) << 30));
}
__device__ __forceinline__ void rec_offsets(uint2 rec, int (&rb)[4]) {
  rb[0] = (int)(rec.x & 0x1ffe0u);
  rb[1] = (int)((rec.x >> 12) & 0x1ffe0u);
  rb[2] = (int)(rec.y & 0x1ffe0u);
  rb[3] = (int)((rec.y >> 12) & 0x1ffe0u);
}

// V phases: what a lane derives from its own token's record (row offsets and the
// flip masks of rows 1..3); the other lanes of the quad fetch it with quad
// broadcasts, so a record is taken apart once per quad.
struct VOwn {
  int o0, o1, o2, o3;
  uint32_t f0, f1, f2, f3;
};
__device__ __forceinline__ VOwn v_own(uint2 rec) {
  int rb[4];
  rec_offsets(rec, rb);
  return VOwn{rb[0], rb[1], rb[2], rb[3], (uint32_t)((int)(rec.x << 1) >> 31) & 0x80008000u,
              (uint32_t)((int)rec.x >> 31) & 0x80008000u, (uint32_t)((int)rec.y >> 31) & 0x80008000u,
              (uint32_t)((int)(rec.y << 1) >> 31) & 0x80008000u};
}
struct VItem {
  Rows4 rows;
  uint32_t f0, f1, f2, f3;
};
template <int J, int MODE>
__device__ __forceinline__ void v_fetch(VItem& o, const VOwn& own, const unsigned char* s_sk, int co) {
  int rb[4];
  rb[0] = (int)quad_bcast<J>((uint32_t)own.o0) + co;
  rb[1] = (int)quad_bcast<J>((uint32_t)own.o1) + co;
  rb[2] = (int)quad_bcast<J>((uint32_t)own.o2) + co;
  rb[3] = (int)quad_bcast<J>((uint32_t)own.o3) + co;
  o.f0 = (MODE == KVR_MEDIAN_MIDMEAN) ? 0u : quad_bcast<J>(own.f0);
  o.f1 = quad_bcast<J>(own.f1);
  o.f2 = quad_bcast<J>(own.f2);
  o.f3 = quad_bcast<J>(own.f3);
  load_rows4(o.rows, s_sk, rb, 0);
}
template <int MODE>
__device__ __forceinline__ uint2 v_median(const VItem& it) {
  Rows4 x;
  x.r0 = it.rows.r0;
  if constexpr (MODE != KVR_MEDIAN_MIDMEAN) x.r0 = make_uint2(it.rows.r0.x ^ it.f0, it.rows.r0.y ^ it.f0);
  x.r1 = make_uint2(it.rows.r1.x ^ it.f1, it.rows.r1.y ^ it.f1);
  x.r2 = make_uint2(it.rows.r2.x ^ it.f2, it.rows.r2.y ^ it.f2);
  x.r3 = make_uint2(it.rows.r3.x ^ it.f3, it.rows.r3.y ^ it.f3);
  return median4<MODE>(x);
}

// acc[c] (4 head sums of channel c of the half piece) += weights (4 heads x 4 tokens,
// bf16 hi + lo) x values (4 tokens x 4 channels)
__device__ __forceinline__ void pv_half_piece(const uint2 (&med)[4], short4_t a_hi, short4_t a_lo, f32x4_t (&acc)[4]) {
  short4_t b[4];
  b[0] = pack_k4(pair_lo(med[0].x, med[1].x), pair_lo(med[2].x, med[3].x));
  b[1] = pack_k4(pair_hi(med[0].x, med[1].x), pair_hi(med[2].x, med[3].x));
  b[2] = pack_k4(pair_lo(med[0].y, med[1].y), pair_lo(med[2].y, med[3].y));
  b[3] = pack_k4(pair_hi(med[0].y, med[1].y), pair_hi(med[2].y, med[3].y));
#pragma unroll
  for (int c = 0; c < 4; ++c) acc[c] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(a_hi, b[c], acc[c], 0, 0, 0);
#pragma unroll
  for (int c = 0; c < 4; ++c) acc[c] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(a_lo, b[c], acc[c], 0, 0, 0);
}

// The same value, but the compiler can no longer tell: whatever is derived from
// it is computed where it is used instead of once per kernel and kept in
// registers through all phases.
__device__ __forceinline__ uint2 opaque(uint2 v) {
  asm volatile("" : "+v"(v.x), "+v"(v.y));
  return v;
}
__device__ __forceinline__ int opaque_s(int v) {
  asm volatile("" : "+s"(v));
  return v;
}

#define KVR_PIN() __builtin_amdgcn_sched_barrier(0)

// The two waves that share a SIMD take turns in having the higher issue priority,
// round by round; both levels are above the default 0.
__device__ __forceinline__ void take_turn(int t) {
  if (t & 1) __builtin_amdgcn_s_setprio(2);
  else __builtin_amdgcn_s_setprio(1);
}

// K pass over NK rounds of one chunk.  qx[j]: the 4 channels of q for head (lane
// mod 4) that belong to the half piece this lane's block reads at step j (byte
// offset co[j] of the row).  s[k][i]: logit of token i of this lane's quad in round
// k, for head (lane mod 4).  Pipeline over the steps t = 4 k + j: rows of step t + 2
// requested, median of step t + 1 formed, matrix instruction of step t issued.
template <int NK, int MODE>
__device__ __forceinline__ void k_pass(const unsigned char* s_sk, const uint2 (&info)[R4_KMAX],
                                       const uint2 (&qx)[R4_NHP], const int (&co)[R4_NHP], int turn,
                                       float (&s)[R4_KMAX][4]) {
  Rows4 buf[3];                          // rows of step t live in buf[t % 3]
  int rb[4];
  rec_offsets(opaque(info[0]), rb);
  load_rows4(buf[0], s_sk, rb, co[0]);
  load_rows4(buf[1], s_sk, rb, co[1]);
  uint2 m[2];                            // median of step t in m[t % 2]
  m[0] = median4<MODE>(buf[0]);
#pragma unroll
  for (int k = 0; k < NK; ++k) {
    int rn[4] = {0, 0, 0, 0};
    if (k + 1 < NK) rec_offsets(opaque(info[k + 1]), rn);
    f32x4_t ax = {0.f, 0.f, 0.f, 0.f};
    take_turn(k + turn);
#pragma unroll
    for (int j = 0; j < R4_NHP; ++j) {
      const int t = R4_NHP * k + j;
      if (j + 2 < R4_NHP) load_rows4(buf[(t + 2) % 3], s_sk, rb, co[j + 2]);
      else if (k + 1 < NK) load_rows4(buf[(t + 2) % 3], s_sk, rn, co[j + 2 - R4_NHP]);
      KVR_PIN();
      if (j + 1 < R4_NHP || k + 1 < NK) m[(t + 1) & 1] = median4<MODE>(buf[(t + 1) % 3]);
      KVR_PIN();
      const uint2 mc = m[t & 1];
      ax = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(pack_k4(mc.x, mc.y), pack_k4(qx[j].x, qx[j].y), ax, 0, 0, 0);
      KVR_PIN();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) s[k][i] += ax[i];
#pragma unroll
    for (int i = 0; i < 4; ++i) rb[i] = rn[i];
  }
  __builtin_amdgcn_s_setprio(1);
}

// V pass over NK rounds of one chunk for the half piece at byte offset co of each
// row: the quad's 4 tokens per round, same kind of pipeline.
template <int NK, int MODE>
__device__ __forceinline__ void v_pass(const unsigned char* s_sk, const uint2 (&info)[R4_KMAX],
                                       const uint32_t (&W)[R4_KMAX][4], int co, int turn, f32x4_t (&acc)[4]) {
  VItem buf[4];
  VOwn own = v_own(info[0]);
  v_fetch<0, MODE>(buf[0], own, s_sk, co);
  v_fetch<1, MODE>(buf[1], own, s_sk, co);
#pragma unroll
  for (int k = 0; k < NK; ++k) {
    uint2 med[4];
    take_turn(k + turn);
    v_fetch<2, MODE>(buf[2], own, s_sk, co);
    KVR_PIN();
    med[0] = v_median<MODE>(buf[0]);
    KVR_PIN();
    v_fetch<3, MODE>(buf[3], own, s_sk, co);
    if (k + 1 < NK) own = v_own(info[k + 1]);
    KVR_PIN();
    med[1] = v_median<MODE>(buf[1]);
    KVR_PIN();
    if (k + 1 < NK) v_fetch<0, MODE>(buf[0], own, s_sk, co);
    KVR_PIN();
    med[2] = v_median<MODE>(buf[2]);
    KVR_PIN();
    if (k + 1 < NK) v_fetch<1, MODE>(buf[1], own, s_sk, co);
    KVR_PIN();
    med[3] = v_median<MODE>(buf[3]);
    pv_half_piece(med, pack_k4(W[k][0], W[k][1]), pack_k4(W[k][2], W[k][3]), acc);
    KVR_PIN();
  }
  __builtin_amdgcn_s_setprio(1);
}

// the round count is uniform over a wave: one scalar branch into straight-line code
#define KVR_DISPATCH_NK(n, CALL) \
  switch (n) {                   \
    case 1: { constexpr int NK = 1; CALL; } break; \
    case 2: { constexpr int NK = 2; CALL; } break; \
    case 3: { constexpr int NK = 3; CALL; } break; \
    case 4: { constexpr int NK = 4; CALL; } break; \
    case 5: { constexpr int NK = 5; CALL; } break; \
    case 6: { constexpr int NK = 6; CALL; } break; \
    case 7: { constexpr int NK = 7; CALL; } break; \
    case 8: { constexpr int NK = 8; CALL; } break; \
    case 9: { constexpr int NK = 9; CALL; } break; \
    case 10: { constexpr int NK = 10; CALL; } break; \
    case 11: { constexpr int NK = 11; CALL; } break; \
    case 12: { constexpr int NK = 12; CALL; } break; \
    case 13: { constexpr int NK = 13; CALL; } break; \
    default: break;              \
  }
static_assert(STAGED_R4_KMAX <= 13, "KVR_DISPATCH_NK covers 1..13 rounds");

// LDS of a workgroup: one chunk, two sets of V partial sums [NROW][G][CH], wave statistics, q
__host__ __device__ constexpr int chunk_bytes(int w) { return (4 * w * R4_ROWB + 1023) & ~1023; }
__host__ __device__ constexpr int stat_floats(int G) { return 3 * ST_WAVES * G; }
__host__ __device__ constexpr size_t lds_need(int w, int G) {
  return (size_t)chunk_bytes(w) + (size_t)2 * R4_NROW * G * R4_CH * 4 + (size_t)stat_floats(G) * 4 + (size_t)G * 256;
}

}  // namespace

template <int G, int MODE>
__global__ __launch_bounds__(ST_THREADS) void attend_vague_staged_r4_kernel(DevDesc d, AttendArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  constexpr int KMAX = R4_KMAX, CH = R4_CH;

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
  const int cb = chunk_bytes(w);
  unsigned char* s_sk = smem;                                             // one 16-channel chunk
  float* s_part = reinterpret_cast<float*>(smem + cb);                    // [2][NROW][G][CH]
  float* s_stat = s_part + 2 * R4_NROW * G * CH;                          // [8 waves][G] maxima, sums, factors
  uint2* s_q = reinterpret_cast<uint2*>(s_stat + stat_floats(G));         // [G][32] half pieces of q

  const int nv = clampi(a.n_vague[unit], 0, a.vague_cap);
  const int rounds_total = (nv + 63) >> 6;
  const int NWT = a.n_vslices * ST_WAVES;
  const int gw = vs * ST_WAVES + wave;
  int n_k = gw < rounds_total ? (rounds_total - gw + NWT - 1) / NWT : 0;
  if (n_k > KMAX) n_k = KMAX;             // cannot happen when the plan was made for vague_cap
  n_k = __builtin_amdgcn_readfirstlane(n_k);      // equal in all lanes of a wave; now the compiler knows
  const int turn = __builtin_amdgcn_readfirstlane(wave >> 2);   // waves i and i + 4 share a SIMD

  const size_t sk_unit = (size_t)unit * 4 * w * D;      // elements
  const unsigned char* skg = reinterpret_cast<const unsigned char*>((const bf16_t*)a.sk + sk_unit);
  const unsigned char* svg = reinterpret_cast<const unsigned char*>((const bf16_t*)a.sv + sk_unit);
  const int n_pieces = 4 * w * (R4_ROWB / 16);          // 16-byte pieces of a chunk

  __builtin_amdgcn_s_setprio(1);
  // ---- loads first: Vague positions of this wave's tokens and q ---------------
  int Jv[KMAX];
  const int32_t* vpos = a.vague_pos + (size_t)unit * a.vague_cap;
#pragma unroll
  for (int k = 0; k < KMAX; ++k) {
    const int tok = (gw + k * NWT) * 64 + lane;
    Jv[k] = (k < n_k && tok < nv) ? vpos[tok] : -1;
  }
  uint4 qv = make_uint4(0u, 0u, 0u, 0u);
  if (tid < G * 16)
    qv = reinterpret_cast<const uint4*>((const bf16_t*)a.q + ((size_t)b * d.Hq + (size_t)hk * G) * D)[tid];
  // Wait for them here, so that the hashes below do not have to wait for the chunk
  // copy that is started next: memory operations complete in order.
  __builtin_amdgcn_s_waitcnt(0x0F70);

  // ---- the first K chunk is on its way while the hashes are computed ----------
  stage_issue<R4_ROWB / 16, R4_ROWB>(skg, s_sk, n_pieces, 0, tid);

  uint2 info[KMAX];
#pragma unroll
  for (int k = 0; k < KMAX; ++k) {
    const int J = Jv[k];
    info[k] = (J >= 0) ? make_record<MODE>(d, w, J) : make_uint2(0u, 0u);
  }
  if (tid < G * 16) reinterpret_cast<uint4*>(s_q)[tid] = qv;

  // ---- K phases: logits -----------------------------------------------------
  // s[k][i]: token i of this lane's quad in round k, head (lane mod 4)
  float s[KMAX][4];
#pragma unroll
  for (int k = 0; k < KMAX; ++k)
#pragma unroll
    for (int i = 0; i < 4; ++i) s[k][i] = 0.f;

  const int sub = lane & 3, tl = lane >> 2;
  for (int cc = 0; cc < R4_NCHUNK; ++cc) {
    stage_wait();
    lds_barrier();                         // chunk cc is complete
    {
      uint2 qx[R4_NHP];
      int co[R4_NHP];
#pragma unroll
      for (int j = 0; j < R4_NHP; ++j) {
        const int hp = (tl + j) & (R4_NHP - 1);       // the block's half piece at step j
        co[j] = hp * 8;
        qx[j] = (sub < G) ? s_q[sub * 32 + cc * R4_NHP + hp] : make_uint2(0u, 0u);
      }
      KVR_DISPATCH_NK(n_k, (k_pass<NK, MODE>(s_sk, info, qx, co, turn, s)))
    }
    lds_barrier();                         // every wave is done with chunk cc
    if (cc + 1 < R4_NCHUNK) stage_issue<R4_ROWB / 16, R4_ROWB>(skg, s_sk, n_pieces, cc + 1, tid);
    else stage_issue<R4_ROWB / 16, R4_ROWB>(svg, s_sk, n_pieces, 0, tid);       // the first V chunk, under the softmax
  }

  // ---- softmax weights against the wave's own maximum ---------------------------
  // Lane (quad t, sub) holds the logits of the quad's 4 tokens for head `sub` (nothing
  // of use if there is no such head).
  const int tot_cap = a.ret_cap + a.vague_cap;
  const int unit_l = opaque_s(__builtin_amdgcn_readfirstlane(unit));
  const int gw_l = opaque_s(__builtin_amdgcn_readfirstlane(gw));
  const bool head_ok = sub < G;
  float mx = -__builtin_inff();
#pragma unroll
  for (int k = 0; k < KMAX; ++k) {
    if (k >= n_k) continue;                // uniform over the wave: rounds it does not have cost nothing
    const int tok0 = (gw_l + k * NWT) * 64 + (lane & ~3);        // first token of the quad in this round
    const int n_ok = nv - tok0;                                   // tokens i < n_ok of the quad exist
    float* lg = a.logits + ((size_t)unit_l * tot_cap + a.ret_cap + tok0) * G + sub;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const bool valid = i < n_ok;
      s[k][i] = valid ? s[k][i] * d.scale : -__builtin_inff();
      mx = fmaxf(mx, s[k][i]);
      if (a.logits != nullptr && valid && head_ok) lg[i * G] = s[k][i];
    }
  }
  // Weights are formed against the wave's own maximum, which needs no barrier; the
  // workgroup's maximum is put together after the barrier that publishes the first
  // V chunk, and each wave's sums are rescaled by exp(own maximum - workgroup
  // maximum) when they are merged.  s_stat: [8 waves][G] maxima, [8 waves][G] sums.
  {
    // maximum over the lanes of this head: the quads of a 16-lane row, then the four rows
    float x = dpp_max<0x124>(mx);
    x = dpp_max<0x128>(x);
    x = fmaxf(x, __shfl_xor(x, 16));
    x = fmaxf(x, __shfl_xor(x, 32));
    if (lane < G) s_stat[wave * G + lane] = x;
    float lsum = 0.f;
#pragma unroll
    for (int k = 0; k < KMAX; ++k) {
      if (k >= n_k) continue;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float p = (s[k][i] == -__builtin_inff()) ? 0.f : __expf(s[k][i] - x);
        s[k][i] = p;                 // from here on s holds the weights
        lsum += p;
      }
    }
    lsum = row_sum<4>(lsum);
    lsum += __shfl_xor(lsum, 16);
    lsum += __shfl_xor(lsum, 32);
    if (lane < G) s_stat[ST_WAVES * G + wave * G + lane] = lsum;
  }
  const size_t part = (size_t)unit_l * a.n_slices + a.n_rslices + opaque_s(__builtin_amdgcn_readfirstlane(vs));

  // ---- weights into matrix-core operand form ----------------------------------
  // The A operand of the V phases is, per lane, the weights of head `sub` for the
  // quad's 4 tokens: what the lane holds already.  The sign g_0 of each token (bit 0
  // of its record, which lives in the lane that owns the token) is folded in, the
  // weight is split into bf16 hi + lo (16 mantissa bits together), and the two
  // halves are packed as the two A operands of a round.
  uint32_t W[KMAX][4];
#pragma unroll
  for (int k = 0; k < KMAX; ++k) {
    W[k][0] = W[k][1] = W[k][2] = W[k][3] = 0u;
    if (k >= n_k) continue;
    const uint32_t rx = info[k].x;
    const uint32_t sg[4] = {quad_bcast<0>(rx) << 31, quad_bcast<1>(rx) << 31, quad_bcast<2>(rx) << 31,
                            quad_bcast<3>(rx) << 31};
    uint32_t hb[4], lb[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const float pt = head_ok ? __uint_as_float(__float_as_uint(s[k][t]) ^ sg[t]) : 0.f;
      hb[t] = __float_as_uint(pt) & 0xffff0000u;
      lb[t] = __float_as_uint(pt - __uint_as_float(hb[t]));
    }
    W[k][0] = pair_hi(hb[0], hb[1]);
    W[k][1] = pair_hi(hb[2], hb[3]);
    W[k][2] = pair_hi(lb[0], lb[1]);
    W[k][3] = pair_hi(lb[2], lb[3]);
  }

  // ---- V phases: weighted values ------------------------------------------------
  float* s_fw = s_stat + 2 * ST_WAVES * G;          // [8 waves][G]: exp(wave maximum - workgroup maximum)
  const int prow = wave * 4 + (lane >> 4);
  static_assert(G * R4_CH <= ST_THREADS, "one output element per thread and chunk");
  for (int cc = 0; cc < R4_NCHUNK; ++cc) {
    stage_wait();
    lds_barrier();             // V chunk cc complete; partial sums of chunk cc - 1 visible
    if (cc == 0) {
      // every wave's maximum and sum are visible now (this wave's own maximum is read
      // back too: it would not survive in registers without being spilled)
      float mo[G], mw[G], so[G];
#pragma unroll
      for (int g = 0; g < G; ++g) {
        mo[g] = s_stat[(lane & 7) * G + g];                          // maximum of wave (lane mod 8)
        so[g] = s_stat[ST_WAVES * G + (lane & 7) * G + g];           // its sum
        mw[g] = s_stat[wave * G + g];
      }
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float M = dpp_max<0x121>(mo[g]);
        M = dpp_max<0x122>(M);
        M = dpp_max<0x124>(M);                               // over 8 neighbouring lanes = all 8 waves
        if (lane == 0) s_fw[wave * G + g] = (mw[g] == -__builtin_inff()) ? 0.f : __expf(mw[g] - M);
        if (wave == 0) {
          float x = so[g] * ((mo[g] == -__builtin_inff()) ? 0.f : __expf(mo[g] - M));
          x = dpp_add<0x121>(x);
          x = dpp_add<0x122>(x);
          x = dpp_add<0x124>(x);                             // sum over the 8 waves
          if (lane == 0) {
            a.part_ml[(part * G + g) * 2] = M;
            a.part_ml[(part * G + g) * 2 + 1] = x;
          }
        }
      }
    } else if (tid < G * CH) {
      // chunk cc - 1's output element: the NROW rows of partial sums that the barrier just published
      const float* sp = s_part + ((cc - 1) & 1) * (R4_NROW * G * CH);
      float v = 0.f;
#pragma unroll
      for (int pr = 0; pr < R4_NROW; ++pr) v += sp[pr * G * CH + tid];
      a.part_o[part * G * D + (tid / CH) * D + (cc - 1) * CH + (tid % CH)] = v;
    }
    f32x4_t acc[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) acc[c] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    KVR_DISPATCH_NK(n_k, (v_pass<NK, MODE>(s_sk, info, W, sub * 8, turn, acc)))
    lds_barrier();                         // every wave is done with this V chunk
    if (cc + 1 < R4_NCHUNK) stage_issue<R4_ROWB / 16, R4_ROWB>(svg, s_sk, n_pieces, cc + 1, tid);

    // Reduction over the workgroup's tokens.  Lane (quad, sub) holds, per head, the 4
    // channels of half piece `sub` summed over the tokens of its quad; the four quads of
    // a 16-lane row are added with two DPP rotations, and the NROW rows meet in LDS.
    {
      float* sp = s_part + (cc & 1) * (R4_NROW * G * CH);
      float o[G][4];
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float f = s_fw[wave * G + g];
#pragma unroll
        for (int c = 0; c < 4; ++c) o[g][c] = row_sum<4>(acc[c][g]) * f;
      }
      if ((lane & 15) < 4) {
#pragma unroll
        for (int g = 0; g < G; ++g)
          *reinterpret_cast<float4*>(sp + (prow * G + g) * CH + sub * 4) = make_float4(o[g][0], o[g][1], o[g][2], o[g][3]);
      }
    }
  }
  lds_barrier();
  if (tid < G * CH) {
    const float* sp = s_part + ((R4_NCHUNK - 1) & 1) * (R4_NROW * G * CH);
    float v = 0.f;
#pragma unroll
    for (int pr = 0; pr < R4_NROW; ++pr) v += sp[pr * G * CH + tid];
    a.part_o[part * G * D + (tid / CH) * D + (R4_NCHUNK - 1) * CH + (tid % CH)] = v;
  }
}

template <int G, int MODE>
static hipError_t launch_r4(const DevDesc& d, const AttendArgs& a, const AttendPlan& plan, hipStream_t st) {
  auto kern = attend_vague_staged_r4_kernel<G, MODE>;
  static std::once_flag once;
  static hipError_t attr_rc = hipSuccess;
  std::call_once(once, [&]() {
    attr_rc = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  160 * 1024);
  });
  if (attr_rc != hipSuccess) return attr_rc;
  const int units = d.B * d.Hkv;
  const int units_pad = (units + 7) / 8 * 8;
  hipLaunchKernelGGL(kern, dim3(units_pad * plan.n_vslices), dim3(ST_THREADS), lds_need(d.w, G), st, d, a);
  return hipGetLastError();
}

template <int G>
static hipError_t launch_r4_mode(const DevDesc& d, const AttendArgs& a, const AttendPlan& plan, hipStream_t st) {
  return d.median_mode == KVR_MEDIAN_LOWER ? launch_r4<G, KVR_MEDIAN_LOWER>(d, a, plan, st)
                                           : launch_r4<G, KVR_MEDIAN_MIDMEAN>(d, a, plan, st);
}

bool staged_r4_applies(const DevDesc& d) {
  return d.r == 4 && 4 * d.w <= 4096 && d.G <= 4 && d.sign_mask == 2 && lds_need(d.w, d.G) <= (size_t)160 * 1024;
}

hipError_t launch_attend_vague_staged_r4(const DevDesc& d, const AttendArgs& a, const AttendPlan& plan,
                                         hipStream_t st) {
  if (!staged_r4_applies(d) || plan.n_vslices < 1) return hipErrorInvalidValue;    // 12-bit LDS row indices, LDS size
  switch (d.G) {
    case 1: return launch_r4_mode<1>(d, a, plan, st);
    case 2: return launch_r4_mode<2>(d, a, plan, st);
    case 4: return launch_r4_mode<4>(d, a, plan, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace kvr
