// Staged attention kernel over the Vague list, specialised for r = 3 sketch rows
// and a sketch narrow enough that 64 channels of all 3 w slots fit into LDS at
// once (the common case: w <= ~320).  Same contract and the same token -> wave
// mapping as the general staged kernel (kvr_attend_staged.hip); what differs:
//
//  * LDS latency is hidden inside each wave.  A workgroup owns its CU's LDS, so
//    only two waves share a SIMD and they cannot cover each other's LDS round
//    trips; every loop over pieces therefore runs as a software pipeline that
//    keeps the row reads of the next two pieces in flight while the medians and
//    dot products of the current one are computed.
//  * V phases work on quads: lanes 4t .. 4t+3 rebuild the 4 tokens that these
//    same lanes own (one piece per lane and pass, two passes), so a token's
//    hashes reach the quad by DPP quad broadcasts and its softmax weights are
//    brought into matrix-core operand form (4x4 transpose inside the quad,
//    sign g_0 folded in, bf16 hi + lo split) once, after the softmax, instead
//    of once per token and phase.  No LDS copy of the hashes is needed.
//  * Copies overlap: the first K chunk is fetched while the hashes are
//    computed, the first V chunk during the softmax, the second V chunk during
//    the reduction of the first (which has LDS scratch of its own).
#include "kvr_staged.h"

namespace kvr {

struct Rows3 {
  uint4 r0, r1, r2;
};

__device__ __forceinline__ void load_rows3(Rows3& o, const unsigned char* s_sk, const int (&rb)[3], int co) {
  o.r0 = *reinterpret_cast<const uint4*>(s_sk + rb[0] + co);
  o.r1 = *reinterpret_cast<const uint4*>(s_sk + rb[1] + co);
  o.r2 = *reinterpret_cast<const uint4*>(s_sk + rb[2] + co);
}

__device__ __forceinline__ uint4 median3(const Rows3& x) {
  return med3_piece(x.r0, x.r1, x.r2);
}

// value of lane J of this lane's quad
template <int J>
__device__ __forceinline__ uint32_t quad_bcast(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, J | (J << 2) | (J << 4) | (J << 6), 0xf, 0xf, true);
}
template <int J>
__device__ __forceinline__ float quad_bcast_f(float v) {
  return __uint_as_float(quad_bcast<J>(__float_as_uint(v)));
}

// value of lane (l ^ 4): neighbouring quads trade (row rotations by 12 and by 4,
// each written into the lanes where it is the wanted direction)
__device__ __forceinline__ float xchg4(float x) {
  const int v = __float_as_int(x);
  int r = __builtin_amdgcn_update_dpp(v, v, 0x12C, 0xf, 0x5, false);   // lanes 0-3, 8-11 of a row
  r = __builtin_amdgcn_update_dpp(r, v, 0x124, 0xf, 0xa, false);       // lanes 4-7, 12-15
  return __int_as_float(r);
}

// Byte addresses (relative to base) of a token's three rows for the 128-byte
// row pitch of this kernel, and the mask that flips the third listed row.
// A median does not care about the order of its arguments, so the record lists
// the rows in an order of its own: of the three signs g_0, g_1, g_2 at least two
// agree; that majority sign is folded into the token's softmax weight, and the
// row with the other sign (if there is one) is listed last, so that only one row
// ever has to be flipped.
__device__ __forceinline__ void rec_offsets(uint2 rec, int base, int (&rb)[3]) {
  rb[0] = (int)(rec.x & 0x1ff80u) + base;
  rb[1] = (int)(__builtin_amdgcn_ubfe(rec.x, 17, 10) << 7) + base;
  rb[2] = (int)(rec.y & 0x1ff80u) + base;
}
__device__ __forceinline__ uint32_t rec_flip2(uint2 rec) { return (uint32_t)((int)rec.y >> 31) & 0x80008000u; }

// V phases: the rows of one piece of token J of the quad, plus the mask that
// flips the last row relative to the other two
struct VItem {
  Rows3 rows;
  uint32_t fm2;
};

// What a lane derives from its own token's record for the V phases: the three
// row offsets and the flip mask.  The other lanes of the quad fetch them with
// quad broadcasts (DPP operands of the address additions and of the flips), so
// a record is taken apart once per quad instead of once per lane.
struct VOwn {
  int o0, o1, o2;
  uint32_t fm;
};
__device__ __forceinline__ VOwn v_own(uint2 rec) {
  int rb[3];
  rec_offsets(rec, 0, rb);
  return VOwn{rb[0], rb[1], rb[2], rec_flip2(rec)};
}

template <int J>
__device__ __forceinline__ void v_fetch(VItem& o, const VOwn& own, const unsigned char* s_sk, int co) {
  int rb[3];
  rb[0] = (int)quad_bcast<J>((uint32_t)own.o0) + co;
  rb[1] = (int)quad_bcast<J>((uint32_t)own.o1) + co;
  rb[2] = (int)quad_bcast<J>((uint32_t)own.o2) + co;
  o.fm2 = quad_bcast<J>(own.fm);
  load_rows3(o.rows, s_sk, rb, 0);
}

__device__ __forceinline__ uint4 v_median(const VItem& it) {
  Rows3 x;
  x.r0 = it.rows.r0;
  x.r1 = it.rows.r1;
  x.r2 = xor4(it.rows.r2, it.fm2);
  return median3(x);
}

// acc[c] (4 head sums of channel c of the piece) += weights (4 heads x 4 tokens,
// bf16 hi + lo) x values (4 tokens x 8 channels).  All hi products first, so
// that two matrix instructions on one accumulator are 8 instructions apart.
__device__ __forceinline__ void pv_piece(const uint4 (&med)[4], short4_t a_hi, short4_t a_lo, f32x4_t (&acc)[8]) {
  short4_t be[4], bo[4];
  be[0] = pack_k4(pair_lo(med[0].x, med[1].x), pair_lo(med[2].x, med[3].x));
  bo[0] = pack_k4(pair_hi(med[0].x, med[1].x), pair_hi(med[2].x, med[3].x));
  be[1] = pack_k4(pair_lo(med[0].y, med[1].y), pair_lo(med[2].y, med[3].y));
  bo[1] = pack_k4(pair_hi(med[0].y, med[1].y), pair_hi(med[2].y, med[3].y));
  be[2] = pack_k4(pair_lo(med[0].z, med[1].z), pair_lo(med[2].z, med[3].z));
  bo[2] = pack_k4(pair_hi(med[0].z, med[1].z), pair_hi(med[2].z, med[3].z));
  be[3] = pack_k4(pair_lo(med[0].w, med[1].w), pair_lo(med[2].w, med[3].w));
  bo[3] = pack_k4(pair_hi(med[0].w, med[1].w), pair_hi(med[2].w, med[3].w));
#pragma unroll
  for (int dw = 0; dw < 4; ++dw) {
    acc[2 * dw] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(a_hi, be[dw], acc[2 * dw], 0, 0, 0);
    acc[2 * dw + 1] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(a_hi, bo[dw], acc[2 * dw + 1], 0, 0, 0);
  }
#pragma unroll
  for (int dw = 0; dw < 4; ++dw) {
    acc[2 * dw] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(a_lo, be[dw], acc[2 * dw], 0, 0, 0);
    acc[2 * dw + 1] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(a_lo, bo[dw], acc[2 * dw + 1], 0, 0, 0);
  }
}

// The same value, but the compiler can no longer tell: whatever is derived from
// it is computed where it is used instead of once per kernel and kept in
// registers through all phases (the row offsets of every round would be).
__device__ __forceinline__ uint2 opaque(uint2 v) {
  asm volatile("" : "+v"(v.x), "+v"(v.y));
  return v;
}
// same for a wave-uniform integer: addresses built from it are formed where they
// are needed instead of at the top of the kernel (where they would be spilled)
__device__ __forceinline__ int opaque_s(int v) {
  asm volatile("" : "+s"(v));
  return v;
}

// Nothing may be moved across this point by the instruction scheduler: keeps the
// row reads of later pieces ahead of the arithmetic of the current one.
#define KVR_PIN() __builtin_amdgcn_sched_barrier(0)

// The two waves that share a SIMD take turns in having the higher issue
// priority, round by round (turn is even for one of them and odd for the
// other).  Left alone, the older wave wins every arbitration, finishes a phase
// far ahead of the younger one and idles at the barrier while the younger one
// runs alone, with nobody to cover its latencies.
// Both levels are above the default 0, at which the retained-slot kernel runs
// when it shares the CU: its waves stream from HBM and need few issue slots, and
// every slot they win from a wave of this kernel delays a whole workgroup at the
// next barrier.
__device__ __forceinline__ void take_turn(int t) {
  if (t & 1) __builtin_amdgcn_s_setprio(2);
  else __builtin_amdgcn_s_setprio(1);
}

// K phase on the matrix cores.  One lane = one token; v_mfma_f32_4x4x4 works on
// blocks of 4 lanes and multiplies a 4 x 4 matrix A (row i from lane i of the
// block: here 4 channels of q for head i) with B (column j from lane j: 4
// channels of the token rebuilt by lane j); lane j receives the 4 head sums of
// its token.  All columns of a block must therefore hold the same channels,
// while LDS wants neighbouring lanes on different 16-byte pieces.  Compromise:
// the two lanes of a pair share the piece ((lane / 2 + step) mod 8), so 16
// neighbouring lanes still cover all 8 pieces (and the 2 x 8 bank groups of
// the 256-byte LDS line, unless both tokens of a pair sit in rows of equal
// parity), and every block issues each product twice, once with q for the
// piece of its first pair and once for its second pair; a lane keeps the sum
// that was formed with its own pair's channels.
//
// qx[j]: q of head (lane mod 4) for the piece that the block's first pair reads
// at step j; the second pair reads the piece one further, i.e. qx[(j + 1) mod 8].
template <int NK, int G>
__device__ __forceinline__ void k_pass(const unsigned char* s_sk, const uint2 (&info)[ST_KMAX],
                                       const uint4 (&qx)[8], const int (&co)[8], bool second_pair,
                                       int turn, float (&s)[ST_KMAX][G]) {
  // Three-stage pipeline over the steps t = 8 k + j of all rounds: at step t the
  // rows of step t + 3 are requested, the medians of step t + 1 are formed, and
  // the matrix instructions of step t run on medians formed one step earlier.
  Rows3 buf[3];                          // rows of step t live in buf[t % 3]
  int rb[3];
  rec_offsets(opaque(info[0]), 0, rb);
  load_rows3(buf[0], s_sk, rb, co[0]);
  load_rows3(buf[1], s_sk, rb, co[1]);
  load_rows3(buf[2], s_sk, rb, co[2]);
  uint4 m[2];                            // medians of step t in m[t % 2]
  m[0] = median3(buf[0]);
#pragma unroll
  for (int k = 0; k < NK; ++k) {
    int rn[3] = {0, 0, 0};
    if (k + 1 < NK) rec_offsets(opaque(info[k + 1]), 0, rn);
    f32x4_t ax = {0.f, 0.f, 0.f, 0.f}, ay = {0.f, 0.f, 0.f, 0.f};
    take_turn(k + turn);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int t = 8 * k + j;
      if (j < 5) load_rows3(buf[(t + 3) % 3], s_sk, rb, co[j + 3]);
      else if (k + 1 < NK) load_rows3(buf[(t + 3) % 3], s_sk, rn, co[j - 5]);
      KVR_PIN();
      if (j < 7 || k + 1 < NK) m[(t + 1) & 1] = median3(buf[(t + 1) % 3]);
      KVR_PIN();
      const uint4 mc = m[t & 1];
      const short4_t b_lo = pack_k4(mc.x, mc.y), b_hi = pack_k4(mc.z, mc.w);
      const uint4 qa = qx[j], qb = qx[(j + 1) & 7];
      ax = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(pack_k4(qa.x, qa.y), b_lo, ax, 0, 0, 0);
      ay = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(pack_k4(qb.x, qb.y), b_lo, ay, 0, 0, 0);
      ax = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(pack_k4(qa.z, qa.w), b_hi, ax, 0, 0, 0);
      ay = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(pack_k4(qb.z, qb.w), b_hi, ay, 0, 0, 0);
      KVR_PIN();
    }
#pragma unroll
    for (int g = 0; g < G; ++g) s[k][g] += second_pair ? ay[g] : ax[g];
    rb[0] = rn[0]; rb[1] = rn[1]; rb[2] = rn[2];
  }
  __builtin_amdgcn_s_setprio(1);
}

// One V pass over NK rounds for the piece at byte offset co of each row: the
// quad's 4 tokens per round, same pipeline, then the matrix instructions.
template <int NK>
__device__ __forceinline__ void v_pass(const unsigned char* s_sk, const uint2 (&info)[ST_KMAX],
                                       const uint32_t (&W)[ST_KMAX][4], int co, int turn, f32x4_t (&acc)[8]) {
  VItem buf[4];
  VOwn own = v_own(info[0]);
  v_fetch<0>(buf[0], own, s_sk, co);
  v_fetch<1>(buf[1], own, s_sk, co);
#pragma unroll
  for (int k = 0; k < NK; ++k) {
    uint4 med[4];
    take_turn(k + turn);
    v_fetch<2>(buf[2], own, s_sk, co);
    KVR_PIN();
    med[0] = v_median(buf[0]);
    KVR_PIN();
    v_fetch<3>(buf[3], own, s_sk, co);
    if (k + 1 < NK) own = v_own(info[k + 1]);
    KVR_PIN();
    med[1] = v_median(buf[1]);
    KVR_PIN();
    if (k + 1 < NK) v_fetch<0>(buf[0], own, s_sk, co);
    KVR_PIN();
    med[2] = v_median(buf[2]);
    KVR_PIN();
    if (k + 1 < NK) v_fetch<1>(buf[1], own, s_sk, co);
    KVR_PIN();
    med[3] = v_median(buf[3]);
    pv_piece(med, pack_k4(W[k][0], W[k][1]), pack_k4(W[k][2], W[k][3]), acc);
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
    default: break;              \
  }
static_assert(ST_KMAX == 6, "KVR_DISPATCH_NK covers 1..6 rounds");

template <int G>
// Register cap: 192 per lane (the attribute counts in units of two on this target).  Two
// waves of this kernel and one wave of the retained-slot kernel in its 128-register form
// then fill a SIMD's 512 registers exactly, which is what lets the two kernels run side by
// side on a CU.
__global__ __launch_bounds__(ST_THREADS) __attribute__((amdgpu_num_vgpr(96))) void attend_vague_staged64_kernel(
    DevDesc d, AttendArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  constexpr int R = 3, CH = 64, NC = 8, ROWB = 128, ROWB_LOG2 = 7, NPH = D / CH, KMAX = ST_KMAX;
  constexpr int NROW = ST_WAVES * 4;         // 16-lane rows per workgroup

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
  const int sk_bytes = (R * w * ROWB + 1023) & ~1023;
  unsigned char* s_sk = smem;                                             // one 64-channel chunk
  float* s_part = reinterpret_cast<float*>(smem + sk_bytes);              // [NROW][G][CH]
  float* s_stat = s_part + NROW * G * CH;                                 // [2][NROW][G] floats of room
  uint4* s_q = reinterpret_cast<uint4*>(s_stat + 2 * NROW * G);           // [G][16]

  const int nv = clampi(a.n_vague[unit], 0, a.vague_cap);
  const int rounds_total = (nv + 63) >> 6;
  const int NWT = a.n_vslices * ST_WAVES;
  const int gw = vs * ST_WAVES + wave;
  int n_k = gw < rounds_total ? (rounds_total - gw + NWT - 1) / NWT : 0;
  if (n_k > KMAX) n_k = KMAX;             // cannot happen when the plan was made for vague_cap
  n_k = __builtin_amdgcn_readfirstlane(n_k);      // equal in all lanes of a wave; now the compiler knows
  const int turn = __builtin_amdgcn_readfirstlane(wave >> 2);   // waves i and i + 4 share a SIMD

  const size_t sk_unit = (size_t)unit * R * w * D;      // elements
  const unsigned char* skg = reinterpret_cast<const unsigned char*>((const bf16_t*)a.sk + sk_unit);
  const unsigned char* svg = reinterpret_cast<const unsigned char*>((const bf16_t*)a.sv + sk_unit);
  const int n_pieces = R * w * NC;

  __builtin_amdgcn_s_setprio(1);
  // ---- loads first: Vague positions of this wave's tokens, q, and a touch of
  //      this workgroup's share of the unit's two sketches (so that the later
  //      chunks' lines are in L2 when their turn comes) ----------------------------
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
  // Wait for them here (vmcnt(0), as an instruction the compiler's wait-count
  // bookkeeping sees), so that the hashes below do not have to wait for the
  // chunk copy that is started next: memory operations complete in order.
  __builtin_amdgcn_s_waitcnt(0x0F70);

  // ---- the first K chunk is on its way while the hashes are computed ----------
  stage_issue<NC, ROWB>(skg, s_sk, n_pieces, 0, tid);

  // ---- hash every token once (kept in registers); q to LDS -------------------
  uint2 info[KMAX];
  uint32_t vmask = 0;
#pragma unroll
  for (int k = 0; k < KMAX; ++k) {
    const int J = Jv[k];
    uint2 pk = make_uint2(0u, 0u);
    if (J >= 0) {
      // token record (2 dwords), laid out so that every field is one or two
      // instructions away from its use: LDS row indices (< 1024 here) sit at
      // bit 7 (first listed row: x[7..16], third: y[7..16]) or at bit 17 (second:
      // x[17..26]); bit 0 of x is the majority sign of g_0, g_1, g_2 (1 = minus),
      // bit 31 of y says whether the third listed row has the other sign.  The
      // row whose sign differs from the other two, if any, is listed third.
      const uint32_t r0 = (uint32_t)bucket_of(d, 0, J), r1 = (uint32_t)(w + bucket_of(d, 1, J)),
                     r2 = (uint32_t)(2 * w + bucket_of(d, 2, J));
      const uint32_t s0 = sign_neg(d, 0, J) ? 1u : 0u, s1 = sign_neg(d, 1, J) ? 1u : 0u,
                     s2 = sign_neg(d, 2, J) ? 1u : 0u;
      const uint32_t maj = (s0 & s1) | (s0 & s2) | (s1 & s2);
      // the odd one out: row 0 if s0 != maj, else row 1 if s1 != maj, else row 2 (flipped or not)
      const bool odd0 = s0 != maj, odd1 = s1 != maj;
      const uint32_t ra = odd0 ? r2 : r0;                    // first listed
      const uint32_t rbk = odd1 ? r2 : r1;                   // second listed
      const uint32_t rc = odd0 ? r0 : (odd1 ? r1 : r2);      // third listed
      const uint32_t flip = (s0 ^ s1) | (s0 ^ s2);           // 1 iff the signs are not all equal
      pk = make_uint2((ra << 7) | (rbk << 17) | maj, (rc << 7) | (flip << 31));
      vmask |= 1u << k;
    }
    info[k] = pk;
  }
  asm volatile("" ::"v"(touched));       // the touch load has no other use: keep it
  if (tid < G * 16) s_q[tid] = qv;
  stage_wait();
  lds_barrier();

  // ---- K phases: logits -----------------------------------------------------
  float s[KMAX][G];
#pragma unroll
  for (int k = 0; k < KMAX; ++k)
#pragma unroll
    for (int g = 0; g < G; ++g) s[k][g] = 0.f;

  for (int cc = 0; cc < NPH; ++cc) {
    if (cc > 0) {
      lds_barrier();
      stage_issue<NC, ROWB>(skg, s_sk, n_pieces, cc, tid);
      stage_wait();
      lds_barrier();
    }
    {
      const int head = lane & 3, pair = lane >> 1, blk2 = (lane >> 2) * 2;
      uint4 qx[8];
      int co[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        co[j] = ((pair + j) & 7) * 16;
        qx[j] = (head < G) ? s_q[head * 16 + cc * NC + ((blk2 + j) & 7)] : make_uint4(0u, 0u, 0u, 0u);
      }
      const bool second_pair = (lane & 2) != 0;
      KVR_DISPATCH_NK(n_k, (k_pass<NK, G>(s_sk, info, qx, co, second_pair, turn, s)))
    }
  }

  // ---- the first V chunk is on its way during the softmax ----------------------
  lds_barrier();                           // every wave is done with the K chunk
  stage_issue<NC, ROWB>(svg, s_sk, n_pieces, 0, tid);

  // ---- softmax weights against the workgroup's own maximum -------------------
  const int tot_cap = a.ret_cap + a.vague_cap;
  const int unit_l = opaque_s(__builtin_amdgcn_readfirstlane(unit));
  const int gw_l = opaque_s(__builtin_amdgcn_readfirstlane(gw));
  float mx[G];
#pragma unroll
  for (int g = 0; g < G; ++g) mx[g] = -__builtin_inff();
#pragma unroll
  for (int k = 0; k < KMAX; ++k) {
    if (k >= n_k) break;                   // uniform over the wave: rounds it does not have cost nothing
    const bool valid = (vmask >> k) & 1u;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      s[k][g] = valid ? s[k][g] * d.scale : -__builtin_inff();
      mx[g] = fmaxf(mx[g], s[k][g]);
    }
    if (a.logits != nullptr && valid) {
      const int tok = (gw_l + k * NWT) * 64 + lane;
      float* lg = a.logits + ((size_t)unit_l * tot_cap + a.ret_cap + tok) * G;
      if constexpr (G == 4) {
        *reinterpret_cast<float4*>(lg) = make_float4(s[k][0], s[k][1], s[k][2], s[k][3]);
      } else {
#pragma unroll
        for (int g = 0; g < G; ++g) lg[g] = s[k][g];
      }
    }
  }
  // Weights are formed against the wave's own maximum, which needs no barrier; the
  // workgroup's maximum is put together after the barrier that publishes the first
  // V chunk, and each wave's sums are rescaled by exp(own maximum - workgroup
  // maximum) when they are merged.  s_stat: [8 waves][G] maxima, [NROW][G] row sums.
  const int prow = wave * 4 + (lane >> 4);
  float lsum[G];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float x = row_max(mx[g]);
    x = fmaxf(x, __shfl_xor(x, 16));
    x = fmaxf(x, __shfl_xor(x, 32));
    if (lane == 0) s_stat[wave * G + g] = x;
    lsum[g] = 0.f;
#pragma unroll
    for (int k = 0; k < KMAX; ++k) {
      if (k >= n_k) break;
      const float p = (s[k][g] == -__builtin_inff()) ? 0.f : __expf(s[k][g] - x);
      s[k][g] = p;                 // from here on s holds the weights
      lsum[g] += p;
    }
  }
#pragma unroll
  for (int g = 0; g < G; ++g) {
    lsum[g] = row_sum<1>(lsum[g]);
    if ((lane & 15) == 0) s_stat[ST_WAVES * G + prow * G + g] = lsum[g];
  }
  const size_t part = (size_t)unit_l * a.n_slices + a.n_rslices + opaque_s(__builtin_amdgcn_readfirstlane(vs));

  // ---- weights into matrix-core operand form ----------------------------------
  // Lane `sub` of quad t needs, for the quad's 4 tokens, the weight of head
  // `sub` (zero if there is no such head), with the sign g_0 of the token folded
  // in: a 4x4 transpose inside the quad.  Split into bf16 hi + lo (16 mantissa
  // bits together) and packed as the two A operands of a round.
  const int sub = lane & 3, tl = lane >> 2;
  uint32_t W[KMAX][4];
#pragma unroll
  for (int k = 0; k < KMAX; ++k) {
    W[k][0] = W[k][1] = W[k][2] = W[k][3] = 0u;
    if (k >= n_k) continue;
    const uint32_t sgn = info[k].x << 31;
    float pf[G];
#pragma unroll
    for (int g = 0; g < G; ++g) pf[g] = __uint_as_float(__float_as_uint(s[k][g]) ^ sgn);
    float T[4];
#define KVR_TRANSPOSE_COL(J)                                          \
  {                                                                   \
    float t = quad_bcast_f<J>(pf[0]);                                 \
    if constexpr (G > 1) { const float u = quad_bcast_f<J>(pf[1]); t = (sub == 1) ? u : t; } \
    if constexpr (G > 2) { const float u = quad_bcast_f<J>(pf[2]); t = (sub == 2) ? u : t; } \
    if constexpr (G > 3) { const float u = quad_bcast_f<J>(pf[3]); t = (sub == 3) ? u : t; } \
    T[J] = (sub < G) ? t : 0.f;                                       \
  }
    KVR_TRANSPOSE_COL(0)
    KVR_TRANSPOSE_COL(1)
    KVR_TRANSPOSE_COL(2)
    KVR_TRANSPOSE_COL(3)
#undef KVR_TRANSPOSE_COL
    uint32_t hb[4], lb[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      hb[t] = __float_as_uint(T[t]) & 0xffff0000u;
      lb[t] = __float_as_uint(T[t] - __uint_as_float(hb[t]));
    }
    W[k][0] = pair_hi(hb[0], hb[1]);
    W[k][1] = pair_hi(hb[2], hb[3]);
    W[k][2] = pair_hi(lb[0], lb[1]);
    W[k][3] = pair_hi(lb[2], lb[3]);
  }

  // ---- V phases: weighted values ------------------------------------------------
  // the two pieces of this lane: odd quads take them in the opposite order, so
  // that 8 neighbouring lanes always cover 8 different 16-byte bank groups
  const int pa = sub + ((tl & 1) ? 4 : 0);
  const int pb = sub + ((tl & 1) ? 0 : 4);
  float* s_fw = s_stat + (ST_WAVES + NROW) * G;     // [8 waves][G]: exp(wave maximum - workgroup maximum)
  float pend_v = 0.f;                      // chunk 0's output element of this thread, stored one barrier later
  for (int cc = 0; cc < NPH; ++cc) {
    stage_wait();
    lds_barrier();
    if (cc == 0) {
      // every wave's maximum and row sums are visible now (this wave's own maximum is
      // read back too: it would not survive in registers without being spilled)
      float mo[G], mw[G], mr[G], sr[G];
#pragma unroll
      for (int g = 0; g < G; ++g) {
        mo[g] = s_stat[(lane & 7) * G + g];                          // maximum of wave (lane mod 8)
        mw[g] = s_stat[wave * G + g];
        // lane l < 32 takes row l, which belongs to wave l / 4
        mr[g] = s_stat[((lane & (NROW - 1)) >> 2) * G + g];
        sr[g] = s_stat[ST_WAVES * G + (lane & (NROW - 1)) * G + g];
      }
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float M = dpp_max<0x121>(mo[g]);
        M = dpp_max<0x122>(M);
        M = dpp_max<0x124>(M);                               // over 8 neighbouring lanes = all 8 waves
        // kept in LDS rather than in registers through the V phases; only this wave reads it back
        if (lane == 0) s_fw[wave * G + g] = (mw[g] == -__builtin_inff()) ? 0.f : __expf(mw[g] - M);
        if (wave == 0) {
          const float fr = (mr[g] == -__builtin_inff()) ? 0.f : __expf(mr[g] - M);
          float x = row_sum<1>(sr[g] * fr);
          x += __shfl_xor(x, 16);
          if (lane == 0) {
            a.part_ml[(part * G + g) * 2] = M;
            a.part_ml[(part * G + g) * 2 + 1] = x;
          }
        }
      }
    } else if (tid < G * CH) {
      // chunk cc - 1's element; its latency now hides under this chunk's arithmetic
      a.part_o[part * G * D + (tid / CH) * D + (cc - 1) * CH + (tid % CH)] = pend_v;
    }
    // One accumulator set serves both passes.  Pass 0 sums piece pa of the quad's
    // own tokens; then neighbouring quads (lane ^ 4) trade accumulators, so that
    // every lane now holds its neighbour's sums for the piece it takes in pass 1
    // (pb of an even quad = pa of the odd quad next to it, and vice versa), and
    // pass 1 adds the own tokens' share of that piece on top.
    f32x4_t acc[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[c] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    KVR_DISPATCH_NK(n_k, (v_pass<NK>(s_sk, info, W, pa * 16, turn, acc)))
#pragma unroll
    for (int c = 0; c < 8; ++c)
#pragma unroll
      for (int g = 0; g < 4; ++g) acc[c][g] = xchg4(acc[c][g]);
    KVR_DISPATCH_NK(n_k, (v_pass<NK>(s_sk, info, W, pb * 16, turn + 1, acc)))
    lds_barrier();                         // every wave is done with this V chunk
    if (cc + 1 < NPH) stage_issue<NC, ROWB>(svg, s_sk, n_pieces, cc + 1, tid);

    // Reduction over the workgroup's tokens.  Lane (quad, sub) holds, per head,
    // the 8 channels of piece pb summed over the tokens of its quad and of the
    // neighbouring quad; lanes l and l + 8 of a 16-lane row hold the same piece
    // (one DPP rotation adds them), and the NROW rows meet in LDS.
    if constexpr (true) {
      float o[G][8];
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float f = s_fw[wave * G + g];
#pragma unroll
        for (int c = 0; c < 8; ++c) o[g][c] = dpp_add<0x128>(acc[c][g]) * f;
      }
      if ((lane & 15) < 8) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
          float* dst = s_part + (prow * G + g) * CH + pb * 8;
          *reinterpret_cast<float4*>(dst) = make_float4(o[g][0], o[g][1], o[g][2], o[g][3]);
          *reinterpret_cast<float4*>(dst + 4) = make_float4(o[g][4], o[g][5], o[g][6], o[g][7]);
        }
      }
    }
    lds_barrier();
    static_assert(G * CH <= ST_THREADS, "one output element per thread and chunk");
    if (tid < G * CH) {
      float v = 0.f;
#pragma unroll
      for (int pr = 0; pr < NROW; ++pr) v += s_part[pr * G * CH + tid];
      // The wait before the next barrier would also wait for this store: all but the
      // last chunk's element are held back until that barrier has passed.
      if (cc + 1 < NPH) pend_v = v;
      else a.part_o[part * G * D + (tid / CH) * D + cc * CH + (tid % CH)] = v;
    }
    // the next iteration's barrier (after its stage_wait) orders these reads
    // before the next writes into s_part
  }
}

template <int G>
static hipError_t launch64(const DevDesc& d, const AttendArgs& a, const AttendPlan& plan, hipStream_t st) {
  auto kern = attend_vague_staged64_kernel<G>;
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

hipError_t launch_attend_vague_staged64(const DevDesc& d, const AttendArgs& a, const AttendPlan& plan,
                                        hipStream_t st) {
  if (d.r != 3 || plan.ch != 64 || 3 * d.w > 1024) return hipErrorInvalidValue;   // 10-bit LDS row indices
  // LDS: chunk + [32][G][64] floats + statistics + q; the plan reserves at least that
  const size_t need = (((size_t)3 * d.w * 128 + 1023) & ~(size_t)1023) + (size_t)32 * d.G * 64 * 4 +
                      (size_t)2 * 32 * d.G * 4 + (size_t)d.G * 256;
  if (need > (size_t)plan.lds_bytes) return hipErrorInvalidValue;
  switch (d.G) {
    case 1: return launch64<1>(d, a, plan, st);
    case 2: return launch64<2>(d, a, plan, st);
    case 4: return launch64<4>(d, a, plan, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace kvr
