// kvr_attend_multi: the Calculation Phase for several query tokens at once (a
// chunk of prompt or of drafted tokens).  As the paper describes the phase, the
// cache of the layer is rebuilt once (Algorithm 4: retained tokens reused, Vague
// tokens queried from the sketch, Algorithm 2) and attention then runs over the
// rebuilt cache; with n_q queries per sequence the rebuild is shared by all of
// them, which is the point of batching them.
//
//   1. the dense kernel below runs over the retained slots,
//   2. the Vague index list goes through the LDS-staged kernel of
//      kvr_attend_multi_staged.hip when the sketch allows it (three rows, values
//      signed only, a 64-channel chunk fits LDS); else the dense kernel runs again
//      over the list: with three sketch rows it rebuilds each 16-token tile itself
//      (sketch rows gathered from L2, median by selection; a rebuilt piece serves
//      all columns and never reaches memory); otherwise
//      kvr_reconstruct's kernel first writes the rebuilt tokens to workspace (one
//      layer's worth) and the dense kernel reads them like retained rows,
//   3. the merge kernel of kvr_attend_decode combines the slice partials, writes
//      `out` and adds the probabilities to the cumulative scores.
//
// The dense kernel is the retained-slot kernel of kvr_attend_decode with the
// columns of its q.k matrix product fully used: column c = (query t, head g of the
// kv head's group), c = t * G + g, NCOL = n_q * G <= 16.  Per 16-token tile, four
// v_mfma_f32_16x16x32_bf16 with the K rows as the A operand and the NCOL query
// vectors as the B operand give lane l the logits of tokens 4 (l div 16) + {0..3}
// for column l mod 16.  Query t sits at position n_ctx - n_q + t and sees the
// tokens at positions up to its own; what it does not see gets the logit -inf.
// Online softmax per column.  p * v is a second matrix product per tile,
// out[column][channel] += P[column][token] V[token][channel], on
// v_mfma_f32_16x16x16_bf16: the weights a lane holds (its column, its four tokens)
// are already an A operand (split into bf16 hi + lo, 16 mantissa bits together);
// a lane's four V pieces (its four tokens, channels 8 (l mod 16) .. +7) give, one
// channel at a time, eight B operands after a 4 x 8 transpose in registers; the
// instruction for channel c of the pieces leaves lane l with the sums of columns
// 4 (l div 16) + {0..3} for channel 8 (l mod 16) + c.
#include "kvr_staged.h"

namespace kvr {

typedef __bf16 bf16x8m_t __attribute__((ext_vector_type(8)));
typedef float f32x4m_t __attribute__((ext_vector_type(4)));


// One call of the dense kernel: rows [0, cap) of k / v per unit, position of row
// s in pos (negative: empty), rows >= n_valid[unit] (if given) do not exist.
struct DenseArgs {
  const bf16_t* q;          // [B, n_q, Hq, D]
  const int32_t* n_ctx;     // [B]
  int n_q;
  const bf16_t* k;          // [units, cap, D]
  const bf16_t* v;
  const int32_t* pos;       // [units, cap]
  const int32_t* n_valid;   // [units] or null
  int cap;
  const bf16_t* sk;         // sketch mode: k and v are not read; the rows are rebuilt from the unit's
  const bf16_t* sv;         // sketches [units, 3, w, D] by Algorithm 2, tile by tile (three rows only)
  int slice_tokens, n_slices_here;
  int slice0, n_slices;     // partial index of this call's first slice / partials per unit
  int tok0, tot_cap;        // logits index of row 0 / logits rows per unit
  float* part_o;            // [units, n_slices, NCOL, D]
  float* part_ml;           // [units, n_slices, NCOL, 2]
  float* logits;            // [units, tot_cap, NCOL] or null
};

template <int NCOL, bool SKETCH>
__global__ __launch_bounds__(256) void attend_dense_multi_kernel(DevDesc d, DenseArgs a) {
  constexpr int NW = 4;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r16 = lane >> 4, col = lane & 15;
  const int n_items = d.B * d.Hkv * a.n_slices_here;
  const float NEG_INF = -__builtin_inff();
  __shared__ float s_acc[NW][NCOL][D];
  __shared__ float s_m[NW][NCOL], s_l[NW][NCOL];

  for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
    const int unit = item / a.n_slices_here, slice = item % a.n_slices_here;
    const int b = unit / d.Hkv, hk = unit % d.Hkv;
    const int rows = a.n_valid ? clampi(a.n_valid[unit], 0, a.cap) : a.cap;
    const int t_begin = slice * a.slice_tokens;
    const int t_end = min(t_begin + a.slice_tokens, rows);
    const bf16_t* kk = a.k + (size_t)unit * a.cap * D;
    const bf16_t* vv = a.v + (size_t)unit * a.cap * D;
    const int32_t* pp = a.pos + (size_t)unit * a.cap;
    float* logits_unit = a.logits ? a.logits + (size_t)unit * a.tot_cap * NCOL : nullptr;

    // this lane's column: query tq, head g
    const int tq = col / d.G, g = col % d.G;
    const bool col_live = col < NCOL;
    const int qpos = a.n_ctx[b] - a.n_q + tq;
    uint4 qb[4];
    {
      const bf16_t* q = a.q + (((size_t)b * a.n_q + (col_live ? tq : 0)) * d.Hq + (size_t)hk * d.G + (col_live ? g : 0)) * D + 8 * r16;
#pragma unroll
      for (int kx = 0; kx < 4; ++kx) {
        qb[kx] = *reinterpret_cast<const uint4*>(q + 32 * kx);
        if (!col_live) qb[kx] = make_uint4(0u, 0u, 0u, 0u);
      }
    }
    float m_run = NEG_INF, l_run = 0.f;
    f32x4_t acc[8];            // acc[c][i]: column 4 r16 + i, channel 8 col + c
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[c] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    const int n_tiles = (t_end > t_begin) ? (t_end - t_begin + 15) >> 4 : 0;
    for (int ti = wave; ti < n_tiles; ti += NW) {
      const int t0 = t_begin + ti * 16;
      // K: token t0 + col, channels 32 kx + 8 r16 .. +7;  V: token t0 + 4 r16 + j, channels 8 col .. +7
      uint4 ka[4], vt[4];
      int tpos[4];
      if constexpr (SKETCH) {
        // Lane (r16, col) hashes token t0 + col once: its three slots (16 bits each) and the
        // rows' signs for keys (bits 16..18 of y) and values (bits 19..21).  The K operand is
        // that token's; the V pieces belong to tokens t0 + 4 r16 + j, whose records sit in
        // lanes 4 r16 + j of this 16-lane row.
        const int tk = t0 + col;
        const int J = (tk < t_end) ? pp[min(tk, a.cap - 1)] : -1;
        uint32_t rx, ry;
        {
          const uint32_t h0 = (uint32_t)bucket_of(d, 0, J), h1 = (uint32_t)bucket_of(d, 1, J),
                         h2 = (uint32_t)bucket_of(d, 2, J);
          uint32_t sg = 0;
#pragma unroll
          for (int i = 0; i < 3; ++i) sg |= sign_neg(d, i, J) ? (1u << i) : 0u;
          rx = h0 | (h1 << 16);
          ry = h2 | (((d.sign_mask & 1) ? sg : 0u) << 16) | (((d.sign_mask & 2) ? sg : 0u) << 19);
        }
        const bf16_t* skk = a.sk + (size_t)unit * 3 * d.w * D;
        const bf16_t* svv = a.sv + (size_t)unit * 3 * d.w * D;
        {
          const int h[3] = {(int)(rx & 0xffffu), (int)(rx >> 16), (int)(ry & 0xffffu)};
          const uint32_t fl[3] = {(ry >> 16) & 1u ? 0x80008000u : 0u, (ry >> 17) & 1u ? 0x80008000u : 0u,
                                  (ry >> 18) & 1u ? 0x80008000u : 0u};
#pragma unroll
          for (int kx = 0; kx < 4; ++kx) ka[kx] = query_piece3(d, skk, h, fl, 32 * kx + 8 * r16);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int src = (lane & 48) + 4 * r16 + j;
          const uint32_t vx = (uint32_t)__shfl((int)rx, src), vy = (uint32_t)__shfl((int)ry, src);
          tpos[j] = __shfl(J, src);
          const int h[3] = {(int)(vx & 0xffffu), (int)(vx >> 16), (int)(vy & 0xffffu)};
          const uint32_t fl[3] = {(vy >> 19) & 1u ? 0x80008000u : 0u, (vy >> 20) & 1u ? 0x80008000u : 0u,
                                  (vy >> 21) & 1u ? 0x80008000u : 0u};
          vt[j] = query_piece3(d, svv, h, fl, 8 * col);
        }
      } else {
        const int tk = min(t0 + col, a.cap - 1);
#pragma unroll
        for (int kx = 0; kx < 4; ++kx) ka[kx] = *reinterpret_cast<const uint4*>(kk + (size_t)tk * D + 32 * kx + 8 * r16);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int tt = t0 + 4 * r16 + j;
          const int tc = min(tt, a.cap - 1);
          vt[j] = *reinterpret_cast<const uint4*>(vv + (size_t)tc * D + 8 * col);
          tpos[j] = (tt < t_end) ? pp[tc] : -1;
        }
      }
      f32x4m_t S = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kx = 0; kx < 4; ++kx)
        S = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8m_t, ka[kx]),
                                                    __builtin_bit_cast(bf16x8m_t, qb[kx]), S, 0, 0, 0);
      float s[4];
      bool invalid = false;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const bool ok = tpos[i] >= 0 && tpos[i] <= qpos && col_live;
        s[i] = ok ? S[i] * d.scale : NEG_INF;
        invalid = invalid || tpos[i] < 0;
      }
      if (logits_unit != nullptr && col_live) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int tt = t0 + 4 * r16 + i;
          if (tt < t_end) logits_unit[(size_t)(a.tok0 + tt) * NCOL + col] = s[i];
        }
      }
      float mx = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m_run, mx);
      if (__any(m_new > m_run)) {
        const float corr = (m_run == NEG_INF) ? 0.f : __expf(m_run - m_new);
        l_run *= corr;
        // this lane's accumulators belong to columns 4 r16 + i: their factors sit in
        // lanes 4 r16 + i of this 16-lane row
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float ci = __shfl(corr, (lane & 48) + 4 * r16 + i);
#pragma unroll
          for (int c = 0; c < 8; ++c) acc[c][i] *= ci;
        }
      }
      m_run = m_new;
      float p[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        p[i] = (s[i] == NEG_INF) ? 0.f : __expf(s[i] - m_new);
        l_run += p[i];
      }
      if (__any(invalid)) {           // an empty row may hold anything, even NaN: weight 0 is not enough
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (tpos[j] < 0) vt[j] = make_uint4(0u, 0u, 0u, 0u);
      }
      // weights as A operands: bf16 hi + lo of the four tokens of this lane's column
      uint32_t hb[4], lb[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        hb[i] = __float_as_uint(p[i]) & 0xffff0000u;
        lb[i] = __float_as_uint(p[i] - __uint_as_float(hb[i]));
      }
      const short4_t a_hi = pack_k4(pair_hi(hb[0], hb[1]), pair_hi(hb[2], hb[3]));
      const short4_t a_lo = pack_k4(pair_hi(lb[0], lb[1]), pair_hi(lb[2], lb[3]));
      // values as B operands: channel c of the four tokens' pieces
      short4_t bop[8];
      bop[0] = pack_k4(pair_lo(vt[0].x, vt[1].x), pair_lo(vt[2].x, vt[3].x));
      bop[1] = pack_k4(pair_hi(vt[0].x, vt[1].x), pair_hi(vt[2].x, vt[3].x));
      bop[2] = pack_k4(pair_lo(vt[0].y, vt[1].y), pair_lo(vt[2].y, vt[3].y));
      bop[3] = pack_k4(pair_hi(vt[0].y, vt[1].y), pair_hi(vt[2].y, vt[3].y));
      bop[4] = pack_k4(pair_lo(vt[0].z, vt[1].z), pair_lo(vt[2].z, vt[3].z));
      bop[5] = pack_k4(pair_hi(vt[0].z, vt[1].z), pair_hi(vt[2].z, vt[3].z));
      bop[6] = pack_k4(pair_lo(vt[0].w, vt[1].w), pair_lo(vt[2].w, vt[3].w));
      bop[7] = pack_k4(pair_hi(vt[0].w, vt[1].w), pair_hi(vt[2].w, vt[3].w));
#pragma unroll
      for (int c = 0; c < 8; ++c) acc[c] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a_hi, bop[c], acc[c], 0, 0, 0);
#pragma unroll
      for (int c = 0; c < 8; ++c) acc[c] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a_lo, bop[c], acc[c], 0, 0, 0);
    }

    // a lane's sums of weights cover its own four tokens of every tile: add the four 16-lane rows
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);

    __syncthreads();             // the previous item's readers are done with the LDS arrays
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int c_ = 4 * r16 + i;
      if (c_ < NCOL) {
#pragma unroll
        for (int c = 0; c < 8; ++c) s_acc[wave][c_][col * 8 + c] = acc[c][i];
      }
    }
    if (r16 == 0 && col_live) { s_m[wave][col] = m_run; s_l[wave][col] = l_run; }
    __syncthreads();
    const size_t part = (size_t)unit * a.n_slices + a.slice0 + slice;
    float* po = a.part_o + part * NCOL * D;
    float* pml = a.part_ml + part * NCOL * 2;
    for (int idx = threadIdx.x; idx < NCOL * D; idx += 256) {
      const int c_ = idx / D, c = idx % D;
      float M = s_m[0][c_];
#pragma unroll
      for (int w_ = 1; w_ < NW; ++w_) M = fmaxf(M, s_m[w_][c_]);
      float L = 0.f, O = 0.f;
#pragma unroll
      for (int w_ = 0; w_ < NW; ++w_) {
        const float e = (s_m[w_][c_] == NEG_INF) ? 0.f : __expf(s_m[w_][c_] - M);
        L += s_l[w_][c_] * e;
        O += s_acc[w_][c_][c] * e;
      }
      po[idx] = O;
      if (c == 0) { pml[c_ * 2] = M; pml[c_ * 2 + 1] = L; }
    }
  }
}

template <int NCOL>
static hipError_t launch_dense(const DevDesc& d, const DenseArgs& a, hipStream_t st) {
  const int n_wgs = d.B * d.Hkv * a.n_slices_here;
  if (n_wgs < 1) return hipSuccess;
  if (a.sk != nullptr)
    hipLaunchKernelGGL((attend_dense_multi_kernel<NCOL, true>), dim3(n_wgs), dim3(256), 0, st, d, a);
  else
    hipLaunchKernelGGL((attend_dense_multi_kernel<NCOL, false>), dim3(n_wgs), dim3(256), 0, st, d, a);
  return hipGetLastError();
}

static size_t align_up_m(size_t x, size_t a) { return (x + a - 1) / a * a; }

MultiPlan attend_multi_plan(const DevDesc& d, int n_q, long long ret_cap, long long vague_cap) {
  MultiPlan p;
  const long long units = (long long)d.B * d.Hkv;
  const int ncol = n_q * d.G;
  p.rslice_tokens = attend_slice_tokens(ret_cap, units);
  p.n_rslices = (int)((ret_cap + p.rslice_tokens - 1) / p.rslice_tokens);
  p.staged = vague_cap > 0 && multi_staged_applies(d, vague_cap);
  if (p.staged) p.vslice_tokens = multi_staged_part_tokens(vague_cap, units);
  else p.vslice_tokens = vague_cap > 0 ? attend_slice_tokens(vague_cap, units) : 64;
  p.n_vslices = vague_cap > 0 ? (int)((vague_cap + p.vslice_tokens - 1) / p.vslice_tokens) : 0;
  p.n_slices = p.n_rslices + p.n_vslices;
  // the staged kernel reads its scratch arrays (records in the first rebuilt-token area, partial logits in
  // the second, final logits) a few tiles past the end without clamping
  const size_t pad = p.staged ? (size_t)multi_staged_pad_tokens() * ncol * sizeof(float) : 0;
  size_t off = 0;
  p.off_khat = off;
  off = align_up_m(off + (size_t)units * vague_cap * D * sizeof(uint16_t) + pad, 256);
  p.off_vhat = off;
  off = align_up_m(off + (size_t)units * vague_cap * D * sizeof(uint16_t) + pad, 256);
  p.off_part_o = off;
  off = align_up_m(off + (size_t)units * p.n_slices * ncol * D * sizeof(float), 256);
  p.off_part_ml = off;
  off = align_up_m(off + (size_t)units * p.n_slices * ncol * 2 * sizeof(float), 256);
  p.off_logits = off;
  off = align_up_m(off + (size_t)units * (size_t)(ret_cap + vague_cap) * ncol * sizeof(float) + pad, 256);
  p.total_bytes = off;
  return p;
}

template <int NCOL>
static hipError_t launch_multi_n(const DevDesc& d, const AttendArgs& a0, const int32_t* n_ctx, int n_q,
                                 const MultiPlan& plan, void* ws, hipStream_t st) {
  char* base = (char*)ws;
  bf16_t* khat = (bf16_t*)(base + plan.off_khat);
  bf16_t* vhat = (bf16_t*)(base + plan.off_vhat);
  hipError_t e = hipSuccess;
  // three sketch rows: the dense kernel rebuilds the Vague tokens itself, tile by tile (each
  // rebuilt piece serves all columns of the tile and never reaches memory); otherwise
  // they go through the workspace
  const bool in_kernel = d.r == 3 && d.w <= 65535;
  if (a0.vague_cap > 0 && !in_kernel && !plan.staged) {
    e = launch_reconstruct(d, KVR_BF16, a0.sk, a0.sv, a0.vague_pos, a0.n_vague, a0.vague_cap, khat, vhat, st);
    if (e != hipSuccess) return e;
  }
  DenseArgs da;
  da.q = (const bf16_t*)a0.q;
  da.n_ctx = n_ctx;
  da.n_q = n_q;
  da.n_slices = plan.n_slices;
  da.tot_cap = a0.ret_cap + a0.vague_cap;
  da.part_o = (float*)(base + plan.off_part_o);
  da.part_ml = (float*)(base + plan.off_part_ml);
  da.logits = a0.scores ? (float*)(base + plan.off_logits) : nullptr;
  // retained slots
  da.k = (const bf16_t*)a0.k_ret;
  da.v = (const bf16_t*)a0.v_ret;
  da.sk = da.sv = nullptr;
  da.pos = a0.ret_pos;
  da.n_valid = nullptr;
  da.cap = a0.ret_cap;
  da.slice_tokens = plan.rslice_tokens;
  da.n_slices_here = plan.n_rslices;
  da.slice0 = 0;
  da.tok0 = 0;
  e = launch_dense<NCOL>(d, da, st);
  if (e != hipSuccess) return e;
  // rebuilt Vague tokens
  if (a0.vague_cap > 0 && plan.staged) {
    // the rebuilt-token areas of the workspace are free on this route: they hold the token records and
    // the logits after the first K chunk (8 + 4 NCOL <= 256 bytes per token)
    e = launch_attend_multi_staged(d, a0, n_ctx, n_q, plan.vslice_tokens, plan.n_vslices, plan.n_rslices,
                                   plan.n_slices, da.part_o, da.part_ml, (float*)(base + plan.off_logits), khat,
                                   vhat, st);
    if (e != hipSuccess) return e;
  } else if (a0.vague_cap > 0) {
    da.k = khat;
    da.v = vhat;
    if (in_kernel) {
      da.sk = (const bf16_t*)a0.sk;
      da.sv = (const bf16_t*)a0.sv;
    }
    da.pos = a0.vague_pos;
    da.n_valid = a0.n_vague;
    da.cap = a0.vague_cap;
    da.slice_tokens = plan.vslice_tokens;
    da.n_slices_here = plan.n_vslices;
    da.slice0 = plan.n_rslices;
    da.tok0 = a0.ret_cap;
    e = launch_dense<NCOL>(d, da, st);
    if (e != hipSuccess) return e;
  }
  AttendArgs a = a0;
  a.part_o = da.part_o;
  a.part_ml = da.part_ml;
  a.logits = da.logits;
  a.n_slices = plan.n_slices;
  a.n_q = n_q;
  return launch_attend_combine(d, a, NCOL, st);
}

hipError_t launch_attend_multi(const DevDesc& d, const AttendArgs& a, const int32_t* n_ctx, int n_q,
                               const MultiPlan& plan, void* ws, hipStream_t st) {
  switch (n_q * d.G) {
    case 1: return launch_multi_n<1>(d, a, n_ctx, n_q, plan, ws, st);
    case 2: return launch_multi_n<2>(d, a, n_ctx, n_q, plan, ws, st);
    case 4: return launch_multi_n<4>(d, a, n_ctx, n_q, plan, ws, st);
    case 8: return launch_multi_n<8>(d, a, n_ctx, n_q, plan, ws, st);
    case 16: return launch_multi_n<16>(d, a, n_ctx, n_q, plan, ws, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace kvr
