// Attention over the retained slots (raw Recent + Candidate tokens), bf16.
//
// This part of the step is a plain stream over HBM: every retained K and V row
// is read exactly once.  q.k for the G query heads of the kv head is a small
// dense contraction and goes to the matrix cores: per 16-token tile, four
// v_mfma_f32_16x16x32_bf16 with the K rows as the A operand (lane l supplies
// token l mod 16, channels 8 (l div 16) .. +7 of each 32-channel block) and q as
// the B operand (column n = head n, zero for n >= G).  The result leaves lane l
// with the logits of tokens 4 (l div 16) + {0,1,2,3} for head l mod 16.  The V
// rows are loaded so that lane l holds channels 8 (l mod 16) .. +7 of exactly
// those four tokens; the weight of (token, head g) then sits in lane g of the
// same 16-lane row and is fetched with a DPP row broadcast.  p * v is
// accumulated in float32 on the vector ALUs (an MFMA would need V transposed).
// Online softmax per wave; the four waves of a workgroup are merged through LDS
// into one partial per slice.
//
// A workgroup walks over (unit, slice) items with a grid stride, so the launch
// can be as wide as the item count (stand-alone: many workgroups per CU hide the
// HBM latency) or as narrow as one workgroup per CU (next to the staged kernel,
// whose registers and LDS leave room for exactly that).
#include "kvr_launch.h"

namespace kvr {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

// value held by lane N of the caller's 16-lane row
template <int N>
__device__ __forceinline__ float row_bcast(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x150 + N, 0xf, 0xf, true));
}

template <int G, int I>
struct AccStep {
  __device__ static __forceinline__ void fma(float (&acc)[G][8], float p, const float (&v)[8]) {
    const float pg = row_bcast<I>(p);
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[I][c] = fmaf(pg, v[c], acc[I][c]);
    AccStep<G, I + 1>::fma(acc, p, v);
  }
  __device__ static __forceinline__ void scale(float (&acc)[G][8], float corr) {
    const float cg = row_bcast<I>(corr);
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[I][c] *= cg;
    AccStep<G, I + 1>::scale(acc, corr);
  }
};
template <int G>
struct AccStep<G, G> {
  __device__ static __forceinline__ void fma(float (&)[G][8], float, const float (&)[8]) {}
  __device__ static __forceinline__ void scale(float (&)[G][8], float) {}
};

struct RetTile {
  uint4 ka[4];   // K: token t0 + (lane mod 16), channels 32 kk + 8 (lane div 16) .. +7
  uint4 vv[4];   // V: token t0 + 4 (lane div 16) + j, channels 8 (lane mod 16) .. +7
  int pos[4];    // position of token t0 + 4 (lane div 16) + j, -1 = empty slot / past the slice
};

// 16 bytes that are read exactly once: non-temporal, so that the stream does not
// push the sketch (which the staged kernel reads many times) out of L2
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 stream_load16(const bf16_t* p) {
  const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(v[0], v[1], v[2], v[3]);
}

__device__ __forceinline__ void load_tile(RetTile& t, const bf16_t* __restrict__ kret,
                                          const bf16_t* __restrict__ vret, const int32_t* __restrict__ rp,
                                          int t0, int t_end, int ret_cap, int r16, int col) {
  const int tk = min(t0 + col, ret_cap - 1);
#pragma unroll
  for (int kk = 0; kk < 4; ++kk)
    t.ka[kk] = stream_load16(kret + (size_t)tk * D + 32 * kk + 8 * r16);
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int tt = t0 + 4 * r16 + j;
    const int tc = min(tt, ret_cap - 1);
    t.vv[j] = stream_load16(vret + (size_t)tc * D + 8 * col);
    t.pos[j] = (tt < t_end) ? (rp ? rp[tc] : tt) : -1;
  }
}

template <int G>
__device__ __forceinline__ void compute_tile(const RetTile& t, const uint4 (&qb)[4], float scale, int t0,
                                             int t_end, int r16, int col, float* __restrict__ logits_unit,
                                             float& m_run, float& l_run, float (&acc)[G][8]) {
  const float NEG_INF = -__builtin_inff();
  f32x4_t S = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int kk = 0; kk < 4; ++kk)
    S = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, t.ka[kk]),
                                                __builtin_bit_cast(bf16x8_t, qb[kk]), S, 0, 0, 0);
  float s[4];
  bool invalid = false;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const bool ok = t.pos[i] >= 0 && col < G;
    s[i] = ok ? S[i] * scale : NEG_INF;
    invalid = invalid || t.pos[i] < 0;
  }
  if (logits_unit != nullptr && col < G) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int tt = t0 + 4 * r16 + i;
      if (tt < t_end) logits_unit[(size_t)tt * G + col] = s[i];
    }
  }
  float mx = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
  mx = fmaxf(mx, __shfl_xor(mx, 16));
  mx = fmaxf(mx, __shfl_xor(mx, 32));
  const float m_new = fmaxf(m_run, mx);
  if (__any(m_new > m_run)) {
    const float corr = (m_run == NEG_INF) ? 0.f : __expf(m_run - m_new);
    l_run *= corr;
    AccStep<G, 0>::scale(acc, corr);
  }
  m_run = m_new;
  float p[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    p[i] = (s[i] == NEG_INF) ? 0.f : __expf(s[i] - m_new);
    l_run += p[i];
  }
  const bool any_invalid = __any(invalid);
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    float v[8] = {__uint_as_float(t.vv[j].x << 16), __uint_as_float(t.vv[j].x & 0xffff0000u),
                  __uint_as_float(t.vv[j].y << 16), __uint_as_float(t.vv[j].y & 0xffff0000u),
                  __uint_as_float(t.vv[j].z << 16), __uint_as_float(t.vv[j].z & 0xffff0000u),
                  __uint_as_float(t.vv[j].w << 16), __uint_as_float(t.vv[j].w & 0xffff0000u)};
    if (any_invalid) {            // an empty slot may hold anything, even NaN: weight 0 is not enough
      const bool dead = t.pos[j] < 0;
#pragma unroll
      for (int c = 0; c < 8; ++c) v[c] = dead ? 0.f : v[c];
    }
    AccStep<G, 0>::fma(acc, p[j], v);
  }
}

template <int G>
__device__ __forceinline__ void attend_retained_body(const DevDesc& d, const AttendArgs& a, int n_rslices) {
  constexpr int NW = 4;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r16 = lane >> 4, col = lane & 15;
  const int tot_cap = a.ret_cap + a.vague_cap;
  const int n_items = d.B * d.Hkv * n_rslices;
  const float NEG_INF = -__builtin_inff();
  __shared__ float s_acc[NW][G][D];
  __shared__ float s_m[NW][G], s_l[NW][G];

  // Same issue priority as the lower of the two levels that the staged kernel's
  // waves alternate between: measured best when the two kernels share the CUs.
  __builtin_amdgcn_s_setprio(1);
  for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
    const int unit = item / n_rslices, slice = item % n_rslices;
    const int b = unit / d.Hkv, hk = unit % d.Hkv;
    const int t_begin = slice * a.slice_tokens;
    const int t_end = min(t_begin + a.slice_tokens, a.ret_cap);
    const bf16_t* kret = (const bf16_t*)a.k_ret + (size_t)unit * a.ret_cap * D;
    const bf16_t* vret = (const bf16_t*)a.v_ret + (size_t)unit * a.ret_cap * D;
    const int32_t* rp = a.ret_pos ? a.ret_pos + (size_t)unit * a.ret_cap : nullptr;
    float* logits_unit = a.logits ? a.logits + (size_t)unit * tot_cap * G : nullptr;

    uint4 qb[4];
    {
      const bf16_t* q = (const bf16_t*)a.q + ((size_t)b * d.Hq + (size_t)hk * G + (col < G ? col : 0)) * D + 8 * r16;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        qb[kk] = *reinterpret_cast<const uint4*>(q + 32 * kk);
        if (col >= G) qb[kk] = make_uint4(0u, 0u, 0u, 0u);
      }
    }
    float m_run = NEG_INF, l_run = 0.f;
    float acc[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int c = 0; c < 8; ++c) acc[g][c] = 0.f;

    const int n_tiles = (t_end > t_begin) ? (t_end - t_begin + 15) >> 4 : 0;
    for (int ti = wave; ti < n_tiles; ti += NW) {
      RetTile ta;
      load_tile(ta, kret, vret, rp, t_begin + ti * 16, t_end, a.ret_cap, r16, col);
      compute_tile<G>(ta, qb, d.scale, t_begin + ti * 16, t_end, r16, col, logits_unit, m_run, l_run, acc);
    }

    // the four 16-lane rows of the wave hold different tokens: add them
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        acc[g][c] += __shfl_xor(acc[g][c], 16);
        acc[g][c] += __shfl_xor(acc[g][c], 32);
      }
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);

    __syncthreads();             // the previous item's readers are done with the LDS arrays
    if (r16 == 0) {
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int c = 0; c < 8; ++c) s_acc[wave][g][col * 8 + c] = acc[g][c];
      if (col < G) { s_m[wave][col] = m_run; s_l[wave][col] = l_run; }
    }
    __syncthreads();
    float* po = a.part_o + ((size_t)unit * a.n_slices + slice) * G * D;
    float* pml = a.part_ml + ((size_t)unit * a.n_slices + slice) * G * 2;
    for (int idx = threadIdx.x; idx < G * D; idx += 256) {
      const int g = idx / D, c = idx % D;
      float M = s_m[0][g];
#pragma unroll
      for (int w_ = 1; w_ < NW; ++w_) M = fmaxf(M, s_m[w_][g]);
      float L = 0.f, O = 0.f;
#pragma unroll
      for (int w_ = 0; w_ < NW; ++w_) {
        const float e = (s_m[w_][g] == NEG_INF) ? 0.f : __expf(s_m[w_][g] - M);
        L += s_l[w_][g] * e;
        O += s_acc[w_][g][c] * e;
      }
      po[idx] = O;
      if (c == 0) { pml[g * 2] = M; pml[g * 2 + 1] = L; }
    }
  }
}

// Two kernels around the same body.  Alone, the kernel takes the registers it likes (135 for G = 4).  Next to
// the staged kernel it is capped at 124 + 4 accumulation registers (the attribute counts in units of two on
// this target): 2 x 192 (two waves of the staged kernel, which then needs no spills) + 128 fill a SIMD's 512
// registers exactly; the few spills of this kernel, which waits for HBM most of the time, cost nothing.
template <int G>
__global__ __launch_bounds__(256) void attend_retained_kernel(DevDesc d, AttendArgs a, int n_rslices) {
  attend_retained_body<G>(d, a, n_rslices);
}
template <int G>
__global__ __launch_bounds__(256) __attribute__((amdgpu_num_vgpr(62))) void attend_retained_shared_kernel(
    DevDesc d, AttendArgs a, int n_rslices) {
  attend_retained_body<G>(d, a, n_rslices);
}

// Third form, 76 + 4 registers: what two waves of the general staged kernel with 16- or 8-channel chunks and
// four query heads (about 212 registers each) leave of a SIMD.  It spills a lot and is slow, but it has six
// times the general staged kernel's duration to finish in.
template <int G>
__global__ __launch_bounds__(256) __attribute__((amdgpu_num_vgpr(38))) void attend_retained_tight_kernel(
    DevDesc d, AttendArgs a, int n_rslices) {
  attend_retained_body<G>(d, a, n_rslices);
}

hipError_t launch_attend_retained(const DevDesc& d, const AttendArgs& a, int n_rslices, int max_wgs,
                                  int reg_form, hipStream_t st) {
  int n_wgs = d.B * d.Hkv * n_rslices;
  if (max_wgs > 0 && n_wgs > max_wgs) n_wgs = max_wgs;
  if (n_wgs < 1) return hipSuccess;
  const dim3 grid(n_wgs), block(256);
  if (reg_form == 2 && d.G == 4) {      // next to the general staged kernel in its widest form
    hipLaunchKernelGGL(attend_retained_tight_kernel<4>, grid, block, 0, st, d, a, n_rslices);
    return hipGetLastError();
  }
  if (reg_form == 1) {                  // next to the 64-channel staged kernel
    switch (d.G) {
      case 1: hipLaunchKernelGGL(attend_retained_shared_kernel<1>, grid, block, 0, st, d, a, n_rslices); break;
      case 2: hipLaunchKernelGGL(attend_retained_shared_kernel<2>, grid, block, 0, st, d, a, n_rslices); break;
      case 4: hipLaunchKernelGGL(attend_retained_shared_kernel<4>, grid, block, 0, st, d, a, n_rslices); break;
      default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
  }
  switch (d.G) {
    case 1: hipLaunchKernelGGL(attend_retained_kernel<1>, grid, block, 0, st, d, a, n_rslices); break;
    case 2: hipLaunchKernelGGL(attend_retained_kernel<2>, grid, block, 0, st, d, a, n_rslices); break;
    case 4: hipLaunchKernelGGL(attend_retained_kernel<4>, grid, block, 0, st, d, a, n_rslices); break;
    case 8: hipLaunchKernelGGL(attend_retained_kernel<8>, grid, block, 0, st, d, a, n_rslices); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace kvr
