// kvr_reconstruct: batched V.Query (Vague Sketch, Algorithm 2).
// One token per lane group; each lane owns a 16-byte channel chunk, gathers the
// r sketch rows of its token for K and for V, and writes the per-channel median.
#include "kvr_staged.h"

namespace kvr {

template <typename T, int R>
__global__ __launch_bounds__(256) void reconstruct_kernel(DevDesc d, const T* __restrict__ sk,
                                                          const T* __restrict__ sv,
                                                          const int32_t* __restrict__ tok_pos,
                                                          const int32_t* __restrict__ count, int cap,
                                                          T* __restrict__ k_out, T* __restrict__ v_out) {
  constexpr int VEC = Store<T>::VEC;
  constexpr int LPT = D / VEC;          // lanes per token
  constexpr int TPB = 256 / LPT;        // tokens per block
  const int unit = blockIdx.y;
  const int n = clampi(count[unit], 0, cap);
  const int t = blockIdx.x * TPB + threadIdx.x / LPT;
  if (t >= n) return;
  const int c0 = (threadIdx.x % LPT) * VEC;
  const int J = tok_pos[(size_t)unit * cap + t];
  const size_t sk_unit = (size_t)unit * d.r * d.w * D;
  float kf[VEC], vf[VEC];
  query_chunk<T, R>(d, sk + sk_unit, J, c0, (d.sign_mask & 1) != 0, kf);
  query_chunk<T, R>(d, sv + sk_unit, J, c0, (d.sign_mask & 2) != 0, vf);
  const size_t o = ((size_t)unit * cap + t) * D + c0;
  Store<T>::store16(k_out + o, kf);
  Store<T>::store16(v_out + o, vf);
}

// bf16 storage, three or four rows: the rows are flipped and reduced on their packed
// bits (v_med3_f16 / packed min and max order bf16 bit patterns like the values
// they encode; the mean of the two middle values of four is taken in float32 and
// rounded once).
template <int R>
__global__ __launch_bounds__(256) void reconstruct_bf16_kernel(DevDesc d, const bf16_t* __restrict__ sk,
                                                               const bf16_t* __restrict__ sv,
                                                               const int32_t* __restrict__ tok_pos,
                                                               const int32_t* __restrict__ count, int cap,
                                                               bf16_t* __restrict__ k_out,
                                                               bf16_t* __restrict__ v_out) {
  constexpr int LPT = 16, TPB = 256 / LPT;
  const int unit = blockIdx.y;
  const int n = clampi(count[unit], 0, cap);
  const int t = blockIdx.x * TPB + threadIdx.x / LPT;
  if (t >= n) return;
  const int c0 = (threadIdx.x % LPT) * 8;
  const int J = tok_pos[(size_t)unit * cap + t];
  const size_t sk_unit = (size_t)unit * R * d.w * D;
  uint4 rk[R], rv[R];
#pragma unroll
  for (int i = 0; i < R; ++i) {
    const size_t o = sk_unit + ((size_t)i * d.w + bucket_of(d, i, J)) * D + c0;
    rk[i] = *reinterpret_cast<const uint4*>(sk + o);
    rv[i] = *reinterpret_cast<const uint4*>(sv + o);
  }
#pragma unroll
  for (int i = 0; i < R; ++i) {
    const uint32_t neg = sign_neg(d, i, J) ? 0x80008000u : 0u;
    rk[i] = xor4(rk[i], (d.sign_mask & 1) ? neg : 0u);
    rv[i] = xor4(rv[i], (d.sign_mask & 2) ? neg : 0u);
  }
  const size_t o = ((size_t)unit * cap + t) * D + c0;
  *reinterpret_cast<uint4*>(k_out + o) = median_piece<R>(rk, d.median_mode);
  *reinterpret_cast<uint4*>(v_out + o) = median_piece<R>(rv, d.median_mode);
}

template <typename T>
static hipError_t launch_t(const DevDesc& d, const void* sk, const void* sv, const int32_t* tok_pos,
                           const int32_t* count, int cap, void* k_out, void* v_out, hipStream_t st) {
  constexpr int TPB = 256 / (D / Store<T>::VEC);
  dim3 grid((cap + TPB - 1) / TPB, d.B * d.Hkv);
  dim3 block(256);
#define KVR_GO(R)                                                                                   \
  hipLaunchKernelGGL((reconstruct_kernel<T, R>), grid, block, 0, st, d, (const T*)sk, (const T*)sv, \
                     tok_pos, count, cap, (T*)k_out, (T*)v_out)
  switch (d.r) {
    case 3: KVR_GO(3); break;
    case 4: KVR_GO(4); break;
    default: KVR_GO(0); break;
  }
#undef KVR_GO
  return hipGetLastError();
}

hipError_t launch_reconstruct(const DevDesc& d, int dtype, const void* sk, const void* sv,
                              const int32_t* tok_pos, const int32_t* count, int cap, void* k_out,
                              void* v_out, hipStream_t st) {
  if (cap <= 0) return hipSuccess;
  if (dtype == KVR_BF16 && (d.r == 3 || d.r == 4)) {
    const dim3 grid((cap + 15) / 16, d.B * d.Hkv);
    if (d.r == 3)
      hipLaunchKernelGGL(reconstruct_bf16_kernel<3>, grid, dim3(256), 0, st, d, (const bf16_t*)sk, (const bf16_t*)sv,
                         tok_pos, count, cap, (bf16_t*)k_out, (bf16_t*)v_out);
    else
      hipLaunchKernelGGL(reconstruct_bf16_kernel<4>, grid, dim3(256), 0, st, d, (const bf16_t*)sk, (const bf16_t*)sv,
                         tok_pos, count, cap, (bf16_t*)k_out, (bf16_t*)v_out);
    return hipGetLastError();
  }
  if (dtype == KVR_F32) return launch_t<float>(d, sk, sv, tok_pos, count, cap, k_out, v_out, st);
  return launch_t<bf16_t>(d, sk, sv, tok_pos, count, cap, k_out, v_out, st);
}

}  // namespace kvr
