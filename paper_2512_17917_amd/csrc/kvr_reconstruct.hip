// kvr_reconstruct: batched V.Query (Vague Sketch, Algorithm 2).
// One token per lane group; each lane owns a 16-byte channel chunk, gathers the
// r sketch rows of its token for K and for V, and writes the per-channel median.
// Long lists with bf16 storage and three rows go through an LDS copy of the sketch
// instead (reconstruct_staged3_kernel).
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

// ---------------------------------------------------------------------------
// bf16, three rows, long lists: the sketch goes through LDS.
//
// The kernel above gathers r rows of 256 bytes for K and for V per token out of L2: three times the
// bytes it writes, and L2 bandwidth bounds it.  Here a workgroup copies one 64-channel chunk of one
// tensor of its unit into LDS once (global_load_lds, as the attention kernels do) and rebuilds that
// half row of every token of its share of the list from it: (unit, tensor, half, token slice) per
// workgroup, the four chunks of a unit independent of each other.  Tokens are taken in tiles (as
// many tokens as LDS has room for a 4-byte record each, at most RS_TILE_MAX): first every thread
// hashes its tokens of the tile and leaves a record (three 9-bit buckets, three sign bits) in LDS,
// then groups of 8 lanes take one token each, a lane one 16-byte piece: three LDS reads, the
// flips, one packed median, one 16-byte store.  A group writes 128 contiguous bytes.
constexpr int RS_TILE_MAX = 8192;

__global__ __launch_bounds__(ST_THREADS) void reconstruct_staged3_kernel(
    DevDesc d, const bf16_t* __restrict__ sk, const bf16_t* __restrict__ sv,
    const int32_t* __restrict__ tok_pos, const int32_t* __restrict__ count, int cap,
    bf16_t* __restrict__ k_out, bf16_t* __restrict__ v_out, int n_tslices, int slice_tokens, int tile) {
  extern __shared__ __align__(16) unsigned char smem[];
  // workgroup ids are dealt round-robin to the 8 XCDs: a unit's workgroups share one L2
  const int lin = blockIdx.x, xcd = lin & 7, jj = lin >> 3;
  const int per_unit = 4 * n_tslices;
  const int unit = (jj / per_unit) * 8 + xcd;
  if (unit >= d.B * d.Hkv) return;
  const int within = jj % per_unit, chunk = within & 3, ts = within >> 2;
  const int n = clampi(count[unit], 0, cap);
  const int t_begin = ts * slice_tokens, t_end = min(n, t_begin + slice_tokens);
  if (t_begin >= t_end) return;                 // uniform over the workgroup, before any barrier
  const int tid = threadIdx.x;
  const int w = d.w;
  const bool is_v = chunk >= 2;
  const int half = chunk & 1;
  const int sk_bytes = (3 * w * 128 + 1023) & ~1023;
  unsigned char* s_sk = smem;                                         // [3 w] rows of 128 bytes
  uint32_t* s_rec = reinterpret_cast<uint32_t*>(smem + sk_bytes);     // [tile] token records
  const unsigned char* src =
      reinterpret_cast<const unsigned char*>((is_v ? sv : sk) + (size_t)unit * 3 * w * D);
  stage_issue<8, 128>(src, s_sk, 3 * w * 8, half, tid);
  const uint32_t flip = ((d.sign_mask >> (is_v ? 1 : 0)) & 1) ? 0x80008000u : 0u;
  const int32_t* tp = tok_pos + (size_t)unit * cap;
  bf16_t* out = (is_v ? v_out : k_out) + (size_t)unit * cap * D + half * 64;
  const int piece = tid & 7, tg = tid >> 3;     // 64 groups of 8 lanes
  const uint32_t w7 = (uint32_t)w << 7;
  for (int tile0 = t_begin; tile0 < t_end; tile0 += tile) {
    for (int tl0 = tid; tl0 < tile; tl0 += 8 * ST_THREADS) {        // eight positions requested together
      int J[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int t = tile0 + tl0 + u * ST_THREADS;
        J[u] = (tl0 + u * ST_THREADS < tile && t < t_end) ? tp[t] : 0;
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int tl = tl0 + u * ST_THREADS;
        if (tl < tile && tile0 + tl < t_end)
          s_rec[tl] = (uint32_t)bucket_of(d, 0, J[u]) | ((uint32_t)bucket_of(d, 1, J[u]) << 9) |
                      ((uint32_t)bucket_of(d, 2, J[u]) << 18) | (sign_neg(d, 0, J[u]) ? 1u << 27 : 0u) |
                      (sign_neg(d, 1, J[u]) ? 1u << 28 : 0u) | (sign_neg(d, 2, J[u]) ? 1u << 29 : 0u);
      }
    }
    if (tile0 == t_begin) stage_wait();         // the chunk has arrived
    lds_barrier();                              // chunk and records visible
    // four tokens per lane in flight: two waves per SIMD cannot hide the LDS latency of the
    // record -> rows -> median chain for each other
    constexpr int NT = 4, STEP = ST_THREADS / 8;
    for (int tl0 = tg; tl0 < tile && tile0 + tl0 < t_end; tl0 += NT * STEP) {
      uint32_t rec[NT];
#pragma unroll
      for (int u = 0; u < NT; ++u) rec[u] = s_rec[min(tl0 + u * STEP, tile - 1)];
      uint4 ra[NT], rb[NT], rc[NT];
#pragma unroll
      for (int u = 0; u < NT; ++u) {
        const bool live = tl0 + u * STEP < tile && tile0 + tl0 + u * STEP < t_end;     // else a stale record: row 0
        const uint32_t x = live ? rec[u] : 0u;
        ra[u] = *reinterpret_cast<const uint4*>(s_sk + ((x & 511u) << 7) + piece * 16);
        rb[u] = *reinterpret_cast<const uint4*>(s_sk + w7 + (((x >> 9) & 511u) << 7) + piece * 16);
        rc[u] = *reinterpret_cast<const uint4*>(s_sk + 2 * w7 + (((x >> 18) & 511u) << 7) + piece * 16);
      }
#pragma unroll
      for (int u = 0; u < NT; ++u) {
        const int t = tile0 + tl0 + u * STEP;
        if (tl0 + u * STEP < tile && t < t_end) {
          const uint32_t m0 = ((rec[u] >> 27) & 1u) ? flip : 0u, m1 = ((rec[u] >> 28) & 1u) ? flip : 0u,
                         m2 = ((rec[u] >> 29) & 1u) ? flip : 0u;
          // written once and not read again by this kernel: past the caches
          const uint4 med = med3_piece(xor4(ra[u], m0), xor4(rb[u], m1), xor4(rc[u], m2));
          typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
          __builtin_nontemporal_store(u32x4_t{med.x, med.y, med.z, med.w},
                                      reinterpret_cast<u32x4_t*>(out + (size_t)t * D + piece * 8));
        }
      }
    }
    lds_barrier();                              // everyone is done with this tile's records
  }
}

static bool reconstruct_staged_applies(const DevDesc& d, int cap) {
  return d.r == 3 && 3 * d.w <= 1024 && cap >= 4096;      // the chunk fits LDS (9-bit buckets); a list worth a chunk copy
}

static hipError_t launch_reconstruct_staged(const DevDesc& d, const void* sk, const void* sv,
                                            const int32_t* tok_pos, const int32_t* count, int cap, void* k_out,
                                            void* v_out, hipStream_t st) {
  static std::once_flag once;
  static hipError_t attr_rc = hipSuccess;
  std::call_once(once, [&]() {
    attr_rc = hipFuncSetAttribute(reinterpret_cast<const void*>(reconstruct_staged3_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  });
  if (attr_rc != hipSuccess) return attr_rc;
  const int units = d.B * d.Hkv;
  // about two workgroups per CU in all, a slice of at least 1024 tokens
  int n_tslices = (512 + units * 4 - 1) / (units * 4);
  if (n_tslices > cap / 1024) n_tslices = cap / 1024;
  if (n_tslices < 1) n_tslices = 1;
  const int slice_tokens = ((cap + n_tslices - 1) / n_tslices + 63) / 64 * 64;
  n_tslices = (cap + slice_tokens - 1) / slice_tokens;
  // token records: what LDS has left, in whole rounds of the workgroup
  const size_t sk_bytes = ((size_t)3 * d.w * 128 + 1023) & ~(size_t)1023;
  int tile = (int)(((size_t)160 * 1024 - sk_bytes) / 4) / ST_THREADS * ST_THREADS;
  if (tile > RS_TILE_MAX) tile = RS_TILE_MAX;
  if (tile > slice_tokens) tile = (slice_tokens + ST_THREADS - 1) / ST_THREADS * ST_THREADS;
  const size_t lds = sk_bytes + (size_t)tile * 4;
  const int units_pad = (units + 7) / 8 * 8;
  hipLaunchKernelGGL(reconstruct_staged3_kernel, dim3(units_pad * 4 * n_tslices), dim3(ST_THREADS), lds, st, d,
                     (const bf16_t*)sk, (const bf16_t*)sv, tok_pos, count, cap, (bf16_t*)k_out, (bf16_t*)v_out,
                     n_tslices, slice_tokens, tile);
  return hipGetLastError();
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
  if (dtype == KVR_BF16 && reconstruct_staged_applies(d, cap))
    return launch_reconstruct_staged(d, sk, sv, tok_pos, count, cap, k_out, v_out, st);
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
