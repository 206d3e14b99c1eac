// kvr_select: Recent / Candidate / Vague partition (Recent and Candidate,
// Algorithm 3 without the swap loop), and kvr_append (R.Push of the new token).
//
// One workgroup per unit.  Every eligible slot gets a 64-bit key
//   (order-preserving image of its float32 score) << 32 | ~position
// so that "higher score first, then lower position" is plain integer order and
// all keys are distinct.  The k-th largest key is found by an 8-pass radix
// select on LDS histograms; the slots below it are emitted in ascending slot
// order with a block-wide prefix sum.
#include "kvr_launch.h"

namespace kvr {

constexpr int SEL_THREADS = 1024;

__device__ __forceinline__ bool slot_key(const int32_t* __restrict__ rp, const float* __restrict__ sc,
                                         int slot, int ret_cap, int recent_from, long long n_cap,
                                         unsigned long long& key, int& pos) {
  if (slot >= ret_cap) return false;
  pos = rp[slot];
  if (pos < 0 || pos >= recent_from || pos >= n_cap) return false;
  uint32_t b = __float_as_uint(sc[pos]);
  if (b == 0x80000000u) b = 0u;                                   // -0 ranks as +0
  const uint32_t mono = b ^ ((b >> 31) ? 0xffffffffu : 0x80000000u);
  key = ((unsigned long long)mono << 32) | (uint32_t)(~(uint32_t)pos);
  return true;
}

__global__ __launch_bounds__(SEL_THREADS) void select_kernel(
    DevDesc d, const float* __restrict__ scores, long long n_cap, int32_t* __restrict__ ret_pos,
    int ret_cap, const int32_t* __restrict__ n_ctx, int n_recent, int k_cand,
    int32_t* __restrict__ evict_slot, int32_t* __restrict__ evict_pos, int32_t* __restrict__ n_evict,
    int evict_cap, int32_t* __restrict__ vague_pos, int32_t* __restrict__ n_vague, int vague_cap) {
  const int unit = blockIdx.x;
  const int b = unit / d.Hkv;
  const int tid = threadIdx.x;
  int32_t* rp = ret_pos + (size_t)unit * ret_cap;
  const float* sc = scores + (size_t)unit * n_cap;
  const int recent_from = n_ctx[b] - n_recent;
  if (k_cand < 0) k_cand = 0;

  __shared__ unsigned hist[256];
  __shared__ unsigned long long s_prefix;
  __shared__ int s_krem, s_cnt, s_base;
  __shared__ int s_wsum[SEL_THREADS / WAVE];

  if (tid == 0) { s_cnt = 0; s_base = 0; s_prefix = 0ull; s_krem = k_cand; }
  __syncthreads();
  {
    int c = 0;
    for (int slot = tid; slot < ret_cap; slot += SEL_THREADS) {
      unsigned long long key; int pos;
      c += slot_key(rp, sc, slot, ret_cap, recent_from, n_cap, key, pos) ? 1 : 0;
    }
    if (c) atomicAdd(&s_cnt, c);
  }
  __syncthreads();
  const int n_e = s_cnt - k_cand;
  if (n_e <= 0) {
    if (tid == 0) n_evict[unit] = 0;
    return;
  }
  const int nv_old = (vague_pos && n_vague) ? clampi(n_vague[unit], 0, vague_cap) : 0;
  if (n_e > evict_cap || (vague_pos && n_vague && nv_old + n_e > vague_cap)) {
    if (tid == 0) n_evict[unit] = -n_e;
    return;
  }

  const bool evict_all = (k_cand == 0);
  if (!evict_all) {
    for (int byte = 7; byte >= 0; --byte) {
      if (tid < 256) hist[tid] = 0u;
      __syncthreads();
      const unsigned long long prefix = s_prefix;
      for (int slot = tid; slot < ret_cap; slot += SEL_THREADS) {
        unsigned long long key; int pos;
        if (slot_key(rp, sc, slot, ret_cap, recent_from, n_cap, key, pos)) {
          const bool match = (byte == 7) || ((key >> (8 * (byte + 1))) == (prefix >> (8 * (byte + 1))));
          if (match) atomicAdd(&hist[(unsigned)(key >> (8 * byte)) & 255u], 1u);
        }
      }
      __syncthreads();
      if (tid == 0) {
        int krem = s_krem;
        unsigned cum = 0;
        for (int dg = 255; dg >= 0; --dg) {
          const unsigned c = hist[dg];
          if (cum + c >= (unsigned)krem) {
            s_krem = krem - (int)cum;
            s_prefix = prefix | ((unsigned long long)dg << (8 * byte));
            break;
          }
          cum += c;
        }
      }
      __syncthreads();
    }
  }
  const unsigned long long T = s_prefix;   // the k-th largest key (unused when evict_all)

  const int lane = tid & 63, wave = tid >> 6;
  for (int chunk0 = 0; chunk0 < ret_cap; chunk0 += SEL_THREADS) {
    const int slot = chunk0 + tid;
    unsigned long long key = 0; int pos = -1;
    bool flag = slot_key(rp, sc, slot, ret_cap, recent_from, n_cap, key, pos);
    flag = flag && (evict_all || key < T);
    const unsigned long long bal = __ballot(flag);
    const int in_wave = __popcll(bal & ((1ull << lane) - 1ull));
    if (lane == 0) s_wsum[wave] = __popcll(bal);
    __syncthreads();
    int before = 0, tot = 0;
#pragma unroll
    for (int w_ = 0; w_ < SEL_THREADS / WAVE; ++w_) {
      const int c = s_wsum[w_];
      before += (w_ < wave) ? c : 0;
      tot += c;
    }
    const int base = s_base;
    if (flag) {
      const int idx = base + before + in_wave;      // < n_e <= evict_cap
      evict_slot[(size_t)unit * evict_cap + idx] = slot;
      evict_pos[(size_t)unit * evict_cap + idx] = pos;
      rp[slot] = -1;
      if (vague_pos && n_vague) vague_pos[(size_t)unit * vague_cap + nv_old + idx] = pos;
    }
    __syncthreads();
    if (tid == 0) s_base = base + tot;
    __syncthreads();
  }
  if (tid == 0) {
    n_evict[unit] = n_e;
    if (vague_pos && n_vague) n_vague[unit] = nv_old + n_e;
  }
}

hipError_t launch_select(const DevDesc& d, const float* scores, long long n_cap, int32_t* ret_pos,
                         int ret_cap, const int32_t* n_ctx, int n_recent, int k_candidate,
                         int32_t* evict_slot, int32_t* evict_pos, int32_t* n_evict, int evict_cap,
                         int32_t* vague_pos, int32_t* n_vague, int vague_cap, hipStream_t st) {
  hipLaunchKernelGGL(select_kernel, dim3(d.B * d.Hkv), dim3(SEL_THREADS), 0, st, d, scores, n_cap, ret_pos,
                     ret_cap, n_ctx, n_recent, k_candidate, evict_slot, evict_pos, n_evict, evict_cap,
                     vague_pos, n_vague, vague_cap);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void append_kernel(DevDesc d, const T* __restrict__ k_new,
                                                     const T* __restrict__ v_new,
                                                     const int32_t* __restrict__ n_ctx, T* __restrict__ k_ret,
                                                     T* __restrict__ v_ret, int32_t* __restrict__ ret_pos,
                                                     int ret_cap, int32_t* __restrict__ out_slot) {
  constexpr int VEC = Store<T>::VEC;
  constexpr int LPT = D / VEC;     // 16 (bf16) or 32 (f32) lanes copy one row
  const int unit = blockIdx.x;
  const int tid = threadIdx.x;
  int32_t* rp = ret_pos + (size_t)unit * ret_cap;
  __shared__ int s_free;
  if (tid == 0) s_free = 0x7fffffff;
  __syncthreads();
  int mine = 0x7fffffff;
  for (int s0 = 0; s0 < ret_cap; s0 += 256) {       // lowest empty slot
    const int s = s0 + tid;
    if (s < ret_cap && rp[s] < 0) { mine = s; break; }
  }
  if (mine != 0x7fffffff) atomicMin(&s_free, mine);
  __syncthreads();
  const int s = s_free;
  if (s >= ret_cap) {
    if (tid == 0 && out_slot) out_slot[unit] = -1;
    return;
  }
  const size_t dst = ((size_t)unit * ret_cap + s) * D;
  if (tid < LPT) {
    const uint4 v = *reinterpret_cast<const uint4*>(k_new + (size_t)unit * D + tid * VEC);
    *reinterpret_cast<uint4*>(k_ret + dst + tid * VEC) = v;
  } else if (tid < 2 * LPT) {
    const int l2 = tid - LPT;
    const uint4 v = *reinterpret_cast<const uint4*>(v_new + (size_t)unit * D + l2 * VEC);
    *reinterpret_cast<uint4*>(v_ret + dst + l2 * VEC) = v;
  }
  if (tid == 0) {
    rp[s] = n_ctx[unit / d.Hkv] - 1;
    if (out_slot) out_slot[unit] = s;
  }
}

hipError_t launch_append(const DevDesc& d, int dtype, const void* k_new, const void* v_new,
                         const int32_t* n_ctx, void* k_ret, void* v_ret, int32_t* ret_pos, int ret_cap,
                         int32_t* out_slot, hipStream_t st) {
  const dim3 grid(d.B * d.Hkv), block(256);
  if (dtype == KVR_F32)
    hipLaunchKernelGGL(append_kernel<float>, grid, block, 0, st, d, (const float*)k_new, (const float*)v_new,
                       n_ctx, (float*)k_ret, (float*)v_ret, ret_pos, ret_cap, out_slot);
  else
    hipLaunchKernelGGL(append_kernel<bf16_t>, grid, block, 0, st, d, (const bf16_t*)k_new,
                       (const bf16_t*)v_new, n_ctx, (bf16_t*)k_ret, (bf16_t*)v_ret, ret_pos, ret_cap,
                       out_slot);
  return hipGetLastError();
}

}  // namespace kvr
