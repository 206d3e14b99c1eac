// kvr_select, kvr_append and the fused kvr_step_update: the Recent / Candidate /
// Vague bookkeeping of one decode step (Recent and Candidate, Algorithm 3
// without the swap loop).
//
// One workgroup per unit.  Every eligible slot gets a 64-bit key
//   (order-preserving image of its float32 score) << 32 | ~position
// so that "higher score first, then lower position" is plain integer order and
// all keys are distinct.  The slots to evict are the n_e = eligible - k lowest
// keys.  Two ways to find the cut:
//   - n_e small (the decode steady state evicts one token per unit per step):
//     n_e rounds of a block-wide minimum over keys above the previous minimum;
//   - otherwise an 8-pass radix select of the k-th largest key on LDS histograms
//     whose 256 bins are scanned by 256 threads.
// Up to 8192 slots the keys are computed once and stay in registers (8 per
// thread); larger slot arrays (a whole prompt) recompute them from memory in
// every pass.  The evicted slots are emitted in ascending slot order with a
// ballot / prefix-sum compaction.
//
// kvr_step_update runs append -> select -> encode (small regime) of a unit in
// one workgroup (slot arrays up to 32768 entries: 8 or 32 slots per thread), one launch instead of three; the steps communicate through the
// same global arrays as the separate calls, ordered by workgroup barriers.
#include "kvr_launch.h"
#include "kvr_update.h"

namespace kvr {

template <bool REG, int KPT>
__global__ __launch_bounds__(SEL_THREADS) void select_kernel(
    DevDesc d, const float* __restrict__ scores, long long n_cap, int32_t* __restrict__ ret_pos,
    int ret_cap, const int32_t* __restrict__ n_ctx, int n_recent, int k_cand,
    int32_t* __restrict__ evict_slot, int32_t* __restrict__ evict_pos, int32_t* __restrict__ n_evict,
    int evict_cap, int32_t* __restrict__ vague_pos, int32_t* __restrict__ n_vague, int vague_cap) {
  select_body<REG, KPT>(d, blockIdx.x, scores, n_cap, ret_pos, ret_cap, n_ctx, n_recent, k_cand, evict_slot,
                   evict_pos, n_evict, evict_cap, vague_pos, n_vague, vague_cap);
}

hipError_t launch_select(const DevDesc& d, const float* scores, long long n_cap, int32_t* ret_pos,
                         int ret_cap, const int32_t* n_ctx, int n_recent, int k_candidate,
                         int32_t* evict_slot, int32_t* evict_pos, int32_t* n_evict, int evict_cap,
                         int32_t* vague_pos, int32_t* n_vague, int vague_cap, hipStream_t st) {
  const dim3 grid(d.B * d.Hkv), block(SEL_THREADS);
#define KVR_LAUNCH_SELECT(REG, KPT)                                                                            \
  hipLaunchKernelGGL((select_kernel<REG, KPT>), grid, block, 0, st, d, scores, n_cap, ret_pos, ret_cap, n_ctx, \
                     n_recent, k_candidate, evict_slot, evict_pos, n_evict, evict_cap, vague_pos, n_vague,     \
                     vague_cap)
  if (ret_cap <= SEL_THREADS * 8) KVR_LAUNCH_SELECT(true, 8);
  else if (ret_cap <= SEL_THREADS * 32) KVR_LAUNCH_SELECT(true, 32);
  else KVR_LAUNCH_SELECT(false, 1);
#undef KVR_LAUNCH_SELECT
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void append_kernel(DevDesc d, const T* __restrict__ k_new,
                                                     const T* __restrict__ v_new,
                                                     const int32_t* __restrict__ n_ctx, T* __restrict__ k_ret,
                                                     T* __restrict__ v_ret, int32_t* __restrict__ ret_pos,
                                                     int ret_cap, int32_t* __restrict__ out_slot) {
  const int s = append_body<T, 256>(d, blockIdx.x, k_new, v_new, n_ctx, k_ret, v_ret, ret_pos, ret_cap);
  if (threadIdx.x == 0 && out_slot) out_slot[blockIdx.x] = s;
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

// ---------------------------------------------------------------------------
// KPT: retained slots per thread (8: up to 8192 slots, the 32k workloads; 32: up to 32768 slots, the
// 131k workload)
template <typename T, int KPT>
__global__ __launch_bounds__(SEL_THREADS) void step_update_kernel(
    DevDesc d, const T* __restrict__ k_new, const T* __restrict__ v_new, const int32_t* __restrict__ n_ctx,
    T* __restrict__ k_ret, T* __restrict__ v_ret, int32_t* __restrict__ ret_pos, int ret_cap,
    const float* __restrict__ scores, long long n_cap, int n_recent, int k_cand,
    int32_t* __restrict__ evict_slot, int32_t* __restrict__ evict_pos, int32_t* __restrict__ n_evict,
    int evict_cap, int32_t* __restrict__ vague_pos, int32_t* __restrict__ n_vague, int vague_cap,
    T* __restrict__ sk, T* __restrict__ sv) {
  const int unit = blockIdx.x;
  // the slot positions are read once and serve both the search for a free slot and
  // the selection keys (the token appended in between is Recent unless n_recent = 0:
  // for the selection its slot might as well still be empty)
  int pre[KPT];
  {
    const int32_t* rp = ret_pos + (size_t)unit * ret_cap;
#pragma unroll
    for (int j = 0; j < KPT; ++j) {
      const int s = j * SEL_THREADS + threadIdx.x;
      pre[j] = (s < ret_cap) ? rp[s] : 0;
    }
  }
  // the new token's rows are requested with the positions, one round trip ahead of their store
  uint4 row_in = make_uint4(0u, 0u, 0u, 0u);
  {
    constexpr int LPT = D / Store<T>::VEC;
    const int t = threadIdx.x;
    if (t < LPT) row_in = *reinterpret_cast<const uint4*>(k_new + (size_t)unit * D + t * Store<T>::VEC);
    else if (t < 2 * LPT) row_in = *reinterpret_cast<const uint4*>(v_new + (size_t)unit * D + (t - LPT) * Store<T>::VEC);
  }
  // the scores the selection will rank by are requested now: their round trip overlaps the append
  float pre_sc[KPT];
  {
    const float* sc = scores + (size_t)unit * n_cap;
    const int recent_from = n_ctx[unit / d.Hkv] - n_recent;
#pragma unroll
    for (int j = 0; j < KPT; ++j) {
      const int pos = pre[j];
      pre_sc[j] = (pos >= 0 && pos < recent_from && pos < n_cap) ? sc[pos] : 0.f;
    }
  }
  const int s_new = append_body_pre<T, SEL_THREADS, KPT>(d, unit, k_new, v_new, n_ctx, k_ret, v_ret, ret_pos,
                                                         ret_cap, pre, &row_in);
  if (n_recent == 0 && s_new >= 0) {
    // an empty Recent window: the token just appended is a Candidate like any other, so the
    // thread that holds its slot ranks it by its real position instead of the stale "empty"
    const int pos_new = n_ctx[unit / d.Hkv] - 1;
#pragma unroll
    for (int j = 0; j < KPT; ++j)
      if (j * SEL_THREADS + (int)threadIdx.x == s_new) {
        pre[j] = pos_new;
        pre_sc[j] = (pos_new >= 0 && pos_new < n_cap) ? scores[(size_t)unit * n_cap + pos_new] : 0.f;
      }
  }
  __shared__ EvictHandOver ho;
  __syncthreads();          // the new row and its ret_pos entry are visible to the whole workgroup
  select_body<true, KPT>(d, unit, scores, n_cap, ret_pos, ret_cap, n_ctx, n_recent, k_cand, evict_slot, evict_pos,
                         n_evict, evict_cap, vague_pos, n_vague, vague_cap, pre, pre_sc, &ho);
  __syncthreads();          // the eviction list and its count are visible (in LDS; global memory has them too)
  encode_small_body<T>(d, unit, k_ret, v_ret, ret_cap, evict_slot, evict_pos, n_evict, evict_cap, sk, sv,
                       nullptr, nullptr, &ho);
}

hipError_t launch_step_update(const DevDesc& d, int dtype, const void* k_new, const void* v_new,
                              const int32_t* n_ctx, void* k_ret, void* v_ret, int32_t* ret_pos, int ret_cap,
                              const float* scores, long long n_cap, int n_recent, int k_candidate,
                              int32_t* evict_slot, int32_t* evict_pos, int32_t* n_evict, int evict_cap,
                              int32_t* vague_pos, int32_t* n_vague, int vague_cap, void* sk, void* sv,
                              hipStream_t st) {
  const dim3 grid(d.B * d.Hkv), block(SEL_THREADS);
#define KVR_LAUNCH_STEP(T, KPT)                                                                                 \
  hipLaunchKernelGGL((step_update_kernel<T, KPT>), grid, block, 0, st, d, (const T*)k_new, (const T*)v_new,     \
                     n_ctx, (T*)k_ret, (T*)v_ret, ret_pos, ret_cap, scores, n_cap, n_recent, k_candidate,       \
                     evict_slot, evict_pos, n_evict, evict_cap, vague_pos, n_vague, vague_cap, (T*)sk, (T*)sv)
  if (ret_cap <= SEL_THREADS * 8) {
    if (dtype == KVR_F32) KVR_LAUNCH_STEP(float, 8);
    else KVR_LAUNCH_STEP(bf16_t, 8);
  } else {
    if (dtype == KVR_F32) KVR_LAUNCH_STEP(float, 32);
    else KVR_LAUNCH_STEP(bf16_t, 32);
  }
#undef KVR_LAUNCH_STEP
  return hipGetLastError();
}

}  // namespace kvr
