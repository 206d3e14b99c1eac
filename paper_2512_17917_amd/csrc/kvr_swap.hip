// kvr_swap_back: the swap loop of Algorithm 3 (Recent and Candidate):
//
//     while C.Min_Score() * ReplaceRate < V.Max_Score():
//         tmp <- V.Query(V.Max_Score_Index());  V.Delete(tmp)
//         V.Insert(C.Top_Pop());                C.Push(tmp)
//
// One workgroup per unit, at most max_swaps rounds.  A round:
//   1. every thread scans a strided share of the Vague index list for the highest
//      cumulative score and of the retained slots for the lowest Candidate score,
//      as 64-bit keys (order-preserving image of the float32 score) << 32 | ~position,
//      the same keys kvr_select ranks by, so "highest score, then earlier position"
//      is the largest key and "lowest score, then later position" the smallest, and
//      all keys are distinct; the workgroup reduces them and the two owner threads
//      publish slot, list index, position and score;
//   2. the loop condition is evaluated in float32, the type the scores are kept in;
//   3. thread c < D owns channel c of the key tensors, thread D + c channel c of the
//      value tensors: it reads its channel of the r sketch rows of the Vague token,
//      takes the median (Algorithm 2), reads the Candidate's channel, writes
//      sketch = round(float32(old) - estimate) and round(float32(old) + candidate)
//      (one sum, one rounding, if both fall into the same slot of a row: delete
//      first, then insert), and stores the estimate into the Candidate's slot.  A
//      channel is only ever touched by its own thread, so no barrier is needed
//      between the query and the update;
//   4. thread 0 exchanges the two positions in ret_pos / vague_pos.
#include "kvr_launch.h"

namespace kvr {

constexpr int SWP_THREADS = 1024;
constexpr int SWP_WAVES = SWP_THREADS / WAVE;
constexpr unsigned long long SWP_NONE_MAX = 0ull;      // below every key (the low word ~position of a key is never 0)
constexpr unsigned long long SWP_NONE_MIN = ~0ull;     // above every key of a finite score

struct SwapShared {
  unsigned long long wmax[SWP_WAVES], wmin[SWP_WAVES];
  unsigned long long kmax, kmin;
  int v_idx, v_pos, c_slot, c_pos;
  float v_score, c_score;
};

// key of (score, position): larger = higher score, then earlier position.  -0 ranks as +0.
// Never 0 and never ~0 for a valid position (0 <= pos < 2^30).
__device__ __forceinline__ unsigned long long swap_key(float score, int pos) {
  uint32_t b = __float_as_uint(score);
  if (b == 0x80000000u) b = 0u;
  const uint32_t mono = b ^ ((b >> 31) ? 0xffffffffu : 0x80000000u);
  return ((unsigned long long)mono << 32) | (uint32_t)(~(uint32_t)pos);
}

__device__ __forceinline__ unsigned long long shfl_xor_u64s(unsigned long long v, int m) {
  const uint32_t lo = __shfl_xor((int)(uint32_t)v, m), hi = __shfl_xor((int)(uint32_t)(v >> 32), m);
  return ((unsigned long long)hi << 32) | lo;
}

template <typename T>
__global__ __launch_bounds__(SWP_THREADS) void swap_back_kernel(
    DevDesc d, const float* __restrict__ scores, long long n_cap, T* k_ret, T* v_ret, int32_t* ret_pos,
    int ret_cap, const int32_t* __restrict__ n_ctx, int n_recent, float replace_rate, int max_swaps, T* sk,
    T* sv, int32_t* vague_pos, const int32_t* __restrict__ n_vague, int vague_cap,
    int32_t* __restrict__ n_swapped, int32_t* __restrict__ swap_log) {
  const int unit = blockIdx.x;
  const int b = unit / d.Hkv;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  __shared__ SwapShared sh;
  int32_t* rp = ret_pos + (size_t)unit * ret_cap;
  int32_t* vp = vague_pos + (size_t)unit * vague_cap;
  const float* sc = scores + (size_t)unit * n_cap;
  const int recent_from = n_ctx[b] - n_recent;
  const int nv = clampi(n_vague[unit], 0, vague_cap);
  int done = 0;

  for (int round = 0; round < max_swaps; ++round) {
    // ---- 1. this thread's share of both scans; four independent chains of loads ----
    unsigned long long kmax = SWP_NONE_MAX, kmin = SWP_NONE_MIN;
    int imax = -1, smin = -1;
    for (int i0 = tid; i0 < nv; i0 += SWP_THREADS * 4) {
      int pos[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int i = i0 + u * SWP_THREADS;
        pos[u] = (i < nv) ? vp[i] : -1;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (pos[u] >= 0 && pos[u] < n_cap) {
          const unsigned long long key = swap_key(sc[pos[u]], pos[u]);
          if (key > kmax) { kmax = key; imax = i0 + u * SWP_THREADS; }
        }
      }
    }
    for (int s0 = tid; s0 < ret_cap; s0 += SWP_THREADS * 4) {
      int pos[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int s = s0 + u * SWP_THREADS;
        pos[u] = (s < ret_cap) ? rp[s] : -1;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (pos[u] >= 0 && pos[u] < recent_from && pos[u] < n_cap) {
          const unsigned long long key = swap_key(sc[pos[u]], pos[u]);
          if (key < kmin) { kmin = key; smin = s0 + u * SWP_THREADS; }
        }
      }
    }
    unsigned long long wmx = kmax, wmn = kmin;
#pragma unroll
    for (int m = 1; m < WAVE; m <<= 1) {
      const unsigned long long o1 = shfl_xor_u64s(wmx, m), o2 = shfl_xor_u64s(wmn, m);
      wmx = o1 > wmx ? o1 : wmx;
      wmn = o2 < wmn ? o2 : wmn;
    }
    if (lane == 0) { sh.wmax[wave] = wmx; sh.wmin[wave] = wmn; }
    __syncthreads();
    if (tid == 0) {
      unsigned long long a = sh.wmax[0], c = sh.wmin[0];
#pragma unroll
      for (int w_ = 1; w_ < SWP_WAVES; ++w_) {
        a = sh.wmax[w_] > a ? sh.wmax[w_] : a;
        c = sh.wmin[w_] < c ? sh.wmin[w_] : c;
      }
      sh.kmax = a;
      sh.kmin = c;
    }
    __syncthreads();
    const unsigned long long gmax = sh.kmax, gmin = sh.kmin;
    if (gmax == SWP_NONE_MAX || gmin == SWP_NONE_MIN) break;        // a part is empty (uniform)
    if (kmax == gmax) {                                             // keys are distinct: one owner each
      const int pos = (int)(~(uint32_t)gmax);
      sh.v_idx = imax;
      sh.v_pos = pos;
      sh.v_score = sc[pos];
    }
    if (kmin == gmin) {
      const int pos = (int)(~(uint32_t)gmin);
      sh.c_slot = smin;
      sh.c_pos = pos;
      sh.c_score = sc[pos];
    }
    __syncthreads();
    // ---- 2. loop condition, in float32 ---------------------------------------------
    const float lhs = sh.c_score * replace_rate;
    if (!(lhs < sh.v_score)) break;                                 // uniform
    const int J = sh.v_pos, pc = sh.c_pos, v_idx = sh.v_idx, c_slot = sh.c_slot;

    // ---- 3. query, delete, insert, push: one thread per channel and tensor --------
    if (tid < 2 * D) {
      const bool is_v = tid >= D;
      const int c = is_v ? tid - D : tid;
      T* sx = is_v ? sv : sk;
      T* xr = is_v ? v_ret : k_ret;
      const bool flip = is_v ? (d.sign_mask & 2) != 0 : (d.sign_mask & 1) != 0;
      const size_t sk_unit = (size_t)unit * d.r * d.w * D;
      float rows[KVR_MAX_ROWS];
      size_t idx_d[KVR_MAX_ROWS], idx_c[KVR_MAX_ROWS];
      float gd[KVR_MAX_ROWS], gc[KVR_MAX_ROWS];
#pragma unroll
      for (int i = 0; i < KVR_MAX_ROWS; ++i) {
        rows[i] = 0.f;
        if (i < d.r) {
          idx_d[i] = sk_unit + ((size_t)i * d.w + bucket_of(d, i, J)) * D + c;
          idx_c[i] = sk_unit + ((size_t)i * d.w + bucket_of(d, i, pc)) * D + c;
          gd[i] = (flip && sign_neg(d, i, J)) ? -1.f : 1.f;
          gc[i] = (flip && sign_neg(d, i, pc)) ? -1.f : 1.f;
          const float x = Store<T>::load1(sx + idx_d[i]);
          rows[i] = gd[i] < 0.f ? -x : x;
        }
      }
      const float est = median_rows<0, T>(rows, d.r, d.median_mode);
      const size_t cslot_idx = ((size_t)unit * ret_cap + c_slot) * D + c;
      const float cand = Store<T>::load1(xr + cslot_idx);
#pragma unroll
      for (int i = 0; i < KVR_MAX_ROWS; ++i) {
        if (i < d.r) {
          // delete first, then insert; float32 sums, one rounding per touched slot
          float acc = Store<T>::load1(sx + idx_d[i]);
          acc = acc + (-gd[i]) * est;
          if (idx_c[i] == idx_d[i]) {
            acc = acc + gc[i] * cand;
            Store<T>::store1(sx + idx_d[i], acc);
          } else {
            Store<T>::store1(sx + idx_d[i], acc);
            float acc2 = Store<T>::load1(sx + idx_c[i]);
            acc2 = acc2 + gc[i] * cand;
            Store<T>::store1(sx + idx_c[i], acc2);
          }
        }
      }
      Store<T>::store1(xr + cslot_idx, est);
    }
    // ---- 4. the two tokens change parts --------------------------------------------
    if (tid == 0) {
      rp[c_slot] = J;
      vp[v_idx] = pc;
      if (swap_log) {
        swap_log[((size_t)unit * max_swaps + done) * 2] = J;
        swap_log[((size_t)unit * max_swaps + done) * 2 + 1] = pc;
      }
    }
    ++done;
    __syncthreads();             // the exchanged positions are visible to the next round's scans
  }
  if (tid == 0 && n_swapped) n_swapped[unit] = done;
}

hipError_t launch_swap_back(const DevDesc& d, int dtype, const float* scores, long long n_cap, void* k_ret,
                            void* v_ret, int32_t* ret_pos, int ret_cap, const int32_t* n_ctx, int n_recent,
                            float replace_rate, int max_swaps, void* sk, void* sv, int32_t* vague_pos,
                            const int32_t* n_vague, int vague_cap, int32_t* n_swapped, int32_t* swap_log,
                            hipStream_t st) {
  const dim3 grid(d.B * d.Hkv), block(SWP_THREADS);
  if (dtype == KVR_F32)
    hipLaunchKernelGGL(swap_back_kernel<float>, grid, block, 0, st, d, scores, n_cap, (float*)k_ret,
                       (float*)v_ret, ret_pos, ret_cap, n_ctx, n_recent, replace_rate, max_swaps, (float*)sk,
                       (float*)sv, vague_pos, n_vague, vague_cap, n_swapped, swap_log);
  else
    hipLaunchKernelGGL(swap_back_kernel<bf16_t>, grid, block, 0, st, d, scores, n_cap, (bf16_t*)k_ret,
                       (bf16_t*)v_ret, ret_pos, ret_cap, n_ctx, n_recent, replace_rate, max_swaps, (bf16_t*)sk,
                       (bf16_t*)sv, vague_pos, n_vague, vague_cap, n_swapped, swap_log);
  return hipGetLastError();
}

}  // namespace kvr
