// kvr_select: Recent / Candidate / Vague partition (Recent and Candidate,
// Algorithm 3 without the swap loop), and kvr_append (R.Push of the new token).
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
#include "kvr_launch.h"

namespace kvr {

constexpr int SEL_THREADS = 1024;
constexpr int SEL_WAVES = SEL_THREADS / WAVE;
constexpr int SEL_KPT = 8;                       // keys per thread held in registers
constexpr int SEL_REG_SLOTS = SEL_THREADS * SEL_KPT;
constexpr int SEL_SMALL = 8;                     // up to this many evictions: repeated minimum
constexpr unsigned long long KEY_NONE = ~0ull;   // no valid key is all ones (position bits would be ~pos of pos = 0 with score image all ones = NaN)

struct SelShared {
  unsigned hist[256];
  unsigned long long wmin[SEL_WAVES];
  unsigned long long prefix;
  int wsum[SEL_WAVES];
  int wscan[4];
  int krem, cnt, base;
};

__device__ __forceinline__ bool slot_key(const int32_t* __restrict__ rp, const float* __restrict__ sc,
                                         int slot, int ret_cap, int recent_from, long long n_cap,
                                         unsigned long long& key) {
  if (slot >= ret_cap) return false;
  const int pos = rp[slot];
  if (pos < 0 || pos >= recent_from || pos >= n_cap) return false;
  uint32_t b = __float_as_uint(sc[pos]);
  if (b == 0x80000000u) b = 0u;                                   // -0 ranks as +0
  const uint32_t mono = b ^ ((b >> 31) ? 0xffffffffu : 0x80000000u);
  key = ((unsigned long long)mono << 32) | (uint32_t)(~(uint32_t)pos);
  return true;
}

__device__ __forceinline__ int key_pos(unsigned long long key) { return (int)(~(uint32_t)key); }

__device__ __forceinline__ unsigned long long shfl_xor_u64(unsigned long long v, int m) {
  const uint32_t lo = __shfl_xor((int)(uint32_t)v, m), hi = __shfl_xor((int)(uint32_t)(v >> 32), m);
  return ((unsigned long long)hi << 32) | lo;
}

// Block-wide minimum of one value per thread (KEY_NONE = nothing).
__device__ __forceinline__ unsigned long long block_min(unsigned long long v, SelShared& sh) {
#pragma unroll
  for (int m = 1; m < WAVE; m <<= 1) {
    const unsigned long long o = shfl_xor_u64(v, m);
    v = o < v ? o : v;
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();                       // wmin may still be read from the previous round
  if (lane == 0) sh.wmin[wave] = v;
  __syncthreads();
  unsigned long long r = sh.wmin[0];
#pragma unroll
  for (int w_ = 1; w_ < SEL_WAVES; ++w_) r = sh.wmin[w_] < r ? sh.wmin[w_] : r;
  return r;
}

// 256 bins, scanned from the top: pick the bin where the running count reaches
// krem; updates sh.krem and ors the digit into sh.prefix.  All threads call it.
__device__ __forceinline__ void pick_digit(SelShared& sh, int byte) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int c = 0, incl = 0;
  if (tid < 256) {
    c = (int)sh.hist[255 - tid];
    incl = c;
#pragma unroll
    for (int off = 1; off < WAVE; off <<= 1) {
      const int y = __shfl_up(incl, off);
      if (lane >= off) incl += y;
    }
    if (lane == WAVE - 1) sh.wscan[wave] = incl;
  }
  __syncthreads();
  if (tid < 256) {
    int before = 0;
#pragma unroll
    for (int w_ = 0; w_ < 4; ++w_) before += (w_ < wave) ? sh.wscan[w_] : 0;
    incl += before;
    const int krem = sh.krem;
    if (incl >= krem && incl - c < krem) {          // exactly one thread
      sh.krem = krem - (incl - c);
      sh.prefix |= (unsigned long long)(255 - tid) << (8 * byte);
    }
  }
  __syncthreads();
}

template <bool REG>
__global__ __launch_bounds__(SEL_THREADS) void select_kernel(
    DevDesc d, const float* __restrict__ scores, long long n_cap, int32_t* __restrict__ ret_pos,
    int ret_cap, const int32_t* __restrict__ n_ctx, int n_recent, int k_cand,
    int32_t* __restrict__ evict_slot, int32_t* __restrict__ evict_pos, int32_t* __restrict__ n_evict,
    int evict_cap, int32_t* __restrict__ vague_pos, int32_t* __restrict__ n_vague, int vague_cap) {
  const int unit = blockIdx.x;
  const int b = unit / d.Hkv;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  int32_t* rp = ret_pos + (size_t)unit * ret_cap;
  const float* sc = scores + (size_t)unit * n_cap;
  const int recent_from = n_ctx[b] - n_recent;
  if (k_cand < 0) k_cand = 0;
  __shared__ SelShared sh;

  // keys of this thread's slots: slot = j * SEL_THREADS + tid
  unsigned long long rkey[REG ? SEL_KPT : 1];
  const int n_chunks = (ret_cap + SEL_THREADS - 1) / SEL_THREADS;
  auto get_key = [&](int j, unsigned long long& key) -> bool {
    if constexpr (REG) {
      key = rkey[j];
      return key != KEY_NONE;
    } else {
      return slot_key(rp, sc, j * SEL_THREADS + tid, ret_cap, recent_from, n_cap, key);
    }
  };

  if (tid == 0) { sh.cnt = 0; sh.base = 0; sh.prefix = 0ull; sh.krem = k_cand; }
  __syncthreads();
  {
    int c = 0;
    if constexpr (REG) {
#pragma unroll
      for (int j = 0; j < SEL_KPT; ++j) {
        unsigned long long key = KEY_NONE;
        const bool ok = slot_key(rp, sc, j * SEL_THREADS + tid, ret_cap, recent_from, n_cap, key);
        rkey[j] = ok ? key : KEY_NONE;
        c += ok ? 1 : 0;
      }
    } else {
      for (int j = 0; j < n_chunks; ++j) {
        unsigned long long key;
        c += get_key(j, key) ? 1 : 0;
      }
    }
    if (c) atomicAdd(&sh.cnt, c);
  }
  __syncthreads();
  const int n_e = sh.cnt - k_cand;
  if (n_e <= 0) {
    if (tid == 0) n_evict[unit] = 0;
    return;
  }
  const int nv_old = (vague_pos && n_vague) ? clampi(n_vague[unit], 0, vague_cap) : 0;
  if (n_e > evict_cap || (vague_pos && n_vague && nv_old + n_e > vague_cap)) {
    if (tid == 0) n_evict[unit] = -n_e;
    return;
  }

  // cut: evict every eligible key <= cut
  unsigned long long cut;
  if (k_cand == 0) {
    cut = KEY_NONE - 1;
  } else if (REG && n_e <= SEL_SMALL) {
    unsigned long long last = 0;
    bool have = false;
    for (int it = 0; it < n_e; ++it) {
      unsigned long long mine = KEY_NONE;
#pragma unroll
      for (int j = 0; j < (REG ? SEL_KPT : 1); ++j) {
        const unsigned long long key = rkey[j];
        if (key != KEY_NONE && (!have || key > last) && key < mine) mine = key;
      }
      last = block_min(mine, sh);
      have = true;
    }
    cut = last;
  } else {
    for (int byte = 7; byte >= 0; --byte) {
      if (tid < 256) sh.hist[tid] = 0u;
      __syncthreads();
      const unsigned long long prefix = sh.prefix;
#pragma unroll
      for (int j = 0; j < (REG ? SEL_KPT : n_chunks); ++j) {
        unsigned long long key;
        if (get_key(j, key)) {
          const bool match = (byte == 7) || ((key >> (8 * (byte + 1))) == (prefix >> (8 * (byte + 1))));
          if (match) atomicAdd(&sh.hist[(unsigned)(key >> (8 * byte)) & 255u], 1u);
        }
      }
      __syncthreads();
      pick_digit(sh, byte);
    }
    cut = sh.prefix - 1;       // prefix = the k-th largest key; it stays
  }

#pragma unroll
  for (int j = 0; j < (REG ? SEL_KPT : n_chunks); ++j) {
    if (REG && j >= n_chunks) break;
    const int slot = j * SEL_THREADS + tid;
    unsigned long long key = 0;
    bool flag = get_key(j, key);
    flag = flag && key <= cut;
    const unsigned long long bal = __ballot(flag);
    const int in_wave = __popcll(bal & ((1ull << lane) - 1ull));
    if (lane == 0) sh.wsum[wave] = __popcll(bal);
    __syncthreads();
    int before = 0, tot = 0;
#pragma unroll
    for (int w_ = 0; w_ < SEL_WAVES; ++w_) {
      const int c = sh.wsum[w_];
      before += (w_ < wave) ? c : 0;
      tot += c;
    }
    const int base = sh.base;
    if (flag) {
      const int idx = base + before + in_wave;      // < n_e <= evict_cap
      const int pos = key_pos(key);
      evict_slot[(size_t)unit * evict_cap + idx] = slot;
      evict_pos[(size_t)unit * evict_cap + idx] = pos;
      rp[slot] = -1;
      if (vague_pos && n_vague) vague_pos[(size_t)unit * vague_cap + nv_old + idx] = pos;
    }
    __syncthreads();
    if (tid == 0) sh.base = base + tot;
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
  if (ret_cap <= SEL_REG_SLOTS)
    hipLaunchKernelGGL(select_kernel<true>, dim3(d.B * d.Hkv), dim3(SEL_THREADS), 0, st, d, scores, n_cap,
                       ret_pos, ret_cap, n_ctx, n_recent, k_candidate, evict_slot, evict_pos, n_evict,
                       evict_cap, vague_pos, n_vague, vague_cap);
  else
    hipLaunchKernelGGL(select_kernel<false>, dim3(d.B * d.Hkv), dim3(SEL_THREADS), 0, st, d, scores, n_cap,
                       ret_pos, ret_cap, n_ctx, n_recent, k_candidate, evict_slot, evict_pos, n_evict,
                       evict_cap, vague_pos, n_vague, vague_cap);
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
  for (int s0 = 0; s0 < ret_cap; s0 += 256 * 8) {       // lowest empty slot, 8 independent loads a round
    int p[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int s = s0 + u * 256 + tid;
      p[u] = (s < ret_cap) ? rp[s] : 0;
    }
#pragma unroll
    for (int u = 7; u >= 0; --u) {
      const int s = s0 + u * 256 + tid;
      if (s < ret_cap && p[u] < 0 && s < mine) mine = s;
    }
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
