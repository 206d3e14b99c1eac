// Device bodies of the three small per-step updates of a unit's storage
// (Recent and Candidate, Algorithm 3; Vague Sketch, Algorithm 1):
//   append_body        R.Push of the new token into the lowest empty slot
//   select_body        which retained tokens leave for the Vague part
//   encode_small_body  V.Insert of up to 64 listed tokens
// Each is called by all threads of a workgroup for one unit.  The stand-alone
// kernels of kvr_append / kvr_select / kvr_encode and the fused kvr_step_update
// kernel are thin wrappers around them.
#pragma once
#include "kvr_dev.h"

namespace kvr {

constexpr int SEL_THREADS = 1024;
constexpr int SEL_WAVES = SEL_THREADS / WAVE;
constexpr int SEL_KPT = 8;                       // keys per thread held in registers
constexpr int SEL_REG_SLOTS = SEL_THREADS * SEL_KPT;
constexpr int SEL_SMALL = 8;                     // up to this many evictions: repeated minimum
constexpr unsigned long long KEY_NONE = ~0ull;   // not a valid key (it would be a NaN score at position 0)
constexpr int ENC_SMALL_CAP = 64;

struct SelShared {
  unsigned hist[256];
  unsigned long long wmin[SEL_WAVES];
  unsigned long long prefix;
  int wsum[SEL_WAVES];
  int wscan[4];
  int krem, cnt, base;
  int nlist, list[SEL_SMALL];        // small eviction counts: the evicted slots, in any order
};

// Eviction list of one unit in LDS: how the fused update kernel hands the selection's result to the
// insert without a round trip through global memory (the lists in global memory are written as well).
struct EvictHandOver {
  int cnt;                           // 0 if nothing is evicted or the lists would overflow
  int slot[ENC_SMALL_CAP];
  int pos[ENC_SMALL_CAP];
};

// ---------------------------------------------------------------------------
// append
// ---------------------------------------------------------------------------
// NT = threads of the workgroup.  Returns (in every thread) the slot used, or -1.
template <typename T, int NT>
__device__ __forceinline__ int append_body(const DevDesc& d, int unit, const T* __restrict__ k_new,
                                           const T* __restrict__ v_new, const int32_t* __restrict__ n_ctx,
                                           T* __restrict__ k_ret, T* __restrict__ v_ret,
                                           int32_t* __restrict__ ret_pos, int ret_cap) {
  constexpr int VEC = Store<T>::VEC;
  constexpr int LPT = D / VEC;     // 16 (bf16) or 32 (f32) lanes copy one row
  const int tid = threadIdx.x;
  int32_t* rp = ret_pos + (size_t)unit * ret_cap;
  __shared__ int s_free;
  if (tid == 0) s_free = 0x7fffffff;
  __syncthreads();
  int mine = 0x7fffffff;
  for (int s0 = 0; s0 < ret_cap; s0 += NT * 8) {       // lowest empty slot, 8 independent loads a round
    int p[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int s = s0 + u * NT + tid;
      p[u] = (s < ret_cap) ? rp[s] : 0;
    }
#pragma unroll
    for (int u = 7; u >= 0; --u) {
      const int s = s0 + u * NT + tid;
      if (s < ret_cap && p[u] < 0 && s < mine) mine = s;
    }
  }
  if (mine != 0x7fffffff) atomicMin(&s_free, mine);
  __syncthreads();
  const int s = s_free;
  if (s >= ret_cap) return -1;
  const size_t dst = ((size_t)unit * ret_cap + s) * D;
  if (tid < LPT) {
    const uint4 v = *reinterpret_cast<const uint4*>(k_new + (size_t)unit * D + tid * VEC);
    *reinterpret_cast<uint4*>(k_ret + dst + tid * VEC) = v;
  } else if (tid < 2 * LPT) {
    const int l2 = tid - LPT;
    const uint4 v = *reinterpret_cast<const uint4*>(v_new + (size_t)unit * D + l2 * VEC);
    *reinterpret_cast<uint4*>(v_ret + dst + l2 * VEC) = v;
  }
  if (tid == 0) rp[s] = n_ctx[unit / d.Hkv] - 1;
  return s;
}

// The same with the slot positions already in registers (pre[j] = ret_pos of slot
// j * NT + tid, or 0 for slots past ret_cap): no scan of ret_pos.
template <typename T, int NT, int KPT>
__device__ __forceinline__ int append_body_pre(const DevDesc& d, int unit, const T* __restrict__ k_new,
                                               const T* __restrict__ v_new, const int32_t* __restrict__ n_ctx,
                                               T* __restrict__ k_ret, T* __restrict__ v_ret,
                                               int32_t* __restrict__ ret_pos, int ret_cap, const int (&pre)[KPT],
                                               const uint4* row_in = nullptr) {
  // row_in (may be null): this thread's 16 bytes of the new K row (tid < LPT) or V row (tid < 2 LPT),
  // loaded by the caller ahead of time
  constexpr int VEC = Store<T>::VEC;
  constexpr int LPT = D / VEC;
  const int tid = threadIdx.x;
  int32_t* rp = ret_pos + (size_t)unit * ret_cap;
  __shared__ int s_free;
  if (tid == 0) s_free = 0x7fffffff;
  __syncthreads();
  int mine = 0x7fffffff;
#pragma unroll
  for (int j = KPT - 1; j >= 0; --j) {
    const int s = j * NT + tid;
    if (s < ret_cap && pre[j] < 0) mine = s;
  }
  if (mine != 0x7fffffff) atomicMin(&s_free, mine);
  __syncthreads();
  const int s = s_free;
  if (s >= ret_cap) return -1;
  const size_t dst = ((size_t)unit * ret_cap + s) * D;
  if (tid < LPT) {
    const uint4 v = row_in ? *row_in : *reinterpret_cast<const uint4*>(k_new + (size_t)unit * D + tid * VEC);
    *reinterpret_cast<uint4*>(k_ret + dst + tid * VEC) = v;
  } else if (tid < 2 * LPT) {
    const int l2 = tid - LPT;
    const uint4 v = row_in ? *row_in : *reinterpret_cast<const uint4*>(v_new + (size_t)unit * D + l2 * VEC);
    *reinterpret_cast<uint4*>(v_ret + dst + l2 * VEC) = v;
  }
  if (tid == 0) rp[s] = n_ctx[unit / d.Hkv] - 1;
  return s;
}

// ---------------------------------------------------------------------------
// select
// ---------------------------------------------------------------------------
// key of a slot whose position is already known
__device__ __forceinline__ bool pos_key(int pos, const float* __restrict__ sc, int slot, int ret_cap,
                                        int recent_from, long long n_cap, unsigned long long& key) {
  if (slot >= ret_cap) return false;
  if (pos < 0 || pos >= recent_from || pos >= n_cap) return false;
  uint32_t b = __float_as_uint(sc[pos]);
  if (b == 0x80000000u) b = 0u;                                   // -0 ranks as +0
  const uint32_t mono = b ^ ((b >> 31) ? 0xffffffffu : 0x80000000u);
  key = ((unsigned long long)mono << 32) | (uint32_t)(~(uint32_t)pos);
  return true;
}

// the same with the token's score already in a register (scv = scores[pos], read only if pos is eligible)
__device__ __forceinline__ bool pos_key_val(int pos, float scv, int slot, int ret_cap, int recent_from,
                                            long long n_cap, unsigned long long& key) {
  if (slot >= ret_cap) return false;
  if (pos < 0 || pos >= recent_from || pos >= n_cap) return false;
  uint32_t b = __float_as_uint(scv);
  if (b == 0x80000000u) b = 0u;                                   // -0 ranks as +0
  const uint32_t mono = b ^ ((b >> 31) ? 0xffffffffu : 0x80000000u);
  key = ((unsigned long long)mono << 32) | (uint32_t)(~(uint32_t)pos);
  return true;
}

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

// Workgroup of SEL_THREADS threads.  REG: ret_cap <= SEL_THREADS * KPT, keys live
// in registers (KPT per thread: 8 for the retained slots of a decode step, 32 for
// a 32k prompt).  Writes the eviction lists, frees the slots, appends to the Vague
// list, sets n_evict (negative = needed count on overflow, nothing evicted).
// pre (REG only, may be null): positions of this thread's slots, read by the caller
// ahead of time.  The fused update kernel reads them before it appends the new
// token: while that token is Recent it ranks like an empty slot, so the stale
// value serves; with an empty Recent window the kernel patches the one entry.
// pre_sc (with pre, may be null): the scores at those positions, gathered by the
// caller ahead of time (valid where the position is eligible).
template <bool REG, int KPT = SEL_KPT>
__device__ __forceinline__ void select_body(
    const DevDesc& d, int unit, const float* __restrict__ scores, long long n_cap,
    int32_t* __restrict__ ret_pos, int ret_cap, const int32_t* __restrict__ n_ctx, int n_recent, int k_cand,
    int32_t* __restrict__ evict_slot, int32_t* __restrict__ evict_pos, int32_t* __restrict__ n_evict,
    int evict_cap, int32_t* __restrict__ vague_pos, int32_t* __restrict__ n_vague, int vague_cap,
    const int* pre = nullptr, const float* pre_sc = nullptr, EvictHandOver* ho = nullptr) {
  const int b = unit / d.Hkv;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  int32_t* rp = ret_pos + (size_t)unit * ret_cap;
  const float* sc = scores + (size_t)unit * n_cap;
  const int recent_from = n_ctx[b] - n_recent;
  if (k_cand < 0) k_cand = 0;
  __shared__ SelShared sh;

  // keys of this thread's slots: slot = j * SEL_THREADS + tid
  unsigned long long rkey[REG ? KPT : 1];
  const int n_chunks = (ret_cap + SEL_THREADS - 1) / SEL_THREADS;
  auto get_key = [&](int j, unsigned long long& key) -> bool {
    if constexpr (REG) {
      key = rkey[j];
      return key != KEY_NONE;
    } else {
      return slot_key(rp, sc, j * SEL_THREADS + tid, ret_cap, recent_from, n_cap, key);
    }
  };

  if (tid == 0) { sh.cnt = 0; sh.base = 0; sh.prefix = 0ull; sh.krem = k_cand; sh.nlist = 0; }
  __syncthreads();
  {
    int c = 0;
    if constexpr (REG) {
#pragma unroll
      for (int j = 0; j < KPT; ++j) {
        unsigned long long key = KEY_NONE;
        const bool ok = pre_sc ? pos_key_val(pre[j], pre_sc[j], j * SEL_THREADS + tid, ret_cap, recent_from, n_cap, key)
                        : pre  ? pos_key(pre[j], sc, j * SEL_THREADS + tid, ret_cap, recent_from, n_cap, key)
                               : slot_key(rp, sc, j * SEL_THREADS + tid, ret_cap, recent_from, n_cap, key);
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
    if (tid == 0) {
      n_evict[unit] = 0;
      if (ho) ho->cnt = 0;
    }
    return;
  }
  const int nv_old = (vague_pos && n_vague) ? clampi(n_vague[unit], 0, vague_cap) : 0;
  if (n_e > evict_cap || (vague_pos && n_vague && nv_old + n_e > vague_cap)) {
    if (tid == 0) {
      n_evict[unit] = -n_e;
      if (ho) ho->cnt = 0;
    }
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
      for (int j = 0; j < (REG ? KPT : 1); ++j) {
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
      for (int j = 0; j < (REG ? KPT : n_chunks); ++j) {
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

  if (REG && n_e <= SEL_SMALL) {
    // a handful of evictions: the owners put their slots into a short list (any
    // order), and each then takes the rank of its slot as its place in the output
    if constexpr (REG) {
#pragma unroll
      for (int j = 0; j < KPT; ++j)
        if (rkey[j] != KEY_NONE && rkey[j] <= cut) sh.list[atomicAdd(&sh.nlist, 1)] = j * SEL_THREADS + tid;
      __syncthreads();
#pragma unroll
      for (int j = 0; j < KPT; ++j) {
        if (rkey[j] != KEY_NONE && rkey[j] <= cut) {
          const int slot = j * SEL_THREADS + tid;
          int idx = 0;
          for (int x = 0; x < n_e; ++x) idx += (sh.list[x] < slot) ? 1 : 0;
          const int pos = key_pos(rkey[j]);
          evict_slot[(size_t)unit * evict_cap + idx] = slot;
          evict_pos[(size_t)unit * evict_cap + idx] = pos;
          if (ho && idx < ENC_SMALL_CAP) { ho->slot[idx] = slot; ho->pos[idx] = pos; }
          rp[slot] = -1;
          if (vague_pos && n_vague) vague_pos[(size_t)unit * vague_cap + nv_old + idx] = pos;
        }
      }
    }
    if (tid == 0) {
      n_evict[unit] = n_e;
      if (ho) ho->cnt = n_e;
      if (vague_pos && n_vague) n_vague[unit] = nv_old + n_e;
    }
    return;
  }

#pragma unroll
  for (int j = 0; j < (REG ? KPT : n_chunks); ++j) {
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
      if (ho && idx < ENC_SMALL_CAP) { ho->slot[idx] = slot; ho->pos[idx] = pos; }
      rp[slot] = -1;
      if (vague_pos && n_vague) vague_pos[(size_t)unit * vague_cap + nv_old + idx] = pos;
    }
    __syncthreads();
    if (tid == 0) sh.base = base + tot;
    __syncthreads();
  }
  if (tid == 0) {
    n_evict[unit] = n_e;
    if (ho) ho->cnt = n_e;
    if (vague_pos && n_vague) n_vague[unit] = nv_old + n_e;
  }
}

// ---------------------------------------------------------------------------
// encode, up to ENC_SMALL_CAP listed tokens
// ---------------------------------------------------------------------------
// Called by a workgroup of at least D threads; the hashes of the listed tokens go
// to LDS, then thread (row group, channel) walks the list and owns the slots it
// meets first (list order = summation order, one rounding per slot).
template <typename T>
__device__ __forceinline__ void encode_small_body(
    const DevDesc& d, int unit, const T* __restrict__ k_src, const T* __restrict__ v_src, int src_rows,
    const int32_t* __restrict__ src_slot, const int32_t* __restrict__ tok_pos,
    const int32_t* __restrict__ count, int cap, T* __restrict__ sk, T* __restrict__ sv,
    int32_t* __restrict__ out_bucket, uint8_t* __restrict__ out_sign, const EvictHandOver* ho = nullptr) {
  __shared__ int s_bucket[ENC_SMALL_CAP][KVR_MAX_ROWS];
  __shared__ int s_slot[ENC_SMALL_CAP];
  __shared__ unsigned s_sign[ENC_SMALL_CAP];
  const int tid = threadIdx.x;
  // the list comes from LDS when the selection ran in this workgroup just before (fused update)
  const int cnt = clampi(ho ? ho->cnt : count[unit], 0, min(cap, ENC_SMALL_CAP));
  if (tid < cnt) {
    const int J = ho ? ho->pos[tid] : tok_pos[(size_t)unit * cap + tid];
    const int slot = ho ? ho->slot[tid] : src_slot[(size_t)unit * cap + tid];
    s_slot[tid] = (slot >= 0 && slot < src_rows) ? slot : -1;
    unsigned sg = 0;
    for (int i = 0; i < d.r; ++i) {
      const int bk = bucket_of(d, i, J);
      s_bucket[tid][i] = bk;
      if (sign_neg(d, i, J)) sg |= 1u << i;
      if (out_bucket) out_bucket[((size_t)unit * cap + tid) * d.r + i] = bk;
    }
    s_sign[tid] = sg;
    if (out_sign) out_sign[(size_t)unit * cap + tid] = (uint8_t)sg;
  }
  __syncthreads();
  // thread = (row group, channel): rows i0, i0 + groups, ... (groups = blockDim / D)
  const int c = tid % D;
  const int groups = blockDim.x / D;
  const int i0 = tid / D;
  if (i0 >= groups) return;
  const bool fk = (d.sign_mask & 1) != 0, fv = (d.sign_mask & 2) != 0;
  for (int i = i0; i < d.r; i += groups) {
    for (int e = 0; e < cnt; ++e) {
      if (s_slot[e] < 0) continue;
      const int bk = s_bucket[e][i];
      bool first = true;
      for (int e2 = 0; e2 < e; ++e2) first = first && !(s_slot[e2] >= 0 && s_bucket[e2][i] == bk);
      if (!first) continue;
      const size_t idx = (((size_t)unit * d.r + i) * d.w + bk) * D + c;
      float ak = Store<T>::load1(sk + idx), av = Store<T>::load1(sv + idx);
      for (int e2 = e; e2 < cnt; ++e2) {
        if (s_slot[e2] >= 0 && s_bucket[e2][i] == bk) {
          const bool neg = (s_sign[e2] >> i) & 1u;
          const size_t src = ((size_t)unit * src_rows + s_slot[e2]) * D + c;
          const float kv = Store<T>::load1(k_src + src), vv = Store<T>::load1(v_src + src);
          ak += (fk && neg) ? -kv : kv;
          av += (fv && neg) ? -vv : vv;
        }
      }
      Store<T>::store1(sk + idx, ak);
      Store<T>::store1(sv + idx, av);
    }
  }
}

}  // namespace kvr
