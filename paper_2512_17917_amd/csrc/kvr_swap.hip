// kvr_swap_back: the swap loop of Algorithm 3 (Recent and Candidate; its second
// while-loop): as long as the weakest Candidate's score times ReplaceRate is below
// the strongest Vague token's score, that Vague token is queried from the sketch
// and deleted from it, the Candidate is popped and inserted into the sketch, and
// the queried estimate is pushed into the Candidate part in its place.
//
// One workgroup per unit, at most max_swaps rounds.
//
// Ranking.  Every token gets the 64-bit key
//     (order-preserving image of its float32 score) << 32 | ~position,
// the key kvr_select ranks by: "highest score, then earlier position" is the
// largest key, "lowest score, then later position" the smallest, and all keys are
// distinct.  V.Max is the largest key of the Vague index list, C.Min the smallest
// key of the retained slots outside the Recent window.
//
// One scan serves many rounds.  The keys are loaded once (REG: into registers, up
// to 26 Vague tokens and 8 slots per thread; otherwise they are re-read from
// memory), and the m = min(max_swaps, 16) largest Vague keys and m smallest
// Candidate keys are extracted by m workgroup-wide reductions into two sorted
// lists in LDS.  A swap pops both heads and inserts each token's key into the
// other list; since a round removes only the head, the head of a list stays the
// true extreme of its part for m rounds (the j-th extreme of the scanned part is
// in the list for j <= m, and every key that entered the part since is in it
// too).  After m swaps the parts are scanned again.
//
// A swap.  Thread c < D owns channel c of the key tensors, thread D + c channel c
// of the value tensors: it reads its channel of the r sketch rows of the Vague
// token, takes the median (Algorithm 2), reads the Candidate's channel, writes
// sketch = round(float32(old) - estimate) and round(float32(old) + candidate)
// (one sum, one rounding, if both fall into the same slot of a row: delete first,
// then insert), and stores the estimate into the Candidate's slot.  A channel is
// only ever touched by its own thread, so no barrier is needed between the query
// and the update.  Thread 0 exchanges the two positions in ret_pos / vague_pos.
#include "kvr_launch.h"

namespace kvr {

constexpr int SWP_THREADS = 1024;
constexpr int SWP_WAVES = SWP_THREADS / WAVE;
constexpr int SWP_KV = 26;                             // REG: Vague keys per thread
constexpr int SWP_KC = 8;                              // REG: slot keys per thread
constexpr int SWP_LIST = 16;                           // list length per scan
constexpr unsigned long long SWP_NONE_MAX = 0ull;      // below every key (the low word ~position of a key is never 0)
constexpr unsigned long long SWP_NONE_MIN = ~0ull;     // above every key of a finite score

struct SwapShared {
  unsigned long long wmax[2][SWP_WAVES], wmin[2][SWP_WAVES];
  unsigned long long vkey[SWP_LIST + 1], ckey[SWP_LIST + 1];   // sorted: vkey descending, ckey ascending
  int vidx[SWP_LIST + 1], cslot[SWP_LIST + 1];                 // Vague list index / retained slot of each entry
  int nvl, ncl;                                                // entries in use
  int go;                                                      // swaps decided for this scan
  int dec[SWP_LIST][4];                                        // per swap: Vague position, Candidate position, list index, slot
};

// key of (score, position): larger = higher score, then earlier position.  -0 ranks as +0.
// Never 0 and never ~0 for a valid position (0 <= pos < 2^30) and a finite score.
__device__ __forceinline__ unsigned long long swap_key(float score, int pos) {
  uint32_t b = __float_as_uint(score);
  if (b == 0x80000000u) b = 0u;
  const uint32_t mono = b ^ ((b >> 31) ? 0xffffffffu : 0x80000000u);
  return ((unsigned long long)mono << 32) | (uint32_t)(~(uint32_t)pos);
}
// the score a key was made from (-0 comes back as +0, which compares and multiplies alike)
__device__ __forceinline__ float key_score(unsigned long long key) {
  const uint32_t mono = (uint32_t)(key >> 32);
  return __uint_as_float(mono ^ ((mono >> 31) ? 0x80000000u : 0xffffffffu));
}

__device__ __forceinline__ unsigned long long shfl_xor_u64s(unsigned long long v, int m) {
  const uint32_t lo = __shfl_xor((int)(uint32_t)v, m), hi = __shfl_xor((int)(uint32_t)(v >> 32), m);
  return ((unsigned long long)hi << 32) | lo;
}

__device__ __forceinline__ unsigned long long vague_key_at(const int32_t* vp, const float* sc, int i, int nv,
                                                           long long n_cap) {
  if (i >= nv) return SWP_NONE_MAX;
  const int pos = vp[i];
  return (pos >= 0 && pos < n_cap) ? swap_key(sc[pos], pos) : SWP_NONE_MAX;
}
__device__ __forceinline__ unsigned long long cand_key_at(const int32_t* rp, const float* sc, int s, int ret_cap,
                                                          int recent_from, long long n_cap) {
  if (s >= ret_cap) return SWP_NONE_MIN;
  const int pos = rp[s];
  return (pos >= 0 && pos < recent_from && pos < n_cap) ? swap_key(sc[pos], pos) : SWP_NONE_MIN;
}

// Scan both parts of a unit and leave the m largest Vague keys and the m
// smallest Candidate keys, in order, in sh (with the Vague list index / the
// retained slot of each).  Not inlined: the keys it holds in registers (REG) are
// dead when it returns and must not count against the caller's registers.
template <bool REG>
__device__ __noinline__ void swap_build_lists(SwapShared& sh, const int32_t* vp, const int32_t* rp,
                                              const float* sc, int nv, int ret_cap, int recent_from,
                                              long long n_cap, int m) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  unsigned long long vk[REG ? SWP_KV : 1], ck[REG ? SWP_KC : 1];
  if constexpr (REG) {
    // all positions first, then all scores (clamped addresses, no branches): two
    // rounds of independent loads instead of one dependent pair per token
    int pv[SWP_KV], pc[SWP_KC];
#pragma unroll
    for (int j = 0; j < SWP_KV; ++j) {
      const int i = j * SWP_THREADS + tid;
      pv[j] = vp[min(i, max(nv - 1, 0))];
      if (i >= nv || pv[j] >= n_cap) pv[j] = -1;
    }
#pragma unroll
    for (int j = 0; j < SWP_KC; ++j) {
      const int s_ = j * SWP_THREADS + tid;
      pc[j] = rp[min(s_, ret_cap - 1)];
      if (s_ >= ret_cap || pc[j] >= recent_from || pc[j] >= n_cap) pc[j] = -1;
    }
    float sv_[SWP_KV], sc_[SWP_KC];
#pragma unroll
    for (int j = 0; j < SWP_KV; ++j) sv_[j] = sc[max(pv[j], 0)];
#pragma unroll
    for (int j = 0; j < SWP_KC; ++j) sc_[j] = sc[max(pc[j], 0)];
#pragma unroll
    for (int j = 0; j < SWP_KV; ++j) vk[j] = pv[j] >= 0 ? swap_key(sv_[j], pv[j]) : SWP_NONE_MAX;
#pragma unroll
    for (int j = 0; j < SWP_KC; ++j) ck[j] = pc[j] >= 0 ? swap_key(sc_[j], pc[j]) : SWP_NONE_MIN;
  }
  // A thread offers the best key it still has; only the thread whose key was taken
  // looks for its next one (the taken keys are exactly those beyond the last extreme).
  unsigned long long vprev = SWP_NONE_MIN, cprev = SWP_NONE_MAX;       // previous extremes (exclusive bounds)
  int n_vl = 0, n_cl = 0;
  unsigned long long kmax = SWP_NONE_MAX, kmin = SWP_NONE_MIN;
  int imax = -1, smin = -1;
  bool redo_v = true, redo_c = true;
  for (int k = 0; k < m; ++k) {
    if (redo_v) {
      kmax = SWP_NONE_MAX;
      imax = -1;
      if constexpr (REG) {
#pragma unroll
        for (int j = 0; j < SWP_KV; ++j)
          if (vk[j] < vprev && vk[j] > kmax) { kmax = vk[j]; imax = j * SWP_THREADS + tid; }
      } else {
        for (int i = tid; i < nv; i += SWP_THREADS) {
          const unsigned long long key = vague_key_at(vp, sc, i, nv, n_cap);
          if (key < vprev && key > kmax) { kmax = key; imax = i; }
        }
      }
      redo_v = false;
    }
    if (redo_c) {
      kmin = SWP_NONE_MIN;
      smin = -1;
      if constexpr (REG) {
#pragma unroll
        for (int j = 0; j < SWP_KC; ++j)
          if (ck[j] > cprev && ck[j] < kmin) { kmin = ck[j]; smin = j * SWP_THREADS + tid; }
      } else {
        for (int s_ = tid; s_ < ret_cap; s_ += SWP_THREADS) {
          const unsigned long long key = cand_key_at(rp, sc, s_, ret_cap, recent_from, n_cap);
          if (key > cprev && key < kmin) { kmin = key; smin = s_; }
        }
      }
      redo_c = false;
    }
    unsigned long long wmx = kmax, wmn = kmin;
#pragma unroll
    for (int x = 1; x < WAVE; x <<= 1) {
      const unsigned long long o1 = shfl_xor_u64s(wmx, x), o2 = shfl_xor_u64s(wmn, x);
      wmx = o1 > wmx ? o1 : wmx;
      wmn = o2 < wmn ? o2 : wmn;
    }
    if (lane == 0) { sh.wmax[k & 1][wave] = wmx; sh.wmin[k & 1][wave] = wmn; }
    __syncthreads();
    unsigned long long gmax = sh.wmax[k & 1][0], gmin = sh.wmin[k & 1][0];
#pragma unroll
    for (int w_ = 1; w_ < SWP_WAVES; ++w_) {
      gmax = sh.wmax[k & 1][w_] > gmax ? sh.wmax[k & 1][w_] : gmax;
      gmin = sh.wmin[k & 1][w_] < gmin ? sh.wmin[k & 1][w_] : gmin;
    }
    // keys are distinct: each extreme has exactly one owner
    if (gmax != SWP_NONE_MAX) {
      if (kmax == gmax) { sh.vkey[n_vl] = gmax; sh.vidx[n_vl] = imax; redo_v = true; }
      ++n_vl;
      vprev = gmax;
    }
    if (gmin != SWP_NONE_MIN) {
      if (kmin == gmin) { sh.ckey[n_cl] = gmin; sh.cslot[n_cl] = smin; redo_c = true; }
      ++n_cl;
      cprev = gmin;
    }
    if (gmax == SWP_NONE_MAX && gmin == SWP_NONE_MIN) break;             // both parts exhausted (uniform)
  }
  if (tid == 0) { sh.nvl = n_vl; sh.ncl = n_cl; }
  __syncthreads();
}

template <typename T, bool REG>
__global__ __launch_bounds__(SWP_THREADS) void swap_back_kernel(
    DevDesc d, const float* __restrict__ scores, long long n_cap, T* k_ret, T* v_ret, int32_t* ret_pos,
    int ret_cap, const int32_t* __restrict__ n_ctx, int n_recent, float replace_rate, int max_swaps, T* sk,
    T* sv, int32_t* vague_pos, const int32_t* __restrict__ n_vague, int vague_cap,
    int32_t* __restrict__ n_swapped, int32_t* __restrict__ swap_log) {
  const int unit = blockIdx.x;
  const int b = unit / d.Hkv;
  const int tid = threadIdx.x;
  __shared__ SwapShared sh;
  int32_t* rp = ret_pos + (size_t)unit * ret_cap;
  int32_t* vp = vague_pos + (size_t)unit * vague_cap;
  const float* sc = scores + (size_t)unit * n_cap;
  const int recent_from = n_ctx[b] - n_recent;
  const int nv = clampi(n_vague[unit], 0, vague_cap);
  int done = 0;

  while (done < max_swaps) {
    const int m = min(max_swaps - done, SWP_LIST);
    swap_build_lists<REG>(sh, vp, rp, sc, nv, ret_cap, recent_from, n_cap, m);

    // ---- up to m swaps on the lists.  Which tokens change places depends on scores and
    //      positions only, not on sketch contents: thread 0 decides all swaps of this scan
    //      first and leaves the pairs in LDS, then the channel threads carry them out one
    //      after the other without a barrier in between (a later swap that touches a slot
    //      or a retained row of an earlier one is ordered by the thread's own program
    //      order: a channel is only ever touched by its own thread). -------------------------
    if (tid == 0) {
      int n_dec = 0;
      for (int k = 0; k < m; ++k) {
        if (sh.nvl <= 0 || sh.ncl <= 0) break;
        const unsigned long long kv = sh.vkey[0], kc = sh.ckey[0];
        const float lhs = key_score(kc) * replace_rate;                   // float32 product, float32 compare
        if (!(lhs < key_score(kv))) break;
        const int v_idx = sh.vidx[0], c_slot = sh.cslot[0];
        sh.dec[n_dec][0] = (int)(~(uint32_t)kv);
        sh.dec[n_dec][1] = (int)(~(uint32_t)kc);
        sh.dec[n_dec][2] = v_idx;
        sh.dec[n_dec][3] = c_slot;
        ++n_dec;
        // pop both heads; the Candidate's key enters the Vague list (at the Vague token's list
        // index), the Vague token's key enters the Candidate list (in the Candidate's slot)
        int n = sh.nvl - 1, at = 0;
        for (int i = 0; i < n; ++i) { sh.vkey[i] = sh.vkey[i + 1]; sh.vidx[i] = sh.vidx[i + 1]; }
        while (at < n && sh.vkey[at] > kc) ++at;
        for (int i = n; i > at; --i) { sh.vkey[i] = sh.vkey[i - 1]; sh.vidx[i] = sh.vidx[i - 1]; }
        sh.vkey[at] = kc;
        sh.vidx[at] = v_idx;
        n = sh.ncl - 1;
        at = 0;
        for (int i = 0; i < n; ++i) { sh.ckey[i] = sh.ckey[i + 1]; sh.cslot[i] = sh.cslot[i + 1]; }
        while (at < n && sh.ckey[at] < kv) ++at;
        for (int i = n; i > at; --i) { sh.ckey[i] = sh.ckey[i - 1]; sh.cslot[i] = sh.cslot[i - 1]; }
        sh.ckey[at] = kv;
        sh.cslot[at] = c_slot;
      }
      sh.go = n_dec;
    }
    __syncthreads();
    const int swaps_here = sh.go;
    const bool stop = swaps_here < m;                                       // the loop condition failed (uniform)
    for (int k = 0; k < swaps_here; ++k) {
      const int J = sh.dec[k][0], pc = sh.dec[k][1], v_idx = sh.dec[k][2], c_slot = sh.dec[k][3];
      if (tid < 2 * D) {
        const bool is_v = tid >= D;
        const int c = is_v ? tid - D : tid;
        T* sx = (is_v ? sv : sk) + (size_t)unit * d.r * d.w * D + c;
        T* xr = (is_v ? v_ret : k_ret) + ((size_t)unit * ret_cap + c_slot) * D + c;
        const bool flip = is_v ? (d.sign_mask & 2) != 0 : (d.sign_mask & 1) != 0;
        // every value the update needs is requested before any is used: one round trip
        int off_d[KVR_MAX_ROWS], off_c[KVR_MAX_ROWS];
        float old_d[KVR_MAX_ROWS], old_c[KVR_MAX_ROWS], rows[KVR_MAX_ROWS];
#pragma unroll
        for (int i = 0; i < KVR_MAX_ROWS; ++i) {
          off_d[i] = off_c[i] = 0;
          old_d[i] = old_c[i] = 0.f;
          if (i < d.r) {
            off_d[i] = (i * d.w + bucket_of(d, i, J)) * D;
            off_c[i] = (i * d.w + bucket_of(d, i, pc)) * D;
            old_d[i] = Store<T>::load1(sx + off_d[i]);
            old_c[i] = Store<T>::load1(sx + off_c[i]);
          }
        }
        const float cand = Store<T>::load1(xr);
#pragma unroll
        for (int i = 0; i < KVR_MAX_ROWS; ++i)
          rows[i] = (i < d.r && flip && sign_neg(d, i, J)) ? -old_d[i] : old_d[i];
        const float est = median_rows<0, T>(rows, d.r, d.median_mode);
#pragma unroll
        for (int i = 0; i < KVR_MAX_ROWS; ++i) {
          if (i < d.r) {
            // delete first, then insert; float32 sums, one rounding per touched slot
            const float gd = (flip && sign_neg(d, i, J)) ? -1.f : 1.f;
            const float gc = (flip && sign_neg(d, i, pc)) ? -1.f : 1.f;
            float acc = old_d[i] + (-gd) * est;
            if (off_c[i] == off_d[i]) {
              acc = acc + gc * cand;
              Store<T>::store1(sx + off_d[i], acc);
            } else {
              Store<T>::store1(sx + off_d[i], acc);
              Store<T>::store1(sx + off_c[i], old_c[i] + gc * cand);
            }
          }
        }
        Store<T>::store1(xr, est);
      }
      if (tid == 0) {
        rp[c_slot] = J;
        vp[v_idx] = pc;
        if (swap_log) {
          swap_log[((size_t)unit * max_swaps + done + k) * 2] = J;
          swap_log[((size_t)unit * max_swaps + done + k) * 2 + 1] = pc;
        }
      }
    }
    __syncthreads();             // sh.go / the pairs may be overwritten; positions visible to a later scan
    done += swaps_here;
    if (stop) break;
  }
  if (tid == 0 && n_swapped) n_swapped[unit] = done;
}

template <typename T>
static void launch_swap_t(const DevDesc& d, const float* scores, long long n_cap, void* k_ret, void* v_ret,
                          int32_t* ret_pos, int ret_cap, const int32_t* n_ctx, int n_recent, float replace_rate,
                          int max_swaps, void* sk, void* sv, int32_t* vague_pos, const int32_t* n_vague,
                          int vague_cap, int32_t* n_swapped, int32_t* swap_log, hipStream_t st) {
  const dim3 grid(d.B * d.Hkv), block(SWP_THREADS);
  // keys in registers when both parts fit (vague_cap bounds n_vague)
  if (vague_cap <= SWP_KV * SWP_THREADS && ret_cap <= SWP_KC * SWP_THREADS)
    hipLaunchKernelGGL((swap_back_kernel<T, true>), grid, block, 0, st, d, scores, n_cap, (T*)k_ret, (T*)v_ret,
                       ret_pos, ret_cap, n_ctx, n_recent, replace_rate, max_swaps, (T*)sk, (T*)sv, vague_pos,
                       n_vague, vague_cap, n_swapped, swap_log);
  else
    hipLaunchKernelGGL((swap_back_kernel<T, false>), grid, block, 0, st, d, scores, n_cap, (T*)k_ret, (T*)v_ret,
                       ret_pos, ret_cap, n_ctx, n_recent, replace_rate, max_swaps, (T*)sk, (T*)sv, vague_pos,
                       n_vague, vague_cap, n_swapped, swap_log);
}

hipError_t launch_swap_back(const DevDesc& d, int dtype, const float* scores, long long n_cap, void* k_ret,
                            void* v_ret, int32_t* ret_pos, int ret_cap, const int32_t* n_ctx, int n_recent,
                            float replace_rate, int max_swaps, void* sk, void* sv, int32_t* vague_pos,
                            const int32_t* n_vague, int vague_cap, int32_t* n_swapped, int32_t* swap_log,
                            hipStream_t st) {
  if (dtype == KVR_F32)
    launch_swap_t<float>(d, scores, n_cap, k_ret, v_ret, ret_pos, ret_cap, n_ctx, n_recent, replace_rate,
                         max_swaps, sk, sv, vague_pos, n_vague, vague_cap, n_swapped, swap_log, st);
  else
    launch_swap_t<bf16_t>(d, scores, n_cap, k_ret, v_ret, ret_pos, ret_cap, n_ctx, n_recent, replace_rate,
                          max_swaps, sk, sv, vague_pos, n_vague, vague_cap, n_swapped, swap_log, st);
  return hipGetLastError();
}

}  // namespace kvr
