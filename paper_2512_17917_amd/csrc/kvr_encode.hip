// kvr_encode: batched V.Insert (Vague Sketch, Algorithm 1) without global
// atomics and with a fixed summation order, so the stored sketch is
// reproducible bit for bit: every touched slot = round_to_storage(float32(old
// content) + contributions in list order, added left to right in float32).
//
// Two regimes.
//   small (cap <= 64, the steady state of decode: about one eviction per unit
//     per step): one workgroup per unit; hashes of the listed tokens go to LDS,
//     then every (row, channel) thread walks the list and owns the slots it meets
//     first.
//   bulk (cap > 64, compressing a prompt): hash all tokens, counting-sort the
//     token ordinals of each (unit, row) by slot (stable, so list order survives
//     inside a slot), then one wave per (unit, row, slot) adds its segment
//     sequentially, lanes across channels.
#include "kvr_launch.h"
#include "kvr_update.h"

namespace kvr {

constexpr int ENC_BULK_MAX_W = 8192;     // LDS cursor array of the sort kernel

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

EncodePlan encode_plan(const DevDesc& d, long long cap) {
  EncodePlan p;
  p.bulk = cap > ENC_SMALL_CAP;
  p.off_bucket = p.off_order = p.off_start = 0;
  p.total_bytes = 0;
  if (p.bulk) {
    const size_t ur = (size_t)d.B * d.Hkv * d.r;
    size_t off = 0;
    p.off_bucket = off;
    off = align_up(off + ur * (size_t)cap * sizeof(int32_t), 256);
    p.off_order = off;
    off = align_up(off + ur * (size_t)cap * sizeof(int32_t), 256);
    p.off_start = off;
    off = align_up(off + ur * (size_t)(d.w + 1) * sizeof(int32_t), 256);
    p.total_bytes = off;
  }
  return p;
}

// ------------------------------------------------------------------ small
template <typename T>
__global__ __launch_bounds__(4 * D) void encode_small_kernel(
    DevDesc d, const T* __restrict__ k_src, const T* __restrict__ v_src, int src_rows,
    const int32_t* __restrict__ src_slot, const int32_t* __restrict__ tok_pos,
    const int32_t* __restrict__ count, int cap, T* __restrict__ sk, T* __restrict__ sv,
    int32_t* __restrict__ out_bucket, uint8_t* __restrict__ out_sign) {
  encode_small_body<T>(d, blockIdx.x, k_src, v_src, src_rows, src_slot, tok_pos, count, cap, sk, sv, out_bucket,
                       out_sign);
}

// ------------------------------------------------------------------ bulk
__global__ __launch_bounds__(256) void encode_hash_kernel(
    DevDesc d, int src_rows, const int32_t* __restrict__ src_slot, const int32_t* __restrict__ tok_pos,
    const int32_t* __restrict__ count, int cap, int32_t* __restrict__ ws_bucket,
    int32_t* __restrict__ out_bucket, uint8_t* __restrict__ out_sign) {
  const int unit = blockIdx.y;
  const int e = blockIdx.x * 256 + threadIdx.x;
  const int cnt = clampi(count[unit], 0, cap);
  if (e >= cnt) return;
  const int J = tok_pos[(size_t)unit * cap + e];
  const int slot = src_slot[(size_t)unit * cap + e];
  const bool ok = slot >= 0 && slot < src_rows;
  unsigned sg = 0;
  for (int i = 0; i < d.r; ++i) {
    const int bk = bucket_of(d, i, J);
    ws_bucket[((size_t)unit * d.r + i) * cap + e] = ok ? bk : -1;
    if (sign_neg(d, i, J)) sg |= 1u << i;
    if (out_bucket) out_bucket[((size_t)unit * cap + e) * d.r + i] = bk;
  }
  if (out_sign) out_sign[(size_t)unit * cap + e] = (uint8_t)sg;
}

// One workgroup per (unit, row): stable counting sort of token ordinals by slot.
// The list is cut into one contiguous segment per wave.
//   1. every wave counts its segment's slots in a row of its own (LDS atomics:
//      order does not matter for a count);
//   2. per slot, the segment counts are turned into running offsets, the slot
//      totals are scanned into start[], and row g of the table becomes the write
//      cursor of slot s for segment g;
//   3. every wave walks its segment 64 tokens at a time, in order: a token's
//      place is its slot's cursor plus the number of lower lanes with the same
//      slot, and the highest lane of each slot moves the cursor on.  Waves work
//      on disjoint rows of the table and on disjoint ranges of the output, so
//      there is no barrier inside the walk.
// A slot's tokens come out in list order, which fixes the summation order.  What
// is written per token is its source row with the sign of this sketch row in
// the top bit (source rows are below 2^30).
constexpr int SORT_MAX_SEGS = 16;
constexpr int SORT_LDS_INTS = 15360;       // 60 KB of table: segs * w + w <= this

static int sort_segments(int w) {
  int segs = (SORT_LDS_INTS - w) / w;
  if (segs > SORT_MAX_SEGS) segs = SORT_MAX_SEGS;
  if (segs < 1) segs = 1;
  return segs;
}

__global__ __launch_bounds__(SORT_MAX_SEGS * WAVE) void encode_sort_kernel(
    DevDesc d, const int32_t* __restrict__ count, int cap, const int32_t* __restrict__ ws_bucket,
    const int32_t* __restrict__ src_slot, const int32_t* __restrict__ tok_pos,
    int32_t* __restrict__ ws_order, int32_t* __restrict__ ws_start) {
  extern __shared__ int s_tab[];             // [segs][w] counts / cursors, then [w] totals / starts
  const int w = d.w;
  const int segs = blockDim.x / WAVE;
  int* s_tot = s_tab + segs * w;
  const int ur = blockIdx.x;                 // unit * r + row
  const int unit = ur / d.r, row = ur % d.r;
  const int tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid / WAVE;
  const int cnt = clampi(count[unit], 0, cap);
  const int32_t* bk = ws_bucket + (size_t)ur * cap;
  int32_t* order = ws_order + (size_t)ur * cap;
  int32_t* start = ws_start + (size_t)ur * (w + 1);
  // segment of this wave: whole 64-token chunks
  const int chunks = (cnt + WAVE - 1) / WAVE;
  const int per = (chunks + segs - 1) / segs;
  const int lo = min(wave * per * WAVE, cnt), hi = min((wave + 1) * per * WAVE, cnt);
  for (int i = tid; i < segs * w; i += blockDim.x) s_tab[i] = 0;
  __syncthreads();
  int* mine = s_tab + wave * w;
  for (int e0 = lo + lane; e0 < hi; e0 += 8 * WAVE) {      // eight loads in flight per lane
    int s8[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) s8[u] = (e0 + u * WAVE < hi) ? bk[e0 + u * WAVE] : -1;
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (s8[u] >= 0) atomicAdd(&mine[s8[u]], 1);
  }
  __syncthreads();
  for (int s = tid; s < w; s += blockDim.x) {
    int run = 0;
    for (int g = 0; g < segs; ++g) {
      const int t = s_tab[g * w + s];
      s_tab[g * w + s] = run;
      run += t;
    }
    s_tot[s] = run;
  }
  __syncthreads();
  if (wave == 0) {                            // exclusive scan of the slot totals
    int carry = 0;
    for (int s0 = 0; s0 < w; s0 += WAVE) {
      const int s = s0 + lane;
      const int c = (s < w) ? s_tot[s] : 0;
      int incl = c;
#pragma unroll
      for (int off = 1; off < WAVE; off <<= 1) {
        const int y = __shfl_up(incl, off);
        if (lane >= off) incl += y;
      }
      if (s < w) { s_tot[s] = carry + incl - c; start[s] = carry + incl - c; }
      carry += __shfl(incl, WAVE - 1);
    }
    if (lane == 0) start[w] = carry;
  }
  __syncthreads();
  for (int s = tid; s < w; s += blockDim.x) {
    const int st = s_tot[s];
    for (int g = 0; g < segs; ++g) s_tab[g * w + s] += st;
  }
  __syncthreads();
  volatile int* cur = mine;
  constexpr int NA = 4;                       // 64-token chunks whose loads are requested together
  for (int e00 = lo; e00 < hi; e00 += NA * WAVE) {
    int s4[NA], slot4[NA], pos4[NA];
#pragma unroll
    for (int u = 0; u < NA; ++u) {
      const int e = e00 + u * WAVE + lane;
      const bool in = e < hi;
      s4[u] = in ? bk[e] : -1;
      slot4[u] = in ? src_slot[(size_t)unit * cap + e] : 0;
      pos4[u] = in ? tok_pos[(size_t)unit * cap + e] : 0;
    }
#pragma unroll
    for (int u = 0; u < NA; ++u) {
      if (e00 + u * WAVE >= hi) break;        // uniform over the wave
      const int s = s4[u];
      // what the accumulation needs of this token, so that it does not have to chase
      // the ordinal: its source row and, in the top bit, whether g_row(J) = -1
      int rec = 0;
      if (s >= 0) {
        rec = slot4[u];
        if (sign_neg(d, row, pos4[u])) rec |= (int)0x80000000u;
      }
      // lanes with the same slot: one ballot per bit of the slot number (13 bits cover
      // the largest w of this path; -1 = no token gets a bit pattern of its own)
      unsigned long long same = ~0ull;
      const unsigned su = (unsigned)s & 0x3fffu;
#pragma unroll
      for (int bit = 0; bit < 14; ++bit) {
        const bool one = (su >> bit) & 1u;
        const unsigned long long bal = __ballot(one);
        same &= one ? bal : ~bal;
      }
      const int lower = __popcll(same & ((1ull << lane) - 1ull));
      const bool higher = (lane < WAVE - 1) && ((same >> (lane + 1)) != 0ull);
      if (s >= 0) {
        const int dst = cur[s] + lower;
        order[dst] = rec;
        if (!higher) cur[s] = dst + 1;     // read above, written here by one lane per slot: same wave, program order
      }
      __builtin_amdgcn_wave_barrier();
    }
  }
}

// two neighbouring channels with one load
__device__ __forceinline__ void load_pair(const float* p, float& a, float& b) {
  const float2 v = *reinterpret_cast<const float2*>(p);
  a = v.x; b = v.y;
}
__device__ __forceinline__ void load_pair(const bf16_t* p, float& a, float& b) {
  const uint32_t v = *reinterpret_cast<const uint32_t*>(p);
  a = __uint_as_float(v << 16); b = __uint_as_float(v & 0xffff0000u);
}

// One wave per (unit, row, slot): sequential float32 accumulation of the slot's
// segment, lanes across channels (2 per lane).
template <typename T>
__global__ __launch_bounds__(256) void encode_accum_kernel(
    DevDesc d, const T* __restrict__ k_src, const T* __restrict__ v_src, int src_rows, int cap,
    const int32_t* __restrict__ ws_order, const int32_t* __restrict__ ws_start, T* __restrict__ sk,
    T* __restrict__ sv) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // Workgroup ids are dealt round-robin to the 8 XCDs: all workgroups of a unit get ids that are equal
  // modulo 8, and within a unit the sketch rows alternate fastest, so that the r owners of a token's
  // slots, which walk the unit's list in the same ascending order at about the same time, share one L2.
  const int per_unit = d.r * ((d.w + 3) >> 2);
  const int xcd = blockIdx.x & 7, jj = blockIdx.x >> 3;
  const int unit = (jj / per_unit) * 8 + xcd;
  if (unit >= d.B * d.Hkv) return;
  const int within = jj % per_unit;
  const int row = within % d.r;
  const int s = (within / d.r) * 4 + wave;
  if (s >= d.w) return;
  const size_t ur = (size_t)unit * d.r + row;
  const int lo = ws_start[ur * (d.w + 1) + s], hi = ws_start[ur * (d.w + 1) + s + 1];
  if (hi <= lo) return;
  const int32_t* order = ws_order + ur * cap;
  const size_t idx = ((ur * d.w) + s) * D + 2 * lane;
  float ak0 = Store<T>::load1(sk + idx), ak1 = Store<T>::load1(sk + idx + 1);
  float av0 = Store<T>::load1(sv + idx), av1 = Store<T>::load1(sv + idx + 1);
  const bool fk = (d.sign_mask & 1) != 0, fv = (d.sign_mask & 2) != 0;
  for (int p0 = lo; p0 < hi; p0 += WAVE) {
    // lanes fetch up to 64 list entries, then the wave walks them in order
    int my_slot = 0;
    bool my_neg = false;
    if (p0 + lane < hi) {
      const int rec = order[p0 + lane];
      my_slot = rec & 0x7fffffff;
      my_neg = rec < 0;
    }
    const unsigned long long negs = __ballot(my_neg);
    const int n = min(WAVE, hi - p0);
    // eight tokens' rows are requested together, then added in list order
    constexpr int NB = 8;
    for (int j0 = 0; j0 < n; j0 += NB) {
      float k0[NB], k1[NB], v0[NB], v1[NB];
#pragma unroll
      for (int u = 0; u < NB; ++u) {
        const int slot = __shfl(my_slot, min(j0 + u, n - 1));
        const size_t src = ((size_t)unit * src_rows + slot) * D + 2 * lane;
        load_pair(k_src + src, k0[u], k1[u]);
        load_pair(v_src + src, v0[u], v1[u]);
      }
#pragma unroll
      for (int u = 0; u < NB; ++u) {
        if (j0 + u < n) {
          const bool neg = (negs >> (j0 + u)) & 1ull;
          ak0 += (fk && neg) ? -k0[u] : k0[u];
          ak1 += (fk && neg) ? -k1[u] : k1[u];
          av0 += (fv && neg) ? -v0[u] : v0[u];
          av1 += (fv && neg) ? -v1[u] : v1[u];
        }
      }
    }
  }
  Store<T>::store1(sk + idx, ak0);
  Store<T>::store1(sk + idx + 1, ak1);
  Store<T>::store1(sv + idx, av0);
  Store<T>::store1(sv + idx + 1, av1);
}

template <typename T>
static hipError_t launch_t(const DevDesc& d, const void* k_src, const void* v_src, int src_rows,
                           const int32_t* src_slot, const int32_t* tok_pos, const int32_t* count, int cap,
                           void* sk, void* sv, int32_t* out_bucket, uint8_t* out_sign, void* ws,
                           const EncodePlan& plan, hipStream_t st) {
  const int units = d.B * d.Hkv;
  if (!plan.bulk) {
    hipLaunchKernelGGL(encode_small_kernel<T>, dim3(units), dim3(D * (d.r < 4 ? d.r : 4)), 0, st, d, (const T*)k_src,
                       (const T*)v_src, src_rows, src_slot, tok_pos, count, cap, (T*)sk, (T*)sv, out_bucket,
                       out_sign);
    return hipGetLastError();
  }
  if (d.w > ENC_BULK_MAX_W) return hipErrorInvalidValue;
  char* base = (char*)ws;
  int32_t* ws_bucket = (int32_t*)(base + plan.off_bucket);
  int32_t* ws_order = (int32_t*)(base + plan.off_order);
  int32_t* ws_start = (int32_t*)(base + plan.off_start);
  hipLaunchKernelGGL(encode_hash_kernel, dim3((cap + 255) / 256, units), dim3(256), 0, st, d, src_rows,
                     src_slot, tok_pos, count, cap, ws_bucket, out_bucket, out_sign);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  {
    const int segs = sort_segments(d.w);
    hipLaunchKernelGGL(encode_sort_kernel, dim3(units * d.r), dim3(segs * WAVE),
                       (size_t)(segs + 1) * d.w * sizeof(int), st, d, count, cap, ws_bucket, src_slot, tok_pos,
                       ws_order, ws_start);
  }
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(encode_accum_kernel<T>, dim3((unsigned)(((units + 7) / 8) * 8 * d.r * ((d.w + 3) / 4))), dim3(256), 0, st, d,
                     (const T*)k_src, (const T*)v_src, src_rows, cap, ws_order, ws_start, (T*)sk, (T*)sv);
  return hipGetLastError();
}

hipError_t launch_encode(const DevDesc& d, int dtype, const void* k_src, const void* v_src, int src_rows,
                         const int32_t* src_slot, const int32_t* tok_pos, const int32_t* count, int cap,
                         void* sk, void* sv, int32_t* out_bucket, uint8_t* out_sign, void* ws,
                         const EncodePlan& plan, hipStream_t st) {
  if (cap <= 0) return hipSuccess;
  if (dtype == KVR_F32)
    return launch_t<float>(d, k_src, v_src, src_rows, src_slot, tok_pos, count, cap, sk, sv, out_bucket,
                           out_sign, ws, plan, st);
  return launch_t<bf16_t>(d, k_src, v_src, src_rows, src_slot, tok_pos, count, cap, sk, sv, out_bucket,
                          out_sign, ws, plan, st);
}

}  // namespace kvr
