// kvr_attend_decode: cache rebuild (Algorithm 4) fused with decode attention and
// the accumulation of per-token attention probabilities (Overview, Calculation
// Phase).  Retained tokens are streamed from their slots, Vague tokens are
// rebuilt on the fly from the sketch (Algorithm 2) and never written out.
//
// A unit's tokens are numbered t = 0 .. ret_cap-1 (retained slots) followed by
// ret_cap .. ret_cap+n_vague-1 (Vague index list) and cut into slices; every
// slice leaves a partial (max, sum, weighted V) per query head, and the merge
// kernel combines the partials, writes `out`, and turns the spilled logits into
// probabilities that are added to the cumulative scores.
//
// This file: the plan, the generic slice kernel (any storage type, any r, any
// sign setting; Vague rows gathered straight from global memory), the merge
// kernel and the dispatch.  The LDS-staged kernel for the Vague list is in
// kvr_attend_staged.hip.
#include "kvr_launch.h"

namespace kvr {

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

constexpr int STAGED_KMAX = 6;                    // wave-rounds (64 tokens) per wave, staged kernel
constexpr int STAGED_LDS_LIMIT = 160 * 1024;      // LDS per workgroup on gfx950

// Tokens per slice: about 1280 slices per launch (measured on the 32k workloads: fewer, larger slices leave
// the merge kernel fewer partials to fold and cost the retained kernel nothing), in multiples of
// 64 tokens, at least 128 when a unit has a long list (a workgroup of four waves with a single 16-token tile
// per wave is mostly start-up), at most 1024.
static int slice_tokens_for(long long tokens, long long units) {
  long long st = (tokens * units + 1279) / 1280;
  st = (st + 63) / 64 * 64;
  const long long mn = tokens >= 1024 ? 128 : 64;
  if (st < mn) st = mn;
  if (st > 1024) st = 1024;
  return (int)st;
}

int attend_slice_tokens(long long tokens, long long units) { return slice_tokens_for(tokens, units); }

AttendPlan attend_plan(const DevDesc& d, int dtype, long long ret_cap, long long vague_cap) {
  AttendPlan p;
  const long long units = (long long)d.B * d.Hkv;
  const long long tot_cap = ret_cap + vague_cap;
  p.staged = false;
  p.n_vslices = 0;
  p.ch = 0;
  p.lds_bytes = 0;
  // staged kernel: bf16, the paper's sign setting, G <= 4, r = 3 or 4, bucket fits 15 bits
  if (dtype == KVR_BF16 && d.sign_mask == 2 && d.G <= 4 && (d.r == 3 || d.r == 4) && d.w <= 32768 &&
      vague_cap >= 64) {
    const int fixed = STAGED_KMAX * 512 * 8 + 8 * d.G * 64 * 4 + 1024 + d.G * 256;
    int ch = 0;
    for (int c = 64; c >= 8; c >>= 1) {
      if ((long long)d.r * d.w * c * 2 + 1024 + fixed <= STAGED_LDS_LIMIT) { ch = c; break; }
    }
    if (ch) {
      const long long wr = (vague_cap + 63) / 64;          // wave-rounds to cover the list
      // Cost model: a workgroup that gives every wave rho rounds of 64 tokens takes
      // about (fixed + rho) round times (fixed part: staging the sketch chunks,
      // hashes, softmax, reductions: 2.8 rounds' worth for four 64-channel chunks,
      // 7.5 for the sixteen 16-channel chunks of the four-row kernel, whose waves may
      // also take more rounds), and the launch runs ceil(workgroups / 256)
      // such workgroups one after another on each CU.
      const bool r4 = staged_r4_applies(d);
      const int kmax = r4 ? STAGED_R4_KMAX : STAGED_KMAX;
      const double fixed_rounds = r4 ? 7.5 : 2.8;
      double best = 1e30;
      int best_rho = 1, best_n = 1;
      for (int rho = 1; rho <= kmax; ++rho) {
        const long long n = (wr + 8 * rho - 1) / (8 * rho);
        const long long rho_eff = (wr + 8 * n - 1) / (8 * n);      // rounds the busiest wave really gets
        const long long waves_of_wgs = (units * n + 255) / 256;
        const double cost = (double)waves_of_wgs * (fixed_rounds + (double)rho_eff);
        if (cost < best - 1e-9) { best = cost; best_rho = rho; best_n = (int)n; }
      }
      (void)best_rho;
      p.staged = true;
      p.ch = ch;
      p.n_vslices = best_n;
      // the chunk buffer doubles as reduction scratch [32 rows][G][ch] floats
      // and is padded to whole kilobytes (a wave stages 1 KB at a time)
      size_t buf = align_up((size_t)d.r * d.w * ch * 2, 1024);
      const size_t red = (size_t)32 * d.G * ch * 4;
      if (buf < red) buf = red;
      p.lds_bytes = (int)buf + fixed;
    }
  }
  p.mfma_retained = (dtype == KVR_BF16);
  // 8 query heads per kv head: too many logits per token for the register-resident staged kernels; the
  // streaming kernel of kvr_attend_multi takes the list with the 8 heads as its columns (one query)
  p.streamed = !p.staged && dtype == KVR_BF16 && d.G == 8 && multi_staged_applies(d, vague_cap);
  p.vslice_tokens = 0;
  if (p.mfma_retained || p.staged) {
    // retained slots and the Vague list are cut separately
    p.rslice_tokens = slice_tokens_for(ret_cap, units);
    p.n_rslices = (int)((ret_cap + p.rslice_tokens - 1) / p.rslice_tokens);
    if (p.streamed) {
      p.vslice_tokens = multi_staged_part_tokens(vague_cap, units);
      p.n_vslices = (int)((vague_cap + p.vslice_tokens - 1) / p.vslice_tokens);
    } else if (!p.staged && vague_cap > 0) {
      p.vslice_tokens = slice_tokens_for(vague_cap, units);
      p.n_vslices = (int)((vague_cap + p.vslice_tokens - 1) / p.vslice_tokens);
    }
    p.n_slices = p.n_rslices + p.n_vslices;
  } else {
    // one generic launch over all tokens
    p.rslice_tokens = slice_tokens_for(tot_cap, units);
    p.n_rslices = (int)((tot_cap + p.rslice_tokens - 1) / p.rslice_tokens);
    if (p.n_rslices < 1) p.n_rslices = 1;
    p.n_slices = p.n_rslices;
  }
  size_t off = 0;
  p.off_part_o = off;
  off = align_up(off + (size_t)units * p.n_slices * d.G * D * sizeof(float), 256);
  p.off_part_ml = off;
  off = align_up(off + (size_t)units * p.n_slices * d.G * 2 * sizeof(float), 256);
  // the streaming kernel reads its arrays a few tiles past the end without clamping
  const size_t pad_tok = p.streamed ? (size_t)multi_staged_pad_tokens() : 0;
  p.off_logits = off;
  off = align_up(off + ((size_t)units * (size_t)tot_cap + pad_tok) * d.G * sizeof(float), 256);
  p.off_rec = p.off_partial = off;
  if (p.streamed) {
    off = align_up(off + ((size_t)units * (size_t)vague_cap + pad_tok) * 8, 256);
    p.off_partial = off;
    off = align_up(off + ((size_t)units * (size_t)vague_cap + pad_tok) * d.G * sizeof(float), 256);
  }
  p.total_bytes = off;
  return p;
}

// ---------------------------------------------------------------------------
// generic slice kernel
// ---------------------------------------------------------------------------
template <typename T, int G, int R>
__global__ __launch_bounds__(256) void attend_main_kernel(DevDesc d, AttendArgs a) {
  constexpr int VEC = Store<T>::VEC;
  constexpr int LPT = D / VEC;       // lanes that share one token
  constexpr int TPW = WAVE / LPT;    // tokens per wave per iteration
  constexpr int NW = 4;
  const int unit = blockIdx.y, slice = blockIdx.x;
  const int b = unit / d.Hkv, hk = unit % d.Hkv;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane % LPT, tl = lane / LPT;
  const int c0 = sub * VEC;

  float qf[G][VEC];
  {
    const T* q = (const T*)a.q + ((size_t)b * d.Hq + (size_t)hk * G) * D + c0;
#pragma unroll
    for (int g = 0; g < G; ++g) Store<T>::load16(q + (size_t)g * D, qf[g]);
  }
  const int nv = a.n_vague ? clampi(a.n_vague[unit], 0, a.vague_cap) : 0;
  const int tot_cap = a.ret_cap + a.vague_cap;
  const int total = min(a.ret_cap + nv, a.tok_limit);
  const int t_begin = a.tok_start + slice * a.slice_tokens;
  const int t_end = min(t_begin + a.slice_tokens, total);

  const T* kret = (const T*)a.k_ret + (size_t)unit * a.ret_cap * D;
  const T* vret = (const T*)a.v_ret + (size_t)unit * a.ret_cap * D;
  const size_t sk_unit = (size_t)unit * d.r * d.w * D;
  const T* sk = (const T*)a.sk + sk_unit;
  const T* sv = (const T*)a.sv + sk_unit;
  const bool flip_k = (d.sign_mask & 1) != 0, flip_v = (d.sign_mask & 2) != 0;

  float m[G], l[G], acc[G][VEC];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m[g] = -__builtin_inff();
    l[g] = 0.f;
#pragma unroll
    for (int c = 0; c < VEC; ++c) acc[g][c] = 0.f;
  }

  for (int t0 = t_begin + wave * TPW; t0 < t_end; t0 += NW * TPW) {
    const int t = t0 + tl;
    bool valid = t < t_end;
    float kf[VEC], vf[VEC];
#pragma unroll
    for (int c = 0; c < VEC; ++c) { kf[c] = 0.f; vf[c] = 0.f; }
    if (valid) {
      if (t < a.ret_cap) {
        const int pos = a.ret_pos ? a.ret_pos[(size_t)unit * a.ret_cap + t] : t;
        if (pos < 0) {
          valid = false;
        } else {
          Store<T>::load16(kret + (size_t)t * D + c0, kf);
          Store<T>::load16(vret + (size_t)t * D + c0, vf);
        }
      } else {
        const int J = a.vague_pos[(size_t)unit * a.vague_cap + (t - a.ret_cap)];
        query_chunk<T, R>(d, sk, J, c0, flip_k, kf);
        query_chunk<T, R>(d, sv, J, c0, flip_v, vf);
      }
    }
    float s[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float x = 0.f;
#pragma unroll
      for (int c = 0; c < VEC; ++c) x = fmaf(qf[g][c], kf[c], x);
#pragma unroll
      for (int off = LPT / 2; off >= 1; off >>= 1) x += __shfl_xor(x, off);
      s[g] = valid ? x * d.scale : -__builtin_inff();
    }
    if (a.logits != nullptr && sub == 0 && t < t_end) {
      float* lg = a.logits + ((size_t)unit * tot_cap + t) * G;
#pragma unroll
      for (int g = 0; g < G; ++g) lg[g] = s[g];
    }
    if (valid) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        if (s[g] > m[g]) {
          const float corr = expf(m[g] - s[g]);     // exp(-inf) = 0 on the first token
          m[g] = s[g];
          l[g] = l[g] * corr + 1.f;
#pragma unroll
          for (int c = 0; c < VEC; ++c) acc[g][c] = fmaf(acc[g][c], corr, vf[c]);
        } else {
          const float pr = expf(s[g] - m[g]);
          l[g] += pr;
#pragma unroll
          for (int c = 0; c < VEC; ++c) acc[g][c] = fmaf(pr, vf[c], acc[g][c]);
        }
      }
    }
  }

  // merge the token lane groups of a wave (they hold the same channels)
#pragma unroll
  for (int off = LPT; off < WAVE; off <<= 1) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float m2 = __shfl_xor(m[g], off);
      const float l2 = __shfl_xor(l[g], off);
      const float mn = fmaxf(m[g], m2);
      const float e1 = (m[g] == -__builtin_inff()) ? 0.f : expf(m[g] - mn);
      const float e2 = (m2 == -__builtin_inff()) ? 0.f : expf(m2 - mn);
      l[g] = l[g] * e1 + l2 * e2;
#pragma unroll
      for (int c = 0; c < VEC; ++c) {
        const float a2 = __shfl_xor(acc[g][c], off);
        acc[g][c] = acc[g][c] * e1 + a2 * e2;
      }
      m[g] = mn;
    }
  }

  __shared__ float s_acc[NW][G][D];
  __shared__ float s_m[NW][G], s_l[NW][G];
  if (tl == 0) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
      for (int c = 0; c < VEC; ++c) s_acc[wave][g][c0 + c] = acc[g][c];
      if (sub == 0) { s_m[wave][g] = m[g]; s_l[wave][g] = l[g]; }
    }
  }
  __syncthreads();
  float* po = a.part_o + ((size_t)unit * a.n_slices + a.slice0 + slice) * G * D;
  float* pml = a.part_ml + ((size_t)unit * a.n_slices + a.slice0 + slice) * G * 2;
  for (int idx = threadIdx.x; idx < G * D; idx += 256) {
    const int g = idx / D, c = idx % D;
    float M = s_m[0][g];
#pragma unroll
    for (int w_ = 1; w_ < NW; ++w_) M = fmaxf(M, s_m[w_][g]);
    float L = 0.f, O = 0.f;
#pragma unroll
    for (int w_ = 0; w_ < NW; ++w_) {
      const float e = (s_m[w_][g] == -__builtin_inff()) ? 0.f : expf(s_m[w_][g] - M);
      L += s_l[w_][g] * e;
      O += s_acc[w_][g][c] * e;
    }
    po[idx] = O;
    if (c == 0) { pml[g * 2] = M; pml[g * 2 + 1] = L; }
  }
}

// ---------------------------------------------------------------------------
// merge kernel
// ---------------------------------------------------------------------------

template <int G>
__global__ __launch_bounds__(256) void attend_combine_kernel(DevDesc d, AttendArgs a) {
  const int unit = blockIdx.y;
  const int b = unit / d.Hkv, hk = unit % d.Hkv;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  __shared__ float sM[G], sL[G];
  const float* pml = a.part_ml + (size_t)unit * a.n_slices * G * 2;

  // ---- score pass, first half: everything that does not depend on the global
  //      statistics is requested before they are formed (token positions, the
  //      spilled logits and the old scores), so that the two chains of memory
  //      round trips (slice statistics -> reduction, position -> old score) run
  //      side by side instead of one after the other.  Four tokens per thread. ----
  constexpr int U = 4;
  const bool do_scores = a.scores != nullptr;
  const int tot_cap = a.ret_cap + a.vague_cap;
  int total = 0;
  int pos[U];
  float x[U][G], old[U];
  float* sc = do_scores ? a.scores + (size_t)unit * a.n_cap : nullptr;
  const int t0 = blockIdx.x * 256 * U + tid;
  if (do_scores) {
    const int nv = a.n_vague ? clampi(a.n_vague[unit], 0, a.vague_cap) : 0;
    total = a.ret_cap + nv;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int t = t0 + u * 256;
      pos[u] = -1;
      if (t < total) {
        if (t < a.ret_cap) pos[u] = a.ret_pos ? a.ret_pos[(size_t)unit * a.ret_cap + t] : t;
        else pos[u] = a.vague_pos[(size_t)unit * a.vague_cap + (t - a.ret_cap)];
        if (pos[u] >= a.n_cap) pos[u] = -1;
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int t = t0 + u * 256;
#pragma unroll
      for (int g = 0; g < G; ++g) x[u][g] = -__builtin_inff();
      if (t < total) {
        const float* lg = a.logits + ((size_t)unit * tot_cap + t) * G;
        if constexpr (G % 4 == 0) {
#pragma unroll
          for (int g4 = 0; g4 < G; g4 += 4) {
            const float4 v = *reinterpret_cast<const float4*>(lg + g4);
            x[u][g4] = v.x; x[u][g4 + 1] = v.y; x[u][g4 + 2] = v.z; x[u][g4 + 3] = v.w;
          }
        } else {
#pragma unroll
          for (int g = 0; g < G; ++g) x[u][g] = lg[g];
        }
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) old[u] = (pos[u] >= 0) ? sc[pos[u]] : 0.f;
  }

  // ---- global max and sum per head: wave w takes heads w, w + 4 ----------------
  for (int g = wave; g < G; g += 4) {
    float M = -__builtin_inff(), L = 0.f;
    for (int s = lane; s < a.n_slices; s += WAVE) {
      const float ms = pml[(s * G + g) * 2], ls = pml[(s * G + g) * 2 + 1];
      if (ls > 0.f) {
        const float mn = fmaxf(M, ms);
        L = L * expf(M - mn) + ls * expf(ms - mn);
        M = mn;
      }
    }
    // the wave's maximum first (no exponentials), then one rescaling per lane and a plain sum
    float Mw = M;
#pragma unroll
    for (int off = 1; off < WAVE; off <<= 1) Mw = fmaxf(Mw, __shfl_xor(Mw, off));
    float Lw = (L > 0.f) ? L * expf(M - Mw) : 0.f;
#pragma unroll
    for (int off = 1; off < WAVE; off <<= 1) Lw += __shfl_xor(Lw, off);
    if (lane == 0) { sM[g] = Mw; sL[g] = Lw; }
  }
  __syncthreads();

  // ---- score pass, second half ----------------------------------------------------
  if (do_scores) {
    float invL[G], M[G];
#pragma unroll
    for (int g = 0; g < G; ++g) { M[g] = sM[g]; invL[g] = sL[g] > 0.f ? 1.f / sL[g] : 0.f; }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float acc = 0.f;
#pragma unroll
      for (int g = 0; g < G; ++g)
        if (x[u][g] != -__builtin_inff()) acc += __expf(x[u][g] - M[g]) * invL[g];
      if (pos[u] >= 0) sc[pos[u]] = old[u] + acc;
    }
    // tokens beyond the launch width (the dispatch covers every token with one
    // round; this loop only runs if a caller launches a narrower grid)
    for (int base = (blockIdx.x + gridDim.x) * 256 * U; base < total; base += gridDim.x * 256 * U) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int t = base + tid + u * 256;
        if (t >= total) continue;
        int ps;
        if (t < a.ret_cap) ps = a.ret_pos ? a.ret_pos[(size_t)unit * a.ret_cap + t] : t;
        else ps = a.vague_pos[(size_t)unit * a.vague_cap + (t - a.ret_cap)];
        if (ps < 0 || ps >= a.n_cap) continue;
        const float* lg = a.logits + ((size_t)unit * tot_cap + t) * G;
        float acc = 0.f;
#pragma unroll
        for (int g = 0; g < G; ++g)
          if (lg[g] != -__builtin_inff()) acc += __expf(lg[g] - M[g]) * invL[g];
        sc[ps] += acc;
      }
    }
  }

  // ---- the unit's output: spread over the first nb workgroups of the unit (a power
  //      of two): workgroup bx takes G*D/nb output elements, `tpe` threads per
  //      element, each summing every tpe-th slice with eight loads in flight.  A
  //      unit cut into many slices (few units, long lists) gets 16 threads per
  //      element and up to 32 workgroups, so that a thread's walk over the slices
  //      is one batch of loads; otherwise 4 threads and up to 8 workgroups. ----------
  const int tpe = (a.n_slices > 32) ? 16 : 4;
  const int epw = 256 / tpe;                  // output elements per workgroup and round
  int nb = 1;
  while (nb * 2 <= 2 * tpe && nb * 2 <= (int)gridDim.x && G * D / (nb * 2) >= epw) nb *= 2;
  if ((int)blockIdx.x < nb) {
    __shared__ float sO[16][64];               // [slice share][output element of this round]
    const int per_wg = G * D / nb;             // a multiple of epw
    const float* po = a.part_o + (size_t)unit * a.n_slices * G * D;
    for (int o0 = 0; o0 < per_wg; o0 += epw) {
      const int el = tid % epw, sq = tid / epw;
      const int idx = blockIdx.x * per_wg + o0 + el;
      const int g = idx / D;
      const float M = sM[g];
      float o = 0.f;
      for (int s0 = sq; s0 < a.n_slices; s0 += tpe * 8) {
        float v[8], wgt[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int s_ = s0 + tpe * j;
          v[j] = 0.f;
          wgt[j] = 0.f;
          if (s_ < a.n_slices) {
            v[j] = po[(size_t)s_ * G * D + idx];
            const float ms = pml[(s_ * G + g) * 2], ls = pml[(s_ * G + g) * 2 + 1];
            wgt[j] = (ls > 0.f) ? expf(ms - M) : 0.f;
          }
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) o = fmaf(v[j], wgt[j], o);
      }
      __syncthreads();                         // previous round's readers are done with sO
      sO[sq][el] = o;
      __syncthreads();
      if (sq == 0) {
        float tot = 0.f;
        if (tpe == 4) {
          tot = (sO[0][el] + sO[1][el]) + (sO[2][el] + sO[3][el]);
        } else {
#pragma unroll
          for (int k = 0; k < 16; k += 4) tot += (sO[k][el] + sO[k + 1][el]) + (sO[k + 2][el] + sO[k + 3][el]);
        }
        const float L = sL[g];
        // column g of the partials = (query tq, head gh of the group); out is [B, n_q, Hq, D]
        const int tq = g / d.G, gh = g % d.G;
        a.out[((((size_t)b * a.n_q + tq) * d.Hq) + (size_t)hk * d.G + gh) * D + (idx % D)] = (L > 0.f) ? tot / L : 0.f;
      }
    }
  }
}

// ---------------------------------------------------------------------------
// compute units of the current device (the runtime answers from its own tables; nothing is cached here)
static int cu_count() {
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
    cus = 256;
  return cus;
}

template <typename T, int G>
static void launch_main_r(const DevDesc& d, const AttendArgs& a, dim3 grid, hipStream_t st) {
  switch (d.r) {
    case 3: hipLaunchKernelGGL((attend_main_kernel<T, G, 3>), grid, dim3(256), 0, st, d, a); break;
    case 4: hipLaunchKernelGGL((attend_main_kernel<T, G, 4>), grid, dim3(256), 0, st, d, a); break;
    default: hipLaunchKernelGGL((attend_main_kernel<T, G, 0>), grid, dim3(256), 0, st, d, a); break;
  }
}

hipError_t launch_attend_combine(const DevDesc& d, const AttendArgs& a, int n_cols, hipStream_t st) {
  const int units = d.B * d.Hkv;
  const long long tot_cap = (long long)a.ret_cap + a.vague_cap;
  int cx = (int)((tot_cap + 1023) / 1024);
  if (cx < 1) cx = 1;
  const dim3 grid(cx, units), block(256);
  switch (n_cols) {
    case 1: hipLaunchKernelGGL((attend_combine_kernel<1>), grid, block, 0, st, d, a); break;
    case 2: hipLaunchKernelGGL((attend_combine_kernel<2>), grid, block, 0, st, d, a); break;
    case 4: hipLaunchKernelGGL((attend_combine_kernel<4>), grid, block, 0, st, d, a); break;
    case 8: hipLaunchKernelGGL((attend_combine_kernel<8>), grid, block, 0, st, d, a); break;
    case 16: hipLaunchKernelGGL((attend_combine_kernel<16>), grid, block, 0, st, d, a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

template <int G>
static hipError_t launch_g(const DevDesc& d, int dtype, const AttendArgs& a0, const AttendPlan& plan,
                           hipStream_t st, const AttendSide& sd) {
  const int units = d.B * d.Hkv;
  AttendArgs a = a0;
  a.n_slices = plan.n_slices;
  a.n_rslices = plan.n_rslices;
  a.n_vslices = plan.n_vslices;
  if (sd.prof_start) (void)hipEventRecord(sd.prof_start, st);
  hipError_t e = hipSuccess;
  // 1. retained slots (or, for f32 storage without staging, everything at once)
  a.slice_tokens = plan.rslice_tokens;
  a.tok_start = 0;
  a.slice0 = 0;
  // The retained kernel is bound by HBM, the staged kernel by the vector ALUs and
  // LDS, and their registers and LDS fit on a CU together: when the caller lends a
  // second stream they run side by side, the retained kernel on that stream, forked
  // from and joined back into `st` with the caller's two events.
  // Only when the staged kernel fills the chip several times over: a launch of a few workgroups is
  // short, the fork and join then cost more than the overlap saves, and the retained kernel is better
  // off with a launch as wide as its item count than with one workgroup per CU.
  const int cus = cu_count();
  const bool big = (long long)units * plan.n_vslices >= 2ll * cus;
  // Not next to the four-row kernel either: its two waves per SIMD hold up to 2 x 238 of the 512
  // registers, so the retained kernel would only find room where a workgroup of it has just ended
  // (measured on the 131k workload: 571 us side by side, 511 us back to back).
  const bool side = sd.stream != nullptr && plan.mfma_retained && plan.staged && big && !staged_r4_applies(d);
  if (side) {
    e = hipEventRecord(sd.fork, st);
    if (e == hipSuccess) e = hipStreamWaitEvent(sd.stream, sd.fork, 0);
    if (e == hipSuccess) {
      // From here on the side stream may hold work that writes the caller's workspace: whatever
      // fails below, `st` is made to wait for it before this call returns.
      // what the staged kernel's two waves leave of a SIMD's 512 registers: 128 next to the 64-channel
      // kernel, 80 next to the widest general form
      const bool s64 = d.r == 3 && plan.ch == 64 && 3 * d.w <= 1024;
      const int reg_form = s64 ? 1 : ((d.G == 4 && plan.ch <= 16) ? 2 : 0);
      e = launch_attend_retained(d, a, plan.n_rslices, cus, reg_form, sd.stream);
      const hipError_t ej = hipEventRecord(sd.join, sd.stream);
      if (e == hipSuccess && ej == hipSuccess) e = launch_attend_vague_staged(d, a, plan, st);
      hipError_t ew = (ej == hipSuccess) ? hipStreamWaitEvent(st, sd.join, 0) : ej;
      if (ew != hipSuccess) {
        (void)hipStreamSynchronize(sd.stream);      // no event to order by: wait on the host (error path only)
        if (e == hipSuccess) e = ew;
      }
    }
  } else if (plan.mfma_retained) {
    e = launch_attend_retained(d, a, plan.n_rslices, 0, 0, st);
  } else {
    a.tok_limit = plan.staged ? a.ret_cap : a.ret_cap + a.vague_cap;
    dim3 grid(plan.n_rslices, units);
    if (dtype == KVR_F32) launch_main_r<float, G>(d, a, grid, st);
    else launch_main_r<bf16_t, G>(d, a, grid, st);
    e = hipGetLastError();
  }
  // 2. the Vague list
  if (side) {
    // already launched above
  } else if (e == hipSuccess && plan.staged) {
    e = launch_attend_vague_staged(d, a, plan, st);
  } else if (e == hipSuccess && plan.streamed && plan.n_vslices > 0) {
    // no causal mask in a decode call: every listed token is visible (n_ctx = null)
    e = launch_attend_multi_staged(d, a, nullptr, 1, plan.vslice_tokens, plan.n_vslices, plan.n_rslices,
                                   plan.n_slices, a.part_o, a.part_ml, a.logits_buf, a.scratch_rec,
                                   a.scratch_partial, st);
  } else if (e == hipSuccess && plan.mfma_retained && plan.n_vslices > 0) {
    a.slice_tokens = plan.vslice_tokens;
    a.tok_start = a.ret_cap;
    a.tok_limit = a.ret_cap + a.vague_cap;
    a.slice0 = plan.n_rslices;
    dim3 grid(plan.n_vslices, units);
    launch_main_r<bf16_t, G>(d, a, grid, st);
    e = hipGetLastError();
  }
  // 3. merge
  if (e == hipSuccess) e = launch_attend_combine(d, a, G, st);
  if (sd.prof_stop) (void)hipEventRecord(sd.prof_stop, st);
  return e;
}

hipError_t launch_attend(const DevDesc& d, int dtype, const AttendArgs& a, const AttendPlan& plan,
                         hipStream_t st, const AttendSide& sd) {
  switch (d.G) {
    case 1: return launch_g<1>(d, dtype, a, plan, st, sd);
    case 2: return launch_g<2>(d, dtype, a, plan, st, sd);
    case 4: return launch_g<4>(d, dtype, a, plan, st, sd);
    case 8: return launch_g<8>(d, dtype, a, plan, st, sd);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace kvr
