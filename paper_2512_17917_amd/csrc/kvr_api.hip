// C ABI of libkvr: argument validation, workspace planning, dispatch.
// Everything that can be checked on the host is checked before the first HIP
// call, so the error paths work on a machine without a GPU.
#include <string.h>

#include "kvr_launch.h"

namespace {

thread_local int32_t g_last_hip_error = 0;

constexpr uint64_t LCG_MUL = 6364136223846793005ull;
constexpr uint64_t LCG_INC = 1442695040888963407ull;

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Returns KVR_OK and fills `d`, or an error code.
int32_t check_desc(const kvr_desc* desc, kvr::DevDesc& d) {
  if (desc == nullptr) return KVR_ERR_INVALID_ARG;
  if (desc->batch < 1 || desc->n_q_heads < 1 || desc->n_kv_heads < 1) return KVR_ERR_INVALID_ARG;
  if (desc->r < 1 || desc->r > KVR_MAX_ROWS || desc->w < 1 || desc->w > 65536) return KVR_ERR_INVALID_ARG;
  if (desc->dtype != KVR_F32 && desc->dtype != KVR_BF16) return KVR_ERR_INVALID_ARG;
  if (desc->sign_mask < 0 || desc->sign_mask > 3) return KVR_ERR_INVALID_ARG;
  if (desc->median_mode != KVR_MEDIAN_MIDMEAN && desc->median_mode != KVR_MEDIAN_LOWER)
    return KVR_ERR_INVALID_ARG;
  if (!(desc->softmax_scale == desc->softmax_scale)) return KVR_ERR_INVALID_ARG;
  if (desc->head_dim != KVR_HEAD_DIM) return KVR_ERR_UNSUPPORTED;
  if (desc->n_q_heads % desc->n_kv_heads != 0) return KVR_ERR_UNSUPPORTED;
  const int G = desc->n_q_heads / desc->n_kv_heads;
  if (G != 1 && G != 2 && G != 4 && G != 8) return KVR_ERR_UNSUPPORTED;
  if ((long long)desc->batch * desc->n_kv_heads > 65535) return KVR_ERR_UNSUPPORTED;
  d.B = desc->batch;
  d.Hq = desc->n_q_heads;
  d.Hkv = desc->n_kv_heads;
  d.G = G;
  d.r = desc->r;
  d.w = desc->w;
  d.sign_mask = desc->sign_mask;
  d.median_mode = desc->median_mode;
  d.scale = desc->softmax_scale;
  memcpy(d.hp, desc->hash_params, sizeof(d.hp));
  return KVR_OK;
}

int32_t finish(hipError_t e) {
  if (e == hipSuccess) return KVR_OK;
  g_last_hip_error = (int32_t)e;
  return KVR_ERR_HIP;
}

constexpr long long MAX_TOKENS = 1ll << 30;

// ---------------------------------------------------------------------------
// Workspace of kvr_attend_decode_static: a fixed array in device memory that is
// part of the library's code object, so every GPU the library runs on holds its
// own copy, at its own address, from the moment the code object is loaded there
// until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress; the address it yields for the current device is what
// kernels and copies are given.
static __device__ __align__(256) unsigned char scratch[KVR_STATIC_SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[MAX_DEVICES];       // per device: address of its copy of `scratch`, null until looked up

// Address of the current device's copy (looked up on the first call on that device).
int32_t static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) { g_last_hip_error = (int32_t)e; return KVR_ERR_HIP; }
  if (dev < 0 || dev >= MAX_DEVICES) return KVR_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || p == nullptr) {
      g_last_hip_error = (int32_t)(e != hipSuccess ? e : hipErrorInvalidSymbol);
      return KVR_ERR_HIP;
    }
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return KVR_OK;
}

}  // namespace

extern "C" {

const char* kvr_version(void) { return "kvr 0.1 (gfx950)"; }

int32_t kvr_last_hip_error(void) { return g_last_hip_error; }

int32_t kvr_recent_size(int32_t r_size, int32_t r_budget, int32_t slack) {
  if (r_size < 0 || r_budget < 0 || slack < 0) return KVR_ERR_INVALID_ARG;
  return ((long long)r_size > (long long)r_budget + slack) ? r_budget : r_size;
}

int32_t kvr_hash_params_from_seed(uint64_t seed, int32_t r, uint64_t* out) {
  if (out == nullptr || r < 1 || r > KVR_MAX_ROWS) return KVR_ERR_INVALID_ARG;
  uint64_t x = seed;
  for (int i = 0; i < r; ++i) {
    for (int k = 0; k < 4; ++k) {
      x = x * LCG_MUL + LCG_INC;
      out[i * 4 + k] = x;
    }
    out[i * 4 + 0] |= 1ull;
    out[i * 4 + 2] |= 1ull;
  }
  return KVR_OK;
}

int32_t kvr_hash_host(const kvr_desc* desc, int32_t J, int32_t* bucket, int32_t* sign) {
  if (desc == nullptr || bucket == nullptr || sign == nullptr || J < 0) return KVR_ERR_INVALID_ARG;
  if (desc->r < 1 || desc->r > KVR_MAX_ROWS || desc->w < 1 || desc->w > 65536) return KVR_ERR_INVALID_ARG;
  for (int i = 0; i < desc->r; ++i) {
    const uint64_t u = desc->hash_params[i][0] * (uint64_t)(uint32_t)J + desc->hash_params[i][1];
    bucket[i] = (int32_t)(((u >> 32) * (uint64_t)(uint32_t)desc->w) >> 32);
    const uint64_t s = desc->hash_params[i][2] * (uint64_t)(uint32_t)J + desc->hash_params[i][3];
    sign[i] = (s >> 63) ? -1 : 1;
  }
  return KVR_OK;
}

int32_t kvr_workspace_size(const kvr_desc* desc, int32_t op, int64_t n_a, int64_t n_b, size_t* bytes) {
  kvr::DevDesc d;
  const int32_t rc = check_desc(desc, d);
  if (rc != KVR_OK) return rc;
  if (bytes == nullptr || n_a < 0 || n_a > MAX_TOKENS || n_b < 0 || n_b > MAX_TOKENS) return KVR_ERR_INVALID_ARG;
  switch (op) {
    case KVR_OP_SELECT:
    case KVR_OP_RECONSTRUCT:
      *bytes = 0;
      return KVR_OK;
    case KVR_OP_ENCODE:
      *bytes = kvr::encode_plan(d, n_a).total_bytes;
      return KVR_OK;
    case KVR_OP_ATTEND:
      *bytes = kvr::attend_plan(d, desc->dtype, n_a, n_b).total_bytes;
      return KVR_OK;
    default:
      return KVR_ERR_INVALID_ARG;
  }
}

int32_t kvr_append(const kvr_desc* desc, const void* k_new, const void* v_new, const int32_t* n_ctx,
                   void* k_ret, void* v_ret, int32_t* ret_pos, int32_t ret_cap, int32_t* out_slot,
                   void* stream) {
  kvr::DevDesc d;
  const int32_t rc = check_desc(desc, d);
  if (rc != KVR_OK) return rc;
  if (!k_new || !v_new || !n_ctx || !k_ret || !v_ret || !ret_pos) return KVR_ERR_INVALID_ARG;
  if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(k_ret) || !aligned16(v_ret))
    return KVR_ERR_INVALID_ARG;
  if (ret_cap < 1 || ret_cap > MAX_TOKENS) return KVR_ERR_INVALID_ARG;
  return finish(kvr::launch_append(d, desc->dtype, k_new, v_new, n_ctx, k_ret, v_ret, ret_pos, ret_cap,
                                   out_slot, (hipStream_t)stream));
}

int32_t kvr_select(const kvr_desc* desc, const float* scores, int64_t n_cap, int32_t* ret_pos,
                   int32_t ret_cap, const int32_t* n_ctx, int32_t n_recent, int32_t k_candidate,
                   int32_t* evict_slot, int32_t* evict_pos, int32_t* n_evict, int32_t evict_cap,
                   int32_t* vague_pos, int32_t* n_vague, int32_t vague_cap, void* ws, size_t ws_bytes,
                   void* stream) {
  (void)ws;
  (void)ws_bytes;
  kvr::DevDesc d;
  const int32_t rc = check_desc(desc, d);
  if (rc != KVR_OK) return rc;
  if (!scores || !ret_pos || !n_ctx || !evict_slot || !evict_pos || !n_evict) return KVR_ERR_INVALID_ARG;
  if ((vague_pos == nullptr) != (n_vague == nullptr)) return KVR_ERR_INVALID_ARG;
  if (n_cap < 1 || n_cap > MAX_TOKENS || ret_cap < 1 || ret_cap > MAX_TOKENS) return KVR_ERR_INVALID_ARG;
  if (n_recent < 0 || k_candidate < 0 || evict_cap < 1) return KVR_ERR_INVALID_ARG;
  if (vague_pos != nullptr && vague_cap < 1) return KVR_ERR_INVALID_ARG;
  return finish(kvr::launch_select(d, scores, n_cap, ret_pos, ret_cap, n_ctx, n_recent, k_candidate,
                                   evict_slot, evict_pos, n_evict, evict_cap, vague_pos, n_vague, vague_cap,
                                   (hipStream_t)stream));
}

int32_t kvr_encode(const kvr_desc* desc, const void* k_src, const void* v_src, int32_t src_rows,
                   const int32_t* src_slot, const int32_t* tok_pos, const int32_t* count, int32_t cap,
                   void* sketch_k, void* sketch_v, int32_t* out_bucket, uint8_t* out_sign, void* ws,
                   size_t ws_bytes, void* stream) {
  kvr::DevDesc d;
  const int32_t rc = check_desc(desc, d);
  if (rc != KVR_OK) return rc;
  if (!k_src || !v_src || !src_slot || !tok_pos || !count || !sketch_k || !sketch_v)
    return KVR_ERR_INVALID_ARG;
  if (!aligned16(k_src) || !aligned16(v_src) || !aligned16(sketch_k) || !aligned16(sketch_v))
    return KVR_ERR_INVALID_ARG;
  if (src_rows < 1 || src_rows > MAX_TOKENS || cap < 0 || cap > MAX_TOKENS) return KVR_ERR_INVALID_ARG;
  const kvr::EncodePlan plan = kvr::encode_plan(d, cap);
  if (plan.bulk && d.w > 8192) return KVR_ERR_UNSUPPORTED;
  if (plan.total_bytes > 0) {
    if (ws == nullptr || !aligned16(ws)) return KVR_ERR_INVALID_ARG;
    if (ws_bytes < plan.total_bytes) return KVR_ERR_WORKSPACE_TOO_SMALL;
  }
  return finish(kvr::launch_encode(d, desc->dtype, k_src, v_src, src_rows, src_slot, tok_pos, count, cap,
                                   sketch_k, sketch_v, out_bucket, out_sign, ws, plan, (hipStream_t)stream));
}

int32_t kvr_step_update(const kvr_desc* desc, const void* k_new, const void* v_new, const int32_t* n_ctx,
                        void* k_ret, void* v_ret, int32_t* ret_pos, int32_t ret_cap, const float* scores,
                        int64_t n_cap, int32_t n_recent, int32_t k_candidate, int32_t* evict_slot,
                        int32_t* evict_pos, int32_t* n_evict, int32_t evict_cap, int32_t* vague_pos,
                        int32_t* n_vague, int32_t vague_cap, void* sketch_k, void* sketch_v, void* stream) {
  kvr::DevDesc d;
  const int32_t rc = check_desc(desc, d);
  if (rc != KVR_OK) return rc;
  if (!k_new || !v_new || !n_ctx || !k_ret || !v_ret || !ret_pos || !scores || !evict_slot || !evict_pos ||
      !n_evict || !sketch_k || !sketch_v)
    return KVR_ERR_INVALID_ARG;
  if ((vague_pos == nullptr) != (n_vague == nullptr)) return KVR_ERR_INVALID_ARG;
  if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(k_ret) || !aligned16(v_ret) ||
      !aligned16(sketch_k) || !aligned16(sketch_v))
    return KVR_ERR_INVALID_ARG;
  if (n_cap < 1 || n_cap > MAX_TOKENS || ret_cap < 1 || n_recent < 0 || k_candidate < 0 || evict_cap < 1)
    return KVR_ERR_INVALID_ARG;
  if (vague_pos != nullptr && vague_cap < 1) return KVR_ERR_INVALID_ARG;
  if (ret_cap > 32768 || evict_cap > 64) return KVR_ERR_UNSUPPORTED;
  return finish(kvr::launch_step_update(d, desc->dtype, k_new, v_new, n_ctx, k_ret, v_ret, ret_pos, ret_cap,
                                        scores, n_cap, n_recent, k_candidate, evict_slot, evict_pos, n_evict,
                                        evict_cap, vague_pos, n_vague, vague_cap, sketch_k, sketch_v,
                                        (hipStream_t)stream));
}

int32_t kvr_swap_back(const kvr_desc* desc, const float* scores, int64_t n_cap, void* k_ret, void* v_ret,
                      int32_t* ret_pos, int32_t ret_cap, const int32_t* n_ctx, int32_t n_recent,
                      float replace_rate, int32_t max_swaps, void* sketch_k, void* sketch_v,
                      int32_t* vague_pos, const int32_t* n_vague, int32_t vague_cap, int32_t* n_swapped,
                      int32_t* swap_log, void* stream) {
  kvr::DevDesc d;
  const int32_t rc = check_desc(desc, d);
  if (rc != KVR_OK) return rc;
  if (!scores || !k_ret || !v_ret || !ret_pos || !n_ctx || !sketch_k || !sketch_v || !vague_pos || !n_vague)
    return KVR_ERR_INVALID_ARG;
  if (!aligned16(k_ret) || !aligned16(v_ret) || !aligned16(sketch_k) || !aligned16(sketch_v))
    return KVR_ERR_INVALID_ARG;
  if (n_cap < 1 || n_cap > MAX_TOKENS || ret_cap < 1 || ret_cap > MAX_TOKENS || vague_cap < 1 ||
      vague_cap > MAX_TOKENS || n_recent < 0)
    return KVR_ERR_INVALID_ARG;
  if (!(replace_rate > 0.f) || !(replace_rate < 3.0e38f)) return KVR_ERR_INVALID_ARG;   // also rejects NaN
  if (max_swaps < 0 || max_swaps > 65536) return KVR_ERR_INVALID_ARG;
  return finish(kvr::launch_swap_back(d, desc->dtype, scores, n_cap, k_ret, v_ret, ret_pos, ret_cap, n_ctx,
                                      n_recent, replace_rate, max_swaps, sketch_k, sketch_v, vague_pos,
                                      n_vague, vague_cap, n_swapped, swap_log, (hipStream_t)stream));
}

int32_t kvr_reconstruct(const kvr_desc* desc, const void* sketch_k, const void* sketch_v,
                        const int32_t* tok_pos, const int32_t* count, int32_t cap, void* k_out, void* v_out,
                        void* stream) {
  kvr::DevDesc d;
  const int32_t rc = check_desc(desc, d);
  if (rc != KVR_OK) return rc;
  if (!sketch_k || !sketch_v || !tok_pos || !count || !k_out || !v_out) return KVR_ERR_INVALID_ARG;
  if (!aligned16(sketch_k) || !aligned16(sketch_v) || !aligned16(k_out) || !aligned16(v_out))
    return KVR_ERR_INVALID_ARG;
  if (cap < 0 || cap > MAX_TOKENS) return KVR_ERR_INVALID_ARG;
  return finish(kvr::launch_reconstruct(d, desc->dtype, sketch_k, sketch_v, tok_pos, count, cap, k_out,
                                        v_out, (hipStream_t)stream));
}

static int32_t attend_decode_common(bool static_ws, const kvr_desc* desc, const void* q, const void* k_ret, const void* v_ret,
                          const int32_t* ret_pos, int32_t ret_cap, const void* sketch_k,
                          const void* sketch_v, const int32_t* vague_pos, const int32_t* n_vague,
                          int32_t vague_cap, float* out, float* scores, int64_t n_cap, void* ws,
                          size_t ws_bytes, const kvr_attend_opts* opts, void* stream) {
  kvr::DevDesc d;
  const int32_t rc = check_desc(desc, d);
  if (rc != KVR_OK) return rc;
  if (!q || !k_ret || !v_ret || !out) return KVR_ERR_INVALID_ARG;
  kvr::AttendSide sd = {nullptr, nullptr, nullptr, nullptr, nullptr};
  if (opts != nullptr) {
    const int n_side = (opts->side_stream != nullptr) + (opts->fork_event != nullptr) + (opts->join_event != nullptr);
    if (n_side != 0 && n_side != 3) return KVR_ERR_INVALID_ARG;
    if ((opts->prof_start == nullptr) != (opts->prof_stop == nullptr)) return KVR_ERR_INVALID_ARG;
    if (opts->side_stream != nullptr && opts->side_stream == stream) return KVR_ERR_INVALID_ARG;
    sd.stream = (hipStream_t)opts->side_stream;
    sd.fork = (hipEvent_t)opts->fork_event;
    sd.join = (hipEvent_t)opts->join_event;
    sd.prof_start = (hipEvent_t)opts->prof_start;
    sd.prof_stop = (hipEvent_t)opts->prof_stop;
  }
  if ((vague_pos == nullptr) != (n_vague == nullptr)) return KVR_ERR_INVALID_ARG;
  if (n_vague != nullptr && (!sketch_k || !sketch_v)) return KVR_ERR_INVALID_ARG;
  if (ret_cap < 1 || ret_cap > MAX_TOKENS) return KVR_ERR_INVALID_ARG;
  if (n_vague == nullptr) vague_cap = 0;
  if (vague_cap < 0 || vague_cap > MAX_TOKENS) return KVR_ERR_INVALID_ARG;
  if (scores != nullptr && (n_cap < 1 || n_cap > MAX_TOKENS)) return KVR_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k_ret) || !aligned16(v_ret) || !aligned16(out) ||
      !aligned16(sketch_k) || !aligned16(sketch_v))
    return KVR_ERR_INVALID_ARG;
  const kvr::AttendPlan plan = kvr::attend_plan(d, desc->dtype, ret_cap, vague_cap);
  if (static_ws) {
    // the workspace is this device's copy of the library's static array
    if (plan.total_bytes > (size_t)KVR_STATIC_SCRATCH_BYTES) return KVR_ERR_WORKSPACE_TOO_SMALL;
    const int32_t rs = static_scratch(&ws);
    if (rs != KVR_OK) return rs;
    ws_bytes = (size_t)KVR_STATIC_SCRATCH_BYTES;
  }
  if (ws == nullptr || !aligned16(ws)) return KVR_ERR_INVALID_ARG;
  if (ws_bytes < plan.total_bytes) return KVR_ERR_WORKSPACE_TOO_SMALL;
  kvr::AttendArgs a;
  a.q = q;
  a.k_ret = k_ret;
  a.v_ret = v_ret;
  a.ret_pos = ret_pos;
  a.ret_cap = ret_cap;
  a.sk = sketch_k;
  a.sv = sketch_v;
  a.vague_pos = vague_pos;
  a.n_vague = n_vague;
  a.vague_cap = vague_cap;
  a.out = out;
  a.scores = scores;
  a.n_cap = n_cap;
  char* base = (char*)ws;
  a.part_o = (float*)(base + plan.off_part_o);
  a.part_ml = (float*)(base + plan.off_part_ml);
  a.logits = scores ? (float*)(base + plan.off_logits) : nullptr;
  a.logits_buf = (float*)(base + plan.off_logits);
  a.scratch_rec = plan.streamed ? (void*)(base + plan.off_rec) : nullptr;
  a.scratch_partial = plan.streamed ? (void*)(base + plan.off_partial) : nullptr;
  a.n_q = 1;
  return finish(kvr::launch_attend(d, desc->dtype, a, plan, (hipStream_t)stream, sd));
}

int32_t kvr_attend_decode(const kvr_desc* desc, const void* q, const void* k_ret, const void* v_ret,
                          const int32_t* ret_pos, int32_t ret_cap, const void* sketch_k,
                          const void* sketch_v, const int32_t* vague_pos, const int32_t* n_vague,
                          int32_t vague_cap, float* out, float* scores, int64_t n_cap, void* ws,
                          size_t ws_bytes, const kvr_attend_opts* opts, void* stream) {
  return attend_decode_common(false, desc, q, k_ret, v_ret, ret_pos, ret_cap, sketch_k, sketch_v, vague_pos, n_vague,
                              vague_cap, out, scores, n_cap, ws, ws_bytes, opts, stream);
}

int32_t kvr_attend_decode_static(const kvr_desc* desc, const void* q, const void* k_ret, const void* v_ret,
                                 const int32_t* ret_pos, int32_t ret_cap, const void* sketch_k,
                                 const void* sketch_v, const int32_t* vague_pos, const int32_t* n_vague,
                                 int32_t vague_cap, float* out, float* scores, int64_t n_cap,
                                 const kvr_attend_opts* opts, void* stream) {
  return attend_decode_common(true, desc, q, k_ret, v_ret, ret_pos, ret_cap, sketch_k, sketch_v, vague_pos, n_vague,
                              vague_cap, out, scores, n_cap, nullptr, 0, opts, stream);
}

static int32_t check_multi(const kvr_desc* desc, kvr::DevDesc& d, int32_t n_q) {
  const int32_t rc = check_desc(desc, d);
  if (rc != KVR_OK) return rc;
  if (n_q < 1) return KVR_ERR_INVALID_ARG;
  if (desc->dtype != KVR_BF16) return KVR_ERR_UNSUPPORTED;
  const long long ncol = (long long)n_q * d.G;
  if (ncol != 1 && ncol != 2 && ncol != 4 && ncol != 8 && ncol != 16) return KVR_ERR_UNSUPPORTED;
  return KVR_OK;
}

int32_t kvr_attend_multi_workspace_size(const kvr_desc* desc, int32_t n_q, int64_t ret_cap, int64_t vague_cap,
                                        size_t* bytes) {
  kvr::DevDesc d;
  const int32_t rc = check_multi(desc, d, n_q);
  if (rc != KVR_OK) return rc;
  if (bytes == nullptr || ret_cap < 1 || ret_cap > MAX_TOKENS || vague_cap < 0 || vague_cap > MAX_TOKENS)
    return KVR_ERR_INVALID_ARG;
  *bytes = kvr::attend_multi_plan(d, n_q, ret_cap, vague_cap).total_bytes;
  return KVR_OK;
}

int32_t kvr_attend_multi(const kvr_desc* desc, const void* q, int32_t n_q, const int32_t* n_ctx,
                         const void* k_ret, const void* v_ret, const int32_t* ret_pos, int32_t ret_cap,
                         const void* sketch_k, const void* sketch_v, const int32_t* vague_pos,
                         const int32_t* n_vague, int32_t vague_cap, float* out, float* scores, int64_t n_cap,
                         void* ws, size_t ws_bytes, void* stream) {
  kvr::DevDesc d;
  const int32_t rc = check_multi(desc, d, n_q);
  if (rc != KVR_OK) return rc;
  if (!q || !n_ctx || !k_ret || !v_ret || !ret_pos || !out) return KVR_ERR_INVALID_ARG;
  if ((vague_pos == nullptr) != (n_vague == nullptr)) return KVR_ERR_INVALID_ARG;
  if (n_vague != nullptr && (!sketch_k || !sketch_v)) return KVR_ERR_INVALID_ARG;
  if (ret_cap < 1 || ret_cap > MAX_TOKENS) return KVR_ERR_INVALID_ARG;
  if (n_vague == nullptr) vague_cap = 0;
  if (vague_cap < 0 || vague_cap > MAX_TOKENS) return KVR_ERR_INVALID_ARG;
  if (scores != nullptr && (n_cap < 1 || n_cap > MAX_TOKENS)) return KVR_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k_ret) || !aligned16(v_ret) || !aligned16(out) || !aligned16(sketch_k) ||
      !aligned16(sketch_v))
    return KVR_ERR_INVALID_ARG;
  const kvr::MultiPlan plan = kvr::attend_multi_plan(d, n_q, ret_cap, vague_cap);
  if (ws == nullptr || !aligned16(ws)) return KVR_ERR_INVALID_ARG;
  if (ws_bytes < plan.total_bytes) return KVR_ERR_WORKSPACE_TOO_SMALL;
  kvr::AttendArgs a;
  memset(&a, 0, sizeof(a));
  a.q = q;
  a.k_ret = k_ret;
  a.v_ret = v_ret;
  a.ret_pos = ret_pos;
  a.ret_cap = ret_cap;
  a.sk = sketch_k;
  a.sv = sketch_v;
  a.vague_pos = vague_pos;
  a.n_vague = n_vague;
  a.vague_cap = vague_cap;
  a.out = out;
  a.scores = scores;
  a.n_cap = n_cap;
  a.n_q = n_q;
  return finish(kvr::launch_attend_multi(d, a, n_ctx, n_q, plan, ws, (hipStream_t)stream));
}

}  // extern "C"
