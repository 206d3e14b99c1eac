// Host-side launcher declarations: one per kernel family.  Each launcher
// receives already validated arguments and returns the hipError_t of its last
// launch.
#pragma once
#include <hip/hip_runtime.h>

#include <mutex>

#include "kvr_dev.h"

namespace kvr {

// How one kvr_attend_decode call is cut into workgroups.  Slices 0 .. n_rslices-1
// cover the retained slots, slices n_rslices .. n_slices-1 the Vague index list.
struct AttendPlan {
  bool staged;          // Vague tokens by the LDS-staged kernel (else by the generic kernel)
  bool mfma_retained;   // retained slots by the MFMA kernel (bf16) (else by the generic kernel)
  int n_slices;         // partial results per unit
  int n_rslices;        // of which: retained slices
  int rslice_tokens;    // tokens per retained slice
  int n_vslices;        // slices (generic) or workgroups (staged) per unit over the Vague list
  int vslice_tokens;    // generic kernel over the Vague list: tokens per slice
  int ch;               // staged: channels per LDS phase
  int lds_bytes;        // staged: dynamic LDS per workgroup
  bool streamed;        // Vague tokens by the streaming LDS-staged kernel of kvr_attend_multi with one query
                        // (8 query heads per kv head; vslice_tokens / n_vslices are its parts)
  size_t off_part_o, off_part_ml, off_logits, off_rec, off_partial, total_bytes;
};
AttendPlan attend_plan(const DevDesc& d, int dtype, long long ret_cap, long long vague_cap);

struct AttendArgs {
  const void* q;
  const void* k_ret;
  const void* v_ret;
  const int32_t* ret_pos;
  int ret_cap;
  const void* sk;
  const void* sv;
  const int32_t* vague_pos;
  const int32_t* n_vague;
  int vague_cap;
  float* out;
  float* scores;
  long long n_cap;
  // workspace carve-up
  float* part_o;     // [units, n_slices, G, D]
  float* part_ml;    // [units, n_slices, G, 2]
  float* logits;     // [units, ret_cap + vague_cap, G] or nullptr when scores == nullptr
  float* logits_buf; // the same area, always (the streaming kernel needs the logits itself)
  void* scratch_rec; // streaming kernel: token records / partial logits (null when the plan is not streamed)
  void* scratch_partial;
  int n_slices;      // partial results per unit (all kinds)
  int slice_tokens;  // generic / retained kernel: tokens per slice
  int tok_start;     // generic kernel: first token it handles
  int tok_limit;     // generic kernel: it handles tokens t < min(tok_limit, ret_cap + n_vague)
  int slice0;        // generic kernel: index of its first partial
  int n_rslices;     // staged kernel: index of its first partial
  int n_vslices;     // staged kernel: workgroups per unit
  int n_q;           // merge kernel: query tokens per sequence (1 for kvr_attend_decode); the partials'
                     // columns are then (query t, head g) = t * G + g and out is [B, n_q, Hq, D]
};

// Retained slots by the MFMA kernel (bf16): slices 0 .. n_rslices-1 of a.slice_tokens slots.
// max_wgs > 0 caps the launch width (the workgroups then walk the items with a grid stride).
// reg_form: 0 = the kernel takes the registers it likes; 1 = capped at 128 (it shares the SIMDs with the
// 64-channel staged kernel); 2 = capped at 80 (with the general staged kernel's widest form; G = 4 only).
hipError_t launch_attend_retained(const DevDesc& d, const AttendArgs& a, int n_rslices, int max_wgs,
                                  int reg_form, hipStream_t st);

struct EncodePlan {
  bool bulk;
  size_t off_bucket, off_order, off_start, total_bytes;
};
EncodePlan encode_plan(const DevDesc& d, long long cap);

hipError_t launch_reconstruct(const DevDesc& d, int dtype, const void* sk, const void* sv,
                              const int32_t* tok_pos, const int32_t* count, int cap,
                              void* k_out, void* v_out, hipStream_t st);

// What the caller of kvr_attend_decode lends to a call (all may be null): a second stream with a fork and a
// join event for running the retained-slot kernel next to the staged kernel, and two events that are
// recorded on `st` right before the call's first and right after its last kernel.
struct AttendSide {
  hipStream_t stream;
  hipEvent_t fork, join;
  hipEvent_t prof_start, prof_stop;
};
hipError_t launch_attend(const DevDesc& d, int dtype, const AttendArgs& a, const AttendPlan& plan,
                         hipStream_t st, const AttendSide& sd);

// tokens per slice when `tokens` tokens of each of `units` units are cut for about 1280 workgroups
int attend_slice_tokens(long long tokens, long long units);

// merge kernel alone: n_cols = partial columns per unit (G for one query, n_q * G for several)
hipError_t launch_attend_combine(const DevDesc& d, const AttendArgs& a, int n_cols, hipStream_t st);

// kvr_attend_multi: workspace carve-up and launch (bf16, n_q * G in {1, 2, 4, 8, 16})
struct MultiPlan {
  int rslice_tokens, n_rslices, vslice_tokens, n_vslices, n_slices;
  bool staged;           // Vague list through the LDS-staged kernel (vslice_tokens / n_vslices = its parts)
  size_t off_khat, off_vhat, off_part_o, off_part_ml, off_logits, total_bytes;
};
// LDS-staged kernel of kvr_attend_multi over the Vague list (bf16, r = 3, values signed only, 3 w <= 1024)
bool multi_staged_applies(const DevDesc& d, long long vague_cap);
int multi_staged_part_tokens(long long vague_cap, long long units);
int multi_staged_pad_tokens();   // tokens the staged kernel may read past the end of its scratch arrays
hipError_t launch_attend_multi_staged(const DevDesc& d, const AttendArgs& a, const int32_t* n_ctx, int n_q,
                                      int part_tokens, int n_parts, int slice0, int n_slices, float* part_o,
                                      float* part_ml, float* logits, void* scratch_rec, void* scratch_partial,
                                      hipStream_t st);
MultiPlan attend_multi_plan(const DevDesc& d, int n_q, long long ret_cap, long long vague_cap);
hipError_t launch_attend_multi(const DevDesc& d, const AttendArgs& a, const int32_t* n_ctx, int n_q,
                               const MultiPlan& plan, void* ws, hipStream_t st);

// Staged kernel over the Vague list (bf16, values signed only, G <= 4, r in {3,4}).
hipError_t launch_attend_vague_staged(const DevDesc& d, const AttendArgs& a, const AttendPlan& plan,
                                      hipStream_t st);
// Its specialisation for r = 4 (kvr_attend_staged_r4.hip; launch_attend_vague_staged forwards to it).  A wave
// of that kernel takes up to STAGED_R4_KMAX rounds of 64 tokens (every workgroup stages the unit's whole
// sketch, sixteen chunks of it, so few large workgroups are better than many small ones).
constexpr int STAGED_R4_KMAX = 13;
bool staged_r4_applies(const DevDesc& d);
hipError_t launch_attend_vague_staged_r4(const DevDesc& d, const AttendArgs& a, const AttendPlan& plan,
                                         hipStream_t st);
// Its specialisation for r = 3 and plan.ch = 64 (launch_attend_vague_staged forwards to it).
hipError_t launch_attend_vague_staged64(const DevDesc& d, const AttendArgs& a, const AttendPlan& plan,
                                        hipStream_t st);


hipError_t launch_select(const DevDesc& d, const float* scores, long long n_cap, int32_t* ret_pos,
                         int ret_cap, const int32_t* n_ctx, int n_recent, int k_candidate,
                         int32_t* evict_slot, int32_t* evict_pos, int32_t* n_evict, int evict_cap,
                         int32_t* vague_pos, int32_t* n_vague, int vague_cap, hipStream_t st);

hipError_t launch_append(const DevDesc& d, int dtype, const void* k_new, const void* v_new,
                         const int32_t* n_ctx, void* k_ret, void* v_ret, int32_t* ret_pos, int ret_cap,
                         int32_t* out_slot, hipStream_t st);

// append -> select -> encode of every unit in one launch (ret_cap <= 32768, evict_cap <= 64)
hipError_t launch_step_update(const DevDesc& d, int dtype, const void* k_new, const void* v_new,
                              const int32_t* n_ctx, void* k_ret, void* v_ret, int32_t* ret_pos, int ret_cap,
                              const float* scores, long long n_cap, int n_recent, int k_candidate,
                              int32_t* evict_slot, int32_t* evict_pos, int32_t* n_evict, int evict_cap,
                              int32_t* vague_pos, int32_t* n_vague, int vague_cap, void* sk, void* sv,
                              hipStream_t st);

// swap loop of Algorithm 3: at most max_swaps exchanges between the Candidate and the Vague part per unit
hipError_t launch_swap_back(const DevDesc& d, int dtype, const float* scores, long long n_cap, void* k_ret,
                            void* v_ret, int32_t* ret_pos, int ret_cap, const int32_t* n_ctx, int n_recent,
                            float replace_rate, int max_swaps, void* sk, void* sv, int32_t* vague_pos,
                            const int32_t* n_vague, int vague_cap, int32_t* n_swapped, int32_t* swap_log,
                            hipStream_t st);

hipError_t launch_encode(const DevDesc& d, int dtype, const void* k_src, const void* v_src, int src_rows,
                         const int32_t* src_slot, const int32_t* tok_pos, const int32_t* count, int cap,
                         void* sk, void* sv, int32_t* out_bucket, uint8_t* out_sign,
                         void* ws, const EncodePlan& plan, hipStream_t st);

}  // namespace kvr
