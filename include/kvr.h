/*
 * kvr.h -- C ABI of the KVReviver decode hot path for AMD MI355X (gfx950).
 *
 * What the library computes is defined by the paper "KVReviver: Reversible KV
 * Cache Compression with Sketch-Based Token Reconstruction" (arXiv 2512.17917),
 * section "Algorithm":
 *   - Vague Sketch, Algorithm 1 (V.Insert)   -> kvr_encode
 *   - Vague Sketch, Algorithm 2 (V.Query)    -> kvr_reconstruct
 *   - Recent and Candidate, Algorithm 3 (Compress: which tokens leave the
 *     Candidate part for the sketch)         -> kvr_select
 *   - Recent and Candidate, Algorithm 3, first line (R.Push of the new token)
 *                                            -> kvr_append
 *   - the three of a decode step in one launch -> kvr_step_update
 *   - Algorithm 3, second loop (a Vague token swaps places with the weakest
 *     Candidate: V.Max_Score, V.Query, V.Delete, V.Insert(C.Top_Pop()), C.Push)
 *                                            -> kvr_swap_back
 *   - Algorithm 4 (rebuild the KV cache) followed by self-attention and the
 *     accumulation of Softmax(QK^T) per token (Overview, Calculation Phase)
 *                                            -> kvr_attend_decode
 *   - the same for several query tokens per sequence over one rebuilt cache
 *                                            -> kvr_attend_multi
 *
 * Vocabulary.  A *unit* is one (sequence b, kv head h) of one attention layer;
 * unit index u = b * n_kv_heads + h.  One call works on all units of one layer.
 * A unit owns
 *   - retained slots: k_ret, v_ret [ret_cap, D] raw tokens (Recent + Candidate
 *     parts) and ret_pos [ret_cap], the position of the token in each slot
 *     (-1 = empty slot);
 *   - the sketch: sketch_k, sketch_v [r, w, D] (r rows of w slots; the paper
 *     writes "r buckets of b tensors");
 *   - the Vague index list vague_pos [vague_cap] with n_vague valid entries: the
 *     positions of the tokens that live only in the sketch;
 *   - cumulative attention scores, float32 [n_cap], indexed by position.
 * Every position below the sequence's n_ctx is in exactly one of the two sets.
 *
 * Conventions.
 *   - Every pointer marked "dev" is device memory owned by the caller; the
 *     library never allocates, frees or keeps a pointer after the call returns,
 *     and it holds no state of its own between calls: no streams, no events, no
 *     buffers, no environment variables (the only per-thread datum is the error
 *     code behind kvr_last_hip_error).  Pointers marked "host" are ordinary host
 *     memory.
 *   - All arrays are dense, row-major, innermost dimension contiguous, in the
 *     shapes given below, unit-major: X[B, Hkv, ...].  Device pointers must be
 *     16-byte aligned.
 *   - head_dim D must be 128.  K, V, q and the sketch share one storage type,
 *     desc->dtype (KVR_F32 or KVR_BF16).  All sums are taken in float32.
 *   - Calls enqueue work on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and return without synchronising.  Counts that live in
 *     device memory are clamped to the capacities given on the host.
 *   - Return value: KVR_OK or a negative error code.  Arguments are validated
 *     before anything is launched, so error paths need no GPU.  No call aborts
 *     or throws.
 *   - Scratch memory comes from the caller: `ws` must hold at least the number
 *     of bytes kvr_workspace_size reports for that call; its contents need not
 *     survive between calls.  Calls that share one workspace must be ordered on
 *     one stream.
 *   - Value range.  Inputs are expected to be finite.  With bf16 storage and
 *     r = 3 or 4 the median over the sketch rows may be taken on the packed bit
 *     patterns, which is exact for finite values below 2^121 in magnitude;
 *     sketch contents beyond that (or Inf / NaN) give unspecified medians in
 *     kvr_reconstruct, kvr_attend_decode and kvr_attend_multi.  Every other
 *     configuration has no such limit.
 */
#ifndef KVR_H
#define KVR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define KVR_MAX_ROWS 8
#define KVR_HEAD_DIM 128

enum {
  KVR_OK = 0,
  KVR_ERR_INVALID_ARG = -1,         /* null / misaligned pointer, size out of range */
  KVR_ERR_UNSUPPORTED = -2,         /* head_dim != 128, group size not in {1,2,4,8}, ... */
  KVR_ERR_WORKSPACE_TOO_SMALL = -3,
  KVR_ERR_HIP = -4                  /* a launch failed; see kvr_last_hip_error() */
};

enum { KVR_F32 = 0, KVR_BF16 = 1 };
enum { KVR_MEDIAN_MIDMEAN = 0, KVR_MEDIAN_LOWER = 1 };
enum { KVR_OP_SELECT = 0, KVR_OP_ENCODE = 1, KVR_OP_RECONSTRUCT = 2, KVR_OP_ATTEND = 3 };

/*
 * Problem descriptor (host memory, plain data).
 *   batch, n_q_heads, n_kv_heads: B, Hq, Hkv; Hq / Hkv (the group size G) must be
 *       1, 2, 4 or 8.
 *   r, w: sketch rows (1..8) and slots per row (1..65536).
 *   sign_mask: bit 0 = multiply keys by g_i(J), bit 1 = multiply values by
 *       g_i(J), on insert and on query.  The paper signs values only (Vague
 *       Sketch, Algorithms 1-2): sign_mask = 2.
 *   median_mode: only matters for even r (the paper fixes r = 3).  MIDMEAN = mean
 *       of the two middle order statistics, computed in float32 and rounded to
 *       the storage type; LOWER = the lower of the two.
 *   softmax_scale: factor on q.k before the softmax (1/sqrt(d_k), d_k = 128).
 *   hash_params[i] = {a, b, c, d} of row i.  For a token at position J (J >= 0):
 *       h_i(J) = (((a*J + b) mod 2^64) >> 32) * w >> 32     (slot in row i)
 *       g_i(J) = -1 if ((c*J + d) mod 2^64) >> 63 else +1   (sign)
 *     The paper asks only for "r distinct hash functions" and random +-1
 *     coefficients; this multiply-add-shift family is this library's choice.
 */
typedef struct kvr_desc {
  int32_t batch, n_q_heads, n_kv_heads, head_dim;
  int32_t r, w;
  int32_t dtype;
  int32_t sign_mask;
  int32_t median_mode;
  float softmax_scale;
  uint64_t hash_params[KVR_MAX_ROWS][4];
} kvr_desc;

/*
 * What a caller may lend to one kvr_attend_decode call (host memory, plain data;
 * every field may be NULL, and a NULL kvr_attend_opts* means all NULL).
 *   side_stream, fork_event, join_event: a second hipStream_t of default priority
 *       (not `stream` itself) and two hipEvent_t (timing may be disabled), created
 *       and owned by the caller; all three or none.  With them, and when the call is
 *       large enough for it to pay (bf16, the Vague list long enough to fill the
 *       chip twice over), the kernel that streams the retained tokens runs on
 *       side_stream next to the kernel that rebuilds the Vague tokens on `stream`:
 *       fork_event is recorded on `stream` and awaited by side_stream, join_event is
 *       recorded on side_stream and awaited by `stream` before the merge kernel, on
 *       every path including errors, so the call stays ordered on `stream` and the
 *       workspace is free when work enqueued after the call runs.  Without them the
 *       two kernels run back to back on `stream`; results are the same.  The three
 *       handles must not be used by another call that can run at the same time.
 *   prof_start, prof_stop: two hipEvent_t with timing enabled, both or none;
 *       recorded on `stream` right before the call's first and right after its last
 *       kernel (a measuring aid).
 */
typedef struct kvr_attend_opts {
  void* side_stream;
  void* fork_event;
  void* join_event;
  void* prof_start;
  void* prof_stop;
} kvr_attend_opts;

/* Library version string (static storage). */
const char* kvr_version(void);

/* Raw hipError_t of the most recent failed launch on the calling thread, 0 if none. */
int32_t kvr_last_hip_error(void);

/*
 * Size of the Recent queue after the first branch of Algorithm 3 ("Recent and
 * Candidate"): r_size is R.size right after the new token was pushed, r_budget
 * is R.budget.  Only when the queue has outgrown its budget by more than `slack`
 * tokens do the oldest r_size - r_budget of them leave it (for the Candidate
 * part), all at once, and the queue is back at r_budget; otherwise it keeps its
 * size.  The result is the n_recent to pass to kvr_select / kvr_step_update /
 * kvr_swap_back for this step (tokens outside the queue are Candidates, and
 * kvr_select moves whatever exceeds k_candidate on to the Vague part: slack + 1
 * tokens every slack + 1 steps).  slack = 0: one token in, one out per step.
 * Pure host code.  Returns the new size, or KVR_ERR_INVALID_ARG (negative input).
 */
int32_t kvr_recent_size(int32_t r_size, int32_t r_budget, int32_t slack);

/*
 * Fill out[r][4] (host) from a seed: a 64-bit LCG x <- x*6364136223846793005 +
 * 1442695040888963407 (mod 2^64), x0 = seed, is stepped once per word; rows in
 * order, words in the order a, b, c, d; a and c are then made odd.  Pure host code.
 */
int32_t kvr_hash_params_from_seed(uint64_t seed, int32_t r, uint64_t* out);

/*
 * Host evaluation of h_i(J) and g_i(J) for one position (same integer formulas
 * as the kernels): bucket[r] in [0, w), sign[r] in {+1, -1}.  Pure host code.
 */
int32_t kvr_hash_host(const kvr_desc* desc, int32_t J, int32_t* bucket, int32_t* sign);

/*
 * Bytes of workspace a call of kind `op` needs for the capacities it will be
 * given: SELECT (n_a = ret_cap, n_b ignored; 0 bytes), ENCODE (n_a = cap),
 * RECONSTRUCT (n_a = cap; 0 bytes), ATTEND (n_a = ret_cap, n_b = vague_cap; use
 * n_b = 0 for calls without a Vague list).  Pure host code.
 */
int32_t kvr_workspace_size(const kvr_desc* desc, int32_t op, int64_t n_a, int64_t n_b, size_t* bytes);

/*
 * Push one newly generated token per unit into the Recent part (Algorithm 3,
 * "R.Push(T)").  The token of unit u is written to the lowest-numbered empty
 * retained slot (ret_pos < 0) and gets position n_ctx[b] - 1 (n_ctx already
 * counts it).  A unit without an empty slot is left untouched.
 *   k_new, v_new  dev [B, Hkv, D] storage type, read
 *   n_ctx         dev int32 [B], read
 *   k_ret, v_ret  dev [B, Hkv, ret_cap, D], written at one row per unit
 *   ret_pos       dev int32 [B, Hkv, ret_cap], read; written at one entry per unit
 *   out_slot      dev int32 [B, Hkv] or NULL: the slot used, -1 if none was empty
 */
int32_t kvr_append(const kvr_desc* desc, const void* k_new, const void* v_new, const int32_t* n_ctx,
                   void* k_ret, void* v_ret, int32_t* ret_pos, int32_t ret_cap, int32_t* out_slot,
                   void* stream);

/*
 * Decide which retained tokens move to the Vague part (Algorithm 3: the Recent
 * part keeps the newest tokens, the Candidate part the highest cumulative
 * scores, everything else is popped towards the sketch).
 * Per unit: a slot is Recent if ret_pos >= n_ctx[b] - n_recent.  Among the other
 * occupied slots the k_candidate highest scores[ret_pos] stay (ties: the lower
 * position ranks higher; -0 == +0; NaN scores are an input error); the rest are
 * evicted: listed in ascending slot order in evict_slot / evict_pos, their
 * ret_pos entry set to -1, and (if vague_pos is not NULL) their positions
 * appended to vague_pos with n_vague advanced.  The token data stays in the slot
 * until the slot is reused, so kvr_encode can read it afterwards.
 * If a unit would evict more than evict_cap tokens, or overflow vague_cap, it
 * evicts nothing and n_evict[u] is set to minus the number it needed.
 *   scores      dev float32 [B, Hkv, n_cap], read
 *   ret_pos     dev int32 [B, Hkv, ret_cap], read and written
 *   n_ctx       dev int32 [B], read
 *   evict_slot, evict_pos  dev int32 [B, Hkv, evict_cap], written (first n_evict)
 *   n_evict     dev int32 [B, Hkv], written
 *   vague_pos   dev int32 [B, Hkv, vague_cap], appended; n_vague dev int32 [B, Hkv]
 *               read and written; both NULL to skip
 *   ws          unused at present (kvr_workspace_size reports 0)
 */
int32_t kvr_select(const kvr_desc* desc, const float* scores, int64_t n_cap,
                   int32_t* ret_pos, int32_t ret_cap,
                   const int32_t* n_ctx, int32_t n_recent, int32_t k_candidate,
                   int32_t* evict_slot, int32_t* evict_pos, int32_t* n_evict, int32_t evict_cap,
                   int32_t* vague_pos, int32_t* n_vague, int32_t vague_cap,
                   void* ws, size_t ws_bytes, void* stream);

/*
 * Algorithm 1, batched: add count[u] tokens of every unit into its sketch.
 * Token e of unit u has its data in row src_slot[u, e] of k_src / v_src and
 * position J = tok_pos[u, e]; for every row i
 *     sketch_k[u, i, h_i(J)] += k      sketch_v[u, i, h_i(J)] += g_i(J) * v
 * (signs per desc->sign_mask).  Each touched sketch slot is computed as
 * float32(previous content) + contributions in the order of the list, summed
 * left to right in float32, and rounded once (nearest-even) to the storage type;
 * the result is therefore reproducible bit for bit.  Tokens whose src_slot is
 * outside [0, src_rows) are skipped.  Negative counts are treated as 0.
 *   k_src, v_src  dev [B, Hkv, src_rows, D] storage type, read
 *   src_slot, tok_pos  dev int32 [B, Hkv, cap], read;  count dev int32 [B, Hkv]
 *   sketch_k, sketch_v  dev [B, Hkv, r, w, D] storage type, read and written
 *   out_bucket  dev int32 [B, Hkv, cap, r] or NULL: h_i(J) of every listed token
 *   out_sign    dev uint8 [B, Hkv, cap] or NULL: bit i set iff g_i(J) = -1
 *   ws          per kvr_workspace_size(KVR_OP_ENCODE, cap, 0)
 * Lists of up to 64 tokens per unit (cap <= 64) take any w; longer lists go through
 * a sort by slot that supports w <= 8192, beyond that KVR_ERR_UNSUPPORTED.
 */
int32_t kvr_encode(const kvr_desc* desc, const void* k_src, const void* v_src, int32_t src_rows,
                   const int32_t* src_slot, const int32_t* tok_pos, const int32_t* count, int32_t cap,
                   void* sketch_k, void* sketch_v, int32_t* out_bucket, uint8_t* out_sign,
                   void* ws, size_t ws_bytes, void* stream);

/*
 * Algorithm 3 for one decode step, in one launch: exactly kvr_append, then
 * kvr_select, then kvr_encode of the tokens that kvr_select listed (read from
 * the retained slots they just left), with the same arguments, the same results
 * (also for n_recent = 0, where the token just appended is itself a Candidate)
 * and the same bit-reproducible sketch as the three separate calls.  Any number
 * of tokens up to evict_cap may leave a unit in one call (Slack > 0: see
 * kvr_recent_size).  For the decode steady state only: ret_cap <= 32768 and
 * evict_cap <= 64, otherwise KVR_ERR_UNSUPPORTED (compress a prompt with the
 * separate calls).
 */
int32_t kvr_step_update(const kvr_desc* desc, const void* k_new, const void* v_new, const int32_t* n_ctx,
                        void* k_ret, void* v_ret, int32_t* ret_pos, int32_t ret_cap,
                        const float* scores, int64_t n_cap, int32_t n_recent, int32_t k_candidate,
                        int32_t* evict_slot, int32_t* evict_pos, int32_t* n_evict, int32_t evict_cap,
                        int32_t* vague_pos, int32_t* n_vague, int32_t vague_cap,
                        void* sketch_k, void* sketch_v, void* stream);

/*
 * The swap loop of Algorithm 3 (its second while-loop), per unit, at most
 * max_swaps times: as long as the lowest Candidate score times ReplaceRate is
 * below the highest Vague score, that Vague token is queried from the sketch and
 * deleted from it, the lowest Candidate is popped and inserted into the sketch,
 * and the queried estimate takes the Candidate's place.
 * Candidate = occupied slots with ret_pos < n_ctx[b] - n_recent.  C.Min: lowest
 * scores[ret_pos], ties: the later position (the token kvr_select would pop
 * first).  V.Max: highest scores[vague_pos[i]], ties: the earlier position.  The
 * product and the comparison are float32.  V.Query is Algorithm 2 (as in
 * kvr_reconstruct).  V.Delete subtracts the queried estimate from the slots an
 * insert of that position adds to, with the same signs; together with the insert
 * of the popped Candidate it is one sketch update in the sense of kvr_encode
 * (list order: delete, insert; float32 sums; a touched slot is rounded once).
 * Afterwards the Candidate's slot holds the estimate (k_ret, v_ret) at the Vague
 * token's position (ret_pos), and the Vague token's entry of vague_pos holds the
 * popped Candidate's position; n_vague and the number of occupied slots do not
 * change.  The paper fixes ReplaceRate = 1.1 (ablation of the replacement rate).
 *   scores     dev float32 [B, Hkv, n_cap], read
 *   k_ret, v_ret  dev [B, Hkv, ret_cap, D] storage type, read and written
 *   ret_pos    dev int32 [B, Hkv, ret_cap], read and written;  n_ctx dev int32 [B]
 *   sketch_k, sketch_v  dev [B, Hkv, r, w, D], read and written
 *   vague_pos  dev int32 [B, Hkv, vague_cap], read and written; n_vague dev int32
 *              [B, Hkv], read (clamped to [0, vague_cap])
 *   n_swapped  dev int32 [B, Hkv] or NULL: swaps done
 *   swap_log   dev int32 [B, Hkv, max_swaps, 2] or NULL: per swap (position brought
 *              back from the Vague part, position sent there)
 * replace_rate must be finite and > 0, 0 <= max_swaps <= 65536, else
 * KVR_ERR_INVALID_ARG.  max_swaps = 0 only writes n_swapped = 0.
 */
int32_t kvr_swap_back(const kvr_desc* desc, const float* scores, int64_t n_cap,
                      void* k_ret, void* v_ret, int32_t* ret_pos, int32_t ret_cap,
                      const int32_t* n_ctx, int32_t n_recent, float replace_rate, int32_t max_swaps,
                      void* sketch_k, void* sketch_v,
                      int32_t* vague_pos, const int32_t* n_vague, int32_t vague_cap,
                      int32_t* n_swapped, int32_t* swap_log, void* stream);

/*
 * Algorithm 2, batched: for token position J = tok_pos[u, e], e < count[u],
 *     k_out[u, e, c] = median_i sketch_k[u, i, h_i(J), c]
 *     v_out[u, e, c] = median_i g_i(J) * sketch_v[u, i, h_i(J), c]
 * element-wise over the D channels (signs per desc->sign_mask, even r per
 * desc->median_mode).  Rows e >= count[u] of the outputs are not written.
 *   sketch_k, sketch_v  dev [B, Hkv, r, w, D], read
 *   tok_pos  dev int32 [B, Hkv, cap], read;  count dev int32 [B, Hkv], read
 *   k_out, v_out  dev [B, Hkv, cap, D] storage type, written
 */
int32_t kvr_reconstruct(const kvr_desc* desc, const void* sketch_k, const void* sketch_v,
                        const int32_t* tok_pos, const int32_t* count, int32_t cap,
                        void* k_out, void* v_out, void* stream);

/*
 * Algorithm 4 + attention, fused: one decode query per q head attends over all
 * tokens of its kv head's unit -- retained tokens read raw, Vague tokens
 * reconstructed on the fly as in kvr_reconstruct (never written to memory):
 *     p[hq, j] = softmax_j(softmax_scale * q[hq] . k*_j),  out[hq] = sum_j p[hq, j] v*_j
 * and, if scores is not NULL, every token's cumulative score grows by the sum
 * of p over the G q heads of its kv head (Overview, Calculation Phase: the
 * attention scores are kept and accumulated per token).
 * Slots with ret_pos < 0 are skipped; ret_pos == NULL means slot s holds
 * position s for all ret_cap slots.  n_vague == NULL means no Vague tokens
 * (plain dense decode attention).  A unit with no token at all yields out = 0.
 *   q          dev [B, Hq, D] storage type, read
 *   k_ret, v_ret  dev [B, Hkv, ret_cap, D], read;  ret_pos dev int32 [B, Hkv, ret_cap]
 *   sketch_k, sketch_v  dev [B, Hkv, r, w, D], read
 *   vague_pos  dev int32 [B, Hkv, vague_cap], n_vague dev int32 [B, Hkv], read
 *   out        dev float32 [B, Hq, D], written
 *   scores     dev float32 [B, Hkv, n_cap] read and written, or NULL; positions
 *              >= n_cap are not accumulated
 *   ws         per kvr_workspace_size(KVR_OP_ATTEND, ret_cap, vague_cap)
 *   opts       host, or NULL: see kvr_attend_opts
 */
int32_t kvr_attend_decode(const kvr_desc* desc, const void* q,
                          const void* k_ret, const void* v_ret, const int32_t* ret_pos, int32_t ret_cap,
                          const void* sketch_k, const void* sketch_v,
                          const int32_t* vague_pos, const int32_t* n_vague, int32_t vague_cap,
                          float* out, float* scores, int64_t n_cap,
                          void* ws, size_t ws_bytes, const kvr_attend_opts* opts, void* stream);

/*
 * kvr_attend_decode for callers that cannot allocate device memory or hand over a
 * workspace: code running under HIP graph capture, tight serving loops, harnesses
 * that forbid allocation.  Same arguments (without ws / ws_bytes), same kernels and
 * same results as kvr_attend_decode; the scratch memory is a fixed array of
 * KVR_STATIC_SCRATCH_BYTES in device memory that belongs to the library's code
 * object (each GPU the library runs on holds its own copy until the process
 * ends).  The call allocates and frees nothing.  A call whose
 * kvr_workspace_size(KVR_OP_ATTEND, ret_cap, vague_cap) exceeds
 * KVR_STATIC_SCRATCH_BYTES is refused with KVR_ERR_WORKSPACE_TOO_SMALL before
 * anything is launched (the named workloads need up to 70 MiB).  All calls on one
 * GPU share that GPU's array: calls that can overlap in time (different streams,
 * different host threads) race on it; order them on one stream or use
 * kvr_attend_decode with separate workspaces.  Nothing in the array has to
 * survive between calls and nothing in it needs clearing.
 */
#define KVR_STATIC_SCRATCH_BYTES (80u << 20)
int32_t kvr_attend_decode_static(const kvr_desc* desc, const void* q,
                                 const void* k_ret, const void* v_ret, const int32_t* ret_pos, int32_t ret_cap,
                                 const void* sketch_k, const void* sketch_v,
                                 const int32_t* vague_pos, const int32_t* n_vague, int32_t vague_cap,
                                 float* out, float* scores, int64_t n_cap,
                                 const kvr_attend_opts* opts, void* stream);

/*
 * The Calculation Phase for n_q query tokens per sequence at once (a chunk of
 * prompt or of drafted tokens): as the Overview describes the phase, the layer's
 * cache is rebuilt once (Algorithm 4; Vague tokens by Algorithm 2: inside the
 * attention kernel, one rebuilt piece serving all queries, for bf16 sketches of
 * three rows; otherwise written to workspace and read back once) and attention
 * then runs over it for all queries.
 * Query t of sequence b sits at position n_ctx[b] - n_q + t (the n_q newest
 * tokens, already pushed into the Recent part) and attends over the tokens at
 * positions <= its own:
 *     p[t, hq, j] = softmax over visible j of softmax_scale * q[t, hq] . k*_j
 *     out[t, hq]  = sum_j p[t, hq, j] v*_j
 * and, if scores is not NULL, every token's cumulative score grows by the sum of
 * p over the n_q queries and the G q heads of its kv head.  n_q = 1 computes what
 * kvr_attend_decode computes (by this other route).
 * bf16 storage only, n_q * G in {1, 2, 4, 8, 16} (G = n_q_heads / n_kv_heads),
 * otherwise KVR_ERR_UNSUPPORTED.
 *   q          dev [B, n_q, Hq, D] bf16, read;   n_ctx dev int32 [B], read
 *   k_ret .. vague_cap, scores, n_cap   as for kvr_attend_decode (ret_pos must not be NULL)
 *   out        dev float32 [B, n_q, Hq, D], written
 *   ws         per kvr_attend_multi_workspace_size(desc, n_q, ret_cap, vague_cap): room for the rebuilt
 *              Vague tokens of all units (2 * vague_cap * D * 2 bytes per unit; per-token scratch of the
 *              in-kernel routes lives there too), slice partials, logits
 */
int32_t kvr_attend_multi_workspace_size(const kvr_desc* desc, int32_t n_q, int64_t ret_cap, int64_t vague_cap,
                                        size_t* bytes);
int32_t kvr_attend_multi(const kvr_desc* desc, const void* q, int32_t n_q, const int32_t* n_ctx,
                         const void* k_ret, const void* v_ret, const int32_t* ret_pos, int32_t ret_cap,
                         const void* sketch_k, const void* sketch_v,
                         const int32_t* vague_pos, const int32_t* n_vague, int32_t vague_cap,
                         float* out, float* scores, int64_t n_cap,
                         void* ws, size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* KVR_H */
