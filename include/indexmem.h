/*
 * indexmem.h - C ABI of libindexmem: the bounded-budget KV step of IndexMem on one MI355X.
 *
 * One attention layer keeps, per unit (batch element b, KV head h), a slot array of cached
 * keys / values, their indexer keys and token positions, a live length, and a fixed-size
 * latent memory state (M, b).  A step of the path is
 *     append new (k, v)  ->  im_index_score  ->  im_topb_select  ->  im_memory_update
 *                        ->  im_compact_kv   ->  im_decode_attn_with_readout
 * i.e. the score -> TopK -> Gather eviction framework of Section 2.2 of the paper with the
 * learnable indexer of Section 3.1 as the score function, the online latent-memory write of
 * Section 3.2 for the evicted entries, and decode attention over the retained entries plus
 * the gated memory readout (Eq. latent_residual_fuse).
 *
 * Two state layouts.  head_shared = 0 (default): everything above is kept per unit; indexer keys
 * come from the cached key rows with d_index = 64.  head_shared = 1, the layer-wide form of the
 * paper's text (Section 3.1: one indexer key per token from the hidden state, shared by all heads;
 * Section 3.2 and Algorithm 1: one memory module per layer shared across heads, evicted rows summed
 * across heads per token; Section 4: d_index = d_head / 8 = 16): all KV heads of a sequence form
 * one SET that holds the same tokens in the same slots; Kidx, pos, len, n_projected, the scores,
 * the keep / evict lists and (M, b) exist once per sequence (the H_kv axis below is dropped) and
 * K, V stay per unit.  Tokens enter through im_append_kv_hidden.  The step-by-step entry points and
 * im_decode_step serve both layouts; im_attend_step and im_decode_step_shared have the twins
 * im_attend_step_hidden and im_decode_step_shared_hidden.
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers unless a comment says "host".  The caller owns all
 *     device memory, including the workspace; the library never allocates device memory.
 *   - `stream` is a hipStream_t passed as void*.  Calls only enqueue work on it; they do not
 *     synchronise (im_query_status is the one exception) and may be captured in a HIP graph.
 *   - bf16 tensors are raw 16-bit patterns (uint16_t).  Tensors are dense, row-major, in the
 *     shapes given, with no padding.
 *   - Return value: IM_OK, or a negative error.  Argument validation is done on the host
 *     before anything is enqueued, so an invalid call leaves all buffers untouched.
 *     im_last_error() gives a text for the last error of a handle.
 *   - Calls on one handle must not overlap (they share the workspace); different layers may
 *     share a handle when their calls are issued in stream order.
 */
#ifndef INDEXMEM_H
#define INDEXMEM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define IM_OK 0
#define IM_ERR_INVALID_ARG (-1)  /* null pointer, shape or range violation                  */
#define IM_ERR_UNSUPPORTED (-2)  /* valid in principle, not built (e.g. head_dim != 128)     */
#define IM_ERR_LAUNCH (-3)       /* a HIP call failed; see im_last_error()                   */

/* bits of the device-side status word returned by im_query_status() */
#define IM_STATUS_APPEND_OVERFLOW 1 /* an append would have exceeded `capacity`; it was dropped */
#define IM_STATUS_LIVE_EXCEEDED 2   /* a unit's length exceeded the im_set_max_live() promise   */
#define IM_STATUS_OVER_BUDGET 8     /* im_decode_step: a unit entered with len > budget; only one
                                       entry was evicted from it                                  */

typedef struct im_handle im_handle; /* opaque: validated config + workspace pointer, host memory */

/* Shape of one layer's state and the method's constants. */
typedef struct im_config {
  int32_t batch;        /* B                                                                  */
  int32_t n_q_heads;    /* H   (multiple of n_kv_heads; H / H_kv <= 8)                        */
  int32_t n_kv_heads;   /* H_kv                                                               */
  int32_t head_dim;     /* d_head, must be 128                                                */
  int32_t capacity;     /* C: slots per unit in K, V, Kidx, pos, scores and the index lists   */
  int32_t n_idx_heads;  /* H_index (1..16); the paper uses H / 4 (Section 4)                  */
  int32_t idx_dim;      /* d_index: 64 with head_shared = 0, 16 with head_shared = 1          */
  int32_t mem_dim;      /* d_mem, must be 128                                                 */
  int32_t gate_in_dim;  /* width of the gate input X_s (multiple of 16)                       */
  int32_t n_sink;       /* first token positions always kept (4 in the paper, Section 4)      */
  int32_t n_recent;     /* newest positions always kept (0: none)                             */
  int32_t fold_block;   /* evicted rows are folded into the memory in blocks of this (64;
                           a multiple of 32)                                                   */
  int32_t max_queries;  /* largest n_q a call to im_index_score will pass                     */
  int32_t head_shared;  /* 0: state per (batch, KV head); 1: one set per sequence (see above);
                           then gate_in_dim is also d_model, the width of the hidden states     */
  float rms_eps;        /* RMSNorm epsilon of the indexer's QK-Norm                           */
  float mem_eps;        /* epsilon of the readout denominator (Eq. latent_readout)            */
  float softmax_scale;  /* attention logit scale, 1/sqrt(d_head)                              */
} im_config;

/* Slow weights of one layer (device pointers, bf16, read-only). */
typedef struct im_params {
  const void* Uq;       /* [H_index * d_index, H * d_head]  query down-projection            */
  const void* G;        /* [H_index, gate_in_dim]           head gate                        */
  const void* Uk;       /* [d_index, d_head]                key projection, shared by heads
                           (head_shared = 1: [d_index, gate_in_dim], applied to hidden states) */
  const void* norm_q_w; /* [d_index] RMSNorm weight of indexer queries, or NULL for ones     */
  const void* norm_k_w; /* [d_index] RMSNorm weight of indexer keys, or NULL for ones        */
  const void* Wtheta;   /* [d_mem, d_head] Linear_theta of the memory (no bias)              */
  const void* wg;       /* [d_head] weight of the read gate g(q) = sigmoid(wg . q + cg)      */
  float cg;             /* bias of the read gate                                             */
} im_params;

/* State of one layer (device pointers, read and written in place).  With head_shared = 1 every
 * array but K and V drops its H_kv axis: Kidx [B, C, d_index], pos [B, C], len [B], M [B, d_mem,
 * d_head], ... */
typedef struct im_state {
  void* K;              /* [B, H_kv, C, d_head]  bf16                                        */
  void* V;              /* [B, H_kv, C, d_head]  bf16                                        */
  void* Kidx;           /* [B, H_kv, C, d_index] bf16: normalised indexer keys               */
  int32_t* pos;         /* [B, H_kv, C] token position of each slot                          */
  int32_t* len;         /* [B, H_kv] live slots: [0, len)                                    */
  int32_t* n_projected; /* [B, H_kv] slots [0, n_projected) have a valid Kidx row            */
  float* M;             /* [B, H_kv, d_mem, d_head] fp32 fast weights                        */
  float* b;             /* [B, H_kv, d_mem]         fp32 stabiliser                          */
} im_state;

/* Bytes of workspace a handle for `cfg` needs (0 if cfg is invalid).  Host only. */
size_t im_workspace_bytes(const im_config* cfg);

/* Validate `cfg` (host pointer) and create a handle that uses `workspace` (device pointer,
 * 256-byte aligned, at least im_workspace_bytes(cfg) bytes, contents arbitrary).  Host only:
 * touches no GPU.  The first enqueuing call clears the part of the workspace that needs it. */
int32_t im_create(const im_config* cfg, void* workspace, size_t workspace_bytes, im_handle** out);
void im_destroy(im_handle* h);
const char* im_last_error(const im_handle* h);   /* h = NULL: the calling thread's last error of a call
                                                    that takes no handle */

/* Promise that no unit's `len` exceeds `max_live` until the next call of this function;
 * kernels size their grids by it (default: capacity).  A unit (set) found longer than that sets
 * IM_STATUS_LIVE_EXCEEDED; its entries beyond max_live are not looked at (scores are written and
 * attention runs over the first max_live entries only), and nothing is dropped on that basis:
 * im_topb_select gives it a keep list of those entries and an empty evict list, im_compact_kv leaves
 * it as it is, and the fused steps append its new token but evict nothing from it and keep its
 * true length. */
int32_t im_set_max_live(im_handle* h, int32_t max_live);

/* Copy the device status word to *status_host (host pointer), clear it, and WAIT for `stream`. */
int32_t im_query_status(im_handle* h, int32_t* status_host, void* stream);

/* Helper: new tokens enter the cache.  Copies k_new, v_new [B, H_kv, n_new, d_head] (bf16) to
 * slots [len, len + n_new) of every unit, pos_new [B, n_new] to their positions, and adds n_new
 * to len.  A unit with len + n_new > capacity is left unchanged and IM_STATUS_APPEND_OVERFLOW is
 * set.  1 <= n_new <= capacity.
 * k_new = v_new = NULL: the rows are already in place in slots [len, len + n_new) of K and V (the
 * state's K / V may be the very buffers a prompt's K / V projections were written to); only the
 * positions and lengths follow.  This is how a prompt is evicted BEFORE it is cached (Section 3.1,
 * "pre-eviction"): run the step on such a state of capacity L, then copy the first n_keep slots of
 * its arrays to the budget-sized state that decoding uses. */
int32_t im_append_kv(im_handle* h, const im_state* st, const void* k_new, const void* v_new,
                     const int32_t* pos_new, int32_t n_new, void* stream);

/* The same for head_shared = 1 (im_append_kv then returns IM_ERR_UNSUPPORTED): K, V rows as above,
 * one position / length per sequence, and the tokens' indexer keys from their hidden states
 * (Section 3.1 "Architecture": k_t = Norm(U_k X_t), one key for all heads):
 * Kidx[b, len + i] = bf16(RMSNorm(Uk x_new[b, i])), fp64 arithmetic; n_projected follows len.
 * x_new [B, n_new, gate_in_dim] bf16.  n_new <= capacity. */
int32_t im_append_kv_hidden(im_handle* h, const im_params* p, const im_state* st, const void* k_new,
                            const void* v_new, const void* x_new, const int32_t* pos_new,
                            int32_t n_new, void* stream);

/* Step a1, the indexer (Section 3.1 "Architecture"; Algorithm 1, `indexer`).
 *  (i)  keys: every slot in [n_projected, len) gets Kidx = bf16(RMSNorm(Uk K_slot)); then
 *       n_projected = len.
 *  (ii) queries, once per (b, s) and shared by the KV heads: q_s = RMSNorm per indexer head of
 *       Uq flatten(q_new[b, s]) (kept in fp32), alpha_s = G x_gate[b, s] / sqrt(H_index d_index).
 *  (iii) scores_out[b, h, t] = max over s with q_pos[b, s] >= pos[b, h, t] of
 *        sum_j alpha_{s,j} ReLU(q_{s,j} . Kidx[b, h, t]),  -inf if no query may see slot t.
 * q_new [B, n_q, H, d_head] bf16; x_gate [B, n_q, gate_in_dim] bf16; q_pos [B, n_q] int32;
 * scores_out [B, H_kv, C] fp32, written for slots < len only.  1 <= n_q <= max_queries.
 * All arithmetic that feeds the stored bf16 / fp32 values is fp64.
 * head_shared = 1: (i) is skipped (the keys were made at the append), x_gate holds the queries'
 * hidden states, and scores_out is [B, C]: one score per token of the sequence. */
int32_t im_index_score(im_handle* h, const im_params* p, const im_state* st, const void* q_new,
                       const void* x_gate, const int32_t* q_pos, int32_t n_q, float* scores_out,
                       void* stream);

/* Step a2, per-unit top-B (Section 2.2, I = TopK(S, L'); sink retention: Section 4 "Models and
 * Evaluation Setup").  Keeps n_keep = min(budget, len) slots: those whose position is < n_sink
 * or among the n_recent newest count as score +inf; the order is score descending, then position
 * ascending, then slot ascending (-0 equals +0; NaN scores are a caller error).
 * keep_idx / evict_idx [B, H_kv, C] int32 receive the kept / evicted slots in ascending order,
 * n_keep / n_evict [B, H_kv] their counts (n_keep + n_evict = len).
 * n_sink + n_recent <= budget <= capacity. */
int32_t im_topb_select(im_handle* h, const float* scores, const im_state* st, int32_t budget,
                       int32_t* keep_idx, int32_t* evict_idx, int32_t* n_keep, int32_t* n_evict,
                       void* stream);

/* Step a3, latent-memory write (Eqs. latent_write_A, latent_write_b; Algorithm 1, `mem_write`):
 * for every unit with n_evict > 0, with phi_i = Wtheta K_i over the evicted slots i,
 *     M <- lambda M + eta sum_i phi_i V_i^T,     b <- lambda b + eta sum_i phi_i * phi_i.
 * One call is one eviction event: lambda is applied once.  Units with n_evict = 0 are untouched.
 * Reads the evicted rows through evict_idx from the cache as it is BEFORE im_compact_kv.
 * 0 < lambda <= 1, eta > 0.
 * head_shared = 1: one memory per sequence; K_i and V_i are the sums over the KV heads of the rows
 * in evicted slot i (Algorithm 1, `mem_write`: evicted rows are summed across heads per token). */
int32_t im_memory_update(im_handle* h, const im_params* p, const im_state* st,
                         const int32_t* evict_idx, const int32_t* n_evict, float lambda, float eta,
                         void* stream);

/* Step a4, the Gather of Section 2.2 in place: kept entries in slots >= n_keep move, in ascending
 * order, into the evicted slots < n_keep, in ascending order (rows of K, V, Kidx and pos); then
 * len = n_projected = n_keep.  Requires n_projected == len on entry (im_index_score was called
 * after the last append) and the lists of im_topb_select for the current cache.
 * head_shared = 1: the sequence's lists are applied to the rows of each of its KV heads. */
int32_t im_compact_kv(im_handle* h, const im_state* st, const int32_t* keep_idx,
                      const int32_t* n_keep, const int32_t* evict_idx, const int32_t* n_evict,
                      void* stream);

/* Step a4 out of place, for evicting a prompt BEFORE it is cached (Section 3.1, "pre-eviction ... caches
 * only the selected KV states"): the kept entries of `src` (a state of this handle's capacity, e.g. one
 * that has adopted the prompt's K / V buffers through im_append_kv with no rows, after im_index_score,
 * im_topb_select and im_memory_update) are written to `dst`, a state of the same shape but with
 * dst_capacity slots per unit, in the very slots im_compact_kv would leave them in: rows of K, V, Kidx
 * and pos of slots [0, n_keep); M and b are copied; dst's len = n_projected = n_keep.  src is only
 * read; the two states must not share buffers.  A unit whose n_keep exceeds dst_capacity is left out
 * and sets IM_STATUS_APPEND_OVERFLOW.  Lists as im_topb_select wrote them for src. */
int32_t im_gather_kept(im_handle* h, const im_state* src, const im_state* dst, int32_t dst_capacity,
                       const int32_t* keep_idx, const int32_t* n_keep, const int32_t* evict_idx,
                       const int32_t* n_evict, void* stream);

/* Step a5, decode attention over the retained entries plus the gated memory readout
 * (Section 2.1 "KV Caching"; Eqs. latent_readout, latent_residual_fuse): for query head j of
 * KV head h = j / (H / H_kv),
 *     o_attn = softmax(softmax_scale q_j K^T) V over slots [0, len)   (0 if len = 0)
 *     phi = Wtheta q_j,  m = phi^T M / (sum_c phi_c^2 b_c + mem_eps),  g = sigmoid(wg . q_j + cg)
 *     out[b, j] = bf16(o_attn + g m);   readout_dbg[b, j] = g m  (fp32; may be NULL).
 * q, out [B, H, d_head] bf16; readout_dbg [B, H, d_head] fp32.
 * head_shared = 1: every query head of the sequence reads the sequence's one (M, b). */
int32_t im_decode_attn_with_readout(im_handle* h, const im_params* p, const im_state* st,
                                    const void* q, void* out, float* readout_dbg, void* stream);

/* For callers that cannot allocate device memory or bring a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): im_decode_attn_with_readout without a handle
 * and without a workspace.  The attention partials go to a buffer of IM_STATIC_SCRATCH_BYTES that is
 * part of the library's device code (one copy per GPU, held until the process ends); the call
 * allocates nothing, on the host or on the device, and only enqueues work on `stream`.
 * cfg (host pointer) is validated on every call; max_live (1..capacity) bounds every unit's length as
 * im_set_max_live does.  Needs 256 + 520 * batch * n_q_heads * ceil(max_live / 128) bytes of the
 * buffer: a larger call is rejected with IM_ERR_INVALID_ARG before anything is enqueued
 * (im_last_error(NULL) gives this thread's text for a call without a handle).
 * status_dev: optional device word that IM_STATUS_LIVE_EXCEEDED is OR-ed into (NULL: not reported).
 * Results are those of im_decode_attn_with_readout, bit for bit.
 * The GPU that owns `stream` must be the current device.  All calls on one GPU share that GPU's
 * buffer: calls that overlap in time on one GPU (two streams, two threads) race; calls in stream
 * order on one stream do not.  The first call on a GPU looks the buffer's address up
 * (hipGetSymbolAddress): make it outside a graph capture. */
#define IM_STATIC_SCRATCH_BYTES (16u << 20)
int32_t im_decode_attn_with_readout_static(const im_config* cfg, int32_t max_live, const im_params* p,
                                           const im_state* st, const void* q, void* out,
                                           float* readout_dbg, int32_t* status_dev, void* stream);

/* The whole step for ONE new token per sequence, fused into three launches: exactly
 *   im_append_kv(n_new = 1) -> im_index_score(n_q = 1) -> im_topb_select(budget) ->
 *   im_memory_update(lambda, eta) -> im_compact_kv -> im_decode_attn_with_readout
 * (Sections 2.2, 3.1, 3.2 of the paper, as cited at those calls) for the steady state of decoding
 * with one eviction per step: every unit must enter with len <= budget, so that at most one entry
 * (the one ranked last by im_topb_select's order) leaves.  A unit that enters above the budget
 * still evicts only one entry and raises IM_STATUS_OVER_BUDGET.
 * q [B, H, d_head] bf16 is both the indexer's query input and the attention query; x_gate
 * [B, gate_in_dim] bf16; q_pos [B] int32; k_new, v_new [B, H_kv, 1, d_head] bf16; pos_new [B].
 * out [B, H, d_head] bf16.  Optional (NULL to skip): readout_dbg [B, H, d_head] fp32,
 * evicted_slot [B, H_kv] int32 (slot that was evicted, before compaction; -1 if none),
 * scores_dbg [B, H_kv, C] fp32 (as im_index_score writes them).
 * batch <= 64.  n_sink + n_recent <= budget <= capacity - 1 is not required, but a unit with
 * len = capacity cannot take the new token (IM_STATUS_APPEND_OVERFLOW).
 * head_shared = 1: the same step as im_append_kv_hidden(n_new = 1) -> ... in four launches; x_gate
 * [B, gate_in_dim] is the new token's hidden state (it feeds the head gate and the token's indexer
 * key); evicted_slot is [B], scores_dbg [B, C]; at most 16 KV heads and max_live <= 8193. */
int32_t im_decode_step(im_handle* h, const im_params* p, const im_state* st, const void* q,
                       const void* x_gate, const int32_t* q_pos, const void* k_new, const void* v_new,
                       const int32_t* pos_new, int32_t budget, float lambda, float eta, void* out,
                       float* readout_dbg, int32_t* evicted_slot, float* scores_dbg, void* stream);

/* One token of the periodic decode schedule (Section 4, "Models and Evaluation Setup": attention
 * every step, compression once per interval), fused into two launches: exactly
 *   im_append_kv(n_new = 1) -> im_decode_attn_with_readout
 * Nothing is scored or evicted; the new entry's indexer key is computed on the way (n_projected
 * follows len), so the interval's im_index_score has nothing left to project.  The caller bounds
 * the live length with im_set_max_live (budget + interval).  Arguments as in im_decode_step. */
int32_t im_attend_step(im_handle* h, const im_params* p, const im_state* st, const void* q,
                       const void* k_new, const void* v_new, const int32_t* pos_new, void* out,
                       float* readout_dbg, void* stream);

/* The same for head_shared = 1: x_new [B, gate_in_dim] bf16 is the new token's hidden state, from
 * which its indexer key is made on the way (Section 3.1 "Architecture": k_t = Norm(U_k X_t)).
 * At most 16 KV heads, max_live <= 8193. */
int32_t im_attend_step_hidden(im_handle* h, const im_params* p, const im_state* st, const void* q,
                              const void* x_new, const void* k_new, const void* v_new,
                              const int32_t* pos_new, void* out, float* readout_dbg, void* stream);

/* Index reuse across neighbouring layers (Appendix "From Running Mean to IndexCache": the indexer
 * runs once per group of layers and the other layers of the group reuse its decision).  The step
 * of a FOLLOWER layer for one new token per sequence, three launches, nothing scored: exactly
 *   im_append_kv(n_new = 1) -> im_memory_update + im_compact_kv with the single entry in slot
 *   evict_slot[b, h] (as the cache stands after the append; -1 or >= len: nothing leaves) ->
 *   im_decode_attn_with_readout.
 * evict_slot [B, H_kv] int32 is what im_decode_step wrote to its evicted_slot output for the
 * group's leading layer; the follower's cache must have the leader's slot layout (same appends,
 * same evictions since the start, e.g. a prefill compacted with the leader's keep / evict lists).
 * Other arguments as in im_decode_step. */
int32_t im_decode_step_shared(im_handle* h, const im_params* p, const im_state* st, const void* q,
                              const void* k_new, const void* v_new, const int32_t* pos_new,
                              const int32_t* evict_slot, float lambda, float eta, void* out,
                              float* readout_dbg, void* stream);

/* The same for head_shared = 1: evict_slot is [B] (one slot per sequence, as im_decode_step reports it
 * in this layout), x_new [B, gate_in_dim] the new token's hidden state (its indexer key is made and
 * stored as in im_attend_step_hidden, so that the follower's Kidx stays consistent). */
int32_t im_decode_step_shared_hidden(im_handle* h, const im_params* p, const im_state* st, const void* q,
                                     const void* x_new, const void* k_new, const void* v_new,
                                     const int32_t* pos_new, const int32_t* evict_slot, float lambda,
                                     float eta, void* out, float* readout_dbg, void* stream);

/* Measurement only (not part of the method): one launch that reads `bytes` (a multiple of 16) from
 * src (device, 16-byte aligned) with 16-byte streaming loads on all CUs and writes nothing, unless the
 * XOR of all words read equals `never`, in which case that word goes to sink[0] (device; pass a value
 * the data cannot produce).  The benchmark times it at the decode step's bytes per launch, as the
 * plain-read ceiling printed beside the step's own rate. */
int32_t im_stream_read(const void* src, size_t bytes, uint32_t never, void* sink, void* stream);

/* Kernel timing for benchmarks (not part of the method).  After im_profile_start, every
 * im_decode_step on this handle brackets part of its launch sequence (prep kernel, main kernel,
 * tail kernel) with a pair of HIP events on the launch stream, for at most max_records calls:
 *   IM_PROFILE_MAIN           the main kernel alone (scoring and attention partials of every
 *                             128-key split: the launch that streams the cache);
 *   IM_PROFILE_PREP           the prep kernel alone;
 *   IM_PROFILE_PREP_AND_MAIN  both, with no event between them.
 * An event pair around one launch also spans the hand-over between the event and the dispatch;
 * mean(PREP_AND_MAIN) - mean(PREP) is the main kernel as it runs behind the prep kernel.
 * im_profile_stop WAITS for `stream`, writes the elapsed milliseconds of the recorded spans to
 * ms_host[0 .. *n_records) (host pointers; ms_host holds max_records floats) and releases the
 * events.  Do not use while the stream is being captured into a graph. */
#define IM_PROFILE_MAIN 0
#define IM_PROFILE_PREP 1
#define IM_PROFILE_PREP_AND_MAIN 2
int32_t im_profile_start(im_handle* h, int32_t max_records, int32_t span);
int32_t im_profile_stop(im_handle* h, float* ms_host, int32_t* n_records, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* INDEXMEM_H */
