/* prefix_attn.h -- C ABI of the prefix-shared GRPO prefill attention library (gfx950 / MI355X).
 *
 * The operation (paper Sec. 4.2: G responses are sampled for one question; Sec. 5.1:
 * the gathered video embeddings are computed once and reused by every rollout;
 * Sec. 5.2: every rollout is prefilled over the whole multimodal sequence):
 *
 *   One call handles one (video, question) pair.  The video tokens form a prefix of
 *   P tokens whose keys/values are shared by all G rollouts.  Rollout g owns a
 *   suffix of S_g = prompt + response_g tokens.  For rollout g, query head h
 *   (kv head c = h / (Hq/Hkv)) and suffix row i, the visible keys are all P prefix
 *   keys of kv head c and the rollout's own suffix keys 0..i (diagonal included):
 *
 *       s_j = softmax_scale * <q, k_j>,   LSE = ln sum_j exp(s_j),
 *       out = sum_j exp(s_j - LSE) v_j.
 *
 *   The library computes this in three steps: a prefix pass (no mask; all rollouts'
 *   rows of one kv head stacked against LDS-staged prefix K/V tiles), a causal suffix
 *   pass, and a log-sum-exp merge of the two partial results (a kernel of its own on the
 *   fp32 path; on the bf16 path the suffix pass does it in its epilogue).  On the bf16
 *   path a small layout pre-pass first rewrites V into transposed, LDS-ready tile images.
 *
 * Conventions
 *   - No C++ types, no exceptions and no printing cross this boundary.  Every call
 *     returns a pa_status_t (0 = PA_OK); nothing aborts.
 *   - Layouts are token-major and contiguous.  T = sum_g S_g; rollouts are packed
 *     back to back in rollout order.
 *   - Pointers named q, k_*, v_*, out, workspace, lse_out are DEVICE pointers on the
 *     plan's device and must be 16-byte aligned (else PA_ERR_ALIGN).  `desc`,
 *     `suffix_lens`, `plan_out`, `workspace_bytes_out` are HOST pointers.
 *   - The caller owns every device buffer, including the workspace.  The plan owns
 *     host metadata and small device-side schedule tables which prefix_attn_plan
 *     allocates and prefix_attn_destroy frees.  prefix_attn_forward and
 *     prefix_attn_lse allocate nothing and never synchronise: they only enqueue work
 *     on the given stream.
 *   - A plan is immutable; forward calls on different streams are safe when they use
 *     different workspaces.
 */
#ifndef PREFIX_ATTN_H_
#define PREFIX_ATTN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct prefix_attn_plan prefix_attn_plan_t; /* opaque, library-owned */

typedef enum {
  PA_OK = 0,
  PA_ERR_NULL = 1,        /* a required pointer is NULL */
  PA_ERR_SHAPE = 2,       /* a size is out of range or inconsistent */
  PA_ERR_UNSUPPORTED = 3, /* valid but not implemented (head_dim, dtype; bf16: a prefix or one rollout
                             whose K rows, len * Hkv * D * 2 bytes, reach 2 GiB) */
  PA_ERR_ALIGN = 4,       /* a device pointer is not 16-byte aligned */
  PA_ERR_WORKSPACE = 5,   /* workspace_bytes is smaller than the plan requires */
  PA_ERR_ALLOC = 6,       /* host or device allocation failed in prefix_attn_plan */
  PA_ERR_HIP = 7          /* a HIP runtime call or kernel launch failed */
} pa_status_t;

typedef enum { PA_F32 = 0, PA_BF16 = 1 } pa_dtype_t;

typedef struct {
  int32_t num_q_heads;        /* Hq >= 1 */
  int32_t num_kv_heads;       /* Hkv >= 1, Hq % Hkv == 0; q head h reads kv head h / (Hq/Hkv) */
  int32_t head_dim;           /* D in {64, 128} */
  int64_t prefix_len;         /* P >= 0; 0 gives plain packed causal attention */
  int32_t num_rollouts;       /* G >= 1 */
  const int32_t* suffix_lens; /* HOST array [G]; S_g >= 1; copied by prefix_attn_plan */
  float softmax_scale;        /* finite and > 0, e.g. 1/sqrt(D) */
  int32_t dtype;              /* pa_dtype_t of q, k, v, out; LSE is always fp32 */
  int32_t device;             /* HIP device ordinal; -1 = host-only plan (validation and
                                 schedule only; forward/lse on it return PA_ERR_UNSUPPORTED) */
} prefix_attn_desc_t;

/* Validate `desc`, build the work lists of the prefix pass and the suffix pass and
 * report the workspace size a forward call needs.  On success *plan_out receives a
 * plan to be released with prefix_attn_destroy; on failure *plan_out is NULL. */
int prefix_attn_plan(const prefix_attn_desc_t* desc, prefix_attn_plan_t** plan_out,
                     size_t* workspace_bytes_out);

/* Enqueue prefix pass, suffix pass and merge on `hip_stream` (a hipStream_t; NULL =
 * the default stream).
 *   q         [T, Hq,  D]  queries of all suffix tokens
 *   k_prefix  [P, Hkv, D]  shared video keys    (may be NULL when P == 0)
 *   v_prefix  [P, Hkv, D]  shared video values  (may be NULL when P == 0)
 *   k_suffix  [T, Hkv, D]  per-rollout prompt+response keys
 *   v_suffix  [T, Hkv, D]  per-rollout prompt+response values
 *   out       [T, Hq,  D]  attention output, same dtype as q
 *   workspace              scratch of at least the planned size; holds the two fp32
 *                          partial results, the merged LSE and (bf16) the V tile images
 *                          and the per-work-item flags the two kernels of a pass share
 * Argument errors are reported before anything is launched. */
int prefix_attn_forward(const prefix_attn_plan_t* plan, const void* q, const void* k_prefix,
                        const void* v_prefix, const void* k_suffix, const void* v_suffix, void* out,
                        void* workspace, size_t workspace_bytes, void* hip_stream);

/* prefix_attn_forward for callers that cannot allocate device memory or hold a workspace: code running
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and
 * result as prefix_attn_forward followed by prefix_attn_lse, but the workspace is an array of
 * PA_STATIC_SCRATCH_BYTES inside the library's device image (one per GPU, held until the process
 * ends); the call allocates nothing, frees nothing and does not synchronise.
 *   lse_out [Hq, T] fp32 DEVICE, 16-byte aligned, or NULL when the LSE is not wanted.
 * A plan whose workspace (workspace_bytes_out of prefix_attn_plan) exceeds PA_STATIC_SCRATCH_BYTES is
 * rejected with PA_ERR_WORKSPACE before anything is launched.  All calls on a GPU share that GPU's
 * array: calls that may overlap there (different streams, or threads, without ordering between them)
 * race and must use prefix_attn_forward with workspaces of their own.  Nothing in the array has to
 * survive between calls and nothing in it needs clearing. */
#define PA_STATIC_SCRATCH_BYTES (64u << 20)
int prefix_attn_forward_static(const prefix_attn_plan_t* plan, const void* q, const void* k_prefix,
                               const void* v_prefix, const void* k_suffix, const void* v_suffix, void* out,
                               float* lse_out, void* hip_stream);

/* Measurement variant of prefix_attn_forward: same arguments and result, but each of the
 * launches is bracketed by HIP events on `hip_stream` and the call WAITS for them.
 * kernel_ms (HOST [4]) receives the durations in milliseconds of {V layout pre-pass, prefix
 * pass, suffix pass, merge}; the prefix entry is ~0 when P == 0 or when the plan runs the
 * single sweep (then timed in the suffix-pass entry), the pre-pass entry is ~0 for fp32
 * plans, and the merge entry is ~0 when the suffix pass merges in its epilogue.  Creates and destroys events, so it is not for stream capture or
 * latency-critical loops. */
int prefix_attn_forward_timed(const prefix_attn_plan_t* plan, const void* q, const void* k_prefix,
                              const void* v_prefix, const void* k_suffix, const void* v_suffix,
                              void* out, void* workspace, size_t workspace_bytes, void* hip_stream,
                              float* kernel_ms);

/* Copy the merged log-sum-exp (natural log, fp32) of the last forward call that used
 * `workspace` into lse_out [Hq, T].  Must be enqueued after that forward call on the
 * same stream (or otherwise ordered after it); calling it on a workspace that no
 * forward call has filled yields unspecified values.  LSE is the hand-off for
 * merging with attention over further key shards. */
int prefix_attn_lse(const prefix_attn_plan_t* plan, const void* workspace, float* lse_out,
                    void* hip_stream);

/* ---- composition over key shards (paper Sec. 5.2: the prefill is spread over devices by
 *      sequence parallelism; here the shared prefix keys of one question are split into shards,
 *      each device attends all suffix rows to its shard, and the partial results are combined).
 *      These two calls are the part one device computes; moving partials between devices is the
 *      caller's business. ---- */

/* Like prefix_attn_forward, but the result stays an fp32 partial result over the keys this call
 * covers:  o_partial [T, Hq, D] (normalised over those keys), lse_partial [T, Hq] (natural log).
 * The plan's prefix_len is the number of prefix keys of THIS shard (k_prefix / v_prefix hold only
 * them).  include_suffix != 0: the keys covered are the shard and every rollout's own suffix keys
 * (exactly one shard of a sharded call does this); include_suffix == 0: the shard's prefix keys
 * only (needs prefix_len > 0, else PA_ERR_SHAPE; k_suffix / v_suffix may then be NULL).
 * Partials over disjoint key sets are combined with prefix_attn_merge_partials. */
int prefix_attn_forward_partial(const prefix_attn_plan_t* plan, const void* q, const void* k_prefix,
                                const void* v_prefix, const void* k_suffix, const void* v_suffix,
                                int32_t include_suffix, float* o_partial, float* lse_partial,
                                void* workspace, size_t workspace_bytes, void* hip_stream);

/* Combine n partial results over disjoint key sets of the same queries:
 *   LSE = ln sum_i e^{LSE_i},   out = sum_i e^{LSE_i - LSE} O_i,
 * which is the softmax over the union of the key sets.  o_partials / lse_partials are HOST arrays
 * of n DEVICE pointers ([T, Hq, D] and [T, Hq] fp32, 1 <= n <= PA_MAX_PARTIALS, else
 * PA_ERR_SHAPE).  out [T, Hq, D] has the plan's dtype; lse_out [Hq, T] fp32 may be NULL.  Only
 * T, Hq, D and the dtype of `plan` are used. */
#define PA_MAX_PARTIALS 16
int prefix_attn_merge_partials(const prefix_attn_plan_t* plan, int32_t n, const float* const* o_partials,
                               const float* const* lse_partials, void* out, float* lse_out,
                               void* hip_stream);

/* ---- backward (the policy model is trained through this attention: paper Eq. 1, Sec. 5.2) ----
 *
 * Given d_out = dL/d(out), computes the gradients of L with respect to the five inputs of the
 * forward call.  With W the softmax weights of a query row over its visible keys,
 *   dV_j = sum_rows W_j dO,   dS_j = W_j (<dO, v_j> - <dO, O>),
 *   dQ   = scale sum_j dS_j k_j,   dK_j = scale sum_rows dS_j q,
 * where a kv head sums over the q heads of its group and a PREFIX key/value additionally sums
 * over all G rollouts, because every rollout attends to the same cached video prefix
 * (Sec. 5.1).  The LSE is treated as a saved statistic, not as a differentiated output. */

/* Bytes of backward workspace a plan needs (per-row statistics; for bf16 also re-laid-out
 * copies of Q, dO and K, and for a short prefix fp32 partial prefix gradients of the row ranges
 * its key blocks are split over). */
int prefix_attn_backward_workspace(const prefix_attn_plan_t* plan, size_t* workspace_bytes_out);

/* Enqueue the backward on `hip_stream`.  All tensors are DEVICE pointers, 16-byte aligned, in
 * the plan's dtype, with the shapes of the forward call:
 *   q, k_prefix, v_prefix, k_suffix, v_suffix   the forward inputs, unchanged
 *   out    [T, Hq, D]   the forward output
 *   d_out  [T, Hq, D]   gradient of the objective with respect to `out`
 *   lse    [Hq, T]      fp32 log-sum-exp of the forward call on these inputs, as written by
 *                       prefix_attn_lse (the saved softmax statistic)
 *   dq [T, Hq, D], dk_prefix, dv_prefix [P, Hkv, D] (may be NULL when P == 0),
 *   dk_suffix, dv_suffix [T, Hkv, D]             outputs, fully overwritten
 *   workspace           scratch of at least prefix_attn_backward_workspace bytes (the forward
 *                       workspace is not needed and may be reused for it if large enough)
 * Every gradient element is produced by exactly one workgroup in a fixed order (no atomics),
 * so results are bitwise reproducible.  bf16 plans with T * (Hq/Hkv) * D * 2 >= 2^31 bytes of
 * stacked rows per kv head (about 8.4 M token-heads at D = 128) return PA_ERR_UNSUPPORTED.  Argument errors are reported before anything is
 * launched. */
int prefix_attn_backward(const prefix_attn_plan_t* plan, const void* q, const void* k_prefix,
                         const void* v_prefix, const void* k_suffix, const void* v_suffix,
                         const void* out, const void* d_out, const float* lse, void* dq,
                         void* dk_prefix, void* dv_prefix, void* dk_suffix, void* dv_suffix,
                         void* workspace, size_t workspace_bytes, void* hip_stream);

/* Measurement variant: same arguments and result, but the stages are bracketed by HIP events
 * and the call WAITS for them.  kernel_ms (HOST [4]) receives the durations in milliseconds of
 * {pre-pass (delta, layouts), dQ pass, dK/dV pass over the prefix keys, dK/dV pass over the
 * rollouts' own keys}; for fp32 plans entry 2 is the whole dK/dV kernel and entry 3 is ~0. */
int prefix_attn_backward_timed(const prefix_attn_plan_t* plan, const void* q, const void* k_prefix,
                               const void* v_prefix, const void* k_suffix, const void* v_suffix,
                               const void* out, const void* d_out, const float* lse,
                               void* dq, void* dk_prefix, void* dv_prefix, void* dk_suffix,
                               void* dv_suffix, void* workspace, size_t workspace_bytes,
                               void* hip_stream, float* kernel_ms);

/* ---- response-token log-probabilities and group advantages (paper Eq. 1 consumes the
 *      probabilities the policy / old policy / reference model give to the sampled response
 *      tokens; each device computes the logits of its token slice, Sec. 5.2; Eq. 2 normalises the
 *      rewards of a group) ---- */

/* For token n with final hidden state h_n, LM-head matrix W and sampled token id y_n:
 *     z_v = logit_scale * <w_v, h_n>,   LSE_n = ln sum_v exp(z_v),   logprob_n = z_{y_n} - LSE_n,
 * computed without materialising the [num_tokens, vocab] logits.
 *   hidden   [num_tokens, hidden_dim] bf16, DEVICE      (hidden_dim a multiple of 64, else
 *   lm_head  [vocab, hidden_dim]      bf16, DEVICE       PA_ERR_UNSUPPORTED)
 *   targets  [num_tokens] int32, DEVICE; an id outside [0, vocab) (an ignore index such as -100 on
 *            a padded slot) gives that token logprob = NaN, its lse is still computed
 *   logit_scale  1 / sampling temperature, finite and > 0
 *   logprob_out [num_tokens] fp32; lse_out [num_tokens] fp32 or NULL
 *   workspace of at least token_logprob_workspace bytes, DEVICE, 16-byte aligned
 * Enqueues two kernels on `hip_stream` on the current device; allocates nothing. */
int token_logprob_workspace(int64_t num_tokens, int32_t hidden_dim, int32_t vocab, size_t* workspace_bytes_out);
int token_logprob_forward(const void* hidden, const void* lm_head, const int32_t* targets,
                          int64_t num_tokens, int32_t hidden_dim, int32_t vocab, float logit_scale,
                          float* logprob_out, float* lse_out, void* workspace, size_t workspace_bytes,
                          void* hip_stream);

/* Eq. 2 for num_groups groups of group_size rewards each (DEVICE, fp32, group-major):
 * A_i = (r_i - mean) / std with the population standard deviation of the group; a group whose
 * rewards are all equal gets zeros. */
int grpo_group_advantages(const float* rewards, int32_t group_size, int32_t num_groups,
                          float* advantages_out, void* hip_stream);

/* Release a plan (NULL is allowed).  Work enqueued with the plan must have finished. */
void prefix_attn_destroy(prefix_attn_plan_t* plan);

/* Static, NUL-terminated description of a status code. */
const char* prefix_attn_status_string(int status);

/* ---- introspection of the schedule (host only; used by tests and the benchmark) ---- */

/* Tile geometry: stacked query rows per work item and keys per LDS tile.  A stacked
 * row index inside rollout g is m = i * (Hq/Hkv) + (h % (Hq/Hkv)). */
int prefix_attn_plan_tiles(const prefix_attn_plan_t* plan, int32_t* rows_per_item, int32_t* keys_per_tile);

/* Number of work items of a pass (0 = prefix pass, 1 = suffix pass, 2 = the backward's dQ pass,
 * 3 = the forward's single sweep, empty unless the plan uses it), padding items included. */
int64_t prefix_attn_plan_num_items(const prefix_attn_plan_t* plan, int32_t pass);

/* Copy the work list of a pass into items_out [num_items][6] (HOST) in launch order:
 * {rollout g (-1 = padding item), first stacked row inside the rollout, kv head c,
 *  nkeys, key0, pkeys}.
 * Prefix pass: the item sweeps prefix keys [key0, key0 + nkeys); that is the whole prefix
 * unless the call has so few rows that the prefix is cut into several key ranges per block
 * of rows (bf16 only): the ranges of a block are disjoint, cover the prefix, and their
 * partials are merged.  pkeys = 0.
 * Suffix pass: the item sweeps the rollout's own keys [0, nkeys); key0 = pkeys = 0.
 * dQ pass: the item sweeps prefix keys [key0, key0 + pkeys) and then the rollout's own keys
 * [0, nkeys); with key ranges exactly one item of a block has nkeys > 0; the list may hold
 * padding items.
 * Single sweep (whole bf16 calls whose prefix is at most 1,024 tiles and not cut into key
 * ranges run as one pass per block of rows instead of prefix pass + suffix pass): like the
 * dQ pass with key0 = 0 and pkeys = P, laid out over the XCDs like the prefix pass. */
int prefix_attn_plan_items(const prefix_attn_plan_t* plan, int32_t pass, int32_t* items_out);

/* Work lists of the backward dK/dV pass, padding entries included.  pass 0 = prefix key blocks, 1 = the
 * rollouts' own key blocks (masked kernel), 2 = the rollouts' own key blocks once more for the mask-free
 * kernel (empty unless the plan splits that pass: long rollouts, bf16).  items_out [num_items][6] (HOST):
 * {rollout g (-1 in passes 0 and 2), first key of the block (pass 0: prefix index; pass 1: position inside the
 *  rollout; pass 2: packed token index), kv head c (-1 = padding entry), number of keys in the block, and the
 *  range [tile0, tile1) of 64-row tiles of the kv head's stacked query rows that the item streams}.
 * Pass 0: a short prefix is split over several items per key block.  Passes 1 and 2 of a split plan: a block's
 * masked item streams the tiles that hold rows needing the causal mask (its diagonal) plus, via
 * prefix_attn_plan_key_item_extra_tiles, the rollout's last tile when rows of the next rollout share it; its
 * mask-free item streams the tiles between; together they cover every tile from the block's first key to the
 * rollout's end exactly once. */
int64_t prefix_attn_plan_num_key_items(const prefix_attn_plan_t* plan, int32_t pass);
int prefix_attn_plan_key_items(const prefix_attn_plan_t* plan, int32_t pass, int32_t* items_out);
/* tiles_out [num_items] (HOST): for pass 1 the one row tile an item streams after [tile0, tile1), or -1. */
int prefix_attn_plan_key_item_extra_tiles(const prefix_attn_plan_t* plan, int32_t pass, int32_t* tiles_out);

/* Total suffix tokens T of the plan. */
int64_t prefix_attn_plan_total_tokens(const prefix_attn_plan_t* plan);

#ifdef __cplusplus
}
#endif
#endif /* PREFIX_ATTN_H_ */
