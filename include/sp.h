/*
 * sp.h -- C ABI of the superposition-prompting hot path for AMD MI355X (gfx950).
 *
 * The library computes, on ONE GPU, the data-parallel core of superposition prompting:
 *   - ForkJoin prefill attention over a prompt DAG           (paper Sec. 3.2, 3.2.1, App. B.3)
 *   - Bayesian path saliency from language-model logits       (Sec. 3.2.3, App. B.1 Eq. 2)
 *   - greedy top-k path pruning                               (Sec. 3.2.3, Alg. 3)
 *   - decode attention over the joined (pruned) KV cache      (Sec. 3.2.3, Alg. 3)
 *   - equilibrium position assignment (host helper)           (Sec. 3.2.2 Eq. 1, App. B.2)
 *
 * Conventions
 *   Pointers are marked HOST or DEVICE.  The caller owns every tensor; the library owns only
 *   sp_ctx / sp_plan objects and their internal workspace, released by the matching destroy.
 *   Every entry point returns sp_status; arguments and tables are validated on the host before
 *   any kernel launch; nothing is printed; sp_last_error() returns the detail of the last
 *   failure on that context.  Kernels are enqueued on the context's HIP stream and the call
 *   returns without synchronising.  No floating-point atomics are used: equal inputs give
 *   bit-identical outputs.  Supported: head_dim 64 or 128; dtype fp32 or bf16 (storage of
 *   Q/K/V/O and logits; all arithmetic accumulates in fp32); n_q_heads a multiple of
 *   n_kv_heads (query head h reads KV head h / (n_q_heads / n_kv_heads)).
 *   Threads: a context (and the plans made on it) is used by one host thread at a time;
 *   different contexts are independent.  The launching calls only enqueue kernels (no memsets; the
 *   saliency workspace is allocated in sp_create for 65536 rows and 16384 path slots, and a call that
 *   needs more allocates a larger block once and keeps the old one until sp_destroy, so a captured graph
 *   never names freed memory), so they may be captured into a HIP graph on the context's stream.
 *   A plan keeps its context alive: sp_destroy may be called before sp_plan_destroy.
 */
#ifndef SP_H_
#define SP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sp_ctx sp_ctx;    /* device id + HIP stream + workspace                      */
typedef struct sp_plan sp_plan;  /* validated segment table, derived work lists, device copy */

typedef enum {
  SP_OK = 0,
  SP_ERR_INVALID_ARG = -1,  /* null pointer, non-positive size, bad enum                     */
  SP_ERR_BAD_TABLE = -2,    /* segment table / index table violates a structural rule        */
  SP_ERR_UNSUPPORTED = -3,  /* valid request outside the supported shapes                    */
  SP_ERR_WORKSPACE = -4,    /* internal workspace could not be (re)allocated                 */
  SP_ERR_HIP = -5           /* a HIP runtime call failed (no device, launch error, ...)      */
} sp_status;

typedef enum { SP_F32 = 0, SP_BF16 = 1 } sp_dtype;
typedef enum { SP_SALIENCY_SUM = 0, SP_SALIENCY_MEAN = 1 } sp_saliency_mode;

/*
 * Segment table: the prompt DAG of Sec. 3.2 for a batch of prompts.  Nodes are token
 * segments; seg_parent gives each node's single parent (ForkJoin and iterated ForkJoin are
 * trees up to the join, which sp_pruned_decode handles).  A token attends to every token of
 * its strict ancestor segments and to the tokens of its own segment up to and including
 * itself.  Tokens of all prompts are packed in one index space [0, n_tokens).
 * All pointers are HOST pointers; sp_plan_create copies what it needs.
 *
 * Structural rules (else SP_ERR_BAD_TABLE):
 *   prompt_seg_off is a CSR over segments: [0]=0, non-decreasing, every prompt non-empty,
 *   last = n_segments;  seg_tok_len > 0;  token ranges lie in [0, n_tokens) and do not
 *   overlap;  seg_parent is -1 or the id of an EARLIER segment of the SAME prompt;
 *   seg_path >= -1; a segment on path p >= 0 has a parent that is shared (-1) or on the same
 *   path; a shared segment has a shared parent or none; path ids of a prompt are dense
 *   (0..n_paths-1, each used); tok_pos finite when given; alibi_slopes finite and >= 0.
 */
typedef struct {
  int32_t n_prompts, n_segments, n_tokens;
  const int32_t *prompt_seg_off; /* [n_prompts+1]                                            */
  const int32_t *seg_tok_start;  /* [n_segments] first packed token index                    */
  const int32_t *seg_tok_len;    /* [n_segments]                                             */
  const int32_t *seg_parent;     /* [n_segments] global segment id, -1 = root                */
  const int32_t *seg_path;       /* [n_segments] path id within its prompt, -1 = shared      */
  const float *tok_pos;          /* [n_tokens] real-valued positions (Sec. 3.2.2); may be NULL
                                    when alibi_slopes is NULL                                */
  const float *alibi_slopes;     /* [n_q_heads] linear distance-penalty slopes; NULL = none  */
  const uint8_t *seg_cached;     /* [n_segments] nonzero: the segment's K/V come from a path cache
                                    (Sec. 3.3.1, Alg. 2): its tokens serve as keys only and no
                                    output rows are produced for them; NULL = nothing cached     */
} sp_segtable;

/* ---- context ------------------------------------------------------------------------- */

/* Create a context on `device`; hip_stream is a hipStream_t (NULL = the null stream).
 * SP_ERR_HIP when the device cannot be used. */
sp_status sp_create(sp_ctx **out, int device, void *hip_stream);
void sp_destroy(sp_ctx *ctx);
sp_status sp_set_stream(sp_ctx *ctx, void *hip_stream);
/* Detail of the last failure on ctx (ctx-owned, valid until the next call on ctx).
 * With ctx == NULL returns the detail of the last failure of a call that had no context. */
const char *sp_last_error(const sp_ctx *ctx);
const char *sp_version(void);

/* ---- plan (host work: validation, ancestor chains, tile work list; Sec. 3.2) ---------- */

/* Validate the table and derive the work lists.  With ctx == NULL the plan is host-only
 * (inspection calls work, launches return SP_ERR_INVALID_ARG); otherwise tables are uploaded
 * to ctx's device.  Layer-independent: reuse one plan for every layer of a model. */
sp_status sp_plan_create(sp_ctx *ctx, const sp_segtable *table, int32_t n_q_heads, int32_t n_kv_heads,
                         int32_t head_dim, sp_dtype dtype, sp_plan **out);
void sp_plan_destroy(sp_plan *plan);
/* Rebuild `plan` in place for another table (same head counts, head_dim and dtype): the prompt DAG
 * changes per request -- one table per query (Alg. 3), one per round of iterative superposition
 * (Sec. 4.1.2) -- while the plan object, and its device block when the new tables fit, stay.  On any
 * error the plan is unchanged.  Tables travel in one asynchronous copy from a pinned staging buffer
 * on the context's stream (also in sp_plan_create), ordered behind the work already enqueued there;
 * device blocks of destroyed plans are kept by the context and reused, so a steady request loop
 * calls neither hipMalloc nor hipFree.  Not for use while the stream is being captured.
 * Ordering: a plan's tables are replaced (update) or handed to the next plan (destroy, then create)
 * in the order of the context's stream, so launches that were enqueued on that stream before still
 * read the old tables.  Work enqueued with the plan on another stream (sp_set_stream in between)
 * must have finished before the plan is updated or destroyed. */
sp_status sp_plan_update(sp_plan *plan, const sp_segtable *table);

/* info[0]=n_prompts [1]=n_segments [2]=n_tokens [3]=n_path_slots [4]=n_row_groups (runs of
 * segments fused for the query side) [5]=n_tiles [6]=n_work_items [7]=max ancestor ranges.
 * HOST out pointer. */
sp_status sp_plan_info(const sp_plan *plan, int64_t info[8]);
/* Host inspection of the prefill work list as the kernel walks it.  Item i is 8 int32:
 * {first token of its row group, first row of the tile inside the group, rows in the tile, ancestor keys,
 * index of its first ancestor range, number of ancestor ranges, first query head | KV head << 16, first
 * token of ancestor range 0}; the rows see the ancestor ranges (sp_plan_key_ranges: pairs {first token,
 * length}, root to leaf) completely and the rows of their own group causally.  Worker slot s (a wave or a
 * workgroup, depending on the kernel the plan selected; sp_plan_work_slots of them) owns items
 * [slot_begin[s], slot_begin[s+1]).  Each call writes at most cap entries and returns the full count, or a
 * negative sp_status (slot_begin has sp_plan_work_slots() + 1 entries).  HOST pointers. */
int64_t sp_plan_work_items(const sp_plan *plan, int32_t *items_out, int64_t cap_items, int32_t *slot_begin_out,
                           int64_t cap_slots);
int64_t sp_plan_key_ranges(const sp_plan *plan, int32_t *ranges_out, int64_t cap);
int64_t sp_plan_work_slots(const sp_plan *plan);
/* Visible (query token, key token) pairs per head over the rows that are computed (tokens of
 * cached segments are keys only), the unit of the prefill FLOP count
 * 4 * head_dim * n_q_heads * pairs. */
int64_t sp_plan_visible_pairs(const sp_plan *plan);
/* HOST out [n_prompts+1]: CSR of global path slots (slot = path_off[prompt] + path id). */
sp_status sp_plan_path_offsets(const sp_plan *plan, int32_t *path_off_out);
/* DEVICE pointer to the same CSR (NULL for a host-only plan); valid while the plan lives. */
const int32_t *sp_plan_path_offsets_device(const sp_plan *plan);
/* Host inspection: the packed token indices visible to `token`, in the order the kernels
 * visit them (ancestors root-to-leaf, then own segment up to the token).  Writes at most
 * `cap` indices to HOST `out`, returns the full count, or a negative sp_status. */
int64_t sp_plan_visible_keys(const sp_plan *plan, int32_t token, int32_t *out, int64_t cap);
/* Host inspection: joined-cache token indices of `prompt` for the kept paths (shared
 * segments, then each kept path's segments in the given order), as sp_pruned_decode
 * gathers them.  Same return convention as sp_plan_visible_keys. */
int64_t sp_plan_joined_keys(const sp_plan *plan, int32_t prompt, const int32_t *kept, int32_t k,
                            int32_t *out, int64_t cap);

/* ---- a1: ForkJoin prefill attention (Sec. 3.2.1, App. B.3 batched model call) ---------- */
/*
 * For every token t covered by the table and every query head h:
 *   O[t,h,:] = sum_s softmax_s( scale * <Q[t,h,:], K[s,g(h),:]> - slope_h * (pos[t]-pos[s]) ) V[s,g(h),:]
 * over the tokens s visible to t.  One launch covers all prompts, paths and heads.
 * Q, O: DEVICE [n_tokens, n_q_heads, head_dim]; K, V: DEVICE [n_tokens, n_kv_heads, head_dim];
 * element strides given explicitly (innermost stride 1); dtype as in the plan; O must not
 * alias an input; rows of tokens not covered by any segment, and rows of segments flagged
 * seg_cached, are left untouched.
 * Layout limits (SP_ERR_UNSUPPORTED / SP_ERR_INVALID_ARG otherwise): base pointers 16-byte
 * aligned; strides multiples of 16 bytes (8 bf16 or 4 fp32 elements); all strides >= head_dim;
 * Q and O token-major (token stride >= head stride); K and V token-major or head-major (a KV
 * cache stored per head: head stride >= n_tokens * token stride), head stride below 2^31
 * elements; token strides below 2^26 elements; softmax_scale positive and finite.
 */
sp_status sp_forkjoin_prefill(sp_ctx *ctx, const sp_plan *plan, const void *Q, const void *K, const void *V,
                              void *O, int64_t q_tok_stride, int64_t q_head_stride, int64_t kv_tok_stride,
                              int64_t kv_head_stride, float softmax_scale);

/* ---- a2: path saliency (Sec. 3.2.3; App. B.1 Eq. 2) ------------------------------------ */
/*
 * lp[r] = logits[r, target[r]] - logsumexp_v logits[r, v]          (rows with target < 0 are skipped)
 * score[i] = sum (SUM) or mean (MEAN) of lp over scored rows with row_path == i, + prior[i].
 * logits: DEVICE [n_rows, vocab], row_stride in elements, dtype fp32 or bf16; target, row_path:
 * DEVICE int32 [n_rows]; prior: DEVICE fp32 [n_path_slots] or NULL; score: DEVICE fp32
 * [n_path_slots], fully overwritten (a slot without scored rows gets 0 + prior).
 * Contract: 0 <= target[r] < vocab or target[r] < 0; 0 <= row_path[r] < n_path_slots.  The
 * kernels clamp out-of-contract ids instead of faulting; results for such rows are undefined.
 */
sp_status sp_path_saliency(sp_ctx *ctx, const void *logits, sp_dtype dtype, int64_t n_rows, int64_t vocab,
                           int64_t row_stride, const int32_t *target, const int32_t *row_path,
                           const float *prior, int32_t n_path_slots, sp_saliency_mode mode, float *score);
/*
 * sp_path_saliency for callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): same arguments, same result, but the scratch
 * memory of the kernels (one log-likelihood per row, the per-path accumulators) is a static device array
 * of the library, 1.25 MiB per GPU, held until the process ends, instead of the context's workspace, and
 * the call makes no hipMalloc / hipFree.  Limits: n_rows <= 65536 and n_path_slots <= 16384, else
 * SP_ERR_UNSUPPORTED.  The array is shared by every call on that GPU: calls that overlap in time on one
 * GPU (different streams or contexts) race; calls on one stream are safe.  Each launch leaves the
 * accumulators it used at zero, the state the next one expects.
 */
sp_status sp_path_saliency_static(sp_ctx *ctx, const void *logits, sp_dtype dtype, int64_t n_rows, int64_t vocab,
                                  int64_t row_stride, const int32_t *target, const int32_t *row_path,
                                  const float *prior, int32_t n_path_slots, sp_saliency_mode mode, float *score);

/* ---- a3: top-k pruning (Sec. 3.2.3; Alg. 3) -------------------------------------------- */
/*
 * Per prompt b, the k local path indices with the largest score, in descending score order,
 * ties to the lower index (NaN ranks last).  score: DEVICE fp32; path_off: DEVICE int32
 * [n_prompts+1] CSR into score; kept: DEVICE int32 [n_prompts, k].  If a prompt has fewer than
 * k paths the remaining entries are -1.  n_paths_max (HOST value) sizes the launch's LDS copy of a
 * prompt's scores (SP_ERR_UNSUPPORTED above 4096); a prompt with more paths than that is still ranked
 * completely, from global memory, only slower.
 */
sp_status sp_prune_topk(sp_ctx *ctx, const float *score, const int32_t *path_off, int32_t n_prompts,
                        int32_t n_paths_max, int32_t k, int32_t *kept);

/* ---- a4: decode attention over the joined cache (Sec. 3.2.3; Alg. 3 generation loop) --- */
/*
 * One decode step for all prompts of the plan.  For prompt b the key/value set is
 *   shared segments (+) segments of path kept[b,0] (+) ... (+) kept[b,k-1]   (gathered from the
 *   packed prefill cache through the plan's tables, never copied)
 *   (+) response cache rows [0, len_b) (+) the new token,    len_b = resp_len[b] + resp_len_add.
 * The call first stores k_new/v_new (and new_pos) at row len_b of the response cache, then
 * attends.  kept entries < 0 are ignored.  The caller advances resp_len (or resp_len_add).
 * K_prefill, V_prefill: DEVICE, layout/strides as in sp_forkjoin_prefill (kv strides).
 * K_resp, V_resp: DEVICE [n_prompts, resp_capacity, n_kv_heads, head_dim] contiguous;
 * pos_resp: DEVICE fp32 [n_prompts, resp_capacity] or NULL (required with slopes);
 * resp_len: DEVICE int32 [n_prompts] or NULL (= zeros); new_pos: DEVICE fp32 [n_prompts] or NULL;
 * q_new, o_out: DEVICE [n_prompts, n_q_heads, head_dim]; k_new, v_new: DEVICE [n_prompts,
 * n_kv_heads, head_dim].  Contract: len_b < resp_capacity (rows beyond are dropped, not written).
 */
sp_status sp_pruned_decode(sp_ctx *ctx, const sp_plan *plan, const int32_t *kept, int32_t k,
                           const void *K_prefill, const void *V_prefill, int64_t kv_tok_stride,
                           int64_t kv_head_stride, void *K_resp, void *V_resp, float *pos_resp,
                           int32_t resp_capacity, const int32_t *resp_len, int32_t resp_len_add,
                           const float *new_pos, const void *q_new, const void *k_new, const void *v_new,
                           void *o_out, float softmax_scale);

/* ---- host helper: equilibrium positions (Sec. 3.2.2 Eq. 1; App. B.2 Eq. 3, Alg. 1) ----- */
/*
 * Fills HOST tok_pos_out[n_tokens] for a ForkJoin-shaped table: root segments at 0,1,2,...;
 * the children of a node that fork into paths ("documents") are spaced by S/len_i from the
 * parent's end, S the harmonic mean of the sibling lengths, so all siblings span the same
 * interval; a single child continues from where its parent's span ends with step 1
 * (the shared query positions of Alg. 3).  HOST pointers only; no device needed.
 */
sp_status sp_equilibrium_positions(const sp_segtable *table, float *tok_pos_out);

#ifdef __cplusplus
}
#endif
#endif /* SP_H_ */
