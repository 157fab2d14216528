/*
 * sparsevila.h -- C ABI of the MI355X (gfx950) sparse decode library.
 *
 * One decode step of SparseVILA's decode stage (paper section 3.2, "Decode
 * Phase: Query-Aware Retrieval"): the visual part of the KV cache stays
 * resident in full; for the current query the library
 *   (1) scores every cached visual key         -> sv_score_visual
 *   (2) keeps the k highest-scoring tokens     -> sv_topk_select
 *   (3) attends over all text tokens plus the
 *       kept visual tokens                     -> sv_sparse_decode_attn
 * and sv_decode_step chains the three.  The paper retrieves once per
 * conversation round and then decodes many tokens; that use is
 * sv_score_visual + sv_topk_select once, then sv_sparse_decode_attn per token
 * with the same idx.  Retrieving at every step is sv_decode_step.
 *
 * Conventions that hold for every entry point
 * -------------------------------------------
 * Pointers.  The sv_shape struct itself is HOST memory.  Every other pointer
 *   (q, k_*, v_*, scores, idx, count, out, lse, workspace, and the vis_len /
 *   txt_len pointers stored inside sv_shape) is DEVICE memory owned by the
 *   caller.  The library never allocates, frees or keeps a pointer after the
 *   call returns; q/K/V/vis_len/txt_len are only read.
 * Layout.  head_dim is contiguous everywhere.  q is [B, Hq, D] addressed with
 *   q_stride_b/q_stride_h; visual K and V share one set of strides
 *   [B, Hkv, n_vis_max, D] (kv_vis_stride_*), text K and V another
 *   (kv_txt_stride_*).  Strides are in ELEMENTS.  Outputs are dense:
 *   scores [B, Hkv, n_vis_max] float, idx [B, Hkv, k] int32, count [B, Hkv]
 *   int32, out [B, Hq, D] float, lse [B, Hq] float.
 * Alignment.  Every K/V/q base pointer and every row (stride * element size)
 *   must be a multiple of 16 bytes: rows are read with 128-bit loads.
 * Groups.  Query head h reads kv head h / (Hq / Hkv).
 * Ragged batches.  vis_len[b] <= n_vis_max and txt_len[b] <= n_txt_max give the
 *   live rows of sequence b; NULL means "all rows".  Rows past the length never
 *   influence a result and may hold anything (uninitialised memory, NaN bit
 *   patterns); a kernel may still fetch them, so the whole capacity must be
 *   mapped device memory.
 * Streams.  `stream` is a hipStream_t passed as void* (NULL = the default
 *   stream).  All work is enqueued asynchronously; nothing synchronises the
 *   host.  Results are valid once the caller has synchronised the stream.
 *   Calls that share a workspace must be ordered on one stream (or by the
 *   caller's events).  Since nothing allocates or synchronises, a call may be
 *   captured into a HIP graph once the same entry point has run uncaptured on
 *   that device (one-time host set-up happens on first use); replays see the
 *   tensors' current contents.
 * Errors.  The return value is an sv_status; SV_OK is 0, errors are negative.
 *   Arguments are checked on the host before anything is launched, so a failed
 *   call has launched nothing.  A launch failure reported by the HIP runtime
 *   maps to SV_ERR_LAUNCH.  Nothing is printed and nothing is thrown.
 * Determinism.  Equal inputs give bit-identical scores, idx, count, out, lse.
 * Inputs are assumed finite; behaviour on NaN is unspecified.
 */
#ifndef SPARSEVILA_H
#define SPARSEVILA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SV_OK = 0,
    SV_ERR_NULL = -1,      /* a required pointer is NULL                          */
    SV_ERR_SHAPE = -2,     /* sizes/strides out of range or inconsistent          */
    SV_ERR_DTYPE = -3,     /* dtype is neither SV_F16 nor SV_F32                  */
    SV_ERR_ALIGN = -4,     /* a base pointer or row stride is not 16-byte aligned */
    SV_ERR_WORKSPACE = -5, /* workspace missing, misaligned or too small          */
    SV_ERR_LAUNCH = -6     /* the HIP runtime rejected a launch                   */
} sv_status;

typedef enum { SV_F16 = 0, SV_F32 = 1 } sv_dtype;

typedef struct sv_shape {
    int32_t batch;       /* B >= 1; independent layers may be folded in here        */
    int32_t n_q_heads;   /* Hq, a multiple of n_kv_heads                             */
    int32_t n_kv_heads;  /* Hkv >= 1                                                 */
    int32_t head_dim;    /* D: 64 or 128                                             */
    int32_t n_vis_max;   /* rows of the visual segment per (b, kv head), >= 0        */
    int32_t n_txt_max;   /* rows of the text segment per (b, kv head), >= 0          */
    int32_t k;           /* visual tokens to keep, >= 0; k_b = min(k, vis_len[b])    */
    int32_t dtype;       /* sv_dtype of q, K and V                                   */
    float scale;         /* softmax / score scale; 0 selects 1/sqrt(D)               */
    int32_t reserved;    /* must be 0                                                */
    const int32_t *vis_len; /* DEVICE [B] or NULL                                    */
    const int32_t *txt_len; /* DEVICE [B] or NULL                                    */
    int64_t q_stride_b, q_stride_h;
    int64_t kv_vis_stride_b, kv_vis_stride_h, kv_vis_stride_n;
    int64_t kv_txt_stride_b, kv_txt_stride_h, kv_txt_stride_n;
} sv_shape;

/* Fills the eight stride fields for dense row-major tensors of this shape. */
void sv_shape_set_contiguous(sv_shape *shape);

/*
 * Bytes of device workspace that sv_topk_select, sv_sparse_decode_attn and
 * sv_decode_step need for this shape (the maximum over the three; it covers the
 * split partial results of step 3 and, for sv_decode_step called without a
 * scores buffer, the scores).  Returns 0 for an invalid shape.  The workspace
 * must be 256-byte aligned; its contents need not be preserved between calls.
 */
size_t sv_workspace_bytes(const sv_shape *shape);

/*
 * Bytes sv_topk_select alone needs (never more than sv_workspace_bytes): 0 for rows of up to 16384
 * scores and for an invalid shape.  A function of batch, n_kv_heads, n_vis_max and k only.
 */
size_t sv_select_workspace_bytes(const sv_shape *shape);

/*
 * Step 1 -- query-aware relevance (section 3.2, "Query-Aware Token Selection":
 * the aggregate attention strength between the query and each visual entry of
 * the KV cache).  The paper gives no formula; the aggregate used here is the
 * sum, over the query heads of the key's GQA group, of the scaled logit:
 *   scores[b,g,j] = sum_{h in group g} scale * <q[b,h,:], k_vis[b,g,j,:]>,
 * accumulated in fp32, for j < vis_len[b]; -inf for vis_len[b] <= j < n_vis_max.
 * k and the text fields of the shape are ignored.
 */
sv_status sv_score_visual(const sv_shape *shape, const void *q, const void *k_vis,
                          float *scores, void *stream);

/*
 * Step 2 -- retention (section 3.2: the tokens with the highest relevance are
 * kept for decoding, the rest stay cached but inactive).  For every (b, g):
 * idx[b,g,0..count) = the k_b = min(k, vis_len[b]) indices j < vis_len[b] with
 * the largest scores[b,g,j]; equal scores are resolved toward the lower index
 * (+0 and -0 are equal); indices ascend; idx[b,g,count..k) = -1;
 * count[b,g] = k_b.  Only batch, n_kv_heads, n_vis_max, vis_len and k of the
 * shape are used (the other fields must still describe a valid shape).
 * Integer-exact: the result is the unique set defined above for the given
 * float scores.  k == 0 is valid (nothing is written to idx).  Rows of up to
 * 16384 scores need no workspace (workspace may be NULL for such shapes); longer
 * rows need sv_select_workspace_bytes(shape) bytes, 256-byte aligned.
 */
sv_status sv_topk_select(const sv_shape *shape, const float *scores,
                         int32_t *idx, int32_t *count,
                         void *workspace, size_t workspace_bytes, void *stream);

/*
 * Step 3 -- sparse decode attention (section 3.2, first paragraph: only the
 * most query-relevant visual tokens take part in decoding attention; section
 * 4.5, "Decoding Attention Kernel Efficiency": the step is bound by KV-cache
 * traffic, which shrinks with the kept set).  For every query head h with kv
 * head g: one softmax over T = text tokens i < txt_len[b] followed by visual
 * tokens idx[b,g,0..count[b,g]), logits scale * <q[b,h,:], key>,
 *   out[b,h,:] = sum_t softmax_t * value_t      lse[b,h] = log sum_t exp(logit_t).
 * The caller appends the current token's own K/V to the text segment before the
 * call; there is no mask and no rotary embedding inside.  idx entries must lie
 * in [0, vis_len[b]); count[b,g] <= k.  With k == 0, idx and count may be NULL
 * (text-only attention).  With k > 0 and idx == NULL the visual segment is taken as
 * PACKED: its rows 0..count[b,g) are the kept tokens (see sv_pack_selected; pass the
 * packed buffers as k_vis/v_vis with n_vis_max = k).  A (b,g) with no token at all yields out = 0 and
 * lse = -inf.  lse may be NULL.  Accumulation is fp32; T is processed in
 * chunks whose partial results are merged by a second pass.
 */
sv_status sv_sparse_decode_attn(const sv_shape *shape, const void *q,
                                const void *k_vis, const void *v_vis,
                                const void *k_txt, const void *v_txt,
                                const int32_t *idx, const int32_t *count,
                                float *out, float *lse,
                                void *workspace, size_t workspace_bytes, void *stream);

/*
 * Step 1 as the paper runs it, once per conversation round, with the whole question as the
 * query (section 3.2, "Query-Aware Token Selection": the aggregate attention strength
 * between the query embeddings and the visual entries of the KV cache; section 3.1,
 * "Efficient Implementation": softmax normalisation and salience accumulation are streamed,
 * the attention matrix is never formed).  q_multi holds the n_query_tokens tokens of the
 * question, [B, Tq, Hq, D] fp16 addressed with q_stride_b, q_stride_t (ELEMENTS, a multiple
 * of 8) and q_stride_h.  The question's tokens are the LAST Tq rows of the text segment
 * (query token i is text row txt_len[b] - Tq + i); row (i, h) attends, as in the model, to
 * the text rows up to and including its own and to every visual row j < vis_len[b], with one
 * softmax over all of them, logits scale * <q, key>.  Then
 *   scores[b,g,j] = sum_{i < Tq} sum_{h in group g} softmax_(i,h)[j]     (attention mass),
 * -inf for vis_len[b] <= j < n_vis_max, and lse[b,i,h] (optional output, [B, Tq, Hq]) is the
 * log of the row's normaliser.  The scores feed sv_topk_select unchanged.  fp16 only
 * (SV_ERR_DTYPE otherwise); head_dim may also be 96 here (dims 72 or 80 zero-padded, the
 * caller's own scale); Tq * (Hq / Hkv) <= 256 (SV_ERR_SHAPE otherwise; the mass is
 * additive over groups of query tokens).  k is ignored.  The workspace must hold
 * sv_mass_workspace_bytes(shape, Tq) bytes.
 * For the sum-of-logits aggregate of a multi-token query no separate call is needed: the sum
 * is linear, so sv_score_visual on a shape whose query heads are the Tq * Hq rows (grouped
 * per kv head) gives it.
 */
size_t sv_mass_workspace_bytes(const sv_shape *shape, int32_t n_query_tokens);
sv_status sv_score_visual_mass(const sv_shape *shape, const void *q_multi, int32_t n_query_tokens,
                               int64_t q_stride_t, const void *k_vis, const void *k_txt,
                               float *scores, float *lse,
                               void *workspace, size_t workspace_bytes, void *stream);

/*
 * Query-agnostic salience of the tokens of one vision-encoder layer (section 3.1, "Token
 * Salience Estimation": for encoders without a summary token, importance is the intra-visual
 * attention averaged over all tokens; "Efficient Implementation": normalisation and
 * accumulation are streamed, the N x N attention matrix is never formed).  The prefill-side
 * pruning keeps the tokens of highest salience: the output feeds sv_topk_select (on a shape
 * with one kv head) unchanged.
 *   salience[b, j] = 1 / (H n_b) * sum_h sum_{i < n_b} softmax_(i,h)[j],     n_b = vis_len[b],
 * where row (i, h) is the query of token i, head h, and its softmax runs over the keys of the
 * n_b live tokens of the same head with logits scale * <q, key>; no mask.  The salience of the
 * live tokens of a batch entry sums to 1; -inf for n_b <= j < n_vis_max.
 * Fields of the shape that are used: batch (images, frames or windows: attention stays inside a
 * batch entry), n_q_heads = n_kv_heads = H (SV_ERR_SHAPE otherwise), head_dim 64, 96 or 128
 * (an encoder with 72 or 80 dims per head zero-pads q and k to 96 and passes its own scale),
 * n_vis_max = N (token capacity), vis_len, scale, dtype (fp16 only, SV_ERR_DTYPE otherwise),
 * q_stride_b / q_stride_h and the kv_vis strides; the text fields and k are ignored.
 *   q_all  [B, N, H, D] addressed with q_stride_b, q_stride_t (ELEMENTS, a multiple of 8), q_stride_h
 *   k_all  [B, H, N, D] addressed with kv_vis_stride_b, kv_vis_stride_h, kv_vis_stride_n
 *          (both accept the token-major layout of a fused qkv projection through the strides)
 *   salience [B, N] fp32 (output);  lse [B, N, H] fp32 or NULL (optional output: log of every
 *          row's normaliser, +inf past vis_len)
 * The workspace must hold sv_salience_workspace_bytes(shape) bytes (0 for an invalid shape).
 * Deterministic: the same inputs give the same bits.
 * Encoders WITH summary tokens (the same paragraph: attention directed toward one or a few summary
 * rows) need no call of their own: sv_score_visual_mass with those rows as q_multi and
 * n_txt_max = 0 gives the attention each patch token receives from them.
 */
size_t sv_salience_workspace_bytes(const sv_shape *shape);
sv_status sv_salience_self(const sv_shape *shape, const void *q_all, int64_t q_stride_t,
                           const void *k_all, float *salience, float *lse,
                           void *workspace, size_t workspace_bytes, void *stream);

/*
 * Packing (section 3.2: the selected visual KV entries are packed into a contiguous
 * region, so that the attention of the tokens decoded afterwards reads no irregular
 * pattern).  k_pack/v_pack are dense DEVICE buffers [B, Hkv, k, D] of the shape's dtype:
 *   k_pack[b,g,i,:] = k_vis[b,g,idx[b,g,i],:],  v_pack likewise,  for i < count[b,g];
 * rows count[b,g] <= i < k are zero-filled.  A byte-exact copy.  The paper's use, one
 * retrieval per conversation round: sv_score_visual + sv_topk_select + sv_pack_selected
 * once, then per decoded token sv_sparse_decode_attn on the packed buffers (shape with
 * n_vis_max = k and contiguous visual strides, idx = NULL, the same count).
 * Only the visual fields, k and dtype of the shape are used; k == 0 does nothing.
 */
sv_status sv_pack_selected(const sv_shape *shape, const void *k_vis, const void *v_vis,
                           const int32_t *idx, const int32_t *count,
                           void *k_pack, void *v_pack, void *stream);

/*
 * Steps 1 -> 2 -> 3 on one stream.  scores may be NULL (the workspace then
 * holds them); idx and count are outputs and are required when k > 0; with k == 0
 * count, if given, is set to 0, no key is scored and `scores` is left untouched
 * (text-only attention needs no retrieval).
 */
sv_status sv_decode_step(const sv_shape *shape, const void *q,
                         const void *k_vis, const void *v_vis,
                         const void *k_txt, const void *v_txt,
                         float *scores, int32_t *idx, int32_t *count,
                         float *out, float *lse,
                         void *workspace, size_t workspace_bytes, void *stream);

/*
 * sv_decode_step for callers that cannot allocate device memory and have no workspace to hand over:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * same results (bit for bit) as sv_decode_step, without `workspace`: the step's scratch (scores when
 * the caller passes none, split partial results, candidate records) lives in one array of
 * SV_STATIC_SCRATCH_BYTES inside the library's code object, one copy per GPU, held from the moment the
 * library is loaded on that GPU until the process ends.  The call allocates and frees nothing and
 * calls no allocating routine; the first call on a device looks the array's address up once.
 * A shape with sv_workspace_bytes(shape) > SV_STATIC_SCRATCH_BYTES is rejected with SV_ERR_WORKSPACE
 * before anything is launched (32 MiB covers up to eight decoder layers of a 50 176-token video folded
 * into the batch, all 28 layers of a 12 544-token video, or a batch of 16 sequences of 8 192 visual
 * tokens; beyond that fold fewer layers per call, or use sv_decode_step with a workspace of your own).
 * All calls on one GPU share that GPU's array: calls whose execution may overlap on one GPU (different
 * streams without an ordering, several host threads) race on it and must be ordered by the caller.
 * The array keeps what the last call left; nothing in it has to start at zero.  The device that is
 * current when the call is made must be the device of `stream` and of every pointer.
 */
#define SV_STATIC_SCRATCH_BYTES (32u << 20)
sv_status sv_decode_step_static(const sv_shape *shape, const void *q,
                                const void *k_vis, const void *v_vis,
                                const void *k_txt, const void *v_txt,
                                float *scores, int32_t *idx, int32_t *count,
                                float *out, float *lse, void *stream);

/*
 * Measurement aid, not part of the decode path: copies `bytes` (a multiple of 16; both
 * DEVICE pointers 16-byte aligned, non-overlapping) with a plain kernel.  Hardware
 * traffic counters are calibrated against the known size of this copy.
 */
sv_status sv_copy_bytes(void *dst, const void *src, size_t bytes, void *stream);

/*
 * Measurement aid, not part of the decode path: reads `bytes` (a multiple of 16) from the 16-byte
 * aligned DEVICE pointer `src` once, as a plain stream of 128-bit loads, and folds what it read into
 * `sink` (DEVICE, 16-byte aligned, SV_READ_SINK_BYTES bytes, caller-owned; its content afterwards is
 * unspecified, it only keeps the loads alive).  Its rate is what a kernel that has to read every byte once can reach on the device.
 */
#define SV_READ_SINK_BYTES 4096
sv_status sv_read_bytes(const void *src, size_t bytes, uint32_t *sink, void *stream);

/* Static, human-readable name of a status code; takes an int so that any value may be asked about
 * ("unknown status" for one that is no sv_status). */
const char *sv_strerror(int status);

/*
 * Launch-shape knobs for measurement sweeps (not needed for correct use):
 *   "score_rows_per_block"  rows of visual K one scoring workgroup covers, 64..65536, 0 = default
 *   "attn_chunk"            tokens per attention workgroup, multiple of 64 in 64..1024, 0 = default
 *   "score_stream_loads"    1 = non-temporal loads of visual K, 0 = plain loads, -1 = default
 *   "attn_mfma"             fp16 caches: 1 = logits on the matrix cores, 0 = vector FMA, -1 = default
 *   "attn_batches"          fp16 caches with head_dim 128 on the matrix cores: 32-token batches each wavefront
 *                           walks through (a workgroup covers 128 times as many tokens), 1..8; 0 = chosen per
 *                           call from the shape so that the workgroups fill the chip in whole rounds
 *   "select_filter"         sv_decode_step on long rows: 1 = the scoring kernel hands the selection only the
 *                           scores above a sampled threshold, 0 = the selection re-reads every score, -1 = default
 *   "filter_rank"           which order statistic of the sampled rows is that threshold, 1..448; 0 = derived
 *                           from k / vis_len.  Any value gives the same result (a threshold that admits too
 *                           few or too many candidates makes the row fall back to the full selection)
 *   "filter_samples"        rows of that sample: 256 or 512; 0 = by the size of the scoring launch (a launch of
 *                           few tiles waits for its samplers and takes 256).  Any value gives the same result
 *   "filter_spread"         1 (default) = a sample of 256 rows is dealt over four sampler workgroups that score it in one
 *                           round of loads; 0 = one sampler workgroup per (b, g) scores it in rounds.  Same result
 * Unknown names and values outside a knob's range are rejected with SV_ERR_SHAPE and change nothing.
 * Process-wide.  Every knob is one atomic word and a call reads each knob once, when it starts: setting
 * a knob while calls are in flight on other threads is safe and affects calls that start later.
 * No knob can leave an output unwritten or change what is computed.  scores, idx and count never depend on
 * the knobs; out and lse depend on them only through fp32 summation order in step 3 and, for
 * "attn_mfma", through the rounding of the softmax weights to fp16 on the matrix-core path.
 */
sv_status sv_set_tuning(const char *name, int32_t value);
int32_t sv_get_tuning(const char *name);   /* -1 for an unknown name */

/*
 * 0 in libsparsevila.so.  The repository's tests and benchmark also build the same sources with
 * -DSV_TEST_HOOKS into libsparsevila_hooks.so (identical kernels), where this returns 1 and
 * sv_set_tuning knows two more names that a product build must not have:
 *   "filter_test_mode"  1 / 2 make every third tile of the scoring kernel ignore the sampled threshold and
 *                       hand over none / all of its scores (tests of the selection's consistency check)
 *   "step_stages"       sv_decode_step returns after its first 1 (scoring launch) or 2 (scoring and
 *                       selection) stages, later outputs unwritten (timing of a stage as the step issues it)
 */
int32_t sv_has_test_hooks(void);

#ifdef __cplusplus
}
#endif
#endif /* SPARSEVILA_H */
