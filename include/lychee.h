/*
 * lychee.h — C ABI of the MI355X (gfx950) decode-step hybrid-head sparse attention.
 *
 * One decode step of LycheeDecode's attention (Sec. 3.1; Alg. 1, the per-head loop of
 * App. B): in every layer the few *retrieval heads* attend over the whole KV cache
 * (Eq. 1) and pick the k highest-scoring positions (Eq. 2); the *sparse heads* attend
 * only over the k rows named by the set inherited from the previous layer (Eq. 3) and
 * hand that set on unchanged.  Under grouped-query attention there is one set per KV
 * head, ranked by the mean logit of the group's retrieval heads (App. F).  Head types
 * are an input (the trained HardKuma assignment of Sec. 3.2, thresholded).
 *
 * Conventions shared by every call
 *   - Pointers are DEVICE pointers unless a parameter says HOST.  The caller owns every
 *     buffer; the library neither frees nor keeps them after the call's stream-ordered
 *     work has finished.  Nothing is allocated inside a call (a context allocates, once, in
 *     lychee_create: a 4 MiB device arena with its pinned mirror, and about 0.6 MiB of flags and
 *     counters through which the workgroups of a layer launch hand results to one another).
 *   - Calls only enqueue work on `hip_stream` (a hipStream_t; NULL = the default stream) and
 *     never read device memory from the host.  The layer calls (lychee_decode_attn,
 *     lychee_decode_attn_static, lychee_decode_attn_deferred, lychee_select_flush,
 *     lychee_dense_decode_attn) and the layer-after-layer steps enqueue kernel launches only,
 *     one per layer, and never wait.  The phased steps and the cache append keep their layer
 *     descriptors in the arena: they enqueue one small asynchronous host-to-device copy when the
 *     call's pointers differ from those of earlier calls, and once the arena has seen about
 *     4 MiB of distinct tables such a call waits for the stream once and starts the arena over
 *     - unless a stream capture has seen the arena: a captured graph keeps pointing into it, so
 *     its tables are never recycled and the call returns LYCHEE_EARENA instead.
 *   - bf16 means the upper 16 bits of an IEEE fp32.  Scores and accumulation are fp32;
 *     `out` is rounded to nearest-even bf16.
 *   - KV-cache element (b, g, t, i), g a KV head, t a position, i < 128, lives at
 *         base + b*kv_stride_batch + g*kv_stride_head + t*kv_stride_tok + i   (elements).
 *     K and V use the same strides.  The preferred layout is [B][H_kv][L_cap][128] with
 *     256-byte aligned rows: each (b, g) is then one contiguous stream of 256-byte rows
 *     (two 128-byte lines), which is what the streaming kernel is tuned for.
 *   - Index sets are int32 [B][H_kv][k]: positions in [0, L_b), distinct, valid entries
 *     first, -1 padding after (when k > L_b).  Sets written by the library are ascending
 *     by position; ties in the score go to the lower position.  Entries of `idx_in` that
 *     are negative or >= L_b are ignored (never dereferenced).
 *   - Return value: 0, or a negative LYCHEE_E* code; on an error nothing was enqueued.
 *   - Results are deterministic: the same inputs give bit-identical outputs.
 *   - Two calls that share a workspace must be ordered on one stream.
 */
#ifndef LYCHEE_H
#define LYCHEE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LYCHEE_OK            0
#define LYCHEE_EINVAL       (-1)  /* a NULL / misaligned pointer or an inconsistent value       */
#define LYCHEE_EUNSUPPORTED (-2)  /* a valid request this build does not serve                 */
#define LYCHEE_EWORKSPACE   (-3)  /* workspace NULL, misaligned or smaller than required       */
#define LYCHEE_EHIP         (-4)  /* a HIP runtime call failed (no device, launch error, ...)  */
#define LYCHEE_EARENA       (-5)  /* the context's descriptor arena is full and cannot be recycled
                                     because a captured graph uses it: create another context   */

#define LYCHEE_HEAD_DIM      128  /* the only head dimension served                            */
#define LYCHEE_MAX_KV_HEADS   64
#define LYCHEE_MAX_GROUP       4  /* query heads per KV head served (1..4)                     */
#define LYCHEE_MAX_BATCH     256

typedef struct lychee_ctx lychee_ctx; /* opaque; holds the device id, tuning, a small device
                                         arena for descriptor tables and the hand-off flags of
                                         the layer launches; use one context per stream, and do
                                         not let two calls on one context overlap.  The attention
                                         calls only enqueue kernels (and at most one
                                         host-to-device copy of a descriptor table from the
                                         context's pinned memory), so a stream that is being
                                         captured into a HIP graph can take them, and the graph can be
                                         replayed while the context lives and timing is off. */

/* Problem shape of one layer call (the inputs of Alg. 1 that are not tensors). */
typedef struct lychee_shape {
    int32_t batch;       /* B in [1, LYCHEE_MAX_BATCH]                                       */
    int32_t n_q_heads;   /* H_q, a multiple of n_kv_heads with H_q / H_kv <= LYCHEE_MAX_GROUP */
    int32_t n_kv_heads;  /* H_kv in [1, LYCHEE_MAX_KV_HEADS]                                 */
    int32_t head_dim;    /* must be LYCHEE_HEAD_DIM                                          */
    int32_t max_len;     /* host-known upper bound of lengths[]; sizes grids and workspace,
                            so that no call has to read lengths[] on the host              */
    int32_t k;           /* token budget of Eq. 2 / Eq. 3, >= 1; the capacity of every set      */
    int64_t kv_stride_batch, kv_stride_head, kv_stride_tok; /* elements; each a multiple of 8
                            (16-byte vector loads), kv_stride_tok >= 128                    */
    int32_t keep_ppm;    /* 0: Eq. 2 selects min(k, L_b) positions.  1 .. 1000000: the Ratio rule
                            of Sec. 4.4.1, a budget proportional to the sequence length:
                            min(k, ceil(L_b * keep_ppm / 10^6)) positions, at least 1.  (The
                            paper's theta is the share of tokens dropped, App. E.2: theta = 70 %
                            is keep_ppm = 300000.)  Sparse heads attend over whatever valid
                            entries the inherited set holds, under either rule.               */
    int32_t block_size;  /* 0 or 1: sets name positions (Sec. 3.1).  64: the block-granular variant of
                            App. C / Sec. 4.3.2: a set entry e names the positions [64e, 64e+63]
                            below L_b, a block is ranked by the best pooled score inside it, and k,
                            idx_in / idx_out and the Ratio rule all count blocks.               */
    int32_t prob_rule;   /* 0: none.  LYCHEE_RULE_THRESHOLD (1), LYCHEE_RULE_TOP_P (2): the rules of
                            Sec. 4.4.1 on attention probabilities, here the softmax over the whole
                            sequence of the pooled selection logits (App. F's pooled query).
                            Threshold keeps the positions whose probability exceeds prob_param;
                            Top-p keeps the shortest prefix of the descending order whose
                            probabilities sum to at least prob_param.  Both keep at least the best
                            position and at most min(k, L_b) - the best ones, if the rule wants
                            more -, break ties like Eq. 2, and pad the set with -1.  Positions
                            only (block_size <= 1), and not together with keep_ppm.  Decisions are
                            taken in fp32: a position whose probability (cumulative probability)
                            lies within rounding of the parameter may fall on either side.     */
    float prob_param;    /* tau or p, in (0, 1]                                                  */
} lychee_shape;
#define LYCHEE_RULE_THRESHOLD 1
#define LYCHEE_RULE_TOP_P     2

/* Create / destroy a context bound to HIP device `device`.  Needs a GPU. */
int lychee_create(lychee_ctx **ctx, int device);
int lychee_destroy(lychee_ctx *ctx);

/* Pure host functions (no GPU needed).
 * lychee_check_shape: validates `shape`; if `head_type_mask` (HOST, [H_q]) is given it also
 *   checks that sparse heads come with an inherited set (`has_idx_in` != 0).
 * lychee_workspace_bytes: bytes of scratch any call below needs for `shape` (selection
 *   candidates and scores, split partials); 0 if the shape is invalid.  lychee_decode_step
 *   needs lychee_step_workspace_bytes (the same per layer).
 *   The workspace must be 256-byte aligned; its contents are don't-care on entry. */
int    lychee_check_shape(const lychee_shape *shape, const uint8_t *head_type_mask, int has_idx_in);
size_t lychee_workspace_bytes(const lychee_shape *shape);
size_t lychee_step_workspace_bytes(const lychee_shape *shape, int32_t n_layers); /* for lychee_decode_step */

/*
 * One layer of Alg. 1's per-head loop (retrieval branch: Eq. 1, Eq. 2, o = A V; sparse
 * branch: Eq. 3), for all sequences of a batch.
 *   q               bf16 [B][H_q][128], 16-byte aligned
 *   k_cache,v_cache bf16, strided as in `shape`, 16-byte aligned, read-only
 *   head_type_mask  HOST uint8 [H_q]: 1 = retrieval head, 0 = sparse head
 *   idx_in          int32 [B][H_kv][k], the sets inherited from the previous layer; may be
 *                   NULL only if every head is a retrieval head (the first layer)
 *   out             bf16 [B][H_q][128], 16-byte aligned
 *   idx_out         int32 [B][H_kv][k]: for a KV head whose group holds a retrieval head,
 *                   the min(k, L_b) positions with the highest mean retrieval logit; for any
 *                   other KV head a verbatim copy of idx_in.  Must not alias idx_in.
 *   lengths         int32 [B], 1 <= L_b <= max_len, the current token included (values
 *                   outside that range are clamped into it)
 * Errors: EINVAL (NULL / misaligned pointer, bad shape, sparse heads without idx_in,
 * idx_out == idx_in), EUNSUPPORTED (head_dim, group size; more than 2^31 blocks of 16 cache rows in
 * one launch, far beyond what fits a GPU), EWORKSPACE, EHIP.
 */
int lychee_decode_attn(lychee_ctx *ctx, const lychee_shape *shape, const void *q,
                       const void *k_cache, const void *v_cache, const uint8_t *head_type_mask,
                       const int32_t *idx_in, void *out, int32_t *idx_out, const int32_t *lengths,
                       void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * The same layer (Alg. 1's per-head loop), for a caller that runs layer after layer: in Alg. 1
 * the set S a retrieval head updates is read again only by the next layer's sparse heads, so
 * `out` does not have to wait for it.  This call enqueues everything that `out` needs and
 * leaves the selection (Eq. 2) of its layer PENDING; the next lychee_decode_attn_deferred call
 * on the same context runs the pending selection in its first launch, beside its own
 * preparations and before its sparse heads read their sets, and lychee_select_flush runs it
 * alone.  Arguments and errors as for lychee_decode_attn, except:
 *   workspace   lychee_step_workspace_bytes(shape, 2) bytes: the pending layer's selection
 *               candidates live in one half while the next layer fills the other
 *   idx_out     complete (in stream order) only after the call that runs the pending
 *               selection; nothing else may write it in between
 *   q           may be reused as soon as this call's work is done (the library keeps a copy of
 *               what a selection can still need)
 *   idx_in, k_cache, lengths (pointer AND contents), the workspace: unchanged until the
 *               pending selection has run.  In particular flush before the lengths grow for
 *               the next token, and before the workspace serves any other call.
 * While a selection is pending, the next deferred call must pass the same shape, lengths
 * pointer and workspace (else EINVAL: flush first), and every other call that is given that
 * workspace returns EINVAL.
 * Each such call is ONE kernel launch.  Inside it the pending selection runs on a few workgroups
 * of its own, the layer's sparse heads wait (with a bounded wait) until it has published the set
 * they read, and the workgroup that finishes a head's last piece merges the head's partials.
 * lychee_select_flush: enqueues a pending selection, if there is one (one small launch); EINVAL
 * for a NULL ctx.  A model that overlaps work on a second stream can flush there, off its
 * critical path, as long as the flush is ordered before the next layer's call.
 */
int lychee_decode_attn_deferred(lychee_ctx *ctx, const lychee_shape *shape, const void *q,
                                const void *k_cache, const void *v_cache, const uint8_t *head_type_mask,
                                const int32_t *idx_in, void *out, int32_t *idx_out, const int32_t *lengths,
                                void *workspace, size_t workspace_bytes, void *hip_stream);
int lychee_select_flush(lychee_ctx *ctx, void *hip_stream);

/*
 * lychee_decode_attn for callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): the same layer call without a workspace
 * argument.  Its scratch is an array of LYCHEE_STATIC_SCRATCH_BYTES bytes that is part of the
 * library's device code, so every GPU the library runs on holds it until the process ends; the
 * call allocates nothing, on the device or on the host.  Arguments, results and errors as for
 * lychee_decode_attn, and:
 *   EWORKSPACE    lychee_workspace_bytes(shape) exceeds LYCHEE_STATIC_SCRATCH_BYTES (the Qwen3-8B-shaped
 *                 128K layer at batch 1 needs about 22 MiB); nothing is enqueued
 *   EUNSUPPORTED  per-launch timing is enabled on the context (it creates events)
 * All calls on one GPU share the one array, whatever their context or stream, and it keeps the last
 * call's contents (which no call depends on): calls that overlap on a GPU race, so order them on one
 * stream or with events.
 */
#define LYCHEE_STATIC_SCRATCH_BYTES (32u << 20)
int lychee_decode_attn_static(lychee_ctx *ctx, const lychee_shape *shape, const void *q,
                              const void *k_cache, const void *v_cache, const uint8_t *head_type_mask,
                              const int32_t *idx_in, void *out, int32_t *idx_out, const int32_t *lengths,
                              void *hip_stream);

/* Dense decode attention on the same buffers: every head runs Eq. 1 and o = A V, nothing
 * is selected.  The in-run speed baseline; `shape->k` is ignored (any value >= 1). */
int lychee_dense_decode_attn(lychee_ctx *ctx, const lychee_shape *shape, const void *q,
                             const void *k_cache, const void *v_cache, void *out,
                             const int32_t *lengths, void *workspace, size_t workspace_bytes,
                             void *hip_stream);

/*
 * The attention of a whole decode step (Alg. 1, the layer loop restricted to its per-head
 * loop): layers 0 .. n_layers-1 in order, the sets written by layer l feeding layer l+1
 * (Sec. 3.1: the set is propagated to the next layer).  All layers share `shape` and
 * `lengths`.
 *   q, k_cache, v_cache, out   HOST arrays of n_layers device pointers
 *   head_type_masks            HOST uint8 [n_layers][H_q]
 *   idx_in                     sets entering layer 0, or NULL when layer 0 is all-retrieval
 *                              (Sec. 3.1: every head of the first layer is a retrieval head)
 *   idx_out                    the sets leaving the last layer; may be NULL
 *   workspace                  at least lychee_step_workspace_bytes(shape, n_layers) bytes
 * Because every layer's query is an input of the call, only the sparse heads of layer l+1
 * depend on layer l (through its sets).  STEP_MODE chooses how that is used:
 *   LYCHEE_STEP_PHASED (default)  five launches for the whole step: the selection
 *     thresholds of all layers, the retrieval streaming of all layers pooled in one launch,
 *     the selects, the sparse gathers of all layers, and the combines.  out[l] of every layer is complete only
 *     when the call's work has finished.
 *   LYCHEE_STEP_LAYERWISE  layer after layer, ONE launch per layer, each as
 *     lychee_decode_attn_deferred (layer l's selection runs inside layer l+1's launch, the last
 *     one alone); out[l] is complete before layer l+1 starts, as a model that computes q[l+1]
 *     from out[l] needs.
 * Fewer than 128 layers; PHASED falls back to LAYERWISE when n_layers * batch > 2048, and a
 * single layer always runs as lychee_decode_attn does.
 */
int lychee_decode_step(lychee_ctx *ctx, const lychee_shape *shape, int32_t n_layers,
                       const void *const *q, const void *const *k_cache,
                       const void *const *v_cache, const uint8_t *head_type_masks,
                       const int32_t *idx_in, void *const *out, int32_t *idx_out,
                       const int32_t *lengths, void *workspace, size_t workspace_bytes,
                       void *hip_stream);

/* Alg. 1, "C.append(k, v)": the decoded token's key and value rows
 *   k_new, v_new   bf16 [B][H_kv][128], 16-byte aligned
 * become row lengths[b] - 1 of every KV head of k_cache / v_cache (strided as in `shape`; lengths
 * count the token being decoded).  One small launch on the stream; needs no workspace. */
int lychee_append_kv(lychee_ctx *ctx, const lychee_shape *shape, const void *k_new,
                     const void *v_new, void *k_cache, void *v_cache, const int32_t *lengths,
                     void *hip_stream);

/* lychee_decode_step with each layer's cache append inside the call (Alg. 1: append, then
 * attend): k_new[l], v_new[l] (HOST arrays of n_layers device pointers, each bf16 [B][H_kv][128])
 * are written to row lengths[b] - 1 of layer l's caches before any of the step's attention
 * reads them.  In the phased step the appends ride in the first launch (the selection
 * thresholds, whose sample never touches the newest row), so they cost no launch of their own
 * (with block-granular sets, which need no thresholds, they are one small launch); layer after
 * layer, all layers' appends are one small launch in front of the first layer. */
int lychee_decode_step_append(lychee_ctx *ctx, const lychee_shape *shape, int32_t n_layers,
                              const void *const *q, const void *const *k_new,
                              const void *const *v_new, void *const *k_cache, void *const *v_cache,
                              const uint8_t *head_type_masks, const int32_t *idx_in,
                              void *const *out, int32_t *idx_out, const int32_t *lengths,
                              void *workspace, size_t workspace_bytes, void *hip_stream);

/* Dense attention for all layers of a step (Eq. 1 and o = A V for every head, no selection), in
 * the order STEP_MODE names: PHASED = all layers' streaming pooled in one launch, then the
 * combines; LAYERWISE = layer after layer as lychee_dense_decode_attn.  The in-run baseline of
 * lychee_decode_step; arguments as there, workspace of lychee_step_workspace_bytes. */
int lychee_dense_decode_step(lychee_ctx *ctx, const lychee_shape *shape, int32_t n_layers,
                             const void *const *q, const void *const *k_cache,
                             const void *const *v_cache, void *const *out, const int32_t *lengths,
                             void *workspace, size_t workspace_bytes, void *hip_stream);

const char *lychee_strerror(int code);

/* ==========================================================================================
 * Tuning and diagnostics.  Nothing below is needed to run the path; results never depend on any
 * of it beyond the fp32 rounding order of the split merge (index sets do not depend on it at all).
 * ========================================================================================== */

/* Options of a context.
 *   DEFAULTS      puts every option back to its default (value ignored)
 *   WG_PER_CU     workgroups per compute unit in every launch (1..3, default 2)
 *   N_WG          workgroups per launch, overriding WG_PER_CU (0 = CUs x WG_PER_CU; at most 768)
 *   STEP_MODE     how lychee_decode_step orders its work (see there)
 *   TAIL_PERMILLE permille of a phased launch's streaming / gather rows that workgroups claim
 *                 dynamically, in small chunks, after their fixed share (0..1000, default 250;
 *                 launches too short to hold several chunks per workgroup use none); it levels out
 *                 compute units that stream at different speeds
 *   GATHER_BLOCK  set entries whose gather is balanced against 64 streamed rows (a multiple
 *                 of 16 in [16, 128], default 48: a gathered row costs more than a streamed one)
 *   SELECT_MARGIN tenths of a standard deviation by which the sampled selection threshold is
 *                 lowered below its estimate of the k-th score (-10000..100000, default 60).
 *                 A larger margin makes more rows candidates of the exact select; a margin so
 *                 small that fewer than k rows pass, or so large that the candidate list
 *                 overflows, costs time (the row is then ranked from all of its scores) but
 *                 never changes a result
 *   SELECT_LEAD   layer launches: blocks of 64 rows the device streams while a pending select
 *                 runs (default 3000); the gathers that wait for that select get workgroups for
 *                 the work that is left by then */
#define LYCHEE_OPT_DEFAULTS     0
#define LYCHEE_OPT_WG_PER_CU    1
#define LYCHEE_OPT_STEP_MODE    2
#define LYCHEE_OPT_GATHER_BLOCK 6
#define LYCHEE_OPT_N_WG         7
#define LYCHEE_OPT_TAIL_PERMILLE 8
#define LYCHEE_OPT_SELECT_MARGIN 9
#define LYCHEE_OPT_SELECT_LEAD  10
#define LYCHEE_STEP_PHASED      1
#define LYCHEE_STEP_LAYERWISE   0
int lychee_set_option(lychee_ctx *ctx, int32_t option, int32_t value);

/* Debug helper (synchronous): counts entries of idx [B][H_kv][k] that break the index
 * conventions (out of [0, L_b), duplicated, or valid after a -1) into *n_bad (HOST).  The one call
 * of the library that allocates (and frees) device memory, 8 bytes: not for a captured stream. */
int lychee_validate_idx(lychee_ctx *ctx, const lychee_shape *shape, const int32_t *idx,
                        const int32_t *lengths, int64_t *n_bad, void *hip_stream);

/* Debug helper (synchronous): how many score rows, since the context was created, the select had
 * to rank from all of their scores because the sampled threshold let fewer than the budget
 * through (*too_few) or more than the candidate list holds (*too_many).  Both cost time, never
 * correctness; on smooth score distributions both stay 0. */
int lychee_select_stats(lychee_ctx *ctx, int64_t *too_few, int64_t *too_many, void *hip_stream);

/* Debug helper (synchronous): how many bounded waits inside layer launches have given up since the
 * context was created (a piece waiting for its row's threshold, a gather waiting for its set).
 * It stays 0 unless the device cannot keep a launch's workgroups resident together; a piece that
 * gives up on a threshold costs time only (its row is ranked whole), a gather that gives up on a
 * set reads the set as it is. */
int lychee_wait_timeouts(lychee_ctx *ctx, int64_t *timeouts, void *hip_stream);

/* Per-launch timing with HIP events on the caller's stream.  While enabled, every launch of
 * the library's kernels is bracketed by an event pair.  lychee_timing_read waits for the
 * recorded events, adds up the milliseconds and launches per launch class since the last
 * read and clears the record (arrays of LYCHEE_N_KERNEL_CLASSES entries). */
#define LYCHEE_KERNEL_STREAM  0   /* retrieval streaming of a phased step; a layer launch       */
#define LYCHEE_KERNEL_GATHER  1   /* sparse gather only                                     */
#define LYCHEE_KERNEL_THRESHOLD 2 /* selection thresholds                                   */
#define LYCHEE_KERNEL_SELECT  3   /* select / set copies only                               */
#define LYCHEE_KERNEL_COMBINE 4   /* combine (alone, with select or with set copies)        */
#define LYCHEE_N_KERNEL_CLASSES 5
int lychee_timing_enable(lychee_ctx *ctx, int on);
int lychee_timing_read(lychee_ctx *ctx, float *ms_per_class, int32_t *launches_per_class);

/* Plain streaming kernels used to calibrate the measurements: a read of `bytes` bytes
 * (sum folded into *sink, 4 bytes) and a copy of `bytes` bytes.  16-byte aligned, bytes a
 * multiple of 16. */
int lychee_probe_read(lychee_ctx *ctx, const void *src, size_t bytes, void *sink, void *hip_stream);
int lychee_probe_copy(lychee_ctx *ctx, void *dst, const void *src, size_t bytes, void *hip_stream);



#ifdef __cplusplus
}
#endif
#endif /* LYCHEE_H */
