/*
 * shifter.h - C ABI of the prune-and-compact pass for CNN variant portfolios
 *             (DNNShifter, arXiv 2309.06973), implemented as HIP kernels for gfx950.
 *
 * The pass turns one dense fp32 CNN into a sparse variant and then into a smaller
 * dense ("pruned") variant:
 *
 *   shifter_global_threshold   unstructured magnitude ranking over all prunable
 *                              weights (Sec. II-A, Sec. III-C)
 *   shifter_apply_mask         the sparse model: zeros written in place of the
 *                              lowest-magnitude weights (Sec. II-A, Sec. III-C)
 *   shifter_dead_channel_scan  Module 2, Sparsity Analyser (Sec. III-D)
 *   shifter_propagate_groups   Module 3, Prune Planner, Algorithm 1 (Sec. III-D)
 *   shifter_compact            Module 4, Model Pruner, Algorithm 2 (Sec. III-D)
 *
 * Conventions
 *   - Pointers named d_* are DEVICE pointers owned by the caller; h_* are HOST
 *     pointers owned by the caller.  The library never frees or keeps either.
 *   - A network is a flat fp32 weight arena (every conv / linear weight tensor, OIHW
 *     row-major, at the element offset its descriptor names) and a flat fp32 vector
 *     arena (BatchNorm gamma / beta / running mean / running variance, biases).
 *   - Channel groups: a group is a channel space.  Tensors whose out_group is G write
 *     it (producers), vectors whose group is G hold one value per channel of it,
 *     tensors whose in_group is G read it (consumers).  Residual adds put several
 *     producers into one group.  Pinned groups (network input, logits) never shrink.
 *   - Global index g: prunable tensors in descriptor order, each row-major.  The
 *     order on weights is (|w|, g) ascending; |w| is compared as the fp32 bit pattern
 *     with the sign cleared, so -0.0 == +0.0, denormals are exact, +-inf is largest.
 *     NaN among prunable weights is an error.
 *   - Every call enqueues its kernels on the context's stream and returns without
 *     waiting, except where a non-NULL h_* output is passed (documented per call):
 *     then the call waits for the stream and fills it.
 *   - A call that is given no h_* output puts kernels on the stream and nothing else
 *     (no allocation once the model is bound, no wait, no memset): such calls can be
 *     recorded into a HIP graph by capturing the context's stream after one eager call
 *     has bound the model.  A graph holds the pointers and prune counts of the recorded
 *     calls, not the data.  shifter_global_threshold with h_thr = NULL is the ranking
 *     to record: it needs no decision on the host.
 *   - Every function returns a shifter_status.  No exceptions or aborts cross the
 *     ABI; shifter_last_error() gives the text of the last failure.  Argument and
 *     descriptor errors are found on the host before anything is launched.
 *   - The library allocates device memory only in shifter_create and the first call
 *     that uses a model with a context (tables and scratch sized from the model);
 *     later calls allocate nothing (the codec calls are the one exception, see there).
 *   - A context, and a model bound to it, serve one call at a time: calls on the same
 *     context from several host threads must be serialised by the caller (the scratch
 *     of a model is shared by all calls that use it).  Different contexts are
 *     independent.
 */
#ifndef SHIFTER_H
#define SHIFTER_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct shifter_ctx shifter_ctx;     /* device, stream, scratch              */
typedef struct shifter_model shifter_model; /* validated copy of the descriptors    */

typedef enum {
    SHIFTER_OK = 0,
    SHIFTER_ERR_INVALID_ARG = 1, /* NULL pointer, count out of range, ...             */
    SHIFTER_ERR_BAD_MODEL = 2,   /* descriptors inconsistent                          */
    SHIFTER_ERR_NONFINITE = 3,   /* NaN among the prunable weights                    */
    SHIFTER_ERR_CAPACITY = 4,    /* output buffer too small; needed sizes reported    */
    SHIFTER_ERR_NO_DEVICE = 5,   /* no usable GPU                                     */
    SHIFTER_ERR_HIP = 6,         /* a HIP call failed                                 */
    SHIFTER_ERR_OOM = 7,         /* device or host allocation failed                  */
    SHIFTER_ERR_INTERNAL = 8,    /* an invariant of the library did not hold           */
    SHIFTER_WARN_COLLAPSE = 100  /* some group has no surviving channel (layer
                                    collapse, Sec. IV-B.1); outputs are still valid    */
} shifter_status;

/* One conv / linear weight tensor, OIHW row-major. linear: kh = kw = 1. */
typedef struct {
    uint64_t offset;    /* fp32 element offset in the weight arena                    */
    uint32_t out_ch;    /* O: must equal width of out_group                           */
    uint32_t in_ch;     /* I: input features = width of in_group * in_mult            */
    uint32_t kh, kw;
    uint32_t in_mult;   /* input features per input channel (flatten -> linear), else 1 */
    int32_t out_group;
    int32_t in_group;
    uint32_t prunable;  /* 1: ranked and masked; 0: copied, scanned and compacted only */
} shifter_tensor_desc;

typedef struct {
    uint64_t offset;    /* fp32 element offset in the vector arena                    */
    uint32_t len;       /* must equal width of group                                  */
    int32_t group;
} shifter_vec_desc;

typedef struct {
    uint32_t width;
    uint32_t pinned;    /* 1: never shrunk                                            */
} shifter_group_desc;

/* Result of the ranking for one prune count P.  Weight g is removed iff
 *      ((uint64_t)key(w_g) << 32 | g)  <  cut
 * i.e. iff (|w_g|, g) is among the P smallest pairs.  P = 0 gives cut = 0. */
typedef struct {
    uint64_t cut;
    uint32_t t_key;     /* bit pattern of |w| of the P-th smallest pair (0 if P = 0)  */
    uint32_t reserved;
    uint64_t g_cut;     /* global index of that pair (UINT64_MAX if P = 0)            */
    uint64_t n_prune;   /* P                                                          */
    uint64_t n_less;    /* weights with key <  t_key                                  */
    uint64_t n_equal;   /* weights with key == t_key                                  */
} shifter_threshold;

/* Sizes derived from the descriptors; the caller sizes its buffers from these. */
typedef struct {
    uint64_t n_prunable;      /* N: length of the global index space and of the mask  */
    uint64_t w_extent;        /* weight arena must hold at least this many floats     */
    uint64_t v_extent;        /* vector arena likewise                                */
    uint64_t w_elems;         /* sum of tensor sizes (capacity that always suffices)  */
    uint64_t v_elems;         /* sum of vector lengths                                */
    uint64_t sum_out_ch;      /* length of the out_alive flag array                   */
    uint64_t sum_in_ch;       /* length of the in_alive flag array                    */
    uint64_t sum_group_width; /* length of group_alive / index_map / keep             */
    uint32_t n_tensors, n_vecs, n_groups, reserved;
} shifter_model_info;

#define SHIFTER_GROUPS_JOINT 0u           /* residual-add groups pruned jointly        */
#define SHIFTER_PAPER_FREEZE_RESIDUAL 1u  /* groups with several producers left whole:
                                             skip / downsample connections are not
                                             pruned (Sec. IV-B.2)                      */

#define SHIFTER_GROUPS_FIXPOINT 2u        /* accepted (and implied) by
                                             shifter_propagate_groups_fixpoint        */

#define SHIFTER_MAX_VARIANTS 64u          /* prune counts per shifter_global_threshold */

/* --- contexts and models ---------------------------------------------------------- */

/* Creates a context on `device` (HIP ordinal).  `hip_stream` is a hipStream_t owned by
 * the caller (NULL = the default stream); every kernel of this context runs on it.
 * Fails with SHIFTER_ERR_NO_DEVICE when the device does not exist. */
int shifter_create(shifter_ctx** out, int device, void* hip_stream);
int shifter_destroy(shifter_ctx* ctx);

/* Text of the last failure on this context (or of the last failed call that had no
 * context when ctx is NULL).  Valid until the next call on the same thread. */
const char* shifter_last_error(const shifter_ctx* ctx);

/* Validates and copies the descriptor tables.  Host only: touches no GPU.
 * Errors (SHIFTER_ERR_BAD_MODEL): group index out of range, out_ch / in_ch / len not
 * matching the group widths, zero-sized dimension, overlapping tensors or vectors,
 * tensor of 2^32 - 8192 or more elements, N >= 2^32 - 1, more than 65535 tensors. */
int shifter_model_create(const shifter_tensor_desc* tensors, uint32_t n_tensors,
                         const shifter_vec_desc* vecs, uint32_t n_vecs,
                         const shifter_group_desc* groups, uint32_t n_groups,
                         shifter_model** out);
int shifter_model_destroy(shifter_model* model);
int shifter_model_get_info(const shifter_model* model, shifter_model_info* out);

/* Offsets of tensor t inside the out_alive / in_alive arrays and of group g inside the
 * per-group arrays (arrays of n_tensors / n_tensors / n_groups entries, any may be
 * NULL). */
int shifter_model_get_layout(const shifter_model* model, uint64_t* h_out_flag_off,
                             uint64_t* h_in_flag_off, uint64_t* h_group_off);

/* --- the five steps ---------------------------------------------------------------- */

/* Unstructured magnitude ranking (Sec. II-A; Sec. III-C): for each of the K prune
 * counts h_n_prune[k] (0 <= P <= N, K <= SHIFTER_MAX_VARIANTS) finds the P-th smallest
 * pair (|w_g|, g) over all prunable weights and writes its record to d_thr[k].  One
 * pass structure serves all K counts (a portfolio ranks the same dense weights).
 *   d_w        device, weight arena, w_extent floats, read only
 *   d_thr      device, K records, written
 *   h_thr      host, K records, or NULL.  Non-NULL: the call waits for the stream,
 *              copies the records and reports SHIFTER_ERR_NONFINITE if a prunable
 *              weight is NaN.  NULL: no wait and no NaN report (a NaN compares above
 *              +inf; the records are then meaningless).  A waiting call may use the
 *              single-pass selection (see shifter_set_select_path). */
int shifter_global_threshold(shifter_ctx* ctx, const shifter_model* model,
                             const float* d_w, const uint64_t* h_n_prune, uint32_t K,
                             shifter_threshold* d_thr, shifter_threshold* h_thr);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving or training loops, harnesses that forbid it): the ranking of
 * shifter_global_threshold for ONE flat run of n weights (global index = element index; a
 * single tensor's weights, or an arena without gaps), with no model and no allocation.  It
 * calls no hipMalloc / hipFree and no allocating routine, puts only kernels on the
 * context's stream (no wait, no copy, no memset) and keeps its tables, histograms and
 * per-tile counts in a device array that is part of the library's code object: about
 * 4.7 MB that every GPU the library runs on holds until the process ends.
 *   d_w        device, n floats, 16-byte aligned, read only (may be NULL when n = 0)
 *   h_n_prune  host, K prune counts, each <= n; 1 <= K <= SHIFTER_MAX_VARIANTS
 *   d_thr      device, K records, written (same records as shifter_global_threshold's
 *              multi-pass select on a model of one prunable tensor of n weights; no NaN
 *              report, as with h_thr = NULL there)
 * Limits: n <= SHIFTER_STATIC_MAX_WEIGHTS and K * ceil(n / 4096) <=
 * SHIFTER_STATIC_MAX_TILE_COUNTS, else SHIFTER_ERR_CAPACITY (nothing is enqueued).
 * All calls on one GPU share that GPU's array, whatever their context or stream: calls
 * that overlap in time on one GPU race; calls on one stream, or otherwise ordered, are
 * fine.  What must start at zero is cleared by the call's first kernel. */
#define SHIFTER_STATIC_MAX_WEIGHTS (1ull << 28)
#define SHIFTER_STATIC_MAX_TILE_COUNTS (1ull << 20)
int shifter_global_threshold_static(shifter_ctx* ctx, const float* d_w, uint64_t n,
                                    const uint64_t* h_n_prune, uint32_t K,
                                    shifter_threshold* d_thr);

/* Which selection algorithm shifter_global_threshold and shifter_prune_fused may use:
 * 0 (default) the single-pass selection where it applies (waiting or two-call form,
 * at most 32 prune counts above zero), with the multi-pass radix select as its
 * fall-back (taken when the pass's own check fails: a sample that misjudged a quantile,
 * tens of thousands of weights equal to a threshold, or - for several prune counts -
 * an index space beyond about 10^9 weights); 1 the multi-pass radix select only.  Both
 * give the same records. */
int shifter_set_select_path(shifter_ctx* ctx, int path);

/* Half-width of the key interval the single-pass selection predicts from its sample,
 * in standard deviations of a binomial sample of the same size (default 4; doubled
 * automatically, up to 64, each time a prediction misses).  A wider
 * interval means more candidate weights to settle after the pass, a narrower one a
 * higher chance that the pass cannot decide and the multi-pass select runs.  Never
 * affects results. */
int shifter_set_margin_sigmas(shifter_ctx* ctx, double sigmas);

/* Blocks of the multi-pass select's histogram kernels, which walk the tiles with a stride
 * of the grid (default eight per compute unit; 1 .. 65536).  A launch shape only: the
 * records, and everything computed from them, are the same bytes for every value. */
int shifter_set_select_grid(shifter_ctx* ctx, uint32_t blocks);

/* Arena size, in bytes, above which shifter_portfolio_begin ranks and masks a portfolio in
 * one fused read of the arena; at or below it the counting pass and the batched mask pass
 * run as two launches, which is faster while the arena stays in the last-level cache
 * between them (default 192 MiB).  0: always fused; UINT64_MAX: never.  A choice of
 * kernels only: every output is the same bytes either way. */
int shifter_set_fused_min_bytes(shifter_ctx* ctx, uint64_t bytes);

/* Outcome of the last waiting selection on this context, for measurement:
 * out8 = { path (1 single pass decided, 2 multi-pass select ran, 0 none yet), P,
 *          weights below the interval, weights inside it, sample size, interval low key,
 *          interval high key, status bits of the single pass }. */
int shifter_get_select_stats(const shifter_ctx* ctx, uint64_t* out8);

/* Ranking, sparse model and zero-channel scan for ONE prune count in a single read of
 * the arena (Sec. II-A; Sec. III-C; Module 2 of Sec. III-D): same outputs as
 * shifter_global_threshold(K = 1) followed by shifter_apply_mask with the scan.
 * The pass predicts a narrow key interval around the threshold from a sample, writes
 * the final value of every weight outside it while counting, and settles the few
 * weights inside it once the exact threshold is known; if the prediction fails its own
 * exactness check the two separate steps are run instead.
 *   d_w_out      device, w_extent floats; must differ from d_w
 *   d_mask       device, N bytes, or NULL
 *   d_out_alive, d_in_alive   device, required
 *   d_thr        device, one record, required
 *   h_thr        host, one record, or NULL.  Non-NULL: the call waits for the stream; a NaN
 *                among the prunable weights gives SHIFTER_ERR_NONFINITE (outputs are then
 *                unspecified).  NULL (and the single pass allowed): the call only
 *                enqueues work and the outcome is collected later by
 *                shifter_prune_fused_result; the caller may enqueue the steps that
 *                consume the outputs in between, at the risk of having to repeat them.
 *                The pointers of a deferred call must stay valid until it is collected,
 *                and no other shifter_prune_fused may be issued on the context before.
 *
 * shifter_prune_fused_result waits for the stream and settles a deferred call: h_thr
 * (may be NULL) receives the record; *h_redone = 0 if the single pass was exact, 1 if the
 * two separate steps had to be run now - every output of shifter_prune_fused has then been
 * rewritten and whatever was derived from them since must be computed again.  Without a
 * deferred call pending it only waits and h_thr receives the record of the last
 * shifter_prune_fused that waited itself. */
int shifter_prune_fused(shifter_ctx* ctx, const shifter_model* model, const float* d_w,
                        uint64_t n_prune, shifter_threshold* d_thr, float* d_w_out,
                        uint8_t* d_mask, uint8_t* d_out_alive, uint8_t* d_in_alive,
                        shifter_threshold* h_thr);
int shifter_prune_fused_result(shifter_ctx* ctx, shifter_threshold* h_thr, int* h_redone);

/* The sparse model (Sec. II-A; Sec. III-C): d_w_out[e] = removed ? +0.0f : d_w[e] for
 * every element of every tensor (non-prunable tensors are copied), d_mask[g] = 0 for
 * removed weights else 1.
 *   d_thr        device, ONE record (as written by shifter_global_threshold)
 *   d_w_out      device, w_extent floats; may equal d_w (in place); gaps between
 *                tensors are not written
 *   d_mask       device, N bytes, or NULL
 *   d_out_alive, d_in_alive
 *                both NULL, or both non-NULL: the scan of shifter_dead_channel_scan
 *                is then done on the sparse values in the same pass (same outputs). */
int shifter_apply_mask(shifter_ctx* ctx, const shifter_model* model, const float* d_w,
                       const shifter_threshold* d_thr, float* d_w_out, uint8_t* d_mask,
                       uint8_t* d_out_alive, uint8_t* d_in_alive);

/* Module 2, Sparsity Analyser (Sec. III-D): a kernel is the kh x kw slice of one
 * (filter, input feature) pair.  For every tensor t (prunable or not):
 *   d_out_alive[out_flag_off[t] + o] = 1 iff filter o holds a non-zero, else 0
 *   d_in_alive [in_flag_off[t]  + i] = 1 iff input feature i holds a non-zero in any
 *                                       filter, else 0
 * Arrays of sum_out_ch / sum_in_ch bytes, fully written.  -0.0 counts as zero. */
int shifter_dead_channel_scan(shifter_ctx* ctx, const shifter_model* model,
                              const float* d_w_sparse, uint8_t* d_out_alive,
                              uint8_t* d_in_alive);

/* Module 3, Prune Planner (Algorithm 1, Sec. III-D), stated on groups: channel c of
 * group G survives iff G is pinned or some producer of G has out_alive on c (with
 * SHIFTER_PAPER_FREEZE_RESIDUAL also iff G has more than one producer).  On a chain
 * this gives, for layer n, C_out = zero filters of layer n and C_in = zero filters of
 * layer n-1, and no C_in for the first layer.  Single pass: removing input channels
 * never triggers further removals.  d_in_alive is accepted for symmetry and not used
 * by either rule (may be NULL).
 *   d_group_alive  device, sum_group_width bytes: 1 survives / 0 removed
 *   d_index_map    device, sum_group_width int32: new index of a channel, or -1
 *   d_keep         device, sum_group_width uint32: per group, the surviving old
 *                  indices ascending, then UINT32_MAX up to the group's width
 *   d_new_width    device, n_groups uint32
 *   h_new_width    host, n_groups uint32, or NULL.  Non-NULL: waits for the stream and
 *                  returns SHIFTER_WARN_COLLAPSE if some group kept no channel. */
int shifter_propagate_groups(shifter_ctx* ctx, const shifter_model* model,
                             const uint8_t* d_out_alive, const uint8_t* d_in_alive,
                             uint32_t flags, uint8_t* d_group_alive,
                             int32_t* d_index_map, uint32_t* d_keep,
                             uint32_t* d_new_width, uint32_t* h_new_width);

/* --- liveness fixpoint (an extension beyond Algorithm 1's single pass) --------------
 *
 * Module 2 indexes zero kernels before it indexes zero channels (Sec. III-D).  On that
 * kernel-level index the plan can go further than Algorithm 1: a channel c of a group
 * that is neither pinned nor frozen stays only while it is
 *   produced: some tensor writing the group has, in filter c, a non-zero kernel whose
 *             input feature belongs to a surviving channel, and
 *   read:     some tensor reading the group has a non-zero kernel on a feature of c in a
 *             filter whose channel survives.
 * Starting from all channels, failing channels are removed and the rules applied again
 * until nothing changes; the result is the largest rule-consistent set.  It is a subset
 * of the single-pass plan.  (Under the convention that a removed channel emits 0, which
 * Algorithm 2 already applies by dropping its bias, the rebuilt network computes the same
 * function.)
 *
 * shifter_model_get_kernel_layout
 *   h_kernel_off   host, n_tensors: offset of tensor t's [out_ch][in_ch] block in the
 *                  kernel index, or NULL;  h_sum_kernels: its total length, or NULL
 * shifter_kernel_scan
 *   d_kernel_nz    device, sum_kernels bytes, fully written: byte kernel_off[t] +
 *                  o * in_ch + i is 1 iff the kernel of filter o and input feature i of
 *                  tensor t holds a non-zero (-0.0 counts as zero), else 0
 * shifter_propagate_groups_fixpoint
 *   d_kernel_nz    as written by shifter_kernel_scan
 *   flags          SHIFTER_PAPER_FREEZE_RESIDUAL keeps groups with several producers
 *                  whole; SHIFTER_GROUPS_FIXPOINT is accepted
 *   outputs        as shifter_propagate_groups
 *   h_rounds       host, number of rounds run (the last one removed nothing), or NULL
 * Rounds are enqueued in batches of four with no wait between them: the kernels of a round
 * return at once when the round before removed nothing, and each batch ends with the plan
 * of what is alive then.  With h_new_width or h_rounds given the call waits once per
 * batch and goes on until the fixpoint is reached (one wait for up to four rounds).  With
 * both NULL it waits for nothing and enqueues four batches (so it can be recorded into a
 * HIP graph); should sixteen rounds not reach the fixpoint, the plan written is that of
 * the sixteenth round - every channel it removes is one the fixpoint removes too, so the
 * rebuilt network still computes the same function, only larger than need be.
 * shifter_fixpoint_status
 *   reads what the last call's kernels reported, once the caller has waited for the
 *   stream: h_rounds (rounds run) and h_settled (1 iff the last round removed nothing),
 *   either may be NULL. */
int shifter_model_get_kernel_layout(const shifter_model* model, uint64_t* h_kernel_off,
                                    uint64_t* h_sum_kernels);
int shifter_kernel_scan(shifter_ctx* ctx, const shifter_model* model, const float* d_w_sparse,
                        uint8_t* d_kernel_nz);
int shifter_propagate_groups_fixpoint(shifter_ctx* ctx, const shifter_model* model,
                                      const uint8_t* d_kernel_nz, uint32_t flags,
                                      uint8_t* d_group_alive, int32_t* d_index_map,
                                      uint32_t* d_keep, uint32_t* d_new_width,
                                      uint32_t* h_new_width, uint32_t* h_rounds);
int shifter_fixpoint_status(shifter_ctx* ctx, const shifter_model* model, uint32_t* h_rounds,
                            uint32_t* h_settled);

/* --- Module 1, Model Pre-Processor (Sec. III-D): conv + BatchNorm fold ----------------
 *
 * Merges every layer with the BatchNorm that follows it, so that the later modules see
 * convolutions with a bias and nothing else.  For a listed tensor with a BatchNorm
 * (gamma, beta, running mean, running variance), in fp32:
 *   s_o      = gamma_o / sqrt(var_o + eps)
 *   W'[o, :] = W[o, :] * s_o
 *   b'_o     = beta_o + (b_o - mean_o) * s_o      (b_o = 0 without a bias vector)
 * A listed tensor without a BatchNorm keeps its weights and gets b' = b.  Tensors that
 * are not listed are copied unchanged.  Zero weights stay zero, so a sparse arena keeps
 * its zero structure (gamma_o = 0 zeroes filter o).  Each result is the correctly rounded
 * fp32 operation sequence above (the product (b_o - mean_o) * s_o is not rounded before
 * beta_o is added); against exact arithmetic the weights are within 4 * 2^-24 relative.
 *
 * One entry per layer; vector fields index the model's vector descriptors, -1 = absent.
 * gamma, beta, mean and var are given together or not at all; every vector named must
 * have the tensor's out_ch elements. */
typedef struct {
    uint32_t tensor;
    int32_t gamma, beta, mean, var;
    int32_t bias;
    uint64_t out_offset;   /* fp32 element offset of the layer's out_ch biases in d_bias_out */
} shifter_fold_desc;

/*   h_fold, n_fold   host, the layers to fold; a tensor may be listed once; the
 *                    [out_offset, out_offset + out_ch) ranges must not overlap
 *   eps              the BatchNorm's epsilon, finite and >= 0
 *   d_w              device, weight arena in the model's layout (dense or sparse)
 *   d_vecs           device, the model's vector arena
 *   d_w_out          device, weight arena of the same layout; may be d_w (in place);
 *                    elements outside the tensors are not touched
 *   d_bias_out       device, cap_bias floats; only the listed ranges are written
 * The validated layer table stays on the device with the model.  A call whose list
 * equals that of the call before only enqueues the fold: no upload, no wait, and the call
 * may be recorded into a HIP graph.  A call with another list (the first one included)
 * waits for the work already on the context's stream, uploads the table, then enqueues
 * the fold; on a capturing stream it is refused with SHIFTER_ERR_INVALID_ARG.
 * Errors: SHIFTER_ERR_INVALID_ARG for a bad list (nothing is enqueued). */
int shifter_fold_bn(shifter_ctx* ctx, const shifter_model* model,
                    const shifter_fold_desc* h_fold, uint32_t n_fold, float eps,
                    const float* d_w, const float* d_vecs, float* d_w_out,
                    float* d_bias_out, uint64_t cap_bias);

/* --- Phase 3 codec (Sec. III-E): Module 7 deflates inactive models, Module 8 inflates --
 *
 * shifter_deflate turns a byte buffer (a model's arena) into one DEFLATE stream (RFC
 * 1951) that any inflater reads, laid out for chunk-parallel decoding:
 *   - the input is cut into chunks of SHIFTER_CODEC_CHUNK bytes and every chunk into
 *     sub-chunks of SHIFTER_CODEC_SUB bytes; chunk c becomes the byte-aligned segment
 *     [seg_off[c], seg_off[c + 1]) of the stream;
 *   - tokens of a sub-chunk, left to right: a maximal run of r >= 4 equal bytes (cut at the
 *     sub-chunk's end) is one literal and distance-1 matches over the other r - 1 bytes
 *     (258 while more than 260 remain; then one piece, or the pieces (rest - 3, 3) when 259
 *     or 260 remain); every other byte is a literal;
 *   - a sub-chunk whose tokens would take more than 8 * (its bytes) + 48 bits is stored
 *     (a stored block of its own: shorter, and copied instead of decoded); the others are
 *     coded with the fixed Huffman codes;
 *   - a segment walks its sub-chunks: a coded one opens a fixed-Huffman block (BFINAL = 0)
 *     unless one is open and appends its tokens; a stored one closes the open block with
 *     end-of-block and is a stored block (BFINAL = 0, padding to a byte, LEN, NLEN, the
 *     bytes); after the last sub-chunk the open block is closed and an empty stored block
 *     pads to a byte boundary.  If that is not shorter than one stored block holding the
 *     whole chunk (its size + 5 bytes), the segment is that block.  BFINAL = 1 only on the
 *     last block of the last segment; an empty input gives the 5-byte stream
 *     01 00 00 FF FF;
 *   - side information, not part of the stream: seg_off, and per sub-chunk a uint16: its
 *     token bits if coded, 0xFFFF if stored (all 0 when the chunk is one stored block);
 *   - a mark per sub-chunk (uint64), with which four lanes decode a coded sub-chunk of n
 *     bytes side by side: for q = 1, 2, 3 let B_q = min(128 q, n), o_q the offset of the
 *     first literal token at or after B_q (n if none) and b_q the bits of all tokens
 *     before that literal (a run's matches go with the literal that starts it; all token
 *     bits if none), b_0 = 0; the mark is the sum over q of
 *     ((b_q - b_(q-1)) | (o_q - B_q) << 11) << 20 (q - 1).  Lane q decodes bits
 *     [b_q, b_(q+1)) into bytes [o_q, o_(q+1)).  Stored and empty sub-chunks, and chunks
 *     stored as one block, have mark 0.  Marks take 8 bytes per 512 bytes of input and the
 *     token bits 2: together 2 % of the input, beside the stream.
 * The output is a deterministic function of the input.
 *
 * shifter_codec_layout   sizes for n_bytes of input: chunks (at least 1), bytes of
 *                        workspace, and the largest possible stream (any of the three
 *                        outputs may be NULL)
 * shifter_deflate
 *   d_in, n_bytes        device, 16-byte aligned input (may be NULL when n_bytes = 0)
 *   d_work, work_bytes   device, 256-byte aligned scratch of at least the layout's size
 *   d_stream, stream_cap device, 16-byte aligned; capacity in bytes
 *   d_seg_off            device, n_chunks + 1 uint64; the last entry is the stream's size
 *   d_sub_bits           device, n_chunks * (CHUNK / SUB) uint16: the per-sub-chunk side
 *                        information
 *   d_sub_marks          device, n_chunks * (CHUNK / SUB) uint64: the per-sub-chunk marks
 *   h_stream_bytes       host or NULL.  Non-NULL: the call waits for the stream and stores
 *                        the stream's size; returns SHIFTER_ERR_CAPACITY (size still
 *                        stored, nothing written to d_stream) when stream_cap is too small.
 *                        NULL: kernels are enqueued and nothing is waited for (the size is
 *                        the last entry of d_seg_off, and shifter_codec_status has it)
 * shifter_inflate        decodes a stream made by shifter_deflate, given its side
 *                        information and marks, into n_bytes at d_out (device, 16-byte
 *                        aligned).  stream_bytes: the bytes readable at d_stream, at least
 *                        the stream's size (which is the last entry of d_seg_off).  wait != 0: waits, and returns SHIFTER_ERR_INVALID_ARG
 *                        with "bad stream" when the stream, the offsets, the side
 *                        information or the marks do not fit together (sizes, block
 *                        headers, token set and every lane's range are checked; all
 *                        accesses stay inside the buffers up to the 4-byte granule that
 *                        holds the stream's last byte; d_out is then unspecified).
 *                        wait = 0: kernels are enqueued and nothing is waited for; whether
 *                        the stream was bad is then asked of shifter_codec_status.
 *                        DEFLATE carries no checksum: a damaged literal that still parses
 *                        is not found.
 * shifter_codec_status   what the context's last codec call reported, once the caller has
 *                        waited for the stream: the stream's size (deflate) and whether
 *                        the stream was bad (inflate) or did not fit (deflate); either
 *                        pointer may be NULL.
 * The codec calls need no model.  They keep chunk lists of 8 bytes per chunk of device
 * memory in the context, allocated when an input with more chunks than before comes (so
 * a call recorded into a HIP graph must follow an eager one of at least that size). */
#define SHIFTER_CODEC_CHUNK 32768u
#define SHIFTER_CODEC_SUB 512u
int shifter_codec_layout(uint64_t n_bytes, uint64_t* h_n_chunks, uint64_t* h_work_bytes,
                         uint64_t* h_stream_bound);
int shifter_deflate(shifter_ctx* ctx, const void* d_in, uint64_t n_bytes, void* d_work,
                    uint64_t work_bytes, uint8_t* d_stream, uint64_t stream_cap,
                    uint64_t* d_seg_off, uint16_t* d_sub_bits, uint64_t* d_sub_marks,
                    uint64_t* h_stream_bytes);
int shifter_inflate(shifter_ctx* ctx, const uint8_t* d_stream, uint64_t stream_bytes,
                    const uint64_t* d_seg_off, const uint16_t* d_sub_bits,
                    const uint64_t* d_sub_marks, uint64_t n_bytes, void* d_out, int wait);
int shifter_codec_status(shifter_ctx* ctx, uint64_t* h_stream_bytes, uint32_t* h_bad);

/* Module 4, Model Pruner (Algorithm 2, Sec. III-D): every layer rebuilt without its
 * prunable channels.  For tensor t with out-group A, in-group B, m = in_mult:
 *   W'[o', i', y, x] = W[keep_A[o'], keep_B[i' / m] * m + i' % m, y, x]
 * and for every vector v of group A: v'[j] = v[keep_A[j]].  Outputs are dense, in
 * descriptor order, row-major, the first tensor at element 0.
 *   d_w_sparse, d_vecs   device, source arenas
 *   d_keep, d_new_width  device, as written by shifter_propagate_groups
 *   d_w_out, cap_w       device, capacity in floats (w_elems always suffices)
 *   d_vecs_out, cap_v    device, capacity in floats (v_elems always suffices)
 *   h_out_tensors        host, n_tensors descriptors of the rebuilt tensors, or NULL
 *   h_out_vecs           host, n_vecs descriptors, or NULL
 *   h_elems_w, h_elems_v host, floats written to each output arena, or NULL
 * If any h_* is non-NULL the call waits for the stream and fills them.  When a
 * capacity is too small nothing is gathered; a waiting call then returns
 * SHIFTER_ERR_CAPACITY with the needed sizes in h_elems_w / h_elems_v. */
int shifter_compact(shifter_ctx* ctx, const shifter_model* model, const float* d_w_sparse,
                    const float* d_vecs, const uint32_t* d_keep,
                    const uint32_t* d_new_width, float* d_w_out, uint64_t cap_w,
                    float* d_vecs_out, uint64_t cap_v, shifter_tensor_desc* h_out_tensors,
                    shifter_vec_desc* h_out_vecs, uint64_t* h_elems_w,
                    uint64_t* h_elems_v);

/* --- a whole portfolio per call ------------------------------------------------------ */

/* Steps 2-5 for the K variants of a portfolio in one launch per step (Sec. III-C: the
 * variants of a portfolio mask the same dense weights at growing sparsity; Sec. III-D
 * Module 4: every layer's channels removed by one operation).  Results per variant are
 * identical to the single-variant calls; variant k's buffers sit k strides after
 * variant 0's.  The dense arena is read once for all K sparse arenas.
 *
 * shifter_apply_mask_batch
 *   d_thr        device, K records (as written by shifter_global_threshold)
 *   d_w_out      device, K arenas, w_stride floats apart (w_stride >= w_extent, multiple
 *                of 4 for full speed); must not overlap d_w.  NULL: the sparse arenas
 *                are not materialised (shifter_compact_batch_masked rebuilds from the
 *                dense arena and d_thr); masks and flags are produced as usual
 *   d_mask       device, K masks, mask_stride bytes apart (>= N), or NULL
 *   d_out_alive  device, K * sum_out_ch bytes, required
 *   d_in_alive   device, K * sum_in_ch bytes, or NULL
 * shifter_propagate_groups_batch
 *   d_out_alive  as above; d_group_alive / d_index_map / d_keep: K * sum_group_width
 *   entries; d_new_width: K * n_groups; h_new_width: host, K * n_groups, or NULL (waits)
 * shifter_compact_batch
 *   d_w_sparse   the K sparse arenas (w_stride apart); d_keep, d_new_width as above
 *   d_w_out      device, K output arenas cap_w floats apart (cap_w a multiple of 4);
 *   d_vecs_out   K vector arenas cap_v floats apart
 *   h_out_tensors K * n_tensors, h_out_vecs K * n_vecs, h_elems_w / h_elems_v K entries,
 *   each or NULL; any non-NULL makes the call wait.  SHIFTER_ERR_CAPACITY if any variant
 *   does not fit (that variant is not gathered), SHIFTER_WARN_COLLAPSE if any collapsed.
 * shifter_compact_batch_masked
 *   the same rebuild with the dense arena d_w and the K threshold records d_thr as its
 *   source: variant k's mask (removed <=> composite < d_thr[k].cut, prunable tensors
 *   only) is applied while its weights are gathered, so the K rebuilds share one source
 *   and the K sparse arenas are not read again.  Outputs are identical to
 *   shifter_compact_batch on the arenas shifter_apply_mask_batch wrote for d_thr. */
/* Steps 1-3 for the K prune counts of a portfolio in ONE read of the dense arena: the
 * ranking of shifter_global_threshold (records in d_thr / h_thr, caller order) and the
 * outputs of shifter_apply_mask_batch (d_w_out may be NULL, d_mask may be NULL, d_in_alive
 * may be NULL), identical to calling the two in turn.  Always waits (the host decides
 * whether the single pass was exact; if not, it runs the two calls instead).
 * SHIFTER_ERR_NONFINITE if a prunable weight is NaN. */
int shifter_prune_fused_batch(shifter_ctx* ctx, const shifter_model* model, const float* d_w,
                              const uint64_t* h_n_prune, uint32_t K, shifter_threshold* d_thr,
                              float* d_w_out, uint64_t w_stride, uint8_t* d_mask,
                              uint64_t mask_stride, uint8_t* d_out_alive, uint8_t* d_in_alive,
                              shifter_threshold* h_thr);
/* shifter_global_threshold in two halves, so that a portfolio step waits once: _begin
 * enqueues the ranking of the K prune counts (the single pass over the arena where it
 * applies) and returns; the caller enqueues the later steps, which read d_thr on the
 * device, and waits for them; _end then waits for the stream (a formality by then), stores
 * the K records in h_thr (or NULL) and says in *h_redone (or NULL) whether the single pass
 * had to be replaced by the multi-pass select: if so, d_thr now holds the exact records
 * and everything enqueued behind _begin must be repeated (rare: heavy ties).  One
 * _begin at a time per context.  SHIFTER_ERR_NONFINITE from _end if a prunable weight
 * is NaN. */
/* All five steps for the K prune counts of a portfolio (K = 1 included) behind one pair of
 * calls (Sec. III-C, Sec. III-D Modules 2-4): _begin checks the arguments and enqueues the
 * whole step - ranking, sparse arenas, masks, flags, group plans, rebuilt variants - in the
 * order and with the kernel fusion that suits the arena's size, and returns without
 * waiting; _end waits for the stream once and returns the records and the rebuilt
 * variants' descriptors.  Every output is identical to what the single steps give
 * (shifter_global_threshold, shifter_apply_mask_batch, shifter_propagate_groups_batch,
 * shifter_compact_batch).  If the single-pass ranking could not decide (rare: heavy ties),
 * _end runs the multi-pass select and repeats the later steps itself before it returns.
 *   d_w, d_vecs       device, the dense weight arena and the vector arena
 *   h_n_prune, K      host, K prune counts
 *   flags             as shifter_propagate_groups
 *   d_thr             device, K records, written
 *   d_w_sparse        device, K sparse arenas w_stride floats apart, or NULL (not materialised)
 *   d_mask            device, K masks mask_stride bytes apart, or NULL
 *   d_out_alive       device, K * sum_out_ch bytes; d_in_alive: K * sum_in_ch bytes, or NULL
 *   d_group_alive, d_index_map, d_keep: device, K * sum_group_width entries each;
 *   d_new_width       device, K * n_groups
 *   d_w_out, cap_w    device, K output arenas cap_w floats apart (a multiple of 4 if K > 1)
 *   d_vecs_out, cap_v device, K vector arenas cap_v floats apart
 * The pointers must stay valid until _end; one _begin at a time per context, and no other
 * call on the context in between.
 * _end: h_thr K records; h_out_tensors K * n_tensors, h_out_vecs K * n_vecs, h_elems_w /
 * h_elems_v K entries; each may be NULL.  Returns SHIFTER_ERR_NONFINITE (NaN among the
 * prunable weights), SHIFTER_ERR_CAPACITY (a variant does not fit and was not gathered),
 * SHIFTER_WARN_COLLAPSE (some variant lost a whole group; outputs valid). */
typedef struct {
    const float* d_w;
    const float* d_vecs;
    const uint64_t* h_n_prune;
    uint32_t K;
    uint32_t flags;
    shifter_threshold* d_thr;
    float* d_w_sparse;
    uint64_t w_stride;
    uint8_t* d_mask;
    uint64_t mask_stride;
    uint8_t* d_out_alive;
    uint8_t* d_in_alive;
    uint8_t* d_group_alive;
    int32_t* d_index_map;
    uint32_t* d_keep;
    uint32_t* d_new_width;
    float* d_w_out;
    uint64_t cap_w;
    float* d_vecs_out;
    uint64_t cap_v;
} shifter_portfolio_args;
int shifter_portfolio_begin(shifter_ctx* ctx, const shifter_model* model,
                            const shifter_portfolio_args* args);
int shifter_portfolio_end(shifter_ctx* ctx, shifter_threshold* h_thr,
                          shifter_tensor_desc* h_out_tensors, shifter_vec_desc* h_out_vecs,
                          uint64_t* h_elems_w, uint64_t* h_elems_v);
int shifter_global_threshold_begin(shifter_ctx* ctx, const shifter_model* model,
                                   const float* d_w, const uint64_t* h_n_prune, uint32_t K,
                                   shifter_threshold* d_thr);
int shifter_global_threshold_end(shifter_ctx* ctx, shifter_threshold* h_thr, int* h_redone);
int shifter_apply_mask_batch(shifter_ctx* ctx, const shifter_model* model, const float* d_w,
                             const shifter_threshold* d_thr, uint32_t K, float* d_w_out,
                             uint64_t w_stride, uint8_t* d_mask, uint64_t mask_stride,
                             uint8_t* d_out_alive, uint8_t* d_in_alive);
int shifter_propagate_groups_batch(shifter_ctx* ctx, const shifter_model* model,
                                   const uint8_t* d_out_alive, uint32_t K, uint32_t flags,
                                   uint8_t* d_group_alive, int32_t* d_index_map,
                                   uint32_t* d_keep, uint32_t* d_new_width,
                                   uint32_t* h_new_width);
int shifter_compact_batch(shifter_ctx* ctx, const shifter_model* model, const float* d_w_sparse,
                          uint64_t w_stride, const float* d_vecs, const uint32_t* d_keep,
                          const uint32_t* d_new_width, uint32_t K, float* d_w_out,
                          uint64_t cap_w, float* d_vecs_out, uint64_t cap_v,
                          shifter_tensor_desc* h_out_tensors, shifter_vec_desc* h_out_vecs,
                          uint64_t* h_elems_w, uint64_t* h_elems_v);
int shifter_compact_batch_masked(shifter_ctx* ctx, const shifter_model* model, const float* d_w,
                                 const shifter_threshold* d_thr, const float* d_vecs,
                                 const uint32_t* d_keep, const uint32_t* d_new_width,
                                 uint32_t K, float* d_w_out, uint64_t cap_w, float* d_vecs_out,
                                 uint64_t cap_v, shifter_tensor_desc* h_out_tensors,
                                 shifter_vec_desc* h_out_vecs, uint64_t* h_elems_w,
                                 uint64_t* h_elems_v);

/* --- measurement ------------------------------------------------------------------- */

/* Per-kernel timing with HIP events on the context's stream.  While enabled every
 * kernel launch of this context is bracketed by two events.  shifter_profile_read waits
 * for the stream, then for each kernel that ran since the last reset writes its name,
 * launch count and total milliseconds (up to `cap` entries; returns the number in
 * *n_out) and resets the records.  Names are static strings owned by the library. */
int shifter_profile_enable(shifter_ctx* ctx, int on);
int shifter_profile_read(shifter_ctx* ctx, const char** names, uint32_t* counts,
                         double* total_ms, uint32_t cap, uint32_t* n_out);

/* Plain device-to-device copy kernel of n floats (dwordx4 loads and stores; both
 * pointers 16-byte aligned), used to
 * calibrate the memory-traffic counters against a transfer of known size and to
 * measure the copy bandwidth this chip sustains. */
int shifter_copy_f32(shifter_ctx* ctx, const float* d_src, float* d_dst, uint64_t n);

#ifdef __cplusplus
}
#endif
#endif /* SHIFTER_H */
