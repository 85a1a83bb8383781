/*
 * pop.h -- C ABI of the POP (Partition-guided Online Pruning) pruned-FFN library for MI355X (gfx950).
 *
 * One layer = one SwiGLU FFN  y = W_down (silu(W_gate x) * (W_up x))  with hidden size d and
 * intermediate size m.  "Channel" always means one of the m intermediate channels: row j of W_gate and
 * W_up, column j of W_down (Sec. 3.1: an output channel of the first projections is one dimension of the
 * intermediate representation, shared by the consecutive linear maps).
 *
 * Importance (Sec. 3.1 Eq. 1-2, Sec. 3.4 Eq. 3), read on the down projection and its input activations:
 *     I_j = || W_down[:, j] ||_2 * sqrt( sum over tokens t of H[t][j]^2 ),   H = silu(X W_gate^T) * (X W_up^T).
 * The same formula is used at prefill (all prompt tokens) and at a decode step (one token).
 *
 * Conventions for every entry point
 *   - returns a status code (POP_OK == 0, negative on error); never throws, never exits.
 *   - pointers marked "dev" are device (HBM) pointers, "host" are host pointers.  The caller owns every
 *     buffer it passes; the library never frees or keeps them beyond the call, except that
 *     pop_layer_create reads the three weight matrices once and keeps its own repacked copy
 *     (device memory cost: one extra copy of the weights plus O(max_batch * m) scratch).
 *   - argument errors are found on the host before anything is launched.  Device work is enqueued on
 *     the given HIP stream (a hipStream_t passed as void*, NULL = the null stream) and is NOT
 *     synchronised: the caller synchronises the stream before reading outputs.
 *   - a layer handle may be used from one stream at a time.  Calls on one handle that overlap in time race.
 *   - index lists are int32, ascending by channel; regions are one byte per channel.
 *   - dtype of x, weights: the layer's wdtype (float32, or bf16 stored as 16-bit patterns).
 *     bf16 layers need d % 8 == 0, float32 layers d % 4 == 0 (128-bit loads), else POP_EUNSUPPORTED.
 *   - device pointers to activations (x, x_t), weights and outputs y must be 16-byte aligned (the kernels use
 *     128-bit accesses); a misaligned one is rejected with POP_EINVAL.
 *   - inputs must be finite; with non-finite inputs results are deterministic but unspecified.
 */
#ifndef POP_H
#define POP_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pop_layer pop_layer_t; /* opaque, owned by the library */

typedef enum { POP_F32 = 0, POP_BF16 = 1 } pop_dtype_t;

enum {
    POP_OK = 0,
    POP_EINVAL = -1,       /* NULL pointer, negative size, bad enum */
    POP_ESHAPE = -2,       /* sizes inconsistent with the layer or with each other */
    POP_ENOMEM = -3,       /* device allocation failed */
    POP_EHIP = -4,         /* a HIP call failed; text via pop_last_hip_error() */
    POP_ESTATE = -5,       /* call order violated (e.g. decode before prefill) */
    POP_EUNSUPPORTED = -6, /* valid request this build does not implement */
    POP_EDEVICE = -7       /* a kernel gave up a bounded wait; results of that step are invalid */
};

enum { POP_REGION_RETAINED = 0, POP_REGION_CANDIDATE = 1, POP_REGION_PRUNED = 2 };

#define POP_MAX_BATCH 8 /* largest B of pop_decode_mask / largest token chunk processed per pass */

int pop_version(void);
const char *pop_strerror(int status);      /* static storage */
const char *pop_last_hip_error(void);      /* text of the last failing HIP call on this thread */

/* Host only.  Region sizes from fractions (Sec. 3.3: thresholds at quantile levels r-delta and r+delta,
 * realised as exact rank counts):  n_ret = floor(f_ret*m + 1/2),  n_ret + n_cand = floor((f_ret+f_cand)*m + 1/2),
 * n_prn = m - n_ret - n_cand.  With the paper's (r, delta): f_ret = 1-r-delta, f_cand = 2*delta. */
int pop_region_counts(int m, double f_ret, double f_cand, int *n_ret, int *n_cand, int *n_prn);

/* Host only.  Number of candidates to select per token so that the active channel count is
 * floor((1-r)*m + 1/2) (Sec. 3.3 "Decoding Stage"), clamped to [0, n_cand]. */
int pop_k_for_ratio(int m, double r, int n_ret, int n_cand, int *k);

/* Host only.  Region sizes and per-token k of the decode strategies compared in the paper's ablation (Sec. 5,
 * trade-off table), all with floor((1-r)*m + 1/2) active channels per token:
 *   POP_STRATEGY_POP          the method: candidate band of gamma*m channels centred on the sparsity quantile
 *                             (f_ret = 1-r-gamma/2, f_cand = gamma; counts and k as in the two functions above);
 *   POP_STRATEGY_STATIC_MASK  Variant (1): the prefill mask is reused at every step (n_cand = 0, all active
 *                             channels retained): no re-scoring, no selection, no overhead;
 *   POP_STRATEGY_RESCORE_ALL  Variant (2): every channel is a candidate at every step (n_ret = 0, n_cand = m).
 * The counts go to pop_prefill_partition / pop_decode_mask unchanged.  gamma is ignored by the two variants.
 * Errors: a band that leaves [0, 1] or an unknown strategy -> POP_EINVAL. */
enum { POP_STRATEGY_POP = 0, POP_STRATEGY_STATIC_MASK = 1, POP_STRATEGY_RESCORE_ALL = 2 };
int pop_strategy_counts(int strategy, int m, double r, double gamma, int *n_ret, int *n_cand, int *k);
/* Value for n_ret, n_cand (both), k0 and - as a NULL pointer - k in the calls below: "what the layer's strategy says"
 * (pop_layer_set_strategy). */
enum { POP_FROM_STRATEGY = -1 };

/* Create a layer.  w_gate, w_up: dev [m][d]; w_down: dev [d][m]; all of dtype wdtype, read once, on `stream`,
 * and repacked channel-major (one contiguous gate+up row pair and one contiguous down column per channel).
 * Also computes the data-free weight factor n_j = ||W_down[:,j]||_2 of Eq. 3.
 * max_tokens: largest T of pop_prefill_partition; max_batch: largest B (1..POP_MAX_BATCH).
 * The stream is synchronised before returning (the caller may free the source weights afterwards). */
int pop_layer_create(pop_layer_t **out, int d, int m, pop_dtype_t wdtype,
                     const void *w_gate, const void *w_up, const void *w_down,
                     int max_tokens, int max_batch, void *stream);
int pop_layer_destroy(pop_layer_t *layer);

/* Prefill (Sec. 3.3 "Prefilling Stage"): H for all m channels and all T prompt tokens (x: dev [T][d]),
 * I_j over the T tokens, then the three regions by rank in the order (score descending, channel ascending):
 * the best n_ret channels are retained, the next n_cand are candidates, the rest are pruned.
 * Outputs (dev, any may be NULL): scores [m] float32; region [m] (POP_REGION_*); ret_idx [n_ret];
 * cand_idx [n_cand].  The partition is also kept inside the layer for the decode calls.
 * T == 0 is allowed (x may then be NULL): with no tokens every importance is zero and the regions follow the
 * channel order (an expert of a mixture that no prompt token was routed to).
 * Errors: T < 0 or T > max_tokens, n_ret/n_cand < 0 or n_ret + n_cand > m -> POP_ESHAPE. */
int pop_prefill_partition(pop_layer_t *layer, const void *x, int T, int n_ret, int n_cand,
                          float *scores, unsigned char *region, int *ret_idx, int *cand_idx, void *stream);

/* Prefilling stage with its output (Sec. 3.3 "Prefilling Stage", Sec. 3.4: the prompt's forward pass runs under the
 * pruning structure the prompt itself determines).  Everything pop_prefill_partition does, with the same outputs
 * and errors, and then the pruned FFN of the T prompt tokens, y: dev [T][d] of dtype ydtype, under the prefill mask:
 * the retained channels plus the best k0 candidates by prefill score (same order as above), i.e. the n_ret + k0
 * channels of highest prefill importance.  mask: dev [m], 1 = active (may be NULL).
 * On bf16 layers with T >= 32 the hidden activations of the contraction are kept (rounded to bf16), the active
 * columns are gathered, and the down projection runs as one matrix-core GEMM; otherwise the call is
 * pop_prefill_partition followed by pop_pruned_ffn(mask).  Scratch for H (2 x T x m x 2 bytes, plus up to
 * 8 x 256 x d x 4 bytes of partial outputs) is allocated at the first call and when T grows, which synchronises
 * the device; it stays with the layer.
 * Errors: as pop_prefill_partition; k0 < 0 or k0 > n_cand -> POP_ESHAPE; y == NULL or bad ydtype -> POP_EINVAL. */
int pop_prefill_forward(pop_layer_t *layer, const void *x, int T, int n_ret, int n_cand, int k0,
                        void *y, pop_dtype_t ydtype, float *scores, unsigned char *region, int *ret_idx,
                        int *cand_idx, unsigned char *mask, void *stream);

/* Decode step, mask part (Sec. 3.3 "Decoding Stage", Sec. 3.4 two-step decoding).  x_t: dev [B][d].
 * Pass 1 evaluates h_j = silu(g_j) * u_j for every retained and candidate channel, for each of the B
 * sequences; candidates are re-scored, I_j(t) = n_j * |h_j|, and for sequence b the best k[b] (host array [B],
 * 0 <= k[b] <= n_cand) are selected with the same tie rule as above.
 * Outputs (dev, any may be NULL): cand_scores [B][n_cand] float32 in cand_idx order; mask [B][m], 1 = active
 * (retained or selected); active_idx [B][n_ret + n_cand], row b holds the retained channels ascending followed
 * by the selected ones ascending, n_active[b] = n_ret + k[b] entries valid; n_active [B].
 * h and the masks stay cached in the layer for pop_pruned_ffn(mask = NULL).
 * Errors: no partition yet -> POP_ESTATE; B < 1 or B > max_batch, k[b] out of range -> POP_ESHAPE. */
int pop_decode_mask(pop_layer_t *layer, const void *x_t, int B, const int *k,
                    float *cand_scores, unsigned char *mask, int *active_idx, int *n_active, void *stream);

/* Pruned FFN output (Sec. 3.3: only retained and selected channels form the step's computation;
 * Sec. 3.4 final computation).  y: dev [T][d] of dtype ydtype.
 *   mask == NULL: finish the decode step started by the immediately preceding pop_decode_mask on this layer
 *       (T must equal its B; x is not read again):  y_b = sum over active j of h_bj * W_down[:, j].
 *   mask != NULL: stand-alone pruned FFN of x (dev [T][d]) under the given masks, dev [mask_rows][m],
 *       mask_rows == 1 (shared by all tokens) or == T (one per token); any T >= 1.  Does not need a
 *       partition.  An all-ones mask gives the dense FFN.  bf16 layers with T >= 32 run this on the matrix
 *       cores: gate/up over the channels active in any row, H rounded to bf16, then one GEMM over those channels
 *       (scratch is allocated at the first such call and when T grows, which synchronises the device); smaller
 *       T and float32 layers take the decode kernels, eight tokens at a time, and keep H in float32.
 * Errors: mask == NULL without a preceding decode step -> POP_ESTATE; T mismatch, bad mask_rows -> POP_ESHAPE. */
int pop_pruned_ffn(pop_layer_t *layer, const void *x, int T, const unsigned char *mask, int mask_rows,
                   void *y, pop_dtype_t ydtype, void *stream);

/* Whole decode step in one call (Sec. 3.3 "Decoding Stage", Sec. 3.4: pass 1 over retained and candidate
 * channels, candidate re-scoring, per-token selection, then the output over retained and selected channels):
 * the same results, bit for bit, as pop_decode_mask followed by pop_pruned_ffn(mask = NULL), with y: dev [B][d] of
 * dtype ydtype and the other outputs as in pop_decode_mask (each may be NULL).
 * It issues exactly those two calls' launches.  A B == 1 step on a shape the fused single-sequence kernel takes is
 * two launches: that kernel, whose workgroups hand each other the candidates' h and the selection inside the launch,
 * and a small kernel that sums their partial outputs.  Neither keeps host-side state per launch, so captured
 * launches can be replayed.  The waits inside the fused launch, and inside the first launch of a B > 1 step (its
 * selecting workgroups wait for the candidates' scores), are bounded (pop_layer_set_wait_limit): if one gives
 * up, the step's results are invalid, pop_layer_sync_status reports POP_EDEVICE, every kernel still exits and the
 * next step is unaffected.
 * Errors: as pop_decode_mask; y == NULL or bad ydtype -> POP_EINVAL. */
int pop_decode_step(pop_layer_t *layer, const void *x_t, int B, const int *k, void *y, pop_dtype_t ydtype,
                    float *cand_scores, unsigned char *mask, int *active_idx, int *n_active, void *stream);

/* ---- pieces of the path exposed on their own (selection parity is defined on caller-supplied scores) ---- */

/* Three regions from given scores (dev [m] float32), as in pop_prefill_partition.  Needs no layer. */
int pop_partition_from_scores(const float *scores, int m, int n_ret, int n_cand,
                              unsigned char *region, int *ret_idx, int *cand_idx, void *stream);

/* The same, and in the same launch the n_top best channels of that order, 0 <= n_top <= m: the mask a prompt's own
 * forward pass runs under (Sec. 3.4; pop_prefill_forward uses n_top = n_ret + k0: the retained channels plus the best
 * k0 candidates by prefill score are the n_ret + k0 best channels overall).  Outputs (dev): top_mask [m] (1 = among
 * the n_top best; may be NULL), top_list [n_top] ascending channel numbers (required).
 * Errors: as pop_partition_from_scores; top_list == NULL -> POP_EINVAL; n_top out of range -> POP_ESHAPE. */
int pop_partition_top_from_scores(const float *scores, int m, int n_ret, int n_cand, int n_top,
                                  unsigned char *region, int *ret_idx, int *cand_idx,
                                  unsigned char *top_mask, int *top_list, void *stream);

/* Step selection from given candidate scores (Sec. 3.3 "Decoding Stage": of the candidate region the k channels of
 * highest step score stay active next to the retained region; equal scores by lower channel number):
 * cand_scores dev [n_cand] in cand_idx order, cand_idx dev [n_cand] ascending, region dev [m], 0 <= k <= n_cand.
 * Outputs (dev, may be NULL): mask [m] (retained + selected), sel_idx [k] ascending.
 * Errors: NULL inputs -> POP_EINVAL; sizes out of range -> POP_ESHAPE. */
int pop_topk_from_scores(const float *cand_scores, const int *cand_idx, int n_cand, int k,
                         const unsigned char *region, int m, unsigned char *mask, int *sel_idx, void *stream);

/* Column-wise importance reduction alone (Eq. 3): h dev [T][m] (float32 or bf16), nrm dev [m] float32,
 * scores[j] = nrm[j] * sqrt(sum_t h[t][j]^2).  The tokens are summed in chunks; the per-chunk partial sums
 * (at most 32 x m doubles) live in scratch that this call allocates and frees on `stream` (hipMallocAsync).
 * Errors: NULL pointers, bad dtype -> POP_EINVAL; T < 1 or m < 1 -> POP_ESHAPE; no memory -> POP_ENOMEM. */
int pop_importance_reduce(const void *h, pop_dtype_t hdtype, int T, int m, const float *nrm,
                          float *scores, void *stream);

/* Allocates, now, the scratch that pop_prefill_forward and pop_pruned_ffn(mask) need for prompts of up to T tokens
 * (they otherwise allocate it at their first call and when T grows, which synchronises the device), so that those
 * calls only enqueue work afterwards.  New buffers are cleared on `stream`.  Sec. 3.4 (the prompt's forward pass).
 * Errors: T < 1 or T > max_tokens -> POP_ESHAPE; allocation failure -> POP_ENOMEM. */
int pop_layer_reserve_prompt(pop_layer_t *layer, int T, void *stream);

/* pop_importance_reduce for callers that cannot allocate (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): the same kernels, arguments, results (bit for bit) and errors, but the per-chunk partial
 * sums live in a static device array of 8 MiB that every GPU the library runs on holds until the process ends; the
 * call allocates and frees nothing.  Limit: m <= 32768 channels, else POP_EUNSUPPORTED (use pop_importance_reduce).
 * All calls on one GPU share that array: calls that overlap in time on one GPU (different streams) race; calls on one
 * stream are ordered and safe.  A failing HIP call gives POP_EHIP (no text is recorded for pop_last_hip_error). */
int pop_importance_reduce_static(const void *h, pop_dtype_t hdtype, int T, int m, const float *nrm,
                                 float *scores, void *stream);

/* Read-only views of layer state, for tests and callers that build on the partition.
 * Copies are enqueued on `stream`; outputs dev, any may be NULL: nrm [m] float32 (n_j of Eq. 3),
 * h [B][m] float32 of the last decode step (0 for pruned channels is NOT guaranteed: only retained and
 * candidate entries are defined). */
int pop_layer_get_norms(pop_layer_t *layer, float *nrm, void *stream);
/* Synchronises `stream`, then reports whether any decode step on this layer since the last report (or the last
 * prefill) hit the bound of an in-kernel wait: POP_OK, or POP_EDEVICE (the results of such a step are invalid; repeat
 * it).  The record is cleared by the report.  Every kernel exits either way; this call is how a caller finds out. */
int pop_layer_sync_status(pop_layer_t *layer, void *stream);
int pop_layer_get_hidden(pop_layer_t *layer, float *h, int B, void *stream);
/* Host only.  Makes one of the ablation's decode strategies (Sec. 5, trade-off table; see pop_strategy_counts) the
 * layer's mode at sparsity r (and band gamma for POP_STRATEGY_POP): pop_prefill_partition and pop_prefill_forward
 * called with n_ret = n_cand = POP_FROM_STRATEGY (and k0 = POP_FROM_STRATEGY) then take the strategy's region sizes
 * (and its k), and pop_decode_mask / pop_decode_step called with k == NULL select the strategy's k for every
 * sequence.  Explicit counts keep working next to it.  Does not touch an existing partition.
 * Errors: as pop_strategy_counts; without a strategy the sentinels give POP_ESTATE (prefill) / POP_EINVAL (k). */
int pop_layer_set_strategy(pop_layer_t *layer, int strategy, double r, double gamma);
/* Host only.  How many times a bounded in-kernel wait of a decode step looks for what it waits for before it gives
 * up (default 65536: a fraction of a second).  Two kernels wait: the fused single-sequence step (Sec. 3.4: its
 * workgroups hand each other the candidates' h and the selection) and the batched step's first launch, whose
 * selecting workgroups wait for the candidates' scores.  A wait that gives up flags the step (pop_layer_sync_status:
 * POP_EDEVICE) and leaves its results invalid; every kernel still exits, and the next step is unaffected.  0 makes
 * every wait give up at once unless the data is already there: a testing knob.
 * Errors: NULL layer or looks < 0 -> POP_EINVAL. */
int pop_layer_set_wait_limit(pop_layer_t *layer, int looks);
/* Host only.  Which reading of Sec. 3.1 defines channel importance on this layer (the paper's equations admit two):
 *   POP_IMPORTANCE_OUTPUT_SIDE (default)  the down projection and the intermediate activations, as at the top of
 *       this file; the decode step scores candidates from h (Sec. 3.4's two-step decoding).
 *   POP_IMPORTANCE_INPUT_SIDE             Eq. 1-2 literally on the first projections and the FFN input:
 *       I_j = || [W_gate[j,:], W_up[j,:]] * s ||_2,  s_k = sqrt(sum over tokens of x[t][k]^2)  (a channel is removed
 *       from both matrices, so its weights are both rows); at a decode step s_k = |x_k|, per sequence.  Prefill
 *       then needs no contraction (one pass over the gate and up rows).  A single-sequence decode step runs in the
 *       fused kernel, which forms a candidate's score from the same two rows it reads for h; a step with B > 1
 *       selects first and runs the forward pass over retained and selected channels only, as separate launches: h
 *       of an unselected candidate is then not computed, so pop_layer_get_hidden is defined on active channels
 *       only under this reading.  With the shared batch mask s_k runs over the step's B rows.
 * Changing the reading discards the layer's partition (prefill again).  Errors: unknown value -> POP_EINVAL. */
enum { POP_IMPORTANCE_OUTPUT_SIDE = 0, POP_IMPORTANCE_INPUT_SIDE = 1 };
int pop_layer_set_importance(pop_layer_t *layer, int reading);
/* Host only.  How a decode step with B > 1 scores its candidates.  off (default): every sequence by its own
 * activation, I_j = n_j |h_bj|, its own top-k and mask.  on: the activation norm of Eq. 3 runs over the step's B
 * sequences ("tokens and samples", Sec. 3.1), I_j = n_j sqrt(sum_b h_bj^2), and one selection serves the whole
 * batch: all k[b] must be equal (else POP_ESHAPE), every row of cand_scores, mask and active_idx comes out the
 * same.  B == 1 is unaffected.  Invalidates a cached decode step. */
int pop_layer_set_shared_batch_mask(pop_layer_t *layer, int on);
/* Host only.  Which implementation the last successful decode step on this layer used: 0 = none yet,
 * 1 = the fused single-sequence kernel, 2 = the batch-general kernels.  If workgroups != NULL it
 * receives the fused kernel's grid size for the current partition (0 when the fused kernel does not apply). */
int pop_layer_step_kind(pop_layer_t *layer, int *workgroups);

/* ---- measurement aids: bare reads of device memory (they compute nothing of the method) ----
 * The decode step (Sec. 3.3 "Decoding Stage", Sec. 3.4) is bound by the bytes it must stream; these two calls request
 * such bytes and nothing else, so that timing them (events on `stream`) gives the time the memory system itself needs:
 * the yardstick next to the published peak bandwidth.  sink: dev, one unsigned int the kernels may OR a bit into.
 *   pop_probe_read       contiguous read of `bytes` (rounded down to 16) of buf (dev, 16-byte aligned).
 *   pop_probe_step_read  the weight rows one decode step of the layer's current partition reads: gate and up rows of
 *                        all retained and candidate channels, down rows of the retained channels and of the first k
 *                        candidates (standing in for the selected ones).
 * workgroups: grid size (512 threads each).  Errors: NULL / misaligned pointers -> POP_EINVAL; no partition ->
 * POP_ESTATE; sizes out of range -> POP_ESHAPE. */
int pop_probe_read(const void *buf, size_t bytes, int workgroups, unsigned int *sink, void *stream);
int pop_probe_step_read(pop_layer_t *layer, int k, int workgroups, unsigned int *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* POP_H */
