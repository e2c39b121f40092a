/*
 * pf.h -- C ABI of libpf: the neuron-aware sparse FFN of one LLM decode step on one
 * MI355X (gfx950), after PowerInfer (arXiv 2312.12456).
 *
 * The paper's problem statement for one layer (Sec. 4.2 single-layer example, Sec. 5.1
 * predictors, Sec. 5.4 neuron-aware operators): a hidden state comes in; a small MLP
 * predictor marks the FFN neurons expected to fire; only for those neurons the FC1 row
 * (and gate row), the activation and the FC2 column are read and computed; the FFN
 * output goes out.  Everything here runs on the GPU (no CPU half, no merge step): the
 * whole model is resident in HBM.
 *
 * Conventions
 *  - Every data pointer is a DEVICE pointer unless a comment says "host".  Pointers
 *    passed in pf_layer_weights are BORROWED: the library keeps them and the caller
 *    keeps the memory alive and unchanged until pf_layer_destroy.  The library owns
 *    only its per-context scratch.
 *  - Row-major, neuron-major: one neuron of FC1, of the gate matrix and of FC2 is one
 *    contiguous run.  FC2 is therefore passed transposed, [ffn][d].
 *  - All compute calls are asynchronous on `stream` (a hipStream_t passed as void*,
 *    NULL = the default stream), never synchronise with the host and never copy the
 *    active count back: the sparse kernels size their work from device memory.
 *  - A pf_ctx (its scratch) may be used by one stream at a time.
 *  - Every function returns a pf_status; nothing throws, exits or prints.  Argument
 *    errors are detected on the host before anything is launched.
 */
#ifndef PF_H
#define PF_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PF_OK = 0,
    PF_EINVAL = 1,       /* null pointer, negative size, batch above the context's limit */
    PF_ESHAPE = 2,       /* ffn % 64, d % 8, r % 8, (int4) d % 128, layer larger than ctx */
    PF_ENOMEM = 3,       /* device or host allocation failed                             */
    PF_EHIP = 4,         /* a HIP call failed; pf_last_error has its text                */
    PF_EUNSUPPORTED = 5, /* activation / weight type combination not built               */
    PF_ELIMIT = 6        /* pf_layer_step_noalloc: a size beyond its fixed maxima        */
} pf_status;

typedef enum {
    PF_ACT_RELU = 0,  /* OPT-style: h = ReLU(w_up.x + b_up)                      (Sec. 2.1) */
    PF_ACT_REGLU = 1, /* ReLU-gated: h = ReLU(w_gate.x + b_up) * (w_up.x)  (Table "model_eval") */
    PF_ACT_DRELU = 2  /* dReLU: h = ReLU(w_gate.x + b_up) * ReLU(w_up.x): the activation named for
                         Bamboo-7B in Table "model_eval"; the paper gives no formula, this is
                         the reading taken (ReLU on both branches of the gated block)          */
} pf_act;

typedef enum {
    PF_W_FP16 = 0,      /* IEEE binary16 weights                                  (Sec. 8.1) */
    PF_W_INT4_G128 = 1  /* nibble u in [0,15], value = scale * (u - 8), one fp16 scale per
                           128 consecutive elements of a neuron's row; element 2j in the low
                           nibble of byte j, 2j+1 in the high nibble             (Sec. 8.1) */
} pf_wtype;

typedef struct {
    int32_t d;          /* model width                      */
    int32_t ffn;        /* neurons in the FFN block         */
    int32_t r;          /* predictor hidden width           */
    int32_t act;        /* pf_act                           */
    int32_t wtype;      /* pf_wtype (predictor is always fp16) */
    float threshold;    /* predictor score threshold in (0,1): active iff score > threshold */
} pf_layer_desc;

typedef struct {
    const void *w_up;    /* [ffn][d] fp16, or [ffn][d/2] packed int4                     */
    const void *w_gate;  /* same shape; NULL for PF_ACT_RELU, required otherwise          */
    const void *w_down;  /* FC2 transposed, [ffn][d] / [ffn][d/2]                        */
    const void *s_up;    /* [ffn][d/128] fp16 scales, int4 only, else NULL               */
    const void *s_gate;
    const void *s_down;
    const float *b_up;   /* [ffn] FC1 bias (the gate bias when gated) or NULL            */
    const float *b_down; /* [d] FC2 bias or NULL                                         */
    const void *p1;      /* [r][d]   fp16 predictor input layer                          */
    const void *p2;      /* [ffn][r] fp16 predictor output layer                         */
    const float *p_bias; /* [ffn] added to the predictor logit, or NULL                  */
} pf_layer_weights;

typedef struct pf_ctx pf_ctx;
typedef struct pf_layer pf_layer;
typedef struct pf_plan pf_plan;

/* Arithmetic (Sec. 8.1: fp16 or int4 weights, fp32 activations): every product is accumulated
 * in fp32.  Small batches multiply fp32 activations with the widened weights on the vector
 * units.  From 4 tokens on -- from 3 where d > 4096 -- FC1 and the predictor of fp16 layers
 * run on the matrix cores, where each
 * fp32 activation enters as the sum of two fp16 numbers (rounded value + residual, 21 bits
 * kept); activations there must lie inside the fp16 range (|x| < 65504), which normalised
 * hidden states do by orders of magnitude.
 *
 * Context: binds a device and owns scratch sized for the given maxima (hidden vector,
 * mask words, index list, FC1 outputs, FC2 partial sums).  `device` is a HIP ordinal.
 * Errors: PF_EINVAL (out == NULL, sizes < 1, max_batch > 8), PF_ESHAPE, PF_ENOMEM, PF_EHIP. */
pf_status pf_ctx_create(pf_ctx **out, int device, int max_d, int max_ffn, int max_r,
                        int max_batch);
void pf_ctx_destroy(pf_ctx *ctx);

/* Layer: validates the descriptor against the context and records the borrowed weight
 * pointers (no weight is copied and nothing is launched; the layer owns 256 bytes of device
 * state for pf_layer_step_adaptive).  p1/p2 may be NULL for a layer that is only
 * used with pf_sparse_ffn. */
pf_status pf_layer_create(pf_ctx *ctx, const pf_layer_desc *desc, const pf_layer_weights *w,
                          pf_layer **out);
void pf_layer_destroy(pf_layer *layer);

/* Activation predictor (Sec. 5.1: input, one hidden, output layer):
 *   t = ReLU(p1 . x),  logit = p2 . t + p_bias,  score = 1/(1+exp(-logit)),
 *   neuron i is active iff score_i > threshold for at least one of the B tokens.
 * x [B][d] fp32.  scores: optional [B][ffn] fp32 (NULL to skip).  mask_words: [ffn/64]
 * uint64, bit b of word w = neuron 64*w + b.  The comparison is made on the fp32 logit
 * against logit(threshold), which is the same decision in exact arithmetic. */
pf_status pf_predict(pf_ctx *ctx, const pf_layer *layer, const float *x, int B, float *scores,
                     uint64_t *mask_words, void *stream);

/* Active-index compaction: idx[0..count) = ascending positions of the set bits of
 * mask_words[0..ffn/64), *count = their number (a device int32).  idx has capacity ffn;
 * entries from count on are left unspecified.  (The paper tests activation inside every
 * thread block, Sec. 5.4; compacting first is this library's choice for a 256-CU part.) */
pf_status pf_compact(pf_ctx *ctx, const uint64_t *mask_words, int ffn, int32_t *idx,
                     int32_t *count, void *stream);

/* Neuron-aware FFN over an index list (Sec. 5.4; Sec. 2.1 for the block itself):
 *   for j < *count, i = idx[j]:  h_j = act(row i of FC1 (and gate) . x + b_up[i])
 *   y[b][:] = b_down + sum_j h_j[b] * (row i of FC2^T)
 * for every token b of the batch (the list is the union over the batch, Sec. 8.2).
 * idx: ascending, no duplicates, entries in [0, ffn) (out-of-range entries are skipped);
 * the array must hold ffn entries whatever *count is (entries from *count on may be read
 * ahead of the count and are ignored).  count: device int32, clamped to [0, ffn].  y [B][d] fp32 is fully overwritten, also
 * when *count == 0 (then y = b_down).  Accumulation is fp32, in a fixed order. */
pf_status pf_sparse_ffn(pf_ctx *ctx, const pf_layer *layer, const float *x, int B,
                        const int32_t *idx, const int32_t *count, float *y, void *stream);

/* One layer of the decode step: predict -> compact -> sparse FFN, on one stream with no
 * host involvement (Sec. 4.2 without the CPU half).  x [B][d] -> y [B][d]. */
pf_status pf_layer_step(pf_ctx *ctx, const pf_layer *layer, const float *x, int B, float *y,
                        void *stream);

/* pf_layer_step for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  The same kernels and launches as
 * pf_layer_step, but no context: the scratch (hidden vector, mask words, index list, count,
 * FC1 outputs, FC2 partial sums) is a fixed array in the library's device image, about 1.2 MB
 * that every GPU the library runs on holds until the process ends.  The call allocates and
 * frees nothing, on the device or through any library.  It runs on the calling thread's
 * current device; desc / w as for pf_layer_create (weights are only read during the call's
 * kernels), x [B][d] -> y [B][d], asynchronous on `stream`.
 * Limits: d <= 8192, ffn <= 32768, r <= 2048, B <= 4; beyond them PF_ELIMIT, before anything is
 * launched.  Other argument errors as for pf_layer_create / pf_layer_step (status only: there
 * is no context to hold a message).
 * All calls on one GPU share that GPU's array, which keeps the previous call's contents: every
 * piece is rewritten before it is read, so nothing needs clearing, but two calls that overlap
 * on one GPU (different streams or threads) race -- serialise them. */
pf_status pf_layer_step_noalloc(const pf_layer_desc *desc, const pf_layer_weights *w, const float *x,
                                int B, float *y, void *stream);

/* Dense FFN of the layer: every neuron is computed and the predictor is not used
 * (Sec. 8.2: dense computation when the joint activation of a long prompt or a large batch
 * covers nearly all neurons).  Equal to pf_sparse_ffn over the list 0 .. ffn-1.
 * x [B][d] -> y [B][d]; the layer needs no predictor weights. */
pf_status pf_dense_ffn(pf_ctx *ctx, const pf_layer *layer, const float *x, int B, float *y,
                       void *stream);

/* Layer step with the dense fallback of Sec. 8.2: when density_hint -- the caller's
 * expectation of count / ffn for this step, e.g. the previous step's, or 1 for a long
 * prompt -- is at least crossover (a fraction in (0, 1]), the dense path runs and the
 * predictor is skipped; otherwise this is pf_layer_step.  The decision is taken on the host
 * before anything is launched: once the predictor has run its cost is sunk, and the sparse
 * kernels are then never slower than the dense ones.  Returns PF_EINVAL for a crossover
 * outside (0, 1] or a negative hint. */
pf_status pf_layer_step_auto(pf_ctx *ctx, const pf_layer *layer, const float *x, int B,
                             float density_hint, float crossover, float *y, void *stream);

/* Layer step that takes the dense decision of Sec. 8.2 on the DEVICE: the layer keeps a few
 * words of device state -- how many neurons the previous adaptive step of this layer saw, and
 * whether that was at least crossover * ffn.  If so this step runs dense: the predictor's
 * kernels return at once (their cost is not paid) and every neuron is listed; otherwise it is
 * pf_layer_step.  A sparse step sees the size of its predicted list; a dense step computes
 * every neuron and therefore sees the exact number of neurons whose FC1 output is non-zero
 * for some token -- which is what lets the layer fall back to the sparse path when the
 * density drops again.  Nothing is copied to the host and the same launches are enqueued in
 * both modes, so the call can be recorded into a HIP graph.  The first step of a layer is
 * sparse.  crossover: fraction in (0, 1].  Errors as pf_layer_step. */
pf_status pf_layer_step_adaptive(pf_ctx *ctx, pf_layer *layer, const float *x, int B, float crossover,
                                 float *y, void *stream);

/* The adaptive state of a layer, for inspection: host_state[0] = 1 if the next adaptive step
 * will run dense, [1] = neurons seen at the last one, [2] = 1 if the last one ran dense.
 * Synchronises with the device (a test and tuning aid, not for the token loop).  reset != 0
 * puts the layer back into its initial state afterwards.  host_state may be NULL. */
pf_status pf_layer_adaptive_state(pf_layer *layer, int32_t *host_state, int reset);

/* Activation profiler (the counting of Sec. 6.1 that fills the neuron table): counts[i] += 1
 * for every neuron i -- in the model's numbering when the layer has a neuron table -- of the
 * list the context used last (pf_layer_step, pf_layer_step_auto,
 * pf_dense_ffn; not pf_sparse_ffn, whose list is the caller's).  counts: [ffn] uint32 on the
 * device, caller-owned, zeroed by the caller before the first call.  One launch on `stream`,
 * no host synchronisation; the list holds no duplicates, so no atomics are involved. */
pf_status pf_count_activations(pf_ctx *ctx, const pf_layer *layer, uint32_t *counts, void *stream);

/* Neuron table of a layer (Sec. 5.2 neuron tables, Sec. 6.1 offline profiling): the weights
 * handed to pf_layer_create may be stored in another neuron order than the model's -- hot-first
 * from a profile, which is what a sort by activation frequency (Eq. 1 on a single memory tier)
 * gives.  stored_to_original: device array [ffn], a permutation, entry j = the model's number
 * of the neuron stored at position j; borrowed until pf_layer_destroy; NULL = identity.
 * always_on: the first always_on stored neurons (a multiple of 64, at most ffn - 64) are
 * treated as active in every step WITHOUT being predicted: the predictor's output layer
 * skips their rows (2 r bytes each) and their mask bits and scores read 1.  All internal lists
 * and masks (pf_predict, pf_ctx_last_active, the mask trace) stay in stored numbering;
 * pf_layer_active_original and pf_count_activations translate through the table.  Takes effect
 * for the calls made, and the plans created, afterwards.  Errors: PF_EINVAL (null layer,
 * always_on not a multiple of 64 or outside [0, ffn - 64]). */
pf_status pf_layer_set_neuron_table(pf_layer *layer, const int32_t *stored_to_original, int always_on);

/* The active set the context used last (as pf_ctx_last_active), in the MODEL's neuron numbering:
 * mask_words [ffn/64] uint64 (bit b of word w = original neuron 64 w + b), idx [ffn capacity]
 * int32 ascending original numbers, *count their number; all device, caller-owned, fully
 * overwritten.  Three small launches on `stream`, no host synchronisation. */
pf_status pf_layer_active_original(pf_ctx *ctx, const pf_layer *layer, uint64_t *mask_words,
                                   int32_t *idx, int32_t *count, void *stream);

/* Device pointers to the mask words, index list and count left by the last layer step on
 * this context (valid until the next compute call).  After a dense step idx / count are the
 * full list and *mask_words is NULL. */
pf_status pf_ctx_last_active(pf_ctx *ctx, const uint64_t **mask_words, const int32_t **idx,
                             const int32_t **count);

/* Look-ahead prediction (Sec. 2.1: the activations of a layer can be predicted a few layers
 * ahead, from an earlier layer's input).  With distance 1, pf_stack_step and the plans
 * created afterwards take the active set of layer l >= 1 from layer l's predictor applied to
 * the INPUT of layer l-1 (layer 0: its own input), so that the predictor of layer l and the
 * sparse kernels of layer l-1 are independent and a layer costs about max(predictor, sparse
 * FFN) instead of their sum.  A layer then runs as two launches whose block ranges play two
 * roles (hidden layer of the next predictor beside FC1; FC2 beside the next predictor's output
 * layer): stacks of fp16 layers at any batch (vector kernels up to batch 3, matrix-core
 * kernels above) and stacks of int4 layers up to batch 3.  Other stacks (mixed weight types,
 * int4 at batch >= 4, row lengths the matrix-core kernels do not take) run the predictors on a
 * second stream of the library or behind the sparse kernels of the layer before on the same
 * stream, whichever measured faster for the shape.  This changes which neurons are listed
 * (an approximation whose accuracy depends on trained predictors and is not measured here);
 * every other call is unaffected.  distance: 0 (off, the default) or 1. */
pf_status pf_ctx_set_lookahead(pf_ctx *ctx, int distance);

/* Dispatch and launch-shape options of a context (this library's own tuning surface; the
 * defaults are the measured optima and every setting computes the same function).  They take
 * effect for the calls made, and the plans created, afterwards.  value 0 restores the default
 * rule of an option unless stated otherwise.
 *   PF_OPT_FUSED            inner layers of a stack in three launches (see pf_stack_step):
 *                           0 never, 1 where measured faster (default), 2 wherever it applies
 *   PF_OPT_SEG_STRIDED      the three-launch form groups neurons g, g + ffn/64, ... into a
 *                           segment instead of 64 neighbours (for models stored hot-first): 0 / 1
 *   PF_OPT_MFMA_MIN_BATCH   batch size from which FC1 and the predictor run on the matrix
 *                           cores (default rule: 4, and 3 where d > 4096); 0 = default rule
 *   PF_OPT_HIDDEN_MFMA_MIN_ELEMS  the predictor's hidden layer joins them only above this
 *                           B * d (default 20480; every value >= 0 is taken as given)
 *   PF_OPT_UP_GRID          workgroups of the vector FC1 kernel (default 8 per CU; int4: 2)
 *   PF_OPT_MFMA_GRID        workgroups of the matrix-core FC1 kernel (default one per CU)
 *   PF_OPT_DOWN_SPLIT       row groups of FC2, 1 .. 4 (default CUs / column tiles, at most 4)
 *   PF_OPT_LOOKAHEAD_FORM   how a look-ahead stack is scheduled (see pf_ctx_set_lookahead):
 *                           0 automatic (default), 1 two launches per layer where that form
 *                           applies, 2 predictors on a second stream, 3 everything on one stream
 * Errors: PF_EINVAL for an unknown key or a value outside the stated range. */
typedef enum {
    PF_OPT_FUSED = 0,
    PF_OPT_SEG_STRIDED = 1,
    PF_OPT_MFMA_MIN_BATCH = 2,
    PF_OPT_HIDDEN_MFMA_MIN_ELEMS = 3,
    PF_OPT_UP_GRID = 4,
    PF_OPT_MFMA_GRID = 5,
    PF_OPT_DOWN_SPLIT = 6,
    PF_OPT_LOOKAHEAD_FORM = 7
} pf_option;
pf_status pf_ctx_set_option(pf_ctx *ctx, int key, int value);
pf_status pf_ctx_get_option(const pf_ctx *ctx, int key, int *value);

/* Inspection of a stack step: with a trace buffer set, pf_stack_step and the plans created
 * afterwards store the mask words every layer used -- layer l at trace + l * (max_ffn / 64)
 * words, bit b of word w = neuron 64 w + b whichever form the layer ran in -- for the layers
 * l < n_layers_capacity, with one small extra launch per layer (the compute launches are the
 * same).  trace: device buffer of n_layers_capacity * (max_ffn / 64) uint64, caller-owned;
 * NULL switches it off.  This is how a test reads the active set of every layer of the stack
 * (Sec. 5.1) without a host round trip between the layers. */
pf_status pf_ctx_set_mask_trace(pf_ctx *ctx, uint64_t *trace, int n_layers_capacity);

/* Glue of the synthetic FFN stack used for benchmarking (not in the paper): residual add
 * and scale-only RMS normalisation, x_next = s * (x + y) * sqrt(d) / ||x + y||_2 per token,
 * where s is a fixed +/-1 pattern over (batch row, column) that is all +1 for row 0: it keeps
 * the rows of a batch from aligning over the layers of a stack. */
pf_status pf_stack_glue(pf_ctx *ctx, const float *x, const float *y, int d, int B,
                        float *x_next, void *stream);

/* One decode step of a whole FFN stack: for each layer, pf_layer_step then pf_stack_glue.
 * layers: HOST array of n_layers layer handles of equal d.  x [B][d] in, x_out [B][d]
 * out (may alias x).  Up to batch 3 the layers before the last may run the same computation
 * in three launches (predictor output layer and FC1 fused per 64 neurons, FC2 over those
 * segments; no index list is built): same active sets bit for bit, FC2 summed in another
 * fixed order.  pf_ctx_last_active after a stack step refers to the last layer, which always
 * runs as pf_layer_step. */
pf_status pf_stack_step(pf_ctx *ctx, pf_layer *const *layers, int n_layers, const float *x,
                        int B, float *x_out, void *stream);

/* The same step recorded once into a HIP graph and replayed: removes per-kernel launch
 * cost from the token loop.  x and x_out are fixed at creation; each pf_plan_run reads x
 * and writes x_out.  The plan borrows ctx and the layers. */
pf_status pf_plan_create(pf_ctx *ctx, pf_layer *const *layers, int n_layers, const float *x,
                         int B, float *x_out, void *stream, pf_plan **out);
pf_status pf_plan_run(pf_plan *plan, void *stream);
void pf_plan_destroy(pf_plan *plan);

/* Per-kernel timing for measurement.  Between pf_profile_begin and pf_profile_end every
 * kernel the library launches eagerly on this context (not inside a recorded plan) is
 * timed with a pair of HIP events on its own stream, up to 32768 launches.
 * pf_profile_end waits for the recorded events (the only call here that synchronises with
 * the host) and fills one entry per kernel: name (host string), launches, summed ms.
 * stats: HOST array of `capacity` >= 16 entries; *n_out receives the number filled.
 * The events are stamped by the launch itself (hipExtLaunchKernelGGL) with the kernel's
 * start and end on its stream, so launch gaps are not part of the figures. */
typedef struct {
    const char *name;
    uint64_t launches;
    double total_ms;
} pf_kernel_stat;
pf_status pf_profile_begin(pf_ctx *ctx);
pf_status pf_profile_end(pf_ctx *ctx, pf_kernel_stat *stats, int capacity, int *n_out);

const char *pf_strerror(pf_status s);
/* Text of the last error on this context (host string, valid until the next call). */
const char *pf_last_error(const pf_ctx *ctx);
/* Library version string (host). */
const char *pf_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PF_H */
