/*
 * lga.h - C ABI of the layered-gradient-accumulation layer-stack library (MI355X / gfx950).
 *
 * One GPU's share of a training step over n_mu micro-batches of a stack of identical pre-LN
 * GPT decoder layers (paper section 5 "Model": attention module + two-layer feed-forward of
 * width d_I; Table B.1 fixes the per-layer inventory at 12 d_m^2 + 13 d_m parameters, i.e.
 * biases on all four linear maps and gain + bias on both layer norms).
 *
 * Conventions for every entry point
 *  - Returns an lga_status code; nothing throws across this boundary.  A human-readable
 *    message for the last failure on the calling thread is available from lga_last_error().
 *  - All argument validation happens on the host before anything is launched.
 *  - Pointers marked "dev" are device (HBM) addresses, "host" are host addresses.
 *  - Work is enqueued on the HIP stream given in lga_config.stream (borrowed; NULL = the
 *    default stream) and the call returns without synchronising; the caller synchronises.
 *  - That stream must not be in graph capture: lga_forward_layered, lga_backward_layered, lga_forward_layer,
 *    lga_backward_layer, lga_step_mbmajor and lga_adam_step_layer ask it first and return LGA_ERR_STATE, with
 *    nothing enqueued, while it is being captured (capture of whole sweeps is not a supported use).
 *  - The caller owns x, y, dy, dx.  The library owns weights, Adam moments, gradient
 *    buffer(s), the 16-bit parameter copies, the activation checkpoints and all scratch:
 *    one arena, sized from the configuration and allocated once in lga_init_stack
 *    (section 2.5: pre-allocated contiguous buffers, one fused tensor per layer).
 *  - Pointers handed out by lga_grads / lga_params / lga_moments / lga_checkpoint are
 *    borrowed: valid until the next call that overwrites that data or lga_destroy_stack.
 *
 * Canonical parameter layout of one layer (flat fp32 vector of length p_l; matrices are
 * row-major [in, out] so that y = x W + b; W_qkv columns are [Q | K | V] and head h owns
 * columns h*d_h .. (h+1)*d_h-1 inside each of the three):
 *   ln1_g[d] ln1_b[d] W_qkv[d,3d] b_qkv[3d] W_o[d,d] b_o[d] ln2_g[d] ln2_b[d]
 *   W_1[d,d_I] b_1[d_I] W_2[d_I,d] b_2[d]
 * Gradients, moments and parameters are all exposed in this same layout.
 *
 * Activation tensors x, y, dy, dx are [n_micro, micro_batch, seq_len, d_model], contiguous,
 * of the configured dtype (float, or bfloat16 / IEEE half stored as 16-bit).
 */
#ifndef LGA_H
#define LGA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct lga_stack lga_stack; /* opaque, library-owned */

/* Activation / GEMM-input type.  Master weights, gradients and Adam moments are always fp32
 * (section 2.2: bulk of the computation in 16 bits, weights stored and updated in fp32).
 * LGA_BF16 and LGA_FP16 run the same kernels on the two 16-bit formats section 2.2 names: bfloat16 has fp32's exponent
 * range; IEEE half (5 exponent bits, largest value 65504) has three more mantissa bits and needs the gradients scaled
 * (lga_adam.loss_scale, lga_loss_scaler_update) so that they neither underflow nor overflow.  Every shape rule stated
 * below for "the 16-bit modes" holds for both. */
enum lga_dtype { LGA_FP32 = 0, LGA_BF16 = 1, LGA_FP16 = 2 };

enum lga_status {
    LGA_OK = 0,
    LGA_ERR_ARG = -1,   /* NULL pointer, layer index out of range, bad enum value */
    LGA_ERR_SHAPE = -2, /* configuration the kernels do not support (see lga_init_stack) */
    LGA_ERR_OOM = -3,   /* device allocation failed */
    LGA_ERR_STATE = -4, /* call sequence violated (backward before forward, ...) */
    LGA_ERR_HIP = -5    /* HIP runtime error (no device, launch failure) */
};

/* Work the library may run on a second stream of its own (lga_config.overlap). */
enum lga_overlap { LGA_OVERLAP_NONE = 0, LGA_OVERLAP_RESTORE = 1, LGA_OVERLAP_ADAM = 2 };

/* Which positions a position attends to (lga_config.attention).  The benchmark workloads are causal decoders; the
 * paper's own model (section 5, "Model") is an encoder, whose positions attend to their whole sequence. */
enum lga_attention { LGA_ATTN_CAUSAL = 0, LGA_ATTN_FULL = 1 };

/* Order in which (layer, micro-batch) pairs are visited. */
enum lga_order { LGA_ORDER_LAYERED = 0, LGA_ORDER_MICROBATCH_MAJOR = 1 };

typedef struct lga_config {
    int32_t n_layers;     /* d_l  >= 1 */
    int32_t d_model;      /* d_m */
    int32_t n_heads;      /* d_a; d_h = d_model / n_heads */
    int32_t d_ff;         /* d_I (4 * d_model in the paper's models) */
    int32_t seq_len;      /* d_s */
    int32_t micro_batch;  /* b_mu: sequences per micro-batch */
    int32_t n_micro;      /* n_mu: micro-batches per step */
    int32_t dtype;        /* enum lga_dtype */
    int32_t group;        /* micro-batches handed to each kernel launch together (1..n_micro,
                             must divide n_micro).  Only the layered order can use > 1: it
                             contracts weight-gradient GEMMs over the concatenated tokens. */
    int32_t retain_grads; /* 1: one fp32 gradient buffer per layer (needed by the micro-batch-major
                             order and by unfused Adam when n_layers > 1); 0: a single layer-sized
                             buffer, reused layer after layer (appendix C.3: gradient storage made
                             negligible by updating a layer's weights at once) */
    int32_t wgrad_groups; /* 16-bit modes, layered order: consecutive groups of a layer whose weight-gradient
                             GEMMs are merged into one that contracts over all their tokens (their
                             transposed operands are kept side by side until then: 2 (2 d_ff + 8 d_model)
                             bytes per token, counted by lga_arena_bytes).  The sum over micro-batches then happens in
                             the GEMM's k loop instead of by read-modify-write of the fp32 buffer.
                             1 = no merging, 0 = automatic (as many as keep those operand buffers within
                             a quarter of the rest of the arena), at most n_micro / group. */
    int32_t param_buffers; /* 16-bit modes: how many layers' 16-bit parameter copies are kept (figure 2, table C.1:
                             parameter buffers).  0 = one per layer: nothing is ever restored, every Adam step
                             rewrites its layer's copies.  With fewer, layer l uses buffer l % param_buffers and
                             its fp32 masters are cast again ("restore") whenever another layer has used that
                             buffer since: once per layer and pass in the layered order, once per layer, pass
                             and micro-batch in the micro-batch-major order.  Results do not depend on it. */
    int32_t overlap;      /* bits of enum lga_overlap.  If any is set the library creates a second stream (default
                             priority) and runs on it, beside the layer sweeps on `stream`:
                             LGA_OVERLAP_RESTORE  the restore of the next layer's 16-bit parameters while the
                                                  current layer's sweep runs (param_buffers < n_layers; table C.1);
                             LGA_OVERLAP_ADAM     each layer's fused Adam step of lga_backward_layered while the
                                                  next layer's backward sweep runs; needs a second gradient
                                                  buffer when retain_grads = 0, so two layers' gradients stay
                                                  readable afterwards.
                             Every entry point still returns with all its work ordered on `stream`: a caller that
                             synchronises `stream` sees everything finished.  Results do not depend on it. */
    int32_t attention;    /* enum lga_attention: LGA_ATTN_CAUSAL (0) decoder, LGA_ATTN_FULL encoder (no mask) */
    int32_t offload_checkpoints; /* 1: the layer-boundary activations (activation checkpoints, section 2.5) live in
                             pinned host memory that the library allocates; the device keeps two boundary-sized
                             slots (appendix C.5, "CPU-GPU transfers": checkpoint offload).  In the layered order each
                             boundary crosses the bus once per pass as one transfer of all micro-batches, on a second
                             stream of the library's own (default priority): to the host beside the next layer's
                             forward sweep, back beside the previous layer's backward sweep.  lga_checkpoint then
                             returns host addresses.  Not available to lga_step_mbmajor.  Results do not depend
                             on it.  0: every boundary stays on the device. */
    float ln_eps;         /* LayerNorm epsilon, inside the root (1e-5 in the benchmarks) */
    void *stream;         /* hipStream_t, borrowed; NULL = default stream */
} lga_config;

/* Adam hyper-parameters (section 5 "Training": Adam assumed; Kingma-Ba form with bias
 * correction, no weight decay, eps added to sqrt(v_hat)).  step is t >= 1.
 * Gradient scaling (section 2.2: with half precision the gradients are scaled dynamically against underflow and
 * overflow).  The caller multiplies the output gradient dy by loss_scale before the backward pass; every Adam step
 * then divides the accumulated fp32 gradient by loss_scale before using it (0 and 1 both mean no scaling, and leave
 * the arithmetic exactly as without it).  lga_grads keeps returning the scaled gradient.
 * skip_nonfinite = 1: before a layer is updated its accumulated gradient is tested for infinities and NaNs; if it
 * holds any, that layer's update is left out as a whole - parameters, moments and 16-bit copies keep their values -
 * and the layer is reported by lga_nonfinite_layers.  With the per-layer update fused into the layer-major backward
 * pass the decision is per layer by necessity: layers above the one whose gradient overflowed have already been
 * updated, and every layer below it receives the non-finite activation gradient and is skipped too.  A caller that
 * wants all-or-nothing steps sets retain_grads, runs the backward pass unfused, asks lga_grads_nonfinite, and only
 * when that reports no layer calls lga_adam_step_layer for every layer.
 * Consequence for the step count: after a fused backward pass in which some layers were left out, the layers above
 * them HAVE taken update number `step` (moments advanced, bias correction of `step` applied) and the others have
 * not.  The library keeps no per-layer count.  A caller that backs the scale off and repeats the pass with the same
 * `step` gives the already updated layers a second update under that same bias correction; one that wants every
 * layer to see each step number exactly once reads lga_nonfinite_layers, keeps a count per layer, and drives the
 * repeat through lga_backward_layer, which takes its own lga_adam per layer (or uses the unfused path above). */
typedef struct lga_adam {
    float lr, beta1, beta2, eps;
    int32_t step;
    float loss_scale;       /* 0 or 1: none */
    int32_t skip_nonfinite; /* 0 or 1 */
} lga_adam;

/* Dynamic loss scale, host side (section 2.2; the usual rule of mixed precision training: back off at once when
 * a step overflowed, grow again after growth_interval steps in a row that did not).
 *   overflowed != 0:  scale = max(scale * backoff, min_scale), good_steps = 0
 *   else:             good_steps += 1; when it reaches growth_interval: scale = min(scale * growth, max_scale),
 *                     good_steps = 0
 * Typical: scale 65536, growth 2, backoff 0.5, growth_interval 2000, min_scale 1, max_scale 2^24.
 * LGA_ERR_ARG unless scale > 0, growth >= 1, 0 < backoff <= 1, growth_interval >= 1, 0 < min_scale <= max_scale,
 * good_steps >= 0.  Touches no device. */
typedef struct lga_loss_scaler {
    float scale, growth, backoff, min_scale, max_scale;
    int32_t growth_interval, good_steps;
} lga_loss_scaler;
int lga_loss_scaler_update(lga_loss_scaler *scaler, int32_t overflowed);

/* Create a stack.
 *  cfg          host, copied.
 *  host_params  host, n_layers * p_l floats, layer after layer in the canonical layout; copied.
 *               NULL: weights are filled on the device by a counter-based generator
 *               (matrices ~ N(0, 0.02^2), gains 1, biases 0), for throughput runs at sizes where a
 *               host copy is impractical.
 *  out          host, receives the handle.
 * Adam moments start at zero.  The 16-bit parameter copy of every layer is produced here
 * (section 2.5: parameters are converted to 16 bits before use) and refreshed by each Adam step.
 * LGA_ERR_SHAPE if any size is < 1, d_model % n_heads != 0, n_micro % group != 0, or, in the 16-bit modes,
 * d_h % 8 != 0, d_model % 8 != 0 or d_ff % 8 != 0, or if a leading dimension of a GEMM operand would exceed
 * 2 097 151 elements (3 d_model, d_ff, group * micro_batch * seq_len + 64, and with an explicit wgrad_groups that
 * many groups' tokens + 64; the automatic wgrad_groups stays within it).  Head sizes up to 160 have MFMA attention kernels in the 16-bit modes
 * (built for 32, 64, 96, 128, 160; sizes in between run in the next larger one).  Larger head sizes (table B.1's
 * X_[x] family has d_h = 2 x) run an attention built from batched GEMMs over the heads when seq_len is a multiple of 8
 * (at most 32768); the arena then holds one sequence's score matrices, 12 seq_len^2 bytes per head for as many
 * heads as fit 4 GiB.  Otherwise, and in the fp32 mode, a one-wavefront-per-position kernel is used that is meant
 * for checking, not for speed, and limits seq_len (2 seq_len + 2 d_h <= 15000).  LGA_ERR_OOM if the arena does not
 * fit. */
int lga_init_stack(const lga_config *cfg, const float *host_params, lga_stack **out);

void lga_destroy_stack(lga_stack *stack);

/* Layer-major forward (section 3): for each layer, every micro-batch group goes through it
 * before the next layer starts; only layer-boundary activations (the checkpoints) are kept.
 *  x  dev, in,  [n_micro, micro_batch, seq_len, d_model]
 *  y  dev, out, same shape; may be NULL (the output stays readable through lga_checkpoint). */
int lga_forward_layered(lga_stack *stack, const void *x, void *y);

/* Layer-major backward (section 3; recompute inside the layer from its checkpoint, section 2.5).
 * From the last layer down: every micro-batch group is recomputed and back-propagated through
 * layer l, its weight gradients summed in fp32 into layer l's gradient buffer, and - if fused is
 * not NULL - Adam is applied to layer l before layer l-1 starts (appendix C.3).
 *  dy     dev, in,  gradient of the loss w.r.t. the stack output
 *  dx     dev, out, gradient w.r.t. the stack input; may be NULL
 *  fused  host, Adam hyper-parameters, or NULL to leave the gradients for lga_adam_step_layer.
 * LGA_ERR_STATE if no forward pass precedes it, or if fused == NULL, retain_grads == 0 and
 * n_layers > 1 (all but the last-computed gradient would be lost). */
int lga_backward_layered(lga_stack *stack, const void *dy, void *dx, const lga_adam *fused);

/* One Adam update of layer `layer` from its accumulated gradient; refreshes its 16-bit copy.
 * LGA_ERR_STATE if that gradient is not (or no longer) available. */
int lga_adam_step_layer(lga_stack *stack, int32_t layer, const lga_adam *adam);

/* Borrow the accumulated fp32 gradient of a layer (canonical layout, *count = p_l).
 * LGA_ERR_STATE if not available (never computed, or its buffer was reused by a later layer). */
int lga_grads(lga_stack *stack, int32_t layer, const float **dev_ptr, size_t *count);

/* Borrow the fp32 master parameters / Adam moments of a layer (canonical layout).
 * The moment pointers are writable so that a caller can restore optimizer state. */
int lga_params(lga_stack *stack, int32_t layer, const float **dev_master, size_t *count);
int lga_moments(lga_stack *stack, int32_t layer, float **dev_m, float **dev_v, size_t *count);

/* Borrow boundary activation `boundary` (0 = stack input ... n_layers = stack output) for all
 * micro-batches: [n_micro, micro_batch, seq_len, d_model] of the configured dtype.  A device address, or with
 * offload_checkpoints a pinned host address (a valid source for hipMemcpy with hipMemcpyDefault); either way the
 * data is complete once the stack's stream has been synchronised after the call that produced it. */
int lga_checkpoint(lga_stack *stack, int32_t boundary, const void **dev_ptr, size_t *bytes);

/* The comparison order (section 2.5, standard gradient accumulation): each micro-batch goes
 * through the whole stack forward and backward before the next; gradients accumulate in
 * per-layer fp32 buffers with beta = 1; Adam (if adam != NULL) runs for all layers at the end.
 * Same kernels as the layered calls.  Requires retain_grads == 1 and group == 1. */
int lga_step_mbmajor(lga_stack *stack, const void *x, const void *dy, void *y, void *dx, const lga_adam *adam);

/* Modular layer sets (section 4, modular pipeline parallelism: a device holds layers k, k + n_l, ... and each
 * layer's input arrives from another device).  One layer's share of the layer-major sweeps:
 *
 * lga_forward_layer   runs layer `layer` over all n_micro micro-batches (in groups, like lga_forward_layered).
 *                     x_in: device, [n_micro, micro_batch, seq_len, d_model] of the configured dtype; it is copied
 *                     into the layer's input checkpoint (boundary `layer`), from which the backward pass recomputes
 *                     - unless x_in already is that checkpoint's address (lga_checkpoint), then nothing is copied.
 *                     x_out: device, same shape, receives the layer's output; NULL leaves it in boundary layer + 1.
 * lga_backward_layer  recomputes the layer from its input checkpoint, back-propagates dy (device, same shape) through
 *                     it for all micro-batches, accumulates the layer's fp32 gradient and, if fused != NULL, applies
 *                     Adam to the layer at once.  dx (device, same shape, or NULL) receives the input gradient.
 *                     With fused == NULL the gradient stays readable (lga_grads, lga_adam_step_layer) until another
 *                     layer's backward reuses its buffer (retain_grads == 0: the very next one).
 *
 * Calling lga_forward_layer for layers 0 .. L-1, feeding each output to the next, and lga_backward_layer for
 * L-1 .. 0 likewise computes exactly what lga_forward_layered / lga_backward_layered compute (same kernels, same
 * order).  LGA_ERR_STATE: lga_backward_layer without a forward of that layer since its weights last changed.
 * x_in / x_out / dy / dx are caller-owned and only read / written during the call's enqueued work. */
int lga_forward_layer(lga_stack *stack, int32_t layer, const void *x_in, void *x_out);
int lga_backward_layer(lga_stack *stack, int32_t layer, const void *dy, void *dx, const lga_adam *fused);

/* Number of restores (casts of one layer's parameters into a 16-bit parameter buffer, section 2.5 /
 * figure 2) the stack has done since it was created; the initial fill is not counted.  count: host. */
int lga_restore_count(lga_stack *stack, uint64_t *count);

/* Host-only analytic model of one step (no device needed), for printing beside measured
 * counters.  order is enum lga_order.
 *  param_bytes  HBM bytes of parameter traffic: 16-bit weight reads by the forward, recompute and
 *               input-gradient GEMM families per group, plus Adam's read of w, m, v and write of
 *               w, m, v, the 16-bit copy and the transposed 16-bit copy of the matrices, plus - with
 *               param_buffers < n_layers - the restores of a steady-state step (figure 2: constant in
 *               n_micro for the layered order, proportional to it for the micro-batch-major order).
 *  grad_bytes   HBM bytes of fp32 gradient-buffer traffic: read-modify-write per group (write
 *               only for a layer's first group) plus Adam's read.
 *  flops        executed flops: GEMMs 2 flop per token per parameter for forward, recompute
 *               (which skips the second feed-forward GEMM), input gradient and weight gradient
 *               (appendix C.1), plus the attention products the paper neglects (half of them with the causal mask). */
int lga_traffic_model(const lga_config *cfg, int32_t order, uint64_t *param_bytes, uint64_t *grad_bytes,
                      double *flops);

/* Bytes of device memory lga_init_stack would allocate for cfg (host arithmetic only). */
int lga_arena_bytes(const lga_config *cfg, uint64_t *bytes);

/* Bytes of pinned host memory lga_init_stack would allocate for cfg: the boundary activations when
 * offload_checkpoints is set, else 0 (host arithmetic only). */
int lga_host_bytes(const lga_config *cfg, uint64_t *bytes);

/* Which layers' most recent Adam step with skip_nonfinite = 1 found a non-finite gradient and was left out.
 *  flags  host, n_layers int32 (1 = left out), or NULL.   count  host, receives how many.
 * A layer's flag is rewritten by each of its Adam steps that has skip_nonfinite = 1 and is 0 before the first.
 * Synchronises the stack's stream. */
int lga_nonfinite_layers(lga_stack *stack, int32_t *flags, int32_t *count);

/* Tests the accumulated gradient of every layer that currently holds one (all layers after an unfused backward
 * pass with retain_grads = 1; else the one layer whose gradient lga_grads would return) for infinities and NaNs.
 *  flags  host, n_layers int32 (1 = holds a non-finite value; 0 also for layers without a gradient), or NULL.
 *  count  host, receives how many layers were flagged.
 * Changes nothing but the flags lga_nonfinite_layers reports.  Synchronises the stack's stream. */
int lga_grads_nonfinite(lga_stack *stack, int32_t *flags, int32_t *count);

/* p_l for cfg: 4 d^2 + 2 d d_I + 9 d + d_I (= 12 d^2 + 13 d when d_I = 4 d, Table B.1). */
int lga_params_per_layer(const lga_config *cfg, uint64_t *count);

/* Per-kernel timing of the library's own launches, for the benchmark's roofline figures.
 * Between lga_profile_begin and lga_profile_end every kernel launch of this library (on any stack
 * of the calling process) is bracketed by a HIP event pair on its stream.  lga_profile_end
 * synchronises the stack's stream and returns one record per kernel name, sorted by total time:
 * launches, summed event time in ms, and the summed algorithmic flops and HBM bytes of those
 * launches (each operand read once, each result written once).  out holds `capacity` records;
 * *count receives the number of distinct kernels (which may exceed capacity).
 * lga_profile_begin_only brackets only the launches whose kernel name starts with `kernel_name` (host string, copied;
 * NULL or empty: all of them) - two event records per launch are a measurable share of a step made of thousands of
 * short launches, so a benchmark that needs one kernel's times asks for that kernel alone. */
typedef struct lga_kernel_stat {
    char name[112];
    uint64_t launches;
    double ms, flops, bytes;
} lga_kernel_stat;
int lga_profile_begin(lga_stack *stack);
int lga_profile_begin_only(lga_stack *stack, const char *kernel_name);
int lga_profile_end(lga_stack *stack, lga_kernel_stat *out, int32_t capacity, int32_t *count);

const char *lga_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* LGA_H */
