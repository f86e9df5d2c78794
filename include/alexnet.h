/*
 * libalexnet_hip -- one AlexNet SGD training step on one MI355X (gfx950).
 *
 * C ABI of the training hot path of "Theano-based Large-Scale Visual
 * Recognition with Multiple GPUs" (arXiv 1412.2302): preprocessing of a
 * minibatch (Section 2.1), one training iteration of AlexNet (Section 2,
 * "Methods"), an inference pass (Section 3, validation error) and the
 * exchange-and-average step between two replicas (Section 2.2).
 *
 * General rules for every call
 *  - Pointers named d_* are DEVICE pointers, borrowed for the duration the
 *    handle lives (alexnet_create) or of the enqueued work (all others).  The
 *    library never allocates or frees device memory; the caller owns
 *    parameters, momentum and workspace.
 *  - `stream` is a hipStream_t (0 = the null stream).  Calls only enqueue work
 *    and return; they never synchronise the device.
 *  - Return value: ALEXNET_OK (0) or a negative ALEXNET_E* code;
 *    alexnet_last_error() returns a thread-local message for the last failure.
 *  - Canonical (external) tensor layouts are float32 NCHW activations, OIHW
 *    convolution weights and [out][in] dense weights with the flatten order
 *    (c, h, w).  The flat canonical parameter vector is: every weight tensor
 *    conv1..conv5, fc6..fc8, then every bias in the same layer order.  The
 *    library keeps its own internal layout inside d_params / d_momentum; use
 *    alexnet_set_params / alexnet_get_params to convert.
 *  - alexnet_train_step runs part of the update on a stream of the handle's
 *    own, forked from and joined back into `stream` by events inside the
 *    call: for the caller everything is ordered on `stream` as usual.
 *  - Calls on one handle, or on two handles passed to
 *    alexnet_average_replicas, must be ordered by the caller (same stream or
 *    events).  Preprocessing into slot s may overlap a training step reading
 *    the other slot.
 */
#ifndef ALEXNET_H_
#define ALEXNET_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ALEXNET_OK 0
#define ALEXNET_EINVAL (-1)   /* null pointer, bad enum, bad slot ...            */
#define ALEXNET_ESHAPE (-2)   /* configuration whose layer shapes do not work out */
#define ALEXNET_EALIGN (-3)   /* device pointer not 256-byte aligned              */
#define ALEXNET_ELABEL (-4)   /* a label outside [0, classes) was seen            */
#define ALEXNET_EHIP (-5)     /* a HIP runtime call or kernel launch failed       */
#define ALEXNET_ENOTIMPL (-6) /* feature not available in this build              */
#define ALEXNET_ENOMEM (-7)   /* workspace smaller than alexnet_query reports     */

/* alexnet_config_t.precision: arithmetic of the matrix products (convolutions and
 * dense layers).  Everything else, and every tensor in memory, stays fp32.
 * BF16 rounds both operands to bfloat16 (nearest even) as they enter the
 * multiplier and accumulates in fp32; products whose operands cannot be read
 * 16 bytes at a time (channel counts not a multiple of 4) keep fp32. */
#define ALEXNET_PRECISION_FP32 0
#define ALEXNET_PRECISION_BF16 1

/* alexnet_config_t.flags.  DIRECT_CONV keeps every convolution stage on the
 * direct implicit GEMM (see alexnet_query); unknown bits are refused with
 * ALEXNET_EINVAL. */
#define ALEXNET_FLAG_DIRECT_CONV 1

typedef struct alexnet alexnet_t; /* opaque; host memory owned by the library */

/* One convolution stage: conv -> ReLU -> [LRN] -> [3x3 stride-2 max-pool]. */
typedef struct {
  int32_t cout, k, stride, pad, groups;
  int32_t lrn;  /* 1: cross-channel response normalisation after the ReLU */
  int32_t pool; /* 1: 3x3 stride-2 max-pool (floor output size) after that */
} alexnet_conv_t;

/* Network and optimiser description (Section 2 names the layer census: five
 * convolutions, three of them pooled, two dense layers and a softmax layer;
 * every number below is the caller's). */
typedef struct {
  int32_t batch;
  int32_t in_c, crop_h, crop_w; /* network input C x H x W                     */
  int32_t raw_h, raw_w;         /* stored picture size; crop offsets are drawn */
                                /* from [0, raw - crop]                        */
  alexnet_conv_t conv[5];
  int32_t fc[3];                /* dense output widths; fc[2] = classes        */
  int32_t lrn_n;                /* s = k + alpha * sum over n channels of a^2; */
  float lrn_k, lrn_alpha, lrn_beta; /* b = a * s^-beta (alpha not divided by n) */
  float dropout_p;              /* drop probability after fc6 and fc7          */
  float lr, momentum, weight_decay; /* v <- mu v - lr (g + wd w); w <- w + v;  */
                                /* wd applies to weights, not to biases        */
  int32_t precision;            /* ALEXNET_PRECISION_*                         */
  int32_t flags;                /* ALEXNET_FLAG_* or'ed together; 0 = defaults */
  uint64_t seed;                /* keys the crop / flip / dropout generator    */
} alexnet_config_t;

/* Sizes the caller must allocate: n_params floats each for parameters and
 * momentum, and workspace_bytes of scratch.  Host-only; no GPU work.
 *
 * In fp32, convolution stages with 3x3 or 5x5 kernels, unit stride and
 * channel counts per group that are multiples of 4 (conv2-5 of Section 2's
 * network) are computed through F(4x4, 3x3) tile transforms (a 5x5 kernel as
 * four 3x3 sub-kernels): the same result up to rounding order with 2.6x fewer
 * multiplications, at the price of more workspace.  ALEXNET_FLAG_DIRECT_CONV
 * in cfg->flags keeps those stages on the direct implicit GEMM; the flag is
 * part of the configuration, so alexnet_query and alexnet_create size and lay
 * out the workspace for the same choice. */
int alexnet_query(const alexnet_config_t* cfg, size_t* n_params, size_t* workspace_bytes);

/* Builds a replica over caller-owned device memory (Section 2.2: replicas are
 * created identically by giving them the same parameters).  d_params and
 * d_momentum hold n_params floats each in the library's internal layout and
 * d_workspace holds workspace_bytes; all three must be 256-byte aligned and
 * outlive the handle.  Contents of d_params / d_momentum are not touched
 * (fill them with alexnet_set_params / alexnet_set_momentum).  The workspace
 * is cleared on `stream`. */
int alexnet_create(const alexnet_config_t* cfg, void* d_params, void* d_momentum, void* d_workspace,
                   size_t workspace_bytes, void* stream, alexnet_t** out);
void alexnet_destroy(alexnet_t* net);

/* Section 2.1 footnote: subtract the mean image, cut a random crop_h x crop_w
 * window and mirror it at random.  d_raw: uint8 [batch][in_c][raw_h][raw_w];
 * d_mean: float32 [in_c][raw_h][raw_w].  The mean is taken at the source
 * pixel, then the window is cut, then mirrored.  Offsets and the flip bit of
 * picture n are functions of (seed, step, n) only.  Writes input slot `slot`
 * (0 or 1) inside the workspace. */
int alexnet_preprocess(alexnet_t* net, const uint8_t* d_raw, const float* d_mean, uint64_t step,
                       int32_t slot, void* stream);

/* Loads an already preprocessed float32 NCHW batch into input slot `slot`. */
int alexnet_set_input(alexnet_t* net, const float* d_input_nchw, int32_t slot, void* stream);

/* One training iteration on the batch in `slot` (Section 2: forward, backward,
 * update): conv/ReLU/LRN/pool stack, fc6/fc7 with dropout masks keyed by
 * `step`, fc8, softmax cross-entropy averaged over the batch, gradients of
 * every parameter, momentum/weight-decay update in place.  d_labels: int32
 * [batch] in [0, classes); a label out of range is clamped for the arithmetic
 * and raises a sticky flag reported by alexnet_check().  d_loss: one float32,
 * written on the device. */
int alexnet_train_step(alexnet_t* net, int32_t slot, const int32_t* d_labels, uint64_t step, float* d_loss,
                       void* stream);

/* Forward + backward only: as alexnet_train_step without the update.  The
 * gradients stay readable through alexnet_get_grads. */
int alexnet_forward_backward(alexnet_t* net, int32_t slot, const int32_t* d_labels, uint64_t step,
                             float* d_loss, void* stream);

/* The update alone, from the gradients left by the last backward pass. */
int alexnet_apply_update(alexnet_t* net, void* stream);

/* Inference (Section 3, validation): d_input_nchw float32
 * [batch][in_c][crop_h][crop_w] already preprocessed; d_probs float32
 * [batch][classes].  No dropout; fc6/fc7 activations are scaled by
 * (1 - dropout_p). */
int alexnet_forward(alexnet_t* net, const float* d_input_nchw, float* d_probs, void* stream);

/* Section 2.2, steps 2 and 3 for two replicas living on the same GPU: after
 * the call both replicas hold 0.5*(a+b) for every weight, bias and momentum
 * value, bit-identical on both sides.  Configurations must match. */
int alexnet_average_replicas(alexnet_t* a, alexnet_t* b, void* stream);

/* A variant of the Section 2.2 exchange that sends gradients instead of
 * parameters: from the gradients left by alexnet_forward_backward on each
 * replica, g = 0.5*(g_a + g_b), then each replica applies
 * v <- mu v - lr (g + wd w), w <- w + v to its own weights and momentum (one
 * pass over both).  The rule is affine in g, so replicas that hold the same w
 * and v end up bit-identical and equal, up to rounding, to updating separately
 * and then calling alexnet_average_replicas.  Configurations must match. */
int alexnet_average_gradients_update(alexnet_t* a, alexnet_t* b, void* stream);

/* Validation (Section 3).  alexnet_preprocess_center writes the mean-subtracted
 * central crop (offsets floor((raw - crop) / 2), not mirrored) of d_raw into
 * input slot `slot`.  alexnet_validate runs the inference pass (as
 * alexnet_forward) on that slot and adds, for each of the nk <= 8 host values
 * ks[j] >= 1, the number of pictures whose label is among the ks[j] highest
 * scores to d_counts[j] (device int32; the caller zeroes them; a label counts
 * when fewer than k classes score strictly higher).  Labels as in
 * alexnet_train_step. */
int alexnet_preprocess_center(alexnet_t* net, const uint8_t* d_raw, const float* d_mean, int32_t slot, void* stream);
int alexnet_validate(alexnet_t* net, int32_t slot, const int32_t* d_labels, const int32_t* ks, int32_t nk,
                     int32_t* d_counts, void* stream);

/* Loading thread of Section 2.1 (Figure 1): while the GPU trains on minibatch
 * k, a host thread brings minibatch k+1 from the stored pictures to the GPU.
 *
 * host_images (uint8 [count][in_c][raw_h][raw_w]) and host_labels (int32
 * [count]) are ordinary host memory and stand for the disk; minibatch k is
 * pictures (k*batch + i) mod count.  The caller owns, for `depth` (2..16)
 * staging sets, pinned host memory pinned_raw (depth*batch*in_c*raw_h*raw_w
 * bytes) and pinned_labels (depth*batch int32), and device memory d_raw /
 * d_labels of the same sizes; all must outlive the loader.  The thread copies
 * minibatch k into staging set k % depth and issues its host-to-device copies
 * on copy_stream, at most `depth` minibatches ahead of alexnet_loader_done.
 * copy_stream is best the side stream later given to alexnet_loader_stage:
 * a copy always precedes the preprocessing of the same minibatch there, and
 * a process then needs only four streams (default, compute, side, the
 * handle's own), which is the number of hardware queues HIP gives a process
 * by default -- a fifth stream shares a queue with one of the others and its
 * waits then hold that one up (measured: 4.6 -> 5.1 ms per step).  Null makes
 * the loader create a stream of its own.
 *
 * alexnet_loader_stage(k): k must be the next minibatch in order and at most
 * two ahead of alexnet_loader_done (there are two input slots).  Blocks the
 * calling host thread until the copies of minibatch k have been issued, then
 * enqueues on side_stream: wait for them, alexnet_preprocess(step k, slot k%2);
 * makes compute_stream wait for that, and returns the device address of the
 * minibatch's labels.  The caller then enqueues the training step of slot k%2
 * on compute_stream and calls alexnet_loader_done(k, compute_stream), which
 * lets the thread reuse that staging set once the step has run.
 * alexnet_loader_destroy stops the thread and waits for copies in flight.
 * Errors: ALEXNET_EINVAL for calls out of order, ALEXNET_EHIP if a HIP call
 * fails (also one made by the thread). */
typedef struct alexnet_loader alexnet_loader_t;
int alexnet_loader_create(alexnet_t* net, const alexnet_config_t* cfg, const uint8_t* host_images,
                          const int32_t* host_labels, int64_t count, int32_t depth, void* pinned_raw,
                          void* pinned_labels, void* d_raw, void* d_labels, void* copy_stream,
                          alexnet_loader_t** out);
int alexnet_loader_stage(alexnet_loader_t* loader, uint64_t k, const float* d_mean, void* side_stream,
                         void* compute_stream, const int32_t** d_labels_k);
int alexnet_loader_done(alexnet_loader_t* loader, uint64_t k, void* compute_stream);
int alexnet_loader_destroy(alexnet_loader_t* loader);

/* Canonical <-> internal conversion of the flat parameter / momentum /
 * gradient vectors (n_params float32 each, device memory). */
int alexnet_set_params(alexnet_t* net, const float* d_canonical, void* stream);
int alexnet_get_params(alexnet_t* net, float* d_canonical, void* stream);
int alexnet_set_momentum(alexnet_t* net, const float* d_canonical, void* stream);
int alexnet_get_momentum(alexnet_t* net, float* d_canonical, void* stream);
int alexnet_get_grads(alexnet_t* net, float* d_canonical, void* stream);

/* Intermediate tensors of the last pass, converted to canonical layout.
 * `layer` is 1..5 for convolution stages, 6..8 for dense layers. */
enum {
  ALEXNET_T_INPUT = 0,    /* float32 NCHW, `layer` = slot                          */
  ALEXNET_T_CONV_ACT = 1, /* float32 NCHW, output of the stage's ReLU              */
  ALEXNET_T_LRN = 2,      /* float32 NCHW, normalised output (stages with lrn)     */
  ALEXNET_T_POOL = 3,     /* float32 NCHW, pooled output (stages with pool)        */
  ALEXNET_T_ARGMAX = 4,   /* int32 NCHW, y_in*W_in + x_in of the winning tap       */
  ALEXNET_T_FC_ACT = 5,   /* float32 [batch][width]: fc6/fc7 after ReLU+dropout, fc8 logits */
  ALEXNET_T_CROP_X = 6,   /* int32 [batch], `layer` = slot                         */
  ALEXNET_T_CROP_Y = 7,   /* int32 [batch], `layer` = slot                         */
  ALEXNET_T_FLIP = 8,     /* int32 [batch], `layer` = slot                         */
  ALEXNET_T_DLOGITS = 9,  /* float32 [batch][classes]: (p - onehot)/batch          */
  ALEXNET_T_CONV_DACT = 10 /* float32 NCHW, gradient w.r.t. the stage's pre-ReLU output */
};
int alexnet_tensor_elems(alexnet_t* net, int32_t kind, int32_t layer, size_t* elems);
int alexnet_get_tensor(alexnet_t* net, int32_t kind, int32_t layer, void* d_out, void* stream);

/* Synchronises `stream` and reports sticky device-side conditions:
 * ALEXNET_ELABEL if a label was out of range since the last check. */
int alexnet_check(alexnet_t* net, void* stream);

/* --- single-operator entry points (used to measure and test one layer alone) ---
 * All tensors canonical float32 on the device, shapes as the stage `layer`
 * (1..5) of the handle's configuration defines them:
 *   x  [batch][Cin][H][W]     y, dy [batch][Cout][Ho][Wo]
 *   w  [Cout][Cin/groups][k][k]      b [Cout]
 * The *_nhwc variants take the library's internal channel-last activations
 * ([batch][H][W][C]) and packed weights, so that no conversion kernel is part
 * of what is timed; alexnet_pack_conv_weight produces the packed form.      */
int alexnet_conv_forward(alexnet_t* net, int32_t layer, const float* d_x, const float* d_w, const float* d_b,
                         int32_t relu, float* d_y, void* stream);
int alexnet_conv_backward_data(alexnet_t* net, int32_t layer, const float* d_dy, const float* d_w, float* d_dx,
                               void* stream);
int alexnet_conv_backward_weight(alexnet_t* net, int32_t layer, const float* d_x, const float* d_dy, float* d_dw,
                                 float* d_db, void* stream);

int alexnet_nchw_to_nhwc(const float* d_src, float* d_dst, int32_t n, int32_t c, int32_t h, int32_t w, void* stream);
int alexnet_nhwc_to_nchw(const float* d_src, float* d_dst, int32_t n, int32_t c, int32_t h, int32_t w, void* stream);
/* packed forward weights [groups][(r,s,c)][Cout/groups] and the backward-data
 * form [groups][(r,s,o)][Cin/groups]; each holds Cout*Cin/groups*k*k floats. */
int alexnet_pack_conv_weight(alexnet_t* net, int32_t layer, const float* d_w_oihw, float* d_w_fwd, float* d_w_bwd,
                             void* stream);
int alexnet_unpack_conv_weight(alexnet_t* net, int32_t layer, const float* d_w_fwd, float* d_w_oihw, void* stream);
int alexnet_conv_forward_nhwc(alexnet_t* net, int32_t layer, const float* d_x, const float* d_w_fwd,
                              const float* d_b, int32_t relu, float* d_y, void* stream);
/* d_w_fwd may be null; when given, a strided ungrouped stage is computed phase by phase from it. */
int alexnet_conv_backward_data_nhwc(alexnet_t* net, int32_t layer, const float* d_dy, const float* d_w_fwd,
                                    const float* d_w_bwd, float* d_dx, void* stream);
/* d_dw_fwd receives the gradient in the packed forward-weight layout. */
int alexnet_conv_backward_weight_nhwc(alexnet_t* net, int32_t layer, const float* d_x, const float* d_dy,
                                      float* d_dw_fwd, float* d_db, void* stream);

/* The bandwidth-bound operators alone, canonical float32 tensors, shapes of
 * stage `layer`'s convolution output [batch][Cout][Ho][Wo] (LRN, pool input)
 * and pooled output.  They stage through the handle's training buffers, so
 * they overwrite the intermediates of the last training pass.
 * LRN: b = a * (k + alpha * sum_{window} a^2)^-beta across channels; the
 * backward call returns dL/da given dL/db, multiplied by [a > 0] if relu_gate.
 * Pool: 3x3 stride 2, first maximum wins; argmax = y_in*Wo + x_in (int32). */
int alexnet_lrn_forward(alexnet_t* net, int32_t layer, const float* d_a, float* d_b, void* stream);
int alexnet_lrn_backward(alexnet_t* net, int32_t layer, const float* d_a, const float* d_db, int32_t relu_gate,
                         float* d_da, void* stream);
int alexnet_pool_forward(alexnet_t* net, int32_t layer, const float* d_x, float* d_y, int32_t* d_argmax,
                         void* stream);
int alexnet_pool_backward(alexnet_t* net, int32_t layer, const float* d_x, const float* d_dy, int32_t relu_gate,
                          float* d_dx, void* stream);
/* A stage that normalises and pools (conv1, conv2 of Section 2's network) runs both
 * in one kernel during a training step, and their adjoints, the ReLU gate and
 * the bias-gradient sums in another.  These two calls run exactly those
 * kernels alone: y = pool(lrn(a)) with the winning taps; da = gate(lrn^T(
 * pool^T(dy))) where the taps are those of the fused forward kernel on the same
 * a, and db[c] = sum of da over batch and pixels (d_db may be null; 16-byte
 * aligned otherwise).  ALEXNET_ENOTIMPL for a stage that does not take the
 * fused kernels (no LRN or no pool, or channels not a multiple of 4). */
int alexnet_lrn_pool_forward(alexnet_t* net, int32_t layer, const float* d_a, float* d_y, int32_t* d_argmax,
                             void* stream);
int alexnet_pool_lrn_backward(alexnet_t* net, int32_t layer, const float* d_a, const float* d_dy,
                              int32_t relu_gate, float* d_da, float* d_db, void* stream);
/* Dense layer `layer` (6..8) as plain matrices: x [batch][in], w [out][in],
 * y, dy [batch][out]; y = act(x w^T + b), dx = dy w, dw = dy^T x, db = sum dy. */
int alexnet_fc_forward(alexnet_t* net, int32_t layer, const float* d_x, const float* d_w, const float* d_b,
                       int32_t relu, float* d_y, void* stream);
int alexnet_fc_backward(alexnet_t* net, int32_t layer, const float* d_x, const float* d_w, const float* d_dy,
                        float* d_dx, float* d_dw, float* d_db, void* stream);
/* logits [batch][classes] -> dz = (softmax - onehot)/batch and the mean loss. */
int alexnet_softmax_xent(alexnet_t* net, const float* d_logits, const int32_t* d_labels, float* d_dz,
                         float* d_loss, void* stream);

/* alexnet_softmax_xent for callers that cannot allocate device memory or keep a
 * handle's workspace: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same kernels and same results as
 * alexnet_softmax_xent, but no handle: the per-row losses and the label flag
 * live in an array built into the library's device code (16.6 KB per GPU, held
 * until the process ends), and the call allocates nothing.
 *   d_logits [batch][classes], d_labels [batch] -> d_dz [batch][classes] =
 *   (softmax - onehot)/batch, d_loss[0] = mean loss, and, when d_bad_label is
 *   not null, d_bad_label[0] = 1 if a label was outside [0, classes) (such a
 *   label is clamped for the arithmetic), else 0.  All device pointers.
 * batch <= 4096, else ALEXNET_ENOMEM (use the handle-based call).  Every call
 * on one GPU shares that GPU's array: calls that overlap in time on one GPU
 * (different streams without ordering) race on it; calls on one stream, or
 * ordered by events, are safe, and each clears what it needs first. */
int alexnet_softmax_xent_static(const float* d_logits, const int32_t* d_labels, int32_t batch, int32_t classes,
                                float* d_dz, float* d_loss, int32_t* d_bad_label, void* stream);

/* --- per-kernel timing (measurement aid; not part of the training path) ---
 * Between alexnet_profile_begin and alexnet_profile_end every kernel the
 * calling thread launches through this library is bracketed by two HIP events
 * on the stream it is launched on.  alexnet_profile_end waits for those
 * events, writes up to `cap` entries (one per distinct kernel and layer) to
 * the HOST array `out` and the number of distinct entries to *n.  flops and
 * bytes are the algorithmic work summed over the calls (2*M*N*K per GEMM;
 * each tensor read or written once for the bandwidth-bound kernels). */
typedef struct {
  char name[48];     /* e.g. "conv2.fwd:gemm", "conv1:lrn_fwd", "sgd_update" */
  int32_t calls;
  float total_ms;
  double flops;
  double bytes;
} alexnet_prof_entry_t;
int alexnet_profile_begin(void);
int alexnet_profile_end(alexnet_prof_entry_t* out, int32_t cap, int32_t* n);

const char* alexnet_last_error(void);
/* Library version string, e.g. "alexnet-hip gfx950 fp32". Host-only. */
const char* alexnet_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ALEXNET_H_ */
