/*
 * jz.h -- C ABI of libjz: the single-GPU hot path of mixed-precision CNN training
 * with LARS (Jia et al. 2018, "Highly Scalable Deep Learning Training System with
 * Mixed-Precision", Section 4.1) for AMD MI355X (gfx950).
 *
 * What the path is (Section 4.1, Fig. 2; Section 2.2's three techniques; Section 5.2):
 *   forward / backward in FP16 storage with FP32 accumulation, result rounded to
 *   FP16 before it is stored; an FP32 master copy of the weights; gradients that
 *   carry a loss scale S; weights and gradients widened to FP32 before the layer-wise
 *   adaptive rate of Eq. 1 is applied and narrowed to FP16 afterwards.
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller and 16-byte aligned.
 *     Descriptor / table pointers are HOST pointers unless said otherwise.
 *   - "fp16" means IEEE binary16 bit patterns (2 bytes per element).
 *   - Activations are NHWC, filters KRSC, conv outputs NPQK, innermost index
 *     contiguous; P = floor((H + 2*pad_h - R)/stride_h) + 1, likewise Q.
 *   - Convolution is cross-correlation (no filter flip), zero padding, dilation 1,
 *     one group.
 *   - Work is enqueued on `hip_stream` (a hipStream_t, NULL = default stream); calls
 *     return without synchronising.  Nothing is allocated or freed by the
 *     library; scratch comes from the caller's workspace `ws` (size from the matching
 *     *_workspace_bytes call; may be NULL when that size is 0).
 *   - Return value: JZ_OK or a negative JZ_ERR_* code.  Argument errors (every code but
 *     JZ_ERR_LAUNCH) are found on the host before anything is enqueued: no output and no
 *     workspace byte was touched.  JZ_ERR_LAUNCH means the HIP runtime refused a launch; an
 *     entry point made of several launches may then have left outputs and the workspace
 *     partially written.  Inf/NaN in data are not errors: they propagate per IEEE in the
 *     GEMMs, and in the LARS update they raise the overflow flag.
 *   - Outputs must not overlap inputs or the workspace (checked for the pointers
 *     given; JZ_ERR_ALIAS), except the in-place state buffers of the LARS update.
 *   - Same inputs give bit-identical outputs from run to run (no float atomics).
 */
#ifndef JZ_H_
#define JZ_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  JZ_OK = 0,
  JZ_ERR_NULL = -1,        /* a required pointer is NULL */
  JZ_ERR_SHAPE = -2,       /* non-positive dimension, empty output, pad >= filter size, bad offsets table */
  JZ_ERR_UNSUPPORTED = -3, /* valid but not implemented (e.g. a conv tensor with 2^30 or more elements) */
  JZ_ERR_WORKSPACE = -4,   /* workspace NULL or smaller than *_workspace_bytes reports */
  JZ_ERR_ALIGN = -5,       /* a device pointer is not 16-byte aligned */
  JZ_ERR_ALIAS = -6,       /* an output overlaps an input or the workspace */
  JZ_ERR_LAUNCH = -7,      /* the HIP runtime refused a launch or copy */
  JZ_ERR_NOT_PREPARED = -8 /* LARS workspace was not prepared for this parameter set */
};

enum { JZ_FWD = 0, JZ_BWD_DATA = 1, JZ_BWD_WEIGHT = 2 };

/* One convolution layer: x[N,H,W,C] (*) w[K,R,S,C] -> y[N,P,Q,K]. */
typedef struct {
  int N, H, W, C;
  int K, R, S;
  int stride_h, stride_w;
  int pad_h, pad_w;
} jz_conv_desc;

/* Scratch bytes `op` (JZ_FWD / JZ_BWD_DATA / JZ_BWD_WEIGHT) needs for this layer. */
int jz_conv2d_workspace_bytes(int op, const jz_conv_desc* desc, size_t* bytes);

/* Forward pass of one layer (Section 4.1: forward propagation in FP16, FP32 accumulate):
 *   y[n,p,q,k] = RNE16( sum_{r,s,c} x[n, p*stride_h - pad_h + r, q*stride_w - pad_w + s, c] * w[k,r,s,c] )
 * x16: in [N,H,W,C] fp16; w16: in [K,R,S,C] fp16 (the FP16 rounding of the master weights);
 * y16: out [N,P,Q,K] fp16. */
int jz_conv2d_fwd(const jz_conv_desc* desc, const void* x16, const void* w16, void* y16, void* ws, size_t ws_bytes,
                  void* hip_stream);

/* Backward pass w.r.t. the layer input (Section 4.1: backward propagation in FP16): the adjoint of the
 * forward map in x,
 *   dx[n,h,w,c] = RNE16( sum over (p,q,k,r,s) with p*stride_h - pad_h + r == h and q*stride_w - pad_w + s == w
 *                        of dy[n,p,q,k] * w[k,r,s,c] ),
 * input pixels no output reads get 0.
 * dy16: in [N,P,Q,K] fp16 (loss-scaled); w16: in [K,R,S,C]; dx16: out [N,H,W,C] fp16, fully overwritten.
 * A strided layer with a filter of more than one tap needs workspace (a repacked copy of the filter). */
int jz_conv2d_bwd_data(const jz_conv_desc* desc, const void* dy16, const void* w16, void* dx16, void* ws,
                       size_t ws_bytes, void* hip_stream);

/* Backward pass w.r.t. the filter (the weight gradients Section 4.1 hands to LARS): the adjoint in w,
 *   dw[k,r,s,c] = RNE16( sum_{n,p,q} dy[n,p,q,k] * x[n, p*stride_h - pad_h + r, q*stride_w - pad_w + s, c] ),
 * no division by N.  The sum over (n,p,q) is split across workgroups; the partial sums stay FP32 in `ws`
 * and are added in a fixed order before the single rounding to FP16 (overflow gives +-Inf, which the
 * LARS update reports through its flag).
 * x16: in [N,H,W,C]; dy16: in [N,P,Q,K]; dw16: out [K,R,S,C] fp16 -- may point into a fused gradient buffer. */
int jz_conv2d_bwd_weight(const jz_conv_desc* desc, const void* x16, const void* dy16, void* dw16, void* ws,
                         size_t ws_bytes, void* hip_stream);

/* The weight gradient together with its sum of squares.  Eq. 1 needs ||g_t|| of every tensor before the update can
 * start; taking it here, while the gradient is being written, saves the optimiser a second pass over the gradients
 * (jz_lars_mp_update_presummed below consumes it).  A sink is JZ_SUMSQ_SINK_BYTES of DEVICE memory, 128-byte aligned,
 * plus one DEVICE int: 64 accumulators 128 bytes apart, each four unsigned 64-bit counters, counter i in units of
 * 2^(20 i - 48).  A finite FP16 value is an integer multiple of 2^-24, so its square is an integer number of units of
 * 2^-48: the kernels add those integers (carried into base-2^20 digits per workgroup, one atomic integer add per digit),
 * hence the counters hold the EXACT sum of squares of the values written to dw16, whatever the order in which
 * workgroups arrive and whatever kernel plan ran (bit-identical from run to run).  sum = (c3 2^60 + c2 2^40 + c1 2^20 +
 * c0) 2^-48 with c_i the sum of counter i over the 64 accumulators.  The calls ADD to the sink (several calls may share
 * one; the caller clears it: jz_lars_begin_step does for the sinks inside a LARS workspace) and set *nonfinite = 1 if an
 * element of dw16 is +-Inf or NaN (they never clear it; the counters are then left as they were).  dw16 holds the same bits as from
 * jz_conv2d_bwd_weight / jz_gemm_fc(JZ_BWD_WEIGHT).  JZ_ERR_ALIGN / JZ_ERR_ALIAS / JZ_ERR_NULL for a bad sink. */
#define JZ_SUMSQ_SINK_BYTES 8192
typedef struct {
  void* sums;     /* DEVICE, JZ_SUMSQ_SINK_BYTES, 128-byte aligned */
  int* nonfinite; /* DEVICE */
} jz_sumsq_sink;
int jz_conv2d_bwd_weight_sumsq(const jz_conv_desc* desc, const void* x16, const void* dy16, void* dw16, void* ws,
                               size_t ws_bytes, const jz_sumsq_sink* sink, void* hip_stream);

/* jz_conv2d_bwd_weight for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc) and therefore have no workspace to pass: same kernels, same bits, with the
 * scratch (split-K partial sums, the padded copy of a small-channel layer) in a fixed array of
 * JZ_STATIC_SCRATCH_BYTES inside the library.  Every GPU the library runs on holds its own copy of that array for the
 * life of the process.  Calls nothing that allocates.  JZ_ERR_WORKSPACE when the layer needs more scratch than the
 * array holds (jz_conv2d_workspace_bytes(JZ_BWD_WEIGHT, ...) says how much); other status codes as
 * jz_conv2d_bwd_weight.  All calls on one GPU share the array: calls that may overlap in time on one GPU (different
 * streams, different threads) race on it and must be ordered by the caller; nothing in it needs clearing between
 * calls (every byte that is read was written by the same call). */
#define JZ_STATIC_SCRATCH_BYTES (64u << 20)
int jz_conv2d_bwd_weight_static(const jz_conv_desc* desc, const void* x16, const void* dy16, void* dw16, void* hip_stream);

/* Fully connected layer, the classifier GEMMs of AlexNet / ResNet-50 (Table 3's models), same
 * FP16-storage / FP32-accumulate rule.  Row-major x[batch,in], w[out,in], y[batch,out]:
 *   JZ_FWD        out16 = y  = RNE16(x  * w^T)   a16 = x  [batch,in],  b16 = w [out,in]
 *   JZ_BWD_DATA   out16 = dx = RNE16(dy * w)     a16 = dy [batch,out], b16 = w [out,in]
 *   JZ_BWD_WEIGHT out16 = dw = RNE16(dy^T * x)   a16 = dy [batch,out], b16 = x [batch,in]   */
int jz_gemm_fc_workspace_bytes(int mode, int batch, int in_features, int out_features, size_t* bytes);
int jz_gemm_fc(int mode, int batch, int in_features, int out_features, const void* a16, const void* b16, void* out16,
               void* ws, size_t ws_bytes, void* hip_stream);

/* jz_gemm_fc(JZ_BWD_WEIGHT, ...) with the gradient's sum of squares added to a sink (see jz_conv2d_bwd_weight_sumsq). */
int jz_gemm_fc_bwd_weight_sumsq(int batch, int in_features, int out_features, const void* dy16, const void* x16, void* dw16,
                                void* ws, size_t ws_bytes, const jz_sumsq_sink* sink, void* hip_stream);

/* ---- the same four operations in single precision (Section 5.4, Table 9: the FP32 side of the paper's FP32 versus
 * mixed-precision throughput comparison) --------------------------------------------------------------------------
 * FP32 storage, FP32 products and sums (v_mfma_f32_32x32x2_f32), no rounding to FP16 anywhere: same definitions, same
 * layouts (NHWC / KRSC / NPQK), same GEMM view, same conventions and status codes as the FP16 entry points above, with
 * float tensors (DEVICE, 16-byte aligned).  Split reductions leave FP32 partial sums in `ws` and are added in index
 * order (deterministic).  Meant as the baseline the mixed-precision path is compared with: one kernel family sized
 * for the FP32 matrix peak, no table of tuned variants. */
int jz_conv2d_f32_workspace_bytes(int op, const jz_conv_desc* desc, size_t* bytes);
int jz_conv2d_fwd_f32(const jz_conv_desc* desc, const float* x32, const float* w32, float* y32, void* ws, size_t ws_bytes,
                      void* hip_stream);
int jz_conv2d_bwd_data_f32(const jz_conv_desc* desc, const float* dy32, const float* w32, float* dx32, void* ws,
                           size_t ws_bytes, void* hip_stream);
int jz_conv2d_bwd_weight_f32(const jz_conv_desc* desc, const float* x32, const float* dy32, float* dw32, void* ws,
                             size_t ws_bytes, void* hip_stream);
int jz_gemm_fc_f32_workspace_bytes(int mode, int batch, int in_features, int out_features, size_t* bytes);
int jz_gemm_fc_f32(int mode, int batch, int in_features, int out_features, const float* a32, const float* b32, float* out32,
                   void* ws, size_t ws_bytes, void* hip_stream);

/* ---- mixed-precision LARS update (Section 4.1, Eq. 1, Fig. 2) -------------------------------------------- */

enum {
  JZ_PARAM_WEIGHT_DECAY = 1, /* tensor is regularised (Eq. 2); clear for bias and batch-norm gamma/beta (Section 4.2) */
  JZ_PARAM_LARS = 2,         /* tensor uses the local rate of Eq. 1; clear = plain momentum SGD (rho = 1) */
  JZ_PARAM_GRAD_PRESUMMED = 4 /* the kernel that produces this tensor's gradient also leaves its sum of squares in the
                                 tensor's sink (jz_lars_sumsq_sink): jz_lars_grad_sumsq leaves the tensor out.  Ignored by
                                 jz_lars_mp_update[_dyn], which read every gradient themselves. */
};

typedef struct {
  float lr;           /* gamma of Eq. 1: global learning rate */
  float momentum;     /* m; the paper's equations carry none, 0 reproduces them */
  float weight_decay; /* lambda of Eq. 2 */
  float trust_coef;   /* eta of Eq. 1, the LARS coefficient (0.001 in Section 5.2) */
  float loss_scale;   /* S > 0: the gradients in grad16 are S times the true ones */
} jz_lars_hparams;

/* All trainable tensors of a model fused into flat buffers (the fused buffer of Section 4.3's tensor
 * fusion, reused as the optimiser's layout).  Tensor t occupies elements [offsets[t], offsets[t+1]). */
typedef struct {
  int64_t num_tensors;    /* T >= 0 */
  const int64_t* offsets; /* HOST [T+1], offsets[0] = 0, non-decreasing; offsets[T] = P */
  const uint8_t* flags;   /* HOST [T], JZ_PARAM_* bits */
  float* master_w;        /* DEVICE [P] fp32 master weights, updated in place */
  float* momentum;        /* DEVICE [P] fp32 momentum buffer, updated in place */
  const void* grad16;     /* DEVICE [P] fp16 gradients, loss-scaled, read only */
  void* weight16;         /* DEVICE [P] fp16 weights for the next forward pass, written */
} jz_param_set;

/* Bytes of device workspace the update needs for this table (depends on offsets only). */
int jz_lars_workspace_bytes(const jz_param_set* ps, size_t* bytes);

/* Writes the tensor/chunk tables for `ps` into `ws` (a blocking host-to-device copy on `hip_stream`).
 * Call once per parameter-set layout; `ws` must then be kept intact and passed to every update.
 * The workspace also carries state from one update to the next: while an update writes the new master weights it
 * accumulates each tensor's sum of squares, so the next update does not have to read the weights to get ||w_t||.
 * Consequently, if master_w is written by anything other than jz_lars_mp_update (initialisation, a checkpoint
 * restore), call jz_lars_prepare again before the next update; it discards the carried sums. */
int jz_lars_prepare(const jz_param_set* ps, void* ws, size_t ws_bytes, void* hip_stream);

/* One optimiser step over every tensor:
 *   found_inf = any element of grad16 is +-Inf or NaN (anywhere in [0,P));  if so nothing else is written.
 *   per tensor t:  g = float(g16) / S ;  rho_t = eta * ||w_t|| / ||g_t||  (Eq. 1; 1 if a norm is 0 or the LARS bit
 *                  is clear) ;  lambda_t = weight_decay if the decay bit is set else 0
 *   per element:   v <- m*v + lr * rho_t * (g + lambda_t * w) ;  w <- w - v ;  w16 <- RNE16(w)      (FP32 arithmetic,
 *                  norms accumulated in FP64 in a fixed order)
 * found_inf_dev: DEVICE int, set to 0 or 1; valid once the stream has been synchronised.
 * Returns JZ_ERR_NOT_PREPARED if `ws` was not prepared for this table by jz_lars_prepare (the host keeps a
 * checksum of the offsets/flags per prepared workspace pointer).  The kernels check the table header in `ws`
 * again on the device before anything is written; if it does not match, *found_inf_dev = -1 and no state changes. */
int jz_lars_mp_update(const jz_param_set* ps, const jz_lars_hparams* hp, int* found_inf_dev, void* ws,
                      size_t ws_bytes, void* hip_stream);

/* Dynamic loss scaling around the LARS update.  Section 4.1 multiplies the loss by a scale S so that small gradients
 * survive FP16 and divides by S before the update; Section 5.3 calls this required at large batch sizes and gives no
 * policy.  The policy here is the usual one: an update that found Inf/NaN is skipped (as jz_lars_mp_update does) and
 * S <- max(S * backoff_factor, min_scale); after growth_interval clean updates in a row S <- min(S * growth_factor,
 * max_scale).  S lives in DEVICE memory, so a training loop never has to read the overflow flag back: the next
 * backward pass multiplies its loss gradient by state->scale on the device.
 *   jz_loss_scale_init:    writes {initial_scale, 0} to *state_dev (DEVICE, 8-byte aligned) on the stream.
 *   jz_lars_mp_update_dyn: jz_lars_mp_update with S read from state_dev->scale on the device (hp->loss_scale is
 *                          ignored), followed by the controller step above (inside the last kernel of the update: no
 *                          further launch; a call whose workspace header does not match, found_inf = -1, leaves the
 *                          state as it was).  state_dev must not overlap any other buffer.  Everything else (workspace, prepare,
 *                          found_inf_dev, status codes) as for jz_lars_mp_update; JZ_ERR_SHAPE for a policy with
 *                          growth_factor < 1, backoff_factor outside (0, 1], growth_interval < 1 or min_scale > max_scale. */
typedef struct {
  float scale;    /* S */
  int good_steps; /* clean updates since S last changed */
} jz_loss_scale_state;
typedef struct {
  float growth_factor;  /* >= 1, e.g. 2 */
  float backoff_factor; /* in (0, 1], e.g. 0.5 */
  int growth_interval;  /* >= 1, e.g. 2000 */
  float min_scale;      /* > 0 */
  float max_scale;      /* >= min_scale */
} jz_loss_scale_policy;
int jz_loss_scale_init(jz_loss_scale_state* state_dev, float initial_scale, void* hip_stream);
int jz_lars_mp_update_dyn(const jz_param_set* ps, const jz_lars_hparams* hp, const jz_loss_scale_policy* policy,
                          jz_loss_scale_state* state_dev, int* found_inf_dev, void* ws, size_t ws_bytes, void* hip_stream);

/* The update in ONE launch, for a training step whose gradient norms are taken where the gradients are produced
 * (Section 4.1 / Eq. 1; jz_conv2d_bwd_weight_sumsq and jz_gemm_fc_bwd_weight_sumsq above).  The gradient is then read
 * once, by the update itself: 20 bytes per parameter move instead of 22, and the two launches in front of the update
 * (reduce, per-tensor rates) disappear from the end of the step.  One step, all on streams ordered as listed:
 *
 *   jz_lars_begin_step        after the previous update, before the first gradient of this step: clears every tensor's
 *                             sink, adds up the sums of squares of the master weights that the previous update left
 *                             (first step after jz_lars_prepare: squares the weights themselves), and, when state_dev
 *                             is not NULL, notes the loss scale S the step runs with.  One small launch.
 *   jz_lars_sumsq_sink        (host only, no launch) the sink of tensor t inside `ws`, to be handed to the kernel that
 *                             produces that tensor's gradient.
 *   jz_lars_grad_sumsq        the sum of squares and overflow check of those tensors in [first, first + num) whose
 *                             JZ_PARAM_GRAD_PRESUMMED bit is clear, read from ps->grad16: for the tensors no producing
 *                             kernel covers (batch-norm scale and shift, bias).  Any time after those gradients exist.
 *                             ADDS to the sinks: call it once per tensor and step.
 *   jz_lars_mp_update_presummed[_dyn]   the update of jz_lars_mp_update[_dyn]: same arithmetic per element, same flag,
 *                             same skip rule, same loss-scale controller, with ||g_t||^2 from the sinks and ||w_t||^2
 *                             from jz_lars_begin_step.  Every tensor's sink must hold exactly the sum of squares of that
 *                             tensor's slice of grad16 (and *nonfinite != 0 iff the slice has an Inf / NaN).
 *                             JZ_ERR_NOT_PREPARED unless jz_lars_begin_step ran on this workspace since the last presummed
 *                             update, with the same state_dev (NULL for the fixed-scale call).
 *
 * Both update paths can be mixed on one workspace (each leaves the carried sums of squares of the weights valid for
 * the other).  Bit-identical from run to run; the rates can differ from jz_lars_mp_update's in the last FP32 bit
 * (the same FP64 partial sums are added as integers here, left to right there). */
int jz_lars_begin_step(const jz_param_set* ps, const jz_loss_scale_state* state_dev, void* ws, size_t ws_bytes, void* hip_stream);
int jz_lars_sumsq_sink(const jz_param_set* ps, void* ws, size_t ws_bytes, int64_t tensor, jz_sumsq_sink* sink);
int jz_lars_grad_sumsq(const jz_param_set* ps, int64_t first_tensor, int64_t num_tensors, void* ws, size_t ws_bytes,
                       void* hip_stream);
int jz_lars_mp_update_presummed(const jz_param_set* ps, const jz_lars_hparams* hp, int* found_inf_dev, void* ws,
                                size_t ws_bytes, void* hip_stream);
int jz_lars_mp_update_presummed_dyn(const jz_param_set* ps, const jz_lars_hparams* hp, const jz_loss_scale_policy* policy,
                                    jz_loss_scale_state* state_dev, int* found_inf_dev, void* ws, size_t ws_bytes,
                                    void* hip_stream);

/* Backward-data of a convolution together with the backward pass of the batch normalization + ReLU that produced the
 * convolution's input (Section 4.2's layer; the counterpart of jz_conv2d_bn_relu_fwd):  y = relu(bn(c)) was the input of
 * this convolution in the forward pass.  One call computes
 *   dz      = jz_conv2d_bwd_data(desc, dy16, w16)              the gradient w.r.t. y, [N,H,W,C]
 *   dc, dgamma, dbeta = jz_bn_relu_bwd(rows = N*H*W, C, x = bn_x16 (= c), y = bn_y16, dy = dz, relu = 1)
 * with the statistics of the normalization's backward (sum g, sum g x^ over g = dz where y > 0) taken in the
 * convolution's epilogue, while the dz tile is on chip, when the convolution's kernel allows it (not split, unit stride
 * or no scatter form, C a multiple of 8); otherwise the statistics pass runs as in jz_bn_relu_bwd.  dz16 holds the same
 * bits as from jz_conv2d_bwd_data; bn_dx16 / dgamma16 / dbeta16 meet jz_bn_relu_bwd's within the rounding of FP32 sums
 * taken in another (fixed, deterministic) order.  bn_y16 is the tensor the forward pass fed to this convolution; bn_x16
 * the normalization's input; gamma, save_mean, save_invstd as for jz_bn_relu_bwd.  Outputs must not overlap anything.
 * Workspace: jz_conv2d_bwd_data_bn_relu_bwd_workspace_bytes.  Status codes as for the two calls it replaces. */
int jz_conv2d_bwd_data_bn_relu_bwd_workspace_bytes(const jz_conv_desc* desc, size_t* bytes);
int jz_conv2d_bwd_data_bn_relu_bwd(const jz_conv_desc* desc, const void* dy16, const void* w16, const void* bn_x16,
                                   const void* bn_y16, const float* gamma, const float* save_mean, const float* save_invstd,
                                   void* dz16, void* bn_dx16, void* dgamma16, void* dbeta16, void* ws, size_t ws_bytes,
                                   void* hip_stream);

/* The same for a convolution whose input was the output of a residual block, y_out = relu(bn(x) + shortcut) (Section 4.2's
 * layer at the end of a bottleneck block): this convolution's backward-data result is one contribution to the gradient of
 * y_out, dyb16 the other (the shortcut consumer's; may be NULL).  One call computes
 *   g16 = RNE16(RNE16(jz_conv2d_bwd_data(desc, dy16, w16)) [+ dyb16]) where y_out16 > 0, else 0        [N,H,W,C]
 *   bn_dx16, dgamma16, dbeta16 = jz_bn_relu_bwd(rows = N*H*W, C, x = bn_x16, dy = g16, relu = 0)
 * i.e. jz_conv2d_bwd_data followed by jz_bn_bwd_block_end, without the convolution's result ever being stored: the
 * epilogue reads the matching tiles of dyb16, y_out16 and bn_x16, stores g and takes its sums.  g16 holds the same bits
 * as from those two calls; the other outputs meet theirs within the rounding of FP32 sums taken in another (fixed) order.
 * Kernels that cannot do this (split reduction, strided scatter form) run the two-call sequence inside the call.
 * Workspace: jz_conv2d_bwd_data_bn_relu_bwd_workspace_bytes.  Status codes as for the two calls it replaces. */
int jz_conv2d_bwd_data_block_end_bwd(const jz_conv_desc* desc, const void* dy16, const void* w16, const void* dyb16,
                                     const void* bn_x16, const void* y_out16, const float* gamma, const float* save_mean,
                                     const float* save_invstd, void* g16, void* bn_dx16, void* dgamma16, void* dbeta16, void* ws,
                                     size_t ws_bytes, void* hip_stream);

/* The backward pass at the end of a residual block, y_out = relu(bn(x) + shortcut), in one call: the gradient of the sum,
 * g = RNE16(dya [+ dyb]) where y_out > 0 and 0 elsewhere (dyb may be NULL; two contributions arrive when the block above
 * has two consumers of y_out), is formed inside the statistics pass of the batch-norm backward and written to g16 for
 * the shortcut branch; dx16, dgamma16, dbeta16 are those of jz_bn_relu_bwd(relu = 0) on dy = g.  The same bits as
 * jz_relu_bwd_sum (or jz_relu_bwd) followed by jz_bn_relu_bwd, one pass over g less.  Workspace: jz_bn_workspace_bytes. */
int jz_bn_bwd_block_end(int64_t rows, int channels, const void* x16, const void* y_out16, const void* dya16, const void* dyb16,
                        const float* gamma, const float* save_mean, const float* save_invstd, void* g16, void* dx16,
                        void* dgamma16, void* dbeta16, void* ws, size_t ws_bytes, void* hip_stream);

/* Forward convolution followed by training-mode batch normalization (+ ReLU) in one call: conv_out16 = x16 (*) w16 exactly
 * as jz_conv2d_fwd writes it, y16 / save_mean / save_invstd exactly as jz_bn_relu_fwd would compute them from conv_out16
 * (Section 4.2's formulas on the FP16 tensor of Section 4.1), but the per-channel sums of the statistics are taken in
 * the convolution kernel's epilogue, from the FP16 values it stores, instead of by a pass of their own over conv_out16
 * (when the planner's kernel for this shape cannot do that, e.g. a split reduction, the pass is run: same results up
 * to the order of the FP32 partial sums).  residual16 (may be NULL; same shape as y16, must not overlap an output): the
 * tensor a bottleneck block adds in front of its last ReLU, y = [relu](bn(conv_out) + residual), added in FP32 before
 * the single rounding of y.  conv_out16 is kept because the backward pass needs it.  Workspace from
 * jz_conv2d_bn_relu_fwd_workspace_bytes; other arguments, checks and status codes as for the two separate calls. */
int jz_conv2d_bn_relu_fwd_workspace_bytes(const jz_conv_desc* desc, size_t* bytes);
int jz_conv2d_bn_relu_fwd(const jz_conv_desc* desc, const void* x16, const void* w16, const float* gamma, const float* beta,
                          float eps, const void* residual16, int relu, void* conv_out16, void* y16, float* save_mean,
                          float* save_invstd, void* ws, size_t ws_bytes, void* hip_stream);

/* The small layers between the convolutions of a ResNet-style network (the paper trains stock ResNet-50 / AlexNet,
 * Section 5, and does not restate them), on FP16 NHWC DEVICE tensors, the storage type Section 4.1 gives every forward
 * and backward tensor.  Each is its textbook definition evaluated in FP32 with one rounding to FP16 on the store;
 * element counts and channel counts must be multiples of 8, tensor pointers 16-byte aligned (JZ_ERR_SHAPE /
 * JZ_ERR_ALIGN otherwise); nothing is allocated, everything is enqueued on hip_stream; empty inputs are JZ_OK.
 *   jz_add_fwd      y = a + b, followed by max(., 0) when relu != 0 (the residual connection).  y may be a or b.
 *   jz_relu_bwd     dx = dy where the forward output y is > 0, else 0.  dx may be dy.
 *   jz_relu_bwd_sum dx = RNE16(dya + dyb) where y > 0, else 0: the same as jz_add_fwd (no ReLU) followed by jz_relu_bwd, bit for
 *                   bit, in one pass (a block output whose gradient arrives from two consumers).  dx may be dya or dyb.
 *   jz_maxpool_fwd  x[N,H,W,C] -> y[N,P,Q,C], P = (H + 2 pad - window) / stride + 1 (same for Q); padding never wins.
 *                   arg8 (may be NULL; DEVICE, 8-byte aligned, one byte per output element) receives the position
 *                   r * window + s inside its window of each output's first maximum in (row, column) order.
 *   jz_maxpool_bwd  dx[N,H,W,C] from dy[N,P,Q,C]: each dy goes to the first maximum of its window; a position that wins
 *                   several windows gets their sum (FP32, window order).  With arg8 from the forward call the winners
 *                   are taken from it and x16 may be NULL; with arg8 == NULL they are derived again from x16 (same
 *                   result, several times the arithmetic).  pad < window <= 16.
 *   jz_avgpool_fwd  global average: x[N,HW,C] -> y[N,C] = sum over the HW positions (FP32, in order) / HW.
 *   jz_avgpool_bwd  dy[N,C] -> dx[N,HW,C] = dy / HW at every position.
 *   jz_bias_add     out[rows,C] = y[rows,C] + b[C].  out may be y.
 *   jz_bias_grad    db[C] = sum over rows of dy[rows,C] (FP32, fixed order: deterministic).  Meant for a fully connected
 *                   layer's bias (rows = batch size); it uses C/32 workgroups whatever rows is.
 *   jz_softmax_xent_bwd  z[rows,classes] FP16 logits, labels_dev[rows] int32 (DEVICE): loss_dev[n] = log(sum_j exp z_nj) -
 *                   z_n,label (FP32, DEVICE) and dz = S * (softmax(z_n) - onehot(label_n)) / rows in FP16, the gradient of the
 *                   batch-mean loss times the loss scale S of Section 4.1.  S is state_dev->scale when state_dev (DEVICE,
 *                   as in jz_lars_mp_update_dyn) is not NULL, else loss_scale.  A label outside [0, classes) gives a NaN loss
 *                   and a zero gradient row.  classes need not be a multiple of 8 here (2-byte alignment suffices). */
int jz_add_fwd(int64_t n, const void* a16, const void* b16, int relu, void* y16, void* hip_stream);
int jz_relu_bwd(int64_t n, const void* y16, const void* dy16, void* dx16, void* hip_stream);
int jz_relu_bwd_sum(int64_t n, const void* y16, const void* dya16, const void* dyb16, void* dx16, void* hip_stream);
int jz_maxpool_fwd(int N, int H, int W, int C, int window, int stride, int pad, const void* x16, void* y16, void* arg8,
                   void* hip_stream);
int jz_maxpool_bwd(int N, int H, int W, int C, int window, int stride, int pad, const void* x16, const void* arg8,
                   const void* dy16, void* dx16, void* hip_stream);
int jz_avgpool_fwd(int N, int HW, int C, const void* x16, void* y16, void* hip_stream);
int jz_avgpool_bwd(int N, int HW, int C, const void* dy16, void* dx16, void* hip_stream);
int jz_bias_add(int64_t rows, int C, const void* y16, const void* b16, void* out16, void* hip_stream);
int jz_bias_grad(int64_t rows, int C, const void* dy16, void* db16, void* hip_stream);
int jz_softmax_xent_bwd(int rows, int classes, const void* z16, const int* labels_dev, float loss_scale,
                        const jz_loss_scale_state* state_dev, void* dz16, float* loss_dev, void* hip_stream);

/* Batch normalization in training mode with an optional ReLU behind it (Section 4.2 of the paper writes the layer as
 * x^ = (x - mean_B) / sqrt(var_B + eps), y = gamma * x^ + beta; mean_B and var_B are the mean and the plain (biased)
 * variance of the mini-batch, per channel, over all rows = N*H*W positions).  Not part of the convolution / LARS hot path
 * the benchmark times; the first piece of the layers that sit between the convolutions.
 *   x16, y16, dy16, dx16: DEVICE FP16 [rows][channels] (NHWC flattened), 16-byte aligned; channels a multiple of 8, <= 2048
 *   gamma, beta, save_mean, save_invstd: DEVICE FP32 [channels] (master precision), 16-byte aligned
 *   dgamma16, dbeta16: DEVICE FP16 [channels]: the parameter gradients as the optimizer's FP16 gradient buffer takes them
 *                      (they carry whatever loss scale dy16 carries)
 *   ws: DEVICE workspace of jz_bn_workspace_bytes(rows, channels) bytes (per-slab partial sums and per-channel
 *       coefficients); contents need not survive between the forward and the backward call
 * jz_bn_relu_fwd: y = gamma * (x - mean) * invstd + beta, then max(., 0) when relu != 0, rounded once to FP16; writes the
 *   statistics it used (invstd = 1 / sqrt(var + eps)) to save_mean / save_invstd.  Sums are FP32 within a slab of rows
 *   and FP64 across slabs, in an order that depends only on (rows, channels): results are deterministic.
 * jz_bn_relu_bwd: with g = dy (relu == 0) or dy where y16 > 0 and 0 elsewhere (relu != 0; y16 is the forward output):
 *   dbeta = sum g, dgamma = sum g * x^, dx = gamma * invstd * (g - dbeta / rows - x^ * dgamma / rows).  y16 may be NULL
 *   when relu == 0.
 * Status codes as for the convolutions (JZ_ERR_UNSUPPORTED for channel counts outside the range above). */
int jz_bn_workspace_bytes(int64_t rows, int channels, size_t* bytes);
int jz_bn_relu_fwd(int64_t rows, int channels, const void* x16, const float* gamma, const float* beta, float eps, int relu,
                   void* y16, float* save_mean, float* save_invstd, void* ws, size_t ws_bytes, void* hip_stream);
int jz_bn_relu_bwd(int64_t rows, int channels, const void* x16, const void* y16, const void* dy16, const float* gamma,
                   const float* save_mean, const float* save_invstd, int relu, void* dx16, void* dgamma16, void* dbeta16,
                   void* ws, size_t ws_bytes, void* hip_stream);

/* Writes into `text` (HOST, NUL-terminated, at most text_bytes) one line saying how the library would run this
 * operation: GEMM dimensions, kernel variant (output tile, k tile depth, wavefronts), tiles, split of the reduction.
 * For tuning and bug reports; the wording is not part of the contract.  Same status codes as the workspace query. */
int jz_conv2d_describe_plan(int op, const jz_conv_desc* desc, char* text, size_t text_bytes);

/* Planner tuning hook (HOST state, process-wide, guarded by a mutex).  jz_conv2d_tune_set records, for the GEMM that
 * `op` on `desc` maps to, which kernel variant to run: output tile tile_m x tile_n, k tile depth, wavefronts per
 * workgroup, ring depth (LDS stages) and the number of splits of the reduction (not split at all where a split would be
 * shorter than four k tiles).  Later calls for that shape use it in place of the built-in table of measured
 * choices and of the cost model; nothing else overrides the planner (the library reads no environment variables).
 * The variant must be one the library has (jz_conv2d_describe_plan shows the names: e.g. 128x128 tile, k tile 64,
 * 8 wavefronts, ring 4), else JZ_ERR_UNSUPPORTED; shapes that gather with per-load tap arithmetic take the four
 * 4-wavefront tiles, 32 deep, ring 4; a strided multi-tap backward-data layer, which runs as one launch per parity
 * class of its stride, takes the variant for every one of those launches (never split); shapes on the element-wise
 * kernel cannot be tuned (JZ_ERR_UNSUPPORTED).
 * Results never depend on the choice beyond the summation order of the reduction.
 * jz_conv2d_tune_use_table(0) makes the planner skip its built-in table of measured choices (cost model only),
 * jz_conv2d_tune_use_table(1) restores it.  jz_conv2d_tune_clear forgets every recorded choice and restores the
 * table.  Used by the tests to force every kernel variant and by `python -m paper_1807_11205_amd.tune`. */
int jz_conv2d_tune_set(int op, const jz_conv_desc* desc, int tile_m, int tile_n, int k_tile, int wavefronts, int ring,
                       int splits);
int jz_conv2d_tune_use_table(int on);
int jz_conv2d_tune_clear(void);

/* Human-readable name of a status code; static storage. */
const char* jz_status_string(int status);

/* Library version, e.g. 100 for 0.1.0. */
int jz_version(void);

#ifdef __cplusplus
}
#endif
#endif /* JZ_H_ */
