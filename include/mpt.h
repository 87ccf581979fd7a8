/*
 * mpt -- the hot path of one mixed-precision training step on AMD MI355X (gfx950).
 *
 * Method: "Mixed Precision Training", arXiv 1710.03740.  Tensors are stored in
 * IEEE binary16; dot products accumulate in FP32 and round once to FP16 on
 * store (Sec. 3.3); the loss is scaled by S so that small gradients survive the
 * FP16 store, weight gradients are unscaled by 1/S before the update and an
 * Inf/NaN among them makes the step a no-op (Sec. 3.2); the optimizer updates an
 * FP32 master copy of the weights, which is rounded to FP16 for the next
 * iteration (Sec. 3.1); a dynamic policy raises or lowers S (Sec. 5).
 *
 * Conventions for EVERY entry point unless stated otherwise
 *   - Pointers named *_dev or documented "device" are DEVICE pointers owned by
 *     the caller.  The library never allocates, retains or frees memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work on it and never synchronise.
 *   - FP16 data is passed as uint16_t (IEEE binary16 bit patterns).
 *   - Matrices are row-major; `ld*` is the element stride between rows and must
 *     be >= the row length.
 *   - Return value: MPT_OK (0) or a negative mpt_status.  Arguments are checked
 *     before anything is enqueued; on error nothing has been enqueued.
 *   - Inputs are never modified.  Outputs are fully overwritten unless the
 *     entry point says "accumulate" or "no-op when flagged".
 *   - FP16 stores round to nearest even and overflow to Inf (no saturation).
 */
#ifndef MPT_H
#define MPT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum mpt_status {
  MPT_OK = 0,
  MPT_ERR_NULL = -1,      /* a required pointer is NULL */
  MPT_ERR_SHAPE = -2,     /* a size is < 1, a leading dimension is too small, or a size exceeds the supported maximum */
  MPT_ERR_ALIGN = -3,     /* a pointer is not aligned to its element type */
  MPT_ERR_WORKSPACE = -4, /* workspace given but smaller than mpt_gemm_workspace_bytes() */
  MPT_ERR_ARG = -5,       /* a scalar argument is out of range (e.g. non-finite or non-positive scale) */
  MPT_ERR_HIP = -6        /* the HIP runtime refused the launch */
} mpt_status;

/* Static string for a status code.  Never NULL. */
const char* mpt_status_string(int status);

/* Library version: major*10000 + minor*100 + patch. */
int mpt_version(void);

/* ------------------------------------------------------------------------- *
 * Dense contractions (Sec. 3.3: FP16 products, FP32 accumulation, one RNE
 * rounding to FP16 on store; Sec. 3.1 / Fig. 1: forward, backward-activation
 * and backward-weight of a layer).  X[M,K] activations, W[K,N] weights,
 * Y[M,N] outputs, dY[M,N] upstream gradient, all row-major with a leading
 * dimension in elements.  Any M,N,K from 1 to 2^31 - 513 (else MPT_ERR_SHAPE).
 * Fast path: base pointers 16-byte aligned and leading dimensions multiples of 8; anything else (2-byte alignment is the
 * minimum) takes a slower element-wise loader with identical results.
 *
 * Workspace: split-reduction needs FP32 partials in caller memory.  Pass
 * ws_dev = NULL, ws_bytes = 0 to forbid splitting (always legal), or a device
 * buffer of at least mpt_gemm_workspace_bytes(op, M, N, K) bytes, 16-byte
 * aligned.  The size is an upper bound over the kernels the library may pick
 * for the shape (a whole number of [I][J] FP32 partial outputs; which kernel
 * runs also depends on the operands' alignment); the partials written lead
 * the buffer as [split][I][J].  Partials are summed in a fixed order (results
 * are run-to-run deterministic) and rounded once.
 * ------------------------------------------------------------------------- */
typedef enum mpt_gemm_op { MPT_OP_FWD = 0, MPT_OP_DGRAD = 1, MPT_OP_WGRAD = 2 } mpt_gemm_op;

size_t mpt_gemm_workspace_bytes(int op, int64_t M, int64_t N, int64_t K);

/* Y[m,n] = rne16( sum_k X[m,k] * W[k,n] ) */
int mpt_gemm_fwd(void* stream, int64_t M, int64_t N, int64_t K,
                 const uint16_t* X_dev, int64_t ldx,
                 const uint16_t* W_dev, int64_t ldw,
                 uint16_t* Y_dev, int64_t ldy,
                 void* ws_dev, size_t ws_bytes);

/* dX[m,k] = rne16( sum_n dY[m,n] * W[k,n] ) */
int mpt_gemm_dgrad(void* stream, int64_t M, int64_t N, int64_t K,
                   const uint16_t* dY_dev, int64_t ldy,
                   const uint16_t* W_dev, int64_t ldw,
                   uint16_t* dX_dev, int64_t ldx,
                   void* ws_dev, size_t ws_bytes);

/* The pointwise non-linearity of a layer (Sec. 3.3, third category) folded into the store of the contraction that
 * produces its input, so the activation tensor makes one trip to memory instead of three:
 *   fwd_relu:   H[m,n]  = rne16( max( sum_k X[m,k] * W[k,n], 0 ) )      (anything not > 0, NaN included, stores +0)
 *   dgrad_relu: dX[m,k] = H[m,k] > 0 ? rne16( sum_n dY[m,n] * W[k,n] ) : +0
 * where H[M,K] (ldh >= K) is the FP16 output that the layer below stored with fwd_relu.  Same shapes, alignment
 * rules, workspace and error behaviour as mpt_gemm_fwd / mpt_gemm_dgrad; H is only read. */
int mpt_gemm_fwd_relu(void* stream, int64_t M, int64_t N, int64_t K,
                      const uint16_t* X_dev, int64_t ldx,
                      const uint16_t* W_dev, int64_t ldw,
                      uint16_t* H_dev, int64_t ldh,
                      void* ws_dev, size_t ws_bytes);
int mpt_gemm_dgrad_relu(void* stream, int64_t M, int64_t N, int64_t K,
                        const uint16_t* dY_dev, int64_t ldy,
                        const uint16_t* W_dev, int64_t ldw,
                        const uint16_t* H_dev, int64_t ldh,
                        uint16_t* dX_dev, int64_t ldx,
                        void* ws_dev, size_t ws_bytes);

/* dW[k,n] = sum_m X[m,k] * dY[m,n].
 *   out_fp32 = 0: dW_dev is uint16_t*, FP16 store (the paper's stored weight gradient); accumulate must be 0.
 *   out_fp32 = 1: dW_dev is float*, FP32 store; accumulate = 1 adds this call's sum to the buffer's
 *                 current contents (per-timestep contributions never pass through FP16).
 *   flag_dev (nullable, device uint32_t): when given, 1 is OR-ed into it if any stored element is Inf/NaN
 *                 (Sec. 3.2's overflow test folded into the producer; never cleared here). */
int mpt_gemm_wgrad(void* stream, int64_t M, int64_t N, int64_t K,
                   const uint16_t* X_dev, int64_t ldx,
                   const uint16_t* dY_dev, int64_t ldy,
                   void* dW_dev, int64_t lddw,
                   int out_fp32, int accumulate, uint32_t* flag_dev,
                   void* ws_dev, size_t ws_bytes);

/* mpt_gemm_wgrad for callers that cannot allocate device memory: code under HIP graph capture, tight serving or
 * training loops, harnesses that forbid hipMalloc.  Same arguments, results (bit for bit) and errors as
 * mpt_gemm_wgrad, without the workspace: the FP32 split partials go to a device array of MPT_STATIC_SCRATCH_BYTES
 * that is part of the library's code object (one copy per GPU, held until the process ends).  The call allocates
 * and frees nothing; its first use on a device looks the array's address up (hipGetSymbolAddress), so make one call
 * per device before capturing a graph.  A shape whose split needs more than the array
 * (mpt_gemm_workspace_bytes(MPT_OP_WGRAD, M, N, K) > MPT_STATIC_SCRATCH_BYTES) is refused with MPT_ERR_WORKSPACE and
 * nothing is launched.  Every call on one GPU shares that GPU's array: calls that may overlap in time on one GPU
 * (different streams) race and must not be made; calls on one stream are ordered and safe.  Partials are written
 * before they are read, so the array needs no clearing between calls. */
#define MPT_STATIC_SCRATCH_BYTES (32u << 20)
int mpt_gemm_wgrad_static(void* stream, int64_t M, int64_t N, int64_t K,
                          const uint16_t* X_dev, int64_t ldx,
                          const uint16_t* dY_dev, int64_t ldy,
                          void* dW_dev, int64_t lddw,
                          int out_fp32, int accumulate, uint32_t* flag_dev);

/* ------------------------------------------------------------------------- *
 * 3x3 convolution, stride 1, zero padding 1, as an implicit GEMM (Sec. 3.3 and
 * Sec. 4 list convolutions among the FP32-accumulated dot products).
 * x[Nb,H,W,C] NHWC, w[Kf,3,3,C] KRSC, y/dy[Nb,H,W,Kf]; all dense, 16-byte
 * aligned, C and Kf multiples of 8.  Cross-correlation (no filter flip):
 *   y [n,p,q,k] = rne16( sum_{r,s,c} x[n,p+r-1,q+s-1,c] * w[k,r,s,c] )
 *   dx[n,h,v,c] = rne16( sum_{r,s,k} dy[n,h-r+1,v-s+1,k] * w[k,r,s,c] )
 *   dw[k,r,s,c] = rne16( sum_{n,p,q} dy[n,p,q,k] * x[n,p+r-1,q+s-1,c] )
 * Workspace as for the GEMMs, sized by mpt_conv3x3_workspace_bytes().
 * ------------------------------------------------------------------------- */
size_t mpt_conv3x3_workspace_bytes(int op, int64_t Nb, int64_t H, int64_t W, int64_t C, int64_t Kf);

int mpt_conv3x3_fwd(void* stream, int64_t Nb, int64_t H, int64_t W, int64_t C, int64_t Kf,
                    const uint16_t* x_dev, const uint16_t* w_dev, uint16_t* y_dev,
                    void* ws_dev, size_t ws_bytes);
int mpt_conv3x3_dgrad(void* stream, int64_t Nb, int64_t H, int64_t W, int64_t C, int64_t Kf,
                      const uint16_t* dy_dev, const uint16_t* w_dev, uint16_t* dx_dev,
                      void* ws_dev, size_t ws_bytes);
int mpt_conv3x3_wgrad(void* stream, int64_t Nb, int64_t H, int64_t W, int64_t C, int64_t Kf,
                      const uint16_t* x_dev, const uint16_t* dy_dev, uint16_t* dw_dev,
                      uint32_t* flag_dev, void* ws_dev, size_t ws_bytes);

/* ------------------------------------------------------------------------- *
 * Loss-scale state (Sec. 5 sketches the dynamic policy and fixes no constants).
 * Policy: on overflow scale *= backoff, good_steps = 0; otherwise good_steps += 1
 * and when it reaches growth_interval: scale *= growth, good_steps = 0.  scale is
 * clamped to [min_scale, max_scale]; inv_scale = 1/scale in FP32.
 * The struct may live in host memory (mpt_loss_scale_update) or in device memory
 * (mpt_loss_scale_update_dev); layout is fixed, 32 bytes.
 * ------------------------------------------------------------------------- */
typedef struct mpt_scaler {
  float scale;
  float inv_scale;
  int32_t good_steps;
  int32_t growth_interval;
  float growth;
  float backoff;
  float min_scale;
  float max_scale;
} mpt_scaler;

/* Fill *s (host memory): given initial scale and interval, growth 2, backoff 1/2, clamps [1, 2^24]. */
int mpt_scaler_init(mpt_scaler* s, float scale, int32_t growth_interval);

/* Host-side policy step on a host-resident struct.  overflow != 0 means the step was skipped. */
int mpt_loss_scale_update(mpt_scaler* s, int overflow);

/* Device-side policy step: one tiny kernel reads *flag_dev, applies the policy to
 * *s_dev (device memory, 4-byte aligned) and clears *flag_dev, so a training step
 * needs no host synchronisation. */
int mpt_loss_scale_update_dev(void* stream, mpt_scaler* s_dev, uint32_t* flag_dev);

/* ------------------------------------------------------------------------- *
 * Unscale + overflow check (Sec. 3.2: gradients are unscaled before the update;
 * overflow is detected by inspecting the weight gradients).
 *   flag |= any_i( grad[i] is Inf or NaN )         (tested on the stored bits)
 *   g32_out[i] = float(grad[i]) * inv_scale          (only when g32_out_dev != NULL)
 * grad_dev: n elements, uint16_t (grad_is_fp32 = 0) or float (grad_is_fp32 = 1).
 * flag_dev: device uint32_t, OR-ed into (the caller, or
 * mpt_loss_scale_update_dev, clears it).  n = 0 is a legal no-op.
 * inv_scale must be finite and > 0.
 * ------------------------------------------------------------------------- */
int mpt_unscale_check(void* stream, const void* grad_dev, int grad_is_fp32, size_t n,
                      float inv_scale, float* g32_out_dev, uint32_t* flag_dev);

/* ------------------------------------------------------------------------- *
 * FP32 master update + FP16 working copy (Sec. 3.1), skipped on overflow
 * (Sec. 3.2).  Each step is one separately rounded IEEE FP32 operation:
 *   g  = float(grad) * inv_scale
 *   m' = momentum * m + g ;  w' = w - lr * m'       (m32_dev != NULL)
 *        w' = w - lr * g                            (m32_dev == NULL, plain SGD)
 *   w16' = rne16(w')
 * In place on w32_dev / m32_dev; w16_dev is overwritten.
 * flag_dev (nullable): if *flag_dev != 0 when the kernel runs, the call is a
 * no-op: master, momentum and FP16 copy keep their bits.
 * scaler_dev (nullable): when given, inv_scale is read from scaler_dev->inv_scale
 * on the device and the inv_scale argument is ignored.
 * n = 0 is a legal no-op.  lr and momentum must be finite; inv_scale finite, > 0.
 * ------------------------------------------------------------------------- */
int mpt_master_update(void* stream, size_t n, float* w32_dev, float* m32_dev,
                      const void* grad_dev, int grad_is_fp32, uint16_t* w16_dev,
                      float inv_scale, const mpt_scaler* scaler_dev,
                      float lr, float momentum, const uint32_t* flag_dev);

/* ------------------------------------------------------------------------- *
 * mpt_master_update for many parameter tensors in as few launches as possible
 * (Sec. 3.1: every layer's weights have an FP32 master copy; the update is one
 * pass over all of them).  items_host[k] names tensor k's device buffers and
 * its element count; every tensor gets exactly the update mpt_master_update
 * would give it (same operations, same bits), with the same inv_scale /
 * scaler_dev, lr, momentum and skip flag.  m32_dev: given for all tensors or
 * for none (ARG otherwise).  Tensors with n = 0 are skipped; count = 0 is a
 * legal no-op.  The array is read during the call and may be freed after it.
 * Nothing is launched unless every item is valid.
 * Errors: NULL, ARG, ALIGN (as mpt_master_update, per tensor), SHAPE (n > 2^40).
 * ------------------------------------------------------------------------- */
typedef struct mpt_update_item {
  float* w32_dev;        /* FP32 master weights, updated in place */
  float* m32_dev;        /* FP32 momentum, updated in place; NULL = plain SGD */
  const void* grad_dev;  /* FP16 or FP32 gradient (grad_is_fp32 of the call) */
  uint16_t* w16_dev;     /* FP16 working copy, overwritten */
  size_t n;              /* elements */
} mpt_update_item;

int mpt_master_update_multi(void* stream, int count, const mpt_update_item* items_host, int grad_is_fp32,
                            float inv_scale, const mpt_scaler* scaler_dev,
                            float lr, float momentum, const uint32_t* flag_dev);

/* ------------------------------------------------------------------------- *
 * The same step in ONE pass over the gradient (Sec. 3.2: the overflow test and
 * the unscaled update read the same values): 20 B per element with momentum
 * and an FP16 gradient instead of 2 + 20 for mpt_unscale_check followed by
 * mpt_master_update.  Whether the step must be skipped is known only once every
 * gradient has been seen, so the results go to a second set of buffers:
 *   flag_dev[0] |= 1 if any stored gradient is Inf or NaN (tested on the stored
 *                    bits; at most one atomic per wavefront);
 *   w32_out, m32_out, w16_out receive the update of mpt_master_update computed
 *                    as if the step were taken, always.
 * The caller adopts the output set as the current state only if the flag
 * stayed 0 (swap the two sets' roles), and keeps the input set otherwise; with
 * the flag set the outputs hold arithmetic on Inf / NaN and must not be used.
 * The input set is never written.  m32_in and m32_out are both NULL (plain SGD)
 * or both given.  The output buffers must not overlap the input buffers (ARG).
 * Pairs of elements move together when the FP32 arrays are 8-byte and the FP16
 * arrays 4-byte aligned, else one at a time.  Costs 10 B per element of extra
 * memory for the second set.
 * Errors: NULL, ARG (as mpt_master_update; overlap; one momentum pointer only), ALIGN.
 * ------------------------------------------------------------------------- */
int mpt_master_update_fused(void* stream, size_t n, const float* w32_in_dev, const float* m32_in_dev,
                            const void* grad_dev, int grad_is_fp32,
                            float* w32_out_dev, float* m32_out_dev, uint16_t* w16_out_dev,
                            float inv_scale, const mpt_scaler* scaler_dev,
                            float lr, float momentum, uint32_t* flag_dev);

/* ------------------------------------------------------------------------- *
 * Pointwise / reduction glue for a whole step on the device (Sec. 3.3: softmax
 * reduces in FP32 with FP16 input and output; non-linearities are pointwise).
 *   add_fp16:  out[i] = rne16(a[i] + b[i])                  (exact sum, one rounding; out may alias a or b: where a
 *              gradient reaches a tensor along two paths, e.g. a recurrent layer's output at step t, used by the
 *              layer above and by step t+1)
 *   relu_fwd:  h[i]  = max(y[i], 0)
 *   relu_bwd:  dy[i] = y[i] > 0 ? dh[i] : 0
 *   softmax_xent_scaled: p = softmax(logits[b,:]);
 *       row_loss_dev[b] = -log p[b,label_b]                (FP32[B]; nullable unless loss_dev is given)
 *       loss_dev[0] = mean_b row_loss_dev[b]               (FP32; nullable; summed in a fixed order)
 *       dlogits[b,c] = rne16( scale * (p[b,c] - [c==label_b]) / B )
 *     which applies Sec. 3.2's loss scale at the head of back-propagation.
 *     labels_dev: int32, each in [0, C) (a value outside is clamped into the range).  C <= 2^24.  Each row is read once and written once when C <= 65536
 *     (16-byte accesses when both tensors are 16-byte aligned with C and the row strides multiples of 8).
 * ------------------------------------------------------------------------- */
int mpt_add_fp16(void* stream, size_t n, const uint16_t* a_dev, const uint16_t* b_dev, uint16_t* out_dev);
int mpt_relu_fwd(void* stream, size_t n, const uint16_t* y_dev, uint16_t* h_dev);
int mpt_relu_bwd(void* stream, size_t n, const uint16_t* dh_dev, const uint16_t* y_dev, uint16_t* dy_dev);
int mpt_softmax_xent_scaled(void* stream, int64_t B, int64_t C,
                            const uint16_t* logits_dev, int64_t ldl, const int32_t* labels_dev,
                            float scale, float* loss_dev, float* row_loss_dev, uint16_t* dlogits_dev, int64_t ldd);

/* ------------------------------------------------------------------------- *
 * Other optimizers in the same fused pass (Sec. 4 trains with momentum SGD,
 * Nesterov SGD, Adagrad and Adam; Sec. 3.1 keeps weights and with them the
 * optimizer state in FP32; Sec. 3.2: the gradient is unscaled before anything
 * else touches it, so weight decay and every other hyper-parameter is the
 * same as in FP32 training).  The paper prints no update rule; the customary
 * ones are used, each a fixed sequence of individually rounded FP32
 * operations, (*) (+) (-) (/) sqrt:
 *     g = float(grad) (*) inv_S        [if clip_factor_dev:    g = g (*) *clip_factor_dev]
 *                                      [if weight_decay != 0:  g = g (+) (weight_decay (*) w)]
 *   MOMENTUM  m' = (mu (*) m) (+) g               w' = w (-) (lr (*) m')
 *   NESTEROV  m' = (mu (*) m) (+) g               w' = w (-) (lr (*) (g (+) (mu (*) m')))
 *   ADAGRAD   h' = h (+) (g (*) g)                w' = w (-) ((lr (*) g) (/) (sqrt(h') (+) eps))
 *   ADAM      m' = (beta1 (*) m) (+) (one_minus_beta1 (*) g)
 *             v' = (beta2 (*) v) (+) (one_minus_beta2 (*) (g (*) g))
 *             w' = w (-) ((lr (*) (m' (/) bias_corr1)) (/) (sqrt(v' (/) bias_corr2) (+) eps))
 *     w16' = rne16(w')
 * state1 is m / h / m, state2 is Adam's v (ignored otherwise, may be NULL).
 * `momentum` holds mu, or beta1 for Adam; one_minus_beta* and bias_corr*
 * (1 - beta^t for the 1-based step t) are supplied by the caller already
 * rounded to FP32.  hp is a HOST pointer, read before the call returns.
 * inv_scale / scaler_dev / flag_dev as in mpt_master_update: a nonzero flag
 * makes the call a no-op, state included.  All arrays are device memory of n
 * elements owned by the caller; pairs of elements are moved together when
 * the FP32 arrays are 8-byte and the FP16 arrays 4-byte aligned, else one at
 * a time.  Traffic per element with an FP16 gradient: 20 B (28 B for Adam).
 * Errors: NULL, ARG (unknown kind, non-finite or negative hyper-parameter,
 * bias correction not > 0), ALIGN.
 * ------------------------------------------------------------------------- */
typedef enum mpt_opt_kind { MPT_OPT_MOMENTUM = 0, MPT_OPT_NESTEROV = 1, MPT_OPT_ADAGRAD = 2, MPT_OPT_ADAM = 3 } mpt_opt_kind;
typedef struct mpt_opt_params {
  float lr;
  float momentum;
  float beta2;
  float eps;
  float weight_decay;
  float one_minus_beta1, one_minus_beta2;
  float bias_corr1, bias_corr2;
  const float* clip_factor_dev;  /* NULL, or a device FP32 written by mpt_clip_factor: g = g (*) factor right after unscaling */
} mpt_opt_params;
int mpt_optimizer_update(void* stream, size_t n, int kind, const mpt_opt_params* hp_host,
                         float* w32_dev, float* state1_dev, float* state2_dev,
                         const void* grad_dev, int grad_is_fp32, uint16_t* w16_dev,
                         float inv_scale, const mpt_scaler* scaler_dev, const uint32_t* flag_dev);

/* ------------------------------------------------------------------------- *
 * Gradient clipping by global norm (Sec. 3.2: gradients are unscaled before
 * the update precisely so that clipping thresholds and weight decay keep
 * their FP32 values; the paper prints no rule, the customary one is used).
 *   mpt_grad_sumsq:  sumsq (+)= sum_i ( float(grad[i]) (*) inv_S )^2   each square exact, FP64 sum in an order fixed
 *                    by n and the alignment alone (same bits every run);  flag |= any Inf/NaN among the stored
 *                    values (the overflow test of mpt_unscale_check from the same read: 2 B per FP16 element).
 *                    accumulate = 0 stores, != 0 adds to *sumsq_dev (several buffers, one global norm).
 *                    sumsq_dev: device double.  ws_dev: device scratch of mpt_grad_norm_workspace_bytes() bytes,
 *                    8-byte aligned.  inv_scale / scaler_dev as in mpt_master_update.  n = 0 is legal.
 *   mpt_clip_factor: norm = sqrt(*sumsq_dev) in FP64;  *factor_dev = 1 if norm <= max_norm (or NaN: the step is
 *                    skipped anyway), else the FP64 quotient max_norm / norm rounded once to FP32;
 *                    *norm_dev (nullable) = norm rounded to FP32.  max_norm finite, > 0.
 *   mpt_optimizer_update multiplies the unscaled gradient by *hp->clip_factor_dev (one FP32 multiplication, before
 *   weight decay) when that pointer is set.  No host synchronisation anywhere.
 * Errors: NULL, ARG, ALIGN, WORKSPACE.
 * ------------------------------------------------------------------------- */
size_t mpt_grad_norm_workspace_bytes(void);
int mpt_grad_sumsq(void* stream, const void* grad_dev, int grad_is_fp32, size_t n,
                   float inv_scale, const mpt_scaler* scaler_dev, int accumulate,
                   double* sumsq_dev, uint32_t* flag_dev, void* ws_dev, size_t ws_bytes);
int mpt_clip_factor(void* stream, const double* sumsq_dev, float max_norm, float* factor_dev, float* norm_dev);

/* ------------------------------------------------------------------------- *
 * Gradient statistics (Sec. 3.2: exponent histograms of the gradients show
 * what FP16 would lose, and a constant loss scale is chosen so that
 * scale * max|g| stays below 65504).  Over the stored FP16 values:
 *   hist_dev[0]            zeros (+0, -0)
 *   hist_dev[1 + e + 24]   finite non-zero values with floor(log2 |g|) = e, e = -24 .. 15
 *   hist_dev[41]           Inf and NaN
 *   absmax_bits_dev[0]     bit pattern (sign cleared) of the largest finite magnitude, 0 if none
 * hist_dev: uint64[42], absmax_bits_dev: uint32, device memory.  accumulate = 0
 * clears both first; accumulate != 0 adds to what they hold (several buffers,
 * one histogram).  Counts are integers, so the result does not depend on the
 * order of evaluation.  mpt_suggest_loss_scale_log2 (host, pure C) returns k
 * with 2^k the largest power of two such that 2^k * max <= 65504, clamped to
 * [-24, 40]; max is given as the FP16 bit pattern; 0 yields `if_zero`.
 * ------------------------------------------------------------------------- */
#define MPT_GRAD_STATS_BINS 42
int mpt_grad_stats(void* stream, const uint16_t* grad_dev, size_t n, int accumulate,
                   uint64_t* hist_dev, uint32_t* absmax_bits_dev);
int mpt_suggest_loss_scale_log2(uint32_t absmax_bits, int if_zero);

/* ------------------------------------------------------------------------- *
 * Batch normalisation over an FP16 tensor x[P, C], channels contiguous, row
 * stride ldx >= C elements (an NHWC activation with P = N*H*W).  Sec. 3.3: the
 * statistics are large reductions and are accumulated wide; the layer reads
 * and writes FP16 and computes in FP32.  Training-mode definition (the paper
 * prints no formulas), per channel c:
 *   mean_c = (1/P) sum_p x[p,c]        var_c = (1/P) sum_p (x[p,c] - mean_c)^2
 *   y[p,c] = rne16( x*scale_c + shift_c ),  scale_c = gamma_c * (1/sqrt(var_c + eps)),
 *            shift_c = beta_c - mean_c*scale_c      (then max(.,0) if relu != 0)
 *   dbeta_c = sum_p dy[p,c]     dgamma_c = sum_p dy[p,c] * xhat[p,c],
 *            xhat = (x - mean_c) * (1/sqrt(var_c + eps))
 *   dx[p,c] = rne16( a_c * ((dy - dbeta_c/P) - xhat * dgamma_c/P) ),  a_c = gamma_c * (1/sqrt(var_c + eps))
 * Every pointwise operation is an individually rounded FP32 operation in the
 * order written (no fused multiply-add), so results are reproducible bit for
 * bit from the same statistics.  Reductions run as FP32 chains of at most 16
 * rows folded into FP64, in a fixed order (run-to-run identical), and are
 * rounded once to FP32.  dy may carry the loss scale; dgamma / dbeta / dx
 * then carry it too (everything is linear in dy).
 *
 * All pointers are device pointers owned by the caller; mean, var, gamma,
 * beta, dgamma, dbeta are FP32[C].  Fast path: 16-byte aligned tensors, C and
 * row strides multiples of 8; anything else takes a scalar path with the same
 * results.  ws_dev: caller scratch of at least mpt_bn_workspace_bytes(P, C)
 * bytes, 16-byte aligned (FP64 partial sums), required by the two reductions.
 * Errors (nothing enqueued): NULL, SHAPE (P < 1 or >= 2^40, C < 1 or > 2^21, stride < C), ALIGN,
 * WORKSPACE, ARG (eps negative or not finite).
 * ------------------------------------------------------------------------- */
size_t mpt_bn_workspace_bytes(int64_t P, int64_t C);
int mpt_bn_stats(void* stream, int64_t P, int64_t C, const uint16_t* x_dev, int64_t ldx,
                 float* mean_dev, float* var_dev, void* ws_dev, size_t ws_bytes);
int mpt_bn_apply(void* stream, int64_t P, int64_t C, const uint16_t* x_dev, int64_t ldx,
                 const float* mean_dev, const float* var_dev, const float* gamma_dev, const float* beta_dev,
                 float eps, int relu, uint16_t* y_dev, int64_t ldy);
int mpt_bn_bwd_reduce(void* stream, int64_t P, int64_t C, const uint16_t* x_dev, int64_t ldx,
                      const uint16_t* dy_dev, int64_t lddy, const float* mean_dev, const float* var_dev, float eps,
                      float* dgamma_dev, float* dbeta_dev, void* ws_dev, size_t ws_bytes);
int mpt_bn_bwd_apply(void* stream, int64_t P, int64_t C, const uint16_t* x_dev, int64_t ldx,
                     const uint16_t* dy_dev, int64_t lddy, const float* mean_dev, const float* var_dev,
                     const float* gamma_dev, float eps, const float* dgamma_dev, const float* dbeta_dev,
                     uint16_t* dx_dev, int64_t lddx);

/* ------------------------------------------------------------------------- *
 * Pointwise part of an LSTM cell (Sec. 3.3 "point-wise operations"; the
 * recurrent layers of Sec. 4): FP16 tensors, FP32 math.  The products that
 * feed it (time-batched x W_x, per-step r W_r, projection h W_p) are
 * mpt_gemm_fwd calls.  Gate order (i, f, g, o) along the 4H axis; the paper
 * prints no cell equations, the customary ones are used:
 *   a = gx + gr (+ bias);  i,f,o = sigmoid(a_i, a_f, a_o);  g = tanh(a_g)
 *   c = f * c_prev + i * g;   h = o * tanh(c)              (tanh of the unrounded c)
 *   stores act = rne16(i,f,g,o) [B,4H], c [B,H], h [B,H]
 * backward, from the stored act, c, c_prev, the gradient dh of h and the
 * state gradient dc_next carried from the next step (NULL = 0):
 *   tc = tanh(c);  dc = dh*o*(1 - tc^2) + dc_next
 *   da = ( dc*g*i(1-i), dc*c_prev*f(1-f), dc*i*(1-g^2), dh*tc*o(1-o) )   dc_prev = dc * f
 * gr and bias (FP32[4H]) may be NULL.  c may alias c_prev and dc_prev may
 * alias dc_next (each element is read and written by the same thread);
 * otherwise outputs must not overlap inputs.  Row strides are in elements.
 * 16-byte accesses when H % 8 == 0 and every tensor is 16-byte aligned with
 * a stride that is a multiple of 8; else element-wise, same results.
 * Results agree with an FP64 evaluation to within one FP16 step (hardware
 * exponential and reciprocal, library tanh); they are not specified bit for bit.
 * Errors: NULL, SHAPE (B, H < 1, stride too small), ALIGN.
 * ------------------------------------------------------------------------- */
int mpt_lstm_cell_fwd(void* stream, int64_t B, int64_t H,
                      const uint16_t* gx_dev, int64_t ldgx, const uint16_t* gr_dev, int64_t ldgr, const float* bias_dev,
                      const uint16_t* c_prev_dev, int64_t ldcp,
                      uint16_t* act_dev, int64_t ldact, uint16_t* c_dev, int64_t ldc, uint16_t* h_dev, int64_t ldh);
int mpt_lstm_cell_bwd(void* stream, int64_t B, int64_t H,
                      const uint16_t* dh_dev, int64_t lddh, const uint16_t* dc_next_dev, int64_t lddcn,
                      const uint16_t* act_dev, int64_t ldact, const uint16_t* c_dev, int64_t ldc,
                      const uint16_t* c_prev_dev, int64_t ldcp,
                      uint16_t* da_dev, int64_t ldda, uint16_t* dc_prev_dev, int64_t lddcp);

/* ------------------------------------------------------------------------- *
 * Diagnostic (not a step of the method): the sustained rate of the FP16 MFMA
 * instruction out of registers, with no memory traffic.  The GPU's clock under
 * matrix work depends on the operand bits, so this is the ceiling against which
 * GEMM rates on a given kind of data are read.  One launch runs `iters` x 64
 * v_mfma_f32_16x16x32_f16 per wavefront on 1024 wavefronts (one per SIMD):
 * iters * 64 * 16384 * 1024 FLOP; the caller times it with events.
 * random_operands = 0: all-zero operands; 1: random sign and mantissa, magnitude
 * 2^-5 .. 2^-1.  sink_dev: one FP32 of device memory (never written in practice).
 * Errors: NULL, ARG (iters outside 1 .. 2^20), ALIGN.
 * ------------------------------------------------------------------------- */
int mpt_probe_mfma(void* stream, int iters, int random_operands, float* sink_dev);

#ifdef __cplusplus
}
#endif
#endif /* MPT_H */
