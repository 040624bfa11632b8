/*
 * rn50_hip.h — C ABI of the MI355X (gfx950) library that runs one worker's share
 * of the large-minibatch ResNet-50 training step: convolution forward /
 * data-gradient / weight-gradient, fused BatchNorm+ReLU forward / backward,
 * pooling, the classifier, softmax cross-entropy and the layer-wise LARS +
 * momentum update of single-precision master weights.
 *
 * Conventions (all functions)
 *  - Every pointer called "device" is GPU memory owned by the caller; the
 *    library never allocates, frees or synchronizes, and creates no streams.
 *    All work is enqueued in order on `stream` (a hipStream_t passed as void*;
 *    NULL = the default stream).  Pointers called "host" are ordinary CPU memory
 *    read during the call only.
 *  - Activations are NHWC, convolution weights KRSC (output channel, filter
 *    row, filter column, input channel), all contiguous; every device base
 *    pointer must be 16-byte aligned.
 *  - dtype: RN50_F32 (float) or RN50_BF16 (bfloat16 storage, float arithmetic
 *    and accumulation).  Per-channel BN vectors, gradients of parameters,
 *    logits and the loss are always float.
 *  - Return value: 0 on success, negative on error; on error nothing has been
 *    launched.  rn50_last_error() returns a thread-local description.
 *  - Scratch memory: each operation has a *_workspace_bytes() query; pass a
 *    device buffer of at least that size (16-byte aligned).  Its contents on
 *    entry are irrelevant and on return unspecified.
 */
#ifndef RN50_HIP_H
#define RN50_HIP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define RN50_OK 0
#define RN50_ERR_INVALID (-1)     /* null pointer, non-positive size, bad enum       */
#define RN50_ERR_UNSUPPORTED (-2) /* shape / dtype / layout the kernels do not cover */
#define RN50_ERR_WORKSPACE (-3)   /* workspace smaller than *_workspace_bytes()      */
#define RN50_ERR_ALIGN (-4)       /* a device pointer is not 16-byte aligned         */
#define RN50_ERR_HIP (-5)         /* the HIP runtime reported an error at launch     */

#define RN50_F32 0
#define RN50_BF16 1

/* Thread-local text of the last error returned on this thread ("" if none). */
const char* rn50_last_error(void);
/* Library version, for the binding's sanity check. */
int rn50_version(void);

/* Measurement aid (not part of the method): while enabled, every launch whose kernel
 * tag begins with `kernel_tag` ("conv_fwd", "conv_dgrad", "conv_wgrad", "splitk_reduce"
 * (the second pass of a split weight gradient), "bn_stats", "bn_finalize", "bn_apply", "bn_bwd_reduce",
 * "bn_bwd_finalize", "bn_bwd_apply", "lars_norms", "lars_apply", "fc_bwd_da"; the empty
 * string matches every tagged launch) is given a HIP event pair that receives the begin and end timestamps of that dispatch
 * on the launch stream, up to max_records launches.  rn50_profile_end waits for the
 * last recorded launch, writes the milliseconds each recorded kernel ran, in launch
 * order, to ms_out (host, capacity floats), disables recording and returns the number
 * of records; rn50_profile_tag(i) then names the kernel tag of record i (until the next
 * rn50_profile_begin).  A timed launch costs a few microseconds more than a plain one, so a caller
 * timing whole steps can sample: rn50_profile_pause(1) suspends recording (launches are
 * plain again), rn50_profile_pause(0) resumes it.  Events are the only resource created;
 * all three calls are host-side and not thread-safe. */
int rn50_profile_begin(const char* kernel_tag, int max_records);
void rn50_profile_pause(int paused);
int rn50_profile_end(float* ms_out, int capacity);
/* As rn50_profile_end; also writes to start_ms_out (host, capacity floats; may be NULL) when each
 * recorded dispatch began, in milliseconds after the begin of the first recorded one: with the
 * durations, the timeline of the step's launches on all of its streams. */
int rn50_profile_end_timeline(float* ms_out, float* start_ms_out, int capacity);
const char* rn50_profile_tag(int record);

/* ------------------------------------------------------------------ convolution
 * y[n,p,q,k] = sum_{r,s,c} x[n, p*stride-pad+r, q*stride-pad+s, c] * w[k,r,s,c]
 * (cross-correlation, zero padding, no bias: the paper's appendix logs
 * "use_bias: false" for its convolutions), with Ho = (H+2*pad-R)/stride+1.
 * Supported: Cin % 8 == 0 (bf16) or % 4 == 0 (f32), or the stem case Cin == 3
 * with R == S == 7, stride 2, pad 3; Cout % 8 == 0. */
typedef struct {
  int N, H, W, Cin, Cout, R, S, stride, pad;
  int dtype; /* RN50_F32 or RN50_BF16: storage type of x, w, y, dy, dx */
} rn50_conv_desc;

size_t conv_fwd_workspace_bytes(const rn50_conv_desc* d);
size_t conv_dgrad_workspace_bytes(const rn50_conv_desc* d);
size_t conv_wgrad_workspace_bytes(const rn50_conv_desc* d);

/* Forward.  x [N,H,W,Cin], w [Cout,R,S,Cin], y [N,Ho,Wo,Cout]: device, dtype. */
int conv_fwd(const rn50_conv_desc* d, const void* x, const void* w, void* y, void* workspace,
             size_t workspace_bytes, void* stream);
/* Data gradient: dx[n,h,w,c] = sum over (k,r,s) with h = p*stride-pad+r,
 * w = q*stride-pad+s of dy[n,p,q,k] * w[k,r,s,c].  dy [N,Ho,Wo,Cout], dx [N,H,W,Cin]. */
int conv_dgrad(const rn50_conv_desc* d, const void* dy, const void* w, void* dx, void* workspace,
               size_t workspace_bytes, void* stream);
/* Weight gradient: dw[k,r,s,c] = sum_{n,p,q} dy[n,p,q,k] * x[n,p*stride-pad+r,q*stride-pad+s,c].
 * dw is always float [Cout,R,S,Cin] (it feeds the single-precision update). */
int conv_wgrad(const rn50_conv_desc* d, const void* x, const void* dy, float* dw, void* workspace,
               size_t workspace_bytes, void* stream);

/* ------------------------------------------------------- batch norm (+ReLU, +add)
 * Training-mode batch normalization over the local batch only (the paper keeps
 * BN statistics per process, Sec. III-A3; appendix: epsilon 1e-5, scale and
 * centre on, moving-average momentum 0.9), fused with what follows it in a
 * bottleneck block.  With m = N*H*W and per channel c:
 *   mu = mean_m x, var = mean_m (x-mu)^2, rstd = 1/sqrt(var+eps), xhat = (x-mu)*rstd
 *   v = gamma*xhat + beta
 *   mode 0: y = v          mode 1: y = max(v,0)      mode 2: y = max(v+residual,0)
 * C % 8 == 0 (bf16) or % 4 == 0 (f32). */
typedef struct {
  int N, H, W, C;
  float eps;
  int dtype;
  int mode;
} rn50_bn_desc;

size_t bn_relu_fwd_workspace_bytes(const rn50_bn_desc* d);
size_t bn_relu_bwd_workspace_bytes(const rn50_bn_desc* d);

/* x, y, residual (mode 2 only, else NULL): device [m,C] dtype.  gamma, beta,
 * save_mean, save_rstd: device float[C] (save_* are outputs kept for backward).
 * running_mean / running_var: device float[C] or NULL; when given they are
 * updated in place as running = momentum*running + (1-momentum)*batch statistic
 * (biased variance).  relu_mask: device uint8 [m*C/V] or NULL, V = 8 (bf16) / 4 (f32)
 * elements per 16-byte vector; when given (modes 1, 2) it receives, per vector, bit j =
 * [stored y_j > 0]: the ReLU decisions, for a backward pass that then need not read y. */
int bn_relu_fwd(const rn50_bn_desc* d, const void* x, const float* gamma, const float* beta,
                const void* residual, void* y, uint8_t* relu_mask, float* save_mean,
                float* save_rstd, float* running_mean, float* running_var, float momentum,
                void* workspace, size_t workspace_bytes, void* stream);
/* Backward of the above.  dz (and optional dz2, summed with it: the two branches
 * that consume a block's output), x: device [m,C] dtype.  The ReLU mask is
 * z > 0, taken from relu_mask (the bits bn_relu_fwd recorded) when it is given, else
 * from z (the forward output) when z != NULL; in mode 1 both may be NULL and the mask
 * is recomputed from x, gamma, beta (required then).  Mode 2 needs relu_mask or z.
 * g = (dz+dz2)*mask;  dbeta = sum_m g;  dgamma = sum_m g*xhat;
 * dx = gamma*rstd*(g - dbeta/m - xhat*dgamma/m);  mode 2: dresidual = g (NULL: not stored).
 * dx, dresidual: device [m,C] dtype; dgamma, dbeta: device float[C]. */
int bn_relu_bwd(const rn50_bn_desc* d, const void* dz, const void* dz2, const void* x,
                const void* z, const uint8_t* relu_mask, const float* gamma, const float* beta, const float* save_mean,
                const float* save_rstd, void* dx, void* dresidual, float* dgamma, float* dbeta,
                void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------- convolution + batch norm with fused sums
 * The same operations, with the per-channel sums of the batch norm taken in the
 * output stage of the convolution that produces the tensor they range over
 * (one row of partial sums per output tile), so that no separate pass re-reads
 * that tensor.
 * Forward: conv_fwd_bn_sums produces y and `sums`; bn_relu_fwd_from_sums(d, producer,
 * y, sums, ...) then gives what bn_relu_fwd(d, y, ...) gives.
 * Backward, for a BN layer with ReLU (mode 1 or 2) whose output z feeds the
 * convolution `producer`: conv_dgrad_bn_sums computes
 *   dz = data gradient of that convolution (+ addend, when z has a second consumer
 *        whose gradient is already known: device [N,H,W,Cin] dtype or NULL; the sum is
 *        formed in float and rounded once.  With addend_mask, the ReLU bits a residual-add
 *        BN layer recorded, the addend is that layer's unmasked output gradient and counts
 *        only where its bit is set: the identity shortcut's gradient, taken without a copy),
 * stores it in dx, and takes the sums over g = dz*[z>0] and g*xhat of the BN layer
 * (bn_x: the BN layer's input, [N,H,W,Cin]; relu_mask: the bits its forward pass
 * recorded, or NULL in mode 1 to recompute the decision from bn_x; gamma, beta,
 * save_mean, save_rstd: the layer's, device float[Cin]).  bn_relu_bwd_from_sums then
 * gives what bn_relu_bwd(d, dz, NULL, x, ...) gives (mode 2: relu_mask required).  The sums are formed from the rounded values that are stored, in a fixed
 * order.
 * sums: device float, conv_bn_sums_bytes(d) bytes (16-byte aligned), layout private
 * to the pair of calls; `producer` must be the descriptor the sums were made with. */
size_t conv_bn_sums_bytes(const rn50_conv_desc* d);
int conv_fwd_bn_sums(const rn50_conv_desc* d, const void* x, const void* w, void* y, float* sums,
                     size_t sums_bytes, void* workspace, size_t workspace_bytes, void* stream);
int bn_relu_fwd_from_sums(const rn50_bn_desc* d, const rn50_conv_desc* producer, const void* x,
                          const float* sums, const float* gamma, const float* beta,
                          const void* residual, void* y, uint8_t* relu_mask, float* save_mean,
                          float* save_rstd, float* running_mean, float* running_var, float momentum,
                          void* stream);
int conv_dgrad_bn_sums(const rn50_conv_desc* d, const void* dy, const void* w, void* dx,
                       const void* addend, const uint8_t* addend_mask, const void* bn_x, const uint8_t* relu_mask,
                       const float* gamma, const float* beta, const float* save_mean,
                       const float* save_rstd, float* sums, size_t sums_bytes, void* workspace,
                       size_t workspace_bytes, void* stream);
int bn_relu_bwd_from_sums(const rn50_bn_desc* d, const rn50_conv_desc* producer, const void* dz,
                          const void* x, const uint8_t* relu_mask, const float* gamma,
                          const float* beta, const float* save_mean, const float* save_rstd,
                          const float* sums, void* dx, void* dresidual, float* dgamma, float* dbeta,
                          void* stream);

/* ----------------------- convolution whose input is a BN+ReLU layer's output, applied on the fly
 * The other half of the convolution <-> batch-norm fusion: a 1x1, stride-1, unpadded convolution
 * (conv3 of a bottleneck block) reads the INPUT x of the BN+ReLU layer in front of it and applies
 *   z = max(gamma*(x-mean)*rstd + beta, 0)     (mode 1 of bn_relu_fwd, rounded once to dtype)
 * to every operand vector after it has been loaded, so that z is never stored and the stand-alone
 * BN pass over it disappears.  The results are bit for bit those of conv_fwd / conv_wgrad on the z
 * that bn_relu_fwd stores (same arithmetic, same rounding).
 * in_gamma, in_beta, in_mean, in_rstd: device float[Cin], the BN layer's parameters and the
 * statistics its forward pass saved.  x [N,H,W,Cin]: that layer's input.  conv_fwd_bn_in: sums
 * (or NULL) as in conv_fwd_bn_sums, for the BN layer BEHIND this convolution.  Unsupported
 * (RN50_ERR_UNSUPPORTED): any filter other than 1x1 / stride 1 / pad 0, Cin > 4096. */
int conv_fwd_bn_in(const rn50_conv_desc* d, const void* x, const float* in_gamma, const float* in_beta,
                   const float* in_mean, const float* in_rstd, const void* w, void* y, float* sums,
                   size_t sums_bytes, void* stream);
int conv_wgrad_bn_in(const rn50_conv_desc* d, const void* x, const float* in_gamma, const float* in_beta,
                     const float* in_mean, const float* in_rstd, const void* dy, float* dw, void* workspace,
                     size_t workspace_bytes, void* stream);

/* --------------------------------------------------------------------- pooling
 * Max pooling, window 3x3, stride 2, pad 1 (the appendix's 112 -> 56 step);
 * padding never wins; among equal maxima the first in row-major window order
 * wins.  Forward optionally records the winner's window position r*3+s per output
 * element in argmax (device uint8 [N,Ho,Wo,C], or NULL).  Backward adds dy (+ optional
 * dy2) to the winner, taken from argmax when given, else recomputed from x (then x is
 * required).  x, dx [N,H,W,C]; y, dy, dy2 [N,Ho,Wo,C]; device, dtype; C % 8 == 0
 * (bf16) or % 4 (f32). */
int maxpool_fwd(int N, int H, int W, int C, int dtype, const void* x, void* y, uint8_t* argmax,
                void* stream);
int maxpool_bwd(int N, int H, int W, int C, int dtype, const void* x, const uint8_t* argmax,
                const void* dy, const void* dy2, void* dx, void* stream);
/* Global average pool over the HW positions of each image and its adjoint.
 * x, dx [N,HW,C]; y, dy [N,C]; device, dtype. */
int avgpool_fwd(int N, int HW, int C, int dtype, const void* x, void* y, void* stream);
int avgpool_bwd(int N, int HW, int C, int dtype, const void* dy, void* dx, void* stream);

/* ------------------------------------------------------------------ classifier
 * logits[n,k] = sum_c a[n,c]*W[k,c] + b[k].  a [N,Cin], W [K,Cin]: device dtype;
 * b, logits: device float; Cin a multiple of the 16-byte vector.  Backward:
 * da[n,c] = sum_k dlogits[n,k]*W[k,c] (dtype; dlogits is rounded to dtype for this product),
 * dW[k,c] = sum_n dlogits[n,k]*a[n,c], db[k] = sum_n dlogits[n,k] (float); with dW and db both
 * NULL the parameter gradients are left out (da only). */
int fc_fwd(int N, int Cin, int K, int dtype, const void* a, const void* W, const float* b,
           float* logits, void* stream);
size_t fc_bwd_workspace_bytes(int N, int Cin, int K, int dtype);
int fc_bwd(int N, int Cin, int K, int dtype, const void* a, const void* W, const float* dlogits,
           void* da, float* dW, float* db, void* workspace, size_t workspace_bytes, void* stream);

/* ----------------------------------------------------- softmax cross-entropy
 * With label smoothing (Sec. III-A2 of the paper).  Per row n: p = softmax(logits[n,:])
 * (maximum subtracted first), q_k = (1-ls)*[k==label]+ls/K, row_loss[n] = -sum_k q_k log p_k,
 * loss = mean_n row_loss, dlogits[n,k] = grad_scale*(p_k-q_k)/N.
 * logits, dlogits: device float [N,K]; labels: device int32[N] in [0,K);
 * loss_out: device float[1]; row_loss_out: device float[N] (required: the mean is
 * taken over it in a fixed order).  A label outside [0,K) matches no class.  K <= 65536. */
int xent_fwd_bwd(int N, int K, const float* logits, const int32_t* labels, float label_smoothing,
                 float grad_scale, float* loss_out, float* row_loss_out, float* dlogits,
                 void* stream);

/* ------------------------------------------------------------------------ LARS
 * Layer-wise adaptive rate scaling with momentum over a table of parameter
 * tensors ("layers", Sec. III-A1), the norms of all tensors computed by one
 * batched launch (Sec. III-B2), on single-precision master weights (Sec. IV):
 *   wn = ||w||_2, gn = ||g||_2
 *   local = eta*wn/(gn + weight_decay*wn + eps)  if apply_trust && wn>0 && gn>0, else 1
 *   v <- momentum*v + lr*local*(g + weight_decay*w);   w <- w - v
 *   w_lowp <- bf16(w) when w_lowp != NULL (the model copy of mixed precision). */
typedef struct {
  float* w;       /* device float[n], updated in place                       */
  const void* g;  /* device gradient[n]: float, or bf16 when grad_dtype is BF16 */
  float* v;       /* device float[n] momentum buffer, updated in place       */
  void* w_lowp;   /* device bf16[n] or NULL                                   */
  int64_t n;
  float weight_decay;
  int apply_trust;
} rn50_lars_tensor;

typedef struct {
  int num_tensors;
  float eta, momentum, lr, eps;
  int grad_dtype;
} rn50_lars_desc;

size_t lars_update_workspace_bytes(const rn50_lars_desc* d, const rn50_lars_tensor* table_host);
/* table_host: host array[num_tensors]; table_dev: a device copy of the same
 * array (made by the caller).  norms_out: device float[num_tensors*2] receiving
 * (||w||, ||g||) per tensor, or NULL. */
int lars_update(const rn50_lars_desc* d, const rn50_lars_tensor* table_host,
                const rn50_lars_tensor* table_dev, float* norms_out, void* workspace,
                size_t workspace_bytes, void* stream);
/* lars_update for callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): same arguments, arithmetic and
 * results as lars_update, but the partial norms live in a device array built into the library
 * (256 KB, held on every GPU the library runs on until the process ends) instead of a caller
 * workspace, and the call allocates nothing.  Limit: the table's tensors may need at most
 * lars_update_noalloc_max_chunks() chunks of 8192 elements in all (one chunk per started 8192
 * elements of each tensor; 32768 chunks, i.e. up to 268 M parameters); a larger table
 * is rejected with RN50_ERR_WORKSPACE and nothing is launched.  All calls on one GPU share that
 * array: calls that overlap in time on one GPU (different streams or threads) race; calls on
 * one stream, or otherwise ordered, are safe.  Nothing in the array has to survive between
 * calls. */
int64_t lars_update_noalloc_max_chunks(void);
int lars_update_noalloc(const rn50_lars_desc* d, const rn50_lars_tensor* table_host,
                        const rn50_lars_tensor* table_dev, float* norms_out, void* stream);

/* ----------------------------------------------------------------- whole step
 * One training step of ResNet-50 v1.5 on the local batch: forward, softmax
 * cross-entropy, backward, LARS update of every parameter tensor (the gradient
 * exchange between workers, Sec. III-C, would sit between backward and LARS and
 * is not part of this library).
 *
 * Parameter order (161 tensors for the full network): stem W, gamma, beta; per
 * bottleneck block conv1 W, gamma, beta, conv2 ..., conv3 ..., and, in the first
 * block of a stage, projection W, gamma, beta; then FC W, FC b. */
typedef struct {
  int N;          /* local batch                                    */
  int image_hw;   /* input height = width (224)                      */
  int classes;    /* 1000                                            */
  int dtype;      /* RN50_BF16: mixed precision; RN50_F32: all float */
  int widths[4];  /* bottleneck widths per stage: 64,128,256,512     */
  int blocks[4];  /* blocks per stage: 3,4,6,3                       */
  int stem;       /* stem filters: 64                                */
  int expansion;  /* block output = expansion*width: 4               */
  float bn_eps;   /* 1e-5 */
  float label_smoothing, grad_scale;
  float eta, momentum, weight_decay, lars_eps; /* LARS; weight decay on conv/FC weights only */
} rn50_step_config;

typedef struct rn50_plan rn50_plan; /* host-side object (layout, two streams, events); holds no device memory */

/* Checks every layer's shape against what the kernels cover (so that a step cannot fail on a
 * shape half-way through) and lays out the workspace.  On error no plan is returned. */
int resnet_plan_create(const rn50_step_config* cfg, rn50_plan** plan_out);
void resnet_plan_destroy(rn50_plan* plan);
/* Creates the plan's two streams and their events now instead of at the first step (needs the
 * GPU; all or nothing; a second call is a no-op).  Call it before capturing a step into a graph
 * when no step has run outside the capture yet. */
int resnet_plan_prepare(rn50_plan* plan);
/* on != 0: in every bottleneck block, conv3 applies conv2's BN+ReLU while it loads its operand
 * (conv_fwd_bn_in in the forward pass, conv_wgrad_bn_in for conv3's weight gradient): conv2's BN
 * pass only finalises its statistics and its normalised output is never stored.  Results of the
 * step are bit for bit the same either way; only the time differs.  Off when the plan is created.
 * Applies to resnet_step / resnet_train_step (resnet_infer always stores every layer's output). */
int resnet_plan_fuse_conv3_input(rn50_plan* plan, int on);
int resnet_plan_num_tensors(const rn50_plan* plan);
/* Shape of parameter tensor i: dims_out[4] = {K,R,S,C} for convolution weights,
 * {K,C,0,0} for the FC weight, {C,0,0,0} for vectors.  Returns the element count. */
int64_t resnet_plan_tensor_shape(const rn50_plan* plan, int i, int dims_out[4]);
/* Element offset of tensor i inside each parameter arena (multiple of 64). */
int64_t resnet_plan_tensor_offset(const rn50_plan* plan, int i);
/* Total elements of one parameter arena, and the device workspace the step needs. */
int64_t resnet_plan_arena_elems(const rn50_plan* plan);
size_t resnet_plan_workspace_bytes(const rn50_plan* plan);

/* Arenas (device, each resnet_plan_arena_elems long, tensors at their offsets):
 *   master  float  : master weights, updated in place by LARS
 *   velocity float : momentum buffers, updated in place
 *   grads   float  : gradients of this step (output)
 *   model   dtype  : the weights the forward/backward passes read; in BF16 mode the
 *                    bf16 copy, refreshed from master by the LARS update; in F32
 *                    mode pass the master arena itself.
 * images: device [N,hw,hw,3] dtype (NHWC); labels: device int32[N].
 * loss_out: device float[1]; logits_out: device float[N,classes] or NULL.
 * lr: the learning rate of this step (schedules live with the caller).
 * If update == 0 the step stops after backward (gradients only).
 * Errors: every argument is checked before the first launch (the shapes at plan creation, the
 * pointers, alignment and workspace here); after that only a launch failure reported by the HIP
 * runtime (RN50_ERR_HIP) can end a step early, with the kernels enqueued so far left to run.
 * Stream semantics: everything is ordered after the work `stream` holds at the call and
 * is complete when the work this call enqueues on `stream` is.  Inside, independent parts
 * (weight gradients, the projection shortcuts, the weight transposition) run on two
 * streams the plan creates at its first step (default priority; host-side handles, no
 * device memory) and are forked from / joined into `stream` with events; the fork/join
 * can be captured into a graph together with `stream`.  One step at a time per plan. */
int resnet_step(rn50_plan* plan, const void* images, const int32_t* labels, float* master,
                float* velocity, float* grads, void* model, float lr, int update, float* loss_out,
                float* logits_out, void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------- training loop
 * The inner loop of the paper's training with its optimizer controls (Sec. III-A): the
 * learning rate follows a gradual warm-up and then one of the decay patterns the paper
 * lists (step, polynomial, linear) or a table the caller supplies; label smoothing is the
 * plan's; every BN layer keeps moving averages of its batch mean and (biased) batch
 * variance (Sec. III-A2; appendix log: momentum 0.9).  The step counter, the learning rate
 * and the moving averages live in device memory, so a step takes no per-step host values
 * and a captured graph of it can be replayed step after step.
 *
 * lr(t), t = 0, 1, ... (computed on the device in double, stored as float):
 *   t < warmup_steps:  warmup_start_lr + (base_lr - warmup_start_lr)*t/warmup_steps
 *   else, u = t - warmup_steps, D = total_steps - warmup_steps:
 *     RN50_DECAY_NONE    base_lr
 *     RN50_DECAY_STEP    base_lr * step_factor^floor(u/step_every)
 *     RN50_DECAY_POLY    end_lr + (base_lr - end_lr)*(1 - min(u,D)/D)^power
 *     RN50_DECAY_LINEAR  the polynomial with power 1
 *   RN50_DECAY_TABLE     table[min(t, table_len-1)] for every t (warm-up fields ignored) */
#define RN50_DECAY_NONE 0
#define RN50_DECAY_STEP 1
#define RN50_DECAY_POLY 2
#define RN50_DECAY_LINEAR 3
#define RN50_DECAY_TABLE 4
typedef struct {
  float base_lr, warmup_start_lr;
  int warmup_steps;
  int decay;          /* RN50_DECAY_*                                        */
  int total_steps;    /* POLY, LINEAR: > warmup_steps                        */
  float end_lr, power;
  int step_every;     /* STEP: > 0                                           */
  float step_factor;
  const float* table; /* TABLE: device float[table_len], read at every step  */
  int table_len;
} rn50_lr_schedule;

/* Training state: one device buffer of resnet_train_state_bytes(plan) bytes, owned by the caller:
 *   byte 0    int64  t, the number of steps taken (the next step uses lr(t))
 *   byte 8    float  the learning rate of the last step taken
 *   byte 256  float  running_mean[resnet_plan_bn_channels(plan)]
 *   then      float  running_var [resnet_plan_bn_channels(plan)]
 * BN layer i (0 .. resnet_plan_num_bn-1, parameter order: stem, then per block conv1, conv2,
 * conv3, projection) owns the C_i entries starting at resnet_plan_bn_offset(plan, i, &C_i) of
 * both arrays (offsets are multiples of 64; the entries in the gaps are not used). */
int resnet_plan_num_bn(const rn50_plan* plan);
int64_t resnet_plan_bn_channels(const rn50_plan* plan);
int64_t resnet_plan_bn_offset(const rn50_plan* plan, int i, int* channels_out);
size_t resnet_train_state_bytes(const rn50_plan* plan);
/* t = first_step, running means 0, running variances 1.  Enqueued on `stream`. */
int resnet_train_state_init(const rn50_plan* plan, void* state, size_t state_bytes, int64_t first_step,
                            void* stream);
/* One step of the loop: resnet_step (same arenas, workspace and stream semantics, update
 * always on) with lr = lr(t) taken from the state on the device, the moving averages
 * updated as running <- bn_momentum*running + (1-bn_momentum)*batch statistic, and t
 * advanced by one.  `schedule` is read at the call (its table at run time).  Errors as
 * resnet_step, plus RN50_ERR_INVALID for an inconsistent schedule. */
int resnet_train_step(rn50_plan* plan, const rn50_lr_schedule* schedule, void* state, float bn_momentum,
                      const void* images, const int32_t* labels, float* master, float* velocity,
                      float* grads, void* model, float* loss_out, float* logits_out, void* workspace,
                      size_t workspace_bytes, void* stream);

/* ------------------------------------------------- seeded parallel initialization
 * Sec. III-B1: every worker holds the same seed and fills its own copy of the parameters,
 * in parallel, so no broadcast is needed.  Each value is a function of (seed, tensor index,
 * element index) alone: the first 32-bit output x0 of Philox4x32-10 (Salmon et al., SC'11)
 * for counter (element low word, element high word, tensor index, 0) and key (seed low word,
 * seed high word); u = (x0 + 1/2)/2^32; z = Phi^-1(Phi(-2) + u*(Phi(2) - Phi(-2))), the
 * truncated-normal initializer of the appendix log cut at two standard deviations;
 * weight = sqrt(2/fan_in)*z (He scaling; fan_in = R*S*Cin, or Cin for the FC layer), BN gamma 1,
 * BN beta and the FC bias 0, gaps between tensors 0.  The element index is the flat index in
 * the tensor's own (KRSC) layout.  Fills the whole master arena; velocity (or NULL) is
 * zeroed; in BF16 mode `model` (or NULL) receives the rounded copy. */
int resnet_init_params(const rn50_plan* plan, uint64_t seed, float* master, float* velocity, void* model,
                       void* stream);

/* ------------------------------------------------------------------ evaluation
 * BN in evaluation mode: y = gamma*(x - running_mean)/sqrt(running_var + eps) + beta, then the
 * mode's tail as in bn_relu_fwd.  workspace: bn_relu_infer_workspace_bytes (one float per channel). */
size_t bn_relu_infer_workspace_bytes(const rn50_bn_desc* d);
int bn_relu_infer(const rn50_bn_desc* d, const void* x, const float* gamma, const float* beta,
                  const float* running_mean, const float* running_var, const void* residual, void* y,
                  void* workspace, size_t workspace_bytes, void* stream);
/* pred_out[n] = the first maximum of logits[n,:] (device int32[N]); correct_out[0] = the number
 * of rows with pred_out[n] == labels[n] (device int32[1]). */
int top1_accuracy(int N, int K, const float* logits, const int32_t* labels, int32_t* pred_out,
                  int32_t* correct_out, void* stream);
/* The forward pass of the plan's network in evaluation mode on one batch (appendix log:
 * eval_accuracy), with the moving averages of a training state (read only), then top1_accuracy.
 * Arenas, images, workspace as in resnet_step (the same workspace size); everything runs on
 * `stream`; logits_out may be NULL. */
int resnet_eval(rn50_plan* plan, const void* state, const void* images, const int32_t* labels,
                const float* master, const void* model, float* logits_out, int32_t* pred_out,
                int32_t* correct_out, void* workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* RN50_HIP_H */
