// resnet_step: the launch sequence of one ResNet-50 v1.5 training step on the
// local batch (forward, softmax cross-entropy, backward, LARS) on the caller's
// stream plus two private streams for work off the critical path (weight
// gradients, projection shortcuts), using a caller-provided workspace.  Wiring follows the paper's
// appendix log (stem convolution stride 2 / 64 filters / no bias -> BN -> ReLU
// -> max-pool 112 -> 56, bottleneck blocks) and He et al.; the gradient exchange
// between workers (Sec. III-C) would sit between backward and the LARS call.
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <memory>
#include <vector>

#include "common.h"
#include "step_internal.h"

namespace rn50 {

struct Unit {  // convolution + BN (+ReLU / +add+ReLU)
  rn50_conv_desc conv;
  rn50_bn_desc bn;
  int iw, ig, ib;        // parameter tensor indices: weight, gamma, beta
  size_t y, z;           // workspace offsets of the conv output and the BN output
  size_t dy;             // workspace offset of the gradient with respect to the conv output
  size_t mean, rstd;     // workspace offsets (float[C])
  size_t relu_mask;      // residual-add layers: the ReLU decision bits (1 byte per 16-byte vector of z)
  int64_t bn_off;        // first entry of this BN layer in the moving-average arrays of a training state
  int P, Q;
};

struct Block {
  int u1, u2, u3, up;  // unit indices; up = -1 without projection
};

struct Tensor {
  int dims[4];
  int64_t count, offset;
  bool decay;
  int fan_in;  // weights: inputs per output (He scaling of the initializer); 0: BN gamma (ones); -1: zeros
};

}  // namespace rn50

struct rn50_plan {
  rn50_step_config cfg;
  std::vector<rn50::Tensor> tensors;
  std::vector<rn50::Unit> units;
  std::vector<rn50::Block> blocks;
  int64_t arena_elems = 0;
  int64_t bn_channels = 0;  // length of the moving-average arrays (every layer's share rounded up to 64)
  int es = 2;  // element size of the activation dtype
  int fc_in = 0, final_hw = 0;
  // workspace layout (byte offsets)
  size_t ws_bytes = 0;
  size_t xp = 0, wp = 0, pool = 0, avg = 0, logits = 0, dlogits = 0, row_loss = 0, davg = 0;
  size_t g[5] = {0, 0, 0, 0, 0};
  size_t wT = 0, wgrad_scratch = 0, bn_scratch = 0, lars_scratch = 0, pool_argmax = 0, fc_scratch = 0;
  size_t bn_scratch_bytes = 0, fc_scratch_bytes = 0;
  std::vector<rn50::TransposeEntry> transposes;
  rn50::LarsArenaSpec lars_rest, lars_stem;  // every tensor but the stem's weight / the stem's weight
  size_t lars_stem_scratch = 0;
  // Second stream for the work that is off the step's critical path (weight gradients, the weight
  // transposition), with the events that order it against the caller's stream.  Created at the first
  // step (default priority), destroyed with the plan.
  hipStream_t side = nullptr;
  hipEvent_t ev_fork = nullptr, ev_wt = nullptr;
  // Third stream: the projection shortcut of a stage's first block, forward and backward, runs beside the
  // block's main branch (its own BN scratch; fork/join events reused block after block).
  hipStream_t branch = nullptr;
  hipEvent_t ev_bfork = nullptr, ev_bjoin = nullptr;
  size_t bn_scratch2 = 0;
  std::vector<hipEvent_t> ev_dy, ev_wg;  // per block: its dy tensors are ready / its weight gradients are done
  bool streams_ready = false;            // all of the above exist
  // conv3 of every block applies conv2's BN+ReLU while it loads its operand (forward and weight gradient):
  // conv2's normalised output is then never stored.
  bool fuse_conv3_input = false;
};

using namespace rn50;

namespace {

int add_tensor(rn50_plan* p, int d0, int d1, int d2, int d3, bool decay, bool ones = false) {
  Tensor t;
  t.dims[0] = d0; t.dims[1] = d1; t.dims[2] = d2; t.dims[3] = d3;
  t.count = 1;
  for (int i = 0; i < 4; ++i)
    if (t.dims[i] > 0) t.count *= t.dims[i];
  t.fan_in = decay ? static_cast<int>(t.count / d0) : (ones ? 0 : -1);
  t.offset = p->arena_elems;
  t.decay = decay;
  p->arena_elems += (t.count + 63) / 64 * 64;
  p->tensors.push_back(t);
  return static_cast<int>(p->tensors.size()) - 1;
}

int add_unit(rn50_plan* p, int N, int H, int W, int Cin, int Cout, int R, int stride, int pad, int mode) {
  Unit u{};
  u.conv = rn50_conv_desc{N, H, W, Cin, Cout, R, R, stride, pad, p->cfg.dtype};
  u.P = (H + 2 * pad - R) / stride + 1;
  u.Q = (W + 2 * pad - R) / stride + 1;
  u.bn = rn50_bn_desc{N, u.P, u.Q, Cout, p->cfg.bn_eps, p->cfg.dtype, mode};
  u.iw = add_tensor(p, Cout, R, R, Cin, true);
  u.ig = add_tensor(p, Cout, 0, 0, 0, false, true);
  u.ib = add_tensor(p, Cout, 0, 0, 0, false);
  u.bn_off = p->bn_channels;
  p->bn_channels += (Cout + 63) / 64 * 64;
  p->units.push_back(u);
  return static_cast<int>(p->units.size()) - 1;
}

size_t bump(size_t* top, size_t bytes) {
  const size_t at = *top;
  *top += align_up(bytes, 256);
  return at;
}

}  // namespace

extern "C" int resnet_plan_create(const rn50_step_config* cfg, rn50_plan** plan_out) {
  clear_error();
  RN50_REQUIRE(cfg && plan_out, RN50_ERR_INVALID, "resnet_plan_create: null pointer");
  RN50_REQUIRE(cfg->N > 0 && cfg->image_hw >= 32 && cfg->classes > 0 && cfg->stem > 0 && cfg->expansion > 0,
               RN50_ERR_INVALID, "resnet_plan_create: bad sizes");
  RN50_REQUIRE(cfg->dtype == RN50_F32 || cfg->dtype == RN50_BF16, RN50_ERR_INVALID, "resnet_plan_create: dtype");
  const int V = cfg->dtype == RN50_BF16 ? 8 : 4;
  RN50_REQUIRE(cfg->stem % V == 0, RN50_ERR_UNSUPPORTED, "resnet_plan_create: stem width %% %d", V);
  for (int i = 0; i < 4; ++i)
    RN50_REQUIRE(cfg->widths[i] > 0 && cfg->widths[i] % V == 0 && cfg->blocks[i] > 0, RN50_ERR_UNSUPPORTED,
                 "resnet_plan_create: stage %d width/blocks", i);
  std::unique_ptr<rn50_plan> owner(new rn50_plan());  // freed on every error path below
  rn50_plan* p = owner.get();
  p->cfg = *cfg;
  p->es = cfg->dtype == RN50_BF16 ? 2 : 4;
  const int N = cfg->N;
  int H = cfg->image_hw;
  const int stem = add_unit(p, N, H, H, 3, cfg->stem, 7, 2, 3, 1);
  (void)stem;
  H = p->units[0].P;          // 112
  const int Hpool = (H - 1) / 2 + 1;  // 56
  H = Hpool;
  int cin = cfg->stem;
  for (int st = 0; st < 4; ++st)
    for (int b = 0; b < cfg->blocks[st]; ++b) {
      const int wd = cfg->widths[st], cout = wd * cfg->expansion;
      const int stride = (b == 0 && st > 0) ? 2 : 1;
      Block blk;
      blk.u1 = add_unit(p, N, H, H, cin, wd, 1, 1, 0, 1);
      blk.u2 = add_unit(p, N, H, H, wd, wd, 3, stride, 1, 1);
      const int Ho = p->units[blk.u2].P;
      blk.u3 = add_unit(p, N, Ho, Ho, wd, cout, 1, 1, 0, 2);
      blk.up = b == 0 ? add_unit(p, N, H, H, cin, cout, 1, stride, 0, 0) : -1;
      p->blocks.push_back(blk);
      H = Ho;
      cin = cout;
    }
  p->fc_in = cin;
  p->final_hw = H;
  add_tensor(p, cfg->classes, cin, 0, 0, true);
  add_tensor(p, cfg->classes, 0, 0, 0, false);
  RN50_REQUIRE(p->arena_elems < (1ll << 31), RN50_ERR_UNSUPPORTED, "resnet_plan_create: too many parameters");
  // Every shape-dependent condition that the operations of a step check is checked here, once, so that a
  // step, after its own pointer / alignment / workspace checks, cannot fail on an argument half-way through.
  for (const Unit& u : p->units) {
    if (int rc = conv_desc_check(&u.conv, "resnet_plan_create")) return rc;
    if (int rc = bn_desc_check(&u.bn, "resnet_plan_create")) return rc;
  }
  RN50_REQUIRE(N <= 65535 && p->units[0].P <= 131070, RN50_ERR_UNSUPPORTED,
               "resnet_plan_create: N=%d or image size beyond the pooling kernels' launch grid", N);
  RN50_REQUIRE(cfg->classes <= 65536, RN50_ERR_UNSUPPORTED, "resnet_plan_create: more than 65536 classes");
  RN50_REQUIRE(cin % V == 0, RN50_ERR_UNSUPPORTED, "resnet_plan_create: classifier input width %d", cin);
  RN50_REQUIRE(cfg->label_smoothing >= 0.f && cfg->label_smoothing <= 1.f, RN50_ERR_INVALID,
               "resnet_plan_create: label_smoothing %g", static_cast<double>(cfg->label_smoothing));

  // ---- workspace layout
  size_t top = 0;
  const size_t es = p->es;
  const Unit& u0 = p->units[0];
  p->xp = bump(&top, stem_padded_input_bytes(&u0.conv));
  p->wp = bump(&top, stem_padded_weight_bytes(&u0.conv));
  size_t max_act = 0, max_wT = 0, max_wg = 0, max_bn = 0;
  for (Unit& u : p->units) {
    const size_t out_elems = static_cast<size_t>(N) * u.P * u.Q * u.conv.Cout;
    const size_t in_elems = static_cast<size_t>(N) * u.conv.H * u.conv.W * u.conv.Cin;
    u.y = bump(&top, out_elems * es);
    u.z = bump(&top, out_elems * es);
    u.relu_mask = u.bn.mode == 2 ? bump(&top, out_elems * es / 16) : 0;
    // Every unit keeps its own dy: the weight gradients read them on the side stream as late as they like,
    // and the backward pass never waits for a buffer (all of them together are smaller than a ring of 16
    // buffers of the largest activation, the depth at which a ring stops making the main stream wait).
    u.dy = bump(&top, out_elems * es);
    u.mean = bump(&top, u.conv.Cout * sizeof(float));
    u.rstd = bump(&top, u.conv.Cout * sizeof(float));
    if (out_elems > max_act) max_act = out_elems;
    if (in_elems > max_act && u.conv.Cin != 3) max_act = in_elems;
    if (u.conv.Cin != 3 && dgrad_wt_bytes(&u.conv) > max_wT) max_wT = dgrad_wt_bytes(&u.conv);
    if (wgrad_partial_bytes(&u.conv) > max_wg) max_wg = wgrad_partial_bytes(&u.conv);
    if (bn_relu_fwd_workspace_bytes(&u.bn) > max_bn) max_bn = bn_relu_fwd_workspace_bytes(&u.bn);
    // sums fused into the convolutions: one row per output tile, at most ceil(M/64) rows of 16 bytes per channel
    const size_t fwd_rows = ceil_div(static_cast<int64_t>(N) * u.P * u.Q, 64);
    const size_t dgrad_rows = u.conv.Cin != 3 ? dgrad_partial_rows_bound(&u.conv) : 0;
    max_bn = std::max(max_bn, align_up(fwd_rows * 4 * u.conv.Cout * sizeof(float), 256));
    if (u.conv.Cin != 3) max_bn = std::max(max_bn, align_up(dgrad_rows * 2 * u.conv.Cin * sizeof(float), 256));
  }
  p->pool = bump(&top, static_cast<size_t>(N) * Hpool * Hpool * cfg->stem * es);
  p->avg = bump(&top, static_cast<size_t>(N) * cin * es);
  p->davg = bump(&top, static_cast<size_t>(N) * cin * es);
  p->logits = bump(&top, static_cast<size_t>(N) * cfg->classes * sizeof(float));
  p->dlogits = bump(&top, static_cast<size_t>(N) * cfg->classes * sizeof(float));
  p->row_loss = bump(&top, static_cast<size_t>(N) * sizeof(float));
  for (int i = 0; i < 5; ++i) p->g[i] = bump(&top, max_act * es);
  (void)max_wT;
  p->wT = bump(&top, static_cast<size_t>(p->arena_elems) * es);  // transposed copy of every conv weight
  for (const Unit& u : p->units)
    if (u.conv.Cin != 3)
      p->transposes.push_back(TransposeEntry{p->tensors[u.iw].offset, u.conv.Cout, u.conv.R * u.conv.S, u.conv.Cin});
  p->pool_argmax = bump(&top, static_cast<size_t>(N) * Hpool * Hpool * cfg->stem);
  p->fc_scratch_bytes = fc_bwd_workspace_bytes(N, cin, cfg->classes, cfg->dtype);
  p->fc_scratch = bump(&top, p->fc_scratch_bytes);
  p->wgrad_scratch = bump(&top, max_wg);
  p->bn_scratch = bump(&top, max_bn);
  p->bn_scratch2 = bump(&top, max_bn);
  p->bn_scratch_bytes = max_bn;
  // The stem's weight gradient is the last thing the backward pass produces; the update of every other
  // tensor runs beside it.
  for (size_t i = 0; i < p->tensors.size(); ++i) {
    const Tensor& t = p->tensors[i];
    LarsArenaSpec& sp = i == static_cast<size_t>(p->units[0].iw) ? p->lars_stem : p->lars_rest;
    sp.offset.push_back(t.offset);
    sp.count.push_back(t.count);
    sp.decay.push_back(t.decay ? 1 : 0);
    ++sp.num;
  }
  p->lars_scratch = bump(&top, lars_arena_partial_bytes(p->lars_rest));
  p->lars_stem_scratch = bump(&top, lars_arena_partial_bytes(p->lars_stem));
  p->ws_bytes = top;
  *plan_out = owner.release();
  return RN50_OK;
}

namespace {
void destroy_streams(rn50_plan* p);
}
extern "C" void resnet_plan_destroy(rn50_plan* plan) {
  if (!plan) return;
  destroy_streams(plan);
  delete plan;
}

namespace {
// The side streams and their events (host-side handles only; no device memory).  All or nothing: after a
// failure every handle made so far is destroyed again, so a later call starts from scratch.
void destroy_streams(rn50_plan* p) {
  if (p->side) {
    (void)hipStreamSynchronize(p->side);
    (void)hipStreamDestroy(p->side);
  }
  if (p->branch) {
    (void)hipStreamSynchronize(p->branch);
    (void)hipStreamDestroy(p->branch);
  }
  for (hipEvent_t* e : {&p->ev_bfork, &p->ev_bjoin, &p->ev_fork, &p->ev_wt})
    if (*e) {
      (void)hipEventDestroy(*e);
      *e = nullptr;
    }
  for (hipEvent_t e : p->ev_dy) (void)hipEventDestroy(e);
  for (hipEvent_t e : p->ev_wg) (void)hipEventDestroy(e);
  p->ev_dy.clear();
  p->ev_wg.clear();
  p->side = p->branch = nullptr;
  p->streams_ready = false;
}
int ensure_side_stream(rn50_plan* p) {
  if (p->streams_ready) return RN50_OK;
  auto ok = [](hipError_t e) { return e == hipSuccess; };
  bool good = ok(hipStreamCreateWithFlags(&p->side, hipStreamNonBlocking)) &&
              ok(hipStreamCreateWithFlags(&p->branch, hipStreamNonBlocking)) &&
              ok(hipEventCreateWithFlags(&p->ev_bfork, hipEventDisableTiming)) &&
              ok(hipEventCreateWithFlags(&p->ev_bjoin, hipEventDisableTiming)) &&
              ok(hipEventCreateWithFlags(&p->ev_fork, hipEventDisableTiming)) &&
              ok(hipEventCreateWithFlags(&p->ev_wt, hipEventDisableTiming));
  for (size_t i = 0; good && i < p->blocks.size() + 1; ++i) {  // the blocks and the stem
    hipEvent_t a = nullptr, b = nullptr;
    good = ok(hipEventCreateWithFlags(&a, hipEventDisableTiming)) && ok(hipEventCreateWithFlags(&b, hipEventDisableTiming));
    if (a) p->ev_dy.push_back(a);
    if (b) p->ev_wg.push_back(b);
  }
  if (!good) {
    (void)hipGetLastError();
    destroy_streams(p);
    return fail(RN50_ERR_HIP, "resnet_step: could not create the side streams or their events");
  }
  p->streams_ready = true;
  return RN50_OK;
}
}  // namespace
extern "C" int resnet_plan_prepare(rn50_plan* plan) {
  clear_error();
  RN50_REQUIRE(plan, RN50_ERR_INVALID, "resnet_plan_prepare: null plan");
  return ensure_side_stream(plan);
}
extern "C" int resnet_plan_fuse_conv3_input(rn50_plan* plan, int on) {
  clear_error();
  RN50_REQUIRE(plan, RN50_ERR_INVALID, "resnet_plan_fuse_conv3_input: null plan");
  for (const rn50::Block& b : plan->blocks)
    RN50_REQUIRE(!on || plan->units[b.u3].conv.Cin <= 4096, RN50_ERR_UNSUPPORTED,
                 "resnet_plan_fuse_conv3_input: a conv3 with more than 4096 input channels");
  plan->fuse_conv3_input = on != 0;
  return RN50_OK;
}
extern "C" int resnet_plan_num_tensors(const rn50_plan* plan) {
  return plan ? static_cast<int>(plan->tensors.size()) : 0;
}
extern "C" int64_t resnet_plan_tensor_shape(const rn50_plan* plan, int i, int dims_out[4]) {
  if (!plan || i < 0 || i >= static_cast<int>(plan->tensors.size())) return 0;
  if (dims_out) memcpy(dims_out, plan->tensors[i].dims, sizeof(int) * 4);
  return plan->tensors[i].count;
}
extern "C" int64_t resnet_plan_tensor_offset(const rn50_plan* plan, int i) {
  if (!plan || i < 0 || i >= static_cast<int>(plan->tensors.size())) return -1;
  return plan->tensors[i].offset;
}
extern "C" int64_t resnet_plan_arena_elems(const rn50_plan* plan) { return plan ? plan->arena_elems : 0; }
extern "C" size_t resnet_plan_workspace_bytes(const rn50_plan* plan) { return plan ? plan->ws_bytes : 0; }

#define STEP_TRY(expr)           \
  do {                           \
    const int rc_ = (expr);      \
    if (rc_ != RN50_OK) return rc_; \
  } while (0)

namespace {

// What resnet_train_step adds to a step: the device-side learning rate and step counter, the moving averages.
struct TrainCtl {
  rn50_lr_schedule sched;
  int64_t* t;        // device: steps taken
  float* lr;         // device: the learning rate of the step
  float *run_mean, *run_var;
  float bn_momentum;
};

// lr(t) of the schedule (in double), and t <- t + 1.
__global__ void lr_tick_kernel(const rn50_lr_schedule sc, int64_t* t_ptr, float* lr_out) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  const int64_t t = *t_ptr;
  const double base = sc.base_lr, end = sc.end_lr;
  double lr;
  if (sc.decay == RN50_DECAY_TABLE) {
    lr = sc.table[t < sc.table_len ? (t < 0 ? 0 : t) : sc.table_len - 1];
  } else if (t < sc.warmup_steps) {
    const double start = sc.warmup_start_lr;
    lr = start + (base - start) * (static_cast<double>(t) / sc.warmup_steps);
  } else {
    const int64_t u = t - sc.warmup_steps;
    if (sc.decay == RN50_DECAY_STEP) {
      lr = base * pow(static_cast<double>(sc.step_factor), static_cast<double>(u / sc.step_every));
    } else if (sc.decay == RN50_DECAY_POLY || sc.decay == RN50_DECAY_LINEAR) {
      const int64_t D = sc.total_steps - sc.warmup_steps;
      const double frac = 1.0 - static_cast<double>(u < D ? u : D) / static_cast<double>(D);
      lr = end + (base - end) * (sc.decay == RN50_DECAY_LINEAR ? frac : pow(frac, static_cast<double>(sc.power)));
    } else {
      lr = base;
    }
  }
  *lr_out = static_cast<float>(lr);
  *t_ptr = t + 1;
}

__global__ void train_state_init_kernel(int64_t* t_ptr, float* lr, float* run_mean, float* run_var, int64_t n,
                                        int64_t first_step) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i == 0) {
    *t_ptr = first_step;
    *lr = 0.f;
  }
  if (i < n) {
    run_mean[i] = 0.f;
    run_var[i] = 1.f;
  }
}

constexpr size_t kStateHeader = 256;  // bytes before the moving averages

int run_step(const char* who, rn50_plan* plan, const void* images, const int32_t* labels, float* master,
             float* velocity, float* grads, void* model, float lr, const TrainCtl* ctl, int update, float* loss_out,
             float* logits_out, void* workspace, size_t workspace_bytes, void* stream) {
  RN50_REQUIRE(plan && images && labels && grads && model && loss_out && workspace, RN50_ERR_INVALID,
               "resnet_step: null pointer");
  RN50_REQUIRE(!update || (master && velocity), RN50_ERR_INVALID, "resnet_step: update needs master and velocity");
  RN50_REQUIRE(aligned16(images) && aligned16(master) && aligned16(velocity) && aligned16(grads) &&
                   aligned16(model) && aligned16(workspace) && aligned16(logits_out),
               RN50_ERR_ALIGN, "resnet_step: pointer not 16-byte aligned");
  RN50_REQUIRE(workspace_bytes >= plan->ws_bytes, RN50_ERR_WORKSPACE, "resnet_step: workspace %zu < %zu bytes",
               workspace_bytes, plan->ws_bytes);
  const rn50_step_config& cfg = plan->cfg;
  RN50_REQUIRE(cfg.dtype == RN50_BF16 || model == static_cast<void*>(master) || !update, RN50_ERR_INVALID,
               "resnet_step: in F32 mode the model arena must be the master arena");
  hipStream_t s = static_cast<hipStream_t>(stream);
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  const size_t es = plan->es;
  const int dt = cfg.dtype;
  auto W = [&](int ti) -> const void* { return static_cast<const unsigned char*>(model) + plan->tensors[ti].offset * es; };
  auto MP = [&](int ti) -> const float* {  // per-channel vectors are read in float from the master arena
    return (master ? master : static_cast<const float*>(model)) + plan->tensors[ti].offset;
  };
  auto G = [&](int ti) -> float* { return grads + plan->tensors[ti].offset; };
  auto F = [&](size_t off) -> float* { return reinterpret_cast<float*>(ws + off); };
  void* bn_ws = ws + plan->bn_scratch;
  const size_t bn_ws_bytes = plan->bn_scratch_bytes;
  RN50_REQUIRE(cfg.dtype == RN50_F32 || master, RN50_ERR_INVALID,
               "resnet_step: BF16 mode reads BN gamma/beta and the FC bias from the float master arena");

  // The side stream starts after whatever the caller's stream holds so far (the previous step's update
  // of the model weights, for one) and transposes the weights for the data gradients while the forward
  // pass runs: [Cout][R][S][Cin] -> [Cin][R][S][Cout], every convolution in one launch.
  STEP_TRY(ensure_side_stream(plan));
#ifdef RN50_TUNING  // what-if measurement: the whole step on the caller's stream (no concurrency between its parts)
  static const bool one_stream = getenv("RN50_ONE_STREAM") != nullptr;
#else
  constexpr bool one_stream = false;
#endif
  hipStream_t side = one_stream ? s : plan->side;
  (void)hipEventRecord(plan->ev_fork, s);
  (void)hipStreamWaitEvent(side, plan->ev_fork, 0);
  // the learning rate of this step (read by the update at the end, which waits for the side stream)
  if (ctl) hipLaunchKernelGGL(lr_tick_kernel, dim3(1), dim3(64), 0, side, ctl->sched, ctl->t, ctl->lr);
  transpose_batch_run(plan->transposes, dt, model, ws + plan->wT, side);
  (void)hipEventRecord(plan->ev_wt, side);
  float* const run_mean = ctl ? ctl->run_mean : nullptr;
  float* const run_var = ctl ? ctl->run_var : nullptr;
  const float bn_momentum = ctl ? ctl->bn_momentum : 0.f;
  const float* const lr_dev = ctl ? ctl->lr : nullptr;

  // --------------------------------------------------------------- forward
  Unit& u0 = plan->units[0];
  stem_pad_input(&u0.conv, images, ws + plan->xp, s);
  // Every convolution leaves the sums its batch norm needs, one row per output tile, in bn_ws.
  float* sums = static_cast<float*>(bn_ws);
  hipStream_t branch = one_stream ? s : plan->branch;
  void* bn_ws2 = ws + plan->bn_scratch2;  // the projection branch's own BN scratch
  float* sums2 = static_cast<float*>(bn_ws2);
  // stats_only: the layer's output is not stored (its consumer applies it on the fly).
  auto bn_after_conv = [&](Unit& u, const void* residual, float* sm, hipStream_t st, bool stats_only = false) {
    const PartialRows pr = fwd_partial_rows(&u.conv);
    // the residual-add layers record their ReLU decisions: their backward pass then reads one byte per
    // vector instead of z
    bn_fwd_from_partials(&u.bn, ws + u.y, sm, pr.num, pr.rows, MP(u.ig), MP(u.ib), residual,
                         stats_only ? nullptr : ws + u.z, u.bn.mode == 2 ? ws + u.relu_mask : nullptr, F(u.mean), F(u.rstd),
                         run_mean ? run_mean + u.bn_off : nullptr, run_var ? run_var + u.bn_off : nullptr, bn_momentum, st);
  };
  stem_fwd_padded(&u0.conv, ws + plan->xp, W(u0.iw), ws + plan->wp, ws + u0.y, sums, s);
  bn_after_conv(u0, nullptr, sums, s);
  STEP_TRY(maxpool_fwd(cfg.N, u0.P, u0.Q, cfg.stem, dt, ws + u0.z, ws + plan->pool, ws + plan->pool_argmax, s));
  const unsigned char* cur = ws + plan->pool;
  auto conv_bn = [&](Unit& u, const void* in, const void* residual, float* sm, hipStream_t st) {
    fwd_run(&u.conv, in, W(u.iw), ws + u.y, sm, st);
    bn_after_conv(u, residual, sm, st);
  };
  for (const Block& b : plan->blocks) {
    Unit &u1 = plan->units[b.u1], &u2 = plan->units[b.u2], &u3 = plan->units[b.u3];
    const void* shortcut = cur;
    if (b.up >= 0) {  // the projection shortcut runs beside conv1 and conv2
      Unit& up = plan->units[b.up];
      (void)hipEventRecord(plan->ev_bfork, s);
      (void)hipStreamWaitEvent(branch, plan->ev_bfork, 0);
      conv_bn(up, cur, nullptr, sums2, branch);
      (void)hipEventRecord(plan->ev_bjoin, branch);
      shortcut = ws + up.z;
    }
    conv_bn(u1, cur, nullptr, sums, s);
    if (plan->fuse_conv3_input) {  // conv3 reads conv2's raw output and applies BN+ReLU in its operand load
      fwd_run(&u2.conv, ws + u1.z, W(u2.iw), ws + u2.y, sums, s);
      bn_after_conv(u2, nullptr, sums, s, true);
      if (b.up >= 0) (void)hipStreamWaitEvent(s, plan->ev_bjoin, 0);
      const BnIn in{MP(u2.ig), MP(u2.ib), F(u2.mean), F(u2.rstd)};
      fwd_run(&u3.conv, ws + u2.y, W(u3.iw), ws + u3.y, sums, s, "conv_fwd", &in);
      bn_after_conv(u3, shortcut, sums, s);
    } else {
      conv_bn(u2, ws + u1.z, nullptr, sums, s);
      if (b.up >= 0) (void)hipStreamWaitEvent(s, plan->ev_bjoin, 0);
      conv_bn(u3, ws + u2.z, shortcut, sums, s);
    }
    cur = ws + u3.z;
  }
  const int HW = plan->final_hw * plan->final_hw;
  const int fcw = static_cast<int>(plan->tensors.size()) - 2, fcb = fcw + 1;
  float* logits = logits_out ? logits_out : F(plan->logits);
  STEP_TRY(avgpool_fwd(cfg.N, HW, plan->fc_in, dt, cur, ws + plan->avg, s));
  STEP_TRY(fc_fwd(cfg.N, plan->fc_in, cfg.classes, dt, ws + plan->avg, W(fcw), MP(fcb), logits, s));
  STEP_TRY(xent_fwd_bwd(cfg.N, cfg.classes, logits, labels, cfg.label_smoothing, cfg.grad_scale, loss_out,
                        F(plan->row_loss), F(plan->dlogits), s));

  // -------------------------------------------------------------- backward
  // the classifier's parameter gradients, which only the update reads, run on the side stream
  (void)hipEventRecord(plan->ev_fork, s);
  (void)hipStreamWaitEvent(side, plan->ev_fork, 0);
  fc_bwd_params(cfg.N, plan->fc_in, cfg.classes, dt, ws + plan->avg, F(plan->dlogits), G(fcw), G(fcb), side);
  STEP_TRY(fc_bwd(cfg.N, plan->fc_in, cfg.classes, dt, ws + plan->avg, W(fcw), F(plan->dlogits), ws + plan->davg,
                  nullptr, nullptr, ws + plan->fc_scratch, plan->fc_scratch_bytes, s));
  (void)hipStreamWaitEvent(s, plan->ev_wt, 0);  // the transposed weights
  unsigned char* g[5];
  for (int i = 0; i < 5; ++i) g[i] = ws + plan->g[i];
  // g[0], g[1]: the two summands of the gradient w.r.t. the current block output (g[1] may be unused)
  STEP_TRY(avgpool_bwd(cfg.N, HW, plan->fc_in, dt, ws + plan->davg, g[0], s));
  int dgrad_sums_rows = 0;
  // BN backward + wgrad + dgrad of one unit.  dz (+dz2) -> dy; dgrad into `dx` (skipped if null).
  // `sums_ready`: the data gradient that produced dz already left this BN layer's sums in bn_ws.
  // `below`: the unit whose BN output is this unit's input, when dx (+ addend, the gradient of that
  // output's other consumer) is its complete dz: the data gradient then stores the sum and leaves that
  // layer's sums in bn_ws.
  // The weight gradients are off the critical path (nothing in the backward pass reads them): they run
  // on the side stream, a block's worth at a time (one event each way per block: an event is a packet
  // the stream has to drain for).  Every unit has a dy buffer of its own, so the backward pass never waits
  // for the weight gradients.
  struct PendingWgrad {
    Unit* u;
    const void* in;
    void* dy;
    bool bn_in;  // `in` is the input of the BN+ReLU layer in front of the convolution, applied on the fly
    BnIn bn;
  };
  PendingWgrad pending[4];
  int npending = 0, blk = 0;  // blocks processed so far in this backward pass
  auto block_end = [&]() {
    (void)hipEventRecord(plan->ev_dy[blk], s);
    (void)hipStreamWaitEvent(side, plan->ev_dy[blk], 0);
#ifdef RN50_TUNING  // what-if measurement: the step without its weight gradients
    static const bool skip_wgrad = getenv("RN50_SKIP_WGRAD") != nullptr;
    if (skip_wgrad) npending = 0;
#endif
    for (int i = 0; i < npending; ++i)
      wgrad_run(&pending[i].u->conv, pending[i].in, pending[i].dy, G(pending[i].u->iw), ws + plan->wgrad_scratch, side,
                pending[i].bn_in ? &pending[i].bn : nullptr);
    (void)hipEventRecord(plan->ev_wg[blk], side);
    npending = 0;
    ++blk;
  };
  // Phase 1 of a unit: BN backward, dz (+dz2) -> dy (the unit's buffer; returned), on stream st with BN scratch wsx.
  // outer_bits: dz is still to be masked by the ReLU bits another layer recorded (the projection shortcut's
  // BN, whose output gradient is the block output's gradient under the block's ReLU): for the backward
  // arithmetic that is a BN+ReLU layer with recorded bits.
  auto unit_bn_bwd = [&](Unit& u, const void* in, const void* dz, const void* dz2, void* dres, bool sums_ready,
                         hipStream_t st, void* wsx, void** dy_out, const uint8_t* outer_bits = nullptr,
                         const BnIn* bn_in = nullptr) -> int {
    void* dy = ws + u.dy;
    // the ReLU mask: recorded bits (residual-add layers) or recomputed from x (BN+ReLU layers)
    const uint8_t* bits = u.bn.mode == 2 ? ws + u.relu_mask : nullptr;
    if (outer_bits) {
      rn50_bn_desc masked = u.bn;
      masked.mode = 1;
      STEP_TRY(bn_relu_bwd(&masked, dz, dz2, ws + u.y, nullptr, outer_bits, MP(u.ig), MP(u.ib), F(u.mean), F(u.rstd), dy,
                           nullptr, G(u.ig), G(u.ib), wsx, bn_ws_bytes, st));
    } else if (sums_ready) {
      bn_bwd_from_partials(&u.bn, dz, ws + u.y, bits, MP(u.ig), MP(u.ib), F(u.mean), F(u.rstd),
                           static_cast<const float*>(wsx), dgrad_sums_rows, dy, u.bn.mode == 2 ? dres : nullptr,
                           G(u.ig), G(u.ib), st);
    } else {
      STEP_TRY(bn_relu_bwd(&u.bn, dz, dz2, ws + u.y, nullptr, bits, MP(u.ig), MP(u.ib), F(u.mean), F(u.rstd), dy, dres,
                           G(u.ig), G(u.ib), wsx, bn_ws_bytes, st));
    }
    pending[npending++] = PendingWgrad{&u, in, dy, bn_in != nullptr, bn_in ? *bn_in : BnIn{}};
    *dy_out = dy;
    return RN50_OK;
  };
  // Phase 2: the data gradient of dy into dx.  `below`: the unit whose BN output is this unit's input,
  // when dx (+ addend, the gradient of that output's other consumer) is its complete dz: the data gradient
  // then stores the sum and leaves that layer's sums in bn_ws.
  auto unit_dgrad = [&](Unit& u, const void* dy, void* dx, Unit* below, const void* addend, hipStream_t st,
                        const uint8_t* addend_mask = nullptr) {
    BnBwdSums fuse{};
    if (below) {
      fuse = BnBwdSums{ws + below->y, MP(below->ig), MP(below->ib), F(below->mean), F(below->rstd), sums, addend,
                       below->bn.mode == 2 ? ws + below->relu_mask : nullptr, addend_mask};
      dgrad_sums_rows = dgrad_partial_rows(&u.conv).num;
    }
    dgrad_run(&u.conv, dy, ws + plan->wT + plan->tensors[u.iw].offset * es, dx, below ? &fuse : nullptr, st);
  };
  auto unit_bwd = [&](Unit& u, const void* in, const void* dz, const void* dz2, void* dres, void* dx,
                      bool sums_ready, Unit* below, const void* addend) -> int {
    void* dy = nullptr;
    STEP_TRY(unit_bn_bwd(u, in, dz, dz2, dres, sums_ready, s, bn_ws, &dy));
    if (dx) unit_dgrad(u, dy, dx, below, addend, s);
    return RN50_OK;
  };
  // dzo (+ dzo2): the gradient w.r.t. the current block's output; top_sums: its BN sums are in bn_ws.
  // It alternates between two buffers: a block's conv1 data gradient reads the old one (as the shortcut's
  // gradient) while it writes the new one.
  const void *dzo = g[0], *dzo2 = nullptr;
  unsigned char* dz_next = g[2];
  bool top_sums = false;
  for (int bi = static_cast<int>(plan->blocks.size()) - 1; bi >= 0; --bi) {
    const Block& b = plan->blocks[bi];
    Unit &u1 = plan->units[b.u1], &u2 = plan->units[b.u2], &u3 = plan->units[b.u3];
    Unit* prev = bi > 0 ? &plan->units[plan->blocks[bi - 1].u3] : nullptr;  // its BN output is this block's input
    const void* block_in = prev ? static_cast<const void*>(ws + prev->z) : static_cast<const void*>(ws + plan->pool);
    // The block input has two consumers (conv1 and the shortcut).  conv1's data gradient comes last: it
    // adds the shortcut's gradient and takes the sums of the previous block's last BN layer.
    // The shortcut's gradient is dzo under the block output's ReLU mask.  No copy of it is made: an identity
    // shortcut's share is added by conv1's data gradient below, which reads dzo with the recorded bits, and
    // a projection shortcut's BN backward reads dzo with the same bits.
    void* dy3 = nullptr;
    if (plan->fuse_conv3_input) {
      const BnIn in{MP(u2.ig), MP(u2.ib), F(u2.mean), F(u2.rstd)};
      STEP_TRY(unit_bn_bwd(u3, ws + u2.y, dzo, dzo2, nullptr, top_sums, s, bn_ws, &dy3, nullptr, &in));
    } else {
      STEP_TRY(unit_bn_bwd(u3, ws + u2.z, dzo, dzo2, nullptr, top_sums, s, bn_ws, &dy3));
    }
    const void* shortcut_grad = dzo;
    const uint8_t* shortcut_mask = ws + u3.relu_mask;
    if (b.up >= 0) {  // the projection's backward pass runs beside the main branch, on its own stream
      Unit& up = plan->units[b.up];
      (void)hipEventRecord(plan->ev_bfork, s);
      (void)hipStreamWaitEvent(branch, plan->ev_bfork, 0);
      void* dyp = nullptr;
      STEP_TRY(unit_bn_bwd(up, block_in, dzo, dzo2, nullptr, false, branch, bn_ws2, &dyp, ws + u3.relu_mask));
      unit_dgrad(up, dyp, g[1], nullptr, nullptr, branch);
      (void)hipEventRecord(plan->ev_bjoin, branch);
      shortcut_grad = g[1];
      shortcut_mask = nullptr;
    }
    unit_dgrad(u3, dy3, g[4], &u2, nullptr, s);
    STEP_TRY(unit_bwd(u2, ws + u1.z, g[4], nullptr, nullptr, g[4], true, &u1, nullptr));
    void* dy1 = nullptr;
    STEP_TRY(unit_bn_bwd(u1, block_in, g[4], nullptr, nullptr, true, s, bn_ws, &dy1));
    if (b.up >= 0) (void)hipStreamWaitEvent(s, plan->ev_bjoin, 0);
    unsigned char* const dz_new = dz_next;
    dz_next = const_cast<unsigned char*>(static_cast<const unsigned char*>(dzo));
    if (prev) {
      unit_dgrad(u1, dy1, dz_new, prev, shortcut_grad, s, shortcut_mask);
      dzo = dz_new; dzo2 = nullptr; top_sums = true;
    } else {  // the first block (it has a projection): the max-pool's backward pass adds the two branches
      unit_dgrad(u1, dy1, dz_new, nullptr, nullptr, s);
      dzo = dz_new; dzo2 = shortcut_grad; top_sums = false;
    }
    block_end();
  }
  STEP_TRY(maxpool_bwd(cfg.N, u0.P, u0.Q, cfg.stem, dt, ws + u0.z, ws + plan->pool_argmax, dzo, dzo2, dz_next, s));
  STEP_TRY(unit_bwd(u0, ws + plan->xp, dz_next, nullptr, nullptr, nullptr, false, nullptr, nullptr));
  block_end();
  // ------------------------------------------------------------------ LARS
  // The side stream runs in order: the event of the last block but one covers every weight gradient
  // except the stem's, which is still running while the other tensors are updated.
  void* lowp = cfg.dtype == RN50_BF16 ? model : nullptr;
  if (update) {
    if (blk >= 2) (void)hipStreamWaitEvent(s, plan->ev_wg[blk - 2], 0);
    lars_arena_run(plan->lars_rest, master, grads, velocity, lowp, cfg.eta, cfg.momentum, lr, lr_dev, cfg.lars_eps,
                   cfg.weight_decay, F(plan->lars_scratch), s);
  }
  (void)hipStreamWaitEvent(s, plan->ev_wg[blk - 1], 0);  // join
  if (update)
    lars_arena_run(plan->lars_stem, master, grads, velocity, lowp, cfg.eta, cfg.momentum, lr, lr_dev, cfg.lars_eps,
                   cfg.weight_decay, F(plan->lars_stem_scratch), s);
  return launch_status(who);
}

}  // namespace

extern "C" int resnet_step(rn50_plan* plan, const void* images, const int32_t* labels, float* master,
                           float* velocity, float* grads, void* model, float lr, int update, float* loss_out,
                           float* logits_out, void* workspace, size_t workspace_bytes, void* stream) {
  clear_error();
  return run_step("resnet_step", plan, images, labels, master, velocity, grads, model, lr, nullptr, update, loss_out,
                  logits_out, workspace, workspace_bytes, stream);
}

// ------------------------------------------------------------------ seeded parallel initialization
namespace {
constexpr int kInitMaxTensors = 192;
struct InitArgs {
  float* master;
  float* velocity;  // or null
  uint16_t* lowp;   // or null
  int num;
  uint32_t seed_lo, seed_hi;
  double cdf_lo, cdf_span;  // Phi(-2), Phi(2) - Phi(-2)
  int64_t total;            // arena elements
  uint32_t offset[kInitMaxTensors];
  uint32_t count[kInitMaxTensors];
  int fan_in[kInitMaxTensors];
  int tensor0;              // index of the first tensor of this launch
};

// Philox4x32-10 (Salmon et al., SC'11): first output word for counter (c0, c1, c2, 0) and key (k0, k1).
__device__ __forceinline__ uint32_t philox4x32_10_x0(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t k0, uint32_t k1) {
  uint32_t c3 = 0;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    c0 = hi1 ^ c1 ^ k0;
    c1 = lo1;
    c2 = hi0 ^ c3 ^ k1;
    c3 = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return c0;
}

// One thread per arena element: every value is a function of (seed, tensor, element) alone, so any
// worker produces the same arena with no exchange.
__global__ __launch_bounds__(256) void init_params_kernel(const InitArgs a) {
  const int64_t e = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (e >= a.total) return;
  int lo = 0, hi = a.num;  // last tensor whose offset <= e
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (a.offset[mid] <= e) lo = mid; else hi = mid;
  }
  const int64_t i = e - a.offset[lo];
  float w = 0.f;
  if (i < a.count[lo]) {
    const int fan = a.fan_in[lo];
    if (fan == 0) {
      w = 1.f;
    } else if (fan > 0) {
      const uint32_t x0 = philox4x32_10_x0(static_cast<uint32_t>(i), static_cast<uint32_t>(i >> 32),
                                           static_cast<uint32_t>(a.tensor0 + lo), a.seed_lo, a.seed_hi);
      const double u = (static_cast<double>(x0) + 0.5) * (1.0 / 4294967296.0);
      const double z = normcdfinv(a.cdf_lo + u * a.cdf_span);
      w = static_cast<float>(sqrt(2.0 / static_cast<double>(fan)) * z);
    }
  }
  a.master[e] = w;
  if (a.velocity) a.velocity[e] = 0.f;
  if (a.lowp) a.lowp[e] = float_to_bf16_bits(w);
}
}  // namespace

extern "C" int resnet_init_params(const rn50_plan* plan, uint64_t seed, float* master, float* velocity, void* model,
                                  void* stream) {
  clear_error();
  RN50_REQUIRE(plan && master, RN50_ERR_INVALID, "resnet_init_params: null pointer");
  RN50_REQUIRE(aligned16(master) && aligned16(velocity) && aligned16(model), RN50_ERR_ALIGN,
               "resnet_init_params: pointer not 16-byte aligned");
  RN50_REQUIRE(plan->tensors.size() <= kInitMaxTensors, RN50_ERR_UNSUPPORTED, "resnet_init_params: %zu tensors",
               plan->tensors.size());
  InitArgs a{};
  a.master = master;
  a.velocity = velocity;
  a.lowp = (plan->cfg.dtype == RN50_BF16 && model && model != static_cast<void*>(master)) ? static_cast<uint16_t*>(model)
                                                                                          : nullptr;
  a.num = static_cast<int>(plan->tensors.size());
  a.seed_lo = static_cast<uint32_t>(seed);
  a.seed_hi = static_cast<uint32_t>(seed >> 32);
  a.cdf_lo = 0.5 * erfc(2.0 / sqrt(2.0));
  a.cdf_span = (1.0 - a.cdf_lo) - a.cdf_lo;
  a.total = plan->arena_elems;
  a.tensor0 = 0;
  for (int t = 0; t < a.num; ++t) {
    a.offset[t] = static_cast<uint32_t>(plan->tensors[t].offset);
    a.count[t] = static_cast<uint32_t>(plan->tensors[t].count);
    a.fan_in[t] = plan->tensors[t].fan_in;
  }
  hipLaunchKernelGGL(init_params_kernel, dim3(static_cast<unsigned>(ceil_div(a.total, 256))), dim3(256), 0,
                     static_cast<hipStream_t>(stream), a);
  return launch_status("resnet_init_params");
}

// ------------------------------------------------------------------ evaluation
extern "C" int resnet_eval(rn50_plan* plan, const void* state, const void* images, const int32_t* labels,
                           const float* master, const void* model, float* logits_out, int32_t* pred_out,
                           int32_t* correct_out, void* workspace, size_t workspace_bytes, void* stream) {
  clear_error();
  RN50_REQUIRE(plan && state && images && labels && master && model && pred_out && correct_out && workspace,
               RN50_ERR_INVALID, "resnet_eval: null pointer");
  RN50_REQUIRE(aligned16(state) && aligned16(images) && aligned16(master) && aligned16(model) && aligned16(workspace) &&
                   aligned16(logits_out),
               RN50_ERR_ALIGN, "resnet_eval: pointer not 16-byte aligned");
  RN50_REQUIRE(workspace_bytes >= plan->ws_bytes, RN50_ERR_WORKSPACE, "resnet_eval: workspace %zu < %zu bytes",
               workspace_bytes, plan->ws_bytes);
  const rn50_step_config& cfg = plan->cfg;
  hipStream_t s = static_cast<hipStream_t>(stream);
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  const size_t es = plan->es;
  const int dt = cfg.dtype;
  const float* run_mean = reinterpret_cast<const float*>(static_cast<const unsigned char*>(state) + kStateHeader);
  const float* run_var = run_mean + plan->bn_channels;
  auto W = [&](int ti) -> const void* { return static_cast<const unsigned char*>(model) + plan->tensors[ti].offset * es; };
  auto MP = [&](int ti) -> const float* { return master + plan->tensors[ti].offset; };
  auto F = [&](size_t off) -> float* { return reinterpret_cast<float*>(ws + off); };
  auto bn = [&](Unit& u, const void* residual) {
    bn_infer_run(&u.bn, ws + u.y, MP(u.ig), MP(u.ib), run_mean + u.bn_off, run_var + u.bn_off, residual, ws + u.z,
                 F(u.rstd), s);
  };
  Unit& u0 = plan->units[0];
  stem_pad_input(&u0.conv, images, ws + plan->xp, s);
  stem_fwd_padded(&u0.conv, ws + plan->xp, W(u0.iw), ws + plan->wp, ws + u0.y, nullptr, s);
  bn(u0, nullptr);
  STEP_TRY(maxpool_fwd(cfg.N, u0.P, u0.Q, cfg.stem, dt, ws + u0.z, ws + plan->pool, ws + plan->pool_argmax, s));
  const unsigned char* cur = ws + plan->pool;
  for (const Block& b : plan->blocks) {
    Unit &u1 = plan->units[b.u1], &u2 = plan->units[b.u2], &u3 = plan->units[b.u3];
    const void* shortcut = cur;
    if (b.up >= 0) {
      Unit& up = plan->units[b.up];
      fwd_run(&up.conv, cur, W(up.iw), ws + up.y, nullptr, s);
      bn(up, nullptr);
      shortcut = ws + up.z;
    }
    fwd_run(&u1.conv, cur, W(u1.iw), ws + u1.y, nullptr, s);
    bn(u1, nullptr);
    fwd_run(&u2.conv, ws + u1.z, W(u2.iw), ws + u2.y, nullptr, s);
    bn(u2, nullptr);
    fwd_run(&u3.conv, ws + u2.z, W(u3.iw), ws + u3.y, nullptr, s);
    bn(u3, shortcut);
    cur = ws + u3.z;
  }
  const int HW = plan->final_hw * plan->final_hw;
  const int fcw = static_cast<int>(plan->tensors.size()) - 2, fcb = fcw + 1;
  float* logits = logits_out ? logits_out : F(plan->logits);
  STEP_TRY(avgpool_fwd(cfg.N, HW, plan->fc_in, dt, cur, ws + plan->avg, s));
  STEP_TRY(fc_fwd(cfg.N, plan->fc_in, cfg.classes, dt, ws + plan->avg, W(fcw), MP(fcb), logits, s));
  STEP_TRY(top1_accuracy(cfg.N, cfg.classes, logits, labels, pred_out, correct_out, s));
  return launch_status("resnet_eval");
}

extern "C" int resnet_plan_num_bn(const rn50_plan* plan) { return plan ? static_cast<int>(plan->units.size()) : 0; }
extern "C" int64_t resnet_plan_bn_channels(const rn50_plan* plan) { return plan ? plan->bn_channels : 0; }
extern "C" int64_t resnet_plan_bn_offset(const rn50_plan* plan, int i, int* channels_out) {
  if (!plan || i < 0 || i >= static_cast<int>(plan->units.size())) return -1;
  if (channels_out) *channels_out = plan->units[i].conv.Cout;
  return plan->units[i].bn_off;
}
extern "C" size_t resnet_train_state_bytes(const rn50_plan* plan) {
  return plan ? kStateHeader + 2 * static_cast<size_t>(plan->bn_channels) * sizeof(float) : 0;
}

extern "C" int resnet_train_state_init(const rn50_plan* plan, void* state, size_t state_bytes, int64_t first_step,
                                       void* stream) {
  clear_error();
  RN50_REQUIRE(plan && state, RN50_ERR_INVALID, "resnet_train_state_init: null pointer");
  RN50_REQUIRE(aligned16(state), RN50_ERR_ALIGN, "resnet_train_state_init: state not 16-byte aligned");
  RN50_REQUIRE(state_bytes >= resnet_train_state_bytes(plan), RN50_ERR_WORKSPACE,
               "resnet_train_state_init: state %zu < %zu bytes", state_bytes, resnet_train_state_bytes(plan));
  RN50_REQUIRE(first_step >= 0, RN50_ERR_INVALID, "resnet_train_state_init: first_step < 0");
  unsigned char* st = static_cast<unsigned char*>(state);
  float* rm = reinterpret_cast<float*>(st + kStateHeader);
  const int64_t n = plan->bn_channels;
  hipLaunchKernelGGL(train_state_init_kernel, dim3(static_cast<unsigned>(ceil_div(n, 256))), dim3(256), 0,
                     static_cast<hipStream_t>(stream), reinterpret_cast<int64_t*>(st), reinterpret_cast<float*>(st + 8),
                     rm, rm + n, n, first_step);
  return launch_status("resnet_train_state_init");
}

extern "C" int resnet_train_step(rn50_plan* plan, const rn50_lr_schedule* sc, void* state, float bn_momentum,
                                 const void* images, const int32_t* labels, float* master, float* velocity,
                                 float* grads, void* model, float* loss_out, float* logits_out, void* workspace,
                                 size_t workspace_bytes, void* stream) {
  clear_error();
  RN50_REQUIRE(plan && sc && state && master && velocity, RN50_ERR_INVALID, "resnet_train_step: null pointer");
  RN50_REQUIRE(aligned16(state), RN50_ERR_ALIGN, "resnet_train_step: state not 16-byte aligned");
  RN50_REQUIRE(sc->decay >= RN50_DECAY_NONE && sc->decay <= RN50_DECAY_TABLE, RN50_ERR_INVALID,
               "resnet_train_step: decay = %d", sc->decay);
  if (sc->decay == RN50_DECAY_TABLE) {
    RN50_REQUIRE(sc->table && sc->table_len > 0, RN50_ERR_INVALID, "resnet_train_step: empty learning-rate table");
  } else {
    RN50_REQUIRE(sc->warmup_steps >= 0, RN50_ERR_INVALID, "resnet_train_step: warmup_steps = %d", sc->warmup_steps);
    RN50_REQUIRE(sc->decay != RN50_DECAY_STEP || sc->step_every > 0, RN50_ERR_INVALID,
                 "resnet_train_step: step_every = %d", sc->step_every);
    RN50_REQUIRE((sc->decay != RN50_DECAY_POLY && sc->decay != RN50_DECAY_LINEAR) || sc->total_steps > sc->warmup_steps,
                 RN50_ERR_INVALID, "resnet_train_step: total_steps %d <= warmup_steps %d", sc->total_steps,
                 sc->warmup_steps);
  }
  RN50_REQUIRE(bn_momentum >= 0.f && bn_momentum <= 1.f, RN50_ERR_INVALID, "resnet_train_step: bn_momentum = %g",
               bn_momentum);
  unsigned char* st = static_cast<unsigned char*>(state);
  TrainCtl ctl;
  ctl.sched = *sc;
  ctl.t = reinterpret_cast<int64_t*>(st);
  ctl.lr = reinterpret_cast<float*>(st + 8);
  ctl.run_mean = reinterpret_cast<float*>(st + kStateHeader);
  ctl.run_var = ctl.run_mean + plan->bn_channels;
  ctl.bn_momentum = bn_momentum;
  return run_step("resnet_train_step", plan, images, labels, master, velocity, grads, model, 0.f, &ctl, 1, loss_out,
                  logits_out, workspace, workspace_bytes, stream);
}
