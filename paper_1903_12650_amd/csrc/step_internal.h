// Entry points of the kernel files that the whole-step driver calls directly
// (below the argument checking of the C ABI), so that padded / transposed
// operands and scratch buffers are shared across the passes of one step.
#pragma once
#include <hip/hip_runtime.h>

#include <vector>

#include "../../include/rn50_hip.h"

namespace rn50 {

// The descriptor checks of the C ABI's own entry points (0, or the error code with the text set).
int conv_desc_check(const rn50_conv_desc* d, const char* who);
int bn_desc_check(const rn50_bn_desc* d, const char* who);

// conv.hip
size_t stem_padded_input_bytes(const rn50_conv_desc* d);
size_t stem_padded_weight_bytes(const rn50_conv_desc* d);
void stem_pad_input(const rn50_conv_desc* d, const void* x, void* xp, hipStream_t s);
// Batch-norm sums fused into a convolution's output stage come as one row of partial sums per output
// tile: `num` rows over `rows` consecutive output pixels each (the last row may cover fewer).
struct PartialRows {
  int rows, num;
};
PartialRows fwd_partial_rows(const rn50_conv_desc* d);    // tiles of the forward convolution's output
PartialRows dgrad_partial_rows(const rn50_conv_desc* d);  // tiles of the data gradient
int64_t dgrad_partial_rows_bound(const rn50_conv_desc* d);  // most rows any tile choice gives (tiles of >= 64 pixels)
// bn_partial (null: none): float[3][Cout][num] = shift, sum(y - shift), sum((y - shift)^2) per tile.
void stem_fwd_padded(const rn50_conv_desc* d, const void* xp, const void* w, void* wp, void* y, float* bn_partial,
                     hipStream_t s);
// A BN+ReLU layer applied to a convolution's input on the fly (1x1, stride 1 convolutions only): its parameters
// and saved statistics, float[Cin] each.
// The BN sums that a convolution's output stage leaves (one row per row tile) are stored ROW-major when there are
// few tile rows: the BN apply pass (forward or backward) then adds them up itself, in every workgroup, for the
// channels it applies, and the finalize launch in front of it -- about 4 us on the step's dependency chain whatever
// it computes -- is gone.  Forward: per tile row and channel the doubles (sum y, sum y^2), moved from the tile's
// shift to shift 0 by the writer so that the readers only add; backward: float planes [plane][tile row][C].
// Otherwise channel-major float planes, partial[plane][C][tile row], for the finalize kernels.  The writer and the
// reader both decide by this function.  Threshold from whole-step measurements at batch 40 (40 / 128 / 256 rows
// against none: 4.613 / 4.577 / 4.666 against 4.649 ms): up to 123 tile rows (the 14x14 and 7x7 layers) the
// redundant sums cost less than the launch; at 245 (28x28) every workgroup would read more sums than data (raising
// the backward threshold alone to 256 / 512 rows: 4.78 -> 4.83 / 4.84 ms).
constexpr int kBnSelfFinalizeRows = 128, kBnSelfFinalizeRowsBwd = 128;
inline bool bn_partials_row_major(int nrows, bool backward) {
  return nrows <= (backward ? kBnSelfFinalizeRowsBwd : kBnSelfFinalizeRows);
}

struct BnIn {
  const float *gamma, *beta, *mean, *rstd;
};
void fwd_run(const rn50_conv_desc* d, const void* x, const void* w, void* y, float* bn_partial, hipStream_t s,
             const char* tag = "conv_fwd", const BnIn* in = nullptr);
// The BN layer (with ReLU) whose output gradient a data gradient produces: x is that
// layer's input [N*H*W][Cin]; partial receives float[2][Cin][num] = sum(g), sum(g * xhat) per tile.
// addend (or null): a second branch of the gradient, [N*H*W][Cin], added to the data gradient before it
// is stored; relu_mask (or null): the BN layer's recorded ReLU decisions (else recomputed from x);
// addend_mask (or null): ReLU bits under which the addend counts (the addend is then the still unmasked
// output gradient of the residual-add layer that recorded them).
struct BnBwdSums {
  const void* x;
  const float *gamma, *beta, *mean, *rstd;
  float* partial;
  const void* addend = nullptr;
  const uint8_t* relu_mask = nullptr;
  const uint8_t* addend_mask = nullptr;
};
size_t dgrad_wt_bytes(const rn50_conv_desc* d);
void dgrad_transpose_weights(const rn50_conv_desc* d, const void* w, void* wT, hipStream_t s);
void dgrad_run(const rn50_conv_desc* d, const void* dy, const void* wT, void* dx, const BnBwdSums* bn, hipStream_t s);
struct TransposeEntry {
  int64_t offset;  // element offset of the tensor in both arenas
  int K, taps, C;
};
void transpose_batch_run(const std::vector<TransposeEntry>& list, int dtype, const void* src_arena, void* dst_arena,
                         hipStream_t s);
size_t wgrad_partial_bytes(const rn50_conv_desc* d);
void wgrad_run(const rn50_conv_desc* d, const void* x_or_xp, const void* dy, float* dw, void* scratch, hipStream_t s,
               const BnIn* in = nullptr);

// bn.hip: the part of the forward / backward pass that follows the sums
void bn_fwd_from_partials(const rn50_bn_desc* d, const void* x, const float* partial, int nrows, int rpp,
                          const float* gamma, const float* beta, const void* residual, void* y,
                          uint8_t* relu_mask, float* save_mean, float* save_rstd, float* rm, float* rv,
                          float momentum, hipStream_t s);
// relu_mask: recorded ReLU decisions (required in mode 2, where dres receives the masked gradient), or
// null: recomputed from x (mode 1).
void bn_bwd_from_partials(const rn50_bn_desc* d, const void* dz, const void* x, const uint8_t* relu_mask,
                          const float* gamma, const float* beta, const float* mean, const float* rstd,
                          const float* partial, int nrows, void* dx, void* dres, float* dgamma, float* dbeta,
                          hipStream_t s);

// evaluation mode (moving averages instead of batch statistics); rstd_scratch: float[C]
void bn_infer_run(const rn50_bn_desc* d, const void* x, const float* gamma, const float* beta,
                  const float* running_mean, const float* running_var, const void* residual, void* y,
                  float* rstd_scratch, hipStream_t s);

// head.hip: the classifier's parameter gradients alone (fc_bwd with dW = db = null leaves them out)
void fc_bwd_params(int N, int Cin, int K, int dtype, const void* a, const float* dlogits, float* dW, float* db,
                   hipStream_t s);

// lars.hip
struct LarsArenaSpec {
  int num = 0;
  std::vector<int64_t> offset, count;
  std::vector<char> decay;
};
size_t lars_arena_partial_bytes(const LarsArenaSpec& sp);
void lars_arena_run(const LarsArenaSpec& sp, float* master, const float* grads, float* velocity, void* lowp,
                    float eta, float momentum, float lr, const float* lr_dev, float eps, float weight_decay,
                    float* partial, hipStream_t s);

}  // namespace rn50
