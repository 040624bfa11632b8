/*
 * CPU oracle for one worker's share of the large-minibatch ResNet-50 training
 * step (Sec. III of the paper: SGD + LARS, batch normalization, label
 * smoothing, mixed precision with a single-precision weight update; appendix
 * log: stem convolution stride 2 / 64 filters / no bias, BN momentum 0.9 and
 * epsilon 1e-5 with scale and centre, max-pool 112 -> 56, bottleneck blocks).
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is the slow, plain definition of every
 * operation, used only to check the GPU library and to time a CPU baseline.
 * Nothing in the product path may call it, and it shares no code with the GPU
 * kernels.
 *
 * Every operation is the textbook definition evaluated with nested loops.
 * Tensors are stored as REAL (float or double; the file is compiled once for
 * each) and every sum is accumulated in double.  Activations are NHWC,
 * convolution weights are KRSC (output channel, filter row, filter column,
 * input channel).  No blocking, no BLAS.
 *
 * The paper prints no formula for these operations; it names them (Sec. II:
 * batch normalization, LARS; Sec. III-A: label smoothing; Sec. IV: mixed
 * precision).  The definitions used are the standard ones of the works it
 * cites; every reading is listed in the repository's design notes.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef REAL
#define REAL float
#define SUFFIX _f32
#endif

#define ORC_CAT_(a, b) a##b
#define ORC_CAT(a, b) ORC_CAT_(a, b)
#define FN(name) ORC_CAT(name, SUFFIX)

typedef int64_t i64;

static int out_dim(int in, int pad, int k, int stride) { return (in + 2 * pad - k) / stride + 1; }

/* ------------------------------------------------------------------------
 * Convolution forward (cross-correlation, zero padding, no bias; the stem's
 * "use_bias: false" in the appendix log holds for every convolution):
 *   y[n,p,q,k] = sum_{r,s,c} x[n, p*stride-pad+r, q*stride-pad+s, c] * w[k,r,s,c]
 * ---------------------------------------------------------------------- */
void FN(orc_conv_fwd)(const REAL* x, const REAL* w, REAL* y, int N, int H, int W, int C, int K,
                      int R, int S, int stride, int pad) {
  const int P = out_dim(H, pad, R, stride), Q = out_dim(W, pad, S, stride);
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int p = 0; p < P; ++p)
      for (int q = 0; q < Q; ++q)
        for (int k = 0; k < K; ++k) {
          double acc = 0.0;
          for (int r = 0; r < R; ++r) {
            const int ih = p * stride - pad + r;
            if (ih < 0 || ih >= H) continue;
            for (int s = 0; s < S; ++s) {
              const int iw = q * stride - pad + s;
              if (iw < 0 || iw >= W) continue;
              const REAL* xp = x + (((i64)n * H + ih) * W + iw) * C;
              const REAL* wp = w + (((i64)k * R + r) * S + s) * C;
              double a = 0.0;
#pragma omp simd reduction(+ : a)
              for (int c = 0; c < C; ++c) a += (double)xp[c] * (double)wp[c];
              acc += a;
            }
          }
          y[(((i64)n * P + p) * Q + q) * K + k] = (REAL)acc;
        }
}

/* ------------------------------------------------------------------------
 * Convolution data gradient (the adjoint of the forward map in x):
 *   dx[n,h,w,c] = sum over (k,r,s) with h = p*stride-pad+r, w = q*stride-pad+s
 *                 of dy[n,p,q,k] * w[k,r,s,c]
 * One double accumulator per input channel of the pixel.
 * ---------------------------------------------------------------------- */
void FN(orc_conv_dgrad)(const REAL* dy, const REAL* w, REAL* dx, int N, int H, int W, int C, int K,
                        int R, int S, int stride, int pad) {
  const int P = out_dim(H, pad, R, stride), Q = out_dim(W, pad, S, stride);
#pragma omp parallel
  {
    double* acc = (double*)malloc(sizeof(double) * (size_t)C);
#pragma omp for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
      for (int h = 0; h < H; ++h)
        for (int wi = 0; wi < W; ++wi) {
          for (int c = 0; c < C; ++c) acc[c] = 0.0;
          for (int r = 0; r < R; ++r) {
            const int th = h + pad - r;
            if (th < 0 || th % stride != 0) continue;
            const int p = th / stride;
            if (p >= P) continue;
            for (int s = 0; s < S; ++s) {
              const int tw = wi + pad - s;
              if (tw < 0 || tw % stride != 0) continue;
              const int q = tw / stride;
              if (q >= Q) continue;
              const REAL* dyp = dy + (((i64)n * P + p) * Q + q) * K;
              for (int k = 0; k < K; ++k) {
                const double d = (double)dyp[k];
                const REAL* wp = w + (((i64)k * R + r) * S + s) * C;
                for (int c = 0; c < C; ++c) acc[c] += d * (double)wp[c];
              }
            }
          }
          REAL* dxp = dx + (((i64)n * H + h) * W + wi) * C;
          for (int c = 0; c < C; ++c) dxp[c] = (REAL)acc[c];
        }
    free(acc);
  }
}

/* ------------------------------------------------------------------------
 * Convolution weight gradient (the adjoint of the forward map in w):
 *   dw[k,r,s,c] = sum_{n,p,q} dy[n,p,q,k] * x[n, p*stride-pad+r, q*stride-pad+s, c]
 * One double accumulator per (r,s,c) of the output channel.
 * ---------------------------------------------------------------------- */
void FN(orc_conv_wgrad)(const REAL* x, const REAL* dy, REAL* dw, int N, int H, int W, int C, int K,
                        int R, int S, int stride, int pad) {
  const int P = out_dim(H, pad, R, stride), Q = out_dim(W, pad, S, stride);
  const i64 rsc = (i64)R * S * C;
#pragma omp parallel
  {
    double* acc = (double*)malloc(sizeof(double) * (size_t)rsc);
#pragma omp for schedule(dynamic, 1)
    for (int k = 0; k < K; ++k) {
      for (i64 i = 0; i < rsc; ++i) acc[i] = 0.0;
      for (int n = 0; n < N; ++n)
        for (int p = 0; p < P; ++p)
          for (int q = 0; q < Q; ++q) {
            const double d = (double)dy[(((i64)n * P + p) * Q + q) * K + k];
            for (int r = 0; r < R; ++r) {
              const int ih = p * stride - pad + r;
              if (ih < 0 || ih >= H) continue;
              for (int s = 0; s < S; ++s) {
                const int iw = q * stride - pad + s;
                if (iw < 0 || iw >= W) continue;
                const REAL* xp = x + (((i64)n * H + ih) * W + iw) * C;
                double* ap = acc + ((i64)r * S + s) * C;
                for (int c = 0; c < C; ++c) ap[c] += d * (double)xp[c];
              }
            }
          }
      REAL* dwp = dw + (i64)k * rsc;
      for (i64 i = 0; i < rsc; ++i) dwp[i] = (REAL)acc[i];
    }
    free(acc);
  }
}

/* ------------------------------------------------------------------------
 * Batch normalization, training mode (Sec. II, Ioffe & Szegedy; appendix log:
 * epsilon 1e-5, scale and centre on, statistics of the local batch only,
 * Sec. III-A3).  x is [m][C] (m = N*H*W).  Per channel:
 *   mu = mean_m x, var = mean_m (x-mu)^2 (biased), rstd = 1/sqrt(var+eps),
 *   xhat = (x-mu)*rstd, v = gamma*xhat + beta,
 *   mode 0: y = v; mode 1: y = max(v,0); mode 2: y = max(v + residual, 0).
 * mu and rstd are returned for the backward pass.
 * ---------------------------------------------------------------------- */
void FN(orc_bn_fwd)(const REAL* x, const REAL* gamma, const REAL* beta, const REAL* residual,
                    REAL* y, REAL* save_mean, REAL* save_rstd, i64 m, int C, double eps, int mode) {
#pragma omp parallel for schedule(static)
  for (int c = 0; c < C; ++c) {
    double s = 0.0;
    for (i64 i = 0; i < m; ++i) s += (double)x[i * C + c];
    const double mu = s / (double)m;
    double ss = 0.0;
    for (i64 i = 0; i < m; ++i) {
      const double d = (double)x[i * C + c] - mu;
      ss += d * d;
    }
    const double var = ss / (double)m;
    const double rstd = 1.0 / sqrt(var + eps);
    save_mean[c] = (REAL)mu;
    save_rstd[c] = (REAL)rstd;
    const double g = (double)gamma[c], b = (double)beta[c];
    for (i64 i = 0; i < m; ++i) {
      double v = g * (((double)x[i * C + c] - mu) * rstd) + b;
      if (mode == 2) v += (double)residual[i * C + c];
      if (mode >= 1 && !(v > 0.0)) v = 0.0;
      y[i * C + c] = (REAL)v;
    }
  }
}

/* Moving averages of the batch statistics (appendix log: momentum 0.9):
 *   running <- momentum*running + (1-momentum)*batch, with the biased variance. */
void FN(orc_bn_running)(const REAL* x, REAL* running_mean, REAL* running_var, i64 m, int C,
                        double momentum) {
#pragma omp parallel for schedule(static)
  for (int c = 0; c < C; ++c) {
    double s = 0.0;
    for (i64 i = 0; i < m; ++i) s += (double)x[i * C + c];
    const double mu = s / (double)m;
    double ss = 0.0;
    for (i64 i = 0; i < m; ++i) {
      const double d = (double)x[i * C + c] - mu;
      ss += d * d;
    }
    running_mean[c] = (REAL)(momentum * (double)running_mean[c] + (1.0 - momentum) * mu);
    running_var[c] = (REAL)(momentum * (double)running_var[c] + (1.0 - momentum) * (ss / (double)m));
  }
}

/* ------------------------------------------------------------------------
 * Backward of the block above.  z is the forward output (used only for the
 * ReLU mask z > 0; the derivative at 0 is taken as 0).  Per channel:
 *   g = dz * [z > 0]            (modes 1, 2; mode 0: g = dz)
 *   dbeta = sum_m g, dgamma = sum_m g*xhat
 *   dx = gamma*rstd*(g - dbeta/m - xhat*dgamma/m)
 *   mode 2: dresidual = g
 * ---------------------------------------------------------------------- */
void FN(orc_bn_bwd)(const REAL* dz, const REAL* x, const REAL* z, const REAL* gamma,
                    const REAL* save_mean, const REAL* save_rstd, REAL* dx, REAL* dresidual,
                    REAL* dgamma, REAL* dbeta, i64 m, int C, int mode) {
#pragma omp parallel for schedule(static)
  for (int c = 0; c < C; ++c) {
    const double mu = (double)save_mean[c], rstd = (double)save_rstd[c];
    double sg = 0.0, sgx = 0.0;
    for (i64 i = 0; i < m; ++i) {
      double g = (double)dz[i * C + c];
      if (mode >= 1 && !((double)z[i * C + c] > 0.0)) g = 0.0;
      const double xh = ((double)x[i * C + c] - mu) * rstd;
      sg += g;
      sgx += g * xh;
    }
    dbeta[c] = (REAL)sg;
    dgamma[c] = (REAL)sgx;
    const double a = (double)gamma[c] * rstd;
    const double mg = sg / (double)m, mgx = sgx / (double)m;
    for (i64 i = 0; i < m; ++i) {
      double g = (double)dz[i * C + c];
      if (mode >= 1 && !((double)z[i * C + c] > 0.0)) g = 0.0;
      const double xh = ((double)x[i * C + c] - mu) * rstd;
      dx[i * C + c] = (REAL)(a * (g - mg - xh * mgx));
      if (mode == 2) dresidual[i * C + c] = (REAL)g;
    }
  }
}

/* ------------------------------------------------------------------------
 * Max pooling (appendix log: 112 -> 56 after the stem): window ksize, given
 * stride and symmetric padding; padded positions never win.  Among equal
 * maxima the first in row-major window order wins.  idx (optional) receives
 * the winning input offset (h*W + w) per output element.
 * ---------------------------------------------------------------------- */
void FN(orc_maxpool_fwd)(const REAL* x, REAL* y, int32_t* idx, int N, int H, int W, int C,
                         int ksize, int stride, int pad) {
  const int P = out_dim(H, pad, ksize, stride), Q = out_dim(W, pad, ksize, stride);
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int p = 0; p < P; ++p)
      for (int q = 0; q < Q; ++q)
        for (int c = 0; c < C; ++c) {
          int have = 0, best_at = -1;
          REAL best = 0;
          for (int r = 0; r < ksize; ++r) {
            const int ih = p * stride - pad + r;
            if (ih < 0 || ih >= H) continue;
            for (int s = 0; s < ksize; ++s) {
              const int iw = q * stride - pad + s;
              if (iw < 0 || iw >= W) continue;
              const REAL v = x[(((i64)n * H + ih) * W + iw) * C + c];
              if (!have || v > best) {
                best = v;
                best_at = ih * W + iw;
                have = 1;
              }
            }
          }
          const i64 o = (((i64)n * P + p) * Q + q) * C + c;
          y[o] = best;
          if (idx) idx[o] = best_at;
        }
}

/* Backward: every output gradient goes to the input position that won. */
void FN(orc_maxpool_bwd)(const REAL* x, const REAL* dy, REAL* dx, int N, int H, int W, int C,
                         int ksize, int stride, int pad) {
  const int P = out_dim(H, pad, ksize, stride), Q = out_dim(W, pad, ksize, stride);
  const i64 per_img = (i64)H * W * C;
#pragma omp parallel
  {
    double* acc = (double*)malloc(sizeof(double) * (size_t)per_img);
#pragma omp for schedule(static)
    for (int n = 0; n < N; ++n) {
      for (i64 i = 0; i < per_img; ++i) acc[i] = 0.0;
      for (int p = 0; p < P; ++p)
        for (int q = 0; q < Q; ++q)
          for (int c = 0; c < C; ++c) {
            int have = 0, bh = 0, bw = 0;
            REAL best = 0;
            for (int r = 0; r < ksize; ++r) {
              const int ih = p * stride - pad + r;
              if (ih < 0 || ih >= H) continue;
              for (int s = 0; s < ksize; ++s) {
                const int iw = q * stride - pad + s;
                if (iw < 0 || iw >= W) continue;
                const REAL v = x[(((i64)n * H + ih) * W + iw) * C + c];
                if (!have || v > best) {
                  best = v;
                  bh = ih;
                  bw = iw;
                  have = 1;
                }
              }
            }
            if (have) acc[((i64)bh * W + bw) * C + c] += (double)dy[(((i64)n * P + p) * Q + q) * C + c];
          }
      for (i64 i = 0; i < per_img; ++i) dx[(i64)n * per_img + i] = (REAL)acc[i];
    }
    free(acc);
  }
}

/* Global average pooling over the HW positions of each image, and its adjoint. */
void FN(orc_avgpool_fwd)(const REAL* x, REAL* y, int N, int HW, int C) {
#pragma omp parallel for schedule(static)
  for (int n = 0; n < N; ++n)
    for (int c = 0; c < C; ++c) {
      double s = 0.0;
      for (int i = 0; i < HW; ++i) s += (double)x[((i64)n * HW + i) * C + c];
      y[(i64)n * C + c] = (REAL)(s / (double)HW);
    }
}

void FN(orc_avgpool_bwd)(const REAL* dy, REAL* dx, int N, int HW, int C) {
#pragma omp parallel for schedule(static)
  for (int n = 0; n < N; ++n)
    for (int i = 0; i < HW; ++i)
      for (int c = 0; c < C; ++c)
        dx[((i64)n * HW + i) * C + c] = (REAL)((double)dy[(i64)n * C + c] / (double)HW);
}

/* ------------------------------------------------------------------------
 * Fully connected classifier: logits[n,k] = sum_c a[n,c]*W[k,c] + b[k], and the
 * three gradients da, dW, db.
 * ---------------------------------------------------------------------- */
void FN(orc_fc_fwd)(const REAL* a, const REAL* W, const REAL* b, REAL* logits, int N, int Cin,
                    int K) {
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int k = 0; k < K; ++k) {
      double s = 0.0;
      for (int c = 0; c < Cin; ++c) s += (double)a[(i64)n * Cin + c] * (double)W[(i64)k * Cin + c];
      logits[(i64)n * K + k] = (REAL)(s + (double)b[k]);
    }
}

void FN(orc_fc_bwd)(const REAL* a, const REAL* W, const REAL* dlogits, REAL* da, REAL* dW, REAL* db,
                    int N, int Cin, int K) {
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int c = 0; c < Cin; ++c) {
      double s = 0.0;
      for (int k = 0; k < K; ++k) s += (double)dlogits[(i64)n * K + k] * (double)W[(i64)k * Cin + c];
      da[(i64)n * Cin + c] = (REAL)s;
    }
#pragma omp parallel for schedule(static)
  for (int k = 0; k < K; ++k) {
    double sb = 0.0;
    for (int n = 0; n < N; ++n) sb += (double)dlogits[(i64)n * K + k];
    db[k] = (REAL)sb;
    for (int c = 0; c < Cin; ++c) {
      double s = 0.0;
      for (int n = 0; n < N; ++n) s += (double)dlogits[(i64)n * K + k] * (double)a[(i64)n * Cin + c];
      dW[(i64)k * Cin + c] = (REAL)s;
    }
  }
}

/* ------------------------------------------------------------------------
 * Softmax cross-entropy with label smoothing (Sec. III-A2).  Per row n:
 *   p = softmax(logits[n,:]) (maximum subtracted first),
 *   q_k = (1-ls)*[k == label] + ls/K,
 *   row_loss[n] = -sum_k q_k log p_k,  loss = mean_n row_loss[n],
 *   dlogits[n,k] = grad_scale * (p_k - q_k) / N.
 * ---------------------------------------------------------------------- */
void FN(orc_xent)(const REAL* logits, const int32_t* labels, int N, int K, double ls,
                  double grad_scale, REAL* loss, REAL* row_loss, REAL* dlogits) {
  double total = 0.0;
  for (int n = 0; n < N; ++n) {
    const REAL* l = logits + (i64)n * K;
    double mx = (double)l[0];
    for (int k = 1; k < K; ++k)
      if ((double)l[k] > mx) mx = (double)l[k];
    double se = 0.0;
    for (int k = 0; k < K; ++k) se += exp((double)l[k] - mx);
    const double lse = mx + log(se);
    double rl = 0.0;
    for (int k = 0; k < K; ++k) {
      const double logp = (double)l[k] - lse;
      const double q = (1.0 - ls) * (k == labels[n] ? 1.0 : 0.0) + ls / (double)K;
      rl -= q * logp;
      dlogits[(i64)n * K + k] = (REAL)(grad_scale * (exp(logp) - q) / (double)N);
    }
    if (row_loss) row_loss[n] = (REAL)rl;
    total += rl;
  }
  *loss = (REAL)(total / (double)N);
}

/* ------------------------------------------------------------------------
 * LARS update of one parameter tensor ("layer", Sec. III-A1 and III-B2):
 *   wn = ||w||_2, gn = ||g||_2
 *   local = eta*wn / (gn + wd*wn + eps)   if apply_trust and wn > 0 and gn > 0
 *         = 1                             otherwise
 *   v <- momentum*v + lr*local*(g + wd*w)
 *   w <- w - v
 * norms_out (optional) receives {wn, gn} as doubles.
 * ---------------------------------------------------------------------- */
void FN(orc_lars)(REAL* w, const REAL* g, REAL* v, i64 n, double eta, double momentum, double lr,
                  double wd, double eps, int apply_trust, double* norms_out) {
  double sw = 0.0, sg = 0.0;
  for (i64 i = 0; i < n; ++i) {
    sw += (double)w[i] * (double)w[i];
    sg += (double)g[i] * (double)g[i];
  }
  const double wn = sqrt(sw), gn = sqrt(sg);
  double local = 1.0;
  if (apply_trust && wn > 0.0 && gn > 0.0) local = eta * wn / (gn + wd * wn + eps);
  for (i64 i = 0; i < n; ++i) {
    const double vi = momentum * (double)v[i] + lr * local * ((double)g[i] + wd * (double)w[i]);
    v[i] = (REAL)vi;
    w[i] = (REAL)((double)w[i] - vi);
  }
  if (norms_out) {
    norms_out[0] = wn;
    norms_out[1] = gn;
  }
}
