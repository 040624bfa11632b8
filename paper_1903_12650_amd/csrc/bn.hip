// Training-mode batch normalization fused with ReLU and the residual add
// (Sec. II and III-A3 of the paper: statistics over the local batch only;
// appendix log: epsilon 1e-5, scale and centre on, momentum 0.9).
//
// All kernels are HBM-bound.  x is [m][C] with channels contiguous, so a
// workgroup of 256 threads is laid out as TY rows x TX 16-byte channel vectors
// (TX*16 B contiguous per row, consecutive rows contiguous in memory), every
// thread keeps its own channels in registers while it walks down the rows, and
// rows are only combined once per workgroup through LDS.
//
// Forward:  stats (per-workgroup partial sums) -> finalize (mean, rstd) -> apply.
// Backward: reduce (partial sums of g and g*xhat) -> finalize (dgamma, dbeta) -> apply.
// Partial sums are combined in a fixed order, so results are bitwise reproducible.
//
// Variance uses sums shifted by the channel's first element, K = x[0][c]:
//   mean = K + S1/m, var = S2/m - (S1/m)^2 with S1 = sum(x-K), S2 = sum((x-K)^2),
// which removes the cancellation of the plain E[x^2]-E[x]^2 form whenever K lies
// within a few standard deviations of the mean; partial sums of all workgroups
// then combine by plain addition (done in double).
#include "common.h"

namespace rn50 {

struct BnGeom {
  int V;        // elements per 16-byte vector
  int cvecs;    // C / V
  int tx_log2;  // TX = 1 << tx_log2 threads across channel vectors
  int gy;       // workgroups across channel vectors
  int rpb;      // rows per workgroup
  int nblk;     // workgroups across rows
};

static BnGeom bn_geom(int64_t m, int C, int dtype) {
  BnGeom g;
  g.V = dtype == RN50_BF16 ? 8 : 4;
  g.cvecs = C / g.V;
  g.tx_log2 = 0;
  while ((1 << g.tx_log2) < g.cvecs && g.tx_log2 < 5) ++g.tx_log2;
  const int TX = 1 << g.tx_log2, TY = 256 / TX;
  g.gy = static_cast<int>(ceil_div(g.cvecs, TX));
  int64_t rpb = ceil_div(m, 1024);
  if (rpb < TY * 8) rpb = TY * 8;
  rpb = ceil_div(rpb, TY) * TY;
  g.rpb = static_cast<int>(rpb);
  g.nblk = static_cast<int>(ceil_div(m, rpb));
  return g;
}

// The affine step, written once so that forward and backward take the ReLU
// decision from bit-identical arithmetic.
__device__ __forceinline__ float bn_affine(float x, float scale, float bias) {
  return fmaf(x, scale, bias);
}

// Tree-combine NV floats per thread over the TY rows of the workgroup; the
// result lands in the threads of row 0.
template <int NV>
__device__ __forceinline__ void combine_rows(float* vals, float* lds, int tx_log2) {
  const int TX = 1 << tx_log2, TY = 256 >> tx_log2;
  const int tcol = threadIdx.x & (TX - 1), trow = threadIdx.x >> tx_log2;
  float* mine = lds + static_cast<size_t>(threadIdx.x) * NV;
#pragma unroll
  for (int j = 0; j < NV; ++j) mine[j] = vals[j];
  __syncthreads();
  for (int s = TY >> 1; s >= 1; s >>= 1) {
    if (trow < s) {
      const float* other = lds + static_cast<size_t>((trow + s) * TX + tcol) * NV;
#pragma unroll
      for (int j = 0; j < NV; ++j) mine[j] += other[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int j = 0; j < NV; ++j) vals[j] = mine[j];
}

// ------------------------------------------------------------------- forward
template <typename T>
__global__ __launch_bounds__(256) void bn_stats_kernel(const T* __restrict__ x, int64_t m, int C,
                                                       int tx_log2, int rpb,
                                                       float* __restrict__ partial) {
  constexpr int V = Elem<T>::VEC;
  extern __shared__ float lds[];
  const int TX = 1 << tx_log2, TY = 256 >> tx_log2;
  const int tcol = threadIdx.x & (TX - 1), trow = threadIdx.x >> tx_log2;
  const int col = blockIdx.y * TX + tcol;
  const bool active = col < C / V;
  float acc[2 * V];
#pragma unroll
  for (int j = 0; j < 2 * V; ++j) acc[j] = 0.f;
  if (active) {
    float K[V];
    Elem<T>::unpack(load16(x + static_cast<int64_t>(col) * V), K);
    const int64_t r0 = static_cast<int64_t>(blockIdx.x) * rpb;
    const int64_t r1 = min(r0 + rpb, m);
    const T* p = x + static_cast<int64_t>(col) * V;
#pragma unroll 4
    for (int64_t r = r0 + trow; r < r1; r += TY) {
      float f[V];
      Elem<T>::unpack(load16(p + r * C), f);
#pragma unroll
      for (int j = 0; j < V; ++j) {
        const float d = f[j] - K[j];
        acc[j] += d;
        acc[V + j] = fmaf(d, d, acc[V + j]);
      }
    }
  }
  combine_rows<2 * V>(acc, lds, tx_log2);
  if (active && trow == 0) {
    float* o1 = partial + (static_cast<int64_t>(blockIdx.x) * 2) * C + col * V;
    float* o2 = o1 + C;
#pragma unroll
    for (int j = 0; j < V; ++j) {
      o1[j] = acc[j];
      o2[j] = acc[V + j];
    }
  }
}

// One wave per channel: sums the nblk partials in double (fixed order).
template <typename T>
__global__ __launch_bounds__(256) void bn_finalize_kernel(const T* __restrict__ x,
                                                          const float* __restrict__ partial,
                                                          int nblk, int64_t m, int C, float eps,
                                                          float* __restrict__ mean_out,
                                                          float* __restrict__ rstd_out,
                                                          float* running_mean, float* running_var,
                                                          float momentum) {
  const int c = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (c >= C) return;
  const int lane = threadIdx.x & 63;
  double s1 = 0.0, s2 = 0.0;
  for (int b = lane; b < nblk; b += 64) {
    s1 += static_cast<double>(partial[(static_cast<int64_t>(b) * 2) * C + c]);
    s2 += static_cast<double>(partial[(static_cast<int64_t>(b) * 2 + 1) * C + c]);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    s1 += __shfl_xor(s1, off, 64);
    s2 += __shfl_xor(s2, off, 64);
  }
  if (lane == 0) {
    const double K = static_cast<double>(Elem<T>::load(x + c));
    const double d = s1 / static_cast<double>(m);
    double var = s2 / static_cast<double>(m) - d * d;
    if (var < 0.0) var = 0.0;
    const double mean = K + d;
    mean_out[c] = static_cast<float>(mean);
    rstd_out[c] = static_cast<float>(1.0 / sqrt(var + static_cast<double>(eps)));
    if (running_mean) running_mean[c] = momentum * running_mean[c] + (1.f - momentum) * static_cast<float>(mean);
    if (running_var) running_var[c] = momentum * running_var[c] + (1.f - momentum) * static_cast<float>(var);
  }
}

template <typename T>
__global__ __launch_bounds__(256) void bn_apply_kernel(const T* __restrict__ x,
                                                       const float* __restrict__ gamma,
                                                       const float* __restrict__ beta,
                                                       const float* __restrict__ mean,
                                                       const float* __restrict__ rstd,
                                                       const T* __restrict__ residual,
                                                       T* __restrict__ y, int64_t m, int C,
                                                       int tx_log2, int rpb, int mode) {
  constexpr int V = Elem<T>::VEC;
  const int TX = 1 << tx_log2, TY = 256 >> tx_log2;
  const int tcol = threadIdx.x & (TX - 1), trow = threadIdx.x >> tx_log2;
  const int col = blockIdx.y * TX + tcol;
  if (col >= C / V) return;
  float scale[V], bias[V];
#pragma unroll
  for (int j = 0; j < V; ++j) {
    const int c = col * V + j;
    scale[j] = gamma[c] * rstd[c];
    bias[j] = beta[c] - mean[c] * scale[j];
  }
  const int64_t r0 = static_cast<int64_t>(blockIdx.x) * rpb;
  const int64_t r1 = min(r0 + rpb, m);
#pragma unroll 4
  for (int64_t r = r0 + trow; r < r1; r += TY) {
    const int64_t off = r * C + static_cast<int64_t>(col) * V;
    float f[V];
    Elem<T>::unpack(load16(x + off), f);
    if (mode == 2) {
      float rr[V];
      Elem<T>::unpack(load16(residual + off), rr);
#pragma unroll
      for (int j = 0; j < V; ++j) f[j] = fmaxf(bn_affine(f[j], scale[j], bias[j]) + rr[j], 0.f);
    } else if (mode == 1) {
#pragma unroll
      for (int j = 0; j < V; ++j) f[j] = fmaxf(bn_affine(f[j], scale[j], bias[j]), 0.f);
    } else {
#pragma unroll
      for (int j = 0; j < V; ++j) f[j] = bn_affine(f[j], scale[j], bias[j]);
    }
    Vec16 o;
    Elem<T>::pack(f, o);
    store16(y + off, o);
  }
}

// ------------------------------------------------------------------ backward
// g = (dz + dz2) * mask for one 16-byte vector.
template <typename T>
__device__ __forceinline__ void masked_grad(const T* dz, const T* dz2, const T* z, int64_t off,
                                            const float* xf, const float* scale, const float* bias,
                                            int mode, float* g) {
  constexpr int V = Elem<T>::VEC;
  Elem<T>::unpack(load16(dz + off), g);
  if (dz2) {
    float g2[V];
    Elem<T>::unpack(load16(dz2 + off), g2);
#pragma unroll
    for (int j = 0; j < V; ++j) g[j] += g2[j];
  }
  if (mode >= 1) {
    if (z) {
      float zf[V];
      Elem<T>::unpack(load16(z + off), zf);
#pragma unroll
      for (int j = 0; j < V; ++j) g[j] = zf[j] > 0.f ? g[j] : 0.f;
    } else {
#pragma unroll
      for (int j = 0; j < V; ++j) g[j] = bn_affine(xf[j], scale[j], bias[j]) > 0.f ? g[j] : 0.f;
    }
  }
}

template <typename T>
__global__ __launch_bounds__(256) void bn_bwd_reduce_kernel(
    const T* __restrict__ dz, const T* __restrict__ dz2, const T* __restrict__ x,
    const T* __restrict__ z, const float* __restrict__ gamma, const float* __restrict__ beta,
    const float* __restrict__ mean, const float* __restrict__ rstd, int64_t m, int C, int tx_log2,
    int rpb, int mode, float* __restrict__ partial) {
  constexpr int V = Elem<T>::VEC;
  extern __shared__ float lds[];
  const int TX = 1 << tx_log2, TY = 256 >> tx_log2;
  const int tcol = threadIdx.x & (TX - 1), trow = threadIdx.x >> tx_log2;
  const int col = blockIdx.y * TX + tcol;
  const bool active = col < C / V;
  float acc[2 * V];
#pragma unroll
  for (int j = 0; j < 2 * V; ++j) acc[j] = 0.f;
  if (active) {
    float scale[V], bias[V], rs[V], nmr[V];
#pragma unroll
    for (int j = 0; j < V; ++j) {
      const int c = col * V + j;
      rs[j] = rstd[c];
      nmr[j] = -mean[c] * rs[j];
      scale[j] = gamma[c] * rs[j];
      bias[j] = (beta ? beta[c] : 0.f) - mean[c] * scale[j];
    }
    const int64_t r0 = static_cast<int64_t>(blockIdx.x) * rpb;
    const int64_t r1 = min(r0 + rpb, m);
#pragma unroll 2
    for (int64_t r = r0 + trow; r < r1; r += TY) {
      const int64_t off = r * C + static_cast<int64_t>(col) * V;
      float xf[V], g[V];
      Elem<T>::unpack(load16(x + off), xf);
      masked_grad<T>(dz, dz2, z, off, xf, scale, bias, mode, g);
#pragma unroll
      for (int j = 0; j < V; ++j) {
        acc[j] += g[j];
        acc[V + j] = fmaf(g[j], fmaf(xf[j], rs[j], nmr[j]), acc[V + j]);
      }
    }
  }
  combine_rows<2 * V>(acc, lds, tx_log2);
  if (active && trow == 0) {
    float* o1 = partial + (static_cast<int64_t>(blockIdx.x) * 2) * C + col * V;
    float* o2 = o1 + C;
#pragma unroll
    for (int j = 0; j < V; ++j) {
      o1[j] = acc[j];
      o2[j] = acc[V + j];
    }
  }
}

__global__ __launch_bounds__(256) void bn_bwd_finalize_kernel(const float* __restrict__ partial,
                                                              int nblk, int C,
                                                              float* __restrict__ dgamma,
                                                              float* __restrict__ dbeta) {
  const int c = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (c >= C) return;
  const int lane = threadIdx.x & 63;
  double s1 = 0.0, s2 = 0.0;
  for (int b = lane; b < nblk; b += 64) {
    s1 += static_cast<double>(partial[(static_cast<int64_t>(b) * 2) * C + c]);
    s2 += static_cast<double>(partial[(static_cast<int64_t>(b) * 2 + 1) * C + c]);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    s1 += __shfl_xor(s1, off, 64);
    s2 += __shfl_xor(s2, off, 64);
  }
  if (lane == 0) {
    dbeta[c] = static_cast<float>(s1);
    dgamma[c] = static_cast<float>(s2);
  }
}

template <typename T>
__global__ __launch_bounds__(256) void bn_bwd_apply_kernel(
    const T* __restrict__ dz, const T* __restrict__ dz2, const T* __restrict__ x,
    const T* __restrict__ z, const float* __restrict__ gamma, const float* __restrict__ beta,
    const float* __restrict__ mean, const float* __restrict__ rstd,
    const float* __restrict__ dgamma, const float* __restrict__ dbeta, T* __restrict__ dx,
    T* __restrict__ dres, int64_t m, int C, int tx_log2, int rpb, int mode) {
  constexpr int V = Elem<T>::VEC;
  const int TX = 1 << tx_log2, TY = 256 >> tx_log2;
  const int tcol = threadIdx.x & (TX - 1), trow = threadIdx.x >> tx_log2;
  const int col = blockIdx.y * TX + tcol;
  if (col >= C / V) return;
  const float inv_m = 1.0f / static_cast<float>(m);
  float scale[V], bias[V], rs[V], nmr[V], mg[V], mgx[V];
#pragma unroll
  for (int j = 0; j < V; ++j) {
    const int c = col * V + j;
    rs[j] = rstd[c];
    nmr[j] = -mean[c] * rs[j];
    scale[j] = gamma[c] * rs[j];
    bias[j] = (beta ? beta[c] : 0.f) - mean[c] * scale[j];
    mg[j] = dbeta[c] * inv_m;
    mgx[j] = dgamma[c] * inv_m;
  }
  const int64_t r0 = static_cast<int64_t>(blockIdx.x) * rpb;
  const int64_t r1 = min(r0 + rpb, m);
#pragma unroll 2
  for (int64_t r = r0 + trow; r < r1; r += TY) {
    const int64_t off = r * C + static_cast<int64_t>(col) * V;
    float xf[V], g[V], o[V];
    Elem<T>::unpack(load16(x + off), xf);
    masked_grad<T>(dz, dz2, z, off, xf, scale, bias, mode, g);
#pragma unroll
    for (int j = 0; j < V; ++j) {
      const float xh = fmaf(xf[j], rs[j], nmr[j]);
      o[j] = scale[j] * (g[j] - mg[j] - xh * mgx[j]);
    }
    Vec16 ov;
    Elem<T>::pack(o, ov);
    store16(dx + off, ov);
    if (mode == 2) {
      Vec16 gv;
      Elem<T>::pack(g, gv);
      store16(dres + off, gv);
    }
  }
}

static int check_desc(const rn50_bn_desc* d, const char* who) {
  RN50_REQUIRE(d, RN50_ERR_INVALID, "%s: null descriptor", who);
  RN50_REQUIRE(d->N > 0 && d->H > 0 && d->W > 0 && d->C > 0, RN50_ERR_INVALID,
               "%s: non-positive size N=%d H=%d W=%d C=%d", who, d->N, d->H, d->W, d->C);
  RN50_REQUIRE(d->dtype == RN50_F32 || d->dtype == RN50_BF16, RN50_ERR_INVALID, "%s: dtype %d", who, d->dtype);
  RN50_REQUIRE(d->mode >= 0 && d->mode <= 2, RN50_ERR_INVALID, "%s: mode %d", who, d->mode);
  RN50_REQUIRE(d->C % (d->dtype == RN50_BF16 ? 8 : 4) == 0, RN50_ERR_UNSUPPORTED,
               "%s: C=%d is not a multiple of the 16-byte vector", who, d->C);
  RN50_REQUIRE(d->eps >= 0.f, RN50_ERR_INVALID, "%s: eps < 0", who);
  return RN50_OK;
}

static size_t bn_ws_bytes(const rn50_bn_desc* d) {
  const int64_t m = static_cast<int64_t>(d->N) * d->H * d->W;
  const BnGeom g = bn_geom(m, d->C, d->dtype);
  return align_up(static_cast<size_t>(g.nblk) * 2 * d->C * sizeof(float), 256);
}

template <typename T>
static void launch_fwd(const rn50_bn_desc* d, const BnGeom& g, int64_t m, const void* x,
                       const float* gamma, const float* beta, const void* residual, void* y,
                       float* save_mean, float* save_rstd, float* rm, float* rv, float momentum,
                       float* partial, hipStream_t s) {
  const size_t lds = 256 * 2 * Elem<T>::VEC * sizeof(float);
  RN50_TIMED("bn_stats", s,
             hipLaunchKernelGGL(bn_stats_kernel<T>, dim3(g.nblk, g.gy), dim3(256), lds, s,
                                static_cast<const T*>(x), m, d->C, g.tx_log2, g.rpb, partial));
  hipLaunchKernelGGL(bn_finalize_kernel<T>, dim3(ceil_div(d->C, 4)), dim3(256), 0, s,
                     static_cast<const T*>(x), partial, g.nblk, m, d->C, d->eps, save_mean,
                     save_rstd, rm, rv, momentum);
  RN50_TIMED("bn_apply", s,
             hipLaunchKernelGGL(bn_apply_kernel<T>, dim3(g.nblk, g.gy), dim3(256), 0, s,
                                static_cast<const T*>(x), gamma, beta, save_mean, save_rstd,
                                static_cast<const T*>(residual), static_cast<T*>(y), m, d->C,
                                g.tx_log2, g.rpb, d->mode));
}

template <typename T>
static void launch_bwd(const rn50_bn_desc* d, const BnGeom& g, int64_t m, const void* dz,
                       const void* dz2, const void* x, const void* z, const float* gamma,
                       const float* beta, const float* mean, const float* rstd, void* dx,
                       void* dres, float* dgamma, float* dbeta, float* partial, hipStream_t s) {
  const size_t lds = 256 * 2 * Elem<T>::VEC * sizeof(float);
  RN50_TIMED("bn_bwd_reduce", s,
             hipLaunchKernelGGL(bn_bwd_reduce_kernel<T>, dim3(g.nblk, g.gy), dim3(256), lds, s,
                                static_cast<const T*>(dz), static_cast<const T*>(dz2),
                                static_cast<const T*>(x), static_cast<const T*>(z), gamma, beta,
                                mean, rstd, m, d->C, g.tx_log2, g.rpb, d->mode, partial));
  hipLaunchKernelGGL(bn_bwd_finalize_kernel, dim3(ceil_div(d->C, 4)), dim3(256), 0, s, partial,
                     g.nblk, d->C, dgamma, dbeta);
  RN50_TIMED("bn_bwd_apply", s,
             hipLaunchKernelGGL(bn_bwd_apply_kernel<T>, dim3(g.nblk, g.gy), dim3(256), 0, s,
                                static_cast<const T*>(dz), static_cast<const T*>(dz2),
                                static_cast<const T*>(x), static_cast<const T*>(z), gamma, beta,
                                mean, rstd, dgamma, dbeta, static_cast<T*>(dx),
                                static_cast<T*>(dres), m, d->C, g.tx_log2, g.rpb, d->mode));
}

}  // namespace rn50

using namespace rn50;

extern "C" size_t bn_relu_fwd_workspace_bytes(const rn50_bn_desc* d) {
  if (!d || d->N <= 0 || d->H <= 0 || d->W <= 0 || d->C <= 0) return 0;
  return bn_ws_bytes(d);
}
extern "C" size_t bn_relu_bwd_workspace_bytes(const rn50_bn_desc* d) {
  return bn_relu_fwd_workspace_bytes(d);
}

extern "C" int bn_relu_fwd(const rn50_bn_desc* d, const void* x, const float* gamma,
                           const float* beta, const void* residual, void* y, float* save_mean,
                           float* save_rstd, float* running_mean, float* running_var,
                           float momentum, void* workspace, size_t workspace_bytes, void* stream) {
  clear_error();
  if (int rc = check_desc(d, "bn_relu_fwd")) return rc;
  RN50_REQUIRE(x && gamma && beta && y && save_mean && save_rstd && workspace, RN50_ERR_INVALID,
               "bn_relu_fwd: null pointer");
  RN50_REQUIRE((d->mode == 2) == (residual != nullptr), RN50_ERR_INVALID,
               "bn_relu_fwd: residual must be given exactly in mode 2");
  RN50_REQUIRE(aligned16(x) && aligned16(y) && aligned16(residual) && aligned16(workspace) &&
                   aligned16(gamma) && aligned16(beta) && aligned16(save_mean) && aligned16(save_rstd),
               RN50_ERR_ALIGN, "bn_relu_fwd: pointer not 16-byte aligned");
  RN50_REQUIRE(workspace_bytes >= bn_ws_bytes(d), RN50_ERR_WORKSPACE,
               "bn_relu_fwd: workspace %zu < %zu bytes", workspace_bytes, bn_ws_bytes(d));
  const int64_t m = static_cast<int64_t>(d->N) * d->H * d->W;
  const BnGeom g = bn_geom(m, d->C, d->dtype);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (d->dtype == RN50_BF16)
    launch_fwd<uint16_t>(d, g, m, x, gamma, beta, residual, y, save_mean, save_rstd, running_mean,
                         running_var, momentum, static_cast<float*>(workspace), s);
  else
    launch_fwd<float>(d, g, m, x, gamma, beta, residual, y, save_mean, save_rstd, running_mean,
                      running_var, momentum, static_cast<float*>(workspace), s);
  return launch_status("bn_relu_fwd");
}

extern "C" int bn_relu_bwd(const rn50_bn_desc* d, const void* dz, const void* dz2, const void* x,
                           const void* z, const float* gamma, const float* beta,
                           const float* save_mean, const float* save_rstd, void* dx,
                           void* dresidual, float* dgamma, float* dbeta, void* workspace,
                           size_t workspace_bytes, void* stream) {
  clear_error();
  if (int rc = check_desc(d, "bn_relu_bwd")) return rc;
  RN50_REQUIRE(dz && x && gamma && save_mean && save_rstd && dx && dgamma && dbeta && workspace,
               RN50_ERR_INVALID, "bn_relu_bwd: null pointer");
  RN50_REQUIRE(d->mode != 2 || (z && dresidual), RN50_ERR_INVALID,
               "bn_relu_bwd: mode 2 needs z and dresidual");
  RN50_REQUIRE(d->mode != 1 || z || beta, RN50_ERR_INVALID,
               "bn_relu_bwd: mode 1 needs z, or beta to recompute the ReLU mask");
  RN50_REQUIRE(aligned16(dz) && aligned16(dz2) && aligned16(x) && aligned16(z) && aligned16(dx) &&
                   aligned16(dresidual) && aligned16(workspace),
               RN50_ERR_ALIGN, "bn_relu_bwd: pointer not 16-byte aligned");
  RN50_REQUIRE(workspace_bytes >= bn_ws_bytes(d), RN50_ERR_WORKSPACE,
               "bn_relu_bwd: workspace %zu < %zu bytes", workspace_bytes, bn_ws_bytes(d));
  const int64_t m = static_cast<int64_t>(d->N) * d->H * d->W;
  const BnGeom g = bn_geom(m, d->C, d->dtype);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (d->dtype == RN50_BF16)
    launch_bwd<uint16_t>(d, g, m, dz, dz2, x, z, gamma, beta, save_mean, save_rstd, dx, dresidual,
                         dgamma, dbeta, static_cast<float*>(workspace), s);
  else
    launch_bwd<float>(d, g, m, dz, dz2, x, z, gamma, beta, save_mean, save_rstd, dx, dresidual,
                      dgamma, dbeta, static_cast<float*>(workspace), s);
  return launch_status("bn_relu_bwd");
}
