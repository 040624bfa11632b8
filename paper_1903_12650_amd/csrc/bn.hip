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
// The first pass of either direction can be left to the convolution that produces
// the tensor (its output stage writes the same rows of partial sums, one per
// output tile): the *_from_partials entry points then run finalize + apply only.
// Partial sums are combined in a fixed order, so results are bitwise reproducible.
//
// Variance uses shifted sums: every row of partials carries its own shift K (the
// first element its producer saw), S1 = sum(x-K), S2 = sum((x-K)^2); the finalize
// pass moves all rows to the first row's shift exactly, in double, and then
//   mean = K + S1/m, var = S2/m - (S1/m)^2,
// which removes the cancellation of the plain E[x^2]-E[x]^2 form whenever K lies
// within a few standard deviations of the mean.
#include <stdlib.h>

#include "common.h"
#include "step_internal.h"

namespace rn50 {

constexpr int kBnRows = 4;  // rows a thread loads before it touches any of them (memory-level parallelism)

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
  // rows per thread: aim at ~1024 workgroups in all, but at least 64 rows per workgroup so that the
  // per-workgroup partial sums stay a few percent of the tensor; a multiple of the 4 rows whose loads
  // are issued together
  const int64_t nblk_target = 1024 / g.gy > 0 ? 1024 / g.gy : 1;
  int64_t rpt = ceil_div(m, static_cast<int64_t>(TY) * nblk_target);
  if (rpt * TY < 64) rpt = ceil_div(64, TY);
  rpt = ceil_div(rpt, kBnRows) * kBnRows;
  const int64_t rpb = rpt * TY;
  g.rpb = static_cast<int>(rpb);
  g.nblk = static_cast<int>(ceil_div(m, rpb));
  return g;
}

// The elementwise passes have no sums to combine, so their geometry is free: at most `target` workgroups,
// each thread streaming 4 to 32 rows.  Measured inside the training step (profiles/bn_apply_grid_step_time_batch40.txt)
// and on a plain copy kernel: many small workgroups that make one round of loads each stream faster than few
// long-running ones (a 16-byte-per-thread copy of 1 GiB runs at 6.2 TB/s, the same copy by 2,048 looping workgroups
// at 4.9), so the target is high enough that every thread of ResNet-50's layers takes its minimum of 4 rows.
constexpr int kBnApplyGroups = 16384, kBnBwdApplyGroups = 16383;  // (distinct values: the tuning override tells them apart)
static BnGeom bn_apply_geom(int64_t m, int C, int dtype, int target) {
  BnGeom g = bn_geom(m, C, dtype);
#ifdef RN50_TUNING  // tuning builds only: RN50_BN_TARGET=forward,backward workgroup targets of the apply passes
  if (const char* e = getenv("RN50_BN_TARGET")) {
    int tf = 0, tb = 0;
    if (sscanf(e, "%d,%d", &tf, &tb) == 2) target = target == kBnApplyGroups ? tf : tb;
  }
#endif
  const int TY = 256 >> g.tx_log2;
  int64_t rpt = ceil_div(m * g.gy, static_cast<int64_t>(TY) * target);
  rpt = ceil_div(rpt, kBnRows) * kBnRows;
  if (rpt > 32) rpt = 32;
  g.rpb = static_cast<int>(rpt) * TY;
  g.nblk = static_cast<int>(ceil_div(m, g.rpb));
  return g;
}

// Geometry of an apply pass that finalizes by itself: column slices of 8 vectors (TY = 32 rows per pass), about
// kBnSelfFinalizeGroups workgroups, every thread a multiple of 4 rows.
constexpr int kBnSelfFinalizeGroups = 768;
static void bn_self_finalize_geom(int64_t m, int C, int V, int* gy_out, int* rpb_out) {
  int target = kBnSelfFinalizeGroups;
#ifdef RN50_TUNING  // tuning builds only: RN50_BN_FIN_TARGET=workgroups
  if (const char* e = getenv("RN50_BN_FIN_TARGET")) target = atoi(e) > 0 ? atoi(e) : target;
#endif
  const int TY = 32;
  const int gy = static_cast<int>(ceil_div(C / V, 8));
  const int64_t nblk_target = target / gy > 0 ? target / gy : 1;
  int64_t rpt = ceil_div(m, TY * nblk_target);
  rpt = ceil_div(rpt, kBnRows) * kBnRows;
  *gy_out = gy;
  *rpb_out = static_cast<int>(rpt) * TY;
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
  float acc[2 * V], K[V];
#pragma unroll
  for (int j = 0; j < 2 * V; ++j) acc[j] = 0.f;
  if (active) {
    Elem<T>::unpack(load16(x + static_cast<int64_t>(col) * V), K);
    const int64_t r0 = static_cast<int64_t>(blockIdx.x) * rpb;
    const int64_t r1 = min(r0 + rpb, m);
    const T* p = x + static_cast<int64_t>(col) * V;
    for (int64_t r = r0 + trow; r < r1; r += kBnRows * TY) {
      Vec16 v[kBnRows];
#pragma unroll
      for (int u = 0; u < kBnRows; ++u) v[u] = load16(p + min(r + u * TY, r1 - 1) * C);
#pragma unroll
      for (int u = 0; u < kBnRows; ++u) {
        if (r + u * TY < r1) {
          float f[V];
          Elem<T>::unpack(v[u], f);
#pragma unroll
          for (int j = 0; j < V; ++j) {
            const float d = f[j] - K[j];
            acc[j] += d;
            acc[V + j] = fmaf(d, d, acc[V + j]);
          }
        }
      }
    }
  }
  combine_rows<2 * V>(acc, lds, tx_log2);
  if (active && trow == 0) {
    // partial[plane][c][row]: the rows of one channel are contiguous for the finalize pass
    const int64_t nrows = gridDim.x;
#pragma unroll
    for (int j = 0; j < V; ++j) {
      float* o = partial + static_cast<int64_t>(col * V + j) * nrows + blockIdx.x;
      o[0] = K[j];
      o[C * nrows] = acc[j];
      o[2 * C * nrows] = acc[V + j];
    }
  }
}

// Finalize passes.  The partial sums lie as partial[plane][c][row], `nrows` rows per channel, so one wave
// reads the rows of one channel with contiguous 256-byte loads.  A workgroup serves 4/wpc channels with
// wpc (1 or 4) waves each; lane l of wave w adds rows (w*64 + l) + 64*wpc*i, i = 0, 1, ... in order, then
// the lanes are combined by a fixed butterfly and the waves in order: all in double, a fixed order.
__device__ __forceinline__ double wave_sum_double(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
// Combines (s1, s2) over the waves of a channel; true in lane 0 of the channel's first wave, with the totals.
__device__ __forceinline__ bool finalize_combine(double* s1, double* s2, int wpc, int c, int C) {
  __shared__ double red[2][4];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  double a = wave_sum_double(*s1), b = wave_sum_double(*s2);
  if (wpc == 1) {
    *s1 = a; *s2 = b;
    return lane == 0 && c < C;
  }
  if (lane == 0) {
    red[0][wave] = a;
    red[1][wave] = b;
  }
  __syncthreads();
  *s1 = ((red[0][0] + red[0][1]) + red[0][2]) + red[0][3];
  *s2 = ((red[1][0] + red[1][1]) + red[1][2]) + red[1][3];
  return threadIdx.x == 0 && c < C;
}
static int finalize_wpc(int nrows) { return nrows >= 512 ? 4 : 1; }
static int finalize_grid(int C, int nrows) { return static_cast<int>(ceil_div(C * finalize_wpc(nrows), 4)); }

// Forward statistics: rows [shift, S1, S2] over `rpp` consecutive rows of x each (the last may cover
// fewer), every row with a shift of its own: S1 = sum(x - shift), S2 = sum((x - shift)^2).  They are moved
// to the first row's shift K0 exactly, in double,
//   sum(x - K0) = S1 + n e,  sum((x - K0)^2) = S2 + 2 e S1 + n e^2,  e = shift - K0.
__global__ __launch_bounds__(256) void bn_finalize_kernel(const float* __restrict__ partial, int nrows, int rpp,
                                                          int64_t m, int C, int wpc, int row_major, float eps,
                                                          float* __restrict__ mean_out,
                                                          float* __restrict__ rstd_out,
                                                          float* running_mean, float* running_var,
                                                          float momentum) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int c = wpc == 1 ? blockIdx.x * 4 + wave : blockIdx.x;
  const int first = (wpc == 1 ? 0 : wave * 64) + lane, step = 64 * wpc;
  double s1 = 0.0, s2 = 0.0, k0 = 0.0;
  if (c < C && row_major) {
    // the layout of layers with few tile rows, whose apply pass normally finalizes by itself: per tile row and
    // channel the doubles (sum y, sum y^2); k0 stays 0
    const double2* pd = reinterpret_cast<const double2*>(partial) + c;
    for (int b = first; b < nrows; b += step) {
      const double2 v = pd[static_cast<int64_t>(b) * C];
      s1 += v.x;
      s2 += v.y;
    }
  } else if (c < C) {
    const int64_t rs = 1;
    const float* pk = partial + static_cast<int64_t>(c) * nrows;
    const float* p1 = pk + static_cast<int64_t>(C) * nrows;
    const float* p2 = p1 + static_cast<int64_t>(C) * nrows;
    k0 = static_cast<double>(pk[0]);
    constexpr int U = 4;
    int b = first;
    for (; b + (U - 1) * step < nrows; b += U * step) {
      float vk[U], v1[U], v2[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        vk[u] = pk[(b + u * step) * rs];
        v1[u] = p1[(b + u * step) * rs];
        v2[u] = p2[(b + u * step) * rs];
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int64_t left = m - static_cast<int64_t>(b + u * step) * rpp;
        const double n = static_cast<double>(left < rpp ? left : rpp);
        const double e = static_cast<double>(vk[u]) - k0, a1 = static_cast<double>(v1[u]);
        s1 += a1 + n * e;
        s2 += static_cast<double>(v2[u]) + e * (2.0 * a1 + n * e);
      }
    }
    for (; b < nrows; b += step) {
      const int64_t left = m - static_cast<int64_t>(b) * rpp;
      const double n = static_cast<double>(left < rpp ? left : rpp);
      const double e = static_cast<double>(pk[b * rs]) - k0, a1 = static_cast<double>(p1[b * rs]);
      s1 += a1 + n * e;
      s2 += static_cast<double>(p2[b * rs]) + e * (2.0 * a1 + n * e);
    }
  }
  if (!finalize_combine(&s1, &s2, wpc, c, C)) return;
  const double d = s1 / static_cast<double>(m);
  double var = s2 / static_cast<double>(m) - d * d;
  if (var < 0.0) var = 0.0;
  const double mean = k0 + d;
  mean_out[c] = static_cast<float>(mean);
  rstd_out[c] = static_cast<float>(1.0 / sqrt(var + static_cast<double>(eps)));
  if (running_mean) running_mean[c] = momentum * running_mean[c] + (1.f - momentum) * static_cast<float>(mean);
  if (running_var) running_var[c] = momentum * running_var[c] + (1.f - momentum) * static_cast<float>(var);
}

// What a pass that finalizes its own statistics gets on top of the apply pass's arguments (FIN kernels below):
// the per-tile sums in ROW-major order (forward: double2 per tile row and channel, sums at shift 0; backward: float
// planes partial[plane][tile row][C]) and where the results go (backward: mean_out = dbeta, rstd_out = dgamma).
struct BnFinArgs {
  const float* partial;
  int nrows, rpp;  // tile rows; (unused by the row-major layouts) pixel rows summed per tile row
  float eps, momentum;
  float *mean_out, *rstd_out, *running_mean, *running_var;
};
// Forward statistics of the CS channels from c0 on, by all 256 threads of a workgroup, into mean_s / rstd_s (LDS),
// from row-major sums: per tile row and channel the doubles (sum y, sum y^2) that the convolution's output stage
// made of its shifted float sums.  Thread (channel ch, part p) adds tile rows p, p + P, ... in order, the P parts
// are added in order: a fixed order, the same in every workgroup that computes these channels.  Ends with a barrier.
template <int CS>
__device__ __forceinline__ void finalize_slice_fwd(const BnFinArgs& f, int64_t m, int C, int c0, bool writer,
                                                   float* mean_s, float* rstd_s) {
  constexpr int P = 256 / CS, U = 4;
  __shared__ double red[2][256];
  const int ch = threadIdx.x % CS, part = threadIdx.x / CS;
  const int c = min(c0 + ch, C - 1);
  const double2* pk = reinterpret_cast<const double2*>(f.partial) + c;
  double s1 = 0.0, s2 = 0.0;
  for (int b = part; b < f.nrows; b += P * U) {
    double2 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = pk[static_cast<int64_t>(min(b + u * P, f.nrows - 1)) * C];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (b + u * P < f.nrows) {
        s1 += v[u].x;
        s2 += v[u].y;
      }
    }
  }
  red[0][threadIdx.x] = s1;
  red[1][threadIdx.x] = s2;
  __syncthreads();
  if (threadIdx.x < CS) {
    double t1 = red[0][ch], t2 = red[1][ch];
#pragma unroll
    for (int q = 1; q < P; ++q) {
      t1 += red[0][q * CS + ch];
      t2 += red[1][q * CS + ch];
    }
    const double mean = t1 / static_cast<double>(m);
    double var = t2 / static_cast<double>(m) - mean * mean;
    if (var < 0.0) var = 0.0;
    const float mf = static_cast<float>(mean), rf = static_cast<float>(1.0 / sqrt(var + static_cast<double>(f.eps)));
    mean_s[ch] = mf;
    rstd_s[ch] = rf;
    if (writer && c0 + ch < C) {
      f.mean_out[c] = mf;
      f.rstd_out[c] = rf;
      if (f.running_mean) f.running_mean[c] = f.momentum * f.running_mean[c] + (1.f - f.momentum) * mf;
      if (f.running_var) f.running_var[c] = f.momentum * f.running_var[c] + (1.f - f.momentum) * static_cast<float>(var);
    }
  }
  __syncthreads();
}

// FIN: the pass takes its statistics from the row-major per-tile sums itself (fin), every workgroup for the 8
// vector columns it applies (tx_log2 = 3), and the first row block of every column slice stores them: no
// finalize launch in front.  For layers with few tile rows the redundant reads of the sums are far cheaper than a
// launch on the step's dependency chain (about 4 us whatever it computes).
template <typename T, bool FIN = false>
__global__ __launch_bounds__(256) void bn_apply_kernel(const T* __restrict__ x,
                                                       const float* __restrict__ gamma,
                                                       const float* __restrict__ beta,
                                                       const float* __restrict__ mean,
                                                       const float* __restrict__ rstd,
                                                       const T* __restrict__ residual,
                                                       T* __restrict__ y, uint8_t* __restrict__ relu_mask,
                                                       int64_t m, int C, int tx_log2, int rpb, int mode,
                                                       const BnFinArgs fin) {
  constexpr int V = Elem<T>::VEC;
  const int TX = 1 << tx_log2, TY = 256 >> tx_log2;
  const int tcol = threadIdx.x & (TX - 1), trow = threadIdx.x >> tx_log2;
  const int col = blockIdx.y * TX + tcol;
  __shared__ float mean_s[FIN ? 8 * V : 1], rstd_s[FIN ? 8 * V : 1];
  if (!FIN && col >= C / V) return;
  const bool live = col < C / V;  // (FIN: every thread takes part in the statistics)
  const int64_t r0 = static_cast<int64_t>(blockIdx.x) * rpb;
  const int64_t r1 = min(r0 + rpb, m);
  int64_t r = r0 + trow;
  int64_t off[kBnRows];
  Vec16 vx[kBnRows], vr[kBnRows];
  auto load_rows = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int u = 0; u < kBnRows; ++u) {
      off[u] = min(r + u * TY, r1 - 1) * C + static_cast<int64_t>(col) * V;
      vx[u] = load16(x + off[u]);
    }
    if (mode == 2) {
#pragma unroll
      for (int u = 0; u < kBnRows; ++u) vr[u] = load16(residual + off[u]);
    }
  };
  // the first rows are requested before the per-channel values, so both arrive in one round trip
  if (live && r < r1) load_rows();
  float scale[V], bias[V], cg[V], cb[V], cm[V], cr[V];
  if (live) {
    load_floats<V>(gamma + col * V, cg);
    load_floats<V>(beta + col * V, cb);
  }
  if constexpr (FIN) {
    finalize_slice_fwd<8 * V>(fin, m, C, blockIdx.y * 8 * V, blockIdx.x == 0, mean_s, rstd_s);
    if (!live) return;
#pragma unroll
    for (int j = 0; j < V; ++j) {
      cm[j] = mean_s[tcol * V + j];
      cr[j] = rstd_s[tcol * V + j];
    }
  } else {
    load_floats<V>(mean + col * V, cm);
    load_floats<V>(rstd + col * V, cr);
  }
#pragma unroll
  for (int j = 0; j < V; ++j) bn_coeffs(cg[j], cb[j], cm[j], cr[j], &scale[j], &bias[j]);
  for (; r < r1; r += kBnRows * TY) {
    if (r != r0 + trow) load_rows();
#pragma unroll
    for (int u = 0; u < kBnRows; ++u) {
      if (r + u * TY < r1) {
        float f[V];
        Elem<T>::unpack(vx[u], f);
        if (mode == 2) {
          float rr[V];
          Elem<T>::unpack(vr[u], rr);
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
        store16(y + off[u], o);
        if (relu_mask) {  // bit j: stored output j is positive; one byte per 16-byte vector
          float zf[V];
          Elem<T>::unpack(o, zf);
          uint32_t bits = 0;
#pragma unroll
          for (int j = 0; j < V; ++j) bits |= (zf[j] > 0.f ? 1u : 0u) << j;
          relu_mask[off[u] / V] = static_cast<uint8_t>(bits);
        }
      }
    }
  }
}

// ------------------------------------------------------------------ backward
// The backward kernels are compiled per operand set, so that a thread only holds registers for what its
// launch reads: DZ2 = a second gradient branch is added; ZK = where the ReLU decision comes from
// (0: recomputed from x, or no ReLU; 1: the forward output z; 2: the recorded bits).
// The operands of kBnRows rows, loaded before any is used.
template <bool DZ2, int ZK>
struct BwdRows {
  Vec16 x[kBnRows], dz[kBnRows], dz2[DZ2 ? kBnRows : 1], z[ZK == 1 ? kBnRows : 1];
  uint32_t zbits[ZK == 2 ? kBnRows : 1];
  int64_t off[kBnRows];
};
template <typename T, bool DZ2, int ZK>
__device__ __forceinline__ void load_bwd_rows(BwdRows<DZ2, ZK>& b, const T* dz, const T* dz2, const T* x,
                                              const T* z, const uint8_t* zmask, int64_t r, int64_t r1, int TY,
                                              int C, int col) {
  constexpr int V = Elem<T>::VEC;
#pragma unroll
  for (int u = 0; u < kBnRows; ++u) {
    b.off[u] = min(r + u * TY, r1 - 1) * C + static_cast<int64_t>(col) * V;
    b.x[u] = load16(x + b.off[u]);
    b.dz[u] = load16(dz + b.off[u]);
  }
  if (DZ2) {
#pragma unroll
    for (int u = 0; u < kBnRows; ++u) b.dz2[DZ2 ? u : 0] = load16(dz2 + b.off[u]);
  }
  if (ZK == 2) {
#pragma unroll
    for (int u = 0; u < kBnRows; ++u) b.zbits[ZK == 2 ? u : 0] = zmask[b.off[u] / V];
  } else if (ZK == 1) {
#pragma unroll
    for (int u = 0; u < kBnRows; ++u) b.z[ZK == 1 ? u : 0] = load16(z + b.off[u]);
  }
}

// g = (dz + dz2) * mask for one 16-byte vector.
template <typename T, bool DZ2, int ZK>
__device__ __forceinline__ void masked_grad(const BwdRows<DZ2, ZK>& b, int u, const float* xf, const float* scale,
                                            const float* bias, int mode, float* g) {
  constexpr int V = Elem<T>::VEC;
  const Vec16& vdz = b.dz[u];
  const Vec16& vdz2 = b.dz2[DZ2 ? u : 0];
  const Vec16& vz = b.z[ZK == 1 ? u : 0];
  const uint32_t zbits = b.zbits[ZK == 2 ? u : 0];
  constexpr bool has_dz2 = DZ2, has_z = ZK == 1, has_zbits = ZK == 2;
  Elem<T>::unpack(vdz, g);
  if (has_dz2) {
    float g2[V];
    Elem<T>::unpack(vdz2, g2);
#pragma unroll
    for (int j = 0; j < V; ++j) g[j] += g2[j];
  }
  if (mode >= 1) {
    if (has_zbits) {
#pragma unroll
      for (int j = 0; j < V; ++j) g[j] = (zbits >> j) & 1u ? g[j] : 0.f;
    } else if (has_z) {
      float zf[V];
      Elem<T>::unpack(vz, zf);
#pragma unroll
      for (int j = 0; j < V; ++j) g[j] = zf[j] > 0.f ? g[j] : 0.f;
    } else {
#pragma unroll
      for (int j = 0; j < V; ++j) g[j] = bn_affine(xf[j], scale[j], bias[j]) > 0.f ? g[j] : 0.f;
    }
  }
}

template <typename T, bool DZ2, int ZK>
__global__ __launch_bounds__(256) void bn_bwd_reduce_kernel(
    const T* __restrict__ dz, const T* __restrict__ dz2, const T* __restrict__ x,
    const T* __restrict__ z, const uint8_t* __restrict__ zmask, const float* __restrict__ gamma,
    const float* __restrict__ beta,
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
    float scale[V], bias[V], rs[V], nmr[V], cg[V], cb[V], cm[V];
    load_floats<V>(gamma + col * V, cg);
    load_floats<V>(mean + col * V, cm);
    load_floats<V>(rstd + col * V, rs);
    if (beta) {
      load_floats<V>(beta + col * V, cb);
    } else {
#pragma unroll
      for (int j = 0; j < V; ++j) cb[j] = 0.f;
    }
#pragma unroll
    for (int j = 0; j < V; ++j) {
      nmr[j] = -cm[j] * rs[j];
      bn_coeffs(cg[j], cb[j], cm[j], rs[j], &scale[j], &bias[j]);
    }
    const int64_t r0 = static_cast<int64_t>(blockIdx.x) * rpb;
    const int64_t r1 = min(r0 + rpb, m);
    for (int64_t r = r0 + trow; r < r1; r += kBnRows * TY) {
      BwdRows<DZ2, ZK> b;
      load_bwd_rows<T, DZ2, ZK>(b, dz, dz2, x, z, zmask, r, r1, TY, C, col);
#pragma unroll
      for (int u = 0; u < kBnRows; ++u) {
        if (r + u * TY < r1) {
          float xf[V], g[V];
          Elem<T>::unpack(b.x[u], xf);
          masked_grad<T, DZ2, ZK>(b, u, xf, scale, bias, mode, g);
#pragma unroll
          for (int j = 0; j < V; ++j) {
            acc[j] += g[j];
            acc[V + j] = fmaf(g[j], fmaf(xf[j], rs[j], nmr[j]), acc[V + j]);
          }
        }
      }
    }
  }
  combine_rows<2 * V>(acc, lds, tx_log2);
  if (active && trow == 0) {
    const int64_t nrows = gridDim.x;
#pragma unroll
    for (int j = 0; j < V; ++j) {
      float* o = partial + static_cast<int64_t>(col * V + j) * nrows + blockIdx.x;
      o[0] = acc[j];
      o[C * nrows] = acc[V + j];
    }
  }
}

__global__ __launch_bounds__(256) void bn_bwd_finalize_kernel(const float* __restrict__ partial,
                                                              int nrows, int C, int wpc,
                                                              float* __restrict__ dgamma,
                                                              float* __restrict__ dbeta) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int c = wpc == 1 ? blockIdx.x * 4 + wave : blockIdx.x;
  const int first = (wpc == 1 ? 0 : wave * 64) + lane, step = 64 * wpc;
  double s1 = 0.0, s2 = 0.0;
  if (c < C) {
    const float* p1 = partial + static_cast<int64_t>(c) * nrows;
    const float* p2 = p1 + static_cast<int64_t>(C) * nrows;
    constexpr int U = 4;
    int b = first;
    for (; b + (U - 1) * step < nrows; b += U * step) {
      float v1[U], v2[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        v1[u] = p1[b + u * step];
        v2[u] = p2[b + u * step];
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        s1 += static_cast<double>(v1[u]);
        s2 += static_cast<double>(v2[u]);
      }
    }
    for (; b < nrows; b += step) {
      s1 += static_cast<double>(p1[b]);
      s2 += static_cast<double>(p2[b]);
    }
  }
  if (!finalize_combine(&s1, &s2, wpc, c, C)) return;
  dbeta[c] = static_cast<float>(s1);
  dgamma[c] = static_cast<float>(s2);
}

// Backward sums of the CS channels from c0 on, from row-major float planes partial[plane][tile row][C]
// (plane 0: sum g, plane 1: sum g * xhat), by all 256 threads, in double and in the fixed order of
// finalize_slice_fwd; dbeta / dgamma land in db_s / dg_s (LDS).  Ends with a barrier.
template <int CS>
__device__ __forceinline__ void finalize_slice_bwd(const BnFinArgs& f, int C, int c0, bool writer, float* db_s,
                                                   float* dg_s) {
  constexpr int P = 256 / CS, U = 4;
  __shared__ double red[2][256];
  const int ch = threadIdx.x % CS, part = threadIdx.x / CS;
  const int c = min(c0 + ch, C - 1);
  const int64_t plane = static_cast<int64_t>(f.nrows) * C;
  const float* p1 = f.partial + c;
  double s1 = 0.0, s2 = 0.0;
  for (int b = part; b < f.nrows; b += P * U) {
    float v1[U], v2[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t at = static_cast<int64_t>(min(b + u * P, f.nrows - 1)) * C;
      v1[u] = p1[at];
      v2[u] = p1[plane + at];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (b + u * P < f.nrows) {
        s1 += static_cast<double>(v1[u]);
        s2 += static_cast<double>(v2[u]);
      }
    }
  }
  red[0][threadIdx.x] = s1;
  red[1][threadIdx.x] = s2;
  __syncthreads();
  if (threadIdx.x < CS) {
    double t1 = red[0][ch], t2 = red[1][ch];
#pragma unroll
    for (int q = 1; q < P; ++q) {
      t1 += red[0][q * CS + ch];
      t2 += red[1][q * CS + ch];
    }
    db_s[ch] = static_cast<float>(t1);
    dg_s[ch] = static_cast<float>(t2);
    if (writer && c0 + ch < C) {
      f.mean_out[c] = static_cast<float>(t1);  // dbeta
      f.rstd_out[c] = static_cast<float>(t2);  // dgamma
    }
  }
  __syncthreads();
}

// FIN: as in bn_apply_kernel -- the pass adds up the row-major per-tile sums of its 8 vector columns itself
// (tx_log2 = 3) and the first row block of every column slice stores dgamma / dbeta.
template <typename T, bool DZ2, int ZK, bool FIN = false>
__global__ __launch_bounds__(256) void bn_bwd_apply_kernel(
    const T* __restrict__ dz, const T* __restrict__ dz2, const T* __restrict__ x,
    const T* __restrict__ z, const uint8_t* __restrict__ zmask, const float* __restrict__ gamma,
    const float* __restrict__ beta,
    const float* __restrict__ mean, const float* __restrict__ rstd,
    const float* __restrict__ dgamma, const float* __restrict__ dbeta, T* __restrict__ dx,
    T* __restrict__ dres, int64_t m, int C, int tx_log2, int rpb, int mode, const BnFinArgs fin) {
  constexpr int V = Elem<T>::VEC;
  const int TX = 1 << tx_log2, TY = 256 >> tx_log2;
  const int tcol = threadIdx.x & (TX - 1), trow = threadIdx.x >> tx_log2;
  int col = blockIdx.y * TX + tcol;
  __shared__ float db_s[FIN ? 8 * V : 1], dg_s[FIN ? 8 * V : 1];
  if (!FIN && col >= C / V) return;
  const bool live = col < C / V;  // (FIN: every thread takes part in the sums)
  if (!live) col = C / V - 1;      // (its loads stay in range; it leaves before it stores anything)
  const int64_t r0 = static_cast<int64_t>(blockIdx.x) * rpb;
  const int64_t r1 = min(r0 + rpb, m);
  int64_t r = r0 + trow;
  // the first rows are requested before the per-channel values, so both arrive in one round trip
  BwdRows<DZ2, ZK> b;
  if (live && r < r1) load_bwd_rows<T, DZ2, ZK>(b, dz, dz2, x, z, zmask, r, r1, TY, C, col);
  const float inv_m = 1.0f / static_cast<float>(m);
  float scale[V], bias[V], rs[V], nmr[V], mg[V], mgx[V], cg[V], cb[V], cm[V];
  load_floats<V>(gamma + col * V, cg);
  load_floats<V>(mean + col * V, cm);
  load_floats<V>(rstd + col * V, rs);
  if constexpr (FIN) {
    finalize_slice_bwd<8 * V>(fin, C, blockIdx.y * 8 * V, blockIdx.x == 0, db_s, dg_s);
    if (!live) return;
#pragma unroll
    for (int j = 0; j < V; ++j) {
      mg[j] = db_s[tcol * V + j];
      mgx[j] = dg_s[tcol * V + j];
    }
  } else {
    load_floats<V>(dbeta + col * V, mg);
    load_floats<V>(dgamma + col * V, mgx);
  }
  if (beta) {
    load_floats<V>(beta + col * V, cb);
  } else {
#pragma unroll
    for (int j = 0; j < V; ++j) cb[j] = 0.f;
  }
#pragma unroll
  for (int j = 0; j < V; ++j) {
    nmr[j] = -cm[j] * rs[j];
    bn_coeffs(cg[j], cb[j], cm[j], rs[j], &scale[j], &bias[j]);
    mg[j] *= inv_m;
    mgx[j] *= inv_m;
  }
  for (; r < r1; r += kBnRows * TY) {
    if (r != r0 + trow) load_bwd_rows<T, DZ2, ZK>(b, dz, dz2, x, z, zmask, r, r1, TY, C, col);
#pragma unroll
    for (int u = 0; u < kBnRows; ++u) {
      if (r + u * TY < r1) {
        float xf[V], g[V], o[V];
        Elem<T>::unpack(b.x[u], xf);
        masked_grad<T, DZ2, ZK>(b, u, xf, scale, bias, mode, g);
#pragma unroll
        for (int j = 0; j < V; ++j) {
          const float xh = fmaf(xf[j], rs[j], nmr[j]);
          o[j] = scale[j] * (g[j] - mg[j] - xh * mgx[j]);
        }
        Vec16 ov;
        Elem<T>::pack(o, ov);
        store16(dx + b.off[u], ov);
        if (mode == 2 && dres) {
          Vec16 gv;
          Elem<T>::pack(g, gv);
          store16(dres + b.off[u], gv);
        }
      }
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

int bn_desc_check(const rn50_bn_desc* d, const char* who) { return check_desc(d, who); }

static size_t bn_ws_bytes(const rn50_bn_desc* d) {
  const int64_t m = static_cast<int64_t>(d->N) * d->H * d->W;
  const BnGeom g = bn_geom(m, d->C, d->dtype);
  return align_up(static_cast<size_t>(g.nblk) * 3 * d->C * sizeof(float), 256);
}

// finalize + apply from partial statistics rows (see bn_finalize_kernel)
template <typename T>
static void launch_fwd_tail(const rn50_bn_desc* d, const BnGeom& g, int64_t m, const void* x,
                            const float* gamma, const float* beta, const void* residual, void* y,
                            uint8_t* relu_mask, float* save_mean, float* save_rstd, float* rm, float* rv,
                            float momentum, const float* partial, int nrows, int rpp, bool row_major, hipStream_t s) {
  if (row_major && y) {
    // few tile rows: the apply pass finalizes for itself
    int gy, rpb;
    bn_self_finalize_geom(m, d->C, d->dtype == RN50_BF16 ? 8 : 4, &gy, &rpb);
    const BnFinArgs fin{partial, nrows, rpp, d->eps, momentum, save_mean, save_rstd, rm, rv};
    RN50_LAUNCH("bn_apply", (bn_apply_kernel<T, true>), dim3(static_cast<unsigned>(ceil_div(m, rpb)), gy), dim3(256), 0, s, static_cast<const T*>(x), gamma, beta, nullptr, nullptr, static_cast<const T*>(residual), static_cast<T*>(y), relu_mask, m, d->C, 3, rpb, d->mode, fin);
    return;
  }
#ifdef RN50_TUNING  // what-if measurement: the step without its finalize launches (results are then wrong)
  static const bool skip_fin = getenv("RN50_SKIP_BN_FINALIZE") != nullptr;
  static const int skip_below = getenv("RN50_SKIP_BN_FINALIZE_ROWS") ? atoi(getenv("RN50_SKIP_BN_FINALIZE_ROWS")) : 1 << 30;
  if (!skip_fin || nrows > skip_below)
#endif
  RN50_LAUNCH("bn_finalize", bn_finalize_kernel, dim3(finalize_grid(d->C, nrows)), dim3(256), 0, s, partial, nrows, rpp, m, d->C, finalize_wpc(nrows), row_major ? 1 : 0, d->eps, save_mean, save_rstd, rm, rv, momentum);
  if (!y) return;  // statistics only: the consumer applies the layer while it loads its operand
  const BnGeom ga = bn_apply_geom(m, d->C, d->dtype, kBnApplyGroups);
  RN50_LAUNCH("bn_apply", bn_apply_kernel<T>, dim3(ga.nblk, ga.gy), dim3(256), 0, s, static_cast<const T*>(x), gamma, beta, save_mean, save_rstd, static_cast<const T*>(residual), static_cast<T*>(y), relu_mask, m, d->C, ga.tx_log2, ga.rpb, d->mode, BnFinArgs{});
}

template <typename T>
static void launch_fwd(const rn50_bn_desc* d, const BnGeom& g, int64_t m, const void* x,
                       const float* gamma, const float* beta, const void* residual, void* y,
                       uint8_t* relu_mask, float* save_mean, float* save_rstd, float* rm, float* rv,
                       float momentum, float* partial, hipStream_t s) {
  const size_t lds = 256 * 2 * Elem<T>::VEC * sizeof(float);
  RN50_LAUNCH("bn_stats", bn_stats_kernel<T>, dim3(g.nblk, g.gy), dim3(256), lds, s, static_cast<const T*>(x), m, d->C, g.tx_log2, g.rpb, partial);
  launch_fwd_tail<T>(d, g, m, x, gamma, beta, residual, y, relu_mask, save_mean, save_rstd, rm, rv, momentum,
                     partial, g.nblk, g.rpb, false, s);
}

// finalize + apply from partial sums rows [sum g, sum g*xhat]
template <typename T>
static void launch_bwd_tail(const rn50_bn_desc* d, const BnGeom& g, int64_t m, const void* dz,
                            const void* dz2, const void* x, const void* z, const uint8_t* zmask,
                            const float* gamma, const float* beta, const float* mean, const float* rstd,
                            void* dx, void* dres, float* dgamma, float* dbeta, const float* partial,
                            int nrows, bool row_major, hipStream_t s) {
  BnGeom ga = bn_apply_geom(m, d->C, d->dtype, kBnBwdApplyGroups);
  BnFinArgs fin{};
  if (row_major) {
    // few tile rows: the apply pass adds them up itself
    ga.tx_log2 = 3;
    bn_self_finalize_geom(m, d->C, ga.V, &ga.gy, &ga.rpb);
    ga.nblk = static_cast<int>(ceil_div(m, ga.rpb));
    fin = BnFinArgs{partial, nrows, 0, 0.f, 0.f, dbeta, dgamma, nullptr, nullptr};
  } else {
#ifdef RN50_TUNING
    static const bool skip_fin = getenv("RN50_SKIP_BN_FINALIZE") != nullptr;
    static const int skip_below = getenv("RN50_SKIP_BN_FINALIZE_ROWS") ? atoi(getenv("RN50_SKIP_BN_FINALIZE_ROWS")) : 1 << 30;
    if (!skip_fin || nrows > skip_below)
#endif
    RN50_LAUNCH("bn_bwd_finalize", bn_bwd_finalize_kernel, dim3(finalize_grid(d->C, nrows)), dim3(256), 0, s, partial, nrows, d->C, finalize_wpc(nrows), dgamma, dbeta);
  }
#define RN50_BWD_APPLY_K(DZ2, ZK, FIN)                                                                             \
  RN50_LAUNCH("bn_bwd_apply", (bn_bwd_apply_kernel<T, DZ2, ZK, FIN>), dim3(ga.nblk, ga.gy), dim3(256), 0, s,       \
              static_cast<const T*>(dz), static_cast<const T*>(dz2), static_cast<const T*>(x),                     \
              static_cast<const T*>(z), zmask, gamma, beta, mean, rstd, dgamma, dbeta, static_cast<T*>(dx),        \
              static_cast<T*>(dres), m, d->C, ga.tx_log2, ga.rpb, d->mode, fin)
#define RN50_BWD_APPLY(DZ2, ZK)                                                  \
  do {                                                                           \
    if (row_major) RN50_BWD_APPLY_K(DZ2, ZK, true); else RN50_BWD_APPLY_K(DZ2, ZK, false); \
  } while (0)
  const int zk = d->mode == 0 ? 0 : (zmask ? 2 : (z ? 1 : 0));
  if (dz2) {
    if (zk == 2) RN50_BWD_APPLY(true, 2); else if (zk == 1) RN50_BWD_APPLY(true, 1); else RN50_BWD_APPLY(true, 0);
  } else {
    if (zk == 2) RN50_BWD_APPLY(false, 2); else if (zk == 1) RN50_BWD_APPLY(false, 1); else RN50_BWD_APPLY(false, 0);
  }
#undef RN50_BWD_APPLY
#undef RN50_BWD_APPLY_K
}

template <typename T>
static void launch_bwd(const rn50_bn_desc* d, const BnGeom& g, int64_t m, const void* dz,
                       const void* dz2, const void* x, const void* z, const uint8_t* zmask,
                       const float* gamma, const float* beta, const float* mean, const float* rstd, void* dx,
                       void* dres, float* dgamma, float* dbeta, float* partial, hipStream_t s) {
  const size_t lds = 256 * 2 * Elem<T>::VEC * sizeof(float);
#define RN50_BWD_REDUCE(DZ2, ZK)                                                                                 \
  RN50_LAUNCH("bn_bwd_reduce", (bn_bwd_reduce_kernel<T, DZ2, ZK>), dim3(g.nblk, g.gy), dim3(256), lds, s,          \
              static_cast<const T*>(dz), static_cast<const T*>(dz2), static_cast<const T*>(x),                     \
              static_cast<const T*>(z), zmask, gamma, beta, mean, rstd, m, d->C, g.tx_log2, g.rpb, d->mode, partial)
  const int zk = d->mode == 0 ? 0 : (zmask ? 2 : (z ? 1 : 0));
  if (dz2) {
    if (zk == 2) RN50_BWD_REDUCE(true, 2); else if (zk == 1) RN50_BWD_REDUCE(true, 1); else RN50_BWD_REDUCE(true, 0);
  } else {
    if (zk == 2) RN50_BWD_REDUCE(false, 2); else if (zk == 1) RN50_BWD_REDUCE(false, 1); else RN50_BWD_REDUCE(false, 0);
  }
#undef RN50_BWD_REDUCE
  launch_bwd_tail<T>(d, g, m, dz, dz2, x, z, zmask, gamma, beta, mean, rstd, dx, dres, dgamma, dbeta, partial,
                     g.nblk, false, s);
}

// Entry points for the whole-step driver and the fused C-ABI calls: the sums come from the output stage
// of the convolution that produced x (forward) or dz (backward).
void bn_fwd_from_partials(const rn50_bn_desc* d, const void* x, const float* partial, int nrows, int rpp,
                          const float* gamma, const float* beta, const void* residual, void* y,
                          uint8_t* relu_mask, float* save_mean, float* save_rstd, float* rm, float* rv,
                          float momentum, hipStream_t s) {
  const int64_t m = static_cast<int64_t>(d->N) * d->H * d->W;
  const BnGeom g = bn_geom(m, d->C, d->dtype);
  if (d->dtype == RN50_BF16)
    launch_fwd_tail<uint16_t>(d, g, m, x, gamma, beta, residual, y, relu_mask, save_mean, save_rstd, rm, rv,
                              momentum, partial, nrows, rpp, bn_partials_row_major(nrows, false), s);
  else
    launch_fwd_tail<float>(d, g, m, x, gamma, beta, residual, y, relu_mask, save_mean, save_rstd, rm, rv, momentum,
                           partial, nrows, rpp, bn_partials_row_major(nrows, false), s);
}
// Evaluation mode: 1/sqrt(running_var + eps) per channel, then the training pass's apply kernel with the
// moving averages in place of the batch statistics.
__global__ __launch_bounds__(256) void bn_infer_rstd_kernel(const float* __restrict__ running_var, float eps, int C,
                                                            float* __restrict__ rstd) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c < C) rstd[c] = static_cast<float>(1.0 / sqrt(static_cast<double>(running_var[c]) + static_cast<double>(eps)));
}
void bn_infer_run(const rn50_bn_desc* d, const void* x, const float* gamma, const float* beta,
                  const float* running_mean, const float* running_var, const void* residual, void* y,
                  float* rstd_scratch, hipStream_t s) {
  const int64_t m = static_cast<int64_t>(d->N) * d->H * d->W;
  hipLaunchKernelGGL(bn_infer_rstd_kernel, dim3(static_cast<unsigned>(ceil_div(d->C, 256))), dim3(256), 0, s,
                     running_var, d->eps, d->C, rstd_scratch);
  const BnGeom ga = bn_apply_geom(m, d->C, d->dtype, kBnApplyGroups);
  if (d->dtype == RN50_BF16)
    RN50_LAUNCH("bn_apply", bn_apply_kernel<uint16_t>, dim3(ga.nblk, ga.gy), dim3(256), 0, s, static_cast<const uint16_t*>(x), gamma, beta, running_mean, rstd_scratch, static_cast<const uint16_t*>(residual), static_cast<uint16_t*>(y), static_cast<uint8_t*>(nullptr), m, d->C, ga.tx_log2, ga.rpb, d->mode, BnFinArgs{});
  else
    RN50_LAUNCH("bn_apply", bn_apply_kernel<float>, dim3(ga.nblk, ga.gy), dim3(256), 0, s, static_cast<const float*>(x), gamma, beta, running_mean, rstd_scratch, static_cast<const float*>(residual), static_cast<float*>(y), static_cast<uint8_t*>(nullptr), m, d->C, ga.tx_log2, ga.rpb, d->mode, BnFinArgs{});
}

void bn_bwd_from_partials(const rn50_bn_desc* d, const void* dz, const void* x, const uint8_t* relu_mask,
                          const float* gamma, const float* beta, const float* mean, const float* rstd,
                          const float* partial, int nrows, void* dx, void* dres, float* dgamma, float* dbeta,
                          hipStream_t s) {
  const int64_t m = static_cast<int64_t>(d->N) * d->H * d->W;
  const BnGeom g = bn_geom(m, d->C, d->dtype);
  if (d->dtype == RN50_BF16)
    launch_bwd_tail<uint16_t>(d, g, m, dz, nullptr, x, nullptr, relu_mask, gamma, beta, mean, rstd, dx, dres, dgamma,
                              dbeta, partial, nrows, bn_partials_row_major(nrows, true), s);
  else
    launch_bwd_tail<float>(d, g, m, dz, nullptr, x, nullptr, relu_mask, gamma, beta, mean, rstd, dx, dres, dgamma,
                           dbeta, partial, nrows, bn_partials_row_major(nrows, true), s);
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
                           const float* beta, const void* residual, void* y, uint8_t* relu_mask,
                           float* save_mean, float* save_rstd, float* running_mean, float* running_var,
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
    launch_fwd<uint16_t>(d, g, m, x, gamma, beta, residual, y, relu_mask, save_mean, save_rstd, running_mean,
                         running_var, momentum, static_cast<float*>(workspace), s);
  else
    launch_fwd<float>(d, g, m, x, gamma, beta, residual, y, relu_mask, save_mean, save_rstd, running_mean,
                      running_var, momentum, static_cast<float*>(workspace), s);
  return launch_status("bn_relu_fwd");
}

extern "C" int bn_relu_bwd(const rn50_bn_desc* d, const void* dz, const void* dz2, const void* x,
                           const void* z, const uint8_t* relu_mask, const float* gamma, const float* beta,
                           const float* save_mean, const float* save_rstd, void* dx,
                           void* dresidual, float* dgamma, float* dbeta, void* workspace,
                           size_t workspace_bytes, void* stream) {
  clear_error();
  if (int rc = check_desc(d, "bn_relu_bwd")) return rc;
  RN50_REQUIRE(dz && x && gamma && save_mean && save_rstd && dx && dgamma && dbeta && workspace,
               RN50_ERR_INVALID, "bn_relu_bwd: null pointer");
  RN50_REQUIRE(d->mode != 2 || z || relu_mask, RN50_ERR_INVALID, "bn_relu_bwd: mode 2 needs z or relu_mask");
  RN50_REQUIRE(d->mode != 1 || z || relu_mask || beta, RN50_ERR_INVALID,
               "bn_relu_bwd: mode 1 needs z, relu_mask, or beta to recompute the ReLU mask");
  RN50_REQUIRE(aligned16(dz) && aligned16(dz2) && aligned16(x) && aligned16(z) && aligned16(dx) &&
                   aligned16(dresidual) && aligned16(workspace) && aligned16(gamma) && aligned16(beta) &&
                   aligned16(save_mean) && aligned16(save_rstd) && aligned16(dgamma) && aligned16(dbeta),
               RN50_ERR_ALIGN, "bn_relu_bwd: pointer not 16-byte aligned");
  RN50_REQUIRE(workspace_bytes >= bn_ws_bytes(d), RN50_ERR_WORKSPACE,
               "bn_relu_bwd: workspace %zu < %zu bytes", workspace_bytes, bn_ws_bytes(d));
  const int64_t m = static_cast<int64_t>(d->N) * d->H * d->W;
  const BnGeom g = bn_geom(m, d->C, d->dtype);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (d->dtype == RN50_BF16)
    launch_bwd<uint16_t>(d, g, m, dz, dz2, x, z, relu_mask, gamma, beta, save_mean, save_rstd, dx, dresidual,
                         dgamma, dbeta, static_cast<float*>(workspace), s);
  else
    launch_bwd<float>(d, g, m, dz, dz2, x, z, relu_mask, gamma, beta, save_mean, save_rstd, dx, dresidual,
                      dgamma, dbeta, static_cast<float*>(workspace), s);
  return launch_status("bn_relu_bwd");
}

// ---- batch norm from sums fused into the producing convolution (conv_fwd_bn_sums / conv_dgrad_bn_sums)
extern "C" int bn_relu_fwd_from_sums(const rn50_bn_desc* d, const rn50_conv_desc* producer, const void* x,
                                     const float* sums, const float* gamma, const float* beta,
                                     const void* residual, void* y, uint8_t* relu_mask, float* save_mean,
                                     float* save_rstd, float* running_mean, float* running_var, float momentum,
                                     void* stream) {
  clear_error();
  if (int rc = check_desc(d, "bn_relu_fwd_from_sums")) return rc;
  RN50_REQUIRE(producer && conv_bn_sums_bytes(producer) > 0, RN50_ERR_INVALID,
               "bn_relu_fwd_from_sums: bad producer descriptor");
  RN50_REQUIRE(x && sums && gamma && beta && y && save_mean && save_rstd, RN50_ERR_INVALID,
               "bn_relu_fwd_from_sums: null pointer");
  RN50_REQUIRE((d->mode == 2) == (residual != nullptr), RN50_ERR_INVALID,
               "bn_relu_fwd_from_sums: residual must be given exactly in mode 2");
  RN50_REQUIRE(aligned16(x) && aligned16(y) && aligned16(residual) && aligned16(sums) && aligned16(gamma) &&
                   aligned16(beta) && aligned16(save_mean) && aligned16(save_rstd),
               RN50_ERR_ALIGN, "bn_relu_fwd_from_sums: pointer not 16-byte aligned");
  const int P = (producer->H + 2 * producer->pad - producer->R) / producer->stride + 1;
  const int Q = (producer->W + 2 * producer->pad - producer->S) / producer->stride + 1;
  RN50_REQUIRE(producer->N == d->N && P == d->H && Q == d->W && producer->Cout == d->C &&
                   producer->dtype == d->dtype,
               RN50_ERR_INVALID, "bn_relu_fwd_from_sums: the producer's output is not this layer's input");
  const PartialRows pr = fwd_partial_rows(producer);
  bn_fwd_from_partials(d, x, sums, pr.num, pr.rows, gamma, beta, residual, y, relu_mask, save_mean, save_rstd,
                       running_mean, running_var, momentum, static_cast<hipStream_t>(stream));
  return launch_status("bn_relu_fwd_from_sums");
}

extern "C" int bn_relu_bwd_from_sums(const rn50_bn_desc* d, const rn50_conv_desc* producer, const void* dz,
                                     const void* x, const uint8_t* relu_mask, const float* gamma,
                                     const float* beta, const float* save_mean, const float* save_rstd,
                                     const float* sums, void* dx, void* dresidual, float* dgamma, float* dbeta,
                                     void* stream) {
  clear_error();
  if (int rc = check_desc(d, "bn_relu_bwd_from_sums")) return rc;
  RN50_REQUIRE(d->mode == 1 || d->mode == 2, RN50_ERR_UNSUPPORTED, "bn_relu_bwd_from_sums: mode %d (needs a ReLU)",
               d->mode);
  RN50_REQUIRE(d->mode != 2 || relu_mask, RN50_ERR_INVALID, "bn_relu_bwd_from_sums: mode 2 needs relu_mask");
  RN50_REQUIRE(producer && conv_bn_sums_bytes(producer) > 0, RN50_ERR_INVALID,
               "bn_relu_bwd_from_sums: bad producer descriptor");
  RN50_REQUIRE(dz && x && gamma && beta && save_mean && save_rstd && sums && dx && dgamma && dbeta,
               RN50_ERR_INVALID, "bn_relu_bwd_from_sums: null pointer");
  RN50_REQUIRE(aligned16(dz) && aligned16(x) && aligned16(dx) && aligned16(sums) && aligned16(dresidual) &&
                   aligned16(gamma) && aligned16(beta) && aligned16(save_mean) && aligned16(save_rstd) &&
                   aligned16(dgamma) && aligned16(dbeta),
               RN50_ERR_ALIGN, "bn_relu_bwd_from_sums: pointer not 16-byte aligned");
  RN50_REQUIRE(producer->N == d->N && producer->H == d->H && producer->W == d->W && producer->Cin == d->C &&
                   producer->dtype == d->dtype,
               RN50_ERR_INVALID, "bn_relu_bwd_from_sums: the producer's input is not this layer's output");
  const PartialRows pr = dgrad_partial_rows(producer);
  bn_bwd_from_partials(d, dz, x, relu_mask, gamma, beta, save_mean, save_rstd, sums, pr.num, dx,
                       d->mode == 2 ? dresidual : nullptr, dgamma, dbeta, static_cast<hipStream_t>(stream));
  return launch_status("bn_relu_bwd_from_sums");
}

extern "C" size_t bn_relu_infer_workspace_bytes(const rn50_bn_desc* d) {
  if (!d || d->C <= 0) return 0;
  return align_up(static_cast<size_t>(d->C) * sizeof(float), 256);
}

extern "C" int bn_relu_infer(const rn50_bn_desc* d, const void* x, const float* gamma, const float* beta,
                             const float* running_mean, const float* running_var, const void* residual, void* y,
                             void* workspace, size_t workspace_bytes, void* stream) {
  clear_error();
  if (int rc = check_desc(d, "bn_relu_infer")) return rc;
  RN50_REQUIRE(x && gamma && beta && running_mean && running_var && y && workspace, RN50_ERR_INVALID,
               "bn_relu_infer: null pointer");
  RN50_REQUIRE((d->mode == 2) == (residual != nullptr), RN50_ERR_INVALID,
               "bn_relu_infer: residual must be given exactly in mode 2");
  RN50_REQUIRE(aligned16(x) && aligned16(y) && aligned16(residual) && aligned16(workspace) && aligned16(gamma) &&
                   aligned16(beta) && aligned16(running_mean) && aligned16(running_var),
               RN50_ERR_ALIGN, "bn_relu_infer: pointer not 16-byte aligned");
  RN50_REQUIRE(workspace_bytes >= bn_relu_infer_workspace_bytes(d), RN50_ERR_WORKSPACE,
               "bn_relu_infer: workspace %zu < %zu bytes", workspace_bytes, bn_relu_infer_workspace_bytes(d));
  bn_infer_run(d, x, gamma, beta, running_mean, running_var, residual, y, static_cast<float*>(workspace),
               static_cast<hipStream_t>(stream));
  return launch_status("bn_relu_infer");
}
