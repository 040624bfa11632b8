// Pooling, classifier and loss kernels: max-pool 3x3/2 (appendix log of the
// paper: 112 -> 56 after the stem), global average pool, the fully connected
// classifier, and softmax cross-entropy with label smoothing (Sec. III-A2).
// All are bandwidth- or latency-bound and small next to the convolutions.
#include "common.h"
#include "step_internal.h"

namespace rn50 {

// ------------------------------------------------------------------ max pool
template <typename T>
__global__ __launch_bounds__(256) void maxpool_fwd_kernel(const T* __restrict__ x,
                                                          T* __restrict__ y,
                                                          uint8_t* __restrict__ argmax, int N,
                                                          int H, int W, int C, int P, int Q, FastDiv div_cv) {
  // grid: (vectors of one output row, output rows, images) -- no index arithmetic beyond one division
  constexpr int V = Elem<T>::VEC;
  const int cv = C / V;
  const int xi = blockIdx.x * 256 + threadIdx.x;
  if (xi >= Q * cv) return;
  const int q = static_cast<int>(fdiv(static_cast<uint32_t>(xi), div_cv)), c = xi - q * cv;
  const int p = blockIdx.y, n = blockIdx.z;
  const int64_t i = (static_cast<int64_t>(n) * P + p) * Q * cv + xi;
  float best[V];
  int at[V];  // window position r*3+s of the first maximum
  bool have = false;
  for (int r = 0; r < 3; ++r) {
    const int ih = p * 2 - 1 + r;
    if (ih < 0 || ih >= H) continue;
    for (int s = 0; s < 3; ++s) {
      const int iw = q * 2 - 1 + s;
      if (iw < 0 || iw >= W) continue;
      float f[V];
      Elem<T>::unpack(load16(x + ((static_cast<int64_t>(n) * H + ih) * W + iw) * C + c * V), f);
      if (!have) {
#pragma unroll
        for (int j = 0; j < V; ++j) {
          best[j] = f[j];
          at[j] = r * 3 + s;
        }
        have = true;
      } else {
#pragma unroll
        for (int j = 0; j < V; ++j)
          if (f[j] > best[j]) {
            best[j] = f[j];
            at[j] = r * 3 + s;
          }
      }
    }
  }
  Vec16 o;
  Elem<T>::pack(best, o);
  store16(y + i * V, o);
  if (argmax) {
    uint32_t w0 = 0, w1 = 0;
#pragma unroll
    for (int j = 0; j < V; ++j) {
      if (j < 4) w0 |= static_cast<uint32_t>(at[j]) << (8 * j);
      else w1 |= static_cast<uint32_t>(at[j]) << (8 * (j - 4));
    }
    if (V == 8) *reinterpret_cast<uint2*>(argmax + i * V) = make_uint2(w0, w1);
    else *reinterpret_cast<uint32_t*>(argmax + i * V) = w0;
  }
}

// Backward from the stored window positions: one thread per 2x2 block of input pixel vectors
// (rows 2a, 2a+1; columns 2b, 2b+1).  The block lies in exactly the four windows (a..a+1, b..b+1), each
// of which is loaded once and dealt to the pixel its recorded position names: pixel (2a,2b) can only be
// the centre of window (a,b); (2a,2b+1) position 5 of (a,b) or 3 of (a,b+1); (2a+1,2b) position 7 of
// (a,b) or 1 of (a+1,b); (2a+1,2b+1) position 8, 6, 2, 0 of the four.  The summands of a pixel are
// added in window order (p, then q).
template <typename T>
__global__ __launch_bounds__(256) void maxpool_bwd_idx_kernel(const uint8_t* __restrict__ argmax,
                                                              const T* __restrict__ dy,
                                                              const T* __restrict__ dy2,
                                                              T* __restrict__ dx, int N, int H, int W,
                                                              int C, int P, int Q, FastDiv div_cv) {
  // grid: (vectors of one row of 2x2 pixel blocks, rows of blocks, images)
  constexpr int V = Elem<T>::VEC;
  const int cv = C / V;
  const int Wb = (W + 1) / 2;
  const int xi = blockIdx.x * 256 + threadIdx.x;
  if (xi >= Wb * cv) return;
  const int b = static_cast<int>(fdiv(static_cast<uint32_t>(xi), div_cv)), c = xi - b * cv;
  const int a = blockIdx.y, n = blockIdx.z;
  float acc[2][2][V];
#pragma unroll
  for (int k = 0; k < 4; ++k)
#pragma unroll
    for (int j = 0; j < V; ++j) acc[k >> 1][k & 1][j] = 0.f;
#pragma unroll
  for (int dp = 0; dp < 2; ++dp)
#pragma unroll
    for (int dq = 0; dq < 2; ++dq) {
      const int p = a + dp, q = b + dq;
      if (p >= P || q >= Q) continue;
      const int64_t o = ((static_cast<int64_t>(n) * P + p) * Q + q) * C + c * V;
      uint8_t idx[V];
      if (V == 8) *reinterpret_cast<uint2*>(idx) = *reinterpret_cast<const uint2*>(argmax + o);
      else *reinterpret_cast<uint32_t*>(idx) = *reinterpret_cast<const uint32_t*>(argmax + o);
      float g[V];
      Elem<T>::unpack(load16(dy + o), g);
      if (dy2) {
        float g2[V];
        Elem<T>::unpack(load16(dy2 + o), g2);
#pragma unroll
        for (int j = 0; j < V; ++j) g[j] += g2[j];
      }
      // pixel (2a+i, 2b+jj) sits at window position (2a+i - (2p-1))*3 + (2b+jj - (2q-1))
#pragma unroll
      for (int ii = dp; ii < 2; ++ii)      // window row a+1 starts at pixel row 2a+1
#pragma unroll
        for (int jj = dq; jj < 2; ++jj) {
          const int pos = (ii + 1 - 2 * dp) * 3 + (jj + 1 - 2 * dq);
#pragma unroll
          for (int j = 0; j < V; ++j) acc[ii][jj][j] += idx[j] == pos ? g[j] : 0.f;
        }
    }
#pragma unroll
  for (int ii = 0; ii < 2; ++ii)
#pragma unroll
    for (int jj = 0; jj < 2; ++jj) {
      const int h = 2 * a + ii, w = 2 * b + jj;
      if (h < H && w < W) {
        Vec16 ov;
        Elem<T>::pack(acc[ii][jj], ov);
        store16(dx + ((static_cast<int64_t>(n) * H + h) * W + w) * C + c * V, ov);
      }
    }
}

// One thread per input pixel vector.  The pixel receives dy of window (p,q) iff
// it is that window's first maximum in row-major order: strictly greater than
// every earlier tap and not less than every later one.
template <typename T>
__global__ __launch_bounds__(256) void maxpool_bwd_kernel(const T* __restrict__ x,
                                                          const T* __restrict__ dy,
                                                          const T* __restrict__ dy2,
                                                          T* __restrict__ dx, int N, int H, int W,
                                                          int C, int P, int Q) {
  constexpr int V = Elem<T>::VEC;
  const int cv = C / V;
  const int64_t total = static_cast<int64_t>(N) * H * W * cv;
  const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (i >= total) return;
  const int c = static_cast<int>(i % cv);
  int64_t t = i / cv;
  const int w = static_cast<int>(t % W); t /= W;
  const int h = static_cast<int>(t % H);
  const int n = static_cast<int>(t / H);
  float mine[V], acc[V];
  Elem<T>::unpack(load16(x + i * V), mine);
#pragma unroll
  for (int j = 0; j < V; ++j) acc[j] = 0.f;
  // windows containing (h,w): p*2-1 <= h <= p*2+1
  const int p_lo = max((h - 1 + 1) / 2, 0), p_hi = min((h + 1) / 2, P - 1);
  const int q_lo = max((w - 1 + 1) / 2, 0), q_hi = min((w + 1) / 2, Q - 1);
  for (int p = p_lo; p <= p_hi; ++p)
    for (int q = q_lo; q <= q_hi; ++q) {
      const int my_r = h - (p * 2 - 1), my_s = w - (q * 2 - 1);
      const int my_pos = my_r * 3 + my_s;
      bool win[V];
#pragma unroll
      for (int j = 0; j < V; ++j) win[j] = true;
      for (int r = 0; r < 3; ++r) {
        const int ih = p * 2 - 1 + r;
        if (ih < 0 || ih >= H) continue;
        for (int s = 0; s < 3; ++s) {
          const int iw = q * 2 - 1 + s;
          if (iw < 0 || iw >= W) continue;
          const int pos = r * 3 + s;
          if (pos == my_pos) continue;
          float f[V];
          Elem<T>::unpack(load16(x + ((static_cast<int64_t>(n) * H + ih) * W + iw) * C + c * V), f);
          if (pos < my_pos) {
#pragma unroll
            for (int j = 0; j < V; ++j) win[j] = win[j] && (mine[j] > f[j]);
          } else {
#pragma unroll
            for (int j = 0; j < V; ++j) win[j] = win[j] && (mine[j] >= f[j]);
          }
        }
      }
      const int64_t o = ((static_cast<int64_t>(n) * P + p) * Q + q) * C + c * V;
      float g[V];
      Elem<T>::unpack(load16(dy + o), g);
      if (dy2) {
        float g2[V];
        Elem<T>::unpack(load16(dy2 + o), g2);
#pragma unroll
        for (int j = 0; j < V; ++j) g[j] += g2[j];
      }
#pragma unroll
      for (int j = 0; j < V; ++j) acc[j] += win[j] ? g[j] : 0.f;
    }
  Vec16 o;
  Elem<T>::pack(acc, o);
  store16(dx + i * V, o);
}

// -------------------------------------------------------------- average pool
template <typename T>
__global__ __launch_bounds__(64) void avgpool_fwd_kernel(const T* __restrict__ x,
                                                         T* __restrict__ y, int N, int HW, int C) {
  constexpr int V = Elem<T>::VEC;
  const int cv = C / V;
  const int i = blockIdx.x * 64 + threadIdx.x;
  if (i >= N * cv) return;
  const int n = i / cv, c = i % cv;
  float acc[V];
#pragma unroll
  for (int j = 0; j < V; ++j) acc[j] = 0.f;
  const T* p = x + static_cast<int64_t>(n) * HW * C + c * V;
  // the rows are requested sixteen at a time (a thread's loads are what this kernel waits for) and added in
  // row order
  constexpr int U = 16;
  int r = 0;
  for (; r + U <= HW; r += U) {
    Vec16 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = load16(p + static_cast<int64_t>(r + u) * C);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float f[V];
      Elem<T>::unpack(v[u], f);
#pragma unroll
      for (int j = 0; j < V; ++j) acc[j] += f[j];
    }
  }
  for (; r < HW; ++r) {
    float f[V];
    Elem<T>::unpack(load16(p + static_cast<int64_t>(r) * C), f);
#pragma unroll
    for (int j = 0; j < V; ++j) acc[j] += f[j];
  }
  const float inv = 1.0f / static_cast<float>(HW);
#pragma unroll
  for (int j = 0; j < V; ++j) acc[j] *= inv;
  Vec16 o;
  Elem<T>::pack(acc, o);
  store16(y + static_cast<int64_t>(i) * V, o);
}

template <typename T>
__global__ __launch_bounds__(256) void avgpool_bwd_kernel(const T* __restrict__ dy,
                                                          T* __restrict__ dx, int N, int HW,
                                                          int C) {
  constexpr int V = Elem<T>::VEC;
  const int cv = C / V;
  const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (i >= static_cast<int64_t>(N) * HW * cv) return;
  const int c = static_cast<int>(i % cv);
  const int n = static_cast<int>(i / (static_cast<int64_t>(HW) * cv));
  float f[V];
  Elem<T>::unpack(load16(dy + (static_cast<int64_t>(n) * cv + c) * V), f);
  const float inv = 1.0f / static_cast<float>(HW);
#pragma unroll
  for (int j = 0; j < V; ++j) f[j] *= inv;
  Vec16 o;
  Elem<T>::pack(f, o);
  store16(dx + i * V, o);
}

// ---------------------------------------------------- small strided GEMM (FC)
// C[i,j] = sum_k A(i,k)*B(k,j) (+ bias[j]); A(i,k) = a[i*as_i + k*as_k], same for B.
// 64x64 tile per workgroup, 16-deep LDS stages, 4x4 outputs per thread, float
// accumulation.  The classifier is ~0.05% of the step's arithmetic.
template <typename TA, typename TB, typename TC>
__global__ __launch_bounds__(256) void small_gemm_kernel(const TA* __restrict__ a, int64_t as_i,
                                                         int64_t as_k, const TB* __restrict__ b,
                                                         int64_t bs_k, int64_t bs_j,
                                                         const float* __restrict__ bias,
                                                         TC* __restrict__ c, int M, int Nn, int K) {
  __shared__ float As[16][65];
  __shared__ float Bs[16][65];
  const int i0 = blockIdx.y * 64, j0 = blockIdx.x * 64;
  const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
  float acc[4][4];
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int v = 0; v < 4; ++v) acc[u][v] = 0.f;
  for (int k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int idx = threadIdx.x + e * 256;  // 0..1023
      {
        // A tile: choose the faster-varying index to follow the smaller stride
        const int kk = as_k == 1 ? (idx & 15) : (idx >> 6);
        const int ii = as_k == 1 ? (idx >> 4) : (idx & 63);
        const int gi = i0 + ii, gk = k0 + kk;
        As[kk][ii] = (gi < M && gk < K) ? Elem<TA>::load(a + gi * as_i + gk * as_k) : 0.f;
      }
      {
        const int kk = bs_k == 1 ? (idx & 15) : (idx >> 6);
        const int jj = bs_k == 1 ? (idx >> 4) : (idx & 63);
        const int gj = j0 + jj, gk = k0 + kk;
        Bs[kk][jj] = (gj < Nn && gk < K) ? Elem<TB>::load(b + gk * bs_k + gj * bs_j) : 0.f;
      }
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float av[4], bv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) av[u] = As[kk][ty * 4 + u];
#pragma unroll
      for (int v = 0; v < 4; ++v) bv[v] = Bs[kk][tx * 4 + v];
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[u][v] = fmaf(av[u], bv[v], acc[u][v]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int gi = i0 + ty * 4 + u, gj = j0 + tx * 4 + v;
      if (gi < M && gj < Nn)
        Elem<TC>::store(c + static_cast<int64_t>(gi) * Nn + gj, acc[u][v] + (bias ? bias[gj] : 0.f));
    }
}

// logits[n][k] = sum_c a[n][c]*W[k][c] + b[k]: one wave per class k.  The wave streams its weight row
// once per block of 8 batch rows (the activations, N*Cin elements, stay in cache), accumulates in
// float and finishes each dot product with a wave reduction.
__device__ __forceinline__ f32x16 mfma_bf16_32x32x16(const Vec16& a, const Vec16& b, f32x16 acc) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8*>(&a),
                                                 *reinterpret_cast<const bf16x8*>(&b), acc, 0, 0, 0);
}

// Matrix-core form for bf16 and a batch of at most 64 rows: a workgroup owns 32 classes; its four waves
// split the input channels (wave w takes channels 16*(w + 4i)..+15), each multiplying the [32 classes x
// 16] weight fragment with the [16 x 32 rows] activation fragments read straight from memory
// (v_mfma_f32_32x32x16_bf16: lane l supplies row l%32, k = 8*(l/32)..+7 of both operands).  The waves'
// partial tiles are added through LDS in wave order.  Every workgroup reads the activations once.
__global__ __launch_bounds__(256) void fc_fwd_mfma_kernel(const uint16_t* __restrict__ a,
                                                          const uint16_t* __restrict__ W,
                                                          const float* __restrict__ b,
                                                          float* __restrict__ logits, int N, int Cin, int K) {
  __shared__ float red[4][2][32 * 32];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int k0 = blockIdx.x * 32;
  const int krow = min(k0 + (lane & 31), K - 1);
  const int n_lo = min(lane & 31, N - 1), n_hi = min(32 + (lane & 31), N - 1);
  const bool hi_ok = 32 + (lane & 31) < N, lo_ok = (lane & 31) < N;
  const uint16_t* wp = W + static_cast<int64_t>(krow) * Cin + 8 * (lane >> 5);
  const uint16_t* ap0 = a + static_cast<int64_t>(n_lo) * Cin + 8 * (lane >> 5);
  const uint16_t* ap1 = a + static_cast<int64_t>(n_hi) * Cin + 8 * (lane >> 5);
  f32x16 acc0, acc1;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc0[v] = acc1[v] = 0.f;
  constexpr int U = 8;  // loads in flight per operand: the kernel runs at the latency of its batches of loads
  int c = wave * 16;
  for (; c + (U - 1) * 64 < Cin; c += U * 64) {
    Vec16 fw[U], f0[U], f1[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      fw[u] = load16(wp + c + u * 64);
      f0[u] = load16(ap0 + c + u * 64);
      f1[u] = load16(ap1 + c + u * 64);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (!lo_ok) f0[u].u = make_uint4(0, 0, 0, 0);
      if (!hi_ok) f1[u].u = make_uint4(0, 0, 0, 0);
      acc0 = mfma_bf16_32x32x16(fw[u], f0[u], acc0);
      acc1 = mfma_bf16_32x32x16(fw[u], f1[u], acc1);
    }
  }
  for (; c < Cin; c += 64) {
    Vec16 fw = load16(wp + c), f0 = load16(ap0 + c), f1 = load16(ap1 + c);
    if (!lo_ok) f0.u = make_uint4(0, 0, 0, 0);
    if (!hi_ok) f1.u = make_uint4(0, 0, 0, 0);
    acc0 = mfma_bf16_32x32x16(fw, f0, acc0);
    acc1 = mfma_bf16_32x32x16(fw, f1, acc1);
  }
  // D[class][row]: class = (v/4)*8 + (lane/32)*4 + v%4, row = lane%32
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int cls = (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
    red[wave][0][cls * 32 + (lane & 31)] = acc0[v];
    red[wave][1][cls * 32 + (lane & 31)] = acc1[v];
  }
  __syncthreads();
  for (int i = threadIdx.x; i < 2 * 32 * 32; i += 256) {
    const int t = i >> 10, cls = (i >> 5) & 31, row = t * 32 + (i & 31);
    const int k = k0 + cls;
    if (k < K && row < N) {
      const int j = cls * 32 + (i & 31);
      logits[static_cast<int64_t>(row) * K + k] = ((red[0][t][j] + red[1][t][j]) + red[2][t][j]) + red[3][t][j] + b[k];
    }
  }
}

template <typename T>
__global__ __launch_bounds__(256) void fc_fwd_kernel(const T* __restrict__ a, const T* __restrict__ W,
                                                     const float* __restrict__ b,
                                                     float* __restrict__ logits, int N, int Cin, int K) {
  constexpr int V = Elem<T>::VEC;
  const int k = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (k >= K) return;
  const int lane = threadIdx.x & 63;
  const T* wrow = W + static_cast<int64_t>(k) * Cin;
  const float bias = b[k];
  for (int n0 = 0; n0 < N; n0 += 8) {
    float acc[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) acc[u] = 0.f;
    for (int c = lane * V; c < Cin; c += 64 * V) {
      float wv[V];
      if (c + V <= Cin) {
        Elem<T>::unpack(load16(wrow + c), wv);
      } else {
#pragma unroll
        for (int j = 0; j < V; ++j) wv[j] = c + j < Cin ? Elem<T>::load(wrow + c + j) : 0.f;
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if (n0 + u < N) {
          const T* arow = a + static_cast<int64_t>(n0 + u) * Cin + c;
          float av[V];
          if (c + V <= Cin) {
            Elem<T>::unpack(load16(arow), av);
          } else {
#pragma unroll
            for (int j = 0; j < V; ++j) av[j] = c + j < Cin ? Elem<T>::load(arow + j) : 0.f;
          }
#pragma unroll
          for (int j = 0; j < V; ++j) acc[u] = fmaf(av[j], wv[j], acc[u]);
        }
      }
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const float sum = wave_sum(acc[u]);
      if (lane == 0 && n0 + u < N) logits[static_cast<int64_t>(n0 + u) * K + k] = sum + bias;
    }
  }
}

template <typename T>
__global__ __launch_bounds__(256) void cast_from_float_kernel(const float* __restrict__ in, T* __restrict__ out, int64_t n) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (i < n) Elem<T>::store(out + i, in[i]);
}

// db[k] = sum_n dlogits[n,k]
__global__ __launch_bounds__(256) void colsum_kernel(const float* __restrict__ dl, float* __restrict__ db,
                                                     int N, int K) {
  const int k = blockIdx.x * 256 + threadIdx.x;
  if (k >= K) return;
  float s = 0.f;
  for (int n = 0; n < N; ++n) s += dl[static_cast<int64_t>(n) * K + k];
  db[k] = s;
}

template <typename TA, typename TB, typename TC>
static void small_gemm(const TA* a, int64_t as_i, int64_t as_k, const TB* b, int64_t bs_k,
                       int64_t bs_j, const float* bias, TC* c, int M, int Nn, int K, hipStream_t s) {
  RN50_LAUNCH("fc_gemm", (small_gemm_kernel<TA, TB, TC>), dim3(ceil_div(Nn, 64), ceil_div(M, 64)),
                     dim3(256), 0, s, a, as_i, as_k, b, bs_k, bs_j, bias, c, M, Nn, K);
}

// ------------------------------------------------------ softmax cross-entropy
// One workgroup per row.
__global__ __launch_bounds__(256) void xent_rows_kernel(const float* __restrict__ logits,
                                                        const int32_t* __restrict__ labels, int N,
                                                        int K, float ls, float grad_scale,
                                                        float* __restrict__ row_loss,
                                                        float* __restrict__ dlogits) {
  __shared__ float red[8];
  const int n = blockIdx.x;
  const float* l = logits + static_cast<int64_t>(n) * K;
  float mx = -INFINITY;
  for (int k = threadIdx.x; k < K; k += 256) mx = fmaxf(mx, l[k]);
  mx = wave_max(mx);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  float se = 0.f, sl = 0.f;  // sum exp(l-mx), sum (l-mx)
  for (int k = threadIdx.x; k < K; k += 256) {
    const float d = l[k] - mx;
    se += expf(d);
    sl += d;
  }
  se = block256_sum(se, red);
  sl = block256_sum(sl, red + 4);
  const float lse = logf(se);  // log-sum-exp relative to mx
  const int label = labels[n];
  const float qoff = ls / static_cast<float>(K), qon = 1.0f - ls;
  const float coef = grad_scale / static_cast<float>(N);
  for (int k = threadIdx.x; k < K; k += 256) {
    const float logp = l[k] - mx - lse;
    const float q = qoff + (k == label ? qon : 0.f);
    dlogits[static_cast<int64_t>(n) * K + k] = coef * (expf(logp) - q);
  }
  if (threadIdx.x == 0) {
    // -sum_k q_k logp_k = -(ls/K) * sum_k logp_k - (1-ls) * logp_label
    const float sum_logp = sl - static_cast<float>(K) * lse;
    float rl = -qoff * sum_logp;
    if (label >= 0 && label < K) rl -= qon * (l[label] - mx - lse);
    row_loss[n] = rl;
  }
}

__global__ __launch_bounds__(256) void mean_kernel(const float* __restrict__ v, int n,
                                                   float* __restrict__ out) {
  __shared__ float red[4];
  float s = 0.f;
  for (int i = threadIdx.x; i < n; i += 256) s += v[i];
  s = block256_sum(s, red);
  if (threadIdx.x == 0) out[0] = s / static_cast<float>(n);
}

static int check_dtype(int dtype, const char* who) {
  RN50_REQUIRE(dtype == RN50_F32 || dtype == RN50_BF16, RN50_ERR_INVALID, "%s: dtype %d", who, dtype);
  return RN50_OK;
}

}  // namespace rn50

using namespace rn50;

#define DISPATCH_T(dtype, ...)             \
  do {                                     \
    if ((dtype) == RN50_BF16) {            \
      typedef uint16_t T;                  \
      __VA_ARGS__;                         \
    } else {                               \
      typedef float T;                     \
      __VA_ARGS__;                         \
    }                                      \
  } while (0)

extern "C" int maxpool_fwd(int N, int H, int W, int C, int dtype, const void* x, void* y,
                           uint8_t* argmax, void* stream) {
  clear_error();
  if (int rc = check_dtype(dtype, "maxpool_fwd")) return rc;
  RN50_REQUIRE(N > 0 && H > 0 && W > 0 && C > 0, RN50_ERR_INVALID, "maxpool_fwd: non-positive size");
  RN50_REQUIRE(N <= 65535 && H <= 131070, RN50_ERR_UNSUPPORTED, "maxpool_fwd: N=%d or H=%d beyond the launch grid", N, H);
  RN50_REQUIRE(x && y, RN50_ERR_INVALID, "maxpool_fwd: null pointer");
  RN50_REQUIRE(C % (dtype == RN50_BF16 ? 8 : 4) == 0, RN50_ERR_UNSUPPORTED, "maxpool_fwd: C=%d", C);
  RN50_REQUIRE(aligned16(x) && aligned16(y), RN50_ERR_ALIGN, "maxpool_fwd: pointer not 16-byte aligned");
  const int P = (H + 2 - 3) / 2 + 1, Q = (W + 2 - 3) / 2 + 1;
  hipStream_t s = static_cast<hipStream_t>(stream);
  DISPATCH_T(dtype, {
    const int cv = C / Elem<T>::VEC;
    RN50_LAUNCH("maxpool_fwd", maxpool_fwd_kernel<T>, dim3(ceil_div(Q * cv, 256), P, N), dim3(256), 0, s,
                       static_cast<const T*>(x), static_cast<T*>(y), argmax, N, H, W, C, P, Q, make_fastdiv(cv));
  });
  return launch_status("maxpool_fwd");
}

extern "C" int maxpool_bwd(int N, int H, int W, int C, int dtype, const void* x,
                           const uint8_t* argmax, const void* dy, const void* dy2, void* dx,
                           void* stream) {
  clear_error();
  if (int rc = check_dtype(dtype, "maxpool_bwd")) return rc;
  RN50_REQUIRE(N > 0 && H > 0 && W > 0 && C > 0, RN50_ERR_INVALID, "maxpool_bwd: non-positive size");
  RN50_REQUIRE(N <= 65535 && H <= 131070, RN50_ERR_UNSUPPORTED, "maxpool_bwd: N=%d or H=%d beyond the launch grid", N, H);
  RN50_REQUIRE((x || argmax) && dy && dx, RN50_ERR_INVALID, "maxpool_bwd: null pointer");
  RN50_REQUIRE(C % (dtype == RN50_BF16 ? 8 : 4) == 0, RN50_ERR_UNSUPPORTED, "maxpool_bwd: C=%d", C);
  RN50_REQUIRE(aligned16(x) && aligned16(dy) && aligned16(dy2) && aligned16(dx) && aligned16(argmax),
               RN50_ERR_ALIGN, "maxpool_bwd: pointer not 16-byte aligned");
  const int P = (H + 2 - 3) / 2 + 1, Q = (W + 2 - 3) / 2 + 1;
  hipStream_t s = static_cast<hipStream_t>(stream);
  DISPATCH_T(dtype, {
    const int64_t total = static_cast<int64_t>(N) * H * W * (C / Elem<T>::VEC);
    if (argmax)
      RN50_LAUNCH("maxpool_bwd", maxpool_bwd_idx_kernel<T>, dim3(ceil_div(((W + 1) / 2) * (C / Elem<T>::VEC), 256), (H + 1) / 2, N),
                         dim3(256), 0, s, argmax, static_cast<const T*>(dy), static_cast<const T*>(dy2),
                         static_cast<T*>(dx), N, H, W, C, P, Q, make_fastdiv(C / Elem<T>::VEC));
    else
      RN50_LAUNCH("maxpool_bwd", maxpool_bwd_kernel<T>, dim3(ceil_div(total, 256)), dim3(256), 0, s,
                         static_cast<const T*>(x), static_cast<const T*>(dy),
                         static_cast<const T*>(dy2), static_cast<T*>(dx), N, H, W, C, P, Q);
  });
  return launch_status("maxpool_bwd");
}

extern "C" int avgpool_fwd(int N, int HW, int C, int dtype, const void* x, void* y, void* stream) {
  clear_error();
  if (int rc = check_dtype(dtype, "avgpool_fwd")) return rc;
  RN50_REQUIRE(N > 0 && HW > 0 && C > 0, RN50_ERR_INVALID, "avgpool_fwd: non-positive size");
  RN50_REQUIRE(x && y, RN50_ERR_INVALID, "avgpool_fwd: null pointer");
  RN50_REQUIRE(C % (dtype == RN50_BF16 ? 8 : 4) == 0, RN50_ERR_UNSUPPORTED, "avgpool_fwd: C=%d", C);
  RN50_REQUIRE(aligned16(x) && aligned16(y), RN50_ERR_ALIGN, "avgpool_fwd: pointer not 16-byte aligned");
  hipStream_t s = static_cast<hipStream_t>(stream);
  DISPATCH_T(dtype, {
    const int total = N * (C / Elem<T>::VEC);
    RN50_LAUNCH("avgpool_fwd", avgpool_fwd_kernel<T>, dim3(ceil_div(total, 64)), dim3(64), 0, s,
                       static_cast<const T*>(x), static_cast<T*>(y), N, HW, C);
  });
  return launch_status("avgpool_fwd");
}

extern "C" int avgpool_bwd(int N, int HW, int C, int dtype, const void* dy, void* dx, void* stream) {
  clear_error();
  if (int rc = check_dtype(dtype, "avgpool_bwd")) return rc;
  RN50_REQUIRE(N > 0 && HW > 0 && C > 0, RN50_ERR_INVALID, "avgpool_bwd: non-positive size");
  RN50_REQUIRE(dy && dx, RN50_ERR_INVALID, "avgpool_bwd: null pointer");
  RN50_REQUIRE(C % (dtype == RN50_BF16 ? 8 : 4) == 0, RN50_ERR_UNSUPPORTED, "avgpool_bwd: C=%d", C);
  RN50_REQUIRE(aligned16(dy) && aligned16(dx), RN50_ERR_ALIGN, "avgpool_bwd: pointer not 16-byte aligned");
  hipStream_t s = static_cast<hipStream_t>(stream);
  DISPATCH_T(dtype, {
    const int64_t total = static_cast<int64_t>(N) * HW * (C / Elem<T>::VEC);
    RN50_LAUNCH("avgpool_bwd", avgpool_bwd_kernel<T>, dim3(ceil_div(total, 256)), dim3(256), 0, s,
                       static_cast<const T*>(dy), static_cast<T*>(dx), N, HW, C);
  });
  return launch_status("avgpool_bwd");
}

extern "C" int fc_fwd(int N, int Cin, int K, int dtype, const void* a, const void* W,
                      const float* b, float* logits, void* stream) {
  clear_error();
  if (int rc = check_dtype(dtype, "fc_fwd")) return rc;
  RN50_REQUIRE(N > 0 && Cin > 0 && K > 0, RN50_ERR_INVALID, "fc_fwd: non-positive size");
  RN50_REQUIRE(a && W && b && logits, RN50_ERR_INVALID, "fc_fwd: null pointer");
  RN50_REQUIRE(Cin % (dtype == RN50_BF16 ? 8 : 4) == 0, RN50_ERR_UNSUPPORTED, "fc_fwd: Cin=%d", Cin);
  RN50_REQUIRE(aligned16(a) && aligned16(W), RN50_ERR_ALIGN, "fc_fwd: pointer not 16-byte aligned");
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (dtype == RN50_BF16 && N <= 64 && Cin % 16 == 0) {
    RN50_LAUNCH("fc_fwd", fc_fwd_mfma_kernel, dim3(ceil_div(K, 32)), dim3(256), 0, s, static_cast<const uint16_t*>(a),
                static_cast<const uint16_t*>(W), b, logits, N, Cin, K);
    return launch_status("fc_fwd");
  }
  DISPATCH_T(dtype, {
    RN50_LAUNCH("fc_fwd", fc_fwd_kernel<T>, dim3(ceil_div(K, 4)), dim3(256), 0, s, static_cast<const T*>(a),
                       static_cast<const T*>(W), b, logits, N, Cin, K);
  });
  return launch_status("fc_fwd");
}

// The data gradient runs on the matrix cores when the shapes allow it (Cin and K multiples of the
// 16-byte vector): da = dl x W as a 1x1 "convolution" over N pixels with K input channels, reading
// dl in the storage type and W transposed to [Cin][K].
static bool fc_mfma_ok(int Cin, int K, int dtype) {
  const int V = dtype == RN50_BF16 ? 8 : 4;
  return Cin % V == 0 && K % V == 0;
}
static rn50_conv_desc fc_dgrad_desc(int N, int Cin, int K, int dtype) {
  return rn50_conv_desc{N, 1, 1, K, Cin, 1, 1, 1, 0, dtype};  // "input channels" K -> "output channels" Cin
}

extern "C" size_t fc_bwd_workspace_bytes(int N, int Cin, int K, int dtype) {
  if (N <= 0 || Cin <= 0 || K <= 0 || !fc_mfma_ok(Cin, K, dtype)) return 0;
  const size_t es = dtype == RN50_BF16 ? 2 : 4;
  return align_up(static_cast<size_t>(N) * K * es, 256) + align_up(static_cast<size_t>(K) * Cin * es, 256);
}

namespace rn50 {
// The parameter gradients of the classifier: dW[k,c] = sum_n dl[n,k] * a[n,c] (float dl: the parameter gradient
// keeps float accuracy) and db[k] = sum_n dl[n,k].  Nothing in the backward pass reads them.
void fc_bwd_params(int N, int Cin, int K, int dtype, const void* a, const float* dlogits, float* dW, float* db,
                   hipStream_t s) {
  DISPATCH_T(dtype, {
    small_gemm<float, T, float>(dlogits, 1, K, static_cast<const T*>(a), Cin, 1, nullptr, dW, K, Cin, N, s);
  });
  RN50_LAUNCH("fc_bwd_bias", colsum_kernel, dim3(ceil_div(K, 256)), dim3(256), 0, s, dlogits, db, N, K);
}
}  // namespace rn50

extern "C" int fc_bwd(int N, int Cin, int K, int dtype, const void* a, const void* W,
                      const float* dlogits, void* da, float* dW, float* db, void* workspace,
                      size_t workspace_bytes, void* stream) {
  clear_error();
  if (int rc = check_dtype(dtype, "fc_bwd")) return rc;
  RN50_REQUIRE(N > 0 && Cin > 0 && K > 0, RN50_ERR_INVALID, "fc_bwd: non-positive size");
  RN50_REQUIRE(a && W && dlogits && da && (dW != nullptr) == (db != nullptr), RN50_ERR_INVALID, "fc_bwd: null pointer");
  const size_t need = fc_bwd_workspace_bytes(N, Cin, K, dtype);
  RN50_REQUIRE(workspace_bytes >= need && (need == 0 || workspace), RN50_ERR_WORKSPACE,
               "fc_bwd: workspace %zu < %zu bytes", workspace_bytes, need);
  RN50_REQUIRE(aligned16(a) && aligned16(W) && aligned16(da) && aligned16(dlogits) && aligned16(workspace),
               RN50_ERR_ALIGN, "fc_bwd: pointer not 16-byte aligned");
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (fc_mfma_ok(Cin, K, dtype)) {
    const size_t es = dtype == RN50_BF16 ? 2 : 4;
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    const void* dl_t = dlogits;
    if (dtype == RN50_BF16) {
      const int64_t n = static_cast<int64_t>(N) * K;
      RN50_LAUNCH("fc_bwd_cast", cast_from_float_kernel<uint16_t>, dim3(ceil_div(n, 256)), dim3(256), 0, s, dlogits,
                         reinterpret_cast<uint16_t*>(ws), n);
      dl_t = ws;
    }
    void* wT = ws + align_up(static_cast<size_t>(N) * K * es, 256);
    const rn50_conv_desc wdesc{1, 1, 1, Cin, K, 1, 1, 1, 0, dtype};  // W [K][Cin] -> wT [Cin][K]
    dgrad_transpose_weights(&wdesc, W, wT, s);
    const rn50_conv_desc d = fc_dgrad_desc(N, Cin, K, dtype);
    fwd_run(&d, dl_t, wT, da, nullptr, s, "fc_bwd_da");
  } else {
    DISPATCH_T(dtype, {
      small_gemm<float, T, T>(dlogits, K, 1, static_cast<const T*>(W), Cin, 1, nullptr,
                              static_cast<T*>(da), N, Cin, K, s);
    });
  }
  // (internal callers that run the parameter gradients elsewhere pass dW = db = null)
  if (dW && db) fc_bwd_params(N, Cin, K, dtype, a, dlogits, dW, db, s);
  return launch_status("fc_bwd");
}

extern "C" int xent_fwd_bwd(int N, int K, const float* logits, const int32_t* labels,
                            float label_smoothing, float grad_scale, float* loss_out,
                            float* row_loss_out, float* dlogits, void* stream) {
  clear_error();
  RN50_REQUIRE(N > 0 && K > 0 && K <= 65536, RN50_ERR_INVALID, "xent_fwd_bwd: N=%d K=%d", N, K);
  RN50_REQUIRE(logits && labels && loss_out && row_loss_out && dlogits, RN50_ERR_INVALID,
               "xent_fwd_bwd: null pointer");
  RN50_REQUIRE(label_smoothing >= 0.f && label_smoothing <= 1.f, RN50_ERR_INVALID,
               "xent_fwd_bwd: label_smoothing %g", label_smoothing);
  hipStream_t s = static_cast<hipStream_t>(stream);
  RN50_LAUNCH("xent", xent_rows_kernel, dim3(N), dim3(256), 0, s, logits, labels, N, K,
                     label_smoothing, grad_scale, row_loss_out, dlogits);
  RN50_LAUNCH("xent", mean_kernel, dim3(1), dim3(256), 0, s, row_loss_out, N, loss_out);
  return launch_status("xent_fwd_bwd");
}

// ------------------------------------------------------------------ top-1
namespace rn50 {
// One workgroup per row: the first maximum of the row (ties go to the lower class index).
__global__ __launch_bounds__(256) void top1_rows_kernel(const float* __restrict__ logits, int K, int32_t* __restrict__ pred) {
  __shared__ float sv[256];
  __shared__ int si[256];
  const float* row = logits + static_cast<int64_t>(blockIdx.x) * K;
  float best = -INFINITY;
  int at = 0x7fffffff;
  for (int k = threadIdx.x; k < K; k += 256) {
    const float v = row[k];
    if (at == 0x7fffffff || v > best) {  // strictly greater keeps the first
      best = v;
      at = k;
    }
  }
  sv[threadIdx.x] = best;
  si[threadIdx.x] = at;
  __syncthreads();
  for (int step = 128; step > 0; step >>= 1) {
    if (threadIdx.x < step) {
      const float ov = sv[threadIdx.x + step];
      const int oi = si[threadIdx.x + step];
      if (oi != 0x7fffffff && (si[threadIdx.x] == 0x7fffffff || ov > sv[threadIdx.x] || (ov == sv[threadIdx.x] && oi < si[threadIdx.x]))) {
        sv[threadIdx.x] = ov;
        si[threadIdx.x] = oi;
      }
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) pred[blockIdx.x] = si[0];
}
// One workgroup: how many predictions equal their label.
__global__ __launch_bounds__(256) void top1_count_kernel(const int32_t* __restrict__ pred, const int32_t* __restrict__ labels,
                                                         int N, int32_t* __restrict__ correct) {
  __shared__ int sc[256];
  int c = 0;
  for (int n = threadIdx.x; n < N; n += 256) c += pred[n] == labels[n];
  sc[threadIdx.x] = c;
  __syncthreads();
  for (int step = 128; step > 0; step >>= 1) {
    if (threadIdx.x < step) sc[threadIdx.x] += sc[threadIdx.x + step];
    __syncthreads();
  }
  if (threadIdx.x == 0) correct[0] = sc[0];
}
}  // namespace rn50

extern "C" int top1_accuracy(int N, int K, const float* logits, const int32_t* labels, int32_t* pred_out,
                             int32_t* correct_out, void* stream) {
  rn50::clear_error();
  RN50_REQUIRE(N > 0 && K > 0, RN50_ERR_INVALID, "top1_accuracy: N=%d K=%d", N, K);
  RN50_REQUIRE(logits && labels && pred_out && correct_out, RN50_ERR_INVALID, "top1_accuracy: null pointer");
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipLaunchKernelGGL(rn50::top1_rows_kernel, dim3(N), dim3(256), 0, s, logits, K, pred_out);
  hipLaunchKernelGGL(rn50::top1_count_kernel, dim3(1), dim3(256), 0, s, pred_out, labels, N, correct_out);
  return rn50::launch_status("top1_accuracy");
}
