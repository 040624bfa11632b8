// Shared host/device helpers of the gfx950 library (error reporting, bf16
// conversion, 16-byte vector access, wave/block reductions).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdarg.h>
#include <stdint.h>
#include <stdio.h>

#include "../../include/rn50_hip.h"

namespace rn50 {

// ---------------------------------------------------------------- host: errors
int fail(int code, const char* fmt, ...);
void clear_error();
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

#define RN50_REQUIRE(cond, code, ...) \
  do {                                \
    if (!(cond)) return ::rn50::fail((code), __VA_ARGS__); \
  } while (0)

// Call after a launch sequence: turns a launch error into RN50_ERR_HIP.
inline int launch_status(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(RN50_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
  return RN50_OK;
}

// Launch timing (see rn50_profile_begin): when it is enabled for `tag`, the launch below hands the runtime an
// event pair that receives the dispatch's own begin and end timestamps, i.e. the kernel's duration on
// the GPU without the cost of separate event packets; otherwise both events are null and the launch is
// an ordinary one.
class KernelTimer {
 public:
  explicit KernelTimer(const char* tag);
  hipEvent_t start() const { return start_; }
  hipEvent_t stop() const { return stop_; }
 private:
  hipEvent_t start_ = nullptr, stop_ = nullptr;
};
#define RN50_LAUNCH(tag, kernel, grid, block, lds, stream, ...)                                          \
  do {                                                                                                   \
    ::rn50::KernelTimer timer_((tag));                                                                   \
    hipExtLaunchKernelGGL(kernel, grid, block, lds, stream, timer_.start(), timer_.stop(), 0, __VA_ARGS__); \
  } while (0)

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t align_up(size_t a, size_t b) { return (a + b - 1) / b * b; }

// ------------------------------------------- division by a launch constant
struct FastDiv {  // exact unsigned division by a runtime constant (Granlund-Montgomery)
  uint32_t mul, sh1, sh2;
};
inline FastDiv make_fastdiv(uint32_t d) {
  if (d == 0) d = 1;  // (an empty dimension: nothing is divided by it)
  uint32_t l = 0;
  while ((1ull << l) < d) ++l;
  FastDiv f;
  f.mul = static_cast<uint32_t>(((1ull << 32) * ((1ull << l) - d)) / d + 1);
  f.sh1 = l < 1 ? l : 1;
  f.sh2 = l > 0 ? l - 1 : 0;
  return f;
}
__device__ __forceinline__ uint32_t fdiv(uint32_t n, const FastDiv& f) {
  const uint32_t t = __umulhi(f.mul, n);
  return (t + ((n - t) >> f.sh1)) >> f.sh2;
}

// -------------------------------------------------------------- device: types
typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// 16 bytes of storage, viewed either as 8 bf16 or as 4 floats.
union alignas(16) Vec16 {
  uint4 u;
  float f[4];
  uint16_t h[8];
};

__device__ __forceinline__ float bf16_bits_to_float(uint16_t h) {
  return __uint_as_float(static_cast<uint32_t>(h) << 16);
}
// Round to nearest even; NaN stays NaN.  The conversion is gfx950's own instruction (v_cvt_pk_bf16_f32,
// two values at a time): written out with integer arithmetic and a NaN test it costs 13 instructions and
// a branch per element, which was most of the convolutions' output stage.
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) {
  return __builtin_bit_cast(uint16_t, static_cast<__bf16>(f));
}
__device__ __forceinline__ uint32_t float2_to_bf16x2_bits(float lo, float hi) {
  f32x2 v;
  v.x = lo; v.y = hi;
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// Element traits: VEC elements per 16-byte vector.
template <typename T> struct Elem;
template <> struct Elem<float> {
  static constexpr int VEC = 4;
  static __device__ __forceinline__ void unpack(const Vec16& v, float* out) {
#pragma unroll
    for (int i = 0; i < 4; ++i) out[i] = v.f[i];
  }
  static __device__ __forceinline__ void pack(const float* in, Vec16& v) {
#pragma unroll
    for (int i = 0; i < 4; ++i) v.f[i] = in[i];
  }
  static __device__ __forceinline__ float load(const float* p) { return *p; }
  static __device__ __forceinline__ void store(float* p, float x) { *p = x; }
};
template <> struct Elem<uint16_t> {  // bf16 storage
  static constexpr int VEC = 8;
  static __device__ __forceinline__ void unpack(const Vec16& v, float* out) {
#pragma unroll
    for (int i = 0; i < 8; ++i) out[i] = bf16_bits_to_float(v.h[i]);
  }
  static __device__ __forceinline__ void pack(const float* in, Vec16& v) {
    v.u = make_uint4(float2_to_bf16x2_bits(in[0], in[1]), float2_to_bf16x2_bits(in[2], in[3]),
                     float2_to_bf16x2_bits(in[4], in[5]), float2_to_bf16x2_bits(in[6], in[7]));
  }
  static __device__ __forceinline__ float load(const uint16_t* p) { return bf16_bits_to_float(*p); }
  static __device__ __forceinline__ void store(uint16_t* p, float x) { *p = float_to_bf16_bits(x); }
};

template <typename T>
__device__ __forceinline__ Vec16 load16(const T* p) {
  Vec16 v;
  v.u = *reinterpret_cast<const uint4*>(p);
  return v;
}
template <typename T>
__device__ __forceinline__ void store16(T* p, const Vec16& v) {
  *reinterpret_cast<uint4*>(p) = v.u;
}

// ------------------------------------------------- device: batch-norm affine
// The affine step y = x*scale + bias and its coefficients, written once so that every kernel that takes
// a ReLU decision from it (forward, backward, the sums fused into the convolutions) uses bit-identical
// arithmetic.
__device__ __forceinline__ float bn_affine(float x, float scale, float bias) { return fmaf(x, scale, bias); }
__device__ __forceinline__ void bn_coeffs(float gamma, float beta, float mean, float rstd, float* scale,
                                          float* bias) {
  *scale = gamma * rstd;
  *bias = fmaf(-mean, *scale, beta);
}

// V (4 or 8) consecutive floats from a 16-byte aligned address, as 16-byte loads.
template <int V>
__device__ __forceinline__ void load_floats(const float* __restrict__ p, float* out) {
#pragma unroll
  for (int i = 0; i < V / 4; ++i) {
    const float4 v = *reinterpret_cast<const float4*>(p + 4 * i);
    out[4 * i] = v.x; out[4 * i + 1] = v.y; out[4 * i + 2] = v.z; out[4 * i + 3] = v.w;
  }
}

// ------------------------------------------------------- device: reductions
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}
// Sum over a 256-thread block; result valid in every thread.  `lds` holds >= 4 floats.
__device__ __forceinline__ float block256_sum(float v, float* lds) {
  v = wave_sum(v);
  const int wave = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) lds[wave] = v;
  __syncthreads();
  return (lds[0] + lds[1]) + (lds[2] + lds[3]);
}

}  // namespace rn50
