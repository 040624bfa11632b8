// Multi-tensor LARS + momentum update (Sec. III-A1 of the paper) with the
// batched norm computation of Sec. III-B2: the squared norms of every tensor's
// weights and gradients are produced by ONE launch whose grid covers all
// tensors in fixed-size chunks, so the 107 tiny tensors of ResNet-50 do not
// each cost a launch that cannot fill the GPU.  A second launch over the same
// chunks finishes the per-tensor sums (fixed order, so results are bitwise
// reproducible), forms the local learning rate and updates w and v in place.
//
// HBM traffic per parameter: 8 B (norm pass: w, g) + 20 B (update: w, g, v read,
// w, v written) + 2 B for the bf16 model copy.  The second read of w and g can
// be served by the 256 MB last-level cache when the model fits.
#include <mutex>

#include "common.h"
#include "step_internal.h"

namespace rn50 {

constexpr int kLarsChunk = 8192;      // elements per workgroup
constexpr int kLarsMaxTensors = 480;  // per launch (chunk table travels as a kernel argument)

struct LarsArgs {
  const rn50_lars_tensor* table;  // device, already offset to this launch's first tensor
  int num;
  int grad_bf16;
  float eta, momentum, lr, eps;
  const float* lr_dev;  // when set, the learning rate is read from here at run time instead of `lr`
  float* partial;    // [total_chunks][2]
  float* norms_out;  // [num][2] or null, offset like table
  int chunk_prefix[kLarsMaxTensors + 1];
  __device__ __forceinline__ rn50_lars_tensor tensor(int t) const { return table[t]; }
};

// The same launch for tensors that live at known offsets of four arenas (the whole-step
// driver): the table travels entirely in the kernel arguments.
constexpr int kLarsArenaMaxTensors = 192;
struct LarsArenaArgs {
  float* master;
  const void* grads;
  float* velocity;
  uint16_t* lowp;  // or null
  int num;
  int grad_bf16;
  float eta, momentum, lr, eps, weight_decay;
  const float* lr_dev;  // as in LarsArgs
  float* partial;
  float* norms_out;
  uint32_t offset[kLarsArenaMaxTensors];  // elements
  uint32_t count[kLarsArenaMaxTensors];
  uint32_t decay_mask[kLarsArenaMaxTensors / 32];
  int chunk_prefix[kLarsArenaMaxTensors + 1];
  __device__ __forceinline__ rn50_lars_tensor tensor(int t) const {
    rn50_lars_tensor T;
    T.w = master + offset[t];
    T.g = grad_bf16 ? static_cast<const void*>(static_cast<const uint16_t*>(grads) + offset[t])
                    : static_cast<const void*>(static_cast<const float*>(grads) + offset[t]);
    T.v = velocity + offset[t];
    T.w_lowp = lowp ? lowp + offset[t] : nullptr;
    T.n = count[t];
    T.weight_decay = ((decay_mask[t >> 5] >> (t & 31)) & 1u) ? weight_decay : 0.f;
    T.apply_trust = 1;
    return T;
  }
};

template <typename Args>
__device__ __forceinline__ int find_tensor(const Args& a, int chunk) {
  int lo = 0, hi = a.num;  // invariant: prefix[lo] <= chunk < prefix[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (a.chunk_prefix[mid] <= chunk) lo = mid; else hi = mid;
  }
  return lo;
}

template <bool GBF16>
__device__ __forceinline__ void load_g4(const void* g, int64_t i, float* out) {
  if (GBF16) {
    const uint2 r = *reinterpret_cast<const uint2*>(static_cast<const uint16_t*>(g) + i);
    out[0] = __uint_as_float(r.x << 16);
    out[1] = __uint_as_float(r.x & 0xffff0000u);
    out[2] = __uint_as_float(r.y << 16);
    out[3] = __uint_as_float(r.y & 0xffff0000u);
  } else {
    const float4 r = *reinterpret_cast<const float4*>(static_cast<const float*>(g) + i);
    out[0] = r.x; out[1] = r.y; out[2] = r.z; out[3] = r.w;
  }
}
template <bool GBF16>
__device__ __forceinline__ float load_g1(const void* g, int64_t i) {
  if (GBF16) return bf16_bits_to_float(static_cast<const uint16_t*>(g)[i]);
  return static_cast<const float*>(g)[i];
}

template <bool GBF16, typename Args>
__global__ __launch_bounds__(256) void lars_norms_kernel(const Args a) {
  __shared__ float red[8];
  const int chunk = blockIdx.x;
  const int t = find_tensor(a, chunk);
  const rn50_lars_tensor T = a.tensor(t);
  const int64_t base = static_cast<int64_t>(chunk - a.chunk_prefix[t]) * kLarsChunk;
  const int64_t end = min(base + static_cast<int64_t>(kLarsChunk), T.n);
  const int64_t vend = base + ((end - base) & ~static_cast<int64_t>(3));
  float sw = 0.f, sg = 0.f;
  // all of a thread's vectors of the chunk are requested before the first is used (16 loads in flight per thread:
  // the pass is a pure stream, and its rate is the bytes in flight); they are added in index order
  constexpr int NV = kLarsChunk / 1024;
  float4 w4[NV];
  float g4[NV][4];
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    const int64_t i = base + threadIdx.x * 4 + k * 1024;
    if (i < vend) {
      w4[k] = *reinterpret_cast<const float4*>(T.w + i);
      load_g4<GBF16>(T.g, i, g4[k]);
    }
  }
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    if (base + threadIdx.x * 4 + k * 1024 < vend) {
      sw += (w4[k].x * w4[k].x + w4[k].y * w4[k].y) + (w4[k].z * w4[k].z + w4[k].w * w4[k].w);
      sg += (g4[k][0] * g4[k][0] + g4[k][1] * g4[k][1]) + (g4[k][2] * g4[k][2] + g4[k][3] * g4[k][3]);
    }
  }
  for (int64_t i = vend + threadIdx.x; i < end; i += 256) {
    const float w = T.w[i], g = load_g1<GBF16>(T.g, i);
    sw += w * w;
    sg += g * g;
  }
  sw = block256_sum(sw, red);
  sg = block256_sum(sg, red + 4);
  if (threadIdx.x == 0) {
    a.partial[2 * chunk] = sw;
    a.partial[2 * chunk + 1] = sg;
  }
}

template <bool GBF16, typename Args>
__global__ __launch_bounds__(256) void lars_apply_kernel(const Args a) {
  __shared__ float red[8];
  const int chunk = blockIdx.x;
  const int t = find_tensor(a, chunk);
  const rn50_lars_tensor T = a.tensor(t);
  const int c0 = a.chunk_prefix[t], c1 = a.chunk_prefix[t + 1];
  // Finish the two sums of this tensor: same order in every block of the tensor.
  float sw = 0.f, sg = 0.f;
  for (int c = c0 + threadIdx.x; c < c1; c += 256) {
    sw += a.partial[2 * c];
    sg += a.partial[2 * c + 1];
  }
  sw = block256_sum(sw, red);
  sg = block256_sum(sg, red + 4);
  const float wn = sqrtf(sw), gn = sqrtf(sg);
  float local = 1.0f;
  if (T.apply_trust && wn > 0.f && gn > 0.f) local = a.eta * wn / (gn + T.weight_decay * wn + a.eps);
  const float lr = a.lr_dev ? *a.lr_dev : a.lr;
  const float step = lr * local, wd = T.weight_decay, mu = a.momentum;
  if (chunk == c0 && threadIdx.x == 0 && a.norms_out) {
    a.norms_out[2 * t] = wn;
    a.norms_out[2 * t + 1] = gn;
  }
  const int64_t base = static_cast<int64_t>(chunk - c0) * kLarsChunk;
  const int64_t end = min(base + static_cast<int64_t>(kLarsChunk), T.n);
  const int64_t vend = base + ((end - base) & ~static_cast<int64_t>(3));
  uint16_t* lowp = static_cast<uint16_t*>(T.w_lowp);
  for (int64_t i = base + threadIdx.x * 4; i < vend; i += 1024) {
    float4 w4 = *reinterpret_cast<const float4*>(T.w + i);
    float4 v4 = *reinterpret_cast<const float4*>(T.v + i);
    float g4[4];
    load_g4<GBF16>(T.g, i, g4);
    v4.x = mu * v4.x + step * (g4[0] + wd * w4.x);
    v4.y = mu * v4.y + step * (g4[1] + wd * w4.y);
    v4.z = mu * v4.z + step * (g4[2] + wd * w4.z);
    v4.w = mu * v4.w + step * (g4[3] + wd * w4.w);
    w4.x -= v4.x; w4.y -= v4.y; w4.z -= v4.z; w4.w -= v4.w;
    *reinterpret_cast<float4*>(T.v + i) = v4;
    *reinterpret_cast<float4*>(T.w + i) = w4;
    if (lowp) {
      uint2 p;
      p.x = float2_to_bf16x2_bits(w4.x, w4.y);
      p.y = float2_to_bf16x2_bits(w4.z, w4.w);
      *reinterpret_cast<uint2*>(lowp + i) = p;
    }
  }
  for (int64_t i = vend + threadIdx.x; i < end; i += 256) {
    const float w = T.w[i], g = load_g1<GBF16>(T.g, i);
    const float v = mu * T.v[i] + step * (g + wd * w);
    const float wnew = w - v;
    T.v[i] = v;
    T.w[i] = wnew;
    if (lowp) lowp[i] = float_to_bf16_bits(wnew);
  }
}

static int64_t total_chunks(const rn50_lars_desc* d, const rn50_lars_tensor* tab) {
  int64_t c = 0;
  for (int t = 0; t < d->num_tensors; ++t) c += ceil_div(tab[t].n, kLarsChunk);
  return c;
}

static int check_table(const rn50_lars_desc* d, const rn50_lars_tensor* tab) {
  RN50_REQUIRE(d && tab, RN50_ERR_INVALID, "lars_update: null descriptor or table");
  RN50_REQUIRE(d->num_tensors > 0, RN50_ERR_INVALID, "lars_update: num_tensors = %d", d->num_tensors);
  RN50_REQUIRE(d->grad_dtype == RN50_F32 || d->grad_dtype == RN50_BF16, RN50_ERR_INVALID,
               "lars_update: grad_dtype = %d", d->grad_dtype);
  for (int t = 0; t < d->num_tensors; ++t) {
    RN50_REQUIRE(tab[t].n > 0, RN50_ERR_INVALID, "lars_update: tensor %d has n = %lld", t,
                 (long long)tab[t].n);
    RN50_REQUIRE(tab[t].w && tab[t].g && tab[t].v, RN50_ERR_INVALID,
                 "lars_update: tensor %d has a null pointer", t);
    RN50_REQUIRE(aligned16(tab[t].w) && aligned16(tab[t].g) && aligned16(tab[t].v) &&
                     aligned16(tab[t].w_lowp),
                 RN50_ERR_ALIGN, "lars_update: tensor %d is not 16-byte aligned", t);
  }
  return RN50_OK;
}

// Arena form used by the whole-step driver.  partial: lars_arena_partial_bytes().
size_t lars_arena_partial_bytes(const LarsArenaSpec& sp) {
  int64_t chunks = 0;
  for (int t = 0; t < sp.num; ++t) chunks += ceil_div(sp.count[t], kLarsChunk);
  return align_up(static_cast<size_t>(chunks) * 2 * sizeof(float), 256);
}

void lars_arena_run(const LarsArenaSpec& sp, float* master, const float* grads, float* velocity, void* lowp,
                    float eta, float momentum, float lr, const float* lr_dev, float eps, float weight_decay,
                    float* partial, hipStream_t s) {
  for (int t0 = 0; t0 < sp.num; t0 += kLarsArenaMaxTensors) {
    LarsArenaArgs a{};
    a.num = sp.num - t0 < kLarsArenaMaxTensors ? sp.num - t0 : kLarsArenaMaxTensors;
    a.master = master; a.grads = grads; a.velocity = velocity; a.lowp = static_cast<uint16_t*>(lowp);
    a.grad_bf16 = 0;
    a.eta = eta; a.momentum = momentum; a.lr = lr; a.lr_dev = lr_dev; a.eps = eps; a.weight_decay = weight_decay;
    a.partial = partial; a.norms_out = nullptr;
    a.chunk_prefix[0] = 0;
    for (int t = 0; t < a.num; ++t) {
      a.offset[t] = static_cast<uint32_t>(sp.offset[t0 + t]);
      a.count[t] = static_cast<uint32_t>(sp.count[t0 + t]);
      if (sp.decay[t0 + t]) a.decay_mask[t >> 5] |= 1u << (t & 31);
      a.chunk_prefix[t + 1] = a.chunk_prefix[t] + static_cast<int>(ceil_div(sp.count[t0 + t], kLarsChunk));
    }
    const int grid = a.chunk_prefix[a.num];
    RN50_LAUNCH("lars_norms", (lars_norms_kernel<false, LarsArenaArgs>), dim3(grid), dim3(256), 0, s, a);
    RN50_LAUNCH("lars_apply", (lars_apply_kernel<false, LarsArenaArgs>), dim3(grid), dim3(256), 0, s, a);
    partial += 2 * static_cast<size_t>(grid);
  }
}

}  // namespace rn50

using namespace rn50;

extern "C" size_t lars_update_workspace_bytes(const rn50_lars_desc* d,
                                              const rn50_lars_tensor* table_host) {
  if (!d || !table_host || d->num_tensors <= 0) return 0;
  return align_up(static_cast<size_t>(total_chunks(d, table_host)) * 2 * sizeof(float), 256);
}

// Both entry points below: the two launches per group of at most kLarsMaxTensors tensors.
static void run_table(const rn50_lars_desc* d, const rn50_lars_tensor* table_host, const rn50_lars_tensor* table_dev,
                      float* norms_out, float* partial, hipStream_t s) {
  for (int t0 = 0; t0 < d->num_tensors; t0 += kLarsMaxTensors) {
    LarsArgs a;
    a.num = d->num_tensors - t0 < kLarsMaxTensors ? d->num_tensors - t0 : kLarsMaxTensors;
    a.table = table_dev + t0;
    a.grad_bf16 = d->grad_dtype == RN50_BF16;
    a.eta = d->eta; a.momentum = d->momentum; a.lr = d->lr; a.eps = d->eps;
    a.lr_dev = nullptr;
    a.partial = partial;
    a.norms_out = norms_out ? norms_out + 2 * t0 : nullptr;
    a.chunk_prefix[0] = 0;
    for (int t = 0; t < a.num; ++t)
      a.chunk_prefix[t + 1] = a.chunk_prefix[t] + static_cast<int>(ceil_div(table_host[t0 + t].n, kLarsChunk));
    const int grid = a.chunk_prefix[a.num];
    if (a.grad_bf16) {
      RN50_LAUNCH("lars_norms", (lars_norms_kernel<true, LarsArgs>), dim3(grid), dim3(256), 0, s, a);
      RN50_LAUNCH("lars_apply", (lars_apply_kernel<true, LarsArgs>), dim3(grid), dim3(256), 0, s, a);
    } else {
      RN50_LAUNCH("lars_norms", (lars_norms_kernel<false, LarsArgs>), dim3(grid), dim3(256), 0, s, a);
      RN50_LAUNCH("lars_apply", (lars_apply_kernel<false, LarsArgs>), dim3(grid), dim3(256), 0, s, a);
    }
    partial += 2 * static_cast<size_t>(grid);
  }
}

extern "C" int lars_update(const rn50_lars_desc* d, const rn50_lars_tensor* table_host,
                           const rn50_lars_tensor* table_dev, float* norms_out, void* workspace,
                           size_t workspace_bytes, void* stream) {
  clear_error();
  if (int rc = check_table(d, table_host)) return rc;
  RN50_REQUIRE(table_dev && workspace, RN50_ERR_INVALID, "lars_update: null device table or workspace");
  RN50_REQUIRE(aligned16(table_dev) && aligned16(workspace), RN50_ERR_ALIGN,
               "lars_update: table_dev / workspace not 16-byte aligned");
  RN50_REQUIRE(workspace_bytes >= lars_update_workspace_bytes(d, table_host), RN50_ERR_WORKSPACE,
               "lars_update: workspace %zu < %zu bytes", workspace_bytes,
               lars_update_workspace_bytes(d, table_host));
  RN50_REQUIRE(total_chunks(d, table_host) < (1ll << 30), RN50_ERR_UNSUPPORTED,
               "lars_update: too many elements");
  run_table(d, table_host, table_dev, norms_out, static_cast<float*>(workspace), static_cast<hipStream_t>(stream));
  return launch_status("lars_update");
}

// ---- lars_update for callers that cannot allocate: the partial norms live in a device array of the
// library itself.  Every GPU holds its own copy of the array at its own address; the address is looked
// up once per device (with that device current) and kept.
constexpr int kLarsStaticChunks = 32768;  // 8192-element chunks: 268 M elements, 256 KB of partial sums
static __device__ __align__(256) float lars_static_scratch[2 * kLarsStaticChunks];

constexpr int kMaxDevices = 64;
static std::mutex scratch_lock;
static float* scratch_ptr[kMaxDevices];  // device address of lars_static_scratch on device i, once known

// Device address of the scratch array on the current device (null + error text on failure).
static float* static_scratch_for_current_device() {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    fail(RN50_ERR_HIP, "lars_update_noalloc: hipGetDevice: %s (device %d)", hipGetErrorString(e), dev);
    return nullptr;
  }
  std::lock_guard<std::mutex> hold(scratch_lock);
  if (!scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(lars_static_scratch));
    if (e != hipSuccess || !p) {
      fail(RN50_ERR_HIP, "lars_update_noalloc: hipGetSymbolAddress: %s", hipGetErrorString(e));
      return nullptr;
    }
    scratch_ptr[dev] = static_cast<float*>(p);
  }
  return scratch_ptr[dev];
}

extern "C" int64_t lars_update_noalloc_max_chunks(void) { return kLarsStaticChunks; }

extern "C" int lars_update_noalloc(const rn50_lars_desc* d, const rn50_lars_tensor* table_host,
                                   const rn50_lars_tensor* table_dev, float* norms_out, void* stream) {
  clear_error();
  if (int rc = check_table(d, table_host)) return rc;
  RN50_REQUIRE(table_dev, RN50_ERR_INVALID, "lars_update_noalloc: null device table");
  RN50_REQUIRE(aligned16(table_dev), RN50_ERR_ALIGN, "lars_update_noalloc: table_dev not 16-byte aligned");
  const int64_t chunks = total_chunks(d, table_host);
  RN50_REQUIRE(chunks <= kLarsStaticChunks, RN50_ERR_WORKSPACE,
               "lars_update_noalloc: the table needs %lld chunks of %d elements, the built-in scratch holds %d "
               "(use lars_update with a workspace)", (long long)chunks, kLarsChunk, kLarsStaticChunks);
  float* partial = static_scratch_for_current_device();
  if (!partial) return RN50_ERR_HIP;
  // Every partial sum the second launch reads is written by the first launch of the same call, so
  // nothing of an earlier call's contents is ever read and nothing needs clearing.
  run_table(d, table_host, table_dev, norms_out, partial, static_cast<hipStream_t>(stream));
  return launch_status("lars_update_noalloc");
}
