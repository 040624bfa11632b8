// Convolution forward, data gradient and weight gradient as implicit GEMMs on
// the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16 for bf16 storage,
// v_mfma_f32_32x32x2_f32 for float storage; float accumulation in both).
//
// Forward and data gradient share one kernel, igemm_kernel:
//     C[m][n] = sum_k A[m][k] * B[n][k]
// where row m is an output pixel, A is gathered on the fly from the NHWC
// activation tensor (k = tap*Cg + channel, 128 contiguous bytes per tap and row,
// zero outside the image), and B is the weight matrix with K contiguous
// (the KRSC weights as they are for the forward pass; for the data gradient a
// [Cin][R][S][Cout] transposition written by a small kernel first).
// 256 threads = 4 waves; global -> registers -> LDS double buffering (one
// barrier per 128-byte K chunk); each wave owns 32x32 MFMA tiles fed by 16-byte
// LDS reads; the MFMA is issued with the weight fragment as its first operand
// so that every lane ends up with 4 consecutive output channels of one pixel,
// which the epilogue packs, stages through LDS and stores as full rows.
//
// The weight gradient, wgrad_kernel, is the GEMM whose reduction runs over the
// pixels: dw[ko][tap][c] = sum_m dy[m][ko] * A[m][tap*Cg + c].  Both operands
// have the reduction index as their slow (row) index in memory, so tiles are
// copied to LDS untransposed and the bf16 fragments are fetched with the
// gfx950 transposing LDS read (ds_read_b64_tr_b16); the reduction is split over
// workgroups and finished by a fixed-order sum (bitwise reproducible).
//
// The output stage of igemm_kernel can also take the per-channel sums of the
// batch norm that consumes the output (forward: shifted sum and sum of squares
// per tile; data gradient: sum(g), sum(g*xhat) of the BN layer below, with an
// optional second gradient branch added before the one rounding), so that no
// separate pass re-reads the tensor.  Stride-2 data gradients process the output
// pixels in four parity classes, each looping over its own taps only.
#include <stdlib.h>

#include <mutex>

#include "common.h"
#include "step_internal.h"

namespace rn50 {

// ----------------------------------------------------------- small utilities
template <typename T> struct Mma;
template <> struct Mma<uint16_t> {  // bf16: one 32x32x16 MFMA per 16-byte fragment pair
  static __device__ __forceinline__ void run(const Vec16& a, const Vec16& b, f32x16& acc) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8*>(&a),
                                                  *reinterpret_cast<const bf16x8*>(&b), acc, 0, 0, 0);
  }
};
template <> struct Mma<float> {  // float: four 32x32x2 MFMAs (k pairs {j, 4+j} of the 8 in flight)
  static __device__ __forceinline__ void run(const Vec16& a, const Vec16& b, f32x16& acc) {
#pragma unroll
    for (int j = 0; j < 4; ++j) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.f[j], b.f[j], acc, 0, 0, 0);
  }
};

// Workgroups are dealt to the 8 XCDs round-robin; renumber them so that consecutive logical ids
// (which share rows of the activation tile) run on the same XCD and meet in its L2.
__device__ __forceinline__ int xcd_remap(int id, int n) {
  const int xcd = id & 7, idx = id >> 3;
  const int q = n >> 3, rem = n & 7;
  return xcd < rem ? xcd * (q + 1) + idx : rem * (q + 1) + (xcd - rem) * q + idx;
}

// ------------------------------------------------- forward / dgrad implicit GEMM
struct IgemmArgs {
  const void* act;  // gathered activation tensor [N][H][W] pixels of PS elements
  const void* wgt;  // B: [Ncols][Ktot]
  void* out;        // C: [M][Ncols]
  uint32_t act_bytes, wgt_bytes;
  int M, Ncols, Ktot;
  int H, W;         // spatial size of the gathered tensor
  int P, Q;         // spatial size of the output pixel grid (M = N*P*Q)
  int PS;           // pixel stride of the gathered tensor, in elements
  int Cg;           // channels per tap
  int R, S, stride, pad;
  int cpt;          // 128-byte chunks per tap
  int ntn;          // number of column tiles
  int pair;         // stem in bf16: a 128-byte chunk holds two filter rows (pieces 0-3: row 2r, 4-7: row 2r+1)
  int nimg;         // images (M = nimg*P*Q)
  // Divisions of the tile / pixel decode by exact multiply-shift (an integer division costs a wave some 40
  // instructions, and every workgroup starts with several of them).  div_w / div_h: by the width / height of
  // the row tiles' pixel grid -- [1] for the odd parity class of a stride-2 data gradient.
  int mtiles;       // row tiles (grid = mtiles * ntn)
  int linear;       // 1x1 filter, stride 1, no padding: row m of the output is pixel m of the gathered tensor
  FastDiv div_ntn, div_w[2], div_h[2];
  int mode;         // host side only: selects the MODE template argument
  // Optional batch-norm sums over the rows of each output tile, taken from the rounded values that are
  // stored (null: none).  Forward: partial[3][Ncols][tiles] = shift (the tile's first row), sum(y - shift),
  // sum((y - shift)^2).  Data gradient: partial[2][Ncols][tiles] = sum(g), sum(g * xhat) with g the output
  // gradient masked by the ReLU of the BN layer whose conv output is bn_x [M][Ncols], xhat its
  // normalized input.
  float* partial;
  const void* bn_x;
  const float *bn_gamma, *bn_beta, *bn_mean, *bn_rstd;
  // Data gradient with sums only.  addend [M][Ncols] (or null): a second gradient branch, added to the
  // product in float before the one rounding to the storage type (the stored output is the sum).
  // bn_zmask (or null): the BN layer's recorded ReLU decision bits, one byte per 16-byte vector of its
  // output; without them the decision is recomputed from bn_x.
  // addend_mask (or null): the addend is the output gradient of a residual-add layer that is still
  // unmasked; it counts only where that layer's recorded ReLU bit is set (same byte layout as bn_zmask).
  const void* addend;
  const uint8_t* bn_zmask;
  const uint8_t* addend_mask;
  // Forward, 1x1 / stride 1 only (BNIN kernels): the gathered tensor is the INPUT of a BN+ReLU layer, whose
  // relu(x*scale + bias) is applied to every operand vector once it sits in LDS (null: the tensor is used as is).
  // in_lds: byte offset of the per-channel coefficient table behind the ring (host side: lds bytes without it).
  const float *in_gamma, *in_beta, *in_mean, *in_rstd;
  int in_lds;
  // Sums stored row-major for a BN pass that finalizes by itself (bn_partials_row_major).  Forward: per tile row and
  // channel the two doubles (sum y, sum y^2), the tile's shifted float sums moved to shift 0 here; data gradient:
  // partial[plane][tile row][Ncols] in float.
  int partial_rm;
};

// relu(bn(x)) of one 16-byte vector with the arithmetic of the stand-alone BN pass (bn_affine, one rounding to
// the storage type), so that a convolution reading it sees bit for bit the tensor that pass would have stored.
template <typename T>
__device__ __forceinline__ Vec16 bn_relu_vector(const Vec16& v, const float* scale, const float* bias) {
  constexpr int V = 16 / sizeof(T);
  float f[V];
  Elem<T>::unpack(v, f);
#pragma unroll
  for (int j = 0; j < V; ++j) f[j] = fmaxf(bn_affine(f[j], scale[j], bias[j]), 0.f);
  Vec16 o;
  Elem<T>::pack(f, o);
  return o;
}
// Barrier behind LDS writes of this wave (s_barrier alone does not wait for them), leaving vector-memory loads in flight.
__device__ __forceinline__ void lds_writes_then_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0); vmcnt, expcnt: no wait
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

constexpr uint32_t kOob = 0x80000000u;  // buffer offset beyond every tensor: the load returns zeros

// Raw buffer descriptor over a tensor: loads whose offset is >= bytes return 0, which is how padding,
// tile tails and ragged channel counts are zero-filled without any per-element masking.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, static_cast<int>(bytes), 0x00020000);
}
__device__ __forceinline__ uint4 buffer_load16(__amdgpu_buffer_rsrc_t r, uint32_t voffset, uint32_t soffset) {
  typedef int v4i __attribute__((ext_vector_type(4)));
  const v4i v = __builtin_amdgcn_raw_buffer_load_b128(r, static_cast<int>(voffset), static_cast<int>(soffset), 0);
  return make_uint4(v.x, v.y, v.z, v.w);
}
// The same load with LDS as its destination (buffer_load_dwordx4 ... lds): lane l of the wave writes its 16
// bytes to LDS address lds_addr + 16*l (lds_addr uniform, taken from M0), so one instruction fills 1 KB; lanes
// whose offset is out of range write zeros.  Nothing passes through registers; the transfer is counted by
// vmcnt like any other vector-memory load.  Written as assembly on purpose: the compiler would make every
// later LDS read wait for ALL outstanding loads of this kind (it cannot tell the ring buffers apart), which
// is the prefetch distance this kernel lives on; the waits are placed by hand (wait_loads_then_barrier).
typedef int rsrc_words __attribute__((ext_vector_type(4)));
__device__ __forceinline__ rsrc_words make_rsrc_words(const void* p, uint32_t bytes) {
  const uint64_t addr = reinterpret_cast<uint64_t>(p);
  rsrc_words r;
  r.x = static_cast<int>(addr);
  r.y = static_cast<int>((addr >> 32) & 0xffffu);  // stride 0: a raw buffer
  r.z = static_cast<int>(bytes);
  r.w = 0x00020000;
  return r;
}
__device__ __forceinline__ void buffer_load16_to_lds(rsrc_words r, uint32_t lds_addr, uint32_t voffset, uint32_t soffset) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :
               : "s"(lds_addr), "v"(voffset), "s"(r), "s"(soffset)
               : "memory");  // (m0 is reserved: the compiler keeps nothing in it across statements)
}
// Wait until at most N of this wave's vector-memory loads are outstanding, then the workgroup barrier, without
// the full memory fence of __syncthreads() (which would also wait for the loads of the chunks still in flight).
template <int N>
__device__ __forceinline__ void wait_loads_then_barrier() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  // s_waitcnt immediate on gfx9: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] << 14; 7 / 15 = no wait
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// Top of iteration kc of a ring of NSTAGE chunk buffers (loads NSTAGE-1 chunks ahead, NL load instructions per
// thread and chunk): wait until this wave's loads of chunk kc have landed -- those of the chunks behind it that
// have been issued, at most NSTAGE-2 of them and none past the last chunk, may stay in flight -- then the barrier.
template <int NSTAGE, int NL>
__device__ __forceinline__ void ring_wait(int chunks_after) {
  static_assert(NSTAGE >= 2 && NSTAGE <= 6 && NL * (NSTAGE - 2) < 64, "ring depth");
  const int ahead = chunks_after < NSTAGE - 2 ? chunks_after : NSTAGE - 2;
  if (NSTAGE >= 6 && ahead == 4) wait_loads_then_barrier<(NSTAGE >= 6 ? 4 : 0) * NL>();
  else if (NSTAGE >= 5 && ahead == 3) wait_loads_then_barrier<(NSTAGE >= 5 ? 3 : 0) * NL>();
  else if (NSTAGE >= 4 && ahead == 2) wait_loads_then_barrier<(NSTAGE >= 4 ? 2 : 0) * NL>();
  else if (NSTAGE >= 3 && ahead == 1) wait_loads_then_barrier<(NSTAGE >= 3 ? 1 : 0) * NL>();
  else wait_loads_then_barrier<0>();
}

// MODE 0: forward gather  ih = p*stride - pad + r.
// MODE 1: data-gradient gather  ih = (p + pad - r)/stride when divisible (stride 1 or 2).  With stride 2
// an output pixel only receives the taps r = (p + pad) mod 2, s = (q + pad) mod 2 (mod 2), so the pixels
// are processed in four parity classes (p mod 2, q mod 2): a row tile holds pixels of one class and loops
// over that class's taps only (a quarter of the taps on average, none for three classes of a 1x1 filter,
// whose tiles just store zeros).
// LIN: compiled for a 1x1 filter with stride 1 and no padding (output row m is pixel m of the gathered
// tensor): no pixel decode, no tap cursor, no bounds checks -- these layers have the shortest reductions
// of the network, and a workgroup's instruction count outside the main loop is what bounds them.
//
// Tile BM x BN, WM x WN waves (4 or 8), each wave a (BM/WM) x (BN/WN) tile of 32x32 MFMA blocks.  A 128-byte
// K chunk of the tile is (BM + BN) rows of 128 bytes in LDS, filled by buffer loads that write LDS directly
// (8 lanes per row, 8 rows per wave instruction) into a ring of three chunk buffers: the loads of chunk k+2 are
// issued when chunk k starts, one barrier per chunk.  Within a row the eight 16-byte pieces are stored
// permuted, piece p of row r in slot p ^ ((r >> 1) & 7): the MFMA fragment reads (lane = row, 16 bytes of one
// piece) then touch every bank once per 16 lanes.  What bounds the main loop per compute unit, measured:
// 16-byte vector loads deliver ~60 B/clk, 16-byte LDS reads ~220 B/clk, one 32x32x16 MFMA per SIMD every 32
// clocks.  A 32x32 wave tile reads 2 KB of fragments per MFMA (LDS-bound at half the MFMA rate), a 64x64
// wave tile 1 KB; a 64x64 workgroup tile loads 16 KB per 128 MFMA-clocks (load-bound at half the MFMA rate),
// a 128x128 tile 32 KB per 512.  Hence the largest tile that still gives every compute unit work is chosen
// per layer shape (igemm_tile below).
// Chunk buffers in the ring: three (loads two chunks ahead), or two where three would leave room for only one
// four-wave workgroup per compute unit (160 KB of LDS): two workgroups hide each other's barriers and latencies.
template <int BM, int BN, int NW>
constexpr int igemm_ring() {
  return (NW == 4 && 3 * (BM + BN) * 128 > 80 * 1024) ? 2 : 3;
}
//
// HALO: compiled for a 3x3 filter with stride 1 and padding 1 (output pixel m reads input pixels m + dy*W + dx,
// dy, dx in -1..1, of the same flat pixel index space).  The nine taps of a tile then read one contiguous run of
// BM + 2W + 2 input pixels: that run is brought into LDS once per 128-byte channel chunk (instead of a gathered
// BM-row tile per tap: nine times the operand traffic), and the fragment reads of tap (dy, dx) start dy*W + dx rows
// further down in it.  Taps that fall off the image (or into the neighbouring image of the run) are zeroed in
// the fragment registers, by a per-lane bit mask computed once.  The weights go through a ring of three
// BN-row tiles, two taps ahead; the next chunk's run is loaded one pass per tap while the
// current one is in use, so that every step issues the same number of loads (the load waits count them).
template <typename T, int BM, int BN, int WM, int WN, int MODE, bool LIN = false, bool BNIN = false, bool HALO = false>
__global__ __launch_bounds__(64 * WM * WN) void igemm_kernel(const IgemmArgs a) {
  static_assert(!BNIN || (LIN && MODE == 0), "the input-side BN is compiled for the linear forward kernel only");
  static_assert(!HALO || (!LIN && !BNIN), "the halo main loop is a kernel of its own");
  constexpr int NW = WM * WN, NT = 64 * NW;
  constexpr int V = 16 / sizeof(T);
  constexpr int BK = 128 / sizeof(T);
  constexpr int RPL = NT / 8;                   // tile rows covered by one load pass of the workgroup
  constexpr int RA = BM / RPL, RB = BN / RPL;  // load passes (= load instructions per thread and chunk)
  constexpr int NL = RA + RB;
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  constexpr int STAGE = (BM + BN) * 128;
  constexpr int NSTAGE = igemm_ring<BM, BN, WM * WN>();
  constexpr int CP = BN * sizeof(T) + 16;  // epilogue pitch
  static_assert((NW == 4 || NW == 8) && TM >= 1 && TN >= 1 && RA >= 1 && RB >= 1, "tile shape");
  static_assert(BM % RPL == 0 && BN % RPL == 0, "every load pass covers whole rows of the tile");
  constexpr int CPW = BN * 4 + 16;         // pitch of a float output tile (bf16 data gradient with an addend)
  // (the launch sizes the dynamic LDS as the larger of the ring and what the output stage stores in it)
  extern __shared__ __align__(16) unsigned char smem[];

  const int tid = threadIdx.x, slot = tid & 7, lrow = tid >> 3;
  const int piece = slot ^ ((lrow >> 1) & 7);  // the 16-byte piece of its rows' chunk this thread fetches
  const int wave = tid >> 6, lane = tid & 63;
  const int wm = wave % WM, wn = wave / WM;
  const int bid = xcd_remap(blockIdx.x, gridDim.x);
  const int mt = static_cast<int>(fdiv(static_cast<uint32_t>(bid), a.div_ntn)), nt = bid - mt * a.ntn;
  const int n0 = nt * BN;
  const rsrc_words rsA = make_rsrc_words(a.act, a.act_bytes), rsB = make_rsrc_words(a.wgt, a.wgt_bytes);

  // Rows of this tile: pixels m0.. of the whole output grid, or of one parity class of it.
  const bool classes = !LIN && MODE == 1 && a.stride == 2;
  __shared__ int pix_s[BM];  // classes only: output pixel index of every tile row
  // Data gradient with batch-norm sums: the per-channel coefficients of this tile's columns, fetched by one
  // thread per column while the main loop runs (every thread loading its own copies costs the texture path
  // as much as two chunks of the main loop).
  __shared__ float prm_s[MODE == 1 ? 4 * BN : 4];
  float pg = 0.f, pb = 0.f, pm = 0.f, pr = 0.f;
  if (MODE == 1 && a.partial != nullptr && tid < BN) {
    const int c = min(n0 + tid, a.Ncols - 1);
    pg = a.bn_gamma[c]; pb = a.bn_beta[c]; pm = a.bn_mean[c]; pr = a.bn_rstd[c];
  }
  int ph = 0, pw = 0, Hc = a.P, Wc = a.Q, Mc = a.M, m0 = mt * BM;
  int r0 = 0, s0 = 0, tstep = 1;
  if (classes) {
    // the four classes of one pixel range are neighbours in the tile order: they read the same rows of
    // the incoming gradient, and every XCD gets its share of the classes that have taps
    const int cls = mt & 3;
    m0 = (mt >> 2) * BM;
    ph = cls >> 1; pw = cls & 1;
    Hc = (a.P - ph + 1) >> 1; Wc = (a.Q - pw + 1) >> 1;
    Mc = a.nimg * Hc * Wc;
    r0 = (ph + a.pad) & 1; s0 = (pw + a.pad) & 1; tstep = 2;
  }
  const int nr = r0 < a.R ? (a.R - r0 + tstep - 1) >> (tstep - 1) : 0, ns = s0 < a.S ? (a.S - s0 + tstep - 1) >> (tstep - 1) : 0;
  FastDiv dvw, dvh;  // selected field by field, by value
  dvw.mul = pw ? +a.div_w[1].mul : +a.div_w[0].mul; dvw.sh1 = pw ? +a.div_w[1].sh1 : +a.div_w[0].sh1; dvw.sh2 = pw ? +a.div_w[1].sh2 : +a.div_w[0].sh2;
  dvh.mul = ph ? +a.div_h[1].mul : +a.div_h[0].mul; dvh.sh1 = ph ? +a.div_h[1].sh1 : +a.div_h[0].sh1; dvh.sh2 = ph ? +a.div_h[1].sh2 : +a.div_h[0].sh2;

  // per-thread rows of the A tile: decode the output pixel once
  int a_h0[RA], a_w0[RA], a_base[RA];
#pragma unroll
  for (int i = 0; i < RA; ++i) {
    const int m = m0 + lrow + RPL * i;
    const bool ok = m < Mc;
    const int mm = ok ? m : 0;
    if (LIN || a.linear) {  // no pixel decode: "image" base mm, coordinates (0, 0)
      a_base[i] = mm;
      a_h0[i] = ok ? 0 : -(1 << 20);
      a_w0[i] = 0;
      continue;
    }
    const int t = static_cast<int>(fdiv(static_cast<uint32_t>(mm), dvw));
    int q = mm - t * Wc;
    const int n = static_cast<int>(fdiv(static_cast<uint32_t>(t), dvh));
    int p = t - n * Hc;
    if (classes) {
      p = 2 * p + ph; q = 2 * q + pw;
      if (slot == 0) pix_s[lrow + RPL * i] = ok ? (n * a.P + p) * a.Q + q : 0;
    }
    a_base[i] = n * a.H * a.W;
    // a row beyond the last gets coordinates that fail every bounds check below
    a_h0[i] = ok ? (MODE == 0 ? p * a.stride - a.pad : p + a.pad) : -(1 << 20);
    a_w0[i] = MODE == 0 ? q * a.stride - a.pad : q + a.pad;
  }
  uint32_t b_row[RB];
#pragma unroll
  for (int i = 0; i < RB; ++i) {
    const int n = n0 + lrow + RPL * i;
    b_row[i] = n < a.Ncols ? static_cast<uint32_t>(n * a.Ktot + piece * V) * sizeof(T) : kOob;
  }

  // Load cursor: tap (r,s), chunk cc within the tap.  Per tap, the byte offset of every row's pixel (or
  // kOob); within a tap successive chunks only differ by a scalar offset.
  const int nchunks = nr * ns * a.cpt;
  int cur_r = r0, cur_s = s0, cur_cc = 0, cur = 0;
  uint32_t a_off[RA], b_tap = static_cast<uint32_t>((r0 * a.S + s0) * a.Cg) * sizeof(T);
  const bool ragged = (a.Cg % BK) != 0;
  auto tap_setup = [&]() __attribute__((always_inline)) {
    if constexpr (LIN) {
#pragma unroll
      for (int i = 0; i < RA; ++i)
        a_off[i] = a_h0[i] < 0 ? kOob : static_cast<uint32_t>(a_base[i] * a.PS + piece * V) * sizeof(T);
      return;
    }
#pragma unroll
    for (int i = 0; i < RA; ++i) {
      int ih, iw;
      bool ok = true;
      if (MODE == 0) {
        ih = a_h0[i] + (a.pair ? 2 * cur_r + (piece >> 2) : cur_r);
        iw = a_w0[i] + cur_s;
      } else {
        const int th = a_h0[i] - cur_r, tw = a_w0[i] - cur_s;
        const int msk = a.stride - 1;  // stride is 1 or 2
        ok = th >= 0 && tw >= 0 && ((th | tw) & msk) == 0;
        ih = th >> msk;
        iw = tw >> msk;
      }
      ok = ok && static_cast<unsigned>(ih) < static_cast<unsigned>(a.H) &&
           static_cast<unsigned>(iw) < static_cast<unsigned>(a.W);
      const int pc = (MODE == 0 && a.pair) ? (piece & 3) : piece;
      a_off[i] = ok ? static_cast<uint32_t>((a_base[i] + ih * a.W + iw) * a.PS + pc * V) * sizeof(T) : kOob;
    }
  };
  // One chunk into one ring buffer: every wave fills its 8 rows of each load pass (1 KB per instruction).
  typedef __attribute__((address_space(3))) unsigned char* lds_byte_ptr;
  const uint32_t wave_dst = __builtin_amdgcn_readfirstlane(
      static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_byte_ptr)smem)) + static_cast<uint32_t>(wave) * 1024u);
  auto load_chunk = [&](int stage) __attribute__((always_inline)) {
    const uint32_t so = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(cur_cc) * 128u);
    const bool cval = !ragged || (cur_cc * BK + piece * V < a.Cg);
    ++cur;
    const uint32_t sa = wave_dst + static_cast<uint32_t>(stage) * STAGE;
    const uint32_t sb = sa + BM * 128;
    const uint32_t sob = __builtin_amdgcn_readfirstlane(b_tap + so);
#pragma unroll
    for (int i = 0; i < RA; ++i) buffer_load16_to_lds(rsA, sa + i * (RPL * 128), cval ? a_off[i] : kOob, so);
#pragma unroll
    for (int i = 0; i < RB; ++i) buffer_load16_to_lds(rsB, sb + i * (RPL * 128), cval ? b_row[i] : kOob, sob);
    // advance the cursor
    if constexpr (LIN) {
      ++cur_cc;
    } else if (++cur_cc == a.cpt) {
      cur_cc = 0;
      cur_s += tstep;
      if (cur_s >= a.S) {
        cur_s = s0;
        cur_r += tstep;
      }
      b_tap = static_cast<uint32_t>((cur_r * a.S + cur_s) * a.Cg) * sizeof(T);
      if (cur < nchunks) tap_setup();  // (nothing is loaded past the last chunk)
    }
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // Fragment of a 32-row block for k step kk: row = lane % 32, piece 2*kk + lane/32, in its permuted slot
  // (the block starts at a multiple of 32 rows, so the permutation depends on the lane alone).
  int frag_off[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk)
    frag_off[kk] = (lane & 31) * 128 + (((2 * kk + (lane >> 5)) ^ ((lane >> 1) & 7)) << 4);
  // The fragment reads run ahead of the MFMAs that use them -- a whole chunk ahead for the small wave tiles
  // (one MFMA per k step is far shorter than an LDS read's latency), one k step ahead for 64x64 wave tiles --
  // so a wave pays the LDS latency once per chunk, not once per k step.
  constexpr int AHEAD = (TM + TN <= 3) ? 4 : 1;  // k steps whose fragments are in registers before the first MFMA
  auto compute = [&](int stage) __attribute__((always_inline)) {
    const unsigned char* sa = smem + stage * STAGE + wm * (BM / WM) * 128;
    const unsigned char* sb = smem + stage * STAGE + BM * 128 + wn * (BN / WN) * 128;
    Vec16 fa[4][TM], fb[4][TN];
    auto read_frags = [&](int kk) __attribute__((always_inline)) {
#pragma unroll
      for (int i = 0; i < TM; ++i) fa[kk][i].u = *reinterpret_cast<const uint4*>(sa + i * 32 * 128 + frag_off[kk]);
#pragma unroll
      for (int j = 0; j < TN; ++j) fb[kk][j].u = *reinterpret_cast<const uint4*>(sb + j * 32 * 128 + frag_off[kk]);
    };
#pragma unroll
    for (int kk = 0; kk < AHEAD; ++kk) read_frags(kk);
    __builtin_amdgcn_sched_barrier(0);  // (the instruction scheduler would sink every read to its first use)
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      if (kk + AHEAD < 4) {
        read_frags(kk + AHEAD);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) Mma<T>::run(fb[kk][j], fa[kk][i], acc[i][j]);  // D'[n][m]
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // Ring of NSTAGE chunk buffers, loads NSTAGE-1 chunks ahead.  At the top of iteration kc this wave waits for
  // its own loads of chunk kc (those of the later chunks may still be in flight), then the barrier: behind it
  // every wave's part of chunk kc is in LDS and every wave is done reading chunk kc-1, whose buffer the loads
  // of chunk kc+NSTAGE-1 issued next will overwrite.
  if constexpr (HALO) {
    constexpr int NSB = 3;                       // weight tiles in the ring
    const int Wd = a.W;
    const int NA = (BM + 2 * Wd + 2 + RPL - 1) / RPL;  // load passes of one run (the host checked NA <= 8)
    const uint32_t run_bytes = static_cast<uint32_t>(NA) * (RPL * 128);
    const int cpt = a.cpt;
    const uint32_t b_base = (cpt > 1 ? 2u : 1u) * run_bytes;  // two runs when there is a next chunk to prefetch
    const uint32_t dump = b_base + NSB * BN * 128;          // where the loads that only keep the count go (zeros)
    const uint32_t lds0 = wave_dst;                           // LDS address of smem + this wave's 1 KB share of a pass
    const int q0 = m0 - Wd - 1 + lrow;                        // input pixel of this thread's row in pass 0 of a run
    auto load_run_pass = [&](int j, int cc, int buf) __attribute__((always_inline)) {
      const int q = q0 + RPL * j;
      const bool ok = static_cast<unsigned>(q) < static_cast<unsigned>(a.M) && (!ragged || cc * BK + piece * V < a.Cg);
      const uint32_t off = ok ? static_cast<uint32_t>(q * a.PS + piece * V) * sizeof(T) : kOob;
      buffer_load16_to_lds(rsA, lds0 + static_cast<uint32_t>(buf) * run_bytes + static_cast<uint32_t>(j) * (RPL * 128), off,
                           __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(cc) * 128u));
    };
    auto load_b_tile = [&](int stage, int cc, int tap, bool live) __attribute__((always_inline)) {
      const bool cval = live && (!ragged || cc * BK + piece * V < a.Cg);
      const uint32_t sob = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(tap * a.Cg) * static_cast<uint32_t>(sizeof(T)) +
                                                          static_cast<uint32_t>(cc) * 128u);
#pragma unroll
      for (int i = 0; i < RB; ++i)
        buffer_load16_to_lds(rsB, lds0 + b_base + static_cast<uint32_t>(stage) * (BN * 128) + i * (RPL * 128),
                             cval ? b_row[i] : kOob, sob);
    };
    auto load_nothing = [&]() __attribute__((always_inline)) { buffer_load16_to_lds(rsA, lds0 + dump, kOob, 0); };
    // Which taps of which rows exist: bit `tap` of vmask[i] for this lane's row of the wave's row block i.
    uint32_t vmask[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int m = m0 + wm * (BM / WM) + i * 32 + (lane & 31);
      const bool ok = m < a.M;
      const int mm = ok ? m : 0;
      const int t = static_cast<int>(fdiv(static_cast<uint32_t>(mm), a.div_w[0]));
      const int x = mm - t * a.Q;
      const int y = t - static_cast<int>(fdiv(static_cast<uint32_t>(t), a.div_h[0])) * a.P;
      uint32_t bits = 0;
#pragma unroll
      for (int tap = 0; tap < 9; ++tap) {
        const int dyo = MODE == 0 ? tap / 3 - 1 : 1 - tap / 3, dxo = MODE == 0 ? tap % 3 - 1 : 1 - tap % 3;
        const bool v = ok && static_cast<unsigned>(y + dyo) < static_cast<unsigned>(a.H) &&
                       static_cast<unsigned>(x + dxo) < static_cast<unsigned>(a.W);
        bits |= v ? (1u << tap) : 0u;
      }
      vmask[i] = bits;
    }
    auto compute_tap = [&](int buf, int bstage, int tap, int dyo, int dxo) __attribute__((always_inline)) {
      const int rl = (lane & 31) + (dyo + 1) * Wd + (dxo + 1);  // row of the run this lane's row 0 reads
      const int swz = (rl >> 1) & 7;
      int aoff[4];
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) aoff[kk] = rl * 128 + (((2 * kk + (lane >> 5)) ^ swz) << 4);
      uint32_t mk[TM];
#pragma unroll
      for (int i = 0; i < TM; ++i) mk[i] = ((vmask[i] >> tap) & 1u) ? 0xffffffffu : 0u;
      const unsigned char* sa = smem + static_cast<uint32_t>(buf) * run_bytes + wm * (BM / WM) * 128;
      const unsigned char* sb = smem + b_base + bstage * (BN * 128) + wn * (BN / WN) * 128;
      Vec16 fa[4][TM], fb[4][TN];
      auto read_frags = [&](int kk) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[kk][i].u = *reinterpret_cast<const uint4*>(sa + i * 32 * 128 + aoff[kk]);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[kk][j].u = *reinterpret_cast<const uint4*>(sb + j * 32 * 128 + frag_off[kk]);
      };
      constexpr int AH = (TM + TN <= 3) ? 4 : 1;
#pragma unroll
      for (int kk = 0; kk < AH; ++kk) read_frags(kk);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        if (kk + AH < 4) {
          read_frags(kk + AH);
          __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int i = 0; i < TM; ++i) {
          fa[kk][i].u.x &= mk[i]; fa[kk][i].u.y &= mk[i]; fa[kk][i].u.z &= mk[i]; fa[kk][i].u.w &= mk[i];
#pragma unroll
          for (int j = 0; j < TN; ++j) Mma<T>::run(fb[kk][j], fa[kk][i], acc[i][j]);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    // Prologue: the first run, the weight tiles of steps 0 and 1.  Every step of the loop then issues RB + 1
    // loads (the weight tile two steps ahead; one pass of the next chunk's run, or a load of nothing), so at its
    // top "at most RB + 1 outstanding" means: everything up to the step before the previous one has landed.
    for (int j = 0; j < NA; ++j) load_run_pass(j, 0, 0);
    load_b_tile(0, 0, 0, true);
    load_b_tile(1, 0, 1, true);
    load_nothing();
    int bstage = 0;
    for (int cc = 0; cc < cpt; ++cc) {
      const int buf = cpt > 1 ? (cc & 1) : 0;
#pragma unroll
      for (int tap = 0; tap < 9; ++tap) {
        wait_loads_then_barrier<RB + 1>();
        const int tap2 = (tap + 2) % 9, cc2 = cc + (tap + 2 >= 9 ? 1 : 0);
        load_b_tile(bstage >= 1 ? bstage - 1 : NSB - 1, cc2, tap2, cc2 < cpt);  // the tile of step - 1: free again
        if (tap < NA && cc + 1 < cpt) load_run_pass(tap, cc + 1, buf ^ 1);
        else load_nothing();
        compute_tap(buf, bstage, tap, MODE == 0 ? tap / 3 - 1 : 1 - tap / 3, MODE == 0 ? tap % 3 - 1 : 1 - tap % 3);
        bstage = bstage == NSB - 1 ? 0 : bstage + 1;
      }
    }
    // (the loads still in flight carry nothing and land in the dump area or in weight tiles nobody reads again;
    // they are waited for before the output stage reuses LDS)
    wait_loads_then_barrier<0>();
  } else {
  tap_setup();
  float* const in_tab = reinterpret_cast<float*>(smem + (BNIN ? a.in_lds : 0));  // [2][nchunks * BK]: scale, bias
  if constexpr (BNIN) {
    const int kpad = nchunks * BK;
    for (int c = tid; c < kpad; c += NT) {
      float sc = 0.f, bi = 0.f;
      if (c < a.Cg) bn_coeffs(a.in_gamma[c], a.in_beta[c], a.in_mean[c], a.in_rstd[c], &sc, &bi);
      in_tab[c] = sc;
      in_tab[kpad + c] = bi;
    }
    __syncthreads();
  }
#pragma unroll
  for (int c = 0; c < NSTAGE - 1; ++c)
    if (c < nchunks) load_chunk(c);
  int stage = 0;
  for (int kc = 0; kc < nchunks; ++kc) {
    ring_wait<NSTAGE, NL>(nchunks - 1 - kc);
    if (kc + NSTAGE - 1 < nchunks) load_chunk(stage >= 1 ? stage - 1 : NSTAGE - 1);  // buffer (kc - 1) mod NSTAGE
    if constexpr (BNIN) {
      // every thread transforms, in place, the vectors of chunk kc that its own loads brought (its slot of its
      // rows holds piece `piece`, i.e. channels kc*BK + piece*V ..), then a second barrier
      float scale[V], bias[V];
      const int kpad = nchunks * BK;
      load_floats<V>(in_tab + kc * BK + piece * V, scale);
      load_floats<V>(in_tab + kpad + kc * BK + piece * V, bias);
#pragma unroll
      for (int i = 0; i < RA; ++i) {
        uint4* p = reinterpret_cast<uint4*>(smem + stage * STAGE + (lrow + RPL * i) * 128 + slot * 16);
        Vec16 v;
        v.u = *p;
        *p = bn_relu_vector<T>(v, scale, bias).u;
      }
      lds_writes_then_barrier();
    }
    compute(stage);
    stage = stage == NSTAGE - 1 ? 0 : stage + 1;
  }
  }
  __builtin_amdgcn_s_barrier();  // the output tile below reuses the pipeline buffers
  asm volatile("" ::: "memory");

  // Epilogue.  acc[i][j][v]: output channel n = j*32 + (v/4)*8 + (lane/32)*4 + v%4, pixel m = i*32 + lane%32.
  // The tile goes to LDS in the storage type, or in float when a bf16 data gradient has an addend.
  const bool wide = sizeof(T) == 2 && MODE == 1 && a.partial != nullptr && a.addend != nullptr;
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int row = wm * (BM / WM) + i * 32 + (lane & 31);
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int col = wn * (BN / WN) + j * 32 + g * 8 + (lane >> 5) * 4;
        unsigned char* dst = smem + row * CP + col * sizeof(T);
        if (wide) {
          *reinterpret_cast<float4*>(smem + row * CPW + col * 4) =
              make_float4(acc[i][j][g * 4 + 0], acc[i][j][g * 4 + 1], acc[i][j][g * 4 + 2], acc[i][j][g * 4 + 3]);
        } else if (sizeof(T) == 2) {
          uint2 p;
          p.x = float2_to_bf16x2_bits(acc[i][j][g * 4 + 0], acc[i][j][g * 4 + 1]);
          p.y = float2_to_bf16x2_bits(acc[i][j][g * 4 + 2], acc[i][j][g * 4 + 3]);
          *reinterpret_cast<uint2*>(dst) = p;
        } else {
          *reinterpret_cast<float4*>(dst) = make_float4(acc[i][j][g * 4 + 0], acc[i][j][g * 4 + 1], acc[i][j][g * 4 + 2], acc[i][j][g * 4 + 3]);
        }
      }
    }
  if (MODE == 1 && a.partial != nullptr && tid < BN) {
    float sc, bi;
    bn_coeffs(pg, pb, pm, pr, &sc, &bi);
    prm_s[tid] = sc; prm_s[BN + tid] = bi; prm_s[2 * BN + tid] = pr; prm_s[3 * BN + tid] = -pm * pr;
  }
  __syncthreads();
  constexpr int PPR = BN * sizeof(T) / 16;  // 16-byte pieces per output row
  constexpr int RPP = NT / PPR;             // rows per pass
  constexpr int NPASS = BM / RPP;
  T* out = static_cast<T*>(a.out);
  const int op = tid % PPR, orow = tid / PPR;
  const int n = n0 + op * V;
  if (a.partial == nullptr) {
#pragma unroll
    for (int pass = 0; pass < NPASS; ++pass) {
      const int row = orow + pass * RPP;
      const int m = m0 + row;
      if (m < Mc && n < a.Ncols) {
        const int pix = classes ? pix_s[row] : m;
        *reinterpret_cast<uint4*>(out + (static_cast<int64_t>(pix) * a.Ncols + n)) =
            *reinterpret_cast<const uint4*>(smem + row * CP + op * 16);
      }
    }
    return;
  }

  // Output stage with batch-norm sums: every thread owns V channels and NPASS rows of the tile.
  const bool col_ok = n < a.Ncols;
  float s1[V], s2[V];
#pragma unroll
  for (int j = 0; j < V; ++j) s1[j] = s2[j] = 0.f;
  if (MODE == 0) {
    float shift[V];
    Vec16 k0;
    k0.u = *reinterpret_cast<const uint4*>(smem + op * 16);  // row m0 of the tile always exists
    Elem<T>::unpack(k0, shift);
#pragma unroll
    for (int pass = 0; pass < NPASS; ++pass) {
      const int row = orow + pass * RPP;
      const int m = m0 + row;
      if (m < Mc && col_ok) {
        Vec16 v;
        v.u = *reinterpret_cast<const uint4*>(smem + row * CP + op * 16);
        *reinterpret_cast<uint4*>(out + (static_cast<int64_t>(m) * a.Ncols + n)) = v.u;
        float f[V];
        Elem<T>::unpack(v, f);
#pragma unroll
        for (int j = 0; j < V; ++j) {
          const float d = f[j] - shift[j];
          s1[j] += d;
          s2[j] = fmaf(d, d, s2[j]);
        }
      }
    }
  } else {
    const T* bx = static_cast<const T*>(a.bn_x);
    const int nc = col_ok ? n : 0;
    const T* add = static_cast<const T*>(a.addend);
    Vec16 xv[NPASS], av[NPASS];
    uint32_t zb[NPASS], ab[NPASS];
    int pix[NPASS];
#pragma unroll
    for (int pass = 0; pass < NPASS; ++pass) {
      const int row = orow + pass * RPP;
      pix[pass] = classes ? pix_s[row] : min(m0 + row, a.M - 1);  // rows past the last read a valid pixel
      const int64_t at = static_cast<int64_t>(pix[pass]) * a.Ncols + nc;
      xv[pass] = load16(bx + at);
      if (add) av[pass] = load16(add + at);
      if (a.bn_zmask) zb[pass] = a.bn_zmask[at / V];
      ab[pass] = a.addend_mask ? a.addend_mask[at / V] : 0xffu;
    }
    float scale[V], bias[V], rs[V], nmr[V];
#pragma unroll
    for (int j = 0; j < V; ++j) {
      scale[j] = prm_s[op * V + j]; bias[j] = prm_s[BN + op * V + j];
      rs[j] = prm_s[2 * BN + op * V + j]; nmr[j] = prm_s[3 * BN + op * V + j];
    }
#pragma unroll
    for (int pass = 0; pass < NPASS; ++pass) {
      const int row = orow + pass * RPP;
      if (m0 + row < Mc && col_ok) {
        Vec16 v;
        float g[V], xf[V];
        if (add) {
          float ad[V];
          Elem<T>::unpack(av[pass], ad);
#pragma unroll
          for (int j = 0; j < V; ++j) ad[j] = ((ab[pass] >> j) & 1u) ? ad[j] : 0.f;
          if (wide) {
            const float4 lo = *reinterpret_cast<const float4*>(smem + row * CPW + op * 32);
            const float4 hi = *reinterpret_cast<const float4*>(smem + row * CPW + op * 32 + 16);
            const float t[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
#pragma unroll
            for (int j = 0; j < V; ++j) g[j] = t[j] + ad[j];
          } else {
            v.u = *reinterpret_cast<const uint4*>(smem + row * CP + op * 16);
            Elem<T>::unpack(v, g);
#pragma unroll
            for (int j = 0; j < V; ++j) g[j] += ad[j];
          }
          Elem<T>::pack(g, v);
        } else {
          v.u = *reinterpret_cast<const uint4*>(smem + row * CP + op * 16);
        }
        *reinterpret_cast<uint4*>(out + (static_cast<int64_t>(pix[pass]) * a.Ncols + n)) = v.u;
        Elem<T>::unpack(v, g);  // the sums range over the stored (rounded) values
        Elem<T>::unpack(xv[pass], xf);
#pragma unroll
        for (int j = 0; j < V; ++j) {
          const bool on = a.bn_zmask ? ((zb[pass] >> j) & 1u) != 0 : bn_affine(xf[j], scale[j], bias[j]) > 0.f;
          const float gm = on ? g[j] : 0.f;
          s1[j] += gm;
          s2[j] = fmaf(gm, fmaf(xf[j], rs[j], nmr[j]), s2[j]);
        }
      }
    }
  }
  // The per-thread sums of a column meet through LDS: [row group][plane][column], over the tile buffer
  // (every thread is done with its rows of the tile), then one thread per plane and column adds the RPP row
  // groups in order.  (Wave shuffles here -- 6 * V of them per thread -- cost more than the whole loop above.)
  float kshift = 0.f;
  if (MODE == 0 && tid < BN) kshift = Elem<T>::load(reinterpret_cast<const T*>(smem) + tid);  // row m0 of the tile
  __syncthreads();
  float* cs = reinterpret_cast<float*>(smem);
  static_assert(RPP * 2 * BN * 4 <= BM * CPW, "the column sums fit where the output tile was");
  static_assert(2 * BN <= NT && NPASS >= 1, "one thread per plane and column");
#pragma unroll
  for (int j = 0; j < V; j += 4) {
    *reinterpret_cast<float4*>(cs + (orow * 2 + 0) * BN + op * V + j) = make_float4(s1[j], s1[j + 1], s1[j + 2], s1[j + 3]);
    *reinterpret_cast<float4*>(cs + (orow * 2 + 1) * BN + op * V + j) = make_float4(s2[j], s2[j + 1], s2[j + 2], s2[j + 3]);
  }
  __syncthreads();
  // partial[plane][channel][tile row]: the rows of one channel are contiguous for the finalize pass
  const int64_t nrows = a.mtiles, plane = static_cast<int64_t>(a.Ncols) * nrows;
  if (MODE == 0 && a.partial_rm) {
    // row-major, for an apply pass that finalizes by itself: one thread per column moves the tile's sums from the
    // tile's shift k to shift 0, exactly enough in double (S1 + n k, S2 + 2 k S1 + n k^2), so that the readers only add
    if (tid < BN && n0 + tid < a.Ncols) {
      float t1 = 0.f, t2 = 0.f;
#pragma unroll 8
      for (int r = 0; r < RPP; ++r) {
        t1 += cs[(r * 2 + 0) * BN + tid];
        t2 += cs[(r * 2 + 1) * BN + tid];
      }
      const double k = static_cast<double>(kshift), n = static_cast<double>(min(BM, Mc - m0));
      const double d1 = static_cast<double>(t1), d2 = static_cast<double>(t2);
      double2* out2 = reinterpret_cast<double2*>(a.partial);
      out2[static_cast<int64_t>(mt) * a.Ncols + n0 + tid] = make_double2(d1 + n * k, d2 + k * (2.0 * d1 + n * k));
    }
    return;
  }
  if (tid < 2 * BN) {
    const int pl = tid / BN, ch = tid % BN;
    float t = 0.f;
#pragma unroll 8
    for (int r = 0; r < RPP; ++r) t += cs[(r * 2 + pl) * BN + ch];
    if (n0 + ch < a.Ncols)
      a.partial[(MODE == 0 ? pl + 1 : pl) * plane +
                (a.partial_rm ? static_cast<int64_t>(mt) * a.Ncols + n0 + ch : static_cast<int64_t>(n0 + ch) * nrows + mt)] = t;
  }
  if (MODE == 0 && tid < BN && n0 + tid < a.Ncols) a.partial[static_cast<int64_t>(n0 + tid) * nrows + mt] = kshift;
}

// ------------------------------------------------------------ weight gradient
struct WgradArgs {
  const void* x;   // gathered activation tensor (as in IgemmArgs, forward gather)
  const void* dy;  // [M][Cout]
  float* out;      // dw [Cout][Ktot], or split partials
  uint32_t x_bytes, dy_bytes;
  int M, Cout, Ktot;
  int H, W, P, Q, PS, Cg, R, S, stride, pad;
  int ctiles;          // column tiles per tap
  int tiles_per_split; // taps * ctiles * output-channel tiles
  int rows_per_split;  // multiple of the K chunk
  int linear;          // 1x1, stride 1, pad 0: gathered row m is pixel m
  int pair;            // stem in bf16: a tap is two filter rows (column pieces 0-3: row 2r, 4-7: row 2r+1)
  int64_t split_stride;
  FastDiv divQ, divP;
  FastDiv div_tps, div_tiles_x, div_ctiles, div_S;  // the tile decode's divisors
  // BNIN kernels (1x1, stride 1): x is the INPUT of a BN+ReLU layer whose output is the convolution's input;
  // relu(x*scale + bias) is applied to the x tile in LDS (as in igemm_kernel).  Null: x is used as is.
  const float *in_gamma, *in_beta, *in_mean, *in_rstd;
  // wgrad3x3_kernel: the padded pixel index space, Gpad = N * (H + 1) * (W + 1) positions
  int Gpad;
  FastDiv div_img, div_w1;  // by (H + 1) * (W + 1) and by W + 1
  int whatif;  // tuning builds only: 1 = leave out the stores of the result, 2 = leave out the MFMAs (what-if timings)
};

template <typename T> struct WgradCfg;
template <> struct WgradCfg<uint16_t> { static constexpr int BKM = 64; };
template <> struct WgradCfg<float> { static constexpr int BKM = 32; };

// LDS tiles of the weight gradient are [k row][column] with rows of RBY = 16 * (columns per 16 bytes ...) bytes,
// filled by LDS-destination loads (RBY/16 lanes per row).  The 16-byte slots of a row are stored permuted,
// slot s of row r at s ^ wgrad_swz(r), so that the fragment reads below touch every bank once:
//   bf16, 128-byte rows: a transposing read's 32 lanes take 64 bytes of 4 consecutive rows -- rows two apart
//                        share their banks, so they swap halves;
//   bf16, 256-byte rows: the same 4 rows all start at bank 0 -- each is rotated by a different 64 bytes;
//   float:               lanes 32-63 read the row 4 below lanes 0-31 -- it is shifted by 128 bytes.
template <typename T, int RBY>
__device__ __forceinline__ int wgrad_swz(int row) {
  if (sizeof(T) == 4) return ((row >> 2) & 1) << 3;
  return RBY == 128 ? ((row >> 1) & 1) << 2 : (row & 3) << 2;
}
// Byte offset, inside a tile, of this lane's first read for the MFMA operand "32 columns from col0 x one k step"
// at k step 0; step kk is KSTEP * kk rows further down.
template <typename T, int RBY>
__device__ __forceinline__ int wgrad_frag_base(int lane, int col0) {
  if (sizeof(T) == 2) {
    // ds_read_b64_tr_b16: within 16 lanes, lane t supplies the address of row t/4, columns 4*(t%4)..+3 and
    // receives column t of rows 0..3.  Two reads (rows +0 and +4) give 8 k values of column lane%32.
    const int g = lane >> 4, t = lane & 15;
    const int krow = 8 * (g >> 1) + (t >> 2);
    const int cb = 2 * (col0 + 16 * (g & 1) + 4 * (t & 3));
    return krow * RBY + (((cb >> 4) ^ wgrad_swz<T, RBY>(krow)) << 4) + (cb & 15);
  }
  const int krow = (lane >> 5) * 4;  // + j, j = 0..3: the permutation only looks at bit 2
  const int cb = 4 * (col0 + (lane & 31));
  return krow * RBY + (((cb >> 4) ^ wgrad_swz<T, RBY>(krow)) << 4) + (cb & 15);
}
template <typename T, int RBY>
__device__ __forceinline__ Vec16 wgrad_read_frag(const unsigned char* tile, int base, int kk) {
  Vec16 v;
  if constexpr (sizeof(T) == 2) {
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
    const unsigned char* p0 = tile + base + kk * 16 * RBY;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p0));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p0 + 4 * RBY));
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      v.h[j] = static_cast<uint16_t>(lo[j]);
      v.h[4 + j] = static_cast<uint16_t>(hi[j]);
    }
  } else {
    const unsigned char* p = tile + base + kk * 8 * RBY;
#pragma unroll
    for (int j = 0; j < 4; ++j) v.f[j] = *reinterpret_cast<const float*>(p + j * RBY);
  }
  return v;
}


// One workgroup: the BMO x BC tile (output channels x input channels of one tap) of one split of the pixel
// range.  2 x 2 waves; per 64-row (32 in float) chunk of pixels the dy and x rows go straight into LDS
// (a ring of chunk buffers, one barrier per chunk, as in igemm_kernel) and are read back transposed.
// NSTAGE: chunk buffers in the ring.  Both operands stream past a workgroup exactly once, from memory that is cold
// inside a training step, so a workgroup's rate is (bytes in flight) / (memory latency): the launch picks the
// deepest ring that the workgroups sharing a compute unit have LDS for (wgrad_stages).
template <typename T, int BMO, int BC, int NSTAGE, bool BNIN = false>
__global__ __launch_bounds__(256) void wgrad_kernel(const WgradArgs a) {
  constexpr int V = 16 / sizeof(T);
  constexpr int BKM = WgradCfg<T>::BKM;
  constexpr int KSTEP = sizeof(T) == 2 ? 16 : 8;
  constexpr int RA = BMO * sizeof(T), RB = BC * sizeof(T);  // row bytes of the two tiles
  constexpr int LA = RA / 16, LB = RB / 16;                  // lanes (16-byte pieces) per row
  constexpr int NA = BKM * LA / 256, NB = BKM * LB / 256;    // load instructions per thread and chunk
  constexpr int NL = NA + NB;
  constexpr int STAGE = BKM * (RA + RB);
  constexpr int TM = BMO / 64, TN = BC / 64;  // 2x2 waves
  static_assert(NA >= 1 && NB >= 1 && 256 % LA == 0 && 256 % LB == 0, "tile shape");
  extern __shared__ __align__(16) unsigned char smem[];

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int wm = wave & 1, wn = wave >> 1;
  // Logical id = (split, output-channel tile, tap, column tile), the last fastest.  All tiles of one
  // split read the same rows of x and dy, so the renumbering keeps them on one XCD and in its L2.
  const int lid = xcd_remap(blockIdx.x, gridDim.x);
  const int split = static_cast<int>(fdiv(static_cast<uint32_t>(lid), a.div_tps)), tile = lid - split * a.tiles_per_split;
  const int tiles_x = a.R * a.S * a.ctiles;
  const int ko_tile = static_cast<int>(fdiv(static_cast<uint32_t>(tile), a.div_tiles_x)), tx = tile - ko_tile * tiles_x;
  const int tap = static_cast<int>(fdiv(static_cast<uint32_t>(tx), a.div_ctiles)), c0 = (tx - tap * a.ctiles) * BC;
  const int r = static_cast<int>(fdiv(static_cast<uint32_t>(tap), a.div_S)), s = tap - r * a.S;
  const int ko0 = ko_tile * BMO;
  const int row_begin = split * a.rows_per_split;
  const int row_end = min(row_begin + a.rows_per_split, a.M);
  const rsrc_words rsX = make_rsrc_words(a.x, a.x_bytes), rsD = make_rsrc_words(a.dy, a.dy_bytes);

  // this thread's rows of a chunk and the 16-byte piece of them it fetches (the slot's permuted partner)
  const int rowa = tid / LA, rowb = tid / LB;
  const int pa = (tid % LA) ^ wgrad_swz<T, RA>(rowa), pb = (tid % LB) ^ wgrad_swz<T, RB>(rowb);
  const bool a_col_ok = ko0 + pa * V < a.Cout;
  const bool b_col_ok = c0 + pb * V < a.Cg;
  // byte offsets of this thread's first rows at m = row_begin; later chunks add a scalar offset
  uint32_t a_off[NA], b_off[NB];
#pragma unroll
  for (int i = 0; i < NA; ++i)
    a_off[i] = a_col_ok ? static_cast<uint32_t>((row_begin + rowa + i * (256 / LA)) * a.Cout + ko0 + pa * V) * sizeof(T) : kOob;
#pragma unroll
  for (int i = 0; i < NB; ++i)
    b_off[i] = b_col_ok ? static_cast<uint32_t>((row_begin + rowb + i * (256 / LB)) * a.PS + c0 + pb * V) * sizeof(T) : kOob;

  typedef __attribute__((address_space(3))) unsigned char* lds_byte_ptr;
  const uint32_t wave_dst = __builtin_amdgcn_readfirstlane(
      static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_byte_ptr)smem)) + static_cast<uint32_t>(wave) * 1024u);
  int cur = 0;  // chunk index of the load cursor
  // Rows past row_end load zeros (no memory access): the last chunk of a split needs no special case.
  auto load_chunk = [&](int stage) __attribute__((always_inline)) {
    const int m_base = row_begin + cur * BKM;
    const int left = row_end - m_base;  // rows of this chunk that belong to the split
    const uint32_t sa = wave_dst + static_cast<uint32_t>(stage) * STAGE, sb = sa + BKM * RA;
    const uint32_t soA = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(cur) * static_cast<uint32_t>(BKM * a.Cout) * sizeof(T));
#pragma unroll
    for (int i = 0; i < NA; ++i)
      buffer_load16_to_lds(rsD, sa + i * 4096, (rowa + i * (256 / LA) < left) ? a_off[i] : kOob, soA);
    if (a.linear) {
      const uint32_t soB = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(cur) * static_cast<uint32_t>(BKM * a.PS) * sizeof(T));
#pragma unroll
      for (int i = 0; i < NB; ++i)
        buffer_load16_to_lds(rsX, sb + i * 4096, (rowb + i * (256 / LB) < left) ? b_off[i] : kOob, soB);
    } else {
#pragma unroll
      for (int i = 0; i < NB; ++i) {
        const int lr = rowb + i * (256 / LB);
        bool ok = b_col_ok && lr < left;
        const uint32_t mm = ok ? static_cast<uint32_t>(m_base + lr) : 0u;
        const uint32_t t = fdiv(mm, a.divQ);
        const int q = static_cast<int>(mm - t * a.Q);
        const uint32_t n = fdiv(t, a.divP);
        const int p = static_cast<int>(t - n * a.P);
        const int ih = p * a.stride - a.pad + (a.pair ? 2 * r + (pb >> 2) : r), iw = q * a.stride - a.pad + s;
        ok = ok && static_cast<unsigned>(ih) < static_cast<unsigned>(a.H) &&
             static_cast<unsigned>(iw) < static_cast<unsigned>(a.W);
        const int pcol = a.pair ? (pb & 3) * V : c0 + pb * V;
        const uint32_t off = static_cast<uint32_t>(((static_cast<int>(n) * a.H + ih) * a.W + iw) * a.PS + pcol) * sizeof(T);
        buffer_load16_to_lds(rsX, sb + i * 4096, ok ? off : kOob, 0u);
      }
    }
    ++cur;
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  int fa_base[TM], fb_base[TN];
#pragma unroll
  for (int i = 0; i < TM; ++i) fa_base[i] = wgrad_frag_base<T, RA>(lane, wm * (BMO / 2) + i * 32);
#pragma unroll
  for (int j = 0; j < TN; ++j) fb_base[j] = BKM * RA + wgrad_frag_base<T, RB>(lane, wn * (BC / 2) + j * 32);
  const int nchunks = (row_end - row_begin + BKM - 1) / BKM;
  constexpr int KK = BKM / KSTEP;
  constexpr int AHEAD = (TM + TN <= 3) ? KK : 1;  // k steps whose fragments are read before the first MFMA
  auto compute = [&](int stage) __attribute__((always_inline)) {
    const unsigned char* st = smem + stage * STAGE;
    Vec16 fa[KK][TM], fb[KK][TN];
    auto read_frags = [&](int kk) __attribute__((always_inline)) {
#pragma unroll
      for (int i = 0; i < TM; ++i) fa[kk][i] = wgrad_read_frag<T, RA>(st, fa_base[i], kk);
#pragma unroll
      for (int j = 0; j < TN; ++j) fb[kk][j] = wgrad_read_frag<T, RB>(st, fb_base[j], kk);
    };
#pragma unroll
    for (int kk = 0; kk < AHEAD; ++kk) read_frags(kk);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      if (kk + AHEAD < KK) {
        read_frags(kk + AHEAD);
        __builtin_amdgcn_sched_barrier(0);
      }
#ifdef RN50_TUNING
      if (a.whatif == 2) {  // the fragments are still read; one add keeps them alive
        acc[0][0][0] += fa[kk][0].f[0] + fb[kk][0].f[0];
        continue;
      }
#endif
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) Mma<T>::run(fa[kk][i], fb[kk][j], acc[i][j]);  // D[ko][c]
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // BNIN: this thread's piece of every x row is the same 16 bytes of channels for the whole launch
  float in_scale[V], in_bias[V];
  if constexpr (BNIN) {
#pragma unroll
    for (int j = 0; j < V; ++j) {
      const int c = min(c0 + pb * V + j, a.Cg - 1);
      bn_coeffs(a.in_gamma[c], a.in_beta[c], a.in_mean[c], a.in_rstd[c], &in_scale[j], &in_bias[j]);
    }
  }
  // the ring of igemm_kernel: loads NSTAGE-1 chunks ahead, one barrier per chunk
#pragma unroll
  for (int c = 0; c < NSTAGE - 1; ++c)
    if (c < nchunks) load_chunk(c);
  int stage = 0;
  for (int kc = 0; kc < nchunks; ++kc) {
    ring_wait<NSTAGE, NL>(nchunks - 1 - kc);
    if (kc + NSTAGE - 1 < nchunks) load_chunk(stage >= 1 ? stage - 1 : NSTAGE - 1);
    if constexpr (BNIN) {
      // every thread transforms, in place, the x vectors of chunk kc that its own loads brought.  Rows past the
      // split's end (loaded as zeros) become relu(bias); their dy rows are zeros, so they add nothing.
#pragma unroll
      for (int i = 0; i < NB; ++i) {
        uint4* p = reinterpret_cast<uint4*>(smem + stage * STAGE + BKM * RA + i * 4096 + tid * 16);
        Vec16 v;
        v.u = *p;
        *p = bn_relu_vector<T>(v, in_scale, in_bias).u;
      }
      lds_writes_then_barrier();
    }
    compute(stage);
    stage = stage == NSTAGE - 1 ? 0 : stage + 1;
  }

  // acc[i][j][v]: ko = i*32 + (v/4)*8 + (lane/32)*4 + v%4, c = j*32 + lane%32
  float* out = a.out + static_cast<int64_t>(split) * a.split_stride;
#ifdef RN50_TUNING
  if (a.whatif == 1 && acc[0][0][0] != 12345.678f) return;
#endif
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int c = c0 + wn * (BC / 2) + j * 32 + (lane & 31);
      if (c >= a.Cg) continue;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int ko = ko0 + wm * (BMO / 2) + i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
        if (ko < a.Cout) out[static_cast<int64_t>(ko) * a.Ktot + tap * a.Cg + c] = acc[i][j][v];
      }
    }
}

// Weight gradient of a 3x3 / stride 1 / padding 1 layer, bf16, all nine taps in one workgroup.
// The reduction index is a PADDED pixel position: every image row gets one more column and every image one more
// row, whose dy and x are zero (never stored: the loads of those positions carry an out-of-range offset and
// write zeros).  In that index space tap (r, s) of position k reads x at k + (r-1)(W+1) + (s-1), a constant shift,
// and every tap that falls off the image lands on a zero position -- so there is nothing to mask: per chunk of 64
// positions the workgroup brings one dy tile [64][64 output channels] and one x run [64 + 2W + 4][64 input
// channels] into LDS and multiplies the dy tile with nine row-shifted windows of the run (transposing reads, the
// slot permutation follows the shifted row) into nine 64x64 accumulator tiles.  Against one gathered tile per tap
// that is 9x fewer dy loads and 9 / (1 + (2W+4)/64) fewer x loads; the reduction grows by (1+1/H)(1+1/W).
// NBX: load passes (32 rows each) of the run; NSTAGE: chunk buffers in the ring (as in wgrad_kernel).
template <int NBX, int NSTAGE>
__global__ __launch_bounds__(256) void wgrad3x3_kernel(const WgradArgs a) {
  typedef uint16_t T;
  constexpr int V = 8, BKM = 64, RBY = 128, KK = 4;
  constexpr int NA = 2, NL = NA + NBX;
  constexpr int STAGE = BKM * RBY + NBX * 4096;
  extern __shared__ __align__(16) unsigned char smem[];

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int wm = wave & 1, wn = wave >> 1;
  // logical id = (split, output-channel tile, input-channel tile): the tiles of a split share its rows
  const int lid = xcd_remap(blockIdx.x, gridDim.x);
  const int split = static_cast<int>(fdiv(static_cast<uint32_t>(lid), a.div_tps)), tile = lid - split * a.tiles_per_split;
  const int ko_tile = static_cast<int>(fdiv(static_cast<uint32_t>(tile), a.div_ctiles));
  const int c0 = (tile - ko_tile * a.ctiles) * 64, ko0 = ko_tile * 64;
  const int row_begin = split * a.rows_per_split;
  const int row_end = min(row_begin + a.rows_per_split, a.Gpad);
  const rsrc_words rsX = make_rsrc_words(a.x, a.x_bytes), rsD = make_rsrc_words(a.dy, a.dy_bytes);

  const int row = tid >> 3;                                  // this thread's row in every 32-row load pass
  const int pc = (tid & 7) ^ wgrad_swz<T, RBY>(row);        // the 16-byte piece of its rows it fetches
  const bool a_col_ok = ko0 + pc * V < a.Cout, b_col_ok = c0 + pc * V < a.Cg;
  const int W1 = a.W + 1, IMG = (a.H + 1) * W1;
  // padded position -> pixel index; ok: the position is a real pixel
  auto pixel_of = [&](int g, bool* ok) __attribute__((always_inline)) {
    const bool in = static_cast<unsigned>(g) < static_cast<unsigned>(a.Gpad);
    const uint32_t gg = in ? static_cast<uint32_t>(g) : 0u;
    const uint32_t n = fdiv(gg, a.div_img), rem = gg - n * static_cast<uint32_t>(IMG);
    const uint32_t y = fdiv(rem, a.div_w1), x = rem - y * static_cast<uint32_t>(W1);
    *ok = in && y < static_cast<uint32_t>(a.H) && x < static_cast<uint32_t>(a.W);
    return static_cast<int>((n * a.H + y) * a.W + x);
  };
  typedef __attribute__((address_space(3))) unsigned char* lds_byte_ptr;
  const uint32_t wave_dst = __builtin_amdgcn_readfirstlane(
      static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_byte_ptr)smem)) + static_cast<uint32_t>(wave) * 1024u);
  int cur = 0;
  auto load_chunk = [&](int stage) __attribute__((always_inline)) {
    const int g0 = row_begin + cur * BKM;
    const uint32_t sa = wave_dst + static_cast<uint32_t>(stage) * STAGE, sb = sa + BKM * RBY;
#pragma unroll
    for (int i = 0; i < NA; ++i) {  // dy: positions of this split only (the others belong to other workgroups)
      const int g = g0 + row + 32 * i;
      bool ok;
      const int pix = pixel_of(g, &ok);
      ok = ok && a_col_ok && g < row_end;
      buffer_load16_to_lds(rsD, sa + i * 4096, ok ? static_cast<uint32_t>(pix * a.Cout + ko0 + pc * V) * 2u : kOob, 0u);
    }
#pragma unroll
    for (int i = 0; i < NBX; ++i) {  // x: the run starts W + 2 positions before the chunk
      const int g = g0 - (a.W + 2) + row + 32 * i;
      bool ok;
      const int pix = pixel_of(g, &ok);
      ok = ok && b_col_ok;
      buffer_load16_to_lds(rsX, sb + i * 4096, ok ? static_cast<uint32_t>(pix * a.PS + c0 + pc * V) * 2u : kOob, 0u);
    }
    ++cur;
  };

  f32x16 acc[9];
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;

  // Fragment addresses.  dy: as in wgrad_kernel.  x: the same transposing read r*(W+1) + s rows further down the
  // run; the slot permutation of a row depends on bit 1 of the row, so it is taken from the shifted row (the
  // reads' +4 and +16*kk rows leave that bit alone).
  const int fa_base = wgrad_frag_base<T, RBY>(lane, wm * 32);
  int fb_base[9];
  {
    const int g4 = lane >> 4, t = lane & 15;
    const int krow = 8 * (g4 >> 1) + (t >> 2);
    const int cb = 2 * (wn * 32 + 16 * (g4 & 1) + 4 * (t & 3));
#pragma unroll
    for (int tap = 0; tap < 9; ++tap) {
      const int kr = krow + (tap / 3) * W1 + (tap % 3);
      fb_base[tap] = BKM * RBY + kr * RBY + (((cb >> 4) ^ wgrad_swz<T, RBY>(kr)) << 4) + (cb & 15);
    }
  }
  const int nchunks = (row_end - row_begin + BKM - 1) / BKM;
  auto compute = [&](int stage) __attribute__((always_inline)) {
    const unsigned char* st = smem + stage * STAGE;
    Vec16 fa[KK], fb[2][KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) fa[kk] = wgrad_read_frag<T, RBY>(st, fa_base, kk);
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) fb[0][kk] = wgrad_read_frag<T, RBY>(st, fb_base[0], kk);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int tap = 0; tap < 9; ++tap) {
      if (tap + 1 < 9) {
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) fb[(tap + 1) & 1][kk] = wgrad_read_frag<T, RBY>(st, fb_base[tap + 1], kk);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) Mma<T>::run(fa[kk], fb[tap & 1][kk], acc[tap]);  // D[ko][c]
      __builtin_amdgcn_sched_barrier(0);
    }
  };
#pragma unroll
  for (int c = 0; c < NSTAGE - 1; ++c)
    if (c < nchunks) load_chunk(c);
  int stage = 0;
  for (int kc = 0; kc < nchunks; ++kc) {
    ring_wait<NSTAGE, NL>(nchunks - 1 - kc);
    if (kc + NSTAGE - 1 < nchunks) load_chunk(stage >= 1 ? stage - 1 : NSTAGE - 1);
    compute(stage);
    stage = stage == NSTAGE - 1 ? 0 : stage + 1;
  }

  // acc[tap][v]: ko = (v/4)*8 + (lane/32)*4 + v%4, c = lane%32 of this wave's 32x32 block
  float* out = a.out + static_cast<int64_t>(split) * a.split_stride;
  const int c = c0 + wn * 32 + (lane & 31);
  if (c < a.Cg) {
#pragma unroll
    for (int tap = 0; tap < 9; ++tap)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int ko = ko0 + wm * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
        if (ko < a.Cout) out[static_cast<int64_t>(ko) * a.Ktot + tap * a.Cg + c] = acc[tap][v];
      }
  }
}

// dw[i] = sum_s partial[s][i].  A workgroup owns 64 float4 outputs; its four waves each sum every
// fourth split (ascending) and the four sums are added in wave order: a fixed order.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ partial, int splits,
                                                            int64_t n, float* __restrict__ out) {
  __shared__ float4 red[4][64];
  const int lane = threadIdx.x & 63, grp = threadIdx.x >> 6;
  const int64_t i = (static_cast<int64_t>(blockIdx.x) * 64 + lane) * 4;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  if (i + 4 <= n) {
#pragma unroll 4
    for (int k = grp; k < splits; k += 4) {
      const float4 v = *reinterpret_cast<const float4*>(partial + k * n + i);
      s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
  } else if (i < n) {
    for (int k = grp; k < splits; k += 4) {
      const float* p = partial + k * n + i;
      s.x += p[0];
      if (i + 1 < n) s.y += p[1];
      if (i + 2 < n) s.z += p[2];
    }
  }
  red[grp][lane] = s;
  __syncthreads();
  if (grp == 0 && i < n) {
    const float4 a = red[0][lane], b = red[1][lane], c = red[2][lane], d = red[3][lane];
    const float4 r = make_float4((a.x + b.x) + (c.x + d.x), (a.y + b.y) + (c.y + d.y), (a.z + b.z) + (c.z + d.z),
                                 (a.w + b.w) + (c.w + d.w));
    if (i + 4 <= n) {
      *reinterpret_cast<float4*>(out + i) = r;
    } else {
      out[i] = r.x;
      if (i + 1 < n) out[i + 1] = r.y;
      if (i + 2 < n) out[i + 2] = r.z;
    }
  }
}

// ------------------------------------------------------- layout helper kernels
// wT[c][t][k] = w[k][t][c]  (t = r*S+s): the B matrix of the data gradient.
template <typename T>
__global__ __launch_bounds__(256) void transpose_kc_kernel(const T* __restrict__ w, T* __restrict__ wT,
                                                           int K, int taps, int C) {
  __shared__ T tile[32][33];
  const int t = blockIdx.z, c0 = blockIdx.x * 32, k0 = blockIdx.y * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  for (int i = ty; i < 32; i += 8) {
    const int k = k0 + i, c = c0 + tx;
    if (k < K && c < C) tile[i][tx] = w[(static_cast<int64_t>(k) * taps + t) * C + c];
  }
  __syncthreads();
  for (int i = ty; i < 32; i += 8) {
    const int c = c0 + i, k = k0 + tx;
    if (k < K && c < C) wT[(static_cast<int64_t>(c) * taps + t) * K + k] = tile[tx][i];
  }
}

// The same transposition for a whole list of weight tensors in one launch (the step's backward pass
// needs every convolution's [Cin][R][S][Cout] form once per step).
constexpr int kTransposeBatchMax = 64;
struct TransposeBatchArgs {
  const void* src;  // arena of [K][taps][C] tensors
  void* dst;        // arena of [C][taps][K] tensors, same offsets
  int num;
  int tile_prefix[kTransposeBatchMax + 1];
  uint32_t offset[kTransposeBatchMax];  // elements
  int K[kTransposeBatchMax], taps[kTransposeBatchMax], C[kTransposeBatchMax];
};
template <typename T>
__global__ __launch_bounds__(256) void transpose_batch_kernel(const TransposeBatchArgs a) {
  __shared__ T tile[32][33];
  int lo = 0, hi = a.num;
  const int b = blockIdx.x;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (a.tile_prefix[mid] <= b) lo = mid; else hi = mid;
  }
  const int K = a.K[lo], taps = a.taps[lo], C = a.C[lo];
  const T* w = static_cast<const T*>(a.src) + a.offset[lo];
  T* wT = static_cast<T*>(a.dst) + a.offset[lo];
  int rem = b - a.tile_prefix[lo];
  const int ct = (C + 31) / 32, kt = (K + 31) / 32;
  const int c0 = (rem % ct) * 32; rem /= ct;
  const int k0 = (rem % kt) * 32;
  const int t = rem / kt;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  for (int i = ty; i < 32; i += 8) {
    const int k = k0 + i, c = c0 + tx;
    if (k < K && c < C) tile[i][tx] = w[(static_cast<int64_t>(k) * taps + t) * C + c];
  }
  __syncthreads();
  for (int i = ty; i < 32; i += 8) {
    const int c = c0 + i, k = k0 + tx;
    if (k < K && c < C) wT[(static_cast<int64_t>(c) * taps + t) * K + k] = tile[tx][i];
  }
}

// Stem input: x [N][H][W][3] -> xp [N][H+6][Wp][4], zero border (3 pixels each side, Wp - W - 3 on the
// right) and zero 4th channel, so that a 7-tap filter row is 8 pixels = 32 contiguous elements.
template <typename T>
__global__ __launch_bounds__(256) void stem_pad_input_kernel(const T* __restrict__ x, T* __restrict__ xp,
                                                             int N, int H, int W, int Hp, int Wp) {
  // grid: (padded row, padded rows, images)
  const int wq = blockIdx.x * 256 + threadIdx.x;
  if (wq >= Wp) return;
  const int hq = blockIdx.y, n = blockIdx.z;
  const int64_t i = (static_cast<int64_t>(n) * Hp + hq) * Wp + wq;
  const int h = hq - 3, w = wq - 3;
  T v[4] = {0, 0, 0, 0};
  if (h >= 0 && h < H && w >= 0 && w < W) {
    const T* s = x + ((static_cast<int64_t>(n) * H + h) * W + w) * 3;
    v[0] = s[0]; v[1] = s[1]; v[2] = s[2];
  }
  T* d = xp + i * 4;
  d[0] = v[0]; d[1] = v[1]; d[2] = v[2]; d[3] = v[3];
}
// Stem weights: w [K][7][7][3] -> wp [K][8][8][4] with zeros in filter row 7, tap column 7 and channel 3.
constexpr int kStemK = 256;  // padded reduction length of the stem: 8 filter rows x 8 taps x 4 channels
template <typename T>
__global__ __launch_bounds__(256) void stem_pad_weight_kernel(const T* __restrict__ w, T* __restrict__ wp, int K) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= K * kStemK) return;
  const int c = i & 3, s = (i >> 2) & 7, r = (i >> 5) & 7, k = i >> 8;
  wp[i] = (c < 3 && s < 7 && r < 7) ? w[((k * 7 + r) * 7 + s) * 3 + c] : static_cast<T>(0);
}
// dw [K][7][7][3] <- dwp [K][8][8][4]
__global__ __launch_bounds__(256) void stem_unpad_dw_kernel(const float* __restrict__ dwp, float* __restrict__ dw, int K) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= K * 147) return;
  const int c = i % 3, s = (i / 3) % 7, r = (i / 21) % 7, k = i / 147;
  dw[i] = dwp[((k * 8 + r) * 8 + s) * 4 + c];
}

// ------------------------------------------------------------------ host side
template <typename K>
static void allow_big_lds(K kernel, int bytes) {
  if (bytes > 48 * 1024) (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}

template <typename T, int BM, int BN, int WM, int WN, int MODE, bool LIN, bool BNIN = false>
static void launch_igemm_mode(IgemmArgs a, const char* tag, int64_t grid, hipStream_t s) {
  constexpr int NT = 64 * WM * WN;
  constexpr int stage = (BM + BN) * 128;
  constexpr int es = static_cast<int>(sizeof(T));
  // the output stage reuses the ring: the tile (in float when a bf16 data gradient adds a second branch) and
  // the column sums of the fused batch norm
  constexpr int out_tile = BM * (BN * 4 + 16);
  constexpr int col_sums = (NT / (BN * es / 16)) * 2 * BN * 4;
  constexpr int out_need = out_tile > col_sums ? out_tile : col_sums;
  static std::once_flag once;
  constexpr int nring = igemm_ring<BM, BN, WM * WN>();
  constexpr int kInTabMax = 8 * 4096;  // input-side BN coefficients: two floats per channel, at most 4096 channels
  std::call_once(once, [] {
    allow_big_lds(igemm_kernel<T, BM, BN, WM, WN, MODE, LIN, BNIN>,
                  (nring * stage > out_need ? nring * stage : out_need) + (BNIN ? kInTabMax : 0));
  });
  // A short reduction never touches the later ring buffers; without them more workgroups fit a CU (the 1x1
  // layers with 64 channels, the largest pixel counts of the net, have a single chunk).
  const int chunks = a.R * a.S * a.cpt;
  const int ring = (chunks < nring ? (chunks < 1 ? 1 : chunks) : nring) * stage;
  int lds = ring > out_need ? ring : out_need;
  if (BNIN) {
    a.in_lds = lds;
    lds += 8 * chunks * (128 / es);
  }
  RN50_LAUNCH(tag, (igemm_kernel<T, BM, BN, WM, WN, MODE, LIN, BNIN>), dim3(static_cast<unsigned>(grid)), dim3(NT), lds, s, a);
}
// The halo kernel (3x3, stride 1, padding 1): LDS bytes of its main loop for an image width, or 0 when the shape
// does not fit it (a run of more than 8 load passes, more LDS than a compute unit has).
static bool igemm_halo_shape(const IgemmArgs& a);
constexpr int kHaloLdsMax = 152 * 1024;  // (the kernel's static arrays come on top; a compute unit has 160 KB)
template <int BM, int BN, int WM, int WN>
static int halo_lds_bytes(int W, int cpt) {
  constexpr int NW = WM * WN, RPL = NW * 8;
  const int passes = (BM + 2 * W + 2 + RPL - 1) / RPL;
  if (passes > 8) return 0;
  const int bytes = (cpt > 1 ? 2 : 1) * passes * RPL * 128 + 3 * BN * 128 + NW * 1024;
  return bytes <= kHaloLdsMax ? bytes : 0;
}
template <typename T, int BM, int BN, int WM, int WN, int MODE>
static void launch_igemm_halo(IgemmArgs a, const char* tag, int64_t grid, int main_lds, hipStream_t s) {
  constexpr int NT = 64 * WM * WN;
  constexpr int es = static_cast<int>(sizeof(T));
  constexpr int out_tile = BM * (BN * 4 + 16);
  constexpr int col_sums = (NT / (BN * es / 16)) * 2 * BN * 4;
  constexpr int out_need = out_tile > col_sums ? out_tile : col_sums;
  static std::once_flag once;
  std::call_once(once, [] { allow_big_lds(igemm_kernel<T, BM, BN, WM, WN, MODE, false, false, true>, kHaloLdsMax); });
  const int lds = main_lds > out_need ? main_lds : out_need;
  RN50_LAUNCH(tag, (igemm_kernel<T, BM, BN, WM, WN, MODE, false, false, true>), dim3(static_cast<unsigned>(grid)), dim3(NT), lds, s, a);
}
template <typename T, int BM, int BN, int WM, int WN>
static void launch_igemm_cfg(IgemmArgs a, const char* tag, hipStream_t s) {
  a.ntn = static_cast<int>(ceil_div(a.Ncols, BN));
  a.nimg = a.M / (a.P * a.Q);
  // stride-2 data gradient: four parity classes of the output pixels, each with its own row tiles
  const int64_t tiles_per_class = ceil_div(static_cast<int64_t>(a.nimg) * ((a.P + 1) / 2) * ((a.Q + 1) / 2), BM);
  const bool classes = a.mode == 1 && a.stride == 2;
  a.mtiles = static_cast<int>(classes ? 4 * tiles_per_class : ceil_div(a.M, BM));
  const int64_t grid = static_cast<int64_t>(a.mtiles) * a.ntn;
  a.partial_rm = a.partial != nullptr && bn_partials_row_major(a.mtiles, a.mode == 1);
  a.div_ntn = make_fastdiv(a.ntn);
  a.linear = a.R == 1 && a.S == 1 && a.stride == 1 && a.pad == 0 && !a.pair && a.H == a.P && a.W == a.Q;
  for (int c = 0; c < 2; ++c) {
    a.div_w[c] = make_fastdiv(classes ? (a.Q - c + 1) >> 1 : a.Q);
    a.div_h[c] = make_fastdiv(classes ? (a.P - c + 1) >> 1 : a.P);
  }
  if (a.linear) {
    if (a.mode == 0 && a.in_gamma) launch_igemm_mode<T, BM, BN, WM, WN, 0, true, true>(a, tag, grid, s);
    else if (a.mode == 0) launch_igemm_mode<T, BM, BN, WM, WN, 0, true>(a, tag, grid, s);
    else launch_igemm_mode<T, BM, BN, WM, WN, 1, true>(a, tag, grid, s);
    return;
  }
  const bool halo_shape = igemm_halo_shape(a);
  if (const int halo_lds = halo_shape ? halo_lds_bytes<BM, BN, WM, WN>(a.W, a.cpt) : 0) {
    if (a.mode == 0) launch_igemm_halo<T, BM, BN, WM, WN, 0>(a, tag, grid, halo_lds, s);
    else launch_igemm_halo<T, BM, BN, WM, WN, 1>(a, tag, grid, halo_lds, s);
    return;
  }
  if (a.mode == 0) launch_igemm_mode<T, BM, BN, WM, WN, 0, false>(a, tag, grid, s);
  else launch_igemm_mode<T, BM, BN, WM, WN, 1, false>(a, tag, grid, s);
}

// Tile per layer shape.  The compiled shapes: rows x columns of the workgroup tile, waves along rows x columns.
struct TileShape {
  int bm, bn, wm, wn;
};
#define RN50_IGEMM_SHAPES(X) X(64, 64, 2, 2) X(128, 64, 2, 2) X(128, 128, 2, 2) X(256, 128, 4, 2)
static bool igemm_shape_compiled(const TileShape& t) {
#define X(BM, BN, WM, WN) if (t.bm == BM && t.bn == BN && t.wm == WM && t.wn == WN) return true;
  RN50_IGEMM_SHAPES(X)
#undef X
  return false;
}
// The tile of a layer shape: M rows (output pixels; of one parity class for a stride-2 data gradient, `live` of
// whose four classes have any taps), Ncols output channels, `chunks` 128-byte steps of the reduction.  The rule
// is fitted to per-layer sweeps of all compiled shapes over ResNet-50's 23 convolution shapes at batch 40 and at
// batch 256 (profiles/conv_tile_sweep_*.txt): the largest tile that still leaves about two workgroups per
// compute unit wins -- larger tiles load fewer operand bytes per flop (the main loop's bound) but a grid that
// does not give every compute unit at least one and a half workgroups leaves the latencies of a workgroup's load -> LDS -> MFMA chain exposed; a
// reduction of one or two chunks has nothing to reuse and takes the smallest tile.
static TileShape igemm_tile(int64_t M, int Ncols, int chunks, bool dgrad, bool strided_dgrad, int live = 4) {
#ifdef RN50_TUNING  // tuning builds only: RN50_IGEMM_TILE=bm,bn,wm,wn forces a compiled tile shape
  if (const char* e = getenv("RN50_IGEMM_TILE")) {
    TileShape f{0, 0, 0, 0};
    if (sscanf(e, "%d,%d,%d,%d", &f.bm, &f.bn, &f.wm, &f.wn) == 4 && igemm_shape_compiled(f)) return f;
  }
#endif
  const int64_t classes = strided_dgrad ? live : 1;
  auto groups = [&](int bm, int bn) { return ceil_div(M, bm) * ceil_div(Ncols, bn) * classes; };
  constexpr int64_t kCover = 384;  // workgroups: one and a half per compute unit (two four-wave workgroups fit each)
  if (chunks <= 1) return TileShape{64, 64, 2, 2};
  if (Ncols > 64) {
    // (the eight-wave tile pays off in the data gradients of the largest layers only)
    if (dgrad && chunks >= 2 && groups(256, 128) >= 4 * kCover) return TileShape{256, 128, 4, 2};
    if (groups(128, 128) >= kCover) return TileShape{128, 128, 2, 2};
  }
  if (chunks >= 8 && groups(128, 64) >= kCover) return TileShape{128, 64, 2, 2};
  return TileShape{64, 64, 2, 2};
}
// The tile of a 3x3 / stride 1 / padding 1 layer, which runs the halo main loop (forward and data gradient
// alike): fitted to sweeps of the compiled shapes over ResNet-50's four such layers at batch 40 and 256.  The
// eight-wave 256x128 tile once it gives three quarters of the compute units a workgroup, else 128x64 while that
// leaves one and a half workgroups per compute unit, else 64x64 (the 128x128 tile never won: its two runs and
// three weight tiles leave room for one workgroup per compute unit only).
static TileShape igemm_halo_tile(int64_t M, int Ncols) {
  auto groups = [&](int bm, int bn) { return ceil_div(M, bm) * ceil_div(Ncols, bn); };
  if (Ncols > 64 && groups(256, 128) >= 192) return TileShape{256, 128, 4, 2};
  if (groups(128, 64) >= 384) return TileShape{128, 64, 2, 2};
  return TileShape{64, 64, 2, 2};
}
// A 3x3 filter with stride 1 and padding 1 (the gathered tensor and the output have the same pixel grid): the
// layers of the halo main loop.  The launch and the callers that size the batch-norm sums (one row per row tile)
// both go through halo_filter / igemm_halo_tile, so they agree on the tile.
static bool halo_filter(int R, int S, int stride, int pad) {
#ifdef RN50_TUNING  // tuning builds only: a forced tile shape, or RN50_NO_HALO, send these layers down the general path
  static const bool off = getenv("RN50_IGEMM_TILE") != nullptr || getenv("RN50_NO_HALO") != nullptr;
  if (off) return false;
#endif
  return R == 3 && S == 3 && stride == 1 && pad == 1;
}
static bool igemm_halo_shape(const IgemmArgs& a) {
  return halo_filter(a.R, a.S, a.stride, a.pad) && !a.pair && a.H == a.P && a.W == a.Q;
}
template <typename T>
static void launch_igemm(const IgemmArgs& a, const char* tag, hipStream_t s) {
  const bool classes = a.mode == 1 && a.stride == 2;
  const int64_t rows = classes ? static_cast<int64_t>(a.M / (a.P * a.Q)) * ((a.P + 1) / 2) * ((a.Q + 1) / 2) : a.M;
  TileShape t = igemm_tile(rows, a.Ncols, a.R * a.S * a.cpt, a.mode == 1, classes, a.R * a.S > 1 ? 4 : 1);
  if (igemm_halo_shape(a)) t = igemm_halo_tile(a.M, a.Ncols);
#define X(BM, BN, WM, WN) if (t.bm == BM && t.bn == BN && t.wm == WM && t.wn == WN) return launch_igemm_cfg<T, BM, BN, WM, WN>(a, tag, s);
  RN50_IGEMM_SHAPES(X)
#undef X
}

struct WgradPlan {
  int bmo, bc, ctiles, splits, rows_per_split;
};
// Tile shape and number of reduction splits.  Inside a training step the weight gradients run beside the
// backward pass on a stream of their own (nothing waits for them until the update), so what counts is the
// compute-unit time and the memory traffic they take from the kernels next to them, not their latency alone:
// the largest tile the channel counts allow (a 64x64 wave tile reads half the LDS bytes per MFMA of a 32x32
// one, a 128x128 workgroup tile loads half the operand bytes per flop of a 64x64 one), and only as many splits
// of the pixel range as give about 192 workgroups (384 for very long reductions), each at least 8 chunks
// long -- every split costs a full-size partial result written and read again by the reduction pass.
// Measured on the whole step at batch 40 (profiles/wgrad_plan_step_time_batch40.txt): 128 to 256 workgroups
// are within 1 % of each other, 64 and 576 lose 13 % and 3 %.
static WgradPlan plan_wgrad(int M, int Cout, int Cg, int taps, int dtype, bool tunable = true) {
  const int bkm = dtype == RN50_BF16 ? 64 : 32;
  WgradPlan best{};
  auto fill = [&](int bmo, int bc, int64_t want_splits, int min_chunks) {
    const int64_t cap = M / (min_chunks * bkm) > 1 ? M / (min_chunks * bkm) : 1;
    int64_t sp = want_splits < 1 ? 1 : (want_splits > cap ? cap : want_splits);
    const int64_t rps = ceil_div(ceil_div(M, sp), bkm) * bkm;
    best.bmo = bmo; best.bc = bc; best.ctiles = static_cast<int>(ceil_div(Cg, bc));
    best.splits = static_cast<int>(ceil_div(M, rps));
    best.rows_per_split = static_cast<int>(rps);
  };
  int target = M > 200000 ? 384 : 192, min_chunks = 8;
  int bmo = Cout >= 128 ? 128 : 64, bc = Cg >= 128 ? 128 : 64;
#ifdef RN50_TUNING  // tuning builds only: RN50_WGRAD_PLAN=bmo,bc,splits or RN50_WGRAD_TARGET=workgroups[,min chunks]
  if (const char* e = tunable ? getenv("RN50_WGRAD_PLAN") : nullptr) {
    int fbmo = 0, fbc = 0, sp = 0;
    if (sscanf(e, "%d,%d,%d", &fbmo, &fbc, &sp) == 3 && (fbmo == 64 || fbmo == 128) && (fbc == 64 || fbc == 128) && sp >= 1) {
      fill(fbmo, fbc, sp, 1);
      return best;
    }
  }
  if (const char* e2 = tunable ? getenv("RN50_WGRAD_TARGET") : nullptr) sscanf(e2, "%d,%d", &target, &min_chunks);
#else
  (void)tunable;
#endif
  const int64_t tiles = static_cast<int64_t>(taps) * ceil_div(Cg, bc) * ceil_div(Cout, bmo);
  fill(bmo, bc, (target + tiles / 2) / tiles, min_chunks);
  return best;
}

// Ring depth of a weight-gradient launch: as many chunk buffers as fit when the compute unit's 160 KB of LDS
// are shared by the workgroups it will hold (grid / 256 compute units, rounded up, at most 3), between 2 and 6.
static int wgrad_stages(int stage_bytes, int64_t grid) {
#ifdef RN50_TUNING  // tuning builds only: RN50_WGRAD_STAGES=n forces the depth
  if (const char* e = getenv("RN50_WGRAD_STAGES")) {
    const int n = atoi(e);
    if (n >= 2 && n <= 6 && n * stage_bytes <= 160 * 1024) return n;
  }
#endif
  int64_t per_cu = ceil_div(grid, 256);
  if (per_cu > 3) per_cu = 3;
  int n = static_cast<int>((156 * 1024 / per_cu) / stage_bytes);
  return n < 2 ? 2 : (n > 6 ? 6 : n);
}
template <typename T, int BMO, int BC, int NSTAGE>
static void launch_wgrad_ring(const WgradArgs& b, dim3 grid, hipStream_t s) {
  constexpr int BKM = WgradCfg<T>::BKM;
  constexpr int lds = NSTAGE * BKM * (BMO + BC) * static_cast<int>(sizeof(T));
  if (b.in_gamma) {  // the input-side BN variant is compiled for the two deepest rings only
    if constexpr (NSTAGE == 2 || NSTAGE == 3) {
      static std::once_flag once_in;
      std::call_once(once_in, [] { allow_big_lds(wgrad_kernel<T, BMO, BC, NSTAGE, true>, lds); });
      RN50_LAUNCH("conv_wgrad", (wgrad_kernel<T, BMO, BC, NSTAGE, true>), grid, dim3(256), lds, s, b);
      return;
    }
  }
  static std::once_flag once;
  std::call_once(once, [] { allow_big_lds(wgrad_kernel<T, BMO, BC, NSTAGE>, lds); });
  RN50_LAUNCH("conv_wgrad", (wgrad_kernel<T, BMO, BC, NSTAGE>), grid, dim3(256), lds, s, b);
}
template <typename T, int BMO, int BC>
static void launch_wgrad_cfg(const WgradArgs& a, int splits, hipStream_t s) {
  constexpr int BKM = WgradCfg<T>::BKM;
  constexpr int stage = BKM * (BMO + BC) * static_cast<int>(sizeof(T));
  WgradArgs b = a;
  b.tiles_per_split = a.R * a.S * a.ctiles * static_cast<int>(ceil_div(a.Cout, BMO));
  b.div_tps = make_fastdiv(b.tiles_per_split);
  b.div_tiles_x = make_fastdiv(a.R * a.S * a.ctiles);
  b.div_ctiles = make_fastdiv(a.ctiles);
  b.div_S = make_fastdiv(a.S);
  const dim3 grid(static_cast<unsigned>(b.tiles_per_split) * splits);
  int stages = wgrad_stages(stage, grid.x);
  if (b.in_gamma) stages = (stages >= 3 && 3 * stage <= 160 * 1024) ? 3 : 2;
  switch (stages) {
    case 2: return launch_wgrad_ring<T, BMO, BC, 2>(b, grid, s);
    case 3: return launch_wgrad_ring<T, BMO, BC, 3>(b, grid, s);
    case 4: return launch_wgrad_ring<T, BMO, BC, 4>(b, grid, s);
    case 5: return launch_wgrad_ring<T, BMO, BC, (stage * 5 <= 160 * 1024 ? 5 : 4)>(b, grid, s);
    default: return launch_wgrad_ring<T, BMO, BC, (stage * 6 <= 160 * 1024 ? 6 : 4)>(b, grid, s);
  }
}

template <typename T>
static void launch_wgrad(WgradArgs a, const WgradPlan& p, float* dw, float* partial, hipStream_t s) {
  a.ctiles = p.ctiles;
  a.rows_per_split = p.rows_per_split;
  a.split_stride = static_cast<int64_t>(a.Cout) * a.Ktot;
  a.out = p.splits > 1 ? partial : dw;
#ifdef RN50_TUNING
  static const int whatif = getenv("RN50_WGRAD_WHATIF") ? atoi(getenv("RN50_WGRAD_WHATIF")) : 0;
  a.whatif = whatif;
#endif
  a.divQ = make_fastdiv(a.Q);
  a.divP = make_fastdiv(a.P);
  if (p.bmo == 128 && p.bc == 128) launch_wgrad_cfg<T, 128, 128>(a, p.splits, s);
  else if (p.bmo == 128) launch_wgrad_cfg<T, 128, 64>(a, p.splits, s);
  else if (p.bc == 128) launch_wgrad_cfg<T, 64, 128>(a, p.splits, s);
  else launch_wgrad_cfg<T, 64, 64>(a, p.splits, s);
  if (p.splits > 1) {
    const int64_t n = a.split_stride;
#ifdef RN50_TUNING  // what-if measurement: the weight gradients without their reduction launches (results wrong)
    static const bool skip_red = getenv("RN50_SKIP_SPLITK_REDUCE") != nullptr;
    if (!skip_red)
#endif
    RN50_LAUNCH("splitk_reduce", splitk_reduce_kernel, dim3(static_cast<unsigned>(ceil_div(ceil_div(n, 4), 64))), dim3(256), 0, s, partial, p.splits, n, dw);
  }
}

static int out_dim(int in, int pad, int k, int stride) { return (in + 2 * pad - k) / stride + 1; }
static bool is_stem(const rn50_conv_desc* d) {
  return d->Cin == 3 && d->R == 7 && d->S == 7 && d->stride == 2 && d->pad == 3;
}
static int esize(int dtype) { return dtype == RN50_BF16 ? 2 : 4; }

static int check_conv(const rn50_conv_desc* d, const char* who) {
  RN50_REQUIRE(d, RN50_ERR_INVALID, "%s: null descriptor", who);
  RN50_REQUIRE(d->N > 0 && d->H > 0 && d->W > 0 && d->Cin > 0 && d->Cout > 0 && d->R > 0 && d->S > 0 &&
                   d->stride > 0 && d->pad >= 0,
               RN50_ERR_INVALID, "%s: non-positive size", who);
  RN50_REQUIRE(d->dtype == RN50_F32 || d->dtype == RN50_BF16, RN50_ERR_INVALID, "%s: dtype %d", who, d->dtype);
  const int V = 16 / esize(d->dtype);
  RN50_REQUIRE(d->H + 2 * d->pad >= d->R && d->W + 2 * d->pad >= d->S, RN50_ERR_INVALID, "%s: filter larger than padded input", who);
  RN50_REQUIRE(d->Cout % V == 0, RN50_ERR_UNSUPPORTED, "%s: Cout=%d is not a multiple of %d", who, d->Cout, V);
  RN50_REQUIRE(d->Cin % V == 0 || is_stem(d), RN50_ERR_UNSUPPORTED,
               "%s: Cin=%d is neither a multiple of %d nor the 7x7/2 pad-3 stem", who, d->Cin, V);
  RN50_REQUIRE(d->pad < d->R && d->pad < d->S, RN50_ERR_UNSUPPORTED, "%s: pad >= filter size", who);
  RN50_REQUIRE(!is_stem(d) || (d->N <= 65535 && d->H + 6 <= 65535), RN50_ERR_UNSUPPORTED,
               "%s: stem with N=%d, H=%d is beyond the padding kernel's launch grid", who, d->N, d->H);
  const int P = out_dim(d->H, d->pad, d->R, d->stride), Q = out_dim(d->W, d->pad, d->S, d->stride);
  const int64_t lim = ((1ll << 31) - 1) / esize(d->dtype);  // byte offsets are 31-bit
  RN50_REQUIRE(static_cast<int64_t>(d->N) * (d->H + 6) * (d->W + 16) * (d->Cin < 4 ? 4 : d->Cin) < lim &&
                   static_cast<int64_t>(d->N) * P * Q * d->Cout < lim &&
                   static_cast<int64_t>(d->Cout) * d->R * d->S * (d->Cin < 4 ? 32 : d->Cin) < lim,
               RN50_ERR_UNSUPPORTED, "%s: a tensor is 2 GiB or larger", who);
  return RN50_OK;
}

// Geometry of the padded stem: 7 "taps" (filter rows) of 32 elements on pixels of 4 channels.
struct StemGeom {
  int Hp, Wp;
  size_t xp_bytes, wp_bytes;
};
static StemGeom stem_geom(const rn50_conv_desc* d) {
  StemGeom g;
  g.Hp = d->H + 6;
  g.Wp = (d->W + 6 + 2 + 3) / 4 * 4;  // room for the 8th (zero-weight) tap, row pitch a multiple of 16 bytes
  g.xp_bytes = align_up(static_cast<size_t>(d->N) * g.Hp * g.Wp * 4 * esize(d->dtype), 256);
  g.wp_bytes = align_up(static_cast<size_t>(d->Cout) * kStemK * esize(d->dtype), 256);
  return g;
}

}  // namespace rn50

using namespace rn50;

// Internal entry points shared with the whole-step driver (declared in step_internal.h).
namespace rn50 {

int conv_desc_check(const rn50_conv_desc* d, const char* who) { return check_conv(d, who); }

void stem_pad_input(const rn50_conv_desc* d, const void* x, void* xp, hipStream_t s) {
  const StemGeom g = stem_geom(d);
  const dim3 grid(static_cast<unsigned>(ceil_div(g.Wp, 256)), g.Hp, d->N);
  if (d->dtype == RN50_BF16)
    RN50_LAUNCH("stem_pad", stem_pad_input_kernel<uint16_t>, grid, dim3(256), 0, s,
                       static_cast<const uint16_t*>(x), static_cast<uint16_t*>(xp), d->N, d->H, d->W, g.Hp, g.Wp);
  else
    RN50_LAUNCH("stem_pad", stem_pad_input_kernel<float>, grid, dim3(256), 0, s,
                       static_cast<const float*>(x), static_cast<float*>(xp), d->N, d->H, d->W, g.Hp, g.Wp);
}

size_t stem_padded_input_bytes(const rn50_conv_desc* d) { return stem_geom(d).xp_bytes; }
size_t stem_padded_weight_bytes(const rn50_conv_desc* d) { return stem_geom(d).wp_bytes; }

static int chunks_per_tap(int channels, int dtype) { return static_cast<int>(ceil_div(channels * esize(dtype), 128)); }
// stride-2 data gradient: four parity classes of ceil(N * ceil(H/2) * ceil(W/2) / bm) row tiles each
static PartialRows class_tile_rows(const rn50_conv_desc* d) {
  const int64_t rows = static_cast<int64_t>(d->N) * ((d->H + 1) / 2) * ((d->W + 1) / 2);
  const int bm = igemm_tile(rows, d->Cin, d->R * d->S * chunks_per_tap(d->Cout, d->dtype), true, true, d->R * d->S > 1 ? 4 : 1).bm;
  return PartialRows{bm, static_cast<int>(4 * ceil_div(rows, bm))};
}
PartialRows fwd_partial_rows(const rn50_conv_desc* d) {
  const int64_t M = static_cast<int64_t>(d->N) * out_dim(d->H, d->pad, d->R, d->stride) * out_dim(d->W, d->pad, d->S, d->stride);
  // the chunk count as the launch computes it (the bf16 stem runs as 4 taps of one chunk, the float stem as 7)
  const int chunks = is_stem(d) ? (d->dtype == RN50_BF16 ? 4 : 7) : d->R * d->S * chunks_per_tap(d->Cin, d->dtype);
  const int bm = halo_filter(d->R, d->S, d->stride, d->pad) ? igemm_halo_tile(M, d->Cout).bm
                                                            : igemm_tile(M, d->Cout, chunks, false, false).bm;
  return PartialRows{bm, static_cast<int>(ceil_div(M, bm))};
}
int64_t dgrad_partial_rows_bound(const rn50_conv_desc* d) {
  const int64_t plain = ceil_div(static_cast<int64_t>(d->N) * d->H * d->W, 64);
  const int64_t classes = 4 * ceil_div(static_cast<int64_t>(d->N) * ((d->H + 1) / 2) * ((d->W + 1) / 2), 64);
  return d->stride == 2 && classes > plain ? classes : plain;
}
PartialRows dgrad_partial_rows(const rn50_conv_desc* d) {
  if (d->stride == 2) return class_tile_rows(d);
  const int64_t M = static_cast<int64_t>(d->N) * d->H * d->W;
  const int bm = halo_filter(d->R, d->S, d->stride, d->pad)
                     ? igemm_halo_tile(M, d->Cin).bm
                     : igemm_tile(M, d->Cin, d->R * d->S * chunks_per_tap(d->Cout, d->dtype), true, false).bm;
  return PartialRows{bm, static_cast<int>(ceil_div(M, bm))};
}

static IgemmArgs stem_igemm_args(const rn50_conv_desc* d, const void* xp, const void* wp, void* y) {
  const StemGeom g = stem_geom(d);
  IgemmArgs a{};
  a.act = xp; a.wgt = wp; a.out = y;
  a.P = out_dim(d->H, 3, 7, 2); a.Q = out_dim(d->W, 3, 7, 2);
  a.M = d->N * a.P * a.Q; a.Ncols = d->Cout; a.Ktot = kStemK;
  a.H = g.Hp; a.W = g.Wp; a.PS = 4; a.stride = 2; a.pad = 0; a.mode = 0; a.S = 1;
  a.cpt = 1;
  // A filter row is 8 padded taps x 4 channels = 32 elements: a whole 128-byte chunk in float, half of
  // one in bf16, where two filter rows share a chunk (4 "taps" of 64 elements; the 8th row is zero weights).
  a.pair = d->dtype == RN50_BF16;
  a.R = a.pair ? 4 : 7;
  a.Cg = a.pair ? 64 : 32;
  a.act_bytes = static_cast<uint32_t>(static_cast<size_t>(d->N) * g.Hp * g.Wp * 4 * esize(d->dtype));
  a.wgt_bytes = static_cast<uint32_t>(static_cast<size_t>(d->Cout) * kStemK * esize(d->dtype));
  return a;
}

// Forward of the stem from an already padded input; wp is scratch for the padded weights.
void stem_fwd_padded(const rn50_conv_desc* d, const void* xp, const void* w, void* wp, void* y, float* bn_partial,
                     hipStream_t s) {
  const int nw = d->Cout * kStemK;
  IgemmArgs a = stem_igemm_args(d, xp, wp, y);
  a.partial = bn_partial;
  if (d->dtype == RN50_BF16) {
    RN50_LAUNCH("stem_pad", stem_pad_weight_kernel<uint16_t>, dim3(ceil_div(nw, 256)), dim3(256), 0, s,
                       static_cast<const uint16_t*>(w), static_cast<uint16_t*>(wp), d->Cout);
    launch_igemm<uint16_t>(a, "conv_fwd", s);
  } else {
    RN50_LAUNCH("stem_pad", stem_pad_weight_kernel<float>, dim3(ceil_div(nw, 256)), dim3(256), 0, s,
                       static_cast<const float*>(w), static_cast<float*>(wp), d->Cout);
    launch_igemm<float>(a, "conv_fwd", s);
  }
}

static int esize(int dtype);
static bool is_stem(const rn50_conv_desc* d);

// The nine-tap weight gradient (wgrad3x3_kernel): bf16, 3x3, stride 1, padding 1, and an image width whose run
// of 2W + 68 rows fits six load passes.  Plan: 64x64 tiles, the padded pixel range split to give about 192
// workgroups (384 for the longest reductions), each at least 8 chunks long (as for wgrad_kernel).
struct Wgrad3x3Plan {
  int nbx;  // load passes of the x run: 3, 4 or 6; 0: the layer does not run this kernel
  int ctiles, kotiles, splits, rows_per_split, gpad;
};
static Wgrad3x3Plan plan_wgrad3x3(const rn50_conv_desc* d) {
  Wgrad3x3Plan p{};
#ifdef RN50_TUNING  // tuning builds only: RN50_NO_WGRAD3X3 sends these layers through the per-tap kernel
  static const bool off = getenv("RN50_NO_WGRAD3X3") != nullptr;
  if (off) return p;
#endif
  if (d->dtype != RN50_BF16 || d->R != 3 || d->S != 3 || d->stride != 1 || d->pad != 1 || is_stem(d)) return p;
  const int need = static_cast<int>(ceil_div(2 * d->W + 68, 32));
  if (need > 6) return p;
  const int64_t gpad = static_cast<int64_t>(d->N) * (d->H + 1) * (d->W + 1);
  if (gpad >= (1ll << 31) - 64) return p;
  p.nbx = need <= 3 ? 3 : (need == 4 ? 4 : 6);
  p.ctiles = static_cast<int>(ceil_div(d->Cin, 64));
  p.kotiles = static_cast<int>(ceil_div(d->Cout, 64));
  p.gpad = static_cast<int>(gpad);
  int target = 384, min_chunks = 8;
  bool always = false;
#ifdef RN50_TUNING  // RN50_WGRAD3X3_TARGET=workgroups,min chunks[,1: every eligible layer]
  if (const char* e = getenv("RN50_WGRAD3X3_TARGET")) {
    int al = 0;
    sscanf(e, "%d,%d,%d", &target, &min_chunks, &al);
    always = al != 0;
  }
#endif
  // Where it pays (per-layer sweeps at batch 40 and 256, profiles/wgrad3x3_nine_tap_sweep_batch40_batch256_bf16.txt): where the
  // per-tap kernel is held to 64-wide tiles by the channel counts, and where its plan leaves a workgroup a
  // reduction of 100 chunks or more (few, long-running workgroups: the wide layers at large batch).  Elsewhere
  // the per-tap kernel's 128x128 tiles (64x64 wave tiles: half the LDS reads per MFMA) are as fast or faster.
  if (!always && d->Cin > 64 && d->Cout > 64 &&
      plan_wgrad(d->N * d->H * d->W, d->Cout, d->Cin, 9, d->dtype).rows_per_split < 100 * 64) {
    p.nbx = 0;
    return p;
  }
  const int64_t tiles = static_cast<int64_t>(p.ctiles) * p.kotiles;
  const int64_t cap = gpad / (min_chunks * 64) > 1 ? gpad / (min_chunks * 64) : 1;
  int64_t sp = (target + tiles / 2) / tiles;
  sp = sp < 1 ? 1 : (sp > cap ? cap : sp);
  const int64_t rps = ceil_div(ceil_div(gpad, sp), 64) * 64;
  p.rows_per_split = static_cast<int>(rps);
  p.splits = static_cast<int>(ceil_div(gpad, rps));
  return p;
}
template <int NBX, int NSTAGE>
static void launch_wgrad3x3_ring(const WgradArgs& a, dim3 grid, hipStream_t s) {
  constexpr int lds = NSTAGE * (64 * 128 + NBX * 4096);
  static std::once_flag once;
  std::call_once(once, [] { allow_big_lds(wgrad3x3_kernel<NBX, NSTAGE>, lds); });
  RN50_LAUNCH("conv_wgrad", (wgrad3x3_kernel<NBX, NSTAGE>), grid, dim3(256), lds, s, a);
}
template <int NBX>
static void launch_wgrad3x3_nbx(const WgradArgs& a, dim3 grid, hipStream_t s) {
  // three chunk buffers where the workgroups sharing a compute unit have the LDS for them, else two
  int64_t per_cu = ceil_div(grid.x, 256);
  if (per_cu > 3) per_cu = 3;
  const bool three = 3 * (64 * 128 + NBX * 4096) * per_cu <= 156 * 1024;
  if (three) launch_wgrad3x3_ring<NBX, 3>(a, grid, s);
  else launch_wgrad3x3_ring<NBX, 2>(a, grid, s);
}
static void launch_wgrad3x3(WgradArgs a, const Wgrad3x3Plan& p, int H, float* dw, float* partial, hipStream_t s) {
  a.ctiles = p.ctiles;
  a.tiles_per_split = p.ctiles * p.kotiles;
  a.rows_per_split = p.rows_per_split;
  a.split_stride = static_cast<int64_t>(a.Cout) * a.Ktot;
  a.out = p.splits > 1 ? partial : dw;
  a.Gpad = p.gpad;
  a.div_tps = make_fastdiv(a.tiles_per_split);
  a.div_ctiles = make_fastdiv(a.ctiles);
  a.div_img = make_fastdiv((H + 1) * (a.W + 1));
  a.div_w1 = make_fastdiv(a.W + 1);
  const dim3 grid(static_cast<unsigned>(a.tiles_per_split) * p.splits);
  if (p.nbx == 3) launch_wgrad3x3_nbx<3>(a, grid, s);
  else if (p.nbx == 4) launch_wgrad3x3_nbx<4>(a, grid, s);
  else launch_wgrad3x3_nbx<6>(a, grid, s);
  if (p.splits > 1) {
    const int64_t n = a.split_stride;
    RN50_LAUNCH("splitk_reduce", splitk_reduce_kernel, dim3(static_cast<unsigned>(ceil_div(ceil_div(n, 4), 64))), dim3(256), 0, s, partial, p.splits, n, dw);
  }
}
static WgradArgs wgrad_args(const rn50_conv_desc* d, const void* x, const void* dy) {
  WgradArgs a{};
  a.x = x; a.dy = dy;
  a.P = out_dim(d->H, d->pad, d->R, d->stride); a.Q = out_dim(d->W, d->pad, d->S, d->stride);
  a.M = d->N * a.P * a.Q; a.Cout = d->Cout; a.Ktot = d->R * d->S * d->Cin;
  a.H = d->H; a.W = d->W; a.PS = d->Cin; a.Cg = d->Cin; a.R = d->R; a.S = d->S; a.stride = d->stride; a.pad = d->pad;
  a.x_bytes = static_cast<uint32_t>(static_cast<size_t>(d->N) * d->H * d->W * d->Cin * esize(d->dtype));
  a.dy_bytes = static_cast<uint32_t>(static_cast<size_t>(a.M) * d->Cout * esize(d->dtype));
  a.linear = d->R == 1 && d->S == 1 && d->stride == 1 && d->pad == 0;
  return a;
}
static WgradArgs stem_wgrad_args(const rn50_conv_desc* d, const void* xp, const void* dy) {
  const StemGeom g = stem_geom(d);
  WgradArgs a{};
  a.x = xp; a.dy = dy;
  a.P = out_dim(d->H, 3, 7, 2); a.Q = out_dim(d->W, 3, 7, 2);
  a.M = d->N * a.P * a.Q; a.Cout = d->Cout; a.Ktot = kStemK;
  a.H = g.Hp; a.W = g.Wp; a.PS = 4; a.S = 1; a.stride = 2; a.pad = 0;
  a.pair = d->dtype == RN50_BF16;  // as in stem_igemm_args
  a.R = a.pair ? 4 : 7;
  a.Cg = a.pair ? 64 : 32;
  a.x_bytes = static_cast<uint32_t>(static_cast<size_t>(d->N) * g.Hp * g.Wp * 4 * esize(d->dtype));
  a.dy_bytes = static_cast<uint32_t>(static_cast<size_t>(a.M) * d->Cout * esize(d->dtype));
  a.linear = 0;
  return a;
}

size_t wgrad_partial_bytes(const rn50_conv_desc* d) {
  const bool stem = is_stem(d);
  const int P = out_dim(d->H, d->pad, d->R, d->stride), Q = out_dim(d->W, d->pad, d->S, d->stride);
  const int M = d->N * P * Q;
  const bool pair = d->dtype == RN50_BF16;
  const WgradPlan p = stem ? plan_wgrad(M, d->Cout, pair ? 64 : 32, pair ? 4 : 7, d->dtype, false)
                           : plan_wgrad(M, d->Cout, d->Cin, d->R * d->S, d->dtype);
  const size_t dw_elems = static_cast<size_t>(d->Cout) * (stem ? kStemK : d->R * d->S * d->Cin);
  const Wgrad3x3Plan p9 = plan_wgrad3x3(d);
  const int splits = p9.nbx ? p9.splits : p.splits;
  size_t b = splits > 1 ? align_up(dw_elems * splits * sizeof(float), 256) : 0;
  if (stem) b += align_up(dw_elems * sizeof(float), 256);  // padded dw
  return b;
}

// Weight gradient; for the stem x must be the padded input.  scratch: wgrad_partial_bytes(d).
void wgrad_run(const rn50_conv_desc* d, const void* x_or_xp, const void* dy, float* dw, void* scratch, hipStream_t s,
               const BnIn* in) {
  const bool stem = is_stem(d);
  WgradArgs a = stem ? stem_wgrad_args(d, x_or_xp, dy) : wgrad_args(d, x_or_xp, dy);
  if (in) { a.in_gamma = in->gamma; a.in_beta = in->beta; a.in_mean = in->mean; a.in_rstd = in->rstd; }
  if (const Wgrad3x3Plan p9 = plan_wgrad3x3(d); p9.nbx && !in) {
    launch_wgrad3x3(a, p9, d->H, dw, static_cast<float*>(scratch), s);
    return;
  }
  const WgradPlan p = plan_wgrad(a.M, a.Cout, a.Cg, a.R * a.S, d->dtype, !stem);  // the stem's tile is fixed (64x64)
  float* partial = static_cast<float*>(scratch);
  float* target = dw;
  if (stem) {
    target = partial;
    partial += align_up(static_cast<size_t>(d->Cout) * kStemK * sizeof(float), 256) / sizeof(float);
  }
  if (d->dtype == RN50_BF16) launch_wgrad<uint16_t>(a, p, target, partial, s);
  else launch_wgrad<float>(a, p, target, partial, s);
  if (stem)
    RN50_LAUNCH("stem_unpad", stem_unpad_dw_kernel, dim3(ceil_div(d->Cout * 147, 256)), dim3(256), 0, s, target, dw, d->Cout);
}

void fwd_run(const rn50_conv_desc* d, const void* x, const void* w, void* y, float* bn_partial, hipStream_t s,
             const char* tag, const BnIn* in) {
  IgemmArgs a{};
  a.act = x; a.wgt = w; a.out = y; a.partial = bn_partial;
  if (in) { a.in_gamma = in->gamma; a.in_beta = in->beta; a.in_mean = in->mean; a.in_rstd = in->rstd; }
  a.P = out_dim(d->H, d->pad, d->R, d->stride); a.Q = out_dim(d->W, d->pad, d->S, d->stride);
  a.M = d->N * a.P * a.Q; a.Ncols = d->Cout; a.Ktot = d->R * d->S * d->Cin;
  a.H = d->H; a.W = d->W; a.PS = d->Cin; a.Cg = d->Cin; a.R = d->R; a.S = d->S; a.stride = d->stride; a.pad = d->pad;
  a.mode = 0;
  a.act_bytes = static_cast<uint32_t>(static_cast<size_t>(d->N) * d->H * d->W * d->Cin * esize(d->dtype));
  a.wgt_bytes = static_cast<uint32_t>(static_cast<size_t>(d->Cout) * a.Ktot * esize(d->dtype));
  a.cpt = static_cast<int>(ceil_div(d->Cin * esize(d->dtype), 128));
  if (d->dtype == RN50_BF16) launch_igemm<uint16_t>(a, tag, s); else launch_igemm<float>(a, tag, s);
}

size_t dgrad_wt_bytes(const rn50_conv_desc* d) {
  return align_up(static_cast<size_t>(d->Cout) * d->R * d->S * d->Cin * esize(d->dtype), 256);
}
void dgrad_transpose_weights(const rn50_conv_desc* d, const void* w, void* wT, hipStream_t s) {
  const dim3 grid(ceil_div(d->Cin, 32), ceil_div(d->Cout, 32), d->R * d->S);
  if (d->dtype == RN50_BF16)
    hipLaunchKernelGGL(transpose_kc_kernel<uint16_t>, grid, dim3(256), 0, s, static_cast<const uint16_t*>(w),
                       static_cast<uint16_t*>(wT), d->Cout, d->R * d->S, d->Cin);
  else
    hipLaunchKernelGGL(transpose_kc_kernel<float>, grid, dim3(256), 0, s, static_cast<const float*>(w),
                       static_cast<float*>(wT), d->Cout, d->R * d->S, d->Cin);
}
void transpose_batch_run(const std::vector<TransposeEntry>& list, int dtype, const void* src_arena, void* dst_arena,
                         hipStream_t s) {
  for (size_t i0 = 0; i0 < list.size(); i0 += kTransposeBatchMax) {
    TransposeBatchArgs a{};
    a.src = src_arena; a.dst = dst_arena;
    a.num = static_cast<int>(list.size() - i0 < kTransposeBatchMax ? list.size() - i0 : kTransposeBatchMax);
    a.tile_prefix[0] = 0;
    for (int i = 0; i < a.num; ++i) {
      const TransposeEntry& e = list[i0 + i];
      a.offset[i] = static_cast<uint32_t>(e.offset);
      a.K[i] = e.K; a.taps[i] = e.taps; a.C[i] = e.C;
      a.tile_prefix[i + 1] = a.tile_prefix[i] + static_cast<int>(ceil_div(e.K, 32) * ceil_div(e.C, 32) * e.taps);
    }
    const int grid = a.tile_prefix[a.num];
    if (dtype == RN50_BF16) RN50_LAUNCH("weight_transpose", transpose_batch_kernel<uint16_t>, dim3(grid), dim3(256), 0, s, a);
    else RN50_LAUNCH("weight_transpose", transpose_batch_kernel<float>, dim3(grid), dim3(256), 0, s, a);
  }
}

// Data gradient from already transposed weights wT [Cin][R][S][Cout].
void dgrad_run(const rn50_conv_desc* d, const void* dy, const void* wT, void* dx, const BnBwdSums* bn, hipStream_t s) {
  IgemmArgs a{};
  a.act = dy; a.wgt = wT; a.out = dx;
  if (bn) {
    a.partial = bn->partial; a.bn_x = bn->x;
    a.bn_gamma = bn->gamma; a.bn_beta = bn->beta; a.bn_mean = bn->mean; a.bn_rstd = bn->rstd;
    a.addend = bn->addend; a.bn_zmask = bn->relu_mask; a.addend_mask = bn->addend ? bn->addend_mask : nullptr;
  }
  a.P = d->H; a.Q = d->W;
  a.H = out_dim(d->H, d->pad, d->R, d->stride); a.W = out_dim(d->W, d->pad, d->S, d->stride);
  a.M = d->N * d->H * d->W; a.Ncols = d->Cin; a.Ktot = d->R * d->S * d->Cout;
  a.PS = d->Cout; a.Cg = d->Cout; a.R = d->R; a.S = d->S; a.stride = d->stride; a.pad = d->pad;
  a.mode = 1;
  a.act_bytes = static_cast<uint32_t>(static_cast<size_t>(d->N) * a.H * a.W * d->Cout * esize(d->dtype));
  a.wgt_bytes = static_cast<uint32_t>(static_cast<size_t>(d->Cin) * a.Ktot * esize(d->dtype));
  a.cpt = static_cast<int>(ceil_div(d->Cout * esize(d->dtype), 128));
  if (d->dtype == RN50_BF16) launch_igemm<uint16_t>(a, "conv_dgrad", s); else launch_igemm<float>(a, "conv_dgrad", s);
}

}  // namespace rn50

extern "C" size_t conv_fwd_workspace_bytes(const rn50_conv_desc* d) {
  if (!d || check_conv(d, "conv_fwd_workspace_bytes")) return 0;
  if (!is_stem(d)) return 0;
  const StemGeom g = stem_geom(d);
  return g.xp_bytes + g.wp_bytes;
}
extern "C" size_t conv_dgrad_workspace_bytes(const rn50_conv_desc* d) {
  if (!d || check_conv(d, "conv_dgrad_workspace_bytes")) return 0;
  return dgrad_wt_bytes(d);
}
extern "C" size_t conv_wgrad_workspace_bytes(const rn50_conv_desc* d) {
  if (!d || check_conv(d, "conv_wgrad_workspace_bytes")) return 0;
  return wgrad_partial_bytes(d) + (is_stem(d) ? stem_geom(d).xp_bytes : 0);
}

extern "C" int conv_fwd(const rn50_conv_desc* d, const void* x, const void* w, void* y, void* workspace,
                        size_t workspace_bytes, void* stream) {
  clear_error();
  if (int rc = check_conv(d, "conv_fwd")) return rc;
  RN50_REQUIRE(x && w && y, RN50_ERR_INVALID, "conv_fwd: null pointer");
  RN50_REQUIRE(aligned16(x) && aligned16(w) && aligned16(y) && aligned16(workspace), RN50_ERR_ALIGN,
               "conv_fwd: pointer not 16-byte aligned");
  const size_t need = conv_fwd_workspace_bytes(d);
  RN50_REQUIRE(workspace_bytes >= need && (need == 0 || workspace), RN50_ERR_WORKSPACE,
               "conv_fwd: workspace %zu < %zu bytes", workspace_bytes, need);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (is_stem(d)) {
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    stem_pad_input(d, x, ws, s);
    stem_fwd_padded(d, ws, w, ws + stem_geom(d).xp_bytes, y, nullptr, s);
  } else {
    fwd_run(d, x, w, y, nullptr, s);
  }
  return launch_status("conv_fwd");
}

extern "C" int conv_dgrad(const rn50_conv_desc* d, const void* dy, const void* w, void* dx, void* workspace,
                          size_t workspace_bytes, void* stream) {
  clear_error();
  if (int rc = check_conv(d, "conv_dgrad")) return rc;
  RN50_REQUIRE(!is_stem(d) && d->Cin % (16 / esize(d->dtype)) == 0, RN50_ERR_UNSUPPORTED,
               "conv_dgrad: the 3-channel stem has no data gradient here (the network input needs none)");
  RN50_REQUIRE(d->stride == 1 || d->stride == 2, RN50_ERR_UNSUPPORTED, "conv_dgrad: stride %d", d->stride);
  RN50_REQUIRE(dy && w && dx && workspace, RN50_ERR_INVALID, "conv_dgrad: null pointer");
  RN50_REQUIRE(aligned16(dy) && aligned16(w) && aligned16(dx) && aligned16(workspace), RN50_ERR_ALIGN,
               "conv_dgrad: pointer not 16-byte aligned");
  RN50_REQUIRE(workspace_bytes >= dgrad_wt_bytes(d), RN50_ERR_WORKSPACE, "conv_dgrad: workspace %zu < %zu bytes",
               workspace_bytes, dgrad_wt_bytes(d));
  hipStream_t s = static_cast<hipStream_t>(stream);
  dgrad_transpose_weights(d, w, workspace, s);
  dgrad_run(d, dy, workspace, dx, nullptr, s);
  return launch_status("conv_dgrad");
}

extern "C" int conv_wgrad(const rn50_conv_desc* d, const void* x, const void* dy, float* dw, void* workspace,
                          size_t workspace_bytes, void* stream) {
  clear_error();
  if (int rc = check_conv(d, "conv_wgrad")) return rc;
  RN50_REQUIRE(x && dy && dw, RN50_ERR_INVALID, "conv_wgrad: null pointer");
  RN50_REQUIRE(aligned16(x) && aligned16(dy) && aligned16(dw) && aligned16(workspace), RN50_ERR_ALIGN,
               "conv_wgrad: pointer not 16-byte aligned");
  const size_t need = conv_wgrad_workspace_bytes(d);
  RN50_REQUIRE(workspace_bytes >= need && (need == 0 || workspace), RN50_ERR_WORKSPACE,
               "conv_wgrad: workspace %zu < %zu bytes", workspace_bytes, need);
  hipStream_t s = static_cast<hipStream_t>(stream);
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  if (is_stem(d)) {
    stem_pad_input(d, x, ws, s);
    wgrad_run(d, ws, dy, dw, ws + stem_geom(d).xp_bytes, s);
  } else {
    wgrad_run(d, x, dy, dw, ws, s);
  }
  return launch_status("conv_wgrad");
}

// ---- fused batch-norm sums (the BN side is in bn.hip)
extern "C" size_t conv_bn_sums_bytes(const rn50_conv_desc* d) {
  if (!d || check_conv(d, "conv_bn_sums_bytes")) return 0;
  // one row per output tile of at least 64 pixels; forward three float planes or, row-major, two doubles per
  // channel and row; two planes backward
  const int P = out_dim(d->H, d->pad, d->R, d->stride), Q = out_dim(d->W, d->pad, d->S, d->stride);
  const size_t fwd = static_cast<size_t>(ceil_div(static_cast<int64_t>(d->N) * P * Q, 64)) * 4 * d->Cout;
  const size_t bwd = static_cast<size_t>(dgrad_partial_rows_bound(d)) * 2 * d->Cin;
  return align_up((fwd > bwd ? fwd : bwd) * sizeof(float), 256);
}

extern "C" int conv_fwd_bn_sums(const rn50_conv_desc* d, const void* x, const void* w, void* y, float* sums,
                                size_t sums_bytes, void* workspace, size_t workspace_bytes, void* stream) {
  clear_error();
  if (int rc = check_conv(d, "conv_fwd_bn_sums")) return rc;
  RN50_REQUIRE(x && w && y && sums, RN50_ERR_INVALID, "conv_fwd_bn_sums: null pointer");
  RN50_REQUIRE(aligned16(x) && aligned16(w) && aligned16(y) && aligned16(workspace) && aligned16(sums),
               RN50_ERR_ALIGN, "conv_fwd_bn_sums: pointer not 16-byte aligned");
  const size_t need = conv_fwd_workspace_bytes(d);
  RN50_REQUIRE(workspace_bytes >= need && (need == 0 || workspace), RN50_ERR_WORKSPACE,
               "conv_fwd_bn_sums: workspace %zu < %zu bytes", workspace_bytes, need);
  RN50_REQUIRE(sums_bytes >= conv_bn_sums_bytes(d), RN50_ERR_WORKSPACE, "conv_fwd_bn_sums: sums %zu < %zu bytes",
               sums_bytes, conv_bn_sums_bytes(d));
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (is_stem(d)) {
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    stem_pad_input(d, x, ws, s);
    stem_fwd_padded(d, ws, w, ws + stem_geom(d).xp_bytes, y, sums, s);
  } else {
    fwd_run(d, x, w, y, sums, s);
  }
  return launch_status("conv_fwd_bn_sums");
}

extern "C" int conv_dgrad_bn_sums(const rn50_conv_desc* d, const void* dy, const void* w, void* dx,
                                  const void* addend, const uint8_t* addend_mask, const void* bn_x,
                                  const uint8_t* relu_mask, const float* gamma, const float* beta,
                                  const float* save_mean, const float* save_rstd, float* sums,
                                  size_t sums_bytes, void* workspace, size_t workspace_bytes, void* stream) {
  clear_error();
  if (int rc = check_conv(d, "conv_dgrad_bn_sums")) return rc;
  RN50_REQUIRE(!is_stem(d) && d->Cin % (16 / esize(d->dtype)) == 0, RN50_ERR_UNSUPPORTED,
               "conv_dgrad_bn_sums: the 3-channel stem has no data gradient here");
  RN50_REQUIRE(d->stride == 1 || d->stride == 2, RN50_ERR_UNSUPPORTED, "conv_dgrad_bn_sums: stride %d", d->stride);
  RN50_REQUIRE(dy && w && dx && workspace && bn_x && gamma && beta && save_mean && save_rstd && sums,
               RN50_ERR_INVALID, "conv_dgrad_bn_sums: null pointer");
  RN50_REQUIRE(aligned16(dy) && aligned16(w) && aligned16(dx) && aligned16(workspace) && aligned16(bn_x) &&
                   aligned16(sums) && aligned16(addend) && aligned16(gamma) && aligned16(beta) &&
                   aligned16(save_mean) && aligned16(save_rstd),
               RN50_ERR_ALIGN, "conv_dgrad_bn_sums: pointer not 16-byte aligned");
  RN50_REQUIRE(workspace_bytes >= dgrad_wt_bytes(d), RN50_ERR_WORKSPACE,
               "conv_dgrad_bn_sums: workspace %zu < %zu bytes", workspace_bytes, dgrad_wt_bytes(d));
  RN50_REQUIRE(sums_bytes >= conv_bn_sums_bytes(d), RN50_ERR_WORKSPACE, "conv_dgrad_bn_sums: sums %zu < %zu bytes",
               sums_bytes, conv_bn_sums_bytes(d));
  RN50_REQUIRE(!addend_mask || addend, RN50_ERR_INVALID, "conv_dgrad_bn_sums: addend_mask without addend");
  hipStream_t s = static_cast<hipStream_t>(stream);
  dgrad_transpose_weights(d, w, workspace, s);
  const BnBwdSums bn{bn_x, gamma, beta, save_mean, save_rstd, sums, addend, relu_mask, addend_mask};
  dgrad_run(d, dy, workspace, dx, &bn, s);
  return launch_status("conv_dgrad_bn_sums");
}

// ---- convolution whose input is the output of a BN+ReLU layer that is applied on the fly
static int check_bn_in(const rn50_conv_desc* d, const char* who) {
  RN50_REQUIRE(d->R == 1 && d->S == 1 && d->stride == 1 && d->pad == 0, RN50_ERR_UNSUPPORTED,
               "%s: only 1x1 convolutions with stride 1 and no padding take their input through a BN layer", who);
  RN50_REQUIRE(d->Cin <= 4096, RN50_ERR_UNSUPPORTED, "%s: Cin=%d > 4096", who, d->Cin);
  return RN50_OK;
}
extern "C" int conv_fwd_bn_in(const rn50_conv_desc* d, const void* x, const float* in_gamma, const float* in_beta,
                              const float* in_mean, const float* in_rstd, const void* w, void* y, float* sums,
                              size_t sums_bytes, void* stream) {
  clear_error();
  if (int rc = check_conv(d, "conv_fwd_bn_in")) return rc;
  if (int rc = check_bn_in(d, "conv_fwd_bn_in")) return rc;
  RN50_REQUIRE(x && w && y && in_gamma && in_beta && in_mean && in_rstd, RN50_ERR_INVALID, "conv_fwd_bn_in: null pointer");
  RN50_REQUIRE(aligned16(x) && aligned16(w) && aligned16(y) && aligned16(sums), RN50_ERR_ALIGN,
               "conv_fwd_bn_in: pointer not 16-byte aligned");
  RN50_REQUIRE(!sums || sums_bytes >= conv_bn_sums_bytes(d), RN50_ERR_WORKSPACE, "conv_fwd_bn_in: sums %zu < %zu bytes",
               sums_bytes, conv_bn_sums_bytes(d));
  const BnIn in{in_gamma, in_beta, in_mean, in_rstd};
  fwd_run(d, x, w, y, sums, static_cast<hipStream_t>(stream), "conv_fwd", &in);
  return launch_status("conv_fwd_bn_in");
}
extern "C" int conv_wgrad_bn_in(const rn50_conv_desc* d, const void* x, const float* in_gamma, const float* in_beta,
                                const float* in_mean, const float* in_rstd, const void* dy, float* dw, void* workspace,
                                size_t workspace_bytes, void* stream) {
  clear_error();
  if (int rc = check_conv(d, "conv_wgrad_bn_in")) return rc;
  if (int rc = check_bn_in(d, "conv_wgrad_bn_in")) return rc;
  RN50_REQUIRE(x && dy && dw && in_gamma && in_beta && in_mean && in_rstd, RN50_ERR_INVALID, "conv_wgrad_bn_in: null pointer");
  RN50_REQUIRE(aligned16(x) && aligned16(dy) && aligned16(dw) && aligned16(workspace), RN50_ERR_ALIGN,
               "conv_wgrad_bn_in: pointer not 16-byte aligned");
  const size_t need = conv_wgrad_workspace_bytes(d);
  RN50_REQUIRE(workspace_bytes >= need && (need == 0 || workspace), RN50_ERR_WORKSPACE,
               "conv_wgrad_bn_in: workspace %zu < %zu bytes", workspace_bytes, need);
  const BnIn in{in_gamma, in_beta, in_mean, in_rstd};
  wgrad_run(d, x, dy, dw, workspace, static_cast<hipStream_t>(stream), &in);
  return launch_status("conv_wgrad_bn_in");
}
