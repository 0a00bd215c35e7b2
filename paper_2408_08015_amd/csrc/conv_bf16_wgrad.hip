// Weight gradient of the 3x3 'same' stride-1 convolution on NHWC bf16 tensors (and, with one
// tap, of a 1x1 convolution) on the gfx950 matrix cores:
//
//   dW[co][tap][ci] = sum_p dy[p][co] * x[p + shift(tap)][ci]      p = flattened (image, row, column)
//
// a product whose contraction index (the pixel) is the ROW index of both operands in memory.  The
// tiles go to LDS exactly as they lie in memory ([pixel][channel], `buffer_load_dwordx4 ... lds`,
// no registers in between) and the MFMA operands are read with ds_read_b64_tr_b16, which hands
// lane i of a group of 16 the four pixels of channel i from a 4-pixel x 16-channel block: the
// transposition costs nothing.  Each 16-byte chunk sits at chunk ^ ((pixel & 3) << 2) of its row,
// so the four rows such a read touches fall into different banks.
//
// Block = 8 wavefronts (4 x 2) = 256 output channels x 64*TN input channels of ONE tap over a
// range of pixels (split-K: taps x splits blocks fill the chip); K-tile = 48 pixels, three LDS
// stages, loads issued two to three K-tiles ahead and waited for with explicit vmcnt counts; one
// s_barrier per K-tile, placed before the last third of its MFMAs.  The x operand of a tap is the
// tile shifted by the tap's offset; rows whose shifted pixel lies outside the image are requested
// beyond the buffer's extent, which the hardware turns into zeros.  Every block writes its fp32
// partial [co][ci]; a reduction kernel adds the splits into G in a fixed order.
#include "device_utils.h"
#include "kernels_bf16.h"
#include "prof.h"

#include <cstdlib>
#include <type_traits>

namespace ast {

namespace {

struct WgArgs {
  const bf16_t* dy;  // [P][Cout]
  const bf16_t* x;   // [P][Cin]
  float* part;       // [splits][taps][Cout][Cin]
  float* bias_part;  // [splits][Cout] or NULL: column sums of dy (the bias gradient) per split
  float* acc_out;    // grouped launches (one split): [Cout][Cin] that the product is ADDED to, instead of `part`
  float* bias_acc;   // ... and [Cout] that the column sums of dy are added to (or NULL)
  int P, H, W, Cout, Cin;
  int taps;          // 9 (3x3) or 1
  int k_per_split;   // pixels per split, a multiple of the K-tile
  int tiles_m, tiles_n;
  int step_q, step_r;  // K-tile / W, K-tile % W: how (row, column) of a pixel advance per K-tile
  unsigned x_bytes;
};

constexpr int WG_BK = 48;                 // pixels per K-tile
constexpr int WG_A_BYTES = WG_BK * 512;   // dy tile: 256 channels per row
constexpr unsigned WG_OOB = 0x80000000u;

typedef __attribute__((address_space(3))) void wg_lds_void;
typedef short wg_short4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) wg_short4 wg_lds_short4;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t wg_rsrc(const void* p, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, bytes, 0x00020000);
}
__device__ __forceinline__ void wg_wait_vmcnt0() { __builtin_amdgcn_s_waitcnt(0x0f70); }
__device__ __forceinline__ void wg_wait_vmcnt5() { __builtin_amdgcn_s_waitcnt(0x0f75); }
__device__ __forceinline__ void wg_wait_vmcnt6() { __builtin_amdgcn_s_waitcnt(0x0f76); }
__device__ __forceinline__ void wg_wait_vmcnt10() { __builtin_amdgcn_s_waitcnt(0x0f7a); }
__device__ __forceinline__ void wg_wait_vmcnt12() { __builtin_amdgcn_s_waitcnt(0x0f7c); }
__device__ __forceinline__ void wg_wait_lds() { __builtin_amdgcn_s_waitcnt(0xc07f); }
__device__ __forceinline__ void wg_fence() { asm volatile("" ::: "memory"); }

// eight pixels (k) of one channel for the MFMA: two transposed reads of four pixels each
__device__ __forceinline__ bf16x8 wg_read_tr(const unsigned char* smem, int off) {
  const wg_short4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((wg_lds_short4*)(smem + off));
  const wg_short4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((wg_lds_short4*)(smem + off + 4 * 512));
  typedef short short8 __attribute__((ext_vector_type(8)));
  const short8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, v);
}

// block: 256 output channels x 64*TN input channels, 8 wavefronts as 4 x 2; wavefront tile 64 x 32*TN.
// (Four wavefronts of 128 x 128 with the accumulators in the accumulation registers - a third less LDS
// read traffic per MFMA - were measured: 190-210 us against 137-149 us for the 256 -> 256 channel layer.)
template <int TN>
__device__ __forceinline__ void conv_wgrad_tr_body(const WgArgs& g, int bid) {  // bid: block of this product
  constexpr int NW = 8;
  constexpr int TM = 16 / NW;
  constexpr int NT = NW * 64;                        // threads
  constexpr int NCI = 64 * TN;                       // input channels per block
  constexpr int BPITCH = NCI * 2;                    // bytes per pixel row of the x tile
  constexpr int B_BYTES = TN == 4 ? WG_BK * 512 : 16 * 1024;  // TN == 2: 12 KB of rows + 4 KB never read
  constexpr int STAGE = WG_A_BYTES + B_BYTES;
  constexpr int AQ = 24 / NW;                        // dy-tile load instructions per wavefront and K-tile
  constexpr int BQ = TN == 4 ? 24 / NW : 2;          // x-tile load instructions per wavefront and K-tile
  constexpr int NL = AQ + BQ;                        // loads per wavefront and K-tile
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int lrow = lane & 31, lgrp = lane >> 5;
  const int tile_n = bid % g.tiles_n; bid /= g.tiles_n;
  const int tile_m = bid % g.tiles_m; bid /= g.tiles_m;
  const int tap = bid % g.taps, split = bid / g.taps;
  const int co0 = tile_m * 256, ci0 = tile_n * NCI;
  const int k_begin = split * g.k_per_split, k_end = min(k_begin + g.k_per_split, g.P);
  const int nk = (k_end - k_begin + WG_BK - 1) / WG_BK;
  const int W = g.W, H = g.H;
  const int du = g.taps == 9 ? tap / 3 - 1 : 0, dv = g.taps == 9 ? tap % 3 - 1 : 0;

  // dy is read up to the end of the split's range only: rows past it come back as zeros
  const __amdgpu_buffer_rsrc_t rdy = wg_rsrc(g.dy, (unsigned)k_end * (unsigned)g.Cout * 2u);
  const __amdgpu_buffer_rsrc_t rx = wg_rsrc(g.x, g.x_bytes);

  // ---- what this lane copies.  dy tile: instruction q of the wavefront fills rows 2*(wave+8q),
  // +1 (512 bytes each); the lane's row and 16-byte chunk, un-swizzled, give its source address.
  unsigned avoff[AQ];
#pragma unroll
  for (int q = 0; q < AQ; ++q) {
    const int row = 2 * (wave + NW * q) + (lane >> 5);
    const int lc = (lane & 31) ^ ((row & 3) << 2);
    const int co = co0 + lc * 8;
    avoff[q] = co < g.Cout ? (unsigned)(((k_begin + row) * g.Cout + co) * 2) : WG_OOB;
  }
  // x tile: rows of BPITCH bytes; per instruction the lane's row, its pixel's (row, column) in the
  // image (advanced per K-tile) and the linear byte offset of the SHIFTED pixel's chunk
  int b_y[BQ], b_x[BQ];
  unsigned b_lin[BQ];
  bool b_on[BQ];
#pragma unroll
  for (int q = 0; q < BQ; ++q) {
    const int row = TN == 4 ? 2 * (wave + NW * q) + (lane >> 5) : 4 * (wave + NW * q) + (lane >> 4);
    const int pc = TN == 4 ? (lane & 31) : (lane & 15);
    const int lc = pc ^ ((row & 3) << 2);
    const int ci = ci0 + lc * 8;
    const int p = k_begin + row;
    const int rem = p % (H * W);
    b_y[q] = rem / W;
    b_x[q] = rem - b_y[q] * W;
    b_on[q] = row < WG_BK && ci < g.Cin;
    b_lin[q] = (unsigned)(((p + du * W + dv) * g.Cin + ci) * 2);  // may be "negative" while the row is invalid
  }
  auto issue = [&](int stage_off) __attribute__((always_inline)) {
#pragma unroll
    for (int q = 0; q < AQ; ++q) {
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rdy, (wg_lds_void*)(smem + stage_off + (wave + NW * q) * 1024), 16,
                                               avoff[q], 0, 0, 0);
      avoff[q] += (unsigned)(WG_BK * 2) * (unsigned)g.Cout;  // (an offset beyond the extent stays beyond it)
    }
#pragma unroll
    for (int q = 0; q < BQ; ++q) {
      const bool ok = b_on[q] && (unsigned)(b_y[q] + du) < (unsigned)H && (unsigned)(b_x[q] + dv) < (unsigned)W;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (wg_lds_void*)(smem + stage_off + WG_A_BYTES + (wave + NW * q) * 1024),
                                               16, ok ? b_lin[q] : WG_OOB, 0, 0, 0);
      b_lin[q] += (unsigned)(WG_BK * 2) * (unsigned)g.Cin;
      int nx = b_x[q] + g.step_r, ny = b_y[q] + g.step_q;
      if (nx >= W) { nx -= W; ++ny; }
      while (ny >= H) ny -= H;
      b_x[q] = nx;
      b_y[q] = ny;
    }
  };

  // ---- operand fragments.  Lane l of a transposed read supplies the address of 4 channels of
  // one pixel: 16-lane group b = l / 16 covers channels 16*(b & 1) .. +15 and pixels 8*(b >> 1) .. +3
  // of the fragment, lane j = l % 16 of the group pixel j / 4, channels 4*(j % 4) .. +3.
  const int j16 = lane & 15, blk = lane >> 4;
  const int krow = 8 * (blk >> 1) + (j16 >> 2);
  const int swz = ((j16 >> 2) & 3) << 2;  // = (pixel & 3) << 2 for every step and half
  int aoff[TM], boff[TN];
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int col = wm * (32 * TM) + i * 32 + 16 * (blk & 1) + 4 * (j16 & 3);
    aoff[i] = krow * 512 + (((col >> 3) ^ swz) << 4) + (col & 7) * 2;
  }
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int col = wn * (32 * TN) + j * 32 + 16 * (blk & 1) + 4 * (j16 & 3);
    boff[j] = WG_A_BYTES + krow * BPITCH + (((col >> 3) ^ swz) << 4) + (col & 7) * 2;
  }

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // Bias gradient = column sums of dy: the blocks of the centre tap (first input-channel tile)
  // add up the dy tile they hold in LDS anyway.  Thread -> one 16-byte chunk (8 channels) of three
  // (six) pixel rows per K-tile; the 16 (8) row groups are added in a fixed order at the end.
  const bool do_bias = (g.bias_part != nullptr || g.bias_acc != nullptr) && tap == (g.taps == 9 ? 4 : 0) && tile_n == 0;
  float bsum[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) bsum[e] = 0.f;
  auto bias_rows = [&](int stage_off) __attribute__((always_inline)) {
    constexpr int RPT = WG_BK / (NT / 32);  // rows per thread
    const int c = tid & 31, rg = tid >> 5;
#pragma unroll
    for (int rr = 0; rr < RPT; ++rr) {
      const int row = rg * RPT + rr;
      const uint4 v = *reinterpret_cast<const uint4*>(smem + stage_off + row * 512 + ((c ^ ((row & 3) << 2)) << 4));
      const uint32_t w4[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        bsum[2 * e] += __uint_as_float(w4[e] << 16);
        bsum[2 * e + 1] += __uint_as_float(w4[e] & 0xffff0000u);
      }
    }
  };

  bf16x8 fa[2][TM], fb[2][TN];
  auto read_frags = [&](int par, int stage_off, int ks) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[par][i] = wg_read_tr(smem, stage_off + aoff[i] + ks * 16 * 512);
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      // (the second half of the pair is 4 rows further: wg_read_tr adds 4 * 512, the x tile's rows
      // are BPITCH apart)
      const int o = stage_off + boff[j] + ks * 16 * BPITCH;
      const wg_short4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((wg_lds_short4*)(smem + o));
      const wg_short4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((wg_lds_short4*)(smem + o + 4 * BPITCH));
      typedef short short8 __attribute__((ext_vector_type(8)));
      const short8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
      fb[par][j] = __builtin_bit_cast(bf16x8, v);
    }
  };
  auto mma = [&](int par) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[par][i], fb[par][j], acc[i][j], 0, 0, 0);
  };

  // ---- prologue: three K-tiles in flight.  Every wavefront issues the loads of every K-tile up to
  // three beyond the (even) number the loop runs over - past the split's range they come back as
  // zeros or are never multiplied - so the wait counts are the same in every step, and the loop body
  // has no branch that carries an accumulator or an operand fragment (a conditional second half, or
  // conditional operand reads, cost a register copy per accumulator and iteration).
  const int nk2 = (nk + 1) & ~1;
  issue(0);
  issue(STAGE);
  issue(2 * STAGE);
  if (NL == 6) wg_wait_vmcnt12(); else wg_wait_vmcnt10();  // the first tile is in LDS
  static_assert(NL == 5 || NL == 6, "wait counts");
  wg_fence();
  __builtin_amdgcn_s_barrier();
  wg_fence();
  read_frags(0, 0, 0);

  // ---- one K-tile: three 16-pixel steps; `par` = fragment set that holds step 0
  auto tile_body = [&](auto par_t, int st, int st_next) __attribute__((always_inline)) {
    constexpr int P0 = decltype(par_t)::value;
    if (do_bias) bias_rows(st);
    read_frags(P0 ^ 1, st, 1);
    __builtin_amdgcn_sched_barrier(0);
    mma(P0);
    __builtin_amdgcn_sched_barrier(0);
    read_frags(P0, st, 2);
    __builtin_amdgcn_sched_barrier(0);
    mma(P0 ^ 1);
    __builtin_amdgcn_sched_barrier(0);
    // every LDS read of this K-tile has returned; of the two K-tiles in flight the older has to have landed
    wg_wait_lds();
    if (NL == 6) wg_wait_vmcnt6(); else wg_wait_vmcnt5();
    wg_fence();
    __builtin_amdgcn_s_barrier();
    wg_fence();
    issue(st);  // three K-tiles ahead, into the stage this K-tile has released
    read_frags(P0 ^ 1, st_next, 0);
    __builtin_amdgcn_sched_barrier(0);
    mma(P0);
    __builtin_amdgcn_sched_barrier(0);
  };
  int st = 0;
  for (int kt = 0; kt < nk2; kt += 2) {
    const int st1 = st == 2 * STAGE ? 0 : st + STAGE;
    const int st2 = st1 == 2 * STAGE ? 0 : st1 + STAGE;
    tile_body(std::integral_constant<int, 0>{}, st, st1);
    tile_body(std::integral_constant<int, 1>{}, st1, st2);
    st = st2;
  }
  // the loads issued past the last K-tile still target the stages
  wg_wait_vmcnt0();
  wg_wait_lds();
  wg_fence();
  __builtin_amdgcn_s_barrier();
  wg_fence();

  if (do_bias) {  // (uniform over the block) [16 row groups][256 channels] through LDS, summed in order
    wg_wait_lds();
    wg_fence();
    __builtin_amdgcn_s_barrier();
    wg_fence();
    float* sb = reinterpret_cast<float*>(smem);
    const int c = tid & 31, rg = tid >> 5;
#pragma unroll
    for (int e = 0; e < 8; ++e) sb[rg * 256 + c * 8 + e] = bsum[e];
    __syncthreads();
    if (tid < 256 && co0 + tid < g.Cout) {
      float t = 0.f;
#pragma unroll
      for (int r = 0; r < NT / 32; ++r) t += sb[r * 256 + tid];
      if (g.bias_acc) g.bias_acc[co0 + tid] += t;  // (this block alone owns these channels)
      else g.bias_part[(size_t)split * g.Cout + co0 + tid] = t;
    }
  }

  // ---- the partial: accumulator register r of lane l is D[8*(r/4) + 4*(l/32) + r%4][l%32]
  const bool accumulate = g.acc_out != nullptr;  // every output entry belongs to this block alone: a plain add
  float* out = accumulate ? g.acc_out : g.part + ((size_t)(split * g.taps + tap) * g.Cout) * g.Cin;
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int ci = ci0 + wn * (32 * TN) + j * 32 + lrow;
      if (ci >= g.Cin) continue;
      wg_fence();  // one tile's loads and stores at a time (hoisted together they would not fit in registers)
      float old[16];
      if (accumulate) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int co = co0 + wm * (32 * TM) + i * 32 + 8 * (r >> 2) + 4 * lgrp + (r & 3);
          old[r] = co < g.Cout ? out[(size_t)co * g.Cin + ci] : 0.f;
        }
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int co = co0 + wm * (32 * TM) + i * 32 + 8 * (r >> 2) + 4 * lgrp + (r & 3);
        if (co < g.Cout) out[(size_t)co * g.Cin + ci] = accumulate ? old[r] + acc[i][j][r] : acc[i][j][r];
      }
    }
}

__global__ __launch_bounds__(512) void conv_wgrad_tr_kernel_n256(WgArgs g) {
  conv_wgrad_tr_body<4>(g, (int)xcd_grouped(blockIdx.x, gridDim.x));
}
__global__ __launch_bounds__(512) void conv_wgrad_tr_kernel_n128(WgArgs g) {
  conv_wgrad_tr_body<2>(g, (int)xcd_grouped(blockIdx.x, gridDim.x));
}

// Many products in one launch (the weight gradients of all linear layers of a stage: nothing later in
// a backward pass depends on them): block -> (product, block of that product) through a table;
// every product runs unsplit and adds its result straight into the gradient arena.
__global__ __launch_bounds__(512) void wgrad_grouped_kernel(const WgArgs* __restrict__ tasks,
                                                            const unsigned short* __restrict__ block_task,
                                                            const unsigned* __restrict__ task_block0, int block_base) {
  const int b = block_base + (int)blockIdx.x;  // (a launch may cover a sub-range of the table's blocks)
  const int t = block_task[b];
  const WgArgs g = tasks[t];
  conv_wgrad_tr_body<4>(g, b - (int)task_block0[t]);
}
constexpr size_t wg_lds_bytes(int tn) { return 3 * (size_t)(WG_A_BYTES + (tn == 4 ? WG_BK * 512 : 16 * 1024)); }

bool wg_attr_ok() {
  static int ok = -1;
  if (ok < 0) {
    ok = hipFuncSetAttribute((const void*)conv_wgrad_tr_kernel_n256, hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)wg_lds_bytes(4)) == hipSuccess &&
                 hipFuncSetAttribute((const void*)wgrad_grouped_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                     (int)wg_lds_bytes(4)) == hipSuccess &&

                 hipFuncSetAttribute((const void*)conv_wgrad_tr_kernel_n128, hipFuncAttributeMaxDynamicSharedMemorySize,
                                     (int)wg_lds_bytes(2)) == hipSuccess
             ? 1
             : 0;
    if (!ok) (void)hipGetLastError();
  }
  return ok == 1;
}

constexpr int kWgBlocks = 256;  // compute units of the device the split count aims at

inline long wg_cdiv(long a, long b) { return (a + b - 1) / b; }

}  // namespace

// Number of K-splits (= partial copies) of the transposed-read weight-gradient kernel: the blocks
// of all taps and channel tiles together fill the chip once; every split is a whole number of
// K-tiles.  Depends on the shape only (the workspace is sized with it before a device is touched).
int conv_wgrad_tr_splits(long P, int Cin, int Cout, int taps) {
  const long tiles = (long)taps * wg_cdiv(Cout, 256) * wg_cdiv(Cin, Cin > 128 ? 256 : 128);
  long s = kWgBlocks / tiles;
  if (s < 1) s = 1;
  const long max_s = wg_cdiv(P, 4 * WG_BK);  // at least four K-tiles per split
  if (s > max_s) s = max_s;
  const long kps = wg_cdiv(wg_cdiv(P, s), WG_BK) * WG_BK;
  return (int)wg_cdiv(P, kps);
}

bool conv_wgrad_tr_supported(int N, int H, int W, int Cin, int Cout, int k) {
  const long P = (long)N * H * W;
  return (k == 3 || k == 1) && Cin % 8 == 0 && Cout % 8 == 0 && P * Cin * 2 < (1L << 31) && P * Cout * 2 < (1L << 31) &&
         P >= WG_BK && wg_attr_ok();
}

// part[split][tap][Cout][Cin] = the splits' partial weight gradients (conv_wgrad_tr_splits() of them);
// bias_part[split][Cout] (may be NULL) = the splits' column sums of dy
void conv_wgrad_tr_bf16(hipStream_t st, const bf16_t* dy, const bf16_t* x, float* part, float* bias_part, int N, int H,
                        int W, int Cin, int Cout, int k) {
  WgArgs g = {};
  g.dy = dy; g.x = x; g.part = part; g.bias_part = bias_part;
  g.P = N * H * W; g.H = H; g.W = W; g.Cout = Cout; g.Cin = Cin;
  g.taps = k * k;
  const int splits = conv_wgrad_tr_splits(g.P, Cin, Cout, g.taps);
  g.k_per_split = (int)(wg_cdiv(wg_cdiv(g.P, splits), WG_BK) * WG_BK);
  g.tiles_m = (int)wg_cdiv(Cout, 256);
  g.step_q = WG_BK / W; g.step_r = WG_BK % W;
  g.x_bytes = (unsigned)((size_t)g.P * Cin * 2);
  if (Cin > 128) {
    g.tiles_n = (int)wg_cdiv(Cin, 256);
    KLAUNCH_NAMED("conv_wgrad_tr_kernel_n256", conv_wgrad_tr_kernel_n256,
                  dim3((unsigned)(splits * g.taps * g.tiles_m * g.tiles_n)), dim3(512), wg_lds_bytes(4), st, g);
  } else {
    g.tiles_n = (int)wg_cdiv(Cin, 128);
    KLAUNCH_NAMED("conv_wgrad_tr_kernel_n128", conv_wgrad_tr_kernel_n128,
                  dim3((unsigned)(splits * g.taps * g.tiles_m * g.tiles_n)), dim3(512), wg_lds_bytes(2), st, g);
  }
}

// ---- grouped launch: descriptors are built on the host (wgrad_group_task), copied to the device by
// the caller once, and launched as one grid.
size_t wgrad_group_task_bytes() { return sizeof(WgArgs); }
bool wgrad_group_supported(size_t rows, int Cin, int Cout) {
  return Cin % 8 == 0 && Cout % 8 == 0 && rows >= (size_t)WG_BK && rows * Cin * 2 < (1ul << 31) && rows * Cout * 2 < (1ul << 31) &&
         wg_attr_ok();
}
// Writes the descriptor of GW[Cout][Cin] += dy[rows][Cout]^T x[rows][Cin] (and Gb[Cout] += column sums of dy,
// if Gb) to `task_out`; returns the number of blocks the product takes.
int wgrad_group_task(void* task_out, const bf16_t* dy, const bf16_t* x, float* GW, float* Gb, size_t rows, int Cin, int Cout) {
  WgArgs g = {};
  g.dy = dy; g.x = x; g.acc_out = GW; g.bias_acc = Gb;
  g.P = (int)rows; g.H = 1; g.W = 1; g.Cout = Cout; g.Cin = Cin;
  g.taps = 1;
  g.k_per_split = (int)(wg_cdiv((long)rows, WG_BK) * WG_BK);
  g.tiles_m = (int)wg_cdiv(Cout, 256);
  g.tiles_n = (int)wg_cdiv(Cin, 256);
  g.step_q = 0; g.step_r = 0;   // (one tap: no pixel is ever outside the image)
  g.x_bytes = (unsigned)(rows * Cin * 2);
  *static_cast<WgArgs*>(task_out) = g;
  return g.tiles_m * g.tiles_n;
}
void wgrad_group_launch(hipStream_t st, const void* tasks_dev, const unsigned short* block_task_dev,
                        const unsigned* task_block0_dev, int block_base, int nblocks) {
  if (nblocks <= 0) return;
  KLAUNCH(wgrad_grouped_kernel, dim3((unsigned)nblocks), dim3(512), wg_lds_bytes(4), st,
          static_cast<const WgArgs*>(tasks_dev), block_task_dev, task_block0_dev, block_base);
}

}  // namespace ast
