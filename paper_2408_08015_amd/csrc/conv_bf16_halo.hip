// 3x3 'same' stride-1 convolution of NHWC bf16 images as an implicit GEMM on the gfx950 matrix
// cores (v_mfma_f32_32x32x16_bf16), for the dense-convolution stage (forward, and the input
// gradient: the same product on the output gradient with point-reflected taps).
//
//   y[p][n] = sum_{tap, c} x[p + shift(tap)][c] * w[n][tap][c]     p = flattened (image, row, column)
//
// Block = 8 wavefronts = one tile of 256 consecutive pixels x BN output channels (BN = 256 or 128).
// For every 64-channel slice of the input the block stages its 256 pixels TOGETHER WITH THEIR HALO
// (W + 1 pixels before and after, in flattened order) in LDS once, and multiplies all nine taps from that
// copy: the pixel operand of tap (u, v) is the same LDS tile read (u*W + v) rows further down, so
// the input crosses the L2 -> LDS path once per slice and not once per tap.  Pixels whose shifted
// neighbour lies outside the image (where the flattened shift would wrap into the neighbouring
// row or image) get a zero operand by a per-lane select.
//
// Global -> LDS copies are `buffer_load_dwordx4 ... lds` (no registers in between): a wavefront
// instruction fills 1 KB = 8 rows of 128 bytes; the 16-byte chunk a lane fetches is chosen so that
// the tile lands XOR-swizzled (chunk ^= (row >> 1) & 7), which makes the MFMA operand reads (16
// consecutive rows, one chunk, at ANY row offset) free of bank conflicts.  The weight tile (BN
// rows x 64) of each (tap, slice) is double-buffered, the halo tile of the next slice is fetched
// during taps 0..5 of the current one.  One s_barrier per K-tile, placed before the last quarter of the
// tile's MFMAs, which then cover the latency of the first operand reads of the next tile; the
// loads are waited for with explicit s_waitcnt vmcnt counts (the compiler does not track them).
//
// The MFMA takes the weights as its first operand, so an accumulator register group holds four
// consecutive output channels of one pixel: the epilogue packs them into 8-byte LDS writes and the
// tile leaves through LDS in 16-byte rows (bias, ReLU, the mask of a ReLU in front folded in).
#include "device_utils.h"
#include "kernels_bf16.h"
#include "prof.h"

#include <type_traits>

namespace ast {

namespace {

struct HaloArgs {
  const bf16_t* x;     // [M][C] pixels
  const bf16_t* w;     // [N][9][C]
  bf16_t* y;           // [M][N]
  const float* bias;   // [N] or NULL
  const bf16_t* mask;  // [M][N] or NULL: the output is zeroed where mask <= 0
  int M, H, W, C, N;
  int act;
  int tiles_n;
  unsigned x_bytes, w_bytes;
};

constexpr int HALO_BM = 256;             // pixels per tile
constexpr int HALO_AQ = 6;               // halo groups (8 rows) per wavefront: 48 KB per buffer, W <= 63
constexpr int HALO_A_BYTES = HALO_AQ * 8 * 1024;
constexpr unsigned HALO_OOB = 0x80000000u;  // buffer offset beyond every extent: the load returns zeros

typedef __attribute__((address_space(3))) void lds_void;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t halo_rsrc(const void* p, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, bytes, 0x00020000);
}
// s_waitcnt with only the vector-memory counter / only the LDS counter set (gfx9 encoding:
// vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8)
__device__ __forceinline__ void wait_vmcnt0() { __builtin_amdgcn_s_waitcnt(0x0f70); }
__device__ __forceinline__ void wait_vmcnt1() { __builtin_amdgcn_s_waitcnt(0x0f71); }
__device__ __forceinline__ void wait_vmcnt2() { __builtin_amdgcn_s_waitcnt(0x0f72); }
__device__ __forceinline__ void wait_vmcnt4() { __builtin_amdgcn_s_waitcnt(0x0f74); }
__device__ __forceinline__ void wait_lds() { __builtin_amdgcn_s_waitcnt(0xc07f); }
__device__ __forceinline__ void fence() { asm volatile("" ::: "memory"); }

template <int TN>  // wavefront tile: 64 pixels x 32*TN channels; block 4 x 2 wavefronts
__device__ __forceinline__ void conv3x3_halo_body(const HaloArgs& g) {
  constexpr int BN = 64 * TN;
  constexpr int B_BYTES = BN * 128;
  constexpr int BQ = BN / 64;  // weight groups (8 rows) per wavefront and K-tile
  static_assert(BQ == 2 || BQ == 4, "the prologue waits for BQ loads");
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  unsigned char* const sA = smem;                     // two halo buffers
  unsigned char* const sB = smem + 2 * HALO_A_BYTES;  // two weight buffers

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int lrow = lane & 31, lgrp = lane >> 5;
  const int bid = (int)xcd_grouped(blockIdx.x, gridDim.x);
  const int tile_m = bid / g.tiles_n, tile_n = bid - tile_m * g.tiles_n;
  const int m0 = tile_m * HALO_BM, n0 = tile_n * BN;
  const int W = g.W, C = g.C;
  const int NS = C >> 6;

  const __amdgpu_buffer_rsrc_t rx = halo_rsrc(g.x, g.x_bytes), rw = halo_rsrc(g.w, g.w_bytes);
  // byte offsets of this lane's chunk in each group it copies (without the channel-slice / tap part)
  unsigned avoff[HALO_AQ], bvoff[BQ];
#pragma unroll
  for (int q = 0; q < HALO_AQ; ++q) {
    const int row = (wave + 8 * q) * 8 + (lane >> 3);
    const int lc = (lane & 7) ^ ((row >> 1) & 7);
    const int p = m0 - (W + 1) + row;
    avoff[q] = (p >= 0 && p < g.M) ? (unsigned)((p * C + lc * 8) * 2) : HALO_OOB;
  }
#pragma unroll
  for (int q = 0; q < BQ; ++q) {
    const int row = (wave * BQ + q) * 8 + (lane >> 3);
    const int lc = (lane & 7) ^ ((row >> 1) & 7);
    const int n = n0 + row;
    bvoff[q] = n < g.N ? (unsigned)((n * 9 * C + lc * 8) * 2) : HALO_OOB;
  }
  auto issue_A = [&](int q, int slice, int buf) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (lds_void*)(sA + buf * HALO_A_BYTES + (wave + 8 * q) * 1024), 16,
                                             avoff[q], (unsigned)(slice * 128), 0, 0);
  };
  auto issue_B1 = [&](int q, unsigned soff, int buf) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, (lds_void*)(sB + buf * B_BYTES + (wave * BQ + q) * 1024), 16, bvoff[q],
                                             soff, 0, 0);
  };
  auto issue_B = [&](int tap, int slice, int buf) {
    const unsigned soff = (unsigned)((tap * C + slice * 64) * 2);
    issue_B1(0, soff, buf);
    issue_B1(1, soff, buf);
    if (BQ == 4) {
      issue_B1(BQ - 2, soff, buf);
      issue_B1(BQ - 1, soff, buf);
    }
  };

  // which taps of this lane's two pixels read inside the image
  bool vy0[2], vy2[2], vx0[2], vx2[2];
  {
    const int HW = g.H * W;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int p = m0 + wm * 64 + i * 32 + lrow;
      const int rem = p % HW;
      const int yy = rem / W, xx = rem - yy * W;
      vy0[i] = yy >= 1; vy2[i] = yy <= g.H - 2; vx0[i] = xx >= 1; vx2[i] = xx <= W - 2;
    }
  }
  // LDS byte offsets of the operand fragments.  Rows 32 apart share their swizzle term, so the
  // second pixel tile and the channel tiles of a wavefront are immediate offsets (i * 4096,
  // j * 4096) from one address, and the four 16-deep steps of a K-tile are that address with
  // bits 5 and 6 flipped.
  const int arow0 = wm * 64 + lrow;  // halo row of pixel tile 0 at shift 0
  const int lg16 = lgrp << 4;
  auto a_base = [&](int row) -> int { return (row << 7) | (((row << 3) & 0x70) ^ lg16); };
  const int brow0 = wn * (32 * TN) + lrow;
  const int b_base = (brow0 << 7) | (((brow0 << 3) & 0x70) ^ lg16);
  floatx16 acc[TN][2];
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[j][i][r] = 0.f;

  bf16x8 fa[2][2], fb[2][TN];
  // aoff / boff: fragment offsets of the tile at step 0, the buffer's offset included
  auto read_frags = [&](int par, int aoff, int boff, int ks) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
      fa[par][i] = *reinterpret_cast<const bf16x8*>(smem + ((aoff ^ (ks << 5)) + i * 4096));
#pragma unroll
    for (int j = 0; j < TN; ++j)
      fb[par][j] = *reinterpret_cast<const bf16x8*>(smem + ((boff ^ (ks << 5)) + j * 4096));
  };
  const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
  auto mma = [&](int par, bool v0, bool v1) {
    const bf16x8 a0 = v0 ? fa[par][0] : zero8, a1 = v1 ? fa[par][1] : zero8;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      acc[j][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[par][j], a0, acc[j][0], 0, 0, 0);
      acc[j][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[par][j], a1, acc[j][1], 0, 0, 0);
    }
  };

  // ---------------- prologue: halo of slice 0, weight tiles 0 and 1
#pragma unroll
  for (int q = 0; q < HALO_AQ; ++q) issue_A(q, 0, 0);
  issue_B(0, 0, 0);
  issue_B(1, 0, 1);
  if (BQ == 4) wait_vmcnt4(); else wait_vmcnt2();  // everything but the second weight tile
  fence();
  __builtin_amdgcn_s_barrier();
  fence();
  read_frags(0, a_base(arow0), 2 * HALO_A_BYTES + b_base, 0);

  // ---------------- main loop: slices of 64 channels, nine taps each
  auto slice_body = [&](auto has_next_t, int s) {
    constexpr bool HN = decltype(has_next_t)::value;
    const int abuf = (s & 1) * HALO_A_BYTES, abuf_next = HALO_A_BYTES - abuf;
    // the fragment addresses are recomputed per tap (a handful of integer operations) instead of
    // being kept in registers across the slice loop: `vary` hides from the compiler that they repeat
    int vary;
    asm volatile("v_mov_b32 %0, 0" : "=v"(vary));
    const int arow = arow0 + vary;
#pragma unroll
    for (int t = 0; t < 9; ++t) {
      const int ty = t / 3, tx = t - ty * 3;
      const int par_b = (s + t) & 1;  // = (9 s + t) & 1
      const int aoff = a_base(arow + ty * W + tx) + abuf;
      const int boff = 2 * HALO_A_BYTES + par_b * B_BYTES + b_base;
      const bool v0 = (ty == 0 ? vy0[0] : ty == 2 ? vy2[0] : true) && (tx == 0 ? vx0[0] : tx == 2 ? vx2[0] : true);
      const bool v1 = (ty == 0 ? vy0[1] : ty == 2 ? vy2[1] : true) && (tx == 0 ? vx0[1] : tx == 2 ? vx2[1] : true);
      read_frags(1, aoff, boff, 1);
      mma(0, v0, v1);
      read_frags(0, aoff, boff, 2);
      mma(1, v0, v1);
      read_frags(1, aoff, boff, 3);
      mma(0, v0, v1);
      // Every LDS read of this tile has returned: after the barrier its weight buffer (and, behind
      // tap 8, the halo buffer) may be overwritten.  The loads of the next weight tile were issued
      // one tile ago, followed by at most one halo load, which may stay in flight.
      wait_lds();
      if (HN && t >= 1 && t <= HALO_AQ) wait_vmcnt1(); else wait_vmcnt0();
      fence();
      __builtin_amdgcn_s_barrier();
      fence();
      if (HN || t < 7) {  // weight tile two steps ahead, into the buffer just released
        const int t2 = (t + 2) % 9;
        issue_B(t2, s + (t + 2) / 9, par_b);
      }
      if (HN && t < HALO_AQ) issue_A(t, s + 1, (s + 1) & 1);
      if (HN || t < 8) {
        const int t1 = (t + 1) % 9;
        read_frags(0, a_base(arow + (t1 / 3) * W + t1 % 3) + (t < 8 ? abuf : abuf_next),
                   2 * HALO_A_BYTES + (par_b ^ 1) * B_BYTES + b_base, 0);
      }
      mma(1, v0, v1);
    }
  };
  for (int s = 0; s + 1 < NS; ++s) slice_body(std::true_type{}, s);
  slice_body(std::false_type{}, NS - 1);

  // ---------------- epilogue: tile -> LDS as bf16 [256][BN] (rows padded by 16 bytes) -> global
  constexpr int CP = BN * 2 + 16;
  fence();
  __builtin_amdgcn_s_barrier();
  fence();
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      const int nl = wn * (32 * TN) + j * 32 + 8 * r4 + 4 * lgrp;  // four consecutive channels
      float4 bv = make_float4(0.f, 0.f, 0.f, 0.f);
      if (g.bias && n0 + nl < g.N) {  // the channel count is a multiple of 8; the bias need not be 16-byte aligned
        const float* bp = g.bias + n0 + nl;
        bv = make_float4(bp[0], bp[1], bp[2], bp[3]);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        float v0 = acc[j][i][4 * r4 + 0] + bv.x, v1 = acc[j][i][4 * r4 + 1] + bv.y;
        float v2 = acc[j][i][4 * r4 + 2] + bv.z, v3 = acc[j][i][4 * r4 + 3] + bv.w;
        if (g.act == ACT_RELU) { v0 = fmaxf(v0, 0.f); v1 = fmaxf(v1, 0.f); v2 = fmaxf(v2, 0.f); v3 = fmaxf(v3, 0.f); }
        uint2 pk;
        pk.x = (uint32_t)f2bf(v0) | ((uint32_t)f2bf(v1) << 16);
        pk.y = (uint32_t)f2bf(v2) | ((uint32_t)f2bf(v3) << 16);
        *reinterpret_cast<uint2*>(smem + (wm * 64 + i * 32 + lrow) * CP + nl * 2) = pk;
      }
    }
  __syncthreads();
  constexpr int CPR = BN / 8;  // 16-byte chunks per row
  for (int idx = tid; idx < HALO_BM * CPR; idx += 512) {
    const int row = idx / CPR, ch = idx - row * CPR;
    const long m = (long)m0 + row;
    const int n = n0 + ch * 8;
    if (m < g.M && n < g.N) {
      uint4 v = *reinterpret_cast<const uint4*>(smem + row * CP + ch * 16);
      if (g.mask) {
        const uint4 o = *reinterpret_cast<const uint4*>(g.mask + m * g.N + n);
        uint32_t* vw = reinterpret_cast<uint32_t*>(&v);
        const uint32_t* ow = reinterpret_cast<const uint32_t*>(&o);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          // bf16 > 0: sign clear and not zero
          const uint32_t lo = ow[k] & 0xffffu, hi = ow[k] >> 16;
          const uint32_t keep = ((lo != 0u && lo < 0x8000u) ? 0x0000ffffu : 0u) | ((hi != 0u && hi < 0x8000u) ? 0xffff0000u : 0u);
          vw[k] &= keep;
        }
      }
      *reinterpret_cast<uint4*>(g.y + m * g.N + n) = v;
    }
  }
}

// (plain kernels around the templated body: the host pass of the compiler drops the stub of a
// kernel template with this body without a diagnostic)
__global__ __launch_bounds__(512) void conv3x3_halo_kernel_n256(HaloArgs g) { conv3x3_halo_body<4>(g); }
__global__ __launch_bounds__(512) void conv3x3_halo_kernel_n128(HaloArgs g) { conv3x3_halo_body<2>(g); }

template <int TN>
bool launch_halo(hipStream_t st, HaloArgs& g) {
  constexpr int BN = 64 * TN;
  constexpr size_t lds = 2 * HALO_A_BYTES + 2 * BN * 128;
  static_assert(lds >= (size_t)HALO_BM * (BN * 2 + 16), "the output tile must fit in the same LDS");
  auto kern = TN == 4 ? conv3x3_halo_kernel_n256 : conv3x3_halo_kernel_n128;
  static int ok = -1;  // dynamic LDS beyond 64 KiB has to be allowed per kernel
  if (ok < 0) ok = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) == hipSuccess ? 1 : 0;
  if (!ok) {
    (void)hipGetLastError();
    return false;
  }
  const int tm = (g.M + HALO_BM - 1) / HALO_BM;
  g.tiles_n = (g.N + BN - 1) / BN;
  KLAUNCH_NAMED(TN == 4 ? "conv3x3_halo_kernel_n256" : "conv3x3_halo_kernel_n128", kern,
                dim3((unsigned)(tm * g.tiles_n)), dim3(512), lds, st, g);
  return true;
}

}  // namespace

// The shapes the kernel covers: whole 64-channel slices, image rows short enough for the halo
// buffer, extents below 2^31 bytes (32-bit buffer offsets), at least one full tile.
bool conv3x3_halo_supported(int N, int H, int W, int Cin, int Cout) {
  const long M = (long)N * H * W;
  return Cin % 64 == 0 && Cout % 8 == 0 && W >= 2 && H >= 2 && HALO_BM + 2 * (W + 1) <= HALO_AQ * 64 &&
         M * Cin * 2 < (1L << 31) && (long)Cout * 9 * Cin * 2 < (1L << 31) && M * Cout * 2 < (1L << 31);
}

// y = act(conv3x3(x) + bias), optionally zeroed where mask <= 0; w is [Cout][tap][Cin].
// Returns false (nothing launched) if the device refuses the kernel's LDS size.
bool conv3x3_halo_bf16(hipStream_t st, const bf16_t* x, const bf16_t* w, const float* bias, const bf16_t* mask,
                       bf16_t* y, int N, int H, int W, int Cin, int Cout, int act) {
  HaloArgs g = {};
  g.x = x; g.w = w; g.y = y; g.bias = bias; g.mask = mask;
  g.M = N * H * W; g.H = H; g.W = W; g.C = Cin; g.N = Cout; g.act = act;
  g.x_bytes = (unsigned)((size_t)g.M * Cin * 2);
  g.w_bytes = (unsigned)((size_t)Cout * 9 * Cin * 2);
  if (Cout > 128) return launch_halo<4>(st, g);
  return launch_halo<2>(st, g);
}

}  // namespace ast
