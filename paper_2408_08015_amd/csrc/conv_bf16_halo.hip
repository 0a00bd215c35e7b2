// 3x3 'same' stride-1 convolution of NHWC bf16 images as an implicit GEMM on the gfx950 matrix
// cores (v_mfma_f32_32x32x16_bf16), for the dense-convolution stage (forward, and the input
// gradient: the same product on the output gradient with point-reflected taps).
//
//   y[p][n] = sum_{tap, c} x[p + shift(tap)][c] * w[n][tap][c]     p = flattened (image, row, column)
//
// Block = 8 wavefronts.  A block owns a contiguous range of pixels (the grid is one block per
// compute unit where the image is large enough) and walks it in tiles of 256 pixels x BN output
// channels (BN = 256 or 128).  For every 64-channel slice of the input the block stages the tile's
// 256 pixels TOGETHER WITH THEIR HALO (W + 1 pixels before and after, in flattened order) in LDS once,
// and multiplies all nine taps from that copy: the pixel operand of tap (u, v) is the same LDS tile
// read (u*W + v) rows further down, so the input crosses the L2 -> LDS path once per slice and not
// once per tap.  Pixels whose shifted neighbour lies outside the image (where the flattened shift
// would wrap into the neighbouring row or image) get a zero operand by a per-lane select.
//
// Global -> LDS copies are `buffer_load_dwordx4 ... lds` (no registers in between): a wavefront
// instruction fills 1 KB = 8 rows of 128 bytes; the 16-byte chunk a lane fetches is chosen so that
// the tile lands XOR-swizzled (chunk ^= (row >> 1) & 7), which makes the MFMA operand reads (16
// consecutive rows, one chunk, at ANY row offset) free of bank conflicts.  The weights come from a
// copy laid out [slice][tap][channel][64]: the BN x 64 tile of a (slice, tap) is one contiguous
// 32 KB run, spread evenly over the L2 channels (rows of the [channel][tap][Cin] layout are 9*Cin*2
// bytes apart and hit half of the channels, with every block of an XCD asking for the same lines at
// the same time).  The weight tile is double-buffered, the halo tile of the next slice - of this
// tile or of the block's next one - is fetched during taps 0..5 of the current slice, so the stream
// of K-tiles never drains between tiles.  One s_barrier per K-tile, placed before the last quarter
// of the tile's MFMAs, which then cover the latency of the first operand reads of the next tile;
// the loads are waited for with explicit s_waitcnt vmcnt counts (the compiler does not track them).
//
// The MFMA takes the weights as its first operand, so an accumulator register group holds four
// consecutive output channels of one pixel.  A finished tile leaves in four passes through the halo
// buffer that has just been released (8-byte LDS writes, 16-byte rows out; bias, ReLU and the mask
// of a ReLU in front folded in) while the loads of the next tile are already in flight.  A last tile
// with fewer than 256 pixels skips the MFMAs of its empty 32-pixel groups.
#include "device_utils.h"
#include "kernels_bf16.h"
#include "prof.h"

#include <type_traits>

namespace ast {

namespace {

struct HaloArgs {
  const bf16_t* x;     // [M][C] pixels
  const bf16_t* w;     // [C/64][9][N][64]
  bf16_t* y;           // [M][N]
  const float* bias;   // [N] or NULL
  const bf16_t* mask;  // [M][N] or NULL: the output is zeroed where mask <= 0
  int M, H, W, C, N;
  int act;
  int tiles_n;         // channel tiles of BN
  int rows_per_block;  // pixels per block
  unsigned x_bytes, w_bytes;
};

constexpr int HALO_BM = 256;             // pixels per tile
constexpr int HALO_AQ = 6;               // halo groups (8 rows) per wavefront: 48 KB per buffer, W <= 63
constexpr int HALO_A_BYTES = HALO_AQ * 8 * 1024;
constexpr unsigned HALO_OOB = 0x80000000u;  // buffer offset beyond every extent: the load returns zeros
constexpr int HALO_CP = 272;             // row pitch of the output staging tile: 2 x 128 bytes + 16

typedef __attribute__((address_space(3))) void lds_void;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ __amdgpu_buffer_rsrc_t halo_rsrc(const void* p, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, bytes, 0x00020000);
}
// s_waitcnt with only the vector-memory counter / only the LDS counter set (gfx9 encoding:
// vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8)
__device__ __forceinline__ void wait_vmcnt0() { __builtin_amdgcn_s_waitcnt(0x0f70); }
__device__ __forceinline__ void wait_vmcnt1() { __builtin_amdgcn_s_waitcnt(0x0f71); }
__device__ __forceinline__ void wait_vmcnt2() { __builtin_amdgcn_s_waitcnt(0x0f72); }
__device__ __forceinline__ void wait_vmcnt4() { __builtin_amdgcn_s_waitcnt(0x0f74); }
__device__ __forceinline__ void wait_vmcnt8() { __builtin_amdgcn_s_waitcnt(0x0f78); }
__device__ __forceinline__ void wait_vmcnt16() { __builtin_amdgcn_s_waitcnt(0x4f70); }
__device__ __forceinline__ void wait_lds() { __builtin_amdgcn_s_waitcnt(0xc07f); }
__device__ __forceinline__ void fence() { asm volatile("" ::: "memory"); }
// barrier that does not wait for vector-memory operations in flight (__syncthreads() would)
__device__ __forceinline__ void lds_barrier() {
  wait_lds();
  fence();
  __builtin_amdgcn_s_barrier();
  fence();
}

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
  const int blk_m = bid / g.tiles_n, tile_n = bid - blk_m * g.tiles_n;
  const int n0 = tile_n * BN;
  const int m_begin = blk_m * g.rows_per_block, m_end = min(m_begin + g.rows_per_block, g.M);
  const int ntile = (m_end - m_begin + HALO_BM - 1) / HALO_BM;
  const int W = g.W, C = g.C;
  const int NS = C >> 6;
  const int HW = g.H * W;

  const __amdgpu_buffer_rsrc_t rx = halo_rsrc(g.x, g.x_bytes), rw = halo_rsrc(g.w, g.w_bytes);
  const unsigned y_bytes = (unsigned)g.M * (unsigned)g.N * 2u;
  const __amdgpu_buffer_rsrc_t ry = halo_rsrc(g.y, y_bytes), rmask = halo_rsrc(g.mask ? g.mask : g.y, y_bytes);
  // bias of the block's channels: one value per thread, kept for the whole kernel (an epilogue
  // passes it on through LDS: no global load there)
  float bias_mine = 0.f;
  if (g.bias && tid < BN && n0 + tid < g.N) bias_mine = g.bias[n0 + tid];
  // byte offsets of this lane's chunk in each group it copies (without the channel-slice / tap part)
  unsigned avoff[HALO_AQ], bvoff[BQ];
  auto set_avoff = [&](int m0) __attribute__((always_inline)) {
#pragma unroll
    for (int q = 0; q < HALO_AQ; ++q) {
      const int row = (wave + 8 * q) * 8 + (lane >> 3);
      const int lc = (lane & 7) ^ ((row >> 1) & 7);
      const int p = m0 - (W + 1) + row;
      avoff[q] = (p >= 0 && p < g.M) ? (unsigned)((p * C + lc * 8) * 2) : HALO_OOB;
    }
  };
#pragma unroll
  for (int q = 0; q < BQ; ++q) {
    const int row = (wave * BQ + q) * 8 + (lane >> 3);
    const int lc = (lane & 7) ^ ((row >> 1) & 7);
    const int n = n0 + row;
    bvoff[q] = n < g.N ? (unsigned)((n * 64 + lc * 8) * 2) : HALO_OOB;
  }
  auto issue_A = [&](int q, int slice, int buf) __attribute__((always_inline)) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (lds_void*)(sA + buf * HALO_A_BYTES + (wave + 8 * q) * 1024), 16,
                                             avoff[q], (unsigned)(slice * 128), 0, 0);
  };
  auto issue_B1 = [&](int q, unsigned soff, int buf) __attribute__((always_inline)) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, (lds_void*)(sB + buf * B_BYTES + (wave * BQ + q) * 1024), 16, bvoff[q],
                                             soff, 0, 0);
  };
  const unsigned w_tile_bytes = (unsigned)g.N * 128u;  // one (slice, tap) of the weight copy
  auto issue_B = [&](int tap, int slice, int buf) __attribute__((always_inline)) {
    const unsigned soff = (unsigned)(slice * 9 + tap) * w_tile_bytes;
    issue_B1(0, soff, buf);
    issue_B1(1, soff, buf);
    if (BQ == 4) {
      issue_B1(BQ - 2, soff, buf);
      issue_B1(BQ - 1, soff, buf);
    }
  };

  // per tile: which taps of this lane's two pixels read inside the image
  bool vy0[2], vy2[2], vx0[2], vx2[2];
  auto set_valid = [&](int m0) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int p = m0 + wm * 64 + i * 32 + lrow;
      const int rem = p % HW;
      const int yy = rem / W, xx = rem - yy * W;
      vy0[i] = yy >= 1; vy2[i] = yy <= g.H - 2; vx0[i] = xx >= 1; vx2[i] = xx <= W - 2;
    }
  };
  // LDS byte offsets of the operand fragments.  Rows 32 apart share their swizzle term, so the
  // second pixel group and the channel tiles of a wavefront are immediate offsets (i * 4096,
  // j * 4096) from one address, and the four 16-deep steps of a K-tile are that address with
  // bits 5 and 6 flipped.
  const int arow0 = wm * 64 + lrow;  // halo row of pixel group 0 at shift 0
  const int lg16 = lgrp << 4;
  auto a_base = [&](int row) __attribute__((always_inline)) -> int { return (row << 7) | (((row << 3) & 0x70) ^ lg16); };
  const int brow0 = wn * (32 * TN) + lrow;
  const int b_base = (brow0 << 7) | (((brow0 << 3) & 0x70) ^ lg16);

  floatx16 acc[TN][2];
  auto zero_acc = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][i][r] = 0.f;
  };
  zero_acc();

  bf16x8 fa[2][2], fb[2][TN];
  // aoff / boff: fragment offsets of the tile at step 0, the buffer's offset included
  auto read_frags = [&](auto groups_t, int par, int aoff, int boff, int ks) __attribute__((always_inline)) {
    constexpr int GROUPS = decltype(groups_t)::value;
#pragma unroll
    for (int i = 0; i < GROUPS; ++i)
      fa[par][i] = *reinterpret_cast<const bf16x8*>(smem + ((aoff ^ (ks << 5)) + i * 4096));
    if (GROUPS >= 1) {
#pragma unroll
      for (int j = 0; j < TN; ++j)
        fb[par][j] = *reinterpret_cast<const bf16x8*>(smem + ((boff ^ (ks << 5)) + j * 4096));
    }
  };
  typedef std::integral_constant<int, 2> both_groups;
  const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
  // GROUPS: how many of the wavefront's two pixel groups hold pixels of the tile (2, or in a last,
  // shorter tile 1 or 0): the MFMAs of an empty group are not in the code path the wavefront takes
  auto mma = [&](auto groups_t, int par, bool v0, bool v1) __attribute__((always_inline)) {
    constexpr int GROUPS = decltype(groups_t)::value;
    if (GROUPS >= 1) {
      const bf16x8 a0 = v0 ? fa[par][0] : zero8;
#pragma unroll
      for (int j = 0; j < TN; ++j) acc[j][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[par][j], a0, acc[j][0], 0, 0, 0);
    }
    if (GROUPS >= 2) {
      const bf16x8 a1 = v1 ? fa[par][1] : zero8;
#pragma unroll
      for (int j = 0; j < TN; ++j) acc[j][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[par][j], a1, acc[j][1], 0, 0, 0);
    }
  };

  // ---------------- prologue: halo of the first slice, weight tiles 0 and 1
  set_avoff(m_begin);  // (the first tile starts at m_begin in either order)
#pragma unroll
  for (int q = 0; q < HALO_AQ; ++q) issue_A(q, 0, 0);
  issue_B(0, 0, 0);
  issue_B(1, 0, 1);
  set_valid(m_begin);
  if (BQ == 4) wait_vmcnt4(); else wait_vmcnt2();  // everything but the second weight tile
  fence();
  __builtin_amdgcn_s_barrier();
  fence();
  read_frags(both_groups{}, 0, a_base(arow0), 2 * HALO_A_BYTES + b_base, 0);

  // ---------------- one 64-channel slice: nine taps.  s: slice of the tile, sig: slices done by
  // the block so far (buffer parities), hn: another slice follows (of this tile or the next),
  // s_next: its index, fresh: the slice follows an epilogue
  auto slice_body = [&](auto groups_t, int s, int sig, bool hn, int s_next, bool fresh) __attribute__((always_inline)) {
    const int abuf = (sig & 1) * HALO_A_BYTES, abuf_next = HALO_A_BYTES - abuf;
    // the fragment addresses are recomputed per tap (a handful of integer operations) instead of
    // being kept in registers across the slice loop: `vary` hides from the compiler that they repeat
    int vary;
    asm volatile("v_mov_b32 %0, 0" : "=v"(vary));
    const int arow = arow0 + vary;
#pragma unroll
    for (int t = 0; t < 9; ++t) {
      const int ty = t / 3, tx = t - ty * 3;
      const int par_b = (sig + t) & 1;  // = (9 sig + t) & 1
      const int aoff = a_base(arow + ty * W + tx) + abuf;
      const int boff = 2 * HALO_A_BYTES + par_b * B_BYTES + b_base;
      const bool v0 = (ty == 0 ? vy0[0] : ty == 2 ? vy2[0] : true) && (tx == 0 ? vx0[0] : tx == 2 ? vx2[0] : true);
      const bool v1 = (ty == 0 ? vy0[1] : ty == 2 ? vy2[1] : true) && (tx == 0 ? vx0[1] : tx == 2 ? vx2[1] : true);
      // each step: request the next step's operands, then multiply the current ones (the
      // scheduling barriers keep that order, so a request has eight MFMAs to complete)
      read_frags(groups_t, 1, aoff, boff, 1);
      __builtin_amdgcn_sched_barrier(0);
      mma(groups_t, 0, v0, v1);
      __builtin_amdgcn_sched_barrier(0);
      read_frags(groups_t, 0, aoff, boff, 2);
      __builtin_amdgcn_sched_barrier(0);
      mma(groups_t, 1, v0, v1);
      __builtin_amdgcn_sched_barrier(0);
      read_frags(groups_t, 1, aoff, boff, 3);
      __builtin_amdgcn_sched_barrier(0);
      mma(groups_t, 0, v0, v1);
      __builtin_amdgcn_sched_barrier(0);
      // Every LDS read of this K-tile has returned: after the barrier its weight buffer (and, behind
      // tap 8, the halo buffer) may be overwritten.  The loads of the next weight tile were issued
      // one K-tile ago, followed by at most one halo load, which may stay in flight.
      wait_lds();
      if (t == 0 && fresh) {  // behind an epilogue: its stores (TN passes x 4) may stay in flight
        if (TN == 4) wait_vmcnt16(); else wait_vmcnt8();
      } else if (t >= 1 && t <= HALO_AQ && hn) wait_vmcnt1();
      else wait_vmcnt0();
      fence();
      __builtin_amdgcn_s_barrier();
      fence();
      if (hn || t < 7) {  // weight tile two steps ahead, into the buffer just released
        const int t2 = (t + 2) % 9;
        issue_B(t2, t + 2 >= 9 ? s_next : s, par_b);
      }
      if (t < HALO_AQ && hn) issue_A(t, s_next, (sig + 1) & 1);
      if (hn || t < 8) {
        const int t1 = (t + 1) % 9;
        // (behind tap 8 the next slice may be a full tile's: all operands are requested then)
        read_frags(both_groups{}, 0, a_base(arow + (t1 / 3) * W + t1 % 3) + (t < 8 ? abuf : abuf_next),
                   2 * HALO_A_BYTES + (par_b ^ 1) * B_BYTES + b_base, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
      mma(groups_t, 1, v0, v1);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // ---------------- a finished tile: four passes (pixel group i, channel half jh) through the halo
  // buffer `scratch` that the tile's last slice has released: [128 rows][2 x 128 bytes + 16]
  auto epilogue = [&](int m0, int m_stop, unsigned char* scratch) __attribute__((always_inline)) {
    constexpr int NP = TN;  // passes: 2 pixel groups x TN/2 channel halves
    float* const sbias = reinterpret_cast<float*>(scratch + 128 * HALO_CP);  // [BN], behind the staging tile
    if (tid < BN) sbias[tid] = bias_mine;
    // The rows this thread sends out in pass p: buffer offset in y (and in the mask), beyond the
    // extent where the row is past the block's range or the channel past N - such a store is
    // dropped by the hardware, so every wavefront issues the same number of stores (the wait
    // counts of the next tile rely on that).
    auto out_off = [&](int p, int k) __attribute__((always_inline)) -> unsigned {
      const int i = p / (TN / 2), jh = p % (TN / 2);
      const int idx = tid + 512 * k, row = idx >> 4, ch = idx & 15;
      const int m = m0 + (row >> 5) * 64 + i * 32 + (row & 31);
      const int n = n0 + (ch >> 3) * (32 * TN) + jh * 64 + (ch & 7) * 8;
      return (m < m_stop && n < g.N) ? (unsigned)((m * g.N + n) * 2) : HALO_OOB;
    };
    // mask words of a pass are requested one pass ahead, before that pass's stores: a load
    // cannot overtake an older store in the vector-memory counter
    u32x4 mk[2][4];
    if (g.mask) {
#pragma unroll
      for (int k = 0; k < 4; ++k) mk[0][k] = __builtin_amdgcn_raw_buffer_load_b128(rmask, out_off(0, k), 0, 0);
    }
    lds_barrier();  // bias in LDS
#pragma unroll
    for (int p = 0; p < NP; ++p) {
      const int i = p / (TN / 2), jh = p % (TN / 2);
      if (p > 0) lds_barrier();  // the previous pass has been read
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        const int j = 2 * jh + jj;
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const int c4 = 8 * r4 + 4 * lgrp;  // four consecutive channels of tile j
          const float4 bv = *reinterpret_cast<const float4*>(sbias + wn * (32 * TN) + j * 32 + c4);
          float v0 = acc[j][i][4 * r4 + 0] + bv.x, v1 = acc[j][i][4 * r4 + 1] + bv.y;
          float v2 = acc[j][i][4 * r4 + 2] + bv.z, v3 = acc[j][i][4 * r4 + 3] + bv.w;
          if (g.act == ACT_RELU) { v0 = fmaxf(v0, 0.f); v1 = fmaxf(v1, 0.f); v2 = fmaxf(v2, 0.f); v3 = fmaxf(v3, 0.f); }
          uint2 pk;
          pk.x = f2bf_pk(v0, v1);
          pk.y = f2bf_pk(v2, v3);
          *reinterpret_cast<uint2*>(scratch + (wm * 32 + lrow) * HALO_CP + wn * 128 + jj * 64 + c4 * 2) = pk;
        }
      }
      lds_barrier();
      if (g.mask && p + 1 < NP) {
#pragma unroll
        for (int k = 0; k < 4; ++k) mk[(p + 1) & 1][k] = __builtin_amdgcn_raw_buffer_load_b128(rmask, out_off(p + 1, k), 0, 0);
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int idx = tid + 512 * k, row = idx >> 4, ch = idx & 15;
        u32x4 v = *reinterpret_cast<const u32x4*>(scratch + row * HALO_CP + ch * 16);
        if (g.mask) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {  // bf16 > 0: sign clear and not zero
            const uint32_t o = mk[p & 1][k][e];
            const uint32_t lo = o & 0xffffu, hi = o >> 16;
            const uint32_t keep = ((lo != 0u && lo < 0x8000u) ? 0x0000ffffu : 0u) | ((hi != 0u && hi < 0x8000u) ? 0xffff0000u : 0u);
            v[e] &= keep;
          }
        }
        __builtin_amdgcn_raw_buffer_store_b128(v, ry, out_off(p, k), 0, 0);
      }
    }
  };

  // ---------------- the block's tiles, as one stream of slices.  The short tile of the range (if
  // any) comes last in even blocks and first in odd ones, so that the blocks of the grid do not
  // all send out a finished tile - a burst of stores - at the same moments.
  const int short_rows = (m_end - m_begin) - (ntile - 1) * HALO_BM;  // 1..256
  const bool short_first = (blk_m & 1) != 0 && short_rows < HALO_BM;
  auto tile_begin = [&](int tl) __attribute__((always_inline)) -> int {
    return short_first ? (tl == 0 ? m_begin : m_begin + short_rows + (tl - 1) * HALO_BM) : m_begin + tl * HALO_BM;
  };
  auto tile_rows = [&](int tl) __attribute__((always_inline)) -> int {
    return (short_first ? tl == 0 : tl == ntile - 1) ? short_rows : HALO_BM;
  };
  int sig = 0;
  for (int tl = 0; tl < ntile; ++tl) {
    const int m0 = tile_begin(tl);
    const int rows = tile_rows(tl);
    const bool more = tl + 1 < ntile;
    for (int s = 0; s < NS; ++s, ++sig) {
      const bool last = s + 1 == NS;
      if (last && more) set_avoff(tile_begin(tl + 1));  // from here on the halo loads are the next tile's
      const bool hn = !last || more;
      const int s_next = last ? 0 : s + 1;
      const int mine = rows - wm * 64;  // pixels of the tile in this wavefront's two groups
      const bool fresh = s == 0 && tl > 0;
      if (mine > 32) slice_body(both_groups{}, s, sig, hn, s_next, fresh);
      else if (mine > 0) slice_body(std::integral_constant<int, 1>{}, s, sig, hn, s_next, fresh);
      else slice_body(std::integral_constant<int, 0>{}, s, sig, hn, s_next, fresh);
    }
    // sig counts this tile's last slice already: its halo buffer is the one before
    epilogue(m0, m0 + rows, sA + ((sig - 1) & 1) * HALO_A_BYTES);
    if (more) {
      zero_acc();
      set_valid(tile_begin(tl + 1));
    }
  }
}

// (plain kernels around the templated body: the host pass of the compiler drops the stub of a
// kernel template with this body without a diagnostic)
__global__ __launch_bounds__(512) void conv3x3_halo_kernel_n256(HaloArgs g) { conv3x3_halo_body<4>(g); }
__global__ __launch_bounds__(512) void conv3x3_halo_kernel_n128(HaloArgs g) { conv3x3_halo_body<2>(g); }

template <int TN>
constexpr size_t halo_lds_bytes() { return 2 * HALO_A_BYTES + 2 * (64 * TN) * 128; }
static_assert(128 * HALO_CP + 256 * 4 <= HALO_A_BYTES, "the output staging tile and the bias must fit in one halo buffer");

// dynamic LDS beyond 64 KiB has to be allowed per kernel, once per process
bool halo_attr_ok() {
  static int ok = -1;
  if (ok < 0) {
    ok = hipFuncSetAttribute((const void*)conv3x3_halo_kernel_n256, hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)halo_lds_bytes<4>()) == hipSuccess &&
                 hipFuncSetAttribute((const void*)conv3x3_halo_kernel_n128, hipFuncAttributeMaxDynamicSharedMemorySize,
                                     (int)halo_lds_bytes<2>()) == hipSuccess
             ? 1
             : 0;
    if (!ok) (void)hipGetLastError();
  }
  return ok == 1;
}

int halo_num_cus() {
  static int n = 0;
  if (n == 0) {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess) n = prop.multiProcessorCount;
    if (n <= 0) n = 256;
  }
  return n;
}

template <int TN>
void launch_halo(hipStream_t st, HaloArgs& g) {
  constexpr int BN = 64 * TN;
  g.tiles_n = (g.N + BN - 1) / BN;
  // one block per compute unit, each with an equal share of the pixels (at least one tile's worth)
  const int tiles_m = (g.M + HALO_BM - 1) / HALO_BM;
  int blocks_m = halo_num_cus() / g.tiles_n;
  if (blocks_m < 1) blocks_m = 1;
  if (blocks_m > tiles_m) blocks_m = tiles_m;
  g.rows_per_block = (g.M + blocks_m - 1) / blocks_m;
  blocks_m = (g.M + g.rows_per_block - 1) / g.rows_per_block;
  KLAUNCH_NAMED(TN == 4 ? "conv3x3_halo_kernel_n256" : "conv3x3_halo_kernel_n128",
                TN == 4 ? conv3x3_halo_kernel_n256 : conv3x3_halo_kernel_n128, dim3((unsigned)(blocks_m * g.tiles_n)),
                dim3(512), halo_lds_bytes<TN>(), st, g);
}

}  // namespace

// The shapes the kernel covers: whole 64-channel slices, image rows short enough for the halo
// buffer, extents below 2^31 bytes (32-bit buffer offsets); and a device that grants the LDS size.
bool conv3x3_halo_supported(int N, int H, int W, int Cin, int Cout) {
  const long M = (long)N * H * W;
  return Cin % 64 == 0 && Cout % 8 == 0 && W >= 2 && H >= 2 && HALO_BM + 2 * (W + 1) <= HALO_AQ * 64 &&
         M * Cin * 2 < (1L << 31) && (long)Cout * 9 * Cin * 2 < (1L << 31) && M * Cout * 2 < (1L << 31) && halo_attr_ok();
}

// y = act(conv3x3(x) + bias), optionally zeroed where mask <= 0; w is the tiled copy
// [Cin/64][tap][Cout][64].
void conv3x3_halo_bf16(hipStream_t st, const bf16_t* x, const bf16_t* w, const float* bias, const bf16_t* mask,
                       bf16_t* y, int N, int H, int W, int Cin, int Cout, int act) {
  HaloArgs g = {};
  g.x = x; g.w = w; g.y = y; g.bias = bias; g.mask = mask;
  g.M = N * H * W; g.H = H; g.W = W; g.C = Cin; g.N = Cout; g.act = act;
  g.x_bytes = (unsigned)((size_t)g.M * Cin * 2);
  g.w_bytes = (unsigned)((size_t)Cout * 9 * Cin * 2);
  if (Cout > 128) launch_halo<4>(st, g);
  else launch_halo<2>(st, g);
}

}  // namespace ast
