// Dense-layer products of the transformer stage on the gfx950 matrix cores
// (v_mfma_f32_32x32x16_bf16), forward and input gradient alike:
//
//   C[m][n] = epilogue( sum_k A[m][k] * B[n][k] )        A [M][K] bf16 rows, B the weights
//
// These products are short in K (512 .. 2048) and a few thousand rows tall, so a block computes one
// output tile and what decides the time is how little of it is spent outside the MFMAs: staging
// arithmetic, barriers, the prologue and the epilogue.
//
// Block = 8 wavefronts (4 along M x 2 along N), tile 128*TM rows x 64*TN columns, wavefront tile
// 32*TM x 32*TN: 256 x 128 where that still gives most compute units a tile, 128 x 128 and 128 x 64
// for the narrow outputs (a narrow tile re-reads more operand bytes per flop: what bounds those
// products is the L2 -> LDS path, 64 bytes per clock and compute unit, so they want every compute
// unit pulling).  K advances in stages of 64 (128 for the smallest tile, as two 64-deep sub-tiles)
// through a ring of LDS stages.  Global -> LDS copies are
// `buffer_load_dwordx4 ... lds` (no registers, no address arithmetic in the loop: a per-lane byte
// offset fixed for the whole kernel plus a scalar offset per K-tile); a wavefront instruction fills
// 1 KB = 8 rows of 128 bytes, and the 16-byte chunk a lane fetches is chosen so that the tile lands
// XOR-swizzled (chunk ^= (row >> 1) & 7): the MFMA operand reads (16 consecutive rows, one chunk)
// are free of bank conflicts, fragments 32 rows apart are an immediate offset of 4096 bytes and the
// four 16-deep steps of a K-tile are one address with bits 5 and 6 flipped.  The weights come from
// a copy laid out [K/64][N][64]: the 128 x 64 tile of a K-step is one contiguous 16 KB run.
//
// The loads of K-tile t + NSTAGE are issued when tile t has been consumed, so a load has
// NSTAGE - 1 tiles of MFMAs to land; they are waited for with explicit s_waitcnt vmcnt counts (the
// compiler does not track them).  Every thread issues the same number of loads per tile - beyond the
// last K-tile with an out-of-range offset, which the hardware turns into a zero fill of a stage
// nobody reads - so those counts are exact.  One s_barrier per stage, between the two halves of
// the stage's MFMAs: the second half covers the latency of the next stage's first operand reads.
//
// The MFMA takes the weights as its first operand, so an accumulator register group holds four
// consecutive output columns of one row.  The finished tile leaves in TM passes through LDS (8-byte
// writes, 16-byte rows out) with bias, ReLU or GELU (the pre-activation as a second output), a
// residual sum, or the product with GELU'(t) of a stored pre-activation folded in, applied exactly
// where the general kernel applies them (sum and product on the bf16-rounded result).
#include "device_utils.h"
#include "kernels_bf16.h"
#include "prof.h"

#include <cstdlib>

namespace ast {

namespace {

struct LinArgs {
  const bf16_t* a;     // [M][K]
  const bf16_t* b;     // [K/64][N][64]
  bf16_t* c;           // [M][N]
  bf16_t* pre;         // GELU: the pre-activation [M][N]
  const float* bias;   // [N] or NULL
  const bf16_t* add;   // [M][N] or NULL: added to the rounded result
  const bf16_t* gmul;  // [M][N] or NULL: the rounded result is multiplied by GELU'(gmul)
  int M, N, K;
  int act;
  int tiles_n;
  unsigned a_bytes, b_bytes;
};

constexpr unsigned LIN_OOB = 0x80000000u;  // buffer offset beyond every extent: loads give zeros, stores are dropped

typedef __attribute__((address_space(3))) void lds_void;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ __amdgpu_buffer_rsrc_t lin_rsrc(const void* p, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, bytes, 0x00020000);
}
// s_waitcnt with only the vector-memory counter / only the LDS counter set (gfx9 encoding:
// vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8)
__device__ __forceinline__ void lin_wait_vmcnt0() { __builtin_amdgcn_s_waitcnt(0x0f70); }
__device__ __forceinline__ void lin_wait_vmcnt6() { __builtin_amdgcn_s_waitcnt(0x0f76); }
__device__ __forceinline__ void lin_wait_vmcnt8() { __builtin_amdgcn_s_waitcnt(0x0f78); }
__device__ __forceinline__ void lin_wait_vmcnt12() { __builtin_amdgcn_s_waitcnt(0x0f7c); }
__device__ __forceinline__ void lin_wait_lds() { __builtin_amdgcn_s_waitcnt(0xc07f); }
__device__ __forceinline__ void lin_fence() { asm volatile("" ::: "memory"); }
// barrier that does not wait for vector-memory operations in flight (__syncthreads() would)
__device__ __forceinline__ void lin_lds_barrier() {
  lin_wait_lds();
  lin_fence();
  __builtin_amdgcn_s_barrier();
  lin_fence();
}

// LDS stages of a tile shape: as many as fit next to each other (3 x 48 KB, 4 x 32 KB)
template <int TM, int TN, int KSUB>
constexpr int lin_stages() { return KSUB * (128 * TM + 64 * TN) * 128 > 32768 ? 3 : 4; }

// wavefront tile: 32*TM rows x 32*TN columns; a stage holds KSUB sub-tiles of 64 along K
template <int TM, int TN, int KSUB>
__device__ __forceinline__ void linear_dl_body(const LinArgs& g) {
  constexpr int BM = 128 * TM, BN = 64 * TN;
  constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128, SUB = A_BYTES + B_BYTES, STAGE = KSUB * SUB;
  constexpr int NSTAGE = lin_stages<TM, TN, KSUB>();
  constexpr int AQ = BM / 64, BQ = BN / 64;  // groups of 8 rows per wavefront and sub-tile
  constexpr int LPT = KSUB * (AQ + BQ);      // loads per thread and stage
  static_assert((NSTAGE - 1) * LPT == 12 && ((NSTAGE - 2) * LPT == 6 || (NSTAGE - 2) * LPT == 8), "wait counts below");
  constexpr int UNIT = 2 * KSUB;             // 16-deep steps per half stage
  constexpr int CP = BN * 2 + 16;            // row pitch of the output staging tile
  constexpr int CH = BN / 8;                 // 16-byte chunks per output row of the tile
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int lrow = lane & 31, lgrp = lane >> 5;
  // neighbouring tiles in (row tile, column tile) order run on the same XCD: they share the row
  // tile's A rows, and the whole weight matrix stays in that XCD's L2
  const int bid = (int)xcd_grouped(blockIdx.x, gridDim.x);
  const int tile_m = bid / g.tiles_n, tile_n = bid - tile_m * g.tiles_n;
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const int nk = g.K >> 6;                       // sub-tiles
  const int nst = (nk + KSUB - 1) / KSUB;        // stages

  const __amdgpu_buffer_rsrc_t ra = lin_rsrc(g.a, g.a_bytes), rb = lin_rsrc(g.b, g.b_bytes);
  unsigned avoff[AQ], bvoff[BQ];
#pragma unroll
  for (int q = 0; q < AQ; ++q) {
    const int row = (wave + 8 * q) * 8 + (lane >> 3);
    const int lc = (lane & 7) ^ ((row >> 1) & 7);
    const int m = m0 + row;
    avoff[q] = m < g.M ? (unsigned)((m * g.K + lc * 8) * 2) : LIN_OOB;
  }
#pragma unroll
  for (int q = 0; q < BQ; ++q) {
    const int row = (wave + 8 * q) * 8 + (lane >> 3);
    const int lc = (lane & 7) ^ ((row >> 1) & 7);
    const int n = n0 + row;
    bvoff[q] = n < g.N ? (unsigned)((n * 64 + lc * 8) * 2) : LIN_OOB;
  }
  const unsigned b_tile_bytes = (unsigned)g.N * 128u;  // one 64-deep slice of the weight copy
  auto issue = [&](int st, int stage_off) __attribute__((always_inline)) {
#pragma unroll
    for (int sub = 0; sub < KSUB; ++sub) {
      const int kt = st * KSUB + sub;
      const bool live = kt < nk;
#pragma unroll
      for (int q = 0; q < AQ; ++q)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, (lds_void*)(smem + stage_off + sub * SUB + (wave + 8 * q) * 1024), 16,
                                                 live ? avoff[q] : LIN_OOB, (unsigned)(kt * 128), 0, 0);
#pragma unroll
      for (int q = 0; q < BQ; ++q)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            rb, (lds_void*)(smem + stage_off + sub * SUB + A_BYTES + (wave + 8 * q) * 1024), 16, live ? bvoff[q] : LIN_OOB,
            (unsigned)kt * b_tile_bytes, 0, 0);
    }
  };

  // LDS byte offsets of this lane's operand fragments inside a sub-tile, at step 0
  const int arow = wm * (32 * TM) + lrow, brow = wn * (32 * TN) + lrow;
  const int lg16 = lgrp << 4;
  const int a_frag = (arow << 7) | (((arow << 3) & 0x70) ^ lg16);
  const int b_frag = A_BYTES + ((brow << 7) | (((brow << 3) & 0x70) ^ lg16));

  floatx16 acc[TN][TM];
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[j][i][r] = 0.f;

  // operand fragments of half a stage (UNIT 16-deep steps), double-buffered
  bf16x8 fa[2][UNIT][TM], fb[2][UNIT][TN];
  auto read_half = [&](int par, int stage_off, int h) __attribute__((always_inline)) {
#pragma unroll
    for (int kk = 0; kk < UNIT; ++kk) {
      const int step = h * UNIT + kk;  // 16-deep step of the stage
      const int flip = (step & 3) << 5;
      const int base = stage_off + (step >> 2) * SUB;
#pragma unroll
      for (int i = 0; i < TM; ++i)
        fa[par][kk][i] = *reinterpret_cast<const bf16x8*>(smem + base + ((a_frag ^ flip) + i * 4096));
#pragma unroll
      for (int j = 0; j < TN; ++j)
        fb[par][kk][j] = *reinterpret_cast<const bf16x8*>(smem + base + ((b_frag ^ flip) + j * 4096));
    }
  };
  auto mma_half = [&](int par) __attribute__((always_inline)) {
#pragma unroll
    for (int kk = 0; kk < UNIT; ++kk)
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[par][kk][j], fa[par][kk][i], acc[j][i], 0, 0, 0);
  };

  // ---------------- prologue: the first NSTAGE K-tiles
#pragma unroll
  for (int t = 0; t < NSTAGE; ++t) issue(t, t * STAGE);
  lin_wait_vmcnt12();  // all but the last NSTAGE - 1 tiles: tile 0 is in LDS
  lin_fence();
  __builtin_amdgcn_s_barrier();
  lin_fence();
  read_half(0, 0, 0);

  // ---------------- K loop
  int rs = 0;  // byte offset of the stage being read
  for (int kt = 0; kt < nst; ++kt) {
    read_half(1, rs, 1);
    __builtin_amdgcn_sched_barrier(0);
    mma_half(0);
    __builtin_amdgcn_sched_barrier(0);
    // Every LDS read of this tile has returned: after the barrier its stage may be overwritten.
    // Outstanding loads: stages kt+1 .. kt+NSTAGE-1; the oldest must have landed.
    lin_wait_lds();
    if ((NSTAGE - 2) * LPT == 6) lin_wait_vmcnt6(); else lin_wait_vmcnt8();
    lin_fence();
    __builtin_amdgcn_s_barrier();
    lin_fence();
    issue(kt + NSTAGE, rs);
    rs = rs + STAGE == NSTAGE * STAGE ? 0 : rs + STAGE;
    read_half(0, rs, 0);  // (behind the last stage: a stage of zeros, never multiplied)
    __builtin_amdgcn_sched_barrier(0);
    mma_half(1);
    __builtin_amdgcn_sched_barrier(0);
  }
  // the zero fills issued behind the last tiles still target the stages: drain before reusing LDS
  lin_wait_vmcnt0();
  lin_lds_barrier();

  // ---------------- epilogue
  unsigned char* const stage0 = smem;              // [128 rows][CP]: the result (GELU: the pre-activation)
  unsigned char* const stage1 = smem + 128 * CP;   // GELU: the activation
  float* const sbias = reinterpret_cast<float*>(smem + 2 * 128 * CP);
  static_assert(2 * 128 * CP + BN * 4 <= NSTAGE * STAGE, "the output staging tiles and the bias must fit");
  constexpr int SPT = 128 * CH / 512;  // 16-byte stores per thread and pass
  if (tid < BN) sbias[tid] = (g.bias && n0 + tid < g.N) ? g.bias[n0 + tid] : 0.f;
  const unsigned c_bytes = (unsigned)g.M * (unsigned)g.N * 2u;
  const __amdgpu_buffer_rsrc_t rc = lin_rsrc(g.c, c_bytes), rpre = lin_rsrc(g.pre ? g.pre : g.c, c_bytes);
  const bf16_t* const other = g.add ? g.add : g.gmul;
  const __amdgpu_buffer_rsrc_t ro = lin_rsrc(other ? other : g.c, c_bytes);
  const bool gelu = g.act == ACT_GELU;
  auto out_off = [&](int i, int k) __attribute__((always_inline)) -> unsigned {
    const int idx = tid + 512 * k, row = idx / CH, ch = idx % CH;
    const int m = m0 + (row >> 5) * (32 * TM) + i * 32 + (row & 31);
    const int n = n0 + ch * 8;
    return (m < g.M && n < g.N) ? (unsigned)((m * g.N + n) * 2) : LIN_OOB;
  };
  u32x4 ot[2][SPT];
  if (other) {
#pragma unroll
    for (int k = 0; k < SPT; ++k) ot[0][k] = __builtin_amdgcn_raw_buffer_load_b128(ro, out_off(0, k), 0, 0);
  }
  lin_lds_barrier();  // bias in LDS
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    if (i > 0) lin_lds_barrier();  // the previous pass has been read
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int c4 = 8 * r4 + 4 * lgrp;  // four consecutive columns of tile j
        const float4 bv = *reinterpret_cast<const float4*>(sbias + wn * (32 * TN) + j * 32 + c4);
        float v0 = acc[j][i][4 * r4 + 0] + bv.x, v1 = acc[j][i][4 * r4 + 1] + bv.y;
        float v2 = acc[j][i][4 * r4 + 2] + bv.z, v3 = acc[j][i][4 * r4 + 3] + bv.w;
        if (g.act == ACT_RELU) { v0 = fmaxf(v0, 0.f); v1 = fmaxf(v1, 0.f); v2 = fmaxf(v2, 0.f); v3 = fmaxf(v3, 0.f); }
        const int at = (wm * 32 + lrow) * CP + wn * (64 * TN) + j * 64 + c4 * 2;
        uint2 pk;
        pk.x = f2bf_pk(v0, v1);
        pk.y = f2bf_pk(v2, v3);
        *reinterpret_cast<uint2*>(stage0 + at) = pk;
        if (gelu) {
          pk.x = f2bf_pk(gelu_fast(v0), gelu_fast(v1));
          pk.y = f2bf_pk(gelu_fast(v2), gelu_fast(v3));
          *reinterpret_cast<uint2*>(stage1 + at) = pk;
        }
      }
    }
    lin_lds_barrier();
    if (other && i + 1 < TM) {
#pragma unroll
      for (int k = 0; k < SPT; ++k) ot[(i + 1) & 1][k] = __builtin_amdgcn_raw_buffer_load_b128(ro, out_off(i + 1, k), 0, 0);
    }
#pragma unroll
    for (int k = 0; k < SPT; ++k) {
      const int idx = tid + 512 * k, row = idx / CH, ch = idx % CH;
      const unsigned off = out_off(i, k);
      u32x4 v = *reinterpret_cast<const u32x4*>(stage0 + row * CP + ch * 16);
      if (gelu) {
        __builtin_amdgcn_raw_buffer_store_b128(v, rpre, off, 0, 0);
        v = *reinterpret_cast<const u32x4*>(stage1 + row * CP + ch * 16);
      } else if (other) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const uint32_t o = ot[i & 1][k][e];
          float a0 = __uint_as_float(v[e] << 16), a1 = __uint_as_float(v[e] & 0xffff0000u);
          const float b0 = __uint_as_float(o << 16), b1 = __uint_as_float(o & 0xffff0000u);
          if (g.add) { a0 += b0; a1 += b1; }
          else { a0 *= gelu_grad_fast(b0); a1 *= gelu_grad_fast(b1); }
          v[e] = f2bf_pk(a0, a1);
        }
      }
      __builtin_amdgcn_raw_buffer_store_b128(v, rc, off, 0, 0);
    }
  }
}

// (plain kernels around the templated body: the host pass of the compiler drops the stub of a
// kernel template with this body without a diagnostic)
__global__ __launch_bounds__(512) void linear_dl_kernel_256x128(LinArgs g) { linear_dl_body<2, 2, 1>(g); }
__global__ __launch_bounds__(512) void linear_dl_kernel_128x128(LinArgs g) { linear_dl_body<1, 2, 1>(g); }
__global__ __launch_bounds__(512) void linear_dl_kernel_128x64(LinArgs g) { linear_dl_body<1, 1, 2>(g); }

template <int TM, int TN, int KSUB>
constexpr size_t lin_lds_bytes() { return (size_t)lin_stages<TM, TN, KSUB>() * KSUB * (128 * TM + 64 * TN) * 128; }

// dynamic LDS beyond 64 KiB has to be allowed per kernel, once per process
bool lin_attr_ok() {
  static int ok = -1;
  if (ok < 0) {
    ok = hipFuncSetAttribute((const void*)linear_dl_kernel_256x128, hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)lin_lds_bytes<2, 2, 1>()) == hipSuccess &&
                 hipFuncSetAttribute((const void*)linear_dl_kernel_128x128, hipFuncAttributeMaxDynamicSharedMemorySize,
                                     (int)lin_lds_bytes<1, 2, 1>()) == hipSuccess &&
                 hipFuncSetAttribute((const void*)linear_dl_kernel_128x64, hipFuncAttributeMaxDynamicSharedMemorySize,
                                     (int)lin_lds_bytes<1, 1, 2>()) == hipSuccess
             ? 1
             : 0;
    if (!ok) (void)hipGetLastError();
  }
  return ok == 1;
}

}  // namespace

// The shapes the kernel covers: whole K-tiles of 64, 16-byte output chunks, extents below 2^31
// bytes (32-bit buffer offsets); and a device that grants the LDS size.  ASTEROID_LINEAR_DL=0
// switches it off (experiment switch).
bool linear_dl_supported(size_t R, int K, int N) {
  static const int on = [] {
    const char* e = getenv("ASTEROID_LINEAR_DL");
    return e ? atoi(e) : 1;
  }();
  const long M = (long)R;
  return on && K >= 64 && K % 64 == 0 && N >= 64 && N % 8 == 0 && M >= 64 && M * K * 2 < (1L << 31) &&
         M * N * 2 < (1L << 31) && (long)N * K * 2 < (1L << 31) && lin_attr_ok();
}

// c = epilogue(a b^T): a [R][K], b the tiled weight copy [K/64][N][64].  act: none, ReLU, or GELU
// (then pre receives the pre-activation); add / gmul as in the general kernel, at most one of them,
// and neither together with GELU.
void linear_dl_bf16(hipStream_t st, const bf16_t* a, const bf16_t* b, const float* bias, bf16_t* c, bf16_t* pre,
                    const bf16_t* add, const bf16_t* gmul, size_t R, int K, int N, int act) {
  LinArgs g = {};
  g.a = a; g.b = b; g.c = c; g.pre = act == ACT_GELU ? pre : nullptr; g.bias = bias; g.add = add; g.gmul = gmul;
  g.M = (int)R; g.N = N; g.K = K; g.act = act;
  g.a_bytes = (unsigned)(R * (size_t)K * 2);
  g.b_bytes = (unsigned)((size_t)N * K * 2);
  // The tallest, widest tile that still yields enough blocks to occupy most compute units
  // (ASTEROID_LINEAR_TILE = 1, 2, 3 forces one: experiment switch).
  static const int force = [] {
    const char* e = getenv("ASTEROID_LINEAR_TILE");
    return e ? atoi(e) : 0;
  }();
  const long t256 = (long)((g.M + 255) / 256) * ((N + 127) / 128);
  const long t128 = (long)((g.M + 127) / 128) * ((N + 127) / 128);
  const long t64 = (long)((g.M + 127) / 128) * ((N + 63) / 64);
  const int pick = force ? force : (t256 >= 160 ? 1 : (t128 >= 160 ? 2 : 3));
  if (pick == 1) {
    g.tiles_n = (N + 127) / 128;
    KLAUNCH_NAMED("linear_dl_kernel_256x128", linear_dl_kernel_256x128, dim3((unsigned)t256), dim3(512),
                  (lin_lds_bytes<2, 2, 1>()), st, g);
  } else if (pick == 2) {
    g.tiles_n = (N + 127) / 128;
    KLAUNCH_NAMED("linear_dl_kernel_128x128", linear_dl_kernel_128x128, dim3((unsigned)t128), dim3(512),
                  (lin_lds_bytes<1, 2, 1>()), st, g);
  } else {
    g.tiles_n = (N + 63) / 64;
    KLAUNCH_NAMED("linear_dl_kernel_128x64", linear_dl_kernel_128x64, dim3((unsigned)t64), dim3(512),
                  (lin_lds_bytes<1, 1, 2>()), st, g);
  }
}

}  // namespace ast
