// bf16 x bf16 -> fp32 matrix products on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16),
// LDS-staged, serving the dense layers of the VGG-style and transformer stages:
//   linear forward / input gradient            C[m][n] = sum_k A[m][k] B[n][k]
//   3x3 / 1x1 'same' convolution, NHWC         A gathered on the fly (implicit GEMM)
//   weight gradients                           C[m][n] = sum_k A[k][m] B[k][n], K = rows/pixels,
//                                              split over K, deterministic fp32 reduction into G
//
// Block = 256 threads = 2 x 2 wavefronts; each wavefront owns a WTM x WTN tile made of
// 32x32 MFMA tiles; K advances 64 per step.  Both operands sit in LDS as [row][k] with k
// contiguous, rows and 16-byte chunks permuted so that operand reads and staging writes
// are free of bank conflicts (see lds_off).  The global loads of K-tile t+1 are issued
// before the MFMAs of tile t; with two LDS buffers they are written to the other buffer
// after them (one barrier per tile), with one buffer at the top of the next step.  MFMA 32x32x16: lane l supplies A[l%32][8*(l/32) .. +7] and B likewise;
// accumulator register r of lane l is D[8*(r/4) + 4*(l/32) + r%4][l%32].
// Operands stored with the contraction index strided (weight gradients) are transposed in
// registers (4 x 8 blocks) on their way into LDS.  The bf16 output tile goes through LDS
// so that every lane stores 16 contiguous bytes.
#include "device_utils.h"
#include "kernels_bf16.h"
#include <cstdlib>

#include "prof.h"

namespace ast {

namespace {

constexpr int BK = 64;

enum { A_ROW = 0, A_IM2COL = 1, OP_T = 2, B_ROW = 0, B_T_SHIFT = 3 };
enum { E_BF16 = 0, E_PART = 1 };

struct GemmArgs {
  const bf16_t* A;
  const bf16_t* B;
  long M, N, K;
  long lda, ldb;
  int H, W, C, ksize;  // image geometry of the gathered / shifted operand
  int fastc;           // implicit GEMM: C % 64 == 0, so a K-tile lies inside one tap
  int step_q, step_r;  // 64 / W, 64 % W: pixel advance of one K-tile (shifted operand)
  long k_per_split;    // K range per split (multiple of BK)
  // epilogue
  bf16_t* Cb;          // bf16 output [M][ldc]
  bf16_t* pre;         // optional pre-activation copy
  float* part;         // fp32 partials [split][tap][M][N]
  long ldc;
  const float* bias;
  const bf16_t* add;   // optional residual input [M][ldc], added to the (rounded) output
  const bf16_t* gmul;  // optional [M][ldc] tensor t: the output is multiplied by GELU'(t), or
                       // (gmul_relu) zeroed where t <= 0 (ReLU mask by the activation's output)
  int gmul_relu;
  int act;
  int tiles_n;         // number of tiles along N
  int tiles_mn;        // number of output tiles; block id = (split * taps + tap) * tiles_mn + tile
  int taps;            // weight gradient of a k x k conv: k*k products per launch, else 1
  unsigned a_bytes, b_bytes;  // extents of the operands (below 2^31): range of the buffer loads
};

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
// 16-byte load through a buffer descriptor: an offset at or beyond the extent returns zeros
// (the hardware's range check), so padding and ragged edges need neither a branch nor a select.
__device__ __forceinline__ uint4 buf_load16(__amdgpu_buffer_rsrc_t r, unsigned byte_off) {
  const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, 0);
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, bytes, 0x00020000);
}

// Element offset of 16-byte chunk c16 (0..7) of LDS row `row`.  The LDS has 64 banks of
// 4 bytes; a 16-byte operand read is served 16 lanes at a time, an 8-byte write 32 lanes at
// a time, and either runs at full rate only if those lanes cover all 64 banks once.  Rows
// are 128 bytes (no padding), two rows per bank sweep, with
//   physical row = row with bits 0 and 3 exchanged,   chunk ^= (row & 7) ^ ((row >> 4) & 7):
// the MFMA operand reads (16 consecutive rows, one chunk) then split 8 / 8 over the two
// halves of a sweep with 8 distinct chunks each, and so do the transposed writes of the
// weight-gradient operands (16 rows 8 apart, one chunk).  Measured on MI355X: 210 B/clk/CU
// for the reads against 80 for a 144-byte row stride with chunk ^= row >> 3.
template <int BKT>
__device__ __forceinline__ int lds_off(int row, int c16) {
  if (BKT == 64) {
    const int prow = (row & ~9) | ((row & 1) << 3) | ((row >> 3) & 1);
    return prow * 64 + ((c16 ^ (row & 7) ^ ((row >> 4) & 7)) << 3);
  }
  // deeper tiles (rows of 256 bytes or more = whole bank sweeps): 16 consecutive rows reading
  // the same chunk must land in 16 different 16-byte slots of a sweep
  return row * BKT + ((c16 ^ (row & 15)) << 3);
}

__device__ __forceinline__ float gelu_f(float x) { return gelu_fast(x); }
// d/dx of the exact GELU: Phi(x) + x phi(x)
__device__ __forceinline__ float gelu_grad_f(float x) { return gelu_grad_fast(x); }

template <int WTM, int WTN, int AMODE, int BMODE, int EMODE, bool DBUF, bool FASTC, int PF = 1, int BKT = 64>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmArgs g) {
  static_assert(BKT == 64 || (AMODE == A_ROW && BMODE == B_ROW), "deep K-tiles: plain row operands only");
  constexpr int CPR = BKT / 8;    // 16-byte chunks per LDS row
  constexpr int RPP = 256 / CPR;  // rows staged per pass of the block
  constexpr int BM = 2 * WTM, BN = 2 * WTN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int STAGE = (BM + BN) * BKT;  // elements per buffer
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t* smem = reinterpret_cast<bf16_t*>(smem_raw);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  // Blocks are dealt to the 8 XCDs round-robin; renumber them so that each XCD (own L2) works
  // on a contiguous range of the flat (split, tap, tile) order: the N-tiles of one row tile
  // and neighbouring row tiles (which share halo pixels in the implicit GEMM), or all taps
  // and tiles of one K-split of a weight gradient (which read the same rows of both
  // operands), then hit the same L2.
  int bid = blockIdx.x;
  {
    const int nb = gridDim.x, q = nb >> 3, r = nb & 7, xcd = bid & 7;
    bid = xcd * q + min(xcd, r) + (bid >> 3);
  }
  const int tile = bid % g.tiles_mn, rest = bid / g.tiles_mn;
  const int tap = rest % g.taps, split = rest / g.taps;
  const long m0 = (long)(tile / g.tiles_n) * BM;
  const long n0 = (long)(tile % g.tiles_n) * BN;
  const long kbeg = (long)split * g.k_per_split;
  const long kend = min(kbeg + g.k_per_split, g.K);
  const int nk = (int)((kend - kbeg + BKT - 1) / BKT);

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // ---------------- staging
  constexpr bool ROWMODE = (AMODE != OP_T);
  // row mode: 16-byte chunks, 8 per row; slot j of a thread: chunk tid + 256*j -> row (tid>>3) + 32*j
  constexpr int NA = ROWMODE ? BM / RPP : 0;  // slots holding A chunks
  constexpr int NB = ROWMODE ? BN / RPP : 0;
  // transposed mode: tasks of 4(k) x 8(cols); 16 k-quads per tile
  constexpr int TASKS_A = 2 * BM, TASKS_B = 2 * BN;
  constexpr int NTASK = ROWMODE ? 0 : (TASKS_A + TASKS_B) / 256;
  // register staging: PF K-tiles in flight (one LDS buffer), one otherwise
  constexpr int NSLOT = ROWMODE ? (NA + NB) : NTASK * 4;
  uint4 rgs[DBUF ? 1 : PF][NSLOT];
  const int kc = tid % CPR;  // row mode: which 8-element chunk of the K-tile
  const int kr = tid / CPR;  // and which row of a pass

  // Row mode: per slot the element offset of the row (without the K position), so that the
  // per-tile address is one add.  Implicit GEMM: offset of the row's own pixel and its (y, x).
  long a_off[ROWMODE ? NA : 1];
  int a_yx[ROWMODE ? NA : 1];
  long b_off[ROWMODE ? NB : 1];
  bool b_ok[ROWMODE ? NB : 1];
  if (ROWMODE) {
    const int HWi = AMODE == A_IM2COL ? g.H * g.W : 1;
#pragma unroll
    for (int j = 0; j < NA; ++j) {
      long row = m0 + kr + RPP * j;
      a_off[j] = 0;
      a_yx[j] = -1;
      if (row < g.M) {
        if (AMODE == A_IM2COL) {
          int rem = (int)(row % HWi);
          int y = rem / g.W;
          a_off[j] = row * g.C;
          a_yx[j] = (y << 16) | (rem - y * g.W);
        } else {
          a_off[j] = row * g.lda + kc * 8;
          a_yx[j] = 0;
        }
      }
    }
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      long row = n0 + kr + RPP * j;
      b_ok[j] = row < g.N;
      b_off[j] = b_ok[j] ? row * g.ldb + kc * 8 : 0;
    }
  }
  // implicit GEMM with C % 64 == 0: the tap and channel offset of the current K-tile, kept as
  // loop-carried uniform state (no division inside the loop)
  // Row mode with a tile-uniform tap (plain rows, or C % 64 == 0): buffer loads.  Per slot the
  // byte offset of the row's own data (the extent = "out of range" for rows past the edge)
  // and, for the implicit GEMM, the set of taps whose shifted pixel lies inside the image.
  constexpr bool BUFPATH = ROWMODE && (AMODE == A_ROW || FASTC);
  unsigned a_voff[BUFPATH ? NA : 1], a_taps[BUFPATH ? NA : 1], b_voff[BUFPATH ? NB : 1];
  const __amdgpu_buffer_rsrc_t rsrcA = make_rsrc(g.A, g.a_bytes), rsrcB = make_rsrc(g.B, g.b_bytes);
  if (BUFPATH) {
#pragma unroll
    for (int j = 0; j < NA; ++j) {
      a_voff[j] = g.a_bytes;
      a_taps[j] = 0;
      if (a_yx[j] >= 0) {
        a_voff[j] = (unsigned)(a_off[j] + (AMODE == A_IM2COL ? kc * 8 : 0)) * 2u;
        if (AMODE == A_IM2COL && g.ksize == 3) {
          const int y = a_yx[j] >> 16, x = a_yx[j] & 0xffff;
          for (int tp = 0; tp < 9; ++tp) {
            const int iy = y + tp / 3 - 1, ix = x + tp % 3 - 1;
            if (iy >= 0 && iy < g.H && ix >= 0 && ix < g.W) a_taps[j] |= 1u << tp;
          }
        } else {
          a_taps[j] = 0xffffffffu;
        }
      }
    }
#pragma unroll
    for (int j = 0; j < NB; ++j) b_voff[j] = b_ok[j] ? (unsigned)b_off[j] * 2u : g.b_bytes;
  }
  // Implicit GEMM with a tile-uniform tap: K runs tap-major ([tap][ci], the layout of the weight
  // copy), the tap and channel offset of the current K-tile are loop-carried uniform state.
  // (Visiting the nine taps of one 64-channel slice back to back, for L1 reuse of the shifted
  // pixels, was measured: same time, 25 % more HBM traffic.)  These launches are never split over K.
  int cur_tap = 0, cur_ci = 0;
  // shifted operand of the conv weight gradient: (y, x) of the first pixel row of each B task
  int t_y[(!ROWMODE && BMODE == B_T_SHIFT) ? NTASK : 1], t_x[(!ROWMODE && BMODE == B_T_SHIFT) ? NTASK : 1];
  // transposed mode, per task: byte offset of its first row in the current K-tile (the tap
  // shift of the conv operand folded in), column validity, rows left before kend
  static_assert(ROWMODE || TASKS_A % 256 == 0, "a task slot must hold one operand only");
  unsigned t_off[ROWMODE ? 1 : NTASK];
  bool t_cv[ROWMODE ? 1 : NTASK];
  int t_rem[ROWMODE ? 1 : NTASK];
  if (!ROWMODE) {
    const int HWi = g.H * g.W;
    const int sh = (BMODE == B_T_SHIFT && g.ksize == 3) ? (tap / 3 - 1) * g.W + tap % 3 - 1 : 0;
#pragma unroll
    for (int j = 0; j < NTASK; ++j) {
      const int t = tid + 256 * j;
      const bool isA = t < TASKS_A;
      const int tt = isA ? t : t - TASKS_A;
      const int per = (isA ? BM : BN) / 8;
      const int kq = tt / per, mc = tt - kq * per;
      const long col = (isA ? m0 : n0) + mc * 8;
      t_cv[j] = col < (isA ? g.M : g.N);
      t_rem[j] = (int)(kend - kbeg) - kq * 4;
      const long row = kbeg + kq * 4 + (isA ? 0 : sh);
      t_off[j] = (unsigned)((row * (isA ? g.lda : g.ldb) + col) * 2);
      if (BMODE == B_T_SHIFT) {
        int rem = (int)((kbeg + kq * 4) % HWi);
        t_y[j] = rem / g.W;
        t_x[j] = rem - t_y[j] * g.W;
      }
    }
  }

  // Loads are unconditional from an always-valid address (the operand base when the element
  // is padding or out of range) and zeroed by a select afterwards: no branches, so the
  // loads of a tile issue back to back.
  auto load_tile = [&](int kt, uint4* rg) {
    const long k0 = kbeg + (long)kt * BKT;
    if (BUFPATH) {
      const bool kv = k0 + kc * 8 < kend;
      unsigned tapbit = 1u, da, db;
      if (AMODE == A_IM2COL) {
        const int dy = g.ksize == 3 ? cur_tap / 3 - 1 : 0, dx = g.ksize == 3 ? cur_tap - (cur_tap / 3) * 3 - 1 : 0;
        tapbit = 1u << cur_tap;
        da = (unsigned)(((dy * g.W + dx) * g.C + cur_ci) * 2);  // may be "negative": wraps back in the sum
        db = (unsigned)((cur_tap * g.C + cur_ci) * 2);
        cur_ci += BK;
        if (cur_ci >= g.C) { cur_ci = 0; ++cur_tap; }
      } else {
        da = db = (unsigned)k0 * 2u;
      }
#pragma unroll
      for (int j = 0; j < NA; ++j)
        rg[j] = buf_load16(rsrcA, (kv && (a_taps[j] & tapbit)) ? a_voff[j] + da : g.a_bytes);
#pragma unroll
      for (int j = 0; j < NB; ++j) rg[NA + j] = buf_load16(rsrcB, kv ? b_voff[j] + db : g.b_bytes);
    } else if (ROWMODE) {
      const long k = k0 + kc * 8;
      const bool kv = k < kend;
      long kb = k0;  // K offset of the tile in the B rows
      int toff = 0, dy = 0, dx = 0;
      if (AMODE == A_IM2COL) {
        int t, ci;
        if (FASTC) {  // uniform over the tile; advanced incrementally
          t = cur_tap;
          ci = cur_ci + kc * 8;
          kb = (long)cur_tap * g.C + cur_ci;
          if (++cur_tap >= g.ksize * g.ksize) { cur_tap = 0; cur_ci += BK; }
        } else {
          t = (int)(k / g.C);
          ci = (int)(k - (long)t * g.C);
        }
        if (g.ksize == 3) { dy = t / 3 - 1; dx = t - (t / 3) * 3 - 1; }
        toff = (dy * g.W + dx) * g.C + ci;
      }
#pragma unroll
      for (int j = 0; j < NA; ++j) {
        bool ok;
        long off;
        if (AMODE == A_ROW) {
          ok = a_yx[j] >= 0 && kv;
          off = a_off[j] + k0;
        } else {
          int iy = (a_yx[j] >> 16) + dy, ix = (a_yx[j] & 0xffff) + dx;
          ok = kv && a_yx[j] >= 0 && iy >= 0 && iy < g.H && ix >= 0 && ix < g.W;
          off = a_off[j] + toff;
        }
        uint4 v = *reinterpret_cast<const uint4*>(g.A + (ok ? off : 0));
        rg[j] = ok ? v : make_uint4(0, 0, 0, 0);
      }
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        const bool ok = b_ok[j] && kv;
        uint4 v = *reinterpret_cast<const uint4*>(g.B + (ok ? b_off[j] + kb : 0));
        rg[NA + j] = ok ? v : make_uint4(0, 0, 0, 0);
      }
    } else {
      (void)k0;
#pragma unroll
      for (int j = 0; j < NTASK; ++j) {
        const bool isA = tid + 256 * j < TASKS_A;  // uniform: TASKS_A is a multiple of the block size
        const unsigned ld2 = (unsigned)(isA ? g.lda : g.ldb) * 2u;
        const unsigned oob = isA ? g.a_bytes : g.b_bytes;
        bool ok[4];
        if (BMODE == B_T_SHIFT && !isA) {
          const int dy = g.ksize == 3 ? tap / 3 - 1 : 0, dx = g.ksize == 3 ? tap % 3 - 1 : 0;
          int y = t_y[j], x = t_x[j];
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            ok[r] = r < t_rem[j] && (unsigned)(y + dy) < (unsigned)g.H && (unsigned)(x + dx) < (unsigned)g.W;
            if (++x >= g.W) { x = 0; if (++y >= g.H) y = 0; }  // next pixel
          }
          // advance the task's first pixel by one K-tile (64 pixels)
          int nx = t_x[j] + g.step_r, ny = t_y[j] + g.step_q;
          if (nx >= g.W) { nx -= g.W; ++ny; }
          while (ny >= g.H) ny -= g.H;
          t_x[j] = nx;
          t_y[j] = ny;
        } else {
#pragma unroll
          for (int r = 0; r < 4; ++r) ok[r] = r < t_rem[j];
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          // the sum is formed here, modulo 2^32: t_off may be "negative" while row r is valid
          const unsigned off = (t_cv[j] && ok[r]) ? t_off[j] + r * ld2 : oob;
          rg[j * 4 + r] = isA ? buf_load16(rsrcA, off) : buf_load16(rsrcB, off);
        }
        t_off[j] += BK * ld2;
        t_rem[j] -= BK;
      }
    }
  };

  auto store_tile = [&](int buf, const uint4* rg) {
    bf16_t* sA = smem + buf * STAGE;
    bf16_t* sB = sA + BM * BKT;
    if (ROWMODE) {
#pragma unroll
      for (int j = 0; j < NA; ++j)
        *reinterpret_cast<uint4*>(&sA[lds_off<BKT>(kr + RPP * j, kc)]) = rg[j];
#pragma unroll
      for (int j = 0; j < NB; ++j)
        *reinterpret_cast<uint4*>(&sB[lds_off<BKT>(kr + RPP * j, kc)]) = rg[NA + j];
    } else {
#pragma unroll
      for (int j = 0; j < NTASK; ++j) {
        int t = tid + 256 * j;
        const bool isA = t < TASKS_A;
        int tt = isA ? t : t - TASKS_A;
        const int per = (isA ? BM : BN) / 8;
        int kq = tt / per, mc = tt - kq * per;
        bf16_t* base = isA ? sA : sB;
        const uint32_t* r0 = reinterpret_cast<const uint32_t*>(&rg[j * 4 + 0]);
        const uint32_t* r1 = reinterpret_cast<const uint32_t*>(&rg[j * 4 + 1]);
        const uint32_t* r2 = reinterpret_cast<const uint32_t*>(&rg[j * 4 + 2]);
        const uint32_t* r3 = reinterpret_cast<const uint32_t*>(&rg[j * 4 + 3]);
#pragma unroll
        for (int w = 0; w < 4; ++w) {  // dword w holds columns 2w (low half) and 2w+1 (high half)
          uint2 lo, hi;
          lo.x = __builtin_amdgcn_perm(r1[w], r0[w], 0x05040100u);  // low halves of rows 0, 1
          lo.y = __builtin_amdgcn_perm(r3[w], r2[w], 0x05040100u);
          hi.x = __builtin_amdgcn_perm(r1[w], r0[w], 0x07060302u);  // high halves
          hi.y = __builtin_amdgcn_perm(r3[w], r2[w], 0x07060302u);
          *reinterpret_cast<uint2*>(base + lds_off<64>(mc * 8 + 2 * w, kq >> 1) + (kq & 1) * 4) = lo;
          *reinterpret_cast<uint2*>(base + lds_off<64>(mc * 8 + 2 * w + 1, kq >> 1) + (kq & 1) * 4) = hi;
        }
      }
    }
  };

  const int lrow = lane & 31, lgrp = lane >> 5;
  auto mma_tile = [&](int buf) {
    const bf16_t* sA = smem + buf * STAGE;
    const bf16_t* sB = sA + BM * BKT;
#pragma unroll
    for (int ks = 0; ks < BKT / 16; ++ks) {
      bf16x8 af[TM], bfr[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        af[i] = *reinterpret_cast<const bf16x8*>(&sA[lds_off<BKT>(wm * WTM + i * 32 + lrow, ks * 2 + lgrp)]);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        bfr[j] = *reinterpret_cast<const bf16x8*>(&sB[lds_off<BKT>(wn * WTN + j * 32 + lrow, ks * 2 + lgrp)]);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          // bf16 output: the B rows as the first operand, so that an accumulator register group holds
          // four consecutive COLUMNS of one output row (packed 8-byte LDS writes in the epilogue);
          // partials: rows and columns as the operands come
          acc[i][j] = EMODE == E_BF16 ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0)
                                      : __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
  };
  if (DBUF) {
    if (nk > 0) {
      load_tile(0, rgs[0]);
      store_tile(0, rgs[0]);
    }
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
      const int buf = kt & 1;
      if (kt + 1 < nk) load_tile(kt + 1, rgs[0]);
      mma_tile(buf);
      if (kt + 1 < nk) store_tile(buf ^ 1, rgs[0]);
      __syncthreads();
    }
  } else {
    // One LDS buffer, PF K-tiles in flight in registers: the loads of tile kt + PF are issued
    // when tile kt has been written to LDS, so a load has PF - 1 whole steps (and the other
    // resident blocks) to land before its registers are needed.
#pragma unroll
    for (int p = 0; p < PF; ++p)
      if (p < nk) load_tile(p, rgs[p]);
    // Steady state without a branch around any load: the compiler's wait counts are exact
    // only then (a conditional load makes it wait for every outstanding one, which would
    // undo the prefetch depth).
    int kt0 = 0;
    for (; kt0 + 2 * PF <= nk; kt0 += PF) {
#pragma unroll
      for (int p = 0; p < PF; ++p) {
        __syncthreads();
        store_tile(0, rgs[p]);
        __syncthreads();
        load_tile(kt0 + p + PF, rgs[p]);
        mma_tile(0);
      }
    }
#pragma unroll
    for (int r = 0; r < 2 * PF; ++r) {  // the last tiles: tile kt0 + r sits in slot r % PF
      const int kt = kt0 + r;
      if (kt < nk) {  // uniform
        __syncthreads();
        store_tile(0, rgs[r % PF]);
        __syncthreads();
        if (kt + PF < nk) load_tile(kt + PF, rgs[r % PF]);
        mma_tile(0);
      }
    }
    __syncthreads();
  }

  // ---------------- epilogue
  if (EMODE == E_PART) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const long n = n0 + wn * WTN + j * 32 + lrow;
        if (n >= g.N) continue;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const long m = m0 + wm * WTM + i * 32 + 8 * (r >> 2) + 4 * lgrp + (r & 3);
          if (m < g.M) g.part[(((long)split * g.taps + tap) * g.M + m) * g.N + n] = acc[i][j][r];
        }
      }
    return;
  }
  // bf16 tile through LDS: [BM][BN + 8]; two passes when the pre-activation is wanted too
  constexpr int CS = BN + 8;
  const int npass = (g.act == ACT_GELU) ? 2 : 1;
  for (int pass = 0; pass < npass; ++pass) {
    if (pass) __syncthreads();
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int ml = wm * WTM + i * 32 + lrow;  // accumulator register r of lane l is C[l % 32][8*(r/4) + 4*(l/32) + r%4]
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const int nl = wn * WTN + j * 32 + 8 * r4 + 4 * lgrp;  // four consecutive columns
          float v[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const long n = n0 + nl + e;
            v[e] = acc[i][j][4 * r4 + e] + ((g.bias && n < g.N) ? g.bias[n] : 0.f);
            if (g.act == ACT_RELU) v[e] = fmaxf(v[e], 0.f);
            if (g.act == ACT_GELU && pass == 1) v[e] = gelu_f(v[e]);
          }
          uint2 pk;
          pk.x = f2bf_pk(v[0], v[1]);
          pk.y = f2bf_pk(v[2], v[3]);
          *reinterpret_cast<uint2*>(&smem[ml * CS + nl]) = pk;
        }
      }
    __syncthreads();
    bf16_t* out = (g.act == ACT_GELU && pass == 0) ? g.pre : g.Cb;
    for (int idx = tid; idx < BM * (BN / 8); idx += 256) {
      int row = idx / (BN / 8), ch = idx - row * (BN / 8);
      long m = m0 + row, n = n0 + ch * 8;
      if (m < g.M && n < g.N) {
        uint4 v = *reinterpret_cast<const uint4*>(&smem[row * CS + ch * 8]);
        if (out == g.Cb && (g.add || g.gmul)) {
          // applied to the bf16-rounded product, exactly as a separate kernel would see it
          const uint4 o = *reinterpret_cast<const uint4*>((g.add ? g.add : g.gmul) + m * g.ldc + n);
          uint32_t* vw = reinterpret_cast<uint32_t*>(&v);
          const uint32_t* ow = reinterpret_cast<const uint32_t*>(&o);
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            float a0 = __uint_as_float(vw[w] << 16), a1 = __uint_as_float(vw[w] & 0xffff0000u);
            const float b0 = __uint_as_float(ow[w] << 16), b1 = __uint_as_float(ow[w] & 0xffff0000u);
            if (g.add) { a0 += b0; a1 += b1; }
            else if (g.gmul_relu) { a0 = b0 > 0.f ? a0 : 0.f; a1 = b1 > 0.f ? a1 : 0.f; }
            else { a0 *= gelu_grad_f(b0); a1 *= gelu_grad_f(b1); }
            vw[w] = f2bf_pk(a0, a1);
          }
        }
        *reinterpret_cast<uint4*>(out + m * g.ldc + n) = v;
      }
    }
  }
}

// G[co][ci][tap] += sum_s part[s][tap][co][ci]   (taps == 1: plain [M][N] accumulate).
// 64 outputs x 4 interleaved split lanes per block, combined through LDS in a fixed order.
__global__ __launch_bounds__(256) void reduce_wgrad_kernel(const float* __restrict__ part,
                                                           float* __restrict__ G, long M, long N, int taps,
                                                           int splits) {
  __shared__ float sh[4][64];
  const int o = threadIdx.x & 63, q = threadIdx.x >> 6;
  const long i = (long)blockIdx.x * 64 + o;
  const long total = (long)taps * M * N;
  float s = 0.f;
  if (i < total) {
    int k = q;
    for (; k + 12 < splits; k += 16) {  // four independent loads in flight
      const float v0 = part[(long)k * total + i], v1 = part[(long)(k + 4) * total + i];
      const float v2 = part[(long)(k + 8) * total + i], v3 = part[(long)(k + 12) * total + i];
      s += (v0 + v1) + (v2 + v3);
    }
    for (; k < splits; k += 4) s += part[(long)k * total + i];
  }
  sh[q][o] = s;
  __syncthreads();
  if (q == 0 && i < total) {
    int t = (int)(i / (M * N));
    long rem = i - (long)t * M * N;  // = co * N + ci
    G[rem * taps + t] += (sh[0][o] + sh[1][o]) + (sh[2][o] + sh[3][o]);
  }
}

// taps == 1 and M*N % 4 == 0: 16-byte loads, one thread per four outputs, every split's load
// issued before the first add; the splits are added in index order.
__global__ __launch_bounds__(256) void reduce_wgrad4_kernel(const float4* __restrict__ part,
                                                            float4* __restrict__ G, long total4, int splits) {
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i >= total4) return;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  int k = 0;
  for (; k + 4 <= splits; k += 4) {
    const float4 v0 = part[(long)k * total4 + i], v1 = part[(long)(k + 1) * total4 + i];
    const float4 v2 = part[(long)(k + 2) * total4 + i], v3 = part[(long)(k + 3) * total4 + i];
    s.x += (v0.x + v1.x) + (v2.x + v3.x);
    s.y += (v0.y + v1.y) + (v2.y + v3.y);
    s.z += (v0.z + v1.z) + (v2.z + v3.z);
    s.w += (v0.w + v1.w) + (v2.w + v3.w);
  }
  for (; k < splits; ++k) {
    const float4 v = part[(long)k * total4 + i];
    s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
  }
  float4 gv = G[i];
  gv.x += s.x; gv.y += s.y; gv.z += s.z; gv.w += s.w;
  G[i] = gv;
}

// column sums of a bf16 [R][C] matrix into fp32: stage 1 partials [S][C], stage 2 accumulate
__global__ __launch_bounds__(256) void colsum_partial_kernel(const bf16_t* __restrict__ g,
                                                             float* __restrict__ part, long R, int C,
                                                             long rows_per_block) {
  // thread -> 8 consecutive columns (one 16-byte load); blockDim.x / (C/8) row lanes
  const int cg = C / 8;
  const int colg = threadIdx.x % cg, rl = threadIdx.x / cg, nrl = blockDim.x / cg;
  const long r0 = (long)blockIdx.x * rows_per_block, r1 = min(r0 + rows_per_block, R);
  float acc[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) acc[k] = 0.f;
  if (rl < nrl) {
    const bf16_t* gc = g + colg * 8;
    for (long r = r0 + rl; r < r1; r += 4 * nrl) {  // four loads in flight
      uint4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const long rr = r + (long)u * nrl;
        v[u] = rr < r1 ? *reinterpret_cast<const uint4*>(gc + rr * C) : make_uint4(0, 0, 0, 0);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const uint32_t* w = reinterpret_cast<const uint32_t*>(&v[u]);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          acc[2 * k] += __uint_as_float(w[k] << 16);
          acc[2 * k + 1] += __uint_as_float(w[k] & 0xffff0000u);
        }
      }
    }
  }
  extern __shared__ float sh[];  // [nrl][C]
  if (rl < nrl)
#pragma unroll
    for (int k = 0; k < 8; ++k) sh[rl * C + colg * 8 + k] = acc[k];
  __syncthreads();
  for (int c = threadIdx.x; c < C; c += blockDim.x) {
    float s = 0.f;
    for (int q = 0; q < nrl; ++q) s += sh[q * C + c];
    part[(long)blockIdx.x * C + c] = s;
  }
}
// 16 columns x 16 interleaved partial lanes per block, butterfly-added in a fixed order
__global__ __launch_bounds__(256) void colsum_final_kernel(const float* __restrict__ part,
                                                           float* __restrict__ G, int C, int S) {
  const int c = blockIdx.x * 16 + (threadIdx.x & 15), q = threadIdx.x >> 4;
  float s = 0.f;
  if (c < C) {
    int k = q;
    for (; k + 48 < S; k += 64) {  // four loads in flight
      const float v0 = part[(long)k * C + c], v1 = part[(long)(k + 16) * C + c];
      const float v2 = part[(long)(k + 32) * C + c], v3 = part[(long)(k + 48) * C + c];
      s += (v0 + v1) + (v2 + v3);
    }
    for (; k < S; k += 16) s += part[(long)k * C + c];
  }
  // lanes with equal (threadIdx.x & 15) inside a wavefront differ by multiples of 16
  s += __shfl_xor(s, 16, 64);
  s += __shfl_xor(s, 32, 64);
  __shared__ float sh[4][16];
  if ((threadIdx.x & 63) < 16) sh[threadIdx.x >> 6][threadIdx.x & 15] = s;
  __syncthreads();
  if (threadIdx.x < 16 && c < C)
    G[c] += (sh[0][threadIdx.x] + sh[1][threadIdx.x]) + (sh[2][threadIdx.x] + sh[3][threadIdx.x]);
}

inline long cdivl(long a, long b) { return (a + b - 1) / b; }

// split count of a weight-gradient product: enough blocks to fill the chip, K ranges of
// at least 16 tiles, multiple of BK.  Every split writes, and the reduction reads, a full copy
// of the gradient: on the transformer stage (K = 4096 rows) 8 splits made 1.2 GB of partial
// traffic per backward pass; 4 measured 6 % faster for the whole step, 2, 3, 5 and 6 slower.
int env_int(const char* name);
int choose_splits(long tiles, long K) {
  static const int target = env_int("ASTEROID_WG_TARGET") > 0 ? env_int("ASTEROID_WG_TARGET") : 768;  // experiment switch
  long want = cdivl(target, tiles);
  long maxs = K / (BK * 16);
  if (maxs < 1) maxs = 1;
  if (want > maxs) want = maxs;
  if (want < 1) want = 1;
  return (int)want;
}

constexpr int WG_T = 64;  // wave tile of the weight-gradient kernels (block tile 128 x 128)

// number of K-splits (= partial copies) launch_wgrad uses
int wgrad_splits(long M, long N, long K, int taps) {
  long tiles = cdivl(M, 2 * WG_T) * cdivl(N, 2 * WG_T) * taps;
  int s = choose_splits(tiles, K);
  long kps = cdivl(cdivl(K, s), BK) * BK;
  return (int)cdivl(K, kps);
}
size_t wgrad_ws_floats(long M, long N, long K, int taps) {
  long tiles = cdivl(M, 2 * WG_T) * cdivl(N, 2 * WG_T) * taps;
  return (size_t)choose_splits(tiles, K) * taps * M * N;
}
// weight partials at ws[0, bias_off), bias partials from ws + bias_off (both 64-float aligned)
static size_t align64f(size_t f) { return (f + 63) / 64 * 64; }
constexpr int kColsumBlocks = 256;
size_t colsum_ws_floats(int C) { return (size_t)kColsumBlocks * C; }

struct ColsumShape { int threads, nrl; long blocks, rpb; };
ColsumShape colsum_shape(long R, int C) {
  // threads: C/8 column groups x row lanes; C up to 8192
  ColsumShape s;
  int cg = C / 8;
  s.threads = cg > 256 ? 1024 : 256;
  s.nrl = s.threads / cg;
  if (s.nrl < 1) s.nrl = 1;
  s.blocks = kColsumBlocks;
  if (s.blocks > cdivl(R, s.nrl)) s.blocks = cdivl(R, s.nrl);
  s.rpb = cdivl(R, s.blocks);
  s.blocks = cdivl(R, s.rpb);
  return s;
}
// partials into ws[blocks][C]; with G the final accumulation follows, else it is the caller's
void launch_colsum(hipStream_t st, const bf16_t* g, float* G, float* ws, long R, int C) {
  const ColsumShape s = colsum_shape(R, C);
  KLAUNCH(colsum_partial_kernel, dim3((unsigned)s.blocks), dim3(s.threads), (size_t)s.nrl * C * sizeof(float), st, g,
          ws, R, C, s.rpb);
  if (G) KLAUNCH(colsum_final_kernel, dim3((unsigned)cdivl(C, 16)), dim3(256), 0, st, ws, G, C, (int)s.blocks);
}

template <int WTM, int WTN, bool DBUF, int BKT = 64>
constexpr size_t lds_bytes() {
  size_t stage = (size_t)(2 * WTM + 2 * WTN) * BKT * sizeof(bf16_t);
  size_t ctile = (size_t)2 * WTM * (2 * WTN + 8) * sizeof(bf16_t);  // output tile of the epilogue
  size_t need = DBUF ? 2 * stage : stage;
  return need > ctile ? need : ctile;
}

// experiment switch: ASTEROID_GEMM_VARIANT=<int> overrides the tile choice of forward-like products
int gemm_variant() {
  static int v = -2;
  if (v == -2) {
    const char* e = getenv("ASTEROID_GEMM_VARIANT");
    v = e ? atoi(e) : -1;
  }
  return v;
}

template <int WTM, int AMODE>
constexpr const char* fwd_name() {
  if (AMODE == A_IM2COL) return WTM == 128 ? "gemm_bf16_kernel<256x128,im2col>" : (WTM == 64 ? "gemm_bf16_kernel<128x128,im2col>" : "gemm_bf16_kernel<64x64,im2col>");
  return WTM == 128 ? "gemm_bf16_kernel<256x128,rows>" : (WTM == 64 ? "gemm_bf16_kernel<128x128,rows>" : "gemm_bf16_kernel<64x64,rows>");
}

template <int WTM, int WTN, int AMODE, bool DBUF, bool FASTC, int PF, int BKT = 64>
void launch_tile_c(hipStream_t st, GemmArgs& g) {
  long tm = cdivl(g.M, 2 * WTM), tn = cdivl(g.N, 2 * WTN);
  g.tiles_n = (int)tn;
  g.tiles_mn = (int)(tm * tn);
  g.taps = 1;
  g.k_per_split = cdivl(g.K, BKT) * BKT;
  g.a_bytes = (unsigned)((AMODE == A_IM2COL ? g.M * g.C : g.M * g.lda) * 2);
  g.b_bytes = (unsigned)(g.N * g.ldb * 2);
  auto kern = gemm_bf16_kernel<WTM, WTN, AMODE, B_ROW, E_BF16, DBUF, FASTC, PF, BKT>;
  constexpr size_t lds = lds_bytes<WTM, WTN, DBUF, BKT>();
  static bool once = false;  // more than 64 KiB of dynamic LDS has to be allowed per kernel
  if (!once) {
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    once = true;
  }
  KLAUNCH_NAMED((fwd_name<WTM, AMODE>()), kern, dim3((unsigned)(tm * tn), 1, 1), dim3(256), lds, st, g);
}

template <int WTM, int WTN, int AMODE, bool DBUF, int PF = 1, int BKT = 64>
void launch_tile(hipStream_t st, GemmArgs& g) {
  if (AMODE == A_IM2COL && !g.fastc) launch_tile_c<WTM, WTN, AMODE, DBUF, false, 1>(st, g);
  else launch_tile_c<WTM, WTN, AMODE, DBUF, true, PF, BKT>(st, g);
}

// experiment switches: ASTEROID_GEMM_PF=<int> overrides the prefetch depth, ASTEROID_GEMM_BK the
// K-tile depth of the plain-row products
int env_int(const char* name) {
  const char* e = getenv(name);
  return e ? atoi(e) : -1;
}
int gemm_pf() {
  static int v = env_int("ASTEROID_GEMM_PF");
  return v;
}
int gemm_bk() {
  static int v = env_int("ASTEROID_GEMM_BK");
  return v;
}

// forward-like products: the largest block tile that still yields >= 256 blocks
template <int AMODE>
void launch_fwd_like(hipStream_t st, GemmArgs& g) {
  auto blocks = [&](int bm, int bn) { return cdivl(g.M, bm) * cdivl(g.N, bn); };
  switch (gemm_variant()) {
    case 1: launch_tile<64, 64, AMODE, true>(st, g); return;
    case 5: launch_tile<128, 64, AMODE, false>(st, g); return;
    default: break;
  }
  const int pf = gemm_pf(), bk = gemm_bk();
  static const int big_min = env_int("ASTEROID_GEMM_BIG") > 0 ? env_int("ASTEROID_GEMM_BIG") : 256;  // experiment switch
  const bool big = blocks(128, 128) >= big_min;
  if constexpr (AMODE == A_ROW) {
    // Deeper K-tiles (fewer, longer steps) were measured on the transformer products
    // (4096 x {512,1536,2048} x {512,2048}): no gain over 64, so they stay an experiment switch.
    if (bk > 64 && g.K >= 256) {
      if (big) {
        if (pf == 2) launch_tile<64, 64, AMODE, false, 2, 128>(st, g);
        else launch_tile<64, 64, AMODE, false, 1, 128>(st, g);
      } else if (bk == 128) {
        if (pf == 1) launch_tile<32, 32, AMODE, false, 1, 128>(st, g);
        else launch_tile<32, 32, AMODE, false, 2, 128>(st, g);
      } else {
        if (pf == 1) launch_tile<32, 32, AMODE, false, 1, 256>(st, g);
        else launch_tile<32, 32, AMODE, false, 2, 256>(st, g);
      }
      return;
    }
  }
  // measured on MI355X: more resident blocks beat bigger tiles (the loop is latency-bound),
  // so the 128x128 tile with one LDS buffer (3 blocks per CU) is the default
  if (big) {
    if (pf == 2) launch_tile<64, 64, AMODE, false, 2>(st, g);
    else launch_tile<64, 64, AMODE, false, 1>(st, g);
  } else {
    if (pf == 1) launch_tile<32, 32, AMODE, false, 1>(st, g);
    else if (pf == 2) launch_tile<32, 32, AMODE, false, 2>(st, g);
    else launch_tile<32, 32, AMODE, false, 4>(st, g);
  }
}

template <int BMODE>
void launch_wgrad(hipStream_t st, GemmArgs& g, float* G, float* ws, int taps) {
  long tm = cdivl(g.M, 2 * WG_T), tn = cdivl(g.N, 2 * WG_T);
  int splits = choose_splits(tm * tn * taps, g.K);
  g.tiles_n = (int)tn;
  g.tiles_mn = (int)(tm * tn);
  g.taps = taps;
  g.k_per_split = cdivl(cdivl(g.K, splits), BK) * BK;
  splits = (int)cdivl(g.K, g.k_per_split);
  g.part = ws;
  g.a_bytes = (unsigned)(g.K * g.lda * 2);
  g.b_bytes = (unsigned)(g.K * g.ldb * 2);
  auto kern = gemm_bf16_kernel<WG_T, WG_T, OP_T, BMODE, E_PART, true, true>;
  constexpr size_t lds = lds_bytes<WG_T, WG_T, true>();
  static bool once = false;
  if (!once) {
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    once = true;
  }
  KLAUNCH_NAMED(BMODE == B_T_SHIFT ? "gemm_bf16_kernel<128x128,wgrad_conv>" : "gemm_bf16_kernel<128x128,wgrad_rows>", kern,
                dim3((unsigned)(tm * tn * taps * splits), 1, 1), dim3(256), lds, st, g);
  long total = (long)taps * g.M * g.N;
  if (!G) return;  // the caller reduces the partials
  // G sits at an arbitrary float offset of the parameter arena: the 16-byte path needs it aligned
  if (taps == 1 && total % 4 == 0 && (reinterpret_cast<uintptr_t>(G) & 15) == 0)
    KLAUNCH(reduce_wgrad4_kernel, dim3((unsigned)cdivl(total / 4, 256)), dim3(256), 0, st,
            reinterpret_cast<const float4*>(ws), reinterpret_cast<float4*>(G), total / 4, splits);
  else
    KLAUNCH(reduce_wgrad_kernel, dim3((unsigned)cdivl(total, 64)), dim3(256), 0, st, ws, G, g.M, g.N, taps, splits);
}

void set_geometry(GemmArgs& g, int H, int W, int C, int k) {
  g.H = H; g.W = W; g.C = C; g.ksize = k;
  g.fastc = (C % BK == 0) ? 1 : 0;
  g.step_q = BK / W;
  g.step_r = BK % W;
}

}  // namespace

// ------------------------------------------------------------------ public launchers
// experiment switch: ASTEROID_WGRAD_TR=0 keeps the conv weight gradients on the generic kernel
static bool conv_wgrad_uses_tr(int N, int H, int W, int Cin, int Cout, int k) {
  static const bool on = env_int("ASTEROID_WGRAD_TR") != 0;
  return on && conv_wgrad_tr_supported(N, H, W, Cin, Cout, k);
}
// floats of weight-gradient partials: room for whichever kernel runs (the choice needs a device,
// the size must not)
static size_t conv_wgrad_part_floats(int N, int H, int W, int Cin, int Cout, int k) {
  const long P = (long)N * H * W;
  const size_t a = wgrad_ws_floats(Cout, Cin, P, k * k);
  const size_t b = (size_t)conv_wgrad_tr_splits(P, Cin, Cout, k * k) * k * k * Cout * Cin;
  return a > b ? a : b;
}
size_t conv_bf16_ws_bytes(int N, int H, int W, int Cin, int Cout, int k) {
  return (align64f(conv_wgrad_part_floats(N, H, W, Cin, Cout, k)) + colsum_ws_floats(Cout)) * sizeof(float) + 256;
}
WgradParts conv_bf16_wgrad_parts(int N, int H, int W, int Cin, int Cout, int k) {
  WgradParts p;
  p.splits = conv_wgrad_uses_tr(N, H, W, Cin, Cout, k) ? conv_wgrad_tr_splits((long)N * H * W, Cin, Cout, k * k)
                                                      : wgrad_splits(Cout, Cin, (long)N * H * W, k * k);
  p.bias_off = align64f(conv_wgrad_part_floats(N, H, W, Cin, Cout, k));
  p.bias_parts = conv_wgrad_uses_tr(N, H, W, Cin, Cout, k) ? p.splits : (int)colsum_shape((long)N * H * W, Cout).blocks;
  return p;
}

// experiment switch: ASTEROID_CONV_HALO=0 keeps the 3x3 products on the generic implicit-GEMM kernel
bool conv_bf16_uses_halo(int N, int H, int W, int Cin, int Cout, int k) {
  static const bool on = env_int("ASTEROID_CONV_HALO") != 0;
  return on && k == 3 && conv3x3_halo_supported(N, H, W, Cin, Cout);
}

void conv_bf16_fwd(hipStream_t st, const bf16_t* x, const bf16_t* sh_fwd, const float* bias, bf16_t* y, int N,
                   int H, int W, int Cin, int Cout, int k, int act) {
  if (conv_bf16_uses_halo(N, H, W, Cin, Cout, k)) {  // sh_fwd is the tiled copy then
    conv3x3_halo_bf16(st, x, sh_fwd, bias, nullptr, y, N, H, W, Cin, Cout, act);
    return;
  }
  GemmArgs g = {};
  g.A = x; g.B = sh_fwd;
  g.M = (long)N * H * W; g.N = Cout; g.K = (long)k * k * Cin;
  g.ldb = g.K;
  set_geometry(g, H, W, Cin, k);
  g.Cb = y; g.ldc = Cout; g.bias = bias; g.act = act;
  launch_fwd_like<A_IM2COL>(st, g);
}

void conv_bf16_dgrad(hipStream_t st, const bf16_t* gy, const bf16_t* sh_dgrad, bf16_t* dx, const bf16_t* relu_out,
                     int N, int H, int W, int Cin, int Cout, int k) {
  // the input gradient is the same product with the roles of the channel counts exchanged
  if (conv_bf16_uses_halo(N, H, W, Cout, Cin, k)) {
    conv3x3_halo_bf16(st, gy, sh_dgrad, nullptr, relu_out, dx, N, H, W, Cout, Cin, 0);
    return;
  }
  GemmArgs g = {};
  g.gmul = relu_out;
  g.gmul_relu = 1;
  g.A = gy; g.B = sh_dgrad;
  g.M = (long)N * H * W; g.N = Cin; g.K = (long)k * k * Cout;
  g.ldb = g.K;
  set_geometry(g, H, W, Cout, k);
  g.Cb = dx; g.ldc = Cin; g.bias = nullptr; g.act = 0;
  launch_fwd_like<A_IM2COL>(st, g);
}

void conv_bf16_wgrad(hipStream_t st, const bf16_t* gy, const bf16_t* x, float* GW, float* Gb, bool has_bias,
                     bool defer, void* ws, int N, int H, int W, int Cin, int Cout, int k) {
  if (conv_wgrad_uses_tr(N, H, W, Cin, Cout, k)) {  // the bias gradient's partials come from the same launch
    float* bias_ws = reinterpret_cast<float*>(ws) + align64f(conv_wgrad_part_floats(N, H, W, Cin, Cout, k));
    const int splits = conv_wgrad_tr_splits((long)N * H * W, Cin, Cout, k * k);
    conv_wgrad_tr_bf16(st, gy, x, reinterpret_cast<float*>(ws), has_bias ? bias_ws : nullptr, N, H, W, Cin, Cout, k);
    if (!defer) {
      const long total = (long)k * k * Cout * Cin;
      KLAUNCH(reduce_wgrad_kernel, dim3((unsigned)cdivl(total, 64)), dim3(256), 0, st, reinterpret_cast<const float*>(ws), GW,
              (long)Cout, (long)Cin, k * k, splits);
      if (has_bias) KLAUNCH(colsum_final_kernel, dim3((unsigned)cdivl(Cout, 16)), dim3(256), 0, st, bias_ws, Gb, Cout, splits);
    }
    return;
  } else {
    GemmArgs g = {};
    g.A = gy; g.B = x;
    g.M = Cout; g.N = Cin; g.K = (long)N * H * W;
    g.lda = Cout; g.ldb = Cin;
    set_geometry(g, H, W, Cin, k);
    launch_wgrad<B_T_SHIFT>(st, g, defer ? nullptr : GW, reinterpret_cast<float*>(ws), k * k);
  }
  if (has_bias)
    launch_colsum(st, gy, defer ? nullptr : Gb,
                  reinterpret_cast<float*>(ws) + align64f(conv_wgrad_part_floats(N, H, W, Cin, Cout, k)),
                  (long)N * H * W, Cout);
}

size_t linear_bf16_ws_bytes(size_t R, int Cin, int Cout) {
  return (align64f(wgrad_ws_floats(Cout, Cin, (long)R, 1)) + colsum_ws_floats(Cout)) * sizeof(float) + 256;
}
WgradParts linear_bf16_wgrad_parts(size_t R, int Cin, int Cout) {
  WgradParts p;
  p.splits = wgrad_splits(Cout, Cin, (long)R, 1);
  p.bias_off = align64f(wgrad_ws_floats(Cout, Cin, (long)R, 1));
  p.bias_parts = (int)colsum_shape((long)R, Cout).blocks;
  return p;
}

void linear_bf16_fwd(hipStream_t st, const bf16_t* x, const bf16_t* sh, const float* bias, bf16_t* y, bf16_t* pre,
                     const bf16_t* add, size_t R, int Cin, int Cout, int act) {
  if (linear_dl_supported(R, Cin, Cout)) {
    linear_dl_bf16(st, x, sh, bias, y, pre, add, nullptr, R, Cin, Cout, act);
    return;
  }
  GemmArgs g = {};
  g.add = add;
  g.A = x; g.B = sh;
  g.M = (long)R; g.N = Cout; g.K = Cin; g.lda = Cin; g.ldb = Cin;
  g.Cb = y; g.pre = pre; g.ldc = Cout; g.bias = bias; g.act = act;
  launch_fwd_like<A_ROW>(st, g);
}

void linear_bf16_dgrad(hipStream_t st, const bf16_t* gy, const bf16_t* sh_t, bf16_t* dx, const bf16_t* gelu_pre,
                       const bf16_t* add, size_t R, int Cin, int Cout) {
  if (linear_dl_supported(R, Cout, Cin)) {
    linear_dl_bf16(st, gy, sh_t, nullptr, dx, nullptr, add, gelu_pre, R, Cout, Cin, 0);
    return;
  }
  GemmArgs g = {};
  g.gmul = gelu_pre;  // at most one of the two is given
  g.add = add;
  g.A = gy; g.B = sh_t;
  g.M = (long)R; g.N = Cin; g.K = Cout; g.lda = Cout; g.ldb = Cout;
  g.Cb = dx; g.ldc = Cin; g.act = 0;
  launch_fwd_like<A_ROW>(st, g);
}

void linear_bf16_wgrad(hipStream_t st, const bf16_t* gy, const bf16_t* x, float* GW, float* Gb, bool has_bias,
                       bool defer, void* ws, size_t R, int Cin, int Cout) {
  GemmArgs g = {};
  g.A = gy; g.B = x;
  g.M = Cout; g.N = Cin; g.K = (long)R; g.lda = Cout; g.ldb = Cin;
  set_geometry(g, 1, 1, Cin, 1);
  launch_wgrad<OP_T>(st, g, defer ? nullptr : GW, reinterpret_cast<float*>(ws), 1);
  if (has_bias)
    launch_colsum(st, gy, defer ? nullptr : Gb,
                  reinterpret_cast<float*>(ws) + align64f(wgrad_ws_floats(Cout, Cin, (long)R, 1)), (long)R, Cout);
}

}  // namespace ast
