// bf16 x bf16 -> fp32 matrix products on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16),
// LDS-staged, serving the dense layers of the VGG-style and transformer stages:
//   linear forward / input gradient            C[m][n] = sum_k A[m][k] B[n][k]
//   3x3 / 1x1 'same' convolution, NHWC         A gathered on the fly (implicit GEMM)
//   weight gradients                           C[m][n] = sum_k A[k][m] B[k][n], K = rows/pixels,
//                                              split over K, deterministic fp32 reduction into G
//
// Block = 256 threads = 2 x 2 wavefronts; each wavefront owns a WTM x WTN tile made of
// 32x32 MFMA tiles.  Both operands sit in LDS as [row][k] with k contiguous (row stride 40
// elements = 80 bytes, which spreads the 16-byte operand reads of 8 consecutive lanes over
// all banks).  MFMA 32x32x16: lane l supplies A[l%32][8*(l/32) .. +7] and B likewise;
// accumulator register r of lane l is D[8*(r/4) + 4*(l/32) + r%4][l%32].
// Operands stored with the contraction index strided (weight gradients) are transposed in
// registers (4 x 8 blocks) on their way into LDS.
// Global loads of the next K-tile are issued before the MFMAs of the current one.
#include "device_utils.h"
#include "kernels_bf16.h"
#include "prof.h"

namespace ast {

namespace {

constexpr int BK = 32;
constexpr int LDS_STRIDE = 40;  // elements per LDS row

enum { A_ROW = 0, A_IM2COL = 1, OP_T = 2, B_ROW = 0, B_T_SHIFT = 3 };
enum { E_BF16 = 0, E_PART = 1 };

struct GemmArgs {
  const bf16_t* A;
  const bf16_t* B;
  long M, N, K;
  long lda, ldb;
  int H, W, C, ksize;  // image geometry of the gathered / shifted operand
  long k_per_split;    // K range per blockIdx.z (multiple of BK)
  // epilogue
  bf16_t* Cb;          // bf16 output [M][ldc]
  bf16_t* pre;         // optional pre-activation copy
  float* part;         // fp32 partials [split][tap][M][N]
  long ldc;
  const float* bias;
  int act;
  int tiles_n;         // number of tiles along N (blockIdx.x = tile_m * tiles_n + tile_n)
};

__device__ __forceinline__ float gelu_f(float x) { return 0.5f * x * (1.f + erff(x * 0.70710678118654752f)); }

template <int WTM, int WTN, int AMODE, int BMODE, int EMODE>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmArgs g) {
  constexpr int BM = 2 * WTM, BN = 2 * WTN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  __shared__ __attribute__((aligned(16))) bf16_t sA[BM * LDS_STRIDE];
  __shared__ __attribute__((aligned(16))) bf16_t sB[BN * LDS_STRIDE];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const long m0 = (long)(blockIdx.x / g.tiles_n) * BM;
  const long n0 = (long)(blockIdx.x % g.tiles_n) * BN;
  const int tap = blockIdx.y;  // weight-gradient of a 3x3 conv: one tap per blockIdx.y
  const long kbeg = (long)blockIdx.z * g.k_per_split;
  const long kend = min(kbeg + g.k_per_split, g.K);
  const int nk = (int)((kend - kbeg + BK - 1) / BK);

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // ---------------- staging registers
  constexpr bool ROWMODE = (AMODE != OP_T);
  // row mode: 16-byte chunks; chunk c -> row c/4, k-chunk c%4
  constexpr int NCH = ROWMODE ? (BM + BN) * 4 / 256 : 0;
  // transposed mode: tasks of 4(k) x 8(m); task t -> kq = t / (rows/8), mc = t % (rows/8)
  constexpr int NTASK = ROWMODE ? 0 : (BM + BN) / 256;
  uint4 rg[ROWMODE ? NCH : NTASK * 4];

  // per-chunk pixel coordinates of the implicit-GEMM A operand (fixed over K tiles)
  int pix_y[AMODE == A_IM2COL ? NCH : 1], pix_x[AMODE == A_IM2COL ? NCH : 1];
  long pix_n[AMODE == A_IM2COL ? NCH : 1];
  if (AMODE == A_IM2COL) {
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
      int c = tid + 256 * j;
      if (c < BM * 4) {
        long row = m0 + (c >> 2);
        if (row < g.M) {
          long n = row / ((long)g.H * g.W);
          int rem = (int)(row - n * g.H * g.W);
          pix_n[j] = n;
          pix_y[j] = rem / g.W;
          pix_x[j] = rem - pix_y[j] * g.W;
        } else {
          pix_n[j] = -1; pix_y[j] = 0; pix_x[j] = 0;
        }
      }
    }
  }

  auto load_tile = [&](int kt) {
    const long k0 = kbeg + (long)kt * BK;
    if (ROWMODE) {
#pragma unroll
      for (int j = 0; j < NCH; ++j) {
        int c = tid + 256 * j;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (c < BM * 4) {
          long k = k0 + (c & 3) * 8;
          if (AMODE == A_ROW) {
            long row = m0 + (c >> 2);
            if (row < g.M && k < kend) v = *reinterpret_cast<const uint4*>(g.A + row * g.lda + k);
          } else {  // implicit GEMM: k = tap * C + ci over the NHWC image
            if (pix_n[j] >= 0 && k < kend) {
              int t = (int)(k / g.C);
              int ci = (int)(k - (long)t * g.C);
              int dy = 0, dx = 0;
              if (g.ksize == 3) { dy = t / 3 - 1; dx = t - (t / 3) * 3 - 1; }
              int iy = pix_y[j] + dy, ix = pix_x[j] + dx;
              if (iy >= 0 && iy < g.H && ix >= 0 && ix < g.W)
                v = *reinterpret_cast<const uint4*>(g.A + ((pix_n[j] * g.H + iy) * g.W + ix) * g.C + ci);
            }
          }
        } else {
          int cb = c - BM * 4;
          long row = n0 + (cb >> 2);
          long k = k0 + (cb & 3) * 8;
          if (row < g.N && k < kend) v = *reinterpret_cast<const uint4*>(g.B + row * g.ldb + k);
        }
        rg[j] = v;
      }
    } else {
#pragma unroll
      for (int j = 0; j < NTASK; ++j) {
        int t = tid + 256 * j;
        const bool isA = t < BM;
        int tt = isA ? t : t - BM;
        const int per = (isA ? BM : BN) / 8;
        int kq = tt / per, mc = tt - kq * per;
        long col = (isA ? m0 : n0) + mc * 8;
        const long ncols = isA ? g.M : g.N;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          long k = k0 + kq * 4 + r;  // contraction index = matrix row (a pixel or a token)
          uint4 v = make_uint4(0, 0, 0, 0);
          if (k < kend && col < ncols) {
            if (isA) {
              v = *reinterpret_cast<const uint4*>(g.A + k * g.lda + col);
            } else if (BMODE == B_T_SHIFT) {
              long n = k / ((long)g.H * g.W);
              int rem = (int)(k - n * g.H * g.W);
              int y = rem / g.W, x = rem - y * g.W;
              int iy = y + tap / 3 - 1, ix = x + tap % 3 - 1;
              if (g.ksize == 1) { iy = y; ix = x; }
              if (iy >= 0 && iy < g.H && ix >= 0 && ix < g.W)
                v = *reinterpret_cast<const uint4*>(g.B + ((n * g.H + iy) * g.W + ix) * g.ldb + col);
            } else {
              v = *reinterpret_cast<const uint4*>(g.B + k * g.ldb + col);
            }
          }
          rg[j * 4 + r] = v;
        }
      }
    }
  };

  auto store_tile = [&]() {
    if (ROWMODE) {
#pragma unroll
      for (int j = 0; j < NCH; ++j) {
        int c = tid + 256 * j;
        if (c < BM * 4)
          *reinterpret_cast<uint4*>(&sA[(c >> 2) * LDS_STRIDE + (c & 3) * 8]) = rg[j];
        else {
          int cb = c - BM * 4;
          *reinterpret_cast<uint4*>(&sB[(cb >> 2) * LDS_STRIDE + (cb & 3) * 8]) = rg[j];
        }
      }
    } else {
#pragma unroll
      for (int j = 0; j < NTASK; ++j) {
        int t = tid + 256 * j;
        const bool isA = t < BM;
        int tt = isA ? t : t - BM;
        const int per = (isA ? BM : BN) / 8;
        int kq = tt / per, mc = tt - kq * per;
        bf16_t* dst = (isA ? sA : sB) + (mc * 8) * LDS_STRIDE + kq * 4;
        const uint32_t* r0 = reinterpret_cast<const uint32_t*>(&rg[j * 4 + 0]);
        const uint32_t* r1 = reinterpret_cast<const uint32_t*>(&rg[j * 4 + 1]);
        const uint32_t* r2 = reinterpret_cast<const uint32_t*>(&rg[j * 4 + 2]);
        const uint32_t* r3 = reinterpret_cast<const uint32_t*>(&rg[j * 4 + 3]);
#pragma unroll
        for (int w = 0; w < 4; ++w) {  // dword w holds columns 2w (low half) and 2w+1 (high half)
          uint2 lo, hi;
          lo.x = (r0[w] & 0xffffu) | (r1[w] << 16);
          lo.y = (r2[w] & 0xffffu) | (r3[w] << 16);
          hi.x = (r0[w] >> 16) | (r1[w] & 0xffff0000u);
          hi.y = (r2[w] >> 16) | (r3[w] & 0xffff0000u);
          *reinterpret_cast<uint2*>(dst + (2 * w) * LDS_STRIDE) = lo;
          *reinterpret_cast<uint2*>(dst + (2 * w + 1) * LDS_STRIDE) = hi;
        }
      }
    }
  };

  const int lrow = lane & 31, lgrp = lane >> 5;
  if (nk > 0) load_tile(0);
  for (int kt = 0; kt < nk; ++kt) {
    __syncthreads();
    store_tile();
    __syncthreads();
    if (kt + 1 < nk) load_tile(kt + 1);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 af[TM], bfr[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        af[i] = *reinterpret_cast<const bf16x8*>(&sA[(wm * WTM + i * 32 + lrow) * LDS_STRIDE + ks * 16 + lgrp * 8]);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        bfr[j] = *reinterpret_cast<const bf16x8*>(&sB[(wn * WTN + j * 32 + lrow) * LDS_STRIDE + ks * 16 + lgrp * 8]);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
  }

  // ---------------- epilogue
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const long n = n0 + wn * WTN + j * 32 + lrow;
      if (n >= g.N) continue;
      const float bv = (EMODE == E_BF16 && g.bias) ? g.bias[n] : 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const long m = m0 + wm * WTM + i * 32 + 8 * (r >> 2) + 4 * lgrp + (r & 3);
        if (m >= g.M) continue;
        float v = acc[i][j][r];
        if (EMODE == E_BF16) {
          v += bv;
          if (g.act == ACT_RELU) v = fmaxf(v, 0.f);
          if (g.act == ACT_GELU) {
            g.pre[m * g.ldc + n] = f2bf(v);
            v = gelu_f(v);
          }
          g.Cb[m * g.ldc + n] = f2bf(v);
        } else {
          g.part[(((long)blockIdx.z * gridDim.y + tap) * g.M + m) * g.N + n] = v;
        }
      }
    }
  }
}

// G[co][ci][tap] += sum_s part[s][tap][co][ci]   (taps == 1: plain [M][N] accumulate)
__global__ void reduce_wgrad_kernel(const float* __restrict__ part, float* __restrict__ G, long M, long N,
                                    int taps, int splits) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  long total = (long)taps * M * N;
  if (i >= total) return;
  int t = (int)(i / (M * N));
  long rem = i - (long)t * M * N;  // = co * N + ci
  float s = 0.f;
  for (int k = 0; k < splits; ++k) s += part[(long)k * total + i];
  G[rem * taps + t] += s;
}

// column sums of a bf16 [R][C] matrix into fp32: stage 1 partials [S][C], stage 2 accumulate
__global__ __launch_bounds__(256) void colsum_partial_kernel(const bf16_t* __restrict__ g,
                                                             float* __restrict__ part, long R, int C,
                                                             long rows_per_block) {
  // thread -> 8 consecutive columns (one 16-byte load); blockDim.x/ (C/8) row lanes
  const int cg = C / 8;
  const int colg = threadIdx.x % cg, rl = threadIdx.x / cg, nrl = blockDim.x / cg;
  const long r0 = (long)blockIdx.x * rows_per_block, r1 = min(r0 + rows_per_block, R);
  float acc[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) acc[k] = 0.f;
  if (rl < nrl) {
    for (long r = r0 + rl; r < r1; r += nrl) {
      uint4 v = *reinterpret_cast<const uint4*>(g + r * C + colg * 8);
      const uint32_t* w = reinterpret_cast<const uint32_t*>(&v);
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        acc[2 * k] += __uint_as_float(w[k] << 16);
        acc[2 * k + 1] += __uint_as_float(w[k] & 0xffff0000u);
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
__global__ void colsum_final_kernel(const float* __restrict__ part, float* __restrict__ G, int C, int S) {
  int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= C) return;
  float s = 0.f;
  for (int k = 0; k < S; ++k) s += part[(long)k * C + c];
  G[c] += s;
}

inline long cdivl(long a, long b) { return (a + b - 1) / b; }

// split count of a weight-gradient product: enough blocks to fill the chip, K ranges of
// at least 8 tiles, multiple of BK
int choose_splits(long tiles, long K) {
  long want = cdivl(768, tiles);
  long maxs = K / (BK * 8);
  if (maxs < 1) maxs = 1;
  if (want > maxs) want = maxs;
  if (want < 1) want = 1;
  return (int)want;
}

constexpr int WG_T = 64;  // wave tile of the weight-gradient kernels (block tile 128 x 128)

size_t wgrad_ws_floats(long M, long N, long K, int taps) {
  long tiles = cdivl(M, 2 * WG_T) * cdivl(N, 2 * WG_T) * taps;
  int s = choose_splits(tiles, K);
  return (size_t)s * taps * M * N;
}
constexpr int kColsumBlocks = 256;
size_t colsum_ws_floats(int C) { return (size_t)kColsumBlocks * C; }

void launch_colsum(hipStream_t st, const bf16_t* g, float* G, float* ws, long R, int C) {
  // threads: C/8 column groups x row lanes; C up to 8192
  int cg = C / 8;
  int threads = 256;
  if (cg > 256) threads = 1024;
  int nrl = threads / cg;
  if (nrl < 1) nrl = 1;
  long blocks = kColsumBlocks;
  if (blocks > cdivl(R, nrl)) blocks = cdivl(R, nrl);
  long rpb = cdivl(R, blocks);
  blocks = cdivl(R, rpb);
  KLAUNCH(colsum_partial_kernel, dim3((unsigned)blocks), dim3(threads), (size_t)nrl * C * sizeof(float), st, g, ws, R,
          C, rpb);
  KLAUNCH(colsum_final_kernel, dim3((unsigned)cdivl(C, 256)), dim3(256), 0, st, ws, G, C, (int)blocks);
}

template <int AMODE>
void launch_fwd_like(hipStream_t st, GemmArgs& g) {
  // block tile 128 x 128 (4 wavefronts of 64 x 64)
  constexpr int WT = 64;
  long tm = cdivl(g.M, 2 * WT), tn = cdivl(g.N, 2 * WT);
  g.tiles_n = (int)tn;
  g.k_per_split = cdivl(g.K, BK) * BK;
  KLAUNCH((gemm_bf16_kernel<WT, WT, AMODE, B_ROW, E_BF16>), dim3((unsigned)(tm * tn), 1, 1), dim3(256), 0, st, g);
}

template <int BMODE>
void launch_wgrad(hipStream_t st, GemmArgs& g, float* G, float* ws, int taps) {
  long tm = cdivl(g.M, 2 * WG_T), tn = cdivl(g.N, 2 * WG_T);
  int splits = choose_splits(tm * tn * taps, g.K);
  g.tiles_n = (int)tn;
  g.k_per_split = cdivl(cdivl(g.K, splits), BK) * BK;
  splits = (int)cdivl(g.K, g.k_per_split);
  g.part = ws;
  KLAUNCH((gemm_bf16_kernel<WG_T, WG_T, OP_T, BMODE, E_PART>), dim3((unsigned)(tm * tn), taps, splits), dim3(256), 0,
          st, g);
  long total = (long)taps * g.M * g.N;
  KLAUNCH(reduce_wgrad_kernel, dim3((unsigned)cdivl(total, 256)), dim3(256), 0, st, ws, G, g.M, g.N, taps, splits);
}

}  // namespace

// ------------------------------------------------------------------ public launchers
size_t conv_bf16_ws_bytes(int N, int H, int W, int Cin, int Cout, int k) {
  size_t a = wgrad_ws_floats(Cout, Cin, (long)N * H * W, k * k);
  size_t b = colsum_ws_floats(Cout);
  return (a > b ? a : b) * sizeof(float) + 256;
}

void conv_bf16_fwd(hipStream_t st, const bf16_t* x, const bf16_t* sh_fwd, const float* bias, bf16_t* y, int N,
                   int H, int W, int Cin, int Cout, int k, int act) {
  GemmArgs g = {};
  g.A = x; g.B = sh_fwd;
  g.M = (long)N * H * W; g.N = Cout; g.K = (long)k * k * Cin;
  g.ldb = g.K; g.H = H; g.W = W; g.C = Cin; g.ksize = k;
  g.Cb = y; g.ldc = Cout; g.bias = bias; g.act = act;
  launch_fwd_like<A_IM2COL>(st, g);
}

void conv_bf16_dgrad(hipStream_t st, const bf16_t* gy, const bf16_t* sh_dgrad, bf16_t* dx, int N, int H, int W,
                     int Cin, int Cout, int k) {
  GemmArgs g = {};
  g.A = gy; g.B = sh_dgrad;
  g.M = (long)N * H * W; g.N = Cin; g.K = (long)k * k * Cout;
  g.ldb = g.K; g.H = H; g.W = W; g.C = Cout; g.ksize = k;
  g.Cb = dx; g.ldc = Cin; g.bias = nullptr; g.act = 0;
  launch_fwd_like<A_IM2COL>(st, g);
}

void conv_bf16_wgrad(hipStream_t st, const bf16_t* gy, const bf16_t* x, float* GW, float* Gb, void* ws, int N,
                     int H, int W, int Cin, int Cout, int k) {
  GemmArgs g = {};
  g.A = gy; g.B = x;
  g.M = Cout; g.N = Cin; g.K = (long)N * H * W;
  g.lda = Cout; g.ldb = Cin; g.H = H; g.W = W; g.C = Cin; g.ksize = k;
  launch_wgrad<B_T_SHIFT>(st, g, GW, reinterpret_cast<float*>(ws), k * k);
  if (Gb) launch_colsum(st, gy, Gb, reinterpret_cast<float*>(ws), (long)N * H * W, Cout);
}

size_t linear_bf16_ws_bytes(size_t R, int Cin, int Cout) {
  size_t a = wgrad_ws_floats(Cout, Cin, (long)R, 1);
  size_t b = colsum_ws_floats(Cout);
  return (a > b ? a : b) * sizeof(float) + 256;
}

void linear_bf16_fwd(hipStream_t st, const bf16_t* x, const bf16_t* sh, const float* bias, bf16_t* y, bf16_t* pre,
                     size_t R, int Cin, int Cout, int act) {
  GemmArgs g = {};
  g.A = x; g.B = sh;
  g.M = (long)R; g.N = Cout; g.K = Cin; g.lda = Cin; g.ldb = Cin;
  g.Cb = y; g.pre = pre; g.ldc = Cout; g.bias = bias; g.act = act;
  launch_fwd_like<A_ROW>(st, g);
}

void linear_bf16_dgrad(hipStream_t st, const bf16_t* gy, const bf16_t* sh_t, bf16_t* dx, size_t R, int Cin,
                       int Cout) {
  GemmArgs g = {};
  g.A = gy; g.B = sh_t;
  g.M = (long)R; g.N = Cin; g.K = Cout; g.lda = Cout; g.ldb = Cout;
  g.Cb = dx; g.ldc = Cin; g.act = 0;
  launch_fwd_like<A_ROW>(st, g);
}

void linear_bf16_wgrad(hipStream_t st, const bf16_t* gy, const bf16_t* x, float* GW, float* Gb, void* ws,
                       size_t R, int Cin, int Cout) {
  GemmArgs g = {};
  g.A = gy; g.B = x;
  g.M = Cout; g.N = Cin; g.K = (long)R; g.lda = Cout; g.ldb = Cin; g.ksize = 1; g.H = 1; g.W = 1;
  launch_wgrad<OP_T>(st, g, GW, reinterpret_cast<float*>(ws), 1);
  if (Gb) launch_colsum(st, gy, Gb, reinterpret_cast<float*>(ws), (long)R, Cout);
}

}  // namespace ast
