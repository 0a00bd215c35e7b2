// fp32 dense convolutions on the matrix cores for the ResNet workload (Table 4): 3x3 with padding 1
// and stride 1 or 2, and the 1x1 stride-2 projection of a shortcut.  The KS*KS taps are KS*KS
// pointwise products accumulated in the same registers.
//
// Forward / input gradient: as the pointwise kernel -- a wavefront owns 32 pixels of the result and
// one or two 32-row tiles of its channels, MFMA 32x32x2 with the pixels on the N dimension, the B
// operand straight from global memory -- but the operand pixel of tap (u, v) is, forward, the
// result pixel times the stride shifted by (u, v) minus the padding, and, for the input gradient,
// the output pixel ((r + pad - u) / stride, (c + pad - v) / stride) where that division is exact;
// zero outside the tensor.  The A operand of tap t comes from the t-th packed weight copy (one set
// of KS*KS copies per direction).
// Weight gradient: as the pointwise weight-gradient kernel (output pixels are the contraction
// index), one block per (pixel chunk, 32x32 tile of (cout, cin)) with KS*KS accumulator tiles, one
// per tap: g is loaded once per pass, x once per tap, shifted, strided and masked.
// Partials per pixel chunk, layout [chunk][cout][cin][tap] = the layout of the weights.
#include "device_utils.h"
#include "kernels.h"
#include "prof.h"

namespace ast {

namespace {

inline int cdiv(long a, long b) { return (int)((a + b - 1) / b); }

// Block coordinates from the flat block id with the tiles of one pixel block (or pixel chunk)
// fastest inside XCD-grouped ids: the blocks that read the same pixels run side by side on one XCD
// and share its L2.  gx = pixel blocks, gt = tiles.
__device__ __forceinline__ void tile_fastest(unsigned gx, unsigned gt, int& bx, int& t) {
  const unsigned flat = (blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x;
  const unsigned id = xcd_grouped(flat, gx * gt);
  t = (int)(id % gt);
  bx = (int)(id / gt);
}

struct C3Args {
  const float4* Wp;   // KS*KS packed copies, tap_stride float4 words apart
  const float* X;     // operand tensor [N][Kdim][XH][XW]
  float* Y;           // result tensor  [N][Mdim][PH][PW]
  const float* bias;
  long NQ;            // N * PH * PW
  int PH, PW, XH, XW, S, Kdim, Mdim, KG;
  size_t tap_stride;
};

// MT = 32-row tiles of result channels per wavefront (1 or 2): with two, a pixel operand loaded once
// feeds both tiles.  DGRAD: the operand is the upstream gradient (see the file comment).
template <int NCH, int MT, int KS, bool DGRAD>
__global__ __launch_bounds__(256) void conv_mfma_f32_kernel(C3Args a) {
  constexpr int PAD = KS / 2;
  const float4* __restrict__ Wp = a.Wp;
  const float* __restrict__ X = a.X;
  float* __restrict__ Y = a.Y;
  const int PW = a.PW, PHW = a.PH * a.PW, XH = a.XH, XW = a.XW, XHW = a.XH * a.XW, S = a.S;
  const int Kdim = a.Kdim, Mdim = a.Mdim, KG = a.KG;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 31, half = lane >> 5;
  int bx, by;
  tile_fastest(gridDim.x, gridDim.y, bx, by);
  const int tile0 = by * MT;  // first 32-row tile of this block
  const unsigned q = (unsigned)bx * 128u + wave * 32 + col;  // pixels per micro-batch < 2^31 (checked at create)
  const bool qv = q < a.NQ;
  unsigned n = 0;
  int p = 0;
  if (qv) {
    n = q / (unsigned)PHW;  // 32-bit: a 64-bit division is ~150 instructions
    p = (int)(q - n * (unsigned)PHW);
  }
  const int pi = p / PW, pj = p - pi * PW;
  const float* xn = X + (size_t)n * Kdim * XHW;
  const float4* wl = Wp + (size_t)tile0 * KG * 64 + lane;
  const bool t1 = MT > 1 && (tile0 + 1) * 32 < Mdim;  // the second tile exists (uniform)
  floatx16 acc[MT];
#pragma unroll
  for (int m = 0; m < MT; ++m)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[m][r] = 0.f;
  for (int tap = 0; tap < KS * KS; ++tap) {
    const int u = tap / KS, v = tap - u * KS;
    int xr, xc;
    bool ok = qv;
    if (DGRAD) {
      const int ar = pi + PAD - u, ac = pj + PAD - v;
      ok = ok && ar >= 0 && ac >= 0;
      xr = S == 1 ? ar : ar >> 1;
      xc = S == 1 ? ac : ac >> 1;
      if (S == 2) ok = ok && !((ar | ac) & 1);
    } else {
      xr = pi * S - PAD + u;
      xc = pj * S - PAD + v;
      ok = ok && xr >= 0 && xc >= 0;
    }
    ok = ok && xr < XH && xc < XW;
    // branch-free operand loads: a tap outside the tensor reads pixel 0 and is replaced by zero, rows
    // past Kdim read the last row (they meet zero weights in the packed copy)
    const float* xt = xn + (ok ? xr * XW + xc : 0);
    const float4* wt = wl + (size_t)tap * a.tap_stride;
    for (int g0 = 0; g0 < KG; g0 += NCH * 4) {
      float4 av[MT][NCH * 4];
      float b[NCH * 16];
#pragma unroll
      for (int g = 0; g < NCH * 4; ++g) {
        const bool gv = g0 + g < KG;
        av[0][g] = gv ? wt[(size_t)(g0 + g) * 64] : make_float4(0.f, 0.f, 0.f, 0.f);
        if (MT > 1) av[MT - 1][g] = (gv && t1) ? wt[(size_t)(KG + g0 + g) * 64] : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int k = min((g0 + g) * 8 + 2 * e + half, Kdim - 1);
          const float val = xt[(size_t)k * XHW];
          b[4 * g + e] = ok ? val : 0.f;
        }
      }
#pragma unroll
      for (int g = 0; g < NCH * 4; ++g) {
        if (g0 + g >= KG) break;  // uniform
#pragma unroll
        for (int m = 0; m < MT; ++m) {
          acc[m] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[m][g].x, b[4 * g + 0], acc[m], 0, 0, 0);
          acc[m] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[m][g].y, b[4 * g + 1], acc[m], 0, 0, 0);
          acc[m] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[m][g].z, b[4 * g + 2], acc[m], 0, 0, 0);
          acc[m] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[m][g].w, b[4 * g + 3], acc[m], 0, 0, 0);
        }
      }
    }
  }
  if (qv) {
    float* yq = Y + (size_t)n * Mdim * PHW + p;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = (tile0 + mt) * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
        if (m < Mdim) yq[(size_t)m * PHW] = acc[mt][r] + (a.bias ? a.bias[m] : 0.f);
      }
  }
}

struct C3WgArgs {
  const float* g;   // [N][Cout][Ho][Wo]
  const float* x;   // [N][Cin][H][W]
  float* part;
  int Cin, Cout, H, W, Ho, Wo, S, cps, pxw;
};

// Block (chunk of output pixels, ci tile, co tile), all KS*KS taps: a pass loads 16 pixel pairs of g
// once and, per tap, the shifted, strided, masked pixels of x (cache hits after the first tap),
// 16 MFMAs per tap into that tap's accumulator tile.  Wavefront w of the block takes the w-th
// quarter of the chunk; the four wavefronts' tiles are added through LDS, tap after tap.
template <int KS>
__global__ __launch_bounds__(256) void conv_wgrad_mfma_f32_kernel(C3WgArgs w) {
  constexpr int PAD = KS / 2, KK = KS * KS;
  __shared__ float sR[4][16][64];
  const float* __restrict__ g = w.g;
  const float* __restrict__ x = w.x;
  const int Cin = w.Cin, Cout = w.Cout, H = w.H, W = w.W, Wo = w.Wo, HWo = w.Ho * w.Wo, S = w.S;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row = lane & 31, half = lane >> 5;
  int chunk, tile;
  tile_fastest(gridDim.x, gridDim.y * gridDim.z, chunk, tile);
  const int n = chunk / w.cps;
  const int p0 = ((chunk - n * w.cps) * 4 + wave) * w.pxw;
  const int p1 = min(p0 + w.pxw, HWo);
  const int ci_base = (tile % (int)gridDim.y) * 32, co_base = (tile / (int)gridDim.y) * 32;
  const bool av = co_base + row < Cout, bv = ci_base + row < Cin;
  const float* ga = g + ((size_t)n * Cout + (av ? co_base + row : 0)) * HWo;
  const float* xb = x + ((size_t)n * Cin + (bv ? ci_base + row : 0)) * H * W;
  floatx16 acc[KK];
#pragma unroll
  for (int t = 0; t < KK; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
  for (int p = p0; p < p1; p += 32) {
    float a[16];
    int iu[16], ju[16];  // x coordinates of tap (0, 0) for this lane's 16 output pixels (pixel p + 2u + half)
    {
      int pp = p + half;
      int i = pp / Wo, j = pp - i * Wo;
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        a[u] = 0.f;
        if (av && pp < p1) a[u] = ga[pp];
        iu[u] = pp < p1 ? i * S - PAD : -8;  // beyond the chunk: no tap is valid
        ju[u] = j * S - PAD;
        pp += 2;
        j += 2;
        if (j >= Wo) {  // at most one row further per step unless the plane is narrower than two pixels
          j -= Wo;
          ++i;
          if (j >= Wo) { i += j / Wo; j %= Wo; }
        }
      }
    }
#pragma unroll
    for (int t = 0; t < KK; ++t) {
      const int tu = t / KS, tv = t % KS;
      float b[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const int r = iu[u] + tu, c = ju[u] + tv;
        b[u] = 0.f;
        if (bv && (unsigned)r < (unsigned)H && (unsigned)c < (unsigned)W) b[u] = xb[r * W + c];
      }
#pragma unroll
      for (int u = 0; u < 16; ++u) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u], b[u], acc[t], 0, 0, 0);
    }
  }
  float* out = w.part + (size_t)chunk * Cout * Cin * KK;
  const int ci = ci_base + row;
#pragma unroll
  for (int t = 0; t < KK; ++t) {
    if (t) __syncthreads();  // the previous tap's tiles have been read
#pragma unroll
    for (int r = 0; r < 16; ++r) sR[wave][r][lane] = acc[t][r];
    __syncthreads();
    if (ci < Cin) {
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        const int r = 4 * wave + rr;
        const int co = co_base + 8 * (r >> 2) + 4 * half + (r & 3);
        if (co < Cout)
          out[((size_t)co * Cin + ci) * KK + t] = (sR[0][r][lane] + sR[1][r][lane]) + (sR[2][r][lane] + sR[3][r][lane]);
      }
    }
  }
}

// The 3x3 stride-1 case for W % 4 == 0 (so H*W % 4 == 0 and every aligned group of four pixels lies in one image
// row): 16-byte loads.  A lane's fragment is eight pixels b .. b+7 (b = p + 16f + 8*half): g as two
// float4, and per row shift du the two float4 of x at b + du*W plus the pixel to the left of the
// first and to the right of the second; the three column shifts are re-combinations of these ten
// values (left / right neighbours are zero at the image border).  28 load instructions feed the
// 144 MFMAs of a pass (two fragments), against 160 in the scalar kernel.
__global__ __launch_bounds__(256) void conv3x3_wgrad_vec_mfma_f32_kernel(C3WgArgs w) {
  __shared__ float sR[4][16][64];
  const float* __restrict__ g = w.g;
  const float* __restrict__ x = w.x;
  const int Cin = w.Cin, Cout = w.Cout, H = w.H, W = w.W, HW = w.H * w.W;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row = lane & 31, half = lane >> 5;
  int chunk, tile;
  tile_fastest(gridDim.x, gridDim.y * gridDim.z, chunk, tile);
  const int n = chunk / w.cps;
  const int p0 = ((chunk - n * w.cps) * 4 + wave) * w.pxw;
  const int p1 = min(p0 + w.pxw, HW);
  const int ci_base = (tile % (int)gridDim.y) * 32, co_base = (tile / (int)gridDim.y) * 32;
  const bool av = co_base + row < Cout, bv = ci_base + row < Cin;
  const float* ga = g + ((size_t)n * Cout + (av ? co_base + row : 0)) * HW;
  const float* xb = x + ((size_t)n * Cin + (bv ? ci_base + row : 0)) * HW;
  const float4 z4 = make_float4(0.f, 0.f, 0.f, 0.f);
  floatx16 acc[9];
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
  for (int p = p0; p < p1; p += 32) {
#pragma unroll
    for (int f = 0; f < 2; ++f) {
      const int b0 = p + 16 * f + 8 * half, b1 = b0 + 4;   // the fragment's two groups of four pixels
      const bool in0 = b0 < p1, in1 = b1 < p1;              // (p1 is a multiple of four)
      // Branch-free loads: a pixel group past the chunk reads pixel 0 and gets a zero g operand (its x
      // operand then does not matter); rows past Cout / Cin read channel 0 and land in rows / columns of
      // the tile that are never stored; an x row outside the image reads pixel 0 and becomes zero.
      float4 a0 = *reinterpret_cast<const float4*>(ga + (in0 ? b0 : 0));
      float4 a1 = *reinterpret_cast<const float4*>(ga + (in1 ? b1 : 0));
      if (!in0) a0 = z4;
      if (!in1) a1 = z4;
      const int i0 = b0 / W, j0 = b0 - i0 * W;
      int i1 = i0, j1 = j0 + 4;
      if (j1 >= W) { j1 -= W; ++i1; }
#pragma unroll
      for (int du = -1; du <= 1; ++du) {
        const bool v0 = in0 && (unsigned)(i0 + du) < (unsigned)H;
        const bool v1 = in1 && (unsigned)(i1 + du) < (unsigned)H;
        const bool vl = v0 && j0 > 0, vr = v1 && j1 + 4 < W;
        float4 f0 = *reinterpret_cast<const float4*>(xb + (v0 ? b0 + du * W : 0));
        float4 f1 = *reinterpret_cast<const float4*>(xb + (v1 ? b1 + du * W : 0));
        float l0 = xb[vl ? b0 + du * W - 1 : 0];
        float r1 = xb[vr ? b1 + du * W + 4 : 0];
        if (!v0) f0 = z4;
        if (!v1) f1 = z4;
        if (!vl) l0 = 0.f;
        if (!vr) r1 = 0.f;
        // neighbours across the two groups: only inside one image row
        const float r0 = (j0 + 4 < W) ? f1.x : 0.f;
        const float l1 = (j1 > 0) ? f0.w : 0.f;
        const float xm[8] = {l0, f0.x, f0.y, f0.z, l1, f1.x, f1.y, f1.z};    // column shift -1
        const float xc[8] = {f0.x, f0.y, f0.z, f0.w, f1.x, f1.y, f1.z, f1.w};  // 0
        const float xp[8] = {f0.y, f0.z, f0.w, r0, f1.y, f1.z, f1.w, r1};      // +1
        const float av8[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
        const int t0 = (du + 1) * 3;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[t0] = __builtin_amdgcn_mfma_f32_32x32x2f32(av8[e], xm[e], acc[t0], 0, 0, 0);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[t0 + 1] = __builtin_amdgcn_mfma_f32_32x32x2f32(av8[e], xc[e], acc[t0 + 1], 0, 0, 0);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[t0 + 2] = __builtin_amdgcn_mfma_f32_32x32x2f32(av8[e], xp[e], acc[t0 + 2], 0, 0, 0);
      }
    }
  }
  float* out = w.part + (size_t)chunk * Cout * Cin * 9;
  const int ci = ci_base + row;
#pragma unroll
  for (int t = 0; t < 9; ++t) {
    if (t) __syncthreads();  // the previous tap's tiles have been read
#pragma unroll
    for (int r = 0; r < 16; ++r) sR[wave][r][lane] = acc[t][r];
    __syncthreads();
    if (ci < Cin) {
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        const int r = 4 * wave + rr;
        const int co = co_base + 8 * (r >> 2) + 4 * half + (r & 3);
        if (co < Cout)
          out[((size_t)co * Cin + ci) * 9 + t] = (sR[0][r][lane] + sR[1][r][lane]) + (sR[2][r][lane] + sR[3][r][lane]);
      }
    }
  }
}

// ---- few input channels, large window (ResNet's 7x7 stride-2 stem on 3 channels): the contraction index is
// the flattened (ci, u, v), K' = Cin*KS*KS, so the weights [Cout][K'] are one pointwise matrix (one packed
// copy) and the pixel operand of index k is x[ci(k)][pi*S - pad + u(k)][pj*S - pad + v(k)], gathered.
struct GkArgs {
  const float4* Wp;
  const float* X;   // [N][Cin][H][W]
  float* Y;         // [N][Mdim][Ho][Wo]
  const float* bias;
  long NQ;          // N * Ho * Wo
  int H, W, Ho, Wo, S, PAD, Cin, Kdim, Mdim, KG;
};

template <int KS>
__global__ __launch_bounds__(256) void conv_gatherk_mfma_f32_kernel(GkArgs a) {
  constexpr int KK = KS * KS, NCH = 2;
  const float4* __restrict__ Wp = a.Wp;
  const float* __restrict__ X = a.X;
  float* __restrict__ Y = a.Y;
  const int H = a.H, W = a.W, HW = a.H * a.W, Wo = a.Wo, HWo = a.Ho * a.Wo, S = a.S, PAD = a.PAD;
  const int Kdim = a.Kdim, Mdim = a.Mdim, KG = a.KG;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 31, half = lane >> 5;
  int bx, by;
  tile_fastest(gridDim.x, gridDim.y, bx, by);
  const int m_base = by * 32;
  const unsigned q = (unsigned)bx * 128u + wave * 32 + col;  // pixels per micro-batch < 2^31 (checked at create)
  const bool qv = q < a.NQ;
  unsigned n = 0;
  int p = 0;
  if (qv) {
    n = q / (unsigned)HWo;  // 32-bit: a 64-bit division is ~150 instructions
    p = (int)(q - n * (unsigned)HWo);
  }
  const int pi = p / Wo, pj = p - pi * Wo;
  const int r0 = pi * S - PAD, c0 = pj * S - PAD;
  const float* xn = X + (size_t)n * a.Cin * HW;
  const float4* wl = Wp + (size_t)by * KG * 64 + lane;
  floatx16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  for (int g0 = 0; g0 < KG; g0 += NCH * 4) {
    float4 av[NCH * 4];
    float b[NCH * 16];
#pragma unroll
    for (int g = 0; g < NCH * 4; ++g) {
      av[g] = g0 + g < KG ? wl[(size_t)(g0 + g) * 64] : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int k = (g0 + g) * 8 + 2 * e + half;
        const int ci = k / KK, t = k - ci * KK, u = t / KS, v = t - u * KS;
        const int xr = r0 + u, xc = c0 + v;
        float val = 0.f;
        if (qv && k < Kdim && (unsigned)xr < (unsigned)H && (unsigned)xc < (unsigned)W) val = xn[(size_t)ci * HW + xr * W + xc];
        b[4 * g + e] = val;
      }
    }
#pragma unroll
    for (int g = 0; g < NCH * 4; ++g) {
      if (g0 + g >= KG) break;  // uniform
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av[g].x, b[4 * g + 0], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av[g].y, b[4 * g + 1], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av[g].z, b[4 * g + 2], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av[g].w, b[4 * g + 3], acc, 0, 0, 0);
    }
  }
  if (qv) {
    float* yq = Y + (size_t)n * Mdim * HWo + p;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int m = m_base + 8 * (r >> 2) + 4 * half + (r & 3);
      if (m < Mdim) yq[(size_t)m * HWo] = acc[r] + (a.bias ? a.bias[m] : 0.f);
    }
  }
}

// weight gradient of the same: rows of the B operand are the flattened (ci, u, v); block (chunk of output
// pixels, k tile, co tile); partials [chunk][cout][K']
template <int KS>
__global__ __launch_bounds__(256) void conv_gatherk_wgrad_mfma_f32_kernel(C3WgArgs w, int PAD) {
  constexpr int KK = KS * KS;
  __shared__ float sR[4][16][64];
  const float* __restrict__ g = w.g;
  const float* __restrict__ x = w.x;
  const int Cin = w.Cin, Cout = w.Cout, H = w.H, W = w.W, Wo = w.Wo, HWo = w.Ho * w.Wo, S = w.S;
  const int Kdim = Cin * KK;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row = lane & 31, half = lane >> 5;
  int chunk, tile;
  tile_fastest(gridDim.x, gridDim.y * gridDim.z, chunk, tile);
  const int n = chunk / w.cps;
  const int p0 = ((chunk - n * w.cps) * 4 + wave) * w.pxw;
  const int p1 = min(p0 + w.pxw, HWo);
  const int k_base = (tile % (int)gridDim.y) * 32, co_base = (tile / (int)gridDim.y) * 32;
  const int k = k_base + row;
  const bool av = co_base + row < Cout, bv = k < Kdim;
  const int ci = bv ? k / KK : 0, t = k - (k / KK) * KK, tu = t / KS, tv = t - tu * KS;
  const float* ga = g + ((size_t)n * Cout + (av ? co_base + row : 0)) * HWo;
  const float* xb = x + ((size_t)n * Cin + ci) * H * W;
  floatx16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  for (int p = p0; p < p1; p += 32) {
    float a[16], b[16];
    int pp = p + half;
    int i = pp / Wo, j = pp - i * Wo;
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      a[u] = 0.f;
      b[u] = 0.f;
      const int r = i * S - PAD + tu, c = j * S - PAD + tv;
      if (av && pp < p1) a[u] = ga[pp];
      if (bv && pp < p1 && (unsigned)r < (unsigned)H && (unsigned)c < (unsigned)W) b[u] = xb[r * W + c];
      pp += 2;
      j += 2;
      if (j >= Wo) {
        j -= Wo;
        ++i;
        if (j >= Wo) { i += j / Wo; j %= Wo; }
      }
    }
#pragma unroll
    for (int u = 0; u < 16; ++u) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u], b[u], acc, 0, 0, 0);
  }
#pragma unroll
  for (int r = 0; r < 16; ++r) sR[wave][r][lane] = acc[r];
  __syncthreads();
  float* out = w.part + (size_t)chunk * Cout * Kdim;
  if (bv) {
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
      const int r = 4 * wave + rr;
      const int co = co_base + 8 * (r >> 2) + 4 * half + (r & 3);
      if (co < Cout) out[(size_t)co * Kdim + k] = (sR[0][r][lane] + sR[1][r][lane]) + (sR[2][r][lane] + sR[3][r][lane]);
    }
  }
}

// G[i] += sum over the chunks of part[chunk][i]
__global__ __launch_bounds__(256) void conv3x3_reduce_kernel(const float* __restrict__ part, float* __restrict__ G, size_t n,
                                                             int parts) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  float s = 0.f;
  for (int c0 = 0; c0 < parts; c0 += 8) {
    float v[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] = c0 + k < parts ? part[(size_t)(c0 + k) * n + i] : 0.f;
#pragma unroll
    for (int k = 0; k < 8; ++k) s += v[k];
  }
  G[i] += s;
}

// pixels per wavefront of the weight-gradient kernel: the largest of {256, 128, 64, 32} that still
// gives 768 blocks
int c3_pxw(int N, int Cin, int Cout, int HWo) {
  const long tiles = (long)cdiv(Cin, 32) * cdiv(Cout, 32);
  const int cand[4] = {256, 128, 64, 32};
  for (int c : cand)
    if ((long)N * cdiv(HWo, 4 * c) * tiles >= 768) return c;
  return 32;
}

inline int out_dim(int H, int k, int stride) { return (H + 2 * (k / 2) - k) / stride + 1; }

// Y[N][Mdim][PH][PW] = sum over taps of A_tap X(tap)
template <int KS, bool DGRAD>
void launch_product(hipStream_t st, const char* name, const float* Wp, const float* X, float* Y, const float* bias, int N,
                    int Kdim, int Mdim, int PH, int PW, int XH, int XW, int S) {
  C3Args a;
  a.Wp = reinterpret_cast<const float4*>(Wp);
  a.X = X; a.Y = Y; a.bias = bias;
  a.NQ = (long)N * PH * PW;
  a.PH = PH; a.PW = PW; a.XH = XH; a.XW = XW; a.S = S;
  a.Kdim = Kdim; a.Mdim = Mdim; a.KG = cdiv(Kdim, 8);
  a.tap_stride = pw_pack_floats(Mdim, Kdim) / 4;
  // two tiles of result channels per wavefront while that leaves two blocks per compute unit
  const int mt = (Mdim > 32 && (long)cdiv(a.NQ, 128) * cdiv(Mdim, 64) >= 512) ? 2 : 1;
  const dim3 grid((unsigned)cdiv(a.NQ, 128), (unsigned)cdiv(Mdim, 32 * mt));
  if (mt == 2) {
    if (Kdim > 32) KLAUNCH_NAMED(name, (conv_mfma_f32_kernel<2, 2, KS, DGRAD>), grid, dim3(256), 0, st, a);
    else KLAUNCH_NAMED(name, (conv_mfma_f32_kernel<1, 2, KS, DGRAD>), grid, dim3(256), 0, st, a);
  } else {
    if (Kdim > 32) KLAUNCH_NAMED(name, (conv_mfma_f32_kernel<2, 1, KS, DGRAD>), grid, dim3(256), 0, st, a);
    else KLAUNCH_NAMED(name, (conv_mfma_f32_kernel<1, 1, KS, DGRAD>), grid, dim3(256), 0, st, a);
  }
}

const char* product_name(int k, int stride) {
  return k == 3 && stride == 1 ? "conv3x3_mfma_f32_kernel" : (k == 3 ? "conv3x3s2_mfma_f32_kernel" : "conv1x1s2_mfma_f32_kernel");
}

}  // namespace

// ---- few input channels, 7x7 window
bool conv_gatherk_supported(int Cin, int Cout, int k, int stride, int pad, int groups, int H, int W) {
  return k == 7 && groups == 1 && Cin >= 1 && Cin < 8 && Cout >= 8 && stride >= 1 && stride <= 4 && pad >= 0 && pad <= 3 &&
         H + 2 * pad >= k && W + 2 * pad >= k && (long)H * W < (1L << 30);
}
size_t conv_gatherk_pack_floats(int Cin, int Cout, int k) { return pw_pack_floats(Cout, Cin * k * k); }
static int gk_out(int H, int k, int stride, int pad) { return (H + 2 * pad - k) / stride + 1; }
int conv_gatherk_wgrad_parts(int N, int Cin, int Cout, int H, int W, int k, int stride, int pad) {
  const int HWo = gk_out(H, k, stride, pad) * gk_out(W, k, stride, pad);
  return N * cdiv(HWo, 4 * c3_pxw(N, Cin * k * k, Cout, HWo));
}
size_t conv_gatherk_wgrad_ws(int N, int Cin, int Cout, int H, int W, int k, int stride, int pad) {
  return (size_t)conv_gatherk_wgrad_parts(N, Cin, Cout, H, W, k, stride, pad) * Cin * Cout * k * k;
}
void conv_gatherk_fwd_f32(hipStream_t st, const float* Wp, const float* x, float* y, const float* bias, int N, int Cin,
                          int Cout, int H, int W, int k, int stride, int pad) {
  GkArgs a;
  a.Wp = reinterpret_cast<const float4*>(Wp);
  a.X = x; a.Y = y; a.bias = bias;
  a.H = H; a.W = W; a.Ho = gk_out(H, k, stride, pad); a.Wo = gk_out(W, k, stride, pad);
  a.NQ = (long)N * a.Ho * a.Wo;
  a.S = stride; a.PAD = pad; a.Cin = Cin; a.Kdim = Cin * k * k; a.Mdim = Cout; a.KG = cdiv(a.Kdim, 8);
  const dim3 grid((unsigned)cdiv(a.NQ, 128), (unsigned)cdiv(Cout, 32));
  KLAUNCH_NAMED("conv7x7_gatherk_mfma_f32_kernel", (conv_gatherk_mfma_f32_kernel<7>), grid, dim3(256), 0, st, a);
}
// weight gradient only (a layer with so few input channels is a model's first: its input gradient, if asked
// for, comes from the generic kernel)
void conv_gatherk_wgrad_f32(hipStream_t st, const float* g, const float* x, float* part, float* G, int N, int Cin, int Cout,
                            int H, int W, int k, int stride, int pad) {
  C3WgArgs w;
  w.g = g; w.x = x; w.part = part;
  w.Cin = Cin; w.Cout = Cout; w.H = H; w.W = W; w.Ho = gk_out(H, k, stride, pad); w.Wo = gk_out(W, k, stride, pad); w.S = stride;
  const int Kdim = Cin * k * k;
  w.pxw = c3_pxw(N, Kdim, Cout, w.Ho * w.Wo);
  w.cps = cdiv(w.Ho * w.Wo, 4 * w.pxw);
  const dim3 grid((unsigned)(N * w.cps), (unsigned)cdiv(Kdim, 32), (unsigned)cdiv(Cout, 32));
  KLAUNCH_NAMED("conv7x7_gatherk_wgrad_mfma_f32_kernel", (conv_gatherk_wgrad_mfma_f32_kernel<7>), grid, dim3(256), 0, st, w, pad);
  const size_t n = (size_t)Cout * Kdim;
  if (G) KLAUNCH(conv3x3_reduce_kernel, dim3((unsigned)cdiv(n, 256)), dim3(256), 0, st, part, G, n, (int)grid.x);
}

bool conv_mfma_supported(int Cin, int Cout, int k, int stride, int pad, int groups, int H, int W) {
  const bool shape = (k == 3 && pad == 1 && (stride == 1 || stride == 2)) || (k == 1 && pad == 0 && stride == 2);
  return shape && groups == 1 && Cin >= 8 && Cout >= 8 && H >= 1 && W >= 1 && (long)H * W < (1L << 30);
}

size_t conv_mfma_pack_floats(int Mdim, int Kdim, int k) { return (size_t)k * k * pw_pack_floats(Mdim, Kdim); }

int conv_mfma_wgrad_parts(int N, int Cin, int Cout, int H, int W, int k, int stride) {
  const int HWo = out_dim(H, k, stride) * out_dim(W, k, stride);
  return N * cdiv(HWo, 4 * c3_pxw(N, Cin, Cout, HWo));
}

size_t conv_mfma_wgrad_ws(int N, int Cin, int Cout, int H, int W, int k, int stride) {
  return (size_t)conv_mfma_wgrad_parts(N, Cin, Cout, H, W, k, stride) * Cin * Cout * k * k;
}

void conv_mfma_fwd_f32(hipStream_t st, const float* Wp, const float* x, float* y, const float* bias, int N, int Cin,
                       int Cout, int H, int W, int k, int stride) {
  const int Ho = out_dim(H, k, stride), Wo = out_dim(W, k, stride);
  if (k == 3) launch_product<3, false>(st, product_name(k, stride), Wp, x, y, bias, N, Cin, Cout, Ho, Wo, H, W, stride);
  else launch_product<1, false>(st, product_name(k, stride), Wp, x, y, bias, N, Cin, Cout, Ho, Wo, H, W, stride);
}

void conv_mfma_bwd_f32(hipStream_t st, const float* Wp_t, const float* g, float* dx, const float* x, float* part,
                       float* G, int N, int Cin, int Cout, int H, int W, int k, int stride) {
  const int Ho = out_dim(H, k, stride), Wo = out_dim(W, k, stride);
  if (dx) {
    if (k == 3) launch_product<3, true>(st, product_name(k, stride), Wp_t, g, dx, nullptr, N, Cout, Cin, H, W, Ho, Wo, stride);
    else launch_product<1, true>(st, product_name(k, stride), Wp_t, g, dx, nullptr, N, Cout, Cin, H, W, Ho, Wo, stride);
  }
  C3WgArgs w;
  w.g = g; w.x = x; w.part = part;
  w.Cin = Cin; w.Cout = Cout; w.H = H; w.W = W; w.Ho = Ho; w.Wo = Wo; w.S = stride;
  w.pxw = c3_pxw(N, Cin, Cout, Ho * Wo);
  w.cps = cdiv(Ho * Wo, 4 * w.pxw);
  const dim3 grid((unsigned)(N * w.cps), (unsigned)cdiv(Cin, 32), (unsigned)cdiv(Cout, 32));
  if (k == 3 && stride == 1 && W % 4 == 0) KLAUNCH(conv3x3_wgrad_vec_mfma_f32_kernel, grid, dim3(256), 0, st, w);
  else if (k == 3) KLAUNCH_NAMED("conv3x3_wgrad_mfma_f32_kernel", (conv_wgrad_mfma_f32_kernel<3>), grid, dim3(256), 0, st, w);
  else KLAUNCH_NAMED("conv1x1s2_wgrad_mfma_f32_kernel", (conv_wgrad_mfma_f32_kernel<1>), grid, dim3(256), 0, st, w);
  const size_t n = (size_t)Cin * Cout * k * k;
  if (G) KLAUNCH(conv3x3_reduce_kernel, dim3((unsigned)cdiv(n, 256)), dim3(256), 0, st, part, G, n, (int)grid.x);
}

}  // namespace ast
