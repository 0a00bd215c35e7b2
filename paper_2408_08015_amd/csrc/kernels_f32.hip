// fp32 NCHW kernels of the MobileNetV2-style stages: pointwise convolution on the
// fp32 matrix cores (v_mfma_f32_32x32x2f32), depthwise 3x3, BatchNorm (+ReLU6,
// +residual), pooling, linear, softmax cross-entropy, momentum SGD.
//
// In NCHW a sample's channel plane is contiguous, so a wavefront that maps lanes to
// consecutive pixels reads and writes 128/256-byte runs; the pointwise convolution
// keeps pixels on the MFMA N dimension for exactly that reason (the B operand is
// loaded straight from global memory, the small weight matrix is staged in LDS).
#include "device_utils.h"
#include "kernels.h"
#include "prof.h"

namespace ast {

static inline int cdiv(long a, long b) { return (int)((a + b - 1) / b); }

// ============================================================== pointwise conv (fwd / dgrad)
// Block = 4 wavefronts; wavefront w owns pixels [128*bx + 32*w, +32) of the flattened
// (n, p) index and NT 32-row tiles of output channels.  MFMA 32x32x2: lane l supplies
// A[m = l%32][k = l/32] and B[k = l/32][q = l%32]; accumulator register r of lane l is
// D[8*(r/4) + 4*(l/32) + r%4][l%32].
template <int NT>
__global__ __launch_bounds__(256) void pw_conv_f32_kernel(
    const float* __restrict__ W, int lda_m, int lda_k, const float* __restrict__ X,
    float* __restrict__ Y, const float* __restrict__ bias, const float* __restrict__ add, long NQ,
    int HW, int Kdim, int Mdim) {
  constexpr int KC = 32;
  constexpr int MT = 32 * NT;
  __shared__ float sW[KC][MT];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 31, half = lane >> 5;
  const int m_base = blockIdx.y * MT;
  const long q = (long)blockIdx.x * 128 + wave * 32 + col;
  const bool qv = q < NQ;
  long n = 0;
  int p = 0;
  if (qv) {
    n = q / HW;
    p = (int)(q - n * HW);
  }
  const float* xq = X + (size_t)n * Kdim * HW + p;
  floatx16 acc[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;

  for (int k0 = 0; k0 < Kdim; k0 += KC) {
    __syncthreads();
    for (int idx = threadIdx.x; idx < KC * MT; idx += 256) {
      int kk, mm;
      if (lda_k == 1) {  // k contiguous in memory
        kk = idx % KC;
        mm = idx / KC;
      } else {
        mm = idx % MT;
        kk = idx / MT;
      }
      int m = m_base + mm, k = k0 + kk;
      float v = 0.f;
      if (m < Mdim && k < Kdim) v = W[(size_t)m * lda_m + (size_t)k * lda_k];
      sW[kk][mm] = v;
    }
    __syncthreads();
    float b[KC / 2];
#pragma unroll
    for (int j = 0; j < KC / 2; ++j) {
      int k = k0 + 2 * j + half;
      b[j] = (qv && k < Kdim) ? xq[(size_t)k * HW] : 0.f;
    }
#pragma unroll
    for (int j = 0; j < KC / 2; ++j) {
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        float a = sW[2 * j + half][t * 32 + col];
        acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b[j], acc[t], 0, 0, 0);
      }
    }
  }
  if (!qv) return;
  float* yq = Y + (size_t)n * Mdim * HW + p;
  const float* aq = add ? add + (size_t)n * Mdim * HW + p : nullptr;
#pragma unroll
  for (int t = 0; t < NT; ++t) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      int m = m_base + t * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
      if (m < Mdim) {
        float v = acc[t][r];
        if (bias) v += bias[m];
        if (aq) v += aq[(size_t)m * HW];
        yq[(size_t)m * HW] = v;
      }
    }
  }
}

void pw_conv_f32(hipStream_t st, const float* W, int lda_m, int lda_k, const float* X, float* Y,
                 const float* bias, const float* add, int N, int Kdim, int Mdim, int HW) {
  long NQ = (long)N * HW;
  int mt = cdiv(Mdim, 32);
  dim3 block(256);
#define PW_LAUNCH(NT)                                                                         \
  KLAUNCH(pw_conv_f32_kernel<NT>, dim3(cdiv(NQ, 128), cdiv(mt, NT)), block, 0, st, W, \
                     lda_m, lda_k, X, Y, bias, add, NQ, HW, Kdim, Mdim)
  if (mt == 1) PW_LAUNCH(1);
  else if (mt == 2) PW_LAUNCH(2);
  else if (mt % 6 == 0) PW_LAUNCH(6);
  else if (mt % 5 == 0) PW_LAUNCH(5);
  else if (mt % 4 == 0) PW_LAUNCH(4);
  else if (mt % 3 == 0) PW_LAUNCH(3);
  else PW_LAUNCH(4);
#undef PW_LAUNCH
}

// ============================================================== pointwise conv wgrad
// Wavefront = one 32(co) x 32(ci) tile of dW over one pixel chunk of one sample; the
// contraction index is the pixel.  Lane (m = l%32, h = l/32) loads four consecutive
// pixels of row m starting at 4h and feeds four MFMAs; both operands use the same
// pixel for a given (h, t), which is all the contraction needs.
constexpr int kWgChunk = 512;  // pixels per chunk

__global__ __launch_bounds__(256) void pw_wgrad_f32_kernel(const float* __restrict__ g,
                                                           const float* __restrict__ x,
                                                           float* __restrict__ part, int Cin, int Cout,
                                                           int HW, int chunks_per_sample, int vec) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row = lane & 31, half = lane >> 5;
  const int chunk = blockIdx.x;
  const int n = chunk / chunks_per_sample;
  const int p0 = (chunk - n * chunks_per_sample) * kWgChunk;
  const int p1 = min(p0 + kWgChunk, HW);
  const int ci_base = blockIdx.y * 32;
  const int co_tile = blockIdx.z * 4 + wave;
  const int co_base = co_tile * 32;
  if (co_base >= Cout) return;  // no block-level synchronisation below
  const bool av = co_base + row < Cout, bv = ci_base + row < Cin;
  const float* ga = g + ((size_t)n * Cout + (av ? co_base + row : 0)) * HW;
  const float* xb = x + ((size_t)n * Cin + (bv ? ci_base + row : 0)) * HW;
  floatx16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  if (vec) {  // HW % 4 == 0: aligned 16-byte loads, 8 pixels per step
    for (int p = p0; p < p1; p += 8) {
      int pp = p + 4 * half;
      float4 a = make_float4(0.f, 0.f, 0.f, 0.f), b = a;
      if (pp < p1) {
        if (av) a = *reinterpret_cast<const float4*>(ga + pp);
        if (bv) b = *reinterpret_cast<const float4*>(xb + pp);
      }
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b.x, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b.y, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, b.z, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, b.w, acc, 0, 0, 0);
    }
  } else {
    for (int p = p0; p < p1; p += 2) {
      int pp = p + half;
      float a = (av && pp < p1) ? ga[pp] : 0.f;
      float b = (bv && pp < p1) ? xb[pp] : 0.f;
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
    }
  }
  float* out = part + (size_t)chunk * Cout * Cin;
  const int ci = ci_base + row;
  if (ci < Cin) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      int co = co_base + 8 * (r >> 2) + 4 * half + (r & 3);
      if (co < Cout) out[(size_t)co * Cin + ci] = acc[r];
    }
  }
}

__global__ void reduce_parts_acc_kernel(const float* __restrict__ part, float* __restrict__ G,
                                        size_t n, int parts) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float s = 0.f;
  for (int c = 0; c < parts; ++c) s += part[(size_t)c * n + i];
  G[i] += s;
}

static inline int wg_chunks(int HW) { return cdiv(HW, kWgChunk); }
size_t pw_wgrad_f32_ws(int N, int Cin, int Cout, int HW) {
  return (size_t)N * wg_chunks(HW) * Cin * Cout;
}
void pw_wgrad_f32(hipStream_t st, const float* g, const float* x, float* part, float* G, int N,
                  int Cin, int Cout, int HW) {
  int cps = wg_chunks(HW);
  int chunks = N * cps;
  dim3 grid(chunks, cdiv(Cin, 32), cdiv(cdiv(Cout, 32), 4));
  // the vector path needs every chunk start to be a multiple of 8 pixels and aligned rows
  int vec = (HW % 4 == 0) ? 1 : 0;
  KLAUNCH(pw_wgrad_f32_kernel, grid, dim3(256), 0, st, g, x, part, Cin, Cout, HW, cps, vec);
  size_t n = (size_t)Cin * Cout;
  KLAUNCH(reduce_parts_acc_kernel, dim3(cdiv(n, 256)), dim3(256), 0, st, part, G, n, chunks);
}

// ============================================================== depthwise 3x3
__global__ __launch_bounds__(256) void dw3x3_fwd_f32_kernel(const float* __restrict__ x,
                                                            const float* __restrict__ w,
                                                            float* __restrict__ y, int C, int H, int W,
                                                            int Ho, int Wo, int stride, size_t total) {
  size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  int j = (int)(idx % Wo);
  size_t t = idx / Wo;
  int i = (int)(t % Ho);
  size_t nc = t / Ho;
  int c = (int)(nc % C);
  const float* xp = x + nc * (size_t)H * W;
  const float* wc = w + c * 9;
  float acc = 0.f;
#pragma unroll
  for (int u = 0; u < 3; ++u) {
    int ii = i * stride - 1 + u;
    if (ii < 0 || ii >= H) continue;
#pragma unroll
    for (int v = 0; v < 3; ++v) {
      int jj = j * stride - 1 + v;
      if (jj < 0 || jj >= W) continue;
      acc += wc[u * 3 + v] * xp[(size_t)ii * W + jj];
    }
  }
  y[idx] = acc;
}

__global__ __launch_bounds__(256) void dw3x3_dgrad_f32_kernel(const float* __restrict__ g,
                                                              const float* __restrict__ w,
                                                              float* __restrict__ dx, int C, int H,
                                                              int W, int Ho, int Wo, int stride,
                                                              size_t total) {
  size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  int j = (int)(idx % W);
  size_t t = idx / W;
  int i = (int)(t % H);
  size_t nc = t / H;
  int c = (int)(nc % C);
  const float* gp = g + nc * (size_t)Ho * Wo;
  const float* wc = w + c * 9;
  float acc = 0.f;
#pragma unroll
  for (int u = 0; u < 3; ++u) {
    int a = i + 1 - u;  // = io * stride
    if (a < 0) continue;
    int io = a / stride;
    if (io * stride != a || io >= Ho) continue;
#pragma unroll
    for (int v = 0; v < 3; ++v) {
      int b = j + 1 - v;
      if (b < 0) continue;
      int jo = b / stride;
      if (jo * stride != b || jo >= Wo) continue;
      acc += wc[u * 3 + v] * gp[(size_t)io * Wo + jo];
    }
  }
  dx[idx] = acc;
}

// Per channel c and split s: partial sums of the 9 weight gradients over a share of the
// (n, output pixel) range.  part[(c*S + s)*9 + t].
__global__ __launch_bounds__(256) void dw3x3_wgrad_f32_kernel(const float* __restrict__ g,
                                                              const float* __restrict__ x,
                                                              float* __restrict__ part, int N, int C,
                                                              int H, int W, int Ho, int Wo, int stride,
                                                              int S) {
  __shared__ float sh[16];
  const int c = blockIdx.x, s = blockIdx.y;
  const long per = (long)N * Ho * Wo;
  const long len = (per + S - 1) / S;
  const long e0 = s * len, e1 = min(e0 + len, per);
  float acc[9];
#pragma unroll
  for (int t = 0; t < 9; ++t) acc[t] = 0.f;
  for (long e = e0 + threadIdx.x; e < e1; e += 256) {
    int n = (int)(e / ((long)Ho * Wo));
    int r = (int)(e - (long)n * Ho * Wo);
    int i = r / Wo, j = r - i * Wo;
    float gv = g[((size_t)n * C + c) * Ho * Wo + r];
    const float* xp = x + ((size_t)n * C + c) * H * W;
#pragma unroll
    for (int u = 0; u < 3; ++u) {
      int ii = i * stride - 1 + u;
      if (ii < 0 || ii >= H) continue;
#pragma unroll
      for (int v = 0; v < 3; ++v) {
        int jj = j * stride - 1 + v;
        if (jj < 0 || jj >= W) continue;
        acc[u * 3 + v] += gv * xp[(size_t)ii * W + jj];
      }
    }
  }
#pragma unroll
  for (int t = 0; t < 9; ++t) {
    float v = block_sum<float>(acc[t], sh);
    if (threadIdx.x == 0) part[((size_t)c * S + s) * 9 + t] = v;
  }
}

__global__ void dw3x3_wgrad_final_kernel(const float* __restrict__ part, float* __restrict__ G, int C,
                                         int S) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= C * 9) return;
  int c = i / 9, t = i - c * 9;
  float s = 0.f;
  for (int k = 0; k < S; ++k) s += part[((size_t)c * S + k) * 9 + t];
  G[i] += s;
}

static inline int dw_split(int N, int C, int Ho, int Wo) {
  long per = (long)N * Ho * Wo;
  int S = cdiv(2048, C);
  int maxS = (int)((per + 2047) / 2048);
  if (S > maxS) S = maxS;
  return S < 1 ? 1 : S;
}
static inline int conv_out(int H, int k, int stride, int pad) { return (H + 2 * pad - k) / stride + 1; }

void dw3x3_fwd_f32(hipStream_t st, const float* x, const float* w, float* y, int N, int C, int H,
                   int W, int stride) {
  int Ho = conv_out(H, 3, stride, 1), Wo = conv_out(W, 3, stride, 1);
  size_t total = (size_t)N * C * Ho * Wo;
  KLAUNCH(dw3x3_fwd_f32_kernel, dim3(cdiv(total, 256)), dim3(256), 0, st, x, w, y, C, H, W,
                     Ho, Wo, stride, total);
}
void dw3x3_dgrad_f32(hipStream_t st, const float* g, const float* w, float* dx, int N, int C, int H,
                     int W, int stride) {
  int Ho = conv_out(H, 3, stride, 1), Wo = conv_out(W, 3, stride, 1);
  size_t total = (size_t)N * C * H * W;
  KLAUNCH(dw3x3_dgrad_f32_kernel, dim3(cdiv(total, 256)), dim3(256), 0, st, g, w, dx, C, H,
                     W, Ho, Wo, stride, total);
}
size_t dw3x3_wgrad_f32_ws(int N, int C, int H, int W, int stride) {
  int Ho = conv_out(H, 3, stride, 1), Wo = conv_out(W, 3, stride, 1);
  return (size_t)C * dw_split(N, C, Ho, Wo) * 9;
}
void dw3x3_wgrad_f32(hipStream_t st, const float* g, const float* x, float* part, float* G, int N,
                     int C, int H, int W, int stride) {
  int Ho = conv_out(H, 3, stride, 1), Wo = conv_out(W, 3, stride, 1);
  int S = dw_split(N, C, Ho, Wo);
  KLAUNCH(dw3x3_wgrad_f32_kernel, dim3(C, S), dim3(256), 0, st, g, x, part, N, C, H, W, Ho,
                     Wo, stride, S);
  KLAUNCH(dw3x3_wgrad_final_kernel, dim3(cdiv(C * 9, 256)), dim3(256), 0, st, part, G, C, S);
}

// ============================================================== generic direct conv
__global__ __launch_bounds__(256) void conv_direct_fwd_kernel(
    const float* __restrict__ x, const float* __restrict__ w, const float* __restrict__ bias,
    float* __restrict__ y, int Cin, int H, int W, int Cout, int Ho, int Wo, int k, int stride, int pad,
    int groups, size_t total) {
  size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  int j = (int)(idx % Wo);
  size_t t = idx / Wo;
  int i = (int)(t % Ho);
  t /= Ho;
  int o = (int)(t % Cout);
  size_t n = t / Cout;
  int cg = Cin / groups, og = Cout / groups;
  int grp = o / og;
  float acc = bias ? bias[o] : 0.f;
  for (int c = 0; c < cg; ++c) {
    const float* xp = x + ((size_t)n * Cin + grp * cg + c) * H * W;
    const float* wp = w + ((size_t)o * cg + c) * k * k;
    for (int u = 0; u < k; ++u) {
      int ii = i * stride - pad + u;
      if (ii < 0 || ii >= H) continue;
      for (int v = 0; v < k; ++v) {
        int jj = j * stride - pad + v;
        if (jj < 0 || jj >= W) continue;
        acc += wp[u * k + v] * xp[(size_t)ii * W + jj];
      }
    }
  }
  y[idx] = acc;
}

__global__ __launch_bounds__(256) void conv_direct_dgrad_kernel(
    const float* __restrict__ g, const float* __restrict__ w, float* __restrict__ dx, int Cin, int H,
    int W, int Cout, int Ho, int Wo, int k, int stride, int pad, int groups, size_t total) {
  size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  int j = (int)(idx % W);
  size_t t = idx / W;
  int i = (int)(t % H);
  t /= H;
  int ci = (int)(t % Cin);
  size_t n = t / Cin;
  int cg = Cin / groups, og = Cout / groups;
  int grp = ci / cg, c = ci - grp * cg;
  float acc = 0.f;
  for (int oo = 0; oo < og; ++oo) {
    int o = grp * og + oo;
    const float* gp = g + ((size_t)n * Cout + o) * Ho * Wo;
    const float* wp = w + ((size_t)o * cg + c) * k * k;
    for (int u = 0; u < k; ++u) {
      int a = i + pad - u;
      if (a < 0) continue;
      int io = a / stride;
      if (io * stride != a || io >= Ho) continue;
      for (int v = 0; v < k; ++v) {
        int b = j + pad - v;
        if (b < 0) continue;
        int jo = b / stride;
        if (jo * stride != b || jo >= Wo) continue;
        acc += wp[u * k + v] * gp[(size_t)io * Wo + jo];
      }
    }
  }
  dx[idx] = acc;
}

// one block per weight element
__global__ __launch_bounds__(256) void conv_direct_wgrad_kernel(
    const float* __restrict__ g, const float* __restrict__ x, float* __restrict__ G, int N, int Cin,
    int H, int W, int Cout, int Ho, int Wo, int k, int stride, int pad, int groups) {
  __shared__ float sh[16];
  int widx = blockIdx.x;
  int v = widx % k;
  int t = widx / k;
  int u = t % k;
  t /= k;
  int cg = Cin / groups, og = Cout / groups;
  int c = t % cg;
  int o = t / cg;
  int grp = o / og;
  long per = (long)N * Ho * Wo;
  float acc = 0.f;
  for (long e = threadIdx.x; e < per; e += 256) {
    int n = (int)(e / ((long)Ho * Wo));
    int r = (int)(e - (long)n * Ho * Wo);
    int i = r / Wo, j = r - i * Wo;
    int ii = i * stride - pad + u, jj = j * stride - pad + v;
    if (ii < 0 || ii >= H || jj < 0 || jj >= W) continue;
    acc += g[((size_t)n * Cout + o) * Ho * Wo + r] *
           x[(((size_t)n * Cin + grp * cg + c) * H + ii) * W + jj];
  }
  float s = block_sum<float>(acc, sh);
  if (threadIdx.x == 0) G[widx] += s;
}

void conv_direct_fwd_f32(hipStream_t st, const float* x, const float* w, const float* bias, float* y,
                         int N, int Cin, int H, int W, int Cout, int k, int stride, int pad,
                         int groups) {
  int Ho = conv_out(H, k, stride, pad), Wo = conv_out(W, k, stride, pad);
  size_t total = (size_t)N * Cout * Ho * Wo;
  KLAUNCH(conv_direct_fwd_kernel, dim3(cdiv(total, 256)), dim3(256), 0, st, x, w, bias, y,
                     Cin, H, W, Cout, Ho, Wo, k, stride, pad, groups, total);
}
void conv_direct_dgrad_f32(hipStream_t st, const float* g, const float* w, float* dx, int N, int Cin,
                           int H, int W, int Cout, int k, int stride, int pad, int groups) {
  int Ho = conv_out(H, k, stride, pad), Wo = conv_out(W, k, stride, pad);
  size_t total = (size_t)N * Cin * H * W;
  KLAUNCH(conv_direct_dgrad_kernel, dim3(cdiv(total, 256)), dim3(256), 0, st, g, w, dx, Cin,
                     H, W, Cout, Ho, Wo, k, stride, pad, groups, total);
}
void conv_direct_wgrad_f32(hipStream_t st, const float* g, const float* x, float* G, int N, int Cin,
                           int H, int W, int Cout, int k, int stride, int pad, int groups) {
  int Ho = conv_out(H, k, stride, pad), Wo = conv_out(W, k, stride, pad);
  int nw = Cout * (Cin / groups) * k * k;
  KLAUNCH(conv_direct_wgrad_kernel, dim3(nw), dim3(256), 0, st, g, x, G, N, Cin, H, W, Cout,
                     Ho, Wo, k, stride, pad, groups);
}

__global__ __launch_bounds__(256) void channel_sum_acc_kernel(const float* __restrict__ g,
                                                              float* __restrict__ G, int N, int C,
                                                              int HW) {
  __shared__ float sh[16];
  int c = blockIdx.x;
  long per = (long)N * HW;
  float acc = 0.f;
  for (long e = threadIdx.x; e < per; e += 256) {
    long n = e / HW;
    int p = (int)(e - n * HW);
    acc += g[((size_t)n * C + c) * HW + p];
  }
  float s = block_sum<float>(acc, sh);
  if (threadIdx.x == 0) G[c] += s;
}
void channel_sum_acc_f32(hipStream_t st, const float* g, float* G, int N, int C, int HW) {
  KLAUNCH(channel_sum_acc_kernel, dim3(C), dim3(256), 0, st, g, G, N, C, HW);
}

// ============================================================== BatchNorm
// Statistics are reduced in two levels: (channel, split) blocks accumulate fp32 per
// thread, combine in fp64 and write partials; one thread per channel finishes in fp64.
static inline int bn_split(int C, size_t per) {
  int S = cdiv(2048, C);
  int maxS = (int)((per + 4095) / 4096);
  if (S > maxS) S = maxS;
  return S < 1 ? 1 : S;
}
size_t bn_ws_doubles(int C, size_t per) { return (size_t)C * bn_split(C, per) * 2; }

// element range of split s, aligned to 4 elements
__device__ __forceinline__ void split_range(long per, int S, int s, long& e0, long& e1) {
  long len = ((per + S - 1) / S + 3) & ~3L;
  e0 = (long)s * len;
  e1 = min(e0 + len, per);
  if (e0 > per) e0 = per;
}

template <bool VEC>
__global__ __launch_bounds__(256) void bn_stats_partial_kernel(const float* __restrict__ x,
                                                               double* __restrict__ ws, int N, int C,
                                                               int HW, int S) {
  __shared__ double sh[16];
  const int c = blockIdx.x, s = blockIdx.y;
  long e0, e1;
  split_range((long)N * HW, S, s, e0, e1);
  float s1 = 0.f, s2 = 0.f;
  if (VEC) {
    for (long e = e0 + 4L * threadIdx.x; e < e1; e += 1024) {
      long n = e / HW;
      int p = (int)(e - n * HW);
      float4 v = *reinterpret_cast<const float4*>(x + ((size_t)n * C + c) * HW + p);
      s1 += (v.x + v.y) + (v.z + v.w);
      s2 += (v.x * v.x + v.y * v.y) + (v.z * v.z + v.w * v.w);
    }
  } else {
    for (long e = e0 + threadIdx.x; e < e1; e += 256) {
      long n = e / HW;
      int p = (int)(e - n * HW);
      float v = x[((size_t)n * C + c) * HW + p];
      s1 += v;
      s2 += v * v;
    }
  }
  double d1 = block_sum<double>((double)s1, sh);
  double d2 = block_sum<double>((double)s2, sh);
  if (threadIdx.x == 0) {
    ws[((size_t)c * S + s) * 2 + 0] = d1;
    ws[((size_t)c * S + s) * 2 + 1] = d2;
  }
}

__global__ void bn_stats_final_kernel(const double* __restrict__ ws, const float* __restrict__ gamma,
                                      const float* __restrict__ beta, float* __restrict__ stat,
                                      float* __restrict__ scale_shift, float* __restrict__ running,
                                      int C, int S, double count, float eps) {
  int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= C) return;
  double s1 = 0, s2 = 0;
  for (int s = 0; s < S; ++s) {
    s1 += ws[((size_t)c * S + s) * 2 + 0];
    s2 += ws[((size_t)c * S + s) * 2 + 1];
  }
  double mean = s1 / count;
  double var = s2 / count - mean * mean;
  if (var < 0) var = 0;
  double istd = 1.0 / sqrt(var + (double)eps);
  stat[c] = (float)mean;
  stat[C + c] = (float)istd;
  double sc = (double)gamma[c] * istd;
  scale_shift[c] = (float)sc;
  scale_shift[C + c] = (float)((double)beta[c] - mean * sc);
  if (running) {
    double unb = count > 1 ? var * count / (count - 1) : var;
    running[c] += 0.1f * ((float)mean - running[c]);
    running[C + c] += 0.1f * ((float)unb - running[C + c]);
  }
}

void bn_stats_f32(hipStream_t st, const float* x, const float* gamma, const float* beta, float* stat,
                  float* scale_shift, float* running, double* ws, int N, int C, int HW, float eps) {
  size_t per = (size_t)N * HW;
  int S = bn_split(C, per);
  if (HW % 4 == 0)
    KLAUNCH(bn_stats_partial_kernel<true>, dim3(C, S), dim3(256), 0, st, x, ws, N, C, HW, S);
  else
    KLAUNCH(bn_stats_partial_kernel<false>, dim3(C, S), dim3(256), 0, st, x, ws, N, C, HW, S);
  KLAUNCH(bn_stats_final_kernel, dim3(cdiv(C, 128)), dim3(128), 0, st, ws, gamma, beta, stat,
                     scale_shift, running, C, S, (double)per, eps);
}

template <bool VEC>
__global__ __launch_bounds__(256) void bn_apply_kernel(const float* __restrict__ x,
                                                       const float* __restrict__ ss,
                                                       const float* __restrict__ skip,
                                                       float* __restrict__ y, int C, int HW, int act,
                                                       size_t total) {
  if (VEC) {
    size_t i4 = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i4 >= total) return;
    int c = (int)((i4 / HW) % C);
    float sc = ss[c], sf = ss[C + c];
    float4 v = *reinterpret_cast<const float4*>(x + i4);
    v.x = apply_act(v.x * sc + sf, act);
    v.y = apply_act(v.y * sc + sf, act);
    v.z = apply_act(v.z * sc + sf, act);
    v.w = apply_act(v.w * sc + sf, act);
    if (skip) {
      float4 k = *reinterpret_cast<const float4*>(skip + i4);
      v.x += k.x; v.y += k.y; v.z += k.z; v.w += k.w;
    }
    *reinterpret_cast<float4*>(y + i4) = v;
  } else {
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    int c = (int)((i / HW) % C);
    float v = apply_act(x[i] * ss[c] + ss[C + c], act);
    if (skip) v += skip[i];
    y[i] = v;
  }
}

void bn_apply_f32(hipStream_t st, const float* x, const float* ss, const float* skip, float* y, int N,
                  int C, int HW, int act) {
  size_t total = (size_t)N * C * HW;
  if (HW % 4 == 0)
    KLAUNCH(bn_apply_kernel<true>, dim3(cdiv(total / 4, 256)), dim3(256), 0, st, x, ss, skip,
                       y, C, HW, act, total);
  else
    KLAUNCH(bn_apply_kernel<false>, dim3(cdiv(total, 256)), dim3(256), 0, st, x, ss, skip, y,
                       C, HW, act, total);
}

template <bool VEC>
__global__ __launch_bounds__(256) void bn_bwd_partial_kernel(const float* __restrict__ g,
                                                             const float* __restrict__ x,
                                                             const float* __restrict__ stat,
                                                             const float* __restrict__ ss,
                                                             double* __restrict__ ws, int N, int C,
                                                             int HW, int S, int act) {
  __shared__ double sh[16];
  const int c = blockIdx.x, s = blockIdx.y;
  long e0, e1;
  split_range((long)N * HW, S, s, e0, e1);
  const float mean = stat[c], istd = stat[C + c], sc = ss[c], sf = ss[C + c];
  float s1 = 0.f, s2 = 0.f;
  if (VEC) {
    for (long e = e0 + 4L * threadIdx.x; e < e1; e += 1024) {
      long n = e / HW;
      int p = (int)(e - n * HW);
      size_t off = ((size_t)n * C + c) * HW + p;
      float4 xv = *reinterpret_cast<const float4*>(x + off);
      float4 gv = *reinterpret_cast<const float4*>(g + off);
      float g0 = gv.x * act_mask(xv.x * sc + sf, act), g1 = gv.y * act_mask(xv.y * sc + sf, act);
      float g2 = gv.z * act_mask(xv.z * sc + sf, act), g3 = gv.w * act_mask(xv.w * sc + sf, act);
      s1 += (g0 + g1) + (g2 + g3);
      s2 += (g0 * ((xv.x - mean) * istd) + g1 * ((xv.y - mean) * istd)) +
            (g2 * ((xv.z - mean) * istd) + g3 * ((xv.w - mean) * istd));
    }
  } else {
    for (long e = e0 + threadIdx.x; e < e1; e += 256) {
      long n = e / HW;
      int p = (int)(e - n * HW);
      size_t off = ((size_t)n * C + c) * HW + p;
      float xv = x[off];
      float gv = g[off] * act_mask(xv * sc + sf, act);
      s1 += gv;
      s2 += gv * ((xv - mean) * istd);
    }
  }
  double d1 = block_sum<double>((double)s1, sh);
  double d2 = block_sum<double>((double)s2, sh);
  if (threadIdx.x == 0) {
    ws[((size_t)c * S + s) * 2 + 0] = d1;
    ws[((size_t)c * S + s) * 2 + 1] = d2;
  }
}

// coef[c] = gamma*istd, coef[C+c] = mean(g'), coef[2C+c] = mean(g'*xhat)
__global__ void bn_bwd_final_kernel(const double* __restrict__ ws, const float* __restrict__ stat,
                                    const float* __restrict__ gamma, float* __restrict__ Ggamma,
                                    float* __restrict__ Gbeta, float* __restrict__ coef, int C, int S,
                                    double count) {
  int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= C) return;
  double s1 = 0, s2 = 0;
  for (int s = 0; s < S; ++s) {
    s1 += ws[((size_t)c * S + s) * 2 + 0];
    s2 += ws[((size_t)c * S + s) * 2 + 1];
  }
  Gbeta[c] += (float)s1;
  Ggamma[c] += (float)s2;
  coef[c] = gamma[c] * stat[C + c];
  coef[C + c] = (float)(s1 / count);
  coef[2 * C + c] = (float)(s2 / count);
}

template <bool VEC>
__global__ __launch_bounds__(256) void bn_bwd_apply_kernel(const float* __restrict__ g,
                                                           const float* __restrict__ x,
                                                           const float* __restrict__ stat,
                                                           const float* __restrict__ ss,
                                                           const float* __restrict__ coef,
                                                           float* __restrict__ dx, int C, int HW,
                                                           int act, size_t total) {
  size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * (VEC ? 4 : 1);
  if (i >= total) return;
  int c = (int)((i / HW) % C);
  const float mean = stat[c], istd = stat[C + c], sc = ss[c], sf = ss[C + c];
  const float k = coef[c], m1 = coef[C + c], m2 = coef[2 * C + c];
  if (VEC) {
    float4 xv = *reinterpret_cast<const float4*>(x + i);
    float4 gv = *reinterpret_cast<const float4*>(g + i);
    float4 o;
    o.x = k * (gv.x * act_mask(xv.x * sc + sf, act) - m1 - (xv.x - mean) * istd * m2);
    o.y = k * (gv.y * act_mask(xv.y * sc + sf, act) - m1 - (xv.y - mean) * istd * m2);
    o.z = k * (gv.z * act_mask(xv.z * sc + sf, act) - m1 - (xv.z - mean) * istd * m2);
    o.w = k * (gv.w * act_mask(xv.w * sc + sf, act) - m1 - (xv.w - mean) * istd * m2);
    *reinterpret_cast<float4*>(dx + i) = o;
  } else {
    float xv = x[i];
    dx[i] = k * (g[i] * act_mask(xv * sc + sf, act) - m1 - (xv - mean) * istd * m2);
  }
}

void bn_bwd_f32(hipStream_t st, const float* g, const float* x, const float* stat, const float* ss,
                const float* gamma, float* dx, float* Ggamma, float* Gbeta, double* ws, float* coef,
                int N, int C, int HW, int act) {
  size_t per = (size_t)N * HW, total = per * C;
  int S = bn_split(C, per);
  bool vec = HW % 4 == 0;
  if (vec)
    KLAUNCH(bn_bwd_partial_kernel<true>, dim3(C, S), dim3(256), 0, st, g, x, stat, ss, ws, N,
                       C, HW, S, act);
  else
    KLAUNCH(bn_bwd_partial_kernel<false>, dim3(C, S), dim3(256), 0, st, g, x, stat, ss, ws, N,
                       C, HW, S, act);
  KLAUNCH(bn_bwd_final_kernel, dim3(cdiv(C, 128)), dim3(128), 0, st, ws, stat, gamma, Ggamma,
                     Gbeta, coef, C, S, (double)per);
  if (!dx) return;  // the input gradient is not wanted
  if (vec)
    KLAUNCH(bn_bwd_apply_kernel<true>, dim3(cdiv(total / 4, 256)), dim3(256), 0, st, g, x,
                       stat, ss, coef, dx, C, HW, act, total);
  else
    KLAUNCH(bn_bwd_apply_kernel<false>, dim3(cdiv(total, 256)), dim3(256), 0, st, g, x, stat,
                       ss, coef, dx, C, HW, act, total);
}

// ============================================================== elementwise
__global__ void act_fwd_kernel(const float* __restrict__ x, float* __restrict__ y, size_t n, int act) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) y[i] = apply_act(x[i], act);
}
__global__ void act_bwd_kernel(const float* __restrict__ g, const float* __restrict__ x,
                               float* __restrict__ dx, size_t n, int act) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dx[i] = g[i] * act_mask(x[i], act);
}
// y may alias a (in-place accumulation of a skip gradient): no __restrict__ here
__global__ void add_kernel(const float* a, const float* b, float* y, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) y[i] = a[i] + b[i];
}
// 16-byte copy / zero; sizes are multiples of 16 bytes by construction of the arenas,
// a ragged tail is handled bytewise by the last threads.
__global__ void copy16_kernel(const uint4* __restrict__ s, uint4* __restrict__ d, size_t n16,
                              const unsigned char* sb, unsigned char* db, size_t tail0, size_t bytes) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n16) d[i] = s[i];
  size_t t = tail0 + i;
  if (i < 16 && t < bytes) db[t] = sb[t];
}
__global__ void zero16_kernel(uint4* __restrict__ d, size_t n16, unsigned char* db, size_t tail0,
                              size_t bytes) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n16) d[i] = make_uint4(0, 0, 0, 0);
  size_t t = tail0 + i;
  if (i < 16 && t < bytes) db[t] = 0;
}
void act_fwd_f32(hipStream_t st, const float* x, float* y, size_t n, int act) {
  KLAUNCH(act_fwd_kernel, dim3(cdiv(n, 256)), dim3(256), 0, st, x, y, n, act);
}
void act_bwd_f32(hipStream_t st, const float* g, const float* x, float* dx, size_t n, int act) {
  KLAUNCH(act_bwd_kernel, dim3(cdiv(n, 256)), dim3(256), 0, st, g, x, dx, n, act);
}
void add_f32(hipStream_t st, const float* a, const float* b, float* y, size_t n) {
  KLAUNCH(add_kernel, dim3(cdiv(n, 256)), dim3(256), 0, st, a, b, y, n);
}
void copy_bytes(hipStream_t st, const void* src, void* dst, size_t bytes) {
  if (!bytes) return;
  size_t n16 = bytes / 16;
  size_t threads = n16 > 16 ? n16 : 16;
  KLAUNCH(copy16_kernel, dim3(cdiv(threads, 256)), dim3(256), 0, st, (const uint4*)src,
                     (uint4*)dst, n16, (const unsigned char*)src, (unsigned char*)dst, n16 * 16, bytes);
}
void fill_zero(hipStream_t st, void* dst, size_t bytes) {
  if (!bytes) return;
  size_t n16 = bytes / 16;
  size_t threads = n16 > 16 ? n16 : 16;
  KLAUNCH(zero16_kernel, dim3(cdiv(threads, 256)), dim3(256), 0, st, (uint4*)dst, n16,
                     (unsigned char*)dst, n16 * 16, bytes);
}

// ============================================================== pooling
__global__ __launch_bounds__(256) void gap_fwd_kernel(const float* __restrict__ x,
                                                      float* __restrict__ y, int NC, int HW) {
  int plane = blockIdx.x * 4 + (threadIdx.x >> 6);
  int lane = threadIdx.x & 63;
  if (plane >= NC) return;
  const float* xp = x + (size_t)plane * HW;
  float s = 0.f;
  for (int p = lane; p < HW; p += 64) s += xp[p];
  s = wave_sum(s);
  if (lane == 0) y[plane] = s / (float)HW;
}
__global__ void gap_bwd_kernel(const float* __restrict__ g, float* __restrict__ dx, size_t total,
                               int HW) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < total) dx[i] = g[i / HW] / (float)HW;
}
void gap_fwd_f32(hipStream_t st, const float* x, float* y, int NC, int HW) {
  KLAUNCH(gap_fwd_kernel, dim3(cdiv(NC, 4)), dim3(256), 0, st, x, y, NC, HW);
}
void gap_bwd_f32(hipStream_t st, const float* g, float* dx, int NC, int HW) {
  size_t total = (size_t)NC * HW;
  KLAUNCH(gap_bwd_kernel, dim3(cdiv(total, 256)), dim3(256), 0, st, g, dx, total, HW);
}

__device__ __forceinline__ int first_argmax4(float a, float b, float c, float d) {
  int k = 0;
  float m = a;
  if (b > m) { m = b; k = 1; }
  if (c > m) { m = c; k = 2; }
  if (d > m) { m = d; k = 3; }
  return k;
}
__global__ void maxpool_fwd_kernel(const float* __restrict__ x, float* __restrict__ y, int H, int W,
                                   int Ho, int Wo, size_t total) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  int j = (int)(idx % Wo);
  size_t t = idx / Wo;
  int i = (int)(t % Ho);
  size_t nc = t / Ho;
  const float* xp = x + nc * (size_t)H * W + (size_t)(2 * i) * W + 2 * j;
  y[idx] = fmaxf(fmaxf(xp[0], xp[1]), fmaxf(xp[W], xp[W + 1]));
}
__global__ void maxpool_bwd_kernel(const float* __restrict__ g, const float* __restrict__ x,
                                   float* __restrict__ dx, int H, int W, int Ho, int Wo, size_t total) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  int j = (int)(idx % W);
  size_t t = idx / W;
  int i = (int)(t % H);
  size_t nc = t / H;
  int io = i >> 1, jo = j >> 1;
  float v = 0.f;
  if (io < Ho && jo < Wo) {
    const float* xp = x + nc * (size_t)H * W + (size_t)(2 * io) * W + 2 * jo;
    int k = first_argmax4(xp[0], xp[1], xp[W], xp[W + 1]);
    if (k == ((i & 1) * 2 + (j & 1))) v = g[nc * (size_t)Ho * Wo + (size_t)io * Wo + jo];
  }
  dx[idx] = v;
}
void maxpool_fwd_f32(hipStream_t st, const float* x, float* y, int NC, int H, int W) {
  int Ho = H / 2, Wo = W / 2;
  size_t total = (size_t)NC * Ho * Wo;
  KLAUNCH(maxpool_fwd_kernel, dim3(cdiv(total, 256)), dim3(256), 0, st, x, y, H, W, Ho, Wo,
                     total);
}
void maxpool_bwd_f32(hipStream_t st, const float* g, const float* x, float* dx, int NC, int H, int W) {
  int Ho = H / 2, Wo = W / 2;
  size_t total = (size_t)NC * H * W;
  KLAUNCH(maxpool_bwd_kernel, dim3(cdiv(total, 256)), dim3(256), 0, st, g, x, dx, H, W, Ho,
                     Wo, total);
}

// ============================================================== linear (small row counts)
// one wavefront per output feature; rows processed 8 at a time
__global__ __launch_bounds__(256) void linear_fwd_kernel(const float* __restrict__ x,
                                                         const float* __restrict__ W,
                                                         const float* __restrict__ b,
                                                         float* __restrict__ y, int R, int Cin,
                                                         int Cout) {
  int o = blockIdx.x * 4 + (threadIdx.x >> 6);
  int lane = threadIdx.x & 63;
  if (o >= Cout) return;
  const float* wr = W + (size_t)o * Cin;
  for (int r0 = 0; r0 < R; r0 += 8) {
    float acc[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) acc[k] = 0.f;
    for (int i = lane; i < Cin; i += 64) {
      float wv = wr[i];
#pragma unroll
      for (int k = 0; k < 8; ++k)
        if (r0 + k < R) acc[k] += wv * x[(size_t)(r0 + k) * Cin + i];
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      float s = wave_sum(acc[k]);
      if (lane == 0 && r0 + k < R) y[(size_t)(r0 + k) * Cout + o] = s + (b ? b[o] : 0.f);
    }
  }
}
__global__ void linear_dgrad_kernel(const float* __restrict__ g, const float* __restrict__ W,
                                    float* __restrict__ dx, int R, int Cin, int Cout) {
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= R * Cin) return;
  int r = idx / Cin, i = idx - r * Cin;
  float acc = 0.f;
  for (int o = 0; o < Cout; ++o) acc += g[(size_t)r * Cout + o] * W[(size_t)o * Cin + i];
  dx[idx] = acc;
}
__global__ void linear_wgrad_kernel(const float* __restrict__ g, const float* __restrict__ x,
                                    float* __restrict__ GW, float* __restrict__ Gb, int R, int Cin,
                                    int Cout) {
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx < Cout * Cin) {
    int o = idx / Cin, i = idx - o * Cin;
    float acc = 0.f;
    for (int r = 0; r < R; ++r) acc += g[(size_t)r * Cout + o] * x[(size_t)r * Cin + i];
    GW[idx] += acc;
  }
  if (Gb && idx < Cout) {
    float acc = 0.f;
    for (int r = 0; r < R; ++r) acc += g[(size_t)r * Cout + idx];
    Gb[idx] += acc;
  }
}
void linear_fwd_f32(hipStream_t st, const float* x, const float* W, const float* b, float* y, int R,
                    int Cin, int Cout) {
  KLAUNCH(linear_fwd_kernel, dim3(cdiv(Cout, 4)), dim3(256), 0, st, x, W, b, y, R, Cin, Cout);
}
void linear_dgrad_f32(hipStream_t st, const float* g, const float* W, float* dx, int R, int Cin,
                      int Cout) {
  KLAUNCH(linear_dgrad_kernel, dim3(cdiv((long)R * Cin, 256)), dim3(256), 0, st, g, W, dx, R,
                     Cin, Cout);
}
void linear_wgrad_f32(hipStream_t st, const float* g, const float* x, float* GW, float* Gb, int R,
                      int Cin, int Cout) {
  KLAUNCH(linear_wgrad_kernel, dim3(cdiv((long)Cout * Cin, 256)), dim3(256), 0, st, g, x, GW,
                     Gb, R, Cin, Cout);
}

// ============================================================== softmax cross-entropy
__global__ __launch_bounds__(256) void softmax_ce_fwd_kernel(const float* __restrict__ z,
                                                             const int32_t* __restrict__ labels,
                                                             float* __restrict__ p,
                                                             float* __restrict__ row_loss, int C) {
  __shared__ float sh[16];
  __shared__ float shm[4];
  int r = blockIdx.x;
  const float* zr = z + (size_t)r * C;
  float m = -INFINITY;
  for (int i = threadIdx.x; i < C; i += 256) m = fmaxf(m, zr[i]);
  m = wave_max(m);
  if ((threadIdx.x & 63) == 0) shm[threadIdx.x >> 6] = m;
  __syncthreads();
  m = fmaxf(fmaxf(shm[0], shm[1]), fmaxf(shm[2], shm[3]));
  float s = 0.f;
  for (int i = threadIdx.x; i < C; i += 256) s += expf(zr[i] - m);
  s = block_sum<float>(s, sh);
  float inv = 1.f / s;
  for (int i = threadIdx.x; i < C; i += 256) p[(size_t)r * C + i] = expf(zr[i] - m) * inv;
  if (threadIdx.x == 0) {
    int lab = labels[r];
    row_loss[r] = (lab >= 0 && lab < C) ? -(zr[lab] - m - logf(s)) : 0.f;
  }
}
__global__ void loss_sum_kernel(const float* __restrict__ row_loss, float* __restrict__ out, int R,
                                float inv_denom) {
  // a single wavefront, fixed order: deterministic
  float s = 0.f;
  for (int i = threadIdx.x; i < R; i += 64) s += row_loss[i];
  s = wave_sum(s);
  if (threadIdx.x == 0) out[0] = s * inv_denom;
}
__global__ void softmax_ce_bwd_kernel(const float* __restrict__ p, const int32_t* __restrict__ labels,
                                      float* __restrict__ dz, int R, int C, float inv_denom) {
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= R * C) return;
  int r = idx / C, i = idx - r * C;
  float v = p[idx] - (labels[r] == i ? 1.f : 0.f);
  dz[idx] = v * inv_denom;
}
void softmax_ce_fwd_f32(hipStream_t st, const float* z, const int32_t* labels, float* p,
                        float* row_loss, float* loss_out, int R, int C, float inv_denom) {
  KLAUNCH(softmax_ce_fwd_kernel, dim3(R), dim3(256), 0, st, z, labels, p, row_loss, C);
  if (loss_out)
    KLAUNCH(loss_sum_kernel, dim3(1), dim3(64), 0, st, row_loss, loss_out, R, inv_denom);
}
void softmax_ce_bwd_f32(hipStream_t st, const float* p, const int32_t* labels, float* dz, int R, int C,
                        float inv_denom) {
  KLAUNCH(softmax_ce_bwd_kernel, dim3(cdiv((long)R * C, 256)), dim3(256), 0, st, p, labels,
                     dz, R, C, inv_denom);
}

// ============================================================== momentum SGD
__global__ __launch_bounds__(256) void sgd_kernel(float* __restrict__ w, float* __restrict__ g,
                                                  float* __restrict__ v, size_t n, float lr, float mu) {
  size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i + 3 < n) {
    float4 gv = *reinterpret_cast<float4*>(g + i);
    float4 vv = *reinterpret_cast<float4*>(v + i);
    float4 wv = *reinterpret_cast<float4*>(w + i);
    vv.x = mu * vv.x + gv.x; vv.y = mu * vv.y + gv.y; vv.z = mu * vv.z + gv.z; vv.w = mu * vv.w + gv.w;
    wv.x -= lr * vv.x; wv.y -= lr * vv.y; wv.z -= lr * vv.z; wv.w -= lr * vv.w;
    *reinterpret_cast<float4*>(v + i) = vv;
    *reinterpret_cast<float4*>(w + i) = wv;
    *reinterpret_cast<float4*>(g + i) = make_float4(0.f, 0.f, 0.f, 0.f);
  } else {
    for (; i < n; ++i) {
      float vv = mu * v[i] + g[i];
      v[i] = vv;
      w[i] -= lr * vv;
      g[i] = 0.f;
    }
  }
}
void sgd_momentum_f32(hipStream_t st, float* w, float* g, float* v, size_t n, float lr, float mu) {
  if (!n) return;
  KLAUNCH(sgd_kernel, dim3(cdiv(cdiv(n, 4), 256)), dim3(256), 0, st, w, g, v, n, lr, mu);
}

}  // namespace ast
