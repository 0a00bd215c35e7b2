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

static inline int conv_out(int H, int k, int stride, int pad) { return (H + 2 * pad - k) / stride + 1; }

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

// Dense 3x3 conv (pad 1, any stride) with up to 4 input channels (an RGB stem), forward: a thread
// owns one output position and eight output channels: its CG*9 inputs are read once into
// registers, the block's 8 x CG*9 weights sit in LDS (read as broadcasts), the eight results go
// out as eight coalesced stores.  The generic kernel spends ~400 instructions per output on
// index arithmetic and bounds checks; this one about 45.
template <int CG>
__global__ __launch_bounds__(256) void conv3x3_small_cin_fwd_kernel(const float* __restrict__ x,
                                                                    const float* __restrict__ w,
                                                                    const float* __restrict__ bias,
                                                                    float* __restrict__ y, int H, int W, int Cout,
                                                                    int Ho, int Wo, int stride) {
  constexpr int T = CG * 9, OC = 8;
  __shared__ float sw[OC * T];
  const int o0 = blockIdx.y * OC, n = blockIdx.z;
  for (int i = threadIdx.x; i < OC * T; i += 256) {
    const int oo = i / T;
    sw[i] = o0 + oo < Cout ? w[(size_t)(o0 + oo) * T + (i - oo * T)] : 0.f;
  }
  __syncthreads();
  const int r = blockIdx.x * 256 + threadIdx.x;
  if (r >= Ho * Wo) return;
  const int i = r / Wo, j = r - i * Wo;
  const int i0 = i * stride - 1, j0 = j * stride - 1;
  float xin[T];
#pragma unroll
  for (int c = 0; c < CG; ++c) {
    const float* xc = x + ((size_t)n * CG + c) * H * W;
#pragma unroll
    for (int u = 0; u < 3; ++u)
#pragma unroll
      for (int v = 0; v < 3; ++v) {
        const int ii = i0 + u, jj = j0 + v;
        const bool ok = ii >= 0 && ii < H && jj >= 0 && jj < W;
        xin[(c * 3 + u) * 3 + v] = ok ? xc[(size_t)ii * W + jj] : 0.f;
      }
  }
#pragma unroll
  for (int oo = 0; oo < OC; ++oo) {
    if (o0 + oo >= Cout) break;  // uniform
    float acc = bias ? bias[o0 + oo] : 0.f;
#pragma unroll
    for (int k = 0; k < T; ++k) acc += sw[oo * T + k] * xin[k];
    y[((size_t)n * Cout + o0 + oo) * Ho * Wo + r] = acc;
  }
}

// Dense 3x3 conv with up to 4 input channels (an RGB stem), weight gradient: block = four output
// channels x one chunk of the flattened (n, i, j) output positions; a thread reads the CG*9
// inputs of a position once and keeps the 4 x CG*9 sums of its positions in registers; the block
// adds them (DPP adds inside the rows of 16 lanes, then the 16 row sums through LDS in a fixed order)
// and writes one partial per chunk.  Positions are 32-bit (fewer than 2^31 per micro-batch, checked
// at create).
template <int CG>
__global__ __launch_bounds__(256) void conv3x3_small_cin_wgrad_kernel(
    const float* __restrict__ g, const float* __restrict__ x, float* __restrict__ part, int N, int H, int W,
    int Cout, int Ho, int Wo, int stride, int pad, int per_chunk) {
  constexpr int T = CG * 9, OC = 4;
  __shared__ float sh[16][OC * T];
  const int o0 = blockIdx.x * OC, chunk = blockIdx.y;
  const unsigned HWo = (unsigned)(Ho * Wo), per = (unsigned)N * HWo;
  const unsigned e0 = (unsigned)chunk * (unsigned)per_chunk, e1 = min(e0 + (unsigned)per_chunk, per);
  float acc[OC][T];
#pragma unroll
  for (int oo = 0; oo < OC; ++oo)
#pragma unroll
    for (int k = 0; k < T; ++k) acc[oo][k] = 0.f;
  for (unsigned e = e0 + threadIdx.x; e < e1; e += 256) {
    const int n = (int)(e / HWo);
    const int r = (int)(e - (unsigned)n * HWo);
    const int i = r / Wo, j = r - i * Wo;
    float gv[OC];
#pragma unroll
    for (int oo = 0; oo < OC; ++oo)
      gv[oo] = o0 + oo < Cout ? g[((size_t)n * Cout + o0 + oo) * Ho * Wo + r] : 0.f;
    const int i0 = i * stride - pad, j0 = j * stride - pad;
#pragma unroll
    for (int c = 0; c < CG; ++c) {
      const float* xc = x + ((size_t)n * CG + c) * H * W;
#pragma unroll
      for (int u = 0; u < 3; ++u) {
        const int ii = i0 + u;
#pragma unroll
        for (int v = 0; v < 3; ++v) {
          const int jj = j0 + v;
          const bool ok = ii >= 0 && ii < H && jj >= 0 && jj < W;
          const float xv = ok ? xc[(size_t)ii * W + jj] : 0.f;
#pragma unroll
          for (int oo = 0; oo < OC; ++oo) acc[oo][(c * 3 + u) * 3 + v] += gv[oo] * xv;
        }
      }
    }
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int oo = 0; oo < OC; ++oo)
#pragma unroll
    for (int k = 0; k < T; ++k) {
      const float s = row16_sum(acc[oo][k]);
      if ((lane & 15) == 0) sh[wave * 4 + (lane >> 4)][oo * T + k] = s;
    }
  __syncthreads();
  for (int q = threadIdx.x; q < OC * T; q += 256) {
    const int oo = q / T;
    if (o0 + oo < Cout) {
      float s = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) s += sh[r][q];
      part[((size_t)chunk * Cout + o0 + oo) * T + (q - oo * T)] = s;
    }
  }
}

static int small_cin_chunks(int N, int Ho, int Wo, int Cout) {
  long per = (long)N * Ho * Wo;
  const int og = (Cout + 3) / 4;                   // blocks per chunk: four output channels each
  int want = (int)((1024 + og - 1) / og);          // about 1024 blocks
  long cap = (per + 1023) / 1024;                  // at least 1024 positions per block
  if (want > cap) want = (int)cap;
  return want < 1 ? 1 : want;
}
static bool small_cin_case(int Cin, int k, int groups) { return groups == 1 && k == 3 && Cin >= 1 && Cin <= 4; }

size_t conv_direct_wgrad_ws(int N, int Cin, int H, int W, int Cout, int k, int stride, int pad, int groups) {
  if (!small_cin_case(Cin, k, groups)) return 0;
  int Ho = conv_out(H, k, stride, pad), Wo = conv_out(W, k, stride, pad);
  return (size_t)small_cin_chunks(N, Ho, Wo, Cout) * Cout * Cin * 9;
}

void conv_direct_fwd_f32(hipStream_t st, const float* x, const float* w, const float* bias, float* y,
                         int N, int Cin, int H, int W, int Cout, int k, int stride, int pad,
                         int groups) {
  int Ho = conv_out(H, k, stride, pad), Wo = conv_out(W, k, stride, pad);
  if (small_cin_case(Cin, k, groups) && pad == 1 && N <= 65535) {
    dim3 grid(cdiv((long)Ho * Wo, 256), cdiv(Cout, 8), N);
    switch (Cin) {
      case 1: KLAUNCH(conv3x3_small_cin_fwd_kernel<1>, grid, dim3(256), 0, st, x, w, bias, y, H, W, Cout, Ho, Wo, stride); break;
      case 2: KLAUNCH(conv3x3_small_cin_fwd_kernel<2>, grid, dim3(256), 0, st, x, w, bias, y, H, W, Cout, Ho, Wo, stride); break;
      case 3: KLAUNCH(conv3x3_small_cin_fwd_kernel<3>, grid, dim3(256), 0, st, x, w, bias, y, H, W, Cout, Ho, Wo, stride); break;
      default: KLAUNCH(conv3x3_small_cin_fwd_kernel<4>, grid, dim3(256), 0, st, x, w, bias, y, H, W, Cout, Ho, Wo, stride); break;
    }
    return;
  }
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
void conv_direct_wgrad_f32(hipStream_t st, const float* g, const float* x, float* G, float* ws, int N, int Cin,
                           int H, int W, int Cout, int k, int stride, int pad, int groups) {
  int Ho = conv_out(H, k, stride, pad), Wo = conv_out(W, k, stride, pad);
  if (ws && small_cin_case(Cin, k, groups)) {
    const int chunks = small_cin_chunks(N, Ho, Wo, Cout);
    const int per_chunk = cdiv((long)N * Ho * Wo, chunks);
    dim3 grid(cdiv(Cout, 4), chunks);
    switch (Cin) {
      case 1: KLAUNCH(conv3x3_small_cin_wgrad_kernel<1>, grid, dim3(256), 0, st, g, x, ws, N, H, W, Cout, Ho, Wo, stride, pad, per_chunk); break;
      case 2: KLAUNCH(conv3x3_small_cin_wgrad_kernel<2>, grid, dim3(256), 0, st, g, x, ws, N, H, W, Cout, Ho, Wo, stride, pad, per_chunk); break;
      case 3: KLAUNCH(conv3x3_small_cin_wgrad_kernel<3>, grid, dim3(256), 0, st, g, x, ws, N, H, W, Cout, Ho, Wo, stride, pad, per_chunk); break;
      default: KLAUNCH(conv3x3_small_cin_wgrad_kernel<4>, grid, dim3(256), 0, st, g, x, ws, N, H, W, Cout, Ho, Wo, stride, pad, per_chunk); break;
    }
    reduce_parts_acc_f32(st, ws, G, (size_t)Cout * Cin * 9, chunks);
    return;
  }
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

// ============================================================== elementwise
// the standalone activation layers also know swish and sigmoid
__device__ __forceinline__ float act_value(float v, int act) {
  if (act == ACT_SWISH) return v * sigmoid_f(v);
  if (act == ACT_SIGMOID) return sigmoid_f(v);
  return apply_act(v, act);
}
// derivative of the activation at pre-activation v
__device__ __forceinline__ float act_slope(float v, int act) {
  if (act == ACT_SWISH) return act_slope_sw<true>(v, act);
  if (act == ACT_SIGMOID) { const float s = sigmoid_f(v); return s * (1.f - s); }
  return act_mask(v, act);
}
__global__ void act_fwd_kernel(const float* __restrict__ x, float* __restrict__ y, size_t n, int act) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) y[i] = act_value(x[i], act);
}
__global__ void act_bwd_kernel(const float* __restrict__ g, const float* __restrict__ x,
                               float* __restrict__ dx, size_t n, int act) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dx[i] = g[i] * act_slope(x[i], act);
}
// four elements per thread (n4 = n / 4 whole float4; buffers are 256-byte aligned arena slices)
__global__ void act_fwd4_kernel(const float4* __restrict__ x, float4* __restrict__ y, size_t n4, int act) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n4) return;
  float4 v = x[i];
  v.x = act_value(v.x, act); v.y = act_value(v.y, act); v.z = act_value(v.z, act); v.w = act_value(v.w, act);
  y[i] = v;
}
__global__ void act_bwd4_kernel(const float4* __restrict__ g, const float4* __restrict__ x, float4* __restrict__ dx,
                                size_t n4, int act) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n4) return;
  const float4 v = x[i];
  float4 d = g[i];
  d.x *= act_slope(v.x, act); d.y *= act_slope(v.y, act); d.z *= act_slope(v.z, act); d.w *= act_slope(v.w, act);
  dx[i] = d;
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
static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
void act_fwd_f32(hipStream_t st, const float* x, float* y, size_t n, int act) {
  if (n % 4 == 0 && n >= 4096 && aligned16(x) && aligned16(y))
    KLAUNCH(act_fwd4_kernel, dim3(cdiv(n / 4, 256)), dim3(256), 0, st, (const float4*)x, (float4*)y, n / 4, act);
  else
    KLAUNCH(act_fwd_kernel, dim3(cdiv(n, 256)), dim3(256), 0, st, x, y, n, act);
}
void act_bwd_f32(hipStream_t st, const float* g, const float* x, float* dx, size_t n, int act) {
  if (n % 4 == 0 && n >= 4096 && aligned16(g) && aligned16(x) && aligned16(dx))
    KLAUNCH(act_bwd4_kernel, dim3(cdiv(n / 4, 256)), dim3(256), 0, st, (const float4*)g, (const float4*)x, (float4*)dx,
            n / 4, act);
  else
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
// mean over each plane; TPP threads per plane (a wavefront for small planes, the block for large ones:
// a squeeze-and-excitation block pools 120 x 120 planes), four loads in flight per thread
template <int TPP>
__global__ __launch_bounds__(256) void gap_fwd_kernel(const float* __restrict__ x, float* __restrict__ y, int NC, int HW) {
  __shared__ float sh[4];
  const int plane = blockIdx.x * (256 / TPP) + threadIdx.x / TPP;
  const int t = threadIdx.x % TPP, lane = threadIdx.x & 63;
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
  if (plane < NC) {
    const float* xp = x + (size_t)plane * HW;
    if ((HW & 3) == 0) {
      const float4* x4 = reinterpret_cast<const float4*>(xp);
      const int n4 = HW / 4;
      int p = t;
      for (; p + 3 * TPP < n4; p += 4 * TPP) {
        const float4 a = x4[p], b = x4[p + TPP], c = x4[p + 2 * TPP], d = x4[p + 3 * TPP];
        s0 += (a.x + a.y) + (a.z + a.w);
        s1 += (b.x + b.y) + (b.z + b.w);
        s2 += (c.x + c.y) + (c.z + c.w);
        s3 += (d.x + d.y) + (d.z + d.w);
      }
      for (; p < n4; p += TPP) {
        const float4 a = x4[p];
        s0 += (a.x + a.y) + (a.z + a.w);
      }
    } else {
      int p = t;
      for (; p + 3 * TPP < HW; p += 4 * TPP) {
        s0 += xp[p]; s1 += xp[p + TPP]; s2 += xp[p + 2 * TPP]; s3 += xp[p + 3 * TPP];
      }
      for (; p < HW; p += TPP) s0 += xp[p];
    }
  }
  float s = wave_sum((s0 + s1) + (s2 + s3));
  if (TPP == 64) {
    if (lane == 0 && plane < NC) y[plane] = s / (float)HW;
  } else {
    if (lane == 0) sh[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0 && plane < NC) y[plane] = ((sh[0] + sh[1]) + (sh[2] + sh[3])) / (float)HW;
  }
}
__global__ void gap_bwd_kernel(const float* __restrict__ g, float* __restrict__ dx, size_t total,
                               int HW) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < total) dx[i] = g[i / HW] / (float)HW;
}
void gap_fwd_f32(hipStream_t st, const float* x, float* y, int NC, int HW) {
  if (HW >= 2048) KLAUNCH_NAMED("gap_fwd_kernel", (gap_fwd_kernel<256>), dim3(NC), dim3(256), 0, st, x, y, NC, HW);
  else KLAUNCH_NAMED("gap_fwd_kernel", (gap_fwd_kernel<64>), dim3(cdiv(NC, 4)), dim3(256), 0, st, x, y, NC, HW);
}
__global__ void gap_bwd_acc_kernel(const float* __restrict__ g, float* __restrict__ dx, size_t total, int HW) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < total) dx[i] += g[i / HW] / (float)HW;
}
void gap_bwd_f32(hipStream_t st, const float* g, float* dx, int NC, int HW, bool accumulate) {
  size_t total = (size_t)NC * HW;
  if (accumulate) KLAUNCH(gap_bwd_acc_kernel, dim3(cdiv(total, 256)), dim3(256), 0, st, g, dx, total, HW);
  else KLAUNCH(gap_bwd_kernel, dim3(cdiv(total, 256)), dim3(256), 0, st, g, dx, total, HW);
}

// ============================================================== squeeze-and-excitation scale
// y[plane][p] = x[plane][p] * gate[plane]; one wavefront per plane (sample, channel), four per block
__global__ __launch_bounds__(256) void se_scale_fwd_kernel(const float* __restrict__ x, const float* __restrict__ gate,
                                                           float* __restrict__ y, int NC, int HW) {
  const int plane = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (plane >= NC) return;
  const float gt = gate[plane];
  const float* xp = x + (size_t)plane * HW;
  float* yp = y + (size_t)plane * HW;
  if ((HW & 3) == 0) {
    const float4* x4 = reinterpret_cast<const float4*>(xp);
    float4* y4 = reinterpret_cast<float4*>(yp);
    for (int p = lane; p < HW / 4; p += 64) {
      float4 v = x4[p];
      v.x *= gt; v.y *= gt; v.z *= gt; v.w *= gt;
      y4[p] = v;
    }
  } else {
    for (int p = lane; p < HW; p += 64) yp[p] = xp[p] * gt;
  }
}
// dgate[plane] = sum_p dy*x;  dx[plane][p] = dy[plane][p] * gate[plane]  (dx may be NULL)
__global__ __launch_bounds__(256) void se_scale_bwd_kernel(const float* __restrict__ dy, const float* __restrict__ x,
                                                           const float* __restrict__ gate, float* __restrict__ dgate,
                                                           float* __restrict__ dx, int NC, int HW) {
  const int plane = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (plane >= NC) return;
  const float gt = gate[plane];
  const float* gp = dy + (size_t)plane * HW;
  const float* xp = x + (size_t)plane * HW;
  float* dp = dx ? dx + (size_t)plane * HW : nullptr;
  float acc = 0.f;
  if ((HW & 3) == 0) {
    const float4* g4 = reinterpret_cast<const float4*>(gp);
    const float4* x4 = reinterpret_cast<const float4*>(xp);
    float4* d4 = reinterpret_cast<float4*>(dp);
    for (int p = lane; p < HW / 4; p += 64) {
      float4 g = g4[p];
      const float4 v = x4[p];
      acc += g.x * v.x + g.y * v.y + g.z * v.z + g.w * v.w;
      if (dp) {
        g.x *= gt; g.y *= gt; g.z *= gt; g.w *= gt;
        d4[p] = g;
      }
    }
  } else {
    for (int p = lane; p < HW; p += 64) {
      const float g = gp[p];
      acc += g * xp[p];
      if (dp) dp[p] = g * gt;
    }
  }
  acc = wave_sum(acc);
  if (lane == 0) dgate[plane] = acc;
}
void se_scale_fwd_f32(hipStream_t st, const float* x, const float* gate, float* y, int NC, int HW) {
  KLAUNCH(se_scale_fwd_kernel, dim3(cdiv(NC, 4)), dim3(256), 0, st, x, gate, y, NC, HW);
}
void se_scale_bwd_f32(hipStream_t st, const float* dy, const float* x, const float* gate, float* dgate, float* dx,
                      int NC, int HW) {
  KLAUNCH(se_scale_bwd_kernel, dim3(cdiv(NC, 4)), dim3(256), 0, st, dy, x, gate, dgate, dx, NC, HW);
}

// first maximum (row-major) of the 3x3 window of output (i, j): window rows 2i-1 .. 2i+1, columns 2j-1 .. 2j+1,
// positions outside the image skipped.  Returns the flat input index; the window always holds (2i, 2j).
__device__ __forceinline__ int maxpool3_argmax(const float* __restrict__ xp, int H, int W, int i, int j, float& best) {
  int arg = -1;
  best = 0.f;
#pragma unroll
  for (int u = 0; u < 3; ++u) {
    const int ii = 2 * i - 1 + u;
    if (ii < 0 || ii >= H) continue;
#pragma unroll
    for (int v = 0; v < 3; ++v) {
      const int jj = 2 * j - 1 + v;
      if (jj < 0 || jj >= W) continue;
      const float val = xp[(size_t)ii * W + jj];
      if (arg < 0 || val > best) { best = val; arg = ii * W + jj; }
    }
  }
  return arg;
}
__global__ void maxpool3x3s2_fwd_kernel(const float* __restrict__ x, float* __restrict__ y, int H, int W, int Ho, int Wo,
                                        size_t total) {
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int j = (int)(idx % Wo);
  const size_t t = idx / Wo;
  const int i = (int)(t % Ho);
  const size_t plane = t / Ho;
  float best;
  maxpool3_argmax(x + plane * H * W, H, W, i, j, best);
  y[idx] = best;
}
// thread per input position: the windows that hold it are those of outputs (ceil((r-1)/2) .. floor((r+1)/2)) per axis
__global__ void maxpool3x3s2_bwd_kernel(const float* __restrict__ g, const float* __restrict__ x, float* __restrict__ dx,
                                        int H, int W, int Ho, int Wo, size_t total) {
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int c = (int)(idx % W);
  const size_t t = idx / W;
  const int r = (int)(t % H);
  const size_t plane = t / H;
  const float* xp = x + plane * H * W;
  const float* gp = g + plane * Ho * Wo;
  const int self = r * W + c;
  float acc = 0.f;
  const int i0 = r / 2, i1 = min((r + 1) / 2, Ho - 1);   // ceil((r-1)/2) = r/2 for r >= 0
  const int j0 = c / 2, j1 = min((c + 1) / 2, Wo - 1);
  for (int i = i0; i <= i1; ++i)
    for (int j = j0; j <= j1; ++j) {
      float best;
      if (maxpool3_argmax(xp, H, W, i, j, best) == self) acc += gp[(size_t)i * Wo + j];
    }
  dx[idx] = acc;
}
void maxpool3x3s2_fwd_f32(hipStream_t st, const float* x, float* y, int NC, int H, int W) {
  const int Ho = (H - 1) / 2 + 1, Wo = (W - 1) / 2 + 1;
  const size_t total = (size_t)NC * Ho * Wo;
  KLAUNCH(maxpool3x3s2_fwd_kernel, dim3(cdiv(total, 256)), dim3(256), 0, st, x, y, H, W, Ho, Wo, total);
}
void maxpool3x3s2_bwd_f32(hipStream_t st, const float* g, const float* x, float* dx, int NC, int H, int W) {
  const int Ho = (H - 1) / 2 + 1, Wo = (W - 1) / 2 + 1;
  const size_t total = (size_t)NC * H * W;
  KLAUNCH(maxpool3x3s2_bwd_kernel, dim3(cdiv(total, 256)), dim3(256), 0, st, g, x, dx, H, W, Ho, Wo, total);
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
    for (int i0 = lane; i0 < Cin; i0 += 256) {  // four weights and their inputs requested at once
      float wv[4], xv[4][8];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int i = i0 + 64 * u;
        wv[u] = i < Cin ? wr[i] : 0.f;
#pragma unroll
        for (int k = 0; k < 8; ++k) xv[u][k] = (i < Cin && r0 + k < R) ? x[(size_t)(r0 + k) * Cin + i] : 0.f;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int k = 0; k < 8; ++k) acc[k] += wv[u] * xv[u][k];
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      float s = wave_sum(acc[k]);
      if (lane == 0 && r0 + k < R) y[(size_t)(r0 + k) * Cout + o] = s + (b ? b[o] : 0.f);
    }
  }
}
// dx[r][i] = sum_o g[r][o] W[o][i].  Block = 64 input features x 16 slices of the output
// features; a wavefront streams its rows of W (coalesced) against up to eight rows of g at a
// time, the sixteen partial sums are added through LDS in a fixed order.
__global__ __launch_bounds__(1024) void linear_dgrad_kernel(const float* __restrict__ g, const float* __restrict__ W,
                                                            float* __restrict__ dx, int R, int Cin, int Cout) {
  __shared__ float sh[16][8][64];
  const int il = threadIdx.x & 63, os = threadIdx.x >> 6;
  const int i = blockIdx.x * 64 + il;
  const bool iv = i < Cin;
  for (int r0 = 0; r0 < R; r0 += 8) {
    float acc[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) acc[q] = 0.f;
    for (int o0 = os; o0 < Cout; o0 += 64) {  // four weights and their gradients requested at once
      float wv[4], gv[4][8];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int o = o0 + 16 * u;
        wv[u] = (iv && o < Cout) ? W[(size_t)o * Cin + i] : 0.f;
#pragma unroll
        for (int q = 0; q < 8; ++q) gv[u][q] = (o < Cout && r0 + q < R) ? g[(size_t)(r0 + q) * Cout + o] : 0.f;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int q = 0; q < 8; ++q) acc[q] += gv[u][q] * wv[u];
    }
    __syncthreads();  // the previous round's sums have been read
#pragma unroll
    for (int q = 0; q < 8; ++q) sh[os][q][il] = acc[q];
    __syncthreads();
    if (os < 8 && r0 + os < R && iv) {
      float s = 0.f;
#pragma unroll
      for (int k = 0; k < 16; ++k) s += sh[k][os][il];
      dx[(size_t)(r0 + os) * Cin + i] = s;
    }
  }
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
  KLAUNCH(linear_dgrad_kernel, dim3(cdiv(Cin, 64)), dim3(1024), 0, st, g, W, dx, R, Cin, Cout);
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
