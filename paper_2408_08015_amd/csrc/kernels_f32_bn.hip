// BatchNorm2d (training mode, NCHW, fp32) forward and backward, HBM-bound.
//
// Each direction is two streaming kernels and nothing else:
//   partial:  (channel, part) blocks reduce a few whole samples or one plane chunk of the
//             channel (fp32 per thread, fp64 across threads) into ws[channel][part][2];
//   apply:    one block per (plane, chunk); its first wavefront adds the channel's partials
//             in a fixed butterfly order in fp64 (every block of a channel computes bit-identical
//             coefficients), then the block streams its chunk.  The block of sample 0 /
//             chunk 0 also records the channel's statistics, or accumulates dgamma / dbeta
//             into G.
// Doing the tiny "finish the reduction" step inside the consumer removes two
// latency-bound launches per BatchNorm per micro-batch.
#include "bn_common.h"
#include "device_utils.h"
#include "kernels.h"
#include "prof.h"

namespace ast {

static inline int cdiv(long a, long b) { return (int)((a + b - 1) / b); }

// A channel's N*HW elements are N contiguous planes.  A partial-sum block takes `spb` whole
// samples (small planes) or one chunk of one plane (large planes) of one channel, so it
// streams contiguous memory with no index arithmetic per element; P = groups * chunks
// partial pairs per channel.
struct BnSplit { int spb, groups, nchunks, chunk, P; };
static inline BnSplit bn_split(int N, int HW) {
  BnSplit b;
  b.nchunks = cdiv(HW, 4096);
  b.chunk = (cdiv(HW, b.nchunks) + 3) & ~3;
  b.nchunks = cdiv(HW, b.chunk);
  b.spb = b.nchunks > 1 ? 1 : 4096 / HW;
  if (b.spb < 1) b.spb = 1;
  if (b.spb > N) b.spb = N;
  b.groups = cdiv(N, b.spb);
  b.P = b.groups * b.nchunks;
  return b;
}
size_t bn_ws_doubles(int C, int N, int HW) { return (size_t)C * bn_split(N, HW).P * 2; }

// both sums of a block in one pass; the result is valid in thread 0
__device__ __forceinline__ void block_sum2(float f1, float f2, double* sh, double& d1, double& d2) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const double a = wave_sum_d((double)f1), b = wave_sum_d((double)f2);
  if (lane == 0) {
    sh[w] = a;
    sh[4 + w] = b;
  }
  __syncthreads();
  d1 = (sh[0] + sh[1]) + (sh[2] + sh[3]);
  d2 = (sh[4] + sh[5]) + (sh[6] + sh[7]);
}

template <bool VEC>
__global__ __launch_bounds__(256) void bn_stats_partial_kernel(const float* __restrict__ x,
                                                               double* __restrict__ ws, int N, int C, int HW,
                                                               BnSplit b) {
  __shared__ double sh[8];
  const int c = blockIdx.x, grp = blockIdx.y / b.nchunks, ch = blockIdx.y - grp * b.nchunks;
  const int n0 = grp * b.spb, n1 = min(n0 + b.spb, N);
  const int e0 = ch * b.chunk, e1 = min(e0 + b.chunk, HW), len = e1 - e0;
  float s1 = 0.f, s2 = 0.f;
  if (VEC) {
    // a block's share is at most 4096 elements: all of a thread's words are requested at once
    const int q = len >> 2, total = (n1 - n0) * q;
    for (int i0 = threadIdx.x; i0 < total; i0 += 1024) {
      float4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int idx = i0 + 256 * u;
        v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (idx < total) {
          const int nl = idx / q, e = e0 + 4 * (idx - nl * q);
          v[u] = *reinterpret_cast<const float4*>(x + ((size_t)(n0 + nl) * C + c) * HW + e);
        }
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        s1 += (v[u].x + v[u].y) + (v[u].z + v[u].w);
        s2 += (v[u].x * v[u].x + v[u].y * v[u].y) + (v[u].z * v[u].z + v[u].w * v[u].w);
      }
    }
  } else {
    const int total = (n1 - n0) * len;
    for (int idx = threadIdx.x; idx < total; idx += 256) {
      const int nl = idx / len, e = e0 + idx - nl * len;
      const float v = x[((size_t)(n0 + nl) * C + c) * HW + e];
      s1 += v;
      s2 += v * v;
    }
  }
  double d1, d2;
  block_sum2(s1, s2, sh, d1, d2);
  if (threadIdx.x == 0) {
    ws[((size_t)c * b.P + blockIdx.y) * 2 + 0] = d1;
    ws[((size_t)c * b.P + blockIdx.y) * 2 + 1] = d2;
  }
}

// y = act(x*scale + shift) (+ skip); grid (planes, chunks)
template <bool VEC, bool SW = false>
__global__ __launch_bounds__(256) void bn_apply_kernel(const float* __restrict__ x,
                                                       const double* __restrict__ ws,
                                                       const float* __restrict__ gamma,
                                                       const float* __restrict__ beta,
                                                       const float* __restrict__ skip, float* __restrict__ y,
                                                       float* __restrict__ stat, float* __restrict__ ss,
                                                       float* __restrict__ running, int C, int HW, int S,
                                                       double count, float eps, int act, int chunk) {
  __shared__ float coef[2];
  const int plane = blockIdx.x, c = plane % C;
  const int e0 = blockIdx.y * chunk, e1 = min(e0 + chunk, HW);
  const size_t base = (size_t)plane * HW;
  // The chunk's data (at most 4096 elements: four 16-byte words per thread) is requested before
  // the statistics are finished, so the two memory latencies overlap instead of adding up.
  float4 xv[4], kv[4];
  if (VEC) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int e = e0 + 4 * threadIdx.x + 1024 * u;
      if (e < e1) {
        xv[u] = *reinterpret_cast<const float4*>(x + base + e);
        if (skip) kv[u] = *reinterpret_cast<const float4*>(skip + base + e);
      }
    }
  }
  if (threadIdx.x < 64) {
    double s1, s2;
    bn_add_partials(ws, c, S, s1, s2);
    if (threadIdx.x == 0)  // sample 0, chunk 0 records the channel's statistics
      bn_coefficients(s1, s2, count, gamma[c], beta[c], eps, c, C, plane < C && blockIdx.y == 0, stat, ss, running,
                      coef[0], coef[1]);
  }
  __syncthreads();
  const float sc = coef[0], sf = coef[1];
  if (VEC) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int e = e0 + 4 * threadIdx.x + 1024 * u;
      if (e < e1) {
        float4 v = xv[u];
        v.x = apply_act_sw<SW>(v.x * sc + sf, act);
        v.y = apply_act_sw<SW>(v.y * sc + sf, act);
        v.z = apply_act_sw<SW>(v.z * sc + sf, act);
        v.w = apply_act_sw<SW>(v.w * sc + sf, act);
        if (skip) {
          v.x += kv[u].x; v.y += kv[u].y; v.z += kv[u].z; v.w += kv[u].w;
        }
        *reinterpret_cast<float4*>(y + base + e) = v;
      }
    }
    for (int e = e0 + 4 * threadIdx.x + 4096; e < e1; e += 1024) {  // longer chunks (not produced by the launcher)
      float4 v = *reinterpret_cast<const float4*>(x + base + e);
      v.x = apply_act_sw<SW>(v.x * sc + sf, act);
      v.y = apply_act_sw<SW>(v.y * sc + sf, act);
      v.z = apply_act_sw<SW>(v.z * sc + sf, act);
      v.w = apply_act_sw<SW>(v.w * sc + sf, act);
      if (skip) {
        float4 k = *reinterpret_cast<const float4*>(skip + base + e);
        v.x += k.x; v.y += k.y; v.z += k.z; v.w += k.w;
      }
      *reinterpret_cast<float4*>(y + base + e) = v;
    }
  } else {
    for (int e = e0 + threadIdx.x; e < e1; e += 256) {
      float v = apply_act_sw<SW>(x[base + e] * sc + sf, act);
      if (skip) v += skip[base + e];
      y[base + e] = v;
    }
  }
}

static inline void bn_chunking(int HW, int& nchunks, int& chunk) {
  nchunks = cdiv(HW, 4096);
  chunk = (cdiv(HW, nchunks) + 3) & ~3;
  nchunks = cdiv(HW, chunk);
}

int bn_parts(int N, int HW) { return bn_split(N, HW).P; }

void bn_stats_f32(hipStream_t st, const float* x, double* ws, int N, int C, int HW) {
  const BnSplit b = bn_split(N, HW);
  if (HW % 4 == 0) KLAUNCH(bn_stats_partial_kernel<true>, dim3(C, b.P), dim3(256), 0, st, x, ws, N, C, HW, b);
  else KLAUNCH(bn_stats_partial_kernel<false>, dim3(C, b.P), dim3(256), 0, st, x, ws, N, C, HW, b);
}

void bn_apply_f32(hipStream_t st, const float* x, const float* gamma, const float* beta, const float* skip, float* y,
                  float* stat, float* scale_shift, float* running, const double* ws, int P, int N, int C, int HW,
                  float eps, int act) {
  size_t per = (size_t)N * HW;
  int nchunks, chunk;
  bn_chunking(HW, nchunks, chunk);
  dim3 grid((unsigned)(N * C), nchunks);
#define BN_APPLY(name, kern)                                                                                          \
  KLAUNCH_NAMED(name, kern, grid, dim3(256), 0, st, x, ws, gamma, beta, skip, y, stat, scale_shift, running, C, HW, P, \
                (double)per, eps, act, chunk)
  const bool sw = act == ACT_SWISH;  // the swish instantiations share the profile names of the others
  if (HW % 4 == 0) {
    if (sw) BN_APPLY("bn_apply_kernel<true>", (bn_apply_kernel<true, true>));
    else BN_APPLY("bn_apply_kernel<true>", (bn_apply_kernel<true, false>));
  } else {
    if (sw) BN_APPLY("bn_apply_kernel<false>", (bn_apply_kernel<false, true>));
    else BN_APPLY("bn_apply_kernel<false>", (bn_apply_kernel<false, false>));
  }
#undef BN_APPLY
}

void bn_fwd_f32(hipStream_t st, const float* x, const float* gamma, const float* beta, const float* skip,
                float* y, float* stat, float* scale_shift, float* running, double* ws, int N, int C, int HW,
                float eps, int act) {
  bn_stats_f32(st, x, ws, N, C, HW);
  bn_apply_f32(st, x, gamma, beta, skip, y, stat, scale_shift, running, ws, bn_parts(N, HW), N, C, HW, eps, act);
}

template <bool VEC, bool SW = false>
__global__ __launch_bounds__(256) void bn_bwd_partial_kernel(const float* __restrict__ g,
                                                             const float* __restrict__ x,
                                                             const float* __restrict__ stat,
                                                             const float* __restrict__ ss,
                                                             double* __restrict__ ws, int N, int C,
                                                             int HW, BnSplit b, int act) {
  __shared__ double sh[8];
  const int c = blockIdx.x, grp = blockIdx.y / b.nchunks, ch = blockIdx.y - grp * b.nchunks;
  const int n0 = grp * b.spb, n1 = min(n0 + b.spb, N);
  const int e0 = ch * b.chunk, e1 = min(e0 + b.chunk, HW), len = e1 - e0;
  const float mean = stat[c], istd = stat[C + c], sc = ss[c], sf = ss[C + c];
  float s1 = 0.f, s2 = 0.f;
  if (VEC) {
    // a block's share is at most 4096 elements: all of a thread's words are requested at once
    const int q = len >> 2, total = (n1 - n0) * q;
    for (int i0 = threadIdx.x; i0 < total; i0 += 1024) {
      float4 xq[4], gq[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int idx = i0 + 256 * u;
        xq[u] = gq[u] = make_float4(0.f, 0.f, 0.f, 0.f);  // g = 0 adds nothing to either sum
        if (idx < total) {
          const int nl = idx / q, e = e0 + 4 * (idx - nl * q);
          const size_t off = ((size_t)(n0 + nl) * C + c) * HW + e;
          xq[u] = *reinterpret_cast<const float4*>(x + off);
          gq[u] = *reinterpret_cast<const float4*>(g + off);
        }
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const float4 xv = xq[u], gv = gq[u];
        float g0 = gv.x * act_slope_sw<SW>(xv.x * sc + sf, act), g1 = gv.y * act_slope_sw<SW>(xv.y * sc + sf, act);
        float g2 = gv.z * act_slope_sw<SW>(xv.z * sc + sf, act), g3 = gv.w * act_slope_sw<SW>(xv.w * sc + sf, act);
        s1 += (g0 + g1) + (g2 + g3);
        s2 += (g0 * ((xv.x - mean) * istd) + g1 * ((xv.y - mean) * istd)) +
              (g2 * ((xv.z - mean) * istd) + g3 * ((xv.w - mean) * istd));
      }
    }
  } else {
    const int total = (n1 - n0) * len;
    for (int idx = threadIdx.x; idx < total; idx += 256) {
      const int nl = idx / len, e = e0 + idx - nl * len;
      const size_t off = ((size_t)(n0 + nl) * C + c) * HW + e;
      float xv = x[off];
      float gv = g[off] * act_slope_sw<SW>(xv * sc + sf, act);
      s1 += gv;
      s2 += gv * ((xv - mean) * istd);
    }
  }
  double d1, d2;
  block_sum2(s1, s2, sh, d1, d2);
  if (threadIdx.x == 0) {
    ws[((size_t)c * b.P + blockIdx.y) * 2 + 0] = d1;
    ws[((size_t)c * b.P + blockIdx.y) * 2 + 1] = d2;
  }
}

// dx = gamma*istd*(g' - mean(g') - xhat*mean(g'*xhat)); sample 0 / chunk 0 blocks add dgamma, dbeta to G
template <bool VEC, bool SW = false>
__global__ __launch_bounds__(256) void bn_bwd_apply_kernel(const float* __restrict__ g,
                                                           const float* __restrict__ x,
                                                           const float* __restrict__ stat,
                                                           const float* __restrict__ ss,
                                                           const float* __restrict__ gamma,
                                                           const double* __restrict__ ws, float* __restrict__ dx,
                                                           float* __restrict__ Ggamma, float* __restrict__ Gbeta,
                                                           int C, int HW, int S, double count, int act,
                                                           int chunk) {
  __shared__ float coef[3];
  const int plane = blockIdx.x, c = plane % C;
  const float mean = stat[c], istd = stat[C + c], sc = ss[c], sf = ss[C + c];
  const int e0 = blockIdx.y * chunk, e1 = min(e0 + chunk, HW);
  const size_t base = (size_t)plane * HW;
  // the chunk's data (at most 4096 elements) is requested before the sums are finished
  float4 xpre[4], gpre[4];
  if (VEC && dx) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int e = e0 + 4 * threadIdx.x + 1024 * u;
      if (e < e1) {
        xpre[u] = *reinterpret_cast<const float4*>(x + base + e);
        gpre[u] = *reinterpret_cast<const float4*>(g + base + e);
      }
    }
  }
  if (threadIdx.x < 64) {
    double s1, s2;
    bn_add_partials(ws, c, S, s1, s2);
    if (threadIdx.x == 0) {
      coef[0] = gamma[c] * stat[C + c];
      coef[1] = (float)(s1 / count);
      coef[2] = (float)(s2 / count);
      if (plane < C && blockIdx.y == 0) {
        Gbeta[c] += (float)s1;
        Ggamma[c] += (float)s2;
      }
    }
  }
  __syncthreads();
  if (!dx) return;  // the input gradient is not wanted
  const float k = coef[0], m1 = coef[1], m2 = coef[2];
  if (VEC) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int e = e0 + 4 * threadIdx.x + 1024 * u;
      if (e < e1) {
        const float4 xv = xpre[u], gv = gpre[u];
        float4 o;
        o.x = k * (gv.x * act_slope_sw<SW>(xv.x * sc + sf, act) - m1 - (xv.x - mean) * istd * m2);
        o.y = k * (gv.y * act_slope_sw<SW>(xv.y * sc + sf, act) - m1 - (xv.y - mean) * istd * m2);
        o.z = k * (gv.z * act_slope_sw<SW>(xv.z * sc + sf, act) - m1 - (xv.z - mean) * istd * m2);
        o.w = k * (gv.w * act_slope_sw<SW>(xv.w * sc + sf, act) - m1 - (xv.w - mean) * istd * m2);
        *reinterpret_cast<float4*>(dx + base + e) = o;
      }
    }
    for (int e = e0 + 4 * threadIdx.x + 4096; e < e1; e += 1024) {  // longer chunks (not produced by the launcher)
      float4 xv = *reinterpret_cast<const float4*>(x + base + e);
      float4 gv = *reinterpret_cast<const float4*>(g + base + e);
      float4 o;
      o.x = k * (gv.x * act_slope_sw<SW>(xv.x * sc + sf, act) - m1 - (xv.x - mean) * istd * m2);
      o.y = k * (gv.y * act_slope_sw<SW>(xv.y * sc + sf, act) - m1 - (xv.y - mean) * istd * m2);
      o.z = k * (gv.z * act_slope_sw<SW>(xv.z * sc + sf, act) - m1 - (xv.z - mean) * istd * m2);
      o.w = k * (gv.w * act_slope_sw<SW>(xv.w * sc + sf, act) - m1 - (xv.w - mean) * istd * m2);
      *reinterpret_cast<float4*>(dx + base + e) = o;
    }
  } else {
    for (int e = e0 + threadIdx.x; e < e1; e += 256) {
      float xv = x[base + e];
      dx[base + e] = k * (g[base + e] * act_slope_sw<SW>(xv * sc + sf, act) - m1 - (xv - mean) * istd * m2);
    }
  }
}

// ---------------------------------------------------------------- small tensors: one pass
// A channel with at most 8192 elements (N*HW) is handled by ONE block that keeps the channel in
// registers (eight values per thread): statistics and normalisation, or backward sums and input
// gradient, in a single launch instead of two, each reading its inputs once.  Element k of thread
// t is flat index t + k*T of the channel's N planes.
template <int T>
__device__ __forceinline__ void block_sum2_t(float f1, float f2, double* sh, double& d1, double& d2) {
  constexpr int NW = T / 64;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const double a = wave_sum_d((double)f1), b = wave_sum_d((double)f2);
  if (lane == 0) {
    sh[w] = a;
    sh[NW + w] = b;
  }
  __syncthreads();
  d1 = 0.0;
  d2 = 0.0;
#pragma unroll
  for (int k = 0; k < NW; ++k) {  // fixed order, the same in every thread
    d1 += sh[k];
    d2 += sh[NW + k];
  }
}

template <int T>
__global__ __launch_bounds__(T) void bn_fwd_onepass_kernel(const float* __restrict__ x,
                                                           const float* __restrict__ gamma,
                                                           const float* __restrict__ beta,
                                                           const float* __restrict__ skip, float* __restrict__ y,
                                                           float* __restrict__ stat, float* __restrict__ ss,
                                                           float* __restrict__ running, int N, int C, int HW,
                                                           float eps, int act) {
  __shared__ double sh[2 * (T / 64)];
  const int c = blockIdx.x, E = N * HW;
  float v[8], kv[8];
  size_t off[8];
  float s1 = 0.f, s2 = 0.f;
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const int idx = threadIdx.x + k * T;
    v[k] = 0.f;
    kv[k] = 0.f;
    off[k] = 0;
    if (idx < E) {
      const int n = idx / HW, e = idx - n * HW;
      off[k] = ((size_t)n * C + c) * HW + e;
      v[k] = x[off[k]];
      if (skip) kv[k] = skip[off[k]];
    }
  }
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    s1 += v[k];
    s2 += v[k] * v[k];
  }
  double d1, d2;
  block_sum2_t<T>(s1, s2, sh, d1, d2);
  float sc, sf;  // every thread computes the same coefficients; thread 0 records them
  bn_coefficients(d1, d2, (double)E, gamma[c], beta[c], eps, c, C, threadIdx.x == 0, stat, ss, running, sc, sf);
#pragma unroll
  for (int k = 0; k < 8; ++k)
    if (threadIdx.x + k * T < E) y[off[k]] = apply_act(v[k] * sc + sf, act) + kv[k];
}

template <int T>
__global__ __launch_bounds__(T) void bn_bwd_onepass_kernel(const float* __restrict__ g,
                                                           const float* __restrict__ x,
                                                           const float* __restrict__ stat,
                                                           const float* __restrict__ ss,
                                                           const float* __restrict__ gamma, float* __restrict__ dx,
                                                           float* __restrict__ Ggamma, float* __restrict__ Gbeta,
                                                           int N, int C, int HW, int act) {
  __shared__ double sh[2 * (T / 64)];
  const int c = blockIdx.x, E = N * HW;
  const float mean = stat[c], istd = stat[C + c], sc = ss[c], sf = ss[C + c];
  float gm[8], xh[8];  // masked upstream gradient, normalised input
  size_t off[8];
  float s1 = 0.f, s2 = 0.f;
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const int idx = threadIdx.x + k * T;
    gm[k] = 0.f;
    xh[k] = 0.f;
    off[k] = 0;
    if (idx < E) {
      const int n = idx / HW, e = idx - n * HW;
      off[k] = ((size_t)n * C + c) * HW + e;
      const float xv = x[off[k]];
      gm[k] = g[off[k]] * act_mask(xv * sc + sf, act);
      xh[k] = (xv - mean) * istd;
    }
  }
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    s1 += gm[k];
    s2 += gm[k] * xh[k];
  }
  double d1, d2;
  block_sum2_t<T>(s1, s2, sh, d1, d2);
  if (threadIdx.x == 0) {
    Gbeta[c] += (float)d1;
    Ggamma[c] += (float)d2;
  }
  if (!dx) return;  // the input gradient is not wanted
  const float kk = gamma[c] * istd, m1 = (float)(d1 / (double)E), m2 = (float)(d2 / (double)E);
#pragma unroll
  for (int k = 0; k < 8; ++k)
    if (threadIdx.x + k * T < E) dx[off[k]] = kk * (gm[k] - m1 - xh[k] * m2);
}

bool bn_onepass_fits(int N, int HW) { return (long)N * HW <= 8192; }

void bn_fwd_onepass_f32(hipStream_t st, const float* x, const float* gamma, const float* beta, const float* skip,
                        float* y, float* stat, float* scale_shift, float* running, int N, int C, int HW, float eps,
                        int act) {
  if ((long)N * HW <= 2048)
    KLAUNCH_NAMED("bn_fwd_onepass_kernel", (bn_fwd_onepass_kernel<256>), dim3(C), dim3(256), 0, st, x, gamma, beta,
                  skip, y, stat, scale_shift, running, N, C, HW, eps, act);
  else
    KLAUNCH_NAMED("bn_fwd_onepass_kernel", (bn_fwd_onepass_kernel<1024>), dim3(C), dim3(1024), 0, st, x, gamma, beta,
                  skip, y, stat, scale_shift, running, N, C, HW, eps, act);
}

void bn_bwd_onepass_f32(hipStream_t st, const float* g, const float* x, const float* stat, const float* ss,
                        const float* gamma, float* dx, float* Ggamma, float* Gbeta, int N, int C, int HW, int act) {
  if ((long)N * HW <= 2048)
    KLAUNCH_NAMED("bn_bwd_onepass_kernel", (bn_bwd_onepass_kernel<256>), dim3(C), dim3(256), 0, st, g, x, stat, ss,
                  gamma, dx, Ggamma, Gbeta, N, C, HW, act);
  else
    KLAUNCH_NAMED("bn_bwd_onepass_kernel", (bn_bwd_onepass_kernel<1024>), dim3(C), dim3(1024), 0, st, g, x, stat, ss,
                  gamma, dx, Ggamma, Gbeta, N, C, HW, act);
}

void bn_bwd_partial_f32(hipStream_t st, const float* g, const float* x, const float* stat, const float* ss,
                        double* ws, int N, int C, int HW, int act) {
  const BnSplit b = bn_split(N, HW);
#define BN_BWDP(name, kern) KLAUNCH_NAMED(name, kern, dim3(C, b.P), dim3(256), 0, st, g, x, stat, ss, ws, N, C, HW, b, act)
  const bool sw = act == ACT_SWISH;
  if (HW % 4 == 0) {
    if (sw) BN_BWDP("bn_bwd_partial_kernel<true>", (bn_bwd_partial_kernel<true, true>));
    else BN_BWDP("bn_bwd_partial_kernel<true>", (bn_bwd_partial_kernel<true, false>));
  } else {
    if (sw) BN_BWDP("bn_bwd_partial_kernel<false>", (bn_bwd_partial_kernel<false, true>));
    else BN_BWDP("bn_bwd_partial_kernel<false>", (bn_bwd_partial_kernel<false, false>));
  }
#undef BN_BWDP
}

void bn_bwd_apply_f32(hipStream_t st, const float* g, const float* x, const float* stat, const float* ss,
                      const float* gamma, const double* ws, int P, float* dx, float* Ggamma, float* Gbeta, int N,
                      int C, int HW, int act) {
  size_t per = (size_t)N * HW;
  int nchunks, chunk;
  bn_chunking(HW, nchunks, chunk);
  // without an input gradient only the sample-0 / chunk-0 blocks have work (dgamma, dbeta)
  dim3 grid(dx ? (unsigned)(N * C) : (unsigned)C, dx ? nchunks : 1);
#define BN_BWDA(name, kern)                                                                                        \
  KLAUNCH_NAMED(name, kern, grid, dim3(256), 0, st, g, x, stat, ss, gamma, ws, dx, Ggamma, Gbeta, C, HW, P, (double)per, \
                act, chunk)
  const bool sw = act == ACT_SWISH;
  if (HW % 4 == 0) {
    if (sw) BN_BWDA("bn_bwd_apply_kernel<true>", (bn_bwd_apply_kernel<true, true>));
    else BN_BWDA("bn_bwd_apply_kernel<true>", (bn_bwd_apply_kernel<true, false>));
  } else {
    if (sw) BN_BWDA("bn_bwd_apply_kernel<false>", (bn_bwd_apply_kernel<false, true>));
    else BN_BWDA("bn_bwd_apply_kernel<false>", (bn_bwd_apply_kernel<false, false>));
  }
#undef BN_BWDA
}

void bn_bwd_f32(hipStream_t st, const float* g, const float* x, const float* stat, const float* ss,
                const float* gamma, float* dx, float* Ggamma, float* Gbeta, double* ws, int N, int C, int HW,
                int act) {
  bn_bwd_partial_f32(st, g, x, stat, ss, ws, N, C, HW, act);
  bn_bwd_apply_f32(st, g, x, stat, ss, gamma, ws, bn_parts(N, HW), dx, Ggamma, Gbeta, N, C, HW, act);
}

}  // namespace ast
