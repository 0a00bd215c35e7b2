// BatchNorm2d (training mode, NCHW, fp32) forward and backward, HBM-bound.
//
// Each direction is two streaming kernels and nothing else:
//   partial:  (channel, split) blocks reduce a share of the channel's N*H*W elements
//             (fp32 per thread, fp64 across threads) into ws[channel][split][2];
//   apply:    one block per (plane, chunk); its first wavefront adds the channel's partials
//             in a fixed butterfly order in fp64 (every block of a channel computes bit-identical
//             coefficients), then the block streams its chunk.  The block of sample 0 /
//             chunk 0 also records the channel's statistics, or accumulates dgamma / dbeta
//             into G.
// Doing the tiny "finish the reduction" step inside the consumer removes two
// latency-bound launches per BatchNorm per micro-batch.
#include "device_utils.h"
#include "kernels.h"
#include "prof.h"

namespace ast {

static inline int cdiv(long a, long b) { return (int)((a + b - 1) / b); }

static inline int bn_split(int C, size_t per) {
  int S = cdiv(2048, C);
  int maxS = (int)((per + 4095) / 4096);
  if (S > maxS) S = maxS;
  if (S > 64) S = 64;  // one wavefront adds the partials
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

// sums of the channel's partial pairs, identical in every lane of the calling wavefront
__device__ __forceinline__ void add_partials(const double* __restrict__ ws, int c, int S, double& s1, double& s2) {
  const int lane = threadIdx.x & 63;
  double a = 0.0, b = 0.0;
  if (lane < S) {
    a = ws[((size_t)c * S + lane) * 2 + 0];
    b = ws[((size_t)c * S + lane) * 2 + 1];
  }
  s1 = wave_sum_d(a);
  s2 = wave_sum_d(b);
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

// y = act(x*scale + shift) (+ skip); grid (planes, chunks)
template <bool VEC>
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
  if (threadIdx.x < 64) {
    double s1, s2;
    add_partials(ws, c, S, s1, s2);
    if (threadIdx.x == 0) {
      double mean = s1 / count;
      double var = s2 / count - mean * mean;
      if (var < 0) var = 0;
      double istd = 1.0 / sqrt(var + (double)eps);
      double sc = (double)gamma[c] * istd;
      float scf = (float)sc, sff = (float)((double)beta[c] - mean * sc);
      coef[0] = scf;
      coef[1] = sff;
      if (plane < C && blockIdx.y == 0) {  // sample 0, chunk 0: record the channel's statistics
        stat[c] = (float)mean;
        stat[C + c] = (float)istd;
        ss[c] = scf;
        ss[C + c] = sff;
        if (running) {
          double unb = count > 1 ? var * count / (count - 1) : var;
          running[c] += 0.1f * ((float)mean - running[c]);
          running[C + c] += 0.1f * ((float)unb - running[C + c]);
        }
      }
    }
  }
  __syncthreads();
  const float sc = coef[0], sf = coef[1];
  const int e0 = blockIdx.y * chunk, e1 = min(e0 + chunk, HW);
  const size_t base = (size_t)plane * HW;
  if (VEC) {
    for (int e = e0 + 4 * threadIdx.x; e < e1; e += 1024) {
      float4 v = *reinterpret_cast<const float4*>(x + base + e);
      v.x = apply_act(v.x * sc + sf, act);
      v.y = apply_act(v.y * sc + sf, act);
      v.z = apply_act(v.z * sc + sf, act);
      v.w = apply_act(v.w * sc + sf, act);
      if (skip) {
        float4 k = *reinterpret_cast<const float4*>(skip + base + e);
        v.x += k.x; v.y += k.y; v.z += k.z; v.w += k.w;
      }
      *reinterpret_cast<float4*>(y + base + e) = v;
    }
  } else {
    for (int e = e0 + threadIdx.x; e < e1; e += 256) {
      float v = apply_act(x[base + e] * sc + sf, act);
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

void bn_fwd_f32(hipStream_t st, const float* x, const float* gamma, const float* beta, const float* skip,
                float* y, float* stat, float* scale_shift, float* running, double* ws, int N, int C, int HW,
                float eps, int act) {
  size_t per = (size_t)N * HW;
  int S = bn_split(C, per);
  const bool vec = HW % 4 == 0;
  if (vec) KLAUNCH(bn_stats_partial_kernel<true>, dim3(C, S), dim3(256), 0, st, x, ws, N, C, HW, S);
  else KLAUNCH(bn_stats_partial_kernel<false>, dim3(C, S), dim3(256), 0, st, x, ws, N, C, HW, S);
  int nchunks, chunk;
  bn_chunking(HW, nchunks, chunk);
  dim3 grid((unsigned)(N * C), nchunks);
  if (vec)
    KLAUNCH(bn_apply_kernel<true>, grid, dim3(256), 0, st, x, ws, gamma, beta, skip, y, stat, scale_shift, running, C,
            HW, S, (double)per, eps, act, chunk);
  else
    KLAUNCH(bn_apply_kernel<false>, grid, dim3(256), 0, st, x, ws, gamma, beta, skip, y, stat, scale_shift, running,
            C, HW, S, (double)per, eps, act, chunk);
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

// dx = gamma*istd*(g' - mean(g') - xhat*mean(g'*xhat)); sample 0 / chunk 0 blocks add dgamma, dbeta to G
template <bool VEC>
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
  if (threadIdx.x < 64) {
    double s1, s2;
    add_partials(ws, c, S, s1, s2);
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
  const float mean = stat[c], istd = stat[C + c], sc = ss[c], sf = ss[C + c];
  const int e0 = blockIdx.y * chunk, e1 = min(e0 + chunk, HW);
  const size_t base = (size_t)plane * HW;
  if (VEC) {
    for (int e = e0 + 4 * threadIdx.x; e < e1; e += 1024) {
      float4 xv = *reinterpret_cast<const float4*>(x + base + e);
      float4 gv = *reinterpret_cast<const float4*>(g + base + e);
      float4 o;
      o.x = k * (gv.x * act_mask(xv.x * sc + sf, act) - m1 - (xv.x - mean) * istd * m2);
      o.y = k * (gv.y * act_mask(xv.y * sc + sf, act) - m1 - (xv.y - mean) * istd * m2);
      o.z = k * (gv.z * act_mask(xv.z * sc + sf, act) - m1 - (xv.z - mean) * istd * m2);
      o.w = k * (gv.w * act_mask(xv.w * sc + sf, act) - m1 - (xv.w - mean) * istd * m2);
      *reinterpret_cast<float4*>(dx + base + e) = o;
    }
  } else {
    for (int e = e0 + threadIdx.x; e < e1; e += 256) {
      float xv = x[base + e];
      dx[base + e] = k * (g[base + e] * act_mask(xv * sc + sf, act) - m1 - (xv - mean) * istd * m2);
    }
  }
}

void bn_bwd_f32(hipStream_t st, const float* g, const float* x, const float* stat, const float* ss,
                const float* gamma, float* dx, float* Ggamma, float* Gbeta, double* ws, int N, int C, int HW,
                int act) {
  size_t per = (size_t)N * HW;
  int S = bn_split(C, per);
  const bool vec = HW % 4 == 0;
  if (vec) KLAUNCH(bn_bwd_partial_kernel<true>, dim3(C, S), dim3(256), 0, st, g, x, stat, ss, ws, N, C, HW, S, act);
  else KLAUNCH(bn_bwd_partial_kernel<false>, dim3(C, S), dim3(256), 0, st, g, x, stat, ss, ws, N, C, HW, S, act);
  int nchunks, chunk;
  bn_chunking(HW, nchunks, chunk);
  // without an input gradient only the sample-0 / chunk-0 blocks have work (dgamma, dbeta)
  dim3 grid(dx ? (unsigned)(N * C) : (unsigned)C, dx ? nchunks : 1);
  if (vec)
    KLAUNCH(bn_bwd_apply_kernel<true>, grid, dim3(256), 0, st, g, x, stat, ss, gamma, ws, dx, Ggamma, Gbeta, C, HW, S,
            (double)per, act, chunk);
  else
    KLAUNCH(bn_bwd_apply_kernel<false>, grid, dim3(256), 0, st, g, x, stat, ss, gamma, ws, dx, Ggamma, Gbeta, C, HW,
            S, (double)per, act, chunk);
}

}  // namespace ast
