// BatchNorm pieces shared by the BatchNorm kernels and by kernels that normalise on load:
// finishing the statistics of a channel from its partial sums, and the resulting affine
// coefficients y = x*scale + shift.
#pragma once
#include "device_utils.h"

namespace ast {

// sums of the channel's P partial pairs ws[c][P][2] in a fixed order, identical in every lane
// of the calling wavefront
__device__ __forceinline__ void bn_add_partials(const double* __restrict__ ws, int c, int P, double& s1, double& s2) {
  const int lane = threadIdx.x & 63;
  double a = 0.0, b = 0.0;
  for (int k = lane; k < P; k += 64) {
    a += ws[((size_t)c * P + k) * 2 + 0];
    b += ws[((size_t)c * P + k) * 2 + 1];
  }
  s1 = wave_sum_d(a);
  s2 = wave_sum_d(b);
}

// Training-mode statistics of channel c from (sum, sum of squares) over `count` elements:
// scale = gamma/sqrt(var + eps), shift = beta - mean*scale.  With `record` the statistics are
// also stored (mean, 1/std -> stat[c], stat[C + c]; scale, shift -> ss[c], ss[C + c]) and the
// running statistics updated (momentum 0.1, unbiased variance).  Every caller of one channel
// computes bit-identical coefficients.
__device__ __forceinline__ void bn_coefficients(double s1, double s2, double count, float gamma, float beta, float eps,
                                                int c, int C, bool record, float* __restrict__ stat,
                                                float* __restrict__ ss, float* __restrict__ running, float& scale,
                                                float& shift) {
  const double mean = s1 / count;
  double var = s2 / count - mean * mean;
  if (var < 0) var = 0;
  const double istd = 1.0 / sqrt(var + (double)eps);
  const double sc = (double)gamma * istd;
  scale = (float)sc;
  shift = (float)((double)beta - mean * sc);
  if (record) {
    stat[c] = (float)mean;
    stat[C + c] = (float)istd;
    ss[c] = scale;
    ss[C + c] = shift;
    if (running) {
      const double unb = count > 1 ? var * count / (count - 1) : var;
      running[c] += 0.1f * ((float)mean - running[c]);
      running[C + c] += 0.1f * ((float)unb - running[C + c]);
    }
  }
}

}  // namespace ast
