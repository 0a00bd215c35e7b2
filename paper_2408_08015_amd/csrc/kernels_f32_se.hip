// Squeeze-and-excitation gate of the EfficientNet blocks (Table 4 workload) in one launch per
// direction: pooled vector p[B][C] -> h_pre = W1 p + b1 -> h = swish(h_pre) -> z = W2 h + b2 ->
// gate = sigmoid(z), with C a few hundred and Cr = C/24 or so.  The layer-by-layer path spends six
// launches of 4-13 us on these few kFLOP per sample; here a block owns a sample.  Every
// intermediate is still written to its place in the stash (the backward reads them).
//
// Backward, launch A (block per sample): dz = dgate * sigmoid'(z); dh = W2^T dz;
// dh_pre = dh * swish'(h_pre); dp = W1^T dh_pre.  dz and dh_pre stay in the gradient buffers of z and
// h_pre.  Launch B (thread per parameter): the sums over the samples, in order, into G.
#include "device_utils.h"
#include "kernels.h"
#include "prof.h"

namespace ast {

namespace {

inline int cdiv(long a, long b) { return (int)((a + b - 1) / b); }

// dot product of a row with the LDS vector over the lanes of a wavefront, four loads in flight
__device__ __forceinline__ float wave_dot(const float* __restrict__ row, const float* __restrict__ sv, int C, int lane) {
  float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
  int c = lane;
  for (; c + 192 < C; c += 256) {
    const float w0 = row[c], w1 = row[c + 64], w2 = row[c + 128], w3 = row[c + 192];
    a0 += w0 * sv[c]; a1 += w1 * sv[c + 64]; a2 += w2 * sv[c + 128]; a3 += w3 * sv[c + 192];
  }
  for (; c < C; c += 64) a0 += row[c] * sv[c];
  return wave_sum((a0 + a1) + (a2 + a3));
}

// sum_r w[r * stride] * sv[r], r < n, eight loads in flight
__device__ __forceinline__ float strided_dot(const float* __restrict__ w, size_t stride, const float* __restrict__ sv, int n) {
  float a = 0.f;
  for (int r0 = 0; r0 < n; r0 += 8) {
    float v[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] = r0 + k < n ? w[(size_t)(r0 + k) * stride] : 0.f;
#pragma unroll
    for (int k = 0; k < 8; ++k) a += v[k] * (r0 + k < n ? sv[r0 + k] : 0.f);
  }
  return a;
}

// Block = one sample, 1024 threads (16 wavefronts: the hidden units are dealt over them).  LDS: p[C] then h[Cr]
__global__ __launch_bounds__(1024) void se_gate_fwd_kernel(const float* __restrict__ p, const float* __restrict__ W1,
                                                           const float* __restrict__ b1, const float* __restrict__ W2,
                                                           const float* __restrict__ b2, float* __restrict__ hpre,
                                                           float* __restrict__ h, float* __restrict__ z,
                                                           float* __restrict__ gate, int C, int Cr) {
  extern __shared__ float sh[];
  float* sp = sh;
  float* shh = sh + C;
  const int n = blockIdx.x, lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  for (int c = threadIdx.x; c < C; c += 1024) sp[c] = p[(size_t)n * C + c];
  __syncthreads();
  for (int r = wv; r < Cr; r += 16) {  // a wavefront per hidden unit
    const float a = wave_dot(W1 + (size_t)r * C, sp, C, lane) + (b1 ? b1[r] : 0.f);
    if (lane == 0) {
      hpre[(size_t)n * Cr + r] = a;
      const float hv = a * sigmoid_f(a);
      h[(size_t)n * Cr + r] = hv;
      shh[r] = hv;
    }
  }
  __syncthreads();
  for (int c = threadIdx.x; c < C; c += 1024) {
    float a = b2 ? b2[c] : 0.f;
    const float* wr = W2 + (size_t)c * Cr;  // (a plain loop: eight explicit loads in flight measured slower here)
    for (int r = 0; r < Cr; ++r) a += wr[r] * shh[r];
    z[(size_t)n * C + c] = a;
    gate[(size_t)n * C + c] = sigmoid_f(a);
  }
}

// LDS: dz[C], dhp[Cr], then per-wavefront partial sums [16][Cr]
__global__ __launch_bounds__(1024) void se_gate_bwd_kernel(const float* __restrict__ dgate, const float* __restrict__ z,
                                                           const float* __restrict__ hpre, const float* __restrict__ W1,
                                                           const float* __restrict__ W2, float* __restrict__ dz,
                                                           float* __restrict__ dhp, float* __restrict__ dp, int C, int Cr) {
  extern __shared__ float sh[];
  float* sdz = sh;
  float* sdh = sh + C;
  float* spart = sdh + Cr;  // [16][Cr]
  const int n = blockIdx.x, lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  for (int c = threadIdx.x; c < C; c += 1024) {
    const float s = sigmoid_f(z[(size_t)n * C + c]);
    const float v = dgate[(size_t)n * C + c] * s * (1.f - s);
    sdz[c] = v;
    dz[(size_t)n * C + c] = v;
  }
  __syncthreads();
  // dh[r] = sum_c W2[c][r] dz[c]: a lane owns channel c and walks its row of W2 (consecutive r: the row stays in
  // cache), the wavefront adds the 64 products of each r; wavefronts take the channel groups in turn and their
  // sums meet in LDS in a fixed order
  for (int r = 0; r < Cr; ++r) {
    float a = 0.f;
    for (int c = wv * 64 + lane; c < C; c += 1024) a += W2[(size_t)c * Cr + r] * sdz[c];
    a = wave_sum(a);
    if (lane == 0) spart[wv * Cr + r] = a;
  }
  __syncthreads();
  for (int r = threadIdx.x; r < Cr; r += 1024) {
    float a = 0.f;
    for (int k = 0; k < 16; ++k) a += spart[k * Cr + r];
    const float v = a * act_slope_sw<true>(hpre[(size_t)n * Cr + r], ACT_SWISH);
    sdh[r] = v;
    dhp[(size_t)n * Cr + r] = v;
  }
  __syncthreads();
  if (dp)
    for (int c = threadIdx.x; c < C; c += 1024) dp[(size_t)n * C + c] = strided_dot(W1 + c, (size_t)C, sdh, Cr);
}

// sum over the samples of a[n*sa + ia] * b[n*sb + ib] (b == NULL: of a alone), eight loads in flight
__device__ __forceinline__ float sample_dot(const float* __restrict__ a, size_t sa, size_t ia, const float* __restrict__ b,
                                            size_t sb, size_t ib, int N) {
  float acc = 0.f;
  for (int n0 = 0; n0 < N; n0 += 8) {
    float av[8], bv[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const bool ok = n0 + k < N;
      av[k] = ok ? a[(size_t)(n0 + k) * sa + ia] : 0.f;
      bv[k] = (ok && b) ? b[(size_t)(n0 + k) * sb + ib] : 1.f;
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) acc += av[k] * bv[k];
  }
  return acc;
}

// parameters in the order [W1: Cr*C][b1: Cr][W2: C*Cr][b2: C]; G* may be NULL for an absent bias
__global__ void se_gate_wgrad_kernel(const float* __restrict__ dz, const float* __restrict__ dhp,
                                     const float* __restrict__ p, const float* __restrict__ h, float* __restrict__ GW1,
                                     float* __restrict__ Gb1, float* __restrict__ GW2, float* __restrict__ Gb2, int N, int C,
                                     int Cr) {
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  const int nW = C * Cr;
  if (idx < nW) {  // W1[r][c]
    const int r = idx / C, c = idx - r * C;
    GW1[idx] += sample_dot(dhp, Cr, r, p, C, c, N);
    return;
  }
  idx -= nW;
  if (idx < Cr) {
    if (Gb1) Gb1[idx] += sample_dot(dhp, Cr, idx, nullptr, 0, 0, N);
    return;
  }
  idx -= Cr;
  if (idx < nW) {  // W2[c][r]
    const int c = idx / Cr, r = idx - c * Cr;
    GW2[idx] += sample_dot(dz, C, c, h, Cr, r, N);
    return;
  }
  idx -= nW;
  if (idx < C && Gb2) Gb2[idx] += sample_dot(dz, C, idx, nullptr, 0, 0, N);
}

}  // namespace

bool se_gate_supported(int C, int Cr) { return C >= 1 && Cr >= 1 && (size_t)(C + 17 * Cr) * sizeof(float) <= 48 * 1024; }

void se_gate_fwd_f32(hipStream_t st, const float* p, const float* W1, const float* b1, const float* W2, const float* b2,
                     float* hpre, float* h, float* z, float* gate, int N, int C, int Cr) {
  KLAUNCH(se_gate_fwd_kernel, dim3(N), dim3(1024), (size_t)(C + Cr) * sizeof(float), st, p, W1, b1, W2, b2, hpre, h, z, gate,
          C, Cr);
}

void se_gate_bwd_f32(hipStream_t st, const float* dgate, const float* z, const float* hpre, const float* p, const float* h,
                     const float* W1, const float* W2, float* dz, float* dhp, float* dp, float* GW1, float* Gb1, float* GW2,
                     float* Gb2, int N, int C, int Cr) {
  KLAUNCH(se_gate_bwd_kernel, dim3(N), dim3(1024), (size_t)(C + 17 * Cr) * sizeof(float), st, dgate, z, hpre, W1, W2, dz, dhp,
          dp, C, Cr);
  KLAUNCH(se_gate_wgrad_kernel, dim3(cdiv(2L * C * Cr + C + Cr, 256)), dim3(256), 0, st, dz, dhp, p, h, GW1, Gb1, GW2, Gb2, N,
          C, Cr);
}

}  // namespace ast
