// Device-side helpers shared by the gfx950 kernels: wavefront (64-lane) reductions,
// bf16 conversion, MFMA vector types.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ast {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned short bf16_t;  // storage type of one bf16 value

constexpr int kWave = 64;

// Lane exchanges inside the VALU (data-parallel primitives) instead of through the LDS crossbar
// (ds_bpermute, which __shfl_* compile to: an LDS instruction and its latency per exchange).
// dpp_move<CTRL>(v) = v of the lane that control CTRL pairs this lane with, 0 where there is none.
constexpr int DPP_QUAD_SWAP1 = 0xB1;    // quad_perm [1,0,3,2]: lane ^ 1
constexpr int DPP_QUAD_SWAP2 = 0x4E;    // quad_perm [2,3,0,1]: lane ^ 2
constexpr int DPP_HALF_MIRROR = 0x141;  // lane i of a group of 8 <- lane 7 - i (the other quad)
constexpr int DPP_ROW_MIRROR = 0x140;   // lane i of a row of 16 <- lane 15 - i (the other half row)
constexpr int DPP_WAVE_SHR1 = 0x138;    // lane i <- lane i - 1 over the whole wavefront
constexpr int DPP_WAVE_SHL1 = 0x130;    // lane i <- lane i + 1
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
template <int CTRL>
__device__ __forceinline__ double dpp_move(double v) {
  const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, 0xF, 0xF, true);
  const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, 0xF, 0xF, true);
  return __hiloint2double(hi, lo);
}
// v of lane - 1 / lane + 1 (0 at the ends of the wavefront)
__device__ __forceinline__ float lane_up1(float v) { return dpp_move<DPP_WAVE_SHR1>(v); }
__device__ __forceinline__ float lane_down1(float v) { return dpp_move<DPP_WAVE_SHL1>(v); }
// sum over the 2, 4, 8, 16 lanes of the aligned group of this lane, valid in each of its lanes (the
// partner of every step lies in the other half of the group, so all lanes add the same pairs)
template <typename T> __device__ __forceinline__ T group4_sum(T v) {
  v += dpp_move<DPP_QUAD_SWAP1>(v);
  v += dpp_move<DPP_QUAD_SWAP2>(v);
  return v;
}
template <typename T> __device__ __forceinline__ T group8_sum(T v) {
  v = group4_sum(v);
  v += dpp_move<DPP_HALF_MIRROR>(v);
  return v;
}
template <typename T> __device__ __forceinline__ T row16_sum(T v) {
  v = group8_sum(v);
  v += dpp_move<DPP_ROW_MIRROR>(v);
  return v;
}
// Sums over the wavefront, valid in every lane: four steps inside the rows of 16, the two steps
// across rows through the LDS crossbar (an inactive lane contributes 0 in both).
__device__ __forceinline__ float wave_sum(float v) {
  v = row16_sum(v);
  v += __shfl_xor(v, 16, 64);
  v += __shfl_xor(v, 32, 64);
  return v;
}
__device__ __forceinline__ double wave_sum_d(double v) {
  v = row16_sum(v);
  v += __shfl_xor(v, 16, 64);
  v += __shfl_xor(v, 32, 64);
  return v;
}
// maximum over the wavefront; all 64 lanes must be active
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_move<DPP_QUAD_SWAP1>(v));
  v = fmaxf(v, dpp_move<DPP_QUAD_SWAP2>(v));
  v = fmaxf(v, dpp_move<DPP_HALF_MIRROR>(v));
  v = fmaxf(v, dpp_move<DPP_ROW_MIRROR>(v));
  v = fmaxf(v, __shfl_xor(v, 16, 64));
  v = fmaxf(v, __shfl_xor(v, 32, 64));
  return v;
}

// Block-wide sum for blocks of up to 1024 threads; result valid in every thread.
// `sh` must hold at least 16 entries.
template <typename T>
__device__ __forceinline__ T block_sum(T v, T* sh) {
  int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  v = row16_sum(v);
  v += __shfl_xor(v, 16, 64);
  v += __shfl_xor(v, 32, 64);
  __syncthreads();
  if (lane == 0) sh[w] = v;
  __syncthreads();
  T r = 0;
  for (int i = 0; i < nw; ++i) r += sh[i];
  return r;
}

// bf16 <-> fp32, round to nearest even (NaN kept quiet).
__device__ __forceinline__ bf16_t f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
__device__ __forceinline__ float bf2f(bf16_t h) { return __uint_as_float(((uint32_t)h) << 16); }
// two values at once with the hardware conversion (v_cvt_pk_bf16_f32, round to nearest even: the same
// result as f2bf for every finite value); a in the low half
__device__ __forceinline__ uint32_t f2bf_pk(float a, float b) {
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  typedef float float2_t __attribute__((ext_vector_type(2)));
  const float2_t f = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));
}

// Phi(x) of the standard normal distribution, and E = exp(-x^2 / 2), in about a dozen operations:
// erfc(z) = (a1 t + ... + a5 t^5) exp(-z^2) with t = 1 / (1 + p z), z = |x| / sqrt(2) (Abramowitz &
// Stegun 7.1.26, |error| <= 1.5e-7; measured in fp32: |Phi error| < 3e-7, x Phi(x) within 6e-7
// relative for x > 0).  The negative side is the complementary value itself, so it keeps its relative
// accuracy where 1 + erf would cancel.  The exact GELU is x Phi(x), its derivative Phi(x) + x phi(x).
__device__ __forceinline__ float norm_cdf(float x, float& E) {
  const float z = fabsf(x) * 0.70710678f;
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, z, 1.f));
  E = __builtin_amdgcn_exp2f(x * x * -0.72134752f);
  float p = fmaf(1.061405429f, t, -1.453152027f);
  p = fmaf(p, t, 1.421413741f);
  p = fmaf(p, t, -0.284496736f);
  p = fmaf(p, t, 0.254829592f);
  const float h = 0.5f * (p * t) * E;
  return x >= 0.f ? 1.f - h : h;
}
__device__ __forceinline__ float gelu_fast(float x) {
  float E;
  return x * norm_cdf(x, E);
}
__device__ __forceinline__ float gelu_grad_fast(float x) {
  float E;
  const float c = norm_cdf(x, E);
  return fmaf(x * 0.3989422804f, E, c);
}

// Workgroups are dealt to the 8 XCDs (each with an L2 of its own) round-robin by their flat index.
// Renumbering: XCD x gets the contiguous range of ids that starts at x*(n/8) + min(x, n%8), so
// blocks with neighbouring renumbered ids run on the same XCD at about the same time.  A bijection
// on [0, n).
__device__ __forceinline__ unsigned xcd_grouped(unsigned id, unsigned n) {
  const unsigned q = n >> 3, r = n & 7, x = id & 7;
  return x * q + min(x, r) + (id >> 3);
}

__device__ __forceinline__ float relu6f(float v) { return fminf(fmaxf(v, 0.f), 6.f); }

// activation codes used by fused kernels
enum : int { ACT_NONE = 0, ACT_RELU = 1, ACT_RELU6 = 2, ACT_GELU = 3, ACT_SWISH = 4, ACT_SIGMOID = 5 };

// hardware exponential and reciprocal (a few ulp; the fp32 parity bars are 1e-4): the swish
// kernels are bound by this arithmetic, not by memory
__device__ __forceinline__ float sigmoid_f(float v) { return __frcp_rn(1.f + __expf(-v)); }
// ReLU / ReLU6, the activations every fused kernel knows (`act` is uniform over a launch)
__device__ __forceinline__ float apply_act(float v, int act) {
  if (act == ACT_RELU) return fmaxf(v, 0.f);
  if (act == ACT_RELU6) return relu6f(v);
  return v;
}
// derivative mask of the activation evaluated at pre-activation v (0 at the kinks); the activated
// value gives the same answer
__device__ __forceinline__ float act_mask(float v, int act) {
  if (act == ACT_RELU) return v > 0.f ? 1.f : 0.f;
  if (act == ACT_RELU6) return (v > 0.f && v < 6.f) ? 1.f : 0.f;
  return 1.f;
}
// ... and the variants of the kernels that also fuse swish (instantiated apart, so that the ReLU
// kernels carry no exponential): value and derivative at pre-activation v
template <bool SW>
__device__ __forceinline__ float apply_act_sw(float v, int act) {
  if (SW) return v * sigmoid_f(v);
  return apply_act(v, act);
}
template <bool SW>
__device__ __forceinline__ float act_slope_sw(float v, int act) {
  if (SW) {
    const float s = sigmoid_f(v);
    return s + v * s * (1.f - s);
  }
  return act_mask(v, act);
}

}  // namespace ast
