// Self-attention core (no mask, head size 64, S % 32 == 0, S <= 256) on packed
// qkv [B][S][3D]: forward with online softmax, and backward as two kernels
// (dK/dV parallel over keys, dQ parallel over queries).  The S x S score matrix never
// leaves the chip: bytes moved are Q, K, V, O (+ dO, dQ, dK, dV) only.
//
// Every product is computed in the orientation that keeps the softmax reductions inside
// a lane.  With MFMA 32x32x16 the accumulator of lane l holds column l%32 and 16 rows
// (register r -> row 8*(r/4) + 4*(l/32) + r%4).  The forward computes S^T = K Q^T, so a
// lane owns one query and its registers run over keys: the row max / row sum need one
// cross-half shuffle, and the probabilities are already laid out as the B operand of
// O^T = V^T P^T (slot (g, e) of MFMA u <-> key 16u + 8*(e/4) + 4g + e%4; the V^T operand is
// read from a transposed LDS copy with the same slot order).  The backward kernels use
// the same trick with the roles of queries and keys chosen per product.
#include "device_utils.h"
#include "kernels_bf16.h"
#include "prof.h"

namespace ast {

namespace {

constexpr int HD = 64;        // head size
constexpr int RS = HD + 8;    // LDS row stride of [row][d] copies (elements)

__device__ __forceinline__ bf16x8 ld_frag(const bf16_t* p) { return *reinterpret_cast<const bf16x8*>(p); }

__device__ __forceinline__ bf16x8 pack_frag(const float* f) {
  uint4 v;
  uint32_t* w = reinterpret_cast<uint32_t*>(&v);
#pragma unroll
  for (int k = 0; k < 4; ++k) w[k] = f2bf_pk(f[2 * k], f[2 * k + 1]);
  return __builtin_bit_cast(bf16x8, v);
}
// two 8-byte reads -> one operand fragment (slots e = 0..3 and 4..7)
__device__ __forceinline__ bf16x8 ld_frag_2x4(const bf16_t* p0, const bf16_t* p1) {
  uint4 v;
  uint2 a = *reinterpret_cast<const uint2*>(p0);
  uint2 b = *reinterpret_cast<const uint2*>(p1);
  v.x = a.x; v.y = a.y; v.z = b.x; v.w = b.y;
  return __builtin_bit_cast(bf16x8, v);
}

// Staging of two [S][64] tensors (row strides ld0 / ld1 elements in global memory) into LDS, each as a row copy
// [S][RS] (R0 / R1) and / or a transposed copy [64][S + 8] (T0 / T1), from ONE set of loads: a task is 4 rows x 8
// columns of both tensors, and its eight 16-byte loads are requested before the first LDS write (loops with one
// load, one wait and one write per trip made a block wait for a dozen memory round trips one after the other).
__device__ __forceinline__ void write_rows4(bf16_t* dst, const uint4 (&v)[4], int rq, int cg) {
#pragma unroll
  for (int r = 0; r < 4; ++r) *reinterpret_cast<uint4*>(dst + (rq * 4 + r) * RS + cg * 8) = v[r];
}
__device__ __forceinline__ void write_T4(bf16_t* dst, const uint4 (&v)[4], int rq, int cg, int TS) {
  const uint32_t* r0 = reinterpret_cast<const uint32_t*>(&v[0]);
  const uint32_t* r1 = reinterpret_cast<const uint32_t*>(&v[1]);
  const uint32_t* r2 = reinterpret_cast<const uint32_t*>(&v[2]);
  const uint32_t* r3 = reinterpret_cast<const uint32_t*>(&v[3]);
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    uint2 lo, hi;
    lo.x = (r0[w] & 0xffffu) | (r1[w] << 16);
    lo.y = (r2[w] & 0xffffu) | (r3[w] << 16);
    hi.x = (r0[w] >> 16) | (r1[w] & 0xffff0000u);
    hi.y = (r2[w] >> 16) | (r3[w] & 0xffff0000u);
    *reinterpret_cast<uint2*>(dst + (cg * 8 + 2 * w) * TS + rq * 4) = lo;
    *reinterpret_cast<uint2*>(dst + (cg * 8 + 2 * w + 1) * TS + rq * 4) = hi;
  }
}
template <bool R0, bool T0, bool R1, bool T1>
__device__ __forceinline__ void stage_pair(bf16_t* rows0, bf16_t* tr0, const bf16_t* src0, long ld0, bf16_t* rows1,
                                           bf16_t* tr1, const bf16_t* src1, long ld1, int S) {
  const int TS = S + 8;
  for (int t = threadIdx.x; t < (S / 4) * 8; t += blockDim.x) {
    const int rq = t >> 3, cg = t & 7;
    uint4 a[4], c[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      a[r] = *reinterpret_cast<const uint4*>(src0 + (long)(rq * 4 + r) * ld0 + cg * 8);
      c[r] = *reinterpret_cast<const uint4*>(src1 + (long)(rq * 4 + r) * ld1 + cg * 8);
    }
    if (R0) write_rows4(rows0, a, rq, cg);
    if (R1) write_rows4(rows1, c, rq, cg);
    if (T0) write_T4(tr0, a, rq, cg, TS);
    if (T1) write_T4(tr1, c, rq, cg, TS);
  }
}

// row index held by accumulator register r of a lane in half g
__device__ __forceinline__ int acc_row(int r, int g) { return 8 * (r >> 2) + 4 * g + (r & 3); }

// ------------------------------------------------------------------ forward
__global__ __launch_bounds__(256) void attention_fwd_kernel(const bf16_t* __restrict__ qkv,
                                                            bf16_t* __restrict__ o, float* __restrict__ lse,
                                                            int S, int D, int H) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16_t* sK = reinterpret_cast<bf16_t*>(smem);  // [S][RS]
  bf16_t* sVt = sK + S * RS;                     // [64][S+8]
  const int TS = S + 8;
  const int b = blockIdx.z, h = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 31, g = lane >> 5;
  const long ld = 3L * D;
  const bf16_t* base = qkv + (long)b * S * ld + h * HD;
  // everything this wavefront reads from global memory is requested before the staging copies wait for theirs
  const int q0 = blockIdx.x * 128 + wave * 32;
  const bool live = q0 < S;
  const int q = live ? q0 + col : 0;
  bf16x8 qf[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) qf[t] = ld_frag(base + (long)q * ld + 16 * t + 8 * g);
  stage_pair<true, false, false, true>(sK, nullptr, base + D, ld, nullptr, sVt, base + 2 * D, ld, S);
  __syncthreads();
  if (!live) return;

  floatx16 oacc[2];
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[dt][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float scale = 0.125f;  // 1/sqrt(64)

  for (int kt = 0; kt < S / 32; ++kt) {
    floatx16 s;
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
    for (int t = 0; t < 4; ++t)
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ld_frag(sK + (kt * 32 + col) * RS + 16 * t + 8 * g), qf[t], s, 0, 0, 0);
    float tmax = -INFINITY;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      s[r] *= scale;
      tmax = fmaxf(tmax, s[r]);
    }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
    const float m_new = fmaxf(m_run, tmax);
    const float alpha = __expf(m_run - m_new);
    float p[16], rs = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      p[r] = __expf(s[r] - m_new);
      rs += p[r];
    }
    rs += __shfl_xor(rs, 32, 64);
    l_run = l_run * alpha + rs;
    m_run = m_new;
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[dt][r] *= alpha;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      bf16x8 pf = pack_frag(p + 8 * u);
#pragma unroll
      for (int dt = 0; dt < 2; ++dt) {
        const bf16_t* vp = sVt + (dt * 32 + col) * TS + kt * 32 + 16 * u + 4 * g;
        oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ld_frag_2x4(vp, vp + 8), pf, oacc[dt], 0, 0, 0);
      }
    }
  }
  const float inv = 1.f / l_run;
  bf16_t* orow = o + ((long)b * S + q) * D + h * HD;
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      uint2 v;
      v.x = f2bf_pk(oacc[dt][4 * r4] * inv, oacc[dt][4 * r4 + 1] * inv);
      v.y = f2bf_pk(oacc[dt][4 * r4 + 2] * inv, oacc[dt][4 * r4 + 3] * inv);
      *reinterpret_cast<uint2*>(orow + dt * 32 + 8 * r4 + 4 * g) = v;
    }
  if (g == 0) lse[((long)b * H + h) * S + q] = m_run + __logf(l_run);
}

// ------------------------------------------------------------------ backward
// Half of Dsum[q] = sum_d dO[q][d] * O[q][d]: the 32 elements d = 16 t + 8 g + e (t < 4, e < 8) of one row, in
// that order; Dsum = half(g = 0) + half(g = 1).  Both backward roles form it this way (bitwise the same value).
struct DsumWords { uint4 a[4], d[4]; };  // half a row of O and of dO
__device__ __forceinline__ void dsum_load(const bf16_t* __restrict__ po, const bf16_t* __restrict__ pd, int g, DsumWords& w) {
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    w.a[t] = *reinterpret_cast<const uint4*>(po + 16 * t + 8 * g);
    w.d[t] = *reinterpret_cast<const uint4*>(pd + 16 * t + 8 * g);
  }
}
__device__ __forceinline__ float dsum_math(const DsumWords& w) {
  float s = 0.f;
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const uint32_t aw[4] = {w.a[t].x, w.a[t].y, w.a[t].z, w.a[t].w}, dw[4] = {w.d[t].x, w.d[t].y, w.d[t].z, w.d[t].w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      s += __uint_as_float(aw[k] << 16) * __uint_as_float(dw[k] << 16);
      s += __uint_as_float(aw[k] & 0xffff0000u) * __uint_as_float(dw[k] & 0xffff0000u);
    }
  }
  return s;
}
__device__ __forceinline__ float dsum_half(const bf16_t* __restrict__ po, const bf16_t* __restrict__ pd, int g) {
  DsumWords w;
  dsum_load(po, pd, g, w);
  return dsum_math(w);
}

// dK, dV: a wavefront owns 32 keys (lane = key), loops over query tiles.
__device__ __forceinline__ void attention_bwd_dkv_body(const bf16_t* __restrict__ qkv,
                                                       const bf16_t* __restrict__ d_o,
                                                       const float* __restrict__ lse,
                                                       const bf16_t* __restrict__ o,
                                                       bf16_t* __restrict__ dqkv, int S, int D, int H, int bx,
                                                       unsigned char* smem) {
  const int TS = S + 8;
  bf16_t* sQ = reinterpret_cast<bf16_t*>(smem);  // [S][RS]
  bf16_t* sdO = sQ + S * RS;                     // [S][RS]
  bf16_t* sQt = sdO + S * RS;                    // [64][TS]
  bf16_t* sdOt = sQt + HD * TS;                  // [64][TS]
  float* sL = reinterpret_cast<float*>(sdOt + HD * TS);  // [S] lse, then [S] dsum
  float* sD = sL + S;
  const int b = blockIdx.z, h = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 31, g = lane >> 5;
  const long ld = 3L * D;
  const bf16_t* base = qkv + (long)b * S * ld + h * HD;
  const bf16_t* dobase = d_o + (long)b * S * D + h * HD;
  // Everything read from global memory is requested before the staging copies wait for theirs: this wavefront's
  // K and V fragments, the log-sum-exp values, and the words of the first round of row sums of dO * O.
  const int k0 = bx * 128 + wave * 32;
  const bool live = k0 < S;
  const int key = live ? k0 + col : 0;
  bf16x8 kf[4], vf[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    kf[t] = ld_frag(base + D + (long)key * ld + 16 * t + 8 * g);
    vf[t] = ld_frag(base + 2 * D + (long)key * ld + 16 * t + 8 * g);
  }
  const int tid = threadIdx.x;
  const float lse_mine = tid < S ? lse[((long)b * H + h) * S + tid] : 0.f;  // blockDim.x = 256 >= S
  DsumWords w0;
  const bool has0 = tid < 2 * S;  // uniform per wavefront (2 S is a multiple of 64)
  if (has0) {  // thread -> (row, half): neighbouring lanes hold the two halves
    const long at = ((long)b * S + (tid >> 1)) * D + h * HD;
    dsum_load(o + at, d_o + at, tid & 1, w0);
  }
  stage_pair<true, true, true, true>(sQ, sQt, base, ld, sdO, sdOt, dobase, D, S);
  if (tid < S) sL[tid] = lse_mine;
  if (has0) {
    const float half = dsum_math(w0);
    const float other = __shfl_xor(half, 1);
    if (!(tid & 1)) sD[tid >> 1] = half + other;
  }
  for (int i = tid + (int)blockDim.x; i < 2 * S; i += blockDim.x) {  // S = 256: the second round
    const int row = i >> 1;
    const long at = ((long)b * S + row) * D + h * HD;
    const float half = dsum_half(o + at, d_o + at, i & 1);
    const float other = __shfl_xor(half, 1);
    if (!(i & 1)) sD[row] = half + other;
  }
  __syncthreads();
  if (!live) return;
  floatx16 dk[2], dv[2];
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) { dk[dt][r] = 0.f; dv[dt][r] = 0.f; }
  const float scale = 0.125f;

  for (int qt = 0; qt < S / 32; ++qt) {
    floatx16 s, dp;
#pragma unroll
    for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ld_frag(sQ + (qt * 32 + col) * RS + 16 * t + 8 * g), kf[t], s, 0, 0, 0);
      dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ld_frag(sdO + (qt * 32 + col) * RS + 16 * t + 8 * g), vf[t], dp, 0, 0, 0);
    }
    float p[16], ds[16];
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {  // registers 4 r4 .. 4 r4 + 3 are four consecutive queries: one 16-byte read each
      const int qq = qt * 32 + acc_row(4 * r4, g);
      const float4 l4 = *reinterpret_cast<const float4*>(sL + qq);
      const float4 d4 = *reinterpret_cast<const float4*>(sD + qq);
      const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dv4[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int r = 4 * r4 + e;
        p[r] = __expf(s[r] * scale - lv[e]);
        ds[r] = p[r] * (dp[r] - dv4[e]);
      }
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      bf16x8 pf = pack_frag(p + 8 * u), dsf = pack_frag(ds + 8 * u);
#pragma unroll
      for (int dt = 0; dt < 2; ++dt) {
        const int off = (dt * 32 + col) * TS + qt * 32 + 16 * u + 4 * g;
        dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ld_frag_2x4(sdOt + off, sdOt + off + 8), pf, dv[dt], 0, 0, 0);
        dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ld_frag_2x4(sQt + off, sQt + off + 8), dsf, dk[dt], 0, 0, 0);
      }
    }
  }
  bf16_t* krow = dqkv + ((long)b * S + key) * ld + D + h * HD;
  bf16_t* vrow = krow + D;
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      uint2 a, c;
      a.x = f2bf_pk(dk[dt][4 * r4] * scale, dk[dt][4 * r4 + 1] * scale);
      a.y = f2bf_pk(dk[dt][4 * r4 + 2] * scale, dk[dt][4 * r4 + 3] * scale);
      c.x = f2bf_pk(dv[dt][4 * r4], dv[dt][4 * r4 + 1]);
      c.y = f2bf_pk(dv[dt][4 * r4 + 2], dv[dt][4 * r4 + 3]);
      *reinterpret_cast<uint2*>(krow + dt * 32 + 8 * r4 + 4 * g) = a;
      *reinterpret_cast<uint2*>(vrow + dt * 32 + 8 * r4 + 4 * g) = c;
    }
}

// dQ: a wavefront owns 32 queries (lane = query), loops over key tiles.
__device__ __forceinline__ void attention_bwd_dq_body(const bf16_t* __restrict__ qkv,
                                                      const bf16_t* __restrict__ d_o,
                                                      const float* __restrict__ lse,
                                                      const bf16_t* __restrict__ o,
                                                      bf16_t* __restrict__ dqkv, int S, int D, int H, int bx,
                                                      unsigned char* smem) {
  const int TS = S + 8;
  bf16_t* sK = reinterpret_cast<bf16_t*>(smem);  // [S][RS]
  bf16_t* sV = sK + S * RS;                      // [S][RS]
  bf16_t* sKt = sV + S * RS;                     // [64][TS]
  const int b = blockIdx.z, h = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 31, g = lane >> 5;
  const long ld = 3L * D;
  const bf16_t* base = qkv + (long)b * S * ld + h * HD;
  // (all global reads of this wavefront are requested before the staging copies wait for theirs)
  const int q0 = bx * 128 + wave * 32;
  const bool live = q0 < S;
  const int q = live ? q0 + col : 0;
  bf16x8 qf[4], dof[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    qf[t] = ld_frag(base + (long)q * ld + 16 * t + 8 * g);
    dof[t] = ld_frag(d_o + ((long)b * S + q) * D + h * HD + 16 * t + 8 * g);
  }
  const float lq = lse[((long)b * H + h) * S + q];
  DsumWords wq;
  {
    const long at = ((long)b * S + q) * D + h * HD;
    dsum_load(o + at, d_o + at, g, wq);
  }
  stage_pair<true, true, true, false>(sK, sKt, base + D, ld, sV, nullptr, base + 2 * D, ld, S);
  __syncthreads();
  if (!live) return;
  float dq_sum;
  {
    const float half = dsum_math(wq);
    const float other = __shfl_xor(half, 32);
    dq_sum = g == 0 ? half + other : other + half;  // half(0) + half(1) in both lanes
  }
  floatx16 dq[2];
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) dq[dt][r] = 0.f;
  const float scale = 0.125f;
  for (int kt = 0; kt < S / 32; ++kt) {
    floatx16 s, dp;
#pragma unroll
    for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ld_frag(sK + (kt * 32 + col) * RS + 16 * t + 8 * g), qf[t], s, 0, 0, 0);
      dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ld_frag(sV + (kt * 32 + col) * RS + 16 * t + 8 * g), dof[t], dp, 0, 0, 0);
    }
    float ds[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) ds[r] = __expf(s[r] * scale - lq) * (dp[r] - dq_sum);
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      bf16x8 dsf = pack_frag(ds + 8 * u);
#pragma unroll
      for (int dt = 0; dt < 2; ++dt) {
        const int off = (dt * 32 + col) * TS + kt * 32 + 16 * u + 4 * g;
        dq[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ld_frag_2x4(sKt + off, sKt + off + 8), dsf, dq[dt], 0, 0, 0);
      }
    }
  }
  bf16_t* qrow = dqkv + ((long)b * S + q) * ld + h * HD;
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      uint2 a;
      a.x = f2bf_pk(dq[dt][4 * r4] * scale, dq[dt][4 * r4 + 1] * scale);
      a.y = f2bf_pk(dq[dt][4 * r4 + 2] * scale, dq[dt][4 * r4 + 3] * scale);
      *reinterpret_cast<uint2*>(qrow + dt * 32 + 8 * r4 + 4 * g) = a;
    }
}

size_t lds_fwd(int S) { return ((size_t)S * RS + (size_t)HD * (S + 8)) * 2; }
size_t lds_dkv(int S) { return ((size_t)2 * S * RS + (size_t)2 * HD * (S + 8)) * 2 + (size_t)2 * S * 4; }
size_t lds_dq(int S) { return ((size_t)2 * S * RS + (size_t)HD * (S + 8)) * 2; }

// kernels may need more than the default 64 KiB of dynamic LDS (S = 256)
// dK/dV and dQ in ONE launch: the two are independent and each alone is a short latency-bound
// chain, so their blocks are dealt from one grid: block ids [0, nx) of the x dimension are the
// key tiles of the dK/dV role, [nx, 2 nx) the query tiles of the dQ role.
__global__ __launch_bounds__(256) void attention_bwd_kernel(const bf16_t* __restrict__ qkv,
                                                            const bf16_t* __restrict__ d_o,
                                                            const float* __restrict__ lse,
                                                            const bf16_t* __restrict__ o,
                                                            bf16_t* __restrict__ dqkv, int S, int D, int H, int nx) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  if ((int)blockIdx.x < nx) attention_bwd_dkv_body(qkv, d_o, lse, o, dqkv, S, D, H, (int)blockIdx.x, smem);  // uniform
  else attention_bwd_dq_body(qkv, d_o, lse, o, dqkv, S, D, H, (int)blockIdx.x - nx, smem);
}

void allow_lds(const void* fn, size_t bytes) {
  (void)hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

}  // namespace

size_t mha_bf16_ws_bytes(int B, int S, int D, int heads) {
  (void)D;
  return (size_t)B * heads * S * sizeof(float) + 256;  // Dsum
}

void attention_fwd_bf16(hipStream_t st, const bf16_t* qkv, bf16_t* o, float* lse, int B, int S, int D, int heads) {
  size_t lds = lds_fwd(S);
  allow_lds((const void*)attention_fwd_kernel, lds);
  KLAUNCH(attention_fwd_kernel, dim3((S + 127) / 128, heads, B), dim3(256), lds, st, qkv, o, lse, S, D, heads);
}

void attention_bwd_bf16(hipStream_t st, const bf16_t* qkv, const bf16_t* o, const bf16_t* d_o, const float* lse,
                        bf16_t* dqkv, float* dsum, int B, int S, int D, int heads) {
  (void)dsum;  // the row sums of dO * O are formed inside the kernel (they were a launch of their own)
  const size_t l1 = lds_dkv(S), l2 = lds_dq(S), lds = l1 > l2 ? l1 : l2;
  allow_lds((const void*)attention_bwd_kernel, lds);
  const int nx = (S + 127) / 128;
  dim3 grid(2 * nx, heads, B);
  KLAUNCH(attention_bwd_kernel, grid, dim3(256), lds, st, qkv, d_o, lse, o, dqkv, S, D, heads, nx);
}

}  // namespace ast
