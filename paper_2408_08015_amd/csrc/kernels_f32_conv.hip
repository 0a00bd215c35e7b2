// fp32 NCHW convolution kernels of the MobileNetV2-style stages.
//
// Pointwise (1x1) convolution = per-pixel matrix product on the fp32 matrix cores
// (v_mfma_f32_32x32x2f32).  In NCHW a channel plane is contiguous, so pixels go on the MFMA
// N dimension: lane l supplies B[k = l/32][pixel = l%32] with one coalesced global load,
// the small weight matrix is A[m = l%32][k = l/32], read from a copy packed in exactly that
// lane order, and accumulator register r of lane l is D[8*(r/4) + 4*(l/32) + r%4][l%32].
// At these shapes the kernels are HBM / latency bound, so the launch shapes are chosen for
// wavefront count first.
//
// Depthwise 3x3: a block stages whole (n, c) planes (they are contiguous) with a zero halo
// in LDS; the backward kernel produces the input gradient and the nine weight-gradient
// sums of each plane from one read of g and x.
#include "bn_common.h"
#include "device_utils.h"
#include "kernels.h"
#include "prof.h"

namespace ast {

static inline int cdiv(long a, long b) { return (int)((a + b - 1) / b); }
static inline int conv_out(int H, int k, int stride, int pad) { return (H + 2 * pad - k) / stride + 1; }

// ============================================================== pointwise conv (fwd / dgrad)
// Block = 4 wavefronts; wavefront w owns pixels [128*bx + 32*w, +32) of the flattened
// (n, p) index and one 32-row tile of output channels.  MFMA 32x32x2: lane l supplies
// A[m = l%32][k = l/32] and B[k = l/32][q = l%32]; accumulator register r of lane l is
// D[8*(r/4) + 4*(l/32) + r%4][l%32].
struct PwArgs {  // one pointwise-conv product Y = A X (+ bias) (+ add)
  const float4* Wp;
  const float* X;
  float* Y;
  const float* bias;
  const float* add;
  double* stats;  // or NULL: per block (sum, sum of squares) of the output per channel, stats[m][gridDim.x][2]
  long NQ;
  int HW, Kdim, Mdim, KG;
  int tile_order;  // 1: the channel tiles of one pixel block run side by side on one XCD (they share X)
};
struct WgArgs {  // one pointwise-conv weight-gradient launch (partials only)
  const float* g;
  const float* x;
  float* part;
  int Cin, Cout, HW, cps, pxw;
  int tile_order;  // 1: the (ci, co) tiles of one pixel chunk run side by side on one XCD
};

// Block coordinates of a product grid of gx pixel blocks x gy channel tiles from the flat block id:
// pixel blocks fastest, or (tile_order) channel tiles fastest within XCD-grouped ids, so that the
// gy blocks that read the same pixels of X hit one L2.
__device__ __forceinline__ void pw_block_xy(unsigned id, unsigned gx, unsigned gy, int tile_order, int& bx, int& by) {
  if (tile_order) {
    id = xcd_grouped(id, gx * gy);
    by = (int)(id % gy);
    bx = (int)(id / gy);
  } else {
    bx = (int)(id % gx);
    by = (int)(id / gx);
  }
}

// The A operand comes from a packed copy of the weights (pw_pack_f32): for m-tile t and
// k-group g (8 consecutive k), lane l = (m%32, h) finds the four values A[m][8g + 2e + h],
// e = 0..3, as one 16-byte word at Wp[(t*KG + g)*64 + l]; out-of-range m and k are zero
// there.  A wavefront therefore reads its operands with fully coalesced 16-byte loads
// and needs neither LDS nor a barrier, and all loads of a pass are issued before its first
// MFMA.  NCH = 32-channel chunks per pass.
// Statistics epilogue of the forward product (for a BatchNorm behind the convolution): lane l
// holds, for each of its 16 accumulator rows, the sum s and sum of squares q of its pixels; the
// block adds them per channel over its pixels (through LDS, two rounds of 16 KB) and writes one
// (sum, sum of squares) pair per channel and block.  All 256 threads take part.
__device__ __forceinline__ void pw_stats_epilogue(const float (&s)[16], const float (&q)[16], float (*sR)[16][64],
                                                  double* __restrict__ stats, int m_base, int Mdim, int bx, int P) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int ci = threadIdx.x >> 3, part = threadIdx.x & 7;  // channel of the 32-row tile, slice of its 128 values
  const int r = 4 * (ci >> 3) + (ci & 3), half = (ci >> 2) & 1;
  const int w = part >> 1, c0 = half * 32 + (part & 1) * 16;
  const int rot = (ci & 3) * 4 + w;  // start of the 16-value walk: the 64 lanes of a wavefront hit 64 banks
  float tot[2];
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    if (pass) __syncthreads();  // the first round has been read
#pragma unroll
    for (int k = 0; k < 16; ++k) sR[wave][k][lane] = pass ? q[k] : s[k];
    __syncthreads();
    float v = 0.f;
#pragma unroll
    for (int k = 0; k < 16; ++k) v += sR[w][r][c0 + ((k + rot) & 15)];
    v = group8_sum(v);
    tot[pass] = v;
  }
  if (part == 0 && m_base + ci < Mdim) {
    double* o = stats + ((size_t)(m_base + ci) * P + bx) * 2;
    o[0] = (double)tot[0];
    o[1] = (double)tot[1];
  }
}

template <int NCH>
__device__ __forceinline__ void pw_pk_body(const PwArgs& a, int bx, int by, float (*sR)[16][64], int P) {
  const float4* __restrict__ Wp = a.Wp;
  const float* __restrict__ X = a.X;
  float* __restrict__ Y = a.Y;
  const float* __restrict__ bias = a.bias;
  const float* __restrict__ add = a.add;
  const long NQ = a.NQ;
  const int HW = a.HW, Kdim = a.Kdim, Mdim = a.Mdim, KG = a.KG;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 31, half = lane >> 5;
  const int m_base = by * 32;
  const unsigned q = (unsigned)bx * 128u + wave * 32 + col;  // pixels per micro-batch < 2^31 (checked at create)
  const bool qv = q < NQ;
  unsigned n = 0;
  int p = 0;
  if (qv) {
    n = q / (unsigned)HW;  // 32-bit: a 64-bit division is ~150 instructions
    p = (int)(q - n * (unsigned)HW);
  }
  const float* xq = X + (size_t)n * Kdim * HW + p;
  const float4* wl = Wp + (size_t)by * KG * 64 + lane;
  floatx16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  for (int g0 = 0; g0 < KG; g0 += NCH * 4) {
    float4 a[NCH * 4];
    float b[NCH * 16];
#pragma unroll
    for (int g = 0; g < NCH * 4; ++g) {
      const bool ok = g0 + g < KG;
      a[g] = ok ? wl[(size_t)(g0 + g) * 64] : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        // branch-free: rows past Kdim read the last row (zero weights in the packed copy), pixels past
        // NQ read pixel 0 and are replaced by zero (the statistics epilogue sums every column)
        const int k = min((g0 + g) * 8 + 2 * e + half, Kdim - 1);
        const float val = xq[(size_t)k * HW];
        b[4 * g + e] = qv ? val : 0.f;
      }
    }
#pragma unroll
    for (int g = 0; g < NCH * 4; ++g) {
      if (NCH > 1 && g0 + g >= KG) break;  // uniform: skip the empty tail of the last pass
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[g].x, b[4 * g + 0], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[g].y, b[4 * g + 1], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[g].z, b[4 * g + 2], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[g].w, b[4 * g + 3], acc, 0, 0, 0);
    }
  }
  if (qv) {
    float* yq = Y + (size_t)n * Mdim * HW + p;
    const float* aq = add ? add + (size_t)n * Mdim * HW + p : nullptr;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int m = m_base + 8 * (r >> 2) + 4 * half + (r & 3);
      if (m < Mdim) {
        float v = acc[r];
        if (bias) v += bias[m];
        if (aq) v += aq[(size_t)m * HW];
        yq[(size_t)m * HW] = v;
      }
    }
  }
  if (a.stats) {  // uniform; only without bias / add (the accumulators are the outputs; invalid pixels hold zeros)
    float s[16], q2[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      s[r] = acc[r];
      q2[r] = acc[r] * acc[r];
    }
    pw_stats_epilogue(s, q2, sR, a.stats, m_base, Mdim, bx, P);
  }
}
template <int NCH>
__global__ __launch_bounds__(256) void pw_conv_f32_pk_kernel(PwArgs a) {
  __shared__ float sR[4][16][64];
  int bx, by;
  pw_block_xy(blockIdx.y * gridDim.x + blockIdx.x, gridDim.x, gridDim.y, a.tile_order, bx, by);
  pw_pk_body<NCH>(a, bx, by, sR, gridDim.x);
}

// Few pixels, long K (the 14x14 / 7x7 layers of a whole network): the four wavefronts of a
// block share one 32-pixel x 32-channel output tile and split K between them, so there are
// four times as many wavefronts and a quarter of the dependent passes; the four partial
// tiles are added through LDS in a fixed order.
template <int WV>  // wavefronts per block = ways K is split (4, 8 or 16)
__device__ __forceinline__ void pw_pkks_body(const PwArgs& a, int bx, int by, float (*sR)[16][64]) {
  const float4* __restrict__ Wp = a.Wp;
  const float* __restrict__ X = a.X;
  float* __restrict__ Y = a.Y;
  const float* __restrict__ bias = a.bias;
  const float* __restrict__ add = a.add;
  const long NQ = a.NQ;
  const int HW = a.HW, Kdim = a.Kdim, Mdim = a.Mdim, KG = a.KG;

  constexpr int NCH = 2;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 31, half = lane >> 5;
  const int m_base = by * 32;
  const unsigned q = (unsigned)bx * 32u + col;  // pixels per micro-batch < 2^31 (checked at create)
  const bool qv = q < NQ;
  unsigned n = 0;
  int p = 0;
  if (qv) {
    n = q / (unsigned)HW;  // 32-bit: a 64-bit division is ~150 instructions
    p = (int)(q - n * (unsigned)HW);
  }
  const float* xq = X + (size_t)n * Kdim * HW + p;
  const float4* wl = Wp + (size_t)by * KG * 64 + lane;
  const int gper = (KG + WV - 1) / WV;  // k-groups per wavefront
  const int gbeg = wave * gper, gend = min(gbeg + gper, KG);
  floatx16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  for (int g0 = gbeg; g0 < gend; g0 += NCH * 4) {
    float4 a[NCH * 4];
    float b[NCH * 16];
#pragma unroll
    for (int g = 0; g < NCH * 4; ++g) {
      const bool ok = g0 + g < gend;
      a[g] = ok ? wl[(size_t)(g0 + g) * 64] : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int k = min((g0 + g) * 8 + 2 * e + half, Kdim - 1);  // branch-free, as above
        const float val = xq[(size_t)k * HW];
        b[4 * g + e] = qv ? val : 0.f;
      }
    }
#pragma unroll
    for (int g = 0; g < NCH * 4; ++g) {
      if (g0 + g >= gend) break;  // uniform
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[g].x, b[4 * g + 0], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[g].y, b[4 * g + 1], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[g].z, b[4 * g + 2], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[g].w, b[4 * g + 3], acc, 0, 0, 0);
    }
  }
#pragma unroll
  for (int r = 0; r < 16; ++r) sR[wave][r][lane] = acc[r];
  __syncthreads();
  if (!qv) return;
  float* yq = Y + (size_t)n * Mdim * HW + p;
  const float* aq = add ? add + (size_t)n * Mdim * HW + p : nullptr;
  constexpr int RW = 16 / WV;  // rows of the register layout each wavefront finishes
#pragma unroll
  for (int rr = 0; rr < RW; ++rr) {
    const int r = RW * wave + rr;
    const int m = m_base + 8 * (r >> 2) + 4 * half + (r & 3);
    if (m < Mdim) {
      float v = 0.f;
#pragma unroll
      for (int k = 0; k < WV; k += 4)  // fixed order
        v += (sR[k][r][lane] + sR[k + 1][r][lane]) + (sR[k + 2][r][lane] + sR[k + 3][r][lane]);
      if (bias) v += bias[m];
      if (aq) v += aq[(size_t)m * HW];
      yq[(size_t)m * HW] = v;
    }
  }
}
template <int WV>
__global__ __launch_bounds__(64 * WV) void pw_conv_f32_pkks_kernel(PwArgs a) {
  __shared__ float sR[WV][16][64];
  pw_pkks_body<WV>(a, blockIdx.x, blockIdx.y, sR);
}

// Large images: a wavefront owns 128 pixels; every lane loads four consecutive pixels
// (16 bytes) per input channel and feeds four MFMA column tiles (column j of tile t is
// pixel 4j + t), so each output row is stored as 16 bytes per lane.  Four times the bytes
// per memory instruction and a quarter of the weight traffic of the kernel above; needs
// HW % 4 == 0.
__device__ __forceinline__ void pw_pk4_body(const PwArgs& a, int bx, int by, float (*sR)[16][64], int P) {
  const float4* __restrict__ Wp = a.Wp;
  const float* __restrict__ X = a.X;
  float* __restrict__ Y = a.Y;
  const float* __restrict__ bias = a.bias;
  const float* __restrict__ add = a.add;
  const long NQ = a.NQ;
  const int HW = a.HW, Kdim = a.Kdim, Mdim = a.Mdim, KG = a.KG;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 31, half = lane >> 5;
  const int m_base = by * 32;
  const unsigned q = (unsigned)bx * 512u + wave * 128 + col * 4;  // pixels per micro-batch < 2^31 (checked at create)
  const bool qv = q < NQ;  // NQ % 4 == 0: the four pixels are valid together
  unsigned n = 0;
  int p = 0;
  if (qv) {
    n = q / (unsigned)HW;  // 32-bit: a 64-bit division is ~150 instructions
    p = (int)(q - n * (unsigned)HW);
  }
  const float* xq = X + (size_t)n * Kdim * HW + p;
  const float4* wl = Wp + (size_t)by * KG * 64 + lane;
  floatx16 acc[4];
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
  for (int g0 = 0; g0 < KG; g0 += 4) {
    float4 a[4];
    float4 b[16];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const bool ok = g0 + g < KG;
      a[g] = ok ? wl[(size_t)(g0 + g) * 64] : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int k = min((g0 + g) * 8 + 2 * e + half, Kdim - 1);  // branch-free, as above
        const float4 val = *reinterpret_cast<const float4*>(xq + (size_t)k * HW);
        b[4 * g + e] = qv ? val : make_float4(0.f, 0.f, 0.f, 0.f);
      }
    }
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      if (g0 + g >= KG) break;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float av = e == 0 ? a[g].x : e == 1 ? a[g].y : e == 2 ? a[g].z : a[g].w;
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, b[4 * g + e].x, acc[0], 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, b[4 * g + e].y, acc[1], 0, 0, 0);
        acc[2] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, b[4 * g + e].z, acc[2], 0, 0, 0);
        acc[3] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, b[4 * g + e].w, acc[3], 0, 0, 0);
      }
    }
  }
  if (qv) {
    float* yq = Y + (size_t)n * Mdim * HW + p;
    const float* aq = add ? add + (size_t)n * Mdim * HW + p : nullptr;
    // bias and addend of eight rows at a time are requested before the first is used (rows past Mdim
    // read the last row)
#pragma unroll
    for (int r0 = 0; r0 < 16; r0 += 8) {
      float bv[8];
      float4 kv[8];
#pragma unroll
      for (int rr = 0; rr < 8; ++rr) {
        const int r = r0 + rr;
        const int mc = min(m_base + 8 * (r >> 2) + 4 * half + (r & 3), Mdim - 1);
        bv[rr] = 0.f;
        kv[rr] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (bias) bv[rr] = bias[mc];
        if (aq) kv[rr] = *reinterpret_cast<const float4*>(aq + (size_t)mc * HW);
      }
#pragma unroll
      for (int rr = 0; rr < 8; ++rr) {
        const int r = r0 + rr;
        const int m = m_base + 8 * (r >> 2) + 4 * half + (r & 3);
        if (m < Mdim)
          *reinterpret_cast<float4*>(yq + (size_t)m * HW) =
              make_float4(acc[0][r] + bv[rr] + kv[rr].x, acc[1][r] + bv[rr] + kv[rr].y, acc[2][r] + bv[rr] + kv[rr].z,
                          acc[3][r] + bv[rr] + kv[rr].w);
      }
    }
  }
  if (a.stats) {  // uniform; only without bias / add (invalid pixels hold zeros)
    float s[16], q2[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      s[r] = (acc[0][r] + acc[1][r]) + (acc[2][r] + acc[3][r]);
      q2[r] = (acc[0][r] * acc[0][r] + acc[1][r] * acc[1][r]) + (acc[2][r] * acc[2][r] + acc[3][r] * acc[3][r]);
    }
    pw_stats_epilogue(s, q2, sR, a.stats, m_base, Mdim, bx, P);
  }
}
__global__ __launch_bounds__(256) void pw_conv_f32_pk4_kernel(PwArgs a) {
  __shared__ float sR[4][16][64];
  int bx, by;
  pw_block_xy(blockIdx.y * gridDim.x + blockIdx.x, gridDim.x, gridDim.y, a.tile_order, bx, by);
  pw_pk4_body(a, bx, by, sR, gridDim.x);
}

// Packed operand copy: Wp[((t*KG + g)*64 + l)*4 + e] = A[32t + l%32][8g + 2e + l/32], zero
// outside Mdim x Kdim, with A[m][k] = W[m*lda_m + k*lda_k].
__global__ void pw_pack_kernel(const float* __restrict__ W, int lda_m, int lda_k, float* __restrict__ Wp,
                               int Mdim, int Kdim, int KG, size_t total) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int e = (int)(i & 3), l = (int)((i >> 2) & 63);
  const size_t tg = i >> 8;
  const int g = (int)(tg % KG), t = (int)(tg / KG);
  const int m = 32 * t + (l & 31), k = 8 * g + 2 * e + (l >> 5);
  Wp[i] = (m < Mdim && k < Kdim) ? W[(size_t)m * lda_m + (size_t)k * lda_k] : 0.f;
}

size_t pw_pack_floats(int Mdim, int Kdim) { return (size_t)cdiv(Mdim, 32) * cdiv(Kdim, 8) * 256; }

// Every packed copy of a stage in one launch: the copies sit back to back in one arena, each a
// multiple of 256 floats, so block b (256 floats of the arena) belongs to one task.
__global__ __launch_bounds__(256) void pw_pack_all_kernel(const PackTask* __restrict__ tasks,
                                                          const unsigned short* __restrict__ block_task,
                                                          float* __restrict__ arena) {
  const PackTask t = tasks[block_task[blockIdx.x]];
  const size_t i = (size_t)(blockIdx.x - t.block0) * 256 + threadIdx.x;  // index inside the copy
  const int e = (int)(i & 3), l = (int)((i >> 2) & 63);
  const size_t tg = i >> 8;
  const int g = (int)(tg % t.KG), tt = (int)(tg / t.KG);
  const int m = 32 * tt + (l & 31), k = 8 * g + 2 * e + (l >> 5);
  arena[(size_t)blockIdx.x * 256 + threadIdx.x] =
      (m < t.Mdim && k < t.Kdim) ? t.W[(size_t)m * t.lda_m + (size_t)k * t.lda_k] : 0.f;
}
void pw_pack_all_f32(hipStream_t st, const PackTask* tasks_dev, const unsigned short* block_task_dev, float* arena,
                     int nblocks) {
  KLAUNCH(pw_pack_all_kernel, dim3(nblocks), dim3(256), 0, st, tasks_dev, block_task_dev, arena);
}

void pw_pack_f32(hipStream_t st, const float* W, int lda_m, int lda_k, float* Wp, int Mdim, int Kdim) {
  const size_t total = pw_pack_floats(Mdim, Kdim);
  KLAUNCH(pw_pack_kernel, dim3((unsigned)cdiv(total, 256)), dim3(256), 0, st, W, lda_m, lda_k, Wp, Mdim, Kdim,
          cdiv(Kdim, 8), total);
}

// which product kernel serves a shape, and its grid
struct PwPick { int var; dim3 grid; int wv; };  // wv: wavefronts per block of the K-split kernel
static PwPick pw_pick(long NQ, int HW, int Kdim, int Mdim) {
  const int mt = cdiv(Mdim, 32), KG = cdiv(Kdim, 8);
  PwPick p;
  // Measured on 32-sample micro-batches: 128-pixel wavefronts win from 56x56 images up,
  // 32-pixel ones below (more wavefronts in flight matter more than bytes per instruction);
  // under one block per CU and K >= 128 the block splits K instead.
  p.wv = 4;
  if ((long)cdiv(NQ, 128) * mt < 256 && KG >= 16) {
    p.var = 2;
    p.grid = dim3((unsigned)cdiv(NQ, 32), mt);
    // one pass of 64 channels per wavefront where K allows: a longer K is a chain of dependent
    // load-then-multiply passes, the whole cost of these small products
    p.wv = KG <= 32 ? 4 : (KG <= 64 ? 8 : 16);
  }
  else if (HW % 4 == 0 && NQ >= 65536) { p.var = 3; p.grid = dim3((unsigned)cdiv(NQ, 512), mt); }
  else if (Kdim > 32) { p.var = 1; p.grid = dim3((unsigned)cdiv(NQ, 128), mt); }
  else { p.var = 0; p.grid = dim3((unsigned)cdiv(NQ, 128), mt); }
  return p;
}
static int pw_tile_order() {
  static const int v = [] { const char* e = getenv("ASTEROID_PW_TILE_ORDER"); return e ? atoi(e) : 3; }();
  return v;
}
static PwArgs pw_args(const float* Wp, const float* X, float* Y, const float* bias, const float* add, int N, int Kdim,
                      int Mdim, int HW) {
  PwArgs a;
  a.Wp = reinterpret_cast<const float4*>(Wp);
  a.X = X; a.Y = Y; a.bias = bias; a.add = add;
  a.stats = nullptr;
  a.NQ = (long)N * HW;
  a.HW = HW; a.Kdim = Kdim; a.Mdim = Mdim; a.KG = cdiv(Kdim, 8);
  a.tile_order = (pw_tile_order() & 1) && Mdim > 32;
  return a;
}

static void launch_pkks(hipStream_t st, const PwArgs& a, const PwPick& p) {
  if (p.wv == 16) KLAUNCH_NAMED("pw_conv_f32_pkks_kernel<16>", (pw_conv_f32_pkks_kernel<16>), p.grid, dim3(1024), 0, st, a);
  else if (p.wv == 8) KLAUNCH_NAMED("pw_conv_f32_pkks_kernel<8>", (pw_conv_f32_pkks_kernel<8>), p.grid, dim3(512), 0, st, a);
  else KLAUNCH_NAMED("pw_conv_f32_pkks_kernel", (pw_conv_f32_pkks_kernel<4>), p.grid, dim3(256), 0, st, a);
}

// Partial pairs per channel that the forward product can leave for a BatchNorm behind it: the
// number of pixel blocks of the 32- and 128-pixel-wavefront kernels while that is at most 256
// (more would cost the consumer more than a statistics pass of its own); 0 = not offered.
int pw_conv_stats_parts(int N, int Kdim, int Mdim, int HW) {
  const PwPick p = pw_pick((long)N * HW, HW, Kdim, Mdim);
  if (p.var == 2 || p.grid.x > 256) return 0;
  return (int)p.grid.x;
}

void pw_conv_f32(hipStream_t st, const float* Wp, const float* X, float* Y, const float* bias, const float* add,
                 int N, int Kdim, int Mdim, int HW, double* stats) {
  PwArgs a = pw_args(Wp, X, Y, bias, add, N, Kdim, Mdim, HW);
  const PwPick p = pw_pick(a.NQ, HW, Kdim, Mdim);
  if (stats && !bias && !add && p.var != 2) a.stats = stats;
  switch (p.var) {
    case 2: launch_pkks(st, a, p); break;
    case 3: KLAUNCH(pw_conv_f32_pk4_kernel, p.grid, dim3(256), 0, st, a); break;
    case 1: KLAUNCH(pw_conv_f32_pk_kernel<2>, p.grid, dim3(256), 0, st, a); break;
    default: KLAUNCH(pw_conv_f32_pk_kernel<1>, p.grid, dim3(256), 0, st, a); break;
  }
}

// ============================================================== pointwise conv wgrad
// Block = one 32(co) x 32(ci) tile of dW over 4*pxw pixels of one sample; each wavefront
// contracts pxw pixels (lane (m = l%32, h = l/32) loads eight consecutive pixels of row m
// and feeds eight MFMAs; both operands use the same pixel per slot), the four accumulators
// are added through LDS and written as one partial.  A second kernel adds the partials in a
// fixed order and performs G += (in-place gradient accumulation).
template <bool VEC>
__device__ __forceinline__ void pw_wgrad_body(const WgArgs& w, int bx, int by, int bz, float (*sR)[16][64]) {
  const float* __restrict__ g = w.g;
  const float* __restrict__ x = w.x;
  float* __restrict__ part = w.part;
  const int Cin = w.Cin, Cout = w.Cout, HW = w.HW, cps = w.cps, pxw = w.pxw;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row = lane & 31, half = lane >> 5;
  const int chunk = bx;
  const int n = chunk / cps;
  const int p0 = ((chunk - n * cps) * 4 + wave) * pxw;
  const int p1 = min(p0 + pxw, HW);
  const int ci_base = by * 32, co_base = bz * 32;
  const bool av = co_base + row < Cout, bv = ci_base + row < Cin;
  const float* ga = g + ((size_t)n * Cout + (av ? co_base + row : 0)) * HW;
  const float* xb = x + ((size_t)n * Cin + (bv ? ci_base + row : 0)) * HW;
  floatx16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  if (VEC) {  // HW % 4 == 0: aligned 16-byte loads, 16 pixels per fragment, two fragments in flight
    struct Frag { float4 a0, a1, b0, b1; };
    // Branch-free: rows beyond Cout / Cin read channel 0 (their products land in rows / columns of the
    // tile that are never stored); pixels beyond the chunk read pixel 0 and get a zero g operand.
    auto ld = [&](int p, Frag& f) {
      const int pp = p + 8 * half;
      const bool v0 = pp < p1, v1 = pp + 4 < p1;
      const int q0 = v0 ? pp : 0, q1 = v1 ? pp + 4 : 0;
      f.a0 = *reinterpret_cast<const float4*>(ga + q0);
      f.b0 = *reinterpret_cast<const float4*>(xb + q0);
      f.a1 = *reinterpret_cast<const float4*>(ga + q1);
      f.b1 = *reinterpret_cast<const float4*>(xb + q1);
      if (!v0) f.a0 = make_float4(0.f, 0.f, 0.f, 0.f);
      if (!v1) f.a1 = make_float4(0.f, 0.f, 0.f, 0.f);
    };
    auto mma = [&](const Frag& f) {
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a0.x, f.b0.x, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a0.y, f.b0.y, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a0.z, f.b0.z, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a0.w, f.b0.w, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a1.x, f.b1.x, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a1.y, f.b1.y, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a1.z, f.b1.z, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a1.w, f.b1.w, acc, 0, 0, 0);
    };
    Frag f0, f1, f2, f3;
    for (int p = p0; p < p1; p += 64) {  // four fragments issued before the first MFMA
      const bool more = p + 32 < p1;     // uniform: a 32-pixel wavefront has two fragments only
      ld(p, f0);
      ld(p + 16, f1);
      if (more) {
        ld(p + 32, f2);
        ld(p + 48, f3);
      }
      mma(f0);
      mma(f1);
      if (more) {
        mma(f2);
        mma(f3);
      }
    }
  } else {
    for (int p = p0; p < p1; p += 32) {  // sixteen pixel pairs requested before the first MFMA
      float a[16], b[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const int pp = p + 2 * u + half;
        a[u] = (av && pp < p1) ? ga[pp] : 0.f;
        b[u] = (bv && pp < p1) ? xb[pp] : 0.f;
      }
#pragma unroll
      for (int u = 0; u < 16; ++u) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u], b[u], acc, 0, 0, 0);
    }
  }
#pragma unroll
  for (int r = 0; r < 16; ++r) sR[wave][r][lane] = acc[r];
  __syncthreads();
  float* out = part + (size_t)chunk * Cout * Cin;
  const int ci = ci_base + row;
  if (ci < Cin) {
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
      const int r = 4 * wave + rr;
      const int co = co_base + 8 * (r >> 2) + 4 * half + (r & 3);
      if (co < Cout)
        out[(size_t)co * Cin + ci] = (sR[0][r][lane] + sR[1][r][lane]) + (sR[2][r][lane] + sR[3][r][lane]);
    }
  }
}
template <bool VEC>
__global__ __launch_bounds__(256) void pw_wgrad_f32_kernel(WgArgs w) {
  __shared__ float sR[4][16][64];
  int bx, t;
  pw_block_xy((blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x, gridDim.x, gridDim.y * gridDim.z,
              w.tile_order, bx, t);
  pw_wgrad_body<VEC>(w, bx, t % (int)gridDim.y, t / (int)gridDim.y, sR);
}

// Input gradient and weight-gradient partials of one pointwise conv in ONE launch: the two
// products only share their input g, and each alone is too short to fill the chip (they
// are bound by the latency of one load-compute-store chain), so their blocks are dealt from
// one grid: block ids [0, nA) form the (x, y) grid of the input-gradient product, the rest
// the (x, y, z) grid of the weight-gradient kernel.  VAR selects the product kernel:
// 0 / 1 = 32-pixel wavefronts with one / two 32-channel chunks per pass, 2 = K split over the
// block, 3 = 128-pixel wavefronts.
template <int VAR, bool VEC>
__global__ __launch_bounds__(256) void pw_bwd_dual_kernel(PwArgs a, WgArgs w, unsigned nA, unsigned gAx,
                                                          unsigned gWx, unsigned gWy) {
  __shared__ float sR[4][16][64];
  if (blockIdx.x < nA) {  // uniform per block
    int bx, by;
    pw_block_xy(blockIdx.x, gAx, nA / gAx, a.tile_order, bx, by);
    if (VAR == 0) pw_pk_body<1>(a, bx, by, sR, 0);
    else if (VAR == 1) pw_pk_body<2>(a, bx, by, sR, 0);
    else if (VAR == 2) pw_pkks_body<4>(a, bx, by, sR);
    else pw_pk4_body(a, bx, by, sR, 0);
  } else {
    int bx, t;  // the weight-gradient ids start at nA: ids that agree mod 8 still share an XCD
    pw_block_xy(blockIdx.x - nA, gWx, (gridDim.x - nA) / gWx, w.tile_order, bx, t);
    pw_wgrad_body<VEC>(w, bx, t % (int)gWy, t / (int)gWy, sR);
  }
}

// G[i] += sum_c part[c][i]: 64 outputs per block, four interleaved part lanes, fixed order
__global__ __launch_bounds__(256) void reduce_parts_acc_kernel(const float* __restrict__ part,
                                                               float* __restrict__ G, size_t n, int parts) {
  __shared__ float sh[4][64];
  const int o = threadIdx.x & 63, q = threadIdx.x >> 6;
  const size_t i = (size_t)blockIdx.x * 64 + o;
  float s = 0.f;
  if (i < n) {
    int c = q;
    for (; c + 28 < parts; c += 32) {  // eight independent loads in flight
      float v0 = part[(size_t)c * n + i], v1 = part[(size_t)(c + 4) * n + i];
      float v2 = part[(size_t)(c + 8) * n + i], v3 = part[(size_t)(c + 12) * n + i];
      float v4 = part[(size_t)(c + 16) * n + i], v5 = part[(size_t)(c + 20) * n + i];
      float v6 = part[(size_t)(c + 24) * n + i], v7 = part[(size_t)(c + 28) * n + i];
      s += ((v0 + v1) + (v2 + v3)) + ((v4 + v5) + (v6 + v7));
    }
    for (; c < parts; c += 4) s += part[(size_t)c * n + i];
  }
  sh[q][o] = s;
  __syncthreads();
  if (q == 0 && i < n) G[i] += (sh[0][o] + sh[1][o]) + (sh[2][o] + sh[3][o]);
}

// pixels per wavefront: the largest of {256,128,64,32} that still gives >= 768 blocks
static int wg_pxw(int N, int Cin, int Cout, int HW) {
  long tiles = (long)cdiv(Cin, 32) * cdiv(Cout, 32);
  const int cand[4] = {256, 128, 64, 32};
  for (int c : cand)
    if ((long)N * cdiv(HW, 4 * c) * tiles >= 768) return c;
  return 32;
}
size_t pw_wgrad_f32_ws(int N, int Cin, int Cout, int HW) {
  int pxw = wg_pxw(N, Cin, Cout, HW);
  return (size_t)N * cdiv(HW, 4 * pxw) * Cin * Cout;
}
static WgArgs wg_args(const float* g, const float* x, float* part, int N, int Cin, int Cout, int HW, dim3& grid) {
  WgArgs w;
  w.g = g; w.x = x; w.part = part;
  w.Cin = Cin; w.Cout = Cout; w.HW = HW;
  w.pxw = wg_pxw(N, Cin, Cout, HW);
  w.cps = cdiv(HW, 4 * w.pxw);
  w.tile_order = (pw_tile_order() & 2) && (Cin > 32 || Cout > 32);
  grid = dim3(N * w.cps, cdiv(Cin, 32), cdiv(Cout, 32));
  return w;
}
void pw_wgrad_f32(hipStream_t st, const float* g, const float* x, float* part, float* G, int N,
                  int Cin, int Cout, int HW) {
  dim3 grid;
  const WgArgs w = wg_args(g, x, part, N, Cin, Cout, HW, grid);
  if (HW % 4 == 0) KLAUNCH(pw_wgrad_f32_kernel<true>, grid, dim3(256), 0, st, w);
  else KLAUNCH(pw_wgrad_f32_kernel<false>, grid, dim3(256), 0, st, w);
  size_t n = (size_t)Cin * Cout;
  if (G) KLAUNCH(reduce_parts_acc_kernel, dim3(cdiv(n, 64)), dim3(256), 0, st, part, G, n, (int)grid.x);
}

template <int VAR>
static void launch_dual(hipStream_t st, const PwArgs& a, const WgArgs& w, dim3 gA, dim3 gW, bool vec) {
  const unsigned nA = gA.x * gA.y, nW = gW.x * gW.y * gW.z;
  constexpr const char* name = VAR == 0 ? "pw_bwd_dual_kernel<pk1>" : VAR == 1 ? "pw_bwd_dual_kernel<pk2>"
                             : VAR == 2 ? "pw_bwd_dual_kernel<pkks>" : "pw_bwd_dual_kernel<pk4>";
  if (vec) KLAUNCH_NAMED(name, (pw_bwd_dual_kernel<VAR, true>), dim3(nA + nW), dim3(256), 0, st, a, w, nA, gA.x, gW.x, gW.y);
  else KLAUNCH_NAMED(name, (pw_bwd_dual_kernel<VAR, false>), dim3(nA + nW), dim3(256), 0, st, a, w, nA, gA.x, gW.x, gW.y);
}

void pw_conv_bwd_f32(hipStream_t st, const float* Wp_t, const float* g, float* dx, const float* add, const float* x,
                     float* part, float* G, int N, int Cin, int Cout, int HW) {
  const PwArgs a = pw_args(Wp_t, g, dx, nullptr, add, N, Cout, Cin, HW);  // dx = W^T g (+ add)
  const PwPick p = pw_pick(a.NQ, HW, Cout, Cin);
  dim3 gW;
  const WgArgs w = wg_args(g, x, part, N, Cin, Cout, HW, gW);
  const bool vec = HW % 4 == 0;
  if (p.var == 2 && p.wv > 4) {
    // long K: the input gradient runs as wider blocks (K split 8 or 16 ways) than the weight-gradient
    // kernel's, so the two go as separate launches
    launch_pkks(st, a, p);
    if (vec) KLAUNCH(pw_wgrad_f32_kernel<true>, gW, dim3(256), 0, st, w);
    else KLAUNCH(pw_wgrad_f32_kernel<false>, gW, dim3(256), 0, st, w);
  } else switch (p.var) {
    case 2: launch_dual<2>(st, a, w, p.grid, gW, vec); break;
    case 3: launch_dual<3>(st, a, w, p.grid, gW, vec); break;
    case 1: launch_dual<1>(st, a, w, p.grid, gW, vec); break;
    default: launch_dual<0>(st, a, w, p.grid, gW, vec); break;
  }
  size_t n = (size_t)Cin * Cout;
  if (G) KLAUNCH(reduce_parts_acc_kernel, dim3(cdiv(n, 64)), dim3(256), 0, st, part, G, n, (int)gW.x);
}

__global__ __launch_bounds__(256) void reduce_tasks_kernel(const RedTask* __restrict__ tasks,
                                                           const unsigned short* __restrict__ block_task) {
  __shared__ float sh[4][64];
  const RedTask t = tasks[block_task[blockIdx.x]];
  if (t.wide) {  // uniform per block
    const size_t i4 = ((size_t)(blockIdx.x - t.block0) * 256 + threadIdx.x) * 4;
    if (i4 >= t.n) return;
    const float* p4 = t.part + i4;
    const size_t st4 = t.stride;
    const int parts4 = (int)t.parts;
    float4 s4 = make_float4(0.f, 0.f, 0.f, 0.f);
    int c4 = 0;
    for (; c4 + 4 <= parts4; c4 += 4) {
      const float4 v0 = *reinterpret_cast<const float4*>(p4 + (size_t)c4 * st4);
      const float4 v1 = *reinterpret_cast<const float4*>(p4 + (size_t)(c4 + 1) * st4);
      const float4 v2 = *reinterpret_cast<const float4*>(p4 + (size_t)(c4 + 2) * st4);
      const float4 v3 = *reinterpret_cast<const float4*>(p4 + (size_t)(c4 + 3) * st4);
      s4.x += (v0.x + v1.x) + (v2.x + v3.x);
      s4.y += (v0.y + v1.y) + (v2.y + v3.y);
      s4.z += (v0.z + v1.z) + (v2.z + v3.z);
      s4.w += (v0.w + v1.w) + (v2.w + v3.w);
    }
    for (; c4 < parts4; ++c4) {
      const float4 v = *reinterpret_cast<const float4*>(p4 + (size_t)c4 * st4);
      s4.x += v.x; s4.y += v.y; s4.z += v.z; s4.w += v.w;
    }
    const float sv[4] = {s4.x, s4.y, s4.z, s4.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      size_t out = i4 + e;
      if (t.taps > 1) {
        const size_t tp = out / t.mn;
        out = (out - tp * t.mn) * t.taps + tp;
      }
      t.G[out] += sv[e];
    }
    return;
  }
  const int o = threadIdx.x & 63, q = threadIdx.x >> 6;
  const size_t n = t.n, st = t.stride;
  const size_t i = (size_t)(blockIdx.x - t.block0) * 64 + o;
  const int parts = (int)t.parts;
  const float* p = t.part + i;
  float s = 0.f;
  if (i < n) {
    int c = q;
    for (; c + 28 < parts; c += 32) {  // eight independent loads in flight
      float v0 = p[(size_t)c * st], v1 = p[(size_t)(c + 4) * st];
      float v2 = p[(size_t)(c + 8) * st], v3 = p[(size_t)(c + 12) * st];
      float v4 = p[(size_t)(c + 16) * st], v5 = p[(size_t)(c + 20) * st];
      float v6 = p[(size_t)(c + 24) * st], v7 = p[(size_t)(c + 28) * st];
      s += ((v0 + v1) + (v2 + v3)) + ((v4 + v5) + (v6 + v7));
    }
    for (; c < parts; c += 4) s += p[(size_t)c * st];
  }
  sh[q][o] = s;
  __syncthreads();
  if (q == 0 && i < n) {
    size_t out = i;
    if (t.taps > 1) {
      const size_t tp = i / t.mn;
      out = (i - tp * t.mn) * t.taps + tp;
    }
    t.G[out] += (sh[0][o] + sh[1][o]) + (sh[2][o] + sh[3][o]);
  }
}
void reduce_tasks_f32(hipStream_t st, const RedTask* tasks_dev, const unsigned short* block_task_dev, int nblocks) {
  KLAUNCH(reduce_tasks_kernel, dim3(nblocks), dim3(256), 0, st, tasks_dev, block_task_dev);
}
int pw_wgrad_f32_parts(int N, int Cin, int Cout, int HW) { return N * cdiv(HW, 4 * wg_pxw(N, Cin, Cout, HW)); }

void reduce_parts_acc_f32(hipStream_t st, const float* part, float* G, size_t n, int parts) {
  KLAUNCH(reduce_parts_acc_kernel, dim3(cdiv(n, 64)), dim3(256), 0, st, part, G, n, parts);
}

// ============================================================== depthwise 3x3 (pad 1, stride 1 or 2)
struct DwGeom {
  int C, H, W, Ho, Wo, stride, ppb, NC;
};

// planes per block: about 4096 input elements per block, a power of two in [1, 16]
// planes per block of the LDS kernels: a power of two up to 16 with about 4096 elements per
// block, but fewer while that leaves under 1024 blocks (small tensors are latency-bound: more,
// shorter blocks, and one wavefront per plane in the BatchNorm prologues)
static int dw_ppb(int H, int W, long NC) {
  int p = 4096 / (H * W);
  int r = 1;
  while (r * 2 <= p && r < 16 && NC / (r * 2) >= 1024) r *= 2;
  return r;
}

// Zero `count` floats of LDS (all 256 threads), then barrier.
__device__ __forceinline__ void dw_zero(float* dst, int count) {
  for (int i = threadIdx.x; i < count; i += 256) dst[i] = 0.f;
  __syncthreads();
}
// Copy one h x w plane into an LDS plane of (h+2) x (w+2) (halo already zero) with the tpp
// threads of the plane's group (t = index in the group).  Four loads are issued before
// the first LDS write so the memory latency is paid once per four elements, not per element.
// With act >= 0 every element is first mapped to act(v*sc + sf): the plane is the input of a
// BatchNorm(+activation) whose output is never written out.
// `pre` (w % 4 == 0 only): the first four words of this thread, requested earlier with
// dw_stage_preload so that their latency overlaps the kernel's prologue.
struct DwPre { float4 v[4]; };
struct DwPreS { float v[4]; };  // the same for widths that are not multiples of four (4-byte words)
__device__ __forceinline__ void dw_stage_preload_s(DwPreS& pre, const float* __restrict__ src, int ne, int t, int tpp) {
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int e = t + u * tpp;
    pre.v[u] = e < ne ? src[e] : 0.f;
  }
}
__device__ __forceinline__ void dw_stage_preload(DwPre& pre, const float* __restrict__ src, int h, int w, int t,
                                                 int tpp) {
  const int nq = (h * w) >> 2;
  const float4* s4 = reinterpret_cast<const float4*>(src);
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int q = t + u * tpp;
    pre.v[u] = q < nq ? s4[q] : make_float4(0.f, 0.f, 0.f, 0.f);
  }
}
__device__ __forceinline__ void dw_stage_plane(float* dst, const float* __restrict__ src, int h, int w, int t,
                                               int tpp, float sc = 1.f, float sf = 0.f, int act = -1,
                                               const DwPre* pre = nullptr, const DwPreS* pres = nullptr) {
  const int pw = w + 2;
  if ((w & 3) == 0) {
    const int nq = (h * w) >> 2, qpr = w >> 2;
    const float4* s4 = reinterpret_cast<const float4*>(src);
    for (int q0 = t; q0 < nq; q0 += 4 * tpp) {
      float4 v[4];
      if (pre && q0 == t) {
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = pre->v[u];
      } else {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          int q = q0 + u * tpp;
          v[u] = q < nq ? s4[q] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        int q = q0 + u * tpp;
        if (q < nq) {
          int i = q / qpr, j = (q - i * qpr) * 4;
          float* d = dst + (i + 1) * pw + j + 1;
          if (act >= 0) {
            v[u].x = apply_act(v[u].x * sc + sf, act); v[u].y = apply_act(v[u].y * sc + sf, act);
            v[u].z = apply_act(v[u].z * sc + sf, act); v[u].w = apply_act(v[u].w * sc + sf, act);
          }
          d[0] = v[u].x; d[1] = v[u].y; d[2] = v[u].z; d[3] = v[u].w;
        }
      }
    }
  } else {
    const int ne = h * w;
    for (int e0 = t; e0 < ne; e0 += 4 * tpp) {
      float v[4];
      if (pres && e0 == t) {
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = pres->v[u];
      } else {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          int e = e0 + u * tpp;
          v[u] = e < ne ? src[e] : 0.f;
        }
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        int e = e0 + u * tpp;
        if (e < ne) {
          int i = e / w, j = e - i * w;
          dst[(i + 1) * pw + j + 1] = act >= 0 ? apply_act(v[u] * sc + sf, act) : v[u];
        }
      }
    }
  }
}

__global__ __launch_bounds__(256) void dw3x3_fwd_f32_kernel(const float* __restrict__ x,
                                                            const float* __restrict__ w,
                                                            float* __restrict__ y, DwGeom gm, DwBnIn bi, DwBnOut bo) {
  extern __shared__ float sm[];
  const int PW = gm.W + 2, PSZ = (gm.H + 2) * PW;
  float* sx = sm;
  float* sw = sm + gm.ppb * PSZ;   // [ppb][9]
  float* scoef = sw + gm.ppb * 9;  // [ppb][2] scale, shift of the input BatchNorm
  double* sred = reinterpret_cast<double*>(sm + ((gm.ppb * (PSZ + 11) + 1) & ~1));  // [4 waves][2]
  const int plane0 = blockIdx.x * gm.ppb;
  const int np = min(gm.ppb, gm.NC - plane0);
  const int tpp = 256 / gm.ppb;
  const int pl = threadIdx.x / tpp, t = threadIdx.x - pl * tpp;
  const bool live = pl < np;
  // the first words of the plane are requested before the prologue and the LDS clear
  const bool vecw = (gm.W & 3) == 0;
  DwPre pre;
  DwPreS pres;
  if (live && vecw) dw_stage_preload(pre, x + (size_t)(plane0 + pl) * gm.H * gm.W, gm.H, gm.W, t, tpp);
  if (live && !vecw) dw_stage_preload_s(pres, x + (size_t)(plane0 + pl) * gm.H * gm.W, gm.H * gm.W, t, tpp);
  if (bi.on) {  // finish the statistics of each plane's channel: one wavefront per plane
    for (int q = threadIdx.x >> 6; q < np; q += 4) {
      const int plane = plane0 + q, c = plane % gm.C;
      double s1, s2;
      bn_add_partials(bi.ws, c, bi.P, s1, s2);
      if ((threadIdx.x & 63) == 0)  // the sample-0 plane of a channel records its statistics
        bn_coefficients(s1, s2, bi.count, bi.gamma[c], bi.beta[c], bi.eps, c, gm.C, plane < gm.C, bi.stat, bi.ss,
                        bi.running, scoef[2 * q], scoef[2 * q + 1]);
    }
  }
  dw_zero(sx, gm.ppb * PSZ);  // ends with a barrier: the coefficients are visible
  if (live) {
    if (bi.on)
      dw_stage_plane(sx + pl * PSZ, x + (size_t)(plane0 + pl) * gm.H * gm.W, gm.H, gm.W, t, tpp, scoef[2 * pl],
                     scoef[2 * pl + 1], bi.act, vecw ? &pre : nullptr, vecw ? nullptr : &pres);
    else
      dw_stage_plane(sx + pl * PSZ, x + (size_t)(plane0 + pl) * gm.H * gm.W, gm.H, gm.W, t, tpp, 1.f, 0.f, -1,
                     vecw ? &pre : nullptr, vecw ? nullptr : &pres);
  }
  for (int i = threadIdx.x; i < np * 9; i += 256) sw[i] = w[((plane0 + i / 9) % gm.C) * 9 + i % 9];
  __syncthreads();
  float s1 = 0.f, s2 = 0.f;
  if (live) {
    const float* wc = sw + pl * 9;
    const float w0 = wc[0], w1 = wc[1], w2 = wc[2], w3 = wc[3], w4 = wc[4], w5 = wc[5], w6 = wc[6], w7 = wc[7], w8 = wc[8];
    const float* sp = sx + pl * PSZ;
    float* yp = y + (size_t)(plane0 + pl) * gm.Ho * gm.Wo;
    const int s = gm.stride;
    for (int o = t; o < gm.Ho * gm.Wo; o += tpp) {
      int i = o / gm.Wo, j = o - i * gm.Wo;
      const float* b = sp + (i * s) * PW + j * s;
      float acc = w0 * b[0] + w1 * b[1] + w2 * b[2];
      acc += w3 * b[PW] + w4 * b[PW + 1] + w5 * b[PW + 2];
      acc += w6 * b[2 * PW] + w7 * b[2 * PW + 1] + w8 * b[2 * PW + 2];
      yp[o] = acc;
      s1 += acc;
      s2 += acc * acc;
    }
  }
  if (!bo.on) return;  // uniform
  // per-plane (sum, sum of squares) of the output for the BatchNorm that follows: fp32 per
  // thread, fp64 across the tpp threads of the plane (tpp is a power of two >= 16)
  double d1 = (double)s1, d2 = (double)s2;
  const int span = tpp < 64 ? tpp : 64;
  d1 = row16_sum(d1);
  d2 = row16_sum(d2);
  for (int o = 16; o < span; o <<= 1) {  // across the rows of 16 lanes of a wider plane group
    d1 += __shfl_xor(d1, o, 64);
    d2 += __shfl_xor(d2, o, 64);
  }
  const int plane = plane0 + pl;
  const int N = gm.NC / gm.C;
  double* out = bo.ws + ((size_t)(plane % gm.C) * N + plane / gm.C) * 2;
  if (tpp <= 64) {
    if (live && t == 0) {
      out[0] = d1;
      out[1] = d2;
    }
  } else {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) {
      sred[2 * wave] = d1;
      sred[2 * wave + 1] = d2;
    }
    __syncthreads();
    if (live && t == 0) {
      const int w0i = threadIdx.x >> 6, nw = tpp >> 6;
      double a = 0.0, b = 0.0;
      for (int q = 0; q < nw; ++q) {
        a += sred[2 * (w0i + q)];
        b += sred[2 * (w0i + q) + 1];
      }
      out[0] = a;
      out[1] = b;
    }
  }
}

// BatchNorm backward folded into the load of the conv's upstream gradient (see DwBwdFuse)
struct DwBnBwd {
  float k, m1, m2, mean, istd, sc, sf;
  int act;
};
__device__ __forceinline__ float dw_bn_dx(float g, float y, const DwBnBwd& b) {
  return b.k * (g * act_mask(y * b.sc + b.sf, b.act) - b.m1 - (y - b.mean) * b.istd * b.m2);
}
// whole wavefront: finish the backward sums of channel c; with `record` lane 0 adds dbeta, dgamma
__device__ __forceinline__ DwBnBwd dw_bn_bwd_coef(const DwBwdFuse& f, int c, int C, bool record) {
  double s1, s2;
  bn_add_partials(f.ws_out, c, f.P_out, s1, s2);
  DwBnBwd b;
  b.mean = f.ystat[c]; b.istd = f.ystat[C + c]; b.sc = f.yss[c]; b.sf = f.yss[C + c];
  b.k = f.ygamma[c] * b.istd;
  b.m1 = (float)(s1 / f.ycount);
  b.m2 = (float)(s2 / f.ycount);
  b.act = f.yact;
  if (record && (threadIdx.x & 63) == 0) {
    f.Gbeta[c] += (float)s1;
    f.Ggamma[c] += (float)s2;
  }
  return b;
}

// Input gradient (if dx) and the nine weight-gradient sums of every plane:
//   dx[i][j] = sum_{u,v} w[u][v] g[(i+1-u)/s][(j+1-v)/s]   (terms with a non-integer index drop)
//   part[plane][u*3+v] = sum_{i,j} g[i][j] x[i*s-1+u][j*s-1+v]
__global__ __launch_bounds__(256) void dw3x3_bwd_f32_kernel(const float* __restrict__ g,
                                                            const float* __restrict__ x,
                                                            const float* __restrict__ w,
                                                            float* __restrict__ dx, float* __restrict__ part,
                                                            DwGeom gm, DwBwdFuse f) {
  extern __shared__ float sm[];
  const int PW = gm.W + 2, PSZ = (gm.H + 2) * PW;
  const int GW = gm.Wo + 2, GSZ = (gm.Ho + 2) * GW;
  float* sx = sm;
  float* sg = sx + gm.ppb * PSZ;
  float* sw = sg + gm.ppb * GSZ;   // [ppb][9]
  float* sred = sw + gm.ppb * 9;   // [4 waves][11]
  float* scoef = sred + 44;        // [ppb][3]: k, m1, m2 of the BatchNorm behind the conv
  const int plane0 = blockIdx.x * gm.ppb;
  const int np = min(gm.ppb, gm.NC - plane0);
  const int tpp = 256 / gm.ppb;
  const int pl = threadIdx.x / tpp, t = threadIdx.x - pl * tpp;
  const bool live = pl < np;
  // Widths that are not multiples of four (the usual case here): a thread's first four words of
  // x, g (and y) are requested before the prologue and the LDS clear; the thread that stages
  // element e also computes dx[e], so x is not read again for the sums of the BatchNorm in front.
  const bool vecw = (gm.W & 3) == 0, vecg = (gm.Wo & 3) == 0;
  DwPreS xpre{}, gpre{}, ypre{};
  if (live && !vecw) dw_stage_preload_s(xpre, x + (size_t)(plane0 + pl) * gm.H * gm.W, gm.H * gm.W, t, tpp);
  if (live && (f.y || !vecg)) {
    dw_stage_preload_s(gpre, g + (size_t)(plane0 + pl) * gm.Ho * gm.Wo, gm.Ho * gm.Wo, t, tpp);
    if (f.y) dw_stage_preload_s(ypre, f.y + (size_t)(plane0 + pl) * gm.Ho * gm.Wo, gm.Ho * gm.Wo, t, tpp);
  }
  if (f.y) {  // one wavefront per plane finishes the sums of the BatchNorm behind the conv
    for (int q = threadIdx.x >> 6; q < np; q += 4) {
      const DwBnBwd b = dw_bn_bwd_coef(f, (plane0 + q) % gm.C, gm.C, plane0 + q < gm.C);
      if ((threadIdx.x & 63) == 0) {
        scoef[3 * q] = b.k;
        scoef[3 * q + 1] = b.m1;
        scoef[3 * q + 2] = b.m2;
      }
    }
  }
  dw_zero(sx, gm.ppb * (PSZ + GSZ));  // sx and sg are adjacent; ends with a barrier
  const int ch = (plane0 + (live ? pl : 0)) % gm.C;
  if (live) {
    if (f.xss)  // x is the input of a BatchNorm(+activation) whose output the convolution saw
      dw_stage_plane(sx + pl * PSZ, x + (size_t)(plane0 + pl) * gm.H * gm.W, gm.H, gm.W, t, tpp, f.xss[ch],
                     f.xss[gm.C + ch], f.xact, nullptr, vecw ? nullptr : &xpre);
    else
      dw_stage_plane(sx + pl * PSZ, x + (size_t)(plane0 + pl) * gm.H * gm.W, gm.H, gm.W, t, tpp, 1.f, 0.f, -1, nullptr,
                     vecw ? nullptr : &xpre);
    if (f.y) {  // the conv's upstream gradient = input gradient of the BatchNorm behind it
      DwBnBwd b;
      b.k = scoef[3 * pl]; b.m1 = scoef[3 * pl + 1]; b.m2 = scoef[3 * pl + 2];
      b.mean = f.ystat[ch]; b.istd = f.ystat[gm.C + ch]; b.sc = f.yss[ch]; b.sf = f.yss[gm.C + ch]; b.act = f.yact;
      const float* gsrc = g + (size_t)(plane0 + pl) * gm.Ho * gm.Wo;
      const float* ysrc = f.y + (size_t)(plane0 + pl) * gm.Ho * gm.Wo;
      float* dst = sg + pl * GSZ;
      const int ne = gm.Ho * gm.Wo;
      for (int e0 = t; e0 < ne; e0 += 4 * tpp) {
        float gv[4], yv[4];
        if (e0 == t) {
#pragma unroll
          for (int u = 0; u < 4; ++u) { gv[u] = gpre.v[u]; yv[u] = ypre.v[u]; }
        } else {
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int e = e0 + u * tpp;
            gv[u] = e < ne ? gsrc[e] : 0.f;
            yv[u] = e < ne ? ysrc[e] : 0.f;
          }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int e = e0 + u * tpp;
          if (e < ne) {
            const int i = e / gm.Wo, jj = e - i * gm.Wo;
            dst[(i + 1) * GW + jj + 1] = dw_bn_dx(gv[u], yv[u], b);
          }
        }
      }
    } else {
      dw_stage_plane(sg + pl * GSZ, g + (size_t)(plane0 + pl) * gm.Ho * gm.Wo, gm.Ho, gm.Wo, t, tpp, 1.f, 0.f, -1, nullptr,
                     vecg ? nullptr : &gpre);
    }
  }
  for (int i = threadIdx.x; i < np * 9; i += 256) sw[i] = w[((plane0 + i / 9) % gm.C) * 9 + i % 9];
  __syncthreads();
  const int s = gm.stride;
  float acc[11];  // nine weight-gradient sums, then the two sums of the BatchNorm in front
#pragma unroll
  for (int k = 0; k < 11; ++k) acc[k] = 0.f;
  if (live) {
    const float* wc = sw + pl * 9;
    const float* gp = sg + pl * GSZ;
    const float* xp = sx + pl * PSZ;
    if (dx) {
      float* dp = dx + (size_t)(plane0 + pl) * gm.H * gm.W;
      const float* xraw = x + (size_t)(plane0 + pl) * gm.H * gm.W;
      const float mean1 = f.ws_in ? f.xstat[ch] : 0.f, istd1 = f.ws_in ? f.xstat[gm.C + ch] : 0.f;
      auto dx_at = [&](int e, float raw) {
        int i = e / gm.W, j = e - i * gm.W;
        float v = 0.f;
#pragma unroll
        for (int u = 0; u < 3; ++u) {
          int a = i + 1 - u;
          if (s == 2 && (a & 1)) continue;
          int io = s == 2 ? (a >> 1) : a;  // in [-1, Ho]: the halo holds zeros
#pragma unroll
          for (int v3 = 0; v3 < 3; ++v3) {
            int bb = j + 1 - v3;
            if (s == 2 && (bb & 1)) continue;
            int jo = s == 2 ? (bb >> 1) : bb;
            v += wc[u * 3 + v3] * gp[(io + 1) * GW + jo + 1];
          }
        }
        dp[e] = v;
        if (f.ws_in) {  // backward sums of the BatchNorm in front: g' = dx*act'(.), g'*xhat
          const float gmk = v * act_mask(xp[(i + 1) * PW + j + 1], f.xact);
          acc[9] += gmk;
          acc[10] += gmk * ((raw - mean1) * istd1);
        }
      };
      const int ne = gm.H * gm.W;
      int e = t;
      if (!vecw) {  // the first four elements of this thread: x is still in registers
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          if (t + u * tpp < ne) dx_at(t + u * tpp, xpre.v[u]);
        }
        e = t + 4 * tpp;
      }
      for (; e < ne; e += tpp) dx_at(e, f.ws_in ? xraw[e] : 0.f);
    }
    for (int o = t; o < gm.Ho * gm.Wo; o += tpp) {
      int i = o / gm.Wo, j = o - i * gm.Wo;
      float gv = gp[(i + 1) * GW + j + 1];
      const float* b = xp + (i * s) * PW + j * s;
#pragma unroll
      for (int u = 0; u < 3; ++u)
#pragma unroll
        for (int v3 = 0; v3 < 3; ++v3) acc[u * 3 + v3] += gv * b[u * PW + v3];
    }
  }
  // reduce the sums over the tpp threads of each plane (tpp is a power of two >= 16)
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int span = tpp < 64 ? tpp : 64;
#pragma unroll
  for (int k = 0; k < 11; ++k) {
    acc[k] = row16_sum(acc[k]);
    for (int o = 16; o < span; o <<= 1) acc[k] += __shfl_xor(acc[k], o, 64);  // across rows of 16 lanes
  }
  const int N = gm.NC / gm.C;
  double* bws = f.ws_in ? f.ws_in + ((size_t)ch * N + (plane0 + pl) / gm.C) * 2 : nullptr;
  if (tpp <= 64) {
    if (live && t == 0) {
#pragma unroll
      for (int k = 0; k < 9; ++k) part[(size_t)(plane0 + pl) * 9 + k] = acc[k];
      if (bws) {
        bws[0] = (double)acc[9];
        bws[1] = (double)acc[10];
      }
    }
  } else {
    if (lane == 0)
#pragma unroll
      for (int k = 0; k < 11; ++k) sred[wave * 11 + k] = acc[k];
    __syncthreads();
    if (live && t == 0) {
      const int w0 = threadIdx.x >> 6, nw = tpp >> 6;
      float v[11];
      for (int k = 0; k < 11; ++k) {
        v[k] = 0.f;
        for (int q = 0; q < nw; ++q) v[k] += sred[(w0 + q) * 11 + k];
      }
      for (int k = 0; k < 9; ++k) part[(size_t)(plane0 + pl) * 9 + k] = v[k];
      if (bws) {
        bws[0] = (double)v[9];
        bws[1] = (double)v[10];
      }
    }
  }
}

// ============================================================== depthwise, register windows
// Kernels without LDS for widths that are a multiple of the strip width VW (4, 2 or 1 pixels:
// 16-, 8- or 4-byte accesses) with at most 64 strips per row: one wavefront per (n, c) plane
// (or per band of rows of a plane).  Lane (s = l % SW, rg = l / SW) owns the VW-pixel column
// strip s (SW = W/VW strips per row) of the rows of row group rg and slides a three-row
// register window down them; the columns left and right of a strip come from the neighbouring
// lanes, zeros at the image border.  Rows travel as raw words (zeros where not readable), some
// steps ahead, and are only transformed when they enter the window, so a load is not waited
// for before the rows ahead of it are used up.  Sums stay in registers and are reduced over
// the wavefront at the end.
template <int VW> struct DwVec { float e[VW]; };
template <int VW>
__device__ __forceinline__ DwVec<VW> dw_zero_vec() {
  DwVec<VW> r;
#pragma unroll
  for (int j = 0; j < VW; ++j) r.e[j] = 0.f;
  return r;
}
template <int VW>
__device__ __forceinline__ DwVec<VW> dw_ldv(const float* __restrict__ p) {
  DwVec<VW> r;
  if constexpr (VW == 4) {
    const float4 t = *reinterpret_cast<const float4*>(p);
    r.e[0] = t.x; r.e[1] = t.y; r.e[2] = t.z; r.e[3] = t.w;
  } else if constexpr (VW == 2) {
    const float2 t = *reinterpret_cast<const float2*>(p);
    r.e[0] = t.x; r.e[1] = t.y;
  } else {
    r.e[0] = *p;
  }
  return r;
}
template <int VW>
__device__ __forceinline__ void dw_stv(float* __restrict__ p, const DwVec<VW>& v) {
  if constexpr (VW == 4) *reinterpret_cast<float4*>(p) = make_float4(v.e[0], v.e[1], v.e[2], v.e[3]);
  else if constexpr (VW == 2) *reinterpret_cast<float2*>(p) = make_float2(v.e[0], v.e[1]);
  else *p = v.e[0];
}
template <int VW>
__device__ __forceinline__ DwVec<VW> dw_norm(DwVec<VW> v, float sc, float sf, int act) {
#pragma unroll
  for (int j = 0; j < VW; ++j) v.e[j] = apply_act(v.e[j] * sc + sf, act);
  return v;
}
// a row of the window: v[0] = the column left of the strip, v[1..VW] = the strip, v[VW+1] = the
// column right of it
template <int VW> struct DwRow { float v[VW + 2]; };
template <int VW>
__device__ __forceinline__ DwRow<VW> dw_make_row(const DwVec<VW>& c, int s, int SW) {
  DwRow<VW> r;
  const float left = lane_up1(c.e[VW - 1]), right = lane_down1(c.e[0]);
  r.v[0] = s == 0 ? 0.f : left;
#pragma unroll
  for (int j = 0; j < VW; ++j) r.v[j + 1] = c.e[j];
  r.v[VW + 1] = s == SW - 1 ? 0.f : right;
  return r;
}

// Stride-1 backward: per row a lane issues one load of g, of x (and of y with a BatchNorm behind)
// and one store of dx.  D = rows requested ahead of the window.
template <int VW, int D>
__global__ __launch_bounds__(256) void dw3x3_bwd_s1_f32_kernel(const float* __restrict__ g,
                                                               const float* __restrict__ x,
                                                               const float* __restrict__ w, float* __restrict__ dx,
                                                               float* __restrict__ part, int NC, int C, int H,
                                                               int W, int RPG, DwBands bd, DwBwdFuse f) {
  typedef DwVec<VW> Vec;
  typedef DwRow<VW> Row;
  const int lane = threadIdx.x & 63;
  const int pb = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (pb >= NC * bd.bands) return;  // whole wavefront
  const int plane = pb / bd.bands, band = pb - plane * bd.bands;
  const int b0 = band * bd.rpb, b1 = min(b0 + bd.rpb, H);  // this wavefront's rows of the plane
  const int ch = plane % C;
  const int pidx = (plane / C) * bd.bands + band, nparts = (NC / C) * bd.bands;  // partial index, partials per channel
  const int SW = W / VW;
  const int rg = lane / SW, s = lane - rg * SW;
  const int r0 = b0 + rg * RPG;
  const int r1 = min(r0 + RPG, b1);  // lanes past the last group: r0 >= b1, no rows
  const float* gp = g + (size_t)plane * H * W + VW * s;
  const float* xp = x + (size_t)plane * H * W + VW * s;
  const float* yp = f.y ? f.y + (size_t)plane * H * W + VW * s : nullptr;
  float* dp = dx ? dx + (size_t)plane * H * W + VW * s : nullptr;
  float wk[9];
  const float* wc = w + (size_t)ch * 9;
#pragma unroll
  for (int k = 0; k < 9; ++k) wk[k] = wc[k];
  DwBnBwd yb{};
  // a row is readable by this lane if it lies in the image and the lane has rows at all
  const bool has = r0 < b1;
  auto rowok = [&](int row, bool ok) -> bool { return ok && has && row >= 0 && row < H; };
  struct Pend { Vec g, y, x; };
  auto load_row = [&](int row, bool ok) -> Pend {
    Pend q;
    q.g = q.y = q.x = dw_zero_vec<VW>();
    if (rowok(row, ok)) {
      q.g = dw_ldv<VW>(gp + (size_t)row * W);
      if (f.y) q.y = dw_ldv<VW>(yp + (size_t)row * W);
      q.x = dw_ldv<VW>(xp + (size_t)row * W);
    }
    return q;
  };
  auto use_g = [&](const Pend& q, bool valid) -> Vec {
    Vec gv = q.g;
    if (f.y && valid) {  // input gradient of the BatchNorm behind the conv
#pragma unroll
      for (int j = 0; j < VW; ++j) gv.e[j] = dw_bn_dx(gv.e[j], q.y.e[j], yb);
    }
    return gv;
  };
  // with xss the convolution's input was act(x*scale + shift) (a BatchNorm whose output is not
  // kept); the padding around it stays zero
  const float xsc = f.xss ? f.xss[ch] : 1.f, xsf = f.xss ? f.xss[C + ch] : 0.f;
  const float mean1 = f.ws_in ? f.xstat[ch] : 0.f, istd1 = f.ws_in ? f.xstat[C + ch] : 0.f;
  auto use_x = [&](const Pend& q, bool valid) -> Vec {
    return (f.xss && valid) ? dw_norm<VW>(q.x, xsc, xsf, f.xact) : q.x;
  };
  // the first rows are requested before the BatchNorm sums are finished
  const Pend pm = load_row(r0 - 1, true), pc = load_row(r0, true);
  Pend pn[D];
  pn[0] = load_row(r0 + 1, true);
#pragma unroll
  for (int d = 1; d < D; ++d) pn[d] = load_row(r0 + 1 + d, r0 + 1 + d <= r1);
  if (f.y) yb = dw_bn_bwd_coef(f, ch, C, plane < C && band == 0);
  Row gm = dw_make_row<VW>(use_g(pm, rowok(r0 - 1, true)), s, SW);
  Row gc = dw_make_row<VW>(use_g(pc, rowok(r0, true)), s, SW);
  Row xm = dw_make_row<VW>(use_x(pm, rowok(r0 - 1, true)), s, SW);
  Row xc = dw_make_row<VW>(use_x(pc, rowok(r0, true)), s, SW);
  Vec xcr = pc.x;
  float acc[9];
#pragma unroll
  for (int k = 0; k < 9; ++k) acc[k] = 0.f;
  float bs1 = 0.f, bs2 = 0.f;
  for (int i = 0; i < RPG; ++i) {  // uniform trip count: the lane exchanges need every lane
    const int a = r0 + i;
    // past its last row a lane must not see the next group's rows as its own window
    const bool v1 = rowok(a + 1, a + 1 <= r1);
    const Row gq = dw_make_row<VW>(use_g(pn[0], v1), s, SW), xq = dw_make_row<VW>(use_x(pn[0], v1), s, SW);
    const Vec xqr = pn[0].x;
#pragma unroll
    for (int d = 0; d + 1 < D; ++d) pn[d] = pn[d + 1];
    pn[D - 1] = load_row(a + 1 + D, a + 1 + D <= r1);
    if (a < r1) {
      if (dp) {
        Vec o;
#pragma unroll
        for (int j = 0; j < VW; ++j) {
          float v = 0.f;
#pragma unroll
          for (int q = 0; q < 3; ++q) {  // dx[a][b] = sum_{u,q} w[u][q] g[a-u+1][b-q+1]
            v += wk[0 * 3 + q] * gq.v[j + 2 - q];
            v += wk[1 * 3 + q] * gc.v[j + 2 - q];
            v += wk[2 * 3 + q] * gm.v[j + 2 - q];
          }
          o.e[j] = v;
        }
        dw_stv<VW>(dp + (size_t)a * W, o);
        if (f.ws_in) {  // backward sums of the BatchNorm in front: g' = dx*act'(.), g'*xhat
#pragma unroll
          for (int j = 0; j < VW; ++j) {
            const float gmk = o.e[j] * act_mask(xc.v[j + 1], f.xact);
            bs1 += gmk;
            bs2 += gmk * ((xcr.e[j] - mean1) * istd1);
          }
        }
      }
#pragma unroll
      for (int j = 0; j < VW; ++j) {  // dW[u][q] += g[a][b] x[a+u-1][b+q-1]
        const float gv = gc.v[j + 1];
#pragma unroll
        for (int q = 0; q < 3; ++q) {
          acc[0 * 3 + q] += gv * xm.v[j + q];
          acc[1 * 3 + q] += gv * xc.v[j + q];
          acc[2 * 3 + q] += gv * xq.v[j + q];
        }
      }
    }
    gm = gc; gc = gq;
    xm = xc; xc = xq;
    xcr = xqr;
  }
#pragma unroll
  for (int k = 0; k < 9; ++k) acc[k] = wave_sum(acc[k]);
  if (lane == 0)
#pragma unroll
    for (int k = 0; k < 9; ++k) part[((size_t)pidx * C + ch) * 9 + k] = acc[k];
  if (f.ws_in) {
    const double d1 = wave_sum_d((double)bs1), d2 = wave_sum_d((double)bs2);
    if (lane == 0) {
      double* o = f.ws_in + ((size_t)ch * nparts + pidx) * 2;
      o[0] = d1;
      o[1] = d2;
    }
  }
}

// Stride-2 counterpart (VW = 4 or 2, H even): lane (s, rg) owns input columns VW*s .. VW*s+VW-1
// = output columns (VW/2)*s .., and per step one output row i = two input rows 2i, 2i+1.
// y[i][j] = sum_{u,q} w[u][q] x[2i+u-1][2j+q-1], so an even input row/column meets only the
// centre tap and an odd one the two outer taps of the neighbouring outputs.
template <int VW> struct DwG2 { float v[VW / 2 + 1]; };  // the strip's output columns and the one right of them
template <int VW> struct DwX2 { float v[VW + 1]; };      // the input column left of the strip, then the strip
template <int VW>
__device__ __forceinline__ DwG2<VW> dw_make_g2(const DwVec<VW / 2>& c, int s, int SW) {
  DwG2<VW> r;
  const float right = lane_down1(c.e[0]);
#pragma unroll
  for (int j = 0; j < VW / 2; ++j) r.v[j] = c.e[j];
  r.v[VW / 2] = s == SW - 1 ? 0.f : right;
  return r;
}
template <int VW>
__device__ __forceinline__ DwX2<VW> dw_make_x2(const DwVec<VW>& c, int s) {
  DwX2<VW> r;
  const float left = lane_up1(c.e[VW - 1]);
  r.v[0] = s == 0 ? 0.f : left;
#pragma unroll
  for (int j = 0; j < VW; ++j) r.v[j + 1] = c.e[j];
  return r;
}
// one input row of dx from the output-gradient rows that reach it through kernel rows wa / wb:
// an even input column c meets the centre tap of output column c/2, an odd one the outer taps
// of output columns (c-1)/2 and (c+1)/2
template <int VW>
__device__ __forceinline__ DwVec<VW> dw_dx_row2(const float* wa, const DwG2<VW>& ga, const float* wb,
                                                const DwG2<VW>& gb, bool two) {
  DwVec<VW> o;
#pragma unroll
  for (int c = 0; c < VW; ++c) {
    if (c % 2 == 0) o.e[c] = wa[1] * ga.v[c / 2];
    else o.e[c] = wa[0] * ga.v[(c + 1) / 2] + wa[2] * ga.v[(c - 1) / 2];
  }
  if (two) {
#pragma unroll
    for (int c = 0; c < VW; ++c) {
      if (c % 2 == 0) o.e[c] += wb[1] * gb.v[c / 2];
      else o.e[c] += wb[0] * gb.v[(c + 1) / 2] + wb[2] * gb.v[(c - 1) / 2];
    }
  }
  return o;
}
template <int VW>
__global__ __launch_bounds__(256) void dw3x3_bwd_s2_f32_kernel(const float* __restrict__ g,
                                                               const float* __restrict__ x,
                                                               const float* __restrict__ w, float* __restrict__ dx,
                                                               float* __restrict__ part, int NC, int C, int H,
                                                               int W, int RPG, DwBands bd, DwBwdFuse f) {
  constexpr int VG = VW / 2;  // output columns per lane
  typedef DwVec<VW> Vec;
  typedef DwVec<VG> VecG;
  const int lane = threadIdx.x & 63;
  const int pb = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (pb >= NC * bd.bands) return;  // whole wavefront
  const int plane = pb / bd.bands, band = pb - plane * bd.bands;
  const int ch = plane % C;
  const int pidx = (plane / C) * bd.bands + band, nparts = (NC / C) * bd.bands;  // partial index, partials per channel
  const int SW = W / VW, Ho = H >> 1, Wo = W >> 1;
  const int b0 = band * bd.rpb, b1 = min(b0 + bd.rpb, Ho);  // this wavefront's output rows
  const int rg = lane / SW, s = lane - rg * SW;
  const int r0 = b0 + rg * RPG;       // output rows [r0, r1)
  const int r1 = min(r0 + RPG, b1);
  const bool has = r0 < b1;
  const float* gp = g + (size_t)plane * Ho * Wo + VG * s;
  const float* yp = f.y ? f.y + (size_t)plane * Ho * Wo + VG * s : nullptr;
  const float* xp = x + (size_t)plane * H * W + VW * s;
  float* dp = dx ? dx + (size_t)plane * H * W + VW * s : nullptr;
  float wk[9];
  const float* wc = w + (size_t)ch * 9;
#pragma unroll
  for (int k = 0; k < 9; ++k) wk[k] = wc[k];
  DwBnBwd yb{};
  const float xsc = f.xss ? f.xss[ch] : 1.f, xsf = f.xss ? f.xss[C + ch] : 0.f;
  const float mean1 = f.ws_in ? f.xstat[ch] : 0.f, istd1 = f.ws_in ? f.xstat[C + ch] : 0.f;
  auto xok = [&](int row, bool ok) -> bool { return ok && has && row >= 0 && row < H; };
  auto gok = [&](int row, bool ok) -> bool { return ok && has && row >= 0 && row < Ho; };
  // the words of a step: input rows 2i, 2i+1, gradient row i+1
  struct Pend { Vec x0, x1; VecG g, y; };
  auto load_step = [&](int i, bool ok) -> Pend {
    Pend q;
    q.x0 = q.x1 = dw_zero_vec<VW>();
    q.g = q.y = dw_zero_vec<VG>();
    if (xok(2 * i, ok)) q.x0 = dw_ldv<VW>(xp + (size_t)(2 * i) * W);
    if (xok(2 * i + 1, ok)) q.x1 = dw_ldv<VW>(xp + (size_t)(2 * i + 1) * W);
    if (gok(i + 1, ok)) {
      q.g = dw_ldv<VG>(gp + (size_t)(i + 1) * Wo);
      if (f.y) q.y = dw_ldv<VG>(yp + (size_t)(i + 1) * Wo);
    }
    return q;
  };
  auto use_g = [&](VecG gv, const VecG& yv, bool valid) -> VecG {
    if (f.y && valid) {  // input gradient of the BatchNorm behind the conv
#pragma unroll
      for (int j = 0; j < VG; ++j) gv.e[j] = dw_bn_dx(gv.e[j], yv.e[j], yb);
    }
    return gv;
  };
  // with xss: the BatchNorm(+activation) output the convolution saw; the padding stays zero
  auto use_x = [&](const Vec& raw, bool valid) -> Vec {
    return (f.xss && valid) ? dw_norm<VW>(raw, xsc, xsf, f.xact) : raw;
  };
  // the first rows are requested before the BatchNorm sums are finished
  Vec xm_raw = dw_zero_vec<VW>();
  VecG gc_raw = dw_zero_vec<VG>(), yc_raw = dw_zero_vec<VG>();
  if (xok(2 * r0 - 1, true)) xm_raw = dw_ldv<VW>(xp + (size_t)(2 * r0 - 1) * W);
  if (gok(r0, true)) {
    gc_raw = dw_ldv<VG>(gp + (size_t)r0 * Wo);
    if (f.y) yc_raw = dw_ldv<VG>(yp + (size_t)r0 * Wo);
  }
  Pend p1 = load_step(r0, true), p2 = load_step(r0 + 1, r0 + 1 < r1);
  if (f.y) yb = dw_bn_bwd_coef(f, ch, C, plane < C && band == 0);
  DwX2<VW> xm = dw_make_x2<VW>(use_x(xm_raw, xok(2 * r0 - 1, true)), s);
  DwG2<VW> gc = dw_make_g2<VW>(use_g(gc_raw, yc_raw, gok(r0, true)), s, SW);
  float acc[9];
#pragma unroll
  for (int k = 0; k < 9; ++k) acc[k] = 0.f;
  float bs1 = 0.f, bs2 = 0.f;
  for (int it = 0; it < RPG; ++it) {  // uniform trip count: the lane exchanges need every lane
    const int i = r0 + it;
    const bool ok = it == 0 || i < r1;  // a lane must not see the next group's rows as its own
    const DwX2<VW> x0 = dw_make_x2<VW>(use_x(p1.x0, xok(2 * i, ok)), s);
    const DwX2<VW> x1 = dw_make_x2<VW>(use_x(p1.x1, xok(2 * i + 1, ok)), s);
    const Vec x0r = p1.x0, x1r = p1.x1;
    const DwG2<VW> gq = dw_make_g2<VW>(use_g(p1.g, p1.y, gok(i + 1, ok)), s, SW);
    p1 = p2;
    p2 = load_step(i + 2, i + 2 < r1);
    if (i < r1) {
      if (dp) {
        // input row 2i: centre kernel row of output row i; row 2i+1: kernel row 0 of output
        // row i+1 and kernel row 2 of output row i
        const Vec d0 = dw_dx_row2<VW>(wk + 3, gc, wk + 3, gc, false);
        const Vec d1 = dw_dx_row2<VW>(wk + 0, gq, wk + 6, gc, true);
        dw_stv<VW>(dp + (size_t)(2 * i) * W, d0);
        dw_stv<VW>(dp + (size_t)(2 * i + 1) * W, d1);
        if (f.ws_in) {  // backward sums of the BatchNorm in front: g' = dx*act'(.), g'*xhat
#pragma unroll
          for (int j = 0; j < VW; ++j) {
            const float g0 = d0.e[j] * act_mask(x0.v[j + 1], f.xact), g1 = d1.e[j] * act_mask(x1.v[j + 1], f.xact);
            bs1 += g0 + g1;
            bs2 += g0 * ((x0r.e[j] - mean1) * istd1) + g1 * ((x1r.e[j] - mean1) * istd1);
          }
        }
      }
#pragma unroll
      for (int j = 0; j < VG; ++j) {  // dW[u][q] += g[i][j'] x[2i+u-1][2j'+q-1]
        const float gv = gc.v[j];
#pragma unroll
        for (int q = 0; q < 3; ++q) {
          acc[0 * 3 + q] += gv * xm.v[2 * j + q];
          acc[1 * 3 + q] += gv * x0.v[2 * j + q];
          acc[2 * 3 + q] += gv * x1.v[2 * j + q];
        }
      }
    }
    xm = x1;
    gc = gq;
  }
#pragma unroll
  for (int k = 0; k < 9; ++k) acc[k] = wave_sum(acc[k]);
  if (lane == 0)
#pragma unroll
    for (int k = 0; k < 9; ++k) part[((size_t)pidx * C + ch) * 9 + k] = acc[k];
  if (f.ws_in) {
    const double d1 = wave_sum_d((double)bs1), d2 = wave_sum_d((double)bs2);
    if (lane == 0) {
      double* o = f.ws_in + ((size_t)ch * nparts + pidx) * 2;
      o[0] = d1;
      o[1] = d2;
    }
  }
}

// Forward, the same lane layout: one load and one store per lane and row (stride 2: two loads,
// one half-width store); with a BatchNorm in front rows are normalised when they enter the
// window (padding stays zero).
template <int VW, int D>  // D = rows requested ahead of the window
__global__ __launch_bounds__(256) void dw3x3_fwd_s1_f32_kernel(const float* __restrict__ x,
                                                               const float* __restrict__ w, float* __restrict__ y,
                                                               int NC, int C, int H, int W, int RPG, DwBands bd,
                                                               DwBnIn bi, DwBnOut bo) {
  typedef DwVec<VW> Vec;
  typedef DwRow<VW> Row;
  const int lane = threadIdx.x & 63;
  const int pb = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (pb >= NC * bd.bands) return;  // whole wavefront
  const int plane = pb / bd.bands, band = pb - plane * bd.bands;
  const int b0 = band * bd.rpb, b1 = min(b0 + bd.rpb, H);  // this wavefront's rows of the plane
  const int ch = plane % C;
  const int pidx = (plane / C) * bd.bands + band, nparts = (NC / C) * bd.bands;  // partial index, partials per channel
  const int SW = W / VW;
  const int rg = lane / SW, s = lane - rg * SW;
  const int r0 = b0 + rg * RPG;
  const int r1 = min(r0 + RPG, b1);  // lanes past the last group: r0 >= b1, no rows
  const bool has = r0 < b1;
  const float* xp = x + (size_t)plane * H * W + VW * s;
  float* yp = y + (size_t)plane * H * W + VW * s;
  float wk[9];
  const float* wc = w + (size_t)ch * 9;
#pragma unroll
  for (int k = 0; k < 9; ++k) wk[k] = wc[k];
  auto rowok = [&](int row, bool ok) -> bool { return ok && has && row >= 0 && row < H; };
  auto load_row = [&](int row, bool ok) -> Vec {
    Vec v = dw_zero_vec<VW>();
    if (rowok(row, ok)) v = dw_ldv<VW>(xp + (size_t)row * W);
    return v;
  };
  // the first rows are requested before the statistics of the BatchNorm in front are finished
  const Vec pm = load_row(r0 - 1, true), pc = load_row(r0, true);
  Vec pn[D];
  pn[0] = load_row(r0 + 1, true);
#pragma unroll
  for (int d = 1; d < D; ++d) pn[d] = load_row(r0 + 1 + d, r0 + 1 + d <= r1);
  float sc = 1.f, sf = 0.f;
  if (bi.on) {  // every lane computes the same coefficients; lane 0 of a sample-0 plane records them
    double s1, s2;
    bn_add_partials(bi.ws, ch, bi.P, s1, s2);
    bn_coefficients(s1, s2, bi.count, bi.gamma[ch], bi.beta[ch], bi.eps, ch, C, plane < C && band == 0 && lane == 0,
                    bi.stat, bi.ss, bi.running, sc, sf);
  }
  auto use_x = [&](const Vec& raw, bool valid) -> Vec {
    return (bi.on && valid) ? dw_norm<VW>(raw, sc, sf, bi.act) : raw;
  };
  Row xm = dw_make_row<VW>(use_x(pm, rowok(r0 - 1, true)), s, SW);
  Row xc = dw_make_row<VW>(use_x(pc, rowok(r0, true)), s, SW);
  float t1 = 0.f, t2 = 0.f;
  for (int i = 0; i < RPG; ++i) {  // uniform trip count: the lane exchanges need every lane
    const int a = r0 + i;
    // past its last row a lane must not see the next group's rows as its own window
    const Row xq = dw_make_row<VW>(use_x(pn[0], rowok(a + 1, a + 1 <= r1)), s, SW);
#pragma unroll
    for (int d = 0; d + 1 < D; ++d) pn[d] = pn[d + 1];
    pn[D - 1] = load_row(a + 1 + D, a + 1 + D <= r1);
    if (a < r1) {
      Vec o;
#pragma unroll
      for (int j = 0; j < VW; ++j) {  // y[a][b] = sum_{u,q} w[u][q] x[a+u-1][b+q-1]
        float v = 0.f;
#pragma unroll
        for (int q = 0; q < 3; ++q) {
          v += wk[0 * 3 + q] * xm.v[j + q];
          v += wk[1 * 3 + q] * xc.v[j + q];
          v += wk[2 * 3 + q] * xq.v[j + q];
        }
        o.e[j] = v;
        t1 += v;
        t2 += v * v;
      }
      dw_stv<VW>(yp + (size_t)a * W, o);
    }
    xm = xc;
    xc = xq;
  }
  if (bo.on) {  // (sum, sum of squares) of this wavefront's rows for the BatchNorm behind
    const double d1 = wave_sum_d((double)t1), d2 = wave_sum_d((double)t2);
    if (lane == 0) {
      double* o = bo.ws + ((size_t)ch * nparts + pidx) * 2;
      o[0] = d1;
      o[1] = d2;
    }
  }
}

// stride 2 (VW = 4 or 2, H even): per step one output row i = input rows 2i, 2i+1 (row 2i-1 is
// carried over)
template <int VW>
__global__ __launch_bounds__(256) void dw3x3_fwd_s2_f32_kernel(const float* __restrict__ x,
                                                               const float* __restrict__ w, float* __restrict__ y,
                                                               int NC, int C, int H, int W, int RPG, DwBands bd,
                                                               DwBnIn bi, DwBnOut bo) {
  constexpr int VG = VW / 2;  // output columns per lane
  typedef DwVec<VW> Vec;
  const int lane = threadIdx.x & 63;
  const int pb = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (pb >= NC * bd.bands) return;  // whole wavefront
  const int plane = pb / bd.bands, band = pb - plane * bd.bands;
  const int ch = plane % C;
  const int pidx = (plane / C) * bd.bands + band, nparts = (NC / C) * bd.bands;  // partial index, partials per channel
  const int SW = W / VW, Ho = H >> 1, Wo = W >> 1;
  const int b0 = band * bd.rpb, b1 = min(b0 + bd.rpb, Ho);  // this wavefront's output rows
  const int rg = lane / SW, s = lane - rg * SW;
  const int r0 = b0 + rg * RPG;  // output rows [r0, r1)
  const int r1 = min(r0 + RPG, b1);
  const bool has = r0 < b1;
  const float* xp = x + (size_t)plane * H * W + VW * s;
  float* yp = y + (size_t)plane * Ho * Wo + VG * s;
  float wk[9];
  const float* wc = w + (size_t)ch * 9;
#pragma unroll
  for (int k = 0; k < 9; ++k) wk[k] = wc[k];
  auto rowok = [&](int row, bool ok) -> bool { return ok && has && row >= 0 && row < H; };
  auto load_row = [&](int row, bool ok) -> Vec {
    Vec v = dw_zero_vec<VW>();
    if (rowok(row, ok)) v = dw_ldv<VW>(xp + (size_t)row * W);
    return v;
  };
  const Vec pm = load_row(2 * r0 - 1, true);
  Vec p1a = load_row(2 * r0, true), p1b = load_row(2 * r0 + 1, true);
  Vec p2a = load_row(2 * r0 + 2, r0 + 1 < r1), p2b = load_row(2 * r0 + 3, r0 + 1 < r1);
  float sc = 1.f, sf = 0.f;
  if (bi.on) {
    double s1, s2;
    bn_add_partials(bi.ws, ch, bi.P, s1, s2);
    bn_coefficients(s1, s2, bi.count, bi.gamma[ch], bi.beta[ch], bi.eps, ch, C, plane < C && band == 0 && lane == 0,
                    bi.stat, bi.ss, bi.running, sc, sf);
  }
  auto use_x = [&](const Vec& raw, bool valid) -> Vec {
    return (bi.on && valid) ? dw_norm<VW>(raw, sc, sf, bi.act) : raw;
  };
  DwX2<VW> xm = dw_make_x2<VW>(use_x(pm, rowok(2 * r0 - 1, true)), s);
  float t1 = 0.f, t2 = 0.f;
  for (int it = 0; it < RPG; ++it) {  // uniform trip count: the lane exchanges need every lane
    const int i = r0 + it;
    const bool ok = it == 0 || i < r1;  // a lane must not see the next group's rows as its own
    const DwX2<VW> x0 = dw_make_x2<VW>(use_x(p1a, rowok(2 * i, ok)), s);
    const DwX2<VW> x1 = dw_make_x2<VW>(use_x(p1b, rowok(2 * i + 1, ok)), s);
    p1a = p2a;
    p1b = p2b;
    p2a = load_row(2 * i + 4, i + 2 < r1);
    p2b = load_row(2 * i + 5, i + 2 < r1);
    if (i < r1) {
      DwVec<VG> o;
#pragma unroll
      for (int j = 0; j < VG; ++j) {  // y[i][j'] = sum_{u,q} w[u][q] x[2i+u-1][2j'+q-1]
        float v = 0.f;
#pragma unroll
        for (int q = 0; q < 3; ++q) {
          v += wk[0 * 3 + q] * xm.v[2 * j + q];
          v += wk[1 * 3 + q] * x0.v[2 * j + q];
          v += wk[2 * 3 + q] * x1.v[2 * j + q];
        }
        o.e[j] = v;
        t1 += v;
        t2 += v * v;
      }
      dw_stv<VG>(yp + (size_t)i * Wo, o);
    }
    xm = x1;
  }
  if (bo.on) {
    const double d1 = wave_sum_d((double)t1), d2 = wave_sum_d((double)t2);
    if (lane == 0) {
      double* o = bo.ws + ((size_t)ch * nparts + pidx) * 2;
      o[0] = d1;
      o[1] = d2;
    }
  }
}

// G[c][t] += sum_n part[n][c][t]: eight sample lanes per output, fixed butterfly order
__global__ __launch_bounds__(256) void dw3x3_wgrad_final_kernel(const float* __restrict__ part,
                                                                float* __restrict__ G, int N, int C) {
  const int i = blockIdx.x * 32 + (threadIdx.x >> 3), nl = threadIdx.x & 7;
  float s = 0.f;
  if (i < C * 9)
    for (int n = nl; n < N; n += 8) s += part[(size_t)n * C * 9 + i];
  s = group8_sum(s);
  if (nl == 0 && i < C * 9) G[i] += s;
}

// The register-window kernels give a plane to one wavefront, or to several (each a band of
// rows) while there are too few planes to fill the chip; every wavefront leaves its own partial
// sums, so a channel has dw3x3_parts() partials instead of N.
// strip width of the register-window kernels for a shape: the widest of 4, 2, 1 pixels that
// divides W with at most 64 strips per row (stride 2: even H and W); 0 = LDS kernels
static int dw_vw(int H, int W, int stride) {
  if (stride == 2 && (H % 2 || W % 2)) return 0;
  if (stride != 1 && stride != 2) return 0;
  if (W % 4 == 0 && W / 4 <= 64) return 4;
  if (W % 2 == 0 && W / 2 <= 64) return 2;
  if (stride == 1 && W <= 64) return 1;
  return 0;
}
static DwBands dw_bands(int N, int C, int H, int W, int stride) {
  DwBands b{1, stride == 1 ? H : H / 2};
  const int vw = dw_vw(H, W, stride);
  if (!vw) return b;
  const int rows = b.rpb, groups = 64 / (W / vw);
  const long want = (4096 + (long)N * C - 1) / ((long)N * C);  // wavefronts wanted per plane
  const int cap = rows / (2 * groups) > 1 ? rows / (2 * groups) : 1;  // at least two rows per lane group
  int bands = (int)(want < cap ? want : cap);
  if (bands < 1) bands = 1;
  b.rpb = cdiv(rows, bands);
  b.bands = cdiv(rows, b.rpb);
  return b;
}
int dw3x3_parts(int N, int C, int H, int W, int stride) { return N * dw_bands(N, C, H, W, stride).bands; }
// Shapes the depthwise kernels cover: every shape with register windows; otherwise one padded
// plane of x and of g must fit the LDS kernels' 160 KB
bool dw3x3_supported(int H, int W, int stride) {
  if (stride != 1 && stride != 2) return false;
  if (dw_vw(H, W, stride)) return true;
  const long Ho = conv_out(H, 3, stride, 1), Wo = conv_out(W, 3, stride, 1);
  return ((long)(H + 2) * (W + 2) + (Ho + 2) * (Wo + 2) + 64) * 4 <= 150 * 1024;
}

static DwGeom dw_geom(int N, int C, int H, int W, int stride) {
  DwGeom gm;
  gm.C = C; gm.H = H; gm.W = W; gm.stride = stride;
  gm.Ho = conv_out(H, 3, stride, 1); gm.Wo = conv_out(W, 3, stride, 1);
  gm.NC = N * C;
  gm.ppb = dw_ppb(H, W, gm.NC);
  return gm;
}

void dw3x3_fwd_f32(hipStream_t st, const float* x, const float* w, float* y, int N, int C, int H, int W,
                   int stride, const DwBnIn* bn_in, double* stats_out) {
  DwBnIn bi{};
  if (bn_in) bi = *bn_in;
  DwBnOut bo{stats_out, stats_out != nullptr};
  if (const int vw = dw_vw(H, W, stride)) {
    const DwBands bd = dw_bands(N, C, H, W, stride);
    const int groups = 64 / (W / vw);
    const int rpg = cdiv(bd.rpb, groups);
    const dim3 grid(cdiv((long)N * C * bd.bands, 4));
#define DW_FWD(name, kern) KLAUNCH_NAMED(name, kern, grid, dim3(256), 0, st, x, w, y, N * C, C, H, W, rpg, bd, bi, bo)
    if (stride == 2) {
      if (vw == 4) DW_FWD("dw3x3_fwd_s2_f32_kernel<w4>", (dw3x3_fwd_s2_f32_kernel<4>));
      else DW_FWD("dw3x3_fwd_s2_f32_kernel<w2>", (dw3x3_fwd_s2_f32_kernel<2>));
    } else if (rpg <= 4) {  // short row groups: every row of a lane is requested up front
      if (vw == 4) DW_FWD("dw3x3_fwd_s1_f32_kernel<w4,4>", (dw3x3_fwd_s1_f32_kernel<4, 4>));
      else if (vw == 2) DW_FWD("dw3x3_fwd_s1_f32_kernel<w2,4>", (dw3x3_fwd_s1_f32_kernel<2, 4>));
      else DW_FWD("dw3x3_fwd_s1_f32_kernel<w1,4>", (dw3x3_fwd_s1_f32_kernel<1, 4>));
    } else {
      if (vw == 4) DW_FWD("dw3x3_fwd_s1_f32_kernel<w4,2>", (dw3x3_fwd_s1_f32_kernel<4, 2>));
      else if (vw == 2) DW_FWD("dw3x3_fwd_s1_f32_kernel<w2,2>", (dw3x3_fwd_s1_f32_kernel<2, 2>));
      else DW_FWD("dw3x3_fwd_s1_f32_kernel<w1,2>", (dw3x3_fwd_s1_f32_kernel<1, 2>));
    }
#undef DW_FWD
    return;
  }
  DwGeom gm = dw_geom(N, C, H, W, stride);
  // planes, weights, coefficients; then (8-byte aligned) four pairs of doubles
  size_t lds = ((((size_t)gm.ppb * ((H + 2) * (W + 2) + 11)) + 1) & ~(size_t)1) * sizeof(float) + 8 * sizeof(double);
  (void)hipFuncSetAttribute((const void*)dw3x3_fwd_f32_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  KLAUNCH(dw3x3_fwd_f32_kernel, dim3(cdiv(gm.NC, gm.ppb)), dim3(256), lds, st, x, w, y, gm, bi, bo);
}
size_t dw3x3_bwd_f32_ws(int N, int C, int H, int W, int stride) {
  return (size_t)dw3x3_parts(N, C, H, W, stride) * C * 9;
}
void dw3x3_bwd_f32(hipStream_t st, const float* g, const float* x, const float* w, float* dx, float* part,
                   float* G, int N, int C, int H, int W, int stride, const DwBwdFuse* fuse) {
  DwBwdFuse f;
  if (fuse) f = *fuse;
  if (!dx || !f.xss) f.ws_in = nullptr;  // those sums need dx and the normalised input
  if (const int vw = dw_vw(H, W, stride)) {
    const DwBands bd = dw_bands(N, C, H, W, stride);
    const int groups = 64 / (W / vw);
    const int rpg = cdiv(bd.rpb, groups);
    const dim3 grid(cdiv((long)N * C * bd.bands, 4));
#define DW_BWD(name, kern) KLAUNCH_NAMED(name, kern, grid, dim3(256), 0, st, g, x, w, dx, part, N * C, C, H, W, rpg, bd, f)
    // stride 1: two rows ahead; four cost a wavefront of occupancy at 16-byte strips (three tensors
    // per row) and measured slower there; narrow strips have the registers for it
    if (stride == 1) {
      if (vw == 4) DW_BWD("dw3x3_bwd_s1_f32_kernel<w4>", (dw3x3_bwd_s1_f32_kernel<4, 2>));
      else if (vw == 2) DW_BWD("dw3x3_bwd_s1_f32_kernel<w2>", (dw3x3_bwd_s1_f32_kernel<2, 4>));
      else DW_BWD("dw3x3_bwd_s1_f32_kernel<w1>", (dw3x3_bwd_s1_f32_kernel<1, 4>));
    } else {
      if (vw == 4) DW_BWD("dw3x3_bwd_s2_f32_kernel<w4>", (dw3x3_bwd_s2_f32_kernel<4>));
      else DW_BWD("dw3x3_bwd_s2_f32_kernel<w2>", (dw3x3_bwd_s2_f32_kernel<2>));
    }
#undef DW_BWD
    if (G) KLAUNCH(dw3x3_wgrad_final_kernel, dim3(cdiv(C * 9, 32)), dim3(256), 0, st, part, G, N * bd.bands, C);
    return;
  }
  DwGeom gm = dw_geom(N, C, H, W, stride);
  size_t lds =
      ((size_t)gm.ppb * ((H + 2) * (W + 2) + (gm.Ho + 2) * (gm.Wo + 2) + 9 + 3) + 44) * sizeof(float);
  (void)hipFuncSetAttribute((const void*)dw3x3_bwd_f32_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  KLAUNCH(dw3x3_bwd_f32_kernel, dim3(cdiv(gm.NC, gm.ppb)), dim3(256), lds, st, g, x, w, dx, part, gm, f);
  if (G) KLAUNCH(dw3x3_wgrad_final_kernel, dim3(cdiv(C * 9, 32)), dim3(256), 0, st, part, G, N, C);
}

}  // namespace ast
