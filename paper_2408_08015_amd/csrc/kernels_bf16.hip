// Bandwidth-bound bf16 kernels of the VGG-style and transformer stages: weight-copy
// refresh, ReLU / GELU backward, residual add, 2x2 max-pool (NHWC), LayerNorm forward and
// backward with wavefront-shuffle reductions.  Arithmetic is fp32; storage is bf16; every
// global access is a 16-byte vector (8 bf16) on the contiguous channel / feature dimension.
#include "device_utils.h"
#include "kernels_bf16.h"
#include "prof.h"

namespace ast {

namespace {
inline unsigned cdivu(size_t a, size_t b) { return (unsigned)((a + b - 1) / b); }

__device__ __forceinline__ void unpack8(const uint4& v, float* f) {
  const uint32_t* w = reinterpret_cast<const uint32_t*>(&v);
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    f[2 * k] = __uint_as_float(w[k] << 16);
    f[2 * k + 1] = __uint_as_float(w[k] & 0xffff0000u);
  }
}
__device__ __forceinline__ uint4 pack8(const float* f) {
  uint4 v;
  uint32_t* w = reinterpret_cast<uint32_t*>(&v);
#pragma unroll
  for (int k = 0; k < 4; ++k) w[k] = f2bf_pk(f[2 * k], f[2 * k + 1]);
  return v;
}
__device__ __forceinline__ float gelu_grad(float x) { return gelu_grad_fast(x); }
__device__ __forceinline__ float gelu_val(float x) { return gelu_fast(x); }
}  // namespace

// ------------------------------------------------------------------ weight copies
__global__ void conv_shadow_kernel(const float* __restrict__ w, bf16_t* __restrict__ fwd,
                                   bf16_t* __restrict__ dgr, int Cout, int Cin, int kk, int tiled_fwd, int tiled_dgrad) {
  // master [co][ci][t]; fwd [co][t][ci]; dgrad [ci][kk-1-t][co]; tiled: [slice of 64][tap][row][64]
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t total = (size_t)Cout * Cin * kk;
  if (i >= total) return;
  int t = (int)(i % kk);
  size_t r = i / kk;
  int ci = (int)(r % Cin);
  int co = (int)(r / Cin);
  bf16_t v = f2bf(w[i]);
  if (tiled_fwd) fwd[(((size_t)(ci >> 6) * kk + t) * Cout + co) * 64 + (ci & 63)] = v;
  else fwd[((size_t)co * kk + t) * Cin + ci] = v;
  if (tiled_dgrad) dgr[(((size_t)(co >> 6) * kk + (kk - 1 - t)) * Cin + ci) * 64 + (co & 63)] = v;
  else dgr[((size_t)ci * kk + (kk - 1 - t)) * Cout + co] = v;
}
void conv_weight_shadow_bf16(hipStream_t st, const float* w, bf16_t* sh_fwd, bf16_t* sh_dgrad, int Cout, int Cin,
                             int k, bool tiled_fwd, bool tiled_dgrad) {
  size_t total = (size_t)Cout * Cin * k * k;
  KLAUNCH(conv_shadow_kernel, dim3(cdivu(total, 256)), dim3(256), 0, st, w, sh_fwd, sh_dgrad, Cout, Cin, k * k,
          tiled_fwd ? 1 : 0, tiled_dgrad ? 1 : 0);
}

// sh [Cout][Cin] and sht [Cin][Cout]; tiled: [K/64][rows][64] with K the contraction index of the
// product that reads the copy (Cin for sh, Cout for sht) - the layout of the direct-to-LDS kernel.
// One 32 x 32 tile (bx: ci, by: co) per block.
__device__ __forceinline__ void linear_shadow_tile(const float* __restrict__ w, bf16_t* __restrict__ sh,
                                                   bf16_t* __restrict__ sht, int Cout, int Cin, int tiled, int tiled_t,
                                                   int bx, int by) {
  __shared__ float tile[32][33];
  int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
  for (int r = ty; r < 32; r += 8) {
    int co = by + r, ci = bx + tx;
    float v = (co < Cout && ci < Cin) ? w[(size_t)co * Cin + ci] : 0.f;
    tile[r][tx] = v;
    if (co < Cout && ci < Cin)
      sh[tiled ? ((size_t)(ci >> 6) * Cout + co) * 64 + (ci & 63) : (size_t)co * Cin + ci] = f2bf(v);
  }
  __syncthreads();
  for (int r = ty; r < 32; r += 8) {
    int ci = bx + r, co = by + tx;
    if (co < Cout && ci < Cin)
      sht[tiled_t ? ((size_t)(co >> 6) * Cin + ci) * 64 + (co & 63) : (size_t)ci * Cout + co] = f2bf(tile[tx][r]);
  }
}
__global__ void linear_shadow_kernel(const float* __restrict__ w, bf16_t* __restrict__ sh,
                                     bf16_t* __restrict__ sht, int Cout, int Cin, int tiled, int tiled_t) {
  linear_shadow_tile(w, sh, sht, Cout, Cin, tiled, tiled_t, blockIdx.x * 32, blockIdx.y * 32);
}
void linear_weight_shadow_bf16(hipStream_t st, const float* w, bf16_t* sh, bf16_t* sh_t, int Cout, int Cin, bool tiled,
                               bool tiled_t) {
  KLAUNCH(linear_shadow_kernel, dim3(cdivu(Cin, 32), cdivu(Cout, 32)), dim3(256), 0, st, w, sh, sh_t, Cout, Cin,
          tiled ? 1 : 0, tiled_t ? 1 : 0);
}
// the copies of every dense layer of a stage in one launch: block -> (matrix, tile) through a table
__global__ void linear_shadow_all_kernel(const LinShadowTask* __restrict__ tasks, const unsigned short* __restrict__ block_task) {
  const LinShadowTask t = tasks[block_task[blockIdx.x]];
  const unsigned local = blockIdx.x - t.block0;
  const unsigned nbx = (unsigned)(t.Cin + 31) / 32;
  linear_shadow_tile(t.w, t.sh, t.sht, t.Cout, t.Cin, t.tiled, t.tiled_t, (int)(local % nbx) * 32, (int)(local / nbx) * 32);
}
unsigned linear_shadow_blocks(int Cout, int Cin) { return (unsigned)(cdivu(Cin, 32) * cdivu(Cout, 32)); }
void linear_weight_shadow_all_bf16(hipStream_t st, const LinShadowTask* tasks_dev, const unsigned short* block_task_dev,
                                   int nblocks) {
  if (nblocks > 0) KLAUNCH(linear_shadow_all_kernel, dim3((unsigned)nblocks), dim3(256), 0, st, tasks_dev, block_task_dev);
}

__global__ void f32_to_bf16_kernel(const float* __restrict__ s, bf16_t* __restrict__ d, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) d[i] = f2bf(s[i]);
}
void f32_to_bf16(hipStream_t st, const float* src, bf16_t* dst, size_t n) {
  KLAUNCH(f32_to_bf16_kernel, dim3(cdivu(n, 256)), dim3(256), 0, st, src, dst, n);
}

// ------------------------------------------------------------------ elementwise (n % 8 == 0)
__global__ void act_fwd_bf16_kernel(const uint4* __restrict__ x, uint4* __restrict__ y, size_t n8, int act) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n8) return;
  float f[8];
  unpack8(x[i], f);
#pragma unroll
  for (int k = 0; k < 8; ++k) f[k] = act == ACT_GELU ? gelu_val(f[k]) : apply_act(f[k], act);
  y[i] = pack8(f);
}
// ReLU: ref = output (mask y > 0); ReLU6: ref = output (0 < y < 6); GELU: ref = pre-activation
__global__ void act_bwd_bf16_kernel(const uint4* __restrict__ g, const uint4* __restrict__ ref,
                                    uint4* __restrict__ out, size_t n8, int act) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n8) return;
  float gv[8], rv[8];
  unpack8(g[i], gv);
  unpack8(ref[i], rv);
#pragma unroll
  for (int k = 0; k < 8; ++k) gv[k] *= act == ACT_GELU ? gelu_grad(rv[k]) : act_mask(rv[k], act);
  out[i] = pack8(gv);
}
// y may alias a
__global__ void add_bf16_kernel(const uint4* a, const uint4* b, uint4* y, size_t n8) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n8) return;
  float av[8], bv[8];
  unpack8(a[i], av);
  unpack8(b[i], bv);
#pragma unroll
  for (int k = 0; k < 8; ++k) av[k] += bv[k];
  y[i] = pack8(av);
}
void act_fwd_bf16(hipStream_t st, const bf16_t* x, bf16_t* y, size_t n, int act) {
  KLAUNCH(act_fwd_bf16_kernel, dim3(cdivu(n / 8, 256)), dim3(256), 0, st, (const uint4*)x, (uint4*)y, n / 8, act);
}
void act_bwd_bf16(hipStream_t st, const bf16_t* g, const bf16_t* ref, bf16_t* out, size_t n, int act) {
  KLAUNCH(act_bwd_bf16_kernel, dim3(cdivu(n / 8, 256)), dim3(256), 0, st, (const uint4*)g, (const uint4*)ref,
          (uint4*)out, n / 8, act);
}
void add_bf16(hipStream_t st, const bf16_t* a, const bf16_t* b, bf16_t* y, size_t n) {
  KLAUNCH(add_bf16_kernel, dim3(cdivu(n / 8, 256)), dim3(256), 0, st, (const uint4*)a, (const uint4*)b, (uint4*)y,
          n / 8);
}

// ------------------------------------------------------------------ max-pool 2x2, NHWC
__global__ void maxpool_fwd_bf16_kernel(const bf16_t* __restrict__ x, bf16_t* __restrict__ y, int H, int W,
                                        int C, int Ho, int Wo, size_t total8) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total8) return;
  int c8 = C / 8;
  int cg = (int)(i % c8);
  size_t t = i / c8;
  int ox = (int)(t % Wo);
  t /= Wo;
  int oy = (int)(t % Ho);
  size_t n = t / Ho;
  const bf16_t* p = x + ((n * H + 2 * oy) * W + 2 * ox) * C + cg * 8;
  float a[8], b[8], c[8], d[8];
  unpack8(*reinterpret_cast<const uint4*>(p), a);
  unpack8(*reinterpret_cast<const uint4*>(p + C), b);
  unpack8(*reinterpret_cast<const uint4*>(p + (size_t)W * C), c);
  unpack8(*reinterpret_cast<const uint4*>(p + (size_t)W * C + C), d);
#pragma unroll
  for (int k = 0; k < 8; ++k) a[k] = fmaxf(fmaxf(a[k], b[k]), fmaxf(c[k], d[k]));
  *reinterpret_cast<uint4*>(y + i * 8) = pack8(a);
}
// one thread per output window and 8 channels: writes the four input-gradient vectors
__global__ void maxpool_bwd_bf16_kernel(const bf16_t* __restrict__ g, const bf16_t* __restrict__ x,
                                        bf16_t* __restrict__ dx, int H, int W, int C, int Ho, int Wo,
                                        size_t total8, int relu_mask) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total8) return;
  int c8 = C / 8;
  int cg = (int)(i % c8);
  size_t t = i / c8;
  int ox = (int)(t % Wo);
  t /= Wo;
  int oy = (int)(t % Ho);
  size_t n = t / Ho;
  size_t off = ((n * H + 2 * oy) * W + 2 * ox) * C + cg * 8;
  float v[4][8], gv[8], o[4][8];
  unpack8(*reinterpret_cast<const uint4*>(x + off), v[0]);
  unpack8(*reinterpret_cast<const uint4*>(x + off + C), v[1]);
  unpack8(*reinterpret_cast<const uint4*>(x + off + (size_t)W * C), v[2]);
  unpack8(*reinterpret_cast<const uint4*>(x + off + (size_t)W * C + C), v[3]);
  unpack8(*reinterpret_cast<const uint4*>(g + i * 8), gv);
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    int am = 0;
    float m = v[0][k];
    if (v[1][k] > m) { m = v[1][k]; am = 1; }
    if (v[2][k] > m) { m = v[2][k]; am = 2; }
    if (v[3][k] > m) { m = v[3][k]; am = 3; }
    // relu_mask: x is the output of a ReLU whose backward is applied here as well (gradient only where x > 0)
    const float gk = (relu_mask && !(m > 0.f)) ? 0.f : gv[k];
#pragma unroll
    for (int q = 0; q < 4; ++q) o[q][k] = q == am ? gk : 0.f;
  }
  *reinterpret_cast<uint4*>(dx + off) = pack8(o[0]);
  *reinterpret_cast<uint4*>(dx + off + C) = pack8(o[1]);
  *reinterpret_cast<uint4*>(dx + off + (size_t)W * C) = pack8(o[2]);
  *reinterpret_cast<uint4*>(dx + off + (size_t)W * C + C) = pack8(o[3]);
}
// rows / columns not covered by a window (odd H or W) get a zero gradient
__global__ void maxpool_bwd_edge_kernel(bf16_t* __restrict__ dx, int H, int W, int C, int Ho, int Wo,
                                        size_t total) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  int c = (int)(i % C);
  size_t t = i / C;
  int x = (int)(t % W);
  t /= W;
  int y = (int)(t % H);
  if (y >= 2 * Ho || x >= 2 * Wo) dx[i] = 0;
  (void)c;
}
void maxpool_fwd_bf16(hipStream_t st, const bf16_t* x, bf16_t* y, int N, int H, int W, int C) {
  int Ho = H / 2, Wo = W / 2;
  size_t total8 = (size_t)N * Ho * Wo * (C / 8);
  KLAUNCH(maxpool_fwd_bf16_kernel, dim3(cdivu(total8, 256)), dim3(256), 0, st, x, y, H, W, C, Ho, Wo, total8);
}
void maxpool_bwd_bf16(hipStream_t st, const bf16_t* g, const bf16_t* x, bf16_t* dx, int N, int H, int W, int C,
                      bool relu_mask) {
  int Ho = H / 2, Wo = W / 2;
  size_t total8 = (size_t)N * Ho * Wo * (C / 8);
  KLAUNCH(maxpool_bwd_bf16_kernel, dim3(cdivu(total8, 256)), dim3(256), 0, st, g, x, dx, H, W, C, Ho, Wo, total8,
          relu_mask ? 1 : 0);
  if ((H & 1) || (W & 1)) {
    size_t total = (size_t)N * H * W * C;
    KLAUNCH(maxpool_bwd_edge_kernel, dim3(cdivu(total, 256)), dim3(256), 0, st, dx, H, W, C, Ho, Wo, total);
  }
}

// ------------------------------------------------------------------ LayerNorm
// One wavefront per row; the row (D <= 1024, D % 8 == 0) lives in registers as LN_MAXV
// vectors of 8 per lane.  Statistics in fp32 with a centred second pass over registers.

template <int LN_MAXV>
__global__ __launch_bounds__(256) void layernorm_fwd_kernel(const bf16_t* __restrict__ x,
                                                            const float* __restrict__ gamma,
                                                            const float* __restrict__ beta,
                                                            bf16_t* __restrict__ y, float* __restrict__ stat,
                                                            size_t R, int D, float eps) {
  size_t row = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  int lane = threadIdx.x & 63;
  if (row >= R) return;
  const int nv = D / 8;  // vectors per row
  float v[LN_MAXV][8];
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < LN_MAXV; ++j) {
    int vi = lane + 64 * j;
    if (vi < nv) {
      unpack8(*reinterpret_cast<const uint4*>(x + row * D + vi * 8), v[j]);
#pragma unroll
      for (int k = 0; k < 8; ++k) s += v[j][k];
    }
  }
  const float mean = wave_sum(s) / (float)D;
  float q = 0.f;
#pragma unroll
  for (int j = 0; j < LN_MAXV; ++j) {
    int vi = lane + 64 * j;
    if (vi < nv)
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        float d = v[j][k] - mean;
        q += d * d;
      }
  }
  const float istd = rsqrtf(wave_sum(q) / (float)D + eps);
  if (lane == 0) {
    stat[row] = mean;
    stat[R + row] = istd;
  }
#pragma unroll
  for (int j = 0; j < LN_MAXV; ++j) {
    int vi = lane + 64 * j;
    if (vi < nv) {
      float o[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) o[k] = (v[j][k] - mean) * istd * gamma[vi * 8 + k] + beta[vi * 8 + k];
      *reinterpret_cast<uint4*>(y + row * D + vi * 8) = pack8(o);
    }
  }
}

// Backward: per row dx = istd * (gh - mean(gh) - xhat * mean(gh * xhat)), gh = g * gamma.
// dgamma / dbeta: each block accumulates its rows' contributions per feature in LDS
// (fixed order), writes a partial; a second kernel adds the partials into G.
template <int LN_MAXV>
__global__ __launch_bounds__(256) void layernorm_bwd_kernel(const bf16_t* __restrict__ g,
                                                            const bf16_t* __restrict__ x,
                                                            const float* __restrict__ stat,
                                                            const float* __restrict__ gamma,
                                                            const bf16_t* __restrict__ add,
                                                            bf16_t* __restrict__ dx, float* __restrict__ part,
                                                            size_t R, int D, size_t rows_per_block) {
  extern __shared__ float sh[];  // [4 waves][2][D]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nv = D / 8;
  float* my = sh + (size_t)wave * 2 * D;
  const size_t r0 = (size_t)blockIdx.x * rows_per_block;
  const size_t r1 = r0 + rows_per_block < R ? r0 + rows_per_block : R;
  // A lane owns the same features in every row of its wavefront: dgamma / dbeta stay in
  // registers until the rows are done.  The words of the next row are requested before this
  // row is worked on.
  float dg[LN_MAXV][8], db[LN_MAXV][8], gam[LN_MAXV][8];
#pragma unroll
  for (int j = 0; j < LN_MAXV; ++j) {
    const int vi = lane + 64 * j;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      dg[j][k] = 0.f;
      db[j][k] = 0.f;
      gam[j][k] = vi < nv ? gamma[vi * 8 + k] : 0.f;
    }
  }
  struct RowWords { uint4 x[LN_MAXV], g[LN_MAXV], a[LN_MAXV]; };
  auto load_row = [&](size_t row, RowWords& w) {
#pragma unroll
    for (int j = 0; j < LN_MAXV; ++j) {
      const int vi = lane + 64 * j;
      w.x[j] = w.g[j] = w.a[j] = make_uint4(0u, 0u, 0u, 0u);
      if (row < r1 && vi < nv) {
        w.x[j] = *reinterpret_cast<const uint4*>(x + row * D + vi * 8);
        w.g[j] = *reinterpret_cast<const uint4*>(g + row * D + vi * 8);
        if (add && dx) w.a[j] = *reinterpret_cast<const uint4*>(add + row * D + vi * 8);
      }
    }
  };
  RowWords nxt;
  load_row(r0 + wave, nxt);
  for (size_t row = r0 + wave; row < r1; row += 4) {
    const RowWords cur = nxt;
    load_row(row + 4, nxt);
    const float mean = stat[row], istd = stat[R + row];
    float xh[LN_MAXV][8], gh[LN_MAXV][8];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int j = 0; j < LN_MAXV; ++j) {
      int vi = lane + 64 * j;
      if (vi < nv) {
        float gv[8];
        unpack8(cur.x[j], xh[j]);
        unpack8(cur.g[j], gv);
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          xh[j][k] = (xh[j][k] - mean) * istd;
          dg[j][k] += gv[k] * xh[j][k];  // dgamma (this lane owns these features)
          db[j][k] += gv[k];             // dbeta
          gh[j][k] = gv[k] * gam[j][k];
          s1 += gh[j][k];
          s2 += gh[j][k] * xh[j][k];
        }
      }
    }
    s1 = wave_sum(s1) / (float)D;
    s2 = wave_sum(s2) / (float)D;
    if (dx) {
#pragma unroll
      for (int j = 0; j < LN_MAXV; ++j) {
        int vi = lane + 64 * j;
        if (vi < nv) {
          float o[8];
#pragma unroll
          for (int k = 0; k < 8; ++k) o[k] = istd * (gh[j][k] - s1 - xh[j][k] * s2);
          if (add) {  // gradient arriving over the residual connection around this LayerNorm
            float av[8];
            unpack8(cur.a[j], av);
#pragma unroll
            for (int k = 0; k < 8; ++k) o[k] += av[k];
          }
          *reinterpret_cast<uint4*>(dx + row * D + vi * 8) = pack8(o);
        }
      }
    }
  }
#pragma unroll
  for (int j = 0; j < LN_MAXV; ++j) {
    const int vi = lane + 64 * j;
    if (vi < nv) {
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        my[vi * 8 + k] = dg[j][k];
        my[D + vi * 8 + k] = db[j][k];
      }
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < 2 * D; i += 256)
    part[(size_t)blockIdx.x * 2 * D + i] = (sh[i] + sh[2 * D + i]) + (sh[4 * D + i] + sh[6 * D + i]);
}
// 16 outputs x 16 interleaved partial lanes per block, added in a fixed order
__global__ __launch_bounds__(256) void layernorm_bwd_final_kernel(const float* __restrict__ part,
                                                                  float* __restrict__ Ggamma,
                                                                  float* __restrict__ Gbeta, int D, int blocks) {
  const int i = blockIdx.x * 16 + (threadIdx.x & 15), q = threadIdx.x >> 4;
  float s = 0.f;
  if (i < 2 * D)
    for (int b = q; b < blocks; b += 16) s += part[(size_t)b * 2 * D + i];
  s += __shfl_xor(s, 16, 64);
  s += __shfl_xor(s, 32, 64);
  __shared__ float sh[4][16];
  if ((threadIdx.x & 63) < 16) sh[threadIdx.x >> 6][threadIdx.x & 15] = s;
  __syncthreads();
  if (threadIdx.x < 16 && i < 2 * D) {
    float v = (sh[0][threadIdx.x] + sh[1][threadIdx.x]) + (sh[2][threadIdx.x] + sh[3][threadIdx.x]);
    if (i < D) Ggamma[i] += v;
    else Gbeta[i - D] += v;
  }
}

static inline size_t ln_blocks(size_t R) {
  size_t b = (R + 15) / 16;  // at least 16 rows per block
  return b > 512 ? 512 : (b < 1 ? 1 : b);
}
size_t layernorm_bf16_ws_bytes(size_t R, int D) { return ln_blocks(R) * 2 * D * sizeof(float) + 256; }

void layernorm_fwd_bf16(hipStream_t st, const bf16_t* x, const float* gamma, const float* beta, bf16_t* y,
                        float* stat, size_t R, int D, float eps) {
  if (D <= 512) KLAUNCH(layernorm_fwd_kernel<1>, dim3(cdivu(R, 4)), dim3(256), 0, st, x, gamma, beta, y, stat, R, D, eps);
  else KLAUNCH(layernorm_fwd_kernel<2>, dim3(cdivu(R, 4)), dim3(256), 0, st, x, gamma, beta, y, stat, R, D, eps);
}
void layernorm_bwd_bf16(hipStream_t st, const bf16_t* g, const bf16_t* x, const float* stat, const float* gamma,
                        const bf16_t* add, bf16_t* dx, void* ws, size_t R, int D) {
  size_t blocks = ln_blocks(R);
  size_t rpb = (R + blocks - 1) / blocks;
  float* part = reinterpret_cast<float*>(ws);
  if (D <= 512)
    KLAUNCH(layernorm_bwd_kernel<1>, dim3((unsigned)((R + rpb - 1) / rpb)), dim3(256), (size_t)8 * D * sizeof(float), st,
            g, x, stat, gamma, add, dx, part, R, D, rpb);
  else
    KLAUNCH(layernorm_bwd_kernel<2>, dim3((unsigned)((R + rpb - 1) / rpb)), dim3(256), (size_t)8 * D * sizeof(float), st,
            g, x, stat, gamma, add, dx, part, R, D, rpb);
}

int layernorm_bwd_parts(size_t R) {
  size_t blocks = ln_blocks(R);
  size_t rpb = (R + blocks - 1) / blocks;
  return (int)((R + rpb - 1) / rpb);
}

void layernorm_bwd_params_bf16(hipStream_t st, const void* ws, float* Ggamma, float* Gbeta, size_t R, int D) {
  size_t blocks = ln_blocks(R);
  size_t rpb = (R + blocks - 1) / blocks;
  blocks = (R + rpb - 1) / rpb;
  KLAUNCH(layernorm_bwd_final_kernel, dim3(cdivu(2 * (size_t)D, 16)), dim3(256), 0, st,
          reinterpret_cast<const float*>(ws), Ggamma, Gbeta, D, (int)blocks);
}

}  // namespace ast
