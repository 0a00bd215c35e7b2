// Host-side launchers of the gfx950 kernels.  Every launcher enqueues on `st` and
// returns immediately; none allocates.  Shapes are validated by the stage runtime
// before any launch.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace ast {

typedef unsigned short bf16_t;

// ------------------------------------------------------------------ fp32, NCHW
// Pointwise (1x1) convolution as a per-pixel matrix product on the fp32 matrix cores:
//   Y[n][m][p] = sum_k A[m][k] * X[n][k][p] (+ bias[m]) (+ add[n][m][p])
// A is given as a packed copy Wp (pw_pack_floats(Mdim, Kdim) floats, written by
// pw_pack_f32 from A[m][k] = W[m*lda_m + k*lda_k]), so the same kernel serves the forward
// pass (A = W[Cout][Cin]) and the input gradient (A = W^T).
size_t pw_pack_floats(int Mdim, int Kdim);
void pw_pack_f32(hipStream_t st, const float* W, int lda_m, int lda_k, float* Wp, int Mdim, int Kdim);
// All packed copies of a stage in one launch.  The copies lie back to back in `arena` in task
// order (each pw_pack_floats() long = a whole number of 256-float blocks); block b of the
// launch writes arena[256*b, +256) for task block_task[b], whose first block is block0.
struct PackTask {
  const float* W;
  int lda_m, lda_k, Mdim, Kdim, KG;
  unsigned block0;
};
void pw_pack_all_f32(hipStream_t st, const PackTask* tasks_dev, const unsigned short* block_task_dev, float* arena,
                     int nblocks);
// stats (may be NULL; needs bias == add == NULL and pw_conv_stats_parts() > 0): the kernel also
// leaves (sum, sum of squares) of Y per channel and pixel block, stats[Mdim][pw_conv_stats_parts()][2],
// for a BatchNorm behind the convolution.
int pw_conv_stats_parts(int N, int Kdim, int Mdim, int HW);
void pw_conv_f32(hipStream_t st, const float* Wp, const float* X, float* Y, const float* bias,
                 const float* add, int N, int Kdim, int Mdim, int HW, double* stats = nullptr);
// Weight gradient of the pointwise convolution, split over pixel chunks:
//   part[chunk][co][ci] = sum_{p in chunk} g[n][co][p] * x[n][ci][p];  then G += sum_chunk part.
// `part` must hold pw_wgrad_f32_ws(N,Cin,Cout,HW) floats; with G = NULL only the partials are
// written (pw_wgrad_f32_parts of them, Cout*Cin floats each).
size_t pw_wgrad_f32_ws(int N, int Cin, int Cout, int HW);
void pw_wgrad_f32(hipStream_t st, const float* g, const float* x, float* part, float* G, int N,
                  int Cin, int Cout, int HW);

// Depthwise 3x3 convolution, pad 1, stride 1 or 2, weights [C][3][3].
// The forward kernel can take over the BatchNorm passes around it:
// DwBnIn: its input is x' = act(x*scale[c] + shift[c]) of a BatchNorm over the tensor passed as x;
//   the kernel finishes that BatchNorm's statistics from the P partial pairs ws[c][P][2]
//   (records them as the BatchNorm's own apply pass would) and normalises while staging;
// DwBnOut: it leaves (sum, sum of squares) of its output in ws[c][dw3x3_parts()][2] for the
//   BatchNorm that follows.
struct DwBnIn {
  const double* ws;
  const float* gamma;
  const float* beta;
  float* stat;
  float* ss;
  float* running;
  double count;
  float eps;
  int P, act, on;
};
struct DwBnOut {
  double* ws;
  int on;
};
// bn_in (may be NULL): see DwBnIn, `on` must be 1; stats_out (may be NULL): DwBnOut's ws.
void dw3x3_fwd_f32(hipStream_t st, const float* x, const float* w, float* y, int N, int C, int H,
                   int W, int stride, const DwBnIn* bn_in = nullptr, double* stats_out = nullptr);
// Backward of the depthwise conv from one read of g and x: dx (skipped if NULL) and
// G[C][3][3] += weight gradient.  `part` holds dw3x3_bwd_f32_ws(...) floats: dw3x3_parts() partials of
// C*9 sums; with G = NULL the reduction is left to the caller (reduce_tasks_f32).
size_t dw3x3_bwd_f32_ws(int N, int C, int H, int W, int stride);
// Partial sums per channel that the depthwise kernels leave (weight-gradient partials, BatchNorm
// sums): one per sample, or several where a plane is split into bands of rows over wavefronts.
int dw3x3_parts(int N, int C, int H, int W, int stride);
bool dw3x3_supported(int H, int W, int stride);  // else the generic grouped-conv kernels apply
// Dense conv on the matrix cores: 3x3 pad 1 with stride 1 or 2, and 1x1 stride 2.  Wp: k*k packed copies
// (pw_pack layout, one per tap, conv_mfma_pack_floats(Mdim, Kdim, k) floats in all): forward copy t holds
// A[co][ci] = W[co][ci][t], input-gradient copy t holds A[ci][co] = W[co][ci][t].  Backward: dx (may be NULL)
// and the weight-gradient partials in `part` (conv_mfma_wgrad_ws floats, conv_mfma_wgrad_parts chunks of
// [Cout][Cin][k*k]); G (may be NULL: the caller reduces the partials) += their sum.
bool conv_mfma_supported(int Cin, int Cout, int k, int stride, int pad, int groups, int H, int W);
size_t conv_mfma_pack_floats(int Mdim, int Kdim, int k);
int conv_mfma_wgrad_parts(int N, int Cin, int Cout, int H, int W, int k, int stride);
size_t conv_mfma_wgrad_ws(int N, int Cin, int Cout, int H, int W, int k, int stride);
void conv_mfma_fwd_f32(hipStream_t st, const float* Wp, const float* x, float* y, const float* bias, int N, int Cin,
                       int Cout, int H, int W, int k, int stride);
void conv_mfma_bwd_f32(hipStream_t st, const float* Wp_t, const float* g, float* dx, const float* x, float* part,
                       float* G, int N, int Cin, int Cout, int H, int W, int k, int stride);
// 7x7 dense conv with fewer than 8 input channels (ResNet's stem) on the matrix cores: the contraction index is
// the flattened (ci, u, v); Wp = pw_pack of W as the [Cout][Cin*49] matrix.  Forward and weight gradient
// (partials [chunk][Cout][Cin*49] in `part`, G may be NULL: the caller reduces).
bool conv_gatherk_supported(int Cin, int Cout, int k, int stride, int pad, int groups, int H, int W);
size_t conv_gatherk_pack_floats(int Cin, int Cout, int k);
int conv_gatherk_wgrad_parts(int N, int Cin, int Cout, int H, int W, int k, int stride, int pad);
size_t conv_gatherk_wgrad_ws(int N, int Cin, int Cout, int H, int W, int k, int stride, int pad);
void conv_gatherk_fwd_f32(hipStream_t st, const float* Wp, const float* x, float* y, const float* bias, int N, int Cin,
                          int Cout, int H, int W, int k, int stride, int pad);
void conv_gatherk_wgrad_f32(hipStream_t st, const float* g, const float* x, float* part, float* G, int N, int Cin, int Cout,
                            int H, int W, int k, int stride, int pad);
// Depthwise K x K (K = 5), pad K/2, stride 1 or 2, no bias: one block per plane, taps from LDS.
// Backward: dx (may be NULL), and G[C][K][K] += weight gradient through `part`
// (dwk_bwd_f32_ws floats of scratch: one K*K partial per plane, added over the samples in order).
bool dwk_supported(int K, int H, int W, int stride);
size_t dwk_bwd_f32_ws(int N, int C, int K);
void dwk_fwd_f32(hipStream_t st, const float* x, const float* w, float* y, int N, int C, int H, int W, int K,
                 int stride);
void dwk_bwd_f32(hipStream_t st, const float* g, const float* x, const float* w, float* dx, float* part, float* G,
                 int N, int C, int H, int W, int K, int stride);
struct DwBands {
  int bands, rpb;  // bands per plane, rows per band
};
// Optional BatchNorm work of the depthwise backward kernel (a NULL pointer switches a part off).
struct DwBwdFuse {
  // BatchNorm(+act) in front of the conv whose output was never written: the conv's input is
  // act(x*xss[c] + xss[C + c]), recomputed on load
  const float* xss = nullptr;
  int xact = 0;
  // ... and that BatchNorm's backward sums: ws_in[c][dw3x3_parts()][2] =
  // (sum g', sum g'*xhat), g' = dx*act'(.), xhat = (x - xstat[c])*xstat[C + c]; needs xss and dx
  const float* xstat = nullptr;
  double* ws_in = nullptr;
  // BatchNorm(+act) behind the conv: `g` is THAT BatchNorm's upstream gradient, y its input (the
  // conv's output); the conv's own upstream gradient is the BatchNorm's input gradient, formed on
  // load from g, y and the backward sums ws_out[c][P_out][2]; the kernel adds dgamma and dbeta
  const float* y = nullptr;
  const float* ystat = nullptr;   // mean[C], 1/std[C]
  const float* yss = nullptr;     // scale[C], shift[C]
  const float* ygamma = nullptr;
  const double* ws_out = nullptr;
  float* Ggamma = nullptr;
  float* Gbeta = nullptr;
  double ycount = 0;              // elements per channel of y
  int P_out = 0, yact = 0;
};
void dw3x3_bwd_f32(hipStream_t st, const float* g, const float* x, const float* w, float* dx, float* part,
                   float* G, int N, int C, int H, int W, int stride, const DwBwdFuse* fuse = nullptr);

// Generic direct convolution (any k, stride, pad, groups); the fallback for shapes the
// specialised kernels do not cover (e.g. a 3-channel stem).
void conv_direct_fwd_f32(hipStream_t st, const float* x, const float* w, const float* bias, float* y,
                         int N, int Cin, int H, int W, int Cout, int k, int stride, int pad,
                         int groups);
void conv_direct_dgrad_f32(hipStream_t st, const float* g, const float* w, float* dx, int N, int Cin,
                           int H, int W, int Cout, int k, int stride, int pad, int groups);
// `ws` holds conv_direct_wgrad_ws(...) floats (0: none needed).
size_t conv_direct_wgrad_ws(int N, int Cin, int H, int W, int Cout, int k, int stride, int pad, int groups);
void conv_direct_wgrad_f32(hipStream_t st, const float* g, const float* x, float* G, float* ws, int N, int Cin,
                           int H, int W, int Cout, int k, int stride, int pad, int groups);
// G[i] += sum_c part[c*n + i], c < parts, in a fixed order.
void reduce_parts_acc_f32(hipStream_t st, const float* part, float* G, size_t n, int parts);
// The same reduction for a whole list of (part, G, n, parts) in ONE launch: the weight-gradient
// kernels of a backward pass only write their partials (pass G = NULL to them) and the list is
// reduced once at the end of the pass, instead of one few-microsecond launch per layer.
// Block b of the launch works on task block_task[b], outputs [64*(b - block0), +64).
// General form: G[out(i)] += sum_{c < parts} part[c*stride + i], i < n, with out(i) = i, or for
// the k x k conv layout (taps > 1, n = taps*mn) out(i) = (i % mn)*taps + i / mn.
// wide != 0: the task's blocks cover 1024 outputs each (one thread = four consecutive outputs
// read with 16-byte loads, all partials of a thread in flight together; needs part 16-byte
// aligned and n, stride multiples of 4), else 64 outputs x 4 interleaved partial lanes.
struct RedTask {
  const float* part;
  float* G;
  unsigned n, parts, block0, stride, taps, mn, wide, pad;
};
void reduce_tasks_f32(hipStream_t st, const RedTask* tasks_dev, const unsigned short* block_task_dev, int nblocks);
int pw_wgrad_f32_parts(int N, int Cin, int Cout, int HW);  // partial count of pw_wgrad_f32
// Backward of a pointwise conv in one launch: dx = W^T g (+ add) with Wp_t the packed W^T, and
// the weight-gradient partials (then G += their sum, unless G is NULL: left to the caller).
void pw_conv_bwd_f32(hipStream_t st, const float* Wp_t, const float* g, float* dx, const float* add, const float* x,
                     float* part, float* G, int N, int Cin, int Cout, int HW);
// G[c] += sum_{n,p} g[n][c][p]
void channel_sum_acc_f32(hipStream_t st, const float* g, float* G, int N, int C, int HW);

// BatchNorm2d, training mode.  `ws` holds bn_ws_doubles(C, N, HW) doubles.
size_t bn_ws_doubles(int C, int N, int HW);
// Forward: batch statistics of x, then y = act(x*scale[c] + shift[c]) (+ skip).
// mean/istd -> stat[0..C) / stat[C..2C); scale/shift -> scale_shift[0..2C);
// running[0..C) mean, running[C..2C) var updated in place (momentum 0.1, unbiased variance).
void bn_fwd_f32(hipStream_t st, const float* x, const float* gamma, const float* beta, const float* skip,
                float* y, float* stat, float* scale_shift, float* running, double* ws, int N, int C, int HW,
                float eps, int act);
// Backward: g' = g * act'(x*scale+shift); dbeta += sum g'; dgamma += sum g'*xhat;
// dx = gamma*istd*(g' - mean(g') - xhat*mean(g'*xhat)); dx may be NULL (not wanted).
// The two halves of bn_fwd_f32, for stages that take one of them over: statistics partials
// ws[C][bn_parts(N, HW)][2] (sum, sum of squares), and the normalisation from P partial pairs per
// channel (P = bn_parts() for bn_stats_f32's, or whatever the producer of `ws` wrote).
int bn_parts(int N, int HW);
void bn_stats_f32(hipStream_t st, const float* x, double* ws, int N, int C, int HW);
void bn_apply_f32(hipStream_t st, const float* x, const float* gamma, const float* beta, const float* skip, float* y,
                  float* stat, float* scale_shift, float* running, const double* ws, int P, int N, int C, int HW,
                  float eps, int act);
void bn_bwd_f32(hipStream_t st, const float* g, const float* x, const float* stat, const float* scale_shift,
                const float* gamma, float* dx, float* Ggamma, float* Gbeta, double* ws, int N, int C, int HW,
                int act);
// Small tensors (bn_onepass_fits: at most 8192 elements per channel): forward and backward as ONE
// launch each, one block per channel, no workspace.
bool bn_onepass_fits(int N, int HW);
void bn_fwd_onepass_f32(hipStream_t st, const float* x, const float* gamma, const float* beta, const float* skip,
                        float* y, float* stat, float* scale_shift, float* running, int N, int C, int HW, float eps,
                        int act);
void bn_bwd_onepass_f32(hipStream_t st, const float* g, const float* x, const float* stat, const float* scale_shift,
                        const float* gamma, float* dx, float* Ggamma, float* Gbeta, int N, int C, int HW, int act);
// Its two halves: the partial sums ws[C][bn_parts(N, HW)][2] = (sum g', sum g'*xhat), and the input
// gradient (+ dgamma, dbeta) from P partial pairs per channel, whoever wrote them.
void bn_bwd_partial_f32(hipStream_t st, const float* g, const float* x, const float* stat, const float* scale_shift,
                        double* ws, int N, int C, int HW, int act);
void bn_bwd_apply_f32(hipStream_t st, const float* g, const float* x, const float* stat, const float* scale_shift,
                      const float* gamma, const double* ws, int P, float* dx, float* Ggamma, float* Gbeta, int N,
                      int C, int HW, int act);

// Elementwise
void act_fwd_f32(hipStream_t st, const float* x, float* y, size_t n, int act);
void act_bwd_f32(hipStream_t st, const float* g, const float* x, float* dx, size_t n, int act);
void add_f32(hipStream_t st, const float* a, const float* b, float* y, size_t n);
void copy_bytes(hipStream_t st, const void* src, void* dst, size_t bytes);
void fill_zero(hipStream_t st, void* dst, size_t bytes);

// Pooling
void gap_fwd_f32(hipStream_t st, const float* x, float* y, int NC, int HW);
void gap_bwd_f32(hipStream_t st, const float* g, float* dx, int NC, int HW, bool accumulate = false);
// Squeeze-and-excitation gate in one launch per direction: p [N][C] -> hpre = W1 p + b1 [N][Cr] ->
// h = swish(hpre) -> z = W2 h + b2 [N][C] -> gate = sigmoid(z).  Backward: dz and dhp (the gradients
// of z and hpre) are written as by-products, dp may be NULL; G* += the parameter gradients (a bias
// gradient pointer is NULL when the layer has no bias).
bool se_gate_supported(int C, int Cr);
void se_gate_fwd_f32(hipStream_t st, const float* p, const float* W1, const float* b1, const float* W2, const float* b2,
                     float* hpre, float* h, float* z, float* gate, int N, int C, int Cr);
void se_gate_bwd_f32(hipStream_t st, const float* dgate, const float* z, const float* hpre, const float* p, const float* h,
                     const float* W1, const float* W2, float* dz, float* dhp, float* dp, float* GW1, float* Gb1, float* GW2,
                     float* Gb2, int N, int C, int Cr);
// squeeze-and-excitation scale: y = x * gate[plane]; backward: dgate[plane] = sum dy*x, dx = dy * gate (dx may be NULL)
void se_scale_fwd_f32(hipStream_t st, const float* x, const float* gate, float* y, int NC, int HW);
void se_scale_bwd_f32(hipStream_t st, const float* dy, const float* x, const float* gate, float* dgate, float* dx,
                      int NC, int HW);
// 3x3 window, stride 2, padding 1 (padding never wins); backward in gather form: an input position collects
// the gradient of every window whose first maximum (row-major) it is
void maxpool3x3s2_fwd_f32(hipStream_t st, const float* x, float* y, int NC, int H, int W);
void maxpool3x3s2_bwd_f32(hipStream_t st, const float* g, const float* x, float* dx, int NC, int H, int W);
void maxpool_fwd_f32(hipStream_t st, const float* x, float* y, int NC, int H, int W);
void maxpool_bwd_f32(hipStream_t st, const float* g, const float* x, float* dx, int NC, int H, int W);

// Linear on [R][Cin] rows, fp32.
void linear_fwd_f32(hipStream_t st, const float* x, const float* W, const float* b, float* y, int R,
                    int Cin, int Cout);
void linear_dgrad_f32(hipStream_t st, const float* g, const float* W, float* dx, int R, int Cin,
                      int Cout);
void linear_wgrad_f32(hipStream_t st, const float* g, const float* x, float* GW, float* Gb, int R,
                      int Cin, int Cout);

// Softmax cross-entropy over [R][C] logits; p is stashed; loss = sum_r(-log p[r][label])*inv_denom.
void softmax_ce_fwd_f32(hipStream_t st, const float* z, const int32_t* labels, float* p,
                        float* row_loss, float* loss_out, int R, int C, float inv_denom);
void softmax_ce_bwd_f32(hipStream_t st, const float* p, const int32_t* labels, float* dz, int R,
                        int C, float inv_denom);

// Momentum SGD over the flat arenas: v = mu*v + g; w -= lr*v; g = 0.
void sgd_momentum_f32(hipStream_t st, float* w, float* g, float* v, size_t n, float lr, float mu);

}  // namespace ast
