// Host-side launchers of the bf16-operand / fp32-accumulate kernels (NHWC images and
// [rows][features] token matrices).  All matrix products run on the gfx950 matrix cores
// (v_mfma_f32_32x32x16_bf16) from LDS-staged tiles.  None of the launchers allocates.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace ast {

typedef unsigned short bf16_t;

// ---- weight copies (refreshed by the optimizer step from the fp32 master weights)
// conv: master [Cout][Cin][k][k] -> fwd operand [Cout][tap][Cin] and input-gradient operand
// [Cin][tap'][Cout] with tap' the point-reflected tap.  With tiled_fwd / tiled_dgrad the copy is
// laid out for the LDS-halo kernel instead: [Cin/64][tap][Cout][64] / [Cout/64][tap'][Cin][64].
void conv_weight_shadow_bf16(hipStream_t st, const float* w, bf16_t* sh_fwd, bf16_t* sh_dgrad, int Cout,
                             int Cin, int k, bool tiled_fwd, bool tiled_dgrad);
// linear: master [Cout][Cin] -> copy [Cout][Cin] and transpose [Cin][Cout]
void linear_weight_shadow_bf16(hipStream_t st, const float* w, bf16_t* sh, bf16_t* sh_t, int Cout, int Cin,
                               bool tiled, bool tiled_t);
// ... and for all dense layers of a stage in one launch: the table lives in device memory, block_task maps a
// block to its matrix, a matrix takes linear_shadow_blocks() consecutive blocks from block0.
struct LinShadowTask {
  const float* w;
  bf16_t* sh;
  bf16_t* sht;
  int Cout, Cin, tiled, tiled_t;
  unsigned block0;
};
unsigned linear_shadow_blocks(int Cout, int Cin);
void linear_weight_shadow_all_bf16(hipStream_t st, const LinShadowTask* tasks_dev, const unsigned short* block_task_dev,
                                   int nblocks);

// ---- dense 'same' convolution, stride 1, NHWC, k in {1,3}
size_t conv_bf16_ws_bytes(int N, int H, int W, int Cin, int Cout, int k);
// y = act(conv(x) + bias)
void conv_bf16_fwd(hipStream_t st, const bf16_t* x, const bf16_t* sh_fwd, const float* bias, bf16_t* y,
                   int N, int H, int W, int Cin, int Cout, int k, int act);
// dx = conv^T(g); with `relu_out` ([N][H][W][Cin], may be NULL: the output of a ReLU that feeds this
// conv) dx is zeroed where relu_out <= 0: that ReLU's backward, folded into the epilogue.
void conv_bf16_dgrad(hipStream_t st, const bf16_t* g, const bf16_t* sh_dgrad, bf16_t* dx, const bf16_t* relu_out,
                     int N, int H, int W, int Cin, int Cout, int k);
// The same 3x3 product with the input tile and its halo staged in LDS once per 64-channel slice
// (conv_bf16_halo.hip).  conv_bf16_uses_halo(N, H, W, Cin, Cout, k): conv_bf16_fwd takes that
// kernel for this shape and expects the tiled weight copy [Cin/64][tap][Cout][64]; the input
// gradient asks with Cin and Cout exchanged.  The answer is fixed for the life of the process
// (it needs a device: the kernel's LDS size has to be granted).
// conv3x3_halo_bf16: act is 0 or ReLU; the output is zeroed where mask <= 0 (mask may be NULL).
bool conv_bf16_uses_halo(int N, int H, int W, int Cin, int Cout, int k);
bool conv3x3_halo_supported(int N, int H, int W, int Cin, int Cout);
void conv3x3_halo_bf16(hipStream_t st, const bf16_t* x, const bf16_t* w, const float* bias, const bf16_t* mask,
                       bf16_t* y, int N, int H, int W, int Cin, int Cout, int act);
// Weight gradient with both operands read transposed from LDS (conv_bf16_wgrad.hip): partials
// part[split][tap][Cout][Cin], conv_wgrad_tr_splits() of them (a function of the shape alone), and,
// with bias_part, the splits' column sums of dy [split][Cout] (the bias gradient's partials).
// conv_bf16_wgrad uses it where conv_wgrad_tr_supported() (needs a device: LDS size granted).
int conv_wgrad_tr_splits(long P, int Cin, int Cout, int taps);
bool conv_wgrad_tr_supported(int N, int H, int W, int Cin, int Cout, int k);
void conv_wgrad_tr_bf16(hipStream_t st, const bf16_t* dy, const bf16_t* x, float* part, float* bias_part, int N, int H,
                        int W, int Cin, int Cout, int k);
// Grouped weight gradients of linear layers (same kernel, one launch for many products, no split-K:
// each product is added straight into its gradient): the caller builds one descriptor per product on
// the host (wgrad_group_task returns the product's block count), a block -> product table and the
// first block of each product, copies the three arrays to the device once, and launches them together
// (or a contiguous range of the table's blocks: block_base, nblocks).
size_t wgrad_group_task_bytes();
bool wgrad_group_supported(size_t rows, int Cin, int Cout);
int wgrad_group_task(void* task_out, const bf16_t* dy, const bf16_t* x, float* GW, float* Gb, size_t rows, int Cin, int Cout);
void wgrad_group_launch(hipStream_t st, const void* tasks_dev, const unsigned short* block_task_dev,
                        const unsigned* task_block0_dev, int block_base, int nblocks);
// Scratch layout of a weight-gradient call: `splits` partial copies of the weight gradient at
// ws[0, ...), `bias_parts` partial bias gradients ([bias_parts][Cout]) from float offset bias_off.
struct WgradParts { int splits; size_t bias_off; int bias_parts; };
WgradParts conv_bf16_wgrad_parts(int N, int H, int W, int Cin, int Cout, int k);
// GW[Cout][Cin][k][k] += conv weight gradient, Gb[Cout] += sum of g (if has_bias).  With
// `defer` only the partials are written and the caller reduces them (reduce_tasks_f32).
void conv_bf16_wgrad(hipStream_t st, const bf16_t* g, const bf16_t* x, float* GW, float* Gb, bool has_bias,
                     bool defer, void* ws, int N, int H, int W, int Cin, int Cout, int k);

// ---- linear on [R][Cin] rows
// Whether the product of [R][K] rows with an [N][K] weight matrix runs in the direct-to-LDS kernel,
// which reads its weights from the tiled copy [K/64][N][64] (linear_weight_shadow_bf16: `tiled` for
// the forward copy with K = Cin, N = Cout; `tiled_t` for the transposed one with K = Cout, N = Cin).
bool linear_dl_supported(size_t R, int K, int N);
void linear_dl_bf16(hipStream_t st, const bf16_t* a, const bf16_t* b, const float* bias, bf16_t* c, bf16_t* pre,
                    const bf16_t* add, const bf16_t* gmul, size_t R, int K, int N, int act);
size_t linear_bf16_ws_bytes(size_t R, int Cin, int Cout);
// y = act(x W^T + b) (+ add); with act == GELU the pre-activation goes to `pre` as well
// `add` (may be NULL): residual input [R][Cout] added to the rounded output.
void linear_bf16_fwd(hipStream_t st, const bf16_t* x, const bf16_t* sh, const float* bias, bf16_t* y,
                     bf16_t* pre, const bf16_t* add, size_t R, int Cin, int Cout, int act);
// dx = g W; with `gelu_pre` ([R][Cin], may be NULL) dx is further multiplied by GELU'(gelu_pre):
// the backward of a GELU in front of this layer, folded into the epilogue; with `add` ([R][Cin],
// may be NULL) the gradient arriving over a residual connection is added.  At most one of the two.
void linear_bf16_dgrad(hipStream_t st, const bf16_t* g, const bf16_t* sh_t, bf16_t* dx, const bf16_t* gelu_pre,
                       const bf16_t* add, size_t R, int Cin, int Cout);
WgradParts linear_bf16_wgrad_parts(size_t R, int Cin, int Cout);
void linear_bf16_wgrad(hipStream_t st, const bf16_t* g, const bf16_t* x, float* GW, float* Gb, bool has_bias,
                       bool defer, void* ws, size_t R, int Cin, int Cout);

// ---- elementwise on bf16
// g' = g * act'(.) : ReLU masks by the OUTPUT y (> 0), GELU uses the stashed pre-activation.
void act_bwd_bf16(hipStream_t st, const bf16_t* g, const bf16_t* ref, bf16_t* out, size_t n, int act);
void act_fwd_bf16(hipStream_t st, const bf16_t* x, bf16_t* y, size_t n, int act);
void add_bf16(hipStream_t st, const bf16_t* a, const bf16_t* b, bf16_t* y, size_t n);
void maxpool_fwd_bf16(hipStream_t st, const bf16_t* x, bf16_t* y, int N, int H, int W, int C);
void maxpool_bwd_bf16(hipStream_t st, const bf16_t* g, const bf16_t* x, bf16_t* dx, int N, int H, int W,
                      int C, bool relu_mask);

// ---- LayerNorm over the last dimension of [R][D]
size_t layernorm_bf16_ws_bytes(size_t R, int D);
void layernorm_fwd_bf16(hipStream_t st, const bf16_t* x, const float* gamma, const float* beta,
                        bf16_t* y, float* stat /*[2][R]*/, size_t R, int D, float eps);
// Backward in two launches: dx (+ add, the gradient arriving over a residual connection around
// the LayerNorm; may be NULL) and per-block partials of dgamma / dbeta into ws; then
// Ggamma / Gbeta += the partials (may run on another stream once the first launch is done).
void layernorm_bwd_bf16(hipStream_t st, const bf16_t* g, const bf16_t* x, const float* stat,
                        const float* gamma, const bf16_t* add, bf16_t* dx, void* ws, size_t R, int D);
void layernorm_bwd_params_bf16(hipStream_t st, const void* ws, float* Ggamma, float* Gbeta, size_t R, int D);
int layernorm_bwd_parts(size_t R);  // number of [2][D] partial rows the backward kernel writes

// ---- self-attention core on packed qkv [B][S][3D] (head size 64, S % 32 == 0, S <= 256):
// o [B][S][D], lse [B][H][S]
size_t mha_bf16_ws_bytes(int B, int S, int D, int heads);
void attention_fwd_bf16(hipStream_t st, const bf16_t* qkv, bf16_t* o, float* lse, int B, int S, int D,
                        int heads);
// `dsum` is scratch of mha_bf16_ws_bytes() bytes
void attention_bwd_bf16(hipStream_t st, const bf16_t* qkv, const bf16_t* o, const bf16_t* d_o,
                        const float* lse, bf16_t* dqkv, float* dsum, int B, int S, int D, int heads);

// bf16 <-> fp32 conversion of flat buffers
void f32_to_bf16(hipStream_t st, const float* src, bf16_t* dst, size_t n);

}  // namespace ast
