// Stage runtime: turns the layer list of a stage model into an execution plan of
// fused operators over flat arenas (parameters W, accumulated gradients G, velocity V),
// a ring of K activation stashes and one gradient/scratch workspace, and enforces the
// one-forward-one-backward call discipline (Sec. 3.2; memory model Eq. (3)).
#pragma once
#include <hip/hip_runtime.h>

#include <string>
#include <vector>

#include "../../include/asteroid.h"

namespace ast {

enum OpKind {
  OP_CONV_PW,      // fp32 1x1 dense conv (matrix cores)
  OP_CONV_DW,      // fp32 depthwise 3x3
  OP_CONV_DWK,     // fp32 depthwise 5x5 (LDS-staged planes)
  OP_CONV_3X3,     // fp32 dense 3x3 (pad 1, stride 1 or 2) or 1x1 stride 2 on the matrix cores (k*k packed weight copies
                   // per direction)
  OP_CONV_GK,      // fp32 7x7 conv with few input channels (matrix cores, contraction over (ci, u, v))
  OP_CONV_DIRECT,  // fp32 generic conv
  OP_CONV_IGEMM,   // bf16 NHWC implicit-GEMM conv (+bias, +ReLU)
  OP_BN,           // BatchNorm (+ReLU/ReLU6) (+residual add)
  OP_ACT,          // standalone ReLU / ReLU6 / GELU / swish / sigmoid
  OP_SE_BEGIN,     // squeeze-and-excitation: marks the tensor that OP_SE_SCALE multiplies by its gate
  OP_SE_SCALE,     // in = gate [B][C], skip = the image tensor of the matching OP_SE_BEGIN
  OP_SE_GATE,      // linear -> swish -> linear -> sigmoid on the pooled vector, as one launch (takes the place of
                   // the first linear op; the three ops behind it are marked `absorbed`)
  OP_RES_BEGIN,
  OP_RES_SWAP,     // two-branch residual block: the shortcut branch starts (no work of its own)
  OP_RES_ADD,
  OP_GAP,
  OP_MAXPOOL,
  OP_LINEAR,       // fp32 rows (vectors) or bf16 token GEMM (+GELU)
  OP_SOFTMAX_CE,
  OP_LAYERNORM,    // (+ residual add fused in front)
  OP_MHA
};

struct Act {
  int n = 0, c = 0, h = 1, w = 1;  // logical dims; tokens: h = S, c = D; vectors: h = w = 1
  int rank = 4;                    // 4 image, 3 tokens, 2 vectors
  int esize = 4;                   // bytes per element (4 fp32, 2 bf16)
  size_t elems = 0, bytes = 0;
  size_t slot_off = 0;             // byte offset inside a stash slot
  size_t grad_off = 0;             // byte offset inside the gradient workspace
  int grad_alias = -1;             // gradient buffer shared with this activation's
  int data_alias = -1;             // same tensor as this activation (own gradient buffer): the input of a shortcut branch
  int layer = -1;                  // layer index whose output this is (-1: stage input)
};

struct Op {
  OpKind kind;
  int layer = -1;         // first layer index covered by this op
  int in = -1, out = -1;  // activation ids
  int skip = -1;          // residual partner: skip input (BN/LN/RES_ADD) or, for RES_BEGIN /
                          // a fused dgrad add, the activation whose gradient is the skip gradient
  int act = 0;            // fused activation code
  size_t w_off = 0, b_off = 0;  // offsets (floats) into the flat arenas; b_off valid iff has_bias
  int has_bias = 0;
  int cin = 0, cout = 0, k = 1, stride = 1, pad = 0, groups = 1;
  int heads = 0;
  float eps = 1e-5f;
  size_t aux_off = 0, aux_bytes = 0;  // per-slot extras (statistics, probabilities, ...)
  size_t run_off = 0;                 // BatchNorm running statistics (floats, persistent)
  int dgrad_add = -1;                 // pointwise conv / LayerNorm: add this activation's gradient to dx
  int res_in = -1;                    // bf16 linear / MHA: residual input added in the output epilogue
  int gelu_from = -1;                 // bf16 linear behind a fused linear+GELU: that op's pre-activation;
                                      // the input gradient is multiplied by GELU'(pre) in the epilogue
  bool gelu_bwd_fused = false;        // linear+GELU whose GELU backward the consumer already applied
  int relu_from = -1;                 // bf16 conv behind a fused conv+ReLU: that op's output; the input
                                      // gradient is masked by it in the epilogue
  bool relu_bwd_fused = false;        // conv+ReLU whose ReLU backward the consumer already applied
  bool noop_bwd = false;              // RES_BEGIN whose add was fused into the next dgrad
  bool absorbed = false;              // executed by the OP_SE_GATE in front of it: skipped in both passes
  bool grad_accum = false;            // global average pool that opens a squeeze-and-excitation branch: its input
                                      // gradient is added to the one OP_SE_SCALE has already written
  size_t sh_off = 0, sh2_off = 0;     // bf16 weight copies (elements) in the shadow arena
  size_t wp_off = 0, wp2_off = 0;     // fp32 pointwise conv: packed forward / dgrad operands (floats)
  size_t sc_off = 0;                  // this op's private scratch region (bytes past scratch_off)
  size_t fsc_off = 0;                 // BatchNorm: its forward-pass scratch (bytes past fscratch_off)
  // fp32 BatchNorm passes taken over by the depthwise conv next to them:
  bool bn_lazy = false;               // BatchNorm(+act) feeding a depthwise conv: the output is never written; the
                                      // conv normalises on load (forward and backward) and finishes the statistics
  bool bn_stats_given = false;        // BatchNorm behind a depthwise conv: the conv's epilogue leaves per-plane sums
  bool bn_bwd_sums_given = false;     // lazy BatchNorm: the conv's backward leaves its backward sums per plane
  bool bn_bwd_apply_fused = false;    // BatchNorm behind a depthwise conv: the conv's backward forms the
                                      // BatchNorm's input gradient on load and adds dgamma, dbeta
  int given_parts = 0;                // BatchNorm: partial pairs per channel the depthwise conv in front leaves (forward)
  int given_bwd_parts = 0;            // BatchNorm: ... the depthwise conv behind leaves (backward)
  int bn_in_op = -1;                  // depthwise conv: index of the lazy BatchNorm op in front
  int bn_out_op = -1;                 // depthwise conv: index of the BatchNorm op it writes statistics for
  int bn_bwd_out_op = -1;             // depthwise conv: index of the BatchNorm op whose backward apply it does
  int stats_op = -1;                  // pointwise conv: index of the BatchNorm op it writes statistics for
  bool wg_grouped = false;            // bf16 linear / attention projections: the weight (and bias) gradient is part of
                                      // the stage's one grouped weight-gradient launch at the end of the backward pass
};

struct Stage {
  ast_stage_cfg cfg;
  std::vector<ast_layer> layers;
  std::vector<Act> acts;
  std::vector<Op> ops;
  std::vector<int> layer_act;  // layer -> activation id holding its output (-1 if fused away)
  hipStream_t stream = nullptr;
  bool bf16 = false;
  bool loss_tail = false;
  int final_act = 0;  // activation id of the stage output (logits for a loss tail)
  bool final_in_slot = false;  // the backward reads the stage output (a fused ReLU mask): it is
                               // produced in the stash and copied to the caller's buffer
  int n_classes = 0;

  size_t nparams = 0;
  float *W = nullptr, *G = nullptr, *V = nullptr;  // flat arenas (device)
  unsigned short* shadow = nullptr;                // bf16 weight copies
  size_t shadow_elems = 0;
  float* wpack = nullptr;  // packed pointwise-conv operands (fp32 stages)
  size_t wpack_floats = 0;
  float* running = nullptr;  // BatchNorm running mean/var
  size_t running_floats = 0;

  size_t slot_bytes = 0;
  std::vector<char*> slots;  // K stash slots
  char* ws = nullptr;        // workspace: activation gradients + scratch
  size_t ws_bytes = 0, grad_bytes = 0;
  size_t scratch_off = 0, scratch_bytes = 0;  // per-op scratch regions (masked gradients, partials)
  size_t fscratch_off = 0;                    // per-op scratch of the forward pass (behind the backward's)

  // fp32 stages: the per-layer reductions of weight-gradient partials into G, batched into one
  // launch at the end of every backward pass (device-side task table, built at create)
  void* pack_tasks = nullptr;            // PackTask[]: all packed pointwise-conv copies, one launch
  unsigned short* pack_block_task = nullptr;
  int pack_nblocks = 0;
  void* lsh_tasks = nullptr;             // LinShadowTask[]: the bf16 copies of all dense-layer weights, one launch
  unsigned short* lsh_block_task = nullptr;
  int lsh_nblocks = 0;
  void* red_tasks = nullptr;             // RedTask[]
  void* red_tasks_static = nullptr;      // the same table with the partials' addresses in the static workspace
  char* static_ws = nullptr;             // this device's static workspace, if the stage fits into it
  unsigned short* red_block_task = nullptr;
  int red_nblocks = 0;

  // Grouped weight gradients of the bf16 linear layers: descriptor tables on the device, one per stash
  // slot (the layer inputs live there) and workspace (the stage's own, the static array), index 2*slot + static
  struct WgGroup { void* tasks = nullptr; unsigned short* block_task = nullptr; unsigned* task_block0 = nullptr; };
  std::vector<WgGroup> wg_groups;
  int wg_nblocks = 0;
  // the products are launched in two halves on the second stream: the first as soon as the backward pass has
  // gone through op `wg_split_op` (the gradients its products read exist then) and overlaps the rest of the
  // pass, the second at the end
  int wg_first_blocks = 0, wg_split_op = -1;

  // Second stream for the weight-gradient kernels, which no later kernel of the same
  // backward pass depends on (NULL: everything runs on `stream`).
  hipStream_t side = nullptr;
  std::vector<hipEvent_t> fork_ev;
  hipEvent_t join_ev = nullptr;
  unsigned fork_i = 0;

  // Optional stream of the forward passes (NULL: they run on `stream`).  With K >= 2 the forward of a later
  // micro-batch and the backward of an earlier one touch different stash slots and different scratch, so the
  // two passes may overlap; the events order what does depend: backward(mb) behind forward(mb), a forward that
  // reuses a slot behind the backward that released it, the first forward of a round behind the weight update
  // (behind the main stream's position when that forward is called).
  hipStream_t fwd_stream = nullptr;
  std::vector<hipEvent_t> fwd_done, bwd_done;  // per slot
  std::vector<char> bwd_done_set;              // the slot's bwd_done event has been recorded in this round
  hipEvent_t round_ev = nullptr;

  // 1F1B state
  int next_fwd = 0, next_bwd = 0;
  std::vector<int> mb_slot;
  std::vector<int> free_slots;

  // per-call boundary pointers
  const void* cur_dy = nullptr;
  void* cur_dx = nullptr;
  void* cur_y = nullptr;

};

// plan.cpp
ast_status build_plan(Stage& s, std::string& err);
// exec.cpp
ast_status run_forward(Stage& s, int slot, const void* x, const int32_t* labels, void* y, float* loss,
                       std::string& err);
ast_status run_backward(Stage& s, int slot, const void* dy, void* dx, char* static_ws, std::string& err);
ast_status run_step(Stage& s, float lr, float mu, std::string& err);
ast_status refresh_shadow(Stage& s, std::string& err);
ast_status build_reduce_tasks(Stage& s, std::string& err);  // after the workspace is allocated

}  // namespace ast
