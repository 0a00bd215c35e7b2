// Plan construction: shape inference over the layer list, operator fusion, and the
// layout of the flat arenas, the stash slot and the workspace.  Host code only.
#include <algorithm>
#include <cstdio>
#include <cstdlib>

#include "kernels.h"
#include "kernels_bf16.h"
#include "stage.h"

namespace ast {

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

static std::string fmt(const char* f, int a = 0, int b = 0, int c = 0) {
  char buf[256];
  snprintf(buf, sizeof buf, f, a, b, c);
  return buf;
}

static int new_act(Stage& s, int n, int c, int h, int w, int rank, int layer, int esize) {
  Act a;
  a.n = n; a.c = c; a.h = h; a.w = w; a.rank = rank; a.layer = layer; a.esize = esize;
  a.elems = (size_t)n * c * h * w;
  a.bytes = a.elems * esize;
  s.acts.push_back(a);
  return (int)s.acts.size() - 1;
}

ast_status build_plan(Stage& s, std::string& err) {
  const ast_stage_cfg& cfg = s.cfg;
  const int B = cfg.B;
  const int nl = (int)s.layers.size();
  s.bf16 = cfg.dtype == AST_BF16_F32ACC;
  const int es = s.bf16 ? 2 : 4;
  if (B <= 0 || cfg.M <= 0 || cfg.K <= 0) { err = "B, M, K must be positive"; return AST_EINVAL; }
  if (cfg.dtype != AST_F32 && cfg.dtype != AST_BF16_F32ACC) { err = "unknown dtype"; return AST_EINVAL; }
  if (!s.bf16 && cfg.layout == AST_NHWC) { err = "fp32 stages use NCHW or BSD"; return AST_EUNSUPPORTED; }
  if (s.bf16 && cfg.layout == AST_NCHW) { err = "bf16 stages use NHWC or BSD"; return AST_EUNSUPPORTED; }

  int cur;
  if (cfg.layout == AST_BSD) {
    if (cfg.in_shape[0] <= 0 || cfg.in_shape[1] <= 0) { err = "bad in_shape"; return AST_EINVAL; }
    cur = new_act(s, B, cfg.in_shape[1], cfg.in_shape[0], 1, 3, -1, es);
  } else if (cfg.layout == AST_NCHW || cfg.layout == AST_NHWC) {
    if (cfg.in_shape[0] <= 0 || cfg.in_shape[1] <= 0 || cfg.in_shape[2] <= 0) { err = "bad in_shape"; return AST_EINVAL; }
    cur = new_act(s, B, cfg.in_shape[0], cfg.in_shape[1], cfg.in_shape[2], 4, -1, es);
  } else { err = "unknown layout"; return AST_EINVAL; }

  s.layer_act.assign(nl, -1);
  std::vector<int> res_stack;      // activation ids of open RES_BEGINs
  std::vector<int> res_op_stack;   // op indices of those RES_BEGINs
  std::vector<char> res_swapped;   // per open RES_BEGIN: its shortcut branch has begun (RES_SWAP seen)
  const char* c3env = getenv("ASTEROID_CONV3_MFMA");   // 0: dense 3x3 / strided 1x1 convs on the generic kernels
  const bool conv3_mfma = !c3env || atoi(c3env) != 0;
  std::vector<int> se_stack;       // activation ids of open SE_BEGINs
  bool se_opens = false;           // the previous layer was an SE_BEGIN
  size_t poff = 0, aux = 0, run = 0, shadow = 0;
  auto take_aux = [&](Op& op, size_t bytes) { op.aux_off = aux; op.aux_bytes = bytes; aux = align_up(aux + bytes, 256); };

  for (int i = 0; i < nl; ++i) {
    const ast_layer& L = s.layers[i];
    const Act A = s.acts[cur];
    Op op;
    op.layer = i;
    op.in = cur;
    switch (L.kind) {
      case AST_CONV2D: {
        int Cin = L.p[0], Cout = L.p[1], k = L.p[2], st = L.p[3], pad = L.p[4], g = L.p[5], hb = L.p[6];
        if (A.rank != 4) { err = fmt("layer %d: conv2d needs an image tensor", i); return AST_EINVAL; }
        if (Cin != A.c || Cout <= 0 || k <= 0 || st <= 0 || pad < 0 || g <= 0 || Cin % g || Cout % g) {
          err = fmt("layer %d: conv2d parameters do not match input (C=%d)", i, A.c); return AST_EINVAL; }
        int Ho = (A.h + 2 * pad - k) / st + 1, Wo = (A.w + 2 * pad - k) / st + 1;
        if (A.h + 2 * pad < k || A.w + 2 * pad < k || Ho <= 0 || Wo <= 0) { err = fmt("layer %d: conv2d output is empty", i); return AST_EINVAL; }
        op.cin = Cin; op.cout = Cout; op.k = k; op.stride = st; op.pad = pad; op.groups = g; op.has_bias = hb ? 1 : 0;
        op.w_off = poff; poff += (size_t)Cout * (Cin / g) * k * k;
        if (hb) { op.b_off = poff; poff += Cout; }
        if (!s.bf16 && (size_t)B * std::max((size_t)A.h * A.w, (size_t)Ho * Wo) >= ((size_t)1 << 31)) {  // 32-bit pixel indices
          err = fmt("layer %d: conv2d needs fewer than 2^31 pixels per micro-batch", i);
          return AST_EUNSUPPORTED; }
        if (s.bf16) {
          if (!(g == 1 && (k == 1 || k == 3) && st == 1 && pad == (k - 1) / 2 && Cin % 8 == 0 && Cout % 8 == 0)) {
            err = fmt("layer %d: bf16 conv2d supports dense 1x1/3x3 stride 1 'same' with channels %% 8 == 0", i);
            return AST_EUNSUPPORTED; }
          if ((size_t)B * A.h * A.w * std::max(Cin, Cout) >= ((size_t)1 << 30)) {  // 32-bit byte offsets
            err = fmt("layer %d: bf16 conv2d tensors must stay below 2^30 elements", i);
            return AST_EUNSUPPORTED; }
          op.kind = OP_CONV_IGEMM;
          op.sh_off = shadow; shadow += (size_t)Cout * k * k * Cin;   // [Cout][tap][Cin]
          op.sh2_off = shadow; shadow += (size_t)Cout * k * k * Cin;  // [Cin][tap flipped][Cout]
          if (i + 1 < nl && s.layers[i + 1].kind == AST_RELU) { op.act = 1; ++i; }
        } else if (k == 1 && st == 1 && pad == 0 && g == 1) {
          op.kind = OP_CONV_PW;
        } else if (k == 3 && pad == 1 && g == Cin && Cin == Cout && (st == 1 || st == 2) && !hb &&
                   dw3x3_supported(A.h, A.w, st)) {
          op.kind = OP_CONV_DW;
        } else if (g == Cin && Cin == Cout && pad == k / 2 && !hb && dwk_supported(k, A.h, A.w, st)) {
          op.kind = OP_CONV_DWK;
        } else if (conv3_mfma && conv_mfma_supported(Cin, Cout, k, st, pad, g, A.h, A.w)) {
          op.kind = OP_CONV_3X3;
        } else if (conv3_mfma && conv_gatherk_supported(Cin, Cout, k, st, pad, g, A.h, A.w)) {
          op.kind = OP_CONV_GK;
        } else {
          op.kind = OP_CONV_DIRECT;
        }
        op.out = cur = new_act(s, B, Cout, Ho, Wo, 4, i, es);
        break;
      }
      case AST_BATCHNORM2D: {
        if (s.bf16) { err = fmt("layer %d: BatchNorm is fp32-only", i); return AST_EUNSUPPORTED; }
        if (A.rank != 4 || L.p[0] != A.c) { err = fmt("layer %d: batchnorm channels %d != %d", i, L.p[0], A.c); return AST_EINVAL; }
        op.kind = OP_BN; op.cin = op.cout = A.c; op.eps = L.eps;
        op.w_off = poff; poff += A.c; op.b_off = poff; poff += A.c; op.has_bias = 1;
        op.run_off = run; run += 2 * (size_t)A.c;
        take_aux(op, 4 * sizeof(float) * A.c);  // mean, istd, scale, shift
        if (i + 1 < nl && (s.layers[i + 1].kind == AST_RELU || s.layers[i + 1].kind == AST_RELU6 ||
                           s.layers[i + 1].kind == AST_SWISH)) {
          op.act = s.layers[i + 1].kind == AST_RELU ? 1 : s.layers[i + 1].kind == AST_RELU6 ? 2 : 4; ++i;
        }
        if (i + 1 < nl && s.layers[i + 1].kind == AST_RES_ADD && !res_stack.empty() && !res_swapped.back()) {
          const Act& K = s.acts[res_stack.back()];
          if (K.elems != A.elems || K.c != A.c) { err = fmt("layer %d: residual shapes differ", i + 1); return AST_EINVAL; }
          op.skip = res_stack.back();
          s.ops[res_op_stack.back()].skip = -2;  // patched below once `out` is known
          ++i;
        }
        op.out = cur = new_act(s, B, A.c, A.h, A.w, 4, i, es);
        if (op.skip >= 0) {
          s.ops[res_op_stack.back()].skip = cur;
          res_stack.pop_back(); res_op_stack.pop_back(); res_swapped.pop_back();
        }
        break;
      }
      case AST_RELU: case AST_RELU6: case AST_GELU: case AST_SWISH: case AST_SIGMOID: {
        op.kind = OP_ACT;
        op.act = L.kind == AST_RELU ? 1 : L.kind == AST_RELU6 ? 2 : L.kind == AST_GELU ? 3 : L.kind == AST_SWISH ? 4 : 5;
        if (!s.bf16 && op.act == 3) { err = fmt("layer %d: GELU is bf16-only", i); return AST_EUNSUPPORTED; }
        if (s.bf16 && op.act > 3) { err = fmt("layer %d: swish / sigmoid are fp32-only", i); return AST_EUNSUPPORTED; }
        op.out = cur = new_act(s, A.n, A.c, A.h, A.w, A.rank, i, es);
        break;
      }
      case AST_SE_BEGIN: {
        if (s.bf16 || A.rank != 4) { err = fmt("layer %d: SE_BEGIN needs an fp32 image tensor", i); return AST_EUNSUPPORTED; }
        if (i + 1 >= nl || s.layers[i + 1].kind != AST_GLOBAL_AVGPOOL) {
          err = fmt("layer %d: SE_BEGIN must be followed by GLOBAL_AVGPOOL", i); return AST_EINVAL; }
        op.kind = OP_SE_BEGIN; op.out = cur;
        se_stack.push_back(cur);
        se_opens = true;
        s.layer_act[i] = -1;
        s.ops.push_back(op);
        continue;
      }
      case AST_SE_SCALE: {
        if (se_stack.empty()) { err = fmt("layer %d: SE_SCALE without SE_BEGIN", i); return AST_EINVAL; }
        const Act& X = s.acts[se_stack.back()];
        if (A.rank != 2 || A.n != X.n || A.c != X.c) {
          err = fmt("layer %d: SE_SCALE needs a gate [B][%d]", i, X.c); return AST_EINVAL; }
        op.kind = OP_SE_SCALE; op.skip = se_stack.back();
        se_stack.pop_back();
        op.out = cur = new_act(s, X.n, X.c, X.h, X.w, 4, i, es);
        break;
      }
      case AST_RES_BEGIN: {
        op.kind = OP_RES_BEGIN; op.out = cur; op.skip = -1;
        res_stack.push_back(cur);
        res_swapped.push_back(0);
        res_op_stack.push_back((int)s.ops.size());
        s.layer_act[i] = -1;
        s.ops.push_back(op);
        continue;
      }
      case AST_RES_SWAP: {
        if (res_stack.empty() || res_swapped.back()) { err = fmt("layer %d: RES_SWAP needs an open RES_BEGIN without a RES_SWAP", i); return AST_EINVAL; }
        // The shortcut branch reads the block's input through a second activation entry: same
        // tensor, own gradient buffer.  RES_BEGIN's backward adds that gradient (the shortcut's
        // share) to the one the main branch leaves.
        const Act X = s.acts[res_stack.back()];
        const int alias = new_act(s, X.n, X.c, X.h, X.w, X.rank, i, es);
        s.acts[alias].data_alias = res_stack.back();
        s.ops[res_op_stack.back()].skip = alias;
        op.kind = OP_RES_SWAP; op.out = alias;
        res_stack.back() = cur;   // the main branch's result waits for RES_ADD
        res_swapped.back() = 1;
        cur = alias;
        s.layer_act[i] = -1;
        s.ops.push_back(op);
        continue;
      }
      case AST_RES_ADD: {
        if (res_stack.empty()) { err = fmt("layer %d: RES_ADD without RES_BEGIN", i); return AST_EINVAL; }
        const Act& K = s.acts[res_stack.back()];
        if (K.elems != A.elems || K.c != A.c || K.rank != A.rank) { err = fmt("layer %d: residual shapes differ", i); return AST_EINVAL; }
        op.kind = OP_RES_ADD; op.skip = res_stack.back();
        op.out = cur = new_act(s, A.n, A.c, A.h, A.w, A.rank, i, es);
        if (res_swapped.back()) s.acts[op.skip].grad_alias = cur;  // the main branch's result shares dy with the shortcut's
        else s.ops[res_op_stack.back()].skip = cur;
        res_stack.pop_back(); res_op_stack.pop_back(); res_swapped.pop_back();
        break;
      }
      case AST_GLOBAL_AVGPOOL: {
        if (s.bf16 || A.rank != 4) { err = fmt("layer %d: global avg-pool needs an fp32 image tensor", i); return AST_EUNSUPPORTED; }
        op.kind = OP_GAP;
        op.grad_accum = se_opens;  // the pooled tensor is also scaled by the gate: two gradients meet
        se_opens = false;
        op.out = cur = new_act(s, B, A.c, 1, 1, 2, i, es);
        break;
      }
      case AST_MAXPOOL2X2: {
        if (A.rank != 4 || A.h < 2 || A.w < 2) { err = fmt("layer %d: maxpool needs an image of at least 2x2", i); return AST_EINVAL; }
        if (s.bf16 && A.c % 8) { err = fmt("layer %d: bf16 maxpool needs channels %% 8 == 0", i); return AST_EUNSUPPORTED; }
        op.kind = OP_MAXPOOL; op.k = 2; op.stride = 2; op.pad = 0;
        op.out = cur = new_act(s, B, A.c, A.h / 2, A.w / 2, 4, i, es);
        break;
      }
      case AST_MAXPOOL3X3S2: {
        if (s.bf16 || A.rank != 4) { err = fmt("layer %d: the 3x3 stride-2 max-pool needs an fp32 image tensor", i); return AST_EUNSUPPORTED; }
        op.kind = OP_MAXPOOL; op.k = 3; op.stride = 2; op.pad = 1;
        op.out = cur = new_act(s, B, A.c, (A.h - 1) / 2 + 1, (A.w - 1) / 2 + 1, 4, i, es);
        break;
      }
      case AST_LINEAR: {
        int Cin = L.p[0], Cout = L.p[1], hb = L.p[2];
        if (A.rank == 4 || Cin != A.c || Cout <= 0) { err = fmt("layer %d: linear in=%d does not match input %d", i, Cin, A.c); return AST_EINVAL; }
        if (!s.bf16 && A.rank != 2) { err = fmt("layer %d: fp32 linear works on [B][C] vectors", i); return AST_EUNSUPPORTED; }
        if (s.bf16 && (Cin % 8 || Cout % 8)) { err = fmt("layer %d: bf16 linear needs features %% 8 == 0", i); return AST_EUNSUPPORTED; }
        if (s.bf16 && A.elems / A.c * std::max(Cin, Cout) >= ((size_t)1 << 30)) {  // 32-bit byte offsets
          err = fmt("layer %d: bf16 linear tensors must stay below 2^30 elements", i); return AST_EUNSUPPORTED;
        }
        op.kind = OP_LINEAR; op.cin = Cin; op.cout = Cout; op.has_bias = hb ? 1 : 0;
        op.w_off = poff; poff += (size_t)Cout * Cin;
        if (hb) { op.b_off = poff; poff += Cout; }
        if (s.bf16) {
          op.sh_off = shadow; shadow += (size_t)Cout * Cin;   // W  [Cout][Cin]
          op.sh2_off = shadow; shadow += (size_t)Cout * Cin;  // W^T [Cin][Cout]
          if (i + 1 < nl && s.layers[i + 1].kind == AST_GELU) {
            // pre-activation is stashed for the backward; output = GELU(pre)
            op.act = 3;
            op.skip = new_act(s, A.n, Cout, A.h, A.w, A.rank, i, es);  // pre-activation
            s.layer_act[i] = op.skip;
            ++i;
          }
        }
        bool lin_res = false;
        if (s.bf16 && op.act == 0 && i + 1 < nl && s.layers[i + 1].kind == AST_RES_ADD && !res_stack.empty() &&
            !res_swapped.back()) {
          const Act& K = s.acts[res_stack.back()];  // residual add folded into the output epilogue
          if (K.elems == A.elems / A.c * Cout && K.c == Cout && K.rank == A.rank) {
            op.res_in = res_stack.back();
            lin_res = true;
            ++i;
          }
        }
        op.out = cur = new_act(s, A.n, Cout, A.h, A.w, A.rank, i, es);
        if (lin_res) {
          s.ops[res_op_stack.back()].skip = cur;
          res_stack.pop_back(); res_op_stack.pop_back(); res_swapped.pop_back();
        }
        break;
      }
      case AST_SOFTMAX_CE: {
        if (i != nl - 1) { err = "SOFTMAX_CE must be the last layer"; return AST_EINVAL; }
        if (s.bf16 || A.rank != 2) { err = "SOFTMAX_CE needs fp32 [B][classes] logits"; return AST_EUNSUPPORTED; }
        op.kind = OP_SOFTMAX_CE; op.cout = A.c;
        s.loss_tail = true; s.n_classes = A.c;
        take_aux(op, sizeof(float) * ((size_t)B * A.c + B) + sizeof(int32_t) * B);  // p, row loss, labels
        op.out = cur;  // no new activation: the loss is a scalar
        s.layer_act[i] = -1;
        s.ops.push_back(op);
        continue;
      }
      case AST_LAYERNORM: {
        if (!s.bf16 || A.rank == 4 || L.p[0] != A.c) { err = fmt("layer %d: layernorm needs bf16 rows with D=%d", i, A.c); return s.bf16 ? AST_EINVAL : AST_EUNSUPPORTED; }
        if (A.c % 8 || A.c > 1024) { err = fmt("layer %d: layernorm needs D %% 8 == 0 and D <= 1024", i); return AST_EUNSUPPORTED; }
        op.kind = OP_LAYERNORM; op.cin = op.cout = A.c; op.eps = L.eps;
        op.w_off = poff; poff += A.c; op.b_off = poff; poff += A.c; op.has_bias = 1;
        take_aux(op, 2 * sizeof(float) * (size_t)A.n * A.h);  // mean, istd per row
        op.out = cur = new_act(s, A.n, A.c, A.h, A.w, A.rank, i, es);
        break;
      }
      case AST_MHA: {
        int D = L.p[0], H = L.p[1];
        if (!s.bf16 || A.rank != 3) { err = fmt("layer %d: MHA needs bf16 token input", i); return AST_EUNSUPPORTED; }
        if (D != A.c || H <= 0 || D % H) { err = fmt("layer %d: MHA D=%d heads=%d do not match input", i, D, H); return AST_EINVAL; }
        if (D / H != 64 || A.h % 32 || A.h > 256) { err = fmt("layer %d: MHA kernels cover head size 64 and S %% 32 == 0, S <= 256", i); return AST_EUNSUPPORTED; }
        if ((size_t)A.n * A.h * 3 * D >= ((size_t)1 << 30)) { err = fmt("layer %d: MHA tensors must stay below 2^30 elements", i); return AST_EUNSUPPORTED; }
        op.kind = OP_MHA; op.cin = op.cout = D; op.heads = H; op.has_bias = 1;
        op.w_off = poff; poff += (size_t)3 * D * D + 3 * D + (size_t)D * D + D;
        op.sh_off = shadow; shadow += (size_t)4 * D * D;   // W_qkv [3D][D], W_o [D][D]
        op.sh2_off = shadow; shadow += (size_t)4 * D * D;  // W_qkv^T [D][3D], W_o^T [D][D]
        // per-slot: qkv [rows][3D] bf16, o [rows][D] bf16, lse [B][H][S] fp32
        take_aux(op, (size_t)A.n * A.h * 4 * D * 2 + (size_t)A.n * H * A.h * 4);
        bool mha_res = false;
        if (i + 1 < nl && s.layers[i + 1].kind == AST_RES_ADD && !res_stack.empty() && !res_swapped.back()) {
          const Act& K = s.acts[res_stack.back()];  // residual add folded into the output projection
          if (K.elems == A.elems && K.c == A.c && K.rank == A.rank) {
            op.res_in = res_stack.back();
            mha_res = true;
            ++i;
          }
        }
        op.out = cur = new_act(s, A.n, D, A.h, 1, 3, i, es);
        if (mha_res) {
          s.ops[res_op_stack.back()].skip = cur;
          res_stack.pop_back(); res_op_stack.pop_back(); res_swapped.pop_back();
        }
        break;
      }
      default:
        err = fmt("layer %d: unknown layer kind %d", i, L.kind);
        return AST_EINVAL;
    }
    s.layer_act[i] = cur;
    s.ops.push_back(op);
  }
  if (!res_stack.empty()) { err = "RES_BEGIN without RES_ADD"; return AST_EINVAL; }
  if (!se_stack.empty()) { err = "SE_BEGIN without SE_SCALE"; return AST_EINVAL; }
  if (s.ops.empty()) { err = "empty stage"; return AST_EINVAL; }
  s.nparams = poff;
  s.running_floats = run;
  s.shadow_elems = shadow;
  // fp32 pointwise convs read their weights from packed copies: A = W for the forward
  // product, A = W^T for the input gradient.
  size_t wpk = 0;
  for (Op& op : s.ops)
    if (op.kind == OP_CONV_PW) {
      op.wp_off = wpk; wpk += pw_pack_floats(op.cout, op.cin);
      op.wp2_off = wpk; wpk += pw_pack_floats(op.cin, op.cout);
    } else if (op.kind == OP_CONV_GK) {   // the weights as one [cout][cin*k*k] matrix
      op.wp_off = wpk; wpk += conv_gatherk_pack_floats(op.cin, op.cout, op.k);
    } else if (op.kind == OP_CONV_3X3) {  // k*k copies (one per tap) for each direction
      op.wp_off = wpk; wpk += conv_mfma_pack_floats(op.cout, op.cin, op.k);
      op.wp2_off = wpk; wpk += conv_mfma_pack_floats(op.cin, op.cout, op.k);
    }
  s.wpack_floats = wpk;

  // Squeeze-and-excitation gate: linear -> swish -> linear -> sigmoid between the pooling and the
  // scale becomes one launch per direction (ASTEROID_SE_FUSE=0 keeps the layer-by-layer path).
  {
    const char* e = getenv("ASTEROID_SE_FUSE");
    const bool on = !e || atoi(e) != 0;
    for (size_t j = 1; on && !s.bf16 && j + 4 < s.ops.size(); ++j) {
      Op& l1 = s.ops[j];
      Op& a1 = s.ops[j + 1];
      Op& l2 = s.ops[j + 2];
      Op& a2 = s.ops[j + 3];
      const Op& gp = s.ops[j - 1];
      const Op& sc = s.ops[j + 4];
      if (gp.kind != OP_GAP || !gp.grad_accum || l1.kind != OP_LINEAR || l1.in != gp.out || a1.kind != OP_ACT ||
          a1.act != 4 || a1.in != l1.out || l2.kind != OP_LINEAR || l2.in != a1.out || a2.kind != OP_ACT || a2.act != 5 ||
          a2.in != l2.out || sc.kind != OP_SE_SCALE || sc.in != a2.out)
        continue;
      if (l2.cin != l1.cout || l2.cout != l1.cin || !se_gate_supported(l1.cin, l1.cout)) continue;
      l1.kind = OP_SE_GATE;
      a1.absorbed = l2.absorbed = a2.absorbed = true;
    }
  }

  // GELU backward folded into the input-gradient epilogue of the linear layer that consumes
  // the GELU output: g_pre = (g W) * GELU'(pre).
  for (size_t j = 1; j < s.ops.size(); ++j) {
    Op& pr = s.ops[j - 1];
    Op& nx = s.ops[j];
    if (s.bf16 && pr.kind == OP_LINEAR && pr.act == 3 && nx.kind == OP_LINEAR && nx.in == pr.out) {
      nx.gelu_from = pr.skip;
      pr.gelu_bwd_fused = true;
    }
    // likewise the ReLU of a fused conv+ReLU, masked by its output: g_pre = (conv^T g) * [y > 0]
    if (s.bf16 && pr.kind == OP_CONV_IGEMM && pr.act == 1 && nx.kind == OP_CONV_IGEMM && nx.in == pr.out) {
      nx.relu_from = pr.out;
      pr.relu_bwd_fused = true;
    }
    // ... or a 2x2 max pool behind it: the pool's backward sees the ReLU output anyway (it is its input)
    // and hands the gradient to a window's maximum only where that maximum is positive
    if (s.bf16 && pr.kind == OP_CONV_IGEMM && pr.act == 1 && nx.kind == OP_MAXPOOL && nx.k == 2 && nx.in == pr.out) {
      nx.relu_from = pr.out;
      pr.relu_bwd_fused = true;
    }
  }

  // Fuse the skip-gradient add of a residual block into the input-gradient kernel of the op
  // that opens the block: dx = W^T g + g_skip (pointwise conv, bf16 linear, attention input
  // projection) or dx = LN'(g) + g_skip.
  for (size_t j = 0; j + 1 < s.ops.size(); ++j) {
    Op& rb = s.ops[j];
    Op& nx = s.ops[j + 1];
    const bool can = nx.kind == OP_CONV_PW || nx.kind == OP_LAYERNORM || nx.kind == OP_MHA ||
                     (nx.kind == OP_LINEAR && s.bf16 && nx.gelu_from < 0);
    if (rb.kind == OP_RES_BEGIN && can && nx.in == rb.in && rb.skip >= 0) {
      nx.dgrad_add = rb.skip;
      rb.noop_bwd = true;
    }
  }

  // fp32 inverted-residual pattern BN(+act) -> depthwise 3x3 -> BN: BatchNorm passes move into the
  // convolution.  ASTEROID_BN_FUSE is a bit mask of the moves to make (default: all):
  //   1  forward: the first BatchNorm's apply pass (normalise on load, also in the conv's backward)
  //      and the second one's statistics pass (conv epilogue)
  //   2  backward: the first BatchNorm's partial sums (conv backward epilogue); needs 1
  //   4  backward: the second BatchNorm's apply pass (on load of the conv's upstream gradient)
  //   8  see below (pointwise conv -> BatchNorm)
  std::vector<char> virtual_act(s.acts.size(), 0);  // activations that are never materialised
  {
    const char* e = getenv("ASTEROID_BN_FUSE");
    const int fuse = e ? atoi(e) : 15;
    for (size_t j = 0; fuse && j < s.ops.size(); ++j) {
      Op& dw = s.ops[j];
      if (dw.kind != OP_CONV_DW) continue;
      const Act& DI = s.acts[dw.in];
      const int dparts = dw3x3_parts(DI.n, DI.c, DI.h, DI.w, dw.stride);  // partial sums per channel it leaves
      if (j > 0 && (fuse & 1)) {
        Op& bn = s.ops[j - 1];
        // (the conv's kernels apply ReLU / ReLU6 only, and mask by the recomputed activated value)
        if (bn.kind == OP_BN && bn.out == dw.in && bn.skip < 0 && bn.act <= 2) {
          bn.bn_lazy = true;
          bn.bn_bwd_sums_given = (fuse & 2) != 0;
          bn.given_bwd_parts = dparts;
          dw.bn_in_op = (int)j - 1;
          virtual_act[bn.out] = 1;
          for (int& la : s.layer_act)
            if (la == bn.out) la = -1;
        }
      }
      if (j + 1 < s.ops.size()) {
        Op& bn = s.ops[j + 1];
        if (bn.kind == OP_BN && bn.in == dw.out) {
          if (fuse & 1) {
            bn.bn_stats_given = true;
            bn.given_parts = dparts;
            dw.bn_out_op = (int)j + 1;
          }
          if ((fuse & 4) && bn.act <= 2) {  // the conv's kernels know ReLU / ReLU6 only
            bn.bn_bwd_apply_fused = true;
            dw.bn_bwd_out_op = (int)j + 1;
          }
        }
      }
    }
  }

  // ... and bit 8: a pointwise conv (no bias) directly in front of a BatchNorm leaves that
  // BatchNorm's statistics partials in its epilogue, where its launch shape offers them.
  {
    const char* e = getenv("ASTEROID_BN_FUSE");
    const int fuse = e ? atoi(e) : 15;
    for (size_t j = 0; (fuse & 8) && j + 1 < s.ops.size(); ++j) {
      Op& pw = s.ops[j];
      Op& bn = s.ops[j + 1];
      if (pw.kind != OP_CONV_PW || pw.has_bias || bn.kind != OP_BN || bn.in != pw.out || bn.bn_stats_given) continue;
      const Act& I = s.acts[pw.in];
      const int parts = pw_conv_stats_parts(I.n, pw.cin, pw.cout, I.h * I.w);
      if (parts <= 0) continue;
      bn.bn_stats_given = true;
      bn.given_parts = parts;
      pw.stats_op = (int)j + 1;
    }
  }

  // Stash slot: every activation (the stage input is copied in; the final output goes to
  // the caller's buffer) followed by the per-op extras.
  size_t off = 0;
  const int final_act = cur;
  s.final_act = cur;
  // An op that masks its upstream gradient by its own OUTPUT needs that output in the backward.
  for (const Op& op : s.ops)
    if (op.out == cur && op.kind != OP_RES_BEGIN && op.kind != OP_SOFTMAX_CE &&
        ((op.kind == OP_CONV_IGEMM && op.act) || (op.kind == OP_ACT && s.bf16 && op.act != 3)))
      s.final_in_slot = true;
  for (size_t a = 0; a < s.acts.size(); ++a) {
    if ((int)a == final_act && !s.loss_tail && a != 0 && !s.final_in_slot) continue;
    if (virtual_act[a] || s.acts[a].data_alias >= 0) continue;
    s.acts[a].slot_off = off;
    off = align_up(off + s.acts[a].bytes, 256);
  }
  for (Act& a : s.acts)  // a shortcut branch's input is the tensor RES_BEGIN remembered
    if (a.data_alias >= 0) a.slot_off = s.acts[a.data_alias].slot_off;
  for (Op& op : s.ops) op.aux_off += off;
  s.slot_bytes = align_up(off + aux, 256);

  // Gradient workspace: one buffer per activation except the stage input (caller's dx)
  // and the final output (caller's dy).
  size_t goff = 0;
  for (size_t a = 0; a < s.acts.size(); ++a) {
    if (a == 0) continue;
    if ((int)a == final_act && !s.loss_tail) continue;
    s.acts[a].grad_off = goff;
    goff = align_up(goff + s.acts[a].bytes, 256);
  }
  // RES_ADD passes its output gradient through unchanged: share the buffer.
  for (Op& op : s.ops)
    if (op.kind == OP_RES_ADD) s.acts[op.in].grad_alias = op.out;
  s.grad_bytes = goff;

  // Scratch: one private region per op (masked upstream gradients, reduction partials), so
  // that kernels of different ops may overlap on two streams without sharing a buffer.
  size_t sc = 0;
  for (Op& op : s.ops) {
    const Act& I = s.acts[op.in];
    size_t need = 0;
    switch (op.kind) {
      case OP_CONV_PW: need = pw_wgrad_f32_ws(I.n, op.cin, op.cout, I.h * I.w) * sizeof(float); break;
      case OP_CONV_DW: need = dw3x3_bwd_f32_ws(I.n, I.c, I.h, I.w, op.stride) * sizeof(float); break;
      case OP_CONV_DWK: need = dwk_bwd_f32_ws(I.n, I.c, op.k) * sizeof(float); break;
      case OP_CONV_GK:
        need = std::max(conv_gatherk_wgrad_ws(I.n, op.cin, op.cout, I.h, I.w, op.k, op.stride, op.pad),
                        conv_direct_wgrad_ws(I.n, op.cin, I.h, I.w, op.cout, op.k, op.stride, op.pad, op.groups)) * sizeof(float);
        break;
      case OP_CONV_3X3: need = conv_mfma_wgrad_ws(I.n, op.cin, op.cout, I.h, I.w, op.k, op.stride) * sizeof(float); break;
      case OP_CONV_DIRECT:
        need = conv_direct_wgrad_ws(I.n, op.cin, I.h, I.w, op.cout, op.k, op.stride, op.pad, op.groups) * sizeof(float);
        break;
      case OP_BN:
        need = std::max(bn_ws_doubles(I.c, I.n, I.h * I.w),
                        (size_t)2 * I.c * std::max(op.given_parts, op.given_bwd_parts)) * sizeof(double);
        break;
      case OP_CONV_IGEMM:  // masked upstream gradient + split-K partials
        need = align_up(s.acts[op.out].bytes, 256) + conv_bf16_ws_bytes(I.n, I.h, I.w, op.cin, op.cout, op.k);
        break;
      case OP_LINEAR:
        if (s.bf16)
          need = align_up(s.acts[op.out].bytes, 256) + linear_bf16_ws_bytes((size_t)I.n * I.h * I.w, op.cin, op.cout);
        break;
      case OP_LAYERNORM: need = layernorm_bf16_ws_bytes((size_t)I.n * I.h, I.c); break;
      case OP_MHA:  // d_o and dqkv, the row sums, then the split-K partials of each projection
        need = align_up((size_t)I.n * I.h * 4 * op.cin * 2, 256) +
               align_up(mha_bf16_ws_bytes(I.n, I.h, op.cin, op.heads), 256) +
               align_up(linear_bf16_ws_bytes((size_t)I.n * I.h, op.cin, op.cin), 256) +
               linear_bf16_ws_bytes((size_t)I.n * I.h, op.cin, 3 * op.cin);
        break;
      default: break;
    }
    op.sc_off = sc;
    sc += align_up(need, 256);
  }
  // The forward pass has scratch of its own (BatchNorm statistics partials), so that the forward of one
  // micro-batch may run beside the backward of another.
  size_t fsc = 0;
  for (Op& op : s.ops) {
    if (op.kind != OP_BN) continue;
    const Act& I = s.acts[op.in];
    op.fsc_off = fsc;
    fsc += align_up(std::max(bn_ws_doubles(I.c, I.n, I.h * I.w), (size_t)2 * I.c * op.given_parts) * sizeof(double), 256);
  }
  s.scratch_off = align_up(goff, 256);
  s.scratch_bytes = align_up(sc, 256);
  s.fscratch_off = s.scratch_off + s.scratch_bytes;
  s.ws_bytes = s.fscratch_off + align_up(fsc, 256) + 256;
  return AST_OK;
}

}  // namespace ast
