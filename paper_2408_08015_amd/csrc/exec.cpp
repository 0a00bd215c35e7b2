// Plan execution: forward, backward and optimizer step of a stage, as kernel launches
// on the stage's stream.  No allocation, no host synchronisation.
#include <cstdint>
#include <cstdlib>
#include <vector>

#include "kernels.h"
#include "kernels_bf16.h"
#include "stage.h"
#include "static_scratch.h"

namespace ast {

namespace {

struct Ctx {
  Stage& s;
  char* slot;
  int final_act;
  char* ws;  // workspace of this call: the stage's own, or the static array (backward_static)
  hipStream_t st;  // stream of this pass
  bool forked = false;
};

inline int final_act_of(const Stage& s) { return s.final_act; }

inline void* act_ptr(Ctx& c, int id) {
  if (id == c.final_act && !c.s.loss_tail && id != 0 && !c.s.final_in_slot) return c.s.cur_y;
  return c.slot + c.s.acts[id].slot_off;
}
inline void* grad_ptr(Ctx& c, int id) {
  while (c.s.acts[id].grad_alias >= 0) id = c.s.acts[id].grad_alias;
  if (id == 0) return c.s.cur_dx;  // may be NULL: the input gradient is not wanted
  if (id == c.final_act && !c.s.loss_tail) return const_cast<void*>(c.s.cur_dy);  // id != 0 here
  return c.ws + c.s.acts[id].grad_off;
}
inline char* scratch(Ctx& c, const Op& op) { return c.ws + c.s.scratch_off + op.sc_off; }
// scratch of the forward pass (BatchNorm statistics partials): always in the stage's own workspace
inline char* fscratch(Ctx& c, const Op& op) { return c.s.ws + c.s.fscratch_off + op.fsc_off; }
// Stream for a weight-gradient kernel.  Nothing later in the same backward pass reads a
// parameter gradient, so these kernels leave the dependency chain: they run on the stage's
// second stream, ordered after all work enqueued so far on the main stream, and the pass
// joins the two streams before it returns.  Kernels that accumulate into the same
// parameter all run on that one stream, so the accumulation order stays fixed.
// The hand-over between two hardware queues costs several microseconds, so only the bf16
// GEMM-sized weight gradients take it; the fp32 ones (tens of microseconds each) stay put.
inline hipStream_t fork_side(Ctx& c) {
  Stage& s = c.s;
  if (!s.side || !s.bf16) return s.stream;
  hipEvent_t e = s.fork_ev[s.fork_i++ % s.fork_ev.size()];
  (void)hipEventRecord(e, s.stream);
  (void)hipStreamWaitEvent(s.side, e, 0);
  c.forked = true;
  return s.side;
}
inline size_t align256(size_t v) { return (v + 255) / 256 * 256; }
// attention scratch: [d_o, dqkv][row sums of dO*O][weight-gradient partials ...]
inline size_t mha_lw_offset(int B, int S, int D, int heads) {
  return align256((size_t)B * S * 4 * D * sizeof(bf16_t)) + align256(mha_bf16_ws_bytes(B, S, D, heads));
}

typedef const float* cf;
typedef const bf16_t* cb;

void fwd_op(Ctx& c, const Op& op, const int32_t* labels, float* loss) {
  Stage& s = c.s;
  hipStream_t st = c.st;
  const Act& I = s.acts[op.in];
  const int HW = I.h * I.w;
  if (op.absorbed) return;
  switch (op.kind) {
    case OP_SE_GATE: {  // this op is the first linear layer; swish, the second linear layer and sigmoid follow it
      const Op* q = &op;
      const Op &a1 = q[1], &l2 = q[2], &a2 = q[3];
      se_gate_fwd_f32(st, (cf)act_ptr(c, op.in), s.W + op.w_off, op.has_bias ? s.W + op.b_off : nullptr, s.W + l2.w_off,
                      l2.has_bias ? s.W + l2.b_off : nullptr, (float*)act_ptr(c, op.out), (float*)act_ptr(c, a1.out),
                      (float*)act_ptr(c, l2.out), (float*)act_ptr(c, a2.out), I.n, op.cin, op.cout);
      break;
    }
    case OP_CONV_PW:
      pw_conv_f32(st, s.wpack + op.wp_off, (cf)act_ptr(c, op.in), (float*)act_ptr(c, op.out),
                  op.has_bias ? s.W + op.b_off : nullptr, nullptr, I.n, op.cin, op.cout, HW,
                  op.stats_op >= 0 ? reinterpret_cast<double*>(fscratch(c, s.ops[op.stats_op])) : nullptr);
      break;
    case OP_CONV_DW:
    {
      DwBnIn bi{};
      cf x = (cf)act_ptr(c, op.in);
      if (op.bn_in_op >= 0) {  // normalise the BatchNorm's input on load; finish and record its statistics
        const Op& bn = s.ops[op.bn_in_op];
        const Act& BI = s.acts[bn.in];
        float* aux = reinterpret_cast<float*>(c.slot + bn.aux_off);
        x = (cf)act_ptr(c, bn.in);
        bi.ws = reinterpret_cast<const double*>(fscratch(c, bn));
        bi.gamma = s.W + bn.w_off; bi.beta = s.W + bn.b_off;
        bi.stat = aux; bi.ss = aux + 2 * I.c; bi.running = s.running + bn.run_off;
        bi.count = (double)BI.n * BI.h * BI.w; bi.eps = bn.eps;
        bi.P = bn.bn_stats_given ? bn.given_parts : bn_parts(BI.n, BI.h * BI.w);
        bi.act = bn.act; bi.on = 1;
      }
      dw3x3_fwd_f32(st, x, s.W + op.w_off, (float*)act_ptr(c, op.out), I.n, I.c, I.h, I.w, op.stride,
                    op.bn_in_op >= 0 ? &bi : nullptr,
                    op.bn_out_op >= 0 ? reinterpret_cast<double*>(fscratch(c, s.ops[op.bn_out_op])) : nullptr);
      break;
    }
    case OP_CONV_GK:
      conv_gatherk_fwd_f32(st, s.wpack + op.wp_off, (cf)act_ptr(c, op.in), (float*)act_ptr(c, op.out),
                           op.has_bias ? s.W + op.b_off : nullptr, I.n, op.cin, op.cout, I.h, I.w, op.k, op.stride, op.pad);
      break;
    case OP_CONV_3X3:
      conv_mfma_fwd_f32(st, s.wpack + op.wp_off, (cf)act_ptr(c, op.in), (float*)act_ptr(c, op.out),
                        op.has_bias ? s.W + op.b_off : nullptr, I.n, op.cin, op.cout, I.h, I.w, op.k, op.stride);
      break;
    case OP_CONV_DWK:
      dwk_fwd_f32(st, (cf)act_ptr(c, op.in), s.W + op.w_off, (float*)act_ptr(c, op.out), I.n, I.c, I.h, I.w, op.k,
                  op.stride);
      break;
    case OP_CONV_DIRECT:
      conv_direct_fwd_f32(st, (cf)act_ptr(c, op.in), s.W + op.w_off, op.has_bias ? s.W + op.b_off : nullptr,
                          (float*)act_ptr(c, op.out), I.n, op.cin, I.h, I.w, op.cout, op.k, op.stride,
                          op.pad, op.groups);
      break;
    case OP_CONV_IGEMM:
      conv_bf16_fwd(st, (cb)act_ptr(c, op.in), s.shadow + op.sh_off, op.has_bias ? s.W + op.b_off : nullptr,
                    (bf16_t*)act_ptr(c, op.out), I.n, I.h, I.w, op.cin, op.cout, op.k, op.act);
      break;
    case OP_BN: {
      float* aux = reinterpret_cast<float*>(c.slot + op.aux_off);
      double* ws = reinterpret_cast<double*>(fscratch(c, op));
      cf x = (cf)act_ptr(c, op.in);
      if (!op.bn_stats_given && !op.bn_lazy && op.act != 4 && bn_onepass_fits(I.n, HW)) {  // small tensor: one launch
        bn_fwd_onepass_f32(st, x, s.W + op.w_off, s.W + op.b_off, op.skip >= 0 ? (cf)act_ptr(c, op.skip) : nullptr,
                           (float*)act_ptr(c, op.out), aux, aux + 2 * I.c, s.running + op.run_off, I.n, I.c, HW, op.eps,
                           op.act);
        break;
      }
      // statistics: from the depthwise conv in front (one partial pair per plane) or a pass of its own
      if (!op.bn_stats_given) bn_stats_f32(st, x, ws, I.n, I.c, HW);
      if (!op.bn_lazy)  // else the depthwise conv behind normalises on load
        bn_apply_f32(st, x, s.W + op.w_off, s.W + op.b_off, op.skip >= 0 ? (cf)act_ptr(c, op.skip) : nullptr,
                     (float*)act_ptr(c, op.out), aux, aux + 2 * I.c, s.running + op.run_off, ws,
                     op.bn_stats_given ? op.given_parts : bn_parts(I.n, HW), I.n, I.c, HW, op.eps, op.act);
      break;
    }
    case OP_ACT:
      if (s.bf16) act_fwd_bf16(st, (cb)act_ptr(c, op.in), (bf16_t*)act_ptr(c, op.out), I.elems, op.act);
      else act_fwd_f32(st, (cf)act_ptr(c, op.in), (float*)act_ptr(c, op.out), I.elems, op.act);
      break;
    case OP_RES_BEGIN:
    case OP_RES_SWAP:
    case OP_SE_BEGIN:
      break;
    case OP_SE_SCALE: {
      const Act& X = s.acts[op.skip];
      se_scale_fwd_f32(st, (cf)act_ptr(c, op.skip), (cf)act_ptr(c, op.in), (float*)act_ptr(c, op.out), X.n * X.c, X.h * X.w);
      break;
    }
    case OP_RES_ADD:
      if (s.bf16) add_bf16(st, (cb)act_ptr(c, op.in), (cb)act_ptr(c, op.skip), (bf16_t*)act_ptr(c, op.out), I.elems);
      else add_f32(st, (cf)act_ptr(c, op.in), (cf)act_ptr(c, op.skip), (float*)act_ptr(c, op.out), I.elems);
      break;
    case OP_GAP:
      gap_fwd_f32(st, (cf)act_ptr(c, op.in), (float*)act_ptr(c, op.out), I.n * I.c, HW);
      break;
    case OP_MAXPOOL:
      if (s.bf16) maxpool_fwd_bf16(st, (cb)act_ptr(c, op.in), (bf16_t*)act_ptr(c, op.out), I.n, I.h, I.w, I.c);
      else if (op.k == 3) maxpool3x3s2_fwd_f32(st, (cf)act_ptr(c, op.in), (float*)act_ptr(c, op.out), I.n * I.c, I.h, I.w);
      else maxpool_fwd_f32(st, (cf)act_ptr(c, op.in), (float*)act_ptr(c, op.out), I.n * I.c, I.h, I.w);
      break;
    case OP_LINEAR:
      if (s.bf16) {
        linear_bf16_fwd(st, (cb)act_ptr(c, op.in), s.shadow + op.sh_off, op.has_bias ? s.W + op.b_off : nullptr,
                        (bf16_t*)act_ptr(c, op.out), op.act == 3 ? (bf16_t*)act_ptr(c, op.skip) : nullptr,
                        op.res_in >= 0 ? (cb)act_ptr(c, op.res_in) : nullptr, (size_t)I.n * I.h * I.w, op.cin, op.cout,
                        op.act);
      } else {
        linear_fwd_f32(st, (cf)act_ptr(c, op.in), s.W + op.w_off, op.has_bias ? s.W + op.b_off : nullptr,
                       (float*)act_ptr(c, op.out), I.n, op.cin, op.cout);
      }
      break;
    case OP_SOFTMAX_CE: {
      float* p = reinterpret_cast<float*>(c.slot + op.aux_off);
      float* row_loss = p + (size_t)I.n * I.c;
      int32_t* lab = reinterpret_cast<int32_t*>(row_loss + I.n);
      copy_bytes(st, labels, lab, sizeof(int32_t) * I.n);
      softmax_ce_fwd_f32(st, (cf)act_ptr(c, op.in), lab, p, row_loss, loss, I.n, I.c,
                         1.f / ((float)s.cfg.M * (float)s.cfg.B));
      if (s.cur_y) copy_bytes(st, act_ptr(c, op.in), s.cur_y, I.bytes);
      break;
    }
    case OP_LAYERNORM:
      layernorm_fwd_bf16(st, (cb)act_ptr(c, op.in), s.W + op.w_off, s.W + op.b_off, (bf16_t*)act_ptr(c, op.out),
                         reinterpret_cast<float*>(c.slot + op.aux_off), (size_t)I.n * I.h, I.c, op.eps);
      break;
    case OP_MHA: {
      const int D = op.cin;
      const size_t R = (size_t)I.n * I.h;
      bf16_t* qkv = reinterpret_cast<bf16_t*>(c.slot + op.aux_off);
      bf16_t* o = qkv + R * 3 * D;
      float* lse = reinterpret_cast<float*>(o + R * D);
      const float* bq = s.W + op.w_off + (size_t)3 * D * D;
      const float* bo = bq + 3 * D + (size_t)D * D;
      linear_bf16_fwd(st, (cb)act_ptr(c, op.in), s.shadow + op.sh_off, bq, qkv, nullptr, nullptr, R, D, 3 * D, 0);
      attention_fwd_bf16(st, qkv, o, lse, I.n, I.h, D, op.heads);
      linear_bf16_fwd(st, o, s.shadow + op.sh_off + (size_t)3 * D * D, bo, (bf16_t*)act_ptr(c, op.out), nullptr,
                      op.res_in >= 0 ? (cb)act_ptr(c, op.res_in) : nullptr, R, D, D, 0);
      break;
    }
  }
}

void bwd_op(Ctx& c, const Op& op) {
  Stage& s = c.s;
  hipStream_t st = s.stream;
  const Act& I = s.acts[op.in];
  const int HW = I.h * I.w;
  void* gin = grad_ptr(c, op.in);  // NULL: not wanted
  if (op.absorbed) return;
  switch (op.kind) {
    case OP_SE_GATE: {
      const Op* q = &op;
      const Op &a1 = q[1], &l2 = q[2], &a2 = q[3];
      se_gate_bwd_f32(st, (cf)grad_ptr(c, a2.out), (cf)act_ptr(c, l2.out), (cf)act_ptr(c, op.out), (cf)act_ptr(c, op.in),
                      (cf)act_ptr(c, a1.out), s.W + op.w_off, s.W + l2.w_off, (float*)grad_ptr(c, l2.out),
                      (float*)grad_ptr(c, op.out), (float*)gin, s.G + op.w_off, op.has_bias ? s.G + op.b_off : nullptr,
                      s.G + l2.w_off, l2.has_bias ? s.G + l2.b_off : nullptr, I.n, op.cin, op.cout);
      break;
    }
    case OP_CONV_PW: {
      cf g = (cf)grad_ptr(c, op.out);
      float* part = reinterpret_cast<float*>(scratch(c, op));
      float* Gw = s.red_nblocks ? nullptr : s.G + op.w_off;
      if (gin)  // input gradient and weight-gradient partials share one launch
        pw_conv_bwd_f32(st, s.wpack + op.wp2_off, g, (float*)gin,
                        op.dgrad_add >= 0 ? (cf)grad_ptr(c, op.dgrad_add) : nullptr, (cf)act_ptr(c, op.in), part, Gw,
                        I.n, op.cin, op.cout, HW);
      else
        pw_wgrad_f32(st, g, (cf)act_ptr(c, op.in), part, Gw, I.n, op.cin, op.cout, HW);
      if (op.has_bias) channel_sum_acc_f32(st, g, s.G + op.b_off, I.n, op.cout, HW);
      break;
    }
    case OP_CONV_DW: {
      cf g = (cf)grad_ptr(c, op.out);
      cf x = (cf)act_ptr(c, op.in);
      DwBwdFuse f;
      if (op.bn_in_op >= 0) {  // recompute the BatchNorm output from its input and recorded coefficients
        const Op& bn = s.ops[op.bn_in_op];
        const float* aux = reinterpret_cast<const float*>(c.slot + bn.aux_off);
        x = (cf)act_ptr(c, bn.in);
        f.xss = aux + 2 * I.c;
        f.xact = bn.act;
        if (bn.bn_bwd_sums_given) {  // and leave that BatchNorm's backward sums, one pair per plane
          f.xstat = aux;
          f.ws_in = reinterpret_cast<double*>(scratch(c, bn));
        }
      }
      if (op.bn_bwd_out_op >= 0) {  // the upstream gradient is still the BatchNorm's: finish its backward on load
        const Op& bn = s.ops[op.bn_bwd_out_op];
        const Act& O = s.acts[op.out];
        const float* aux = reinterpret_cast<const float*>(c.slot + bn.aux_off);
        g = (cf)grad_ptr(c, bn.out);
        f.y = (cf)act_ptr(c, op.out);
        f.ystat = aux; f.yss = aux + 2 * O.c; f.ygamma = s.W + bn.w_off;
        f.ws_out = reinterpret_cast<const double*>(scratch(c, bn));
        f.Ggamma = s.G + bn.w_off; f.Gbeta = s.G + bn.b_off;
        f.ycount = (double)O.n * O.h * O.w;
        f.P_out = bn.bn_bwd_sums_given ? bn.given_bwd_parts : bn_parts(O.n, O.h * O.w);
        f.yact = bn.act;
      }
      dw3x3_bwd_f32(st, g, x, s.W + op.w_off, (float*)gin, reinterpret_cast<float*>(scratch(c, op)),
                    s.red_nblocks ? nullptr : s.G + op.w_off, I.n, I.c, I.h, I.w, op.stride, &f);
      break;
    }
    case OP_CONV_GK: {
      cf g = (cf)grad_ptr(c, op.out);
      const Act& O = s.acts[op.out];
      if (gin)  // rarely wanted (the layer is a model's first): the generic kernel
        conv_direct_dgrad_f32(st, g, s.W + op.w_off, (float*)gin, I.n, op.cin, I.h, I.w, op.cout, op.k, op.stride, op.pad,
                              op.groups);
      conv_gatherk_wgrad_f32(st, g, (cf)act_ptr(c, op.in), reinterpret_cast<float*>(scratch(c, op)),
                             s.red_nblocks ? nullptr : s.G + op.w_off, I.n, op.cin, op.cout, I.h, I.w, op.k, op.stride, op.pad);
      if (op.has_bias) channel_sum_acc_f32(st, g, s.G + op.b_off, I.n, op.cout, O.h * O.w);
      break;
    }
    case OP_CONV_3X3: {
      cf g = (cf)grad_ptr(c, op.out);
      const Act& O = s.acts[op.out];
      conv_mfma_bwd_f32(st, s.wpack + op.wp2_off, g, (float*)gin, (cf)act_ptr(c, op.in),
                        reinterpret_cast<float*>(scratch(c, op)), s.red_nblocks ? nullptr : s.G + op.w_off, I.n, op.cin,
                        op.cout, I.h, I.w, op.k, op.stride);
      if (op.has_bias) channel_sum_acc_f32(st, g, s.G + op.b_off, I.n, op.cout, O.h * O.w);
      break;
    }
    case OP_CONV_DWK:
      dwk_bwd_f32(st, (cf)grad_ptr(c, op.out), (cf)act_ptr(c, op.in), s.W + op.w_off, (float*)gin,
                  reinterpret_cast<float*>(scratch(c, op)), s.G + op.w_off, I.n, I.c, I.h, I.w, op.k, op.stride);
      break;
    case OP_CONV_DIRECT: {
      cf g = (cf)grad_ptr(c, op.out);
      const Act& O = s.acts[op.out];
      hipStream_t sw = fork_side(c);
      if (gin)
        conv_direct_dgrad_f32(st, g, s.W + op.w_off, (float*)gin, I.n, op.cin, I.h, I.w, op.cout, op.k,
                              op.stride, op.pad, op.groups);
      conv_direct_wgrad_f32(sw, g, (cf)act_ptr(c, op.in), s.G + op.w_off, reinterpret_cast<float*>(scratch(c, op)),
                            I.n, op.cin, I.h, I.w, op.cout,
                            op.k, op.stride, op.pad, op.groups);
      if (op.has_bias) channel_sum_acc_f32(sw, g, s.G + op.b_off, I.n, op.cout, O.h * O.w);
      break;
    }
    case OP_CONV_IGEMM: {
      const Act& O = s.acts[op.out];
      cb g = (cb)grad_ptr(c, op.out);
      char* sc = scratch(c, op);  // [masked upstream gradient][weight-gradient partials]
      if (op.act && !op.relu_bwd_fused) {  // mask by the ReLU output
        bf16_t* gm = reinterpret_cast<bf16_t*>(sc);
        act_bwd_bf16(st, g, (cb)act_ptr(c, op.out), gm, O.elems, op.act);
        g = gm;
      }
      sc += align256(O.bytes);
      hipStream_t sw = fork_side(c);
      if (gin)
        conv_bf16_dgrad(st, g, s.shadow + op.sh2_off, (bf16_t*)gin,
                        op.relu_from >= 0 ? (cb)act_ptr(c, op.relu_from) : nullptr, I.n, I.h, I.w, op.cin, op.cout, op.k);
      conv_bf16_wgrad(sw, g, (cb)act_ptr(c, op.in), s.G + op.w_off, s.G + op.b_off, op.has_bias != 0, s.red_nblocks != 0,
                      sc, I.n, I.h, I.w, op.cin, op.cout, op.k);
      break;
    }
    case OP_BN: {
      float* aux = reinterpret_cast<float*>(c.slot + op.aux_off);
      double* ws = reinterpret_cast<double*>(scratch(c, op));
      cf g = (cf)grad_ptr(c, op.out), x = (cf)act_ptr(c, op.in);
      // partial sums: left per plane by the backward of the depthwise conv behind (it ran just before), or
      // a pass of its own; input gradient: formed by the depthwise conv in front on load, or a pass of its own
      const bool given = op.bn_bwd_sums_given;
      if (!given && !op.bn_bwd_apply_fused && op.act != 4 && bn_onepass_fits(I.n, HW)) {  // small tensor: one launch
        bn_bwd_onepass_f32(st, g, x, aux, aux + 2 * I.c, s.W + op.w_off, (float*)gin, s.G + op.w_off, s.G + op.b_off, I.n,
                           I.c, HW, op.act);
        break;
      }
      if (!given) bn_bwd_partial_f32(st, g, x, aux, aux + 2 * I.c, ws, I.n, I.c, HW, op.act);
      if (!op.bn_bwd_apply_fused)
        bn_bwd_apply_f32(st, g, x, aux, aux + 2 * I.c, s.W + op.w_off, ws, given ? op.given_bwd_parts : bn_parts(I.n, HW), (float*)gin,
                         s.G + op.w_off, s.G + op.b_off, I.n, I.c, HW, op.act);
      break;
    }
    case OP_ACT:
      if (!gin) break;
      if (s.bf16)
        act_bwd_bf16(st, (cb)grad_ptr(c, op.out), op.act == 3 ? (cb)act_ptr(c, op.in) : (cb)act_ptr(c, op.out),
                     (bf16_t*)gin, I.elems, op.act);
      else
        act_bwd_f32(st, (cf)grad_ptr(c, op.out), (cf)act_ptr(c, op.in), (float*)gin, I.elems, op.act);
      break;
    case OP_SE_BEGIN:  // both gradients of the tensor are already in its buffer (OP_SE_SCALE, then the pool)
    case OP_RES_SWAP:
      break;
    case OP_SE_SCALE: {
      const Act& X = s.acts[op.skip];
      se_scale_bwd_f32(st, (cf)grad_ptr(c, op.out), (cf)act_ptr(c, op.skip), (cf)act_ptr(c, op.in), (float*)gin,
                       (float*)grad_ptr(c, op.skip), X.n * X.c, X.h * X.w);
      break;
    }
    case OP_RES_BEGIN:
      if (op.noop_bwd || !gin || op.skip < 0) break;
      if (s.bf16) add_bf16(st, (cb)gin, (cb)grad_ptr(c, op.skip), (bf16_t*)gin, I.elems);
      else add_f32(st, (cf)gin, (cf)grad_ptr(c, op.skip), (float*)gin, I.elems);
      break;
    case OP_RES_ADD:
      if (gin && gin != grad_ptr(c, op.out)) copy_bytes(st, grad_ptr(c, op.out), gin, I.bytes);
      break;
    case OP_GAP:
      if (gin) gap_bwd_f32(st, (cf)grad_ptr(c, op.out), (float*)gin, I.n * I.c, HW, op.grad_accum);
      break;
    case OP_MAXPOOL:
      if (!gin) break;
      if (s.bf16)
        maxpool_bwd_bf16(st, (cb)grad_ptr(c, op.out), (cb)act_ptr(c, op.in), (bf16_t*)gin, I.n, I.h, I.w, I.c,
                         op.relu_from >= 0);
      else if (op.k == 3)
        maxpool3x3s2_bwd_f32(st, (cf)grad_ptr(c, op.out), (cf)act_ptr(c, op.in), (float*)gin, I.n * I.c, I.h, I.w);
      else maxpool_bwd_f32(st, (cf)grad_ptr(c, op.out), (cf)act_ptr(c, op.in), (float*)gin, I.n * I.c, I.h, I.w);
      break;
    case OP_LINEAR:
      if (s.bf16) {
        const Act& O = s.acts[op.out];
        const size_t R = (size_t)I.n * I.h * I.w;
        cb g = (cb)grad_ptr(c, op.out);
        char* sc = scratch(c, op);  // [GELU-masked upstream gradient][weight-gradient partials]
        if (op.act == 3 && !op.gelu_bwd_fused) {
          bf16_t* gp = reinterpret_cast<bf16_t*>(sc);
          act_bwd_bf16(st, g, (cb)act_ptr(c, op.skip), gp, O.elems, 3);
          g = gp;
        }
        sc += align256(O.bytes);
        hipStream_t sw = op.wg_grouped ? st : fork_side(c);
        if (gin)
          linear_bf16_dgrad(st, g, s.shadow + op.sh2_off, (bf16_t*)gin,
                            op.gelu_from >= 0 ? (cb)act_ptr(c, op.gelu_from) : nullptr,
                            op.dgrad_add >= 0 ? (cb)grad_ptr(c, op.dgrad_add) : nullptr, R, op.cin, op.cout);
        if (!op.wg_grouped)  // else: part of the grouped launch at the end of the pass
          linear_bf16_wgrad(sw, g, (cb)act_ptr(c, op.in), s.G + op.w_off, s.G + op.b_off, op.has_bias != 0,
                            s.red_nblocks != 0, sc, R, op.cin, op.cout);
      } else {
        cf g = (cf)grad_ptr(c, op.out);
        hipStream_t sw = fork_side(c);
        if (gin) linear_dgrad_f32(st, g, s.W + op.w_off, (float*)gin, I.n, op.cin, op.cout);
        linear_wgrad_f32(sw, g, (cf)act_ptr(c, op.in), s.G + op.w_off, op.has_bias ? s.G + op.b_off : nullptr,
                         I.n, op.cin, op.cout);
      }
      break;
    case OP_SOFTMAX_CE: {
      float* p = reinterpret_cast<float*>(c.slot + op.aux_off);
      int32_t* lab = reinterpret_cast<int32_t*>(p + (size_t)I.n * I.c + I.n);
      softmax_ce_bwd_f32(st, p, lab, (float*)gin, I.n, I.c, 1.f / ((float)s.cfg.M * (float)s.cfg.B));
      break;
    }
    case OP_LAYERNORM:
      layernorm_bwd_bf16(st, (cb)grad_ptr(c, op.out), (cb)act_ptr(c, op.in),
                         reinterpret_cast<float*>(c.slot + op.aux_off), s.W + op.w_off,
                         (gin && op.dgrad_add >= 0) ? (cb)grad_ptr(c, op.dgrad_add) : nullptr, (bf16_t*)gin,
                         scratch(c, op), (size_t)I.n * I.h, I.c);
      // the parameter gradients only need the partials of the kernel above
      if (!s.red_nblocks)
        layernorm_bwd_params_bf16(fork_side(c), scratch(c, op), s.G + op.w_off, s.G + op.b_off, (size_t)I.n * I.h, I.c);
      break;
    case OP_MHA: {
      const int D = op.cin;
      const size_t R = (size_t)I.n * I.h;
      bf16_t* qkv = reinterpret_cast<bf16_t*>(c.slot + op.aux_off);
      bf16_t* o = qkv + R * 3 * D;
      float* lse = reinterpret_cast<float*>(o + R * D);
      float* Gq = s.G + op.w_off;
      float* Gbq = Gq + (size_t)3 * D * D;
      float* Go = Gbq + 3 * D;
      float* Gbo = Go + (size_t)D * D;
      char* sc = scratch(c, op);
      bf16_t* d_o = reinterpret_cast<bf16_t*>(sc);
      bf16_t* dqkv = d_o + R * D;
      float* dsum = reinterpret_cast<float*>(sc + align256(R * 4 * D * sizeof(bf16_t)));
      // partials of the two projections' weight gradients: output projection, then qkv
      char* lw_o = sc + mha_lw_offset(I.n, I.h, D, op.heads);
      char* lw_q = lw_o + align256(linear_bf16_ws_bytes(R, D, D));
      const bool defer = s.red_nblocks != 0;
      cb g = (cb)grad_ptr(c, op.out);
      hipStream_t sw = op.wg_grouped ? st : fork_side(c);
      linear_bf16_dgrad(st, g, s.shadow + op.sh2_off + (size_t)3 * D * D, d_o, nullptr, nullptr, R, D, D);
      if (!op.wg_grouped) linear_bf16_wgrad(sw, g, o, Go, Gbo, true, defer, lw_o, R, D, D);
      attention_bwd_bf16(st, qkv, o, d_o, lse, dqkv, dsum, I.n, I.h, D, op.heads);
      if (!op.wg_grouped) sw = fork_side(c);
      if (gin)
        linear_bf16_dgrad(st, dqkv, s.shadow + op.sh2_off, (bf16_t*)gin, nullptr,
                          op.dgrad_add >= 0 ? (cb)grad_ptr(c, op.dgrad_add) : nullptr, R, D, 3 * D);
      if (!op.wg_grouped) linear_bf16_wgrad(sw, dqkv, (cb)act_ptr(c, op.in), Gq, Gbq, true, defer, lw_q, R, D, 3 * D);
      break;
    }
  }
}

ast_status check_launch(std::string& err, const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    err = std::string(what) + ": " + hipGetErrorString(e);
    return AST_EHIP;
  }
  return AST_OK;
}

}  // namespace

ast_status run_forward(Stage& s, int slot, const void* x, const int32_t* labels, void* y, float* loss,
                       std::string& err) {
  const bool two = s.fwd_stream != nullptr;
  Ctx c{s, s.slots[slot], final_act_of(s), s.ws, two ? s.fwd_stream : s.stream};
  s.cur_y = y;
  s.cur_dy = nullptr;
  s.cur_dx = nullptr;
  if (two) {
    if (s.next_fwd == 0) {
      // a round's first forward starts behind whatever the main stream holds at this moment: the previous
      // round's backward passes and weight update (a fork from the main stream, so a caller may also capture
      // a whole round into a graph from there)
      (void)hipEventRecord(s.round_ev, s.stream);
      (void)hipStreamWaitEvent(c.st, s.round_ev, 0);
      s.bwd_done_set.assign(s.bwd_done_set.size(), 0);
    }
    if (s.bwd_done_set[slot]) (void)hipStreamWaitEvent(c.st, s.bwd_done[slot], 0);  // the slot's previous reader
  }
  copy_bytes(c.st, x, c.slot + s.acts[0].slot_off, s.acts[0].bytes);
  for (const Op& op : s.ops) fwd_op(c, op, labels, loss);
  if (s.final_in_slot && !s.loss_tail)
    copy_bytes(c.st, c.slot + s.acts[s.final_act].slot_off, y, s.acts[s.final_act].bytes);
  if (two) (void)hipEventRecord(s.fwd_done[slot], c.st);
  return check_launch(err, "forward");
}

ast_status run_backward(Stage& s, int slot, const void* dy, void* dx, char* static_ws, std::string& err) {
  Ctx c{s, s.slots[slot], final_act_of(s), static_ws ? static_ws : s.ws, s.stream};
  if (s.fwd_stream) (void)hipStreamWaitEvent(s.stream, s.fwd_done[slot], 0);  // the stash of this micro-batch
  if (static_ws) static_scratch_zero(s.stream, static_ws, s.ws_bytes);  // what the stage's own workspace was at create
  s.cur_y = nullptr;
  s.cur_dy = dy;
  s.cur_dx = dx;
  // the weight (and bias) gradients of all grouped linear layers: two launches on the second stream, each
  // adding its products into G (every entry of G belongs to one block of one launch)
  const Stage::WgGroup* wg = s.wg_nblocks ? &s.wg_groups[2 * slot + (static_ws ? 1 : 0)] : nullptr;
  for (int j = (int)s.ops.size() - 1; j >= 0; --j) {
    bwd_op(c, s.ops[j]);
    if (wg && j == s.wg_split_op)
      wgrad_group_launch(fork_side(c), wg->tasks, wg->block_task, wg->task_block0, 0, s.wg_first_blocks);
  }
  if (wg)
    wgrad_group_launch(fork_side(c), wg->tasks, wg->block_task, wg->task_block0, s.wg_first_blocks,
                       s.wg_nblocks - s.wg_first_blocks);
  if (s.red_nblocks)  // every layer's partials -> G, one launch (behind all of this pass's kernels)
    reduce_tasks_f32(fork_side(c), static_cast<const RedTask*>(static_ws ? s.red_tasks_static : s.red_tasks), s.red_block_task,
                     s.red_nblocks);
  if (c.forked) {  // join: whatever follows on the main stream sees every gradient
    (void)hipEventRecord(s.join_ev, s.side);
    (void)hipStreamWaitEvent(s.stream, s.join_ev, 0);
  }
  if (s.fwd_stream) {  // the slot is free for a later forward from here on
    (void)hipEventRecord(s.bwd_done[slot], s.stream);
    s.bwd_done_set[slot] = 1;
  }
  return check_launch(err, "backward");
}

static ast_status build_pack_tasks(Stage& s, std::string& err) {
  std::vector<PackTask> tasks;
  std::vector<unsigned short> block_task;
  auto add = [&](const float* W, int lda_m, int lda_k, size_t off, int Mdim, int Kdim) {
    PackTask t = {};
    t.W = W; t.lda_m = lda_m; t.lda_k = lda_k; t.Mdim = Mdim; t.Kdim = Kdim; t.KG = (Kdim + 7) / 8;
    t.block0 = (unsigned)block_task.size();
    if (off != (size_t)t.block0 * 256) return false;  // the arena is laid out in op order: cannot happen
    for (size_t b = 0; b < pw_pack_floats(Mdim, Kdim) / 256; ++b) block_task.push_back((unsigned short)tasks.size());
    tasks.push_back(t);
    return true;
  };
  for (const Op& op : s.ops)
    if (op.kind == OP_CONV_PW) {
      if (tasks.size() + 2 >= 65535) return AST_OK;  // per-conv launches instead
      if (!add(s.W + op.w_off, op.cin, 1, op.wp_off, op.cout, op.cin) ||
          !add(s.W + op.w_off, 1, op.cin, op.wp2_off, op.cin, op.cout))
        return AST_OK;
    } else if (op.kind == OP_CONV_GK) {
      if (tasks.size() + 1 >= 65535) return AST_OK;
      const int kd = op.cin * op.k * op.k;
      if (!add(s.W + op.w_off, kd, 1, op.wp_off, op.cout, kd)) return AST_OK;
    } else if (op.kind == OP_CONV_3X3) {
      // W[co][ci][tap]: forward copy t is A[co][ci] = W[..][t]; input-gradient copy t is A[ci][co] = W[..][t]
      const int kk = op.k * op.k;
      if (tasks.size() + 2 * kk >= 65535) return AST_OK;
      const float* W = s.W + op.w_off;
      for (int t = 0; t < kk; ++t)
        if (!add(W + t, op.cin * kk, kk, op.wp_off + t * pw_pack_floats(op.cout, op.cin), op.cout, op.cin)) return AST_OK;
      for (int t = 0; t < kk; ++t)
        if (!add(W + t, kk, op.cin * kk, op.wp2_off + t * pw_pack_floats(op.cin, op.cout), op.cin, op.cout)) return AST_OK;
    }
  if (tasks.empty()) return AST_OK;
  hipError_t e;
  if ((e = hipMalloc(&s.pack_tasks, tasks.size() * sizeof(PackTask))) != hipSuccess ||
      (e = hipMalloc((void**)&s.pack_block_task, block_task.size() * sizeof(unsigned short))) != hipSuccess ||
      (e = hipMemcpy(s.pack_tasks, tasks.data(), tasks.size() * sizeof(PackTask), hipMemcpyHostToDevice)) != hipSuccess ||
      (e = hipMemcpy(s.pack_block_task, block_task.data(), block_task.size() * sizeof(unsigned short),
                     hipMemcpyHostToDevice)) != hipSuccess) {
    err = std::string("pack task table: ") + hipGetErrorString(e);
    return e == hipErrorOutOfMemory ? AST_ENOMEM : AST_EHIP;
  }
  s.pack_nblocks = (int)block_task.size();
  return AST_OK;
}

// The bf16 copies of all dense-layer weight matrices (linear layers, attention projections) in one launch.
static ast_status build_linear_shadow_tasks(Stage& s, std::string& err) {
  if (!s.bf16) return AST_OK;
  std::vector<LinShadowTask> tasks;
  std::vector<unsigned short> block_task;
  auto add = [&](const float* w, size_t sh_off, size_t sh2_off, int Cout, int Cin, size_t R) {
    LinShadowTask t = {};
    t.w = w; t.sh = s.shadow + sh_off; t.sht = s.shadow + sh2_off; t.Cout = Cout; t.Cin = Cin;
    t.tiled = linear_dl_supported(R, Cin, Cout) ? 1 : 0;   // the kernel each direction will run decides the layout
    t.tiled_t = linear_dl_supported(R, Cout, Cin) ? 1 : 0;
    t.block0 = (unsigned)block_task.size();
    for (unsigned b = 0; b < linear_shadow_blocks(Cout, Cin); ++b) block_task.push_back((unsigned short)tasks.size());
    tasks.push_back(t);
  };
  for (const Op& op : s.ops) {
    if (tasks.size() + 2 >= 65535) return AST_OK;  // per-layer launches instead
    const Act& I = s.acts[op.in];
    if (op.kind == OP_LINEAR) {
      add(s.W + op.w_off, op.sh_off, op.sh2_off, op.cout, op.cin, (size_t)I.n * I.h * I.w);
    } else if (op.kind == OP_MHA) {
      const int D = op.cin;
      const size_t R = (size_t)I.n * I.h;
      const float* wq = s.W + op.w_off;
      add(wq, op.sh_off, op.sh2_off, 3 * D, D, R);
      add(wq + (size_t)3 * D * D + 3 * D, op.sh_off + (size_t)3 * D * D, op.sh2_off + (size_t)3 * D * D, D, D, R);
    }
  }
  if (tasks.size() < 2) return AST_OK;
  hipError_t e;
  if ((e = hipMalloc(&s.lsh_tasks, tasks.size() * sizeof(LinShadowTask))) != hipSuccess ||
      (e = hipMalloc((void**)&s.lsh_block_task, block_task.size() * sizeof(unsigned short))) != hipSuccess ||
      (e = hipMemcpy(s.lsh_tasks, tasks.data(), tasks.size() * sizeof(LinShadowTask), hipMemcpyHostToDevice)) != hipSuccess ||
      (e = hipMemcpy(s.lsh_block_task, block_task.data(), block_task.size() * sizeof(unsigned short),
                     hipMemcpyHostToDevice)) != hipSuccess) {
    err = std::string("weight copy task table: ") + hipGetErrorString(e);
    return e == hipErrorOutOfMemory ? AST_ENOMEM : AST_EHIP;
  }
  s.lsh_nblocks = (int)block_task.size();
  return AST_OK;
}

// Grouped weight gradients (bf16 stages): every linear layer and attention projection whose operands lie
// in the stash and the workspace (i.e. not in a buffer of the caller) becomes one product of a single
// launch at the end of the backward pass.  ASTEROID_WGRAD_GROUP=0 keeps the per-layer launches.
static ast_status build_wgrad_groups(Stage& s, char* static_ws, std::string& err) {
  if (!s.bf16) return AST_OK;
  if (const char* e = getenv("ASTEROID_WGRAD_GROUP"))
    if (e[0] == '0') return AST_OK;
  // addresses as forward / backward will compute them, or NULL where they depend on the call
  auto act_at = [&](char* slot, int id) -> char* {
    if (id == s.final_act && !s.loss_tail && id != 0 && !s.final_in_slot) return nullptr;  // the caller's y
    return slot + s.acts[id].slot_off;
  };
  auto grad_at = [&](char* ws, int id) -> char* {
    while (s.acts[id].grad_alias >= 0) id = s.acts[id].grad_alias;
    if (id == 0 || (id == s.final_act && !s.loss_tail)) return nullptr;  // the caller's dx / dy
    return ws + s.acts[id].grad_off;
  };
  struct Prod { const bf16_t* dy; const bf16_t* x; float* GW; float* Gb; size_t rows; int cin, cout; };
  auto products = [&](const Op& op, char* slot, char* ws, std::vector<Prod>& out) -> bool {
    const Act& I = s.acts[op.in];
    char* sc = ws + s.scratch_off + op.sc_off;
    if (op.kind == OP_LINEAR) {
      const size_t R = (size_t)I.n * I.h * I.w;
      char* g = (op.act == 3 && !op.gelu_bwd_fused) ? sc : grad_at(ws, op.out);  // the GELU-masked gradient lies in the scratch
      char* x = act_at(slot, op.in);
      if (!g || !x || !wgrad_group_supported(R, op.cin, op.cout)) return false;
      out.push_back({(const bf16_t*)g, (const bf16_t*)x, s.G + op.w_off, op.has_bias ? s.G + op.b_off : nullptr, R, op.cin, op.cout});
      return true;
    }
    if (op.kind == OP_MHA) {
      const int D = op.cin;
      const size_t R = (size_t)I.n * I.h;
      bf16_t* qkv = reinterpret_cast<bf16_t*>(slot + op.aux_off);
      bf16_t* o = qkv + R * 3 * D;
      bf16_t* dqkv = reinterpret_cast<bf16_t*>(sc) + R * D;
      float* Gq = s.G + op.w_off;
      float* Gbq = Gq + (size_t)3 * D * D;
      float* Go = Gbq + 3 * D;
      float* Gbo = Go + (size_t)D * D;
      char* g = grad_at(ws, op.out);
      char* x = act_at(slot, op.in);
      if (!g || !x || !wgrad_group_supported(R, D, 3 * D)) return false;
      out.push_back({(const bf16_t*)g, o, Go, Gbo, R, D, D});
      out.push_back({dqkv, (const bf16_t*)x, Gq, Gbq, R, D, 3 * D});
      return true;
    }
    return false;
  };
  // which ops take part (the same for every slot and workspace)
  bool any = false;
  for (Op& op : s.ops) {
    std::vector<Prod> tmp;
    op.wg_grouped = !op.absorbed && (op.kind == OP_LINEAR || op.kind == OP_MHA) && products(op, s.slots[0], s.ws, tmp);
    any = any || op.wg_grouped;
  }
  if (!any) return AST_OK;
  const size_t tb = wgrad_group_task_bytes();
  s.wg_groups.assign(2 * s.slots.size(), Stage::WgGroup());
  for (size_t k = 0; k < s.slots.size(); ++k)
    for (int v = 0; v < (static_ws ? 2 : 1); ++v) {
      std::vector<Prod> prods;
      std::vector<int> prod_op;
      for (int j = (int)s.ops.size() - 1; j >= 0; --j)  // the order of the backward pass
        if (s.ops[j].wg_grouped) {
          products(s.ops[j], s.slots[k], v ? static_ws : s.ws, prods);
          prod_op.resize(prods.size(), j);
        }
      std::vector<char> tasks(prods.size() * tb);
      std::vector<unsigned short> block_task;
      std::vector<unsigned> block0;
      for (size_t t = 0; t < prods.size(); ++t) {
        const Prod& p = prods[t];
        const int nb = wgrad_group_task(tasks.data() + t * tb, p.dy, p.x, p.GW, p.Gb, p.rows, p.cin, p.cout);
        block0.push_back((unsigned)block_task.size());
        for (int b = 0; b < nb; ++b) block_task.push_back((unsigned short)t);
      }
      if (prods.size() >= 65535) {  // (absurdly long stage) back to per-layer launches
        for (Op& op : s.ops) op.wg_grouped = false;
        s.wg_groups.clear();
        return AST_OK;
      }
      Stage::WgGroup& wg = s.wg_groups[2 * k + v];
      hipError_t e;
      if ((e = hipMalloc(&wg.tasks, tasks.size())) != hipSuccess ||
          (e = hipMalloc((void**)&wg.block_task, block_task.size() * sizeof(unsigned short))) != hipSuccess ||
          (e = hipMalloc((void**)&wg.task_block0, block0.size() * sizeof(unsigned))) != hipSuccess ||
          (e = hipMemcpy(wg.tasks, tasks.data(), tasks.size(), hipMemcpyHostToDevice)) != hipSuccess ||
          (e = hipMemcpy(wg.block_task, block_task.data(), block_task.size() * sizeof(unsigned short), hipMemcpyHostToDevice)) != hipSuccess ||
          (e = hipMemcpy(wg.task_block0, block0.data(), block0.size() * sizeof(unsigned), hipMemcpyHostToDevice)) != hipSuccess) {
        err = std::string("grouped weight-gradient table: ") + hipGetErrorString(e);
        return e == hipErrorOutOfMemory ? AST_ENOMEM : AST_EHIP;
      }
      s.wg_nblocks = (int)block_task.size();
      // first launch: the products of the ops the pass reaches first, up to about half of the blocks
      s.wg_first_blocks = 0;
      s.wg_split_op = -1;
      for (size_t t = 0; t + 1 < prods.size(); ++t)
        if (prod_op[t + 1] != prod_op[t] && (int)block0[t + 1] * 2 >= s.wg_nblocks) {
          s.wg_first_blocks = (int)block0[t + 1];
          s.wg_split_op = prod_op[t];
          break;
        }
    }
  return AST_OK;
}

ast_status build_reduce_tasks(Stage& s, std::string& err) {
  if (ast_status r = build_pack_tasks(s, err)) return r;
  if (ast_status r = build_linear_shadow_tasks(s, err)) return r;
  char* static_ws = nullptr;
  if (s.ws_bytes <= kStaticScratchBytes) {
    std::string ignore;
    (void)static_scratch_ptr(&static_ws, ignore);  // no static variant for this stage if this fails
  }
  s.static_ws = static_ws;
  if (const char* e = getenv("ASTEROID_BATCHED_REDUCE"))
    if (e[0] == '0') return AST_OK;  // per-layer reduction launches instead
  if (ast_status r = build_wgrad_groups(s, static_ws, err)) return r;
  // the table holds absolute addresses of the partials: one table per workspace the backward
  // may run in (the stage's own; the static array, if the stage fits into it)
  for (int pass = 0; pass < (static_ws ? 2 : 1); ++pass) {
  char* const ws_base = pass == 0 ? s.ws : static_ws;
  std::vector<RedTask> tasks;
  std::vector<unsigned short> block_task;
  bool overflow = false;
  auto add = [&](const float* part, float* G, size_t n, int parts, size_t stride, int taps, size_t mn) {
    if (tasks.size() >= 65535 || n >= 0xffffffffu || stride >= 0xffffffffu) { overflow = true; return; }
    RedTask t = {};
    t.part = part; t.G = G;
    t.n = (unsigned)n; t.parts = (unsigned)parts; t.stride = (unsigned)stride;
    t.taps = (unsigned)taps; t.mn = (unsigned)mn;
    t.block0 = (unsigned)block_task.size();
    // many outputs, few partials: 16-byte loads, a thread sums all partials of its outputs
    t.wide = (n >= 16384 && n % 4 == 0 && stride % 4 == 0 && (reinterpret_cast<uintptr_t>(part) & 15) == 0) ? 1u : 0u;
    const size_t per_block = t.wide ? 1024 : 64;
    for (size_t b = 0; b < (n + per_block - 1) / per_block; ++b) block_task.push_back((unsigned short)tasks.size());
    tasks.push_back(t);
  };
  auto add_wgrad = [&](float* base, const WgradParts& wp, float* GW, float* Gb, size_t cout, size_t cin, int taps) {
    const size_t mn = cout * cin;
    add(base, GW, taps * mn, wp.splits, taps * mn, taps, mn);
    if (Gb) add(base + wp.bias_off, Gb, cout, wp.bias_parts, cout, 1, cout);
  };
  for (const Op& op : s.ops) {
    const Act& I = s.acts[op.in];
    char* sc = ws_base + s.scratch_off + op.sc_off;
    float* scf = reinterpret_cast<float*>(sc);
    switch (op.kind) {
      case OP_CONV_PW: {
        const size_t n = (size_t)op.cin * op.cout;
        add(scf, s.G + op.w_off, n, pw_wgrad_f32_parts(I.n, op.cin, op.cout, I.h * I.w), n, 1, n);
        break;
      }
      case OP_CONV_GK: {
        const size_t n = (size_t)op.cin * op.cout * op.k * op.k;
        add(scf, s.G + op.w_off, n, conv_gatherk_wgrad_parts(I.n, op.cin, op.cout, I.h, I.w, op.k, op.stride, op.pad), n, 1, n);
        break;
      }
      case OP_CONV_3X3: {
        const size_t n = (size_t)op.cin * op.cout * op.k * op.k;
        add(scf, s.G + op.w_off, n, conv_mfma_wgrad_parts(I.n, op.cin, op.cout, I.h, I.w, op.k, op.stride), n, 1, n);
        break;
      }
      case OP_CONV_DW:
        add(scf, s.G + op.w_off, (size_t)I.c * 9, dw3x3_parts(I.n, I.c, I.h, I.w, op.stride), (size_t)I.c * 9, 1, (size_t)I.c * 9);
        break;
      case OP_CONV_IGEMM:
        add_wgrad(reinterpret_cast<float*>(sc + align256(s.acts[op.out].bytes)),
                  conv_bf16_wgrad_parts(I.n, I.h, I.w, op.cin, op.cout, op.k), s.G + op.w_off,
                  op.has_bias ? s.G + op.b_off : nullptr, op.cout, op.cin, op.k * op.k);
        break;
      case OP_LINEAR:
        if (s.bf16 && !op.wg_grouped)
          add_wgrad(reinterpret_cast<float*>(sc + align256(s.acts[op.out].bytes)),
                    linear_bf16_wgrad_parts((size_t)I.n * I.h * I.w, op.cin, op.cout), s.G + op.w_off,
                    op.has_bias ? s.G + op.b_off : nullptr, op.cout, op.cin, 1);
        break;
      case OP_MHA: {
        const int D = op.cin;
        const size_t R = (size_t)I.n * I.h;
        float* Gq = s.G + op.w_off;
        float* Gbq = Gq + (size_t)3 * D * D;
        float* Go = Gbq + 3 * D;
        float* Gbo = Go + (size_t)D * D;
        char* lw_o = sc + mha_lw_offset(I.n, I.h, D, op.heads);
        char* lw_q = lw_o + align256(linear_bf16_ws_bytes(R, D, D));
        if (op.wg_grouped) break;
        add_wgrad(reinterpret_cast<float*>(lw_o), linear_bf16_wgrad_parts(R, D, D), Go, Gbo, D, D, 1);
        add_wgrad(reinterpret_cast<float*>(lw_q), linear_bf16_wgrad_parts(R, D, 3 * D), Gq, Gbq, (size_t)3 * D, D, 1);
        break;
      }
      case OP_LAYERNORM: {
        const int parts = layernorm_bwd_parts((size_t)I.n * I.h);
        add(scf, s.G + op.w_off, I.c, parts, (size_t)2 * I.c, 1, I.c);          // dgamma
        add(scf + I.c, s.G + op.b_off, I.c, parts, (size_t)2 * I.c, 1, I.c);    // dbeta
        break;
      }
      default: break;
    }
  }
  if (tasks.empty() || overflow) return AST_OK;  // (absurdly long stage: per-layer launches)
  hipError_t e;
  void** table = pass == 0 ? &s.red_tasks : &s.red_tasks_static;
  if ((e = hipMalloc(table, tasks.size() * sizeof(RedTask))) != hipSuccess ||
      (e = hipMemcpy(*table, tasks.data(), tasks.size() * sizeof(RedTask), hipMemcpyHostToDevice)) != hipSuccess ||
      (pass == 0 &&
       ((e = hipMalloc((void**)&s.red_block_task, block_task.size() * sizeof(unsigned short))) != hipSuccess ||
        (e = hipMemcpy(s.red_block_task, block_task.data(), block_task.size() * sizeof(unsigned short),
                       hipMemcpyHostToDevice)) != hipSuccess))) {
    err = std::string("reduction task table: ") + hipGetErrorString(e);
    return e == hipErrorOutOfMemory ? AST_ENOMEM : AST_EHIP;
  }
  if (pass == 0) s.red_nblocks = (int)block_task.size();
  }
  return AST_OK;
}

ast_status refresh_shadow(Stage& s, std::string& err) {
  if (s.pack_nblocks)
    pw_pack_all_f32(s.stream, static_cast<const PackTask*>(s.pack_tasks), s.pack_block_task, s.wpack, s.pack_nblocks);
  if (s.lsh_nblocks)
    linear_weight_shadow_all_bf16(s.stream, static_cast<const LinShadowTask*>(s.lsh_tasks), s.lsh_block_task, s.lsh_nblocks);
  for (const Op& op : s.ops) {
    if (op.kind == OP_CONV_PW) {
      if (s.pack_nblocks) continue;
      pw_pack_f32(s.stream, s.W + op.w_off, op.cin, 1, s.wpack + op.wp_off, op.cout, op.cin);
      pw_pack_f32(s.stream, s.W + op.w_off, 1, op.cin, s.wpack + op.wp2_off, op.cin, op.cout);
    } else if (op.kind == OP_CONV_GK) {
      if (s.pack_nblocks) continue;
      const int kd = op.cin * op.k * op.k;
      pw_pack_f32(s.stream, s.W + op.w_off, kd, 1, s.wpack + op.wp_off, op.cout, kd);
    } else if (op.kind == OP_CONV_3X3) {
      if (s.pack_nblocks) continue;
      const float* W = s.W + op.w_off;
      const int kk = op.k * op.k;
      for (int t = 0; t < kk; ++t) {
        pw_pack_f32(s.stream, W + t, op.cin * kk, kk, s.wpack + op.wp_off + t * pw_pack_floats(op.cout, op.cin), op.cout,
                    op.cin);
        pw_pack_f32(s.stream, W + t, kk, op.cin * kk, s.wpack + op.wp2_off + t * pw_pack_floats(op.cin, op.cout), op.cin,
                    op.cout);
      }
    } else if (!s.bf16) {
      continue;  // the remaining copies are bf16 layouts
    } else if (op.kind == OP_CONV_IGEMM) {
      const Act& I = s.acts[op.in];  // the kernel each direction will run decides the layout of its copy
      conv_weight_shadow_bf16(s.stream, s.W + op.w_off, s.shadow + op.sh_off, s.shadow + op.sh2_off, op.cout,
                              op.cin, op.k, conv_bf16_uses_halo(I.n, I.h, I.w, op.cin, op.cout, op.k),
                              conv_bf16_uses_halo(I.n, I.h, I.w, op.cout, op.cin, op.k));
    } else if (s.lsh_nblocks) {
      continue;  // the dense-layer copies went out in one launch above
    } else if (op.kind == OP_LINEAR) {
      const Act& I = s.acts[op.in];  // the kernel each direction will run decides the layout of its copy
      const size_t R = (size_t)I.n * I.h * I.w;
      linear_weight_shadow_bf16(s.stream, s.W + op.w_off, s.shadow + op.sh_off, s.shadow + op.sh2_off, op.cout,
                                op.cin, linear_dl_supported(R, op.cin, op.cout), linear_dl_supported(R, op.cout, op.cin));
    } else if (op.kind == OP_MHA) {
      const int D = op.cin;
      const float* wq = s.W + op.w_off;
      const float* wo = wq + (size_t)3 * D * D + 3 * D;
      const Act& I = s.acts[op.in];
      const size_t R = (size_t)I.n * I.h;
      linear_weight_shadow_bf16(s.stream, wq, s.shadow + op.sh_off, s.shadow + op.sh2_off, 3 * D, D,
                                linear_dl_supported(R, D, 3 * D), linear_dl_supported(R, 3 * D, D));
      linear_weight_shadow_bf16(s.stream, wo, s.shadow + op.sh_off + (size_t)3 * D * D,
                                s.shadow + op.sh2_off + (size_t)3 * D * D, D, D, linear_dl_supported(R, D, D),
                                linear_dl_supported(R, D, D));
    }
  }
  return check_launch(err, "weight copy refresh");
}

ast_status run_step(Stage& s, float lr, float mu, std::string& err) {
  sgd_momentum_f32(s.stream, s.W, s.G, s.V, s.nparams, lr, mu);
  ast_status r = check_launch(err, "step");
  if (r != AST_OK) return r;
  return refresh_shadow(s, err);
}

}  // namespace ast
