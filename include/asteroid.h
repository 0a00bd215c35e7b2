/*
 * asteroid.h -- C ABI of the MI355X stage-training library.
 *
 * One object = one pipeline stage held by one device: a "stage model" made of
 * consecutive network layers (Sec. 3.2, "HPP Architecture and Workflow").  A
 * mini-batch is split into M micro-batches of size B; the device runs the forward
 * pass (FP) and backward pass (BP) of its stage model per micro-batch, accumulates
 * gradients over all M micro-batches, and applies them to the parameters once at
 * the end of the mini-batch (one "HPP-Round", Sec. 3.2).  Micro-batches are
 * scheduled one-forward-one-backward after K warm-up forwards, so at most K
 * micro-batches' activations are alive (Sec. 3.2, "Memory-efficient 1F1B
 * Micro-batch Scheduling"; memory model Eq. (3)).
 *
 * Pointer conventions: every `*_dev` argument is DEVICE memory owned by the
 * caller and must be 16-byte aligned (AST_EINVAL otherwise); every `host_*`
 * argument is HOST memory owned by the caller.  The library
 * owns parameters, accumulated gradients, optimizer state, reduced-precision
 * weight copies, the activation stash and its workspace; all are allocated in
 * asteroid_stage_create and none in forward/backward/step.
 *
 * All work is enqueued on the HIP stream given at creation (the forward passes on a
 * second one after asteroid_stage_set_forward_stream) and is asynchronous to the host.
 * forward / backward / step consist of kernel launches and event waits only - no
 * allocation, no memset, no host synchronisation - so the calls of a whole round may be
 * recorded into a HIP graph by stream capture on the creation stream and replayed (the
 * buffers, lr and momentum of the recording are then the graph's; the checks of the
 * call discipline happen while recording).
 * Every function returns an ast_status; nothing throws or aborts.
 * asteroid_last_error() gives a thread-local message for the last failure.
 */
#ifndef ASTEROID_H
#define ASTEROID_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct asteroid_stage asteroid_stage; /* opaque */

typedef enum {
  AST_OK = 0,
  AST_EINVAL = -1,       /* bad argument, shape mismatch, NULL where a buffer is required */
  AST_ESTATE = -2,       /* 1F1B discipline violated (see forward/backward/step)           */
  AST_ENOMEM = -3,       /* device allocation failed in create                            */
  AST_EHIP = -4,         /* a HIP runtime call failed                                     */
  AST_EUNSUPPORTED = -5  /* layer kind / shape the kernels do not cover                   */
} ast_status;

/* Arithmetic of the stage.
 *   AST_F32:          fp32 activations, weights and arithmetic.
 *   AST_BF16_F32ACC:  bf16 activations and weight copies as matrix operands, fp32
 *                     accumulation; fp32 master weights, gradients and velocity.
 *                     Boundary tensors x, y, dy, dx are bf16. */
typedef enum { AST_F32 = 0, AST_BF16_F32ACC = 1 } ast_dtype;

/* Memory order of boundary tensors (and of activations inside the stage).
 *   AST_NCHW: [B][C][H][W]     AST_NHWC: [B][H][W][C]     AST_BSD: [B][S][D] tokens. */
typedef enum { AST_NCHW = 0, AST_NHWC = 1, AST_BSD = 2 } ast_layout;

/* The layer sequence of a stage model (a model is a topologically sorted sequence of
 * layers, split only between layers; Sec. 3.3 "Asteroid Profiler"). */
typedef enum {
  AST_CONV2D = 0,      /* p = {Cin, Cout, k, stride, pad, groups, has_bias}; cross-correlation, zero pad */
  AST_BATCHNORM2D = 1, /* p = {C}; eps; training mode: statistics of the micro-batch          */
  AST_RELU = 2,
  AST_RELU6 = 3,
  AST_RES_BEGIN = 4,   /* remembers the current activation as the skip input                  */
  AST_RES_ADD = 5,     /* adds the remembered skip input                                      */
  AST_GLOBAL_AVGPOOL = 6,
  AST_LINEAR = 7,      /* p = {in, out, has_bias}; y = x W^T + b on the last dimension        */
  AST_SOFTMAX_CE = 8,  /* loss tail: mean over the whole mini-batch (divides by M*B)          */
  AST_MAXPOOL2X2 = 9,  /* 2x2 window, stride 2; gradient to the first maximum in row-major order */
  AST_LAYERNORM = 10,  /* p = {D}; eps; over the last dimension                               */
  AST_MHA = 11,        /* p = {D, heads}; self-attention, no mask, no dropout                 */
  AST_GELU = 12,       /* x * Phi(x) with the exact erf form                                  */
  AST_SWISH = 13,      /* x * sigmoid(x)  (fp32 stages; the EfficientNet workload of Table 4)  */
  AST_SIGMOID = 14,    /* 1 / (1 + exp(-x))  (fp32 stages)                                     */
  AST_SE_BEGIN = 15,   /* squeeze-and-excitation: remembers the current image tensor x; must be
                          followed by AST_GLOBAL_AVGPOOL; the layers up to AST_SE_SCALE compute
                          a gate [B][C] from the pooled vector                                 */
  AST_SE_SCALE = 16,   /* y[b][c][h][w] = x[b][c][h][w] * gate[b][c], x from the matching
                          AST_SE_BEGIN; the gradient reaches x through the product and through
                          the gate                                                             */
  AST_RES_SWAP = 17,   /* inside AST_RES_BEGIN ... AST_RES_ADD: ends the main branch of a two-branch
                          residual block (a ResNet block with a projection shortcut; Table 4
                          workload).  The layers from here to AST_RES_ADD are the shortcut branch:
                          they run on the tensor AST_RES_BEGIN remembered, and AST_RES_ADD adds
                          the main branch's result to theirs                                    */
  AST_MAXPOOL3X3S2 = 18 /* 3x3 window, stride 2, padding 1 (padding never wins); fp32 stages; gradient
                          to the first maximum in row-major order                               */
} ast_layer_kind;

typedef struct {
  int32_t kind;  /* ast_layer_kind */
  int32_t p[8];
  float eps;
} ast_layer;

typedef struct {
  int32_t B;             /* micro-batch size                                         */
  int32_t M;             /* micro-batches per mini-batch (per HPP-Round)             */
  int32_t K;             /* maximum micro-batches forwarded but not yet backwarded   */
  int32_t in_shape[4];   /* per-sample logical input shape: {C,H,W,0} or {S,D,0,0}   */
  int32_t dtype;         /* ast_dtype                                                */
  int32_t layout;        /* ast_layout                                               */
  int32_t needs_input_grad; /* 0 for a first stage: backward writes no dx             */
} ast_stage_cfg;

/* Flat parameter vector (set/get_params, get_grads, set/get_velocity), fp32:
 * layer order; inside a layer weight then bias.  CONV2D weight is logically
 * [Cout][Cin/groups][kh][kw]; LINEAR weight [out][in]; BATCHNORM2D / LAYERNORM
 * gamma then beta; MHA: W_qkv[3D][D] (rows Q, K, V), b_qkv[3D], W_o[D][D], b_o[D].
 * These orders are independent of `layout`. */

/* Build a stage (Sec. 3.2: the stage model a device takes charge of).
 * `layers` (host) is copied.  `hip_stream` is a hipStream_t (NULL = default stream).
 * Parameters start at 0 (BatchNorm/LayerNorm gamma at 1), gradients and velocity at 0.
 * Errors: AST_EINVAL (bad sizes, unbalanced RES_BEGIN/RES_ADD, shapes that do not
 * chain), AST_EUNSUPPORTED, AST_ENOMEM, AST_EHIP.  On error *out is NULL. */
ast_status asteroid_stage_create(const ast_layer* layers, int32_t n_layers,
                                 const ast_stage_cfg* cfg, void* hip_stream,
                                 asteroid_stage** out);

/* FP of micro-batch `mb` (Sec. 3.2).  x_dev: B samples in `layout`/`dtype`, read before
 * the call's work completes on the stream and copied into the stash (the caller may reuse
 * it after the stream passes this call).  labels_dev: int32[B], required iff the stage
 * ends in SOFTMAX_CE.  y_dev: receives the stage output (B samples) or, for a loss tail,
 * the fp32 logits [B][classes]; may be NULL for a loss tail.  loss_dev: one fp32 that
 * receives this micro-batch's share of the mini-batch mean loss; may be NULL.
 * AST_ESTATE if mb is outside [0,M), was already forwarded this round, is not the next
 * micro-batch in order, or K forwarded micro-batches still await their backward. */
ast_status asteroid_stage_forward(asteroid_stage* s, int32_t mb, const void* x_dev,
                                  const int32_t* labels_dev, void* y_dev, float* loss_dev);

/* BP of micro-batch `mb`: dx = J_x^T dy, and G += J_W^T dy in place (gradient
 * accumulation over the micro-batches of the mini-batch, Sec. 3.2); releases the
 * activations stashed by forward(mb).  dy_dev: upstream gradient of y (B samples),
 * NULL iff the stage ends in SOFTMAX_CE.  dx_dev: receives the gradient of x; NULL iff
 * needs_input_grad == 0.  AST_ESTATE if mb was not forwarded, or is not the oldest
 * forwarded micro-batch (backwards run in micro-batch order). */
ast_status asteroid_stage_backward(asteroid_stage* s, int32_t mb, const void* dy_dev,
                                   void* dx_dev);

/* Optional second stream for the forward passes.  A stage that keeps K >= 2 micro-batches in flight
 * (Sec. 3.2: K_p forward passes before one-forward-one-backward is enforced) is handed the forward of a
 * later micro-batch before the backward of an earlier one; the two are independent (different stash
 * slots, G is written by backward passes only, W changes in asteroid_stage_step only).  After this call
 * asteroid_stage_forward enqueues on `hip_stream` (a hipStream_t of default priority) and
 * asteroid_stage_backward / _step stay on the stream given to create, so the two passes may overlap on
 * the GPU; the library orders what does depend through events: backward(mb) behind forward(mb), a
 * forward that reuses a stash slot behind the backward that released it, the first forward of a round
 * behind everything the main stream holds when it is called (the previous round's weight update).  Results are bit-identical to the one-stream execution.  The caller's part:
 * x_dev / labels_dev are ready, and y_dev / loss_dev are read, in the order of `hip_stream`; dy_dev /
 * dx_dev in the order of the main stream.  NULL (or the main stream) returns to one stream.  Waits for
 * the stage's work.  AST_ESTATE inside a round (after a forward and before the step). */
ast_status asteroid_stage_set_forward_stream(asteroid_stage* s, void* hip_stream);

/* A stream for the call above, for callers without a stream API of their own at hand: a new hipStream_t
 * of default priority that does not synchronise with the NULL stream (*out; NULL on error), and its
 * release (waits for nothing: the caller has synchronised; NULL is a no-op).  A process has few hardware
 * queues (four by default) and the runtime deals streams onto them: two streams meant to overlap must not
 * land on one queue, which is likelier the more streams the process holds - a framework's stream pool
 * creates dozens.  Creating the few streams that are used, and destroying them after use, avoids that. */
ast_status asteroid_stream_create(void** out);
ast_status asteroid_stream_destroy(void* hip_stream);

/* For callers that cannot allocate or let a library allocate on their behalf (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): asteroid_stage_backward with the
 * stage's workspace - activation gradients, per-operator scratch, reduction partials - taken from
 * a file-scope device array of AST_STATIC_SCRATCH_BYTES instead of the memory the stage allocated
 * at create.  Same arguments, same results (bit-identical), same AST_ESTATE rules; the call itself
 * allocates nothing and records no memset (the array's used part is cleared by a kernel).
 * AST_EINVAL if the stage's workspace (asteroid_stage_memory) is larger than the array.  Every GPU
 * the library runs on holds one such array until the process ends, and all stages on that GPU
 * share it: calls that overlap in time on one GPU race; calls on one stream do not. */
#define AST_STATIC_SCRATCH_BYTES (32u << 20)
ast_status asteroid_stage_backward_static(asteroid_stage* s, int32_t mb, const void* dy_dev,
                                          void* dx_dev);

/* Weight update at the end of the HPP-Round (Sec. 3.2): v = momentum*v + G;
 * W = W - lr*v; G = 0; reduced-precision weight copies are refreshed.
 * AST_ESTATE unless all M micro-batches have been forwarded and backwarded. */
ast_status asteroid_stage_step(asteroid_stage* s, float lr, float momentum);

/* Waits for the stage's stream, then frees everything the stage owns.  NULL is a no-op. */
void asteroid_stage_destroy(asteroid_stage* s);

/* Number of fp32 entries of the flat parameter vector. */
size_t asteroid_stage_num_params(const asteroid_stage* s);

/* Host <-> device copies of the flat vectors; synchronous (they wait for the stream). */
ast_status asteroid_stage_set_params(asteroid_stage* s, const float* host_flat);
ast_status asteroid_stage_get_params(asteroid_stage* s, float* host_flat);
ast_status asteroid_stage_get_grads(asteroid_stage* s, float* host_flat);
ast_status asteroid_stage_set_velocity(asteroid_stage* s, const float* host_flat);
ast_status asteroid_stage_get_velocity(asteroid_stage* s, float* host_flat);

/* Bytes held, in the terms of the memory model Eq. (3): mod = parameters + accumulated
 * gradients (+ derived weight copies: bf16 layouts, packed pointwise-conv operands); opt = optimizer state (velocity);
 * act_per_mb = activation stash of one micro-batch (the stage holds K of them);
 * workspace = activation-gradient and reduction scratch, independent of K.  Eq. (3)'s sum
 * MOD + OPT + K * ACT has no term for the workspace: a memory check against a device budget has to add
 * it (the profiler tables of this library fold it into the per-sample activation bytes).
 * Any output pointer may be NULL. */
ast_status asteroid_stage_memory(const asteroid_stage* s, size_t* mod, size_t* opt,
                                 size_t* act_per_mb, size_t* workspace);

/* The same four byte counts for a stage that is not built: shape inference and arena
 * layout only, no device call (usable by a planner that must respect a device's memory
 * budget before placing a stage, Sec. 3.2 Eq. (3)).  Same errors as create. */
ast_status asteroid_stage_plan_memory(const ast_layer* layers, int32_t n_layers,
                                      const ast_stage_cfg* cfg, size_t* mod, size_t* opt,
                                      size_t* act_per_mb, size_t* workspace);

/* Introspection for parity tests: copy to host (converted to fp32, in the stage's
 * layout) the activation produced by layer `layer` in the stash of micro-batch `mb`,
 * which must be forwarded and not yet backwarded.  *n_out receives the element count;
 * host_out may be NULL to query the count.  Synchronous.  AST_EINVAL for a layer whose
 * output is fused away or is the stage output (that one is in the caller's y buffer). */
ast_status asteroid_stage_debug_activation(asteroid_stage* s, int32_t mb, int32_t layer,
                                           float* host_out, size_t* n_out);

/* Per-kernel timing with HIP events on the stage's stream (for roofline reports).
 * profile_begin: from now on, every kernel launch of this stage made by the calling
 * thread whose kernel name contains `filter` (NULL or "" = every kernel) is bracketed by
 * an event pair, up to `max_launches` launches (the pool is created here, not in the hot
 * calls).  profile_end: waits for the stream, then aggregates the elapsed times by kernel
 * name and stops recording.  profile_entry(i): name (copied, NUL-terminated, at most
 * name_cap bytes), launch count and summed milliseconds of the i-th aggregated kernel;
 * AST_EINVAL once i is past the last entry. */
ast_status asteroid_stage_profile_begin(asteroid_stage* s, const char* filter, int32_t max_launches);
ast_status asteroid_stage_profile_end(asteroid_stage* s);
ast_status asteroid_stage_profile_entry(asteroid_stage* s, int32_t i, char* name_out, size_t name_cap,
                                        int32_t* launches, double* total_ms);

/* Thread-local message of the last failing call on this thread ("" if none). */
const char* asteroid_last_error(void);

/* Warm-up depth of stage p (0-indexed) in a pipeline of P stages: K_p = 2*(P-p)-1
 * (Sec. 3.2; e.g. P=3 gives 5, 3, 1).  Returns -1 if p is outside [0,P). */
int32_t asteroid_kp(int32_t P, int32_t p);

#ifdef __cplusplus
}
#endif
#endif /* ASTEROID_H */
