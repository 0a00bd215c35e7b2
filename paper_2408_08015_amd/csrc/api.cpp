// C ABI of the stage-training library (see include/asteroid.h): argument checks, the
// 1F1B call discipline (Sec. 3.2), allocation in create, and the flat-vector accessors.
#include <cstring>
#include <new>
#include <cstdlib>
#include <string>
#include <vector>

#include "kernels.h"
#include "kernels_bf16.h"
#include "prof.h"
#include "stage.h"

namespace ast {
thread_local Profiler* g_prof = nullptr;
}

struct ProfEntry {
  std::string name;
  int launches = 0;
  double ms = 0;
};

struct asteroid_stage {
  ast::Stage s;
  ast::Profiler prof;
  bool prof_on = false;
  std::vector<ProfEntry> prof_result;
};

namespace {
// activates the stage's profiler on this thread for the duration of one hot call
struct ProfGuard {
  explicit ProfGuard(asteroid_stage* h) { ast::g_prof = h->prof_on ? &h->prof : nullptr; }
  ~ProfGuard() { ast::g_prof = nullptr; }
};
}  // namespace

namespace {
thread_local std::string g_err;

ast_status fail(ast_status code, const std::string& msg) {
  g_err = msg;
  return code;
}
ast_status hip_fail(hipError_t e, const char* what) {
  g_err = std::string(what) + ": " + hipGetErrorString(e);
  return e == hipErrorOutOfMemory ? AST_ENOMEM : AST_EHIP;
}
#define HIPCHK(call, what)                        \
  do {                                            \
    hipError_t e_ = (call);                       \
    if (e_ != hipSuccess) return hip_fail(e_, what); \
  } while (0)

void free_stage(ast::Stage& s) {
  if (s.W) (void)hipFree(s.W);
  if (s.G) (void)hipFree(s.G);
  if (s.V) (void)hipFree(s.V);
  if (s.shadow) (void)hipFree(s.shadow);
  if (s.running) (void)hipFree(s.running);
  if (s.pack_tasks) (void)hipFree(s.pack_tasks);
  if (s.pack_block_task) (void)hipFree(s.pack_block_task);
  s.pack_tasks = nullptr;
  s.pack_block_task = nullptr;
  s.pack_nblocks = 0;
  if (s.lsh_tasks) (void)hipFree(s.lsh_tasks);
  if (s.lsh_block_task) (void)hipFree(s.lsh_block_task);
  s.lsh_tasks = nullptr;
  s.lsh_block_task = nullptr;
  s.lsh_nblocks = 0;
  if (s.red_tasks) (void)hipFree(s.red_tasks);
  if (s.red_tasks_static) (void)hipFree(s.red_tasks_static);
  s.red_tasks_static = nullptr;
  if (s.red_block_task) (void)hipFree(s.red_block_task);
  s.red_tasks = nullptr;
  s.red_block_task = nullptr;
  s.red_nblocks = 0;
  for (ast::Stage::WgGroup& wg : s.wg_groups) {
    if (wg.tasks) (void)hipFree(wg.tasks);
    if (wg.block_task) (void)hipFree(wg.block_task);
    if (wg.task_block0) (void)hipFree(wg.task_block0);
  }
  s.wg_groups.clear();
  s.wg_nblocks = 0;
  if (s.wpack) (void)hipFree(s.wpack);
  s.wpack = nullptr;
  if (s.ws) (void)hipFree(s.ws);
  for (char* p : s.slots)
    if (p) (void)hipFree(p);
  s.slots.clear();
  for (hipEvent_t ev : s.fork_ev) (void)hipEventDestroy(ev);
  s.fork_ev.clear();
  for (hipEvent_t ev : s.fwd_done) (void)hipEventDestroy(ev);
  for (hipEvent_t ev : s.bwd_done) (void)hipEventDestroy(ev);
  s.fwd_done.clear();
  s.bwd_done.clear();
  if (s.round_ev) (void)hipEventDestroy(s.round_ev);
  s.round_ev = nullptr;
  s.fwd_stream = nullptr;
  if (s.join_ev) (void)hipEventDestroy(s.join_ev);
  if (s.side) (void)hipStreamDestroy(s.side);
  s.join_ev = nullptr;
  s.side = nullptr;
  s.W = s.G = s.V = nullptr;
  s.shadow = nullptr;
  s.running = nullptr;
  s.ws = nullptr;
}

// initial parameter values: 0, with BatchNorm / LayerNorm gamma at 1
std::vector<float> initial_params(const ast::Stage& s) {
  std::vector<float> w(s.nparams, 0.f);
  for (const ast::Op& op : s.ops)
    if (op.kind == ast::OP_BN || op.kind == ast::OP_LAYERNORM)
      for (int c = 0; c < op.cin; ++c) w[op.w_off + c] = 1.f;
  return w;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// waits for everything the stage has enqueued: the forward stream (if any), then the main stream
hipError_t sync_stage(ast::Stage& s) {
  if (s.fwd_stream) {
    hipError_t e = hipStreamSynchronize(s.fwd_stream);
    if (e != hipSuccess) return e;
  }
  return hipStreamSynchronize(s.stream);
}
}  // namespace

namespace ast {
// message for asteroid_last_error() from the other translation units of the library
void set_last_error(const std::string& msg) { g_err = msg; }
}  // namespace ast

extern "C" {

const char* asteroid_last_error(void) { return g_err.c_str(); }

int32_t asteroid_kp(int32_t P, int32_t p) {
  if (P <= 0 || p < 0 || p >= P) return -1;
  return 2 * (P - p) - 1;
}

ast_status asteroid_stage_create(const ast_layer* layers, int32_t n_layers, const ast_stage_cfg* cfg,
                                 void* hip_stream, asteroid_stage** out) {
  if (out) *out = nullptr;
  if (!layers || n_layers <= 0 || !cfg || !out) return fail(AST_EINVAL, "create: NULL argument or no layers");
  if (cfg->K > cfg->M) return fail(AST_EINVAL, "create: K must not exceed M");
  asteroid_stage* h = new (std::nothrow) asteroid_stage();
  if (!h) return fail(AST_ENOMEM, "create: host allocation failed");
  ast::Stage& s = h->s;
  s.cfg = *cfg;
  s.layers.assign(layers, layers + n_layers);
  s.stream = static_cast<hipStream_t>(hip_stream);
  std::string err;
  ast_status r = ast::build_plan(s, err);
  if (r != AST_OK) {
    delete h;
    return fail(r, "create: " + err);
  }
  auto bail = [&](hipError_t e, const char* what) {
    ast_status st = hip_fail(e, what);
    free_stage(s);
    delete h;
    return st;
  };
  hipError_t e;
  const size_t pbytes = (s.nparams + 4) * sizeof(float);
  if ((e = hipMalloc((void**)&s.W, pbytes)) != hipSuccess) return bail(e, "create: hipMalloc(W)");
  if ((e = hipMalloc((void**)&s.G, pbytes)) != hipSuccess) return bail(e, "create: hipMalloc(G)");
  if ((e = hipMalloc((void**)&s.V, pbytes)) != hipSuccess) return bail(e, "create: hipMalloc(V)");
  if (s.shadow_elems && (e = hipMalloc((void**)&s.shadow, s.shadow_elems * 2 + 16)) != hipSuccess)
    return bail(e, "create: hipMalloc(weight copies)");
  if (s.wpack_floats && (e = hipMalloc((void**)&s.wpack, s.wpack_floats * sizeof(float))) != hipSuccess)
    return bail(e, "create: hipMalloc(packed weights)");
  if (s.running_floats && (e = hipMalloc((void**)&s.running, s.running_floats * sizeof(float))) != hipSuccess)
    return bail(e, "create: hipMalloc(running stats)");
  if ((e = hipMalloc((void**)&s.ws, s.ws_bytes)) != hipSuccess) return bail(e, "create: hipMalloc(workspace)");
  s.slots.assign(cfg->K, nullptr);
  for (int k = 0; k < cfg->K; ++k)
    if ((e = hipMalloc((void**)&s.slots[k], s.slot_bytes)) != hipSuccess) return bail(e, "create: hipMalloc(stash)");
  // Second stream (default priority) for the weight-gradient kernels; ASTEROID_SIDE_STREAM=0
  // keeps everything on the caller's stream.
  const char* side_env = getenv("ASTEROID_SIDE_STREAM");
  if (!(side_env && side_env[0] == '0')) {
    if ((e = hipStreamCreateWithFlags(&s.side, hipStreamNonBlocking)) != hipSuccess) return bail(e, "create: side stream");
    if ((e = hipEventCreateWithFlags(&s.join_ev, hipEventDisableTiming)) != hipSuccess) return bail(e, "create: event");
    for (int i = 0; i < 128; ++i) {
      hipEvent_t ev;
      if ((e = hipEventCreateWithFlags(&ev, hipEventDisableTiming)) != hipSuccess) return bail(e, "create: event");
      s.fork_ev.push_back(ev);
    }
  }
  if ((e = hipMemset(s.G, 0, pbytes)) != hipSuccess) return bail(e, "create: memset");
  if ((e = hipMemset(s.V, 0, pbytes)) != hipSuccess) return bail(e, "create: memset");
  if ((e = hipMemset(s.ws, 0, s.ws_bytes)) != hipSuccess) return bail(e, "create: memset");
  if (s.running) {
    std::vector<float> rs(s.running_floats, 0.f);
    for (const ast::Op& op : s.ops)
      if (op.kind == ast::OP_BN)
        for (int c = 0; c < op.cin; ++c) rs[op.run_off + op.cin + c] = 1.f;
    if ((e = hipMemcpy(s.running, rs.data(), rs.size() * sizeof(float), hipMemcpyHostToDevice)) != hipSuccess)
      return bail(e, "create: memcpy");
  }
  std::vector<float> w0 = initial_params(s);
  w0.resize(s.nparams + 4, 0.f);
  if ((e = hipMemcpy(s.W, w0.data(), pbytes, hipMemcpyHostToDevice)) != hipSuccess) return bail(e, "create: memcpy");
  s.mb_slot.assign(cfg->M, -1);
  for (int k = cfg->K - 1; k >= 0; --k) s.free_slots.push_back(k);
  r = ast::build_reduce_tasks(s, err);
  if (r == AST_OK) r = ast::refresh_shadow(s, err);
  if (r == AST_OK && (e = hipStreamSynchronize(s.stream)) != hipSuccess) return bail(e, "create: sync");
  if (r != AST_OK) {
    free_stage(s);
    delete h;
    return fail(r, "create: " + err);
  }
  *out = h;
  return AST_OK;
}

ast_status asteroid_stream_create(void** out) {
  if (!out) return fail(AST_EINVAL, "stream_create: NULL argument");
  *out = nullptr;
  hipStream_t st;
  HIPCHK(hipStreamCreateWithFlags(&st, hipStreamNonBlocking), "stream_create");
  *out = st;
  return AST_OK;
}

ast_status asteroid_stream_destroy(void* hip_stream) {
  if (!hip_stream) return AST_OK;
  HIPCHK(hipStreamDestroy(static_cast<hipStream_t>(hip_stream)), "stream_destroy");
  return AST_OK;
}

ast_status asteroid_stage_set_forward_stream(asteroid_stage* h, void* hip_stream) {
  if (!h) return fail(AST_EINVAL, "set_forward_stream: NULL stage");
  ast::Stage& s = h->s;
  if (s.next_fwd != 0 || s.next_bwd != 0) return fail(AST_ESTATE, "set_forward_stream: only between rounds");
  HIPCHK(sync_stage(s), "set_forward_stream");
  hipStream_t f = static_cast<hipStream_t>(hip_stream);
  if (f == s.stream) f = nullptr;
  if (f && s.fwd_done.empty()) {
    for (int k = 0; k < 2 * s.cfg.K + 1; ++k) {
      hipEvent_t ev;
      HIPCHK(hipEventCreateWithFlags(&ev, hipEventDisableTiming), "set_forward_stream: event");
      if (k == 2 * s.cfg.K) s.round_ev = ev;
      else (k < s.cfg.K ? s.fwd_done : s.bwd_done).push_back(ev);
    }
  }
  s.bwd_done_set.assign(s.cfg.K, 0);
  s.fwd_stream = f;
  return AST_OK;
}

ast_status asteroid_stage_forward(asteroid_stage* h, int32_t mb, const void* x_dev, const int32_t* labels_dev,
                                  void* y_dev, float* loss_dev) {
  if (!h) return fail(AST_EINVAL, "forward: NULL stage");
  ast::Stage& s = h->s;
  if (mb < 0 || mb >= s.cfg.M) return fail(AST_ESTATE, "forward: micro-batch index outside [0, M)");
  if (mb != s.next_fwd) return fail(AST_ESTATE, "forward: micro-batches are forwarded in order, once per round");
  if (s.next_fwd - s.next_bwd >= s.cfg.K) return fail(AST_ESTATE, "forward: K forwarded micro-batches await their backward");
  if (!x_dev) return fail(AST_EINVAL, "forward: x_dev is NULL");
  if (!aligned16(x_dev) || !aligned16(y_dev) || !aligned16(labels_dev)) return fail(AST_EINVAL, "forward: buffers must be 16-byte aligned");
  if (s.loss_tail && !labels_dev) return fail(AST_EINVAL, "forward: labels_dev required for a SOFTMAX_CE tail");
  if (!s.loss_tail && !y_dev) return fail(AST_EINVAL, "forward: y_dev is NULL");
  int slot = s.free_slots.back();
  std::string err;
  ProfGuard pg(h);
  ast_status r = ast::run_forward(s, slot, x_dev, labels_dev, y_dev, loss_dev, err);
  if (r != AST_OK) return fail(r, err);
  s.free_slots.pop_back();
  s.mb_slot[mb] = slot;
  s.next_fwd++;
  return AST_OK;
}

static ast_status backward_impl(asteroid_stage* h, int32_t mb, const void* dy_dev, void* dx_dev, bool use_static) {
  if (!h) return fail(AST_EINVAL, "backward: NULL stage");
  ast::Stage& s = h->s;
  if (mb < 0 || mb >= s.cfg.M) return fail(AST_ESTATE, "backward: micro-batch index outside [0, M)");
  if (mb >= s.next_fwd) return fail(AST_ESTATE, "backward: micro-batch was not forwarded");
  if (mb != s.next_bwd) return fail(AST_ESTATE, "backward: backwards run in micro-batch order, once each");
  if (!s.loss_tail && !dy_dev) return fail(AST_EINVAL, "backward: dy_dev is NULL");
  if (s.loss_tail && dy_dev) return fail(AST_EINVAL, "backward: dy_dev must be NULL for a SOFTMAX_CE tail");
  if (s.cfg.needs_input_grad && !dx_dev) return fail(AST_EINVAL, "backward: dx_dev is NULL");
  if (!s.cfg.needs_input_grad && dx_dev) return fail(AST_EINVAL, "backward: dx_dev must be NULL when needs_input_grad == 0");
  if (!aligned16(dy_dev) || !aligned16(dx_dev)) return fail(AST_EINVAL, "backward: buffers must be 16-byte aligned");
  if (use_static) {
    if (s.ws_bytes > (size_t)AST_STATIC_SCRATCH_BYTES)
      return fail(AST_EINVAL, "backward_static: the stage's workspace (" + std::to_string(s.ws_bytes) +
                                  " bytes) exceeds AST_STATIC_SCRATCH_BYTES (" + std::to_string((size_t)AST_STATIC_SCRATCH_BYTES) + ")");
    if (!s.static_ws) return fail(AST_EHIP, "backward_static: the static workspace of this device could not be located at create");
  }
  int slot = s.mb_slot[mb];
  std::string err;
  ProfGuard pg(h);
  ast_status r = ast::run_backward(s, slot, dy_dev, dx_dev, use_static ? s.static_ws : nullptr, err);
  if (r != AST_OK) return fail(r, err);
  s.mb_slot[mb] = -1;
  s.free_slots.push_back(slot);  // the backward releases the stash
  s.next_bwd++;
  return AST_OK;
}

ast_status asteroid_stage_backward(asteroid_stage* h, int32_t mb, const void* dy_dev, void* dx_dev) {
  return backward_impl(h, mb, dy_dev, dx_dev, false);
}

ast_status asteroid_stage_backward_static(asteroid_stage* h, int32_t mb, const void* dy_dev, void* dx_dev) {
  return backward_impl(h, mb, dy_dev, dx_dev, true);
}

ast_status asteroid_stage_step(asteroid_stage* h, float lr, float momentum) {
  if (!h) return fail(AST_EINVAL, "step: NULL stage");
  ast::Stage& s = h->s;
  if (s.next_bwd != s.cfg.M) return fail(AST_ESTATE, "step: not all M micro-batches have been forwarded and backwarded");
  std::string err;
  ProfGuard pg(h);
  ast_status r = ast::run_step(s, lr, momentum, err);
  if (r != AST_OK) return fail(r, err);
  s.next_fwd = s.next_bwd = 0;
  return AST_OK;
}

void asteroid_stage_destroy(asteroid_stage* h) {
  if (!h) return;
  (void)sync_stage(h->s);
  for (hipEvent_t e : h->prof.events) (void)hipEventDestroy(e);
  free_stage(h->s);
  delete h;
}

size_t asteroid_stage_num_params(const asteroid_stage* h) { return h ? h->s.nparams : 0; }

static ast_status copy_flat(asteroid_stage* h, float* dev, float* host_out, const float* host_in, const char* what) {
  if (!h || (!host_out && !host_in)) return fail(AST_EINVAL, std::string(what) + ": NULL argument");
  ast::Stage& s = h->s;
  HIPCHK(sync_stage(s), what);
  if (host_in) HIPCHK(hipMemcpy(dev, host_in, s.nparams * sizeof(float), hipMemcpyHostToDevice), what);
  else HIPCHK(hipMemcpy(host_out, dev, s.nparams * sizeof(float), hipMemcpyDeviceToHost), what);
  return AST_OK;
}

ast_status asteroid_stage_set_params(asteroid_stage* h, const float* host_flat) {
  ast_status r = copy_flat(h, h ? h->s.W : nullptr, nullptr, host_flat, "set_params");
  if (r != AST_OK) return r;
  std::string err;
  r = ast::refresh_shadow(h->s, err);
  if (r != AST_OK) return fail(r, err);
  HIPCHK(hipStreamSynchronize(h->s.stream), "set_params");
  return AST_OK;
}
ast_status asteroid_stage_get_params(asteroid_stage* h, float* host_flat) {
  return copy_flat(h, h ? h->s.W : nullptr, host_flat, nullptr, "get_params");
}
ast_status asteroid_stage_get_grads(asteroid_stage* h, float* host_flat) {
  return copy_flat(h, h ? h->s.G : nullptr, host_flat, nullptr, "get_grads");
}
ast_status asteroid_stage_set_velocity(asteroid_stage* h, const float* host_flat) {
  return copy_flat(h, h ? h->s.V : nullptr, nullptr, host_flat, "set_velocity");
}
ast_status asteroid_stage_get_velocity(asteroid_stage* h, float* host_flat) {
  return copy_flat(h, h ? h->s.V : nullptr, host_flat, nullptr, "get_velocity");
}

ast_status asteroid_stage_memory(const asteroid_stage* h, size_t* mod, size_t* opt, size_t* act_per_mb,
                                 size_t* workspace) {
  if (!h) return fail(AST_EINVAL, "memory: NULL stage");
  const ast::Stage& s = h->s;
  if (mod) *mod = 2 * s.nparams * sizeof(float) + s.shadow_elems * 2 + s.wpack_floats * sizeof(float);
  if (opt) *opt = s.nparams * sizeof(float);
  if (act_per_mb) *act_per_mb = s.slot_bytes;
  if (workspace) *workspace = s.ws_bytes;
  return AST_OK;
}

ast_status asteroid_stage_plan_memory(const ast_layer* layers, int32_t n_layers, const ast_stage_cfg* cfg,
                                      size_t* mod, size_t* opt, size_t* act_per_mb, size_t* workspace) {
  if (!layers || n_layers <= 0 || !cfg) return fail(AST_EINVAL, "plan_memory: NULL argument or no layers");
  if (cfg->K > cfg->M) return fail(AST_EINVAL, "plan_memory: K must not exceed M");
  asteroid_stage tmp;
  tmp.s.cfg = *cfg;
  tmp.s.layers.assign(layers, layers + n_layers);
  std::string err;
  ast_status r = ast::build_plan(tmp.s, err);
  if (r != AST_OK) return fail(r, "plan_memory: " + err);
  return asteroid_stage_memory(&tmp, mod, opt, act_per_mb, workspace);
}

ast_status asteroid_stage_debug_activation(asteroid_stage* h, int32_t mb, int32_t layer, float* host_out,
                                           size_t* n_out) {
  if (!h) return fail(AST_EINVAL, "debug_activation: NULL stage");
  ast::Stage& s = h->s;
  if (layer < 0 || layer >= (int)s.layers.size() || s.layer_act[layer] < 0)
    return fail(AST_EINVAL, "debug_activation: layer has no materialised output");
  if (mb < 0 || mb >= s.cfg.M || s.mb_slot[mb] < 0) return fail(AST_ESTATE, "debug_activation: micro-batch has no live stash");
  int id = s.layer_act[layer];
  const ast::Act& A = s.acts[id];
  if (id == s.final_act && !s.loss_tail && !s.final_in_slot) return fail(AST_EINVAL, "debug_activation: the stage output lives in the caller's buffer");
  if (n_out) *n_out = A.elems;
  if (!host_out) return AST_OK;
  HIPCHK(sync_stage(s), "debug_activation");
  const char* src = s.slots[s.mb_slot[mb]] + A.slot_off;
  if (A.esize == 4) {
    HIPCHK(hipMemcpy(host_out, src, A.bytes, hipMemcpyDeviceToHost), "debug_activation");
  } else {
    std::vector<unsigned short> tmp(A.elems);
    HIPCHK(hipMemcpy(tmp.data(), src, A.bytes, hipMemcpyDeviceToHost), "debug_activation");
    for (size_t i = 0; i < A.elems; ++i) {
      uint32_t u = ((uint32_t)tmp[i]) << 16;
      std::memcpy(&host_out[i], &u, 4);
    }
  }
  return AST_OK;
}

ast_status asteroid_stage_profile_begin(asteroid_stage* h, const char* filter, int32_t max_launches) {
  if (!h || max_launches <= 0) return fail(AST_EINVAL, "profile_begin: bad argument");
  ast::Profiler& p = h->prof;
  p.filter = filter ? filter : "";
  while (p.events.size() < (size_t)max_launches * 2) {
    hipEvent_t e;
    HIPCHK(hipEventCreate(&e), "profile_begin");
    p.events.push_back(e);
  }
  p.used = 0;
  p.names.clear();
  h->prof_result.clear();
  h->prof_on = true;
  return AST_OK;
}

ast_status asteroid_stage_profile_end(asteroid_stage* h) {
  if (!h) return fail(AST_EINVAL, "profile_end: NULL stage");
  h->prof_on = false;
  HIPCHK(sync_stage(h->s), "profile_end");
  ast::Profiler& p = h->prof;
  h->prof_result.clear();
  for (size_t i = 0; i < p.used; ++i) {
    float ms = 0.f;
    HIPCHK(hipEventElapsedTime(&ms, p.events[2 * i], p.events[2 * i + 1]), "profile_end");
    ProfEntry* e = nullptr;
    for (ProfEntry& q : h->prof_result)
      if (q.name == p.names[i]) { e = &q; break; }
    if (!e) {
      h->prof_result.push_back(ProfEntry());
      e = &h->prof_result.back();
      e->name = p.names[i];
    }
    e->launches++;
    e->ms += ms;
  }
  p.used = 0;
  p.names.clear();
  return AST_OK;
}

ast_status asteroid_stage_profile_entry(asteroid_stage* h, int32_t i, char* name_out, size_t name_cap,
                                        int32_t* launches, double* total_ms) {
  if (!h || i < 0 || i >= (int)h->prof_result.size()) return fail(AST_EINVAL, "profile_entry: index past the last entry");
  const ProfEntry& e = h->prof_result[i];
  if (name_out && name_cap) {
    std::strncpy(name_out, e.name.c_str(), name_cap - 1);
    name_out[name_cap - 1] = 0;
  }
  if (launches) *launches = e.launches;
  if (total_ms) *total_ms = e.ms;
  return AST_OK;
}

}  // extern "C"
