// Optional per-kernel timing with HIP events on the stage's stream.  Launch sites use
// KLAUNCH(kernel, grid, block, shmem, stream, args...); when a profiler is active on the
// calling thread and the kernel's name contains the filter, the launch carries an event
// pair.  Inactive cost: one thread-local pointer test per launch.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <cstring>
#include <string>
#include <tuple>
#include <utility>
#include <vector>

namespace ast {

struct Profiler {
  std::string filter;             // substring of the kernel name; empty = every kernel
  std::vector<hipEvent_t> events; // pairs (start, stop)
  std::vector<const char*> names; // one per pair (string literals)
  size_t used = 0;                // pairs in use
};

extern thread_local Profiler* g_prof;

// A slot of the active profiler for a launch whose name passes the filter (p == nullptr: none).
struct ProfSlot {
  Profiler* p = nullptr;
  size_t idx = 0;
  explicit ProfSlot(const char* name) {
    Profiler* q = g_prof;
    if (!q) return;
    if (!q->filter.empty() && !std::strstr(name, q->filter.c_str())) return;
    if ((q->used + 1) * 2 > q->events.size()) return;  // pool exhausted: stop recording
    p = q;
    idx = q->used++;
    q->names.push_back(name);
  }
  hipEvent_t start() const { return p->events[2 * idx]; }
  hipEvent_t stop() const { return p->events[2 * idx + 1]; }
};

// Launch with the event pair attached to the dispatch itself (hipExtLaunchKernel): the events
// carry the kernel's own begin and end timestamps, so their difference is the kernel's
// duration without the few microseconds that two separately recorded events add around it.
template <typename... Params, typename... Args, size_t... I>
inline void launch_timed_impl(void (*kern)(Params...), dim3 grid, dim3 block, size_t shm, hipStream_t st, hipEvent_t e0,
                              hipEvent_t e1, std::index_sequence<I...>, Args&&... args) {
  std::tuple<Params...> conv{static_cast<Params>(args)...};  // every argument converted to its parameter type
  void* ptrs[sizeof...(Params)] = {static_cast<void*>(&std::get<I>(conv))...};
  (void)hipExtLaunchKernel(reinterpret_cast<const void*>(kern), grid, block, ptrs, shm, st, e0, e1, 0);
}
template <typename... Params, typename... Args>
inline void launch_timed(void (*kern)(Params...), dim3 grid, dim3 block, size_t shm, hipStream_t st, hipEvent_t e0,
                         hipEvent_t e1, Args&&... args) {
  static_assert(sizeof...(Params) == sizeof...(Args), "argument count");
  launch_timed_impl(kern, grid, block, shm, st, e0, e1, std::index_sequence_for<Params...>{},
                    std::forward<Args>(args)...);
}

#define KLAUNCH_NAMED(name, kern, grid, block, shm, st, ...)                                              \
  do {                                                                                                    \
    ::ast::ProfSlot prof_slot_(name);                                                                     \
    if (prof_slot_.p)                                                                                     \
      ::ast::launch_timed(kern, grid, block, shm, st, prof_slot_.start(), prof_slot_.stop(), __VA_ARGS__); \
    else                                                                                                  \
      hipLaunchKernelGGL(kern, grid, block, shm, st, __VA_ARGS__);                                        \
  } while (0)

#define KLAUNCH(kern, grid, block, shm, st, ...) KLAUNCH_NAMED(#kern, kern, grid, block, shm, st, __VA_ARGS__)

}  // namespace ast
