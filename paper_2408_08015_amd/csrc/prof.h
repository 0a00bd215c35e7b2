// Optional per-kernel timing with HIP events on the stage's stream.  Launch sites use
// KLAUNCH(kernel, grid, block, shmem, stream, args...); when a profiler is active on the
// calling thread and the kernel's name contains the filter, the launch is bracketed by
// an event pair.  Inactive cost: one thread-local pointer test per launch.
#pragma once
#include <hip/hip_runtime.h>

#include <cstring>
#include <string>
#include <vector>

namespace ast {

struct Profiler {
  std::string filter;             // substring of the kernel name; empty = every kernel
  std::vector<hipEvent_t> events; // pairs (start, stop)
  std::vector<const char*> names; // one per pair (string literals)
  size_t used = 0;                // pairs in use
};

extern thread_local Profiler* g_prof;

struct ProfScope {
  Profiler* p = nullptr;
  hipStream_t st;
  size_t idx = 0;
  ProfScope(const char* name, hipStream_t s) : st(s) {
    Profiler* q = g_prof;
    if (!q) return;
    if (!q->filter.empty() && !std::strstr(name, q->filter.c_str())) return;
    if ((q->used + 1) * 2 > q->events.size()) return;  // pool exhausted: stop recording
    p = q;
    idx = q->used++;
    q->names.push_back(name);
    (void)hipEventRecord(q->events[2 * idx], st);
  }
  ~ProfScope() {
    if (p) (void)hipEventRecord(p->events[2 * idx + 1], st);
  }
};

#define KLAUNCH(kern, grid, block, shm, st, ...)                    \
  do {                                                              \
    ::ast::ProfScope prof_scope_(#kern, st);                        \
    hipLaunchKernelGGL(kern, grid, block, shm, st, __VA_ARGS__);    \
  } while (0)

// same, with an explicit display name (for template kernels launched through a pointer)
#define KLAUNCH_NAMED(name, kern, grid, block, shm, st, ...)       \
  do {                                                              \
    ::ast::ProfScope prof_scope_(name, st);                         \
    hipLaunchKernelGGL(kern, grid, block, shm, st, __VA_ARGS__);    \
  } while (0)

}  // namespace ast
