// A workspace that is not allocated: a file-scope device array, for the backward entry point
// that callers use who cannot allocate (asteroid_stage_backward_static: HIP graph capture, tight
// loops, harnesses that forbid hipMalloc).  Every GPU the library runs on holds its own copy of
// the array until the process ends; the name of the array is a host-side stand-in, its device
// address comes from hipGetSymbolAddress, once per device.
#include <hip/hip_runtime.h>

#include <mutex>
#include <string>

#include "prof.h"
#include "static_scratch.h"

static __device__ __align__(256) unsigned char scratch[ast::kStaticScratchBytes];

namespace ast {

namespace {
constexpr int kMaxDevices = 64;
char* g_ptr[kMaxDevices] = {};
std::mutex g_mu;

__global__ void fill_zero16_kernel(uint4* __restrict__ p, size_t n16) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n16) p[i] = make_uint4(0, 0, 0, 0);
}
}  // namespace

// Device address of the current device's copy of the array (looked up on first use per device).
ast_status static_scratch_ptr(char** out, std::string& err) {
  *out = nullptr;
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    err = std::string("static scratch: hipGetDevice: ") + (e != hipSuccess ? hipGetErrorString(e) : "device index out of range");
    return AST_EHIP;
  }
  std::lock_guard<std::mutex> lk(g_mu);
  if (!g_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      err = std::string("static scratch: hipGetSymbolAddress: ") + hipGetErrorString(e);
      return AST_EHIP;
    }
    g_ptr[dev] = static_cast<char*>(p);
  }
  *out = g_ptr[dev];
  return AST_OK;
}

// Zero the first `bytes` of the array (rounded up to 16) with a kernel: a memset node must not end
// up in a graph a caller may be capturing.
void static_scratch_zero(hipStream_t st, char* ptr, size_t bytes) {
  const size_t n16 = (bytes + 15) / 16;
  if (!n16) return;
  KLAUNCH(fill_zero16_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, st, reinterpret_cast<uint4*>(ptr), n16);
}

}  // namespace ast
