// The statically allocated workspace of asteroid_stage_backward_static (static_scratch.hip).
#pragma once
#include <hip/hip_runtime.h>

#include <string>

#include "../../include/asteroid.h"

namespace ast {

constexpr size_t kStaticScratchBytes = (size_t)AST_STATIC_SCRATCH_BYTES;

ast_status static_scratch_ptr(char** out, std::string& err);
void static_scratch_zero(hipStream_t st, char* ptr, size_t bytes);

}  // namespace ast
