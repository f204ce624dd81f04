// Small utility kernels (internal).
#pragma once

#include "common.h"
#include "prof.h"

namespace hgnn {

int32_t launch_copy_f32(hipStream_t st, const float* src, float* dst, int64_t n);
int32_t launch_fill_f32(hipStream_t st, float* dst, int64_t n, float v);

}  // namespace hgnn
