// Small utility kernels (internal).
#pragma once

#include "common.h"
#include "prof.h"

namespace hgnn {

int32_t launch_copy_f32(hipStream_t st, const float* src, float* dst, int64_t n);
int32_t launch_fill_f32(hipStream_t st, float* dst, int64_t n, float v);
// g_rvec_e = alpha x_e g_v[dst_e]: gradient with respect to the edge vectors of v'_i = v_i + alpha sum x_e rvec_e
int32_t launch_edge_grvec(hipStream_t st, int64_t E, const int32_t* dst, const float* xe, const float* g_v, float alpha,
                          float* g_rvec);

}  // namespace hgnn
