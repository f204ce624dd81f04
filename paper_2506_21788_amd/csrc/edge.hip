// Small utility kernels (copy, fill).
#include "edgeops.h"

namespace hgnn {

static inline unsigned nblk64(int64_t n, int t) { return (unsigned)((n + t - 1) / t); }

__global__ void k_copy_f32(const float* __restrict__ s, float* __restrict__ d, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) d[i] = s[i];
}

int32_t launch_copy_f32(hipStream_t st, const float* src, float* dst, int64_t n) {
  if (n <= 0) return HGNN_OK;
  ProfScope ps(PT_MISC, st);
  k_copy_f32<<<nblk64(n, 256), 256, 0, st>>>(src, dst, n);
  HGNN_LAUNCH_CHECK("k_copy_f32");
  return HGNN_OK;
}


__global__ void k_fill_f32(float* __restrict__ d, int64_t n, float v) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) d[i] = v;
}

int32_t launch_fill_f32(hipStream_t st, float* dst, int64_t n, float v) {
  if (n <= 0) return HGNN_OK;
  k_fill_f32<<<nblk64(n, 256), 256, 0, st>>>(dst, n, v);
  HGNN_LAUNCH_CHECK("k_fill_f32");
  return HGNN_OK;
}

}  // namespace hgnn
