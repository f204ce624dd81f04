// Small utility kernels (copy, fill) and the radial basis of the edge lengths.
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

// attr[e][j] = exp(-gamma (d - mu_j)^2) * (cos(pi d / rc) + 1) / 2,  d = sqrt(d2[e]),  mu_j = j rc / (k - 1),
// gamma = ((k - 1) / rc)^2   (float32, library expf / cosf)
__global__ void k_edge_rbf(int64_t E, int k, const float* __restrict__ d2, float rc, float* __restrict__ attr) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= E * k) return;
  const int64_t e = idx / k;
  const int j = (int)(idx - e * k);
  const float d = sqrtf(d2[e]);
  const float mu = (float)j * (rc / (float)(k - 1));
  const float gamma = ((float)(k - 1) / rc) * ((float)(k - 1) / rc);
  const float fc = 0.5f * (cosf(3.14159265358979323846f * d / rc) + 1.0f);
  const float t = d - mu;
  attr[idx] = expf(-gamma * t * t) * fc;
}

}  // namespace hgnn

extern "C" int32_t hgnn_edge_rbf(void* stream, int64_t E, const float* d2, int32_t k, float rc, float* attr) {
  using namespace hgnn;
  HGNN_REQUIRE(E >= 0 && k >= 2 && k <= 16 && rc > 0.f, HGNN_ERR_BAD_SHAPE, "edge_rbf: need E >= 0, 2 <= k <= 16, rc > 0");
  if (E == 0) return HGNN_OK;
  HGNN_REQUIRE(d2 && attr, HGNN_ERR_NULLPTR, "edge_rbf: null pointer");
  hipStream_t st = static_cast<hipStream_t>(stream);
  ProfScope ps(PT_MISC, st);
  k_edge_rbf<<<nblk64(E * k, 256), 256, 0, st>>>(E, k, d2, rc, attr);
  HGNN_LAUNCH_CHECK("k_edge_rbf");
  return HGNN_OK;
}
