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

__global__ void k_edge_grvec(int64_t E, const int32_t* __restrict__ dst, const float* __restrict__ xe,
                             const float* __restrict__ g_v, float alpha, float* __restrict__ g_rvec) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= E) return;
  const size_t i = (size_t)dst[e];
  const float t = alpha * xe[e];
  g_rvec[3 * e] = t * g_v[3 * i];
  g_rvec[3 * e + 1] = t * g_v[3 * i + 1];
  g_rvec[3 * e + 2] = t * g_v[3 * i + 2];
}

int32_t launch_edge_grvec(hipStream_t st, int64_t E, const int32_t* dst, const float* xe, const float* g_v, float alpha,
                          float* g_rvec) {
  if (E <= 0) return HGNN_OK;
  ProfScope ps(PT_MISC, st);
  k_edge_grvec<<<nblk64(E, 256), 256, 0, st>>>(E, dst, xe, g_v, alpha, g_rvec);
  HGNN_LAUNCH_CHECK("k_edge_grvec");
  return HGNN_OK;
}

// attr[e][j] = exp(-gamma (d - mu_j)^2) * fc(d),  d = sqrt(d2[e]),  mu_j = j rc / (k - 1),  gamma = ((k - 1) / rc)^2,
// fc(d) = (cos(pi d / rc) + 1) / 2 inside the cutoff, 0 from the cutoff on   (float32, library expf / cosf)
__global__ void k_edge_rbf(int64_t E, int k, const float* __restrict__ d2, float rc, float* __restrict__ attr) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= E * k) return;
  const int64_t e = idx / k;
  const int j = (int)(idx - e * k);
  const float d = sqrtf(d2[e]);
  const float mu = (float)j * (rc / (float)(k - 1));
  const float gamma = ((float)(k - 1) / rc) * ((float)(k - 1) / rc);
  const float fc = d < rc ? 0.5f * (cosf(3.14159265358979323846f * d / rc) + 1.0f) : 0.f;
  const float t = d - mu;
  attr[idx] = expf(-gamma * t * t) * fc;
}

// g_d2[e] = sum_j g_attr[e][j] * d attr_j / d d2,  d/d d2 = (1 / 2d) d/dd,
// d attr_j / dd = exp(-gamma (d - mu_j)^2) (-2 gamma (d - mu_j) fc(d) + fc'(d)),  fc'(d) = -(pi / 2 rc) sin(pi d / rc)
__global__ void k_edge_rbf_bwd(int64_t E, int k, const float* __restrict__ d2, float rc,
                               const float* __restrict__ g_attr, float* __restrict__ g_d2) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= E) return;
  const float d = sqrtf(d2[e]);
  const float step = rc / (float)(k - 1);
  const float gamma = ((float)(k - 1) / rc) * ((float)(k - 1) / rc);
  const bool inside = d < rc;
  const float ph = 3.14159265358979323846f * d / rc;
  const float fc = inside ? 0.5f * (cosf(ph) + 1.0f) : 0.f;
  const float dfc = inside ? -(3.14159265358979323846f / (2.0f * rc)) * sinf(ph) : 0.f;
  float acc = 0.f;
  for (int j = 0; j < k; ++j) {
    const float t = d - (float)j * step;
    acc += g_attr[e * k + j] * (expf(-gamma * t * t) * (-2.0f * gamma * t * fc + dfc));
  }
  g_d2[e] = acc / (2.0f * d);
}

// rvec_e = rvec0_e + (v[dst_e] - v[col_e]),  d2_e = |rvec_e|^2
__global__ void k_edge_geom_fwd(int64_t E, const float* __restrict__ rvec0, const float* __restrict__ v,
                                const int32_t* __restrict__ dst, const int32_t* __restrict__ col,
                                float* __restrict__ rvec, float* __restrict__ d2) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= E) return;
  const size_t i = (size_t)dst[e], j = (size_t)col[e];
  const float x = rvec0[3 * e] + (v[3 * i] - v[3 * j]);
  const float y = rvec0[3 * e + 1] + (v[3 * i + 1] - v[3 * j + 1]);
  const float z = rvec0[3 * e + 2] + (v[3 * i + 2] - v[3 * j + 2]);
  rvec[3 * e] = x; rvec[3 * e + 1] = y; rvec[3 * e + 2] = z;
  d2[e] = x * x + y * y + z * z;
}

// g_r_e = g_rvec_e + 2 g_d2_e rvec_e (g_d2 optional); optionally summed into g_r_sum
__global__ void k_edge_geom_bwd_edge(int64_t E, const float* __restrict__ rvec, const float* g_rvec,
                                     const float* __restrict__ g_d2, float* g_r, float* __restrict__ g_r_sum) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= 3 * E) return;
  float t = g_rvec[idx];
  if (g_d2) t += 2.0f * g_d2[idx / 3] * rvec[idx];
  g_r[idx] = t;
  if (g_r_sum) g_r_sum[idx] += t;
}

// g_v[i] += sum over the edges into i of g_r - sum over the edges out of i of g_r: 16 lanes per atom, each lane its
// edges in order, then a fixed butterfly
__global__ void __launch_bounds__(256) k_edge_geom_bwd_node(int N, const int32_t* __restrict__ row_ptr,
                                                            const int32_t* __restrict__ colT_ptr,
                                                            const int32_t* __restrict__ permT,
                                                            const float* __restrict__ g_r, float* __restrict__ g_v) {
  const int l = threadIdx.x & 15;
  const int i = blockIdx.x * 16 + (threadIdx.x >> 4);
  float s[3] = {0.f, 0.f, 0.f};
  if (i < N) {
    for (int e = row_ptr[i] + l; e < row_ptr[i + 1]; e += 16) {
      s[0] += g_r[3 * (size_t)e]; s[1] += g_r[3 * (size_t)e + 1]; s[2] += g_r[3 * (size_t)e + 2];
    }
    for (int t = colT_ptr[i] + l; t < colT_ptr[i + 1]; t += 16) {
      const size_t e = (size_t)permT[t];
      s[0] -= g_r[3 * e]; s[1] -= g_r[3 * e + 1]; s[2] -= g_r[3 * e + 2];
    }
  }
#pragma unroll
  for (int c = 0; c < 3; ++c) {
#pragma unroll
    for (int o = 8; o >= 1; o >>= 1) s[c] += __shfl_xor(s[c], o);
  }
  if (i < N && l < 3) g_v[3 * (size_t)i + l] += (l == 0 ? s[0] : l == 1 ? s[1] : s[2]);
}

}  // namespace hgnn

using namespace hgnn;

extern "C" int32_t hgnn_edge_rbf(void* stream, int64_t E, const float* d2, int32_t k, float rc, float* attr) {
  HGNN_REQUIRE(E >= 0 && k >= 2 && k <= 16 && rc > 0.f, HGNN_ERR_BAD_SHAPE, "edge_rbf: need E >= 0, 2 <= k <= 16, rc > 0");
  if (E == 0) return HGNN_OK;
  HGNN_REQUIRE(d2 && attr, HGNN_ERR_NULLPTR, "edge_rbf: null pointer");
  hipStream_t st = static_cast<hipStream_t>(stream);
  ProfScope ps(PT_MISC, st);
  k_edge_rbf<<<nblk64(E * k, 256), 256, 0, st>>>(E, k, d2, rc, attr);
  HGNN_LAUNCH_CHECK("k_edge_rbf");
  return HGNN_OK;
}

extern "C" int32_t hgnn_edge_rbf_bwd(void* stream, int64_t E, const float* d2, int32_t k, float rc,
                                     const float* g_attr, float* g_d2) {
  HGNN_REQUIRE(E >= 0 && k >= 2 && k <= 16 && rc > 0.f, HGNN_ERR_BAD_SHAPE, "edge_rbf_bwd: need E >= 0, 2 <= k <= 16, rc > 0");
  if (E == 0) return HGNN_OK;
  HGNN_REQUIRE(d2 && g_attr && g_d2, HGNN_ERR_NULLPTR, "edge_rbf_bwd: null pointer");
  hipStream_t st = static_cast<hipStream_t>(stream);
  ProfScope ps(PT_MISC, st);
  k_edge_rbf_bwd<<<nblk64(E, 256), 256, 0, st>>>(E, k, d2, rc, g_attr, g_d2);
  HGNN_LAUNCH_CHECK("k_edge_rbf_bwd");
  return HGNN_OK;
}

extern "C" int32_t hgnn_edge_geometry_fwd(void* stream, int32_t N, int64_t E, const float* rvec0, const float* v,
                                          const int32_t* dst, const int32_t* col, float* rvec, float* d2) {
  HGNN_REQUIRE(N >= 0 && E >= 0, HGNN_ERR_BAD_SHAPE, "edge_geometry_fwd: negative N or E");
  if (E == 0) return HGNN_OK;
  HGNN_REQUIRE(rvec0 && v && dst && col && rvec && d2, HGNN_ERR_NULLPTR, "edge_geometry_fwd: null pointer");
  hipStream_t st = static_cast<hipStream_t>(stream);
  ProfScope ps(PT_MISC, st);
  k_edge_geom_fwd<<<nblk64(E, 256), 256, 0, st>>>(E, rvec0, v, dst, col, rvec, d2);
  HGNN_LAUNCH_CHECK("k_edge_geom_fwd");
  return HGNN_OK;
}

extern "C" int32_t hgnn_edge_geometry_bwd(void* stream, int32_t N, int64_t E, const int32_t* row_ptr,
                                          const int32_t* colT_ptr, const int32_t* permT, const float* rvec,
                                          const float* g_rvec, const float* g_d2, float* g_r, float* g_r_sum,
                                          float* g_v) {
  HGNN_REQUIRE(N >= 0 && E >= 0, HGNN_ERR_BAD_SHAPE, "edge_geometry_bwd: negative N or E");
  HGNN_REQUIRE(E <= 2147483647LL / 3, HGNN_ERR_OVERFLOW, "edge_geometry_bwd: edge count too large");
  if (E == 0 || N == 0) return HGNN_OK;
  HGNN_REQUIRE(g_rvec && g_r && (!g_d2 || rvec), HGNN_ERR_NULLPTR, "edge_geometry_bwd: null pointer");
  HGNN_REQUIRE(!g_v || (row_ptr && colT_ptr && permT), HGNN_ERR_NULLPTR, "edge_geometry_bwd: null index array");
  HGNN_REQUIRE(g_r_sum != g_r && g_r_sum != g_rvec, HGNN_ERR_BAD_SHAPE, "edge_geometry_bwd: g_r_sum may not alias g_r or g_rvec");
  hipStream_t st = static_cast<hipStream_t>(stream);
  ProfScope ps(PT_MISC, st);
  k_edge_geom_bwd_edge<<<nblk64(3 * E, 256), 256, 0, st>>>(E, rvec, g_rvec, g_d2, g_r, g_r_sum);
  HGNN_LAUNCH_CHECK("k_edge_geom_bwd_edge");
  if (g_v) {
    k_edge_geom_bwd_node<<<(unsigned)((N + 15) / 16), 256, 0, st>>>(N, row_ptr, colT_ptr, permT, g_r, g_v);
    HGNN_LAUNCH_CHECK("k_edge_geom_bwd_node");
  }
  return HGNN_OK;
}
