// Bandwidth-bound kernels of the message-passing layer. Every reduction runs in a fixed order
// (edges of a row in list order inside one wavefront, then a butterfly over lanes): no atomics.
#include "devmath.h"
#include "edgeops.h"

namespace hgnn {

static inline unsigned nblk64(int64_t n, int t) { return (unsigned)((n + t - 1) / t); }

// ---------------------------------------------------------------------------------------------
template <bool WITH_S1>
__global__ void __launch_bounds__(256)
k_edge_pre(int H, int64_t E, const int32_t* __restrict__ dst, const int32_t* __restrict__ col,
           const float* __restrict__ d2, const float* __restrict__ PQ, const float* __restrict__ w1d,
           float* __restrict__ a1, float* __restrict__ s1) {
  const int CH = H >> 2;
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= E * CH) return;
  const int64_t e = idx / CH;
  const int q = (int)(idx - e * CH);
  const long i = dst[e], j = col[e];
  const float dd = d2[e];
  const float4 p = *reinterpret_cast<const float4*>(PQ + i * 2 * H + q * 4);
  const float4 qq = *reinterpret_cast<const float4*>(PQ + j * 2 * H + H + q * 4);
  const float4 w = *reinterpret_cast<const float4*>(w1d + q * 4);
  float z[4] = {p.x + qq.x + dd * w.x, p.y + qq.y + dd * w.y, p.z + qq.z + dd * w.z, p.w + qq.w + dd * w.w};
  float y[4], dy[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) silu_both(z[k], y[k], dy[k]);
  *reinterpret_cast<float4*>(a1 + e * H + q * 4) = make_float4(y[0], y[1], y[2], y[3]);
  if (WITH_S1) *reinterpret_cast<float4*>(s1 + e * H + q * 4) = make_float4(dy[0], dy[1], dy[2], dy[3]);
}

int32_t launch_edge_pre(hipStream_t st, int H, int64_t E, const int32_t* dst, const int32_t* col, const float* d2,
                        const float* PQ, const float* w1d, float* a1, float* s1) {
  if (E <= 0) return HGNN_OK;
  const int64_t n = E * (H / 4);
  ProfScope ps(PT_EDGE_PRE, st);
  if (s1) k_edge_pre<true><<<nblk64(n, 256), 256, 0, st>>>(H, E, dst, col, d2, PQ, w1d, a1, s1);
  else k_edge_pre<false><<<nblk64(n, 256), 256, 0, st>>>(H, E, dst, col, d2, PQ, w1d, a1, s1);
  HGNN_LAUNCH_CHECK("k_edge_pre");
  return HGNN_OK;
}

// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
  return x;
}

template <int VPL>  // columns per lane = H / 64
__global__ void __launch_bounds__(256)
k_seg_fwd(int N, const int32_t* __restrict__ row_ptr, const float* __restrict__ z2, const float* __restrict__ rvec,
          const float* __restrict__ wx, float alpha, const float* __restrict__ v_in, float* __restrict__ M,
          float* __restrict__ v_out) {
  constexpr int H = VPL * 64;
  const int i = (int)(((size_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6);
  const int lane = threadIdx.x & 63;
  if (i >= N) return;
  const int e0 = row_ptr[i], e1 = row_ptr[i + 1];
  float acc[VPL], tx[VPL], ty[VPL], tz[VPL];
#pragma unroll
  for (int k = 0; k < VPL; ++k) acc[k] = tx[k] = ty[k] = tz[k] = 0.f;
  for (int e = e0; e < e1; ++e) {
    const float* zr = z2 + (size_t)e * H + lane * VPL;
    const float rx = rvec[3 * (size_t)e], ry = rvec[3 * (size_t)e + 1], rz = rvec[3 * (size_t)e + 2];
    float zv[VPL];
    if (VPL == 4) {
      const float4 t = *reinterpret_cast<const float4*>(zr);
      zv[0] = t.x; zv[1 % VPL] = t.y; zv[2 % VPL] = t.z; zv[3 % VPL] = t.w;
    } else if (VPL == 2) {
      const float2 t = *reinterpret_cast<const float2*>(zr);
      zv[0] = t.x; zv[1 % VPL] = t.y;
    } else {
      zv[0] = zr[0];
    }
#pragma unroll
    for (int k = 0; k < VPL; ++k) {
      const float m = silu_f(zv[k]);
      acc[k] += m;
      tx[k] += m * rx;
      ty[k] += m * ry;
      tz[k] += m * rz;
    }
  }
  float sx = 0.f, sy = 0.f, sz = 0.f;
#pragma unroll
  for (int k = 0; k < VPL; ++k) {
    const float w = wx[lane * VPL + k];
    M[(size_t)i * H + lane * VPL + k] = alpha * acc[k];
    sx += w * tx[k];
    sy += w * ty[k];
    sz += w * tz[k];
  }
  sx = wave_sum(sx);
  sy = wave_sum(sy);
  sz = wave_sum(sz);
  if (lane == 0) {
    v_out[3 * (size_t)i] = v_in[3 * (size_t)i] + alpha * sx;
    v_out[3 * (size_t)i + 1] = v_in[3 * (size_t)i + 1] + alpha * sy;
    v_out[3 * (size_t)i + 2] = v_in[3 * (size_t)i + 2] + alpha * sz;
  }
}

int32_t launch_seg_fwd(hipStream_t st, int H, int N, const int32_t* row_ptr, const float* z2, const float* rvec,
                       const float* wx, float alpha, const float* v_in, float* M, float* v_out) {
  if (N <= 0) return HGNN_OK;
  const unsigned g = nblk64((int64_t)N * 64, 256);
  ProfScope ps(PT_SEG_FWD, st);
  switch (H) {
    case 64: k_seg_fwd<1><<<g, 256, 0, st>>>(N, row_ptr, z2, rvec, wx, alpha, v_in, M, v_out); break;
    case 128: k_seg_fwd<2><<<g, 256, 0, st>>>(N, row_ptr, z2, rvec, wx, alpha, v_in, M, v_out); break;
    case 256: k_seg_fwd<4><<<g, 256, 0, st>>>(N, row_ptr, z2, rvec, wx, alpha, v_in, M, v_out); break;
    default: return set_error(HGNN_ERR_BAD_SHAPE, "H must be 64, 128 or 256");
  }
  HGNN_LAUNCH_CHECK("k_seg_fwd");
  return HGNN_OK;
}

// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
k_edge_gz2(int H, int64_t E, const int32_t* __restrict__ dst, const float* __restrict__ rvec,
           const float* __restrict__ z2, const float* __restrict__ gM, int ldgM, const float* __restrict__ g_v,
           const float* __restrict__ wx, float alpha, float* __restrict__ g_z2, float* __restrict__ cvec) {
  const int CH = H >> 2;
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= E * CH) return;
  const int64_t e = idx / CH;
  const int q = (int)(idx - e * CH);
  const long i = dst[e];
  const float c = alpha * (g_v[3 * i] * rvec[3 * e] + g_v[3 * i + 1] * rvec[3 * e + 1] + g_v[3 * i + 2] * rvec[3 * e + 2]);
  if (q == 0) cvec[e] = c;
  const float4 z = *reinterpret_cast<const float4*>(z2 + e * H + q * 4);
  const float4 gm = *reinterpret_cast<const float4*>(gM + i * ldgM + q * 4);
  const float4 w = *reinterpret_cast<const float4*>(wx + q * 4);
  float4 o;
  o.x = (alpha * gm.x + c * w.x) * dsilu_f(z.x);
  o.y = (alpha * gm.y + c * w.y) * dsilu_f(z.y);
  o.z = (alpha * gm.z + c * w.z) * dsilu_f(z.z);
  o.w = (alpha * gm.w + c * w.w) * dsilu_f(z.w);
  *reinterpret_cast<float4*>(g_z2 + e * H + q * 4) = o;
}

int32_t launch_edge_gz2(hipStream_t st, int H, int64_t E, const int32_t* dst, const float* rvec, const float* z2,
                        const float* gM, int ldgM, const float* g_v, const float* wx, float alpha, float* g_z2,
                        float* cvec) {
  if (E <= 0) return HGNN_OK;
  const int64_t n = E * (H / 4);
  ProfScope ps(PT_EDGE_GZ2, st);
  k_edge_gz2<<<nblk64(n, 256), 256, 0, st>>>(H, E, dst, rvec, z2, gM, ldgM, g_v, wx, alpha, g_z2, cvec);
  HGNN_LAUNCH_CHECK("k_edge_gz2");
  return HGNN_OK;
}

// ---------------------------------------------------------------------------------------------
template <int VPL>
__global__ void __launch_bounds__(256)
k_segsum(int N, const int32_t* __restrict__ ptr, const int32_t* __restrict__ perm, const float* __restrict__ X,
         float* __restrict__ out, int ldo) {
  constexpr int H = VPL * 64;
  const int i = (int)(((size_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6);
  const int lane = threadIdx.x & 63;
  if (i >= N) return;
  const int t0 = ptr[i], t1 = ptr[i + 1];
  float acc[VPL];
#pragma unroll
  for (int k = 0; k < VPL; ++k) acc[k] = 0.f;
  for (int t = t0; t < t1; ++t) {
    const size_t e = perm ? (size_t)perm[t] : (size_t)t;
    const float* xr = X + e * H + lane * VPL;
    if (VPL == 4) {
      const float4 v = *reinterpret_cast<const float4*>(xr);
      acc[0] += v.x; acc[1 % VPL] += v.y; acc[2 % VPL] += v.z; acc[3 % VPL] += v.w;
    } else if (VPL == 2) {
      const float2 v = *reinterpret_cast<const float2*>(xr);
      acc[0] += v.x; acc[1 % VPL] += v.y;
    } else {
      acc[0] += xr[0];
    }
  }
#pragma unroll
  for (int k = 0; k < VPL; ++k) out[(size_t)i * ldo + lane * VPL + k] = acc[k];
}

int32_t launch_segsum(hipStream_t st, int H, int N, const int32_t* ptr, const int32_t* perm, const float* X,
                      float* out, int ldo, int tag) {
  if (N <= 0) return HGNN_OK;
  const unsigned g = nblk64((int64_t)N * 64, 256);
  ProfScope ps(tag, st);
  switch (H) {
    case 64: k_segsum<1><<<g, 256, 0, st>>>(N, ptr, perm, X, out, ldo); break;
    case 128: k_segsum<2><<<g, 256, 0, st>>>(N, ptr, perm, X, out, ldo); break;
    case 256: k_segsum<4><<<g, 256, 0, st>>>(N, ptr, perm, X, out, ldo); break;
    default: return set_error(HGNN_ERR_BAD_SHAPE, "H must be 64, 128 or 256");
  }
  HGNN_LAUNCH_CHECK("k_segsum");
  return HGNN_OK;
}

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
