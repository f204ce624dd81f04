// hgnn_adamw_step: AdamW update of a flat fp32 parameter buffer in one pass.
//
// The paper's training setup names AdamW with learning rate 1e-3 and nothing else; the update is the published
// algorithm (Adam with decoupled weight decay):
//     m <- b1 m + (1-b1) g,   v <- b2 v + (1-b2) g^2,
//     w <- w - lr * ( (m / (1-b1^t)) / (sqrt(v / (1-b2^t)) + eps) + decay * w ).
// One thread takes four consecutive parameters (16-byte accesses); the kernel is a pure stream: it reads w, g, m, v
// and writes w, m, v, 28 bytes per parameter. The constants arrive as doubles; 1 - beta and the bias corrections
// are formed once on the host in double and rounded to float.
#include <cmath>

#include "common.h"
#include "prof.h"

namespace hgnn {

struct AdamWArgs {
  int64_t n;
  float* w;
  const float* g;
  float *m, *v;
  float lr, b1, b2, eps, decay;
  float omb1, omb2;  // 1 - b1, 1 - b2 (formed in double on the host: in float the difference loses five digits)
  float inv_c1;      // 1 / (1 - b1^t)
  float inv_c2;      // 1 / (1 - b2^t)
};

__device__ __forceinline__ void adamw_one(float& w, float g, float& m, float& v, const AdamWArgs& a) {
  m = a.b1 * m + a.omb1 * g;
  v = a.b2 * v + a.omb2 * g * g;
  const float mhat = m * a.inv_c1;
  const float vhat = v * a.inv_c2;
  w = w - a.lr * (mhat / (sqrtf(vhat) + a.eps) + a.decay * w);
}

__global__ void __launch_bounds__(256) k_adamw(AdamWArgs a) {
  const int64_t i4 = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
  if (i4 >= a.n) return;
  if (i4 + 4 <= a.n) {
    float4 w = *reinterpret_cast<const float4*>(a.w + i4);
    const float4 g = *reinterpret_cast<const float4*>(a.g + i4);
    float4 m = *reinterpret_cast<const float4*>(a.m + i4);
    float4 v = *reinterpret_cast<const float4*>(a.v + i4);
    adamw_one(w.x, g.x, m.x, v.x, a);
    adamw_one(w.y, g.y, m.y, v.y, a);
    adamw_one(w.z, g.z, m.z, v.z, a);
    adamw_one(w.w, g.w, m.w, v.w, a);
    *reinterpret_cast<float4*>(a.w + i4) = w;
    *reinterpret_cast<float4*>(a.m + i4) = m;
    *reinterpret_cast<float4*>(a.v + i4) = v;
  } else {
    for (int64_t i = i4; i < a.n; ++i) {
      float w = a.w[i], m = a.m[i], v = a.v[i];
      adamw_one(w, a.g[i], m, v, a);
      a.w[i] = w; a.m[i] = m; a.v[i] = v;
    }
  }
}

}  // namespace hgnn

using namespace hgnn;

extern "C" int32_t hgnn_adamw_step(void* stream, int64_t n, float* w, const float* g, float* m, float* v,
                                   int32_t step, double lr, double beta1, double beta2, double eps,
                                   double weight_decay) {
  HGNN_REQUIRE(n >= 0, HGNN_ERR_BAD_SHAPE, "negative parameter count");
  HGNN_REQUIRE(step >= 1, HGNN_ERR_BAD_SHAPE, "updates are counted from 1 (got %d)", step);
  HGNN_REQUIRE(beta1 >= 0.0 && beta1 < 1.0 && beta2 >= 0.0 && beta2 < 1.0, HGNN_ERR_BAD_SHAPE,
               "beta1 and beta2 must lie in [0, 1)");
  if (n == 0) return HGNN_OK;
  HGNN_REQUIRE(w && g && m && v, HGNN_ERR_NULLPTR, "adamw: null buffer");
  AdamWArgs a;
  a.n = n; a.w = w; a.g = g; a.m = m; a.v = v;
  a.lr = (float)lr; a.b1 = (float)beta1; a.b2 = (float)beta2; a.eps = (float)eps; a.decay = (float)weight_decay;
  a.omb1 = (float)(1.0 - beta1); a.omb2 = (float)(1.0 - beta2);
  a.inv_c1 = (float)(1.0 / (1.0 - std::pow(beta1, (double)step)));
  a.inv_c2 = (float)(1.0 / (1.0 - std::pow(beta2, (double)step)));
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int64_t nthreads = (n + 3) / 4;
  ProfScope ps(PT_MISC, st);
  k_adamw<<<dim3((unsigned)((nthreads + 255) / 256)), 256, 0, st>>>(a);
  HGNN_LAUNCH_CHECK("k_adamw");
  return HGNN_OK;
}
