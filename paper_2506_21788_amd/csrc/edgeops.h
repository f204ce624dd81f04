// Bandwidth-bound kernels of the message-passing layer (internal): per-edge gathers of projected
// node features, destination- and source-sorted segmented reductions, small per-atom helpers.
#pragma once

#include "common.h"
#include "prof.h"

namespace hgnn {

// a1[e,:] = silu(z1), z1 = P[dst[e],:] + Q[col[e],:] + d2[e]*w1d   (P, Q = halves of PQ[N,2H]);
// s1 (optional) = silu'(z1)
int32_t launch_edge_pre(hipStream_t st, int H, int64_t E, const int32_t* dst, const int32_t* col, const float* d2,
                        const float* PQ, const float* w1d, float* a1, float* s1);

// per destination row i (edges row_ptr[i]:row_ptr[i+1]):
//   M[i,:] = alpha * sum silu(z2[e,:]);  v_out[i,:] = v_in[i,:] + alpha * sum (wx . silu(z2[e,:])) * rvec[e,:]
int32_t launch_seg_fwd(hipStream_t st, int H, int N, const int32_t* row_ptr, const float* z2, const float* rvec,
                       const float* wx, float alpha, const float* v_in, float* M, float* v_out);

// g_z2[e,:] = (alpha*gM[dst[e],:] + c_e*wx) * silu'(z2[e,:]),  c_e = alpha * (g_v[dst[e],:] . rvec[e,:]); c -> cvec[e]
int32_t launch_edge_gz2(hipStream_t st, int H, int64_t E, const int32_t* dst, const float* rvec, const float* z2,
                        const float* gM, int ldgM, const float* g_v, const float* wx, float alpha, float* g_z2,
                        float* cvec);

// out[i,:] = sum over t in ptr[i]:ptr[i+1] of X[perm ? perm[t] : t, :]
int32_t launch_segsum(hipStream_t st, int H, int N, const int32_t* ptr, const int32_t* perm, const float* X,
                      float* out, int ldo, int tag);

int32_t launch_copy_f32(hipStream_t st, const float* src, float* dst, int64_t n);
int32_t launch_fill_f32(hipStream_t st, float* dst, int64_t n, float v);

}  // namespace hgnn
