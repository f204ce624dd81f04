// Fused per-edge kernels of the message-passing layer (internal).
//
// Edge tensors [E,H] that only travel between these kernels are kept in "fragment order": the order
// in which a wavefront holds a 32-edge x 32-column block in its matrix-core accumulator registers
// (lane l, register v  <->  edge 8*(v>>2) + 4*(l>>5) + (v&3), column (l&31) of the block). Two
// variants, both addressed by 32-edge block eb = e/32 and 32-column block cb = n/32:
//   v-major          ((eb*(H/32) + cb)*16 + v)*64 + l            one element per lane per register
//   operand-packed   bf16: (((eb*(H/32) + cb)*2 + v/8)*64 + l)*8 + v%8
//                    fp32: (((eb*(H/32) + cb)*4 + v/4)*64 + l)*4 + v%4
// The operand-packed form is, unchanged, the A/B operand of the matrix-core instruction that
// contracts over edges (the weight-gradient product), so that product needs no transpose and no LDS.
// With bf16 operands and H = 256 (two column blocks per lane, see edge_pairs()) the v-major tensors hold
// one 32-bit word per lane and register instead: ((eb*(H/64) + wc)*16 + v)*64 + l, the bf16 pair of columns
// wc*64 + (l&31) and wc*64 + 32 + (l&31).
// E is padded to a multiple of 32 in these buffers; padded edges hold zeros where they are summed.
#pragma once

#include "common.h"
#include "prof.h"

namespace hgnn {

inline size_t frag_rows(int64_t E) { return (size_t)((E + 31) / 32 * 32); }

// With bf16 operands and H = 256 each lane of the fused kernels owns two 32-column blocks (2*wc and
// 2*wc+1); node tensors they gather are then stored as bf16 PAIRS: 32-bit word (wc*32 + x) of a row
// holds columns wc*64 + x (low half) and wc*64 + 32 + x (high half).
inline bool edge_pairs(int H, bool bf16) { return bf16 && H == 256; }

struct EdgeFwdArgs {
  int64_t E;
  const int32_t *dst, *col;
  const float* d2;
  const void* PQ;      // [N,2H] fp32: P = h W1a + b1 | Q = h W1b; or bf16 pairs (see edge_pairs())
  const float* w1d;    // [H]
  const void* W2p;     // packed W2 block
  const float* b2;     // [H]
  void* a1_pk;         // out: silu(z1), operand-packed (bf16 or fp32); null: not stored
  void* z2_vm;         // out: z2, v-major (bf16 or fp32)
  // k > 1 edge attributes in place of d2 (bf16 operands only): z1 = P[dst] + Q[col] + attr_e . W1a, the last term
  // formed on the matrix cores from a bf16 copy of the tile's attributes; null: the d2 term above
  const float* attr = nullptr;   // [E,k]
  int k = 0;                     // 2..16
  const float* W1a = nullptr;    // [k,H] rows of W1 that act on the attributes
};
int32_t launch_edge_fwd(hipStream_t st, int H, bool bf16, const EdgeFwdArgs& a);

// M[i,:] = alpha * sum_{e in row i} silu(z2[e,:]);  v_out = v_in + alpha * sum (wx . silu(z2[e,:])) rvec[e,:]
// xe (optional): [E] out, x_e = wx . m_e of every edge
int32_t launch_seg_fwd_vm(hipStream_t st, int H, bool bf16, int N, const int32_t* row_ptr, const void* z2_vm,
                          const float* rvec, const float* wx, float alpha, const float* v_in, float* M,
                          float* v_out, float* xe = nullptr);

// what finishes the rows of g_P that the reverse edge kernel left as per-unit partials (see EdgeBwdArgs::gP)
struct DsumFix {
  const int32_t* row_ptr;
  const float* dpart;
  float* gP;       // null: nothing to finish
  int ldgP;
};

struct EdgeBwdArgs {
  int64_t E;
  const int32_t *dst, *col;
  const float* d2;
  const void* PQ;      // as in the forward kernel
  const float* w1d;
  const void* W2Tp;    // packed W2^T block
  const void* z2_vm;   // saved by the forward kernel
  const void* gM;      // gradient of the aggregated messages: fp32 [N, ldgM], or alpha * g_M as bf16 pairs [N, ldgM words]
  int ldgM;
  const float* cvec;   // [E] c_e = alpha * (g_v[dst[e]] . rvec[e])
  const float* wx;     // [H]
  float alpha;
  void* gz2_pk;        // out: g_z2, operand-packed
  void* gz1_vm;        // out: g_z1, v-major (bf16 or fp32, like the operands)
  float* colpart;      // scratch: [splits][3][H] partial column sums (b2, wx, w1d)
  float* g_b2;         // out [H]
  float* g_wx;         // out [H]
  float* g_w1d;        // out [H] (null with edge attributes)
  // k > 1 edge attributes in place of d2 (see EdgeFwdArgs); g_W1a[j][c] = sum_e attr[e][j] g_z1[e][c]
  const float* attr = nullptr;
  int k = 0;
  const float* W1a = nullptr;
  float* attrpart = nullptr;     // scratch: [splits][k][H] partial sums, edge_bwd_attrpart_floats()
  float* g_W1a = nullptr;        // out [k,H]
  // g_P[i,:] = sum of g_z1 over the edges of destination row i, formed inside the kernel from the tile's g_z1 in LDS
  // (where edge_bwd_sums_dst() holds, without edge attributes; null: not formed, the caller runs launch_segsum_vm).
  // A row that lies inside one unit of DSUM_UNIT edges is written directly; the others leave one partial per unit in dpart
  // ([units][2][H]: slot 1 = the unit in which the row starts, slot 0 = every later unit); edge_bwd_dsum_fix() below
  // names what adds them in unit order and writes zeros for empty rows.
  float* gP = nullptr;           // out [N, ldgP]
  int ldgP = 0;
  float* dpart = nullptr;        // scratch: edge_bwd_dpart_floats(E, H)
  const int32_t* row_ptr = nullptr;   // [N+1], the rows of dst
  int N = 0;
};
// The caller passes this to the launch_segsum_vm call that follows (the source-sorted sum: one wavefront per atom as
// well), which adds the partials on its way; a launch of its own for that would cost about 20 us.
inline DsumFix edge_bwd_dsum_fix(const EdgeBwdArgs& a) { return DsumFix{a.row_ptr, a.dpart, a.gP, a.ldgP}; }
// edges per unit of those sums: the kernel's 64-edge tile. Its two halves are walked by two wavefronts each and the
// row that crosses the middle is put together inside the workgroup, so partials only arise at tile borders (with
// 32-edge units nearly every row of 30 edges left partials: 160 MB of traffic per layer on config 4).
constexpr int DSUM_UNIT = 64;
inline size_t edge_bwd_dpart_floats(int64_t E, int H) { return (size_t)((E + DSUM_UNIT - 1) / DSUM_UNIT) * 2 * H; }
// the operand types and widths for which k_edge_bwd can form g_P itself (an edge's g_z1 is 128 words there)
inline bool edge_bwd_sums_dst(int H, bool bf16) { return edge_pairs(H, bf16) || (!bf16 && H == 128); }
size_t edge_bwd_attrpart_floats(int H);
size_t edge_bwd_colpart_floats(int H);
int32_t launch_edge_bwd(hipStream_t st, int H, bool bf16, const EdgeBwdArgs& a);

// c[e] = alpha * (g_v[dst[e],:] . rvec[e,:])
int32_t launch_edge_cvec(hipStream_t st, int64_t E, const int32_t* dst, const float* rvec, const float* g_v,
                         float alpha, float* cvec);

// gW2[k1][k2] = sum_e a1[e][k1] * g_z2[e][k2], both operands operand-packed; partial: scratch
size_t wgrad_frag_partial_floats(int H);
int32_t launch_wgrad_frag(hipStream_t st, int H, bool bf16, int64_t E, const void* a1_pk, const void* gz2_pk,
                          float* partial, float* gW2);

// The same gradient with a1 = silu(P[dst] + Q[col] + d2*w1d) recomputed from the bf16-pair projected features
// (edge_pairs() layouts only); the forward pass need not store a1 then.
int32_t launch_wgrad_frag_recompute(hipStream_t st, int H, int64_t E, const int32_t* dst, const int32_t* col,
                                    const float* d2, const void* PQ, const float* w1d, const void* gz2_pk,
                                    float* partial, float* gW2);

// The same for fp32 operands at H = 128 (PQ: [N, 2H] fp32); see a1_recomputed() in layer.hip for where it is used.
int32_t launch_wgrad_frag_recompute32(hipStream_t st, int H, int64_t E, const int32_t* dst, const int32_t* col,
                                      const float* d2, const float* PQ, const float* w1d, const void* gz2_pk,
                                      float* partial, float* gW2);

// out[i, 0..H) (row pitch ldo) = sum over t in ptr[i]:ptr[i+1] of X[perm ? perm[t] : t, :], X v-major (bf16 or
// fp32), accumulated in fp32
// fix (optional): wavefront i also finishes row i of the g_P that the reverse edge kernel started (H = 128 or 256)
// dot (optional): [E] out, dot[e] = sum_c wdot[c] X[e][c] for every edge of the list
int32_t launch_segsum_vm(hipStream_t st, int H, bool bf16, int N, const int32_t* ptr, const int32_t* perm,
                         const void* X_vm, float* out, int ldo, int tag, const float* wdot = nullptr,
                         float* dot = nullptr, const DsumFix* fix = nullptr);

// g_attr[e][j] = sum_c X[e][c] W1a[j][c] for every edge (X = g_z1, v-major bf16; 2 <= k <= 16): the gradient with
// respect to k > 1 edge attributes, for callers that ask for it
int32_t launch_gattr_vm(hipStream_t st, int H, int64_t E, const void* X_vm, const float* W1a, int k, float* g_attr);

}  // namespace hgnn
