// Fragment-layout matrix products and the converters around them (internal; layouts in wide.h).
// Grouped calls (grp_ptr != null): rows are positions of S groups, group s = positions grp_ptr[s] .. grp_ptr[s+1];
// inside fragment tensors every group starts at a multiple of 256 rows (its rows padded with zeros), so a tensor of
// M positions in S groups takes at most frag_group_rows(M, S) rows.
#pragma once

#include "common.h"
#include "prof.h"

namespace hgnn {

enum { EPI_T = 0, EPI_ROW = 1, EPI_PART = 2 };

inline int64_t frag_group_rows(int64_t M, int S) { return (M + 255) / 256 * 256 + 256 * (int64_t)S; }

struct FGemmArgs {
  const char* A = nullptr;   // fragment (i, kb) at A + (i * a_si + kb * a_sk) KiB
  long a_si = 0, a_sk = 0;
  const char* B = nullptr;   // fragment (j, kb) at B + group * b_grp_stride + (j * b_sj + kb * b_sk) KiB
  long b_sj = 0, b_sk = 0;
  long b_grp_stride = 0;     // bytes
  int nI = 0, nJ = 0;        // 32-blocks of the two free dimensions (multiples of the workgroup tile); grouped
                             // row products: nI covers the largest possible group
  int nkb = 0;               // 16-blocks of the contraction (even); grouped weight gradients: of the largest group
  int kper = 0;              // per split (even)
  int nsplit = 1;
  const int32_t* grp_ptr = nullptr;
  int S = 1;
  // EPI_T: bf16 T fragments, t_ncb column blocks per row group
  char* T = nullptr;
  int t_ncb = 0;
  // EPI_ROW
  int M = 0;                 // valid rows (ungrouped)
  const int32_t* row_idx = nullptr;   // grouped: position -> output row
  float* Cf = nullptr;       // fp32 out, columns < ncol_f
  long ldc = 0;
  int ncol_f = 0;
  unsigned short* Cb = nullptr;   // bf16 out, all columns of the tile
  long ldcb = 0;
  const float* r1 = nullptr;      // residuals added to Cf (columns < ncol_f)
  long ld1 = 0;
  const float* r2 = nullptr;
  long ld2 = 0;
  int vec = 1;                    // floats per access of Cf / r1 / r2 (set by the launcher from their alignment)
  // EPI_T and EPI_ROW: bias[group * bias_grp_stride + col] for col < nbias
  const float* bias = nullptr;
  int nbias = 0;
  long bias_grp_stride = 0;
  // EPI_PART: fp32 partial[group][split][row][col]
  float* P = nullptr;
  long ldp = 0, split_stride = 0;
  int tag = PT_GEMM_NODE;
  // launch_fgemm_rows_T only, optional (seg_dst != null): rows are destination-sorted edges and the product is z2.
  // The kernel then also sums m = silu(z2) per destination atom over each wavefront's strip of 64 rows:
  //   atoms that lie inside one strip:  seg_M[atom][col] = seg_alpha * sum
  //   atoms that reach past the strip's end / begin before it:  seg_last / seg_first [strip][col] = sum (unscaled)
  // and x_e = wx . m_e per edge and column tile:  seg_xe[tile * seg_xe_stride + edge]
  const int32_t* seg_dst = nullptr;
  const int32_t* seg_row_ptr = nullptr;
  const float* seg_wx = nullptr;
  int seg_H = 0;            // valid columns of wx
  long seg_E = 0;           // valid rows
  float seg_alpha = 0.f;
  float* seg_M = nullptr;
  long seg_ldm = 0;
  float* seg_first = nullptr;
  float* seg_last = nullptr;
  long seg_ldp = 0;         // pitch of seg_first / seg_last
  float* seg_xe = nullptr;
  long seg_xe_stride = 0;
};
int32_t launch_fgemm_rows(hipStream_t st, const FGemmArgs& a);     // EPI_ROW, 256 x 128 tiles (128 x 128 for few rows)
int32_t launch_fgemm_rows_T(hipStream_t st, const FGemmArgs& a);   // EPI_T, 256 x 128 tiles

// dest[group * dest_grp_stride + pa * strideA + pb * strideB + r1 * HB + r2] = (A^T B)[pa * HpA + r1][pb * HpB + r2]
// for r1 < HA, r2 < HB, summed over the rows (of each group) in a fixed order. A, B: T fragments.
struct FWgradArgs {
  const char* A_T = nullptr;
  int a_ncb = 0, a_cb0 = 0, nI = 0;   // column blocks per row group, first block used, blocks used (multiple of 4)
  const char* B_T = nullptr;
  int b_ncb = 0, b_cb0 = 0, nJ = 0;
  int64_t rows = 0;                    // padded rows (ungrouped), or the largest possible group's padded rows
  const int32_t* grp_ptr = nullptr;
  int S = 1;
  int HpA = 0, HA = 0, HpB = 0, HB = 0;
  float* partial = nullptr;
  size_t partial_floats = 0;
  float* dest = nullptr;
  long strideA = 0, strideB = 0, dest_grp_stride = 0;
  int tag = PT_WGRAD_NODE;
};
int32_t launch_fwgrad(hipStream_t st, const FWgradArgs& a);

struct PackPart {
  long src_off;        // B[k][n] = src[src_off + k * sk + n * sn] for k < K, n < Nn, else 0
  int sk, sn;
  long dst_off;        // element offset of the destination matrix this part belongs to
  int nkb_total;       // fragments per column block of that destination
  int kb0, nb0;        // where the part's (Kp/16 x Np/32) fragments sit in it
};
struct PackFragArgs {
  const float* src = nullptr;
  unsigned short* dst = nullptr;
  int K = 0, Nn = 0;   // valid extent of every part
  int Kp = 0, Np = 0;  // padded extent of every part
  int nparts = 0;
  PackPart part[8];
  int groups = 1;
  long src_grp_stride = 0, dst_grp_stride = 0;   // elements
};
int32_t launch_pack_frag(hipStream_t st, const PackFragArgs& a);

// row-major fp32 -> fragments.  mode 0: x, 1: silu(x), 2: x * silu'(z)
struct ToFragArgs {
  const float* X = nullptr;
  long ldx = 0;
  const float* Z = nullptr;
  long ldz = 0;
  int mode = 0;
  int M = 0;          // valid rows (ungrouped)
  int Mp = 0;         // rows covered (multiple of 256; grouped: enough for the largest possible group)
  int ncol = 0;       // valid columns
  int Cp = 0;         // columns covered (multiple of 32), columns >= ncol give zeros
  const int32_t* grp_ptr = nullptr;
  int S = 1;
  const int32_t* row_idx = nullptr;   // grouped: position -> source row; null: the source is indexed by padded row
  char* R = nullptr;  // R fragments: r_nkb contraction blocks per row block, this tensor starts at block r_kb0
  int r_nkb = 0, r_kb0 = 0;
  char* T = nullptr;  // T fragments: t_ncb column blocks per row group, this tensor starts at block t_cb0
  int t_ncb = 0, t_cb0 = 0;
};
int32_t launch_to_frag(hipStream_t st, const ToFragArgs& a);

// dest[group * dest_grp_stride + c] = sum over the rows (of each group) of w[row] * f(X[row][c]), c < ncol;
// f as in ToFragArgs::mode, w optional; fixed summation order
struct ColsumRowsArgs {
  const float* X = nullptr;
  long ldx = 0;
  const float* Z = nullptr;
  long ldz = 0;
  int mode = 0;
  const float* w = nullptr;
  int M = 0;                          // rows (ungrouped), or the largest possible group
  int ncol = 0;
  const int32_t* grp_ptr = nullptr;
  int S = 1;
  const int32_t* row_idx = nullptr;   // as in ToFragArgs
  float* partial = nullptr;           // colsum_rows_partial_floats(M, ncol, S)
  float* dest = nullptr;
  long dest_grp_stride = 0;
};
size_t colsum_rows_partial_floats(int M, int ncol, int S);
int32_t launch_colsum_rows(hipStream_t st, const ColsumRowsArgs& a);

}  // namespace hgnn
