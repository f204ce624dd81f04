// Dense building blocks on the matrix cores (internal): packed H x H weight blocks, a row-tile GEMM
// with fused load transform / epilogue, the transposed ("weight gradient") GEMM with deterministic
// split-K, and column sums.
#pragma once

#include "common.h"
#include "prof.h"

namespace hgnn {

// ---- packed weights -------------------------------------------------------------------------
// One H x H block B[k][n] is stored in the order the matrix-core B operand is consumed, so that a
// wavefront's load is one contiguous kilobyte. Elements per block: H*H (bf16 or fp32).
struct PackDesc {
  long src_off;  // element offset into the fp32 source buffer
  int sk, sn;    // B[k][n] = src[src_off + k*sk + n*sn]
};
constexpr int MAX_PACK = 16;
struct PackArgs {
  const float* src;
  void* dst;  // block b goes to dst + b*H*H elements
  int nblocks;
  PackDesc d[MAX_PACK];
  // optional (fp32 packing only): one more block, d[x3_desc], also as three bf16 planes of H*H elements each
  // (hi, mid, lo: the block is their sum), every plane in the bf16 B-operand order: what the fused edge kernels
  // multiply with when the operands are fp32
  void* x3_dst = nullptr;
  int x3_desc = 0;
};
int32_t launch_pack(hipStream_t st, int H, bool bf16, const PackArgs& a, int groups = 1, long src_grp_stride = 0,
                    long dst_grp_stride_elems = 0);
inline size_t packed_block_bytes(int H, bool bf16) { return (size_t)H * H * (bf16 ? 2 : 4); }
inline size_t packed_x3_bytes(int H) { return (size_t)H * H * 6; }

// ---- row-tile GEMM --------------------------------------------------------------------------
// C[rows, cb*H + (0..H)] = epilogue( sum_kc  f(A[kc][rows, 0..H]) x B[blk[kc][cb]] )
struct GemmArgs {
  const float* A[2] = {nullptr, nullptr};
  int lda[2] = {0, 0};
  int nkc = 1;
  int a_silu = 0;            // apply silu to A on load
  const void* B = nullptr;   // packed blocks
  long blk[2][2] = {{0, 0}, {0, 0}};  // block index (in units of blocks) for [kc][cb]
  long grp_blk_stride = 0;   // blocks to skip per group
  const int32_t* row_idx = nullptr;   // optional: position -> row (gather A / scatter C)
  const int32_t* grp_ptr = nullptr;   // optional: [S+1] positions of each group
  int S = 1;
  int M = 0;                 // number of positions
  const float* bias = nullptr;
  int bias_cb_mask = 0;      // bit cb set: add bias[col] on that column block
  long grp_bias_stride = 0;
  const float* mul = nullptr;  // multiply by mul[row, col] (or dsilu(mul) when mul_is_z)
  int ldmul = 0;
  int mul_is_z = 0;
  const float* add1 = nullptr;
  int ldadd1 = 0;
  int add1_cb_mask = 3;      // bit cb set: add1 applies to that column block
  const float* add2 = nullptr;
  int ldadd2 = 0;
  float* C = nullptr;
  int ldc = 0;
  int ncb = 1;
  // optional: column blocks in pair_cb_mask are written as bf16 pairs (see edge_pairs()) into Cpair instead of C:
  // word (wc*32 + x) of a row at word offset pair_off[cb]; plain bias only (no mul / add) on those blocks
  unsigned* Cpair = nullptr;
  int ldpair = 0;
  int pair_cb_mask = 0;
  int pair_off[2] = {0, 0};
  float pair_scale = 1.f;   // factor on the pair output (after the bias)
  int tag = PT_GEMM_NODE;  // timing class
};
int32_t launch_gemm(hipStream_t st, int H, bool bf16, const GemmArgs& a);
// Two products in a row per row tile, the second one reading the first one's finished tile (through silu when
// keep_silu is set) from LDS instead of its own A; with first == nullptr the second one alone, its A tile (one k
// chunk) staged once for all of its column blocks. One launch; no groups, no row indirection.
int32_t launch_gemm_chain(hipStream_t st, int H, bool bf16, const GemmArgs* first, const GemmArgs& second, int keep_silu);

// ---- transposed GEMM (sum over rows of outer products), split-K ------------------------------
// block (ia, ib): out[k1][k2] = sum_r f(A[ia][r][k1]) * B[ib][r][k2]
struct WgradArgs {
  const float* A[2] = {nullptr, nullptr};
  int lda[2] = {0, 0};
  int nA = 1;
  int a_silu = 0;
  const float* B[2] = {nullptr, nullptr};
  int ldb[2] = {0, 0};
  int nB = 1;
  const int32_t* row_idx = nullptr;
  const int32_t* grp_ptr = nullptr;
  int S = 1;
  int64_t M = 0;
  float* dest[4] = {nullptr, nullptr, nullptr, nullptr};  // block ia*nB+ib -> H*H floats, row-major
  long grp_dest_stride = 0;
  float* partial = nullptr;  // scratch, wgrad_partial_floats()
  // optional: column sums of the B operands (the bias gradients that go with these weight gradients), taken from
  // the tiles the kernel stages anyway: colsum_dest[ib] (H floats, may be null) = sum over rows of B[ib]
  float* colsum_dest[2] = {nullptr, nullptr};
  float* colsum_partial = nullptr;   // scratch, wgrad_colsum_partial_floats()
  int tag = PT_WGRAD_NODE;
};
size_t wgrad_colsum_partial_floats(int H, int64_t M);   // room for the column sums of four B operands
// Up to three such products over the same rows in ONE launch (no groups, no row indirection): every job keeps its own
// operands and destinations; `partial` and `colsum_partial` of job 0 serve all of them and must hold
// wgrad_partial_floats(H, M, total blocks, 1) and wgrad_colsum_partial_floats(H, M) floats. At most 8 blocks and 4
// B operands in total.
int32_t launch_wgrad_multi(hipStream_t st, int H, bool bf16, const WgradArgs* jobs, int njobs);
int wgrad_splits(int64_t M);
size_t wgrad_partial_floats(int H, int64_t M, int nblocks, int S);
int32_t launch_wgrad(hipStream_t st, int H, bool bf16, const WgradArgs& a);

// ---- column sums ----------------------------------------------------------------------------
// out[c] = sum_r w[r] * f(X[r][c])   (w optional; f = identity or silu), grouped like the above
struct ColsumArgs {
  const float* X = nullptr;
  int ldx = 0;
  const float* w = nullptr;
  int f_silu = 0;
  const int32_t* row_idx = nullptr;
  const int32_t* grp_ptr = nullptr;
  int S = 1;
  int64_t M = 0;
  float* dest = nullptr;  // [H] (+ grp*grp_dest_stride)
  long grp_dest_stride = 0;
  float* partial = nullptr;  // scratch, colsum_partial_floats()
};
size_t colsum_partial_floats(int H, int64_t M, int S);
int32_t launch_colsum(hipStream_t st, int H, const ColsumArgs& a);

// dest[blk][i] (+ grp*grp_dest_stride) = sum over s < nsplit of partial[((grp*nsplit + s)*nblk + blk)*blk_elems + i],
// summed in ascending s
int32_t launch_reduce_partials(hipStream_t st, const float* partial, int nsplit, int nblk, long blk_elems,
                               float* const dest[4], int groups, long grp_dest_stride);

// While a ReduceQueueScope is alive on this host thread, reductions of split partials (the ones above, also the
// ones the weight-gradient and edge kernels' launchers ask for) are collected instead of launched; flush() runs
// them all as one launch on the scope's stream. The caller keeps every partial buffer untouched until then, and
// nothing it enqueues before the flush may read a reduction's result. A scope that is destroyed without a flush
// drops its jobs (error paths).
struct ReduceQueueScope {
  explicit ReduceQueueScope(hipStream_t st, bool enable);
  ~ReduceQueueScope();
  int32_t flush();
  ReduceQueueScope(const ReduceQueueScope&) = delete;
  ReduceQueueScope& operator=(const ReduceQueueScope&) = delete;
 private:
  bool active_;
};

}  // namespace hgnn
