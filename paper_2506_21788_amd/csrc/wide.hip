// Message-passing layer for hidden widths other than 64 / 128 / 256 (see wide.h for the operand layouts):
//   k_fgemm        out[i][j] += A(i, kb) x B(j, kb) over 1 KiB fragments staged through LDS; epilogues: row-major
//                  fp32 / bf16 with bias and residuals (atom tensors), fp32 split partials (weight gradients)
//   k_fgemm_ad     the per-edge products (result as T fragments), A fragments straight into registers; the z2 product
//                  also forms M_i = alpha sum silu(z2) per destination atom and x_e = wx . m_e in its epilogue
//   k_seg_fwd_fix  the atoms whose edges span several 64-row strips of that epilogue, v'_i = v_i + alpha sum x_e rvec_e
//   k_pack_frag    fp32 weight slices -> B fragments (zero padded)
//   k_to_frag      row-major fp32 atom tensor -> R and / or T fragments (optionally silu(x) or x * silu'(z))
//   k_edge_elem    the three element-wise edge kernels on 32 x 128 tiles: a1 = silu(P[dst] + Q[col] + d2 w1d) -> R, T;
//                  g_z2 = (alpha g_M[dst] + c_e wx) silu'(z2) -> R, T (+ column sums for g_b2, g_wx);
//                  g_z1 = g_a1 silu'(z1) -> row-major (+ column sums for g_b1, g_w1d)
//   k_segsum_rows  per-atom sums of g_z1 over the destination-sorted rows and over the source-sorted edge list
// The layer follows the same algebra as the narrow path: the first edge layer is split by linearity into per-atom
// products P = h W1a + b1, Q = h W1b that the edges gather.
#include "wide.h"

#include "devmath.h"
#include "frag.h"
#include "side.h"
#include "edge_fused.h"
#include "edgeops.h"

namespace hgnn {

typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));

// row of slot u of lane half g in the 16-row group rb16 (the accumulator layout of the 32x32 matrix-core tile)
__device__ __forceinline__ int tset_row(int rb16, int g, int u) { return rb16 * 16 + 8 * (u >> 2) + 4 * g + (u & 3); }
// rows of group grp are the positions ptr[grp] .. ptr[grp+1]; in fragment tensors every group starts at a multiple
// of 256 rows: pad0 = first padded row of the group
__device__ __forceinline__ void group_range(const int32_t* ptr, int grp, int& pos0, int& n, int& pad0) {
  pad0 = 0;
  for (int t = 0; t < grp; ++t) pad0 += (ptr[t + 1] - ptr[t] + 255) / 256 * 256;
  pos0 = ptr[grp];
  n = ptr[grp + 1] - pos0;
}
__device__ __forceinline__ float bf_lo(unsigned w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf_hi(unsigned w) { return __uint_as_float(w & 0xffff0000u); }

// ---------------------------------------------------------------------------------------------
// fragment GEMM
// ---------------------------------------------------------------------------------------------
// NW wavefronts per workgroup, arranged (NW / 2) x 2 over the tile; each owns WI x WJ blocks of 32 x 32
template <int WI, int WJ, int NW = 4, int KC_ = 2>
struct FCfg {
  static constexpr int KC = KC_;             // contraction blocks staged per step
  static constexpr int TI = (NW / 2) * WI, TJ = 2 * WJ;
  static constexpr int NF = KC * (TI + TJ);  // fragments per step
  static constexpr int PASSES = NF / NW;     // each wavefront copies one fragment per pass
  static constexpr int LDS_BYTES = 2 * NF * 1024;   // two steps: one being multiplied, one being written
  static_assert(NF % NW == 0, "fragments per step must divide among the wavefronts");
};

template <int WI, int WJ, int EPI, int NW = 4, int KC = 2>
__global__ void __launch_bounds__(64 * NW, (WI * WJ <= 8 ? 2 : 1)) k_fgemm(FGemmArgs p) {
  static_assert(EPI == EPI_ROW || EPI == EPI_PART, "results as T fragments come from k_fgemm_ad");
  using C = FCfg<WI, WJ, NW, KC>;
  extern __shared__ __align__(16) u32x4_t lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wi = wave >> 1, wj = wave & 1;
  // Workgroups go to the 8 XCDs round-robin by blockIdx.x, and each XCD has its own L2. Workgroups that read the
  // same operand panel are therefore given ids of the same residue mod 8, next to each other in that XCD's order:
  // row products: the column tiles of one row tile; split partials: all tiles of one split. blockIdx.z: group.
  const int xcd = blockIdx.x & 7, q = blockIdx.x >> 3;
  const int nTj = (p.nJ + C::TJ - 1) / C::TJ;
  int ti, tj, split = 0;
  if (EPI == EPI_PART) {
    const int tiles = ((p.nI + C::TI - 1) / C::TI) * nTj;   // a last row tile may stick out past nI
    const int t = q % tiles;
    split = (q / tiles) * 8 + xcd;     // the launcher makes the split count a multiple of 8
    ti = t / nTj;
    tj = t % nTj;
  } else {
    ti = (q / nTj) * 8 + xcd;
    tj = q % nTj;
    if (ti >= p.nI / C::TI) return;    // uniform over the workgroup, before any barrier
  }
  int i0 = ti * C::TI;
  const int j0 = tj * C::TJ;
  const int grp = blockIdx.z;
  int mvalid = p.M, pos0 = 0, pad0 = 0, kbase = 0, knum = p.nkb;
  if (p.grp_ptr) {
    int n;
    group_range(p.grp_ptr, grp, pos0, n, pad0);
    const int npad = (n + 255) / 256 * 256;
    if (EPI == EPI_PART) {
      kbase = pad0 / 16;
      knum = npad / 16;
    } else {
      if (ti * C::TI * 32 >= npad) return;   // uniform over the workgroup, before any barrier
      i0 += pad0 / 32;
      mvalid = pad0 + n;
    }
  }
  const int kbeg = kbase + split * p.kper;
  const int kend = kbeg + p.kper < kbase + knum ? kbeg + p.kper : kbase + knum;
  const char* Bg = p.B + (long)grp * p.b_grp_stride;

  // pass s copies fragment f = 4 s + wave of the step: first the KC x TI fragments of A, then the KC x TJ of B
  const char* src[C::PASSES];
  long kst[C::PASSES];
#pragma unroll
  for (int s = 0; s < C::PASSES; ++s) {
    const int f = NW * s + wave;
    if (f < C::KC * C::TI) {
      const int kk = f / C::TI, ii = f % C::TI;
      // (split partials: row blocks past nI repeat the last one and are never stored)
      const int ib = (EPI == EPI_PART && i0 + ii >= p.nI) ? p.nI - 1 : i0 + ii;
      src[s] = p.A + ((long)ib * p.a_si + (long)kk * p.a_sk) * 1024 + lane * 16;
      kst[s] = p.a_sk * 1024;
    } else {
      const int f2 = f - C::KC * C::TI;
      const int kk = f2 / C::TJ, jj = f2 % C::TJ;
      // (a column tile may stick out past the last block: those fragments repeat the last one and are never stored)
      const int jb = j0 + jj < p.nJ ? j0 + jj : p.nJ - 1;
      src[s] = Bg + ((long)jb * p.b_sj + (long)kk * p.b_sk) * 1024 + lane * 16;
      kst[s] = p.b_sk * 1024;
    }
  }
  f32x16_t acc[WI][WJ];
#pragma unroll
  for (int i = 0; i < WI; ++i)
#pragma unroll
    for (int j = 0; j < WJ; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // Pipeline: the LDS holds two steps; two register sets carry the steps on their way. In iteration c the products
  // read step c from one half, the set that holds step c+1 (asked for two iterations ago) is written to the other
  // half, step c+3 is asked for into that set, one barrier, and the sets swap roles. Loads are unconditional from a
  // clamped step, so the staging registers stay registers.
  const int nch = kbeg < kend ? (kend - kbeg) / C::KC : 0;
  u32x4_t preX[C::PASSES], preY[C::PASSES];
  auto kclamp = [&](int ch) { return kbeg + (ch < nch ? ch : (nch > 0 ? nch - 1 : 0)) * C::KC; };
  constexpr int STAGE = C::NF * 64;   // 16-byte units per half
  if (nch > 0) {
    {
      const long k0 = kclamp(0), k1 = kclamp(1), k2 = kclamp(2);
#pragma unroll
      for (int s = 0; s < C::PASSES; ++s) preX[s] = *reinterpret_cast<const u32x4_t*>(src[s] + k0 * kst[s]);
#pragma unroll
      for (int s = 0; s < C::PASSES; ++s) preY[s] = *reinterpret_cast<const u32x4_t*>(src[s] + k1 * kst[s]);
#pragma unroll
      for (int s = 0; s < C::PASSES; ++s) lds[(NW * s + wave) * 64 + lane] = preX[s];
#pragma unroll
      for (int s = 0; s < C::PASSES; ++s) preX[s] = *reinterpret_cast<const u32x4_t*>(src[s] + k2 * kst[s]);
    }
    __syncthreads();
    // after the prologue: half 0 = step 0, Y = step 1, X = step 2
    // (the number of steps is even, see the launcher: the loop body has no branch, which lets the compiler count the
    // outstanding loads exactly instead of waiting for all of them)
    for (int c = 0; c < nch; c += 2) {
#pragma unroll
      for (int par = 0; par < 2; ++par) {
        const int cc = c + par;
        {
          const u32x4_t* cur = lds + par * STAGE;
          const int nslot = par ^ 1;
#pragma unroll
          for (int kk = 0; kk < C::KC; ++kk) {
            bf16x8_t a[WI], b[WJ];
#pragma unroll
            for (int i = 0; i < WI; ++i) a[i] = __builtin_bit_cast(bf16x8_t, cur[(kk * C::TI + wi * WI + i) * 64 + lane]);
#pragma unroll
            for (int j = 0; j < WJ; ++j)
              b[j] = __builtin_bit_cast(bf16x8_t, cur[(C::KC * C::TI + kk * C::TJ + wj * WJ + j) * 64 + lane]);
#pragma unroll
            for (int i = 0; i < WI; ++i)
#pragma unroll
              for (int j = 0; j < WJ; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
          }
          // step cc+1 into the ring, step cc+3 on its way (even iterations use set Y, odd ones set X)
          const long kn = kclamp(cc + 3);
          if (par == 0) {
#pragma unroll
            for (int s = 0; s < C::PASSES; ++s) lds[nslot * STAGE + (NW * s + wave) * 64 + lane] = preY[s];
#pragma unroll
            for (int s = 0; s < C::PASSES; ++s) preY[s] = *reinterpret_cast<const u32x4_t*>(src[s] + kn * kst[s]);
          } else {
#pragma unroll
            for (int s = 0; s < C::PASSES; ++s) lds[nslot * STAGE + (NW * s + wave) * 64 + lane] = preX[s];
#pragma unroll
            for (int s = 0; s < C::PASSES; ++s) preX[s] = *reinterpret_cast<const u32x4_t*>(src[s] + kn * kst[s]);
          }
          __syncthreads();
        }
      }
    }
  }

  // accumulator register v of lane (g, x): row 8 (v >> 2) + 4 g + (v & 3), column x of the 32 x 32 block
  const int g = lane >> 5, x = lane & 31;
  if constexpr (EPI == EPI_ROW) {
    // Row-major results go through the LDS, one 32-row block per wavefront row at a time (64 rows x 128 columns of
    // fp32), so that bias, residuals and the output move as whole rows: a thread owns four consecutive columns.
    static_assert(C::TJ == 4 && NW == 4 && C::LDS_BYTES >= 64 * 128 * 4, "staging tile is 64 rows x 128 columns");
    float* stg = reinterpret_cast<float*>(lds);
    const int c4 = (tid & 31) * 4, r8 = tid >> 5;
    const int col = j0 * 32 + c4;
    const bool col_ok = col < p.nJ * 32;
    float bias4[4] = {0.f, 0.f, 0.f, 0.f};
    if (p.bias) {
#pragma unroll
      for (int t = 0; t < 4; ++t)
        if (col + t < p.nbias) bias4[t] = p.bias[(long)grp * p.bias_grp_stride + col + t];
    }
#pragma unroll
    for (int i = 0; i < WI; ++i) {
      __syncthreads();   // the fragments (or the previous block row) have been read
#pragma unroll
      for (int j = 0; j < WJ; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          stg[(wi * 32 + 8 * (v >> 2) + 4 * g + (v & 3)) * 128 + wj * 64 + j * 32 + x] = acc[i][j][v];
      __syncthreads();
#pragma unroll
      for (int rr = 0; rr < 8; ++rr) {
        const int lrow = rr * 8 + r8;
        const int prow = (i0 + (lrow >> 5) * WI + i) * 32 + (lrow & 31);
        if (prow < mvalid && col_ok) {
          const long row = p.row_idx ? p.row_idx[pos0 + prow - pad0] : prow;   // scatter to the caller's rows
          const float4 sv = *reinterpret_cast<const float4*>(&stg[lrow * 128 + c4]);
          float val[4] = {sv.x + bias4[0], sv.y + bias4[1], sv.z + bias4[2], sv.w + bias4[3]};
          if (p.Cf && col < p.ncol_f) {
            float* cp = p.Cf + row * p.ldc + col;
            const float* p1 = p.r1 ? p.r1 + row * p.ld1 + col : nullptr;
            const float* p2 = p.r2 ? p.r2 + row * p.ld2 + col : nullptr;
            if (p.vec == 4 && col + 4 <= p.ncol_f) {
              if (p1) { const float4 t = *reinterpret_cast<const float4*>(p1); val[0] += t.x; val[1] += t.y; val[2] += t.z; val[3] += t.w; }
              if (p2) { const float4 t = *reinterpret_cast<const float4*>(p2); val[0] += t.x; val[1] += t.y; val[2] += t.z; val[3] += t.w; }
              *reinterpret_cast<float4*>(cp) = make_float4(val[0], val[1], val[2], val[3]);
            } else if (p.vec >= 2 && col + 4 <= p.ncol_f) {
#pragma unroll
              for (int h2 = 0; h2 < 2; ++h2) {
                if (p1) { const float2 t = *reinterpret_cast<const float2*>(p1 + 2 * h2); val[2 * h2] += t.x; val[2 * h2 + 1] += t.y; }
                if (p2) { const float2 t = *reinterpret_cast<const float2*>(p2 + 2 * h2); val[2 * h2] += t.x; val[2 * h2 + 1] += t.y; }
                *reinterpret_cast<float2*>(cp + 2 * h2) = make_float2(val[2 * h2], val[2 * h2 + 1]);
              }
            } else {
#pragma unroll
              for (int t = 0; t < 4; ++t)
                if (col + t < p.ncol_f) {
                  if (p1) val[t] += p1[t];
                  if (p2) val[t] += p2[t];
                  cp[t] = val[t];
                }
            }
          }
          if (p.Cb) {   // all columns of the tile (the pitch is a multiple of 128)
            uint2 w;
            w.x = pack_bf16x2(val[0], val[1]);
            w.y = pack_bf16x2(val[2], val[3]);
            *reinterpret_cast<uint2*>(p.Cb + row * p.ldcb + col) = w;
          }
        }
      }
    }
    return;
  }
#pragma unroll
  for (int j = 0; j < WJ; ++j) {
    const int jb = j0 + wj * WJ + j;
    if (jb >= p.nJ) continue;   // partial column tile
    const int colx = jb * 32 + x;
#pragma unroll
    for (int i = 0; i < WI; ++i) {
      const int ib = i0 + wi * WI + i;
      if (ib >= p.nI) continue;   // partial row tile
      float* out = p.P + ((long)grp * p.nsplit + split) * p.split_stride;   // [group][split]
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = ib * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
        out[(long)row * p.ldp + colx] = acc[i][j][v];
      }
    }
  }
}

template <int WI, int WJ, int EPI, int NW = 4, int KC = 2>
static int32_t launch_fgemm_t(hipStream_t st, const FGemmArgs& a) {
  using C = FCfg<WI, WJ, NW, KC>;
  // (an even number of steps per workgroup: contraction counts are multiples of two steps)
  HGNN_REQUIRE((a.nI % C::TI == 0 || EPI == EPI_PART) && (a.nJ % C::TJ == 0 || EPI != EPI_PART) && a.nkb % (2 * C::KC) == 0 &&
                   a.kper % (2 * C::KC) == 0 && a.kper > 0,
               HGNN_ERR_BAD_SHAPE, "fragment GEMM: %d x %d blocks, %d contraction blocks do not tile", a.nI, a.nJ, a.nkb);
  if (a.nI == 0 || a.nJ == 0) return HGNN_OK;
  HGNN_REQUIRE(EPI == EPI_PART ? (a.nsplit % 8 == 0 && (long)a.nsplit * a.kper >= a.nkb) : (a.nsplit == 1 && a.kper == a.nkb),
               HGNN_ERR_BAD_SHAPE, "fragment GEMM: bad split of the contraction");
  const int groups = a.grp_ptr ? a.S : 1;
  const long nTi = (a.nI + C::TI - 1) / C::TI, nTj = (a.nJ + C::TJ - 1) / C::TJ;
  const long gx = EPI == EPI_PART ? (long)a.nsplit * nTi * nTj : (nTi + 7) / 8 * 8 * nTj;
  HGNN_REQUIRE(gx <= 2147483647L && groups <= 65535, HGNN_ERR_OVERFLOW, "fragment GEMM: grid too large");
  static bool lds_set = false;   // the ring may exceed the default dynamic LDS limit: raise it once per variant
  if (!lds_set) {
    HGNN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&k_fgemm<WI, WJ, EPI, NW, KC>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES));
    lds_set = true;
  }
  ProfScope ps(a.tag, st);
  k_fgemm<WI, WJ, EPI, NW, KC><<<dim3((unsigned)gx, 1, groups), 64 * NW, C::LDS_BYTES, st>>>(a);
  HGNN_LAUNCH_CHECK("k_fgemm");
  return HGNN_OK;
}

// Row product with the result as T fragments, tile 256 x 128, A fragments straight from memory into registers:
// wavefront w owns row blocks i0 + 2 w, + 1 and all four column blocks, so nobody else needs its A fragments. A sits
// in a register ring of four steps, asked for three steps ahead; only B (shared by the four wavefronts) passes
// through the LDS: per matrix-core instruction half an LDS fragment read instead of three quarters and a third of
// the LDS writes. Steps of 32 k, four per loop body (the contraction is a multiple of 128).
// (Measured against this: the same kernel with eight wavefronts on a 256 x 256 tile, which loads a third fewer
// operand bytes per flop, runs 12 - 20 % slower: one workgroup per compute unit leaves nothing to run while its
// wavefronts meet at the barrier; with 128 x 128 tiles and three workgroups per compute unit it runs 20 % slower.)
// SEG: the rows are destination-sorted edges and the product is z2: the epilogue also forms m = silu(z2), its sums per
// destination atom over the wavefront's 64 rows and x_e = wx . m_e per edge (see FGemmArgs::seg_*), so that no other
// kernel has to read z2 in the forward pass. The vector units are idle during the products: the other resident
// workgroup keeps the matrix cores busy meanwhile.
template <bool SEG>
__global__ void __launch_bounds__(256, 2) k_fgemm_ad(FGemmArgs p) {
  constexpr int NW = 4, WI = 2, WJ = 4, KC = 2, TI = 8, TJ = 4;
  constexpr int STAGE = KC * TJ * 64;   // 16-byte units of B per step
  __shared__ __align__(16) u32x4_t lds[2 * STAGE];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wi = wave, wj = 0;
  const int xcd = blockIdx.x & 7, q = blockIdx.x >> 3;
  const int nTj = p.nJ / TJ;
  const int ti = (q / nTj) * 8 + xcd, tj = q % nTj;   // the column tiles of a row tile share an XCD (one L2)
  if (ti >= p.nI / TI) return;                         // uniform over the workgroup, before any barrier
  const int i0 = ti * TI, j0 = tj * TJ;
  const int nch = p.nkb / KC;
  auto kclamp = [&](int ch) { return (long)(ch < nch ? ch : nch - 1) * KC; };

  const char* asrc[WI];
#pragma unroll
  for (int i = 0; i < WI; ++i) asrc[i] = p.A + (long)(i0 + wi * WI + i) * p.a_si * 1024 + lane * 16;
  const long akst = p.a_sk * 1024;
  // B: pass s copies fragment f = NW s + wave of the step's KC x TJ fragments (kk = f / TJ, jj = f % TJ)
  const char* bsrc[2];
#pragma unroll
  for (int s = 0; s < 2; ++s) {
    const int f = NW * s + wave, kk = f / TJ, jj = f % TJ;
    bsrc[s] = p.B + ((long)(j0 + jj) * p.b_sj + (long)kk * p.b_sk) * 1024 + lane * 16;
  }
  const long bkst = p.b_sk * 1024;

  f32x16_t acc[WI][WJ];
#pragma unroll
  for (int i = 0; i < WI; ++i)
#pragma unroll
    for (int j = 0; j < WJ; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // (the B loads come first: the compiler merges the load counts of this prologue into the loop's own, and fewer
  // loads behind Y here than in the loop would make every iteration wait for nearly all of its loads)
  u32x4_t aR[4][KC][WI], pre[4][2];   // pre[k]: the B fragments of the step whose number is k modulo 4
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const long kk0 = kclamp(k);
#pragma unroll
    for (int s = 0; s < 2; ++s) pre[k][s] = *reinterpret_cast<const u32x4_t*>(bsrc[s] + kk0 * bkst);
  }
#pragma unroll
  for (int st = 0; st < 3; ++st) {
    const long k0 = kclamp(st);
#pragma unroll
    for (int kk = 0; kk < KC; ++kk)
#pragma unroll
      for (int i = 0; i < WI; ++i) aR[st][kk][i] = *reinterpret_cast<const u32x4_t*>(asrc[i] + (k0 + kk) * akst);
  }
  {
    const long k4 = kclamp(4);
#pragma unroll
    for (int s = 0; s < 2; ++s) lds[(NW * s + wave) * 64 + lane] = pre[0][s];
#pragma unroll
    for (int s = 0; s < 2; ++s) pre[0][s] = *reinterpret_cast<const u32x4_t*>(bsrc[s] + k4 * bkst);
  }
  __syncthreads();
  // after the prologue: LDS half 0 = B of step 0, pre[1..3] = B of steps 1..3, pre[0] = B of step 4, aR[0..2] = A of
  // steps 0..2. Loads complete in the order of their issue, so the shortest distance between a load and its use is
  // what counts: A three steps, B four steps (two with only two register sets: every step then waited for loads
  // issued two steps earlier).
  for (int c = 0; c < nch; c += 4) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int half = r & 1;
      const u32x4_t* cur = lds + half * STAGE;
#pragma unroll
      for (int kk = 0; kk < KC; ++kk) {
        bf16x8_t b[WJ];
#pragma unroll
        for (int j = 0; j < WJ; ++j) b[j] = __builtin_bit_cast(bf16x8_t, cur[(kk * TJ + wj * WJ + j) * 64 + lane]);
#pragma unroll
        for (int i = 0; i < WI; ++i)
#pragma unroll
          for (int j = 0; j < WJ; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, aR[r][kk][i]), b[j],
                                                                acc[i][j], 0, 0, 0);
      }
      const long kn = kclamp(c + r + 3);
#pragma unroll
      for (int kk = 0; kk < KC; ++kk)
#pragma unroll
        for (int i = 0; i < WI; ++i)
          aR[(r + 3) & 3][kk][i] = *reinterpret_cast<const u32x4_t*>(asrc[i] + (kn + kk) * akst);
      {
        const long kb5 = kclamp(c + r + 5);
        u32x4_t* nxt = lds + (half ^ 1) * STAGE;
#pragma unroll
        for (int s = 0; s < 2; ++s) nxt[(NW * s + wave) * 64 + lane] = pre[(r + 1) & 3][s];
#pragma unroll
        for (int s = 0; s < 2; ++s) pre[(r + 1) & 3][s] = *reinterpret_cast<const u32x4_t*>(bsrc[s] + kb5 * bkst);
      }
      __syncthreads();
    }
  }
  const int x = lane & 31, g = lane >> 5;
  const long R0 = (long)(i0 + wi * WI) * 32;   // first row of this wavefront's strip of 64 rows
  float xe[SEG ? 32 : 1];                      // SEG: wx . m of the rows (i, v) of this lane, index 16 i + v
  if constexpr (SEG) {
#pragma unroll
    for (int q = 0; q < 32; ++q) xe[q] = 0.f;
  }
#pragma unroll
  for (int j = 0; j < WJ; ++j) {
    const int jb = j0 + wj * WJ + j;
    const int colx = jb * 32 + x;
    float bv = 0.f;
    if (p.bias && colx < p.nbias) bv = p.bias[colx];
    float wxv = 0.f;
    if constexpr (SEG) wxv = colx < p.seg_H ? p.seg_wx[colx] : 0.f;
#pragma unroll
    for (int i = 0; i < WI; ++i) {
      const int ib = i0 + wi * WI + i;
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        uint4 w;
        w.x = pack_bf16x2(acc[i][j][8 * hh + 0] + bv, acc[i][j][8 * hh + 1] + bv);
        w.y = pack_bf16x2(acc[i][j][8 * hh + 2] + bv, acc[i][j][8 * hh + 3] + bv);
        w.z = pack_bf16x2(acc[i][j][8 * hh + 4] + bv, acc[i][j][8 * hh + 5] + bv);
        w.w = pack_bf16x2(acc[i][j][8 * hh + 6] + bv, acc[i][j][8 * hh + 7] + bv);
        *reinterpret_cast<uint4*>(p.T + ((long)(2 * ib + hh) * p.t_ncb + jb) * 1024 + lane * 16) = w;
        if constexpr (SEG) {
          // m = silu of the stored (rounded) z2, as the reverse pass will see it; rows past the last edge give 0
          const unsigned ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
          for (int t = 0; t < 8; ++t) {
            const int v = 8 * hh + t;
            const float z = (t & 1) ? bf_hi(ww[t >> 1]) : bf_lo(ww[t >> 1]);
            const long row = R0 + 32 * i + 8 * (v >> 2) + 4 * g + (v & 3);
            const float m = row < p.seg_E ? silu_f(z) : 0.f;
            acc[i][j][v] = m;
            xe[16 * i + v] = fmaf(wxv, m, xe[16 * i + v]);
          }
        }
      }
    }
  }
  if constexpr (SEG) {
    // x_e: the 32 row sums over the 32 lanes of a half share one butterfly, each exchange halving the values a lane
    // still carries (31 exchanges instead of 160); lane x ends up with the sum of value x = 16 i + v
    {
      float a16[16], a8[8], a4[4], a2[2];
      const bool b4 = x & 16, b3 = x & 8, b2 = x & 4, b1 = x & 2, b0 = x & 1;
#pragma unroll
      for (int q = 0; q < 16; ++q) a16[q] = (b4 ? xe[16 + q] : xe[q]) + __shfl_xor(b4 ? xe[q] : xe[16 + q], 16);
#pragma unroll
      for (int q = 0; q < 8; ++q) a8[q] = (b3 ? a16[8 + q] : a16[q]) + __shfl_xor(b3 ? a16[q] : a16[8 + q], 8);
#pragma unroll
      for (int q = 0; q < 4; ++q) a4[q] = (b2 ? a8[4 + q] : a8[q]) + __shfl_xor(b2 ? a8[q] : a8[4 + q], 4);
#pragma unroll
      for (int q = 0; q < 2; ++q) a2[q] = (b1 ? a4[2 + q] : a4[q]) + __shfl_xor(b1 ? a4[q] : a4[2 + q], 2);
      const float tot = (b0 ? a2[1] : a2[0]) + __shfl_xor(b0 ? a2[0] : a2[1], 1);
      const int i = x >> 4, v = x & 15;
      const long row = R0 + 32 * i + 8 * (v >> 2) + 4 * g + (v & 3);
      if (row < p.seg_E) p.seg_xe[(long)tj * p.seg_xe_stride + row] = tot;
    }
    // sums per destination atom over the strip: the atoms of the strip one after the other (rows are sorted by
    // destination; an atom without edges has an empty range)
    if (R0 < p.seg_E) {
      const long Rend = R0 + 64 < p.seg_E ? R0 + 64 : p.seg_E;
      const int a_first = __builtin_amdgcn_readfirstlane(p.seg_dst[R0]);
      const int a_last = __builtin_amdgcn_readfirstlane(p.seg_dst[Rend - 1]);
      const long strip = R0 >> 6;
      for (int a = a_first; a <= a_last; ++a) {
        const long e0 = __builtin_amdgcn_readfirstlane(p.seg_row_ptr[a]);
        const long e1 = __builtin_amdgcn_readfirstlane(p.seg_row_ptr[a + 1]);
        const int lo = (int)((e0 > R0 ? e0 : R0) - R0), hi = (int)((e1 < R0 + 64 ? e1 : R0 + 64) - R0);
        if (lo >= hi) continue;
        float t[WJ];
#pragma unroll
        for (int j = 0; j < WJ; ++j) t[j] = 0.f;
#pragma unroll
        for (int i = 0; i < WI; ++i)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int rr = 32 * i + 8 * (v >> 2) + (v & 3) + 4 * g;
            const bool in = (unsigned)(rr - lo) < (unsigned)(hi - lo);
#pragma unroll
            for (int j = 0; j < WJ; ++j) t[j] += in ? acc[i][j][v] : 0.f;
          }
#pragma unroll
        for (int j = 0; j < WJ; ++j) t[j] += __shfl_xor(t[j], 32);
        float* dest;
        float scale = 1.f;
        if (e0 < R0) dest = p.seg_first + strip * p.seg_ldp;
        else if (e1 > R0 + 64) dest = p.seg_last + strip * p.seg_ldp;
        else { dest = p.seg_M + (long)a * p.seg_ldm; scale = p.seg_alpha; }
        if (g == 0) {
#pragma unroll
          for (int j = 0; j < WJ; ++j) dest[(j0 + wj * WJ + j) * 32 + x] = scale * t[j];
        }
      }
    }
  }
}

// Second half of the per-atom sums of the forward pass (one wavefront per atom): M of the atoms whose edges span
// several 64-row strips from the strips' partial sums, in strip order; zeros for atoms without edges;
// v'_i = v_i + alpha sum_e x_e rvec_e with x_e the sum of its column tiles' parts (also kept: xe_out[e]).
__global__ void __launch_bounds__(256) k_seg_fwd_fix(int N, int Hp, int ntj, const int32_t* __restrict__ row_ptr,
                                                     const float* __restrict__ pfirst, const float* __restrict__ plast,
                                                     const float* __restrict__ xe_part, long xe_stride,
                                                     const float* __restrict__ rvec, float alpha,
                                                     const float* __restrict__ v_in, float* __restrict__ M,
                                                     float* __restrict__ v_out, float* __restrict__ xe_out) {
  const int lane = threadIdx.x & 63;
  const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (i >= N) return;
  const int e0 = row_ptr[i], e1 = row_ptr[i + 1];
  if (e0 == e1) {
    for (int c = lane; c < Hp; c += 64) M[(long)i * Hp + c] = 0.f;
  } else {
    const int s0 = e0 >> 6, s1 = (e1 - 1) >> 6;
    if (s0 != s1) {
      for (int c = lane; c < Hp; c += 64) {
        float t = plast[(long)s0 * Hp + c];
        for (int s = s0 + 1; s <= s1; ++s) t += pfirst[(long)s * Hp + c];
        M[(long)i * Hp + c] = alpha * t;
      }
    }
  }
  float s[3] = {0.f, 0.f, 0.f};
  for (int e = e0 + lane; e < e1; e += 64) {
    float xv = 0.f;
    for (int t = 0; t < ntj; ++t) xv += xe_part[(long)t * xe_stride + e];
    xe_out[e] = xv;
    s[0] = fmaf(xv, rvec[3 * (long)e], s[0]);
    s[1] = fmaf(xv, rvec[3 * (long)e + 1], s[1]);
    s[2] = fmaf(xv, rvec[3 * (long)e + 2], s[2]);
  }
#pragma unroll
  for (int d = 0; d < 3; ++d) {
    float t = s[d];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) t += __shfl_xor(t, o);
    if (lane == 0) v_out[3 * (long)i + d] = v_in[3 * (long)i + d] + alpha * t;
  }
}

static int32_t launch_fgemm_ad(hipStream_t st, const FGemmArgs& a) {
  HGNN_REQUIRE(a.nI % 8 == 0 && a.nJ % 4 == 0 && a.nkb % 8 == 0 && a.nkb > 0 && !a.grp_ptr && a.nsplit == 1 && a.kper == a.nkb,
               HGNN_ERR_BAD_SHAPE, "fragment GEMM: %d x %d blocks, %d contraction blocks do not tile", a.nI, a.nJ, a.nkb);
  if (a.nI == 0 || a.nJ == 0) return HGNN_OK;
  const long gx = (a.nI / 8 + 7) / 8 * 8 * (long)(a.nJ / 4);
  HGNN_REQUIRE(gx <= 2147483647L, HGNN_ERR_OVERFLOW, "fragment GEMM: grid too large");
  ProfScope ps(a.tag, st);
  if (a.seg_dst) {
    HGNN_REQUIRE(a.seg_row_ptr && a.seg_wx && a.seg_M && a.seg_first && a.seg_last && a.seg_xe && a.seg_E <= (long)a.nI * 32,
                 HGNN_ERR_NULLPTR, "fragment GEMM: incomplete per-atom sum arguments");
    k_fgemm_ad<true><<<dim3((unsigned)gx), 256, 0, st>>>(a);
  } else {
    k_fgemm_ad<false><<<dim3((unsigned)gx), 256, 0, st>>>(a);
  }
  HGNN_LAUNCH_CHECK("k_fgemm_ad");
  return HGNN_OK;
}

// ---------------------------------------------------------------------------------------------
// weights -> B fragments:  fragment (nb, kb) of the destination, lane (g, x), slot u  =  B[16 kb + 8 g + u][32 nb + x]
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_pack_frag(PackFragArgs a) {
  const PackPart pt = a.part[blockIdx.y];
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;   // 16-byte piece of the part: [nb][kb][lane], 8 slots u each
  const int nkb = a.Kp / 16;
  if (idx >= (long)a.Kp * a.Np / 8) return;
  const int lane = idx & 63;
  const int f = (int)(idx >> 6);
  const int kb = f % nkb, nb = f / nkb;
  const int k0 = kb * 16 + (lane >> 5) * 8, n = nb * 32 + (lane & 31);
  const float* src = a.src + blockIdx.z * a.src_grp_stride + pt.src_off + (long)n * pt.sn;
  float v[8];
#pragma unroll
  for (int u = 0; u < 8; ++u) v[u] = (k0 + u < a.K && n < a.Nn) ? src[(long)(k0 + u) * pt.sk] : 0.f;
  uint4 w;
  w.x = pack_bf16x2(v[0], v[1]); w.y = pack_bf16x2(v[2], v[3]); w.z = pack_bf16x2(v[4], v[5]); w.w = pack_bf16x2(v[6], v[7]);
  *reinterpret_cast<uint4*>(a.dst + blockIdx.z * a.dst_grp_stride + pt.dst_off +
                            (((long)(pt.nb0 + nb) * pt.nkb_total + pt.kb0 + kb) * 64 + lane) * 8) = w;
}

int32_t launch_pack_frag(hipStream_t st, const PackFragArgs& a) {
  ProfScope ps(PT_PACK, st);
  k_pack_frag<<<dim3((unsigned)(((long)a.Kp * a.Np / 8 + 255) / 256), a.nparts, a.groups), 256, 0, st>>>(a);
  HGNN_LAUNCH_CHECK("k_pack_frag");
  return HGNN_OK;
}

// ---------------------------------------------------------------------------------------------
// row-major fp32 -> fragments.  mode 0: x, 1: silu(x), 2: x * silu'(z)
// ---------------------------------------------------------------------------------------------
// One workgroup per tile of 32 rows x 128 columns, in the two mappings of the element-wise edge kernels below:
// compute mapping thread (q, x) = the 8 rows of one row set x the column pair 128 slab + 2 x, + 1 (T fragments leave
// in this mapping, 32 bytes per lane), R fragments through an LDS copy of the tile (one whole fragment per store
// instruction). VEC2: the column pair is read with one 8-byte load (the launcher checks the alignment).
template <bool VEC2>
__global__ void __launch_bounds__(256) k_to_frag(ToFragArgs a) {
  __shared__ __align__(16) unsigned short tile[32 * 136];
  const int tid = threadIdx.x, x = tid & 63;
  const int q = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int slab = blockIdx.x, rb = blockIdx.y;
  int pos0 = 0, pad0 = 0, n = a.M, npad = a.Mp;
  if (a.grp_ptr) {
    group_range(a.grp_ptr, blockIdx.z, pos0, n, pad0);
    npad = (n + 255) / 256 * 256;
  }
  if (rb * 32 >= npad) return;   // uniform over the workgroup, before any barrier
  const int hh = q >> 1, g = q & 1;
  const int c = slab * 128 + 2 * x;
  unsigned packed[8];   // [u]: columns c (low half), c + 1
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    const int r = tset_row(2 * rb + hh, g, u);   // row inside the group
    const long sr = r < n ? (a.row_idx ? a.row_idx[pos0 + r] : pad0 + r) : 0;
    float x0 = 0.f, x1 = 0.f, z0 = 0.f, z1 = 0.f;
    if (r < n && c < a.ncol) {
      // both columns are read where the row pitch covers them; a column past ncol is zeroed below
      if (VEC2 && c + 2 <= a.ldx) {
        const float2 xx = *reinterpret_cast<const float2*>(a.X + sr * a.ldx + c);
        x0 = xx.x; x1 = xx.y;
        if (a.mode == 2) {
          const float2 zz = *reinterpret_cast<const float2*>(a.Z + sr * a.ldz + c);
          z0 = zz.x; z1 = zz.y;
        }
      } else {
        x0 = a.X[sr * a.ldx + c];
        if (a.mode == 2) z0 = a.Z[sr * a.ldz + c];
        if (c + 1 < a.ncol) {
          x1 = a.X[sr * a.ldx + c + 1];
          if (a.mode == 2) z1 = a.Z[sr * a.ldz + c + 1];
        }
      }
    }
    if (a.mode == 1) { x0 = silu_f(x0); x1 = silu_f(x1); }
    else if (a.mode == 2) { x0 *= dsilu_f(z0); x1 *= dsilu_f(z1); }
    if (c + 1 >= a.ncol) x1 = 0.f;
    if (c >= a.ncol) x0 = 0.f;
    packed[u] = pack_bf16x2(x0, x1);
  }
  if (a.T) {   // destination rows are the padded ones
    const long rb16 = pad0 / 16 + 2 * rb + hh;
    const long tfrag = ((rb16 * a.t_ncb + a.t_cb0 + (c >> 5)) * 64 + g * 32 + (c & 31)) * 16;
    u32x4_t t0, t1;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      t0[k] = (packed[2 * k] & 0xffffu) | (packed[2 * k + 1] << 16);
      t1[k] = (packed[2 * k] >> 16) | (packed[2 * k + 1] & 0xffff0000u);
    }
    *reinterpret_cast<u32x4_t*>(a.T + tfrag) = t0;
    *reinterpret_cast<u32x4_t*>(a.T + tfrag + 16) = t1;
  }
  if (a.R) {
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int lr = 16 * hh + 8 * (u >> 2) + 4 * g + (u & 3);
      *reinterpret_cast<unsigned*>(&tile[lr * 136 + 2 * x]) = packed[u];
    }
    __syncthreads();
    const int lr = x & 31, g2 = x >> 5;
#pragma unroll
    for (int kb2 = 0; kb2 < 2; ++kb2) {
      const int kbl = 2 * q + kb2;   // contraction block inside the tile
      const u32x4_t w = *reinterpret_cast<const u32x4_t*>(&tile[lr * 136 + kbl * 16 + g2 * 8]);
      const long frag = (long)(pad0 / 32 + rb) * a.r_nkb + a.r_kb0 + 8 * slab + kbl;
      *reinterpret_cast<u32x4_t*>(a.R + (frag * 64 + x) * 16) = w;
    }
  }
}

int32_t launch_to_frag(hipStream_t st, const ToFragArgs& a) {
  HGNN_REQUIRE(a.Mp % 256 == 0 && a.Cp % 128 == 0, HGNN_ERR_BAD_SHAPE, "to_frag: padded extents do not tile");
  if (a.Mp == 0 || a.Cp == 0) return HGNN_OK;
  HGNN_REQUIRE(a.Mp / 32 <= 65535, HGNN_ERR_OVERFLOW, "to_frag: too many rows");
  ProfScope ps(PT_TO_FRAG, st);
  const dim3 grid(a.Cp / 128, a.Mp / 32, a.grp_ptr ? a.S : 1);
  const auto even = [](const float* p, long ld) { return p == nullptr || (reinterpret_cast<uintptr_t>(p) % 8 == 0 && ld % 2 == 0); };
  if (even(a.X, a.ldx) && (a.mode != 2 || even(a.Z, a.ldz))) k_to_frag<true><<<grid, 256, 0, st>>>(a);
  else k_to_frag<false><<<grid, 256, 0, st>>>(a);
  HGNN_LAUNCH_CHECK("k_to_frag");
  return HGNN_OK;
}

// ---------------------------------------------------------------------------------------------
// column sums of small row-major tensors and ordered reduction of per-block partial rows
// ---------------------------------------------------------------------------------------------
// dest[c] = sum over s < nsplit of partial[s * stride + c], c < ncol   (blockIdx.y: group). Fixed order: 16 row
// phases each sum a contiguous run of partials in ascending order, then the phases are added in ascending order.
__global__ void __launch_bounds__(1024) k_reduce_cols(const float* __restrict__ partial, int nsplit, long stride,
                                                      int ncol, float* __restrict__ dest, long partial_grp_stride,
                                                      long dest_grp_stride) {
  __shared__ float sh[16][64];
  const int cl = threadIdx.x & 63, ph = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + cl;
  const int per = (nsplit + 15) / 16;
  const int k0 = ph * per;
  const int k1 = k0 + per < nsplit ? k0 + per : nsplit;
  float s = 0.f;
  if (c < ncol) {
    const float* p = partial + blockIdx.y * partial_grp_stride + c;
    int k = k0;
    for (; k + 8 <= k1; k += 8) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = p[(long)(k + u) * stride];
#pragma unroll
      for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (; k < k1; ++k) s += p[(long)k * stride];
  }
  sh[ph][cl] = s;
  __syncthreads();
  if (ph == 0 && c < ncol) {
    float t = sh[0][cl];
#pragma unroll
    for (int q = 1; q < 16; ++q) t += sh[q][cl];
    dest[blockIdx.y * dest_grp_stride + c] = t;
  }
}
static int32_t launch_reduce_cols(hipStream_t st, const float* partial, int nsplit, long stride, int ncol, float* dest,
                                  int groups = 1, long partial_grp_stride = 0, long dest_grp_stride = 0) {
  k_reduce_cols<<<dim3((ncol + 63) / 64, groups), 1024, 0, st>>>(partial, nsplit, stride, ncol, dest, partial_grp_stride,
                                                                 dest_grp_stride);
  HGNN_LAUNCH_CHECK("k_reduce_cols");
  return HGNN_OK;
}

constexpr int CS_ROWS = 16;   // rows per partial of k_colsum_rows
// partial[group][split][c] = sum over the split's rows of w * f(X[r][c])   (blockIdx.y: split, blockIdx.z: group)
__global__ void __launch_bounds__(256) k_colsum_rows(ColsumRowsArgs a, int nsplit) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= a.ncol) return;
  int pos0 = 0, pad0 = 0, n = a.M;
  if (a.grp_ptr) group_range(a.grp_ptr, blockIdx.z, pos0, n, pad0);
  const int r0 = blockIdx.y * CS_ROWS;
  float s = 0.f;
  if (r0 < n) {   // uniform
    // all rows of the partial are asked for before the first is used (rows past the end: the last one again, left
    // out of the sum); summed in row order
    long sr[CS_ROWS];
    float xv[CS_ROWS], zv[CS_ROWS], wv[CS_ROWS];
#pragma unroll
    for (int u = 0; u < CS_ROWS; ++u) {
      const int r = r0 + u < n ? r0 + u : n - 1;
      sr[u] = a.row_idx ? a.row_idx[pos0 + r] : pad0 + r;
    }
#pragma unroll
    for (int u = 0; u < CS_ROWS; ++u) {
      xv[u] = a.X[sr[u] * a.ldx + c];
      zv[u] = a.mode == 2 ? a.Z[sr[u] * a.ldz + c] : 0.f;
      wv[u] = a.w ? a.w[sr[u]] : 1.f;
    }
#pragma unroll
    for (int u = 0; u < CS_ROWS; ++u) {
      float v = xv[u];
      if (a.mode == 1) v = silu_f(v);
      else if (a.mode == 2) v *= dsilu_f(zv[u]);
      if (a.w) v *= wv[u];
      if (r0 + u < n) s += v;
    }
  }
  a.partial[((long)blockIdx.z * nsplit + blockIdx.y) * a.ncol + c] = s;
}
size_t colsum_rows_partial_floats(int M, int ncol, int S) {
  return (size_t)((M + CS_ROWS - 1) / CS_ROWS + 1) * ncol * (S < 1 ? 1 : S);
}
int32_t launch_colsum_rows(hipStream_t st, const ColsumRowsArgs& a) {
  ProfScope ps(PT_COLSUM, st);
  const int ns = (a.M + CS_ROWS - 1) / CS_ROWS;
  const int groups = a.grp_ptr ? a.S : 1;
  if (ns > 0) {
    k_colsum_rows<<<dim3((a.ncol + 255) / 256, ns, groups), 256, 0, st>>>(a, ns);
    HGNN_LAUNCH_CHECK("k_colsum_rows");
  }
  return launch_reduce_cols(st, a.partial, ns, a.ncol, a.ncol, a.dest, groups, (long)ns * a.ncol, a.dest_grp_stride);
}

// dest[group * dest_grp_stride + pa * strideA + pb * strideB + r1 * HB + r2] = sum over splits (ascending) of
// partial[group][s][k1][k2], k1 = pa * HpA + r1, k2 = pb * HpB + r2; padding (r1 >= HA or r2 >= HB) is dropped
__global__ void __launch_bounds__(256) k_reduce_wgrad(const float* __restrict__ partial, int nsplit, long split_stride,
                                                      int K1p, int K2p, int HpA, int HA, int HpB, int HB,
                                                      float* __restrict__ dest, long strideA, long strideB,
                                                      long dest_grp_stride) {
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long)K1p * K2p) return;
  const int k1 = (int)(idx / K2p), k2 = (int)(idx % K2p);
  const int pa = k1 / HpA, r1 = k1 % HpA, pb = k2 / HpB, r2 = k2 % HpB;
  if (r1 >= HA || r2 >= HB) return;
  const float* p = partial + (long)blockIdx.y * nsplit * split_stride;
  float s = 0.f;
  for (int k = 0; k < nsplit; ++k) s += p[(long)k * split_stride + idx];
  dest[blockIdx.y * dest_grp_stride + pa * strideA + pb * strideB + (long)r1 * HB + r2] = s;
}

// ---------------------------------------------------------------------------------------------
// element-wise edge kernels. A workgroup walks tiles of 32 edges (one row block) x 128 columns:
//   compute mapping, thread (q, x) = (tid >> 6, tid & 63): the 8 edges of row set (row group 2 rb32 + (q >> 1), lane
//     half q & 1) in the column pair 128 slab + 2 x, + 1. T fragments are loaded and stored in this mapping (32 bytes
//     per lane, a wavefront moves four contiguous half fragments); a gather fetches both columns with one 4-byte load
//     (the vector memory pipe takes one address per lane whatever the width: 2-byte gathers made these kernels
//     address-bound).
//   R mapping (through an LDS copy of the tile), wavefront q: contraction blocks 8 slab + 2 q, + 1, lane x of the
//     fragment (row x & 31, 8 columns from 8 (x >> 5)): one whole 1 KiB fragment per store instruction.
// Every global store instruction writes whole cache lines.
// ---------------------------------------------------------------------------------------------
struct EdgeElemArgs {
  int64_t E = 0;
  int nrb = 0;             // 32-row blocks covered (padded rows / 32)
  int H = 0, Hp = 0;
  const int32_t* dst = nullptr;
  const int32_t* col = nullptr;
  const float* attr = nullptr;          // [E, k] edge attributes (k = 1: the squared distance d2)
  int k = 1;
  const unsigned short* PQ = nullptr;   // [N, 2 Hp] bf16 row-major: P | Q
  const float* w1d = nullptr;           // [k, H]: the rows of W1 that act on the attributes
  char* a1_R = nullptr;
  char* a1_T = nullptr;
  // reverse
  const char* z2_T = nullptr;
  const unsigned short* gM = nullptr;   // bf16 row-major g_M, row pitch ldgM elements
  long ldgM = 0;
  const float* cvec = nullptr;
  const float* wx = nullptr;            // [H]
  float alpha = 1.f;
  char* gz2_R = nullptr;
  char* gz2_T = nullptr;
  const char* ga1_T = nullptr;          // g_a1
  unsigned short* gz1_rm = nullptr;     // g_z1, bf16 row-major [rows, Hp]: what the two per-atom sums read
  float* colpart = nullptr;             // [gridDim.y][2 (g_z2) or 1 + k (g_z1)][Hp] column-sum partials
};

__device__ __forceinline__ void unpack8(const uint4 w, float (&f)[8]) {
  f[0] = bf_lo(w.x); f[1] = bf_hi(w.x); f[2] = bf_lo(w.y); f[3] = bf_hi(w.y);
  f[4] = bf_lo(w.z); f[5] = bf_hi(w.z); f[6] = bf_lo(w.w); f[7] = bf_hi(w.w);
}
__device__ __forceinline__ uint4 pack8(const float (&f)[8]) {
  uint4 w;
  w.x = pack_bf16x2(f[0], f[1]); w.y = pack_bf16x2(f[2], f[3]);
  w.z = pack_bf16x2(f[4], f[5]); w.w = pack_bf16x2(f[6], f[7]);
  return w;
}

enum { EE_A1 = 0, EE_GZ2 = 1, EE_GZ1 = 2 };
constexpr int EE_PITCH = 136;   // LDS tile row pitch in bf16 elements (128 + 8: 16-byte reads of a column of rows spread over the banks)

// EE_A1:  a1 = silu(z1), z1 = P[dst] + Q[col] + sum_j attr_j w1d_j               -> R and T
// EE_GZ2: g_z2 = (alpha g_M[dst] + c_e wx) silu'(z2)                            -> R and T; sums: g_b2 = sum g_z2, g_wx = sum c_e silu(z2)
// EE_GZ1: g_z1 = g_a1 silu'(z1), z1 recomputed from the gathers                 -> row-major; sums: g_b1 = sum g_z1, g_w1d_j = sum attr_j g_z1
// KMAX: most edge attributes the instance handles (1: the squared distance alone; 16: p.k of them, p.k <= 16)
template <int MODE, int KMAX>
__global__ void __launch_bounds__(256) k_edge_elem(EdgeElemArgs p) {
  constexpr int NV = MODE == EE_GZ1 ? 1 + KMAX : 2;   // column sums kept per column
  __shared__ __align__(16) unsigned short tile[32 * EE_PITCH];
  __shared__ float csum[4][NV][128];
  // the attributes of the tile's 32 rows (several attributes: every lane of a wavefront needs the same values, so
  // they are fetched once per tile and read back as LDS broadcasts)
  __shared__ __align__(16) float attr_s[KMAX > 1 && MODE != EE_GZ2 ? 32 * KMAX : 4];
  const int tid = threadIdx.x, x = tid & 63;
  const int q = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int slab = blockIdx.x;
  const int c = slab * 128 + 2 * x;       // this thread's columns: c, c + 1
  const int ncb = p.Hp >> 5, nkb = p.Hp >> 4;
  const int hh = q >> 1, g = q & 1;
  // wx of this thread's two columns (g_z2), or the rows of W1 that act on the edge attributes
  float w0[KMAX], w1[KMAX];
#pragma unroll
  for (int j = 0; j < KMAX; ++j) {
    const float* wv = MODE == EE_GZ2 ? p.wx : p.w1d + (long)j * p.H;
    const bool on = MODE == EE_GZ2 ? j == 0 : j < p.k;
    w0[j] = on && c < p.H ? wv[c] : 0.f;
    w1[j] = on && c + 1 < p.H ? wv[c + 1] : 0.f;
  }
  const long lastrow = p.E > 0 ? p.E - 1 : 0;
  char* Tdst = MODE == EE_A1 ? p.a1_T : p.gz2_T;
  float s00 = 0.f, s01 = 0.f;          // column sums of the result
  float s10[KMAX], s11[KMAX];          // weighted column sums
#pragma unroll
  for (int j = 0; j < KMAX; ++j) { s10[j] = 0.f; s11[j] = 0.f; }
  for (int rb = blockIdx.y; rb < p.nrb; rb += gridDim.y) {
    const int rb16 = 2 * rb + hh;
    if (KMAX > 1 && MODE != EE_GZ2) {
      // (the previous tile's arithmetic lies before its two barriers, so the buffer is free)
      for (int t = tid; t < 32 * KMAX; t += 256) {
        const long r = (long)rb * 32 + t / KMAX;
        const int j = t % KMAX;
        attr_s[t] = r < p.E && j < p.k ? p.attr[r * p.k + j] : 0.f;
      }
      __syncthreads();
    }
    // the two columns are neighbouring 16-byte slots of one half fragment
    const long tfrag = ((long)rb16 * ncb + (c >> 5)) * 1024 + (g * 32 + (c & 31)) * 16;
    u32x4_t in0, in1;
    if (MODE == EE_GZ2) {
      in0 = *reinterpret_cast<const u32x4_t*>(p.z2_T + tfrag);
      in1 = *reinterpret_cast<const u32x4_t*>(p.z2_T + tfrag + 16);
    }
    if (MODE == EE_GZ1) {
      in0 = *reinterpret_cast<const u32x4_t*>(p.ga1_T + tfrag);
      in1 = *reinterpret_cast<const u32x4_t*>(p.ga1_T + tfrag + 16);
    }
    unsigned ga[8], gb[8];
    float sc[8];
    bool ok[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const long r = tset_row(rb16, g, u);     // the same for all lanes of the wavefront
      ok[u] = r < p.E;
      const long rr = ok[u] ? r : lastrow;
      const long di = p.dst[rr];
      if (MODE == EE_GZ2) {
        sc[u] = p.cvec[rr];
        ga[u] = *reinterpret_cast<const unsigned*>(p.gM + di * p.ldgM + c);
      } else {
        const long ci = p.col[rr];
        if (KMAX == 1) sc[u] = p.attr[rr];
        ga[u] = *reinterpret_cast<const unsigned*>(p.PQ + di * 2 * p.Hp + c);
        gb[u] = *reinterpret_cast<const unsigned*>(p.PQ + ci * 2 * p.Hp + p.Hp + c);
      }
    }
    float o0[8], o1[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const unsigned i0w = MODE == EE_A1 ? 0u : in0[u >> 1], i1w = MODE == EE_A1 ? 0u : in1[u >> 1];
      const float x0 = (u & 1) ? bf_hi(i0w) : bf_lo(i0w), x1 = (u & 1) ? bf_hi(i1w) : bf_lo(i1w);
      if (MODE == EE_GZ2) {
        float y0, d0, y1, d1;
        silu_both(x0, y0, d0);
        silu_both(x1, y1, d1);
        const float gz0 = ok[u] ? fmaf(sc[u], w0[0], p.alpha * bf_lo(ga[u])) * d0 : 0.f;
        const float gz1 = ok[u] ? fmaf(sc[u], w1[0], p.alpha * bf_hi(ga[u])) * d1 : 0.f;
        s00 += gz0; s01 += gz1;
        s10[0] += ok[u] ? sc[u] * y0 : 0.f;
        s11[0] += ok[u] ? sc[u] * y1 : 0.f;
        o0[u] = gz0; o1[u] = gz1;
      } else {
        // the attributes of the row (the same for all lanes of the wavefront)
        float at[KMAX];
        if (KMAX == 1) {
          at[0] = sc[u];
        } else {
          const int lr = 16 * hh + 8 * (u >> 2) + 4 * g + (u & 3);   // row inside the tile
#pragma unroll
          for (int j = 0; j < KMAX; ++j) at[j] = attr_s[lr * KMAX + j];
        }
        float z0 = bf_lo(ga[u]) + bf_lo(gb[u]), z1 = bf_hi(ga[u]) + bf_hi(gb[u]);
#pragma unroll
        for (int j = 0; j < KMAX; ++j) {
          z0 = fmaf(at[j], w0[j], z0);
          z1 = fmaf(at[j], w1[j], z1);
        }
        if (MODE == EE_A1) {
          o0[u] = ok[u] ? silu_f(z0) : 0.f;
          o1[u] = ok[u] ? silu_f(z1) : 0.f;
        } else {
          const float gz0 = ok[u] ? x0 * dsilu_f(z0) : 0.f;
          const float gz1 = ok[u] ? x1 * dsilu_f(z1) : 0.f;
          s00 += gz0; s01 += gz1;
#pragma unroll
          for (int j = 0; j < KMAX; ++j) {
            s10[j] = fmaf(at[j], gz0, s10[j]);
            s11[j] = fmaf(at[j], gz1, s11[j]);
          }
          o0[u] = gz0; o1[u] = gz1;
        }
      }
      // (several attributes: keep the rows apart, or the scheduler fetches the attributes of all eight rows first
      // and the kernel runs out of registers)
      if (KMAX > 1) __builtin_amdgcn_sched_barrier(0);
    }
    if (MODE != EE_GZ1) {   // g_z1 is only read row by row: it goes out row-major below
      u32x4_t t0, t1;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        t0[k] = pack_bf16x2(o0[2 * k], o0[2 * k + 1]);
        t1[k] = pack_bf16x2(o1[2 * k], o1[2 * k + 1]);
      }
      *reinterpret_cast<u32x4_t*>(Tdst + tfrag) = t0;
      *reinterpret_cast<u32x4_t*>(Tdst + tfrag + 16) = t1;
    }
    // the tile in row-major order for the second mapping (rows of this row set: 16 hh + 8 (u >> 2) + 4 g + (u & 3))
    __syncthreads();   // the previous tile has been read
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int lr = 16 * hh + 8 * (u >> 2) + 4 * g + (u & 3);
      *reinterpret_cast<unsigned*>(&tile[lr * EE_PITCH + 2 * x]) = pack_bf16x2(o0[u], o1[u]);
    }
    __syncthreads();
    if (MODE == EE_GZ1) {
      // row-major copy: 16 pieces of 16 bytes per tile row; thread -> row tid >> 4 (+ 16), piece tid & 15
#pragma unroll
      for (int hrow = 0; hrow < 2; ++hrow) {
        const int lr = (tid >> 4) + 16 * hrow, pc = tid & 15;
        const u32x4_t w = *reinterpret_cast<const u32x4_t*>(&tile[lr * EE_PITCH + pc * 8]);
        *reinterpret_cast<u32x4_t*>(p.gz1_rm + ((long)rb * 32 + lr) * p.Hp + slab * 128 + pc * 8) = w;
      }
    } else {
      const int lr = x & 31, g2 = x >> 5;
      char* Rdst = MODE == EE_A1 ? p.a1_R : p.gz2_R;
#pragma unroll
      for (int kb2 = 0; kb2 < 2; ++kb2) {
        const int kbl = 2 * q + kb2;   // contraction block inside the tile
        const u32x4_t w = *reinterpret_cast<const u32x4_t*>(&tile[lr * EE_PITCH + kbl * 16 + g2 * 8]);
        *reinterpret_cast<u32x4_t*>(Rdst + (((long)rb * nkb + 8 * slab + kbl) * 64 + x) * 16) = w;
      }
    }
  }
  if (MODE != EE_A1) {
    // column sums of the workgroup: the four row sets are added in order
    csum[q][0][2 * x] = s00; csum[q][0][2 * x + 1] = s01;
#pragma unroll
    for (int j = 0; j < NV - 1; ++j) { csum[q][1 + j][2 * x] = s10[j]; csum[q][1 + j][2 * x + 1] = s11[j]; }
    __syncthreads();
    const int nv = MODE == EE_GZ2 ? 2 : 1 + p.k;
    if (tid < 128) {
      float* o = p.colpart + (long)blockIdx.y * nv * p.Hp + slab * 128 + tid;
#pragma unroll
      for (int j = 0; j < NV; ++j)
        if (j < nv) o[(long)j * p.Hp] = ((csum[0][j][tid] + csum[1][j][tid]) + csum[2][j][tid]) + csum[3][j][tid];
    }
  }
}

constexpr int ELEM_MAX_BLOCKS = 512;   // row-block phases (= column-sum partials) of the element-wise edge kernels
static dim3 elem_grid(int nrb, int Hp) {
  return dim3(Hp / 128, nrb < 1 ? 1 : (nrb < ELEM_MAX_BLOCKS ? nrb : ELEM_MAX_BLOCKS));
}

// out[i][c] = sum over k in ptr[i] .. ptr[i+1] of X[perm[k]][c] (perm == null: X[k][c]), X bf16 row-major with pitch
// Hp (one wavefront per atom, 16-byte pieces of a row per lane, two rows in flight)
__global__ void __launch_bounds__(256) k_segsum_rows(int N, int Hp, const int32_t* __restrict__ ptr,
                                                     const int32_t* __restrict__ perm, const unsigned short* __restrict__ X,
                                                     float* __restrict__ out, long ldo) {
  const int lane = threadIdx.x & 63;
  const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (i >= N) return;
  const int e0 = ptr[i], e1 = ptr[i + 1];
  const int nch = Hp >> 3;                 // 16-byte pieces per row (at most 128)
  const bool two = lane + 64 < nch;
  float a0[8] = {}, a1[8] = {};
  const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
  int k = e0;
  for (; k + 2 <= e1; k += 2) {
    const unsigned short* r0 = X + (long)(perm ? perm[k] : k) * Hp;
    const unsigned short* r1 = X + (long)(perm ? perm[k + 1] : k + 1) * Hp;
    const uint4 w00 = *reinterpret_cast<const uint4*>(r0 + lane * 8);
    const uint4 w10 = *reinterpret_cast<const uint4*>(r1 + lane * 8);
    const uint4 w01 = two ? *reinterpret_cast<const uint4*>(r0 + (lane + 64) * 8) : zero;
    const uint4 w11 = two ? *reinterpret_cast<const uint4*>(r1 + (lane + 64) * 8) : zero;
    float f[8];
    unpack8(w00, f);
#pragma unroll
    for (int u = 0; u < 8; ++u) a0[u] += f[u];
    unpack8(w10, f);
#pragma unroll
    for (int u = 0; u < 8; ++u) a0[u] += f[u];
    unpack8(w01, f);
#pragma unroll
    for (int u = 0; u < 8; ++u) a1[u] += f[u];
    unpack8(w11, f);
#pragma unroll
    for (int u = 0; u < 8; ++u) a1[u] += f[u];
  }
  if (k < e1) {
    const unsigned short* r0 = X + (long)(perm ? perm[k] : k) * Hp;
    float f[8];
    unpack8(*reinterpret_cast<const uint4*>(r0 + lane * 8), f);
#pragma unroll
    for (int u = 0; u < 8; ++u) a0[u] += f[u];
    unpack8(two ? *reinterpret_cast<const uint4*>(r0 + (lane + 64) * 8) : zero, f);
#pragma unroll
    for (int u = 0; u < 8; ++u) a1[u] += f[u];
  }
  float* o = out + (long)i * ldo;
  if (lane < nch) {
    *reinterpret_cast<float4*>(o + lane * 8) = make_float4(a0[0], a0[1], a0[2], a0[3]);
    *reinterpret_cast<float4*>(o + lane * 8 + 4) = make_float4(a0[4], a0[5], a0[6], a0[7]);
  }
  if (two) {
    *reinterpret_cast<float4*>(o + (lane + 64) * 8) = make_float4(a1[0], a1[1], a1[2], a1[3]);
    *reinterpret_cast<float4*>(o + (lane + 64) * 8 + 4) = make_float4(a1[4], a1[5], a1[6], a1[7]);
  }
}

// g_attr[e][j] = sum_c g_z1[e][c] W1d[j][c], j < k <= 32: a product with one 32-column block of output. W1d^T sits in
// LDS as B fragments (built once per workgroup), every wavefront multiplies 32-row blocks of the row-major bf16 g_z1,
// whose 16-byte pieces are A fragments as they stand (lane (g, r): row r, columns 16 kb + 8 g ..).
__global__ void __launch_bounds__(256) k_gattr(int64_t E, int nrb, int H, int Hp, int k,
                                               const unsigned short* __restrict__ gz1, const float* __restrict__ w1d,
                                               float* __restrict__ g_attr) {
  extern __shared__ __align__(16) u32x4_t bfrag[];
  const int lane = threadIdx.x & 63, g = lane >> 5, n = lane & 31;
  const int wave = threadIdx.x >> 6;
  const int nkb = Hp >> 4;
  for (int kb = wave; kb < nkb; kb += 4) {
    u32x4_t wv;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int c0 = 16 * kb + 8 * g + 2 * q;
      const float f0 = (n < k && c0 < H) ? w1d[(long)n * H + c0] : 0.f;
      const float f1 = (n < k && c0 + 1 < H) ? w1d[(long)n * H + c0 + 1] : 0.f;
      wv[q] = pack_bf16x2(f0, f1);
    }
    bfrag[kb * 64 + lane] = wv;
  }
  __syncthreads();
  for (int rb = blockIdx.x * 4 + wave; rb < nrb; rb += gridDim.x * 4) {
    f32x16_t acc;
#pragma unroll
    for (int u = 0; u < 16; ++u) acc[u] = 0.f;
    const char* base = reinterpret_cast<const char*>(gz1) + ((long)rb * 32 + n) * Hp * 2 + g * 16;
    for (int kb0 = 0; kb0 < nkb; kb0 += 8) {   // Hp is a multiple of 128: eight loads in flight
      u32x4_t av[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) av[q] = *reinterpret_cast<const u32x4_t*>(base + (kb0 + q) * 32);
#pragma unroll
      for (int q = 0; q < 8; ++q)
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, av[q]),
                                                      __builtin_bit_cast(bf16x8_t, bfrag[(kb0 + q) * 64 + lane]), acc, 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const long row = (long)rb * 32 + 8 * (u >> 2) + 4 * g + (u & 3);
      if (n < k && row < E) g_attr[row * k + n] = acc[u];
    }
  }
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
struct WideDims {
  int N, H, Hp, Np, ncb, nkb, k;
  int64_t E, Ep;
  WideDims(int N_, int64_t E_, int H_, int k_) : N(N_), H(H_), k(k_), E(E_) {
    Hp = wide_pad_cols(H);
    Np = (int)wide_pad_rows(N);
    Ep = wide_pad_rows(E);
    ncb = Hp / 32;
    nkb = Hp / 16;
  }
  size_t edge_bytes() const { return (size_t)Ep * Hp * 2; }
  size_t node_frag_bytes(int parts) const { return (size_t)Np * Hp * 2 * parts; }
};

struct LayerOffW {
  long W1, b1, W2, b2, wx, W3, b3, W4, b4, total;
  LayerOffW(long H, long k) {   // k edge attributes: W1 has 2H + k rows
    long o = 0;
    W1 = o; o += (2 * H + k) * H;
    b1 = o; o += H;
    W2 = o; o += H * H;
    b2 = o; o += H;
    wx = o; o += H;
    W3 = o; o += 2 * H * H;
    b3 = o; o += H;
    W4 = o; o += H * H;
    b4 = o; o += H;
    total = o;
  }
};

struct WideSaved {
  unsigned short* PQ;   // [Np, 2 Hp] bf16 row-major
  char* a1_R;           // [Ep, Hp]
  char* a1_T;
  char* z2_T;
  float* M;             // [Np, Hp] fp32 row-major
  float* z3;            // [Np, Hp]
  char* hM_T;           // [Np, 2 Hp] T fragments of [h ; M]     (operands of the reverse pass's weight gradients)
  char* a3_T;           // [Np, Hp] T fragments of silu(z3)
  float* xe;            // [Ep] x_e = wx . m_e
  size_t bytes;
};
static WideSaved carve_saved_w(void* p, const WideDims& d) {
  Carver c(p);
  WideSaved s;
  s.PQ = c.take<unsigned short>((size_t)d.Np * 2 * d.Hp);
  s.a1_R = c.take<char>(d.edge_bytes());
  s.a1_T = c.take<char>(d.edge_bytes());
  s.z2_T = c.take<char>(d.edge_bytes());
  s.M = c.take<float>((size_t)d.Np * d.Hp);
  s.z3 = c.take<float>((size_t)d.Np * d.Hp);
  s.hM_T = c.take<char>(d.node_frag_bytes(2));
  s.a3_T = c.take<char>(d.node_frag_bytes(1));
  s.xe = c.take<float>((size_t)d.Ep + 4);
  s.bytes = c.used();
  return s;
}

struct WideWs {
  unsigned short* packed;   // 6 Hp^2 bf16 (the forward or the transposed set)
  char* hM_R;               // [Np, 2 Hp] R fragments of [h ; M]
  char* x_R;                // [Np, 2 Hp] scratch R operand (a3, g_h', g_z3, g_PQ)
  char* gh_T;               // [Np, Hp] T operands of the weight gradients (read on the side stream: each its own)
  char* gz3_T;              // [Np, Hp]
  char* gPQ_T;              // [Np, 2 Hp]
  float* nodeA;             // [Np, Hp] fp32 g_a3
  float* nodeB;             // [Np, 2 Hp] fp32 g_hM
  unsigned short* gM_b;     // [Np, 2 Hp] bf16 row-major copy of g_hM
  float* g_PQ;              // [Np, 2 Hp] fp32
  char* gz2_R;              // [Ep, Hp]
  char* gz2_T;
  char* ga1_T;
  float* seg_first;         // [Ep / 64, Hp] forward: sums of m over the part of a 64-row strip that belongs to an atom
  float* seg_last;          //   that began before the strip / reaches past its end
  float* xe_part;           // [ncb / 4, Ep] x_e per column tile
  float* cvec;              // [E]
  float* colpart;           // ELEM_MAX_BLOCKS x 2 x Hp (g_z2 kernel)
  float* colpart2;          // the same for the g_z1 kernel
  float* cs_partial;        // column sums over atoms
  float* partial;           // split partials of the atom-level weight-gradient products (side stream)
  size_t partial_floats;
  float* partial_e;         // split partials of g_W2 (caller's stream)
  size_t partial_e_floats;
  size_t bytes;
};
static WideWs carve_ws_w(void* p, const WideDims& d) {
  Carver c(p);
  WideWs w;
  w.packed = c.take<unsigned short>((size_t)6 * d.Hp * d.Hp);
  w.hM_R = c.take<char>(d.node_frag_bytes(2));
  w.x_R = c.take<char>(d.node_frag_bytes(2));
  w.gh_T = c.take<char>(d.node_frag_bytes(1));
  w.gz3_T = c.take<char>(d.node_frag_bytes(1));
  w.gPQ_T = c.take<char>(d.node_frag_bytes(2));
  w.nodeA = c.take<float>((size_t)d.Np * d.Hp);
  w.nodeB = c.take<float>((size_t)d.Np * 2 * d.Hp);
  w.gM_b = c.take<unsigned short>((size_t)d.Np * 2 * d.Hp);
  w.g_PQ = c.take<float>((size_t)d.Np * 2 * d.Hp);
  w.gz2_R = c.take<char>(d.edge_bytes());
  w.gz2_T = c.take<char>(d.edge_bytes());
  w.ga1_T = c.take<char>(d.edge_bytes());
  w.cvec = c.take<float>((size_t)d.E + 4);
  w.colpart = c.take<float>((size_t)ELEM_MAX_BLOCKS * 2 * d.Hp);
  w.colpart2 = c.take<float>((size_t)ELEM_MAX_BLOCKS * (1 + d.k) * d.Hp);
  w.cs_partial = c.take<float>(colsum_rows_partial_floats(d.N, d.Hp, 1));
  w.partial_floats = (size_t)24 * 2 * d.Hp * d.Hp;
  w.partial = c.take<float>(w.partial_floats);
  w.partial_e_floats = (size_t)(d.Hp <= 512 ? 96 : 24) * d.Hp * d.Hp;   // narrow outputs need more splits to fill the chip
  w.partial_e = c.take<float>(w.partial_e_floats);
  w.seg_first = c.take<float>((size_t)(d.Ep / 64) * d.Hp);
  w.seg_last = c.take<float>((size_t)(d.Ep / 64) * d.Hp);
  w.xe_part = c.take<float>((size_t)(d.ncb / 4) * d.Ep);
  w.bytes = c.used();
  return w;
}

void wide_layer_sizes(int N, int64_t E, int H, int k, size_t* ws_bytes, size_t* saved_bytes) {
  const WideDims d(N, E, H, k);
  *ws_bytes = carve_ws_w(nullptr, d).bytes;
  *saved_bytes = carve_saved_w(nullptr, d).bytes;
}

// C = A x W over rows (R fragments of A with a_nkb contraction blocks, packed W with nJ column blocks)
static FGemmArgs nn_args(const char* A_R, int a_nkb, int nI, const unsigned short* Wp, int nJ, int tag) {
  FGemmArgs g;
  g.A = A_R; g.a_si = a_nkb; g.a_sk = 1;
  g.B = reinterpret_cast<const char*>(Wp); g.b_sj = a_nkb; g.b_sk = 1;
  g.nI = nI; g.nJ = nJ; g.nkb = a_nkb; g.kper = a_nkb; g.nsplit = 1;
  g.tag = tag;
  return g;
}

constexpr int WIDE_MAX_SPLITS = 256;   // (the partial buffers hold 24 splits of the widest outputs, more of narrow ones)
int32_t launch_fwgrad(hipStream_t st, const FWgradArgs& a) {
  FGemmArgs g;
  g.A = a.A_T + (long)a.a_cb0 * 1024; g.a_si = 1; g.a_sk = a.a_ncb;
  g.B = a.B_T + (long)a.b_cb0 * 1024; g.b_sj = 1; g.b_sk = a.b_ncb;
  g.nI = a.nI; g.nJ = a.nJ;
  g.nkb = (int)(a.rows / 16);
  g.grp_ptr = a.grp_ptr; g.S = a.S;
  const int groups = a.grp_ptr ? a.S : 1;
  // Long contractions over many rows (the per-edge gradient) take 256 x 128 tiles, which load a quarter fewer operand
  // bytes per flop (a last row tile may be half empty); everything else 128 x 128 tiles.
  // Enough splits for about three (two) workgroups per CU, as many as the partial buffer holds.
  long cap = (long)(a.partial_floats / ((size_t)a.nI * 32 * a.nJ * 32 * groups));
  if (cap > WIDE_MAX_SPLITS) cap = WIDE_MAX_SPLITS;
  const long big_tiles = (long)((a.nI + 7) / 8) * (a.nJ / 4);
  // (atom-level gradients measured the same either way; narrow outputs have too few large tiles to fill the chip)
  const bool big = !a.grp_ptr && a.nI >= 8 && a.rows >= 65536 && big_tiles * cap >= 2L * num_cus();
  const long tiles = big ? big_tiles : (long)(a.nI / 4) * (a.nJ / 4) * groups;
  long want = ((big ? 2L : 3L) * num_cus() + tiles - 1) / tiles;
  if (want > cap) want = cap;
  want = want / 8 * 8;   // a multiple of 8: one XCD per residue (see k_fgemm)
  if (want < 8) want = 8;
  HGNN_REQUIRE(cap >= 8, HGNN_ERR_WORKSPACE_TOO_SMALL, "weight-gradient partials do not fit the workspace");
  int kper = (int)((g.nkb + want - 1) / want);
  kper = (kper + 3) / 4 * 4;   // whole pairs of steps
  if (kper < 4) kper = 4;
  g.kper = kper;
  g.nsplit = (int)want;   // splits past the end of the rows write zeros
  g.P = a.partial; g.ldp = (long)a.nJ * 32; g.split_stride = (long)a.nI * 32 * a.nJ * 32;
  g.tag = a.tag;
  HGNN_REQUIRE((size_t)g.nsplit * groups * g.split_stride <= a.partial_floats, HGNN_ERR_WORKSPACE_TOO_SMALL,
               "weight-gradient partials do not fit the workspace");
  if (big) HGNN_TRY((launch_fgemm_t<4, 2, EPI_PART>(st, g)));
  else HGNN_TRY((launch_fgemm_t<2, 2, EPI_PART>(st, g)));
  ProfScope ps(a.tag, st);
  const long n = g.split_stride;
  k_reduce_wgrad<<<dim3((unsigned)((n + 255) / 256), groups), 256, 0, st>>>(
      a.partial, g.nsplit, g.split_stride, a.nI * 32, a.nJ * 32, a.HpA, a.HA, a.HpB, a.HB, a.dest, a.strideA, a.strideB,
      a.dest_grp_stride);
  HGNN_LAUNCH_CHECK("k_reduce_wgrad");
  return HGNN_OK;
}
// widest access (floats) that the fp32 output and the residuals of a row product allow
static int row_io_width(const FGemmArgs& a) {
  const auto fits = [&](int vec) {
    const auto ok = [&](const float* p, long ld) {
      return p == nullptr || (reinterpret_cast<uintptr_t>(p) % (4 * vec) == 0 && ld % vec == 0);
    };
    return ok(a.Cf, a.ldc) && ok(a.r1, a.ld1) && ok(a.r2, a.ld2);
  };
  return fits(4) ? 4 : (fits(2) ? 2 : 1);
}
int32_t launch_fgemm_rows(hipStream_t st, const FGemmArgs& a0) {
  FGemmArgs a = a0;
  a.vec = row_io_width(a);
  // few rows (atoms, graphs): 128 x 128 tiles give the launch enough workgroups to cover the chip
  const long big_tiles = (long)((a.nI + 7) / 8) * (a.nJ / 4) * (a.grp_ptr ? a.S : 1);
  if (big_tiles < 4L * num_cus()) return launch_fgemm_t<2, 2, EPI_ROW>(st, a);
  return launch_fgemm_t<4, 2, EPI_ROW>(st, a);
}
int32_t launch_fgemm_rows_T(hipStream_t st, const FGemmArgs& a) { return launch_fgemm_ad(st, a); }

// layer-level shorthand: square Hp blocks, no groups
static int32_t wgrad_w(hipStream_t st, const WideDims& d, const char* A_T, int a_ncb, int a_cb0, int nI, const char* B_T,
                       int b_ncb, int b_cb0, int nJ, int64_t rows, float* partial, size_t partial_floats, float* dest,
                       long strideA, long strideB, int tag) {
  FWgradArgs a;
  a.A_T = A_T; a.a_ncb = a_ncb; a.a_cb0 = a_cb0; a.nI = nI;
  a.B_T = B_T; a.b_ncb = b_ncb; a.b_cb0 = b_cb0; a.nJ = nJ;
  a.rows = rows;
  a.HpA = d.Hp; a.HA = d.H; a.HpB = d.Hp; a.HB = d.H;
  a.partial = partial; a.partial_floats = partial_floats;
  a.dest = dest; a.strideA = strideA; a.strideB = strideB;
  a.tag = tag;
  return launch_fwgrad(st, a);
}
static int32_t colsum_w(hipStream_t st, const float* X, long ldx, const float* Z, long ldz, int mode, int M, int ncol,
                        float* partial, float* dest) {
  ColsumRowsArgs c;
  c.X = X; c.ldx = ldx; c.Z = Z; c.ldz = ldz; c.mode = mode; c.M = M; c.ncol = ncol;
  c.partial = partial; c.dest = dest;
  return launch_colsum_rows(st, c);
}

int32_t wide_layer_fwd(hipStream_t st, const WideLayerArgs& a) {
  const int k = a.k;   // edge attributes: a.attr [E, k], or d2 alone (k = 1) when a.attr is null
  const WideDims d(a.N, a.E, a.H, k);
  const int H = d.H, Hp = d.Hp;
  WideWs w = carve_ws_w(a.ws, d);
  WideSaved s = carve_saved_w(a.saved, d);
  const LayerOffW o(H, k);
  const long HH = (long)H * H, PP = (long)Hp * Hp;
  const float* W = a.W;

  // packed (elements): [W1a | W1b] at 0 (K = Hp, 2 ncb column blocks), W2 at 2 PP, [W3a ; W3b] at 3 PP (K = 2 Hp), W4 at 5 PP
  {
    PackFragArgs pk;
    pk.src = W; pk.K = H; pk.Nn = H; pk.Kp = Hp; pk.Np = Hp;
    pk.dst = w.packed; pk.nparts = 6;
    pk.part[0] = {o.W1, H, 1, 0, d.nkb, 0, 0};
    pk.part[1] = {o.W1 + HH, H, 1, 0, d.nkb, 0, d.ncb};
    pk.part[2] = {o.W2, H, 1, 2 * PP, d.nkb, 0, 0};
    pk.part[3] = {o.W3, H, 1, 3 * PP, 2 * d.nkb, 0, 0};
    pk.part[4] = {o.W3 + HH, H, 1, 3 * PP, 2 * d.nkb, d.nkb, 0};
    pk.part[5] = {o.W4, H, 1, 5 * PP, d.nkb, 0, 0};
    HGNN_TRY(launch_pack_frag(st, pk));
  }
  {  // h -> first half of the [h ; M] operand
    ToFragArgs t;
    t.X = a.h_in; t.ldx = H; t.M = d.N; t.Mp = d.Np; t.ncol = H; t.Cp = Hp;
    t.R = w.hM_R; t.r_nkb = 2 * d.nkb; t.r_kb0 = 0;
    t.T = s.hM_T; t.t_ncb = 2 * d.ncb; t.t_cb0 = 0;
    HGNN_TRY(launch_to_frag(st, t));
  }
  {  // P | Q = h [W1a | W1b] + [b1 | 0], bf16 row-major for the edge gathers
    FGemmArgs g = nn_args(w.hM_R, 2 * d.nkb, d.Np / 32, w.packed, 2 * d.ncb, PT_GEMM_NODE);
    g.nkb = d.nkb; g.kper = d.nkb;            // only the h half of the operand rows
    g.b_sj = d.nkb;
    g.M = d.N; g.Cb = s.PQ; g.ldcb = 2 * Hp;
    g.bias = W + o.b1; g.nbias = H;
    HGNN_TRY(launch_fgemm_rows(st, g));
  }
  EdgeElemArgs e;
  e.E = d.E; e.nrb = (int)(d.Ep / 32); e.H = H; e.Hp = Hp;
  e.dst = a.dst; e.col = a.col; e.attr = a.attr ? a.attr : a.d2; e.k = k; e.PQ = s.PQ; e.w1d = W + o.W1 + 2 * HH;
  e.a1_R = s.a1_R; e.a1_T = s.a1_T;
  if (d.Ep > 0) {
    {
      ProfScope ps(PT_EDGE_ELEM, st);
      if (k == 1) k_edge_elem<EE_A1, 1><<<elem_grid(e.nrb, Hp), 256, 0, st>>>(e);
      else k_edge_elem<EE_A1, 16><<<elem_grid(e.nrb, Hp), 256, 0, st>>>(e);
      HGNN_LAUNCH_CHECK("k_edge_elem (a1)");
    }
    // z2 = a1 W2 + b2 (T fragments)
    FGemmArgs g = nn_args(s.a1_R, d.nkb, (int)(d.Ep / 32), w.packed + 2 * PP, d.ncb, PT_FRAG_GEMM_EDGE);
    g.T = s.z2_T; g.t_ncb = d.ncb;
    g.bias = W + o.b2; g.nbias = H;
    // with the per-atom sums of m = silu(z2) and x_e = wx . m_e formed in the epilogue
    g.seg_dst = a.dst; g.seg_row_ptr = a.row_ptr; g.seg_wx = W + o.wx; g.seg_H = H; g.seg_E = d.E; g.seg_alpha = a.alpha;
    g.seg_M = s.M; g.seg_ldm = Hp; g.seg_first = w.seg_first; g.seg_last = w.seg_last; g.seg_ldp = Hp;
    g.seg_xe = w.xe_part; g.seg_xe_stride = d.Ep;
    HGNN_TRY(launch_fgemm_rows_T(st, g));
  }
  if (d.N > 0) {  // atoms whose edges span several strips, atoms without edges, v'
    ProfScope ps(PT_SEG_FWD, st);
    k_seg_fwd_fix<<<(unsigned)((d.N + 3) / 4), 256, 0, st>>>(d.N, Hp, d.ncb / 4, a.row_ptr, w.seg_first, w.seg_last,
                                                            w.xe_part, d.Ep, a.rvec, a.alpha, a.v_in, s.M, a.v_out, s.xe);
    HGNN_LAUNCH_CHECK("k_seg_fwd_fix");
  }
  {  // M -> second half of the [h ; M] operand
    ToFragArgs t;
    t.X = s.M; t.ldx = Hp; t.M = d.N; t.Mp = d.Np; t.ncol = Hp; t.Cp = Hp;
    t.R = w.hM_R; t.r_nkb = 2 * d.nkb; t.r_kb0 = d.nkb;
    t.T = s.hM_T; t.t_ncb = 2 * d.ncb; t.t_cb0 = d.ncb;
    HGNN_TRY(launch_to_frag(st, t));
  }
  {  // z3 = [h ; M] W3 + b3
    FGemmArgs g = nn_args(w.hM_R, 2 * d.nkb, d.Np / 32, w.packed + 3 * PP, d.ncb, PT_GEMM_NODE);
    g.M = d.N; g.Cf = s.z3; g.ldc = Hp; g.ncol_f = Hp;
    g.bias = W + o.b3; g.nbias = H;
    HGNN_TRY(launch_fgemm_rows(st, g));
  }
  {  // a3 = silu(z3)
    ToFragArgs t;
    t.X = s.z3; t.ldx = Hp; t.mode = 1; t.M = d.N; t.Mp = d.Np; t.ncol = H; t.Cp = Hp;
    t.R = w.x_R; t.r_nkb = d.nkb; t.r_kb0 = 0;
    t.T = s.a3_T; t.t_ncb = d.ncb; t.t_cb0 = 0;
    HGNN_TRY(launch_to_frag(st, t));
  }
  {  // h' = h + a3 W4 + b4
    FGemmArgs g = nn_args(w.x_R, d.nkb, d.Np / 32, w.packed + 5 * PP, d.ncb, PT_GEMM_NODE);
    g.M = d.N; g.Cf = a.h_out; g.ldc = H; g.ncol_f = H;
    g.r1 = a.h_in; g.ld1 = H;
    g.bias = W + o.b4; g.nbias = H;
    HGNN_TRY(launch_fgemm_rows(st, g));
  }
  return HGNN_OK;
}

int32_t wide_layer_bwd(hipStream_t st, const WideLayerArgs& a) {
  const int k = a.k;   // edge attributes: a.attr [E, k], or d2 alone (k = 1) when a.attr is null
  const WideDims d(a.N, a.E, a.H, k);
  const int H = d.H, Hp = d.Hp;
  WideWs w = carve_ws_w(a.ws, d);
  WideSaved s = carve_saved_w(a.saved, d);
  const LayerOffW o(H, k);
  const long HH = (long)H * H, PP = (long)Hp * Hp;
  const float* W = a.W;
  float* gW = a.gW;

  // packed (elements): W4^T at 0, [W3a^T | W3b^T] at PP (K = Hp, 2 ncb column blocks), W2^T at 3 PP,
  // [W1a^T ; W1b^T] at 4 PP (K = 2 Hp)
  {
    PackFragArgs pk;
    pk.src = W; pk.K = H; pk.Nn = H; pk.Kp = Hp; pk.Np = Hp;
    pk.dst = w.packed; pk.nparts = 6;
    pk.part[0] = {o.W4, 1, H, 0, d.nkb, 0, 0};
    pk.part[1] = {o.W3, 1, H, PP, d.nkb, 0, 0};
    pk.part[2] = {o.W3 + HH, 1, H, PP, d.nkb, 0, d.ncb};
    pk.part[3] = {o.W2, 1, H, 3 * PP, d.nkb, 0, 0};
    pk.part[4] = {o.W1, 1, H, 4 * PP, 2 * d.nkb, 0, 0};
    pk.part[5] = {o.W1 + HH, 1, H, 4 * PP, 2 * d.nkb, d.nkb, 0};
    HGNN_TRY(launch_pack_frag(st, pk));
  }
  // Weight gradients and bias sums feed nothing downstream: they run on the library's side stream (sx), which forks
  // from and joins the caller's stream through events. Buffers read on sx are written once per call on st.
  SideStream& ss = side_stream();
  HGNN_REQUIRE(ss.ok, HGNN_ERR_HIP, "could not create the side stream");
  hipStream_t sx = side_stream_enabled(true) ? ss.s : st;
  {  // g_h' as R and T ([h ; M] and silu(z3) were left as T fragments by the forward pass)
    ToFragArgs u;
    u.X = a.g_h_out; u.ldx = H; u.M = d.N; u.Mp = d.Np; u.ncol = H; u.Cp = Hp;
    u.R = w.x_R; u.r_nkb = d.nkb; u.r_kb0 = 0;
    u.T = w.gh_T; u.t_ncb = d.ncb; u.t_cb0 = 0;
    HGNN_TRY(launch_to_frag(st, u));
  }
  HGNN_TRY(stream_after(sx, st, ss.ev[0]));
  // side: g_W4 = a3^T g_h', g_b4 = column sums of g_h'
  HGNN_TRY(wgrad_w(sx, d, s.a3_T, d.ncb, 0, d.ncb, w.gh_T, d.ncb, 0, d.ncb, d.Np, w.partial, w.partial_floats, gW + o.W4,
                   0, 0, PT_WGRAD_NODE));
  HGNN_TRY(colsum_w(sx, a.g_h_out, H, nullptr, 0, 0, d.N, H, w.cs_partial, gW + o.b4));
  {  // g_a3 = g_h' W4^T
    FGemmArgs g = nn_args(w.x_R, d.nkb, d.Np / 32, w.packed, d.ncb, PT_GEMM_NODE);
    g.M = d.N; g.Cf = w.nodeA; g.ldc = Hp; g.ncol_f = Hp;
    HGNN_TRY(launch_fgemm_rows(st, g));
  }
  {  // g_z3 = g_a3 silu'(z3) as R and T
    ToFragArgs t;
    t.X = w.nodeA; t.ldx = Hp; t.Z = s.z3; t.ldz = Hp; t.mode = 2; t.M = d.N; t.Mp = d.Np; t.ncol = H; t.Cp = Hp;
    t.R = w.x_R; t.r_nkb = d.nkb; t.r_kb0 = 0;
    t.T = w.gz3_T; t.t_ncb = d.ncb; t.t_cb0 = 0;
    HGNN_TRY(launch_to_frag(st, t));
  }
  HGNN_TRY(stream_after(sx, st, ss.ev[1]));
  // side: g_b3 = column sums of g_z3, g_W3 = [h ; M]^T g_z3
  HGNN_TRY(colsum_w(sx, w.nodeA, Hp, s.z3, Hp, 2, d.N, H, w.cs_partial, gW + o.b3));
  HGNN_TRY(wgrad_w(sx, d, s.hM_T, 2 * d.ncb, 0, 2 * d.ncb, w.gz3_T, d.ncb, 0, d.ncb, d.Np, w.partial, w.partial_floats,
                   gW + o.W3, HH, 0, PT_WGRAD_NODE));
  {  // [g_h(a) | g_M] = g_z3 [W3a^T | W3b^T]: fp32 for the residual, bf16 for the edge gathers
    FGemmArgs g = nn_args(w.x_R, d.nkb, d.Np / 32, w.packed + PP, 2 * d.ncb, PT_GEMM_NODE);
    g.M = d.N; g.Cf = w.nodeB; g.ldc = 2 * Hp; g.ncol_f = 2 * Hp;
    g.Cb = w.gM_b; g.ldcb = 2 * Hp;
    HGNN_TRY(launch_fgemm_rows(st, g));
  }
  // edge part
  EdgeElemArgs e;
  e.E = d.E; e.nrb = (int)(d.Ep / 32); e.H = H; e.Hp = Hp;
  e.dst = a.dst; e.col = a.col; e.attr = a.attr ? a.attr : a.d2; e.k = k; e.PQ = s.PQ; e.w1d = W + o.W1 + 2 * HH;
  e.z2_T = s.z2_T; e.gM = w.gM_b + Hp; e.ldgM = 2 * Hp; e.cvec = w.cvec; e.wx = W + o.wx; e.alpha = a.alpha;
  e.gz2_R = w.gz2_R; e.gz2_T = w.gz2_T; e.ga1_T = w.ga1_T; e.colpart = w.colpart;
  e.gz1_rm = reinterpret_cast<unsigned short*>(w.gz2_R);   // free again once g_a1 has been formed
  const dim3 egrid = elem_grid(e.nrb, Hp);
  const int eg = (int)egrid.y;   // column-sum partials
  HGNN_TRY(launch_edge_cvec(st, d.E, a.dst, a.rvec, a.g_v_out, a.alpha, w.cvec));
  {
    ProfScope ps(PT_EDGE_ELEM, st);
    k_edge_elem<EE_GZ2, 1><<<egrid, 256, 0, st>>>(e);
    HGNN_LAUNCH_CHECK("k_edge_elem (g_z2)");
  }
  HGNN_TRY(stream_after(sx, st, ss.ev[2]));
  {  // side: g_b2, g_wx from the kernel's column sums
    ProfScope ps(PT_COLSUM, sx);
    HGNN_TRY(launch_reduce_cols(sx, w.colpart, eg, 2 * Hp, H, gW + o.b2));
    HGNN_TRY(launch_reduce_cols(sx, w.colpart + Hp, eg, 2 * Hp, H, gW + o.wx));
  }
  // g_W2 = a1^T g_z2 fills the chip by itself: it stays on the caller's stream, with a partial buffer of its own
  HGNN_TRY(wgrad_w(st, d, s.a1_T, d.ncb, 0, d.ncb, w.gz2_T, d.ncb, 0, d.ncb, d.Ep, w.partial_e, w.partial_e_floats,
                   gW + o.W2, 0, 0, PT_FRAG_WGRAD_EDGE));
  if (d.Ep > 0) {  // g_a1 = g_z2 W2^T (T fragments)
    FGemmArgs g = nn_args(w.gz2_R, d.nkb, (int)(d.Ep / 32), w.packed + 3 * PP, d.ncb, PT_FRAG_GEMM_EDGE);
    g.T = w.ga1_T; g.t_ncb = d.ncb;
    HGNN_TRY(launch_fgemm_rows_T(st, g));
  }
  e.colpart = w.colpart2;
  {
    ProfScope ps(PT_EDGE_ELEM, st);
    if (k == 1) k_edge_elem<EE_GZ1, 1><<<egrid, 256, 0, st>>>(e);
    else k_edge_elem<EE_GZ1, 16><<<egrid, 256, 0, st>>>(e);
    HGNN_LAUNCH_CHECK("k_edge_elem (g_z1)");
  }
  if (a.g_attr && d.E > 0) {  // gradient with respect to the edge attributes: g_z1 W1d^T
    ProfScope ps(PT_EDGE_ELEM, st);
    const int nwg = std::min(e.nrb / 4, 512);   // Ep is a multiple of 256: nrb / 4 >= 2
    k_gattr<<<nwg, 256, (size_t)(Hp / 16) * 1024, st>>>(d.E, e.nrb, H, Hp, k, e.gz1_rm, e.w1d, a.g_attr);
    HGNN_LAUNCH_CHECK("k_gattr");
  }
  if (a.g_rvec) HGNN_TRY(launch_edge_grvec(st, d.E, a.dst, s.xe, a.g_v_out, a.alpha, a.g_rvec));
  // g_P, g_Q: per-atom sums of g_z1 over the destination-sorted and the source-sorted lists
  if (d.N > 0) {
    ProfScope ps(PT_SEGSUM_DST, st);
    k_segsum_rows<<<(unsigned)((d.N + 3) / 4), 256, 0, st>>>(d.N, Hp, a.row_ptr, nullptr, e.gz1_rm, w.g_PQ, 2 * Hp);
    HGNN_LAUNCH_CHECK("k_segsum_rows");
  }
  if (d.N > 0) {
    ProfScope ps(PT_SEGSUM_SRC, st);
    k_segsum_rows<<<(unsigned)((d.N + 3) / 4), 256, 0, st>>>(d.N, Hp, a.colT_ptr, a.permT, e.gz1_rm, w.g_PQ + Hp, 2 * Hp);
    HGNN_LAUNCH_CHECK("k_segsum_rows");
  }
  {  // [g_P | g_Q] as R (contraction 2 Hp) and T
    ToFragArgs t;
    t.X = w.g_PQ; t.ldx = 2 * Hp; t.M = d.N; t.Mp = d.Np; t.ncol = 2 * Hp; t.Cp = 2 * Hp;
    t.R = w.x_R; t.r_nkb = 2 * d.nkb; t.r_kb0 = 0;
    t.T = w.gPQ_T; t.t_ncb = 2 * d.ncb; t.t_cb0 = 0;
    HGNN_TRY(launch_to_frag(st, t));
  }
  HGNN_TRY(stream_after(sx, st, ss.ev[3]));
  {  // side: g_b1, g_w1d from the g_z1 kernel's column sums; g_W1a = h^T g_P, g_W1b = h^T g_Q
    ProfScope ps(PT_COLSUM, sx);
    HGNN_TRY(launch_reduce_cols(sx, w.colpart2, eg, (long)(1 + k) * Hp, H, gW + o.b1));
    // the k rows of W1 that act on the edge attributes: one group per row
    HGNN_TRY(launch_reduce_cols(sx, w.colpart2 + Hp, eg, (long)(1 + k) * Hp, H, gW + o.W1 + 2 * HH, k, Hp, H));
  }
  HGNN_TRY(wgrad_w(sx, d, s.hM_T, 2 * d.ncb, 0, d.ncb, w.gPQ_T, 2 * d.ncb, 0, 2 * d.ncb, d.Np, w.partial, w.partial_floats,
                   gW + o.W1, 0, HH, PT_WGRAD_NODE));
  {  // g_h = g_h' + g_h(a) + [g_P | g_Q] [W1a^T ; W1b^T]
    FGemmArgs g = nn_args(w.x_R, 2 * d.nkb, d.Np / 32, w.packed + 4 * PP, d.ncb, PT_GEMM_NODE);
    g.M = d.N; g.Cf = a.g_h_in; g.ldc = H; g.ncol_f = H;
    g.r1 = a.g_h_out; g.ld1 = H;
    g.r2 = w.nodeB; g.ld2 = 2 * Hp;
    HGNN_TRY(launch_fgemm_rows(st, g));
  }
  HGNN_TRY(stream_after(st, sx, ss.ev[4]));   // join: the caller's stream now also orders after every gradient
  if (a.g_v_in != a.g_v_out) HGNN_TRY(launch_copy_f32(st, a.g_v_out, a.g_v_in, (int64_t)d.N * 3));
  return HGNN_OK;
}

}  // namespace hgnn
