// Matrix-core kernels for gfx950 (wave64, MFMA):
//   k_pack    fp32 [in,out] weight slices -> blocks in B-operand order (bf16 or fp32)
//   k_gemm    row tile x (H x H) blocks, A staged through padded LDS, B streamed from L2 in operand
//             order, epilogue (bias / SiLU' / residual adds) applied on the accumulator registers
//   k_wgrad   sum over rows of outer products with split-K partials reduced in a fixed order
//   k_colsum  column sums with the same deterministic two-stage reduction
//
// Operand layouts used below (v_mfma_f32_32x32x16_bf16 and v_mfma_f32_32x32x2_f32):
//   A: lane l holds row (l & 31); bf16: 8 consecutive k at 8*(l>>5); fp32: the single k = (l>>5)
//   B: lane l holds column (l & 31), same k as A
//   D: register v of lane l is element (row 8*(v>>2) + 4*(l>>5) + (v&3), column (l & 31))
// For fp32 the k index inside a block of 8 is permuted (lane half g takes k = 4g..4g+3 over four
// consecutive instructions) so that both operands are fetched as one float4; the permutation is the
// same for A and B and therefore cancels.
#include "devmath.h"
#include "gemm.h"

namespace hgnn {

// ---------------------------------------------------------------------------------------------
// pack
// ---------------------------------------------------------------------------------------------
template <bool BF16>
__global__ void k_pack(PackArgs a, int H, long src_grp_stride, long dst_grp_stride) {
  const int b = blockIdx.y;
  const int grp = blockIdx.z;
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= H * H) return;
  if (b == a.nblocks) {   // the extra block as three bf16 planes (see split_bf16x3), each in the bf16 operand order
    const PackDesc d = a.d[a.x3_desc];
    const int t = idx & 7, lane = (idx >> 3) & 63, kb = (idx >> 9) % (H / 16), nb = (idx >> 9) / (H / 16);
    const int n = nb * 32 + (lane & 31);
    const int k = kb * 16 + (lane >> 5) * 8 + t;
    const float v = a.src[d.src_off + (long)k * d.sk + (long)n * d.sn];
    const unsigned h = f2bf_bits(v);
    const float r = v - __uint_as_float(h << 16);
    const unsigned m = f2bf_bits(r);
    const float q = r - __uint_as_float(m << 16);
    unsigned short* dst = static_cast<unsigned short*>(a.x3_dst);
    dst[idx] = (unsigned short)h;
    dst[(long)H * H + idx] = (unsigned short)m;
    dst[2L * H * H + idx] = (unsigned short)f2bf_bits(q);
    return;
  }
  const PackDesc d = a.d[b];
  const float* src = a.src + grp * src_grp_stride + d.src_off;
  int n, k;
  if (BF16) {
    const int t = idx & 7, lane = (idx >> 3) & 63, kb = (idx >> 9) % (H / 16), nb = (idx >> 9) / (H / 16);
    n = nb * 32 + (lane & 31);
    k = kb * 16 + (lane >> 5) * 8 + t;
  } else {
    const int t = idx & 3, lane = (idx >> 2) & 63, kb = (idx >> 8) % (H / 8), nb = (idx >> 8) / (H / 8);
    n = nb * 32 + (lane & 31);
    k = kb * 8 + (lane >> 5) * 4 + t;
  }
  const float v = src[(long)k * d.sk + (long)n * d.sn];
  const long o = grp * dst_grp_stride + (long)b * H * H + idx;
  if (BF16) {
    reinterpret_cast<unsigned short*>(a.dst)[o] = (unsigned short)f2bf_bits(v);
  } else {
    reinterpret_cast<float*>(a.dst)[o] = v;
  }
}

int32_t launch_pack(hipStream_t st, int H, bool bf16, const PackArgs& a, int groups, long src_grp_stride,
                    long dst_grp_stride_elems) {
  if (a.nblocks <= 0 || groups <= 0) return HGNN_OK;
  ProfScope ps(PT_PACK, st);
  const bool x3 = a.x3_dst != nullptr && !bf16 && groups == 1;
  dim3 grid((H * H + 255) / 256, a.nblocks + (x3 ? 1 : 0), groups);
  if (bf16) k_pack<true><<<grid, 256, 0, st>>>(a, H, src_grp_stride, dst_grp_stride_elems);
  else k_pack<false><<<grid, 256, 0, st>>>(a, H, src_grp_stride, dst_grp_stride_elems);
  HGNN_LAUNCH_CHECK("k_pack");
  return HGNN_OK;
}

// ---------------------------------------------------------------------------------------------
// row-tile GEMM
// ---------------------------------------------------------------------------------------------
// 32-bit byte offsets from a uniform base (row * pitch fits 24 x 24 -> 32 bits for every node tensor here):
// one full-rate multiply per row instead of 64-bit index arithmetic per element
__device__ __forceinline__ float ld_f32(const float* base, unsigned byte_off) {
  return *reinterpret_cast<const float*>(reinterpret_cast<const char*>(base) + byte_off);
}
__device__ __forceinline__ float4 ld_f32x4(const float* base, unsigned byte_off) {
  return *reinterpret_cast<const float4*>(reinterpret_cast<const char*>(base) + byte_off);
}
__device__ __forceinline__ void st_f32(float* base, unsigned byte_off, float v) {
  *reinterpret_cast<float*>(reinterpret_cast<char*>(base) + byte_off) = v;
}

// TM_ rows per workgroup tile
template <int H, bool BF16, int TM_ = 64>
struct GemmCfg {
  static constexpr int TM = TM_;
  static constexpr int WC = (H / 32 < 4) ? H / 32 : 4;   // wavefronts side by side over columns
  static constexpr int WR = 4 / WC;                      // and over rows
  static constexpr int WROWS = TM / WR;
  static constexpr int WCOLS = H / WC;
  static constexpr int RB = WROWS / 32;
  static constexpr int CB = WCOLS / 32;
  static constexpr int STRIDE = BF16 ? H + 8 : H + 4;    // LDS row pitch in elements (bank spread)
  static constexpr int CSTR = H + 4;                      // epilogue staging row pitch (floats)
  static constexpr size_t A_BYTES = (size_t)TM * STRIDE * (BF16 ? 2 : 4);
  static constexpr size_t C_BYTES = (size_t)WR * 32 * CSTR * 4;
  static constexpr size_t LDS_BYTES = A_BYTES > C_BYTES ? A_BYTES : C_BYTES;
  static_assert(WROWS % 32 == 0 && (TM * (H / 4)) % 256 == 0, "tile height does not fit the wavefront grid");
};

__device__ __forceinline__ bool tile_of_group(const int32_t* grp_ptr, int S, int TM, int tile, int& grp, int& rbeg,
                                              int& rend) {
  for (int s = 0; s < S; ++s) {
    const int b = grp_ptr[s], e = grp_ptr[s + 1];
    const int nt = (e - b + TM - 1) / TM;
    if (tile < nt) {
      grp = s;
      rbeg = b + tile * TM;
      rend = e;
      return true;
    }
    tile -= nt;
  }
  return false;
}

// The three parts of a row-tile product. They share the workgroup's LDS: the A tile of one k chunk, then (after a
// barrier) the accumulators on their way to row-major stores.
template <int H, bool BF16, int TM>
__device__ __forceinline__ void gemm_stage_a(const GemmArgs& p, int kc, int rbeg, int rend, unsigned char* smem) {
  using C = GemmCfg<H, BF16, TM>;
  const int tid = threadIdx.x;
  {
    // ---- stage the A tile (rows rbeg.., all H columns of chunk kc) into LDS
    const float* __restrict__ A = p.A[kc];
    const int lda = p.lda[kc];
    constexpr int CH = H / 4;
    constexpr int ITER = C::TM * CH / 256;
    constexpr int UN = ITER % 8 == 0 ? 8 : (ITER % 6 == 0 ? 6 : (ITER % 4 == 0 ? 4 : (ITER % 2 == 0 ? 2 : 1)));
    static_assert(ITER % UN == 0, "staging loop must divide evenly");
    for (int it0 = 0; it0 < ITER; it0 += UN) {
      float4 v[UN];
      long gr[UN];
      // all loads of the batch are issued before any of them is used (rows past the end are clamped, then zeroed).
      // The row indices come first, under one uniform branch: with the test inside the loop every load waited
      // for the one before it.
#pragma unroll
      for (int u = 0; u < UN; ++u) {
        const int r = (tid + (it0 + u) * 256) / CH;
        const int pos = rbeg + r;
        gr[u] = pos < rend ? pos : rend - 1;
      }
      if (p.row_idx) {
#pragma unroll
        for (int u = 0; u < UN; ++u) gr[u] = p.row_idx[gr[u]];
      }
#pragma unroll
      for (int u = 0; u < UN; ++u) {
        const int c = tid + (it0 + u) * 256;
        const int q = c % CH;
        v[u] = *reinterpret_cast<const float4*>(A + gr[u] * lda + q * 4);
      }
#pragma unroll
      for (int u = 0; u < UN; ++u) {
        const int c = tid + (it0 + u) * 256;
        const int r = c / CH, q = c - r * CH;
        float4 w = v[u];
        if (p.a_silu) {
          w.x = silu_f(w.x); w.y = silu_f(w.y); w.z = silu_f(w.z); w.w = silu_f(w.w);
        }
        if (rbeg + r >= rend) w = make_float4(0.f, 0.f, 0.f, 0.f);
        if (BF16) {
          uint2 o;
          o.x = pack_bf16x2(w.x, w.y);
          o.y = pack_bf16x2(w.z, w.w);
          *reinterpret_cast<uint2*>(smem + ((size_t)r * C::STRIDE + q * 4) * 2) = o;
        } else {
          *reinterpret_cast<float4*>(smem + ((size_t)r * C::STRIDE + q * 4) * 4) = w;
        }
      }
    }
  }
}

template <int H, bool BF16, int TM>
__device__ __forceinline__ void gemm_multiply(const GemmArgs& p, int kc, int cb, int grp, const unsigned char* smem,
                                              f32x16_t (&acc)[GemmCfg<H, BF16, TM>::RB][GemmCfg<H, BF16, TM>::CB]) {
  using C = GemmCfg<H, BF16, TM>;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: fragment offsets stay in scalar registers
  const int wr = wave / C::WC, wc = wave % C::WC;
  {
    // ---- multiply. All workgroups run this loop at about the same time over the same packed block: each starts at
    // a different k step so that they do not all ask the same L2 lines at once.
    const int krot = blockIdx.x * 5;
    const long bblk0 = grp * p.grp_blk_stride + p.blk[kc][cb];
    if (BF16) {
      // B fragments D steps ahead in a register ring, through buffer loads (resource and fragment offset in scalar
      // registers, one per-lane offset register); A fragments one step ahead. With each load next to its use the
      // loop was a chain of L2 round trips, one per step. The scheduling barrier keeps the refills where they are.
      constexpr int NKB = H / 16;
      constexpr int D = NKB < 4 ? NKB : 4;
      const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
          const_cast<char*>(reinterpret_cast<const char*>(p.B)) + bblk0 * (long)(H * H * 2), 0, H * H * 2, 0x00020000);
      unsigned lo = lane * 16u;
      unsigned ao = (unsigned)(((wr * C::WROWS + (lane & 31)) * C::STRIDE + (lane >> 5) * 8) * 2);
      asm volatile("" : "+v"(lo), "+v"(ao));   // kept as one register each: not folded into per-step addresses
      bf16x8_t b[D][C::CB], a[2][C::RB];
      auto load_b = [&](int kk, bf16x8_t (&o)[C::CB]) {
        const int kb = (kk + krot) & (NKB - 1);
#pragma unroll
        for (int j = 0; j < C::CB; ++j)
          o[j] = __builtin_bit_cast(bf16x8_t, __builtin_amdgcn_raw_buffer_load_b128(
                                                  rs, lo, ((wc * C::CB + j) * NKB + kb) * 1024, 0));
      };
      auto load_a = [&](int kk, bf16x8_t (&o)[C::RB]) {
        const int kb = (kk + krot) & (NKB - 1);
#pragma unroll
        for (int i = 0; i < C::RB; ++i)
          o[i] = *reinterpret_cast<const bf16x8_t*>(smem + ao + (i * 32 * C::STRIDE + kb * 16) * 2);
      };
#pragma unroll
      for (int d = 0; d < D; ++d) load_b(d, b[d]);
      load_a(0, a[0]);
#pragma unroll
      for (int kk = 0; kk < NKB; ++kk) {
        if (kk + 1 < NKB) load_a(kk + 1, a[(kk + 1) & 1]);
#pragma unroll
        for (int j = 0; j < C::CB; ++j)
#pragma unroll
          for (int i = 0; i < C::RB; ++i)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[kk & 1][i], b[kk % D][j], acc[i][j], 0, 0, 0);
        if (kk + D < NKB) load_b(kk + D, b[kk % D]);
        __builtin_amdgcn_sched_barrier(0);
      }
    } else {
      // the same ring for fp32 operands (four steps of 8 k ahead; A fragments one step ahead)
      constexpr int NKB = H / 8;
      constexpr int D = 4;
      const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
          const_cast<char*>(reinterpret_cast<const char*>(p.B)) + bblk0 * (long)(H * H * 4), 0, H * H * 4, 0x00020000);
      unsigned lo = lane * 16u;
      unsigned ao = (unsigned)(((wr * C::WROWS + (lane & 31)) * C::STRIDE + (lane >> 5) * 4) * 4);
      asm volatile("" : "+v"(lo), "+v"(ao));
      typedef float f32x4v_t __attribute__((ext_vector_type(4)));
      f32x4v_t b[D][C::CB], a[2][C::RB];
      auto load_b = [&](int kk, f32x4v_t (&o)[C::CB]) {
        const int kb = (kk + krot) & (NKB - 1);
#pragma unroll
        for (int j = 0; j < C::CB; ++j)
          o[j] = __builtin_bit_cast(f32x4v_t, __builtin_amdgcn_raw_buffer_load_b128(
                                                  rs, lo, ((wc * C::CB + j) * NKB + kb) * 1024, 0));
      };
      auto load_a = [&](int kk, f32x4v_t (&o)[C::RB]) {
        const int kb = (kk + krot) & (NKB - 1);
#pragma unroll
        for (int i = 0; i < C::RB; ++i)
          o[i] = *reinterpret_cast<const f32x4v_t*>(smem + ao + (i * 32 * C::STRIDE + kb * 8) * 4);
      };
#pragma unroll
      for (int d = 0; d < D; ++d) load_b(d, b[d]);
      load_a(0, a[0]);
#pragma unroll
      for (int kk = 0; kk < NKB; ++kk) {
        if (kk + 1 < NKB) load_a(kk + 1, a[(kk + 1) & 1]);
#pragma unroll
        for (int j = 0; j < C::CB; ++j)
#pragma unroll
          for (int i = 0; i < C::RB; ++i) {
            const f32x4v_t av = a[kk & 1][i], bv = b[kk % D][j];
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av.x, bv.x, acc[i][j], 0, 0, 0);
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av.y, bv.y, acc[i][j], 0, 0, 0);
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av.z, bv.z, acc[i][j], 0, 0, 0);
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av.w, bv.w, acc[i][j], 0, 0, 0);
          }
        if (kk + D < NKB) load_b(kk + D, b[kk % D]);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
}

// KEEP: the finished values (through silu when keep_silu is set; zeros in rows past the end) also go, in the layout
// of an A tile, to `keep`, which must not overlap `smem`: the next product of a chain takes them from there.
template <int H, bool BF16, int TM, bool KEEP>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs& p, int cb, int grp, int rbeg, int rend,
                                              f32x16_t (&acc)[GemmCfg<H, BF16, TM>::RB][GemmCfg<H, BF16, TM>::CB],
                                              unsigned char* smem, unsigned char* keep, int keep_silu) {
  using C = GemmCfg<H, BF16, TM>;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wr = wave / C::WC, wc = wave % C::WC;
  // ---- epilogue: the accumulators go through LDS, one 32-row block per wavefront row at a time, so that the
  // auxiliary operands and C are accessed row-major with 16-byte loads and stores (few, wide, whole cache lines)
  const bool use_bias = p.bias && ((p.bias_cb_mask >> cb) & 1);
  const bool pair_out = C::CB == 2 && ((p.pair_cb_mask >> cb) & 1);
  const bool use_add = p.add1 && ((p.add1_cb_mask >> cb) & 1);
  constexpr int CH = H / 4;                 // 4-column chunks per row
  constexpr int PROWS = C::WR * 32;         // rows per pass
  constexpr int RSTEP = 256 / CH;           // rows swept by the 256 threads at once
  constexpr int NCH = PROWS / RSTEP;        // chunks per thread and pass
  float* cst = reinterpret_cast<float*>(smem);
  const int q = tid % CH, r0 = tid / CH;
  float4 bv = make_float4(0.f, 0.f, 0.f, 0.f);
  if (use_bias && !pair_out) bv = *reinterpret_cast<const float4*>(p.bias + grp * p.grp_bias_stride + q * 4);
#pragma unroll
  for (int i = 0; i < C::RB; ++i) {
    __syncthreads();   // nobody reads the A tile (or the previous pass) any more
#pragma unroll
    for (int j = 0; j < C::CB; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v)
        cst[(wr * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3)) * C::CSTR + wc * C::WCOLS + j * 32 + (lane & 31)] = acc[i][j][v];
    __syncthreads();
    if (pair_out) {
      if constexpr (C::CB == 2) {
        // bf16 pairs: word w = wc'*32 + x' of a row holds columns wc'*64 + x' and wc'*64 + 32 + x'
        constexpr int WCH = H / 8;          // 4-word chunks per row
        constexpr int WSTEP = 256 / WCH;
        const int qw = tid % WCH, rw0 = tid / WCH;
        const int c_lo = (qw * 4 / 32) * 64 + (qw * 4) % 32;
        float4 b_lo = make_float4(0.f, 0.f, 0.f, 0.f), b_hi = b_lo;
        if (use_bias) {
          b_lo = *reinterpret_cast<const float4*>(p.bias + grp * p.grp_bias_stride + c_lo);
          b_hi = *reinterpret_cast<const float4*>(p.bias + grp * p.grp_bias_stride + c_lo + 32);
        }
#pragma unroll
        for (int k = 0; k < PROWS / WSTEP; ++k) {
          const int sr = rw0 + k * WSTEP;
          const int pos = rbeg + (sr / 32) * C::WROWS + i * 32 + (sr % 32);
          if (pos < rend) {
            const long gr = p.row_idx ? p.row_idx[pos] : pos;
            const float4 lo = *reinterpret_cast<const float4*>(cst + sr * C::CSTR + c_lo);
            const float4 hi = *reinterpret_cast<const float4*>(cst + sr * C::CSTR + c_lo + 32);
            uint4 o;
            o.x = pack_bf16x2((lo.x + b_lo.x) * p.pair_scale, (hi.x + b_hi.x) * p.pair_scale);
            o.y = pack_bf16x2((lo.y + b_lo.y) * p.pair_scale, (hi.y + b_hi.y) * p.pair_scale);
            o.z = pack_bf16x2((lo.z + b_lo.z) * p.pair_scale, (hi.z + b_hi.z) * p.pair_scale);
            o.w = pack_bf16x2((lo.w + b_lo.w) * p.pair_scale, (hi.w + b_hi.w) * p.pair_scale);
            *reinterpret_cast<uint4*>(p.Cpair + gr * p.ldpair + p.pair_off[cb] + qw * 4) = o;
          }
        }
      }
    } else {
      const int gcol = cb * H + q * 4;
      long grow[NCH];
      bool ok[NCH];
      float4 mv[NCH], a1[NCH], a2[NCH];
      // every auxiliary load of the pass is issued before any result is stored (rows past the end are clamped)
      // (each kind of operand under one uniform branch around its loads, not one branch per load)
#pragma unroll
      for (int k = 0; k < NCH; ++k) {
        const int sr = r0 + k * RSTEP;
        const int pos = rbeg + (sr / 32) * C::WROWS + i * 32 + (sr % 32);
        ok[k] = pos < rend;
        grow[k] = ok[k] ? pos : rend - 1;
      }
      if (p.row_idx) {
#pragma unroll
        for (int k = 0; k < NCH; ++k) grow[k] = p.row_idx[grow[k]];
      }
      if (p.mul) {
#pragma unroll
        for (int k = 0; k < NCH; ++k) mv[k] = *reinterpret_cast<const float4*>(p.mul + grow[k] * p.ldmul + gcol);
      }
      if (use_add) {
#pragma unroll
        for (int k = 0; k < NCH; ++k) a1[k] = *reinterpret_cast<const float4*>(p.add1 + grow[k] * p.ldadd1 + gcol);
      }
      if (p.add2) {
#pragma unroll
        for (int k = 0; k < NCH; ++k) a2[k] = *reinterpret_cast<const float4*>(p.add2 + grow[k] * p.ldadd2 + gcol);
      }
#pragma unroll
      for (int k = 0; k < NCH; ++k) {
        const int sr = r0 + k * RSTEP;
        float4 x = *reinterpret_cast<const float4*>(cst + sr * C::CSTR + q * 4);
        x.x += bv.x; x.y += bv.y; x.z += bv.z; x.w += bv.w;
        if (p.mul) {
          if (p.mul_is_z) {
            x.x *= dsilu_f(mv[k].x); x.y *= dsilu_f(mv[k].y); x.z *= dsilu_f(mv[k].z); x.w *= dsilu_f(mv[k].w);
          } else {
            x.x *= mv[k].x; x.y *= mv[k].y; x.z *= mv[k].z; x.w *= mv[k].w;
          }
        }
        if (use_add) { x.x += a1[k].x; x.y += a1[k].y; x.z += a1[k].z; x.w += a1[k].w; }
        if (p.add2) { x.x += a2[k].x; x.y += a2[k].y; x.z += a2[k].z; x.w += a2[k].w; }
        if (ok[k]) *reinterpret_cast<float4*>(p.C + grow[k] * p.ldc + gcol) = x;
        if constexpr (KEEP) {
          float4 y = x;
          if (keep_silu) { y.x = silu_f(y.x); y.y = silu_f(y.y); y.z = silu_f(y.z); y.w = silu_f(y.w); }
          if (!ok[k]) y = make_float4(0.f, 0.f, 0.f, 0.f);
          const int trow = (sr / 32) * C::WROWS + i * 32 + (sr % 32);   // row of the tile
          if (BF16) {
            uint2 o;
            o.x = pack_bf16x2(y.x, y.y);
            o.y = pack_bf16x2(y.z, y.w);
            *reinterpret_cast<uint2*>(keep + ((size_t)trow * C::STRIDE + q * 4) * 2) = o;
          } else {
            *reinterpret_cast<float4*>(keep + ((size_t)trow * C::STRIDE + q * 4) * 4) = y;
          }
        }
      }
    }
  }
}

template <int H, bool BF16, int TM>
__global__ void __launch_bounds__(256, TM <= 32 ? 4 : 2) k_gemm(GemmArgs p) {
  using C = GemmCfg<H, BF16, TM>;
  extern __shared__ __align__(16) unsigned char smem[];
  const int cb = blockIdx.y;
  int grp = 0, rbeg, rend;
  if (p.grp_ptr) {
    if (!tile_of_group(p.grp_ptr, p.S, C::TM, blockIdx.x, grp, rbeg, rend)) return;
  } else {
    rbeg = blockIdx.x * C::TM;
    rend = p.M;
    if (rbeg >= rend) return;
  }
  f32x16_t acc[C::RB][C::CB];
#pragma unroll
  for (int i = 0; i < C::RB; ++i)
#pragma unroll
    for (int j = 0; j < C::CB; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  for (int kc = 0; kc < p.nkc; ++kc) {
    if (kc) __syncthreads();
    gemm_stage_a<H, BF16, TM>(p, kc, rbeg, rend, smem);
    __syncthreads();
    gemm_multiply<H, BF16, TM>(p, kc, cb, grp, smem, acc);
  }
  gemm_epilogue<H, BF16, TM, false>(p, cb, grp, rbeg, rend, acc, smem, nullptr, 0);
}

// Two products in a row on one row tile, the second one taking the first one's finished tile from LDS as its A
// operand (has_first), or only the second one with its A tile staged once for all of its column blocks: the rows
// are read once and what lies between the two products never leaves the compute unit. LDS: [staging / epilogue |
// the kept A tile]. No groups and no row indirection here.
template <int H, bool BF16, int TM>
__global__ void __launch_bounds__(256, 3) k_gemm_chain(GemmArgs p1, GemmArgs p2, int has_first, int keep_silu) {
  using C = GemmCfg<H, BF16, TM>;
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* keep = smem + C::LDS_BYTES;
  const int rbeg = blockIdx.x * C::TM, rend = p2.M;
  if (rbeg >= rend) return;
  f32x16_t acc[C::RB][C::CB];
  if (has_first) {
#pragma unroll
    for (int i = 0; i < C::RB; ++i)
#pragma unroll
      for (int j = 0; j < C::CB; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    for (int kc = 0; kc < p1.nkc; ++kc) {
      if (kc) __syncthreads();
      gemm_stage_a<H, BF16, TM>(p1, kc, rbeg, rend, smem);
      __syncthreads();
      gemm_multiply<H, BF16, TM>(p1, kc, 0, 0, smem, acc);
    }
    gemm_epilogue<H, BF16, TM, true>(p1, 0, 0, rbeg, rend, acc, smem, keep, keep_silu);
  } else {
    gemm_stage_a<H, BF16, TM>(p2, 0, rbeg, rend, keep);
  }
  __syncthreads();
  for (int cb = 0; cb < p2.ncb; ++cb) {
#pragma unroll
    for (int i = 0; i < C::RB; ++i)
#pragma unroll
      for (int j = 0; j < C::CB; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    gemm_multiply<H, BF16, TM>(p2, 0, cb, 0, keep, acc);
    gemm_epilogue<H, BF16, TM, false>(p2, cb, 0, rbeg, rend, acc, smem, nullptr, 0);
  }
}

// workgroups of this variant that one CU holds at a time (asked once; also raises the LDS limit of the kernel)
template <int H, bool BF16, int TM>
static int gemm_resident_wgs() {
  using C = GemmCfg<H, BF16, TM>;
  static int n = 0;
  if (n == 0) {
    const void* fn = reinterpret_cast<const void*>(&k_gemm<H, BF16, TM>);
    int occ = 0;
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::LDS_BYTES) != hipSuccess ||
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, fn, 256, C::LDS_BYTES) != hipSuccess || occ < 1)
      occ = 1;
    n = occ;
  }
  return n;
}

template <int H, bool BF16, int TM>
static int32_t launch_gemm_tm(hipStream_t st, const GemmArgs& a) {
  using C = GemmCfg<H, BF16, TM>;
  const int tiles = (a.M + C::TM - 1) / C::TM + (a.grp_ptr ? a.S : 0);
  gemm_resident_wgs<H, BF16, TM>();
  ProfScope ps(a.tag, st);
  k_gemm<H, BF16, TM><<<dim3(tiles, a.ncb), 256, C::LDS_BYTES, st>>>(a);
  HGNN_LAUNCH_CHECK("k_gemm");
  return HGNN_OK;
}

// Tile height: a workgroup runs load -> product -> epilogue as one dependent chain whose length grows with the tile
// height, so the shortest tile the wavefront grid allows (32 rows where the four wavefronts sit side by side over
// the columns, i.e. H >= 128; four workgroups per compute unit) gives the most chains in flight. Measured per step
// against 64 / 96-row tiles: config 3 0.64 -> 0.37 ms, config 4 1.69 -> 1.50 ms, config 5 1.28 -> 1.22 ms.
template <int H, bool BF16>
static int32_t launch_gemm_t(hipStream_t st, const GemmArgs& a) {
  if (a.M <= 0) return HGNN_OK;
  if constexpr (GemmCfg<H, BF16>::WR == 1) return launch_gemm_tm<H, BF16, 32>(st, a);
  else return launch_gemm_tm<H, BF16, 64>(st, a);
}

template <int H, bool BF16>
static int32_t launch_gemm_chain_t(hipStream_t st, const GemmArgs* first, const GemmArgs& second, int keep_silu) {
  constexpr int TM = GemmCfg<H, BF16>::WR == 1 ? 32 : 64;
  using C = GemmCfg<H, BF16, TM>;
  if (second.M <= 0) return HGNN_OK;
  constexpr size_t LDS = C::LDS_BYTES + C::A_BYTES;
  static bool raised = false;   // the kernel's LDS limit is raised once per variant
  if (!raised) {
    HGNN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_chain<H, BF16, TM>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS));
    raised = true;
  }
  const int tiles = (second.M + TM - 1) / TM;
  ProfScope ps(second.tag, st);
  k_gemm_chain<H, BF16, TM><<<dim3(tiles), 256, LDS, st>>>(first ? *first : second, second, first ? 1 : 0, keep_silu);
  HGNN_LAUNCH_CHECK("k_gemm_chain");
  return HGNN_OK;
}

// `first` (optional): one column block, its finished tile (through silu when keep_silu) is the A operand of `second`,
// whose own A fields are then ignored; without `first`, `second` runs alone with its A tile (one k chunk) staged
// once for all its column blocks.
int32_t launch_gemm_chain(hipStream_t st, int H, bool bf16, const GemmArgs* first, const GemmArgs& second, int keep_silu) {
  for (const GemmArgs* g : {first, &second}) {
    if (!g) continue;
    HGNN_REQUIRE(!g->row_idx && !g->grp_ptr, HGNN_ERR_BAD_SHAPE, "gemm chain: no groups, no row indirection");
    HGNN_REQUIRE(g->B && (g->C || g->Cpair), HGNN_ERR_NULLPTR, "gemm chain: null operand");
    HGNN_REQUIRE(g->pair_cb_mask == 0 || (H == 256 && g->Cpair), HGNN_ERR_BAD_SHAPE, "gemm chain: pair output needs H = 256");
  }
  HGNN_REQUIRE(second.ncb >= 1 && second.ncb <= 2, HGNN_ERR_BAD_SHAPE, "gemm chain: bad chunk counts");
  if (first) {
    HGNN_REQUIRE(first->nkc >= 1 && first->nkc <= 2 && first->ncb == 1 && first->A[0] && first->pair_cb_mask == 0 &&
                     first->M == second.M,
                 HGNN_ERR_BAD_SHAPE, "gemm chain: bad first product");
  } else {
    HGNN_REQUIRE(second.nkc == 1 && second.A[0], HGNN_ERR_BAD_SHAPE, "gemm chain: the lone product takes one k chunk");
  }
  switch (H) {
    case 64: return bf16 ? launch_gemm_chain_t<64, true>(st, first, second, keep_silu) : launch_gemm_chain_t<64, false>(st, first, second, keep_silu);
    case 128: return bf16 ? launch_gemm_chain_t<128, true>(st, first, second, keep_silu) : launch_gemm_chain_t<128, false>(st, first, second, keep_silu);
    case 256: return bf16 ? launch_gemm_chain_t<256, true>(st, first, second, keep_silu) : launch_gemm_chain_t<256, false>(st, first, second, keep_silu);
  }
  return set_error(HGNN_ERR_BAD_SHAPE, "H must be 64, 128 or 256 (got %d)", H);
}

int32_t launch_gemm(hipStream_t st, int H, bool bf16, const GemmArgs& a) {
  HGNN_REQUIRE(a.nkc >= 1 && a.nkc <= 2 && a.ncb >= 1 && a.ncb <= 2, HGNN_ERR_BAD_SHAPE, "gemm: bad chunk counts");
  HGNN_REQUIRE(a.A[0] && a.B && (a.C || a.Cpair), HGNN_ERR_NULLPTR, "gemm: null operand");
  HGNN_REQUIRE(a.pair_cb_mask == 0 || (H == 256 && a.Cpair), HGNN_ERR_BAD_SHAPE, "gemm: pair output needs H = 256");
  switch (H) {
    case 64: return bf16 ? launch_gemm_t<64, true>(st, a) : launch_gemm_t<64, false>(st, a);
    case 128: return bf16 ? launch_gemm_t<128, true>(st, a) : launch_gemm_t<128, false>(st, a);
    case 256: return bf16 ? launch_gemm_t<256, true>(st, a) : launch_gemm_t<256, false>(st, a);
  }
  return set_error(HGNN_ERR_BAD_SHAPE, "H must be 64, 128 or 256 (got %d)", H);
}

// ---------------------------------------------------------------------------------------------
// deterministic reduction of split partials:  dest[blk][i] = sum_s partial[grp][s][blk][i]
// ---------------------------------------------------------------------------------------------
struct ReduceArgs {
  const float* partial;
  int nsplit;
  int nblk;
  long blk_elems;
  float* dest[8];
  long grp_dest_stride;
};

// wide blocks: one thread per element
__device__ __forceinline__ void reduce_wide(const ReduceArgs& a, int bx, int blk, int grp) {
  const long i = (long)bx * 256 + threadIdx.x;
  if (i >= a.blk_elems || !a.dest[blk]) return;
  const float* p = a.partial + ((long)grp * a.nsplit * a.nblk + blk) * a.blk_elems + i;
  const long step = (long)a.nblk * a.blk_elems;
  if (a.nsplit == 1) {   // a plain copy (also of negative zeros)
    a.dest[blk][grp * a.grp_dest_stride + i] = p[0];
    return;
  }
  // ascending order of the partials is kept; sixteen loads are in flight at a time
  float s = 0.f;
  int k = 0;
  for (; k + 16 <= a.nsplit; k += 16) {
    float v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) v[u] = p[(long)(k + u) * step];
#pragma unroll
    for (int u = 0; u < 16; ++u) s += v[u];
  }
  for (; k < a.nsplit; ++k) s += p[(long)k * step];
  a.dest[blk][grp * a.grp_dest_stride + i] = s;
}

// Few elements, many partials (bias-type sums): 4 threads per element take a contiguous quarter of the
// partials each (in order), then the quarters are added in order. sh: 256 floats of LDS. Every thread of the
// workgroup calls it.
__device__ __forceinline__ void reduce_tall(const ReduceArgs& a, int bx, int blk, int grp, float* sh) {
  const int e = threadIdx.x & 63, ph = threadIdx.x >> 6;
  const long i = (long)bx * 64 + e;
  const int per = (a.nsplit + 3) / 4;
  const int k0 = ph * per;
  const int k1 = k0 + per < a.nsplit ? k0 + per : a.nsplit;
  float s = 0.f;
  if (!a.dest[blk]) return;   // uniform over the block
  if (i < a.blk_elems) {
    const float* p = a.partial + ((long)grp * a.nsplit * a.nblk + blk) * a.blk_elems + i;
    const long step = (long)a.nblk * a.blk_elems;
    int k = k0;
    for (; k + 16 <= k1; k += 16) {
      float v[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) v[u] = p[(long)(k + u) * step];
#pragma unroll
      for (int u = 0; u < 16; ++u) s += v[u];
    }
    for (; k < k1; ++k) s += p[(long)k * step];
  }
  sh[threadIdx.x] = s;
  __syncthreads();
  if (ph == 0 && i < a.blk_elems) a.dest[blk][grp * a.grp_dest_stride + i] = ((sh[e] + sh[64 + e]) + sh[128 + e]) + sh[192 + e];
}
static bool reduce_is_tall(long blk_elems, int nsplit) { return blk_elems <= 1024 && nsplit >= 64; }
static unsigned reduce_xblocks(long blk_elems, int nsplit) {
  return reduce_is_tall(blk_elems, nsplit) ? (unsigned)((blk_elems + 63) / 64) : (unsigned)((blk_elems + 255) / 256);
}

__global__ void __launch_bounds__(256) k_reduce_partials(ReduceArgs a) { reduce_wide(a, blockIdx.x, blockIdx.y, blockIdx.z); }
__global__ void __launch_bounds__(256) k_reduce_partials_tall(ReduceArgs a) {
  __shared__ float sh[256];
  reduce_tall(a, blockIdx.x, blockIdx.y, blockIdx.z, sh);
}

// several reductions in one launch: blockIdx.y counts the blocks of all jobs one after the other, blockIdx.z the
// groups of the job with the most groups
constexpr int REDUCE_QUEUE_MAX = 6;
struct ReduceQueueArgs {
  ReduceArgs job[REDUCE_QUEUE_MAX];
  int njobs;
  int yoff[REDUCE_QUEUE_MAX + 1];
  unsigned xblocks[REDUCE_QUEUE_MAX];
  int groups[REDUCE_QUEUE_MAX];
  unsigned char tall[REDUCE_QUEUE_MAX];
};
__global__ void __launch_bounds__(256) k_reduce_queue(ReduceQueueArgs q) {
  __shared__ float sh[256];
  int j = 0;   // uniform over the workgroup
  while (j + 1 < q.njobs && (int)blockIdx.y >= q.yoff[j + 1]) ++j;
  if (blockIdx.x >= q.xblocks[j] || (int)blockIdx.z >= q.groups[j]) return;
  const int blk = blockIdx.y - q.yoff[j];
  if (q.tall[j]) reduce_tall(q.job[j], blockIdx.x, blk, blockIdx.z, sh);
  else reduce_wide(q.job[j], blockIdx.x, blk, blockIdx.z);
}

struct ReduceQueue {
  hipStream_t st;
  ReduceQueueArgs q;
};
static thread_local ReduceQueue* tl_reduce_queue = nullptr;

ReduceQueueScope::ReduceQueueScope(hipStream_t st, bool enable) : active_(enable && tl_reduce_queue == nullptr) {
  if (active_) {
    tl_reduce_queue = new ReduceQueue;
    tl_reduce_queue->st = st;
    tl_reduce_queue->q.njobs = 0;
    tl_reduce_queue->q.yoff[0] = 0;
  }
}
ReduceQueueScope::~ReduceQueueScope() {
  if (active_) {
    delete tl_reduce_queue;
    tl_reduce_queue = nullptr;
  }
}
int32_t ReduceQueueScope::flush() {
  if (!active_ || tl_reduce_queue->q.njobs == 0) return HGNN_OK;
  ReduceQueueArgs& q = tl_reduce_queue->q;
  unsigned gx = 1, gz = 1;
  for (int j = 0; j < q.njobs; ++j) {
    gx = q.xblocks[j] > gx ? q.xblocks[j] : gx;
    gz = (unsigned)q.groups[j] > gz ? (unsigned)q.groups[j] : gz;
  }
  k_reduce_queue<<<dim3(gx, (unsigned)q.yoff[q.njobs], gz), 256, 0, tl_reduce_queue->st>>>(q);
  q.njobs = 0;
  HGNN_LAUNCH_CHECK("k_reduce_queue");
  return HGNN_OK;
}

static int32_t launch_reduce_partials_n(hipStream_t st, const float* partial, int nsplit, int nblk, long blk_elems,
                                         float* const* dest, int ndest, int groups, long grp_dest_stride);
int32_t launch_reduce_partials(hipStream_t st, const float* partial, int nsplit, int nblk, long blk_elems,
                               float* const dest[4], int groups, long grp_dest_stride) {
  return launch_reduce_partials_n(st, partial, nsplit, nblk, blk_elems, dest, 4, groups, grp_dest_stride);
}
static int32_t launch_reduce_partials_n(hipStream_t st, const float* partial, int nsplit, int nblk, long blk_elems,
                                         float* const* dest, int ndest, int groups, long grp_dest_stride) {
  ReduceArgs r;
  r.partial = partial;
  r.nsplit = nsplit;
  r.nblk = nblk;
  r.blk_elems = blk_elems;
  for (int i = 0; i < 8; ++i) r.dest[i] = i < ndest ? dest[i] : nullptr;
  r.grp_dest_stride = grp_dest_stride;
  if (tl_reduce_queue && groups >= 1 && groups <= 65535 && tl_reduce_queue->q.njobs < REDUCE_QUEUE_MAX) {
    // collected: runs with the others when the scope is flushed
    ReduceQueueArgs& q = tl_reduce_queue->q;
    const int j = q.njobs++;
    q.job[j] = r;
    q.tall[j] = reduce_is_tall(blk_elems, nsplit) ? 1 : 0;
    q.xblocks[j] = reduce_xblocks(blk_elems, nsplit);
    q.groups[j] = groups;
    q.yoff[j + 1] = q.yoff[j] + nblk;
    return HGNN_OK;
  }
  if (reduce_is_tall(blk_elems, nsplit))
    k_reduce_partials_tall<<<dim3(reduce_xblocks(blk_elems, nsplit), nblk, groups), 256, 0, st>>>(r);
  else
    k_reduce_partials<<<dim3(reduce_xblocks(blk_elems, nsplit), nblk, groups), 256, 0, st>>>(r);
  HGNN_LAUNCH_CHECK("k_reduce_partials");
  return HGNN_OK;
}

// ---------------------------------------------------------------------------------------------
// transposed GEMM
// ---------------------------------------------------------------------------------------------
constexpr int WG_RC = 32;  // rows staged per step

template <int H>
struct WgradCfg {
  static constexpr int OT = H < 128 ? H : 128;  // output tile edge
  static constexpr int WT = OT / 2;             // per-wave edge (2 x 2 wavefronts)
  static constexpr int NB = WT / 32;
  static constexpr int STRIDE = OT + 4;
  static constexpr int TILES = H / OT;
};

// the jobs of one launch: their output tiles are numbered one job after the other (ny_off), so are their blocks in
// the partial buffer (blk_off) and their B operands in the column-sum partials (cs_off)
struct WgradJobs {
  WgradArgs job[3];
  int njobs;
  int ny_off[4], blk_off[4], cs_off[4];
  float* partial;
  float* colsum_partial;
};

template <int H, bool BF16>
__global__ void __launch_bounds__(256, 2) k_wgrad(WgradJobs m, int nsplit, int rows_per_split, int ny) {
  using C = WgradCfg<H>;
  __shared__ __align__(16) float sA[WG_RC * C::STRIDE];
  __shared__ __align__(16) float sB[WG_RC * C::STRIDE];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wa = wave >> 1, wb = wave & 1;
  // Workgroups are dealt to the 8 XCDs round-robin. The ny workgroups that read the same rows (one per output tile)
  // take consecutive places on one XCD, so that they run at the same time behind the same L2 and the rows come
  // from memory once: split s lives on XCD s % 8.
  const int xcd = blockIdx.x & 7, place = blockIdx.x >> 3;
  const int split = (place / ny) * 8 + xcd, grp = blockIdx.z;
  if (split >= nsplit) return;   // uniform over the workgroup (the grid is padded to whole groups of 8 splits)
  int y = place % ny;
  int jb = 0;   // uniform over the workgroup
  if (m.njobs > 1 && y >= m.ny_off[1]) jb = 1;
  if (m.njobs > 2 && y >= m.ny_off[2]) jb = 2;
  y -= m.ny_off[jb];
  const WgradArgs& p = m.job[jb];
  const int tb = y % C::TILES; y /= C::TILES;
  const int ta = y % C::TILES; y /= C::TILES;
  const int ib = y % p.nB;
  const int ia = y / p.nB;
  const int blkid = ia * p.nB + ib;
  long gbeg = 0, gend = p.M;
  if (p.grp_ptr) { gbeg = p.grp_ptr[grp]; gend = p.grp_ptr[grp + 1]; }
  long rbeg = gbeg + (long)split * rows_per_split;
  long rend = rbeg + rows_per_split;
  if (rend > gend) rend = gend;

  f32x16_t acc[C::NB][C::NB];
#pragma unroll
  for (int i = 0; i < C::NB; ++i)
#pragma unroll
    for (int j = 0; j < C::NB; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const float* __restrict__ A = p.A[ia];
  const float* __restrict__ B = p.B[ib];
  const int lda = p.lda[ia], ldb = p.ldb[ib];
  constexpr int CH = C::OT / 4;
  constexpr int ITER = WG_RC * CH / 256;   // 1, 2 or 4
  // the rows of step r0 (clamped to the last valid row; rows past the end are zeroed when they are staged). The
  // row indices are read first, under one uniform branch: with the test inside the loop every load waited for the
  // one before it.
  auto fetch = [&](long r0, float4 (&va)[ITER], float4 (&vb)[ITER]) {
    long gr[ITER];
#pragma unroll
    for (int u = 0; u < ITER; ++u) {
      const long pos = r0 + (tid + u * 256) / CH;
      gr[u] = pos < rend ? pos : rend - 1;
    }
    if (p.row_idx) {
#pragma unroll
      for (int u = 0; u < ITER; ++u) gr[u] = p.row_idx[gr[u]];
    }
#pragma unroll
    for (int u = 0; u < ITER; ++u) {
      const int q = (tid + u * 256) % CH;
      va[u] = *reinterpret_cast<const float4*>(A + gr[u] * lda + ta * C::OT + q * 4);
      vb[u] = *reinterpret_cast<const float4*>(B + gr[u] * ldb + tb * C::OT + q * 4);
    }
  };
  // column sums of this workgroup's B tile ride along where they are asked for (one workgroup per B tile: the
  // one of the first A block and the first A tile); a thread's chunk column is the same at every step
  const bool do_cs = m.colsum_partial != nullptr && (p.colsum_dest[0] || p.colsum_dest[1]) && ia == 0 && ta == 0;
  static_assert(256 % CH == 0, "a thread keeps its chunk column over the steps");
  float4 cs = make_float4(0.f, 0.f, 0.f, 0.f);
  // one step: the rows held in va / vb go to LDS, the registers are refilled with the rows two steps on (they travel
  // while this step and the next are multiplied), then the product
  auto step = [&](long r0, float4 (&va)[ITER], float4 (&vb)[ITER]) {
    __syncthreads();
#pragma unroll
    for (int u = 0; u < ITER; ++u) {
      const int c = tid + u * 256;
      const int r = c / CH, q = c - r * CH;
      float4 a = va[u], b = vb[u];
      if (p.a_silu) { a.x = silu_f(a.x); a.y = silu_f(a.y); a.z = silu_f(a.z); a.w = silu_f(a.w); }
      if (r0 + r >= rend) { a = make_float4(0.f, 0.f, 0.f, 0.f); b = a; }
      cs.x += b.x; cs.y += b.y; cs.z += b.z; cs.w += b.w;
      *reinterpret_cast<float4*>(&sA[r * C::STRIDE + q * 4]) = a;
      *reinterpret_cast<float4*>(&sB[r * C::STRIDE + q * 4]) = b;
    }
    if (r0 + 2 * WG_RC < rend) fetch(r0 + 2 * WG_RC, va, vb);
    __syncthreads();
    if (BF16) {
#pragma unroll
      for (int ks = 0; ks < WG_RC / 16; ++ks) {
        const int rr = ks * 16 + (lane >> 5) * 8;
        bf16x8_t a[C::NB], b[C::NB];
#pragma unroll
        for (int i = 0; i < C::NB; ++i) {
          const int ca = wa * C::WT + i * 32 + (lane & 31);
          const int cbb = wb * C::WT + i * 32 + (lane & 31);
          unsigned ua[4], ub[4];
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            ua[t] = pack_bf16x2(sA[(rr + 2 * t) * C::STRIDE + ca], sA[(rr + 2 * t + 1) * C::STRIDE + ca]);
            ub[t] = pack_bf16x2(sB[(rr + 2 * t) * C::STRIDE + cbb], sB[(rr + 2 * t + 1) * C::STRIDE + cbb]);
          }
          uint4 pa = make_uint4(ua[0], ua[1], ua[2], ua[3]);
          uint4 pb = make_uint4(ub[0], ub[1], ub[2], ub[3]);
          a[i] = *reinterpret_cast<bf16x8_t*>(&pa);
          b[i] = *reinterpret_cast<bf16x8_t*>(&pb);
        }
#pragma unroll
        for (int i = 0; i < C::NB; ++i)
#pragma unroll
          for (int j = 0; j < C::NB; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
      }
    } else {
#pragma unroll
      for (int ks = 0; ks < WG_RC / 2; ++ks) {
        const int rr = ks * 2 + (lane >> 5);
        float a[C::NB], b[C::NB];
#pragma unroll
        for (int i = 0; i < C::NB; ++i) {
          a[i] = sA[rr * C::STRIDE + wa * C::WT + i * 32 + (lane & 31)];
          b[i] = sB[rr * C::STRIDE + wb * C::WT + i * 32 + (lane & 31)];
        }
#pragma unroll
        for (int i = 0; i < C::NB; ++i)
#pragma unroll
          for (int j = 0; j < C::NB; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
      }
    }
  };
  float4 va0[ITER], vb0[ITER], va1[ITER], vb1[ITER];
  if (rbeg < rend) fetch(rbeg, va0, vb0);
  if (rbeg + WG_RC < rend) fetch(rbeg + WG_RC, va1, vb1);
  for (long r0 = rbeg; r0 < rend; r0 += 2 * WG_RC) {
    step(r0, va0, vb0);
    if (r0 + WG_RC < rend) step(r0 + WG_RC, va1, vb1);
  }
  if (do_cs) {   // uniform over the workgroup: row phases are added in order through LDS
    __syncthreads();
    float4* sh = reinterpret_cast<float4*>(sA);
    sh[tid] = cs;
    __syncthreads();
    if (tid < CH) {
      float4 s = sh[tid];
      for (int k = 1; k < 256 / CH; ++k) {
        const float4 t = sh[k * CH + tid];
        s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
      }
      *reinterpret_cast<float4*>(m.colsum_partial + (((long)grp * nsplit + split) * m.cs_off[m.njobs] + m.cs_off[jb] + ib) * H + tb * C::OT + tid * 4) = s;
    }
  }
  const int nblk = m.blk_off[m.njobs];
  float* out = m.partial + (((long)grp * nsplit + split) * nblk + m.blk_off[jb] + blkid) * (long)(H * H);
#pragma unroll
  for (int i = 0; i < C::NB; ++i)
#pragma unroll
    for (int j = 0; j < C::NB; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int k1 = ta * C::OT + wa * C::WT + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        const int k2 = tb * C::OT + wb * C::WT + j * 32 + (lane & 31);
        out[k1 * H + k2] = acc[i][j][v];
      }
}

int wgrad_splits(int64_t M) {
  int64_t s = (M + 63) / 64;   // about 64 rows per split (two steps): short chains when there are few atoms
  if (s < 1) s = 1;
  if (s > 160) s = 160;
  return (int)s;
}

size_t wgrad_colsum_partial_floats(int H, int64_t M) { return (size_t)wgrad_splits(M) * 4 * H; }

size_t wgrad_partial_floats(int H, int64_t M, int nblocks, int S) {
  return (size_t)wgrad_splits(M) * nblocks * S * H * H;
}

// workgroups of k_wgrad that one CU holds at a time (asked once per variant)
template <int H, bool BF16>
static int wgrad_resident_wgs() {
  static int n = 0;
  if (n == 0) {
    int occ = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, reinterpret_cast<const void*>(&k_wgrad<H, BF16>), 256, 0) !=
            hipSuccess || occ < 1)
      occ = 1;
    n = occ;
  }
  return n;
}

template <int H, bool BF16>
static int32_t launch_wgrad_t(hipStream_t st, const WgradArgs* jobs, int njobs) {
  using C = WgradCfg<H>;
  const WgradArgs& a = jobs[0];
  WgradJobs m;
  m.njobs = njobs;
  m.partial = a.partial;
  m.colsum_partial = nullptr;
  m.ny_off[0] = m.blk_off[0] = m.cs_off[0] = 0;
  for (int j = 0; j < njobs; ++j) {
    m.job[j] = jobs[j];
    m.ny_off[j + 1] = m.ny_off[j] + jobs[j].nA * jobs[j].nB * C::TILES * C::TILES;
    m.blk_off[j + 1] = m.blk_off[j] + jobs[j].nA * jobs[j].nB;
    m.cs_off[j + 1] = m.cs_off[j] + jobs[j].nB;
    if (jobs[j].colsum_dest[0] || jobs[j].colsum_dest[1]) m.colsum_partial = a.colsum_partial;
  }
  for (int j = njobs; j < 3; ++j) m.ny_off[j + 1] = m.blk_off[j + 1] = m.cs_off[j + 1] = 0;
  const int nblk = m.blk_off[njobs];
  const int groups = a.grp_ptr ? a.S : 1;
  const int ny = m.ny_off[njobs];
  // Splits: never more than the workspace was sized for, and at most one round of resident workgroups (a second,
  // partly filled round costs a whole one). Split s runs on XCD s % 8, so the round is counted per XCD: a whole
  // number of splits on each of them (25 splits of 20 workgroups put 80 workgroups on the first XCD's 64 places
  // and doubled the kernel's time). Below one round: a whole number of workgroups per CU, so that no CU carries two
  // while its neighbour carries one. Fewer splits also mean fewer partials to write and add up.
  int nsplit = wgrad_splits(a.M);
  const long per_split = (long)ny * groups;
  const long xcd_places = (long)wgrad_resident_wgs<H, BF16>() * (num_cus() / 8);
  const long one_round = xcd_places / per_split >= 1 ? 8 * (xcd_places / per_split)
                                                     : (long)wgrad_resident_wgs<H, BF16>() * num_cus() / per_split;
  if (nsplit > one_round) {
    nsplit = one_round < 1 ? 1 : (int)one_round;
  } else {
    const long whole = nsplit * per_split / num_cus();
    if (whole >= 1) nsplit = (int)(whole * num_cus() / per_split);
  }
  if (nsplit < 1) nsplit = 1;   // many groups with few rows each: per_split alone can exceed the CU count
  int64_t rps = (a.M + nsplit - 1) / nsplit;
  rps = (rps + WG_RC - 1) / WG_RC * WG_RC;
  if (rps < WG_RC) rps = WG_RC;
  ProfScope ps(a.tag, st);
  k_wgrad<H, BF16><<<dim3((unsigned)((nsplit + 7) / 8 * 8 * ny), 1, groups), 256, 0, st>>>(m, nsplit, (int)rps, ny);
  HGNN_LAUNCH_CHECK("k_wgrad");
  float* dest[8] = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
  float* cd[4] = {nullptr, nullptr, nullptr, nullptr};
  for (int j = 0; j < njobs; ++j) {
    for (int b = 0; b < jobs[j].nA * jobs[j].nB; ++b) dest[m.blk_off[j] + b] = jobs[j].dest[b];
    for (int b = 0; b < jobs[j].nB; ++b) cd[m.cs_off[j] + b] = jobs[j].colsum_dest[b];
  }
  HGNN_TRY(launch_reduce_partials_n(st, m.partial, nsplit, nblk, (long)H * H, dest, 8, groups, a.grp_dest_stride));
  if (m.colsum_partial) HGNN_TRY(launch_reduce_partials_n(st, m.colsum_partial, nsplit, m.cs_off[njobs], H, cd, 4, 1, 0));
  return HGNN_OK;
}

int32_t launch_wgrad_multi(hipStream_t st, int H, bool bf16, const WgradArgs* jobs, int njobs) {
  HGNN_REQUIRE(jobs && njobs >= 1 && njobs <= 3, HGNN_ERR_BAD_SHAPE, "wgrad: one to three jobs");
  int blocks = 0, nb = 0;
  for (int j = 0; j < njobs; ++j) {
    const WgradArgs& a = jobs[j];
    HGNN_REQUIRE(a.nA >= 1 && a.nB >= 1 && a.nA * a.nB <= 4, HGNN_ERR_BAD_SHAPE, "wgrad: bad block counts");
    HGNN_REQUIRE(a.A[0] && a.B[0] && a.dest[0], HGNN_ERR_NULLPTR, "wgrad: null operand");
    HGNN_REQUIRE(!(a.colsum_dest[0] || a.colsum_dest[1]) || jobs[0].colsum_partial, HGNN_ERR_NULLPTR, "wgrad: no room for the column sums");
    HGNN_REQUIRE(njobs == 1 || (!a.grp_ptr && !a.row_idx && a.M == jobs[0].M), HGNN_ERR_BAD_SHAPE,
                 "wgrad: several jobs share their rows (no groups, no row indirection)");
    blocks += a.nA * a.nB;
    nb += a.nB;
  }
  HGNN_REQUIRE(jobs[0].partial, HGNN_ERR_NULLPTR, "wgrad: null partial buffer");
  HGNN_REQUIRE(blocks <= 8 && nb <= 4, HGNN_ERR_BAD_SHAPE, "wgrad: too many blocks in one launch");
  HGNN_REQUIRE(!(jobs[0].colsum_partial && (jobs[0].colsum_dest[0] || jobs[0].colsum_dest[1])) || !jobs[0].grp_ptr,
               HGNN_ERR_BAD_SHAPE, "wgrad: column sums are not available per group");
  switch (H) {
    case 64: return bf16 ? launch_wgrad_t<64, true>(st, jobs, njobs) : launch_wgrad_t<64, false>(st, jobs, njobs);
    case 128: return bf16 ? launch_wgrad_t<128, true>(st, jobs, njobs) : launch_wgrad_t<128, false>(st, jobs, njobs);
    case 256: return bf16 ? launch_wgrad_t<256, true>(st, jobs, njobs) : launch_wgrad_t<256, false>(st, jobs, njobs);
  }
  return set_error(HGNN_ERR_BAD_SHAPE, "H must be 64, 128 or 256 (got %d)", H);
}

int32_t launch_wgrad(hipStream_t st, int H, bool bf16, const WgradArgs& a) { return launch_wgrad_multi(st, H, bf16, &a, 1); }

// ---------------------------------------------------------------------------------------------
// column sums
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_colsum(ColsumArgs p, int H, int nsplit, int rows_per_split) {
  // thread = (4-column chunk q, row phase ph); every phase walks its rows with four loads in flight
  __shared__ float4 sh[256];
  const int tid = threadIdx.x;
  const int CH = H >> 2;
  const int q = tid % CH, ph = tid / CH, nph = 256 / CH;
  const int split = blockIdx.x, grp = blockIdx.y;
  long gbeg = 0, gend = p.M;
  if (p.grp_ptr) { gbeg = p.grp_ptr[grp]; gend = p.grp_ptr[grp + 1]; }
  long rbeg = gbeg + (long)split * rows_per_split;
  long rend = rbeg + rows_per_split;
  if (rend > gend) rend = gend;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  for (long r0 = rbeg + ph; r0 < rend; r0 += 4 * nph) {
    float4 xv[4];
    float wv[4];
    long gr[4];
    // (indices, rows and weights each under one uniform branch: with the tests inside the loop the loads wait for
    // one another)
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const long r = r0 + (long)u * nph;
      gr[u] = r < rend ? r : rend - 1;
      wv[u] = 1.f;
    }
    if (p.row_idx) {
#pragma unroll
      for (int u = 0; u < 4; ++u) gr[u] = p.row_idx[gr[u]];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) xv[u] = *reinterpret_cast<const float4*>(p.X + gr[u] * p.ldx + q * 4);
    if (p.w) {
#pragma unroll
      for (int u = 0; u < 4; ++u) wv[u] = p.w[gr[u]];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (r0 + (long)u * nph >= rend) wv[u] = 0.f;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      float4 x = xv[u];
      if (p.f_silu) { x.x = silu_f(x.x); x.y = silu_f(x.y); x.z = silu_f(x.z); x.w = silu_f(x.w); }
      s.x += wv[u] * x.x; s.y += wv[u] * x.y; s.z += wv[u] * x.z; s.w += wv[u] * x.w;
    }
  }
  sh[tid] = s;
  __syncthreads();
  if (ph == 0) {
    for (int k = 1; k < nph; ++k) {
      const float4 t = sh[k * CH + q];
      s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
    }
    *reinterpret_cast<float4*>(p.partial + ((long)grp * nsplit + split) * H + q * 4) = s;
  }
}

static int colsum_splits(int64_t M) {
  int64_t s = (M + 63) / 64;   // 64 rows per workgroup: four trips of loads each (at 256 rows a workgroup's chain of trips set the kernel's time)
  if (s < 1) s = 1;
  if (s > 1024) s = 1024;
  return (int)s;
}

size_t colsum_partial_floats(int H, int64_t M, int S) { return (size_t)colsum_splits(M) * S * H; }

int32_t launch_colsum(hipStream_t st, int H, const ColsumArgs& a) {
  HGNN_REQUIRE(a.X && a.dest && a.partial, HGNN_ERR_NULLPTR, "colsum: null operand");
  HGNN_REQUIRE(valid_H(H), HGNN_ERR_BAD_SHAPE, "H must be 64, 128 or 256 (got %d)", H);
  const int nsplit = colsum_splits(a.M);
  int64_t rps = (a.M + nsplit - 1) / nsplit;
  if (rps < 1) rps = 1;
  const int groups = a.grp_ptr ? a.S : 1;
  ProfScope ps(PT_COLSUM, st);
  k_colsum<<<dim3(nsplit, groups), 256, 0, st>>>(a, H, nsplit, (int)rps);
  HGNN_LAUNCH_CHECK("k_colsum");
  float* dest[4] = {a.dest, nullptr, nullptr, nullptr};
  return launch_reduce_partials(st, a.partial, nsplit, 1, H, dest, groups, a.grp_dest_stride);
}

}  // namespace hgnn
