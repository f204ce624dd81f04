// Fused per-edge kernels (see edge_fused.h for the fragment-order layouts).
//
//   k_edge_fwd    gather P[dst]+Q[col]+d2*w1d -> SiLU -> (A tile in LDS) x W2 on the matrix cores -> z2
//   k_seg_fwd_vm  destination-sorted segmented reduction of SiLU(z2) into M and the vector channel
//   k_edge_bwd    g_z2 from z2 / g_M / g_v -> x W2^T -> recompute z1 -> g_z1, plus the three per-column
//                 sums that are bias / vector gradients
//   k_wgrad_frag  g_W2 = a1^T g_z2 streamed straight from memory into matrix-core operands
//   k_wgrad_frag_rc  the same with a1 recomputed from the projected node features (bf16 pairs), so that the
//                 forward kernel need not store it
//   k_segsum_vm   segmented sums of g_z1 per destination and (through the transpose plan) per source
//
// All element-wise work uses the accumulator mapping (lane <-> column, register <-> edge), so what one
// kernel stores is what the next one loads, coalesced, without any transpose. Every sum has a fixed
// order; there are no atomics.
#include <type_traits>

#include "devmath.h"
#include "edge_fused.h"
#include "gemm.h"

namespace hgnn {

// largest edge count the 32-bit edge indices of these kernels reach (a whole tile beyond E must still fit)
constexpr int64_t EDGE_MAX_E = 2147483647LL - 128;

template <int H, bool BF16>
struct ECfg {
  static constexpr int TM = 64;                       // edges per tile
  static constexpr int NCB = H / 32;                  // 32-column blocks
  static constexpr int WC = NCB < 4 ? NCB : 4;        // wavefronts over columns
  static constexpr int WR = 4 / WC;                   // wavefronts over rows
  static constexpr int RB = (TM / 32) / WR;           // 32-row blocks per wavefront
  static constexpr int CB = NCB / WC;                 // 32-column blocks per wavefront
  static constexpr int STRIDE = BF16 ? H + 8 : H + 4; // LDS row pitch (elements)
  static constexpr size_t LDS_BYTES = (size_t)TM * STRIDE * (BF16 ? 2 : 4);
};

__device__ __forceinline__ float bf_bits_to_f(unsigned short b) { return __uint_as_float(((unsigned)b) << 16); }

// Streaming accesses are written as (uniform 64-bit base) + (32-bit per-lane byte offset): the base lives in scalar
// registers, the lane part is one register shared by every access, and constant strides fold into the instruction.
template <typename T>
__device__ __forceinline__ T ldg_nt(const void* ubase, unsigned off) {
  return __builtin_nontemporal_load(reinterpret_cast<const T*>(reinterpret_cast<const char*>(ubase) + off));
}
template <typename T>
__device__ __forceinline__ T ldg_at(const void* ubase, unsigned off) {
  return *reinterpret_cast<const T*>(reinterpret_cast<const char*>(ubase) + off);
}
template <typename T>
__device__ __forceinline__ void stg_nt(void* ubase, unsigned off, T v) {
  __builtin_nontemporal_store(v, reinterpret_cast<T*>(reinterpret_cast<char*>(ubase) + off));
}
__device__ __forceinline__ const char* uoff(const void* base, size_t bytes) { return reinterpret_cast<const char*>(base) + bytes; }
__device__ __forceinline__ char* uoff(void* base, size_t bytes) { return reinterpret_cast<char*>(base) + bytes; }

// 8 accumulator-mapped values of one half of a 32x32 block (column n of the tile, registers v = 8*vh .. 8*vh+7,
// rows rbase + 8*(v>>2) + 4g + (v&3)): written row-major into the LDS tile and, operand-packed, to memory.
// bf16 values are converted once. packed == null: only the LDS tile is written.
template <bool BF16, int STRIDE>
__device__ __forceinline__ void emit_half(unsigned char* smem, int rbase, int g, int n, const float* vals, int vh,
                                          void* packed, size_t blk, int lane) {
  if (BF16) {
    unsigned pk[4];
    unsigned short* s16 = reinterpret_cast<unsigned short*>(smem);
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      pk[t] = pack_bf16x2(vals[2 * t], vals[2 * t + 1]);
      const int row = rbase + 8 * (2 * vh + (t >> 1)) + 4 * g + 2 * (t & 1);
      s16[row * STRIDE + n] = (unsigned short)(pk[t] & 0xffffu);
      s16[(row + 1) * STRIDE + n] = (unsigned short)(pk[t] >> 16);
    }
    {
      typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
      const u32x4_t w = {pk[0], pk[1], pk[2], pk[3]};
      if (packed) stg_nt<u32x4_t>(uoff(packed, (blk * 2 + vh) * 1024), lane * 16u, w);
    }
  } else {
    float* s32 = reinterpret_cast<float*>(smem);
#pragma unroll
    for (int u = 0; u < 8; ++u) s32[(rbase + 8 * (2 * vh + (u >> 2)) + 4 * g + (u & 3)) * STRIDE + n] = vals[u];
    char* pb = uoff(packed, (blk * 4 + 2 * vh) * 1024);
    const f32x4_t w0 = {vals[0], vals[1], vals[2], vals[3]};
    const f32x4_t w1 = {vals[4], vals[5], vals[6], vals[7]};
    if (packed) {
      stg_nt<f32x4_t>(pb, lane * 16u, w0);
      stg_nt<f32x4_t>(pb, lane * 16u + 1024u, w1);
    }
  }
}

// persistent tile loop that keeps each XCD (workgroups are dealt to the 8 XCDs round-robin) on its own
// contiguous eighth of the tiles, so that the node rows an XCD gathers stay in that XCD's L2
struct TileRange {
  int first, end, step;
};
__device__ __forceinline__ TileRange xcd_tile_range(int ntiles) {
  const int G = gridDim.x;
  if ((G & 7) != 0 || ntiles < 64) return {(int)blockIdx.x, ntiles, G};
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int per = (ntiles + 7) >> 3;
  const int lo = xcd * per;
  const int hi = lo + per < ntiles ? lo + per : ntiles;
  return {lo + slot, hi, G >> 3};
}

// The B fragments of the first steps of a tile product, asked for before the workgroup meets at the barrier in front of
// the product: a wavefront's B stream is a chain of L2 round trips, and with loads issued only where they are used
// every pair of steps waited for one of them. The fragments come through buffer loads (resource in scalar registers,
// one per-lane offset register, the fragment's offset in a scalar register), so that no per-fragment 64-bit address
// lives in vector registers.
typedef unsigned u32x4_buf_t __attribute__((ext_vector_type(4)));
template <int H, bool BF16>
struct BRing {
  static constexpr int NKB = H / 16;
  static constexpr int D = BF16 ? (NKB < 4 ? NKB : 4) : 2;   // steps in flight
  static constexpr int P = BF16 ? 1 : 3;                      // planes of B (fp32 operands: three bf16 terms)
  bf16x8_t b[D][ECfg<H, BF16>::CB][P];
  __amdgpu_buffer_rsrc_t rsrc;
  unsigned lo;   // lane offset in bytes
};
template <int H, bool BF16>
__device__ __forceinline__ void tile_b_load(BRing<H, BF16>& ring, int wc, int kb,
                                            bf16x8_t (&o)[ECfg<H, BF16>::CB][BRing<H, BF16>::P]) {
  using C = ECfg<H, BF16>;
#pragma unroll
  for (int j = 0; j < C::CB; ++j)
#pragma unroll
    for (int q = 0; q < BRing<H, BF16>::P; ++q)
      o[j][q] = __builtin_bit_cast(bf16x8_t, __builtin_amdgcn_raw_buffer_load_b128(
                                                 ring.rsrc, ring.lo, q * (H * H * 2) + ((wc * C::CB + j) * (H / 16) + kb) * 1024, 0));
}
// Bpacked: the packed H x H block (bf16: H * H * 2 bytes; fp32 operands: three such planes)
template <int H, bool BF16>
__device__ __forceinline__ void tile_mma_prefetch(const void* Bpacked, int wc, int lane, BRing<H, BF16>& ring) {
  ring.rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(Bpacked), 0, BRing<H, BF16>::P * H * H * 2, 0x00020000);
  ring.lo = lane * 16u;
  asm volatile("" : "+v"(ring.lo));   // kept as one register: not folded into per-fragment addresses
#pragma unroll
  for (int d = 0; d < BRing<H, BF16>::D; ++d) tile_b_load<H, BF16>(ring, wc, d, ring.b[d]);
}

// A tile (LDS, row-major, padded) x packed B block -> accumulators; same tiling as the row-tile GEMM.
// The accumulators start from zero (the first step feeds a constant zero, so they need no clearing).
// bf16: ring holds the B fragments of the first D steps (tile_mma_prefetch); each step asks for those of step + D.
template <int H, bool BF16>
__device__ __forceinline__ void tile_mma(const unsigned char* smem, const void* Bpacked, int wr, int wc, int lane,
                                         f32x16_t (&acc)[ECfg<H, BF16>::RB][ECfg<H, BF16>::CB], BRing<H, BF16>& ring) {
  using C = ECfg<H, BF16>;
  const f32x16_t zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if constexpr (BF16) {
    constexpr int NKB = H / 16;
    constexpr int D = BRing<H, BF16>::D;
    // LDS byte offset of this lane's A fragment of the first row block and step (one register; row blocks and steps
    // are immediate offsets)
    unsigned ao = (unsigned)(((wr * C::RB * 32 + (lane & 31)) * C::STRIDE + (lane >> 5) * 8) * 2);
    asm volatile("" : "+v"(ao));
    bf16x8_t a[2][C::RB];   // A fragments of this step and the next
#pragma unroll
    for (int i = 0; i < C::RB; ++i) a[0][i] = *reinterpret_cast<const bf16x8_t*>(smem + ao + (i * 32 * C::STRIDE) * 2);
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) {
      if (kb + 1 < NKB) {
#pragma unroll
        for (int i = 0; i < C::RB; ++i)
          a[(kb + 1) & 1][i] = *reinterpret_cast<const bf16x8_t*>(smem + ao + (i * 32 * C::STRIDE + (kb + 1) * 16) * 2);
      }
#pragma unroll
      for (int j = 0; j < C::CB; ++j)
#pragma unroll
        for (int i = 0; i < C::RB; ++i)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[kb & 1][i], ring.b[kb % D][j][0], kb == 0 ? zero : acc[i][j], 0, 0, 0);
      if (kb + D < NKB) tile_b_load<H, BF16>(ring, wc, kb + D, ring.b[kb % D]);
      // (without this the scheduler moves every refill down to the step that uses it)
      __builtin_amdgcn_sched_barrier(0);
    }
  } else {
    // fp32 operands: the A tile stays fp32 in LDS and is split into three bf16 terms as it is read; B comes as
    // three bf16 planes (launch_pack_x3); six bf16 products per step of 16 k (see split_bf16x3)
    constexpr int NKB = H / 16;
    constexpr int D = BRing<H, BF16>::D;
    unsigned ao = (unsigned)(((wr * C::RB * 32 + (lane & 31)) * C::STRIDE + (lane >> 5) * 8) * 4);
    asm volatile("" : "+v"(ao));
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) {
      bf16x8_t a[C::RB][3];
#pragma unroll
      for (int i = 0; i < C::RB; ++i) {
        const unsigned char* ap = smem + ao + (i * 32 * C::STRIDE + kb * 16) * 4;
        const float4 lo = *reinterpret_cast<const float4*>(ap), hi = *reinterpret_cast<const float4*>(ap + 16);
        const float x[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
        split_bf16x3(x, a[i]);
      }
#pragma unroll
      for (int j = 0; j < C::CB; ++j)
#pragma unroll
        for (int i = 0; i < C::RB; ++i) acc[i][j] = mfma_bf16x3(a[i], ring.b[kb % D][j], kb == 0 ? zero : acc[i][j]);
      if (kb + D < NKB) tile_b_load<H, BF16>(ring, wc, kb + D, ring.b[kb % D]);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
}

// Same product with this wavefront's slice of B held in registers for the whole kernel.
template <int H, bool BF16>
struct BFrag {
  using type = float4;
  static constexpr int NKB = H / 8;
};
template <int H>
struct BFrag<H, true> {
  using type = bf16x8_t;
  static constexpr int NKB = H / 16;
};

template <int H, bool BF16>
__device__ __forceinline__ void load_b_resident(const void* Bpacked, int wc, int lane,
                                                typename BFrag<H, BF16>::type (&breg)[BFrag<H, BF16>::NKB][ECfg<H, BF16>::CB]) {
  using C = ECfg<H, BF16>;
  using T = typename BFrag<H, BF16>::type;
  constexpr int NKB = BFrag<H, BF16>::NKB;
  const T* __restrict__ Bp = reinterpret_cast<const T*>(Bpacked);
#pragma unroll
  for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
    for (int j = 0; j < C::CB; ++j) breg[kb][j] = Bp[((wc * C::CB + j) * NKB + kb) * 64 + lane];
}

template <int H, bool BF16>
__device__ __forceinline__ void tile_mma_res(const unsigned char* smem, int wr, int lane,
                                             const typename BFrag<H, BF16>::type (&breg)[BFrag<H, BF16>::NKB][ECfg<H, BF16>::CB],
                                             f32x16_t (&acc)[ECfg<H, BF16>::RB][ECfg<H, BF16>::CB]) {
  using C = ECfg<H, BF16>;
  constexpr int NKB = BFrag<H, BF16>::NKB;
#pragma unroll
  for (int kb = 0; kb < NKB; ++kb) {
    if constexpr (BF16) {
      bf16x8_t a[C::RB];
#pragma unroll
      for (int i = 0; i < C::RB; ++i) {
        const int row = (wr * C::RB + i) * 32 + (lane & 31);
        a[i] = *reinterpret_cast<const bf16x8_t*>(smem + ((size_t)row * C::STRIDE + kb * 16 + (lane >> 5) * 8) * 2);
      }
#pragma unroll
      for (int j = 0; j < C::CB; ++j)
#pragma unroll
        for (int i = 0; i < C::RB; ++i)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], breg[kb][j], acc[i][j], 0, 0, 0);
    } else {
      float4 a[C::RB];
#pragma unroll
      for (int i = 0; i < C::RB; ++i) {
        const int row = (wr * C::RB + i) * 32 + (lane & 31);
        a[i] = *reinterpret_cast<const float4*>(smem + ((size_t)row * C::STRIDE + kb * 8 + (lane >> 5) * 4) * 4);
      }
#pragma unroll
      for (int j = 0; j < C::CB; ++j)
#pragma unroll
        for (int i = 0; i < C::RB; ++i) {
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i].x, breg[kb][j].x, acc[i][j], 0, 0, 0);
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i].y, breg[kb][j].y, acc[i][j], 0, 0, 0);
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i].z, breg[kb][j].z, acc[i][j], 0, 0, 0);
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i].w, breg[kb][j].w, acc[i][j], 0, 0, 0);
        }
    }
  }
}

// Per-edge scalars of a tile, fetched one tile ahead into LDS: element tid of [NARR][TM] with arrays
// dst | col | d2 bits (| c bits); zeros beyond the last edge (row 0 is always a valid row to gather)
template <int TM, int NARR>
__device__ __forceinline__ int fetch_edge_scalar(const int32_t* __restrict__ dst, const int32_t* __restrict__ col,
                                                 const float* __restrict__ d2, const float* __restrict__ cvec, int tile,
                                                 int tile_end, int E, int tid) {
  const int which = tid / TM, r = tid - which * TM;
  const int e = tile * TM + r;
  if (which >= NARR || tile >= tile_end || e >= E) return 0;
  switch (which) {
    case 0: return dst[e];
    case 1: return col[e];
    case 2: return d2 ? __float_as_int(d2[e]) : 0;
    default: return __float_as_int(cvec[e]);
  }
}

// Loads at a 32-bit byte offset from a uniform base: one address register per lane and no 64-bit arithmetic.
// (The host checks that every gathered node tensor is smaller than 4 GiB.)
__device__ __forceinline__ unsigned ldg_u32(const void* base, unsigned byte_off) {
  return *reinterpret_cast<const unsigned*>(reinterpret_cast<const char*>(base) + byte_off);
}
__device__ __forceinline__ float ldg_f32(const void* base, unsigned byte_off) {
  return *reinterpret_cast<const float*>(reinterpret_cast<const char*>(base) + byte_off);
}

// Row pitch in bytes of the projected features [P | Q]: H words of bf16 pairs, or 2H floats
template <int H, bool PAIRS>
struct PQPitch {
  static constexpr unsigned ROW = PAIRS ? H * 4u : 2u * H * 4u;
  static constexpr unsigned QOFF = PAIRS ? H * 2u : H * 4u;   // byte offset of the Q half inside a row
};

// z1 = P[dst] + Q[col] + d2*w1d for 8 edges and this lane's CB column blocks. colb = byte offset of this
// lane's first column inside the P half of a row.
// PAIRS: the projected features are stored as bf16 pairs, one 32-bit word holding this lane's two
// columns (block 2*wc and block 2*wc+1) of P or Q; a row is [H/2 words of P | H/2 words of Q].
template <int H, int CB, bool PAIRS>
__device__ __forceinline__ void gather_z1(const void* __restrict__ PQ, const int* di, const int* ci, const float* dd,
                                          const float* w1d, unsigned colb, float (&z)[CB][8]) {
  using P = PQPitch<H, PAIRS>;
  if constexpr (PAIRS) {
    static_assert(CB == 2, "pair storage needs two column blocks per lane");
    unsigned wp[8], wq[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      wp[u] = ldg_u32(PQ, (unsigned)di[u] * P::ROW + colb);
      wq[u] = ldg_u32(PQ, (unsigned)ci[u] * P::ROW + colb + P::QOFF);
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      z[0][u] = __uint_as_float(wp[u] << 16) + __uint_as_float(wq[u] << 16) + dd[u] * w1d[0];
      z[1][u] = __uint_as_float(wp[u] & 0xffff0000u) + __uint_as_float(wq[u] & 0xffff0000u) + dd[u] * w1d[1];
    }
  } else {
#pragma unroll
    for (int j = 0; j < CB; ++j) {
      float a[8], b[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        a[u] = ldg_f32(PQ, (unsigned)di[u] * P::ROW + colb + j * 128u);
        b[u] = ldg_f32(PQ, (unsigned)ci[u] * P::ROW + colb + j * 128u + P::QOFF);
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) z[j][u] = a[u] + b[u] + dd[u] * w1d[j];
    }
  }
}

// the 8 per-edge scalars of rows rblk*32 + 8*(2*vh + jj) + 4*g + ii (jj < 2, ii < 4) from an LDS array
__device__ __forceinline__ void lds_rows8(const int* s, int rblk, int vh, int g, int* o) {
#pragma unroll
  for (int jj = 0; jj < 2; ++jj) {
    const int4 t = *reinterpret_cast<const int4*>(s + rblk * 32 + 8 * (2 * vh + jj) + 4 * g);
    o[4 * jj + 0] = t.x; o[4 * jj + 1] = t.y; o[4 * jj + 2] = t.z; o[4 * jj + 3] = t.w;
  }
}
__device__ __forceinline__ void lds_rows8(const int* s, int rblk, int vh, int g, float* o) {
#pragma unroll
  for (int jj = 0; jj < 2; ++jj) {
    const float4 t = *reinterpret_cast<const float4*>(s + rblk * 32 + 8 * (2 * vh + jj) + 4 * g);
    o[4 * jj + 0] = t.x; o[4 * jj + 1] = t.y; o[4 * jj + 2] = t.z; o[4 * jj + 3] = t.w;
  }
}
// bit u set <=> edge eb*32 + 8*(2*vh + (u>>2)) + 4*g + (u&3) exists
__device__ __forceinline__ unsigned rows8_mask(int eb, int vh, int g, int E) {
  unsigned ok = 0;
#pragma unroll
  for (int u = 0; u < 8; ++u) ok |= (eb * 32 + 8 * (2 * vh + (u >> 2)) + 4 * g + (u & 3) < E ? 1u : 0u) << u;
  return ok;
}

// ---------------------------------------------------------------------------------------------
// k > 1 edge attributes (bf16 operands): the term attr_e . W1a of z1 is one matrix-core step per 32 x 32 block
// ([32 edges x 16 attribute slots] x [16 x 32 columns]) out of a bf16 copy of the tile's attributes in LDS, in the
// accumulator mapping in which z1 is formed anyway. Attribute slots beyond k hold zeros.
// ---------------------------------------------------------------------------------------------
constexpr int ATTR_K = 16;                        // attribute slots per edge in LDS
constexpr int ATTR_TILE = 64 * ATTR_K;            // bf16 elements of one tile's attributes, [64 edges][16]
constexpr int ATTR_T_PITCH = 72;                  // row pitch of the transposed copy [16][64 edges] (reverse kernel)
constexpr int ATTR_T_TILE = ATTR_K * ATTR_T_PITCH;

// thread tid's share of a tile's attributes: edge tid/4, slots 4*(tid%4) .. +3, as two bf16 pairs (zeros beyond E / k)
__device__ __forceinline__ uint2 fetch_attr4(const float* __restrict__ attr, int k, int tile, int tile_end, int E, int tid) {
  const int row = tid >> 2, q = tid & 3;
  const int e = tile * 64 + row;
  float a[4] = {0.f, 0.f, 0.f, 0.f};
  if (tile < tile_end && e < E) {
#pragma unroll
    for (int t = 0; t < 4; ++t)
      if (4 * q + t < k) a[t] = attr[(size_t)e * k + 4 * q + t];
  }
  return make_uint2(pack_bf16x2(a[0], a[1]), pack_bf16x2(a[2], a[3]));
}
__device__ __forceinline__ void store_attr4(unsigned short* at, int tid, uint2 v) {
  *reinterpret_cast<uint2*>(at + (tid >> 2) * ATTR_K + 4 * (tid & 3)) = v;
}
// the same four values into the transposed copy: slot-major, edges contiguous
__device__ __forceinline__ void store_attr4_t(unsigned short* att, int tid, uint2 v) {
  const int row = tid >> 2, q = tid & 3;
  att[(4 * q + 0) * ATTR_T_PITCH + row] = (unsigned short)(v.x & 0xffffu);
  att[(4 * q + 1) * ATTR_T_PITCH + row] = (unsigned short)(v.x >> 16);
  att[(4 * q + 2) * ATTR_T_PITCH + row] = (unsigned short)(v.y & 0xffffu);
  att[(4 * q + 3) * ATTR_T_PITCH + row] = (unsigned short)(v.y >> 16);
}
// B operand of the attribute step for this lane's column n: rows 8*(lane>>5) .. +7 of W1a (zeros beyond k)
__device__ __forceinline__ bf16x8_t attr_weight_operand(const float* __restrict__ W1a, int k, int H, int n, int lane) {
  typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
  u32x4_t w;
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int r = (lane >> 5) * 8 + 2 * t;
    const float v0 = r < k ? W1a[(size_t)r * H + n] : 0.f;
    const float v1 = r + 1 < k ? W1a[(size_t)(r + 1) * H + n] : 0.f;
    w[t] = pack_bf16x2(v0, v1);
  }
  return __builtin_bit_cast(bf16x8_t, w);
}
// A operand of the attribute gradient g_W1a += attr^T g_z1 for the 16 edges (block rblk, register half vh) whose
// g_z1 a lane holds in 8 registers: lane (slot m = lane & 31, half g) takes attr[e][m] of edges 16vh + 4g + 0..3 and
// 16vh + 8 + 4g + 0..3 of the block from the transposed copy (slots >= 16 do not exist: zeros)
__device__ __forceinline__ bf16x8_t attr_t_operand(const unsigned short* att, int rblk, int vh, int lane) {
  typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
  const int m = lane & 31, g = lane >> 5;
  u32x4_t w = {0u, 0u, 0u, 0u};
  if (m < ATTR_K) {
    const unsigned short* r = att + m * ATTR_T_PITCH + rblk * 32 + 16 * vh + 4 * g;
    const uint2 lo = *reinterpret_cast<const uint2*>(r);
    const uint2 hi = *reinterpret_cast<const uint2*>(r + 8);
    w[0] = lo.x; w[1] = lo.y; w[2] = hi.x; w[3] = hi.y;
  }
  return __builtin_bit_cast(bf16x8_t, w);
}
__device__ __forceinline__ bf16x8_t pack_operand8(const float* v) {
  typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
  const u32x4_t w = {pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7])};
  return __builtin_bit_cast(bf16x8_t, w);
}
// attribute term of z1 for the 32-edge block rblk of the tile: one accumulator block per column block of this lane
template <int CB>
__device__ __forceinline__ void attr_z1_block(const unsigned short* at, int rblk, int lane, const bf16x8_t (&bW)[CB],
                                              f32x16_t (&zat)[CB]) {
  const f32x16_t zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const bf16x8_t a = *reinterpret_cast<const bf16x8_t*>(at + (rblk * 32 + (lane & 31)) * ATTR_K + (lane >> 5) * 8);
#pragma unroll
  for (int j = 0; j < CB; ++j) zat[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bW[j], zero, 0, 0, 0);
}

// ---------------------------------------------------------------------------------------------
// forward
// ---------------------------------------------------------------------------------------------
// Gathers of one group of 8 edges (bf16 pairs): the pair words of P[dst] and Q[col] and d2, from the tile's
// scalars in LDS. Group gi of a wavefront: row block gi >> 1, register half gi & 1.
template <int H, bool BF16>
__device__ __forceinline__ void fwd_issue_group(const void* PQ, const int* s, int wr, int gi, int g, unsigned colb,
                                                unsigned (&wpo)[8], unsigned (&wqo)[8], float (&ddo)[8]) {
  using C = ECfg<H, BF16>;
  using PQP = PQPitch<H, true>;
  const int rblk = wr * C::RB + (gi >> 1), vh = gi & 1;
  int di[8], ci[8];
  lds_rows8(s, rblk, vh, g, di);
  lds_rows8(s + C::TM, rblk, vh, g, ci);
  lds_rows8(s + 2 * C::TM, rblk, vh, g, ddo);
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    wpo[u] = ldg_u32(PQ, (unsigned)di[u] * PQP::ROW + colb);
    wqo[u] = ldg_u32(PQ, (unsigned)ci[u] * PQP::ROW + colb + PQP::QOFF);
  }
}

// One tile of the forward kernel. FULL: all TM edges of the tile exist (no masking anywhere).
// wp0 / wq0 / dd0 (bf16 pairs only): the gathers of this tile's first group, asked for at the end of the previous
// tile; on return they hold those of the next tile's first group.
// ATTR: k > 1 edge attributes take the place of the d2 term (at: this tile's attributes in LDS, at_next / nxa: where and
// what to store for the next tile, bW1a: this lane's attribute weights as matrix-core operands).
template <int H, bool BF16, bool BRES, bool FULL, bool ATTR>
__device__ __forceinline__ void edge_fwd_tile(
    const EdgeFwdArgs& p, unsigned char* smem, const int* s, int* s_next, int nxt, int tile, int E, int tid, int wr,
    int wc, int lane, const float (&w1d)[ECfg<H, BF16>::CB], const float (&b2)[ECfg<H, BF16>::CB],
    const typename BFrag<H, BF16>::type (&breg)[BRES ? BFrag<H, BF16>::NKB : 1][ECfg<H, BF16>::CB],
    unsigned (&wp0)[8], unsigned (&wq0)[8], float (&dd0)[8], const unsigned short* at, unsigned short* at_next,
    uint2 nxa, const bf16x8_t (&bW1a)[ECfg<H, BF16>::CB]) {
  using C = ECfg<H, BF16>;
  constexpr bool PAIRS = BF16 && C::CB == 2;
  const int g = lane >> 5, x = lane & 31;
  // byte offset of this lane's first column inside a row: word wc*32 + x of bf16 pairs, else column wc*CB*32 + x
  const unsigned colb = (unsigned)((PAIRS ? wc * 32 : wc * C::CB * 32) + x) * 4u;
  // attribute term of z1 for all of this wavefront's blocks (the accumulator registers are free in this phase)
  f32x16_t zat[ATTR ? C::RB : 1][C::CB];
  if constexpr (ATTR) {
#pragma unroll
    for (int i = 0; i < C::RB; ++i) attr_z1_block<C::CB>(at, wr * C::RB + i, lane, bW1a, zat[i]);
  }
  // ---- produce a1 for this wavefront's blocks: memory (operand-packed) and LDS (row-major)
  if constexpr (PAIRS && FULL) {
    // Groups of 8 edges, software-pipelined: the gathers of the next group are in flight while this one is turned
    // into a1 (the accumulator registers are free in this phase and hold the second set of gathered words; a third
    // set would spill).
    constexpr int NG = C::RB * 2;
    static_assert(NG % 2 == 0, "even groups use the carried buffers, odd ones the local set");
    unsigned wp1[8], wq1[8];
    float dd1[8];
#pragma unroll
    for (int gi = 0; gi < NG; ++gi) {
      // the first group's gathers were asked for at the end of the previous tile
      if (gi + 1 < NG) {
        if ((gi + 1) & 1) fwd_issue_group<H, BF16>(p.PQ, s, wr, gi + 1, g, colb, wp1, wq1, dd1);
        else fwd_issue_group<H, BF16>(p.PQ, s, wr, gi + 1, g, colb, wp0, wq0, dd0);
      }
      const unsigned (&wpc)[8] = (gi & 1) ? wp1 : wp0;
      const unsigned (&wqc)[8] = (gi & 1) ? wq1 : wq0;
      const float (&ddc)[8] = (gi & 1) ? dd1 : dd0;
      const int rblk = wr * C::RB + (gi >> 1), vh = gi & 1;
      const int eb = tile * (C::TM / 32) + rblk;
#pragma unroll
      for (int j = 0; j < C::CB; ++j) {
        const int cblk = wc * C::CB + j;
        float vals[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const float zp = j == 0 ? __uint_as_float(wpc[u] << 16) : __uint_as_float(wpc[u] & 0xffff0000u);
          const float zq = j == 0 ? __uint_as_float(wqc[u] << 16) : __uint_as_float(wqc[u] & 0xffff0000u);
          if constexpr (ATTR) vals[u] = silu_f(zp + zq + zat[gi >> 1][j][8 * (gi & 1) + u]);
          else vals[u] = silu_f(zp + zq + ddc[u] * w1d[j]);
        }
        emit_half<BF16, C::STRIDE>(smem, rblk * 32, g, cblk * 32 + x, vals, vh, p.a1_pk, (size_t)eb * C::NCB + cblk, lane);
      }
    }
  } else
#pragma unroll
  for (int i = 0; i < C::RB; ++i) {
    const int rblk = wr * C::RB + i;
    const int eb = tile * (C::TM / 32) + rblk;
    if (!FULL && eb * 32 >= E) continue;
#pragma unroll
    for (int vh = 0; vh < 2; ++vh) {
      int di[8], ci[8];
      float dd[8];
      lds_rows8(s, rblk, vh, g, di);
      lds_rows8(s + C::TM, rblk, vh, g, ci);
      lds_rows8(s + 2 * C::TM, rblk, vh, g, dd);
      const unsigned ok = FULL ? 0xffu : rows8_mask(eb, vh, g, E);
      float z[C::CB][8];
      gather_z1<H, C::CB, PAIRS>(p.PQ, di, ci, dd, w1d, colb, z);
#pragma unroll
      for (int j = 0; j < C::CB; ++j) {
        const int cblk = wc * C::CB + j;
        const int n = cblk * 32 + x;
        float vals[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          if constexpr (ATTR) vals[u] = silu_f(z[j][u] + zat[i][j][8 * vh + u]);
          else vals[u] = silu_f(z[j][u]);
          if (!FULL && !((ok >> u) & 1u)) vals[u] = 0.f;
        }
        emit_half<BF16, C::STRIDE>(smem, rblk * 32, g, n, vals, vh, p.a1_pk, (size_t)eb * C::NCB + cblk, lane);
      }
    }
  }
  BRing<H, BF16> ring;
  if constexpr (!BRES) tile_mma_prefetch<H, BF16>(p.W2p, wc, lane, ring);
  __syncthreads();
  f32x16_t acc[C::RB][C::CB];
#pragma unroll
  for (int i = 0; i < C::RB; ++i)
#pragma unroll
    for (int j = 0; j < C::CB; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  if constexpr (BRES) tile_mma_res<H, BF16>(smem, wr, lane, breg, acc);
  else tile_mma<H, BF16>(smem, p.W2p, wr, wc, lane, acc, ring);
  if (tid < 3 * C::TM) s_next[tid] = nxt;
  if constexpr (ATTR) store_attr4(at_next, tid, nxa);
  __syncthreads();
  // ---- z2 = acc + b2, stored v-major (as bf16 pairs of this lane's two column blocks when PAIRS)
#pragma unroll
  for (int i = 0; i < C::RB; ++i) {
    const int eb = tile * (C::TM / 32) + wr * C::RB + i;
    if (!FULL && eb * 32 >= E) continue;
    if constexpr (PAIRS) {
      char* o = uoff(p.z2_vm, ((size_t)eb * (C::NCB / 2) + wc) * 16 * 256);
#pragma unroll
      for (int v = 0; v < 16; ++v)
        stg_nt<unsigned>(o, lane * 4u + v * 256u, pack_bf16x2(acc[i][0][v] + b2[0], acc[i][1][v] + b2[1]));
      // the next tile's scalars are in LDS now: its first gathers travel behind the first block's stores, whose
      // accumulators are free by then (past the last tile the scalars are zeros and the gathers read row 0)
      if (FULL && i == 0) fwd_issue_group<H, BF16>(p.PQ, s_next, wr, 0, g, colb, wp0, wq0, dd0);
    } else {
#pragma unroll
      for (int j = 0; j < C::CB; ++j) {
        const size_t blk = ((size_t)eb * C::NCB + (wc * C::CB + j)) * 16 * 64;   // first element of the block
        if (BF16) {
          char* o = uoff(p.z2_vm, blk * 2);
#pragma unroll
          for (int t = 0; t < 8; ++t) {
            const unsigned pk = pack_bf16x2(acc[i][j][2 * t] + b2[j], acc[i][j][2 * t + 1] + b2[j]);
            stg_nt<unsigned short>(o, lane * 2u + (2 * t) * 128u, (unsigned short)(pk & 0xffffu));
            stg_nt<unsigned short>(o, lane * 2u + (2 * t + 1) * 128u, (unsigned short)(pk >> 16));
          }
        } else {
          char* o = uoff(p.z2_vm, blk * 4);
#pragma unroll
          for (int v = 0; v < 16; ++v) stg_nt<float>(o, lane * 4u + v * 256u, acc[i][j][v] + b2[j]);
        }
      }
    }
  }
  if constexpr (PAIRS && !FULL) fwd_issue_group<H, BF16>(p.PQ, s_next, wr, 0, g, colb, wp0, wq0, dd0);
}

template <int H, bool BF16, bool BRES_REQ, bool ATTR>
__global__ void __launch_bounds__(256, 2) k_edge_fwd(EdgeFwdArgs p, int ntiles) {
  using C = ECfg<H, BF16>;
  static_assert(!ATTR || (BF16 && C::TM == 64), "edge attributes: bf16 operands, 64-edge tiles");
  // keep this wavefront's slice of W2 in registers? (not with attributes: their accumulators need the room)
  constexpr bool BRES = BRES_REQ && BF16 && !ATTR;   // fp32 operands take W2 as three bf16 planes from L2
  extern __shared__ __align__(16) unsigned char smem[];
  int* sc = reinterpret_cast<int*>(smem + C::LDS_BYTES);   // [2][3][TM] per-edge scalars, double buffered
  unsigned short* atb = reinterpret_cast<unsigned short*>(smem + C::LDS_BYTES + 6 * C::TM * 4);   // [2][ATTR_TILE] (ATTR)
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: tile addresses stay in scalar registers
  const int wr = wave / C::WC, wc = wave % C::WC;
  const int x = lane & 31;
  const int E = (int)p.E;
  float w1d[C::CB], b2[C::CB];
  bf16x8_t bW1a[C::CB];
#pragma unroll
  for (int j = 0; j < C::CB; ++j) {
    const int n = (wc * C::CB + j) * 32 + x;
    w1d[j] = ATTR ? 0.f : p.w1d[n];
    b2[j] = p.b2[n];
    if constexpr (ATTR) bW1a[j] = attr_weight_operand(p.W1a, p.k, H, n, lane);
  }
  typename BFrag<H, BF16>::type breg[BRES ? BFrag<H, BF16>::NKB : 1][C::CB];
  if constexpr (BRES) load_b_resident<H, BF16>(p.W2p, wc, lane, breg);
  const TileRange tr = xcd_tile_range(ntiles);
  {
    const int s0 = fetch_edge_scalar<C::TM, 3>(p.dst, p.col, p.d2, nullptr, tr.first, tr.end, E, tid);
    if (tid < 3 * C::TM) sc[tid] = s0;
    if constexpr (ATTR) store_attr4(atb, tid, fetch_attr4(p.attr, p.k, tr.first, tr.end, E, tid));
  }
  __syncthreads();
  unsigned wp0[8], wq0[8];   // bf16 pairs: gathers of the coming tile's first group (see edge_fwd_tile)
  float dd0[8];
  if constexpr (BF16 && C::CB == 2)
    fwd_issue_group<H, BF16>(p.PQ, sc, wr, 0, lane >> 5, (unsigned)(wc * 32 + x) * 4u, wp0, wq0, dd0);
  int buf = 0;
  for (int tile = tr.first; tile < tr.end; tile += tr.step, buf ^= 1) {
    // the next tile's scalars travel while this tile is processed
    const int nxt = fetch_edge_scalar<C::TM, 3>(p.dst, p.col, p.d2, nullptr, tile + tr.step, tr.end, E, tid);
    uint2 nxa = make_uint2(0u, 0u);
    if constexpr (ATTR) nxa = fetch_attr4(p.attr, p.k, tile + tr.step, tr.end, E, tid);
    const int* s = sc + buf * 3 * C::TM;
    int* s_next = sc + (buf ^ 1) * 3 * C::TM;
    const unsigned short* at = atb + buf * ATTR_TILE;
    unsigned short* at_next = atb + (buf ^ 1) * ATTR_TILE;
    if ((tile + 1) * C::TM <= E)
      edge_fwd_tile<H, BF16, BRES, true, ATTR>(p, smem, s, s_next, nxt, tile, E, tid, wr, wc, lane, w1d, b2, breg, wp0, wq0,
                                               dd0, at, at_next, nxa, bW1a);
    else
      edge_fwd_tile<H, BF16, BRES, false, ATTR>(p, smem, s, s_next, nxt, tile, E, tid, wr, wc, lane, w1d, b2, breg, wp0, wq0,
                                                dd0, at, at_next, nxa, bW1a);
  }
}

// Workgroups of a kernel that one compute unit holds at once (registers and LDS decide). The persistent edge kernels
// launch exactly that many per compute unit: a grid that is not a multiple of it runs a last, partly empty round
// (four workgroups on a unit that holds three take as long as six).
static int resident_per_cu(const void* kernel, size_t dyn_lds, int fallback) {
  int n = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kernel, 256, dyn_lds) != hipSuccess || n < 1) {
    (void)hipGetLastError();
    return fallback;
  }
  return n > 8 ? 8 : n;
}

template <int H, bool BF16, bool ATTR>
static int32_t launch_edge_fwd_t(hipStream_t st, const EdgeFwdArgs& a) {
  using C = ECfg<H, BF16>;
  const int64_t ntiles = (a.E + C::TM - 1) / C::TM;
  if (ntiles <= 0) return HGNN_OK;
  constexpr size_t lds = C::LDS_BYTES + 6 * C::TM * 4 + (ATTR ? 2 * ATTR_TILE * 2 : 0);
  static int per_cu = 0;
  if (!per_cu) {
    HGNN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&k_edge_fwd<H, BF16, true, ATTR>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    per_cu = resident_per_cu(reinterpret_cast<const void*>(&k_edge_fwd<H, BF16, true, ATTR>), lds, 2);
  }
  int64_t grid = (int64_t)num_cus() * per_cu;
  if (grid > ntiles) grid = ntiles;
  ProfScope ps(PT_EDGE_FUSED_FWD, st);
  k_edge_fwd<H, BF16, true, ATTR><<<dim3((unsigned)grid), 256, lds, st>>>(a, (int)ntiles);
  HGNN_LAUNCH_CHECK("k_edge_fwd");
  return HGNN_OK;
}

int32_t launch_edge_fwd(hipStream_t st, int H, bool bf16, const EdgeFwdArgs& a) {
  HGNN_REQUIRE(a.E >= 0 && a.E <= EDGE_MAX_E, HGNN_ERR_BAD_SHAPE, "edge kernels index edges with 32 bits (E = %lld)",
               (long long)a.E);
  if (a.k > 1) {
    HGNN_REQUIRE(bf16 && a.k <= ATTR_K && a.W1a && (a.attr || a.E == 0), HGNN_ERR_BAD_SHAPE,
                 "edge attributes on the fused kernels: bf16 operands, 2 <= k <= %d", ATTR_K);
    switch (H) {
      case 64: return launch_edge_fwd_t<64, true, true>(st, a);
      case 128: return launch_edge_fwd_t<128, true, true>(st, a);
      case 256: return launch_edge_fwd_t<256, true, true>(st, a);
    }
    return set_error(HGNN_ERR_BAD_SHAPE, "H must be 64, 128 or 256 (got %d)", H);
  }
  switch (H) {
    case 64: return bf16 ? launch_edge_fwd_t<64, true, false>(st, a) : launch_edge_fwd_t<64, false, false>(st, a);
    case 128: return bf16 ? launch_edge_fwd_t<128, true, false>(st, a) : launch_edge_fwd_t<128, false, false>(st, a);
    case 256: return bf16 ? launch_edge_fwd_t<256, true, false>(st, a) : launch_edge_fwd_t<256, false, false>(st, a);
  }
  return set_error(HGNN_ERR_BAD_SHAPE, "H must be 64, 128 or 256 (got %d)", H);
}

// ---------------------------------------------------------------------------------------------
// segmented reductions over v-major tensors: one wavefront per segment
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float wave_sum64(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
  return x;
}

// element offset of (edge e, column block cb, lane-in-block x) in a v-major tensor
template <int NCB>
__device__ __forceinline__ size_t vm_index(size_t e, int cb, int x) {
  const int r = (int)(e & 31);
  const int v = 4 * (r >> 3) + (r & 3);
  const int gg = (r >> 2) & 1;
  return (((e >> 5) * NCB + cb) * 16 + v) * 64 + gg * 32 + x;
}

// Two columns of edge e for one lane of a segment kernel. Lane (hp = lane>>5, x = lane&31), pass c:
//   PAIRS: one 32-bit word = columns (2c+hp)*64 + x and (2c+hp)*64 + 32 + x      (passes: NCB/4)
//   else:  column block 2c+hp, single column (2c+hp)*32 + x; second value unused  (passes: NCB/2)
template <int H, bool BF16, bool PAIRS>
struct SegCols {
  static constexpr int NCB = H / 32;
  static constexpr int NPASS = PAIRS ? NCB / 4 : NCB / 2;
  static constexpr int PER = PAIRS ? 2 : 1;
  __device__ static __forceinline__ void fetch(const void* __restrict__ X, size_t e, int c, int hp, int x, float* out) {
    // streamed once: non-temporal, so that the lines do not displace what the neighbouring kernels keep in the L2
    if constexpr (PAIRS) {
      const unsigned w = __builtin_nontemporal_load(reinterpret_cast<const unsigned*>(X) + vm_index<NCB / 2>(e, 2 * c + hp, x));
      out[0] = __uint_as_float(w << 16);
      out[1] = __uint_as_float(w & 0xffff0000u);
    } else {
      const size_t idx = vm_index<NCB>(e, 2 * c + hp, x);
      out[0] = BF16 ? bf_bits_to_f(__builtin_nontemporal_load(reinterpret_cast<const unsigned short*>(X) + idx))
                    : __builtin_nontemporal_load(reinterpret_cast<const float*>(X) + idx);
    }
  }
  __device__ static __forceinline__ int column(int c, int hp, int x, int k) {
    return PAIRS ? (2 * c + hp) * 64 + 32 * k + x : (2 * c + hp) * 32 + x;
  }
  // The same fetch for an edge index that is uniform over the wavefront: everything that depends on the edge goes
  // into the (scalar) base address, and a lane adds only its constant byte offset lane_off(c, hp, x) of pass c.
  static constexpr unsigned ESZ = PAIRS ? 4u : (BF16 ? 2u : 4u);
  static constexpr int NB = PAIRS ? NCB / 2 : NCB;
  __device__ static __forceinline__ unsigned lane_off(int c, int hp, int x) {
    return (unsigned)((2 * c + hp) * 1024 + x) * ESZ;
  }
  __device__ static __forceinline__ void fetch_u(const void* __restrict__ X, int e, unsigned loff, float* out) {
    const int r = e & 31;
    const size_t first = (((size_t)(e >> 5) * NB) * 16 + 4 * (r >> 3) + (r & 3)) * 64 + ((r >> 2) & 1) * 32;
    const char* base = reinterpret_cast<const char*>(X) + first * ESZ;
    if constexpr (PAIRS) {
      const unsigned w = __builtin_nontemporal_load(reinterpret_cast<const unsigned*>(base + loff));
      out[0] = __uint_as_float(w << 16);
      out[1] = __uint_as_float(w & 0xffff0000u);
    } else if constexpr (BF16) {
      out[0] = bf_bits_to_f(__builtin_nontemporal_load(reinterpret_cast<const unsigned short*>(base + loff)));
    } else {
      out[0] = __builtin_nontemporal_load(reinterpret_cast<const float*>(base + loff));
    }
  }
};

// XE: also keep x_e = wx . m_e of every edge (for the gradient with respect to the edge vectors); v' is then summed
// from the x_e (another summation order than without XE)
template <int H, bool BF16, bool XE>
__global__ void __launch_bounds__(256)
k_seg_fwd_vm(int N, const int32_t* __restrict__ row_ptr, const void* __restrict__ z2_vm,
             const float* __restrict__ rvec, const float* __restrict__ wx, float alpha,
             const float* __restrict__ v_in, float* __restrict__ M, float* __restrict__ v_out,
             float* __restrict__ xe) {
  using S = SegCols<H, BF16, BF16 && H == 256>;
  constexpr int NV = S::NPASS * S::PER;
  const int i = __builtin_amdgcn_readfirstlane((int)(((size_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6));
  const int lane = threadIdx.x & 63;
  if (i >= N) return;
  const int hp = lane >> 5, x = lane & 31;
  const int e0 = row_ptr[i], e1 = row_ptr[i + 1];
  unsigned loff[S::NPASS];   // kept as registers of their own: loads take a scalar base plus one of them
#pragma unroll
  for (int c = 0; c < S::NPASS; ++c) {
    loff[c] = S::lane_off(c, hp, x);
    asm volatile("" : "+v"(loff[c]));
  }
  if constexpr (XE) {
    float acc[NV], wl[NV];
#pragma unroll
    for (int c = 0; c < S::NPASS; ++c)
#pragma unroll
      for (int k = 0; k < S::PER; ++k) {
        acc[c * S::PER + k] = 0.f;
        wl[c * S::PER + k] = wx[S::column(c, hp, x, k)];
      }
    float sx = 0.f, sy = 0.f, sz = 0.f;
    constexpr int EPT = 4;
    for (int e = e0; e < e1; e += EPT) {   // four edges per trip (clamped at the end of the row)
      float z[EPT][NV], xs[EPT];
#pragma unroll
      for (int u = 0; u < EPT; ++u) {
        const int ee = e + u < e1 ? e + u : e1 - 1;
#pragma unroll
        for (int c = 0; c < S::NPASS; ++c) S::fetch_u(z2_vm, ee, loff[c], &z[u][c * S::PER]);
      }
#pragma unroll
      for (int u = 0; u < EPT; ++u) {
        const bool on = e + u < e1;
        float t = 0.f;
#pragma unroll
        for (int c = 0; c < NV; ++c) {
          const float m = on ? silu_f(z[u][c]) : 0.f;
          acc[c] += m;
          t = fmaf(wl[c], m, t);
        }
        xs[u] = wave_sum64(t);
      }
#pragma unroll
      for (int u = 0; u < EPT; ++u)
        if (e + u < e1) {
          const size_t ee = (size_t)(e + u);
          if (lane == 0) xe[ee] = xs[u];
          sx = fmaf(xs[u], rvec[3 * ee], sx);
          sy = fmaf(xs[u], rvec[3 * ee + 1], sy);
          sz = fmaf(xs[u], rvec[3 * ee + 2], sz);
        }
    }
#pragma unroll
    for (int c = 0; c < S::NPASS; ++c)
#pragma unroll
      for (int k = 0; k < S::PER; ++k) M[(size_t)i * H + S::column(c, hp, x, k)] = alpha * acc[c * S::PER + k];
    if (lane == 0) {
      v_out[3 * (size_t)i] = v_in[3 * (size_t)i] + alpha * sx;
      v_out[3 * (size_t)i + 1] = v_in[3 * (size_t)i + 1] + alpha * sy;
      v_out[3 * (size_t)i + 2] = v_in[3 * (size_t)i + 2] + alpha * sz;
    }
    return;
  }
  // x_e = wx . m_e stays spread over the lanes: a lane adds its share of x_e r_e for every edge and the lanes are
  // summed once per atom
  float acc[NV], wl[NV];
#pragma unroll
  for (int c = 0; c < S::NPASS; ++c)
#pragma unroll
    for (int k = 0; k < S::PER; ++k) {
      acc[c * S::PER + k] = 0.f;
      wl[c * S::PER + k] = wx[S::column(c, hp, x, k)];
    }
  float sx = 0.f, sy = 0.f, sz = 0.f;
  // a row's edges are summed in list order; four edges per trip so that their loads are in flight together
  // (asking for the next four while these are summed changes nothing: the kernel runs at the rate the memory
  // system gives for this access pattern)
  constexpr int EPT = 4;
  int e = e0;
  for (; e + EPT <= e1; e += EPT) {
    float r[EPT][3], z[EPT][NV];
#pragma unroll
    for (int u = 0; u < EPT; ++u) {
#pragma unroll
      for (int k = 0; k < 3; ++k) r[u][k] = rvec[3 * (size_t)(e + u) + k];
#pragma unroll
      for (int c = 0; c < S::NPASS; ++c) S::fetch_u(z2_vm, e + u, loff[c], &z[u][c * S::PER]);
    }
#pragma unroll
    for (int u = 0; u < EPT; ++u) {
      float t = 0.f;
#pragma unroll
      for (int c = 0; c < NV; ++c) {
        const float m = silu_f(z[u][c]);
        acc[c] += m;
        t = fmaf(wl[c], m, t);
      }
      sx = fmaf(t, r[u][0], sx);
      sy = fmaf(t, r[u][1], sy);
      sz = fmaf(t, r[u][2], sz);
    }
  }
  for (; e < e1; ++e) {
    const float rx = rvec[3 * (size_t)e], ry = rvec[3 * (size_t)e + 1], rz = rvec[3 * (size_t)e + 2];
    float z[NV];
#pragma unroll
    for (int c = 0; c < S::NPASS; ++c) S::fetch_u(z2_vm, e, loff[c], &z[c * S::PER]);
    float t = 0.f;
#pragma unroll
    for (int c = 0; c < NV; ++c) {
      const float m = silu_f(z[c]);
      acc[c] += m;
      t = fmaf(wl[c], m, t);
    }
    sx = fmaf(t, rx, sx);
    sy = fmaf(t, ry, sy);
    sz = fmaf(t, rz, sz);
  }
#pragma unroll
  for (int c = 0; c < S::NPASS; ++c)
#pragma unroll
    for (int k = 0; k < S::PER; ++k) M[(size_t)i * H + S::column(c, hp, x, k)] = alpha * acc[c * S::PER + k];
  sx = wave_sum64(sx);
  sy = wave_sum64(sy);
  sz = wave_sum64(sz);
  if (lane == 0) {
    v_out[3 * (size_t)i] = v_in[3 * (size_t)i] + alpha * sx;
    v_out[3 * (size_t)i + 1] = v_in[3 * (size_t)i + 1] + alpha * sy;
    v_out[3 * (size_t)i + 2] = v_in[3 * (size_t)i + 2] + alpha * sz;
  }
}

int32_t launch_seg_fwd_vm(hipStream_t st, int H, bool bf16, int N, const int32_t* row_ptr, const void* z2_vm,
                          const float* rvec, const float* wx, float alpha, const float* v_in, float* M,
                          float* v_out, float* xe) {
  if (N <= 0) return HGNN_OK;
  const unsigned grid = (unsigned)(((int64_t)N * 64 + 255) / 256);
  ProfScope ps(PT_SEG_FWD, st);
#define HGNN_SEGF(HH, BB)                                                                                        \
  if (xe) k_seg_fwd_vm<HH, BB, true><<<grid, 256, 0, st>>>(N, row_ptr, z2_vm, rvec, wx, alpha, v_in, M, v_out, xe); \
  else k_seg_fwd_vm<HH, BB, false><<<grid, 256, 0, st>>>(N, row_ptr, z2_vm, rvec, wx, alpha, v_in, M, v_out, xe)
  switch (H) {
    case 64: if (bf16) { HGNN_SEGF(64, true); } else { HGNN_SEGF(64, false); } break;
    case 128: if (bf16) { HGNN_SEGF(128, true); } else { HGNN_SEGF(128, false); } break;
    case 256: if (bf16) { HGNN_SEGF(256, true); } else { HGNN_SEGF(256, false); } break;
    default: return set_error(HGNN_ERR_BAD_SHAPE, "H must be 64, 128 or 256");
  }
#undef HGNN_SEGF
  HGNN_LAUNCH_CHECK("k_seg_fwd_vm");
  return HGNN_OK;
}

// g_P rows that k_edge_bwd could not finish inside one unit of DSUM_UNIT edges (see EdgeBwdArgs::gP): the partial of the unit in
// which row i starts (slot 1) plus the partials of the later units (slot 0), in unit order; an empty row is set to
// zero. One wavefront per atom, H/64 columns per lane. In two steps, so that the loads of the first four partials
// travel while the wavefront does its other work.
template <int H>
struct DsumFixRow {
  static_assert(H % 64 == 0, "whole columns per lane");
  typedef float vec_t __attribute__((ext_vector_type(H / 64)));
  static constexpr int AHEAD = 4;
  vec_t p[AHEAD];
  int ra, rb, u0, uk;
  __device__ __forceinline__ void issue(int i, int lane, const DsumFix& f) {
    ra = f.row_ptr[i];
    rb = f.row_ptr[i + 1];
    u0 = ra / DSUM_UNIT;
    uk = rb > ra ? (rb - 1) / DSUM_UNIT : u0;
#pragma unroll
    for (int q = 0; q < AHEAD; ++q) {
      p[q] = vec_t(0.f);
      if (u0 < uk && u0 + q <= uk)
        p[q] = reinterpret_cast<const vec_t*>(f.dpart + ((size_t)(u0 + q) * 2 + (q == 0 ? 1 : 0)) * H)[lane];
    }
  }
  __device__ __forceinline__ void finish(int i, int lane, const DsumFix& f) const {
    vec_t* o = reinterpret_cast<vec_t*>(f.gP + (size_t)i * f.ldgP) + lane;
    if (ra == rb) {
      *o = vec_t(0.f);
      return;
    }
    if (u0 == uk) return;
    vec_t a = p[0];
#pragma unroll
    for (int q = 1; q < AHEAD; ++q) a += p[q];   // units beyond the row's last one hold zeros here
    for (int u = u0 + AHEAD; u <= uk; ++u) a += reinterpret_cast<const vec_t*>(f.dpart + (size_t)u * 2 * H)[lane];
    *o = a;
  }
};

// DOT: also dot[e] = sum_c wdot[c] X[e][c] for every edge of the list (the gradient with respect to d2 when X = g_z1
// and wdot is the row of W1 that acts on d2)
template <int H, bool BF16, bool DOT>
__global__ void __launch_bounds__(256)
k_segsum_vm(int N, const int32_t* __restrict__ ptr, const int32_t* __restrict__ perm, const void* __restrict__ X,
            float* __restrict__ out, int ldo, const float* __restrict__ wdot, float* __restrict__ dot, DsumFix fix) {
  using S = SegCols<H, BF16, BF16 && H == 256>;
  constexpr int NV = S::NPASS * S::PER;
  const int i = __builtin_amdgcn_readfirstlane((int)(((size_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6));
  const int lane = threadIdx.x & 63;
  if (i >= N) return;
  const int hp = lane >> 5, x = lane & 31;
  const int t0 = ptr[i], t1 = ptr[i + 1];
  // on request this wavefront also finishes atom i's row of another sum, the one the reverse edge kernel started
  DsumFixRow<H> fr;
  if (fix.gP) fr.issue(i, lane, fix);
  if constexpr (DOT) {
    float acc[NV], wl[NV];
#pragma unroll
    for (int c = 0; c < S::NPASS; ++c)
#pragma unroll
      for (int k = 0; k < S::PER; ++k) {
        acc[c * S::PER + k] = 0.f;
        wl[c * S::PER + k] = wdot[S::column(c, hp, x, k)];
      }
    constexpr int EPT = 4;
    for (int t = t0; t < t1; t += EPT) {   // four edges per trip (clamped at the end of the list)
      float vv[EPT][NV];
      size_t ee[EPT];
#pragma unroll
      for (int u = 0; u < EPT; ++u) {
        const int tt = t + u < t1 ? t + u : t1 - 1;
        ee[u] = perm ? (size_t)perm[tt] : (size_t)tt;
#pragma unroll
        for (int c = 0; c < S::NPASS; ++c) S::fetch(X, ee[u], c, hp, x, &vv[u][c * S::PER]);
      }
#pragma unroll
      for (int u = 0; u < EPT; ++u) {
        const bool on = t + u < t1;
        float d = 0.f;
#pragma unroll
        for (int c = 0; c < NV; ++c) {
          acc[c] += on ? vv[u][c] : 0.f;
          d = fmaf(wl[c], vv[u][c], d);
        }
        d = wave_sum64(d);
        if (on && lane == 0) dot[ee[u]] = d;
      }
    }
#pragma unroll
    for (int c = 0; c < S::NPASS; ++c)
#pragma unroll
      for (int k = 0; k < S::PER; ++k) out[(size_t)i * ldo + S::column(c, hp, x, k)] = acc[c * S::PER + k];
    if (fix.gP) fr.finish(i, lane, fix);
    return;
  }
  float acc[NV];
#pragma unroll
  for (int c = 0; c < NV; ++c) acc[c] = 0.f;
  int t = t0;
  constexpr int EPT = 4;
  for (; t + EPT <= t1; t += EPT) {   // four edges per trip: their loads are independent; summed in list order
    size_t ee[EPT];
#pragma unroll
    for (int u = 0; u < EPT; ++u) ee[u] = perm ? (size_t)perm[t + u] : (size_t)(t + u);
    float vv[EPT][NV];
#pragma unroll
    for (int u = 0; u < EPT; ++u)
#pragma unroll
      for (int c = 0; c < S::NPASS; ++c) S::fetch(X, ee[u], c, hp, x, &vv[u][c * S::PER]);
#pragma unroll
    for (int u = 0; u < EPT; ++u)
#pragma unroll
      for (int c = 0; c < NV; ++c) acc[c] += vv[u][c];
  }
  for (; t < t1; ++t) {
    const size_t ea = perm ? (size_t)perm[t] : (size_t)t;
    float va[NV];
#pragma unroll
    for (int c = 0; c < S::NPASS; ++c) S::fetch(X, ea, c, hp, x, &va[c * S::PER]);
#pragma unroll
    for (int c = 0; c < NV; ++c) acc[c] += va[c];
  }
#pragma unroll
  for (int c = 0; c < S::NPASS; ++c)
#pragma unroll
    for (int k = 0; k < S::PER; ++k) out[(size_t)i * ldo + S::column(c, hp, x, k)] = acc[c * S::PER + k];
  if (fix.gP) fr.finish(i, lane, fix);
}

int32_t launch_segsum_vm(hipStream_t st, int H, bool bf16, int N, const int32_t* ptr, const int32_t* perm,
                         const void* X_vm, float* out, int ldo, int tag, const float* wdot, float* dot,
                         const DsumFix* fix) {
  if (N <= 0) return HGNN_OK;
  const DsumFix fx = fix ? *fix : DsumFix{nullptr, nullptr, nullptr, 0};
  const unsigned grid = (unsigned)(((int64_t)N * 64 + 255) / 256);
  ProfScope ps(tag, st);
#define HGNN_SEGS(HH, BB)                                                                            \
  if (dot) k_segsum_vm<HH, BB, true><<<grid, 256, 0, st>>>(N, ptr, perm, X_vm, out, ldo, wdot, dot, fx); \
  else k_segsum_vm<HH, BB, false><<<grid, 256, 0, st>>>(N, ptr, perm, X_vm, out, ldo, wdot, dot, fx)
  switch (H) {
    case 64: if (bf16) { HGNN_SEGS(64, true); } else { HGNN_SEGS(64, false); } break;
    case 128: if (bf16) { HGNN_SEGS(128, true); } else { HGNN_SEGS(128, false); } break;
    case 256: if (bf16) { HGNN_SEGS(256, true); } else { HGNN_SEGS(256, false); } break;
    default: return set_error(HGNN_ERR_BAD_SHAPE, "H must be 64, 128 or 256");
  }
#undef HGNN_SEGS
  HGNN_LAUNCH_CHECK("k_segsum_vm");
  return HGNN_OK;
}

// A skinny product on the matrix cores: per 64-edge tile the v-major g_z1 (the accumulator mapping: lane <-> column)
// is copied into a row-major LDS tile, from which two wavefronts read it as the A operand (lane <-> edge) of
// [32 edges x H] x [H x 16 slots]; the B operands (W1a transposed, bf16) are laid out in LDS once per workgroup.
template <int H>
__global__ void __launch_bounds__(256)
k_gattr_vm(int E, const void* __restrict__ X, const float* __restrict__ W1a, int k, float* __restrict__ g_attr) {
  using C = ECfg<H, true>;
  constexpr bool PAIRS = H == 256;
  constexpr int NKB = H / 16;
  __shared__ __align__(16) unsigned short tile[C::TM * C::STRIDE];
  __shared__ __align__(16) unsigned short bpk[NKB * 64 * 8];   // operand order: [k step][lane][8]
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wr = wave / C::WC, wc = wave % C::WC;
  const int g = lane >> 5, x = lane & 31;
  // B[k = column][n = slot]: lane (n, half) of step kb holds W1a[n][16 kb + 8 half + 0..7]
  for (int idx = tid; idx < NKB * 64; idx += 256) {
    const int kb = idx >> 6, l = idx & 63;
    const int n = l & 31, c0 = kb * 16 + (l >> 5) * 8;
#pragma unroll
    for (int t = 0; t < 8; ++t) bpk[idx * 8 + t] = n < k ? (unsigned short)f2bf_bits(W1a[(size_t)n * H + c0 + t]) : 0;
  }
  const int ntiles = (E + C::TM - 1) / C::TM;
  for (int t = blockIdx.x; t < ntiles; t += gridDim.x) {
    __syncthreads();   // the previous tile has been read (first trip: bpk is complete)
    // ---- v-major -> row-major: this wavefront's blocks, as the fused kernels hold them
#pragma unroll
    for (int i = 0; i < C::RB; ++i) {
      const int rblk = wr * C::RB + i;
      const int eb = t * (C::TM / 32) + rblk;
      if (eb * 32 >= E) {   // rows beyond the last edge: zeros
#pragma unroll
        for (int v = 0; v < 16; ++v)
#pragma unroll
          for (int j = 0; j < C::CB; ++j)
            tile[(rblk * 32 + 8 * (v >> 2) + 4 * g + (v & 3)) * C::STRIDE + (wc * C::CB + j) * 32 + x] = 0;
        continue;
      }
      if constexpr (PAIRS) {
        const char* zp = uoff(X, ((size_t)eb * (C::NCB / 2) + wc) * 16 * 256);
        unsigned w[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) w[v] = ldg_nt<unsigned>(zp, lane * 4u + v * 256u);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = rblk * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
          tile[row * C::STRIDE + (wc * 2) * 32 + x] = (unsigned short)(w[v] & 0xffffu);
          tile[row * C::STRIDE + (wc * 2 + 1) * 32 + x] = (unsigned short)(w[v] >> 16);
        }
      } else {
#pragma unroll
        for (int j = 0; j < C::CB; ++j) {
          const int cblk = wc * C::CB + j;
          const char* zp = uoff(X, (((size_t)eb * C::NCB + cblk) * 16) * 64 * 2);
          unsigned short w[16];
#pragma unroll
          for (int v = 0; v < 16; ++v) w[v] = ldg_nt<unsigned short>(zp, lane * 2u + v * 128u);
#pragma unroll
          for (int v = 0; v < 16; ++v) tile[(rblk * 32 + 8 * (v >> 2) + 4 * g + (v & 3)) * C::STRIDE + cblk * 32 + x] = w[v];
        }
      }
    }
    __syncthreads();
    // ---- two wavefronts, one 32-edge block each
    if (wave < C::TM / 32) {
      f32x16_t acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
      for (int kb = 0; kb < NKB; ++kb) {
        const bf16x8_t a = *reinterpret_cast<const bf16x8_t*>(&tile[(wave * 32 + x) * C::STRIDE + kb * 16 + g * 8]);
        const bf16x8_t b = *reinterpret_cast<const bf16x8_t*>(&bpk[(kb * 64 + lane) * 8]);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
      }
      // D: lane (slot x, half g), register v <-> edge 8*(v>>2) + 4g + (v&3) of the block
      if (x < k) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int e = t * C::TM + wave * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
          if (e < E) g_attr[(size_t)e * k + x] = acc[v];
        }
      }
    }
  }
}

int32_t launch_gattr_vm(hipStream_t st, int H, int64_t E, const void* X_vm, const float* W1a, int k, float* g_attr) {
  if (E <= 0) return HGNN_OK;
  HGNN_REQUIRE(k >= 2 && k <= 16 && E <= EDGE_MAX_E, HGNN_ERR_BAD_SHAPE, "gattr: bad k or E");
  ProfScope ps(PT_MISC, st);
  int64_t grid = (int64_t)num_cus() * 4;
  const int64_t ntiles = (E + 63) / 64;
  if (grid > ntiles) grid = ntiles;
  switch (H) {
    case 64: k_gattr_vm<64><<<(unsigned)grid, 256, 0, st>>>((int)E, X_vm, W1a, k, g_attr); break;
    case 128: k_gattr_vm<128><<<(unsigned)grid, 256, 0, st>>>((int)E, X_vm, W1a, k, g_attr); break;
    case 256: k_gattr_vm<256><<<(unsigned)grid, 256, 0, st>>>((int)E, X_vm, W1a, k, g_attr); break;
    default: return set_error(HGNN_ERR_BAD_SHAPE, "H must be 64, 128 or 256");
  }
  HGNN_LAUNCH_CHECK("k_gattr_vm");
  return HGNN_OK;
}

// ---------------------------------------------------------------------------------------------
// backward
// ---------------------------------------------------------------------------------------------
__global__ void k_edge_cvec(int64_t E, const int32_t* __restrict__ dst, const float* __restrict__ rvec,
                            const float* __restrict__ g_v, float alpha, float* __restrict__ cvec) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= E) return;
  const size_t i = (size_t)dst[e];
  cvec[e] = alpha * (g_v[3 * i] * rvec[3 * e] + g_v[3 * i + 1] * rvec[3 * e + 1] + g_v[3 * i + 2] * rvec[3 * e + 2]);
}

int32_t launch_edge_cvec(hipStream_t st, int64_t E, const int32_t* dst, const float* rvec, const float* g_v,
                         float alpha, float* cvec) {
  if (E <= 0) return HGNN_OK;
  ProfScope ps(PT_MISC, st);
  k_edge_cvec<<<(unsigned)((E + 255) / 256), 256, 0, st>>>(E, dst, rvec, g_v, alpha, cvec);
  HGNN_LAUNCH_CHECK("k_edge_cvec");
  return HGNN_OK;
}

// One tile of the reverse kernel. FULL: all TM edges of the tile exist (no masking anywhere).
// ATTR: k > 1 edge attributes take the place of d2 (at / att: this tile's attributes in LDS, edge-major and
// slot-major; *_next / nxa: where and what to store for the next tile; bW1a: the attribute weights as matrix-core
// operands; gacc: running g_W1a of this wavefront's columns, slots in the accumulator rows).
template <int H, bool BF16, bool FULL, bool ATTR, bool DSUM>
__device__ __forceinline__ void edge_bwd_tile(const EdgeBwdArgs& p, unsigned char* smem, const int* s, int* s_next,
                                              int nxt, int tile, int E, int tid, int wr, int wc, int lane,
                                              const float (&w1d)[ECfg<H, BF16>::CB], const float (&wxn)[ECfg<H, BF16>::CB],
                                              float (&sb2)[ECfg<H, BF16>::CB], float (&swx)[ECfg<H, BF16>::CB],
                                              float (&sw1)[ECfg<H, BF16>::CB], const unsigned short* at,
                                              const unsigned short* att, unsigned short* at_next, unsigned short* att_next,
                                              uint2 nxa, const bf16x8_t (&bW1a)[ECfg<H, BF16>::CB],
                                              f32x16_t (&gacc)[ECfg<H, BF16>::CB]) {
  using C = ECfg<H, BF16>;
  constexpr bool PAIRS = BF16 && C::CB == 2;
  constexpr unsigned GM_ROW = PAIRS ? H * 2u : 2u * H * 4u;   // row pitch of g_M in bytes (checked by the launcher)
  const int g = lane >> 5, x = lane & 31;
  // byte offset of this lane's first column inside a row: word wc*32 + x of bf16 pairs, else column wc*CB*32 + x
  const unsigned colb = (unsigned)((PAIRS ? wc * 32 : wc * C::CB * 32) + x) * 4u;
  static_assert(!DSUM || ((PAIRS || (!BF16 && H == 128)) && !ATTR),
                "the in-kernel destination sums take 128 words per edge (bf16 pairs at H = 256, fp32 at H = 128)");
  // DSUM: the last phase also leaves the tile's g_z1 words row-major in LDS (row pitch of the A tile, which is no
  // longer needed then); this lane writes word wc*32 + x of the rows 4g + (constant)
  constexpr int DPITCH = PAIRS ? C::STRIDE / 2 : C::STRIDE;
  unsigned* dsw = reinterpret_cast<unsigned*>(smem) + (4 * g) * DPITCH + wc * 32 + x;
  // the destinations of the edges next to the tile decide whether its first and last row are complete here
  int dprev = -1, dnext = -1;
  if constexpr (DSUM) {
    if (tile > 0) dprev = p.dst[(size_t)tile * C::TM - 1];
    if ((tile + 1) * C::TM < E) dnext = p.dst[(size_t)(tile + 1) * C::TM];
  }
  // ---- g_z2 = (alpha*g_M[dst] + c*wx) * silu'(z2): operand-packed to memory, row-major to LDS
  if constexpr (PAIRS && FULL) {
    // groups of 8 edges, software-pipelined: the loads of the next group are in flight while this one is processed
    // (the accumulator registers are free in this phase; the same in the last phase, where they are not, spills)
    constexpr int NG = C::RB * 2;
    unsigned zw[2][8], gw[2][8];
    float cc[2][8];
    auto issue = [&](int gi, unsigned (&zo)[8], unsigned (&go)[8], float (&co)[8]) {
      const int rblk = wr * C::RB + (gi >> 1), vh = gi & 1;
      const int eb = tile * (C::TM / 32) + rblk;
      int di[8];
      lds_rows8(s, rblk, vh, g, di);
      lds_rows8(s + 3 * C::TM, rblk, vh, g, co);
      const char* zp = uoff(p.z2_vm, (((size_t)eb * (C::NCB / 2) + wc) * 16 + 8 * vh) * 256);
#pragma unroll
      for (int u = 0; u < 8; ++u) zo[u] = ldg_nt<unsigned>(zp, lane * 4u + u * 256u);
#pragma unroll
      for (int u = 0; u < 8; ++u) go[u] = ldg_u32(p.gM, (unsigned)di[u] * GM_ROW + colb);
    };
    issue(0, zw[0], gw[0], cc[0]);
#pragma unroll
    for (int gi = 0; gi < NG; ++gi) {
      if (gi + 1 < NG) issue(gi + 1, zw[(gi + 1) & 1], gw[(gi + 1) & 1], cc[(gi + 1) & 1]);
      const int sl = gi & 1;
      const int rblk = wr * C::RB + (gi >> 1), vh = gi & 1;
      const int eb = tile * (C::TM / 32) + rblk;
#pragma unroll
      for (int j = 0; j < C::CB; ++j) {
        const int cblk = wc * C::CB + j;
        float vals[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const float zz = j == 0 ? __uint_as_float(zw[sl][u] << 16) : __uint_as_float(zw[sl][u] & 0xffff0000u);
          const float gmv = j == 0 ? __uint_as_float(gw[sl][u] << 16) : __uint_as_float(gw[sl][u] & 0xffff0000u);
          float m, dm;
          silu_both(zz, m, dm);
          const float gz = fmaf(cc[sl][u], wxn[j], gmv) * dm;   // the pair form holds alpha * g_M
          vals[u] = gz;
          sb2[j] += gz;
          swx[j] += cc[sl][u] * m;
        }
        emit_half<BF16, C::STRIDE>(smem, rblk * 32, g, cblk * 32 + x, vals, vh, p.gz2_pk, (size_t)eb * C::NCB + cblk, lane);
      }
#pragma unroll
      for (int j = 0; j < C::CB; ++j) asm volatile("" : "+v"(sb2[j]), "+v"(swx[j]));
    }
  } else
#pragma unroll
  for (int i = 0; i < C::RB; ++i) {
    const int rblk = wr * C::RB + i;
    const int eb = tile * (C::TM / 32) + rblk;
    if (!FULL && eb * 32 >= E) continue;
#pragma unroll
    for (int vh = 0; vh < 2; ++vh) {
      int di[8];
      float cc[8];
      lds_rows8(s, rblk, vh, g, di);
      lds_rows8(s + 3 * C::TM, rblk, vh, g, cc);
      const unsigned ok = FULL ? 0xffu : rows8_mask(eb, vh, g, E);
      float gm[C::CB][8];
      unsigned zw[8];   // PAIRS: z2 of both column blocks, one word per edge
      if constexpr (PAIRS) {
        const char* zp = uoff(p.z2_vm, (((size_t)eb * (C::NCB / 2) + wc) * 16 + 8 * vh) * 256);
#pragma unroll
        for (int u = 0; u < 8; ++u) zw[u] = ldg_nt<unsigned>(zp, lane * 4u + u * 256u);
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const unsigned w = ldg_u32(p.gM, (unsigned)di[u] * GM_ROW + colb);
          gm[0][u] = __uint_as_float(w << 16);
          gm[1][u] = __uint_as_float(w & 0xffff0000u);
        }
      } else {
#pragma unroll
        for (int j = 0; j < C::CB; ++j)
#pragma unroll
          for (int u = 0; u < 8; ++u) gm[j][u] = ldg_f32(p.gM, (unsigned)di[u] * GM_ROW + colb + j * 128u);
      }
#pragma unroll
      for (int j = 0; j < C::CB; ++j) {
        const int cblk = wc * C::CB + j;
        const int n = cblk * 32 + x;
        const size_t zblk = (((size_t)eb * C::NCB + cblk) * 16 + 8 * vh) * 64;   // first element of the half block
        float zz[8], vals[8];
        if constexpr (PAIRS) {
#pragma unroll
          for (int u = 0; u < 8; ++u) zz[u] = j == 0 ? __uint_as_float(zw[u] << 16) : __uint_as_float(zw[u] & 0xffff0000u);
        } else {
#pragma unroll
          for (int u = 0; u < 8; ++u)
            zz[u] = BF16 ? bf_bits_to_f(ldg_nt<unsigned short>(uoff(p.z2_vm, zblk * 2), lane * 2u + u * 128u))
                         : ldg_nt<float>(uoff(p.z2_vm, zblk * 4), lane * 4u + u * 256u);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          float m, dm;
          silu_both(zz[u], m, dm);
          float gz = fmaf(cc[u], wxn[j], PAIRS ? gm[j][u] : p.alpha * gm[j][u]) * dm;   // the pair form holds alpha * g_M
          if (!FULL && !((ok >> u) & 1u)) gz = 0.f;   // c is zero there, so the wx sum needs no mask
          vals[u] = gz;
          sb2[j] += gz;
          swx[j] += cc[u] * m;
        }
        emit_half<BF16, C::STRIDE>(smem, rblk * 32, g, n, vals, vh, p.gz2_pk, (size_t)eb * C::NCB + cblk, lane);
      }
      // the running column sums are complete for this group here: without this the compiler defers their chains
      // past the matrix product and keeps every operand alive (in scratch memory) until then
#pragma unroll
      for (int j = 0; j < C::CB; ++j) asm volatile("" : "+v"(sb2[j]), "+v"(swx[j]));
    }
  }
  BRing<H, BF16> ring;
  tile_mma_prefetch<H, BF16>(p.W2Tp, wc, lane, ring);
  __syncthreads();
  f32x16_t acc[C::RB][C::CB];
  tile_mma<H, BF16>(smem, p.W2Tp, wr, wc, lane, acc, ring);
  s_next[tid] = nxt;
  if constexpr (ATTR) {
    store_attr4(at_next, tid, nxa);
    store_attr4_t(att_next, tid, nxa);
  }
  __syncthreads();
  f32x16_t zat[C::CB];   // ATTR: attribute term of z1 of the 32-edge block at hand
  // ---- g_z1 = g_a1 * silu'(z1), z1 recomputed from the projected node features
  if constexpr (PAIRS && FULL) {
    // the same pipelining; d2 is read from LDS when it is used so that only the gathered words live twice
    using PQP = PQPitch<H, true>;
    constexpr int NG = C::RB * 2;
    unsigned wp[2][8], wq[2][8];
    auto issue = [&](int gi, unsigned (&wpo)[8], unsigned (&wqo)[8]) {
      const int rblk = wr * C::RB + (gi >> 1), vh = gi & 1;
      int di[8], ci[8];
      lds_rows8(s, rblk, vh, g, di);
      lds_rows8(s + C::TM, rblk, vh, g, ci);
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        wpo[u] = ldg_u32(p.PQ, (unsigned)di[u] * PQP::ROW + colb);
        wqo[u] = ldg_u32(p.PQ, (unsigned)ci[u] * PQP::ROW + colb + PQP::QOFF);
      }
    };
    issue(0, wp[0], wq[0]);
#pragma unroll
    for (int gi = 0; gi < NG; ++gi) {
      if (gi + 1 < NG) issue(gi + 1, wp[(gi + 1) & 1], wq[(gi + 1) & 1]);
      const int sl = gi & 1;
      const int i = gi >> 1, vh = gi & 1;
      const int rblk = wr * C::RB + i;
      const int eb = tile * (C::TM / 32) + rblk;
      float dd[8];
      if constexpr (!ATTR) lds_rows8(s + 2 * C::TM, rblk, vh, g, dd);
      if constexpr (ATTR) {
        if (vh == 0) attr_z1_block<C::CB>(at, rblk, lane, bW1a, zat);
      }
      char* o = uoff(p.gz1_vm, (((size_t)eb * (C::NCB / 2) + wc) * 16 + 8 * vh) * 256);
      float ga[2][8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const float t0 = ATTR ? zat[0][8 * vh + u] : dd[u] * w1d[0];
        const float t1 = ATTR ? zat[1][8 * vh + u] : dd[u] * w1d[1];
        const float z0 = __uint_as_float(wp[sl][u] << 16) + __uint_as_float(wq[sl][u] << 16) + t0;
        const float z1 = __uint_as_float(wp[sl][u] & 0xffff0000u) + __uint_as_float(wq[sl][u] & 0xffff0000u) + t1;
        const float g0 = acc[i][0][8 * vh + u] * dsilu_f(z0);
        const float g1 = acc[i][1][8 * vh + u] * dsilu_f(z1);
        if constexpr (ATTR) {
          ga[0][u] = g0;
          ga[1][u] = g1;
        } else {
          sw1[0] += dd[u] * g0;
          sw1[1] += dd[u] * g1;
        }
        const unsigned pw = pack_bf16x2(g0, g1);
        stg_nt<unsigned>(o, lane * 4u + u * 256u, pw);
        if constexpr (DSUM) dsw[(rblk * 32 + 8 * (2 * vh + (u >> 2)) + (u & 3)) * DPITCH] = pw;
      }
      if constexpr (ATTR) {
        const bf16x8_t aT = attr_t_operand(att, rblk, vh, lane);
#pragma unroll
        for (int j = 0; j < C::CB; ++j)
          gacc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aT, pack_operand8(ga[j]), gacc[j], 0, 0, 0);
      } else {
#pragma unroll
        for (int j = 0; j < C::CB; ++j) asm volatile("" : "+v"(sw1[j]));
      }
    }
  } else
#pragma unroll
  for (int i = 0; i < C::RB; ++i) {
    const int rblk = wr * C::RB + i;
    const int eb = tile * (C::TM / 32) + rblk;
    if (!FULL && eb * 32 >= E) continue;
#pragma unroll
    for (int vh = 0; vh < 2; ++vh) {
      int di[8], ci[8];
      float dd[8];
      lds_rows8(s, rblk, vh, g, di);
      lds_rows8(s + C::TM, rblk, vh, g, ci);
      lds_rows8(s + 2 * C::TM, rblk, vh, g, dd);
      float z[C::CB][8];
      gather_z1<H, C::CB, PAIRS>(p.PQ, di, ci, dd, w1d, colb, z);
      if constexpr (ATTR) {
        if (vh == 0) attr_z1_block<C::CB>(at, rblk, lane, bW1a, zat);
      }
      float gv[C::CB][8];
#pragma unroll
      for (int j = 0; j < C::CB; ++j)
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const float zz = ATTR ? z[j][u] + zat[j][8 * vh + u] : z[j][u];
          gv[j][u] = acc[i][j][8 * vh + u] * dsilu_f(zz);   // rows beyond E have acc == 0
          if constexpr (!ATTR) sw1[j] += dd[u] * gv[j][u];
        }
      if constexpr (ATTR) {
        const bf16x8_t aT = attr_t_operand(att, rblk, vh, lane);
#pragma unroll
        for (int j = 0; j < C::CB; ++j)
          gacc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aT, pack_operand8(gv[j]), gacc[j], 0, 0, 0);
      }
      if constexpr (PAIRS) {
        char* o = uoff(p.gz1_vm, (((size_t)eb * (C::NCB / 2) + wc) * 16 + 8 * vh) * 256);
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const unsigned pw = pack_bf16x2(gv[0][u], gv[1][u]);
          stg_nt<unsigned>(o, lane * 4u + u * 256u, pw);
          if constexpr (DSUM) dsw[(rblk * 32 + 8 * (2 * vh + (u >> 2)) + (u & 3)) * DPITCH] = pw;
        }
      } else {
#pragma unroll
        for (int j = 0; j < C::CB; ++j) {
          const size_t blk = (((size_t)eb * C::NCB + (wc * C::CB + j)) * 16 + 8 * vh) * 64;
          if constexpr (BF16) {
            char* o = uoff(p.gz1_vm, blk * 2);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
              const unsigned pk = pack_bf16x2(gv[j][2 * t], gv[j][2 * t + 1]);
              stg_nt<unsigned short>(o, lane * 2u + (2 * t) * 128u, (unsigned short)(pk & 0xffffu));
              stg_nt<unsigned short>(o, lane * 2u + (2 * t + 1) * 128u, (unsigned short)(pk >> 16));
            }
          } else {
            char* o = uoff(p.gz1_vm, blk * 4);
#pragma unroll
            for (int u = 0; u < 8; ++u) {
              stg_nt<float>(o, lane * 4u + u * 256u, gv[j][u]);
              if constexpr (DSUM) dsw[(rblk * 32 + 8 * (2 * vh + (u >> 2)) + (u & 3)) * DPITCH] = __float_as_uint(gv[j][u]);
            }
          }
        }
      }
#pragma unroll
      for (int j = 0; j < C::CB; ++j) asm volatile("" : "+v"(sw1[j]));
    }
  }
  // ---- g_P: the tile's g_z1 words summed per destination out of LDS. The edges are sorted by destination, so a row
  // is a run of consecutive edges. A thread owns one word (two bf16 columns or one fp32 column) of one of the
  // tile's two halves of 32 edges and adds the half's edges in order; where the destination changes (the same place
  // for every thread of a wavefront: scalar branches on one ballot mask) the finished run goes to g_P when it is the
  // whole row, otherwise to the tile's partial slot: slot 1 when the row starts in this tile, slot 0 when it
  // started earlier. DsumFixRow adds a row's slots.
  if constexpr (DSUM) {
    static_assert(C::TM == 64 && DSUM_UNIT == C::TM, "one partial unit per tile, walked as two halves of 32 edges");
    __syncthreads();
    const unsigned* gw = reinterpret_cast<const unsigned*>(smem);
    float2* carry = reinterpret_cast<float2*>(smem + C::LDS_BYTES + 8 * C::TM * 4);   // [128], see below
    const int hf = __builtin_amdgcn_readfirstlane(tid >> 7);   // the half of the tile that this wavefront walks
    const int w = tid & 127;
    const int dl = s[lane];
    const int dq = s[lane ? lane - 1 : 0];
    const unsigned long long starts = __ballot(dl != (lane ? dq : dprev));   // bit r: edge r of the tile starts a row
    const int t0e = tile * C::TM;
    const int ge0 = t0e + 32 * hf;
    const int nvalid = FULL ? 32 : (E - ge0 < 32 ? E - ge0 : 32);
    // a finished run goes to g_P when it is its whole row, else to the tile's partial slot (1: the row starts in
    // this tile, 0: it started earlier)
    auto put = [&](bool sf, bool ef, int d, float v0, float v1) {
      float* o = (sf && ef) ? p.gP + (size_t)d * p.ldgP : p.dpart + ((size_t)tile * 2 + (sf ? 1 : 0)) * H;
      if constexpr (PAIRS) {
        o[(w >> 5) * 64 + (w & 31)] = v0;
        o[(w >> 5) * 64 + 32 + (w & 31)] = v1;
      } else {
        o[w] = v0;
      }
    };
    // the row that crosses the middle of the tile is summed by both halves: the first half hands its part over in
    // LDS, the second half keeps its own part in registers and finishes the row behind the barrier below
    const bool cont = (FULL || t0e + 32 < E) && ((starts >> 32) & 1ull) == 0ull;
    float c0 = 0.f, c1 = 0.f;
    int cd = 0;
    bool cef = false;
    if (FULL || nvalid > 0) {
      unsigned wd[32];
#pragma unroll
      for (int k = 0; k < 32; ++k) wd[k] = (FULL || k < nvalid) ? gw[(32 * hf + k) * DPITCH + w] : 0u;
      const unsigned m32 = (unsigned)(starts >> (32 * hf));
      const bool ends = ge0 + 32 >= E || (hf == 0 ? ((starts >> 32) & 1ull) != 0ull
                                                  : dnext != __builtin_amdgcn_readfirstlane(s[C::TM - 1]));
      float a0 = 0.f, a1 = 0.f;
      int k0 = 0;
      bool sf = (m32 & 1u) != 0u;   // the run at hand starts its row
      bool first = true;            // ... and is the first one of this half
      auto flush = [&](bool ef, bool last) {
        const int d = __builtin_amdgcn_readfirstlane(s[32 * hf + k0]);
        if (hf == 0 && last && cont) {
          carry[w] = make_float2(a0, a1);
        } else if (hf == 1 && first && cont) {
          c0 = a0; c1 = a1; cd = d; cef = ef;
        } else {
          put(sf, ef, d, a0, a1);
        }
      };
#pragma unroll
      for (int k = 0; k < 32; ++k) {
        if (__builtin_expect(k > 0 && ((m32 >> k) & 1u) && (FULL || k < nvalid), 0)) {   // about one edge in thirty
          flush(true, false);
          a0 = a1 = 0.f;
          k0 = k;
          sf = true;
          first = false;
        }
        if (FULL || k < nvalid) {
          if constexpr (PAIRS) {
            a0 += __uint_as_float(wd[k] << 16);
            a1 += __uint_as_float(wd[k] & 0xffff0000u);
          } else {
            a0 += __uint_as_float(wd[k]);
          }
        }
      }
      flush(ends, true);
    }
    __syncthreads();   // the next tile's first phase writes the A tile again; the carried parts are in LDS
    if (hf == 1 && cont) {
      const float2 c = carry[w];   // (written again two barriers into the next tile at the earliest)
      put((starts & 0xffffffffull) != 0ull, cef, cd, c.x + c0, c.y + c1);
    }
  }
}

template <int H, bool BF16, bool ATTR, bool DSUM>
__global__ void __launch_bounds__(256, ATTR ? 2 : 3) k_edge_bwd(EdgeBwdArgs p, int ntiles) {
  using C = ECfg<H, BF16>;
  static_assert(!ATTR || (BF16 && C::TM == 64), "edge attributes: bf16 operands, 64-edge tiles");
  extern __shared__ __align__(16) unsigned char smem[];
  int* sc = reinterpret_cast<int*>(smem + C::LDS_BYTES);   // [2][4][TM] per-edge scalars dst|col|d2|c, double buffered
  // ATTR: [2][ATTR_TILE] attributes edge-major, then [2][ATTR_T_TILE] slot-major
  unsigned short* atb = reinterpret_cast<unsigned short*>(smem + C::LDS_BYTES + 8 * C::TM * 4);
  unsigned short* attb = atb + 2 * ATTR_TILE;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: tile addresses stay in scalar registers
  const int wr = wave / C::WC, wc = wave % C::WC;
  const int g = lane >> 5, x = lane & 31;
  const int E = (int)p.E;
  static_assert(4 * C::TM == 256, "one per-edge scalar per thread");
  float w1d[C::CB], wxn[C::CB], sb2[C::CB], swx[C::CB], sw1[C::CB];
  bf16x8_t bW1a[C::CB];
  f32x16_t gacc[C::CB];
#pragma unroll
  for (int j = 0; j < C::CB; ++j) {
    const int n = (wc * C::CB + j) * 32 + x;
    w1d[j] = ATTR ? 0.f : p.w1d[n];
    wxn[j] = p.wx[n];
    sb2[j] = swx[j] = sw1[j] = 0.f;
    if constexpr (ATTR) {
      bW1a[j] = attr_weight_operand(p.W1a, p.k, H, n, lane);
#pragma unroll
      for (int v = 0; v < 16; ++v) gacc[j][v] = 0.f;
    }
  }
  const TileRange tr = xcd_tile_range(ntiles);
  sc[tid] = fetch_edge_scalar<C::TM, 4>(p.dst, p.col, p.d2, p.cvec, tr.first, tr.end, E, tid);
  if constexpr (ATTR) {
    const uint2 a0 = fetch_attr4(p.attr, p.k, tr.first, tr.end, E, tid);
    store_attr4(atb, tid, a0);
    store_attr4_t(attb, tid, a0);
  }
  __syncthreads();
  int buf = 0;
  for (int tile = tr.first; tile < tr.end; tile += tr.step, buf ^= 1) {
    // the next tile's scalars travel while this tile is processed
    const int nxt = fetch_edge_scalar<C::TM, 4>(p.dst, p.col, p.d2, p.cvec, tile + tr.step, tr.end, E, tid);
    uint2 nxa = make_uint2(0u, 0u);
    if constexpr (ATTR) nxa = fetch_attr4(p.attr, p.k, tile + tr.step, tr.end, E, tid);
    const int* s = sc + buf * 4 * C::TM;
    int* s_next = sc + (buf ^ 1) * 4 * C::TM;
    const unsigned short* at = atb + buf * ATTR_TILE;
    const unsigned short* att = attb + buf * ATTR_T_TILE;
    unsigned short* at_next = atb + (buf ^ 1) * ATTR_TILE;
    unsigned short* att_next = attb + (buf ^ 1) * ATTR_T_TILE;
    if ((tile + 1) * C::TM <= E)
      edge_bwd_tile<H, BF16, true, ATTR, DSUM>(p, smem, s, s_next, nxt, tile, E, tid, wr, wc, lane, w1d, wxn, sb2, swx, sw1, at, att,
                                         at_next, att_next, nxa, bW1a, gacc);
    else
      edge_bwd_tile<H, BF16, false, ATTR, DSUM>(p, smem, s, s_next, nxt, tile, E, tid, wr, wc, lane, w1d, wxn, sb2, swx, sw1, at, att,
                                          at_next, att_next, nxa, bW1a, gacc);
  }
  // ---- per-column partial sums of this wavefront: combine the two lane halves, one writer per column
#pragma unroll
  for (int j = 0; j < C::CB; ++j) {
    const float a = sb2[j] + __shfl_xor(sb2[j], 32);
    const float b = swx[j] + __shfl_xor(swx[j], 32);
    const float c = sw1[j] + __shfl_xor(sw1[j], 32);
    const int n = (wc * C::CB + j) * 32 + x;
    if (g == 0) {
      float* o = p.colpart + ((size_t)(blockIdx.x * C::WR + wr) * 3) * H + n;
      o[0] = a;
      o[H] = b;
      o[2 * H] = c;
    }
    if constexpr (ATTR) {
      // accumulator row 8*(v>>2) + 4g + (v&3) is attribute slot m; slots 0..15 sit in registers 0..7
      float* o = p.attrpart + (size_t)(blockIdx.x * C::WR + wr) * p.k * H + n;
#pragma unroll
      for (int v = 0; v < 8; ++v) {
        const int m = 8 * (v >> 2) + 4 * g + (v & 3);
        if (m < p.k) o[(size_t)m * H] = gacc[j][v];
      }
    }
  }
}

constexpr int EDGE_BWD_MAX_GRID = 2048;
size_t edge_bwd_colpart_floats(int H) { return (size_t)EDGE_BWD_MAX_GRID * 2 * 3 * H; }
size_t edge_bwd_attrpart_floats(int H) { return (size_t)EDGE_BWD_MAX_GRID * 2 * ATTR_K * H; }

template <int H, bool BF16, bool ATTR, bool DSUM = false>
static int32_t launch_edge_bwd_t(hipStream_t st, const EdgeBwdArgs& a) {
  using C = ECfg<H, BF16>;
  const int64_t ntiles = (a.E + C::TM - 1) / C::TM;
  static_assert(!(ATTR && DSUM), "the carried parts of the destination sums take the place of the attribute tiles");
  constexpr size_t lds = C::LDS_BYTES + 8 * C::TM * 4 + (ATTR ? 2 * (ATTR_TILE + ATTR_T_TILE) * 2 : 0) + (DSUM ? 1024 : 0);
  static int per_cu = 0;
  if (!per_cu) {
    HGNN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&k_edge_bwd<H, BF16, ATTR, DSUM>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    per_cu = resident_per_cu(reinterpret_cast<const void*>(&k_edge_bwd<H, BF16, ATTR, DSUM>), lds, ATTR ? 2 : 3);
  }
  int64_t grid = (int64_t)num_cus() * per_cu;
  if (grid > EDGE_BWD_MAX_GRID) grid = EDGE_BWD_MAX_GRID;
  if (grid > ntiles) grid = ntiles;
  if (grid < 1) grid = 1;  // E == 0: one block writes zero partials
  {
    ProfScope ps(PT_EDGE_FUSED_BWD, st);
    k_edge_bwd<H, BF16, ATTR, DSUM><<<dim3((unsigned)grid), 256, lds, st>>>(a, (int)ntiles);
    HGNN_LAUNCH_CHECK("k_edge_bwd");
  }
  float* dest[4] = {a.g_b2, a.g_wx, a.g_w1d, nullptr};
  HGNN_TRY(launch_reduce_partials(st, a.colpart, (int)grid * C::WR, 3, H, dest, 1, 0));
  if (ATTR) {
    float* adest[4] = {a.g_W1a, nullptr, nullptr, nullptr};
    HGNN_TRY(launch_reduce_partials(st, a.attrpart, (int)grid * C::WR, 1, (long)a.k * H, adest, 1, 0));
  }
  return HGNN_OK;
}

int32_t launch_edge_bwd(hipStream_t st, int H, bool bf16, const EdgeBwdArgs& a) {
  HGNN_REQUIRE(a.E >= 0 && a.E <= EDGE_MAX_E, HGNN_ERR_BAD_SHAPE, "edge kernels index edges with 32 bits (E = %lld)",
               (long long)a.E);
  HGNN_REQUIRE(a.ldgM == (edge_pairs(H, bf16) ? H / 2 : 2 * H), HGNN_ERR_BAD_SHAPE,
               "g_M must be the second half of a [N,2H] tensor, or [N,H/2] words of bf16 pairs");
  HGNN_REQUIRE(!a.gP || (edge_bwd_sums_dst(H, bf16) && a.k <= 1 && a.dpart && a.row_ptr && a.N > 0 && a.ldgP >= H &&
                         a.ldgP % 4 == 0),
               HGNN_ERR_BAD_SHAPE,
               "in-kernel destination sums: bf16 operands at H = 256 or fp32 operands at H = 128, no edge attributes");
  if (a.k > 1) {
    HGNN_REQUIRE(bf16 && a.k <= ATTR_K && a.W1a && a.attrpart && a.g_W1a && (a.attr || a.E == 0), HGNN_ERR_BAD_SHAPE,
                 "edge attributes on the fused kernels: bf16 operands, 2 <= k <= %d", ATTR_K);
    switch (H) {
      case 64: return launch_edge_bwd_t<64, true, true>(st, a);
      case 128: return launch_edge_bwd_t<128, true, true>(st, a);
      case 256: return launch_edge_bwd_t<256, true, true>(st, a);
    }
    return set_error(HGNN_ERR_BAD_SHAPE, "H must be 64, 128 or 256 (got %d)", H);
  }
  switch (H) {
    case 64: return bf16 ? launch_edge_bwd_t<64, true, false>(st, a) : launch_edge_bwd_t<64, false, false>(st, a);
    case 128:
      if (!bf16 && a.gP) return launch_edge_bwd_t<128, false, false, true>(st, a);
      return bf16 ? launch_edge_bwd_t<128, true, false>(st, a) : launch_edge_bwd_t<128, false, false>(st, a);
    case 256:
      if (bf16 && a.gP) return launch_edge_bwd_t<256, true, false, true>(st, a);
      return bf16 ? launch_edge_bwd_t<256, true, false>(st, a) : launch_edge_bwd_t<256, false, false>(st, a);
  }
  return set_error(HGNN_ERR_BAD_SHAPE, "H must be 64, 128 or 256 (got %d)", H);
}

// ---------------------------------------------------------------------------------------------
// weight gradient of W2: operands streamed in operand-packed order, contraction over edges
// ---------------------------------------------------------------------------------------------
template <int H, bool BF16>
__global__ void __launch_bounds__(256)
k_wgrad_frag(int64_t nblk32, const void* __restrict__ a1_pk, const void* __restrict__ gz2_pk,
             float* __restrict__ partial) {
  constexpr int NCB = H / 32;
  constexpr int NBW = NCB / 2;  // 32-blocks per wavefront along each output dimension
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wa = wave >> 1, wb = wave & 1;
  f32x16_t acc[NBW][NBW];
#pragma unroll
  for (int i = 0; i < NBW; ++i)
#pragma unroll
    for (int j = 0; j < NBW; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  // 32-edge blocks are dealt round-robin: at any moment the workgroups together read one contiguous window of
  // each operand (DRAM page locality), and every workgroup still sums its blocks in a fixed order
  const int64_t G = gridDim.x;
  const int64_t nmine = nblk32 > (int64_t)blockIdx.x ? (nblk32 - blockIdx.x + G - 1) / G : 0;
  // one chunk = one matrix-core operand per block column: 16 edges (bf16) or 4 edges (fp32, four instructions);
  // four chunk buffers in registers keep three chunks of loads in flight behind the products of the current one
  constexpr int CPB = BF16 ? 2 : 4;   // chunks per 32-edge block
  const int64_t nchunk = nmine * CPB;
#define HGNN_WG_LOAD(c, a, b)                                                                          \
  {                                                                                                    \
    const size_t eb_ = (size_t)(blockIdx.x + ((c) / CPB) * G);                                         \
    const int sub_ = (int)((c) % CPB);                                                                 \
    _Pragma("unroll") for (int i = 0; i < NBW; ++i) {                                                  \
      a[i] = __builtin_nontemporal_load(A + ((eb_ * NCB + wa * NBW + i) * CPB + sub_) * 64 + lane);    \
      b[i] = __builtin_nontemporal_load(B + ((eb_ * NCB + wb * NBW + i) * CPB + sub_) * 64 + lane);    \
    }                                                                                                  \
  }
  // The loop takes four chunks per trip without any branch around the products (a branch there makes the compiler
  // copy the accumulators). Loads past the end are clamped to the last chunk and their A operand is replaced by
  // zeros when it is used, so the extra products of the last trip add nothing.
#define HGNN_WG_CL(c) ((c) < nchunk ? (c) : nchunk - 1)
#define HGNN_WG_PIPELINE                                                                               \
  if (nchunk > 0) {                                                                                    \
    HGNN_WG_LOAD(0, a0, b0)                                                                            \
    HGNN_WG_LOAD(HGNN_WG_CL(1), a1, b1)                                                                \
    HGNN_WG_LOAD(HGNN_WG_CL(2), a2, b2)                                                                \
    for (int64_t c = 0; c < nchunk; c += 4) {                                                          \
      HGNN_WG_LOAD(HGNN_WG_CL(c + 3), a3, b3)                                                          \
      HGNN_WG_MMA(a0, b0, true)                                                                        \
      HGNN_WG_LOAD(HGNN_WG_CL(c + 4), a0, b0)                                                          \
      HGNN_WG_MMA(a1, b1, c + 1 < nchunk)                                                              \
      HGNN_WG_LOAD(HGNN_WG_CL(c + 5), a1, b1)                                                          \
      HGNN_WG_MMA(a2, b2, c + 2 < nchunk)                                                              \
      HGNN_WG_LOAD(HGNN_WG_CL(c + 6), a2, b2)                                                          \
      HGNN_WG_MMA(a3, b3, c + 3 < nchunk)                                                              \
    }                                                                                                  \
  }
  if constexpr (BF16) {
    const bf16x8_t* __restrict__ A = reinterpret_cast<const bf16x8_t*>(a1_pk);
    const bf16x8_t* __restrict__ B = reinterpret_cast<const bf16x8_t*>(gz2_pk);
    bf16x8_t a0[NBW], b0[NBW], a1[NBW], b1[NBW], a2[NBW], b2[NBW], a3[NBW], b3[NBW];
#define HGNN_WG_MMA(a, b, valid)                                                                       \
  {                                                                                                    \
    const bool ok_ = (valid);                                                                          \
    const bf16x8_t zero_ = {0, 0, 0, 0, 0, 0, 0, 0};                                                   \
    _Pragma("unroll") for (int i = 0; i < NBW; ++i) {                                                  \
      const bf16x8_t az_ = ok_ ? a[i] : zero_;                                                         \
      _Pragma("unroll") for (int j = 0; j < NBW; ++j)                                                  \
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(az_, b[j], acc[i][j], 0, 0, 0);          \
    }                                                                                                  \
  }
    HGNN_WG_PIPELINE
#undef HGNN_WG_MMA
  } else {
    // fp32 operands: two chunks of four edges make one step of the bf16 matrix cores (eight edges per lane, the
    // same eight for both operands); both operands are split into three bf16 terms on the way (split_bf16x3).
    // Four chunks per block, so every trip of the loop is full.
    const f32x4_t* __restrict__ A = reinterpret_cast<const f32x4_t*>(a1_pk);
    const f32x4_t* __restrict__ B = reinterpret_cast<const f32x4_t*>(gz2_pk);
    f32x4_t a0[NBW], b0[NBW], a1[NBW], b1[NBW], a2[NBW], b2[NBW], a3[NBW], b3[NBW];
#define HGNN_WG_MMA2(ax, bx, ay, by)                                                                   \
  {                                                                                                    \
    bf16x8_t as_[NBW][3], bs_[NBW][3];                                                                 \
    _Pragma("unroll") for (int i = 0; i < NBW; ++i) {                                                  \
      const float xa_[8] = {ax[i][0], ax[i][1], ax[i][2], ax[i][3], ay[i][0], ay[i][1], ay[i][2], ay[i][3]}; \
      const float xb_[8] = {bx[i][0], bx[i][1], bx[i][2], bx[i][3], by[i][0], by[i][1], by[i][2], by[i][3]}; \
      split_bf16x3(xa_, as_[i]);                                                                       \
      split_bf16x3(xb_, bs_[i]);                                                                       \
    }                                                                                                  \
    _Pragma("unroll") for (int i = 0; i < NBW; ++i)                                                    \
      _Pragma("unroll") for (int j = 0; j < NBW; ++j) acc[i][j] = mfma_bf16x3(as_[i], bs_[j], acc[i][j]); \
  }
    // (eight chunk buffers instead of four, i.e. three pairs of loads in flight, measured no faster)
    if (nchunk > 0) {
      HGNN_WG_LOAD(0, a0, b0)
      HGNN_WG_LOAD(1, a1, b1)
      HGNN_WG_LOAD(2, a2, b2)
      HGNN_WG_LOAD(3, a3, b3)
      for (int64_t c = 0; c < nchunk; c += 4) {
        HGNN_WG_MMA2(a0, b0, a1, b1)
        HGNN_WG_LOAD(HGNN_WG_CL(c + 4), a0, b0)
        HGNN_WG_LOAD(HGNN_WG_CL(c + 5), a1, b1)
        HGNN_WG_MMA2(a2, b2, a3, b3)
        HGNN_WG_LOAD(HGNN_WG_CL(c + 6), a2, b2)
        HGNN_WG_LOAD(HGNN_WG_CL(c + 7), a3, b3)
      }
    }
#undef HGNN_WG_MMA2
  }
#undef HGNN_WG_LOAD
#undef HGNN_WG_PIPELINE
#undef HGNN_WG_CL
  float* out = partial + (size_t)blockIdx.x * H * H;
#pragma unroll
  for (int i = 0; i < NBW; ++i)
#pragma unroll
    for (int j = 0; j < NBW; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int k1 = (wa * NBW + i) * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        const int k2 = (wb * NBW + j) * 32 + (lane & 31);
        out[k1 * H + k2] = acc[i][j][v];
      }
}


// The same weight gradient with a1 = silu(z1) recomputed from the projected node features instead of read back
// (bf16 pairs, H = 256 only): the forward pass then never stores a1, and this kernel trades vector work for half of
// its memory traffic. One workgroup of eight wavefronts per compute unit holds the whole H x H accumulator (two row
// blocks x four column blocks per wavefront), so two wavefronts share a SIMD and one's sigmoids overlap the other's
// matrix products. Per 16-edge chunk every wavefront is a producer first: for four consecutive edges (the same for
// all its lanes, so their indices sit in scalar registers and a gather is one 256-byte piece of a row) it gathers
// 64 pair words of P[dst] and Q[col], forms silu(z1) for the four column blocks those words cover and writes its
// share of four A operands into an LDS stage; it also loads one of the eight g_z2 operands of the chunk for the
// workgroup. Everything is software-pipelined with fixed register rings. Loads complete in the order they were
// issued, so what counts is the shortest distance between any load and its first use: every load here is used at
// least three chunks after it was issued (edge indices eight chunks ahead, used for the gathers four chunks ahead;
// g_z2 eight chunks ahead). One barrier per chunk publishes the next stage (two stages: chunk c is multiplied while
// chunk c + 1 is written).
struct WgradRcArgs {
  int64_t nblk32;    // number of 32-edge blocks, the last one possibly ragged
  int E;
  const int32_t *dst, *col;
  const float* d2;
  const void* PQ;
  const float* w1d;
  const void* gz2_pk;   // rows past the last edge of the last block hold zeros
  float* partial;
};

template <int H>
__global__ void __launch_bounds__(512) k_wgrad_frag_rc(WgradRcArgs p) {
  constexpr int NCB = H / 32;
  constexpr int STAGE = NCB * 1024;   // bytes of the eight operands of one kind for one chunk
  static_assert(H == 256, "pair storage, eight wavefronts");
  using PQP = PQPitch<H, true>;
  __shared__ __align__(16) unsigned char stage_a[4 * STAGE];
  __shared__ __align__(16) unsigned char stage_b[4 * STAGE];
  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int x = lane & 31;
  // as a producer: words wcc * 64 + lane of a row, i.e. pair group pg, column blocks 2 pg (low halves) and 2 pg + 1;
  // edges 4 q .. 4 q + 3 of the chunk, which are elements 4 (q >> 1) .. + 3 of operand lane group q & 1
  const int wcc = w >> 2, q = w & 3;
  const int pg = 2 * wcc + (lane >> 5);
  // as a consumer: A blocks 2 ra, 2 ra + 1; g_z2 blocks 4 cb .. 4 cb + 3
  const int ra = w >> 1, cb = w & 1;
  f32x16_t acc[2][4];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  const float w1lo = p.w1d[pg * 64 + x], w1hi = p.w1d[pg * 64 + 32 + x];
  const int G = gridDim.x, bid = blockIdx.x;
  const int nblk = (int)p.nblk32;
  const int E = p.E;
  // Which blocks are this workgroup's: with a grid that is a multiple of eight every XCD (workgroups are dealt to
  // the 8 XCDs round-robin) takes a contiguous eighth of the blocks, dealt round-robin inside the XCD, so that the
  // node rows an XCD gathers stay in its own L2; otherwise plain round-robin.
  int bfirst, bstride, nmine;
  if ((G & 7) == 0) {
    const int xcd = bid & 7, r = bid >> 3;
    bstride = G >> 3;
    const int lo = (int)((int64_t)nblk * xcd / 8), hi = (int)((int64_t)nblk * (xcd + 1) / 8);
    nmine = hi - lo > r ? (hi - lo - r + bstride - 1) / bstride : 0;
    bfirst = lo + r;
  } else {
    bstride = G;
    nmine = nblk > bid ? (nblk - bid + G - 1) / G : 0;
    bfirst = bid;
  }
  const int nchunk = nmine * 2;   // two 16-edge chunks per 32-edge block
  const unsigned colb = (unsigned)(wcc * 64 + lane) * 4u;   // this lane's pair word inside a row
  // lanes 0..3 fetch dst, 4..7 col, 8..11 d2 of the wavefront's four edges
  const int32_t* const idx_arr = lane < 4 ? p.dst : (lane < 8 ? p.col : reinterpret_cast<const int32_t*>(p.d2));
  unsigned char* const a_out = stage_a + (2 * pg) * 1024 + ((q & 1) * 32 + x) * 16 + 8 * (q >> 1);

  // chunk c, clamped to this workgroup's last chunk: its block, and which half of it
  auto chunk_blk = [&](int c) { const int cc = c < nchunk ? c : nchunk - 1; return bfirst + (cc >> 1) * bstride; };
  auto chunk_half = [&](int c) { const int cc = c < nchunk ? c : nchunk - 1; return cc & 1; };
  // indices and d2 of the wavefront's four edges of chunk c, one value per lane (zeros past the last edge: row 0 is
  // always a valid row, and g_z2 is zero there)
  auto load_iv = [&](int c, int& iv) {
    const int e = chunk_blk(c) * 32 + chunk_half(c) * 16 + 4 * q + (lane & 3);
    iv = 0;
    if (lane < 12 && e < E) iv = idx_arr[e];
  };
  auto gather = [&](const int iv, unsigned (&wp)[4], unsigned (&wq)[4]) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const unsigned rd = (unsigned)__builtin_amdgcn_readlane(iv, u), rc = (unsigned)__builtin_amdgcn_readlane(iv, 4 + u);
      wp[u] = ldg_u32(uoff(p.PQ, rd * PQP::ROW), colb);
      wq[u] = ldg_u32(uoff(p.PQ, rc * PQP::ROW + PQP::QOFF), colb);
    }
  };
  // this wavefront's g_z2 operand of chunk c (column block w): memory -> registers, registers -> LDS stage
  auto load_b = [&](int c, bf16x8_t& b) {
    b = ldg_nt<bf16x8_t>(uoff(p.gz2_pk, (((size_t)chunk_blk(c) * NCB + w) * 2 + chunk_half(c)) * 1024), lane * 16u);
  };
  auto stage_b_put = [&](int st, const bf16x8_t& b) {
    *reinterpret_cast<bf16x8_t*>(stage_b + st * STAGE + w * 1024 + lane * 16) = b;
  };
  // this wavefront's share of four A operands of chunk c (zeros for chunks past the workgroup's last one)
  auto stage_a_put = [&](int c, int st, const unsigned (&wp)[4], const unsigned (&wq)[4], const int iv) {
    float vl[4], vh[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const unsigned a = wp[u], b = wq[u];
      const float d = __int_as_float(__builtin_amdgcn_readlane(iv, 8 + u));
      vl[u] = silu_f((__uint_as_float(a << 16) + __uint_as_float(b << 16)) + d * w1lo);
      vh[u] = silu_f((__uint_as_float(a & 0xffff0000u) + __uint_as_float(b & 0xffff0000u)) + d * w1hi);
    }
    // no branch here: the sigmoids are meant to be scheduled between the matrix products of the same step
    const unsigned keep = c < nchunk ? 0xffffffffu : 0u;   // uniform over the workgroup
    const uint2 lo = make_uint2(pack_bf16x2(vl[0], vl[1]) & keep, pack_bf16x2(vl[2], vl[3]) & keep);
    const uint2 hi = make_uint2(pack_bf16x2(vh[0], vh[1]) & keep, pack_bf16x2(vh[2], vh[3]) & keep);
    *reinterpret_cast<uint2*>(a_out + st * STAGE) = lo;
    *reinterpret_cast<uint2*>(a_out + st * STAGE + 1024) = hi;
  };
  auto mma_fetch = [&](int st, bf16x8_t (&a)[2], bf16x8_t (&b)[4]) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
      a[i] = *reinterpret_cast<const bf16x8_t*>(stage_a + st * STAGE + (2 * ra + i) * 1024 + lane * 16);
#pragma unroll
    for (int j = 0; j < 4; ++j)
      b[j] = *reinterpret_cast<const bf16x8_t*>(stage_b + st * STAGE + (4 * cb + j) * 1024 + lane * 16);
  };
  auto mma = [&](const bf16x8_t (&a)[2], const bf16x8_t (&b)[4]) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
  };

  if (nchunk > 0) {   // uniform over the workgroup
    int iv[8];                            // index ring: slot = chunk mod 8
    unsigned wp[4][4], wq[4][4];          // gather ring: slot = chunk mod 4
    bf16x8_t bb[8];                       // g_z2 load ring: slot = chunk mod 8
    // prologue: g_z2 and indices of chunks 0..7, gathers of chunks 0..3, chunks 0 and 1 staged
#pragma unroll
    for (int k = 0; k < 8; ++k) load_b(k, bb[k]);
#pragma unroll
    for (int k = 0; k < 8; ++k) load_iv(k, iv[k]);
#pragma unroll
    for (int k = 0; k < 4; ++k) gather(iv[k], wp[k], wq[k]);
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      stage_b_put(k, bb[k]);
      stage_a_put(k, k, wp[k], wq[k], iv[k]);
    }
    __syncthreads();
    for (int c = 0; c < nchunk; c += 8) {
      // step for chunk j = c + k: fetch the operands of chunk j from their stage, ask for the g_z2 of chunk j + 8,
      // gather chunk j + 4, ask for the indices of chunk j + 8, multiply chunk j while chunk j + 2 is formed and
      // staged; a barrier after every second step (four stages)
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        bf16x8_t oa[2], ob[4];
        mma_fetch(k & 3, oa, ob);
        load_b(c + k + 8, bb[k]);
        gather(iv[(k + 4) & 7], wp[k & 3], wq[k & 3]);
        load_iv(c + k + 8, iv[k]);
        mma(oa, ob);
        stage_b_put((k + 2) & 3, bb[(k + 2) & 7]);
        stage_a_put(c + k + 2, (k + 2) & 3, wp[(k + 2) & 3], wq[(k + 2) & 3], iv[(k + 2) & 7]);
        // one matrix product, then a share of the vector work, eight times: a wavefront's products then run behind
        // its own sigmoids instead of blocking both wavefronts of the SIMD at the start of every step
        __builtin_amdgcn_sched_group_barrier(0x100, 6, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, 20, 0);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x002, 10, 0);
        }
        if (k & 1) __syncthreads();
      }
    }
  }
  float* out = p.partial + (size_t)blockIdx.x * H * H;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int k1 = (2 * ra + i) * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        const int k2 = (4 * cb + j) * 32 + (lane & 31);
        out[k1 * H + k2] = acc[i][j][v];
      }
}

// The recomputing weight gradient for fp32 operands at H = 128: the same scheme with four wavefronts (2 x 2 blocks
// of the 128 x 128 accumulator each, two workgroups per compute unit). Every value is split into its three bf16
// terms (split_bf16x3) once, by the wavefront that produces it, and the LDS stages hold three planes of ready
// operands; the consumers take six products per block pair. A producer wavefront forms silu(z1) for 64 columns and
// eight of a chunk's sixteen edges; it also splits one column block of the chunk's g_z2 (two 16-byte pieces per
// lane, already in operand order) into the stage. Two stages, one barrier per chunk.
struct WgradRc32Args {
  int64_t nblk32;
  int E;
  const int32_t *dst, *col;
  const float* d2;
  const float* PQ;      // [N, 2H] fp32: P | Q
  const float* w1d;
  const void* gz2_pk;   // fp32, operand-packed; rows past the last edge of the last block hold zeros
  float* partial;
};

template <int H>
__global__ void __launch_bounds__(256, 2) k_wgrad_frag_rc32(WgradRc32Args p) {
  constexpr int NCB = H / 32;
  constexpr int PLANE = NCB * 1024;   // one bf16 plane of the four operand blocks of a chunk: [block][64 slots][8 bf16]
  constexpr int STAGE = 3 * PLANE;
  static_assert(H == 128, "four wavefronts, 2 x 2 blocks each");
  using PQP = PQPitch<H, false>;
  typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
  __shared__ __align__(16) unsigned char stage_a[2 * STAGE];
  __shared__ __align__(16) unsigned char stage_b[2 * STAGE];
  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int x = lane & 31;
  // as a producer: columns wcc * 64 + lane (block 2 wcc + (lane >> 5)), edges 8 hh .. 8 hh + 7 of the chunk: edge
  // 8 hh + j is element 4 hh + (j & 3) of operand lane group j >> 2
  const int wcc = w >> 1, hh = w & 1;
  // as a consumer: A blocks 2 wa, 2 wa + 1; g_z2 blocks 2 wb, 2 wb + 1
  const int wa = w >> 1, wb = w & 1;
  f32x16_t acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  const float w1 = p.w1d[wcc * 64 + lane];
  const int G = gridDim.x, bid = blockIdx.x;
  const int nblk = (int)p.nblk32;
  const int E = p.E;
  int bfirst, bstride, nmine;   // this workgroup's blocks, by XCD as in the bf16-pair kernel
  if ((G & 7) == 0) {
    const int xcd = bid & 7, r = bid >> 3;
    bstride = G >> 3;
    const int lo = (int)((int64_t)nblk * xcd / 8), hi = (int)((int64_t)nblk * (xcd + 1) / 8);
    nmine = hi - lo > r ? (hi - lo - r + bstride - 1) / bstride : 0;
    bfirst = lo + r;
  } else {
    bstride = G;
    nmine = nblk > bid ? (nblk - bid + G - 1) / G : 0;
    bfirst = bid;
  }
  const int nchunk = nmine * 2;   // two 16-edge chunks per 32-edge block
  const unsigned colb = (unsigned)(wcc * 64 + lane) * 4u;
  // lanes 0..7 fetch dst, 8..15 col, 16..23 d2 of the wavefront's eight edges
  const int32_t* const idx_arr = lane < 8 ? p.dst : (lane < 16 ? p.col : reinterpret_cast<const int32_t*>(p.d2));
  unsigned char* const a_out = stage_a + (2 * wcc + (lane >> 5)) * 1024 + x * 16 + 8 * hh;

  auto chunk_blk = [&](int c) { const int cc = c < nchunk ? c : nchunk - 1; return bfirst + (cc >> 1) * bstride; };
  auto chunk_half = [&](int c) { const int cc = c < nchunk ? c : nchunk - 1; return cc & 1; };
  auto load_iv = [&](int c, int& iv) {
    const int e = chunk_blk(c) * 32 + chunk_half(c) * 16 + 8 * hh + (lane & 7);
    iv = 0;
    if (lane < 24 && e < E) iv = idx_arr[e];   // past the last edge: row 0 (always valid), and g_z2 is zero there
  };
  auto gather = [&](const int iv, float (&vp)[8], float (&vq)[8]) {
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const unsigned rd = (unsigned)__builtin_amdgcn_readlane(iv, u), rc = (unsigned)__builtin_amdgcn_readlane(iv, 8 + u);
      vp[u] = ldg_f32(uoff(p.PQ, rd * PQP::ROW), colb);
      vq[u] = ldg_f32(uoff(p.PQ, rc * PQP::ROW + PQP::QOFF), colb);
    }
  };
  // this wavefront's column block (w) of the chunk's g_z2: the two pieces are elements 0..3 and 4..7 of every slot
  auto load_b = [&](int c, f32x4_t (&b)[2]) {
    const char* src = uoff(p.gz2_pk, (((size_t)chunk_blk(c) * NCB + w) * 4 + 2 * chunk_half(c)) * 1024);
#pragma unroll
    for (int s = 0; s < 2; ++s) b[s] = ldg_nt<f32x4_t>(src + s * 1024, lane * 16u);
  };
  auto stage_b_put = [&](int st, const f32x4_t (&b)[2]) {
    const float xs[8] = {b[0][0], b[0][1], b[0][2], b[0][3], b[1][0], b[1][1], b[1][2], b[1][3]};
    bf16x8_t o[3];
    split_bf16x3(xs, o);
#pragma unroll
    for (int q = 0; q < 3; ++q)
      *reinterpret_cast<bf16x8_t*>(stage_b + st * STAGE + q * PLANE + w * 1024 + lane * 16) = o[q];
  };
  auto stage_a_put = [&](int c, int st, const float (&vp)[8], const float (&vq)[8], const int iv) {
    const float keep = c < nchunk ? 1.f : 0.f;   // uniform over the workgroup; chunks past the end give zeros
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const float d = __int_as_float(__builtin_amdgcn_readlane(iv, 16 + u));
      v[u] = silu_f(vp[u] + vq[u] + d * w1) * keep;
    }
    bf16x8_t o[3];
    split_bf16x3(v, o);
#pragma unroll
    for (int q = 0; q < 3; ++q) {
      const u32x4_t wv = __builtin_bit_cast(u32x4_t, o[q]);
      unsigned char* dstp = a_out + st * STAGE + q * PLANE;
      *reinterpret_cast<uint2*>(dstp) = make_uint2(wv[0], wv[1]);         // edges 8 hh + 0..3: lane group 0
      *reinterpret_cast<uint2*>(dstp + 512) = make_uint2(wv[2], wv[3]);   // edges 8 hh + 4..7: lane group 1
    }
  };
  auto mma = [&](int st) {
    bf16x8_t a[2][3], b[2][3];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int q = 0; q < 3; ++q)
        a[i][q] = *reinterpret_cast<const bf16x8_t*>(stage_a + st * STAGE + q * PLANE + (2 * wa + i) * 1024 + lane * 16);
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int q = 0; q < 3; ++q)
        b[j][q] = *reinterpret_cast<const bf16x8_t*>(stage_b + st * STAGE + q * PLANE + (2 * wb + j) * 1024 + lane * 16);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) acc[i][j] = mfma_bf16x3(a[i], b[j], acc[i][j]);
  };

  if (nchunk > 0) {   // uniform over the workgroup
    int iv[8];                    // index ring: slot = chunk mod 8
    float vp[4][8], vq[4][8];     // gather ring: slot = chunk mod 4
    f32x4_t bb[4][2];             // g_z2 load ring: slot = chunk mod 4
    // prologue: indices of chunks 0..8, g_z2 and gathers of chunks 0..4, chunk 0 staged
#pragma unroll
    for (int k = 0; k < 8; ++k) load_iv(k, iv[k]);
#pragma unroll
    for (int k = 0; k < 4; ++k) load_b(k, bb[k]);
#pragma unroll
    for (int k = 0; k < 4; ++k) gather(iv[k], vp[k], vq[k]);
    stage_b_put(0, bb[0]);
    stage_a_put(0, 0, vp[0], vq[0], iv[0]);
    load_b(4, bb[0]);   // chunk 4 takes the ring slots chunk 0 has just left
    gather(iv[4], vp[0], vq[0]);
    load_iv(8, iv[0]);
    __syncthreads();
    for (int c = 0; c < nchunk; c += 8) {
      // step for chunk j = c + k: multiply chunk j out of its stage and form and stage chunk j + 1; then ask for the
      // g_z2 and the gathers of chunk j + 5 (ring slots of chunk j + 1, just emptied) and the indices of chunk j + 9
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        mma(k & 1);
        stage_b_put((k + 1) & 1, bb[(k + 1) & 3]);
        stage_a_put(c + k + 1, (k + 1) & 1, vp[(k + 1) & 3], vq[(k + 1) & 3], iv[(k + 1) & 7]);
        load_b(c + k + 5, bb[(k + 1) & 3]);
        gather(iv[(k + 5) & 7], vp[(k + 1) & 3], vq[(k + 1) & 3]);
        load_iv(c + k + 9, iv[(k + 1) & 7]);
        // one matrix product, then a share of the vector work: the products of a step run behind its sigmoids and
        // splits instead of blocking both wavefronts of the SIMD
#pragma unroll
        for (int i = 0; i < 24; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x002, 10, 0);
        }
        __syncthreads();
      }
    }
  }
  float* out = p.partial + (size_t)blockIdx.x * H * H;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int k1 = (2 * wa + i) * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        const int k2 = (2 * wb + j) * 32 + (lane & 31);
        out[k1 * H + k2] = acc[i][j][v];
      }
}

// most workgroups (= partial H x H results) of one launch: the partial buffer holds 32 Mi floats at every H
constexpr int WGRAD_FRAG_MAX_GRID = 512;                        // at H = 256
static int wgrad_frag_max_grid(int H) { return WGRAD_FRAG_MAX_GRID * (256 / H) * (256 / H); }
size_t wgrad_frag_partial_floats(int H) { return (size_t)wgrad_frag_max_grid(H) * H * H; }

template <int H, bool BF16>
static int32_t launch_wgrad_frag_t(hipStream_t st, int64_t E, const void* a1_pk, const void* gz2_pk, float* partial,
                                   float* gW2) {
  const int64_t nblk32 = (E + 31) / 32;
  // one workgroup per CU holds the whole accumulator at H = 256; narrower ones leave room for four (eight)
  int64_t grid = (int64_t)num_cus() * (H == 256 ? 1 : (H == 128 ? 4 : 8));
  if (grid > wgrad_frag_max_grid(H)) grid = wgrad_frag_max_grid(H);
  if (grid > nblk32) grid = nblk32;
  if (grid < 1) grid = 1;
  {
    ProfScope ps(PT_WGRAD_EDGE, st);
    k_wgrad_frag<H, BF16><<<dim3((unsigned)grid), 256, 0, st>>>(nblk32, a1_pk, gz2_pk, partial);
    HGNN_LAUNCH_CHECK("k_wgrad_frag");
  }
  float* dest[4] = {gW2, nullptr, nullptr, nullptr};
  return launch_reduce_partials(st, partial, (int)grid, 1, (long)H * H, dest, 1, 0);
}

int32_t launch_wgrad_frag(hipStream_t st, int H, bool bf16, int64_t E, const void* a1_pk, const void* gz2_pk,
                          float* partial, float* gW2) {
  switch (H) {
    case 64: return bf16 ? launch_wgrad_frag_t<64, true>(st, E, a1_pk, gz2_pk, partial, gW2)
                         : launch_wgrad_frag_t<64, false>(st, E, a1_pk, gz2_pk, partial, gW2);
    case 128: return bf16 ? launch_wgrad_frag_t<128, true>(st, E, a1_pk, gz2_pk, partial, gW2)
                          : launch_wgrad_frag_t<128, false>(st, E, a1_pk, gz2_pk, partial, gW2);
    case 256: return bf16 ? launch_wgrad_frag_t<256, true>(st, E, a1_pk, gz2_pk, partial, gW2)
                          : launch_wgrad_frag_t<256, false>(st, E, a1_pk, gz2_pk, partial, gW2);
  }
  return set_error(HGNN_ERR_BAD_SHAPE, "H must be 64, 128 or 256 (got %d)", H);
}

int32_t launch_wgrad_frag_recompute(hipStream_t st, int H, int64_t E, const int32_t* dst, const int32_t* col,
                                    const float* d2, const void* PQ, const float* w1d, const void* gz2_pk,
                                    float* partial, float* gW2) {
  HGNN_REQUIRE(H == 256, HGNN_ERR_BAD_SHAPE, "the recomputing weight-gradient kernel needs bf16 pairs (H = 256)");
  HGNN_REQUIRE(E >= 0 && E <= EDGE_MAX_E, HGNN_ERR_BAD_SHAPE, "edge kernels index edges with 32 bits (E = %lld)",
               (long long)E);
  // One workgroup per compute unit, each leaving one partial; fewer when there are fewer than two blocks for each
  // (a multiple of eight where possible, so that the blocks are dealt by XCD). E == 0: one workgroup writes zeros.
  const int64_t nblk32 = (E + 31) / 32;
  int64_t grid = num_cus();
  if (grid > WGRAD_FRAG_MAX_GRID) grid = WGRAD_FRAG_MAX_GRID;
  if (grid > (nblk32 + 1) / 2) grid = (nblk32 + 1) / 2;
  if (grid >= 8) grid &= ~(int64_t)7;
  if (grid < 1) grid = 1;
  WgradRcArgs a;
  a.nblk32 = nblk32; a.E = (int)E; a.dst = dst; a.col = col; a.d2 = d2; a.PQ = PQ; a.w1d = w1d;
  a.gz2_pk = gz2_pk; a.partial = partial;
  {
    ProfScope ps(PT_WGRAD_EDGE, st);
    k_wgrad_frag_rc<256><<<dim3((unsigned)grid), 512, 0, st>>>(a);
    HGNN_LAUNCH_CHECK("k_wgrad_frag_rc");
  }
  float* dest[4] = {gW2, nullptr, nullptr, nullptr};
  return launch_reduce_partials(st, partial, (int)grid, 1, (long)H * H, dest, 1, 0);
}

int32_t launch_wgrad_frag_recompute32(hipStream_t st, int H, int64_t E, const int32_t* dst, const int32_t* col,
                                      const float* d2, const float* PQ, const float* w1d, const void* gz2_pk,
                                      float* partial, float* gW2) {
  HGNN_REQUIRE(H == 128, HGNN_ERR_BAD_SHAPE, "the recomputing fp32 weight-gradient kernel exists at H = 128");
  HGNN_REQUIRE(E >= 0 && E <= EDGE_MAX_E, HGNN_ERR_BAD_SHAPE, "edge kernels index edges with 32 bits (E = %lld)",
               (long long)E);
  // two workgroups per compute unit, each leaving one partial; fewer when there are fewer than two blocks for each
  const int64_t nblk32 = (E + 31) / 32;
  int64_t grid = 2 * (int64_t)num_cus();
  if (grid > wgrad_frag_max_grid(H)) grid = wgrad_frag_max_grid(H);
  if (grid > (nblk32 + 1) / 2) grid = (nblk32 + 1) / 2;
  if (grid >= 8) grid &= ~(int64_t)7;
  if (grid < 1) grid = 1;
  WgradRc32Args a;
  a.nblk32 = nblk32; a.E = (int)E; a.dst = dst; a.col = col; a.d2 = d2; a.PQ = PQ; a.w1d = w1d;
  a.gz2_pk = gz2_pk; a.partial = partial;
  {
    ProfScope ps(PT_WGRAD_EDGE, st);
    k_wgrad_frag_rc32<128><<<dim3((unsigned)grid), 256, 0, st>>>(a);
    HGNN_LAUNCH_CHECK("k_wgrad_frag_rc32");
  }
  float* dest[4] = {gW2, nullptr, nullptr, nullptr};
  return launch_reduce_partials(st, partial, (int)grid, 1, (long)H * H, dest, 1, 0);
}

}  // namespace hgnn
