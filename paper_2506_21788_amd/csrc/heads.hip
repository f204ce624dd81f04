// Embedding, pooling, routing plan and the per-source decoding heads (grouped GEMMs: one weight set
// per source, rows of each source made contiguous through the plan's permutations).
#include "devmath.h"
#include "edgeops.h"
#include "gemm.h"
#include "plan.h"

namespace hgnn {

static inline unsigned nb64(int64_t n, int t) { return (unsigned)((n + t - 1) / t); }

__device__ inline int find_graph_of_atom(const int32_t* __restrict__ graph_off, int G, int i) {
  int lo = 0, hi = G - 1;
  while (lo < hi) {
    int mid = (lo + hi) >> 1;
    if (graph_off[mid + 1] > i) hi = mid; else lo = mid + 1;
  }
  return lo;
}

// ---------------------------------------------------------------------------------------------
// embedding
// ---------------------------------------------------------------------------------------------
__global__ void k_embed_fwd(int N, int H, const int32_t* __restrict__ Z, const float* __restrict__ emb,
                            float* __restrict__ h) {
  const int CH = H >> 2;
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)N * CH) return;
  const int64_t i = idx / CH;
  const int q = (int)(idx - i * CH);
  int z = Z[i];
  z = z < 0 ? 0 : (z > HGNN_ZMAX ? HGNN_ZMAX : z);
  *reinterpret_cast<float4*>(h + i * H + q * 4) = *reinterpret_cast<const float4*>(emb + (long)z * H + q * 4);
}

// block (z, chunk): fixed-order sum over the atoms of one chunk that have Z == z; chunks are then
// summed in order by a second kernel
constexpr int EMB_CHUNK = 2048;

// (1024 threads: the common species of a chunk have a thousand rows, which the row phases walk one after the other)
__global__ void __launch_bounds__(1024)
k_embed_bwd_part(int N, int H, const int32_t* __restrict__ Z, const float* __restrict__ g_h,
                 float* __restrict__ part /*[nchunk][ZMAX+1][H]*/) {
  __shared__ float4 sh[1024];
  const int z = blockIdx.x, chunk = blockIdx.y;
  const int CH = H >> 2;
  const int q = threadIdx.x % CH, ph = threadIdx.x / CH, nph = 1024 / CH;
  const int lo = chunk * EMB_CHUNK;
  const int hi = lo + EMB_CHUNK < N ? lo + EMB_CHUNK : N;
  // the chunk's atomic numbers once per workgroup (every row phase of every column chunk asks for all of them)
  __shared__ int zs[EMB_CHUNK];
  for (int i = threadIdx.x; i < EMB_CHUNK; i += 1024) zs[i] = lo + i < hi ? Z[lo + i] : -1;
  __syncthreads();
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int i0 = lo + ph; i0 < hi; i0 += 8 * nph) {
    int zz[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int i = i0 + u * nph;
      zz[u] = i < hi ? zs[i - lo] : -1;
    }
    // the rows that match are all asked for before the first one is added (same order of additions)
    float4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (zz[u] == z) v[u] = *reinterpret_cast<const float4*>(g_h + (size_t)(i0 + u * nph) * H + q * 4);
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if (zz[u] == z) { acc.x += v[u].x; acc.y += v[u].y; acc.z += v[u].z; acc.w += v[u].w; }
    }
  }
  sh[threadIdx.x] = acc;
  __syncthreads();
  if (ph == 0) {
    for (int k = 1; k < nph; ++k) {
      const float4 v = sh[k * CH + q];
      acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    *reinterpret_cast<float4*>(part + ((size_t)chunk * (HGNN_ZMAX + 1) + z) * H + q * 4) = acc;
  }
}

__global__ void k_embed_bwd_sum(int nchunk, int H, const float* __restrict__ part, float* __restrict__ g_emb) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  const int total = (HGNN_ZMAX + 1) * H;
  if (idx >= total) return;
  float s = 0.f;
  for (int c = 0; c < nchunk; ++c) s += part[(size_t)c * total + idx];
  g_emb[idx] = s;
}

// ---------------------------------------------------------------------------------------------
// pooling
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(1024)
k_pool_fwd(int H, int mode, const int32_t* __restrict__ graph_off, const float* __restrict__ h, float* __restrict__ p) {
  __shared__ float sh[1024 * 4];
  const int g = blockIdx.x;
  const int CH = H >> 2;
  const int q = threadIdx.x % CH, ph = threadIdx.x / CH, nph = 1024 / CH;
  const int lo = graph_off[g], hi = graph_off[g + 1];
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int i = lo + ph; i < hi; i += nph) {
    const float4 v = *reinterpret_cast<const float4*>(h + (size_t)i * H + q * 4);
    acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
  }
  reinterpret_cast<float4*>(sh)[threadIdx.x] = acc;
  __syncthreads();
  if (ph == 0) {
    for (int k = 1; k < nph; ++k) {
      const float4 v = reinterpret_cast<float4*>(sh)[k * CH + q];
      acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    const float sc = (mode == HGNN_POOL_MEAN && hi > lo) ? 1.0f / (float)(hi - lo) : 1.0f;
    *reinterpret_cast<float4*>(p + (size_t)g * H + q * 4) = make_float4(acc.x * sc, acc.y * sc, acc.z * sc, acc.w * sc);
  }
}

// The same pooling for few, large graphs (crystals of thousands of atoms): one workgroup per (graph, 4-column chunk),
// every thread a row phase with four rows in flight; the phases are added in a fixed order (32 groups of 32).
__global__ void __launch_bounds__(1024)
k_pool_fwd_tall(int H, int mode, const int32_t* __restrict__ graph_off, const float* __restrict__ h, float* __restrict__ p) {
  __shared__ float4 sh[1024];
  const int g = blockIdx.x, q = blockIdx.y;
  const int lo = graph_off[g], hi = graph_off[g + 1];
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int i0 = lo + (int)threadIdx.x; i0 < hi; i0 += 4 * 1024) {
    float4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = i0 + u * 1024;
      v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (i < hi) v[u] = *reinterpret_cast<const float4*>(h + (size_t)i * H + q * 4);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) { acc.x += v[u].x; acc.y += v[u].y; acc.z += v[u].z; acc.w += v[u].w; }
  }
  sh[threadIdx.x] = acc;
  __syncthreads();
  if (threadIdx.x < 32) {
    float4 s = sh[threadIdx.x * 32];
    for (int k = 1; k < 32; ++k) {
      const float4 t = sh[threadIdx.x * 32 + k];
      s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
    }
    sh[threadIdx.x * 32] = s;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    float4 s = sh[0];
    for (int k = 1; k < 32; ++k) {
      const float4 t = sh[k * 32];
      s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
    }
    const float sc = (mode == HGNN_POOL_MEAN && hi > lo) ? 1.0f / (float)(hi - lo) : 1.0f;
    *reinterpret_cast<float4*>(p + (size_t)g * H + q * 4) = make_float4(s.x * sc, s.y * sc, s.z * sc, s.w * sc);
  }
}

__global__ void k_pool_bwd(int N, int G, int H, int mode, const int32_t* __restrict__ graph_off,
                           const float* __restrict__ g_p, float* __restrict__ g_h, int accumulate) {
  const int CH = H >> 2;
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)N * CH) return;
  const int i = (int)(idx / CH);
  const int q = (int)(idx - (int64_t)i * CH);
  const int g = find_graph_of_atom(graph_off, G, i);
  const int n = graph_off[g + 1] - graph_off[g];
  const float sc = (mode == HGNN_POOL_MEAN) ? 1.0f / (float)n : 1.0f;
  float4 v = *reinterpret_cast<const float4*>(g_p + (size_t)g * H + q * 4);
  v.x *= sc; v.y *= sc; v.z *= sc; v.w *= sc;
  float4* o = reinterpret_cast<float4*>(g_h + (size_t)i * H + q * 4);
  if (accumulate) {
    const float4 c = *o;
    v.x += c.x; v.y += c.y; v.z += c.z; v.w += c.w;
  }
  *o = v;
}

// ---------------------------------------------------------------------------------------------
// the same four operations for any other width (one element per thread; same summation orders as above would need
// the same chunking, so these are used only where the vector forms do not apply: H outside {64, 128, 256})
// ---------------------------------------------------------------------------------------------
inline bool any_H(int H) { return H >= 1 && H <= 1024; }

__global__ void k_embed_fwd_any(int N, int H, const int32_t* __restrict__ Z, const float* __restrict__ emb,
                                float* __restrict__ h) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)N * H) return;
  const int64_t i = idx / H;
  const int c = (int)(idx - i * H);
  int z = Z[i];
  z = z < 0 ? 0 : (z > HGNN_ZMAX ? HGNN_ZMAX : z);
  h[idx] = emb[(long)z * H + c];
}

// block (z, chunk): the atoms of the chunk with Z == z are listed in ascending order (each thread scans 8 consecutive
// atoms, an exclusive scan over the threads places its matches), then every column is summed over that list
__global__ void __launch_bounds__(256)
k_embed_bwd_part_any(int N, int H, const int32_t* __restrict__ Z, const float* __restrict__ g_h,
                     float* __restrict__ part /*[nchunk][ZMAX+1][H]*/) {
  static_assert(EMB_CHUNK == 2048, "8 atoms per thread");
  __shared__ int list[EMB_CHUNK];
  __shared__ int cnt[257];
  const int z = blockIdx.x, chunk = blockIdx.y, tid = threadIdx.x;
  const int lo = chunk * EMB_CHUNK;
  const int hi = lo + EMB_CHUNK < N ? lo + EMB_CHUNK : N;
  bool m[8];
  int n = 0;
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    const int i = lo + tid * 8 + u;
    m[u] = i < hi && Z[i] == z;
    n += m[u] ? 1 : 0;
  }
  cnt[tid + 1] = n;
  if (tid == 0) cnt[0] = 0;
  __syncthreads();
  if (tid == 0)
    for (int k = 1; k <= 256; ++k) cnt[k] += cnt[k - 1];
  __syncthreads();
  int o = cnt[tid];
#pragma unroll
  for (int u = 0; u < 8; ++u)
    if (m[u]) list[o++] = lo + tid * 8 + u;
  __syncthreads();
  const int total = cnt[256];
  for (int c = tid; c < H; c += 256) {
    float acc = 0.f;
    for (int k = 0; k < total; ++k) acc += g_h[(size_t)list[k] * H + c];
    part[((size_t)chunk * (HGNN_ZMAX + 1) + z) * H + c] = acc;
  }
}

// block (graph, 64-column slab): 4 row phases take every fourth atom, then the phases are added in order
__global__ void __launch_bounds__(256)
k_pool_fwd_any(int H, int mode, const int32_t* __restrict__ graph_off, const float* __restrict__ h, float* __restrict__ p) {
  __shared__ float sh[4][64];
  const int g = blockIdx.x;
  const int cl = threadIdx.x & 63, ph = threadIdx.x >> 6;
  const int c = blockIdx.y * 64 + cl;
  const int lo = graph_off[g], hi = graph_off[g + 1];
  float acc = 0.f;
  if (c < H)
    for (int i = lo + ph; i < hi; i += 4) acc += h[(size_t)i * H + c];
  sh[ph][cl] = acc;
  __syncthreads();
  if (ph == 0 && c < H) {
    const float sc = (mode == HGNN_POOL_MEAN && hi > lo) ? 1.0f / (float)(hi - lo) : 1.0f;
    p[(size_t)g * H + c] = (((sh[0][cl] + sh[1][cl]) + sh[2][cl]) + sh[3][cl]) * sc;
  }
}

__global__ void k_pool_bwd_any(int N, int G, int H, int mode, const int32_t* __restrict__ graph_off,
                               const float* __restrict__ g_p, float* __restrict__ g_h, int accumulate) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)N * H) return;
  const int i = (int)(idx / H);
  const int c = (int)(idx - (int64_t)i * H);
  const int g = find_graph_of_atom(graph_off, G, i);
  const int n = graph_off[g + 1] - graph_off[g];
  const float sc = (mode == HGNN_POOL_MEAN) ? 1.0f / (float)n : 1.0f;
  float v = g_p[(size_t)g * H + c] * sc;
  if (accumulate) v += g_h[idx];
  g_h[idx] = v;
}

// ---------------------------------------------------------------------------------------------
// routing plan
// ---------------------------------------------------------------------------------------------
// One workgroup. Counts per source (integer atomics: the sums do not depend on their order), an in-place scan over
// the sources, then the stable placement: graphs are taken 1024 at a time, a thread ranks its graph among the
// earlier graphs of the same source inside the chunk (all 1024 sources of the chunk sit in LDS) and adds the
// per-source cursor that the chunks before it left behind.
__global__ void __launch_bounds__(1024)
k_plan_graphs(int G, int S, const int32_t* __restrict__ graph_off, const int32_t* __restrict__ source_id, PlanView v) {
  __shared__ int sh_a[1024];
  __shared__ int sh_b[1024];
  const int tid = threadIdx.x;
  if (tid == 0) v.status[0] = 0;
  for (int s = tid; s <= S; s += 1024) {
    v.grp_graph_ptr[s] = 0;
    v.grp_atom_ptr[s] = 0;
  }
  __syncthreads();
  // validation, copy, counts (entry s + 1 counts source s). Few sources: the counters live in LDS (many graphs hit
  // few counters, which global atomics would serialise); many sources: global atomics.
  const bool lds_counts = S <= 1024;
  if (lds_counts) {
    sh_a[tid] = 0;
    sh_b[tid] = 0;
    __syncthreads();
  }
  for (int g = tid; g < G; g += 1024) {
    const int s = source_id[g];
    v.graph_src[g] = s;
    if (s < 0 || s >= S) {
      atomicOr(v.status, 1);
    } else if (lds_counts) {
      atomicAdd(&sh_a[s], 1);
      atomicAdd(&sh_b[s], graph_off[g + 1] - graph_off[g]);
    } else {
      atomicAdd(&v.grp_graph_ptr[s + 1], 1);
      atomicAdd(&v.grp_atom_ptr[s + 1], graph_off[g + 1] - graph_off[g]);
    }
  }
  if (lds_counts) {
    __syncthreads();
    if (tid < S) {
      v.grp_graph_ptr[tid + 1] = sh_a[tid];
      v.grp_atom_ptr[tid + 1] = sh_b[tid];
    }
  }
  __threadfence_block();
  __syncthreads();
  if (v.status[0]) return;
  // inclusive scan over entries 0..S of both arrays, 1024 at a time with a carry
  int carry_g = 0, carry_a = 0;
  for (int s0 = 0; s0 <= S; s0 += 1024) {
    const int s = s0 + tid;
    int cg = s <= S ? v.grp_graph_ptr[s] : 0, ca = s <= S ? v.grp_atom_ptr[s] : 0;
    sh_a[tid] = cg;
    sh_b[tid] = ca;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {
      const int ag = tid >= o ? sh_a[tid - o] : 0, aa = tid >= o ? sh_b[tid - o] : 0;
      __syncthreads();
      sh_a[tid] += ag;
      sh_b[tid] += aa;
      __syncthreads();
    }
    if (s <= S) {
      v.grp_graph_ptr[s] = carry_g + sh_a[tid];
      v.grp_atom_ptr[s] = carry_a + sh_b[tid];
    }
    carry_g += sh_a[1023];
    carry_a += sh_b[1023];
    __syncthreads();
  }
  __threadfence_block();
  __syncthreads();
  // stable placement by one wavefront, 64 graphs at a time: a lane ranks its graph among the earlier lanes of the
  // same source (lane values are read one by one), adds the cursor that the groups before left for that source, and
  // the last lane of every source moves the cursor on. The cursors live in LDS when they fit.
  int* cur_g = lds_counts ? sh_a : v.cur_graph;
  int* cur_a = lds_counts ? sh_b : v.cur_atom;
  for (int s = tid; s < S; s += 1024) {
    cur_g[s] = v.grp_graph_ptr[s];
    cur_a[s] = v.grp_atom_ptr[s];
  }
  __threadfence_block();
  __syncthreads();
  if (tid >= 64) return;
  // the next group's source and atom count are asked for while this group is placed
  int s_nx = tid < G ? source_id[tid] : -1;
  int na_nx = tid < G ? graph_off[tid + 1] - graph_off[tid] : 0;
  for (int g0 = 0; g0 < G; g0 += 64) {
    const int g = g0 + tid;
    const bool on = g < G;
    const int s = s_nx, na = na_nx;
    {
      const int gn = g + 64;
      s_nx = gn < G ? source_id[gn] : -1;
      na_nx = gn < G ? graph_off[gn + 1] - graph_off[gn] : 0;
    }
    int before = 0, atoms_before = 0;
    bool last = true;
    const int n = G - g0 < 64 ? G - g0 : 64;
    for (int t = 0; t < n; ++t) {
      const int st = __builtin_amdgcn_readlane(s, t), nt = __builtin_amdgcn_readlane(na, t);
      const bool same = st == s;
      if (same && t < tid) { ++before; atoms_before += nt; }
      if (same && t > tid) last = false;
    }
    int bg = 0, ba = 0;
    if (on) {
      bg = cur_g[s];
      ba = cur_a[s];
      v.graph_perm[bg + before] = g;
      v.graph_dst_off[g] = ba + atoms_before;
    }
    // every lane has read the cursors before any of them moves on (LDS accesses of one wavefront complete in
    // order; cursors in global memory need the fence)
    if (!lds_counts) __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
    __builtin_amdgcn_wave_barrier();
    if (on && last) {
      cur_g[s] = bg + before + 1;
      cur_a[s] = ba + atoms_before + na;
    }
    if (!lds_counts) __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
    __builtin_amdgcn_wave_barrier();
  }
}

__global__ void k_plan_atoms(int N, int G, const int32_t* __restrict__ graph_off, PlanView v) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= N) return;
  const int g = find_graph_of_atom(graph_off, G, i);
  v.atom_graph[i] = g;
  v.atom_perm[v.graph_dst_off[g] + (i - graph_off[g])] = i;
}

// ---------------------------------------------------------------------------------------------
// head output layers (width Hh -> 1) and their reverse
// ---------------------------------------------------------------------------------------------
struct HeadOff {  // element offsets inside one branch
  long We1, be1, We2, be2, Wf1, bf1, Wf2, bf2, per;
  HeadOff(long H, long Hh) {
    long o = 0;
    We1 = o; o += H * Hh;
    be1 = o; o += Hh;
    We2 = o; o += Hh;
    be2 = o; o += 1;
    Wf1 = o; o += H * Hh;
    bf1 = o; o += Hh;
    Wf2 = o; o += Hh;
    bf2 = o; o += 1;
    per = o;
  }
};

__device__ __forceinline__ float wsum(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
  return x;
}

// rows 0..G-1: graphs (energy); rows G..G+N-1: atoms (force). One wavefront per row.
__global__ void __launch_bounds__(256)
k_head_out_fwd(int N, int G, int Hh, const float* __restrict__ ze, const float* __restrict__ zf,
               const float* __restrict__ Whead, HeadOff o, const int32_t* __restrict__ graph_src,
               const int32_t* __restrict__ atom_graph, const float* __restrict__ v, float* __restrict__ energy,
               float* __restrict__ force, float* __restrict__ qsave) {
  const int r = (int)(((size_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6);
  const int lane = threadIdx.x & 63;
  if (r >= G + N) return;
  const bool is_graph = r < G;
  const int i = is_graph ? r : r - G;
  const int s = graph_src[is_graph ? i : atom_graph[i]];
  const float* z = is_graph ? ze + (size_t)i * Hh : zf + (size_t)i * Hh;
  const float* w2 = Whead + s * o.per + (is_graph ? o.We2 : o.Wf2);
  float acc = 0.f;
  for (int c = lane; c < Hh; c += 64) acc += w2[c] * silu_f(z[c]);
  acc = wsum(acc);
  if (lane == 0) {
    const float out = acc + Whead[s * o.per + (is_graph ? o.be2 : o.bf2)];
    if (is_graph) {
      energy[i] = out;
    } else {
      qsave[i] = out;
      force[3 * (size_t)i] = out * v[3 * (size_t)i];
      force[3 * (size_t)i + 1] = out * v[3 * (size_t)i + 1];
      force[3 * (size_t)i + 2] = out * v[3 * (size_t)i + 2];
    }
  }
}

// g_z = g_out * W2 * silu'(z); also g_v = q * g_force, and the per-row scalar g_out (gq / copy of gE)
__global__ void __launch_bounds__(256)
k_head_out_bwd(int N, int G, int Hh, const float* __restrict__ ze, const float* __restrict__ zf,
               const float* __restrict__ Whead, HeadOff o, const int32_t* __restrict__ graph_src,
               const int32_t* __restrict__ atom_graph, const float* __restrict__ v, const float* __restrict__ qsave,
               const float* __restrict__ g_energy, const float* __restrict__ g_force, float* __restrict__ g_ze,
               float* __restrict__ g_zf, float* __restrict__ gq, float* __restrict__ g_v) {
  const int r = (int)(((size_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6);
  const int lane = threadIdx.x & 63;
  if (r >= G + N) return;
  const bool is_graph = r < G;
  const int i = is_graph ? r : r - G;
  const int s = graph_src[is_graph ? i : atom_graph[i]];
  float go;
  if (is_graph) {
    go = g_energy[i];
  } else {
    const float gx = g_force[3 * (size_t)i], gy = g_force[3 * (size_t)i + 1], gz = g_force[3 * (size_t)i + 2];
    go = gx * v[3 * (size_t)i] + gy * v[3 * (size_t)i + 1] + gz * v[3 * (size_t)i + 2];
    if (lane == 0) {
      const float q = qsave[i];
      gq[i] = go;
      g_v[3 * (size_t)i] = q * gx;
      g_v[3 * (size_t)i + 1] = q * gy;
      g_v[3 * (size_t)i + 2] = q * gz;
    }
  }
  const float* z = is_graph ? ze + (size_t)i * Hh : zf + (size_t)i * Hh;
  float* gz_ = is_graph ? g_ze + (size_t)i * Hh : g_zf + (size_t)i * Hh;
  const float* w2 = Whead + s * o.per + (is_graph ? o.We2 : o.Wf2);
  for (int c = lane; c < Hh; c += 64) gz_[c] = go * w2[c] * dsilu_f(z[c]);
}

// dest[s*stride] = sum over positions of group s of w[row_idx[pos]]   (one block per group, fixed order)
__global__ void __launch_bounds__(1024)
k_group_scalar_sum(const float* __restrict__ w, const int32_t* __restrict__ row_idx,
                   const int32_t* __restrict__ grp_ptr, float* __restrict__ dest, long stride) {
  __shared__ float sh[16];
  const int s = blockIdx.x;
  float acc = 0.f;
  for (int t = grp_ptr[s] + threadIdx.x; t < grp_ptr[s + 1]; t += 1024) acc += w[row_idx[t]];
  acc = wsum(acc);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    float tot = 0.f;
    for (int k = 0; k < 16; ++k) tot += sh[k];
    dest[s * stride] = tot;
  }
}

struct HeadSaved {
  float *ze, *zf, *q;
  size_t bytes;
};
static HeadSaved carve_head_saved(void* p, int N, int G, int Hh) {
  Carver c(p);
  HeadSaved s;
  s.ze = c.take<float>((size_t)G * Hh);
  s.zf = c.take<float>((size_t)N * Hh);
  s.q = c.take<float>((size_t)N + 1);
  s.bytes = c.used();
  return s;
}
struct HeadWs {
  void* packed;  // [S][2] blocks
  float *g_ze, *g_zf, *gq, *partial;
  // reverse pass: partials of the two column sums and of the weight gradient of each branch (energy, force); they all
  // live until the pass's one reduction launch
  float *pcs[2][2], *pwg[2];
  size_t bytes;
};
static HeadWs carve_head_ws(void* p, int N, int G, int H, int Hh, int S, bool bf16) {
  Carver c(p);
  HeadWs w;
  w.packed = c.take<char>((size_t)S * 2 * packed_block_bytes(H, bf16));
  w.g_ze = c.take<float>((size_t)G * Hh);
  w.g_zf = c.take<float>((size_t)N * Hh);
  w.gq = c.take<float>((size_t)N + 1);
  const int64_t mx = N > G ? N : G;
  size_t pf = wgrad_partial_floats(H, mx, 1, S);
  size_t cf = colsum_partial_floats(H, mx, S);
  w.partial = c.take<float>(pf > cf ? pf : cf);
  for (int br = 0; br < 2; ++br) {
    const int64_t M = br == 0 ? G : N;
    w.pcs[br][0] = c.take<float>(colsum_partial_floats(H, M, S));
    w.pcs[br][1] = c.take<float>(colsum_partial_floats(H, M, S));
    w.pwg[br] = c.take<float>(wgrad_partial_floats(H, M, 1, S));
  }
  w.bytes = c.used();
  return w;
}

static int32_t check_head_args(int N, int G, int H, int Hh, int S, int dtype) {
  HGNN_REQUIRE(N >= 0 && G >= 0, HGNN_ERR_BAD_SHAPE, "negative N or G");
  HGNN_REQUIRE(S >= 1 && S <= 65535, HGNN_ERR_BAD_SHAPE, "S must be in 1..65535 (got %d)", S);
  HGNN_REQUIRE(valid_H(H), HGNN_ERR_BAD_SHAPE, "H must be 64, 128 or 256 (got %d)", H);
  HGNN_REQUIRE(Hh == H, HGNN_ERR_BAD_SHAPE, "head width Hh must equal H (got %d vs %d)", Hh, H);
  HGNN_REQUIRE(dtype == HGNN_F32 || dtype == HGNN_BF16, HGNN_ERR_BAD_SHAPE, "unknown dtype %d", dtype);
  return HGNN_OK;
}

}  // namespace hgnn

using namespace hgnn;

// plain heads at a width the block kernels do not serve (H outside {64, 128, 256} or Hh != H): the same computation
// is the one-hidden-layer case of the deep heads (same buffer layout)
static bool heads_need_fragment_path(int H, int Hh) { return !valid_H(H) || Hh != H; }

extern "C" int32_t hgnn_embed_fwd(void* stream, int32_t N, int32_t H, const int32_t* Z, const float* emb, float* h) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  HGNN_REQUIRE(N >= 0 && any_H(H), HGNN_ERR_BAD_SHAPE, "embed_fwd: bad N or H");
  if (N == 0) return HGNN_OK;
  HGNN_REQUIRE(Z && emb && h, HGNN_ERR_NULLPTR, "embed_fwd: null pointer");
  ProfScope ps(PT_EMBED, st);
  if (valid_H(H)) k_embed_fwd<<<nb64((int64_t)N * (H / 4), 256), 256, 0, st>>>(N, H, Z, emb, h);
  else k_embed_fwd_any<<<nb64((int64_t)N * H, 256), 256, 0, st>>>(N, H, Z, emb, h);
  HGNN_LAUNCH_CHECK("k_embed_fwd");
  return HGNN_OK;
}

extern "C" int32_t hgnn_embed_bwd_workspace_bytes(int32_t N, int32_t H, size_t* ws_bytes_host) {
  HGNN_REQUIRE(N >= 0 && any_H(H), HGNN_ERR_BAD_SHAPE, "embed_bwd: bad N or H");
  HGNN_REQUIRE(ws_bytes_host, HGNN_ERR_NULLPTR, "null size pointer");
  const size_t nchunk = ((size_t)N + EMB_CHUNK - 1) / EMB_CHUNK;
  *ws_bytes_host = align_up((nchunk > 0 ? nchunk : 1) * (HGNN_ZMAX + 1) * H * sizeof(float));
  return HGNN_OK;
}

// both entry points of the embedding gradient: `part` holds the per-chunk sums, every entry of which is written before
// it is read, so it needs no clearing
static int32_t embed_bwd_launch(hipStream_t st, int32_t N, int32_t H, const int32_t* Z, const float* g_h, float* g_emb,
                                float* part) {
  const int nchunk = (N + EMB_CHUNK - 1) / EMB_CHUNK;
  ProfScope ps(PT_EMBED, st);
  if (nchunk > 0) {
    if (valid_H(H)) k_embed_bwd_part<<<dim3(HGNN_ZMAX + 1, nchunk), 1024, 0, st>>>(N, H, Z, g_h, part);
    else k_embed_bwd_part_any<<<dim3(HGNN_ZMAX + 1, nchunk), 256, 0, st>>>(N, H, Z, g_h, part);
    HGNN_LAUNCH_CHECK("k_embed_bwd_part");
  }
  k_embed_bwd_sum<<<((HGNN_ZMAX + 1) * H + 255) / 256, 256, 0, st>>>(nchunk, H, part, g_emb);
  HGNN_LAUNCH_CHECK("k_embed_bwd_sum");
  return HGNN_OK;
}

extern "C" int32_t hgnn_embed_bwd(void* stream, int32_t N, int32_t H, const int32_t* Z, const float* g_h, float* g_emb,
                                  void* ws, size_t ws_bytes) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  HGNN_REQUIRE(N >= 0 && any_H(H), HGNN_ERR_BAD_SHAPE, "embed_bwd: bad N or H");
  HGNN_REQUIRE(g_emb && ws && (N == 0 || (Z && g_h)), HGNN_ERR_NULLPTR, "embed_bwd: null pointer");
  size_t need = 0;
  HGNN_TRY(hgnn_embed_bwd_workspace_bytes(N, H, &need));
  HGNN_REQUIRE(ws_bytes >= need, HGNN_ERR_WORKSPACE_TOO_SMALL, "embed_bwd workspace: need %zu bytes, got %zu", need, ws_bytes);
  return embed_bwd_launch(st, N, H, Z, g_h, g_emb, static_cast<float*>(ws));
}

// ---------------------------------------------------------------------------------------------
// The embedding gradient for callers that cannot allocate: the per-chunk sums live in a file-scope device array.
// In host code the array's name only stands for the symbol; the memory is reached through the address that
// hipGetSymbolAddress returns, asked for once per device (every device holds its own copy at its own address).
// ---------------------------------------------------------------------------------------------
constexpr size_t EMB_STATIC_BYTES = (size_t)HGNN_EMBED_BWD_STATIC_MAX_BYTES;
static __device__ __align__(256) unsigned char scratch[EMB_STATIC_BYTES];

static int32_t embed_static_scratch(float** out) {
  constexpr int MAX_DEV = 64;
  static void* ptr[MAX_DEV] = {};
  int dev = -1;
  HGNN_HIP(hipGetDevice(&dev));
  HGNN_REQUIRE(dev >= 0 && dev < MAX_DEV, HGNN_ERR_HIP, "embed_bwd_static: device index %d out of range", dev);
  if (!ptr[dev]) {
    void* p = nullptr;
    HGNN_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    HGNN_REQUIRE(p != nullptr, HGNN_ERR_HIP, "embed_bwd_static: no address for the scratch array");
    ptr[dev] = p;
  }
  *out = static_cast<float*>(ptr[dev]);
  return HGNN_OK;
}

extern "C" int32_t hgnn_embed_bwd_static(void* stream, int32_t N, int32_t H, const int32_t* Z, const float* g_h,
                                         float* g_emb) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  HGNN_REQUIRE(N >= 0 && any_H(H), HGNN_ERR_BAD_SHAPE, "embed_bwd_static: bad N or H");
  HGNN_REQUIRE(g_emb && (N == 0 || (Z && g_h)), HGNN_ERR_NULLPTR, "embed_bwd_static: null pointer");
  size_t need = 0;
  HGNN_TRY(hgnn_embed_bwd_workspace_bytes(N, H, &need));
  HGNN_REQUIRE(need <= EMB_STATIC_BYTES, HGNN_ERR_WORKSPACE_TOO_SMALL,
               "embed_bwd_static: N = %d, H = %d needs %zu bytes of scratch, the built-in array holds %zu "
               "(use hgnn_embed_bwd with a workspace)", N, H, need, EMB_STATIC_BYTES);
  float* part = nullptr;
  HGNN_TRY(embed_static_scratch(&part));
  return embed_bwd_launch(st, N, H, Z, g_h, g_emb, part);
}

extern "C" int32_t hgnn_pool_by_graph_fwd(void* stream, int32_t N, int32_t G, int32_t H, int32_t mode,
                                          const int32_t* graph_off, const float* h, float* p) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  HGNN_REQUIRE(N >= 0 && G >= 0 && any_H(H), HGNN_ERR_BAD_SHAPE, "pool_fwd: bad N, G or H");
  HGNN_REQUIRE(mode == HGNN_POOL_SUM || mode == HGNN_POOL_MEAN, HGNN_ERR_BAD_SHAPE, "pool_fwd: unknown mode");
  if (G == 0) return HGNN_OK;
  HGNN_REQUIRE(graph_off && p && (h || N == 0), HGNN_ERR_NULLPTR, "pool_fwd: null pointer");
  ProfScope ps(PT_POOL, st);
  // few large graphs: a workgroup per graph would leave most of the chip idle (the order of the additions, fixed in
  // either kernel, depends on which one runs, i.e. on N, G and H only)
  if (valid_H(H) && (int64_t)N >= 4096 * (int64_t)G) k_pool_fwd_tall<<<dim3(G, H / 4), 1024, 0, st>>>(H, mode, graph_off, h, p);
  else if (valid_H(H)) k_pool_fwd<<<G, 1024, 0, st>>>(H, mode, graph_off, h, p);
  else k_pool_fwd_any<<<dim3(G, (H + 63) / 64), 256, 0, st>>>(H, mode, graph_off, h, p);
  HGNN_LAUNCH_CHECK("k_pool_fwd");
  return HGNN_OK;
}

extern "C" int32_t hgnn_pool_by_graph_bwd(void* stream, int32_t N, int32_t G, int32_t H, int32_t mode,
                                          const int32_t* graph_off, const float* g_p, float* g_h, int32_t accumulate) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  HGNN_REQUIRE(N >= 0 && G >= 0 && any_H(H), HGNN_ERR_BAD_SHAPE, "pool_bwd: bad N, G or H");
  HGNN_REQUIRE(mode == HGNN_POOL_SUM || mode == HGNN_POOL_MEAN, HGNN_ERR_BAD_SHAPE, "pool_bwd: unknown mode");
  if (N == 0) return HGNN_OK;
  HGNN_REQUIRE(G > 0 && graph_off && g_p && g_h, HGNN_ERR_NULLPTR, "pool_bwd: null pointer");
  ProfScope ps(PT_POOL, st);
  if (valid_H(H)) k_pool_bwd<<<nb64((int64_t)N * (H / 4), 256), 256, 0, st>>>(N, G, H, mode, graph_off, g_p, g_h, accumulate);
  else k_pool_bwd_any<<<nb64((int64_t)N * H, 256), 256, 0, st>>>(N, G, H, mode, graph_off, g_p, g_h, accumulate);
  HGNN_LAUNCH_CHECK("k_pool_bwd");
  return HGNN_OK;
}

extern "C" int64_t hgnn_multihead_plan_ints(int32_t N, int32_t G, int32_t S) {
  if (N < 0 || G < 0 || S < 1) return -1;
  return plan_view<int32_t>(nullptr, N, G, S).ints;
}

extern "C" int32_t hgnn_multihead_plan(void* stream, int32_t N, int32_t G, int32_t S, const int32_t* graph_off,
                                       const int32_t* source_id, int32_t* plan) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  HGNN_REQUIRE(N >= 0 && G >= 0, HGNN_ERR_BAD_SHAPE, "negative N or G");
  HGNN_REQUIRE(S >= 1 && S <= 65535, HGNN_ERR_BAD_SHAPE, "S must be in 1..65535 (got %d)", S);
  HGNN_REQUIRE(plan && graph_off && (source_id || G == 0), HGNN_ERR_NULLPTR, "multihead_plan: null pointer");
  PlanView v = plan_view(plan, N, G, S);
  k_plan_graphs<<<1, 1024, 0, st>>>(G, S, graph_off, source_id, v);
  HGNN_LAUNCH_CHECK("k_plan_graphs");
  int32_t status = 0;
  HGNN_HIP(hipMemcpyAsync(&status, v.status, sizeof(status), hipMemcpyDeviceToHost, st));
  HGNN_HIP(wait_stream(st));
  HGNN_REQUIRE(status == 0, HGNN_ERR_BAD_SOURCE_ID, "a source id lies outside [0, %d)", S);
  if (N > 0) {
    k_plan_atoms<<<nb64(N, 256), 256, 0, st>>>(N, G, graph_off, v);
    HGNN_LAUNCH_CHECK("k_plan_atoms");
  }
  return HGNN_OK;
}

extern "C" int32_t hgnn_multihead_decode_workspace_bytes(int32_t N, int32_t G, int32_t H, int32_t Hh, int32_t S,
                                                         int32_t dtype, size_t* ws_bytes_host,
                                                         size_t* saved_bytes_host) {
  if (heads_need_fragment_path(H, Hh))
    return hgnn_multihead_deep_workspace_bytes(N, G, H, Hh, 1, S, dtype, ws_bytes_host, saved_bytes_host);
  HGNN_TRY(check_head_args(N, G, H, Hh, S, dtype));
  HGNN_REQUIRE(ws_bytes_host && saved_bytes_host, HGNN_ERR_NULLPTR, "null size pointer");
  *ws_bytes_host = carve_head_ws(nullptr, N, G, H, Hh, S, dtype == HGNN_BF16).bytes;
  *saved_bytes_host = carve_head_saved(nullptr, N, G, Hh).bytes;
  return HGNN_OK;
}

extern "C" int32_t hgnn_multihead_decode_fwd(void* stream, int32_t N, int32_t G, int32_t H, int32_t Hh, int32_t S,
                                             int32_t dtype, const int32_t* plan, const float* p, const float* h,
                                             const float* v, const float* Whead, float* energy, float* force,
                                             void* saved, size_t saved_bytes, void* ws, size_t ws_bytes) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (heads_need_fragment_path(H, Hh))
    return hgnn_multihead_deep_fwd(stream, N, G, H, Hh, 1, S, dtype, plan, p, h, v, Whead, energy, force, saved,
                                   saved_bytes, ws, ws_bytes);
  HGNN_TRY(check_head_args(N, G, H, Hh, S, dtype));
  if (G == 0 && N == 0) return HGNN_OK;
  HGNN_REQUIRE(plan && Whead && saved && ws, HGNN_ERR_NULLPTR, "multihead_decode_fwd: null pointer");
  HGNN_REQUIRE((G == 0 || (p && energy)) && (N == 0 || (h && v && force)), HGNN_ERR_NULLPTR,
               "multihead_decode_fwd: null pointer");
  const bool bf16 = dtype == HGNN_BF16;
  HeadWs w = carve_head_ws(ws, N, G, H, Hh, S, bf16);
  HeadSaved s = carve_head_saved(saved, N, G, Hh);
  HGNN_REQUIRE(ws_bytes >= w.bytes, HGNN_ERR_WORKSPACE_TOO_SMALL, "decode workspace: need %zu bytes, got %zu", w.bytes, ws_bytes);
  HGNN_REQUIRE(saved_bytes >= s.bytes, HGNN_ERR_WORKSPACE_TOO_SMALL, "decode saved buffer: need %zu bytes, got %zu", s.bytes, saved_bytes);
  PlanView pv = plan_view(plan, N, G, S);
  const HeadOff o(H, Hh);
  const long HH = (long)H * H;

  PackArgs pk;
  pk.src = Whead;
  pk.dst = w.packed;
  pk.nblocks = 2;
  pk.d[0] = {o.We1, Hh, 1};
  pk.d[1] = {o.Wf1, Hh, 1};
  HGNN_TRY(launch_pack(st, H, bf16, pk, S, o.per, 2 * HH));
  if (G > 0) {
    GemmArgs g;
    g.A[0] = p; g.lda[0] = H;
    g.B = w.packed; g.blk[0][0] = 0; g.grp_blk_stride = 2;
    g.row_idx = pv.graph_perm; g.grp_ptr = pv.grp_graph_ptr; g.S = S; g.M = G;
    g.bias = Whead + o.be1; g.bias_cb_mask = 1; g.grp_bias_stride = o.per;
    g.C = s.ze; g.ldc = Hh;
    HGNN_TRY(launch_gemm(st, H, bf16, g));
  }
  if (N > 0) {
    GemmArgs g;
    g.A[0] = h; g.lda[0] = H;
    g.B = w.packed; g.blk[0][0] = 1; g.grp_blk_stride = 2;
    g.row_idx = pv.atom_perm; g.grp_ptr = pv.grp_atom_ptr; g.S = S; g.M = N;
    g.bias = Whead + o.bf1; g.bias_cb_mask = 1; g.grp_bias_stride = o.per;
    g.C = s.zf; g.ldc = Hh;
    HGNN_TRY(launch_gemm(st, H, bf16, g));
  }
  ProfScope ps(PT_HEAD_OUT, st);
  k_head_out_fwd<<<nb64((int64_t)(G + N) * 64, 256), 256, 0, st>>>(N, G, Hh, s.ze, s.zf, Whead, o, pv.graph_src,
                                                                    pv.atom_graph, v, energy, force, s.q);
  HGNN_LAUNCH_CHECK("k_head_out_fwd");
  return HGNN_OK;
}

extern "C" int32_t hgnn_multihead_decode_bwd(void* stream, int32_t N, int32_t G, int32_t H, int32_t Hh, int32_t S,
                                             int32_t dtype, const int32_t* plan, const float* p, const float* h,
                                             const float* v, const float* Whead, const void* saved,
                                             size_t saved_bytes, const float* g_energy, const float* g_force,
                                             float* g_p, float* g_h, float* g_v, float* gWhead, void* ws,
                                             size_t ws_bytes) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (heads_need_fragment_path(H, Hh))
    return hgnn_multihead_deep_bwd(stream, N, G, H, Hh, 1, S, dtype, plan, p, h, v, Whead, saved, saved_bytes, g_energy,
                                   g_force, g_p, g_h, g_v, gWhead, ws, ws_bytes);
  HGNN_TRY(check_head_args(N, G, H, Hh, S, dtype));
  HGNN_REQUIRE(gWhead && Whead && ws, HGNN_ERR_NULLPTR, "multihead_decode_bwd: null pointer");
  const HeadOff o(H, Hh);
  if (G == 0 && N == 0) return launch_fill_f32(st, gWhead, o.per * S, 0.f);
  HGNN_REQUIRE(plan && saved, HGNN_ERR_NULLPTR, "multihead_decode_bwd: null pointer");
  HGNN_REQUIRE((G == 0 || (p && g_energy && g_p)) && (N == 0 || (h && v && g_force && g_h && g_v)), HGNN_ERR_NULLPTR,
               "multihead_decode_bwd: null pointer");
  const bool bf16 = dtype == HGNN_BF16;
  HeadWs w = carve_head_ws(ws, N, G, H, Hh, S, bf16);
  HeadSaved s = carve_head_saved(const_cast<void*>(saved), N, G, Hh);
  HGNN_REQUIRE(ws_bytes >= w.bytes, HGNN_ERR_WORKSPACE_TOO_SMALL, "decode workspace: need %zu bytes, got %zu", w.bytes, ws_bytes);
  HGNN_REQUIRE(saved_bytes >= s.bytes, HGNN_ERR_WORKSPACE_TOO_SMALL, "decode saved buffer: need %zu bytes, got %zu", s.bytes, saved_bytes);
  PlanView pv = plan_view(plan, N, G, S);
  const long HH = (long)H * H;

  PackArgs pk;  // transposed first layers
  pk.src = Whead;
  pk.dst = w.packed;
  pk.nblocks = 2;
  pk.d[0] = {o.We1, 1, Hh};
  pk.d[1] = {o.Wf1, 1, Hh};
  HGNN_TRY(launch_pack(st, H, bf16, pk, S, o.per, 2 * HH));

  {
  ProfScope ps(PT_HEAD_OUT, st);
  k_head_out_bwd<<<nb64((int64_t)(G + N) * 64, 256), 256, 0, st>>>(N, G, Hh, s.ze, s.zf, Whead, o, pv.graph_src,
                                                                    pv.atom_graph, v, s.q, g_energy, g_force, w.g_ze,
                                                                    w.g_zf, w.gq, g_v);
  }
  HGNN_LAUNCH_CHECK("k_head_out_bwd");

  // ---- energy branch (rows = graphs) and force branch (rows = atoms), same five steps each; their six reductions
  // of split partials (nothing here reads a result) run as one launch at the end
  ReduceQueueScope reductions(st, true);
  for (int br = 0; br < 2; ++br) {
    const bool en = br == 0;
    const int64_t M = en ? G : N;
    const int32_t* ridx = en ? pv.graph_perm : pv.atom_perm;
    const int32_t* gptr = en ? pv.grp_graph_ptr : pv.grp_atom_ptr;
    const float* X = en ? p : h;              // first-layer input
    const float* z = en ? s.ze : s.zf;
    float* gz = en ? w.g_ze : w.g_zf;
    const float* gout = en ? g_energy : w.gq;  // per-row upstream scalar
    const long oW1 = en ? o.We1 : o.Wf1, ob1 = en ? o.be1 : o.bf1, oW2 = en ? o.We2 : o.Wf2, ob2 = en ? o.be2 : o.bf2;
    if (M == 0) {
      // nothing routed anywhere: this branch's gradients are zero for every source
      for (int sidx = 0; sidx < S; ++sidx)
        HGNN_TRY(launch_fill_f32(st, gWhead + sidx * o.per + oW1, (int64_t)H * Hh + 2 * Hh + 1, 0.f));
      continue;
    }
    {  // second layer weight and bias
      ColsumArgs c;
      c.X = z; c.ldx = Hh; c.f_silu = 1; c.w = gout; c.row_idx = ridx; c.grp_ptr = gptr; c.S = S; c.M = M;
      c.dest = gWhead + oW2; c.grp_dest_stride = o.per; c.partial = w.pcs[br][0];
      HGNN_TRY(launch_colsum(st, Hh, c));
      k_group_scalar_sum<<<S, 1024, 0, st>>>(gout, ridx, gptr, gWhead + ob2, o.per);
      HGNN_LAUNCH_CHECK("k_group_scalar_sum");
    }
    {  // first layer bias and weight
      ColsumArgs c;
      c.X = gz; c.ldx = Hh; c.row_idx = ridx; c.grp_ptr = gptr; c.S = S; c.M = M;
      c.dest = gWhead + ob1; c.grp_dest_stride = o.per; c.partial = w.pcs[br][1];
      HGNN_TRY(launch_colsum(st, Hh, c));
      WgradArgs a;
      a.A[0] = X; a.lda[0] = H;
      a.B[0] = gz; a.ldb[0] = Hh;
      a.row_idx = ridx; a.grp_ptr = gptr; a.S = S; a.M = M;
      a.dest[0] = gWhead + oW1; a.grp_dest_stride = o.per;
      a.partial = w.pwg[br];
      HGNN_TRY(launch_wgrad(st, H, bf16, a));
    }
    {  // input gradient
      GemmArgs g;
      g.A[0] = gz; g.lda[0] = Hh;
      g.B = w.packed; g.blk[0][0] = en ? 0 : 1; g.grp_blk_stride = 2;
      g.row_idx = ridx; g.grp_ptr = gptr; g.S = S; g.M = (int)M;
      g.C = en ? g_p : g_h; g.ldc = H;
      HGNN_TRY(launch_gemm(st, H, bf16, g));
    }
  }
  {
    ProfScope ps(PT_COLSUM, st);
    HGNN_TRY(reductions.flush());
  }
  return HGNN_OK;
}
