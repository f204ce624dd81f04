// Radius graph on the GPU: cell-list candidate search, exact float32 cutoff test, destination-sorted
// CSR with rows ordered by (source, shift), and the source-sorted transpose plan.
//
// Design for gfx950: atoms are sorted by bin (bins live in fractional coordinates of the graph's cell, at least
// one cutoff wide wherever the cell allows it; cells thinner than the cutoff are covered by integer image shifts
// instead) into an array of (x, y, z, atom) quadruples, so a bin's atoms are one contiguous run of 16-byte records.
// A workgroup takes up to 16 destination atoms of ONE bin: it stages the shifted positions of every candidate of
// the (2R+1)^3 bins around it in LDS once (coalesced loads, no pointer chasing) and each wavefront then tests
// whole groups of 64 candidates per destination atom out of LDS; hits are compacted with a ballot into a per-
// wavefront LDS row, ranked there against each other (rows are short) and written out in (source, shift) order.
// The same kernel counts (first call) and fills (second call). Rows with more hits than the LDS row holds go
// through a slower path that ranks from memory. Only integer atomics are used (bin histogram / cursors); the
// output does not depend on their order.
//
// The cutoff test is the one fixed in include/hgnn.h: each float operation is an explicitly rounded
// intrinsic so that the compiler cannot contract them into fused multiply-adds.
#include "common.h"
#include "prof.h"

namespace hgnn {

// ---------------------------------------------------------------------------------------------
// error text (thread local), shared by all translation units
// ---------------------------------------------------------------------------------------------
static thread_local char g_err[512] = "";

int32_t set_error(int32_t code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

// ---------------------------------------------------------------------------------------------
// exclusive scan (three small kernels; block sums kept in int64 so that overflow is detectable)
// ---------------------------------------------------------------------------------------------
constexpr int SCAN_T = 256;
constexpr int SCAN_PER = 4;
constexpr int SCAN_BLK = SCAN_T * SCAN_PER;

__device__ inline int block_exclusive_scan_256(int v, int* total, int* sh) {
  // sh: 256 ints. Hillis-Steele inclusive scan, then shift.
  const int t = threadIdx.x;
  sh[t] = v;
  __syncthreads();
  for (int o = 1; o < SCAN_T; o <<= 1) {
    int add = (t >= o) ? sh[t - o] : 0;
    __syncthreads();
    sh[t] += add;
    __syncthreads();
  }
  int incl = sh[t];
  *total = sh[SCAN_T - 1];
  __syncthreads();
  return incl - v;
}

__global__ void k_scan_local(const int32_t* __restrict__ in, int32_t* __restrict__ out, int64_t n,
                             long long* __restrict__ blocksum) {
  __shared__ int sh[SCAN_T];
  const int64_t base = (int64_t)blockIdx.x * SCAN_BLK + (int64_t)threadIdx.x * SCAN_PER;
  int v[SCAN_PER];
  int s = 0;
#pragma unroll
  for (int k = 0; k < SCAN_PER; ++k) {
    v[k] = (base + k < n) ? in[base + k] : 0;
    s += v[k];
  }
  int tot;
  int ex = block_exclusive_scan_256(s, &tot, sh);
#pragma unroll
  for (int k = 0; k < SCAN_PER; ++k) {
    if (base + k < n) out[base + k] = ex;
    ex += v[k];
  }
  if (threadIdx.x == 0) blocksum[blockIdx.x] = tot;
}

__global__ void k_scan_blocksums(long long* __restrict__ blocksum, int64_t nb) {
  // single thread block; serial carry over chunks of 256 block sums (nb is small)
  __shared__ long long sh[SCAN_T];
  __shared__ long long carry;
  if (threadIdx.x == 0) carry = 0;
  __syncthreads();
  for (int64_t c0 = 0; c0 < nb; c0 += SCAN_T) {
    const int64_t idx = c0 + threadIdx.x;
    long long v = idx < nb ? blocksum[idx] : 0;
    sh[threadIdx.x] = v;
    __syncthreads();
    for (int o = 1; o < SCAN_T; o <<= 1) {
      long long add = (threadIdx.x >= o) ? sh[threadIdx.x - o] : 0;
      __syncthreads();
      sh[threadIdx.x] += add;
      __syncthreads();
    }
    long long incl = sh[threadIdx.x];
    long long c = carry;
    if (idx < nb) blocksum[idx] = c + incl - v;
    __syncthreads();
    if (threadIdx.x == SCAN_T - 1) carry = c + incl;
    __syncthreads();
  }
  if (threadIdx.x == 0) blocksum[nb] = carry;  // grand total
}

__global__ void k_scan_add(int32_t* __restrict__ out, int64_t n, const long long* __restrict__ blocksum,
                           int64_t nb) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) out[i] = (int32_t)(out[i] + blocksum[i / SCAN_BLK]);
  if (i == n) out[n] = (int32_t)blocksum[nb];
}

size_t scan_scratch_ints(int64_t n) {
  int64_t nb = (n + SCAN_BLK - 1) / SCAN_BLK;
  return (size_t)(2 * (nb + 2));  // int64 entries counted in int32 units
}

// short inputs: one workgroup walks the array in chunks of SCAN_BLK with a running carry (one launch instead of three);
// leaves the same block sums and grand total behind as the three-kernel form
__global__ void k_scan_small(const int32_t* __restrict__ in, int32_t* __restrict__ out, int64_t n,
                             long long* __restrict__ blocksum) {
  __shared__ int sh[SCAN_T];
  long long carry = 0;
  const int64_t nb = (n + SCAN_BLK - 1) / SCAN_BLK;
  for (int64_t b = 0; b < nb; ++b) {
    const int64_t base = b * SCAN_BLK + (int64_t)threadIdx.x * SCAN_PER;
    int v[SCAN_PER];
    int s = 0;
#pragma unroll
    for (int k = 0; k < SCAN_PER; ++k) {
      v[k] = (base + k < n) ? in[base + k] : 0;
      s += v[k];
    }
    int tot;
    int ex = block_exclusive_scan_256(s, &tot, sh);
#pragma unroll
    for (int k = 0; k < SCAN_PER; ++k) {
      if (base + k < n) out[base + k] = (int32_t)(carry + ex);
      ex += v[k];
    }
    if (threadIdx.x == 0) blocksum[b] = carry;
    carry += tot;
  }
  if (threadIdx.x == 0) {
    blocksum[nb] = carry;
    out[n] = (int32_t)carry;
  }
}
constexpr int64_t SCAN_SMALL_MAX = 16 * SCAN_BLK;

int32_t exclusive_scan_i32(hipStream_t st, const int32_t* in, int32_t* out, int64_t n, int32_t* scratch) {
  long long* bs = reinterpret_cast<long long*>(scratch);
  int64_t nb = (n + SCAN_BLK - 1) / SCAN_BLK;
  if (n <= SCAN_SMALL_MAX) {
    k_scan_small<<<dim3(1), dim3(SCAN_T), 0, st>>>(in, out, n, bs);
    HGNN_LAUNCH_CHECK("k_scan_small");
    return HGNN_OK;
  }
  if (nb > 0) {
    k_scan_local<<<dim3((unsigned)nb), dim3(SCAN_T), 0, st>>>(in, out, n, bs);
    HGNN_LAUNCH_CHECK("k_scan_local");
  }
  k_scan_blocksums<<<dim3(1), dim3(SCAN_T), 0, st>>>(bs, nb);
  HGNN_LAUNCH_CHECK("k_scan_blocksums");
  int64_t tot = n + 1;
  k_scan_add<<<dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, st>>>(out, n, bs, nb);
  HGNN_LAUNCH_CHECK("k_scan_add");
  return HGNN_OK;
}

// ---------------------------------------------------------------------------------------------
// per-graph metadata
// ---------------------------------------------------------------------------------------------
struct GMeta {
  float cell[9];   // rows a, b, c (zeros when not periodic)
  float inv[9];    // fractional = (pos - org) * inv   (row vector times matrix)
  float org[3];
  int nb[3];       // bins per lattice direction
  int R[3];        // search reach in bins
  int bin_off;     // first global bin of this graph (filled after the scan)
  int periodic;
  int lo, hi;      // atom range
};

enum : int {
  ST_BAD_OFFSETS = 1,
  ST_BAD_CELL = 2,
  ST_OUT_OF_CELL = 4,
};
// periodic atoms must lie inside their cell: fractional coordinates within this distance of [0, 1]
constexpr float FRAC_TOL = 1e-5f;

constexpr float BIN_MARGIN = 1.001f;  // bins are at least 1.001 * rc wide: absorbs float32 binning error
constexpr int NB_MAX = 256;

// two ranges in one launch (n2 <= n1)
__global__ void k_fill2_i32(int32_t* p1, int64_t n1, int32_t* p2, int64_t n2, int32_t v) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n1) p1[i] = v;
  if (i < n2) p2[i] = v;
}
__global__ void k_fill_i32(int32_t* p, int64_t n, int32_t v) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

__device__ inline float wave_min(float x) {
  for (int o = 32; o > 0; o >>= 1) x = fminf(x, __shfl_xor(x, o));
  return x;
}
__device__ inline float wave_max(float x) {
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
  return x;
}

// one wavefront (block of 64) per graph
__global__ void k_graph_meta(int N, int G, const float* __restrict__ pos, const int32_t* __restrict__ graph_off,
                             const float* __restrict__ cell, const uint8_t* __restrict__ pbc, float rc,
                             GMeta* __restrict__ meta, int32_t* __restrict__ nbins, int32_t* __restrict__ status) {
  const int g = blockIdx.x;
  const int lane = threadIdx.x;
  int lo = graph_off[g], hi = graph_off[g + 1];
  bool bad = (lo > hi) || (lo < 0) || (hi > N) || (g == 0 && lo != 0) || (g == G - 1 && hi != N);
  if (bad) {
    if (lane == 0) {
      atomicOr(status, ST_BAD_OFFSETS);
      GMeta m = {};
      m.nb[0] = m.nb[1] = m.nb[2] = 1;
      meta[g] = m;
      nbins[g] = 1;
    }
    return;
  }
  const bool periodic = (pbc != nullptr) && (cell != nullptr) && (pbc[g] != 0);
  float mn[3] = {3.0e38f, 3.0e38f, 3.0e38f}, mx[3] = {-3.0e38f, -3.0e38f, -3.0e38f};
  if (!periodic) {
    for (int i = lo + lane; i < hi; i += 64) {
#pragma unroll
      for (int c = 0; c < 3; ++c) {
        float x = pos[3 * (size_t)i + c];
        mn[c] = fminf(mn[c], x);
        mx[c] = fmaxf(mx[c], x);
      }
    }
#pragma unroll
    for (int c = 0; c < 3; ++c) {
      mn[c] = wave_min(mn[c]);
      mx[c] = wave_max(mx[c]);
    }
  }
  if (lane != 0) return;
  GMeta m = {};
  m.lo = lo;
  m.hi = hi;
  m.periodic = periodic ? 1 : 0;
  const double rcm = (double)rc * (double)BIN_MARGIN;
  double hgt[3];
  if (periodic) {
    double C[9];
    for (int k = 0; k < 9; ++k) {
      m.cell[k] = cell[9 * (size_t)g + k];
      C[k] = (double)m.cell[k];
    }
    // cross products of the other two lattice vectors
    double cr[3][3];
    for (int k = 0; k < 3; ++k) {
      const double* u = &C[3 * ((k + 1) % 3)];
      const double* w = &C[3 * ((k + 2) % 3)];
      cr[k][0] = u[1] * w[2] - u[2] * w[1];
      cr[k][1] = u[2] * w[0] - u[0] * w[2];
      cr[k][2] = u[0] * w[1] - u[1] * w[0];
    }
    double det = C[0] * cr[0][0] + C[1] * cr[0][1] + C[2] * cr[0][2];
    if (!(fabs(det) >= 1e-6)) {
      atomicOr(status, ST_BAD_CELL);
      m.nb[0] = m.nb[1] = m.nb[2] = 1;
      m.periodic = 0;
      meta[g] = m;
      nbins[g] = 1;
      return;
    }
    // inverse: column k of C^-1 is cr[k] / det  (f_k = (pos . cr[k]) / det)
    for (int k = 0; k < 3; ++k) {
      double nrm = sqrt(cr[k][0] * cr[k][0] + cr[k][1] * cr[k][1] + cr[k][2] * cr[k][2]);
      hgt[k] = fabs(det) / nrm;
      for (int c = 0; c < 3; ++c) m.inv[3 * c + k] = (float)(cr[k][c] / det);
    }
    m.org[0] = m.org[1] = m.org[2] = 0.f;
  } else {
    for (int c = 0; c < 3; ++c) {
      if (hi == lo) { mn[c] = 0.f; mx[c] = 0.f; }
      double ext = (double)mx[c] - (double)mn[c];
      double pad = 1e-3 * (1.0 + ext);
      hgt[c] = ext + 2.0 * pad;
      m.org[c] = (float)((double)mn[c] - pad);
      m.inv[3 * c + c] = (float)(1.0 / hgt[c]);
    }
  }
  long long nat = hi - lo;
  int nb[3];
  for (int k = 0; k < 3; ++k) {
    double q = floor(hgt[k] / rcm);
    nb[k] = q < 1.0 ? 1 : (q > (double)NB_MAX ? NB_MAX : (int)q);
  }
  // keep the number of bins proportional to the number of atoms (bounded workspace)
  long long cap = 4 * nat > 1 ? 4 * nat : 1;
  while ((long long)nb[0] * nb[1] * nb[2] > cap) {
    int k = (nb[0] >= nb[1] && nb[0] >= nb[2]) ? 0 : (nb[1] >= nb[2] ? 1 : 2);
    nb[k] -= 1;
  }
  for (int k = 0; k < 3; ++k) {
    double w = hgt[k] / nb[k];
    int R = (int)ceil(rcm / w);
    if (R < 1) R = 1;
    if (!periodic && R > nb[k] - 1) R = nb[k] - 1;  // nothing outside the bounding box
    if (R > 127) {
      atomicOr(status, ST_BAD_CELL);
      R = 0;
    }
    m.nb[k] = nb[k];
    m.R[k] = R;
  }
  meta[g] = m;
  nbins[g] = nb[0] * nb[1] * nb[2];
}

__global__ void k_set_bin_off(int G, GMeta* __restrict__ meta, const int32_t* __restrict__ bin_off) {
  int g = blockIdx.x * blockDim.x + threadIdx.x;
  if (g < G) meta[g].bin_off = bin_off[g];
}

__device__ inline int find_graph(const int32_t* __restrict__ graph_off, int G, int i) {
  // largest g with graph_off[g] <= i  (empty graphs share an offset; the last of them wins, and its
  // successor is the one that really holds atom i) -> search for the first g with graph_off[g+1] > i
  int lo = 0, hi = G - 1;
  while (lo < hi) {
    int mid = (lo + hi) >> 1;
    if (graph_off[mid + 1] > i) hi = mid; else lo = mid + 1;
  }
  return lo;
}

__global__ void k_bin_atoms_count(int N, int G, const float* __restrict__ pos, const int32_t* __restrict__ graph_off,
                                  const GMeta* __restrict__ meta, int32_t* __restrict__ atom_graph,
                                  int32_t* __restrict__ atom_bin, int32_t* __restrict__ bin_cnt,
                                  int32_t* __restrict__ status) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= N) return;
  int g = find_graph(graph_off, G, i);
  const GMeta& m = meta[g];
  float d[3] = {pos[3 * (size_t)i] - m.org[0], pos[3 * (size_t)i + 1] - m.org[1], pos[3 * (size_t)i + 2] - m.org[2]};
  int b[3];
  bool outside = false;
#pragma unroll
  for (int k = 0; k < 3; ++k) {
    float f = d[0] * m.inv[k] + d[1] * m.inv[3 + k] + d[2] * m.inv[6 + k];
    outside = outside || !(f >= -FRAC_TOL && f <= 1.0f + FRAC_TOL);   // also catches NaN
    int q = (int)floorf(f * (float)m.nb[k]);
    b[k] = q < 0 ? 0 : (q >= m.nb[k] ? m.nb[k] - 1 : q);
  }
  if (outside && m.periodic) atomicOr(status, ST_OUT_OF_CELL);
  int bin = m.bin_off + (b[0] * m.nb[1] + b[1]) * m.nb[2] + b[2];
  atom_graph[i] = g;
  atom_bin[i] = bin;
  atomicAdd(&bin_cnt[bin], 1);
}

// atoms in bin order: their index (for the slow path) and (x, y, z, index) as one 16-byte record
__global__ void k_bin_atoms_fill(int N, const float* __restrict__ pos, const int32_t* __restrict__ atom_bin,
                                 const int32_t* __restrict__ bin_start, int32_t* __restrict__ bin_cur,
                                 int32_t* __restrict__ bin_atoms, float4* __restrict__ spos) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= N) return;
  int bin = atom_bin[i];
  int k = bin_start[bin] + atomicAdd(&bin_cur[bin], 1);
  bin_atoms[k] = i;
  spos[k] = make_float4(pos[3 * (size_t)i], pos[3 * (size_t)i + 1], pos[3 * (size_t)i + 2], __int_as_float(i));
}

// work list of the search: one entry per SR_HOME destination atoms of a non-empty bin (order does not matter)
constexpr int SR_HOME = 16;
__global__ void k_bin_list(int64_t maxbins, const int32_t* __restrict__ bin_cnt, int32_t* __restrict__ nlist,
                           int2* __restrict__ list) {
  const int64_t b = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= maxbins) return;
  const int c = bin_cnt[b];
  if (c <= 0) return;
  const int n = (c + SR_HOME - 1) / SR_HOME;
  const int at = atomicAdd(nlist, n);
  for (int k = 0; k < n; ++k) list[at + k] = make_int2((int)b, k * SR_HOME);
}

// ---------------------------------------------------------------------------------------------
// search: one workgroup per (bin, up to SR_HOME destination atoms), candidates staged in LDS
// ---------------------------------------------------------------------------------------------
__device__ inline int floordiv(int a, int b) { return (a >= 0) ? a / b : -((-a + b - 1) / b); }

constexpr int SR_CHUNK = 1024;   // candidates staged at once
constexpr int SR_EXT = 256;      // bins of the (2R+1)^3 block enumerated at once (one per thread)
constexpr int SR_CAP = 256;      // hits of one row that the LDS row holds; longer rows take the slow path
constexpr int SR_ZERO_CODE = (128 << 16) | (128 << 8) | 128;
constexpr int SR_GRID = 2048;    // workgroups of the search (they walk the work list with this stride)

struct SearchLds {
  __align__(16) unsigned long long row[4][SR_CAP + 4];   // per wavefront: (atom << 24 | code) of the hits of one row
  float cx[SR_CHUNK], cy[SR_CHUNK], cz[SR_CHUNK];   // shifted candidate positions  pos_j + t
  int cj[SR_CHUNK], cc[SR_CHUNK];                   // candidate atom and shift code
  int ch[SR_CHUNK];                                 // hits of each staged candidate in this work item (then, in the
                                                    // filling pass: the candidate's first place in its source group)
  unsigned short rowk[4][SR_CAP];                   // per wavefront: candidate slot of each hit of the row at hand
  unsigned short rinfo[SR_HOME][SR_CAP];            // per destination atom and edge: slot | place among the item's hits << 10
  int rstart[SR_HOME], rcnt[SR_HOME];               // first edge and edge count of the item's rows (0: row not dealt here)
  int ext_start[SR_EXT];                            // first record of each enumerated bin
  int ext_pref[SR_EXT + 1];                         // exclusive prefix of their atom counts
  int ext_code[SR_EXT];
  float ext_t[3][SR_EXT];                           // shift vector t = (s0*a + s1*b) + s2*c
  int scan[4];
};

struct SearchArgs {
  int N;
  const float* pos;
  const GMeta* meta;
  const int32_t* atom_graph;
  const int32_t* bin_start;
  const float4* spos;
  const int32_t* nlist;
  const int2* list;
  const int32_t* status;
  float rc;
  // count
  int32_t* deg;
  int32_t* colT_cnt;
  // fill
  const int32_t* row_ptr;
  int32_t* dst;
  int32_t* col;
  int8_t* shift;
  float* d2;
  float* rvec;
  const int32_t* colT_ptr;   // fill: first place of each source's group
  int32_t* colT_cur;         // fill: places of each group handed out so far
  int32_t* unsorted;         // fill: the groups' edges in the order they were dealt
  int32_t* novf;       // number of rows left to the slow path
  int32_t* ovf_rows;   // those rows
};

// t = (s0*a + s1*b) + s2*c, every operation rounded on its own
__device__ __forceinline__ void shift_vector(const float* cell, int s0, int s1, int s2, float& tx, float& ty, float& tz) {
  const float f0 = (float)s0, f1 = (float)s1, f2 = (float)s2;
  tx = __fadd_rn(__fadd_rn(__fmul_rn(f0, cell[0]), __fmul_rn(f1, cell[3])), __fmul_rn(f2, cell[6]));
  ty = __fadd_rn(__fadd_rn(__fmul_rn(f0, cell[1]), __fmul_rn(f1, cell[4])), __fmul_rn(f2, cell[7]));
  tz = __fadd_rn(__fadd_rn(__fmul_rn(f0, cell[2]), __fmul_rn(f1, cell[5])), __fmul_rn(f2, cell[8]));
}

template <bool FILL>
__global__ void __launch_bounds__(256) k_search(SearchArgs p) {
  __shared__ SearchLds L;
  if (p.status[0] != 0) return;          // bad input: the host reports it, nothing is searched
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nlist = *p.nlist;
  const float rc2 = __fmul_rn(p.rc, p.rc);
  unsigned long long* row = L.row[wave];
  for (int item = blockIdx.x; item < nlist; item += gridDim.x) {
    const int2 it = p.list[item];
    const int hb = it.x, h0 = it.y;
    const int hb_start = p.bin_start[hb];
    const int hb_cnt = p.bin_start[hb + 1] - hb_start;
    const int nhome = hb_cnt - h0 < SR_HOME ? hb_cnt - h0 : SR_HOME;
    const int i_first = __float_as_int(p.spos[hb_start].w);
    const GMeta& m = p.meta[p.atom_graph[i_first]];
    const int nb0 = m.nb[0], nb1 = m.nb[1], nb2 = m.nb[2];
    const int R0 = m.R[0], R1 = m.R[1], R2 = m.R[2];
    const int lb = hb - m.bin_off;
    const int b2 = lb % nb2, b1 = (lb / nb2) % nb1, b0 = lb / (nb1 * nb2);
    const int n1 = 2 * R1 + 1, n2 = 2 * R2 + 1;
    const int next = (2 * R0 + 1) * n1 * n2;
    const bool per = m.periodic != 0;
    float cell[9];
#pragma unroll
    for (int k = 0; k < 9; ++k) cell[k] = m.cell[k];

    // bins eg .. eg+SR_EXT-1 of the block around the home bin: record range, shift, prefix of the atom counts.
    // Returns the number of candidates they hold. All threads call it (it synchronises).
    auto enumerate = [&](int eg) -> int {
      const int q = eg + tid;
      int count = 0, start = 0, code = SR_ZERO_CODE;
      float tx = 0.f, ty = 0.f, tz = 0.f;
      if (q < next) {
        const int d0 = q / (n1 * n2), d1 = (q / n2) % n1, d2 = q % n2;
        const int B0 = b0 + d0 - R0, B1 = b1 + d1 - R1, B2 = b2 + d2 - R2;
        int s0 = 0, s1 = 0, s2 = 0, c0 = B0, c1 = B1, c2 = B2;
        bool ok = true;
        if (per) {
          s0 = floordiv(B0, nb0); c0 = B0 - s0 * nb0;
          s1 = floordiv(B1, nb1); c1 = B1 - s1 * nb1;
          s2 = floordiv(B2, nb2); c2 = B2 - s2 * nb2;
        } else {
          ok = B0 >= 0 && B0 < nb0 && B1 >= 0 && B1 < nb1 && B2 >= 0 && B2 < nb2;
        }
        if (ok) {
          const int bin = m.bin_off + (c0 * nb1 + c1) * nb2 + c2;
          start = p.bin_start[bin];
          count = p.bin_start[bin + 1] - start;
          code = ((s0 + 128) << 16) | ((s1 + 128) << 8) | (s2 + 128);
          shift_vector(cell, s0, s1, s2, tx, ty, tz);
        }
      }
      // exclusive scan over the 256 threads: inside each wavefront by lane shifts, then the four wavefront totals
      int incl = count;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int up = __shfl_up(incl, o);
        if (lane >= o) incl += up;
      }
      if (lane == 63) L.scan[wave] = incl;
      __syncthreads();
      const int w0 = L.scan[0], w1 = L.scan[1], w2 = L.scan[2], w3 = L.scan[3];
      const int total = w0 + w1 + w2 + w3;
      const int ex = incl - count + (wave > 0 ? w0 : 0) + (wave > 1 ? w1 : 0) + (wave > 2 ? w2 : 0);
      L.ext_start[tid] = start;
      L.ext_pref[tid] = ex;
      L.ext_code[tid] = code;
      L.ext_t[0][tid] = tx; L.ext_t[1][tid] = ty; L.ext_t[2][tid] = tz;
      if (tid == 0) L.ext_pref[SR_EXT] = total;
      __syncthreads();
      return total;
    };
    // candidates c0 .. c0+n-1 of the enumerated bins -> LDS (all threads; the caller synchronises)
    auto stage = [&](int c0, int n) {
      if (next <= 32 && c0 == 0 && n == L.ext_pref[SR_EXT]) {
        // few bins and all their atoms at once: eight threads per bin copy its run, no search for the owner
        const int eb = tid >> 3;
        const int lo = L.ext_pref[eb], cnt = L.ext_pref[eb + 1] - lo, src = L.ext_start[eb];
        const float tx = L.ext_t[0][eb], ty = L.ext_t[1][eb], tz = L.ext_t[2][eb];
        const int code = L.ext_code[eb];
        for (int a = tid & 7; a < cnt; a += 8) {
          const float4 r = p.spos[src + a];
          L.cx[lo + a] = __fadd_rn(r.x, tx);
          L.cy[lo + a] = __fadd_rn(r.y, ty);
          L.cz[lo + a] = __fadd_rn(r.z, tz);
          L.cj[lo + a] = __float_as_int(r.w);
          L.cc[lo + a] = code;
        }
        return;
      }
      for (int k = tid; k < n; k += 256) {
        const int q = c0 + k;
        int lo = 0, hi = SR_EXT;               // last bin with ext_pref <= q (bins without atoms share a prefix)
        while (hi - lo > 1) {
          const int mid = (lo + hi) >> 1;
          if (L.ext_pref[mid] <= q) lo = mid; else hi = mid;
        }
        const float4 a = p.spos[L.ext_start[lo] + (q - L.ext_pref[lo])];
        L.cx[k] = __fadd_rn(a.x, L.ext_t[0][lo]);
        L.cy[k] = __fadd_rn(a.y, L.ext_t[1][lo]);
        L.cz[k] = __fadd_rn(a.z, L.ext_t[2][lo]);
        L.cj[k] = __float_as_int(a.w);
        L.cc[k] = L.ext_code[lo];
      }
    };
    // this wavefront's destination atom against the n staged candidates; cnt = hits so far
    // lds_hist (counting pass): a hit adds to the candidate's LDS counter (flushed by the caller) instead of to the
    // source histogram in memory
    auto scan = [&](int i, float pix, float piy, float piz, int n, int& cnt, bool lds_hist) {
      for (int k0 = 0; k0 < n; k0 += 256) {
        // four groups of 64 candidates: their LDS reads are in flight together
        int jj[4], cd[4];
        float qx[4], qy[4], qz[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int k = k0 + 64 * u + lane;
          const int kk = k < n ? k : 0;
          jj[u] = L.cj[kk]; cd[u] = L.cc[kk];
          qx[u] = L.cx[kk]; qy[u] = L.cy[kk]; qz[u] = L.cz[kk];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          if (k0 + 64 * u >= n) break;                       // uniform
          const int k = k0 + 64 * u + lane;
          const float rx = __fsub_rn(pix, qx[u]), ry = __fsub_rn(piy, qy[u]), rz = __fsub_rn(piz, qz[u]);
          const float dd = __fadd_rn(__fadd_rn(__fmul_rn(rx, rx), __fmul_rn(ry, ry)), __fmul_rn(rz, rz));
          const bool hit = k < n && (dd < rc2) && !(cd[u] == SR_ZERO_CODE && jj[u] == i);
          const unsigned long long mask = __ballot(hit);
          if (hit) {
            if (FILL) {
              const int at = cnt + __popcll(mask & ((1ull << lane) - 1ull));
              if (at < SR_CAP) {
                row[at] = ((unsigned long long)(unsigned)jj[u] << 24) | (unsigned)cd[u];
                L.rowk[wave][at] = (unsigned short)k;
              }
            } else if (lds_hist) {
              atomicAdd(&L.ch[k], 1);
            } else {
              atomicAdd(&p.colT_cnt[jj[u]], 1);
            }
          }
          cnt += __popcll(mask);
        }
      }
    };
    // the row is complete: count, or order it and write the edges
    // h >= 0: the row's edges are dealt to their sources at the end of the work item (slot and place kept in LDS);
    // h < 0 (candidates streamed in chunks): every edge takes its place with an addition of its own
    auto finish = [&](int i, float pix, float piy, float piz, int cnt, int h) {
      if (!FILL) {
        if (lane == 0) p.deg[i] = cnt;
        return;
      }
      if (cnt > SR_CAP) {
        if (lane == 0) p.ovf_rows[atomicAdd(p.novf, 1)] = i;
        if (h >= 0 && lane == 0) L.rcnt[h] = 0;
        return;
      }
      if (lane < 3) row[cnt + lane] = ~0ull;   // pad to a multiple of four for the 16-byte reads below
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
      __builtin_amdgcn_wave_barrier();
      const int start = p.row_ptr[i];
      if (h >= 0 && lane == 0) {
        L.rstart[h] = start;
        L.rcnt[h] = cnt;
      }
      for (int t = lane; t < cnt; t += 64) {
        const unsigned long long key = row[t];
        int rank = 0;
        for (int u = 0; u < cnt; u += 4) {
          const ulonglong2 ka = *reinterpret_cast<const ulonglong2*>(&row[u]);
          const ulonglong2 kb = *reinterpret_cast<const ulonglong2*>(&row[u + 2]);
          rank += (ka.x < key) + (ka.y < key) + (kb.x < key) + (kb.y < key);
        }
        const int e = start + rank;
        const int mj = (int)(key >> 24), mc = (int)(key & 0xffffffu);
        const int s0 = ((mc >> 16) & 255) - 128, s1 = ((mc >> 8) & 255) - 128, s2 = (mc & 255) - 128;
        float tx, ty, tz;
        shift_vector(cell, s0, s1, s2, tx, ty, tz);
        const float qx = __fadd_rn(p.pos[3 * (size_t)mj], tx);
        const float qy = __fadd_rn(p.pos[3 * (size_t)mj + 1], ty);
        const float qz = __fadd_rn(p.pos[3 * (size_t)mj + 2], tz);
        const float rx = __fsub_rn(pix, qx), ry = __fsub_rn(piy, qy), rz = __fsub_rn(piz, qz);
        const float dd = __fadd_rn(__fadd_rn(__fmul_rn(rx, rx), __fmul_rn(ry, ry)), __fmul_rn(rz, rz));
        if (h >= 0) {
          const int k = L.rowk[wave][t];
          const int place = atomicAdd(&L.ch[k], 1);   // < SR_HOME: a destination atom hits a slot once
          L.rinfo[h][rank] = (unsigned short)(k | (place << 10));
        } else {
          p.unsorted[p.colT_ptr[mj] + atomicAdd(&p.colT_cur[mj], 1)] = e;
        }
        p.dst[e] = i;
        p.col[e] = mj;
        p.shift[3 * (size_t)e] = (int8_t)s0;
        p.shift[3 * (size_t)e + 1] = (int8_t)s1;
        p.shift[3 * (size_t)e + 2] = (int8_t)s2;
        p.d2[e] = dd;
        p.rvec[3 * (size_t)e] = rx;
        p.rvec[3 * (size_t)e + 1] = ry;
        p.rvec[3 * (size_t)e + 2] = rz;
      }
      __builtin_amdgcn_wave_barrier();   // the row buffer is reused by the next destination atom
    };

    const int nrounds = (nhome + 3) >> 2;          // four destination atoms (one per wavefront) per round
    const int total0 = enumerate(0);
    if (next <= SR_EXT && total0 <= SR_CHUNK) {
      // the usual case: every candidate fits in LDS at once; staged once, then the wavefronts run on their own
      stage(0, total0);
      for (int k = tid; k < total0; k += 256) L.ch[k] = 0;
      __syncthreads();
      for (int r = 0; r < nrounds; ++r) {
        const int h = 4 * r + wave;
        if (h >= nhome) break;
        const float4 a = p.spos[hb_start + h0 + h];
        const int i = __float_as_int(a.w);
        int cnt = 0;
        scan(i, a.x, a.y, a.z, total0, cnt, true);
        finish(i, a.x, a.y, a.z, cnt, h);
      }
      if (!FILL) {
        // the source histogram: one addition per candidate that was hit (a candidate is hit by up to 16 destination
        // atoms of the work item), not one per hit
        __syncthreads();
        for (int k = tid; k < total0; k += 256) {
          const int c = L.ch[k];
          if (c) atomicAdd(&p.colT_cnt[L.cj[k]], c);
        }
      } else {
        // transpose plan: every candidate that was hit takes its places in its source group with one addition, then
        // the item's edges go to their places (any order inside a group: the groups are put in edge order afterwards)
        __syncthreads();
        for (int k = tid; k < total0; k += 256) {
          const int c = L.ch[k];
          if (c) L.ch[k] = atomicAdd(&p.colT_cur[L.cj[k]], c);
        }
        __syncthreads();
        for (int h = wave; h < nhome; h += 4) {
          const int cnt = L.rcnt[h], start = L.rstart[h];
          for (int t = lane; t < cnt; t += 64) {
            const int info = L.rinfo[h][t];
            const int k = info & 1023;
            p.unsorted[p.colT_ptr[L.cj[k]] + L.ch[k] + (info >> 10)] = start + t;
          }
        }
      }
    } else {
      // many periodic images or a crowded bin: the candidates are streamed through LDS in chunks, once per round
      for (int r = 0; r < nrounds; ++r) {
        const int h = 4 * r + wave;
        const bool on = h < nhome;
        float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
        if (on) a = p.spos[hb_start + h0 + h];
        const int i = __float_as_int(a.w);
        int cnt = 0;
        for (int eg = 0; eg < next; eg += SR_EXT) {
          const int total = (eg == 0 && r == 0) ? total0 : enumerate(eg);
          for (int c0 = 0; c0 < total; c0 += SR_CHUNK) {
            const int n = total - c0 < SR_CHUNK ? total - c0 : SR_CHUNK;
            __syncthreads();               // the previous chunk has been read by every wavefront
            stage(c0, n);
            __syncthreads();
            if (on) scan(i, a.x, a.y, a.z, n, cnt, false);
          }
          __syncthreads();                 // before the bin table is overwritten
        }
        if (on) finish(i, a.x, a.y, a.z, cnt, -1);
      }
    }
    __syncthreads();                       // before the next work item reuses the tables
  }
}

// ---------------------------------------------------------------------------------------------
// slow path for rows longer than the LDS row: one wavefront per listed row walks the bins from memory,
// stores the hits unordered and ranks them from memory
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
k_long_rows(const int32_t* __restrict__ novf, const int32_t* __restrict__ ovf_rows, const float* __restrict__ pos,
            const GMeta* __restrict__ meta, const int32_t* __restrict__ atom_graph,
            const int32_t* __restrict__ atom_bin, const int32_t* __restrict__ bin_start,
            const int32_t* __restrict__ bin_atoms, float rc, const int32_t* __restrict__ row_ptr,
            int32_t* key_j, int32_t* key_c, int32_t* __restrict__ dst, int32_t* __restrict__ col,
            int8_t* __restrict__ shift, float* __restrict__ d2, float* __restrict__ rvec,
            const int32_t* __restrict__ colT_ptr, int32_t* __restrict__ colT_cur, int32_t* __restrict__ unsorted) {
  const int w0 = (int)(((size_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6);
  const int nw = (int)(((size_t)gridDim.x * blockDim.x) >> 6);
  const int lane = threadIdx.x & 63;
  const int n = *novf;
  for (int r = w0; r < n; r += nw) {
    const int i = ovf_rows[r];
    const GMeta& m = meta[atom_graph[i]];
    const int nb0 = m.nb[0], nb1 = m.nb[1], nb2 = m.nb[2];
    const int lb = atom_bin[i] - m.bin_off;
    const int b2 = lb % nb2, b1 = (lb / nb2) % nb1, b0 = lb / (nb1 * nb2);
    const float pix = pos[3 * (size_t)i], piy = pos[3 * (size_t)i + 1], piz = pos[3 * (size_t)i + 2];
    const float rc2 = __fmul_rn(rc, rc);
    const bool per = m.periodic != 0;
    int count = 0;
    const int base = row_ptr[i];
    for (int B0 = b0 - m.R[0]; B0 <= b0 + m.R[0]; ++B0) {
      int s0 = 0, c0 = B0;
      if (per) { s0 = floordiv(B0, nb0); c0 = B0 - s0 * nb0; } else if (B0 < 0 || B0 >= nb0) continue;
      for (int B1 = b1 - m.R[1]; B1 <= b1 + m.R[1]; ++B1) {
        int s1 = 0, c1 = B1;
        if (per) { s1 = floordiv(B1, nb1); c1 = B1 - s1 * nb1; } else if (B1 < 0 || B1 >= nb1) continue;
        for (int B2 = b2 - m.R[2]; B2 <= b2 + m.R[2]; ++B2) {
          int s2 = 0, c2 = B2;
          if (per) { s2 = floordiv(B2, nb2); c2 = B2 - s2 * nb2; } else if (B2 < 0 || B2 >= nb2) continue;
          const int bin = m.bin_off + (c0 * nb1 + c1) * nb2 + c2;
          float tx, ty, tz;
          shift_vector(m.cell, s0, s1, s2, tx, ty, tz);
          const bool zero_shift = (s0 | s1 | s2) == 0;
          const int code = ((s0 + 128) << 16) | ((s1 + 128) << 8) | (s2 + 128);
          const int kb = bin_start[bin], ke = bin_start[bin + 1];
          for (int k0 = kb; k0 < ke; k0 += 64) {
            const int k = k0 + lane;
            bool hit = false;
            int j = 0;
            if (k < ke) {
              j = bin_atoms[k];
              const float qx = __fadd_rn(pos[3 * (size_t)j], tx);
              const float qy = __fadd_rn(pos[3 * (size_t)j + 1], ty);
              const float qz = __fadd_rn(pos[3 * (size_t)j + 2], tz);
              const float rx = __fsub_rn(pix, qx), ry = __fsub_rn(piy, qy), rz = __fsub_rn(piz, qz);
              const float dd = __fadd_rn(__fadd_rn(__fmul_rn(rx, rx), __fmul_rn(ry, ry)), __fmul_rn(rz, rz));
              hit = (dd < rc2) && !(zero_shift && j == i);
            }
            const unsigned long long mask = __ballot(hit);
            if (hit) {
              const int off = __popcll(mask & ((1ull << lane) - 1ull));
              key_j[base + count + off] = j;
              key_c[base + count + off] = code;
            }
            count += __popcll(mask);
          }
        }
      }
    }
    // the row's hits are in memory: every lane of this wavefront reads them all below
    __threadfence();
    __builtin_amdgcn_wave_barrier();
    const int start = row_ptr[i], end = row_ptr[i + 1];
    for (int t = start + lane; t < end; t += 64) {
      const int mj = key_j[t], mc = key_c[t];
      int rank = 0;
      for (int u = start; u < end; ++u) {
        const int uj = key_j[u], uc = key_c[u];
        rank += (uj < mj) || (uj == mj && uc < mc);
      }
      const int e = start + rank;
      const int s0 = ((mc >> 16) & 255) - 128, s1 = ((mc >> 8) & 255) - 128, s2 = (mc & 255) - 128;
      float tx, ty, tz;
      shift_vector(m.cell, s0, s1, s2, tx, ty, tz);
      const float qx = __fadd_rn(pos[3 * (size_t)mj], tx);
      const float qy = __fadd_rn(pos[3 * (size_t)mj + 1], ty);
      const float qz = __fadd_rn(pos[3 * (size_t)mj + 2], tz);
      const float rx = __fsub_rn(pix, qx), ry = __fsub_rn(piy, qy), rz = __fsub_rn(piz, qz);
      const float dd = __fadd_rn(__fadd_rn(__fmul_rn(rx, rx), __fmul_rn(ry, ry)), __fmul_rn(rz, rz));
      unsorted[colT_ptr[mj] + atomicAdd(&colT_cur[mj], 1)] = e;   // the edge's place in its source group
      dst[e] = i;
      col[e] = mj;
      shift[3 * (size_t)e] = (int8_t)s0;
      shift[3 * (size_t)e + 1] = (int8_t)s1;
      shift[3 * (size_t)e + 2] = (int8_t)s2;
      d2[e] = dd;
      rvec[3 * (size_t)e] = rx;
      rvec[3 * (size_t)e + 1] = ry;
      rvec[3 * (size_t)e + 2] = rz;
    }
  }
}

__global__ void k_edge_graph_ptr(int G, const int32_t* __restrict__ graph_off, const int32_t* __restrict__ row_ptr,
                                 int32_t* __restrict__ egp) {
  int g = blockIdx.x * blockDim.x + threadIdx.x;
  if (g <= G) egp[g] = row_ptr[graph_off[g]];
}

// ---------------------------------------------------------------------------------------------
// transpose plan: the histogram of sources is taken by the counting search; the filling search deals the edges to
// their source's group (any order, see k_search); here each group is put into ascending edge order, in place
// ---------------------------------------------------------------------------------------------
constexpr int TS_CAP = 512;   // group members ranked out of LDS; longer groups are ranked from memory
__global__ void __launch_bounds__(256)
k_rank_sources(int N, const int32_t* __restrict__ colT_ptr, int32_t* __restrict__ permT, int32_t* __restrict__ copy) {
  // permT holds the groups as they were dealt; copy: room for one int per edge (long groups are ranked out of it)
  const int32_t* unsorted = permT;
  __shared__ __align__(16) int grp[4][TS_CAP + 4];
  const int j = (int)(((size_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6);
  const int lane = threadIdx.x & 63;
  if (j >= N) return;
  const int start = colT_ptr[j], end = colT_ptr[j + 1];
  const int n = end - start;
  if (n <= 0) return;
  if (n <= TS_CAP) {
    int* g = grp[(threadIdx.x >> 6) & 3];
    for (int t = lane; t < n; t += 64) g[t] = unsorted[start + t];
    if (lane < 4) g[n + lane] = 0x7fffffff;      // pad to a multiple of four for the 16-byte reads
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    for (int t = lane; t < n; t += 64) {
      const int me = g[t];
      int rank = 0;
      for (int u = 0; u < n; u += 4) {
        const int4 q = *reinterpret_cast<const int4*>(&g[u]);
        rank += (q.x < me) + (q.y < me) + (q.z < me) + (q.w < me);
      }
      permT[start + rank] = me;
    }
    return;
  }
  for (int t = start + lane; t < end; t += 64) copy[t] = unsorted[t];
  __threadfence();
  __builtin_amdgcn_wave_barrier();
  for (int t = start + lane; t < end; t += 64) {
    const int me = copy[t];
    int rank = 0;
    for (int u = start; u < end; ++u) rank += copy[u] < me;
    permT[start + rank] = me;
  }
}

__global__ void k_copy_i32(const int32_t* __restrict__ src, int32_t* __restrict__ dst, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src[i];
}

// ---------------------------------------------------------------------------------------------
// workspace layout
// ---------------------------------------------------------------------------------------------
struct NeighWs {
  int32_t* status;      // [8]: 0 input errors, 1 work-list length, 2 rows left to the slow path
  GMeta* meta;          // [G]
  int32_t* nbins;       // [G]
  int32_t* bin_off;     // [G+1]
  int32_t* atom_graph;  // [N]
  int32_t* atom_bin;    // [N]
  int32_t* zeroed;      // bin_cnt | bin_cur | colT_cnt | colT_cur, cleared by one launch
  int64_t nzeroed;
  int32_t* bin_cnt;     // [maxbins]
  int32_t* bin_start;   // [maxbins+1]
  int32_t* bin_cur;     // [maxbins]
  int32_t* bin_atoms;   // [N]
  float4* spos;         // [N] (x, y, z, atom) in bin order
  int2* list;           // [N] work list of the search
  int32_t* deg;         // [N]
  int32_t* colT_cnt;    // [N]
  int32_t* colT_cur;    // [N]
  int32_t* colT_ptr;    // [N+1] kept from the counting call for the filling call
  int32_t* ovf_rows;    // [N]
  int32_t* scan;        // scratch
  size_t bytes;
  int64_t maxbins;
};

static NeighWs carve_neigh(void* ws, int N, int G) {
  NeighWs w;
  Carver c(ws);
  w.maxbins = 4ll * N + G + 1;
  w.status = c.take<int32_t>(8);
  w.meta = c.take<GMeta>((size_t)G + 1);
  w.nbins = c.take<int32_t>((size_t)G + 1);
  w.bin_off = c.take<int32_t>((size_t)G + 2);
  w.atom_graph = c.take<int32_t>((size_t)N + 1);
  w.atom_bin = c.take<int32_t>((size_t)N + 1);
  w.nzeroed = 2 * w.maxbins + 2 * ((int64_t)N + 1);
  w.zeroed = c.take<int32_t>((size_t)w.nzeroed);
  w.bin_cnt = w.zeroed;
  w.bin_cur = w.bin_cnt + w.maxbins;
  w.colT_cnt = w.bin_cur + w.maxbins;
  w.colT_cur = w.colT_cnt + N + 1;
  w.bin_start = c.take<int32_t>((size_t)w.maxbins + 1);
  w.bin_atoms = c.take<int32_t>((size_t)N + 1);
  w.spos = c.take<float4>((size_t)N + 1);
  w.list = c.take<int2>((size_t)N + 1);
  w.deg = c.take<int32_t>((size_t)N + 1);
  w.colT_ptr = c.take<int32_t>((size_t)N + 2);
  w.ovf_rows = c.take<int32_t>((size_t)N + 1);
  w.scan = c.take<int32_t>(scan_scratch_ints(w.maxbins + N + G + 8) + 8);
  w.bytes = c.used();
  return w;
}

static inline unsigned nblk(int64_t n, int t) { return (unsigned)((n + t - 1) / t); }

static SearchArgs search_args(const NeighWs& w, int N, const float* pos, float rc) {
  SearchArgs a = {};
  a.N = N; a.pos = pos; a.meta = w.meta; a.atom_graph = w.atom_graph; a.bin_start = w.bin_start; a.spos = w.spos;
  a.nlist = w.status + 1; a.list = w.list; a.status = w.status; a.rc = rc;
  a.novf = w.status + 2; a.ovf_rows = w.ovf_rows;
  return a;
}

}  // namespace hgnn

using namespace hgnn;

extern "C" const char* hgnn_last_error_string(void) { return g_err; }
extern "C" int32_t hgnn_version(void) { return 2; }

extern "C" int32_t hgnn_radius_graph_workspace_bytes(int32_t N, int32_t G, size_t* bytes_host) {
  HGNN_REQUIRE(bytes_host != nullptr, HGNN_ERR_NULLPTR, "bytes_host is null");
  HGNN_REQUIRE(N >= 0 && G >= 0, HGNN_ERR_BAD_SHAPE, "negative N or G");
  *bytes_host = carve_neigh(nullptr, N, G).bytes;
  return HGNN_OK;
}

extern "C" int32_t hgnn_radius_graph_count(void* stream, int32_t N, int32_t G, const float* pos,
                                           const int32_t* graph_off, const float* cell, const uint8_t* pbc,
                                           float rc, void* ws, size_t ws_bytes, int32_t* row_ptr,
                                           int64_t* E_host) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  HGNN_REQUIRE(N >= 0 && G >= 0, HGNN_ERR_BAD_SHAPE, "negative N or G");
  HGNN_REQUIRE(E_host && row_ptr && graph_off && ws, HGNN_ERR_NULLPTR, "radius_graph_count: null pointer");
  HGNN_REQUIRE(pos || N == 0, HGNN_ERR_NULLPTR, "pos is null");
  HGNN_REQUIRE(rc > 0.f && rc < 1e18f, HGNN_ERR_BAD_SHAPE, "cutoff must be positive");
  HGNN_REQUIRE(G > 0 || N == 0, HGNN_ERR_BAD_OFFSETS, "atoms without a graph");
  NeighWs w = carve_neigh(ws, N, G);
  HGNN_REQUIRE(ws_bytes >= w.bytes, HGNN_ERR_WORKSPACE_TOO_SMALL, "radius graph workspace: need %zu bytes, got %zu",
               w.bytes, ws_bytes);
  *E_host = 0;
  k_fill_i32<<<1, 64, 0, st>>>(w.status, 8, 0);
  HGNN_LAUNCH_CHECK("k_fill_i32");
  if (N == 0 || G == 0) {
    k_fill_i32<<<1, 64, 0, st>>>(row_ptr, 1, 0);
    k_fill_i32<<<1, 64, 0, st>>>(w.colT_ptr, 1, 0);
    HGNN_LAUNCH_CHECK("k_fill_i32");
    HGNN_HIP(wait_stream(st));
    return HGNN_OK;
  }
  // Everything below is enqueued in one go: a bad offset or cell is recorded in status[0], leaves every later
  // kernel with in-range (if meaningless) indices, keeps the search from running, and is reported after the one
  // synchronisation at the end.
  {
    ProfScope ps(PT_NEIGH_SETUP, st);
    k_graph_meta<<<G, 64, 0, st>>>(N, G, pos, graph_off, cell, pbc, rc, w.meta, w.nbins, w.status);
    HGNN_LAUNCH_CHECK("k_graph_meta");
    HGNN_TRY(exclusive_scan_i32(st, w.nbins, w.bin_off, G, w.scan));
    k_set_bin_off<<<nblk(G, 256), 256, 0, st>>>(G, w.meta, w.bin_off);
    HGNN_LAUNCH_CHECK("k_set_bin_off");
    k_fill_i32<<<nblk(w.nzeroed, 256), 256, 0, st>>>(w.zeroed, w.nzeroed, 0);
    HGNN_LAUNCH_CHECK("k_fill_i32");
    k_bin_atoms_count<<<nblk(N, 256), 256, 0, st>>>(N, G, pos, graph_off, w.meta, w.atom_graph, w.atom_bin, w.bin_cnt,
                                                    w.status);
    HGNN_LAUNCH_CHECK("k_bin_atoms_count");
    HGNN_TRY(exclusive_scan_i32(st, w.bin_cnt, w.bin_start, w.maxbins, w.scan));
    k_bin_atoms_fill<<<nblk(N, 256), 256, 0, st>>>(N, pos, w.atom_bin, w.bin_start, w.bin_cur, w.bin_atoms, w.spos);
    HGNN_LAUNCH_CHECK("k_bin_atoms_fill");
    k_bin_list<<<nblk(w.maxbins, 256), 256, 0, st>>>(w.maxbins, w.bin_cnt, w.status + 1, w.list);
    HGNN_LAUNCH_CHECK("k_bin_list");
  }
  {
    ProfScope ps(PT_NEIGH_COUNT, st);
    SearchArgs a = search_args(w, N, pos, rc);
    a.deg = w.deg; a.colT_cnt = w.colT_cnt;
    // without a search (bad input) the degrees must still be defined for the scans below
    k_fill_i32<<<nblk(N, 256), 256, 0, st>>>(w.deg, N, 0);
    k_search<false><<<SR_GRID < N ? SR_GRID : N, 256, 0, st>>>(a);
    HGNN_LAUNCH_CHECK("k_search<count>");
  }
  long long total = 0;
  int32_t status_h[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  {
    ProfScope ps(PT_NEIGH_SETUP, st);
    HGNN_TRY(exclusive_scan_i32(st, w.colT_cnt, w.colT_ptr, N, w.scan));
    HGNN_TRY(exclusive_scan_i32(st, w.deg, row_ptr, N, w.scan));
  }
  // grand total (int64) sits behind the block sums of the last scan
  int64_t nbs = ((int64_t)N + SCAN_BLK - 1) / SCAN_BLK;
  HGNN_HIP(hipMemcpyAsync(&total, reinterpret_cast<long long*>(w.scan) + nbs, sizeof(total), hipMemcpyDeviceToHost, st));
  HGNN_HIP(hipMemcpyAsync(status_h, w.status, sizeof(status_h), hipMemcpyDeviceToHost, st));
  HGNN_HIP(wait_stream(st));
  HGNN_REQUIRE(!(status_h[0] & ST_BAD_OFFSETS), HGNN_ERR_BAD_OFFSETS,
               "graph_off must start at 0, be non-decreasing and end at N");
  HGNN_REQUIRE(!(status_h[0] & ST_BAD_CELL), HGNN_ERR_BAD_CELL,
               "a periodic graph has a singular cell or needs more than 127 images per direction");
  HGNN_REQUIRE(!(status_h[0] & ST_OUT_OF_CELL), HGNN_ERR_BAD_CELL,
               "an atom of a periodic graph lies outside its cell (fractional coordinates must be in [0, 1])");
  HGNN_REQUIRE(total < (1ll << 31), HGNN_ERR_OVERFLOW, "edge count %lld does not fit int32", total);
  *E_host = total;
  return HGNN_OK;
}

extern "C" int32_t hgnn_radius_graph_fill(void* stream, int32_t N, int32_t G, const float* pos,
                                          const int32_t* graph_off, const float* cell, const uint8_t* pbc, float rc,
                                          void* ws, size_t ws_bytes, void* tmp, size_t tmp_bytes,
                                          const int32_t* row_ptr, int64_t E, int32_t* dst, int32_t* col,
                                          int8_t* shift, float* d2, float* rvec, int32_t* edge_graph_ptr,
                                          int32_t* colT_ptr, int32_t* permT) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  (void)cell; (void)pbc;
  HGNN_REQUIRE(N >= 0 && G >= 0 && E >= 0, HGNN_ERR_BAD_SHAPE, "negative size");
  HGNN_REQUIRE(E < (1ll << 31), HGNN_ERR_OVERFLOW, "edge count does not fit int32");
  HGNN_REQUIRE(ws && row_ptr && graph_off && edge_graph_ptr && colT_ptr, HGNN_ERR_NULLPTR, "radius_graph_fill: null pointer");
  HGNN_REQUIRE(E == 0 || (tmp && dst && col && shift && d2 && rvec && permT && pos), HGNN_ERR_NULLPTR,
               "radius_graph_fill: null edge array");
  HGNN_REQUIRE(rc > 0.f, HGNN_ERR_BAD_SHAPE, "cutoff must be positive");
  NeighWs w = carve_neigh(ws, N, G);
  HGNN_REQUIRE(ws_bytes >= w.bytes, HGNN_ERR_WORKSPACE_TOO_SMALL, "radius graph workspace too small");
  HGNN_REQUIRE(tmp_bytes >= (size_t)E * 8, HGNN_ERR_WORKSPACE_TOO_SMALL, "radius graph tmp: need %zu bytes", (size_t)E * 8);
  if (N == 0) {
    k_fill_i32<<<nblk(G + 1, 256), 256, 0, st>>>(edge_graph_ptr, G + 1, 0);
    k_fill_i32<<<1, 64, 0, st>>>(colT_ptr, 1, 0);
    HGNN_LAUNCH_CHECK("k_fill_i32");
    return HGNN_OK;
  }
  int32_t* key_j = static_cast<int32_t*>(tmp);
  int32_t* key_c = key_j + E;
  // this call's own counters start at zero, so that a second fill after one count works as the first
  k_fill2_i32<<<nblk((int64_t)N + 1, 256), 256, 0, st>>>(w.colT_cur, (int64_t)N + 1, w.status + 2, 1, 0);
  HGNN_LAUNCH_CHECK("k_fill2_i32");
  if (E > 0) {
    {
      ProfScope ps(PT_NEIGH_FILL, st);
      SearchArgs a = search_args(w, N, pos, rc);
      a.row_ptr = row_ptr; a.dst = dst; a.col = col; a.shift = shift; a.d2 = d2; a.rvec = rvec;
      a.colT_ptr = w.colT_ptr; a.colT_cur = w.colT_cur; a.unsorted = permT;   // the groups are ordered in place below
      k_search<true><<<SR_GRID < N ? SR_GRID : N, 256, 0, st>>>(a);
      HGNN_LAUNCH_CHECK("k_search<fill>");
    }
    ProfScope ps(PT_NEIGH_EMIT, st);
    // rows longer than the LDS row (their number is only known on the device: a fixed grid walks the list)
    const unsigned lgrid = N < 256 ? nblk((int64_t)N * 64, 256) : 64;
    k_long_rows<<<lgrid, 256, 0, st>>>(w.status + 2, w.ovf_rows, pos, w.meta, w.atom_graph, w.atom_bin, w.bin_start,
                                       w.bin_atoms, rc, row_ptr, key_j, key_c, dst, col, shift, d2, rvec, w.colT_ptr,
                                       w.colT_cur, permT);
    HGNN_LAUNCH_CHECK("k_long_rows");
  }
  ProfScope pst(PT_NEIGH_TRANSPOSE, st);
  k_edge_graph_ptr<<<nblk(G + 1, 256), 256, 0, st>>>(G, graph_off, row_ptr, edge_graph_ptr);
  HGNN_LAUNCH_CHECK("k_edge_graph_ptr");
  k_copy_i32<<<nblk((int64_t)N + 1, 256), 256, 0, st>>>(w.colT_ptr, colT_ptr, (int64_t)N + 1);
  HGNN_LAUNCH_CHECK("k_copy_i32");
  if (E > 0) {
    k_rank_sources<<<nblk((int64_t)N * 64, 256), 256, 0, st>>>(N, colT_ptr, permT, key_j);   // the keys are dead by now
    HGNN_LAUNCH_CHECK("k_rank_sources");
  }
  return HGNN_OK;
}
