// Decoding heads with D fully connected hidden layers per head (paper, section "Numerical Results": three layers of
// 889 units in every dataset-specific head), for any input width H and head width Hh up to 1024, bf16 operands.
// Every product is a grouped fragment GEMM (frag.h): the rows of source s (graphs for the energy head, atoms for
// the force head, made contiguous by the routing plan) meet the weights of branch s; hidden activations live in
// the padded per-group row order of the fragment tensors, only the first layer gathers and the last one scatters.
#include "devmath.h"
#include "edgeops.h"
#include "frag.h"
#include "plan.h"
#include "wide.h"

namespace hgnn {

constexpr int DEEP_MAX_D = 8;

struct DeepOff {  // element offsets inside one branch; head 0 = energy, 1 = force; layers 1..D
  long W[2][DEEP_MAX_D + 1], b[2][DEEP_MAX_D + 1], wo[2], bo[2], per;
  DeepOff(long H, long Hh, int D) {
    long o = 0;
    for (int hd = 0; hd < 2; ++hd) {
      for (int l = 1; l <= D; ++l) {
        W[hd][l] = o; o += (l == 1 ? H : Hh) * Hh;
        b[hd][l] = o; o += Hh;
      }
      wo[hd] = o; o += Hh;
      bo[hd] = o; o += 1;
    }
    per = o;
  }
};

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
  return x;
}

// output layers. rows 0..G-1: graphs (energy); rows G..G+N-1: atoms (force). One wavefront per row.
__global__ void __launch_bounds__(256)
k_deep_out_fwd(int N, int G, int Hh, int ldz, const float* __restrict__ ze, const float* __restrict__ zf,
               const float* __restrict__ Whead, long per, long wo_e, long bo_e, long wo_f, long bo_f,
               const int32_t* __restrict__ graph_src, const int32_t* __restrict__ atom_graph, const float* __restrict__ v,
               float* __restrict__ energy, float* __restrict__ force, float* __restrict__ qsave) {
  const int r = (int)(((size_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6);
  const int lane = threadIdx.x & 63;
  if (r >= G + N) return;
  const bool is_graph = r < G;
  const int i = is_graph ? r : r - G;
  const int s = graph_src[is_graph ? i : atom_graph[i]];
  const float* z = (is_graph ? ze : zf) + (size_t)i * ldz;
  const float* w = Whead + s * per + (is_graph ? wo_e : wo_f);
  float acc = 0.f;
  for (int c = lane; c < Hh; c += 64) acc += w[c] * silu_f(z[c]);
  acc = wave_sum(acc);
  if (lane == 0) {
    const float out = acc + Whead[s * per + (is_graph ? bo_e : bo_f)];
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

// g_z = g_out * wo * silu'(z) of the last hidden layer; also g_v = q * g_force and the per-atom scalar gq
__global__ void __launch_bounds__(256)
k_deep_out_bwd(int N, int G, int Hh, int ldz, const float* __restrict__ ze, const float* __restrict__ zf,
               const float* __restrict__ Whead, long per, long wo_e, long wo_f, const int32_t* __restrict__ graph_src,
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
  const float* z = (is_graph ? ze : zf) + (size_t)i * ldz;
  float* gz_ = (is_graph ? g_ze : g_zf) + (size_t)i * ldz;
  const float* w = Whead + s * per + (is_graph ? wo_e : wo_f);
  for (int c = lane; c < Hh; c += 64) gz_[c] = go * w[c] * dsilu_f(z[c]);
}

// dest[s * stride] = sum over the positions of group s of w[row_idx[pos]]   (one block per group, fixed order)
__global__ void __launch_bounds__(1024)
k_deep_scalar_sum(const float* __restrict__ w, const int32_t* __restrict__ row_idx, const int32_t* __restrict__ grp_ptr,
                  float* __restrict__ dest, long stride) {
  __shared__ float sh[16];
  const int s = blockIdx.x;
  float acc = 0.f;
  for (int t = grp_ptr[s] + threadIdx.x; t < grp_ptr[s + 1]; t += 1024) acc += w[row_idx[t]];
  acc = wave_sum(acc);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    float tot = 0.f;
    for (int k = 0; k < 16; ++k) tot += sh[k];
    dest[s * stride] = tot;
  }
}

struct DeepDims {
  int N, G, H, Hh, D, S, Hp, Hhp, Pmax;
  int64_t Pb[2];    // padded rows of the grouped fragment tensors (energy, force)
  int Mp[2];        // padded rows of the largest possible group
  DeepDims(int N_, int G_, int H_, int Hh_, int D_, int S_) : N(N_), G(G_), H(H_), Hh(Hh_), D(D_), S(S_) {
    Hp = wide_pad_cols(H);
    Hhp = wide_pad_cols(Hh);
    Pmax = Hp > Hhp ? Hp : Hhp;
    Pb[0] = frag_group_rows(G, S);
    Pb[1] = frag_group_rows(N, S);
    Mp[0] = (int)wide_pad_rows(G);
    Mp[1] = (int)wide_pad_rows(N);
  }
};

struct DeepSaved {
  float* z[2][DEEP_MAX_D + 1];   // z[hd][l]: l < D in padded row order [Pb, Hhp]; l = D in the caller's row order
  float* q;
  size_t bytes;
};
static DeepSaved carve_deep_saved(void* p, const DeepDims& d) {
  Carver c(p);
  DeepSaved s;
  for (int hd = 0; hd < 2; ++hd) {
    for (int l = 1; l < d.D; ++l) s.z[hd][l] = c.take<float>((size_t)d.Pb[hd] * d.Hhp);
    s.z[hd][d.D] = c.take<float>((size_t)(hd == 0 ? d.G : d.N) * d.Hhp + 4);
  }
  s.q = c.take<float>((size_t)d.N + 1);
  s.bytes = c.used();
  return s;
}

struct DeepWs {
  unsigned short* packed;   // [S][Pmax x Pmax] bf16, one layer at a time
  char *R0, *R1, *T0, *T1;  // fragment operands [Pb, Pmax]
  float* ga;                // [Pb, Hhp] gradient of a hidden activation, padded row order
  float* gzD[2];            // gradient of the last hidden pre-activation, caller's row order
  float* gq;                // [N]
  float* partial;
  size_t partial_floats;
  float* cs_partial;
  size_t bytes;
};
static DeepWs carve_deep_ws(void* p, const DeepDims& d) {
  Carver c(p);
  DeepWs w;
  const int64_t Pb = d.Pb[0] > d.Pb[1] ? d.Pb[0] : d.Pb[1];
  const int M = d.N > d.G ? d.N : d.G;
  w.packed = c.take<unsigned short>((size_t)d.S * d.Pmax * d.Pmax);
  const size_t fb = (size_t)Pb * d.Pmax * 2;
  w.R0 = c.take<char>(fb);
  w.R1 = c.take<char>(fb);
  w.T0 = c.take<char>(fb);
  w.T1 = c.take<char>(fb);
  w.ga = c.take<float>((size_t)Pb * d.Hhp);
  w.gzD[0] = c.take<float>((size_t)d.G * d.Hhp + 4);
  w.gzD[1] = c.take<float>((size_t)d.N * d.Hhp + 4);
  w.gq = c.take<float>((size_t)d.N + 1);
  w.partial_floats = (size_t)8 * d.S * d.Pmax * d.Pmax;
  w.partial = c.take<float>(w.partial_floats);
  w.cs_partial = c.take<float>(colsum_rows_partial_floats(M, d.Hhp, d.S));
  w.bytes = c.used();
  return w;
}

static int32_t check_deep_args(int N, int G, int H, int Hh, int D, int S, int dtype) {
  HGNN_REQUIRE(N >= 0 && G >= 0, HGNN_ERR_BAD_SHAPE, "negative N or G");
  HGNN_REQUIRE(H >= 1 && H <= 1024 && Hh >= 1 && Hh <= 1024, HGNN_ERR_BAD_SHAPE, "H and Hh must lie in 1..1024 (got %d, %d)", H, Hh);
  HGNN_REQUIRE(D >= 1 && D <= DEEP_MAX_D, HGNN_ERR_BAD_SHAPE, "D must lie in 1..%d (got %d)", DEEP_MAX_D, D);
  HGNN_REQUIRE(S >= 1 && S <= 1024, HGNN_ERR_BAD_SHAPE, "S must lie in 1..1024 (got %d)", S);
  HGNN_REQUIRE(dtype == HGNN_F32 || dtype == HGNN_BF16, HGNN_ERR_BAD_SHAPE, "unknown dtype %d", dtype);
  HGNN_REQUIRE(dtype == HGNN_BF16, HGNN_ERR_UNIMPLEMENTED, "the deep heads run with bf16 operands only");
  return HGNN_OK;
}

// fragments of W_l (forward, [in, out]) or of its transpose for all S branches
static int32_t pack_layer(hipStream_t st, const DeepDims& d, const DeepOff& o, const float* Whead, int hd, int l,
                          bool transposed, unsigned short* dst) {
  const int K = l == 1 ? d.H : d.Hh, Kp = l == 1 ? d.Hp : d.Hhp;
  PackFragArgs pk;
  pk.src = Whead; pk.dst = dst; pk.nparts = 1;
  pk.groups = d.S; pk.src_grp_stride = o.per; pk.dst_grp_stride = (long)Kp * d.Hhp;
  if (!transposed) {
    pk.K = K; pk.Nn = d.Hh; pk.Kp = Kp; pk.Np = d.Hhp;
    pk.part[0] = {o.W[hd][l], d.Hh, 1, 0, Kp / 16, 0, 0};
  } else {
    pk.K = d.Hh; pk.Nn = K; pk.Kp = d.Hhp; pk.Np = Kp;
    pk.part[0] = {o.W[hd][l], 1, d.Hh, 0, d.Hhp / 16, 0, 0};
  }
  return launch_pack_frag(st, pk);
}

}  // namespace hgnn

using namespace hgnn;

extern "C" int32_t hgnn_multihead_deep_workspace_bytes(int32_t N, int32_t G, int32_t H, int32_t Hh, int32_t D, int32_t S,
                                                       int32_t dtype, size_t* ws_bytes_host, size_t* saved_bytes_host) {
  HGNN_TRY(check_deep_args(N, G, H, Hh, D, S, dtype));
  HGNN_REQUIRE(ws_bytes_host && saved_bytes_host, HGNN_ERR_NULLPTR, "null size pointer");
  const DeepDims d(N, G, H, Hh, D, S);
  *ws_bytes_host = carve_deep_ws(nullptr, d).bytes;
  *saved_bytes_host = carve_deep_saved(nullptr, d).bytes;
  return HGNN_OK;
}

extern "C" int32_t hgnn_multihead_deep_fwd(void* stream, int32_t N, int32_t G, int32_t H, int32_t Hh, int32_t D, int32_t S,
                                           int32_t dtype, const int32_t* plan, const float* p, const float* h,
                                           const float* v, const float* Whead, float* energy, float* force, void* saved,
                                           size_t saved_bytes, void* ws, size_t ws_bytes) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  HGNN_TRY(check_deep_args(N, G, H, Hh, D, S, dtype));
  if (G == 0 && N == 0) return HGNN_OK;
  HGNN_REQUIRE(plan && Whead && saved && ws, HGNN_ERR_NULLPTR, "multihead_deep_fwd: null pointer");
  HGNN_REQUIRE((G == 0 || (p && energy)) && (N == 0 || (h && v && force)), HGNN_ERR_NULLPTR, "multihead_deep_fwd: null pointer");
  const DeepDims d(N, G, H, Hh, D, S);
  DeepWs w = carve_deep_ws(ws, d);
  DeepSaved s = carve_deep_saved(saved, d);
  HGNN_REQUIRE(ws_bytes >= w.bytes, HGNN_ERR_WORKSPACE_TOO_SMALL, "deep decode workspace: need %zu bytes, got %zu", w.bytes, ws_bytes);
  HGNN_REQUIRE(saved_bytes >= s.bytes, HGNN_ERR_WORKSPACE_TOO_SMALL, "deep decode saved buffer: need %zu bytes, got %zu", s.bytes, saved_bytes);
  PlanView pv = plan_view(plan, N, G, S);
  const DeepOff o(H, Hh, D);

  for (int hd = 0; hd < 2; ++hd) {
    const int M = hd == 0 ? G : N;
    if (M == 0) continue;
    const int32_t* ridx = hd == 0 ? pv.graph_perm : pv.atom_perm;
    const int32_t* gptr = hd == 0 ? pv.grp_graph_ptr : pv.grp_atom_ptr;
    char* Rin = w.R0;
    char* Rout = w.R1;
    {  // the rows of every source, gathered into fragment order
      ToFragArgs t;
      t.X = hd == 0 ? p : h; t.ldx = H; t.ncol = H; t.Cp = d.Hp; t.Mp = d.Mp[hd];
      t.grp_ptr = gptr; t.S = S; t.row_idx = ridx;
      t.R = Rin; t.r_nkb = d.Hp / 16;
      HGNN_TRY(launch_to_frag(st, t));
    }
    for (int l = 1; l <= D; ++l) {
      const int Kp = l == 1 ? d.Hp : d.Hhp;
      HGNN_TRY(pack_layer(st, d, o, Whead, hd, l, false, w.packed));
      FGemmArgs g;
      g.A = Rin; g.a_si = Kp / 16; g.a_sk = 1;
      g.B = reinterpret_cast<const char*>(w.packed); g.b_sj = Kp / 16; g.b_sk = 1; g.b_grp_stride = (long)Kp * d.Hhp * 2;
      g.nI = d.Mp[hd] / 32; g.nJ = d.Hhp / 32; g.nkb = Kp / 16; g.kper = Kp / 16; g.nsplit = 1;
      g.grp_ptr = gptr; g.S = S;
      g.bias = Whead + o.b[hd][l]; g.nbias = Hh; g.bias_grp_stride = o.per;
      g.Cf = s.z[hd][l]; g.ldc = d.Hhp; g.ncol_f = d.Hhp;
      if (l == D) g.row_idx = ridx;   // the last hidden layer goes back to the caller's row order
      g.tag = PT_GEMM_NODE;
      HGNN_TRY(launch_fgemm_rows(st, g));
      if (l < D) {
        ToFragArgs t;
        t.X = s.z[hd][l]; t.ldx = d.Hhp; t.mode = 1; t.ncol = Hh; t.Cp = d.Hhp; t.Mp = d.Mp[hd];
        t.grp_ptr = gptr; t.S = S;
        t.R = Rout; t.r_nkb = d.Hhp / 16;
        HGNN_TRY(launch_to_frag(st, t));
        char* tmp = Rin; Rin = Rout; Rout = tmp;
      }
    }
  }
  {
    ProfScope ps(PT_HEAD_OUT, st);
    k_deep_out_fwd<<<(unsigned)(((int64_t)(G + N) * 64 + 255) / 256), 256, 0, st>>>(
        N, G, Hh, d.Hhp, s.z[0][D], s.z[1][D], Whead, o.per, o.wo[0], o.bo[0], o.wo[1], o.bo[1], pv.graph_src,
        pv.atom_graph, v, energy, force, s.q);
    HGNN_LAUNCH_CHECK("k_deep_out_fwd");
  }
  return HGNN_OK;
}

extern "C" int32_t hgnn_multihead_deep_bwd(void* stream, int32_t N, int32_t G, int32_t H, int32_t Hh, int32_t D, int32_t S,
                                           int32_t dtype, const int32_t* plan, const float* p, const float* h,
                                           const float* v, const float* Whead, const void* saved, size_t saved_bytes,
                                           const float* g_energy, const float* g_force, float* g_p, float* g_h,
                                           float* g_v, float* gWhead, void* ws, size_t ws_bytes) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  HGNN_TRY(check_deep_args(N, G, H, Hh, D, S, dtype));
  HGNN_REQUIRE(gWhead && Whead && ws, HGNN_ERR_NULLPTR, "multihead_deep_bwd: null pointer");
  const DeepOff o(H, Hh, D);
  if (G == 0 && N == 0) return launch_fill_f32(st, gWhead, o.per * S, 0.f);
  HGNN_REQUIRE(plan && saved, HGNN_ERR_NULLPTR, "multihead_deep_bwd: null pointer");
  HGNN_REQUIRE((G == 0 || (p && g_energy && g_p)) && (N == 0 || (h && v && g_force && g_h && g_v)), HGNN_ERR_NULLPTR,
               "multihead_deep_bwd: null pointer");
  const DeepDims d(N, G, H, Hh, D, S);
  DeepWs w = carve_deep_ws(ws, d);
  DeepSaved s = carve_deep_saved(const_cast<void*>(saved), d);
  HGNN_REQUIRE(ws_bytes >= w.bytes, HGNN_ERR_WORKSPACE_TOO_SMALL, "deep decode workspace: need %zu bytes, got %zu", w.bytes, ws_bytes);
  HGNN_REQUIRE(saved_bytes >= s.bytes, HGNN_ERR_WORKSPACE_TOO_SMALL, "deep decode saved buffer: need %zu bytes, got %zu", s.bytes, saved_bytes);
  PlanView pv = plan_view(plan, N, G, S);

  {
    ProfScope ps(PT_HEAD_OUT, st);
    k_deep_out_bwd<<<(unsigned)(((int64_t)(G + N) * 64 + 255) / 256), 256, 0, st>>>(
        N, G, Hh, d.Hhp, s.z[0][D], s.z[1][D], Whead, o.per, o.wo[0], o.wo[1], pv.graph_src, pv.atom_graph, v, s.q,
        g_energy, g_force, w.gzD[0], w.gzD[1], w.gq, g_v);
    HGNN_LAUNCH_CHECK("k_deep_out_bwd");
  }
  for (int hd = 0; hd < 2; ++hd) {
    const int M = hd == 0 ? G : N;
    if (M == 0) {   // nothing routed anywhere: this head's gradients are zero for every source
      for (int sidx = 0; sidx < S; ++sidx)
        HGNN_TRY(launch_fill_f32(st, gWhead + sidx * o.per + o.W[hd][1], o.bo[hd] + 1 - o.W[hd][1], 0.f));
      continue;
    }
    const int32_t* ridx = hd == 0 ? pv.graph_perm : pv.atom_perm;
    const int32_t* gptr = hd == 0 ? pv.grp_graph_ptr : pv.grp_atom_ptr;
    const float* X = hd == 0 ? p : h;
    const float* gout = hd == 0 ? g_energy : w.gq;   // per-row upstream scalar, caller's row order
    {  // output layer: g_wo = sum gout * silu(z_D), g_bo = sum gout
      ColsumRowsArgs c;
      c.X = s.z[hd][D]; c.ldx = d.Hhp; c.mode = 1; c.w = gout; c.M = M; c.ncol = Hh;
      c.grp_ptr = gptr; c.S = S; c.row_idx = ridx;
      c.partial = w.cs_partial; c.dest = gWhead + o.wo[hd]; c.dest_grp_stride = o.per;
      HGNN_TRY(launch_colsum_rows(st, c));
      k_deep_scalar_sum<<<S, 1024, 0, st>>>(gout, ridx, gptr, gWhead + o.bo[hd], o.per);
      HGNN_LAUNCH_CHECK("k_deep_scalar_sum");
    }
    {  // g_z_D into fragment order
      ToFragArgs t;
      t.X = w.gzD[hd]; t.ldx = d.Hhp; t.ncol = Hh; t.Cp = d.Hhp; t.Mp = d.Mp[hd];
      t.grp_ptr = gptr; t.S = S; t.row_idx = ridx;
      t.R = w.R0; t.r_nkb = d.Hhp / 16;
      t.T = w.T0; t.t_ncb = d.Hhp / 32;
      HGNN_TRY(launch_to_frag(st, t));
    }
    for (int l = D; l >= 1; --l) {
      const int K = l == 1 ? H : Hh, Kp = l == 1 ? d.Hp : d.Hhp;
      {  // bias gradient = column sums of g_z_l
        ColsumRowsArgs c;
        c.M = M; c.ncol = Hh; c.grp_ptr = gptr; c.S = S;
        c.partial = w.cs_partial; c.dest = gWhead + o.b[hd][l]; c.dest_grp_stride = o.per;
        if (l == D) { c.X = w.gzD[hd]; c.ldx = d.Hhp; c.row_idx = ridx; }
        else { c.X = w.ga; c.ldx = d.Hhp; c.Z = s.z[hd][l]; c.ldz = d.Hhp; c.mode = 2; }
        HGNN_TRY(launch_colsum_rows(st, c));
      }
      {  // the layer's input as T fragments: the gathered rows, or silu of the previous pre-activation
        ToFragArgs t;
        t.Mp = d.Mp[hd]; t.grp_ptr = gptr; t.S = S;
        t.T = w.T1; t.t_ncb = Kp / 32;
        if (l == 1) { t.X = X; t.ldx = H; t.ncol = H; t.Cp = d.Hp; t.row_idx = ridx; }
        else { t.X = s.z[hd][l - 1]; t.ldx = d.Hhp; t.mode = 1; t.ncol = Hh; t.Cp = d.Hhp; }
        HGNN_TRY(launch_to_frag(st, t));
      }
      {  // g_W_l = input^T g_z_l per source
        FWgradArgs a;
        a.A_T = w.T1; a.a_ncb = Kp / 32; a.nI = Kp / 32;
        a.B_T = w.T0; a.b_ncb = d.Hhp / 32; a.nJ = d.Hhp / 32;
        a.rows = d.Mp[hd]; a.grp_ptr = gptr; a.S = S;
        a.HpA = Kp; a.HA = K; a.HpB = d.Hhp; a.HB = Hh;
        a.partial = w.partial; a.partial_floats = w.partial_floats;
        a.dest = gWhead + o.W[hd][l]; a.dest_grp_stride = o.per;
        a.tag = PT_WGRAD_NODE;
        HGNN_TRY(launch_fwgrad(st, a));
      }
      {  // gradient of the layer's input = g_z_l W_l^T
        HGNN_TRY(pack_layer(st, d, o, Whead, hd, l, true, w.packed));
        FGemmArgs g;
        g.A = w.R0; g.a_si = d.Hhp / 16; g.a_sk = 1;
        g.B = reinterpret_cast<const char*>(w.packed); g.b_sj = d.Hhp / 16; g.b_sk = 1;
        g.b_grp_stride = (long)d.Hhp * Kp * 2;
        g.nI = d.Mp[hd] / 32; g.nJ = Kp / 32; g.nkb = d.Hhp / 16; g.kper = d.Hhp / 16; g.nsplit = 1;
        g.grp_ptr = gptr; g.S = S;
        g.tag = PT_GEMM_NODE;
        if (l > 1) { g.Cf = w.ga; g.ldc = d.Hhp; g.ncol_f = d.Hhp; }
        else { g.Cf = hd == 0 ? g_p : g_h; g.ldc = H; g.ncol_f = H; g.row_idx = ridx; }
        HGNN_TRY(launch_fgemm_rows(st, g));
      }
      if (l > 1) {  // g_z_{l-1} = g_a_{l-1} silu'(z_{l-1})
        ToFragArgs t;
        t.X = w.ga; t.ldx = d.Hhp; t.Z = s.z[hd][l - 1]; t.ldz = d.Hhp; t.mode = 2; t.ncol = Hh; t.Cp = d.Hhp;
        t.Mp = d.Mp[hd]; t.grp_ptr = gptr; t.S = S;
        t.R = w.R0; t.r_nkb = d.Hhp / 16;
        t.T = w.T0; t.t_ncb = d.Hhp / 32;
        HGNN_TRY(launch_to_frag(st, t));
      }
    }
  }
  return HGNN_OK;
}
