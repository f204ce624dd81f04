// Message-passing layer for hidden widths other than 64 / 128 / 256, up to 1024 (the paper's backbone has 866 hidden
// units, section "Numerical Results"): at large widths the per-edge H x H product dominates and is bound by the
// matrix cores, so the edge tensors are materialised and every product runs through one fragment GEMM kernel
// (internal). Small odd widths take the same path for generality, padded to 128.
//
// All matrix operands live in HBM as 1 KiB "fragments" = what one wavefront feeds to one
// v_mfma_f32_32x32x16_bf16 (64 lanes x 8 bf16), so that staging and operand loads are straight copies:
//   R(X) [rb32][kb16][lane][8]  lane (g, r)  holds X[32 rb32 + r, 16 kb16 + 8 g + (0..7)]     (rows x contraction)
//   T(X) [rb16][cb32][lane][8]  lane (g, c)  holds X[16 rb16 + 8 (u >> 2) + 4 g + (u & 3), 32 cb32 + c], u = 0..7
// R feeds products that contract over columns (X W). T feeds products that contract over rows (X^T Y; the row
// order inside a group of 16 is the same for both operands and cancels) and is also exactly what the accumulator
// registers of a product hold, so a product's result is stored as T without any shuffle.
// Widths are padded to a multiple of 128 (Hp) and row counts to a multiple of 256, padding filled with zeros.
#pragma once

#include "common.h"
#include "prof.h"

namespace hgnn {

// every width from 1 to 1024 that the fused narrow kernels (64, 128, 256) do not serve
inline bool wide_H(int H) { return H >= 1 && H <= 1024 && H != 64 && H != 128 && H != 256; }
inline int wide_pad_cols(int H) { return (H + 127) / 128 * 128; }
inline int64_t wide_pad_rows(int64_t M) { return (M + 255) / 256 * 256; }

struct WideLayerArgs {
  int N = 0;
  int64_t E = 0;
  int H = 0;
  float alpha = 1.f;
  const int32_t* row_ptr = nullptr;
  const int32_t* dst = nullptr;
  const int32_t* col = nullptr;
  const float* d2 = nullptr;
  const float* attr = nullptr;   // [E, k] edge attributes in place of d2 (null: d2, k = 1)
  int k = 1;
  const float* rvec = nullptr;
  const int32_t* colT_ptr = nullptr;
  const int32_t* permT = nullptr;
  const float* h_in = nullptr;
  const float* v_in = nullptr;
  const float* W = nullptr;
  float* h_out = nullptr;
  float* v_out = nullptr;
  const float* g_h_out = nullptr;
  const float* g_v_out = nullptr;
  float* g_h_in = nullptr;
  float* g_v_in = nullptr;
  float* gW = nullptr;
  float* g_attr = nullptr;   // optional out [E, k]: gradient with respect to the edge attributes (d2 when attr is null)
  float* g_rvec = nullptr;   // optional out [E, 3]: gradient with respect to the edge vectors (through v')
  void* saved = nullptr;
  void* ws = nullptr;
};

constexpr int WIDE_MAX_ATTR = 16;   // most edge attributes per edge
void wide_layer_sizes(int N, int64_t E, int H, int k, size_t* ws_bytes, size_t* saved_bytes);
int32_t wide_layer_fwd(hipStream_t st, const WideLayerArgs& a);
int32_t wide_layer_bwd(hipStream_t st, const WideLayerArgs& a);

}  // namespace hgnn
