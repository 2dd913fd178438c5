// Shared host-side helpers of libjz (argument checks, launch error mapping).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "jz.h"

namespace jz {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// [a, a+na) and [b, b+nb) share a byte
inline bool overlaps(const void* a, size_t na, const void* b, size_t nb) {
  if (!a || !b || na == 0 || nb == 0) return false;
  uintptr_t pa = reinterpret_cast<uintptr_t>(a), pb = reinterpret_cast<uintptr_t>(b);
  return pa < pb + nb && pb < pa + na;
}

// Forward convolution for the fused convolution + batch normalization entry point.  conv_fwd_stats_plan: the workspace
// the convolution needs and, when its kernel can leave per-tile column sums of y and y^2, the number of row tiles (else
// 0).  conv_fwd_run with stats != nullptr (only after a plan that said so) writes them as [tiles_m][2][K] floats; it
// returns JZ_ERR_UNSUPPORTED, before anything is launched, if the plan no longer has stats_tiles_m row tiles.
int conv_fwd_stats_plan(const jz_conv_desc* d, size_t* conv_ws_bytes, int* tiles_m);
int conv_fwd_run(const jz_conv_desc* d, const void* x, const void* w, void* y, void* ws, size_t ws_bytes, float* stats,
                 int stats_tiles_m, void* stream);

// Backward-data convolution for the fused "backward-data + batch-norm backward" entry point (jz_bn.hip): the layer whose
// output (after batch normalization + ReLU) was this convolution's input.  conv_bwd_data_stats_plan: the convolution's
// workspace and, when its kernel can leave per-tile sums of g and g x^ (g = dx where y > 0), the number of row tiles (else 0);
// conv_bwd_data_run with stats != nullptr (only after a plan that said so) writes them as [tiles_m][2][C] floats.
struct BnBwdOperands {
  const void* x16;      // the normalization's input  [N,H,W,C] of the convolution's input shape
  const void* y16;      // its output after the ReLU = the convolution's forward input
  const float* mean;    // [C]
  const float* invstd;  // [C]
  // block end: y16 = relu(bn(x16) + shortcut) is a residual block's output and the convolution's result is one
  // contribution to its gradient; what the convolution stores (and sums) is g = RNE16(result [+ add16]) where y16 > 0
  bool block_end = false;
  const void* add16 = nullptr;  // the other contribution, optional
};
int conv_bwd_data_stats_plan(const jz_conv_desc* d, size_t* conv_ws_bytes, int* tiles_m);
int conv_bwd_data_run(const jz_conv_desc* d, const void* dy, const void* w, void* dx, void* ws, size_t ws_bytes, float* stats,
                      int stats_tiles_m, const BnBwdOperands* bn, void* stream);

inline int launch_status() { return hipGetLastError() == hipSuccess ? JZ_OK : JZ_ERR_LAUNCH; }

}  // namespace jz
