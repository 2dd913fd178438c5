// Implicit-GEMM core shared by the convolution and fully connected entry points of libjz (gfx950).
//
// Every operation of the FP16 forward/backward pass (Jia et al. 2018, Section 4.1: FP16 storage, FP32
// accumulation, one rounding to FP16 at the end) is a contraction D[m][n] = sum_k A(m,k) * B(n,k):
//
//   op          m            n          k (reduction)   A(m,k)                         B(n,k)
//   FWD         (n,p,q)      k_out      (r,s,c)         x gathered at the tap          w[k_out][r][s][c]
//   BWD_DATA    (n,h,w)      c          (r,s,k_out)     dy gathered at the tap         w[k_out][r][s][c]
//   BWD_WEIGHT  k_out        (r,s,c)    (n,p,q)         dy[(n,p,q)][k_out]             x gathered at the tap
//
// A fully connected layer is the 1x1 case on a 1x1 image.  D is always a plain row-major [M][N] matrix
// (y, dx and dw are all stored with the n index innermost), so one epilogue serves all three.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace jz {

enum { OP_FWD = 0, OP_BWD_DATA = 1, OP_BWD_WEIGHT = 2,
       OP_FWD_STATS = 3,        // forward whose epilogue also leaves per-tile column sums (kernel template arguments only)
       OP_BWD_DATA_STATS = 4,   // backward-data whose epilogue also leaves the sums a batch-norm backward needs
       OP_BWD_DATA_BLOCK_END = 5 };  // ... and first forms the gradient at the end of a residual block from its tile

// Division by a run-time constant through multiply-high (Granlund-Montgomery style), exact for n < 2^31.
struct FastDiv {
  unsigned mult, shift, d;
};
inline FastDiv make_fastdiv(unsigned d) {
  FastDiv f{0u, 0u, d};
  if (d <= 1) return f;
  unsigned lg = 0;
  while ((1ull << lg) < d) ++lg;  // ceil(log2 d) >= 1
  unsigned p = 31 + lg;
  f.mult = (unsigned)(((1ull << p) + d - 1) / d);
  f.shift = p - 32;
  return f;
}
__device__ __forceinline__ unsigned fd_div(unsigned n, const FastDiv& f) {
  return f.d <= 1 ? n : (__umulhi(n, f.mult) >> f.shift);
}

struct ConvGeom {
  int IH, IW, IC;  // the tensor that is gathered (x for FWD / BWD_WEIGHT, dy for BWD_DATA): spatial size, channels
  int OH, OW;      // the pixel grid the GEMM's m index (FWD, BWD_DATA) or k index (BWD_WEIGHT) runs over
  int R, S, sh, sw, ph, pw;
  // Addressing of the gathered tensor, in elements: pixel (n, ih, iw), tap column s, channel c sits at
  //   (n * IH + ih) * row_pitch + iw * pix_step + s_extra + c      with s_extra = 0 here and s * s_step added per tap.
  // A plain NHWC tensor has row_pitch = IW * IC and pix_step = s_step = IC.  The small-channel path (3-channel
  // stems) gathers from a zero-padded 4-channel copy in which one filter row of S taps is a single contiguous run:
  // there IC is the length of that run (the k tile), S = 1, pix_step = 4 and runs of neighbouring pixels overlap.
  int row_pitch, pix_step, s_step;
  int kvalid;  // small-channel forward only: elements of a k tile beyond this are not part of the filter row
  int always_mask;  // build the per-row tap masks even for a single unpadded tap (grids whose sizes are not tied by a stride)
  unsigned tap_rep;  // bit r * S set for every filter row r (when R * S <= 32): spreads a column mask over the rows
  FastDiv d_ohow, d_ow, d_ic, d_s, d_sh, d_sw;
};

struct GemmArgs {
  const unsigned short* A;
  const unsigned short* B;
  unsigned short* D16;  // [M][N] fp16, written when splits == 1
  float* Dpart;         // [splits][M][N] fp32 partial sums, written when splits > 1
  float* stats;         // optional, splits == 1 only: [tiles_m][2][N] column sums of the stored FP16 tile and of its squares
                        // (OP_FWD_STATS), or of g and g x^ (OP_BWD_DATA_STATS) with g = the stored gradient where st_y > 0,
                        // else 0, and x^ = (st_c - st_mean) st_invstd: the batch normalization + ReLU that produced the
                        // convolution's input, st_c its input and st_y its output, both [M][N] like D16
                        // OP_BWD_DATA_BLOCK_END: the tile is one contribution to the gradient of a residual block's output
                        // st_y = relu(bn(st_c) + shortcut); what is stored (and summed) is g = RNE16(tile [+ st_add]) where
                        // st_y > 0, else 0
  const unsigned short* st_y;
  const unsigned short* st_c;
  const unsigned short* st_add;  // optional second contribution, [M][N]
  const float* st_mean;
  const float* st_invstd;
  unsigned bytesA, bytesB;  // sizes of the A / B tensors: the bounds of their buffer descriptors
  int M, N, Kred;
  int nkt;           // number of k tiles = ceil(Kred / BK)
  int kt_per_split;  // k tiles each split handles
  int splits;
  int tiles_m, tiles_n;
  FastDiv d_tiles_mn, d_tiles_n;  // workgroup id -> (split, tile row, tile column) without integer division code
  // strided backward-data: output row m = (n,p,q) is written to pixel (n, p*sc_sh + sc_oh, q*sc_sw + sc_ow) of an
  // sc_H x sc_W image; sc_fill: the other pixels of each sc_sh x sc_sw cell receive zeros (strided 1x1 layers, where no
  // output pixel reads them); without it the launch is one of sc_sh * sc_sw that cover the image between them
  int sc_on, sc_H, sc_W, sc_sh, sc_sw, sc_oh, sc_ow, sc_fill;
  // backward-weight of a 1x1 unit-stride unpadded layer: reduction row j (a pixel) of x starts at j * IC, no gather
  int bw_linear;
  ConvGeom g;
};

}  // namespace jz
