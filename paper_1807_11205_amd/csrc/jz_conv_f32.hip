// FP32-storage / FP32-accumulate convolution forward, backward-data, backward-weight and fully connected GEMMs for
// gfx950: the single-precision side of the paper's FP32-versus-mixed-precision throughput comparison (Jia et al. 2018,
// Section 5.4, Table 9).  Same operations, layouts and GEMM view as the FP16 path (jz_igemm.h):
//
//   D[m][n] = sum_k A(m,k) * B(n,k), every product and sum in FP32 on v_mfma_f32_32x32x2_f32.
//
// One kernel family, built for the 157 TFLOP/s matrix peak of FP32 (a sixteenth of the FP16 one), where the operand
// traffic per flop is small: a workgroup of 4 wavefronts (2 x 2) owns a BM x BN output tile, walks the reduction in
// tiles of 16, and stages operands global -> registers -> LDS, double buffered.  Both tiles sit in LDS as
// [k][row] (row contiguous), so an MFMA operand (lane l: row l % 32, k l / 32) is one conflict-free 4-byte read per
// lane.  Operands that are contiguous along the reduction in memory (x / dy gathered per pixel, the forward filter) are
// fetched as 4 consecutive k of one row and written to LDS as 4 scalars; operands contiguous along their own row index
// (the filter in backward-data, dy and x in backward-weight) as 4 consecutive rows of one k, one 16-byte write.  With
// channel counts that are not multiples of 4 the same kernel fetches element by element (VEC = false).
//
// Addressing is the plain index definition of each operation, bounds-checked per fetched vector; a strided
// backward-data runs over every input pixel and finds the structural zeros by the divisibility test (no compact
// form as in the FP16 path).  Split reductions (backward-weight) leave FP32 partial sums in the workspace, added in
// index order by splitk_reduce_f32: deterministic.
#include <hip/hip_runtime.h>

#include "jz_igemm.h"
#include "jz_internal.h"

namespace {
using namespace jz;

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int F_THREADS = 256;
constexpr int F_BK = 16;  // reduction elements per tile

struct F32Args {
  const float* A;
  const float* B;
  float* D;      // [M][N], written when splits == 1
  float* Dpart;  // [splits][M][N]
  int M, N, Kred;
  int nkt, kt_per_split, splits, tiles_m, tiles_n;
  ConvGeom g;
};

// Address of the gathered tensor's element for pixel `pix` of the (n, OH, OW) grid at filter tap `tap`, channel c, or
// nullptr when the tap falls outside the image (or, backward-data, when no output pixel reads the input pixel through it).
template <int OP>
__device__ __forceinline__ const float* gather_addr(const ConvGeom& g, const float* T, unsigned pix, unsigned tap, unsigned c) {
  const unsigned n = fd_div(pix, g.d_ohow);
  const unsigned rem = pix - n * (unsigned)(g.OH * g.OW);
  const unsigned oh = fd_div(rem, g.d_ow);
  const unsigned ow = rem - oh * (unsigned)g.OW;
  const unsigned r = fd_div(tap, g.d_s);
  const unsigned s = tap - r * (unsigned)g.S;
  int ih, iw;
  if (OP == OP_BWD_DATA) {
    const int th = (int)oh + g.ph - (int)r, tw = (int)ow + g.pw - (int)s;
    if (th < 0 || tw < 0) return nullptr;
    ih = (int)fd_div((unsigned)th, g.d_sh);
    iw = (int)fd_div((unsigned)tw, g.d_sw);
    if (ih * g.sh != th || iw * g.sw != tw) return nullptr;
  } else {
    ih = (int)oh * g.sh - g.ph + (int)r;
    iw = (int)ow * g.sw - g.pw + (int)s;
  }
  if ((unsigned)ih >= (unsigned)g.IH || (unsigned)iw >= (unsigned)g.IW) return nullptr;
  return T + ((size_t)(n * g.IH + ih) * g.IW + iw) * g.IC + c;
}

// A(m, k) and B(n, k) of the three operations (table in jz_igemm.h): address or nullptr (= zero)
template <int OP>
__device__ __forceinline__ const float* addrA(const F32Args& a, int m, int k) {
  if (m >= a.M || k >= a.Kred) return nullptr;
  if (OP == OP_BWD_WEIGHT) return a.A + (size_t)k * a.M + m;  // dy[(n,p,q)][k_out]
  const unsigned tap = fd_div((unsigned)k, a.g.d_ic);
  return gather_addr<OP>(a.g, a.A, (unsigned)m, tap, (unsigned)k - tap * (unsigned)a.g.IC);
}
template <int OP>
__device__ __forceinline__ const float* addrB(const F32Args& a, int n, int k) {
  if (n >= a.N || k >= a.Kred) return nullptr;
  if (OP == OP_FWD) return a.B + (size_t)n * a.Kred + k;  // w[k_out][(r,s,c)]
  if (OP == OP_BWD_DATA) {                                  // w[k_out][r][s][c] read as B(c, (r,s,k_out))
    const unsigned tap = fd_div((unsigned)k, a.g.d_ic);
    const unsigned ko = (unsigned)k - tap * (unsigned)a.g.IC;
    return a.B + ((size_t)ko * (a.g.R * a.g.S) + tap) * a.N + n;
  }
  const unsigned tap = fd_div((unsigned)n, a.g.d_ic);  // backward-weight: n = (r,s,c), k = (n,p,q)
  return gather_addr<OP_FWD>(a.g, a.B, (unsigned)k, tap, (unsigned)n - tap * (unsigned)a.g.IC);
}

// Four operand values: along k (KC = true: row fixed, k .. k+3) or along the row index (row .. row+3, k fixed).  VEC:
// the four lie in one aligned 16-byte piece of memory and share their validity (the host checked the divisibility that
// guarantees it).
template <int OP, bool IS_A, bool KC, bool VEC>
__device__ __forceinline__ float4 fetch4(const F32Args& a, int row, int k) {
  auto at = [&](int r, int kk) { return IS_A ? addrA<OP>(a, r, kk) : addrB<OP>(a, r, kk); };
  if (VEC) {
    const float* p = at(row, k);
    return p ? *reinterpret_cast<const float4*>(p) : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  float v[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float* p = KC ? at(row, k + j) : at(row + j, k);
    v[j] = p ? *p : 0.0f;
  }
  return make_float4(v[0], v[1], v[2], v[3]);
}

template <int OP, bool VEC, int BM, int BN>
__global__ __launch_bounds__(F_THREADS) void igemm_f32_kernel(F32Args a) {
  constexpr bool A_KC = OP != OP_BWD_WEIGHT, B_KC = OP == OP_FWD;
  constexpr int TM = BM / 64, TN = BN / 64;      // 32x32 MFMA tiles per wavefront (2 x 2 wavefronts)
  constexpr int PA = BM + 32, PB = BN + 32;      // LDS row pitch: k and k+1 land in different halves of the banks
  constexpr int QA = BM * F_BK / 4 / F_THREADS;  // 4-element fetches per thread and tile
  constexpr int QB = BN * F_BK / 4 / F_THREADS;
  static_assert(QA >= 1 && QB >= 1, "tile too small for 256 loaders");
  __shared__ __align__(16) float sA[2][F_BK][PA];
  __shared__ __align__(16) float sB[2][F_BK][PB];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  unsigned L = blockIdx.x;
  const int tiles_mn = a.tiles_m * a.tiles_n;
  const int split = (int)(L / (unsigned)tiles_mn);
  L -= (unsigned)split * (unsigned)tiles_mn;
  const int m0 = (int)(L / (unsigned)a.tiles_n) * BM;
  const int n0 = (int)(L % (unsigned)a.tiles_n) * BN;
  const int kt_begin = split * a.kt_per_split;
  const int kt_end = kt_begin + a.kt_per_split < a.nkt ? kt_begin + a.kt_per_split : a.nkt;

  // fetch q of this thread: KC operand: row = f % ROWS, k quad = f / ROWS; row-contiguous operand: row quad = f % (ROWS/4),
  // k = f / (ROWS/4); f = q * 256 + tid.  Consecutive lanes: consecutive rows (KC: conflict-free scalar LDS writes) or
  // consecutive row quads (coalesced 16-byte accesses).
  float4 ra[QA], rb[QB];
  auto fetch = [&](int kt) {
    const int k0 = kt * F_BK;
#pragma unroll
    for (int q = 0; q < QA; ++q) {
      const int f = q * F_THREADS + tid;
      ra[q] = A_KC ? fetch4<OP, true, true, VEC>(a, m0 + f % BM, k0 + 4 * (f / BM))
                   : fetch4<OP, true, false, VEC>(a, m0 + 4 * (f % (BM / 4)), k0 + f / (BM / 4));
    }
#pragma unroll
    for (int q = 0; q < QB; ++q) {
      const int f = q * F_THREADS + tid;
      rb[q] = B_KC ? fetch4<OP, false, true, VEC>(a, n0 + f % BN, k0 + 4 * (f / BN))
                   : fetch4<OP, false, false, VEC>(a, n0 + 4 * (f % (BN / 4)), k0 + f / (BN / 4));
    }
  };
  auto stash = [&](int buf) {
#pragma unroll
    for (int q = 0; q < QA; ++q) {
      const int f = q * F_THREADS + tid;
      if (A_KC) {
        const int row = f % BM, kq = 4 * (f / BM);
        sA[buf][kq][row] = ra[q].x; sA[buf][kq + 1][row] = ra[q].y; sA[buf][kq + 2][row] = ra[q].z; sA[buf][kq + 3][row] = ra[q].w;
      } else {
        *reinterpret_cast<float4*>(&sA[buf][f / (BM / 4)][4 * (f % (BM / 4))]) = ra[q];
      }
    }
#pragma unroll
    for (int q = 0; q < QB; ++q) {
      const int f = q * F_THREADS + tid;
      if (B_KC) {
        const int row = f % BN, kq = 4 * (f / BN);
        sB[buf][kq][row] = rb[q].x; sB[buf][kq + 1][row] = rb[q].y; sB[buf][kq + 2][row] = rb[q].z; sB[buf][kq + 3][row] = rb[q].w;
      } else {
        *reinterpret_cast<float4*>(&sB[buf][f / (BN / 4)][4 * (f % (BN / 4))]) = rb[q];
      }
    }
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  if (kt_begin < kt_end) {
    fetch(kt_begin);
    stash(0);
  }
  __syncthreads();
  int buf = 0;
  const int arow = wm * (BM / 2) + (lane & 31), brow = wn * (BN / 2) + (lane & 31), kh = lane >> 5;
  for (int kt = kt_begin; kt < kt_end; ++kt) {
    const bool more = kt + 1 < kt_end;
    if (more) fetch(kt + 1);  // in flight while this tile is multiplied
#pragma unroll
    for (int ks = 0; ks < F_BK / 2; ++ks) {
      float fa[TM], fb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) fa[i] = sA[buf][2 * ks + kh][arow + 32 * i];
#pragma unroll
      for (int j = 0; j < TN; ++j) fb[j] = sB[buf][2 * ks + kh][brow + 32 * j];
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          // n operand in the first slot: each lane then owns 4 consecutive n for one m (row = lane % 32)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fb[j], fa[i], acc[i][j], 0, 0, 0);
    }
    if (more) stash(buf ^ 1);
    __syncthreads();
    buf ^= 1;
  }

  // accumulator register r of tile (i,j): m = wrow + 32 i + lane % 32, n = wcol + 32 j + 8 (r / 4) + 4 (lane / 32) + r % 4
  float* out = a.splits > 1 ? a.Dpart + (size_t)split * a.M * a.N : a.D;
  const bool vec = (a.N & 3) == 0;
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int m = m0 + wm * (BM / 2) + 32 * i + (lane & 31);
    if (m >= a.M) continue;
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int n = n0 + wn * (BN / 2) + 32 * j + 8 * q4 + 4 * (lane >> 5);
        float* dst = out + (size_t)m * a.N + n;
        if (vec && n + 3 < a.N) {
          *reinterpret_cast<float4*>(dst) = make_float4(acc[i][j][4 * q4], acc[i][j][4 * q4 + 1], acc[i][j][4 * q4 + 2], acc[i][j][4 * q4 + 3]);
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (n + e < a.N) dst[e] = acc[i][j][4 * q4 + e];
        }
      }
  }
}

// D[i] = sum_s part[s][i], splits added in index order
__global__ __launch_bounds__(256) void splitk_reduce_f32(const float* __restrict__ part, float* __restrict__ out, long long MN, int splits) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= MN) return;
  float s = 0.0f;
  for (int k = 0; k < splits; ++k) s += part[(size_t)k * MN + i];
  out[i] = s;
}

struct PlanF32 {
  int op = 0;
  bool vec = false;
  int tile = 128;
  F32Args args{};
  size_t ws_bytes = 0, bytesA = 0, bytesB = 0, bytesD = 0;
};

int out_dim(int in, int pad, int f, int st) { return (in + 2 * pad - f) / st + 1; }

int make_plan_f32(int op, const jz_conv_desc* d, PlanF32* pl) {
  if (!d) return JZ_ERR_NULL;
  if (op != JZ_FWD && op != JZ_BWD_DATA && op != JZ_BWD_WEIGHT) return JZ_ERR_UNSUPPORTED;
  if (d->N <= 0 || d->H <= 0 || d->W <= 0 || d->C <= 0 || d->K <= 0 || d->R <= 0 || d->S <= 0 || d->stride_h <= 0 ||
      d->stride_w <= 0 || d->pad_h < 0 || d->pad_w < 0)
    return JZ_ERR_SHAPE;
  if (d->pad_h >= d->R || d->pad_w >= d->S) return JZ_ERR_SHAPE;
  if (d->H + 2 * d->pad_h < d->R || d->W + 2 * d->pad_w < d->S) return JZ_ERR_SHAPE;
  const int P = out_dim(d->H, d->pad_h, d->R, d->stride_h), Q = out_dim(d->W, d->pad_w, d->S, d->stride_w);
  if (P <= 0 || Q <= 0) return JZ_ERR_SHAPE;
  const long long lim = (1ll << 30) - 1;  // the same bound as the FP16 path: GEMM dimensions and pixel indices fit 32 bits
  const long long nx = (long long)d->N * d->H * d->W * d->C, ny = (long long)d->N * P * Q * d->K,
                  nw = (long long)d->K * d->R * d->S * d->C;
  if (nx > lim || ny > lim || nw > lim) return JZ_ERR_UNSUPPORTED;
  F32Args& a = pl->args;
  ConvGeom& g = a.g;
  pl->op = op;
  g.R = d->R; g.S = d->S; g.sh = d->stride_h; g.sw = d->stride_w; g.ph = d->pad_h; g.pw = d->pad_w;
  g.kvalid = 0; g.tap_rep = 0;
  if (op == JZ_FWD) {
    a.M = d->N * P * Q; a.N = d->K; a.Kred = d->R * d->S * d->C;
    g.IH = d->H; g.IW = d->W; g.IC = d->C; g.OH = P; g.OW = Q;
    pl->vec = d->C % 4 == 0;
    pl->bytesA = 4 * nx; pl->bytesB = 4 * nw; pl->bytesD = 4 * ny;
  } else if (op == JZ_BWD_DATA) {
    a.M = d->N * d->H * d->W; a.N = d->C; a.Kred = d->R * d->S * d->K;
    g.IH = P; g.IW = Q; g.IC = d->K; g.OH = d->H; g.OW = d->W;
    pl->vec = d->K % 4 == 0 && d->C % 4 == 0;
    pl->bytesA = 4 * ny; pl->bytesB = 4 * nw; pl->bytesD = 4 * nx;
  } else {
    a.M = d->K; a.N = d->R * d->S * d->C; a.Kred = d->N * P * Q;
    g.IH = d->H; g.IW = d->W; g.IC = d->C; g.OH = P; g.OW = Q;
    pl->vec = d->K % 4 == 0 && d->C % 4 == 0;
    pl->bytesA = 4 * ny; pl->bytesB = 4 * nx; pl->bytesD = 4 * nw;  // A = dy, B = x
  }
  g.row_pitch = g.IW * g.IC; g.pix_step = g.IC; g.s_step = g.IC;
  g.d_ohow = make_fastdiv((unsigned)(g.OH * g.OW));
  g.d_ow = make_fastdiv((unsigned)g.OW);
  g.d_ic = make_fastdiv((unsigned)g.IC);
  g.d_s = make_fastdiv((unsigned)g.S);
  g.d_sh = make_fastdiv((unsigned)g.sh);
  g.d_sw = make_fastdiv((unsigned)g.sw);
  // Tile and split: 128 x 128 tiles where they give the chip (256 compute units, two workgroups each) enough
  // workgroups, else 64 x 64; then split the reduction until about 512 workgroups exist, never shorter than 8 k tiles.
  a.nkt = (a.Kred + F_BK - 1) / F_BK;
  auto tiles = [&](int t) { return (long long)((a.M + t - 1) / t) * ((a.N + t - 1) / t); };
  pl->tile = tiles(128) >= 384 ? 128 : 64;
  a.tiles_m = (a.M + pl->tile - 1) / pl->tile;
  a.tiles_n = (a.N + pl->tile - 1) / pl->tile;
  long long want = 512 / tiles(pl->tile);
  if (want > a.nkt / 8) want = a.nkt / 8;
  if (want > 256) want = 256;
  if (want < 1) want = 1;
  a.kt_per_split = (int)((a.nkt + want - 1) / want);
  a.splits = (a.nkt + a.kt_per_split - 1) / a.kt_per_split;
  pl->ws_bytes = a.splits > 1 ? (size_t)a.splits * a.M * a.N * sizeof(float) : 0;
  return JZ_OK;
}

template <int OP>
void launch_f32(const PlanF32& pl, hipStream_t st) {
  const F32Args& a = pl.args;
  const dim3 grid((unsigned)a.tiles_m * (unsigned)a.tiles_n * (unsigned)a.splits), block(F_THREADS);
  if (pl.tile == 128) {
    if (pl.vec) hipLaunchKernelGGL((igemm_f32_kernel<OP, true, 128, 128>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((igemm_f32_kernel<OP, false, 128, 128>), grid, block, 0, st, a);
  } else {
    if (pl.vec) hipLaunchKernelGGL((igemm_f32_kernel<OP, true, 64, 64>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((igemm_f32_kernel<OP, false, 64, 64>), grid, block, 0, st, a);
  }
}

// A, B in the kernel's order: FWD (x, w), BWD_DATA (dy, w), BWD_WEIGHT (dy, x)
int run_f32(int op, const jz_conv_desc* d, const void* A, const void* B, void* D, void* ws, size_t ws_bytes, void* stream) {
  PlanF32 pl;
  int rc = make_plan_f32(op, d, &pl);
  if (rc != JZ_OK) return rc;
  if (!A || !B || !D) return JZ_ERR_NULL;
  if (!aligned16(A) || !aligned16(B) || !aligned16(D) || (ws && !aligned16(ws))) return JZ_ERR_ALIGN;
  if (overlaps(D, pl.bytesD, A, pl.bytesA) || overlaps(D, pl.bytesD, B, pl.bytesB)) return JZ_ERR_ALIAS;
  if (pl.ws_bytes > 0 && (!ws || ws_bytes < pl.ws_bytes)) return JZ_ERR_WORKSPACE;
  if (pl.ws_bytes > 0 && (overlaps(ws, pl.ws_bytes, A, pl.bytesA) || overlaps(ws, pl.ws_bytes, B, pl.bytesB) ||
                          overlaps(ws, pl.ws_bytes, D, pl.bytesD)))
    return JZ_ERR_ALIAS;
  hipStream_t st = static_cast<hipStream_t>(stream);
  F32Args& a = pl.args;
  a.A = static_cast<const float*>(A);
  a.B = static_cast<const float*>(B);
  a.D = static_cast<float*>(D);
  a.Dpart = static_cast<float*>(ws);
  if (op == JZ_FWD) launch_f32<OP_FWD>(pl, st);
  else if (op == JZ_BWD_DATA) launch_f32<OP_BWD_DATA>(pl, st);
  else launch_f32<OP_BWD_WEIGHT>(pl, st);
  if ((rc = jz::launch_status()) != JZ_OK) return rc;
  if (a.splits > 1) {
    const long long MN = (long long)a.M * a.N;
    hipLaunchKernelGGL(splitk_reduce_f32, dim3((unsigned)((MN + 255) / 256)), dim3(256), 0, st, (const float*)a.Dpart, a.D, MN, a.splits);
    rc = jz::launch_status();
  }
  return rc;
}

int fc_desc_f32(int mode, int batch, int in_features, int out_features, jz_conv_desc* d) {
  if (mode != JZ_FWD && mode != JZ_BWD_DATA && mode != JZ_BWD_WEIGHT) return JZ_ERR_UNSUPPORTED;
  if (batch <= 0 || in_features <= 0 || out_features <= 0) return JZ_ERR_SHAPE;
  *d = jz_conv_desc{batch, 1, 1, in_features, out_features, 1, 1, 1, 1, 0, 0};  // a 1x1 convolution over a 1x1 image
  return JZ_OK;
}

}  // namespace

extern "C" int jz_conv2d_f32_workspace_bytes(int op, const jz_conv_desc* desc, size_t* bytes) {
  if (!bytes) return JZ_ERR_NULL;
  PlanF32 pl;
  int rc = make_plan_f32(op, desc, &pl);
  if (rc != JZ_OK) return rc;
  *bytes = pl.ws_bytes;
  return JZ_OK;
}

extern "C" int jz_conv2d_fwd_f32(const jz_conv_desc* desc, const float* x32, const float* w32, float* y32, void* ws,
                                 size_t ws_bytes, void* hip_stream) {
  return run_f32(JZ_FWD, desc, x32, w32, y32, ws, ws_bytes, hip_stream);
}

extern "C" int jz_conv2d_bwd_data_f32(const jz_conv_desc* desc, const float* dy32, const float* w32, float* dx32, void* ws,
                                      size_t ws_bytes, void* hip_stream) {
  return run_f32(JZ_BWD_DATA, desc, dy32, w32, dx32, ws, ws_bytes, hip_stream);
}

extern "C" int jz_conv2d_bwd_weight_f32(const jz_conv_desc* desc, const float* x32, const float* dy32, float* dw32, void* ws,
                                        size_t ws_bytes, void* hip_stream) {
  return run_f32(JZ_BWD_WEIGHT, desc, dy32, x32, dw32, ws, ws_bytes, hip_stream);  // A = dy, B = x
}

extern "C" int jz_gemm_fc_f32_workspace_bytes(int mode, int batch, int in_features, int out_features, size_t* bytes) {
  jz_conv_desc d;
  int rc = fc_desc_f32(mode, batch, in_features, out_features, &d);
  if (rc != JZ_OK) return rc;
  return jz_conv2d_f32_workspace_bytes(mode, &d, bytes);
}

extern "C" int jz_gemm_fc_f32(int mode, int batch, int in_features, int out_features, const float* a32, const float* b32,
                              float* out32, void* ws, size_t ws_bytes, void* hip_stream) {
  jz_conv_desc d;
  int rc = fc_desc_f32(mode, batch, in_features, out_features, &d);
  if (rc != JZ_OK) return rc;
  // FWD: (x, w) ; BWD_DATA: (dy, w) ; BWD_WEIGHT: (dy, x) -- already the kernel's (A, B) order in every mode
  return run_f32(mode, &d, a32, b32, out32, ws, ws_bytes, hip_stream);
}
