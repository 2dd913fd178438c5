// Device code of the implicit-GEMM family and its launchers, included by one translation unit per operation:
// element-wise operand access and the kernel built on it (every shape that allows no 16-byte vector access), the
// epilogue shared by all kernels, the production kernel (jz_igemm_dma.h) and the variant dispatch.
#pragma once
#include <type_traits>

#include "jz_conv_plan.h"

namespace {
using namespace jz;

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr int THREADS = 256;
constexpr int BK = 64;
constexpr int LDK = BK + 8;  // LDS row pitch in halves
constexpr int KCH = BK / 8;  // 16-byte chunks per tile row
constexpr int LOADERS = 128; // threads per operand

__device__ __forceinline__ unsigned xcd_remap(unsigned bid, unsigned nb) {
  // consecutive workgroup ids land on different XCDs (each with its own L2); give every XCD one
  // contiguous run of tiles instead so that neighbouring tiles share their operand rows in L2
  const unsigned X = 8;
  unsigned q = nb / X, rem = nb % X, xcd = bid % X, local = bid / X;
  return xcd * q + (xcd < rem ? xcd : rem) + local;
}

// ---------------------------------------------------------------------------------------------
// element-wise (generic) operand access: the plain index definitions, every bound checked
// ---------------------------------------------------------------------------------------------
template <int OP>
__device__ __forceinline__ unsigned short elem_gather(const GemmArgs& a, const unsigned short* T, unsigned pix,
                                                       unsigned tap, unsigned c) {
  // value of the gathered tensor for output pixel `pix` of the (n,OH,OW) grid at filter tap `tap`, channel c
  const ConvGeom& g = a.g;
  unsigned n = fd_div(pix, g.d_ohow);
  unsigned rem = pix - n * (unsigned)(g.OH * g.OW);
  unsigned oh = fd_div(rem, g.d_ow);
  unsigned ow = rem - oh * (unsigned)g.OW;
  unsigned r = fd_div(tap, g.d_s);
  unsigned s = tap - r * (unsigned)g.S;
  int ih, iw;
  if (OP == OP_BWD_DATA) {
    int th = (int)oh + g.ph - (int)r, tw = (int)ow + g.pw - (int)s;
    if (th < 0 || tw < 0) return 0;
    ih = (int)fd_div((unsigned)th, g.d_sh);
    iw = (int)fd_div((unsigned)tw, g.d_sw);
    if (ih * g.sh != th || iw * g.sw != tw) return 0;  // no output pixel reads this input pixel through this tap
  } else {
    ih = (int)oh * g.sh - g.ph + (int)r;
    iw = (int)ow * g.sw - g.pw + (int)s;
  }
  if ((unsigned)ih >= (unsigned)g.IH || (unsigned)iw >= (unsigned)g.IW) return 0;
  return T[((size_t)(n * g.IH + ih) * g.IW + iw) * g.IC + c];
}

template <int OP>
__device__ __forceinline__ unsigned short elemA(const GemmArgs& a, int m, int k) {
  if (m >= a.M || k >= a.Kred) return 0;
  if (OP == OP_BWD_WEIGHT) return a.A[(size_t)k * a.M + m];  // dy[(n,p,q)][k_out]
  unsigned tap = fd_div((unsigned)k, a.g.d_ic);
  unsigned c = (unsigned)k - tap * (unsigned)a.g.IC;
  return elem_gather<OP>(a, a.A, (unsigned)m, tap, c);
}

template <int OP>
__device__ __forceinline__ unsigned short elemB(const GemmArgs& a, int n, int k) {
  if (n >= a.N || k >= a.Kred) return 0;
  if (OP == OP_FWD) return a.B[(size_t)n * a.Kred + k];  // w[k_out][(r,s,c)]
  if (OP == OP_BWD_DATA) {                                // w[k_out][r][s][c] read as B(c, (r,s,k_out))
    unsigned tap = fd_div((unsigned)k, a.g.d_ic);
    unsigned ko = (unsigned)k - tap * (unsigned)a.g.IC;
    return a.B[((size_t)ko * (a.g.R * a.g.S) + tap) * a.N + n];
  }
  unsigned tap = fd_div((unsigned)n, a.g.d_ic);  // BWD_WEIGHT: n = (r,s,c), k = (n,p,q)
  unsigned c = (unsigned)n - tap * (unsigned)a.g.IC;
  return elem_gather<OP_FWD>(a, a.B, (unsigned)k, tap, c);
}

// ---------------------------------------------------------------------------------------------
// epilogue shared by both kernels: fp32 partial sums (split-K) or the single rounding to fp16
// ---------------------------------------------------------------------------------------------
// wrow / wcol: first row / column of this wavefront's share inside the BM x BN tile; NTHREADS: workgroup size;
// EPASS: the fp16 tile is staged through LDS in EPASS slabs of BM / EPASS rows (a 256x256 tile is larger than the ring)
// slabs of rows the fp32 tile of a split reduction is staged in: the slab has to fit LDS_BYTES and hold whole wavefront
// shares (WTM rows); 0 when no such slab exists (the partial sums are then stored straight from the registers)
constexpr int fp32_slabs(int bm, int bn, int wtm, int lds_bytes) {
  for (int s = 1; bm / s >= wtm; s *= 2)
    if ((bm / s) * (bn + 4) * 4 <= lds_bytes) return s;
  return 0;
}

template <int BM, int BN, int TM, int TN, int NTHREADS, int EPASS = 1, int LDS_BYTES = 0, int STATS = 0>
__device__ __forceinline__ void igemm_epilogue_impl(const GemmArgs& a, f32x16 (&acc)[TM][TN], unsigned short* lds, int m0,
                                                    int n0, int split, int tid, int lane, int wrow, int wcol) {
  // ---- epilogue ------------------------------------------------------------------------------
  // accumulator register r of tile (i,j): m = wrow + 32 i + lane%32, n = wcol + 32 j + 8 (r/4) + 4 (lane/32) + r%4
  constexpr int FSL = fp32_slabs(BM, BN, 32 * TM, LDS_BYTES);
  if (a.splits > 1 && FSL > 0 && (a.N & 3) == 0) {
    // fp32 partial sums, staged through LDS slab by slab so that a store instruction writes whole 512-byte row pieces
    // (from the registers a wavefront would write 32 rows x 32 bytes per instruction)
    float* P = a.Dpart + (size_t)split * a.M * a.N;
    constexpr int LDF = BN + 4;            // floats per staged row: 16-byte aligned, rows 16 bytes apart in the banks
    constexpr int RPB = BM / (FSL > 0 ? FSL : 1);  // rows per slab
    constexpr int FCH = BN / 4;            // 16-byte chunks per row
    constexpr int FRPP = NTHREADS / FCH;   // rows per store pass
    static_assert(FRPP >= 1 && RPB % FRPP == 0, "slab rows must divide among the store passes");
    float* sF = reinterpret_cast<float*>(lds);
    const int fch = tid % FCH, frow = tid / FCH;
#pragma unroll
    for (int ps = 0; ps < FSL; ++ps) {
      if (ps > 0) __syncthreads();  // the previous slab has been stored
      if (FSL == 1 || wrow / RPB == ps) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
              int row = wrow - ps * RPB + 32 * i + (lane & 31);
              int col = wcol + 32 * j + 8 * q4 + 4 * (lane >> 5);
              *reinterpret_cast<float4*>(sF + row * LDF + col) =
                  make_float4(acc[i][j][4 * q4], acc[i][j][4 * q4 + 1], acc[i][j][4 * q4 + 2], acc[i][j][4 * q4 + 3]);
            }
      }
      __syncthreads();
#pragma unroll
      for (int i = 0; i < RPB / FRPP; ++i) {
        int row = frow + FRPP * i;
        int m = m0 + ps * RPB + row, n = n0 + fch * 4;
        if (m >= a.M || n >= a.N) continue;
        *reinterpret_cast<float4*>(P + (size_t)m * a.N + n) = *reinterpret_cast<const float4*>(sF + row * LDF + fch * 4);
      }
    }
    return;
  }
  if (a.splits > 1) {
    float* P = a.Dpart + (size_t)split * a.M * a.N;
    const bool vec = (a.N & 3) == 0;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      int m = m0 + wrow + 32 * i + (lane & 31);
      if (m >= a.M) continue;
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          int n = n0 + wcol + 32 * j + 8 * q4 + 4 * (lane >> 5);
          float* dst = P + (size_t)m * a.N + n;
          if (vec && n + 3 < a.N) {
            *reinterpret_cast<float4*>(dst) =
                make_float4(acc[i][j][4 * q4], acc[i][j][4 * q4 + 1], acc[i][j][4 * q4 + 2], acc[i][j][4 * q4 + 3]);
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (n + e < a.N) dst[e] = acc[i][j][4 * q4 + e];
          }
        }
    }
    return;
  }
  // single rounding fp32 -> fp16 (round to nearest even), staged through LDS for 16-byte coalesced stores
  constexpr int LDC = BN + 8;
  constexpr int RPB = BM / EPASS;  // rows per slab
  static_assert(RPB * EPASS == BM && RPB % (32 * TM) == 0, "a wavefront's rows must lie inside one slab");
  unsigned short* sC = lds;  // the k loop ended with a barrier: the tile buffers are free
  constexpr int CCH = BN / 8;             // 16-byte chunks per output row
  constexpr int CRPP = NTHREADS / CCH;    // rows per pass
  static_assert(RPB % CRPP == 0, "slab rows must divide among the store passes");
  const int cch = tid % CCH, crow = tid / CCH;
  const bool nvec = (a.N & 7) == 0;
  // optional per-tile column sums: a thread stores the same 8 columns of every row it handles, so it keeps their sums;
  // they are combined below (a template argument: as a run-time branch in every kernel it cost the step 5 %).
  // STATS 1 (a batch normalization behind a forward convolution): sums of what is stored and of its squares.
  // STATS 2 (backward-data of a convolution whose input came out of batch normalization + ReLU): the sums that layer's
  // backward pass needs, sum g and sum g x^ with g = the stored gradient where the ReLU was open (st_y > 0), else 0.
  // STATS 3 (backward-data whose output is one contribution to the gradient at the end of a residual block): what is
  // stored is g = RNE16(tile [+ st_add]) where st_y > 0, else 0, and the sums are those of that g.
  static_assert(!STATS || LDS_BYTES >= 64 * NTHREADS, "the ring has to hold the partial sums");
  constexpr bool CAN_STATS = STATS != 0;
  constexpr bool stats = STATS != 0;
  float ssum[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}, ssq[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  float st_mu[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}, st_is[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if constexpr (STATS >= 2) {
    const int nn = n0 + cch * 8;  // N is a multiple of 8 in this mode
    if (nn < a.N) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        st_mu[e] = a.st_mean[nn + e];
        st_is[e] = a.st_invstd[nn + e];
      }
    }
  }
#pragma unroll
  for (int ps = 0; ps < EPASS; ++ps) {
    if (ps > 0) __syncthreads();  // the previous slab has been stored
    if (EPASS == 1 || wrow / RPB == ps) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            int row = wrow - ps * RPB + 32 * i + (lane & 31);
            int col = wcol + 32 * j + 8 * q4 + 4 * (lane >> 5);
            _Float16 h[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) h[e] = (_Float16)acc[i][j][4 * q4 + e];
            uint2 pk;
            __builtin_memcpy(&pk, h, 8);
            *reinterpret_cast<uint2*>(sC + row * LDC + col) = pk;
          }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < RPB / CRPP; ++i) {
      int row = crow + CRPP * i;
      int m = m0 + ps * RPB + row, n = n0 + cch * 8;
      if (m >= a.M || n >= a.N) continue;
      const unsigned short* src = sC + row * LDC + cch * 8;
      if constexpr (stats) {
        const uint4 pk = *reinterpret_cast<const uint4*>(src);  // one 16-byte LDS read (columns beyond N hold zeros' worth
        const unsigned pw[4] = {pk.x, pk.y, pk.z, pk.w};          // of padding and are never written out)
        unsigned yw[4] = {0u, 0u, 0u, 0u}, cw[4] = {0u, 0u, 0u, 0u}, dw[4] = {0u, 0u, 0u, 0u}, gw[4] = {0u, 0u, 0u, 0u};
        if constexpr (STATS >= 2) {  // the same 16 bytes of the normalization's output and input (no scatter in this mode)
          const uint4 yq = *reinterpret_cast<const uint4*>(a.st_y + (size_t)m * a.N + n);
          const uint4 cq = *reinterpret_cast<const uint4*>(a.st_c + (size_t)m * a.N + n);
          yw[0] = yq.x; yw[1] = yq.y; yw[2] = yq.z; yw[3] = yq.w;
          cw[0] = cq.x; cw[1] = cq.y; cw[2] = cq.z; cw[3] = cq.w;
          if constexpr (STATS == 3) {
            if (a.st_add) {
              const uint4 dq = *reinterpret_cast<const uint4*>(a.st_add + (size_t)m * a.N + n);
              dw[0] = dq.x; dw[1] = dq.y; dw[2] = dq.z; dw[3] = dq.w;
            }
          }
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const unsigned short hb = (unsigned short)(e & 1 ? pw[e >> 1] >> 16 : pw[e >> 1] & 0xffffu);
          _Float16 hv;
          __builtin_memcpy(&hv, &hb, 2);
          const float v = (float)hv;
          if constexpr (STATS == 1) {
            ssum[e] += v;
            ssq[e] += v * v;
          } else {
            const unsigned short yb = (unsigned short)(e & 1 ? yw[e >> 1] >> 16 : yw[e >> 1] & 0xffffu);
            const unsigned short cb = (unsigned short)(e & 1 ? cw[e >> 1] >> 16 : cw[e >> 1] & 0xffffu);
            _Float16 yv, cv;
            __builtin_memcpy(&yv, &yb, 2);
            __builtin_memcpy(&cv, &cb, 2);
            float g = (float)yv > 0.f ? v : 0.f;
            if constexpr (STATS == 3) {  // the sum of the two contributions is exact in FP32 and rounded once
              const unsigned short db = (unsigned short)(e & 1 ? dw[e >> 1] >> 16 : dw[e >> 1] & 0xffffu);
              _Float16 dv;
              __builtin_memcpy(&dv, &db, 2);
              const _Float16 gh = (_Float16)(v + (float)dv);
              unsigned short gb;
              __builtin_memcpy(&gb, &gh, 2);
              if (!((float)yv > 0.f)) gb = 0;
              gw[e >> 1] |= (unsigned)gb << ((e & 1) * 16);
              _Float16 gm;
              __builtin_memcpy(&gm, &gb, 2);
              g = (float)gm;
            }
            ssum[e] += g;
            ssq[e] += g * (((float)cv - st_mu[e]) * st_is[e]);
          }
        }
        if constexpr (STATS == 3) {  // g replaces the tile's values in the output
          *reinterpret_cast<uint4*>(a.D16 + (size_t)m * a.N + n) = make_uint4(gw[0], gw[1], gw[2], gw[3]);
          continue;
        }
      }
      size_t drow = (size_t)m;
      if (a.sc_on) {  // row m = (n, p, q) of the strided grid goes to input pixel (n, p * sh + oh, q * sw + ow)
        unsigned nimg = fd_div((unsigned)m, a.g.d_ohow);
        unsigned rem = (unsigned)m - nimg * (unsigned)(a.g.OH * a.g.OW);
        unsigned p = fd_div(rem, a.g.d_ow);
        unsigned q = rem - p * (unsigned)a.g.OW;
        drow = ((size_t)nimg * a.sc_H + p * a.sc_sh + a.sc_oh) * a.sc_W + q * a.sc_sw + a.sc_ow;
        // strided 1x1: the other pixels of this sh x sw cell are read by no output pixel: their gradient is zero
        for (int i2 = 0; a.sc_fill && i2 < a.sc_sh; ++i2)
          for (int j2 = 0; j2 < a.sc_sw; ++j2) {
            if ((i2 | j2) == 0 || (int)(p * a.sc_sh) + i2 >= a.sc_H || (int)(q * a.sc_sw) + j2 >= a.sc_W) continue;
            unsigned short* z = a.D16 + (drow + (size_t)i2 * a.sc_W + j2) * a.N + n;
            if (nvec) {
              *reinterpret_cast<uint4*>(z) = make_uint4(0, 0, 0, 0);
            } else {
              for (int e = 0; e < 8 && n + e < a.N; ++e) z[e] = 0;
            }
          }
      }
      unsigned short* dst = a.D16 + drow * a.N + n;
      if (nvec) {
        *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(src);
      } else {
        for (int e = 0; e < 8 && n + e < a.N; ++e) dst[e] = src[e];
      }
    }
  }
  if constexpr (CAN_STATS) {
    // [2][CRPP][BN] floats in LDS (sums, then sums of squares), then one thread per column and kind adds the CRPP row
    // groups in a fixed order: the loads are independent and issued together, consecutive lanes read consecutive words
    __syncthreads();  // the staged tile has been read
    float* sS = reinterpret_cast<float*>(lds);
    float* w0 = sS + (crow * BN + cch * 8);
    float* w1 = w0 + CRPP * BN;
    *reinterpret_cast<float4*>(w0) = make_float4(ssum[0], ssum[1], ssum[2], ssum[3]);
    *reinterpret_cast<float4*>(w0 + 4) = make_float4(ssum[4], ssum[5], ssum[6], ssum[7]);
    *reinterpret_cast<float4*>(w1) = make_float4(ssq[0], ssq[1], ssq[2], ssq[3]);
    *reinterpret_cast<float4*>(w1 + 4) = make_float4(ssq[4], ssq[5], ssq[6], ssq[7]);
    __syncthreads();
    float* out = a.stats + (size_t)(m0 / BM) * 2 * a.N;
    for (int v = tid; v < 2 * BN; v += NTHREADS) {
      const int kind = v / BN, col = v - kind * BN;
      const float* src = sS + kind * CRPP * BN + col;
      float part[CRPP];
#pragma unroll
      for (int r = 0; r < CRPP; ++r) part[r] = src[r * BN];
      float s1 = 0.f;
#pragma unroll
      for (int r = 0; r < CRPP; ++r) s1 += part[r];
      if (n0 + col < a.N) out[kind * a.N + n0 + col] = s1;
    }
  }
}

template <int BM, int BN>
__device__ __forceinline__ void igemm_epilogue(const GemmArgs& a, f32x16 (&acc)[BM / 64][BN / 64], unsigned short* lds,
                                               int m0, int n0, int split, int tid, int lane, int wm, int wn) {
  constexpr int tile_bytes = 2 * (BM + BN) * LDK * 2, epi_bytes = BM * (BN + 8) * 2;
  igemm_epilogue_impl<BM, BN, BM / 64, BN / 64, THREADS, 1, (tile_bytes > epi_bytes ? tile_bytes : epi_bytes)>(
      a, acc, lds, m0, n0, split, tid, lane, wm * (BM / 2), wn * (BN / 2));
}

// ---------------------------------------------------------------------------------------------
// the kernel
// ---------------------------------------------------------------------------------------------
template <int OP, int BM, int BN>
__global__ __launch_bounds__(THREADS) void igemm_kernel(GemmArgs a) {
  constexpr int TM = BM / 64, TN = BN / 64;              // 32x32 MFMA tiles per wavefront
  constexpr int A_HALVES = BM * LDK, B_HALVES = BN * LDK;
  constexpr int RPP = LOADERS / KCH;                     // rows one pass of 128 loader threads covers (16)
  constexpr int PA = BM / RPP, PB = BN / RPP;            // passes over the A / B tile
  constexpr int NREG = PA > PB ? PA : PB;
  extern __shared__ __align__(16) unsigned short lds[];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const bool loadsA = wave < 2;
  const int tt = tid & (LOADERS - 1);
  const int kc = tt % KCH, rsub = tt / KCH;

  unsigned L = xcd_remap(blockIdx.x, gridDim.x);
  const int tiles_mn = a.tiles_m * a.tiles_n;
  const int split = (int)(L / (unsigned)tiles_mn);
  L -= (unsigned)split * (unsigned)tiles_mn;
  const int m0 = (int)(L / (unsigned)a.tiles_n) * BM;
  const int n0 = (int)(L % (unsigned)a.tiles_n) * BN;
  const int kt_begin = split * a.kt_per_split;
  const int kt_end = (kt_begin + a.kt_per_split < a.nkt) ? kt_begin + a.kt_per_split : a.nkt;

  uint4 rg[NREG];

  // fetch k tile `kt` of this thread's operand into rg[], element by element
  auto fetch = [&](int kt) {
    const int k0 = kt * BK;
    const int rows = loadsA ? PA : PB;
#pragma unroll
    for (int i = 0; i < NREG; ++i) {
      if (i < rows) {
        unsigned v[4];
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
          int k = k0 + kc * 8 + e;
          unsigned short lo, hi;
          if (loadsA) {
            lo = elemA<OP>(a, m0 + rsub + RPP * i, k);
            hi = elemA<OP>(a, m0 + rsub + RPP * i, k + 1);
          } else {
            lo = elemB<OP>(a, n0 + rsub + RPP * i, k);
            hi = elemB<OP>(a, n0 + rsub + RPP * i, k + 1);
          }
          v[e >> 1] = (unsigned)lo | ((unsigned)hi << 16);
        }
        rg[i] = make_uint4(v[0], v[1], v[2], v[3]);
      }
    }
  };

  // put rg[] into LDS buffer `buf`
  auto stash = [&](int buf) {
    unsigned short* base = lds + buf * (A_HALVES + B_HALVES) + (loadsA ? 0 : A_HALVES);
    const int rows = loadsA ? PA : PB;
#pragma unroll
    for (int i = 0; i < NREG; ++i)
      if (i < rows) *reinterpret_cast<uint4*>(base + (rsub + RPP * i) * LDK + kc * 8) = rg[i];
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
  for (int kt = kt_begin; kt < kt_end; ++kt) {
    const bool more = kt + 1 < kt_end;
    if (more) fetch(kt + 1);
    const unsigned short* sA = lds + buf * (A_HALVES + B_HALVES);
    const unsigned short* sB = sA + A_HALVES;
    const int arow = wm * (BM / 2) + (lane & 31), brow = wn * (BN / 2) + (lane & 31);
    const int kofs = (lane >> 5) * 8;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      half8 fa[TM], fb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) fa[i] = *reinterpret_cast<const half8*>(sA + (arow + 32 * i) * LDK + ks * 16 + kofs);
#pragma unroll
      for (int j = 0; j < TN; ++j) fb[j] = *reinterpret_cast<const half8*>(sB + (brow + 32 * j) * LDK + ks * 16 + kofs);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          // n operand in the first slot: each lane then owns 4 consecutive n for one m (row = lane % 32)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fb[j], fa[i], acc[i][j], 0, 0, 0);
    }
    if (more) stash(buf ^ 1);
    __syncthreads();
    buf ^= 1;
  }

  igemm_epilogue<BM, BN>(a, acc, lds, m0, n0, split, tid, lane, wm, wn);
}

#include "jz_igemm_dma.h"

template <int OP, int BM, int BN>
int launch_one(const GemmArgs& a, hipStream_t st) {
  constexpr size_t tile_bytes = 2 * (size_t)(BM + BN) * LDK * sizeof(unsigned short);
  constexpr size_t epi_bytes = (size_t)BM * (BN + 8) * sizeof(unsigned short);
  constexpr size_t smem = tile_bytes > epi_bytes ? tile_bytes : epi_bytes;
  static bool attr_set = false;  // per instantiation; setting it twice is harmless
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&igemm_kernel<OP, BM, BN>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
      return JZ_ERR_LAUNCH;
    attr_set = true;
  }
  unsigned grid = (unsigned)a.tiles_m * (unsigned)a.tiles_n * (unsigned)a.splits;
  hipLaunchKernelGGL((igemm_kernel<OP, BM, BN>), dim3(grid), dim3(THREADS), smem, st, a);
  return jz::launch_status();
}

template <int OP, int BM, int BN, int TBK, int NST, bool MASKA = false, int WGM = 2, int WGN = 2, bool GEN = false>
int launch_dma(const GemmArgs& a, hipStream_t st) {
  constexpr size_t ring_bytes = (size_t)NST * (BM + BN) * 2 * TBK;
  constexpr size_t epi_bytes = (size_t)BM / dma_epass(BM, BN) * (BN + 8) * sizeof(unsigned short);
  constexpr size_t smem = ring_bytes > epi_bytes ? ring_bytes : epi_bytes;
  static_assert(smem <= 160 * 1024, "more LDS than a compute unit has");
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&igemm_dma_kernel<OP, BM, BN, TBK, NST, MASKA, WGM, WGN, GEN>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
      return JZ_ERR_LAUNCH;
    attr_set = true;
  }
  unsigned grid = (unsigned)a.tiles_m * (unsigned)a.tiles_n * (unsigned)a.splits;
  hipLaunchKernelGGL((igemm_dma_kernel<OP, BM, BN, TBK, NST, MASKA, WGM, WGN, GEN>), dim3(grid), dim3(64 * WGM * WGN), smem, st, a);
  return jz::launch_status();
}

template <int OP>
int launch_op(const Plan& pl, hipStream_t st) {
  const GemmArgs& a = pl.args;
  constexpr bool IS_FWD = OP == OP_FWD || OP == OP_FWD_STATS;
  if constexpr (OP == OP_FWD_STATS) {
    if (!pl.fast) return JZ_ERR_UNSUPPORTED;  // only the ring kernels come in this form
  } else if constexpr (OP == OP_BWD_DATA_STATS || OP == OP_BWD_DATA_BLOCK_END) {
    if (!pl.fast || pl.gen || a.sc_on || a.splits != 1 || (a.N & 7) != 0) return JZ_ERR_UNSUPPORTED;
  } else {
    if (!pl.fast) return launch_one<OP, 128, 128>(a, st);
  }
  if (pl.packed && IS_FWD) {  // small-channel forward: tail of every gathered run is masked
    if (pl.bk == 32 && pl.nst == 3) {
      if (pl.BM == 128 && pl.BN == 128) return launch_dma<OP, 128, 128, 32, 3, true>(a, st);
      if (pl.BM == 128 && pl.BN == 64) return launch_dma<OP, 128, 64, 32, 3, true>(a, st);
      if (pl.BM == 64 && pl.BN == 128) return launch_dma<OP, 64, 128, 32, 3, true>(a, st);
      if (pl.BM == 64 && pl.BN == 64) return launch_dma<OP, 64, 64, 32, 3, true>(a, st);
    } else if (pl.bk == 32) {
      if (pl.BM == 128 && pl.BN == 128) return launch_dma<OP, 128, 128, 32, 4, true>(a, st);
      if (pl.BM == 128 && pl.BN == 64) return launch_dma<OP, 128, 64, 32, 4, true>(a, st);
      if (pl.BM == 64 && pl.BN == 128) return launch_dma<OP, 64, 128, 32, 4, true>(a, st);
      if (pl.BM == 64 && pl.BN == 64) return launch_dma<OP, 64, 64, 32, 4, true>(a, st);
    } else {
      if (pl.BM == 128 && pl.BN == 128) return launch_dma<OP, 128, 128, 64, 4, true>(a, st);
      if (pl.BM == 128 && pl.BN == 64) return launch_dma<OP, 128, 64, 64, 4, true>(a, st);
      if (pl.BM == 64 && pl.BN == 128) return launch_dma<OP, 64, 128, 64, 4, true>(a, st);
      if (pl.BM == 64 && pl.BN == 64) return launch_dma<OP, 64, 64, 64, 4, true>(a, st);
    }
    return JZ_ERR_UNSUPPORTED;  // the planner only offers the shapes above in this mode
  }
  if constexpr (OP != OP_BWD_WEIGHT && OP != OP_BWD_DATA_STATS && OP != OP_BWD_DATA_BLOCK_END) {
    if (pl.gen) {  // the planner offers the 4-wavefront 32-deep tiles in this mode
      if (pl.BM == 128 && pl.BN == 128) return launch_dma<OP, 128, 128, 32, 4, false, 2, 2, true>(a, st);
      if (pl.BM == 128 && pl.BN == 64) return launch_dma<OP, 128, 64, 32, 4, false, 2, 2, true>(a, st);
      if (pl.BM == 64 && pl.BN == 128) return launch_dma<OP, 64, 128, 32, 4, false, 2, 2, true>(a, st);
      return launch_dma<OP, 64, 64, 32, 4, false, 2, 2, true>(a, st);
    }
  }
  // large tiles, one workgroup of 8 wavefronts per compute unit with (nearly) the whole LDS as its ring
  if (pl.BM == 256 && pl.BN == 256 && pl.bk == 32) return launch_dma<OP, 256, 256, 32, 4, false, 2, 4>(a, st);  // 2x4 wavefronts of 128x64
  if (pl.BM == 256 && pl.BN == 128 && pl.bk == 64) return launch_dma<OP, 256, 128, 64, 3, false, 4, 2>(a, st);
  if (pl.BM == 128 && pl.BN == 128 && pl.bk == 64 && pl.waves == 8) return launch_dma<OP, 128, 128, 64, 4, false, 4, 2>(a, st);
  if (pl.BM == 256 && pl.BN == 128 && pl.bk == 32 && pl.nst == 3) return launch_dma<OP, 256, 128, 32, 3, false, 4, 2>(a, st);
  if (pl.BM == 256 && pl.BN == 128 && pl.bk == 32) return launch_dma<OP, 256, 128, 32, 4, false, 4, 2>(a, st);  // 4x2 wavefronts of 64x64
  if (pl.BM == 128 && pl.BN == 128 && pl.bk == 32 && pl.waves == 8 && pl.nst == 3) return launch_dma<OP, 128, 128, 32, 3, false, 4, 2>(a, st);
  if (pl.BM == 128 && pl.BN == 128 && pl.bk == 32 && pl.waves == 8) return launch_dma<OP, 128, 128, 32, 4, false, 4, 2>(a, st);
  if (pl.bk == 64) {
    if (pl.BM == 128 && pl.BN == 128) return launch_dma<OP, 128, 128, 64, 4>(a, st);
    if (pl.BM == 128 && pl.BN == 64) return launch_dma<OP, 128, 64, 64, 4>(a, st);
    if (pl.BM == 64 && pl.BN == 128) return launch_dma<OP, 64, 128, 64, 4>(a, st);
    return launch_dma<OP, 64, 64, 64, 4>(a, st);
  }
  if (pl.nst == 3) {
    if (pl.BM == 128 && pl.BN == 128) return launch_dma<OP, 128, 128, 32, 3>(a, st);
    if (pl.BM == 128 && pl.BN == 64) return launch_dma<OP, 128, 64, 32, 3>(a, st);
    if (pl.BM == 64 && pl.BN == 128) return launch_dma<OP, 64, 128, 32, 3>(a, st);
    return launch_dma<OP, 64, 64, 32, 3>(a, st);
  }
  if (pl.BM == 128 && pl.BN == 128) return launch_dma<OP, 128, 128, 32, 4>(a, st);
  if (pl.BM == 128 && pl.BN == 64) return launch_dma<OP, 128, 64, 32, 4>(a, st);
  if (pl.BM == 64 && pl.BN == 128) return launch_dma<OP, 64, 128, 32, 4>(a, st);
  return launch_dma<OP, 64, 64, 32, 4>(a, st);
}

}  // namespace
