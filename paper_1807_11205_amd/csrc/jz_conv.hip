// FP16-storage / FP32-accumulate convolution forward, backward-data, backward-weight and the fully
// connected GEMMs (Jia et al. 2018, Section 4.1) as one implicit-GEMM kernel family for gfx950.
//
// This file holds the host side (planner: tile shape, split of the reduction, which kernel; argument checks; the
// extern "C" entry points), the epilogue shared by all kernels, the small helper kernels (split-K reduction, the
// 4-channel padded copy for 3-channel stems), and the register-staged kernel `igemm_kernel`:
//
//   igemm_kernel<OP, FAST=false>  element-wise, fully bounds-checked operand access.  Runs every shape that allows
//                                 no 16-byte vector access (channel counts that are not multiples of 8 or 32).
//   igemm_kernel<OP, FAST=true>   16-byte loads global -> registers -> LDS, double buffered.  Kept as a second,
//                                 independent implementation for debugging (JZ_IGEMM_PATH=reg); not used otherwise.
//
// The production kernel, igemm_dma_kernel (LDS-direct loads, multi-stage ring), lives in jz_igemm_dma.h.
//
// All kernels: workgroup = 256 threads = 4 wavefronts in a 2x2 grid over a BM x BN output tile; each wavefront owns
// (BM/2) x (BN/2) of it as 32x32 MFMA tiles (v_mfma_f32_32x32x16_f16, fp32 accumulators).  The register-staged kernel
// keeps both tiles in LDS as [row][k] with k contiguous (row pitch BK+8 halves: conflict-free 16-byte accesses);
// operands whose memory layout has the other index contiguous are fetched as 8x8 blocks and transposed in registers.
#include <stdio.h>
#include <stdlib.h>

#include <mutex>
#include <type_traits>
#include <vector>

#include "jz_igemm.h"
#include "jz_internal.h"

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

__device__ __forceinline__ uint4 ldg16(const unsigned short* p) { return *reinterpret_cast<const uint4*>(p); }

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

// 8x8 transpose of halves held as 8 rows of 4 dwords: out[e] gets element e of every row
__device__ __forceinline__ void transpose8x8(const uint4 (&in)[8], uint4 (&out)[8]) {
  const unsigned* s = reinterpret_cast<const unsigned*>(in);
  unsigned* d = reinterpret_cast<unsigned*>(out);
#pragma unroll
  for (int e = 0; e < 8; ++e)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      unsigned lo = s[(2 * j) * 4 + (e >> 1)], hi = s[(2 * j + 1) * 4 + (e >> 1)];
      d[e * 4 + j] = __builtin_amdgcn_perm(hi, lo, (e & 1) ? 0x07060302u : 0x05040100u);
    }
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

template <int BM, int BN, int TM, int TN, int NTHREADS, int EPASS = 1, int LDS_BYTES = 0, bool STATS = false>
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
  // optional per-tile column sums of what is stored (for a batch normalization behind a forward convolution): a thread
  // stores the same 8 columns of every row it handles, so it keeps their sums; they are combined below
  // (a template argument: as a run-time branch in every kernel it cost the step 5 %)
  static_assert(!STATS || LDS_BYTES >= 64 * NTHREADS, "the ring has to hold the partial sums");
  constexpr bool CAN_STATS = STATS;
  constexpr bool stats = STATS;
  float ssum[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}, ssq[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
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
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const unsigned short hb = (unsigned short)(e & 1 ? pw[e >> 1] >> 16 : pw[e >> 1] & 0xffffu);
          _Float16 hv;
          __builtin_memcpy(&hv, &hb, 2);
          const float v = (float)hv;
          ssum[e] += v;
          ssq[e] += v * v;
        }
      }
      size_t drow = (size_t)m;
      if (a.sc_on) {  // row m = (n, p, q) of the strided grid goes to input pixel (n, p * sh, q * sw)
        unsigned nimg = fd_div((unsigned)m, a.g.d_ohow);
        unsigned rem = (unsigned)m - nimg * (unsigned)(a.g.OH * a.g.OW);
        unsigned p = fd_div(rem, a.g.d_ow);
        unsigned q = rem - p * (unsigned)a.g.OW;
        drow = ((size_t)nimg * a.sc_H + p * a.sc_sh) * a.sc_W + q * a.sc_sw;
        // the other pixels of this sh x sw cell are read by no output pixel: their gradient is zero
        for (int i2 = 0; i2 < a.sc_sh; ++i2)
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
template <int OP, bool FAST, int BM, int BN>
__global__ __launch_bounds__(THREADS) void igemm_kernel(GemmArgs a) {
  constexpr int TM = BM / 64, TN = BN / 64;              // 32x32 MFMA tiles per wavefront
  constexpr int A_HALVES = BM * LDK, B_HALVES = BN * LDK;
  constexpr int RPP = LOADERS / KCH;                     // rows one pass of 128 loader threads covers (16)
  constexpr int PA = BM / RPP, PB = BN / RPP;            // passes over the A / B tile
  constexpr int NREG = (PA > PB ? PA : PB) < 8 ? 8 : (PA > PB ? PA : PB);
  extern __shared__ __align__(16) unsigned short lds[];

  const ConvGeom& g = a.g;
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

  // ---- per-thread loader state (FAST paths) -------------------------------------------------
  int st0[NREG], st1[NREG], st2[NREG];
  (void)st0; (void)st1; (void)st2;
  if (FAST) {
    if (loadsA && OP != OP_BWD_WEIGHT) {  // gather rows of the pixel grid
#pragma unroll
      for (int i = 0; i < PA; ++i) {
        int m = m0 + rsub + RPP * i;
        if (m < a.M) {
          unsigned n = fd_div((unsigned)m, g.d_ohow);
          unsigned rem = (unsigned)m - n * (unsigned)(g.OH * g.OW);
          unsigned oh = fd_div(rem, g.d_ow);
          unsigned ow = rem - oh * (unsigned)g.OW;
          if (OP == OP_FWD) {
            st1[i] = (int)oh * g.sh - g.ph;
            st2[i] = (int)ow * g.sw - g.pw;
            st0[i] = (((int)n * g.IH + st1[i]) * g.IW + st2[i]) * g.IC;
          } else {
            st0[i] = (int)n * g.IH * g.IW;
            st1[i] = (int)oh + g.ph;
            st2[i] = (int)ow + g.pw;
          }
        } else {
          st0[i] = 0;
          st1[i] = -(1 << 28);  // fails every bounds check below
          st2[i] = -(1 << 28);
        }
      }
    }
    if (!loadsA && OP == OP_BWD_WEIGHT) {  // this thread's 8 columns (r,s,c..c+7) are fixed
      int nn = n0 + rsub * 8;
      if (nn < a.N) {
        unsigned tap = fd_div((unsigned)nn, g.d_ic);
        unsigned r = fd_div(tap, g.d_s);
        st0[0] = nn - (int)tap * g.IC;         // c0
        st1[0] = (int)r - g.ph;                // ih = p*sh + st1
        st2[0] = (int)(tap - r * g.S) - g.pw;  // iw = q*sw + st2
      } else {
        st0[0] = 0;
        st1[0] = -(1 << 28);
        st2[0] = -(1 << 28);
      }
    }
  }

  uint4 rg[NREG];
  const uint4 zero4 = make_uint4(0, 0, 0, 0);

  // fetch k tile `kt` of this thread's operand into rg[]
  auto fetch = [&](int kt) {
    const int k0 = kt * BK;
    if (!FAST) {
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
      return;
    }
    if (OP != OP_BWD_WEIGHT) {
      // the whole k tile lies inside one filter tap (IC % BK == 0): tap arithmetic is wave-uniform
      const unsigned tap = fd_div((unsigned)k0, g.d_ic);
      const int c0 = k0 - (int)tap * g.IC;
      const int r = (int)fd_div(tap, g.d_s);
      const int s = (int)tap - r * g.S;
      if (loadsA) {
#pragma unroll
        for (int i = 0; i < PA; ++i) {
          bool ok;
          int off;
          if (OP == OP_FWD) {
            int ih = st1[i] + r, iw = st2[i] + s;
            ok = (unsigned)ih < (unsigned)g.IH && (unsigned)iw < (unsigned)g.IW;
            off = st0[i] + (r * g.IW + s) * g.IC + c0 + kc * 8;
          } else {
            int th = st1[i] - r, tw = st2[i] - s;
            int ih = th, iw = tw;
            ok = th >= 0 && tw >= 0;
            if (g.sh != 1 || g.sw != 1) {
              ih = (int)fd_div((unsigned)(th < 0 ? 0 : th), g.d_sh);
              iw = (int)fd_div((unsigned)(tw < 0 ? 0 : tw), g.d_sw);
              ok = ok && ih * g.sh == th && iw * g.sw == tw;
            }
            ok = ok && ih < g.IH && iw < g.IW;
            off = (st0[i] + ih * g.IW + iw) * g.IC + c0 + kc * 8;
          }
          rg[i] = ok ? ldg16(a.A + off) : zero4;
        }
      } else if (OP == OP_FWD) {  // filter rows, k contiguous
#pragma unroll
        for (int i = 0; i < PB; ++i) {
          int nn = n0 + rsub + RPP * i;
          rg[i] = nn < a.N ? ldg16(a.B + (size_t)nn * a.Kred + k0 + kc * 8) : zero4;
        }
      } else {  // BWD_DATA filter: B(c, (tap,ko)) = w[ko][tap][c]; 8 ko rows x 8 c, transposed later
        int nn = n0 + rsub * 8;
        bool ok = rsub * 8 < BN && nn < a.N;
        int RS = g.R * g.S;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          int ko = c0 + kc * 8 + i;
          rg[i] = ok ? ldg16(a.B + ((size_t)ko * RS + tap) * a.N + nn) : zero4;
        }
      }
    } else {
      if (loadsA) {  // dy[(n,p,q)][k_out]: 8 reduction rows x 8 k_out
        int mm = m0 + rsub * 8;
        bool okm = rsub * 8 < BM && mm < a.M;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          int j = k0 + kc * 8 + i;
          rg[i] = (okm && j < a.Kred) ? ldg16(a.A + (size_t)j * a.M + mm) : zero4;
        }
      } else {  // x gathered at this thread's tap for 8 consecutive output pixels
        bool okn = rsub * 8 < BN;
        int j = k0 + kc * 8;
        unsigned n = fd_div((unsigned)j, g.d_ohow);
        unsigned rem = (unsigned)j - n * (unsigned)(g.OH * g.OW);
        int p = (int)fd_div(rem, g.d_ow);
        int q = (int)rem - p * g.OW;
        int nb = (int)n;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          int ih = p * g.sh + st1[0], iw = q * g.sw + st2[0];
          bool ok = okn && (j + i) < a.Kred && (unsigned)ih < (unsigned)g.IH && (unsigned)iw < (unsigned)g.IW;
          rg[i] = ok ? ldg16(a.B + ((size_t)(nb * g.IH + ih) * g.IW + iw) * g.IC + st0[0]) : zero4;
          if (++q == g.OW) {
            q = 0;
            if (++p == g.OH) { p = 0; ++nb; }
          }
        }
      }
    }
  };

  // put rg[] into LDS buffer `buf`
  auto stash = [&](int buf) {
    unsigned short* base = lds + buf * (A_HALVES + B_HALVES) + (loadsA ? 0 : A_HALVES);
    const bool transposed = FAST && ((OP == OP_BWD_WEIGHT) || (OP == OP_BWD_DATA && !loadsA));
    if (!transposed) {
      const int rows = loadsA ? PA : PB;
#pragma unroll
      for (int i = 0; i < NREG; ++i)
        if (i < rows) *reinterpret_cast<uint4*>(base + (rsub + RPP * i) * LDK + kc * 8) = rg[i];
    } else {
      const int rows = loadsA ? BM : BN;
      if (rsub * 8 < rows) {
        uint4 in[8], out[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) in[i] = rg[i];
        transpose8x8(in, out);
#pragma unroll
        for (int e = 0; e < 8; ++e) *reinterpret_cast<uint4*>(base + (rsub * 8 + e) * LDK + kc * 8) = out[e];
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

// ---------------------------------------------------------------------------------------------
// small-channel layers (C <= 4: the 3-channel stems of ResNet-50 and AlexNet)
// ---------------------------------------------------------------------------------------------
// With 3 channels a filter tap is 6 bytes: nothing to vectorise.  But in NHWC the S taps of one filter row are
// adjacent in memory, so the input is copied once into a zero-padded 4-channel image xp[N][H+2ph][Wp][4]; one filter
// row of an output pixel is then ONE contiguous, 16-byte aligned run of 4*S halves starting at pixel q*stride_w
// (needs an even stride_w), and the layer becomes an ordinary implicit GEMM whose "taps" are the R filter rows and
// whose "channels" are that run, rounded up to the k tile (32 or 64).  The filter is repacked to match
// (w'[k][r][4 s + c], zeros elsewhere); for backward-weight the GEMM produces dw' in that layout and the real
// entries are copied out.

// One launch does both copies.  Slices z < N of the grid: a workgroup of 128 threads covers 256 padded pixels of image
// row (z, y), two per thread (one 16-byte store; Wp is even).  Slice z = N (present when wp != nullptr) repacks the
// filter: w[K][R][S][C] -> wp[K][R][KT] with wp[k][r][4 s + c] = w[k][r][s][c], zero elsewhere.
__global__ __launch_bounds__(128) void pad_to_c4(const unsigned short* __restrict__ x, unsigned short* __restrict__ xp,
                                                 int N, int H, int W, int C, int Hp, int Wp, int ph, int pw,
                                                 const unsigned short* __restrict__ w, unsigned short* __restrict__ wp,
                                                 int K, int R, int S, int KT) {
  const int z = blockIdx.z;
  if (z == N) {
    const int total = K * R * KT;
    const int stride = gridDim.x * gridDim.y * 128;
    for (int i = (blockIdx.y * gridDim.x + blockIdx.x) * 128 + threadIdx.x; i < total; i += stride) {
      int j = i % KT, kr = i / KT;
      int s = j >> 2, c = j & 3;
      wp[i] = (s < S && c < C) ? w[((size_t)kr * S + s) * C + c] : (unsigned short)0;
    }
    return;
  }
  const int hp = blockIdx.y;
  const int wp0 = 2 * (blockIdx.x * 128 + threadIdx.x);
  if (wp0 >= Wp) return;
  const int h = hp - ph;
  unsigned short v[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if ((unsigned)h < (unsigned)H) {
    const unsigned short* row = x + ((size_t)z * H + h) * W * C;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      const int wi = wp0 + p - pw;
      if ((unsigned)wi < (unsigned)W) {
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if (c < C) v[4 * p + c] = row[(size_t)wi * C + c];
      }
    }
  }
  uint4 pk = make_uint4((unsigned)v[0] | ((unsigned)v[1] << 16), (unsigned)v[2] | ((unsigned)v[3] << 16),
                        (unsigned)v[4] | ((unsigned)v[5] << 16), (unsigned)v[6] | ((unsigned)v[7] << 16));
  *reinterpret_cast<uint4*>(xp + (((size_t)z * Hp + hp) * Wp + wp0) * 4) = pk;
}

// dwp[K][R][KT] -> dw[K][R][S][C]
__global__ __launch_bounds__(256) void unpack_filter_c4(const unsigned short* __restrict__ dwp, unsigned short* __restrict__ dw,
                                                        int K, int R, int S, int C, int KT) {
  int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= K * R * S * C) return;
  int c = i % C, t = i / C;
  int s = t % S, kr = t / S;
  dw[i] = dwp[(size_t)kr * KT + 4 * s + c];
}

// D16[i] = RNE16( sum_s part[s][i] ).  A workgroup owns 256 / G groups of four consecutive outputs and G = 2^lg
// "split lanes": lane g adds splits g, g + G, g + 2G, ... in that order, then the G lane sums are added in lane order.
// The order depends only on (splits, G), so the result is deterministic.  Splitting the reduction over lanes matters
// for the small outputs that need many splits: with one thread per output group those launches were latency-bound.
// KT4 > 0 (small-channel backward-weight): the sums are dw'[K][R][4 KT4] of the padded 4-channel problem; group
// (kr, s) of four goes to dw[kr][s][0..C) when s < S and nowhere otherwise, which saves the separate unpacking launch.
__global__ __launch_bounds__(256) void splitk_reduce(const float* __restrict__ part, unsigned short* __restrict__ out,
                                                     long long MN, int splits, int lg, int KT4, int S, int C) {
  __shared__ float4 red[256];
  const int G = 1 << lg, Q = 256 >> lg;
  const int q = threadIdx.x & (Q - 1), g = threadIdx.x >> (8 - lg);
  const long long i = ((long long)blockIdx.x * Q + q) * 4;
  const bool full = i + 3 < MN;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  if (i < MN) {
    if (full) {
      int k = g;
      for (; k + 3 * G < splits; k += 4 * G) {  // four loads in flight per thread
        float4 t0 = *reinterpret_cast<const float4*>(part + (size_t)k * MN + i);
        float4 t1 = *reinterpret_cast<const float4*>(part + (size_t)(k + G) * MN + i);
        float4 t2 = *reinterpret_cast<const float4*>(part + (size_t)(k + 2 * G) * MN + i);
        float4 t3 = *reinterpret_cast<const float4*>(part + (size_t)(k + 3 * G) * MN + i);
        s.x += t0.x; s.y += t0.y; s.z += t0.z; s.w += t0.w;
        s.x += t1.x; s.y += t1.y; s.z += t1.z; s.w += t1.w;
        s.x += t2.x; s.y += t2.y; s.z += t2.z; s.w += t2.w;
        s.x += t3.x; s.y += t3.y; s.z += t3.z; s.w += t3.w;
      }
      for (; k < splits; k += G) {
        float4 t = *reinterpret_cast<const float4*>(part + (size_t)k * MN + i);
        s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
      }
    } else {  // ragged end of the matrix: element-wise
      float* sv = reinterpret_cast<float*>(&s);
      for (int k = g; k < splits; k += G)
        for (int e = 0; e < 4 && i + e < MN; ++e) sv[e] += part[(size_t)k * MN + i + e];
    }
  }
  if (G > 1) {
    red[threadIdx.x] = s;
    __syncthreads();
    if (g != 0) return;
    for (int gg = 1; gg < G; ++gg) {
      float4 t = red[gg * Q + q];
      s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
    }
  }
  if (i >= MN) return;
  _Float16 h[4] = {(_Float16)s.x, (_Float16)s.y, (_Float16)s.z, (_Float16)s.w};
  if (KT4 > 0) {  // MN is a multiple of 4 here
    const long long grp = i >> 2, kr = grp / KT4;
    const int sx = (int)(grp - kr * KT4);
    if (sx < S) {
#pragma unroll
      for (int c = 0; c < 4; ++c)
        if (c < C) {
          unsigned short bts;
          __builtin_memcpy(&bts, &h[c], 2);
          out[(kr * S + sx) * C + c] = bts;
        }
    }
    return;
  }
  if (full) {
    uint2 pk;
    __builtin_memcpy(&pk, h, 8);
    *reinterpret_cast<uint2*>(out + i) = pk;
  } else {
    for (int e = 0; e < 4 && i + e < MN; ++e) {
      unsigned short bts;
      __builtin_memcpy(&bts, &h[e], 2);
      out[i + e] = bts;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// host side: plan (tile shape, fast/generic, split-K) and launch
// ---------------------------------------------------------------------------------------------
bool use_register_path() {  // debugging aid: JZ_IGEMM_PATH=reg selects the register-staged vector kernels (read per call)
  const char* e = getenv("JZ_IGEMM_PATH");
  return e && e[0] == 'r';
}
int env_int(const char* name) {
  const char* e = getenv(name);
  return e ? atoi(e) : 0;
}
// debugging aids: JZ_IGEMM_BK=64, JZ_IGEMM_TILE=<BM*1000+BN>, JZ_IGEMM_SPLITS=<n>, JZ_IGEMM_WAVES=<4|8>, JZ_IGEMM_NST=<ring depth> override the
// planner, JZ_IGEMM_NOTABLE=1 skips the table of measured choices, JZ_IGEMM_VERBOSE=1 prints the choice (read once per call, not per candidate: the environment is searched
// linearly, and a tuning sweep may change them inside one process)
struct Overrides {
  int bk, tile, splits, waves, verbose, notable, nst;
};
Overrides read_overrides() {
  return Overrides{env_int("JZ_IGEMM_BK"), env_int("JZ_IGEMM_TILE"), env_int("JZ_IGEMM_SPLITS"), env_int("JZ_IGEMM_WAVES"),
                   env_int("JZ_IGEMM_VERBOSE"), env_int("JZ_IGEMM_NOTABLE"), env_int("JZ_IGEMM_NST")};
}

struct Plan {
  int op = 0;
  bool fast = false;    // vector (16-byte) operand access possible
  bool packed = false;  // small-channel layer run on a 4-channel padded copy
  bool gen = false;     // gather with per-load tap arithmetic (more than 32 taps, strided multi-tap backward-data)
  int BM = 128, BN = 128;
  int bk = BK;  // k tile depth of the kernel that will run
  int waves = 4, nst = 4;  // wavefronts per workgroup and ring depth (large tiles come in several variants)
  GemmArgs args{};
  size_t ws_bytes = 0;       // total workspace
  size_t part_offset = 0;    // where the split-K partial sums start inside it
  size_t bytesA = 0, bytesB = 0, bytesD = 0;  // caller's operand sizes in bytes, for the overlap checks
  // packed mode
  int Hp = 0, Wp = 0, KT = 0;
  size_t xp_bytes = 0, wp_bytes = 0;
};

int out_dim(int in, int pad, int f, int st) { return (in + 2 * pad - f) / st + 1; }
size_t up256(size_t x) { return (x + 255) & ~size_t(255); }

// Pick the kernel variant (output tile, k tile depth, wavefronts per workgroup) and the split of the reduction with a
// small cost model, in microseconds:
//   time = fixed + rounds of resident workgroups * k tiles per workgroup * time per k tile of that variant
//          + (split > 1: writing and re-reading the fp32 partial sums, plus one more launch)
// The per-k-tile constants are least-squares fits to timings of the ResNet-50 layer shapes at batch 64 with cold
// caches; the fixed part is kept the same for all variants (per-variant fits of it were noise and chose worse).  The
// 4-wavefront variants run two workgroups per compute unit (512 resident), the 8-wavefront ones a single workgroup
// that owns the whole LDS (256 resident); the latter win when the grid cannot fill 512 slots anyway.
struct Variant {
  int BM, BN, bk, waves, resident;
  double tt[3];  // per k tile: forward, backward-data, backward-weight
  double c0[3];  // fixed part
  int nst;       // ring depth
};
const Variant kVariants[] = {
    {128, 128, 32, 4, 512, {0.306, 0.284, 0.415}, {8.3, 10.3, 8.0}, 4},
    {128, 64, 32, 4, 512, {0.243, 0.220, 0.307}, {8.3, 10.3, 8.0}, 4},
    {64, 128, 32, 4, 512, {0.246, 0.214, 0.336}, {8.3, 10.3, 8.0}, 4},
    {64, 64, 32, 4, 512, {0.202, 0.179, 0.272}, {8.3, 10.3, 8.0}, 4},
    {128, 128, 64, 8, 256, {0.441, 0.433, 0.534}, {8.3, 10.3, 8.0}, 4},
    {256, 128, 64, 8, 256, {0.664, 0.649, 0.822}, {8.3, 10.3, 8.0}, 3},
    {256, 128, 32, 8, 256, {0.380, 0.363, 0.415}, {8.3, 10.3, 8.0}, 4},
    {256, 256, 32, 8, 256, {0.623, 0.597, 0.824}, {8.3, 10.3, 8.0}, 4},
    {128, 128, 64, 4, 256, {0.501, 0.526, 0.721}, {8.3, 10.3, 8.0}, 4},
    {128, 64, 64, 4, 256, {0.395, 0.393, 0.463}, {8.3, 10.3, 8.0}, 4},
    {64, 128, 64, 4, 256, {0.378, 0.428, 0.583}, {8.3, 10.3, 8.0}, 4},
    {64, 64, 64, 4, 512, {0.374, 0.381, 0.374}, {8.3, 10.3, 8.0}, 4},
    // three-stage rings for the 4-wavefront 32-deep tiles: 48 / 36 / 24 KB of LDS, three to six workgroups per compute
    // unit, for layers whose reduction is only a few k tiles long (a workgroup's prologue and epilogue then overlap
    // with the loops of more neighbours)
    {128, 128, 32, 4, 768, {0.306, 0.284, 0.415}, {8.3, 10.3, 8.0}, 3},
    {128, 64, 32, 4, 1024, {0.243, 0.220, 0.307}, {8.3, 10.3, 8.0}, 3},
    {64, 128, 32, 4, 1024, {0.246, 0.214, 0.336}, {8.3, 10.3, 8.0}, 3},
    {64, 64, 32, 4, 1536, {0.202, 0.179, 0.272}, {8.3, 10.3, 8.0}, 3},
    // 8 wavefronts and two or three workgroups per compute unit (32-deep tiles, 72 / 64 / 48 KB of LDS): the neighbour
    // works while one workgroup waits at its barrier
    {256, 128, 32, 8, 512, {0.380, 0.363, 0.415}, {8.3, 10.3, 8.0}, 3},
    {128, 128, 32, 8, 512, {0.306, 0.284, 0.415}, {8.3, 10.3, 8.0}, 4},
    {128, 128, 32, 8, 768, {0.306, 0.284, 0.415}, {8.3, 10.3, 8.0}, 3},
};

// Measured choices for known GEMM shapes (written by `python -m paper_1807_11205_amd.tune --write`): the per-k-tile model
// below ranks variants that differ by a few percent poorly, a table of cold-cache timings does not.
struct Tuned {
  int op, M, N, K, taps, scatter, BM, BN, bk, waves, nst, splits;
};
const Tuned kTuned[] = {
#include "jz_tuned.inc"
#include "jz_tuned_alexnet.inc"
#include "jz_tuned_resnet50_n128.inc"
#include "jz_tuned_resnet50_n256.inc"
#include "jz_tuned_resnet50_n32.inc"
    // the 3-channel stem of ResNet-50 at batch 64 on its padded 4-channel copy ("taps" = the 7 filter rows), measured
    // the same way: forward 62.8 us, backward-weight 67.0 us including the copy
    {0, 802816, 64, 224, 7, 0, 128, 64, 32, 4, 3, 1},
    {2, 64, 224, 802816, 7, 0, 64, 64, 32, 4, 4, 256},
};

// Choices set at run time through jz_conv2d_tune_set: looked up before the table above (an in-place tuning run tries
// candidates this way without rebuilding the library).
std::mutex g_tune_mutex;
std::vector<Tuned> g_tune_rt;

bool same_key(const Tuned& x, const Tuned& y) {
  return x.op == y.op && x.M == y.M && x.N == y.N && x.K == y.K && x.taps == y.taps && x.scatter == y.scatter;
}

// bk64_ok: the 64-deep k tile is usable for this layer; forced_bk: the k tile depth is fixed (register path, packed mode)
void choose_tiling(Plan* pl, bool bk64_ok, int forced_bk, const Overrides& ov) {
  GemmArgs& a = pl->args;
  static const int split_opts[] = {1, 2, 3, 4, 6, 8, 12, 16, 24, 32, 48, 64, 96, 128, 192, 256, 384, 512};
  const int oi = pl->op == JZ_FWD ? 0 : pl->op == JZ_BWD_DATA ? 1 : 2;
  double best = 1e30;
  const Variant* bv = &kVariants[0];
  int bS = 1;
  if (!pl->fast) forced_bk = BK;  // the element-wise kernel: one shape (the first variant's), 64-deep tiles, ~8x slower
  const Tuned* hit = nullptr;
  Tuned rt_hit{};
  if (pl->fast && !pl->gen && (!forced_bk || pl->packed) && !ov.bk && !ov.tile && !ov.splits && !ov.waves && !ov.nst && !ov.notable) {
    const Tuned key{oi, a.M, a.N, a.Kred, a.g.R * a.g.S, a.sc_on, 0, 0, 0, 0, 0, 0};
    auto usable = [&](const Tuned& t) { return same_key(t, key) && (forced_bk ? t.bk == forced_bk : (t.bk == 32 || bk64_ok)); };
    {
      std::lock_guard<std::mutex> lock(g_tune_mutex);
      for (const Tuned& t : g_tune_rt)
        if (usable(t)) {
          rt_hit = t;
          hit = &rt_hit;
          break;
        }
    }
    if (!hit)
      for (const Tuned& t : kTuned)
        if (usable(t)) {
          hit = &t;
          break;
        }
  }
  if (hit) {
    pl->BM = hit->BM; pl->BN = hit->BN; pl->bk = hit->bk; pl->waves = hit->waves;
    pl->nst = hit->nst;
    bS = hit->splits;
    const int nkt_h = (a.Kred + hit->bk - 1) / hit->bk;
    if (bS > 1 && (nkt_h / bS < 4 || a.sc_on)) bS = 1;  // the same admissibility rules as the search below
  } else {
    for (const Variant& v : kVariants) {
      if (!pl->fast && &v != &kVariants[0]) break;
      if ((forced_bk || pl->gen) && (v.waves != 4 || v.bk != 32)) continue;  // those kernels exist as 4-wavefront variants only
      if (!forced_bk && v.bk == 64 && !bk64_ok) continue;
      if (!forced_bk && ov.bk && ov.bk != v.bk) continue;
      if (ov.tile && ov.tile != v.BM * 1000 + v.BN) continue;
      if (ov.waves && ov.waves != v.waves) continue;
      if (ov.nst && ov.nst != v.nst) continue;
      if (v.nst == 3 && v.bk == 32 && ov.nst != 3) continue;  // short rings: from the table of measured choices or on request
      if (v.waves == 8 && v.BM == 128 && v.bk == 32 && ov.waves != 8) continue;  // likewise (the model has no fit for it)
      const int vbk = forced_bk ? forced_bk : v.bk;
      if (v.nst == 3 && vbk != 32) continue;  // the short rings exist for 32-deep tiles
      const int nkt = (a.Kred + vbk - 1) / vbk;
      long long tm = (a.M + v.BM - 1) / v.BM, tn = (a.N + v.BN - 1) / v.BN;
      for (int sp : split_opts) {
        if (sp > 1 && nkt / sp < 4) break;
        if (a.sc_on && sp > 1) break;  // the scatter lives in the fp16 epilogue
        if (ov.splits && sp != ov.splits && !(sp == 1 && nkt / ov.splits < 4)) continue;
        const int kps = (nkt + sp - 1) / sp;
        long long blocks = tm * tn * ((nkt + kps - 1) / kps);
        long long rounds = (blocks + v.resident - 1) / v.resident;
        double t = v.c0[oi] + rounds * kps * v.tt[oi] * (vbk / (double)v.bk) * (pl->fast ? 1.0 : 8.0);
        if (sp > 1) t += 0.185 * (2.0 * sp * (double)a.M * a.N * 4.0) / 1.0e6 + 1.8;
        if (t < best) { best = t; bv = &v; bS = sp; }
      }
    }
    if (best == 1e30) bv = &kVariants[0];  // contradictory overrides: fall back to the default variant
    pl->BM = bv->BM; pl->BN = bv->BN;
    pl->bk = forced_bk ? forced_bk : bv->bk;
    pl->waves = bv->waves;
    pl->nst = bv->nst;
  }
  a.nkt = (a.Kred + pl->bk - 1) / pl->bk;
  a.tiles_m = (a.M + pl->BM - 1) / pl->BM;
  a.tiles_n = (a.N + pl->BN - 1) / pl->BN;
  a.kt_per_split = (a.nkt + bS - 1) / bS;
  a.splits = (a.nkt + a.kt_per_split - 1) / a.kt_per_split;  // drop empty splits
  a.d_tiles_mn = make_fastdiv((unsigned)(a.tiles_m * a.tiles_n));
  a.d_tiles_n = make_fastdiv((unsigned)a.tiles_n);
}

void finish_geometry(ConvGeom& g) {
  g.tap_rep = 0;
  if (g.R * g.S <= 32)
    for (int r = 0; r < g.R; ++r) g.tap_rep |= 1u << (r * g.S);
  g.d_ohow = make_fastdiv((unsigned)(g.OH * g.OW));
  g.d_ow = make_fastdiv((unsigned)g.OW);
  g.d_ic = make_fastdiv((unsigned)g.IC);
  g.d_s = make_fastdiv((unsigned)g.S);
  g.d_sh = make_fastdiv((unsigned)g.sh);
  g.d_sw = make_fastdiv((unsigned)g.sw);
}

void plan_text(const Plan& pl, char* buf, size_t n) {
  const GemmArgs& a = pl.args;
  snprintf(buf, n, "op %d M %d N %d K %d: %s tile %dx%dx%d, %d wavefronts, ring %d, %d x %d tiles, %d splits of %d k tiles%s%s", pl.op, a.M,
           a.N, a.Kred, pl.fast ? "vector" : "element-wise", pl.BM, pl.BN, pl.bk, pl.fast ? pl.waves : 4,
           pl.fast ? pl.nst : 2, a.tiles_m, a.tiles_n,
           a.splits, a.kt_per_split, pl.packed ? ", 4-channel padded copy" : "",
           a.sc_on ? ", scatter epilogue" : pl.gen ? ", per-load tap arithmetic" : "");
}

int make_plan(int op, const jz_conv_desc* d, Plan* pl) {
  if (!d) return JZ_ERR_NULL;
  if (op != JZ_FWD && op != JZ_BWD_DATA && op != JZ_BWD_WEIGHT) return JZ_ERR_UNSUPPORTED;
  if (d->N <= 0 || d->H <= 0 || d->W <= 0 || d->C <= 0 || d->K <= 0 || d->R <= 0 || d->S <= 0 || d->stride_h <= 0 ||
      d->stride_w <= 0 || d->pad_h < 0 || d->pad_w < 0)
    return JZ_ERR_SHAPE;
  if (d->pad_h >= d->R || d->pad_w >= d->S) return JZ_ERR_SHAPE;
  if (d->H + 2 * d->pad_h < d->R || d->W + 2 * d->pad_w < d->S) return JZ_ERR_SHAPE;
  const int P = out_dim(d->H, d->pad_h, d->R, d->stride_h), Q = out_dim(d->W, d->pad_w, d->S, d->stride_w);
  if (P <= 0 || Q <= 0) return JZ_ERR_SHAPE;
  const long long lim = (1ll << 31) - 1;  // byte offsets are formed in unsigned 32-bit integers
  const long long nx = (long long)d->N * d->H * d->W * d->C, ny = (long long)d->N * P * Q * d->K,
                  nw = (long long)d->K * d->R * d->S * d->C;
  if (nx > lim || ny > lim || nw > lim) return JZ_ERR_UNSUPPORTED;
  if ((long long)d->N * P * Q > lim / 2 || (long long)d->N * d->H * d->W > lim / 2) return JZ_ERR_UNSUPPORTED;

  GemmArgs& a = pl->args;
  ConvGeom& g = a.g;
  pl->op = op;
  // k tile depth: 32 lets two workgroups share a compute unit (64 KB ring each), which hides one workgroup's
  // barrier and LDS-latency bubbles behind the other's MFMAs
  // k tile depth for the applicability checks: the register path walks 64-deep tiles; the LDS-direct kernels come
  // 32 and 64 deep (chosen by the planner when the layer allows both)
  int bk = use_register_path() ? 64 : 32;
  bool bk64_ok = true;
  int forced_bk = use_register_path() ? 64 : 0;
  g.R = d->R; g.S = d->S; g.sh = d->stride_h; g.sw = d->stride_w; g.ph = d->pad_h; g.pw = d->pad_w;
  g.kvalid = 0;
  // a single filter tap: the reduction is one contiguous channel run, whose ragged last k tile the vector kernel can mask
  const bool one_tap = d->R == 1 && d->S == 1 && !use_register_path();
  if (op == JZ_FWD) {
    a.M = d->N * P * Q; a.N = d->K; a.Kred = d->R * d->S * d->C;
    g.IH = d->H; g.IW = d->W; g.IC = d->C; g.OH = P; g.OW = Q;
    pl->fast = d->C % bk == 0 || (one_tap && d->C % 8 == 0);
    bk64_ok = d->C % 64 == 0 || (one_tap && d->C % 8 == 0);
    pl->bytesA = 2 * nx; pl->bytesB = 2 * nw; pl->bytesD = 2 * ny;
  } else if (op == JZ_BWD_DATA) {
    a.M = d->N * d->H * d->W; a.N = d->C; a.Kred = d->R * d->S * d->K;
    g.IH = P; g.IW = Q; g.IC = d->K; g.OH = d->H; g.OW = d->W;
    pl->fast = (d->K % bk == 0 || (one_tap && d->K % 8 == 0)) && d->C % 8 == 0;
    bk64_ok = d->K % 64 == 0 || (one_tap && d->K % 8 == 0);
    pl->bytesA = 2 * ny; pl->bytesB = 2 * nw; pl->bytesD = 2 * nx;
  } else {
    a.M = d->K; a.N = d->R * d->S * d->C; a.Kred = d->N * P * Q;
    g.IH = d->H; g.IW = d->W; g.IC = d->C; g.OH = P; g.OW = Q;
    pl->fast = d->K % 8 == 0 && d->C % 8 == 0;
    pl->bytesA = 2 * ny; pl->bytesB = 2 * nx; pl->bytesD = 2 * nw;  // A = dy, B = x
  }
  a.sc_on = 0; a.sc_H = a.sc_W = 0; a.sc_sh = a.sc_sw = 1;
  a.bw_linear = (op == JZ_BWD_WEIGHT && d->R == 1 && d->S == 1 && d->stride_h == 1 && d->stride_w == 1 && d->pad_h == 0 &&
                 d->pad_w == 0) ? 1 : 0;
  if (op == JZ_BWD_DATA && pl->fast && !use_register_path() && d->R == 1 && d->S == 1 && d->pad_h == 0 && d->pad_w == 0 &&
      (d->stride_h > 1 || d->stride_w > 1)) {
    // strided 1x1 layer (the ResNet downsampling convs): only input pixels (p*sh, q*sw) receive gradient, so the GEMM
    // runs over the N*P*Q output pixels as a stride-1 problem and the epilogue scatters its rows (and the zeros)
    a.M = d->N * P * Q;
    g.OH = P; g.OW = Q; g.sh = 1; g.sw = 1;
    a.sc_on = 1; a.sc_H = d->H; a.sc_W = d->W; a.sc_sh = d->stride_h; a.sc_sw = d->stride_w;
  }
  g.row_pitch = g.IW * g.IC;
  g.pix_step = g.IC;
  g.s_step = g.IC;

  // small-channel layers: gather from a zero-padded 4-channel copy (see pad_to_c4)
  if (!pl->fast && !use_register_path() && op != JZ_BWD_DATA && d->C <= 4 && d->stride_w % 2 == 0 && 4 * d->S <= 64 &&
      d->R <= 32 && (op == JZ_FWD || d->K % 8 == 0)) {
    const int KT = 4 * d->S <= 32 ? 32 : 64;
    int Hp = d->H + 2 * d->pad_h, Wp = d->W + 2 * d->pad_w;
    if (Wp < (Q - 1) * d->stride_w + KT / 4) Wp = (Q - 1) * d->stride_w + KT / 4;
    Wp = (Wp + 1) & ~1;  // rows stay 16-byte aligned
    const long long nxp = (long long)d->N * Hp * Wp * 4;
    if (nxp <= lim && Hp <= 65535 && d->N < 65535) {  // the copy kernel's grid is (columns, Hp, N + 1)
      pl->packed = true;
      pl->fast = true;
      pl->Hp = Hp; pl->Wp = Wp; pl->KT = KT;
      pl->xp_bytes = up256((size_t)nxp * 2);
      pl->wp_bytes = up256((size_t)d->K * d->R * KT * 2);
      g.IH = Hp; g.IW = Wp; g.IC = KT; g.S = 1; g.ph = 0; g.pw = 0;
      g.row_pitch = Wp * 4; g.pix_step = 4; g.s_step = 0;
      if (op == JZ_FWD) {
        a.Kred = d->R * KT;
        g.kvalid = 4 * d->S;
        bk = KT;
        forced_bk = KT;
      } else {
        a.N = d->R * KT;
      }
    }
  }
  // the vector kernel marks padding taps with a 32-bit mask per row and, for backward-data, needs the source pixel to
  // be an affine function of the tap (unit stride); other shapes take its variant with per-load tap arithmetic
  pl->gen = pl->fast && !pl->packed && op != JZ_BWD_WEIGHT &&
            (g.R * g.S > 32 || (op == JZ_BWD_DATA && (g.sh != 1 || g.sw != 1)));
  finish_geometry(g);
  if (!pl->fast) bk = BK;  // the element-wise kernel walks 64-deep tiles
  pl->bk = bk;
  if (pl->packed && !forced_bk) forced_bk = 32;  // small-channel backward-weight: 4-wavefront 32-deep kernels
  const Overrides ov = read_overrides();
  choose_tiling(pl, bk64_ok, forced_bk, ov);
  const size_t part = a.splits > 1 ? (size_t)a.splits * a.M * a.N * sizeof(float) : 0;
  pl->part_offset = pl->packed ? pl->xp_bytes + pl->wp_bytes : 0;
  pl->ws_bytes = pl->part_offset + part;
  if (ov.verbose) {  // debugging aid: show what the planner chose
    char line[256];
    plan_text(*pl, line, sizeof line);
    fprintf(stderr, "jz igemm %s\n", line);
  }
  return JZ_OK;
}

template <int OP, bool FAST, int BM, int BN>
int launch_one(const GemmArgs& a, hipStream_t st) {
  constexpr size_t tile_bytes = 2 * (size_t)(BM + BN) * LDK * sizeof(unsigned short);
  constexpr size_t epi_bytes = (size_t)BM * (BN + 8) * sizeof(unsigned short);
  constexpr size_t smem = tile_bytes > epi_bytes ? tile_bytes : epi_bytes;
  static bool attr_set = false;  // per instantiation; setting it twice is harmless
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&igemm_kernel<OP, FAST, BM, BN>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
      return JZ_ERR_LAUNCH;
    attr_set = true;
  }
  unsigned grid = (unsigned)a.tiles_m * (unsigned)a.tiles_n * (unsigned)a.splits;
  hipLaunchKernelGGL((igemm_kernel<OP, FAST, BM, BN>), dim3(grid), dim3(THREADS), smem, st, a);
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
    if (!pl.fast || use_register_path()) return JZ_ERR_UNSUPPORTED;  // only the ring kernels come in this form
  } else {
    if (!pl.fast) return launch_one<OP, false, 128, 128>(a, st);
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
  if constexpr (OP != OP_BWD_WEIGHT) {
    if (pl.gen && !use_register_path()) {  // the planner offers the 4-wavefront 32-deep tiles in this mode
      if (pl.BM == 128 && pl.BN == 128) return launch_dma<OP, 128, 128, 32, 4, false, 2, 2, true>(a, st);
      if (pl.BM == 128 && pl.BN == 64) return launch_dma<OP, 128, 64, 32, 4, false, 2, 2, true>(a, st);
      if (pl.BM == 64 && pl.BN == 128) return launch_dma<OP, 64, 128, 32, 4, false, 2, 2, true>(a, st);
      return launch_dma<OP, 64, 64, 32, 4, false, 2, 2, true>(a, st);
    }
  }
  if (!use_register_path()) {
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
  if constexpr (OP == OP_FWD_STATS) {
    return JZ_ERR_UNSUPPORTED;
  } else {
    if (pl.BM == 128 && pl.BN == 128) return launch_one<OP, true, 128, 128>(a, st);
    if (pl.BM == 128 && pl.BN == 64) return launch_one<OP, true, 128, 64>(a, st);
    if (pl.BM == 64 && pl.BN == 128) return launch_one<OP, true, 64, 128>(a, st);
    return launch_one<OP, true, 64, 64>(a, st);
  }
}

// a forward plan whose kernel can leave the per-tile column sums: the ring kernels (their LDS holds the sums), no split
bool plan_leaves_stats(const Plan& pl) {
  return pl.op == JZ_FWD && pl.fast && !use_register_path() && pl.args.splits == 1;
}

// A, B in the kernel's order: FWD (x, w), BWD_DATA (dy, w), BWD_WEIGHT (dy, x)
int run(int op, const jz_conv_desc* d, const void* A, const void* B, void* D, void* ws, size_t ws_bytes, void* stream,
        float* stats = nullptr, int stats_tiles_m = 0) {
  Plan pl;
  int rc = make_plan(op, d, &pl);
  if (rc != JZ_OK) return rc;
  // the caller sized the buffer of the column sums from an earlier plan: it has to be this plan (the run-time tuning table
  // may have been changed in between)
  if (stats && (!plan_leaves_stats(pl) || pl.args.tiles_m != stats_tiles_m)) return JZ_ERR_UNSUPPORTED;
  if (!A || !B || !D) return JZ_ERR_NULL;
  if (!aligned16(A) || !aligned16(B) || !aligned16(D) || (ws && !aligned16(ws))) return JZ_ERR_ALIGN;
  if (overlaps(D, pl.bytesD, A, pl.bytesA) || overlaps(D, pl.bytesD, B, pl.bytesB)) return JZ_ERR_ALIAS;
  if (pl.ws_bytes > 0 && (!ws || ws_bytes < pl.ws_bytes)) return JZ_ERR_WORKSPACE;
  if (pl.ws_bytes > 0 && (overlaps(ws, pl.ws_bytes, A, pl.bytesA) || overlaps(ws, pl.ws_bytes, B, pl.bytesB) ||
                          overlaps(ws, pl.ws_bytes, D, pl.bytesD)))
    return JZ_ERR_ALIAS;
  hipStream_t st = static_cast<hipStream_t>(stream);
  GemmArgs& a = pl.args;
  a.A = static_cast<const unsigned short*>(A);
  a.B = static_cast<const unsigned short*>(B);
  a.D16 = static_cast<unsigned short*>(D);
  a.bytesA = (unsigned)pl.bytesA;
  a.bytesB = (unsigned)pl.bytesB;
  a.Dpart = reinterpret_cast<float*>(static_cast<char*>(ws) + pl.part_offset);
  a.stats = stats;
  unsigned short* dwp = nullptr;
  if (pl.packed) {
    unsigned short* xp = static_cast<unsigned short*>(ws);
    unsigned short* wp = reinterpret_cast<unsigned short*>(static_cast<char*>(ws) + pl.xp_bytes);
    const unsigned short* x = static_cast<const unsigned short*>(op == JZ_FWD ? A : B);
    const unsigned short* wsrc = op == JZ_FWD ? static_cast<const unsigned short*>(B) : nullptr;
    hipLaunchKernelGGL(pad_to_c4, dim3((unsigned)((pl.Wp / 2 + 127) / 128), (unsigned)pl.Hp, (unsigned)(d->N + (wsrc ? 1 : 0))),
                       dim3(128), 0, st, x, xp, d->N, d->H, d->W, d->C, pl.Hp, pl.Wp, d->pad_h, d->pad_w, wsrc,
                       wsrc ? wp : nullptr, d->K, d->R, d->S, pl.KT);
    if (op == JZ_FWD) {
      a.A = xp; a.bytesA = (unsigned)pl.xp_bytes;
      a.B = wp; a.bytesB = (unsigned)pl.wp_bytes;
    } else {
      a.B = xp; a.bytesB = (unsigned)pl.xp_bytes;
      dwp = wp;
      a.D16 = dwp;
    }
    if ((rc = jz::launch_status()) != JZ_OK) return rc;
  }
  if (op == JZ_FWD) rc = stats ? launch_op<OP_FWD_STATS>(pl, st) : launch_op<OP_FWD>(pl, st);
  else if (op == JZ_BWD_DATA) rc = launch_op<OP_BWD_DATA>(pl, st);
  else rc = launch_op<OP_BWD_WEIGHT>(pl, st);
  if (rc != JZ_OK) return rc;
  if (a.splits > 1) {
    long long MN = (long long)a.M * a.N;
    // split lanes per output group: enough workgroups to cover the chip first, then shorten each thread's chain
    int lg = 0;
    while (lg < 5 && (2 << lg) <= a.splits && ((MN + 3) / 4 + (256 >> lg) - 1) / (256 >> lg) < 1024) ++lg;
    const long long per_block = 256 >> lg;
    unsigned blocks = (unsigned)(((MN + 3) / 4 + per_block - 1) / per_block);
    // small-channel backward-weight: the reduction writes the real filter entries straight into dw
    hipLaunchKernelGGL(splitk_reduce, dim3(blocks), dim3(256), 0, st, a.Dpart, dwp ? static_cast<unsigned short*>(D) : a.D16,
                       MN, a.splits, lg, dwp ? pl.KT / 4 : 0, d->S, d->C);
    if ((rc = jz::launch_status()) != JZ_OK) return rc;
    dwp = nullptr;
  }
  if (dwp) {
    int ndw = d->K * d->R * d->S * d->C;
    hipLaunchKernelGGL(unpack_filter_c4, dim3((unsigned)((ndw + 255) / 256)), dim3(256), 0, st, dwp,
                       static_cast<unsigned short*>(D), d->K, d->R, d->S, d->C, pl.KT);
    rc = jz::launch_status();
  }
  return rc;
}

int fc_desc(int mode, int batch, int in_features, int out_features, jz_conv_desc* d) {
  if (mode != JZ_FWD && mode != JZ_BWD_DATA && mode != JZ_BWD_WEIGHT) return JZ_ERR_UNSUPPORTED;
  if (batch <= 0 || in_features <= 0 || out_features <= 0) return JZ_ERR_SHAPE;
  // a fully connected layer is a 1x1 convolution over a 1x1 image
  *d = jz_conv_desc{batch, 1, 1, in_features, out_features, 1, 1, 1, 1, 0, 0};
  return JZ_OK;
}

}  // namespace

// for the fused convolution + batch normalization entry point (jz_bn.hip)
int jz::conv_fwd_stats_plan(const jz_conv_desc* d, size_t* conv_ws_bytes, int* tiles_m) {
  Plan pl;
  int rc = make_plan(JZ_FWD, d, &pl);
  if (rc != JZ_OK) return rc;
  *conv_ws_bytes = pl.ws_bytes;
  *tiles_m = plan_leaves_stats(pl) ? pl.args.tiles_m : 0;
  return JZ_OK;
}
int jz::conv_fwd_run(const jz_conv_desc* d, const void* x, const void* w, void* y, void* ws, size_t ws_bytes, float* stats,
                     int stats_tiles_m, void* stream) {
  return run(JZ_FWD, d, x, w, y, ws, ws_bytes, stream, stats, stats_tiles_m);
}

extern "C" int jz_conv2d_workspace_bytes(int op, const jz_conv_desc* desc, size_t* bytes) {
  if (!bytes) return JZ_ERR_NULL;
  Plan pl;
  int rc = make_plan(op, desc, &pl);
  if (rc != JZ_OK) return rc;
  *bytes = pl.ws_bytes;
  return JZ_OK;
}

extern "C" int jz_conv2d_describe_plan(int op, const jz_conv_desc* desc, char* text, size_t text_bytes) {
  if (!text || text_bytes == 0) return JZ_ERR_NULL;
  Plan pl;
  int rc = make_plan(op, desc, &pl);
  if (rc != JZ_OK) return rc;
  plan_text(pl, text, text_bytes);
  return JZ_OK;
}

extern "C" int jz_conv2d_tune_set(int op, const jz_conv_desc* desc, int tile_m, int tile_n, int k_tile, int wavefronts,
                                  int ring, int splits) {
  Plan pl;
  int rc = make_plan(op, desc, &pl);
  if (rc != JZ_OK) return rc;
  if (!pl.fast || pl.gen || splits < 1) return JZ_ERR_UNSUPPORTED;  // those paths have one kernel shape each
  const Variant* v = nullptr;
  for (const Variant& c : kVariants)
    if (c.BM == tile_m && c.BN == tile_n && c.bk == k_tile && c.waves == wavefronts && c.nst == ring) v = &c;
  if (!v) return JZ_ERR_UNSUPPORTED;
  // the small-channel path runs the 4-wavefront kernels of the four basic tiles at its own k tile depth only
  if (pl.packed && (v->waves != 4 || v->BM > 128 || v->BN > 128 || k_tile != pl.bk || (ring == 3 && k_tile != 32)))
    return JZ_ERR_UNSUPPORTED;
  const GemmArgs& a = pl.args;
  const Tuned t{op == JZ_FWD ? 0 : op == JZ_BWD_DATA ? 1 : 2, a.M, a.N, a.Kred, a.g.R * a.g.S, a.sc_on,
                tile_m, tile_n, k_tile, wavefronts, ring, splits};
  std::lock_guard<std::mutex> lock(g_tune_mutex);
  for (Tuned& e : g_tune_rt)
    if (same_key(e, t)) {
      e = t;
      return JZ_OK;
    }
  g_tune_rt.push_back(t);
  return JZ_OK;
}

extern "C" int jz_conv2d_tune_clear(void) {
  std::lock_guard<std::mutex> lock(g_tune_mutex);
  g_tune_rt.clear();
  return JZ_OK;
}

extern "C" int jz_conv2d_fwd(const jz_conv_desc* desc, const void* x16, const void* w16, void* y16, void* ws,
                             size_t ws_bytes, void* hip_stream) {
  return run(JZ_FWD, desc, x16, w16, y16, ws, ws_bytes, hip_stream);
}

extern "C" int jz_conv2d_bwd_data(const jz_conv_desc* desc, const void* dy16, const void* w16, void* dx16, void* ws,
                                  size_t ws_bytes, void* hip_stream) {
  return run(JZ_BWD_DATA, desc, dy16, w16, dx16, ws, ws_bytes, hip_stream);
}

extern "C" int jz_conv2d_bwd_weight(const jz_conv_desc* desc, const void* x16, const void* dy16, void* dw16, void* ws,
                                    size_t ws_bytes, void* hip_stream) {
  return run(JZ_BWD_WEIGHT, desc, dy16, x16, dw16, ws, ws_bytes, hip_stream);  // A = dy, B = x
}

extern "C" int jz_gemm_fc_workspace_bytes(int mode, int batch, int in_features, int out_features, size_t* bytes) {
  jz_conv_desc d;
  int rc = fc_desc(mode, batch, in_features, out_features, &d);
  if (rc != JZ_OK) return rc;
  return jz_conv2d_workspace_bytes(mode, &d, bytes);
}

extern "C" int jz_gemm_fc(int mode, int batch, int in_features, int out_features, const void* a16, const void* b16,
                          void* out16, void* ws, size_t ws_bytes, void* hip_stream) {
  jz_conv_desc d;
  int rc = fc_desc(mode, batch, in_features, out_features, &d);
  if (rc != JZ_OK) return rc;
  // FWD: (x, w) ; BWD_DATA: (dy, w) ; BWD_WEIGHT: (dy, x) -- already the kernel's (A, B) order in every mode
  return run(mode, &d, a16, b16, out16, ws, ws_bytes, hip_stream);
}
