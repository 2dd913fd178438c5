// Implicit-GEMM kernel with LDS-direct loads and a multi-stage ring, for channel counts that allow 16-byte
// vector access (see the table in jz_igemm.h for what A, B, m, n, k are in each op).  Included by jz_conv.hip.
//
// Why this shape.  One k tile of a 128x128 output tile is 512 MFMA cycles per wavefront but an HBM round trip
// is several thousand cycles, so a tile's operands have to be requested three tiles ahead.  Staging that much
// through registers costs the occupancy it is meant to buy, so the tiles never touch registers on the way in:
// `buffer_load_dwordx4 ... lds` writes 64 lanes x 16 bytes straight into LDS (wave-uniform base + lane*16), out of
// range offsets deliver zeros (padding taps, rows beyond M/N, the reduction tail), and NST stages of
// (BM+BN) x 128 bytes form a ring.  Each iteration: wait until the oldest stage has landed (vmcnt), one
// workgroup barrier, request the tile NST-1 ahead into the stage that was just consumed, multiply.
//
// LDS layouts (one stage = A tile then B tile, both TBK = 32 or 64 deep):
//   k-contiguous operand  ("KC": x / dy gathered per pixel, the forward filter): [row][TBK/8 chunks of 16 B], rows
//       packed back to back, chunk c of row r stored at position c ^ swizzle(r); MFMA operands are plain ds_read_b128.
//   mn-contiguous operand ("MC": the filter in backward-data, dy and x in backward-weight): [k][ROWS/8 chunks],
//       stored exactly as it sits in memory, chunk c of k-row k at position c ^ swz(k); MFMA operands come from
//       ds_read_b64_tr_b16, which hands each lane four consecutive k of one mn out of such a layout (within 16
//       lanes: lanes 4j..4j+3 supply 16 consecutive mn of k-row j, lane i receives rows 0..3 at mn i).
// The swizzles make both the 1 KB DMA writes and the operand reads bank-conflict free.
//
// The operand reads are issued through inline assembly with hand-placed s_waitcnt: the compiler cannot tell which
// ring stage an LDS read touches and would otherwise wait for every outstanding LDS-direct load (vmcnt(0)) before
// each read, which would serialise the ring.
//
// What bounds it (measured on MI355X on an 8192 x 4096 x 4096 GEMM): with the operand loads removed the loop runs at
// 1.3-1.6 PFLOP/s, with them at 0.6 (128x128 tile) to 1.1 (256x256 tile) PFLOP/s; removing the LDS operand reads or the
// barrier changes little.  The LDS-direct path delivers about 12 TB/s chip-wide into LDS at 8 resident wavefronts per
// compute unit, so what counts is flop per byte brought in (tile size) and whole 128-byte lines per row (a 32-deep k
// tile of a k-contiguous operand uses half a line per row and fetches the line again for the next tile: the 64-deep
// variants exist for that).  Hence the 8-wavefront variants with 256-row tiles next to the 4-wavefront ones.
#pragma once

typedef _Float16 half4v __attribute__((ext_vector_type(4)));
#define JZ_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))

// The host pass of hipcc parses these bodies too and has no AMDGPU register constraints, hence the guards.
template <int OFF>
__device__ __forceinline__ half8 lds_read_b128(unsigned addr) {
  half8 v = {};
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
#endif
  return v;
}
template <int OFF>
__device__ __forceinline__ half4v lds_read_tr16_b64(unsigned addr) {
  half4v v = {};
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
#endif
  return v;
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
#endif
}
// Wait until at most KEEP LDS reads are outstanding ...
template <int KEEP>
__device__ __forceinline__ void lds_wait() {
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(KEEP));
#endif
}
// ... and tie an operand to that point: volatile asm statements keep their order, and an MFMA that consumes the
// "output" of this empty statement cannot be scheduled above it (hence not above the wait either).
__device__ __forceinline__ void lds_pin(half8& v) {
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("" : "+v"(v));
#endif
}

typedef __attribute__((address_space(3))) unsigned char lds_byte;
// one LDS-direct load: 64 lanes x 16 bytes from `rsrc` at per-lane byte offset `voff` to LDS at dst + lane * 16
__device__ __forceinline__ void jz_dma16(__amdgpu_buffer_rsrc_t rsrc, lds_byte* dst, unsigned voff) {
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, dst, 16, (int)voff, 0, 0, 0);
}

// slabs the epilogue stages the fp16 tile in: its staging buffer has to fit the ring
constexpr int dma_epass(int bm, int bn) { return bm * (bn + 8) * 2 > 128 * 1024 ? 2 : 1; }

// WGM x WGN wavefronts share a BM x BN output tile; each owns (BM / WGM) x (BN / WGN) of it.  The larger a
// wavefront's share, the fewer LDS bytes it reads per MFMA (a 128x64 share: 6 operand reads for 8 MFMAs per k step,
// a 64x64 share: 4 for 4), and the larger the workgroup's tile, the fewer bytes come in from L2 per flop.
template <int OP, int BM, int BN, int TBK, int NST, bool MASKA = false, int WGM = 2, int WGN = 2>
__global__ __launch_bounds__(64 * WGM * WGN) void igemm_dma_kernel(GemmArgs a) {
  static_assert(TBK == 32 || TBK == 64, "k tile depth");
  constexpr bool A_KC = OP != OP_BWD_WEIGHT;  // A has k contiguous in memory
  constexpr bool B_KC = OP == OP_FWD;
  constexpr int NW = WGM * WGN, NT = 64 * NW;  // wavefronts, threads
  constexpr int WTM = BM / WGM, WTN = BN / WGN;  // a wavefront's share of the tile
  constexpr int TM = WTM / 32, TN = WTN / 32;    // ... as 32x32 MFMA tiles
  static_assert(TM >= 1 && TN >= 1 && TM * 32 * WGM == BM && TN * 32 * WGN == BN, "tile / wavefront grid mismatch");
  constexpr int NKS = TBK / 16;               // MFMA k steps per tile
  constexpr int RB = 2 * TBK;                 // bytes per row of a KC tile
  constexpr int CR = TBK / 8;                 // 16-byte chunks per row of a KC tile
  constexpr int A_BYTES = BM * RB, B_BYTES = BN * RB, STAGE = A_BYTES + B_BYTES;
  constexpr int LA = BM * CR / NT, LB = BN * CR / NT;  // LDS-direct loads per thread per tile and operand
  static_assert(LA * NT == BM * CR && LB * NT == BN * CR, "tile does not divide among the loaders");
  static_assert(LA >= 1 && LB >= 1, "tile too small for the loader");
  constexpr int LPT = LA + LB;
  extern __shared__ __align__(16) unsigned short lds[];
  lds_byte* const ldsb = (lds_byte*)lds;  // LDS-direct loads take an LDS-address-space pointer
  const unsigned lds_base = (unsigned)(uintptr_t)JZ_LDS_PTR(lds);

  const ConvGeom& g = a.g;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;

  unsigned L = xcd_remap(blockIdx.x, gridDim.x);
  const int tiles_mn = a.tiles_m * a.tiles_n;
  const int split = (int)(L / (unsigned)tiles_mn);
  L -= (unsigned)split * (unsigned)tiles_mn;
  const int m0 = (int)(L / (unsigned)a.tiles_n) * BM;
  const int n0 = (int)(L % (unsigned)a.tiles_n) * BN;
  const int kt_begin = split * a.kt_per_split;
  const int kt_end = (kt_begin + a.kt_per_split < a.nkt) ? kt_begin + a.kt_per_split : a.nkt;
  const int nk = kt_end - kt_begin;

  const __amdgpu_buffer_rsrc_t rsrcA = __builtin_amdgcn_make_buffer_rsrc((void*)a.A, 0, (int)a.bytesA, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrcB = __builtin_amdgcn_make_buffer_rsrc((void*)a.B, 0, (int)a.bytesB, 0x00020000);
  constexpr unsigned OOB = 0xffffffffu;

  // ---- loader geometry ---------------------------------------------------------------------
  // KC tile: one load covers 64 / CR rows; load ii of wave w covers rows (NW ii + w) * (64 / CR) + lane / CR and the
  // lane's LDS slot is chunk position lane % CR, so it fetches global chunk (lane % CR) ^ swizzle(row).  The swizzle
  // ((row >> 1) & 7 for 128-byte rows, (row >> 2) & 3 for 64-byte rows) is the same for every ii and sends any 16
  // consecutive rows' copies of one chunk to 16 different 16-byte bank groups.
  constexpr int KC_RPI = 64 / CR;
  const int kc_row = wave * KC_RPI + lane / CR;  // + NW * KC_RPI * ii
  const int kc_chunk = (lane % CR) ^ (TBK == 64 ? ((kc_row >> 1) & 7) : ((kc_row >> 2) & 3));
  // MC tile with ROWS mn: CPR = ROWS / 8 chunks per k-row, 64 / CPR k-rows per load
  // (k & 7 is the same for every load ii of a lane: NW * (64 / cpr) is a multiple of 8)
  auto mc_k = [&](int rows, int ii) { int cpr = rows / 8; return (NW * ii + wave) * (64 / cpr) + lane / cpr; };
  auto mc_chunk = [&](int rows, int k) {
    int cpr = rows / 8;
    int swz = cpr >= 16 ? 2 * (k & 7) : 2 * (k & 3);
    return (lane % cpr) ^ swz;
  };

  // per-thread gather state
  unsigned sa0[LA];
  int sa1[LA], sa2[LA];
  (void)sa0; (void)sa1; (void)sa2;
  if (OP != OP_BWD_WEIGHT) {  // A rows are pixels of the (n, OH, OW) grid
#pragma unroll
    for (int ii = 0; ii < LA; ++ii) {
      int m = m0 + NW * KC_RPI * ii + kc_row;
      if (m < a.M) {
        unsigned n = fd_div((unsigned)m, g.d_ohow);
        unsigned rem = (unsigned)m - n * (unsigned)(g.OH * g.OW);
        unsigned oh = fd_div(rem, g.d_ow);
        unsigned ow = rem - oh * (unsigned)g.OW;
        if (OP == OP_FWD) {
          sa1[ii] = (int)oh * g.sh - g.ph;
          sa2[ii] = (int)ow * g.sw - g.pw;
          // byte offset of tap (0,0) plus this lane's chunk; may wrap below zero for padded rows, the tap offset
          // brings every in-range access back (unsigned arithmetic)
          sa0[ii] = (unsigned)(((int)n * g.IH + sa1[ii]) * g.row_pitch + sa2[ii] * g.pix_step + kc_chunk * 8) * 2u;
        } else {
          sa0[ii] = n * (unsigned)(g.IH * g.row_pitch);
          sa1[ii] = (int)oh + g.ph;
          sa2[ii] = (int)ow + g.pw;
        }
      } else {
        sa0[ii] = 0;
        sa1[ii] = -(1 << 28);  // fails every bounds check
        sa2[ii] = -(1 << 28);
      }
    }
  }
  // B-side state
  unsigned sb0[LB];
  int sb1 = 0, sb2 = 0, sbc = 0;
  (void)sb0; (void)sb1; (void)sb2; (void)sbc;
  if (OP == OP_FWD) {
#pragma unroll
    for (int ii = 0; ii < LB; ++ii) {
      int nn = n0 + NW * KC_RPI * ii + kc_row;
      sb0[ii] = nn < a.N ? (unsigned)(nn * a.Kred + kc_chunk * 8) * 2u : OOB;
    }
  } else if (OP == OP_BWD_DATA) {
    // filter w[ko][tap][c]: k-row = ko (within the tap), chunk = 8 consecutive c
#pragma unroll
    for (int ii = 0; ii < LB; ++ii) {
      int k = mc_k(BN, ii);
      int nn = n0 + mc_chunk(BN, k) * 8;
      sb0[ii] = nn < a.N ? (unsigned)((k * g.R * g.S) * a.N + nn) * 2u : OOB;  // + (c0 * R * S + tap) * N * 2 per tile
    }
  } else {
    // x gathered: this lane's 8 columns (tap, c..c+7) are the same for every load (k & 7 does not depend on ii)
    int nn = n0 + mc_chunk(BN, mc_k(BN, 0)) * 8;
    if (nn < a.N) {
      unsigned tap = fd_div((unsigned)nn, g.d_ic);
      unsigned r = fd_div(tap, g.d_s);
      sbc = nn - (int)tap * g.IC;
      sb1 = (int)r - g.ph;
      sb2 = (int)(tap - r * g.S) - g.pw;
    } else {
      sb1 = -(1 << 28);
      sb2 = -(1 << 28);
    }
  }
  unsigned sam = 0;  // BWD_WEIGHT A: dy[(n,p,q)][k_out], chunk = 8 consecutive k_out
  if (OP == OP_BWD_WEIGHT) {
    int mm = m0 + mc_chunk(BM, mc_k(BM, 0)) * 8;
    sam = mm < a.M ? (unsigned)mm * 2u : OOB;
  }

  // Requesting k tile kt into ring stage st = LPT loads per thread (LA for A, then LB for B).  They are issued one
  // at a time, in between the MFMA groups of the tile being multiplied, so that their address arithmetic runs in
  // the shadow of the matrix pipe instead of in front of it.
  struct TileCtx {
    int k0, c0, r, s;
    unsigned tap, tapoff, tileoff;
  };
  auto tile_ctx = [&](int kt) {
    TileCtx c;
    c.k0 = kt * TBK;
    c.tap = 0; c.c0 = 0; c.r = 0; c.s = 0; c.tapoff = 0; c.tileoff = 0;
    // the whole tile lies inside one filter tap: wave-uniform values.  Either IC % TBK == 0, or there is only one tap
    // (1x1 layers, fully connected) and the last tile is ragged: chunks at or beyond IC are then not requested.
    if (OP != OP_BWD_WEIGHT) {
      c.tap = fd_div((unsigned)c.k0, g.d_ic);
      c.c0 = c.k0 - (int)c.tap * g.IC;
      c.r = (int)fd_div(c.tap, g.d_s);
      c.s = (int)c.tap - c.r * g.S;
      c.tapoff = (unsigned)(c.r * g.row_pitch + c.s * g.s_step + c.c0) * 2u;
      c.tileoff = (unsigned)((c.c0 * g.R * g.S + (int)c.tap) * a.N) * 2u;
    }
    return c;
  };
  auto issue_load = [&](const TileCtx& c, int st, auto l_tag) {
    constexpr int Lidx = decltype(l_tag)::value;
    if constexpr (Lidx < LPT) {
      lds_byte* sA = ldsb + st * STAGE;
      lds_byte* sB = sA + A_BYTES;
      if constexpr (Lidx < LA) {
        constexpr int ii = Lidx;
        if constexpr (OP == OP_FWD) {
          int ih = sa1[ii] + c.r, iw = sa2[ii] + c.s;
          bool ok = (unsigned)ih < (unsigned)g.IH && (unsigned)iw < (unsigned)g.IW && c.c0 + kc_chunk * 8 < g.IC;
          jz_dma16(rsrcA, sA + (NW * ii + wave) * 1024, ok ? sa0[ii] + c.tapoff : OOB);
        } else if constexpr (OP == OP_BWD_DATA) {
          // input pixel (h,w) receives from output pixel ((h + pad - r) / stride, ...) when the division is exact
          int th = sa1[ii] - c.r, tw = sa2[ii] - c.s;
          int ih = (int)fd_div((unsigned)(th < 0 ? 0 : th), g.d_sh);
          int iw = (int)fd_div((unsigned)(tw < 0 ? 0 : tw), g.d_sw);
          bool ok = ih * g.sh == th && iw * g.sw == tw && ih < g.IH && iw < g.IW &&  // false for negative th / tw too
                    c.c0 + kc_chunk * 8 < g.IC;
          unsigned off = (sa0[ii] + (unsigned)(ih * g.row_pitch + iw * g.pix_step + c.c0 + kc_chunk * 8)) * 2u;
          jz_dma16(rsrcA, sA + (NW * ii + wave) * 1024, ok ? off : OOB);
        } else {  // dy rows j = k0 + k
          int j = c.k0 + mc_k(BM, ii);
          unsigned off = (sam != OOB && j < a.Kred) ? sam + (unsigned)(j * a.M) * 2u : OOB;
          jz_dma16(rsrcA, sA + (NW * ii + wave) * 1024, off);
        }
      } else {
        constexpr int ii = Lidx - LA;
        if constexpr (OP == OP_FWD) {
          const bool ok = sb0[ii] != OOB && c.k0 + kc_chunk * 8 < a.Kred;
          jz_dma16(rsrcB, sB + (NW * ii + wave) * 1024, ok ? sb0[ii] + (unsigned)c.k0 * 2u : OOB);
        } else if constexpr (OP == OP_BWD_DATA) {
          const bool ok = sb0[ii] != OOB && c.c0 + mc_k(BN, ii) < g.IC;
          jz_dma16(rsrcB, sB + (NW * ii + wave) * 1024, ok ? sb0[ii] + c.tileoff : OOB);
        } else {  // x at this lane's tap for output pixel j
          int j = c.k0 + mc_k(BN, ii);
          unsigned n = fd_div((unsigned)j, g.d_ohow);
          unsigned rem = (unsigned)j - n * (unsigned)(g.OH * g.OW);
          int p = (int)fd_div(rem, g.d_ow);
          int q = (int)rem - p * g.OW;
          int ih = p * g.sh + sb1, iw = q * g.sw + sb2;
          bool ok = j < a.Kred && (unsigned)ih < (unsigned)g.IH && (unsigned)iw < (unsigned)g.IW;
          unsigned off = (unsigned)(((int)n * g.IH + ih) * g.row_pitch + iw * g.pix_step + sbc) * 2u;
          jz_dma16(rsrcB, sB + (NW * ii + wave) * 1024, ok ? off : OOB);
        }
      }
    }
  };
  // loads PART, PART + NKS, ... of the tile (PART in 0..NKS-1): one share per MFMA group
  auto issue_part = [&](const TileCtx& c, int st, auto part_tag) {
    constexpr int PART = decltype(part_tag)::value;
    issue_load(c, st, std::integral_constant<int, PART>{});
    issue_load(c, st, std::integral_constant<int, PART + NKS>{});
    issue_load(c, st, std::integral_constant<int, PART + 2 * NKS>{});
    issue_load(c, st, std::integral_constant<int, PART + 3 * NKS>{});
  };
  static_assert(LPT <= 4 * NKS, "issue_part covers at most 4 loads per MFMA group");
  static_assert(NST >= 3 && NST <= 8 && (NST - 2) * LPT <= 63, "ring depth: vmcnt is a 6-bit counter");
  auto issue = [&](int kt, int st) {
    TileCtx c = tile_ctx(kt);
    issue_part(c, st, std::integral_constant<int, 0>{});
    issue_part(c, st, std::integral_constant<int, 1>{});
    if constexpr (NKS == 4) {
      issue_part(c, st, std::integral_constant<int, 2>{});
      issue_part(c, st, std::integral_constant<int, 3>{});
    }
  };

  // ---- MFMA operand read addresses (byte offsets inside a stage) --------------------------------
  // KC: row = base + 32 t + lane % 32, chunk (2 ks + lane / 32) at position chunk ^ swizzle(row); one address per ks,
  //     the 32-row sub-tiles t are 32 * RB bytes apart and share the swizzle (immediate offset).
  // MC: 16-lane group gi = lane / 16 handles mn half gi % 2 and k block gi / 2 of the 32x16 operand; lane 4 j + c4
  //     of the group addresses k-row j, the 8-byte piece c4 of those 16 mn.  One address per (sub-tile t, k half),
  //     ks advances by 16 k-rows (immediate offset).
  unsigned adA[(A_KC ? NKS : 2 * TM)], adB[(B_KC ? NKS : 2 * TN)];
  {
    const int r31 = lane & 31, hi = lane >> 5;
    const int gi = lane >> 4, j = (lane >> 2) & 3, c4 = lane & 3;
    const int kc_swz = TBK == 64 ? ((r31 >> 1) & 7) : ((r31 >> 2) & 3);
    if (A_KC) {
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks)
        adA[ks] = (unsigned)((wm * WTM + r31) * RB + (((2 * ks + hi) ^ kc_swz) * 16));
    } else {
      constexpr int CPR = BM / 8;
#pragma unroll
      for (int t = 0; t < TM; ++t)
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
          int k = 8 * (gi >> 1) + 4 * hf + j;
          int c = (wm * WTM + 32 * t + 16 * (gi & 1) + 4 * c4) / 8;
          int swz = CPR >= 16 ? 2 * (k & 7) : 2 * (k & 3);
          adA[t * 2 + hf] = (unsigned)(k * (BM * 2) + ((c ^ swz) * 16) + (c4 & 1) * 8);
        }
    }
    if (B_KC) {
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks)
        adB[ks] = (unsigned)(A_BYTES + (wn * WTN + r31) * RB + (((2 * ks + hi) ^ kc_swz) * 16));
    } else {
      constexpr int CPR = BN / 8;
#pragma unroll
      for (int t = 0; t < TN; ++t)
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
          int k = 8 * (gi >> 1) + 4 * hf + j;
          int c = (wn * WTN + 32 * t + 16 * (gi & 1) + 4 * c4) / 8;
          int swz = CPR >= 16 ? 2 * (k & 7) : 2 * (k & 3);
          adB[t * 2 + hf] = (unsigned)(A_BYTES + k * (BN * 2) + ((c ^ swz) * 16) + (c4 & 1) * 8);
        }
    }
  }

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  // read the operands of k step KS of the stage at byte address sb
  auto read_frags = [&](unsigned sb, auto ks_tag, half8 (&fa)[TM], half8 (&fb)[TN]) {
    constexpr int KS = decltype(ks_tag)::value;
    if (A_KC) {
      fa[0] = lds_read_b128<0>(sb + adA[KS]);
      if constexpr (TM > 1) fa[1] = lds_read_b128<32 * RB>(sb + adA[KS]);
      if constexpr (TM > 2) fa[2] = lds_read_b128<64 * RB>(sb + adA[KS]);
      if constexpr (TM > 3) fa[3] = lds_read_b128<96 * RB>(sb + adA[KS]);
    } else {
#pragma unroll
      for (int t = 0; t < TM; ++t) {
        half4v lo = lds_read_tr16_b64<KS * 16 * BM * 2>(sb + adA[t * 2]);
        half4v hi = lds_read_tr16_b64<KS * 16 * BM * 2>(sb + adA[t * 2 + 1]);
        fa[t] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      }
    }
    if (B_KC) {
      fb[0] = lds_read_b128<0>(sb + adB[KS]);
      if constexpr (TN > 1) fb[1] = lds_read_b128<32 * RB>(sb + adB[KS]);
      if constexpr (TN > 2) fb[2] = lds_read_b128<64 * RB>(sb + adB[KS]);
      if constexpr (TN > 3) fb[3] = lds_read_b128<96 * RB>(sb + adB[KS]);
    } else {
#pragma unroll
      for (int t = 0; t < TN; ++t) {
        half4v lo = lds_read_tr16_b64<KS * 16 * BN * 2>(sb + adB[t * 2]);
        half4v hi = lds_read_tr16_b64<KS * 16 * BN * 2>(sb + adB[t * 2 + 1]);
        fb[t] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      }
    }
  };
  auto mma = [&](auto ks_tag, half8 (&fa)[TM], half8 (&fb)[TN]) {
    if constexpr (MASKA) {
      // small-channel forward: the tail of each gathered run belongs to the next pixel, not to this filter row;
      // clear it so that it cannot contribute (its weights are zero, but 0 * Inf would not be)
      constexpr int KS = decltype(ks_tag)::value;
#pragma unroll
      for (int t = 0; t < TM; ++t) {
        u32x4 w;
        __builtin_memcpy(&w, &fa[t], 16);
#pragma unroll
        for (int dd = 0; dd < 4; ++dd)
          if (16 * KS + 8 * (lane >> 5) + 2 * dd >= g.kvalid) w[dd] = 0u;
        __builtin_memcpy(&fa[t], &w, 16);
      }
    }
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        // n operand in the first slot: each lane then owns 4 consecutive n for one m (row = lane % 32)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fb[j], fa[i], acc[i][j], 0, 0, 0);
  };
  auto settle = [&](auto keep_tag, half8 (&fa)[TM], half8 (&fb)[TN]) {
    constexpr int KEEP = decltype(keep_tag)::value;
    lds_wait<KEEP>();
#pragma unroll
    for (int t = 0; t < TM; ++t) lds_pin(fa[t]);
#pragma unroll
    for (int t = 0; t < TN; ++t) lds_pin(fb[t]);
  };
  constexpr int READS = (A_KC ? TM : 2 * TM) + (B_KC ? TN : 2 * TN);  // LDS reads per k step
  static_assert(READS <= 15, "lgkmcnt is a 4-bit counter");

  // wait until at most `younger` later tiles (capped at NST-2) are still in flight
  auto wait_tiles = [&](int younger) {
    if (younger >= NST - 2) wait_vmcnt<(NST - 2) * LPT>();
    else if (NST - 2 > 6 && younger == 6) wait_vmcnt<6 * LPT>();
    else if (NST - 2 > 5 && younger == 5) wait_vmcnt<5 * LPT>();
    else if (NST - 2 > 4 && younger == 4) wait_vmcnt<4 * LPT>();
    else if (NST - 2 > 3 && younger == 3) wait_vmcnt<3 * LPT>();
    else if (NST - 2 > 2 && younger == 2) wait_vmcnt<2 * LPT>();
    else if (NST - 2 > 1 && younger == 1) wait_vmcnt<LPT>();
    else wait_vmcnt<0>();
  };

  // ---- the ring ---------------------------------------------------------------------------------
  // One iteration multiplies tile i out of stage i % NST.  Its first operands (k step 0) were already read at the end
  // of the previous iteration, so the matrix pipe never waits for an LDS round trip at the top of an iteration:
  //
  //     read k step 1 .. ; request part of tile i+NST-1 ; MFMA k step 0 ; ... ; all reads of tile i are in registers
  //     wait until tile i+1 has landed ; BARRIER ; read k step 0 of tile i+1 ; MFMA last k step of tile i
  //
  // The barrier therefore sits between two MFMA groups.  It says two things: every wavefront's share of tile i+1
  // is in LDS, and every wavefront has finished reading tile i (its operands are in registers), so stage i % NST
  // may be overwritten by the loads requested in the next iteration.  Barriers are bare (no fence): a fenced
  // barrier makes the compiler drain every LDS-direct load first (vmcnt(0)); the ordering that matters is spelled
  // out by hand with vmcnt / lgkmcnt waits.
  half8 fa0[TM], fb0[TN], fa1[TM], fb1[TN];
  // STEADY: request tile c into stage ist while multiplying; NEXT: there is a tile after this one
  auto iteration = [&](int st, auto steady_tag, const TileCtx& c, int ist, bool has_next, int younger_after_next) {
    constexpr bool ISSUE = decltype(steady_tag)::value;
    const unsigned sb = lds_base + (unsigned)(st * STAGE);
    const unsigned sb_next = lds_base + (unsigned)(((st + 1) % NST) * STAGE);
    read_frags(sb, std::integral_constant<int, 1>{}, fa1, fb1);
    if (ISSUE) issue_part(c, ist, std::integral_constant<int, 0>{});
    settle(std::integral_constant<int, READS>{}, fa0, fb0);
    mma(std::integral_constant<int, 0>{}, fa0, fb0);
    if constexpr (NKS == 4) {
      read_frags(sb, std::integral_constant<int, 2>{}, fa0, fb0);
      if (ISSUE) issue_part(c, ist, std::integral_constant<int, 1>{});
      settle(std::integral_constant<int, READS>{}, fa1, fb1);
      mma(std::integral_constant<int, 1>{}, fa1, fb1);
      read_frags(sb, std::integral_constant<int, NKS - 1>{}, fa1, fb1);
      if (ISSUE) issue_part(c, ist, std::integral_constant<int, 2>{});
      settle(std::integral_constant<int, READS>{}, fa0, fb0);
      mma(std::integral_constant<int, 2>{}, fa0, fb0);
      if (ISSUE) issue_part(c, ist, std::integral_constant<int, NKS - 1>{});
    } else {
      if (ISSUE) issue_part(c, ist, std::integral_constant<int, 1>{});
    }
    settle(std::integral_constant<int, 0>{}, fa1, fb1);  // every LDS read of this tile has completed
    if (ISSUE || has_next) {
      if (ISSUE) wait_vmcnt<(NST - 2) * LPT>();
      else wait_tiles(younger_after_next);
      __builtin_amdgcn_s_barrier();
      read_frags(sb_next, std::integral_constant<int, 0>{}, fa0, fb0);
    }
    mma(std::integral_constant<int, NKS - 1>{}, fa1, fb1);
  };

#pragma unroll
  for (int s = 0; s < NST - 1; ++s)
    if (s < nk) issue(kt_begin + s, s);
  if (nk > 0) {
    wait_tiles(nk - 1);
    __builtin_amdgcn_s_barrier();
    read_frags(lds_base, std::integral_constant<int, 0>{}, fa0, fb0);
  }
  int i = 0;
  for (; i + NST - 1 < nk; ++i) {  // steady state, branch-free body: NST-2 younger tiles stay in flight
    TileCtx c = tile_ctx(kt_begin + i + NST - 1);
    iteration(i % NST, std::true_type{}, c, (i + NST - 1) % NST, true, 0);
  }
  for (; i < nk; ++i) {  // drain: nothing left to request
    TileCtx c{};
    iteration(i % NST, std::false_type{}, c, 0, i + 1 < nk, nk - 2 - i);
  }
  __syncthreads();  // the epilogue reuses the ring as its staging tile

  igemm_epilogue_impl<BM, BN, TM, TN, NT, dma_epass(BM, BN)>(a, acc, lds, m0, n0, split, tid, lane, wm * WTM, wn * WTN);
}
