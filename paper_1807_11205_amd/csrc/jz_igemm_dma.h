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

// compile-time loop: f(std::integral_constant<int, I>{}) for I = B .. E-1 (immediates of inline assembly and the
// slot arithmetic of the schedule need constant expressions)
template <int B, int E, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (B < E) {
    f(std::integral_constant<int, B>{});
    static_for<B + 1, E>(f);
  }
}
// nothing may be moved across this point by the instruction scheduler
__device__ __forceinline__ void sched_fence() {
#if defined(__HIP_DEVICE_COMPILE__)
  __builtin_amdgcn_sched_barrier(0);
#endif
}
// one LDS-direct load with the wave-uniform part of the offset in a scalar register
__device__ __forceinline__ void jz_dma16s(__amdgpu_buffer_rsrc_t rsrc, lds_byte* dst, unsigned voff, unsigned soff) {
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, dst, 16, (int)voff, (int)soff, 0, 0);
}

// WGM x WGN wavefronts share a BM x BN output tile; each owns (BM / WGM) x (BN / WGN) of it.  The larger a
// wavefront's share, the fewer LDS bytes it reads per MFMA (a 128x64 share: 6 operand reads for 8 MFMAs per k step,
// a 64x64 share: 4 for 4), and the larger the workgroup's tile, the fewer bytes come in from L2 per flop.
//
// Instruction budget.  A wavefront issues in order, and the matrix pipe accepts one 32x32x16 MFMA every 32 cycles,
// so everything that is not an MFMA has to fit into the ~8 issue slots between two MFMAs or the pipe idles.  Hence:
//   * a load's address is  descriptor base + per-lane offset (VGPR, fixed for the whole k loop) + per-tile offset
//     (SGPR: filter tap and channel block).  Padding taps and rows beyond M are handled by a per-row bit mask of
//     invalid taps built once in the prologue: one v_bfe_i32 turns the tap's bit into 0 / -1 and an OR sends the
//     lane's offset out of the descriptor's range, which makes the load deliver zeros.  Two VALU instructions per
//     load instead of a dozen, and no divergent control flow inside the loop.
//   * gathered operands whose in-range taps can start before the tensor (padding) use a descriptor whose base is
//     moved down by that margin, so that the per-lane offset is never negative.
//   * the loop body is laid out MFMA by MFMA in the source and fenced (sched_fence) so that the loads and LDS reads
//     sit between the MFMAs instead of in one block in front of them.
// GEN = true keeps the plain per-load tap arithmetic for the shapes the masks do not cover (more than 32 taps;
// strided multi-tap backward-data, whose source pixel is not an affine function of the tap).
// the k lowest bits, k in [0, 32]
__device__ __forceinline__ unsigned low_bits(int k) { return k >= 32 ? 0xffffffffu : (1u << k) - 1u; }
__device__ __forceinline__ int clamp_to(int x, int hi) { return x < 0 ? 0 : (x > hi ? hi : x); }

template <int OP_ARG, int BM, int BN, int TBK, int NST, bool MASKA = false, int WGM = 2, int WGN = 2, bool GEN = false>
__global__ __launch_bounds__(64 * WGM * WGN) void igemm_dma_kernel(GemmArgs a) {
  // the forward kernel with column sums in its epilogue (1), the backward-data kernel with batch-norm backward sums (2),
  // the same with the gradient of a residual block's end formed from the tile first (3)
  constexpr int STATS = OP_ARG == OP_FWD_STATS ? 1 : (OP_ARG == OP_BWD_DATA_STATS ? 2 : (OP_ARG == OP_BWD_DATA_BLOCK_END ? 3 : 0));
  constexpr int OP = STATS == 1 ? OP_FWD : (STATS >= 2 ? OP_BWD_DATA : OP_ARG);
  static_assert(TBK == 32 || TBK == 64, "k tile depth");
  static_assert(!GEN || OP != OP_BWD_WEIGHT, "backward-weight has no generic variant");
  constexpr bool A_KC = OP != OP_BWD_WEIGHT;  // A has k contiguous in memory
  constexpr bool B_KC = OP == OP_FWD;
  constexpr int NW = WGM * WGN, NT = 64 * NW;  // wavefronts, threads
  constexpr int WTM = BM / WGM, WTN = BN / WGN;  // a wavefront's share of the tile
  constexpr int TM = WTM / 32, TN = WTN / 32;    // ... as 32x32 MFMA tiles
  static_assert(TM >= 1 && TN >= 1 && TM * 32 * WGM == BM && TN * 32 * WGN == BN, "tile / wavefront grid mismatch");
  constexpr int NKS = TBK / 16;               // MFMA k steps per tile
  constexpr int G = TM * TN;                  // MFMAs per k step
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
  const int tid = threadIdx.x, lane = tid & 63;
  // the wavefront index as a scalar: everything derived from it (LDS destinations, M0) then stays in SGPRs
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WGN, wn = wave % WGN;

  unsigned L = xcd_remap(blockIdx.x, gridDim.x);
  const int tiles_mn = a.tiles_m * a.tiles_n;
  const int split = (int)fd_div(L, a.d_tiles_mn);
  L -= (unsigned)split * (unsigned)tiles_mn;
  const unsigned trow = fd_div(L, a.d_tiles_n);
  const int m0 = (int)trow * BM;
  const int n0 = (int)(L - trow * (unsigned)a.tiles_n) * BN;
  const int kt_begin = split * a.kt_per_split;
  const int kt_end = (kt_begin + a.kt_per_split < a.nkt) ? kt_begin + a.kt_per_split : a.nkt;
  const int nk = kt_end - kt_begin;

  constexpr unsigned OOB = 0xffffffffu;
  // Margin by which the descriptor of the gathered operand A starts before the tensor (bytes).  Forward: tap (0,0) of
  // a padded row lies up to (ph, pw) pixels before the row's first pixel.  Backward-data (unit stride): the per-tile
  // offset counts taps from the far corner (R-1-r, S-1-s), see below.
  unsigned biasA = 0;
  if (!GEN) {
    if (OP == OP_FWD) biasA = (unsigned)(g.ph * g.row_pitch + g.pw * g.pix_step) * 2u;
    if (OP == OP_BWD_DATA) biasA = (unsigned)((g.R - 1) * g.row_pitch + (g.S - 1) * g.pix_step) * 2u;
  }
  const __amdgpu_buffer_rsrc_t rsrcA =
      __builtin_amdgcn_make_buffer_rsrc((void*)((const char*)a.A - biasA), 0, (int)(a.bytesA + biasA), 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrcB = __builtin_amdgcn_make_buffer_rsrc((void*)a.B, 0, (int)a.bytesB, 0x00020000);

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
    int swz = cpr >= 16 ? 4 * (k & 3) : 2 * (k & 3);
    return (lane % cpr) ^ swz;
  };

  // ---- per-thread loader state ---------------------------------------------------------------
  // vA / vB: byte offset of load ii that does not change over the k loop (OOB: the row or column does not exist);
  // invA: bit t set when filter tap t reads outside the image for this row (all bits set for rows beyond M).
  unsigned vA[LA], invA[LA], vB[LB];
  int ga1[LA], ga2[LA];  // GEN: the row's pixel coordinates, as the per-load arithmetic wants them
  (void)invA; (void)ga1; (void)ga2;
  if (OP != OP_BWD_WEIGHT && GEN) {  // A rows are pixels of the (n, OH, OW) grid
#pragma unroll
    for (int ii = 0; ii < LA; ++ii) {
      int m = m0 + NW * KC_RPI * ii + kc_row;
      vA[ii] = 0; ga1[ii] = -(1 << 28); ga2[ii] = -(1 << 28);
      if (m < a.M) {
        unsigned n = fd_div((unsigned)m, g.d_ohow);
        unsigned rem = (unsigned)m - n * (unsigned)(g.OH * g.OW);
        int oh = (int)fd_div(rem, g.d_ow);
        int ow = (int)rem - oh * g.OW;
        if (OP == OP_FWD) {
          ga1[ii] = oh * g.sh - g.ph;
          ga2[ii] = ow * g.sw - g.pw;
          vA[ii] = (unsigned)(((int)n * g.IH + ga1[ii]) * g.row_pitch + ga2[ii] * g.pix_step + kc_chunk * 8) * 2u;
        } else {
          vA[ii] = n * (unsigned)(g.IH * g.row_pitch);
          ga1[ii] = oh + g.ph;
          ga2[ii] = ow + g.pw;
        }
      }
    }
  } else if (OP != OP_BWD_WEIGHT) {
    // Row ii of a thread is pixel m0 + kc_row + STR * ii of the (n, OH, OW) grid.  The first one is decomposed by
    // division; the others follow by adding the stride's own decomposition STR = sa OH OW + sb OW + sc with one carry
    // per digit (sc < OW, sb < OH), and the byte offset follows by adding what those digit steps are worth: a
    // handful of additions and selects per row instead of two divisions and five multiplications.
    // Forward reads source pixel (oh sh - ph + r, ow sw - pw + s) for tap (r, s); backward-data (unit stride)
    // reads (oh + ph - r, ow + pw - s).
    constexpr unsigned STR = NW * KC_RPI;
    const int shh = OP == OP_FWD ? g.sh : 1, sww = OP == OP_FWD ? g.sw : 1;
    const int offh = OP == OP_FWD ? -g.ph : g.ph, offw = OP == OP_FWD ? -g.pw : g.pw;
    const int dir = OP == OP_FWD ? 1 : -1;
    const unsigned sa = fd_div(STR, g.d_ohow);
    const unsigned srem = STR - sa * (unsigned)(g.OH * g.OW);
    const int sb = (int)fd_div(srem, g.d_ow);
    const int sc = (int)srem - sb * g.OW;
    const unsigned Pn = (unsigned)(g.IH * g.row_pitch) * 2u;   // bytes per image, per source row step, per column step
    const unsigned Ph = (unsigned)(shh * g.row_pitch) * 2u;
    const unsigned Pw = (unsigned)(sww * g.pix_step) * 2u;
    const unsigned dV = sa * Pn + (unsigned)sb * Ph + (unsigned)sc * Pw;
    const unsigned k1 = Ph - (unsigned)g.OW * Pw;               // a carry out of the column digit
    const unsigned k2 = Pn - (unsigned)g.OH * Ph;               // a carry out of the row digit
    // a single unpadded tap is always inside, and so is every tap of a forward pass without padding
    // ((OH - 1) sh + R <= IH)
    const bool masks = g.ph != 0 || g.pw != 0 || (OP == OP_BWD_DATA && g.R * g.S > 1) || g.always_mask != 0;
    const unsigned full = g.S >= 32 ? OOB : (1u << g.S) - 1u;

    int m = m0 + kc_row;
    const unsigned n0img = fd_div((unsigned)m, g.d_ohow);
    const unsigned rem = (unsigned)m - n0img * (unsigned)(g.OH * g.OW);
    int oh = (int)fd_div(rem, g.d_ow);
    int ow = (int)rem - oh * g.OW;
    // offset of the pixel the per-tile scalar offset counts from: tap (0,0) for forward, tap (R-1,S-1) for
    // backward-data; forward adds the descriptor margin, which makes it non-negative
    unsigned v = (unsigned)(((int)n0img * g.IH + oh * shh + offh) * g.row_pitch + (ow * sww + offw) * g.pix_step + kc_chunk * 8) * 2u +
                 (OP == OP_FWD ? biasA : 0u);
#pragma unroll
    for (int ii = 0; ii < LA; ++ii) {
      if (ii > 0) {
        m += (int)STR;
        ow += sc;
        const bool c1 = ow >= g.OW;
        ow -= c1 ? g.OW : 0;
        oh += sb + (c1 ? 1 : 0);
        const bool c2 = oh >= g.OH;
        oh -= c2 ? g.OH : 0;
        v += dV + (c1 ? k1 : 0u) + (c2 ? k2 : 0u);
      }
      vA[ii] = 0; invA[ii] = OOB;
      if (m < a.M) {
        vA[ii] = v;
        unsigned inv = 0;
        if (masks) {
          // Along one axis the taps that fall outside are a run at the start and a run at the end of the filter:
          // position p0 + dir t is below 0 for the first `lo` taps and at or beyond the size from tap `hi` on
          // (dir = -1: the other way round).  Columns give a mask cm of S bits that is copied into every row's slot by
          // one multiplication (tap_rep has bit r S set for every r); rows that are outside fill their whole slots.
          const int ih0 = __mul24(oh, shh) + offh, iw0 = __mul24(ow, sww) + offw;
          const int lo_w = dir > 0 ? -iw0 : iw0 - g.IW + 1, hi_w = dir > 0 ? g.IW - iw0 : iw0 + 1;
          const int lo_h = dir > 0 ? -ih0 : ih0 - g.IH + 1, hi_h = dir > 0 ? g.IH - ih0 : ih0 + 1;
          const unsigned cm = low_bits(clamp_to(lo_w, g.S)) | (full & ~low_bits(clamp_to(hi_w, g.S)));
          inv = cm * g.tap_rep | low_bits(clamp_to(lo_h, g.R) * g.S) | (low_bits(g.R * g.S) & ~low_bits(clamp_to(hi_h, g.R) * g.S));
        }
        invA[ii] = inv;
      }
    }
  }
  int sb1 = 0, sb2 = 0, sbc = 0;
  (void)sb1; (void)sb2; (void)sbc;
  // backward-weight, gathered x: per load the pixel's row and column and the byte offset of its tap, advanced per tile
  int xp[LB], xq[LB], bw_tp = 0, bw_tq = 0;
  unsigned xoff[LB], bw_dv = 0, bw_k1 = 0, bw_k2 = 0;
  (void)xp; (void)xq; (void)xoff; (void)bw_tp; (void)bw_tq; (void)bw_dv; (void)bw_k1; (void)bw_k2;
  if (OP == OP_FWD) {
#pragma unroll
    for (int ii = 0; ii < LB; ++ii) {
      int nn = n0 + NW * KC_RPI * ii + kc_row;
      vB[ii] = nn < a.N ? (unsigned)(nn * a.Kred + kc_chunk * 8) * 2u : OOB;
    }
  } else if (OP == OP_BWD_DATA) {
    // filter w[ko][tap][c]: k-row = ko (within the tap), chunk = 8 consecutive c
#pragma unroll
    for (int ii = 0; ii < LB; ++ii) {
      int k = mc_k(BN, ii);
      int nn = n0 + mc_chunk(BN, k) * 8;
      vB[ii] = nn < a.N ? (unsigned)((k * g.R * g.S) * a.N + nn) * 2u : OOB;  // + (c0 * R * S + tap) * N * 2 per tile
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
    // 1x1, unit stride, no padding: pixel j of x is row j of a plain [Kred][IC] matrix, so the load needs no pixel
    // arithmetic at all (per-lane offset fixed, per-tile offset scalar)
#pragma unroll
    for (int ii = 0; ii < LB; ++ii) vB[ii] = (a.bw_linear && nn < a.N) ? (unsigned)(mc_k(BN, ii) * g.IC + nn) * 2u : OOB;
    // Any other layer: load ii of k tile kt reads, for output pixel j = kt TBK + k-row, the input pixel at this lane's
    // tap.  The pixel of the first tile is decomposed by division here; from tile to tile j grows by TBK, so its
    // (image, row, column) digits and the byte offset advance by TBK's own digits with one carry each (as the rows
    // of the gathered operand do in the other two passes): no division and no slow multiplication inside the k loop.
    if (!a.bw_linear) {
      const unsigned ta = fd_div((unsigned)TBK, g.d_ohow);
      const unsigned trem = (unsigned)TBK - ta * (unsigned)(g.OH * g.OW);
      bw_tp = (int)fd_div(trem, g.d_ow);
      bw_tq = (int)trem - bw_tp * g.OW;
      const unsigned Pn = (unsigned)(g.IH * g.row_pitch) * 2u, Ph = (unsigned)(g.sh * g.row_pitch) * 2u,
                     Pw = (unsigned)(g.sw * g.pix_step) * 2u;
      bw_dv = ta * Pn + (unsigned)bw_tp * Ph + (unsigned)bw_tq * Pw;
      bw_k1 = Ph - (unsigned)g.OW * Pw;
      bw_k2 = Pn - (unsigned)g.OH * Ph;
#pragma unroll
      for (int ii = 0; ii < LB; ++ii) {
        const unsigned j = (unsigned)(kt_begin * TBK + mc_k(BN, ii));
        const unsigned n = fd_div(j, g.d_ohow);
        const unsigned rem = j - n * (unsigned)(g.OH * g.OW);
        const unsigned pp = fd_div(rem, g.d_ow);
        xp[ii] = (int)pp;
        xq[ii] = (int)(rem - pp * (unsigned)g.OW);
        xoff[ii] = ((n * (unsigned)g.IH + pp * (unsigned)g.sh + (unsigned)sb1) * (unsigned)g.row_pitch +
                    ((unsigned)(xq[ii] * g.sw) + (unsigned)sb2) * (unsigned)g.pix_step + (unsigned)sbc) * 2u;
      }
    }
    // dy[(n,p,q)][k_out], chunk = 8 consecutive k_out: row j = k0 + k of the tile at (mm + j M) * 2
    int mm = m0 + mc_chunk(BM, mc_k(BM, 0)) * 8;
#pragma unroll
    for (int ii = 0; ii < LA; ++ii) vA[ii] = mm < a.M ? (unsigned)(mm + mc_k(BM, ii) * a.M) * 2u : OOB;
  }

  // Requesting k tile kt into ring stage st = LPT loads per thread (LA for A, then LB for B), spread over the MFMA
  // slots of the tile being multiplied.  TileCtx holds what is the same for the whole wavefront.
  struct TileCtx {
    int k0, c0, r, s;
    unsigned tap, soffA, soffB;
    unsigned rag;  // per lane: -1 when this lane's chunk of a ragged last k tile lies beyond the channel count
  };
  auto tile_ctx = [&](int kt) {
    TileCtx c;
    c.k0 = kt * TBK;
    c.tap = 0; c.c0 = 0; c.r = 0; c.s = 0; c.soffA = 0; c.soffB = 0; c.rag = 0;
    // the whole tile lies inside one filter tap: wave-uniform values.  Either IC % TBK == 0, or there is only one tap
    // (1x1 layers, fully connected) and the last tile is ragged: chunks at or beyond IC are then not requested.
    if (OP != OP_BWD_WEIGHT) {
      c.tap = fd_div((unsigned)c.k0, g.d_ic);
      c.c0 = c.k0 - (int)c.tap * g.IC;
      c.r = (int)fd_div(c.tap, g.d_s);
      c.s = (int)c.tap - c.r * g.S;
      if (GEN) {
        c.soffA = (unsigned)(c.r * g.row_pitch + c.s * g.s_step + c.c0) * 2u;  // forward only
      } else if (OP == OP_FWD) {
        c.soffA = (unsigned)(c.r * g.row_pitch + c.s * g.s_step + c.c0) * 2u;
      } else {
        c.soffA = (unsigned)((g.R - 1 - c.r) * g.row_pitch + (g.S - 1 - c.s) * g.pix_step + c.c0) * 2u;
      }
      c.soffB = OP == OP_FWD ? (unsigned)c.k0 * 2u : (unsigned)((c.c0 * g.R * g.S + (int)c.tap) * a.N) * 2u;
      c.rag = c.c0 + kc_chunk * 8 < g.IC ? 0u : OOB;
    } else {
      c.soffA = (unsigned)(c.k0 * a.M) * 2u;
      c.soffB = (unsigned)(c.k0 * g.IC) * 2u;  // used by the plain-matrix case only
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
        lds_byte* dst = sA + (NW * ii + wave) * 1024;
        if constexpr (GEN && OP == OP_FWD) {
          int ih = ga1[ii] + c.r, iw = ga2[ii] + c.s;
          bool ok = (unsigned)ih < (unsigned)g.IH && (unsigned)iw < (unsigned)g.IW;
          jz_dma16(rsrcA, dst, ok ? (vA[ii] + c.soffA) | c.rag : OOB);
        } else if constexpr (GEN && OP == OP_BWD_DATA) {
          // input pixel (h,w) receives from output pixel ((h + pad - r) / stride, ...) when the division is exact
          int th = ga1[ii] - c.r, tw = ga2[ii] - c.s;
          int ih = (int)fd_div((unsigned)(th < 0 ? 0 : th), g.d_sh);
          int iw = (int)fd_div((unsigned)(tw < 0 ? 0 : tw), g.d_sw);
          bool ok = ih * g.sh == th && iw * g.sw == tw && ih < g.IH && iw < g.IW;  // false for negative th / tw too
          unsigned off = (vA[ii] + (unsigned)(ih * g.row_pitch + iw * g.pix_step + c.c0 + kc_chunk * 8)) * 2u;
          jz_dma16(rsrcA, dst, ok ? off | c.rag : OOB);
        } else if constexpr (OP != OP_BWD_WEIGHT) {
          // bit `tap` of the row's mask -> 0 / -1; an offset of -1 is outside every descriptor
          const unsigned bad = (unsigned)__builtin_amdgcn_sbfe(invA[ii], c.tap, 1);
          jz_dma16s(rsrcA, dst, vA[ii] | bad | c.rag, c.soffA);
        } else {  // dy rows j = k0 + k; rows at or beyond the reduction length are not requested
          const bool ok = c.k0 + mc_k(BM, ii) < a.Kred;
          jz_dma16s(rsrcA, dst, ok ? vA[ii] : OOB, c.soffA);
        }
      } else {
        constexpr int ii = Lidx - LA;
        lds_byte* dst = sB + (NW * ii + wave) * 1024;
        if constexpr (OP == OP_FWD) {
          jz_dma16s(rsrcB, dst, vB[ii] | c.rag, c.soffB);
        } else if constexpr (OP == OP_BWD_DATA) {
          const bool ok = c.c0 + mc_k(BN, ii) < g.IC;
          jz_dma16s(rsrcB, dst, ok ? vB[ii] : OOB, c.soffB);
        } else if (a.bw_linear) {  // x rows j = k0 + k of a plain matrix
          const bool ok = c.k0 + mc_k(BN, ii) < a.Kred;
          jz_dma16s(rsrcB, dst, ok ? vB[ii] : OOB, c.soffB);
        } else {  // x at this lane's tap for output pixel j = k0 + k-row
          const int ih = __mul24(xp[ii], g.sh) + sb1, iw = __mul24(xq[ii], g.sw) + sb2;
          const bool ok = c.k0 + mc_k(BN, ii) < a.Kred && (unsigned)ih < (unsigned)g.IH && (unsigned)iw < (unsigned)g.IW;
          jz_dma16(rsrcB, dst, ok ? xoff[ii] : OOB);
          // on to the pixel of the next tile
          xq[ii] += bw_tq;
          const bool c1 = xq[ii] >= g.OW;
          xq[ii] -= c1 ? g.OW : 0;
          xp[ii] += bw_tp + (c1 ? 1 : 0);
          const bool c2 = xp[ii] >= g.OH;
          xp[ii] -= c2 ? g.OH : 0;
          xoff[ii] += bw_dv + (c1 ? bw_k1 : 0u) + (c2 ? bw_k2 : 0u);
        }
      }
    }
  };
  static_assert(NST >= 3 && NST <= 8 && (NST - 2) * LPT <= 63, "ring depth: vmcnt is a 6-bit counter");
  auto issue = [&](int kt, int st) {  // all loads of a tile at once (prologue)
    TileCtx c = tile_ctx(kt);
    static_for<0, LPT>([&](auto l) { issue_load(c, st, l); });
  };

  // the first NST-1 tiles are requested before anything else is set up: their round trip to memory is the longest
  // latency of the prologue, and the accumulator and read-address set-up below fits into it
#pragma unroll
  for (int s = 0; s < NST - 1; ++s)
    if (s < nk) issue(kt_begin + s, s);
  sched_fence();

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
          int swz = CPR >= 16 ? 4 * (k & 3) : 2 * (k & 3);
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
          int swz = CPR >= 16 ? 4 * (k & 3) : 2 * (k & 3);
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
    if constexpr (A_KC) {
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
    if constexpr (B_KC) {
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
  // wait until at most KEEP LDS reads are outstanding and tie the operands of the coming MFMAs to that point
  auto settle = [&](auto keep_tag, auto ks_tag, half8 (&fa)[TM], half8 (&fb)[TN]) {
    constexpr int KEEP = decltype(keep_tag)::value;
    lds_wait<KEEP>();
#pragma unroll
    for (int t = 0; t < TM; ++t) lds_pin(fa[t]);
#pragma unroll
    for (int t = 0; t < TN; ++t) lds_pin(fb[t]);
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
  // One iteration multiplies tile i out of stage i % NST, k step by k step (NKS groups of G MFMAs).  The operands of
  // a k step are read two steps ahead, right after the last MFMA of the group that used the same registers, so an
  // LDS round trip has a whole group of MFMAs to hide behind:
  //
  //   group ks:  wait for the reads of step ks ; MFMA 0 ; [loads] ; MFMA 1 ; [loads] ; ... ; MFMA G-1 ;
  //              (ks == NKS-2: wait until tile i+1 has landed and my reads of tile i are complete ; BARRIER)
  //              read step ks+2 (of tile i+1 when ks+2 >= NKS) into the registers this group multiplied from
  //
  // The barrier says two things: every wavefront's share of tile i+1 is in LDS, and every wavefront holds the whole of
  // tile i in registers, so stage i % NST may be overwritten by the loads requested in the next iteration.  Barriers
  // are bare (no fence): a fenced barrier makes the compiler drain every LDS-direct load first (vmcnt(0)); the
  // ordering that matters is spelled out by hand with vmcnt / lgkmcnt waits.
  //
  // Loads of tile i+NST-1: load l goes behind MFMA slot l * NSL / LPT of the NSL = NKS * max(G-1, 1) slots that carry
  // no LDS reads.  LBAR of them are issued before the barrier of the iteration, the rest after it.
  constexpr int SPG = G > 1 ? G - 1 : 1;   // load slots per group
  constexpr int NSL = NKS * SPG;
  constexpr int LBAR = []() constexpr {
    int n = 0;
    for (int l = 0; l < LPT; ++l) n += ((l * NSL / LPT) / SPG <= NKS - 2) ? 1 : 0;
    return n;
  }();
  static_assert((NST - 3) * LPT + LBAR <= 63 && (NST - 3) * LPT + LBAR >= 0, "vmcnt range");
  half8 fa0[TM], fb0[TN], fa1[TM], fb1[TN];
  // STEADY: request tile c into stage ist while multiplying; has_next: there is a tile after this one
  auto iteration = [&](int st, auto steady_tag, const TileCtx& c, int ist, bool has_next, int younger_after_next) {
    constexpr bool ISSUE = decltype(steady_tag)::value;
    const unsigned sb = lds_base + (unsigned)(st * STAGE);
    const unsigned sb_next = lds_base + (unsigned)(((st + 1) % NST) * STAGE);
    static_for<0, NKS>([&](auto ks_tag) {
      constexpr int KS = decltype(ks_tag)::value;
      half8(&fa)[TM] = (KS % 2 == 0) ? fa0 : fa1;
      half8(&fb)[TN] = (KS % 2 == 0) ? fb0 : fb1;
      // steady state: the reads of the following step (READS of them) may still be in flight; while draining the
      // following step may not have been requested, so wait for everything
      if constexpr (ISSUE) settle(std::integral_constant<int, READS>{}, ks_tag, fa, fb);
      else settle(std::integral_constant<int, 0>{}, ks_tag, fa, fb);
      sched_fence();
      static_for<0, G>([&](auto q_tag) {
        constexpr int Q = decltype(q_tag)::value;
        constexpr int I = Q / TN, J = Q % TN;
        // n operand in the first slot: each lane then owns 4 consecutive n for one m (row = lane % 32)
        acc[I][J] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fb[J], fa[I], acc[I][J], 0, 0, 0);
        sched_fence();
        if constexpr (ISSUE && (Q < G - 1 || G == 1)) {
          static_for<0, LPT>([&](auto l_tag) {
            constexpr int Lx = decltype(l_tag)::value;
            if constexpr ((Lx * NSL / LPT) / SPG == KS && (Lx * NSL / LPT) % SPG == Q) issue_load(c, ist, l_tag);
          });
          sched_fence();
        }
      });
      if constexpr (KS + 2 < NKS) {
        read_frags(sb, std::integral_constant<int, (KS + 2 < NKS ? KS + 2 : 0)>{}, fa, fb);
      } else {
        if (ISSUE || has_next) {
          if constexpr (KS == NKS - 2) {
            lds_wait<0>();  // the whole of this tile is in registers
            if (ISSUE) wait_vmcnt<(NST - 3) * LPT + LBAR>();
            else wait_tiles(younger_after_next);
            __builtin_amdgcn_s_barrier();
          }
          read_frags(sb_next, std::integral_constant<int, (KS + 2 >= NKS ? KS + 2 - NKS : 0)>{}, fa, fb);
        }
      }
      sched_fence();
    });
  };

  if (nk > 0) {
    wait_tiles(nk - 1);
    __builtin_amdgcn_s_barrier();
    read_frags(lds_base, std::integral_constant<int, 0>{}, fa0, fb0);
    read_frags(lds_base, std::integral_constant<int, 1>{}, fa1, fb1);
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

  constexpr int ring_bytes = NST * STAGE, epi_bytes = BM / dma_epass(BM, BN) * (BN + 8) * 2;
  igemm_epilogue_impl<BM, BN, TM, TN, NT, dma_epass(BM, BN), (ring_bytes > epi_bytes ? ring_bytes : epi_bytes), STATS>(
      a, acc, lds, m0, n0, split, tid, lane, wm * WTM, wn * WTN);
}
