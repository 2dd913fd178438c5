// FP16-storage / FP32-accumulate convolution forward, backward-data, backward-weight and the fully
// connected GEMMs (Jia et al. 2018, Section 4.1) as one implicit-GEMM kernel family for gfx950.
//
// This file holds the host side: the planner (tile shape, split of the reduction, which kernel), argument checks, the
// extern "C" entry points, and the small helper kernels (split-K reduction, the 4-channel padded copy for 3-channel
// stems).  The GEMM kernels and their epilogue are in jz_igemm_kernels.h / jz_igemm_dma.h, instantiated in one
// translation unit per operation (jz_conv_fwd.hip, ...).
#include <stdio.h>
#include <stdlib.h>

#include <mutex>
#include <type_traits>
#include <vector>

#include "jz_conv_plan.h"
#include "jz_sumsq.h"

namespace {
using namespace jz;

constexpr int BK = 64;  // k tile depth of the element-wise kernel

// ---------------------------------------------------------------------------------------------
// small-channel layers (C <= 4: the 3-channel stems of ResNet-50 and AlexNet)
// ---------------------------------------------------------------------------------------------
// With 3 channels a filter tap is 6 bytes: nothing to vectorise.  But in NHWC the S taps of one filter row are
// adjacent in memory, so the input is copied once into a zero-padded 4-channel image xp[N][H+2ph][Wp][4]; one filter
// row of an output pixel is then ONE contiguous, 16-byte aligned run of 4*S halves starting at pixel q*stride_w
// (needs an even stride_w), and the layer becomes an ordinary implicit GEMM whose "taps" are the R filter rows and
// whose "channels" are that run, rounded up to the k tile (32 or 64; backward-weight, where the runs are columns of the
// GEMM: to whole 16-byte chunks).  The filter is repacked to match
// (w'[k][r][4 s + c], zeros elsewhere); for backward-weight the GEMM produces dw' in that layout and the real
// entries are copied out.

// One launch does both copies.  Slices z < N of the grid: a workgroup of 128 threads covers 256 padded pixels of the
// PAD_ROWS image rows (z, PAD_ROWS y ...), two pixels per thread and row (one 16-byte store; Wp is even).  Slice z = N (present when wp != nullptr) repacks the
// filter: w[K][R][S][C] -> wp[K][R][KT] with wp[k][r][4 s + c] = w[k][r][s][c], zero elsewhere.
constexpr int PAD_ROWS = 4;
__global__ __launch_bounds__(128) void pad_to_c4(const unsigned short* __restrict__ x, unsigned short* __restrict__ xp,
                                                 int N, int H, int W, int C, int Hp, int Wp, int ph, int pw,
                                                 const unsigned short* __restrict__ w, unsigned short* __restrict__ wp,
                                                 int K, int R, int S, int KT, int chunk_major) {
  const int z = blockIdx.z;
  if (z == N) {
    const int total = K * R * KT;
    const int stride = gridDim.x * gridDim.y * 128;
    for (int i = (blockIdx.y * gridDim.x + blockIdx.x) * 128 + threadIdx.x; i < total; i += stride) {
      int j = i % KT, kr = i / KT;
      int s = j >> 2, c = j & 3;
      // chunk_major (the patch kernel's layout): wq[r][j / 8][k][j % 8], 16-byte chunks of one filter row side by side per k
      const int k = kr / R, r = kr - k * R;
      const int dst = chunk_major ? ((r * (KT / 8) + (j >> 3)) * K + k) * 8 + (j & 7) : i;
      wp[dst] = (s < S && c < C) ? w[((size_t)kr * S + s) * C + c] : (unsigned short)0;
    }
    return;
  }
  // PAD_ROWS image rows per workgroup: every load of a thread's rows is in flight before the first store
  const int wp0 = 2 * (blockIdx.x * 128 + threadIdx.x);
  if (wp0 >= Wp) return;
  unsigned short v[PAD_ROWS][8];
#pragma unroll
  for (int rr = 0; rr < PAD_ROWS; ++rr) {
    const int hp = blockIdx.y * PAD_ROWS + rr;
    const int h = hp - ph;
#pragma unroll
    for (int e = 0; e < 8; ++e) v[rr][e] = 0;
    if (hp < Hp && (unsigned)h < (unsigned)H) {
      const unsigned short* row = x + ((size_t)z * H + h) * W * C;
#pragma unroll
      for (int p = 0; p < 2; ++p) {
        const int wi = wp0 + p - pw;
        if ((unsigned)wi < (unsigned)W) {
#pragma unroll
          for (int c = 0; c < 4; ++c)
            if (c < C) v[rr][4 * p + c] = row[(size_t)wi * C + c];
        }
      }
    }
  }
#pragma unroll
  for (int rr = 0; rr < PAD_ROWS; ++rr) {
    const int hp = blockIdx.y * PAD_ROWS + rr;
    if (hp >= Hp) break;
    uint4 pk = make_uint4((unsigned)v[rr][0] | ((unsigned)v[rr][1] << 16), (unsigned)v[rr][2] | ((unsigned)v[rr][3] << 16),
                          (unsigned)v[rr][4] | ((unsigned)v[rr][5] << 16), (unsigned)v[rr][6] | ((unsigned)v[rr][7] << 16));
    *reinterpret_cast<uint4*>(xp + (((size_t)z * Hp + hp) * Wp + wp0) * 4) = pk;
  }
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
  // 16-byte loads need every split's slab to start on a 16-byte boundary: MN a multiple of 4
  const bool full = i + 3 < MN && (MN & 3) == 0;
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

// splitk_reduce that also leaves the sum of squares of the FP16 values it writes (and whether any of them is Inf / NaN)
// in a sink: the weight gradient's norm for Eq. 1, taken while the gradient is still in registers.  Same sums, same order,
// same bits in `out` as splitk_reduce.  A workgroup walks several slabs of outputs (grid stride) and contributes once, so
// that the number of atomic additions per tensor stays in the hundreds.
__global__ __launch_bounds__(256) void splitk_reduce_sumsq(const float* __restrict__ part, unsigned short* __restrict__ out,
                                                           long long MN, int splits, int lg, int KT4, int S, int C,
                                                           long long slabs, jz::SumsqSink sink) {
  __shared__ float4 red[256];
  __shared__ unsigned long long wsum[5];
  if (threadIdx.x < 5) wsum[threadIdx.x] = 0ull;
  __syncthreads();
  const int G = 1 << lg, Q = 256 >> lg;
  const int q = threadIdx.x & (Q - 1), g = threadIdx.x >> (8 - lg);
  jz::SumsqAcc sq;
  int bad = 0;
  for (long long slab = blockIdx.x; slab < slabs; slab += gridDim.x) {
    const long long i = (slab * Q + q) * 4;
    const bool full = i + 3 < MN && (MN & 3) == 0;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i < MN) {
      if (full) {
        int k = g;
        for (; k + 3 * G < splits; k += 4 * G) {
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
      } else {
        float* sv = reinterpret_cast<float*>(&s);
        for (int k = g; k < splits; k += G)
          for (int e = 0; e < 4 && i + e < MN; ++e) sv[e] += part[(size_t)k * MN + i + e];
      }
    }
    if (G > 1) {
      __syncthreads();  // the previous slab's sums have been read
      red[threadIdx.x] = s;
      __syncthreads();
      if (g == 0)
        for (int gg = 1; gg < G; ++gg) {
          float4 t = red[gg * Q + q];
          s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
        }
    }
    if (g != 0 || i >= MN) continue;
    _Float16 h[4] = {(_Float16)s.x, (_Float16)s.y, (_Float16)s.z, (_Float16)s.w};
    unsigned short hb[4];
    __builtin_memcpy(hb, h, 8);
    int nst = 0;  // how many of the four are real outputs
    if (KT4 > 0) {
      const long long grp = i >> 2, kr = grp / KT4;
      const int sx = (int)(grp - kr * KT4);
      if (sx < S) {
        nst = C < 4 ? C : 4;
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if (c < C) out[(kr * S + sx) * C + c] = hb[c];
      }
    } else if (full) {
      nst = 4;
      uint2 pk;
      __builtin_memcpy(&pk, h, 8);
      *reinterpret_cast<uint2*>(out + i) = pk;
    } else {
      for (int e = 0; e < 4 && i + e < MN; ++e) {
        out[i + e] = hb[e];
        nst = e + 1;
      }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (e < nst) bad |= jz::sumsq_acc_add(sq, hb[e]);
  }
  jz::sumsq_block_flush(sq, bad, sink, blockIdx.x, wsum);
}

// sum of squares of n FP16 values into a sink (gradients whose producing kernel has no fused form)
__global__ __launch_bounds__(256) void sumsq_half(const unsigned short* __restrict__ g16, long long n, jz::SumsqSink sink) {
  __shared__ unsigned long long wsum[5];
  if (threadIdx.x < 5) wsum[threadIdx.x] = 0ull;
  __syncthreads();
  jz::SumsqAcc sq;
  int bad = 0;
  const long long groups = n >> 3;  // 16-byte groups; g16 is 16-byte aligned
  for (long long j = (long long)blockIdx.x * 256 + threadIdx.x; j < groups; j += (long long)gridDim.x * 256) {
    const uint4 v = *reinterpret_cast<const uint4*>(g16 + j * 8);
    const unsigned wv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 8; ++e) bad |= jz::sumsq_acc_add(sq, (unsigned short)(wv[e >> 1] >> ((e & 1) * 16)));
  }
  if (blockIdx.x == 0) {  // the tail, at most 7 elements
    const long long i = (groups << 3) + threadIdx.x;
    if (i < n) bad |= jz::sumsq_acc_add(sq, g16[i]);
  }
  jz::sumsq_block_flush(sq, bad, sink, blockIdx.x, wsum);
}

// ---------------------------------------------------------------------------------------------
// host side: plan (tile shape, fast/generic, split-K) and launch
// ---------------------------------------------------------------------------------------------
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
constexpr int kMaxClasses = 16;  // parity classes of a stride (sh * sw) the backward-data decomposition handles

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
#include "jz_tuned_resnet50_v15.inc"
    // the 3-channel stem of ResNet-50 at batch 64 on its padded 4-channel copy ("taps" = the 7 filter rows), measured
    // the same way: forward 62.8 us (what the fused convolution + batch-norm call runs; the plain forward call takes the
    // patch kernel), backward-weight 67.0 us including the copy
    {0, 802816, 64, 224, 7, 0, 128, 64, 32, 4, 3, 1},
    {2, 64, 224, 802816, 7, 0, 64, 64, 32, 4, 4, 256},
    // backward-weight of the 11x11 stride-4 stem at batch 128, chosen inside the AlexNet step (tune.py --model alexnet --in-place)
    {2, 96, 528, 387200, 11, 0, 128, 128, 32, 4, 3, 128},
};

// Choices set at run time through jz_conv2d_tune_set: looked up before the table above (an in-place tuning run tries
// candidates this way without rebuilding the library).  g_use_table: whether the table above is consulted at all
// (jz_conv2d_tune_use_table; the cost model alone is what an unknown shape gets).
std::mutex g_tune_mutex;
std::vector<Tuned> g_tune_rt;
bool g_use_table = true;

bool same_key(const Tuned& x, const Tuned& y) {
  return x.op == y.op && x.M == y.M && x.N == y.N && x.K == y.K && x.taps == y.taps && x.scatter == y.scatter;
}

// bk64_ok: the 64-deep k tile is usable for this layer; forced_bk: the k tile depth is fixed (register path, packed mode)
void choose_tiling(Plan* pl, bool bk64_ok, int forced_bk) {
  GemmArgs& a = pl->args;
  static const int split_opts[] = {1, 2, 3, 4, 6, 8, 12, 16, 24, 32, 48, 64, 96, 128, 192, 256, 384, 512};
  const int oi = pl->op == JZ_FWD ? 0 : pl->op == JZ_BWD_DATA ? 1 : 2;
  double best = 1e30;
  const Variant* bv = &kVariants[0];
  int bS = 1;
  if (!pl->fast) forced_bk = BK;  // the element-wise kernel: one shape (the first variant's), 64-deep tiles, ~8x slower
  const Tuned* hit = nullptr;
  Tuned rt_hit{};
  if (pl->fast && (!forced_bk || pl->packed)) {
    const Tuned key{oi, a.M, a.N, a.Kred, a.g.R * a.g.S, a.sc_on, 0, 0, 0, 0, 0, 0};
    auto usable = [&](const Tuned& t) {
      if (pl->gen && (t.waves != 4 || t.bk != 32 || t.nst != 4)) return false;  // the only kernels of that mode
      return same_key(t, key) && (forced_bk ? t.bk == forced_bk : (t.bk == 32 || bk64_ok));
    };
    bool use_table;
    {
      std::lock_guard<std::mutex> lock(g_tune_mutex);
      use_table = g_use_table;
      for (const Tuned& t : g_tune_rt)
        if (usable(t)) {
          rt_hit = t;
          hit = &rt_hit;
          pl->rt_forced = true;
          break;
        }
    }
    if (!hit && use_table && !pl->gen)
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
      if (v.nst == 3 && v.bk == 32) continue;  // short rings: from the table of measured choices or on request only
      if (v.waves == 8 && v.BM == 128 && v.bk == 32) continue;  // likewise (the model has no fit for it)
      const int vbk = forced_bk ? forced_bk : v.bk;
      if (v.nst == 3 && vbk != 32) continue;  // the short rings exist for 32-deep tiles
      const int nkt = (a.Kred + vbk - 1) / vbk;
      long long tm = (a.M + v.BM - 1) / v.BM, tn = (a.N + v.BN - 1) / v.BN;
      for (int sp : split_opts) {
        if (sp > 1 && nkt / sp < 4) break;
        if (a.sc_on && sp > 1) break;  // the scatter lives in the fp16 epilogue
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

// The patch kernel's view of a packed forward layer (jz_conv_stem.hip); false: the layer stays on the implicit-GEMM kernel
// (output channels not a multiple of 32 or more than 128, filter + patch larger than the LDS).
bool stem_fwd_setup(const Plan& pl, const jz_conv_desc* d, StemArgs* sa) {
  if (!pl.packed || pl.op != JZ_FWD || d->K % 32 != 0 || d->K > 128) return false;
  const int P = out_dim(d->H, d->pad_h, d->R, d->stride_h), Q = out_dim(d->W, d->pad_w, d->S, d->stride_w);
  StemArgs a;
  a.NT = d->K / 32;
  a.NKS = (4 * d->S + 15) / 16;
  const int TM = stem_fwd_tm(a.NT);
  if (TM == 0 || a.NKS < 1 || a.NKS > 4 || a.NKS * 16 > pl.KT) return false;
  const int MB = 4 * TM * 32;
  a.N = d->N; a.Hp = pl.Hp; a.Wp = pl.Wp; a.P = P; a.Q = Q; a.R = d->R; a.sh = d->stride_h; a.sw = d->stride_w;
  a.xp_bytes = (unsigned)((size_t)d->N * pl.Hp * pl.Wp * 8);
  a.wq_bytes = (unsigned)((size_t)d->R * a.NKS * 2 * d->K * 16);
  if (a.wq_bytes > pl.wp_bytes) return false;
  // output rows that MB consecutive pixels can touch, and the input rows under them
  long long rows = ((long long)MB + Q - 2) / Q + 1;
  if (rows > P) rows = P;
  const size_t patch = (size_t)((rows - 1) * d->stride_h + d->R) * pl.Wp * 8;
  const size_t staging = (size_t)4 * 32 * (d->K * 2 + 16);
  const size_t lds_p = ((patch > staging ? patch : staging) + 4095) & ~size_t(4095);
  const size_t lds_w = ((size_t)a.wq_bytes + 4095) & ~size_t(4095);
  if (lds_w + lds_p > 160 * 1024) return false;
  a.lds_w_bytes = (unsigned)lds_w;
  a.lds_p_bytes = (unsigned)lds_p;
  a.blocks_per_image = (P * Q + MB - 1) / MB;
  const long long total = (long long)d->N * a.blocks_per_image;
  if (total > 0x7fffffff) return false;
  a.total_blocks = (int)total;
  // workgroups per compute unit: what the LDS and the instance's register budget allow
  const long long fit = (long long)((160 * 1024) / (lds_w + lds_p));
  const long long slots = 256 * (fit < stem_fwd_wgs(a.NT) ? fit : (long long)stem_fwd_wgs(a.NT));
  a.grid = (int)(total < slots ? total : slots);
  *sa = a;
  return true;
}

void plan_text(const Plan& pl, char* buf, size_t n) {
  const GemmArgs& a = pl.args;
  if (pl.stem) {
    const int mb = 128 * stem_fwd_tm(a.N / 32);
    snprintf(buf, n, "op %d M %d N %d K %d: patch kernel, %d pixels x %d channels per block, %d blocks per image, filter resident in LDS, "
             "4 wavefronts, 4-channel padded copy", pl.op, a.M, a.N, a.Kred, mb, a.N, (a.g.OH * a.g.OW + mb - 1) / mb);
    return;
  }
  snprintf(buf, n, "op %d M %d N %d K %d: %s tile %dx%dx%d, %d wavefronts, ring %d, %d x %d tiles, %d splits of %d k tiles%s%s", pl.op, a.M,
           a.N, a.Kred, pl.fast ? "vector" : "element-wise", pl.BM, pl.BN, pl.bk, pl.fast ? pl.waves : 4,
           pl.fast ? pl.nst : 2, a.tiles_m, a.tiles_n,
           a.splits, a.kt_per_split, pl.packed ? ", 4-channel padded copy" : "",
           a.sc_on ? ", scatter epilogue" : pl.classes ? ", one launch per parity class of the stride" : pl.gen ? ", per-load tap arithmetic" : "");
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
  // Byte offsets are formed in unsigned 32-bit integers, 0xffffffff marks "out of range" and is OR-ed into live
  // offsets, and a gathered operand's descriptor is widened by a margin smaller than the tensor: with at most 2^30 - 1
  // elements (2^31 - 2 bytes) per tensor every live offset, and every descriptor size, stays below 2^32 - 1.
  const long long lim = (1ll << 30) - 1;
  const long long nx = (long long)d->N * d->H * d->W * d->C, ny = (long long)d->N * P * Q * d->K,
                  nw = (long long)d->K * d->R * d->S * d->C;
  if (nx > lim || ny > lim || nw > lim) return JZ_ERR_UNSUPPORTED;
  if ((long long)d->N * P * Q > lim / 2 || (long long)d->N * d->H * d->W > lim / 2) return JZ_ERR_UNSUPPORTED;

  GemmArgs& a = pl->args;
  ConvGeom& g = a.g;
  pl->op = op;
  // k tile depth for the applicability checks: the LDS-direct kernels come 32 and 64 deep (chosen by the planner when
  // the layer allows both; 32 lets two workgroups share a compute unit)
  int bk = 32;
  bool bk64_ok = true;
  int forced_bk = 0;
  g.R = d->R; g.S = d->S; g.sh = d->stride_h; g.sw = d->stride_w; g.ph = d->pad_h; g.pw = d->pad_w;
  g.kvalid = 0;
  // a single filter tap: the reduction is one contiguous channel run, whose ragged last k tile the vector kernel can mask
  const bool one_tap = d->R == 1 && d->S == 1;
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
  a.sc_on = 0; a.sc_H = a.sc_W = 0; a.sc_sh = a.sc_sw = 1; a.sc_oh = a.sc_ow = 0; a.sc_fill = 0;
  g.always_mask = 0;
  a.bw_linear = (op == JZ_BWD_WEIGHT && d->R == 1 && d->S == 1 && d->stride_h == 1 && d->stride_w == 1 && d->pad_h == 0 &&
                 d->pad_w == 0) ? 1 : 0;
  if (op == JZ_BWD_DATA && pl->fast && d->R == 1 && d->S == 1 && d->pad_h == 0 && d->pad_w == 0 &&
      (d->stride_h > 1 || d->stride_w > 1)) {
    // strided 1x1 layer (the ResNet downsampling convs): only input pixels (p*sh, q*sw) receive gradient, so the GEMM
    // runs over the N*P*Q output pixels as a stride-1 problem and the epilogue scatters its rows (and the zeros)
    a.M = d->N * P * Q;
    g.OH = P; g.OW = Q; g.sh = 1; g.sw = 1;
    a.sc_on = 1; a.sc_H = d->H; a.sc_W = d->W; a.sc_sh = d->stride_h; a.sc_sw = d->stride_w; a.sc_fill = 1;
  }
  g.row_pitch = g.IW * g.IC;
  g.pix_step = g.IC;
  g.s_step = g.IC;

  // small-channel layers: gather from a zero-padded 4-channel copy (see pad_to_c4)
  if (!pl->fast && op != JZ_BWD_DATA && d->C <= 4 && d->stride_w % 2 == 0 && 4 * d->S <= 64 &&
      d->R <= 32 && (op == JZ_FWD || d->K % 8 == 0)) {
    // forward: the run of a filter row is one k tile (32 or 64 halves); backward-weight: the runs are columns of the
    // GEMM, whole 16-byte chunks suffice (an 11-tap row: 48 columns instead of 64, a quarter fewer columns to compute)
    const int KT = op == JZ_BWD_WEIGHT ? (4 * d->S + 7) & ~7 : 4 * d->S <= 32 ? 32 : 64;
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
  choose_tiling(pl, bk64_ok, forced_bk);
  if (pl->packed && op == JZ_FWD && !pl->rt_forced) {
    StemArgs sa;
    pl->stem = stem_fwd_setup(*pl, d, &sa);
  }
  const size_t part = a.splits > 1 ? (size_t)a.splits * a.M * a.N * sizeof(float) : 0;
  pl->part_offset = pl->packed ? pl->xp_bytes + pl->wp_bytes : 0;
  pl->ws_bytes = pl->part_offset + part;
  // Strided multi-tap backward-data: input pixel (h, w) only meets the taps r = (h + ph) mod sh (+ sh, + 2 sh, ...) and
  // likewise along w, so the pixels of one parity class (h mod sh, w mod sw) form a unit-stride backward-data problem
  // on the dy grid with the filter's taps of that class: sh * sw launches of the mask kernels that together do the
  // useful multiply-adds only (the per-load variant fetches and masks every tap for every pixel: sh * sw times the work).
  // Every class needs a tap (R >= sh, S >= sw); the class filters are packed into the workspace by one small launch.
  pl->classes = pl->gen && op == JZ_BWD_DATA && (d->stride_h > 1 || d->stride_w > 1) && d->R >= d->stride_h &&
                d->S >= d->stride_w && d->stride_h * d->stride_w <= kMaxClasses &&
                ((d->R + d->stride_h - 1) / d->stride_h) * ((d->S + d->stride_w - 1) / d->stride_w) <= 32;
  if (pl->classes) pl->ws_bytes = up256((size_t)nw * 2);
  return JZ_OK;
}

// One parity class (ca, cb) of a strided multi-tap backward-data layer as a plan of its own (see make_plan).  base: the
// layer's plan; w_off: where this class's packed filter starts in the workspace (elements); false: the class has no pixels.
bool make_class_plan(const jz_conv_desc* d, const Plan& base, int ca, int cb, Plan* pl, size_t* w_elems) {
  const int sh = d->stride_h, sw = d->stride_w;
  const int P = out_dim(d->H, d->pad_h, d->R, sh), Q = out_dim(d->W, d->pad_w, d->S, sw);
  const int Ha = (d->H - ca + sh - 1) / sh, Wb = (d->W - cb + sw - 1) / sw;     // pixels h = ca + sh i, w = cb + sw l
  const int r0 = (ca + d->pad_h) % sh, s0 = (cb + d->pad_w) % sw;               // first tap of the class
  const int Ra = (d->R - r0 + sh - 1) / sh, Sb = (d->S - s0 + sw - 1) / sw;     // taps r0 + sh j, s0 + sw i
  *w_elems = (size_t)d->K * Ra * Sb * d->C;
  if (Ha <= 0 || Wb <= 0) return false;
  *pl = base;
  pl->gen = false;
  pl->classes = false;
  GemmArgs& a = pl->args;
  ConvGeom& g = a.g;
  a.M = d->N * Ha * Wb; a.N = d->C; a.Kred = Ra * Sb * d->K;
  g.IH = P; g.IW = Q; g.IC = d->K; g.OH = Ha; g.OW = Wb;
  g.R = Ra; g.S = Sb; g.sh = 1; g.sw = 1;
  g.ph = (ca + d->pad_h) / sh; g.pw = (cb + d->pad_w) / sw;   // dy row of tap j for pixel row i: i + ph - j
  g.row_pitch = Q * d->K; g.pix_step = d->K; g.s_step = d->K;
  g.kvalid = 0;
  g.always_mask = 1;   // the class grid and the dy grid are not tied by the usual size formula
  a.sc_on = 1; a.sc_H = d->H; a.sc_W = d->W; a.sc_sh = sh; a.sc_sw = sw; a.sc_oh = ca; a.sc_ow = cb; a.sc_fill = 0;
  a.bw_linear = 0;
  finish_geometry(g);
  pl->bytesB = *w_elems * 2;
  pl->bk = 32;
  choose_tiling(pl, d->K % 64 == 0, 0);
  pl->part_offset = 0;
  pl->ws_bytes = 0;
  return true;
}

// class filters: wp[class][k][j][i][c] = w[k][r0 + sh j][s0 + sw i][c], classes in (ca, cb) row-major order
__global__ __launch_bounds__(256) void pack_class_filters(const unsigned short* __restrict__ w, unsigned short* __restrict__ wp,
                                                          int K, int R, int S, int C, int sh, int sw, int ph, int pw) {
  const long long n = (long long)K * R * S * C;
  for (long long idx = (long long)blockIdx.x * 256 + threadIdx.x; idx < n; idx += (long long)gridDim.x * 256) {
    const int c = (int)(idx % C);
    long long t = idx / C;
    const int s_ = (int)(t % S); t /= S;
    const int r = (int)(t % R);
    const int k = (int)(t / R);
    // the class this tap belongs to: r = (ca + ph) mod sh  <=>  ca = (r - ph) mod sh
    const int ca = ((r - ph) % sh + sh) % sh, cb = ((s_ - pw) % sw + sw) % sw;
    const int r0 = (ca + ph) % sh, s0 = (cb + pw) % sw;
    const int j = (r - r0) / sh, i = (s_ - s0) / sw;
    // offset of the class: the filters of all classes before it
    long long off = 0;
    for (int a2 = 0; a2 < sh; ++a2)
      for (int b2 = 0; b2 < sw; ++b2) {
        if (a2 * sw + b2 >= ca * sw + cb) break;
        const int rr = (a2 + ph) % sh, ss = (b2 + pw) % sw;
        off += (long long)K * ((R - rr + sh - 1) / sh) * ((S - ss + sw - 1) / sw) * C;
      }
    const int Ra = (R - r0 + sh - 1) / sh, Sb = (S - s0 + sw - 1) / sw;
    (void)Ra;
    wp[off + (((long long)k * ((R - r0 + sh - 1) / sh) + j) * Sb + i) * C + c] = w[idx];
  }
}

// a forward plan whose kernel can leave the per-tile column sums: the ring kernels (their LDS holds the sums), no split
bool plan_leaves_stats(const Plan& pl) {
  return pl.op == JZ_FWD && pl.fast && pl.args.splits == 1;
}
// a backward-data plan whose kernel can leave the sums of a batch-norm backward: the ring kernels with masks, no split,
// no scatter epilogue, whole 16-byte pieces of a row
bool plan_leaves_bwd_stats(const Plan& pl) {
  return pl.op == JZ_BWD_DATA && pl.fast && !pl.gen && pl.args.splits == 1 && !pl.args.sc_on && (pl.args.N & 7) == 0;
}

// A, B in the kernel's order: FWD (x, w), BWD_DATA (dy, w), BWD_WEIGHT (dy, x)
int run(int op, const jz_conv_desc* d, const void* A, const void* B, void* D, void* ws, size_t ws_bytes, void* stream,
        float* stats = nullptr, int stats_tiles_m = 0, const jz::SumsqSink* sink = nullptr, const jz::BnBwdOperands* bn = nullptr) {
  Plan pl;
  int rc = make_plan(op, d, &pl);
  if (rc != JZ_OK) return rc;
  // the caller sized the buffer of the column sums from an earlier plan: it has to be this plan (the run-time tuning table
  // may have been changed in between)
  if (stats && !(op == JZ_BWD_DATA ? plan_leaves_bwd_stats(pl) && bn != nullptr : plan_leaves_stats(pl))) return JZ_ERR_UNSUPPORTED;
  if (stats && pl.args.tiles_m != stats_tiles_m) return JZ_ERR_UNSUPPORTED;
  if (!A || !B || !D) return JZ_ERR_NULL;
  if (!aligned16(A) || !aligned16(B) || !aligned16(D) || (ws && !aligned16(ws))) return JZ_ERR_ALIGN;
  if (overlaps(D, pl.bytesD, A, pl.bytesA) || overlaps(D, pl.bytesD, B, pl.bytesB)) return JZ_ERR_ALIAS;
  if (pl.ws_bytes > 0 && (!ws || ws_bytes < pl.ws_bytes)) return JZ_ERR_WORKSPACE;
  if (pl.ws_bytes > 0 && (overlaps(ws, pl.ws_bytes, A, pl.bytesA) || overlaps(ws, pl.ws_bytes, B, pl.bytesB) ||
                          overlaps(ws, pl.ws_bytes, D, pl.bytesD)))
    return JZ_ERR_ALIAS;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (pl.classes) {  // strided multi-tap backward-data: pack the class filters, then one unit-stride launch per class
    unsigned short* wp = static_cast<unsigned short*>(ws);
    const long long nwl = (long long)d->K * d->R * d->S * d->C;
    const unsigned pgrid = (unsigned)((nwl + 255) / 256 < 2048 ? (nwl + 255) / 256 : 2048);
    hipLaunchKernelGGL(pack_class_filters, dim3(pgrid), dim3(256), 0, st, static_cast<const unsigned short*>(B), wp, d->K, d->R, d->S,
                       d->C, d->stride_h, d->stride_w, d->pad_h, d->pad_w);
    if ((rc = jz::launch_status()) != JZ_OK) return rc;
    size_t w_off = 0;
    for (int ca = 0; ca < d->stride_h; ++ca)
      for (int cb = 0; cb < d->stride_w; ++cb) {
        Plan cp;
        size_t w_elems = 0;
        const bool any = make_class_plan(d, pl, ca, cb, &cp, &w_elems);
        if (any) {
          GemmArgs& c = cp.args;
          c.A = static_cast<const unsigned short*>(A);
          c.B = wp + w_off;
          c.D16 = static_cast<unsigned short*>(D);
          c.bytesA = (unsigned)pl.bytesA;
          c.bytesB = (unsigned)(w_elems * 2);
          c.Dpart = nullptr;
          c.stats = nullptr;
          c.st_y = c.st_c = c.st_add = nullptr;
          c.st_mean = c.st_invstd = nullptr;
          if ((rc = launch_bwd_data(cp, st)) != JZ_OK) return rc;
        }
        w_off += w_elems;
      }
    return JZ_OK;
  }
  GemmArgs& a = pl.args;
  a.A = static_cast<const unsigned short*>(A);
  a.B = static_cast<const unsigned short*>(B);
  a.D16 = static_cast<unsigned short*>(D);
  a.bytesA = (unsigned)pl.bytesA;
  a.bytesB = (unsigned)pl.bytesB;
  a.Dpart = reinterpret_cast<float*>(static_cast<char*>(ws) + pl.part_offset);
  a.stats = stats;
  a.st_y = a.st_c = a.st_add = nullptr;
  a.st_mean = a.st_invstd = nullptr;
  if (stats && op == JZ_BWD_DATA) {
    a.st_add = static_cast<const unsigned short*>(bn->add16);
    a.st_y = static_cast<const unsigned short*>(bn->y16);
    a.st_c = static_cast<const unsigned short*>(bn->x16);
    a.st_mean = bn->mean;
    a.st_invstd = bn->invstd;
  }
  unsigned short* dwp = nullptr;
  if (pl.packed) {
    unsigned short* xp = static_cast<unsigned short*>(ws);
    unsigned short* wp = reinterpret_cast<unsigned short*>(static_cast<char*>(ws) + pl.xp_bytes);
    const unsigned short* x = static_cast<const unsigned short*>(op == JZ_FWD ? A : B);
    const unsigned short* wsrc = op == JZ_FWD ? static_cast<const unsigned short*>(B) : nullptr;
    StemArgs sa;
    const bool stem = pl.stem && !stats && stem_fwd_setup(pl, d, &sa);
    hipLaunchKernelGGL(pad_to_c4, dim3((unsigned)((pl.Wp / 2 + 127) / 128), (unsigned)((pl.Hp + PAD_ROWS - 1) / PAD_ROWS), (unsigned)(d->N + (wsrc ? 1 : 0))),
                       dim3(128), 0, st, x, xp, d->N, d->H, d->W, d->C, pl.Hp, pl.Wp, d->pad_h, d->pad_w, wsrc,
                       wsrc ? wp : nullptr, d->K, d->R, d->S, stem ? sa.NKS * 16 : pl.KT, stem ? 1 : 0);
    if (stem) {
      if ((rc = jz::launch_status()) != JZ_OK) return rc;
      sa.xp = xp;
      sa.wq = wp;
      sa.y = static_cast<unsigned short*>(D);
      return launch_stem_fwd(sa, st);
    }
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
  if (op == JZ_FWD) rc = stats ? launch_fwd_stats(pl, st) : launch_fwd(pl, st);
  else if (op == JZ_BWD_DATA) rc = !stats ? launch_bwd_data(pl, st) : bn->block_end ? launch_bwd_data_block_end(pl, st) : launch_bwd_data_stats(pl, st);
  else rc = launch_bwd_weight(pl, st);
  if (rc != JZ_OK) return rc;
  if (a.splits > 1) {
    long long MN = (long long)a.M * a.N;
    // split lanes per output group: enough workgroups to cover the chip first, then shorten each thread's chain
    int lg = 0;
    while (lg < 5 && (2 << lg) <= a.splits && ((MN + 3) / 4 + (256 >> lg) - 1) / (256 >> lg) < 1024) ++lg;
    const long long per_block = 256 >> lg;
    unsigned blocks = (unsigned)(((MN + 3) / 4 + per_block - 1) / per_block);
    // small-channel backward-weight: the reduction writes the real filter entries straight into dw
    if (sink) {
      const unsigned grid = blocks < 2048u ? blocks : 2048u;  // at most 32 workgroups per counter quadruple of the sink
      hipLaunchKernelGGL(splitk_reduce_sumsq, dim3(grid), dim3(256), 0, st, a.Dpart, dwp ? static_cast<unsigned short*>(D) : a.D16,
                         MN, a.splits, lg, dwp ? pl.KT / 4 : 0, d->S, d->C, (long long)blocks, *sink);
      sink = nullptr;  // taken
    } else {
      hipLaunchKernelGGL(splitk_reduce, dim3(blocks), dim3(256), 0, st, a.Dpart, dwp ? static_cast<unsigned short*>(D) : a.D16,
                         MN, a.splits, lg, dwp ? pl.KT / 4 : 0, d->S, d->C);
    }
    if ((rc = jz::launch_status()) != JZ_OK) return rc;
    dwp = nullptr;
  }
  if (dwp) {
    int ndw = d->K * d->R * d->S * d->C;
    hipLaunchKernelGGL(unpack_filter_c4, dim3((unsigned)((ndw + 255) / 256)), dim3(256), 0, st, dwp,
                       static_cast<unsigned short*>(D), d->K, d->R, d->S, d->C, pl.KT);
    if ((rc = jz::launch_status()) != JZ_OK) return rc;
  }
  // no split reduction to take the sum of squares in: one pass over the gradient just written (still in cache)
  if (sink) rc = jz::sumsq_half_launch(static_cast<const unsigned short*>(D), (long long)d->K * d->R * d->S * d->C, *sink, st);
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
int jz::conv_bwd_data_stats_plan(const jz_conv_desc* d, size_t* conv_ws_bytes, int* tiles_m) {
  Plan pl;
  int rc = make_plan(JZ_BWD_DATA, d, &pl);
  if (rc != JZ_OK) return rc;
  *conv_ws_bytes = pl.ws_bytes;
  *tiles_m = plan_leaves_bwd_stats(pl) ? pl.args.tiles_m : 0;
  return JZ_OK;
}
int jz::conv_bwd_data_run(const jz_conv_desc* d, const void* dy, const void* w, void* dx, void* ws, size_t ws_bytes, float* stats,
                          int stats_tiles_m, const BnBwdOperands* bn, void* stream) {
  return run(JZ_BWD_DATA, d, dy, w, dx, ws, ws_bytes, stream, stats, stats_tiles_m, nullptr, bn);
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
  if (pl.classes) {  // the launches of the parity classes: the first class stands for all (same filter shape up to a tap row / column)
    Plan cp;
    size_t w_elems;
    if (make_class_plan(desc, pl, 0, 0, &cp, &w_elems)) {
      cp.classes = true;
      cp.args.sc_on = 0;
      plan_text(cp, text, text_bytes);
      return JZ_OK;
    }
  }
  plan_text(pl, text, text_bytes);
  return JZ_OK;
}

extern "C" int jz_conv2d_tune_set(int op, const jz_conv_desc* desc, int tile_m, int tile_n, int k_tile, int wavefronts,
                                  int ring, int splits) {
  Plan pl;
  int rc = make_plan(op, desc, &pl);
  if (rc != JZ_OK) return rc;
  if (!pl.fast || splits < 1) return JZ_ERR_UNSUPPORTED;  // the element-wise path has one kernel shape
  const Variant* v = nullptr;
  for (const Variant& c : kVariants)
    if (c.BM == tile_m && c.BN == tile_n && c.bk == k_tile && c.waves == wavefronts && c.nst == ring) v = &c;
  if (!v) return JZ_ERR_UNSUPPORTED;
  if (pl.classes) {  // the variant goes to every parity class's launch (their reductions are never split)
    std::vector<Tuned> keys;
    for (int ca = 0; ca < desc->stride_h; ++ca)
      for (int cb = 0; cb < desc->stride_w; ++cb) {
        Plan cp;
        size_t w_elems;
        if (!make_class_plan(desc, pl, ca, cb, &cp, &w_elems)) continue;
        const GemmArgs& a = cp.args;
        keys.push_back(Tuned{1, a.M, a.N, a.Kred, a.g.R * a.g.S, a.sc_on, tile_m, tile_n, k_tile, wavefronts, ring, 1});
      }
    std::lock_guard<std::mutex> lock(g_tune_mutex);
    for (const Tuned& t : keys) {
      bool found = false;
      for (Tuned& e : g_tune_rt)
        if (same_key(e, t)) { e = t; found = true; }
      if (!found) g_tune_rt.push_back(t);
    }
    return JZ_OK;
  }
  // per-load tap arithmetic exists for the four basic 4-wavefront tiles, 32 deep, four-stage ring
  if (pl.gen && (v->waves != 4 || v->bk != 32 || v->nst != 4 || v->BM > 128 || v->BN > 128)) return JZ_ERR_UNSUPPORTED;
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
  g_use_table = true;
  return JZ_OK;
}

extern "C" int jz_conv2d_tune_use_table(int on) {
  std::lock_guard<std::mutex> lock(g_tune_mutex);
  g_use_table = on != 0;
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

// ---- backward-weight that also hands the gradient's sum of squares to the optimiser ---------------------------------
namespace {
int check_sink(const jz_sumsq_sink* sink, const void* dw, size_t dw_bytes, const void* ws, size_t ws_bytes, jz::SumsqSink* out) {
  if (!sink || !sink->sums || !sink->nonfinite) return JZ_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(sink->sums) & 127u) || (reinterpret_cast<uintptr_t>(sink->nonfinite) & 3u)) return JZ_ERR_ALIGN;
  if (overlaps(sink->sums, JZ_SUMSQ_SINK_BYTES, dw, dw_bytes) || overlaps(sink->nonfinite, sizeof(int), dw, dw_bytes) ||
      overlaps(sink->sums, JZ_SUMSQ_SINK_BYTES, ws, ws_bytes) || overlaps(sink->nonfinite, sizeof(int), ws, ws_bytes) ||
      overlaps(sink->sums, JZ_SUMSQ_SINK_BYTES, sink->nonfinite, sizeof(int)))
    return JZ_ERR_ALIAS;
  *out = jz::SumsqSink{static_cast<unsigned long long*>(sink->sums), sink->nonfinite};
  return JZ_OK;
}
}  // namespace

int jz::sumsq_half_launch(const unsigned short* g16, long long n, const jz::SumsqSink& sink, hipStream_t st) {
  if (n <= 0) return JZ_OK;
  long long want = (n / 8 + 255) / 256;  // one 16-byte group per thread and pass; at most 2^20 elements per workgroup
  const unsigned grid = (unsigned)(want < 1 ? 1 : (want > 1024 ? 1024 : want));
  hipLaunchKernelGGL(sumsq_half, dim3(grid), dim3(256), 0, st, g16, n, sink);
  return jz::launch_status();
}

extern "C" int jz_conv2d_bwd_weight_sumsq(const jz_conv_desc* desc, const void* x16, const void* dy16, void* dw16, void* ws,
                                          size_t ws_bytes, const jz_sumsq_sink* sink, void* hip_stream) {
  Plan pl;
  int rc = make_plan(JZ_BWD_WEIGHT, desc, &pl);
  if (rc != JZ_OK) return rc;
  jz::SumsqSink sk;
  if ((rc = check_sink(sink, dw16, pl.bytesD, ws, pl.ws_bytes, &sk)) != JZ_OK) return rc;
  return run(JZ_BWD_WEIGHT, desc, dy16, x16, dw16, ws, ws_bytes, hip_stream, nullptr, 0, &sk);
}

// ---- backward-weight without a caller workspace ---------------------------------------------------------------
// For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops): the same
// kernels, with the split-K partial sums (and the padded copy of a small-channel layer) in a fixed array that lives
// in the library's code object.  Every GPU the library runs on holds its own copy of the array at its own address for
// the life of the process; host code must not use the array's name as an address, so the address is looked up once
// per device and kept.
#define JZ_SCRATCH_LEN ((size_t)JZ_STATIC_SCRATCH_BYTES)
constexpr size_t kStaticScratchBytes = JZ_SCRATCH_LEN;
static __device__ __align__(256) unsigned char scratch[JZ_SCRATCH_LEN];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

int static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return JZ_ERR_LAUNCH;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      return JZ_ERR_LAUNCH;
    }
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return JZ_OK;
}

extern "C" int jz_conv2d_bwd_weight_static(const jz_conv_desc* desc, const void* x16, const void* dy16, void* dw16,
                                           void* hip_stream) {
  Plan pl;
  int rc = make_plan(JZ_BWD_WEIGHT, desc, &pl);
  if (rc != JZ_OK) return rc;
  if (pl.ws_bytes > kStaticScratchBytes) return JZ_ERR_WORKSPACE;  // the layer needs more scratch than the array holds
  void* ws = nullptr;
  if (pl.ws_bytes > 0 && (rc = static_scratch(&ws)) != JZ_OK) return rc;
  return run(JZ_BWD_WEIGHT, desc, dy16, x16, dw16, ws, ws ? kStaticScratchBytes : 0, hip_stream);  // A = dy, B = x
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

extern "C" int jz_gemm_fc_bwd_weight_sumsq(int batch, int in_features, int out_features, const void* dy16, const void* x16,
                                           void* dw16, void* ws, size_t ws_bytes, const jz_sumsq_sink* sink, void* hip_stream) {
  jz_conv_desc d;
  int rc = fc_desc(JZ_BWD_WEIGHT, batch, in_features, out_features, &d);
  if (rc != JZ_OK) return rc;
  return jz_conv2d_bwd_weight_sumsq(&d, x16, dy16, dw16, ws, ws_bytes, sink, hip_stream);
}
