// Training-mode batch normalization with an optional ReLU, forward and backward, for gfx950 (Jia et al. 2018,
// Section 4.2: x^ = (x - mean_B) / sqrt(var_B + eps), y = gamma x^ + beta, statistics per channel over the mini-batch).
//
// Activations are FP16 [rows][C] (NHWC with rows = N*H*W), gamma / beta / the saved statistics FP32, all sums FP32 per
// workgroup slab and FP64 across slabs.  Every pass is bound by HBM, so each direction is three stream-ordered launches:
//
//   forward   bn_stats      a workgroup owns a slab of rows: per channel sum(x) and sum(x^2) of the slab (no atomics)
//             bn_fwd_final  per channel: the slabs' sums added in a fixed order in FP64 -> mean, 1/sqrt(var + eps), and the
//                           affine form y = a x + b (a = gamma invstd, b = beta - mean a) for the next pass
//             bn_apply      y = [max(., 0)](a x + b), 16 bytes per lane in and out
//   backward  bn_bwd_stats  per slab and channel: sum(g) and sum(g x^), g = dy masked by (y > 0) when the ReLU is on
//             bn_bwd_final  dbeta = sum g, dgamma = sum g x^ (FP16 copies for the optimizer's gradient buffer)
//             bn_bwd_apply  dx = gamma invstd (g - dbeta/M - x^ dgamma/M), evaluated as a g + P x + Q per channel
//
// A lane always handles 8 consecutive channels (one 16-byte access); the C/8 lanes of a row sit side by side, so a
// wavefront reads whole rows contiguously.  Results are deterministic: the order of every sum depends only on
// (rows, C).
#include <hip/hip_runtime.h>

#include "jz_internal.h"

namespace {

constexpr int BN_THREADS = 256;
constexpr int BN_MAX_C = 2048;       // C / 8 lanes of a row have to fit one workgroup
constexpr int BN_TARGET_SLABS = 512;   // two per compute unit
constexpr int BN_FIN_C = 8;            // channels a finalize workgroup handles (32 contiguous bytes of every slab's sums);
                                       // its 256 / 8 = 32 lanes per channel share the slabs

size_t up256(size_t x) { return (x + 255) & ~size_t(255); }

struct BnPlan {
  int64_t rows = 0;
  int C = 0, cpr = 0;        // 16-byte chunks per row
  int csplit = 1;            // workgroups that share a slab of rows, each with cpr / csplit of the chunks (wide, short tensors)
  int rpp = 0;               // rows one pass of a workgroup covers (BN_THREADS / (cpr / csplit); lanes beyond that idle)
  int64_t rows_per_slab = 0; // a multiple of rpp
  int slabs = 0;
  size_t off_part = 0, off_coef = 0, total = 0;  // workspace: [slabs][2][C] float partial sums, [4][C] float coefficients
};

int make_bn_plan(int64_t rows, int channels, BnPlan* p) {
  if (rows <= 0 || channels <= 0) return JZ_ERR_SHAPE;
  if (channels % 8 != 0 || channels > BN_MAX_C) return JZ_ERR_UNSUPPORTED;
  if (rows * (int64_t)channels >= (int64_t(1) << 40)) return JZ_ERR_UNSUPPORTED;
  p->rows = rows;
  p->C = channels;
  p->cpr = channels / 8;
  // at most BN_TARGET_SLABS slabs, and at least 16 passes of the workgroup and 64 rows per slab: small tensors get fewer
  // slabs, so that the partial sums stay small beside the tensor.  A wide tensor with few rows would then leave most of
  // the chip idle (2048 channels x 3136 rows: 49 slabs), so its slabs are shared by csplit workgroups that take a range
  // of at least 32 chunks (512 contiguous bytes of a row) each: more workgroups, the same number of partial sums.
  for (int cs = 1;; cs *= 2) {
    const int cpr_l = p->cpr / cs;
    p->csplit = cs;
    p->rpp = BN_THREADS / cpr_l;
    // fewer passes per workgroup (16, 8, 4) until at least 256 workgroups exist
    for (int min_passes = 16; min_passes >= 4; min_passes /= 2) {
      int64_t per = (rows + BN_TARGET_SLABS - 1) / BN_TARGET_SLABS;
      if (per < min_passes * (int64_t)p->rpp) per = min_passes * (int64_t)p->rpp;
      if (per < 32) per = 32;
      per = (per + p->rpp - 1) / p->rpp * p->rpp;
      p->rows_per_slab = per;
      p->slabs = (int)((rows + per - 1) / per);
      if ((int64_t)p->slabs * cs >= 256) break;
    }
    if ((int64_t)p->slabs * cs >= 256 || cs == 8 || cpr_l % 2 != 0 || cpr_l / 2 < 32) break;
  }
  p->off_part = 0;
  p->off_coef = up256((size_t)p->slabs * 2 * channels * sizeof(float));
  p->total = p->off_coef + up256((size_t)4 * channels * sizeof(float));
  return JZ_OK;
}

__device__ __forceinline__ void unpack8(const uint4& v, float (&f)[8]) {
  const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    _Float16 lo, hi;
    unsigned short a = (unsigned short)(w[i] & 0xffffu), b = (unsigned short)(w[i] >> 16);
    __builtin_memcpy(&lo, &a, 2);
    __builtin_memcpy(&hi, &b, 2);
    f[2 * i] = (float)lo;
    f[2 * i + 1] = (float)hi;
  }
}

__device__ __forceinline__ uint4 pack8(const float (&f)[8]) {
  unsigned w[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    _Float16 lo = (_Float16)f[2 * i], hi = (_Float16)f[2 * i + 1];  // round to nearest even
    unsigned short a, b;
    __builtin_memcpy(&a, &lo, 2);
    __builtin_memcpy(&b, &hi, 2);
    w[i] = (unsigned)a | ((unsigned)b << 16);
  }
  return make_uint4(w[0], w[1], w[2], w[3]);
}

// Sums over a slab of rows, for the 8 channels of each lane: s0 and s1 are whatever `term` produces per element.
// The rpp lanes that share a channel chunk (one per row of a pass) are then added in row order through LDS, and the
// slab's 2 x C sums are stored.  MODE 0: (x, x^2).  MODE 1: (g, g x^) with g = dy [* (y > 0)].  MODE 2: the end of a
// residual block: g = RNE16(dy [+ dy2]) where y > 0, else 0, is formed here, written to g_out for the other consumers of
// that gradient, and summed as in MODE 1 (the sums see the rounded g, as a pass over g_out would).
template <int MODE>
__global__ __launch_bounds__(BN_THREADS) void bn_stats(const uint4* __restrict__ x, const uint4* __restrict__ y,
                                                      const uint4* __restrict__ dy, const float* __restrict__ mean,
                                                      const float* __restrict__ invstd, float* __restrict__ part, int64_t rows,
                                                      int C, int cpr, int rpp, int64_t rows_per_slab, int relu, int csplit,
                                                      const uint4* __restrict__ dy2 = nullptr, uint4* __restrict__ g_out = nullptr) {
  __shared__ float red[2][BN_THREADS][8];
  const int tid = threadIdx.x;
  const int cpr_l = cpr / csplit;  // chunks of a row this workgroup handles: [cfirst, cfirst + cpr_l)
  const int slab = blockIdx.x / csplit, cfirst = (blockIdx.x % csplit) * cpr_l;
  const int chunk_l = tid % cpr_l, rsub = tid / cpr_l;
  const int chunk = cfirst + chunk_l;
  const int64_t r0 = (int64_t)slab * rows_per_slab;
  int64_t r1 = r0 + rows_per_slab;
  if (r1 > rows) r1 = rows;
  float s0[8], s1[8], mu[8], is[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    s0[e] = 0.f; s1[e] = 0.f; mu[e] = 0.f; is[e] = 0.f;
  }
  if (MODE >= 1 && rsub < rpp) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      mu[e] = mean[chunk * 8 + e];
      is[e] = invstd[chunk * 8 + e];
    }
  }
  // U rows of a lane are requested together (the loop is bound by memory latency otherwise)
  constexpr int U = MODE == 0 ? 8 : 4;
  for (int64_t r = r0 + rsub; rsub < rpp && r < r1; r += (int64_t)U * rpp) {
    uint4 qx[U], qd[U], qy[U], qe[U];
    const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t ru = r + (int64_t)u * rpp;
      const bool in = ru < r1;
      const size_t idx = (size_t)(in ? ru : r) * cpr + chunk;
      qx[u] = x[idx];
      if (MODE >= 1) {
        qd[u] = dy[idx];
        qy[u] = (relu || MODE == 2) ? y[idx] : zero;
      }
      if (MODE == 2) qe[u] = dy2 ? dy2[idx] : zero;
      if (!in) {            // rows beyond the slab add nothing (x = 0 and g = 0 contribute zero to every sum)
        qx[u] = zero;
        if (MODE >= 1) qd[u] = zero;
        if (MODE == 2) qe[u] = zero;
      }
    }
    if (MODE == 2) {        // form g, keep it as this row's dy, and store it
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float a[8], b[8], m[8];
        unpack8(qd[u], a);
        unpack8(qe[u], b);
        unpack8(qy[u], m);
#pragma unroll
        for (int e = 0; e < 8; ++e) a[e] += b[e];  // exact in FP32; pack8 rounds once
        uint4 gq = pack8(a);
        unsigned gw[4] = {gq.x, gq.y, gq.z, gq.w};
#pragma unroll
        for (int k = 0; k < 4; ++k)
          gw[k] = (m[2 * k] > 0.f ? (gw[k] & 0xffffu) : 0u) | (m[2 * k + 1] > 0.f ? (gw[k] & 0xffff0000u) : 0u);
        qd[u] = make_uint4(gw[0], gw[1], gw[2], gw[3]);
        const int64_t ru = r + (int64_t)u * rpp;
        if (ru < r1) g_out[(size_t)ru * cpr + chunk] = qd[u];
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float xv[8];
      unpack8(qx[u], xv);
      if (MODE == 0) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          s0[e] += xv[e];
          s1[e] += xv[e] * xv[e];
        }
      } else {
        float gv[8];
        unpack8(qd[u], gv);
        if (MODE == 1 && relu) {
          float yv[8];
          unpack8(qy[u], yv);
#pragma unroll
          for (int e = 0; e < 8; ++e) gv[e] = yv[e] > 0.f ? gv[e] : 0.f;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          s0[e] += gv[e];
          s1[e] += gv[e] * ((xv[e] - mu[e]) * is[e]);
        }
      }
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    red[0][tid][e] = s0[e];
    red[1][tid][e] = s1[e];
  }
  __syncthreads();
  if (rsub == 0) {
    for (int j = 1; j < rpp; ++j)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        s0[e] += red[0][j * cpr_l + chunk_l][e];
        s1[e] += red[1][j * cpr_l + chunk_l][e];
      }
    float* p0 = part + ((size_t)slab * 2) * C + chunk * 8;
    float* p1 = p0 + C;
    *reinterpret_cast<float4*>(p0) = make_float4(s0[0], s0[1], s0[2], s0[3]);
    *reinterpret_cast<float4*>(p0 + 4) = make_float4(s0[4], s0[5], s0[6], s0[7]);
    *reinterpret_cast<float4*>(p1) = make_float4(s1[0], s1[1], s1[2], s1[3]);
    *reinterpret_cast<float4*>(p1 + 4) = make_float4(s1[4], s1[5], s1[6], s1[7]);
  }
}

// The two sums of channel c over all slabs, FP64: lane js of the channel's 32 lanes adds slabs js, js + 32, ... in that order,
// then lane 0 adds the 32 lane sums in lane order (deterministic).  Returns true on the lane that holds the totals.
__device__ __forceinline__ bool bn_slab_totals(const float* __restrict__ part, int slabs, int C, int c, double& s, double& q) {
  __shared__ double red[2][BN_THREADS];
  constexpr int LANES = BN_THREADS / BN_FIN_C;
  const int js = threadIdx.x / BN_FIN_C;
  s = 0.0;
  q = 0.0;
  if (c < C)
    for (int k = js; k < slabs; k += 8 * LANES) {  // eight slabs' sums requested together, added in slab order
      float a[8], b[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {  // all sixteen loads first (clamped index), the selection afterwards
        const int ku = k + u * LANES;
        const int kc = ku < slabs ? ku : k;
        a[u] = part[((size_t)kc * 2) * C + c];
        b[u] = part[((size_t)kc * 2 + 1) * C + c];
      }
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (k + u * LANES >= slabs) {
          a[u] = 0.f;
          b[u] = 0.f;
        }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        s += (double)a[u];
        q += (double)b[u];
      }
    }
  red[0][threadIdx.x] = s;
  red[1][threadIdx.x] = q;
  __syncthreads();
  if (js != 0 || c >= C) return false;
  for (int l = 1; l < LANES; ++l) {
    s += red[0][l * BN_FIN_C + threadIdx.x];
    q += red[1][l * BN_FIN_C + threadIdx.x];
  }
  return true;
}

__global__ __launch_bounds__(BN_THREADS) void bn_fwd_final(const float* __restrict__ part, int slabs, int C, double inv_rows,
                                                          float eps, const float* __restrict__ gamma,
                                                          const float* __restrict__ beta, float* __restrict__ save_mean,
                                                          float* __restrict__ save_invstd, float* __restrict__ coef) {
  const int c = blockIdx.x * BN_FIN_C + threadIdx.x % BN_FIN_C;
  double s, q;
  if (!bn_slab_totals(part, slabs, C, c, s, q)) return;
  const double m = s * inv_rows;
  double var = q * inv_rows - m * m;
  if (var < 0.0) var = 0.0;
  const double is = 1.0 / sqrt(var + (double)eps);
  const float mf = (float)m, isf = (float)is;
  save_mean[c] = mf;
  save_invstd[c] = isf;
  const float a = gamma[c] * isf;
  coef[c] = a;
  coef[C + c] = beta[c] - mf * a;
}

// RES: a residual tensor is added in front of the ReLU (the end of a bottleneck block)
template <int RES>
__global__ __launch_bounds__(BN_THREADS) void bn_apply(const uint4* __restrict__ x, const uint4* __restrict__ res,
                                                      uint4* __restrict__ y, const float* __restrict__ coef, int64_t n_chunks, int C,
                                                      int cpr, int relu) {
  const int64_t stride = (int64_t)gridDim.x * BN_THREADS;
  for (int64_t i = (int64_t)blockIdx.x * BN_THREADS + threadIdx.x; i < n_chunks; i += stride) {
    const int chunk = (int)(i % cpr);
    float a[8], b[8], v[8];
    const float4* ca = reinterpret_cast<const float4*>(coef + chunk * 8);
    const float4* cb = reinterpret_cast<const float4*>(coef + C + chunk * 8);
    float4 t0 = ca[0], t1 = ca[1], u0 = cb[0], u1 = cb[1];
    a[0] = t0.x; a[1] = t0.y; a[2] = t0.z; a[3] = t0.w; a[4] = t1.x; a[5] = t1.y; a[6] = t1.z; a[7] = t1.w;
    b[0] = u0.x; b[1] = u0.y; b[2] = u0.z; b[3] = u0.w; b[4] = u1.x; b[5] = u1.y; b[6] = u1.z; b[7] = u1.w;
    unpack8(x[i], v);
    float rv[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (RES) unpack8(res[i], rv);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float z = v[e] * a[e] + b[e];
      if (RES) z += rv[e];
      v[e] = (relu && !(z > 0.f)) ? 0.f : z;
    }
    y[i] = pack8(v);
  }
}

__global__ __launch_bounds__(BN_THREADS) void bn_bwd_final(const float* __restrict__ part, int slabs, int C, double inv_rows,
                                                          const float* __restrict__ gamma, const float* __restrict__ mean,
                                                          const float* __restrict__ invstd, unsigned short* __restrict__ dgamma16,
                                                          unsigned short* __restrict__ dbeta16, float* __restrict__ coef) {
  const int c = blockIdx.x * BN_FIN_C + threadIdx.x % BN_FIN_C;
  double sb, sg;
  if (!bn_slab_totals(part, slabs, C, c, sb, sg)) return;
  _Float16 hg = (_Float16)(float)sg, hb = (_Float16)(float)sb;
  unsigned short ug, ub;
  __builtin_memcpy(&ug, &hg, 2);
  __builtin_memcpy(&ub, &hb, 2);
  dgamma16[c] = ug;
  dbeta16[c] = ub;
  // dx = a (g - dbeta/M - x^ dgamma/M) with x^ = (x - mean) invstd, as dx = a g + P x + Q
  const double a = (double)gamma[c] * (double)invstd[c];
  const double t = a * (sg * inv_rows) * (double)invstd[c];
  coef[c] = (float)a;
  coef[C + c] = (float)(-t);
  coef[2 * C + c] = (float)(t * (double)mean[c] - a * (sb * inv_rows));
}

__device__ __forceinline__ void load8(const float* p, float (&f)[8]) {
  const float4 t0 = reinterpret_cast<const float4*>(p)[0], t1 = reinterpret_cast<const float4*>(p)[1];
  f[0] = t0.x; f[1] = t0.y; f[2] = t0.z; f[3] = t0.w; f[4] = t1.x; f[5] = t1.y; f[6] = t1.z; f[7] = t1.w;
}

__global__ __launch_bounds__(BN_THREADS) void bn_bwd_apply(const uint4* __restrict__ x, const uint4* __restrict__ y,
                                                          const uint4* __restrict__ dy, uint4* __restrict__ dx,
                                                          const float* __restrict__ coef, int64_t n_chunks, int C, int cpr, int relu) {
  const int64_t stride = (int64_t)gridDim.x * BN_THREADS;
  for (int64_t i = (int64_t)blockIdx.x * BN_THREADS + threadIdx.x; i < n_chunks; i += stride) {
    const int c0 = (int)(i % cpr) * 8;
    const uint4 qx = x[i], qd = dy[i];
    const uint4 qy = relu ? y[i] : make_uint4(0u, 0u, 0u, 0u);
    float a[8], pc[8], qc[8], xv[8], gv[8], out[8];
    load8(coef + c0, a);
    load8(coef + C + c0, pc);
    load8(coef + 2 * C + c0, qc);
    unpack8(qx, xv);
    unpack8(qd, gv);
    if (relu) {
      float yv[8];
      unpack8(qy, yv);
#pragma unroll
      for (int e = 0; e < 8; ++e) gv[e] = yv[e] > 0.f ? gv[e] : 0.f;
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) out[e] = a[e] * gv[e] + (pc[e] * xv[e] + qc[e]);
    dx[i] = pack8(out);
  }
}

unsigned apply_grid(int64_t n_chunks) {
  int64_t b = (n_chunks + BN_THREADS - 1) / BN_THREADS;
  const int64_t cap = 256 * 16;  // 16 workgroups per compute unit, grid-stride beyond that
  return (unsigned)(b < cap ? b : cap);
}

}  // namespace

extern "C" int jz_bn_workspace_bytes(int64_t rows, int channels, size_t* bytes) {
  if (!bytes) return JZ_ERR_NULL;
  BnPlan p;
  int rc = make_bn_plan(rows, channels, &p);
  if (rc != JZ_OK) return rc;
  *bytes = p.total;
  return JZ_OK;
}

extern "C" int jz_bn_relu_fwd(int64_t rows, int channels, const void* x16, const float* gamma, const float* beta, float eps,
                              int relu, void* y16, float* save_mean, float* save_invstd, void* ws, size_t ws_bytes,
                              void* hip_stream) {
  BnPlan p;
  int rc = make_bn_plan(rows, channels, &p);
  if (rc != JZ_OK) return rc;
  if (!(eps >= 0.f)) return JZ_ERR_SHAPE;
  if (!x16 || !gamma || !beta || !y16 || !save_mean || !save_invstd) return JZ_ERR_NULL;
  if (!ws || ws_bytes < p.total) return JZ_ERR_WORKSPACE;
  if (!jz::aligned16(x16) || !jz::aligned16(y16) || !jz::aligned16(ws) || !jz::aligned16(gamma) || !jz::aligned16(beta) ||
      !jz::aligned16(save_mean) || !jz::aligned16(save_invstd))
    return JZ_ERR_ALIGN;
  const size_t nb = (size_t)rows * channels * 2, nc = (size_t)channels * 4;
  if (jz::overlaps(y16, nb, x16, nb) || jz::overlaps(ws, p.total, x16, nb) || jz::overlaps(ws, p.total, y16, nb) ||
      jz::overlaps(save_mean, nc, x16, nb) || jz::overlaps(save_invstd, nc, x16, nb) || jz::overlaps(save_mean, nc, save_invstd, nc) ||
      jz::overlaps(save_mean, nc, y16, nb) || jz::overlaps(save_invstd, nc, y16, nb))
    return JZ_ERR_ALIAS;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  float* part = reinterpret_cast<float*>(static_cast<char*>(ws) + p.off_part);
  float* coef = reinterpret_cast<float*>(static_cast<char*>(ws) + p.off_coef);
  const uint4* x = static_cast<const uint4*>(x16);
  hipLaunchKernelGGL(bn_stats<0>, dim3((unsigned)(p.slabs * p.csplit)), dim3(BN_THREADS), 0, st, x, nullptr, nullptr, nullptr, nullptr,
                     part, rows, channels, p.cpr, p.rpp, p.rows_per_slab, 0, p.csplit);
  if ((rc = jz::launch_status()) != JZ_OK) return rc;
  hipLaunchKernelGGL(bn_fwd_final, dim3((unsigned)((channels + BN_FIN_C - 1) / BN_FIN_C)), dim3(BN_THREADS), 0, st, part,
                     p.slabs, channels, 1.0 / (double)rows, eps, gamma, beta, save_mean, save_invstd, coef);
  if ((rc = jz::launch_status()) != JZ_OK) return rc;
  const int64_t n_chunks = rows * p.cpr;
  hipLaunchKernelGGL(bn_apply<0>, dim3(apply_grid(n_chunks)), dim3(BN_THREADS), 0, st, x, nullptr, static_cast<uint4*>(y16), coef,
                     n_chunks, channels, p.cpr, relu ? 1 : 0);
  return jz::launch_status();
}

extern "C" int jz_bn_relu_bwd(int64_t rows, int channels, const void* x16, const void* y16, const void* dy16,
                              const float* gamma, const float* save_mean, const float* save_invstd, int relu, void* dx16,
                              void* dgamma16, void* dbeta16, void* ws, size_t ws_bytes, void* hip_stream) {
  BnPlan p;
  int rc = make_bn_plan(rows, channels, &p);
  if (rc != JZ_OK) return rc;
  if (!x16 || !dy16 || !gamma || !save_mean || !save_invstd || !dx16 || !dgamma16 || !dbeta16 || (relu && !y16)) return JZ_ERR_NULL;
  if (!ws || ws_bytes < p.total) return JZ_ERR_WORKSPACE;
  if (!jz::aligned16(x16) || !jz::aligned16(dy16) || !jz::aligned16(dx16) || !jz::aligned16(ws) || (relu && !jz::aligned16(y16)) ||
      !jz::aligned16(gamma) || !jz::aligned16(save_mean) || !jz::aligned16(save_invstd))
    return JZ_ERR_ALIGN;
  const size_t nb = (size_t)rows * channels * 2, nh = (size_t)channels * 2;
  if (jz::overlaps(dx16, nb, x16, nb) || jz::overlaps(dx16, nb, dy16, nb) || (relu && jz::overlaps(dx16, nb, y16, nb)) ||
      jz::overlaps(ws, p.total, x16, nb) || jz::overlaps(ws, p.total, dy16, nb) || jz::overlaps(ws, p.total, dx16, nb) ||
      (relu && jz::overlaps(ws, p.total, y16, nb)) || jz::overlaps(dgamma16, nh, dbeta16, nh) || jz::overlaps(dgamma16, nh, dx16, nb) ||
      jz::overlaps(dbeta16, nh, dx16, nb) || jz::overlaps(dgamma16, nh, x16, nb) || jz::overlaps(dbeta16, nh, x16, nb) ||
      jz::overlaps(dgamma16, nh, dy16, nb) || jz::overlaps(dbeta16, nh, dy16, nb))
    return JZ_ERR_ALIAS;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  float* part = reinterpret_cast<float*>(static_cast<char*>(ws) + p.off_part);
  float* coef = reinterpret_cast<float*>(static_cast<char*>(ws) + p.off_coef);
  const uint4* x = static_cast<const uint4*>(x16);
  const uint4* y = static_cast<const uint4*>(y16);
  const uint4* dy = static_cast<const uint4*>(dy16);
  hipLaunchKernelGGL(bn_stats<1>, dim3((unsigned)(p.slabs * p.csplit)), dim3(BN_THREADS), 0, st, x, y, dy, save_mean, save_invstd, part, rows,
                     channels, p.cpr, p.rpp, p.rows_per_slab, relu ? 1 : 0, p.csplit);
  if ((rc = jz::launch_status()) != JZ_OK) return rc;
  hipLaunchKernelGGL(bn_bwd_final, dim3((unsigned)((channels + BN_FIN_C - 1) / BN_FIN_C)), dim3(BN_THREADS), 0, st, part,
                     p.slabs, channels, 1.0 / (double)rows, gamma, save_mean, save_invstd, static_cast<unsigned short*>(dgamma16),
                     static_cast<unsigned short*>(dbeta16), coef);
  if ((rc = jz::launch_status()) != JZ_OK) return rc;
  const int64_t n_chunks = rows * p.cpr;
  hipLaunchKernelGGL(bn_bwd_apply, dim3(apply_grid(n_chunks)), dim3(BN_THREADS), 0, st, x, y, dy, static_cast<uint4*>(dx16), coef,
                     n_chunks, channels, p.cpr, relu ? 1 : 0);
  return jz::launch_status();
}

extern "C" int jz_bn_bwd_block_end(int64_t rows, int channels, const void* x16, const void* y_out16, const void* dya16,
                                   const void* dyb16, const float* gamma, const float* save_mean, const float* save_invstd,
                                   void* g16, void* dx16, void* dgamma16, void* dbeta16, void* ws, size_t ws_bytes, void* hip_stream) {
  BnPlan p;
  int rc = make_bn_plan(rows, channels, &p);
  if (rc != JZ_OK) return rc;
  if (!x16 || !y_out16 || !dya16 || !gamma || !save_mean || !save_invstd || !g16 || !dx16 || !dgamma16 || !dbeta16) return JZ_ERR_NULL;
  if (!ws || ws_bytes < p.total) return JZ_ERR_WORKSPACE;
  if (!jz::aligned16(x16) || !jz::aligned16(y_out16) || !jz::aligned16(dya16) || !jz::aligned16(dyb16) || !jz::aligned16(g16) ||
      !jz::aligned16(dx16) || !jz::aligned16(ws) || !jz::aligned16(gamma) || !jz::aligned16(save_mean) || !jz::aligned16(save_invstd))
    return JZ_ERR_ALIGN;
  const size_t nb = (size_t)rows * channels * 2, nh = (size_t)channels * 2;
  const void* ins[4] = {x16, y_out16, dya16, dyb16};
  void* outs[2] = {g16, dx16};
  for (void* o : outs) {
    for (const void* i : ins)
      if (jz::overlaps(o, nb, i, nb)) return JZ_ERR_ALIAS;
    if (jz::overlaps(o, nb, ws, p.total) || jz::overlaps(o, nb, dgamma16, nh) || jz::overlaps(o, nb, dbeta16, nh)) return JZ_ERR_ALIAS;
  }
  if (jz::overlaps(g16, nb, dx16, nb) || jz::overlaps(dgamma16, nh, dbeta16, nh)) return JZ_ERR_ALIAS;
  for (const void* i : ins)
    if (jz::overlaps(i, nb, ws, p.total) || jz::overlaps(i, nb, dgamma16, nh) || jz::overlaps(i, nb, dbeta16, nh)) return JZ_ERR_ALIAS;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  float* part = reinterpret_cast<float*>(static_cast<char*>(ws) + p.off_part);
  float* coef = reinterpret_cast<float*>(static_cast<char*>(ws) + p.off_coef);
  const uint4* x = static_cast<const uint4*>(x16);
  hipLaunchKernelGGL(bn_stats<2>, dim3((unsigned)(p.slabs * p.csplit)), dim3(BN_THREADS), 0, st, x, static_cast<const uint4*>(y_out16),
                     static_cast<const uint4*>(dya16), save_mean, save_invstd, part, rows, channels, p.cpr, p.rpp, p.rows_per_slab, 0,
                     p.csplit, static_cast<const uint4*>(dyb16), static_cast<uint4*>(g16));
  if ((rc = jz::launch_status()) != JZ_OK) return rc;
  hipLaunchKernelGGL(bn_bwd_final, dim3((unsigned)((channels + BN_FIN_C - 1) / BN_FIN_C)), dim3(BN_THREADS), 0, st, part,
                     p.slabs, channels, 1.0 / (double)rows, gamma, save_mean, save_invstd, static_cast<unsigned short*>(dgamma16),
                     static_cast<unsigned short*>(dbeta16), coef);
  if ((rc = jz::launch_status()) != JZ_OK) return rc;
  const int64_t n_chunks = rows * p.cpr;
  hipLaunchKernelGGL(bn_bwd_apply, dim3(apply_grid(n_chunks)), dim3(BN_THREADS), 0, st, x, nullptr, static_cast<const uint4*>(g16),
                     static_cast<uint4*>(dx16), coef, n_chunks, channels, p.cpr, 0);
  return jz::launch_status();
}

// ---- convolution + batch normalization (+ ReLU), forward, with the statistics taken in the convolution's epilogue ----
namespace {

struct ConvBnPlan {
  BnPlan bn;
  size_t conv_ws = 0;   // the convolution's own workspace, at offset 0
  int tiles_m = 0;      // > 0: the convolution kernel leaves [tiles_m][2][C] column sums; 0: a statistics pass is needed
  size_t off_bn = 0, total = 0;
};

int make_conv_bn_plan(const jz_conv_desc* d, ConvBnPlan* p) {
  int rc = jz::conv_fwd_stats_plan(d, &p->conv_ws, &p->tiles_m);
  if (rc != JZ_OK) return rc;
  const int P = (d->H + 2 * d->pad_h - d->R) / d->stride_h + 1, Q = (d->W + 2 * d->pad_w - d->S) / d->stride_w + 1;
  rc = make_bn_plan((int64_t)d->N * P * Q, d->K, &p->bn);
  if (rc != JZ_OK) return rc;
  const int slabs = p->tiles_m > p->bn.slabs ? p->tiles_m : p->bn.slabs;
  p->off_bn = up256(p->conv_ws);
  // the batch-norm part of the workspace, laid out like BnPlan's but with room for either number of partial sums
  p->bn.off_part = 0;
  p->bn.off_coef = up256((size_t)slabs * 2 * d->K * sizeof(float));
  p->bn.total = p->bn.off_coef + up256((size_t)4 * d->K * sizeof(float));
  p->total = p->off_bn + p->bn.total;
  return JZ_OK;
}

}  // namespace

extern "C" int jz_conv2d_bn_relu_fwd_workspace_bytes(const jz_conv_desc* desc, size_t* bytes) {
  if (!bytes) return JZ_ERR_NULL;
  ConvBnPlan p;
  int rc = make_conv_bn_plan(desc, &p);
  if (rc != JZ_OK) return rc;
  *bytes = p.total;
  return JZ_OK;
}

extern "C" int jz_conv2d_bn_relu_fwd(const jz_conv_desc* desc, const void* x16, const void* w16, const float* gamma,
                                     const float* beta, float eps, const void* residual16, int relu, void* conv_out16, void* y16,
                                     float* save_mean, float* save_invstd, void* ws, size_t ws_bytes, void* hip_stream) {
  ConvBnPlan p;
  int rc = make_conv_bn_plan(desc, &p);
  if (rc != JZ_OK) return rc;
  if (!(eps >= 0.f)) return JZ_ERR_SHAPE;
  if (!x16 || !w16 || !gamma || !beta || !conv_out16 || !y16 || !save_mean || !save_invstd) return JZ_ERR_NULL;
  if (!ws || ws_bytes < p.total) return JZ_ERR_WORKSPACE;
  if (!jz::aligned16(y16) || !jz::aligned16(ws) || !jz::aligned16(gamma) || !jz::aligned16(beta) || !jz::aligned16(save_mean) ||
      !jz::aligned16(save_invstd) || !jz::aligned16(residual16))
    return JZ_ERR_ALIGN;
  const int64_t rows = p.bn.rows;
  const int C = p.bn.C;
  const size_t nb = (size_t)rows * C * 2, nc = (size_t)C * 4;
  const size_t nx = (size_t)desc->N * desc->H * desc->W * desc->C * 2, nw = (size_t)desc->K * desc->R * desc->S * desc->C * 2;
  if (jz::overlaps(y16, nb, conv_out16, nb) || jz::overlaps(y16, nb, x16, nx) || jz::overlaps(y16, nb, w16, nw) ||
      jz::overlaps(ws, p.total, y16, nb) || jz::overlaps(save_mean, nc, save_invstd, nc) || jz::overlaps(y16, nb, residual16, nb) ||
      jz::overlaps(conv_out16, nb, residual16, nb) || jz::overlaps(ws, p.total, residual16, nb))
    return JZ_ERR_ALIAS;
  for (const float* sv : {save_mean, save_invstd})
    if (jz::overlaps(sv, nc, y16, nb) || jz::overlaps(sv, nc, conv_out16, nb) || jz::overlaps(sv, nc, x16, nx) ||
        jz::overlaps(sv, nc, w16, nw) || jz::overlaps(sv, nc, ws, p.total) || jz::overlaps(sv, nc, residual16, nb))
      return JZ_ERR_ALIAS;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  char* bws = static_cast<char*>(ws) + p.off_bn;
  float* part = reinterpret_cast<float*>(bws + p.bn.off_part);
  float* coef = reinterpret_cast<float*>(bws + p.bn.off_coef);
  // the convolution (its own checks cover x, w, conv_out and its part of the workspace)
  rc = jz::conv_fwd_run(desc, x16, w16, conv_out16, ws, p.conv_ws, p.tiles_m > 0 ? part : nullptr, p.tiles_m, hip_stream);
  if (rc != JZ_OK) return rc;
  const uint4* c = static_cast<const uint4*>(conv_out16);
  int slabs = p.tiles_m;
  if (slabs == 0) {  // this convolution kernel cannot leave the sums: one more pass over its output
    slabs = p.bn.slabs;
    hipLaunchKernelGGL(bn_stats<0>, dim3((unsigned)(slabs * p.bn.csplit)), dim3(BN_THREADS), 0, st, c, nullptr, nullptr, nullptr, nullptr,
                       part, rows, C, p.bn.cpr, p.bn.rpp, p.bn.rows_per_slab, 0, p.bn.csplit);
    if ((rc = jz::launch_status()) != JZ_OK) return rc;
  }
  hipLaunchKernelGGL(bn_fwd_final, dim3((unsigned)((C + BN_FIN_C - 1) / BN_FIN_C)), dim3(BN_THREADS), 0, st, part, slabs, C,
                     1.0 / (double)rows, eps, gamma, beta, save_mean, save_invstd, coef);
  if ((rc = jz::launch_status()) != JZ_OK) return rc;
  const int64_t n_chunks = rows * p.bn.cpr;
  if (residual16)
    hipLaunchKernelGGL(bn_apply<1>, dim3(apply_grid(n_chunks)), dim3(BN_THREADS), 0, st, c, static_cast<const uint4*>(residual16),
                       static_cast<uint4*>(y16), coef, n_chunks, C, p.bn.cpr, relu ? 1 : 0);
  else
    hipLaunchKernelGGL(bn_apply<0>, dim3(apply_grid(n_chunks)), dim3(BN_THREADS), 0, st, c, nullptr, static_cast<uint4*>(y16), coef,
                       n_chunks, C, p.bn.cpr, relu ? 1 : 0);
  return jz::launch_status();
}

// ---- backward-data of a convolution + the backward pass of the batch normalization + ReLU that produced its input ----
// The statistics pass of the normalization's backward (sum g, sum g x^ over g = dz where y > 0) reads dz, y and x; here
// the convolution's epilogue takes the sums while the dz tile is still on chip (it reads the matching y and x tiles), so
// that pass and its launch disappear.
namespace {

struct ConvBnBwdPlan {
  BnPlan bn;            // of the normalization: rows = N*H*W of the convolution's input, C = its channels
  size_t conv_ws = 0;
  int tiles_m = 0;      // > 0: the convolution kernel leaves [tiles_m][2][C] sums; 0: the statistics pass runs
  size_t off_bn = 0, total = 0;
};

int make_conv_bn_bwd_plan(const jz_conv_desc* d, ConvBnBwdPlan* p) {
  int rc = jz::conv_bwd_data_stats_plan(d, &p->conv_ws, &p->tiles_m);
  if (rc != JZ_OK) return rc;
  rc = make_bn_plan((int64_t)d->N * d->H * d->W, d->C, &p->bn);
  if (rc != JZ_OK) return rc;
  const int slabs = p->tiles_m > p->bn.slabs ? p->tiles_m : p->bn.slabs;
  p->off_bn = up256(p->conv_ws);
  p->bn.off_part = 0;
  p->bn.off_coef = up256((size_t)slabs * 2 * d->C * sizeof(float));
  p->bn.total = p->bn.off_coef + up256((size_t)4 * d->C * sizeof(float));
  p->total = p->off_bn + p->bn.total;
  return JZ_OK;
}

}  // namespace

extern "C" int jz_conv2d_bwd_data_bn_relu_bwd_workspace_bytes(const jz_conv_desc* desc, size_t* bytes) {
  if (!bytes) return JZ_ERR_NULL;
  ConvBnBwdPlan p;
  int rc = make_conv_bn_bwd_plan(desc, &p);
  if (rc != JZ_OK) return rc;
  *bytes = p.total;
  return JZ_OK;
}

// block_end false: dz = bwd_data, then the backward of y = relu(bn(x)) for dy = dz.
// block_end true:  y = relu(bn(x) + shortcut) is a residual block's output and bwd_data is one contribution to its gradient:
//                  g = RNE16(bwd_data [+ add]) where y > 0, else 0, goes to `out`, then the backward of bn(x) (no ReLU) for dy = g.
static int conv_bwd_data_bn_bwd(const jz_conv_desc* desc, const void* dy16, const void* w16, const void* bn_x16, const void* bn_y16,
                                const void* add16, bool block_end, const float* gamma, const float* save_mean, const float* save_invstd,
                                void* out16, void* bn_dx16, void* dgamma16, void* dbeta16, void* ws, size_t ws_bytes, void* hip_stream) {
  ConvBnBwdPlan p;
  int rc = make_conv_bn_bwd_plan(desc, &p);
  if (rc != JZ_OK) return rc;
  if (!dy16 || !w16 || !bn_x16 || !bn_y16 || !gamma || !save_mean || !save_invstd || !out16 || !bn_dx16 || !dgamma16 || !dbeta16)
    return JZ_ERR_NULL;
  if (!ws || ws_bytes < p.total) return JZ_ERR_WORKSPACE;
  if (!jz::aligned16(bn_x16) || !jz::aligned16(bn_y16) || !jz::aligned16(add16) || !jz::aligned16(bn_dx16) || !jz::aligned16(ws) ||
      !jz::aligned16(gamma) || !jz::aligned16(save_mean) || !jz::aligned16(save_invstd))
    return JZ_ERR_ALIGN;
  const int64_t rows = p.bn.rows;
  const int C = p.bn.C;
  const size_t nb = (size_t)rows * C * 2, nh = (size_t)C * 2, nc = (size_t)C * 4;
  const int P = (desc->H + 2 * desc->pad_h - desc->R) / desc->stride_h + 1, Q = (desc->W + 2 * desc->pad_w - desc->S) / desc->stride_w + 1;
  const size_t ny = (size_t)desc->N * P * Q * desc->K * 2, nw = (size_t)desc->K * desc->R * desc->S * desc->C * 2;
  // outputs against everything else (the convolution's own checks cover dy, w, its output and its part of the workspace)
  const void* outs[4] = {out16, bn_dx16, dgamma16, dbeta16};
  const size_t outn[4] = {nb, nb, nh, nh};
  const void* ins[8] = {dy16, w16, bn_x16, bn_y16, gamma, save_mean, save_invstd, add16};
  const size_t inn[8] = {ny, nw, nb, nb, nc, nc, nc, add16 ? nb : 0};
  for (int i = 0; i < 4; ++i) {
    for (int j = 0; j < 8; ++j)
      if (inn[j] && jz::overlaps(outs[i], outn[i], ins[j], inn[j])) return JZ_ERR_ALIAS;
    for (int j = i + 1; j < 4; ++j)
      if (jz::overlaps(outs[i], outn[i], outs[j], outn[j])) return JZ_ERR_ALIAS;
    if (jz::overlaps(outs[i], outn[i], ws, p.total)) return JZ_ERR_ALIAS;
  }
  for (int j = 0; j < 8; ++j)
    if (inn[j] && jz::overlaps(ins[j], inn[j], ws, p.total)) return JZ_ERR_ALIAS;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  char* bws = static_cast<char*>(ws) + p.off_bn;
  float* part = reinterpret_cast<float*>(bws + p.bn.off_part);
  float* coef = reinterpret_cast<float*>(bws + p.bn.off_coef);
  jz::BnBwdOperands bn{bn_x16, bn_y16, save_mean, save_invstd};
  bn.block_end = block_end;
  bn.add16 = add16;
  rc = jz::conv_bwd_data_run(desc, dy16, w16, out16, ws, p.conv_ws, p.tiles_m > 0 ? part : nullptr, p.tiles_m, &bn, hip_stream);
  if (rc != JZ_OK) return rc;
  const uint4* x = static_cast<const uint4*>(bn_x16);
  const uint4* y = static_cast<const uint4*>(bn_y16);
  const uint4* dz = static_cast<const uint4*>(out16);
  int slabs = p.tiles_m;
  if (slabs == 0) {  // this convolution kernel cannot leave the sums: the statistics pass, which then also forms g in place
    slabs = p.bn.slabs;
    if (block_end)
      hipLaunchKernelGGL(bn_stats<2>, dim3((unsigned)(slabs * p.bn.csplit)), dim3(BN_THREADS), 0, st, x, y, dz, save_mean, save_invstd, part,
                         rows, C, p.bn.cpr, p.bn.rpp, p.bn.rows_per_slab, 0, p.bn.csplit, static_cast<const uint4*>(add16),
                         static_cast<uint4*>(out16));
    else
      hipLaunchKernelGGL(bn_stats<1>, dim3((unsigned)(slabs * p.bn.csplit)), dim3(BN_THREADS), 0, st, x, y, dz, save_mean, save_invstd, part,
                         rows, C, p.bn.cpr, p.bn.rpp, p.bn.rows_per_slab, 1, p.bn.csplit);
    if ((rc = jz::launch_status()) != JZ_OK) return rc;
  }
  hipLaunchKernelGGL(bn_bwd_final, dim3((unsigned)((C + BN_FIN_C - 1) / BN_FIN_C)), dim3(BN_THREADS), 0, st, part, slabs, C,
                     1.0 / (double)rows, gamma, save_mean, save_invstd, static_cast<unsigned short*>(dgamma16),
                     static_cast<unsigned short*>(dbeta16), coef);
  if ((rc = jz::launch_status()) != JZ_OK) return rc;
  const int64_t n_chunks = rows * p.bn.cpr;
  hipLaunchKernelGGL(bn_bwd_apply, dim3(apply_grid(n_chunks)), dim3(BN_THREADS), 0, st, x, block_end ? nullptr : y, dz,
                     static_cast<uint4*>(bn_dx16), coef, n_chunks, C, p.bn.cpr, block_end ? 0 : 1);
  return jz::launch_status();
}

extern "C" int jz_conv2d_bwd_data_bn_relu_bwd(const jz_conv_desc* desc, const void* dy16, const void* w16, const void* bn_x16,
                                              const void* bn_y16, const float* gamma, const float* save_mean,
                                              const float* save_invstd, void* dz16, void* bn_dx16, void* dgamma16, void* dbeta16,
                                              void* ws, size_t ws_bytes, void* hip_stream) {
  return conv_bwd_data_bn_bwd(desc, dy16, w16, bn_x16, bn_y16, nullptr, false, gamma, save_mean, save_invstd, dz16, bn_dx16, dgamma16,
                              dbeta16, ws, ws_bytes, hip_stream);
}

extern "C" int jz_conv2d_bwd_data_block_end_bwd(const jz_conv_desc* desc, const void* dy16, const void* w16, const void* dyb16,
                                                const void* bn_x16, const void* y_out16, const float* gamma, const float* save_mean,
                                                const float* save_invstd, void* g16, void* bn_dx16, void* dgamma16, void* dbeta16,
                                                void* ws, size_t ws_bytes, void* hip_stream) {
  return conv_bwd_data_bn_bwd(desc, dy16, w16, bn_x16, y_out16, dyb16, true, gamma, save_mean, save_invstd, g16, bn_dx16, dgamma16,
                              dbeta16, ws, ws_bytes, hip_stream);
}
