// The small layers between the convolutions of a ResNet-style network, on FP16 NHWC tensors (the storage type of
// every forward / backward tensor in Section 4.1 of Jia et al. 2018): residual add (+ ReLU) and the ReLU gradient,
// max pooling and global average pooling with their gradients, bias add and bias gradient, and the loss-scaled
// gradient of softmax cross-entropy.  All of them are HBM-bound: one pass, 16-byte accesses along the channel axis,
// FP32 arithmetic, one rounding to FP16 on the store, no atomics (results do not depend on the launch).
#include "jz_internal.h"

namespace {

constexpr int LY_THREADS = 256;
constexpr unsigned LY_MAX_GRID = 256 * 32;

__device__ __forceinline__ void unpack8(const uint4& v, float (&f)[8]) {
  const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    _Float16 lo, hi;
    const unsigned short l = (unsigned short)(w[i] & 0xffffu), h = (unsigned short)(w[i] >> 16);
    __builtin_memcpy(&lo, &l, 2);
    __builtin_memcpy(&hi, &h, 2);
    f[2 * i] = (float)lo;
    f[2 * i + 1] = (float)hi;
  }
}
__device__ __forceinline__ unsigned half_bits(float f) {
  _Float16 x = (_Float16)f;  // round to nearest even, overflow to Inf
  unsigned short h;
  __builtin_memcpy(&h, &x, 2);
  return h;
}
__device__ __forceinline__ uint4 pack8(const float (&f)[8]) {
  uint4 v;
  v.x = half_bits(f[0]) | (half_bits(f[1]) << 16);
  v.y = half_bits(f[2]) | (half_bits(f[3]) << 16);
  v.z = half_bits(f[4]) | (half_bits(f[5]) << 16);
  v.w = half_bits(f[6]) | (half_bits(f[7]) << 16);
  return v;
}
__device__ __forceinline__ float half_to_float(unsigned short h) {
  _Float16 x;
  __builtin_memcpy(&x, &h, 2);
  return (float)x;
}

unsigned grid_for(int64_t items) {
  int64_t g = (items + LY_THREADS - 1) / LY_THREADS;
  if (g < 1) g = 1;
  return (unsigned)(g > LY_MAX_GRID ? LY_MAX_GRID : g);
}

// ---- residual add, ReLU gradient ---------------------------------------------------------------------------------
template <int RELU>
__global__ __launch_bounds__(LY_THREADS) void add_kernel(const uint4* __restrict__ a, const uint4* __restrict__ b,
                                                         uint4* __restrict__ y, int64_t n8) {
  for (int64_t i = (int64_t)blockIdx.x * LY_THREADS + threadIdx.x; i < n8; i += (int64_t)gridDim.x * LY_THREADS) {
    float fa[8], fb[8];
    unpack8(a[i], fa);
    unpack8(b[i], fb);
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      fa[k] += fb[k];  // exact in FP32
      if (RELU) fa[k] = fa[k] > 0.f ? fa[k] : 0.f;
    }
    y[i] = pack8(fa);
  }
}

// dx = (y > 0) ? RNE16(dya + dyb) : 0: a block output whose gradient arrives as two contributions (the next block's
// first convolution and its shortcut); the sum is exact in FP32 and rounded once, as a separate add would round it
__global__ __launch_bounds__(LY_THREADS) void relu_bwd_sum_kernel(const uint4* __restrict__ y, const uint4* __restrict__ dya,
                                                                  const uint4* __restrict__ dyb, uint4* __restrict__ dx, int64_t n8) {
  for (int64_t i = (int64_t)blockIdx.x * LY_THREADS + threadIdx.x; i < n8; i += (int64_t)gridDim.x * LY_THREADS) {
    float fy[8], fa[8], fb[8];
    unpack8(y[i], fy);
    unpack8(dya[i], fa);
    unpack8(dyb[i], fb);
    float s[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) s[k] = fa[k] + fb[k];
    const uint4 o = pack8(s);
    unsigned ow[4] = {o.x, o.y, o.z, o.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) ow[k] = (fy[2 * k] > 0.f ? (ow[k] & 0xffffu) : 0u) | (fy[2 * k + 1] > 0.f ? (ow[k] & 0xffff0000u) : 0u);
    dx[i] = make_uint4(ow[0], ow[1], ow[2], ow[3]);
  }
}

__global__ __launch_bounds__(LY_THREADS) void relu_bwd_kernel(const uint4* __restrict__ y, const uint4* __restrict__ dy,
                                                              uint4* __restrict__ dx, int64_t n8) {
  for (int64_t i = (int64_t)blockIdx.x * LY_THREADS + threadIdx.x; i < n8; i += (int64_t)gridDim.x * LY_THREADS) {
    const uint4 m = y[i], g = dy[i];
    const unsigned mw[4] = {m.x, m.y, m.z, m.w}, gw[4] = {g.x, g.y, g.z, g.w};
    unsigned o[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      // positive FP16: sign clear and not zero (NaN counts as not positive, like the comparison y > 0)
      const unsigned lo = mw[k] & 0xffffu, hi = mw[k] >> 16;
      const bool plo = lo != 0 && lo <= 0x7c00u, phi = hi != 0 && hi <= 0x7c00u;
      o[k] = (plo ? (gw[k] & 0xffffu) : 0u) | (phi ? (gw[k] & 0xffff0000u) : 0u);
    }
    dx[i] = make_uint4(o[0], o[1], o[2], o[3]);
  }
}

// ---- max pooling ---------------------------------------------------------------------------------------------------
struct PoolGeom {
  int N, H, W, C8, P, Q, window, stride, pad;
};

// WIN > 0: window size known at compile time (loops unrolled, the window's loads in flight together); 0: g.window
template <int WIN>
__global__ __launch_bounds__(LY_THREADS) void maxpool_fwd_kernel(const uint4* __restrict__ x, uint4* __restrict__ y,
                                                                 uint2* __restrict__ arg, PoolGeom g) {
  const int window = WIN > 0 ? WIN : g.window;
  const int64_t total = (int64_t)g.N * g.P * g.Q * g.C8;
  for (int64_t i = (int64_t)blockIdx.x * LY_THREADS + threadIdx.x; i < total; i += (int64_t)gridDim.x * LY_THREADS) {
    const int c = (int)(i % g.C8);
    int64_t t = i / g.C8;
    const int q = (int)(t % g.Q);
    t /= g.Q;
    const int p = (int)(t % g.P);
    const int n = (int)(t / g.P);
    float best[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    unsigned win[8] = {0, 0, 0, 0, 0, 0, 0, 0};  // position r * window + s of the first maximum
    bool have = false;
#pragma unroll(WIN > 0 ? WIN : 1)
    for (int r = 0; r < window; ++r) {
      const int h = p * g.stride - g.pad + r;
#pragma unroll(WIN > 0 ? WIN : 1)
      for (int s = 0; s < window; ++s) {
        const int w = q * g.stride - g.pad + s;
        // a position outside the image is read at the nearest inside one and ignored: no branch around the load
        const bool ok = h >= 0 && h < g.H && w >= 0 && w < g.W;
        const int hc = h < 0 ? 0 : (h >= g.H ? g.H - 1 : h), wc = w < 0 ? 0 : (w >= g.W ? g.W - 1 : w);
        float v[8];
        unpack8(x[(((int64_t)n * g.H + hc) * g.W + wc) * g.C8 + c], v);
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const bool better = ok && (!have || v[k] > best[k]);
          best[k] = better ? v[k] : best[k];
          win[k] = better ? (unsigned)(r * window + s) : win[k];
        }
        have = have || ok;
      }
    }
    y[i] = pack8(best);
    if (arg)
      arg[i] = make_uint2(win[0] | (win[1] << 8) | (win[2] << 16) | (win[3] << 24), win[4] | (win[5] << 8) | (win[6] << 16) | (win[7] << 24));
  }
}

// one thread per input position and 8 channels: it looks at every window that contains the position, finds that
// window's first maximum again and takes the window's dy if the position is it
template <int WIN>
__global__ __launch_bounds__(LY_THREADS) void maxpool_bwd_kernel(const uint4* __restrict__ x, const uint4* __restrict__ dy,
                                                                 uint4* __restrict__ dx, PoolGeom g) {
  const int window = WIN > 0 ? WIN : g.window;
  const int64_t total = (int64_t)g.N * g.H * g.W * g.C8;
  for (int64_t i = (int64_t)blockIdx.x * LY_THREADS + threadIdx.x; i < total; i += (int64_t)gridDim.x * LY_THREADS) {
    const int c = (int)(i % g.C8);
    int64_t t = i / g.C8;
    const int w0 = (int)(t % g.W);
    t /= g.W;
    const int h0 = (int)(t % g.H);
    const int n = (int)(t / g.H);
    float acc[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) acc[k] = 0.f;
    // windows p with p*stride - pad <= h0 <= p*stride - pad + window - 1
    int p_lo = h0 + g.pad - window + 1;
    p_lo = p_lo <= 0 ? 0 : (p_lo + g.stride - 1) / g.stride;
    int p_hi = (h0 + g.pad) / g.stride;
    if (p_hi > g.P - 1) p_hi = g.P - 1;
    int q_lo = w0 + g.pad - window + 1;
    q_lo = q_lo <= 0 ? 0 : (q_lo + g.stride - 1) / g.stride;
    int q_hi = (w0 + g.pad) / g.stride;
    if (q_hi > g.Q - 1) q_hi = g.Q - 1;
    for (int p = p_lo; p <= p_hi; ++p)
      for (int q = q_lo; q <= q_hi; ++q) {
        float best[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        bool mine[8] = {false, false, false, false, false, false, false, false};
        bool have = false;
#pragma unroll(WIN > 0 ? WIN : 1)
        for (int r = 0; r < window; ++r) {
          const int h = p * g.stride - g.pad + r;
#pragma unroll(WIN > 0 ? WIN : 1)
          for (int s = 0; s < window; ++s) {
            const int w = q * g.stride - g.pad + s;
            const bool ok = h >= 0 && h < g.H && w >= 0 && w < g.W;
            const int hc = h < 0 ? 0 : (h >= g.H ? g.H - 1 : h), wc = w < 0 ? 0 : (w >= g.W ? g.W - 1 : w);
            float v[8];
            unpack8(x[(((int64_t)n * g.H + hc) * g.W + wc) * g.C8 + c], v);
            const bool here = h == h0 && w == w0;
#pragma unroll
            for (int k = 0; k < 8; ++k) {
              const bool better = ok && (!have || v[k] > best[k]);
              best[k] = better ? v[k] : best[k];
              mine[k] = better ? here : mine[k];
            }
            have = have || ok;
          }
        }
        float gy[8];
        unpack8(dy[(((int64_t)n * g.P + p) * g.Q + q) * g.C8 + c], gy);
#pragma unroll
        for (int k = 0; k < 8; ++k) acc[k] += (have && mine[k]) ? gy[k] : 0.f;
      }
    dx[i] = pack8(acc);
  }
}

// the same gather from the winners the forward pass saved: nothing is re-derived, x is not read
__global__ __launch_bounds__(LY_THREADS) void maxpool_bwd_arg_kernel(const uint2* __restrict__ arg, const uint4* __restrict__ dy,
                                                                     uint4* __restrict__ dx, PoolGeom g) {
  const int64_t total = (int64_t)g.N * g.H * g.W * g.C8;
  for (int64_t i = (int64_t)blockIdx.x * LY_THREADS + threadIdx.x; i < total; i += (int64_t)gridDim.x * LY_THREADS) {
    const int c = (int)(i % g.C8);
    int64_t t = i / g.C8;
    const int w0 = (int)(t % g.W);
    t /= g.W;
    const int h0 = (int)(t % g.H);
    const int n = (int)(t / g.H);
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    int p_lo = h0 + g.pad - g.window + 1;
    p_lo = p_lo <= 0 ? 0 : (p_lo + g.stride - 1) / g.stride;
    int p_hi = (h0 + g.pad) / g.stride;
    if (p_hi > g.P - 1) p_hi = g.P - 1;
    int q_lo = w0 + g.pad - g.window + 1;
    q_lo = q_lo <= 0 ? 0 : (q_lo + g.stride - 1) / g.stride;
    int q_hi = (w0 + g.pad) / g.stride;
    if (q_hi > g.Q - 1) q_hi = g.Q - 1;
    for (int p = p_lo; p <= p_hi; ++p)
      for (int q = q_lo; q <= q_hi; ++q) {
        const unsigned me = (unsigned)((h0 - (p * g.stride - g.pad)) * g.window + (w0 - (q * g.stride - g.pad)));
        const int64_t o = (((int64_t)n * g.P + p) * g.Q + q) * g.C8 + c;
        const uint2 a = arg[o];
        float gy[8];
        unpack8(dy[o], gy);
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const unsigned wk = ((k < 4 ? a.x : a.y) >> (8 * (k & 3))) & 0xffu;
          acc[k] += wk == me ? gy[k] : 0.f;
        }
      }
    dx[i] = pack8(acc);
  }
}

// ---- global average pooling ----------------------------------------------------------------------------------------
__global__ __launch_bounds__(LY_THREADS) void avgpool_fwd_kernel(const uint4* __restrict__ x, uint4* __restrict__ y, int N, int HW,
                                                                 int C8) {
  const int64_t total = (int64_t)N * C8;
  for (int64_t i = (int64_t)blockIdx.x * LY_THREADS + threadIdx.x; i < total; i += (int64_t)gridDim.x * LY_THREADS) {
    const int c = (int)(i % C8);
    const int64_t n = i / C8;
    float acc[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) acc[k] = 0.f;
    for (int j = 0; j < HW; ++j) {
      float v[8];
      unpack8(x[(n * HW + j) * C8 + c], v);
#pragma unroll
      for (int k = 0; k < 8; ++k) acc[k] += v[k];
    }
    const float d = (float)HW;
#pragma unroll
    for (int k = 0; k < 8; ++k) acc[k] = acc[k] / d;
    y[i] = pack8(acc);
  }
}

__global__ __launch_bounds__(LY_THREADS) void avgpool_bwd_kernel(const uint4* __restrict__ dy, uint4* __restrict__ dx, int N, int HW,
                                                                 int C8) {
  const int64_t total = (int64_t)N * HW * C8;
  const float d = (float)HW;
  for (int64_t i = (int64_t)blockIdx.x * LY_THREADS + threadIdx.x; i < total; i += (int64_t)gridDim.x * LY_THREADS) {
    const int c = (int)(i % C8);
    const int64_t n = i / ((int64_t)HW * C8);
    float v[8];
    unpack8(dy[n * C8 + c], v);
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] = v[k] / d;
    dx[i] = pack8(v);
  }
}

// ---- bias ----------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(LY_THREADS) void bias_add_kernel(const uint4* __restrict__ y, const uint4* __restrict__ b,
                                                              uint4* __restrict__ out, int64_t rows, int C8) {
  const int64_t total = rows * C8;
  for (int64_t i = (int64_t)blockIdx.x * LY_THREADS + threadIdx.x; i < total; i += (int64_t)gridDim.x * LY_THREADS) {
    float fa[8], fb[8];
    unpack8(y[i], fa);
    unpack8(b[i % C8], fb);
#pragma unroll
    for (int k = 0; k < 8; ++k) fa[k] += fb[k];
    out[i] = pack8(fa);
  }
}

// one workgroup per 4 chunks of 8 channels; 64 row lanes each walk the rows with stride 64, then a fixed-order tree
constexpr int BG_CHUNKS = 4;
__global__ __launch_bounds__(LY_THREADS) void bias_grad_kernel(const uint4* __restrict__ dy, uint4* __restrict__ db, int64_t rows,
                                                               int C8) {
  __shared__ float red[64][BG_CHUNKS][8 + 1];
  const int cl = threadIdx.x % BG_CHUNKS, rl = threadIdx.x / BG_CHUNKS;
  const int c = blockIdx.x * BG_CHUNKS + cl;
  float acc[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) acc[k] = 0.f;
  if (c < C8)
    for (int64_t r = rl; r < rows; r += 64) {
      float v[8];
      unpack8(dy[r * C8 + c], v);
#pragma unroll
      for (int k = 0; k < 8; ++k) acc[k] += v[k];
    }
#pragma unroll
  for (int k = 0; k < 8; ++k) red[rl][cl][k] = acc[k];
  __syncthreads();
  for (int half = 32; half >= 1; half >>= 1) {
    if (rl < half) {
#pragma unroll
      for (int k = 0; k < 8; ++k) red[rl][cl][k] += red[rl + half][cl][k];
    }
    __syncthreads();
  }
  if (rl == 0 && c < C8) {
#pragma unroll
    for (int k = 0; k < 8; ++k) acc[k] = red[0][cl][k];
    db[c] = pack8(acc);
  }
}

// ---- softmax cross-entropy: loss per sample and loss-scaled gradient of the batch mean -----------------------------
__device__ __forceinline__ float block_max(float v, float* red) {
  for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}
__device__ __forceinline__ float block_add(float v, float* red) {
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}

__global__ __launch_bounds__(LY_THREADS) void softmax_xent_kernel(const unsigned short* __restrict__ z, const int* __restrict__ labels,
                                                                  unsigned short* __restrict__ dz, float* __restrict__ loss, int rows,
                                                                  int K, float scale, const jz_loss_scale_state* __restrict__ state) {
  __shared__ float red[4];
  const int n = blockIdx.x;
  const unsigned short* zr = z + (int64_t)n * K;
  if (state) scale = state->scale;
  const int label = labels[n];
  const bool valid = label >= 0 && label < K;
  float m = -INFINITY;
  for (int j = threadIdx.x; j < K; j += LY_THREADS) m = fmaxf(m, half_to_float(zr[j]));
  m = block_max(m, red);
  float se = 0.f;
  for (int j = threadIdx.x; j < K; j += LY_THREADS) se += expf(half_to_float(zr[j]) - m);
  se = block_add(se, red);
  const float f = scale / (float)rows;
  for (int j = threadIdx.x; j < K; j += LY_THREADS) {
    float p = expf(half_to_float(zr[j]) - m) / se;
    if (j == label) p -= 1.0f;
    dz[(int64_t)n * K + j] = valid ? (unsigned short)half_bits(f * p) : (unsigned short)0;
  }
  if (threadIdx.x == 0) loss[n] = valid ? (logf(se) + m) - half_to_float(zr[label]) : __int_as_float(0x7fc00000);
}

int check_elems(int64_t n) {
  if (n < 0 || (n & 7)) return JZ_ERR_SHAPE;
  if (n > (int64_t)1 << 40) return JZ_ERR_UNSUPPORTED;
  return JZ_OK;
}

int make_pool(int N, int H, int W, int C, int window, int stride, int pad, PoolGeom* g) {
  if (N < 0 || H < 1 || W < 1 || C < 1 || (C & 7) || window < 1 || stride < 1 || pad < 0 || pad >= window || window > H + 2 * pad ||
      window > W + 2 * pad)
    return JZ_ERR_SHAPE;
  if (window > 16) return JZ_ERR_UNSUPPORTED;
  *g = PoolGeom{N, H, W, C / 8, (H + 2 * pad - window) / stride + 1, (W + 2 * pad - window) / stride + 1, window, stride, pad};
  return JZ_OK;
}

}  // namespace

extern "C" int jz_add_fwd(int64_t n, const void* a16, const void* b16, int relu, void* y16, void* hip_stream) {
  int rc = check_elems(n);
  if (rc != JZ_OK) return rc;
  if (n == 0) return JZ_OK;
  if (!a16 || !b16 || !y16) return JZ_ERR_NULL;
  if (!jz::aligned16(a16) || !jz::aligned16(b16) || !jz::aligned16(y16)) return JZ_ERR_ALIGN;
  // in place (y16 == a16 or y16 == b16) is allowed: every element is read before it is written, by the same thread
  const size_t nb = (size_t)n * 2;
  if ((y16 != a16 && jz::overlaps(y16, nb, a16, nb)) || (y16 != b16 && jz::overlaps(y16, nb, b16, nb))) return JZ_ERR_ALIAS;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const uint4 *a = static_cast<const uint4*>(a16), *b = static_cast<const uint4*>(b16);
  if (relu)
    hipLaunchKernelGGL(add_kernel<1>, dim3(grid_for(n / 8)), dim3(LY_THREADS), 0, st, a, b, static_cast<uint4*>(y16), n / 8);
  else
    hipLaunchKernelGGL(add_kernel<0>, dim3(grid_for(n / 8)), dim3(LY_THREADS), 0, st, a, b, static_cast<uint4*>(y16), n / 8);
  return jz::launch_status();
}

extern "C" int jz_relu_bwd(int64_t n, const void* y16, const void* dy16, void* dx16, void* hip_stream) {
  int rc = check_elems(n);
  if (rc != JZ_OK) return rc;
  if (n == 0) return JZ_OK;
  if (!y16 || !dy16 || !dx16) return JZ_ERR_NULL;
  if (!jz::aligned16(y16) || !jz::aligned16(dy16) || !jz::aligned16(dx16)) return JZ_ERR_ALIGN;
  const size_t nb = (size_t)n * 2;
  if (jz::overlaps(dx16, nb, y16, nb) || (dx16 != dy16 && jz::overlaps(dx16, nb, dy16, nb))) return JZ_ERR_ALIAS;
  hipLaunchKernelGGL(relu_bwd_kernel, dim3(grid_for(n / 8)), dim3(LY_THREADS), 0, static_cast<hipStream_t>(hip_stream),
                     static_cast<const uint4*>(y16), static_cast<const uint4*>(dy16), static_cast<uint4*>(dx16), n / 8);
  return jz::launch_status();
}

extern "C" int jz_relu_bwd_sum(int64_t n, const void* y16, const void* dya16, const void* dyb16, void* dx16, void* hip_stream) {
  int rc = check_elems(n);
  if (rc != JZ_OK) return rc;
  if (n == 0) return JZ_OK;
  if (!y16 || !dya16 || !dyb16 || !dx16) return JZ_ERR_NULL;
  if (!jz::aligned16(y16) || !jz::aligned16(dya16) || !jz::aligned16(dyb16) || !jz::aligned16(dx16)) return JZ_ERR_ALIGN;
  const size_t nb = (size_t)n * 2;
  if (jz::overlaps(dx16, nb, y16, nb) || (dx16 != dya16 && jz::overlaps(dx16, nb, dya16, nb)) ||
      (dx16 != dyb16 && jz::overlaps(dx16, nb, dyb16, nb)))
    return JZ_ERR_ALIAS;
  hipLaunchKernelGGL(relu_bwd_sum_kernel, dim3(grid_for(n / 8)), dim3(LY_THREADS), 0, static_cast<hipStream_t>(hip_stream),
                     static_cast<const uint4*>(y16), static_cast<const uint4*>(dya16), static_cast<const uint4*>(dyb16),
                     static_cast<uint4*>(dx16), n / 8);
  return jz::launch_status();
}

extern "C" int jz_maxpool_fwd(int N, int H, int W, int C, int window, int stride, int pad, const void* x16, void* y16,
                              void* arg8, void* hip_stream) {
  PoolGeom g;
  int rc = make_pool(N, H, W, C, window, stride, pad, &g);
  if (rc != JZ_OK) return rc;
  if (N == 0) return JZ_OK;
  if (!x16 || !y16) return JZ_ERR_NULL;
  if (!jz::aligned16(x16) || !jz::aligned16(y16) || (reinterpret_cast<uintptr_t>(arg8) & 7u)) return JZ_ERR_ALIGN;
  const size_t nx = (size_t)N * H * W * C * 2, ny = (size_t)N * g.P * g.Q * C * 2;
  if (jz::overlaps(x16, nx, y16, ny) || jz::overlaps(arg8, ny / 2, x16, nx) || jz::overlaps(arg8, ny / 2, y16, ny)) return JZ_ERR_ALIAS;
  const dim3 grid(grid_for((int64_t)N * g.P * g.Q * g.C8));
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const uint4* x = static_cast<const uint4*>(x16);
  uint4* y = static_cast<uint4*>(y16);
  uint2* arg = static_cast<uint2*>(arg8);
  if (window == 3)
    hipLaunchKernelGGL(maxpool_fwd_kernel<3>, grid, dim3(LY_THREADS), 0, st, x, y, arg, g);
  else if (window == 2)
    hipLaunchKernelGGL(maxpool_fwd_kernel<2>, grid, dim3(LY_THREADS), 0, st, x, y, arg, g);
  else
    hipLaunchKernelGGL(maxpool_fwd_kernel<0>, grid, dim3(LY_THREADS), 0, st, x, y, arg, g);
  return jz::launch_status();
}

extern "C" int jz_maxpool_bwd(int N, int H, int W, int C, int window, int stride, int pad, const void* x16, const void* arg8,
                              const void* dy16, void* dx16, void* hip_stream) {
  PoolGeom g;
  int rc = make_pool(N, H, W, C, window, stride, pad, &g);
  if (rc != JZ_OK) return rc;
  if (N == 0) return JZ_OK;
  if ((!x16 && !arg8) || !dy16 || !dx16) return JZ_ERR_NULL;
  if (!jz::aligned16(x16) || !jz::aligned16(dy16) || !jz::aligned16(dx16) || (reinterpret_cast<uintptr_t>(arg8) & 7u)) return JZ_ERR_ALIGN;
  const size_t nx = (size_t)N * H * W * C * 2, ny = (size_t)N * g.P * g.Q * C * 2;
  if (jz::overlaps(dx16, nx, x16, nx) || jz::overlaps(dx16, nx, dy16, ny) || jz::overlaps(dx16, nx, arg8, ny / 2)) return JZ_ERR_ALIAS;
  const dim3 grid(grid_for((int64_t)N * H * W * g.C8));
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const uint4 *x = static_cast<const uint4*>(x16), *dy = static_cast<const uint4*>(dy16);
  uint4* dx = static_cast<uint4*>(dx16);
  if (arg8)  // the winners are known: x is not needed
    hipLaunchKernelGGL(maxpool_bwd_arg_kernel, grid, dim3(LY_THREADS), 0, st, static_cast<const uint2*>(arg8), dy, dx, g);
  else if (window == 3)
    hipLaunchKernelGGL(maxpool_bwd_kernel<3>, grid, dim3(LY_THREADS), 0, st, x, dy, dx, g);
  else if (window == 2)
    hipLaunchKernelGGL(maxpool_bwd_kernel<2>, grid, dim3(LY_THREADS), 0, st, x, dy, dx, g);
  else
    hipLaunchKernelGGL(maxpool_bwd_kernel<0>, grid, dim3(LY_THREADS), 0, st, x, dy, dx, g);
  return jz::launch_status();
}

extern "C" int jz_avgpool_fwd(int N, int HW, int C, const void* x16, void* y16, void* hip_stream) {
  if (N < 0 || HW < 1 || C < 1 || (C & 7)) return JZ_ERR_SHAPE;
  if (N == 0) return JZ_OK;
  if (!x16 || !y16) return JZ_ERR_NULL;
  if (!jz::aligned16(x16) || !jz::aligned16(y16)) return JZ_ERR_ALIGN;
  if (jz::overlaps(x16, (size_t)N * HW * C * 2, y16, (size_t)N * C * 2)) return JZ_ERR_ALIAS;
  hipLaunchKernelGGL(avgpool_fwd_kernel, dim3(grid_for((int64_t)N * (C / 8))), dim3(LY_THREADS), 0,
                     static_cast<hipStream_t>(hip_stream), static_cast<const uint4*>(x16), static_cast<uint4*>(y16), N, HW, C / 8);
  return jz::launch_status();
}

extern "C" int jz_avgpool_bwd(int N, int HW, int C, const void* dy16, void* dx16, void* hip_stream) {
  if (N < 0 || HW < 1 || C < 1 || (C & 7)) return JZ_ERR_SHAPE;
  if (N == 0) return JZ_OK;
  if (!dy16 || !dx16) return JZ_ERR_NULL;
  if (!jz::aligned16(dy16) || !jz::aligned16(dx16)) return JZ_ERR_ALIGN;
  if (jz::overlaps(dx16, (size_t)N * HW * C * 2, dy16, (size_t)N * C * 2)) return JZ_ERR_ALIAS;
  hipLaunchKernelGGL(avgpool_bwd_kernel, dim3(grid_for((int64_t)N * HW * (C / 8))), dim3(LY_THREADS), 0,
                     static_cast<hipStream_t>(hip_stream), static_cast<const uint4*>(dy16), static_cast<uint4*>(dx16), N, HW, C / 8);
  return jz::launch_status();
}

extern "C" int jz_bias_add(int64_t rows, int C, const void* y16, const void* b16, void* out16, void* hip_stream) {
  if (rows < 0 || C < 1 || (C & 7)) return JZ_ERR_SHAPE;
  if (rows == 0) return JZ_OK;
  if (!y16 || !b16 || !out16) return JZ_ERR_NULL;
  if (!jz::aligned16(y16) || !jz::aligned16(b16) || !jz::aligned16(out16)) return JZ_ERR_ALIGN;
  const size_t nb = (size_t)rows * C * 2;
  if ((out16 != y16 && jz::overlaps(out16, nb, y16, nb)) || jz::overlaps(out16, nb, b16, (size_t)C * 2)) return JZ_ERR_ALIAS;
  hipLaunchKernelGGL(bias_add_kernel, dim3(grid_for(rows * (C / 8))), dim3(LY_THREADS), 0, static_cast<hipStream_t>(hip_stream),
                     static_cast<const uint4*>(y16), static_cast<const uint4*>(b16), static_cast<uint4*>(out16), rows, C / 8);
  return jz::launch_status();
}

extern "C" int jz_bias_grad(int64_t rows, int C, const void* dy16, void* db16, void* hip_stream) {
  if (rows < 0 || C < 1 || (C & 7)) return JZ_ERR_SHAPE;
  if (!dy16 && rows > 0) return JZ_ERR_NULL;
  if (!db16) return JZ_ERR_NULL;
  if (!jz::aligned16(dy16) || !jz::aligned16(db16)) return JZ_ERR_ALIGN;
  if (jz::overlaps(db16, (size_t)C * 2, dy16, (size_t)rows * C * 2)) return JZ_ERR_ALIAS;
  const int C8 = C / 8;
  hipLaunchKernelGGL(bias_grad_kernel, dim3((unsigned)((C8 + BG_CHUNKS - 1) / BG_CHUNKS)), dim3(LY_THREADS), 0,
                     static_cast<hipStream_t>(hip_stream), static_cast<const uint4*>(dy16), static_cast<uint4*>(db16), rows, C8);
  return jz::launch_status();
}

extern "C" int jz_softmax_xent_bwd(int rows, int classes, const void* z16, const int* labels_dev, float loss_scale,
                                   const jz_loss_scale_state* state_dev, void* dz16, float* loss_dev, void* hip_stream) {
  if (rows < 0 || classes < 1) return JZ_ERR_SHAPE;
  if (!state_dev && (!(loss_scale > 0.0f) || !(loss_scale < 3.0e38f))) return JZ_ERR_SHAPE;
  if (rows == 0) return JZ_OK;
  if (!z16 || !labels_dev || !dz16 || !loss_dev) return JZ_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(z16) & 1u) || (reinterpret_cast<uintptr_t>(dz16) & 1u) ||
      (reinterpret_cast<uintptr_t>(labels_dev) & 3u) || (reinterpret_cast<uintptr_t>(loss_dev) & 3u) ||
      (reinterpret_cast<uintptr_t>(state_dev) & 7u))
    return JZ_ERR_ALIGN;
  const size_t nb = (size_t)rows * classes * 2;
  if (jz::overlaps(dz16, nb, z16, nb) || jz::overlaps(dz16, nb, labels_dev, (size_t)rows * 4) ||
      jz::overlaps(dz16, nb, loss_dev, (size_t)rows * 4) || jz::overlaps(loss_dev, (size_t)rows * 4, z16, nb) ||
      jz::overlaps(loss_dev, (size_t)rows * 4, labels_dev, (size_t)rows * 4) ||
      jz::overlaps(state_dev, sizeof(jz_loss_scale_state), dz16, nb) ||
      jz::overlaps(state_dev, sizeof(jz_loss_scale_state), loss_dev, (size_t)rows * 4))
    return JZ_ERR_ALIAS;
  hipLaunchKernelGGL(softmax_xent_kernel, dim3((unsigned)rows), dim3(LY_THREADS), 0, static_cast<hipStream_t>(hip_stream),
                     static_cast<const unsigned short*>(z16), labels_dev, static_cast<unsigned short*>(dz16), loss_dev, rows, classes,
                     loss_scale, state_dev);
  return jz::launch_status();
}
