// Mixed-precision LARS update (Jia et al. 2018, Section 4.1, Eq. 1, Fig. 2) for gfx950.
//
// fp16 loss-scaled gradients and the fp32 master weights are widened, the layer-wise rate
// rho_t = eta*||w_t||/||g_t|| is formed, the momentum step is taken on the fp32 master copy and the
// result is narrowed to fp16 for the next forward pass.  The whole thing is HBM-bound (20 bytes per
// parameter must move), so it is organised as three stream-ordered launches over a fused flat buffer:
//
//   lars_reduce    one workgroup per chunk (<= LARS_CH elements inside one tensor): fp64 partial sums of
//                  g16^2 (and of w^2, unless the workspace still holds them from the previous update) and a
//                  non-finite flag, stored per chunk (no atomics => deterministic)
//   lars_finalize  one workgroup per tensor: adds that tensor's chunk partials in index order, forms
//                  lr*rho_t, ORs the chunk flags
//   lars_update    one workgroup per chunk, walking the buffer in the opposite direction so that the
//                  tail the reduce pass touched last is still in the last-level cache; skips everything
//                  when any tensor raised the flag.  While writing w it accumulates the chunk's sum of w^2,
//                  which the next update's reduce pass then need not read w for.
//
// When the kernels that produce the gradients also leave each tensor's sum of squares (jz_sumsq.h), the first two
// launches have nothing left to do at update time and the update is one launch ("presummed"):
//
//   lars_begin       at the start of a step, one workgroup per tensor: adds the partial sums of w^2 the last update left
//                    (or, for a fresh workspace, squares the tensor itself), clears the tensor's gradient sink
//   lars_grad_sumsq  the reduce pass for the tensors no other kernel covers (batch-norm scale / shift, bias), any time
//                    after their gradients exist
//   lars_update<true>  every wavefront forms lr*rho_t of its chunk's tensor itself from the sink and the sum lars_begin
//                    left; otherwise the same kernel
#include <hip/hip_runtime.h>

#include <mutex>
#include <vector>

#include "jz_internal.h"
#include "jz_sumsq.h"

namespace {

#ifndef JZ_LARS_CH
#define JZ_LARS_CH 4096
#endif
constexpr int LARS_CH = JZ_LARS_CH;  // elements per chunk; a multiple of 2048 (8 per thread and pass)
constexpr int LARS_THREADS = 256;
constexpr int LARS_WAVES = LARS_THREADS / 64;  // every wavefront of a chunk keeps its own partial sums
constexpr uint64_t LARS_MAGIC = 0x4a5a4c4152533031ull;  // "JZLARS01"

// Everything a workgroup needs to know about its chunk in one 16-byte record: a kernel's first loads then depend on
// one table look-up, not on a chain of three (chunk -> tensor -> offsets), each a cold round trip to memory.
struct ChunkRec {
  int64_t start;  // first element
  int count;      // elements (<= LARS_CH)
  int tensor;
};

struct Layout {
  int64_t T = 0, P = 0, n_chunks = 0;
  size_t off_header = 0, off_offsets = 0, off_chunk_begin = 0, off_flags = 0, off_chunk_tensor = 0, off_chunk_rec = 0;
  size_t off_state = 0;
  size_t static_bytes = 0;  // everything up to here is written by prepare
  size_t off_psum_w = 0, off_psum_g = 0, off_pflag = 0, off_coef = 0, off_tflag = 0;
  size_t off_gsum = 0, off_gflag = 0, off_wsum = 0, total = 0;  // presummed path: gradient sinks, their flags, sum of w^2
};

size_t up256(size_t x) { return (x + 255) & ~size_t(255); }

int make_layout(const jz_param_set* ps, Layout* L) {
  if (!ps) return JZ_ERR_NULL;
  if (ps->num_tensors < 0) return JZ_ERR_SHAPE;
  if (ps->num_tensors > 0 && (!ps->offsets || !ps->flags)) return JZ_ERR_NULL;
  L->T = ps->num_tensors;
  int64_t chunks = 0;
  if (L->T > 0) {
    if (ps->offsets[0] != 0) return JZ_ERR_SHAPE;
    for (int64_t t = 0; t < L->T; ++t) {
      int64_t n = ps->offsets[t + 1] - ps->offsets[t];
      if (n < 0) return JZ_ERR_SHAPE;
      if (n >= (int64_t(1) << 31)) return JZ_ERR_UNSUPPORTED;
      chunks += (n + LARS_CH - 1) / LARS_CH;
    }
    L->P = ps->offsets[L->T];
  }
  if (L->T >= (int64_t(1) << 24) || chunks >= (int64_t(1) << 30)) return JZ_ERR_UNSUPPORTED;
  L->n_chunks = chunks;
  size_t o = 0;
  L->off_header = o;        o = up256(o + 64);
  L->off_offsets = o;       o = up256(o + sizeof(int64_t) * (L->T + 1));
  L->off_chunk_begin = o;   o = up256(o + sizeof(int) * (L->T + 1));
  L->off_flags = o;         o = up256(o + sizeof(int) * (L->T ? L->T : 1));
  L->off_chunk_tensor = o;  o = up256(o + sizeof(int) * (chunks ? chunks : 1));
  L->off_chunk_rec = o;     o = up256(o + sizeof(ChunkRec) * (chunks ? chunks : 1));
  L->off_state = o;         o = up256(o + 64);
  L->static_bytes = o;
  const size_t parts = (size_t)(chunks ? chunks : 1) * LARS_WAVES;
  L->off_psum_w = o;        o = up256(o + sizeof(double) * parts);
  L->off_psum_g = o;        o = up256(o + sizeof(double) * parts);
  L->off_pflag = o;         o = up256(o + sizeof(int) * parts);
  L->off_coef = o;          o = up256(o + sizeof(float) * (L->T ? L->T : 1));
  L->off_tflag = o;         o = up256(o + sizeof(int) * (L->T ? L->T : 1));
  L->off_gsum = o;          o = up256(o + jz::kSumsqSinkBytes * (L->T ? L->T : 1));
  L->off_gflag = o;         o = up256(o + sizeof(int) * (L->T ? L->T : 1));
  L->off_wsum = o;          o = up256(o + sizeof(double) * (L->T ? L->T : 1));
  L->total = o;
  return JZ_OK;
}

uint64_t table_checksum(const jz_param_set* ps) {  // FNV-1a over T, offsets and flags
  uint64_t h = 1469598103934665603ull;
  auto mix = [&](const void* p, size_t n) {
    const unsigned char* b = static_cast<const unsigned char*>(p);
    for (size_t i = 0; i < n; ++i) { h ^= b[i]; h *= 1099511628211ull; }
  };
  int64_t T = ps->num_tensors;
  mix(&T, sizeof T);
  if (T > 0) { mix(ps->offsets, sizeof(int64_t) * (T + 1)); mix(ps->flags, T); }
  return h ? h : 1;
}

// host-side note of which workspace holds which table (the device header is checked as well)
// begun: jz_lars_begin_step has run since the last presummed update (and with which loss-scale state)
struct Prepared { void* ws; uint64_t sum; bool begun; const void* begun_state; };
std::mutex g_mu;
Prepared g_prepared[64];
int g_next = 0;

void remember(void* ws, uint64_t sum) {
  std::lock_guard<std::mutex> lk(g_mu);
  for (auto& e : g_prepared)
    if (e.ws == ws) { e = {ws, sum, false, nullptr}; return; }
  g_prepared[g_next] = {ws, sum, false, nullptr};
  g_next = (g_next + 1) % 64;
}
void set_begun(void* ws, bool begun, const void* state) {
  std::lock_guard<std::mutex> lk(g_mu);
  for (auto& e : g_prepared)
    if (e.ws == ws) { e.begun = begun; e.begun_state = state; }
}
bool has_begun(void* ws, const void* state) {
  std::lock_guard<std::mutex> lk(g_mu);
  for (auto& e : g_prepared)
    if (e.ws == ws) return e.begun && e.begun_state == state;
  return false;
}
bool is_prepared(void* ws, uint64_t sum) {
  std::lock_guard<std::mutex> lk(g_mu);
  for (auto& e : g_prepared)
    if (e.ws == ws) return e.sum == sum;
  return false;
}

struct Tables {
  const uint64_t* header;
  const int64_t* offsets;
  const int* chunk_begin;
  const int* flags;
  const int* chunk_tensor;
  const ChunkRec* chunk_rec;
  int* state;    // [0]: 1 when psum_w holds the sums of squares of the current master weights; [1], [2]: 1/S and S as
                 // float bits when the loss scale lives on the device (written by a launch before the update)
  double* psum_w;  // [n_chunks][LARS_WAVES] partial sums of w^2: one per wavefront, so that no kernel needs a barrier
  double* psum_g;  // same for the (loss-scaled) gradient
  int* pflag;      // same: non-finite gradient seen
  float* coef;  // lr * rho_t
  int* tflag;
  unsigned long long* gsum;  // [T][kSumsqSubs * kSumsqSubStride]: gradient sum-of-squares sinks
  int* gflag;                // [T]: non-finite gradient reported to the sink
  double* wsum;              // [T]: sum of squares of the master weights, written by lars_begin
  int T, n_chunks;
  uint64_t checksum;
};

__device__ __forceinline__ bool table_ok(const Tables& tb) { return tb.header[0] == LARS_MAGIC && tb.header[1] == tb.checksum; }

__device__ __forceinline__ bool half_nonfinite(unsigned short h) { return (h & 0x7c00u) == 0x7c00u; }
__device__ __forceinline__ float half_bits_to_float(unsigned short h) {
  _Float16 x;
  __builtin_memcpy(&x, &h, 2);
  return (float)x;
}
__device__ __forceinline__ unsigned short float_to_half_bits(float f) {
  _Float16 x = (_Float16)f;  // round to nearest even, overflow to Inf, subnormals kept
  unsigned short h;
  __builtin_memcpy(&h, &x, 2);
  return h;
}

// Sum over the workgroup in a fixed order: lanes by shuffle tree, then the four waves left to right.
__device__ __forceinline__ double block_sum(double v, double* lds4) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
  int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) lds4[wv] = v;
  __syncthreads();
  return ((lds4[0] + lds4[1]) + lds4[2]) + lds4[3];
}

// Sum over the 64 lanes of a wavefront by a fixed shuffle tree; the total ends up in lane 0.
__device__ __forceinline__ double wave_sum(double v) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
  return v;
}

__device__ __forceinline__ void chunk_range(const ChunkRec& r, int* t_out, int64_t* start, int64_t* end) {
  *t_out = r.tensor;
  *start = r.start;
  *end = r.start + r.count;
}

constexpr int LARS_IT = LARS_CH / (LARS_THREADS * 8);  // 8-element groups per thread and chunk

// 16-byte accesses of the update pass.  Non-temporal variants (JZ_LARS_NT) were measured slower on MI355X (the
// last-level cache then no longer serves the gradient the reduce pass just read), so plain accesses are the default.
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 load_stream_f4(const float* p) {
#ifndef JZ_LARS_NT
  return *reinterpret_cast<const float4*>(p);
#else
  f32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(p));
  return make_float4(t.x, t.y, t.z, t.w);
#endif
}
__device__ __forceinline__ uint4 load_stream_u4(const unsigned short* p) {
#ifndef JZ_LARS_NT
  return *reinterpret_cast<const uint4*>(p);
#else
  u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(t.x, t.y, t.z, t.w);
#endif
}
__device__ __forceinline__ void store_stream_f4(float* p, float a, float b, float c, float d) {
#ifndef JZ_LARS_NT
  *reinterpret_cast<float4*>(p) = make_float4(a, b, c, d);
#else
  f32x4_t t = {a, b, c, d};
  __builtin_nontemporal_store(t, reinterpret_cast<f32x4_t*>(p));
#endif
}
__device__ __forceinline__ void store_stream_u4(unsigned short* p, unsigned a, unsigned b, unsigned c, unsigned d) {
#ifndef JZ_LARS_NT
  *reinterpret_cast<uint4*>(p) = make_uint4(a, b, c, d);
#else
  u32x4_t t = {a, b, c, d};
  __builtin_nontemporal_store(t, reinterpret_cast<u32x4_t*>(p));
#endif
}

// the 8-aligned body [b0,b1) of a chunk [s,e); the rest is at most 7 head and 7 tail elements
__device__ __forceinline__ void chunk_body(int64_t s, int64_t e, int64_t* b0, int64_t* b1) {
  int64_t a = (s + 7) & ~int64_t(7);
  if (a > e) a = e;
  *b0 = a;
  *b1 = a + ((e - a) & ~int64_t(7));
}

// One thread's share of a chunk's sum of w^2, in the order lars_reduce and lars_update add it (the 8-element groups in
// turn, then at most one head / tail element).
__device__ __forceinline__ double chunk_thread_sumsq_w(const ChunkRec& rec, const float* __restrict__ w) {
  int t;
  int64_t s, e, b0, b1;
  chunk_range(rec, &t, &s, &e);
  chunk_body(s, e, &b0, &b1);
  double sw = 0.0;
#pragma unroll
  for (int k = 0; k < LARS_IT; ++k) {
    int64_t i = b0 + (int64_t)(k * LARS_THREADS + threadIdx.x) * 8;
    if (i < b1) {
      const float4 a = *reinterpret_cast<const float4*>(w + i), b = *reinterpret_cast<const float4*>(w + i + 4);
      const float wv[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
      for (int j = 0; j < 8; ++j) sw = fma((double)wv[j], (double)wv[j], sw);
    }
  }
  int64_t nh = b0 - s, nt = e - b1;
  int64_t k = threadIdx.x;
  if (k < nh + nt) {
    int64_t i = (k < nh) ? s + k : b1 + (k - nh);
    sw = fma((double)w[i], (double)w[i], sw);
  }
  return sw;
}

__global__ __launch_bounds__(LARS_THREADS) void lars_reduce(Tables tb, const float* __restrict__ w,
                                                            const unsigned short* __restrict__ g16) {
  const int c = blockIdx.x;
  const ChunkRec rec = tb.chunk_rec[c];  // requested together with the header: garbage if the header is, but then unused
  const bool have_w = tb.state[0] != 0;  // written by the previous update, i.e. by an earlier launch
  if (!table_ok(tb)) return;
  int t;
  int64_t s, e, b0, b1;
  chunk_range(rec, &t, &s, &e);
  chunk_body(s, e, &b0, &b1);
  double sw = 0.0, sg = 0.0;
  int bad = 0;
  uint4 gq[LARS_IT];
  float4 w0[LARS_IT], w1[LARS_IT];
#pragma unroll
  for (int k = 0; k < LARS_IT; ++k) {
    int64_t i = b0 + (int64_t)(k * LARS_THREADS + threadIdx.x) * 8;
    gq[k] = make_uint4(0, 0, 0, 0);
    w0[k] = w1[k] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i < b1) {
      gq[k] = *reinterpret_cast<const uint4*>(g16 + i);
      if (!have_w) {
        w0[k] = *reinterpret_cast<const float4*>(w + i);
        w1[k] = *reinterpret_cast<const float4*>(w + i + 4);
      }
    }
  }
#pragma unroll
  for (int k = 0; k < LARS_IT; ++k) {  // zeros of the groups beyond b1 add nothing
    float wv[8] = {w0[k].x, w0[k].y, w0[k].z, w0[k].w, w1[k].x, w1[k].y, w1[k].z, w1[k].w};
    unsigned gw[4] = {gq[k].x, gq[k].y, gq[k].z, gq[k].w};
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      unsigned short hb = (unsigned short)(gw[j >> 1] >> ((j & 1) * 16));
      bad |= half_nonfinite(hb);
      double gd = (double)half_bits_to_float(hb);
      sg = fma(gd, gd, sg);
    }
    if (!have_w) {
#pragma unroll
      for (int j = 0; j < 8; ++j) sw = fma((double)wv[j], (double)wv[j], sw);
    }
  }
  {  // head and tail, at most 7 elements each
    int64_t nh = b0 - s, nt = e - b1;
    int64_t k = threadIdx.x;
    if (k < nh + nt) {
      int64_t i = (k < nh) ? s + k : b1 + (k - nh);
      unsigned short hb = g16[i];
      bad |= half_nonfinite(hb);
      double wd = have_w ? 0.0 : (double)w[i], gd = (double)half_bits_to_float(hb);
      sw = fma(wd, wd, sw);
      sg = fma(gd, gd, sg);
    }
  }
  sw = wave_sum(sw);
  sg = wave_sum(sg);
  bad = __any(bad);
  if ((threadIdx.x & 63) == 0) {
    const int slot = c * LARS_WAVES + (threadIdx.x >> 6);
    if (!have_w) tb.psum_w[slot] = sw;
    tb.psum_g[slot] = sg;
    tb.pflag[slot] = bad ? 1 : 0;
  }
}

// scale_dev != nullptr: the loss scale lives on the device (dynamic loss scaling) and replaces the argument
__global__ __launch_bounds__(LARS_THREADS) void lars_finalize(Tables tb, float lr, float eta, float loss_scale,
                                                              const float* __restrict__ scale_dev) {
  __shared__ double red[4];
  if (scale_dev) loss_scale = *scale_dev;
  if (!table_ok(tb)) return;
  const int t = blockIdx.x;
  // the update kernel adjusts the device-resident scale itself, so its workgroups take 1/S from here instead
  if (scale_dev && t == 0 && threadIdx.x == 0) tb.state[1] = __float_as_int(1.0f / loss_scale);
  const int c0 = tb.chunk_begin[t] * LARS_WAVES, c1 = tb.chunk_begin[t + 1] * LARS_WAVES;
  double sw = 0.0, sg = 0.0;
  int bad = 0;
  // a thread's first FIN_PRE partials are requested together (the largest ResNet-50 tensor has 9 per thread): one
  // memory round trip instead of one per partial; the additions keep their order
  constexpr int FIN_PRE = 10;
  double pw[FIN_PRE], pg[FIN_PRE];
  int pf[FIN_PRE];
#pragma unroll
  for (int j = 0; j < FIN_PRE; ++j) {
    const int c = c0 + (int)threadIdx.x + j * LARS_THREADS;
    pw[j] = 0.0; pg[j] = 0.0; pf[j] = 0;
    if (c < c1) { pw[j] = tb.psum_w[c]; pg[j] = tb.psum_g[c]; pf[j] = tb.pflag[c]; }
  }
#pragma unroll
  for (int j = 0; j < FIN_PRE; ++j) { sw += pw[j]; sg += pg[j]; bad |= pf[j]; }
  for (int c = c0 + (int)threadIdx.x + FIN_PRE * LARS_THREADS; c < c1; c += LARS_THREADS) {
    sw += tb.psum_w[c];
    sg += tb.psum_g[c];
    bad |= tb.pflag[c];
  }
  sw = block_sum(sw, red);
  sg = block_sum(sg, red);
  bad = __syncthreads_or(bad);
  if (threadIdx.x == 0) {
    double rho = 1.0;
    if ((tb.flags[t] & JZ_PARAM_LARS) && sw > 0.0 && sg > 0.0)
      rho = (double)eta * sqrt(sw) / (sqrt(sg) / (double)loss_scale);  // Eq. 1 on the un-scaled gradient
    tb.coef[t] = (float)((double)lr * rho);
    tb.tflag[t] = bad ? 1 : 0;
  }
}

// Start of a step on the presummed path, one workgroup per tensor (see the top of the file).
__global__ __launch_bounds__(LARS_THREADS) void lars_begin(Tables tb, const float* __restrict__ w,
                                                           const float* __restrict__ scale_dev) {
  __shared__ double red[4];
  if (!table_ok(tb)) return;
  const int t = blockIdx.x;
  const bool have_w = tb.state[0] != 0;  // written by an earlier launch
  constexpr int SINK_WORDS = jz::kSumsqSubs * jz::kSumsqSubStride;
  for (int i = threadIdx.x; i < SINK_WORDS; i += LARS_THREADS) tb.gsum[(size_t)t * SINK_WORDS + i] = 0ull;
  if (threadIdx.x == 0) tb.gflag[t] = 0;
  if (scale_dev && t == 0 && threadIdx.x == 0) {  // the update adjusts the device-resident scale itself: it reads S from here
    const float S = *scale_dev;
    tb.state[1] = __float_as_int(1.0f / S);
    tb.state[2] = __float_as_int(S);
  }
  const int c0 = tb.chunk_begin[t] * LARS_WAVES, c1 = tb.chunk_begin[t + 1] * LARS_WAVES;
  if (!have_w) {
    // Fresh workspace: leave in psum_w what lars_reduce would (same elements per thread, same order), chunk by chunk, so
    // that the sum below is the same bits whether the partial sums were carried or are recomputed here.  One workgroup
    // per tensor makes this slow for large tensors; it runs once per jz_lars_prepare.
    for (int c = tb.chunk_begin[t]; c < tb.chunk_begin[t + 1]; ++c) {
      const double p = wave_sum(chunk_thread_sumsq_w(tb.chunk_rec[c], w));
      if ((threadIdx.x & 63) == 0) tb.psum_w[c * LARS_WAVES + (threadIdx.x >> 6)] = p;
    }
    __threadfence_block();
    __syncthreads();
  }
  // Loads that go past the compute unit's own cache: in the fresh case a partial sum written above may share a cache
  // line with a neighbouring tensor's, which another workgroup on this compute unit may have pulled in before the write.
  double sw = 0.0;
  if (have_w) {
    // carried sums, written by an earlier launch: plain loads, eight requested together, added in the same order as below
    for (int c = c0 + (int)threadIdx.x; c < c1; c += 8 * LARS_THREADS) {
      double v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int cu = c + u * LARS_THREADS;
        v[u] = tb.psum_w[cu < c1 ? cu : c];
      }
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (c + u * LARS_THREADS < c1) sw += v[u];
    }
  } else {
    for (int c = c0 + (int)threadIdx.x; c < c1; c += LARS_THREADS)
      sw += __longlong_as_double((long long)__hip_atomic_load(reinterpret_cast<const unsigned long long*>(tb.psum_w + c),
                                                              __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
  }
  sw = block_sum(sw, red);
  if (threadIdx.x == 0) tb.wsum[t] = sw;
}

// The gradient reduce pass into the sinks, one workgroup per chunk, for chunks chunk0 .. chunk0 + gridDim.x - 1.
__global__ __launch_bounds__(LARS_THREADS) void lars_grad_sumsq(Tables tb, const unsigned short* __restrict__ g16, int chunk0) {
  __shared__ unsigned long long red[5];
  const int c = chunk0 + (int)blockIdx.x;
  const ChunkRec rec = tb.chunk_rec[c];
  if (!table_ok(tb)) return;
  if (threadIdx.x < 5) red[threadIdx.x] = 0ull;
  __syncthreads();
  int t;
  int64_t s, e, b0, b1;
  chunk_range(rec, &t, &s, &e);
  if (tb.flags[t] & JZ_PARAM_GRAD_PRESUMMED) return;  // its producer fills the sink
  chunk_body(s, e, &b0, &b1);
  jz::SumsqAcc sg;
  int bad = 0;
#pragma unroll
  for (int k = 0; k < LARS_IT; ++k) {
    int64_t i = b0 + (int64_t)(k * LARS_THREADS + threadIdx.x) * 8;
    if (i < b1) {
      const uint4 gq = *reinterpret_cast<const uint4*>(g16 + i);
      const unsigned gw[4] = {gq.x, gq.y, gq.z, gq.w};
#pragma unroll
      for (int j = 0; j < 8; ++j) bad |= jz::sumsq_acc_add(sg, (unsigned short)(gw[j >> 1] >> ((j & 1) * 16)));
    }
  }
  {
    int64_t nh = b0 - s, nt = e - b1;
    int64_t k = threadIdx.x;
    if (k < nh + nt) bad |= jz::sumsq_acc_add(sg, g16[(k < nh) ? s + k : b1 + (k - nh)]);
  }
  jz::SumsqSink sink{tb.gsum + (size_t)t * (jz::kSumsqSubs * jz::kSumsqSubStride), tb.gflag + t};
  jz::sumsq_block_flush(sg, bad, sink, (unsigned)(c - tb.chunk_begin[t]), red);
}

// Dynamic loss scaling (Sections 4.1 and 5.3 name the loss scale; the policy is the usual skip / shrink / grow one).
struct DynScale {
  jz_loss_scale_state* st;  // nullptr: fixed loss scale
  float growth, backoff;
  int interval;
  float lo, hi;
};
__device__ __forceinline__ void loss_scale_step(const DynScale& d, int overflow) {
  float sc = d.st->scale;
  int good = d.st->good_steps;
  if (overflow) {
    sc = fmaxf(sc * d.backoff, d.lo);
    good = 0;
  } else if (++good >= d.interval) {
    sc = fminf(sc * d.growth, d.hi);
    good = 0;
  }
  d.st->scale = sc;
  d.st->good_steps = good;
}

__device__ __forceinline__ void lars_step(float& w, float& v, unsigned short gbits, float coef, float lam, float m,
                                          float inv_s, unsigned short& w16) {
  float g = half_bits_to_float(gbits) * inv_s;  // un-scale
  float u = fmaf(lam, w, g);                    // Eq. 2 differentiated: g + lambda*w
  float vn = fmaf(m, v, coef * u);              // momentum step with the local rate lr*rho
  float wn = w - vn;
  v = vn;
  w = wn;
  w16 = float_to_half_bits(wn);                 // cast back for the next forward pass
}

// PRE: the presummed path -- no lars_finalize ran; every wavefront forms its tensor's lr*rho_t itself (lr, eta and, for a
// fixed loss scale, S come as arguments) and the overflow flags are those of the sinks.
template <bool PRE>
__global__ __launch_bounds__(LARS_THREADS) void lars_update(Tables tb, float* __restrict__ w, float* __restrict__ v,
                                                            const unsigned short* __restrict__ g16,
                                                            unsigned short* __restrict__ w16, float m, float wd,
                                                            float inv_s, int* __restrict__ found_inf, DynScale dyn,
                                                            float lr, float eta, float loss_scale) {
  if (dyn.st) {  // written by lars_finalize / lars_begin (not used when there is no tensor)
    inv_s = __int_as_float(tb.state[1]);
    if (PRE) loss_scale = __int_as_float(tb.state[2]);
  }
  // the header, this workgroup's chunk record and the tensor flags are requested together; nothing read through the
  // tables is used before the header has been checked
  const int cidx = (int)blockIdx.x < tb.n_chunks ? tb.n_chunks - 1 - (int)blockIdx.x : 0;
  const ChunkRec rec = tb.n_chunks > 0 ? tb.chunk_rec[cidx] : ChunkRec{0, 0, 0};
  int f = 0;  // every wavefront looks at all tensor flags itself: no barrier anywhere in this kernel
  for (int t = threadIdx.x & 63; t < tb.T; t += 64) f |= PRE ? tb.gflag[t] : tb.tflag[t];
  // PRE: this lane's share of the tensor's gradient sink (the tensor index is garbage if the header is: clamp it)
  // the first wavefront reads the sink (one quadruple per lane) and hands the total to the others through LDS
  __shared__ double sg_shared;
  unsigned long long d0 = 0, d1 = 0, d2 = 0, d3 = 0;
  double sw_t = 0.0;
  if (PRE && tb.n_chunks > 0) {
    const int ts = rec.tensor >= 0 && rec.tensor < tb.T ? rec.tensor : 0;
    static_assert(jz::kSumsqSubs == 64, "one counter quadruple per lane");
    if (threadIdx.x < 64) {
      const ulonglong2* a = reinterpret_cast<const ulonglong2*>(tb.gsum + ((size_t)ts * jz::kSumsqSubs + threadIdx.x) * jz::kSumsqSubStride);
      const ulonglong2 lo = a[0], hi = a[1];
      d0 = lo.x; d1 = lo.y; d2 = hi.x; d3 = hi.y;
    }
    sw_t = tb.wsum[ts];
  }
  if (!table_ok(tb)) {
    if (blockIdx.x == 0 && threadIdx.x == 0) *found_inf = -1;
    return;
  }
  f = __any(f);
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    *found_inf = f ? 1 : 0;
    // skipped or not, psum_w describes the master weights as this launch leaves them: lars_reduce / lars_begin filled it in
    // for the weights as they were, and an update that goes through rewrites every chunk's sums
    tb.state[0] = 1;
    if (dyn.st) loss_scale_step(dyn, f);  // no workgroup of this launch reads dyn.st->scale
  }
  if (f) return;  // overflow under loss scaling: the step is skipped as a whole
  if ((int)blockIdx.x >= tb.n_chunks) return;
  const int c = cidx;
  int t;
  int64_t s, e, b0, b1;
  chunk_range(rec, &t, &s, &e);
  chunk_body(s, e, &b0, &b1);
  float coef;
  if (PRE) {
    if (threadIdx.x < 64) {  // integer sums: the order does not matter
      d0 = jz::wave_total_u64(d0);
      d1 = jz::wave_total_u64(d1);
      d2 = jz::wave_total_u64(d2);
      d3 = jz::wave_total_u64(d3);
      if (threadIdx.x == 63) sg_shared = jz::sumsq_value(d0, d1, d2, d3);
    }
    __syncthreads();  // every wavefront of the workgroup is here: the returns above depend on nothing wave-specific
    const double sg = sg_shared;
    double rho = 1.0;
    if ((tb.flags[t] & JZ_PARAM_LARS) && sw_t > 0.0 && sg > 0.0)
      rho = (double)eta * sqrt(sw_t) / (sqrt(sg) / (double)loss_scale);  // Eq. 1 on the un-scaled gradient
    coef = (float)((double)lr * rho);
  } else {
    coef = tb.coef[t];
  }
  const float lam = (tb.flags[t] & JZ_PARAM_WEIGHT_DECAY) ? wd : 0.0f;
  float4 w0[LARS_IT], w1[LARS_IT], v0[LARS_IT], v1[LARS_IT];
  uint4 gq[LARS_IT];
#pragma unroll
  for (int k = 0; k < LARS_IT; ++k) {  // every load of the chunk is in flight before the first use
    int64_t i = b0 + (int64_t)(k * LARS_THREADS + threadIdx.x) * 8;
    if (i < b1) {
      gq[k] = load_stream_u4(g16 + i);
      w0[k] = load_stream_f4(w + i);
      w1[k] = load_stream_f4(w + i + 4);
      v0[k] = load_stream_f4(v + i);
      v1[k] = load_stream_f4(v + i + 4);
    }
  }
  double sw = 0.0;  // sum of squares of the new weights, in the order lars_reduce would add them
#pragma unroll
  for (int k = 0; k < LARS_IT; ++k) {
    int64_t i = b0 + (int64_t)(k * LARS_THREADS + threadIdx.x) * 8;
    if (i < b1) {
      float wv[8] = {w0[k].x, w0[k].y, w0[k].z, w0[k].w, w1[k].x, w1[k].y, w1[k].z, w1[k].w};
      float vv[8] = {v0[k].x, v0[k].y, v0[k].z, v0[k].w, v1[k].x, v1[k].y, v1[k].z, v1[k].w};
      unsigned gw[4] = {gq[k].x, gq[k].y, gq[k].z, gq[k].w};
      unsigned ow[4];
#pragma unroll
      for (int j = 0; j < 8; j += 2) {
        unsigned short h0, h1;
        lars_step(wv[j], vv[j], (unsigned short)(gw[j >> 1] & 0xffffu), coef, lam, m, inv_s, h0);
        lars_step(wv[j + 1], vv[j + 1], (unsigned short)(gw[j >> 1] >> 16), coef, lam, m, inv_s, h1);
        ow[j >> 1] = (unsigned)h0 | ((unsigned)h1 << 16);
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) sw = fma((double)wv[j], (double)wv[j], sw);
      store_stream_f4(w + i, wv[0], wv[1], wv[2], wv[3]);
      store_stream_f4(w + i + 4, wv[4], wv[5], wv[6], wv[7]);
      store_stream_f4(v + i, vv[0], vv[1], vv[2], vv[3]);
      store_stream_f4(v + i + 4, vv[4], vv[5], vv[6], vv[7]);
      store_stream_u4(w16 + i, ow[0], ow[1], ow[2], ow[3]);
    }
  }
  {
    int64_t nh = b0 - s, nt = e - b1;
    int64_t k = threadIdx.x;
    if (k < nh + nt) {
      int64_t i = (k < nh) ? s + k : b1 + (k - nh);
      float wi = w[i], vi = v[i];
      unsigned short h;
      lars_step(wi, vi, g16[i], coef, lam, m, inv_s, h);
      w[i] = wi;
      v[i] = vi;
      w16[i] = h;
      sw = fma((double)wi, (double)wi, sw);
    }
  }
  sw = wave_sum(sw);
  if ((threadIdx.x & 63) == 0) tb.psum_w[c * LARS_WAVES + (threadIdx.x >> 6)] = sw;
}

__global__ void loss_scale_init(jz_loss_scale_state* __restrict__ st, float scale) {
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    st->scale = scale;
    st->good_steps = 0;
  }
}

Tables make_tables(const Layout& L, void* ws, uint64_t sum) {
  char* b = static_cast<char*>(ws);
  Tables tb;
  tb.header = reinterpret_cast<const uint64_t*>(b + L.off_header);
  tb.offsets = reinterpret_cast<const int64_t*>(b + L.off_offsets);
  tb.chunk_begin = reinterpret_cast<const int*>(b + L.off_chunk_begin);
  tb.flags = reinterpret_cast<const int*>(b + L.off_flags);
  tb.chunk_tensor = reinterpret_cast<const int*>(b + L.off_chunk_tensor);
  tb.chunk_rec = reinterpret_cast<const ChunkRec*>(b + L.off_chunk_rec);
  tb.state = reinterpret_cast<int*>(b + L.off_state);
  tb.psum_w = reinterpret_cast<double*>(b + L.off_psum_w);
  tb.psum_g = reinterpret_cast<double*>(b + L.off_psum_g);
  tb.pflag = reinterpret_cast<int*>(b + L.off_pflag);
  tb.coef = reinterpret_cast<float*>(b + L.off_coef);
  tb.tflag = reinterpret_cast<int*>(b + L.off_tflag);
  tb.gsum = reinterpret_cast<unsigned long long*>(b + L.off_gsum);
  tb.gflag = reinterpret_cast<int*>(b + L.off_gflag);
  tb.wsum = reinterpret_cast<double*>(b + L.off_wsum);
  tb.T = (int)L.T;
  tb.n_chunks = (int)L.n_chunks;
  tb.checksum = sum;
  return tb;
}

}  // namespace

extern "C" int jz_lars_workspace_bytes(const jz_param_set* ps, size_t* bytes) {
  if (!bytes) return JZ_ERR_NULL;
  Layout L;
  int rc = make_layout(ps, &L);
  if (rc != JZ_OK) return rc;
  *bytes = L.total;
  return JZ_OK;
}

extern "C" int jz_lars_prepare(const jz_param_set* ps, void* ws, size_t ws_bytes, void* hip_stream) {
  Layout L;
  int rc = make_layout(ps, &L);
  if (rc != JZ_OK) return rc;
  if (!ws || ws_bytes < L.total) return JZ_ERR_WORKSPACE;
  if (!jz::aligned16(ws)) return JZ_ERR_ALIGN;
  std::vector<char> host(L.static_bytes, 0);
  uint64_t sum = table_checksum(ps);
  uint64_t* hdr = reinterpret_cast<uint64_t*>(host.data() + L.off_header);
  hdr[0] = LARS_MAGIC;
  hdr[1] = sum;
  hdr[2] = (uint64_t)L.T;
  hdr[3] = (uint64_t)L.n_chunks;
  hdr[4] = (uint64_t)L.P;
  int64_t* off = reinterpret_cast<int64_t*>(host.data() + L.off_offsets);
  int* cb = reinterpret_cast<int*>(host.data() + L.off_chunk_begin);
  int* fl = reinterpret_cast<int*>(host.data() + L.off_flags);
  int* ct = reinterpret_cast<int*>(host.data() + L.off_chunk_tensor);
  ChunkRec* cr = reinterpret_cast<ChunkRec*>(host.data() + L.off_chunk_rec);
  int c = 0;
  off[0] = 0;
  cb[0] = 0;
  for (int64_t t = 0; t < L.T; ++t) {
    off[t] = ps->offsets[t];
    off[t + 1] = ps->offsets[t + 1];
    fl[t] = ps->flags[t];
    int64_t n = ps->offsets[t + 1] - ps->offsets[t];
    int nc = (int)((n + LARS_CH - 1) / LARS_CH);
    for (int k = 0; k < nc; ++k) {
      ct[c + k] = (int)t;
      const int64_t st0 = ps->offsets[t] + (int64_t)k * LARS_CH;
      const int64_t en = st0 + LARS_CH < ps->offsets[t + 1] ? st0 + LARS_CH : ps->offsets[t + 1];
      cr[c + k] = ChunkRec{st0, (int)(en - st0), (int)t};
    }
    c += nc;
    cb[t + 1] = c;
  }
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (hipMemcpyAsync(ws, host.data(), L.static_bytes, hipMemcpyHostToDevice, st) != hipSuccess) return JZ_ERR_LAUNCH;
  if (hipStreamSynchronize(st) != hipSuccess) return JZ_ERR_LAUNCH;
  remember(ws, sum);
  return JZ_OK;
}

namespace {

// the update with a fixed loss scale (state == nullptr: hp->loss_scale) or with a device-resident one that the
// controller adjusts afterwards
int lars_run(const jz_param_set* ps, const jz_lars_hparams* hp, const jz_loss_scale_policy* pol, jz_loss_scale_state* state,
             int* found_inf_dev, void* ws, size_t ws_bytes, void* hip_stream, bool presummed = false) {
  if (!hp || !found_inf_dev) return JZ_ERR_NULL;
  Layout L;
  int rc = make_layout(ps, &L);
  if (rc != JZ_OK) return rc;
  if (!state && (!(hp->loss_scale > 0.0f) || !(hp->loss_scale < 3.0e38f))) return JZ_ERR_SHAPE;
  if (state) {
    if (!pol) return JZ_ERR_NULL;
    if (!(pol->growth_factor >= 1.0f) || !(pol->backoff_factor > 0.0f) || !(pol->backoff_factor <= 1.0f) ||
        pol->growth_interval < 1 || !(pol->min_scale > 0.0f) || !(pol->max_scale >= pol->min_scale) || !(pol->max_scale < 3.0e38f))
      return JZ_ERR_SHAPE;
    if (reinterpret_cast<uintptr_t>(state) & 7u) return JZ_ERR_ALIGN;
  }
  if (L.P > 0 && (!ps->master_w || !ps->momentum || !ps->grad16 || !ps->weight16)) return JZ_ERR_NULL;
  if (!ws || ws_bytes < L.total) return JZ_ERR_WORKSPACE;
  if (!jz::aligned16(ws) || !jz::aligned16(ps->master_w) || !jz::aligned16(ps->momentum) ||
      !jz::aligned16(ps->grad16) || !jz::aligned16(ps->weight16) || (reinterpret_cast<uintptr_t>(found_inf_dev) & 3u))
    return JZ_ERR_ALIGN;
  const size_t P = (size_t)L.P;
  const void* bufs[4] = {ps->master_w, ps->momentum, ps->grad16, ps->weight16};
  const size_t lens[4] = {4 * P, 4 * P, 2 * P, 2 * P};
  for (int i = 0; i < 4; ++i) {
    if (jz::overlaps(bufs[i], lens[i], ws, L.total) || jz::overlaps(bufs[i], lens[i], found_inf_dev, sizeof(int)))
      return JZ_ERR_ALIAS;
    for (int j = i + 1; j < 4; ++j)
      if (jz::overlaps(bufs[i], lens[i], bufs[j], lens[j])) return JZ_ERR_ALIAS;
  }
  if (jz::overlaps(found_inf_dev, sizeof(int), ws, L.total)) return JZ_ERR_ALIAS;
  if (state) {
    if (jz::overlaps(state, sizeof(*state), ws, L.total) || jz::overlaps(state, sizeof(*state), found_inf_dev, sizeof(int)))
      return JZ_ERR_ALIAS;
    for (int i = 0; i < 4; ++i)
      if (jz::overlaps(bufs[i], lens[i], state, sizeof(*state))) return JZ_ERR_ALIAS;
  }
  uint64_t sum = table_checksum(ps);
  if (!is_prepared(ws, sum)) return JZ_ERR_NOT_PREPARED;
  // the presummed update consumes what jz_lars_begin_step set up (with the same loss-scale state) and the sinks filled since
  if (presummed && !has_begun(ws, state)) return JZ_ERR_NOT_PREPARED;

  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  Tables tb = make_tables(L, ws, sum);
  const unsigned short* g16 = static_cast<const unsigned short*>(ps->grad16);
  const float* scale_dev = state ? &state->scale : nullptr;
  DynScale dyn{state, 1.0f, 1.0f, 1, 1.0f, 1.0f};
  if (state) dyn = DynScale{state, pol->growth_factor, pol->backoff_factor, pol->growth_interval, pol->min_scale, pol->max_scale};
  if (presummed) {
    set_begun(ws, false, nullptr);
    hipLaunchKernelGGL(lars_update<true>, dim3((unsigned)(L.n_chunks > 0 ? L.n_chunks : 1)), dim3(LARS_THREADS), 0, st, tb,
                       ps->master_w, ps->momentum, g16, static_cast<unsigned short*>(ps->weight16), hp->momentum,
                       hp->weight_decay, state ? 1.0f : 1.0f / hp->loss_scale, found_inf_dev, dyn, hp->lr, hp->trust_coef,
                       state ? 1.0f : hp->loss_scale);
    return jz::launch_status();
  }
  if (L.n_chunks > 0)
    hipLaunchKernelGGL(lars_reduce, dim3((unsigned)L.n_chunks), dim3(LARS_THREADS), 0, st, tb, ps->master_w, g16);
  if (L.T > 0)
    hipLaunchKernelGGL(lars_finalize, dim3((unsigned)L.T), dim3(LARS_THREADS), 0, st, tb, hp->lr, hp->trust_coef,
                       state ? 1.0f : hp->loss_scale, scale_dev);
  // at least one workgroup so that the flag is always written
  hipLaunchKernelGGL(lars_update<false>, dim3((unsigned)(L.n_chunks > 0 ? L.n_chunks : 1)), dim3(LARS_THREADS), 0, st, tb,
                     ps->master_w, ps->momentum, g16, static_cast<unsigned short*>(ps->weight16), hp->momentum,
                     hp->weight_decay, state ? 1.0f : 1.0f / hp->loss_scale, found_inf_dev, dyn, 0.0f, 0.0f, 1.0f);
  return jz::launch_status();
}

// what the entry points of the presummed path have in common: the table, the workspace and that it was prepared
int presummed_common(const jz_param_set* ps, void* ws, size_t ws_bytes, Layout* L, uint64_t* sum) {
  int rc = make_layout(ps, L);
  if (rc != JZ_OK) return rc;
  if (!ws || ws_bytes < L->total) return JZ_ERR_WORKSPACE;
  if (!jz::aligned16(ws)) return JZ_ERR_ALIGN;
  *sum = table_checksum(ps);
  if (!is_prepared(ws, *sum)) return JZ_ERR_NOT_PREPARED;
  return JZ_OK;
}

}  // namespace

extern "C" int jz_lars_mp_update(const jz_param_set* ps, const jz_lars_hparams* hp, int* found_inf_dev, void* ws,
                                 size_t ws_bytes, void* hip_stream) {
  return lars_run(ps, hp, nullptr, nullptr, found_inf_dev, ws, ws_bytes, hip_stream);
}

extern "C" int jz_lars_mp_update_dyn(const jz_param_set* ps, const jz_lars_hparams* hp, const jz_loss_scale_policy* policy,
                                     jz_loss_scale_state* state_dev, int* found_inf_dev, void* ws, size_t ws_bytes,
                                     void* hip_stream) {
  if (!state_dev) return JZ_ERR_NULL;
  return lars_run(ps, hp, policy, state_dev, found_inf_dev, ws, ws_bytes, hip_stream);
}

extern "C" int jz_lars_sumsq_sink(const jz_param_set* ps, void* ws, size_t ws_bytes, int64_t tensor, jz_sumsq_sink* sink) {
  if (!sink) return JZ_ERR_NULL;
  Layout L;
  uint64_t sum;
  int rc = presummed_common(ps, ws, ws_bytes, &L, &sum);
  if (rc != JZ_OK) return rc;
  if (tensor < 0 || tensor >= L.T) return JZ_ERR_SHAPE;
  static_assert(JZ_SUMSQ_SINK_BYTES == jz::kSumsqSinkBytes, "public and internal sink size");
  char* b = static_cast<char*>(ws);
  sink->sums = b + L.off_gsum + (size_t)tensor * jz::kSumsqSinkBytes;
  sink->nonfinite = reinterpret_cast<int*>(b + L.off_gflag) + tensor;
  return JZ_OK;
}

extern "C" int jz_lars_begin_step(const jz_param_set* ps, const jz_loss_scale_state* state_dev, void* ws, size_t ws_bytes,
                                  void* hip_stream) {
  Layout L;
  uint64_t sum;
  int rc = presummed_common(ps, ws, ws_bytes, &L, &sum);
  if (rc != JZ_OK) return rc;
  if (L.P > 0 && !ps->master_w) return JZ_ERR_NULL;
  if (!jz::aligned16(ps->master_w) || (reinterpret_cast<uintptr_t>(state_dev) & 7u)) return JZ_ERR_ALIGN;
  if (jz::overlaps(ps->master_w, 4 * (size_t)L.P, ws, L.total) || jz::overlaps(state_dev, sizeof(*state_dev), ws, L.total))
    return JZ_ERR_ALIAS;
  if (L.T > 0) {
    hipLaunchKernelGGL(lars_begin, dim3((unsigned)L.T), dim3(LARS_THREADS), 0, static_cast<hipStream_t>(hip_stream),
                       make_tables(L, ws, sum), ps->master_w, state_dev ? &state_dev->scale : nullptr);
    if ((rc = jz::launch_status()) != JZ_OK) return rc;
  }
  set_begun(ws, true, state_dev);
  return JZ_OK;
}

extern "C" int jz_lars_grad_sumsq(const jz_param_set* ps, int64_t first_tensor, int64_t num_tensors, void* ws, size_t ws_bytes,
                                  void* hip_stream) {
  Layout L;
  uint64_t sum;
  int rc = presummed_common(ps, ws, ws_bytes, &L, &sum);
  if (rc != JZ_OK) return rc;
  if (first_tensor < 0 || num_tensors < 0 || first_tensor + num_tensors > L.T) return JZ_ERR_SHAPE;
  if (L.P > 0 && !ps->grad16) return JZ_ERR_NULL;
  if (!jz::aligned16(ps->grad16)) return JZ_ERR_ALIGN;
  if (jz::overlaps(ps->grad16, 2 * (size_t)L.P, ws, L.total)) return JZ_ERR_ALIAS;
  int64_t c0 = 0, c1 = 0;  // chunks of tensors [first, first + num)
  for (int64_t t = 0; t < first_tensor + num_tensors; ++t) {
    const int64_t nc = (ps->offsets[t + 1] - ps->offsets[t] + LARS_CH - 1) / LARS_CH;
    if (t < first_tensor) c0 += nc;
    c1 += nc;
  }
  if (c1 > c0)
    hipLaunchKernelGGL(lars_grad_sumsq, dim3((unsigned)(c1 - c0)), dim3(LARS_THREADS), 0, static_cast<hipStream_t>(hip_stream),
                       make_tables(L, ws, sum), static_cast<const unsigned short*>(ps->grad16), (int)c0);
  return jz::launch_status();
}

extern "C" int jz_lars_mp_update_presummed(const jz_param_set* ps, const jz_lars_hparams* hp, int* found_inf_dev, void* ws,
                                           size_t ws_bytes, void* hip_stream) {
  return lars_run(ps, hp, nullptr, nullptr, found_inf_dev, ws, ws_bytes, hip_stream, true);
}

extern "C" int jz_lars_mp_update_presummed_dyn(const jz_param_set* ps, const jz_lars_hparams* hp,
                                               const jz_loss_scale_policy* policy, jz_loss_scale_state* state_dev,
                                               int* found_inf_dev, void* ws, size_t ws_bytes, void* hip_stream) {
  if (!state_dev) return JZ_ERR_NULL;
  return lars_run(ps, hp, policy, state_dev, found_inf_dev, ws, ws_bytes, hip_stream, true);
}

extern "C" int jz_loss_scale_init(jz_loss_scale_state* state_dev, float initial_scale, void* hip_stream) {
  if (!state_dev) return JZ_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(state_dev) & 7u) return JZ_ERR_ALIGN;
  if (!(initial_scale > 0.0f) || !(initial_scale < 3.0e38f)) return JZ_ERR_SHAPE;
  hipLaunchKernelGGL(loss_scale_init, dim3(1), dim3(64), 0, static_cast<hipStream_t>(hip_stream), state_dev, initial_scale);
  return jz::launch_status();
}
