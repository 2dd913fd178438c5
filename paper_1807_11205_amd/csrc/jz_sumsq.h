// Sum of squares of a tensor's FP16 gradient, accumulated where the gradient is produced (the ||g_t|| of Eq. 1,
// Section 4.1) so that the optimiser does not have to read the gradient a second time.
//
// Many workgroups of several launches contribute to one tensor's sum, in no fixed order, and the result has to be the
// same bits on every run.  Floating-point addition is not associative, integer addition is, and the squares of FP16
// values are integers in disguise: a finite FP16 value is k * 2^-24 with an integer |k| < 2^40, so its square is
// k^2 units of 2^-48.  With |k| = a 2^20 + b (a, b < 2^20),  k^2 = a^2 2^40 + 2ab 2^20 + b^2: a thread keeps the three
// sums (a^2, 2ab, b^2) in 64-bit integers, a workgroup adds its threads' sums, carries them into four base-2^20 digits
// and adds each digit to a 64-bit counter with an atomic integer add.  The counters therefore hold the EXACT sum of
// squares, whatever the order and the partition of the work were: the same bits from run to run and for every kernel
// plan.  The three low counters take 2^44 contributions before they could overflow, the top one holds up to 2^76 units
// (more than 2^31 elements of the largest FP16 value).
//
// Atomics on one address queue behind each other (about 12 ns each on MI355X), so a tensor has kSumsqSubs such
// counter quadruples, 128 bytes apart; a contributor picks one by its workgroup index and the reader adds them.
#pragma once
#include <hip/hip_runtime.h>

namespace jz {

constexpr int kSumsqSubs = 16;       // counter quadruples per tensor
constexpr int kSumsqSubStride = 16;  // 64-bit words between quadruples (128 bytes: one cache line each)
constexpr size_t kSumsqSinkBytes = (size_t)kSumsqSubs * kSumsqSubStride * 8;

struct SumsqSink {
  unsigned long long* sums;  // kSumsqSinkBytes; nullptr: no sink
  int* nonfinite;            // set to 1 when a gradient element is Inf or NaN (never cleared here)
};

// a thread's running sums; at most 2^22 elements per thread
struct SumsqAcc {
  unsigned long long aa = 0, ab2 = 0, bb = 0;
};

// adds the square of one FP16 value given by its bit pattern; returns 1 for Inf / NaN (which adds nothing)
__device__ __forceinline__ int sumsq_acc_add(SumsqAcc& s, unsigned short h) {
  const unsigned e = (h >> 10) & 31u, m = h & 1023u;
  if (e == 31u) return 1;
  // |value| = k 2^-24:  subnormal k = m;  normal k = (1024 + m) 2^(e - 1)
  const unsigned long long k = e == 0 ? (unsigned long long)m : (unsigned long long)(1024u + m) << (e - 1);
  const unsigned a = (unsigned)(k >> 20), b = (unsigned)k & 0xfffffu;
  s.aa += (unsigned long long)a * a;
  s.ab2 += 2ull * a * b;
  s.bb += (unsigned long long)b * b;
  return 0;
}

// Workgroup-wide: adds every thread's sums and contributes them to the sink (or raises its flag when any thread saw a
// non-finite value: the update is then skipped as a whole and the counters are not touched).  Every thread of the
// workgroup must call it; `lds` is scratch for 3 * (threads / 64) 64-bit words; at most 2^23 elements per workgroup.
__device__ __forceinline__ void sumsq_block_flush(SumsqAcc s, int bad, const SumsqSink& sink, unsigned which,
                                                  unsigned long long* lds) {
  for (int o = 32; o > 0; o >>= 1) {
    s.aa += __shfl_down(s.aa, o, 64);
    s.ab2 += __shfl_down(s.ab2, o, 64);
    s.bb += __shfl_down(s.bb, o, 64);
  }
  bad = __syncthreads_or(bad);
  const int nw = (int)(blockDim.x >> 6), wv = (int)(threadIdx.x >> 6);
  if ((threadIdx.x & 63) == 0) {
    lds[3 * wv + 0] = s.aa;
    lds[3 * wv + 1] = s.ab2;
    lds[3 * wv + 2] = s.bb;
  }
  __syncthreads();
  if (threadIdx.x != 0) return;
  if (bad) {
    *sink.nonfinite = 1;
    return;
  }
  unsigned long long aa = 0, ab2 = 0, bb = 0;
  for (int w = 0; w < nw; ++w) {
    aa += lds[3 * w + 0];
    ab2 += lds[3 * w + 1];
    bb += lds[3 * w + 2];
  }
  if ((aa | ab2 | bb) == 0) return;
  // total = aa 2^40 + ab2 2^20 + bb (units of 2^-48), carried into digits d0..d2 < 2^20 and the rest d3
  const unsigned long long d0 = bb & 0xfffffull;
  ab2 += bb >> 20;
  const unsigned long long d1 = ab2 & 0xfffffull;
  aa += ab2 >> 20;
  const unsigned long long d2 = aa & 0xfffffull, d3 = aa >> 20;
  unsigned long long* a = sink.sums + (size_t)(which % kSumsqSubs) * kSumsqSubStride;
  if (d0) __hip_atomic_fetch_add(a + 0, d0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (d1) __hip_atomic_fetch_add(a + 1, d1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (d2) __hip_atomic_fetch_add(a + 2, d2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (d3) __hip_atomic_fetch_add(a + 3, d3, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// the value of four digit counters (each the integer sum of one digit over all quadruples)
__device__ __forceinline__ double sumsq_value(unsigned long long d0, unsigned long long d1, unsigned long long d2,
                                              unsigned long long d3) {
  return ((double)d3 * 0x1p12 + (double)d2 * 0x1p-8) + ((double)d1 * 0x1p-28 + (double)d0 * 0x1p-48);
}

// Sum of squares of n FP16 values (bit patterns) into a sink: the fall-back for gradients whose producing kernel has no
// fused form.  Enqueues one launch on `st`.
int sumsq_half_launch(const unsigned short* g16, long long n, const SumsqSink& sink, hipStream_t st);

}  // namespace jz
