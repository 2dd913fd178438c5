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
// Atomics on one cache line queue behind each other (about 12 ns each on MI355X), so a tensor has kSumsqSubs such
// counter quadruples, 128 bytes apart; a contributor picks one by its workgroup index and the reader adds them.
#pragma once
#include <hip/hip_runtime.h>

namespace jz {

constexpr int kSumsqSubs = 64;       // counter quadruples per tensor: one per lane of the wavefront that reads them
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

// one wavefront's total of a 64-bit value, valid in lane 63: row shifts, then the row broadcasts (data-parallel
// primitives: a handful of cycles per step instead of a round trip through the LDS crossbar per shuffle)
__device__ __forceinline__ unsigned long long wave_total_u64(unsigned long long v) {
#if defined(__HIP_DEVICE_COMPILE__)
  // dpp_ctrl: 0x111.. row_shr:n, 0x142 row_bcast:15, 0x143 row_bcast:31; rows / banks that take part per step as in the
  // usual reduction (bound_ctrl false: lanes without a source keep adding 0 via the `old` operand)
#define JZ_DPP_ADD64(ctrl, row_mask)                                                                          \
  {                                                                                                           \
    const unsigned lo = (unsigned)v, hi = (unsigned)(v >> 32);                                                \
    const unsigned slo = (unsigned)__builtin_amdgcn_update_dpp(0, (int)lo, ctrl, row_mask, 0xf, false);       \
    const unsigned shi = (unsigned)__builtin_amdgcn_update_dpp(0, (int)hi, ctrl, row_mask, 0xf, false);       \
    v += ((unsigned long long)shi << 32) | slo;                                                               \
  }
  JZ_DPP_ADD64(0x111, 0xf)  // row_shr:1
  JZ_DPP_ADD64(0x112, 0xf)  // row_shr:2
  JZ_DPP_ADD64(0x114, 0xf)  // row_shr:4
  JZ_DPP_ADD64(0x118, 0xf)  // row_shr:8   -> lane 15 of every row holds the row's total
  JZ_DPP_ADD64(0x142, 0xa)  // row_bcast:15 into rows 1 and 3
  JZ_DPP_ADD64(0x143, 0xc)  // row_bcast:31 into rows 2 and 3 -> lane 63 holds the wavefront's total
#undef JZ_DPP_ADD64
#endif
  return v;
}

// Workgroup-wide: adds every thread's sums and contributes them to the sink (or raises its flag when any thread saw a
// non-finite value: the update is then skipped as a whole).  Every thread of the workgroup must call it, after a
// barrier behind the last use of `lds`; `lds` is scratch for five 64-bit words that the caller has cleared BEFORE that
// barrier; at most 2^22 elements per workgroup.  No barrier in here: each wavefront adds its totals to the words in LDS
// and counts itself in, and the wavefront that finds every other one counted carries the digits and contributes.
// No memory fence either: a fence would make the wavefront wait for the global stores it has just issued (a microsecond
// or two) before it may count itself in, and it is not needed -- the LDS carries out one wavefront's operations in the
// order they were issued, so a wavefront's sums are in LDS before its count is; the compiler is kept from reordering
// the operations by the empty volatile statements.
__device__ __forceinline__ void sumsq_block_flush(SumsqAcc s, int bad, const SumsqSink& sink, unsigned which,
                                                  unsigned long long* lds) {
  s.aa = wave_total_u64(s.aa);
  s.ab2 = wave_total_u64(s.ab2);
  s.bb = wave_total_u64(s.bb);
  bad = __any(bad);
  if ((threadIdx.x & 63) != 63) return;
  const unsigned nw = blockDim.x >> 6;
  atomicAdd(lds + 0, s.aa);
  atomicAdd(lds + 1, s.ab2);
  atomicAdd(lds + 2, s.bb);
  if (bad) atomicAdd(lds + 3, 1ull);
  asm volatile("" ::: "memory");
  const unsigned long long arrived = atomicAdd(lds + 4, 1ull);
  asm volatile("" ::: "memory");
  if (arrived != nw - 1) return;
  unsigned long long aa = atomicAdd(lds + 0, 0ull), ab2 = atomicAdd(lds + 1, 0ull), bb = atomicAdd(lds + 2, 0ull);
  if (atomicAdd(lds + 3, 0ull) != 0) {
    *sink.nonfinite = 1;
    return;
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
