// Shared host-side helpers of libjz (argument checks, launch error mapping).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "jz.h"

namespace jz {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// [a, a+na) and [b, b+nb) share a byte
inline bool overlaps(const void* a, size_t na, const void* b, size_t nb) {
  if (!a || !b || na == 0 || nb == 0) return false;
  uintptr_t pa = reinterpret_cast<uintptr_t>(a), pb = reinterpret_cast<uintptr_t>(b);
  return pa < pb + nb && pb < pa + na;
}

inline int launch_status() { return hipGetLastError() == hipSuccess ? JZ_OK : JZ_ERR_LAUNCH; }

}  // namespace jz
