// 16-byte loads for data that is read exactly once (streamed): the non-temporal hint keeps such data
// from displacing anything in the caches.  Device-side header.
#pragma once
#include <hip/hip_runtime.h>

namespace egtp {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ u32x4 stream_load16(const void *p) { return __builtin_nontemporal_load((const u32x4 *)p); }

}  // namespace egtp
