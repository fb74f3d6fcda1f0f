// Loads for data that a kernel touches once (the 4-bit codes of a W4A16 product): marked
// non-temporal, so the lines are not kept in the caches on the way in.  Reading a layer larger than
// the caches this way left 7-10 % more of the HBM bandwidth to the product on an MI355X.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace aaac {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint4 load_once_16(const void* p) {  // p 16-byte aligned
  const u32x4_t t = __builtin_nontemporal_load(static_cast<const u32x4_t*>(p));
  return make_uint4(t.x, t.y, t.z, t.w);
}

}  // namespace aaac
