// Types and lane-exchange helpers shared by the two shared-block attention kernels (gfx950 only).
#pragma once
#include "hg_internal.h"

namespace hg {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx8 __attribute__((ext_vector_type(8)));
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef short shortx8 __attribute__((ext_vector_type(8)));

#define HG_LDS(p) ((__attribute__((address_space(3))) unsigned char*)(p))
#define HG_GLOBAL(p) ((const __attribute__((address_space(1))) void*)(p))

// Value held by the lane 32 positions away.  v_permlane32_swap exchanges the upper 32 lanes of its first
// operand with the lower 32 lanes of its second, so the partner's value arrives in the first result for
// the upper half of the wavefront and in the second result for the lower half.
__device__ __forceinline__ float other_half(float x) {
    const unsigned u = __builtin_bit_cast(unsigned, x);
    auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __builtin_bit_cast(float, (threadIdx.x & 32) ? r[0] : r[1]);
}
__device__ __forceinline__ float half_max(float x) { return fmaxf(x, other_half(x)); }
__device__ __forceinline__ float half_sum(float x) { return x + other_half(x); }

}  // namespace hg
