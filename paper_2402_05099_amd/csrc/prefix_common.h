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

// Sequences that no block of a grouped level covers (those before the first block's range, behind the last block's, or
// behind the first max_seqs sequences of a block) get an empty result from that level: LSE = -inf in each of the
// level's `nparts` parts (the merge never reads the O of such a part), and O = 0 as well when the level's result is
// written in place (one part, no stride).  The level's n_blocks + 2 candidate ranges are dealt out to the launch's
// workgroups (range r to workgroup r % nwg); the kernels that call this write those rows nowhere else.
__device__ __forceinline__ void mark_uncovered(const PrefixArgs& a, int D, int nparts, int wg, int nwg) {
    if (!a.lv.seq_off) return;     // a level of one block covers every sequence
    const int n = a.lv.n_blocks;
    const int per_seq = a.nq * a.Hq;
    for (int r = wg; r < n + 2; r += nwg) {
        int lo, hi;
        if (r == 0) {
            lo = 0;
            hi = a.lv.seq_off[0];
        } else if (r == n + 1) {
            lo = a.lv.seq_off[n];
            hi = a.B;
        } else {
            hi = a.lv.seq_off[r];
            lo = min(a.lv.seq_off[r - 1] + a.lv.max_seqs, hi);
        }
        lo = max(lo, 0);
        hi = min(hi, a.B);
        if (lo >= hi) continue;
        const int64_t e0 = (int64_t)lo * per_seq, ne = (int64_t)(hi - lo) * per_seq;
        for (int64_t i = threadIdx.x; i < ne * nparts; i += blockDim.x) {
            const int64_t part = i / ne;
            a.out.LSE[part * a.out.part_stride_L + e0 + (i - part * ne)] = -INFINITY;
        }
        if (a.out.part_stride_L == 0) {     // the final output: zero rows
            const int cpr = D / 4;          // pieces of four elements per row
            for (int64_t i = threadIdx.x; i < ne * cpr; i += blockDim.x) {
                const int64_t off = (e0 + i / cpr) * D + 4 * (i % cpr);
                if (a.out.bf16) *reinterpret_cast<uint2*>(static_cast<uint16_t*>(a.out.O) + off) = make_uint2(0u, 0u);
                else *reinterpret_cast<float4*>(static_cast<float*>(a.out.O) + off) = make_float4(0.f, 0.f, 0.f, 0.f);
            }
        }
    }
}

}  // namespace hg
