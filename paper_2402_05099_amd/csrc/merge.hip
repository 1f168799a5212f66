// n-way LSE merge (Eq. 5 of the paper, generalised from two parts to n; App. B's combine routine
// is the two-part form with the largest LSE subtracted first).  HBM-bound elementwise kernel.
#include "hg_internal.h"

namespace hg {

// D/4 lanes per query row, 4 output elements per lane.  Parts with LSE = -inf are skipped (their O may
// be uninitialised memory); a row whose parts are all empty becomes O = 0, LSE = -inf.
// Parts are taken four at a time: their LSEs, then the O pieces of the non-empty ones, are loaded before any is
// used, so that a lane has up to four 16-byte loads in flight; the running maximum is carried across groups (the
// accumulators are rescaled when it grows), which equals the one-pass formula with the global maximum.
template <int D, bool IN_BF16, bool OUT_BF16>
__global__ __launch_bounds__(256) void merge_kernel(MergeArgs a) {
    constexpr int LPR = D / 4;
    constexpr int RPB = 256 / LPR;
    constexpr int U = 4;
    const int64_t row = (int64_t)blockIdx.x * RPB + threadIdx.x / LPR;
    if (row >= a.rows) return;
    const int c = threadIdx.x % LPR;

    float m = -INFINITY;            // running maximum of the LSEs seen so far
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    float den = 0.f;
    for (int i0 = 0; i0 < a.n; i0 += U) {
        float li[U];
        float o[U][4];
#pragma unroll
        for (int u = 0; u < U; ++u) li[u] = i0 + u < a.n ? a.L[i0 + u][row] : -INFINITY;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            o[u][0] = o[u][1] = o[u][2] = o[u][3] = 0.f;
            if (li[u] != -INFINITY) {
                if constexpr (IN_BF16) {
                    const uint2 v = *reinterpret_cast<const uint2*>(static_cast<const uint16_t*>(a.O[i0 + u]) + row * D + 4 * c);
                    o[u][0] = bf16_lo(v.x); o[u][1] = bf16_hi(v.x); o[u][2] = bf16_lo(v.y); o[u][3] = bf16_hi(v.y);
                } else {
                    const float4 v = *reinterpret_cast<const float4*>(static_cast<const float*>(a.O[i0 + u]) + row * D + 4 * c);
                    o[u][0] = v.x; o[u][1] = v.y; o[u][2] = v.z; o[u][3] = v.w;
                }
            }
        }
        float gm = li[0];
#pragma unroll
        for (int u = 1; u < U; ++u) gm = fmaxf(gm, li[u]);
        if (gm > m) {               // (false while everything seen is empty)
            const float r = __builtin_amdgcn_exp2f((m - gm) * kLog2e);   // m = -inf: 0, and acc = den = 0 anyway
            den *= r;
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[j] *= r;
            m = gm;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (li[u] != -INFINITY) {
                const float w = __builtin_amdgcn_exp2f((li[u] - m) * kLog2e);
                den += w;
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[j] = fmaf(w, o[u][j], acc[j]);
            }
        }
    }
    if (m > -INFINITY) {
        const float inv = 1.0f / den;
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] *= inv;
    }
    if constexpr (OUT_BF16) {
        uint2 v;
        v.x = pack_bf16(acc[0], acc[1]);
        v.y = pack_bf16(acc[2], acc[3]);
        *reinterpret_cast<uint2*>(static_cast<uint16_t*>(a.O_out) + row * D + 4 * c) = v;
    } else {
        *reinterpret_cast<float4*>(static_cast<float*>(a.O_out) + row * D + 4 * c) = make_float4(acc[0], acc[1], acc[2], acc[3]);
    }
    if (a.L_out && c == 0) a.L_out[row] = (m > -INFINITY) ? m + __logf(den) : -INFINITY;
}

template <int D>
static hipError_t launch_merge_d(const MergeArgs& a, bool in_bf16, bool out_bf16, hipStream_t s) {
    constexpr int RPB = 256 / (D / 4);
    if (a.rows == 0) return hipSuccess;
    const unsigned grid = (unsigned)((a.rows + RPB - 1) / RPB);
    if (in_bf16) {
        if (out_bf16) merge_kernel<D, true, true><<<grid, 256, 0, s>>>(a);
        else merge_kernel<D, true, false><<<grid, 256, 0, s>>>(a);
    } else {
        if (out_bf16) merge_kernel<D, false, true><<<grid, 256, 0, s>>>(a);
        else merge_kernel<D, false, false><<<grid, 256, 0, s>>>(a);
    }
    return hipGetLastError();
}

hipError_t launch_merge(const MergeArgs& a, int D, bool in_bf16, bool out_bf16, hipStream_t s) {
    return D == 128 ? launch_merge_d<128>(a, in_bf16, out_bf16, s) : launch_merge_d<64>(a, in_bf16, out_bf16, s);
}

// O = 0, LSE = -inf for `rows` query rows (the result of attention over an empty key set).
// Either pointer may be null (then only the other is written).
__global__ __launch_bounds__(256) void fill_empty_kernel(FillArgs a) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;  // one 4-element group of O per thread
    const int64_t groups = a.rows * (a.D / 4);
    if (a.O && i < groups) {
        if (a.bf16) reinterpret_cast<uint2*>(a.O)[i] = make_uint2(0u, 0u);
        else reinterpret_cast<float4*>(a.O)[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    if (a.LSE && i < a.rows) a.LSE[i] = -INFINITY;
}

hipError_t launch_fill_empty(const FillArgs& a, hipStream_t s) {
    if (a.rows == 0 || (!a.O && !a.LSE)) return hipSuccess;
    const int64_t n = a.O ? a.rows * (a.D / 4) : a.rows;
    fill_empty_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(a);
    return hipGetLastError();
}

}  // namespace hg
