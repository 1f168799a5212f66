// KV-cache update of a decode step (Sec. 2.2: the cache holds the keys and values of all earlier tokens and every
// step adds the newest token's; Sec. 3.5: suffix lengths change from step to step while the launch sequence stays
// the same, so lengths live on the device and are advanced there).  Pure data movement: one workgroup per sequence
// copies the nq new K and V rows behind the sequence's last suffix row, then its first thread advances the length.
#include "hg_internal.h"

namespace hg {

__global__ __launch_bounds__(256) void kv_append_kernel(AppendArgs a) {
    const int b = blockIdx.x;
    const int len = a.lengths[b];          // every thread reads the old length before thread 0 replaces it
    __syncthreads();
    const int room = a.capacity - len;
    const int take = len < 0 ? 0 : room < a.nq ? (room > 0 ? room : 0) : a.nq;   // rows that fit below the capacity
    const int vec = a.row_elems / 8;       // 16-byte groups per row (Hkv * D is a multiple of 64)
    for (int i = threadIdx.x; i < take * vec; i += 256) {
        const int t = i / vec, c = i - t * vec;
        const int j = len + t;             // suffix row that token t becomes
        int64_t row;
        if (a.pg.table) {
            int page = a.pg.table[(int64_t)b * a.pg.stride + (j >> a.pg.shift)];
            page = min(max(page, 0), a.pg.n_pages - 1);
            row = ((int64_t)page << a.pg.shift) + (j & ((1 << a.pg.shift) - 1));
        } else {
            row = (int64_t)a.offsets[b] + j;
        }
        const int64_t src = ((int64_t)b * a.nq + t) * vec + c;
        const int64_t dst = row * vec + c;
        reinterpret_cast<uint4*>(a.Ks)[dst] = reinterpret_cast<const uint4*>(a.Knew)[src];
        reinterpret_cast<uint4*>(a.Vs)[dst] = reinterpret_cast<const uint4*>(a.Vnew)[src];
    }
    if (threadIdx.x == 0 && take > 0) a.lengths[b] = len + take;
}

// E4M3 codes of eight bf16 values divided by `scale`: the fp32 quotient (correctly rounded division), magnitudes
// above 448 saturated, then the hardware's round-to-nearest-even conversion; NaN stays NaN.
__device__ __forceinline__ uint2 quantize8(const uint4& r, float scale) {
    const float f[8] = {bf16_lo(r.x), bf16_hi(r.x), bf16_lo(r.y), bf16_hi(r.y), bf16_lo(r.z), bf16_hi(r.z), bf16_lo(r.w), bf16_hi(r.w)};
    float q[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const float x = f[i] / scale;
        q[i] = x != x ? x : fminf(fmaxf(x, -448.0f), 448.0f);
    }
    int lo = 0, hi = 0;
    lo = __builtin_amdgcn_cvt_pk_fp8_f32(q[0], q[1], lo, false);
    lo = __builtin_amdgcn_cvt_pk_fp8_f32(q[2], q[3], lo, true);
    hi = __builtin_amdgcn_cvt_pk_fp8_f32(q[4], q[5], hi, false);
    hi = __builtin_amdgcn_cvt_pk_fp8_f32(q[6], q[7], hi, true);
    return make_uint2((unsigned)lo, (unsigned)hi);
}

// The same update for a cache of E4M3 codes: the new bf16 rows are quantised on the way in.
__global__ __launch_bounds__(256) void kv_append_fp8_kernel(AppendArgs a) {
    const int b = blockIdx.x;
    const int len = a.lengths[b];
    __syncthreads();
    const int room = a.capacity - len;
    const int take = len < 0 ? 0 : room < a.nq ? (room > 0 ? room : 0) : a.nq;
    const int vec = a.row_elems / 8;       // 8-element groups per row: 16 bytes in, 8 bytes out
    for (int i = threadIdx.x; i < take * vec; i += 256) {
        const int t = i / vec, c = i - t * vec;
        const int j = len + t;
        int64_t row;
        if (a.pg.table) {
            int page = a.pg.table[(int64_t)b * a.pg.stride + (j >> a.pg.shift)];
            page = min(max(page, 0), a.pg.n_pages - 1);
            row = ((int64_t)page << a.pg.shift) + (j & ((1 << a.pg.shift) - 1));
        } else {
            row = (int64_t)a.offsets[b] + j;
        }
        const int64_t src = ((int64_t)b * a.nq + t) * vec + c;
        const int64_t dst = row * vec + c;
        reinterpret_cast<uint2*>(a.Ks)[dst] = quantize8(reinterpret_cast<const uint4*>(a.Knew)[src], a.k_scale);
        reinterpret_cast<uint2*>(a.Vs)[dst] = quantize8(reinterpret_cast<const uint4*>(a.Vnew)[src], a.v_scale);
    }
    if (threadIdx.x == 0 && take > 0) a.lengths[b] = len + take;
}

hipError_t launch_kv_append(const AppendArgs& a, hipStream_t s) {
    if (a.B == 0) return hipSuccess;
    if (a.fp8) {
        kv_append_fp8_kernel<<<(unsigned)a.B, 256, 0, s>>>(a);
    } else {
        kv_append_kernel<<<(unsigned)a.B, 256, 0, s>>>(a);
    }
    return hipGetLastError();
}

}  // namespace hg
