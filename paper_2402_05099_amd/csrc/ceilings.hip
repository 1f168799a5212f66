// Two measurement kernels behind include/hydragen_debug.h: what the chip sustains on the two resources the attention
// kernels are priced against, measured on the box the benchmark runs on.  Not part of the attention path.
#include "hg_internal.h"
#include "hydragen_debug.h"
#include "prefix_common.h"

namespace hg {

namespace {

// Register-only loop of v_mfma_f32_32x32x16_bf16: 16 independent accumulator updates per iteration (four accumulators,
// four rounds), nothing else.  With constant operands the matrix cores run at the published rate; with random bf16
// values the same loop pulls the chip to its power limit and the clock drops (the figure an attention kernel on real
// data can approach).  Workgroup 0 reports shader cycles (s_memtime) and 100 MHz ticks (s_memrealtime) of its loop.
__global__ __launch_bounds__(512, 1) void mfma_loop_kernel(int iters, int random_operands, unsigned long long* clocks, float* sink) {
    floatx16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;
    // operands: small constants, or pseudo-random bit patterns with a bf16 exponent in [2^-4, 2^3] (no NaN, no overflow)
    unsigned seed = (blockIdx.x * 512u + threadIdx.x) * 2654435761u + 12345u;
    auto next = [&]() { seed = seed * 1664525u + 1013904223u; return seed; };
    unsigned araw[4][4], braw[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const unsigned r = next();
            // per 16-bit half: sign and 7 mantissa bits random, exponent 123 .. 130
            const unsigned lo = (r & 0x807fu) | ((123u + ((r >> 8) & 7u)) << 7);
            const unsigned hi = ((r >> 16) & 0x807fu) | ((123u + ((r >> 24) & 7u)) << 7);
            araw[i][j] = random_operands ? (lo | (hi << 16)) : 0x3f803f80u;    // 1.0, 1.0
        }
        const unsigned r = next();
        const unsigned lo = (r & 0x807fu) | ((123u + ((r >> 8) & 7u)) << 7);
        const unsigned hi = ((r >> 16) & 0x807fu) | ((123u + ((r >> 24) & 7u)) << 7);
        braw[i] = random_operands ? (lo | (hi << 16)) : 0x3c003c00u;           // 2^-7
    }
    typedef unsigned uintx4 __attribute__((ext_vector_type(4)));
    bf16x8 a[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) a[i] = __builtin_bit_cast(bf16x8, uintx4{araw[i][0], araw[i][1], araw[i][2], araw[i][3]});
    const bf16x8 b = __builtin_bit_cast(bf16x8, uintx4{braw[0], braw[1], braw[2], braw[3]});
    const unsigned long long c0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(i + r) & 3], b, acc[i], 0, 0, 0);
        // keep the sums bounded: random operands would otherwise overflow to infinity within a few thousand rounds
        if ((it & 63) == 63) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 16; ++j) acc[i][j] *= 0.0009765625f;
        }
    }
    const unsigned long long c1 = __builtin_amdgcn_s_memtime(), r1 = __builtin_amdgcn_s_memrealtime();
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) s += acc[i][j];
    if (s == 12345.678f) sink[0] = s;             // never true in practice: keeps the products alive
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        clocks[0] = c1 - c0;
        clocks[1] = r1 - r0;
    }
}

// Plain streaming read: every workgroup walks the buffer with 16-byte nontemporal loads, eight in flight per lane.
typedef unsigned uintv4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void stream_read_kernel(const uintv4* __restrict__ p, size_t n16, float* sink) {
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    unsigned acc = 0;
    for (; i + 7 * stride < n16; i += 8 * stride) {
        uintv4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(p + i + u * stride);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += v[u][u & 3];
    }
    for (; i < n16; i += stride) acc += p[i].x;
    if (acc == 0x12345678u) sink[0] = 1.f;
}

}  // namespace

hipError_t launch_mfma_loop(int iters, int random_operands, unsigned long long* clocks, float* sink, hipStream_t s) {
    mfma_loop_kernel<<<256, 512, 0, s>>>(iters, random_operands, clocks, sink);
    return hipGetLastError();
}

// Which XCD a workgroup runs on: the XCC_ID field (bits 3:0) of the hardware register of that name.  Workgroups are
// handed to the XCDs round-robin, starting wherever the launch before stopped: two workgroups of a launch share an XCD
// exactly when their ids are equal modulo 8.  The shared-block kernels rely on that when they give the workgroups that
// share K/V rows ids that are equal modulo 8; only L2 hits depend on it, no result does.  Launched like the persistent kernel:
// 512 threads and all of a CU's LDS per workgroup.
__global__ __launch_bounds__(512) void xcd_probe_kernel(int* out) {
    extern __shared__ unsigned char probe_smem[];
    if (threadIdx.x == 0) {
        probe_smem[0] = 1;
        const unsigned id = __builtin_amdgcn_s_getreg((3 << 11) | (0 << 6) | 20);     // hwreg(HW_REG_XCC_ID, 0, 4)
        out[blockIdx.x] = (int)(id & 15u) + (probe_smem[0] - 1);
    }
}

hipError_t launch_xcd_probe(int n_workgroups, int* out, hipStream_t s) {
    constexpr int kLds = 160 * 1024;
    static bool attr_set[64] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 64 && !attr_set[dev]) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&xcd_probe_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
        if (e != hipSuccess) return e;
        attr_set[dev] = true;
    }
    xcd_probe_kernel<<<n_workgroups, 512, kLds, s>>>(out);
    return hipGetLastError();
}

hipError_t launch_stream_read(const void* src, size_t bytes, float* sink, hipStream_t s) {
    stream_read_kernel<<<256 * 8, 256, 0, s>>>(static_cast<const uintv4*>(src), bytes / 16, sink);
    return hipGetLastError();
}

}  // namespace hg
