// Per-sequence decode attention over a list of key spans: the suffix part of Hydragen (Sec. 3.2, last
// paragraph: one query per sequence, no batching across sequences) and, with the shared blocks added to
// the span list, the non-decomposed per-sequence comparison (what Sec. 1 / Sec. 2.3 say existing decode
// kernels do: every sequence re-reads the shared rows).  Memory-bound: one wavefront per work item
// (sequence, KV head, group of GT query heads, key chunk), 16-byte bf16 loads, fp32 arithmetic on the
// vector ALU, DPP reductions inside the 16-lane row that holds one key.
#include "hg_internal.h"

namespace hg {

template <int CTRL>
__device__ __forceinline__ float dpp_f32(float x) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true));
}

// sum over the LPR (8 or 16) lanes that share one key row; every lane of the row gets the total
template <int LPR>
__device__ __forceinline__ float row_allreduce_sum(float x) {
    x += dpp_f32<0xB1>(x);   // quad_perm [1,0,3,2]
    x += dpp_f32<0x4E>(x);   // quad_perm [2,3,0,1]
    x += dpp_f32<0x141>(x);  // row_half_mirror: pairs the two quads of each 8 lanes
    if constexpr (LPR == 16) x += dpp_f32<0x140>(x);  // row_mirror: pairs the two halves of 16 lanes
    return x;
}

// tells the compiler that a pointer is the same in every lane of the wavefront (it then lives in scalar registers)
__device__ __forceinline__ const unsigned char* uniform_ptr(const unsigned char* p) {
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const unsigned char*>(((uint64_t)hi << 32) | lo);
}

template <int D, int GT>
struct DecodeState {
    float q[GT][8];    // query elements of this lane's 8-wide column slice, pre-multiplied by scale*log2(e)
    float m[GT];       // running max (log2 domain)
    float l[GT];       // running sum of 2^(s-m)
    float acc[GT][8];  // running sum of 2^(s-m) * v
};

// One batch of U wave-wide loads: KPW keys each, K and V rows of this lane's 8-column slice.
template <int D, int U>
struct KVBatch {
    uint4 k[U], v[U];
};

// 16-byte load from global memory at uniform base + 32-bit lane offset (scalar base register + vector offset form)
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
// STREAM: rows read exactly once (suffix KV) bypass the caches' retention; shared rows are loaded normally so that
// the re-reads of other sequences can hit in L2 / Infinity Cache
template <bool STREAM>
__device__ __forceinline__ uint4 ldg128(const unsigned char* base, unsigned off) {
    const auto* p = reinterpret_cast<const __attribute__((address_space(1))) u32x4*>(
        (const __attribute__((address_space(1))) unsigned char*)base + off);
    const u32x4 v = STREAM ? __builtin_nontemporal_load(p) : *p;
    return make_uint4(v.x, v.y, v.z, v.w);
}

// kb/vb: wavefront-uniform byte pointers to the span's first row of this KV head; rowoff: this lane's byte offset
// of its key in load 0 of the batch (sub-row, column slice and batch start); colb: the column part alone.  Lanes
// whose key lies past the span read the span's first row instead (always valid; their score is masked), so no
// load is predicated and a batch may be requested past the end of the span.
template <int D, int U, bool STREAM>
__device__ __forceinline__ void load_batch(KVBatch<D, U>& bt, const unsigned char* __restrict__ kb,
                                           const unsigned char* __restrict__ vb, unsigned rstride_b, unsigned rowoff,
                                           unsigned colb, int first, int n) {
    constexpr int KPW = 64 / (D / 8);
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int i = first + u * KPW;   // `first` already includes this lane's sub-row
        const unsigned off = i < n ? (unsigned)(u * KPW) * rstride_b + rowoff : colb;
        bt.k[u] = ldg128<STREAM>(kb, off);
        bt.v[u] = ldg128<STREAM>(vb, off);
    }
}

// online-softmax update of the state with one batch (keys first + u*KPW, masked beyond n)
template <int D, int GT, int U>
__device__ __forceinline__ void consume_batch(DecodeState<D, GT>& st, const KVBatch<D, U>& bt, int first, int n) {
    constexpr int LPR = D / 8;
    constexpr int KPW = 64 / LPR;
    float s[U][GT];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const bool ok = first + u * KPW < n;
        const uint4 kr = bt.k[u];
        const float k0 = bf16_lo(kr.x), k1 = bf16_hi(kr.x), k2 = bf16_lo(kr.y), k3 = bf16_hi(kr.y);
        const float k4 = bf16_lo(kr.z), k5 = bf16_hi(kr.z), k6 = bf16_lo(kr.w), k7 = bf16_hi(kr.w);
#pragma unroll
        for (int g = 0; g < GT; ++g) {
            float d = st.q[g][0] * k0;
            d = fmaf(st.q[g][1], k1, d);
            d = fmaf(st.q[g][2], k2, d);
            d = fmaf(st.q[g][3], k3, d);
            d = fmaf(st.q[g][4], k4, d);
            d = fmaf(st.q[g][5], k5, d);
            d = fmaf(st.q[g][6], k6, d);
            d = fmaf(st.q[g][7], k7, d);
            d = row_allreduce_sum<LPR>(d);
            s[u][g] = ok ? d : -INFINITY;
        }
    }
#pragma unroll
    for (int g = 0; g < GT; ++g) {
        float mx = st.m[g];
#pragma unroll
        for (int u = 0; u < U; ++u) mx = fmaxf(mx, s[u][g]);
        const float ms = (mx == -INFINITY) ? 0.f : mx;
        const float alpha = __builtin_amdgcn_exp2f(st.m[g] - ms);
        st.m[g] = mx;
        float p[U];
        float ps = 0.f;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            p[u] = __builtin_amdgcn_exp2f(s[u][g] - ms);
            ps += p[u];
        }
        st.l[g] = fmaf(st.l[g], alpha, ps);
#pragma unroll
        for (int j = 0; j < 8; ++j) st.acc[g][j] *= alpha;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint4 vr = bt.v[u];
            st.acc[g][0] = fmaf(p[u], bf16_lo(vr.x), st.acc[g][0]);
            st.acc[g][1] = fmaf(p[u], bf16_hi(vr.x), st.acc[g][1]);
            st.acc[g][2] = fmaf(p[u], bf16_lo(vr.y), st.acc[g][2]);
            st.acc[g][3] = fmaf(p[u], bf16_hi(vr.y), st.acc[g][3]);
            st.acc[g][4] = fmaf(p[u], bf16_lo(vr.z), st.acc[g][4]);
            st.acc[g][5] = fmaf(p[u], bf16_hi(vr.z), st.acc[g][5]);
            st.acc[g][6] = fmaf(p[u], bf16_lo(vr.w), st.acc[g][6]);
            st.acc[g][7] = fmaf(p[u], bf16_hi(vr.w), st.acc[g][7]);
        }
    }
}

// Online-softmax pass over `n` consecutive KV rows starting at row0, KV head kvh.  Software pipelined: the
// loads of the next batch are issued before the current batch is consumed, so a wavefront always has a
// batch in flight while it computes.
template <int D, int GT, bool STREAM>
__device__ __forceinline__ void decode_span(DecodeState<D, GT>& st, const uint16_t* __restrict__ K,
                                            const uint16_t* __restrict__ V, int64_t row0, int n, int Hkv, int kvh,
                                            int lane) {
    constexpr int LPR = D / 8;
    constexpr int KPW = 64 / LPR;
    constexpr int U = GT >= 8 ? 2 : 4;
    constexpr int STEP = KPW * U;
    const int sub = lane / LPR;
    const unsigned rstride_b = (unsigned)Hkv * D * 2u;
    const unsigned colb = (unsigned)(lane % LPR) * 16u;
    unsigned rowoff = (unsigned)sub * rstride_b + colb;
    const unsigned char* kb = uniform_ptr(reinterpret_cast<const unsigned char*>(K + (row0 * Hkv + kvh) * (int64_t)D));
    const unsigned char* vb = uniform_ptr(reinterpret_cast<const unsigned char*>(V + (row0 * Hkv + kvh) * (int64_t)D));
    const unsigned step_b = (unsigned)STEP * rstride_b;

    // every load is issued unconditionally (see load_batch), so the wait counts the compiler derives are exact
    KVBatch<D, U> ba, bb;
    load_batch<D, U, STREAM>(ba, kb, vb, rstride_b, rowoff, colb, sub, n);
    for (int it = 0; it < n; it += 2 * STEP) {
        rowoff += step_b;
        load_batch<D, U, STREAM>(bb, kb, vb, rstride_b, rowoff, colb, it + STEP + sub, n);
        __builtin_amdgcn_sched_barrier(0);   // keep the loads ahead of the arithmetic that hides their latency
        consume_batch<D, GT, U>(st, ba, it + sub, n);
        rowoff += step_b;
        __builtin_amdgcn_sched_barrier(0);
        load_batch<D, U, STREAM>(ba, kb, vb, rstride_b, rowoff, colb, it + 2 * STEP + sub, n);
        __builtin_amdgcn_sched_barrier(0);
        if (it + STEP < n) consume_batch<D, GT, U>(st, bb, it + STEP + sub, n);
    }
}

// The same pass over rows [start, start+n) of sequence b's suffix when the rows live in a paged pool (`start` is a
// multiple of 32, the span touches at most 64 pages: the host bounds the chunk by 32 pages).  Lane i of the
// wavefront holds the physical page of the span's i-th logical page; the 4 or 8 keys of one wave-wide load never
// straddle a page (pages hold at least 16 rows), so the page of a load is wavefront-uniform: one v_readlane and
// a few scalar instructions per load, the same unpredicated vector loads and the same pipeline as above.
template <int D, int GT>
__device__ __forceinline__ void decode_span_paged(DecodeState<D, GT>& st, const uint16_t* __restrict__ K,
                                                  const uint16_t* __restrict__ V, const PagedDev& pg, int b, int start,
                                                  int n, int Hkv, int kvh, int lane) {
    constexpr int LPR = D / 8;
    constexpr int KPW = 64 / LPR;
    constexpr int U = GT >= 8 ? 2 : 4;
    constexpr int STEP = KPW * U;
    const int sub = lane / LPR;
    const unsigned rstride_b = (unsigned)Hkv * D * 2u;
    const unsigned colb = (unsigned)(lane % LPR) * 16u;
    const unsigned subrow = (unsigned)sub * rstride_b + colb;
    const unsigned char* kb = uniform_ptr(reinterpret_cast<const unsigned char*>(K + (int64_t)kvh * D));
    const unsigned char* vb = uniform_ptr(reinterpret_cast<const unsigned char*>(V + (int64_t)kvh * D));
    const int shift = pg.shift;
    const int lp0 = start >> shift;
    const int lpn = ((start + n - 1) >> shift) - lp0 + 1;
    int pages = 0;
    if (lane < lpn) pages = pg.table[(int64_t)b * pg.stride + lp0 + lane];
    pages = min(max(pages, 0), pg.n_pages - 1);
    // byte offset of the pool row that holds the span's key i0 (i0: wavefront-uniform multiple of KPW)
    auto row_base = [&](int i0) -> unsigned {
        const int pos = start + i0;
        const int page = __builtin_amdgcn_readlane(pages, ((pos >> shift) - lp0) & 63);
        return ((unsigned)(page << shift) + (unsigned)(pos & ((1 << shift) - 1))) * rstride_b;
    };
    const unsigned safe = row_base(0) + colb;   // lanes past the span read its first row (their scores are masked)
    auto load = [&](KVBatch<D, U>& bt, int i0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int iu = i0 + u * KPW;
            const unsigned off = iu + sub < n ? row_base(iu) + subrow : safe;
            bt.k[u] = ldg128<true>(kb, off);
            bt.v[u] = ldg128<true>(vb, off);
        }
    };

    KVBatch<D, U> ba, bb;
    load(ba, 0);
    for (int it = 0; it < n; it += 2 * STEP) {
        load(bb, it + STEP);
        __builtin_amdgcn_sched_barrier(0);
        consume_batch<D, GT, U>(st, ba, it + sub, n);
        __builtin_amdgcn_sched_barrier(0);
        load(ba, it + 2 * STEP);
        __builtin_amdgcn_sched_barrier(0);
        if (it + STEP < n) consume_batch<D, GT, U>(st, bb, it + STEP + sub, n);
    }
}

// rows [begin, begin+count) of the block of level `lv` that covers sequence b (count = 0 if none)
__device__ __forceinline__ void block_of(const LevelDev& lv, int b, int B, int& begin, int& count) {
    if (lv.n_blocks == 1 && lv.seq_off == nullptr) {
        begin = 0;
        count = lv.max_rows;
        return;
    }
    int lo = 0, hi = lv.n_blocks;  // find g with seq_off[g] <= b < seq_off[g+1]
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (lv.seq_off[mid + 1] <= b) lo = mid + 1;
        else hi = mid;
    }
    begin = 0;
    count = 0;
    if (lo < lv.n_blocks && lv.seq_off[lo] <= b) {
        begin = lv.kv_off[lo];
        count = min(lv.kv_off[lo + 1] - begin, lv.max_rows);
        if (count < 0) count = 0;
    }
}

// SHARED = false: suffix rows only (the Hydragen suffix part).  SHARED = true: the shared blocks of every level
// are walked too (the non-decomposed comparison); a separate instantiation so that profiles tell them apart.
// PAGED (only without SHARED): the suffix rows are read through a page table.
template <int D, int GT, bool SHARED, bool PAGED>
__global__ __launch_bounds__(256) void decode_kernel(DecodeArgs a) {
    constexpr int LPR = D / 8;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    int64_t u = (int64_t)blockIdx.x * 4 + wave;
    if (u >= a.units) return;
    const int GB = a.G / GT;
    const int gb = (int)(u % GB); u /= GB;
    const int kvh = (int)(u % a.Hkv); u /= a.Hkv;
    const int c = (int)(u % a.nchunks);
    const int bq = (int)(u / a.nchunks);     // (sequence, query) pair: b*nq + t
    const int b = bq / a.nq;
    const int tq = bq % a.nq;
    const int h0 = kvh * a.G + gb * GT;  // first query head of this work item

    DecodeState<D, GT> st;
    {
        const float qs = a.scale * kLog2e;
        const int col = (lane % LPR) * 8;
#pragma unroll
        for (int g = 0; g < GT; ++g) {
            const uint4 qv = *reinterpret_cast<const uint4*>(a.Q + ((int64_t)bq * a.Hq + h0 + g) * D + col);
            st.q[g][0] = bf16_lo(qv.x) * qs; st.q[g][1] = bf16_hi(qv.x) * qs;
            st.q[g][2] = bf16_lo(qv.y) * qs; st.q[g][3] = bf16_hi(qv.y) * qs;
            st.q[g][4] = bf16_lo(qv.z) * qs; st.q[g][5] = bf16_hi(qv.z) * qs;
            st.q[g][6] = bf16_lo(qv.w) * qs; st.q[g][7] = bf16_hi(qv.w) * qs;
            st.m[g] = -INFINITY;
            st.l[g] = 0.f;
#pragma unroll
            for (int j = 0; j < 8; ++j) st.acc[g][j] = 0.f;
        }
    }

    // walk the concatenated key list (shared blocks root first, then the suffix), clipped to this chunk
    const int64_t lo = (int64_t)c * a.chunk, hi = lo + a.chunk;
    int64_t pos = 0;
    for (int li = 0; SHARED && li < a.n_levels; ++li) {
        int begin, count;
        block_of(a.lv[li], b, a.B, begin, count);
        const int64_t s0 = max(lo, pos), s1 = min(hi, pos + count);
        if (s0 < s1) decode_span<D, GT, false>(st, a.lv[li].K, a.lv[li].V, begin + (s0 - pos), (int)(s1 - s0), a.Hkv, kvh, lane);
        pos += count;
    }
    if (a.lengths) {
        // the nq queries of a sequence are its last nq suffix tokens: query t does not see the later ones
        int count = min(a.lengths[b], a.max_len) - (a.nq - 1 - tq);
        if (count < 0) count = 0;
        const int64_t s0 = max(lo, pos), s1 = min(hi, pos + count);
        if (s0 < s1) {
            if constexpr (PAGED) decode_span_paged<D, GT>(st, a.Ks, a.Vs, a.pg, b, (int)s0, (int)(s1 - s0), a.Hkv, kvh, lane);
            else decode_span<D, GT, true>(st, a.Ks, a.Vs, a.offsets[b] + (s0 - pos), (int)(s1 - s0), a.Hkv, kvh, lane);
        }
    }

    // combine the 64/LPR key sub-streams of the wavefront and write (O, LSE)
#pragma unroll
    for (int g = 0; g < GT; ++g) {
        float M = st.m[g];
#pragma unroll
        for (int off = LPR; off < 64; off <<= 1) M = fmaxf(M, __shfl_xor(M, off));
        const float Ms = (M == -INFINITY) ? 0.f : M;
        const float f = __builtin_amdgcn_exp2f(st.m[g] - Ms);
        float l = st.l[g] * f;
#pragma unroll
        for (int off = LPR; off < 64; off <<= 1) l += __shfl_xor(l, off);
        float o[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            o[j] = st.acc[g][j] * f;
#pragma unroll
            for (int off = LPR; off < 64; off <<= 1) o[j] += __shfl_xor(o[j], off);
        }
        if (lane < LPR) {
            const float inv = l > 0.f ? 1.0f / l : 0.f;
            const int64_t idx = (int64_t)bq * a.Hq + h0 + g;
            const int64_t e = (int64_t)c * a.out.part_stride_O + idx * D + lane * 8;
            if (a.out.bf16) {
                uint4 v;
                v.x = pack_bf16(o[0] * inv, o[1] * inv); v.y = pack_bf16(o[2] * inv, o[3] * inv);
                v.z = pack_bf16(o[4] * inv, o[5] * inv); v.w = pack_bf16(o[6] * inv, o[7] * inv);
                *reinterpret_cast<uint4*>(static_cast<uint16_t*>(a.out.O) + e) = v;
            } else {
                float* op = static_cast<float*>(a.out.O) + e;
                *reinterpret_cast<float4*>(op) = make_float4(o[0] * inv, o[1] * inv, o[2] * inv, o[3] * inv);
                *reinterpret_cast<float4*>(op + 4) = make_float4(o[4] * inv, o[5] * inv, o[6] * inv, o[7] * inv);
            }
            if (lane == 0)
                a.out.LSE[(int64_t)c * a.out.part_stride_L + idx] = l > 0.f ? (Ms + __log2f(l)) * kLn2 : -INFINITY;
        }
    }
}

template <int D, int GT>
static hipError_t launch_decode_t(const DecodeArgs& a, hipStream_t s) {
    if (a.units == 0) return hipSuccess;
    const int64_t grid = (a.units + 3) / 4;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    if (a.pg.table) {
        if (a.n_levels > 0) return hipErrorInvalidValue;   // the comparison kernel has no paged form
        decode_kernel<D, GT, false, true><<<(unsigned)grid, 256, 0, s>>>(a);
    } else if (a.n_levels > 0) {
        decode_kernel<D, GT, true, false><<<(unsigned)grid, 256, 0, s>>>(a);
    } else {
        decode_kernel<D, GT, false, false><<<(unsigned)grid, 256, 0, s>>>(a);
    }
    return hipGetLastError();
}

hipError_t launch_decode(const DecodeArgs& a, int D, int GT, hipStream_t s) {
    if (D == 128) {
        switch (GT) {
            case 1: return launch_decode_t<128, 1>(a, s);
            case 2: return launch_decode_t<128, 2>(a, s);
            case 4: return launch_decode_t<128, 4>(a, s);
            case 8: return launch_decode_t<128, 8>(a, s);
        }
    } else if (D == 64) {
        switch (GT) {
            case 1: return launch_decode_t<64, 1>(a, s);
            case 2: return launch_decode_t<64, 2>(a, s);
            case 4: return launch_decode_t<64, 4>(a, s);
            case 8: return launch_decode_t<64, 8>(a, s);
        }
    }
    return hipErrorInvalidValue;
}

}  // namespace hg
