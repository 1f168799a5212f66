// Per-sequence decode attention over a list of key spans: the suffix part of Hydragen (Sec. 3.2, last
// paragraph: one query per sequence, no batching across sequences) and, with the shared blocks added to
// the span list, the non-decomposed per-sequence comparison (what Sec. 1 / Sec. 2.3 say existing decode
// kernels do: every sequence re-reads the shared rows).  Memory-bound: one wavefront per work item
// (sequence, KV head, group of GT query heads, key chunk), 16-byte bf16 loads, fp32 arithmetic on the
// vector ALU, DPP reductions inside the 16-lane row that holds one key.
// FP8 = true (suffix rows only, packed or paged): the cache holds 8-bit E4M3 codes with one fp32 scale per tensor (not in the
// paper: half the bytes for the part of the method that is bound by them).  The same lanes own the same 8 columns,
// fetched with 8-byte loads and converted two at a time by the hardware; the K scale is folded into the query, the
// V scale into the final normalisation.
#include <type_traits>

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

// Columns of a row that one lane owns: 8 (one 16-byte load of bf16, one 8-byte load of codes), or 16 codes (one
// 16-byte load) where registers allow: an 8-bit row of D = 128 is then covered by 8 lanes, a wave-wide load brings 8
// keys instead of 4, and the per-key overhead (cross-lane sum, exponential, masks) halves per byte.
template <int D, int GT, bool FP8>
constexpr int epl_of() { return (FP8 && D == 128 && GT <= 2) ? 16 : 8; }

// bf16 rows are multiplied two elements at a time with v_dot2_f32_bf16 (products of bf16 values are exact in fp32, the
// sums are taken in fp32): a score is four such instructions on the packed words of K and Q as they come from memory,
// and the value sums take the rounded weights of two keys against those keys' values of one column.  Set to 0 to fall
// back to unpacking every element to fp32 first (four times the instructions for the scores, twice for the values).
#ifndef HG_DECODE_DOT2
#define HG_DECODE_DOT2 1
#endif
typedef __bf16 bf16pair __attribute__((ext_vector_type(2)));
typedef float f32pair __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned pack_pair_bf16(float lo, float hi) {      // v_cvt_pk_bf16_f32, round to nearest even
    f32pair f = {lo, hi};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(f, bf16pair));
}
__device__ __forceinline__ float dot2_bf16(unsigned a, unsigned b, float c) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16pair, a), __builtin_bit_cast(bf16pair, b), c, false);
}

template <int D, int GT, int EPL = 8>
struct DecodeState {
    float q[GT][EPL];    // query elements of this lane's column slice, pre-multiplied by scale*log2(e)
    unsigned qp[GT][EPL / 2];   // the same elements as packed bf16 pairs, unscaled (bf16 rows with HG_DECODE_DOT2)
    float qs;            // scale*log2(e), applied to a score after its sum (same case)
    float m[GT];         // running max (log2 domain)
    float l[GT];         // running sum of 2^(s-m)
    float acc[GT][EPL];  // running sum of 2^(s-m) * v
};

// One batch of U wave-wide loads: KPW keys each, K and V rows of this lane's 8-column slice.
template <int D, int U, bool FP8, int EPL = 8>
struct KVBatch {
    using Row = std::conditional_t<FP8 && EPL == 8, uint2, uint4>;   // this lane's EPL elements of a row
    Row k[U], v[U];
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
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
template <bool STREAM>
__device__ __forceinline__ uint2 ldg64(const unsigned char* base, unsigned off) {
    const auto* p = reinterpret_cast<const __attribute__((address_space(1))) u32x2*>(
        (const __attribute__((address_space(1))) unsigned char*)base + off);
    const u32x2 v = STREAM ? __builtin_nontemporal_load(p) : *p;
    return make_uint2(v.x, v.y);
}
template <bool STREAM, bool HALF>
__device__ __forceinline__ auto ldg_row(const unsigned char* base, unsigned off) {
    if constexpr (HALF) return ldg64<STREAM>(base, off);
    else return ldg128<STREAM>(base, off);
}

// this lane's 8 elements of a row as fp32
typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void unpack8(const uint4& r, float (&f)[8]) {
    f[0] = bf16_lo(r.x); f[1] = bf16_hi(r.x); f[2] = bf16_lo(r.y); f[3] = bf16_hi(r.y);
    f[4] = bf16_lo(r.z); f[5] = bf16_hi(r.z); f[6] = bf16_lo(r.w); f[7] = bf16_hi(r.w);
}
// 16 codes
__device__ __forceinline__ void unpack8(const uint4& r, float (&f)[16]) {
    const unsigned w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const f32x2 a = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[j], false), b = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[j], true);
        f[4 * j] = a.x; f[4 * j + 1] = a.y; f[4 * j + 2] = b.x; f[4 * j + 3] = b.y;
    }
}
__device__ __forceinline__ void unpack8(const uint2& r, float (&f)[8]) {
    const f32x2 a = __builtin_amdgcn_cvt_pk_f32_fp8((int)r.x, false), b = __builtin_amdgcn_cvt_pk_f32_fp8((int)r.x, true);
    const f32x2 c = __builtin_amdgcn_cvt_pk_f32_fp8((int)r.y, false), d = __builtin_amdgcn_cvt_pk_f32_fp8((int)r.y, true);
    f[0] = a.x; f[1] = a.y; f[2] = b.x; f[3] = b.y; f[4] = c.x; f[5] = c.y; f[6] = d.x; f[7] = d.y;
}

// kb/vb: wavefront-uniform byte pointers to the span's first row of this KV head; rowoff: this lane's byte offset
// of its key in load 0 of the batch (sub-row, column slice and batch start); colb: the column part alone.  Lanes
// whose key lies past the span read the span's first row instead (always valid; their score is masked), so no
// load is predicated and a batch may be requested past the end of the span.
template <int D, int U, bool STREAM, bool FP8, int EPL>
__device__ __forceinline__ void load_batch(KVBatch<D, U, FP8, EPL>& bt, const unsigned char* __restrict__ kb,
                                           const unsigned char* __restrict__ vb, unsigned rstride_b, unsigned rowoff,
                                           unsigned colb, int first, int n) {
    constexpr int KPW = 64 / (D / EPL);
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int i = first + u * KPW;   // `first` already includes this lane's sub-row
        const unsigned off = i < n ? (unsigned)(u * KPW) * rstride_b + rowoff : colb;
        bt.k[u] = ldg_row<STREAM, FP8 && EPL == 8>(kb, off);
        bt.v[u] = ldg_row<STREAM, FP8 && EPL == 8>(vb, off);
    }
}

// online-softmax update of the state with one batch (keys first + u*KPW, masked beyond n)
template <int D, int GT, int U, bool FP8, int EPL>
__device__ __forceinline__ void consume_batch(DecodeState<D, GT, EPL>& st, const KVBatch<D, U, FP8, EPL>& bt, int first, int n) {
    constexpr int LPR = D / EPL;
    constexpr int KPW = 64 / LPR;
    float s[U][GT];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const bool ok = first + u * KPW < n;
        if constexpr (!FP8 && HG_DECODE_DOT2) {
            const unsigned kw[4] = {bt.k[u].x, bt.k[u].y, bt.k[u].z, bt.k[u].w};
#pragma unroll
            for (int g = 0; g < GT; ++g) {
                const float d0 = dot2_bf16(kw[2], st.qp[g][2], dot2_bf16(kw[0], st.qp[g][0], 0.f));     // two chains of two
                const float d1 = dot2_bf16(kw[3], st.qp[g][3], dot2_bf16(kw[1], st.qp[g][1], 0.f));
                const float d = row_allreduce_sum<LPR>(d0 + d1) * st.qs;
                s[u][g] = ok ? d : -INFINITY;
            }
        } else {
            float k[EPL];
            unpack8(bt.k[u], k);
#pragma unroll
            for (int g = 0; g < GT; ++g) {
                float d = st.q[g][0] * k[0];
#pragma unroll
                for (int j = 1; j < EPL; ++j) d = fmaf(st.q[g][j], k[j], d);
                d = row_allreduce_sum<LPR>(d);
                s[u][g] = ok ? d : -INFINITY;
            }
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
        for (int j = 0; j < EPL; ++j) st.acc[g][j] *= alpha;
        if constexpr (!FP8 && HG_DECODE_DOT2) {
            static_assert(FP8 || U % 2 == 0, "keys are taken in pairs");
            // weights of two keys, rounded to bf16 (as the matrix-core kernels round theirs; the row sum above keeps
            // the unrounded ones), against the two keys' values of one column: v_perm_b32 gathers the column's pair
#pragma unroll
            for (int u = 0; u < U; u += 2) {
                const unsigned pp = pack_pair_bf16(p[u], p[u + 1]);
                const unsigned va[4] = {bt.v[u].x, bt.v[u].y, bt.v[u].z, bt.v[u].w};
                const unsigned vb[4] = {bt.v[u + 1].x, bt.v[u + 1].y, bt.v[u + 1].z, bt.v[u + 1].w};
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const unsigned lo = __builtin_amdgcn_perm(vb[w], va[w], 0x05040100u);   // (va.lo, vb.lo)
                    const unsigned hi = __builtin_amdgcn_perm(vb[w], va[w], 0x07060302u);   // (va.hi, vb.hi)
                    st.acc[g][2 * w] = dot2_bf16(lo, pp, st.acc[g][2 * w]);
                    st.acc[g][2 * w + 1] = dot2_bf16(hi, pp, st.acc[g][2 * w + 1]);
                }
            }
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float v[EPL];
                unpack8(bt.v[u], v);
#pragma unroll
                for (int j = 0; j < EPL; ++j) st.acc[g][j] = fmaf(p[u], v[j], st.acc[g][j]);
            }
        }
    }
}

// Online-softmax pass over `n` consecutive KV rows starting at row0, KV head kvh.  Software pipelined: the
// loads of the next batch are issued before the current batch is consumed, so a wavefront always has a
// batch in flight while it computes.
template <int D, int GT, bool STREAM, bool FP8 = false, int EPL = 8>
__device__ __forceinline__ void decode_span(DecodeState<D, GT, EPL>& st, const uint16_t* __restrict__ K,
                                            const uint16_t* __restrict__ V, int64_t row0, int n, int Hkv, int kvh,
                                            int lane) {
    constexpr int LPR = D / EPL;
    constexpr int KPW = 64 / LPR;
    constexpr int U = (GT >= 8 ? 2 : 4) / (EPL / 8);   // the same keys per batch whatever a lane owns of a row
    constexpr int STEP = KPW * U;
    constexpr unsigned ES = FP8 ? 1u : 2u;     // bytes per element
    const int sub = lane / LPR;
    const unsigned rstride_b = (unsigned)Hkv * D * ES;
    const unsigned colb = (unsigned)(lane % LPR) * EPL * ES;
    unsigned rowoff = (unsigned)sub * rstride_b + colb;
    const int64_t first_b = (row0 * Hkv + kvh) * (int64_t)D * ES;
    const unsigned char* kb = uniform_ptr(reinterpret_cast<const unsigned char*>(K) + first_b);
    const unsigned char* vb = uniform_ptr(reinterpret_cast<const unsigned char*>(V) + first_b);
    const unsigned step_b = (unsigned)STEP * rstride_b;

    // every load is issued unconditionally (see load_batch), so the wait counts the compiler derives are exact
    KVBatch<D, U, FP8, EPL> ba, bb;
    load_batch<D, U, STREAM, FP8, EPL>(ba, kb, vb, rstride_b, rowoff, colb, sub, n);
    for (int it = 0; it < n; it += 2 * STEP) {
        rowoff += step_b;
        load_batch<D, U, STREAM, FP8, EPL>(bb, kb, vb, rstride_b, rowoff, colb, it + STEP + sub, n);
        __builtin_amdgcn_sched_barrier(0);   // keep the loads ahead of the arithmetic that hides their latency
        consume_batch<D, GT, U, FP8, EPL>(st, ba, it + sub, n);
        rowoff += step_b;
        __builtin_amdgcn_sched_barrier(0);
        load_batch<D, U, STREAM, FP8, EPL>(ba, kb, vb, rstride_b, rowoff, colb, it + 2 * STEP + sub, n);
        __builtin_amdgcn_sched_barrier(0);
        if (it + STEP < n) consume_batch<D, GT, U, FP8, EPL>(st, bb, it + STEP + sub, n);
    }
}

// The same pass over rows [start, start+n) of sequence b's suffix when the rows live in a paged pool (`start` is a
// multiple of 32, the span touches at most 64 pages: the host bounds the chunk by 32 pages).  Lane i of the
// wavefront holds the physical page of the span's i-th logical page; the 4 or 8 keys of one wave-wide load (64 lanes / lanes per row) never
// straddle a page (pages hold at least 16 rows), so the page of a load is wavefront-uniform: one v_readlane and
// a few scalar instructions per load, the same unpredicated vector loads and the same pipeline as above.
template <int D, int GT, bool FP8 = false, int EPL = 8>
__device__ __forceinline__ void decode_span_paged(DecodeState<D, GT, EPL>& st, const uint16_t* __restrict__ K,
                                                  const uint16_t* __restrict__ V, const PagedDev& pg, int b, int start,
                                                  int n, int Hkv, int kvh, int lane) {
    constexpr int LPR = D / EPL;
    constexpr int KPW = 64 / LPR;
    constexpr int U = (GT >= 8 ? 2 : 4) / (EPL / 8);
    constexpr int STEP = KPW * U;
    constexpr unsigned ES = FP8 ? 1u : 2u;     // bytes per element
    const int sub = lane / LPR;
    const unsigned rstride_b = (unsigned)Hkv * D * ES;
    const unsigned colb = (unsigned)(lane % LPR) * EPL * ES;
    const unsigned subrow = (unsigned)sub * rstride_b + colb;
    const unsigned char* kb = uniform_ptr(reinterpret_cast<const unsigned char*>(K) + (int64_t)kvh * D * ES);
    const unsigned char* vb = uniform_ptr(reinterpret_cast<const unsigned char*>(V) + (int64_t)kvh * D * ES);
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
    auto load = [&](KVBatch<D, U, FP8, EPL>& bt, int i0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int iu = i0 + u * KPW;
            const unsigned off = iu + sub < n ? row_base(iu) + subrow : safe;
            bt.k[u] = ldg_row<true, FP8 && EPL == 8>(kb, off);
            bt.v[u] = ldg_row<true, FP8 && EPL == 8>(vb, off);
        }
    };

    KVBatch<D, U, FP8, EPL> ba, bb;
    load(ba, 0);
    for (int it = 0; it < n; it += 2 * STEP) {
        load(bb, it + STEP);
        __builtin_amdgcn_sched_barrier(0);
        consume_batch<D, GT, U, FP8, EPL>(st, ba, it + sub, n);
        __builtin_amdgcn_sched_barrier(0);
        load(ba, it + 2 * STEP);
        __builtin_amdgcn_sched_barrier(0);
        if (it + STEP < n) consume_batch<D, GT, U, FP8, EPL>(st, bb, it + STEP + sub, n);
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
// FP8 (only without SHARED): the suffix rows are E4M3 codes; a key is code * a.k_scale, a value code * a.v_scale.
template <int D, int GT, bool SHARED, bool PAGED, bool FP8 = false>
__global__ __launch_bounds__(256) void decode_kernel(DecodeArgs a) {
    constexpr int EPL = epl_of<D, GT, FP8>();   // columns per lane
    constexpr int LPR = D / EPL;                // lanes per row
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

    DecodeState<D, GT, EPL> st;
    {
        const float qs = FP8 ? a.scale * kLog2e * a.k_scale : a.scale * kLog2e;
        const int col = (lane % LPR) * EPL;
#pragma unroll
        for (int g = 0; g < GT; ++g) {
#pragma unroll
            for (int h8 = 0; h8 < EPL / 8; ++h8) {
                const uint4 qv = *reinterpret_cast<const uint4*>(a.Q + ((int64_t)bq * a.Hq + h0 + g) * D + col + 8 * h8);
                float* const q = &st.q[g][8 * h8];
                st.qp[g][4 * h8] = qv.x; st.qp[g][4 * h8 + 1] = qv.y; st.qp[g][4 * h8 + 2] = qv.z; st.qp[g][4 * h8 + 3] = qv.w;
                q[0] = bf16_lo(qv.x) * qs; q[1] = bf16_hi(qv.x) * qs;
                q[2] = bf16_lo(qv.y) * qs; q[3] = bf16_hi(qv.y) * qs;
                q[4] = bf16_lo(qv.z) * qs; q[5] = bf16_hi(qv.z) * qs;
                q[6] = bf16_lo(qv.w) * qs; q[7] = bf16_hi(qv.w) * qs;
            }
            st.m[g] = -INFINITY;
            st.l[g] = 0.f;
#pragma unroll
            for (int j = 0; j < EPL; ++j) st.acc[g][j] = 0.f;
        }
        st.qs = qs;
    }

    // walk the concatenated key list (shared blocks root first, then the suffix), clipped to this chunk
    const int64_t lo = (int64_t)c * a.chunk, hi = lo + a.chunk;
    int64_t pos = 0;
    for (int li = 0; SHARED && li < a.n_levels; ++li) {
        int begin, count;
        block_of(a.lv[li], b, a.B, begin, count);
        const int64_t s0 = max(lo, pos), s1 = min(hi, pos + count);
        if (s0 < s1) decode_span<D, GT, false, false, EPL>(st, a.lv[li].K, a.lv[li].V, begin + (s0 - pos), (int)(s1 - s0), a.Hkv, kvh, lane);
        pos += count;
    }
    if (a.lengths) {
        // the nq queries of a sequence are its last nq suffix tokens: query t does not see the later ones
        int count = min(a.lengths[b], a.max_len) - (a.nq - 1 - tq);
        if (count < 0) count = 0;
        const int64_t s0 = max(lo, pos), s1 = min(hi, pos + count);
        if (s0 < s1) {
            if constexpr (PAGED) decode_span_paged<D, GT, FP8, EPL>(st, a.Ks, a.Vs, a.pg, b, (int)s0, (int)(s1 - s0), a.Hkv, kvh, lane);
            else decode_span<D, GT, true, FP8, EPL>(st, a.Ks, a.Vs, a.offsets[b] + (s0 - pos), (int)(s1 - s0), a.Hkv, kvh, lane);
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
        float o[EPL];
#pragma unroll
        for (int j = 0; j < EPL; ++j) {
            o[j] = st.acc[g][j] * f;
#pragma unroll
            for (int off = LPR; off < 64; off <<= 1) o[j] += __shfl_xor(o[j], off);
        }
        if (lane < LPR) {
            const float inv = l > 0.f ? (FP8 ? a.v_scale / l : 1.0f / l) : 0.f;
            const int64_t idx = (int64_t)bq * a.Hq + h0 + g;
#pragma unroll
            for (int h8 = 0; h8 < EPL / 8; ++h8) {
                const int64_t e = (int64_t)c * a.out.part_stride_O + idx * D + lane * EPL + 8 * h8;
                const float* const oh = &o[8 * h8];
                if (a.out.bf16) {
                    uint4 v;
                    v.x = pack_bf16(oh[0] * inv, oh[1] * inv); v.y = pack_bf16(oh[2] * inv, oh[3] * inv);
                    v.z = pack_bf16(oh[4] * inv, oh[5] * inv); v.w = pack_bf16(oh[6] * inv, oh[7] * inv);
                    *reinterpret_cast<uint4*>(static_cast<uint16_t*>(a.out.O) + e) = v;
                } else {
                    float* op = static_cast<float*>(a.out.O) + e;
                    *reinterpret_cast<float4*>(op) = make_float4(oh[0] * inv, oh[1] * inv, oh[2] * inv, oh[3] * inv);
                    *reinterpret_cast<float4*>(op + 4) = make_float4(oh[4] * inv, oh[5] * inv, oh[6] * inv, oh[7] * inv);
                }
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
    if (a.fp8) {
        if (a.n_levels > 0) return hipErrorInvalidValue;   // 8-bit rows: suffix only
        if (a.pg.table) decode_kernel<D, GT, false, true, true><<<(unsigned)grid, 256, 0, s>>>(a);
        else decode_kernel<D, GT, false, false, true><<<(unsigned)grid, 256, 0, s>>>(a);
    } else if (a.pg.table) {
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
