// Inter-sequence batched attention over one shared KV block (Sec. 3.2 of the paper): the B*G query rows
// that use a KV head are stacked into one matrix and multiplied against that head's keys/values on the
// matrix cores, with an online softmax in registers, returning (O, LSE) (Eq. 1, Eq. 4).
//
// gfx950 design.  One workgroup = 4 wavefronts = 128 query rows (32 per wavefront) of one KV head and one
// key-range split.  Keys stream through LDS in tiles of 64.  Everything is computed transposed so that a
// lane owns ONE query column:
//     S^T[key, q] = K_tile * Q^T        v_mfma_f32_32x32x16_bf16, A = K rows from LDS, B = Q (registers)
//     O^T[d, q]  += V^T_tile * P^T      A = V^T from LDS, B = P^T = the S^T accumulators, exponentiated
// In the 32x32 accumulator layout lane l holds column l%32 and rows 8*(r/4) + 4*(l/32) + r%4 (r = 0..15),
// so softmax statistics are per-lane scalars (one exchange with lane l^32 per tile), and the accumulators
// of S^T are already in B-operand position for the second product once the key order inside each group of
// 16 keys is relabelled (key 8a+4hl+b -> slot 8hl+4a+b); V^T is written to LDS in that relabelled order.
// The softmax uses exp2 with scale*log2(e) folded into one FMA, and rescales O only when a row maximum
// grows by more than 2^8 (the stale maximum cancels exactly in O = acc / l and LSE = m + log l).
#include "hg_internal.h"

namespace hg {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ float other_half(float x) {
    // value of the lane 32 positions away (v_permlane32_swap exchanges the upper half of the first operand
    // with the lower half of the second)
    const unsigned u = __builtin_bit_cast(unsigned, x);
    auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __builtin_bit_cast(float, (threadIdx.x & 32) ? r[0] : r[1]);
}

template <int D>
__global__ __launch_bounds__(256, 2) void prefix_kernel(PrefixArgs a) {
    constexpr int KT = kPrefixKeys;        // 64 keys per tile
    constexpr int KS = D / 16;             // MFMA k-steps of the first product
    constexpr int DB = D / 32;             // 32-row blocks of O^T
    constexpr int CPR = D / 8;             // 16-byte chunks per K row
    constexpr int KCH = KT * CPR / 256;    // K chunks per thread per tile
    constexpr int NK = D / 8;              // keys per thread when loading V (each thread owns 2 columns)
    constexpr int KBYTES = KT * D * 2;
    constexpr int VBYTES = D * KT * 2;
    constexpr float TAU = 8.0f;            // lazy-rescale threshold, log2 units

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    // [K buf0][K buf1][V^T buf0][V^T buf1]

    // ---- which tile -------------------------------------------------------------------------------
    const int pid = blockIdx.x;
    const int slot = pid >> 3;
    const int L = (pid & 7) * a.per_xcd + slot;  // consecutive logical tiles stay on one XCD (ids round-robin over 8 XCDs)
    if (L >= a.total_tiles) return;
    int t = L;
    const int mt = t % a.mtiles; t /= a.mtiles;
    const int kvh = t % a.Hkv; t /= a.Hkv;
    const int sp = t % a.nsplit;
    const int g = t / a.nsplit;

    int seq0 = 0, seq1 = a.B, kv0 = 0, kv1 = a.lv.max_rows;
    if (a.lv.seq_off) {
        seq0 = a.lv.seq_off[g];
        seq1 = min(a.lv.seq_off[g + 1], seq0 + a.lv.max_seqs);
        kv0 = a.lv.kv_off[g];
        kv1 = min(a.lv.kv_off[g + 1], kv0 + a.lv.max_rows);
    }
    const int nrows = (seq1 - seq0) * a.G;
    const int row0 = mt * kPrefixRows;
    if (row0 >= nrows) return;
    const int ks = kv0 + sp * a.chunk;
    const int ke = min(ks + a.chunk, kv1);

    const int tid = threadIdx.x;
    const int w = tid >> 6, l = tid & 63, lq = l & 31, hl = l >> 5;
    const int r = row0 + w * 32 + lq;     // this lane's query row inside the block
    const bool rv = r < nrows;
    const int rr = rv ? r : 0;
    const int64_t qidx = (int64_t)(seq0 + rr / a.G) * a.Hq + kvh * a.G + rr % a.G;  // b*Hq + h

    float* const Of = static_cast<float*>(a.out.O) + sp * a.out.part_stride_O + qidx * D;
    uint16_t* const Ob = static_cast<uint16_t*>(a.out.O) + sp * a.out.part_stride_O + qidx * D;
    float* const Lp = a.out.LSE + sp * a.out.part_stride_L + qidx;

    if (ks >= ke) {  // empty key range: O = 0, LSE = -inf
        if (rv) {
#pragma unroll
            for (int i = 0; i < D / 8; ++i) {
                const int d = 8 * i + 4 * hl;
                if (a.out.bf16) *reinterpret_cast<uint2*>(Ob + d) = make_uint2(0u, 0u);
                else *reinterpret_cast<float4*>(Of + d) = make_float4(0.f, 0.f, 0.f, 0.f);
            }
            if (hl == 0) *Lp = -INFINITY;
        }
        return;
    }

    // ---- Q operand (registers, whole kernel) ---------------------------------------------------------
    bf16x8 qf[KS];
    {
        const uint16_t* qp = a.Q + qidx * D;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            uint4 v = make_uint4(0, 0, 0, 0);
            if (rv) v = *reinterpret_cast<const uint4*>(qp + 8 * (2 * s + hl));
            qf[s] = __builtin_bit_cast(bf16x8, v);
        }
    }

    // ---- global -> register -> LDS staging ------------------------------------------------------------
    const int64_t rstride = (int64_t)a.Hkv * D;
    const uint16_t* const Kg = a.lv.K + (int64_t)kvh * D;
    const uint16_t* const Vg = a.lv.V + (int64_t)kvh * D;
    const int vdp = tid % (D / 2);   // V column pair owned when staging V
    const int vkg = tid / (D / 2);   // V key group (NK keys each)

    uint4 kreg[KCH];
    uint32_t vreg[NK];

    auto load_tile = [&](int key0) {
        if (key0 + KT <= ke) {  // whole tile in range (workgroup-uniform): unguarded loads
#pragma unroll
            for (int i = 0; i < KCH; ++i) {
                const int id = tid + 256 * i;
                kreg[i] = *reinterpret_cast<const uint4*>(Kg + (key0 + id / CPR) * rstride + 8 * (id % CPR));
            }
#pragma unroll
            for (int i = 0; i < NK; ++i)
                vreg[i] = *reinterpret_cast<const uint32_t*>(Vg + (key0 + vkg * NK + i) * rstride + 2 * vdp);
        } else {                // ragged tail: rows past the range read row ke-1 and are zeroed
#pragma unroll
            for (int i = 0; i < KCH; ++i) {
                const int id = tid + 256 * i;
                const int key = key0 + id / CPR;
                const uint4 v = *reinterpret_cast<const uint4*>(Kg + min(key, ke - 1) * rstride + 8 * (id % CPR));
                kreg[i] = key < ke ? v : make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for (int i = 0; i < NK; ++i) {
                const int key = key0 + vkg * NK + i;
                const uint32_t v = *reinterpret_cast<const uint32_t*>(Vg + min(key, ke - 1) * rstride + 2 * vdp);
                vreg[i] = key < ke ? v : 0u;
            }
        }
    };
    auto store_tile = [&](int buf) {
        unsigned char* kb = smem + buf * KBYTES;
        unsigned char* vb = smem + 2 * KBYTES + buf * VBYTES;
#pragma unroll
        for (int i = 0; i < KCH; ++i) {
            const int id = tid + 256 * i;
            const int row = id / CPR, c = id % CPR;
            *reinterpret_cast<uint4*>(kb + row * (D * 2) + ((c ^ (row & (CPR - 1))) * 16)) = kreg[i];
        }
        // V^T: row d holds the tile's 64 keys; inside each group of 16 keys, key 8a+4h+b sits at slot 8h+4a+b
#pragma unroll
        for (int qd = 0; qd < NK / 4; ++qd) {
            const int kq = vkg * NK + 4 * qd;           // first of 4 consecutive keys (tile relative)
            const int t16 = kq >> 4, aa = (kq >> 3) & 1, hh = (kq >> 2) & 1;
            const int cv = 2 * t16 + hh;                // 16-byte chunk inside the 128-byte row
            const uint32_t w0 = vreg[4 * qd], w1 = vreg[4 * qd + 1], w2 = vreg[4 * qd + 2], w3 = vreg[4 * qd + 3];
            uint2 lo, hi;
            lo.x = __builtin_amdgcn_perm(w1, w0, 0x05040100u);
            lo.y = __builtin_amdgcn_perm(w3, w2, 0x05040100u);
            hi.x = __builtin_amdgcn_perm(w1, w0, 0x07060302u);
            hi.y = __builtin_amdgcn_perm(w3, w2, 0x07060302u);
            const int d0 = 2 * vdp, d1 = d0 + 1;
            *reinterpret_cast<uint2*>(vb + d0 * 128 + ((cv ^ ((d0 >> 1) & 7)) * 16) + 8 * aa) = lo;
            *reinterpret_cast<uint2*>(vb + d1 * 128 + ((cv ^ ((d1 >> 1) & 7)) * 16) + 8 * aa) = hi;
        }
    };

    // ---- online softmax state ----------------------------------------------------------------------------
    floatx16 Oacc[DB];
#pragma unroll
    for (int i = 0; i < DB; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) Oacc[i][j] = 0.f;
    float m_used = -INFINITY;   // raw-score maximum the exponentials are taken against
    float lsum = 0.f;           // this lane's share of the row sum
    const float c2 = a.scale * kLog2e;
    const float tau_raw = TAU / c2;
    float mc = 0.f;             // m_used * c2 (finite stand-in while m_used = -inf is irrelevant: first tile always rescales)

    const int ntiles = (ke - ks + KT - 1) / KT;
    load_tile(ks);
    store_tile(0);
    __syncthreads();

    for (int j = 0; j < ntiles; ++j) {
        const int buf = j & 1;
        const bool more = j + 1 < ntiles;
        if (more) load_tile(ks + (j + 1) * KT);

        const unsigned char* kb = smem + buf * KBYTES;
        const unsigned char* vb = smem + 2 * KBYTES + buf * VBYTES;

        // S^T = K Q^T for the two 32-key halves of the tile
        floatx16 S[2];
#pragma unroll
        for (int sb = 0; sb < 2; ++sb) {
#pragma unroll
            for (int i = 0; i < 16; ++i) S[sb][i] = 0.f;
            const int key = 32 * sb + lq;
            const unsigned char* krow = kb + key * (D * 2);
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const uint4 kv = *reinterpret_cast<const uint4*>(krow + (((2 * s + hl) ^ (key & (CPR - 1))) * 16));
                S[sb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kv), qf[s], S[sb], 0, 0, 0);
            }
        }
        if (!more) {  // mask keys beyond the range in the last tile
            const int base = ks + j * KT + 4 * hl;
#pragma unroll
            for (int sb = 0; sb < 2; ++sb)
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    if (base + 32 * sb + 8 * (i >> 2) + (i & 3) >= ke) S[sb][i] = -INFINITY;
        }
        float tmax = S[0][0];
#pragma unroll
        for (int i = 1; i < 16; ++i) tmax = fmaxf(tmax, S[0][i]);
#pragma unroll
        for (int i = 0; i < 16; ++i) tmax = fmaxf(tmax, S[1][i]);
        tmax = fmaxf(tmax, other_half(tmax));

        if (__any(tmax > m_used + tau_raw)) {
            const float m_new = fmaxf(m_used, tmax);
            const float alpha = __builtin_amdgcn_exp2f((m_used - m_new) * c2);
            m_used = m_new;
            mc = m_new * c2;
            lsum *= alpha;
#pragma unroll
            for (int i = 0; i < DB; ++i)
#pragma unroll
                for (int k = 0; k < 16; ++k) Oacc[i][k] *= alpha;
        }

        // P^T = 2^(S*c2 - m*c2), packed to bf16 in B-operand order; O^T += V^T P^T
        bf16x8 pb[4];
#pragma unroll
        for (int sb = 0; sb < 2; ++sb) {
            floatx8 p0, p1;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                p0[i] = __builtin_amdgcn_exp2f(fmaf(S[sb][i], c2, -mc));
                p1[i] = __builtin_amdgcn_exp2f(fmaf(S[sb][8 + i], c2, -mc));
                lsum += p0[i] + p1[i];
            }
            pb[2 * sb] = __builtin_convertvector(p0, bf16x8);
            pb[2 * sb + 1] = __builtin_convertvector(p1, bf16x8);
        }
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                const int d = 32 * db + lq;
                const uint4 vv = *reinterpret_cast<const uint4*>(vb + d * 128 + (((2 * tt + hl) ^ ((d >> 1) & 7)) * 16));
                Oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vv), pb[tt], Oacc[db], 0, 0, 0);
            }
        }

        if (more) store_tile(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue ----------------------------------------------------------------------------------------
    const float ltot = lsum + other_half(lsum);
    if (rv) {
        const float inv = 1.0f / ltot;
#pragma unroll
        for (int db = 0; db < DB; ++db) {
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int d = 32 * db + 8 * q4 + 4 * hl;
                const float o0 = Oacc[db][4 * q4] * inv, o1 = Oacc[db][4 * q4 + 1] * inv;
                const float o2 = Oacc[db][4 * q4 + 2] * inv, o3 = Oacc[db][4 * q4 + 3] * inv;
                if (a.out.bf16) *reinterpret_cast<uint2*>(Ob + d) = make_uint2(pack_bf16(o0, o1), pack_bf16(o2, o3));
                else *reinterpret_cast<float4*>(Of + d) = make_float4(o0, o1, o2, o3);
            }
        }
        if (hl == 0) *Lp = m_used * a.scale + __logf(ltot);
    }
}

hipError_t launch_prefix(const PrefixArgs& a, int D, hipStream_t s) {
    if (a.total_tiles == 0) return hipSuccess;
    const unsigned grid = (unsigned)a.per_xcd * 8u;
    const size_t shmem = (size_t)2 * (kPrefixKeys * D * 2) * 2;
    hipError_t e;
    if (D == 128) {
        static bool attr128 = false;
        if (!attr128) {
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(prefix_kernel<128>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
            if (e != hipSuccess) return e;
            attr128 = true;
        }
        prefix_kernel<128><<<grid, 256, shmem, s>>>(a);
    } else {
        prefix_kernel<64><<<grid, 256, shmem, s>>>(a);
    }
    return hipGetLastError();
}

}  // namespace hg
