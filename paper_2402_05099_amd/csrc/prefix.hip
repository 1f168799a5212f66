// Inter-sequence batched attention over one shared KV block (Sec. 3.2 of the paper): the B*G query rows
// that use a KV head are stacked into one matrix and multiplied against that head's keys/values on the
// matrix cores, with an online softmax in registers, returning (O, LSE) (Eq. 1, Eq. 4).
//
// gfx950 design.  One workgroup = 4 wavefronts = 128 query rows (32 per wavefront) of one KV head and one
// key-range split.  Keys stream through LDS in tiles of 64, double buffered; K and V tiles keep their HBM
// layout [key][d] and are copied HBM -> LDS directly (global_load_lds_dwordx4, no register staging), with
// the 16-byte chunks of each row XOR-swizzled so that both read patterns below are bank-conflict free.
// Everything is computed transposed so that a lane owns ONE query column:
//     S^T[key, q] = K_tile * Q^T        v_mfma_f32_32x32x16_bf16, A = K rows (ds_read_b128), B = Q (registers)
//     O^T[d, q]  += V^T_tile * P^T      A = V^T via the transposing LDS read ds_read_b64_tr_b16, B = P^T
// In the 32x32 accumulator layout lane l holds column l%32 and rows 8*(r/4) + 4*(l/32) + r%4 (r = 0..15),
// so softmax statistics are per-lane scalars (one exchange with lane l^32 per tile), and the accumulators
// of S^T, exponentiated and packed to bf16, are already the B operand of the second product: k-slot j of
// lane half hl in 16-key step t stands for key 16t + 8*(j/4) + 4*hl + j%4, and the V^T operand is read
// in that same key order.
// The softmax uses exp2 with scale*log2(e) folded into one FMA, and rescales O only when a row maximum
// grows by more than 2^8 (the stale maximum cancels exactly in O = acc / l and LSE = m + log l).
#include <type_traits>

#include "hg_internal.h"
#include "prefix_common.h"

namespace hg {

template <int D>
__global__ __launch_bounds__(256, 2) void prefix_kernel(PrefixArgs a) {
    constexpr int KT = kPrefixKeys;        // 64 keys per tile
    constexpr int KS = D / 16;             // MFMA k-steps of the first product
    constexpr int DB = D / 32;             // 32-row blocks of O^T
    constexpr int CPR = D / 8;             // 16-byte chunks per K/V row
    constexpr int RPI = 64 / CPR;          // rows one wavefront copies per direct-to-LDS instruction
    constexpr int ROUNDS = KT / (4 * RPI); // such instructions per wavefront per tile and tensor
    constexpr int ROWB = D * 2;            // bytes per row
    constexpr int TILEB = KT * ROWB;       // bytes per K (or V) tile
    constexpr int RPC = 256 / ROWB;        // rows per 256 bytes = one pass over the 64 LDS banks
    constexpr float TAU = 8.0f;            // lazy-rescale threshold, log2 units

    // Two K and two V tile buffers, each TILEB bytes, rows of ROWB bytes, chunk c of row r stored at chunk
    // c ^ ((r / RPC) % CPR) for K and c ^ (4 * ((r / RPC) % (CPR / 4))) for V.  The LDS has 64 four-byte banks;
    // ds_read_b128 serves a wavefront in four passes of 16 lanes (lanes {0-3,12-15,20-27}, {4-11,16-19,28-31} and
    // the same +32), ds_read_b64_tr_b16 in two passes of 32 lanes, and the swizzles make the 16 (32) addresses of
    // every pass cover all 64 banks once.  The buffers are four separate LDS objects on purpose: the compiler
    // then knows that a copy in flight into one buffer does not alias reads of the other, and does not make
    // those reads wait for the copy.
    __shared__ __attribute__((aligned(1024))) unsigned char sK0[TILEB];
    __shared__ __attribute__((aligned(1024))) unsigned char sK1[TILEB];
    __shared__ __attribute__((aligned(1024))) unsigned char sV0[TILEB];
    __shared__ __attribute__((aligned(1024))) unsigned char sV1[TILEB];

    mark_uncovered(a, D, a.nsplit, blockIdx.x, gridDim.x);

    // ---- which tile -------------------------------------------------------------------------------
    const int pid = blockIdx.x;
    const int L = (pid & 7) * a.per_xcd + (pid >> 3);  // consecutive logical tiles stay on one XCD (ids that are equal modulo 8 share an XCD)
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
    const int rps = a.nq * a.G;            // query rows of one sequence for this KV head: (query t, head g) at t*G + g
    const int nrows = (seq1 - seq0) * rps;
    const int row0 = mt * kPrefixRowsNarrow;
    if (row0 >= nrows) return;
    const int ks = kv0 + sp * a.chunk;
    const int ke = min(ks + a.chunk, kv1);

    const int tid = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l = tid & 63, lq = l & 31, hl = l >> 5;
    const int r = row0 + w * 32 + lq;     // this lane's query row inside the block
    const bool rv = r < nrows;
    const int rr = rv ? r : 0;
    const int64_t qidx = ((int64_t)(seq0 + rr / rps) * a.nq + (rr % rps) / a.G) * a.Hq + kvh * a.G + rr % a.G;  // (b*nq + t)*Hq + h

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

    // ---- HBM -> LDS copies ------------------------------------------------------------------------------
    // Instruction `i` of wavefront w copies tile rows i*4*RPI + w*RPI + (l / CPR) as one contiguous KiB of
    // LDS (lane l lands at +16*l); the swizzle is applied on the global side: lane l fetches the chunk
    // that belongs in its LDS slot.
    const int64_t rstride = (int64_t)a.Hkv * D;                      // elements between consecutive keys
    const unsigned rstride_b = (unsigned)rstride * 2u;
    const int srow = w * RPI + l / CPR;                              // row inside a group of 4*RPI rows
    const int sch = l % CPR;
    const unsigned swzK = (unsigned)((sch ^ ((srow / RPC) % CPR)) * 16);
    const unsigned swzV = (unsigned)((sch ^ (4 * ((srow / RPC) % (CPR / 4)))) * 16);
    const unsigned voffK = (unsigned)(l / CPR) * rstride_b + swzK;
    const unsigned voffV = (unsigned)(l / CPR) * rstride_b + swzV;
    const unsigned char* const Kg = reinterpret_cast<const unsigned char*>(a.lv.K + (int64_t)kvh * D);
    const unsigned char* const Vg = reinterpret_cast<const unsigned char*>(a.lv.V + (int64_t)kvh * D);

    auto copy_tile = [&](int key0, auto bufc) {
        constexpr int buf = decltype(bufc)::value;
        unsigned char* kdst = (buf ? sK1 : sK0) + w * (RPI * ROWB);
        unsigned char* vdst = (buf ? sV1 : sV0) + w * (RPI * ROWB);
        if (key0 + KT <= ke) {  // whole tile in range (workgroup-uniform)
#pragma unroll
            for (int i = 0; i < ROUNDS; ++i) {
                const int64_t rb = (int64_t)(key0 + i * 4 * RPI + w * RPI) * rstride_b;   // uniform
                __builtin_amdgcn_global_load_lds(HG_GLOBAL(Kg + rb + voffK), HG_LDS(kdst + i * (4 * RPI * ROWB)), 16, 0, 0);
                __builtin_amdgcn_global_load_lds(HG_GLOBAL(Vg + rb + voffV), HG_LDS(vdst + i * (4 * RPI * ROWB)), 16, 0, 0);
            }
        } else {                // ragged tail: rows past the range re-read row ke-1 (their scores are masked)
#pragma unroll
            for (int i = 0; i < ROUNDS; ++i) {
                const int key = min(key0 + i * 4 * RPI + srow, ke - 1);
                const int64_t ro = (int64_t)key * rstride_b;
                __builtin_amdgcn_global_load_lds(HG_GLOBAL(Kg + ro + swzK), HG_LDS(kdst + i * (4 * RPI * ROWB)), 16, 0, 0);
                __builtin_amdgcn_global_load_lds(HG_GLOBAL(Vg + ro + swzV), HG_LDS(vdst + i * (4 * RPI * ROWB)), 16, 0, 0);
            }
        }
    };

    // ---- per-lane LDS read addresses (buffer and sub-block offsets are immediates) -----------------------------
    // K operand for k-step s: row = 32*sb + lq, chunk 2s+hl
    unsigned kaddr[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) kaddr[s] = (unsigned)(lq * ROWB + (((2 * s + hl) ^ ((lq / RPC) % CPR)) * 16));
    // V^T operand for d-block db: within each 16-lane group, lane i addresses key (i/4) of the 4 keys being
    // transposed and columns dbase + 4*(i%4) .. +3; after the transposing read lane i holds column dbase + i
    // of those 4 keys.  Group (l/16)&1 selects the lower/upper 16 columns, hl the key quad.
    unsigned vaddr[DB];
    {
        const int i16 = l & 15, g1 = (l >> 4) & 1;
        const int keyq = 4 * hl + (i16 >> 2);                 // key inside an 8-key half step
        const int fv = 4 * ((keyq / RPC) % (CPR / 4));
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const int chunk = 4 * db + 2 * g1 + ((i16 & 3) >> 1);
            vaddr[db] = (unsigned)(keyq * ROWB + ((chunk ^ fv) * 16) + (i16 & 1) * 8);
        }
    }

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
    float mc = 0.f;             // m_used * c2

    const int ntiles = (ke - ks + KT - 1) / KT;

    auto compute_tile = [&](int j, auto bufc) {
        constexpr int buf = decltype(bufc)::value;
        const unsigned char* kb = buf ? sK1 : sK0;
        const unsigned char* vb = buf ? sV1 : sV0;

        // S^T = K Q^T for the two 32-key halves of the tile
        floatx16 S[2];
#pragma unroll
        for (int sb = 0; sb < 2; ++sb) {
#pragma unroll
            for (int i = 0; i < 16; ++i) S[sb][i] = 0.f;
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const uint4 kv = *reinterpret_cast<const uint4*>(kb + kaddr[s] + sb * 32 * ROWB);
                S[sb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kv), qf[s], S[sb], 0, 0, 0);
            }
        }
        if (j + 1 >= ntiles) {  // mask keys beyond the range in the last tile
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
        tmax = half_max(tmax);

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
                const unsigned char* vp = vb + vaddr[db] + tt * 16 * ROWB;
                const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) shortx4*)HG_LDS(vp));
                const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) shortx4*)HG_LDS(vp + 8 * ROWB));
                const shortx8 vv = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                Oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vv), pb[tt], Oacc[db], 0, 0, 0);
            }
        }
    };

    const std::integral_constant<int, 0> B0{};
    const std::integral_constant<int, 1> B1{};
    copy_tile(ks, B0);
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the direct-to-LDS copies have landed
    __syncthreads();

    for (int j = 0; j < ntiles; j += 2) {
        if (j + 1 < ntiles) copy_tile(ks + (j + 1) * KT, B1);
        compute_tile(j, B0);
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
        if (j + 1 < ntiles) {
            if (j + 2 < ntiles) copy_tile(ks + (j + 2) * KT, B0);
            compute_tile(j + 1, B1);
            __builtin_amdgcn_s_waitcnt(0x0F70);
            __syncthreads();
        }
    }

    // ---- epilogue ----------------------------------------------------------------------------------------
    const float ltot = half_sum(lsum);
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

hipError_t launch_prefix_narrow(const PrefixArgs& a, int D, hipStream_t s) {
    if (a.total_tiles == 0) return hipSuccess;
    const unsigned grid = (unsigned)a.per_xcd * 8u;
    if (D == 128) prefix_kernel<128><<<grid, 256, 0, s>>>(a);
    else prefix_kernel<64><<<grid, 256, 0, s>>>(a);
    return hipGetLastError();
}

}  // namespace hg
