// Inter-sequence batched attention over one shared KV block (Sec. 3.2 of the paper), wide variant for D = 128:
// 256 query rows per workgroup = 8 wavefronts x 32 rows, two wavefronts per SIMD, one workgroup per CU.
//
// Same mathematics and data layout as prefix.hip (transposed products S^T = K Q^T, O^T += V^T P^T with
// v_mfma_f32_32x32x16_bf16, direct HBM->LDS tile copies, swizzled K/V tiles, transposing LDS reads for V,
// lazy rescaling).  What differs, and why:
//   * a workgroup amortises each K/V tile copy over 256 query rows instead of 128: half the L2->LDS traffic
//     per flop;
//   * three K and three V tile buffers (96 KiB): a tile's copy is issued a whole tile before it is waited for,
//     so it has a full tile of arithmetic to arrive from L2 or HBM;
//   * the loop is software pipelined in the source over half tiles (32 keys): the score MFMAs of the next 32
//     keys are issued before the exponentials of the current 32, and the row maxima of the next are taken
//     after the value MFMAs of the current have been issued.  Every wavefront therefore always has matrix-core
//     and vector-ALU work to issue, and the two wavefronts that share a SIMD overlap even though the
//     workgroup barrier keeps them in the same phase.
#include <type_traits>

#include "hg_internal.h"
#include "prefix_common.h"

namespace hg {

namespace {
constexpr int D = 128;
constexpr int NW = 8;                        // wavefronts per workgroup
constexpr int KT = kPrefixKeys;              // 64 keys per tile
constexpr int KS = D / 16;                   // MFMA k-steps of the first product
constexpr int DB = D / 32;                   // 32-row blocks of O^T
constexpr int CPR = D / 8;                   // 16-byte chunks per K/V row
constexpr int RPI = 64 / CPR;                // rows one wavefront copies per direct-to-LDS instruction
constexpr int ROUNDS = KT / (NW * RPI);      // such instructions per wavefront per tile and tensor
constexpr int ROWB = D * 2;                  // bytes per row
constexpr int TILEB = KT * ROWB;             // bytes per K (or V) tile
constexpr float TAU = 8.0f;                  // lazy-rescale threshold, log2 units
static_assert(kPrefixRowsWide == 32 * NW, "one 32-row query block per wavefront");

template <int N> using IC = std::integral_constant<int, N>;
}  // namespace

__global__ __launch_bounds__(64 * NW, 2) void prefix_kernel_wide(PrefixArgs a) {
    // three K and three V tile buffers as separate LDS objects (so that the compiler can tell a copy in flight
    // into one of them from reads of another); rows of ROWB bytes, chunk c of row r at c ^ (r % 16) for K and
    // c ^ (4 * (r % 4)) for V (conflict free over the 64 banks for the 16-lane passes of ds_read_b128 and the
    // 32-lane passes of ds_read_b64_tr_b16)
    __shared__ __attribute__((aligned(1024))) unsigned char sK0[TILEB];
    __shared__ __attribute__((aligned(1024))) unsigned char sK1[TILEB];
    __shared__ __attribute__((aligned(1024))) unsigned char sK2[TILEB];
    __shared__ __attribute__((aligned(1024))) unsigned char sV0[TILEB];
    __shared__ __attribute__((aligned(1024))) unsigned char sV1[TILEB];
    __shared__ __attribute__((aligned(1024))) unsigned char sV2[TILEB];

    // ---- which tile -------------------------------------------------------------------------------
    const int pid = blockIdx.x;
    const int L = (pid & 7) * a.per_xcd + (pid >> 3);  // consecutive logical tiles stay on one XCD
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
    const int row0 = mt * kPrefixRowsWide;
    if (row0 >= nrows) return;
    const int ks = kv0 + sp * a.chunk;
    const int ke = min(ks + a.chunk, kv1);

    const int tid = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l = tid & 63, lq = l & 31, hl = l >> 5;
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

    // ---- HBM -> LDS copies ------------------------------------------------------------------------------
    // Instruction `i` of wavefront w copies tile rows i*NW*RPI + w*RPI + (l / CPR) as one contiguous KiB of LDS
    // (lane l lands at +16*l); the swizzle is applied on the global side: lane l fetches the chunk that belongs
    // in its LDS slot.
    const unsigned rstride_b = (unsigned)a.Hkv * D * 2u;
    const int srow = w * RPI + l / CPR;                // row inside a group of NW*RPI = 32 rows
    const int sch = l % CPR;
    const unsigned swzK = (unsigned)((sch ^ (srow % CPR)) * 16);
    const unsigned swzV = (unsigned)((sch ^ (4 * (srow % 4))) * 16);
    const unsigned voffK = (unsigned)(l / CPR) * rstride_b + swzK;
    const unsigned voffV = (unsigned)(l / CPR) * rstride_b + swzV;
    const unsigned char* const Kg = reinterpret_cast<const unsigned char*>(a.lv.K + (int64_t)kvh * D);
    const unsigned char* const Vg = reinterpret_cast<const unsigned char*>(a.lv.V + (int64_t)kvh * D);

    auto copy_rows = [&](const unsigned char* G, unsigned voff, unsigned swz, int tile, unsigned char* dst) {
        const int key0 = ks + tile * KT;
        unsigned char* d = dst + w * (RPI * ROWB);
        if (key0 + KT <= ke) {  // whole tile in range (workgroup-uniform)
#pragma unroll
            for (int i = 0; i < ROUNDS; ++i) {
                const int64_t rb = (int64_t)(key0 + i * NW * RPI + w * RPI) * rstride_b;   // uniform
                __builtin_amdgcn_global_load_lds(HG_GLOBAL(G + rb + voff), HG_LDS(d + i * (NW * RPI * ROWB)), 16, 0, 0);
            }
        } else {                // ragged tail: rows past the range re-read row ke-1 (their scores are masked)
#pragma unroll
            for (int i = 0; i < ROUNDS; ++i) {
                const int key = min(key0 + i * NW * RPI + srow, ke - 1);
                __builtin_amdgcn_global_load_lds(HG_GLOBAL(G + (int64_t)key * rstride_b + swz), HG_LDS(d + i * (NW * RPI * ROWB)), 16, 0, 0);
            }
        }
    };
    auto kbuf = [&](auto bc) -> unsigned char* {
        constexpr int b = decltype(bc)::value;
        return b == 0 ? sK0 : (b == 1 ? sK1 : sK2);
    };
    auto vbuf = [&](auto bc) -> unsigned char* {
        constexpr int b = decltype(bc)::value;
        return b == 0 ? sV0 : (b == 1 ? sV1 : sV2);
    };

    // ---- per-lane LDS read addresses (buffer and sub-block offsets are immediates; see prefix.hip) -------------
    unsigned kaddr[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) kaddr[s] = (unsigned)(lq * ROWB + (((2 * s + hl) ^ (lq % CPR)) * 16));
    unsigned vaddr[DB];
    {
        const int i16 = l & 15, g1 = (l >> 4) & 1;
        const int keyq = 4 * hl + (i16 >> 2);
        const int fv = 4 * (keyq % 4);
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const int chunk = 4 * db + 2 * g1 + ((i16 & 3) >> 1);
            vaddr[db] = (unsigned)(keyq * ROWB + ((chunk ^ fv) * 16) + (i16 & 1) * 8);
        }
    }

    // ---- state ---------------------------------------------------------------------------------------------
    floatx16 Oacc[DB];
#pragma unroll
    for (int i = 0; i < DB; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) Oacc[i][j] = 0.f;
    float m_used = -INFINITY;   // raw-score maximum the exponentials are taken against
    float mc = 0.f;             // m_used * c2
    float lsum = 0.f;           // this lane's share of the row sum
    const float c2 = a.scale * kLog2e;
    const float tau_raw = TAU / c2;
    const int ntiles = (ke - ks + KT - 1) / KT;
    const bool ragged = ((ke - ks) % KT) != 0;
    floatx16 S;                 // scores of the 32-key half tile whose exponentials come next

    // scores of 32 keys (half `sb` of the tile in K buffer `kb`)
    auto scores_half = [&](floatx16& T, const unsigned char* kb, auto sbc) {
        constexpr int sb = decltype(sbc)::value;
        floatx16 zero;
#pragma unroll
        for (int i = 0; i < 16; ++i) zero[i] = 0.f;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const uint4 kv = *reinterpret_cast<const uint4*>(kb + kaddr[s] + sb * 32 * ROWB);
            T = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kv), qf[s], s == 0 ? zero : T, 0, 0, 0);
        }
    };
    // mask the keys of half `sb` of tile `tile` that lie beyond the range
    auto mask_half = [&](floatx16& T, int tile, int sb) {
        asm volatile("" ::: "memory");   // keeps this rare block a real branch (no speculation into every tile)
        const int base = ks + tile * KT + 32 * sb + 4 * hl;
#pragma unroll
        for (int i = 0; i < 16; ++i)
            if (base + 8 * (i >> 2) + (i & 3) >= ke) T[i] = -INFINITY;
    };
    // row maximum of T; rescale the running state if it outgrew the maximum in use by more than 2^TAU
    auto update_max = [&](const floatx16& T) {
        float m = T[0];
#pragma unroll
        for (int i = 1; i < 16; ++i) m = fmaxf(m, T[i]);
        const float tmax = half_max(m);
        if (__builtin_expect(__any(tmax > m_used + tau_raw), 0)) {
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
    };
    // P^T = 2^(S*c2 - m*c2) of the current half tile, packed to bf16 in B-operand order
    auto exp_half = [&](bf16x8 (&pb)[2]) {
        floatx8 p0, p1;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            p0[i] = __builtin_amdgcn_exp2f(fmaf(S[i], c2, -mc));
            p1[i] = __builtin_amdgcn_exp2f(fmaf(S[8 + i], c2, -mc));
            lsum += p0[i] + p1[i];
        }
        pb[0] = __builtin_convertvector(p0, bf16x8);
        pb[1] = __builtin_convertvector(p1, bf16x8);
    };
    // O^T += V^T P^T for half `sb` of the tile in V buffer `vb`
    auto values_half = [&](const bf16x8 (&pb)[2], const unsigned char* vb, auto sbc) {
        constexpr int sb = decltype(sbc)::value;
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2) {
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                const unsigned char* vp = vb + vaddr[db] + (2 * sb + t2) * 16 * ROWB;
                const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) shortx4*)HG_LDS(vp));
                const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) shortx4*)HG_LDS(vp + 8 * ROWB));
                const shortx8 vv = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                Oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vv), pb[t2], Oacc[db], 0, 0, 0);
            }
        }
    };

    // Tile j (in buffers B = j%3) when a next tile exists.  Entering, S holds the scores of its first half.
    auto tile_step = [&](int j, auto bc) {
        constexpr int B = decltype(bc)::value;
        {   // first half: scores of the second half | exponentials and values of the first
            floatx16 Sn;
            bf16x8 pb[2];
            scores_half(Sn, kbuf(IC<B>{}), IC<1>{});
            exp_half(pb);
            __builtin_amdgcn_sched_barrier(0);   // keeps the value-fragment reads out of the block above (register pressure)
            values_half(pb, vbuf(IC<B>{}), IC<0>{});
            update_max(Sn);
            S = Sn;
        }
        // tile j+1 has landed (its copies were issued a whole tile ago and are the only ones outstanding), and
        // every wavefront is past tile j-1, whose buffers tile j+2 now overwrites
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
        if (j + 2 < ntiles) {
            copy_rows(Kg, voffK, swzK, j + 2, kbuf(IC<(B + 2) % 3>{}));
            copy_rows(Vg, voffV, swzV, j + 2, vbuf(IC<(B + 2) % 3>{}));
        }
        {   // second half: scores of the next tile's first half | exponentials and values of the second
            floatx16 Sn;
            bf16x8 pb[2];
            scores_half(Sn, kbuf(IC<(B + 1) % 3>{}), IC<0>{});
            exp_half(pb);
            __builtin_amdgcn_sched_barrier(0);   // keeps the value-fragment reads out of the block above (register pressure)
            values_half(pb, vbuf(IC<B>{}), IC<1>{});
            if (ragged && j + 2 == ntiles) mask_half(Sn, j + 1, 0);   // the next tile is the ragged last one
            update_max(Sn);
            S = Sn;
        }
    };
    // The last tile (only it can be ragged).  Entering, S holds the scores of its first half.
    auto tile_last = [&](int j, auto bc) {
        constexpr int B = decltype(bc)::value;
        {
            floatx16 Sn;
            bf16x8 pb[2];
            scores_half(Sn, kbuf(IC<B>{}), IC<1>{});
            exp_half(pb);
            __builtin_amdgcn_sched_barrier(0);   // keeps the value-fragment reads out of the block above (register pressure)
            values_half(pb, vbuf(IC<B>{}), IC<0>{});
            if (ragged) mask_half(Sn, j, 1);
            update_max(Sn);
            S = Sn;
        }
        {
            bf16x8 pb[2];
            exp_half(pb);
            __builtin_amdgcn_sched_barrier(0);   // keeps the value-fragment reads out of the block above (register pressure)
            values_half(pb, vbuf(IC<B>{}), IC<1>{});
        }
    };

    // ---- prologue: tiles 0 and 1 in flight, scores of the first half tile -----------------------------------
    copy_rows(Kg, voffK, swzK, 0, sK0);
    copy_rows(Vg, voffV, swzV, 0, sV0);
    if (ntiles > 1) {
        copy_rows(Kg, voffK, swzK, 1, sK1);
        copy_rows(Vg, voffV, swzV, 1, sV1);
        __builtin_amdgcn_s_waitcnt(0x0F70 | (2 * ROUNDS));   // tile 0 landed, tile 1 may still be in flight
    } else {
        __builtin_amdgcn_s_waitcnt(0x0F70);
    }
    __syncthreads();
    scores_half(S, sK0, IC<0>{});
    if (ragged && ntiles == 1) mask_half(S, 0, 0);
    update_max(S);

    // main loop: three tiles per trip so that buffer numbers are compile-time constants; single exit
    int j = 0;
    for (; j + 3 < ntiles; j += 3) {
        tile_step(j, IC<0>{});
        tile_step(j + 1, IC<1>{});
        tile_step(j + 2, IC<2>{});
    }
    // one to three tiles remain; tile j sits in buffer 0 again
    const int rem = ntiles - j;
    if (rem >= 2) tile_step(j, IC<0>{});
    if (rem == 3) tile_step(j + 1, IC<1>{});
    if (rem == 1) tile_last(j, IC<0>{});
    else if (rem == 2) tile_last(j + 1, IC<1>{});
    else tile_last(j + 2, IC<2>{});

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

hipError_t launch_prefix_wide(const PrefixArgs& a, hipStream_t s) {
    if (a.total_tiles == 0) return hipSuccess;
    prefix_kernel_wide<<<(unsigned)a.per_xcd * 8u, 64 * NW, 0, s>>>(a);
    return hipGetLastError();
}

}  // namespace hg
