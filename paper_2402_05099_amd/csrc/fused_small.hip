// The whole of Hydragen's attention (App. B's top-level routine: attention over every shared block, attention over each
// sequence's own suffix, and the merge of the parts by their log-sum-exp, Eq. 5) in ONE launch, for calls with so
// little work that three launches, a second stream and a pass over partial results in HBM cost more than the
// arithmetic.  No workspace, no partial result leaves the chip.
//
// A workgroup owns 32 consecutive rows of the query rows of one KV head (Sec. 3.2's inter-sequence batching: row
// r = sequence * nq * G + query * G + head-in-group).  Their keys are a list of segments: the block of every shared
// level that covers their sequences (all rows of the tile attend to it, or those of the covered sequences when a
// block boundary falls inside the tile), then the suffix of each of the tile's sequences (only that sequence's rows
// attend).  Softmax over the union of all segments is one online softmax: a row that does not attend to a segment has
// its scores masked.  The decomposition of Eq. 5 appears twice: the list is cut into four equal runs of 32-key
// stages, one per wavefront, each with its own running maximum, sum and accumulator; at the end the four partial
// results meet in LDS and are combined with the weights exp(LSE_i - max LSE) into the final (O, LSE).
//
// A wavefront streams its stages through a private ring of two 16 KiB slots (HBM -> LDS copies issued from inline
// asm, counted s_waitcnt, one stage ahead) and multiplies on v_mfma_f32_32x32x16_bf16 with the transposed products,
// XOR swizzles and lazy rescaling of the other kernels (prefix_wide.hip, decode_mfma.hip).
#include "hg_internal.h"
#include "prefix_common.h"

#pragma clang diagnostic ignored "-Winline-asm"

namespace hg {

namespace {

constexpr int KT = 32;                  // keys per stage
constexpr int NWS = 4;                  // wavefronts per workgroup
constexpr int NSL = 2;                  // ring slots per wavefront
constexpr float TAU = 8.0f;             // lazy-rescale threshold, log2 units

typedef unsigned uintx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ unsigned pack_pair(float lo, float hi) {
    floatx2 f = {lo, hi};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(f, bf16x2));
}

template <int N>
__device__ __forceinline__ void wait_vm() {
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

extern __shared__ __attribute__((aligned(1024))) unsigned char fs_smem[];

typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;
typedef const __attribute__((address_space(4))) SmallArgs* kargs_ptr;

// One segment of a tile's key list (uniform over the workgroup).
struct Seg {
    const unsigned char* K;   // the segment's tensor at this KV head (bytes)
    const unsigned char* V;
    int ks, ke;               // key rows [ks, ke) of that tensor
    int rlo, rhi;             // rows [rlo, rhi) of the tile attend to it
    int vis_base;             // suffix: query t of the sequence sees rows below vis_base + t; shared block: INT_MAX / 2
    int nst;                  // stages of 32 keys
};

// Walks the segments of a tile in a fixed order: levels in order, within a level the blocks that cover sequences
// b0 .. b1 in order, then the suffixes of b0 .. b1.  Segments without keys or without rows are skipped.
struct SegIter {
    int level, block, seq;    // position: level < n_levels: block index in that level (-1: not looked up yet); then the suffix of seq
    __device__ void reset(int b0) { level = 0; block = -1; seq = b0; }
};

}  // namespace

template <int D>
__global__ __launch_bounds__(64 * NWS) void fused_small_kernel(SmallArgs a) {
    constexpr int KS = D / 16, DB = D / 32, CPR = D / 8, RPI = 64 / CPR, CPS = KT / RPI, ROWB = D * 2, STB = KT * ROWB;
    constexpr int KVOPS = 2 * CPS;                  // copy instructions per stage
    constexpr int WAVE_LDS = 2 * NSL * STB;         // ring of one wavefront: K slots, then V slots
    static_assert(KVOPS <= 63, "the copies of a stage must fit the vmcnt counter");
    unsigned char* const smem_all = fs_smem;
    const int tid = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l = tid & 63, lq = l & 31, hl = l >> 5;
    unsigned char* const smem = smem_all + w * WAVE_LDS;
    const kargs_ptr k = (kargs_ptr)__builtin_amdgcn_kernarg_segment_ptr();

    const int tile = blockIdx.x % a.tiles, kvh = blockIdx.x / a.tiles;
    const int rps = a.nq * a.G;                     // query rows of one sequence for this KV head
    const int R = a.B * rps;
    const int r0 = tile * 32;
    const int b0 = r0 / rps, b1 = min((r0 + 31) / rps, a.B - 1);
    const int r = r0 + lq;                          // this lane's row
    const bool rv = r < R;
    const int rr = rv ? r : r0;
    const int b_lane = rr / rps, t_lane = (rr % rps) / a.G, g_lane = rr % a.G;
    const int64_t qidx = ((int64_t)b_lane * a.nq + t_lane) * a.Hq + kvh * a.G + g_lane;   // (b*nq + t)*Hq + h

    // ---- Q operand (registers) and the tile's suffix lengths / offsets (lane i: sequence b0 + i), loaded before any copy ----
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
    int len_v = 0, off_v = 0;
    if (a.lengths != nullptr && b0 + l <= b1) {
        len_v = max(min(a.lengths[b0 + l], a.max_len), 0);
        off_v = a.offsets[b0 + l];
    }
    // the loads above are the only ones the compiler sees; it waits for them here, before the first copy is issued
    asm volatile("" : "+v"(len_v), "+v"(off_v));
#pragma unroll
    for (int s = 0; s < KS; ++s) asm volatile("" : "+v"(qf[s]));

    // ---- segment enumeration ---------------------------------------------------------------------------------------------------
    const unsigned rstride_b = (unsigned)a.Hkv * D * 2u;
    auto next_seg = [&](SegIter& it, Seg& s) -> bool {
        for (;;) {
            if (it.level < a.n_levels) {
                const int L = it.level;
                const const_i32_ptr seq_off = (const_i32_ptr)(uintptr_t)k->lv[L].seq_off;
                const const_i32_ptr kv_off = (const_i32_ptr)(uintptr_t)k->lv[L].kv_off;
                int sa = 0, sb = a.B, kv0 = 0, kv1 = k->lv[L].max_rows;
                if (seq_off != nullptr) {
                    const int nb = k->lv[L].n_blocks;
                    if (it.block < 0) {
                        // first block whose sequences end after b0
                        int lo = 0, hi = nb;
                        while (lo < hi) {
                            const int mid = (lo + hi) >> 1;
                            if (seq_off[mid + 1] <= b0) lo = mid + 1;
                            else hi = mid;
                        }
                        it.block = lo;
                    }
                    if (it.block >= nb || seq_off[it.block] > b1) {   // no further block of this level touches the tile
                        ++it.level;
                        it.block = -1;
                        continue;
                    }
                    sa = seq_off[it.block];
                    sb = min(seq_off[it.block + 1], sa + k->lv[L].max_seqs);
                    kv0 = kv_off[it.block];
                    kv1 = min(kv_off[it.block + 1], kv0 + k->lv[L].max_rows);
                    ++it.block;
                } else {
                    ++it.level;
                    it.block = -1;
                }
                s.K = reinterpret_cast<const unsigned char*>(k->lv[L].K + (int64_t)kvh * D);
                s.V = reinterpret_cast<const unsigned char*>(k->lv[L].V + (int64_t)kvh * D);
                s.ks = kv0;
                s.ke = kv1;
                s.rlo = max(max(sa, b0) * rps - r0, 0);
                s.rhi = min(min(sb, b1 + 1) * rps - r0, 32);
                s.vis_base = 0x3fffffff;
            } else {
                if (a.lengths == nullptr || it.seq > b1) return false;
                const int i = it.seq - b0;
                const int cnt = __builtin_amdgcn_readlane(len_v, i), off = __builtin_amdgcn_readlane(off_v, i);
                s.K = reinterpret_cast<const unsigned char*>(k->Ks + (int64_t)kvh * D);
                s.V = reinterpret_cast<const unsigned char*>(k->Vs + (int64_t)kvh * D);
                s.ks = off;
                s.ke = off + cnt;
                s.rlo = max(it.seq * rps - r0, 0);
                s.rhi = min((it.seq + 1) * rps - r0, 32);
                s.vis_base = off + cnt - (a.nq - 1);     // query t sees rows below off + cnt - (nq-1-t)
                ++it.seq;
            }
            s.nst = (s.ke > s.ks && s.rhi > s.rlo) ? (s.ke - s.ks + KT - 1) / KT : 0;
            if (s.nst > 0) return true;
        }
    };

    // total stages of the tile, and this wavefront's run [run_lo, run_hi) of them
    int total = 0;
    {
        SegIter it;
        it.reset(b0);
        Seg s;
        while (next_seg(it, s)) total += s.nst;
    }
    total = __builtin_amdgcn_readfirstlane(total);
    const int run_lo = (int)((long long)w * total / NWS), run_hi = (int)((long long)(w + 1) * total / NWS);

    // ---- HBM -> LDS copies (as in decode_mfma.hip) -----------------------------------------------------------------------------------
    // Stage t of a segment holds rows [k0c, k0c + 32), k0c = min(ks + 32 t, kwin), kwin = max(ke - 32, 0): a partial last
    // stage re-reads the 32 rows that end the range; row i of a stage is a key of it iff ks + 32 t <= k0c + i < ke.
    const int lrow = l / CPR, sch = l % CPR;
    const unsigned ldsb = (unsigned)(uintptr_t)HG_LDS(smem);
    auto kswz = [](int row) { return D == 128 ? row % 16 : (row >> 1) & 7; };
    auto vswz = [](int row) { return D == 128 ? 4 * (row % 4) : 4 * ((row >> 1) & 1); };
    auto scalar_ptr = [&](const unsigned char* vbase) -> const unsigned char* {
        const uint64_t pv = reinterpret_cast<uint64_t>(vbase);
        const uint32_t plo = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)pv);
        const uint32_t phi = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(pv >> 32));
        return reinterpret_cast<const unsigned char*>(((uint64_t)phi << 32) | (uint64_t)plo);
    };
    auto copy16 = [&](const unsigned char* sbase, unsigned voff, unsigned lds_dst) {
        asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase), "s"(lds_dst) : "memory", "m0");
    };

    // A cursor over this wavefront's run: the segment it is in and the next stage of that segment.  Two of them walk
    // the same run: the producer (copies) one stage ahead of the consumer (products).
    struct Cursor {
        SegIter it;
        Seg s;
        int base;     // stages of the tile before this segment
        int t;        // next stage of the segment
        int pos;      // its index in the tile's stage list
    };
    auto cursor_start = [&](Cursor& c) {        // on the stage run_lo (if the run is not empty)
        c.it.reset(b0);
        c.base = 0;
        c.pos = run_lo;
        c.s.nst = 0;
        if (run_lo >= run_hi) return;
        while (next_seg(c.it, c.s)) {
            if (c.base + c.s.nst > run_lo) break;
            c.base += c.s.nst;
        }
        c.t = run_lo - c.base;
    };
    auto cursor_step = [&](Cursor& c) {         // one stage further
        ++c.pos;
        if (++c.t == c.s.nst && c.pos < run_hi) {
            c.base += c.s.nst;
            c.t = 0;
            next_seg(c.it, c.s);                // exists: the run ends within the tile's list
        }
    };

    Cursor pc, cc;
    cursor_start(pc);
    cursor_start(cc);
    int n_issued = 0;
    auto produce_one = [&]() {
        if (pc.pos >= run_hi) return;
        const int kwin = max(pc.s.ke - KT, 0);
        const int k0c = min(pc.s.ks + pc.t * KT, kwin);
        const int rowclamp = min(pc.s.ke - 1 - kwin, KT - 1);     // < 31 only when the range ends before row 32 of the tensor
        const unsigned char* const kg = scalar_ptr(pc.s.K + (int64_t)k0c * rstride_b);
        const unsigned char* const vg = scalar_ptr(pc.s.V + (int64_t)k0c * rstride_b);
        const unsigned dst = (unsigned)__builtin_amdgcn_readfirstlane(ldsb + (unsigned)(n_issued % NSL) * STB);
#pragma unroll
        for (int i = 0; i < CPS; ++i) {
            const int srow = i * RPI + lrow;
            const unsigned ro = (unsigned)min(srow, rowclamp) * rstride_b;
            copy16(kg, ro + (unsigned)((sch ^ kswz(srow)) * 16), dst + i * 1024);
        }
#pragma unroll
        for (int i = 0; i < CPS; ++i) {
            const int srow = i * RPI + lrow;
            const unsigned ro = (unsigned)min(srow, rowclamp) * rstride_b;
            copy16(vg, ro + (unsigned)((sch ^ vswz(srow)) * 16), dst + NSL * STB + i * 1024);
        }
        ++n_issued;
        cursor_step(pc);
    };

    // ---- LDS fragment addresses (relative to the slot), as in prefix_wide.hip ------------------------------------------
    unsigned kaddr[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) kaddr[s] = (unsigned)(lq * ROWB + (((2 * s + hl) ^ kswz(lq)) * 16));
    unsigned vaddr[DB];
    {
        const int i16 = l & 15, g1 = (l >> 4) & 1;
        const int keyq = 4 * hl + (i16 >> 2);
        const int fv = vswz(keyq);
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const int chunk = 4 * db + 2 * g1 + ((i16 & 3) >> 1);
            vaddr[db] = (unsigned)(keyq * ROWB + ((chunk ^ fv) * 16) + (i16 & 1) * 8);   // relative to the V stage
        }
    }

    // ---- this wavefront's share of the softmax ------------------------------------------------------------------------------
    const float c2 = a.scale * kLog2e;
    const float tau_raw = TAU / c2;
    floatx16 Oacc[DB];
#pragma unroll
    for (int i = 0; i < DB; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) Oacc[i][j] = 0.f;
    float m_used = -INFINITY;   // raw-score maximum the exponentials are taken against (-inf: no key seen yet)
    float mc = 0.f;             // m_used * c2, 0 while no key has been seen
    float lsum = 0.f;           // this lane's share of the row sum (unrounded exponentials)

    produce_one();
    int n_done = 0;
    while (cc.pos < run_hi) {
        n_done = __builtin_amdgcn_readfirstlane(n_done);
        produce_one();                               // the stage after this one, into the other slot
        if (n_issued > n_done + 1) wait_vm<KVOPS>();      // the stage after this one may stay in flight
        else wait_vm<0>();
        asm volatile("" ::: "memory");
        const unsigned char* const sb = smem + (n_done % NSL) * STB;
        unsigned char* const vstage = smem + (n_done % NSL) * STB + NSL * STB;
        ++n_done;
        const Seg& s = cc.s;
        const int kwin = max(s.ke - KT, 0);
        const int key0 = s.ks + cc.t * KT;
        const int k0c = min(key0, kwin);
        if (k0c != key0 || s.ke - kwin < KT) {
            // stage rows that are not keys of this stage (re-read from below the range, or past a range that ends before
            // row 32 of the tensor) may hold anything: their probabilities are zero, but 0 * NaN is NaN in the second
            // product, so their V rows are cleared in LDS
            const int nlo = key0 - k0c, nhi = s.ke - k0c;
#pragma unroll
            for (int i = 0; i < CPS; ++i) {
                const int row = i * RPI + lrow;
                if (row < nlo || row >= nhi) *reinterpret_cast<uintx4*>(vstage + row * ROWB + sch * 16) = uintx4{0u, 0u, 0u, 0u};
            }
        }
        // S^T = K Q^T
        floatx16 S;
#pragma unroll
        for (int i = 0; i < 16; ++i) S[i] = 0.f;
#pragma unroll
        for (int q = 0; q < KS; ++q) {
            const uintx4 kv = *reinterpret_cast<const uintx4*>(sb + kaddr[q]);
            S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kv), qf[q], S, 0, 0, 0);
        }
        // masks: keys outside the stage's range, keys this lane's query does not see yet, rows that do not attend
        {
            const bool attends = lq >= s.rlo && lq < s.rhi;
            const int vis_end = min(s.ke, s.vis_base + t_lane);
            const int lo_i = key0 - k0c - 4 * hl, hi_i = (attends ? vis_end : k0c) - k0c - 4 * hl;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int ri = 8 * (i >> 2) + (i & 3);   // stage row of element i is ri + 4*hl
                if (ri < lo_i || ri >= hi_i) S[i] = -INFINITY;
            }
        }
        float tmax = fmaxf(S[0], S[1]);
#pragma unroll
        for (int i = 2; i < 16; i += 2) tmax = fmaxf(fmaxf(tmax, S[i]), S[i + 1]);
        tmax = half_max(tmax);
        if (__any(tmax > m_used + tau_raw)) {
            const float m_new = fmaxf(m_used, tmax);
            // equal maxima (also -inf and -inf: a row that has seen no key yet) keep the accumulators
            const float alpha = (m_new == m_used) ? 1.0f : __builtin_amdgcn_exp2f((m_used - m_new) * c2);
            m_used = m_new;
            mc = (m_new == -INFINITY) ? 0.f : m_new * c2;
            lsum *= alpha;
#pragma unroll
            for (int i = 0; i < DB; ++i)
#pragma unroll
                for (int j = 0; j < 16; ++j) Oacc[i][j] *= alpha;
        }
        uintx4 pb[2];
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
            float p[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                p[i] = __builtin_amdgcn_exp2f(fmaf(S[8 * tt + i], c2, -mc));
                lsum += p[i];
            }
            pb[tt] = uintx4{pack_pair(p[0], p[1]), pack_pair(p[2], p[3]), pack_pair(p[4], p[5]), pack_pair(p[6], p[7])};
        }
        // O^T += V^T P^T
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                const unsigned char* vp = vstage + vaddr[db] + tt * 16 * ROWB;
                const shortx4 vlo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) shortx4*)HG_LDS(vp));
                const shortx4 vhi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) shortx4*)HG_LDS(vp + 8 * ROWB));
                const shortx8 vv = __builtin_shufflevector(vlo, vhi, 0, 1, 2, 3, 4, 5, 6, 7);
                Oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vv), __builtin_bit_cast(bf16x8, pb[tt]), Oacc[db], 0, 0, 0);
            }
        }
        // the accumulators depend on every fragment read of this stage: once they are pinned here the reads have
        // completed, and the next produce_one() may overwrite the slot
#pragma unroll
        for (int db = 0; db < DB; ++db) asm volatile("" : "+v"(Oacc[db]));
        asm volatile("" ::: "memory");
        cursor_step(cc);
    }
    wait_vm<0>();

    // ---- the four partial results meet in LDS (Eq. 5) -------------------------------------------------------------------------------
    // Layout (the rings are free now): O of wavefront v at v * 32 * D * 4, row-major [32][D] fp32 with the 16-byte chunk c of
    // row r at chunk c ^ (r % (D / 4)); then the maxima and sums [NWS][32].
    constexpr int OW = 32 * D * 4;
    constexpr int CH = D / 4;                       // 16-byte chunks per row
    float* const Mw = reinterpret_cast<float*>(smem_all + NWS * OW);
    float* const Lw = Mw + NWS * 32;
    const float ltot = half_sum(lsum);
    __syncthreads();
    {
        unsigned char* const ow = smem_all + w * OW;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int chunk = 8 * db + 2 * q4 + hl;
                *reinterpret_cast<float4*>(ow + lq * (D * 4) + ((chunk ^ (lq & (CH - 1))) * 16)) =
                    make_float4(Oacc[db][4 * q4], Oacc[db][4 * q4 + 1], Oacc[db][4 * q4 + 2], Oacc[db][4 * q4 + 3]);
            }
        if (hl == 0) {
            Mw[w * 32 + lq] = m_used;
            Lw[w * 32 + lq] = ltot;
        }
    }
    __syncthreads();
    {
        // wavefront w finishes rows 8w .. 8w+7: lane -> row 8w + l/8, columns (l%8) * D/8 .. + D/8 - 1
        constexpr int CPL = CH / 8;                  // 16-byte chunks per lane (D = 128: 4, D = 64: 2)
        const int row = 8 * w + (l >> 3), c0 = (l & 7) * CPL;
        float mv[NWS], M = -INFINITY;
#pragma unroll
        for (int v = 0; v < NWS; ++v) {
            mv[v] = Mw[v * 32 + row];
            M = fmaxf(M, mv[v]);
        }
        float f[NWS], Lsum = 0.f;
#pragma unroll
        for (int v = 0; v < NWS; ++v) {
            f[v] = (mv[v] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f((mv[v] - M) * c2);
            Lsum += f[v] * Lw[v * 32 + row];
        }
        const float inv = Lsum > 0.f ? 1.0f / Lsum : 0.f;     // a row without any key: O = 0, LSE = -inf
        const int rg = r0 + row;                                // the row this lane finishes
        const bool ok = rg < R;
        const int rrg = ok ? rg : r0;
        const int64_t oidx = ((int64_t)(rrg / rps) * a.nq + (rrg % rps) / a.G) * a.Hq + kvh * a.G + rrg % a.G;
#pragma unroll
        for (int c = 0; c < CPL; ++c) {
            float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int v = 0; v < NWS; ++v) {
                const float4 o = *reinterpret_cast<const float4*>(smem_all + v * OW + row * (D * 4) + (((c0 + c) ^ (row & (CH - 1))) * 16));
                acc.x += f[v] * o.x; acc.y += f[v] * o.y; acc.z += f[v] * o.z; acc.w += f[v] * o.w;
            }
            acc.x *= inv; acc.y *= inv; acc.z *= inv; acc.w *= inv;
            if (ok) {
                const int d = 4 * (c0 + c);
                if (a.bf16) *reinterpret_cast<uint2*>(static_cast<uint16_t*>(a.O) + oidx * D + d) = make_uint2(pack_bf16(acc.x, acc.y), pack_bf16(acc.z, acc.w));
                else *reinterpret_cast<float4*>(static_cast<float*>(a.O) + oidx * D + d) = acc;
            }
        }
        if (ok && (l & 7) == 0 && a.LSE != nullptr) a.LSE[oidx] = Lsum > 0.f ? M * a.scale + __logf(Lsum) : -INFINITY;
    }
}

hipError_t launch_fused_small(const SmallArgs& a, int D, hipStream_t s) {
    if (a.tiles < 1 || a.Hkv < 1 || (D != 64 && D != 128)) return hipErrorInvalidValue;
    const long long grid = (long long)a.tiles * a.Hkv;
    if (grid >= (1LL << 31)) return hipErrorInvalidValue;
    static bool attr_set[64][2] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const int lds = D == 128 ? NWS * 2 * NSL * KT * 256 : NWS * 2 * NSL * KT * 128;   // the rings; the merge area fits inside
    const void* fn = D == 128 ? reinterpret_cast<const void*>(&fused_small_kernel<128>) : reinterpret_cast<const void*>(&fused_small_kernel<64>);
    if (dev >= 0 && dev < 64 && !attr_set[dev][D == 128]) {
        e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        attr_set[dev][D == 128] = true;
    }
    if (D == 128) fused_small_kernel<128><<<(unsigned)grid, 64 * NWS, lds, s>>>(a);
    else fused_small_kernel<64><<<(unsigned)grid, 64 * NWS, lds, s>>>(a);
    return hipGetLastError();
}

}  // namespace hg
