// Inter-sequence batched attention over one shared KV block (Sec. 3.2 of the paper), persistent 256-row kernel
// for D = 128: the B*G query rows that use a KV head are stacked into one matrix and multiplied against that
// head's keys/values on the matrix cores with an online softmax in registers, returning (O, LSE) per part
// (Eq. 1, Eq. 4); the parts are combined by the LSE merge (Eq. 5).
//
// Same mathematics and LDS layout as prefix.hip (transposed products S^T = K Q^T and O^T += V^T P^T with
// v_mfma_f32_32x32x16_bf16, K/V tiles in their HBM layout with XOR-swizzled 16-byte chunks, transposing LDS
// reads for V, lazy rescaling).  What differs, and why:
//   * One workgroup per CU, 8 wavefronts x 32 query rows = 256 rows: a workgroup amortises each K/V byte it
//     copies from L2 over 256 rows.  On this chip the copies cost power rather than time, and the kernel runs
//     against the power limit (a register-only MFMA loop on random data holds 1.85 GHz, not 2.4).
//   * Persistent: 256 workgroups.  Teams of T workgroups (one per 256-row tile of the query rows) walk the same
//     contiguous range of the flattened (column, stage) space, column = (block, KV head, row group) and stage =
//     32 keys, so a team shares its K/V reads in one XCD's L2 and every team gets the same number of stages: no
//     tail round.  A column that is cut by a range boundary yields several partial results (part index = piece
//     index inside the column); the workgroup that finishes a column marks the unused parts empty.
//   * Ring of 8 stages (K and V, 16 KiB each) in 128 KiB of dynamic LDS, filled by direct HBM->LDS copies that
//     are issued from inline asm and waited for with counted s_waitcnt vmcnt: four stages are in flight while
//     one is consumed.
//   * Software pipeline over stages, written out by gen_prefix_wide_step.py: in one step the scores of stage j+1
//     are produced while the exponentials of stage j are taken and its P*V product runs; fragments are loaded
//     from LDS four MFMAs before their use; the vector-ALU work is spread over the gaps between the MFMAs.
#include <type_traits>

#include "hg_internal.h"
#include "prefix_common.h"

// the copy helper names m0 as clobbered on purpose (it writes it)
#pragma clang diagnostic ignored "-Winline-asm"

namespace hg {

namespace {

constexpr int D = 128;
constexpr int KT = 32;                  // keys per stage
constexpr int NS = 8;                   // ring slots
constexpr int NW = 8;                   // wavefronts per workgroup
constexpr int KS = D / 16;              // MFMA k-steps of the score product
constexpr int DB = D / 32;              // 32-row blocks of O^T
constexpr int CPR = D / 8;              // 16-byte chunks per K/V row
constexpr int RPI = 64 / CPR;           // rows one wavefront copies per direct-to-LDS instruction
constexpr int ROWB = D * 2;             // bytes per row
constexpr int STB = KT * ROWB;          // bytes per stage and tensor
constexpr int VRING = NS * STB;         // byte offset of the V ring
constexpr int LDS_BYTES = 2 * NS * STB; // 128 KiB
constexpr int INFLIGHT = 4;             // stages that may still be in flight at a step's barrier
constexpr float TAU = 8.0f;             // lazy-rescale threshold, log2 units
static_assert(KT == NW * RPI, "one copy instruction per wavefront, stage and tensor");
static_assert(kPrefixRowsWide == 32 * NW, "one 32-row query block per wavefront");

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef unsigned uintx4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void mfma_first(floatx16& S, const uintx4& a, const bf16x8& b) {
    floatx16 z;
#pragma unroll
    for (int i = 0; i < 16; ++i) z[i] = 0.f;
    S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), b, z, 0, 0, 0);
}
__device__ __forceinline__ void mfma_acc(floatx16& S, const uintx4& a, const bf16x8& b) {
    S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), b, S, 0, 0, 0);
}
__device__ __forceinline__ void mfma_acc(floatx16& O, const shortx8& a, const uintx4& b) {
    O = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), O, 0, 0, 0);
}
// Two floats to a packed bf16 pair (RNE).
__device__ __forceinline__ unsigned pack_bf16_pair(float lo, float hi) {
    floatx2 f = {lo, hi};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(f, bf16x2));
}
// plain v_max3 / v_max: the operands are MFMA results or earlier maxima, nothing to quiet
__device__ __forceinline__ float max3f(float a, float b, float c) {
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
__device__ __forceinline__ float max2f(float a, float b) {
    float r;
    asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
// max of a value with the one held 32 lanes away.  v_permlane32_swap exchanges the upper 32 lanes of its first
// operand with the lower 32 lanes of its second: afterwards t holds the lower half's values in both halves and
// x the upper half's.
__device__ __forceinline__ float half_max_swap(float x) {
    float t;
    asm("v_mov_b32 %1, %0\n\ts_nop 1\n\tv_permlane32_swap_b32 %1, %0\n\ts_nop 1\n\tv_max_f32 %0, %0, %1" : "+v"(x), "=&v"(t));
    return x;
}

extern __shared__ __attribute__((aligned(1024))) unsigned char wide_smem[];

// One piece of work: 256-row tile mt of the query rows [seq0*G, seq0*G + nrows) of KV head kvh against keys
// [ks, ke) of the level's K/V rows; result to part sp.  ks < ke is not required (an empty range yields O = 0,
// LSE = -inf).
__device__ __forceinline__ void wide_piece(const PrefixArgs& a, unsigned char* smem, int seq0, int nrows, int kvh, int mt,
                                           int sp, int ks, int ke) {
    const int row0 = mt * kPrefixRowsWide;
    if (row0 >= nrows) return;
    const int tid = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l = tid & 63, lq = l & 31, hl = l >> 5;
    const int r = row0 + w * 32 + lq;     // this lane's query row inside the block
    const bool rv = r < nrows;
    const int rr = rv ? r : 0;
    const int rps = a.nq * a.G;           // query rows of one sequence for this KV head: (query t, head g) at t*G + g
    const int64_t qidx = ((int64_t)(seq0 + rr / rps) * a.nq + (rr % rps) / a.G) * a.Hq + kvh * a.G + rr % a.G;  // (b*nq + t)*Hq + h

    if (ks >= ke) {
        if (rv) {
            float* const Of = static_cast<float*>(a.out.O) + sp * a.out.part_stride_O + qidx * D;
            uint16_t* const Ob = static_cast<uint16_t*>(a.out.O) + sp * a.out.part_stride_O + qidx * D;
#pragma unroll
            for (int i = 0; i < D / 8; ++i) {
                const int d = 8 * i + 4 * hl;
                if (a.out.bf16) *reinterpret_cast<uint2*>(Ob + d) = make_uint2(0u, 0u);
                else *reinterpret_cast<float4*>(Of + d) = make_float4(0.f, 0.f, 0.f, 0.f);
            }
            if (hl == 0) a.out.LSE[sp * a.out.part_stride_L + qidx] = -INFINITY;
        }
        return;
    }

    // ---- Q operand (registers, whole piece) ----------------------------------------------------------------
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

    // ---- HBM -> LDS copies -----------------------------------------------------------------------------------
    // Stage t holds keys [k0c, k0c + 32) with k0c = min(ks + 32 t, kwin), kwin = max(ke - 32, 0): a stage that is
    // partial or past the range re-reads the last 32 rows of the range, so every stage is copied by the same
    // uniform instruction (wavefront w copies rows 4w .. 4w+3, 1 KiB); row i of a stage is a key of that stage
    // iff ks + 32 t <= k0c + i < ke.  The XOR swizzle of the 16-byte chunks is applied on the global side.  The
    // copies are issued from inline asm so that the compiler's wait-count pass does not see them: it would
    // otherwise force vmcnt(0) before every LDS read that follows a copy and serialise the ring.
    const unsigned rstride_b = (unsigned)a.Hkv * D * 2u;
    const int kwin = max(ke - KT, 0);
    const int srow = w * RPI + l / CPR;     // row of the stage this lane copies
    const int sch = l % CPR;
    unsigned voffK, voffV;
    {
        const int row = min(srow, ke - 1 - kwin);    // binds only when the range ends before row 32 of the tensor
        voffK = (unsigned)row * rstride_b + (unsigned)((sch ^ (srow % CPR)) * 16);
        voffV = (unsigned)row * rstride_b + (unsigned)((sch ^ (4 * (srow % 4))) * 16);
    }
    const unsigned char* const Kg = reinterpret_cast<const unsigned char*>(a.lv.K + (int64_t)kvh * D);
    const unsigned char* const Vg = reinterpret_cast<const unsigned char*>(a.lv.V + (int64_t)kvh * D);
    const unsigned ldsw = (unsigned)(uintptr_t)HG_LDS(smem) + (unsigned)w * (RPI * ROWB);

    auto copy16 = [&](const unsigned char* sbase, unsigned voff, unsigned lds_dst) {
        asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase), "s"(lds_dst) : "memory", "m0");
    };
    auto issue_stage = [&](int tstage, int slot) {
        const int k0c = min(ks + tstage * KT, kwin);
        const int64_t off = (int64_t)k0c * rstride_b;
        const unsigned dst = ldsw + (unsigned)slot * STB;
        copy16(Kg + off, voffK, dst);
        copy16(Vg + off, voffV, dst + VRING);
    };

    // ---- LDS fragment reads (addresses relative to the slot) ---------------------------------------------------
    // K operand for k-step q: row lq of the stage, chunk 2q+hl.  V^T operand for d-block db and key half tt:
    // within each 16-lane group lane i addresses key (i/4) of the 4 keys being transposed and columns
    // 4*(i%4) .. +3; group (l/16)&1 selects the lower/upper 16 columns, hl the key quad.
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
            vaddr[db] = (unsigned)(VRING + keyq * ROWB + ((chunk ^ fv) * 16) + (i16 & 1) * 8);
        }
    }
    auto lds_k = [&](int slot, int q) -> uintx4 { return *reinterpret_cast<const uintx4*>(smem + slot * STB + kaddr[q]); };
    auto lds_v = [&](int slot, int tt, int db) -> shortx8 {
        const unsigned char* vp = smem + slot * STB + vaddr[db] + tt * 16 * ROWB;
        const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) shortx4*)HG_LDS(vp));
        const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) shortx4*)HG_LDS(vp + 8 * ROWB));
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    };

    // ---- online softmax state ------------------------------------------------------------------------------------
    floatx16 Oacc[DB];
#pragma unroll
    for (int i = 0; i < DB; ++i)
#pragma unroll
        for (int k = 0; k < 16; ++k) Oacc[i][k] = 0.f;
    float m_used = -INFINITY;   // raw-score maximum the exponentials are taken against
    float lsum[2] = {0.f, 0.f}; // this lane's share of the row sum (of the unrounded exponentials), two chains
    float mc = 0.f;             // m_used * c2
    const float c2 = a.scale * kLog2e;
    const float tau_raw = TAU / c2;

    auto mask_stage = [&](floatx16& S, int tstage) {
        const int key0 = ks + tstage * KT;
        const int k0c = min(key0, kwin);
        const int lo = key0 - k0c - 4 * hl, hi = ke - k0c - 4 * hl;   // row i of this lane is 8*(i/4) + i%4 + 4*hl
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int ri = 8 * (i >> 2) + (i & 3);
            if (ri < lo || ri >= hi) S[i] = -INFINITY;
        }
    };
    auto maybe_rescale = [&](float tmax) {
        if (__any(tmax > m_used + tau_raw)) {
            const float m_new = fmaxf(m_used, tmax);
            // equal maxima (also -inf and -inf) keep the accumulators; otherwise exp2(-inf) = 0 for a first maximum
            const float alpha = (m_new == m_used) ? 1.0f : __builtin_amdgcn_exp2f((m_used - m_new) * c2);
            m_used = m_new;
            mc = m_new * c2;
            lsum[0] *= alpha;
            lsum[1] *= alpha;
#pragma unroll
            for (int i = 0; i < DB; ++i)
#pragma unroll
                for (int k = 0; k < 16; ++k) Oacc[i][k] *= alpha;
        }
    };

    // ---- prologue: stages 0 .. NS-2 in flight, scores of stage 0, first fragments ---------------------------------
#pragma unroll
    for (int s = 0; s < NS - 1; ++s) issue_stage(s, s);
    constexpr int kPrologueOutstanding = (NS - 3) * 2;     // copies of stages 2 .. NS-2 may still be in flight
    __builtin_amdgcn_s_waitcnt(0x0F70 | (kPrologueOutstanding & 15) | ((kPrologueOutstanding >> 4) << 14));
    __builtin_amdgcn_s_barrier();

    constexpr int kStepOutstanding = INFLIGHT * 2;
    constexpr int kStepWait = 0x0F70 | (kStepOutstanding & 15) | ((kStepOutstanding >> 4) << 14);
    const int nst = (ke - ks + KT - 1) / KT;       // stages with at least one key
    const int nfull = (ke - ks) / KT;              // stages with all keys in range

    if (row0 + w * 32 >= nrows) {
        // A wavefront whose 32 rows all lie past the block's last row (blocks of <= 224 rows) has nothing to multiply:
        // it keeps its share of the copies and meets the others at every barrier, one per stage as in step() below.
        for (int j = 0; j < nst; ++j) {
            __builtin_amdgcn_s_waitcnt(kStepWait);
            __builtin_amdgcn_s_barrier();
            issue_stage(j + NS - 1, (j + NS - 1) & (NS - 1));
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);
        return;
    }

    uintx4 kf[KS / 2];
    shortx8 vf[DB];
    floatx16 SA, SB;
    {
        uintx4 k0[KS];
#pragma unroll
        for (int q = 0; q < KS; ++q) k0[q] = lds_k(0, q);
        mfma_first(SA, k0[0], qf[0]);
#pragma unroll
        for (int q = 1; q < KS; ++q) mfma_acc(SA, k0[q], qf[q]);
    }
    if (nfull == 0) mask_stage(SA, 0);
    {
        float t = fmaxf(SA[0], SA[1]);
#pragma unroll
        for (int i = 2; i < 16; i += 2) t = fmaxf(fmaxf(t, SA[i]), SA[i + 1]);
        maybe_rescale(half_max(t));
    }
#pragma unroll
    for (int q = 0; q < KS / 2; ++q) kf[q] = lds_k(1, q);
#pragma unroll
    for (int db = 0; db < DB; ++db) vf[db] = lds_v(0, 0, db);

    // One pipeline step.  On entry: Scur = scores of stage j, kf = K fragments 0..3 of stage j+1, vf = V fragments
    // of keys 0..15 of stage j.  On exit the same with j+1, Snext = scores of stage j+1.  The copy of stage j+NS-1
    // goes into the slot that held stage j-1 (last read in step j-2, consumed in step j-1).  slot = j % NS.
    auto step = [&](int j, int slot, floatx16& Scur, floatx16& Snext, bool check_mask) {
        __builtin_amdgcn_s_waitcnt(kStepWait);    // own copies of stages <= j+2 have landed
        __builtin_amdgcn_s_barrier();             // ... everyone's, and everyone has finished step j-1
        uintx4 pb[2];
        float tmax;
        const int slot1 = (slot + 1) & (NS - 1), slot2 = (slot + 2) & (NS - 1);
#include "prefix_wide_step.inc"
        maybe_rescale(tmax);
    };

    int j = 0;
    // groups of NS steps in which every stage that is scored (j+1 .. j+NS) is either full or past the range:
    // slots are compile-time constants and no masks are needed
    while (j + NS < nfull || (j + NS == nfull && nst == nfull)) {
#pragma unroll
        for (int u = 0; u < NS; u += 2) {
            step(j + u, u, SA, SB, false);
            step(j + u + 1, u + 1, SB, SA, false);
        }
        j += NS;
    }
    for (; j < nst; ++j) {      // remainder: run-time slot, masks where needed
        step(j, j & (NS - 1), SA, SB, true);
        SA = SB;
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);   // drain the copies still in flight before the ring is reused or released

    // ---- epilogue ------------------------------------------------------------------------------------------------
    const float ltot = half_sum(lsum[0] + lsum[1]);
    if (rv) {
        float* const Of = static_cast<float*>(a.out.O) + sp * a.out.part_stride_O + qidx * D;
        uint16_t* const Ob = static_cast<uint16_t*>(a.out.O) + sp * a.out.part_stride_O + qidx * D;
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
        if (hl == 0) a.out.LSE[sp * a.out.part_stride_L + qidx] = m_used * a.scale + __logf(ltot);
    }
}

}  // namespace

__global__ __launch_bounds__(64 * NW, 1) void prefix_kernel_wide(PrefixArgs a) {
    const WidePlan& p = a.wide;
    const int pid = blockIdx.x;
    const int xcd = pid & 7, slot = pid >> 3;         // workgroup ids go round-robin over the 8 XCDs
    const int team_local = slot / p.T, member = slot % p.T;
    if (team_local >= p.tpx) return;
    const int team = xcd * p.tpx + team_local;
    const long long total = (long long)p.ncols * p.n_c;
    long long f0 = (long long)team * p.quota;
    const long long f1 = f0 + p.quota < total ? f0 + p.quota : total;
    int c = (int)(f0 / p.n_c);
    int k0 = (int)(f0 % p.n_c);
    while (f0 < f1) {
        const long long left = f1 - f0;
        const int len = (long long)(p.n_c - k0) < left ? p.n_c - k0 : (int)left;
        const int rg = c % p.rowgroups;
        const int kvh = (c / p.rowgroups) % a.Hkv;
        const int g = c / (p.rowgroups * a.Hkv);
        int seq0 = 0, seq1 = a.B, kv0 = 0, kv1 = a.lv.max_rows;
        if (a.lv.seq_off) {
            seq0 = a.lv.seq_off[g];
            seq1 = min(a.lv.seq_off[g + 1], seq0 + a.lv.max_seqs);
            kv0 = a.lv.kv_off[g];
            kv1 = min(a.lv.kv_off[g + 1], kv0 + a.lv.max_rows);
        }
        const int rps = a.nq * a.G;
        const int nrows = (seq1 - seq0) * rps;
        const int mt = rg * p.T + member;
        const int sp = team - (int)(((long long)c * p.n_c) / p.quota);    // piece index inside the column
        const int ks = kv0 + k0 * KT;
        wide_piece(a, wide_smem, seq0, nrows, kvh, mt, sp, ks, min(ks + len * KT, kv1));
        if (k0 + len == p.n_c) {
            // last piece of the column: the remaining parts of these rows hold no keys
            const int tid = threadIdx.x;
            const int r = mt * kPrefixRowsWide + tid;
            if (tid < kPrefixRowsWide && r < nrows) {
                const int64_t qidx = ((int64_t)(seq0 + r / rps) * a.nq + (r % rps) / a.G) * a.Hq + kvh * a.G + r % a.G;
                for (int q = sp + 1; q < p.nparts; ++q) a.out.LSE[q * a.out.part_stride_L + qidx] = -INFINITY;
            }
        }
        __builtin_amdgcn_s_barrier();   // every wavefront has left the ring before the next piece refills it
        f0 += len;
        ++c;
        k0 = 0;
    }
}

// Work partition of the persistent kernel for a level (host side).  Returns false when the level does not fit
// (more than max_parts partial results per row would be needed).
bool plan_prefix_wide(const LevelDev& lv, int Hkv, int G, int max_parts, int slots_per_xcd, WidePlan* out) {
    // G here is the number of query rows per sequence and KV head (queries per sequence x heads per group)
    WidePlan p{};
    const long long rows = (long long)lv.max_seqs * G;
    const int mtiles = (int)((rows + kPrefixRowsWide - 1) / kPrefixRowsWide);
    if (mtiles < 1 || lv.max_rows < 1) return false;
    if (slots_per_xcd < 1 || slots_per_xcd > 32) return false;
    p.slots = slots_per_xcd;
    p.rowgroups = (mtiles + p.slots - 1) / p.slots;         // the workgroups of a team run on one XCD
    p.T = (mtiles + p.rowgroups - 1) / p.rowgroups;
    p.tpx = p.slots / p.T;
    p.n_c = (lv.max_rows + KT - 1) / KT;
    const long long ncols = (long long)lv.n_blocks * Hkv * p.rowgroups;
    if (ncols >= (1LL << 24)) return false;
    p.ncols = (int)ncols;
    const long long total = ncols * p.n_c;
    const int nteams = 8 * p.tpx;
    long long q = (total + nteams - 1) / nteams;
    if (q >= 64) q = (q + NS - 1) / NS * NS;                // whole groups of NS stages run without masks
    if (q < 1) q = 1;
    auto parts_needed = [&](long long quota) {     // most pieces any column is cut into
        int np = 1;
        for (long long c = 0; c < ncols; ++c) {
            const long long lo = c * p.n_c, hi = lo + p.n_c - 1;
            const int n = (int)(hi / quota - lo / quota) + 1;
            if (n > np) np = n;
        }
        return np;
    };
    if (max_parts < 1) return false;
    int np = parts_needed(q);
    if (np > max_parts) {
        // Longer ranges per team (some teams then stay idle) until the parts fit, as long as the teams still cover
        // the whole space; otherwise whole columns per team, which always fits in one part.
        const long long qa = max_parts >= 2 ? (p.n_c + max_parts - 2) / (max_parts - 1) : 0;
        if (qa >= 1 && qa * nteams >= total && parts_needed(qa) <= max_parts) {
            q = qa;
            np = parts_needed(qa);
        } else {
            q = (ncols + nteams - 1) / nteams * p.n_c;
            np = 1;
        }
    }
    if (q >= (1LL << 30)) return false;
    p.quota = (int)q;
    p.nparts = np;
    *out = p;
    return true;
}

hipError_t launch_prefix_wide(const PrefixArgs& a, hipStream_t s) {
    static bool attr_set[64] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 64 && !attr_set[dev]) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&prefix_kernel_wide), hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set[dev] = true;
    }
    prefix_kernel_wide<<<8 * a.wide.slots, 64 * NW, LDS_BYTES, s>>>(a);
    return hipGetLastError();
}

}  // namespace hg
