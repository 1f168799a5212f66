// Inter-sequence batched attention over one shared KV block (Sec. 3.2 of the paper), persistent 256-row kernel: the
// body shared by prefix_wide.hip (D = 128, HG_WIDE_D = 128) and prefix_wide_d64.hip (D = 64), which define HG_WIDE_D and
// HG_WIDE_KERNEL and include this file; the head dimension is a macro, not a template parameter, so that each
// translation unit sees exactly one kernel.  The B*G query rows that use a KV head are stacked into one matrix and multiplied against that
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
//     KT keys (32 at D = 128, 64 at D = 64: 8 KiB of K and of V either way), so a team shares its K/V reads in one XCD's L2 and every team gets the same number of stages: no
//     tail round.  A column that is cut by a range boundary yields several partial results (part index = piece
//     index inside the column); the workgroup that finishes a column marks the unused parts empty.
//   * Ring of 8 stages (K and V, 16 KiB together) in 128 KiB of dynamic LDS, filled by direct HBM->LDS copies that
//     are issued from inline asm and waited for with counted s_waitcnt vmcnt: four stages are in flight while
//     one is consumed.
//   * Software pipeline over stages, written out by gen_prefix_wide_step.py: in one step the scores of stage j+1
//     are produced while the exponentials of stage j are taken and its P*V product runs; fragments are loaded
//     from LDS four MFMAs before their use; the vector-ALU work is spread over the gaps between the MFMAs.  At D = 64 a
//     stage has two 32-key score tiles: the same 16 MFMAs per step with twice the softmax work between them.
#include <algorithm>
#include <type_traits>

#include "hg_internal.h"
#include "prefix_common.h"

// the copy helper names m0 as clobbered on purpose (it writes it)
#pragma clang diagnostic ignored "-Winline-asm"

namespace hg {

namespace {

constexpr int D = HG_WIDE_D;
constexpr int KT = D == 128 ? 32 : 64;  // keys per stage: 8 KiB of K and 8 KiB of V at either head dimension
constexpr int KB = KT / 32;             // 32-key score tiles per stage
constexpr int NS = 8;                   // ring slots
constexpr int NW = 8;                   // wavefronts per workgroup
constexpr int KS = D / 16;              // MFMA k-steps of the score product
constexpr int DB = D / 32;              // 32-row blocks of O^T
constexpr int NKF = 4, NVF = 4;         // K and V fragment registers a wavefront holds (half a stage's worth each)
constexpr int CPR = D / 8;              // 16-byte chunks per K/V row
constexpr int RPI = 64 / CPR;           // rows one wavefront copies per direct-to-LDS instruction
constexpr int ROWB = D * 2;             // bytes per row
constexpr int STB = KT * ROWB;          // bytes per stage and tensor
constexpr int VRING = NS * STB;         // byte offset of the V ring
constexpr int LDS_RING_BYTES = 2 * NS * STB;        // 128 KiB
constexpr int kStageBytes = 32 * 32 * 4;              // staging area of one wavefront for its results: 32 columns of its 32 rows, fp32
constexpr int LDS_BYTES = LDS_RING_BYTES + NW * kStageBytes;   // 160 KiB, all of a CU's LDS
constexpr int INFLIGHT = 4;             // stages that may still be in flight at a step's barrier
constexpr float TAU = 8.0f;             // lazy-rescale threshold, log2 units
static_assert(KT == NW * RPI, "one copy instruction per wavefront, stage and tensor");
static_assert(kPrefixRowsWide == 32 * NW, "one 32-row query block per wavefront");

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef unsigned uintx4 __attribute__((ext_vector_type(4)));

// XOR swizzle of the 16-byte chunks of LDS row `row` (applied on the global side of the copies).  256-byte rows: K
// chunk ^ row % 16 makes the 16 rows of a ds_read_b128 pass distinct, V chunk ^ 4 (row % 4) separates the 4 rows of a
// transposing read.  128-byte rows are half a bank period, so consecutive rows already differ: K chunk ^ (row / 2) % 8,
// V chunk ^ 4 ((row / 2) % 2).
__device__ __forceinline__ int kswz(int row) { return D == 128 ? row % 16 : (row >> 1) & 7; }
__device__ __forceinline__ int vswz(int row) { return D == 128 ? 4 * (row % 4) : 4 * ((row >> 1) & 1); }

// The scores of one stage as this lane holds them: one 32-key tile at D = 128, two at D = 64.
#if HG_WIDE_D == 128
typedef floatx16 STile;
#else
struct STile { floatx16 a, b; };
#endif

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

// Phase time stamps of a -DHG_TRACE build (a measurement aid, compiled out otherwise): thread 0 of every workgroup
// stores the 100 MHz real-time counter at kernel entry (slot 0) and exit (slot 15) and, for its first three pieces
// p, at 1 + 4p + {0 piece entry, 1 first scores done, 2 main loop done, 3 results stored}; slots 16 + p hold the
// shader-clock cycles of piece p's main loop; slots 19 .. 22 split the boundary between pieces 0 and 1 (next piece
// looked up, its Q requested, Q landed, barrier passed); slots 13, 14 and 23 hold the number of stages of pieces 0, 1
// and 2 (a count, not a time); slots 24 .. 27 split the start of the kernel (first piece looked up, copy cursor set,
// two stages' copies issued, Q requested); slot 28 holds the id of the XCD the workgroup ran on.  hg_debug_read_wide_trace copies the table to the host.
#ifdef HG_TRACE
constexpr int kTraceSlots = 32;
__device__ unsigned long long hg_wide_trace[256 * kTraceSlots];
#define HG_T(slot) do { if (threadIdx.x == 0) hg_wide_trace[blockIdx.x * kTraceSlots + (slot)] = __builtin_amdgcn_s_memrealtime(); } while (0)
#define HG_TP(piece, k) do { if ((piece) < 3) HG_T(1 + 4 * (piece) + (k)); } while (0)
#define HG_TN(piece, n) do { if (threadIdx.x == 0 && (piece) < 3) hg_wide_trace[blockIdx.x * kTraceSlots + ((piece) == 2 ? 23 : 13 + (piece))] = (unsigned long long)(n); } while (0)
#define HG_TC_BEGIN() const unsigned long long hg_tc0 = __builtin_amdgcn_s_memtime()
#define HG_TC_END(piece) do { if (threadIdx.x == 0 && (piece) < 3) hg_wide_trace[blockIdx.x * kTraceSlots + 16 + (piece)] = __builtin_amdgcn_s_memtime() - hg_tc0; } while (0)
#else
#define HG_T(slot) do { } while (0)
#define HG_TP(piece, k) do { } while (0)
#define HG_TN(piece, n) do { } while (0)
#define HG_TC_BEGIN() do { } while (0)
#define HG_TC_END(piece) do { } while (0)
#endif

}  // namespace

// A piece of work: 256-row tile row0/256 of the query rows [seq0*rps, seq0*rps + nrows) of KV head kvh against keys
// [ks, ke) of the level's K/V rows, result to part sp.  Everything here is uniform over the workgroup.
struct WidePiece {
    int seq0, nrows, row0, kvh, sp;
    int ks, ke, kwin;    // kwin = max(ke - 32, 0): first row of the last full window of the range
    int nst, nfull;      // stages with at least one key (0: nothing to multiply), stages with KT keys
    int last_in_col;     // the piece ends its column: the parts above sp are marked empty
    int has_rows;        // row0 < nrows
};

__global__ __launch_bounds__(64 * NW, 1) void HG_WIDE_KERNEL(PrefixArgs a) {
    HG_T(0);
#ifdef HG_TRACE
    if (threadIdx.x == 0) hg_wide_trace[blockIdx.x * kTraceSlots + 28] = __builtin_amdgcn_s_getreg((3 << 11) | 20) & 15u;   // XCC_ID
#endif
    mark_uncovered(a, D, a.wide.nparts, blockIdx.x, gridDim.x);
    unsigned char* const smem = wide_smem;
    const WidePlan& p = a.wide;
    const int pid = blockIdx.x;
    const int xcd = pid & 7, cu_slot = pid >> 3;         // workgroups whose ids are equal modulo 8 run on one XCD (which one varies by launch)
    const int team_local = cu_slot / p.T, member = cu_slot % p.T;
    if (team_local >= p.tpx) return;
    const int team = xcd * p.tpx + team_local;
    const int nteams = 8 * p.tpx;
    const int total = p.ncols * p.n_c;      // the planner keeps this below 2^31 (and the columns below 2^20)

    // ---- this team's range [f0, f1) of the flattened (column, stage) space; sp0 = part index of its first piece ----
    // (32-bit arithmetic: a 64-bit division costs a loop of its own on this chip)
    int f0, f1, sp0;
    if (p.mode == 0) {            // equal contiguous ranges
        const long long lo = (long long)team * p.quota;
        if (lo >= total) return;
        f0 = (int)lo;
        f1 = (int)(lo + p.quota < total ? lo + p.quota : total);
        sp0 = team - (int)((unsigned)(f0 / p.n_c * p.n_c) / (unsigned)p.quota);
    } else if (p.mode == 2) {     // ranges of equal cost, from the planner's table
        f0 = p.starts[team];
        f1 = p.starts[team + 1];
        sp0 = p.first_part[team];
    } else if (p.ncols <= nteams) {   // every column is cut evenly among its own teams
        const int c = team * p.ncols / nteams;
        const int tf = (c * nteams + p.ncols - 1) / p.ncols;
        const int nt = ((c + 1) * nteams + p.ncols - 1) / p.ncols - tf;
        sp0 = team - tf;
        f0 = c * p.n_c + (int)((unsigned)sp0 * (unsigned)p.n_c / (unsigned)nt);
        f1 = c * p.n_c + (int)((unsigned)(sp0 + 1) * (unsigned)p.n_c / (unsigned)nt);
    } else {                      // whole columns per team
        f0 = (int)((unsigned)team * (unsigned)p.ncols / (unsigned)nteams) * p.n_c;
        f1 = (int)((unsigned)(team + 1) * (unsigned)p.ncols / (unsigned)nteams) * p.n_c;
        sp0 = 0;
    }
    if (f0 >= f1) return;

    const int tid = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l = tid & 63, lq = l & 31, hl = l >> 5;
    const unsigned rstride_b = (unsigned)a.Hkv * D * 2u;

    // block offsets are read through the constant address space: nothing writes them while the kernel runs, and the
    // loads then stay on the scalar unit (a vector load would make the compiler wait for vmcnt(0) and drain the ring)
    typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;

    // Everything that happens once per piece reads the kernel's arguments again from the kernarg segment (through a
    // pointer the compiler cannot see through) instead of keeping them in scalar registers across the pipeline
    // steps: the steps need those registers themselves, and what does not fit is parked in vector-register lanes.
    typedef const __attribute__((address_space(4))) PrefixArgs* kargs_ptr;
    auto kargs = [&]() -> kargs_ptr {
        kargs_ptr k = (kargs_ptr)__builtin_amdgcn_kernarg_segment_ptr();
        asm volatile("" : "+s"(k));
        return k;
    };

    // piece at flattened position f = (column c, stage k0) with part index sp; returns its length in stages
    auto load_piece = [&](kargs_ptr k, int f, int c, int k0, int sp, WidePiece& q) -> int {
        const int n_c = k->wide.n_c, rowgroups = k->wide.rowgroups, Hkv = k->Hkv;
        const int len = min(n_c - k0, f1 - f);
        const int rg = c % rowgroups;
        const int kvh = (c / rowgroups) % Hkv;
        const int g = c / (rowgroups * Hkv);
        int seq0 = 0, seq1 = k->B, kv0 = 0, kv1 = k->lv.max_rows;
        const const_i32_ptr seq_off_c = (const_i32_ptr)(uintptr_t)k->lv.seq_off;
        if (seq_off_c) {
            const const_i32_ptr kv_off_c = (const_i32_ptr)(uintptr_t)k->lv.kv_off;
            seq0 = seq_off_c[g];
            seq1 = min(seq_off_c[g + 1], seq0 + k->lv.max_seqs);
            kv0 = kv_off_c[g];
            kv1 = min(kv_off_c[g + 1], kv0 + k->lv.max_rows);
        }
        q.seq0 = seq0;
        q.nrows = (seq1 - seq0) * (k->nq * k->G);
        q.row0 = (rg * k->wide.T + member) * kPrefixRowsWide;
        q.kvh = kvh;
        q.sp = sp;
        q.ks = kv0 + k0 * KT;
        q.ke = min(q.ks + len * KT, kv1);
        q.kwin = max(q.ke - KT, 0);
        q.has_rows = q.row0 < q.nrows;
        const int n = q.ke - q.ks;
        q.nst = (q.has_rows && n > 0) ? (n + KT - 1) / KT : 0;
        q.nfull = n > 0 ? n / KT : 0;
        q.last_in_col = (k0 + len == n_c);
        return len;
    };

    // ---- HBM -> LDS copies -----------------------------------------------------------------------------------------
    // The ring is one stream of stages across all of this workgroup's pieces: global stage g lives in slot g % NS, and
    // the copy side (the cursor below) stays NS-1 stages ahead of the compute side, also across a piece boundary, so
    // that a piece after the first finds its first stages in LDS already.  Stage t of a piece holds keys
    // [k0c, k0c + 32) with k0c = min(ks + 32 t, kwin): a stage that is partial or past the range re-reads the last 32
    // rows of the range, so every stage is copied by the same uniform instruction (wavefront w copies rows 4w .. 4w+3,
    // 1 KiB); row i of a stage is a key of that stage iff ks + 32 t <= k0c + i < ke.  The XOR swizzle of the 16-byte
    // chunks is applied on the global side.  The copies are issued from inline asm so that the compiler's wait-count
    // pass does not see them: it would otherwise force vmcnt(0) before every LDS read that follows a copy.
    const int srow = w * RPI + l / CPR;     // row of the stage this lane copies
    const int sch = l % CPR;
    const unsigned ldsw = (unsigned)(uintptr_t)HG_LDS(smem) + (unsigned)w * (RPI * ROWB);
    struct Cursor {
        const unsigned char* Kg;     // the piece's KV head in the level's K / V tensors
        const unsigned char* Vg;
        int ks, kwin, t, left;       // t: next stage of the piece to copy; left: stages of the piece not yet copied
        unsigned voffK, voffV;       // this lane's byte offset inside a stage (row, swizzled chunk)
        int valid;
    } cur{};
    int cf = f0;                     // position of the piece after the cursor's
    int cc = f0 / p.n_c, ck0 = f0 - cc * p.n_c;
    auto cursor_set = [&](kargs_ptr k, const WidePiece& q) {      // points the cursor at the first stage of piece q (q.nst > 0)
        // (everything but the lane offsets is uniform; saying so keeps it in scalar registers, where the copy
        // instructions take their base address from)
        auto uniform_ptr = [](const uint16_t* ptr) {
            const uint64_t v = reinterpret_cast<uint64_t>(ptr);
            const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
            return reinterpret_cast<const unsigned char*>(((uint64_t)hi << 32) | lo);
        };
        cur.Kg = uniform_ptr(k->lv.K + (int64_t)q.kvh * D);
        cur.Vg = uniform_ptr(k->lv.V + (int64_t)q.kvh * D);
        cur.ks = __builtin_amdgcn_readfirstlane(q.ks);
        cur.kwin = __builtin_amdgcn_readfirstlane(q.kwin);
        cur.t = 0;
        cur.left = __builtin_amdgcn_readfirstlane((q.nst + NS - 1) & ~(NS - 1));     // the stream pads every piece to whole groups of NS stages
        const int row = min(srow, q.ke - 1 - q.kwin);    // binds only when the range ends before row KT of the tensor
        cur.voffK = (unsigned)row * rstride_b + (unsigned)((sch ^ kswz(srow)) * 16);
        cur.voffV = (unsigned)row * rstride_b + (unsigned)((sch ^ vswz(srow)) * 16);
        cur.valid = 1;
    };
    auto cursor_next_piece = [&](kargs_ptr k) {          // moves the cursor to the next piece that has stages, if there is one
        while (cf < f1) {
            WidePiece q;
            const int len = load_piece(k, cf, cc, ck0, 0, q);
            cf += len;
            ++cc;
            ck0 = 0;
            if (q.nst > 0) {
                cursor_set(k, q);
                return;
            }
        }
    };
    auto copy16 = [&](const unsigned char* sbase, unsigned voff, unsigned lds_dst) {
        asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase), "s"(lds_dst) : "memory", "m0");
    };
    // after a stage has been issued: one stage further; past the end of its last piece the cursor stays where it is
    // and keeps re-reading that piece's last window (stages nobody consumes)
    auto cursor_advance = [&]() {
        ++cur.t;
        if (--cur.left == 0) cursor_next_piece(kargs());
    };
    auto cursor_step = [&]() {      // inside a group of NS steps, which is entered only with NS stages left in the cursor's piece
        ++cur.t;
        --cur.left;
    };
    auto issue_stage = [&](int slot) {
        const int64_t off = (int64_t)min(cur.ks + cur.t * KT, cur.kwin) * rstride_b;
        const unsigned dst = ldsw + (unsigned)slot * STB;
        copy16(cur.Kg + off, cur.voffK, dst);
        copy16(cur.Vg + off, cur.voffV, dst + VRING);
        cursor_advance();
    };

    // ---- LDS fragment reads (addresses relative to the slot) ---------------------------------------------------
    // K operand for fragment f = (32-key tile f / KS, k-step q = f % KS): row lq of the tile, chunk 2q+hl (rows 32 apart
    // share their swizzle).  V^T operand for d-block db and 16-key group tt:
    // within each 16-lane group lane i addresses key (i/4) of the 4 keys being transposed and columns
    // 4*(i%4) .. +3; group (l/16)&1 selects the lower/upper 16 columns, hl the key quad.
    unsigned kaddr[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) kaddr[s] = (unsigned)(lq * ROWB + (((2 * s + hl) ^ kswz(lq)) * 16));
    unsigned vaddr[DB];
    {
        const int i16 = l & 15, g1 = (l >> 4) & 1;
        const int keyq = 4 * hl + (i16 >> 2);
        const int fv = vswz(keyq);      // (rows 8 and 16 apart share their swizzle)
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const int chunk = 4 * db + 2 * g1 + ((i16 & 3) >> 1);
            vaddr[db] = (unsigned)(VRING + keyq * ROWB + ((chunk ^ fv) * 16) + (i16 & 1) * 8);
        }
    }
    auto lds_k = [&](int slot, int f) -> uintx4 {
        return *reinterpret_cast<const uintx4*>(smem + slot * STB + (f / KS) * 32 * ROWB + kaddr[f % KS]);
    };
    auto lds_v = [&](int slot, int tt, int db) -> shortx8 {
        const unsigned char* vp = smem + slot * STB + vaddr[db] + tt * 16 * ROWB;
        const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) shortx4*)HG_LDS(vp));
        const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) shortx4*)HG_LDS(vp + 8 * ROWB));
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    };

    // ---- per-lane view of a piece: this lane's query row and where its result goes ------------------------------------
    struct RowCtx { bool rv; int64_t qidx; };
    // a sequence contributes nq * G rows per KV head: (query t, head g) at t*G + g
    auto row_index = [&](kargs_ptr k, const WidePiece& q, int r) -> int64_t {     // (b*nq + t)*Hq + h of row r of the block
        const int G = k->G, nq = k->nq, rps = nq * G;
        return ((int64_t)(q.seq0 + r / rps) * nq + (r % rps) / G) * k->Hq + q.kvh * G + r % G;
    };
    auto row_ctx = [&](kargs_ptr k, const WidePiece& q) -> RowCtx {
        const int r = q.row0 + w * 32 + lq;     // this lane's query row inside the block
        RowCtx rc;
        rc.rv = r < q.nrows;
        rc.qidx = row_index(k, q, rc.rv ? r : 0);
        return rc;
    };
    // Q operand (registers, whole piece).  The KS loads are issued from inline asm, like the copies, and waited for
    // with a counted s_waitcnt: the compiler would answer a load it can see with vmcnt(0) before the first product,
    // which waits for every copy in flight and every result store of the piece before.  Until that wait the registers
    // are only named, never read: the compiler takes them for loaded when the asm statement ends.  Lanes past the
    // block's last row read row 0 of the block (their results are never stored).
    uintx4 qraw[KS];
    auto load_q = [&](kargs_ptr k, const RowCtx& rc) {
        const uint16_t* qp = k->Q + rc.qidx * D + 8 * hl;
#if HG_WIDE_D == 64
        static_assert(KS == 4, "load_q names four registers");
        asm volatile(
            "global_load_dwordx4 %0, %4, off\n\t"
            "global_load_dwordx4 %1, %4, off offset:32\n\t"
            "global_load_dwordx4 %2, %4, off offset:64\n\t"
            "global_load_dwordx4 %3, %4, off offset:96"
            : "=&v"(qraw[0]), "=&v"(qraw[1]), "=&v"(qraw[2]), "=&v"(qraw[3])
            : "v"(qp)
            : "memory");
#else
        static_assert(KS == 8, "load_q names eight registers");
        asm volatile(
            "global_load_dwordx4 %0, %8, off\n\t"
            "global_load_dwordx4 %1, %8, off offset:32\n\t"
            "global_load_dwordx4 %2, %8, off offset:64\n\t"
            "global_load_dwordx4 %3, %8, off offset:96\n\t"
            "global_load_dwordx4 %4, %8, off offset:128\n\t"
            "global_load_dwordx4 %5, %8, off offset:160\n\t"
            "global_load_dwordx4 %6, %8, off offset:192\n\t"
            "global_load_dwordx4 %7, %8, off offset:224"
            : "=&v"(qraw[0]), "=&v"(qraw[1]), "=&v"(qraw[2]), "=&v"(qraw[3]), "=&v"(qraw[4]), "=&v"(qraw[5]), "=&v"(qraw[6]),
              "=&v"(qraw[7])
            : "v"(qp)
            : "memory");
#endif
    };
    // Memory operations of a wavefront complete in the order they were issued.  Waiting until at most `younger`
    // operations are outstanding, where `younger` operations were issued after the Q loads, therefore waits for Q and
    // for every copy issued before it, and for nothing issued after it.
    constexpr int kStoresPerPiece = D / 8 + 1;     // result stores of a wavefront whose 32 rows all exist: 16 of O, 1 of LSE
    enum { kQFirst = 0, kQAfterStores = 1, kQDrain = 2 };
    auto wait_q = [&](int kind) {
        constexpr int kFirst = (NS - 3) * 2;       // kernel start: two stages, Q, then NS-3 stages more, which may stay in flight
        if (kind == kQFirst) __builtin_amdgcn_s_waitcnt(0x0F70 | (kFirst & 15) | ((kFirst >> 4) << 14));
        else if (kind == kQAfterStores) __builtin_amdgcn_s_waitcnt(0x0F70 | (kStoresPerPiece & 15) | ((kStoresPerPiece >> 4) << 14));
        else __builtin_amdgcn_s_waitcnt(0x0F70);
    };
    auto mark_rest_empty = [&](kargs_ptr k, const WidePiece& q) {
        // last piece of a column: the remaining parts of these rows hold no keys
        const int r = q.row0 + tid;
        if (tid < kPrefixRowsWide && r < q.nrows) {
            const int64_t qidx = row_index(k, q, r);
            for (int i = q.sp + 1; i < k->wide.nparts; ++i) k->out.LSE[i * k->out.part_stride_L + qidx] = -INFINITY;
        }
    };
    auto store_empty = [&](kargs_ptr k, const WidePiece& q, const RowCtx& rc) {    // a piece without keys: O = 0, LSE = -inf
        if (rc.rv) {
            float* const Of = static_cast<float*>(k->out.O) + q.sp * k->out.part_stride_O + rc.qidx * D;
            uint16_t* const Ob = static_cast<uint16_t*>(k->out.O) + q.sp * k->out.part_stride_O + rc.qidx * D;
#pragma unroll
            for (int i = 0; i < D / 8; ++i) {
                const int d = 8 * i + 4 * hl;
                if (k->out.bf16) *reinterpret_cast<uint2*>(Ob + d) = make_uint2(0u, 0u);
                else *reinterpret_cast<float4*>(Of + d) = make_float4(0.f, 0.f, 0.f, 0.f);
            }
            if (hl == 0) k->out.LSE[q.sp * k->out.part_stride_L + rc.qidx] = -INFINITY;
        }
    };

    // ---- compute-side piece iterator: skips pieces with nothing to multiply (after writing what they owe) -------------
    int pf = f0;
    int pcol = cc, pk0 = ck0, psp = sp0;
    WidePiece pc{};
    auto next_piece = [&](kargs_ptr k) -> bool {     // false: the range is exhausted
        while (pf < f1) {
            const int len = load_piece(k, pf, pcol, pk0, psp, pc);
            pf += len;
            ++pcol;
            pk0 = 0;
            psp = 0;
            if (pc.nst > 0) return true;
            if (pc.has_rows) {
                store_empty(k, pc, row_ctx(k, pc));
                if (pc.last_in_col) mark_rest_empty(k, pc);
            }
        }
        return false;
    };

    // ---- online softmax state ------------------------------------------------------------------------------------
    floatx16 Oacc[DB];
    float m_used;               // raw-score maximum the exponentials are taken against
    float lsum[2];              // this lane's share of the row sum (of the unrounded exponentials), two chains
    float mc;                   // m_used * c2
    const float c2 = a.scale * kLog2e;
    const float tau_raw = TAU / c2;
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

    constexpr int kStepOutstanding = INFLIGHT * 2;
    constexpr int kStepWait = 0x0F70 | (kStepOutstanding & 15) | ((kStepOutstanding >> 4) << 14);

    // ---- results of a finished piece (its accumulators are still in registers when this runs) -------------------------
    // A lane holds half of one row of O^T (64 values, every other group of four columns), and consecutive lanes hold
    // rows that lie Hq * D elements apart in memory: stored from there, every lane of a store instruction would touch
    // a cache line of its own, and the store unit takes the lanes' addresses one at a time.  The rows therefore go
    // through a 4 KiB staging area per wavefront (in the 32 KiB of LDS behind the ring, which no copy touches), 32
    // columns of all 32 rows at a time, and leave it as whole 128-byte lines, eight rows per store instruction.
    // 16-byte chunk c of staged row r lives at chunk c ^ (r % 8): writes and reads are free of bank conflicts.
    // A wavefront whose 32 rows all exist issues exactly kStoresPerPiece store instructions; one with fewer rows, fewer.
    auto store_piece = [&](kargs_ptr k, const WidePiece& q, bool q_idle) {
        if (q_idle) return;
        // (the lane id is taken through an empty asm statement: the compiler would otherwise compute the staging
        // addresses once, before the first piece, and keep them in registers the pipeline steps need)
        int l = tid & 63;
        asm volatile("" : "+v"(l));
        const int lq = l & 31, hl = l >> 5;
        const RowCtx qrc = row_ctx(k, q);
        const float ltot = half_sum(lsum[0] + lsum[1]);
        const float inv = 1.0f / ltot;
        const int my_row = qrc.rv ? (int)qrc.qidx : -1;            // query row index (b*nq + t)*Hq + h, below 2^31 / D
        if (qrc.rv && hl == 0) k->out.LSE[q.sp * k->out.part_stride_L + qrc.qidx] = m_used * k->scale + __logf(ltot);
        const int nvalid = min(q.nrows - (q.row0 + w * 32), 32);   // rows of this wavefront that exist (>= 1)
        unsigned char* const stg = smem + LDS_RING_BYTES + w * kStageBytes;
        float* const Of = static_cast<float*>(k->out.O) + q.sp * k->out.part_stride_O;
        uint16_t* const Ob = static_cast<uint16_t*>(k->out.O) + q.sp * k->out.part_stride_O;
        const bool out_bf16 = k->out.bf16 != 0;
        int row_of[4];       // the query row this lane forwards in the kk-th store of a pass: row 8 kk + l / 8 of the wavefront
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) row_of[kk] = __shfl(my_row, 8 * kk + (l >> 3));
#pragma unroll
        for (int db = 0; db < DB; ++db) {
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4)
                *reinterpret_cast<float4*>(stg + lq * 128 + (((2 * q4 + hl) ^ (lq & 7)) * 16)) =
                    make_float4(Oacc[db][4 * q4] * inv, Oacc[db][4 * q4 + 1] * inv, Oacc[db][4 * q4 + 2] * inv, Oacc[db][4 * q4 + 3] * inv);
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                if (8 * kk < nvalid) {                             // (uniform: the instruction is issued or not as a whole)
                    const int r = 8 * kk + (l >> 3), c = l & 7;
                    const float4 v = *reinterpret_cast<const float4*>(stg + r * 128 + ((c ^ (r & 7)) * 16));
                    const int row = row_of[kk];
                    if (row >= 0) {
                        if (out_bf16)
                            *reinterpret_cast<uint2*>(Ob + (int64_t)row * D + 32 * db + 4 * c) = make_uint2(pack_bf16(v.x, v.y), pack_bf16(v.z, v.w));
                        else
                            *reinterpret_cast<float4*>(Of + (int64_t)row * D + 32 * db + 4 * c) = v;
                    }
                }
            }
        }
    };

    // ---- the pieces of this workgroup, one per iteration ------------------------------------------------------------------
    {
        const kargs_ptr k = kargs();       // one look at the arguments for everything up to the first copies
        if (!next_piece(k)) return;
        HG_T(24);
        // the copy cursor starts at the piece the compute side has just found (the pieces before it have no stages); its
        // first two stages are requested before Q, which the first products need together with them
        cf = pf;
        cc = pcol;
        ck0 = pk0;
        cursor_set(k, pc);
        HG_T(25);
        issue_stage(0);
        issue_stage(1);
        HG_T(26);
        load_q(k, row_ctx(k, pc));
        HG_T(27);
    }
    int qkind = kQFirst;
#pragma unroll
    for (int s = 2; s < NS - 1; ++s) issue_stage(s);
    int piece_no = 0;

    for (;;) {
        HG_TP(piece_no, 0);
        HG_TN(piece_no, pc.nst);
        // ---- piece prologue ---------------------------------------------------------------------------------------------
        // Q and the stream's next stages have landed, for everyone
        wait_q(qkind);
        if (piece_no == 1) HG_T(21);
        __builtin_amdgcn_s_barrier();
        if (piece_no == 1) HG_T(22);
        bf16x8 qf[KS];
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            asm volatile("" : "+v"(qraw[s]));      // the products below stay behind the wait above
            qf[s] = __builtin_bit_cast(bf16x8, qraw[s]);
        }
        const int ks = pc.ks, ke = pc.ke, kwin = pc.kwin;
        const bool idle = pc.row0 + w * 32 >= pc.nrows;    // blocks of <= 224 rows: this wavefront has nothing to multiply

        // rows of a partial stage that are nobody's keys may hold anything: their scores are masked, and their V rows
        // are cleared in LDS before the second product reads them (0 * NaN would be NaN).  The partial stage is the
        // piece's last; it is cleared at the top of the step before the one that first reads its V rows.
        const int zstep = pc.nst > pc.nfull ? pc.nst - 2 : -8;
        auto clear_partial_v = [&]() {
            const int t = pc.nst - 1;
            const int key0 = ks + t * KT, k0c = min(key0, kwin);
            const int lo = key0 - k0c, hi = ke - k0c;
            const int row = tid / CPR;          // 64 * NW threads = KT rows x CPR chunks
            if (row < lo || row >= hi)
                *reinterpret_cast<uint4*>(smem + VRING + (t & (NS - 1)) * STB + row * ROWB + (tid % CPR) * 16) = make_uint4(0, 0, 0, 0);
            __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0): the writes are done
            __builtin_amdgcn_s_barrier();
        };
        if (zstep == -1) clear_partial_v();

        auto mask_stage = [&](STile& S, int tstage) {
            const int key0 = ks + tstage * KT;
            const int k0c = min(key0, kwin);
            const int lo = key0 - k0c - 4 * hl, hi = ke - k0c - 4 * hl;   // row i of this lane is 8*(i/4) + i%4 + 4*hl (+ 32 in the second tile)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int ri = 8 * (i >> 2) + (i & 3);
#if HG_WIDE_D == 128
                if (ri < lo || ri >= hi) S[i] = -INFINITY;
#else
                if (ri < lo || ri >= hi) S.a[i] = -INFINITY;
                if (ri + 32 < lo || ri + 32 >= hi) S.b[i] = -INFINITY;
#endif
            }
        };

#pragma unroll
        for (int i = 0; i < DB; ++i)
#pragma unroll
            for (int k = 0; k < 16; ++k) Oacc[i][k] = 0.f;
        m_used = -INFINITY;
        lsum[0] = lsum[1] = 0.f;
        mc = 0.f;

        uintx4 kf[NKF];
        shortx8 vf[NVF];
        STile SA, SB;
        if (!idle) {
            constexpr int s0 = 0, s1 = 1;        // a piece starts at slot 0
            uintx4 k0[KB * KS];
#pragma unroll
            for (int q = 0; q < KB * KS; ++q) k0[q] = lds_k(s0, q);
#if HG_WIDE_D == 128
            mfma_first(SA, k0[0], qf[0]);
#pragma unroll
            for (int q = 1; q < KS; ++q) mfma_acc(SA, k0[q], qf[q]);
            if (pc.nfull == 0) mask_stage(SA, 0);
            float t = fmaxf(SA[0], SA[1]);
#pragma unroll
            for (int i = 2; i < 16; i += 2) t = fmaxf(fmaxf(t, SA[i]), SA[i + 1]);
#else
            mfma_first(SA.a, k0[0], qf[0]);
            mfma_first(SA.b, k0[KS], qf[0]);
#pragma unroll
            for (int q = 1; q < KS; ++q) {
                mfma_acc(SA.a, k0[q], qf[q]);
                mfma_acc(SA.b, k0[KS + q], qf[q]);
            }
            if (pc.nfull == 0) mask_stage(SA, 0);
            float t = fmaxf(SA.a[0], SA.b[0]);
#pragma unroll
            for (int i = 1; i < 16; ++i) t = fmaxf(fmaxf(t, SA.a[i]), SA.b[i]);
#endif
            maybe_rescale(half_max(t));
            // K fragments of the first half of stage 1, V fragments of the first half of stage 0 (what a step expects)
#pragma unroll
            for (int q = 0; q < NKF; ++q) kf[q] = lds_k(s1, q);
#pragma unroll
            for (int i = 0; i < NVF; ++i) vf[i] = lds_v(s0, i / DB, i % DB);
        }
        HG_TP(piece_no, 1);
        HG_TC_BEGIN();

        // One pipeline step.  On entry: Scur = scores of stage j, kf = K fragments 0..3 of stage j+1, vf = V fragments
        // of keys 0..15 of stage j.  On exit the same with j+1, Snext = scores of stage j+1 (of whatever follows in
        // the ring when j is the piece's last stage: those scores are dropped).  The step's copy goes into the slot
        // whose stage was consumed in the step before.  slot = (g0 + j) % NS.
        // `plain` steps (the groups of NS) score full stages only and never reach the end of a piece: no mask, no
        // clearing, no look-up of a piece, no branch that would let the compiler move work out of its gap.
        // The body of a step is one basic block (a branch inside it lets the compiler move work out of its gap): the
        // steps outside the groups of NS apply the mask to every stage they score (it changes nothing on a full one).
        auto step_body = [&](int j, int slot, STile& Scur, STile& Snext, auto masked) -> float {
            constexpr bool kMasked = decltype(masked)::value;
            uintx4 pb[KT / 16];
            float tmax;
            const int slot1 = (slot + 1) & (NS - 1), slot2 = (slot + 2) & (NS - 1);
#if HG_WIDE_D == 128
#include "prefix_wide_step.inc"
#else
#include "prefix_wide_step_d64.inc"
#endif
            return tmax;
        };
        // kind 1: a step of a group of NS that is not the piece's last; 0: a step of the last group.
        auto step = [&](int j, int slot, STile& Scur, STile& Snext, auto kind) {
            constexpr int kKind = decltype(kind)::value;
            __builtin_amdgcn_s_waitcnt(kStepWait);    // own copies of the next two stages have landed
            __builtin_amdgcn_s_barrier();             // ... everyone's, and everyone has finished the step before
            if (kKind == 1) {
                maybe_rescale(step_body(j, slot, Scur, Snext, std::false_type{}));
                cursor_step();
            } else {
                if (j == zstep) clear_partial_v();
                const float tmax = step_body(j, slot, Scur, Snext, std::true_type{});
                if (j + 1 < pc.nst) maybe_rescale(tmax);
                cursor_advance();
            }
        };

        if (idle) {
            // nothing to multiply (blocks of <= 224 rows): this wavefront keeps its share of the copies going and meets
            // the others at every barrier
            for (int j = 0; j < pc.nst; ++j) {
                __builtin_amdgcn_s_waitcnt(kStepWait);
                __builtin_amdgcn_s_barrier();
                if (j == zstep) clear_partial_v();
                issue_stage((j + NS - 1) & (NS - 1));
            }
        } else {
            // Whole groups of NS steps at compile-time slots (a piece starts at slot 0: the stream pads every piece to
            // a multiple of NS stages) as long as every stage they score is a full one, which leaves at least the
            // piece's last group to the steps below; the copy cursor reaches the end of its piece only in a piece's
            // last group, so these steps never have to look a piece up.
            int j = 0;
            for (; j + NS < pc.nfull; j += NS) {
#pragma unroll
                for (int u = 0; u < NS; u += 2) {
                    step(j + u, u, SA, SB, std::integral_constant<int, 1>{});
                    step(j + u + 1, u + 1, SB, SA, std::integral_constant<int, 1>{});
                }
            }
            // The rest of the piece (1 .. NS + 1 steps: its last group, and one step more when the stage after a complete
            // group is the partial one), at compile-time slots too: a chain that ends at the first step beyond the
            // piece.  These steps mask every stage they score (it changes nothing on a full one) and may move the copy
            // cursor to the next piece.
            const int rest = pc.nst - j;
            auto tail = [&](auto self, auto uc) -> void {
                constexpr int u = decltype(uc)::value;
                if constexpr (u < NS + 1) {
                    if (u < rest) {
                        if constexpr (u % 2 == 0) step(j + u, u & (NS - 1), SA, SB, std::integral_constant<int, 0>{});
                        else step(j + u, u & (NS - 1), SB, SA, std::integral_constant<int, 0>{});
                        self(self, std::integral_constant<int, u + 1>{});
                    }
                }
            };
            tail(tail, std::integral_constant<int, 0>{});
        }
        // ... and its padding: steps that only keep the stream going (the slots of the padding stay unused)
        for (int j = pc.nst; j & (NS - 1); ++j) {
            __builtin_amdgcn_s_barrier();
            issue_stage((j + NS - 1) & (NS - 1));
        }
        HG_TC_END(piece_no);
        HG_TP(piece_no, 2);

        // ---- the next piece's Q is requested before this piece's results are stored ---------------------------------------
        // (what is stored after the request is counted, see store_piece; the marks of empty parts and the results of
        // pieces without keys go out before it)
        const WidePiece done = pc;
        const kargs_ptr k = kargs();       // one look at the arguments for the whole boundary
        if (done.last_in_col) mark_rest_empty(k, done);
        const bool more = next_piece(k);
        if (piece_no == 0) HG_T(19);
        if (more) load_q(k, row_ctx(k, pc));
        if (piece_no == 0) HG_T(20);
        // a wavefront whose 32 rows all exist issues exactly kStoresPerPiece stores below; any other drains everything
        qkind = (!idle && done.row0 + w * 32 + 32 <= done.nrows) ? kQAfterStores : kQDrain;
        store_piece(k, done, idle);
        HG_TP(piece_no, 3);
        ++piece_no;
        if (!more) break;
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);   // the copies still in flight land before the ring is released
    HG_T(15);
}

#if defined(HG_TRACE) && HG_WIDE_D == 128
}  // namespace hg
// Copies the phase time stamps of the most recent prefix_kernel_wide launches to `out` (HOST, 256 * 32 values) after
// synchronising the device; present only in a -DHG_TRACE build.
extern "C" int hg_debug_read_wide_trace(unsigned long long* out) {
    if (hipDeviceSynchronize() != hipSuccess) return HG_ERR_HIP;
    return hipMemcpyFromSymbol(out, HIP_SYMBOL(hg::hg_wide_trace), sizeof(unsigned long long) * 256 * hg::kTraceSlots) == hipSuccess
               ? HG_OK : HG_ERR_HIP;
}
namespace hg {
#endif

#if HG_WIDE_D == 128
// Work partition of the persistent kernel for a level (host side).  Returns false when the level does not fit
// (more than max_parts partial results per row would be needed).  A stage is 32 keys at D = 128 and 64 keys at D = 64.
bool plan_prefix_wide(const LevelDev& lv, int Hkv, int G, int D, int max_parts, int slots_per_xcd, WidePlan* out) {
    if (D != 128 && D != 64) return false;
    const int KT = D == 128 ? 32 : 64;
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
    if (ncols >= (1LL << 20) || ncols * p.n_c >= (1LL << 31)) return false;    // the kernel walks the space with 32-bit indices
    p.ncols = (int)ncols;
    const long long total = ncols * p.n_c;
    const int nteams = 8 * p.tpx;
    long long q = (total + nteams - 1) / nteams;
    if (q >= 64) q = (q + NS - 1) / NS * NS;                // long ranges: whole groups of NS stages
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
    p.mode = 0;
    // Equal ranges give every team the same number of stages but may cut a team's range at a column boundary, and a
    // workgroup pays a fixed price per piece (its Q tile, the first products outside the pipeline, the result stores:
    // about kPieceCost stages).  When pieces are short that price decides: then ranges aligned to the columns win.
    // cost = most (stages + kPieceCost * pieces) any team has.
    {
        constexpr long long kPieceCost = 4;
        long long pieces0 = 1;
        for (int t = 0; t < nteams; ++t) {                   // exact: columns touched by [t q, (t+1) q)
            const long long lo = (long long)t * q, hi = std::min<long long>(lo + q, total);
            if (lo >= hi) break;
            pieces0 = std::max<long long>(pieces0, (hi - 1) / p.n_c - lo / p.n_c + 1);
        }
        const long long cost0 = q + kPieceCost * pieces0;
        long long cost1, np1;
        if (ncols <= nteams) {
            const long long nt_min = nteams / ncols;                      // teams of the column with the fewest
            np1 = (nteams + ncols - 1) / ncols;
            cost1 = (p.n_c + nt_min - 1) / nt_min + kPieceCost;
        } else {
            const long long cols = (ncols + nteams - 1) / nteams;
            np1 = 1;
            cost1 = cols * (p.n_c + kPieceCost);
        }
        if (cost1 < cost0 && np1 <= max_parts && np1 <= p.n_c) {   // (a column has at least one stage per team)
            p.mode = 1;
            np = (int)np1;
        }
    }
    if (q >= (1LL << 30)) return false;
    p.quota = (int)q;
    p.nparts = np;
    // Equal ranges, some with a column boundary inside and some without: the teams with a boundary finish later by what
    // a second piece costs.  Ranges of equal cost instead (cost = stages + kWideBoundaryCost per boundary inside): the
    // smallest cost C for which the teams, each taking the longest range that costs at most C, cover the space.
    if (p.mode == 0 && nteams <= kWideMaxTeams) {
        const long long nc = p.n_c, kappa = kWideBoundaryCost;
        auto end_of = [&](long long a, long long C) {      // the largest b <= total with (b - a) + kappa * boundaries inside (a, b) <= C
            long long best = a + 1;
            const long long m0 = a / nc * nc;
            for (long long k = 0; C - kappa * k >= 1; ++k) {
                const long long mk = k == 0 ? a : m0 + k * nc;            // k boundaries lie inside when b > m_k
                const long long b = std::min({m0 + (k + 1) * nc, a + C - kappa * k, total});
                if (b > mk) best = std::max(best, b);
                if (mk >= total) break;
            }
            return std::min(best, total);
        };
        auto covers = [&](long long C) {
            long long a = 0;
            for (int t = 0; t < nteams && a < total; ++t) a = end_of(a, C);
            return a >= total;
        };
        int with = 0, without = 0;
        long long cost0 = 0;
        for (int t = 0; t < nteams; ++t) {
            const long long lo = (long long)t * q, hi = std::min<long long>(lo + q, total);
            if (lo >= hi) break;
            const long long inner = (hi - 1) / nc - lo / nc;
            (inner ? with : without) += 1;
            cost0 = std::max(cost0, hi - lo + kappa * inner);
        }
        if (with && without) {
            long long lo = (total + nteams - 1) / nteams, hi = cost0;       // covers(hi) holds: equal ranges cost at most cost0
            while (lo < hi) {
                const long long mid = (lo + hi) / 2;
                if (covers(mid)) hi = mid;
                else lo = mid + 1;
            }
            if (hi < cost0) {
                WidePlan w = p;
                long long a = 0;
                int col = -1, in_col = 0, np2 = 1;
                for (int t = 0; t <= nteams; ++t) w.starts[t] = (int)total;
                for (int t = 0; t < nteams && a < total; ++t) {
                    const long long b = end_of(a, hi);
                    w.starts[t] = (int)a;
                    for (long long c = a / nc; c <= (b - 1) / nc; ++c) {       // the pieces of this team, column by column
                        if ((int)c != col) { col = (int)c; in_col = 0; }
                        if (c == a / nc) w.first_part[t] = in_col;
                        ++in_col;
                        np2 = std::max(np2, in_col);
                    }
                    a = b;
                }
                if (np2 <= max_parts) {
                    w.mode = 2;
                    w.nparts = np2;
                    w.quota = (int)hi;      // (the cost bound; not a length in this mode)
                    p = w;
                }
            }
        }
    }
    *out = p;
    return true;
}

#endif

#if HG_WIDE_D == 128
hipError_t launch_prefix_wide(const PrefixArgs& a, int D, hipStream_t s) {
    if (D == 64) return launch_prefix_wide_d64(a, s);
#else
hipError_t launch_prefix_wide_d64(const PrefixArgs& a, hipStream_t s) {
#endif
    static bool attr_set[64] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 64 && !attr_set[dev]) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&HG_WIDE_KERNEL), hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set[dev] = true;
    }
    HG_WIDE_KERNEL<<<8 * a.wide.slots, 64 * NW, LDS_BYTES, s>>>(a);
    return hipGetLastError();
}

}  // namespace hg
