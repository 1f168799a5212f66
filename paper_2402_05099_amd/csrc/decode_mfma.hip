// Suffix attention on the matrix cores (Sec. 3.2, last paragraph; App. B with num_queries >= 1), D = 64 or 128, packed
// or paged suffix rows.  The per-sequence part of Hydragen is a matrix-vector product only while one KV head serves one
// query row; with grouped-query attention and with several queries per sequence a KV head serves R = nq * G rows,
// and the vector-ALU kernel (decode.hip) then pays R dot products per key and, across queries, re-reads the
// suffix.  Here a work item is (sequence, KV head, 32-row tile of the R rows, key chunk): every K/V row is read
// once and multiplied on v_mfma_f32_32x32x16_bf16 exactly as in the shared-block kernels (transposed products
// S^T = K Q^T, O^T += V^T P^T, a lane owns one query row, lazy rescaling); rows past R idle in the tile, which costs
// nothing because the kernel is bound by HBM, not by the matrix cores.
//
// A workgroup is ONE wavefront that takes a few consecutive work items and streams them through a ring of NS
// 16 KiB slots private to it: per item one Q element (the query tile) and then its K/V stages of 32 keys, copied
// HBM -> LDS by global_load_lds_dwordx4 with the same XOR swizzles as prefix_wide.hip, always NS-1 elements ahead
// of the one being consumed, across item boundaries.  The copies are issued from inline asm and waited for with
// counted s_waitcnt vmcnt (the compiler would otherwise drain every copy before each LDS read), so the kernel
// contains no vector load that the compiler can see: lengths and offsets come through scalar loads.  No barrier
// anywhere.  Four such wavefronts share a CU (NS = 2: 32 KiB of LDS each).
//
// Several queries per sequence: row r of a sequence's R rows is (query t, head g) = (r / G, r % G); query t sees
// suffix rows [0, length - (nq-1-t)), applied as a per-lane bound on the key index in the stages that reach it.
//
// FP8: the suffix rows are 8-bit E4M3 codes (one fp32 scale per tensor; not in the paper).  A K/V ring element is then
// 4 KiB + 4 KiB of codes (half the copy instructions).  Fragments are read as 8 bytes of codes and expanded in
// registers (v_cvt_scalef32_pk_bf16_fp8, exact: every E4M3 value is a bf16 value): K rows directly, V^T through
// ds_read_b64_tr_b8, the 8-bit transposing read.  Products, masks and softmax are the same code.  The K scale
// multiplies the softmax scale, the V scale the final normalisation.  16 KiB of LDS per wavefront (the ring alone).
#include "hg_internal.h"
#include "prefix_common.h"

#pragma clang diagnostic ignored "-Winline-asm"

namespace hg {

namespace {

constexpr int KT = 32;                  // keys per stage
constexpr float TAU = 8.0f;             // lazy-rescale threshold, log2 units

// Sizes that follow from the head dimension, and the XOR swizzles of the 16-byte chunks of a bf16 row in LDS (applied
// on the global side of the copies).  D = 128: a row is 256 bytes, one period of the 64 banks: K (and Q) chunk ^ row % 16
// makes the 16 rows of a ds_read_b128 pass distinct, V chunk ^ 4 (row % 4) separates the 4 rows of a transposing read.
// D = 64: a row is half a period, so consecutive rows already differ; K chunk ^ (row / 2) % 8, V chunk ^ 4 ((row / 2) % 2).
template <int D>
struct Geo {
    static_assert(D == 64 || D == 128, "head dimension");
    static constexpr int KS = D / 16;              // MFMA k-steps of the score product
    static constexpr int DB = D / 32;              // 32-row blocks of O^T
    static constexpr int CPR = D / 8;              // 16-byte chunks per bf16 row
    static constexpr int RPI = 64 / CPR;           // rows one copy instruction covers
    static constexpr int CPS = KT / RPI;           // copy instructions per stage and tensor
    static constexpr int ROWB = D * 2;             // bytes per bf16 row
    static constexpr int STB = KT * ROWB;          // bytes per stage and tensor
    static __device__ __forceinline__ int kswz(int row) { return D == 128 ? row % 16 : (row >> 1) & 7; }
    static __device__ __forceinline__ int vswz(int row) { return D == 128 ? 4 * (row % 4) : 4 * ((row >> 1) & 1); }
};

typedef unsigned uintx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ unsigned pack_pair(float lo, float hi) {
    floatx2 f = {lo, hi};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(f, bf16x2));
}

extern __shared__ __attribute__((aligned(1024))) unsigned char dm_smem[];

// s_waitcnt vmcnt(n) alone (lgkmcnt and expcnt untouched): vmcnt is split over bits [3:0] and [15:14]
template <int N>
__device__ __forceinline__ void wait_vm() {
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

}  // namespace

// PAGED: the suffix rows live in a page pool and are found through a page table (a.pg); rows are then logical rows of
// the sequence, a stage is 32 aligned logical rows and is never shifted, and the four rows of one copy instruction
// lie in one page (pages hold a power of two >= 16 rows), so a copy still has one scalar base.
// SEG: the key range of sequence b is the block of level a.lv[0] that covers b (the non-decomposed comparison walks
// the shared blocks per sequence); every query of the sequence sees all of it.
// TR: query rows per tile.  32: v_mfma_f32_32x32x16_bf16, a lane owns row l % 32 and half of a stage's keys.  16 (when a
// KV head serves at most 16 rows of a sequence): v_mfma_f32_16x16x32_bf16, a lane owns row l % 16 and a quarter of
// the keys; half the matrix work, half the softmax arithmetic and half the registers per stage.
template <int D, int NS, bool PAGED, bool SEG, bool FP8 = false, int TR = 32>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(2))) void decode_mfma_kernel(DecodeArgs a) {
    static_assert(TR == 32 || TR == 16, "query rows per tile");
    using G_ = Geo<D>;
    constexpr int KS = G_::KS, DB = G_::DB, CPR = G_::CPR, RPI = G_::RPI, CPS = G_::CPS, ROWB = G_::ROWB, STB = G_::STB;
    static_assert(NS >= 2 && (NS - 1) * 2 * CPS <= 63, "the copies in flight must fit the vmcnt counter");
    static_assert(!(FP8 && SEG), "shared levels are bf16");
    static_assert(!FP8 || D == 128, "8-bit rows: D = 128 only");
    // bf16: ring slot n holds K (or Q) at n * STB and V at (NS + n) * STB.  FP8: ring slot n holds the K codes at
    // n * STB and the V codes at n * STB + STB / 2 (a Q element fills the slot).
    constexpr int ES = FP8 ? 1 : 2;                // bytes per cache element
    constexpr int CPRG = D * ES / 16;              // 16-byte chunks per cache row
    constexpr int RPIG = 64 / CPRG;                // cache rows one copy instruction covers
    constexpr int CPSG = KT / RPIG;                // copy instructions per stage and tensor
    constexpr int QOPS = TR / RPI, KVOPS = 2 * CPSG;    // copy instructions per ring element
    constexpr int VSLOT = FP8 ? STB / 2 : NS * STB;   // from a ring element's K part to its V part
    unsigned char* const smem = dm_smem;
    const int l = threadIdx.x, lq = l & 31, hl = l >> 5;
    const int ln = l & 15, lg = l >> 4;            // 16-row tiles: row of the tile and lane group (quarter of the keys)
    const int lrw = TR == 16 ? ln : lq;            // this lane's row of the tile
    const int R = a.nq * a.G;
    const int RT = (R + TR - 1) / TR;
    const int item0 = blockIdx.x * a.ipw;
    const int item1 = min(item0 + a.ipw, a.items);

    // lengths and offsets are read through the constant address space: nothing writes them while the kernel runs, and
    // the compiler then keeps these loads on the scalar unit (a vector load here would make it wait for vmcnt(0),
    // which drains every copy in flight)
    typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;
    const const_i32_ptr lengths_c = (const_i32_ptr)(uintptr_t)a.lengths;
    const const_i32_ptr offsets_c = (const_i32_ptr)(uintptr_t)a.offsets;
    const const_i32_ptr table_c = (const_i32_ptr)(uintptr_t)a.pg.table;
    const const_i32_ptr seq_off_c = (const_i32_ptr)(uintptr_t)a.lv[0].seq_off;
    const const_i32_ptr kv_off_c = (const_i32_ptr)(uintptr_t)a.lv[0].kv_off;

    // One work item: (sequence b, key chunk c, 32-row tile rt, KV head kvh), adjacent items on adjacent KV heads.
    // Everything here is wavefront-uniform.
    struct Item {
        int b, c, rt, kvh;
        int off, count;      // first suffix row of the sequence in Ks/Vs; suffix rows the newest query sees
        int ks, ke;          // absolute rows [ks, ke) of this item's keys (empty: ks >= ke)
        int kwin, nst;
    };
    // (b, c, rt, kvh) of item i; integer division runs on the vector unit, readfirstlane brings the (uniform) results
    // back to scalar registers.  Used once per wavefront: the cursors then step from item to item.
    auto index_of = [&](int i, Item& it) {
        int u = i;
        it.kvh = __builtin_amdgcn_readfirstlane(u % a.Hkv); u = __builtin_amdgcn_readfirstlane(u / a.Hkv);
        it.rt = __builtin_amdgcn_readfirstlane(u % RT); u = __builtin_amdgcn_readfirstlane(u / RT);
        it.c = __builtin_amdgcn_readfirstlane(u % a.nchunks);
        it.b = __builtin_amdgcn_readfirstlane(u / a.nchunks);
    };
    auto next_index = [&](Item& it) {
        if (++it.kvh == a.Hkv) {
            it.kvh = 0;
            if (++it.rt == RT) {
                it.rt = 0;
                if (++it.c == a.nchunks) { it.c = 0; ++it.b; }
            }
        }
    };
    // key range of the item whose index fields are set
    auto range_of = [&](Item& it) {
        if (SEG) {
            // rows [begin, begin + count) of the block that covers sequence b: the g with seq_off[g] <= b < seq_off[g+1]
            int begin = 0, count = a.lv[0].max_rows;
            if (seq_off_c != nullptr) {
                int lo = 0, hi = a.lv[0].n_blocks;
                while (lo < hi) {
                    const int mid = (lo + hi) >> 1;
                    if (seq_off_c[mid + 1] <= it.b) lo = mid + 1;
                    else hi = mid;
                }
                count = 0;
                if (lo < a.lv[0].n_blocks && seq_off_c[lo] <= it.b) {
                    begin = kv_off_c[lo];
                    count = max(min(kv_off_c[lo + 1] - begin, a.lv[0].max_rows), 0);
                }
            }
            it.count = __builtin_amdgcn_readfirstlane(count);
            it.off = __builtin_amdgcn_readfirstlane(begin);
        } else {
            it.count = __builtin_amdgcn_readfirstlane(max(min(lengths_c[it.b], a.max_len), 0));
            it.off = PAGED ? 0 : __builtin_amdgcn_readfirstlane(offsets_c[it.b]);
        }
        const int lo = it.c * a.chunk, hi = min(lo + a.chunk, it.count);
        it.ks = __builtin_amdgcn_readfirstlane(it.off + lo);
        it.ke = __builtin_amdgcn_readfirstlane(it.off + max(hi, lo));
        it.kwin = PAGED ? 0x3fffffff : max(it.ke - KT, 0);   // paged: stages stay where they are, rows past ke are masked
        it.nst = (it.ke - it.ks + KT - 1) / KT;
    };

    // ---- HBM -> LDS copies -------------------------------------------------------------------------------------------
    // A wavefront streams a sequence of ring elements: for every non-empty item one Q element (the 32 query rows of
    // the tile, 8 copy instructions) followed by its K/V stages (32 keys, 16 copy instructions), element n in slot
    // n % NS, NS-1 elements ahead of the one being consumed, across item boundaries.  All copies are 1 KiB
    // global_load_lds_dwordx4 issued from inline asm (the compiler must not see them: it would drain them all before
    // every LDS read) and are waited for with counted s_waitcnt vmcnt; loads return in order, so "at most the copies
    // of the younger elements are outstanding" means the current element has landed.  The output stores in between
    // also count in vmcnt and may complete out of order with loads: they can only make a wait longer, never shorter.
    //
    // K/V stage t of an item holds rows [k0c, k0c + 32), k0c = min(ks + 32 t, kwin), kwin = max(ke - 32, 0): a partial
    // last stage re-reads the 32 rows that end the range (rows before ks belong to an earlier chunk or sequence and
    // are masked), so every copy has the same shape; row i of a stage is a key of it iff ks + 32 t <= k0c + i < ke.
    // 16-byte chunks are XOR-swizzled on the global side (K and Q: chunk ^ row % 16, V: chunk ^ 4 (row % 4)).
    const unsigned rstride_b = (unsigned)a.Hkv * D * ES;
    const int lrow = l / CPR, sch = l % CPR;
    const int lrowg = l / CPRG, schg = l % CPRG;   // cache row within a copy instruction and 16-byte chunk of this lane
    const unsigned ldsb = (unsigned)(uintptr_t)HG_LDS(smem);
    // Base pointers and LDS addresses are wavefront-uniform; readfirstlane puts them in scalar registers even where
    // the compiler computed them with vector instructions (64-bit multiplies).  Done once per ring element: a copy
    // is then s_add, s_mov m0 and the load.
    auto scalar_ptr = [&](const unsigned char* vbase) -> const unsigned char* {
        const uint64_t pv = reinterpret_cast<uint64_t>(vbase);
        // readfirstlane returns a signed int: both halves go through uint32_t so that the low half is not sign-extended
        const uint32_t plo = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)pv);
        const uint32_t phi = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(pv >> 32));
        return reinterpret_cast<const unsigned char*>(((uint64_t)phi << 32) | (uint64_t)plo);
    };
    auto copy16 = [&](const unsigned char* sbase, unsigned voff, unsigned lds_dst) {
        // nt: the rows are used once (streaming hint; measured 5.4 -> 5.9 TB/s on long suffixes)
        asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1 nt" ::"v"(voff), "s"(sbase), "s"(lds_dst) : "memory", "m0");
    };

    // ---- LDS fragment addresses (relative to the slot), as in prefix_wide.hip ------------------------------------------
    unsigned kaddr[KS], qaddr[KS];     // K fragments of a stage, Q fragments of a tile (bf16: the same addresses)
#pragma unroll
    for (int s = 0; s < KS; ++s) kaddr[s] = qaddr[s] = (unsigned)(lq * ROWB + (((2 * s + hl) ^ G_::kswz(lq)) * 16));
    // FP8: the 8 codes of K row lq, columns 16 s + 8 hl .. +7: rows lie in copy order (row r at (r/8) KiB + (r%8) 128 B),
    // their 16-byte chunks XOR-swizzled by (r/2) % 8 on the global side so that 16 consecutive lanes hit 32 different banks
    if constexpr (FP8) {
#pragma unroll
        for (int s = 0; s < KS; ++s)
            kaddr[s] = (unsigned)((lq >> 3) * 1024 + (lq & 7) * 128 + ((s ^ ((lq >> 1) & 7)) * 16) + 8 * hl);
    }
    // 16-row tiles.  K (A operand, 16 keys x 32 columns per MFMA) and Q (B operand, 32 columns x 16 rows): lane (lg, ln)
    // holds row ln of the 16-key group (of the tile), columns 32 s + 8 lg .. +7: 16-byte chunk 4 s + lg of that row.
    // V^T (A operand, 16 columns x 32 keys): k-slot e of lane group lg stands for key 16 (e / 4) + 4 lg + e % 4, the key
    // whose score this lane holds as element e % 4 of score tile e / 4; lane s of a group points ds_read_b64_tr_b16 at
    // key 4 lg + s / 4, columns 16 db + 4 (s % 4) .. +3, and receives column 16 db + s of the group's four keys.
    constexpr int KS16 = D / 32, DB16 = D / 16;
    unsigned kaddr16[2][KS16], qaddr16[KS16], vaddr16[DB16];
    if constexpr (TR == 16) {
#pragma unroll
        for (int s = 0; s < KS16; ++s) {
            qaddr16[s] = (unsigned)(ln * ROWB + (((4 * s + lg) ^ G_::kswz(ln)) * 16));
#pragma unroll
            for (int kg = 0; kg < 2; ++kg)
                kaddr16[kg][s] = (unsigned)((16 * kg + ln) * ROWB + (((4 * s + lg) ^ G_::kswz(16 * kg + ln)) * 16));
        }
        const int vrow = 4 * lg + (ln >> 2), q4 = ln & 3;
#pragma unroll
        for (int db = 0; db < DB16; ++db)
            vaddr16[db] = (unsigned)(vrow * ROWB + (((2 * db + (q4 >> 1)) ^ G_::vswz(vrow)) * 16) + (q4 & 1) * 8);
        if constexpr (FP8) {
            // codes, rows in copy order: K row ln of key group kg, columns 32 s + 8 lg .. +7 (8 bytes); V^T through
            // ds_read_b64_tr_b8 as for 32-row tiles, lane s of a group pointing at the key of k-slot s / 2
            // (16 (j / 4) + 4 lg + j % 4) and columns 16 db + 8 (s % 2) .. +7; V chunks swizzled by (r/2) % 2 + 2 ((r/16) % 2)
#pragma unroll
            for (int s = 0; s < KS16; ++s)
#pragma unroll
                for (int kg = 0; kg < 2; ++kg) {
                    const int row = 16 * kg + ln;
                    kaddr16[kg][s] = (unsigned)((row >> 3) * 1024 + (row & 7) * 128 + (((2 * s + (lg >> 1)) ^ ((row >> 1) & 7)) * 16) + 8 * (lg & 1));
                }
            const int j = ln >> 1, pp = ln & 1;
            const int row = 16 * (j >> 2) + 4 * lg + (j & 3);
            const int fsw = ((row >> 1) & 1) | (((row >> 4) & 1) << 1);
#pragma unroll
            for (int db = 0; db < DB16; ++db)
                vaddr16[db] = (unsigned)((row >> 3) * 1024 + (row & 7) * 128 + ((db ^ fsw) * 16) + 8 * pp);
        }
    }
    // FP8, V^T: ds_read_b64_tr_b8 works on groups of 16 lanes: every lane supplies the address of 8 bytes, and lane i
    // of the group receives, as byte j, byte i % 8 of the piece that lane 2 j + i / 8 of the group pointed at.  So
    // lane s of a group points at the V codes of key 8 (j / 4) + 4 hl + j % 4 (j = s / 2, the key of k-slot j), columns
    // 16 g1 + 8 (s % 2) .. +7 of the 32-column block: lane i then holds column 16 g1 + i of the 8 keys in k-slot order.
    // Rows lie in copy order (row r at (r / 8) KiB + (r % 8) 128 B); 16-byte chunks are XOR-swizzled on the global
    // side by (r / 2) % 2 + 2 ((r / 8) % 2), which spreads the 8 rows of a read over all banks.
    unsigned vaddr8[DB];
    if constexpr (FP8) {
        const int sg = l & 15, g1 = (l >> 4) & 1;
        const int j = sg >> 1, pp = sg & 1;
        const int row = 8 * (j >> 2) + 4 * hl + (j & 3);        // + 16 tt
        const int fsw = ((row >> 1) & 1) | (((row >> 3) & 1) << 1);
#pragma unroll
        for (int db = 0; db < DB; ++db)
            vaddr8[db] = (unsigned)((row >> 3) * 1024 + (row & 7) * 128 + (((2 * db + g1) ^ fsw) * 16) + 8 * pp);
    }
    unsigned vaddr[DB];
    {
        const int i16 = l & 15, g1 = (l >> 4) & 1;
        const int keyq = 4 * hl + (i16 >> 2);
        const int fv = G_::vswz(keyq);
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const int chunk = 4 * db + 2 * g1 + ((i16 & 3) >> 1);
            vaddr[db] = (unsigned)(keyq * ROWB + ((chunk ^ fv) * 16) + (i16 & 1) * 8);   // relative to the V stage
        }
    }

    // ---- producer: runs NS-1 elements ahead of the consumer ----------------------------------------------------------------
    int p_item = item0, p_el = -1;     // next element to issue: element -1 of an item is its Q tile
    int n_issued = 0;                  // elements issued so far (element n lives in slot n % NS)
    int pending = 0;                   // copy instructions of the elements issued and not yet consumed
    Item pit{};
    unsigned voffK[CPS], voffV[CPS], voffQ[CPS];   // lane offsets of the producer's item: K/V stage rows, Q tile rows
    int voff_clamp = -1, voff_rt = -1;             // the row clamp / row tile these offsets were computed for
    // position the producer on the next item that has keys and set up its lane offsets
    auto p_load = [&](bool first) {
        if (p_item >= item1) return;
        if (first) index_of(p_item, pit);
        else next_index(pit);
        while (true) {
            range_of(pit);
            if (pit.ks < pit.ke) break;
            if (++p_item >= item1) return;
            next_index(pit);
        }
        const int rowclamp = PAGED ? KT - 1 : min(pit.ke - 1 - pit.kwin, KT - 1);   // < 31 only when the range ends before row 32 of the tensor
        if (rowclamp != voff_clamp) {
            voff_clamp = rowclamp;
#pragma unroll
            for (int i = 0; i < CPSG; ++i) {
                const int srow = i * RPIG + lrowg;
                const unsigned ro = (unsigned)min(srow, rowclamp) * rstride_b;
                if (FP8) {
                    // codes land in copy order (lane l of copy i holds row 8i + l/8), chunks swizzled for the fragment reads
                    voffK[i] = ro + (unsigned)((schg ^ ((srow >> 1) & 7)) * 16);
                    voffV[i] = ro + (unsigned)((schg ^ (((srow >> 1) & 1) | (((srow >> (TR == 16 ? 4 : 3)) & 1) << 1))) * 16);
                } else {
                    voffK[i] = ro + (unsigned)((sch ^ G_::kswz(srow)) * 16);
                    voffV[i] = ro + (unsigned)((sch ^ G_::vswz(srow)) * 16);
                }
            }
        }
        if (pit.rt != voff_rt) {
            voff_rt = pit.rt;
#pragma unroll
            for (int i = 0; i < QOPS; ++i) {
                const int srow = i * RPI + lrow;
                int r = pit.rt * TR + srow;                 // Q tile row i is query row rt*TR + i of (b, kvh); row 0 when past R
                if (r >= R) r = 0;
                voffQ[i] = (unsigned)((r / a.G) * a.Hq + r % a.G) * ROWB + (unsigned)((sch ^ G_::kswz(srow)) * 16);
            }
        }
    };
    auto produce_one = [&]() {
        p_item = __builtin_amdgcn_readfirstlane(p_item);
        p_el = __builtin_amdgcn_readfirstlane(p_el);
        n_issued = __builtin_amdgcn_readfirstlane(n_issued);
        pending = __builtin_amdgcn_readfirstlane(pending);
        if (p_item >= item1) return;
        const unsigned dst = (unsigned)__builtin_amdgcn_readfirstlane(ldsb + (unsigned)(n_issued % NS) * STB);
        if (p_el < 0) {
            const unsigned char* const qg = scalar_ptr(reinterpret_cast<const unsigned char*>(a.Q + ((int64_t)pit.b * a.nq * a.Hq + pit.kvh * a.G) * D));
#pragma unroll
            for (int i = 0; i < QOPS; ++i) copy16(qg, voffQ[i], dst + i * (RPI * ROWB));
            pending += QOPS;
        } else if (PAGED) {
            // logical rows r0 .. r0+31 of the sequence: copy i takes rows r0 + 4i .. +3, all in one page
            const int r0 = pit.ks + p_el * KT;
            const int shift = a.pg.shift, ps_mask = (1 << shift) - 1;
            const int64_t trow = (int64_t)pit.b * a.pg.stride;
            const int e0 = min(r0 >> shift, a.pg.stride - 1), e1 = min((r0 + KT / 2) >> shift, a.pg.stride - 1);
            const int pg0 = min(max(table_c[trow + e0], 0), a.pg.n_pages - 1);   // pages of rows r0.. and r0+16..
            const int pg1 = min(max(table_c[trow + e1], 0), a.pg.n_pages - 1);
#pragma unroll
            for (int i = 0; i < CPSG; ++i) {
                const int jr = r0 + i * RPIG;
                const int page = i < CPSG / 2 ? pg0 : pg1;
                const int64_t prow = ((int64_t)page << shift) + (jr & ps_mask);
                const int64_t goff = prow * rstride_b + (int64_t)pit.kvh * (D * ES);
                const unsigned char* const kg = scalar_ptr(reinterpret_cast<const unsigned char*>(a.Ks) + goff);
                const unsigned char* const vg = scalar_ptr(reinterpret_cast<const unsigned char*>(a.Vs) + goff);
                const unsigned back = (unsigned)(i * RPIG) * rstride_b;    // voffK/V count rows from the stage's first row
                copy16(kg, voffK[i] - back, dst + i * 1024);
                copy16(vg, voffV[i] - back, dst + VSLOT + i * 1024);
            }
            pending += KVOPS;
        } else {
            const int k0c = min(pit.ks + p_el * KT, pit.kwin);
            const int64_t goff = (int64_t)k0c * rstride_b + (int64_t)pit.kvh * (D * ES);
            const unsigned char* const kg = scalar_ptr(reinterpret_cast<const unsigned char*>(a.Ks) + goff);
            const unsigned char* const vg = scalar_ptr(reinterpret_cast<const unsigned char*>(a.Vs) + goff);
#pragma unroll
            for (int i = 0; i < CPSG; ++i) copy16(kg, voffK[i], dst + i * 1024);
#pragma unroll
            for (int i = 0; i < CPSG; ++i) copy16(vg, voffV[i], dst + VSLOT + i * 1024);
            pending += KVOPS;
        }
        ++n_issued;
        if (++p_el == pit.nst) {
            p_el = -1;
            ++p_item;
            p_load(false);
        }
    };
    // wait until at most `younger` copy instructions are outstanding (at most (NS-1) * KVOPS; more than six units: all)
    auto wait_for = [&](int younger) {
        constexpr int WU = QOPS < KVOPS ? QOPS : KVOPS;   // every element is a multiple of this many copies
        switch (younger / WU) {
            case 0: wait_vm<0>(); break;
            case 1: wait_vm<1 * WU>(); break;
            case 2: wait_vm<2 * WU>(); break;
            case 3: wait_vm<3 * WU>(); break;
            case 4: wait_vm<4 * WU>(); break;
            case 5: wait_vm<5 * WU>(); break;
            case 6: wait_vm<6 * WU>(); break;
            default: wait_vm<0>(); break;
        }
        asm volatile("" ::: "memory");
    };
    p_load(true);
#pragma nounroll
    for (int s = 0; s < NS - 1; ++s) produce_one();

    // ---- consumer ---------------------------------------------------------------------------------------------------------
    const float kscale = FP8 ? a.scale * a.k_scale : a.scale;   // raw scores are in units of the codes
    const float c2 = kscale * kLog2e;
    const float tau_raw = TAU / c2;
    int c_item = item0, c_el = -1, n_done = 0;
    Item cit{};
    // lane state of the consumer's item
    bool rv = false;
    int64_t qidx = 0;
    int vis_end = 0, causal_from = 0;
    bf16x8 qf[KS];
    floatx16 Oacc[DB];
    typedef float floatx4 __attribute__((ext_vector_type(4)));
    bf16x8 qf16[KS16];          // 16-row tiles
    floatx4 Oacc16[DB16];
    float m_used = -INFINITY;   // raw-score maximum the exponentials are taken against (-inf: no key seen yet)
    float mc = 0.f;             // m_used * c2, 0 while no key has been seen
    float lsum = 0.f;           // this lane's share of the row sum (unrounded exponentials)
#pragma unroll
    for (int s = 0; s < KS; ++s) qf[s] = __builtin_bit_cast(bf16x8, uintx4{0, 0, 0, 0});
#pragma unroll
    for (int i = 0; i < DB; ++i)
#pragma unroll
        for (int k = 0; k < 16; ++k) Oacc[i][k] = 0.f;
#pragma unroll
    for (int s = 0; s < KS16; ++s) qf16[s] = __builtin_bit_cast(bf16x8, uintx4{0, 0, 0, 0});
#pragma unroll
    for (int i = 0; i < DB16; ++i) Oacc16[i] = floatx4{0.f, 0.f, 0.f, 0.f};

    int lane_rt = -1, lane_tq = 0, lane_g = 0;   // (query, head in the group) of this lane's row, for row tile lane_rt
    auto lane_of = [&](const Item& it) {
        if (it.rt != lane_rt) {
            lane_rt = it.rt;
            const int r = it.rt * TR + lrw;   // this lane's row among the R rows of (b, kvh)
            rv = r < R;
            const int rr = rv ? r : 0;
            lane_tq = rr / a.G;
            lane_g = rr % a.G;
        }
        qidx = ((int64_t)it.b * a.nq + lane_tq) * a.Hq + it.kvh * a.G + lane_g;
        vis_end = it.off + it.count - (SEG ? 0 : a.nq - 1 - lane_tq);   // this lane's query sees absolute rows below vis_end
        causal_from = it.off + it.count - (SEG ? 0 : a.nq - 1);         // below this row every query sees every key
    };
    // position the consumer on the next item that has keys; items without keys get the empty part on the way
    auto c_load = [&](bool first) {
        if (c_item >= item1) return;
        if (first) index_of(c_item, cit);
        else next_index(cit);
        while (true) {
            range_of(cit);
            if (cit.ks < cit.ke) break;
            lane_of(cit);
            if (rv) {
                float* const Of = static_cast<float*>(a.out.O) + (int64_t)cit.c * a.out.part_stride_O + qidx * D;
                uint16_t* const Ob = static_cast<uint16_t*>(a.out.O) + (int64_t)cit.c * a.out.part_stride_O + qidx * D;
                constexpr int LPRW = 64 / TR;     // lanes that share a row: each writes every LPRW-th group of 4 columns
                const int lsub = TR == 16 ? lg : hl;
#pragma unroll
                for (int i = 0; i < D / (4 * LPRW); ++i) {
                    const int d = 4 * LPRW * i + 4 * lsub;
                    if (a.out.bf16) *reinterpret_cast<uint2*>(Ob + d) = make_uint2(0u, 0u);
                    else *reinterpret_cast<float4*>(Of + d) = make_float4(0.f, 0.f, 0.f, 0.f);
                }
                if (lsub == 0) a.out.LSE[(int64_t)cit.c * a.out.part_stride_L + qidx] = -INFINITY;
            }
            if (++c_item >= item1) return;
            next_index(cit);
        }
    };
    c_load(true);

    while (c_item < item1) {
        c_item = __builtin_amdgcn_readfirstlane(c_item);
        c_el = __builtin_amdgcn_readfirstlane(c_el);
        n_done = __builtin_amdgcn_readfirstlane(n_done);
        produce_one();          // refills the slot of the element consumed last (its fragment reads have completed)
        const unsigned char* const sb = smem + (n_done % NS) * STB;
        ++n_done;
        if (c_el < 0) {
            // Q element -> registers; fresh softmax state
            pending -= QOPS;
            wait_for(pending);
            lane_of(cit);
            if constexpr (TR == 16) {
#pragma unroll
                for (int s = 0; s < KS16; ++s) qf16[s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uintx4*>(sb + qaddr16[s]));
#pragma unroll
                for (int i = 0; i < DB16; ++i) Oacc16[i] = floatx4{0.f, 0.f, 0.f, 0.f};
            } else {
#pragma unroll
                for (int s = 0; s < KS; ++s) qf[s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uintx4*>(sb + qaddr[s]));
#pragma unroll
                for (int i = 0; i < DB; ++i)
#pragma unroll
                    for (int k = 0; k < 16; ++k) Oacc[i][k] = 0.f;
            }
            m_used = -INFINITY;
            mc = 0.f;
            lsum = 0.f;
            // the fragments must be in registers before a later copy may overwrite this slot
            if constexpr (TR == 16) {
#pragma unroll
                for (int s = 0; s < KS16; ++s) asm volatile("" : "+v"(qf16[s]));
            } else {
#pragma unroll
                for (int s = 0; s < KS; ++s) asm volatile("" : "+v"(qf[s]));
            }
            asm volatile("" ::: "memory");
        } else {
            pending -= KVOPS;
            wait_for(pending);
            unsigned char* const vstage = smem + (sb - smem) + VSLOT;   // the V part of this element
            const int key0 = cit.ks + c_el * KT;
            const int k0c = min(key0, cit.kwin);
            if (PAGED && key0 + KT > cit.ke) {
                // the rows past the range are a page's unwritten tail (or another page altogether): clear their V rows
                // in LDS, since their zero probabilities would still turn a NaN into a NaN in the second product
                const int nhi = cit.ke - key0;
                unsigned char* const vs = vstage;
                if constexpr (FP8) {   // codes in copy order: lane l of copy i holds row 8i + l/8; code 0 is 0.0
#pragma unroll
                    for (int i = 0; i < CPSG; ++i)
                        if (i * RPIG + lrowg >= nhi) *reinterpret_cast<uintx4*>(vs + i * 1024 + l * 16) = uintx4{0u, 0u, 0u, 0u};
                } else {
#pragma unroll
                    for (int i = 0; i < CPS; ++i) {
                        const int row = i * RPI + lrow;
                        if (row >= nhi) *reinterpret_cast<uintx4*>(vs + row * ROWB + sch * 16) = uintx4{0u, 0u, 0u, 0u};
                    }
                }
            }
            if (k0c != key0) {
                // The stage rows before its first key were re-read from below the range: they may lie in another
                // sequence's slot of the cache, possibly padding that was never written.  Their probabilities are
                // zero, but 0 * NaN is NaN in the second product: clear those V rows in LDS.
                const int nlo = key0 - k0c;
                unsigned char* const vs = vstage;
                if constexpr (FP8) {
#pragma unroll
                    for (int i = 0; i < CPSG; ++i)
                        if (i * RPIG + lrowg < nlo) *reinterpret_cast<uintx4*>(vs + i * 1024 + l * 16) = uintx4{0u, 0u, 0u, 0u};
                } else {
#pragma unroll
                    for (int i = 0; i < CPS; ++i) {
                        const int row = i * RPI + lrow;
                        if (row < nlo) *reinterpret_cast<uintx4*>(vs + row * ROWB + sch * 16) = uintx4{0u, 0u, 0u, 0u};
                    }
                }
            }
            if constexpr (TR == 16) {
                // S^T = K Q^T, two tiles of 16 keys: element i of tile kg is the score of stage row 16 kg + 4 lg + i
                floatx4 S4[2];
#pragma unroll
                for (int kg = 0; kg < 2; ++kg) S4[kg] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < KS16; ++s) {
#pragma unroll
                    for (int kg = 0; kg < 2; ++kg) {
                        uintx4 kv;
                        if constexpr (FP8) {
                            const unsigned __attribute__((ext_vector_type(2))) kc =
                                *reinterpret_cast<const unsigned __attribute__((ext_vector_type(2)))*>(sb + kaddr16[kg][s]);
                            kv[0] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(kc[0], 1.0f, false));
                            kv[1] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(kc[0], 1.0f, true));
                            kv[2] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(kc[1], 1.0f, false));
                            kv[3] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(kc[1], 1.0f, true));
                        } else {
                            kv = *reinterpret_cast<const uintx4*>(sb + kaddr16[kg][s]);
                        }
                        S4[kg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kv), qf16[s], S4[kg], 0, 0, 0);
                    }
                }
                if (k0c != key0 || key0 + KT > cit.ke || key0 + KT > causal_from) {
                    const int lo_i = key0 - k0c - 4 * lg, hi_i = min(cit.ke, vis_end) - k0c - 4 * lg;
#pragma unroll
                    for (int kg = 0; kg < 2; ++kg)
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int ri = 16 * kg + i;
                            if (ri < lo_i || ri >= hi_i) S4[kg][i] = -INFINITY;
                        }
                }
                float tmax = fmaxf(fmaxf(fmaxf(S4[0][0], S4[0][1]), fmaxf(S4[0][2], S4[0][3])),
                                   fmaxf(fmaxf(S4[1][0], S4[1][1]), fmaxf(S4[1][2], S4[1][3])));
                tmax = fmaxf(tmax, __shfl_xor(tmax, 16));      // the four lanes that share a row
                tmax = half_max(tmax);
                if (__any(tmax > m_used + tau_raw)) {
                    const float m_new = fmaxf(m_used, tmax);
                    const float alpha = (m_new == m_used) ? 1.0f : __builtin_amdgcn_exp2f((m_used - m_new) * c2);
                    m_used = m_new;
                    mc = (m_new == -INFINITY) ? 0.f : m_new * c2;
                    lsum *= alpha;
#pragma unroll
                    for (int i = 0; i < DB16; ++i)
#pragma unroll
                        for (int k = 0; k < 4; ++k) Oacc16[i][k] *= alpha;
                }
                // P^T as B operand: k-slot e of this lane is element e % 4 of tile e / 4
                float p[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    p[i] = __builtin_amdgcn_exp2f(fmaf(S4[i >> 2][i & 3], c2, -mc));
                    lsum += p[i];
                }
                const uintx4 pb = uintx4{pack_pair(p[0], p[1]), pack_pair(p[2], p[3]), pack_pair(p[4], p[5]), pack_pair(p[6], p[7])};
                // O^T += V^T P^T, 16 columns per MFMA
#pragma unroll
                for (int db = 0; db < DB16; ++db) {
                    const unsigned char* vp = vstage + vaddr16[db];
                    if constexpr (FP8) {
                        typedef int intx2 __attribute__((ext_vector_type(2)));
                        const intx2 vc = __builtin_amdgcn_ds_read_tr8_b64_v2i32((__attribute__((address_space(3))) intx2*)HG_LDS(vp));
                        uintx4 vv;
                        vv[0] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((unsigned)vc[0], 1.0f, false));
                        vv[1] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((unsigned)vc[0], 1.0f, true));
                        vv[2] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((unsigned)vc[1], 1.0f, false));
                        vv[3] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((unsigned)vc[1], 1.0f, true));
                        Oacc16[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vv), __builtin_bit_cast(bf16x8, pb), Oacc16[db], 0, 0, 0);
                    } else {
                        const shortx4 vlo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) shortx4*)HG_LDS(vp));
                        const shortx4 vhi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) shortx4*)HG_LDS(vp + 16 * ROWB));
                        const shortx8 vv = __builtin_shufflevector(vlo, vhi, 0, 1, 2, 3, 4, 5, 6, 7);
                        Oacc16[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vv), __builtin_bit_cast(bf16x8, pb), Oacc16[db], 0, 0, 0);
                    }
                }
#pragma unroll
                for (int db = 0; db < DB16; ++db) asm volatile("" : "+v"(Oacc16[db]));
                asm volatile("" ::: "memory");
            } else {
                // S^T = K Q^T
                floatx16 S;
    #pragma unroll
                for (int i = 0; i < 16; ++i) S[i] = 0.f;
    #pragma unroll
                for (int s = 0; s < KS; ++s) {
                    uintx4 kv;
                    if constexpr (FP8) {
                        const unsigned __attribute__((ext_vector_type(2))) kc =
                            *reinterpret_cast<const unsigned __attribute__((ext_vector_type(2)))*>(sb + kaddr[s]);
                        kv[0] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(kc[0], 1.0f, false));
                        kv[1] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(kc[0], 1.0f, true));
                        kv[2] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(kc[1], 1.0f, false));
                        kv[3] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(kc[1], 1.0f, true));
                    } else {
                        kv = *reinterpret_cast<const uintx4*>(sb + kaddr[s]);
                    }
                    S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kv), qf[s], S, 0, 0, 0);
                }
                // keys outside [key0, min(ke, vis_end)): stage rows before the stage's first key (window clamp), rows past
                // the range, and rows that this lane's query does not see yet
                if (k0c != key0 || key0 + KT > cit.ke || key0 + KT > causal_from) {
                    const int lo_i = key0 - k0c - 4 * hl, hi_i = min(cit.ke, vis_end) - k0c - 4 * hl;
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
                        for (int k = 0; k < 16; ++k) Oacc[i][k] *= alpha;
                }
                // P^T = 2^(S*c2 - m*c2), packed to bf16 in B-operand order (elements 8*tt .. 8*tt+7 are the k-slots of key half tt)
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
                        if constexpr (FP8) {
                            typedef int intx2 __attribute__((ext_vector_type(2)));
                            const unsigned char* vp = vstage + vaddr8[db] + tt * 2048;     // keys 16 tt ..: two copy blocks further
                            const intx2 vc = __builtin_amdgcn_ds_read_tr8_b64_v2i32((__attribute__((address_space(3))) intx2*)HG_LDS(vp));
                            uintx4 vv;
                            vv[0] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((unsigned)vc[0], 1.0f, false));
                            vv[1] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((unsigned)vc[0], 1.0f, true));
                            vv[2] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((unsigned)vc[1], 1.0f, false));
                            vv[3] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((unsigned)vc[1], 1.0f, true));
                            Oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vv), __builtin_bit_cast(bf16x8, pb[tt]), Oacc[db], 0, 0, 0);
                        } else {
                            const unsigned char* vp = vstage + vaddr[db] + tt * 16 * ROWB;
                            const shortx4 vlo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) shortx4*)HG_LDS(vp));
                            const shortx4 vhi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) shortx4*)HG_LDS(vp + 8 * ROWB));
                            const shortx8 vv = __builtin_shufflevector(vlo, vhi, 0, 1, 2, 3, 4, 5, 6, 7);
                            Oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vv), __builtin_bit_cast(bf16x8, pb[tt]), Oacc[db], 0, 0, 0);
                        }
                    }
                }
                // the accumulators depend on every fragment read of this step: once they are pinned here the reads have
                // completed, and the next produce_one() may overwrite the slot
    #pragma unroll
                for (int db = 0; db < DB; ++db) asm volatile("" : "+v"(Oacc[db]));
                asm volatile("" ::: "memory");
            }
        }
        if (++c_el == cit.nst) {
            // last stage of the item: write (O, LSE) of the part
            float lsub = lsum;
            if constexpr (TR == 16) lsub += __shfl_xor(lsub, 16);
            const float ltot = half_sum(lsub);
            if (rv && TR == 16) {
                float* const Of = static_cast<float*>(a.out.O) + (int64_t)cit.c * a.out.part_stride_O + qidx * D;
                uint16_t* const Ob = static_cast<uint16_t*>(a.out.O) + (int64_t)cit.c * a.out.part_stride_O + qidx * D;
                const float inv = ltot > 0.f ? (FP8 ? a.v_scale / ltot : 1.0f / ltot) : 0.f;
#pragma unroll
                for (int db = 0; db < DB16; ++db) {     // element i of block db is column 16 db + 4 lg + i of this lane's row
                    const int d = 16 * db + 4 * lg;
                    const float o0 = Oacc16[db][0] * inv, o1 = Oacc16[db][1] * inv, o2 = Oacc16[db][2] * inv, o3 = Oacc16[db][3] * inv;
                    if (a.out.bf16) *reinterpret_cast<uint2*>(Ob + d) = make_uint2(pack_bf16(o0, o1), pack_bf16(o2, o3));
                    else *reinterpret_cast<float4*>(Of + d) = make_float4(o0, o1, o2, o3);
                }
                if (lg == 0) a.out.LSE[(int64_t)cit.c * a.out.part_stride_L + qidx] = ltot > 0.f ? m_used * kscale + __logf(ltot) : -INFINITY;
            }
            if (rv && TR == 32) {
                float* const Of = static_cast<float*>(a.out.O) + (int64_t)cit.c * a.out.part_stride_O + qidx * D;
                uint16_t* const Ob = static_cast<uint16_t*>(a.out.O) + (int64_t)cit.c * a.out.part_stride_O + qidx * D;
                const float inv = ltot > 0.f ? (FP8 ? a.v_scale / ltot : 1.0f / ltot) : 0.f;    // a row that sees no key of this chunk: O = 0, LSE = -inf
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
                if (hl == 0) a.out.LSE[(int64_t)cit.c * a.out.part_stride_L + qidx] = ltot > 0.f ? m_used * kscale + __logf(ltot) : -INFINITY;
            }
            c_el = -1;
            ++c_item;
            c_load(false);
        }
    }
}

template <int D>
static hipError_t launch_decode_mfma_t(const DecodeArgs& a, hipStream_t s) {
    constexpr int NS = 2;   // D = 128: 32 KiB of LDS per wavefront, four wavefronts per CU (rings of 3 and 4 were slower)
    constexpr int STB = Geo<D>::STB;
    const int grid = (a.items + a.ipw - 1) / a.ipw;
    if (a.fp8) {
        if constexpr (D == 128) {
            if (a.seg) return hipErrorInvalidValue;
            // (rings of 3 and 4 slots, two and three elements in flight: 77 and 78 us against 76 on config 4)
            if (a.tile_rows == 16) {
                if (a.pg.table) decode_mfma_kernel<D, NS, true, false, true, 16><<<(unsigned)grid, 64, NS * STB, s>>>(a);
                else decode_mfma_kernel<D, NS, false, false, true, 16><<<(unsigned)grid, 64, NS * STB, s>>>(a);
            } else if (a.pg.table) {
                decode_mfma_kernel<D, NS, true, false, true><<<(unsigned)grid, 64, NS * STB, s>>>(a);
            } else {
                decode_mfma_kernel<D, NS, false, false, true><<<(unsigned)grid, 64, NS * STB, s>>>(a);
            }
        } else {
            return hipErrorInvalidValue;   // 8-bit rows on the matrix cores: D = 128 only
        }
    } else if (a.tile_rows == 16) {
        if (a.pg.table) decode_mfma_kernel<D, NS, true, false, false, 16><<<(unsigned)grid, 64, 2 * NS * STB, s>>>(a);
        else if (a.seg) decode_mfma_kernel<D, NS, false, true, false, 16><<<(unsigned)grid, 64, 2 * NS * STB, s>>>(a);
        else decode_mfma_kernel<D, NS, false, false, false, 16><<<(unsigned)grid, 64, 2 * NS * STB, s>>>(a);
    } else if (a.pg.table) {
        decode_mfma_kernel<D, NS, true, false><<<(unsigned)grid, 64, 2 * NS * STB, s>>>(a);
    } else if (a.seg) {
        decode_mfma_kernel<D, NS, false, true><<<(unsigned)grid, 64, 2 * NS * STB, s>>>(a);
    } else {
        decode_mfma_kernel<D, NS, false, false><<<(unsigned)grid, 64, 2 * NS * STB, s>>>(a);
    }
    return hipGetLastError();
}

// Work items: B * nchunks * ceil(nq*G / tile_rows) * Hkv, adjacent ids on adjacent KV heads of the same rows; a.ipw
// consecutive items per wavefront (= workgroup).
hipError_t launch_decode_mfma(const DecodeArgs& a, int D, hipStream_t s) {
    if (a.items == 0) return hipSuccess;
    if (a.ipw < 1 || a.n_levels != (a.seg ? 1 : 0) || (a.seg && a.pg.table)) return hipErrorInvalidValue;
    if (a.tile_rows != 32 && a.tile_rows != 16) return hipErrorInvalidValue;
    if (a.pg.table && (a.pg.shift < 4 || a.pg.stride < 1 || a.pg.n_pages < 1)) return hipErrorInvalidValue;
    if (D == 128) return launch_decode_mfma_t<128>(a, s);
    if (D == 64) return launch_decode_mfma_t<64>(a, s);
    return hipErrorInvalidValue;
}

}  // namespace hg
