// Internal declarations shared by the HIP translation units of libhydragen (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hydragen.h"

namespace hg {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// ---- device-side descriptions --------------------------------------------------------------------

struct LevelDev {
    const uint16_t* K;
    const uint16_t* V;
    const int32_t* kv_off;   // may be null when n_blocks == 1
    const int32_t* seq_off;  // may be null when n_blocks == 1
    int n_blocks;
    int max_rows;
    int max_seqs;
};

// Where a kernel puts a partial (or final) result for query row idx = (b*nq + t)*Hq + h.
struct OutDev {
    void* O;          // [rows, D] fp32 or bf16
    float* LSE;       // [rows]
    int bf16;         // 1: O is bf16
    int64_t part_stride_O;    // elements between consecutive parts (0 when a single part)
    int64_t part_stride_L;
};

constexpr int kWideMaxTeams = 256;        // one team per CU at most
constexpr int kWideBoundaryCost = 9;      // stages a piece boundary costs a workgroup (measured: 8 us at 0.85 us per stage)

// Work partition of the persistent 256-row shared-block kernel (prefix_wide_impl.h).
struct WidePlan {
    int n_c;        // stages per column (32 keys each at D = 128, 64 at D = 64), from the host's bound on rows per block
    int ncols;      // columns = n_blocks * Hkv * rowgroups
    int rowgroups;  // groups of at most 32 query-row tiles
    int T;          // workgroups per team = query-row tiles per row group
    int slots;      // workgroups (CUs) per XCD that the kernel occupies
    int tpx;        // teams per XCD (slots / T)
    int quota;      // stages per team (mode 0)
    int nparts;     // partial results per query row
    int mode;       // how the flattened (column, stage) space is cut into one contiguous range per team:
                    // 0: equal ranges of `quota` stages; 1: ranges that never straddle a column boundary (each column
                    // cut evenly among its own teams, or whole columns per team when there are more columns than teams);
                    // 2: ranges of equal cost from the table below (a column boundary inside a range counts as
                    // kWideBoundaryCost stages: the team's workgroups store a result and load a Q tile there)
    int starts[kWideMaxTeams + 1];      // mode 2: team t walks [starts[t], starts[t + 1])
    int first_part[kWideMaxTeams];      // mode 2: part index of team t's first piece (pieces of its column before it)
};

struct PrefixArgs {
    const uint16_t* Q;
    LevelDev lv;
    int B, Hq, Hkv, G;
    int nq;           // queries per sequence: a sequence contributes nq*G rows per KV head, row = t*G + g
    int mtiles;       // query-row tiles per (block, KV head)
    int nsplit;       // key-range splits per block
    int chunk;        // keys per split (multiple of the key tile)
    int total_tiles;  // n_blocks * nsplit * Hkv * mtiles
    int per_xcd;      // ceil(total_tiles / 8)
    float scale;      // softmax scale
    OutDev out;       // part index = split
    WidePlan wide;    // persistent kernel only
};

// Page table of a paged suffix cache: suffix row j of sequence b is pool row
// (table[b*stride + (j >> shift)] << shift) + (j & ((1 << shift) - 1)); page ids are clamped to [0, n_pages).
struct PagedDev {
    const int32_t* table;   // null: the suffix is addressed by offsets[b] + j
    int shift;              // log2(rows per page), 4..10
    int stride;             // table entries per sequence
    int n_pages;
};

struct DecodeArgs {
    const uint16_t* Q;
    int n_levels;
    LevelDev lv[HG_MAX_LEVELS];
    const uint16_t* Ks;
    const uint16_t* Vs;
    const int32_t* offsets;
    const int32_t* lengths;   // null: no suffix
    PagedDev pg;              // suffix read through a page table when pg.table != null (then offsets is unused)
    int max_len;
    int B, Hq, Hkv, G;
    int nq;           // queries per sequence; query t sees suffix rows [0, length - (nq-1-t))
    int chunk;        // keys per work item
    int nchunks;      // work items per (sequence, KV head, query-head group)
    int64_t units;    // B * nq * nchunks * Hkv * (G / GT)
    int tile_rows;    // matrix-core kernel: query rows per tile, 32 or 16 (16: at most 16 rows per KV head and sequence)
    int items;        // matrix-core kernel: B * nchunks * ceil(nq*G / tile_rows) * Hkv work items
    int ipw;          // matrix-core kernel: consecutive work items per wavefront
    int seg;          // matrix-core kernel: 1 = the keys of sequence b are the rows of the block of lv[0] that covers b
                      // (Ks/Vs then point at that level's tensors; offsets/lengths are unused, no causal bound)
    float scale;
    int fp8;          // vector-ALU kernel, suffix only: Ks/Vs hold E4M3 codes (one byte per element)
    float k_scale, v_scale;   // value = code * scale (fp8 only)
    OutDev out;       // part index = chunk
};

// The single-launch fused kernel (fused_small.hip): every level, the suffix and the merge for 32-row tiles of query rows.
struct SmallArgs {
    const uint16_t* Q;
    int n_levels;
    LevelDev lv[HG_MAX_LEVELS];
    const uint16_t* Ks;
    const uint16_t* Vs;
    const int32_t* offsets;
    const int32_t* lengths;   // null: no suffix
    int max_len;
    int B, Hq, Hkv, G;
    int nq;
    int tiles;                // 32-row tiles of the B * nq * G query rows of one KV head
    float scale;
    void* O;                  // final results: [B, nq, Hq, D] bf16 or fp32, LSE [B, nq, Hq] (may be null)
    float* LSE;
    int bf16;
};

struct MergeArgs {
    const void* O[HG_MAX_PARTS];
    const float* L[HG_MAX_PARTS];
    int n;
    int64_t rows;
    void* O_out;
    float* L_out;     // may be null
};

// KV-cache update of a decode step: nq new rows per sequence appended to the suffix cache, lengths advanced.
struct AppendArgs {
    const uint16_t* Knew;     // [B, nq, Hkv, D]
    const uint16_t* Vnew;
    uint16_t* Ks;             // suffix cache (packed rows or page pool)
    uint16_t* Vs;
    const int32_t* offsets;   // unused when pg.table != null
    int32_t* lengths;
    PagedDev pg;
    int capacity;             // rows reserved per sequence
    int B, nq;
    int row_elems;            // Hkv * D
    int fp8;                  // the cache holds E4M3 codes: code = nearest(value / scale), saturating
    float k_scale, v_scale;
};

struct FillArgs {
    void* O; float* LSE; int bf16; int64_t rows; int D;
};

// ---- launchers (defined next to their kernels) ------------------------------------------------------
hipError_t launch_prefix_narrow(const PrefixArgs& a, int D, hipStream_t s);
hipError_t launch_prefix_wide(const PrefixArgs& a, int D, hipStream_t s);   // a.wide from plan_prefix_wide with the same D
hipError_t launch_prefix_wide_d64(const PrefixArgs& a, hipStream_t s);      // (the D = 64 kernel lives in its own translation unit)
bool plan_prefix_wide(const LevelDev& lv, int Hkv, int G, int D, int max_parts, int slots_per_xcd, WidePlan* out);
hipError_t launch_decode(const DecodeArgs& a, int D, int GT, hipStream_t s);
hipError_t launch_decode_mfma(const DecodeArgs& a, int D, hipStream_t s);   // matrix-core per-sequence kernel (8-bit rows: D = 128 only)
hipError_t launch_merge(const MergeArgs& a, int D, bool in_bf16, bool out_bf16, hipStream_t s);
hipError_t launch_fused_small(const SmallArgs& a, int D, hipStream_t s);
hipError_t launch_mfma_loop(int iters, int random_operands, unsigned long long* clocks, float* sink, hipStream_t s);
hipError_t launch_stream_read(const void* src, size_t bytes, float* sink, hipStream_t s);
hipError_t launch_xcd_probe(int n_workgroups, int* out, hipStream_t s);
hipError_t launch_fill_empty(const FillArgs& a, hipStream_t s);
hipError_t launch_kv_append(const AppendArgs& a, hipStream_t s);

constexpr int kPrefixRowsNarrow = 128;  // query rows per workgroup of the 128-row kernel (4 wavefronts x 32 rows)
constexpr int kPrefixRowsWide = 256;    // query rows per workgroup of the persistent kernel (8 wavefronts x 32 rows)
constexpr int kPrefixKeys = 64;         // keys per prefix LDS tile

// ---- small device helpers -------------------------------------------------------------------------
#ifdef __HIPCC__
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xffff0000u); }

// round-to-nearest-even fp32 -> bf16 bits (finite inputs; NaN stays NaN)
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}
#endif

}  // namespace hg
