// Host side of libhydragen: argument checks, work partitioning, kernel sequencing.  No device allocation,
// no host synchronisation, no copies: every entry point only enqueues kernels on the context's stream.
#include <math.h>
#include <algorithm>
#include <mutex>
#include <new>

#include "hg_internal.h"
#include "hydragen_debug.h"

struct hg_ctx {
    int device;
    hipStream_t stream;
    unsigned char* ws;
    size_t ws_bytes;
    int opt_prefix_splits;
    int opt_suffix_chunk;
    int opt_overlap;
    int opt_naive_chunk;
    int opt_prefix_kernel;
    int opt_wide_slots;
    int opt_nq;            // queries per sequence (1 = decode)
    int opt_suffix_kernel; // 0 automatic, 1 vector-ALU kernel, 2 matrix-core kernel wherever it applies
    int opt_suffix_ipw;    // matrix-core suffix kernel: work items per wavefront (0 automatic)
    int opt_suffix_tile;   // matrix-core suffix kernel: query rows per tile (0 automatic, 16, 32)
    int opt_fused_kernel;  // fused call: 0 automatic, 1 separate kernels, 2 single launch whenever it applies
    hipStream_t aux;       // second stream for the overlap option
    hipEvent_t ev_fork, ev_join;
    // stage timing ring: slot = call % HG_TIMING_RING, 2 events (begin, end) per stage
    int opt_timing;
    hipEvent_t* tev;       // [HG_TIMING_RING][HG_MAX_STAGES][2], created when timing is first enabled
    unsigned char* tused;  // [HG_TIMING_RING][HG_MAX_STAGES]
    long long tcalls;      // fused calls recorded since timing was enabled
};

// Partial-result memory of hg_hydragen_attn_static, the fused call for callers that cannot provide a workspace from an
// allocator: a fixed array in the library's device image (every GPU the library is loaded on holds its own copy until
// the process ends).  In host code the array's name is only a handle for hipGetSymbolAddress: the address a kernel may
// use is looked up once per device in hg_create and kept in g_scratch_ptr.
static __device__ __align__(256) unsigned char scratch[HG_STATIC_SCRATCH_BYTES];
static unsigned char* g_scratch_ptr[64];   // per device, set by hg_create on that device
static std::mutex g_scratch_mu;

namespace {

using namespace hg;

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
inline int round_up(int a, int b) { return ceil_div(a, b) * b; }

struct Parts {   // fp32 partial results carved out of the workspace
    float* O;    // [cap][rows][D]
    float* L;    // [cap][rows]
    int cap;
    int64_t rows;
    int D;
    float* o(int p) const { return O + (int64_t)p * rows * D; }
    float* l(int p) const { return L + (int64_t)p * rows; }
};

struct Ws { unsigned char* p; size_t bytes; };   // device memory that holds the partial results of one call

Parts carve(const Ws& ws, int64_t rows, int D) {
    Parts p{};
    p.rows = rows;
    p.D = D;
    const size_t per = (size_t)rows * (D + 1) * sizeof(float);
    size_t cap = (ws.p && per) ? ws.bytes / per : 0;
    if (cap > HG_MAX_PARTS) cap = HG_MAX_PARTS;
    p.cap = (int)cap;
    p.O = reinterpret_cast<float*>(ws.p);
    p.L = p.O + (int64_t)p.cap * rows * D;
    return p;
}

int check_shape(int B, int Hq, int Hkv, int D, int nq) {
    if (B < 0 || Hq <= 0 || Hkv <= 0 || nq < 1) return HG_ERR_INVALID_ARG;
    if (D != 64 && D != 128) return HG_ERR_UNSUPPORTED;
    if (Hq % Hkv != 0) return HG_ERR_UNSUPPORTED;
    if ((int64_t)B * nq * Hq * D >= (1LL << 31)) return HG_ERR_UNSUPPORTED;
    return HG_OK;
}

// Byte offsets inside one sequence's suffix rows are 32-bit in the kernels: max_len * Hkv * D elements must stay below 2^31.
int check_suffix_span(int max_len, int Hkv, int D) {
    return (int64_t)max_len * Hkv * D >= (1LL << 31) ? HG_ERR_UNSUPPORTED : HG_OK;
}

int check_level(const hg_level* lv, int Hkv, int D) {
    if (!lv) return HG_ERR_INVALID_ARG;
    if (lv->n_blocks < 1 || lv->max_rows < 0 || lv->max_seqs < 0) return HG_ERR_INVALID_ARG;
    if ((lv->kv_off == nullptr) != (lv->seq_off == nullptr)) return HG_ERR_INVALID_ARG;
    if (lv->n_blocks > 1 && !lv->kv_off) return HG_ERR_INVALID_ARG;
    if (lv->max_rows > 0 && (!lv->K || !lv->V)) return HG_ERR_INVALID_ARG;
    if ((int64_t)lv->n_blocks * lv->max_rows * Hkv * D >= (1LL << 31)) return HG_ERR_UNSUPPORTED;
    return HG_OK;
}

LevelDev to_dev(const hg_level& lv, int B) {
    LevelDev d{};
    d.K = static_cast<const uint16_t*>(lv.K);
    d.V = static_cast<const uint16_t*>(lv.V);
    d.kv_off = lv.kv_off;
    d.seq_off = lv.seq_off;
    d.n_blocks = lv.n_blocks;
    d.max_rows = lv.max_rows;
    d.max_seqs = lv.kv_off ? lv.max_seqs : B;
    return d;
}

int pick_gt(int G) {
    for (int gt : {8, 4, 2}) if (G % gt == 0) return gt;
    return 1;
}

int hip_rc(hipError_t e) { return e == hipSuccess ? HG_OK : HG_ERR_HIP; }

// which shared-block kernel runs a level, and how many partial results per row it writes
struct LevelPlan { bool wide; int ns; WidePlan wp; };

// The persistent 256-row kernel runs a level whose blocks have more than 128 query rows; the 128-row
// kernel runs the rest.  (At D = 128, 16 blocks of 128 rows x 512 keys x 40 heads alone: 55 us on the
// persistent kernel against 63 us; but inside the fused call its workgroups take whole CUs from the suffix kernel, where
// 128-row workgroups share them: 0.646 against 0.591 ms on the two-level tree.)
// At D = 64 the same rule holds (fused call on 1024 x 40 heads x 16K keys: 0.351 against 0.377 ms; on the two-level
// tree the automatic choice gives 0.310 ms against 0.321 with 128-row workgroups only and 0.392 with 256-row only).
// HG_OPT_PREFIX_KERNEL = 1 forces the 128-row kernel, 2 the 256-row kernel.  max_parts bounds the
// partial results the plan may use.
// G: query rows per sequence and KV head (queries per sequence x query heads per KV head).
LevelPlan plan_level(const hg_ctx* c, const LevelDev& lv, int Hkv, int G, int D, int max_parts, int wide_slots = 32) {
    LevelPlan p{};
    const long long rows = (long long)lv.max_seqs * G;
    p.wide = false;
    p.ns = 1;
    if (lv.max_rows <= 0) return p;
    if (max_parts < 1) max_parts = 1;
    if (max_parts > HG_MAX_PARTS) max_parts = HG_MAX_PARTS;
    const bool want_wide = c->opt_prefix_kernel != 1 && (c->opt_prefix_kernel == 2 || rows > kPrefixRowsNarrow);
    if (want_wide && plan_prefix_wide(lv, Hkv, G, D, max_parts, c->opt_wide_slots > 0 ? c->opt_wide_slots : wide_slots, &p.wp)) {
        p.wide = true;
        p.ns = p.wp.nparts;
        return p;
    }
    const int slots = 512;   // 128-row workgroups resident on the 256 CUs (two per CU)
    const int64_t base = (int64_t)lv.n_blocks * ceil_div((int)rows, kPrefixRowsNarrow) * Hkv;
    const int max_ns = ceil_div(lv.max_rows, kPrefixKeys);
    int ns;
    if (c->opt_prefix_splits > 0) {
        ns = c->opt_prefix_splits;
    } else {
        // enough workgroups for about two full rounds of the resident slots, in chunks of at least 512 keys;
        // every extra split adds a partial result for the merge to read
        ns = (int)((2 * slots + base - 1) / (base > 0 ? base : 1));
        const int by_len = lv.max_rows / 512;
        if (ns > by_len) ns = by_len;
        if (ns > 16) ns = 16;
    }
    if (ns > max_ns) ns = max_ns;
    if (ns > max_parts) ns = max_parts;
    if (ns < 1) ns = 1;
    p.ns = ns;
    return p;
}

// enqueue the shared-block kernel for one level with `ns` splits writing to `out` (part = split)
int run_level(const void* Q, const LevelDev& lv, LevelPlan plan, int B, int nq, int Hq, int Hkv, int D, float scale,
              const OutDev& out, hipStream_t s) {
    PrefixArgs a{};
    a.Q = static_cast<const uint16_t*>(Q);
    a.lv = lv;
    a.B = B; a.Hq = Hq; a.Hkv = Hkv; a.G = Hq / Hkv;
    a.nq = nq;
    a.scale = scale;
    a.out = out;
    if (plan.wide) {
        a.wide = plan.wp;
        return hip_rc(launch_prefix_wide(a, D, s));
    }
    a.mtiles = ceil_div(lv.max_seqs * a.G * nq, kPrefixRowsNarrow);
    a.nsplit = plan.ns;
    a.chunk = round_up(ceil_div(lv.max_rows > 0 ? lv.max_rows : 1, plan.ns), kPrefixKeys);
    const int64_t total = (int64_t)lv.n_blocks * plan.ns * Hkv * a.mtiles;
    if (total >= (1LL << 28)) return HG_ERR_UNSUPPORTED;
    a.total_tiles = (int)total;
    a.per_xcd = ceil_div(a.total_tiles, 8);
    return hip_rc(launch_prefix_narrow(a, D, s));
}

struct SuffixPlan { int chunk, nchunks, gt; bool mfma; int ipw; };

// Storage format of the suffix cache: bf16 rows, or E4M3 codes with one scale per tensor (value = code * scale).
struct KvFmt { int fp8 = 0; float k_scale = 1.f, v_scale = 1.f; };

// Automatic choice between the two per-sequence kernels (thresholds measured at D = 128).  The matrix-core kernel reads every K/V row
// once for all nq * G query rows that a KV head serves; the vector-ALU kernel pays one dot product per row and key
// and, across queries, re-reads the suffix.  Measured (B = 512, lengths up to 512, matrix-core against vector-ALU):
// nq = 2: 184 against 368 us; G = 3: 96 against 211 us; G = 2: 94 against 114 us, but 178 against 153 us when no
// sequence has more than 128 rows (the per-item cost of the matrix-core kernel).  One row per KV head: the
// matrix-core kernel streams long rows better (6.4 against 5.8-6.0 TB/s from a few hundred rows per sequence on:
// lengths 64..384: 794 against 841 us; 256..1024: 824 against 915 us) and loses on short ones (lengths up to 256:
// 121 against 116 us; 32..128: 328 against 285 us).  At D = 64 that last gain is not consistent (402 against 440 us at
// 64..384 rows, 462 against 427 us at 1024..4096) and the clause is left out.
bool auto_mfma(int nq, int G, int max_len, int D) {
    return nq >= 2 || G >= 3 || (G == 2 && max_len >= 256) || (D == 128 && max_len >= 384);
}

// Work items of the suffix kernel are (sequence, query, KV head, group of query heads, key chunk), one wavefront
// each, in the vector-ALU kernel, and (sequence, KV head, 32-row tile of the nq * G rows, key chunk) in the
// matrix-core kernel (chosen by auto_mfma, HG_OPT_SUFFIX_KERNEL forces either; an 8-bit cache at D = 64 stays on the
// vector ALU).
// 256 keys per chunk by default; when that leaves fewer than eight wavefronts per CU (few sequences or KV heads)
// the chunks shrink, down to 64 keys, so that enough loads are in flight to cover HBM latency.
// max_chunk bounds the keys per work item (a paged cache allows 32 pages per work item).
SuffixPlan plan_suffix(const hg_ctx* c, int max_len, int G, int B, int nq, int Hkv, int D, bool paged, int max_chunk = 1 << 30,
                       bool fp8 = false) {
    SuffixPlan p;
    p.gt = pick_gt(G);
    const int R = nq * G;
    p.ipw = c->opt_suffix_ipw;
    (void)paged;
    p.mfma = (D == 128 || !fp8) && c->opt_suffix_kernel != 1 && (c->opt_suffix_kernel == 2 || auto_mfma(nq, G, max_len, D));   // 8-bit rows on the matrix cores: D = 128 only
    if (p.mfma) max_chunk = 1 << 30;   // the matrix-core kernel looks pages up per stage: no limit on pages per item
    if (c->opt_suffix_chunk > 0) {
        p.chunk = round_up(c->opt_suffix_chunk, 32);
        if (p.chunk > max_chunk) p.chunk = max_chunk;
    } else if (p.mfma) {
        // a wavefront pays a fixed price per work item (its query tile, the first stage's latency, the result's
        // stores): long items, cut only when there would be fewer than three per CU
        p.chunk = 1024;
        const long long per_chunk = (long long)B * Hkv * ceil_div(R, 32);
        while (p.chunk > 128 && per_chunk * ceil_div(max_len > 0 ? max_len : 1, p.chunk) < 768) p.chunk /= 2;
    } else {
        p.chunk = 256;
        const long long per_chunk = (long long)B * nq * Hkv * (G / p.gt);
        while (p.chunk > 64 && per_chunk * ceil_div(max_len > 0 ? max_len : 1, p.chunk) < 2048) p.chunk /= 2;
    }
    if (p.chunk > max_chunk) p.chunk = max_chunk;
    p.nchunks = max_len > 0 ? ceil_div(max_len, p.chunk) : 1;
    return p;
}

int run_decode(const void* Q, int n_levels, const LevelDev* lv, const void* Ks, const void* Vs, const int32_t* offsets,
               const int32_t* lengths, int max_len, int B, int nq, int Hq, int Hkv, int D, float scale, int chunk, int nchunks,
               int gt, const OutDev& out, hipStream_t s, const PagedDev& pg = PagedDev{}, bool mfma = false, int mfma_ipw = 0, bool seg = false,
               const KvFmt& fmt = KvFmt{}, int mfma_tile = 0) {
    DecodeArgs a{};
    a.pg = pg;
    a.fp8 = fmt.fp8;
    a.k_scale = fmt.k_scale;
    a.v_scale = fmt.v_scale;
    a.Q = static_cast<const uint16_t*>(Q);
    a.n_levels = n_levels;
    for (int i = 0; i < n_levels; ++i) a.lv[i] = lv[i];
    a.Ks = static_cast<const uint16_t*>(Ks);
    a.Vs = static_cast<const uint16_t*>(Vs);
    a.offsets = offsets;
    a.lengths = lengths;
    a.max_len = max_len;
    a.B = B; a.Hq = Hq; a.Hkv = Hkv; a.G = Hq / Hkv;
    a.nq = nq;
    a.chunk = chunk;
    a.nchunks = nchunks;
    a.units = (int64_t)B * nq * nchunks * Hkv * (a.G / gt);
    a.scale = scale;
    a.out = out;
    if (mfma) {
        a.seg = seg ? 1 : 0;
        // up to 16 rows per KV head and sequence fit a 16-row tile: half the matrix and softmax work per stage
        a.tile_rows = (nq * a.G <= 16 && mfma_tile != 32) ? 16 : 32;
        const int64_t items = (int64_t)B * nchunks * ceil_div(nq * a.G, a.tile_rows) * Hkv;
        if (items >= (1LL << 31)) return HG_ERR_UNSUPPORTED;
        a.items = (int)items;
        // consecutive items per wavefront: the copies of the next item are in flight while one is finished; few
        // enough per wavefront that the hardware still balances ragged lengths (>= 8 workgroups per resident slot)
        a.ipw = mfma_ipw > 0 ? mfma_ipw : (int)std::min<int64_t>(4, std::max<int64_t>(1, items / (1280 * 8)));
        return hip_rc(launch_decode_mfma(a, D, s));
    }
    return hip_rc(launch_decode(a, D, gt, s));
}

int run_merge(int n, const Parts& parts, int first, int D, void* O_out, int o_dtype, float* LSE_out, hipStream_t s) {
    MergeArgs m{};
    m.n = n;
    for (int i = 0; i < n; ++i) {
        m.O[i] = parts.o(first + i);
        m.L[i] = parts.l(first + i);
    }
    m.rows = parts.rows;
    m.O_out = O_out;
    m.L_out = LSE_out;
    return hip_rc(launch_merge(m, D, false, o_dtype == HG_BF16, s));
}

float eff_scale(float scale, int D) { return scale > 0.f ? scale : 1.0f / sqrtf((float)D); }

OutDev direct_out(void* O, int o_dtype, float* LSE) {
    OutDev o{};
    o.O = O; o.LSE = LSE; o.bf16 = (o_dtype == HG_BF16); o.part_stride_O = 0; o.part_stride_L = 0;
    return o;
}

OutDev parts_out(const Parts& p, int first) {
    OutDev o{};
    o.O = p.o(first); o.LSE = p.l(first); o.bf16 = 0;
    o.part_stride_O = p.rows * p.D; o.part_stride_L = p.rows;
    return o;
}

// CUs per XCD for the persistent shared-block kernel when it overlaps the suffix kernel in the fused call.
// The shared-block kernel runs against the chip's power limit, so it loses little on fewer CUs (measured on
// config 3: 0.96 / 0.90 / 0.82 / 0.69 / 0.54 of its full-chip rate on 28 / 24 / 20 / 16 / 12 CUs per XCD), while
// the memory-bound suffix kernel takes the CUs that are left.  Model: while the shared-block kernel runs the
// suffix kernel streams at 0.7 x 6 TB/s x (its share of the CUs) (measured 0.92 / 1.77 / 2.06 TB/s on 64 / 96 /
// 128 CUs), afterwards at 6 TB/s; pick the count with the smallest finish time.  flops: shared-block work; bytes: suffix KV traffic (estimated from max_len).
int pick_wide_slots(double flops, double bytes, int T) {
    // relative rate of the shared-block kernel on 4, 8, .., 32 CUs per XCD (measured down to 12, scaled below)
    static const double rate[] = {0.18, 0.36, 0.543, 0.693, 0.823, 0.895, 0.964, 1.0};
    const double full_rate = 1.14e15, bw = 6.0e12;
    if (T < 1) T = 1;
    auto rate_at = [&](int eff) { return rate[eff / 4 - 1] + (rate[(eff + 3) / 4 - 1] - rate[eff / 4 - 1]) * (eff % 4) / 4.0; };
    const double ts = bytes / bw, tp32 = flops / full_rate;
    if (ts >= 2.0 * tp32) {
        // the suffix kernel dominates: the fewest CUs on which the shared blocks still finish in half its time
        // (when teams are so wide that no smaller count does, the general model below decides)
        for (int s = 4; s < 32; s += 4) {
            const int eff = s / T * T;
            if (eff >= 4 && flops / (full_rate * rate_at(eff)) <= 0.5 * ts) return eff;
        }
    }
    int best = 32;
    double best_t = 1e30;
    for (int s = 32; s >= 4; s -= 4) {
        const int eff = s / T * T;                 // CUs per XCD that hold whole teams (no workgroup is launched on the others)
        if (eff < 4) break;
        const double tp = flops / (full_rate * rate_at(eff));
        const double conc = 0.7 * bw * (256 - 8 * eff) / 256.0;
        const double t = bytes <= conc * tp ? tp : tp + (bytes - conc * tp) / bw;
        if (t < best_t * 0.995) { best_t = t; best = eff; }
    }
    return best;
}

int fill_empty(void* O, int o_dtype, float* LSE, int64_t rows, int D, hipStream_t s) {
    FillArgs f{};
    f.O = O; f.LSE = LSE; f.bf16 = (o_dtype == HG_BF16); f.rows = rows; f.D = D;
    return hip_rc(launch_fill_empty(f, s));
}

}  // namespace

extern "C" {

int hg_create(hg_ctx** out, int device, void* hip_stream, void* workspace, size_t workspace_bytes) {
    if (!out) return HG_ERR_INVALID_ARG;
    *out = nullptr;
    if (workspace_bytes && !workspace) return HG_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0) return HG_ERR_INVALID_ARG;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || device < 0 || device >= ndev) return HG_ERR_HIP;
    if (hipSetDevice(device) != hipSuccess) return HG_ERR_HIP;
    if (device < 64) {
        // this device's copy of the static scratch array (hg_hydragen_attn_static); the device is current here
        std::lock_guard<std::mutex> lock(g_scratch_mu);
        if (!g_scratch_ptr[device]) {
            void* p = nullptr;
            if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return HG_ERR_HIP;
            g_scratch_ptr[device] = static_cast<unsigned char*>(p);
        }
    }
    hg_ctx* c = new (std::nothrow) hg_ctx();
    if (!c) return HG_ERR_HIP;
    c->device = device;
    c->stream = static_cast<hipStream_t>(hip_stream);
    c->ws = static_cast<unsigned char*>(workspace);
    c->ws_bytes = workspace_bytes;
    c->opt_prefix_splits = c->opt_suffix_chunk = c->opt_overlap = c->opt_naive_chunk = c->opt_prefix_kernel = c->opt_wide_slots = 0;
    c->opt_nq = 1;
    c->opt_suffix_kernel = 0;
    c->opt_suffix_ipw = 0;
    c->opt_suffix_tile = 0;
    c->opt_fused_kernel = 0;
    c->aux = nullptr;
    c->ev_fork = c->ev_join = nullptr;
    c->opt_timing = 0;
    c->tev = nullptr;
    c->tused = nullptr;
    c->tcalls = 0;
    if (hipStreamCreateWithFlags(&c->aux, hipStreamNonBlocking) != hipSuccess ||
        hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming) != hipSuccess) {
        hg_destroy(c);
        return HG_ERR_HIP;
    }
    *out = c;
    return HG_OK;
}

void hg_destroy(hg_ctx* c) {
    if (!c) return;
    if (c->ev_fork) (void)hipEventDestroy(c->ev_fork);
    if (c->ev_join) (void)hipEventDestroy(c->ev_join);
    if (c->aux) (void)hipStreamDestroy(c->aux);
    if (c->tev) {
        for (int i = 0; i < HG_TIMING_RING * HG_MAX_STAGES * 2; ++i)
            if (c->tev[i]) (void)hipEventDestroy(c->tev[i]);
        delete[] c->tev;
    }
    delete[] c->tused;
    delete c;
}

int hg_set_stream(hg_ctx* c, void* hip_stream) {
    if (!c) return HG_ERR_INVALID_ARG;
    c->stream = static_cast<hipStream_t>(hip_stream);
    return HG_OK;
}

int hg_set_option(hg_ctx* c, int option, int value) {
    if (!c || value < 0) return HG_ERR_INVALID_ARG;
    switch (option) {
        case HG_OPT_PREFIX_SPLITS: c->opt_prefix_splits = value; return HG_OK;
        case HG_OPT_SUFFIX_CHUNK: c->opt_suffix_chunk = value; return HG_OK;
        case HG_OPT_OVERLAP:
            if (value > 2) return HG_ERR_INVALID_ARG;
            c->opt_overlap = value;
            return HG_OK;
        case HG_OPT_NAIVE_CHUNK: c->opt_naive_chunk = value; return HG_OK;
        case HG_OPT_PREFIX_KERNEL:
            if (value > 2) return HG_ERR_INVALID_ARG;
            c->opt_prefix_kernel = value;
            return HG_OK;
        case HG_OPT_NUM_QUERIES:
            if (value < 1 || value > 64) return HG_ERR_INVALID_ARG;
            c->opt_nq = value;
            return HG_OK;
        case HG_OPT_SUFFIX_KERNEL:
            if (value > 2) return HG_ERR_INVALID_ARG;
            c->opt_suffix_kernel = value;
            return HG_OK;
        case HG_OPT_SUFFIX_ITEMS_PER_WAVE:
            if (value > 1024) return HG_ERR_INVALID_ARG;
            c->opt_suffix_ipw = value;
            return HG_OK;
        case HG_OPT_SUFFIX_TILE_ROWS:
            if (value != 0 && value != 16 && value != 32) return HG_ERR_INVALID_ARG;
            c->opt_suffix_tile = value;
            return HG_OK;
        case HG_OPT_FUSED_KERNEL:
            if (value > 2) return HG_ERR_INVALID_ARG;
            c->opt_fused_kernel = value;
            return HG_OK;
        case HG_OPT_WIDE_SLOTS:
            if (value > 32) return HG_ERR_INVALID_ARG;
            c->opt_wide_slots = value;
            return HG_OK;
        case HG_OPT_STAGE_TIMING:
            if (value && !c->tev) {
                if (hipSetDevice(c->device) != hipSuccess) return HG_ERR_HIP;
                const int n = HG_TIMING_RING * HG_MAX_STAGES * 2;
                c->tev = new (std::nothrow) hipEvent_t[n]();
                c->tused = new (std::nothrow) unsigned char[HG_TIMING_RING * HG_MAX_STAGES]();
                if (!c->tev || !c->tused) return HG_ERR_HIP;
                for (int i = 0; i < n; ++i)
                    if (hipEventCreate(&c->tev[i]) != hipSuccess) return HG_ERR_HIP;
            }
            c->opt_timing = value ? 1 : 0;
            c->tcalls = 0;
            return HG_OK;
    }
    return HG_ERR_INVALID_ARG;
}

size_t hg_workspace_bytes(int B, int Hq, int D, int parts) {
    if (B <= 0 || Hq <= 0 || D <= 0 || parts <= 0) return 0;
    const size_t n = (size_t)parts * (size_t)B * Hq * (size_t)(D + 1) * sizeof(float);
    return (n + 255) / 256 * 256;
}

int hg_prefix_attn_grouped(hg_ctx* c, const void* Q, const hg_level* level, int B, int Hq, int Hkv, int D, float scale,
                           void* O, int o_dtype, float* LSE) {
    if (!c || !O || !LSE || (o_dtype != HG_F32 && o_dtype != HG_BF16)) return HG_ERR_INVALID_ARG;
    int rc = check_shape(B, Hq, Hkv, D, c ? c->opt_nq : 1);
    if (rc) return rc;
    rc = check_level(level, Hkv, D);
    if (rc) return rc;
    if (B == 0) return HG_OK;
    if (!Q) return HG_ERR_INVALID_ARG;
    if (hipSetDevice(c->device) != hipSuccess) return HG_ERR_HIP;
    scale = eff_scale(scale, D);
    const int nq = c->opt_nq;
    const int64_t rows = (int64_t)B * nq * Hq;
    const LevelDev lv = to_dev(*level, B);
    const Parts parts = carve(Ws{c->ws, c->ws_bytes}, rows, D);
    const LevelPlan plan = plan_level(c, lv, Hkv, nq * (Hq / Hkv), D, parts.cap);
    const int ns = plan.ns;
    hipStream_t s = c->stream;
    if (lv.max_rows == 0 || lv.max_seqs == 0) return fill_empty(O, o_dtype, LSE, rows, D, s);
    if (!plan.wide && (int64_t)lv.n_blocks * ns * Hkv * ceil_div(lv.max_seqs * nq * (Hq / Hkv), kPrefixRowsNarrow) >= (1LL << 28))
        return HG_ERR_UNSUPPORTED;      // (checked before anything is enqueued)
    // (sequences that no block covers are given their empty result by the level's kernel itself)
    if (ns == 1) return run_level(Q, lv, plan, B, nq, Hq, Hkv, D, scale, direct_out(O, o_dtype, LSE), s);
    rc = run_level(Q, lv, plan, B, nq, Hq, Hkv, D, scale, parts_out(parts, 0), s);
    if (rc) return rc;
    return run_merge(ns, parts, 0, D, O, o_dtype, LSE, s);
}

int hg_prefix_attn(hg_ctx* c, const void* Q, const void* Kp, const void* Vp, int B, int Hq, int Hkv, int D, int P,
                   float scale, void* O, int o_dtype, float* LSE) {
    if (P < 0) return HG_ERR_INVALID_ARG;
    hg_level lv{};
    lv.K = Kp; lv.V = Vp; lv.n_blocks = 1; lv.kv_off = nullptr; lv.seq_off = nullptr; lv.max_rows = P; lv.max_seqs = B;
    return hg_prefix_attn_grouped(c, Q, &lv, B, Hq, Hkv, D, scale, O, o_dtype, LSE);
}

// hg_suffix_attn and hg_suffix_attn_paged (pg.table set, offsets unused)
static int suffix_impl(hg_ctx* c, const void* Q, const void* Ks, const void* Vs, const int32_t* offsets,
                       const int32_t* lengths, int max_len, int B, int Hq, int Hkv, int D, float scale, void* O, int o_dtype,
                       float* LSE, const hg::PagedDev& pg, bool paged, const KvFmt& fmt = KvFmt{}) {
    if (!c || !O || !LSE || (o_dtype != HG_F32 && o_dtype != HG_BF16) || max_len < 0) return HG_ERR_INVALID_ARG;
    int rc = check_shape(B, Hq, Hkv, D, c ? c->opt_nq : 1);
    if (rc) return rc;
    rc = check_suffix_span(max_len, Hkv, D);
    if (rc) return rc;
    if (B == 0) return HG_OK;
    if (!Q || (!offsets && !paged) || !lengths) return HG_ERR_INVALID_ARG;
    if (max_len > 0 && (!Ks || !Vs)) return HG_ERR_INVALID_ARG;
    if (hipSetDevice(c->device) != hipSuccess) return HG_ERR_HIP;
    scale = eff_scale(scale, D);
    const int nq = c->opt_nq;
    const int64_t rows = (int64_t)B * nq * Hq;
    hipStream_t s = c->stream;
    if (max_len == 0) return fill_empty(O, o_dtype, LSE, rows, D, s);
    const Parts parts = carve(Ws{c->ws, c->ws_bytes}, rows, D);
    const int max_chunk = pg.table ? 32 << pg.shift : 1 << 30;
    SuffixPlan p = plan_suffix(c, max_len, Hq / Hkv, B, nq, Hkv, D, pg.table != nullptr, max_chunk, fmt.fp8 != 0);
    if (p.nchunks > parts.cap) {  // not enough room for partials: fewer, longer chunks
        p.nchunks = parts.cap > 1 ? parts.cap : 1;
        p.chunk = round_up(ceil_div(max_len, p.nchunks), 32);
        p.nchunks = ceil_div(max_len, p.chunk);
    }
    if (!p.mfma && p.chunk > max_chunk) return HG_ERR_WORKSPACE;
    if (p.nchunks == 1)
        return run_decode(Q, 0, nullptr, Ks, Vs, offsets, lengths, max_len, B, nq, Hq, Hkv, D, scale, p.chunk, 1, p.gt,
                          direct_out(O, o_dtype, LSE), s, pg, p.mfma, p.ipw, false, fmt, c->opt_suffix_tile);
    rc = run_decode(Q, 0, nullptr, Ks, Vs, offsets, lengths, max_len, B, nq, Hq, Hkv, D, scale, p.chunk, p.nchunks, p.gt,
                    parts_out(parts, 0), s, pg, p.mfma, p.ipw, false, fmt, c->opt_suffix_tile);
    if (rc) return rc;
    return run_merge(p.nchunks, parts, 0, D, O, o_dtype, LSE, s);
}

// scales of an 8-bit cache: finite and positive
static bool fp8_fmt(float k_scale, float v_scale, KvFmt* out) {
    if (!(k_scale > 0.f) || !(v_scale > 0.f) || k_scale > 3.0e38f || v_scale > 3.0e38f) return false;
    out->fp8 = 1;
    out->k_scale = k_scale;
    out->v_scale = v_scale;
    return true;
}

// checks an hg_paged_kv against the rows it must be able to address and translates it
static int paged_dev(const hg_paged_kv* kv, int rows_per_seq, int Hkv, int D, hg::PagedDev* out, KvFmt* fmt) {
    if (!kv || !out || !fmt) return HG_ERR_INVALID_ARG;
    *fmt = KvFmt{};
    if (kv->kv_format == HG_KV_E4M3) {
        if (!fp8_fmt(kv->k_scale, kv->v_scale, fmt)) return HG_ERR_INVALID_ARG;
    } else if (kv->kv_format != HG_KV_BF16) {
        return HG_ERR_INVALID_ARG;
    }
    int shift = 0;
    while ((1 << shift) < kv->page_size && shift < 11) ++shift;
    if (kv->page_size < 16 || kv->page_size > 1024 || (1 << shift) != kv->page_size) return HG_ERR_INVALID_ARG;
    if (kv->n_pages < 0 || kv->table_stride < 0) return HG_ERR_INVALID_ARG;
    if ((int64_t)kv->n_pages * kv->page_size * Hkv * D >= (1LL << 31)) return HG_ERR_UNSUPPORTED;
    if (rows_per_seq > 0) {
        if (!kv->K || !kv->V || !kv->page_table || kv->n_pages < 1) return HG_ERR_INVALID_ARG;
        if ((int64_t)kv->table_stride * kv->page_size < rows_per_seq) return HG_ERR_INVALID_ARG;
    }
    out->table = kv->page_table;
    out->shift = shift;
    out->stride = kv->table_stride;
    out->n_pages = kv->n_pages;
    return HG_OK;
}

int hg_suffix_attn(hg_ctx* c, const void* Q, const void* Ks, const void* Vs, const int32_t* offsets,
                   const int32_t* lengths, int max_len, int B, int Hq, int Hkv, int D, float scale, void* O, int o_dtype,
                   float* LSE) {
    return suffix_impl(c, Q, Ks, Vs, offsets, lengths, max_len, B, Hq, Hkv, D, scale, O, o_dtype, LSE, hg::PagedDev{}, false);
}

int hg_suffix_attn_paged(hg_ctx* c, const void* Q, const hg_paged_kv* kv, const int32_t* lengths, int max_len, int B,
                         int Hq, int Hkv, int D, float scale, void* O, int o_dtype, float* LSE) {
    if (max_len < 0 || Hkv <= 0 || (D != 64 && D != 128)) return HG_ERR_INVALID_ARG;
    hg::PagedDev pg{};
    KvFmt fmt;
    const int rc = paged_dev(kv, max_len, Hkv, D, &pg, &fmt);
    if (rc) return rc;
    return suffix_impl(c, Q, kv->K, kv->V, nullptr, lengths, max_len, B, Hq, Hkv, D, scale, O, o_dtype, LSE, pg, true, fmt);
}

int hg_merge(hg_ctx* c, int n, const void* const* O_parts, const float* const* LSE_parts, int o_dtype_in, int64_t rows,
             int D, void* O_out, int o_dtype_out, float* LSE_out) {
    if (!c || n < 1 || n > HG_MAX_PARTS || !O_parts || !LSE_parts || rows < 0 || !O_out) return HG_ERR_INVALID_ARG;
    if ((o_dtype_in != HG_F32 && o_dtype_in != HG_BF16) || (o_dtype_out != HG_F32 && o_dtype_out != HG_BF16))
        return HG_ERR_INVALID_ARG;
    if (D != 64 && D != 128) return HG_ERR_UNSUPPORTED;
    for (int i = 0; i < n; ++i)
        if (!O_parts[i] || !LSE_parts[i]) return HG_ERR_INVALID_ARG;
    if (rows == 0) return HG_OK;
    if (hipSetDevice(c->device) != hipSuccess) return HG_ERR_HIP;
    hg::MergeArgs m{};
    m.n = n;
    for (int i = 0; i < n; ++i) {
        m.O[i] = O_parts[i];
        m.L[i] = LSE_parts[i];
    }
    m.rows = rows;
    m.O_out = O_out;
    m.L_out = LSE_out;
    return hip_rc(hg::launch_merge(m, D, o_dtype_in == HG_BF16, o_dtype_out == HG_BF16, c->stream));
}

static int check_fused(hg_ctx* c, const void* Q, int n_levels, const hg_level* levels, const void* Ks, const void* Vs,
                       const int32_t* offsets, const int32_t* lengths, int max_len, int B, int Hq, int Hkv, int D,
                       void* O_out, int o_dtype, bool paged = false) {
    if (!c || !O_out || (o_dtype != HG_F32 && o_dtype != HG_BF16) || max_len < 0) return HG_ERR_INVALID_ARG;
    if (n_levels < 0 || n_levels > HG_MAX_LEVELS || (n_levels > 0 && !levels)) return HG_ERR_INVALID_ARG;
    int rc = check_shape(B, Hq, Hkv, D, c ? c->opt_nq : 1);
    if (rc) return rc;
    for (int i = 0; i < n_levels; ++i) {
        rc = check_level(&levels[i], Hkv, D);
        if (rc) return rc;
    }
    if (B > 0 && !Q) return HG_ERR_INVALID_ARG;
    if (Ks && max_len > 0 && (!Vs || (!offsets && !paged) || !lengths)) return HG_ERR_INVALID_ARG;
    if (Ks) {
        rc = check_suffix_span(max_len, Hkv, D);
        if (rc) return rc;
    }
    return HG_OK;
}

// hg_hydragen_attn and hg_hydragen_attn_paged (pg.table set, offsets unused)
static int fused_impl(hg_ctx* c, const void* Q, int n_levels, const hg_level* levels, const void* Ks, const void* Vs,
                      const int32_t* offsets, const int32_t* lengths, int max_len, int B, int Hq, int Hkv, int D,
                      float scale, void* O_out, int o_dtype, float* LSE_out, const hg::PagedDev& pg, const KvFmt& fmt = KvFmt{},
                      const Ws* ws_override = nullptr) {
    int rc = check_fused(c, Q, n_levels, levels, Ks, Vs, offsets, lengths, max_len, B, Hq, Hkv, D, O_out, o_dtype,
                         pg.table != nullptr);
    if (rc) return rc;
    if (B == 0) return HG_OK;
    if (hipSetDevice(c->device) != hipSuccess) return HG_ERR_HIP;
    scale = eff_scale(scale, D);
    const int nq = c->opt_nq;
    const int64_t rows = (int64_t)B * nq * Hq;
    const int G = Hq / Hkv;
    const bool has_suffix = Ks != nullptr && max_len > 0;

    // One launch for everything when that is the faster way (packed bf16 suffix rows only): a workgroup of four
    // wavefronts per 32-row tile walks every shared block and the tile's suffixes and merges in LDS (fused_small.hip),
    // against three launches, two event edges and a round trip of the partial results through HBM for the separate
    // kernels.  Both durations are estimated, in microseconds, from fits to measurements on the shape of Sec. 4.2
    // (eight query heads per KV head, B = 64 .. 2048, 256 .. 16384 shared keys, 128 and 512 suffix rows):
    //   single launch: 9 + c x (stages of a tile / 4 wavefronts) x rounds of 256 workgroups, c = 1.24 us per 32-key
    //                  stage while at most half the CUs are busy, 1.6 when the chip is full; never faster than the
    //                  suffix rows stream in (5.5 TB/s);
    //   separate:      24 for the launches and the merge + suffix rows at 5 TB/s + shared blocks at 1.1 PFLOP/s, 8 more
    //                  once a block is long enough to be split.
    // The host knows only an upper bound of the suffix lengths: the single launch is priced at that bound, the separate
    // kernels at a mean of 0.75 of it.  The single launch is taken when its estimate is at most 130 us (beyond that the
    // fit is optimistic: tiles of many short suffixes, 32 per tile with one query row per KV head, pay per segment) and
    // below the other estimate, by a tenth once it exceeds 40 us.  With ragged lengths this errs towards the separate
    // kernels (measured on the full-size configurations, single launch against separate kernels: 0.241 / 0.150 ms,
    // 0.415 / 0.330, 0.578 / 0.370, 0.305 / 0.180, 0.712 / 0.577: there the separate kernels must be, and are, chosen).
    if (!pg.table && !fmt.fp8 && c->opt_fused_kernel != 1 && !c->opt_timing) {
        const int rps = nq * G;
        long long shared_keys = 0;
        double flops = 0.0;
        bool any = has_suffix;
        for (int i = 0; i < n_levels; ++i) {
            const long long seqs = levels[i].kv_off ? levels[i].max_seqs : B;
            if (levels[i].max_rows > 0 && seqs > 0) {
                shared_keys += levels[i].max_rows;
                flops += 4.0 * levels[i].n_blocks * (double)levels[i].max_rows * seqs * nq * Hq * D;
                any = true;
            }
        }
        const int seqs_per_tile = rps >= 32 ? 1 : (32 + rps - 1) / rps + (32 % rps ? 1 : 0);
        const long long stages = (shared_keys + 31) / 32 + (has_suffix ? (long long)seqs_per_tile * ((max_len + 31) / 32) : 0);
        const long long tiles = ((long long)B * rps + 31) / 32;
        const double wgs = (double)(tiles * Hkv);
        const double rounds = wgs > 256.0 ? wgs / 256.0 : 1.0;
        const double suffix_us = has_suffix ? 4.0 * B * (double)max_len * Hkv * D / 5.0e6 : 0.0;      // at 5 TB/s
        const double chain_us = 9.0 + (wgs <= 128.0 ? 1.24 : 1.6) * (double)((stages + 3) / 4) * rounds;
        const double est_single = std::max(chain_us, suffix_us * (5.0 / 5.5) + 4.0);
        const double est_separate = 24.0 + 0.75 * suffix_us + (shared_keys >= 1024 ? 8.0 : 0.0) + flops / 1.1e9;
        const bool small = est_single <= 130.0 && est_single <= (est_single <= 40.0 ? 1.0 : 0.9) * est_separate;
        if (any && tiles * Hkv < (1LL << 31) && (c->opt_fused_kernel == 2 || small)) {
            SmallArgs sa{};
            sa.Q = static_cast<const uint16_t*>(Q);
            sa.n_levels = 0;
            for (int i = 0; i < n_levels; ++i) {
                const LevelDev d = to_dev(levels[i], B);
                if (d.max_rows == 0 || d.max_seqs == 0) continue;
                sa.lv[sa.n_levels++] = d;
            }
            sa.Ks = static_cast<const uint16_t*>(Ks);
            sa.Vs = static_cast<const uint16_t*>(Vs);
            sa.offsets = offsets;
            sa.lengths = has_suffix ? lengths : nullptr;
            sa.max_len = max_len;
            sa.B = B; sa.Hq = Hq; sa.Hkv = Hkv; sa.G = G; sa.nq = nq;
            sa.tiles = (int)tiles;
            sa.scale = scale;
            sa.O = O_out; sa.LSE = LSE_out; sa.bf16 = (o_dtype == HG_BF16);
            return hip_rc(launch_fused_small(sa, D, c->stream));
        }
    }
    const Parts parts = carve(ws_override ? *ws_override : Ws{c->ws, c->ws_bytes}, rows, D);

    // plan: parts per level and for the suffix, shrunk to fit the workspace
    LevelDev lv[HG_MAX_LEVELS];
    LevelPlan plan[HG_MAX_LEVELS];
    int ns[HG_MAX_LEVELS];
    int nlev = 0;
    int wide_slots = 32;
    bool tiny = false;   // so little work that the event edges between two streams cost more than overlap can gain
    if (has_suffix && c->opt_overlap != 1) {
        double flops = 0.0;
        int T = 1;
        for (int i = 0; i < n_levels; ++i) {
            const long long seqs = levels[i].kv_off ? levels[i].max_seqs : B;
            flops += 4.0 * levels[i].n_blocks * (double)levels[i].max_rows * seqs * nq * Hq * D;
            const long long tiles = (seqs * nq * G + kPrefixRowsWide - 1) / kPrefixRowsWide;
            if (seqs * nq * G > kPrefixRowsNarrow && tiles <= 32 && tiles > T) T = (int)tiles;
        }
        // K and V, bf16 (or 8-bit codes; on the matrix cores their expansion costs about a third of the saving); the
        // vector-ALU kernel reads them once per query; mean length taken as 0.75 max_len
        const bool sfx_mfma = plan_suffix(c, max_len, G, B, nq, Hkv, D, pg.table != nullptr, 1 << 30, fmt.fp8 != 0).mfma;
        const double per_elem = fmt.fp8 ? (sfx_mfma ? 2.6 : 2.0) : 4.0;
        const double bytes = per_elem * B * (sfx_mfma ? 1 : nq) * (0.75 * max_len) * Hkv * D;
        wide_slots = pick_wide_slots(flops, bytes, T);
        tiny = c->opt_overlap == 0 && flops / 1.14e15 + bytes / 6.0e12 < 60e-6;
        if (tiny) wide_slots = 32;
    }
    for (int i = 0; i < n_levels; ++i) {
        LevelDev d = to_dev(levels[i], B);
        if (d.max_rows == 0 || d.max_seqs == 0) continue;  // empty level contributes nothing
        lv[nlev] = d;
        plan[nlev] = plan_level(c, d, Hkv, nq * G, D, parts.cap, wide_slots);
        ns[nlev] = plan[nlev].ns;
        ++nlev;
    }
    const int max_chunk = pg.table ? 32 << pg.shift : 1 << 30;
    SuffixPlan sp = plan_suffix(c, max_len, G, B, nq, Hkv, D, pg.table != nullptr, max_chunk, fmt.fp8 != 0);
    if (!has_suffix) sp.nchunks = 0;
    auto total_parts = [&]() { int t = sp.nchunks; for (int i = 0; i < nlev; ++i) t += ns[i]; return t; };
    if (nlev + (has_suffix ? 1 : 0) > parts.cap) return HG_ERR_WORKSPACE;
    while (total_parts() > parts.cap) {  // shrink the largest split count first
        int big = -1, bigv = 1;
        for (int i = 0; i < nlev; ++i) if (ns[i] > bigv) { bigv = ns[i]; big = i; }
        if (sp.nchunks > bigv) {
            sp.nchunks -= 1;
            sp.chunk = round_up(ceil_div(max_len, sp.nchunks), 32);
            sp.nchunks = ceil_div(max_len, sp.chunk);
        } else if (big >= 0) {
            plan[big] = plan_level(c, lv[big], Hkv, nq * G, D, ns[big] - 1, wide_slots);
            ns[big] = plan[big].ns;
        } else {
            return HG_ERR_WORKSPACE;
        }
    }
    if (has_suffix && !sp.mfma && sp.chunk > max_chunk) return HG_ERR_WORKSPACE;
    // every size limit of the launches below is checked here, before anything is enqueued
    for (int i = 0; i < nlev; ++i) {
        if (plan[i].wide) continue;
        const int64_t tiles = (int64_t)lv[i].n_blocks * ns[i] * Hkv * ceil_div(lv[i].max_seqs * nq * G, kPrefixRowsNarrow);
        if (tiles >= (1LL << 28)) return HG_ERR_UNSUPPORTED;
    }
    if (has_suffix && sp.mfma) {
        const int tile_rows = (nq * G <= 16 && c->opt_suffix_tile != 32) ? 16 : 32;
        if ((int64_t)B * sp.nchunks * ceil_div(nq * G, tile_rows) * Hkv >= (1LL << 31)) return HG_ERR_UNSUPPORTED;
    }
    const int np = total_parts();
    hipStream_t s = c->stream;
    if (np == 0) return fill_empty(O_out, o_dtype, LSE_out, rows, D, s);

    // (grouped levels may leave sequences uncovered: the level's kernel marks their partial results empty)

    // Two streams unless asked for one.  In automatic mode a call whose levels all run in the persistent kernel on
    // the whole chip stays on one stream (there is no CU left for the suffix kernel to run beside it), and so does a
    // call with less than about 60 us of work (forking and joining streams costs more than it can gain).
    bool all_wide_full = nlev > 0;
    for (int i = 0; i < nlev; ++i) all_wide_full = all_wide_full && plan[i].wide && plan[i].wp.slots == 32;
    const bool overlap = c->opt_overlap != 1 && has_suffix && nlev > 0 && !(c->opt_overlap == 0 && (all_wide_full || tiny));
    hipStream_t ssfx = s;
    if (overlap) {
        if (hipEventRecord(c->ev_fork, s) != hipSuccess) return HG_ERR_HIP;
        if (hipStreamWaitEvent(c->aux, c->ev_fork, 0) != hipSuccess) return HG_ERR_HIP;
        ssfx = c->aux;
    }
    // optional stage timing: events bracket each kernel on the stream it runs on
    const int slot = c->opt_timing ? (int)(c->tcalls % HG_TIMING_RING) : -1;
    if (slot >= 0)
        for (int i = 0; i < HG_MAX_STAGES; ++i) c->tused[slot * HG_MAX_STAGES + i] = 0;
    auto mark = [&](int stage, int which, hipStream_t st) -> bool {
        if (slot < 0) return true;
        c->tused[slot * HG_MAX_STAGES + stage] = 1;
        return hipEventRecord(c->tev[(slot * HG_MAX_STAGES + stage) * 2 + which], st) == hipSuccess;
    };
    int suffix_first = 0;
    for (int i = 0; i < nlev; ++i) suffix_first += ns[i];
    auto enqueue_suffix = [&]() -> int {
        if (!has_suffix) return HG_OK;
        if (!mark(0, 0, ssfx)) return HG_ERR_HIP;
        const int r = run_decode(Q, 0, nullptr, Ks, Vs, offsets, lengths, max_len, B, nq, Hq, Hkv, D, scale, sp.chunk,
                                 sp.nchunks, sp.gt, parts_out(parts, suffix_first), ssfx, pg, sp.mfma, sp.ipw, false, fmt, c->opt_suffix_tile);
        if (r) return r;
        if (!mark(0, 1, ssfx)) return HG_ERR_HIP;
        if (overlap && hipEventRecord(c->ev_join, c->aux) != hipSuccess) return HG_ERR_HIP;
        return HG_OK;
    };
    auto enqueue_levels = [&]() -> int {
        int part = 0;
        for (int i = 0; i < nlev; ++i) {
            if (!mark(1 + i, 0, s)) return HG_ERR_HIP;
            const int r = run_level(Q, lv[i], plan[i], B, nq, Hq, Hkv, D, scale, parts_out(parts, part), s);
            if (r) return r;
            if (!mark(1 + i, 1, s)) return HG_ERR_HIP;
            part += ns[i];
        }
        return HG_OK;
    };
    // Two streams: the memory-bound suffix kernel and the power-bound shared-block kernels run side by side.  The
    // persistent 256-row kernel takes whole CUs (wide_slots per XCD, chosen above) and is enqueued first so that
    // its workgroups are placed before the suffix kernel fills the chip; 128-row workgroups leave register space
    // for suffix wavefronts on their CUs and go second unless HG_OPT_OVERLAP = 2 asks for them first.
    bool any_wide = false;
    for (int i = 0; i < nlev; ++i) any_wide = any_wide || plan[i].wide;
    // A launch that fails here (a HIP runtime error: the sizes were checked above) leaves work enqueued and the
    // second stream forked: the fork is still joined before the error is returned, so that a stream capture in
    // progress stays valid and nothing runs behind the caller's back on the second stream.
    auto fail = [&](int code) -> int {
        if (overlap) {
            (void)hipEventRecord(c->ev_join, c->aux);
            (void)hipStreamWaitEvent(s, c->ev_join, 0);
        }
        return code;
    };
    if (c->opt_overlap == 2 || (c->opt_overlap == 0 && any_wide)) {
        rc = enqueue_levels();
        if (rc) return fail(rc);
        rc = enqueue_suffix();
        if (rc) return fail(rc);
    } else {
        rc = enqueue_suffix();
        if (rc) return fail(rc);
        rc = enqueue_levels();
        if (rc) return fail(rc);
    }
    if (overlap && hipStreamWaitEvent(s, c->ev_join, 0) != hipSuccess) return HG_ERR_HIP;
    if (!mark(nlev + 1, 0, s)) return HG_ERR_HIP;
    rc = run_merge(np, parts, 0, D, O_out, o_dtype, LSE_out, s);
    if (rc) return rc;
    if (!mark(nlev + 1, 1, s)) return HG_ERR_HIP;
    if (slot >= 0) c->tcalls += 1;
    return HG_OK;
}

int hg_hydragen_attn(hg_ctx* c, const void* Q, int n_levels, const hg_level* levels, const void* Ks, const void* Vs,
                     const int32_t* offsets, const int32_t* lengths, int max_len, int B, int Hq, int Hkv, int D,
                     float scale, void* O_out, int o_dtype, float* LSE_out) {
    return fused_impl(c, Q, n_levels, levels, Ks, Vs, offsets, lengths, max_len, B, Hq, Hkv, D, scale, O_out, o_dtype,
                      LSE_out, hg::PagedDev{});
}

int hg_hydragen_attn_static(hg_ctx* c, const void* Q, int n_levels, const hg_level* levels, const void* Ks, const void* Vs,
                            const int32_t* offsets, const int32_t* lengths, int max_len, int B, int Hq, int Hkv, int D,
                            float scale, void* O_out, int o_dtype, float* LSE_out) {
    if (!c) return HG_ERR_INVALID_ARG;
    if (c->device < 0 || c->device >= 64 || !g_scratch_ptr[c->device]) return HG_ERR_UNSUPPORTED;
    int rc = check_fused(c, Q, n_levels, levels, Ks, Vs, offsets, lengths, max_len, B, Hq, Hkv, D, O_out, o_dtype);
    if (rc) return rc;
    // one fp32 partial result per non-empty shared level and one for the suffix must fit the array
    int need = (Ks != nullptr && max_len > 0) ? 1 : 0;
    for (int i = 0; i < n_levels; ++i)
        if (levels[i].max_rows > 0 && (levels[i].kv_off ? levels[i].max_seqs : B) > 0) ++need;
    const unsigned long long per = (unsigned long long)B * c->opt_nq * Hq * (D + 1) * sizeof(float);
    if ((unsigned long long)need * per > (unsigned long long)HG_STATIC_SCRATCH_BYTES) return HG_ERR_STATIC_LIMIT;
    const Ws ws{g_scratch_ptr[c->device], (size_t)HG_STATIC_SCRATCH_BYTES};
    return fused_impl(c, Q, n_levels, levels, Ks, Vs, offsets, lengths, max_len, B, Hq, Hkv, D, scale, O_out, o_dtype,
                      LSE_out, hg::PagedDev{}, KvFmt{}, &ws);
}

int hg_hydragen_attn_paged(hg_ctx* c, const void* Q, int n_levels, const hg_level* levels, const hg_paged_kv* kv,
                           const int32_t* lengths, int max_len, int B, int Hq, int Hkv, int D, float scale, void* O_out,
                           int o_dtype, float* LSE_out) {
    if (max_len < 0 || Hkv <= 0 || (D != 64 && D != 128)) return HG_ERR_INVALID_ARG;
    hg::PagedDev pg{};
    KvFmt fmt;
    const int rc = paged_dev(kv, max_len, Hkv, D, &pg, &fmt);
    if (rc) return rc;
    if (max_len == 0) pg.table = nullptr;   // no suffix rows: the call reduces to the shared levels
    return fused_impl(c, Q, n_levels, levels, max_len > 0 ? kv->K : nullptr, kv->V, nullptr, lengths, max_len, B, Hq, Hkv, D,
                      scale, O_out, o_dtype, LSE_out, pg, fmt);
}

// hg_kv_append and hg_kv_append_paged
static int append_impl(hg_ctx* c, const void* Knew, const void* Vnew, void* Ks, void* Vs, const int32_t* offsets,
                       int32_t* lengths, int capacity, int B, int Hkv, int D, const hg::PagedDev& pg, const KvFmt& fmt = KvFmt{}) {
    if (!c || B < 0 || Hkv <= 0 || capacity < 0) return HG_ERR_INVALID_ARG;
    if (D != 64 && D != 128) return HG_ERR_UNSUPPORTED;
    if ((int64_t)B * c->opt_nq * Hkv * D >= (1LL << 31)) return HG_ERR_UNSUPPORTED;
    if (B == 0) return HG_OK;
    if (!Knew || !Vnew || !lengths || (!offsets && !pg.table)) return HG_ERR_INVALID_ARG;
    if (capacity > 0 && (!Ks || !Vs)) return HG_ERR_INVALID_ARG;
    if (capacity == 0) return HG_OK;   // no room anywhere: every new row is dropped, lengths stay
    if (hipSetDevice(c->device) != hipSuccess) return HG_ERR_HIP;
    hg::AppendArgs a{};
    a.Knew = static_cast<const uint16_t*>(Knew);
    a.Vnew = static_cast<const uint16_t*>(Vnew);
    a.Ks = static_cast<uint16_t*>(Ks);
    a.Vs = static_cast<uint16_t*>(Vs);
    a.offsets = offsets;
    a.lengths = lengths;
    a.pg = pg;
    a.capacity = capacity;
    a.B = B;
    a.nq = c->opt_nq;
    a.row_elems = Hkv * D;
    a.fp8 = fmt.fp8;
    a.k_scale = fmt.k_scale;
    a.v_scale = fmt.v_scale;
    return hip_rc(hg::launch_kv_append(a, c->stream));
}

int hg_kv_append(hg_ctx* c, const void* Knew, const void* Vnew, void* Ks, void* Vs, const int32_t* offsets,
                 int32_t* lengths, int capacity, int B, int Hkv, int D) {
    return append_impl(c, Knew, Vnew, Ks, Vs, offsets, lengths, capacity, B, Hkv, D, hg::PagedDev{});
}

int hg_kv_append_paged(hg_ctx* c, const void* Knew, const void* Vnew, const hg_paged_kv* kv, int32_t* lengths,
                       int capacity, int B, int Hkv, int D) {
    if (capacity < 0 || Hkv <= 0 || (D != 64 && D != 128)) return HG_ERR_INVALID_ARG;
    hg::PagedDev pg{};
    KvFmt fmt;
    const int rc = paged_dev(kv, capacity, Hkv, D, &pg, &fmt);
    if (rc) return rc;
    if (capacity == 0) return HG_OK;
    return append_impl(c, Knew, Vnew, kv->K, kv->V, nullptr, lengths, capacity, B, Hkv, D, pg, fmt);
}

int hg_suffix_attn_fp8(hg_ctx* c, const void* Q, const void* Ks8, const void* Vs8, float k_scale, float v_scale,
                       const int32_t* offsets, const int32_t* lengths, int max_len, int B, int Hq, int Hkv, int D, float scale,
                       void* O, int o_dtype, float* LSE) {
    KvFmt fmt;
    if (!fp8_fmt(k_scale, v_scale, &fmt)) return HG_ERR_INVALID_ARG;
    return suffix_impl(c, Q, Ks8, Vs8, offsets, lengths, max_len, B, Hq, Hkv, D, scale, O, o_dtype, LSE, hg::PagedDev{}, false, fmt);
}

int hg_hydragen_attn_fp8(hg_ctx* c, const void* Q, int n_levels, const hg_level* levels, const void* Ks8, const void* Vs8,
                         float k_scale, float v_scale, const int32_t* offsets, const int32_t* lengths, int max_len, int B,
                         int Hq, int Hkv, int D, float scale, void* O_out, int o_dtype, float* LSE_out) {
    KvFmt fmt;
    if (!fp8_fmt(k_scale, v_scale, &fmt)) return HG_ERR_INVALID_ARG;
    return fused_impl(c, Q, n_levels, levels, Ks8, Vs8, offsets, lengths, max_len, B, Hq, Hkv, D, scale, O_out, o_dtype,
                      LSE_out, hg::PagedDev{}, fmt);
}

int hg_kv_append_fp8(hg_ctx* c, const void* Knew, const void* Vnew, void* Ks8, void* Vs8, float k_scale, float v_scale,
                     const int32_t* offsets, int32_t* lengths, int capacity, int B, int Hkv, int D) {
    KvFmt fmt;
    if (!fp8_fmt(k_scale, v_scale, &fmt)) return HG_ERR_INVALID_ARG;
    return append_impl(c, Knew, Vnew, Ks8, Vs8, offsets, lengths, capacity, B, Hkv, D, hg::PagedDev{}, fmt);
}

int hg_naive_attn(hg_ctx* c, const void* Q, int n_levels, const hg_level* levels, const void* Ks, const void* Vs,
                  const int32_t* offsets, const int32_t* lengths, int max_len, int B, int Hq, int Hkv, int D, float scale,
                  void* O_out, int o_dtype, float* LSE_out) {
    int rc = check_fused(c, Q, n_levels, levels, Ks, Vs, offsets, lengths, max_len, B, Hq, Hkv, D, O_out, o_dtype);
    if (rc) return rc;
    if (B == 0) return HG_OK;
    if (hipSetDevice(c->device) != hipSuccess) return HG_ERR_HIP;
    scale = eff_scale(scale, D);
    const int nq = c->opt_nq;
    const int64_t rows = (int64_t)B * nq * Hq;
    const int G = Hq / Hkv;
    const bool has_suffix = Ks != nullptr && max_len > 0;
    const Parts parts = carve(Ws{c->ws, c->ws_bytes}, rows, D);
    LevelDev lv[HG_MAX_LEVELS];
    int64_t nmax = has_suffix ? max_len : 0;
    for (int i = 0; i < n_levels; ++i) {
        lv[i] = to_dev(levels[i], B);
        nmax += lv[i].max_rows;
    }
    hipStream_t s = c->stream;
    if (parts.cap < 1) return HG_ERR_WORKSPACE;
    if (nmax == 0) return fill_empty(O_out, o_dtype, LSE_out, rows, D, s);
    if (nmax >= (1LL << 30)) return HG_ERR_UNSUPPORTED;
    // (with one row per KV head the vector-ALU kernel is the faster comparison: 38 against 49 ms on config 3)
    if (c->opt_suffix_kernel != 1 && (c->opt_suffix_kernel == 2 || (nq * G >= 2 && auto_mfma(nq, G, (int)nmax, D)))) {
        // Several query rows per KV head: the per-sequence kernel on the matrix cores, once per level (every sequence
        // walks the block that covers it by itself) and once for the suffix, each writing its own partial results.
        int chunk = c->opt_naive_chunk > 0 ? round_up(c->opt_naive_chunk, 32) : 1024;
        const int cap = parts.cap < HG_MAX_PARTS ? parts.cap : HG_MAX_PARTS;
        auto parts_for = [&](int ch) {
            int n = has_suffix ? ceil_div(max_len, ch) : 0;
            for (int i = 0; i < n_levels; ++i) if (lv[i].max_rows > 0) n += ceil_div(lv[i].max_rows, ch);
            return n;
        };
        while (parts_for(chunk) > cap && chunk < (1 << 29)) chunk *= 2;
        if (parts_for(chunk) > cap) return HG_ERR_WORKSPACE;
        {   // item counts of every launch below, checked before anything is enqueued
            const int tile_rows = (nq * G <= 16 && c->opt_suffix_tile != 32) ? 16 : 32;
            const int64_t per = (int64_t)B * ceil_div(nq * G, tile_rows) * Hkv;
            if (per * parts_for(chunk) >= (1LL << 31)) return HG_ERR_UNSUPPORTED;
        }
        int first = 0;
        for (int i = 0; i < n_levels; ++i) {
            if (lv[i].max_rows <= 0) continue;
            const int n = ceil_div(lv[i].max_rows, chunk);
            rc = run_decode(Q, 1, &lv[i], lv[i].K, lv[i].V, nullptr, nullptr, lv[i].max_rows, B, nq, Hq, Hkv, D, scale, chunk, n, 1,
                            parts_out(parts, first), s, PagedDev{}, true, c->opt_suffix_ipw, true, KvFmt{}, c->opt_suffix_tile);
            if (rc) return rc;
            first += n;
        }
        if (has_suffix) {
            const int n = ceil_div(max_len, chunk);
            rc = run_decode(Q, 0, nullptr, Ks, Vs, offsets, lengths, max_len, B, nq, Hq, Hkv, D, scale, chunk, n, 1,
                            parts_out(parts, first), s, PagedDev{}, true, c->opt_suffix_ipw, false, KvFmt{}, c->opt_suffix_tile);
            if (rc) return rc;
            first += n;
        }
        return run_merge(first, parts, 0, D, O_out, o_dtype, LSE_out, s);
    }
    int chunk = c->opt_naive_chunk > 0 ? round_up(c->opt_naive_chunk, 32) : 512;
    int nchunks = ceil_div((int)nmax, chunk);
    const int cap = parts.cap < 32 ? parts.cap : 32;
    if (nchunks > cap) {
        chunk = round_up(ceil_div((int)nmax, cap), 32);
        nchunks = ceil_div((int)nmax, chunk);
    }
    rc = run_decode(Q, n_levels, lv, has_suffix ? Ks : nullptr, Vs, offsets, has_suffix ? lengths : nullptr, max_len, B, nq, Hq,
                    Hkv, D, scale, chunk, nchunks, pick_gt(G), parts_out(parts, 0), s);
    if (rc) return rc;
    return run_merge(nchunks, parts, 0, D, O_out, o_dtype, LSE_out, s);
}

int hg_read_stage_timings(hg_ctx* c, float* ms, int n_calls) {
    if (!c || !ms || n_calls < 0) return -HG_ERR_INVALID_ARG;
    if (!c->tev) return 0;
    if (hipSetDevice(c->device) != hipSuccess) return -HG_ERR_HIP;
    long long avail = c->tcalls < HG_TIMING_RING ? c->tcalls : HG_TIMING_RING;
    const int n = (int)(n_calls < avail ? n_calls : avail);
    for (int k = 0; k < n; ++k) {
        const int slot = (int)((c->tcalls - 1 - k) % HG_TIMING_RING);
        for (int st = 0; st < HG_MAX_STAGES; ++st) {
            float t = 0.f;
            if (c->tused[slot * HG_MAX_STAGES + st]) {
                hipEvent_t e0 = c->tev[(slot * HG_MAX_STAGES + st) * 2], e1 = c->tev[(slot * HG_MAX_STAGES + st) * 2 + 1];
                if (hipEventSynchronize(e1) != hipSuccess) return -HG_ERR_HIP;
                if (hipEventElapsedTime(&t, e0, e1) != hipSuccess) return -HG_ERR_HIP;
            }
            ms[k * HG_MAX_STAGES + st] = t;
        }
    }
    return n;
}

int hg_debug_wide_plan(int n_blocks, int max_rows, int max_seqs, int Hkv, int rows_per_seq, int max_parts, int slots_per_xcd,
                       int D, int out[9]) {
    if (!out || n_blocks < 1 || max_rows < 0 || max_seqs < 0 || Hkv < 1 || rows_per_seq < 1 || (D != 64 && D != 128)) return 0;
    hg::LevelDev lv{};
    lv.n_blocks = n_blocks;
    lv.max_rows = max_rows;
    lv.max_seqs = max_seqs;
    hg::WidePlan p{};
    if (!hg::plan_prefix_wide(lv, Hkv, rows_per_seq, D, max_parts, slots_per_xcd, &p)) return 0;
    out[0] = p.n_c; out[1] = p.ncols; out[2] = p.rowgroups; out[3] = p.T;
    out[4] = p.slots; out[5] = p.tpx; out[6] = p.quota; out[7] = p.nparts; out[8] = p.mode;
    return 1;
}

int hg_debug_wide_ranges(int n_blocks, int max_rows, int max_seqs, int Hkv, int rows_per_seq, int max_parts, int slots_per_xcd,
                         int D, int starts[257], int first_part[256]) {
    if (!starts || !first_part || n_blocks < 1 || max_rows < 0 || max_seqs < 0 || Hkv < 1 || rows_per_seq < 1 || (D != 64 && D != 128)) return 0;
    hg::LevelDev lv{};
    lv.n_blocks = n_blocks;
    lv.max_rows = max_rows;
    lv.max_seqs = max_seqs;
    hg::WidePlan p{};
    if (!hg::plan_prefix_wide(lv, Hkv, rows_per_seq, D, max_parts, slots_per_xcd, &p) || p.mode != 2) return 0;
    const int nteams = 8 * p.tpx;
    for (int t = 0; t <= nteams; ++t) starts[t] = p.starts[t];
    for (int t = 0; t < nteams; ++t) first_part[t] = p.first_part[t];
    return nteams;
}

int hg_debug_suffix_plan(int B, int nq, int Hq, int Hkv, int D, int max_len, int page_size, int out[4]) {
    if (!out || B < 1 || nq < 1 || Hkv < 1 || Hq < Hkv || Hq % Hkv != 0 || (D != 64 && D != 128) || max_len < 0 || page_size < 0) return 0;
    hg_ctx c{};   // default options
    c.opt_nq = nq;
    const SuffixPlan p = plan_suffix(&c, max_len, Hq / Hkv, B, nq, Hkv, D, page_size > 0, page_size > 0 ? 32 * page_size : 1 << 30);
    out[0] = p.chunk; out[1] = p.nchunks; out[2] = p.mfma ? 1 : 0; out[3] = p.gt;
    return 1;
}

int hg_debug_mfma_loop(hg_ctx* c, int random_operands, int iters, unsigned long long* clocks, float* sink) {
    if (!c || iters < 1 || !clocks || !sink) return HG_ERR_INVALID_ARG;
    if (hipSetDevice(c->device) != hipSuccess) return HG_ERR_HIP;
    return hip_rc(hg::launch_mfma_loop(iters, random_operands ? 1 : 0, clocks, sink, c->stream));
}

int hg_debug_stream_read(hg_ctx* c, const void* src, size_t bytes, float* sink) {
    if (!c || !src || !sink || bytes < 16 || reinterpret_cast<uintptr_t>(src) % 16 != 0) return HG_ERR_INVALID_ARG;
    if (hipSetDevice(c->device) != hipSuccess) return HG_ERR_HIP;
    return hip_rc(hg::launch_stream_read(src, bytes, sink, c->stream));
}

int hg_debug_xcd_of_workgroups(hg_ctx* c, int n_workgroups, int* out) {
    if (!c || !out || n_workgroups < 1 || n_workgroups > 4096) return HG_ERR_INVALID_ARG;
    if (hipSetDevice(c->device) != hipSuccess) return HG_ERR_HIP;
    return hip_rc(hg::launch_xcd_probe(n_workgroups, out, c->stream));
}

const char* hg_strerror(int code) {
    switch (code) {
        case HG_OK: return "ok";
        case HG_ERR_INVALID_ARG: return "invalid argument";
        case HG_ERR_UNSUPPORTED: return "unsupported shape or dtype";
        case HG_ERR_WORKSPACE: return "workspace too small";
        case HG_ERR_HIP: return "HIP runtime error";
        case HG_ERR_STATIC_LIMIT: return "too many query rows for the static scratch array of hg_hydragen_attn_static";
    }
    return "unknown error";
}

}  // extern "C"
