/*
 * hydragen.h - C ABI of the MI355X (gfx950) shared-prefix decode-attention library.
 *
 * The library computes exact softmax attention for a batch of decode queries
 * whose KV caches share prefixes, the way the Hydragen paper (arXiv 2402.05099)
 * states the problem:
 *
 *   - attention over ONE shared KV block, batched across all sequences' queries
 *     into a matrix-matrix product (Sec. 3.2, inter-sequence batching);
 *   - attention over each sequence's own ragged suffix KV (Sec. 3.2, last
 *     paragraph: computed per sequence, one query each);
 *   - each part returns its output and the log-sum-exp of its scaled scores
 *     (Eq. 4), and parts are merged with LSE weights into the exact
 *     full-context result (Eq. 5, proved in App. A);
 *   - the same at every vertex of a tree of shared blocks (Sec. 3.3).
 *
 * Conventions for every call
 *   - All tensor pointers are DEVICE pointers owned by the caller; the library
 *     never allocates or frees device memory after hg_create, never copies to
 *     or from the host, and never synchronises the host (hg_read_stage_timings, a
 *     measurement aid, is the one exception): work is enqueued on
 *     the context's stream and the call returns.  Arrays of lengths/offsets are
 *     read on the device, so their values may change between calls without any
 *     host work.  Scalar shape arguments are host values.
 *   - Layouts (row-major, innermost last), following the shapes in the
 *     docstring of App. B's attention routine with num_queries = 1:
 *       Q        bf16 [B, Hq, D]        one decode query per sequence
 *       K, V     bf16 [rows, Hkv, D]    a shared block stored once, or packed suffix rows
 *       O        [B, Hq, D]             fp32 or bf16 (o_dtype), LSE fp32 [B, Hq], natural log
 *     Query head h uses KV head h / (Hq / Hkv) (grouped-query attention).
 *   - An empty key set is legal everywhere: that part is O = 0, LSE = -inf and
 *     has weight zero in a merge; a row whose parts are all empty is O = 0,
 *     LSE = -inf.  (The paper is silent on empty parts.)
 *   - No causal mask: the decode query attends to every listed key
 *     (its own K/V row is expected to be the last suffix row already).
 *   - Several queries per sequence (App. B's num_queries > 1: the last nq tokens
 *     of every sequence are queried at once, as when draft tokens are verified).
 *     hg_set_option(ctx, HG_OPT_NUM_QUERIES, nq) makes every call of the context
 *     read Q as bf16 [B, nq, Hq, D] and write O [B, nq, Hq, D], LSE [B, nq, Hq];
 *     B stays the number of sequences in shapes, offsets, lengths and seq_off.
 *     Query t (0-based) of sequence b attends to every row of the shared blocks
 *     that cover b and to suffix rows [0, lengths[b] - (nq-1-t)): the nq tokens
 *     are the last nq suffix rows and a token does not see the ones after it
 *     (the paper gives the shape only; the causal reading is this library's).
 *     hg_merge is unaffected (it takes a row count).
 *   - scale <= 0 selects 1/sqrt(D) (Eq. 1).
 *   - Supported: D in {64, 128}; Hq % Hkv == 0; B*nq*Hq*D < 2^31; rows*Hkv*D < 2^31 per tensor.
 *   - Every call returns HG_OK or an error code.  Arguments, shapes, sizes and
 *     the workspace are checked before anything is enqueued: on those errors
 *     (every code but HG_ERR_HIP) nothing is enqueued and outputs are untouched.
 *     HG_ERR_HIP reports a failure of the HIP runtime itself, possibly after
 *     part of the call's work was enqueued: outputs are then undefined, and the
 *     library's second stream has been joined back to the context's stream.
 *     No C++ exception crosses this boundary.
 *   - Calls on one context must not overlap in time from several host threads.
 */
#ifndef HYDRAGEN_H
#define HYDRAGEN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hg_ctx hg_ctx;

enum { HG_OK = 0, HG_ERR_INVALID_ARG = 1, HG_ERR_UNSUPPORTED = 2, HG_ERR_WORKSPACE = 3, HG_ERR_HIP = 4, HG_ERR_STATIC_LIMIT = 5 };
enum { HG_F32 = 0, HG_BF16 = 1 };
enum { HG_KV_BF16 = 0, HG_KV_E4M3 = 1 }; /* element format of a paged suffix cache (hg_paged_kv.kv_format) */
enum { HG_MAX_LEVELS = 4, HG_MAX_PARTS = 64 };
enum { HG_STATIC_SCRATCH_BYTES = 67108864 }; /* 64 MiB: partial-result memory of hg_hydragen_attn_static */

/* Tunables for hg_set_option (0 = library default). */
enum {
    HG_OPT_PREFIX_SPLITS = 1, /* number of key-range splits of each shared block (>=1) */
    HG_OPT_SUFFIX_CHUNK = 2,  /* keys per work item of the suffix kernel (multiple of 32) */
    HG_OPT_OVERLAP = 3,       /* fused call: 0 shared-block and suffix kernels overlap on two streams, 1 one stream, 2 two streams with the shared-block kernels enqueued first */
    HG_OPT_NAIVE_CHUNK = 4,   /* keys per work item of the non-decomposed comparison kernel */
    HG_OPT_STAGE_TIMING = 5,  /* 1: hg_hydragen_attn brackets each of its kernels with timing events */
    HG_OPT_PREFIX_KERNEL = 6, /* shared-block kernel: 0 automatic (persistent 256-row kernel for blocks with more than 128 query rows, else the 128-row kernel), 1 always 128-row, 2 always 256-row */
    HG_OPT_WIDE_SLOTS = 7,    /* CUs per XCD (1..32) that the persistent 256-row kernel occupies; 0 = automatic */
    HG_OPT_NUM_QUERIES = 8,   /* queries per sequence, 1..64 (default 1 = decode); see "Several queries per sequence" below */
    HG_OPT_SUFFIX_ITEMS_PER_WAVE = 10, /* matrix-core suffix kernel: consecutive work items one wavefront takes (1..1024; 0 = automatic) */
    HG_OPT_SUFFIX_TILE_ROWS = 11, /* matrix-core suffix kernel: query rows per tile: 0 automatic (16 when a KV head serves at most 16 rows of a sequence, else 32), 16 (honoured under the same condition), 32 */
    HG_OPT_FUSED_KERNEL = 12, /* hg_hydragen_attn on a packed bf16 suffix cache: 0 automatic (one launch for the whole call when it holds so little work that launches and partial results would dominate, else one kernel per part and a merge), 1 always the separate kernels, 2 the single launch whenever it applies */
    HG_OPT_SUFFIX_KERNEL = 9  /* suffix kernel: 0 automatic (matrix-core kernel when a KV head serves several query rows of a sequence: two or more queries, three or more query heads, or two heads with max_len >= 256; or when D = 128 and max_len >= 384 whatever the rows; else the vector-ALU kernel), 1 always vector-ALU, 2 always matrix-core; an 8-bit cache with D = 64 is always read by the vector-ALU kernel */
};
enum { HG_TIMING_RING = 128, HG_MAX_STAGES = HG_MAX_LEVELS + 2 };

/*
 * Create a context bound to `device`, enqueueing on `hip_stream` (a hipStream_t, NULL = default stream).
 * `workspace` is caller-owned device memory of `workspace_bytes` bytes (256-byte aligned) that the
 * library uses for partial (O, LSE) results; it must stay valid until hg_destroy and must not be shared
 * by contexts used concurrently.  See hg_workspace_bytes.
 */
int hg_create(hg_ctx** out, int device, void* hip_stream, void* workspace, size_t workspace_bytes);
void hg_destroy(hg_ctx* ctx);
int hg_set_stream(hg_ctx* ctx, void* hip_stream);
int hg_set_option(hg_ctx* ctx, int option, int value);

/*
 * Bytes of workspace that hold `parts` fp32 partial results for B*Hq query rows: parts * B*Hq * (D+1) * 4,
 * rounded up to 256.  Every call needs room for at least (number of shared levels + 1) parts; more room
 * lets the library split long key ranges over more workgroups.  Pure host function.
 */
size_t hg_workspace_bytes(int B, int Hq, int D, int parts);

/*
 * Attention of every query over ONE shared KV block (Sec. 3.2): all B*Hq/Hkv query rows that use a KV head
 * are stacked into one matrix against that head's P keys.  P == 0 is legal.
 *   Kp, Vp : bf16 [P, Hkv, D];  O : [B, Hq, D] of o_dtype;  LSE : fp32 [B, Hq].
 */
int hg_prefix_attn(hg_ctx* ctx, const void* Q, const void* Kp, const void* Vp,
                   int B, int Hq, int Hkv, int D, int P, float scale,
                   void* O, int o_dtype, float* LSE);

/*
 * One level of a sharing tree (Sec. 3.3): n_blocks shared blocks stored back to back in K/V.
 * Block g owns KV rows [kv_off[g], kv_off[g+1]) and is attended to by the contiguous sequences
 * [seq_off[g], seq_off[g+1]) (sequences are in tree order).  kv_off/seq_off are DEVICE int32[n_blocks+1],
 * non-decreasing.  max_rows / max_seqs are host upper bounds on rows and sequences per block; a block
 * exceeding them is truncated.  Rows of K/V that are no block's keys (the truncated tail of a block, rows before the
 * first block) may hold anything, NaN included: the kernels may read them but never give them a weight.
 * With n_blocks == 1 both arrays may be NULL: the block is then rows
 * [0, max_rows) shared by sequences [0, B).  Sequences not covered by any block get O = 0, LSE = -inf.
 */
typedef struct {
    const void* K;
    const void* V;
    int n_blocks;
    const int32_t* kv_off;
    const int32_t* seq_off;
    int max_rows;
    int max_seqs;
} hg_level;

int hg_prefix_attn_grouped(hg_ctx* ctx, const void* Q, const hg_level* level,
                           int B, int Hq, int Hkv, int D, float scale,
                           void* O, int o_dtype, float* LSE);

/*
 * Per-sequence attention over ragged suffix KV (Sec. 3.2, last paragraph).  Sequence b owns rows
 * [offsets[b], offsets[b] + lengths[b]) of Ks/Vs (bf16 [T, Hkv, D]); offsets/lengths are DEVICE int32[B];
 * a padded [B, Lmax, Hkv, D] cache is offsets[b] = b * Lmax.  lengths[b] == 0 is legal; lengths above
 * max_len (a host upper bound) are truncated to max_len; max_len * Hkv * D must stay below 2^31 (else
 * HG_ERR_UNSUPPORTED).  Rows of Ks/Vs that no sequence owns (padding, slots of
 * empty sequences) may hold anything, NaN included: they are never given a weight and never reach a result.
 */
int hg_suffix_attn(hg_ctx* ctx, const void* Q, const void* Ks, const void* Vs,
                   const int32_t* offsets, const int32_t* lengths, int max_len,
                   int B, int Hq, int Hkv, int D, float scale,
                   void* O, int o_dtype, float* LSE);

/*
 * n-way LSE merge (Eq. 5 generalised; App. B gives the two-part form):
 *   m = max_i LSE_i;  w_i = exp(LSE_i - m);  O = sum_i w_i O_i / sum_i w_i;  LSE = m + log sum_i w_i.
 * O_parts / LSE_parts are HOST arrays of n device pointers ([rows, D] of o_dtype_in, fp32 [rows]);
 * 1 <= n <= HG_MAX_PARTS.  LSE_out may be NULL.  O_out may alias O_parts[0] when the dtypes are equal.
 */
int hg_merge(hg_ctx* ctx, int n, const void* const* O_parts, const float* const* LSE_parts, int o_dtype_in,
             int64_t rows, int D, void* O_out, int o_dtype_out, float* LSE_out);

/*
 * Fused Hydragen attention (App. B's top-level routine, generalised to n_levels >= 0 levels of shared
 * blocks): one batched attention per level, the suffix attention, and the merge of all partial results.
 * The suffix may be absent (Ks == NULL: lengths are then taken as 0).
 * O_out : [B, Hq, D] of o_dtype;  LSE_out : fp32 [B, Hq] or NULL.
 */
int hg_hydragen_attn(hg_ctx* ctx, const void* Q, int n_levels, const hg_level* levels,
                     const void* Ks, const void* Vs, const int32_t* offsets, const int32_t* lengths, int max_len,
                     int B, int Hq, int Hkv, int D, float scale,
                     void* O_out, int o_dtype, float* LSE_out);

/*
 * hg_hydragen_attn for callers that cannot hand the library memory from an allocator and must not trigger an
 * allocation themselves: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same result and same kernels as hg_hydragen_attn, but the fp32 partial results live in a fixed array of
 * HG_STATIC_SCRATCH_BYTES (64 MiB) inside the library's device image instead of the context's workspace (which may
 * be absent: hg_create(.., NULL, 0)); the call allocates and frees nothing, on the device or through any library.
 * Every GPU the library is loaded on holds the array until the process ends; its address is looked up by hg_create
 * on the context's device.
 * Limit: one partial result per non-empty shared level plus one for the suffix must fit, i.e.
 *   (levels + 1) * B * nq * Hq * (D + 1) * 4 <= HG_STATIC_SCRATCH_BYTES   (two parts at D = 128: B * nq * Hq <= 65027),
 * else HG_ERR_STATIC_LIMIT and nothing is enqueued; with room to spare, long key ranges are split as in
 * hg_hydragen_attn.  Devices numbered 64 and above: HG_ERR_UNSUPPORTED.
 * All calls on one GPU share the array, whatever their context or stream: two such calls that overlap in time on one
 * GPU race on it (calls ordered on one stream do not).  Nothing in it needs to start at zero and nothing is kept
 * from call to call: every part a merge reads is written, or marked empty, by that call's own kernels.
 */
int hg_hydragen_attn_static(hg_ctx* ctx, const void* Q, int n_levels, const hg_level* levels,
                            const void* Ks, const void* Vs, const int32_t* offsets, const int32_t* lengths, int max_len,
                            int B, int Hq, int Hkv, int D, float scale,
                            void* O_out, int o_dtype, float* LSE_out);

/*
 * Paged suffix cache.  Sec. 3.5 contrasts Hydragen's plain suffix cache with PagedAttention's paged one (see also
 * Sec. 1 and Sec. 6); the decomposition itself (Sec. 3.1) does not care how suffix rows are stored, so the suffix part may also
 * read through a page table.  K, V: bf16 [n_pages * page_size, Hkv, D], one pool of fixed-size pages shared by all
 * sequences.  Suffix row j of sequence b is pool row page_table[b * table_stride + j / page_size] * page_size +
 * j % page_size.  page_table is DEVICE int32 [B, table_stride] and is read on the device at run time; only entries
 * of pages that hold rows below lengths[b] are read, and an entry outside [0, n_pages) is clamped into that range
 * (so a bad table gives wrong numbers, never an access outside the pool).  page_size is a power of two in
 * [16, 1024]; table_stride >= ceil(max_len / page_size); n_pages * page_size * Hkv * D < 2^31.
 * Which page a sequence gets is the caller's business (a host-side allocator): the library only reads the table.
 * kv_format = HG_KV_E4M3: the pool holds 8-bit E4M3 codes, one byte per element, with the scales k_scale / v_scale
 * (see "8-bit suffix cache" below; the scales are ignored for HG_KV_BF16).  Zero-initialise the struct to get bf16.
 */
typedef struct {
    void* K;
    void* V;
    const int32_t* page_table;
    int page_size;
    int table_stride;
    int n_pages;
    int kv_format;
    float k_scale;
    float v_scale;
} hg_paged_kv;

/*
 * hg_suffix_attn / hg_hydragen_attn with the suffix rows read through a page table: same results as the
 * calls above on the rows that the table designates (lengths: DEVICE int32[B], rows above max_len are ignored).
 * A work item of the vector-ALU suffix kernel covers at most 32 pages, so when that kernel runs (see
 * HG_OPT_SUFFIX_KERNEL) the workspace must have room for ceil(max_len / (32 * page_size)) partial results (plus one
 * per shared level), else HG_ERR_WORKSPACE.  Pool rows that no sequence owns (page tails, free pages) may hold
 * anything, NaN included.
 */
int hg_suffix_attn_paged(hg_ctx* ctx, const void* Q, const hg_paged_kv* kv, const int32_t* lengths, int max_len,
                         int B, int Hq, int Hkv, int D, float scale, void* O, int o_dtype, float* LSE);
int hg_hydragen_attn_paged(hg_ctx* ctx, const void* Q, int n_levels, const hg_level* levels,
                           const hg_paged_kv* kv, const int32_t* lengths, int max_len,
                           int B, int Hq, int Hkv, int D, float scale,
                           void* O_out, int o_dtype, float* LSE_out);

/*
 * The KV-cache update of a decode step (Sec. 2.2: the keys and values of every earlier token are kept, and each
 * step adds those of the newest token; Sec. 3.5: suffix lengths change from step to step under a captured graph, so
 * the update runs on the device).  Knew, Vnew: bf16 [B, nq, Hkv, D], the rows of the nq new tokens of every
 * sequence (nq = HG_OPT_NUM_QUERIES, 1 by default).  Row t of sequence b is written to suffix row
 * lengths[b] + t (addressed as in hg_suffix_attn, or through the page table, whose entry for that page must already
 * be set), and lengths[b] becomes min(lengths[b] + nq, capacity): rows at or above `capacity` (a host value, the
 * rows reserved per sequence) are dropped.  lengths is DEVICE int32[B], read and written on the device; nothing
 * comes back to the host.  Calling hg_kv_append and then an attention call with max_len >= the new lengths is
 * one decode step: the newest token's query then sees its own key as the last suffix row.
 */
int hg_kv_append(hg_ctx* ctx, const void* Knew, const void* Vnew, void* Ks, void* Vs,
                 const int32_t* offsets, int32_t* lengths, int capacity, int B, int Hkv, int D);
int hg_kv_append_paged(hg_ctx* ctx, const void* Knew, const void* Vnew, const hg_paged_kv* kv,
                       int32_t* lengths, int capacity, int B, int Hkv, int D);

/*
 * 8-bit suffix cache (not in the paper: a bandwidth variant of the suffix part of Sec. 3.2, the part of the method
 * that is bound by the bytes it reads).  Ks8, Vs8: one byte per element, [T, Hkv, D], OCP 8-bit floating point E4M3
 * codes (1 sign, 4 exponent bits with bias 7, 3 mantissa bits; no infinities, largest value 448); a key is
 * code * k_scale and a value code * v_scale, with one finite positive fp32 scale per tensor.  Rows are addressed as
 * in hg_suffix_attn (offsets / lengths: DEVICE int32[B]).  Shared levels, Q and the results keep their formats.
 *   hg_suffix_attn_fp8 / hg_hydragen_attn_fp8: hg_suffix_attn / hg_hydragen_attn over such a cache: the attention
 *     of the decoded values (the codes are expanded exactly; all arithmetic is fp32).  Rows that no sequence owns
 *     may hold any code.  The suffix kernel is chosen as for a bf16 cache (HG_OPT_SUFFIX_KERNEL).
 *   hg_kv_append_fp8: hg_kv_append with the new bf16 rows quantised on the way in:
 *     code = nearest E4M3 value to (x / scale) (fp32 quotient), ties to the even code, magnitudes above 448 -> 448.
 * Invalid scales (zero, negative, infinite, NaN) give HG_ERR_INVALID_ARG.
 * A paged 8-bit cache goes through the paged calls above with hg_paged_kv.kv_format = HG_KV_E4M3
 * (hg_suffix_attn_paged, hg_hydragen_attn_paged, hg_kv_append_paged: same meaning, rows addressed through the table).
 */
int hg_suffix_attn_fp8(hg_ctx* ctx, const void* Q, const void* Ks8, const void* Vs8, float k_scale, float v_scale,
                       const int32_t* offsets, const int32_t* lengths, int max_len,
                       int B, int Hq, int Hkv, int D, float scale, void* O, int o_dtype, float* LSE);
int hg_hydragen_attn_fp8(hg_ctx* ctx, const void* Q, int n_levels, const hg_level* levels,
                         const void* Ks8, const void* Vs8, float k_scale, float v_scale,
                         const int32_t* offsets, const int32_t* lengths, int max_len,
                         int B, int Hq, int Hkv, int D, float scale, void* O_out, int o_dtype, float* LSE_out);
int hg_kv_append_fp8(hg_ctx* ctx, const void* Knew, const void* Vnew, void* Ks8, void* Vs8, float k_scale, float v_scale,
                     const int32_t* offsets, int32_t* lengths, int capacity, int B, int Hkv, int D);

/*
 * Non-decomposed comparison (the behaviour Sec. 1 and Sec. 2.3 attribute to per-sequence decode kernels):
 * same arguments and result as hg_hydragen_attn, but every sequence walks its whole key list
 * (shared blocks, then suffix) by itself, so shared rows are re-read once per sequence.
 */
int hg_naive_attn(hg_ctx* ctx, const void* Q, int n_levels, const hg_level* levels,
                  const void* Ks, const void* Vs, const int32_t* offsets, const int32_t* lengths, int max_len,
                  int B, int Hq, int Hkv, int D, float scale,
                  void* O_out, int o_dtype, float* LSE_out);

/*
 * Stage timings of the most recent fused calls (measurement aid; needs HG_OPT_STAGE_TIMING = 1 before them).
 * Each hg_hydragen_attn call then records device-side timing events around its kernels, on the streams the
 * kernels run on, into a ring of HG_TIMING_RING slots; nothing is synchronised at call time.
 * hg_read_stage_timings waits for the newest recorded call to finish, then fills
 *   ms[c * HG_MAX_STAGES + s] = milliseconds of stage s of the c-th most recent call, c = 0 .. n_calls-1
 * (HOST array of n_calls * HG_MAX_STAGES floats), with stages: 0 = suffix kernel, 1 .. n_levels = the
 * shared-block kernel of each non-empty level in order, n_levels + 1 = merge kernel; unused stages are 0.
 * Returns the number of calls filled (<= n_calls, <= calls recorded since timing was enabled, <= ring size)
 * or a negative error code.
 */
int hg_read_stage_timings(hg_ctx* ctx, float* ms, int n_calls);

const char* hg_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* HYDRAGEN_H */
