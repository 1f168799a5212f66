/*
 * hydragen_debug.h - views of the library's work partitioning and two measurement kernels, for tests, tuning and the
 * benchmark.  Nothing here is part of the attention API (include/hydragen.h); the symbols live in the same library.
 */
#ifndef HYDRAGEN_DEBUG_H
#define HYDRAGEN_DEBUG_H

#include "hydragen.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Host-only views of the library's work partitioning (no device is touched, no context needed).
 *
 * hg_debug_wide_plan: the partition that the persistent 256-row shared-block kernel would use for a level of n_blocks
 * blocks of at most max_rows keys and max_seqs sequences, Hkv KV heads, rows_per_seq query rows per sequence and KV
 * head (queries per sequence x query heads per KV head), head dimension D (128 or 64), at most max_parts partial results
 * per row, on slots_per_xcd CUs of each of the 8 XCDs.  Fills out[9] = { stages per column (32 keys each at D = 128, 64
 * keys each at D = 64), columns, row groups, workgroups per
 * team, slots, teams per XCD, stages per team, partial results per row, mode } and returns 1, or returns 0 if the level
 * does not fit.  With n_c stages per column, C columns and N = 8 * teams per XCD teams, team t walks the flattened
 * (column, stage) positions
 *   mode 0:         [t * quota, min((t+1) * quota, C * n_c)); a column cut by such a range yields one partial result
 *                   per piece, numbered t - floor(column * n_c / quota);
 *   mode 1, C <= N: column c = floor(t * C / N) belongs to the teams ceil(c * N / C) .. ceil((c+1) * N / C) - 1; the
 *                   i-th of its n teams walks its stages [floor(i * n_c / n), floor((i+1) * n_c / n)), part i;
 *   mode 1, C > N:  the whole columns floor(t * C / N) .. floor((t+1) * C / N) - 1, part 0;
 *   mode 2:         [starts[t], starts[t+1]) from hg_debug_wide_ranges: ranges of equal cost, a column boundary inside a
 *                   range counting as 9 stages (the workgroups store a result and load a Q tile there); the team's
 *                   first piece is part first_part[t] of its column, its later pieces part 0 of theirs.  out[6] is then
 *                   the cost bound, not a length.
 *
 * hg_debug_wide_ranges: the same arguments; fills starts[257] and first_part[256] for a mode 2 partition and returns the
 * number of teams N (entries beyond N are not written), or returns 0 if the partition is not of mode 2.
 *
 * hg_debug_suffix_plan: the suffix kernel and chunking chosen with default options for B sequences of at most max_len
 * suffix rows, nq queries each, Hq / Hkv heads of dimension D (page_size > 0: paged cache).  Fills out[4] = { keys per
 * work item, work items per row (= partial results), 1 if the matrix-core kernel runs, query heads per vector-ALU
 * work item } and returns 1, or 0 on invalid arguments.
 */
int hg_debug_wide_plan(int n_blocks, int max_rows, int max_seqs, int Hkv, int rows_per_seq, int max_parts,
                       int slots_per_xcd, int D, int out[9]);
int hg_debug_wide_ranges(int n_blocks, int max_rows, int max_seqs, int Hkv, int rows_per_seq, int max_parts,
                         int slots_per_xcd, int D, int starts[257], int first_part[256]);
int hg_debug_suffix_plan(int B, int nq, int Hq, int Hkv, int D, int max_len, int page_size, int out[4]);

/*
 * What the chip sustains on the two resources the attention kernels are priced against (Sec. 4.2 and App. D.2 time
 * kernels on the machine at hand; these give that machine's ceilings).  Both only enqueue a kernel on the context's
 * stream; the caller times it.
 *
 * hg_debug_mfma_loop: a register-only loop of the matrix instruction the shared-block kernels use
 * (v_mfma_f32_32x32x16_bf16) on every CU: 256 workgroups x 8 wavefronts x iters x 16 instructions of 32768 flop.
 * random_operands = 0: constant operands; 1: pseudo-random bf16 values (data-dependent switching: the chip's power
 * limit then sets the clock).  clocks: DEVICE uint64[2], written by workgroup 0 = { shader-clock cycles, 100 MHz
 * real-time ticks } of its loop (cycles / ticks x 100 MHz = the clock the chip ran at).  sink: DEVICE float[1].
 *
 * hg_debug_stream_read: every CU reads `bytes` bytes at src (DEVICE, 16-byte aligned) once, with 16-byte loads.
 *
 * hg_debug_xcd_of_workgroups: launches n_workgroups (1..4096) workgroups shaped like the persistent shared-block
 * kernel's (512 threads, all of a CU's LDS); workgroup i writes the id of the XCD it runs on to out[i] (DEVICE
 * int32[n_workgroups]).  The shared-block kernels assume that out[i] == out[j] exactly when i % 8 == j % 8 (the
 * XCDs take workgroups round-robin, starting wherever the launch before stopped) when they put the workgroups that share
 * K/V rows on one XCD (Sec. 3.2's batching is the same either way: only L2 hits depend on it).
 */
int hg_debug_mfma_loop(hg_ctx* ctx, int random_operands, int iters, unsigned long long* clocks, float* sink);
int hg_debug_stream_read(hg_ctx* ctx, const void* src, size_t bytes, float* sink);
int hg_debug_xcd_of_workgroups(hg_ctx* ctx, int n_workgroups, int* out);

#ifdef __cplusplus
}
#endif
#endif /* HYDRAGEN_DEBUG_H */
