/*
 * flora_debug.h -- test, measurement and tuning hooks of libflora.so.
 *
 * Nothing here is part of the method (include/flora.h holds that); these entry points exist
 * for the test-suite (the work tables the host builds), the profiler yardstick (a plain copy
 * of known size) and launch-shape sweeps.  Conventions as in flora.h.
 */
#ifndef FLORA_DEBUG_H_
#define FLORA_DEBUG_H_

#include "flora.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Test hook, host only (touches no GPU): the table of workgroups the library would launch for
 * this set of shapes.  kind 0: flora_compress, 1: flora_decompress and the update passes,
 * 2: the state <- state T pass of the transfer, 3: its T = A^T A' pass (ranks 64 and above; a
 * workgroup takes columns [first column, end column) of chunk `part` and slab `rank slice` of
 * the rows of T), 4: flora_compress_mapped with a map other than the identity.  Returns the number of workgroups (or a
 * negative flora_status_t) and writes up to `cap` of them to `out`, 12 int64 each:
 * matrix, first row, rows, first column, rank slice (compress) or column chunk (decompress),
 * row-block index, end column, part, number of parts, arrival counter, offset of the partial
 * products in the workspace (floats), 0.  info (5 int64, may be NULL): rows-per-workgroup code,
 * vector-kernel flag, columns per part, floats of partial products, arrival counters. */
int64_t flora_debug_work_items(int kind, const flora_matrix_t* mats, int count, int r,
                               flora_dtype_t grad_dtype, int64_t* out, int64_t cap, int64_t* info);

/* Test hook, host only: the bytes of a caller-owned workspace (flora_set_workspace) that one
 * plan of the library occupies for this set of shapes (count <= 448): plan_kind 0 flora_compress,
 * 1 flora_decompress / SGD update, 2 the transfer, 3 the Adafactor updates, 4 flora_weight_sumsq.
 * = tables + work area + 8 descriptor images, each rounded up to 256 bytes.  Negative
 * flora_status_t on bad arguments. */
int64_t flora_debug_plan_bytes(int plan_kind, const flora_matrix_t* mats, int count, int r, flora_dtype_t grad_dtype);

/* Measurement hook: a plain device-to-device copy kernel of `bytes` bytes (a multiple of 16;
 * both DEVICE pointers 16-byte aligned, not overlapping).  Profiler byte counters for the
 * hot-path kernels are scaled by what they read for this copy of known size. */
int flora_debug_copy(const void* src, void* dst, size_t bytes, void* hip_stream);

/* Measurement hooks: plain kernels that show what this chip gives a kernel that does nothing but
 * the one thing, to judge the hot-path kernels against (bench.py --ceilings times them).
 * flora_debug_read reads `bytes` bytes (a multiple of 16) at src (DEVICE, 16-byte aligned) and
 * stores nothing (sink: DEVICE, 4 bytes, never written).  pattern 0: contiguous, 16 bytes per lane;
 * pattern 1: the compress kernels' operand pattern over a matrix of bytes / row_bytes rows: a wave
 * instruction covers 16 rows x 64 contiguous bytes, a wave owns 16 rows x chunk_bytes (a multiple
 * of 256 that divides row_bytes), a workgroup 64 rows.
 * flora_debug_compute_loop launches 2048 workgroups of four waves running `iters` rounds of a
 * register-resident loop: kind 0 v_mfma_f32_16x16x32_bf16 (8 per round), 1 v_mfma_f32_32x32x16_bf16
 * (4 per round), 2 v_mfma_f32_16x16x4_f32 (8 per round), 3 the projection's generator (one
 * Philox4x32-10 + Box-Muller quad per round and thread); *work_out (HOST) receives the flops
 * (kinds 0-2) or normals (kind 3) the launch performs. */
int flora_debug_read(const void* src, size_t bytes, int pattern, size_t row_bytes, int chunk_bytes, void* sink,
                     void* hip_stream);
int flora_debug_compute_loop(int kind, int iters, void* sink, double* work_out, void* hip_stream);

/* Tuning hook for sweeps: overrides a launch-shape choice the library otherwise makes itself
 * (value 0 restores the default).  Names: "compress_f32_kgroups" (1, 2, 4: column groups per
 * workgroup in the fp32 compress kernel), "compress_f32_mt" (1, 2: rows per workgroup / 64 in
 * the same kernel), "compress_bf16_mt" (1, 2, 4: rows per workgroup / 128
 * in the bf16 compress kernel; 8 / 16 / 32: its wide variant with 512 / 256 / 128 rows, used only when
 * every m is a multiple of 8), "compress_splitk_cols" (a multiple of 64: in the wide variant,
 * share the columns of a row block between workgroups of about this many columns each), "decompress_rows" (a multiple of 32: rows per workgroup in the
 * decompress / update kernels), "decompress_vec" (1: always the 4-byte-per-lane kernel at
 * ranks >= 64, 2: the 16-byte-per-lane kernel whenever every m is a multiple of 4, which is
 * also the default), "factored_gram" (the factored rule at ranks >= 64: 1 reduction passes over the decompressed
 * gradient, 2 quadratic forms in r x r Gram matrices; by default whichever is less arithmetic for the
 * set), "gram_chunk" (a multiple of 64: entries of m or n per workgroup of the Gram sums),
 * "update_wpolicy" (the update passes: 1 plain
 * accesses to the weights, 2 reads with the non-temporal hint, 3 writes with it, 4 both; by
 * default chosen from the size of the call's weights against the 256 MB last-level cache: a
 * caller that updates a large model a few matrices per call may want 4).  Results never depend
 * on these beyond summation order.
 * Unknown name or value: FLORA_ERR_INVALID.  Drops the cached descriptor tables. */
int flora_set_tuning(const char* name, int value);

#ifdef __cplusplus
}
#endif
#endif /* FLORA_DEBUG_H_ */
