/*
 * flora.h -- C ABI of the MI355X (gfx950) library for Flora's hot path
 * (arXiv 2402.03293: random-projection compression of weight gradients).
 *
 * Orientation.  The paper writes the projection as A_p in R^{r x m} and
 * compresses with G A_p^T (Algorithm 1, compression line).  This library uses
 * A = A_p^T in R^{m x r}: for a weight W and gradient G in R^{n x m}
 * (row-major, leading dimension m) the compressed state (the accumulator C of
 * Algorithm 1 or the momentum M of Algorithm 2) is n x r, row-major fp32.
 * A is never stored: every kernel regenerates the tiles it needs from the
 * 64-bit seed (Section 2.4, "Memory analysis": only the seed is kept).
 *
 * The generator (the paper fixes only "N_s(0, 1/r)"; this is the library's
 * definition, version FLORA_GENERATOR_VERSION):
 *   words  = Philox4x32-10(counter = (j mod 2^32, q, j >> 32, 0),
 *                          key     = (seed mod 2^32, seed >> 32))
 *   u(x)   = ((x >> 9) + 1/2) * 2^-23                       (23 bits, never 0 or 1)
 *   (z0,z1) = sqrt(-2 ln u(w0)) * (cos, sin)(2 pi u(w1)),  (z2,z3) likewise from (w2,w3)
 *   A[j, 4q + i] = z_i / sqrt(r)
 *
 * Conventions for every entry point
 *   - `mats` is a HOST array of `count` descriptors; every pointer inside a
 *     descriptor is a DEVICE pointer owned by the caller, 16-byte aligned.
 *     grad / weight / state of one matrix must not alias.
 *     1 <= n < 2^31 - 1024 and 1 <= m <= 2^24, else FLORA_ERR_INVALID.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default
 *     stream).  All work is enqueued on it; no call synchronises the device
 *     or the stream.
 *   - The return value is a flora_status_t.  Arguments are validated on the
 *     host before anything is enqueued: on FLORA_ERR_INVALID or
 *     FLORA_ERR_UNSUPPORTED nothing has been launched.
 *   - Supported ranks: r in {8, 16, 32} (fp32 matrix cores; fp32 or bf16
 *     gradients are used exactly) and r in {64, 128, 256} (bf16 matrix cores,
 *     fp32 accumulation; A and, when decompressing, the state are rounded to
 *     bf16 on the fly; bf16 gradients are used exactly and take the fastest
 *     kernel, fp32 gradients are rounded to bf16, nearest even, in registers).
 *     Other r: FLORA_ERR_UNSUPPORTED.
 *   - Device memory beyond the caller's tensors ("workspace").  Per (set of matrix shapes,
 *     stream) the library needs the work tables of the grouped launches, the r x r transfer
 *     matrices, statistic partials, for small launches the partial products and arrival counters
 *     of row blocks whose columns are shared between workgroups, and device copies of descriptor
 *     tables.  By default it allocates this with hipMalloc (and pinned staging with
 *     hipHostMalloc) the first time a set of shapes is seen on a stream and reuses it afterwards;
 *     flora_shutdown() releases it.  A caller that wants to place and count that memory itself
 *     hands the library a buffer with flora_set_workspace(): from then on everything above is
 *     carved from the caller's buffer and the library calls neither hipMalloc nor hipHostMalloc.
 *     Either way a call whose pointers have been seen before uploads nothing; one with new
 *     pointers (another buffer of a ring, a freshly allocated gradient) costs one small
 *     asynchronous copy and no allocation or synchronisation, so calling once per matrix from a
 *     training loop stays cheap.  No per-matrix state (seed, step, epoch) is kept between calls:
 *     that lives with the caller.
 *   - HIP graphs.  A call whose shapes and pointers have been seen on its stream is kernel
 *     launches only and may be recorded into a HIP graph (seeds are kernel arguments: a resample
 *     means a new capture or a node update).  The captured kernels read the library's cached
 *     tables and descriptor images, so these must stay where they are for as long as the graph is
 *     replayed: between capture and the last replay do not call flora_set_tuning,
 *     flora_set_workspace or flora_shutdown, do not let calls with other pointer sets on the same
 *     shapes push the captured image out (the library keeps the 16 most recently used images
 *     per plan for sets of more than 32 matrices, 64 for sets of 5 to 32, 512 for smaller ones;
 *     8 with a caller-owned workspace), and stay below 1024 distinct (shape set, stream, entry
 *     point) combinations.
 *   - Calls on one stream execute in order.  Calls issued concurrently from
 *     several host threads are serialised by an internal lock.  Two calls on
 *     the same matrices (the same grad / weight / state pointers) must not
 *     run at the same time on different streams: they would race on the
 *     caller's state.  (Workspace is per stream, so calls on different
 *     matrices of equal shapes may overlap on different streams.)
 *   - Results are bitwise repeatable: every reduction has a fixed order (no
 *     floating-point atomics), also where workgroups combine partial products.
 */
#ifndef FLORA_H_
#define FLORA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FLORA_GENERATOR_VERSION 1

typedef enum { FLORA_F32 = 0, FLORA_BF16 = 1 } flora_dtype_t;

typedef enum {
    FLORA_OK = 0,
    FLORA_ERR_INVALID = -1,      /* null pointer, n/m/count out of range, bad enum, misaligned pointer */
    FLORA_ERR_UNSUPPORTED = -2,  /* valid request with no kernel (rank or dtype outside the list above) */
    FLORA_ERR_DEVICE = -3,       /* a HIP call failed; see flora_last_device_error()                    */
    FLORA_ERR_TOO_LARGE = -4     /* flora_momentum_transfer_static: the request needs more than the fixed buffer */
} flora_status_t;

/* One weight matrix.  Fields a given call does not use may be NULL / 0. */
typedef struct flora_matrix {
    const void* grad;      /* device, n x m row-major, fp32 or bf16; read only                            */
    void*       weight;    /* device, n x m row-major, fp32 or bf16; read-modify-write by the update calls */
    float*      state;     /* device, n x r row-major fp32: C (Algorithm 1) or M (Algorithm 2)           */
    float*      row_stat;  /* device, n floats: factored rule's row second moment R, else NULL           */
    float*      col_stat;  /* device, m floats: factored rule's column second moment K, else NULL        */
    int64_t     n;         /* rows of G and W                                                            */
    int64_t     m;         /* columns of G and W = the compressed axis = rows of A                       */
    uint64_t    seed;      /* seed s_W of the current projection                                         */
    uint64_t    seed_next; /* seed of the projection to move to (flora_momentum_transfer, fused step)    */
    float*      second_moment; /* device, n x m fp32: unfactored rule's second moment V, else NULL       */
    float*      weight_sumsq;  /* device, 1 float: sum of W^2 over the matrix (parameter scale), else NULL */
} flora_matrix_t;

typedef enum { FLORA_RULE_SGD = 0, FLORA_RULE_FACTORED = 1, FLORA_RULE_UNFACTORED = 2 } flora_rule_t;

/* How the decompressed gradient Gt = alpha * state A^T is applied to W. */
typedef struct flora_update {
    int   rule;              /* flora_rule_t                                                            */
    float lr;                /* learning rate eta                                                       */
    float alpha;             /* 1/tau for Algorithm 1 (arithmetic mean over the cycle), 1 for Alg. 2    */
    float beta2;             /* Adafactor rules: decay of the second moment (0 = this step's alone)     */
    float eps1;              /* Adafactor rules: added to Gt^2                                          */
    float clip_d;            /* Adafactor rules: RMS clipping threshold, 0 = no clipping                */
    int   zero_state_after;  /* non-zero: state <- 0 once the update has read it (end of an Alg. 1 cycle) */
    int   scale_parameter;   /* Adafactor rules, non-zero: the step is lr * max(eps2, RMS(W)), lr then
                                being the relative step size rho_t; ignored by FLORA_RULE_SGD           */
    float eps2;              /* floor of the parameter scale RMS(W)                                     */
    float step_weight_mib;   /* 0 when this call updates everything the caller's optimizer step updates;
                                otherwise (one call per layer, say) the MiB of weights, plus elementwise
                                second moments, that the whole step passes through the library: the
                                library picks the cache policy of these arrays from the larger of this
                                and the call's own size (a set beyond the 256 MB last-level cache is
                                streamed past it).  Never changes results.  >= 0 and finite           */
} flora_update_t;

/* Compression (Algorithm 1, compression line: a = b = 1;  Algorithm 2, EMA
 * line: a = beta, b = 1 - beta):
 *     state <- a * state + b * (grad A(seed))
 * Uses grad, state, n, m, seed.  grad is read once, state is read and written
 * once, nothing else is touched. */
int flora_compress(const flora_matrix_t* mats, int count, int r, flora_dtype_t grad_dtype,
                   float a, float b, void* hip_stream);

/* An elementwise map applied to `grad` on its way into the compression. */
typedef enum { FLORA_INPUT_IDENTITY = 0, FLORA_INPUT_SQUARE = 1 } flora_input_map_t;

/* The compressed EMA of another statistic (closing remark of Section 2.4, "Sublinear memory momentum": the scheme of
 * Algorithm 2 extends to other EMA-based statistics):
 *     state <- a * state + b * (phi(grad) A(seed)),   phi elementwise
 * FLORA_INPUT_IDENTITY is flora_compress; FLORA_INPUT_SQUARE makes `state` the compressed
 * second moment (a = beta2, b = 1 - beta2), squared in registers so that grad^2 is never
 * written anywhere.  flora_decompress of such a state is an unbiased estimate of the statistic
 * (not a non-negative one), and flora_momentum_transfer moves it to a new projection like any
 * other state.  At ranks <= 32 the square is taken in fp32; at ranks >= 64 it is squared in
 * fp32 and rounded to bf16 for the matrix cores.  Arguments, requirements and errors as for
 * flora_compress; an unknown map is FLORA_ERR_INVALID. */
int flora_compress_mapped(const flora_matrix_t* mats, int count, int r, flora_dtype_t grad_dtype,
                          flora_input_map_t map, float a, float b, void* hip_stream);

/* Decompression (Algorithm 1, decompression line, with the printed 1/n read
 * as 1/tau; Algorithm 2, yield):
 *     out[l] <- alpha * state A(seed)^T        (n x m, row-major, out_dtype)
 * `out` is a HOST array of `count` DEVICE pointers.  Uses state, n, m, seed. */
int flora_decompress(const flora_matrix_t* mats, int count, int r, float alpha,
                     void* const* out, flora_dtype_t out_dtype, void* hip_stream);

/* Momentum transfer (Algorithm 2, resample branch), computed as
 * T = A(seed)^T A(seed_next) (r x r, in the workspace) and then
 *     state <- state T        ( = state A(seed)^T A(seed_next) )
 * entirely in fp32.  Uses state, n, m, seed, seed_next.  The caller replaces
 * seed by seed_next afterwards. */
int flora_momentum_transfer(const flora_matrix_t* mats, int count, int r, void* hip_stream);

/* For callers that cannot allocate: code under HIP graph capture preparation, tight serving or
 * training loops, harnesses that forbid hipMalloc.  The same operation, arguments, requirements
 * and results (bit for bit) as flora_momentum_transfer, but the device memory it needs beyond M
 * itself -- descriptor table, work tables, the r x r matrices T and their per-chunk partials --
 * lives in a fixed array of FLORA_STATIC_SCRATCH_BYTES bytes inside the library, one copy per
 * GPU, held until the process ends.  The call allocates nothing on the device or in pinned memory
 * (no hipMalloc, hipHostMalloc, hipFree) and ignores flora_set_workspace; it uploads its tables
 * with one asynchronous copy from pageable host memory and launches the transfer's kernels.
 * A request needs  sum over matrices of (1 + [r >= 64] ceil(m / 1024)) * 4 r^2  bytes, rounded up
 * to 256 per term, plus 184 bytes per matrix and 48 bytes per workgroup (about 2 MiB per matrix
 * at r = 256, m = 6400; 16 KiB at r <= 32): beyond the array's size, or with count > 448, the
 * call returns FLORA_ERR_TOO_LARGE and nothing has been enqueued.  All calls on one GPU share that
 * GPU's array and each overwrites what the last one left: calls that may run at the same time on
 * one GPU (different streams, different host threads' streams) race and must be ordered by the
 * caller. */
#define FLORA_STATIC_SCRATCH_BYTES (32u << 20)
int flora_momentum_transfer_static(const flora_matrix_t* mats, int count, int r, void* hip_stream);

/* A compressed accumulator folded into a compressed moving average kept under another
 * projection (Algorithm 1's decompressed mean fed to Algorithm 2's EMA line: a = beta,
 * b = (1 - beta) / tau; the paper notes that the transfer extends to other EMA statistics,
 * Section 2.4), with no n x m pass:
 *     dst[l] <- a * dst[l] + b * state A(seed)^T A(seed_next)
 * equal to compressing the decompressed state, computed as T = A(seed)^T A(seed_next) and
 * state T entirely in fp32.  `dst` is a HOST array of `count` DEVICE pointers to n x r fp32
 * buffers, none of which may be the matrix's own state.  Uses state, n, m, seed, seed_next. */
int flora_transfer_accumulate(const flora_matrix_t* mats, int count, int r, float a, float b,
                              float* const* dst, void* hip_stream);

/* Decompression fused with the base optimizer's update; Gt is never stored:
 *   FLORA_RULE_SGD:       W <- W - lr * Gt            (Section 2.2, update rule)
 *   FLORA_RULE_FACTORED:  Adafactor, the base optimizer of the paper's experiments
 *                         (Section 3.1), with its factored second moment:
 *       Q = Gt^2 + eps1;  R <- beta2 R + (1-beta2) rowmean(Q);  K likewise by column;
 *       U = Gt / sqrt(R_i K_j / mean(R));  U <- U / max(1, RMS(U)/clip_d);  W <- W - step U
 *     (Gt is regenerated for each pass; row_stat and col_stat are updated in place).
 *   FLORA_RULE_UNFACTORED: the variant with an elementwise second moment (Section 3.3,
 *                         "Optimizer with linear memory"):
 *       V <- beta2 V + (1-beta2) (Gt^2 + eps1);  U = Gt / sqrt(V);  clipping and step as above
 *     (second_moment is updated in place).
 *   step = lr, or lr * max(eps2, RMS(W)) with scale_parameter: RMS(W) is taken from
 *   weight_sumsq[0] / (n m) as it stands when the call starts.  Whenever weight_sumsq is not
 *   NULL both Adafactor rules leave the sum of squares of the NEW weights there, so a caller
 *   that changes W by no other means fills it once (flora_weight_sumsq) and never reads W
 *   again for it.  lr and beta2 for step t of the published schedules:
 *   flora_adafactor_schedule.
 * Uses weight, state, n, m, seed (+ row_stat, col_stat | second_moment, + weight_sumsq).
 * weight_dtype: FLORA_F32, or FLORA_BF16 (the update is computed in fp32 from the bf16 weights
 * and rounded to nearest even when stored; the sum of squares is that of the stored values). */
int flora_apply_update(const flora_matrix_t* mats, int count, int r, flora_dtype_t weight_dtype,
                       const flora_update_t* u, void* hip_stream);

/* One whole step of Algorithm 2 for every matrix:
 *   if do_transfer: state <- state A(seed)^T A(seed_next) and the rest uses seed_next
 *   state <- a * state + b * grad A;   W <- W - rule(alpha * state A^T)
 * Equivalent to the three calls above in sequence on the same stream. */
int flora_fused_step(const flora_matrix_t* mats, int count, int r, flora_dtype_t grad_dtype,
                     flora_dtype_t weight_dtype, float a, float b, int do_transfer,
                     const flora_update_t* u, void* hip_stream);

/* weight_sumsq[0] <- sum of W^2 for every matrix (one read of W; fixed summation order).
 * Uses weight, weight_sumsq, n, m. */
int flora_weight_sumsq(const flora_matrix_t* mats, int count, flora_dtype_t weight_dtype, void* hip_stream);

/* Host-side helper: Adafactor's published schedules for step t = 1, 2, ... (t = 0 is read
 * as 1): relative step size *rho = min(1e-2, 1/sqrt(t)) and second-moment decay
 * *beta2 = 1 - t^-0.8 (0 at t = 1).  Either pointer may be NULL.  Never fails. */
void flora_adafactor_schedule(uint64_t t, float* rho, float* beta2);

/* Test hook: writes A(seed) (m x r fp32, row-major) to A_out and/or the raw
 * Philox words (m x ceil(r/4) x 4 uint32) to raw_out; either may be NULL.
 * r: any multiple of 4 up to 1024.  Both are DEVICE pointers. */
int flora_debug_generate(uint64_t seed, int64_t m, int r, float* A_out, uint32_t* raw_out,
                         void* hip_stream);

/* Host-side helper: "an independent random seed" (Algorithm 1 initialisation;
 * Algorithm 2 resample branch) as a pure function of a global seed, the
 * matrix's index and its resample count:
 * first two words of Philox4x32-10(counter = (matrix_id, epoch mod 2^32, epoch >> 32, 1),
 * key = global_seed).  Never fails. */
uint64_t flora_derive_seed(uint64_t global_seed, uint64_t matrix_id, uint64_t epoch);

/* The same for `count` consecutive matrix indices at one epoch:
 * seeds_out[i] = flora_derive_seed(global_seed, first_matrix_id + i, epoch).  seeds_out is a
 * HOST array of `count` entries; nothing happens if it is NULL or count <= 0. */
void flora_derive_seeds(uint64_t global_seed, uint64_t first_matrix_id, int count, uint64_t epoch,
                        uint64_t* seeds_out);

/* Caller-owned workspace (Section 2.4, "Memory analysis": the method's point is what a training
 * step keeps in memory, so the library's own footprint is the caller's to place and count).
 *
 * flora_workspace_bytes: the smallest workspace with which every entry point accepts this set of
 * matrices at rank r, i.e. what the most demanding call occupies: flora_fused_step with a
 * transfer and an Adafactor rule (its transfer, compress and update plans are resident together).
 * Exact, not a bound: with one 256-byte unit less that call returns FLORA_ERR_INVALID.  Only n and
 * m of the descriptors are read.  Host only.  0 for an invalid set or rank.
 *
 * flora_set_workspace: dev_ptr is DEVICE memory, 256-byte aligned, of `bytes` bytes, owned by the
 * caller and kept alive until the workspace is replaced, cleared (dev_ptr NULL and bytes 0:
 * back to library-allocated memory) or flora_shutdown().  While it is set the library calls no
 * hipMalloc / hipHostMalloc: tables, transfer matrices, partials, counters and descriptor images
 * of every call come out of this buffer, and uploads come from pageable host memory.  A call
 * whose plans do not fit is refused with FLORA_ERR_INVALID before anything is enqueued.  When
 * the plans of a call fit but not beside those of earlier calls, the earlier ones are dropped
 * and the buffer is refilled (a step that alternates between calls then re-uploads its tables:
 * give the workspace the sum of what its calls need to avoid that; flora_workspace_bytes is
 * enough for one fused step).  Calls that use the workspace must be ordered by the caller (one
 * stream, or events between streams): the refill relies on it.  Results are bit for bit those
 * of the library-allocated mode.  Drops every cached plan.  Not to be called while kernels of
 * earlier calls may still run, or between a graph capture and its replays. */
size_t flora_workspace_bytes(const flora_matrix_t* mats, int count, int r);
int flora_set_workspace(void* dev_ptr, size_t bytes);

/* hipError_t of the most recent failing HIP call on this thread (0 if none). */
int flora_last_device_error(void);

/* Static string for a status code. */
const char* flora_status_string(int status);

/* Frees the workspace and cached descriptor tables on every device. */
void flora_shutdown(void);

/* Library version: major * 10000 + minor * 100 + patch. */
int flora_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FLORA_H_ */
