// Internal types shared by the host-side C ABI and the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace flora {

// Device-side image of one weight matrix (built on the host from flora_matrix_t).
struct MatDev {
    const void* grad;
    void* weight;       // n x m, fp32 or bf16
    float* state;
    float* row_stat;
    float* col_stat;
    float* vfull;       // n x m second moment of the unfactored rule
    float* wsumsq;      // 1 float: sum of W^2, read for the parameter scale and refreshed by the update
    void* out;          // flora_decompress destination; flora_transfer_accumulate destination (n x r fp32)
    float* T;           // r x r transfer matrix (workspace)
    float* rowpart;     // [ncolchunks][n] partial row sums of Gt^2; transfer: [chunks][r][r] partials of T (workspace)
    float* colpart;     // [nrowblocks][m] partial column sums of Gt^2 (workspace)
    float* itempart;    // [nitems] per-workgroup partial sums of U^2, later of the new W^2 (workspace)
    float* scal;        // [4]: mean(R), clip scale, parameter scale max(eps2, RMS(W)) or 1, spare (workspace)
    uint16_t* gramP;    // r x r bf16: A^T A, later A^T diag(1/K) A (factored rule through Gram matrices; workspace)
    uint16_t* gramQ;    // r x r bf16: S^T S (workspace)
    float* grampart;    // [chunks][r][r] partial Gram matrices of the chunks of m or of n (workspace)
    long long n, m;
    uint32_t seed_lo, seed_hi, seedn_lo, seedn_hi;   // used by the transfer kernels only
    int ncolchunks, nrowblocks;   // decompress tiling of this matrix
    int item0, nitems;            // nitems: decompress workgroups of this matrix; item0: row blocks of the
                                  // quadratic-form pass (its partial sums of U^2 are itempart[0 .. item0))
    int gchunks_m, gchunks_n;     // chunks of the Gram sums over m and over n
};

// Seeds of the matrices of one grouped launch, passed by value as a kernel argument:
// a resample changes nothing in device memory, so there is nothing to upload.
constexpr int kMaxSeedArgs = 448;
struct SeedArgs {
    uint2 s[kMaxSeedArgs];   // (low word, high word) of matrix l's 64-bit seed
};

// One workgroup's share of a grouped launch.
struct WorkItem {
    int mat;     // index into the MatDev table
    int row0;    // first row
    int rows;    // number of rows (may run past n only in padding; kernels mask)
    int col0;    // first column (decompress) / unused
    int slice;   // rank slice index (compress at r >= 128) / column-chunk index
    int rblock;  // row-block index within the matrix
    // decompress: `part` = this workgroup's slot in its matrix's per-workgroup partial sums.
    // fp32 and wide bf16 compress: this workgroup's columns [col0, col1) are part `part` of `nparts`
    // of its (row block, rank slice); with nparts > 1 the partial products live at float offset
    // `poff` of the workspace and arrivals are counted in counter `cidx`
    int col1, part, nparts, cidx;
    long long poff;
};

enum DecompressMode : int {
    kModeOut = 0,      // out <- alpha * state A^T
    kModeSgd = 1,      // W <- W - coef * state A^T
    kModeStats = 2,    // partial row / column sums of (alpha state A^T)^2
    kModeRms = 3,      // partial sums of U^2
    kModeFactored = 4, // W <- W - lr * scale * Gt / sqrt(R_i K_j / mean R); partial sums of the new W^2
    kModeFull1 = 5,    // V <- beta2 V + (1 - beta2) (Gt^2 + eps1); partial sums of U^2 = Gt^2 / V
    kModeFull2 = 6     // W <- W - lr * scale * Gt / sqrt(V); partial sums of the new W^2
};

struct DecompressParams {
    float alpha;   // scale of Gt
    float coef;    // lr * alpha (SGD) or lr (factored, unfactored)
    float beta2;   // kModeFull1: decay of V
    float eps1;    // kModeFull1: added to Gt^2
    int wpolicy;   // update passes: bit 0 weights / second moment read with the non-temporal hint,
                   // bit 1 written with it (chosen from the size of the set, see choose_wpolicy)
};

typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;

// Every pointer in a descriptor is device memory.  Telling the compiler so (address space 1)
// turns generic flat_load/flat_store into global_load/global_store, which neither touch the
// LDS counter nor stall on it.
#define FLORA_GLOBAL __attribute__((address_space(1)))
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));
typedef uint32_t v2u __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float ldg(const float* p) { return *(const FLORA_GLOBAL float*)p; }
__device__ __forceinline__ v4f ldg4(const float* p) { return *(const FLORA_GLOBAL v4f*)p; }
__device__ __forceinline__ v2f ldg2(const float* p) { return *(const FLORA_GLOBAL v2f*)p; }
__device__ __forceinline__ v4u ldg4(const uint16_t* p) { return *(const FLORA_GLOBAL v4u*)p; }
__device__ __forceinline__ v2u ldg2(const uint16_t* p) { return *(const FLORA_GLOBAL v2u*)p; }
__device__ __forceinline__ uint32_t ldg(const uint16_t* p) { return *(const FLORA_GLOBAL uint16_t*)p; }
__device__ __forceinline__ void stg(float* p, float v) { *(FLORA_GLOBAL float*)p = v; }
__device__ __forceinline__ void stg(uint16_t* p, uint16_t v) { *(FLORA_GLOBAL uint16_t*)p = v; }

// Buffer addressing: a wave-uniform resource (base pointer + size in bytes) plus a 32-bit
// per-lane byte offset.  The hardware checks the offset against the size: a load beyond it
// returns zero and a store beyond it is dropped, with no memory traffic.  Sizes are kept
// below 2^31 so that kOob is out of range for every resource; the host guarantees that by
// limiting m to 2^24 columns.  Pipelined loops use this to prefetch unconditionally (a
// prefetch past the end is pointed at kOob) and to mask ragged edges without branches.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
constexpr uint32_t kOob = 0x80000000u;
__device__ __forceinline__ rsrc_t make_rsrc(const void* base, long long bytes)
{
    const uint32_t nb = bytes <= 0 ? 0u : (bytes > 0x7fffffffLL ? 0x7fffffffu : (uint32_t)bytes);
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), (short)0, (int)nb, 0x00020000);
}
__device__ __forceinline__ v4f buf_load_f4(rsrc_t r, uint32_t off)
{
    return __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, 0));
}
__device__ __forceinline__ v4u buf_load_u4(rsrc_t r, uint32_t off)
{
    return __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, 0);
}
__device__ __forceinline__ v2u buf_load_u2(rsrc_t r, uint32_t off)
{
    return __builtin_amdgcn_raw_buffer_load_b64(r, (int)off, 0, 0);
}
// The same with the non-temporal hint, for data a launch reads exactly once (the gradients):
// the lines then do not displace what the caches hold for later (the weights the update has
// just written, the state), which shortens the launches that follow an update.  A second pass
// over the same data in the same launch (rank slices of a wide row block) would miss L2 with
// it, so those launches use the plain loads.
template <bool STREAM>
__device__ __forceinline__ v4f buf_load_f4(rsrc_t r, uint32_t off)
{
    return __builtin_bit_cast(v4f, STREAM ? __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, 2)
                                          : __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, 0));
}
template <bool STREAM>
__device__ __forceinline__ v4u buf_load_u4(rsrc_t r, uint32_t off)
{
    return STREAM ? __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, 2)
                  : __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, 0);
}
template <bool STREAM>
__device__ __forceinline__ v2u buf_load_u2(rsrc_t r, uint32_t off)
{
    return STREAM ? __builtin_amdgcn_raw_buffer_load_b64(r, (int)off, 0, 2)
                  : __builtin_amdgcn_raw_buffer_load_b64(r, (int)off, 0, 0);
}
template <bool STREAM>
__device__ __forceinline__ void buf_store_f4(rsrc_t r, uint32_t off, v4f v)
{
    if (STREAM) __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4u, v), r, (int)off, 0, 2);
    else __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4u, v), r, (int)off, 0, 0);
}
template <bool STREAM>
__device__ __forceinline__ void buf_store_u2(rsrc_t r, uint32_t off, v2u v)
{
    if (STREAM) __builtin_amdgcn_raw_buffer_store_b64(v, r, (int)off, 0, 2);
    else __builtin_amdgcn_raw_buffer_store_b64(v, r, (int)off, 0, 0);
}
__device__ __forceinline__ float buf_load_f(rsrc_t r, uint32_t off)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, (int)off, 0, 0));
}
__device__ __forceinline__ void buf_store_f(rsrc_t r, uint32_t off, float v)
{
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, v), r, (int)off, 0, 0);
}
__device__ __forceinline__ void buf_store_f4(rsrc_t r, uint32_t off, v4f v)
{
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4u, v), r, (int)off, 0, 0);
}
__device__ __forceinline__ void buf_store_u2(rsrc_t r, uint32_t off, v2u v)
{
    __builtin_amdgcn_raw_buffer_store_b64(v, r, (int)off, 0, 0);
}
__device__ __forceinline__ void buf_store_h(rsrc_t r, uint32_t off, uint16_t v)
{
    __builtin_amdgcn_raw_buffer_store_b16(v, r, (int)off, 0, 0);
}

// fp32 -> bf16, round to nearest even (finite inputs).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}
// Two fp32 -> packed bf16, round to nearest even, one v_cvt_pk_bf16_f32.
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    const v2f v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b)
{
    return __builtin_bit_cast(float, b << 16);
}
// One element of an n x m array of fp32 or bf16 (weights), as fp32.
__device__ __forceinline__ float load_elem(const float* p) { return *(const FLORA_GLOBAL float*)p; }
__device__ __forceinline__ float load_elem(const uint16_t* p) { return bf16_bits_to_f32(*(const FLORA_GLOBAL uint16_t*)p); }
// Loads and stores with the non-temporal hint when STREAM is set (cache policy of the update
// passes); stores round to nearest even and return the value that was stored.
template <bool STREAM>
__device__ __forceinline__ float load_elem(const float* p)
{
    return STREAM ? __builtin_nontemporal_load((const FLORA_GLOBAL float*)p) : *(const FLORA_GLOBAL float*)p;
}
template <bool STREAM>
__device__ __forceinline__ float load_elem(const uint16_t* p)
{
    return bf16_bits_to_f32(STREAM ? __builtin_nontemporal_load((const FLORA_GLOBAL uint16_t*)p)
                                   : *(const FLORA_GLOBAL uint16_t*)p);
}
template <bool STREAM>
__device__ __forceinline__ float store_elem(float* p, float v)
{
    if (STREAM) __builtin_nontemporal_store(v, (FLORA_GLOBAL float*)p);
    else *(FLORA_GLOBAL float*)p = v;
    return v;
}
template <bool STREAM>
__device__ __forceinline__ float store_elem(uint16_t* p, float v)
{
    const uint32_t b = f32_to_bf16_bits(v);
    if (STREAM) __builtin_nontemporal_store((uint16_t)b, (FLORA_GLOBAL uint16_t*)p);
    else *(FLORA_GLOBAL uint16_t*)p = (uint16_t)b;
    return bf16_bits_to_f32(b);
}

// ---- launchers implemented in the kernel translation units ----------------
hipError_t launch_debug_generate(uint64_t seed, long long m, int r, float* A_out, uint32_t* raw_out,
                                 hipStream_t s);
hipError_t launch_debug_copy(const void* src, void* dst, long long bytes, hipStream_t s);
hipError_t launch_debug_read(const void* src, long long bytes, int pattern, long long row_bytes, int chunk_bytes,
                             uint32_t* sink, hipStream_t s);
hipError_t launch_debug_compute_loop(int kind, int iters, float* sink, double* work_out, hipStream_t s);
hipError_t launch_compress_f32(const MatDev* mats, const WorkItem* items, int nitems, const SeedArgs& seeds,
                               int r, int grad_is_bf16, int map, float a, float b, int kgroups, int mt,
                               float* partials, uint32_t* counters, hipStream_t s);
hipError_t launch_compress_bf16_mt(const MatDev* mats, const WorkItem* items, int nitems,
                                   const SeedArgs& seeds, int r, int mt, int grad_is_f32, int map, float a, float b,
                                   float* partials, uint32_t* counters, hipStream_t s);
hipError_t launch_decompress_f32(const MatDev* mats, const WorkItem* items, int nitems, const SeedArgs& seeds,
                                 int r, int mode, int out_is_bf16, DecompressParams p, hipStream_t s);
hipError_t launch_decompress_bf16(const MatDev* mats, const WorkItem* items, int nitems, const SeedArgs& seeds,
                                  int r, int mode, int out_is_bf16, int vec, DecompressParams p, hipStream_t s);
hipError_t launch_transfer_T(const MatDev* mats, const WorkItem* items, int nitems, int count, int r, hipStream_t s);
hipError_t launch_apply_T(const MatDev* mats, const WorkItem* items, int nitems, int r, float ca, float cb,
                          hipStream_t s);
hipError_t launch_stats_finalize(const MatDev* mats, int count, float beta2, float eps1, int gram, hipStream_t s);
hipError_t launch_rms_finalize(const MatDev* mats, int count, float clip_d, int scale_parameter, float eps2, int gram,
                               hipStream_t s);
hipError_t launch_gram(const MatDev* mats, const WorkItem* items, int nitems, int count, const SeedArgs& seeds, int r,
                       int src, hipStream_t s);
hipError_t launch_quadform(const MatDev* mats, const WorkItem* items, int nitems, const SeedArgs& seeds, int r, int out,
                           float alpha, float beta2, float eps1, hipStream_t s);
hipError_t launch_wsumsq_finalize(const MatDev* mats, int count, hipStream_t s);
hipError_t launch_weight_sumsq(const MatDev* mats, int count, int weight_is_bf16, float* partials, hipStream_t s);
hipError_t launch_zero_state(const MatDev* mats, int count, int r, hipStream_t s);

// Tiling constants the host needs to build work tables.
constexpr int kCompressBf16Rows = 512;   // rows per workgroup, bf16 matrix-core compress
constexpr int kCompressBf16Slice = 64;   // rank columns per workgroup, bf16 compress
constexpr int kDecompressCols = 128;     // columns per workgroup, 4-byte-per-lane decompress kernels
constexpr int kDecompressColsVec = 256;  // columns per workgroup, 16-byte-per-lane bf16 decompress kernel
constexpr int kDecompressRows = 256;     // rows per workgroup, both decompress kernels
constexpr int kApplyTRows = 32;          // rows per workgroup, state <- state T, ranks below 64
constexpr int kApplyTRowsBig = 64;       // ... ranks 64 and above
constexpr int kTransferChunk = 1024;     // columns per workgroup of the T kernel, ranks 64 and above
constexpr int kSumsqBlocks = 256;        // workgroups per matrix, sum of W^2
constexpr int kGramChunk = 3072;         // long-index entries per workgroup of the Gram sums
constexpr int kQuadformRows = 1024;      // rows of Z per workgroup of the quadratic forms

}  // namespace flora
