// Internal types shared by the host-side C ABI and the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace flora {

// Device-side image of one weight matrix (built on the host from flora_matrix_t).
struct MatDev {
    const void* grad;
    float* weight;
    float* state;
    float* row_stat;
    float* col_stat;
    void* out;          // flora_decompress destination
    float* T;           // r x r transfer matrix (workspace)
    float* rowpart;     // [ncolchunks][n] partial row sums of Gt^2 (workspace)
    float* colpart;     // [nrowblocks][m] partial column sums of Gt^2 (workspace)
    float* itempart;    // [nitems] per-workgroup partial sums of U^2 (workspace)
    float* scal;        // [4]: mean(R), clip scale, spare, spare (workspace)
    long long n, m;
    uint32_t seed_lo, seed_hi, seedn_lo, seedn_hi;   // used by the transfer kernels only
    int ncolchunks, nrowblocks;   // decompress tiling of this matrix
    int item0, nitems;            // this matrix's range in the decompress work table
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
};

enum DecompressMode : int {
    kModeOut = 0,      // out <- alpha * state A^T
    kModeSgd = 1,      // W <- W - coef * state A^T
    kModeStats = 2,    // partial row / column sums of (alpha state A^T)^2
    kModeRms = 3,      // partial sums of U^2
    kModeFactored = 4  // W <- W - lr * scale * Gt / sqrt(R_i K_j / mean R)
};

struct DecompressParams {
    float alpha;   // scale of Gt
    float coef;    // lr * alpha (SGD) or lr (factored)
};

typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;

// fp32 -> bf16, round to nearest even (finite inputs).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b)
{
    return __builtin_bit_cast(float, b << 16);
}

// ---- launchers implemented in the kernel translation units ----------------
hipError_t launch_debug_generate(uint64_t seed, long long m, int r, float* A_out, uint32_t* raw_out,
                                 hipStream_t s);
hipError_t launch_compress_f32(const MatDev* mats, const WorkItem* items, int nitems, const SeedArgs& seeds,
                               int r, int grad_is_bf16, float a, float b, hipStream_t s);
hipError_t launch_compress_bf16_mt(const MatDev* mats, const WorkItem* items, int nitems,
                                   const SeedArgs& seeds, int r, int mt, float a, float b, hipStream_t s);
hipError_t launch_decompress_f32(const MatDev* mats, const WorkItem* items, int nitems, const SeedArgs& seeds,
                                 int r, int mode, int out_is_bf16, DecompressParams p, hipStream_t s);
hipError_t launch_decompress_bf16(const MatDev* mats, const WorkItem* items, int nitems, const SeedArgs& seeds,
                                  int r, int mode, int out_is_bf16, DecompressParams p, hipStream_t s);
hipError_t launch_transfer_T(const MatDev* mats, int count, int r, hipStream_t s);
hipError_t launch_apply_T(const MatDev* mats, const WorkItem* items, int nitems, int r, hipStream_t s);
hipError_t launch_stats_finalize(const MatDev* mats, int count, float beta2, float eps1, hipStream_t s);
hipError_t launch_rms_finalize(const MatDev* mats, int count, float clip_d, hipStream_t s);
hipError_t launch_zero_state(const MatDev* mats, int count, int r, hipStream_t s);

// Tiling constants the host needs to build work tables.
constexpr int kCompressF32Rows = 64;     // rows per workgroup, fp32 matrix-core compress
constexpr int kCompressBf16Rows = 512;   // rows per workgroup, bf16 matrix-core compress
constexpr int kCompressBf16Slice = 64;   // rank columns per workgroup, bf16 compress
constexpr int kDecompressCols = 128;     // columns per workgroup, both decompress kernels
constexpr int kDecompressRows = 256;     // rows per workgroup, both decompress kernels
constexpr int kApplyTRows = 32;          // rows per workgroup, state <- state T

}  // namespace flora
