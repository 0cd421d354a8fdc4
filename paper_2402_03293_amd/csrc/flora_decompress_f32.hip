// Decompression on the fp32 matrix cores, ranks 8 / 16 / 32, fused with what
// consumes the decompressed gradient:
//     Gt = alpha * state A(seed)^T
// (Algorithm 1, decompression line; Algorithm 2, yield).  Gt exists only in
// accumulator registers; the epilogue either stores it (flora_decompress),
// applies SGD to W (Section 2.2, update rule), gathers the second-moment
// statistics of the factored rule, or applies the factored update.
//
// One workgroup (4 waves) owns a block of rows and 128 columns of one matrix;
// each wave owns 32 of those columns.  A lane (column j = lane % 32, half
// g = lane / 32) regenerates A[j, g r/2 .. (g+1) r/2) once, r/8 Philox calls,
// straight into the B operand registers of v_mfma_f32_32x32x2_f32, and keeps
// them while the wave walks down the rows 32 at a time.  The state rows are
// the A operand (lane = row, same half of the rank axis).  No LDS and no
// barrier is needed for the product itself.
#include "flora_gen.hip.h"
#include "flora_internal.h"
#include "flora_epilogue.hip.h"

namespace flora {

namespace {

template <int R, int MODE, typename OT>
__global__ __launch_bounds__(256) void decompress_f32_kernel(const MatDev* __restrict__ mats,
                                                             const WorkItem* __restrict__ items,
                                                             const SeedArgs seeds, DecompressParams p)
{
    constexpr int H = R / 2;   // rank entries per lane
    __shared__ float lds_red[4][32];

    const WorkItem it = items[blockIdx.x];
    const MatDev& M = mats[it.mat];
    const long long n = M.n, m = M.m;
    const float* __restrict__ state = M.state;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int ln = lane & 31, g = lane >> 5;
    const long long j = (long long)it.col0 + 32 * wave + ln;
    const bool jok = j < m;
    const float cgen = neg2_ln2_over(R);
    const uint32_t seed_lo = seeds.s[it.mat].x, seed_hi = seeds.s[it.mat].y;

    float breg[H];
#pragma unroll
    for (int i = 0; i < R / 8; ++i) {
        const Quad z = normal_quad(seed_lo, seed_hi, (uint64_t)(jok ? j : 0),
                                   (uint32_t)(g * (R / 8) + i), cgen);
#pragma unroll
        for (int e = 0; e < 4; ++e) breg[4 * i + e] = z.z[e];
    }

    EpilogueLane ep = epilogue_begin<MODE>(M, p, j, jok);

    const long long row_end = ((long long)it.row0 + it.rows < n) ? (long long)it.row0 + it.rows : n;

    // state rows of a tile: lane = row, this lane's half of the rank axis
    auto load_state = [&](v4f (&dst)[H / 4], long long rb) {
        long long arow = rb + ln;
        if (arow > n - 1) arow = n - 1;
        const float* sp = state + arow * R + g * H;
#pragma unroll
        for (int i = 0; i < H / 4; ++i) dst[i] = ldg4(sp + 4 * i);
    };

    // software pipeline: the next tile's state rows and old weights are in flight while the
    // current tile goes through the matrix cores and is written back
    v4f a_cur[H / 4], a_nxt[H / 4];
    TilePre<MODE> pre_cur, pre_nxt;
    load_state(a_cur, it.row0);
    epilogue_fetch<MODE, OT>(pre_cur, M, p, it.row0, row_end, j, jok);
    for (long long rb = it.row0; rb < row_end; rb += 32) {
        const bool more = rb + 32 < row_end;
        if (more) {
            load_state(a_nxt, rb + 32);
            epilogue_fetch<MODE, OT>(pre_nxt, M, p, rb + 32, row_end, j, jok);
        }
        f32x16 acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
        for (int s = 0; s < H; ++s)
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a_cur[s / 4][s % 4], breg[s], acc, 0, 0, 0);

        epilogue_tile<MODE, OT>(acc, pre_cur, M, it, p, rb, row_end, j, jok, ep, lds_red);
        if (more) {
#pragma unroll
            for (int i = 0; i < H / 4; ++i) a_cur[i] = a_nxt[i];
            pre_cur = pre_nxt;
        }
    }
    epilogue_end<MODE>(M, it, j, jok, ep, lds_red);
}

template <int R, typename OT>
hipError_t launch_mode(const MatDev* mats, const WorkItem* items, int nitems, const SeedArgs& seeds,
                       int mode, DecompressParams p, hipStream_t s)
{
    const dim3 grid((unsigned)nitems), block(256);
    switch (mode) {
    case kModeOut:
        hipLaunchKernelGGL((decompress_f32_kernel<R, kModeOut, OT>), grid, block, 0, s, mats, items, seeds, p);
        break;
    case kModeSgd:
        hipLaunchKernelGGL((decompress_f32_kernel<R, kModeSgd, OT>), grid, block, 0, s, mats, items, seeds, p);
        break;
    case kModeStats:
        hipLaunchKernelGGL((decompress_f32_kernel<R, kModeStats, float>), grid, block, 0, s, mats, items, seeds, p);
        break;
    case kModeRms:
        hipLaunchKernelGGL((decompress_f32_kernel<R, kModeRms, float>), grid, block, 0, s, mats, items, seeds, p);
        break;
    case kModeFactored:
        hipLaunchKernelGGL((decompress_f32_kernel<R, kModeFactored, OT>), grid, block, 0, s, mats, items, seeds, p);
        break;
    case kModeFull1:
        hipLaunchKernelGGL((decompress_f32_kernel<R, kModeFull1, float>), grid, block, 0, s, mats, items, seeds, p);
        break;
    case kModeFull2:
        hipLaunchKernelGGL((decompress_f32_kernel<R, kModeFull2, OT>), grid, block, 0, s, mats, items, seeds, p);
        break;
    default:
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <int R>
hipError_t launch_r(const MatDev* mats, const WorkItem* items, int nitems, const SeedArgs& seeds, int mode,
                    int out_is_bf16, DecompressParams p, hipStream_t s)
{
    // modes that read or write the n x m array whose element type the caller chose (out, or W)
    const bool typed = mode == kModeOut || mode == kModeSgd || mode == kModeFactored || mode == kModeFull2;
    if (typed && out_is_bf16) return launch_mode<R, uint16_t>(mats, items, nitems, seeds, mode, p, s);
    return launch_mode<R, float>(mats, items, nitems, seeds, mode, p, s);
}

}  // namespace

hipError_t launch_decompress_f32(const MatDev* mats, const WorkItem* items, int nitems, const SeedArgs& seeds,
                                 int r, int mode, int out_is_bf16, DecompressParams p, hipStream_t s)
{
    if (nitems == 0) return hipSuccess;
    if (r == 8) return launch_r<8>(mats, items, nitems, seeds, mode, out_is_bf16, p, s);
    if (r == 16) return launch_r<16>(mats, items, nitems, seeds, mode, out_is_bf16, p, s);
    if (r == 32) return launch_r<32>(mats, items, nitems, seeds, mode, out_is_bf16, p, s);
    return hipErrorInvalidValue;
}

}  // namespace flora
