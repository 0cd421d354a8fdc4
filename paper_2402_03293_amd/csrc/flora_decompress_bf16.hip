// Decompression on the bf16 matrix cores, ranks 64 / 128 / 256, fused with
// what consumes the decompressed gradient:
//     Gt = alpha * state A(seed)^T
// (Algorithm 1, decompression line; Algorithm 2, yield).  A and the state are
// rounded to bf16 on the fly; products and sums are fp32
// (v_mfma_f32_32x32x16_bf16).  Gt exists only in accumulator registers.
//
// One workgroup (4 waves) owns a block of rows and 128 columns of one matrix;
// each wave owns 32 of those columns.  Lane (column j = lane % 32, half
// g = lane / 32) regenerates A[j, 16 s + 8 g .. +7] for every step s < r/16
// (r/8 Philox calls) once, into the B operand registers, and keeps them while
// the workgroup walks down the rows 32 at a time.  The 32 x r block of the
// state is converted to bf16 once per workgroup and shared through LDS
// (double buffered: the next block is fetched while the current one is used).
#include "flora_gen.hip.h"
#include "flora_internal.h"
#include "flora_epilogue.hip.h"

namespace flora {

namespace {

template <int R, int MODE, typename OT>
__global__ __launch_bounds__(256) void decompress_bf16_kernel(const MatDev* __restrict__ mats,
                                                              const WorkItem* __restrict__ items,
                                                              const SeedArgs seeds, DecompressParams p)
{
    constexpr int S = R / 16;          // MFMA steps along the rank axis
    constexpr int LDS_ROW = R + 8;     // padded row (bf16 elements)
    constexpr int F4 = R / 32;         // float4 loads per thread for one 32 x R block
    __shared__ __attribute__((aligned(16))) uint16_t ldsS[2][32][LDS_ROW];
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

    bf16x8 breg[S];
#pragma unroll
    for (int s = 0; s < S; ++s) {
        const Quad z0 = normal_quad(seed_lo, seed_hi, (uint64_t)(jok ? j : 0), (uint32_t)(4 * s + 2 * g), cgen);
        const Quad z1 = normal_quad(seed_lo, seed_hi, (uint64_t)(jok ? j : 0), (uint32_t)(4 * s + 2 * g + 1), cgen);
        const uint4 pk = make_uint4(pack_bf16x2(z0.z[0], z0.z[1]), pack_bf16x2(z0.z[2], z0.z[3]),
                                    pack_bf16x2(z1.z[0], z1.z[1]), pack_bf16x2(z1.z[2], z1.z[3]));
        breg[s] = __builtin_bit_cast(bf16x8, pk);
    }

    EpilogueLane ep = epilogue_begin<MODE>(M, p, j, jok);

    const long long row_end = ((long long)it.row0 + it.rows < n) ? (long long)it.row0 + it.rows : n;

    // cooperative fetch of a 32 x R block of the state: float4 number f = tid + 256 i
    // covers row f / (R/4), columns 4 (f % (R/4)) .. +3
    auto fetch = [&](v4f (&dst)[F4], long long rb) {
#pragma unroll
        for (int i = 0; i < F4; ++i) {
            const int f = tid + 256 * i;
            long long row = rb + f / (R / 4);
            if (row > n - 1) row = n - 1;
            dst[i] = ldg4(state + row * R + 4 * (f % (R / 4)));
        }
    };
    auto stash = [&](const v4f (&src)[F4], int buf) {
#pragma unroll
        for (int i = 0; i < F4; ++i) {
            const int f = tid + 256 * i;
            const uint2 pk = make_uint2(pack_bf16x2(src[i].x, src[i].y), pack_bf16x2(src[i].z, src[i].w));
            *reinterpret_cast<uint2*>(&ldsS[buf][f / (R / 4)][4 * (f % (R / 4))]) = pk;
        }
    };

    v4f stage[F4];
    fetch(stage, it.row0);
    TilePre<MODE> pre_cur, pre_nxt;
    epilogue_fetch<MODE>(pre_cur, M, it.row0, row_end, j, jok);
    stash(stage, 0);
    __syncthreads();

    int buf = 0;
    for (long long rb = it.row0; rb < row_end; rb += 32) {
        const bool more = rb + 32 < row_end;
        if (more) {
            fetch(stage, rb + 32);
            epilogue_fetch<MODE>(pre_nxt, M, rb + 32, row_end, j, jok);
        }

        f32x16 acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
        for (int s = 0; s < S; ++s) {
            const bf16x8 av = *reinterpret_cast<const bf16x8*>(&ldsS[buf][ln][16 * s + 8 * g]);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, breg[s], acc, 0, 0, 0);
        }

        epilogue_tile<MODE, OT>(acc, pre_cur, M, it, p, rb, row_end, j, jok, ep, lds_red);

        if (more) {
            stash(stage, buf ^ 1);
            pre_cur = pre_nxt;
        }
        __syncthreads();
        buf ^= 1;
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
        hipLaunchKernelGGL((decompress_bf16_kernel<R, kModeOut, OT>), grid, block, 0, s, mats, items, seeds, p);
        break;
    case kModeSgd:
        hipLaunchKernelGGL((decompress_bf16_kernel<R, kModeSgd, float>), grid, block, 0, s, mats, items, seeds, p);
        break;
    case kModeStats:
        hipLaunchKernelGGL((decompress_bf16_kernel<R, kModeStats, float>), grid, block, 0, s, mats, items, seeds, p);
        break;
    case kModeRms:
        hipLaunchKernelGGL((decompress_bf16_kernel<R, kModeRms, float>), grid, block, 0, s, mats, items, seeds, p);
        break;
    case kModeFactored:
        hipLaunchKernelGGL((decompress_bf16_kernel<R, kModeFactored, float>), grid, block, 0, s, mats, items, seeds, p);
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
    if (mode == kModeOut && out_is_bf16) return launch_mode<R, uint16_t>(mats, items, nitems, seeds, mode, p, s);
    return launch_mode<R, float>(mats, items, nitems, seeds, mode, p, s);
}

}  // namespace

hipError_t launch_decompress_bf16(const MatDev* mats, const WorkItem* items, int nitems, const SeedArgs& seeds,
                                 int r, int mode, int out_is_bf16, DecompressParams p, hipStream_t s)
{
    if (nitems == 0) return hipSuccess;
    if (r == 64) return launch_r<64>(mats, items, nitems, seeds, mode, out_is_bf16, p, s);
    if (r == 128) return launch_r<128>(mats, items, nitems, seeds, mode, out_is_bf16, p, s);
    if (r == 256) return launch_r<256>(mats, items, nitems, seeds, mode, out_is_bf16, p, s);
    return hipErrorInvalidValue;
}

}  // namespace flora
