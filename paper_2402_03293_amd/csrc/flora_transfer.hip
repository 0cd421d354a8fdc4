// Momentum transfer (Algorithm 2, resample branch):
//     M <- M A_old^T A_new
// computed in the re-associated order T = A_old^T A_new (r x r), M <- M T, so
// that no n x m intermediate exists.  Everything stays fp32 (fp32 matrix
// cores): an error made here would be carried by every later step.
//
// transfer_T: one workgroup owns up to 32 rows k1 of T and all r columns,
//   sweeps j = 0..m-1 in tiles of 32, regenerating both projections' tiles
//   into LDS ([j][k] layout) and contracting over j with
//   v_mfma_f32_16x16x4_f32.  The reduction order is fixed, so T is
//   reproducible bit for bit.
// apply_T: one workgroup owns 32 rows of M, keeps them in LDS, multiplies by
//   T (read through the caches) and writes the rows back in place.
#include "flora_gen.hip.h"
#include "flora_internal.h"

namespace flora {

namespace {

constexpr int kBJ = 32;   // rows of A per tile

template <int R>
__global__ __launch_bounds__(256) void transfer_T_kernel(const MatDev* __restrict__ mats)
{
    constexpr int KB1 = (R < 32) ? R : 32;          // rows of T per workgroup
    constexpr int NT1 = (KB1 + 15) / 16;
    constexpr int NT2 = (R + 15) / 16;
    constexpr int NT2W = (NT2 + 3) / 4;             // column tiles of T per wave
    constexpr int P1 = NT1 * 16 + 4, P2 = NT2 * 16 + 4;
    __shared__ float ldsOld[kBJ][P1];
    __shared__ float ldsNew[kBJ][P2];

    constexpr int blocks_per_mat = (R + KB1 - 1) / KB1;
    const int mat = blockIdx.x / blocks_per_mat;
    const int kb = blockIdx.x - mat * blocks_per_mat;
    const MatDev& M = mats[mat];
    const long long m = M.m;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int li = lane & 15, jg = lane >> 4;
    const float cgen = neg2_ln2_over(R);

    // zero the padding columns once (ranks below 16)
    for (int idx = tid; idx < kBJ * P1; idx += 256) ldsOld[idx / P1][idx % P1] = 0.f;
    for (int idx = tid; idx < kBJ * P2; idx += 256) ldsNew[idx / P2][idx % P2] = 0.f;
    __syncthreads();

    f32x4 acc[NT1][NT2W];
#pragma unroll
    for (int a = 0; a < NT1; ++a)
#pragma unroll
        for (int b = 0; b < NT2W; ++b) acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int ntiles = (int)((m + kBJ - 1) / kBJ);
    for (int tile = 0; tile < ntiles; ++tile) {
        const long long j0 = (long long)tile * kBJ;
        // old projection: rows j0.., columns kb*KB1 .. +KB1
        for (int idx = tid; idx < kBJ * (KB1 / 4); idx += 256) {
            const int jl = idx % kBJ, q = idx / kBJ;
            Quad z = normal_quad(M.seed_lo, M.seed_hi, (uint64_t)(j0 + jl), (uint32_t)(kb * (KB1 / 4) + q), cgen);
            const bool ok = j0 + jl < m;
#pragma unroll
            for (int i = 0; i < 4; ++i) ldsOld[jl][4 * q + i] = ok ? z.z[i] : 0.f;
        }
        for (int idx = tid; idx < kBJ * (R / 4); idx += 256) {
            const int jl = idx % kBJ, q = idx / kBJ;
            Quad z = normal_quad(M.seedn_lo, M.seedn_hi, (uint64_t)(j0 + jl), (uint32_t)q, cgen);
            const bool ok = j0 + jl < m;
#pragma unroll
            for (int i = 0; i < 4; ++i) ldsNew[jl][4 * q + i] = ok ? z.z[i] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int c = 0; c < kBJ / 4; ++c) {
            float av[NT1];
#pragma unroll
            for (int a = 0; a < NT1; ++a) av[a] = ldsOld[4 * c + jg][a * 16 + li];
#pragma unroll
            for (int b = 0; b < NT2W; ++b) {
                const int t2 = wave + 4 * b;
                if (t2 < NT2) {
                    const float bv = ldsNew[4 * c + jg][t2 * 16 + li];
#pragma unroll
                    for (int a = 0; a < NT1; ++a)
                        acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[a], bv, acc[a][b], 0, 0, 0);
                }
            }
        }
        __syncthreads();
    }

    // D layout of the 16x16 tile: lane holds column lane % 16, rows 4 * (lane / 16) + v.
#pragma unroll
    for (int a = 0; a < NT1; ++a)
#pragma unroll
        for (int b = 0; b < NT2W; ++b) {
            const int t2 = wave + 4 * b;
            if (t2 < NT2) {
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int k1 = kb * KB1 + a * 16 + 4 * jg + v;
                    const int k2 = t2 * 16 + li;
                    if (a * 16 + 4 * jg + v < KB1 && k2 < R) M.T[k1 * R + k2] = acc[a][b][v];
                }
            }
        }
}

template <int R>
__global__ __launch_bounds__(256) void apply_T_kernel(const MatDev* __restrict__ mats,
                                                      const WorkItem* __restrict__ items, float ca, float cb)
{
    constexpr int RP = (R < 16) ? 16 : R;          // rank padded to the MFMA tile
    constexpr int NT2 = RP / 16;
    constexpr int NT2W = (NT2 + 1) / 2;            // column tiles per wave (2 waves share a row tile)
    constexpr int P = RP + 4;
    __shared__ float ldsM[kApplyTRows][P];

    const WorkItem it = items[blockIdx.x];
    const MatDev& M = mats[it.mat];
    const long long n = M.n;
    const float* state = M.state;
    // destination: the state itself (momentum transfer, ca = 0, cb = 1: every row block is read
    // into LDS before any of it is written) or another n x r buffer that takes
    // ca * dst + cb * (state T)
    float* dst = M.out ? reinterpret_cast<float*>(M.out) : M.state;
    const float* __restrict__ T = M.T;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int li = lane & 15, kg = lane >> 4;
    const int mtile = wave & 1, half = wave >> 1;

    for (int idx = tid; idx < kApplyTRows * RP; idx += 256) {
        const int rr = idx / RP, k = idx - rr * RP;
        const long long row = (long long)it.row0 + rr;
        ldsM[rr][k] = (row < n && k < R) ? state[row * R + k] : 0.f;
    }
    __syncthreads();

    f32x4 acc[NT2W];
#pragma unroll
    for (int b = 0; b < NT2W; ++b) acc[b] = f32x4{0.f, 0.f, 0.f, 0.f};

#pragma unroll 4
    for (int c = 0; c < RP / 4; ++c) {
        const int k1 = 4 * c + kg;
        const float av = ldsM[mtile * 16 + li][k1];
#pragma unroll
        for (int b = 0; b < NT2W; ++b) {
            const int t2 = half + 2 * b;
            const int k2 = t2 * 16 + li;
            if (t2 < NT2) {
                const float bv = (k1 < R && k2 < R) ? T[k1 * R + k2] : 0.f;
                acc[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bv, acc[b], 0, 0, 0);
            }
        }
    }

#pragma unroll
    for (int b = 0; b < NT2W; ++b) {
        const int t2 = half + 2 * b;
        if (t2 < NT2) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const long long row = (long long)it.row0 + mtile * 16 + 4 * kg + v;
                const int k2 = t2 * 16 + li;
                if (row < n && k2 < R) {
                    const float o = (ca != 0.f) ? dst[row * R + k2] : 0.f;
                    dst[row * R + k2] = ca * o + cb * acc[b][v];
                }
            }
        }
    }
}

}  // namespace

hipError_t launch_transfer_T(const MatDev* mats, int count, int r, hipStream_t s)
{
    if (count == 0) return hipSuccess;
    const dim3 block(256);
#define FLORA_T(RR)                                                                              \
    case RR: {                                                                                   \
        constexpr int kb1 = (RR < 32) ? RR : 32;                                                 \
        hipLaunchKernelGGL((transfer_T_kernel<RR>), dim3((unsigned)(count * ((RR + kb1 - 1) / kb1))), \
                           block, 0, s, mats);                                                   \
    } break;
    switch (r) {
        FLORA_T(8) FLORA_T(16) FLORA_T(32) FLORA_T(64) FLORA_T(128) FLORA_T(256)
    default: return hipErrorInvalidValue;
    }
#undef FLORA_T
    return hipGetLastError();
}

hipError_t launch_apply_T(const MatDev* mats, const WorkItem* items, int nitems, int r, float ca, float cb,
                          hipStream_t s)
{
    if (nitems == 0) return hipSuccess;
    const dim3 grid((unsigned)nitems), block(256);
    switch (r) {
    case 8: hipLaunchKernelGGL((apply_T_kernel<8>), grid, block, 0, s, mats, items, ca, cb); break;
    case 16: hipLaunchKernelGGL((apply_T_kernel<16>), grid, block, 0, s, mats, items, ca, cb); break;
    case 32: hipLaunchKernelGGL((apply_T_kernel<32>), grid, block, 0, s, mats, items, ca, cb); break;
    case 64: hipLaunchKernelGGL((apply_T_kernel<64>), grid, block, 0, s, mats, items, ca, cb); break;
    case 128: hipLaunchKernelGGL((apply_T_kernel<128>), grid, block, 0, s, mats, items, ca, cb); break;
    case 256: hipLaunchKernelGGL((apply_T_kernel<256>), grid, block, 0, s, mats, items, ca, cb); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace flora
