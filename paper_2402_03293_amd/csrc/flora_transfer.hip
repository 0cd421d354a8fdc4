// Momentum transfer (Algorithm 2, resample branch):
//     M <- M A_old^T A_new
// computed in the re-associated order T = A_old^T A_new (r x r), M <- M T, so
// that no n x m intermediate exists.  Everything stays fp32 (fp32 matrix
// cores): an error made here would be carried by every later step.
//
// Ranks 8 / 16 / 32 (T is tiny):
// transfer_T: one workgroup owns up to 32 rows k1 of T and all r columns,
//   sweeps j = 0..m-1 in tiles of 32, regenerating both projections' tiles
//   into LDS ([j][k] layout) and contracting over j with
//   v_mfma_f32_16x16x4_f32.  The reduction order is fixed, so T is
//   reproducible bit for bit.
// apply_T: one workgroup owns 32 rows of M, keeps them in LDS, multiplies by
//   T (read through the caches) and writes the rows back in place.
//
// Ranks 64 / 128 / 256 (2 m r^2 + 2 n r^2 flops per matrix, all fp32):
// transfer_T_big: one workgroup (8 waves) owns a slab of up to 128 rows of T,
//   all r columns and a chunk of 1024 of the m columns j, so the work of a
//   launch is many equal pieces and the new projection is regenerated only
//   r / 128 times; the generator's tiles are double buffered in LDS.  Chunk
//   partials are added in chunk order by combine_T (fixed order, no atomics).
// apply_T_big: one workgroup owns 64 rows of M; a wave keeps its 16 rows in
//   registers as the A operand (16 rows x 64 contiguous bytes per load), T
//   streams through LDS in chunks of 16 rows shared by the four waves.
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


template <int R>
__global__ __launch_bounds__(512) void transfer_T_big_kernel(const MatDev* __restrict__ mats,
                                                             const WorkItem* __restrict__ items)
{
    constexpr int SLAB = (R < 128) ? R : 128;     // rows of T per workgroup
    constexpr int NTR = SLAB / 16;                // 16-row tiles of the slab: one per wave (or per pair)
    constexpr int NH = 8 / NTR;                   // waves that share a row tile split the columns
    constexpr int NT2W = (R / 16) / NH;           // column tiles per wave
    constexpr int P1 = SLAB + 16, P2 = R + 16;    // row strides = 16 mod 32 banks: the four j of an
                                                  // MFMA step land in different halves of the banks
    constexpr int NQ = (SLAB + R) / 4;            // quads per column j (old slab, then new)
    constexpr int QPT = 32 * NQ / 512;            // quads per thread and tile
    __shared__ __attribute__((aligned(16))) float ldsOld[2][kBJ][P1];
    __shared__ __attribute__((aligned(16))) float ldsNew[2][kBJ][P2];

    const WorkItem it = items[blockIdx.x];
    const MatDev& M = mats[it.mat];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15, jg = lane >> 4;
    const int tr = wave % NTR, th = wave / NTR;
    const float cgen = neg2_ln2_over(R);
    const uint32_t so_lo = M.seed_lo, so_hi = M.seed_hi, sn_lo = M.seedn_lo, sn_hi = M.seedn_hi;
    const long long jbeg = it.col0, jend = it.col1;           // this chunk's columns
    const int ntiles = (int)((jend - jbeg + kBJ - 1) / kBJ);
    const uint32_t qold0 = (uint32_t)(it.slice * (SLAB / 4));

    auto gen_tile = [&](int buf, int tile) {
        const long long j0 = jbeg + (long long)tile * kBJ;
#pragma unroll
        for (int i = 0; i < QPT; ++i) {
            const int idx = tid + 512 * i;
            const int q = idx % NQ, jl = idx / NQ;
            const long long j = j0 + jl;
            // (one generator call with selected arguments: lanes of a wave may be on either side)
            const bool isold = q < SLAB / 4;
            const Quad z = normal_quad(isold ? so_lo : sn_lo, isold ? so_hi : sn_hi, (uint64_t)j,
                                       isold ? qold0 + (uint32_t)q : (uint32_t)(q - SLAB / 4), cgen);
            const bool ok = j < jend;
            const v4f v = {ok ? z.z[0] : 0.f, ok ? z.z[1] : 0.f, ok ? z.z[2] : 0.f, ok ? z.z[3] : 0.f};
            if (isold) *reinterpret_cast<v4f*>(&ldsOld[buf][jl][4 * q]) = v;
            else *reinterpret_cast<v4f*>(&ldsNew[buf][jl][4 * (q - SLAB / 4)]) = v;
        }
    };

    f32x4 acc[NT2W];
#pragma unroll
    for (int b = 0; b < NT2W; ++b) acc[b] = f32x4{0.f, 0.f, 0.f, 0.f};

    gen_tile(0, 0);
    __syncthreads();
    for (int tile = 0; tile < ntiles; ++tile) {
        const int buf = tile & 1;
        if (tile + 1 < ntiles) gen_tile(buf ^ 1, tile + 1);
#pragma unroll
        for (int c = 0; c < kBJ / 4; ++c) {
            const float av = ldsOld[buf][4 * c + jg][tr * 16 + li];
#pragma unroll
            for (int b = 0; b < NT2W; ++b) {
                const float bv = ldsNew[buf][4 * c + jg][(th * NT2W + b) * 16 + li];
                acc[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bv, acc[b], 0, 0, 0);
            }
        }
        __syncthreads();
    }

    // partial T of this chunk: rows it.slice * SLAB + tr * 16 + 4 jg + v, column (th NT2W + b) 16 + li
    float* part = M.rowpart + (size_t)it.part * R * R;
#pragma unroll
    for (int b = 0; b < NT2W; ++b)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int k1 = it.slice * SLAB + tr * 16 + 4 * jg + v;
            const int k2 = (th * NT2W + b) * 16 + li;
            stg(part + k1 * R + k2, acc[b][v]);
        }
}

// T <- sum over the chunks of their partials, in chunk order
template <int R>
__global__ __launch_bounds__(256) void combine_T_kernel(const MatDev* __restrict__ mats)
{
    const MatDev& M = mats[blockIdx.y];
    const int idx = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (idx >= R * R) return;
    v4f s = {0.f, 0.f, 0.f, 0.f};
    for (int c = 0; c < M.ncolchunks; ++c) {
        const v4f p = ldg4(M.rowpart + (size_t)c * R * R + idx);
        s.x += p.x; s.y += p.y; s.z += p.z; s.w += p.w;
    }
    *reinterpret_cast<FLORA_GLOBAL v4f*>((FLORA_GLOBAL float*)(M.T + idx)) = s;
}

template <int R>
__global__ __launch_bounds__(256) void apply_T_big_kernel(const MatDev* __restrict__ mats,
                                                          const WorkItem* __restrict__ items, float ca, float cb)
{
    constexpr int NT2 = R / 16;
    constexpr int KC = R / 16;          // chunks of 16 rows of T
    constexpr int P = R + 4;            // row stride = 4 mod 32 banks
    constexpr int F4 = 16 * R / 4 / 256;   // float4 loads per thread and chunk
    __shared__ __attribute__((aligned(16))) float ldsT[2][16][P];

    const WorkItem it = items[blockIdx.x];
    const MatDev& M = mats[it.mat];
    const long long n = M.n;
    const float* state = M.state;
    float* dst = M.out ? reinterpret_cast<float*>(M.out) : M.state;
    const float* __restrict__ T = M.T;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15, jg = lane >> 4;

    // A operand: row li of this wave's 16 rows, columns 16 c + 4 jg .. + 3 for every chunk c.
    // MFMA step (c, t) contracts the index set { 16 c + 4 jg + t : jg < 4 }; the B operand
    // below follows the same order.  Everything is loaded before anything is stored, so the
    // destination may be the state itself.
    long long arow = (long long)it.row0 + wave * 16 + li;
    if (arow > n - 1) arow = n - 1;
    v4f areg[KC];
#pragma unroll
    for (int c = 0; c < KC; ++c) areg[c] = ldg4(state + arow * R + 16 * c + 4 * jg);

    auto fetch_T = [&](v4f (&stage)[F4], int c) {
#pragma unroll
        for (int i = 0; i < F4; ++i) {
            const int f = tid + 256 * i;            // float4 number within the 16 x R chunk
            stage[i] = ldg4(T + (size_t)(16 * c + f / (R / 4)) * R + 4 * (f % (R / 4)));
        }
    };
    auto stash_T = [&](const v4f (&stage)[F4], int buf) {
#pragma unroll
        for (int i = 0; i < F4; ++i) {
            const int f = tid + 256 * i;
            *reinterpret_cast<v4f*>(&ldsT[buf][f / (R / 4)][4 * (f % (R / 4))]) = stage[i];
        }
    };

    f32x4 acc[NT2];
#pragma unroll
    for (int b = 0; b < NT2; ++b) acc[b] = f32x4{0.f, 0.f, 0.f, 0.f};

    v4f stage[F4];
    fetch_T(stage, 0);
    stash_T(stage, 0);
    __syncthreads();
#pragma unroll
    for (int c = 0; c < KC; ++c) {
        const int buf = c & 1;
        if (c + 1 < KC) fetch_T(stage, c + 1);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const float av = areg[c][t];
#pragma unroll
            for (int b = 0; b < NT2; ++b)
                acc[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, ldsT[buf][4 * jg + t][b * 16 + li], acc[b], 0, 0, 0);
        }
        if (c + 1 < KC) stash_T(stage, buf ^ 1);
        __syncthreads();
    }

#pragma unroll
    for (int b = 0; b < NT2; ++b)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const long long row = (long long)it.row0 + wave * 16 + 4 * jg + v;
            if (row < n && row < (long long)it.row0 + it.rows) {
                float* o = dst + row * R + b * 16 + li;
                const float old = (ca != 0.f) ? ldg(o) : 0.f;
                stg(o, ca * old + cb * acc[b][v]);
            }
        }
}

}  // namespace

hipError_t launch_transfer_T(const MatDev* mats, const WorkItem* items, int nitems, int count, int r, hipStream_t s)
{
    if (count == 0) return hipSuccess;
    if (r >= 64) {
        // items: (matrix, chunk of columns, slab of rows of T); then the chunks are summed
        const dim3 grid((unsigned)nitems);
        switch (r) {
        case 64:
            hipLaunchKernelGGL((transfer_T_big_kernel<64>), grid, dim3(512), 0, s, mats, items);
            hipLaunchKernelGGL((combine_T_kernel<64>), dim3(64 * 64 / 1024, (unsigned)count), dim3(256), 0, s, mats);
            break;
        case 128:
            hipLaunchKernelGGL((transfer_T_big_kernel<128>), grid, dim3(512), 0, s, mats, items);
            hipLaunchKernelGGL((combine_T_kernel<128>), dim3(128 * 128 / 1024, (unsigned)count), dim3(256), 0, s, mats);
            break;
        case 256:
            hipLaunchKernelGGL((transfer_T_big_kernel<256>), grid, dim3(512), 0, s, mats, items);
            hipLaunchKernelGGL((combine_T_kernel<256>), dim3(256 * 256 / 1024, (unsigned)count), dim3(256), 0, s, mats);
            break;
        default: return hipErrorInvalidValue;
        }
        return hipGetLastError();
    }
    const dim3 block(256);
#define FLORA_T(RR)                                                                              \
    case RR: {                                                                                   \
        constexpr int kb1 = (RR < 32) ? RR : 32;                                                 \
        hipLaunchKernelGGL((transfer_T_kernel<RR>), dim3((unsigned)(count * ((RR + kb1 - 1) / kb1))), \
                           block, 0, s, mats);                                                   \
    } break;
    switch (r) {
        FLORA_T(8) FLORA_T(16) FLORA_T(32)
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
    case 64: hipLaunchKernelGGL((apply_T_big_kernel<64>), grid, block, 0, s, mats, items, ca, cb); break;
    case 128: hipLaunchKernelGGL((apply_T_big_kernel<128>), grid, block, 0, s, mats, items, ca, cb); break;
    case 256: hipLaunchKernelGGL((apply_T_big_kernel<256>), grid, block, 0, s, mats, items, ca, cb); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace flora
