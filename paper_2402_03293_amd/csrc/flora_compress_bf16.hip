// Compression on the bf16 matrix cores, ranks 64 / 128 / 256, bf16 gradients:
//     state <- a * state + b * (G A(seed))
// (Algorithm 1, compression line; Algorithm 2, EMA line).  A is rounded to
// bf16 as it is generated; products are exact in fp32 and accumulated in fp32
// (v_mfma_f32_32x32x16_bf16).
//
// The cost that matters here is regenerating A, not the contraction: every
// workgroup that sweeps the m columns of G must rebuild all the A rows it
// meets, so the number of Philox + Box-Muller evaluations is n m r / (rows per
// workgroup).  A workgroup therefore owns as many rows as its accumulators
// allow (128 * MT, MT <= 4) but only a 64-wide slice of the rank axis; the
// r / 64 workgroups of one row block read the same G (from L2 after the first)
// and write disjoint columns of the state.
//
// Per tile of 32 columns of G: the workgroup regenerates the 32 x 64 slice of A
// into LDS as bf16, transposed ([k][j]); lane (row i = lane % 32, half
// g = lane / 32) loads the 16 consecutive bf16 G[i, j0 + 16 g .. +15] and MFMA
// step t contracts the column set { j0 + 16 g + 8 t + e : g < 2, e < 8 }.
#include "flora_gen.hip.h"
#include "flora_internal.h"

namespace flora {

namespace {

constexpr int kBK = 32;            // columns of G per tile
constexpr int kLda = kBK + 8;      // padded LDS row (bf16 elements): 80 bytes
constexpr int kRS = kCompressBf16Slice;

template <int MT>
__global__ __launch_bounds__(256) void compress_bf16_kernel(const MatDev* __restrict__ mats,
                                                            const WorkItem* __restrict__ items,
                                                            const SeedArgs seeds, int R, float a, float b)
{
    constexpr int NT = kRS / 32;
    __shared__ __attribute__((aligned(16))) uint16_t ldsA[2][kRS][kLda];

    const WorkItem it = items[blockIdx.x];
    const MatDev& M = mats[it.mat];
    const long long n = M.n, m = M.m;
    const uint32_t seed_lo = seeds.s[it.mat].x, seed_hi = seeds.s[it.mat].y;
    const uint16_t* __restrict__ G = reinterpret_cast<const uint16_t*>(M.grad);
    float* __restrict__ state = M.state;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, g = lane >> 5;
    const float cgen = neg2_ln2_over(R);
    const bool vec_ok = (m % 8) == 0;
    const int ntiles = (int)((m + kBK - 1) / kBK);
    const int nfull = vec_ok ? (int)(m / kBK) : 0;
    const int q0 = it.slice * (kRS / 4);   // first Philox quad of this rank slice

    const uint16_t* rowp[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        long long row = (long long)it.row0 + wave * (MT * 32) + mt * 32 + li;
        if (row > n - 1) row = n - 1;
        rowp[mt] = G + row * m;
    }

    auto load_tile = [&](v4u (&dst)[MT][2], int tile) {
        const long long j0 = (long long)tile * kBK + 16 * g;
        if (tile < nfull) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                dst[mt][0] = ldg4(rowp[mt] + j0);
                dst[mt][1] = ldg4(rowp[mt] + j0 + 8);
            }
        } else {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                uint32_t w[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const long long c0 = j0 + 2 * e;
                    const uint32_t lo = (c0 < m) ? ldg(rowp[mt] + c0) : 0u;
                    const uint32_t hi = (c0 + 1 < m) ? ldg(rowp[mt] + c0 + 1) : 0u;
                    w[e] = lo | (hi << 16);
                }
                dst[mt][0] = v4u{w[0], w[1], w[2], w[3]};
                dst[mt][1] = v4u{w[4], w[5], w[6], w[7]};
            }
        }
    };

    // 32 x 64 normals per tile = 512 quads; thread p takes the two quads (j, q), (j + 1, q)
    // with j = 2 (p % 16), q = p / 16, and writes packed pairs of bf16.
    auto gen_tile = [&](int buf, int tile) {
        const int jl = 2 * (tid & 15);
        const int q = tid >> 4;
        const uint64_t j = (uint64_t)tile * kBK + jl;
        const Quad z0 = normal_quad(seed_lo, seed_hi, j, (uint32_t)(q0 + q), cgen);
        const Quad z1 = normal_quad(seed_lo, seed_hi, j + 1, (uint32_t)(q0 + q), cgen);
#pragma unroll
        for (int i = 0; i < 4; ++i)
            *reinterpret_cast<uint32_t*>(&ldsA[buf][4 * q + i][jl]) = pack_bf16x2(z0.z[i], z1.z[i]);
    };

    f32x16 acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mt][nt][v] = 0.f;

    v4u cur[MT][2], nxt[MT][2];
    load_tile(cur, 0);
    gen_tile(0, 0);
    __syncthreads();

    for (int tile = 0; tile < ntiles; ++tile) {
        const int buf = tile & 1;
        if (tile + 1 < ntiles) {
            load_tile(nxt, tile + 1);
            gen_tile(buf ^ 1, tile + 1);
        }
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            bf16x8 bv[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                bv[nt] = *reinterpret_cast<const bf16x8*>(&ldsA[buf][nt * 32 + li][16 * g + 8 * t]);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const bf16x8 av = __builtin_bit_cast(bf16x8, cur[mt][t]);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv[nt], acc[mt][nt], 0, 0, 0);
            }
        }
        __syncthreads();
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            cur[mt][0] = nxt[mt][0];
            cur[mt][1] = nxt[mt][1];
        }
    }

    // D layout of the 32x32 tile: lane holds column lane % 32 and, in register v,
    // row 8 * (v / 4) + 4 * (lane / 32) + v % 4.  Old values are fetched 16 at a time
    // (clamped addresses) before the new ones are stored.
    const long long row_end = ((long long)it.row0 + it.rows < n) ? (long long)it.row0 + it.rows : n;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int k = it.slice * kRS + nt * 32 + li;
            float old[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                long long row = (long long)it.row0 + wave * (MT * 32) + mt * 32 + 8 * (v / 4) + 4 * g + (v % 4);
                if (row > row_end - 1) row = row_end - 1;
                old[v] = (a != 0.f) ? ldg(state + row * R + k) : 0.f;
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const long long row = (long long)it.row0 + wave * (MT * 32) + mt * 32 + 8 * (v / 4) + 4 * g + (v % 4);
                if (row < row_end) stg(state + row * R + k, a * old[v] + b * acc[mt][nt][v]);
            }
        }
    }
}

}  // namespace

// All items of one launch share one MT (rows per workgroup = 128 * MT), chosen by the host.
hipError_t launch_compress_bf16_mt(const MatDev* mats, const WorkItem* items, int nitems,
                                   const SeedArgs& seeds, int r, int mt, float a, float b, hipStream_t s)
{
    if (nitems == 0) return hipSuccess;
    if (r != 64 && r != 128 && r != 256) return hipErrorInvalidValue;
    const dim3 grid((unsigned)nitems), block(256);
    switch (mt) {
    case 1: hipLaunchKernelGGL((compress_bf16_kernel<1>), grid, block, 0, s, mats, items, seeds, r, a, b); break;
    case 2: hipLaunchKernelGGL((compress_bf16_kernel<2>), grid, block, 0, s, mats, items, seeds, r, a, b); break;
    case 4: hipLaunchKernelGGL((compress_bf16_kernel<4>), grid, block, 0, s, mats, items, seeds, r, a, b); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace flora
