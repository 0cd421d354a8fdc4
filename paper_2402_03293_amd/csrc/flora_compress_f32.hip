// Compression on the fp32 matrix cores, ranks 8 / 16 / 32:
//     state <- a * state + b * (G A(seed))
// (Algorithm 1, compression line with a = b = 1; Algorithm 2, EMA line with
// a = beta, b = 1 - beta).  G is fp32 or bf16 and is used exactly; products and
// sums are fp32 (v_mfma_f32_16x16x4_f32).
//
// One workgroup (4 waves) owns 64 * MT rows of one matrix and sweeps all m
// columns in tiles of 64.  For each tile the workgroup regenerates the
// 64 x r slice of A once into LDS (transposed, [k][j]) and every wave reads
// its B operands from there, while G streams from HBM straight into the A
// operand registers: lane (row i = lane % 16, group g = lane / 16) loads the
// four consecutive columns j0 + 16c + 4g .. +3, and MFMA number (c, t) contracts
// the column set { j0 + 16c + 4g + t : g = 0..3 }.  The order in which columns
// are contracted is free as long as both operands agree on it.
#include "flora_gen.hip.h"
#include "flora_internal.h"

namespace flora {

namespace {

constexpr int kBK = 64;         // columns of G per tile
constexpr int kLda = kBK + 4;   // padded LDS row (floats)

__device__ __forceinline__ float4 load4(const float* rowp, long long col, long long m, bool fast)
{
    if (fast) return *reinterpret_cast<const float4*>(rowp + col);
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (col < m) v.x = rowp[col];
    if (col + 1 < m) v.y = rowp[col + 1];
    if (col + 2 < m) v.z = rowp[col + 2];
    if (col + 3 < m) v.w = rowp[col + 3];
    return v;
}

__device__ __forceinline__ float4 load4(const uint16_t* rowp, long long col, long long m, bool fast)
{
    uint32_t e0 = 0, e1 = 0, e2 = 0, e3 = 0;
    if (fast) {
        const uint2 p = *reinterpret_cast<const uint2*>(rowp + col);
        e0 = p.x & 0xffffu; e1 = p.x >> 16; e2 = p.y & 0xffffu; e3 = p.y >> 16;
    } else {
        if (col < m) e0 = rowp[col];
        if (col + 1 < m) e1 = rowp[col + 1];
        if (col + 2 < m) e2 = rowp[col + 2];
        if (col + 3 < m) e3 = rowp[col + 3];
    }
    return make_float4(bf16_bits_to_f32(e0), bf16_bits_to_f32(e1), bf16_bits_to_f32(e2),
                       bf16_bits_to_f32(e3));
}

template <int R, typename GT, int MT>
__global__ __launch_bounds__(256) void compress_f32_kernel(const MatDev* __restrict__ mats,
                                                           const WorkItem* __restrict__ items,
                                                           const SeedArgs seeds, float a, float b)
{
    constexpr int NT = (R + 15) / 16;   // 16-wide column tiles of the state
    constexpr int RP = NT * 16;
    __shared__ float ldsA[2][RP][kLda];

    const WorkItem it = items[blockIdx.x];
    const MatDev& M = mats[it.mat];
    const long long n = M.n, m = M.m;
    const uint32_t seed_lo = seeds.s[it.mat].x, seed_hi = seeds.s[it.mat].y;
    const GT* __restrict__ G = reinterpret_cast<const GT*>(M.grad);
    float* __restrict__ state = M.state;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int li = lane & 15, g = lane >> 4;
    const float cgen = neg2_ln2_over(R);
    const bool vec_ok = (m % 4) == 0;
    const int ntiles = (int)((m + kBK - 1) / kBK);
    const int nfull = vec_ok ? (int)(m / kBK) : 0;

    if (R < RP) {   // rank 8: the upper half of the 16-wide tile is zero padding
        for (int idx = tid; idx < 2 * (RP - R) * kLda; idx += 256) {
            const int bufi = idx / ((RP - R) * kLda);
            const int rem = idx - bufi * (RP - R) * kLda;
            ldsA[bufi][R + rem / kLda][rem % kLda] = 0.f;
        }
    }

    const GT* rowp[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        long long row = (long long)it.row0 + wave * (MT * 16) + mt * 16 + li;
        if (row > n - 1) row = n - 1;
        rowp[mt] = G + row * m;
    }

    auto load_tile = [&](float4 (&dst)[MT][4], int tile) {
        const bool fast = tile < nfull;
        const long long j0 = (long long)tile * kBK;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int c = 0; c < 4; ++c)
                dst[mt][c] = load4(rowp[mt], j0 + 16 * c + 4 * g, m, fast);
    };

    auto gen_tile = [&](int buf, int tile) {
        constexpr int QT = kBK * (R / 4);
        const long long j0 = (long long)tile * kBK;
#pragma unroll
        for (int idx0 = 0; idx0 < QT; idx0 += 256) {
            const int idx = idx0 + tid;
            if (QT % 256 == 0 || idx < QT) {
                const int jl = idx % kBK;
                const int q = idx / kBK;
                const Quad z = normal_quad(seed_lo, seed_hi, (uint64_t)(j0 + jl), (uint32_t)q, cgen);
#pragma unroll
                for (int i = 0; i < 4; ++i) ldsA[buf][4 * q + i][jl] = z.z[i];
            }
        }
    };

    f32x4 acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};

    float4 cur[MT][4], nxt[MT][4];
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
        for (int c = 0; c < 4; ++c) {
            float4 bv[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                bv[nt] = *reinterpret_cast<const float4*>(&ldsA[buf][nt * 16 + li][16 * c + 4 * g]);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const float av[4] = {cur[mt][c].x, cur[mt][c].y, cur[mt][c].z, cur[mt][c].w};
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const float bw[4] = {bv[nt].x, bv[nt].y, bv[nt].z, bv[nt].w};
#pragma unroll
                    for (int t = 0; t < 4; ++t)
                        acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[t], bw[t], acc[mt][nt], 0, 0, 0);
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int c = 0; c < 4; ++c) cur[mt][c] = nxt[mt][c];
    }

    // D layout of the 16x16 tile: lane holds column lane % 16, rows 4 * (lane / 16) + v.
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int k = nt * 16 + li;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const long long row = (long long)it.row0 + wave * (MT * 16) + mt * 16 + 4 * g + v;
                if (row < n && k < R) {
                    float* p = state + row * R + k;
                    const float old = (a != 0.f) ? *p : 0.f;
                    *p = a * old + b * acc[mt][nt][v];
                }
            }
        }
    }
}

template <int R, typename GT>
hipError_t launch_one(const MatDev* mats, const WorkItem* items, int nitems, const SeedArgs& seeds,
                      float a, float b, hipStream_t s)
{
    constexpr int MT = kCompressF32Rows / 64;
    hipLaunchKernelGGL((compress_f32_kernel<R, GT, MT>), dim3((unsigned)nitems), dim3(256), 0, s,
                       mats, items, seeds, a, b);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_compress_f32(const MatDev* mats, const WorkItem* items, int nitems, const SeedArgs& seeds,
                               int r, int grad_is_bf16, float a, float b, hipStream_t s)
{
    if (nitems == 0) return hipSuccess;
    if (!grad_is_bf16) {
        if (r == 8) return launch_one<8, float>(mats, items, nitems, seeds, a, b, s);
        if (r == 16) return launch_one<16, float>(mats, items, nitems, seeds, a, b, s);
        if (r == 32) return launch_one<32, float>(mats, items, nitems, seeds, a, b, s);
    } else {
        if (r == 8) return launch_one<8, uint16_t>(mats, items, nitems, seeds, a, b, s);
        if (r == 16) return launch_one<16, uint16_t>(mats, items, nitems, seeds, a, b, s);
        if (r == 32) return launch_one<32, uint16_t>(mats, items, nitems, seeds, a, b, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace flora
