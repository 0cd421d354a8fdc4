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


// ---------------------------------------------------------------------------
// Wide variant: 8 waves own 512 rows x (32 NT) rank columns and sweep m in tiles
// of 64 columns.  It needs rows of G that start on 16-byte boundaries (m % 8 == 0);
// the kernel above remains for everything else.
//
// What bounds this kernel is, in this order, HBM (G is read once from HBM and
// r / (32 NT) - 1 more times from L2), the vector ALU that regenerates A
// (evaluations = n m r / 512) and the matrix cores.  To let the three overlap:
//   * wave w owns rows 64 w .. 64 w + 63 and all 32 NT columns, so G goes from
//     memory straight into its A-operand registers and is never shared; a lane
//     (row i = lane % 32, half g = lane / 32) loads the 32 consecutive bf16
//     G[i, j0 + 32 g .. +31] and MFMA step t contracts the column set
//     { j0 + 32 g + 8 t + e : g < 2, e < 8 }; per row that is one 128-byte line;
//   * the registers of a tile are refilled with the tile two steps ahead as soon
//     as the MFMAs that read them have been issued (two register sets, loop
//     unrolled by two), so about one and a half tiles are in flight per wave;
//   * the 64 x (32 NT) slice of A is regenerated once per tile by all 512 threads
//     into LDS (bf16, transposed, double buffered); waves 0-3 generate first and
//     multiply second, waves 4-7 the other way round, so that the two waves of
//     a SIMD keep its vector ALU and its matrix core busy at the same time.
constexpr int kWBK = 64;             // columns of G per tile
constexpr int kWLda = kWBK + 8;      // padded LDS row (bf16 elements): 144 bytes

template <int NT>
__global__ __launch_bounds__(512) void compress_bf16_wide_kernel(const MatDev* __restrict__ mats,
                                                                 const WorkItem* __restrict__ items,
                                                                 const SeedArgs seeds, int R, float a, float b)
{
    constexpr int RS = 32 * NT;      // rank columns of this workgroup
    constexpr int JG = kWBK / NT;    // threads along j when generating (each takes NT columns j)
    __shared__ __attribute__((aligned(16))) uint16_t ldsA[2][RS][kWLda];

    const WorkItem it = items[blockIdx.x];
    const MatDev& M = mats[it.mat];
    const long long n = M.n, m = M.m;
    const uint32_t seed_lo = seeds.s[it.mat].x, seed_hi = seeds.s[it.mat].y;
    const uint16_t* __restrict__ G = reinterpret_cast<const uint16_t*>(M.grad);
    float* __restrict__ state = M.state;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 31, g = lane >> 5;
    const float cgen = neg2_ln2_over(R);
    const int ntiles = (int)((m + kWBK - 1) / kWBK);
    const uint32_t q0 = (uint32_t)(it.slice * (RS / 4));   // first Philox quad of this rank slice

    // One buffer resource per 32-row tile of this wave, covering exactly its valid rows:
    // rows past n and (through kOob) columns past m read as zero.
    rsrc_t rs[2];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
        const long long first = (long long)it.row0 + wave * 64 + mt * 32;
        const long long row_end = ((long long)it.row0 + it.rows < n) ? (long long)it.row0 + it.rows : n;
        long long valid = row_end - first;
        valid = valid < 0 ? 0 : (valid > 32 ? 32 : valid);
        rs[mt] = make_rsrc(G + (first < n ? first : 0) * m, valid * m * 2);
    }
    const uint32_t lane_off = ((uint32_t)li * (uint32_t)m + 32u * (uint32_t)g) * 2u;

    // Byte offset of this lane's chunk t of a tile (kOob when the chunk lies past column m;
    // m % 8 == 0, so a chunk is all in or all out).
    auto chunk_off = [&](int tile, int t) -> uint32_t {
        const uint32_t col = (uint32_t)tile * kWBK + 32u * (uint32_t)g + 8u * (uint32_t)t;
        return col < (uint32_t)m ? lane_off + ((uint32_t)tile * kWBK + 8u * (uint32_t)t) * 2u : kOob;
    };
    auto load_tile = [&](v4u (&dst)[2][4], int tile) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const uint32_t off = chunk_off(tile, t);
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) dst[mt][t] = buf_load_u4(rs[mt], off);
        }
    };

    // 64 x RS normals per tile = 16 RS quads, NT per thread: thread p takes quad index
    // q = p / JG for the NT consecutive columns j = NT (p % JG) .. + NT - 1 and writes, for
    // each of the quad's four rank columns, NT packed bf16 along j.  The quads are evaluated
    // one after the other (a wave gains nothing from interleaving them, and the registers
    // are needed elsewhere); the scheduling barriers keep the compiler from mixing them.
    const int gen_j = NT * (tid % JG);
    const uint32_t gen_q = (uint32_t)(tid / JG);
    auto gen_tile = [&](int buf, int tile) {
        const uint64_t j = (uint64_t)tile * kWBK + (uint64_t)gen_j;
        uint32_t pk[NT / 2][4];
#pragma unroll
        for (int e = 0; e < NT; e += 2) {
            const Quad z0 = normal_quad(seed_lo, seed_hi, j + e, q0 + gen_q, cgen);
            __builtin_amdgcn_sched_barrier(0);
            const Quad z1 = normal_quad(seed_lo, seed_hi, j + e + 1, q0 + gen_q, cgen);
#pragma unroll
            for (int i = 0; i < 4; ++i) pk[e / 2][i] = pack_bf16x2(z0.z[i], z1.z[i]);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            uint16_t* dst = &ldsA[buf][4 * gen_q + i][gen_j];
            if (NT == 4) *reinterpret_cast<uint2*>(dst) = make_uint2(pk[0][i], pk[NT / 2 - 1][i]);
            else *reinterpret_cast<uint32_t*>(dst) = pk[0][i];
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    f32x16 acc[2][NT];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mt][nt][v] = 0.f;

    // The tile in `gt` / LDS buffer `buf` goes through the matrix cores; as soon as the MFMAs
    // of chunk t are issued, the registers of chunk t are refilled with the tile two steps
    // ahead (past the end every chunk is out of range and nothing is fetched).
    auto mfma_tile = [&](v4u (&gt)[2][4], int buf, int tile) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            bf16x8 bv[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                bv[nt] = *reinterpret_cast<const bf16x8*>(&ldsA[buf][nt * 32 + li][32 * g + 8 * t]);
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
                const bf16x8 av = __builtin_bit_cast(bf16x8, gt[mt][t]);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv[nt], acc[mt][nt], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            const uint32_t off = chunk_off(tile + 2, t);
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) gt[mt][t] = buf_load_u4(rs[mt], off);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // Schedule.  Barrier number t separates the multiplication of tile t from that of tile
    // t + 1.  Waves 4-7 ("late") generate their share of tile t + 1 right after multiplying
    // tile t, before barrier t; waves 0-3 ("early") generate their share of tile t + 2 right
    // after barrier t, into the buffer tile t has just left, while the late waves already
    // multiply tile t + 1.  Either way a share of tile t + 1 is complete before barrier t and
    // overwrites a buffer whose last readers passed barrier t - 1.  The accumulators are
    // touched by one code path only.
    const bool early = wave < 4;
    auto gen_if = [&](bool mine, int buf, int tile) {
        if (mine && tile < ntiles) gen_tile(buf, tile);
    };

    v4u gx[2][4], gy[2][4];
    load_tile(gx, 0);
    load_tile(gy, 1);
    gen_tile(0, 0);
    gen_if(early, 1, 1);
    __syncthreads();
    for (int tile = 0;; tile += 2) {
        mfma_tile(gx, 0, tile);
        gen_if(!early, 1, tile + 1);
        __syncthreads();
        gen_if(early, 0, tile + 2);
        if (tile + 1 >= ntiles) break;
        mfma_tile(gy, 1, tile + 1);
        gen_if(!early, 0, tile + 2);
        __syncthreads();
        gen_if(early, 1, tile + 3);
        if (tile + 2 >= ntiles) break;
    }

    // D layout of a 32x32 tile: lane holds column lane % 32 and, in register v,
    // row 8 * (v / 4) + 4 * (lane / 32) + v % 4.
    const long long row_end = ((long long)it.row0 + it.rows < n) ? (long long)it.row0 + it.rows : n;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int k = it.slice * RS + nt * 32 + li;
            float old[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                long long row = (long long)it.row0 + wave * 64 + mt * 32 + 8 * (v / 4) + 4 * g + (v % 4);
                if (row > row_end - 1) row = row_end - 1;
                old[v] = (a != 0.f) ? ldg(state + row * R + k) : 0.f;
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const long long row = (long long)it.row0 + wave * 64 + mt * 32 + 8 * (v / 4) + 4 * g + (v % 4);
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
    if (mt == 8) {   // wide kernel: 512 rows per workgroup, rank slices of 128 (64 at r = 64)
        const dim3 grid((unsigned)nitems), block(512);
        if (r == 64) hipLaunchKernelGGL((compress_bf16_wide_kernel<2>), grid, block, 0, s, mats, items, seeds, r, a, b);
        else hipLaunchKernelGGL((compress_bf16_wide_kernel<4>), grid, block, 0, s, mats, items, seeds, r, a, b);
        return hipGetLastError();
    }
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
