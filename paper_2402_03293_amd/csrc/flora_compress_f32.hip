// Compression on the fp32 matrix cores, ranks 8 / 16 / 32:
//     state <- a * state + b * (G A(seed))
// (Algorithm 1, compression line with a = b = 1; Algorithm 2, EMA line with
// a = beta, b = 1 - beta).  G is fp32 or bf16 and is used exactly; products and
// sums are fp32 (v_mfma_f32_16x16x4_f32).  With MAP = 1 the input is the elementwise
// square of G, taken in fp32 on the operand registers (the compressed EMA of another
// statistic that the "Sublinear memory momentum" paragraph of Section 2.4 closes with: here the second moment).
//
// One workgroup owns 64 * MT rows of one matrix and sweeps all m columns in
// tiles of 64.  Its 4 * KG waves form KG column groups of 4 waves; group kg
// takes tiles kg, kg + KG, ... so the chain of dependent tiles per wave is KG
// times shorter, and the groups' partial sums meet in LDS at the end (fixed
// order).  For each tile a group regenerates the 64 x r slice of A once into
// LDS (transposed, [k][j]) and its waves read their B operands from there,
// while G streams from HBM straight into the A
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
constexpr int kPF = 2;          // G tiles in flight per wave (register stages)

__device__ __forceinline__ v4f load4(const float* rowp, long long col, long long m, bool fast)
{
    if (fast) return ldg4(rowp + col);
    v4f v = {0.f, 0.f, 0.f, 0.f};
    if (col < m) v.x = ldg(rowp + col);
    if (col + 1 < m) v.y = ldg(rowp + col + 1);
    if (col + 2 < m) v.z = ldg(rowp + col + 2);
    if (col + 3 < m) v.w = ldg(rowp + col + 3);
    return v;
}

__device__ __forceinline__ v4f load4(const uint16_t* rowp, long long col, long long m, bool fast)
{
    uint32_t e0 = 0, e1 = 0, e2 = 0, e3 = 0;
    if (fast) {
        const v2u p = ldg2(rowp + col);
        e0 = p.x & 0xffffu; e1 = p.x >> 16; e2 = p.y & 0xffffu; e3 = p.y >> 16;
    } else {
        if (col < m) e0 = ldg(rowp + col);
        if (col + 1 < m) e1 = ldg(rowp + col + 1);
        if (col + 2 < m) e2 = ldg(rowp + col + 2);
        if (col + 3 < m) e3 = ldg(rowp + col + 3);
    }
    v4f v = {bf16_bits_to_f32(e0), bf16_bits_to_f32(e1), bf16_bits_to_f32(e2), bf16_bits_to_f32(e3)};
    return v;
}

template <int R, typename GT, int MT, int KG, int MAP>
__global__ __launch_bounds__(256 * KG) void compress_f32_kernel(const MatDev* __restrict__ mats,
                                                                const WorkItem* __restrict__ items,
                                                                const SeedArgs seeds, float a, float b,
                                                                float* __restrict__ partials,
                                                                uint32_t* __restrict__ counters)
{
    constexpr int NT = (R + 15) / 16;   // 16-wide column tiles of the state
    constexpr int RP = NT * 16;
    constexpr int ROWS = 64 * MT;       // rows per workgroup
    __shared__ float ldsA[KG][2][RP][kLda];
    __shared__ float ldsRed[(KG > 1) ? KG - 1 : 1][(KG > 1) ? ROWS : 1][RP + 1];

    const WorkItem it = items[blockIdx.x];
    const MatDev& M = mats[it.mat];
    const long long n = M.n, m = M.m;
    const uint32_t seed_lo = seeds.s[it.mat].x, seed_hi = seeds.s[it.mat].y;
    const GT* __restrict__ G = reinterpret_cast<const GT*>(M.grad);
    float* __restrict__ state = M.state;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave_id = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform by construction
    const int kg = wave_id >> 2;          // column group of this wave
    const int tg = tid & 255;             // thread index within the group
    const int wave = wave_id & 3;         // row slot of this wave within the group
    const int li = lane & 15, g = lane >> 4;
    const float cgen = neg2_ln2_over(R);
    const bool vec_ok = (m % 4) == 0;
    // this workgroup's share of the columns: [col0, col_end), tiles tbase .. tbase + ntiles - 1
    const long long col_end = (it.col1 < m) ? (long long)it.col1 : m;
    const int tbase = it.col0 / kBK;
    const int ntiles = (int)((col_end - it.col0 + kBK - 1) / kBK);
    const int iters = (ntiles + KG - 1) / KG;       // tiles per group (the last may be missing)

    if (R < RP) {   // rank 8: the upper half of the 16-wide tile is zero padding
        for (int idx = tg; idx < 2 * (RP - R) * kLda; idx += 256) {
            const int bufi = idx / ((RP - R) * kLda);
            const int rem = idx - bufi * (RP - R) * kLda;
            ldsA[kg][bufi][R + rem / kLda][rem % kLda] = 0.f;
        }
    }

    const GT* rowp[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        long long row = (long long)it.row0 + wave * (MT * 16) + mt * 16 + li;
        if (row > n - 1) row = n - 1;
        rowp[mt] = G + row * m;
    }

    // Round i gives tile i * KG + kg to group kg.  When rows are 16-byte aligned (m % 4 == 0)
    // every round runs in the pipelined loop: loads go through a per-wave buffer resource
    // that covers exactly the valid rows, a chunk that starts at or beyond column m (ragged
    // last tile) or belongs to a round past the end (prefetch) is pointed out of range and
    // comes back as zeros.  Matrices with unaligned rows take the plain guarded loop below.
    constexpr int ESZ = (int)sizeof(GT);
    const int fast_rounds = vec_ok ? iters : 0;
    rsrc_t rs[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const long long first = (long long)it.row0 + wave * (MT * 16) + mt * 16;
        long long valid = n - first;
        valid = valid < 0 ? 0 : (valid > 16 ? 16 : valid);
        rs[mt] = make_rsrc(G + (first < n ? first : 0) * m, valid * m * ESZ);
    }
    // fp32 gradients are fetched eight rows x 128 bytes per instruction (whole lines, which the
    // load path moves faster than the 16 rows x 64 bytes the operand layout asks for): load
    // (h, L) of a 16-row block takes, in lane (li, g), row 8 h + li % 8 and the 16 bytes at column
    // 32 L + 16 (li / 8) + 4 g.  The lanes li < 8 of load (0, L) and the lanes li >= 8 of load
    // (1, L) then hold what operand registers c = 2 L and c = 2 L + 1 want, and the other halves
    // each other's: settle_tile swaps those within each row of 16 lanes with DPP moves, right
    // before the tile multiplies.  bf16 gradients (8 bytes per lane) keep the direct pattern.
    constexpr bool kLines = ESZ == 4;
    const uint32_t lane_off = kLines ? ((uint32_t)(li & 7) * (uint32_t)m + 4u * (uint32_t)g + 16u * (uint32_t)(li >> 3)) * ESZ
                                     : ((uint32_t)li * (uint32_t)m + 4u * (uint32_t)g) * ESZ;

    auto load_tile_fast = [&](v4f (&dst)[MT][4], int i) {
        const int tile = tbase + kg + KG * i;
        // a round past the end has a tile past the last one, so its columns fail the same test
        if constexpr (kLines) {
            const uint32_t col0 = (uint32_t)tile * kBK + 4u * (uint32_t)g + 16u * (uint32_t)(li >> 3);
#pragma unroll
            for (int L = 0; L < 2; ++L) {
                const bool ok = col0 + 32u * L < (uint32_t)col_end;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const uint32_t off = ok ? lane_off + (8u * h * (uint32_t)m + (uint32_t)tile * kBK + 32u * L) * ESZ : kOob;
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) dst[mt][2 * L + h] = buf_load_f4<true>(rs[mt], off);   // G is read once: streamed
                }
            }
        } else {
            const uint32_t col0 = (uint32_t)tile * kBK + 4u * (uint32_t)g;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const bool ok = col0 + 16u * c < (uint32_t)col_end;
                const uint32_t off = ok ? lane_off + ((uint32_t)tile * kBK + 16u * c) * ESZ : kOob;
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const v2u p2 = buf_load_u2<true>(rs[mt], off);
                    dst[mt][c] = v4f{bf16_bits_to_f32(p2.x & 0xffffu), bf16_bits_to_f32(p2.x >> 16),
                                     bf16_bits_to_f32(p2.y & 0xffffu), bf16_bits_to_f32(p2.y >> 16)};
                }
            }
        }
    };
    auto settle_tile = [&](v4f (&t)[MT][4]) {
        if constexpr (kLines) {
            constexpr int kRor8 = 0x128;      // DPP row_ror:8: lane li of a row of 16 reads lane li ^ 8
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int L = 0; L < 2; ++L)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int lo = __float_as_int(t[mt][2 * L][e]), hi = __float_as_int(t[mt][2 * L + 1][e]);
                        // c = 2 L: lanes li >= 8 (banks 2, 3) take load (1, L)'s lanes li - 8
                        t[mt][2 * L][e] = __int_as_float(__builtin_amdgcn_update_dpp(lo, hi, kRor8, 0xf, 0xc, false));
                        // c = 2 L + 1: lanes li < 8 (banks 0, 1) take load (0, L)'s lanes li + 8
                        t[mt][2 * L + 1][e] = __int_as_float(__builtin_amdgcn_update_dpp(hi, lo, kRor8, 0xf, 0x3, false));
                    }
        }
    };

    auto gen_tile = [&](int buf, int i) {
        constexpr int QT = kBK * (R / 4);
        const long long j0 = (long long)(tbase + kg + KG * i) * kBK;
#pragma unroll
        for (int idx0 = 0; idx0 < QT; idx0 += 256) {
            const int idx = idx0 + tg;
            if (QT % 256 == 0 || idx < QT) {
                const int jl = idx % kBK;
                const int q = idx / kBK;
                const Quad z = normal_quad(seed_lo, seed_hi, (uint64_t)(j0 + jl), (uint32_t)q, cgen);
#pragma unroll
                for (int e = 0; e < 4; ++e) ldsA[kg][buf][4 * q + e][jl] = z.z[e];
            }
        }
    };

    f32x4 acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};

    // A workgroup that owns its rows outright fetches the old state now, so that the read is
    // long finished when the epilogue needs it (clamped addresses; unused lanes read row n-1).
    float old[MT][NT][4];
    const bool direct = it.nparts <= 1;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int k = (nt * 16 + li < R) ? nt * 16 + li : R - 1;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                long long row = (long long)it.row0 + wave * (MT * 16) + mt * 16 + 4 * g + v;
                if (row > n - 1) row = n - 1;
                old[mt][nt][v] = (direct && kg == 0 && a != 0.f) ? ldg(state + row * R + k) : 0.f;
            }
        }

    auto mfma_tile = [&](v4f (&gt)[MT][4], int buf, bool settle) {
        if (settle) settle_tile(gt);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            v4f bv[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                bv[nt] = *reinterpret_cast<const v4f*>(&ldsA[kg][buf][nt * 16 + li][16 * c + 4 * g]);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        const float x = gt[mt][c][t];
                        acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(MAP == 1 ? x * x : x, bv[nt][t],
                                                                           acc[mt][nt], 0, 0, 0);
                    }
        }
    };

    // G tiles are fetched kPF - 1 rounds ahead of their use: a wave's progress is then bound
    // by the matrix cores and the generator, not by one HBM round trip per tile.  The
    // prefetch is unconditional (out-of-range rounds read zeros for free), which lets the
    // compiler wait only for the stage it is about to consume.
    if (fast_rounds > 0) {
        v4f st[kPF][MT][4];
#pragma unroll
        for (int u = 0; u < kPF - 1; ++u) load_tile_fast(st[u], u);
        gen_tile(0, 0);
        __syncthreads();
        // The body is free of branches around memory operations (a round past the end loads
        // nothing, multiplies zeros and skips only the generator): the compiler can then
        // follow the outstanding loads around the loop and waits for the oldest stage alone.
        for (int base = 0; base < fast_rounds; base += kPF) {
#pragma unroll
            for (int u = 0; u < kPF; ++u) {
                const int i = base + u;
                const int buf = i & 1;
                load_tile_fast(st[(u + kPF - 1) % kPF], i + kPF - 1);
                if (i + 1 < fast_rounds) gen_tile(buf ^ 1, i + 1);
                mfma_tile(st[u], buf, true);
                __syncthreads();
            }
        }
    }
    for (int i = fast_rounds; i < iters; ++i) {
        const int tile = kg + KG * i;
        const bool active = tile < ntiles;
        v4f gt[MT][4];
        if (active) {
            const long long j0 = (long long)(tbase + tile) * kBK;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int c = 0; c < 4; ++c) gt[mt][c] = load4(rowp[mt], j0 + 16 * c + 4 * g, col_end, false);
            gen_tile(0, i);
        }
        __syncthreads();
        if (active) mfma_tile(gt, 0, false);
        __syncthreads();
    }

    // D layout of the 16x16 tile: lane holds column lane % 16, rows 4 * (lane / 16) + v.
    // Column groups 1 .. KG-1 hand their partial sums to group 0 through LDS; group 0 adds
    // them in a fixed order, so the result does not depend on timing.
    if (KG > 1) {
        if (kg > 0) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        ldsRed[kg - 1][wave * (MT * 16) + mt * 16 + 4 * g + v][nt * 16 + li] = acc[mt][nt][v];
        }
        __syncthreads();
        if (kg > 0) return;
#pragma unroll
        for (int k2 = 0; k2 < KG - 1; ++k2)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        acc[mt][nt][v] += ldsRed[k2][wave * (MT * 16) + mt * 16 + 4 * g + v][nt * 16 + li];
    }

    if (it.nparts > 1) {
        // The columns of this row block are shared between nparts workgroups (short launches:
        // equal pieces of work spread over the chip).  Each stores its partial product with
        // device scope on the stores themselves; the last to arrive adds the partials in the
        // order 0 .. nparts - 1, whoever it is, and updates the state: no float atomics, the
        // result does not depend on timing.
        __shared__ uint32_t lds_flag;
        float* pb = partials + (size_t)it.poff + (size_t)it.part * (ROWS * RP);
        const rsrc_t prs_w = make_rsrc(pb, (long long)ROWS * RP * 4);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const uint32_t row = (uint32_t)(wave * (MT * 16) + mt * 16 + 4 * g + v);
                    const float val = acc[mt][nt][v];
                    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(val), prs_w,
                                                          (int)((row * RP + nt * 16 + li) * 4u), 0, 16);
                }
        __builtin_amdgcn_s_waitcnt(0x0070);   // vmcnt(0): this thread's partial stores have completed
        __syncthreads();                      // (only column group 0 is left: 256 threads)
        if (tg == 0) lds_flag = atomicAdd(counters + it.cidx, 1u);
        __syncthreads();
        if (lds_flag != (uint32_t)(it.nparts - 1)) return;
        const rsrc_t prs = make_rsrc(partials + (size_t)it.poff, (long long)it.nparts * ROWS * RP * 4);
        long long rows_here = n - it.row0;
        rows_here = rows_here > it.rows ? it.rows : rows_here;
        // Four entries per thread and four parts at a time are fetched before any is added, so
        // the combine costs a few memory round trips, not one per part and entry; a part or an
        // entry that does not exist is pointed out of range and adds an exact zero.  The order
        // of the additions stays 0 .. nparts - 1.
        const int total = (int)rows_here * R;
        const rsrc_t srs = make_rsrc(state + (long long)it.row0 * R, (long long)total * 4);
        for (int f0 = tg; f0 < total; f0 += 4 * 256) {
            uint32_t poff4[4], soff[4];
            float oldv[4], sum[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int f = f0 + 256 * u;
                const bool ok = f < total;
                poff4[u] = ok ? ((uint32_t)(f / R) * RP + (uint32_t)(f % R)) * 4u : kOob;
                soff[u] = ok ? (uint32_t)f * 4u : kOob;
                oldv[u] = (a != 0.f) ? buf_load_f(srs, soff[u]) : 0.f;
                sum[u] = 0.f;
            }
            for (int q0 = 0; q0 < it.nparts; q0 += 4) {
                float pv[4][4];
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const bool ok = q0 + j < it.nparts && poff4[u] != kOob;
                        const uint32_t off = ok ? (uint32_t)(q0 + j) * (uint32_t)(ROWS * RP * 4) + poff4[u] : kOob;
                        pv[j][u] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(prs, (int)off, 0, 16));
                    }
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int u = 0; u < 4; ++u) sum[u] += pv[j][u];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) buf_store_f(srs, soff[u], a * oldv[u] + b * sum[u]);
        }
        if (tg == 0) counters[it.cidx] = 0u;   // every part has arrived: ready for the next launch
        return;
    }

#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int k = nt * 16 + li;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const long long row = (long long)it.row0 + wave * (MT * 16) + mt * 16 + 4 * g + v;
                if (row < n && k < R) stg(state + row * R + k, a * old[mt][nt][v] + b * acc[mt][nt][v]);
            }
        }
}

template <int R, typename GT, int MT, int MAP>
hipError_t launch_mt(const MatDev* mats, const WorkItem* items, int nitems, const SeedArgs& seeds,
                     float a, float b, int kgroups, float* partials, uint32_t* counters, hipStream_t s)
{
    const dim3 grid((unsigned)nitems);
    switch (kgroups) {
    case 1: hipLaunchKernelGGL((compress_f32_kernel<R, GT, MT, 1, MAP>), grid, dim3(256), 0, s, mats, items, seeds, a, b, partials, counters); break;
    case 2: hipLaunchKernelGGL((compress_f32_kernel<R, GT, MT, 2, MAP>), grid, dim3(512), 0, s, mats, items, seeds, a, b, partials, counters); break;
    case 4: hipLaunchKernelGGL((compress_f32_kernel<R, GT, MT, 4, MAP>), grid, dim3(1024), 0, s, mats, items, seeds, a, b, partials, counters); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <int R, typename GT>
hipError_t launch_one(const MatDev* mats, const WorkItem* items, int nitems, const SeedArgs& seeds, int map,
                      float a, float b, int kgroups, int mt, float* partials, uint32_t* counters, hipStream_t s)
{
    if (map == 0) {
        if (mt == 1) return launch_mt<R, GT, 1, 0>(mats, items, nitems, seeds, a, b, kgroups, partials, counters, s);
        if (mt == 2) return launch_mt<R, GT, 2, 0>(mats, items, nitems, seeds, a, b, kgroups, partials, counters, s);
    } else if (map == 1) {
        if (mt == 1) return launch_mt<R, GT, 1, 1>(mats, items, nitems, seeds, a, b, kgroups, partials, counters, s);
        if (mt == 2) return launch_mt<R, GT, 2, 1>(mats, items, nitems, seeds, a, b, kgroups, partials, counters, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_compress_f32(const MatDev* mats, const WorkItem* items, int nitems, const SeedArgs& seeds,
                               int r, int grad_is_bf16, int map, float a, float b, int kgroups, int mt,
                               float* partials, uint32_t* counters, hipStream_t s)
{
    if (nitems == 0) return hipSuccess;
    if (!grad_is_bf16) {
        if (r == 8) return launch_one<8, float>(mats, items, nitems, seeds, map, a, b, kgroups, mt, partials, counters, s);
        if (r == 16) return launch_one<16, float>(mats, items, nitems, seeds, map, a, b, kgroups, mt, partials, counters, s);
        if (r == 32) return launch_one<32, float>(mats, items, nitems, seeds, map, a, b, kgroups, mt, partials, counters, s);
    } else {
        if (r == 8) return launch_one<8, uint16_t>(mats, items, nitems, seeds, map, a, b, kgroups, mt, partials, counters, s);
        if (r == 16) return launch_one<16, uint16_t>(mats, items, nitems, seeds, map, a, b, kgroups, mt, partials, counters, s);
        if (r == 32) return launch_one<32, uint16_t>(mats, items, nitems, seeds, map, a, b, kgroups, mt, partials, counters, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace flora
