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
    epilogue_fetch<MODE, OT>(pre_cur, M, p, it.row0, row_end, j, jok);
    stash(stage, 0);
    __syncthreads();

    int buf = 0;
    for (long long rb = it.row0; rb < row_end; rb += 32) {
        const bool more = rb + 32 < row_end;
        if (more) {
            fetch(stage, rb + 32);
            epilogue_fetch<MODE, OT>(pre_nxt, M, p, rb + 32, row_end, j, jok);
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

// ---------------------------------------------------------------------------
// Vector variant for rows of W that start on 16-byte boundaries (m % 4 == 0):
// the product is taken transposed, Gt^T = A state^T, on
// v_mfma_f32_16x16x32_bf16, so that the accumulator of a 16 x 16 tile holds, per
// lane, four consecutive columns of one row of W (lane % 16 = row, lane / 16 =
// group of four columns); a round trip through a staging tile in LDS that belongs
// to the wave alone then puts eight lanes along each row, and W is read and
// written 16 bytes per lane, 8 rows x 128 contiguous bytes (whole cache lines) per
// instruction.
//
// One workgroup (8 waves) owns 256 columns and a block of rows; a wave owns 32
// columns (two 16-wide tiles).  (The state block a workgroup fetches per 32 rows
// is r * 128 bytes whatever its width; at r = 256 that is as much as the old and
// new weights of 128 columns together, so the wider the workgroup the smaller
// the state's share of the load path.)  Lane (column jj = lane % 16, quarter g = lane / 16)
// regenerates A[j, 32 s + 8 g .. +7] for every step s < r / 32, both tiles, once
// (r / 8 Philox calls), straight into the A operand registers, and keeps them
// while the workgroup walks down the rows 32 at a time.  The 32 x r block of the
// state is converted to bf16 once per workgroup and shared through LDS (double
// buffered).  The old weights of the next two blocks are in flight while the
// current block multiplies.
template <int MODE>
struct VecPre {
    v4f w[(MODE == kModeSgd || MODE == kModeFactored || MODE == kModeFull2) ? 4 : 1];   // rows lane / 8 + 8 p, p < 4
    v4f v[(MODE == kModeFull1 || MODE == kModeFull2) ? 4 : 1];    // unfactored second moment, same rows
    // row statistics: of those four rows (kModeFactored), or of rows li and 16 + li (kModeRms,
    // which works on the accumulator layout)
    float rs[MODE == kModeFactored ? 4 : (MODE == kModeRms ? 2 : 1)];
};

template <int R, int MODE, typename OT>
__global__ __launch_bounds__(512) void decompress_bf16_vec_kernel(const MatDev* __restrict__ mats,
                                                                  const WorkItem* __restrict__ items,
                                                                  const SeedArgs seeds, DecompressParams p)
{
    constexpr int S = R / 32;          // MFMA steps along the rank axis
    constexpr int LDS_ROW = R + 8;     // padded row (bf16 elements)
    constexpr int F4 = R / 64;         // float4 loads per thread for one 32 x R block
    constexpr int TROW = 36;           // padded row of a wave's 32 x 32 staging tile (floats)
    constexpr bool kUsesW = (MODE == kModeSgd || MODE == kModeFactored || MODE == kModeFull2);
    constexpr bool kUsesV = (MODE == kModeFull1 || MODE == kModeFull2);
    // passes that end with one partial sum per workgroup (of U^2, or of the new W^2)
    constexpr bool kTotals = (MODE == kModeRms || MODE == kModeFactored || MODE == kModeFull1 || MODE == kModeFull2);
    // the two reduction passes move no weights: they work on the accumulators where they are
    constexpr bool kReduce = (MODE == kModeStats || MODE == kModeRms);
    __shared__ __attribute__((aligned(16))) uint16_t ldsS[2][32][LDS_ROW];
    __shared__ __attribute__((aligned(16))) float ldsT[kReduce ? 1 : 8][kReduce ? 1 : 32][TROW];
    __shared__ float lds_row[2][8][32];   // kModeStats: per-wave row sums of a block, double buffered
    __shared__ float lds_fin[8];

    const WorkItem it = items[blockIdx.x];
    const MatDev& M = mats[it.mat];
    const long long n = M.n, m = M.m;
    const float* __restrict__ state = M.state;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15, g = lane >> 4;
    const int er = lane >> 3, ec = lane & 7;     // epilogue: row er + 8 p, columns 4 ec .. 4 ec + 3
    const float cgen = neg2_ln2_over(R);
    const uint32_t seed_lo = seeds.s[it.mat].x, seed_hi = seeds.s[it.mat].y;
    const long long row_end = ((long long)it.row0 + it.rows < n) ? (long long)it.row0 + it.rows : n;

    // A operand: this lane's column of each tile, r / 4 entries per tile
    bf16x8 areg[2][S];
#pragma unroll
    for (int jt = 0; jt < 2; ++jt) {
        long long j = (long long)it.col0 + 32 * wave + 16 * jt + li;
        if (j > m - 1) j = m - 1;      // clamped: columns past m are never stored
#pragma unroll
        for (int s = 0; s < S; ++s) {
            const Quad z0 = normal_quad(seed_lo, seed_hi, (uint64_t)j, (uint32_t)(8 * s + 2 * g), cgen);
            const Quad z1 = normal_quad(seed_lo, seed_hi, (uint64_t)j, (uint32_t)(8 * s + 2 * g + 1), cgen);
            const uint4 pk = make_uint4(pack_bf16x2(z0.z[0], z0.z[1]), pack_bf16x2(z0.z[2], z0.z[3]),
                                        pack_bf16x2(z1.z[0], z1.z[1]), pack_bf16x2(z1.z[2], z1.z[3]));
            areg[jt][s] = __builtin_bit_cast(bf16x8, pk);
        }
    }

    // The accumulator of a 16 x 16 tile holds, per lane, four consecutive columns of one row;
    // the wave's 32 x 32 block then goes through its own staging tile in LDS and comes back
    // with eight lanes along each row: lane (er, ec) holds columns 4 ec .. 4 ec + 3 of rows
    // er + 8 p.  A row of the block is one 128-byte line of W, so every load and store
    // instruction moves whole lines (8 rows x 128 bytes), the cheapest pattern for the
    // texture path.  m % 4 == 0: the four columns are all in or all out.
    const uint32_t c0 = (uint32_t)it.col0 + 32u * wave + 4u * ec;
    const bool cok = c0 < (uint32_t)m;

    // the same for the accumulator layout (reduction passes): columns d0[jt] .. d0[jt] + 3
    uint32_t d0[2];
    bool dok[2];
#pragma unroll
    for (int jt = 0; jt < 2; ++jt) {
        d0[jt] = (uint32_t)it.col0 + 32u * wave + 16u * jt + 4u * g;
        dok[jt] = d0[jt] < (uint32_t)m;
    }

    // per-column factors (kModeRms / kModeFactored) and running column sums (kModeStats)
    float kfac[4], colsum[4];          // row-contiguous layout
    float kfacd[2][4], colsumd[2][4];  // accumulator layout
    float total = 0.f;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        kfac[v] = 0.f;
        colsum[v] = 0.f;
        kfacd[0][v] = kfacd[1][v] = 0.f;
        colsumd[0][v] = colsumd[1][v] = 0.f;
    }
    if (MODE == kModeFactored) {
        const float meanR = ldg(M.scal), clip = ldg(M.scal + 1), ps = ldg(M.scal + 2);
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            if (!cok) continue;
            // U = Gt / sqrt(R_i K_j / mean R), scaled by lr, the RMS clip factor and the
            // parameter scale (max(eps2, RMS(W)), or 1)
            kfac[v] = p.coef * p.alpha * clip * ps * sqrtf(meanR) * rsqrtf(ldg(M.col_stat + c0 + v));
        }
    }
    // kModeFull2: U = Gt / sqrt(V_ij), scaled the same way
    const float kfull = (MODE == kModeFull2) ? p.coef * p.alpha * ldg(M.scal + 1) * ldg(M.scal + 2) : 0.f;
    if (MODE == kModeRms) {
        const float meanR = ldg(M.scal);
#pragma unroll
        for (int jt = 0; jt < 2; ++jt)
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (dok[jt]) kfacd[jt][v] = p.alpha * p.alpha * meanR / ldg(M.col_stat + d0[jt] + v);
    }

    // cooperative fetch of a 32 x R block of the state: float4 number f = tid + 512 i
    // covers row f / (R/4), columns 4 (f % (R/4)) .. +3.  The buffer resource covers exactly
    // this workgroup's rows: rows past them read as zero, so Gt is zero there and neither the
    // statistics nor the stores need a row mask (32-bit offsets: rows * R * 4 < 2^31).
    const rsrc_t srs = make_rsrc(state + (long long)it.row0 * R, (row_end - it.row0) * (long long)R * 4);
    uint32_t soff[F4];
#pragma unroll
    for (int i = 0; i < F4; ++i) {
        const int f = tid + 512 * i;
        soff[i] = ((uint32_t)(f / (R / 4)) * R + 4u * (uint32_t)(f % (R / 4))) * 4u;
    }
    auto fetch = [&](v4f (&dst)[F4], long long rb) {
        const uint32_t boff = (uint32_t)(rb - it.row0) * (uint32_t)(R * 4);
#pragma unroll
        for (int i = 0; i < F4; ++i) dst[i] = buf_load_f4(srs, boff + soff[i]);
    };
    auto stash = [&](const v4f (&src)[F4], int buf) {
#pragma unroll
        for (int i = 0; i < F4; ++i) {
            const int f = tid + 512 * i;
            const uint2 pk = make_uint2(pack_bf16x2(src[i].x, src[i].y), pack_bf16x2(src[i].z, src[i].w));
            *reinterpret_cast<uint2*>(&ldsS[buf][f / (R / 4)][4 * (f % (R / 4))]) = pk;
        }
    };

    // Old weights / row statistics of the block that starts at row rb.  The buffer resource
    // covers exactly the block's valid rows: rows past the end read as zero and their
    // stores are dropped; lane offsets stay below 32 m * 4 <= 2^31.
    auto wrsrc = [&](long long rb) -> rsrc_t {
        long long rows = row_end - rb;
        rows = rows < 0 ? 0 : (rows > 32 ? 32 : rows);
        const long long base = rb < n ? rb : 0;
        if (MODE == kModeOut) return make_rsrc(reinterpret_cast<OT*>(M.out) + base * m, rows * m * (long long)sizeof(OT));
        return make_rsrc(reinterpret_cast<OT*>(M.weight) + base * m, rows * m * (long long)sizeof(OT));
    };
    // four consecutive elements of W (fp32: 16 bytes, bf16: 8 bytes per lane); the store returns
    // the values as stored
    // Cache policy of the n x m arrays this launch reads and writes once (weights, elementwise
    // second moment), chosen by the host from their size: a set that fits the last-level cache
    // stays there for the next step (plain accesses); a larger one is written, and a much larger
    // one also read, with the non-temporal hint so that it does not push out what is reused.
    const bool ld_stream = (p.wpolicy & 1) != 0, st_stream = (p.wpolicy & 2) != 0;
    auto load_w4 = [&](rsrc_t rw, uint32_t off) -> v4f {
        if (sizeof(OT) == 4) return ld_stream ? buf_load_f4<true>(rw, off) : buf_load_f4<false>(rw, off);
        const v2u pk = ld_stream ? buf_load_u2<true>(rw, off) : buf_load_u2<false>(rw, off);
        return v4f{bf16_bits_to_f32(pk.x & 0xffffu), bf16_bits_to_f32(pk.x >> 16),
                   bf16_bits_to_f32(pk.y & 0xffffu), bf16_bits_to_f32(pk.y >> 16)};
    };
    auto store_w4 = [&](rsrc_t rw, uint32_t off, v4f v) -> v4f {
        if (sizeof(OT) == 4) {
            if (st_stream) buf_store_f4<true>(rw, off, v);
            else buf_store_f4<false>(rw, off, v);
            return v;
        }
        const v2u pk = {pack_bf16x2(v.x, v.y), pack_bf16x2(v.z, v.w)};
        if (st_stream) buf_store_u2<true>(rw, off, pk);
        else buf_store_u2<false>(rw, off, pk);
        return v4f{bf16_bits_to_f32(pk.x & 0xffffu), bf16_bits_to_f32(pk.x >> 16),
                   bf16_bits_to_f32(pk.y & 0xffffu), bf16_bits_to_f32(pk.y >> 16)};
    };
    auto vrsrc = [&](long long rb) -> rsrc_t {
        long long rows = row_end - rb;
        rows = rows < 0 ? 0 : (rows > 32 ? 32 : rows);
        const long long base = rb < n ? rb : 0;
        return make_rsrc(M.vfull + base * m, rows * m * 4);
    };
    auto woff = [&](int pp) -> uint32_t {
        return cok ? ((uint32_t)(er + 8 * pp) * (uint32_t)m + c0) * (uint32_t)sizeof(OT) : kOob;
    };
    auto voff = [&](int pp) -> uint32_t {     // the second moment is always fp32
        return cok ? ((uint32_t)(er + 8 * pp) * (uint32_t)m + c0) * 4u : kOob;
    };
    auto pre_fetch = [&](VecPre<MODE>& pre, long long rb) {
        if (kUsesW) {
            const rsrc_t rw = wrsrc(rb);
#pragma unroll
            for (int pp = 0; pp < 4; ++pp) pre.w[pp] = load_w4(rw, woff(pp));
        }
        if (kUsesV) {
            const rsrc_t rv = vrsrc(rb);
#pragma unroll
            for (int pp = 0; pp < 4; ++pp) pre.v[pp] = ld_stream ? buf_load_f4<true>(rv, voff(pp)) : buf_load_f4<false>(rv, voff(pp));
        }
        if (MODE == kModeFactored) {
#pragma unroll
            for (int pp = 0; pp < 4; ++pp) {
                long long row = rb + er + 8 * pp;
                if (row > n - 1) row = n - 1;
                pre.rs[pp] = ldg(M.row_stat + row);
            }
        }
        if (MODE == kModeRms) {
#pragma unroll
            for (int itile = 0; itile < 2; ++itile) {
                long long row = rb + 16 * itile + li;
                if (row > n - 1) row = n - 1;
                pre.rs[itile] = ldg(M.row_stat + row);
            }
        }
    };

    v4f stage[F4];
    VecPre<MODE> pre0, pre1, pre2;     // blocks rb, rb + 32, rb + 64
    fetch(stage, it.row0);
    pre_fetch(pre0, it.row0);
    pre_fetch(pre1, (long long)it.row0 + 32);
    stash(stage, 0);
    __syncthreads();

    int buf = 0;
    for (long long rb = it.row0; rb < row_end; rb += 32) {
        const bool more = rb + 32 < row_end;
        if (more) fetch(stage, rb + 32);
        pre_fetch(pre2, rb + 64);      // past the end: empty resource, nothing is fetched

        f32x4 acc[2][2];               // [i-tile][j-tile]
#pragma unroll
        for (int itile = 0; itile < 2; ++itile)
#pragma unroll
            for (int jt = 0; jt < 2; ++jt) acc[itile][jt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < S; ++s) {
#pragma unroll
            for (int itile = 0; itile < 2; ++itile) {
                const bf16x8 bv = *reinterpret_cast<const bf16x8*>(&ldsS[buf][16 * itile + li][32 * s + 8 * g]);
#pragma unroll
                for (int jt = 0; jt < 2; ++jt)
                    acc[itile][jt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(areg[jt][s], bv, acc[itile][jt], 0, 0, 0);
            }
        }

        // ---- accumulators -> row-contiguous layout through this wave's staging tile
        // (acc[itile][jt][v] = (state A^T)[rb + 16 itile + li, 32 wave + 16 jt + 4 g + v])
        v4f gt[4];                     // gt[pp] = (state A^T)[rb + er + 8 pp, c0 .. c0 + 3]
        if (!kReduce) {
#pragma unroll
            for (int itile = 0; itile < 2; ++itile)
#pragma unroll
                for (int jt = 0; jt < 2; ++jt)
                    *reinterpret_cast<f32x4*>(&ldsT[wave][16 * itile + li][16 * jt + 4 * g]) = acc[itile][jt];
#pragma unroll
            for (int pp = 0; pp < 4; ++pp) gt[pp] = *reinterpret_cast<const v4f*>(&ldsT[wave][er + 8 * pp][4 * ec]);
        }

        if (MODE == kModeOut) {
            const rsrc_t rw = wrsrc(rb);
#pragma unroll
            for (int pp = 0; pp < 4; ++pp) {
                const v4f a4 = gt[pp];
                if (sizeof(OT) == 4) {
                    buf_store_f4(rw, woff(pp), v4f{p.alpha * a4.x, p.alpha * a4.y, p.alpha * a4.z, p.alpha * a4.w});
                } else {
                    const v2u pk = {pack_bf16x2(p.alpha * a4.x, p.alpha * a4.y), pack_bf16x2(p.alpha * a4.z, p.alpha * a4.w)};
                    buf_store_u2(rw, woff(pp), pk);
                }
            }
        } else if (MODE == kModeSgd) {
            const rsrc_t rw = wrsrc(rb);
#pragma unroll
            for (int pp = 0; pp < 4; ++pp) {
                const v4f a4 = gt[pp], w = pre0.w[pp];
                store_w4(rw, woff(pp), v4f{w.x - p.coef * a4.x, w.y - p.coef * a4.y,
                                           w.z - p.coef * a4.z, w.w - p.coef * a4.w});
            }
        } else if (MODE == kModeFactored) {
            const rsrc_t rw = wrsrc(rb);
#pragma unroll
            for (int pp = 0; pp < 4; ++pp) {
                const float ri = rsqrtf(pre0.rs[pp]);
                const v4f a4 = gt[pp], w = pre0.w[pp];
                const v4f wn = store_w4(rw, woff(pp), v4f{w.x - kfac[0] * ri * a4.x, w.y - kfac[1] * ri * a4.y,
                                                          w.z - kfac[2] * ri * a4.z, w.w - kfac[3] * ri * a4.w});
                // sum of the new W^2 (rows past the end and columns past m contribute exact zeros:
                // their old weights read as zero and their factors are zero)
                total = __builtin_fmaf(wn.x, wn.x, total);
                total = __builtin_fmaf(wn.y, wn.y, total);
                total = __builtin_fmaf(wn.z, wn.z, total);
                total = __builtin_fmaf(wn.w, wn.w, total);
            }
        } else if (MODE == kModeFull1) {
            // V <- beta2 V + (1 - beta2) (Gt^2 + eps1) and the sum of U^2 = Gt^2 / V.  Stores out
            // of range are dropped by the resource; their terms of the sum are masked (V reads
            // as zero there).
            const rsrc_t rv = vrsrc(rb);
            const float a2 = p.alpha * p.alpha, omb = 1.f - p.beta2;
#pragma unroll
            for (int pp = 0; pp < 4; ++pp) {
                const bool ok = cok && (rb + er + 8 * pp < row_end);
                const v4f a4 = gt[pp], v = pre0.v[pp];
                const v4f g2 = {a2 * a4.x * a4.x, a2 * a4.y * a4.y, a2 * a4.z * a4.z, a2 * a4.w * a4.w};
                const v4f vn = {p.beta2 * v.x + omb * (g2.x + p.eps1), p.beta2 * v.y + omb * (g2.y + p.eps1),
                                p.beta2 * v.z + omb * (g2.z + p.eps1), p.beta2 * v.w + omb * (g2.w + p.eps1)};
                if (st_stream) buf_store_f4<true>(rv, voff(pp), vn);
                else buf_store_f4<false>(rv, voff(pp), vn);
                const float u2 = ((g2.x / vn.x + g2.y / vn.y) + (g2.z / vn.z + g2.w / vn.w));
                total += ok ? u2 : 0.f;
            }
        } else if (MODE == kModeFull2) {
            const rsrc_t rw = wrsrc(rb);
#pragma unroll
            for (int pp = 0; pp < 4; ++pp) {
                const bool ok = cok && (rb + er + 8 * pp < row_end);
                const v4f a4 = gt[pp], w = pre0.w[pp], v = pre0.v[pp];
                const v4f wn = store_w4(rw, woff(pp), v4f{w.x - kfull * rsqrtf(v.x) * a4.x, w.y - kfull * rsqrtf(v.y) * a4.y,
                                                          w.z - kfull * rsqrtf(v.z) * a4.z, w.w - kfull * rsqrtf(v.w) * a4.w});
                const float w2 = ((wn.x * wn.x + wn.y * wn.y) + (wn.z * wn.z + wn.w * wn.w));
                total += ok ? w2 : 0.f;
            }
        } else if (MODE == kModeStats) {
            // squares of state A^T (alpha^2 is applied to the sums at the end): column sums
            // stay in registers for the whole sweep; row sums go over the four column groups
            // of the wave, then over the eight waves through LDS (fixed order).  Rows past the
            // end are zero already; columns past m (their A is a clamped copy) are masked.
#pragma unroll
            for (int itile = 0; itile < 2; ++itile) {
                float rsum = 0.f;
#pragma unroll
                for (int jt = 0; jt < 2; ++jt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const float x = dok[jt] ? acc[itile][jt][v] : 0.f;
                        colsumd[jt][v] = __builtin_fmaf(x, x, colsumd[jt][v]);
                        rsum = __builtin_fmaf(x, x, rsum);
                    }
                rsum += __shfl_xor(rsum, 16);
                rsum += __shfl_xor(rsum, 32);
                if (g == 0) lds_row[buf][wave][16 * itile + li] = p.alpha * p.alpha * rsum;
            }
        } else if (MODE == kModeRms) {
            // sum of U^2 = Gt^2 mean(R) / (R_i K_j): per row the K-weighted sum first, then 1 / R_i
            // (rows past the end are zero; kfacd is zero for columns past m)
#pragma unroll
            for (int itile = 0; itile < 2; ++itile) {
                float t = 0.f;
#pragma unroll
                for (int jt = 0; jt < 2; ++jt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) t = __builtin_fmaf(acc[itile][jt][v] * acc[itile][jt][v], kfacd[jt][v], t);
                total = __builtin_fmaf(t, 1.f / pre0.rs[itile], total);
            }
        }

        if (more) stash(stage, buf ^ 1);
        pre0 = pre1;
        pre1 = pre2;
        __syncthreads();
        if (MODE == kModeStats && tid < 32) {
            // the eight waves' row sums of the block just finished (written before the barrier;
            // the buffer is not written again before the next barrier)
            const long long row = rb + tid;
            if (row < row_end)
                stg(M.rowpart + (long long)it.slice * n + row,
                    (((lds_row[buf][0][tid] + lds_row[buf][1][tid]) + (lds_row[buf][2][tid] + lds_row[buf][3][tid])) +
                     ((lds_row[buf][4][tid] + lds_row[buf][5][tid]) + (lds_row[buf][6][tid] + lds_row[buf][7][tid]))));
        }
        buf ^= 1;
    }

    if (MODE == kModeStats) {
        // column sums over the 16 row-lanes that share a column group, then one store per column
#pragma unroll
        for (int jt = 0; jt < 2; ++jt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                float c = colsumd[jt][v];
                c += __shfl_xor(c, 8);
                c += __shfl_xor(c, 4);
                c += __shfl_xor(c, 2);
                c += __shfl_xor(c, 1);
                if (li == 0 && dok[jt]) stg(M.colpart + (long long)it.rblock * m + d0[jt] + v, p.alpha * p.alpha * c);
            }
    }
    if (kTotals) {
        float t = total;
        t += __shfl_xor(t, 32);
        t += __shfl_xor(t, 16);
        t += __shfl_xor(t, 8);
        t += __shfl_xor(t, 4);
        t += __shfl_xor(t, 2);
        t += __shfl_xor(t, 1);
        if (lane == 0) lds_fin[wave] = t;
        __syncthreads();
        if (tid == 0)
            M.itempart[it.part] = ((lds_fin[0] + lds_fin[1]) + (lds_fin[2] + lds_fin[3])) +
                                  ((lds_fin[4] + lds_fin[5]) + (lds_fin[6] + lds_fin[7]));
    }
}

template <int R, typename OT>
hipError_t launch_mode_vec(const MatDev* mats, const WorkItem* items, int nitems, const SeedArgs& seeds,
                           int mode, DecompressParams p, hipStream_t s)
{
    const dim3 grid((unsigned)nitems), block(512);
    switch (mode) {
    case kModeOut:
        hipLaunchKernelGGL((decompress_bf16_vec_kernel<R, kModeOut, OT>), grid, block, 0, s, mats, items, seeds, p);
        break;
    case kModeSgd:
        hipLaunchKernelGGL((decompress_bf16_vec_kernel<R, kModeSgd, OT>), grid, block, 0, s, mats, items, seeds, p);
        break;
    case kModeStats:
        hipLaunchKernelGGL((decompress_bf16_vec_kernel<R, kModeStats, float>), grid, block, 0, s, mats, items, seeds, p);
        break;
    case kModeRms:
        hipLaunchKernelGGL((decompress_bf16_vec_kernel<R, kModeRms, float>), grid, block, 0, s, mats, items, seeds, p);
        break;
    case kModeFactored:
        hipLaunchKernelGGL((decompress_bf16_vec_kernel<R, kModeFactored, OT>), grid, block, 0, s, mats, items, seeds, p);
        break;
    case kModeFull1:
        hipLaunchKernelGGL((decompress_bf16_vec_kernel<R, kModeFull1, float>), grid, block, 0, s, mats, items, seeds, p);
        break;
    case kModeFull2:
        hipLaunchKernelGGL((decompress_bf16_vec_kernel<R, kModeFull2, OT>), grid, block, 0, s, mats, items, seeds, p);
        break;
    default:
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
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
        hipLaunchKernelGGL((decompress_bf16_kernel<R, kModeSgd, OT>), grid, block, 0, s, mats, items, seeds, p);
        break;
    case kModeStats:
        hipLaunchKernelGGL((decompress_bf16_kernel<R, kModeStats, float>), grid, block, 0, s, mats, items, seeds, p);
        break;
    case kModeRms:
        hipLaunchKernelGGL((decompress_bf16_kernel<R, kModeRms, float>), grid, block, 0, s, mats, items, seeds, p);
        break;
    case kModeFactored:
        hipLaunchKernelGGL((decompress_bf16_kernel<R, kModeFactored, OT>), grid, block, 0, s, mats, items, seeds, p);
        break;
    case kModeFull1:
        hipLaunchKernelGGL((decompress_bf16_kernel<R, kModeFull1, float>), grid, block, 0, s, mats, items, seeds, p);
        break;
    case kModeFull2:
        hipLaunchKernelGGL((decompress_bf16_kernel<R, kModeFull2, OT>), grid, block, 0, s, mats, items, seeds, p);
        break;
    default:
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <int R>
hipError_t launch_r(const MatDev* mats, const WorkItem* items, int nitems, const SeedArgs& seeds, int mode,
                    int out_is_bf16, int vec, DecompressParams p, hipStream_t s)
{
    // modes that read or write the n x m array whose element type the caller chose (out, or W)
    const bool typed = mode == kModeOut || mode == kModeSgd || mode == kModeFactored || mode == kModeFull2;
    if (vec) {
        if (typed && out_is_bf16) return launch_mode_vec<R, uint16_t>(mats, items, nitems, seeds, mode, p, s);
        return launch_mode_vec<R, float>(mats, items, nitems, seeds, mode, p, s);
    }
    if (typed && out_is_bf16) return launch_mode<R, uint16_t>(mats, items, nitems, seeds, mode, p, s);
    return launch_mode<R, float>(mats, items, nitems, seeds, mode, p, s);
}

}  // namespace

// vec: every matrix of the launch has m % 4 == 0 (rows of W / out start on 16-byte boundaries)
hipError_t launch_decompress_bf16(const MatDev* mats, const WorkItem* items, int nitems, const SeedArgs& seeds,
                                 int r, int mode, int out_is_bf16, int vec, DecompressParams p, hipStream_t s)
{
    if (nitems == 0) return hipSuccess;
    if (r == 64) return launch_r<64>(mats, items, nitems, seeds, mode, out_is_bf16, vec, p, s);
    if (r == 128) return launch_r<128>(mats, items, nitems, seeds, mode, out_is_bf16, vec, p, s);
    if (r == 256) return launch_r<256>(mats, items, nitems, seeds, mode, out_is_bf16, vec, p, s);
    return hipErrorInvalidValue;
}

}  // namespace flora
