// Compression on the bf16 matrix cores, ranks 64 / 128 / 256:
//     state <- a * state + b * (G A(seed))
// (Algorithm 1, compression line; Algorithm 2, EMA line).  A is rounded to
// bf16 as it is generated; products are exact in fp32 and accumulated in fp32
// (v_mfma_f32_32x32x16_bf16).  G is bf16, or fp32 rounded to bf16 (nearest even)
// in registers on its way to the matrix cores (first kernel below only).  Both
// kernels also take the elementwise square of G as their input (MAP = 1: squared in
// fp32, then rounded to bf16), for the compressed EMA of the second moment.
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

// both halves of a packed pair of bf16 squared in fp32 and rounded back
__device__ __forceinline__ uint32_t square_bf16x2(uint32_t w)
{
    const float lo = __uint_as_float(w << 16), hi = __uint_as_float(w & 0xffff0000u);
    return pack_bf16x2(lo * lo, hi * hi);
}

template <int MT, typename GT, int MAP>
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
    const GT* __restrict__ G = reinterpret_cast<const GT*>(M.grad);
    float* __restrict__ state = M.state;
    constexpr bool kF32 = sizeof(GT) == 4;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, g = lane >> 5;
    const float cgen = neg2_ln2_over(R);
    const bool vec_ok = (m % (kF32 ? 4 : 8)) == 0;   // rows start on 16-byte boundaries
    const int ntiles = (int)((m + kBK - 1) / kBK);
    const int nfull = vec_ok ? (int)(m / kBK) : 0;
    const int q0 = it.slice * (kRS / 4);   // first Philox quad of this rank slice

    const GT* rowp[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        long long row = (long long)it.row0 + wave * (MT * 32) + mt * 32 + li;
        if (row > n - 1) row = n - 1;
        rowp[mt] = G + row * m;
    }

    // element c of the row (mapped) as bf16 bits (zero past the end)
    auto elem = [&](const GT* rp, long long c) -> uint32_t {
        if (c >= m) return 0u;
        if constexpr (kF32) {
            const float x = ldg(reinterpret_cast<const float*>(rp) + c);
            return f32_to_bf16_bits(MAP == 1 ? x * x : x);
        } else {
            const uint32_t w = ldg(reinterpret_cast<const uint16_t*>(rp) + c);
            return MAP == 1 ? (square_bf16x2(w) & 0xffffu) : w;
        }
    };

    auto load_tile = [&](v4u (&dst)[MT][2], int tile) {
        const long long j0 = (long long)tile * kBK + 16 * g;
        if (tile < nfull) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                if constexpr (kF32) {
                    const float* rp = reinterpret_cast<const float*>(rowp[mt]) + j0;
                    v4f f0 = ldg4(rp), f1 = ldg4(rp + 4), f2 = ldg4(rp + 8), f3 = ldg4(rp + 12);
                    if (MAP == 1) { f0 = f0 * f0; f1 = f1 * f1; f2 = f2 * f2; f3 = f3 * f3; }
                    dst[mt][0] = v4u{pack_bf16x2(f0.x, f0.y), pack_bf16x2(f0.z, f0.w),
                                     pack_bf16x2(f1.x, f1.y), pack_bf16x2(f1.z, f1.w)};
                    dst[mt][1] = v4u{pack_bf16x2(f2.x, f2.y), pack_bf16x2(f2.z, f2.w),
                                     pack_bf16x2(f3.x, f3.y), pack_bf16x2(f3.z, f3.w)};
                } else {
                    const uint16_t* rp = reinterpret_cast<const uint16_t*>(rowp[mt]) + j0;
                    dst[mt][0] = ldg4(rp);
                    dst[mt][1] = ldg4(rp + 8);
                    if (MAP == 1) {
#pragma unroll
                        for (int h = 0; h < 2; ++h)
                            dst[mt][h] = v4u{square_bf16x2(dst[mt][h].x), square_bf16x2(dst[mt][h].y),
                                             square_bf16x2(dst[mt][h].z), square_bf16x2(dst[mt][h].w)};
                    }
                }
            }
        } else {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                uint32_t w[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const long long c0 = j0 + 2 * e;
                    w[e] = elem(rowp[mt], c0) | (elem(rowp[mt], c0 + 1) << 16);
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
// Wide variant: 8 waves own 512 (or 256, 128) rows x RS rank columns (RS = 128, or 64 at
// r = 64) and sweep m in tiles of 64 columns.  It needs rows of G that start on
// 16-byte boundaries (m % 8 == 0); the kernel above remains for everything else.
//
// What bounds this kernel is, in this order, how fast G reaches the registers
// (it is read once from HBM and r / RS - 1 more times from L2), the vector ALU
// that regenerates A (evaluations = n m r / 512) and the matrix cores.
//   * v_mfma_f32_16x16x32_bf16: its A operand wants lane (row i = lane % 16,
//     quarter g = lane / 16) to hold 8 consecutive bf16 of row i, so one load
//     instruction covers 16 rows x 64 contiguous bytes.  The texture path
//     delivers 16-byte pieces scattered over 32 rows (the 32x32 shapes) at
//     about 11 bytes per clock per compute unit, 64-byte pieces clearly faster.
//   * wave w owns rows 64 w .. 64 w + 63 and all RS columns, so G goes from
//     memory straight into its operand registers and is never shared;
//   * the registers of a tile are refilled with the tile two steps ahead as soon
//     as the MFMAs that read them have been issued (two register sets, loop
//     unrolled by two), so about one and a half tiles are in flight per wave
//     (with one rank slice G is read once and streamed past the caches, and a tile's
//     two halves are then refilled together);
//   * the 64 x RS slice of A is regenerated once per tile by all 512 threads
//     into LDS (bf16, transposed, double buffered); waves 0-3 generate while waves
//     4-7 multiply and the other way round, so that the two waves of a SIMD
//     keep its vector ALU and its matrix core busy at the same time;
//   * at the end each wave turns its accumulator tiles into rows through LDS and
//     updates the state with 16-byte accesses, 512 contiguous bytes per row.
constexpr int kWBK = 64;             // columns of G per tile
constexpr int kWLda = kWBK + 8;      // padded LDS row (bf16 elements): 144 bytes

// per wave: CT 16-wide column tiles (RS = 16 CT), RT 16-row tiles; MAP 1: input squared;
// ONCE: r = RS, a single rank slice, so the launch reads G exactly once
template <int CT, int RT, int MAP, bool ONCE>
__global__ __launch_bounds__(512) void compress_bf16_wide_kernel(const MatDev* __restrict__ mats,
                                                                 const WorkItem* __restrict__ items,
                                                                 const SeedArgs seeds, int R, float a, float b,
                                                                 float* __restrict__ partials,
                                                                 uint32_t* __restrict__ counters)
{
    constexpr int WR = 16 * RT;      // rows of one wave
    constexpr int BR = 8 * WR;       // rows of the workgroup
    constexpr int RS = 16 * CT;      // rank columns of this workgroup
    constexpr int NQ = RS / 32;      // quads per thread and tile when generating
    constexpr int JG = kWBK / NQ;    // threads along j when generating (each takes NQ columns j)
    constexpr int LDE = RS + 4;      // padded row of the epilogue staging (floats)
    constexpr int kABytes = 2 * RS * kWLda * 2;
    constexpr int kEBytes = 8 * 16 * LDE * 4;
    __shared__ uint32_t lds_flag;
    __shared__ __attribute__((aligned(16))) unsigned char lds_raw[kABytes > kEBytes ? kABytes : kEBytes];
    typedef uint16_t (*lds_a_t)[RS][kWLda];
    lds_a_t ldsA = reinterpret_cast<lds_a_t>(lds_raw);

    const WorkItem it = items[blockIdx.x];
    const MatDev& M = mats[it.mat];
    const long long n = M.n, m = M.m;
    const uint32_t seed_lo = seeds.s[it.mat].x, seed_hi = seeds.s[it.mat].y;
    const uint16_t* __restrict__ G = reinterpret_cast<const uint16_t*>(M.grad);
    float* __restrict__ state = M.state;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15, g = lane >> 4;
    const float cgen = neg2_ln2_over(R);
    // this workgroup's share of the columns: tiles [tile0, ntiles)
    const long long col_end = (it.col1 < m) ? (long long)it.col1 : m;
    const int tile0 = it.col0 / kWBK;
    const int ntiles = (int)((col_end + kWBK - 1) / kWBK);
    const uint32_t q0 = (uint32_t)(it.slice * (RS / 4));   // first Philox quad of this rank slice
    const long long row_end = ((long long)it.row0 + it.rows < n) ? (long long)it.row0 + it.rows : n;
    const long long wave_row0 = (long long)it.row0 + wave * WR;

    // One buffer resource for the WR rows of this wave, covering exactly its valid rows:
    // rows past the end and (through kOob) columns past m read as zero.
    long long valid = row_end - wave_row0;
    valid = valid < 0 ? 0 : (valid > WR ? WR : valid);
    const rsrc_t rs = make_rsrc(G + (wave_row0 < n ? wave_row0 : 0) * m, valid * m * 2);
    // Chunk (s, g) of a tile holds columns j0 + 32 s + 8 g .. + 7; m % 8 == 0, so a chunk is
    // all in or all out.  Out-of-range chunks are pointed at kOob and fetch nothing.
    //
    // Two ways of fetching a tile.  By halves (two rank slices): lane (li, g) loads what operand
    // (rt, s) wants from it, row li, chunk (s, g): four lanes and 64 bytes per row and
    // instruction; the registers of half s are refilled as soon as its MFMAs are issued.  By
    // lines (one rank slice): eight rows x 128 bytes per instruction, which the load path moves
    // faster: in load x = 2 rt + h of a tile lane (li, g) takes row 16 rt + 8 h + li % 8, chunk
    // (li / 8, g), which leaves the lanes li < 8 of load 2 rt and the lanes li >= 8 of load
    // 2 rt + 1 holding what operand (rt, s) wants for s = 0 and 1, and the other halves each
    // other's; settle_tile swaps those within each row of 16 lanes (two DPP moves per register
    // pair).  All loads of a tile are then refilled together, which keeps less in flight: with
    // two rank slices, where every byte passes the load path twice, that costs more than the
    // whole lines gain (workload 4: 2.70 against 2.31 ms), with one it wins (workload 3: 54
    // against 64 us).
    constexpr bool kLines = ONCE;
    uint32_t lane_off[2 * RT];
#pragma unroll
    for (int x = 0; x < 2 * RT; ++x)
        lane_off[x] = kLines ? ((uint32_t)(8 * x + (li & 7)) * (uint32_t)m + 8u * (uint32_t)(g + 4 * (li >> 3))) * 2u
                             : ((uint32_t)(16 * (x >> 1) + li) * (uint32_t)m + 8u * (uint32_t)g) * 2u;
    auto load_half = [&](v4u (&dst)[RT][2], int tile, int s) {
        const uint32_t col = (uint32_t)tile * kWBK + 32u * (uint32_t)s + 8u * (uint32_t)g;
        const bool ok = col < (uint32_t)col_end;
        const uint32_t coff = ((uint32_t)tile * kWBK + 32u * (uint32_t)s) * 2u;
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) dst[rt][s] = buf_load_u4<ONCE>(rs, ok ? lane_off[2 * rt] + coff : kOob);
    };
    auto load_tile = [&](v4u (&dst)[RT][2], int tile) {
        if (!kLines) {
            load_half(dst, tile, 0);
            load_half(dst, tile, 1);
            return;
        }
        const uint32_t col = (uint32_t)tile * kWBK + 8u * (uint32_t)(g + 4 * (li >> 3));
        const bool ok = col < (uint32_t)col_end;
        const uint32_t coff = (uint32_t)tile * kWBK * 2u;
#pragma unroll
        for (int x = 0; x < 2 * RT; ++x) dst[x >> 1][x & 1] = buf_load_u4<ONCE>(rs, ok ? lane_off[x] + coff : kOob);
    };
    auto settle_tile = [&](v4u (&t)[RT][2]) {
        if (!kLines) return;
        constexpr int kRor8 = 0x128;          // DPP row_ror:8: lane li of a row of 16 reads lane li ^ 8
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t lo = t[rt][0][c], hi = t[rt][1][c];
                // s = 0: lanes li >= 8 (banks 2, 3) take load 2 rt + 1's lanes li - 8
                t[rt][0][c] = (uint32_t)__builtin_amdgcn_update_dpp((int)lo, (int)hi, kRor8, 0xf, 0xc, false);
                // s = 1: lanes li < 8 (banks 0, 1) take load 2 rt's lanes li + 8
                t[rt][1][c] = (uint32_t)__builtin_amdgcn_update_dpp((int)hi, (int)lo, kRor8, 0xf, 0x3, false);
            }
    };

    // 64 x RS normals per tile = 16 RS quads, NQ per thread: thread p takes quad index
    // q = p / JG for the NQ consecutive columns j = NQ (p % JG) .. + NQ - 1 and writes, for
    // each of the quad's four rank columns, NQ packed bf16 along j.  The quads are evaluated
    // one after the other (a wave gains nothing from interleaving them, and the registers
    // are needed elsewhere); the scheduling barriers keep the compiler from mixing them.
    const int gen_j = NQ * (tid % JG);
    const uint32_t gen_q = (uint32_t)(tid / JG);
    auto gen_tile = [&](int buf, int tile) {
        const uint64_t j = (uint64_t)tile * kWBK + (uint64_t)gen_j;
        uint32_t pk[NQ / 2][4];
#pragma unroll
        for (int e = 0; e < NQ; e += 2) {
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
            if (NQ == 4) *reinterpret_cast<uint2*>(dst) = make_uint2(pk[0][i], pk[NQ / 2 - 1][i]);
            else *reinterpret_cast<uint32_t*>(dst) = pk[0][i];
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    f32x4 acc[RT][CT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) acc[rt][ct] = f32x4{0.f, 0.f, 0.f, 0.f};

    // The tile in `gt` / LDS buffer `buf` goes through the matrix cores, one half (32
    // columns) at a time; the B operand of column tile ct + 1 is fetched from LDS while tile
    // ct multiplies.  As soon as the MFMAs of a half are issued its registers are refilled
    // with the tile two steps ahead.
    auto mfma_tile = [&](v4u (&gt)[RT][2], int buf, int tile) {
        settle_tile(gt);
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            if (MAP == 1) {      // the statistic's term: G squared in fp32, rounded back to bf16
#pragma unroll
                for (int rt = 0; rt < RT; ++rt)
                    gt[rt][s] = v4u{square_bf16x2(gt[rt][s].x), square_bf16x2(gt[rt][s].y),
                                    square_bf16x2(gt[rt][s].z), square_bf16x2(gt[rt][s].w)};
            }
            bf16x8 bv = *reinterpret_cast<const bf16x8*>(&ldsA[buf][li][32 * s + 8 * g]);
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
                bf16x8 bn = bv;
                if (ct + 1 < CT) bn = *reinterpret_cast<const bf16x8*>(&ldsA[buf][16 * (ct + 1) + li][32 * s + 8 * g]);
#pragma unroll
                for (int rt = 0; rt < RT; ++rt)
                    acc[rt][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, gt[rt][s]), bv,
                                                                          acc[rt][ct], 0, 0, 0);
                bv = bn;
            }
            __builtin_amdgcn_sched_barrier(0);
            if (!kLines) load_half(gt, tile + 2, s);
            else if (s == 1) load_tile(gt, tile + 2);
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

    v4u gx[RT][2], gy[RT][2];
    load_tile(gx, tile0);
    load_tile(gy, tile0 + 1);
    gen_tile(0, tile0);
    gen_if(early, 1, tile0 + 1);
    __syncthreads();
    for (int tile = tile0; tile < ntiles; tile += 2) {
        mfma_tile(gx, 0, tile);
        gen_if(!early, 1, tile + 1);
        __syncthreads();
        gen_if(early, 0, tile + 2);
        if (tile + 1 < ntiles) mfma_tile(gy, 1, tile + 1);     // uniform over the workgroup
        gen_if(!early, 0, tile + 2);
        __syncthreads();
        gen_if(early, 1, tile + 3);
    }
    __syncthreads();   // the staging area below overlays the A buffers

    // Epilogue.  D layout of a 16x16 tile: lane holds column lane % 16 and, in register v,
    // row 4 * (lane / 16) + v.  Each wave writes one 16 x RS block of rows at a time to its own
    // staging area and reads it back so that a lane holds four consecutive rank columns of
    // one row: memory is then accessed 16 bytes per lane, RS * 4 contiguous bytes per row.
    //
    // A workgroup that owns all columns of its rows updates the state directly.  When the
    // columns of a row block are shared between nparts workgroups (short launches, to fill
    // the chip), each stores its partial product; the one that finishes last adds the
    // partials in the order 0 .. nparts - 1, whoever it is, and updates the state, so the
    // result does not depend on timing.
    float* stage = reinterpret_cast<float*>(lds_raw) + wave * (16 * LDE);
    constexpr int LPR = RS / 4;           // lanes per row when reading back
    constexpr int RPI = 64 / LPR;         // rows per instruction
    constexpr int NP = 16 / RPI;          // passes per block of 16 rows
    const int erow = lane / LPR, echunk = lane % LPR;
    const bool split = it.nparts > 1;
    // direct: the state's buffer resource ends at the last valid row of this wave;
    // split: this part's BR x RS block of the partial area (always whole)
    float* pbase = partials + (size_t)it.poff + (size_t)it.part * (BR * RS) + (size_t)wave * (WR * RS);
    const rsrc_t st_rs = split ? make_rsrc(pbase, (long long)WR * RS * 4)
                               : make_rsrc(state + (wave_row0 < n ? wave_row0 : 0) * R, valid * R * 4);
    const uint32_t row_stride = split ? (uint32_t)RS : (uint32_t)R;
    const uint32_t col_base = split ? 0u : (uint32_t)(it.slice * RS);
    const bool rmw = !split && a != 0.f;
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
            for (int v = 0; v < 4; ++v) stage[(4 * g + v) * LDE + 16 * ct + li] = acc[rt][ct][v];
        // a wave's own LDS writes are visible to its own later reads once they have completed
        __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0)
        v4f oldv[NP];
        uint32_t goff[NP];
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int row = 16 * rt + erow + RPI * p;     // row within the wave's rows
            goff[p] = ((uint32_t)row * row_stride + col_base + 4u * (uint32_t)echunk) * 4u;
            oldv[p] = rmw ? buf_load_f4(st_rs, goff[p]) : v4f{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const v4f nv = *reinterpret_cast<const v4f*>(&stage[(erow + RPI * p) * LDE + 4 * echunk]);
            if (split) {
                // written through to memory (device scope): another XCD's L2 never sees a stale copy
                __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4u, nv), st_rs, (int)goff[p], 0, 16);
            } else {
                buf_store_f4(st_rs, goff[p], v4f{a * oldv[p].x + b * nv.x, a * oldv[p].y + b * nv.y,
                                                 a * oldv[p].z + b * nv.z, a * oldv[p].w + b * nv.w});
            }
        }
        __builtin_amdgcn_s_waitcnt(0xc07f);   // reads done before the next block overwrites the area
    }
    if (!split) return;

    // ---- shared columns: count arrivals; the last one combines.  The partials are stored and
    // loaded with device scope on the accesses themselves (write-through / L2-bypassing), so
    // no cache-wide release or acquire is needed: a store is visible once it has completed.
    // This is the release / acquire pair of the gfx942/gfx950 memory model spelled out for the
    // few accesses that need it: a device-scope release is "write dirty lines through, wait for
    // the stores" and a device-scope acquire is "do not read stale non-coherent lines".  A
    // release fence would write back the whole L2 of this XCD, which holds megabytes of state
    // the launch has just written (measured: tens of microseconds per fence); here only the
    // partial products are written through, the wait below (vmcnt(0), then the barrier) orders
    // them before the arrival count, the count is a device-scope atomic, and the last arriver's
    // loads carry the scope bit that makes them miss lines another XCD may have written.
    __builtin_amdgcn_s_waitcnt(0x0070);       // vmcnt(0): this thread's partial stores have completed ...
    __syncthreads();                          // ... and so have everybody's, before the arrival is counted
    if (tid == 0) lds_flag = atomicAdd(counters + it.cidx, 1u);
    __syncthreads();
    if (lds_flag != (uint32_t)(it.nparts - 1)) return;
    const float* gbase = partials + (size_t)it.poff;
    const rsrc_t prs = make_rsrc(gbase, (long long)it.nparts * BR * RS * 4);
    const long long rows_here = row_end - it.row0;          // valid rows of the block
    const int nvec = (int)rows_here * (RS / 4);
    // Two float4 positions per thread and four parts at a time are fetched before any is added,
    // so the combine costs a few memory round trips, not one per part and position; a part or
    // a position that does not exist is pointed out of range and adds exact zeros.  The order
    // of the additions stays 0 .. nparts - 1.
    const rsrc_t srs = make_rsrc(state + (long long)it.row0 * R, rows_here * (long long)R * 4);
    for (int f0 = tid; f0 < nvec; f0 += 2 * 512) {
        uint32_t poff2[2], soff[2];
        v4f oldv[2], sum[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int f = f0 + 512 * u;
            const bool ok = f < nvec;
            const int row = f / (RS / 4), c4 = f % (RS / 4);
            poff2[u] = ok ? ((uint32_t)row * RS + 4u * (uint32_t)c4) * 4u : kOob;
            soff[u] = ok ? ((uint32_t)row * (uint32_t)R + (uint32_t)(it.slice * RS) + 4u * (uint32_t)c4) * 4u : kOob;
            oldv[u] = (a != 0.f) ? buf_load_f4(srs, soff[u]) : v4f{0.f, 0.f, 0.f, 0.f};
            sum[u] = v4f{0.f, 0.f, 0.f, 0.f};
        }
        for (int q0 = 0; q0 < it.nparts; q0 += 4) {
            v4f pv[4][2];
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    // device-coherent load: the other parts were written by other compute units
                    const bool ok = q0 + j < it.nparts && poff2[u] != kOob;
                    const uint32_t off = ok ? (uint32_t)(q0 + j) * (uint32_t)(BR * RS * 4) + poff2[u] : kOob;
                    pv[j][u] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(prs, (int)off, 0, 16));
                }
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    sum[u].x += pv[j][u].x; sum[u].y += pv[j][u].y; sum[u].z += pv[j][u].z; sum[u].w += pv[j][u].w;
                }
        }
#pragma unroll
        for (int u = 0; u < 2; ++u)
            buf_store_f4(srs, soff[u], v4f{a * oldv[u].x + b * sum[u].x, a * oldv[u].y + b * sum[u].y,
                                           a * oldv[u].z + b * sum[u].z, a * oldv[u].w + b * sum[u].w});
    }
    if (tid == 0) counters[it.cidx] = 0u;     // every part has arrived: ready for the next launch
}

}  // namespace

namespace {

template <int MAP>
hipError_t launch_wide(const MatDev* mats, const WorkItem* items, int nitems, const SeedArgs& seeds, int r, int mt,
                       float a, float b, float* partials, uint32_t* counters, hipStream_t s)
{
    const dim3 grid((unsigned)nitems), block(512);
    if (mt == 32) {
        if (r == 64) hipLaunchKernelGGL((compress_bf16_wide_kernel<4, 1, MAP, true>), grid, block, 0, s, mats, items, seeds, r, a, b, partials, counters);
        else if (r == 128) hipLaunchKernelGGL((compress_bf16_wide_kernel<8, 1, MAP, true>), grid, block, 0, s, mats, items, seeds, r, a, b, partials, counters);
        else hipLaunchKernelGGL((compress_bf16_wide_kernel<8, 1, MAP, false>), grid, block, 0, s, mats, items, seeds, r, a, b, partials, counters);
    } else if (mt == 8) {
        if (r == 64) hipLaunchKernelGGL((compress_bf16_wide_kernel<4, 4, MAP, true>), grid, block, 0, s, mats, items, seeds, r, a, b, partials, counters);
        else if (r == 128) hipLaunchKernelGGL((compress_bf16_wide_kernel<8, 4, MAP, true>), grid, block, 0, s, mats, items, seeds, r, a, b, partials, counters);
        else hipLaunchKernelGGL((compress_bf16_wide_kernel<8, 4, MAP, false>), grid, block, 0, s, mats, items, seeds, r, a, b, partials, counters);
    } else {
        if (r == 64) hipLaunchKernelGGL((compress_bf16_wide_kernel<4, 2, MAP, true>), grid, block, 0, s, mats, items, seeds, r, a, b, partials, counters);
        else if (r == 128) hipLaunchKernelGGL((compress_bf16_wide_kernel<8, 2, MAP, true>), grid, block, 0, s, mats, items, seeds, r, a, b, partials, counters);
        else hipLaunchKernelGGL((compress_bf16_wide_kernel<8, 2, MAP, false>), grid, block, 0, s, mats, items, seeds, r, a, b, partials, counters);
    }
    return hipGetLastError();
}

template <int MAP>
hipError_t launch_narrow(const MatDev* mats, const WorkItem* items, int nitems, const SeedArgs& seeds, int r, int mt,
                         int grad_is_f32, float a, float b, dim3 grid, dim3 block, hipStream_t s)
{
    (void)nitems;
    switch (mt) {
    case 1:
        if (grad_is_f32) hipLaunchKernelGGL((compress_bf16_kernel<1, float, MAP>), grid, block, 0, s, mats, items, seeds, r, a, b);
        else hipLaunchKernelGGL((compress_bf16_kernel<1, uint16_t, MAP>), grid, block, 0, s, mats, items, seeds, r, a, b);
        break;
    case 2:
        if (grad_is_f32) hipLaunchKernelGGL((compress_bf16_kernel<2, float, MAP>), grid, block, 0, s, mats, items, seeds, r, a, b);
        else hipLaunchKernelGGL((compress_bf16_kernel<2, uint16_t, MAP>), grid, block, 0, s, mats, items, seeds, r, a, b);
        break;
    case 4:
        if (grad_is_f32) hipLaunchKernelGGL((compress_bf16_kernel<4, float, MAP>), grid, block, 0, s, mats, items, seeds, r, a, b);
        else hipLaunchKernelGGL((compress_bf16_kernel<4, uint16_t, MAP>), grid, block, 0, s, mats, items, seeds, r, a, b);
        break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace

// All items of one launch share one MT (rows per workgroup = 128 * MT; 8, 16 and 32 select the wide
// kernel), chosen by the host.  partials / counters: workspace of the wide kernel's shared-column
// mode (may be null when no item has nparts > 1).
hipError_t launch_compress_bf16_mt(const MatDev* mats, const WorkItem* items, int nitems,
                                   const SeedArgs& seeds, int r, int mt, int grad_is_f32, int map, float a, float b,
                                   float* partials, uint32_t* counters, hipStream_t s)
{
    if (nitems == 0) return hipSuccess;
    if (r != 64 && r != 128 && r != 256) return hipErrorInvalidValue;
    if (grad_is_f32 && mt > 4) return hipErrorInvalidValue;   // fp32 gradients: first kernel only
    if (map != 0 && map != 1) return hipErrorInvalidValue;
    if (mt == 8 || mt == 16 || mt == 32)     // wide kernel: 512 (8), 256 (16) or 128 (32) rows per workgroup, rank slices of 128 (64 at r = 64)
        return (map == 1) ? launch_wide<1>(mats, items, nitems, seeds, r, mt, a, b, partials, counters, s)
                          : launch_wide<0>(mats, items, nitems, seeds, r, mt, a, b, partials, counters, s);
    const dim3 grid((unsigned)nitems), block(256);
    return (map == 1) ? launch_narrow<1>(mats, items, nitems, seeds, r, mt, grad_is_f32, a, b, grid, block, s)
                      : launch_narrow<0>(mats, items, nitems, seeds, r, mt, grad_is_f32, a, b, grid, block, s);
}

}  // namespace flora
