// The reduction passes of the factored Adafactor rule (the base optimizer of the paper's
// experiments, Section 3.1) without the n x m product.  With Gt = alpha S A^T (S the n x r
// state, A the m x r projection) the row sums, column sums and the clipping sum of the rule are
// quadratic forms in r x r Gram matrices:
//     sum_j Gt_ij^2              = alpha^2 S_i P S_i^T,   P  = A^T A          (r x r, sum over m)
//     sum_i Gt_ij^2              = alpha^2 A_j Q A_j^T,   Q  = S^T S          (r x r, sum over n)
//     sum_ij Gt_ij^2 / (R_i K_j) = alpha^2 sum_i (S_i P' S_i^T) / R_i,   P' = A^T diag(1 / K) A
// which costs 6 (m + n) r^2 flops per matrix instead of the 4 n m r of two passes over the
// decompressed gradient.  Everything runs on the bf16 matrix cores with fp32 accumulation, the
// precision of the decompression itself: A and S are rounded to bf16 exactly as the update pass
// rounds them, the Gram matrices are accumulated in fp32 and rounded to bf16 once.
//
// What the kernels cost is regenerating A (the vector ALU), so the sums are ordered to sweep A
// twice, not three times: Q from one read of S and the column statistics K from a sweep over
// generated rows of A; then ONE further sweep over A yields both P and P'; then the row statistics
// R and the clipping sum from a read of S each.
//
// gram_sym_kernel (ranks >= 128) / gram_kernel (rank 64): one workgroup sums X_t X_t^T over a chunk
//   of the long index t (X_t = row t of A, regenerated, plain and scaled with 1 / K_t; or row t of
//   S, loaded) into partial r x r matrices; tiles of 64 t are staged in LDS transposed ([k][t],
//   bf16), both MFMA operands come from there.  combine_gram_kernel adds the chunks' partials in
//   chunk order and stores the result as bf16 in the arrangement the quadratic-form kernel that
//   reads it copies into LDS.
// quadform_kernel: q_i = Z_i B Z_i^T for a block of rows of Z (rows of S, loaded; at rank 64 also
//   rows of A, regenerated), B a Gram matrix held in LDS.  The product is taken transposed,
//   D[k2][i] = sum_k1 B[k2][k1] Z[i][k1], so that lane (i, g) ends up with D[16 c + 4 g + v][i]; the
//   contraction order over k1 is free, and it is chosen so that the same lane's operand
//   registers hold exactly Z[i][16 c + 4 g + v]: q_i is then a dot product of registers the lane
//   already has, summed over the four lanes that share a row.  quadform_cols_kernel (ranks >= 128)
//   is the same scheme on 32 x 32 x 16 tiles for rows of A generated into the operand registers.
//   The kernels finish the statistics themselves (R_i, K_j, one partial sum of R per row block).
#include <type_traits>

#include "flora_gen.hip.h"
#include "flora_internal.h"

namespace flora {

namespace {

constexpr int kGT = 64;          // long-index entries per tile
constexpr int kGLd = kGT + 8;    // padded LDS row (bf16 elements): 144 bytes

// Position within a 32-block of the contraction index k1 = 32 s + x, x = 16 h + 4 g + v (h < 2, g < 4,
// v < 4): lane group g holds, for step s, the eight values x = 4 g + v and x = 16 + 4 g + v.
__device__ __forceinline__ int perm32(int x) { return 8 * ((x >> 2) & 3) + 4 * (x >> 4) + (x & 3); }
// The same for quadform_cols_kernel (32 x 32 x 16 tiles): x = 8 a + 4 g + v (a < 4, g < 2, v < 4); lane half
// g holds, for step 2 s + (a >> 1) of the contraction, the values x = 8 a + 4 g + v in elements 4 (a & 1) + v.
__device__ __forceinline__ int perm32w(int x) { return 16 * (x >> 4) + 8 * ((x >> 2) & 1) + 4 * ((x >> 3) & 1) + (x & 3); }

// SRC 0: X = A(seed), 1: X = A(seed) diag(1 / sqrt(K)), 2: X = S (the state, fp32 in memory)
template <int R, int SRC>
__global__ __launch_bounds__(512) void gram_kernel(const MatDev* __restrict__ mats, const WorkItem* __restrict__ items,
                                                   const SeedArgs seeds)
{
    constexpr int NTR = R / 16;                       // 16-row tiles of the result
    constexpr int RT = (NTR >= 8) ? NTR / 8 : 1;      // row tiles per wave
    constexpr int NH = (NTR >= 8) ? 1 : 8 / NTR;      // waves that share a row tile split the columns
    constexpr int CT = NTR / NH;                      // column tiles per wave
    __shared__ __attribute__((aligned(16))) uint16_t ldsX[2][R][kGLd];

    const WorkItem it = items[blockIdx.x];
    const MatDev& M = mats[it.mat];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15, g = lane >> 4;
    const long long t0 = it.col0, t1 = it.col1;       // this chunk of the long index
    const int ntiles = (int)((t1 - t0 + kGT - 1) / kGT);
    const int row_tile0 = (NTR >= 8) ? wave * RT : wave % NTR;
    const int col_tile0 = (NTR >= 8) ? 0 : (wave / NTR) * CT;

    // ---- producers: a 64 x R tile of X, transposed, bf16
    const uint32_t seed_lo = seeds.s[it.mat].x, seed_hi = seeds.s[it.mat].y;
    const float cgen = neg2_ln2_over(R);
    constexpr int NQ = R / 32;                        // quads per thread and tile (generated X)
    constexpr int JG = kGT / NQ;
    const int gen_j = NQ * (tid % JG);
    const uint32_t gen_q = (uint32_t)(tid / JG);
    auto produce_generated = [&](int buf, int tile) {
        const long long j = t0 + (long long)tile * kGT + gen_j;
        uint32_t pk[NQ / 2][4];
        // the weights first (clamped addresses, so that the loads are issued together and are
        // long back when the first quad is done)
        float wt[NQ];
#pragma unroll
        for (int e = 0; e < NQ; ++e) {
            wt[e] = 1.f;
            if (SRC == 1) wt[e] = ldg(M.col_stat + ((j + e < t1) ? j + e : t1 - 1));
        }
#pragma unroll
        for (int e = 0; e < NQ; e += 2) {
            const Quad z0 = normal_quad(seed_lo, seed_hi, (uint64_t)(j + e), gen_q, cgen);
            const Quad z1 = normal_quad(seed_lo, seed_hi, (uint64_t)(j + e + 1), gen_q, cgen);
            float w0 = (SRC == 1) ? rsqrtf(wt[e]) : 1.f, w1 = (SRC == 1) ? rsqrtf(wt[e + 1]) : 1.f;
            w0 = (j + e < t1) ? w0 : 0.f;
            w1 = (j + e + 1 < t1) ? w1 : 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i) pk[e / 2][i] = pack_bf16x2(w0 * z0.z[i], w1 * z1.z[i]);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            uint16_t* dst = &ldsX[buf][4 * gen_q + i][gen_j];
            if (NQ == 8) *reinterpret_cast<uint4*>(dst) = make_uint4(pk[0][i], pk[NQ / 8][i], pk[NQ / 4][i], pk[NQ / 2 - 1][i]);
            else if (NQ == 4) *reinterpret_cast<uint2*>(dst) = make_uint2(pk[0][i], pk[NQ / 2 - 1][i]);
            else *reinterpret_cast<uint32_t*>(dst) = pk[0][i];
        }
    };
    // loaded X: unit = (pair of rows 2 p, 2 p + 1; four columns 4 k4 ..): 8 R units per tile, R / 64
    // per thread; eight consecutive lanes take eight row pairs (consecutive words of an LDS row),
    // the lanes 8 apart the next columns (a whole 128-byte line per row)
    constexpr int NU = R / 64;
    // (fetched one tile ahead of being stashed, so that the loads are in flight while the
    // current tile multiplies; rows past the chunk read through a resource that ends there)
    const long long chunk_rows = t1 - t0;
    const rsrc_t srs = make_rsrc(M.state + t0 * R, chunk_rows * (long long)R * 4 < 0x7fffffffLL ? chunk_rows * R * 4 : 0x7fffffffLL);
    auto fetch_loaded = [&](v4f (&st)[NU][2], int tile) {
#pragma unroll
        for (int u = 0; u < NU; ++u) {
            const int flat = tid + 512 * u;
            const int rest = flat >> 3;
            const int k4 = rest % (R / 4);
            const int p = (rest / (R / 4)) * 8 + (flat & 7);
            const long long ra = (long long)tile * kGT + 2 * p;       // relative to the chunk
            const uint32_t off = (uint32_t)((ra * R + 4 * k4) * 4);
            st[u][0] = (ra < chunk_rows) ? buf_load_f4(srs, off) : v4f{0.f, 0.f, 0.f, 0.f};
            st[u][1] = (ra + 1 < chunk_rows) ? buf_load_f4(srs, off + (uint32_t)(R * 4)) : v4f{0.f, 0.f, 0.f, 0.f};
        }
    };
    auto stash_loaded = [&](const v4f (&st)[NU][2], int buf) {
#pragma unroll
        for (int u = 0; u < NU; ++u) {
            const int flat = tid + 512 * u;
            const int rest = flat >> 3;
            const int k4 = rest % (R / 4);
            const int p = (rest / (R / 4)) * 8 + (flat & 7);
            const v4f a = st[u][0], b = st[u][1];
            *reinterpret_cast<uint32_t*>(&ldsX[buf][4 * k4 + 0][2 * p]) = pack_bf16x2(a.x, b.x);
            *reinterpret_cast<uint32_t*>(&ldsX[buf][4 * k4 + 1][2 * p]) = pack_bf16x2(a.y, b.y);
            *reinterpret_cast<uint32_t*>(&ldsX[buf][4 * k4 + 2][2 * p]) = pack_bf16x2(a.z, b.z);
            *reinterpret_cast<uint32_t*>(&ldsX[buf][4 * k4 + 3][2 * p]) = pack_bf16x2(a.w, b.w);
        }
    };

    f32x4 acc[RT][CT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) acc[rt][ct] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Producing the next tile and multiplying the current one are independent within a round, so
    // the two waves of a SIMD (w and w + 4) take them in opposite orders: while one regenerates on
    // the vector ALU the other keeps the matrix core busy.
    const bool produce_first = wave < 4;
    v4f stage[NU][2];
    if (SRC == 2) {
        fetch_loaded(stage, 0);
        stash_loaded(stage, 0);
        if (ntiles > 1) fetch_loaded(stage, 1);
    } else {
        produce_generated(0, 0);
    }
    __syncthreads();
    for (int tile = 0; tile < ntiles; ++tile) {
        const int buf = tile & 1;
        if (SRC != 2 && produce_first && tile + 1 < ntiles) produce_generated(buf ^ 1, tile + 1);
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            bf16x8 av[RT];
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
                av[rt] = *reinterpret_cast<const bf16x8*>(&ldsX[buf][16 * (row_tile0 + rt) + li][32 * s + 8 * g]);
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
                const bf16x8 bv = *reinterpret_cast<const bf16x8*>(&ldsX[buf][16 * (col_tile0 + ct) + li][32 * s + 8 * g]);
#pragma unroll
                for (int rt = 0; rt < RT; ++rt)
                    acc[rt][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[rt], bv, acc[rt][ct], 0, 0, 0);
            }
        }
        if (SRC != 2 && !produce_first && tile + 1 < ntiles) produce_generated(buf ^ 1, tile + 1);
        if (SRC == 2 && tile + 1 < ntiles) {
            stash_loaded(stage, buf ^ 1);                        // tile + 1, fetched a round ago
            if (tile + 2 < ntiles) fetch_loaded(stage, tile + 2);
        }
        __syncthreads();
    }

    // partial of this chunk: D layout, lane holds column 16 ct + li and rows 4 g + v of each tile
    // (partials: those of P over chunks of m, then those of Q over chunks of n, then those of P')
    const int part0 = SRC == 0 ? 0 : (SRC == 2 ? M.gchunks_m : M.gchunks_m + M.gchunks_n);
    float* part = M.grampart + (size_t)(part0 + it.part) * R * R;
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int k1 = 16 * (row_tile0 + rt) + 4 * g + v;
                const int k2 = 16 * (col_tile0 + ct) + li;
                stg(part + k1 * R + k2, acc[rt][ct][v]);
            }
}

// P = A^T A and P' = A^T diag(1 / K) A from ONE regeneration of A, at ranks >= 128.  The vector
// ALU work of the generator is what these sums cost, so both are taken from the same tile: the
// tile goes to LDS twice, plain and with its long-index entries scaled by 1 / K, and
// P'[k1][k2] = sum_t X[t][k1] (X[t][k2] / K_t) takes one operand from each copy.
// 16 waves, so that four share a SIMD and one wave's generator chains run in the shadow of the
// others'; v_mfma_f32_32x32x16_bf16 tiles; only the tiles on or above the diagonal of the
// symmetric results are computed (36 of 64 at r = 256), consecutive ones to a wave (they mostly
// share an operand), every SIMD multiplying the same number of them; a tile off the diagonal is
// also stored as its mirror image.
// MODE 0: P alone (no clipping asked for); 1: P and P'; 2: Q = S^T S, the tiles being rows of the
// state, fetched one tile ahead and rounded to bf16 on their way into LDS.
template <int R>
struct UpperTiles {
    static constexpr int NT = R / 32;                      // 32-wide tiles per dimension
    static constexpr int COUNT = NT * (NT + 1) / 2;
    // the idx-th tile (ti <= tj) in row-major order of the upper triangle
    __device__ static void at(int idx, int& ti, int& tj)
    {
        int c = idx, row = 0;
        while (c >= NT - row) { c -= NT - row; ++row; }
        ti = row; tj = row + c;
    }
};

template <int R, int MODE, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void gram_sym_kernel(const MatDev* __restrict__ mats, const WorkItem* __restrict__ items,
                                                         const SeedArgs seeds)
{
    static_assert(R >= 128, "ranks 128 and 256");
    typedef UpperTiles<R> UT;
    constexpr int TW = (UT::COUNT + WAVES - 1) / WAVES;   // tiles per wave
    constexpr int OWNERS = UT::COUNT < WAVES ? UT::COUNT : WAVES;
    constexpr bool PAIR = MODE == 1;
    constexpr int NC = PAIR ? 2 : 1;                       // copies of a tile: plain, scaled
    constexpr size_t kTileBytes = sizeof(uint16_t) * 2 * NC * R * kGLd, kTurnBytes = sizeof(float) * OWNERS * 32 * 33;
    __shared__ __attribute__((aligned(16))) unsigned char lds_raw[kTileBytes > kTurnBytes ? kTileBytes : kTurnBytes];
    uint16_t (*ldsX)[NC][R][kGLd] = reinterpret_cast<uint16_t (*)[NC][R][kGLd]>(lds_raw);   // [buffer][copy][k][t]

    const WorkItem it = items[blockIdx.x];
    const MatDev& M = mats[it.mat];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ln = lane & 31, g = lane >> 5;
    const long long t0 = it.col0, t1 = it.col1;
    const int ntiles = (int)((t1 - t0 + kGT - 1) / kGT);

    // this wave's tiles of the results: numbers wave, wave + WAVES, ... of the upper triangle, which
    // gives every SIMD (waves w, w + 4, ...) the same number of them
    int ti[TW], tj[TW];
    bool own[TW];
#pragma unroll
    for (int w = 0; w < TW; ++w) {
        const int idx = wave + WAVES * w;
        own[w] = idx < UT::COUNT;
        ti[w] = tj[w] = 0;
        if (own[w]) UT::at(idx, ti[w], tj[w]);
        ti[w] = __builtin_amdgcn_readfirstlane(ti[w]);
        tj[w] = __builtin_amdgcn_readfirstlane(tj[w]);
    }

    const uint32_t seed_lo = seeds.s[it.mat].x, seed_hi = seeds.s[it.mat].y;
    const float cgen = neg2_ln2_over(R);
    constexpr int NQ = R / (4 * WAVES);               // quads per thread and tile
    constexpr int JG = kGT / NQ;
    const int gen_j = NQ * (tid % JG);
    const uint32_t gen_q = (uint32_t)(tid / JG);
    auto produce = [&](int buf, int tile) {
        const long long j = t0 + (long long)tile * kGT + gen_j;
        float wt[NQ];
#pragma unroll
        for (int e = 0; e < NQ; ++e) {
            wt[e] = 1.f;
            if (PAIR) wt[e] = ldg(M.col_stat + ((j + e < t1) ? j + e : t1 - 1));
        }
        uint32_t pk[NC][NQ / 2][4];
#pragma unroll
        for (int e = 0; e < NQ; e += 2) {
            const Quad z0 = normal_quad(seed_lo, seed_hi, (uint64_t)(j + e), gen_q, cgen);
            const Quad z1 = normal_quad(seed_lo, seed_hi, (uint64_t)(j + e + 1), gen_q, cgen);
            const float m0 = (j + e < t1) ? 1.f : 0.f, m1 = (j + e + 1 < t1) ? 1.f : 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i) pk[0][e / 2][i] = pack_bf16x2(m0 * z0.z[i], m1 * z1.z[i]);
            if (PAIR) {
                const float w0 = m0 * __builtin_amdgcn_rcpf(wt[e]), w1 = m1 * __builtin_amdgcn_rcpf(wt[e + 1]);
#pragma unroll
                for (int i = 0; i < 4; ++i) pk[NC - 1][e / 2][i] = pack_bf16x2(w0 * z0.z[i], w1 * z1.z[i]);
            }
        }
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                uint16_t* dst = &ldsX[buf][c][4 * gen_q + i][gen_j];
                if (NQ == 8) *reinterpret_cast<uint4*>(dst) = make_uint4(pk[c][0][i], pk[c][NQ / 8][i], pk[c][NQ / 4][i], pk[c][NQ / 2 - 1][i]);
                else if (NQ == 4) *reinterpret_cast<uint2*>(dst) = make_uint2(pk[c][0][i], pk[c][NQ / 2 - 1][i]);
                else *reinterpret_cast<uint32_t*>(dst) = pk[c][0][i];
            }
    };

    // loaded X (MODE 2): unit = (pair of rows 2 p, 2 p + 1; four columns 4 k4 ..); eight consecutive
    // lanes take eight row pairs (consecutive words of an LDS row), the lanes 8 apart the next
    // columns (a whole 128-byte line per row); rows past the chunk read through a resource that
    // ends there
    constexpr int NU = (8 * R) / (64 * WAVES) > 0 ? (8 * R) / (64 * WAVES) : 1;
    const long long chunk_rows = t1 - t0;
    const rsrc_t srs = make_rsrc(M.state + (MODE == 2 ? t0 * R : 0),
                                 chunk_rows * (long long)R * 4 < 0x7fffffffLL ? chunk_rows * R * 4 : 0x7fffffffLL);
    auto fetch_loaded = [&](v4f (&st)[NU][2], int tile) {
#pragma unroll
        for (int u = 0; u < NU; ++u) {
            const int flat = tid + 64 * WAVES * u;
            const int rest = flat >> 3;
            const int k4 = rest % (R / 4);
            const int p = (rest / (R / 4)) * 8 + (flat & 7);
            const long long ra = (long long)tile * kGT + 2 * p;       // relative to the chunk
            const uint32_t off = (uint32_t)((ra * R + 4 * k4) * 4);
            st[u][0] = (ra < chunk_rows) ? buf_load_f4(srs, off) : v4f{0.f, 0.f, 0.f, 0.f};
            st[u][1] = (ra + 1 < chunk_rows) ? buf_load_f4(srs, off + (uint32_t)(R * 4)) : v4f{0.f, 0.f, 0.f, 0.f};
        }
    };
    auto stash_loaded = [&](const v4f (&st)[NU][2], int buf) {
#pragma unroll
        for (int u = 0; u < NU; ++u) {
            const int flat = tid + 64 * WAVES * u;
            const int rest = flat >> 3;
            const int k4 = rest % (R / 4);
            const int p = (rest / (R / 4)) * 8 + (flat & 7);
            const v4f a = st[u][0], b = st[u][1];
            *reinterpret_cast<uint32_t*>(&ldsX[buf][0][4 * k4 + 0][2 * p]) = pack_bf16x2(a.x, b.x);
            *reinterpret_cast<uint32_t*>(&ldsX[buf][0][4 * k4 + 1][2 * p]) = pack_bf16x2(a.y, b.y);
            *reinterpret_cast<uint32_t*>(&ldsX[buf][0][4 * k4 + 2][2 * p]) = pack_bf16x2(a.z, b.z);
            *reinterpret_cast<uint32_t*>(&ldsX[buf][0][4 * k4 + 3][2 * p]) = pack_bf16x2(a.w, b.w);
        }
    };

    f32x16 acc[NC][TW];
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
        for (int w = 0; w < TW; ++w)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[c][w][v] = 0.f;

    // the waves of a SIMD (w, w + 4, ...) take producing the next tile and multiplying the current
    // one in alternating orders
    const bool produce_first = ((wave >> 2) & 1) == 0;
    v4f stage[NU][2];
    if (MODE == 2) {
        fetch_loaded(stage, 0);
        stash_loaded(stage, 0);
        if (ntiles > 1) fetch_loaded(stage, 1);
    } else {
        produce(0, 0);
    }
    __syncthreads();
    for (int tile = 0; tile < ntiles; ++tile) {
        const int buf = tile & 1;
        if (MODE != 2 && produce_first && tile + 1 < ntiles) produce(buf ^ 1, tile + 1);
        // Straight-line code over all TW slots (a wave that owns TW - 1 tiles multiplies tile (0, 0)
        // again in its last slot and drops the result), so that the LDS reads of several
        // matrix-core instructions are in flight together.
#pragma unroll
        for (int s = 0; s < kGT / 16; ++s) {
#pragma unroll
            for (int w = 0; w < TW; ++w) {
                const bf16x8 av = *reinterpret_cast<const bf16x8*>(&ldsX[buf][0][32 * ti[w] + ln][16 * s + 8 * g]);
                const bf16x8 bv = *reinterpret_cast<const bf16x8*>(&ldsX[buf][0][32 * tj[w] + ln][16 * s + 8 * g]);
                acc[0][w] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc[0][w], 0, 0, 0);
                if (PAIR) {
                    const bf16x8 bs = *reinterpret_cast<const bf16x8*>(&ldsX[buf][NC - 1][32 * tj[w] + ln][16 * s + 8 * g]);
                    acc[NC - 1][w] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bs, acc[NC - 1][w], 0, 0, 0);
                }
            }
        }
        if (MODE != 2 && !produce_first && tile + 1 < ntiles) produce(buf ^ 1, tile + 1);
        if (MODE == 2 && tile + 1 < ntiles) {
            stash_loaded(stage, buf ^ 1);                        // tile + 1, fetched a round ago
            if (tile + 2 < ntiles) fetch_loaded(stage, tile + 2);
        }
        __syncthreads();
    }

    // D layout of a 32 x 32 tile: lane holds column ln and rows 8 (v / 4) + 4 g + v % 4.  A tile off
    // the diagonal is also stored as its mirror image, turned round in a piece of LDS that belongs
    // to the wave alone (the tiles of X are done with), so that both stores write whole lines.
    float* turn = reinterpret_cast<float*>(lds_raw) + wave * (32 * 33);     // (only waves that own tiles touch it)
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        // (partials: those of P over chunks of m, then those of Q over chunks of n, then those of P')
        const int part0 = MODE == 2 ? M.gchunks_m : (c ? M.gchunks_m + M.gchunks_n : 0);
        float* part = M.grampart + (size_t)(part0 + it.part) * R * R;
#pragma unroll
        for (int w = 0; w < TW; ++w) {
            if (own[w]) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int k1 = 8 * (v / 4) + 4 * g + (v % 4);
                    stg(part + (32 * ti[w] + k1) * R + 32 * tj[w] + ln, acc[c][w][v]);
                    if (ti[w] != tj[w]) turn[ln * 33 + k1] = acc[c][w][v];
                }
                if (ti[w] != tj[w]) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int k2 = 2 * v + g;                       // row of the mirror image; ln runs along it
                        stg(part + (32 * tj[w] + k2) * R + 32 * ti[w] + ln, turn[k2 * 33 + ln]);
                    }
                }
            }
        }
    }
}

// B <- sum over the chunks of their partials, in chunk order; stored as bf16 with the columns of
// every 32-block in the order quadform_kernel contracts them.  which 0: P (chunks of m), 1: Q (chunks
// of n), 2: P' (chunks of m; it is kept right behind Q)
template <int R>
__global__ __launch_bounds__(256) void combine_gram_kernel(const MatDev* __restrict__ mats, int which)
{
    const MatDev& M = mats[blockIdx.y];
    const int idx = (blockIdx.x * 256 + threadIdx.x) * 4;       // four consecutive k1 of one row k2
    if (idx >= R * R) return;
    const int nch = which == 1 ? M.gchunks_n : M.gchunks_m;
    const int part0 = which == 0 ? 0 : (which == 1 ? M.gchunks_m : M.gchunks_m + M.gchunks_n);
    v4f s = {0.f, 0.f, 0.f, 0.f};
    for (int c = 0; c < nch; ++c) {
        const v4f p = ldg4(M.grampart + (size_t)(part0 + c) * R * R + idx);
        s.x += p.x; s.y += p.y; s.z += p.z; s.w += p.w;
    }
    uint16_t* B = which == 0 ? M.gramP : (which == 1 ? M.gramQ : M.gramQ + R * R);
    const int k2 = idx / R, k1 = idx % R;                       // k1 % 4 == 0: the four stay together
    // (Q at ranks >= 128 is read by quadform_cols_kernel, everything else by quadform_kernel)
    const int pos = (k1 & ~31) + ((which == 1 && R >= 128) ? perm32w(k1 & 31) : perm32(k1 & 31));
    const v2u pk = {pack_bf16x2(s.x, s.y), pack_bf16x2(s.z, s.w)};
    *reinterpret_cast<FLORA_GLOBAL v2u*>((FLORA_GLOBAL uint16_t*)(B + k2 * R + pos)) = pk;
}

// SRC 0: Z = S (rows of the state), B = P;  SRC 1: Z = A(seed) (rows = columns of W), B = Q.
// The statistics are finished where the sums appear (each row and column belongs to one lane):
// OUT 0: R_i <- beta2 R_i + (1 - beta2) (alpha^2 q_i / m + eps1), and rowpart[block] <- the block's sum
//        of the new R_i (for mean(R));
// OUT 1: K_j <- beta2 K_j + (1 - beta2) (alpha^2 q_j / n + eps1);
// OUT 2: itempart[block] <- alpha^2 sum_i q_i / R_i  (the clipping sum of this row block, but for
//        the factor mean(R), which rms_finalize_kernel supplies)
template <int R, int SRC, int OUT, int WAVES, int ZT>
__global__ __launch_bounds__(64 * WAVES) void quadform_kernel(const MatDev* __restrict__ mats, const WorkItem* __restrict__ items,
                                                       const SeedArgs seeds, float alpha, float beta2, float eps1)
{
    constexpr int S = R / 32;            // contraction steps
    constexpr int CT = R / 16;           // 16-row tiles of B
    constexpr int LDB = R + 8;           // padded LDS row (bf16 elements)
    // (ZT: 16-row tiles of Z per wave and round)
    __shared__ __attribute__((aligned(16))) uint16_t ldsB[R][LDB];
    __shared__ float lds_fin[WAVES];

    const WorkItem it = items[blockIdx.x];
    const MatDev& M = mats[it.mat];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15, g = lane >> 4;
    const long long zn = SRC == 0 ? M.n : M.m;            // rows of Z
    const long long row_end = ((long long)it.row0 + it.rows < zn) ? (long long)it.row0 + it.rows : zn;
    const uint32_t seed_lo = seeds.s[it.mat].x, seed_hi = seeds.s[it.mat].y;
    const float cgen = neg2_ln2_over(R);

    // B into LDS: R rows of R bf16, 16 bytes per thread and step
    {
        const uint16_t* B = SRC == 1 ? M.gramQ : (OUT == 2 ? M.gramQ + R * R : M.gramP);
        for (int f = tid; f < R * (R / 8); f += 64 * WAVES) {
            const int k2 = f / (R / 8), c8 = f % (R / 8);
            *reinterpret_cast<v4u*>(&ldsB[k2][8 * c8]) = ldg4(B + k2 * R + 8 * c8);
        }
    }
    __syncthreads();

    float total = 0.f;
    for (long long rb = it.row0; rb < row_end; rb += WAVES * 16 * ZT) {
        // this wave's rows: rb + wave * 16 ZT + 16 z + li
        bf16x8 zreg[ZT][S];
#pragma unroll
        for (int z = 0; z < ZT; ++z) {
            const long long row = rb + (wave * ZT + z) * 16 + li;
            const bool ok = row < row_end;
#pragma unroll
            for (int s = 0; s < S; ++s) {
                v4f lo = {0.f, 0.f, 0.f, 0.f}, hi = {0.f, 0.f, 0.f, 0.f};
                if (SRC == 0) {
                    if (ok) {
                        lo = ldg4(M.state + row * R + 32 * s + 4 * g);
                        hi = ldg4(M.state + row * R + 32 * s + 16 + 4 * g);
                    }
                } else {
                    // (all lanes generate: rows past the end take the last row's values and are masked below)
                    const long long jr = ok ? row : zn - 1;
                    const Quad q0 = normal_quad(seed_lo, seed_hi, (uint64_t)jr, (uint32_t)(8 * s + g), cgen);
                    const Quad q1 = normal_quad(seed_lo, seed_hi, (uint64_t)jr, (uint32_t)(8 * s + 4 + g), cgen);
                    const float w = ok ? 1.f : 0.f;
                    lo = v4f{w * q0.z[0], w * q0.z[1], w * q0.z[2], w * q0.z[3]};
                    hi = v4f{w * q1.z[0], w * q1.z[1], w * q1.z[2], w * q1.z[3]};
                }
                const v4u pk = {pack_bf16x2(lo.x, lo.y), pack_bf16x2(lo.z, lo.w), pack_bf16x2(hi.x, hi.y), pack_bf16x2(hi.z, hi.w)};
                zreg[z][s] = __builtin_bit_cast(bf16x8, pk);
            }
        }
        float q[ZT];
#pragma unroll
        for (int z = 0; z < ZT; ++z) q[z] = 0.f;
        // two column tiles of D at a time: D[16 ct + 4 g + v][i], then its dot product with Z[i][16 ct + 4 g + v],
        // which is elements 4 (ct % 2) + v of step ct / 2 of this lane's own operand registers
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
            f32x4 acc[ZT];
#pragma unroll
            for (int z = 0; z < ZT; ++z) acc[z] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < S; ++s) {
                const bf16x8 bv = *reinterpret_cast<const bf16x8*>(&ldsB[16 * ct + li][32 * s + 8 * g]);
#pragma unroll
                for (int z = 0; z < ZT; ++z)
                    acc[z] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bv, zreg[z][s], acc[z], 0, 0, 0);
            }
#pragma unroll
            for (int z = 0; z < ZT; ++z) {
                const v4u zz = __builtin_bit_cast(v4u, zreg[z][ct / 2]);
                const uint32_t w0 = (ct & 1) ? zz.z : zz.x, w1 = (ct & 1) ? zz.w : zz.y;
                q[z] = __builtin_fmaf(acc[z][0], __uint_as_float(w0 << 16), q[z]);
                q[z] = __builtin_fmaf(acc[z][1], __uint_as_float(w0 & 0xffff0000u), q[z]);
                q[z] = __builtin_fmaf(acc[z][2], __uint_as_float(w1 << 16), q[z]);
                q[z] = __builtin_fmaf(acc[z][3], __uint_as_float(w1 & 0xffff0000u), q[z]);
            }
            // (keeps the compiler from hoisting every column tile's LDS reads to the top: the
            // registers are the operand tiles' and must not spill)
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int z = 0; z < ZT; ++z) {
            float v = q[z];
            v += __shfl_xor(v, 16);
            v += __shfl_xor(v, 32);             // all four lanes of row li now hold q_i
            const long long row = rb + (wave * ZT + z) * 16 + li;
            if (row < row_end) {
                if (OUT == 0) {
                    if (g == 0) {
                        const float rn = beta2 * ldg(M.row_stat + row) + (1.f - beta2) * (alpha * alpha * v / (float)M.m + eps1);
                        stg(M.row_stat + row, rn);
                        total += rn;
                    }
                } else if (OUT == 1) {
                    if (g == 0)
                        stg(M.col_stat + row, beta2 * ldg(M.col_stat + row) + (1.f - beta2) * (alpha * alpha * v / (float)M.n + eps1));
                } else if (g == 0) {
                    total += v / ldg(M.row_stat + row);
                }
            }
        }
    }
    if (OUT != 1) {
        float t = total;
        t += __shfl_xor(t, 8);
        t += __shfl_xor(t, 4);
        t += __shfl_xor(t, 2);
        t += __shfl_xor(t, 1);
        if (lane == 0) lds_fin[wave] = t;
        __syncthreads();
        if (tid == 0) {
            float fin = 0.f;
#pragma unroll
            for (int w = 0; w < WAVES; ++w) fin += lds_fin[w];
            if (OUT == 0) M.rowpart[it.part] = fin;
            else M.itempart[it.part] = alpha * alpha * fin;
        }
    }
}

// The column statistics at ranks >= 128: K_j <- beta2 K_j + (1 - beta2) (alpha^2 A_j Q A_j^T / n + eps1),
// rows A_j regenerated straight into matrix-core operand registers, Q in LDS.  The scheme of
// quadform_kernel on v_mfma_f32_32x32x16_bf16: a wave owns 32 rows per round, D[k2][j] =
// sum_k1 Q[k2][k1] A[j][k1] comes out with lane (j, g) holding k2 = 32 c + 8 a + 4 g + v, and the
// contraction order is chosen (perm32w) so that the lane's own operand registers hold exactly
// A[j][32 c + 8 a + 4 g + v].  Twice the rows per LDS read of Q and the faster tile shape.
template <int R, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void quadform_cols_kernel(const MatDev* __restrict__ mats,
                                                                   const WorkItem* __restrict__ items, const SeedArgs seeds,
                                                                   float alpha, float beta2, float eps1)
{
    constexpr int S = R / 16;            // contraction steps
    constexpr int CT = R / 32;           // 32-row tiles of Q
    constexpr int LDB = R + 8;           // padded LDS row (bf16 elements)
    __shared__ __attribute__((aligned(16))) uint16_t ldsB[R][LDB];

    const WorkItem it = items[blockIdx.x];
    const MatDev& M = mats[it.mat];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ln = lane & 31, g = lane >> 5;
    const long long zn = M.m;
    const long long row_end = ((long long)it.row0 + it.rows < zn) ? (long long)it.row0 + it.rows : zn;
    const uint32_t seed_lo = seeds.s[it.mat].x, seed_hi = seeds.s[it.mat].y;
    const float cgen = neg2_ln2_over(R);

    for (int f = tid; f < R * (R / 8); f += 64 * WAVES) {
        const int k2 = f / (R / 8), c8 = f % (R / 8);
        *reinterpret_cast<v4u*>(&ldsB[k2][8 * c8]) = ldg4(M.gramQ + k2 * R + 8 * c8);
    }
    __syncthreads();

    for (long long rb = it.row0; rb < row_end; rb += WAVES * 32) {
        const long long row = rb + wave * 32 + ln;
        const bool ok = row < row_end;
        // (all lanes generate: rows past the end take the last row's values and are masked below)
        const long long jr = ok ? row : zn - 1;
        const float w = ok ? 1.f : 0.f;
        bf16x8 zreg[S];
#pragma unroll
        for (int s = 0; s < S; ++s) {
            // step s = 2 beta + sl holds k1 = 32 beta + 16 sl + 4 g + (0..3) and the same + 8: quads 8 beta + 4 sl + g and + 2
            const uint32_t q0 = (uint32_t)(8 * (s >> 1) + 4 * (s & 1) + g);
            const Quad a = normal_quad(seed_lo, seed_hi, (uint64_t)jr, q0, cgen);
            const Quad b = normal_quad(seed_lo, seed_hi, (uint64_t)jr, q0 + 2u, cgen);
            const v4u pk = {pack_bf16x2(w * a.z[0], w * a.z[1]), pack_bf16x2(w * a.z[2], w * a.z[3]),
                            pack_bf16x2(w * b.z[0], w * b.z[1]), pack_bf16x2(w * b.z[2], w * b.z[3])};
            zreg[s] = __builtin_bit_cast(bf16x8, pk);
        }
        float q = 0.f;
#pragma unroll
        for (int c = 0; c < CT; ++c) {
            f32x16 acc;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
            for (int s = 0; s < S; ++s) {
                const bf16x8 bv = *reinterpret_cast<const bf16x8*>(&ldsB[32 * c + ln][16 * s + 8 * g]);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bv, zreg[s], acc, 0, 0, 0);
            }
            // acc[4 a + v] = D[32 c + 8 a + 4 g + v][j]; A[j][that k2] is element 4 (a & 1) + v of step 2 c + (a >> 1)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                const v4u zz = __builtin_bit_cast(v4u, zreg[2 * c + (a >> 1)]);
                const uint32_t w0 = (a & 1) ? zz.z : zz.x, w1 = (a & 1) ? zz.w : zz.y;
                q = __builtin_fmaf(acc[4 * a + 0], __uint_as_float(w0 << 16), q);
                q = __builtin_fmaf(acc[4 * a + 1], __uint_as_float(w0 & 0xffff0000u), q);
                q = __builtin_fmaf(acc[4 * a + 2], __uint_as_float(w1 << 16), q);
                q = __builtin_fmaf(acc[4 * a + 3], __uint_as_float(w1 & 0xffff0000u), q);
            }
            // (keeps the compiler from hoisting every tile's LDS reads to the top)
            __builtin_amdgcn_sched_barrier(0);
        }
        q += __shfl_xor(q, 32);                 // both lanes of row j now hold A_j Q A_j^T
        if (ok && g == 0)
            stg(M.col_stat + row, beta2 * ldg(M.col_stat + row) + (1.f - beta2) * (alpha * alpha * q / (float)M.n + eps1));
    }
}

template <int R>
hipError_t launch_gram_r(const MatDev* mats, const WorkItem* items, int nitems, int count, const SeedArgs& seeds, int src,
                         hipStream_t s)
{
    const dim3 grid((unsigned)nitems), block(512), cgrid((unsigned)(R * R / 1024), (unsigned)count);
    bool p = false, q = false, p2 = false;               // which sums this launch produces
    if constexpr (R >= 128) {
        constexpr int PW = R >= 256 ? 8 : 16;           // waves that can hold both sets of accumulators
        if (src == 0) { hipLaunchKernelGGL((gram_sym_kernel<R, 0, 16>), grid, dim3(1024), 0, s, mats, items, seeds); p = true; }
        if (src == 3) { hipLaunchKernelGGL((gram_sym_kernel<R, 1, PW>), grid, dim3(64 * PW), 0, s, mats, items, seeds); p = p2 = true; }
        if (src == 2) { hipLaunchKernelGGL((gram_sym_kernel<R, 2, 16>), grid, dim3(1024), 0, s, mats, items, seeds); q = true; }
    } else {
        if (src == 0 || src == 3) { hipLaunchKernelGGL((gram_kernel<R, 0>), grid, block, 0, s, mats, items, seeds); p = true; }
        if (src == 3) { hipLaunchKernelGGL((gram_kernel<R, 1>), grid, block, 0, s, mats, items, seeds); p2 = true; }
        if (src == 2) { hipLaunchKernelGGL((gram_kernel<R, 2>), grid, block, 0, s, mats, items, seeds); q = true; }
    }
    if (!p && !q && !p2) return hipErrorInvalidValue;
    if (p) hipLaunchKernelGGL((combine_gram_kernel<R>), cgrid, dim3(256), 0, s, mats, 0);
    if (q) hipLaunchKernelGGL((combine_gram_kernel<R>), cgrid, dim3(256), 0, s, mats, 1);
    if (p2) hipLaunchKernelGGL((combine_gram_kernel<R>), cgrid, dim3(256), 0, s, mats, 2);
    return hipGetLastError();
}

template <int R>
hipError_t launch_quadform_r(const MatDev* mats, const WorkItem* items, int nitems, const SeedArgs& seeds, int out,
                             float alpha, float beta2, float eps1, hipStream_t s)
{
    // r = 256: the operand registers of a row tile are a quarter of a 128-register budget, so 16
    // waves with one row tile each; below that 8 waves with two
    constexpr int W = R >= 256 ? 16 : 8, ZT = R >= 256 ? 1 : 2;
    const dim3 grid((unsigned)nitems), block(64 * W);
    if constexpr (R >= 128) {
        if (out == 1) {
            hipLaunchKernelGGL((quadform_cols_kernel<R, 16>), grid, dim3(1024), 0, s, mats, items, seeds, alpha, beta2, eps1);
            return hipGetLastError();
        }
    }
    switch (out) {
    case 0: hipLaunchKernelGGL((quadform_kernel<R, 0, 0, W, ZT>), grid, block, 0, s, mats, items, seeds, alpha, beta2, eps1); break;
    case 1: hipLaunchKernelGGL((quadform_kernel<R, 1, 1, W, ZT>), grid, block, 0, s, mats, items, seeds, alpha, beta2, eps1); break;
    case 2: hipLaunchKernelGGL((quadform_kernel<R, 0, 2, W, ZT>), grid, block, 0, s, mats, items, seeds, alpha, beta2, eps1); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace

// src 0: P = A^T A; 3: P and P' = A^T diag(1 / K) A from one regeneration of A (over chunks of m);
// 2: Q = S^T S (chunks of n).  Partial sums per work item, then the chunks are added in order and
// stored as bf16.
hipError_t launch_gram(const MatDev* mats, const WorkItem* items, int nitems, int count, const SeedArgs& seeds, int r,
                       int src, hipStream_t s)
{
    if (nitems == 0 || count == 0) return hipSuccess;
    switch (r) {
    case 64: return launch_gram_r<64>(mats, items, nitems, count, seeds, src, s);
    case 128: return launch_gram_r<128>(mats, items, nitems, count, seeds, src, s);
    case 256: return launch_gram_r<256>(mats, items, nitems, count, seeds, src, s);
    default: return hipErrorInvalidValue;
    }
}

// out 0: row sums of Gt^2 (Z = S, B = P) into the row statistics, 1: column sums (Z = A, B = Q) into the
// column statistics, 2: the clipping sum (Z = S, B = P')
hipError_t launch_quadform(const MatDev* mats, const WorkItem* items, int nitems, const SeedArgs& seeds, int r, int out,
                           float alpha, float beta2, float eps1, hipStream_t s)
{
    if (nitems == 0) return hipSuccess;
    switch (r) {
    case 64: return launch_quadform_r<64>(mats, items, nitems, seeds, out, alpha, beta2, eps1, s);
    case 128: return launch_quadform_r<128>(mats, items, nitems, seeds, out, alpha, beta2, eps1, s);
    case 256: return launch_quadform_r<256>(mats, items, nitems, seeds, out, alpha, beta2, eps1, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace flora
