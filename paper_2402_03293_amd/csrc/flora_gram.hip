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
// gram_kernel: one workgroup sums X_t X_t^T over a chunk of the long index t (X_t = row t of A,
//   regenerated, optionally scaled by 1 / sqrt(K_t); or row t of S, loaded) into a partial r x r
//   matrix; tiles of 64 t are staged in LDS transposed ([k][t], bf16), both MFMA operands come
//   from there.  combine_gram_kernel adds the chunks' partials in chunk order and stores the
//   result as bf16 in the arrangement quadform_kernel copies into LDS.
// quadform_kernel: q_i = Z_i B Z_i^T for a block of rows of Z (rows of S, loaded; or rows of A,
//   regenerated), B a Gram matrix held in LDS.  The product is taken transposed,
//   D[k2][i] = sum_k1 B[k2][k1] Z[i][k1], so that lane (i, g) ends up with D[16 c + 4 g + v][i]; the
//   contraction order over k1 is free, and it is chosen so that the same lane's operand
//   registers hold exactly Z[i][16 c + 4 g + v]: q_i is then a dot product of registers the lane
//   already has, summed over the four lanes that share a row.
#include "flora_gen.hip.h"
#include "flora_internal.h"

namespace flora {

namespace {

constexpr int kGT = 64;          // long-index entries per tile
constexpr int kGLd = kGT + 8;    // padded LDS row (bf16 elements): 144 bytes

// Position within a 32-block of the contraction index k1 = 32 s + x, x = 16 h + 4 g + v (h < 2, g < 4,
// v < 4): lane group g holds, for step s, the eight values x = 4 g + v and x = 16 + 4 g + v.
__device__ __forceinline__ int perm32(int x) { return 8 * ((x >> 2) & 3) + 4 * (x >> 4) + (x & 3); }

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
    float* part = M.grampart + (size_t)it.part * R * R;
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

// B <- sum over the chunks of their partials, in chunk order; stored as bf16 with the columns of
// every 32-block in the order quadform_kernel contracts them.  which 0: P (chunks of m), 1: Q (chunks of n)
template <int R>
__global__ __launch_bounds__(256) void combine_gram_kernel(const MatDev* __restrict__ mats, int which)
{
    const MatDev& M = mats[blockIdx.y];
    const int idx = (blockIdx.x * 256 + threadIdx.x) * 4;       // four consecutive k1 of one row k2
    if (idx >= R * R) return;
    const int nch = which ? M.gchunks_n : M.gchunks_m;
    v4f s = {0.f, 0.f, 0.f, 0.f};
    for (int c = 0; c < nch; ++c) {
        const v4f p = ldg4(M.grampart + (size_t)c * R * R + idx);
        s.x += p.x; s.y += p.y; s.z += p.z; s.w += p.w;
    }
    uint16_t* B = which ? M.gramQ : M.gramP;
    const int k2 = idx / R, k1 = idx % R;                       // k1 % 4 == 0: the four stay together
    const int pos = (k1 & ~31) + perm32(k1 & 31);
    const v2u pk = {pack_bf16x2(s.x, s.y), pack_bf16x2(s.z, s.w)};
    *reinterpret_cast<FLORA_GLOBAL v2u*>((FLORA_GLOBAL uint16_t*)(B + k2 * R + pos)) = pk;
}

// SRC 0: Z = S (rows of the state), B = P;  SRC 1: Z = A(seed) (rows = columns of W), B = Q.
// OUT 0: rowpart[i] <- alpha^2 q_i;  OUT 1: colpart[j] <- alpha^2 q_j;
// OUT 2: itempart[block] <- alpha^2 mean(R) sum_i q_i / R_i  (the clipping sum of this row block)
template <int R, int SRC, int OUT>
__global__ __launch_bounds__(512) void quadform_kernel(const MatDev* __restrict__ mats, const WorkItem* __restrict__ items,
                                                       const SeedArgs seeds, float alpha)
{
    constexpr int S = R / 32;            // contraction steps
    constexpr int CT = R / 16;           // 16-row tiles of B
    constexpr int LDB = R + 8;           // padded LDS row (bf16 elements)
    constexpr int ZT = 2;                // 16-row tiles of Z per wave and round
    __shared__ __attribute__((aligned(16))) uint16_t ldsB[R][LDB];
    __shared__ float lds_fin[8];

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
        const uint16_t* B = SRC == 0 ? M.gramP : M.gramQ;
        for (int f = tid; f < R * (R / 8); f += 512) {
            const int k2 = f / (R / 8), c8 = f % (R / 8);
            *reinterpret_cast<v4u*>(&ldsB[k2][8 * c8]) = ldg4(B + k2 * R + 8 * c8);
        }
    }
    __syncthreads();

    float total = 0.f;
    for (long long rb = it.row0; rb < row_end; rb += 8 * 16 * ZT) {
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
                if (OUT == 0) { if (g == 0) stg(M.rowpart + row, alpha * alpha * v); }
                else if (OUT == 1) { if (g == 0) stg(M.colpart + row, alpha * alpha * v); }
                else if (g == 0) total += v / ldg(M.row_stat + row);
            }
        }
    }
    if (OUT == 2) {
        float t = total;
        t += __shfl_xor(t, 8);
        t += __shfl_xor(t, 4);
        t += __shfl_xor(t, 2);
        t += __shfl_xor(t, 1);
        if (lane == 0) lds_fin[wave] = t;
        __syncthreads();
        if (tid == 0)
            M.itempart[it.part] = alpha * alpha * ldg(M.scal) *
                                  (((lds_fin[0] + lds_fin[1]) + (lds_fin[2] + lds_fin[3])) +
                                   ((lds_fin[4] + lds_fin[5]) + (lds_fin[6] + lds_fin[7])));
    }
}

template <int R>
hipError_t launch_gram_r(const MatDev* mats, const WorkItem* items, int nitems, const SeedArgs& seeds, int src, hipStream_t s)
{
    const dim3 grid((unsigned)nitems), block(512);
    switch (src) {
    case 0: hipLaunchKernelGGL((gram_kernel<R, 0>), grid, block, 0, s, mats, items, seeds); break;
    case 1: hipLaunchKernelGGL((gram_kernel<R, 1>), grid, block, 0, s, mats, items, seeds); break;
    case 2: hipLaunchKernelGGL((gram_kernel<R, 2>), grid, block, 0, s, mats, items, seeds); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <int R>
hipError_t launch_quadform_r(const MatDev* mats, const WorkItem* items, int nitems, const SeedArgs& seeds, int out,
                             float alpha, hipStream_t s)
{
    const dim3 grid((unsigned)nitems), block(512);
    switch (out) {
    case 0: hipLaunchKernelGGL((quadform_kernel<R, 0, 0>), grid, block, 0, s, mats, items, seeds, alpha); break;
    case 1: hipLaunchKernelGGL((quadform_kernel<R, 1, 1>), grid, block, 0, s, mats, items, seeds, alpha); break;
    case 2: hipLaunchKernelGGL((quadform_kernel<R, 0, 2>), grid, block, 0, s, mats, items, seeds, alpha); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace

// src 0: P = A^T A, 1: P' = A^T diag(1 / K) A (both over chunks of m), 2: Q = S^T S (chunks of n);
// partial sums per work item, then the chunks are added in order and stored as bf16
hipError_t launch_gram(const MatDev* mats, const WorkItem* items, int nitems, int count, const SeedArgs& seeds, int r,
                       int src, hipStream_t s)
{
    if (nitems == 0 || count == 0) return hipSuccess;
    hipError_t e;
    const dim3 cgrid((unsigned)(r * r / 1024), (unsigned)count);
    switch (r) {
    case 64:
        e = launch_gram_r<64>(mats, items, nitems, seeds, src, s);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((combine_gram_kernel<64>), cgrid, dim3(256), 0, s, mats, src == 2 ? 1 : 0);
        break;
    case 128:
        e = launch_gram_r<128>(mats, items, nitems, seeds, src, s);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((combine_gram_kernel<128>), cgrid, dim3(256), 0, s, mats, src == 2 ? 1 : 0);
        break;
    case 256:
        e = launch_gram_r<256>(mats, items, nitems, seeds, src, s);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((combine_gram_kernel<256>), cgrid, dim3(256), 0, s, mats, src == 2 ? 1 : 0);
        break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// out 0: row sums of Gt^2 (Z = S, B = P), 1: column sums (Z = A, B = Q), 2: the clipping sum (Z = S, B = P')
hipError_t launch_quadform(const MatDev* mats, const WorkItem* items, int nitems, const SeedArgs& seeds, int r, int out,
                           float alpha, hipStream_t s)
{
    if (nitems == 0) return hipSuccess;
    switch (r) {
    case 64: return launch_quadform_r<64>(mats, items, nitems, seeds, out, alpha, s);
    case 128: return launch_quadform_r<128>(mats, items, nitems, seeds, out, alpha, s);
    case 256: return launch_quadform_r<256>(mats, items, nitems, seeds, out, alpha, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace flora
