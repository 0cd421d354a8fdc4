// What happens to a 32 x 32 tile of the decompressed gradient
// Gt = alpha * state A^T while it is still in the accumulator registers of a
// 32x32 MFMA (lane holds column lane % 32; register v holds row
// 8 * (v / 4) + 4 * (lane / 32) + v % 4).  Shared by the fp32 and bf16
// decompression kernels; Gt is never written to memory except by kModeOut.
#pragma once
#include <type_traits>

#include "flora_internal.h"

namespace flora {

__device__ __forceinline__ float half_wave_sum(float v)
{
    // sum over the 32 lanes that share lane / 32
    v += __shfl_xor(v, 16);
    v += __shfl_xor(v, 8);
    v += __shfl_xor(v, 4);
    v += __shfl_xor(v, 2);
    v += __shfl_xor(v, 1);
    return v;
}

// Per-lane state that lives across the row loop of one workgroup.
struct EpilogueLane {
    float colsum;   // kModeStats: sum of Gt^2 down this lane's column; otherwise this lane's running total
                    // (kModeRms / kModeFull1: of U^2; kModeFactored / kModeFull2: of the new W^2)
    float kfac;     // per-column factor of kModeFactored / kModeRms; step factor of kModeFull2
};

template <int MODE>
__device__ __forceinline__ EpilogueLane epilogue_begin(const MatDev& M, const DecompressParams& p,
                                                       long long j, bool jok)
{
    EpilogueLane e;
    e.colsum = 0.f;
    e.kfac = 0.f;
    if (MODE == kModeFactored) {
        // U = Gt / sqrt(R_i K_j / mean R), scaled by lr and the RMS clip factor
        // (scal[2]: the parameter scale max(eps2, RMS(W)), or 1)
        const float meanR = ldg(M.scal), clip = ldg(M.scal + 1), ps = ldg(M.scal + 2);
        e.kfac = jok ? p.coef * p.alpha * clip * ps * sqrtf(meanR) * rsqrtf(ldg(M.col_stat + j)) : 0.f;
    }
    if (MODE == kModeFull2) {
        // U = Gt / sqrt(V_ij), scaled the same way
        const float clip = ldg(M.scal + 1), ps = ldg(M.scal + 2);
        e.kfac = jok ? p.coef * p.alpha * clip * ps : 0.f;
    }
    if (MODE == kModeRms) {
        const float meanR = ldg(M.scal);
        e.kfac = jok ? p.alpha * p.alpha * meanR / ldg(M.col_stat + j) : 0.f;
    }
    return e;
}

// Values of a tile that the epilogue reads from memory (old weights, row statistics),
// fetched one tile ahead so that their latency overlaps the previous tile's work.
template <int MODE>
struct TilePre {
    float w[(MODE == kModeSgd || MODE == kModeFactored || MODE == kModeFull2) ? 16 : 1];
    float rs[(MODE == kModeRms || MODE == kModeFactored) ? 16 : 1];
    float v[(MODE == kModeFull1 || MODE == kModeFull2) ? 16 : 1];
};

// Row of register v of this lane, relative to the tile's first row.
__device__ __forceinline__ int tile_row(int v, int g) { return 8 * (v / 4) + 4 * g + (v % 4); }

// Addresses inside a tile are a workgroup-uniform base (first row of the tile) plus a 32-bit
// per-lane element offset row * m + column: 33 m < 2^32 is guaranteed by the host (m <= 2^26).
template <int MODE, typename OT>
__device__ __forceinline__ void epilogue_fetch(TilePre<MODE>& pre, const MatDev& M, const DecompressParams& p,
                                               long long rb, long long row_end, long long j, bool jok)
{
    // cache policy of the weights and the second moment (uniform over the launch): one branch
    // around each group of 16 loads or stores, not one per access
    const bool ld_stream = (p.wpolicy & 1) != 0;
    const int g = (threadIdx.x & 63) >> 5;
    const uint32_t m32 = (uint32_t)M.m;
    // Clamped coordinates keep every load in bounds, so all 16 loads of a tile are issued
    // back to back; only the stores are predicated.
    const uint32_t jc = jok ? (uint32_t)j : m32 - 1u;
    const int last = (int)(row_end - 1 - rb);          // last valid row of the tile, relative
    if (MODE == kModeSgd || MODE == kModeFactored || MODE == kModeFull2) {
        const OT* tb = reinterpret_cast<const OT*>(M.weight) + rb * M.m;
        if (ld_stream) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const uint32_t rr = (uint32_t)(tile_row(v, g) < last ? tile_row(v, g) : last);
                pre.w[v] = load_elem<true>(tb + (rr * m32 + jc));
            }
        } else {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const uint32_t rr = (uint32_t)(tile_row(v, g) < last ? tile_row(v, g) : last);
                pre.w[v] = load_elem<false>(tb + (rr * m32 + jc));
            }
        }
    }
    if (MODE == kModeFull1 || MODE == kModeFull2) {
        const float* tb = M.vfull + rb * M.m;
        if (ld_stream) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const uint32_t rr = (uint32_t)(tile_row(v, g) < last ? tile_row(v, g) : last);
                pre.v[v] = load_elem<true>(tb + (rr * m32 + jc));
            }
        } else {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const uint32_t rr = (uint32_t)(tile_row(v, g) < last ? tile_row(v, g) : last);
                pre.v[v] = load_elem<false>(tb + (rr * m32 + jc));
            }
        }
    }
    if (MODE == kModeRms || MODE == kModeFactored) {
        const float* rbp = M.row_stat + rb;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const uint32_t rr = (uint32_t)(tile_row(v, g) < last ? tile_row(v, g) : last);
            pre.rs[v] = ldg(rbp + rr);
        }
    }
}

// lds_red: float[4][32] scratch of the workgroup (kModeStats / kModeRms only).
template <int MODE, typename OT>
__device__ __forceinline__ void epilogue_tile(const f32x16& acc, const TilePre<MODE>& pre, const MatDev& M,
                                              const WorkItem& it, const DecompressParams& p, long long rb,
                                              long long row_end, long long j, bool jok,
                                              EpilogueLane& e, float (*lds_red)[32])
{
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int ln = lane & 31, g = lane >> 5;
    const long long n = M.n, m = M.m;
    const int rows_here = (int)((row_end - rb < 32) ? row_end - rb : 32);
    const uint32_t m32 = (uint32_t)m, j32 = (uint32_t)j;
    const bool st_stream = (p.wpolicy & 2) != 0;    // see epilogue_fetch
    float rowsq[16];
    if (MODE == kModeOut) {
        OT* ob = reinterpret_cast<OT*>(M.out) + rb * m;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            if (jok && tile_row(v, g) < rows_here) {
                const float val = p.alpha * acc[v];
                OT* o = ob + ((uint32_t)tile_row(v, g) * m32 + j32);
                if (sizeof(OT) == 4) stg(reinterpret_cast<float*>(o), val);
                else stg(reinterpret_cast<uint16_t*>(o), (uint16_t)f32_to_bf16_bits(val));
            }
        }
    } else if (MODE == kModeSgd) {
        OT* wb = reinterpret_cast<OT*>(M.weight) + rb * m;
        auto sweep = [&](auto stream) {
#pragma unroll
            for (int v = 0; v < 16; ++v)
                if (jok && tile_row(v, g) < rows_here)
                    store_elem<decltype(stream)::value>(wb + ((uint32_t)tile_row(v, g) * m32 + j32),
                                                        pre.w[v] - p.coef * acc[v]);
        };
        if (st_stream) sweep(std::true_type{});
        else sweep(std::false_type{});
    } else if (MODE == kModeStats) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const float gt = p.alpha * acc[v];
            const float q = (jok && tile_row(v, g) < rows_here) ? gt * gt : 0.f;
            e.colsum += q;
            rowsq[v] = q;
        }
    } else if (MODE == kModeRms) {
#pragma unroll
        for (int v = 0; v < 16; ++v)
            if (jok && tile_row(v, g) < rows_here) e.colsum += acc[v] * acc[v] * e.kfac / pre.rs[v];
    } else if (MODE == kModeFactored) {
        OT* wb = reinterpret_cast<OT*>(M.weight) + rb * m;
        auto sweep = [&](auto stream) {
#pragma unroll
            for (int v = 0; v < 16; ++v)
                if (jok && tile_row(v, g) < rows_here) {
                    const float wn = store_elem<decltype(stream)::value>(wb + ((uint32_t)tile_row(v, g) * m32 + j32),
                                                                         pre.w[v] - e.kfac * rsqrtf(pre.rs[v]) * acc[v]);
                    e.colsum = __builtin_fmaf(wn, wn, e.colsum);     // of the value as stored
                }
        };
        if (st_stream) sweep(std::true_type{});
        else sweep(std::false_type{});
    } else if (MODE == kModeFull1) {
        float* vb = M.vfull + rb * m;
        auto sweep = [&](auto stream) {
#pragma unroll
            for (int v = 0; v < 16; ++v)
                if (jok && tile_row(v, g) < rows_here) {
                    const float gt = p.alpha * acc[v];
                    const float vn = p.beta2 * pre.v[v] + (1.f - p.beta2) * (gt * gt + p.eps1);
                    store_elem<decltype(stream)::value>(vb + ((uint32_t)tile_row(v, g) * m32 + j32), vn);
                    e.colsum += gt * gt / vn;
                }
        };
        if (st_stream) sweep(std::true_type{});
        else sweep(std::false_type{});
    } else if (MODE == kModeFull2) {
        OT* wb = reinterpret_cast<OT*>(M.weight) + rb * m;
        auto sweep = [&](auto stream) {
#pragma unroll
            for (int v = 0; v < 16; ++v)
                if (jok && tile_row(v, g) < rows_here) {
                    const float wn = store_elem<decltype(stream)::value>(wb + ((uint32_t)tile_row(v, g) * m32 + j32),
                                                                         pre.w[v] - e.kfac * rsqrtf(pre.v[v]) * acc[v]);
                    e.colsum = __builtin_fmaf(wn, wn, e.colsum);
                }
        };
        if (st_stream) sweep(std::true_type{});
        else sweep(std::false_type{});
    }
    if (MODE == kModeStats) {
        // row sums over this wave's 32 columns, then over the 4 waves in a fixed order
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const float s = half_wave_sum(rowsq[v]);
            if (ln == 0) lds_red[wave][tile_row(v, g)] = s;
        }
        __syncthreads();
        if (tid < 32) {
            const long long row = rb + tid;
            if (row < row_end) {
                const float s = ((lds_red[0][tid] + lds_red[1][tid]) + lds_red[2][tid]) + lds_red[3][tid];
                stg(M.rowpart + (long long)it.slice * n + row, s);
            }
        }
        __syncthreads();
    }
}

template <int MODE>
__device__ __forceinline__ void epilogue_end(const MatDev& M, const WorkItem& it, long long j,
                                             bool jok, EpilogueLane& e, float (*lds_red)[32])
{
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 5;
    if (MODE == kModeStats) {
        e.colsum += __shfl_xor(e.colsum, 32);
        if (g == 0 && jok) stg(M.colpart + (long long)it.rblock * M.m + j, e.colsum);
    }
    if (MODE == kModeRms || MODE == kModeFactored || MODE == kModeFull1 || MODE == kModeFull2) {
        float s = half_wave_sum(e.colsum);
        s += __shfl_xor(s, 32);
        if (lane == 0) lds_red[wave][0] = s;
        __syncthreads();
        if (tid == 0)
            M.itempart[it.part] =
                ((lds_red[0][0] + lds_red[1][0]) + lds_red[2][0]) + lds_red[3][0];
    }
}

}  // namespace flora
