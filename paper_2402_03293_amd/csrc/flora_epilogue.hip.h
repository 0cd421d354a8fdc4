// What happens to a 32 x 32 tile of the decompressed gradient
// Gt = alpha * state A^T while it is still in the accumulator registers of a
// 32x32 MFMA (lane holds column lane % 32; register v holds row
// 8 * (v / 4) + 4 * (lane / 32) + v % 4).  Shared by the fp32 and bf16
// decompression kernels; Gt is never written to memory except by kModeOut.
#pragma once
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
    float colsum;   // kModeStats: sum of Gt^2 down this lane's column; kModeRms: running total
    float kfac;     // per-column factor of kModeFactored / kModeRms
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
        const float meanR = M.scal[0], clip = M.scal[1];
        e.kfac = jok ? p.coef * p.alpha * clip * sqrtf(meanR) * rsqrtf(M.col_stat[j]) : 0.f;
    }
    if (MODE == kModeRms) {
        const float meanR = M.scal[0];
        e.kfac = jok ? p.alpha * p.alpha * meanR / M.col_stat[j] : 0.f;
    }
    return e;
}

// lds_red: float[4][32] scratch of the workgroup (kModeStats / kModeRms only).
template <int MODE, typename OT>
__device__ __forceinline__ void epilogue_tile(const f32x16& acc, const MatDev& M, const WorkItem& it,
                                              const DecompressParams& p, long long rb,
                                              long long row_end, long long j, bool jok,
                                              EpilogueLane& e, float (*lds_red)[32])
{
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int ln = lane & 31, g = lane >> 5;
    const long long n = M.n, m = M.m;
    float rowsq[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const long long row = rb + 8 * (v / 4) + 4 * g + (v % 4);
        const bool ok = jok && row < row_end;
        if (MODE == kModeOut) {
            if (ok) {
                const float val = p.alpha * acc[v];
                OT* o = reinterpret_cast<OT*>(M.out) + row * m + j;
                if (sizeof(OT) == 4) *reinterpret_cast<float*>(o) = val;
                else *reinterpret_cast<uint16_t*>(o) = (uint16_t)f32_to_bf16_bits(val);
            }
        } else if (MODE == kModeSgd) {
            if (ok) {
                float* w = M.weight + row * m + j;
                *w = *w - p.coef * acc[v];
            }
        } else if (MODE == kModeStats) {
            const float gt = p.alpha * acc[v];
            const float q = ok ? gt * gt : 0.f;
            e.colsum += q;
            rowsq[v] = q;
        } else if (MODE == kModeRms) {
            if (ok) e.colsum += acc[v] * acc[v] * e.kfac / M.row_stat[row];
        } else if (MODE == kModeFactored) {
            if (ok) {
                float* w = M.weight + row * m + j;
                *w = *w - e.kfac * rsqrtf(M.row_stat[row]) * acc[v];
            }
        }
    }
    if (MODE == kModeStats) {
        // row sums over this wave's 32 columns, then over the 4 waves in a fixed order
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const float s = half_wave_sum(rowsq[v]);
            if (ln == 0) lds_red[wave][8 * (v / 4) + 4 * g + (v % 4)] = s;
        }
        __syncthreads();
        if (tid < 32) {
            const long long row = rb + tid;
            if (row < row_end) {
                const float s = ((lds_red[0][tid] + lds_red[1][tid]) + lds_red[2][tid]) + lds_red[3][tid];
                M.rowpart[(long long)it.slice * n + row] = s;
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
        if (g == 0 && jok) M.colpart[(long long)it.rblock * M.m + j] = e.colsum;
    }
    if (MODE == kModeRms) {
        float s = half_wave_sum(e.colsum);
        s += __shfl_xor(s, 32);
        if (lane == 0) lds_red[wave][0] = s;
        __syncthreads();
        if (tid == 0)
            M.itempart[(int)blockIdx.x - M.item0] =
                ((lds_red[0][0] + lds_red[1][0]) + lds_red[2][0]) + lds_red[3][0];
    }
}

}  // namespace flora
