// Small grouped kernels around the Adafactor rules (the base optimizer of the
// paper's experiments, Section 3.1; unfactored variant, Section 3.3) and the end of an
// accumulation cycle (Algorithm 1: the accumulator starts each cycle at zero).
// All reductions run in a fixed order, so results are reproducible bit for bit.
#include "flora_internal.h"

namespace flora {

namespace {

__device__ __forceinline__ float block_sum_256(float v, float* lds)
{
    const int tid = threadIdx.x;
    lds[tid] = v;
    __syncthreads();
#pragma unroll
    for (int s = 128; s > 0; s >>= 1) {
        if (tid < s) lds[tid] += lds[tid + s];
        __syncthreads();
    }
    const float r = lds[0];
    __syncthreads();
    return r;
}

// R_i <- beta2 R_i + (1 - beta2) (rowmean(Gt^2) + eps1), K_j likewise by column,
// scal[0] <- mean(R), scal[1] <- 1 (no clipping until rms_finalize says otherwise).
// (gram: the sums came whole, one value per row and column)
__global__ __launch_bounds__(256) void stats_finalize_kernel(const MatDev* __restrict__ mats,
                                                             float beta2, float eps1, int gram)
{
    __shared__ float lds[256];
    const MatDev& M = mats[blockIdx.x];
    const long long n = M.n, m = M.m;
    const int tid = threadIdx.x;
    const int ncc = gram ? 1 : M.ncolchunks, nrb = gram ? 1 : M.nrowblocks;
    float rsum = 0.f;
    for (long long i = tid; i < n; i += 256) {
        float s = 0.f;
        for (int c = 0; c < ncc; ++c) s += M.rowpart[(long long)c * n + i];
        const float r = beta2 * M.row_stat[i] + (1.f - beta2) * (s / (float)m + eps1);
        M.row_stat[i] = r;
        rsum += r;
    }
    for (long long j = tid; j < m; j += 256) {
        float s = 0.f;
        for (int b = 0; b < nrb; ++b) s += M.colpart[(long long)b * m + j];
        M.col_stat[j] = beta2 * M.col_stat[j] + (1.f - beta2) * (s / (float)n + eps1);
    }
    const float tot = block_sum_256(rsum, lds);
    if (tid == 0) {
        M.scal[0] = tot / (float)n;
        M.scal[1] = 1.f;
    }
}

// scal[1] <- 1 / max(1, RMS(U) / clip_d), RMS(U)^2 = sum of the workgroup partials / (n m)
// (1 when clip_d == 0: no clipping);  scal[2] <- max(eps2, RMS(W)) from the caller's sum of W^2
// when the step is relative to the parameter scale, else 1.
// (gram: the partial sums of U^2 are those of the quadratic-form pass, one per row block)
__global__ __launch_bounds__(256) void rms_finalize_kernel(const MatDev* __restrict__ mats, float clip_d,
                                                           int scale_parameter, float eps2, int gram)
{
    __shared__ float lds[256];
    const MatDev& M = mats[blockIdx.x];
    const int tid = threadIdx.x;
    float tot = 0.f;
    if (gram) {
        // mean(R) from the row blocks' sums of the new R, which the quadratic-form pass left in rowpart
        float s = 0.f;
        for (int i = tid; i < M.item0; i += 256) s += M.rowpart[i];
        const float mean_r = block_sum_256(s, lds) / (float)M.n;
        __syncthreads();
        if (tid == 0) { M.scal[0] = mean_r; M.scal[1] = 1.f; }
        tot = mean_r;                                      // the factor the clipping partials still lack
    }
    if (clip_d > 0.f) {
        float s = 0.f;
        const int np = gram ? M.item0 : M.nitems;
        for (int i = tid; i < np; i += 256) s += M.itempart[i];
        tot = block_sum_256(s, lds) * (gram ? tot : 1.f);
    }
    if (tid == 0) {
        float clip = 1.f;
        if (clip_d > 0.f) {
            const float rms = sqrtf(tot / ((float)M.n * (float)M.m));
            const float d = rms / clip_d;
            clip = 1.f / (d > 1.f ? d : 1.f);
        }
        M.scal[1] = clip;
        float ps = 1.f;
        if (scale_parameter) {
            const float rmsw = sqrtf(M.wsumsq[0] / ((float)M.n * (float)M.m));
            ps = rmsw > eps2 ? rmsw : eps2;
        }
        M.scal[2] = ps;
    }
}

// wsumsq <- sum of the update pass's per-workgroup partial sums of the new W^2
__global__ __launch_bounds__(256) void wsumsq_finalize_kernel(const MatDev* __restrict__ mats)
{
    __shared__ float lds[256];
    const MatDev& M = mats[blockIdx.x];
    if (!M.wsumsq) return;
    const int tid = threadIdx.x;
    float s = 0.f;
    for (int i = tid; i < M.nitems; i += 256) s += M.itempart[i];
    const float tot = block_sum_256(s, lds);
    if (tid == 0) M.wsumsq[0] = tot;
}

// Sum of W^2 from scratch: workgroup b of matrix l sums the float4s b, b + 256, ... of W
// (and the last n m % 4 values in workgroup 0) into partials[l][b].
template <typename WT>
__global__ __launch_bounds__(256) void weight_sumsq_kernel(const MatDev* __restrict__ mats,
                                                           float* __restrict__ partials)
{
    __shared__ float lds[256];
    const MatDev& M = mats[blockIdx.y];
    const long long total = M.n * M.m, total4 = total >> 2;
    const WT* W = reinterpret_cast<const WT*>(M.weight);
    const int tid = threadIdx.x;
    float s = 0.f;
    for (long long i = (long long)blockIdx.x * 256 + tid; i < total4; i += (long long)kSumsqBlocks * 256) {
        v4f w;
        if (sizeof(WT) == 4) {
            w = ldg4(reinterpret_cast<const float*>(W) + 4 * i);
        } else {
            const v2u pk = ldg2(reinterpret_cast<const uint16_t*>(W) + 4 * i);
            w = v4f{bf16_bits_to_f32(pk.x & 0xffffu), bf16_bits_to_f32(pk.x >> 16),
                    bf16_bits_to_f32(pk.y & 0xffffu), bf16_bits_to_f32(pk.y >> 16)};
        }
        s = __builtin_fmaf(w.x, w.x, s);
        s = __builtin_fmaf(w.y, w.y, s);
        s = __builtin_fmaf(w.z, w.z, s);
        s = __builtin_fmaf(w.w, w.w, s);
    }
    if (blockIdx.x == 0 && tid < (int)(total & 3)) {
        const float w = load_elem(W + 4 * total4 + tid);
        s = __builtin_fmaf(w, w, s);
    }
    const float tot = block_sum_256(s, lds);
    if (tid == 0) partials[(long long)blockIdx.y * kSumsqBlocks + blockIdx.x] = tot;
}

__global__ __launch_bounds__(256) void weight_sumsq_finalize_kernel(const MatDev* __restrict__ mats,
                                                                    const float* __restrict__ partials)
{
    __shared__ float lds[256];
    const MatDev& M = mats[blockIdx.x];
    const float tot = block_sum_256(partials[(long long)blockIdx.x * kSumsqBlocks + threadIdx.x], lds);
    if (threadIdx.x == 0) M.wsumsq[0] = tot;
}

__global__ __launch_bounds__(256) void zero_state_kernel(const MatDev* __restrict__ mats, int r)
{
    const MatDev& M = mats[blockIdx.y];
    const long long total4 = (M.n * r) >> 2;   // r is a multiple of 4
    float4* p = reinterpret_cast<float4*>(M.state);
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total4; i += (long long)gridDim.x * 256)
        p[i] = make_float4(0.f, 0.f, 0.f, 0.f);
}

}  // namespace

hipError_t launch_stats_finalize(const MatDev* mats, int count, float beta2, float eps1, int gram, hipStream_t s)
{
    if (count == 0) return hipSuccess;
    hipLaunchKernelGGL(stats_finalize_kernel, dim3((unsigned)count), dim3(256), 0, s, mats, beta2, eps1, gram);
    return hipGetLastError();
}

hipError_t launch_rms_finalize(const MatDev* mats, int count, float clip_d, int scale_parameter, float eps2, int gram,
                               hipStream_t s)
{
    if (count == 0) return hipSuccess;
    hipLaunchKernelGGL(rms_finalize_kernel, dim3((unsigned)count), dim3(256), 0, s, mats, clip_d,
                       scale_parameter, eps2, gram);
    return hipGetLastError();
}

hipError_t launch_wsumsq_finalize(const MatDev* mats, int count, hipStream_t s)
{
    if (count == 0) return hipSuccess;
    hipLaunchKernelGGL(wsumsq_finalize_kernel, dim3((unsigned)count), dim3(256), 0, s, mats);
    return hipGetLastError();
}

hipError_t launch_weight_sumsq(const MatDev* mats, int count, int weight_is_bf16, float* partials, hipStream_t s)
{
    if (count == 0) return hipSuccess;
    static_assert(kSumsqBlocks == 256, "one partial per thread of the finalize kernel");
    if (weight_is_bf16)
        hipLaunchKernelGGL(weight_sumsq_kernel<uint16_t>, dim3(kSumsqBlocks, (unsigned)count), dim3(256), 0, s, mats, partials);
    else
        hipLaunchKernelGGL(weight_sumsq_kernel<float>, dim3(kSumsqBlocks, (unsigned)count), dim3(256), 0, s, mats, partials);
    hipLaunchKernelGGL(weight_sumsq_finalize_kernel, dim3((unsigned)count), dim3(256), 0, s, mats, partials);
    return hipGetLastError();
}

hipError_t launch_zero_state(const MatDev* mats, int count, int r, hipStream_t s)
{
    if (count == 0) return hipSuccess;
    hipLaunchKernelGGL(zero_state_kernel, dim3(16, (unsigned)count), dim3(256), 0, s, mats, r);
    return hipGetLastError();
}

}  // namespace flora
