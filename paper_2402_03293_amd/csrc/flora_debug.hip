// Test hook: materialise A(seed) and the raw Philox words so that the
// generator can be compared with the CPU oracle word for word.  The hot-path
// kernels never call this; they rebuild A tiles in registers / LDS.
#include "flora_gen.hip.h"
#include "flora_internal.h"

namespace flora {

__global__ __launch_bounds__(256) void debug_generate_kernel(uint32_t seed_lo, uint32_t seed_hi,
                                                             long long m, int r, float* A_out,
                                                             uint32_t* raw_out)
{
    const int nq = r >> 2;
    const long long total = m * (long long)nq;
    const float c = neg2_ln2_over(r);
    for (long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
         idx += (long long)gridDim.x * blockDim.x) {
        const long long j = idx / nq;
        const uint32_t q = (uint32_t)(idx - j * nq);
        const Words4 x = raw_quad(seed_lo, seed_hi, (uint64_t)j, q);
        if (raw_out) {
            uint4 v = make_uint4(x.w[0], x.w[1], x.w[2], x.w[3]);
            *reinterpret_cast<uint4*>(raw_out + idx * 4) = v;
        }
        if (A_out) {
            float4 z;
            box_muller(x.w[0], x.w[1], c, z.x, z.y);
            box_muller(x.w[2], x.w[3], c, z.z, z.w);
            *reinterpret_cast<float4*>(A_out + j * r + 4 * q) = z;
        }
    }
}

// Plain copy of a known size: the yardstick that profiler byte counters are scaled by.
__global__ __launch_bounds__(256) void debug_copy_kernel(const v4u* __restrict__ src, v4u* __restrict__ dst,
                                                         long long n16)
{
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n16; i += (long long)gridDim.x * 256)
        dst[i] = src[i];
}

hipError_t launch_debug_copy(const void* src, void* dst, long long bytes, hipStream_t s)
{
    const long long n16 = bytes / 16;
    if (n16 == 0) return hipSuccess;
    hipLaunchKernelGGL(debug_copy_kernel, dim3(4096), dim3(256), 0, s, static_cast<const v4u*>(src),
                       static_cast<v4u*>(dst), n16);
    return hipGetLastError();
}

hipError_t launch_debug_generate(uint64_t seed, long long m, int r, float* A_out, uint32_t* raw_out,
                                 hipStream_t s)
{
    const long long total = m * (long long)(r >> 2);
    if (total == 0) return hipSuccess;
    long long blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(debug_generate_kernel, dim3((unsigned)blocks), dim3(256), 0, s,
                       (uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32), m, r, A_out, raw_out);
    return hipGetLastError();
}

}  // namespace flora
