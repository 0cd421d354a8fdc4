// Device-side generator for the projection A ~ N_s(0, 1/r) (Algorithm 1 and
// Algorithm 2, sampling lines).  A is a pure function of (seed, j, k): kernels
// call these helpers to rebuild the tile they need in registers or LDS, so A
// never exists in HBM (Section 2.4, "Memory analysis": only the seed is kept).
//
// Definition (generator version 1):
//   words   = Philox4x32-10(counter = (j mod 2^32, q, j >> 32, 0), key = seed)
//   u(x)    = ((x >> 9) + 1/2) * 2^-23
//   (z0,z1) = sqrt(-2 ln u(w0)) * (cos, sin)(2 pi u(w1));  (z2,z3) from (w2,w3)
//   A[j, 4q+i] = z_i / sqrt(r)
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace flora {

constexpr uint32_t kPhiloxM0 = 0xD2511F53u;
constexpr uint32_t kPhiloxM1 = 0xCD9E8D57u;
constexpr uint32_t kPhiloxW0 = 0x9E3779B9u;
constexpr uint32_t kPhiloxW1 = 0xBB67AE85u;
constexpr uint32_t kDomainA = 0u;
constexpr uint32_t kDomainSeed = 1u;

struct Words4 {
    uint32_t w[4];
};

// Philox4x32-10 (Salmon et al., SC'11).  The key schedule depends only on the
// seed, which is uniform across a workgroup, so it lives in scalar registers.
__host__ __device__ __forceinline__ Words4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2,
                                                         uint32_t c3, uint32_t k0, uint32_t k1)
{
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint64_t p0 = (uint64_t)kPhiloxM0 * (uint64_t)c0;
        const uint64_t p1 = (uint64_t)kPhiloxM1 * (uint64_t)c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += kPhiloxW0;
        k1 += kPhiloxW1;
    }
    Words4 o;
    o.w[0] = c0; o.w[1] = c1; o.w[2] = c2; o.w[3] = c3;
    return o;
}

__device__ __forceinline__ Words4 raw_quad(uint32_t seed_lo, uint32_t seed_hi, uint64_t j, uint32_t q)
{
    return philox4x32_10((uint32_t)j, q, (uint32_t)(j >> 32), kDomainA, seed_lo, seed_hi);
}

// (2 * (x >> 9) + 1) * 2^-24: an odd integer below 2^24 times 2^-24, exact in fp32.
__device__ __forceinline__ float uniform23(uint32_t x)
{
    return __builtin_fmaf((float)(x >> 9), 0x1p-23f, 0x1p-24f);
}

// Box-Muller on two words.  `neg2_ln2_over_r` = -2 ln(2) / r folds the 1/sqrt(r)
// scale into the radius: rho = sqrt(-2 ln(u1) / r) = sqrt(log2(u1) * (-2 ln 2 / r)).
// log2 and the revolution-based sine/cosine map directly onto the hardware's
// transcendental unit; their inputs are exact, so the only error is the unit's own.
__device__ __forceinline__ void box_muller(uint32_t xa, uint32_t xb, float neg2_ln2_over_r,
                                           float& z_cos, float& z_sin)
{
    const float u1 = uniform23(xa);
    const float u2 = uniform23(xb);
    const float rho = __builtin_amdgcn_sqrtf(__builtin_amdgcn_logf(u1) * neg2_ln2_over_r);
    const float s = __builtin_amdgcn_sinf(u2);
    const float c = __builtin_amdgcn_cosf(u2);
    z_cos = rho * c;
    z_sin = rho * s;
}

struct Quad {
    float z[4];
};

// A[j, 4q .. 4q+3], already scaled by 1/sqrt(r).
__device__ __forceinline__ Quad normal_quad(uint32_t seed_lo, uint32_t seed_hi, uint64_t j,
                                            uint32_t q, float neg2_ln2_over_r)
{
    const Words4 x = raw_quad(seed_lo, seed_hi, j, q);
    Quad o;
    box_muller(x.w[0], x.w[1], neg2_ln2_over_r, o.z[0], o.z[1]);
    box_muller(x.w[2], x.w[3], neg2_ln2_over_r, o.z[2], o.z[3]);
    return o;
}

__host__ __device__ __forceinline__ float neg2_ln2_over(int r)
{
    return -1.3862943611198906f / (float)r;
}

}  // namespace flora
