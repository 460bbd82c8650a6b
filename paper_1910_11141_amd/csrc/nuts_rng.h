// Device-side counter-based random numbers: Philox4x32-10 (Salmon et al., SC'11,
// Section 3.3) keyed by the sampler seed, with the counter carrying
// (position, purpose | level << 8, iteration, chain).  Because every draw is a
// pure function of where it is used, a chain's random numbers do not depend on
// how the scheduler interleaves chains (the independence property Section 2 of
// the batching paper relies on).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace nuts {

enum DrawTag : uint32_t {
    kDrawInit = 0,       // position k -> components 2k, 2k+1 of x0
    kDrawMomentum = 1,   // position k -> components 2k, 2k+1 of the momentum
    kDrawDirection = 2,  // position j -> direction of doubling j
    kDrawSubtree = 3,    // position = leapfrog count at the merge, level in bits 8..15
    kDrawTop = 4,        // position j -> acceptance of doubling j
    kDrawSlice = 5       // position 0 -> slice height of the iteration (slice sampler only)
};

struct Words4 {
    uint32_t w0, w1, w2, w3;
};

__device__ __forceinline__ Words4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                                uint32_t k1)
{
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        const uint32_t n0 = hi1 ^ c1 ^ k0;
        const uint32_t n2 = hi0 ^ c3 ^ k1;
        c0 = n0;
        c1 = lo1;
        c2 = n2;
        c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return Words4{c0, c1, c2, c3};
}

struct DrawKey {
    uint32_t k0, k1;  // seed, low and high half
};

__device__ __forceinline__ Words4 draw(DrawKey key, uint32_t position, uint32_t tag, uint32_t level,
                                       uint32_t iteration, uint32_t chain)
{
    return philox4x32_10(position, tag | (level << 8), iteration, chain, key.k0, key.k1);
}

// 52 bits -> midpoint of one of 2^52 cells of (0,1); exact, never 0 or 1.
__device__ __forceinline__ double uniform52(uint32_t a, uint32_t b)
{
    const uint64_t m = ((uint64_t)(a >> 6) << 26) | (uint64_t)(b >> 6);
    return (double)(2 * m + 1) * 0x1p-53;
}

// Box-Muller; `second` picks the sine branch.
__device__ __forceinline__ double normal_of(const Words4& w, bool second)
{
    const double u1 = uniform52(w.w0, w.w1);
    const double u2 = uniform52(w.w2, w.w3);
    const double rho = sqrt(-2.0 * log(u1));
    const double phi = 6.283185307179586476925286766559 * u2;
    double s, c;
    sincos(phi, &s, &c);
    return rho * (second ? s : c);
}

// Both normals of one draw: z0 is the cosine branch (component 2k), z1 the sine branch (component 2k + 1).
__device__ __forceinline__ void normal_pair(const Words4& w, double& z0, double& z1)
{
    const double u1 = uniform52(w.w0, w.w1);
    const double u2 = uniform52(w.w2, w.w3);
    const double rho = sqrt(-2.0 * log(u1));
    const double phi = 6.283185307179586476925286766559 * u2;
    double s, c;
    sincos(phi, &s, &c);
    z0 = rho * c;
    z1 = rho * s;
}

__device__ __forceinline__ double logaddexp(double a, double b)
{
    const double m = a > b ? a : b;
    if (m == -INFINITY) return -INFINITY;
    return m + log1p(exp(-fabs(a - b)));
}

}  // namespace nuts
