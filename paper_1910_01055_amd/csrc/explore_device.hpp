// Device side of the actor's exploration (Sec. 4.1): the counter-based generator Philox4x32-10
// (Salmon, Moraes, Dror, Shaw, "Parallel random numbers: as easy as 1, 2, 3", SC'11) and Box-Muller on
// 24-bit uniforms.  Shared by the stand-alone exploration kernels and the fused forward.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace aq {

struct U4 {
    uint32_t x, y, z, w;
};

// ten rounds; the key advances by the Weyl constants before every round but the first
__device__ __forceinline__ U4 philox4x32_10(U4 c, uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        if (r > 0) {
            k0 += 0x9E3779B9u;
            k1 += 0xBB67AE85u;
        }
        const uint32_t hi0 = __umulhi(0xD2511F53u, c.x), lo0 = 0xD2511F53u * c.x;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c.z), lo1 = 0xCD9E8D57u * c.z;
        c = U4{hi1 ^ c.y ^ k0, lo1, hi0 ^ c.w ^ k1, lo0};
    }
    return c;
}

// Box-Muller on 24-bit uniforms: u1 in (0, 1], u2 in [0, 1)
__device__ __forceinline__ void box_muller(uint32_t a, uint32_t b, float& z_cos, float& z_sin) {
    const float u1 = (float)((a >> 8) + 1u) * 5.9604644775390625e-8f;
    const float u2 = (float)(b >> 8) * 5.9604644775390625e-8f;
    const float rad = sqrtf(-2.0f * logf(u1));
    float sn, cs;
    sincosf(6.283185307179586f * u2, &sn, &cs);
    z_cos = rad * cs;
    z_sin = rad * sn;
}

// the standard normal draw of (row, feature n) at this step: block n / 4, words (0, 1) serve features
// 4 block + (0, 1) as (cos, sin), words (2, 3) features 4 block + (2, 3)
__device__ __forceinline__ float gaussian_draw(uint32_t row, int n, uint32_t k0, uint32_t k1, uint32_t s0, uint32_t s1) {
    const U4 r = philox4x32_10(U4{row, (uint32_t)(n >> 2), s0, s1}, k0, k1);
    float zc, zs;
    if (n & 2) box_muller(r.z, r.w, zc, zs);
    else box_muller(r.x, r.y, zc, zs);
    return (n & 1) ? zs : zc;
}

}  // namespace aq
