// Counter-based random streams of the HIP library (device side).
//
// Philox4x32-10 is the public algorithm of Salmon, Moraes, Dror and Shaw (SC'11).
// The paper (arXiv 2104.02184, Sec. 3) only says that stochastic pulse trains are drawn and
// that steps carry pulse-to-pulse and device-to-device Gaussian variation; which generator
// feeds which draw is this library's choice:
//   key      = 64-bit tile seed
//   counter  = (line or cell index, sample b or Gaussian block, step t, tag<<24 | sub-block)
//   tags     1 = column (x) trains, 2 = row (d) trains, 3 = pulse-to-pulse noise,
//            4 = device-to-device planes
// Gaussian block `blk` of a stream: words (r0,r1) -> numbers 0,1 and (r2,r3) -> numbers 2,3 by
// Box-Muller on 24-bit uniforms u1 = ((ra>>8)+1) 2^-24, u2 = (rb>>8) 2^-24.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace aht {

constexpr uint32_t kTagX = 1u, kTagD = 2u, kTagC2C = 3u, kTagD2D = 4u;

struct U4 {
    uint32_t x, y, z, w;
};

// a ^ b ^ c in one instruction (gfx950 three-input bit operation, truth table 0x96)
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c)
{
    return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

__device__ __forceinline__ U4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                            uint32_t k0, uint32_t k1)
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        const uint32_t n0 = xor3((uint32_t)(p1 >> 32), c1, k0);
        const uint32_t n2 = xor3((uint32_t)(p0 >> 32), c3, k1);
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return U4{c0, c1, c2, c3};
}

// Fast Box-Muller pair on the transcendental unit: v_log_f32 (log2), v_sqrt_f32 and
// v_sin_f32 / v_cos_f32, whose argument is in revolutions -- exactly u2.
__device__ __forceinline__ void box_muller_fast(uint32_t ra, uint32_t rb, float& z_even, float& z_odd)
{
    const float u1 = fmaf((float)(ra >> 8), 0x1p-24f, 0x1p-24f);     // ((ra>>8)+1) 2^-24 in (0, 1], exact
    const float u2 = (float)(rb >> 8) * 0x1p-24f;                    // [0, 1), exact
    const float rad2 = __builtin_amdgcn_logf(u1) * -1.3862943611198906f;  // -2 ln u1 = -2 ln2 log2 u1
    const float rad = __builtin_amdgcn_sqrtf(rad2);
    z_even = rad * __builtin_amdgcn_cosf(u2);
    z_odd = rad * __builtin_amdgcn_sinf(u2);
}

__device__ __forceinline__ void gauss4_fast(uint32_t k0, uint32_t k1, uint32_t index, uint32_t blk,
                                            uint32_t t, uint32_t tag, float z[4])
{
    const U4 r = philox4x32_10(index, blk, t, tag << 24, k0, k1);
    box_muller_fast(r.x, r.y, z[0], z[1]);
    box_muller_fast(r.z, r.w, z[2], z[3]);
}

// The same four Gaussians divided by sqrt(2 ln 2): the radius is sqrt(-log2 u1) as the
// transcendental unit delivers it, and the caller folds the constant into its own scale factor
// (one multiplication less per pair).
constexpr float kGaussUnitScale = 1.1774100225154747f;               // sqrt(2 ln 2)
__device__ __forceinline__ void box_muller_unit(uint32_t ra, uint32_t rb, float& z_even, float& z_odd)
{
    const float u1 = fmaf((float)(ra >> 8), 0x1p-24f, 0x1p-24f);
    const float u2 = (float)(rb >> 8) * 0x1p-24f;
    const float rad = __builtin_amdgcn_sqrtf(-__builtin_amdgcn_logf(u1));
    z_even = rad * __builtin_amdgcn_cosf(u2);
    z_odd = rad * __builtin_amdgcn_sinf(u2);
}

__device__ __forceinline__ void gauss4_unit(uint32_t k0, uint32_t k1, uint32_t index, uint32_t blk, uint32_t t,
                                            uint32_t tag, float z[4])
{
    const U4 r = philox4x32_10(index, blk, t, tag << 24, k0, k1);
    box_muller_unit(r.x, r.y, z[0], z[1]);
    box_muller_unit(r.z, r.w, z[2], z[3]);
}

// Accurate variant (fp64 library functions, one rounding to fp32); used off the hot path,
// at tile creation, so that the per-cell planes carry no approximation error.
__device__ __forceinline__ void gauss4_accurate(uint32_t k0, uint32_t k1, uint32_t index, uint32_t blk,
                                                uint32_t t, uint32_t tag, float z[4])
{
    const U4 r = philox4x32_10(index, blk, t, tag << 24, k0, k1);
    const uint32_t w[4] = {r.x, r.y, r.z, r.w};
    const double two_pi = 6.283185307179586476925286766559;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const double u1 = ((double)(w[2 * p] >> 8) + 1.0) / 16777216.0;
        const double u2 = (double)(w[2 * p + 1] >> 8) / 16777216.0;
        const double rad = sqrt(-2.0 * log(u1));
        z[2 * p] = (float)(rad * cos(two_pi * u2));
        z[2 * p + 1] = (float)(rad * sin(two_pi * u2));
    }
}

}  // namespace aht
