// Device-side generator of the measurement matrix entries (paper Sec. 4.3: iid zero-mean
// normal entries with standard deviation 1/sqrt(r)), from a counter-based stream so that A
// never has to sit in HBM.
//
// Philox4x32-10 (Salmon et al., SC'11): key = (seed low, seed high), counter = (i, j/4, 0, 0)
// -> four words for rows 4*(j/4)..+3 of column i of A. Words (0,1) and (2,3) each feed one
// Box-Muller pair. The float transform uses only exactly rounded operations (fused
// multiply-add, multiply, subtract, square root) in a fixed order, so any IEEE-754 machine
// produces the same bits.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sgc {

struct u32x4 {
    uint32_t x, y, z, w;
};

__device__ __forceinline__ u32x4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t k0, uint32_t k1)
{
    uint32_t c2 = 0u, c3 = 0u;
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint64_t pa = (uint64_t)c0 * 0xD2511F53ull;
        const uint64_t pb = (uint64_t)c2 * 0xCD9E8D57ull;
        const uint32_t t0 = (uint32_t)(pb >> 32) ^ c1 ^ k0;
        const uint32_t t2 = (uint32_t)(pa >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)pb;
        c3 = (uint32_t)pa;
        c0 = t0;
        c2 = t2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return u32x4{c0, c1, c2, c3};
}

#pragma clang fp contract(off)

// -2 ln(n * 2^-24) for an odd integer n in [1, 2^24)
__device__ __forceinline__ float minus_two_log_of_unit(uint32_t n)
{
    const float f = (float)n;
    const uint32_t bits = __float_as_uint(f);
    int e = (int)(bits >> 23) - 127 - 24;
    const uint32_t frac = bits & 0x007fffffu;
    const bool upper = frac > 0x003504f3u; // mantissa above sqrt(2): use m/2 and e+1
    const float m = __uint_as_float(frac | (upper ? 0x3f000000u : 0x3f800000u));
    e += upper ? 1 : 0;
    const float s = m - 1.0f;
    float h = -0x1.4237fep-4f;
    h = __builtin_fmaf(h, s, 0x1.0696e4p-3f);
    h = __builtin_fmaf(h, s, -0x1.0c524cp-3f);
    h = __builtin_fmaf(h, s, 0x1.22973ap-3f);
    h = __builtin_fmaf(h, s, -0x1.548882p-3f);
    h = __builtin_fmaf(h, s, 0x1.99a3ecp-3f);
    h = __builtin_fmaf(h, s, -0x1.000206p-2f);
    h = __builtin_fmaf(h, s, 0x1.55554ep-2f);
    h = __builtin_fmaf(h, s, -0x1.fffffep-2f);
    const float ss = s * s;
    const float log_m = __builtin_fmaf(ss, h, s);
    const float log_u = __builtin_fmaf((float)e, 0x1.62e430p-1f, log_m);
    return -2.0f * log_u;
}

// cosine and sine of oct*pi/4 + (pi/4)*(f+0.5)/2^23 (oct = top 3 bits of w, f = next 23 bits)
__device__ __forceinline__ void octant_cos_sin(uint32_t w, float &co, float &si)
{
    const uint32_t oct = w >> 29;
    uint32_t n = (((w >> 6) & 0x007fffffu) << 1) | 1u;
    n = (oct & 1u) ? (0x01000000u - n) : n;
    const float ph = (float)n * 0x1.0p-24f;
    const float u = ph * ph;
    float ps = -0x1.2d9b7cp-15f;
    ps = __builtin_fmaf(ps, u, 0x1.465ec4p-9f);
    ps = __builtin_fmaf(ps, u, -0x1.4abbbap-4f);
    ps = __builtin_fmaf(ps, u, 0x1.921fb6p-1f);
    const float sn = ps * ph;
    float cs = -0x1.4e5e6ep-12f;
    cs = __builtin_fmaf(cs, u, 0x1.03af5ap-6f);
    cs = __builtin_fmaf(cs, u, -0x1.3bd392p-2f);
    cs = __builtin_fmaf(cs, u, 1.0f);
    const bool swap = ((oct + 1u) & 2u) != 0u;
    float c = swap ? sn : cs;
    float s = swap ? cs : sn;
    c = ((oct + 2u) & 4u) ? -c : c;
    s = (oct & 4u) ? -s : s;
    co = c;
    si = s;
}

__device__ __forceinline__ void normal_pair(uint32_t w0, uint32_t w1, float scale, float &z0, float &z1)
{
    const float t = minus_two_log_of_unit(((w0 >> 9) << 1) | 1u);
    const float rad = sqrtf(t) * scale;
    float c, s;
    octant_cos_sin(w1, c, s);
    z0 = rad * c;
    z1 = rad * s;
}

// A[4*jb .. 4*jb+3][i] (= At[i][4*jb..4*jb+3])
__device__ __forceinline__ float4 matrix_quad(uint32_t i, uint32_t jb, uint32_t k0, uint32_t k1, float scale)
{
    const u32x4 w = philox4x32_10(i, jb, k0, k1);
    float4 o;
    normal_pair(w.x, w.y, scale, o.x, o.y);
    normal_pair(w.z, w.w, scale, o.z, o.w);
    return o;
}

} // namespace sgc
