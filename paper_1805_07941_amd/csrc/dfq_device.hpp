// Device-side arithmetic shared by every dfq kernel: the power-of-two requantization
// (rescale by alpha_x*alpha_y/alpha_z of Eq. 6 when all scales are powers of two), the
// symmetric clamp of Sec. 2.2, and small wavefront helpers.  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dfq {

constexpr int kWave = 64;

// clamp to [-beta_max, beta_max] = [-127, 127]
__device__ __forceinline__ int sat8(int t) { return max(-127, min(127, t)); }

// sat8(v * 2^-s, rounded to nearest, ties to even) for any 32-bit v and any integer s.
//   s <= 0 : exact multiplication, then clamp (|v| is clamped first so the product fits);
//   1..31  : floor shift, then one increment decided from the discarded bits;
//   >= 32  : |v| * 2^-32 <= 1/2 and a tie goes to the even neighbour 0.
__device__ __forceinline__ int requant8(int v, int s)
{
    if (s <= 0) {
        int c = sat8(v);
        int k = -s;
        if (k >= 8) return c == 0 ? 0 : (c > 0 ? 127 : -127);
        return sat8(c << k);
    }
    if (s >= 32) return 0;
    int t = v >> s;                                   // floor
    uint32_t rem = (uint32_t)v & ((1u << s) - 1u);    // v - t*2^s, in [0, 2^s)
    uint32_t half = 1u << (s - 1);
    t += (rem > half || (rem == half && (t & 1))) ? 1 : 0;
    return sat8(t);
}

// Variant for a shift known to lie in [1, 31] (the common case inside conv epilogues).
__device__ __forceinline__ int requant8_rshift(int v, int s, uint32_t mask, uint32_t half)
{
    int t = v >> s;
    uint32_t rem = (uint32_t)v & mask;
    t += (rem > half || (rem == half && (t & 1))) ? 1 : 0;
    return sat8(t);
}

__device__ __forceinline__ uint32_t pack4(int a, int b, int c, int d)
{
    return (uint32_t)(a & 0xff) | ((uint32_t)(b & 0xff) << 8) | ((uint32_t)(c & 0xff) << 16) | ((uint32_t)d << 24);
}

__device__ __forceinline__ int byte_of(uint32_t w, int i)  // sign-extended byte i of w
{
    return (int)(w << (24 - 8 * i)) >> 24;
}

__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = max(v, (uint32_t)__shfl_xor((int)v, off, kWave));
    return v;
}

}  // namespace dfq
