// Epilogue shared by the matrix-core convolution kernels: what happens to the 32-bit sums of
// Eq. 6 after the last product - (bias is already in the accumulator) ReLU, one rounding
// shift by f_in + f_w - f_out, clamp to [-127, 127], pack, store - all in registers.
#pragma once
#include "dfq_device.hpp"
#include "dfq_host.hpp"

namespace dfq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// Per-launch constants of the requantization.  For 1 <= shift <= 23 the fast form is used:
// the sum is first clamped to +-2^(shift+7) (anything beyond saturates anyway; with ReLU the
// lower bound is 0), which makes  (v + 2^(shift-1) - 1 + bit_shift(v)) >> shift  overflow-free;
// that expression is round-half-even of v / 2^shift for two's complement v.
struct Requant {
    int shift;
    int relu;
    int lo, hi;      // pre-clamp bounds (fast form)
    int bias_add;    // 2^(shift-1) - 1
    bool fast;

    __device__ __forceinline__ void init(int s, int r)
    {
        shift = s;
        relu = r;
        fast = s >= 1 && s <= 23;
        hi = fast ? (128 << s) : 0;
        lo = fast ? (r ? 0 : -(128 << s)) : 0;
        bias_add = fast ? ((1 << (s - 1)) - 1) : 0;
    }
    __device__ __forceinline__ int fast_one(int v) const
    {
        v = max(lo, min(v, hi));
        int odd = (v >> shift) & 1;
        int t = (v + bias_add + odd) >> shift;
        return max(-127, min(t, 127));
    }
    __device__ __forceinline__ int slow_one(int v) const { return requant8(relu ? max(v, 0) : v, shift); }
};

__device__ __forceinline__ uint32_t pack4_clamped(int a, int b, int c, int d)
{
    // inputs already in [-127, 127]
    uint32_t lo = (uint32_t)(a & 0xff) | ((uint32_t)(b & 0xff) << 8);
    uint32_t hi = (uint32_t)(c & 0xff) | ((uint32_t)d << 8);
    return lo | (hi << 16);
}

// One lane's share of a 32x32 accumulator tile: 16 consecutive output channels kc..kc+15 of
// pixel m.  `v` already contains the bias.
__device__ __forceinline__ void store_tile_lane(const v16i &v, const ConvArgs &a, const Requant &rq, long long m, int kc,
                                                bool vec_ok)
{
    const bool full = kc + 16 <= a.K;
    if (a.acc_out) {
        int32_t *dst = a.acc_out + (size_t)m * a.K + kc;
        if (full && (a.K & 3) == 0) {
#pragma unroll
            for (int r = 0; r < 16; r += 4) *(int4 *)(dst + r) = make_int4(v[r], v[r + 1], v[r + 2], v[r + 3]);
        } else {
#pragma unroll
            for (int r = 0; r < 16; r++)
                if (kc + r < a.K) dst[r] = v[r];
        }
    }
    if (a.y) {
        int o[16];
        if (rq.fast) {
#pragma unroll
            for (int r = 0; r < 16; r++) o[r] = rq.fast_one(v[r]);
        } else {
#pragma unroll
            for (int r = 0; r < 16; r++) o[r] = rq.slow_one(v[r]);
        }
        int8_t *dst = a.y + (size_t)m * a.ldy + kc;
        if (full && vec_ok) {
            *(uint4 *)dst = make_uint4(pack4_clamped(o[0], o[1], o[2], o[3]), pack4_clamped(o[4], o[5], o[6], o[7]),
                                       pack4_clamped(o[8], o[9], o[10], o[11]), pack4_clamped(o[12], o[13], o[14], o[15]));
        } else {
#pragma unroll
            for (int r = 0; r < 16; r++)
                if (kc + r < a.K) dst[r] = (int8_t)o[r];
        }
    }
}

// exact n / d for 0 <= n < 2^31 by one multiply-high: mul = floor(2^(31+s) / d) + 1 with
// s = ceil(log2 d) >= 1 (d == 1 is flagged by s == 0).
struct FastDiv {
    uint32_t mul;
    int s;
    int d;
};

inline FastDiv make_fastdiv(int d)
{
    FastDiv f;
    f.d = d;
    if (d == 1) { f.mul = 0; f.s = 0; return f; }
    int s = 0;
    while ((1LL << s) < d) s++;
    f.s = s;
    f.mul = (uint32_t)(((1ULL << (31 + s)) / (unsigned long long)d) + 1ULL);
    return f;
}

__device__ __forceinline__ int fastdiv(int n, const FastDiv &f)
{
    if (f.s == 0) return n;
    return (int)(__umulhi((uint32_t)n, f.mul) >> (f.s - 1));
}

}  // namespace dfq
