// Epilogue shared by the matrix-core convolution kernels: what happens to the 32-bit sums of
// Eq. 6 after the last product - (bias is already in the accumulator) ReLU, one rounding
// shift by f_in + f_w - f_out, clamp to [-127, 127], pack, store - all in registers.
#pragma once
#include "dfq_device.hpp"
#include "dfq_host.hpp"

namespace dfq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// The epilogue forms below read the accumulators with instructions inside inline assembly.  The compiler's hazard
// pass inserts the wait states a vector instruction needs behind a matrix instruction that writes its operand (up to
// 19 for the 16-pass int8 forms) only for instructions it can see, so a kernel calls this once between the last
// matrix instruction of a tile and the tile's epilogue: every accumulator passes through a statement that is ordered
// behind the wait, and the wait behind the statements that follow the matrix instructions.
template <int N, typename Acc>
__device__ __forceinline__ void settle_accumulators(Acc *acc)
{
#pragma unroll
    for (int i = 1; i < N; i++) asm volatile("" : "+v"(acc[i]));
    asm volatile("s_nop 15\n\ts_nop 3" : "+v"(acc[0]));
#pragma unroll
    for (int i = 1; i < N; i++) asm volatile("" : "+v"(acc[i]));
}

// Per-launch constants of the requantization.  For 0 <= shift <= 23 the fast form is used:
// the sum is first clamped to +-127 * 2^shift (anything beyond saturates to +-127 anyway; with
// ReLU the lower bound is 0), which makes  (v + 2^(shift-1) - 1 + bit_shift(v)) >> shift
// overflow-free and its result lie in [-127, 127] without a second clamp; that expression is
// round-half-even of v / 2^shift for two's complement v.  With shift == 0 nothing is rounded:
// the added constant is 0 and the rounding bit is read with a field width of 0, i.e. as 0.
struct Requant {
    int shift;
    int relu;
    int lo, hi;      // pre-clamp bounds (fast form)
    int bias_add;    // 2^(shift-1) - 1
    unsigned odd_width;   // width of the field that holds bit `shift` of the sum: 1, or 0 when shift == 0
    bool fast;

    __device__ __forceinline__ void init(int s, int r)
    {
        shift = s;
        relu = r;
        fast = s >= 0 && s <= 23;
        hi = fast ? (127 << s) : 0;
        lo = fast ? (r ? 0 : -(127 << s)) : 0;
        bias_add = (fast && s > 0) ? ((1 << (s - 1)) - 1) : 0;
        odd_width = s > 0 ? 1u : 0u;
    }
    __device__ __forceinline__ int fast_one(int v) const
    {
        asm("v_med3_i32 %0, %1, %2, %3" : "=v"(v) : "v"(v), "s"(lo), "v"(hi));   // clamp to [lo, hi] (lo <= hi)
        const int odd = (int)__builtin_amdgcn_ubfe((unsigned)v, (unsigned)shift, odd_width);
        return (v + bias_add + odd) >> shift;                      // v_add3_u32, v_ashrrev_i32
    }
    // The same for four sums at once, the four results packed into one word of int8: the final
    // shift writes its low byte straight into byte i of the word (sub-dword destination select).
    __device__ __forceinline__ uint32_t fast_four(int v0, int v1, int v2, int v3) const
    {
        int t[4] = {v0, v1, v2, v3};
#pragma unroll
        for (int i = 0; i < 4; i++) {
            asm("v_med3_i32 %0, %1, %2, %3" : "=v"(t[i]) : "v"(t[i]), "s"(lo), "v"(hi));
            t[i] = t[i] + bias_add + (int)__builtin_amdgcn_ubfe((unsigned)t[i], (unsigned)shift, odd_width);
        }
        uint32_t w;
        asm("v_ashrrev_i32_sdwa %0, %1, %2 dst_sel:BYTE_0 dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:DWORD" : "=v"(w) : "v"(shift), "v"(t[0]));
        asm("v_ashrrev_i32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD" : "+v"(w) : "v"(shift), "v"(t[1]));
        asm("v_ashrrev_i32_sdwa %0, %1, %2 dst_sel:BYTE_2 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD" : "+v"(w) : "v"(shift), "v"(t[2]));
        asm("v_ashrrev_i32_sdwa %0, %1, %2 dst_sel:BYTE_3 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD" : "+v"(w) : "v"(shift), "v"(t[3]));
        return w;
    }
    __device__ __forceinline__ int slow_one(int v) const { return requant8(relu ? max(v, 0) : v, shift); }
};

// four values in [-127, 127] -> one word of four int8
__device__ __forceinline__ uint32_t pack4_clamped(int a, int b, int c, int d)
{
    const uint32_t lo = __builtin_amdgcn_perm((uint32_t)b, (uint32_t)a, 0x0c0c0400u);   // {a.b0, b.b0, 0, 0}
    const uint32_t hi = __builtin_amdgcn_perm((uint32_t)d, (uint32_t)c, 0x0c0c0400u);
    return __builtin_amdgcn_perm(hi, lo, 0x05040100u);                                  // {lo.b0, lo.b1, hi.b0, hi.b1}
}

// One lane's share of a 32x32 accumulator tile: 16 consecutive output channels kc..kc+15 of
// pixel m.  `v` already contains the bias.  Hot form: whole 16-channel group inside K, aligned
// output row, shift in the fast range, no accumulator dump.
__device__ __forceinline__ uint4 requant_tile_lane_fast(const v16i &v, const Requant &rq)
{
    return make_uint4(rq.fast_four(v[0], v[1], v[2], v[3]), rq.fast_four(v[4], v[5], v[6], v[7]),
                      rq.fast_four(v[8], v[9], v[10], v[11]), rq.fast_four(v[12], v[13], v[14], v[15]));
}
// The hot form with one weight format per output channel: the four sums belong to four channels,
// each with its own shift s in [0, 23]; hi = 127 << s, badd = 2^(s-1) - 1 (0 for s = 0) come from a
// per-channel table.  Same four instructions per value as the uniform form, operands in registers.
__device__ __forceinline__ uint32_t requant_four_per_channel(int v0, int v1, int v2, int v3, const int4 &s, const int4 &hi,
                                                             const int4 &badd, int relu)
{
    int t[4] = {v0, v1, v2, v3};
    const int sv[4] = {s.x, s.y, s.z, s.w}, hv[4] = {hi.x, hi.y, hi.z, hi.w}, bv[4] = {badd.x, badd.y, badd.z, badd.w};
#pragma unroll
    for (int i = 0; i < 4; i++) {
        const int lo = relu ? 0 : -hv[i];
        asm("v_med3_i32 %0, %1, %2, %3" : "=v"(t[i]) : "v"(t[i]), "v"(lo), "v"(hv[i]));
        t[i] = t[i] + bv[i] + (int)__builtin_amdgcn_ubfe((unsigned)t[i], (unsigned)sv[i], (unsigned)min(sv[i], 1));
    }
    uint32_t w;
    asm("v_ashrrev_i32_sdwa %0, %1, %2 dst_sel:BYTE_0 dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:DWORD" : "=v"(w) : "v"(sv[0]), "v"(t[0]));
    asm("v_ashrrev_i32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD" : "+v"(w) : "v"(sv[1]), "v"(t[1]));
    asm("v_ashrrev_i32_sdwa %0, %1, %2 dst_sel:BYTE_2 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD" : "+v"(w) : "v"(sv[2]), "v"(t[2]));
    asm("v_ashrrev_i32_sdwa %0, %1, %2 dst_sel:BYTE_3 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD" : "+v"(w) : "v"(sv[3]), "v"(t[3]));
    return w;
}

// One sum of a channel with its own shift s in [0, 23] (hi = 127 << s, badd = 2^(s-1) - 1, or 0 for s = 0).
__device__ __forceinline__ int requant_one_per_channel(int v, int s, int hi, int badd, int relu)
{
    const int lo = relu ? 0 : -hi;
    asm("v_med3_i32 %0, %1, %2, %3" : "=v"(v) : "v"(v), "v"(lo), "v"(hi));
    return (v + badd + (int)__builtin_amdgcn_ubfe((unsigned)v, (unsigned)s, (unsigned)min(s, 1))) >> s;
}

// Rescale of one channel whose shift is only known at run time: the four-instruction form when the shift
// lies in [0, 23], the general rounding otherwise.
struct ChannelRequant {
    int s, hi, badd;
    bool fast;
    __device__ __forceinline__ void init(int shift)
    {
        s = shift;
        fast = (unsigned)shift <= 23u;
        hi = 127 << (fast ? shift : 0);
        badd = (fast && shift > 0) ? ((1 << (shift - 1)) - 1) : 0;
    }
    __device__ __forceinline__ int apply(int v, int relu) const
    {
        return fast ? requant_one_per_channel(v, s, hi, badd, relu) : requant8(relu ? max(v, 0) : v, s);
    }
};

// Four channels' sums rescaled per channel, then the fused add of Eq. 10 with the four codes in `other`.
__device__ __forceinline__ uint32_t requant_add_four_per_channel(int v0, int v1, int v2, int v3, const int4 &s, const int4 &hi,
                                                                 const int4 &badd, int relu, uint32_t other, int sa, int sb,
                                                                 const Requant &rq2)
{
    const int v[4] = {v0, v1, v2, v3};
    const int sv[4] = {s.x, s.y, s.z, s.w}, hv[4] = {hi.x, hi.y, hi.z, hi.w}, bv[4] = {badd.x, badd.y, badd.z, badd.w};
    int t[4];
#pragma unroll
    for (int e = 0; e < 4; e++)
        t[e] = (int)((unsigned)requant_one_per_channel(v[e], sv[e], hv[e], bv[e], relu) << sa) + (int)((unsigned)byte_of(other, e) << sb);
    return rq2.fast_four(t[0], t[1], t[2], t[3]);
}

// The same followed by the fused add of Eq. 10: the sixteen int8 results of the convolution (kept as
// integers, never stored) and the sixteen codes of the second operand in `other` are aligned to the
// finer of their two scales, summed and rounded once more with rq2.
__device__ __forceinline__ uint4 requant_add_tile_lane(const v16i &v, const Requant &rq, const v4i &other, int sa, int sb,
                                                       const Requant &rq2)
{
    uint32_t out[4];
#pragma unroll
    for (int j = 0; j < 4; j++) {
        int t[4];
#pragma unroll
        for (int e = 0; e < 4; e++)
            t[e] = (int)((unsigned)rq.fast_one(v[4 * j + e]) << sa) + (int)((unsigned)byte_of((uint32_t)other[j], e) << sb);
        out[j] = rq2.fast_four(t[0], t[1], t[2], t[3]);
    }
    return make_uint4(out[0], out[1], out[2], out[3]);
}
// The single-rounding form of convolution + add: the accumulators themselves (at f_in + f_w, not rounded to a format of
// their own) and the second operand's codes shifted left to that scale are summed and rounded once with rq2.  The
// accumulator is first clamped to +-(127 * 2^23 + 2^29): |other << sb| <= 2^29 (sb <= 22), so beyond that bound the sum
// saturates whatever the second operand holds, and inside it the 32-bit sum cannot overflow.  7 instructions per output.
__device__ __forceinline__ uint4 add_tile_lane_lazy(const v16i &v, const v4i &other, int sb, const Requant &rq2)
{
    constexpr int kBound = (127 << 23) + (1 << 29);
    uint32_t out[4];
#pragma unroll
    for (int j = 0; j < 4; j++) {
        int t[4];
#pragma unroll
        for (int e = 0; e < 4; e++)
            t[e] = max(-kBound, min(kBound, v[4 * j + e])) + (int)((unsigned)byte_of((uint32_t)other[j], e) << sb);
        out[j] = rq2.fast_four(t[0], t[1], t[2], t[3]);
    }
    return make_uint4(out[0], out[1], out[2], out[3]);
}
__device__ __forceinline__ void store_tile_lane_fast(const v16i &v, const ConvArgs &a, const Requant &rq, long long m, int kc)
{
    *(uint4 *)(a.y + (size_t)m * a.ldy + kc) = requant_tile_lane_fast(v, rq);
}

// General form (ragged channel tail, unaligned rows, extreme shifts, accumulator dump, one weight
// format per output channel).
__device__ __forceinline__ void store_tile_lane_general(const v16i &v, const ConvArgs &a, int shift, int relu, long long m, int kc)
{
    // a whole 16-channel group into an aligned row, no accumulator dump: any shifts, one 16-byte store
    if (!a.acc_out && a.y && kc + 16 <= a.K && (((unsigned)a.ldy | (unsigned)kc) & 15u) == 0 && ((uintptr_t)a.y & 15) == 0) {
        uint32_t o[4];
#pragma unroll
        for (int j = 0; j < 4; j++) {
            int q[4];
#pragma unroll
            for (int e = 0; e < 4; e++) {
                const int r = 4 * j + e;
                ChannelRequant cr;
                cr.init(a.frac_w ? shift + a.frac_w[kc + r] : shift);
                q[e] = cr.apply(v[r], relu);
            }
            o[j] = pack4_clamped(q[0], q[1], q[2], q[3]);
        }
        *(uint4 *)(a.y + (size_t)m * a.ldy + kc) = make_uint4(o[0], o[1], o[2], o[3]);
        return;
    }
#pragma unroll
    for (int r = 0; r < 16; r++) {
        if (kc + r < a.K) {
            const int val = v[r];
            if (a.acc_out) a.acc_out[(size_t)m * a.K + kc + r] = val;
            const int s = a.frac_w ? shift + a.frac_w[kc + r] : shift;
            if (a.y) a.y[(size_t)m * a.ldy + kc + r] = (int8_t)requant8(relu ? max(val, 0) : val, s);
        }
    }
}

// One weight format per output channel with the lane's 16 shifts already in registers: whole 16-channel
// group, aligned row, no accumulator dump - one 16-byte store, no loads.
__device__ __forceinline__ void store_tile_lane_per_channel(const v16i &v, const ConvArgs &a, const int (&shifts)[16], int relu,
                                                            long long m, int kc)
{
    uint32_t o[4];
#pragma unroll
    for (int j = 0; j < 4; j++) {
        int q[4];
#pragma unroll
        for (int e = 0; e < 4; e++) {
            ChannelRequant cr;
            cr.init(shifts[4 * j + e]);
            q[e] = cr.apply(v[4 * j + e], relu);
        }
        o[j] = pack4_clamped(q[0], q[1], q[2], q[3]);
    }
    *(uint4 *)(a.y + (size_t)m * a.ldy + kc) = make_uint4(o[0], o[1], o[2], o[3]);
}

// the conditions of store_tile_lane_per_channel for a block whose channel range ends at k_end
__device__ __forceinline__ bool epilogue_is_per_channel_packed(const ConvArgs &a, int k_end)
{
    return a.frac_w && !a.acc_out && a.y && ((a.ldy & 15) == 0) && (((uintptr_t)a.y & 15) == 0) && k_end <= a.K;
}

// true when every tile of a launch can take the hot form (k_end = end of the block's channel range)
__device__ __forceinline__ bool epilogue_is_fast(const ConvArgs &a, const Requant &rq, int k_end)
{
    return rq.fast && !a.frac_w && !a.acc_out && a.y && ((a.ldy & 15) == 0) && (((uintptr_t)a.y & 15) == 0) && k_end <= a.K;
}

// Bias of channels kc..kc+15 (zeros where there is no bias or past K).
__device__ __forceinline__ void load_bias16(const ConvArgs &a, int kc, int (&bv)[16])
{
    if (a.b && kc + 16 <= a.K && (((uintptr_t)a.b & 15) == 0) && (kc & 3) == 0) {
#pragma unroll
        for (int r = 0; r < 16; r += 4) {
            const int4 t = *(const int4 *)(a.b + kc + r);
            bv[r] = t.x; bv[r + 1] = t.y; bv[r + 2] = t.z; bv[r + 3] = t.w;
        }
    } else {
        for (int r = 0; r < 16; r++) bv[r] = (a.b && kc + r < a.K) ? a.b[kc + r] : 0;
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
