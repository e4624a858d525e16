// C-ABI of libdfq: argument validation, kernel selection and the pure host functions.
// Declarations and the contract of every call are in include/dfq.h.
#include "dfq.h"

#include <cmath>

#include "dfq_host.hpp"

using namespace dfq;

namespace {

inline bool fmt_ok(dfq_fmt f) { return f.bits == 8 && f.frac >= -32 && f.frac <= 32; }

inline bool overlaps(const void *a, size_t na, const void *b, size_t nb)
{
    if (!a || !b || !na || !nb) return false;
    uintptr_t pa = (uintptr_t)a, pb = (uintptr_t)b;
    return pa < pb + nb && pb < pa + na;
}

inline dfq_status from_hip(hipError_t e) { return e == hipSuccess ? DFQ_OK : DFQ_EDEVICE; }

inline int out_extent(int in, int pad, int k, int stride)
{
    long long span = (long long)in + 2LL * pad - k;
    if (span < 0) return 0;
    return (int)(span / stride) + 1;
}

// smallest q with 2^(q-1) >= m
int width_for(unsigned long long m)
{
    int q = 1;
    unsigned long long pw = 1;
    while (pw < m) { pw <<= 1; q++; }
    return q;
}

struct ConvCheck {
    dfq_status st;
    ConvArgs a;
};

ConvCheck check_conv(const int8_t *x, const int8_t *w, const int32_t *b, int8_t *y, int32_t *acc_out, int N, int H, int W,
                     int C, int K, int R, int S, int stride, int pad, int groups, int ldy, dfq_fmt fi, dfq_fmt fw,
                     dfq_fmt fo, int relu, bool need_ptrs)
{
    ConvCheck r{};
    r.st = DFQ_OK;
    if (need_ptrs && (!x || !w || (!y && !acc_out))) { r.st = DFQ_EINVAL; return r; }
    if (N < 0) { r.st = DFQ_EINVAL; return r; }
    if (H < 1 || W < 1 || C < 1 || K < 1 || R < 1 || S < 1 || stride < 1 || pad < 0 || groups < 1) { r.st = DFQ_ESHAPE; return r; }
    if (C % groups || K % groups) { r.st = DFQ_ESHAPE; return r; }
    int P = out_extent(H, pad, R, stride), Q = out_extent(W, pad, S, stride);
    if (P < 1 || Q < 1) { r.st = DFQ_ESHAPE; return r; }
    if (need_ptrs && y && ldy < K) { r.st = DFQ_ESHAPE; return r; }
    if (!fmt_ok(fi) || !fmt_ok(fw) || !fmt_ok(fo)) { r.st = DFQ_EFMT; return r; }
    long long kgemm = (long long)R * S * (C / groups);
    // Eq. 9 with q = 32 and codes that may reach -128: the longest exact sum of products
    if (kgemm > dfq_mac_max_len(32, 127, 1, 127, 1)) { r.st = DFQ_EUNSUPPORTED; return r; }
    if ((long long)H * W * C >= (1LL << 31) || (long long)P * Q * (long long)(ldy > K ? ldy : K) >= (1LL << 31)) {
        r.st = DFQ_EUNSUPPORTED;   // one image must be addressable with 32-bit offsets
        return r;
    }
    r.a = ConvArgs{x, w, b, y, acc_out, N, H, W, C, K, R, S, stride, pad, groups, P, Q, ldy, fi.frac + fw.frac - fo.frac,
                   relu ? 1 : 0};
    if (need_ptrs) {
        size_t nx = (size_t)N * H * W * C, npix = (size_t)N * P * Q;
        if (overlaps(x, nx, y, npix * (size_t)ldy) || overlaps(x, nx, acc_out, npix * K * 4)) r.st = DFQ_EINVAL;
    }
    return r;
}

// geometry_only: the pointers, row pitch and shift of `a` are placeholders
dfq_conv_variant select_variant(const ConvArgs &a, bool geometry_only = false)
{
    if (conv_depthwise_supports(a)) return DFQ_CONV_DEPTHWISE;
    if (geometry_only ? conv_pw_geometry_ok(a) : conv_pw_supports(a)) return DFQ_CONV_POINTWISE;
    if (conv_mfma_supports(a)) return DFQ_CONV_MFMA;
    if (conv_smallc_supports(a)) return DFQ_CONV_SMALLC;
    if (conv_grouped_supports(a)) return DFQ_CONV_GROUPED;
    return DFQ_CONV_DIRECT;
}

dfq_status run_conv(dfq_conv_variant variant, const ConvArgs &a, hipStream_t st)
{
    if (variant == DFQ_CONV_AUTO) variant = select_variant(a);
    switch (variant) {
        case DFQ_CONV_DIRECT:
            return from_hip(launch_conv_direct(a, st));
        case DFQ_CONV_MFMA:
            if (!conv_mfma_supports(a)) return DFQ_EUNSUPPORTED;
            return from_hip(launch_conv_mfma(a, st));
        case DFQ_CONV_DEPTHWISE:
            if (!conv_depthwise_supports(a)) return DFQ_EUNSUPPORTED;
            return from_hip(launch_conv_depthwise(a, st));
        case DFQ_CONV_POINTWISE:
            if (!conv_pw_supports(a)) return DFQ_EUNSUPPORTED;
            return from_hip(launch_conv_pw(a, st));
        case DFQ_CONV_SMALLC:
            if (!conv_smallc_supports(a)) return DFQ_EUNSUPPORTED;
            if (conv_stem_supports(a, false)) return from_hip(launch_conv_stem(a, nullptr, 0, st));
            return from_hip(launch_conv_smallc(a, st));
        case DFQ_CONV_GROUPED:
            if (!conv_grouped_supports(a)) return DFQ_EUNSUPPORTED;
            return from_hip(launch_conv_grouped(a, st));
        default:
            return DFQ_EINVAL;
    }
}

// the part of the fused convolution + add calls behind the convolution's own checks
dfq_status run_conv_add(ConvCheck &c, const int8_t *x, const int8_t *other, int8_t *y, int N, int H, int W, int C, int K,
                        int ldy, int ld_other, dfq_fmt fmt_mid, dfq_fmt fmt_other, dfq_fmt fmt_out, int relu_out,
                        dfq_stream stream)
{
    if (c.st != DFQ_OK) return c.st;
    if (!fmt_ok(fmt_other) || !fmt_ok(fmt_out)) return DFQ_EFMT;
    if (!y || !other) return DFQ_EINVAL;
    if (ld_other < K) return DFQ_ESHAPE;
    const int F = fmt_mid.frac > fmt_other.frac ? fmt_mid.frac : fmt_other.frac;
    // Eq. 12: two codes of magnitude <= 2^7 shifted by <= 22 bits sum to at most 2^30
    if (F - fmt_mid.frac > 22 || F - fmt_other.frac > 22) return DFQ_EFMT;
    if (N == 0) return DFQ_OK;
    const size_t npix = (size_t)N * c.a.P * c.a.Q;
    if (overlaps(other, npix * (size_t)ld_other, y, npix * (size_t)ldy) ||
        overlaps(other, npix * (size_t)ld_other, x, (size_t)N * H * W * C))
        return DFQ_EINVAL;
    c.a.add = other;
    c.a.ldadd = ld_other;
    c.a.add_sa = F - fmt_mid.frac;
    c.a.add_sb = F - fmt_other.frac;
    c.a.add_shift = F - fmt_out.frac;
    c.a.add_relu = relu_out ? 1 : 0;
    if (conv_pw_supports(c.a)) return from_hip(launch_conv_pw(c.a, (hipStream_t)stream));
    if (conv_mfma_fuses(c.a)) return from_hip(launch_conv_mfma(c.a, (hipStream_t)stream));
    return DFQ_EUNSUPPORTED;
}

}  // namespace

extern "C" {

const char *dfq_status_string(dfq_status s)
{
    switch (s) {
        case DFQ_OK: return "ok";
        case DFQ_EINVAL: return "invalid argument";
        case DFQ_ESHAPE: return "inconsistent shape";
        case DFQ_EFMT: return "unsupported number format";
        case DFQ_EUNSUPPORTED: return "no kernel for this request";
        case DFQ_EDEVICE: return "HIP launch failed";
    }
    return "unknown status";
}

dfq_status dfq_quantize(const float *x, int8_t *q, size_t n, dfq_fmt fmt, dfq_stream stream)
{
    if (!fmt_ok(fmt)) return DFQ_EFMT;
    if (n == 0) return DFQ_OK;
    if (!x || !q || overlaps(x, n * 4, q, n)) return DFQ_EINVAL;
    return from_hip(launch_quantize(x, q, n, fmt.frac, (hipStream_t)stream));
}

dfq_status dfq_quantize_i32(const float *x, int32_t *q, size_t n, int32_t frac, dfq_stream stream)
{
    if (frac < -64 || frac > 64) return DFQ_EFMT;
    if (n == 0) return DFQ_OK;
    if (!x || !q || overlaps(x, n * 4, q, n * 4)) return DFQ_EINVAL;
    return from_hip(launch_quantize_i32(x, q, n, frac, (hipStream_t)stream));
}

dfq_status dfq_dequantize(const int8_t *q, float *x, size_t n, dfq_fmt fmt, dfq_stream stream)
{
    if (!fmt_ok(fmt)) return DFQ_EFMT;
    if (n == 0) return DFQ_OK;
    if (!x || !q || overlaps(x, n * 4, q, n)) return DFQ_EINVAL;
    return from_hip(launch_dequantize(q, x, n, fmt.frac, (hipStream_t)stream));
}

static bool np_ok(int nbits, int p, int frac)
{
    return nbits >= 2 && nbits <= 8 && p >= 0 && p <= nbits - 1 && nbits - 1 - p <= 5 && frac >= -32 && frac <= 32;
}

dfq_status dfq_quantize_np(const float *x, uint8_t *codes, size_t n, int nbits, int p, int frac, dfq_stream stream)
{
    if (!np_ok(nbits, p, frac)) return DFQ_EFMT;
    if (n == 0) return DFQ_OK;
    if (!x || !codes || overlaps(x, n * 4, codes, n)) return DFQ_EINVAL;
    return from_hip(launch_quantize_np(x, codes, n, nbits, p, frac, (hipStream_t)stream));
}

dfq_status dfq_dequantize_np(const uint8_t *codes, float *x, size_t n, int nbits, int p, int frac, dfq_stream stream)
{
    if (!np_ok(nbits, p, frac)) return DFQ_EFMT;
    if (n == 0) return DFQ_OK;
    if (!x || !codes || overlaps(x, n * 4, codes, n)) return DFQ_EINVAL;
    return from_hip(launch_dequantize_np(codes, x, n, nbits, p, frac, (hipStream_t)stream));
}

dfq_status dfq_np_digits(const uint8_t *codes, size_t n, int p, int8_t *hi, int8_t *lo, dfq_stream stream)
{
    if (p < 4 || p > 7) return DFQ_EFMT;
    if (n == 0) return DFQ_OK;
    if (!codes || !hi || !lo) return DFQ_EINVAL;
    if (overlaps(codes, n, hi, n) || overlaps(codes, n, lo, n) || overlaps(hi, n, lo, n)) return DFQ_EINVAL;
    return from_hip(launch_np_digits(codes, n, p, hi, lo, (hipStream_t)stream));
}

dfq_status dfq_eltwise_np(const int8_t *ah, const int8_t *al, int frac_a, const int8_t *bh, const int8_t *bl, int frac_b, uint8_t *y,
                          int8_t *yh, int8_t *yl, int frac_y, int p_y, size_t n, int relu, dfq_stream stream)
{
    if (p_y < 4 || p_y > 7) return DFQ_EFMT;
    if (frac_a < -32 || frac_a > 32 || frac_b < -32 || frac_b > 32 || frac_y < -32 || frac_y > 32) return DFQ_EFMT;
    const int F = frac_a > frac_b ? frac_a : frac_b;
    // Eq. 12: two twelve-bit integers shifted by at most 18 bits sum to less than 2^31
    if (F - frac_a > 18 || F - frac_b > 18) return DFQ_EFMT;
    if (F - frac_y < -16 || F - frac_y > 31) return DFQ_EFMT;
    if (n == 0) return DFQ_OK;
    if (!ah || !al || !bh || !bl || (!y && !yh && !yl) || ((yh == nullptr) != (yl == nullptr))) return DFQ_EINVAL;
    const void *ins[4] = {ah, al, bh, bl};
    const void *outs[3] = {y, yh, yl};
    for (int i = 0; i < 3; i++) {
        for (int j = 0; j < 4; j++)
            if (overlaps(outs[i], n, ins[j], n)) return DFQ_EINVAL;
        for (int j = i + 1; j < 3; j++)
            if (overlaps(outs[i], n, outs[j], n)) return DFQ_EINVAL;
    }
    return from_hip(launch_eltwise_np(ah, al, bh, bl, y, yh, yl, n, F - frac_a, F - frac_b, F - frac_y, p_y, (int)dfq_beta_max(8, p_y),
                                      relu ? 1 : 0, (hipStream_t)stream));
}

static dfq_status check_conv_np(NpConvArgs &a, int frac_x, int frac_w, int frac_y, bool outputs = true)
{
    if (!a.xh || !a.xl || !a.wh || !a.wl || (outputs && !a.y && !a.yh && !a.yl)) return DFQ_EINVAL;
    if ((a.yh == nullptr) != (a.yl == nullptr)) return DFQ_EINVAL;
    if (a.N < 0) return DFQ_EINVAL;
    if (a.H < 1 || a.W < 1 || a.C < 1 || a.K < 1 || a.R < 1 || a.S < 1 || a.stride < 1 || a.pad < 0 || a.groups < 1) return DFQ_ESHAPE;
    if (a.C % a.groups || a.K % a.groups) return DFQ_ESHAPE;
    a.P = out_extent(a.H, a.pad, a.R, a.stride);
    a.Q = out_extent(a.W, a.pad, a.S, a.stride);
    if (a.P < 1 || a.Q < 1) return DFQ_ESHAPE;
    if (a.p_y < 4 || a.p_y > 7) return DFQ_EFMT;
    if (frac_x < -32 || frac_x > 32 || frac_w < -32 || frac_w > 32 || frac_y < -32 || frac_y > 32) return DFQ_EFMT;
    a.shift = frac_x + frac_w - frac_y;
    if (a.shift < -16 || a.shift > 48) return DFQ_EFMT;
    // Eq. 8 with the largest twelve-bit operands: the sum plus a 32-bit bias must stay below 2^62
    if ((long long)a.R * a.S * (a.C / a.groups) > (1LL << 36)) return DFQ_EUNSUPPORTED;
    if ((long long)a.H * a.W * a.C >= (1LL << 31) || (long long)a.P * a.Q * a.K >= (1LL << 31)) return DFQ_EUNSUPPORTED;
    a.beta_max = (int)dfq_beta_max(8, a.p_y);
    const size_t nx = (size_t)a.N * a.H * a.W * a.C, ny = (size_t)a.N * a.P * a.Q * a.K;
    const void *outs[3] = {a.y, a.yh, a.yl};
    for (int i = 0; i < 3; i++) {
        if (overlaps(outs[i], ny, a.xh, nx) || overlaps(outs[i], ny, a.xl, nx)) return DFQ_EINVAL;
        for (int j = i + 1; j < 3; j++)
            if (overlaps(outs[i], ny, outs[j], ny)) return DFQ_EINVAL;
    }
    return DFQ_OK;
}

dfq_status dfq_conv_np_variant(dfq_conv_variant variant, const int8_t *xh, const int8_t *xl, const int8_t *wh, const int8_t *wl,
                               const int32_t *b, uint8_t *y, int8_t *yh, int8_t *yl, int N, int H, int W, int C, int K, int R, int S,
                               int stride, int pad, int groups, int frac_x, int frac_w, int frac_y, int p_y, int relu,
                               dfq_stream stream)
{
    NpConvArgs a{xh, xl, wh, wl, b, y, yh, yl, N, H, W, C, K, R, S, stride, pad, groups, 0, 0, 0, p_y, 0, relu ? 1 : 0, nullptr, nullptr, 0, 0, 0, 0, nullptr};
    const dfq_status st = check_conv_np(a, frac_x, frac_w, frac_y);
    if (st != DFQ_OK) return st;
    if (N == 0) return DFQ_OK;
    if (variant == DFQ_CONV_AUTO) variant = conv_np_mfma_supports(a) ? DFQ_CONV_MFMA : DFQ_CONV_DIRECT;
    if (variant == DFQ_CONV_MFMA) {
        if (!conv_np_mfma_supports(a)) return DFQ_EUNSUPPORTED;
        return from_hip(launch_conv_np_mfma(a, (hipStream_t)stream));
    }
    if (variant == DFQ_CONV_DIRECT) return from_hip(launch_conv_np_direct(a, (hipStream_t)stream));
    return DFQ_EINVAL;
}

dfq_status dfq_conv_np_add(const int8_t *xh, const int8_t *xl, const int8_t *wh, const int8_t *wl, const int32_t *b, const int8_t *oh,
                           const int8_t *ol, int8_t *yh, int8_t *yl, int N, int H, int W, int C, int K, int R, int S, int stride, int pad,
                           int groups, int frac_x, int frac_w, int frac_mid, int relu_mid, int frac_other, int frac_y, int p, int relu_out,
                           dfq_stream stream)
{
    NpConvArgs a{xh, xl, wh, wl, b, nullptr, yh, yl, N, H, W, C, K, R, S, stride, pad, groups, 0, 0, 0, p, 0, relu_mid ? 1 : 0,
                 oh, ol, 0, 0, 0, relu_out ? 1 : 0, nullptr};
    if (!yh || !yl) return DFQ_EINVAL;
    const dfq_status st = check_conv_np(a, frac_x, frac_w, frac_mid);
    if (st != DFQ_OK) return st;
    if (frac_other < -32 || frac_other > 32 || frac_y < -32 || frac_y > 32) return DFQ_EFMT;
    const int F = frac_mid > frac_other ? frac_mid : frac_other;
    if (F - frac_mid > 18 || F - frac_other > 18) return DFQ_EFMT;              // Eq. 12, as for dfq_eltwise_np
    if (N == 0) return DFQ_OK;
    if (!oh || !ol) return DFQ_EINVAL;
    const size_t ny = (size_t)N * a.P * a.Q * K;
    if (overlaps(yh, ny, oh, ny) || overlaps(yh, ny, ol, ny) || overlaps(yl, ny, oh, ny) || overlaps(yl, ny, ol, ny)) return DFQ_EINVAL;
    a.add_sa = F - frac_mid;
    a.add_sb = F - frac_other;
    a.add_shift = F - frac_y;
    // the fused epilogue covers the 32-bit rounding of the layer's own result and a final factor of at most 1
    if (!conv_np_mfma_supports(a) || a.shift < 7 || a.shift > 36 || a.add_shift < 0 || a.add_shift > 31 || (((uintptr_t)oh | (uintptr_t)ol) & 15))
        return DFQ_EUNSUPPORTED;
    return from_hip(launch_conv_np_mfma(a, (hipStream_t)stream));
}

dfq_status dfq_conv_np_absmax(const int8_t *xh, const int8_t *xl, const int8_t *wh, const int8_t *wl, const int32_t *b, uint64_t *amax_dev,
                              int N, int H, int W, int C, int K, int R, int S, int stride, int pad, int groups, int relu, dfq_stream stream)
{
    if (!amax_dev || ((uintptr_t)amax_dev & 7)) return DFQ_EINVAL;
    // (the format arguments of the shared checks are placeholders: nothing is converted or stored)
    NpConvArgs a{xh, xl, wh, wl, b, nullptr, nullptr, nullptr, N, H, W, C, K, R, S, stride, pad, groups, 0, 0, 0, 4, 0, relu ? 1 : 0, nullptr, nullptr, 0, 0, 0, 0, nullptr};
    const dfq_status st = check_conv_np(a, 0, 0, 0, false);
    if (st != DFQ_OK) return st;
    a.amax = reinterpret_cast<unsigned long long *>(amax_dev);
    hipError_t e = launch_clear_u64(a.amax, (hipStream_t)stream);
    if (e != hipSuccess || N == 0) return from_hip(e);
    return from_hip(launch_conv_np_direct(a, (hipStream_t)stream));
}

dfq_status dfq_eltwise_np_absmax(const int8_t *ah, const int8_t *al, int frac_a, const int8_t *bh, const int8_t *bl, int frac_b,
                                 uint64_t *amax_dev, size_t n, int relu, dfq_stream stream)
{
    if (!amax_dev || ((uintptr_t)amax_dev & 7)) return DFQ_EINVAL;
    if (frac_a < -32 || frac_a > 32 || frac_b < -32 || frac_b > 32) return DFQ_EFMT;
    const int F = frac_a > frac_b ? frac_a : frac_b;
    if (F - frac_a > 18 || F - frac_b > 18) return DFQ_EFMT;
    if (n && (!ah || !al || !bh || !bl)) return DFQ_EINVAL;
    hipError_t e = launch_clear_u64(reinterpret_cast<unsigned long long *>(amax_dev), (hipStream_t)stream);
    if (e != hipSuccess || n == 0) return from_hip(e);
    return from_hip(launch_eltwise_np_absmax(ah, al, bh, bl, n, F - frac_a, F - frac_b, relu ? 1 : 0,
                                             reinterpret_cast<unsigned long long *>(amax_dev), (hipStream_t)stream));
}

dfq_status dfq_np_frac_from_absmax_u64(uint64_t max_abs, int acc_frac, int nbits, int p, int *frac)
{
    if (!frac) return DFQ_EINVAL;
    if (nbits < 2 || nbits > 16 || p < 0 || p > nbits - 1) return DFQ_EFMT;
    if (acc_frac < -128 || acc_frac > 128) return DFQ_EFMT;
    const int64_t bm64 = dfq_beta_max(nbits, p);
    if (bm64 <= 0) return DFQ_EFMT;
    const uint64_t bm = (uint64_t)bm64;
    int f = acc_frac > 32 ? 32 : (acc_frac < -32 ? -32 : acc_frac);
    for (; f > -32; f--) {
        const int sh = acc_frac - f;          // >= 0: the factor 2^(f - acc_frac) stays in (0, 1]
        if (sh >= 64) break;                  // max_abs < 2^64 <= beta_max * 2^sh
        const uint64_t q = max_abs >> sh, r = sh ? (max_abs & ((1ull << sh) - 1ull)) : 0ull;
        if (q < bm || (q == bm && r == 0)) break;      // max_abs <= beta_max * 2^sh without forming the product
    }
    *frac = f;
    return DFQ_OK;
}

dfq_status dfq_pool_np(const int8_t *xh, const int8_t *xl, uint8_t *y, int8_t *yh, int8_t *yl, dfq_pool_mode mode, int N, int H, int W, int C,
                       int k, int stride, int pad, int p_fmt, dfq_stream stream)
{
    if (mode != DFQ_POOL_MAX && mode != DFQ_POOL_AVG) return DFQ_EINVAL;
    if (N < 0) return DFQ_EINVAL;
    if (H < 1 || W < 1 || C < 1 || k < 1 || k > 16 || stride < 1 || pad < 0 || pad >= k) return DFQ_ESHAPE;
    if (mode == DFQ_POOL_AVG && pad != 0) return DFQ_EUNSUPPORTED;
    const int P = out_extent(H, pad, k, stride), Q = out_extent(W, pad, k, stride);
    if (P < 1 || Q < 1) return DFQ_ESHAPE;
    if (p_fmt < 4 || p_fmt > 7) return DFQ_EFMT;
    if (N == 0) return DFQ_OK;
    if (!xh || !xl || (!y && !yh && !yl) || ((yh == nullptr) != (yl == nullptr))) return DFQ_EINVAL;
    const size_t nx = (size_t)N * H * W * C, ny = (size_t)N * P * Q * C;
    const void *outs[3] = {y, yh, yl};
    for (int i = 0; i < 3; i++) {
        if (overlaps(outs[i], ny, xh, nx) || overlaps(outs[i], ny, xl, nx)) return DFQ_EINVAL;
        for (int j = i + 1; j < 3; j++)
            if (overlaps(outs[i], ny, outs[j], ny)) return DFQ_EINVAL;
    }
    return from_hip(launch_pool_np(xh, xl, y, yh, yl, mode == DFQ_POOL_AVG ? 1 : 0, N, H, W, C, k, stride, pad, P, Q, p_fmt,
                                   (int)dfq_beta_max(8, p_fmt), (hipStream_t)stream));
}

dfq_status dfq_stem_pack_x(const int8_t *x, int8_t *y, int N, int H, int W, int C, int R, int S, int pad, dfq_stream stream)
{
    if (N < 0) return DFQ_EINVAL;
    if (H < 1 || W < 1 || C < 1 || C > 4 || R < 1 || S < 1 || R > 8 || S > 8 || pad < 0) return DFQ_ESHAPE;
    const int P = out_extent(H, pad, R, 2), Q = out_extent(W, pad, S, 2);
    if (P < 1 || Q < 1) return DFQ_ESHAPE;
    if (N == 0) return DFQ_OK;
    if (!x || !y || ((uintptr_t)y & 15)) return DFQ_EINVAL;
    const int Hs = P + 3;                   // rows of the packed tensor: output rows plus the 4-row window minus one
    if (overlaps(x, (size_t)N * H * W * C, y, (size_t)N * Hs * Q * 64)) return DFQ_EINVAL;
    return from_hip(launch_stem_pack_x(x, y, N, H, W, C, pad, Hs, Q, (hipStream_t)stream));
}

dfq_status dfq_stem_pack_w(const int8_t *w, int8_t *y, int K, int R, int S, int C, dfq_stream stream)
{
    if (K < 1 || C < 1 || C > 4 || R < 1 || S < 1 || R > 8 || S > 8) return DFQ_ESHAPE;
    if (!w || !y || overlaps(w, (size_t)K * R * S * C, y, (size_t)K * 256)) return DFQ_EINVAL;
    return from_hip(launch_stem_pack_w(w, y, K, R, S, C, (hipStream_t)stream));
}

dfq_status dfq_conv_np(const int8_t *xh, const int8_t *xl, const int8_t *wh, const int8_t *wl, const int32_t *b, uint8_t *y,
                       int8_t *yh, int8_t *yl, int N, int H, int W, int C, int K, int R, int S, int stride, int pad, int groups,
                       int frac_x, int frac_w, int frac_y, int p_y, int relu, dfq_stream stream)
{
    return dfq_conv_np_variant(DFQ_CONV_AUTO, xh, xl, wh, wl, b, y, yh, yl, N, H, W, C, K, R, S, stride, pad, groups, frac_x, frac_w,
                               frac_y, p_y, relu, stream);
}

dfq_status dfq_conv_q_variant(dfq_conv_variant variant, const int8_t *x, const int8_t *w, const int32_t *b, int8_t *y,
                              int32_t *acc_out, int N, int H, int W, int C, int K, int R, int S, int stride, int pad,
                              int groups, int ldy, dfq_fmt fmt_in, dfq_fmt fmt_w, dfq_fmt fmt_out, int relu,
                              dfq_stream stream)
{
    ConvCheck c = check_conv(x, w, b, y, acc_out, N, H, W, C, K, R, S, stride, pad, groups, ldy, fmt_in, fmt_w, fmt_out,
                             relu, true);
    if (c.st != DFQ_OK) return c.st;
    if (N == 0) return DFQ_OK;
    return run_conv(variant, c.a, (hipStream_t)stream);
}

dfq_status dfq_conv_q_pc(const int8_t *x, const int8_t *w, const int32_t *b, int8_t *y, int32_t *acc_out, int N, int H,
                         int W, int C, int K, int R, int S, int stride, int pad, int groups, int ldy, dfq_fmt fmt_in,
                         const int32_t *frac_w, int frac_w_lo, int frac_w_hi, dfq_fmt fmt_out, int relu, dfq_stream stream)
{
    if (frac_w_lo > frac_w_hi || frac_w_lo < -32 || frac_w_hi > 32) return DFQ_EFMT;
    ConvCheck c = check_conv(x, w, b, y, acc_out, N, H, W, C, K, R, S, stride, pad, groups, ldy, fmt_in, dfq_fmt{8, 0},
                             fmt_out, relu, true);
    if (c.st != DFQ_OK) return c.st;
    if (!frac_w || ((uintptr_t)frac_w & 3)) return DFQ_EINVAL;
    if (N == 0) return DFQ_OK;
    c.a.frac_w = frac_w;          // c.a.shift is f_in - f_out (the placeholder weight format has frac 0)
    c.a.frac_w_lo = frac_w_lo;
    c.a.frac_w_hi = frac_w_hi;
    return run_conv(DFQ_CONV_AUTO, c.a, (hipStream_t)stream);
}

dfq_status dfq_conv_q(const int8_t *x, const int8_t *w, const int32_t *b, int8_t *y, int32_t *acc_out, int N, int H, int W,
                      int C, int K, int R, int S, int stride, int pad, int groups, int ldy, dfq_fmt fmt_in, dfq_fmt fmt_w,
                      dfq_fmt fmt_out, int relu, dfq_stream stream)
{
    return dfq_conv_q_variant(DFQ_CONV_AUTO, x, w, b, y, acc_out, N, H, W, C, K, R, S, stride, pad, groups, ldy, fmt_in,
                              fmt_w, fmt_out, relu, stream);
}

dfq_status dfq_conv_q_add(const int8_t *x, const int8_t *w, const int32_t *b, const int8_t *other, int8_t *y, int N, int H,
                          int W, int C, int K, int R, int S, int stride, int pad, int groups, int ldy, int ld_other,
                          dfq_fmt fmt_in, dfq_fmt fmt_w, dfq_fmt fmt_mid, int relu_mid, dfq_fmt fmt_other, dfq_fmt fmt_out,
                          int relu_out, dfq_stream stream)
{
    ConvCheck c = check_conv(x, w, b, y, nullptr, N, H, W, C, K, R, S, stride, pad, groups, ldy, fmt_in, fmt_w, fmt_mid,
                             relu_mid, true);
    return run_conv_add(c, x, other, y, N, H, W, C, K, ldy, ld_other, fmt_mid, fmt_other, fmt_out, relu_out, stream);
}

// x: int8 codes (x_is_float == false) or float images to be converted at fmt_in on the way in
// frac_w != null: one weight format per output channel (fmt_w is then a placeholder with frac 0)
static dfq_status conv_maxpool(const void *x, bool x_is_float, const int8_t *w, const int32_t *b, int8_t *y, int N, int H, int W, int C,
                               int K, int R, int S, int stride, int pad, int groups, int ldy, dfq_fmt fmt_in, dfq_fmt fmt_w,
                               dfq_fmt fmt_out, int relu, int pool_k, int pool_stride, int pool_pad, dfq_stream stream,
                               const int32_t *frac_w = nullptr, int frac_w_lo = 0, int frac_w_hi = 0)
{
    // the convolution's own checks, with a placeholder where its tensor would be (never written)
    ConvCheck c = check_conv((const int8_t *)x, w, b, nullptr, nullptr, N, H, W, C, K, R, S, stride, pad, groups, K, fmt_in, fmt_w, fmt_out, relu,
                             false);
    if (c.st != DFQ_OK) return c.st;
    if (!x || !w || !y) return DFQ_EINVAL;
    if (pool_k < 1 || pool_k > 64 || pool_stride < 1 || pool_pad < 0 || pool_pad >= pool_k) return DFQ_ESHAPE;
    const int PP = out_extent(c.a.P, pool_pad, pool_k, pool_stride), PQ = out_extent(c.a.Q, pool_pad, pool_k, pool_stride);
    if (PP < 1 || PQ < 1 || ldy < K) return DFQ_ESHAPE;
    if (N == 0) return DFQ_OK;
    if (overlaps(x, (size_t)N * H * W * C * (x_is_float ? 4 : 1), y, (size_t)N * PP * PQ * (size_t)ldy)) return DFQ_EINVAL;
    if (pool_k != 3 || pool_stride != 2 || pool_pad != 1) return DFQ_EUNSUPPORTED;
    if (((uintptr_t)y & 15) || (ldy & 15)) return DFQ_EUNSUPPORTED;
    c.a.frac_w = frac_w;
    c.a.frac_w_lo = frac_w_lo;
    c.a.frac_w_hi = frac_w_hi;
    if (x_is_float) {
        if ((uintptr_t)x & 15) return DFQ_EUNSUPPORTED;
        c.a.x = nullptr;
    } else {
        c.a.x = (const int8_t *)x;
    }
    if (!conv_stem_supports(c.a, true, x_is_float)) return DFQ_EUNSUPPORTED;
    return from_hip(launch_conv_stem(c.a, y, ldy, (hipStream_t)stream, x_is_float ? (const float *)x : nullptr, fmt_in.frac));
}

dfq_status dfq_conv_q_maxpool(const int8_t *x, const int8_t *w, const int32_t *b, int8_t *y, int N, int H, int W, int C, int K,
                              int R, int S, int stride, int pad, int groups, int ldy, dfq_fmt fmt_in, dfq_fmt fmt_w, dfq_fmt fmt_out,
                              int relu, int pool_k, int pool_stride, int pool_pad, dfq_stream stream)
{
    return conv_maxpool(x, false, w, b, y, N, H, W, C, K, R, S, stride, pad, groups, ldy, fmt_in, fmt_w, fmt_out, relu, pool_k,
                        pool_stride, pool_pad, stream);
}

dfq_status dfq_quantize_conv_q_maxpool(const float *x, const int8_t *w, const int32_t *b, int8_t *y, int N, int H, int W, int C,
                                       int K, int R, int S, int stride, int pad, int groups, int ldy, dfq_fmt fmt_in, dfq_fmt fmt_w,
                                       dfq_fmt fmt_out, int relu, int pool_k, int pool_stride, int pool_pad, dfq_stream stream)
{
    return conv_maxpool(x, true, w, b, y, N, H, W, C, K, R, S, stride, pad, groups, ldy, fmt_in, fmt_w, fmt_out, relu, pool_k,
                        pool_stride, pool_pad, stream);
}

dfq_status dfq_quantize_conv_q(const float *x, const int8_t *w, const int32_t *b, int8_t *y, int N, int H, int W, int C, int K, int R,
                               int S, int stride, int pad, int groups, int ldy, dfq_fmt fmt_in, dfq_fmt fmt_w, dfq_fmt fmt_out, int relu,
                               dfq_stream stream)
{
    ConvCheck c = check_conv(nullptr, w, b, y, nullptr, N, H, W, C, K, R, S, stride, pad, groups, ldy, fmt_in, fmt_w, fmt_out, relu, false);
    if (c.st != DFQ_OK) return c.st;
    if (!x || !w || !y) return DFQ_EINVAL;
    if (ldy < K) return DFQ_ESHAPE;
    if (N == 0) return DFQ_OK;
    if (overlaps(x, (size_t)N * H * W * C * 4, y, (size_t)N * c.a.P * c.a.Q * (size_t)ldy)) return DFQ_EINVAL;
    if (((uintptr_t)x & 15) || !conv_stem_supports(c.a, false, true)) return DFQ_EUNSUPPORTED;
    return from_hip(launch_conv_stem(c.a, nullptr, 0, (hipStream_t)stream, x, fmt_in.frac));
}

dfq_status dfq_conv_q_pc_maxpool(const int8_t *x, const int8_t *w, const int32_t *b, int8_t *y, int N, int H, int W, int C, int K,
                                 int R, int S, int stride, int pad, int groups, int ldy, dfq_fmt fmt_in, const int32_t *frac_w,
                                 int frac_w_lo, int frac_w_hi, dfq_fmt fmt_out, int relu, int pool_k, int pool_stride, int pool_pad,
                                 dfq_stream stream)
{
    if (frac_w_lo > frac_w_hi || frac_w_lo < -32 || frac_w_hi > 32) return DFQ_EFMT;
    if (!frac_w || ((uintptr_t)frac_w & 3)) return DFQ_EINVAL;
    return conv_maxpool(x, false, w, b, y, N, H, W, C, K, R, S, stride, pad, groups, ldy, fmt_in, dfq_fmt{8, 0}, fmt_out, relu, pool_k,
                        pool_stride, pool_pad, stream, frac_w, frac_w_lo, frac_w_hi);
}

dfq_status dfq_quantize_conv_q_pc_maxpool(const float *x, const int8_t *w, const int32_t *b, int8_t *y, int N, int H, int W, int C,
                                          int K, int R, int S, int stride, int pad, int groups, int ldy, dfq_fmt fmt_in,
                                          const int32_t *frac_w, int frac_w_lo, int frac_w_hi, dfq_fmt fmt_out, int relu, int pool_k,
                                          int pool_stride, int pool_pad, dfq_stream stream)
{
    if (frac_w_lo > frac_w_hi || frac_w_lo < -32 || frac_w_hi > 32) return DFQ_EFMT;
    if (!frac_w || ((uintptr_t)frac_w & 3)) return DFQ_EINVAL;
    return conv_maxpool(x, true, w, b, y, N, H, W, C, K, R, S, stride, pad, groups, ldy, fmt_in, dfq_fmt{8, 0}, fmt_out, relu, pool_k,
                        pool_stride, pool_pad, stream, frac_w, frac_w_lo, frac_w_hi);
}

dfq_status dfq_conv_q_add_lazy(const int8_t *x, const int8_t *w, const int32_t *b, const int8_t *other, int8_t *y, int N, int H,
                               int W, int C, int K, int R, int S, int stride, int pad, int groups, int ldy, int ld_other,
                               dfq_fmt fmt_in, dfq_fmt fmt_w, dfq_fmt fmt_other, dfq_fmt fmt_out, int relu_out, dfq_stream stream)
{
    ConvCheck c = check_conv(x, w, b, y, nullptr, N, H, W, C, K, R, S, stride, pad, groups, ldy, fmt_in, fmt_w, fmt_out, 0, true);
    if (c.st != DFQ_OK) return c.st;
    if (!fmt_ok(fmt_other)) return DFQ_EFMT;
    if (!y || !other) return DFQ_EINVAL;
    if (ld_other < K) return DFQ_ESHAPE;
    // Eq. 12: a code of magnitude <= 2^7 shifted by <= 22 bits stays below 2^29
    const int sb = fmt_in.frac + fmt_w.frac - fmt_other.frac;
    if (sb < 0 || sb > 22) return DFQ_EFMT;
    if (N == 0) return DFQ_OK;
    const size_t npix = (size_t)N * c.a.P * c.a.Q;
    if (overlaps(other, npix * (size_t)ld_other, y, npix * (size_t)ldy) ||
        overlaps(other, npix * (size_t)ld_other, x, (size_t)N * H * W * C))
        return DFQ_EINVAL;
    c.a.add = other;
    c.a.ldadd = ld_other;
    c.a.add_sa = 0;
    c.a.add_sb = sb;
    c.a.add_shift = c.a.shift;                    // f_in + f_w - f_out
    c.a.add_relu = relu_out ? 1 : 0;
    c.a.add_lazy = 1;
    if (conv_pw_supports(c.a)) return from_hip(launch_conv_pw(c.a, (hipStream_t)stream));
    if (conv_mfma_fuses(c.a)) return from_hip(launch_conv_mfma(c.a, (hipStream_t)stream));
    return DFQ_EUNSUPPORTED;
}

dfq_status dfq_conv_q_pc_add(const int8_t *x, const int8_t *w, const int32_t *b, const int8_t *other, int8_t *y, int N,
                             int H, int W, int C, int K, int R, int S, int stride, int pad, int groups, int ldy,
                             int ld_other, dfq_fmt fmt_in, const int32_t *frac_w, int frac_w_lo, int frac_w_hi,
                             dfq_fmt fmt_mid, int relu_mid, dfq_fmt fmt_other, dfq_fmt fmt_out, int relu_out,
                             dfq_stream stream)
{
    if (frac_w_lo > frac_w_hi || frac_w_lo < -32 || frac_w_hi > 32) return DFQ_EFMT;
    ConvCheck c = check_conv(x, w, b, y, nullptr, N, H, W, C, K, R, S, stride, pad, groups, ldy, fmt_in, dfq_fmt{8, 0},
                             fmt_mid, relu_mid, true);
    if (c.st == DFQ_OK && (!frac_w || ((uintptr_t)frac_w & 3))) return DFQ_EINVAL;
    c.a.frac_w = frac_w;
    c.a.frac_w_lo = frac_w_lo;
    c.a.frac_w_hi = frac_w_hi;
    return run_conv_add(c, x, other, y, N, H, W, C, K, ldy, ld_other, fmt_mid, fmt_other, fmt_out, relu_out, stream);
}

dfq_conv_variant dfq_conv_q_select(int N, int H, int W, int C, int K, int R, int S, int stride, int pad, int groups)
{
    dfq_fmt f{8, 0};
    ConvCheck c = check_conv(nullptr, nullptr, nullptr, nullptr, nullptr, N, H, W, C, K, R, S, stride, pad, groups, K, f, f,
                             f, 0, false);
    if (c.st != DFQ_OK) return DFQ_CONV_AUTO;
    return select_variant(c.a, true);
}

dfq_status dfq_eltwise_q(const int8_t *a, dfq_fmt fa, const int8_t *b, dfq_fmt fb, int8_t *y, dfq_fmt fy, int32_t *acc_out,
                         size_t n, int relu, dfq_stream stream)
{
    if (!fmt_ok(fa) || !fmt_ok(fb) || !fmt_ok(fy)) return DFQ_EFMT;
    int F = fa.frac > fb.frac ? fa.frac : fb.frac;
    // Eq. 12: two codes of magnitude <= 2^7 shifted by <= 22 bits sum to at most 2^30
    if (F - fa.frac > 22 || F - fb.frac > 22) return DFQ_EFMT;
    if (n == 0) return DFQ_OK;
    if (!a || !b || (!y && !acc_out)) return DFQ_EINVAL;
    if (overlaps(a, n, y, n) || overlaps(b, n, y, n) || overlaps(a, n, acc_out, n * 4) || overlaps(b, n, acc_out, n * 4))
        return DFQ_EINVAL;
    return from_hip(launch_eltwise(a, fa.frac, b, fb.frac, y, fy.frac, acc_out, n, relu ? 1 : 0, (hipStream_t)stream));
}

dfq_status dfq_concat_q_into(int nbranch, const int8_t *const *xs, const int *Cs, const dfq_fmt *fs, int8_t *y, int ldy,
                             dfq_fmt fy, size_t pixels, dfq_stream stream)
{
    if (nbranch < 1 || nbranch > 8 || !xs || !Cs || !fs) return DFQ_EINVAL;
    if (!fmt_ok(fy)) return DFQ_EFMT;
    int fr[8];
    long long ct = 0;
    for (int i = 0; i < nbranch; i++) {
        if (!fmt_ok(fs[i])) return DFQ_EFMT;
        if (Cs[i] < 1) return DFQ_ESHAPE;
        fr[i] = fs[i].frac;
        ct += Cs[i];
    }
    if (ct >= (1LL << 31) || ldy < ct) return DFQ_ESHAPE;
    if (pixels == 0) return DFQ_OK;
    if (!y) return DFQ_EINVAL;
    for (int i = 0; i < nbranch; i++) {
        if (!xs[i]) return DFQ_EINVAL;
        if (overlaps(xs[i], pixels * (size_t)Cs[i], y, (pixels - 1) * (size_t)ldy + (size_t)ct)) return DFQ_EINVAL;
    }
    return from_hip(launch_concat(nbranch, xs, Cs, fr, y, ldy, fy.frac, pixels, (hipStream_t)stream));
}

dfq_status dfq_concat_q(int nbranch, const int8_t *const *xs, const int *Cs, const dfq_fmt *fs, int8_t *y, dfq_fmt fy,
                        size_t pixels, dfq_stream stream)
{
    long long ct = 0;
    if (nbranch >= 1 && nbranch <= 8 && Cs)
        for (int i = 0; i < nbranch; i++) ct += Cs[i] > 0 ? Cs[i] : 0;
    if (ct >= (1LL << 31)) return DFQ_ESHAPE;
    return dfq_concat_q_into(nbranch, xs, Cs, fs, y, (int)ct, fy, pixels, stream);
}

dfq_status dfq_pool_q(const int8_t *x, int8_t *y, dfq_pool_mode mode, int N, int H, int W, int C, int k, int stride, int pad,
                      dfq_fmt fin, dfq_fmt fout, dfq_stream stream)
{
    if (mode != DFQ_POOL_MAX && mode != DFQ_POOL_AVG) return DFQ_EINVAL;
    if (N < 0) return DFQ_EINVAL;
    if (H < 1 || W < 1 || C < 1 || k < 1 || k > 64 || stride < 1 || pad < 0 || pad >= k) return DFQ_ESHAPE;
    int P = out_extent(H, pad, k, stride), Q = out_extent(W, pad, k, stride);
    if (P < 1 || Q < 1) return DFQ_ESHAPE;
    if (!fmt_ok(fin) || !fmt_ok(fout)) return DFQ_EFMT;
    if (N == 0) return DFQ_OK;
    if (!x || !y) return DFQ_EINVAL;
    if (overlaps(x, (size_t)N * H * W * C, y, (size_t)N * P * Q * C)) return DFQ_EINVAL;
    return from_hip(launch_pool(x, y, (int)mode, N, H, W, C, P, Q, k, stride, pad, fin.frac, fout.frac, (hipStream_t)stream));
}

dfq_status dfq_absmax_f32(const float *x, size_t n, float *out_dev, dfq_stream stream)
{
    if (!out_dev || (n && !x)) return DFQ_EINVAL;
    return from_hip(launch_absmax_f32(x, n, out_dev, (hipStream_t)stream));
}

dfq_status dfq_absmax_i32(const int32_t *x, size_t n, int relu, uint32_t *out_dev, dfq_stream stream)
{
    if (!out_dev || (n && !x)) return DFQ_EINVAL;
    return from_hip(launch_absmax_i32(x, n, relu ? 1 : 0, out_dev, (hipStream_t)stream));
}

dfq_status dfq_quantize_rows(const float *x, int8_t *q, size_t rows, size_t row_len, const int32_t *frac, dfq_stream stream)
{
    if (rows == 0 || row_len == 0) return DFQ_OK;
    if (!x || !q || !frac || overlaps(x, rows * row_len * 4, q, rows * row_len)) return DFQ_EINVAL;
    return from_hip(launch_quantize_rows(x, q, rows, row_len, frac, (hipStream_t)stream));
}

dfq_status dfq_quantize_i32_rows(const float *x, int32_t *q, size_t rows, size_t row_len, const int32_t *frac,
                                 int32_t frac_add, dfq_stream stream)
{
    if (frac_add < -64 || frac_add > 64) return DFQ_EFMT;
    if (rows == 0 || row_len == 0) return DFQ_OK;
    if (!x || !q || !frac || overlaps(x, rows * row_len * 4, q, rows * row_len * 4)) return DFQ_EINVAL;
    return from_hip(launch_quantize_i32_rows(x, q, rows, row_len, frac, frac_add, (hipStream_t)stream));
}

dfq_status dfq_fold_scale_f32(const float *w, const float *b, size_t rows, size_t row_len, const float *scale, const float *shift,
                              float *w_out, float *b_out, dfq_stream stream)
{
    if (rows == 0) return DFQ_OK;
    if (!scale || (row_len && (!w || !w_out))) return DFQ_EINVAL;
    if (!b_out && (b || shift)) return DFQ_EINVAL;               // a bias or shift was given but there is nowhere to put the result
    // in place (w_out == w, b_out == b) is fine: every element is read once, by the lane that writes it
    if ((w_out != w && overlaps(w, rows * row_len * 4, w_out, rows * row_len * 4)) || (b_out && b_out != b && overlaps(b, rows * 4, b_out, rows * 4)))
        return DFQ_EINVAL;
    return from_hip(launch_fold_scale(w, b, rows, row_len, scale, shift, w_out, b_out, (hipStream_t)stream));
}

dfq_status dfq_absmax_f32_rows(const float *x, size_t rows, size_t row_len, float *out_dev, dfq_stream stream)
{
    if (rows == 0) return DFQ_OK;
    if (!out_dev || (row_len && !x)) return DFQ_EINVAL;
    return from_hip(launch_absmax_f32_rows(x, rows, row_len, out_dev, (hipStream_t)stream));
}

dfq_status dfq_absmax_i32_channels(const int32_t *x, size_t pixels, int K, int relu, uint32_t *out_dev, dfq_stream stream)
{
    if (K < 1) return DFQ_ESHAPE;
    if (!out_dev || (pixels && !x)) return DFQ_EINVAL;
    return from_hip(launch_absmax_i32_channels(x, pixels, K, relu ? 1 : 0, out_dev, (hipStream_t)stream));
}

dfq_status dfq_hist_i32(const int32_t *x, size_t n, int relu, int shift, uint32_t *hist_dev, dfq_stream stream)
{
    if (shift < 0 || shift > 31) return DFQ_EINVAL;
    if (!hist_dev || (n && !x)) return DFQ_EINVAL;
    if (n >= ((size_t)1 << 32)) return DFQ_EUNSUPPORTED;      // 32-bit counts
    return from_hip(launch_hist_i32(x, n, relu ? 1 : 0, shift, hist_dev, (hipStream_t)stream));
}

int dfq_hist_shift(int64_t max_abs)
{
    if (max_abs < 0) return -1;
    int j = 0;
    while ((max_abs >> j) >= DFQ_HIST_BINS) j++;
    return j;
}

// Algorithm 1 on a histogram.  All arithmetic in double, every sum in index order, fixed-size storage.
//
// A candidate clips at bin edge i (i bins kept).  Its clipped distribution function r has r[t] = cdf[t] for
// t < i-1 and 1 from bin i-1 on.  The 8-bit format offers the 128 levels k/127 of the clipped range [0, 1]; on the
// bin grid t/(i-1) the quantized distribution function q is r sampled at the levels and linearly interpolated back
// to the grid.  Both interpolations walk two increasing sequences, so each is one merge pass.  The candidate's
// distance is the area between cdf and q over the kept bins plus the area between cdf and 1 over the clipped ones,
// added up in bin order.
dfq_status dfq_threshold_search(const uint32_t *hist, int nbins, int shift, int64_t max_abs, int64_t *gamma_out,
                                double *delta_out)
{
    constexpr int kLevels = 128;               // non-negative codes of the 8-bit format
    if (!hist || !gamma_out || nbins < 1 || nbins > DFQ_HIST_BINS || shift < 0 || shift > 31 || max_abs < 0) return DFQ_EINVAL;
    if ((max_abs >> shift) != nbins - 1) return DFQ_ESHAPE;    // the last bin is the one that holds the maximum
    double total = 0.0;
    for (int t = 0; t < nbins; t++) total += (double)hist[t];
    if (!(total > 0.0) || max_abs == 0) {
        *gamma_out = 0;
        if (delta_out) *delta_out = 0.0;
        return DFQ_OK;
    }
    double cdf[DFQ_HIST_BINS];
    double at_level[kLevels];                  // the clipped distribution function sampled at level k/127
    double run = 0.0;
    for (int t = 0; t < nbins; t++) {
        run += (double)hist[t] / total;
        cdf[t] = run;
    }
    int64_t gamma = max_abs;                   // fewer bins than 129: nothing is clipped
    double best = 0.0;
    bool have = false;
    for (int i = kLevels + 1; i <= nbins; i++) {
        const int last = i - 1;                // index of the bin that receives the clipped mass; grid point t is t / last
        auto r = [&](int t) { return t < last ? cdf[t] : 1.0; };
        auto grid = [&](int t) { return t == last ? 1.0 : (double)t * (1.0 / (double)last); };
        // sample r at the levels: level k lies in grid segment [seg, seg + 1]
        int seg = 0;
        for (int k = 0; k < kLevels; k++) {
            const double lv = (double)k / (double)(kLevels - 1);
            while (seg + 1 < i && grid(seg + 1) <= lv) seg++;
            if (seg == last || grid(seg) == lv) at_level[k] = r(seg);
            else at_level[k] = (r(seg + 1) - r(seg)) / (grid(seg + 1) - grid(seg)) * (lv - grid(seg)) + r(seg);
        }
        // back to the grid and the distance over the kept bins
        double d = 0.0;
        int k = 0;
        for (int t = 0; t < i; t++) {
            const double g = grid(t);
            while (k + 1 < kLevels && (double)(k + 1) / (double)(kLevels - 1) <= g) k++;
            const double lk = (double)k / (double)(kLevels - 1);
            double q;
            if (k == kLevels - 1 || lk == g) q = at_level[k];
            else q = (at_level[k + 1] - at_level[k]) / ((double)(k + 1) / (double)(kLevels - 1) - lk) * (g - lk) + at_level[k];
            d += std::fabs(cdf[t] - q);
        }
        for (int t = i; t < nbins; t++) d += std::fabs(cdf[t] - 1.0);
        if (!have || best > d) {
            have = true;
            best = d;
            const int64_t edge = ((int64_t)i << shift) - 1;
            gamma = edge < max_abs ? edge : max_abs;
        }
    }
    *gamma_out = gamma;
    if (delta_out) *delta_out = best;
    return DFQ_OK;
}

dfq_status dfq_fmt_from_absmax_f32(float gamma, dfq_fmt *out)
{
    if (!out) return DFQ_EINVAL;
    if (!(gamma >= 0.0f) || std::isinf(gamma)) return DFQ_EINVAL;
    // gamma * 2^f is exact in double, so the comparison needs no logarithm
    int f = 32;
    while (f > -32 && std::ldexp((double)gamma, f) > 127.0) f--;
    out->bits = 8;
    out->frac = f;
    return DFQ_OK;
}

dfq_status dfq_np_frac_from_absmax_f32(float gamma, int nbits, int p, int32_t *frac_out)
{
    if (!frac_out) return DFQ_EINVAL;
    if (!(gamma >= 0.0f) || std::isinf(gamma)) return DFQ_EINVAL;
    if (!np_ok(nbits, p, 0)) return DFQ_EFMT;
    const double bmax = (double)dfq_beta_max(nbits, p);
    int f = 32;
    while (f > -32 && std::ldexp((double)gamma, f) > bmax) f--;
    *frac_out = f;
    return DFQ_OK;
}

dfq_status dfq_fmt_from_absmax_i32(int64_t m, int32_t acc_frac, dfq_fmt *out)
{
    if (!out || m < 0) return DFQ_EINVAL;
    int f = acc_frac > 32 ? 32 : acc_frac;
    // lower f until m fits in 127 * 2^(acc_frac - f); m < 2^32 always fits once the gap is 26 bits
    while (f > -32) {
        int gap = acc_frac - f;
        if (gap >= 40 || m <= ((int64_t)127 << gap)) break;
        f--;
    }
    if (f < -32) f = -32;
    out->bits = 8;
    out->frac = f;
    return DFQ_OK;
}

dfq_status dfq_fmt_from_absmax_i32_channels(const uint32_t *m, int K, int32_t frac_in, const int32_t *frac_w, dfq_fmt *out)
{
    if (!m || !frac_w || !out || K < 1) return DFQ_EINVAL;
    int f = 32;
    for (int k = 0; k < K; k++) {
        if (frac_w[k] < -32 || frac_w[k] > 32) return DFQ_EFMT;
        dfq_fmt fk;
        const dfq_status st = dfq_fmt_from_absmax_i32((int64_t)m[k], frac_in + frac_w[k], &fk);
        if (st != DFQ_OK) return st;
        if (fk.frac < f) f = fk.frac;
    }
    out->bits = 8;
    out->frac = f;
    return DFQ_OK;
}

int64_t dfq_beta_max(int n, int p)
{
    if (n < 2 || n > 32 || p < 0 || p > n - 1) return -1;
    if (p == n - 1) return ((int64_t)1 << (n - 1)) - 1;
    int ebits = n - 1 - p;                    // exponent field width
    if (ebits > 5) return -1;                 // result would not fit 64 bits
    int emax = (1 << ebits) - 1;              // all-ones exponent is an ordinary number here
    // largest magnitude: 2^(emax-1) * (2^p + (2^p - 1))
    return ((int64_t)1 << (emax - 1)) * (((int64_t)1 << (p + 1)) - 1);
}

int dfq_mac_acc_bits(int64_t N, int64_t bx, int64_t ex, int64_t by, int64_t ey)
{
    if (N < 1 || bx < 1 || by < 1 || ex < 0 || ey < 0) return -1;
    return width_for((unsigned long long)N * (unsigned long long)(bx + ex) * (unsigned long long)(by + ey) + 1ULL);
}

int64_t dfq_mac_max_len(int q, int64_t bx, int64_t ex, int64_t by, int64_t ey)
{
    if (q < 2 || q > 63 || bx < 1 || by < 1 || ex < 0 || ey < 0) return -1;
    return (((int64_t)1 << (q - 1)) - 1) / ((bx + ex) * (by + ey));
}

int dfq_add_acc_bits(int64_t N, int64_t bx, int64_t ex)
{
    if (N < 1 || bx < 1 || ex < 0) return -1;
    unsigned long long m = (unsigned long long)N * (unsigned long long)bx;
    m += ex == 0 ? 1ULL : (unsigned long long)N * (unsigned long long)ex;
    return width_for(m);
}

int64_t dfq_add_max_len(int q, int64_t bx, int64_t ex)
{
    if (q < 2 || q > 63 || bx < 1 || ex < 0) return -1;
    if (ex == 0) return (((int64_t)1 << (q - 1)) - 1) / bx;
    return ((int64_t)1 << (q - 1)) / (bx + ex);
}

}  // extern "C"
