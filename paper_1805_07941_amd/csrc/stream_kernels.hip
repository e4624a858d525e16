// Bandwidth-bound kernels of the quantized path: float<->code conversion, scaled addition
// (Eq. 10), concat with per-branch rescale, pooling, and the max-|.| reductions used by
// calibration (Sec. 3).  Every kernel moves 16 bytes per lane per access where alignment
// allows and falls back to narrower accesses otherwise; none keeps data in LDS because
// nothing is reused.
#include "dfq_device.hpp"
#include "dfq_host.hpp"
#include "conv_epilogue.hpp"

namespace dfq {

static constexpr int kBlock = 256;

static inline int grid_for(size_t work_items)
{
    size_t blocks = (work_items + kBlock - 1) / kBlock;
    size_t cap = 256 * 16;  // 16 workgroups per compute unit, grid-stride beyond that
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    return (int)blocks;
}

// ------------------------------------------------------------------------------------------
// quantize / dequantize
// ------------------------------------------------------------------------------------------

__device__ __forceinline__ int quant_one(float x, float scale)
{
    // x * 2^f is exact in float (power-of-two scale) except on overflow, which saturates,
    // and on underflow, which rounds to 0 either way.
    float t = __builtin_rintf(x * scale);  // v_rndne_f32: ties to even
    if (!(t == t)) return 0;               // NaN
    t = fminf(fmaxf(t, -127.0f), 127.0f);
    return (int)t;
}

__global__ void __launch_bounds__(kBlock) quantize_vec4(const float4 *__restrict__ x, uint32_t *__restrict__ q,
                                                         size_t n4, float scale)
{
    for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < n4; i += (size_t)gridDim.x * kBlock) {
        float4 v = x[i];
        q[i] = pack4(quant_one(v.x, scale), quant_one(v.y, scale), quant_one(v.z, scale), quant_one(v.w, scale));
    }
}

__global__ void __launch_bounds__(kBlock) quantize_scalar(const float *__restrict__ x, int8_t *__restrict__ q,
                                                           size_t n, float scale)
{
    for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (size_t)gridDim.x * kBlock)
        q[i] = (int8_t)quant_one(x[i], scale);
}

__global__ void __launch_bounds__(kBlock) quantize_i32_kernel(const float *__restrict__ x, int32_t *__restrict__ q,
                                                               size_t n, float scale)
{
    for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (size_t)gridDim.x * kBlock) {
        float t = __builtin_rintf(x[i] * scale);   // exact product; overflow to Inf saturates below
        int32_t c;
        if (!(t == t)) c = 0;
        else if (t >= 2147483648.0f) c = 2147483647;
        else if (t <= -2147483648.0f) c = -2147483647;
        else c = (int32_t)t;
        q[i] = c;
    }
}

__global__ void __launch_bounds__(kBlock) dequantize_vec4(const uint32_t *__restrict__ q, float4 *__restrict__ x,
                                                           size_t n4, float inv_scale)
{
    for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < n4; i += (size_t)gridDim.x * kBlock) {
        uint32_t w = q[i];
        x[i] = make_float4((float)byte_of(w, 0) * inv_scale, (float)byte_of(w, 1) * inv_scale,
                           (float)byte_of(w, 2) * inv_scale, (float)byte_of(w, 3) * inv_scale);
    }
}

__global__ void __launch_bounds__(kBlock) dequantize_scalar(const int8_t *__restrict__ q, float *__restrict__ x,
                                                             size_t n, float inv_scale)
{
    for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (size_t)gridDim.x * kBlock)
        x[i] = (float)q[i] * inv_scale;
}

// ------------------------------------------------------------------------------------------
// General (n, p) dynamic floating-point codes (Sec. 2.1, Eq. 1-5), n <= 8: one byte per code, bit n-1 the
// sign, bits n-2 .. p the exponent field e, bits p-1 .. 0 the significand field m; value
// 2^-frac * (e == 0 ? m : 2^(e-1) * (2^p + m)), every exponent code a number.
// ------------------------------------------------------------------------------------------
struct NpFmt {
    int n, p;
    float scale;      // 2^frac (quantize) or 2^-frac (dequantize)
    float beta_max;   // Eq. 5; p+1 significant bits, exact in float
};

// Nearest representable magnitude, ties to the even significand.  v = |x| * 2^frac is exact in float; below
// 2^(p+1) the representable values are the integers, in [2^(p+k), 2^(p+k+1)) the multiples of 2^k, so the
// value is brought to an integer grid by an exact power-of-two factor, rounded by v_rndne_f32 and scaled back.
__device__ __forceinline__ uint32_t np_quant_one(float x, const NpFmt &f)
{
    float v = x * f.scale;
    if (!(v == v)) return 0u;                                        // NaN
    const float a = fminf(fabsf(v), f.beta_max);
    const int ex = (int)((__float_as_uint(a) >> 23) & 0xffu) - 127;  // floor(log2 a) for a >= 2^-126
    const int k = max(ex - f.p, 0);
    float r = ldexpf(__builtin_rintf(ldexpf(a, -k)), k);
    r = fminf(r, f.beta_max);
    if (r == 0.0f) return 0u;                                        // no negative zero
    const uint32_t bits = __float_as_uint(r);
    const int er = (int)((bits >> 23) & 0xffu) - 127;                // r = 2^er * 1.fraction, at most p fraction bits set
    uint32_t code;
    if (er < f.p) code = (uint32_t)(int)r;                           // subnormal: e = 0, m = r
    else code = ((uint32_t)(er - f.p + 1) << f.p) | ((bits >> (23 - f.p)) & ((1u << f.p) - 1u));
    return code | (v < 0.0f ? (1u << (f.n - 1)) : 0u);
}

__device__ __forceinline__ float np_dequant_one(uint32_t code, const NpFmt &f)
{
    const uint32_t m = code & ((1u << f.p) - 1u);
    const uint32_t e = (code >> f.p) & ((1u << (f.n - 1 - f.p)) - 1u);   // no exponent field when p = n-1
    const float mag = e == 0 ? (float)m : ldexpf((float)((1u << f.p) + m), (int)e - 1);
    const float val = mag * f.scale;
    return ((code >> (f.n - 1)) & 1u) ? -val : val;
}

__global__ void __launch_bounds__(kBlock) quantize_np_vec4(const float4 *__restrict__ x, uint32_t *__restrict__ q, size_t n4, NpFmt f)
{
    for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < n4; i += (size_t)gridDim.x * kBlock) {
        const float4 v = x[i];
        q[i] = np_quant_one(v.x, f) | (np_quant_one(v.y, f) << 8) | (np_quant_one(v.z, f) << 16) | (np_quant_one(v.w, f) << 24);
    }
}

__global__ void __launch_bounds__(kBlock) quantize_np_scalar(const float *__restrict__ x, uint8_t *__restrict__ q, size_t n, NpFmt f)
{
    for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (size_t)gridDim.x * kBlock)
        q[i] = (uint8_t)np_quant_one(x[i], f);
}

__global__ void __launch_bounds__(kBlock) dequantize_np_vec4(const uint32_t *__restrict__ q, float4 *__restrict__ x, size_t n4, NpFmt f)
{
    for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < n4; i += (size_t)gridDim.x * kBlock) {
        const uint32_t w = q[i];
        x[i] = make_float4(np_dequant_one(w & 0xffu, f), np_dequant_one((w >> 8) & 0xffu, f), np_dequant_one((w >> 16) & 0xffu, f),
                           np_dequant_one(w >> 24, f));
    }
}

__global__ void __launch_bounds__(kBlock) dequantize_np_scalar(const uint8_t *__restrict__ q, float *__restrict__ x, size_t n, NpFmt f)
{
    for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (size_t)gridDim.x * kBlock)
        x[i] = np_dequant_one(q[i], f);
}

// Row-wise forms for weights with one format per output channel: row r of x[rows][row_len] is
// converted at the fractional length frac[r] (+ frac_add), read from device memory.
__global__ void __launch_bounds__(kBlock) quantize_rows_kernel(const float *__restrict__ x, int8_t *__restrict__ q, size_t rows,
                                                                size_t row_len, const int32_t *__restrict__ frac)
{
    const size_t n = rows * row_len;
    for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (size_t)gridDim.x * kBlock)
        q[i] = (int8_t)quant_one(x[i], ldexpf(1.0f, frac[i / row_len]));
}

__global__ void __launch_bounds__(kBlock) quantize_i32_rows_kernel(const float *__restrict__ x, int32_t *__restrict__ q, size_t rows,
                                                                    size_t row_len, const int32_t *__restrict__ frac, int frac_add)
{
    const size_t n = rows * row_len;
    for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (size_t)gridDim.x * kBlock) {
        // two exact power-of-two factors, so that a sum of fractional lengths beyond 127 cannot overflow the scale itself
        const int f = frac[i / row_len] + frac_add;
        float t = __builtin_rintf(x[i] * ldexpf(1.0f, f / 2) * ldexpf(1.0f, f - f / 2));
        int32_t c;
        if (!(t == t)) c = 0;
        else if (t >= 2147483648.0f) c = 2147483647;
        else if (t <= -2147483648.0f) c = -2147483647;
        else c = (int32_t)t;
        q[i] = c;
    }
}

// Folding a per-channel affine layer (batch norm in its inference form, a scale layer) that follows a convolution
// into the convolution's float weights and bias, before anything is quantized: w'[k][.] = w[k][.] * scale[k],
// b'[k] = b[k] * scale[k] + shift[k].  Every product and the sum are rounded to float separately (no fused
// multiply-add), so that the result does not depend on how the compiler contracts the expression.
__global__ void __launch_bounds__(kBlock) fold_scale_kernel(const float *__restrict__ w, const float *__restrict__ b, size_t rows,
                                                             size_t row_len, const float *__restrict__ scale,
                                                             const float *__restrict__ shift, float *__restrict__ w_out,
                                                             float *__restrict__ b_out)
{
#pragma clang fp contract(off)
    const size_t n = rows * row_len;
    for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < n + rows; i += (size_t)gridDim.x * kBlock) {
        if (i < n) {
            w_out[i] = w[i] * scale[i / row_len];
        } else if (b_out) {
            const size_t r = i - n;
            float prod = (b ? b[r] : 0.0f) * scale[r];
            asm volatile("" : "+v"(prod));        // the product is rounded on its own: no fused multiply-add
            b_out[r] = prod + (shift ? shift[r] : 0.0f);
        }
    }
}

static inline bool aligned(const void *p, size_t a) { return ((uintptr_t)p % a) == 0; }

hipError_t launch_fold_scale(const float *w, const float *b, size_t rows, size_t row_len, const float *scale, const float *shift,
                             float *w_out, float *b_out, hipStream_t st)
{
    fold_scale_kernel<<<grid_for(rows * row_len + rows), kBlock, 0, st>>>(w, b, rows, row_len, scale, shift, w_out, b_out);
    return hipGetLastError();
}

hipError_t launch_quantize_rows(const float *x, int8_t *q, size_t rows, size_t row_len, const int32_t *frac, hipStream_t st)
{
    quantize_rows_kernel<<<grid_for(rows * row_len), kBlock, 0, st>>>(x, q, rows, row_len, frac);
    return hipGetLastError();
}

hipError_t launch_quantize_i32_rows(const float *x, int32_t *q, size_t rows, size_t row_len, const int32_t *frac, int frac_add,
                                    hipStream_t st)
{
    quantize_i32_rows_kernel<<<grid_for(rows * row_len), kBlock, 0, st>>>(x, q, rows, row_len, frac, frac_add);
    return hipGetLastError();
}

hipError_t launch_quantize(const float *x, int8_t *q, size_t n, int frac, hipStream_t st)
{
    float scale = ldexpf(1.0f, frac);
    if (aligned(x, 16) && aligned(q, 4)) {
        size_t n4 = n / 4;
        if (n4) quantize_vec4<<<grid_for(n4), kBlock, 0, st>>>((const float4 *)x, (uint32_t *)q, n4, scale);
        size_t tail = n - n4 * 4;
        if (tail) quantize_scalar<<<1, kBlock, 0, st>>>(x + n4 * 4, q + n4 * 4, tail, scale);
    } else {
        quantize_scalar<<<grid_for(n), kBlock, 0, st>>>(x, q, n, scale);
    }
    return hipGetLastError();
}

hipError_t launch_quantize_i32(const float *x, int32_t *q, size_t n, int frac, hipStream_t st)
{
    quantize_i32_kernel<<<grid_for(n), kBlock, 0, st>>>(x, q, n, ldexpf(1.0f, frac));
    return hipGetLastError();
}

static NpFmt make_npfmt(int nbits, int p, int frac_signed)
{
    NpFmt f;
    f.n = nbits;
    f.p = p;
    f.scale = ldexpf(1.0f, frac_signed);
    const int emax = p == nbits - 1 ? 1 : (1 << (nbits - 1 - p)) - 1;
    f.beta_max = p == nbits - 1 ? (float)((1 << (nbits - 1)) - 1) : ldexpf((float)((1 << (p + 1)) - 1), emax - 1);
    return f;
}

hipError_t launch_quantize_np(const float *x, uint8_t *q, size_t n, int nbits, int p, int frac, hipStream_t st)
{
    const NpFmt f = make_npfmt(nbits, p, frac);
    if (aligned(x, 16) && aligned(q, 4)) {
        size_t n4 = n / 4;
        if (n4) quantize_np_vec4<<<grid_for(n4), kBlock, 0, st>>>((const float4 *)x, (uint32_t *)q, n4, f);
        size_t tail = n - n4 * 4;
        if (tail) quantize_np_scalar<<<1, kBlock, 0, st>>>(x + n4 * 4, q + n4 * 4, tail, f);
    } else {
        quantize_np_scalar<<<grid_for(n), kBlock, 0, st>>>(x, q, n, f);
    }
    return hipGetLastError();
}

hipError_t launch_dequantize_np(const uint8_t *q, float *x, size_t n, int nbits, int p, int frac, hipStream_t st)
{
    const NpFmt f = make_npfmt(nbits, p, -frac);
    if (aligned(x, 16) && aligned(q, 4)) {
        size_t n4 = n / 4;
        if (n4) dequantize_np_vec4<<<grid_for(n4), kBlock, 0, st>>>((const uint32_t *)q, (float4 *)x, n4, f);
        size_t tail = n - n4 * 4;
        if (tail) dequantize_np_scalar<<<1, kBlock, 0, st>>>(q + n4 * 4, x + n4 * 4, tail, f);
    } else {
        dequantize_np_scalar<<<grid_for(n), kBlock, 0, st>>>(q, x, n, f);
    }
    return hipGetLastError();
}

hipError_t launch_dequantize(const int8_t *q, float *x, size_t n, int frac, hipStream_t st)
{
    float inv = ldexpf(1.0f, -frac);
    if (aligned(x, 16) && aligned(q, 4)) {
        size_t n4 = n / 4;
        if (n4) dequantize_vec4<<<grid_for(n4), kBlock, 0, st>>>((const uint32_t *)q, (float4 *)x, n4, inv);
        size_t tail = n - n4 * 4;
        if (tail) dequantize_scalar<<<1, kBlock, 0, st>>>(q + n4 * 4, x + n4 * 4, tail, inv);
    } else {
        dequantize_scalar<<<grid_for(n), kBlock, 0, st>>>(q, x, n, inv);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// eltwise_q: exact alignment to the finer scale, one add, one rounding
// ------------------------------------------------------------------------------------------

struct EltParams {
    int sa, sb;   // left shifts that bring a and b to the common fractional length F
    int s;        // F - f_y
    int relu;
};

__device__ __forceinline__ int elt_one(int a, int b, const EltParams &p, int &sum_out)
{
    int sum = a * (1 << p.sa) + b * (1 << p.sb);
    sum_out = sum;
    if (p.relu) sum = max(sum, 0);
    return requant8(sum, p.s);
}

template <bool kWantY, bool kWantAcc>
__global__ void __launch_bounds__(kBlock) eltwise_vec16(const uint4 *__restrict__ a, const uint4 *__restrict__ b,
                                                         uint4 *__restrict__ y, int4 *__restrict__ acc, size_t n16,
                                                         EltParams p)
{
    for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < n16; i += (size_t)gridDim.x * kBlock) {
        uint4 va = a[i], vb = b[i];
        const uint32_t wa[4] = {va.x, va.y, va.z, va.w};
        const uint32_t wb[4] = {vb.x, vb.y, vb.z, vb.w};
        uint32_t out[4];
#pragma unroll
        for (int j = 0; j < 4; j++) {
            int s0, s1, s2, s3;
            int r0 = elt_one(byte_of(wa[j], 0), byte_of(wb[j], 0), p, s0);
            int r1 = elt_one(byte_of(wa[j], 1), byte_of(wb[j], 1), p, s1);
            int r2 = elt_one(byte_of(wa[j], 2), byte_of(wb[j], 2), p, s2);
            int r3 = elt_one(byte_of(wa[j], 3), byte_of(wb[j], 3), p, s3);
            out[j] = pack4(r0, r1, r2, r3);
            if (kWantAcc) acc[i * 4 + j] = make_int4(s0, s1, s2, s3);
        }
        if (kWantY) y[i] = make_uint4(out[0], out[1], out[2], out[3]);
    }
}

// The common case - int8 result only, final shift in [0, 23] - with the branch-free rounding
// shift of the convolution epilogue: per element two sign-extracting field reads, a shift, a
// shift-add, then clamp / rounding bit / add / shift-into-byte.
__global__ void __launch_bounds__(kBlock) eltwise_fast16(const uint4 *__restrict__ a, const uint4 *__restrict__ b,
                                                          uint4 *__restrict__ y, size_t n16, EltParams p)
{
    Requant rq;
    rq.init(p.s, p.relu);
    for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < n16; i += (size_t)gridDim.x * kBlock) {
        const uint4 va = a[i], vb = b[i];
        const uint32_t wa[4] = {va.x, va.y, va.z, va.w};
        const uint32_t wb[4] = {vb.x, vb.y, vb.z, vb.w};
        uint32_t out[4];
#pragma unroll
        for (int j = 0; j < 4; j++) {
            int t[4];
#pragma unroll
            for (int e = 0; e < 4; e++)
                t[e] = (int)((unsigned)byte_of(wa[j], e) << p.sa) + (int)((unsigned)byte_of(wb[j], e) << p.sb);
            out[j] = rq.fast_four(t[0], t[1], t[2], t[3]);
        }
        y[i] = make_uint4(out[0], out[1], out[2], out[3]);
    }
}

__global__ void __launch_bounds__(kBlock) eltwise_scalar(const int8_t *__restrict__ a, const int8_t *__restrict__ b,
                                                          int8_t *__restrict__ y, int32_t *__restrict__ acc, size_t n,
                                                          EltParams p)
{
    for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (size_t)gridDim.x * kBlock) {
        int sum;
        int r = elt_one(a[i], b[i], p, sum);
        if (acc) acc[i] = sum;
        if (y) y[i] = (int8_t)r;
    }
}

hipError_t launch_eltwise(const int8_t *a, int fa, const int8_t *b, int fb, int8_t *y, int fy, int32_t *acc, size_t n,
                          int relu, hipStream_t st)
{
    int F = fa > fb ? fa : fb;
    EltParams p{F - fa, F - fb, F - fy, relu};
    bool vec = aligned(a, 16) && aligned(b, 16) && (!y || aligned(y, 16)) && (!acc || aligned(acc, 16));
    size_t n16 = vec ? n / 16 : 0;
    if (n16) {
        int g = grid_for(n16);
        if (y && !acc && p.s >= 0 && p.s <= 23) eltwise_fast16<<<g, kBlock, 0, st>>>((const uint4 *)a, (const uint4 *)b, (uint4 *)y, n16, p);
        else if (y && acc) eltwise_vec16<true, true><<<g, kBlock, 0, st>>>((const uint4 *)a, (const uint4 *)b, (uint4 *)y, (int4 *)acc, n16, p);
        else if (y) eltwise_vec16<true, false><<<g, kBlock, 0, st>>>((const uint4 *)a, (const uint4 *)b, (uint4 *)y, nullptr, n16, p);
        else eltwise_vec16<false, true><<<g, kBlock, 0, st>>>((const uint4 *)a, (const uint4 *)b, nullptr, (int4 *)acc, n16, p);
    }
    size_t done = n16 * 16;
    if (n > done)
        eltwise_scalar<<<grid_for(n - done), kBlock, 0, st>>>(a + done, b + done, y ? y + done : nullptr,
                                                               acc ? acc + done : nullptr, n - done, p);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// concat_q: one launch, every lane produces VEC output bytes of one branch
// ------------------------------------------------------------------------------------------

struct ConcatParams {
    const int8_t *x[8];
    int C[8];       // channels of each branch
    int off[9];     // channel offset of each branch in y; off[nb] = total
    int s[8];       // f_i - f_y
    int nb;
};

// ldy: bytes between consecutive pixels of y (>= the branches' channels together)
template <int VEC>
__global__ void __launch_bounds__(kBlock) concat_kernel(ConcatParams p, int8_t *__restrict__ y, size_t pixels, int ldy)
{
    const int Ct = p.off[p.nb];
    const int per_px = Ct / VEC;
    const size_t total = pixels * (size_t)per_px;
    for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < total; i += (size_t)gridDim.x * kBlock) {
        size_t px = i / per_px;
        int c = (int)(i - px * per_px) * VEC;
        int br = 0;
#pragma unroll
        for (int j = 1; j < 8; j++)
            if (j < p.nb && c >= p.off[j]) br = j;
        const int8_t *src = p.x[br] + px * (size_t)p.C[br] + (c - p.off[br]);
        int8_t *dst = y + px * (size_t)ldy + c;
        const int s = p.s[br];
        if (VEC == 16) {
            uint4 v = *(const uint4 *)src;
            uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int j = 0; j < 4; j++)
                w[j] = pack4(requant8(byte_of(w[j], 0), s), requant8(byte_of(w[j], 1), s),
                             requant8(byte_of(w[j], 2), s), requant8(byte_of(w[j], 3), s));
            *(uint4 *)dst = make_uint4(w[0], w[1], w[2], w[3]);
        } else if (VEC == 4) {
            uint32_t w = *(const uint32_t *)src;
            *(uint32_t *)dst = pack4(requant8(byte_of(w, 0), s), requant8(byte_of(w, 1), s),
                                     requant8(byte_of(w, 2), s), requant8(byte_of(w, 3), s));
        } else {
            *dst = (int8_t)requant8(*src, s);
        }
    }
}

hipError_t launch_concat(int nb, const int8_t *const *xs, const int *Cs, const int *fs, int8_t *y, int ldy, int fy,
                         size_t pixels, hipStream_t st)
{
    ConcatParams p{};
    p.nb = nb;
    int off = 0;
    int vec = 16;
    if (!aligned(y, 16) || ldy % 16) vec = (aligned(y, 4) && ldy % 4 == 0) ? 4 : 1;
    for (int i = 0; i < nb; i++) {
        p.x[i] = xs[i];
        p.C[i] = Cs[i];
        p.off[i] = off;
        p.s[i] = fs[i] - fy;
        off += Cs[i];
        while (vec > 1 && (Cs[i] % vec || !aligned(xs[i], vec))) vec /= 4;
    }
    for (int i = nb; i <= 8; i++) p.off[i] = off;
    size_t total = pixels * (size_t)(off / vec);
    int g = grid_for(total);
    if (vec == 16) concat_kernel<16><<<g, kBlock, 0, st>>>(p, y, pixels, ldy);
    else if (vec == 4) concat_kernel<4><<<g, kBlock, 0, st>>>(p, y, pixels, ldy);
    else concat_kernel<1><<<g, kBlock, 0, st>>>(p, y, pixels, ldy);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// pool_q
// ------------------------------------------------------------------------------------------

struct PoolParams {
    int N, H, W, C, P, Q, k, stride, pad;
    int mode;   // 0 max, 1 avg
    int d;      // f_out - f_in
};

// (sum * 2^d) / (k*k) rounded to nearest, ties to even, clamped.  |sum| <= 128 * 4096.
__device__ __forceinline__ int avg_round(int sum, int win, int d)
{
    if (d >= 32) return sum == 0 ? 0 : (sum > 0 ? 127 : -127);
    if (d <= -40) return 0;
    long long num = sum, den = win;
    if (d >= 0) num <<= d; else den <<= -d;
    long long t = num / den;
    long long rem = num - t * den;
    if (rem < 0) { t -= 1; rem += den; }          // floor
    if (2 * rem > den || (2 * rem == den && (t & 1))) t += 1;
    t = t > 127 ? 127 : (t < -127 ? -127 : t);
    return (int)t;
}

template <int VEC>
__global__ void __launch_bounds__(kBlock) pool_kernel(const int8_t *__restrict__ x, int8_t *__restrict__ y, PoolParams p)
{
    const int cv = p.C / VEC;
    const size_t total = (size_t)p.N * p.P * p.Q * cv;
    for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < total; i += (size_t)gridDim.x * kBlock) {
        int c = (int)(i % cv) * VEC;
        size_t px = i / cv;
        int q = (int)(px % p.Q);
        size_t t = px / p.Q;
        int pp = (int)(t % p.P);
        int n = (int)(t / p.P);
        int acc[VEC];
#pragma unroll
        for (int j = 0; j < VEC; j++) acc[j] = p.mode == 0 ? -1000 : 0;
        for (int r = 0; r < p.k; r++) {
            int ih = pp * p.stride - p.pad + r;
            if (ih < 0 || ih >= p.H) continue;
            for (int s = 0; s < p.k; s++) {
                int iw = q * p.stride - p.pad + s;
                if (iw < 0 || iw >= p.W) continue;
                const int8_t *src = x + (((size_t)n * p.H + ih) * p.W + iw) * p.C + c;
                int v[VEC];
                if (VEC == 16) {
                    uint4 u = *(const uint4 *)src;
                    uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
                    for (int j = 0; j < 16; j++) v[j] = byte_of(w[j / 4], j % 4);
                } else if (VEC == 4) {
                    uint32_t w = *(const uint32_t *)src;
#pragma unroll
                    for (int j = 0; j < 4; j++) v[j] = byte_of(w, j);
                } else {
                    v[0] = *src;
                }
                if (p.mode == 0) {
#pragma unroll
                    for (int j = 0; j < VEC; j++) acc[j] = max(acc[j], v[j]);
                } else {
#pragma unroll
                    for (int j = 0; j < VEC; j++) acc[j] += v[j];
                }
            }
        }
        int out[VEC];
#pragma unroll
        for (int j = 0; j < VEC; j++)
            out[j] = p.mode == 0 ? requant8(acc[j], -p.d) : avg_round(acc[j], p.k * p.k, p.d);
        int8_t *dst = y + px * (size_t)p.C + c;
        if (VEC == 16) {
            *(uint4 *)dst = make_uint4(pack4(out[0], out[1], out[2], out[3]), pack4(out[4], out[5], out[6], out[7]),
                                       pack4(out[8], out[9], out[10], out[11]), pack4(out[12], out[13], out[14], out[15]));
        } else if (VEC == 4) {
            *(uint32_t *)dst = pack4(out[0], out[1], out[2], out[3]);
        } else {
            *dst = (int8_t)out[0];
        }
    }
}

// 3x3 max pooling, 16 channels per lane: window positions in the padding are replaced by the nearest
// position inside the image, which lies in the same window (pad < k), so the nine 16-byte loads are
// unconditional and all in flight together; the running maxima are kept as one integer per channel and
// updated straight from the bytes of the loaded words (sub-dword operand select with sign extension:
// one instruction per byte and window position, no unpacking).
struct MaxPool3Params {
    PoolParams p;
    int cv;              // C / 16
    int total;           // N * P * Q * cv (below 2^31)
    FastDiv div_cv, div_q, div_p;
};

template <int E>
__device__ __forceinline__ int max_with_byte(int acc, uint32_t w)
{
    if constexpr (E == 0) asm("v_max_i32_sdwa %0, %1, sext(%2) dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_0" : "=v"(acc) : "v"(acc), "v"(w));
    else if constexpr (E == 1) asm("v_max_i32_sdwa %0, %1, sext(%2) dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_1" : "=v"(acc) : "v"(acc), "v"(w));
    else if constexpr (E == 2) asm("v_max_i32_sdwa %0, %1, sext(%2) dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_2" : "=v"(acc) : "v"(acc), "v"(w));
    else asm("v_max_i32_sdwa %0, %1, sext(%2) dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_3" : "=v"(acc) : "v"(acc), "v"(w));
    return acc;
}

__global__ void __launch_bounds__(kBlock) maxpool3_kernel(const int8_t *__restrict__ x, int8_t *__restrict__ y, MaxPool3Params prm)
{
    const PoolParams &p = prm.p;
    for (int i = blockIdx.x * kBlock + threadIdx.x; i < prm.total; i += gridDim.x * kBlock) {
        const int px = fastdiv(i, prm.div_cv);
        const int c = (i - px * prm.cv) * 16;
        const int t = fastdiv(px, prm.div_q);
        const int q = px - t * p.Q;
        const int n = fastdiv(t, prm.div_p);
        const int pp = t - n * p.P;
        uint4 u[9];
#pragma unroll
        for (int r = 0; r < 3; r++) {
            const int ih = min(max(pp * p.stride - p.pad + r, 0), p.H - 1);
#pragma unroll
            for (int s2 = 0; s2 < 3; s2++) {
                const int iw = min(max(q * p.stride - p.pad + s2, 0), p.W - 1);
                u[r * 3 + s2] = *(const uint4 *)(x + (((size_t)n * p.H + ih) * p.W + iw) * p.C + c);
            }
        }
        int acc[16];
#pragma unroll
        for (int j = 0; j < 16; j++) acc[j] = -128;
#pragma unroll
        for (int k = 0; k < 9; k++) {
            const uint32_t w[4] = {u[k].x, u[k].y, u[k].z, u[k].w};
#pragma unroll
            for (int j = 0; j < 4; j++) {
                acc[4 * j + 0] = max_with_byte<0>(acc[4 * j + 0], w[j]);
                acc[4 * j + 1] = max_with_byte<1>(acc[4 * j + 1], w[j]);
                acc[4 * j + 2] = max_with_byte<2>(acc[4 * j + 2], w[j]);
                acc[4 * j + 3] = max_with_byte<3>(acc[4 * j + 3], w[j]);
            }
        }
        int out[16];
#pragma unroll
        for (int j = 0; j < 16; j++) out[j] = p.d == 0 ? max(acc[j], -127) : requant8(acc[j], -p.d);
        *(uint4 *)(y + (size_t)px * p.C + c) = make_uint4(pack4(out[0], out[1], out[2], out[3]), pack4(out[4], out[5], out[6], out[7]),
                                                         pack4(out[8], out[9], out[10], out[11]), pack4(out[12], out[13], out[14], out[15]));
    }
}

// Global average pooling (the window is the whole image, one output pixel): a lane sums 4 channels over
// all H*W pixels, seven loads in flight at a time, bytes added straight out of the loaded words.
template <int E>
__device__ __forceinline__ int add_byte(int acc, uint32_t w)
{
    if constexpr (E == 0) asm("v_add_u32_sdwa %0, %1, sext(%2) dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_0" : "=v"(acc) : "v"(acc), "v"(w));
    else if constexpr (E == 1) asm("v_add_u32_sdwa %0, %1, sext(%2) dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_1" : "=v"(acc) : "v"(acc), "v"(w));
    else if constexpr (E == 2) asm("v_add_u32_sdwa %0, %1, sext(%2) dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_2" : "=v"(acc) : "v"(acc), "v"(w));
    else asm("v_add_u32_sdwa %0, %1, sext(%2) dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_3" : "=v"(acc) : "v"(acc), "v"(w));
    return acc;
}

__global__ void __launch_bounds__(kBlock) avgpool_global_kernel(const int8_t *__restrict__ x, int8_t *__restrict__ y, int N, int pixels,
                                                                 int C, int d)
{
    const int cw = C / 4;
    const int i = blockIdx.x * kBlock + threadIdx.x;
    if (i >= N * cw) return;
    const int n = i / cw, c = (i - n * cw) * 4;
    const uint32_t *src = (const uint32_t *)(x + (size_t)n * pixels * C + c);
    const size_t step = (size_t)C / 4;            // words between consecutive pixels
    int acc[4] = {0, 0, 0, 0};
    int px = 0;
    for (; px + 7 <= pixels; px += 7) {
        uint32_t w[7];
#pragma unroll
        for (int j = 0; j < 7; j++) w[j] = src[(size_t)(px + j) * step];
#pragma unroll
        for (int j = 0; j < 7; j++) {
            acc[0] = add_byte<0>(acc[0], w[j]); acc[1] = add_byte<1>(acc[1], w[j]);
            acc[2] = add_byte<2>(acc[2], w[j]); acc[3] = add_byte<3>(acc[3], w[j]);
        }
    }
    for (; px < pixels; px++) {
        const uint32_t w = src[(size_t)px * step];
        acc[0] = add_byte<0>(acc[0], w); acc[1] = add_byte<1>(acc[1], w);
        acc[2] = add_byte<2>(acc[2], w); acc[3] = add_byte<3>(acc[3], w);
    }
    *(uint32_t *)(y + (size_t)n * C + c) = pack4(avg_round(acc[0], pixels, d), avg_round(acc[1], pixels, d),
                                                 avg_round(acc[2], pixels, d), avg_round(acc[3], pixels, d));
}

hipError_t launch_pool(const int8_t *x, int8_t *y, int mode, int N, int H, int W, int C, int P, int Q, int k, int stride,
                       int pad, int fin, int fout, hipStream_t st)
{
    PoolParams p{N, H, W, C, P, Q, k, stride, pad, mode, fout - fin};
    if (mode == 1 && k == H && k == W && pad == 0 && C % 4 == 0 && aligned(x, 4) && aligned(y, 4) &&
        (long long)N * (C / 4) < (1LL << 31) - kBlock) {
        const int lanes = N * (C / 4);
        avgpool_global_kernel<<<(lanes + kBlock - 1) / kBlock, kBlock, 0, st>>>(x, y, N, H * W, C, fout - fin);
        return hipGetLastError();
    }
    if (mode == 0 && k == 3 && C % 16 == 0 && aligned(x, 16) && aligned(y, 16) &&
        (long long)N * P * Q * (C / 16) < (1LL << 31) - 256LL * 16 * kBlock && (long long)N * P * Q * (C / 16) >= 16 * 1024) {
        MaxPool3Params prm;
        prm.p = p;
        prm.cv = C / 16;
        prm.total = (int)((long long)N * P * Q * prm.cv);
        prm.div_cv = make_fastdiv(prm.cv);
        prm.div_q = make_fastdiv(Q);
        prm.div_p = make_fastdiv(P);
        maxpool3_kernel<<<grid_for((size_t)prm.total), kBlock, 0, st>>>(x, y, prm);
        return hipGetLastError();
    }
    int vec = 16;
    while (vec > 1 && (C % vec || !aligned(x, vec) || !aligned(y, vec))) vec /= 4;
    // few outputs (a global pool): narrower lanes give the machine four times the wavefronts
    if (vec == 16 && (size_t)N * P * Q * (C / 16) < (size_t)256 * 1024) vec = 4;
    size_t total = (size_t)N * P * Q * (C / vec);
    int g = grid_for(total);
    if (vec == 16) pool_kernel<16><<<g, kBlock, 0, st>>>(x, y, p);
    else if (vec == 4) pool_kernel<4><<<g, kBlock, 0, st>>>(x, y, p);
    else pool_kernel<1><<<g, kBlock, 0, st>>>(x, y, p);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// max |.| reductions.  The result scalar is first cleared by a one-lane kernel (not a memset,
// so that the sequence can be captured into a HIP graph), then every workgroup folds its
// share with one atomic max.  Non-negative floats order like their bit patterns.
// ------------------------------------------------------------------------------------------

__global__ void clear_u32(uint32_t *p) { *p = 0u; }

__device__ __forceinline__ void block_max_to(uint32_t v, uint32_t *out)
{
    __shared__ uint32_t part[kBlock / kWave];
    v = wave_max_u32(v);
    if ((threadIdx.x & (kWave - 1)) == 0) part[threadIdx.x / kWave] = v;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t m = part[0];
#pragma unroll
        for (int i = 1; i < kBlock / kWave; i++) m = max(m, part[i]);
        if (m) atomicMax(out, m);
    }
}

__global__ void __launch_bounds__(kBlock) absmax_f32_kernel(const float *__restrict__ x, size_t n, uint32_t *out)
{
    uint32_t m = 0;
    for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (size_t)gridDim.x * kBlock) {
        float a = fabsf(x[i]);
        if (a == a) m = max(m, __float_as_uint(a));   // skip NaN
    }
    block_max_to(m, out);
}

__device__ __forceinline__ uint32_t magnitude(int v, int relu)
{
    return v >= 0 ? (uint32_t)v : (relu ? 0u : (uint32_t)0 - (uint32_t)v);
}

// 16 bytes per lane and access where the array is aligned for it; the first lanes of the launch take the tail
__global__ void __launch_bounds__(kBlock) absmax_i32_kernel(const int32_t *__restrict__ x, size_t n, int relu, uint32_t *out)
{
    uint32_t m = 0;
    const size_t t = (size_t)blockIdx.x * kBlock + threadIdx.x, threads = (size_t)gridDim.x * kBlock;
    size_t n4 = 0;
    if (((uintptr_t)x & 15) == 0) {
        n4 = n / 4;
        const int4 *x4 = (const int4 *)x;
        for (size_t i = t; i < n4; i += threads) {
            const int4 v = x4[i];
            m = max(max(m, magnitude(v.x, relu)), max(magnitude(v.y, relu), max(magnitude(v.z, relu), magnitude(v.w, relu))));
        }
    }
    for (size_t i = n4 * 4 + t; i < n; i += threads) m = max(m, magnitude(x[i], relu));
    block_max_to(m, out);
}

// The same maximum per channel of an [pixels][K] array.  Thread t of the launch keeps channel
// t % K and walks the pixel rows t / K, t / K + (threads / K), ... (neighbouring threads read
// neighbouring channels of one row); with more channels than threads a thread takes several.
__global__ void clear_u32_n(uint32_t *p, int n)
{
    const int i = blockIdx.x * kBlock + threadIdx.x;
    if (i < n) p[i] = 0u;
}

__global__ void __launch_bounds__(kBlock) absmax_i32_channels_kernel(const int32_t *__restrict__ x, size_t pixels, int K, int relu,
                                                                      uint32_t *out)
{
    const size_t threads = (size_t)gridDim.x * kBlock;
    const size_t t = (size_t)blockIdx.x * kBlock + threadIdx.x;
    auto fold = [&](size_t k, size_t first, size_t step) {
        uint32_t m = 0;
        for (size_t p = first; p < pixels; p += step) {
            const int v = x[p * (size_t)K + k];
            const uint32_t a = v >= 0 ? (uint32_t)v : (relu ? 0u : (uint32_t)0 - (uint32_t)v);
            m = max(m, a);
        }
        if (m) atomicMax(out + k, m);
    };
    if (threads >= (size_t)K) {
        const size_t rows = threads / (size_t)K;      // pixel rows in flight per pass
        if (t / (size_t)K < rows) fold(t % (size_t)K, t / (size_t)K, rows);
    } else {
        for (size_t k = t; k < (size_t)K; k += threads) fold(k, 0, 1);
    }
}

// max |.| of every row of x[rows][row_len]: one workgroup per row at a time, no atomics
__global__ void __launch_bounds__(kBlock) absmax_f32_rows_kernel(const float *__restrict__ x, size_t rows, size_t row_len, uint32_t *out)
{
    __shared__ uint32_t part[kBlock / kWave];
    for (size_t r = blockIdx.x; r < rows; r += gridDim.x) {
        uint32_t m = 0;
        for (size_t i = threadIdx.x; i < row_len; i += kBlock) {
            float a = fabsf(x[r * row_len + i]);
            if (a == a) m = max(m, __float_as_uint(a));   // skip NaN
        }
        m = wave_max_u32(m);
        if ((threadIdx.x & (kWave - 1)) == 0) part[threadIdx.x / kWave] = m;
        __syncthreads();
        if (threadIdx.x == 0) {
            uint32_t t = part[0];
#pragma unroll
            for (int i = 1; i < kBlock / kWave; i++) t = max(t, part[i]);
            out[r] = t;
        }
        __syncthreads();
    }
}

hipError_t launch_absmax_f32_rows(const float *x, size_t rows, size_t row_len, float *out, hipStream_t st)
{
    size_t g = rows < 4096 ? rows : 4096;
    absmax_f32_rows_kernel<<<(unsigned)g, kBlock, 0, st>>>(x, rows, row_len, (uint32_t *)out);
    return hipGetLastError();
}

hipError_t launch_absmax_f32(const float *x, size_t n, float *out, hipStream_t st)
{
    clear_u32<<<1, 1, 0, st>>>((uint32_t *)out);
    if (n) absmax_f32_kernel<<<grid_for(n), kBlock, 0, st>>>(x, n, (uint32_t *)out);
    return hipGetLastError();
}

hipError_t launch_absmax_i32(const int32_t *x, size_t n, int relu, uint32_t *out, hipStream_t st)
{
    clear_u32<<<1, 1, 0, st>>>(out);
    if (n) absmax_i32_kernel<<<grid_for(n), kBlock, 0, st>>>(x, n, relu, out);
    return hipGetLastError();
}

// Histogram of |x| >> shift over kHistBins bins (Algorithm 1, first step): each workgroup counts its
// share in LDS and adds its non-empty bins to the result, which a small kernel cleared first.  A
// magnitude beyond the last bin (a shift smaller than the caller was told to use) lands in the last bin.
constexpr int kHistBins = 2048;

__global__ void __launch_bounds__(kBlock) hist_i32_kernel(const int32_t *__restrict__ x, size_t n, int relu, int shift, uint32_t *out)
{
    __shared__ uint32_t bins[kHistBins];
    for (int i = threadIdx.x; i < kHistBins; i += kBlock) bins[i] = 0u;
    __syncthreads();
    const size_t t = (size_t)blockIdx.x * kBlock + threadIdx.x, threads = (size_t)gridDim.x * kBlock;
    auto count = [&](int v) { atomicAdd(&bins[min(magnitude(v, relu) >> shift, (uint32_t)(kHistBins - 1))], 1u); };
    size_t n4 = 0;
    if (((uintptr_t)x & 15) == 0) {
        n4 = n / 4;
        const int4 *x4 = (const int4 *)x;
        for (size_t i = t; i < n4; i += threads) {
            const int4 v = x4[i];
            count(v.x); count(v.y); count(v.z); count(v.w);
        }
    }
    for (size_t i = n4 * 4 + t; i < n; i += threads) count(x[i]);
    __syncthreads();
    for (int i = threadIdx.x; i < kHistBins; i += kBlock)
        if (bins[i]) atomicAdd(out + i, bins[i]);
}

hipError_t launch_hist_i32(const int32_t *x, size_t n, int relu, int shift, uint32_t *out, hipStream_t st)
{
    clear_u32_n<<<kHistBins / kBlock, kBlock, 0, st>>>(out, kHistBins);
    if (n) {
        int g = grid_for(n);
        if (g > 1024) g = 1024;                 // every workgroup ends with up to 2048 atomics on the result
        hist_i32_kernel<<<g, kBlock, 0, st>>>(x, n, relu, shift, out);
    }
    return hipGetLastError();
}

hipError_t launch_absmax_i32_channels(const int32_t *x, size_t pixels, int K, int relu, uint32_t *out, hipStream_t st)
{
    clear_u32_n<<<(K + kBlock - 1) / kBlock, kBlock, 0, st>>>(out, K);
    if (pixels) absmax_i32_channels_kernel<<<grid_for(pixels * (size_t)K), kBlock, 0, st>>>(x, pixels, K, relu, out);
    return hipGetLastError();
}

}  // namespace dfq
