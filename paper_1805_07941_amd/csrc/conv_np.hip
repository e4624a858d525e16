// Convolution on 8-bit dynamic floating-point codes with up to twelve-bit integers (Sec. 2.1: (8, p) with p >= 4,
// |beta| <= beta_max(8, 4) = 1984), exact as Eq. 6 asks for, on the int8 matrix cores.
//
// Eq. 6 sums the integer products beta_x * beta_w without loss; for (8, 4) operands Eq. 8 gives 36 bits for the deepest
// reduction of a ResNet-50-shaped network (3 x 3 x 512 terms), and Eq. 9 allows a 32-bit accumulator 545 terms only.
// The chip has no matrix instruction with 12-bit operands, but the sum splits exactly into sums it has: write every
// operand in two sign-and-magnitude digits of base 64,
//     beta = 64 * h + l,   |h| <= 31, |l| <= 63   (both of the sign of beta),
// then  sum beta_x beta_w = 4096 * A + 64 * B + C  with  A = sum h_x h_w,  B = sum (h_x l_w + l_x h_w),  C = sum l_x l_w:
// four int8 matrix products per block into three int32 accumulator sets (|B| <= 3906 per term: 64 A + B stays below
// 2^30 for reductions of up to 13 000 terms, checked by the launcher); once per tile they are combined,
//     sum = 64 * (64 * A + B) + C,
// the bias is added, ReLU applied, and the value times 2^-shift is rounded ONCE to the output format: nearest
// representable integer, ties to the even significand field, saturation at +-beta_max.
// (B = D - A - C with D = sum (h_x + l_x)(h_w + l_w), |h + l| <= 94, needs three products only; built and measured
// 8-10 % slower: the sums h + l are a fifth operand plane through LDS for the weights and a byte-wise add per use
// for the activations, and the kernel is not bound by the matrix pipe alone.)
//
// Tensors of this path travel between kernels as their two digit planes (int8 each, NHWC / [K][R][S][C]): a code is
// decoded once, by the kernel that produces it (np_digits_kernel for inputs and weights, the epilogue here for
// activations), not once per use.  The epilogue writes the digit planes of its result for the next layer and, if
// asked, the codes themselves.
//
// conv_np_mfma_kernel: implicit GEMM, one tile of BP pixels x BC channels per workgroup of four wavefronts, the
// reduction axis in 64-byte steps through a ring of two or three LDS stages of 2 (BP + BC) rows filled by direct
// global -> LDS loads that many steps ahead; rows are 64 bytes with the 16-byte pieces XOR-swizzled as in the int8
// kernels; two or three workgroups share a compute unit.  With ADD the element-wise add that follows the layer
// (Eq. 10) runs in the epilogue.
// conv_np_direct_kernel: one output per lane, any geometry (groups, C not a multiple of 64); also the calibration maxima.
// Further down: the add, pooling and the first layer's space-to-depth packing on digit planes.
#include <type_traits>

#include "conv_ring.hpp"

namespace dfq {

namespace {

// ---- scalar pieces ------------------------------------------------------------------------------------------------

struct NpRound {
    int shift;          // f_x + f_w - f_y
    int p;              // significand bits of the output format
    float beta_max;     // Eq. 5 for the output format (at most 12 bits: exact in float)
    int relu;
};

// The accumulator value v times 2^-shift, rounded to the nearest integer representable with p + 1 significant bits
// (step 1 below 2^(p+1)), ties to the even significand, magnitude clamped to beta_max.  |v| < 2^62.
// The magnitude is first cut to 23 bits with a sticky bit for what was cut (the rounding position is at least 15
// bits above it), which a float holds exactly; the rest is the conversion of a float to the format: scale by an exact
// power of two so that the step becomes 1, round to nearest even, scale back.
__device__ __forceinline__ int np_round_acc(long long v, const NpRound &f)
{
    if (f.relu && v < 0) v = 0;
    const bool neg = v < 0;
    const unsigned long long a = neg ? (unsigned long long)(-v) : (unsigned long long)v;
    const int lz = a ? __clzll((long long)a) : 64;
    const int t = max(41 - lz, 0);                       // bits to cut: the leading bit goes to position 22
    unsigned m = (unsigned)(a >> t);
    if (((unsigned long long)m << t) != a) m |= 1u;      // sticky
    float x = ldexpf((float)m, t - f.shift);
    x = fminf(x, f.beta_max);
    const int ex = (int)((__float_as_uint(x) >> 23) & 0xffu) - 127;
    const int k = max(ex - f.p, 0);
    float r = ldexpf(__builtin_rintf(ldexpf(x, -k)), k);
    r = fminf(r, f.beta_max);
    const int beta = (int)r;
    return neg ? -beta : beta;
}

// The same rounding for the matrix-core kernel's epilogue when 7 <= shift <= 36, through the double-precision adder.  The
// accumulator is V = 64 * T + c with T and c int32 (|V| < 2^37): a double holds it exactly.  With e the binade of |V| the
// result's step is 2^(e' - p) in units of V, e' = max(e, p + shift) (below 2^(p+1) output units the step is one unit).
// Adding M = 1.5 * 2^(e' + 52 - p) puts V into a binade whose unit in the last place is exactly that step, so the adder's
// own round-to-nearest-even does the rounding (M is an even multiple of the step: the parity of the sum's last bit is the
// parity of the quotient q = round(V / step), i.e. of the significand field), and q is the low word of the sum's bit
// pattern (the mantissa field holds 2^51 + q).  The result is q * 2^k, k = e' - p - shift.  Values beyond every format
// of this path (e' capped at p + shift + 11 - p: at least 2^12 output units) still give a q * 2^k >= 2^12 that fits 31
// bits because shift >= 7, and the clamp that follows cuts them.  Returns the signed integer before the clamp.
struct NpFast {
    unsigned base_b;     // biased exponent of the smallest e': 1023 + p + shift
    unsigned top_b;      // base_b + 11 - p
    unsigned m_const;    // ((52 - p) << 20) | 0x80000: exponent offset and the mantissa bit of the factor 1.5
    int bmax;
};

__device__ __forceinline__ int np_round_fast(int T, int c, const NpFast &f)
{
    const double x = __builtin_fma((double)T, 64.0, (double)c);
    const unsigned e_b = __builtin_amdgcn_ubfe((unsigned)__double2hiint(x), 20u, 11u);
    unsigned eb;
    asm("v_med3_u32 %0, %1, %2, %3" : "=v"(eb) : "v"(e_b), "s"(f.base_b), "v"(f.top_b));      // clamp to [base_b, top_b]
    const double M = __hiloint2double((int)((eb << 20) + f.m_const), 0);
    const int q = __double2loint(x + M);
    return q << (eb - f.base_b);
}

// The conversion of a 32-bit sum t (|t| < 2^30) times 2^-shift, 0 <= shift <= 31, by the same device: (double)t is exact.
__device__ __forceinline__ int np_round_fast_i32(int t, const NpFast &f)
{
    const double x = (double)t;
    const unsigned e_b = __builtin_amdgcn_ubfe((unsigned)__double2hiint(x), 20u, 11u);
    unsigned eb;
    asm("v_med3_u32 %0, %1, %2, %3" : "=v"(eb) : "v"(e_b), "s"(f.base_b), "v"(f.top_b));
    const double M = __hiloint2double((int)((eb << 20) + f.m_const), 0);
    const int q = __double2loint(x + M);
    return q << (eb - f.base_b);
}

// byte E of w = low byte of (v >> sh), of (v & msk), of (x - y): the operation writes its result's low byte straight
// into the packed word (sub-dword destination select), the other bytes are kept
template <int E>
__device__ __forceinline__ void put_shr(uint32_t &w, unsigned sh, unsigned v)
{
    if constexpr (E == 0) asm("v_lshrrev_b32_sdwa %0, %1, %2 dst_sel:BYTE_0 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD" : "+v"(w) : "v"(sh), "v"(v));
    if constexpr (E == 1) asm("v_lshrrev_b32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD" : "+v"(w) : "v"(sh), "v"(v));
    if constexpr (E == 2) asm("v_lshrrev_b32_sdwa %0, %1, %2 dst_sel:BYTE_2 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD" : "+v"(w) : "v"(sh), "v"(v));
    if constexpr (E == 3) asm("v_lshrrev_b32_sdwa %0, %1, %2 dst_sel:BYTE_3 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD" : "+v"(w) : "v"(sh), "v"(v));
}
template <int E>
__device__ __forceinline__ void put_ashr(uint32_t &w, unsigned sh, int v)
{
    if constexpr (E == 0) asm("v_ashrrev_i32_sdwa %0, %1, %2 dst_sel:BYTE_0 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD" : "+v"(w) : "v"(sh), "v"(v));
    if constexpr (E == 1) asm("v_ashrrev_i32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD" : "+v"(w) : "v"(sh), "v"(v));
    if constexpr (E == 2) asm("v_ashrrev_i32_sdwa %0, %1, %2 dst_sel:BYTE_2 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD" : "+v"(w) : "v"(sh), "v"(v));
    if constexpr (E == 3) asm("v_ashrrev_i32_sdwa %0, %1, %2 dst_sel:BYTE_3 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD" : "+v"(w) : "v"(sh), "v"(v));
}
template <int E>
__device__ __forceinline__ void put_and(uint32_t &w, unsigned msk, unsigned v)
{
    if constexpr (E == 0) asm("v_and_b32_sdwa %0, %1, %2 dst_sel:BYTE_0 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD" : "+v"(w) : "v"(msk), "v"(v));
    if constexpr (E == 1) asm("v_and_b32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD" : "+v"(w) : "v"(msk), "v"(v));
    if constexpr (E == 2) asm("v_and_b32_sdwa %0, %1, %2 dst_sel:BYTE_2 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD" : "+v"(w) : "v"(msk), "v"(v));
    if constexpr (E == 3) asm("v_and_b32_sdwa %0, %1, %2 dst_sel:BYTE_3 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD" : "+v"(w) : "v"(msk), "v"(v));
}
template <int E>
__device__ __forceinline__ void put_sub(uint32_t &w, unsigned x, unsigned y)
{
    if constexpr (E == 0) asm("v_sub_u32_sdwa %0, %1, %2 dst_sel:BYTE_0 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD" : "+v"(w) : "v"(x), "v"(y));
    if constexpr (E == 1) asm("v_sub_u32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD" : "+v"(w) : "v"(x), "v"(y));
    if constexpr (E == 2) asm("v_sub_u32_sdwa %0, %1, %2 dst_sel:BYTE_2 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD" : "+v"(w) : "v"(x), "v"(y));
    if constexpr (E == 3) asm("v_sub_u32_sdwa %0, %1, %2 dst_sel:BYTE_3 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD" : "+v"(w) : "v"(x), "v"(y));
}

// Eq. 2 inverted: the sign-and-magnitude code of a representable integer (8 bits, p significand bits); +0 for 0.
__device__ __forceinline__ unsigned np_code_of(int beta, int p)
{
    const int mag = beta < 0 ? -beta : beta;
    if (mag == 0) return 0u;
    const int msb = 31 - __clz(mag);
    const unsigned code = msb < p ? (unsigned)mag : (((unsigned)(msb - p + 1) << p) | (((unsigned)mag >> (msb - p)) & ((1u << p) - 1u)));
    return code | (beta < 0 ? 0x80u : 0u);
}

// Eq. 2: the integer of a code of the format (8, p)
__device__ __forceinline__ int np_beta_of(unsigned code, int p)
{
    const unsigned m = code & ((1u << p) - 1u);
    const unsigned e = (code >> p) & ((1u << (7 - p)) - 1u);
    const int mag = e ? (int)(((1u << p) + m) << (e - 1)) : (int)m;
    return (code & 0x80u) ? -mag : mag;
}

__device__ __forceinline__ void np_split(int beta, int &h, int &l)
{
    const int mag = beta < 0 ? -beta : beta;
    const int hu = mag >> 6, lu = mag & 63;
    h = beta < 0 ? -hu : hu;
    l = beta < 0 ? -lu : lu;
}

// Four neighbouring channels of one pixel: accumulators -> one packed word of codes, of high digits, of low digits.
// FAST: 7 <= shift <= 36 (32-bit rounding above), else the 64-bit form; RELU and CODES (codes wanted) as template
// parameters keep the sign handling and the encoding out of the variants that do not need them.
template <bool FAST, bool RELU, bool CODES, int E>
__device__ __forceinline__ void np_finish_one(int A, int Cc, int Bm, const NpRound &rnd, const NpFast &fr, int p_y, uint32_t &wc,
                                              uint32_t &whi, uint32_t &wlo)
{
    const int T = (A << 6) + Bm;                         // 64 A + B (the bias sits in the start values of B and C)
    int beta;
    if constexpr (FAST) {
        beta = np_round_fast(T, Cc, fr);
        asm("v_med3_i32 %0, %1, %2, %3" : "=v"(beta) : "v"(beta), "s"(RELU ? 0 : -fr.bmax), "v"(fr.bmax));
    } else {
        beta = np_round_acc((long long)T * 64 + (long long)Cc, rnd);
    }
    if constexpr (RELU) {
        put_shr<E>(whi, 6u, (unsigned)beta);
        put_and<E>(wlo, 63u, (unsigned)beta);
        if constexpr (CODES) wc |= np_code_of(beta, p_y) << (8 * E);
    } else {
        // digits of the sign of beta: h = trunc(beta / 64), l = beta - 64 h
        const int t = beta + ((beta >> 31) & 63);
        put_ashr<E>(whi, 6u, t);
        put_sub<E>(wlo, (unsigned)beta, (unsigned)t & ~63u);
        if constexpr (CODES) wc |= np_code_of(beta, p_y) << (8 * E);
    }
}

// The fused join: the layer's result (32-bit rounding, clamp with the layer's own ReLU as the lower bound), aligned with
// the other operand's integer 64 h + l, summed, converted a second time and split into digits.
template <bool RELU_OUT, int E>
__device__ __forceinline__ void np_finish_add_one(int A, int Cc, int Bm, uint32_t oh4, uint32_t ol4, int lo1, int sa, int sb, const NpFast &fr,
                                                  const NpFast &fr2, uint32_t &whi, uint32_t &wlo)
{
    int beta = np_round_fast((A << 6) + Bm, Cc, fr);
    asm("v_med3_i32 %0, %1, %2, %3" : "=v"(beta) : "v"(beta), "s"(lo1), "v"(fr.bmax));
    const int other = 64 * byte_of(oh4, E) + byte_of(ol4, E);
    const int t = (beta << sa) + (other << sb);
    int r = np_round_fast_i32(t, fr2);
    asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(r), "s"(RELU_OUT ? 0 : -fr2.bmax), "v"(fr2.bmax));
    if constexpr (RELU_OUT) {
        put_shr<E>(whi, 6u, (unsigned)r);
        put_and<E>(wlo, 63u, (unsigned)r);
    } else {
        const int u = r + ((r >> 31) & 63);
        put_ashr<E>(whi, 6u, u);
        put_sub<E>(wlo, (unsigned)r, (unsigned)u & ~63u);
    }
}

// ---- codes -> digit planes ----------------------------------------------------------------------------------------

__global__ void __launch_bounds__(256) np_digits_kernel(const uint8_t *__restrict__ codes, size_t n, int p, int8_t *__restrict__ hi,
                                                        int8_t *__restrict__ lo)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        int h, l;
        np_split(np_beta_of(codes[i], p), h, l);
        hi[i] = (int8_t)h;
        lo[i] = (int8_t)l;
    }
}

// Maximum of m over the wavefront's lanes, then one atomic max per wavefront into *dst (the word starts at zero).
__device__ __forceinline__ void wave_max_to(unsigned long long *dst, unsigned long long m)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        const unsigned long long other = __shfl_xor(m, o, 64);
        m = other > m ? other : m;
    }
    if ((threadIdx.x & 63) == 0 && m) atomicMax(dst, m);
}

__global__ void clear_u64_kernel(unsigned long long *p) { *p = 0ull; }

// ---- element-wise add (Eq. 10) on digit planes ----------------------------------------------------------------------

// v * 2^-shift for a 32-bit v, rounded to the nearest integer representable with p + 1 significant bits, ties to the even
// significand, magnitude clamped to bmax (< 2^12); -16 <= shift <= 31.  Binade of the value from the leading bit, step 2^k,
// r = shift + k bits go with round-half-even (none when r <= 0: the scaled value is exact).  Returns the magnitude.
__device__ __forceinline__ unsigned np_round_i32(int v, int shift, int p, unsigned bmax, int &sgn)
{
    sgn = v >> 31;
    const unsigned mag = (unsigned)((v ^ sgn) - sgn);
    if (mag == 0) return 0u;
    const int L = 31 - __clz((int)mag);
    const int e = L - shift;                       // floor(log2 of the scaled value)
    if (e > 11) return bmax;                       // at least 2^12: beyond every format of this path
    const int k = max(e - p, 0);
    const int r = shift + k;
    unsigned q;
    if (r > 0) {
        const unsigned odd = (mag >> r) & 1u;      // r <= 31: e >= p + 1 gives r = L - p, else r = shift
        q = (mag + ((1u << (r - 1)) - 1u) + odd) >> r;   // mag < 2^31 and the addend <= 2^30: no carry out of 32 bits
    } else {
        q = mag << (-r);                           // below 2^(p+1): fits
    }
    return min(q << k, bmax);
}

struct NpEltParams {
    const int8_t *ah, *al, *bh, *bl;
    uint8_t *y;
    int8_t *yh, *yl;
    size_t n16;                  // groups of 16 elements
    size_t n;                    // elements
    int sa, sb;                  // left shifts of the two operands to the finer scale
    int shift;                   // finer scale's fractional length minus that of the result
    int p_y;
    int beta_max;
    int relu;
};

__device__ __forceinline__ void np_elt_one(int a_h, int a_l, int b_h, int b_l, const NpEltParams &q, unsigned &code, int &h, int &l)
{
    int t = ((64 * a_h + a_l) << q.sa) + ((64 * b_h + b_l) << q.sb);
    if (q.relu) t = max(t, 0);
    int sgn;
    const unsigned mag = np_round_i32(t, q.shift, q.p_y, (unsigned)q.beta_max, sgn);
    const int hu = (int)(mag >> 6), lu = (int)(mag & 63u);
    h = (hu ^ sgn) - sgn;
    l = (lu ^ sgn) - sgn;
    code = np_code_of((int)mag, q.p_y) | (mag ? ((unsigned)sgn & 0x80u) : 0u);
}

__global__ void __launch_bounds__(256) eltwise_np_kernel(NpEltParams q)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < q.n16; i += (size_t)gridDim.x * 256) {
        const uint4 ah = ((const uint4 *)q.ah)[i], al = ((const uint4 *)q.al)[i], bh = ((const uint4 *)q.bh)[i], bl = ((const uint4 *)q.bl)[i];
        const uint32_t wah[4] = {ah.x, ah.y, ah.z, ah.w}, wal[4] = {al.x, al.y, al.z, al.w};
        const uint32_t wbh[4] = {bh.x, bh.y, bh.z, bh.w}, wbl[4] = {bl.x, bl.y, bl.z, bl.w};
        uint32_t oc[4], oh[4], ol[4];
#pragma unroll
        for (int j = 0; j < 4; j++) {
            uint32_t c4 = 0, h4 = 0, l4 = 0;
#pragma unroll
            for (int e = 0; e < 4; e++) {
                unsigned code;
                int h, l;
                np_elt_one(byte_of(wah[j], e), byte_of(wal[j], e), byte_of(wbh[j], e), byte_of(wbl[j], e), q, code, h, l);
                c4 |= code << (8 * e);
                h4 |= ((uint32_t)h & 0xffu) << (8 * e);
                l4 |= ((uint32_t)l & 0xffu) << (8 * e);
            }
            oc[j] = c4; oh[j] = h4; ol[j] = l4;
        }
        if (q.y) ((uint4 *)q.y)[i] = make_uint4(oc[0], oc[1], oc[2], oc[3]);
        if (q.yh) ((uint4 *)q.yh)[i] = make_uint4(oh[0], oh[1], oh[2], oh[3]);
        if (q.yl) ((uint4 *)q.yl)[i] = make_uint4(ol[0], ol[1], ol[2], ol[3]);
    }
    // ragged tail, element by element
    for (size_t i = q.n16 * 16 + (size_t)blockIdx.x * 256 + threadIdx.x; i < q.n; i += (size_t)gridDim.x * 256) {
        unsigned code;
        int h, l;
        np_elt_one(q.ah[i], q.al[i], q.bh[i], q.bl[i], q, code, h, l);
        if (q.y) q.y[i] = (uint8_t)code;
        if (q.yh) q.yh[i] = (int8_t)h;
        if (q.yl) q.yl[i] = (int8_t)l;
    }
}

// Calibration: the largest magnitude of the exact aligned sum (after ReLU if asked), nothing stored.
__global__ void __launch_bounds__(256) eltwise_np_absmax_kernel(const int8_t *ah, const int8_t *al, const int8_t *bh, const int8_t *bl, size_t n,
                                                                 int sa, int sb, int relu, unsigned long long *amax)
{
    unsigned mx = 0;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        const int t = ((64 * (int)ah[i] + (int)al[i]) << sa) + ((64 * (int)bh[i] + (int)bl[i]) << sb);
        const unsigned m = t < 0 ? (relu ? 0u : (unsigned)(-t)) : (unsigned)t;
        mx = max(mx, m);
    }
    wave_max_to(amax, (unsigned long long)mx);
}

// ---- pooling on digit planes ----------------------------------------------------------------------------------------

// The exact mean tot / D (D > 0) to the nearest integer with p + 1 significant bits, ties to the even significand,
// magnitude clamped to bmax; |tot| < 2^19.  Binade e of the mean from D * 2^e <= |tot| < D * 2^(e+1), step 2^k with
// k = max(e - p, 0), quotient and remainder of |tot| by D * 2^k decide the rounding exactly.
__device__ __forceinline__ int np_round_mean(int tot, int D, int p, int bmax)
{
    const int sgn = tot >> 31;
    const unsigned mag = (unsigned)((tot ^ sgn) - sgn);
    int e = 0;
    while (e < 12 && ((unsigned)D << (e + 1)) <= mag) e++;
    const int k = max(e - p, 0);
    const unsigned den = (unsigned)D << k;
    unsigned q = mag / den;
    const unsigned rem2 = 2u * (mag - q * den);
    if (rem2 > den || (rem2 == den && (q & 1u))) q++;
    const int r = min((int)(q << k), bmax);
    return (r ^ sgn) - sgn;
}

struct NpPoolParams {
    const int8_t *xh, *xl;
    uint8_t *y;
    int8_t *yh, *yl;
    int N, H, W, C, k, stride, pad, P, Q, p_fmt, beta_max, avg;
};

// One lane per output element, channels fastest (neighbouring lanes read neighbouring bytes).
__global__ void __launch_bounds__(256) pool_np_kernel(NpPoolParams a)
{
    const size_t total = (size_t)a.N * a.P * a.Q * a.C;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const int c = (int)(i % a.C);
        const size_t pix = i / a.C;
        const int q = (int)(pix % a.Q);
        const size_t t = pix / a.Q;
        const int p = (int)(t % a.P);
        const int n = (int)(t / a.P);
        int best = -4096, tot = 0;
        for (int r = 0; r < a.k; r++) {
            const int ih = p * a.stride - a.pad + r;
            if (ih < 0 || ih >= a.H) continue;
            for (int s = 0; s < a.k; s++) {
                const int iw = q * a.stride - a.pad + s;
                if (iw < 0 || iw >= a.W) continue;
                const size_t o = (((size_t)n * a.H + ih) * a.W + iw) * a.C + c;
                const int beta = 64 * (int)a.xh[o] + (int)a.xl[o];
                best = max(best, beta);
                tot += beta;
            }
        }
        const int beta = a.avg ? np_round_mean(tot, a.k * a.k, a.p_fmt, a.beta_max) : best;
        if (a.y) a.y[i] = (uint8_t)np_code_of(beta, a.p_fmt);
        int h, l;
        np_split(beta, h, l);
        if (a.yh) a.yh[i] = (int8_t)h;
        if (a.yl) a.yl[i] = (int8_t)l;
    }
}

// Average over the whole unpadded image (k = H = W) with C a multiple of 4: one lane per four channels of an image, word
// loads, the pixels in turn (neighbouring lanes read neighbouring words).
__global__ void __launch_bounds__(256) avgpool_global_np4_kernel(NpPoolParams a)
{
    const int C4 = a.C / 4;
    const int total = a.N * C4;
    const int pixels = a.H * a.W;
    for (int i = blockIdx.x * 256 + threadIdx.x; i < total; i += gridDim.x * 256) {
        const int n = i / C4, c4 = i - n * C4;
        const uint32_t *ph = (const uint32_t *)a.xh + (size_t)n * pixels * C4 + c4;
        const uint32_t *pl = (const uint32_t *)a.xl + (size_t)n * pixels * C4 + c4;
        int tot[4] = {0, 0, 0, 0};
        for (int j = 0; j < pixels; j++) {
            const uint32_t h4 = ph[(size_t)j * C4], l4 = pl[(size_t)j * C4];
#pragma unroll
            for (int e = 0; e < 4; e++) tot[e] += 64 * byte_of(h4, e) + byte_of(l4, e);
        }
        uint32_t oc = 0, oh = 0, ol = 0;
#pragma unroll
        for (int e = 0; e < 4; e++) {
            const int beta = np_round_mean(tot[e], pixels, a.p_fmt, a.beta_max);
            int h, l;
            np_split(beta, h, l);
            oc |= (uint32_t)np_code_of(beta, a.p_fmt) << (8 * e);
            oh |= (uint32_t)(uint8_t)h << (8 * e);
            ol |= (uint32_t)(uint8_t)l << (8 * e);
        }
        if (a.y) ((uint32_t *)a.y)[i] = oc;
        if (a.yh) ((uint32_t *)a.yh)[i] = oh;
        if (a.yl) ((uint32_t *)a.yl)[i] = ol;
    }
}

// 3 x 3 / stride 2 / pad 1 max pooling with C a multiple of 4: one lane per four channels of an output pixel.
__global__ void __launch_bounds__(256) maxpool3_np_kernel(NpPoolParams a)
{
    const int C4 = a.C / 4;
    const size_t total = (size_t)a.N * a.P * a.Q * C4;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const int c4 = (int)(i % C4);
        const size_t pix = i / C4;
        const int q = (int)(pix % a.Q);
        const size_t t = pix / a.Q;
        const int p = (int)(t % a.P);
        const int n = (int)(t / a.P);
        int best[4] = {-4096, -4096, -4096, -4096};
#pragma unroll
        for (int r = 0; r < 3; r++) {
            const int ih = 2 * p - 1 + r;
            if (ih < 0 || ih >= a.H) continue;
#pragma unroll
            for (int s = 0; s < 3; s++) {
                const int iw = 2 * q - 1 + s;
                if (iw < 0 || iw >= a.W) continue;
                const size_t o = ((((size_t)n * a.H + ih) * a.W + iw) * a.C) / 4 + c4;
                const uint32_t h4 = ((const uint32_t *)a.xh)[o], l4 = ((const uint32_t *)a.xl)[o];
#pragma unroll
                for (int e = 0; e < 4; e++) best[e] = max(best[e], 64 * byte_of(h4, e) + byte_of(l4, e));
            }
        }
        uint32_t oc = 0, oh = 0, ol = 0;
#pragma unroll
        for (int e = 0; e < 4; e++) {
            int h, l;
            np_split(best[e], h, l);
            oc |= (uint32_t)np_code_of(best[e], a.p_fmt) << (8 * e);
            oh |= ((uint32_t)h & 0xffu) << (8 * e);
            ol |= ((uint32_t)l & 0xffu) << (8 * e);
        }
        if (a.y) ((uint32_t *)a.y)[i] = oc;
        if (a.yh) ((uint32_t *)a.yh)[i] = oh;
        if (a.yl) ((uint32_t *)a.yl)[i] = ol;
    }
}

// The same for C a multiple of 16 when only the digit planes are wanted: one lane per 16 channels of an output pixel,
// 16-byte loads.  beta = 64 h + l with both digits of beta's sign orders like the pair (h, l), so the maximum is taken
// on 16-bit keys (h in the high byte, l with its sign bit flipped in the low byte: signed order of the key = order of
// beta), two keys per packed instruction - no value is decoded.  Window positions outside the image are replaced by
// the nearest one inside, which lies in the same window.
struct NpMaxPool3Params {
    NpPoolParams a;
    int total;              // N * P * Q * C / 16
    FastDiv div_cv, div_q, div_p;
};

__global__ void __launch_bounds__(256) maxpool3_np16_kernel(NpMaxPool3Params prm)
{
    typedef short v2s __attribute__((ext_vector_type(2)));
    const NpPoolParams &a = prm.a;
    const int cv = a.C / 16;
    for (int i = blockIdx.x * 256 + threadIdx.x; i < prm.total; i += gridDim.x * 256) {
        const int px = fastdiv(i, prm.div_cv);
        const int c = (i - px * cv) * 16;
        const int t = fastdiv(px, prm.div_q);
        const int q = px - t * a.Q;
        const int n = fastdiv(t, prm.div_p);
        const int p = t - n * a.P;
        v2s best[8];
#pragma unroll
        for (int e = 0; e < 8; e++) best[e] = v2s{(short)-32768, (short)-32768};
#pragma unroll
        for (int r = 0; r < 3; r++) {
            const int ih = min(max(2 * p - 1 + r, 0), a.H - 1);
#pragma unroll
            for (int s2 = 0; s2 < 3; s2++) {
                const int iw = min(max(2 * q - 1 + s2, 0), a.W - 1);
                const size_t o = (((size_t)n * a.H + ih) * a.W + iw) * a.C + c;
                const uint4 h4 = *(const uint4 *)(a.xh + o), l4 = *(const uint4 *)(a.xl + o);
                const uint32_t hw[4] = {h4.x, h4.y, h4.z, h4.w}, lw[4] = {l4.x, l4.y, l4.z, l4.w};
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    const uint32_t lx = lw[e] ^ 0x80808080u;
                    const uint32_t k01 = __builtin_amdgcn_perm(hw[e], lx, 0x05010400u);     // {l0, h0, l1, h1}
                    const uint32_t k23 = __builtin_amdgcn_perm(hw[e], lx, 0x07030602u);     // {l2, h2, l3, h3}
                    best[2 * e] = __builtin_elementwise_max(best[2 * e], __builtin_bit_cast(v2s, k01));
                    best[2 * e + 1] = __builtin_elementwise_max(best[2 * e + 1], __builtin_bit_cast(v2s, k23));
                }
            }
        }
        uint32_t oh[4], ol[4];
#pragma unroll
        for (int e = 0; e < 4; e++) {
            const uint32_t k01 = __builtin_bit_cast(uint32_t, best[2 * e]), k23 = __builtin_bit_cast(uint32_t, best[2 * e + 1]);
            oh[e] = __builtin_amdgcn_perm(k23, k01, 0x07050301u);                           // {h0, h1, h2, h3}
            ol[e] = __builtin_amdgcn_perm(k23, k01, 0x06040200u) ^ 0x80808080u;             // {l0, l1, l2, l3}
        }
        const size_t oo = (size_t)px * a.C + c;
        if (a.yh) *(uint4 *)(a.yh + oo) = make_uint4(oh[0], oh[1], oh[2], oh[3]);
        if (a.yl) *(uint4 *)(a.yl + oo) = make_uint4(ol[0], ol[1], ol[2], ol[3]);
    }
}

// ---- space-to-depth packing of a stride-2 first layer with few channels -------------------------------------------------
// A stride-2 convolution with an R x S kernel (R, S <= 8) over C <= 4 channels is a stride-1 convolution with a
// ceil(R/2) x ceil(S/2) kernel over the 2 x 2 space-to-depth image with 4 C channels.  With 16 bytes per such pixel
// (4 C <= 16, the rest zero) four neighbouring pixels are 64 contiguous bytes, i.e. one 64-byte reduction step of the
// matrix-core kernels holds a whole kernel row.  y[n][i][q][16 s' + (2 dy + dx) C + c] = x_padded[n][2 i + dy][2 (q + s') + dx][c],
// s' = 0..3, so that the layer becomes a 4 x 1 convolution over 64 channels with unit stride and no padding.
__global__ void __launch_bounds__(256) stem_pack_x_kernel(const int8_t *x, int8_t *y, int N, int H, int W, int C, int pad, int Hs, int Qs)
{
    const size_t total = (size_t)N * Hs * Qs * 4;                   // one lane per 16-byte piece: (pixel, s')
    const uint8_t *xu = (const uint8_t *)x;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const int sp = (int)(i & 3);
        const size_t pix = i >> 2;
        const int q = (int)(pix % Qs);
        const size_t t = pix / Qs;
        const int ii = (int)(t % Hs);
        const int n = (int)(t / Hs);
        // the piece holds, for dy = 0, 1, the 2 C bytes of the two neighbouring pixels 2 (q + s') - pad + {0, 1} of row 2 ii + dy - pad
        unsigned long long lo = 0, hi = 0;                          // bytes 0..7 and 8..15 of the piece
        const int iw0 = 2 * (q + sp) - pad;
#pragma unroll
        for (int dy = 0; dy < 2; dy++) {
            const int ih = 2 * ii + dy - pad;
            if (ih < 0 || ih >= H) continue;
            const uint8_t *row = xu + ((size_t)n * H + ih) * W * C;
            for (int b = 0; b < 2 * C; b++) {
                const int iw = iw0 + (b >= C ? 1 : 0);
                if (iw < 0 || iw >= W) continue;
                const unsigned long long v = row[(size_t)(iw * C + (b >= C ? b - C : b))];
                const int pos = dy * 2 * C + b;                     // byte position in the piece
                if (pos < 8) lo |= v << (8 * pos);
                else hi |= v << (8 * (pos - 8));
            }
        }
        ((uint4 *)y)[i] = make_uint4((unsigned)lo, (unsigned)(lo >> 32), (unsigned)hi, (unsigned)(hi >> 32));
    }
}

// The same packing with word loads, for inputs below 2^31 bytes: the 2 C bytes a piece takes from one image row - the
// pixels 2 (q + s') - pad and the next one - are contiguous there, so each row's share is cut out of three aligned words
// (range-checked buffer loads: words past the end read as zero) and masked by which of the two pixels exist.
__global__ void __launch_bounds__(256) stem_pack_x_words_kernel(const int8_t *x, int8_t *y, int N, int H, int W, int C, int pad, int Hs, int Qs)
{
    const size_t total = (size_t)N * Hs * Qs * 4;                   // one lane per 16-byte piece: (pixel, s')
    // (the range rounded up to whole words: x is word-aligned, so the word that holds the last byte lies in the same page)
    const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(x), 0, (N * H * W * C + 3) & ~3, 0x00020000);
    const unsigned long long pixel_mask = (1ULL << (8 * C)) - 1ULL;  // C <= 4
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const int sp = (int)(i & 3);
        const size_t pix = i >> 2;
        const int q = (int)(pix % Qs);
        const size_t t = pix / Qs;
        const int ii = (int)(t % Hs);
        const int n = (int)(t / Hs);
        const int iw0 = 2 * (q + sp) - pad;
        const bool first = iw0 >= 0 && iw0 < W, second = iw0 + 1 >= 0 && iw0 + 1 < W;
        unsigned long long part[2];                                 // the 2 C bytes of rows dy = 0, 1
#pragma unroll
        for (int dy = 0; dy < 2; dy++) {
            const int ih = 2 * ii + dy - pad;
            part[dy] = 0;
            if (ih < 0 || ih >= H || !(first || second)) continue;
            // eight bytes from the first existing pixel on
            const int o = ((n * H + ih) * W + (first ? iw0 : iw0 + 1)) * C;
            const int a = o & ~3, sh = o & 3;
            const uint32_t d0 = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(xr, a, 0, 0);
            const uint32_t d1 = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(xr, a + 4, 0, 0);
            const uint32_t d2 = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(xr, a + 8, 0, 0);
            const unsigned long long v = (unsigned long long)__builtin_amdgcn_alignbyte(d1, d0, sh) |
                                         ((unsigned long long)__builtin_amdgcn_alignbyte(d2, d1, sh) << 32);
            if (first) part[dy] = (v & pixel_mask) | (second ? v & (pixel_mask << (8 * C)) : 0ULL);
            else part[dy] = (v & pixel_mask) << (8 * C);            // only the second pixel exists: it is the one loaded
        }
        // bytes 0 .. 2C-1 from row 0, 2C .. 4C-1 from row 1, zeros behind
        unsigned long long lo = part[0], hi = 0;
        if (C == 4) hi = part[1];
        else {
            lo |= part[1] << (16 * C);
            hi = part[1] >> (64 - 16 * C);
        }
        ((uint4 *)y)[i] = make_uint4((unsigned)lo, (unsigned)(lo >> 32), (unsigned)hi, (unsigned)(hi >> 32));
    }
}

// y[k][r'][16 s' + (2 dy + dx) C + c] = w[k][2 r' + dy][2 s' + dx][c] where that tap exists, else 0; r' = 0..3.
__global__ void __launch_bounds__(256) stem_pack_w_kernel(const int8_t *w, int8_t *y, int K, int R, int S, int C)
{
    const int total = K * 4 * 64;
    for (int i = blockIdx.x * 256 + threadIdx.x; i < total; i += gridDim.x * 256) {
        const int byte = i & 63, rp = (i >> 6) & 3, k = i >> 8;
        const int sp = byte >> 4, rest = byte & 15;
        int8_t v = 0;
        if (rest < 4 * C) {
            const int par = rest / C, c = rest - par * C;
            const int r = 2 * rp + (par >> 1), s = 2 * sp + (par & 1);
            if (r < R && s < S) v = w[((k * R + r) * S + s) * C + c];
        }
        y[i] = v;
    }
}

// ---- direct form --------------------------------------------------------------------------------------------------

__global__ void __launch_bounds__(256) conv_np_direct_kernel(NpConvArgs a)
{
    const int Cg = a.C / a.groups;
    const int Kg = a.K / a.groups;
    const size_t total = (size_t)a.N * a.P * a.Q * a.K;
    NpRound rnd = {a.shift, a.p_y, (float)a.beta_max, a.relu};
    unsigned long long mx = 0;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const int k = (int)(i % a.K);
        const size_t pix = i / a.K;
        const int q = (int)(pix % a.Q);
        const size_t t = pix / a.Q;
        const int p = (int)(t % a.P);
        const int n = (int)(t / a.P);
        const int g = k / Kg;
        long long acc = a.b ? (long long)a.b[k] : 0;
        for (int r = 0; r < a.R; r++) {
            const int ih = p * a.stride - a.pad + r;
            if (ih < 0 || ih >= a.H) continue;
            for (int s = 0; s < a.S; s++) {
                const int iw = q * a.stride - a.pad + s;
                if (iw < 0 || iw >= a.W) continue;
                const size_t xo = (((size_t)n * a.H + ih) * a.W + iw) * a.C + (size_t)g * Cg;
                const size_t wo = (((size_t)k * a.R + r) * a.S + s) * Cg;
                for (int c = 0; c < Cg; c++)
                    acc += (long long)((64 * (int)a.xh[xo + c] + (int)a.xl[xo + c]) * (64 * (int)a.wh[wo + c] + (int)a.wl[wo + c]));
            }
        }
        if (a.amax) {
            const unsigned long long m = acc < 0 ? (a.relu ? 0ull : (unsigned long long)(-acc)) : (unsigned long long)acc;
            mx = m > mx ? m : mx;
        }
        const int beta = np_round_acc(acc, rnd);
        if (a.y) a.y[i] = (uint8_t)np_code_of(beta, a.p_y);
        int h, l;
        np_split(beta, h, l);
        if (a.yh) a.yh[i] = (int8_t)h;
        if (a.yl) a.yl[i] = (int8_t)l;
    }
    if (a.amax) wave_max_to(a.amax, mx);
}

// ---- matrix-core form ---------------------------------------------------------------------------------------------

struct NpConvParams {
    NpConvArgs a;
    int M;                  // N * P * Q output pixels
    int nitems;             // 64-byte steps of the reduction: R * S * C / 64
    int csteps;             // C / 64
    int tiles_c;            // channel tiles
    unsigned x_bytes, w_bytes;
    FastDiv div_q, div_p, div_tc;
};

template <int BP, int BC, int OCC, int NSTAGES, bool ADD>
__global__ void __launch_bounds__(256, OCC) conv_np_mfma_kernel(NpConvParams prm)
{
    static_assert(NSTAGES == 2 || NSTAGES == 3, "ring depth");
    constexpr int ROWS = 2 * BP + 2 * BC;                 // LDS rows of 64 bytes per stage: x_h, x_l, w_h, w_l
    constexpr int XH = 0, XL = BP, WH = 2 * BP, WL = 2 * BP + BC;
    constexpr int XJ = BP / 64, WJ = BC / 64;             // 16-row chunks per wavefront, operand plane and step
    constexpr int LPW = 2 * XJ + 2 * WJ;                  // loads per wavefront and step
    static_assert(BP % 64 == 0 && BC % 64 == 0, "whole chunks for four wavefronts");
    constexpr int WP = BP / 2, WC = BC / 2;               // wavefront tile (2 x 2 wavefronts)
    constexpr int PT = WP / 32, CT = WC / 32;
    static_assert(PT * CT == 4 || (PT * CT == 2 && OCC >= 2), "twelve accumulator tiles per wavefront, or six with two workgroups per compute unit");

    extern __shared__ uint4 lds[];
    const NpConvArgs &a = prm.a;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // tile of this workgroup: ids are dealt round-robin to the 8 XCDs; renumbered so that each XCD owns a contiguous
    // range, the channel tiles of one pixel tile (same input rows) then meet in one L2
    const int G = gridDim.x;
    int lb = blockIdx.x;
    {
        const int per = G / 8, rem = G % 8, xcd = lb % 8, idx = lb / 8;
        lb = (xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per) + idx;
    }
    const int pt = fastdiv(lb, prm.div_tc);
    const int ct = lb - pt * prm.tiles_c;

    const v4i xh_rsrc = make_rsrc(a.xh, prm.x_bytes), xl_rsrc = make_rsrc(a.xl, prm.x_bytes);
    const v4i wh_rsrc = make_rsrc(a.wh, prm.w_bytes), wl_rsrc = make_rsrc(a.wl, prm.w_bytes);
    const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) char *)(char *)&lds[0];

    // ---- producer: lane l of a wavefront-wide load supplies row l/4 of a 16-row chunk, physical piece l%4, which holds
    // logical piece (l%4) ^ ((row>>2)&3)
    const int lrow = lane >> 2;
    const int lp = (lane & 3) ^ ((lane >> 4) & 3);
    int ih0[XJ], iw0[XJ], xbase[XJ];
#pragma unroll
    for (int j = 0; j < XJ; j++) {
        const int m = pt * BP + 16 * (wave + 4 * j) + lrow;
        if (m < prm.M) {
            const int t = fastdiv(m, prm.div_q);
            const int oq = m - t * a.Q;
            const int n = fastdiv(t, prm.div_p);
            const int op = t - n * a.P;
            ih0[j] = op * a.stride - a.pad;
            iw0[j] = oq * a.stride - a.pad;
            xbase[j] = ((n * a.H + ih0[j]) * a.W + iw0[j]) * a.C + lp * 16;
        } else {
            ih0[j] = -(1 << 28);      // no kernel row is inside the image
            iw0[j] = 0;
            xbase[j] = 0;
        }
    }
    unsigned woff[WJ];
#pragma unroll
    for (int j = 0; j < WJ; j++) {
        // LDS row i = 8g + 4h + e of a 32-row group receives channel 16h + 4g + e: the matrix instruction then leaves 16
        // consecutive channels in each lane
        const int rr = 16 * (wave + 4 * j) + lrow;
        const int i32 = rr & 31;
        const int k = ct * BC + (rr & ~31) + 16 * ((i32 >> 2) & 1) + 4 * (i32 >> 3) + (i32 & 3);
        woff[j] = k < a.K ? (unsigned)(k * (a.R * a.S * a.C) + lp * 16) : kOutOfRange;
    }
    int p_r = 0, p_s = 0, p_c = 0, p_it = 0;     // kernel row, kernel column, channel step and index of the step fetched next
    auto issue = [&](int stage) __attribute__((always_inline)) {
        const int tap_off = (p_r * a.W + p_s) * a.C + p_c * kStepBytes;
        const unsigned sbase = lds_base + (unsigned)(stage * ROWS) * 64u + (unsigned)wave * 1024u;
#pragma unroll
        for (int j = 0; j < XJ; j++) {
            const bool ok = (unsigned)(ih0[j] + p_r) < (unsigned)a.H && (unsigned)(iw0[j] + p_s) < (unsigned)a.W;
            const unsigned off = ok ? (unsigned)(xbase[j] + tap_off) : kOutOfRange;
            load_piece_to_lds(off, xh_rsrc, (unsigned)__builtin_amdgcn_readfirstlane((int)(sbase + (unsigned)(XH * 64 + j * 4096))));
            load_piece_to_lds(off, xl_rsrc, (unsigned)__builtin_amdgcn_readfirstlane((int)(sbase + (unsigned)(XL * 64 + j * 4096))));
        }
        const unsigned step_off = (unsigned)p_it * kStepBytes;
#pragma unroll
        for (int j = 0; j < WJ; j++) {
            load_piece_to_lds(woff[j] + step_off, wh_rsrc, (unsigned)__builtin_amdgcn_readfirstlane((int)(sbase + (unsigned)(WH * 64 + j * 4096))));
            load_piece_to_lds(woff[j] + step_off, wl_rsrc, (unsigned)__builtin_amdgcn_readfirstlane((int)(sbase + (unsigned)(WL * 64 + j * 4096))));
        }
        ++p_it;
        if (++p_c == prm.csteps) {
            p_c = 0;
            if (++p_s == a.S) {
                p_s = 0;
                ++p_r;
            }
        }
    };

    // ---- consumer
    const int wp0 = (wave & 1) * WP, wc0 = (wave >> 1) * WC;
    const int l32 = lane & 31, lh = lane >> 5;
    const int swz = (l32 >> 2) & 3;
    v16i accA[CT][PT], accC[CT][PT], accB[CT][PT];
    // the bias b = 64 * (b >> 6) + (b & 63) starts the accumulators of the middle and the low products
#pragma unroll
    for (int c = 0; c < CT; c++) {
        const int kc = ct * BC + wc0 + c * 32 + 16 * lh;
        int bias[16];
#pragma unroll
        for (int r4 = 0; r4 < 4; r4++) {
            const int4 bv = (a.b && kc < a.K) ? *(const int4 *)(a.b + kc + 4 * r4) : make_int4(0, 0, 0, 0);
            bias[4 * r4 + 0] = bv.x;
            bias[4 * r4 + 1] = bv.y;
            bias[4 * r4 + 2] = bv.z;
            bias[4 * r4 + 3] = bv.w;
        }
#pragma unroll
        for (int p = 0; p < PT; p++)
#pragma unroll
            for (int r = 0; r < 16; r++) {
                accA[c][p][r] = 0;
                accB[c][p][r] = bias[r] >> 6;
                accC[c][p][r] = bias[r] & 63;
            }
    }

    // Operands of one 32-byte half of a step.  Step i multiplies operands that are already in registers and meanwhile
    // reads those of step i+1: after the first half's matrix instructions the wavefront waits for its own loads of step
    // i+1 and meets the others at the barrier (every wavefront has then also finished reading step i, whose stage the
    // refill overwrites with step i+3), reads the first half of step i+1 into the registers just consumed, issues the
    // second half, refills, and reads the second half.
    struct Half {
        v4i wh[CT], wl[CT];
        v4i xh[PT], xl[PT];
    };
    Half f0, f1;
    auto read_half = [&](Half &f, int kk, int stage) __attribute__((always_inline)) {
        const v4i *st = (const v4i *)lds + stage * ROWS * kPieces;
        const int g = (kk * 2 + lh) ^ swz;
#pragma unroll
        for (int c = 0; c < CT; c++) {
            const int row = wc0 + c * 32 + l32;
            f.wh[c] = st[(WH + row) * kPieces + g];
            f.wl[c] = st[(WL + row) * kPieces + g];
        }
#pragma unroll
        for (int p = 0; p < PT; p++) {
            const int row = wp0 + p * 32 + l32;
            f.xh[p] = st[(XH + row) * kPieces + g];
            f.xl[p] = st[(XL + row) * kPieces + g];
        }
    };
    auto mfma_half = [&](const Half &f) __attribute__((always_inline)) {
#pragma unroll
        for (int p = 0; p < PT; p++)
#pragma unroll
            for (int c = 0; c < CT; c++) {
                accA[c][p] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f.wh[c], f.xh[p], accA[c][p], 0, 0, 0);
                accC[c][p] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f.wl[c], f.xl[p], accC[c][p], 0, 0, 0);
                accB[c][p] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f.wh[c], f.xl[p], accB[c][p], 0, 0, 0);
                accB[c][p] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f.wl[c], f.xh[p], accB[c][p], 0, 0, 0);
            }
    };
    auto ring_barrier = [&]() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };

    const int nitems = prm.nitems;
#pragma unroll
    for (int i = 0; i < NSTAGES; i++)
        if (i < nitems) issue(i);
    if (nitems > 0) {
        // step 0 has landed when at most the loads of steps 1 and 2 are outstanding
        if (NSTAGES > 2 && nitems > 2) wait_loads<(NSTAGES - 1) * LPW>();
        else if (nitems > 1) wait_loads<LPW>();
        else wait_loads<0>();
        ring_barrier();
        read_half(f0, 0, 0);
        read_half(f1, 1, 0);
    }
    int stage = 0;
    for (int it = 0; it < nitems; it++) {
        const int next = stage + 1 == NSTAGES ? 0 : stage + 1;
        const bool has_next = it + 1 < nitems;
        mfma_half(f0);
        __builtin_amdgcn_sched_barrier(0);
        if (has_next) {
            // loads younger than those of step it+1: those of step it+2 (step it+3 is issued below)
            if (NSTAGES > 2 && it + 2 < nitems) wait_loads<(NSTAGES - 2) * LPW>();
            else wait_loads<0>();
            ring_barrier();
            read_half(f0, 0, next);
        }
        __builtin_amdgcn_sched_barrier(0);
        mfma_half(f1);
        __builtin_amdgcn_sched_barrier(0);
        if (has_next) {
            if (it + NSTAGES < nitems) issue(stage);
            read_half(f1, 1, next);
        }
        __builtin_amdgcn_sched_barrier(0);
        stage = next;
    }

    // ---- epilogue: register r of a lane belongs to channel kc + r of pixel m
    const NpRound rnd = {a.shift, a.p_y, (float)a.beta_max, a.relu};
    const NpFast fr = {(unsigned)(1023 + a.p_y + a.shift), (unsigned)(1023 + a.shift + 11), ((unsigned)(52 - a.p_y) << 20) | 0x80000u, a.beta_max};
    auto finish = [&](auto fast, auto relu, auto codes) __attribute__((always_inline)) {
        constexpr bool FAST = decltype(fast)::value, RELU = decltype(relu)::value, CODES = decltype(codes)::value;
#pragma unroll
        for (int c = 0; c < CT; c++) {
            const int kc = ct * BC + wc0 + c * 32 + 16 * lh;
            if (kc >= a.K) continue;
#pragma unroll
            for (int p = 0; p < PT; p++) {
                const int m = pt * BP + wp0 + p * 32 + l32;
                uint32_t oc[4], oh[4], ol[4];
#pragma unroll
                for (int r4 = 0; r4 < 4; r4++) {
                    uint32_t wc = 0, whi = 0, wlo = 0;
                    const int r = 4 * r4;
                    np_finish_one<FAST, RELU, CODES, 0>(accA[c][p][r + 0], accC[c][p][r + 0], accB[c][p][r + 0], rnd, fr, a.p_y, wc, whi, wlo);
                    np_finish_one<FAST, RELU, CODES, 1>(accA[c][p][r + 1], accC[c][p][r + 1], accB[c][p][r + 1], rnd, fr, a.p_y, wc, whi, wlo);
                    np_finish_one<FAST, RELU, CODES, 2>(accA[c][p][r + 2], accC[c][p][r + 2], accB[c][p][r + 2], rnd, fr, a.p_y, wc, whi, wlo);
                    np_finish_one<FAST, RELU, CODES, 3>(accA[c][p][r + 3], accC[c][p][r + 3], accB[c][p][r + 3], rnd, fr, a.p_y, wc, whi, wlo);
                    oc[r4] = wc;
                    oh[r4] = whi;
                    ol[r4] = wlo;
                }
                if (m < prm.M) {
                    const size_t o = (size_t)m * a.K + kc;
                    if (CODES) *(uint4 *)(a.y + o) = make_uint4(oc[0], oc[1], oc[2], oc[3]);
                    if (a.yh) *(uint4 *)(a.yh + o) = make_uint4(oh[0], oh[1], oh[2], oh[3]);
                    if (a.yl) *(uint4 *)(a.yl + o) = make_uint4(ol[0], ol[1], ol[2], ol[3]);
                }
            }
        }
    };
    using T_ = std::true_type;
    using F_ = std::false_type;
    if constexpr (ADD) {
        const NpFast fr2 = {(unsigned)(1023 + a.p_y + a.add_shift), (unsigned)(1023 + a.add_shift + 11), ((unsigned)(52 - a.p_y) << 20) | 0x80000u,
                            a.beta_max};
        const int lo1 = a.relu ? 0 : -a.beta_max;
        auto finish_add = [&](auto relu_out) __attribute__((always_inline)) {
            constexpr bool RELU_OUT = decltype(relu_out)::value;
#pragma unroll
            for (int c = 0; c < CT; c++) {
                const int kc = ct * BC + wc0 + c * 32 + 16 * lh;
                if (kc >= a.K) continue;
                // the other operand of all pixel tiles first, so that the loads are in flight together
                uint4 vh[PT], vl[PT];
#pragma unroll
                for (int p = 0; p < PT; p++) {
                    const int m = min(pt * BP + wp0 + p * 32 + l32, prm.M - 1);
                    const size_t o = (size_t)m * a.K + kc;
                    vh[p] = *(const uint4 *)(a.oh + o);
                    vl[p] = *(const uint4 *)(a.ol + o);
                }
#pragma unroll
                for (int p = 0; p < PT; p++) {
                    const int m = pt * BP + wp0 + p * 32 + l32;
                    const uint32_t h4[4] = {vh[p].x, vh[p].y, vh[p].z, vh[p].w}, l4[4] = {vl[p].x, vl[p].y, vl[p].z, vl[p].w};
                    uint32_t oh[4], ol[4];
#pragma unroll
                    for (int r4 = 0; r4 < 4; r4++) {
                        uint32_t whi = 0, wlo = 0;
                        const int r = 4 * r4;
                        np_finish_add_one<RELU_OUT, 0>(accA[c][p][r + 0], accC[c][p][r + 0], accB[c][p][r + 0], h4[r4], l4[r4], lo1, a.add_sa, a.add_sb, fr, fr2, whi, wlo);
                        np_finish_add_one<RELU_OUT, 1>(accA[c][p][r + 1], accC[c][p][r + 1], accB[c][p][r + 1], h4[r4], l4[r4], lo1, a.add_sa, a.add_sb, fr, fr2, whi, wlo);
                        np_finish_add_one<RELU_OUT, 2>(accA[c][p][r + 2], accC[c][p][r + 2], accB[c][p][r + 2], h4[r4], l4[r4], lo1, a.add_sa, a.add_sb, fr, fr2, whi, wlo);
                        np_finish_add_one<RELU_OUT, 3>(accA[c][p][r + 3], accC[c][p][r + 3], accB[c][p][r + 3], h4[r4], l4[r4], lo1, a.add_sa, a.add_sb, fr, fr2, whi, wlo);
                        oh[r4] = whi;
                        ol[r4] = wlo;
                    }
                    if (m < prm.M) {
                        const size_t o = (size_t)m * a.K + kc;
                        *(uint4 *)(a.yh + o) = make_uint4(oh[0], oh[1], oh[2], oh[3]);
                        *(uint4 *)(a.yl + o) = make_uint4(ol[0], ol[1], ol[2], ol[3]);
                    }
                }
            }
        };
        if (a.add_relu) finish_add(T_{});
        else finish_add(F_{});
        return;
    }
    if (a.shift >= 7 && a.shift <= 36) {
        if (a.y) {
            if (a.relu) finish(T_{}, T_{}, T_{});
            else finish(T_{}, F_{}, T_{});
        } else {
            if (a.relu) finish(T_{}, T_{}, F_{});
            else finish(T_{}, F_{}, F_{});
        }
    } else {
        // rare: no downscale to speak of, or one beyond 36 bits; sign handling and encoding always in
        if (a.y) finish(F_{}, F_{}, T_{});
        else finish(F_{}, F_{}, F_{});
    }
}

template <int BP, int BC, int OCC = 1, int NSTAGES = 3, bool ADD = false>
hipError_t launch_np_mfma(const NpConvArgs &a, hipStream_t st)
{
    NpConvParams prm;
    prm.a = a;
    const long long M = (long long)a.N * a.P * a.Q;
    prm.M = (int)M;
    prm.csteps = a.C / kStepBytes;
    prm.nitems = a.R * a.S * prm.csteps;
    prm.tiles_c = (a.K + BC - 1) / BC;
    prm.x_bytes = (unsigned)((long long)a.N * a.H * a.W * a.C);
    prm.w_bytes = (unsigned)((long long)a.K * a.R * a.S * a.C);
    prm.div_q = make_fastdiv(a.Q);
    prm.div_p = make_fastdiv(a.P);
    prm.div_tc = make_fastdiv(prm.tiles_c);
    const long long tiles = ((M + BP - 1) / BP) * prm.tiles_c;
    if (tiles > 0x7fffffffLL) return hipErrorInvalidValue;
    constexpr size_t lds_bytes = (size_t)NSTAGES * (2 * BP + 2 * BC) * 64;
    static_assert(lds_bytes * OCC <= (size_t)kLdsBytes, "three stages fit");
    static const hipError_t attr = hipFuncSetAttribute((const void *)conv_np_mfma_kernel<BP, BC, OCC, NSTAGES, ADD>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (attr != hipSuccess) return attr;
    conv_np_mfma_kernel<BP, BC, OCC, NSTAGES, ADD><<<(unsigned)tiles, 256, lds_bytes, st>>>(prm);
    return hipGetLastError();
}

}  // namespace

// The matrix-core form takes dense layers whose reduction runs in whole 64-byte steps and whose three int32
// accumulators cannot overflow; byte offsets are 32-bit; outputs are written 16 channels at a time.
bool conv_np_mfma_supports(const NpConvArgs &a)
{
    if (a.groups != 1 || a.C % kStepBytes || a.K % 16) return false;
    if ((long long)a.R * a.S * a.C > 13000) return false;        // |64 A + B| <= 65410 per term: stays below 2^30 (the epilogue doubles it)
    if ((long long)a.N * a.H * a.W * a.C >= (1LL << 31) - (1 << 24)) return false;
    if ((long long)a.K * a.R * a.S * a.C >= (1LL << 31) - (1 << 24)) return false;
    if ((long long)a.N * a.P * a.Q >= (1LL << 31) - 512) return false;
    const uintptr_t al = (uintptr_t)a.xh | (uintptr_t)a.xl | (uintptr_t)a.wh | (uintptr_t)a.wl | (uintptr_t)a.y | (uintptr_t)a.yh |
                         (uintptr_t)a.yl | (uintptr_t)a.b;
    return (al & 15) == 0;
}

hipError_t launch_conv_np_mfma(const NpConvArgs &a, hipStream_t st)
{
    // Tiles of 128 pixels x 64 channels with 64 x 32 per wavefront (six accumulator tiles, 160 registers) leave room for
    // several workgroups per compute unit, so that one workgroup's matrix instructions and loads run under another's
    // epilogue - worth more on every layer shape measured than the larger tiles' fewer LDS reads per matrix
    // instruction.  Up to 36 steps (all but the 3 x 3 x 512 layers): three workgroups with a two-stage ring; longer
    // reductions: two workgroups with three stages.
    if (a.oh) {
        if ((long long)a.R * a.S * a.C <= 36 * kStepBytes) return launch_np_mfma<128, 64, 3, 2, true>(a, st);
        return launch_np_mfma<128, 64, 2, 3, true>(a, st);
    }
    if ((long long)a.R * a.S * a.C <= 36 * kStepBytes) return launch_np_mfma<128, 64, 3, 2>(a, st);
    return launch_np_mfma<128, 64, 2, 3>(a, st);
}

hipError_t launch_conv_np_direct(const NpConvArgs &a, hipStream_t st)
{
    size_t total = (size_t)a.N * a.P * a.Q * a.K;
    size_t blocks = (total + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    conv_np_direct_kernel<<<(int)blocks, 256, 0, st>>>(a);
    return hipGetLastError();
}

hipError_t launch_clear_u64(unsigned long long *p, hipStream_t st)
{
    clear_u64_kernel<<<1, 1, 0, st>>>(p);
    return hipGetLastError();
}

static int grid_for(size_t work)
{
    size_t blocks = (work + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    return blocks < 1 ? 1 : (int)blocks;
}

hipError_t launch_eltwise_np_absmax(const int8_t *ah, const int8_t *al, const int8_t *bh, const int8_t *bl, size_t n, int sa, int sb, int relu,
                                    unsigned long long *amax, hipStream_t st)
{
    eltwise_np_absmax_kernel<<<grid_for(n), 256, 0, st>>>(ah, al, bh, bl, n, sa, sb, relu, amax);
    return hipGetLastError();
}

hipError_t launch_pool_np(const int8_t *xh, const int8_t *xl, uint8_t *y, int8_t *yh, int8_t *yl, int avg, int N, int H, int W, int C, int k,
                          int stride, int pad, int P, int Q, int p_fmt, int beta_max, hipStream_t st)
{
    NpPoolParams a{xh, xl, y, yh, yl, N, H, W, C, k, stride, pad, P, Q, p_fmt, beta_max, avg};
    const uintptr_t al4 = (uintptr_t)xh | (uintptr_t)xl | (uintptr_t)y | (uintptr_t)yh | (uintptr_t)yl;
    const size_t total = (size_t)N * P * Q * C;
    if (!avg && k == 3 && stride == 2 && pad == 1 && !y && C % 16 == 0 && (al4 & 15) == 0 && total / 16 < (1u << 31)) {
        NpMaxPool3Params prm;
        prm.a = a;
        prm.total = (int)(total / 16);
        prm.div_cv = make_fastdiv(C / 16);
        prm.div_q = make_fastdiv(Q);
        prm.div_p = make_fastdiv(P);
        maxpool3_np16_kernel<<<grid_for(total / 16), 256, 0, st>>>(prm);
    } else if (!avg && k == 3 && stride == 2 && pad == 1 && C % 4 == 0 && (al4 & 3) == 0)
        maxpool3_np_kernel<<<grid_for(total / 4), 256, 0, st>>>(a);
    else if (avg && k == H && k == W && pad == 0 && P == 1 && Q == 1 && C % 4 == 0 && (al4 & 3) == 0 && total / 4 < (1u << 31) &&
             (long long)k * k <= (1 << 18))
        avgpool_global_np4_kernel<<<grid_for(total / 4), 256, 0, st>>>(a);
    else
        pool_np_kernel<<<grid_for(total), 256, 0, st>>>(a);
    return hipGetLastError();
}

hipError_t launch_stem_pack_x(const int8_t *x, int8_t *y, int N, int H, int W, int C, int pad, int Hs, int Qs, hipStream_t st)
{
    if ((long long)N * H * W * C < (1LL << 31) - 16 && ((uintptr_t)x & 3) == 0)
        stem_pack_x_words_kernel<<<grid_for((size_t)N * Hs * Qs * 4), 256, 0, st>>>(x, y, N, H, W, C, pad, Hs, Qs);
    else
        stem_pack_x_kernel<<<grid_for((size_t)N * Hs * Qs * 4), 256, 0, st>>>(x, y, N, H, W, C, pad, Hs, Qs);
    return hipGetLastError();
}

hipError_t launch_stem_pack_w(const int8_t *w, int8_t *y, int K, int R, int S, int C, hipStream_t st)
{
    stem_pack_w_kernel<<<grid_for((size_t)K * 256), 256, 0, st>>>(w, y, K, R, S, C);
    return hipGetLastError();
}

hipError_t launch_eltwise_np(const int8_t *ah, const int8_t *al, const int8_t *bh, const int8_t *bl, uint8_t *y, int8_t *yh, int8_t *yl,
                             size_t n, int sa, int sb, int shift, int p_y, int beta_max, int relu, hipStream_t st)
{
    const uintptr_t al16 = (uintptr_t)ah | (uintptr_t)al | (uintptr_t)bh | (uintptr_t)bl | (uintptr_t)y | (uintptr_t)yh | (uintptr_t)yl;
    NpEltParams q{ah, al, bh, bl, y, yh, yl, (al16 & 15) ? 0 : n / 16, n, sa, sb, shift, p_y, beta_max, relu};
    size_t work = q.n16 > 0 ? q.n16 : n;
    size_t blocks = (work + 255) / 256;
    if (blocks > 256 * 16) blocks = 256 * 16;
    if (blocks < 1) blocks = 1;
    eltwise_np_kernel<<<(int)blocks, 256, 0, st>>>(q);
    return hipGetLastError();
}

hipError_t launch_np_digits(const uint8_t *codes, size_t n, int p, int8_t *hi, int8_t *lo, hipStream_t st)
{
    size_t blocks = (n + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    np_digits_kernel<<<(int)blocks, 256, 0, st>>>(codes, n, p, hi, lo);
    return hipGetLastError();
}

}  // namespace dfq
