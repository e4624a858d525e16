/*
 * CPU oracle for the int8 / power-of-two-scale case of the dynamic
 * floating-point quantization scheme (Settle et al., arXiv 1805.07941).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a slow, plain, loop-by-loop statement of
 * what every operation of the quantized-convolution path computes, written so
 * that it can be checked against the paper by eye.  Only the tests, the smoke
 * check and the benchmark's cpu_baseline leg may call it; the GPU library never
 * does, and the two share no code.
 *
 * Number format (Sec. 2.1, Eq. 1 with p = n-1 = 7 and alpha = 2^-f): a tensor
 * element is an int8 code `c`; its value is c * 2^-f, where the integer f
 * ("fractional length") is a property of the tensor.  Codes the scheme emits
 * lie in [-beta_max, beta_max] = [-127, 127] (Eq. 5 and the symmetric clamp
 * rule at the end of the multiply-accumulate analysis, Sec. 2.2).
 *
 * Every integer below is a mathematical integer held in int64_t; nothing is
 * blocked, fused or reordered.  OpenMP is used only across independent output
 * elements.
 *
 * Pins (tests/test_oracle_*.py): closed forms of Eq. 5, 8, 9, 12, 13; exact
 * rational arithmetic (fractions.Fraction / Python big ints) on tiny tensors;
 * numpy int64 matrix product for 1x1 convolutions; algebraic identities
 * (identity convolution, add-as-MAC, ReLU order, odd symmetry).  Network-level
 * results have no pin outside the oracle itself: "parity unpinned" for the
 * end-to-end logits (only their per-layer ingredients are pinned).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>

/* ------------------------------------------------------------------------- */
/* Closed forms of Sec. 2.1 / 2.2                                             */
/* ------------------------------------------------------------------------- */

/* Eq. 5: largest code magnitude of an n-bit format with p significand bits
 * when the Inf/NaN codes are reused as numbers (equality case). */
int64_t orc_beta_max(int n, int p)
{
    if (n < 2 || p < 0 || p > n - 1) return -1;
    if (p == n - 1) return ((int64_t)1 << (n - 1)) - 1;
    int e = (1 << (n - p - 1)) - 2; /* 2^(n-p-1) - 2 */
    if (e > 40) return -1;
    return ((int64_t)1 << e) * (((int64_t)1 << (p + 1)) - 1);
}

/* smallest q with 2^(q-1) >= m, i.e. ceil(log2(m)) + 1, for an integer m >= 1;
 * evaluated with integers so that no logarithm is rounded. */
static int ceil_log2_plus1(uint64_t m)
{
    int q = 1;
    uint64_t pw = 1; /* 2^(q-1) */
    while (pw < m) { pw <<= 1; q++; }
    return q;
}

/* Eq. 8 (reading the second factor as b_y + eps_y, as in Eq. 9): accumulator
 * width for N products of codes in [-(b_x+eps_x), b_x] x [-(b_y+eps_y), b_y]. */
int orc_mac_acc_bits(int64_t N, int64_t bx, int64_t ex, int64_t by, int64_t ey)
{
    if (N < 1 || bx < 1 || by < 1 || ex < 0 || ey < 0) return -1;
    uint64_t m = (uint64_t)N * (uint64_t)(bx + ex) * (uint64_t)(by + ey) + 1;
    return ceil_log2_plus1(m);
}

/* Eq. 9: longest sum of products a q-bit accumulator holds exactly. */
int64_t orc_mac_max_len(int q, int64_t bx, int64_t ex, int64_t by, int64_t ey)
{
    if (q < 2 || q > 63 || bx < 1 || by < 1 || ex < 0 || ey < 0) return -1;
    return ((((int64_t)1) << (q - 1)) - 1) / ((bx + ex) * (by + ey));
}

/* Eq. 12: accumulator width for a sum of N codes in [-(b_x+eps_x), b_x]. */
int orc_add_acc_bits(int64_t N, int64_t bx, int64_t ex)
{
    if (N < 1 || bx < 1 || ex < 0) return -1;
    if (ex == 0) return ceil_log2_plus1((uint64_t)N * (uint64_t)bx + 1);
    return ceil_log2_plus1((uint64_t)N * (uint64_t)bx + (uint64_t)N * (uint64_t)ex);
}

/* Eq. 13: longest sum a q-bit accumulator holds exactly. */
int64_t orc_add_max_len(int q, int64_t bx, int64_t ex)
{
    if (q < 2 || q > 63 || bx < 1 || ex < 0) return -1;
    if (ex == 0) return ((((int64_t)1) << (q - 1)) - 1) / bx;
    return (((int64_t)1) << (q - 1)) / (bx + ex);
}

/* ------------------------------------------------------------------------- */
/* Rounding and saturation                                                    */
/* ------------------------------------------------------------------------- */

/* Symmetric clamp to [-beta_max, beta_max] (Sec. 2.2, eps = 0 requirement). */
static int sat8(int64_t t)
{
    if (t > 127) return 127;
    if (t < -127) return -127;
    return (int)t;
}

/* v * 2^-s rounded to the nearest integer, ties to the even integer.
 * Valid for |v| < 2^62 and any s in [-62, 62] whose result fits int64. */
int64_t orc_rne_shift(int64_t v, int s)
{
    if (s == 0) return v;
    if (s < 0) return v * ((int64_t)1 << (-s));
    int64_t d = (int64_t)1 << s;
    int64_t t = v / d;
    int64_t rem = v % d;
    if (rem < 0) { t -= 1; rem += d; } /* floor division */
    int64_t half = d / 2;
    if (rem > half || (rem == half && (t & 1))) t += 1;
    return t;
}

/* sat8(v * 2^-s rounded ties-to-even) for |v| <= 2^32 and ANY integer s:
 * a large right shift gives 0, a large left shift of a non-zero v saturates. */
int orc_requant8(int64_t v, int s)
{
    if (s >= 40) return 0;              /* |v| * 2^-40 < 1/2 */
    if (s <= -32) return v == 0 ? 0 : (v > 0 ? 127 : -127);
    return sat8(orc_rne_shift(v, s));
}

/* num/den (den > 0) rounded to the nearest integer, ties to even. */
static int64_t rne_div(int64_t num, int64_t den)
{
    int64_t t = num / den;
    int64_t rem = num % den;
    if (rem < 0) { t -= 1; rem += den; }
    if (2 * rem > den || (2 * rem == den && (t & 1))) t += 1;
    return t;
}

/* ------------------------------------------------------------------------- */
/* float <-> code (Sec. 3, conversion paragraph)                              */
/* ------------------------------------------------------------------------- */

/* code = sat8(round_ties_even(x * 2^f)); NaN -> 0; +-Inf -> +-127.
 * x * 2^f is exact in double for every float x and |f| <= 64. */
void orc_quantize(const float *x, int8_t *q, size_t n, int f)
{
    for (size_t i = 0; i < n; i++) {
        double v = (double)x[i];
        int c;
        if (isnan(v)) c = 0;
        else {
            double t = nearbyint(ldexp(v, f)); /* default mode: ties to even */
            if (t > 127.0) c = 127;
            else if (t < -127.0) c = -127;
            else c = (int)t;
        }
        q[i] = (int8_t)c;
    }
}

/* same conversion into a 32-bit code, saturating at +-(2^31 - 1): the bias of a
 * convolution is stored like this at fractional length f_in + f_w (Sec. 3). */
void orc_quantize_i32(const float *x, int32_t *q, size_t n, int f)
{
    const double lim = 2147483647.0;
    for (size_t i = 0; i < n; i++) {
        double v = (double)x[i];
        int32_t c;
        if (isnan(v)) c = 0;
        else {
            double t = nearbyint(ldexp(v, f));
            if (t > lim) c = INT32_MAX;
            else if (t < -lim) c = -INT32_MAX;
            else c = (int32_t)t;
        }
        q[i] = c;
    }
}

/* value = code * 2^-f, exact in float. */
void orc_dequantize(const int8_t *q, float *x, size_t n, int f)
{
    for (size_t i = 0; i < n; i++) x[i] = (float)ldexp((double)q[i], -f);
}

/* ------------------------------------------------------------------------- */
/* Convolution / inner product (Eq. 6): integer sum of products, bias, ReLU,   */
/* one power-of-two rescale, clamp.                                            */
/* ------------------------------------------------------------------------- */

typedef struct {
    int N, H, W, C, K, R, S, stride, pad, groups;
} conv_shape;

static int conv_out_dim(int in, int pad, int k, int stride)
{
    int span = in + 2 * pad - k;
    if (span < 0) return 0;
    return span / stride + 1;
}

/* The accumulator of ONE output element (n, p, q, k): sum over taps (r, s) and
 * the input channels of k's group of code * weight; taps that fall outside the
 * image contribute nothing (the code of the value 0 is 0).  The bias, an
 * integer at fractional length f_in + f_w, is added when present. */
static int64_t conv_acc_one(const int8_t *x, const int8_t *w, const int32_t *b,
                            const conv_shape *sh, int n, int p, int q, int k)
{
    int Cg = sh->C / sh->groups;
    int Kg = sh->K / sh->groups;
    int g = k / Kg;
    int64_t acc = 0;
    for (int r = 0; r < sh->R; r++) {
        int ih = p * sh->stride - sh->pad + r;
        if (ih < 0 || ih >= sh->H) continue;
        for (int s = 0; s < sh->S; s++) {
            int iw = q * sh->stride - sh->pad + s;
            if (iw < 0 || iw >= sh->W) continue;
            const int8_t *xp = x + (((size_t)n * sh->H + ih) * sh->W + iw) * sh->C + (size_t)g * Cg;
            const int8_t *wp = w + (((size_t)k * sh->R + r) * sh->S + s) * Cg;
            for (int c = 0; c < Cg; c++) acc += (int64_t)xp[c] * (int64_t)wp[c];
        }
    }
    if (b) acc += (int64_t)b[k];
    return acc;
}

static int conv_shape_ok(const conv_shape *sh)
{
    if (sh->N < 0 || sh->H < 1 || sh->W < 1 || sh->C < 1 || sh->K < 1 || sh->R < 1 || sh->S < 1) return 0;
    if (sh->stride < 1 || sh->pad < 0 || sh->groups < 1) return 0;
    if (sh->C % sh->groups || sh->K % sh->groups) return 0;
    if (conv_out_dim(sh->H, sh->pad, sh->R, sh->stride) < 1) return 0;
    if (conv_out_dim(sh->W, sh->pad, sh->S, sh->stride) < 1) return 0;
    return 1;
}

/* accumulator (bias included) of one output element; for sampled checks of
 * tensors too large to compute whole. */
int64_t orc_conv_acc_at(const int8_t *x, const int8_t *w, const int32_t *b,
                        int N, int H, int W, int C, int K, int R, int S,
                        int stride, int pad, int groups, int n, int p, int q, int k)
{
    conv_shape sh = {N, H, W, C, K, R, S, stride, pad, groups};
    return conv_acc_one(x, w, b, &sh, n, p, q, k);
}

/*
 * x: [N][H][W][C] codes at f_in; w: [K][R][S][C/groups] codes at f_w;
 * b: [K] int32 at f_in + f_w or NULL; y: [N][P][Q] pixels of ldy bytes each, the
 * first K of which are written (codes at f_out), or NULL; acc_out: [N][P][Q][K]
 * int32 accumulators including the bias, before ReLU, or NULL.
 * Returns 0, -1 for a bad shape, or 1 if some accumulator left the int32 range
 * (the precondition of Eq. 8 / 9 was violated; outputs are then still the exact
 * mathematical result, which a 32-bit accumulator could not have produced).
 */
int orc_conv_q(const int8_t *x, const int8_t *w, const int32_t *b, int8_t *y, int32_t *acc_out,
               int N, int H, int W, int C, int K, int R, int S, int stride, int pad, int groups,
               int ldy, int f_in, int f_w, int f_out, int relu)
{
    conv_shape sh = {N, H, W, C, K, R, S, stride, pad, groups};
    if (!conv_shape_ok(&sh) || ldy < K) return -1;
    int P = conv_out_dim(H, pad, R, stride);
    int Q = conv_out_dim(W, pad, S, stride);
    int shift = f_in + f_w - f_out;
    int overflow = 0;
#pragma omp parallel for collapse(2) schedule(static) reduction(| : overflow)
    for (int n = 0; n < N; n++) {
        for (int p = 0; p < P; p++) {
            for (int q = 0; q < Q; q++) {
                size_t pix = ((size_t)n * P + p) * Q + q;
                for (int k = 0; k < K; k++) {
                    int64_t acc = conv_acc_one(x, w, b, &sh, n, p, q, k);
                    if (acc > INT32_MAX || acc < INT32_MIN) overflow = 1;
                    if (acc_out) acc_out[pix * K + k] = (int32_t)acc;
                    if (y) {
                        int64_t v = (relu && acc < 0) ? 0 : acc;
                        y[pix * (size_t)ldy + k] = (int8_t)orc_requant8(v, shift);
                    }
                }
            }
        }
    }
    return overflow;
}

/* The same layer with one weight format per output channel (Sec. 3, "Calibrating": weight
 * thresholds are taken per output channel): f_w[k] is the fractional length of w[k][.][.][.],
 * b[k] is at f_in + f_w[k], and the rescale of Eq. 6 for channel k is a rounding shift by
 * f_in + f_w[k] - f_out.  Everything else as orc_conv_q. */
int orc_conv_q_pc(const int8_t *x, const int8_t *w, const int32_t *b, int8_t *y, int32_t *acc_out,
                  int N, int H, int W, int C, int K, int R, int S, int stride, int pad, int groups,
                  int ldy, int f_in, const int32_t *f_w, int f_out, int relu)
{
    conv_shape sh = {N, H, W, C, K, R, S, stride, pad, groups};
    if (!conv_shape_ok(&sh) || ldy < K || !f_w) return -1;
    int P = conv_out_dim(H, pad, R, stride);
    int Q = conv_out_dim(W, pad, S, stride);
    int overflow = 0;
#pragma omp parallel for collapse(2) schedule(static) reduction(| : overflow)
    for (int n = 0; n < N; n++) {
        for (int p = 0; p < P; p++) {
            for (int q = 0; q < Q; q++) {
                size_t pix = ((size_t)n * P + p) * Q + q;
                for (int k = 0; k < K; k++) {
                    int64_t acc = conv_acc_one(x, w, b, &sh, n, p, q, k);
                    if (acc > INT32_MAX || acc < INT32_MIN) overflow = 1;
                    if (acc_out) acc_out[pix * K + k] = (int32_t)acc;
                    if (y) {
                        int64_t v = (relu && acc < 0) ? 0 : acc;
                        y[pix * (size_t)ldy + k] = (int8_t)orc_requant8(v, f_in + f_w[k] - f_out);
                    }
                }
            }
        }
    }
    return overflow;
}

/* The last step of Eq. 6 on its own: y[i] = sat8(rne(relu ? max(acc[i],0) : acc[i], shift)).
 * Lets calibration requantize accumulators it already holds instead of convolving again. */
void orc_requant_i32(const int32_t *acc, int8_t *y, size_t n, int shift, int relu)
{
    for (size_t i = 0; i < n; i++) {
        int64_t v = acc[i];
        if (relu && v < 0) v = 0;
        y[i] = (int8_t)orc_requant8(v, shift);
    }
}

/* Convolution followed by an element-wise add with ONE rounding (Sec. 3 wants a value thresholded only when the
 * datapath can carry it no further; Eq. 6 and Eq. 10 at the accumulator's scale): the accumulator
 * acc[i] (sum of Eq. 6 plus bias, at f_acc = f_in + f_w) and the code other[i] (at f_other <= f_acc) brought to f_acc by
 * the exact factor 2^(f_acc - f_other) are summed without loss, ReLU acts on the sum if asked, and the sum is rescaled
 * once to f_out: y[i] = sat8(rne(acc[i] + other[i] * 2^sb, shift)).  Returns -1 unless 0 <= sb <= 22. */
int orc_add_lazy(const int32_t *acc, const int8_t *other, int8_t *y, size_t n, int sb, int shift, int relu)
{
    if (sb < 0 || sb > 22) return -1;
    for (size_t i = 0; i < n; i++) {
        int64_t v = (int64_t)acc[i] + (int64_t)other[i] * ((int64_t)1 << sb);
        if (relu && v < 0) v = 0;
        y[i] = (int8_t)orc_requant8(v, shift);
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Scaled addition (Eq. 10) and the joins built on it                          */
/* ------------------------------------------------------------------------- */

/*
 * y = quantize(value(a) + value(b), f_y): both codes are brought to the finer
 * of the two scales F = max(f_a, f_b) by exact multiplication, added, and the
 * sum is rescaled ONCE to f_y.  acc_out (nullable) receives the sum at F before
 * ReLU.  Requires F - f_a <= 22 and F - f_b <= 22 (the aligned sum then fits a
 * 32-bit accumulator, Eq. 12); returns -1 otherwise.
 */
int orc_eltwise_q(const int8_t *a, int f_a, const int8_t *b, int f_b, int8_t *y, int f_y,
                  int32_t *acc_out, size_t n, int relu)
{
    int F = f_a > f_b ? f_a : f_b;
    if (F - f_a > 22 || F - f_b > 22) return -1;
    int64_t ma = (int64_t)1 << (F - f_a), mb = (int64_t)1 << (F - f_b);
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; i++) {
        int64_t sum = (int64_t)a[i] * ma + (int64_t)b[i] * mb;
        if (acc_out) acc_out[i] = (int32_t)sum;
        if (y) {
            if (relu && sum < 0) sum = 0;
            y[i] = (int8_t)orc_requant8(sum, F - f_y);
        }
    }
    return 0;
}

/*
 * Channel concatenation of nb branches that share the pixel grid: branch i has
 * Cs[i] channels at fractional length fs[i]; every code is rescaled (the N = 1
 * case of Eq. 10) into the common output format and copied to its channel slot.
 */
int orc_concat_q(int nb, const int8_t *const *xs, const int *Cs, const int *fs,
                 int8_t *y, int f_y, size_t pixels)
{
    if (nb < 1) return -1;
    size_t Ct = 0;
    for (int i = 0; i < nb; i++) { if (Cs[i] < 1) return -1; Ct += (size_t)Cs[i]; }
    size_t off = 0;
    for (int i = 0; i < nb; i++) {
        for (size_t px = 0; px < pixels; px++)
            for (int c = 0; c < Cs[i]; c++)
                y[px * Ct + off + c] = (int8_t)orc_requant8(xs[i][px * Cs[i] + c], fs[i] - f_y);
        off += (size_t)Cs[i];
    }
    return 0;
}

/*
 * Pooling over k x k windows, NHWC.  mode 0 = max over the window positions that
 * lie inside the image (padding never wins), then one rescale f_in -> f_out.
 * mode 1 = average: the exact rational  (sum of in-image codes) * 2^(f_out-f_in)
 * / (k*k)  (padded positions count as zeros in the divisor), rounded once to the
 * nearest integer with ties to even, then clamped.
 * A window with no in-image position cannot occur when pad < k.
 */
int orc_pool_q(const int8_t *x, int8_t *y, int mode, int N, int H, int W, int C,
               int k, int stride, int pad, int f_in, int f_out)
{
    if (N < 0 || H < 1 || W < 1 || C < 1 || k < 1 || k > 64 || stride < 1 || pad < 0 || pad >= k) return -1;
    if (mode != 0 && mode != 1) return -1;
    int P = conv_out_dim(H, pad, k, stride), Q = conv_out_dim(W, pad, k, stride);
    if (P < 1 || Q < 1) return -1;
    int d = f_out - f_in;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; n++) {
        for (int p = 0; p < P; p++) {
            for (int q = 0; q < Q; q++) {
                for (int c = 0; c < C; c++) {
                    int64_t mx = -1000, sum = 0;
                    for (int r = 0; r < k; r++) {
                        int ih = p * stride - pad + r;
                        if (ih < 0 || ih >= H) continue;
                        for (int s = 0; s < k; s++) {
                            int iw = q * stride - pad + s;
                            if (iw < 0 || iw >= W) continue;
                            int64_t v = x[(((size_t)n * H + ih) * W + iw) * C + c];
                            if (v > mx) mx = v;
                            sum += v;
                        }
                    }
                    int out;
                    if (mode == 0) out = orc_requant8(mx, -d);
                    else {
                        int64_t win = (int64_t)k * k;
                        if (d >= 32) out = sum == 0 ? 0 : (sum > 0 ? 127 : -127);
                        else if (d <= -40) out = 0;
                        else if (d >= 0) out = sat8(rne_div(sum * ((int64_t)1 << d), win));
                        else out = sat8(rne_div(sum, win * ((int64_t)1 << (-d))));
                    }
                    y[((((size_t)n * P + p) * Q + q)) * C + c] = (int8_t)out;
                }
            }
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Calibration building blocks (Sec. 3): thresholds gamma = max |value| and    */
/* the format they imply, gamma = alpha * beta_max with alpha = 2^-f.          */
/* ------------------------------------------------------------------------- */

/* max |x|; NaN elements are ignored. */
float orc_absmax_f32(const float *x, size_t n)
{
    float m = 0.0f;
    for (size_t i = 0; i < n; i++) {
        float a = fabsf(x[i]);
        if (a > m) m = a; /* false for NaN */
    }
    return m;
}

/* max |v| of 32-bit accumulators; with relu != 0, negative entries count as 0
 * (the threshold of a layer followed by ReLU is taken after the ReLU). */
int64_t orc_absmax_i32(const int32_t *x, size_t n, int relu)
{
    int64_t m = 0;
    for (size_t i = 0; i < n; i++) {
        int64_t v = x[i];
        if (v < 0) v = relu ? 0 : -v;
        if (v > m) m = v;
    }
    return m;
}

/* the same maximum separately for each of the K channels of an [pixels][K] array */
void orc_absmax_i32_channels(const int32_t *x, size_t pixels, int K, int relu, int64_t *out)
{
    for (int k = 0; k < K; k++) out[k] = 0;
    for (size_t i = 0; i < pixels; i++) {
        for (int k = 0; k < K; k++) {
            int64_t v = x[i * (size_t)K + k];
            if (v < 0) v = relu ? 0 : -v;
            if (v > out[k]) out[k] = v;
        }
    }
}

/* largest f in [-32, 32] with gamma * 2^f <= 127 (the smallest power-of-two
 * scale whose range still holds gamma); 32 for gamma = 0; -32 if none fits.
 * Returns -1000 for a negative, infinite or NaN gamma. */
int orc_frac_from_absmax_f32(float gamma)
{
    double g = (double)gamma;
    if (!(g >= 0.0) || isinf(g)) return -1000;
    for (int f = 32; f >= -32; f--)
        if (ldexp(g, f) <= 127.0) return f;
    return -32;
}

/* integer form: m is max |acc| of codes at fractional length acc_frac.  The
 * largest f <= acc_frac (rescale factor 2^(f-acc_frac) in (0, 1], Sec. 3) with
 * m * 2^(f - acc_frac) <= 127, floored at -32. */
int orc_frac_from_absmax_i32(int64_t m, int acc_frac)
{
    if (m < 0) return -1000;
    int f = acc_frac > 32 ? 32 : acc_frac;
    for (; f > -32; f--) {
        int sh = acc_frac - f; /* >= 0 */
        if (sh >= 40) return f; /* 127 * 2^40 exceeds any 32-bit magnitude */
        if (m <= (int64_t)127 * ((int64_t)1 << sh)) return f;
    }
    return -32;
}

/* number of OpenMP threads the loops above use (reported next to oracle timings) */
#ifdef _OPENMP
#include <omp.h>
int orc_num_threads(void) { return omp_get_max_threads(); }
#else
int orc_num_threads(void) { return 1; }
#endif


/* ---- preprocessing: a per-channel affine layer behind a convolution folded into its float weights (Sec. 3:
 * neighbouring linear operations are combined before quantizing).  z = scale[k]*(w[k].x + b[k]) + shift[k]
 * = (scale[k]*w[k]).x + (scale[k]*b[k] + shift[k]).  Single precision, as the weights are; every product and
 * the sum rounded separately (volatile keeps the compiler from contracting them). */
void orc_fold_scale(const float *w, const float *b, size_t rows, size_t row_len, const float *scale, const float *shift,
                    float *w_out, float *b_out)
{
    for (size_t r = 0; r < rows; r++) {
        for (size_t i = 0; i < row_len; i++) {
            volatile float p = w[r * row_len + i] * scale[r];
            w_out[r * row_len + i] = p;
        }
        if (b_out) {
            volatile float p = (b ? b[r] : 0.0f) * scale[r];
            volatile float q = p + (shift ? shift[r] : 0.0f);
            b_out[r] = q;
        }
    }
}
