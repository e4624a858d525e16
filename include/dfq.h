/*
 * dfq - quantized CNN inference primitives for AMD MI355X (gfx950), after
 * Settle et al., "Quantizing Convolutional Neural Networks for Low-Power
 * High-Throughput Inference Engines" (arXiv 1805.07941).
 *
 * The library implements the int8 member of the paper's dynamic floating-point
 * family (Sec. 2.1, Eq. 1 with n = 8, p = n-1 and a power-of-two scale
 * alpha = 2^-frac): a tensor element is an int8 code c whose value is
 * c * 2^-frac, with frac ("fractional length") a per-tensor integer.  Every code
 * the library WRITES lies in the symmetric range [-127, 127] (= +-beta_max of
 * Eq. 5; the clamp rule that closes the multiply-accumulate analysis of
 * Sec. 2.2).  Code -128 is accepted in inputs and weights.
 *
 * Rounding is to nearest, ties to even, everywhere (the paper leaves the mode
 * open; the format is described as an extension of IEEE 754, whose default this
 * is).  rne(v, s) below means v * 2^-s rounded that way (exact multiplication
 * when s < 0) and sat8 the clamp to [-127, 127].
 *
 * Conventions for every call
 *   - All tensor pointers are DEVICE pointers owned by the caller; the library
 *     allocates nothing, keeps no pointer and holds no state between calls.
 *     Arrays described as "host" (branch tables of dfq_concat_q, dfq_fmt* outputs)
 *     are ordinary host memory read or written before the call returns.
 *   - Activations are NHWC int8, densely packed unless a channel stride is given.
 *     Weights are [K][R][S][C/groups] int8.  Bias is [K] int32.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     enqueue work and return without synchronizing; results that live on the
 *     device (including the *_dev scalars) are ready when the stream reaches them.
 *   - Errors are return codes only.  Arguments are validated before anything is
 *     launched; on a non-zero status no work was enqueued.
 *   - Input and output buffers of one call must not overlap.
 */
#ifndef DFQ_H
#define DFQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* A tensor format: bits must be 8; value = code * 2^-frac; frac in [-32, 32]. */
typedef struct { int32_t bits; int32_t frac; } dfq_fmt;

typedef enum {
    DFQ_OK = 0,
    DFQ_EINVAL = 1,        /* null pointer, negative size, bad enum value */
    DFQ_ESHAPE = 2,        /* inconsistent or empty geometry */
    DFQ_EFMT = 3,          /* bits != 8, frac out of range, formats too far apart */
    DFQ_EUNSUPPORTED = 4,  /* valid request this build has no kernel for */
    DFQ_EDEVICE = 5        /* the HIP runtime refused a launch */
} dfq_status;

typedef enum { DFQ_POOL_MAX = 0, DFQ_POOL_AVG = 1 } dfq_pool_mode;

/* Which convolution kernel dfq_conv_q_variant runs. */
typedef enum {
    DFQ_CONV_AUTO = 0,     /* what dfq_conv_q picks */
    DFQ_CONV_DIRECT = 1,   /* one output element per lane; any shape */
    DFQ_CONV_MFMA = 2,     /* implicit GEMM on int8 MFMA; groups == 1, C % 16 == 0 */
    DFQ_CONV_DEPTHWISE = 3,/* groups == C == K, channel-vectorized VALU kernel; C % 4 == 0 */
    DFQ_CONV_SMALLC = 4,   /* implicit GEMM for few input channels (first layers); groups == 1, S*C <= 32 */
    DFQ_CONV_GROUPED = 6,  /* 1 < groups with (C/groups) % 4 == 0: vector-ALU kernel (4-way int8 dot products, weights in LDS);
                              S in {1, 3, 5, 7}, stride 1 or 2, K*R*S*C/groups <= 64 KB, 4-byte aligned x and w */
    DFQ_CONV_POINTWISE = 5 /* int8 MFMA with the input tile resident in LDS; unpadded 1x1 stride 1, groups == 1,
                              C in {64, 128, 192, 256}, K % 64 == 0, K <= 4096, (K / BC) * (C / 64) >= 2 and
                              512*C + 192*BC + 4*K <= 160 KB of LDS with BC = (K % 128 ? 64 : 128),
                              16-byte aligned x, w, y, ldy % 16 == 0, rescale shift f_in + f_w - f_out in [0, 23],
                              no acc_out */
} dfq_conv_variant;

typedef void *dfq_stream;

const char *dfq_status_string(dfq_status s);

/* ---- float <-> code (Sec. 3, the conversion paragraph before Algorithm 1) ------------
 * q[i] = sat8(round_ties_even(x[i] * 2^frac)); NaN -> 0, +-Inf -> +-127.
 * x: n floats, q: n bytes.  n == 0 is a no-op. */
dfq_status dfq_quantize(const float *x, int8_t *q, size_t n, dfq_fmt fmt, dfq_stream stream);

/* Same conversion into 32-bit codes saturating at +-(2^31 - 1); frac in [-64, 64].  Used
 * for the bias of a convolution, held at frac_in + frac_w (Sec. 3: bias thresholds as a
 * function of input and weight thresholds). */
dfq_status dfq_quantize_i32(const float *x, int32_t *q, size_t n, int32_t frac, dfq_stream stream);

/* x[i] = q[i] * 2^-frac, exact in float. */
dfq_status dfq_dequantize(const int8_t *q, float *x, size_t n, dfq_fmt fmt, dfq_stream stream);

/* ---- the general (n, p) dynamic floating-point codes (Sec. 2.1, Eq. 1-5) ----------------------------
 * A code has nbits <= 8 bits in one byte (upper bits zero): bit nbits-1 the sign, bits nbits-2 .. p the exponent
 * field e (Eq. 4; none when p == nbits-1), bits p-1 .. 0 the significand field m.  Sign and magnitude (Eq. 2):
 *   value = (-1)^sign * 2^-frac * (e == 0 ? m : 2^(e-1) * (2^p + m))
 * with subnormals and with every exponent code a number (no infinities, no NaNs: the paper's default), so the
 * largest value is 2^-frac * beta_max(nbits, p) (Eq. 5; dfq_beta_max).  nbits = 8, p = 6 or 7 is the int8 format
 * of the rest of this library in sign-and-magnitude dress; p = 4 and p = 3 are the 8-bit members Sec. 5 reports
 * as the most accurate.
 * dfq_quantize_np: clamp to +-beta_max * 2^-frac, divide by 2^-frac, round to the nearest representable value
 * (ties to the even significand); NaN -> code 0, +-Inf saturate; the code of -0 is never written.
 * dfq_dequantize_np: the value above, exact in float (bits above nbits are ignored).
 * 2 <= nbits <= 8, 0 <= p <= nbits-1, at most 5 exponent bits, frac in [-32, 32]: DFQ_EFMT otherwise.
 * x: n floats, codes: n bytes, both DEVICE.  n == 0 is a no-op. */
dfq_status dfq_quantize_np(const float *x, uint8_t *codes, size_t n, int nbits, int p, int frac, dfq_stream stream);
dfq_status dfq_dequantize_np(const uint8_t *codes, float *x, size_t n, int nbits, int p, int frac, dfq_stream stream);

/* ---- convolution / inner product (Sec. 2.2, Eq. 6) -------------------------------------
 * acc[n,p,q,k] = sum_{r,s,c} x[n, p*stride-pad+r, q*stride-pad+s, g*Cg+c] * w[k,r,s,c] + b[k]
 * with Cg = C/groups, g = k / (K/groups); taps outside the image contribute 0.
 * y[n,p,q,k]   = sat8(rne(relu ? max(acc,0) : acc, fmt_in.frac + fmt_w.frac - fmt_out.frac)).
 * P = floor((H + 2*pad - R)/stride) + 1, Q likewise with W and S.
 *
 * x   [N][H][W][C] int8 at fmt_in          w  [K][R][S][Cg] int8 at fmt_w
 * b   [K] int32 at fmt_in.frac+fmt_w.frac, or NULL (no bias)
 * y   [N*P*Q] pixels of ldy bytes each, the first K written; ldy >= K lets a layer write
 *     straight into a channel slice of a wider tensor.  May be NULL if acc_out is given.
 * acc_out  NULL, or [N][P][Q][K] int32 receiving acc (bias included, before ReLU): the
 *     calibration / debugging view of the wide accumulator.
 * The 32-bit accumulator is exact as long as R*S*Cg <= 131071 (Eq. 9 with q = 32 and
 * codes down to -128) and |b[k]| + R*S*Cg*2^14 < 2^31; the first is checked
 * (DFQ_EUNSUPPORTED), the second is the caller's precondition.
 * A fully connected layer is the case H = W = R = S = 1.  N == 0 is a no-op. */
dfq_status dfq_conv_q(const int8_t *x, const int8_t *w, const int32_t *b, int8_t *y, int32_t *acc_out,
                      int N, int H, int W, int C, int K, int R, int S, int stride, int pad, int groups,
                      int ldy, dfq_fmt fmt_in, dfq_fmt fmt_w, dfq_fmt fmt_out, int relu, dfq_stream stream);

/* Same operation with the kernel chosen by the caller (tests, benchmarks).  Returns
 * DFQ_EUNSUPPORTED if that kernel cannot run the shape. */
dfq_status dfq_conv_q_variant(dfq_conv_variant variant,
                              const int8_t *x, const int8_t *w, const int32_t *b, int8_t *y, int32_t *acc_out,
                              int N, int H, int W, int C, int K, int R, int S, int stride, int pad, int groups,
                              int ldy, dfq_fmt fmt_in, dfq_fmt fmt_w, dfq_fmt fmt_out, int relu, dfq_stream stream);

/* The same layer with one weight format per OUTPUT CHANNEL (Sec. 3, "Calibrating": the weight
 * thresholds are maxima per output channel).  frac_w: DEVICE array of K fractional lengths,
 * 4-byte aligned, read by the kernel only.  frac_w_lo <= frac_w_hi, both in [-32, 32]: bounds
 * the CALLER guarantees for every entry (it computed them); the library picks its kernel from
 * them and cannot check the array itself - an entry outside the declared bounds gives an
 * unspecified code for that channel (never a fault).  w[k][.][.][.] holds codes at
 * frac_w[k], b[k] is at fmt_in.frac + frac_w[k], and channel k is rescaled by one rounding
 * shift of fmt_in.frac + frac_w[k] - fmt_out.frac.  Everything else, including errors and the
 * optional accumulator dump, as dfq_conv_q.  With equal entries the result is that of
 * dfq_conv_q at that format. */
dfq_status dfq_conv_q_pc(const int8_t *x, const int8_t *w, const int32_t *b, int8_t *y, int32_t *acc_out,
                         int N, int H, int W, int C, int K, int R, int S, int stride, int pad, int groups,
                         int ldy, dfq_fmt fmt_in, const int32_t *frac_w, int frac_w_lo, int frac_w_hi,
                         dfq_fmt fmt_out, int relu, dfq_stream stream);

/* Convolution followed by an element-wise add, in one kernel (Sec. 3: adjacent operations are
 * merged; Eq. 10 for the add).  The result is exactly that of
 *     dfq_conv_q(x, w, b, t, NULL, ..., ldy = K, fmt_in, fmt_w, fmt_mid, relu_mid)   followed by
 *     dfq_eltwise_q(t, fmt_mid, other, fmt_other, y, fmt_out, NULL, N*P*Q*K, relu_out)
 * without the int8 tensor t ever being stored: each convolution result is rounded to fmt_mid in
 * registers, aligned with the code of `other` at the finer of the two scales, and the sum is
 * rounded once to fmt_out.  `other`: device, int8 [N, P, Q, K] with ld_other bytes between pixels
 * (>= K), read only, must not overlap y or x.  All other arguments as for dfq_conv_q.
 * Returns DFQ_EUNSUPPORTED - and does nothing - when no fused kernel covers the call (the caller
 * then issues the two calls above).  Fused kernels exist for unpadded 1x1 stride-1 layers with
 * groups == 1 that either meet what DFQ_CONV_POINTWISE needs, or have C % 64 == 0, K % 256 == 0,
 * 16-byte aligned x, w, y, ldy % 16 == 0 and a rescale shift in [0, 23]; both need `other` 16-byte
 * aligned with ld_other % 16 == 0, and max(f_mid, f_other) - f_out in [0, 23]. */
dfq_status dfq_conv_q_add(const int8_t *x, const int8_t *w, const int32_t *b, const int8_t *other, int8_t *y,
                          int N, int H, int W, int C, int K, int R, int S, int stride, int pad, int groups,
                          int ldy, int ld_other, dfq_fmt fmt_in, dfq_fmt fmt_w, dfq_fmt fmt_mid, int relu_mid,
                          dfq_fmt fmt_other, dfq_fmt fmt_out, int relu_out, dfq_stream stream);

/* Convolution followed by max-pooling, in one kernel (Sec. 3: adjacent operations are merged; the paper
 * names max-pool among the layers of the path).  The result is exactly that of
 *     dfq_conv_q(x, w, b, t, NULL, ..., ldy = K, fmt_in, fmt_w, fmt_out, relu)   followed by
 *     dfq_pool_q(t, y, DFQ_POOL_MAX, N, P, Q, K, pool_k, pool_stride, pool_pad, fmt_out, fmt_out)
 * without the int8 tensor t ever being stored (the pooling keeps the convolution's format, so it
 * rounds nothing).  y: device, int8 [N, PP, PQ, K] with ldy bytes between pixels (>= K, a multiple of
 * 16, y 16-byte aligned), PP = floor((P + 2*pool_pad - pool_k)/pool_stride) + 1, PQ likewise; must not
 * overlap x.  All other arguments as for dfq_conv_q.  Returns DFQ_EUNSUPPORTED - and does nothing -
 * when no fused kernel covers the call (the caller then issues the two calls above).  A fused kernel
 * exists for first layers: C == 3, stride 2, groups == 1, R in {3, 7}, S + (pad & 1) <= 8, pad <= 4,
 * K in {32, 64}, W % 4 == 0, W <= 256, P and Q even, Q <= 122, x 4-byte aligned, a rescale shift in
 * [0, 23], followed by a 3x3 / stride 2 / pad 1 pooling. */
dfq_status dfq_conv_q_maxpool(const int8_t *x, const int8_t *w, const int32_t *b, int8_t *y,
                              int N, int H, int W, int C, int K, int R, int S, int stride, int pad, int groups,
                              int ldy, dfq_fmt fmt_in, dfq_fmt fmt_w, dfq_fmt fmt_out, int relu,
                              int pool_k, int pool_stride, int pool_pad, dfq_stream stream);

/* dfq_conv_q_maxpool on float images: the conversion of the network's input (Sec. 3, conversion paragraph)
 * merged into the first layer as well.  The result is exactly that of
 *     dfq_quantize(x, t, N*H*W*C, fmt_in)   followed by   dfq_conv_q_maxpool(t, w, b, y, ...)
 * without the int8 image t ever being stored.  x: device, float32 [N][H][W][C], 16-byte aligned, must not overlap y.
 * Everything else, the DFQ_EUNSUPPORTED rule and the shapes covered as for dfq_conv_q_maxpool. */
dfq_status dfq_quantize_conv_q_maxpool(const float *x, const int8_t *w, const int32_t *b, int8_t *y,
                                       int N, int H, int W, int C, int K, int R, int S, int stride, int pad, int groups,
                                       int ldy, dfq_fmt fmt_in, dfq_fmt fmt_w, dfq_fmt fmt_out, int relu,
                                       int pool_k, int pool_stride, int pool_pad, dfq_stream stream);

/* The conversion of float images merged into a first layer that no pooling follows: exactly
 *     dfq_quantize(x, t, N*H*W*C, fmt_in)   followed by   dfq_conv_q(t, w, b, y, NULL, ...)
 * without the int8 image t being stored.  x: device, float32 [N][H][W][C], 16-byte aligned, must not overlap y; no accumulator
 * dump.  DFQ_EUNSUPPORTED - nothing done - when no fused kernel covers the call: one exists for C == 3, stride 2, groups == 1,
 * R in {3, 7}, S + (pad & 1) <= 8, pad <= 4, K == 32, W % 4 == 0, W <= 256, Q % 16 == 0, y 16-byte aligned with ldy % 16 == 0,
 * a rescale shift in [0, 23]. */
dfq_status dfq_quantize_conv_q(const float *x, const int8_t *w, const int32_t *b, int8_t *y,
                               int N, int H, int W, int C, int K, int R, int S, int stride, int pad, int groups,
                               int ldy, dfq_fmt fmt_in, dfq_fmt fmt_w, dfq_fmt fmt_out, int relu, dfq_stream stream);

/* dfq_conv_q_maxpool and dfq_quantize_conv_q_maxpool with one weight format per output channel: the result of
 * dfq_conv_q_pc(..., fmt_out, relu) followed by dfq_pool_q(., DFQ_POOL_MAX, ..., fmt_out, fmt_out) (with dfq_quantize in
 * front for the second).  frac_w, frac_w_lo, frac_w_hi as in dfq_conv_q_pc; the fused kernel needs every rounding shift
 * fmt_in.frac + frac_w[k] - fmt_out.frac in [0, 23] (judged from the declared bounds); everything else as above. */
dfq_status dfq_conv_q_pc_maxpool(const int8_t *x, const int8_t *w, const int32_t *b, int8_t *y,
                                 int N, int H, int W, int C, int K, int R, int S, int stride, int pad, int groups,
                                 int ldy, dfq_fmt fmt_in, const int32_t *frac_w, int frac_w_lo, int frac_w_hi, dfq_fmt fmt_out,
                                 int relu, int pool_k, int pool_stride, int pool_pad, dfq_stream stream);
dfq_status dfq_quantize_conv_q_pc_maxpool(const float *x, const int8_t *w, const int32_t *b, int8_t *y,
                                          int N, int H, int W, int C, int K, int R, int S, int stride, int pad, int groups,
                                          int ldy, dfq_fmt fmt_in, const int32_t *frac_w, int frac_w_lo, int frac_w_hi,
                                          dfq_fmt fmt_out, int relu, int pool_k, int pool_stride, int pool_pad, dfq_stream stream);

/* Convolution followed by an element-wise add with ONE rounding (Sec. 3 wants a value thresholded only when the
 * datapath can carry it no further): the convolution's accumulator (Eq. 6 with bias, at fmt_in.frac + fmt_w.frac;
 * it gets no format of its own and no ReLU) and the code of `other` brought to that scale by the exact factor
 * 2^(fmt_in.frac + fmt_w.frac - fmt_other.frac) are summed without loss, ReLU acts on the sum if relu_out, and
 *     y = sat8(rne(sum, fmt_in.frac + fmt_w.frac - fmt_out.frac)).
 * A different arithmetic from dfq_conv_q_add (which rounds the convolution's result to fmt_mid first, as Eq. 6
 * followed by Eq. 10 on stored tensors does): results agree where the first rounding loses nothing and are the more
 * accurate ones elsewhere.  fmt_other must be 0 .. 22 bits coarser than the accumulator (DFQ_EFMT otherwise).  Same
 * kernels, argument conventions and DFQ_EUNSUPPORTED rule as dfq_conv_q_add (the final shift must lie in [0, 23]);
 * one weight format per layer only. */
dfq_status dfq_conv_q_add_lazy(const int8_t *x, const int8_t *w, const int32_t *b, const int8_t *other, int8_t *y,
                               int N, int H, int W, int C, int K, int R, int S, int stride, int pad, int groups,
                               int ldy, int ld_other, dfq_fmt fmt_in, dfq_fmt fmt_w, dfq_fmt fmt_other, dfq_fmt fmt_out,
                               int relu_out, dfq_stream stream);

/* dfq_conv_q_add with one weight format per output channel: the result of dfq_conv_q_pc(...,
 * fmt_mid, relu_mid) followed by dfq_eltwise_q(., fmt_mid, other, fmt_other, y, fmt_out, ...).
 * frac_w, frac_w_lo, frac_w_hi as in dfq_conv_q_pc; everything else as in dfq_conv_q_add. */
dfq_status dfq_conv_q_pc_add(const int8_t *x, const int8_t *w, const int32_t *b, const int8_t *other, int8_t *y,
                             int N, int H, int W, int C, int K, int R, int S, int stride, int pad, int groups,
                             int ldy, int ld_other, dfq_fmt fmt_in, const int32_t *frac_w, int frac_w_lo,
                             int frac_w_hi, dfq_fmt fmt_mid, int relu_mid, dfq_fmt fmt_other, dfq_fmt fmt_out,
                             int relu_out, dfq_stream stream);

/* The variant dfq_conv_q would run for this geometry (host, pure) when the tensors are 16-byte
 * aligned, ldy == K, the rescale shift lies in [0, 23] and no accumulator dump is asked for;
 * DFQ_CONV_AUTO if the geometry is invalid. */
dfq_conv_variant dfq_conv_q_select(int N, int H, int W, int C, int K, int R, int S, int stride, int pad, int groups);

/* ---- scaled addition (Sec. 2.2, Eq. 10) -------------------------------------------------
 * F = max(fa.frac, fb.frac); sum = a*2^(F-fa.frac) + b*2^(F-fb.frac)  (exact);
 * y = sat8(rne(relu ? max(sum,0) : sum, F - fy.frac)): the exact sum rounded once.
 * a, b, y: n bytes.  acc_out: NULL or n int32 receiving sum (before ReLU).  y may be NULL
 * if acc_out is given.  Both alignment shifts must be <= 22 (DFQ_EFMT otherwise). */
dfq_status dfq_eltwise_q(const int8_t *a, dfq_fmt fa, const int8_t *b, dfq_fmt fb, int8_t *y, dfq_fmt fy,
                         int32_t *acc_out, size_t n, int relu, dfq_stream stream);

/* ---- concat with per-branch rescale (Sec. 3: matching the scales of the inputs of a join;
 * the N = 1 case of Eq. 10) -----------------------------------------------------------------
 * y[px][off_i + c] = sat8(rne(xs[i][px][c], fs[i].frac - fy.frac)), off_i = Cs[0]+...+Cs[i-1].
 * xs: HOST array of nbranch device pointers, branch i is [pixels][Cs[i]] int8;
 * Cs, fs: HOST arrays.  y: [pixels][sum Cs].  1 <= nbranch <= 8. */
dfq_status dfq_concat_q(int nbranch, const int8_t *const *xs, const int *Cs, const dfq_fmt *fs,
                        int8_t *y, dfq_fmt fy, size_t pixels, dfq_stream stream);
/* The same into a channel slice of a wider tensor: y[px * ldy + off_i + c], ldy >= sum Cs bytes between
 * pixels.  With it a join can be assembled in pieces: branches whose producing convolution already
 * writes the joined format go straight into their slice (ldy of dfq_conv_q) - the explicit downscale in
 * front of a join that Sec. 3 describes - and only the others pass through this call. */
dfq_status dfq_concat_q_into(int nbranch, const int8_t *const *xs, const int *Cs, const dfq_fmt *fs,
                             int8_t *y, int ldy, dfq_fmt fy, size_t pixels, dfq_stream stream);

/* ---- pooling (the paper names max-pool among the layers that may need an explicit
 * downscale, Sec. 3, and gives no arithmetic; average follows Eq. 10) -------------------
 * k x k windows, floor-mode output size, NHWC.
 * MAX: maximum over the window positions inside the image, then sat8(rne(., fin.frac-fout.frac)).
 * AVG: sat8 of the exact rational  (sum of in-image codes) * 2^(fout.frac-fin.frac) / (k*k)
 *      rounded once, ties to even (padded positions count as zeros in the divisor).
 * 1 <= k <= 64, 0 <= pad < k. */
dfq_status dfq_pool_q(const int8_t *x, int8_t *y, dfq_pool_mode mode, int N, int H, int W, int C,
                      int k, int stride, int pad, dfq_fmt fin, dfq_fmt fout, dfq_stream stream);

/* ---- calibration building blocks (Sec. 3: thresholds gamma = max |value| measured on one
 * batch, after the ReLU, on the wide accumulator) ----------------------------------------
 * out_dev: one DEVICE scalar, overwritten.  NaN elements are ignored.  n == 0 gives 0. */
dfq_status dfq_absmax_f32(const float *x, size_t n, float *out_dev, dfq_stream stream);
/* max |x[i]| (as uint32; relu != 0: negative entries count as 0). */
dfq_status dfq_absmax_i32(const int32_t *x, size_t n, int relu, uint32_t *out_dev, dfq_stream stream);

/* ---- preprocessing (Sec. 3: neighbouring linear operations are combined before quantizing) ----
 * Folds a per-channel affine layer z = scale[k] * y + shift[k] that follows a convolution (batch norm in its
 * inference form, a scale layer) into the convolution's FLOAT weights and bias:
 *   w_out[k][i] = w[k][i] * scale[k],   b_out[k] = b[k] * scale[k] + shift[k]
 * each product and the sum rounded to float separately.  w, w_out: [rows][row_len]; b (NULL = zeros), shift (NULL =
 * zeros), scale, b_out: [rows]; all DEVICE.  b_out may be NULL only if b and shift are.  In place (w_out == w,
 * b_out == b) is allowed; partial overlap is DFQ_EINVAL.  The folded layer is then calibrated and quantized like
 * any other; the quantized network has no scale layers left. */
dfq_status dfq_fold_scale_f32(const float *w, const float *b, size_t rows, size_t row_len, const float *scale,
                              const float *shift, float *w_out, float *b_out, dfq_stream stream);

/* Row-wise forms for weights that take one format per output channel (Sec. 3): row r of
 * x[rows][row_len] (weights: rows = K, row_len = R*S*C/groups; bias: row_len = 1).
 * dfq_absmax_f32_rows: out_dev[r] = max |x[r][.]| (NaN ignored; 0 for row_len == 0).
 * dfq_quantize_rows: q[r][i] = sat8(rne(x[r][i] * 2^frac[r])).
 * dfq_quantize_i32_rows: q[r][i] = rne(x[r][i] * 2^(frac[r] + frac_add)) saturated to
 * [-(2^31 - 1), 2^31 - 1], frac_add in [-64, 64].
 * frac, out_dev: DEVICE arrays of `rows` entries (frac entries in [-32, 32], not checked). */
dfq_status dfq_absmax_f32_rows(const float *x, size_t rows, size_t row_len, float *out_dev, dfq_stream stream);
dfq_status dfq_quantize_rows(const float *x, int8_t *q, size_t rows, size_t row_len, const int32_t *frac,
                             dfq_stream stream);
dfq_status dfq_quantize_i32_rows(const float *x, int32_t *q, size_t rows, size_t row_len, const int32_t *frac,
                                 int32_t frac_add, dfq_stream stream);

/* The same maximum separately for each of the K channels of x[pixels][K] (per-channel weight
 * formats put every channel's accumulators at a scale of their own, so the threshold of the
 * layer's output is found channel by channel).  out_dev: K DEVICE words, overwritten. */
dfq_status dfq_absmax_i32_channels(const int32_t *x, size_t pixels, int K, int relu, uint32_t *out_dev,
                                   dfq_stream stream);

/* ---- Algorithm 1 (Sec. 3): a threshold from a histogram of magnitudes instead of the maximum --
 * Readings where the algorithm is open: the tensor is a layer's int32 accumulators (after the
 * ReLU when relu != 0); hist = DFQ_HIST_BINS bins of power-of-two width over the integers |x|;
 * fpspace = the non-negative codes k / 127 of the 8-bit format; measure = sum over the bins of
 * |cdf - q| (the area between the two distribution functions); the threshold of a candidate
 * edge i is the largest integer below it, i * 2^shift - 1, capped at max|x|.
 * dfq_hist_i32: hist_dev[b] = number of elements with (|x| >> shift) == b, DFQ_HIST_BINS DEVICE
 * words, overwritten; the caller picks shift as the smallest with (max|x| >> shift) <
 * DFQ_HIST_BINS (larger magnitudes would be counted in the last bin).  n < 2^32.
 * dfq_threshold_search: host, pure, double precision, sums in bin order, fixed-size storage on the
 * stack (about 17 KB; no allocation).  hist: HOST copy of the
 * first nbins = (max_abs >> shift) + 1 words.  Candidates are the edges i = 129 .. nbins (with
 * fewer bins nothing is clipped); the first candidate with the smallest measure wins.
 * *gamma_out: the threshold in the units of x (0 for an all-zero tensor); *delta_out (may be
 * NULL): its measure.  DFQ_ESHAPE if nbins does not match max_abs and shift. */
#define DFQ_HIST_BINS 2048
/* The bin width the histogram of a tensor with this maximum takes: the smallest shift with
 * (max_abs >> shift) < DFQ_HIST_BINS.  Host, pure; -1 for a negative max_abs. */
int dfq_hist_shift(int64_t max_abs);
dfq_status dfq_hist_i32(const int32_t *x, size_t n, int relu, int shift, uint32_t *hist_dev, dfq_stream stream);
dfq_status dfq_threshold_search(const uint32_t *hist, int nbins, int shift, int64_t max_abs, int64_t *gamma_out,
                                double *delta_out);

/* gamma = alpha * beta_max (Sec. 2.1) solved for a power-of-two alpha: the largest frac in
 * [-32, 32] with gamma * 2^frac <= 127; gamma = 0 gives 32.  Host, pure.  DFQ_EINVAL for a
 * negative, infinite or NaN gamma. */
dfq_status dfq_fmt_from_absmax_f32(float gamma, dfq_fmt *out);
/* Integer form for accumulators held at acc_frac: the largest frac <= acc_frac (rescale factor
 * in (0, 1], Sec. 3) with m * 2^(frac - acc_frac) <= 127, floored at -32.  Host, pure. */
dfq_status dfq_fmt_from_absmax_i32(int64_t m, int32_t acc_frac, dfq_fmt *out);
/* The output format of a layer whose weights have one format per output channel (Sec. 3): channel k's
 * accumulators are at frac_in + frac_w[k], and the layer's int8 output gets the finest format that holds
 * every channel's threshold m[k] with a rescale factor in (0, 1] - the smallest of the per-channel results
 * of dfq_fmt_from_absmax_i32(m[k], frac_in + frac_w[k]).  m (as dfq_absmax_i32_channels leaves it, copied
 * to the host) and frac_w: HOST arrays of K entries.  Host, pure.  DFQ_EFMT for an entry of frac_w outside
 * [-32, 32]. */
dfq_status dfq_fmt_from_absmax_i32_channels(const uint32_t *m, int K, int32_t frac_in, const int32_t *frac_w,
                                            dfq_fmt *out);

/* ---- multiply-accumulate on (8, p) codes with p >= 4 (Sec. 2.2, Eq. 6-9) --------------------------------------
 * Eq. 6 on the integers beta of Eq. 2 (|beta| <= beta_max(8, 4) = 1984 for p = 4; Sec. 5 reports p = 4 and p = 3 as the
 * most accurate 8-bit members): acc = bias[k] + sum over the kernel window and the group's input channels of
 * beta_x * beta_w, exact (Eq. 8: up to 36 bits for 3 x 3 x 512 terms; the kernels carry 64); ReLU if asked;
 * beta_y = acc * 2^-(frac_x + frac_w - frac_y) rounded once to the nearest integer representable in (8, p_y), ties to
 * the even significand field, saturated at +-beta_max(8, p_y).
 * On this path a tensor is held as two int8 DIGIT PLANES of its integers, beta = 64 * hi + lo with hi and lo of the
 * sign of beta (|hi| <= 31, |lo| <= 63), same shape and layout as the tensor (NHWC, [K][R][S][C/groups]).  The
 * matrix-core kernel multiplies the planes as int8 matrices (four products per block) and recombines them exactly.
 * dfq_np_digits: codes of (8, p), 4 <= p <= 7 (DFQ_EFMT otherwise), to planes.  n bytes each, DEVICE, no overlap.
 * dfq_conv_np: xh, xl: input planes; wh, wl: weight planes; b: int32 bias at frac_x + frac_w or NULL;
 *   y: output codes (Eq. 2 sign-and-magnitude bytes, the code of -0 never written) or NULL; yh, yl: output planes,
 *   both or neither NULL; at least one output.  frac_* in [-32, 32], frac_x + frac_w - frac_y in [-16, 48], p_y in
 *   [4, 7]: DFQ_EFMT otherwise.  Geometry and status codes as dfq_conv_q.  Outputs must not overlap inputs or each other.
 *   N == 0 is a no-op.
 * dfq_conv_np_variant: DFQ_CONV_MFMA (groups == 1, C % 64 == 0, K % 16 == 0, R*S*C <= 13000, all pointers 16-byte
 *   aligned; DFQ_EUNSUPPORTED otherwise) or DFQ_CONV_DIRECT (any geometry); DFQ_CONV_AUTO picks MFMA when it applies. */
/* Element-wise add on (8, p >= 4) codes held as digit planes (Eq. 10 with power-of-two scales): the two integers are
 * brought to the finer of the two scales by exact left shifts, summed without loss (Eq. 12: the shifts may be at most 18
 * bits, DFQ_EFMT otherwise), ReLU acts on the sum if asked, and the sum times 2^-(max(frac_a, frac_b) - frac_y) is
 * rounded once into the format (8, p_y): nearest representable integer, ties to the even significand field, saturated.
 * ah, al, bh, bl: input planes, n bytes each; y: output codes or NULL; yh, yl: output planes, both or neither NULL; at
 * least one output; no output may overlap an input or another output.  All DEVICE.  The final factor's exponent must lie
 * in [-16, 31] and p_y in [4, 7] (DFQ_EFMT).  n == 0 is a no-op. */
dfq_status dfq_eltwise_np(const int8_t *ah, const int8_t *al, int frac_a, const int8_t *bh, const int8_t *bl, int frac_b, uint8_t *y,
                          int8_t *yh, int8_t *yl, int frac_y, int p_y, size_t n, int relu, dfq_stream stream);

/* Join fusion on (8, p >= 4) codes (Sec. 3: the add that follows a layer is taken where the layer's result is produced):
 * the bytes dfq_conv_np (output scale frac_mid, ReLU relu_mid, format (8, p)) followed by dfq_eltwise_np (that result and
 * the tensor oh/ol at frac_other, output at frac_y in (8, p), ReLU relu_out on the sum) would leave in yh/yl - both
 * conversions are carried out, the layer's own result is never stored.  oh, ol: [N,P,Q,K] digit planes, 16-byte aligned,
 * must not overlap the outputs.  Matrix-core form only: DFQ_EUNSUPPORTED where dfq_conv_np_variant(DFQ_CONV_MFMA) is, for
 * frac_x + frac_w - frac_mid outside [7, 36] and for max(frac_mid, frac_other) - frac_y outside [0, 31]; the caller then
 * issues the two calls.  All DEVICE. */
dfq_status dfq_conv_np_add(const int8_t *xh, const int8_t *xl, const int8_t *wh, const int8_t *wl, const int32_t *b, const int8_t *oh,
                           const int8_t *ol, int8_t *yh, int8_t *yl, int N, int H, int W, int C, int K, int R, int S, int stride, int pad,
                           int groups, int frac_x, int frac_w, int frac_mid, int relu_mid, int frac_other, int frac_y, int p, int relu_out,
                           dfq_stream stream);

/* Calibration of a layer on (8, p >= 4) codes (Sec. 3: the output threshold is taken on the exact accumulator, after the
 * ReLU where the layer has one, before anything is rounded): the largest |sum + bias| of Eq. 6 over all outputs of the
 * layer (negative sums count as 0 when relu is set), as a 64-bit integer at the scale 2^-(frac_x + frac_w), written to
 * *amax_dev (DEVICE, 8-byte aligned; cleared by the call on the stream, then raised by atomic maxima).  Operands as for
 * dfq_conv_np; nothing else is written.  One output per lane (a calibration batch is small). */
dfq_status dfq_conv_np_absmax(const int8_t *xh, const int8_t *xl, const int8_t *wh, const int8_t *wl, const int32_t *b, uint64_t *amax_dev,
                              int N, int H, int W, int C, int K, int R, int S, int stride, int pad, int groups, int relu, dfq_stream stream);

/* The same for the add of Eq. 10: the largest magnitude of the exact sum at the finer input scale 2^-max(frac_a, frac_b). */
dfq_status dfq_eltwise_np_absmax(const int8_t *ah, const int8_t *al, int frac_a, const int8_t *bh, const int8_t *bl, int frac_b,
                                 uint64_t *amax_dev, size_t n, int relu, dfq_stream stream);

/* HOST.  The scale of a tensor whose largest magnitude is max_abs * 2^-acc_frac: the largest frac <= min(acc_frac, 32) with
 * max_abs * 2^(frac - acc_frac) <= beta_max(nbits, p), floored at -32 (gamma = alpha * beta_max, Sec. 2.1, towards the
 * coarser power of two so that nothing clips; the rescale factor stays in (0, 1] as for dfq_fmt_from_absmax_i32). */
dfq_status dfq_np_frac_from_absmax_u64(uint64_t max_abs, int acc_frac, int nbits, int p, int *frac);

/* Pooling on (8, p_fmt >= 4) digit planes, NHWC, k x k windows, floor-mode output size; the result keeps the input's
 * scale.  MAX: the largest value among the window's taps inside the image (0 <= pad < k).  AVG: the exact mean of the
 * k * k integers rounded once to the format (nearest, ties to the even significand); pad must be 0
 * (DFQ_EUNSUPPORTED otherwise).  Outputs as for dfq_eltwise_np.  k <= 16.  All DEVICE. */
dfq_status dfq_pool_np(const int8_t *xh, const int8_t *xl, uint8_t *y, int8_t *yh, int8_t *yl, dfq_pool_mode mode, int N, int H, int W, int C,
                       int k, int stride, int pad, int p_fmt, dfq_stream stream);

/* Layout helpers for a first layer with few channels (data movement only; each acts on one byte tensor, so a tensor held
 * as two digit planes takes two calls, and int8 codes work the same way).  A stride-2 convolution with an R x S kernel
 * (R, S <= 8) over C <= 4 channels, padding pad, equals a 4 x 1 convolution with unit stride and no padding over 64
 * channels of the packed tensor  y[N][P + 3][Q][64],  y[n][i][q][16 s + (2 dy + dx) C + c] = x_padded[n][2 i + dy][2 (q + s) + dx][c]
 * (s = 0..3, zeros elsewhere), P x Q the layer's output size, with the weights packed alike:
 * y[K][4][1][64],  y[k][r][0][16 s + (2 dy + dx) C + c] = w[k][2 r + dy][2 s + dx][c] where that tap exists, else 0.
 * The sums are the same integers term by term (zero taps add nothing).  y 16-byte aligned; no overlap.  All DEVICE. */
dfq_status dfq_stem_pack_x(const int8_t *x, int8_t *y, int N, int H, int W, int C, int R, int S, int pad, dfq_stream stream);
dfq_status dfq_stem_pack_w(const int8_t *w, int8_t *y, int K, int R, int S, int C, dfq_stream stream);

/* gamma = alpha * beta_max (Sec. 2.1) solved for a power-of-two alpha in the general family: the largest frac in
 * [-32, 32] with gamma * 2^frac <= beta_max(nbits, p); gamma = 0 gives 32.  Host, pure.  DFQ_EINVAL for a negative,
 * infinite or NaN gamma, DFQ_EFMT for a format dfq_quantize_np does not take. */
dfq_status dfq_np_frac_from_absmax_f32(float gamma, int nbits, int p, int32_t *frac_out);
dfq_status dfq_np_digits(const uint8_t *codes, size_t n, int p, int8_t *hi, int8_t *lo, dfq_stream stream);
dfq_status dfq_conv_np(const int8_t *xh, const int8_t *xl, const int8_t *wh, const int8_t *wl, const int32_t *b, uint8_t *y,
                       int8_t *yh, int8_t *yl, int N, int H, int W, int C, int K, int R, int S, int stride, int pad, int groups,
                       int frac_x, int frac_w, int frac_y, int p_y, int relu, dfq_stream stream);
dfq_status dfq_conv_np_variant(dfq_conv_variant variant, const int8_t *xh, const int8_t *xl, const int8_t *wh, const int8_t *wl,
                               const int32_t *b, uint8_t *y, int8_t *yh, int8_t *yl, int N, int H, int W, int C, int K, int R, int S,
                               int stride, int pad, int groups, int frac_x, int frac_w, int frac_y, int p_y, int relu,
                               dfq_stream stream);

/* ---- closed forms of Sec. 2 (host, pure; return -1 on invalid arguments) ----------------- */
int64_t dfq_beta_max(int n, int p);                                        /* Eq. 5, equality case */
int     dfq_mac_acc_bits(int64_t N, int64_t bx, int64_t ex, int64_t by, int64_t ey);   /* Eq. 8 */
int64_t dfq_mac_max_len(int q, int64_t bx, int64_t ex, int64_t by, int64_t ey);        /* Eq. 9 */
int     dfq_add_acc_bits(int64_t N, int64_t bx, int64_t ex);                            /* Eq. 12 */
int64_t dfq_add_max_len(int q, int64_t bx, int64_t ex);                                 /* Eq. 13 */

#ifdef __cplusplus
}
#endif
#endif /* DFQ_H */
