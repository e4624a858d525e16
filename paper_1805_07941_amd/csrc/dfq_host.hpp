// Host-side declarations shared by the translation units of libdfq: one launcher per
// kernel family.  Launchers assume validated arguments and only enqueue work.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace dfq {

// Geometry and formats of one convolution call (Eq. 6), after validation.
struct ConvArgs {
    const int8_t *x;
    const int8_t *w;
    const int32_t *b;    // may be null
    int8_t *y;           // may be null when acc_out is set
    int32_t *acc_out;    // may be null
    int N, H, W, C, K, R, S, stride, pad, groups;
    int P, Q;            // output extent
    int ldy;             // bytes between consecutive output pixels of y
    int shift;           // f_in + f_w - f_out
    int relu;
    // Fused element-wise add (Eq. 10) behind the convolution, or add == null: the convolution's
    // own int8 result (format f_out, `shift` and `relu` above) and the int8 tensor `add` of the
    // same pixels and channels are brought to their finer scale by left shifts, summed, and the
    // sum is rounded once by add_shift into what is stored in y.
    const int8_t *add = nullptr;
    int ldadd = 0;               // bytes between consecutive pixels of `add`
    int add_sa = 0, add_sb = 0;  // left shifts of the convolution result and of `add`
    int add_shift = 0;           // finer scale's fractional length minus that of y
    int add_relu = 0;
    // Single-rounding form: the accumulator itself (no format of its own; `shift` and `relu` are not used) plus
    // `add` << add_sb, rounded once by add_shift = f_in + f_w - f_out; add_sa is 0.
    int add_lazy = 0;
    // One weight format per output channel (Sec. 3), or frac_w == null: a device array of K
    // fractional lengths; `shift` then holds f_in - f_out and channel k is rescaled by a rounding
    // shift of shift + frac_w[k] (its bias is at f_in + frac_w[k]).  The host cannot read the array:
    // kernels that need every shift in a certain range are chosen from the declared bounds.
    const int32_t *frac_w = nullptr;
    int frac_w_lo = 0, frac_w_hi = 0;   // bounds the caller guarantees for the entries of frac_w
};

// One convolution on 8-bit dynamic floating-point codes with p >= 4 significand bits (Eq. 6 on integers of up to
// twelve bits), operands and results as base-64 digit planes: beta = 64 * h + l, h and l of the sign of beta.
struct NpConvArgs {
    const int8_t *xh, *xl;         // input digit planes, NHWC
    const int8_t *wh, *wl;         // weight digit planes, [K][R][S][C/groups]
    const int32_t *b;              // bias at f_x + f_w, may be null
    uint8_t *y;                    // output codes (Eq. 2), may be null
    int8_t *yh, *yl;               // output digit planes, may be null
    int N, H, W, C, K, R, S, stride, pad, groups;
    int P, Q;
    int shift;                     // f_x + f_w - f_y
    int p_y;                       // significand bits of the output format (8, p_y)
    int beta_max;                  // Eq. 5 for the output format
    int relu;
    // fused join (matrix-core form only): the layer's own result, rounded to (8, p_y) at frac_mid, is added to a second
    // tensor as dfq_eltwise_np would add them, and only the sum is stored
    const int8_t *oh, *ol;         // the other operand's digit planes [N,P,Q,K], null: no join
    int add_sa, add_sb;            // left shifts of the layer's result and of the other operand to the finer scale
    int add_shift;                 // that scale's fractional length minus the output's, 0..31
    int add_relu;                  // ReLU on the sum
    unsigned long long *amax;      // calibration: receives max |sum + bias| (after ReLU if relu) by atomic max; direct form only
};

hipError_t launch_quantize(const float *x, int8_t *q, size_t n, int frac, hipStream_t st);
hipError_t launch_quantize_i32(const float *x, int32_t *q, size_t n, int frac, hipStream_t st);
hipError_t launch_dequantize(const int8_t *q, float *x, size_t n, int frac, hipStream_t st);
hipError_t launch_quantize_np(const float *x, uint8_t *q, size_t n, int nbits, int p, int frac, hipStream_t st);
hipError_t launch_dequantize_np(const uint8_t *q, float *x, size_t n, int nbits, int p, int frac, hipStream_t st);
hipError_t launch_eltwise(const int8_t *a, int fa, const int8_t *b, int fb, int8_t *y, int fy, int32_t *acc, size_t n,
                          int relu, hipStream_t st);
hipError_t launch_concat(int nb, const int8_t *const *xs, const int *Cs, const int *fs, int8_t *y, int ldy, int fy,
                         size_t pixels, hipStream_t st);
hipError_t launch_pool(const int8_t *x, int8_t *y, int mode, int N, int H, int W, int C, int P, int Q, int k, int stride,
                       int pad, int fin, int fout, hipStream_t st);
hipError_t launch_absmax_f32(const float *x, size_t n, float *out, hipStream_t st);
hipError_t launch_absmax_i32(const int32_t *x, size_t n, int relu, uint32_t *out, hipStream_t st);
hipError_t launch_quantize_rows(const float *x, int8_t *q, size_t rows, size_t row_len, const int32_t *frac, hipStream_t st);
hipError_t launch_quantize_i32_rows(const float *x, int32_t *q, size_t rows, size_t row_len, const int32_t *frac, int frac_add,
                                    hipStream_t st);
hipError_t launch_fold_scale(const float *w, const float *b, size_t rows, size_t row_len, const float *scale, const float *shift,
                             float *w_out, float *b_out, hipStream_t st);
hipError_t launch_absmax_f32_rows(const float *x, size_t rows, size_t row_len, float *out, hipStream_t st);
hipError_t launch_hist_i32(const int32_t *x, size_t n, int relu, int shift, uint32_t *out, hipStream_t st);
hipError_t launch_absmax_i32_channels(const int32_t *x, size_t pixels, int K, int relu, uint32_t *out, hipStream_t st);

bool conv_direct_supports(const ConvArgs &a);
hipError_t launch_conv_direct(const ConvArgs &a, hipStream_t st);
bool conv_mfma_supports(const ConvArgs &a);
bool conv_mfma_fuses(const ConvArgs &a);     // a.add set: the dense kernel has a fused form for this call
hipError_t launch_conv_mfma(const ConvArgs &a, hipStream_t st);
bool conv_fc_supports(const ConvArgs &a);       // unpadded 1x1 layers over at most 1024 pixels: one wavefront per 32 x 32 tile
hipError_t launch_conv_fc(const ConvArgs &a, hipStream_t st);
bool conv_depthwise_supports(const ConvArgs &a);
hipError_t launch_conv_depthwise(const ConvArgs &a, hipStream_t st);
bool conv_dwm_supports(const ConvArgs &a);      // depthwise layers the matrix-core form takes
hipError_t launch_conv_dwm(const ConvArgs &a, hipStream_t st);
bool conv_pw_geometry_ok(const ConvArgs &a);
bool conv_pw_supports(const ConvArgs &a);
hipError_t launch_conv_pw(const ConvArgs &a, hipStream_t st);
bool conv_grouped_supports(const ConvArgs &a);
hipError_t launch_conv_grouped(const ConvArgs &a, hipStream_t st);
bool conv_sg_supports(const ConvArgs &a);       // grouped layers the matrix-core form (blocks of 64 channels) takes
hipError_t launch_conv_sg(const ConvArgs &a, hipStream_t st);
bool conv_np_mfma_supports(const NpConvArgs &a);
hipError_t launch_conv_np_mfma(const NpConvArgs &a, hipStream_t st);
hipError_t launch_conv_np_direct(const NpConvArgs &a, hipStream_t st);
hipError_t launch_clear_u64(unsigned long long *p, hipStream_t st);
hipError_t launch_eltwise_np_absmax(const int8_t *ah, const int8_t *al, const int8_t *bh, const int8_t *bl, size_t n, int sa, int sb, int relu,
                                    unsigned long long *amax, hipStream_t st);
hipError_t launch_pool_np(const int8_t *xh, const int8_t *xl, uint8_t *y, int8_t *yh, int8_t *yl, int avg, int N, int H, int W, int C, int k,
                          int stride, int pad, int P, int Q, int p_fmt, int beta_max, hipStream_t st);
hipError_t launch_stem_pack_x(const int8_t *x, int8_t *y, int N, int H, int W, int C, int pad, int Hs, int Qs, hipStream_t st);
hipError_t launch_stem_pack_w(const int8_t *w, int8_t *y, int K, int R, int S, int C, hipStream_t st);
hipError_t launch_eltwise_np(const int8_t *ah, const int8_t *al, const int8_t *bh, const int8_t *bl, uint8_t *y, int8_t *yh, int8_t *yl,
                             size_t n, int sa, int sb, int shift, int p_y, int beta_max, int relu, hipStream_t st);
hipError_t launch_np_digits(const uint8_t *codes, size_t n, int p, int8_t *hi, int8_t *lo, hipStream_t st);
bool conv_smallc_supports(const ConvArgs &a);
hipError_t launch_conv_smallc(const ConvArgs &a, hipStream_t st);
bool conv_stem_supports(const ConvArgs &a, bool pool, bool from_float = false);   // first layers (3 channels, stride 2) the strip kernel takes; pool: with the 3x3/2 max-pool behind it
// y_pooled == null: the layer alone, into a.y.  x_float != null (with y_pooled): float images converted to codes at frac_in on the way in.
hipError_t launch_conv_stem(const ConvArgs &a, int8_t *y_pooled, int ld_pooled, hipStream_t st, const float *x_float = nullptr,
                            int frac_in = 0);

}  // namespace dfq
