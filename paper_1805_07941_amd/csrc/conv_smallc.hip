// Convolution with few input channels (the first layer of a network: C = 3) on the int8
// matrix cores.
//
// With NHWC and a small C, the S taps of one kernel row r are S*C CONTIGUOUS bytes of the
// input row (channels of pixel iw0, then of iw0+1, ...).  When S*C <= 32 that run is used as
// one 32-byte block of the reduction axis of Eq. 6: the block for (output pixel, r) is simply
// the 32 bytes starting at x[n, ih, iw0, 0]; the weight block for (k, r) is w[k, r, :, :]
// followed by zeros, so whatever the input bytes beyond S*C hold is multiplied by 0.  The
// reduction is then R blocks long (7 for a 7x7 kernel) instead of R*S*C padded tap by tap.
//
// The pixel operand is read straight from global memory in matrix-operand layout (each lane
// one unaligned 16-byte load per block; neighbouring output pixels overlap heavily, so these
// hit in L1/L2); only the small packed weight tensor lives in LDS, loaded once per workgroup,
// which then walks over pixel tiles (persistent grid).  A run that crosses the left or right
// image border is read from the nearest 16 bytes inside the row and shifted into place, which
// both zero-fills the padding and keeps every access inside the tensor.
#include "conv_epilogue.hpp"

namespace dfq {

namespace {

constexpr int kThreads = 256;
constexpr int kTilePixels = 256;   // 4 wavefronts x 64 pixels

struct SmallCParams {
    ConvArgs a;
    int M;              // N*P*Q  (< 2^31)
    int tiles_p;
    int run;            // S*C, bytes of one kernel row
    int rowlen;         // W*C
    FastDiv div_pq, div_q;
};

template <int CT>   // channel tile = CT * 32
__global__ void __launch_bounds__(kThreads, 2) conv_smallc_kernel(SmallCParams prm)
{
    constexpr int BC = CT * 32;
    extern __shared__ uint4 wlds[];   // [R][BC][2] 16-byte pieces, piece index XOR-ed with bit 3 of k

    const ConvArgs &a = prm.a;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, lh = lane >> 5;
    const int k0 = blockIdx.y * BC;

    // ---- packed weights into LDS: block (r, k) = w[k][r][0 .. run) then zeros
    {
        int8_t *wb = (int8_t *)wlds;
        const int total = a.R * BC * 32;
        for (int i = tid; i < total; i += kThreads) {
            int j = i & 31;
            int kl = (i >> 5) % BC;
            int r = (i >> 5) / BC;
            int k = k0 + kl;
            int8_t v = 0;
            if (j < prm.run && k < a.K) v = a.w[((size_t)k * a.R + r) * prm.run + j];
            // LDS row of channel kl follows the same permutation as the dense kernel: a lane's
            // 16 accumulators are 16 consecutive channels
            int c32 = kl & 31;
            int row = (kl & ~31) + 8 * ((c32 & 15) >> 2) + 4 * (c32 >> 4) + (c32 & 3);
            int piece = (j >> 4) ^ ((row >> 3) & 1);
            wb[((r * BC + row) * 2 + piece) * 16 + (j & 15)] = v;
        }
    }
    __syncthreads();

    Requant rq;
    rq.init(a.shift, a.relu);
    const bool fast = epilogue_is_fast(a, rq, k0 + BC);
    const v4i *wl = (const v4i *)wlds;

    int bias[CT][16];
#pragma unroll
    for (int c = 0; c < CT; c++) load_bias16(a, k0 + c * 32 + 16 * lh, bias[c]);

    for (int tile = blockIdx.x; tile < prm.tiles_p; tile += gridDim.x) {
        const int mbase = tile * kTilePixels + wave * 64;
        const int8_t *rowptr[2];   // address of the lane's 16 bytes in kernel row r = 0
        int ih0[2], rb[2];         // first input row; byte offset of the run inside its row (may be < 0)
        bool any_border[2];
#pragma unroll
        for (int p = 0; p < 2; p++) {
            int m = mbase + p * 32 + l32;
            if (m >= prm.M) m = prm.M - 1;              // duplicate work for the ragged tail, never stored
            int n = fastdiv(m, prm.div_pq);
            int pq = m - n * (a.P * a.Q);
            int pp = fastdiv(pq, prm.div_q);
            int q = pq - pp * a.Q;
            ih0[p] = pp * a.stride - a.pad;
            rb[p] = (q * a.stride - a.pad) * a.C;
            rowptr[p] = a.x + ((long long)n * a.H + ih0[p]) * prm.rowlen + rb[p] + 16 * lh;
            any_border[p] = __any(rb[p] < 0 || rb[p] + 32 > prm.rowlen);   // uniform over the 32-pixel tile pair of lanes
        }

        v16i acc[CT][2];
#pragma unroll
        for (int c = 0; c < CT; c++)
#pragma unroll
            for (int p = 0; p < 2; p++)
#pragma unroll
                for (int r = 0; r < 16; r++) acc[c][p][r] = bias[c][r];

        for (int r = 0; r < a.R; r++) {
            v4i xf[2];
#pragma unroll
            for (int p = 0; p < 2; p++) {
                const int ih = ih0[p] + r;
                const bool row_ok = (unsigned)ih < (unsigned)a.H;
                const int8_t *src = rowptr[p] + (long long)r * prm.rowlen;
                v4i v = {0, 0, 0, 0};
                if (!any_border[p]) {
                    if (row_ok) __builtin_memcpy(&v, src, 16);
                } else if (row_ok) {
                    // piece covers row bytes [o, o+16); bytes outside [0, rowlen) are padding.  The
                    // 16 bytes are read from the nearest position that lies wholly inside the row
                    // and shifted into place, which zero-fills the padding.
                    const int o = rb[p] + 16 * lh;
                    const int oc = min(max(o, 0), prm.rowlen - 16);
                    unsigned __int128 t;
                    __builtin_memcpy(&t, src - o + oc, 16);
                    const int sh = o - oc;          // > 0: piece starts right of what was read
                    if (sh >= 16 || sh <= -16) t = 0;
                    else if (sh > 0) t >>= 8 * sh;
                    else if (sh < 0) t <<= 8 * (-sh);
                    __builtin_memcpy(&v, &t, 16);
                }
                xf[p] = v;
            }
#pragma unroll
            for (int c = 0; c < CT; c++) {
                const int row = c * 32 + l32;
                const v4i wf = wl[(r * BC + row) * 2 + (lh ^ ((row >> 3) & 1))];
#pragma unroll
                for (int p = 0; p < 2; p++)
                    acc[c][p] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf, xf[p], acc[c][p], 0, 0, 0);
            }
        }

#pragma unroll
        for (int c = 0; c < CT; c++) {
            const int kc = k0 + c * 32 + 16 * lh;
#pragma unroll
            for (int p = 0; p < 2; p++) {
                const int m = mbase + p * 32 + l32;
                if (m < prm.M) {
                    if (fast) store_tile_lane_fast(acc[c][p], a, rq, m, kc);
                    else if (kc < a.K) store_tile_lane_general(acc[c][p], a, a.shift, a.relu, m, kc);
                }
            }
        }
    }
}

}  // namespace

bool conv_smallc_supports(const ConvArgs &a)
{
    if (a.groups != 1) return false;
    if (a.S * a.C > 32) return false;
    if (a.W * a.C < 32) return false;                       // clamped border loads need a row of >= 16 bytes
    if ((long long)a.N * a.P * a.Q >= (1LL << 31) - 512) return false;
    if (a.acc_out && ((uintptr_t)a.acc_out & 15)) return false;
    return true;
}

hipError_t launch_conv_smallc(const ConvArgs &a, hipStream_t st)
{
    SmallCParams prm;
    prm.a = a;
    prm.M = (int)((long long)a.N * a.P * a.Q);
    prm.tiles_p = (prm.M + kTilePixels - 1) / kTilePixels;
    prm.run = a.S * a.C;
    prm.rowlen = a.W * a.C;
    prm.div_pq = make_fastdiv(a.P * a.Q);
    prm.div_q = make_fastdiv(a.Q);
    const bool wide = a.K > 32;
    const int BC = wide ? 64 : 32;
    dim3 grid((unsigned)min(prm.tiles_p, 256 * 4), (unsigned)((a.K + BC - 1) / BC));
    size_t lds = (size_t)a.R * BC * 32;
    if (lds > 64 * 1024) return hipErrorInvalidValue;
    if (wide) conv_smallc_kernel<2><<<grid, kThreads, lds, st>>>(prm);
    else conv_smallc_kernel<1><<<grid, kThreads, lds, st>>>(prm);
    return hipGetLastError();
}

}  // namespace dfq
