// Depthwise quantized convolution (groups == C == K): every output channel sums R*S products
// of its own input channel (Eq. 6 with N = R*S), so there is no contraction over channels
// and nothing for the matrix cores to do; the layer moves about as many bytes as it performs
// multiply-accumulates and is bound by HBM and by plain integer ALU work.
//
// A lane owns 4 consecutive channels (one 32-bit word of an NHWC pixel) and TW consecutive
// output pixels of one output row; consecutive lanes take consecutive channel words, so every
// load and store of a wavefront covers whole pixels contiguously.  Each input word is loaded
// once per lane and reused for every tap and output pixel it feeds; weights sit in LDS
// transposed to [tap][channel] so that one word read gives the 4 channels' weights of a tap.
// The 32-bit sums stay in registers through bias, ReLU, rounding shift and clamp.
#include "conv_epilogue.hpp"

namespace dfq {

namespace {

constexpr int kThreads = 256;

struct DwParams {
    ConvArgs a;
    int cw;            // C / 4
    int qblocks;       // ceil(Q / TW)
    long long items;   // N * P * qblocks * cw
};

template <int R, int S, int ST, int TW>
__global__ void __launch_bounds__(kThreads) conv_depthwise_kernel(DwParams prm)
{
    constexpr int IW = (TW - 1) * ST + S;   // input columns one lane touches per kernel row
    extern __shared__ uint32_t wt[];        // [R*S][C/4] words: weights of 4 channels for one tap

    const ConvArgs &a = prm.a;
    // transpose w[c][tap] -> wt[tap][c]
    {
        int8_t *wb = (int8_t *)wt;
        const int total = R * S * a.C;
        for (int i = threadIdx.x; i < total; i += kThreads) {
            int c = i / (R * S), tap = i - c * (R * S);
            wb[tap * a.C + c] = a.w[i];
        }
    }
    __syncthreads();

    Requant rq;
    rq.init(a.shift, a.relu);

    for (long long it = (long long)blockIdx.x * kThreads + threadIdx.x; it < prm.items; it += (long long)gridDim.x * kThreads) {
        const int cwi = (int)(it % prm.cw);
        long long t = it / prm.cw;
        const int qb = (int)(t % prm.qblocks);
        t /= prm.qblocks;
        const int p = (int)(t % a.P);
        const int n = (int)(t / a.P);
        const int c = cwi * 4;
        const int q0 = qb * TW;
        const int iw_first = q0 * ST - a.pad;

        int acc[TW][4];
        {
            int4 bv = make_int4(0, 0, 0, 0);
            if (a.b) bv = *(const int4 *)(a.b + c);
#pragma unroll
            for (int j = 0; j < TW; j++) { acc[j][0] = bv.x; acc[j][1] = bv.y; acc[j][2] = bv.z; acc[j][3] = bv.w; }
        }
        const int8_t *img = a.x + (size_t)n * a.H * a.W * a.C + c;
#pragma unroll
        for (int r = 0; r < R; r++) {
            const int ih = p * ST - a.pad + r;
            if ((unsigned)ih >= (unsigned)a.H) continue;
            const int8_t *row = img + (size_t)ih * a.W * a.C;
            int xv[IW][4];
#pragma unroll
            for (int j = 0; j < IW; j++) {
                const int iw = iw_first + j;
                uint32_t w32 = 0;
                if ((unsigned)iw < (unsigned)a.W) w32 = *(const uint32_t *)(row + (size_t)iw * a.C);
#pragma unroll
                for (int e = 0; e < 4; e++) xv[j][e] = byte_of(w32, e);
            }
#pragma unroll
            for (int s = 0; s < S; s++) {
                const uint32_t ww = wt[(r * S + s) * prm.cw + cwi];
                int wv[4];
#pragma unroll
                for (int e = 0; e < 4; e++) wv[e] = byte_of(ww, e);
#pragma unroll
                for (int j = 0; j < TW; j++)
#pragma unroll
                    for (int e = 0; e < 4; e++) acc[j][e] += xv[j * ST + s][e] * wv[e];
            }
        }
        const size_t pix0 = ((size_t)n * a.P + p) * a.Q + q0;
        int sh[4] = {a.shift, a.shift, a.shift, a.shift};   // one weight format per channel: each its own shift
        if (a.frac_w) {
#pragma unroll
            for (int e = 0; e < 4; e++) sh[e] += a.frac_w[c + e];
        }
#pragma unroll
        for (int j = 0; j < TW; j++) {
            if (q0 + j >= a.Q) break;
            if (a.acc_out) *(int4 *)(a.acc_out + (pix0 + j) * a.K + c) = make_int4(acc[j][0], acc[j][1], acc[j][2], acc[j][3]);
            if (a.y) {
                int o[4];
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    if (a.frac_w) o[e] = requant8(a.relu ? max(acc[j][e], 0) : acc[j][e], sh[e]);
                    else o[e] = rq.fast ? rq.fast_one(acc[j][e]) : rq.slow_one(acc[j][e]);
                }
                *(uint32_t *)(a.y + (pix0 + j) * (size_t)a.ldy + c) = pack4_clamped(o[0], o[1], o[2], o[3]);
            }
        }
    }
}

template <int R, int S, int ST, int TW>
hipError_t launch_dw(const ConvArgs &a, hipStream_t st)
{
    DwParams prm;
    prm.a = a;
    prm.cw = a.C / 4;
    prm.qblocks = (a.Q + TW - 1) / TW;
    prm.items = (long long)a.N * a.P * prm.qblocks * prm.cw;
    long long blocks = (prm.items + kThreads - 1) / kThreads;
    if (blocks > 256 * 16) blocks = 256 * 16;
    if (blocks < 1) blocks = 1;
    size_t lds = (size_t)R * S * a.C;
    conv_depthwise_kernel<R, S, ST, TW><<<(unsigned)blocks, kThreads, lds, st>>>(prm);
    return hipGetLastError();
}

}  // namespace

bool conv_depthwise_supports(const ConvArgs &a)
{
    if (a.groups != a.C || a.K != a.C) return false;
    if (a.C % 4) return false;
    if (a.R != 3 || a.S != 3 || (a.stride != 1 && a.stride != 2)) return false;
    if (a.C * 9 > 48 * 1024) return false;
    if (((uintptr_t)a.x & 3) || (a.y && (((uintptr_t)a.y & 3) || (a.ldy & 3)))) return false;
    if (a.b && ((uintptr_t)a.b & 15)) return false;
    if (a.acc_out && ((uintptr_t)a.acc_out & 15)) return false;
    return true;
}

hipError_t launch_conv_depthwise(const ConvArgs &a, hipStream_t st)
{
    if (a.stride == 1) return launch_dw<3, 3, 1, 4>(a, st);
    return launch_dw<3, 3, 2, 2>(a, st);
}

}  // namespace dfq
