// Depthwise quantized convolution (groups == C == K): every output channel sums R*S products
// of its own input channel (Eq. 6 with N = R*S), so there is no contraction over channels
// and nothing for the matrix cores to do; the layer moves about as many bytes as it performs
// multiply-accumulates and is bound by HBM and by plain integer ALU work.
//
// A lane owns 4 consecutive channels (one 32-bit word of an NHWC pixel) and TW consecutive
// output pixels of one output row; consecutive lanes take consecutive channel words, so every
// load and store of a wavefront covers whole pixels contiguously.  All input words of an item
// (R rows x IW columns) are fetched up front by range-checked buffer loads - positions in the
// padding get an out-of-range offset and arrive as zeros, so there is no branch between the
// loads and they are all in flight together.  The words of four neighbouring columns are then
// transposed in registers (byte permutes) into one word per channel holding that channel's
// four neighbouring pixels; an output's three taps of a kernel row are a byte-aligned window of
// two such words, and one v_dot4_i32_i8 with the row's three weights (fourth factor zero)
// accumulates them.  Weights sit in LDS as one such word per (kernel row, channel).  The 32-bit
// sums stay in registers through bias, ReLU, rounding shift and clamp.
#include "conv_epilogue.hpp"

namespace dfq {

namespace {

constexpr int kThreads = 256;

struct DwParams {
    ConvArgs a;
    int cw;            // C / 4
    int qblocks;       // ceil(Q / TW)
    int items;         // N * P * qblocks * cw (below 2^31)
    unsigned x_bytes;  // size of the input (below 2^31: larger offsets mean "outside")
    FastDiv div_cw, div_qb, div_p;
};

// OWN: the grid's stride over the items is a multiple of C / 4, so a lane meets the same four channels in every item:
// it fetches their 36 weight bytes itself (nine words) and keeps the row words in registers - no gather of all
// channels' weights into LDS in front of a block's first item, which for layers of few pixels and many channels
// (7 x 7 x 1024) took as long as the items.
template <int R, int S, int ST, int TW, bool OWN>
__global__ void __launch_bounds__(kThreads) conv_depthwise_kernel(DwParams prm)
{
    static_assert(S == 3 && (ST == 1 || ST == 2), "windows of three taps inside eight columns");
    constexpr int IW = (TW - 1) * ST + S;   // input columns one lane touches per kernel row
    static_assert(IW <= 6, "two column blocks: columns 0-3 and 4-5");
    extern __shared__ uint32_t wt[];        // [R][C] words: (w[c][r][0], w[c][r][1], w[c][r][2], 0)

    const ConvArgs &a = prm.a;
    uint32_t wown[R][4];                    // OWN: (w[c+e][r][0], w[c+e][r][1], w[c+e][r][2], 0) of the lane's channels c .. c+3
    if constexpr (OWN) {
        static_assert(R == 3 && S == 3, "36 weight bytes per lane");
        const int cwi = (int)((blockIdx.x * (unsigned)kThreads + threadIdx.x) % (unsigned)prm.cw);
        const uint32_t *wp = (const uint32_t *)(a.w + (size_t)cwi * 36);
        uint32_t d[10];
#pragma unroll
        for (int i = 0; i < 9; i++) d[i] = wp[i];
        d[9] = 0;
#pragma unroll
        for (int r = 0; r < R; r++)
#pragma unroll
            for (int e = 0; e < 4; e++) {
                const int k = 9 * e + 3 * r;    // first of the three bytes
                wown[r][e] = __builtin_amdgcn_alignbyte(d[(k >> 2) + 1], d[k >> 2], k & 3) & 0x00ffffffu;
            }
    }
    for (int c = threadIdx.x; !OWN && c < a.C; c += kThreads) {
        // the channel's R*S weight bytes, all loads in flight together
        uint32_t wb[R * S];
#pragma unroll
        for (int i = 0; i < R * S; i++) wb[i] = (uint8_t)a.w[(size_t)c * (R * S) + i];
#pragma unroll
        for (int r = 0; r < R; r++) wt[r * a.C + c] = wb[r * S] | (wb[r * S + 1] << 8) | (wb[r * S + 2] << 16);
    }
    __syncthreads();

    Requant rq;
    rq.init(a.shift, a.relu);
    const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc((void *)a.x, 0, (int)prm.x_bytes, 0x00020000);

    for (int it = blockIdx.x * kThreads + threadIdx.x; it < prm.items; it += gridDim.x * kThreads) {
        // it = ((n * P + p) * qblocks + qb) * cw + cwi, taken apart with multiply-high divisions
        int t = fastdiv(it, prm.div_cw);
        const int cwi = it - t * prm.cw;
        const int t2 = fastdiv(t, prm.div_qb);
        const int qb = t - t2 * prm.qblocks;
        const int n = fastdiv(t2, prm.div_p);
        const int p = t2 - n * a.P;
        const int c = cwi * 4;
        const int q0 = qb * TW;
        const int iw_first = q0 * ST - a.pad;

        // ---- every input word of the item, zeros where the window leaves the image
        uint32_t xw[R][6];
#pragma unroll
        for (int r = 0; r < R; r++) {
            const int ih = p * ST - a.pad + r;
            const bool rowok = (unsigned)ih < (unsigned)a.H;
            const unsigned rowoff = (unsigned)(((n * a.H + ih) * a.W) * a.C + c);
#pragma unroll
            for (int j = 0; j < 6; j++) {
                const int iw = iw_first + j;
                const bool ok = j < IW && rowok && (unsigned)iw < (unsigned)a.W;
                xw[r][j] = j < IW ? (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(xr, ok ? (int)(rowoff + (unsigned)(iw * a.C)) : (int)0x80000000, 0, 0)
                                  : 0u;
            }
        }

        int acc[TW][4];
        {
            int4 bv = make_int4(0, 0, 0, 0);
            if (a.b) bv = *(const int4 *)(a.b + c);
#pragma unroll
            for (int j = 0; j < TW; j++) { acc[j][0] = bv.x; acc[j][1] = bv.y; acc[j][2] = bv.z; acc[j][3] = bv.w; }
        }
#pragma unroll
        for (int r = 0; r < R; r++) {
            uint32_t wrow[4];
            if constexpr (OWN) {
#pragma unroll
                for (int e = 0; e < 4; e++) wrow[e] = wown[r][e];
            } else {
                const uint4 wq = *(const uint4 *)(wt + r * a.C + c);
                wrow[0] = wq.x; wrow[1] = wq.y; wrow[2] = wq.z; wrow[3] = wq.w;
            }
            // columns 0-3 transposed: lo[e] = (x0.e, x1.e, x2.e, x3.e); columns 4-5: hi[e] = (x4.e, x5.e, 0, 0)
            const uint32_t ab_l = __builtin_amdgcn_perm(xw[r][1], xw[r][0], 0x05010400u), ab_h = __builtin_amdgcn_perm(xw[r][1], xw[r][0], 0x07030602u);
            const uint32_t cd_l = __builtin_amdgcn_perm(xw[r][3], xw[r][2], 0x05010400u), cd_h = __builtin_amdgcn_perm(xw[r][3], xw[r][2], 0x07030602u);
            uint32_t lo[4], hi[4];
            lo[0] = __builtin_amdgcn_perm(cd_l, ab_l, 0x05040100u);
            lo[1] = __builtin_amdgcn_perm(cd_l, ab_l, 0x07060302u);
            lo[2] = __builtin_amdgcn_perm(cd_h, ab_h, 0x05040100u);
            lo[3] = __builtin_amdgcn_perm(cd_h, ab_h, 0x07060302u);
            hi[0] = __builtin_amdgcn_perm(xw[r][5], xw[r][4], 0x0c0c0400u);
            hi[1] = __builtin_amdgcn_perm(xw[r][5], xw[r][4], 0x0c0c0501u);
            hi[2] = __builtin_amdgcn_perm(xw[r][5], xw[r][4], 0x0c0c0602u);
            hi[3] = __builtin_amdgcn_perm(xw[r][5], xw[r][4], 0x0c0c0703u);
#pragma unroll
            for (int j = 0; j < TW; j++)
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    // pixels j*ST .. j*ST+3 of channel e; the fourth meets the zero in the weight word
                    const uint32_t win = j * ST == 0 ? lo[e] : __builtin_amdgcn_alignbyte(hi[e], lo[e], j * ST);
                    acc[j][e] = __builtin_amdgcn_sdot4((int)win, (int)wrow[e], acc[j][e], false);
                }
        }
        const size_t pix0 = ((size_t)n * a.P + p) * a.Q + q0;
        ChannelRequant cr[4];                                // one weight format per channel: each its own shift
        if (a.frac_w) {
#pragma unroll
            for (int e = 0; e < 4; e++) cr[e].init(a.shift + a.frac_w[c + e]);
        }
#pragma unroll
        for (int j = 0; j < TW; j++) {
            if (q0 + j >= a.Q) break;
            if (a.acc_out) *(int4 *)(a.acc_out + (pix0 + j) * a.K + c) = make_int4(acc[j][0], acc[j][1], acc[j][2], acc[j][3]);
            if (a.y) {
                int o[4];
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    if (a.frac_w) o[e] = cr[e].apply(acc[j][e], a.relu);
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
    const long long items = (long long)a.N * a.P * prm.qblocks * prm.cw;
    if (items >= (1LL << 31) - 256 * 16 * kThreads) return hipErrorInvalidValue;   // conv_depthwise_supports() rules this out
    prm.items = (int)items;
    prm.x_bytes = (unsigned)((long long)a.N * a.H * a.W * a.C);
    prm.div_cw = make_fastdiv(prm.cw);
    prm.div_qb = make_fastdiv(prm.qblocks);
    prm.div_p = make_fastdiv(a.P);
    long long blocks = (items + kThreads - 1) / kThreads;
    if (blocks > 256 * 8) blocks = 256 * 8;
    if (blocks < 1) blocks = 1;
    // a lane keeps its channels when blocks * kThreads is a multiple of C / 4: C / 4 a divisor of the block size, or a
    // multiple of it with the grid rounded down to whole sets of channels
    if (((uintptr_t)a.w & 3) == 0) {
        if (kThreads % prm.cw == 0) {
            conv_depthwise_kernel<R, S, ST, TW, true><<<(unsigned)blocks, kThreads, 0, st>>>(prm);
            return hipGetLastError();
        }
        if (prm.cw % kThreads == 0 && blocks >= prm.cw / kThreads) {
            blocks -= blocks % (prm.cw / kThreads);
            conv_depthwise_kernel<R, S, ST, TW, true><<<(unsigned)blocks, kThreads, 0, st>>>(prm);
            return hipGetLastError();
        }
    }
    // otherwise every block first gathers the weights of all channels: few, long-lived blocks
    size_t lds = (size_t)R * a.C * 4;
    conv_depthwise_kernel<R, S, ST, TW, false><<<(unsigned)blocks, kThreads, lds, st>>>(prm);
    return hipGetLastError();
}

}  // namespace

bool conv_depthwise_supports(const ConvArgs &a)
{
    if (a.groups != a.C || a.K != a.C) return false;
    if (a.C % 4) return false;
    if (a.R != 3 || a.S != 3 || (a.stride != 1 && a.stride != 2)) return false;
    if (a.C * 12 > 48 * 1024) return false;                                      // weight words in LDS
    if ((long long)a.N * a.H * a.W * a.C >= (1LL << 31)) return false;           // 31-bit byte offsets into the input
    // work items (4 channels x up to 4 pixels each) are numbered with 31 bits
    if ((long long)a.N * a.P * ((a.Q + 1) / 2) * (a.C / 4) >= (1LL << 31) - 256 * 16 * 256) return false;
    if (((uintptr_t)a.x & 3) || (a.y && (((uintptr_t)a.y & 3) || (a.ldy & 3)))) return false;
    if (a.b && ((uintptr_t)a.b & 15)) return false;
    if (a.acc_out && ((uintptr_t)a.acc_out & 15)) return false;
    return true;
}

hipError_t launch_conv_depthwise(const ConvArgs &a, hipStream_t st)
{
    // whole blocks of 64 channels, lean epilogue: the products go to the matrix cores (conv_dwm.hip)
    if (conv_dwm_supports(a)) return launch_conv_dwm(a, st);
    if (a.stride == 1) return launch_dw<3, 3, 1, 4>(a, st);
    return launch_dw<3, 3, 2, 2>(a, st);
}

}  // namespace dfq
