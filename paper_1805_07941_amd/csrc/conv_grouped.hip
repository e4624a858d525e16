// Grouped quantized convolution (1 < groups, C/groups a multiple of 4) on the vector ALUs.
//
// With groups the sum of Eq. 6 runs over the C/groups input channels of the output channel's own
// group only, so the reduction is short (4 .. 64 bytes per tap) and there is no dense contraction
// to give to the matrix cores.  Here a lane owns one output channel k of four neighbouring output
// pixels of a row and keeps their four sums in registers; per kernel row and 4-channel chunk it
// fetches the (3 * stride + S) input words its four pixels' taps cover once - range-checked buffer
// loads, so padding and rows outside the image arrive as zeros without a branch - and multiplies
// them with the S weight words of that row by v_dot4_i32_i8 (four multiply-adds per instruction).
// Consecutive lanes take consecutive output channels: lanes of one group ask for the same input
// word (one request, broadcast), lanes of neighbouring groups for neighbouring words, and the
// output bytes of a wavefront are contiguous.  The weights of all K channels sit in LDS,
// transposed to [tap and chunk][k] words so that a wavefront's read touches 64 different banks.
// Bias is the start value of the sums; ReLU, the rounding shift (one per layer or one per output
// channel) and the clamp follow in registers.
#include "conv_epilogue.hpp"

namespace dfq {

namespace {

constexpr int kGroupedThreads = 256;
constexpr int kPX = 4;                     // output pixels per lane

struct GroupedParams {
    ConvArgs a;
    int Cg, Kg;
    int chunks;                            // Cg / 4
    int qblocks;                           // ceil(Q / kPX)
    int items;                             // N * P * qblocks * K
    unsigned x_bytes;
    FastDiv div_k, div_qb, div_p, div_kg;
};

template <int S, int ST>
__global__ void __launch_bounds__(kGroupedThreads) conv_grouped_kernel(GroupedParams prm)
{
    constexpr int NS = (kPX - 1) * ST + S;                 // input columns the four pixels' taps of one kernel row cover
    extern __shared__ uint32_t wl[];                       // [R][S][chunks][K] weight words
    const ConvArgs &a = prm.a;
    const int K = a.K, R = a.R, chunks = prm.chunks;
    // weights: word (r, s, j) of channel k is bytes 4j .. 4j+3 of w[k][r][s][.]
    {
        const int row_words = R * S * chunks;
        const uint32_t *wg = (const uint32_t *)a.w;
        for (int i = threadIdx.x; i < K * row_words; i += kGroupedThreads) {
            const int k = i / row_words, t = i - k * row_words;
            wl[t * K + k] = wg[i];
        }
    }
    __syncthreads();
    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(a.x), 0, (int)prm.x_bytes, 0x00020000);

    for (int item = blockIdx.x * kGroupedThreads + threadIdx.x; item < prm.items; item += gridDim.x * kGroupedThreads) {
        int t = fastdiv(item, prm.div_k);
        const int k = item - t * K;
        const int pr = fastdiv(t, prm.div_qb);
        const int q0 = (t - pr * prm.qblocks) * kPX;
        const int n = fastdiv(pr, prm.div_p);
        const int p = pr - n * a.P;
        const int g = fastdiv(k, prm.div_kg);
        const int ih0 = p * a.stride - a.pad, iw0 = q0 * ST - a.pad;
        // byte offset of each input column inside an image row; a column outside the row, like a row outside the image,
        // sets the top bit of the load's offset: past the end of the buffer, where the range check returns zeros
        unsigned col_off[NS];
#pragma unroll
        for (int c = 0; c < NS; c++) {
            const int iw = iw0 + c;
            col_off[c] = (iw >= 0 && iw < a.W) ? (unsigned)(iw * a.C) : 0x80000000u;
        }
        const unsigned img_off = (unsigned)(n * a.H * a.W * a.C + g * prm.Cg);
        int acc[kPX];
        const int b0 = a.b ? a.b[k] : 0;
#pragma unroll
        for (int px = 0; px < kPX; px++) acc[px] = b0;
        for (int r = 0; r < R; r++) {
            const int ih = ih0 + r;
            const bool row_in = ih >= 0 && ih < a.H;
            const unsigned row_off = row_in ? img_off + (unsigned)(ih * a.W * a.C) : 0u;
            const unsigned row_bad = row_in ? 0u : 0x80000000u;
            for (int j = 0; j < chunks; j++) {
                uint32_t xv[NS], wv[S];
#pragma unroll
                for (int c = 0; c < NS; c++)
                    xv[c] = __builtin_amdgcn_raw_buffer_load_b32(
                        xrsrc, (int)(((row_off + (unsigned)(4 * j) + (col_off[c] & 0x7fffffffu)) & 0x7fffffffu) | row_bad | (col_off[c] & 0x80000000u)),
                        0, 0);
#pragma unroll
                for (int s = 0; s < S; s++) wv[s] = wl[((r * S + s) * chunks + j) * K + k];
#pragma unroll
                for (int px = 0; px < kPX; px++)
#pragma unroll
                    for (int s = 0; s < S; s++) acc[px] = __builtin_amdgcn_sdot4((int)xv[px * ST + s], (int)wv[s], acc[px], false);
            }
        }
        ChannelRequant cr;
        cr.init(a.frac_w ? a.shift + a.frac_w[k] : a.shift);
#pragma unroll
        for (int px = 0; px < kPX; px++) {
            const int q = q0 + px;
            if (q < a.Q) {
                const size_t pix = ((size_t)n * a.P + p) * a.Q + q;
                if (a.acc_out) a.acc_out[pix * K + k] = acc[px];
                if (a.y) a.y[pix * (size_t)a.ldy + k] = (int8_t)cr.apply(acc[px], a.relu);
            }
        }
    }
}

template <int S, int ST>
hipError_t launch_grouped(const GroupedParams &prm, size_t lds, hipStream_t st)
{
    static const hipError_t attr = hipFuncSetAttribute((const void *)conv_grouped_kernel<S, ST>, hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024);
    if (attr != hipSuccess) return attr;
    long long blocks = ((long long)prm.items + kGroupedThreads - 1) / kGroupedThreads;
    if (blocks > 256 * 8) blocks = 256 * 8;        // every block first gathers all weights: few, long-lived blocks
    conv_grouped_kernel<S, ST><<<(unsigned)blocks, kGroupedThreads, lds, st>>>(prm);
    return hipGetLastError();
}

}  // namespace

bool conv_grouped_supports(const ConvArgs &a)
{
    if (a.groups < 2) return false;
    const int Cg = a.C / a.groups;
    if (Cg % 4) return false;
    if (a.S != 1 && a.S != 3 && a.S != 5 && a.S != 7) return false;
    if (a.stride != 1 && a.stride != 2) return false;
    if ((long long)a.K * a.R * a.S * Cg > 64 * 1024) return false;                 // all weights in LDS
    if ((long long)a.N * a.H * a.W * a.C >= (1LL << 31)) return false;             // 31-bit byte offsets into the input
    if ((long long)a.N * a.P * ((a.Q + kPX - 1) / kPX) * a.K >= (1LL << 31) - 256LL * 8 * kGroupedThreads) return false;
    if (((uintptr_t)a.x & 3) || ((uintptr_t)a.w & 3)) return false;
    return true;
}

hipError_t launch_conv_grouped(const ConvArgs &a, hipStream_t st)
{
    // whole groups inside blocks of 64 channels, lean epilogue: the matrix cores take the layer (conv_sg.hip)
    if (conv_sg_supports(a)) return launch_conv_sg(a, st);
    GroupedParams prm;
    prm.a = a;
    prm.Cg = a.C / a.groups;
    prm.Kg = a.K / a.groups;
    prm.chunks = prm.Cg / 4;
    prm.qblocks = (a.Q + kPX - 1) / kPX;
    prm.items = (int)((long long)a.N * a.P * prm.qblocks * a.K);
    prm.x_bytes = (unsigned)((long long)a.N * a.H * a.W * a.C);
    prm.div_k = make_fastdiv(a.K);
    prm.div_qb = make_fastdiv(prm.qblocks);
    prm.div_p = make_fastdiv(a.P);
    prm.div_kg = make_fastdiv(prm.Kg);
    const size_t lds = (size_t)a.K * a.R * a.S * prm.Cg;
    switch (a.S * 10 + a.stride) {
        case 11: return launch_grouped<1, 1>(prm, lds, st);
        case 12: return launch_grouped<1, 2>(prm, lds, st);
        case 31: return launch_grouped<3, 1>(prm, lds, st);
        case 32: return launch_grouped<3, 2>(prm, lds, st);
        case 51: return launch_grouped<5, 1>(prm, lds, st);
        case 52: return launch_grouped<5, 2>(prm, lds, st);
        case 71: return launch_grouped<7, 1>(prm, lds, st);
        case 72: return launch_grouped<7, 2>(prm, lds, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace dfq
