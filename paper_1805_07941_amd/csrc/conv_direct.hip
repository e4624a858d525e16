// Direct convolution: one output element (pixel, channel) per lane, the sum of Eq. 6 taken
// tap by tap.  Accepts every geometry the library allows (any C, K, groups, stride, pad); it
// is the kernel of last resort for shapes the tiled kernels do not cover, and the simplest
// statement of the operation on the device.  Consecutive lanes take consecutive output
// channels, so activations are broadcast within a wavefront and the output is written
// densely.
#include "dfq_device.hpp"
#include "dfq_host.hpp"

namespace dfq {

__global__ void __launch_bounds__(256) conv_direct_kernel(ConvArgs a)
{
    const int Cg = a.C / a.groups;
    const int Kg = a.K / a.groups;
    const size_t total = (size_t)a.N * a.P * a.Q * a.K;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const int k = (int)(i % a.K);
        const size_t pix = i / a.K;
        const int q = (int)(pix % a.Q);
        const size_t t = pix / a.Q;
        const int p = (int)(t % a.P);
        const int n = (int)(t / a.P);
        const int g = k / Kg;
        int acc = a.b ? a.b[k] : 0;
        for (int r = 0; r < a.R; r++) {
            const int ih = p * a.stride - a.pad + r;
            if (ih < 0 || ih >= a.H) continue;
            for (int s = 0; s < a.S; s++) {
                const int iw = q * a.stride - a.pad + s;
                if (iw < 0 || iw >= a.W) continue;
                const int8_t *xp = a.x + (((size_t)n * a.H + ih) * a.W + iw) * a.C + (size_t)g * Cg;
                const int8_t *wp = a.w + (((size_t)k * a.R + r) * a.S + s) * Cg;
                for (int c = 0; c < Cg; c++) acc += (int)xp[c] * (int)wp[c];
            }
        }
        if (a.acc_out) a.acc_out[i] = acc;
        if (a.y) {
            if (a.relu) acc = max(acc, 0);
            a.y[pix * (size_t)a.ldy + k] = (int8_t)requant8(acc, a.frac_w ? a.shift + a.frac_w[k] : a.shift);
        }
    }
}

bool conv_direct_supports(const ConvArgs &) { return true; }

hipError_t launch_conv_direct(const ConvArgs &a, hipStream_t st)
{
    size_t total = (size_t)a.N * a.P * a.Q * a.K;
    size_t blocks = (total + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    conv_direct_kernel<<<(int)blocks, 256, 0, st>>>(a);
    return hipGetLastError();
}

}  // namespace dfq
