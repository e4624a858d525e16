// Measurement aid, not part of the quantized path: the rate of the int8 matrix instruction that
// the dense convolution kernels use (v_mfma_i32_32x32x32_i8) on operands taken from caller data,
// with nothing else going on - operands are loaded once, the loop touches registers only, one
// word per lane is stored at the end so the work cannot be discarded.  The rate a chip sustains
// depends on the operand values (switching activity under its power limit), so this gives the
// ceiling a convolution on the same data could reach if operand delivery were free.
#include "conv_epilogue.hpp"
#include "dfq_host.hpp"

namespace dfq {

namespace {

constexpr int kProbeThreads = 512;    // eight wavefronts: two per SIMD
constexpr int kProbeA = 2, kProbeB = 4;

__global__ void __launch_bounds__(kProbeThreads, 1) mfma_rate_probe_kernel(const v4i *a_src, const v4i *b_src, int *sink, int iters)
{
    const int t = threadIdx.x;
    v4i a[kProbeA], b[kProbeB];
#pragma unroll
    for (int i = 0; i < kProbeA; i++) a[i] = a_src[i * kProbeThreads + t];
#pragma unroll
    for (int j = 0; j < kProbeB; j++) b[j] = b_src[j * kProbeThreads + t];
    v16i acc[kProbeA][kProbeB];
#pragma unroll
    for (int i = 0; i < kProbeA; i++)
#pragma unroll
        for (int j = 0; j < kProbeB; j++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[i][j][r] = 0;
    for (int it = 0; it < iters; it++) {
#pragma unroll
        for (int i = 0; i < kProbeA; i++)
#pragma unroll
            for (int j = 0; j < kProbeB; j++) acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int i = 0; i < kProbeA; i++)
#pragma unroll
        for (int j = 0; j < kProbeB; j++)
#pragma unroll
            for (int r = 0; r < 16; r++) s += acc[i][j][r];
    sink[blockIdx.x * kProbeThreads + t] = s;
}

}  // namespace

size_t mfma_rate_probe_a_bytes() { return (size_t)kProbeA * kProbeThreads * 16; }
size_t mfma_rate_probe_b_bytes() { return (size_t)kProbeB * kProbeThreads * 16; }
size_t mfma_rate_probe_sink_words(int blocks) { return (size_t)blocks * kProbeThreads; }
double mfma_rate_probe_ops(int blocks, int iters)
{
    return (double)blocks * (kProbeThreads / 64) * (double)iters * (kProbeA * kProbeB) * (2.0 * 32 * 32 * 32);
}

hipError_t launch_mfma_rate_probe(const int8_t *a, const int8_t *b, int32_t *sink, int blocks, int iters, hipStream_t st)
{
    mfma_rate_probe_kernel<<<(unsigned)blocks, kProbeThreads, 0, st>>>((const v4i *)a, (const v4i *)b, sink, iters);
    return hipGetLastError();
}

}  // namespace dfq
