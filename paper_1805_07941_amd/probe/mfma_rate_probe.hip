// Measurement aid, not part of the quantized path: the rate of the int8 matrix instruction that
// the dense convolution kernels use (v_mfma_i32_32x32x32_i8) on operands taken from caller data,
// with nothing else going on - operands are loaded once, the loop touches registers only, one
// word per lane is stored at the end so the work cannot be discarded.  The rate a chip sustains
// depends on the operand values (switching activity under its power limit), so this gives the
// ceiling a convolution on the same data could reach if operand delivery were free.
//
// Built into a library of its own (libdfq_probe.so, include/dfq_probe.h); libdfq.so does not contain it.
#include "dfq_probe.h"

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

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

extern "C" int dfq_probe_mfma_rate(const int8_t *a_codes, const int8_t *b_codes, int32_t *sink, int blocks, int iters,
                                   double *ops_out, void *stream)
{
    if (!a_codes || !b_codes || !sink) return 1;
    if (blocks < 1 || blocks > 65536 || iters < 1 || iters > (1 << 24)) return 1;
    if (((uintptr_t)a_codes & 15) || ((uintptr_t)b_codes & 15) || ((uintptr_t)sink & 3)) return 1;
    if (ops_out) *ops_out = (double)blocks * (kProbeThreads / 64) * (double)iters * (kProbeA * kProbeB) * (2.0 * 32 * 32 * 32);
    mfma_rate_probe_kernel<<<(unsigned)blocks, kProbeThreads, 0, (hipStream_t)stream>>>((const v4i *)a_codes, (const v4i *)b_codes,
                                                                                          sink, iters);
    return hipGetLastError() == hipSuccess ? 0 : 5;
}
