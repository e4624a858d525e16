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

// The item pipeline of the dense convolution kernel without its global loads: a workgroup of eight wavefronts owns a
// 256 x 256 output tile (wavefront tile 64 x 128), LDS holds three stages of (256 + 256) rows x 64 bytes filled once
// from the caller's bytes, and every step issues what the kernel issues per 64-byte reduction step and wavefront -
// sixteen matrix instructions in two halves, one workgroup barrier, twelve 128-bit LDS reads into the registers
// just consumed - in the kernel's order.  Its rate is what the kernel could reach on such data if loads, prologue and
// epilogue were free.
constexpr int kLoopThreads = 512, kLoopCT = 4, kLoopPT = 2, kLoopStages = 3, kLoopRows = 512, kLoopStagePieces = kLoopRows * 4;

__global__ void __launch_bounds__(kLoopThreads, 1) item_loop_probe_kernel(const v4i *a_src, const v4i *b_src, int *sink, int steps)
{
    extern __shared__ v4i lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // pixel rows from b_src (32 KiB), channel rows from a_src (16 KiB), repeated over the stages
    for (int i = tid; i < kLoopStages * kLoopStagePieces; i += kLoopThreads) {
        const int in_stage = i % kLoopStagePieces, stage = i / kLoopStagePieces;
        lds[i] = in_stage < 1024 ? b_src[(in_stage + 1024 * stage) & 2047] : a_src[(in_stage - 1024) & 1023];
    }
    __syncthreads();
    const int wp0 = (wave % 4) * 64, wc0 = (wave / 4) * 128;
    const int l32 = lane & 31, lh = lane >> 5, swz = (l32 >> 2) & 3;
    v16i acc[kLoopCT][kLoopPT];
#pragma unroll
    for (int c = 0; c < kLoopCT; c++)
#pragma unroll
        for (int p = 0; p < kLoopPT; p++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[c][p][r] = 0;
    struct Half {
        v4i w[kLoopCT];
        v4i x[kLoopPT];
    };
    Half f0, f1;
    auto read_half = [&](Half &f, int kk, int stage) __attribute__((always_inline)) {
        const v4i *xs = lds + stage * kLoopStagePieces;
        const v4i *ws = xs + 256 * 4;
        const int g = (kk * 2 + lh) ^ swz;
#pragma unroll
        for (int c = 0; c < kLoopCT; c++) f.w[c] = ws[(wc0 + c * 32 + l32) * 4 + g];
#pragma unroll
        for (int p = 0; p < kLoopPT; p++) f.x[p] = xs[(wp0 + p * 32 + l32) * 4 + g];
    };
    auto mfma_half = [&](const Half &f) __attribute__((always_inline)) {
#pragma unroll
        for (int c = 0; c < kLoopCT; c++)
#pragma unroll
            for (int p = 0; p < kLoopPT; p++) acc[c][p] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f.w[c], f.x[p], acc[c][p], 0, 0, 0);
    };
    read_half(f0, 0, 0);
    read_half(f1, 1, 0);
    int stage = 0;
    for (int it = 0; it < steps; it++) {
        const int next = stage + 1 == kLoopStages ? 0 : stage + 1;
        mfma_half(f0);
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        read_half(f0, 0, next);
        __builtin_amdgcn_sched_barrier(0);
        mfma_half(f1);
        __builtin_amdgcn_sched_barrier(0);
        read_half(f1, 1, next);
        __builtin_amdgcn_sched_barrier(0);
        stage = next;
    }
    int s = f0.w[0][0] + f1.x[0][1];
#pragma unroll
    for (int c = 0; c < kLoopCT; c++)
#pragma unroll
        for (int p = 0; p < kLoopPT; p++)
#pragma unroll
            for (int r = 0; r < 16; r++) s += acc[c][p][r];
    sink[blockIdx.x * kLoopThreads + tid] = s;
}

}  // namespace

extern "C" int dfq_probe_item_loop_rate(const int8_t *a_codes, const int8_t *b_codes, int32_t *sink, int blocks, int steps,
                                        double *ops_out, void *stream)
{
    if (!a_codes || !b_codes || !sink) return 1;
    if (blocks < 1 || blocks > 65536 || steps < 1 || steps > (1 << 24)) return 1;
    if (((uintptr_t)a_codes & 15) || ((uintptr_t)b_codes & 15) || ((uintptr_t)sink & 3)) return 1;
    constexpr size_t lds_bytes = (size_t)kLoopStages * kLoopStagePieces * 16;
    static const hipError_t attr = hipFuncSetAttribute((const void *)item_loop_probe_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                                       (int)lds_bytes);
    if (attr != hipSuccess) return 5;
    if (ops_out) *ops_out = (double)blocks * (kLoopThreads / 64) * (double)steps * (2 * kLoopCT * kLoopPT) * (2.0 * 32 * 32 * 32);
    item_loop_probe_kernel<<<(unsigned)blocks, kLoopThreads, lds_bytes, (hipStream_t)stream>>>((const v4i *)a_codes, (const v4i *)b_codes,
                                                                                                sink, steps);
    return hipGetLastError() == hipSuccess ? 0 : 5;
}

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
