/*
 * dfq_probe - a MEASUREMENT AID for benchmarks of the dfq library, not part of the quantized path and
 * not part of libdfq.so (it is built into libdfq_probe.so): the rate of the int8 matrix instruction that
 * the dense convolution kernels use, v_mfma_i32_32x32x32_i8, on caller-supplied operand bytes, in a loop
 * that touches registers only.  The rate a chip sustains depends on the operand values (switching
 * activity under its power limit), so this is the ceiling a convolution on such data could reach with
 * free operand delivery.  No operation of the paper corresponds to it.
 */
#ifndef DFQ_PROBE_H
#define DFQ_PROBE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* a_codes: DEVICE, 16-byte aligned, at least 16 KiB read; b_codes: DEVICE, 16-byte aligned, at least
 * 32 KiB read; sink: DEVICE, blocks * 512 words, overwritten (content: the sum of a lane's accumulators).
 * 1 <= blocks <= 65536 workgroups of eight wavefronts, 1 <= iters <= 2^24 rounds of eight instructions per
 * wavefront.  *ops_out (host, may be NULL) receives the number of operations (2 per multiply-add) the
 * launch performs; the caller times the launch on `stream` (a hipStream_t; NULL = the default stream).
 * Returns 0, 1 for an invalid argument (nothing launched), 5 when the launch was refused. */
int dfq_probe_mfma_rate(const int8_t *a_codes, const int8_t *b_codes, int32_t *sink, int blocks, int iters,
                        double *ops_out, void *stream);

/* The same measurement for the item pipeline of the dense convolution kernel with its global loads left out: a
 * workgroup of eight wavefronts on a 256 x 256 tile, three LDS stages filled once from the operand bytes, and per
 * 64-byte step and wavefront sixteen matrix instructions, one workgroup barrier and twelve 128-bit LDS reads in the
 * kernel's order - the ceiling of that kernel on such data with free loads, prologue and epilogue.  Arguments and
 * return value as above (steps = reduction steps per workgroup; *ops_out = blocks * 8 * steps * 16 instructions). */
int dfq_probe_item_loop_rate(const int8_t *a_codes, const int8_t *b_codes, int32_t *sink, int blocks, int steps,
                             double *ops_out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* DFQ_PROBE_H */
