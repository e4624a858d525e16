// First layer of an image network (3 input channels, stride 2) on the int8 matrix cores, one workgroup per
// horizontal strip of an image, alone (conv_stem_kernel) or with the 3x3 / stride-2 / pad-1 max-pooling that
// follows it done in the same kernel (conv_stem_pool_kernel).
//
// The sum is that of Eq. 6 term for term; only the way the operands reach the matrix instruction differs from
// conv_smallc.hip.  Input rows are staged in LDS with every pixel padded from 3 to 4 bytes (the fourth byte is
// whatever follows in memory; its weight is 0).  With stride 2 the S taps of a kernel row for output column q
// then start at an even input column, i.e. at LDS byte 8 q + const: the 32-byte block of the reduction axis
// (8 input pixels x 4 bytes, S + (pad & 1) <= 8 of them with non-zero weights) is two aligned 8-byte LDS reads
// per lane, no byte shifting.  A workgroup walks down its strip four output rows at a time ("step"): the
// 6 + R input rows of a step live in a ring of 16 LDS rows, the 8 new rows of the next step are fetched into
// registers while the current step is multiplied.
//
// conv_stem_kernel: a 32-pixel operand group is 16 columns x 2 rows; a wavefront owns one block of 16 columns
// (both row pairs of the step) and stores its rounded results.
//
// conv_stem_pool_kernel: pooling is done on the 32-bit sums, before the rounding (ReLU and the rounding shift
// are monotone, so the maximum of the rounded values is the rounded maximum: same bytes as the two calls).  The
// four operand groups of a wavefront are the four parities (row, column) of the output pixels under 16 pooled
// columns x 2 pooled rows, so that lane (pooled row ph, pooled column pw) holds outputs (2ph, 2pw), (2ph, 2pw+1),
// (2ph+1, 2pw), (2ph+1, 2pw+1) in four accumulator tiles.  Of the nine window positions of pooled pixel (ph, pw)
// four are then in the lane itself, two (column 2pw-1) in the lane to the left - reached by a row shift of the
// data-parallel-primitive path -, two (row 2ph-1) in the lane 16 places away or, for the upper pooled row of a
// step, in what that lane held one step earlier (kept in registers), one in both directions.  Window positions
// outside the image never enter: a lane without a left neighbour keeps its value, the row above the image is the
// smallest integer.  Only the pooled pixels are rounded (a quarter of the rounding work) and stored; the
// convolution's own tensor exists nowhere.  Column blocks overlap by one pooled column (the left neighbour of a
// block's first column is recomputed in the block, its result discarded); a strip that does not start at the top
// of the image recomputes the step above it for the row its first windows need.
#include <cmath>
#include <type_traits>

#include "conv_ring.hpp"

namespace dfq {

namespace {

constexpr int kRowSlots = 16;    // ring of staged input rows
constexpr int kLeftPad = 16;     // LDS bytes in front of input column 0 of a staged row
constexpr int kIntMin = -2147483647 - 1;

struct StemParams {
    ConvArgs a;
    int8_t *yp;          // pooled output [N, PP, PQ, K] with ldyp bytes between pixels (pooling form only)
    int ldyp;
    int PP, PQ;          // pooled extent
    int pitch;           // LDS bytes of a staged input row
    int off0;            // LDS byte, inside a staged row, of the reduction block of output column 0
    int steps;           // ceil(P / 4)
    int strips;          // strips per image
    int steps_per_strip;
    int triples;         // W / 4: 12-byte pieces of an input row
    const float *xf;     // float images [N, H, W, 3] to be converted to codes on the way in, or null
    float scale;         // 2^f_in of that conversion
};

struct Row12 {
    uint32_t d[3];
};

// Weights, bias and an all-zero input ring into LDS.  Weight block (r, k) of 32 bytes = for input pixel i of the
// run (i = 0..7) the 3 channel weights of tap s = i - (pad & 1), a zero in the fourth byte and zeros where there
// is no such tap; rows permuted so that a lane's 16 accumulators are 16 consecutive channels (as in the other
// matrix-core kernels).  The ring starts as zeros: the bytes left and right of the image are never written again.
template <int BC, int R, int THREADS>
__device__ __forceinline__ void stem_setup(const ConvArgs &a, int8_t *lds, int *biasl, int8_t *xin, int ring_bytes)
{
    const int tid = threadIdx.x;
    const int odd = a.pad & 1;
    // one dword (input pixel i of the run of kernel row r, channel k) per iteration
    for (int t = tid; t < R * BC * 8; t += THREADS) {
        const int i = t & 7;
        const int kl = (t >> 3) % BC;
        const int r = (t >> 3) / BC;
        const int s = i - odd;
        uint32_t v = 0;
        if (s >= 0 && s < a.S && kl < a.K) {
            const uint8_t *src = (const uint8_t *)a.w + (((size_t)kl * R + r) * a.S + s) * 3;
            v = (uint32_t)src[0] | ((uint32_t)src[1] << 8) | ((uint32_t)src[2] << 16);
        }
        const int c32 = kl & 31;
        const int row = (kl & ~31) + 8 * ((c32 & 15) >> 2) + 4 * (c32 >> 4) + (c32 & 3);
        const int piece = (i >> 2) ^ ((row >> 3) & 1);
        *(uint32_t *)(lds + ((r * BC + row) * 2 + piece) * 16 + 4 * (i & 3)) = v;
    }
    for (int i = tid; i < BC; i += THREADS) biasl[i] = (a.b && i < a.K) ? a.b[i] : 0;
    for (int i = tid; i < ring_bytes / 8; i += THREADS) ((uint2 *)xin)[i] = make_uint2(0, 0);
}

// `count` input rows from `first` on, dealt to the NW wavefronts: 12 bytes (4 pixels) per lane into registers
template <int NW, int MAXR>
__device__ __forceinline__ void stem_fetch_rows(const ConvArgs &a, const int8_t *ximg, int triples, int wave, int lane, int first,
                                                int count, Row12 (&pf)[MAXR])
{
#pragma unroll
    for (int j = 0; j < MAXR; j++) {
        const int k = wave + j * NW;
        const int row = first + k;
        pf[j].d[0] = pf[j].d[1] = pf[j].d[2] = 0;
        if (k < count && (unsigned)row < (unsigned)a.H && lane < triples) {
            const uint32_t *src = (const uint32_t *)(ximg + (size_t)row * (a.W * 3) + 12 * lane);
            pf[j].d[0] = src[0];
            pf[j].d[1] = src[1];
            pf[j].d[2] = src[2];
        }
    }
}

// ... and into the ring, 16 bytes (4 pixels of 4 bytes) per lane, rows outside the image as zeros.  SKEW: ring rows
// whose slot has bit 2 set start 8 bytes later (see conv_stem_pool_kernel).
template <int NW, int MAXR, bool SKEW>
__device__ __forceinline__ void stem_stage_rows(int8_t *xin, int pitch, int triples, int wave, int lane, int first, int count,
                                                const Row12 (&pf)[MAXR])
{
#pragma unroll
    for (int j = 0; j < MAXR; j++) {
        const int k = wave + j * NW;
        const int row = first + k;
        if (k < count && lane < triples) {
            const uint32_t d0 = pf[j].d[0], d1 = pf[j].d[1], d2 = pf[j].d[2];
            const int slot = (row + 32) & (kRowSlots - 1);
            uint2 *dst = (uint2 *)(xin + slot * pitch + (SKEW ? 2 * (slot & 4) : 0) + kLeftPad + 16 * lane);
            dst[0] = make_uint2(d0, __builtin_amdgcn_alignbit(d1, d0, 24));
            dst[1] = make_uint2(__builtin_amdgcn_alignbit(d2, d1, 16), d2 >> 8);
        }
    }
}

// The same two steps for float images that are converted on the way in (Sec. 3, conversion paragraph; the
// arithmetic of dfq_quantize: x * 2^f is exact, round to nearest even, NaN -> 0, clamp to +-127): 12 floats per lane.
struct Row12f {
    float4 v[3];
};

template <int NW, int MAXR>
__device__ __forceinline__ void stem_fetch_rows(const ConvArgs &a, const float *ximg, int triples, int wave, int lane, int first,
                                                int count, Row12f (&pf)[MAXR])
{
#pragma unroll
    for (int j = 0; j < MAXR; j++) {
        const int k = wave + j * NW;
        const int row = first + k;
        pf[j].v[0] = pf[j].v[1] = pf[j].v[2] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (k < count && (unsigned)row < (unsigned)a.H && lane < triples) {
            const float4 *src = (const float4 *)(ximg + (size_t)row * (a.W * 3) + 12 * lane);
            pf[j].v[0] = src[0];
            pf[j].v[1] = src[1];
            pf[j].v[2] = src[2];
        }
    }
}

__device__ __forceinline__ int stem_code(float x, float scale)
{
    // v_cvt_i32_f32 gives 0 for NaN and saturates beyond the 32-bit range (the instruction, not a C cast, whose result
    // is undefined there), so the clamp can follow the conversion; the rounded value is integral, the conversion exact
    const float t = __builtin_rintf(x * scale);
    int c;
    asm("v_cvt_i32_f32 %0, %1" : "=v"(c) : "v"(t));
    return max(-127, min(127, c));
}

template <int NW, int MAXR, bool SKEW>
__device__ __forceinline__ void stem_stage_rows(int8_t *xin, int pitch, int triples, int wave, int lane, int first, int count,
                                                const Row12f (&pf)[MAXR], float scale)
{
#pragma unroll
    for (int j = 0; j < MAXR; j++) {
        const int k = wave + j * NW;
        const int row = first + k;
        if (k < count && lane < triples) {
            const float4 a0 = pf[j].v[0], a1 = pf[j].v[1], a2 = pf[j].v[2];
            const float f[12] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w, a2.x, a2.y, a2.z, a2.w};
            uint32_t w[4];
#pragma unroll
            for (int px = 0; px < 4; px++)
                w[px] = pack4_clamped(stem_code(f[3 * px], scale), stem_code(f[3 * px + 1], scale), stem_code(f[3 * px + 2], scale), 0);
            const int slot = (row + 32) & (kRowSlots - 1);
            uint2 *dst = (uint2 *)(xin + slot * pitch + (SKEW ? 2 * (slot & 4) : 0) + kLeftPad + 16 * lane);
            dst[0] = make_uint2(w[0], w[1]);
            dst[1] = make_uint2(w[2], w[3]);
        }
    }
}

// XF: float images, converted to codes while they are staged (prm.xf, prm.scale; a.x is not read)
template <int CT, int NW, int R, bool XF>
__global__ void __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(4, 4))) conv_stem_kernel(StemParams prm)
{
    constexpr int BC = CT * 32;
    constexpr int kThreads = NW * 64;
    constexpr int kRowsFirst = R + 6;                       // input rows of one step
    constexpr int MAXR = (8 + NW - 1) / NW;                 // staged rows one wavefront carries at a time (8 rows per round)
    constexpr int kWeightBytes = R * BC * 32;
    extern __shared__ uint4 lds4[];
    const ConvArgs &a = prm.a;
    int8_t *const lds = (int8_t *)lds4;
    int *const biasl = (int *)(lds + kWeightBytes);
    int8_t *const xin = lds + kWeightBytes + BC * 4;

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, lh = lane >> 5;

    stem_setup<BC, R, kThreads>(a, lds, biasl, xin, kRowSlots * prm.pitch);
    __syncthreads();

    Requant rq;
    rq.init(a.shift, a.relu);
    const v4i *const wl = (const v4i *)lds;

    const int n = blockIdx.x / prm.strips;
    const int strip = blockIdx.x - n * prm.strips;
    const int t0 = strip * prm.steps_per_strip;
    const int t1 = min(t0 + prm.steps_per_strip, prm.steps);
    typedef typename std::conditional<XF, float, int8_t>::type In;
    typedef typename std::conditional<XF, Row12f, Row12>::type Rows;
    const In *const ximg = (XF ? (const In *)prm.xf : (const In *)a.x) + (size_t)n * a.H * a.W * 3;
    auto stage = [&](int first, int count, const Rows (&rows)[MAXR]) __attribute__((always_inline)) {
        if constexpr (XF) stem_stage_rows<NW, MAXR, false>(xin, prm.pitch, prm.triples, wave, lane, first, count, rows, prm.scale);
        else stem_stage_rows<NW, MAXR, false>(xin, prm.pitch, prm.triples, wave, lane, first, count, rows);
    };

    Rows pf[MAXR];
    stem_fetch_rows<NW, MAXR>(a, ximg, prm.triples, wave, lane, 8 * t0 - a.pad, 8, pf);
    stage(8 * t0 - a.pad, 8, pf);
    stem_fetch_rows<NW, MAXR>(a, ximg, prm.triples, wave, lane, 8 * t0 - a.pad + 8, kRowsFirst - 8, pf);
    stage(8 * t0 - a.pad + 8, kRowsFirst - 8, pf);
    __syncthreads();

    const int ncb = a.Q >> 4;
    for (int t = t0; t < t1; t++) {
        const bool has_next = t + 1 < t1;
        const int next_first = 8 * t - a.pad + kRowsFirst;
        if (has_next) stem_fetch_rows<NW, MAXR>(a, ximg, prm.triples, wave, lane, next_first, 8, pf);

        for (int cb = wave; cb < ncb; cb += NW) {
            asm volatile("" ::: "memory");      // the weights are read from LDS per use, not kept in registers across blocks
            const int qcol = 16 * cb + (l32 & 15);
            const int rsel = l32 >> 4;
            const int ihb = 2 * (4 * t + rsel) - a.pad + 32;            // input row of kernel row 0, group 0, plus 32
            const int colbyte = 8 * qcol + prm.off0 + 16 * lh;
            v16i acc[CT][2];
#pragma unroll
            for (int c = 0; c < CT; c++)
#pragma unroll
                for (int r4 = 0; r4 < 4; r4++) {
                    const int4 bv = *(const int4 *)(biasl + c * 32 + 16 * lh + 4 * r4);
#pragma unroll
                    for (int g = 0; g < 2; g++) {
                        acc[c][g][4 * r4] = bv.x; acc[c][g][4 * r4 + 1] = bv.y; acc[c][g][4 * r4 + 2] = bv.z; acc[c][g][4 * r4 + 3] = bv.w;
                    }
                }
#pragma unroll
            for (int r = 0; r < R; r++) {
                if (r & 1) asm volatile("" ::: "memory");      // at most two kernel rows' operand reads are in flight together
                v4i xf[2];
#pragma unroll
                for (int g = 0; g < 2; g++) {
                    const uint2 *src = (const uint2 *)(xin + ((ihb + 4 * g + r) & (kRowSlots - 1)) * prm.pitch + colbyte);
                    const uint2 lo = src[0], hi = src[1];
                    xf[g] = v4i{(int)lo.x, (int)lo.y, (int)hi.x, (int)hi.y};
                }
#pragma unroll
                for (int c = 0; c < CT; c++) {
                    const int row = c * 32 + l32;
                    const v4i wf = wl[(r * BC + row) * 2 + (lh ^ ((row >> 3) & 1))];
#pragma unroll
                    for (int g = 0; g < 2; g++) acc[c][g] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf, xf[g], acc[c][g], 0, 0, 0);
                }
            }
            settle_accumulators<CT * 2>(&acc[0][0]);
#pragma unroll
            for (int g = 0; g < 2; g++) {
                const int p = 4 * t + 2 * g + rsel;
#pragma unroll
                for (int c = 0; c < CT; c++) {
                    const uint4 o = requant_tile_lane_fast(acc[c][g], rq);
                    if (p < a.P) *(uint4 *)(a.y + (((size_t)n * a.P + p) * a.Q + qcol) * a.ldy + c * 32 + 16 * lh) = o;
                }
            }
        }
        __syncthreads();          // the step's reads of the input ring are done
        if (has_next) stage(next_first, 8, pf);
        __syncthreads();          // the next step's input rows are staged
    }
}

// value of lane - 1 within rows of 16 lanes; a row's first lane gets its own value back
__device__ __forceinline__ int from_left_lane(int v)
{
    return __builtin_amdgcn_update_dpp(v, v, 0x111 /* row_shr:1 */, 0xf, 0xf, false);
}

// Convolution + 3x3 / 2 / pad 1 max-pooling.  Four wavefronts, wavefront w = block w of pooled columns
// 15 w .. 15 w + 15 (the first column of blocks 1.. is the recomputed left neighbour).  Lane = (pooled column
// 15 w + (lane & 15), pooled row 2t + ((lane >> 4) & 1), half of the reduction block lane >> 5).  Ring rows whose
// slot has bit 2 set are staged 8 bytes later: the two pooled rows of a lane group lie four input rows apart, and
// with the 16-byte lane stride this puts their 8-byte reads on disjoint LDS banks.
// PC: one weight format per output channel (a.frac_w, every rounding shift a.shift + frac_w[k] in [0, 23]): shift, clamp bound
// and rounding constant of each channel come from LDS tables behind the bias.
template <int CT, int R, bool XF, bool PC>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) conv_stem_pool_kernel(StemParams prm)
{
    constexpr int BC = CT * 32;
    constexpr int NW = 4;
    constexpr int kThreads = NW * 64;
    constexpr int kRowsFirst = R + 6;
    constexpr int MAXR = 2;                                 // 8 staged rows at a time over four wavefronts
    constexpr int kWeightBytes = R * BC * 32;
    extern __shared__ uint4 lds4[];
    const ConvArgs &a = prm.a;
    int8_t *const lds = (int8_t *)lds4;
    int *const biasl = (int *)(lds + kWeightBytes);
    int *const pc_shift = biasl + BC, *const pc_hi = biasl + 2 * BC, *const pc_badd = biasl + 3 * BC;   // PC only
    int8_t *const xin = lds + kWeightBytes + BC * 4 * (PC ? 4 : 1);

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, lh = lane >> 5;

    stem_setup<BC, R, kThreads>(a, lds, biasl, xin, kRowSlots * prm.pitch + 16);
    if constexpr (PC) {
        for (int i = tid; i < BC; i += kThreads) {
            const int sh = a.shift + a.frac_w[i];
            pc_shift[i] = sh;
            pc_hi[i] = 127 << sh;
            pc_badd[i] = sh > 0 ? (1 << (sh - 1)) - 1 : 0;
        }
    }
    __syncthreads();

    Requant rq;
    rq.init(a.shift, a.relu);
    const v4i *const wl = (const v4i *)lds;

    const int n = blockIdx.x / prm.strips;
    const int strip = blockIdx.x - n * prm.strips;
    const int t_emit = strip * prm.steps_per_strip;                 // first step whose pooled rows this strip stores
    const int t1 = min(t_emit + prm.steps_per_strip, prm.steps);
    const int t0 = strip > 0 ? t_emit - 1 : t_emit;                 // the strip's first windows reach into the step above
    typedef typename std::conditional<XF, float, int8_t>::type In;
    typedef typename std::conditional<XF, Row12f, Row12>::type Rows;
    const In *const ximg = (XF ? (const In *)prm.xf : (const In *)a.x) + (size_t)n * a.H * a.W * 3;
    auto stage = [&](int first, int count, const Rows (&rows)[MAXR]) __attribute__((always_inline)) {
        if constexpr (XF) stem_stage_rows<NW, MAXR, true>(xin, prm.pitch, prm.triples, wave, lane, first, count, rows, prm.scale);
        else stem_stage_rows<NW, MAXR, true>(xin, prm.pitch, prm.triples, wave, lane, first, count, rows);
    };

    const int j = l32 & 15, rsel = l32 >> 4;
    const int pw = 15 * wave + j;
    const int pwc = min(pw, prm.PQ - 1);                            // lanes right of the image repeat its last column, never stored
    const int colbyte = 16 * pwc + prm.off0 + 16 * lh;              // output column 2 pw; column 2 pw + 1 is 8 bytes further
    const bool stores = pw < prm.PQ && (wave == 0 || j > 0) && 15 * wave < prm.PQ;

    // rows 1 and 3 of `above` (lanes of the lower pooled row) carry, from one step to the next, the maximum over what
    // the windows of the pooled row below them take from this row: outputs (2ph+1, 2pw-1), (2ph+1, 2pw), (2ph+1, 2pw+1)
    int above[CT][16];
#pragma unroll
    for (int c = 0; c < CT; c++)
#pragma unroll
        for (int i = 0; i < 16; i++) above[c][i] = kIntMin;

    Rows pf[MAXR];
    stem_fetch_rows<NW, MAXR>(a, ximg, prm.triples, wave, lane, 8 * t0 - a.pad, 8, pf);
    stage(8 * t0 - a.pad, 8, pf);
    stem_fetch_rows<NW, MAXR>(a, ximg, prm.triples, wave, lane, 8 * t0 - a.pad + 8, kRowsFirst - 8, pf);
    stage(8 * t0 - a.pad + 8, kRowsFirst - 8, pf);
    __syncthreads();

    for (int t = t0; t < t1; t++) {
        const bool has_next = t + 1 < t1;
        const int next_first = 8 * t - a.pad + kRowsFirst;
        if (has_next) stem_fetch_rows<NW, MAXR>(a, ximg, prm.triples, wave, lane, next_first, 8, pf);
        asm volatile("" ::: "memory");          // the weights are read from LDS per use, not kept in registers across steps

        // LDS address of the lane's reduction block in input row (first row of the step) + 4 rsel + k, k = 0 .. R + 1
        const int ihb = 8 * t + 4 * rsel - a.pad + 32;
        int xaddr[R + 2];
#pragma unroll
        for (int k = 0; k < R + 2; k++) {
            const int slot = (ihb + k) & (kRowSlots - 1);
            xaddr[k] = slot * prm.pitch + 2 * (slot & 4) + colbyte;
        }
        // acc[2 * a + b][c]: output (2 ph + a, 2 pw + b), channel tile c
        v16i acc[4][CT];
#pragma unroll
        for (int c = 0; c < CT; c++)
#pragma unroll
            for (int r4 = 0; r4 < 4; r4++) {
                const int4 bv = *(const int4 *)(biasl + c * 32 + 16 * lh + 4 * r4);
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    acc[g][c][4 * r4] = bv.x; acc[g][c][4 * r4 + 1] = bv.y; acc[g][c][4 * r4 + 2] = bv.z; acc[g][c][4 * r4 + 3] = bv.w;
                }
            }
#pragma unroll
        for (int r = 0; r < R; r++) {
            asm volatile("" ::: "memory");      // one kernel row's operand reads in flight at a time
            v4i xf[4];
#pragma unroll
            for (int g = 0; g < 4; g++) {
                const uint2 *src = (const uint2 *)(xin + xaddr[2 * (g >> 1) + r] + 8 * (g & 1));
                const uint2 lo = src[0], hi = src[1];
                xf[g] = v4i{(int)lo.x, (int)lo.y, (int)hi.x, (int)hi.y};
            }
#pragma unroll
            for (int c = 0; c < CT; c++) {
                const int row = c * 32 + l32;
                const v4i wf = wl[(r * BC + row) * 2 + (lh ^ ((row >> 3) & 1))];
#pragma unroll
                for (int g = 0; g < 4; g++) acc[g][c] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf, xf[g], acc[g][c], 0, 0, 0);
            }
        }

        const int ph = 2 * t + rsel;
        const bool emit = stores && t >= t_emit && ph < prm.PP;
#pragma unroll
        for (int c = 0; c < CT; c++) {
            int m[16];
#pragma unroll
            for (int i = 0; i < 16; i++) {
                const int ee = acc[0][c][i], eo = acc[1][c][i], oe = acc[2][c][i], oo = acc[3][c][i];
                const int right = max(eo, oo);                               // what the window one column to the right takes from this lane
                int v = max(max(ee, right), oe);                             // the four positions of this lane
                // a block's first lane has no left neighbour and is handed its own value, which is in the maximum already
                v = max(v, from_left_lane(right));                           // (2ph, 2pw-1), (2ph+1, 2pw-1)
                const int below = max(max(oe, oo), from_left_lane(oo));      // what the window one row below takes from this row
                // the lanes of the upper pooled row hand `below` of this step to the lanes 16 places further (rows 0, 2 of the
                // exchange register); those hand over what they kept from the step before (rows 1, 3)
                int ex = __builtin_amdgcn_update_dpp(above[c][i], below, 0xE4 /* lanes in place */, 0x5, 0xf, false);
                ex = __builtin_amdgcn_ds_swizzle(ex, 0x401F /* lane ^ 16 */);
                m[i] = max(v, ex);                                           // (2ph-1, 2pw-1 .. 2pw+1)
                above[c][i] = below;
            }
            if (emit) {
                uint4 o;
                if constexpr (PC) {
                    uint32_t q[4];
#pragma unroll
                    for (int r4 = 0; r4 < 4; r4++) {
                        const int kr = c * 32 + 16 * lh + 4 * r4;
                        q[r4] = requant_four_per_channel(m[4 * r4], m[4 * r4 + 1], m[4 * r4 + 2], m[4 * r4 + 3], *(const int4 *)(pc_shift + kr),
                                                         *(const int4 *)(pc_hi + kr), *(const int4 *)(pc_badd + kr), a.relu);
                    }
                    o = make_uint4(q[0], q[1], q[2], q[3]);
                } else {
                    o = make_uint4(rq.fast_four(m[0], m[1], m[2], m[3]), rq.fast_four(m[4], m[5], m[6], m[7]),
                                   rq.fast_four(m[8], m[9], m[10], m[11]), rq.fast_four(m[12], m[13], m[14], m[15]));
                }
                *(uint4 *)(prm.yp + (((size_t)n * prm.PP + ph) * prm.PQ + pw) * prm.ldyp + c * 32 + 16 * lh) = o;
            }
        }
        __syncthreads();          // the step's reads of the input ring are done
        if (has_next) stage(next_first, 8, pf);
        __syncthreads();          // the next step's input rows are staged
    }
}

// LDS bytes of a staged input row.  Plain form: = 64 mod 128, so that the two output rows of an operand group (two
// input rows apart, 8-byte lane stride) fall on different banks.  Pooling form: a multiple of 64 (the rows of a lane
// group are four input rows apart; the 8-byte skew of every other group of four ring rows separates them).
int stem_pitch(const ConvArgs &a, bool pool)
{
    const int need = max(kLeftPad + 4 * a.W, 8 * (a.Q - 1) + (kLeftPad - 4 * (a.pad + (a.pad & 1))) + 32) + (pool ? 8 : 0);
    if (pool) return (need + 63) / 64 * 64;
    int pitch = (need + 127) / 128 * 128 + 64;
    if (pitch - 128 >= need) pitch -= 128;
    return pitch;
}

size_t stem_lds_bytes(const ConvArgs &a, bool pool)
{
    return (size_t)a.R * a.K * 32 + (size_t)a.K * 4 * (a.frac_w ? 4 : 1) + (size_t)kRowSlots * stem_pitch(a, pool) + (pool ? 16 : 0);
}

template <typename Kernel>
hipError_t launch_kernel(Kernel k, const StemParams &prm, int threads, size_t lds, hipStream_t st)
{
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    k<<<dim3((unsigned)(prm.a.N * prm.strips)), threads, lds, st>>>(prm);
    return hipGetLastError();
}

template <int CT, int NW>
hipError_t launch_plain(const StemParams &prm, size_t lds, hipStream_t st)
{
    if (prm.xf) {
        if (prm.a.R == 7) return launch_kernel(conv_stem_kernel<CT, NW, 7, true>, prm, NW * 64, lds, st);
        return launch_kernel(conv_stem_kernel<CT, NW, 3, true>, prm, NW * 64, lds, st);
    }
    if (prm.a.R == 7) return launch_kernel(conv_stem_kernel<CT, NW, 7, false>, prm, NW * 64, lds, st);
    return launch_kernel(conv_stem_kernel<CT, NW, 3, false>, prm, NW * 64, lds, st);
}

template <int CT, bool XF, bool PC>
hipError_t launch_pool_r(const StemParams &prm, size_t lds, hipStream_t st)
{
    if (prm.a.R == 7) return launch_kernel(conv_stem_pool_kernel<CT, 7, XF, PC>, prm, 256, lds, st);
    return launch_kernel(conv_stem_pool_kernel<CT, 3, XF, PC>, prm, 256, lds, st);
}

template <int CT>
hipError_t launch_pool(const StemParams &prm, size_t lds, hipStream_t st)
{
    if (prm.xf) return prm.a.frac_w ? launch_pool_r<CT, true, true>(prm, lds, st) : launch_pool_r<CT, true, false>(prm, lds, st);
    return prm.a.frac_w ? launch_pool_r<CT, false, true>(prm, lds, st) : launch_pool_r<CT, false, false>(prm, lds, st);
}

}  // namespace

// What the kernels take: 3 input channels, stride 2, 3 or 7 kernel rows, 32 or 64 output channels, input rows of
// at most 256 pixels and a multiple of 4, the lean epilogue (rounding shifts in [0, 23]: one for the whole layer, or - pooling
// form only - one per output channel; no accumulator dump).  Alone: output rows a multiple of 16 wide, aligned output.  pool (the output is the 3x3 / 2 /
// pad 1 max-pooled tensor): an even number of output rows and columns, at most 61 pooled columns.
bool conv_stem_supports(const ConvArgs &a, bool pool, bool from_float)
{
    if (from_float && !pool && a.K != 32) return false;   // the plain kernel has the registers for float rows at 32 channels only
    if (a.groups != 1 || a.C != 3 || a.stride != 2) return false;
    if (a.R != 3 && a.R != 7) return false;
    if (a.S + (a.pad & 1) > 8 || a.pad > 4) return false;
    if (a.K != 32 && a.K != 64) return false;
    if (a.W % 4 || a.W > 256) return false;
    if ((uintptr_t)a.x & 3) return false;
    if (a.acc_out || a.add) return false;
    if (a.frac_w) {
        // one weight format per output channel: the pooling kernel only, every channel's shift in the lean range
        if (!pool || a.shift + a.frac_w_lo < 0 || a.shift + a.frac_w_hi > 23) return false;
    } else if (a.shift < 0 || a.shift > 23) {
        return false;
    }
    if (pool) {
        if ((a.P & 1) || (a.Q & 1) || a.Q / 2 > 61) return false;
    } else {
        if (a.Q % 16) return false;
        if (!a.y || ((uintptr_t)a.y & 15) || (a.ldy & 15)) return false;
    }
    if ((long long)a.N * a.P * a.Q >= (1LL << 31) / 64) return false;
    if (stem_lds_bytes(a, pool) > (size_t)kLdsBytes / 2) return false;
    return true;
}

// yp == null: the layer itself into a.y.  Otherwise a.y is not used and yp receives the pooled tensor
// [N, (P - 1) / 2 + 1, (Q - 1) / 2 + 1, K] with ldyp bytes between pixels.  x_float (16-byte
// aligned): the input as float images, converted to codes at frac_in inside the kernel; a.x is then not read.
hipError_t launch_conv_stem(const ConvArgs &a, int8_t *yp, int ldyp, hipStream_t st, const float *x_float, int frac_in)
{
    const bool pool = yp != nullptr;
    StemParams prm;
    prm.a = a;
    prm.xf = x_float;
    prm.scale = ldexpf(1.0f, frac_in);
    prm.yp = yp;
    prm.ldyp = ldyp;
    prm.PP = (a.P - 1) / 2 + 1;
    prm.PQ = (a.Q - 1) / 2 + 1;
    prm.pitch = stem_pitch(a, pool);
    prm.off0 = kLeftPad - 4 * (a.pad + (a.pad & 1));
    prm.steps = (a.P + 3) / 4;
    prm.triples = a.W / 4;
    // enough workgroups for two per compute unit, strips of at least four steps
    int strips = max(1, (2 * kNumCU + a.N - 1) / a.N);
    strips = min(strips, max(1, prm.steps / 4));
    prm.steps_per_strip = (prm.steps + strips - 1) / strips;
    prm.strips = (prm.steps + prm.steps_per_strip - 1) / prm.steps_per_strip;
    const size_t lds = stem_lds_bytes(a, pool);
    if (pool) return a.K == 64 ? launch_pool<2>(prm, lds, st) : launch_pool<1>(prm, lds, st);
    const bool seven = ((a.Q >> 4) % 7) == 0;
    if (a.K == 64) return seven ? launch_plain<2, 7>(prm, lds, st) : launch_plain<2, 4>(prm, lds, st);
    return seven ? launch_plain<1, 7>(prm, lds, st) : launch_plain<1, 4>(prm, lds, st);
}

}  // namespace dfq
