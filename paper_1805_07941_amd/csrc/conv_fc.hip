// Dense layers over very few pixels (fully connected layers: a 1x1 convolution whose N*P*Q is a few hundred) on the
// gfx950 int8 matrix cores.
//
// The sum of Eq. 6 is the matrix product acc[k][m] = sum_c W[k][c] * X[m][c] with a long reduction axis and a small
// result: 256 x 1000 outputs over 2048 inputs is 1 GOP and 2.5 MB, microseconds of either.  What decides the time is
// how many compute units take part and how much of the reduction each has in flight: tiles large enough for operand
// reuse leave most of the chip idle, and a workgroup that shares its stages between wavefronts pays a barrier per
// 64-byte step.  Here a workgroup owns one 32 x 32 tile of the result - 256 tiles for the classifier of a batch of
// 256, one per compute unit - and its four wavefronts split the reduction axis: wavefront v takes the 64-byte steps
// v, v + 4, ... alone, with a private LDS ring of kStages steps (32 pixel rows and 32 weight rows, 4 KB, by direct
// loads awaited by the count of younger loads), so that 32 steps are on their way at once and nothing is shared
// until the end, when the partial sums meet in LDS (integer sums: exact in any order) behind the only barrier.
// The epilogue is the general one (any shift, ragged channel tail, unaligned rows, accumulator dump, one weight
// format per channel).
#include "conv_ring.hpp"

namespace dfq {

namespace {

constexpr int kWaves = 4;                          // wavefronts per workgroup, each with every fourth step
constexpr int kStages = 8;                         // ring depth per wavefront: 32 loads in flight, the counter holds 63
constexpr int kStageBytes = 64 * kStepBytes;       // 32 pixel rows, then 32 weight rows, of 64 bytes

struct FcParams {
    ConvArgs a;
    int M;            // N*P*Q
    int nsteps;       // C / 64
    int tiles_p;      // pixel tiles of 32
    unsigned x_bytes, w_bytes;
    FastDiv div_tp;
};

// at most 4 * steps loads outstanding, steps in [0, kStages - 1]
__device__ __forceinline__ void wait_steps_ahead(int steps)
{
    switch (steps) {
#define DFQ_FC_WAIT(N, V) case N: asm volatile("s_waitcnt vmcnt(" #V ")" ::: "memory"); break;
        DFQ_FC_WAIT(0, 0) DFQ_FC_WAIT(1, 4) DFQ_FC_WAIT(2, 8) DFQ_FC_WAIT(3, 12) DFQ_FC_WAIT(4, 16) DFQ_FC_WAIT(5, 20)
        DFQ_FC_WAIT(6, 24)
#undef DFQ_FC_WAIT
        default: asm volatile("s_waitcnt vmcnt(28)" ::: "memory"); break;
    }
    static_assert(kStages == 8, "the cases above cover kStages - 1 = 7 steps ahead");
}

__global__ void __launch_bounds__(kWaves * 64) conv_fc_kernel(FcParams prm)
{
    extern __shared__ uint4 lds[];   // kWaves rings of kStages stages, then the 32 bias words of the tile
    const ConvArgs &a = prm.a;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const int l32 = lane & 31, lh = lane >> 5;
    // this wavefront's steps: wave, wave + kWaves, ...
    const int nmine = prm.nsteps > wave ? (prm.nsteps - wave + kWaves - 1) / kWaves : 0;

    // Workgroup ids are dealt round-robin to the 8 XCDs; renumbered so that each XCD owns a contiguous range, the pixel
    // tiles of one channel tile - which read the same weight rows - share an L2.
    const int G = gridDim.x;
    int lb = blockIdx.x;
    {
        const int per = G / 8, rem = G % 8, xcd = lb % 8, idx = lb / 8;
        lb = (xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per) + idx;
    }
    const int ct = fastdiv(lb, prm.div_tp);
    const int pt = lb - ct * prm.tiles_p;
    const int m0 = pt * 32, k0 = ct * 32;

    const v4i xrsrc = make_rsrc(a.x, prm.x_bytes);
    const v4i wrsrc = make_rsrc(a.w, prm.w_bytes);
    const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) char *)(char *)&lds[0];
    const unsigned ring_base = lds_base + (unsigned)(wave * kStages * kStageBytes);
    const unsigned bias_base = lds_base + (unsigned)(kWaves * kStages * kStageBytes);

    // A wavefront-wide load covers 16 rows of a stage: lane l supplies row l/4, physical piece l%4, which holds logical
    // piece (l%4) ^ ((row>>2)&3), so that 16 consecutive rows put any one logical piece on 16 different bank groups.
    const int lrow = lane >> 2;
    const unsigned lpb = (unsigned)((lane & 3) ^ ((lane >> 4) & 3)) * 16u;
    unsigned xoff[2], woff[2];       // byte offset of the lane's row (+ piece), or out of range: zeros arrive
#pragma unroll
    for (int j = 0; j < 2; j++) {
        const int m = m0 + 16 * j + lrow;
        xoff[j] = m < prm.M ? (unsigned)(m * a.C) + lpb : kOutOfRange;
        // LDS row i = 8g + 4h + e of the weight rows receives channel 16h + 4g + e: the matrix instruction then leaves
        // 16 consecutive channels in each lane
        const int rr = 16 * j + lrow;
        const int k = k0 + 16 * ((rr >> 2) & 1) + 4 * (rr >> 3) + (rr & 3);
        woff[j] = k < a.K ? (unsigned)(k * a.C) + lpb : kOutOfRange;
    }
    // this wavefront's i-th step into stage `stage` of its ring
    auto issue = [&](int i, int stage) __attribute__((always_inline)) {
        const unsigned base = (unsigned)__builtin_amdgcn_readfirstlane((int)(ring_base + (unsigned)(stage * kStageBytes)));
        const unsigned step_off = (unsigned)(wave + kWaves * i) * kStepBytes;
        load_piece_to_lds(xoff[0] + step_off, xrsrc, base);
        load_piece_to_lds(xoff[1] + step_off, xrsrc, base + 1024u);
        load_piece_to_lds(woff[0] + step_off, wrsrc, base + 2048u);
        load_piece_to_lds(woff[1] + step_off, wrsrc, base + 3072u);
    };
    // The tile's bias travels the same way, ahead of everything else of the first wavefront (loads complete in order,
    // so it has arrived when that wavefront's first step has; channels past K are outside the buffer and read as
    // zero): an ordinary load would be tracked by the compiler, whose wait for it would also wait for every younger
    // load of the ring.
    if (a.b && wave == 0) {
        const v4i brsrc = make_rsrc(a.b, (unsigned)a.K * 4u);
        load_piece_to_lds(lane < 8 ? (unsigned)(k0 * 4 + 16 * lane) : kOutOfRange, brsrc,
                          (unsigned)__builtin_amdgcn_readfirstlane((int)bias_base));
    }
    const int ahead0 = min(nmine, kStages);
    for (int i = 0; i < ahead0; i++) issue(i, i);

    v16i acc;
#pragma unroll
    for (int r = 0; r < 16; r++) acc[r] = 0;

    const v4i *rows = (const v4i *)lds + wave * kStages * (kStageBytes / 16);
    const int swz = (l32 >> 2) & 3;
    int stage = 0;
    for (int i = 0; i < nmine; i++) {
        const int ahead = nmine - 1 - i;           // steps issued behind this one, capped by the ring
        if (ahead >= kStages - 1) asm volatile("s_waitcnt vmcnt(28)" ::: "memory");
        else wait_steps_ahead(ahead);
        const v4i *st = rows + stage * (kStageBytes / 16);
        const v4i x0 = st[l32 * kPieces + (lh ^ swz)], x1 = st[l32 * kPieces + ((2 + lh) ^ swz)];
        const v4i w0 = st[(32 + l32) * kPieces + (lh ^ swz)], w1 = st[(32 + l32) * kPieces + ((2 + lh) ^ swz)];
        acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(w0, x0, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(w1, x1, acc, 0, 0, 0);
        // the stage is free once its operands are in registers
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        if (i + kStages < nmine) issue(i + kStages, stage);
        stage = stage + 1 == kStages ? 0 : stage + 1;
    }
    settle_accumulators<1>(&acc);

    // The partial sums of wavefronts 1 .. kWaves-1 go to the start of their own rings (every load into them has been
    // awaited), register r of lane l at word 64 * r + l; the first wavefront adds them to its own.
    int *part = (int *)lds + wave * kStages * (kStageBytes / 4);
    if (wave != 0) {
#pragma unroll
        for (int r = 0; r < 16; r++) part[64 * r + lane] = acc[r];
    }
    __syncthreads();
    if (wave != 0) return;
#pragma unroll
    for (int v = 1; v < kWaves; v++) {
        const int *other = (const int *)lds + v * kStages * (kStageBytes / 4);
#pragma unroll
        for (int r = 0; r < 16; r++) acc[r] += other[64 * r + lane];
    }
    // register r of a lane belongs to channel k0 + 16 * lh + r
    if (a.b) {
        const int *bias = (const int *)(lds + kWaves * kStages * (kStageBytes / 16)) + 16 * lh;
#pragma unroll
        for (int r = 0; r < 16; r++) acc[r] += bias[r];
    }
    const int m = m0 + l32, kc = k0 + 16 * lh;
    if (m < prm.M && kc < a.K) store_tile_lane_general(acc, a, a.shift, a.relu, m, kc);
}

}  // namespace

bool conv_fc_supports(const ConvArgs &a)
{
    if (a.groups != 1 || a.R != 1 || a.S != 1 || a.stride != 1 || a.pad != 0 || a.add) return false;
    if (a.C % kStepBytes) return false;
    const long long M = (long long)a.N * a.P * a.Q;
    if (M > 1024) return false;
    // 32-bit byte offsets with the top bit reserved for "out of range"
    if (M * a.C >= (1LL << 31) || (long long)a.K * a.C >= (1LL << 31)) return false;
    if (((M + 31) / 32) * (((long long)a.K + 31) / 32) > 0x7fffffffLL) return false;
    if (((uintptr_t)a.x & 15) || ((uintptr_t)a.w & 15)) return false;
    return true;
}

hipError_t launch_conv_fc(const ConvArgs &a, hipStream_t st)
{
    FcParams prm;
    prm.a = a;
    prm.M = a.N * a.P * a.Q;
    prm.nsteps = a.C / kStepBytes;
    prm.tiles_p = (prm.M + 31) / 32;
    prm.x_bytes = (unsigned)((long long)prm.M * a.C);
    prm.w_bytes = (unsigned)((long long)a.K * a.C);
    prm.div_tp = make_fastdiv(prm.tiles_p);
    const int grid = prm.tiles_p * ((a.K + 31) / 32);
    if (grid <= 0) return hipSuccess;
    constexpr size_t lds_bytes = (size_t)kWaves * kStages * kStageBytes + 1024;
    static const hipError_t attr = hipFuncSetAttribute((const void *)conv_fc_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                                       (int)lds_bytes);
    if (attr != hipSuccess) return attr;
    conv_fc_kernel<<<(unsigned)grid, kWaves * 64, lds_bytes, st>>>(prm);
    return hipGetLastError();
}

}  // namespace dfq
