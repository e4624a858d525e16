// Grouped quantized convolution (1 < groups, C/groups = K/groups in {4, 8, 16, 32, 64}) on the int8 matrix cores.
//
// A group's reduction (Eq. 6 over R * S * C/groups terms) is far shorter than a 64-byte step of the matrix
// instructions, but 64 consecutive channels hold whole groups, and the sum over a group equals the sum over those 64
// channels with the weights of the other groups' channels set to zero: the layer is C/64 independent dense 64 -> 64
// convolutions with block-diagonal weights.  The zeros cost matrix work (16x for groups of 4), which this chip has to
// spare: measured 3-4x faster than one output per lane with dot products on the vector ALU.
//
// One workgroup of four wavefronts (64 pixels x 32 channels each) computes 128 pixels x the 64 channels of one such block.
// A wavefront's weights - for every kernel tap 32 rows x 64 bytes, zeros included - stay in registers for the whole tile
// (8 per tap and lane, fetched once at the start, the zeros never loaded); the input streams through a ring of LDS
// stages filled by direct global -> LDS loads, one 64-byte step per kernel tap, as in the dense kernels (rows of 64
// bytes, 16-byte pieces XOR-swizzled); three workgroups share a compute unit, so that one's loads and matrix
// instructions run under another's epilogue.  Epilogue in registers: bias as
// start value, ReLU, rounding shift, clamp (the lean form only; the launcher falls back otherwise).
#include "conv_ring.hpp"

namespace dfq {

namespace {

constexpr int kSgBP = 128;          // pixels per tile

struct SgParams {
    ConvArgs a;
    int M;                  // N * P * Q output pixels
    int Cg;                 // channels per group
    int nitems;             // R * S
    int blocks_c;           // C / 64
    unsigned x_bytes;
    FastDiv div_q, div_p, div_bc;
};

template <int NTAPS, int NSTAGES, int OCC>
__global__ void __launch_bounds__(256, OCC) conv_sg_kernel(SgParams prm)
{
    constexpr int BP = kSgBP;
    constexpr int XJ = BP / 64;                            // 16-row chunks per wavefront and step
    constexpr int PT = 2;                                  // 32-pixel tiles per wavefront (64 pixels x 32 channels)
    extern __shared__ uint4 lds[];                         // [NSTAGES * BP input rows], 4 pieces per row
    const ConvArgs &a = prm.a;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    constexpr int nitems = NTAPS;

    // tile of this workgroup: ids are dealt round-robin to the 8 XCDs; renumbered so that each XCD owns a contiguous
    // range (the channel blocks of one pixel tile read the same input lines)
    const int G = gridDim.x;
    int lb = blockIdx.x;
    {
        const int per = G / 8, rem = G % 8, xcd = lb % 8, idx = lb / 8;
        lb = (xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per) + idx;
    }
    const int pt = fastdiv(lb, prm.div_bc);
    const int cb = lb - pt * prm.blocks_c;                 // block of 64 channels

    const v4i x_rsrc = make_rsrc(a.x, prm.x_bytes);
    const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) char *)(char *)&lds[0];

    // ---- input producer: lane l of a wavefront-wide load supplies row l/4 of a 16-row chunk, physical piece l%4, which
    // holds logical piece (l%4) ^ ((row>>2)&3)
    const int lrow = lane >> 2;
    const int lp = (lane & 3) ^ ((lane >> 4) & 3);
    int ih0[XJ], iw0[XJ], xbase[XJ];
#pragma unroll
    for (int j = 0; j < XJ; j++) {
        const int m = pt * BP + 16 * (wave + 4 * j) + lrow;
        if (m < prm.M) {
            const int t = fastdiv(m, prm.div_q);
            const int oq = m - t * a.Q;
            const int n = fastdiv(t, prm.div_p);
            const int op = t - n * a.P;
            ih0[j] = op * a.stride - a.pad;
            iw0[j] = oq * a.stride - a.pad;
            xbase[j] = ((n * a.H + ih0[j]) * a.W + iw0[j]) * a.C + cb * 64 + lp * 16;
        } else {
            ih0[j] = -(1 << 28);      // no kernel row is inside the image
            iw0[j] = 0;
            xbase[j] = 0;
        }
    }
    int p_r = 0, p_s = 0;             // kernel row and column of the step fetched next
    auto issue = [&](int stage) __attribute__((always_inline)) {
        const int tap_off = (p_r * a.W + p_s) * a.C;
        const unsigned sbase = lds_base + (unsigned)(stage * BP) * 64u + (unsigned)wave * 1024u;
#pragma unroll
        for (int j = 0; j < XJ; j++) {
            const bool ok = (unsigned)(ih0[j] + p_r) < (unsigned)a.H && (unsigned)(iw0[j] + p_s) < (unsigned)a.W;
            const unsigned off = ok ? (unsigned)(xbase[j] + tap_off) : kOutOfRange;
            load_piece_to_lds(off, x_rsrc, (unsigned)__builtin_amdgcn_readfirstlane((int)(sbase + (unsigned)(j * 4096))));
        }
        if (++p_s == a.S) {
            p_s = 0;
            ++p_r;
        }
    };
#pragma unroll
    for (int i = 0; i < NSTAGES; i++)
        if (i < nitems) issue(i);

    // ---- consumer
    const int wp0 = (wave & 1) * 64, wc0 = (wave >> 1) * 32;
    const int l32 = lane & 31, lh = lane >> 5;
    const int swz = (l32 >> 2) & 3;
    const int kc = cb * 64 + wc0 + 16 * lh;                // the lane's 16 output channels
    v16i acc[PT];
    {
        int bias[16];
#pragma unroll
        for (int r4 = 0; r4 < 4; r4++) {
            const int4 bv = a.b ? *(const int4 *)(a.b + kc + 4 * r4) : make_int4(0, 0, 0, 0);
            bias[4 * r4 + 0] = bv.x;
            bias[4 * r4 + 1] = bv.y;
            bias[4 * r4 + 2] = bv.z;
            bias[4 * r4 + 3] = bv.w;
        }
#pragma unroll
        for (int p = 0; p < PT; p++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[p][r] = bias[r];
    }
    // ---- weights: the matrix instruction's first operand for tap t and half kk is, in lane (l32, lh), bytes
    // 32 kk + 16 lh .. + 15 of row l32 of the wavefront's 32 x 64 slab.  Row i = 8g + 4h + e holds channel 16h + 4g + e
    // (so that the instruction leaves 16 consecutive channels in each lane); of its 64 bytes only the channels of that
    // output channel's own group are weights, the rest zeros.
    v4i wreg[NTAPS][2];
    {
        const int kl = wc0 + 16 * ((l32 >> 2) & 1) + 4 * (l32 >> 3) + (l32 & 3);        // channel within the block of 64
        const int c_lo = (kl / prm.Cg) * prm.Cg;                                       // first channel of its group, within the block
        const uint32_t *wk = (const uint32_t *)(a.w + (size_t)(cb * 64 + kl) * NTAPS * prm.Cg);
#pragma unroll
        for (int t = 0; t < NTAPS; t++)
#pragma unroll
            for (int kk = 0; kk < 2; kk++)
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    const int c = 32 * kk + 16 * lh + 4 * e - c_lo;                    // channel within the group, if inside
                    wreg[t][kk][e] = (c >= 0 && c < prm.Cg) ? (int)wk[(t * prm.Cg + c) >> 2] : 0;
                }
    }
    struct Half {
        v4i x[PT];
    };
    Half f0, f1;
    auto read_half = [&](Half &f, int kk, int stage) __attribute__((always_inline)) {
        const v4i *base = (const v4i *)lds;
        const int g = (kk * 2 + lh) ^ swz;
#pragma unroll
        for (int p = 0; p < PT; p++) f.x[p] = base[(stage * BP + wp0 + p * 32 + l32) * kPieces + g];
    };
    auto mfma_half = [&](const Half &f, const v4i &w) __attribute__((always_inline)) {
#pragma unroll
        for (int p = 0; p < PT; p++) acc[p] = __builtin_amdgcn_mfma_i32_32x32x32_i8(w, f.x[p], acc[p], 0, 0, 0);
    };
    auto ring_barrier = [&]() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };

    // step 0 has landed when at most the loads of the steps issued after it are outstanding
    wait_ahead<XJ>(min(NSTAGES, nitems) - 1);
    ring_barrier();
    read_half(f0, 0, 0);
    read_half(f1, 1, 0);
#pragma unroll
    for (int it = 0; it < nitems; it++) {
        const int stage = it % NSTAGES, next = (it + 1) % NSTAGES;
        const bool has_next = it + 1 < nitems;
        mfma_half(f0, wreg[it][0]);
        __builtin_amdgcn_sched_barrier(0);
        if (has_next) {
            wait_ahead<XJ>(max(min(NSTAGES - 2, nitems - it - 2), 0));      // step it+1: the steps behind it may still be in flight
            ring_barrier();           // every wavefront has read step it: its stage may be refilled
            read_half(f0, 0, next);
        }
        __builtin_amdgcn_sched_barrier(0);
        mfma_half(f1, wreg[it][1]);
        __builtin_amdgcn_sched_barrier(0);
        if (has_next) {
            if (it + NSTAGES < nitems) issue(stage);
            read_half(f1, 1, next);
        }
        __builtin_amdgcn_sched_barrier(0);
    }

    // ---- epilogue: register r of a lane belongs to channel kc + r of pixel m
    Requant rq;
    rq.init(a.shift, a.relu);
    settle_accumulators<PT>(&acc[0]);
#pragma unroll
    for (int p = 0; p < PT; p++) {
        const int m = pt * BP + wp0 + p * 32 + l32;
        const uint4 out = requant_tile_lane_fast(acc[p], rq);
        if (m < prm.M) *(uint4 *)(a.y + (size_t)m * a.ldy + kc) = out;
    }
}

template <int NTAPS, int NSTAGES, int OCC>
hipError_t launch_sg(const SgParams &prm, long long tiles, hipStream_t st)
{
    constexpr size_t lds_bytes = (size_t)NSTAGES * kSgBP * 64;
    static_assert(lds_bytes * OCC <= (size_t)kLdsBytes, "the workgroups of a compute unit share its LDS");
    conv_sg_kernel<NTAPS, NSTAGES, OCC><<<(unsigned)tiles, 256, lds_bytes, st>>>(prm);
    return hipGetLastError();
}

}  // namespace

bool conv_sg_supports(const ConvArgs &a)
{
    if (a.groups < 2 || a.C % 64 || a.K != a.C) return false;
    const int Cg = a.C / a.groups;
    if (Cg != 4 && Cg != 8 && Cg != 16 && Cg != 32 && Cg != 64) return false;
    const int taps = a.R * a.S;
    if ((taps != 1 && taps != 4 && taps != 6 && taps != 9) || a.stride < 1) return false;      // the tap counts the kernel is built for
    if (a.frac_w || a.add || a.acc_out || !a.y) return false;
    if (a.shift < 0 || a.shift > 23) return false;                                  // the lean epilogue
    if ((a.ldy & 15) || ((uintptr_t)a.y & 15) || ((uintptr_t)a.x & 15) || ((uintptr_t)a.w & 3) || (a.b && ((uintptr_t)a.b & 15))) return false;
    if ((long long)a.N * a.H * a.W * a.C >= (1LL << 31) - (1 << 24)) return false;   // 31-bit byte offsets into the input
    if ((long long)a.N * a.P * a.Q >= (1LL << 31) - 512) return false;
    if ((long long)a.N * a.P * a.Q * a.ldy >= (1LL << 40)) return false;
    const long long tiles = (((long long)a.N * a.P * a.Q + kSgBP - 1) / kSgBP) * (a.C / 64);
    return tiles <= 0x7fffffffLL;
}

hipError_t launch_conv_sg(const ConvArgs &a, hipStream_t st)
{
    SgParams prm;
    prm.a = a;
    const long long M = (long long)a.N * a.P * a.Q;
    prm.M = (int)M;
    prm.Cg = a.C / a.groups;
    prm.nitems = a.R * a.S;
    prm.blocks_c = a.C / 64;
    prm.x_bytes = (unsigned)((long long)a.N * a.H * a.W * a.C);
    prm.div_q = make_fastdiv(a.Q);
    prm.div_p = make_fastdiv(a.P);
    prm.div_bc = make_fastdiv(prm.blocks_c);
    const long long tiles = ((M + kSgBP - 1) / kSgBP) * prm.blocks_c;
    switch (prm.nitems) {
        case 1: return launch_sg<1, 1, 3>(prm, tiles, st);
        case 4: return launch_sg<4, 3, 3>(prm, tiles, st);
        case 6: return launch_sg<6, 4, 3>(prm, tiles, st);
        default: return launch_sg<9, 4, 3>(prm, tiles, st);
    }
}

}  // namespace dfq
