// Depthwise 3 x 3 quantized convolution (groups == C == K, C a multiple of 32) with the products on the int8 matrix cores.
//
// Every output channel sums nine products of its own input channel (Eq. 6 with nine terms): no contraction over
// channels, and on the vector ALU the layer costs about 23 instructions per output - index arithmetic, byte transposes,
// dot products, rounding - which, not memory, bounds it.  v_mfma_i32_16x16x64_i8 multiplies a 16 x 64 by a 64 x 16 matrix;
// take 16 channels as the rows of the first and 16 neighbouring output pixels of an image row as the columns of the
// second, and let the 64 entries of the reduction axis be 4 kernel taps x 16 channels: the second operand's lane
// (pixel q, tap t) then supplies the 16 channel bytes of input pixel q + (offset of tap t) - a plain 16-byte LDS read - and
// the first operand is diagonal in the channel, row c holding the weight of (channel c, tap t) at position 16 t + c and
// zeros elsewhere.  Three such instructions (taps 0-3, 4-7, 8) give the nine-tap sums of 16 channels x 16 pixels, each
// lane ending with four neighbouring channels of one pixel - one packed word of the output.  15 of 16 products are with
// zeros, which the matrix pipe has to spare; what is left on the vector ALU is the read addresses, the rounding and the
// stores, about a third of the instructions of the plain form.
//
// A workgroup of four wavefronts takes 8 output rows x 16 output columns x CB = 64 channels of one image (CB = 32 when C is
// not a multiple of 64).  Its input patch (with the kernel's halo; padding and everything outside the image arrive as
// zeros) is fetched once by direct global -> LDS loads, CB bytes per input pixel, laid out as 64-byte LDS rows with the
// 16-byte pieces XOR-swizzled by (row >> 2) & 3, so that 16 neighbouring pixels' reads of the same channel quarter fall
// into different banks.  The diagonal operands of all taps
// stay in registers.  Epilogue as in the other kernels: bias as start value, ReLU, rounding shift, clamp (lean form only;
// the launcher keeps the vector-ALU kernel for everything else).
#include "conv_ring.hpp"

namespace dfq {

namespace {

constexpr int kDwmTH = 8, kDwmTW = 16;

struct DwmParams {
    ConvArgs a;
    int tiles_x, tiles_y, blocks_c;
    int patches;              // N * tiles_y * tiles_x (streaming form)
    unsigned x_bytes, y_bytes;
    FastDiv div_bc, div_tx, div_ty;
};

// The per-lane constants of a workgroup's channel block: the diagonal first operands of the three tap groups, the row
// offsets of the lane's taps inside a patch, and the bias of the lane's output channels.
template <int ST, int CB>
struct DwmLane {
    static constexpr int NQ = CB / 16;
    static constexpr int IW = (kDwmTW - 1) * ST + 3;
    v4i wd[3][NQ];
    int roff[3];
    v4i bias[NQ];

    __device__ __forceinline__ void init(const ConvArgs &a, int cb, int lane)
    {
        const int l16 = lane & 15, lq = lane >> 4;
        const int wsel = l16 >> 2;         // which word of a first operand holds the lane's weight
        // for tap group g and channel quarter cq the lane holds 16 bytes of row (channel) l16 at reduction positions
        // 16 lq .. 16 lq + 15, i.e. tap 4 g + lq: the weight at byte l16, zeros elsewhere
#pragma unroll
        for (int g = 0; g < 3; g++) {
            const int tap = 4 * g + lq;
            const int tt = min(tap, 8);    // taps 9..11 do not exist: zero weights, any valid row
            const int r = tt / 3, s = tt - 3 * r;
            roff[g] = r * IW + s;
#pragma unroll
            for (int cq = 0; cq < NQ; cq++) {
                const int ch = cb * CB + 16 * cq + l16;
                const int wv = tap < 9 ? (int)(uint8_t)a.w[(size_t)ch * 9 + tap] : 0;
                const int word = wv << (8 * (l16 & 3));
#pragma unroll
                for (int e = 0; e < 4; e++) wd[g][cq][e] = (e == wsel) ? word : 0;
            }
        }
        // the lane's outputs: channels kc .. kc + 3 of every quarter
#pragma unroll
        for (int cq = 0; cq < NQ; cq++) {
            const int kc = cb * CB + 16 * cq + 4 * lq;
            const int4 bv = a.b ? *(const int4 *)(a.b + kc) : make_int4(0, 0, 0, 0);
            bias[cq][0] = bv.x;
            bias[cq][1] = bv.y;
            bias[cq][2] = bv.z;
            bias[cq][3] = bv.w;
        }
    }

    // Output row oy (patch row oyl) of the patch at `rows`: nine-tap sums of 16 pixels x CB channels, rounded; the lane's
    // four packed words belong to four different 16-byte pieces of its pixel's output bytes: exchanged through the
    // wavefront's 1 KB LDS slot, so that every lane holds one whole piece.  Returns that piece (lanes below 16 * NQ:
    // pixel lane / NQ, piece lane % NQ).
    __device__ __forceinline__ uint4 row(const v4i *rows, uint32_t *slot, const Requant &rq, int oyl, int lane) const
    {
        const int l16 = lane & 15, lq = lane >> 4;
        const int base = oyl * ST * IW + l16 * ST;
        v4i acc[NQ];
#pragma unroll
        for (int cq = 0; cq < NQ; cq++) acc[cq] = bias[cq];
#pragma unroll
        for (int g = 0; g < 3; g++) {
            const int p0 = (base + roff[g]) * NQ;                    // linear piece index of the pixel's first quarter
#pragma unroll
            for (int cq = 0; cq < NQ; cq++) {
                const int L = p0 + cq, r = L >> 2;
                const v4i xv = rows[r * kPieces + ((L & 3) ^ ((r >> 2) & 3))];
                acc[cq] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wd[g][cq], xv, acc[cq], 0, 0, 0);
            }
        }
        settle_accumulators<NQ>(&acc[0]);
#pragma unroll
        for (int cq = 0; cq < NQ; cq++) slot[l16 * (CB / 4) + 4 * cq + lq] = rq.fast_four(acc[cq][0], acc[cq][1], acc[cq][2], acc[cq][3]);
        return ((const uint4 *)slot)[lane & (16 * NQ - 1)];         // same wavefront: program order suffices
    }
};

template <int ST, int CB>
__global__ void __launch_bounds__(256) conv_dwm_kernel(DwmParams prm)
{
    constexpr int NQ = CB / 16;                                        // 16-channel quarters (16-byte pieces) per pixel
    constexpr int TH = kDwmTH, TW = kDwmTW;
    constexpr int IH = (TH - 1) * ST + 3, IW = (TW - 1) * ST + 3;      // input patch
    constexpr int PIX = IH * IW;                                       // input pixels of the patch, CB bytes each
    constexpr int CHUNKS = (PIX * NQ + 63) / 64;                       // 64 pieces (16 LDS rows) per wavefront-wide load
    extern __shared__ uint4 lds[];
    const ConvArgs &a = prm.a;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // workgroup -> (image, tile row, tile column, block of 64 channels), channel blocks fastest: neighbouring workgroups
    // read neighbouring 64-byte segments of the same pixels
    // (ids are dealt round-robin to the 8 XCDs; renumbered so that each XCD owns a contiguous range: the channel blocks
    // of a patch and neighbouring patches then meet in one L2)
    int t = blockIdx.x;
    {
        const int G = gridDim.x, per = G / 8, rem = G % 8, xcd = t % 8, idx = t / 8;
        t = (xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per) + idx;
    }
    int q1 = fastdiv(t, prm.div_bc);
    const int cb = t - q1 * prm.blocks_c;
    t = q1;
    q1 = fastdiv(t, prm.div_tx);
    const int ox0 = (t - q1 * prm.tiles_x) * TW;
    t = q1;
    const int n = fastdiv(t, prm.div_ty);
    const int oy0 = (t - n * prm.tiles_y) * TH;

    // ---- the input patch: lane l of a load supplies row l/4 of a 16-row chunk, physical piece l%4 = logical piece (l%4) ^ ((row>>2)&3)
    {
        const v4i x_rsrc = make_rsrc(a.x, prm.x_bytes);
        const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) char *)(char *)&lds[0];
        const int lp = (lane & 3) ^ ((lane >> 4) & 3);
        const int gy0 = oy0 * ST - a.pad, gx0 = ox0 * ST - a.pad;
        for (int c = wave; c < CHUNKS; c += 4) {
            const int piece = 4 * (16 * c + (lane >> 2)) + lp;          // linear index of the lane's logical piece: pixel * NQ + quarter
            const int j = piece / NQ, qq = piece - j * NQ;
            const int iy = j / IW, ix = j - iy * IW;
            const int gy = gy0 + iy, gx = gx0 + ix;
            const bool ok = j < PIX && (unsigned)gy < (unsigned)a.H && (unsigned)gx < (unsigned)a.W;
            const unsigned off = ok ? (unsigned)(((n * a.H + gy) * a.W + gx) * a.C + cb * CB + qq * 16) : kOutOfRange;
            load_piece_to_lds(off, x_rsrc, (unsigned)__builtin_amdgcn_readfirstlane((int)(lds_base + (unsigned)c * 1024u)));
        }
    }

    DwmLane<ST, CB> ln;
    ln.init(a, cb, lane);
    Requant rq;
    rq.init(a.shift, a.relu);

    wait_loads<0>();
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");

    const v4i *rows = (const v4i *)lds;
    uint32_t *slot = (uint32_t *)(lds + CHUNKS * 64) + wave * 256;
    for (int oyl = wave; oyl < TH; oyl += 4) {
        const int oy = oy0 + oyl;
        if (oy >= a.P) break;          // (uniform: the wavefront's row)
        const uint4 piece = ln.row(rows, slot, rq, oyl, lane);
        if (lane < 16 * NQ) {
            const int px = ox0 + lane / NQ;
            if (px < a.Q) *(uint4 *)(a.y + ((size_t)(n * a.P + oy) * a.Q + px) * a.ldy + cb * CB + 16 * (lane % NQ)) = piece;
        }
    }
}

// The streaming form for stride 1: a workgroup keeps its channel block - the diagonal operands and the bias stay in
// registers - and walks over every (G / blocks_c)-th patch of the layer with two patch buffers: the loads of the next
// patch are issued right behind the barrier that releases the buffer and fly while the current patch is multiplied, so
// that what a workgroup waits for is a patch requested one whole iteration earlier.  One barrier per patch: behind it
// every wavefront's share of the patch has landed (each waited for its own loads: everything older than the stores of
// its previous iteration, which are counted) and nobody still reads the other buffer.  Stores go through a buffer
// resource, one instruction per output row whatever the lanes' positions, so that the count is exact.
template <int CB>
__global__ void __launch_bounds__(256) conv_dwm_stream_kernel(DwmParams prm)
{
    constexpr int ST = 1;
    constexpr int NQ = CB / 16;
    constexpr int TH = kDwmTH, TW = kDwmTW;
    constexpr int IH = (TH - 1) * ST + 3, IW = (TW - 1) * ST + 3;
    constexpr int PIX = IH * IW;
    constexpr int CHUNKS = (PIX * NQ + 63) / 64;
    constexpr int MYCH = (CHUNKS + 3) / 4;                             // chunks per wavefront: wave, wave + 4, ...
    extern __shared__ uint4 lds[];                                     // two patches, then one exchange slot per wavefront
    const ConvArgs &a = prm.a;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // workgroup -> channel block (fastest) and first patch; ids renumbered so that each XCD owns a contiguous range: the
    // channel blocks of a patch and neighbouring patches meet in one L2.  The grid is a multiple of blocks_c.
    const int G = gridDim.x;
    int lb = blockIdx.x;
    {
        const int per = G / 8, rem = G % 8, xcd = lb % 8, idx = lb / 8;
        lb = (xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per) + idx;
    }
    const int wg = fastdiv(lb, prm.div_bc);
    const int cb = lb - wg * prm.blocks_c;
    const int nwg = fastdiv(G, prm.div_bc);
    // contiguous, equally long runs of patches: an XCD then owns one contiguous part of the layer, as in the kernels
    // before and behind it (with every nwg-th patch instead, the pointwise layer behind a 14 x 14 layer was 3 us slower)
    const int sp0 = (int)((long long)wg * prm.patches / nwg);
    const int sp_end = (int)((long long)(wg + 1) * prm.patches / nwg);
    constexpr int sp_step = 1;

    const v4i x_rsrc = make_rsrc(a.x, prm.x_bytes);
    const __amdgpu_buffer_rsrc_t y_rsrc = __builtin_amdgcn_make_buffer_rsrc(a.y, 0, (int)prm.y_bytes, 0x00020000);
    const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) char *)(char *)&lds[0];
    // the lane's pieces of a patch: lane l of a load supplies row l/4 of a 16-row chunk, physical piece l%4 = logical
    // piece (l%4) ^ ((row>>2)&3)
    int piy[MYCH], pix[MYCH];
    unsigned pcoff[MYCH];
    {
        const int lp = (lane & 3) ^ ((lane >> 4) & 3);
#pragma unroll
        for (int i = 0; i < MYCH; i++) {
            const int c = wave + 4 * i;
            const int piece = 4 * (16 * c + (lane >> 2)) + lp;          // pixel * NQ + quarter
            const int j = piece / NQ, qq = piece - j * NQ;
            piy[i] = j < PIX ? j / IW : -(1 << 20);                     // past the patch: no row of any image
            pix[i] = j - (j / IW) * IW;
            pcoff[i] = (unsigned)(cb * CB + qq * 16);
        }
    }
    struct Pos { int n, oy0, ox0; };
    auto locate = [&](int sp) __attribute__((always_inline)) {
        Pos p;
        int q1 = fastdiv(sp, prm.div_tx);
        p.ox0 = (sp - q1 * prm.tiles_x) * TW;
        p.n = fastdiv(q1, prm.div_ty);
        p.oy0 = (q1 - p.n * prm.tiles_y) * TH;
        return p;
    };
    auto issue = [&](const Pos &p, int buf) __attribute__((always_inline)) {
        const int gy0 = p.oy0 * ST - a.pad, gx0 = p.ox0 * ST - a.pad;
#pragma unroll
        for (int i = 0; i < MYCH; i++) {
            const int c = wave + 4 * i;
            if (c < CHUNKS) {                                           // (uniform)
                const int gy = gy0 + piy[i], gx = gx0 + pix[i];
                const bool ok = (unsigned)gy < (unsigned)a.H && (unsigned)gx < (unsigned)a.W;
                const unsigned off = ok ? (unsigned)(((p.n * a.H + gy) * a.W + gx) * a.C) + pcoff[i] : kOutOfRange;
                load_piece_to_lds(off, x_rsrc, (unsigned)__builtin_amdgcn_readfirstlane((int)(lds_base + (unsigned)(buf * CHUNKS + c) * 1024u)));
            }
        }
    };

    int sp = sp0;
    Pos cur = locate(min(sp, prm.patches - 1));
    if (sp < sp_end) issue(cur, 0);
    DwmLane<ST, CB> ln;
    ln.init(a, cb, lane);
    Requant rq;
    rq.init(a.shift, a.relu);
    uint32_t *slot = (uint32_t *)(lds + 2 * CHUNKS * 64) + wave * 256;
    const unsigned lane_yoff = lane < 16 * NQ ? (unsigned)((lane / NQ) * a.ldy + cb * CB + 16 * (lane % NQ)) : kOutOfRange;

    int nst = 0;                       // stores this wavefront issued in the previous iteration
    for (int k = 0; sp < sp_end; k++, sp += sp_step) {
        // this patch's loads are older than those stores, and nothing else is younger
        switch (nst) {
            case 0: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
            case 1: asm volatile("s_waitcnt vmcnt(1)" ::: "memory"); break;
            default: asm volatile("s_waitcnt vmcnt(2)" ::: "memory"); break;
        }
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        const int buf = k & 1;
        Pos next = cur;
        if (sp + sp_step < sp_end) {
            next = locate(sp + sp_step);
            issue(next, buf ^ 1);
        }
        const v4i *rows = (const v4i *)lds + buf * CHUNKS * 64;
        nst = 0;
        for (int oyl = wave; oyl < TH; oyl += 4) {
            const int oy = cur.oy0 + oyl;
            if (oy >= a.P) break;      // (uniform: the wavefront's row)
            const uint4 piece = ln.row(rows, slot, rq, oyl, lane);
            // pixels past the end of the image row: outside the buffer, nothing is stored
            const bool live = lane < 16 * NQ && cur.ox0 + lane / NQ < a.Q;
            const unsigned off = live ? lane_yoff + (unsigned)(((cur.n * a.P + oy) * a.Q + cur.ox0) * a.ldy) : kOutOfRange;
            store_piece(piece, off, y_rsrc);
            nst++;
        }
        cur = next;
    }
}

template <int ST, int CB>
hipError_t launch_dwm(const DwmParams &prm, long long blocks, hipStream_t st)
{
    constexpr int IH = (kDwmTH - 1) * ST + 3, IW = (kDwmTW - 1) * ST + 3;
    constexpr size_t lds_bytes = (size_t)((IH * IW * (CB / 16) + 63) / 64) * 1024 + 4 * 1024;      // the patch and one exchange slot per wavefront
    static_assert(lds_bytes <= 64 * 1024, "one patch");
    conv_dwm_kernel<ST, CB><<<(unsigned)blocks, 256, lds_bytes, st>>>(prm);
    return hipGetLastError();
}

// workgroups of the streaming form that share a compute unit: what the registers allow (128 with blocks of 64 channels,
// 72 with blocks of 32)
template <int CB>
constexpr int kDwmStreamPerCU = CB == 64 ? 4 : 7;

template <int CB>
hipError_t launch_dwm_stream(const DwmParams &prm, hipStream_t st)
{
    constexpr int kPerCU = kDwmStreamPerCU<CB>;
    constexpr int IH = kDwmTH + 2, IW = kDwmTW + 2;
    constexpr size_t lds_bytes = (size_t)2 * ((IH * IW * (CB / 16) + 63) / 64) * 1024 + 4 * 1024;   // two patches, the exchange slots
    static_assert(kPerCU * lds_bytes <= (size_t)kLdsBytes, "that many workgroups per compute unit");
    const long long units = (long long)prm.patches * prm.blocks_c;
    long long grid = units < kPerCU * kNumCU ? units : kPerCU * kNumCU;
    grid -= grid % prm.blocks_c;                                   // (units is a multiple, so at least blocks_c remain)
    if (grid <= 0) return hipSuccess;
    conv_dwm_stream_kernel<CB><<<(unsigned)grid, 256, lds_bytes, st>>>(prm);
    return hipGetLastError();
}

}  // namespace

bool conv_dwm_supports(const ConvArgs &a)
{
    if (a.groups != a.C || a.K != a.C || a.C % 32) return false;
    if (a.R != 3 || a.S != 3 || (a.stride != 1 && a.stride != 2) || a.pad > 2) return false;
    if (a.frac_w || a.add || a.acc_out || !a.y) return false;
    if (a.shift < 0 || a.shift > 23) return false;                                   // the lean epilogue
    if (a.Q <= 8 && a.N > 8) return false;      // rows of at most 8 outputs fill half a patch: the vector-ALU kernel is faster (7 x 7: 15 vs 17 us)
    if ((a.ldy & 15) || ((uintptr_t)a.y & 15) || ((uintptr_t)a.x & 15) || (a.b && ((uintptr_t)a.b & 15))) return false;
    if ((long long)a.N * a.H * a.W * a.C >= (1LL << 31) - (1 << 24)) return false;    // 31-bit byte offsets into the input
    if ((long long)a.N * a.P * a.Q >= (1LL << 31)) return false;
    const long long blocks = (long long)a.N * ((a.P + kDwmTH - 1) / kDwmTH) * ((a.Q + kDwmTW - 1) / kDwmTW) * (a.C / 32);
    return blocks <= 0x7fffffffLL;
}

hipError_t launch_conv_dwm(const ConvArgs &a, hipStream_t st)
{
    DwmParams prm;
    prm.a = a;
    prm.tiles_x = (a.Q + kDwmTW - 1) / kDwmTW;
    prm.tiles_y = (a.P + kDwmTH - 1) / kDwmTH;
    const int CB = a.C % 64 ? 32 : 64;
    prm.blocks_c = a.C / CB;
    prm.x_bytes = (unsigned)((long long)a.N * a.H * a.W * a.C);
    prm.div_bc = make_fastdiv(prm.blocks_c);
    prm.div_tx = make_fastdiv(prm.tiles_x);
    prm.div_ty = make_fastdiv(prm.tiles_y);
    const long long blocks = (long long)a.N * prm.tiles_y * prm.tiles_x * prm.blocks_c;
    // stride 1, 31-bit output offsets and at least two patches for every workgroup of a full grid: the streaming form.
    // (MobileNet-shaped pass at batch 128, same box: 112 x 112 x 32 37.9 -> 31.4 us, 56 x 56 x 128 38 -> 32.5,
    // 28 x 28 x 256 24.4 -> 22.4, 14 x 14 x 512 - two patches per workgroup - 15.2 -> 14.3.)
    const long long y_bytes = (long long)a.N * a.P * a.Q * a.ldy;
    const long long min_units = 2LL * (CB == 64 ? kDwmStreamPerCU<64> : kDwmStreamPerCU<32>) * kNumCU;
    if (a.stride == 1 && y_bytes < (1LL << 31) && blocks >= min_units && min_units >= 2LL * prm.blocks_c) {
        prm.patches = a.N * prm.tiles_y * prm.tiles_x;
        prm.y_bytes = (unsigned)y_bytes;
        return CB == 64 ? launch_dwm_stream<64>(prm, st) : launch_dwm_stream<32>(prm, st);
    }
    prm.patches = 0;
    prm.y_bytes = 0;
    if (CB == 64) return a.stride == 1 ? launch_dwm<1, 64>(prm, blocks, st) : launch_dwm<2, 64>(prm, blocks, st);
    return a.stride == 1 ? launch_dwm<1, 32>(prm, blocks, st) : launch_dwm<2, 32>(prm, blocks, st);
}

}  // namespace dfq
