// Pointwise quantized convolution (R = S = 1, stride 1, no padding, groups == 1) on the gfx950
// int8 matrix cores, with the input tile resident in LDS.
//
// For a 1x1 kernel the sum of Eq. 6 is the plain matrix product  acc[k][m] = sum_c W[k][c] * X[m][c]
// over the N*H*W pixels m.  With few input channels (C <= 256) each product term is cheap and the
// layer is bound by memory traffic, so what matters is how often a byte travels from L2 to a
// compute unit.  The general dense kernel gives every (pixel tile, channel tile) pair its own pass
// over the input tile, i.e. K/BC passes per pixel tile.  Here a workgroup keeps the BP x C input
// tile in LDS while it walks over the channel tiles of that pixel tile: the input is fetched once
// per pixel tile (while the previous tile is still being multiplied: two input buffers), and only
// the BC x 64-byte weight slabs stream through a small ring.
//
// Work is cut into units (pixel tile, channel tile), pixel tile major, and every workgroup takes
// one contiguous, equally long run of units, so that the load is even although the number of
// pixel tiles is not a multiple of the number of compute units; a run that starts in the middle
// of a pixel tile fetches that input tile as well.
//
// The inner structure is that of the general dense kernel: items of one 64-byte step, operands of
// the next item read into a second register set while the current one is multiplied, loads
// issued nstages items ahead directly into LDS, one barrier per item, the epilogue (bias as
// start value, ReLU, rounding shift, clamp: the rescale of Eq. 6 for power-of-two scales) in
// registers, 16-byte stores.  Only the lean epilogue exists here; the launcher falls back to the
// general kernel otherwise.
#include "conv_ring.hpp"
#include <type_traits>

namespace dfq {

namespace {

struct PwParams {
    ConvArgs a;
    int M;            // N*H*W
    int nsteps;       // C / 64
    int tiles_c;      // K / BC
    int units;        // pixel tiles * channel tiles
    unsigned x_bytes, w_bytes, y_bytes, add_bytes;
    FastDiv div_tc;
};

// at most BASE + SA * ca + SB * cb outstanding vector-memory operations, ca in [0, 2], cb in [0, 4]
template <int BASE, int SA, int SB>
__device__ __forceinline__ void wait_loads_plus2(int ca, int cb)
{
    switch (cb) {
        case 0: wait_loads_plus<BASE, SA>(min(ca, 2)); break;
        case 1: wait_loads_plus<BASE + SB, SA>(min(ca, 2)); break;
        case 2: wait_loads_plus<BASE + 2 * SB, SA>(min(ca, 2)); break;
        case 3: wait_loads_plus<BASE + 3 * SB, SA>(min(ca, 2)); break;
        default: wait_loads_plus<BASE + 4 * SB, SA>(min(ca, 2)); break;
    }
}

// at most n vector-memory operations outstanding, n known only at run time (uniform); n above 31 waits as for 31
__device__ __forceinline__ void wait_loads_le(int n)
{
    switch (n) {
#define DFQ_WAIT_CASE(N) case N: asm volatile("s_waitcnt vmcnt(" #N ")" ::: "memory"); break;
        DFQ_WAIT_CASE(0) DFQ_WAIT_CASE(1) DFQ_WAIT_CASE(2) DFQ_WAIT_CASE(3) DFQ_WAIT_CASE(4) DFQ_WAIT_CASE(5) DFQ_WAIT_CASE(6) DFQ_WAIT_CASE(7)
        DFQ_WAIT_CASE(8) DFQ_WAIT_CASE(9) DFQ_WAIT_CASE(10) DFQ_WAIT_CASE(11) DFQ_WAIT_CASE(12) DFQ_WAIT_CASE(13) DFQ_WAIT_CASE(14)
        DFQ_WAIT_CASE(15) DFQ_WAIT_CASE(16) DFQ_WAIT_CASE(17) DFQ_WAIT_CASE(18) DFQ_WAIT_CASE(19) DFQ_WAIT_CASE(20) DFQ_WAIT_CASE(21)
        DFQ_WAIT_CASE(22) DFQ_WAIT_CASE(23) DFQ_WAIT_CASE(24) DFQ_WAIT_CASE(25) DFQ_WAIT_CASE(26) DFQ_WAIT_CASE(27) DFQ_WAIT_CASE(28)
        DFQ_WAIT_CASE(29) DFQ_WAIT_CASE(30)
#undef DFQ_WAIT_CASE
        default: asm volatile("s_waitcnt vmcnt(31)" ::: "memory"); break;
    }
}

// FUSE: an element-wise add (Eq. 10) follows the convolution and is taken in the epilogue: the
// second operand's 16 codes per lane and tile are fetched into registers one unit ahead, at the
// start of the previous unit's epilogue, and awaited at that epilogue's end, so that the whole
// epilogue (a few microseconds of vector work) covers the fetch.
// PC: one weight format per output channel, every channel's shift within [0, 23]: shift, clamp bound
// and rounding constant of all K channels sit in LDS behind the bias.
// ROWIO (wavefront tile 32 pixels x 128 channels): the epilogue moves whole 128-byte rows.  In the accumulator
// layout a lane holds 16 channels of one pixel, so a plain store instruction writes 32-byte pieces of 32 different
// rows (and the second operand would be fetched the same way): four times the memory requests of whole cache lines,
// which is what bounds the layers that write more than they read (measured with the stores linearized: 56x56
// 64 -> 256 at batch 256 78 -> 58 us).  Here every wavefront owns a 4 KB LDS slot (two with FUSE): results are
// written there in a swizzled [pixel][channel] layout and read back row-wise, eight full rows per store
// instruction; with FUSE the second operand of the NEXT unit is fetched row-wise straight into the other slot
// (direct-to-LDS loads, lane order chosen so that the epilogue's 16-byte reads are conflict-free) and awaited one
// unit later by an exact count of the younger operations - it is in LDS, not in registers, so nothing of it is
// live in the compiler's view while the load is in flight.
template <int BP, int BC, int WAVES_P, int WAVES_C, bool FUSE, int OCC, bool PC = false, bool ROWIO = false, bool LAZY = false>
__global__ void __launch_bounds__(WAVES_P * WAVES_C * 64, OCC) conv_pw_kernel(PwParams prm)
{
    static_assert(!ROWIO || (WAVES_C == 1 && BC == 128 && BP / WAVES_P == 32), "row-wise epilogue: wavefront tiles of 32 x 128");
    constexpr int kIoSlotBytes = 32 * 128;                // one wavefront tile of int8
    constexpr int kIoBytesPerWave = ROWIO ? (FUSE ? 2 : 1) * kIoSlotBytes : 0;
    constexpr int NSTAGES = 3;                            // depth of the weight ring
    constexpr int NW = WAVES_P * WAVES_C;                 // wavefronts per workgroup
    static_assert(NW == 4 || NW == 8, "four or eight wavefronts per workgroup");
    constexpr int WP = BP / WAVES_P, WC = BC / WAVES_C;   // wavefront tile
    constexpr int PT = WP / 32, CT = WC / 32;             // 32x32 MFMA tiles per wavefront
    constexpr int RPC = 64 / kPieces;                     // LDS rows filled by one wavefront-wide load
    constexpr int XS = BP / (RPC * NW), WS = (BC + RPC * NW - 1) / (RPC * NW);
    constexpr bool kPartialW = BC < RPC * NW;
    static_assert(XS * RPC * NW == BP && (kPartialW || WS * RPC * NW == BC) && BC % 16 == 0, "whole chunks");
    static_assert(WS <= XS, "the wait for the second operand rounds the refill's loads down to 0, WS, XS or WS + XS");
    static_assert(WP % 32 == 0 && WC % 32 == 0, "tile shape");
    constexpr int SLAB_PIECES = BP * kPieces;             // one 64-byte step of the input tile
    constexpr int WSTAGE_PIECES = BC * kPieces;           // one 64-byte step of the weight tile

    // LDS: input buffers [2][nsteps] slabs of BP rows x 64 bytes, weight ring [NSTAGES] slabs of BC rows
    // x 64 bytes, bias of all K channels
    extern __shared__ uint4 lds[];

    const ConvArgs &a = prm.a;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nsteps = prm.nsteps;
    const bool w_active = !kPartialW || wave < BC / RPC;

    // ---- this workgroup's run of units.  Workgroup ids are dealt round-robin to the 8 XCDs;
    // renumbering them so that each XCD owns a contiguous range keeps workgroups that share an
    // input tile in one L2.
    const int G = gridDim.x;
    int lb = blockIdx.x;
    {
        const int per = G / 8, rem = G % 8, xcd = lb % 8, idx = lb / 8;
        lb = (xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per) + idx;
    }
    const int per_wg = prm.units / G, extra = prm.units % G;
    const int u0 = lb * per_wg + min(lb, extra);
    const int nunits = per_wg + (lb < extra ? 1 : 0);
    const int nitems = nunits * nsteps;

    const v4i xrsrc = make_rsrc(a.x, prm.x_bytes);
    const v4i wrsrc = make_rsrc(a.w, prm.w_bytes);
    const __amdgpu_buffer_rsrc_t yrsrc = __builtin_amdgcn_make_buffer_rsrc(a.y, 0, (int)prm.y_bytes, 0x00020000);
    const v4i arsrc = make_rsrc(FUSE ? a.add : a.x, FUSE ? prm.add_bytes : 0u);
    const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) char *)(char *)&lds[0];
    const int ring_piece0 = 2 * nsteps * SLAB_PIECES;
    int *bias_lds = (int *)(lds + ring_piece0 + NSTAGES * WSTAGE_PIECES);
    for (int i = tid; i < a.K; i += NW * 64) bias_lds[i] = a.b ? a.b[i] : 0;
    int *pc_shift = bias_lds + a.K, *pc_hi = pc_shift + a.K, *pc_badd = pc_hi + a.K;
    // ROWIO: this wavefront's slot(s) behind the bias (and the per-channel tables)
    char *io_lds = (char *)(bias_lds + a.K * (PC ? 4 : 1)) + wave * kIoBytesPerWave;
    const unsigned io_addr = lds_base + (unsigned)(io_lds - (char *)&lds[0]);
    if (PC) {
        for (int i = tid; i < a.K; i += NW * 64) {
            const int sk = (a.shift + a.frac_w[i]) & 31;            // in [0, 23] by the caller's word
            pc_shift[i] = sk;
            pc_hi[i] = 127 << min(sk, 23);
            pc_badd[i] = sk > 0 ? ((1 << (sk - 1)) - 1) : 0;
        }
    }

    // ---- producer.  Lane l of a wavefront-wide load supplies row l/4 of a 16-row chunk, physical
    // piece l%4, which holds logical piece (l%4) ^ ((row>>2)&3): 16 consecutive rows then put any
    // one logical piece on 16 different bank groups.
    const int lrow = lane / kPieces;
    const int lp = (lane & 3) ^ ((lane >> 4) & 3);
    unsigned xoff[XS];               // byte offset of the lane's pixel row (+ piece), or out of range past M
    unsigned woff[WS];               // byte offset of the lane's weight row of channel tile 0 (+ piece)
#pragma unroll
    for (int j = 0; j < WS; j++) {
        // LDS row i = 8g + 4h + e of a 32-row group receives channel 16h + 4g + e: the matrix
        // instruction then leaves 16 consecutive channels in each lane
        const int rr = RPC * (wave + NW * j) + lrow;
        const int i32 = rr & 31;
        const int k = (rr & ~31) + 16 * ((i32 >> 2) & 1) + 4 * (i32 >> 3) + (i32 & 3);
        woff[j] = (unsigned)(k * a.C) + (unsigned)lp * 16u;
    }
    int p_pt, p_ct, p_step = 0, p_par = 0;   // unit, step and input buffer the producer fetches next
    bool p_loadx = true;                     // that unit is the run's first of its pixel tile: fetch the input too
    p_pt = fastdiv(u0, prm.div_tc);
    p_ct = u0 - p_pt * prm.tiles_c;
    unsigned p_hist = 0;                     // bit q: the q-th last issued item fetched input
    int young = 0;                           // ROWIO + FUSE: vector-memory operations issued since the last fetch of a second operand

    auto issue = [&](int stage) __attribute__((always_inline)) {
        if (p_step == 0 && p_loadx) {
            const int m0 = p_pt * BP;
#pragma unroll
            for (int j = 0; j < XS; j++) {
                const int m = m0 + RPC * (wave + NW * j) + lrow;
                xoff[j] = m < prm.M ? (unsigned)(m * a.C) + (unsigned)lp * 16u : kOutOfRange;
            }
        }
        const unsigned step_off = (unsigned)p_step * kStepBytes;
        if (p_loadx) {
            const unsigned xbase = (unsigned)__builtin_amdgcn_readfirstlane(
                (int)(lds_base + (unsigned)((p_par * nsteps + p_step) * SLAB_PIECES) * 16u + (unsigned)wave * 1024u));
#pragma unroll
            for (int j = 0; j < XS; j++) load_piece_to_lds(xoff[j] + step_off, xrsrc, xbase + (unsigned)j * (NW * 1024u));
        }
        if (w_active) {
            const unsigned wbase = (unsigned)__builtin_amdgcn_readfirstlane(
                (int)(lds_base + (unsigned)(ring_piece0 + stage * WSTAGE_PIECES) * 16u + (unsigned)wave * 1024u));
            const unsigned tile_off = (unsigned)(p_ct * BC * a.C) + step_off;
#pragma unroll
            for (int j = 0; j < WS; j++) load_piece_to_lds(woff[j] + tile_off, wrsrc, wbase + (unsigned)j * (NW * 1024u));
        }
        if (ROWIO && FUSE) young += (p_loadx ? XS : 0) + (w_active ? WS : 0);
        p_hist = (p_hist << 1) | (p_loadx ? 1u : 0u);
        if (++p_step == nsteps) {
            p_step = 0;
            p_loadx = false;
            if (++p_ct == prm.tiles_c) {
                p_ct = 0;
                ++p_pt;
                p_par ^= 1;
                p_loadx = true;
            }
        }
    };

    const int wp0 = (wave % WAVES_P) * WP;
    const int wc0 = (wave / WAVES_P) * WC;
    const int l32 = lane & 31, lh = lane >> 5;
    const int swz = (l32 >> 2) & 3;
#pragma unroll
    for (int i = 0; i < NSTAGES; i++)
        if (i < nitems) issue(i);

    Requant rq, rq2;
    rq.init(a.shift, a.relu);
    rq2.init(FUSE ? a.add_shift : 1, a.add_relu);
    static_assert(!LAZY || (FUSE && !PC), "the single-rounding join: fused, one weight format per layer");
    constexpr bool lazy = LAZY;               // single-rounding join: the accumulator itself meets the second operand
    __syncthreads();   // bias_lds complete

    // consumer position: unit (c_pt, c_ct) and step of the item being multiplied; reader position:
    // input buffer and step of the item whose operands are read next
    int c_pt = fastdiv(u0, prm.div_tc);
    int c_ct = u0 - c_pt * prm.tiles_c;
    int c_step = 0;
    int r_ct = c_ct, r_step = 0, r_par = 0;

    // accumulators start at the bias: register r of a lane belongs to channel kc + r
    v16i acc[CT][PT];
    auto reset_acc = [&](int ct) __attribute__((always_inline)) {
#pragma unroll
        for (int c = 0; c < CT; c++) {
            const int4 *bp = (const int4 *)(bias_lds + ct * BC + wc0 + c * 32 + 16 * lh);
#pragma unroll
            for (int r4 = 0; r4 < 4; r4++) {
                const int4 bv = bp[r4];
#pragma unroll
                for (int p = 0; p < PT; p++) {
                    acc[c][p][4 * r4 + 0] = bv.x;
                    acc[c][p][4 * r4 + 1] = bv.y;
                    acc[c][p][4 * r4 + 2] = bv.z;
                    acc[c][p][4 * r4 + 3] = bv.w;
                }
            }
        }
    };
    reset_acc(c_ct);

    struct Half {
        v4i w[CT];
        v4i x[PT];
    };
    Half f0, f1;
    // both halves of the reader's item; advances the reader afterwards when `advance`
    auto read_half = [&](Half &f, int kk, int stage) __attribute__((always_inline)) {
        const v4i *xs = (const v4i *)lds + (r_par * nsteps + r_step) * SLAB_PIECES;
        const v4i *ws = (const v4i *)lds + ring_piece0 + stage * WSTAGE_PIECES;
        const int g = (kk * 2 + lh) ^ swz;   // physical piece
#pragma unroll
        for (int c = 0; c < CT; c++) f.w[c] = ws[(wc0 + c * 32 + l32) * kPieces + g];
#pragma unroll
        for (int p = 0; p < PT; p++) f.x[p] = xs[(wp0 + p * 32 + l32) * kPieces + g];
    };
    auto advance_reader = [&]() __attribute__((always_inline)) {
        if (++r_step == nsteps) {
            r_step = 0;
            if (++r_ct == prm.tiles_c) {
                r_ct = 0;
                r_par ^= 1;
            }
        }
    };
    auto mfma_half = [&](const Half &f) __attribute__((always_inline)) {
#pragma unroll
        for (int c = 0; c < CT; c++)
#pragma unroll
            for (int p = 0; p < PT; p++)
                acc[c][p] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f.w[c], f.x[p], acc[c][p], 0, 0, 0);
    };
    auto ring_barrier = [&]() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };

    // ep_hist: bit k set when item i-1-k ended a unit (its epilogue issued kStoresPerUnit stores)
    constexpr int kStoresPerUnit = CT * PT;
    constexpr unsigned kHistMask = (1u << (NSTAGES - 1)) - 1u;
    unsigned ep_hist = 0;
    const unsigned lane_yoff = (unsigned)((wp0 + l32) * a.ldy + wc0 + 16 * lh);
    const unsigned lane_aoff = (unsigned)((wp0 + l32) * a.ldadd + wc0 + 16 * lh);
    static_assert(!FUSE || CT * PT == 4, "the fused form handles four tiles per wavefront");
    v4i other[4], other_next[4];      // FUSE: the second operand of the current unit / of the one after it
    int units_left = nunits;          // units not yet written out
    // `live` false: every lane gets an offset past the buffer (zeros arrive, nothing is read), so that the
    // fetch needs no branch of its own.
    auto fetch_other = [&](int pt, int ct, bool live) __attribute__((always_inline)) {
        const unsigned tile_off = live ? (unsigned)(pt * BP * a.ldadd + ct * BC) : kOutOfRange;
#pragma unroll
        for (int c = 0; c < CT; c++)
#pragma unroll
            for (int p = 0; p < PT; p++)
                load_piece_to_regs(other_next[c * PT + p], lane_aoff + tile_off + (unsigned)(p * 32 * a.ldadd + c * 32), arsrc);
    };
    // ROWIO: the second operand of unit (pt, ct) for this wavefront's 32 pixels x 128 channels, straight into LDS slot
    // `par`: instruction j covers pixel rows 8j .. 8j+7 whole; lane l fetches row 8j + l%8, bytes 16*(l/8) .., and the
    // data lands at slot + 1024*j + 16*l, i.e. as [16-byte column][row]: the epilogue's lanes (one pixel each, eight
    // neighbouring pixels per quarter-wavefront) then read neighbouring 16-byte pieces.
    int io_par = 0;
    auto fetch_other_rows = [&](int pt, int ct, bool live, int par) __attribute__((always_inline)) {
        const unsigned tile_off = live ? (unsigned)(pt * BP * a.ldadd + ct * BC) : kOutOfRange;
        const unsigned lane_off = (unsigned)((wp0 + (lane & 7)) * a.ldadd + (lane >> 3) * 16);
#pragma unroll
        for (int j = 0; j < 4; j++)
            load_piece_to_lds(lane_off + tile_off + (unsigned)(8 * j * a.ldadd), arsrc,
                              (unsigned)__builtin_amdgcn_readfirstlane((int)(io_addr + (unsigned)(par * kIoSlotBytes + j * 1024))));
    };
    auto finish_item = [&]() __attribute__((always_inline)) {
        ep_hist = (ep_hist << 1) & kHistMask;
        if (++c_step == nsteps) {
            settle_accumulators<CT * PT>(&acc[0][0]);
            const unsigned tile_off = (unsigned)(c_pt * BP * a.ldy + c_ct * BC);
            if constexpr (ROWIO) {
                v4i *slot = (v4i *)(io_lds + (FUSE ? io_par * kIoSlotBytes : 0));
                v4i oth[CT];
                if constexpr (FUSE) {
                    // this unit's second operand: fetched at the start of the previous unit's epilogue (or ahead of
                    // the loop) into this slot; `young` operations were issued since
                    wait_loads_le(young);
#pragma unroll
                    for (int c = 0; c < CT; c++) oth[c] = slot[(l32 >> 3) * 64 + (2 * c + lh) * 8 + (l32 & 7)];
                    --units_left;
                    const bool wrap = c_ct + 1 == prm.tiles_c;
                    fetch_other_rows(wrap ? c_pt + 1 : c_pt, wrap ? 0 : c_ct + 1, units_left > 0, io_par ^ 1);
                    young = 0;
                }
                uint4 out[CT];
                if constexpr (PC) {
#pragma unroll
                    for (int c = 0; c < CT; c++) {
                        const int kr = c_ct * BC + c * 32 + 16 * lh;
                        uint32_t o[4];
#pragma unroll
                        for (int r4 = 0; r4 < 4; r4++) {
                            const int4 sv = *(const int4 *)(pc_shift + kr + 4 * r4);
                            const int4 hv = *(const int4 *)(pc_hi + kr + 4 * r4);
                            const int4 bv = *(const int4 *)(pc_badd + kr + 4 * r4);
                            const v16i &v = acc[c][0];
                            if (FUSE)
                                o[r4] = requant_add_four_per_channel(v[4 * r4], v[4 * r4 + 1], v[4 * r4 + 2], v[4 * r4 + 3], sv, hv, bv, a.relu,
                                                                     (uint32_t)oth[c][r4], a.add_sa, a.add_sb, rq2);
                            else
                                o[r4] = requant_four_per_channel(v[4 * r4], v[4 * r4 + 1], v[4 * r4 + 2], v[4 * r4 + 3], sv, hv, bv, a.relu);
                        }
                        out[c] = make_uint4(o[0], o[1], o[2], o[3]);
                    }
                } else {
#pragma unroll
                    for (int c = 0; c < CT; c++)
                        out[c] = !FUSE ? requant_tile_lane_fast(acc[c][0], rq)
                                 : lazy ? add_tile_lane_lazy(acc[c][0], oth[c], a.add_sb, rq2)
                                        : requant_add_tile_lane(acc[c][0], rq, oth[c], a.add_sa, a.add_sb, rq2);
                }
                // results into the slot, [pixel][16-byte piece ^ (pixel & 7)]; the second operand has been read out of it,
                // and LDS operations of one wavefront execute in order
                uint4 *stage = (uint4 *)slot;
#pragma unroll
                for (int c = 0; c < CT; c++) stage[l32 * 8 + ((2 * c + lh) ^ (l32 & 7))] = out[c];
                // back row-wise: eight lanes per 128-byte row, eight rows per store instruction
#pragma unroll
                for (int j = 0; j < 4; j++) {
                    const int r = 8 * j + (lane >> 3);
                    const uint4 v = stage[r * 8 + ((lane & 7) ^ (r & 7))];
                    store_piece(v, tile_off + (unsigned)((wp0 + r) * a.ldy + (lane & 7) * 16), yrsrc);
                }
                if (FUSE) {
                    young += 4;
                    io_par ^= 1;
                }
            } else {
                if (FUSE) {
                    // The second operand of this unit is complete in other_next: its loads were awaited at the end of
                    // the previous unit's epilogue (or ahead of the loop).  The loads of the next unit's are issued here
                    // and awaited at the end of this epilogue, behind its stores - both inside this one block of
                    // straight-line code: the registers are written behind the compiler's back, so a register copy or
                    // a spill between a load and its wait (as register allocation inserts them where values cross
                    // loop boundaries) would read them too early.
#pragma unroll
                    for (int t = 0; t < 4; t++) other[t] = other_next[t];
                    --units_left;
                    const bool wrap = c_ct + 1 == prm.tiles_c;
                    fetch_other(wrap ? c_pt + 1 : c_pt, wrap ? 0 : c_ct + 1, units_left > 0);
                }
                if constexpr (PC) {
#pragma unroll
                    for (int c = 0; c < CT; c++) {
                        const int kr = c_ct * BC + wc0 + c * 32 + 16 * lh;
                        uint32_t o[PT][4];
#pragma unroll
                        for (int r4 = 0; r4 < 4; r4++) {
                            const int4 sv = *(const int4 *)(pc_shift + kr + 4 * r4);
                            const int4 hv = *(const int4 *)(pc_hi + kr + 4 * r4);
                            const int4 bv = *(const int4 *)(pc_badd + kr + 4 * r4);
#pragma unroll
                            for (int p = 0; p < PT; p++) {
                                const v16i &v = acc[c][p];
                                if (FUSE)
                                    o[p][r4] = requant_add_four_per_channel(v[4 * r4], v[4 * r4 + 1], v[4 * r4 + 2], v[4 * r4 + 3], sv, hv, bv,
                                                                            a.relu, (uint32_t)other[c * PT + p][r4], a.add_sa, a.add_sb, rq2);
                                else
                                    o[p][r4] = requant_four_per_channel(v[4 * r4], v[4 * r4 + 1], v[4 * r4 + 2], v[4 * r4 + 3], sv, hv, bv, a.relu);
                            }
                        }
#pragma unroll
                        for (int p = 0; p < PT; p++)
                            store_piece(make_uint4(o[p][0], o[p][1], o[p][2], o[p][3]),
                                        lane_yoff + tile_off + (unsigned)(p * 32 * a.ldy + c * 32), yrsrc);
                    }
                } else {
#pragma unroll
                    for (int c = 0; c < CT; c++)
#pragma unroll
                        for (int p = 0; p < PT; p++) {
                            const unsigned off = lane_yoff + tile_off + (unsigned)(p * 32 * a.ldy + c * 32);
                            if (!FUSE) store_piece(requant_tile_lane_fast(acc[c][p], rq), off, yrsrc);
                            else if (lazy) store_piece(add_tile_lane_lazy(acc[c][p], other[c * PT + p], a.add_sb, rq2), off, yrsrc);
                            else store_piece(requant_add_tile_lane(acc[c][p], rq, other[c * PT + p], a.add_sa, a.add_sb, rq2), off, yrsrc);
                        }
                }
                if (FUSE) wait_loads_for<kStoresPerUnit>(other_next[0], other_next[1], other_next[2], other_next[3]);
            }
            ep_hist |= 1u;
            c_step = 0;
            if (++c_ct == prm.tiles_c) {
                c_ct = 0;
                ++c_pt;
            }
            reset_acc(c_ct);
        }
    };
    // Item i multiplies operands that are already in registers and meanwhile reads those of item
    // i+1: after the first k-step's matrix instructions the wavefront waits for its own loads of
    // item i+1 and meets the others at the barrier; every wavefront has then also finished reading
    // the weight stage of item i, which REFILL overwrites with item i + NSTAGES.
    auto do_item = [&](auto refill, auto has_next, auto wait, int stage) __attribute__((always_inline)) {
        const int next = stage + 1 == NSTAGES ? 0 : stage + 1;
        mfma_half(f0);
        __builtin_amdgcn_sched_barrier(0);
        if (decltype(has_next)::value) {
            wait();
            ring_barrier();
            read_half(f0, 0, next);
        }
        __builtin_amdgcn_sched_barrier(0);
        mfma_half(f1);
        __builtin_amdgcn_sched_barrier(0);
        if (decltype(refill)::value) issue(stage);
        if (decltype(has_next)::value) {
            read_half(f1, 1, next);
            advance_reader();
        }
        __builtin_amdgcn_sched_barrier(0);
        finish_item();
    };

    // Vector-memory operations younger than the loads of item i+1 when item i waits for them:
    // the weight loads of items i+2 .. i+NSTAGES-1, the input loads of those of them that fetch
    // input (p_hist), and the stores of the epilogues of items i+1-NSTAGES .. i-1 (ep_hist; an
    // item refills before its epilogue; with FUSE an epilogue's second-operand loads precede its
    // stores and are complete when it ends).
    // Loads and stores complete in issue order; operations that are not counted only make the
    // wait longer.
    auto steady_wait = [&]() __attribute__((always_inline)) {
        const int cx = __builtin_popcount(p_hist & ((1u << (NSTAGES - 2)) - 1u));
        const int ce = __builtin_popcount(ep_hist);
        // (ROWIO + FUSE: an epilogue's four fetches of the next second operand stay in flight behind it as well)
        constexpr int kEpOps = kStoresPerUnit + ((ROWIO && FUSE) ? 4 : 0);
        if (w_active) wait_loads_plus2<(NSTAGES - 2) * WS, XS, kEpOps>(cx, ce);
        else wait_loads_plus2<0, XS, kEpOps>(cx, ce);
    };
    if (nitems > 0) {
        if (FUSE && ROWIO) {
            fetch_other_rows(c_pt, c_ct, true, 0);
        } else if (FUSE) {
            fetch_other(c_pt, c_ct, true);
            wait_loads_for<0>(other_next[0], other_next[1], other_next[2], other_next[3]);
        }
        wait_loads<0>();
        young = 0;
        ring_barrier();
        read_half(f0, 0, 0);
        read_half(f1, 1, 0);
        advance_reader();
    }
    const int steady = nitems - NSTAGES;     // items that refill their stage
    int it = 0;
    for (; it + NSTAGES <= steady; it += NSTAGES) {
#pragma unroll
        for (int s = 0; s < NSTAGES; s++) do_item(std::true_type{}, std::true_type{}, steady_wait, s);
    }
    int stage = 0;   // it is a multiple of NSTAGES here
    for (; it < steady; it++) {
        do_item(std::true_type{}, std::true_type{}, steady_wait, stage);
        stage = stage + 1 == NSTAGES ? 0 : stage + 1;
    }
    for (; it < nitems - 1; it++) {
        // the ring drains: input loads and stores are not counted, which only lengthens the wait
        const int ahead = nitems - 2 - it;   // items younger than the one awaited
        do_item(std::false_type{}, std::true_type{}, [&]() __attribute__((always_inline)) {
            if (w_active) wait_ahead<WS>(ahead);
            else wait_loads<0>();
        }, stage);
        stage = stage + 1 == NSTAGES ? 0 : stage + 1;
    }
    if (it < nitems) do_item(std::false_type{}, std::false_type{}, steady_wait, stage);
    // the last epilogue's (empty) fetch still targets this workgroup's LDS: it must have landed before the LDS is released
    if (FUSE && ROWIO) wait_loads<0>();
}

inline hipError_t big_lds_pw(void (*k)(PwParams))
{
    return hipFuncSetAttribute((const void *)k, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
}

template <int BP, int BC, int WAVES_P, int WAVES_C, bool ROWIO = false>
size_t pw_lds_bytes(const ConvArgs &a)
{
    // input buffers, weight ring, bias (+ three per-channel tables), row-wise epilogue slots per wavefront
    return (size_t)2 * BP * a.C + (size_t)3 * BC * kStepBytes + (size_t)a.K * 4 * (a.frac_w ? 4 : 1) +
           (ROWIO ? (size_t)WAVES_P * WAVES_C * (a.add ? 2 : 1) * 4096 : 0);
}

template <int BP, int BC, int WAVES_P, int WAVES_C, int PER_CU, bool PC = false, bool ROWIO = false>
hipError_t launch_pw(const ConvArgs &a, hipStream_t st)
{
    constexpr bool kCanFuse = (BP / WAVES_P / 32) * (BC / WAVES_C / 32) == 4;
    PwParams prm;
    prm.a = a;
    const long long M = (long long)a.N * a.P * a.Q;
    prm.M = (int)M;
    prm.nsteps = a.C / kStepBytes;
    prm.tiles_c = a.K / BC;
    const long long units = ((M + BP - 1) / BP) * prm.tiles_c;
    if (units > 0x7fffffffLL) return hipErrorInvalidValue;
    prm.units = (int)units;
    prm.x_bytes = (unsigned)(M * a.C);
    prm.w_bytes = (unsigned)((long long)a.K * a.C);
    prm.y_bytes = (unsigned)(M * a.ldy);
    prm.add_bytes = a.add ? (unsigned)(M * a.ldadd) : 0u;
    prm.div_tc = make_fastdiv(prm.tiles_c);
    int grid = PER_CU * kNumCU;
    if (grid > prm.units) grid = prm.units;
    const size_t lds_bytes = pw_lds_bytes<BP, BC, WAVES_P, WAVES_C, ROWIO>(a);
    if (lds_bytes * PER_CU > (size_t)kLdsBytes) return hipErrorInvalidValue;
    constexpr int occ = PER_CU * WAVES_P * WAVES_C / 4;
    if (a.add) {
        if constexpr (kCanFuse) {
            if (a.add_lazy) {
                if constexpr (!PC) {
                    static const hipError_t attr = big_lds_pw(conv_pw_kernel<BP, BC, WAVES_P, WAVES_C, true, occ, false, ROWIO, true>);
                    if (attr != hipSuccess) return attr;
                    conv_pw_kernel<BP, BC, WAVES_P, WAVES_C, true, occ, false, ROWIO, true><<<(unsigned)grid, WAVES_P * WAVES_C * 64, lds_bytes, st>>>(prm);
                    return hipGetLastError();
                }
                return hipErrorInvalidValue;
            }
            static const hipError_t attr = big_lds_pw(conv_pw_kernel<BP, BC, WAVES_P, WAVES_C, true, occ, PC, ROWIO>);
            if (attr != hipSuccess) return attr;
            conv_pw_kernel<BP, BC, WAVES_P, WAVES_C, true, occ, PC, ROWIO><<<(unsigned)grid, WAVES_P * WAVES_C * 64, lds_bytes, st>>>(prm);
            return hipGetLastError();
        }
        return hipErrorInvalidValue;
    }
    static const hipError_t attr = big_lds_pw(conv_pw_kernel<BP, BC, WAVES_P, WAVES_C, false, occ, PC, ROWIO>);
    if (attr != hipSuccess) return attr;
    conv_pw_kernel<BP, BC, WAVES_P, WAVES_C, false, occ, PC, ROWIO><<<(unsigned)grid, WAVES_P * WAVES_C * 64, lds_bytes, st>>>(prm);
    return hipGetLastError();
}

}  // namespace

// The input-resident form applies to unpadded 1x1 stride-1 layers with C a multiple of 64 whose
// double-buffered input tile fits LDS (C <= 256), whose epilogue is the lean one, and which have at
// least two items per pixel tile (an input buffer is refilled two items ahead of its next use).
bool conv_pw_geometry_ok(const ConvArgs &a)
{
    if (a.groups != 1 || a.R != 1 || a.S != 1 || a.stride != 1 || a.pad != 0) return false;
    if (a.C % kStepBytes || a.C > 256) return false;
    if (a.K % 64 || a.K > 4096) return false;
    const int bc = a.K % 128 == 0 ? 128 : 64;
    if ((a.K / bc) * (a.C / kStepBytes) < 2) return false;
    if ((size_t)2 * 256 * a.C + (size_t)3 * bc * kStepBytes + (size_t)a.K * 4 > (size_t)kLdsBytes) return false;   // input buffers, ring, bias
    const long long M = (long long)a.N * a.P * a.Q;
    if (M * a.C >= (1LL << 31) || M * (long long)(a.ldy > a.K ? a.ldy : a.K) >= (1LL << 31) || M >= (1LL << 31) - 512) return false;
    return true;
}

bool conv_pw_supports(const ConvArgs &a)
{
    if (!conv_pw_geometry_ok(a)) return false;
    if (a.frac_w) {
        // per-channel weight formats: every declared shift in the lean range, and room for the tables
        const int bc = a.K % 128 == 0 ? 128 : 64;
        if ((size_t)2 * 256 * a.C + (size_t)3 * bc * kStepBytes + (size_t)a.K * 16 > (size_t)kLdsBytes) return false;
        if (((uintptr_t)a.frac_w & 3) || a.shift + a.frac_w_lo < 0 || a.shift + a.frac_w_hi > 23) return false;
    }
    if (!(a.frac_w || (a.shift >= 0 && a.shift <= 23)) || a.acc_out || !a.y || (a.ldy & 15) || ((uintptr_t)a.y & 15)) return false;
    if (((uintptr_t)a.x & 15) || ((uintptr_t)a.w & 15)) return false;
    if (a.add) {
        // the fused add: second operand addressable like y, final shift in the range of the fast rounding
        if (((uintptr_t)a.add & 15) || (a.ldadd & 15) || a.ldadd < a.K) return false;
        if ((long long)a.N * a.P * a.Q * a.ldadd >= (1LL << 31)) return false;
        if (!(a.add_shift >= 0 && a.add_shift <= 23) || a.add_sa < 0 || a.add_sa > 22 || a.add_sb < 0 || a.add_sb > 22) return false;
        if (a.add_lazy && a.frac_w) return false;        // the single-rounding join exists for one weight format per layer only
    }
    return true;
}

hipError_t launch_conv_pw(const ConvArgs &a, hipStream_t st)
{
    // Layers that move four times the output (and second-operand) bytes of their input - C = 64 with channel tiles
    // of 128 - take the row-wise epilogue: two workgroups of four wavefronts (32 x 128 each) per compute unit.
    // (Measured at batch 256, 56 x 56, 64 -> 256: plain 79 -> 62 us, fused 116 -> 110 us; with C = 128 only one
    // eight-wavefront workgroup fits beside the slots, and that is 3 % slower than the register epilogue.)
    if (a.K % 128 == 0 && a.C == 64 ) {
        if (a.frac_w) {
            if (2 * pw_lds_bytes<128, 128, 4, 1, true>(a) <= (size_t)kLdsBytes) return launch_pw<128, 128, 4, 1, 2, true, true>(a, st);
        } else {
            if (2 * pw_lds_bytes<128, 128, 4, 1, true>(a) <= (size_t)kLdsBytes) return launch_pw<128, 128, 4, 1, 2, false, true>(a, st);
        }
    }
    if (a.frac_w) {
        // the per-channel epilogue holds more registers: at most two wavefronts per SIMD
        if (a.K % 128 == 0) {
            // (two workgroups per CU only while both sets of per-channel tables fit)
            if (a.add && a.C <= 128 && 2 * pw_lds_bytes<128, 128, 2, 2>(a) <= (size_t)kLdsBytes) return launch_pw<128, 128, 2, 2, 2, true>(a, st);
            return launch_pw<256, 128, 4, 2, 1, true>(a, st);
        }
        if (a.C <= 128 && 2 * pw_lds_bytes<256, 64, 4, 1>(a) <= (size_t)kLdsBytes) return launch_pw<256, 64, 4, 1, 2, true>(a, st);
        return launch_pw<256, 64, 4, 1, 1, true>(a, st);
    }
    // as many workgroups per compute unit as the two input buffers leave room for
    if (a.K % 128 == 0) {
        // (the fused epilogue needs more registers than four wavefronts per SIMD leave it: with C <= 128 two
        // independent four-wavefront workgroups of 128 x 128 per CU, measured 3 % faster than one of 256 x 128)
        if (a.C == 64 && !a.add) return launch_pw<256, 128, 4, 2, 2>(a, st);
        if (a.add && a.C <= 128) return launch_pw<128, 128, 2, 2, 2>(a, st);
        return launch_pw<256, 128, 4, 2, 1>(a, st);
    }
    if (a.C <= 128 && 2 * pw_lds_bytes<256, 64, 4, 1>(a) <= (size_t)kLdsBytes) return launch_pw<256, 64, 4, 1, 2>(a, st);
    return launch_pw<256, 64, 4, 1, 1>(a, st);
}

}  // namespace dfq
