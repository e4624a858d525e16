// Dense quantized convolution as an implicit GEMM on the gfx950 int8 matrix cores.
//
// The sum of Eq. 6 for groups == 1 is a matrix product  acc[k][m] = sum_j Wm[k][j] * Xm[j][m]
// with m running over the N*P*Q output pixels and j over the R*S*C (tap, input channel) pairs.
// In NHWC the C channels of one tap are contiguous, and a weight row [R][S][C] is contiguous
// in exactly the same (tap, channel) order, so both operands are fetched as 16-byte pieces
// that cover the same 16 values of j; taps outside the image are fetched as zeros (the code
// of the value 0).  Nothing is materialized: the im2col matrix exists only as LDS tiles.
//
// A workgroup (4 or 8 wavefronts) is persistent: it walks over BP-pixel x BC-channel output
// tiles (tile numbers blockIdx, blockIdx + gridDim, ...).  The j range of each tile is walked
// in steps of 64 bytes through a ring of LDS stages that is filled by direct global->LDS
// buffer loads (no register staging) issued nstages steps ahead - across tile boundaries, so
// the first loads of the next tile are in flight while the current one is multiplied and
// written out (HBM latency here is about four steps of matrix work).  A wavefront waits only
// for the loads of the step it is about to read (its own counter of outstanding vector memory
// operations, in which the stores of the epilogues are counted too, then one workgroup barrier
// per step), and the operands of step i+1 are read from LDS into the registers of the half of
// step i that has just been multiplied.  Each wavefront-wide load fills 16
// LDS rows of 64 bytes; which 16-byte piece of the step a lane fetches is XOR-ed with bits of
// its row, so the 128-bit operand reads spread over all banks without padding.  Lanes whose
// piece lies outside the image (padding), past the last pixel, past K or past R*S*C are given
// an offset beyond the buffer's size: the hardware range check of buffer loads then writes
// zeros into LDS for them, so padding costs no branch and no extra memory.
//
// Matrix instruction: v_mfma_i32_32x32x32_i8.  Output channels take the role of the rows of
// the first operand and pixels the columns of the second, so a lane ends up holding, for one
// pixel, accumulators of several channels.  Weight rows are placed in LDS in a permuted order
// such that those channels are 16 consecutive ones; the epilogue (ReLU, rounding shift, clamp:
// the rescale of Eq. 6 for power-of-two scales; the bias is the accumulators' start value) then
// packs them into one 16-byte store.  The 32-bit sums never leave registers unless the caller
// asks for them (acc_out).
#include "conv_ring.hpp"
#include <type_traits>

namespace dfq {

namespace {

struct MfmaParams {
    ConvArgs a;
    int M;            // N*P*Q
    int Kgemm;        // R*S*C
    int nsteps;       // ceil(Kgemm / 64)
    int tiles_c;      // channel tiles
    int tiles;        // pixel tiles * channel tiles
    unsigned x_bytes, w_bytes, y_bytes, add_bytes;
    FastDiv div_pq, div_q, div_tc;
};

// UT ("uniform taps"): C is a multiple of 64, so a 64-byte step never straddles two taps and
// the tap is the same for every lane; its bookkeeping then lives in scalar registers.
// PW ("pointwise", needs UT): R = S = 1, stride 1, no padding - output pixel m reads input pixel m,
// so a tile needs no coordinate decoding and no border masks.
// GENERAL: the epilogue may meet a ragged channel tail, an unaligned or strided-odd output row, a
// shift outside [0, 23] or an accumulator dump; the launcher picks the lean instantiation
// (GENERAL = false) whenever none of these applies.  OCC: wavefronts per SIMD to fit registers for.
// PC (excludes GENERAL): the lean epilogue with one weight format per output channel, every
// channel's shift within [0, 23] (the caller of the library vouches for the range of the formats).
// FUSE (excludes GENERAL): an element-wise add (Eq. 10) follows the convolution and is taken in the
// epilogue: the second operand's 16 codes per lane and 32 x 32 tile are loaded at the start of the
// epilogue - ordinary loads the compiler tracks, all issued before the first is used - the
// convolution result is rounded to its own format in registers, aligned with the operand at the
// finer scale and the sum rounded once more.
template <int BP, int BC, int WAVES_P, int WAVES_C, int NSTAGES, bool UT, bool PW, bool GENERAL, int OCC, bool PC = false,
          bool FUSE = false, bool LAZY = false>
__global__ void __launch_bounds__(WAVES_P * WAVES_C * 64, OCC) conv_mfma_kernel(MfmaParams prm)
{
    static_assert(!PC || !GENERAL, "the per-channel form is a lean one");
    static_assert(!FUSE || !GENERAL, "the fused add exists in the lean forms only");
    static_assert(!LAZY || (FUSE && !PC), "the single-rounding join: fused, one weight format per layer");
    static_assert(NSTAGES >= 2 && NSTAGES <= 6, "ring depth");
    static_assert(UT || !PW, "the pointwise form keeps its position in scalar registers");
    constexpr int NW = WAVES_P * WAVES_C;                 // wavefronts per workgroup
    static_assert(NW == 4 || NW == 8 || NW == 16, "4, 8 or 16 wavefronts per workgroup");
    constexpr int RPC = 64 / kPieces;                     // LDS rows filled by one wavefront-wide load (a "chunk")
    constexpr int KK = kStepBytes / 32;                   // matrix-instruction k-steps per stage
    constexpr int WP = BP / WAVES_P, WC = BC / WAVES_C;   // wavefront tile
    constexpr int PT = WP / 32, CT = WC / 32;             // 32x32 MFMA tiles per wavefront
    // chunks each wavefront loads per step; when there are fewer weight chunks than wavefronts
    // only the first BC/RPC wavefronts fetch one
    constexpr int XS = BP / (RPC * NW), WS = (BC + RPC * NW - 1) / (RPC * NW);
    constexpr bool kPartialW = BC < RPC * NW;
    static_assert(XS * RPC * NW == BP && (kPartialW || WS * RPC * NW == BC) && BC % 16 == 0, "whole chunks");
    constexpr int LPW = XS + WS;                          // loads per wavefront per step (with a weight chunk)
    constexpr int STAGE_PIECES = (BP + BC) * kPieces;
    static_assert(WP % 32 == 0 && WC % 32 == 0, "tile shape");
    static_assert(NSTAGES * LPW < 64, "outstanding loads must fit the 6-bit counter");

    extern __shared__ uint4 lds[];   // nstages stages of (BP + BC) rows of 64 bytes, then BC bias words, then 3 * BC words
                                     // of per-channel rescale constants (used with one weight format per channel)

    const ConvArgs &a = prm.a;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    constexpr int nstages = NSTAGES;
    const int nsteps = prm.nsteps;
    const bool w_active = !kPartialW || wave < BC / RPC;  // this wavefront fetches weight chunks

    // ---- this workgroup's tiles: lb, lb + G, lb + 2G, ...  Workgroup ids are dealt round-robin
    // to the 8 XCDs; renumbering them so that each XCD owns a contiguous run keeps tiles that
    // share input rows (neighbouring pixel tiles, the channel tiles of one pixel tile) in one L2.
    const int G = gridDim.x;
    int lb = blockIdx.x;
    {
        const int per = G / 8, rem = G % 8, xcd = lb % 8, idx = lb / 8;
        lb = (xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per) + idx;
    }
    // The last, incomplete round of tiles is dealt round-robin over the XCDs instead of following the
    // contiguous runs (which would put all extra tiles on the first XCDs): extra tile number j goes to
    // the workgroup with raw id b = 8 * idx + xcd where j = (idx / tc) * 8 * tc + xcd * tc + idx % tc
    // (tc = channel tiles): consecutive j cycle through the channel tiles, then the XCDs, and j has the
    // workgroup's own channel tile.  Needs G to be a multiple of 8 * tc; otherwise the strided sequence
    // lb, lb + G, ... is kept for the last round too.
    const int last_round0 = prm.tiles / G * G;                       // first tile of the incomplete round
    const bool deal_last = G % (8 * prm.tiles_c) == 0;
    const int my_extra = ((int)blockIdx.x / 8 / prm.tiles_c) * 8 * prm.tiles_c + ((int)blockIdx.x % 8) * prm.tiles_c +
                         ((int)blockIdx.x / 8) % prm.tiles_c;
    const int ntiles_mine = deal_last ? prm.tiles / G + (my_extra < prm.tiles - last_round0 ? 1 : 0)
                                      : (lb < prm.tiles ? (prm.tiles - lb + G - 1) / G : 0);
    const int nitems = ntiles_mine * nsteps;
    const int last_tile = last_round0 + my_extra;                    // this workgroup's tile of that round, if any
    // G is a multiple of the number of channel tiles, so the channel tile never changes
    const int k0 = (lb - fastdiv(lb, prm.div_tc) * prm.tiles_c) * BC;

    const v4i xrsrc = make_rsrc(a.x, prm.x_bytes);
    const v4i wrsrc = make_rsrc(a.w, prm.w_bytes);
    const __amdgpu_buffer_rsrc_t yrsrc = __builtin_amdgcn_make_buffer_rsrc(a.y, 0, GENERAL ? 0 : (int)prm.y_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t arsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(FUSE ? a.add : a.x), 0,
                                                                           FUSE ? (int)prm.add_bytes : 0, 0x00020000);
    const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) char *)(char *)&lds[0];
    int *bias_lds = (int *)(lds + nstages * STAGE_PIECES);
    int *pc_shift = bias_lds + BC, *pc_hi = pc_shift + BC, *pc_badd = pc_hi + BC;

    // ---- bias of this channel tile into LDS (re-read at every tile start without touching the
    // vector-memory counter that paces the load ring)
    for (int i = tid; i < BC; i += NW * 64) bias_lds[i] = (a.b && k0 + i < a.K) ? a.b[k0 + i] : 0;
    // one weight format per output channel: rescale constants of every channel of the tile
    if (PC) {
        for (int i = tid; i < BC; i += NW * 64) {
            const int sk = (a.shift + a.frac_w[k0 + i]) & 31;       // K % BC == 0 here; in [0, 23] by the caller's word
            pc_shift[i] = sk;
            pc_hi[i] = 127 << min(sk, 23);
            pc_badd[i] = sk > 0 ? ((1 << (sk - 1)) - 1) : 0;
        }
    }

    // ---- producer bookkeeping.  A wavefront-wide load covers RPC consecutive rows (one chunk) of
    // the stage; lane l supplies row l/4 of the chunk, physical piece l%4, which holds logical piece
    // (l%4) ^ ((row>>2)&3) - the same for every chunk of this lane; 16 consecutive rows then put
    // any one logical piece on 16 different bank groups.
    const int lrow = lane / kPieces;
    const int lp = (lane & 3) ^ ((lane >> 4) & 3);
    unsigned xoff[XS];               // byte offset of tap (0,0) of the lane's pixel, plus the lane's piece (mod 2^32)
    uint32_t rinv[XS], cinv[XS];     // bit r / bit s set: that kernel row / column falls OUTSIDE the image
    unsigned woff[WS];               // byte offset of the lane's weight row (+ piece), or out of range past K
#pragma unroll
    for (int j = 0; j < WS; j++) {
        // LDS row i = 8g + 4h + e of a 32-row group receives channel 16h + 4g + e: the matrix
        // instruction then leaves 16 consecutive channels in each lane
        const int rr = RPC * (wave + NW * j) + lrow;
        const int i32 = rr & 31;
        const int k = k0 + (rr & ~31) + 16 * ((i32 >> 2) & 1) + 4 * (i32 >> 3) + (i32 & 3);
        woff[j] = k < a.K ? (unsigned)(k * prm.Kgemm) + (UT ? (unsigned)lp * 16u : 0u) : kOutOfRange;
    }
    // position on the reduction axis.  UT: scalar tap (sr, ss), scalar channel base scb, the lane's
    // piece is already folded into xoff / woff.  Otherwise per lane: byte kb = step*64 + lp*16
    // belongs to tap (tr, ts), channel tc.
    int sr = 0, ss = 0, scb = 0, skb = 0;
    int kb = 0, tr = 0, ts = 0, tc = 0;
    int kb0 = lp * 16, tr0 = 0, ts0 = 0, tc0 = 0;
    if (!UT) {
        const int tap = kb0 / a.C;
        tc0 = kb0 - tap * a.C;
        tr0 = tap / a.S;
        ts0 = tap - tr0 * a.S;
    }
    int p_tile = lb, p_step = 0;     // tile and step the producer will fetch next

    auto begin_tile = [&]() __attribute__((always_inline)) {
        const int m0 = fastdiv(p_tile, prm.div_tc) * BP;
#pragma unroll
        for (int j = 0; j < XS; j++) {
            const int m = m0 + RPC * (wave + NW * j) + lrow;
            const bool live = m < prm.M;
            if (PW) {
                xoff[j] = live ? (unsigned)(m * a.C) + (unsigned)lp * 16u : kOutOfRange;
                continue;
            }
            const int mi = live ? m : 0;
            const int n = fastdiv(mi, prm.div_pq);
            const int pq = mi - n * (a.P * a.Q);
            const int p = fastdiv(pq, prm.div_q), q = pq - p * a.Q;
            const int ih0 = p * a.stride - a.pad, iw0 = q * a.stride - a.pad;
            xoff[j] = (unsigned)(((n * a.H + ih0) * a.W + iw0) * a.C) + (UT ? (unsigned)lp * 16u : 0u);
            // kernel rows r with 0 <= ih0 + r < H are r in [rlo, rhi); likewise columns
            const int rlo = max(0, -ih0), rhi = min(a.R, a.H - ih0);
            const int clo = max(0, -iw0), chi = min(a.S, a.W - iw0);
            rinv[j] = (live && rhi > rlo) ? ~(((1u << (rhi - rlo)) - 1u) << rlo) : 0xffffffffu;
            cinv[j] = (chi > clo) ? ~(((1u << (chi - clo)) - 1u) << clo) : 0xffffffffu;
        }
        // back to the first step of the reduction axis
        if (UT) {
            skb = 0; scb = 0; sr = 0; ss = 0;
        } else {
            kb = kb0; tr = tr0; ts = ts0; tc = tc0;
        }
    };

    auto issue = [&](int stage) __attribute__((always_inline)) {
        if (p_step == 0) begin_tile();
        const unsigned sbase = (unsigned)__builtin_amdgcn_readfirstlane(
            (int)(lds_base + (unsigned)stage * (STAGE_PIECES * 16) + (unsigned)wave * 1024u));
        if (UT) {
            const unsigned soff = PW ? (unsigned)skb : (unsigned)((sr * a.W + ss) * a.C + scb);
#pragma unroll
            for (int j = 0; j < XS; j++) {
                const unsigned bad = PW ? 0u : (unsigned)(__builtin_amdgcn_sbfe((int)rinv[j], sr, 1) | __builtin_amdgcn_sbfe((int)cinv[j], ss, 1));
                load_piece_to_lds((xoff[j] + soff) | bad, xrsrc, sbase + (unsigned)j * (NW * 1024u));
            }
            if (w_active) {
#pragma unroll
                for (int j = 0; j < WS; j++)
                    load_piece_to_lds(woff[j] + (unsigned)skb, wrsrc, sbase + (unsigned)(BP * 64) + (unsigned)j * (NW * 1024u));
            }
            skb += kStepBytes;
            if (!PW) {
                scb += kStepBytes;
                if (scb == a.C) {
                    scb = 0;
                    if (++ss == a.S) { ss = 0; ++sr; }
                }
            }
        } else {
            const unsigned toff = (unsigned)((tr * a.W + ts) * a.C + tc);
            const unsigned past = tr >= a.R ? 0xffffffffu : 0u;   // kb >= Kgemm
            const unsigned rsh = (unsigned)tr & 31u, csh = (unsigned)ts & 31u;
#pragma unroll
            for (int j = 0; j < XS; j++) {
                const unsigned bad = past | (0u - (((rinv[j] >> rsh) | (cinv[j] >> csh)) & 1u));
                load_piece_to_lds((xoff[j] + toff) | bad, xrsrc, sbase + (unsigned)j * (NW * 1024u));
            }
            if (w_active) {
#pragma unroll
                for (int j = 0; j < WS; j++)
                    load_piece_to_lds((woff[j] + (unsigned)kb) | past, wrsrc, sbase + (unsigned)(BP * 64) + (unsigned)j * (NW * 1024u));
            }
            kb += kStepBytes;
            tc += kStepBytes;
            for (int i = 0; i < kStepBytes / 16; i++) {   // a step crosses at most four taps (C >= 16)
                const bool wrapc = tc >= a.C;
                tc -= wrapc ? a.C : 0;
                ts += wrapc ? 1 : 0;
                const bool wraps = ts == a.S;
                ts = wraps ? 0 : ts;
                tr += wraps ? 1 : 0;
            }
        }
        if (++p_step == nsteps) {
            p_step = 0;
            p_tile += G;
            if (deal_last && p_tile >= last_round0) p_tile = last_tile;
        }
    };

    const int wp0 = (wave % WAVES_P) * WP;
    const int wc0 = (wave / WAVES_P) * WC;
    const int l32 = lane & 31, lh = lane >> 5;
    const int swz = (l32 >> 2) & 3;
    // every stage of the ring is filled before the first item is read
#pragma unroll
    for (int i = 0; i < nstages; i++)
        if (i < nitems) issue(i);

    Requant rq, rq2;
    rq.init(a.shift, a.relu);
    rq2.init(FUSE ? a.add_shift : 1, a.add_relu);
    __syncthreads();   // bias_lds and the per-channel constants complete

    // accumulators start at the bias: register r of a lane belongs to channel kc + r
    v16i acc[CT][PT];
    auto reset_acc = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int c = 0; c < CT; c++) {
            const int4 *bp = (const int4 *)(bias_lds + wc0 + c * 32 + 16 * lh);
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
    reset_acc();

    // Operands of one step as the matrix instruction wants them: one register set per 32-byte half.
    struct Half {
        v4i w[CT];
        v4i x[PT];
    };
    Half f0, f1;
    auto read_half = [&](Half &f, int kk, int stage) __attribute__((always_inline)) {
        const v4i *xs = (const v4i *)lds + stage * STAGE_PIECES;
        const v4i *ws = xs + BP * kPieces;
        const int g = (kk * 2 + lh) ^ swz;   // physical piece
#pragma unroll
        for (int c = 0; c < CT; c++) f.w[c] = ws[(wc0 + c * 32 + l32) * kPieces + g];
#pragma unroll
        for (int p = 0; p < PT; p++) f.x[p] = xs[(wp0 + p * 32 + l32) * kPieces + g];
    };
    auto mfma_half = [&](const Half &f) __attribute__((always_inline)) {
#pragma unroll
        for (int c = 0; c < CT; c++)
#pragma unroll
            for (int p = 0; p < PT; p++)
                acc[c][p] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f.w[c], f.x[p], acc[c][p], 0, 0, 0);
    };
    // Workgroup barrier that first completes this wavefront's own LDS reads and waits for no
    // vector-memory operation (the load ring is paced separately).
    auto ring_barrier = [&]() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };

    // The pacing of the load ring counts outstanding vector-memory operations, and the stores
    // of an epilogue are among them (loads and stores complete in issue order).  ep_hist has bit k
    // set when item i-1-k ended a tile whose epilogue issued exactly kStoresPerTile stores; the
    // loads awaited in item i were issued in item i+1-nstages ahead of that item's epilogue, so
    // the epilogues of the last nstages-1 items are younger than they are.  Stores that are not
    // counted only make a wait longer, never too short.
    constexpr int kStoresPerTile = CT * PT;
    constexpr unsigned kHistMask = (1u << (NSTAGES - 1)) - 1u;
    unsigned ep_hist = 0;
    const unsigned lane_yoff = (unsigned)((wp0 + l32) * a.ldy + k0 + wc0 + 16 * lh);   // lean form: y fits 31 bits
    const unsigned lane_aoff = (unsigned)((wp0 + l32) * a.ldadd + k0 + wc0 + 16 * lh);
    int c_step = 0, c_tile = lb;
    auto finish_item = [&]() __attribute__((always_inline)) {
        ep_hist = (ep_hist << 1) & kHistMask;
        if (++c_step == nsteps) {
            // ---- epilogue of this tile: lane holds, per (c, p), channels kc..kc+15 of pixel m
            const int m0 = fastdiv(c_tile, prm.div_tc) * BP;
            settle_accumulators<CT * PT>(&acc[0][0]);
            if (!GENERAL) {
                const unsigned tile_off = (unsigned)(m0 * a.ldy);
                v4u other[FUSE ? CT * PT : 1];
                if constexpr (FUSE) {
                    // rows past the last pixel are outside the buffer: zeros arrive, and their stores are dropped
                    const unsigned add_off = lane_aoff + (unsigned)(m0 * a.ldadd);
#pragma unroll
                    for (int c = 0; c < CT; c++)
#pragma unroll
                        for (int p = 0; p < PT; p++)
                            other[c * PT + p] = __builtin_amdgcn_raw_buffer_load_b128(arsrc, (int)(add_off + (unsigned)(p * 32 * a.ldadd + c * 32)), 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }
                if constexpr (PC) {
                    // groups of four channels; the constants of the next group are fetched while this one is
                    // rescaled, and the scheduler is kept from hoisting all fetches to the front (registers)
                    const int kr0 = wc0 + 16 * lh;
                    int4 sv = *(const int4 *)(pc_shift + kr0), hv = *(const int4 *)(pc_hi + kr0), bv = *(const int4 *)(pc_badd + kr0);
#pragma unroll
                    for (int c = 0; c < CT; c++) {
                        uint32_t o[PT][4];
#pragma unroll
                        for (int r4 = 0; r4 < 4; r4++) {
                            const int g = c * 4 + r4 + 1;                       // next group
                            const int kn = wc0 + (g / 4) * 32 + 16 * lh + 4 * (g % 4);
                            int4 sn = sv, hn = hv, bn = bv;
                            if (g < CT * 4) {
                                sn = *(const int4 *)(pc_shift + kn);
                                hn = *(const int4 *)(pc_hi + kn);
                                bn = *(const int4 *)(pc_badd + kn);
                            }
                            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                            for (int p = 0; p < PT; p++) {
                                if constexpr (FUSE)
                                    o[p][r4] = requant_add_four_per_channel(acc[c][p][4 * r4], acc[c][p][4 * r4 + 1], acc[c][p][4 * r4 + 2],
                                                                            acc[c][p][4 * r4 + 3], sv, hv, bv, a.relu, other[c * PT + p][r4],
                                                                            a.add_sa, a.add_sb, rq2);
                                else
                                    o[p][r4] = requant_four_per_channel(acc[c][p][4 * r4], acc[c][p][4 * r4 + 1], acc[c][p][4 * r4 + 2],
                                                                        acc[c][p][4 * r4 + 3], sv, hv, bv, a.relu);
                            }
                            __builtin_amdgcn_sched_barrier(0);
                            sv = sn; hv = hn; bv = bn;
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
                            if constexpr (FUSE) {
                                const v4i oth = {(int)other[c * PT + p][0], (int)other[c * PT + p][1], (int)other[c * PT + p][2],
                                                 (int)other[c * PT + p][3]};
                                if constexpr (LAZY) store_piece(add_tile_lane_lazy(acc[c][p], oth, a.add_sb, rq2), off, yrsrc);
                                else store_piece(requant_add_tile_lane(acc[c][p], rq, oth, a.add_sa, a.add_sb, rq2), off, yrsrc);
                            } else {
                                store_piece(requant_tile_lane_fast(acc[c][p], rq), off, yrsrc);
                            }
                        }
                }
                ep_hist |= 1u;
            } else {
#pragma unroll
                for (int c = 0; c < CT; c++) {
                    const int kc = k0 + wc0 + c * 32 + 16 * lh;
#pragma unroll
                    for (int p = 0; p < PT; p++) {
                        const int m = m0 + wp0 + p * 32 + l32;
                        if (m < prm.M && kc < a.K) store_tile_lane_general(acc[c][p], a, a.shift, a.relu, m, kc);
                    }
                }
            }
            reset_acc();
            c_step = 0;
            c_tile += G;
            if (deal_last && c_tile >= last_round0) c_tile = last_tile;
        }
    };
    // Item i multiplies step i in KK = 2 k-steps of 32 bytes.  Two register sets alternate: while
    // one is multiplied the other is filled with the operands two k-steps ahead, i.e. those of
    // stage i+1.  Before the first read of stage i+1 the wavefront waits for its own loads of that
    // stage and meets the others at the barrier; every wavefront has then also completed its last
    // read of stage i, so REFILL may overwrite stage i with item i + nstages - it is issued behind
    // the second k-step's matrix instructions, so that a wavefront held up at a full address queue
    // of the memory pipeline still has its matrix work queued.  LDS latency, the barrier and the
    // address arithmetic of the loads all run in the shadow of the matrix pipe.
    auto do_item = [&](auto refill, auto has_next, auto wait, int stage) __attribute__((always_inline)) {
        const int next = stage + 1 == nstages ? 0 : stage + 1;
#pragma unroll
        for (int kk = 0; kk < KK; kk++) {
            Half &f = (kk & 1) ? f1 : f0;
            mfma_half(f);
            __builtin_amdgcn_sched_barrier(0);
            if (kk == KK - 2 && decltype(has_next)::value) {
                wait();
                ring_barrier();
            }
            if (kk == KK - 1 && decltype(refill)::value) issue(stage);
            // the operands two k-steps ahead go into the registers just consumed
            if (kk + 2 < KK) read_half(f, kk + 2, stage);
            else if (decltype(has_next)::value) read_half(f, kk + 2 - KK, next);
            __builtin_amdgcn_sched_barrier(0);
        }
        finish_item();
    };

    // steady state: after the wait nstages-2 younger items stay in flight, after the refill
    // nstages-1.  Unrolled over the ring so that every LDS address and every load destination is
    // a compile-time offset.  The last nstages items drain the ring.
    auto steady_wait = [&]() __attribute__((always_inline)) {
        const int younger_epilogues = __builtin_popcount(ep_hist);
        if (w_active) wait_loads_plus<(nstages - 2) * LPW, kStoresPerTile>(younger_epilogues);
        else wait_loads_plus<(nstages - 2) * XS, kStoresPerTile>(younger_epilogues);
    };
    auto drain_wait_for = [&](int ahead) __attribute__((always_inline)) {
        if (w_active) wait_ahead<LPW>(ahead);
        else wait_ahead<XS>(ahead);
    };
    if (nitems > 0) {
        drain_wait_for(min(nitems, nstages) - 1);
        ring_barrier();
        read_half(f0, 0, 0);
        read_half(f1, 1, 0);
    }
    const int steady = nitems - nstages;     // items that refill their stage
    int it = 0;
    for (; it + nstages <= steady; it += nstages) {
#pragma unroll
        for (int s = 0; s < nstages; s++) do_item(std::true_type{}, std::true_type{}, steady_wait, s);
    }
    int stage = 0;   // it is a multiple of nstages here
    for (; it < steady; it++) {
        do_item(std::true_type{}, std::true_type{}, steady_wait, stage);
        stage = stage + 1 == nstages ? 0 : stage + 1;
    }
    for (; it < nitems - 1; it++) {
        const int ahead = nitems - 2 - it;   // items younger than the one awaited
        do_item(std::false_type{}, std::true_type{}, [&]() __attribute__((always_inline)) { drain_wait_for(ahead); }, stage);
        stage = stage + 1 == nstages ? 0 : stage + 1;
    }
    if (it < nitems) do_item(std::false_type{}, std::false_type{}, steady_wait, stage);
}

inline hipError_t big_lds(void (*k)(MfmaParams))
{
    if (!k) return hipSuccess;
    return hipFuncSetAttribute((const void *)k, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
}

// NSTAGES ring stages of (BP + BC) * 64 bytes plus the bias and the per-channel rescale tables (four
// words per channel of the tile) must fit the LDS share of a workgroup: 160 KB / (workgroups per
// compute unit).
// PER_CU: workgroups per compute unit the kernel is built and launched for (1 or 2)
// The per-channel lean form holds a group's rescale constants in registers on top of everything
// else: it is built for the tile shapes whose register budget has room for them (wavefront tiles of
// 64 x 64 at no more than three wavefronts per SIMD).
template <int BP, int BC, int WAVES_P, int WAVES_C, int NSTAGES, bool UT, bool PW, int OCC, bool FUSE = false>
constexpr void (*per_channel_kernel())(MfmaParams)
{
    if constexpr (OCC <= 3 && (BP / WAVES_P) * (BC / WAVES_C) <= 64 * 64)
        return conv_mfma_kernel<BP, BC, WAVES_P, WAVES_C, NSTAGES, UT, PW, false, OCC, true, FUSE>;
    else
        return nullptr;
}

template <int BP, int BC, int WAVES_P, int WAVES_C, int NSTAGES, int PER_CU>
hipError_t launch_cfg(const ConvArgs &a, hipStream_t st)
{
    MfmaParams prm;
    prm.a = a;
    const long long M = (long long)a.N * a.P * a.Q;
    prm.M = (int)M;
    prm.Kgemm = a.R * a.S * a.C;
    prm.nsteps = (prm.Kgemm + kStepBytes - 1) / kStepBytes;
    prm.tiles_c = (a.K + BC - 1) / BC;
    const long long tiles = ((M + BP - 1) / BP) * prm.tiles_c;
    if (tiles > 0x7fffffffLL) return hipErrorInvalidValue;
    prm.tiles = (int)tiles;
    prm.x_bytes = (unsigned)((long long)a.N * a.H * a.W * a.C);
    prm.w_bytes = (unsigned)((long long)a.K * prm.Kgemm);
    const long long y_bytes = M * a.ldy;
    prm.y_bytes = y_bytes < (1LL << 31) ? (unsigned)y_bytes : 0u;
    prm.add_bytes = a.add ? (unsigned)(M * a.ldadd) : 0u;
    prm.div_pq = make_fastdiv(a.P * a.Q);
    prm.div_q = make_fastdiv(a.Q);
    prm.div_tc = make_fastdiv(prm.tiles_c);

    int grid = PER_CU * kNumCU;
    if (grid > prm.tiles) grid = prm.tiles;
    grid = grid / prm.tiles_c * prm.tiles_c;            // the channel tile of a workgroup must not change
    if (grid < prm.tiles_c) grid = prm.tiles_c;
    constexpr size_t lds_bytes = (size_t)NSTAGES * (BP + BC) * kStepBytes + BC * 4 * 4;   // rings, bias, three per-channel tables
    static_assert(lds_bytes * PER_CU <= kLdsBytes, "rings do not fit the LDS");

    constexpr int occ = PER_CU * WAVES_P * WAVES_C / 4;
    using K = void (*)(MfmaParams);
    const bool ut = a.C % kStepBytes == 0;
    const bool pw = ut && a.R == 1 && a.S == 1 && a.stride == 1 && a.pad == 0;
    static const K kernels[12] = {conv_mfma_kernel<BP, BC, WAVES_P, WAVES_C, NSTAGES, false, false, false, occ>,
                                 conv_mfma_kernel<BP, BC, WAVES_P, WAVES_C, NSTAGES, false, false, true, occ>,
                                 conv_mfma_kernel<BP, BC, WAVES_P, WAVES_C, NSTAGES, true, false, false, occ>,
                                 conv_mfma_kernel<BP, BC, WAVES_P, WAVES_C, NSTAGES, true, false, true, occ>,
                                 conv_mfma_kernel<BP, BC, WAVES_P, WAVES_C, NSTAGES, true, true, false, occ>,
                                 conv_mfma_kernel<BP, BC, WAVES_P, WAVES_C, NSTAGES, true, true, true, occ>,
                                 per_channel_kernel<BP, BC, WAVES_P, WAVES_C, NSTAGES, true, false, occ>(),
                                 per_channel_kernel<BP, BC, WAVES_P, WAVES_C, NSTAGES, true, true, occ>(),
                                 per_channel_kernel<BP, BC, WAVES_P, WAVES_C, NSTAGES, false, false, occ>(),
                                 // unpadded 1x1 stride-1 layers with the add behind them fused into the epilogue
                                 conv_mfma_kernel<BP, BC, WAVES_P, WAVES_C, NSTAGES, true, true, false, occ, false, true>,
                                 per_channel_kernel<BP, BC, WAVES_P, WAVES_C, NSTAGES, true, true, occ, true>(),
                                 // ... with the single-rounding join
                                 conv_mfma_kernel<BP, BC, WAVES_P, WAVES_C, NSTAGES, true, true, false, occ, false, true, true>};
    static const hipError_t attr[12] = {big_lds(kernels[0]), big_lds(kernels[1]), big_lds(kernels[2]), big_lds(kernels[3]),
                                        big_lds(kernels[4]), big_lds(kernels[5]), big_lds(kernels[6]), big_lds(kernels[7]),
                                        big_lds(kernels[8]), big_lds(kernels[9]), big_lds(kernels[10]), big_lds(kernels[11])};
    // shifts the epilogue will meet: one, or with per-channel weight formats the declared range
    const int s_lo = a.shift + (a.frac_w ? a.frac_w_lo : 0), s_hi = a.shift + (a.frac_w ? a.frac_w_hi : 0);
    const bool general = !((!a.frac_w || kernels[6]) && s_lo >= 0 && s_hi <= 23 && !a.acc_out && a.y && (a.ldy & 15) == 0 &&
                           ((uintptr_t)a.y & 15) == 0 && a.K % BC == 0 && y_bytes < (1LL << 31));
    int which = (!general && a.frac_w) ? (pw ? 7 : ut ? 6 : 8) : (pw ? 4 : ut ? 2 : 0) + (general ? 1 : 0);
    if (a.add) {
        // conv_mfma_fuses() has vouched for the lean pointwise form
        if (general || !pw || (a.frac_w && !kernels[10])) return hipErrorInvalidValue;
        which = a.frac_w ? 10 : a.add_lazy ? 11 : 9;
    }
    if (attr[which] != hipSuccess) return attr[which];
    K kernel = kernels[which];
    kernel<<<(unsigned)grid, WAVES_P * WAVES_C * 64, lds_bytes, st>>>(prm);
    return hipGetLastError();
}

}  // namespace

bool conv_mfma_supports(const ConvArgs &a)
{
    if (a.groups != 1) return false;
    if (a.C % 16) return false;
    if (a.R > 31 || a.S > 31) return false;     // per-pixel row / column validity masks are 32 bits wide
    // 32-bit byte offsets with the top bit reserved for "out of range"
    if ((long long)a.N * a.H * a.W * a.C >= (1LL << 31)) return false;
    if ((long long)a.K * a.R * a.S * a.C >= (1LL << 31)) return false;
    if ((long long)a.N * a.P * a.Q >= (1LL << 31) - 512) return false;
    if (((uintptr_t)a.x & 15) || ((uintptr_t)a.w & 15)) return false;
    if (a.acc_out && ((uintptr_t)a.acc_out & 15)) return false;
    return true;
}

// The fused add (a.add set) exists for unpadded 1x1 stride-1 layers with whole 64-byte steps and whole
// channel tiles of any tile shape (K a multiple of 256), in the lean epilogue.
bool conv_mfma_fuses(const ConvArgs &a)
{
    if (!a.add || !conv_mfma_supports(a)) return false;
    if (a.R != 1 || a.S != 1 || a.stride != 1 || a.pad != 0 || a.C % kStepBytes || a.K % 256) return false;
    const int s_lo = a.shift + (a.frac_w ? a.frac_w_lo : 0), s_hi = a.shift + (a.frac_w ? a.frac_w_hi : 0);
    if (s_lo < 0 || s_hi > 23 || a.acc_out || !a.y || (a.ldy & 15) || ((uintptr_t)a.y & 15)) return false;
    const long long M = (long long)a.N * a.P * a.Q;
    if (M * a.ldy >= (1LL << 31) || M * a.ldadd >= (1LL << 31)) return false;
    if (a.frac_w && M <= 1024) return false;      // the tile shape for very few pixels has no per-channel lean form
    if (((uintptr_t)a.add & 15) || (a.ldadd & 15) || a.ldadd < a.K) return false;
    if (!(a.add_shift >= 0 && a.add_shift <= 23) || a.add_sa < 0 || a.add_sa > 22 || a.add_sb < 0 || a.add_sb > 22) return false;
    if (a.add_lazy && a.frac_w) return false;
    return true;
}

hipError_t launch_conv_mfma(const ConvArgs &a, hipStream_t st)
{
    // Measured choices at batch 256 (wavefronts own 64 x 64 outputs unless noted):
    // K <= 64: 256 x 64 tiles (four wavefronts); for kernels larger than 1x1 three workgroups per CU
    //          with a two-stage ring beat two with three stages (more independent workgroups to
    //          overlap epilogues with matrix work);
    // K a multiple of 256, at least 192 tiles of 256 x 256, not a strided kernel larger than 1x1:
    //          those tiles, eight wavefronts of 64 x 128, one workgroup per CU - half the LDS fill
    //          traffic per matrix instruction and half the re-reads of the input (4-12 % faster on
    //          the 14x14 layers and the strided 1x1 shortcuts; with fewer tiles too many CUs stay
    //          idle, and strided 3x3 layers were 8 % slower);
    // else:    256 x 128 tiles (eight wavefronts), two workgroups per CU, for kernels larger than 1x1 with enough of them;
    //          for 1x1 kernels (few items per tile) 128 x 128 tiles (four wavefronts), three per CU.
    const bool pointwise = a.R == 1 && a.S == 1;
    // very few pixels (fully connected layers): one wavefront per 32 x 32 tile, each with its own deep ring and no
    // barrier, where that kernel applies (unpadded 1x1, whole 64-byte steps); else 64 x 64 tiles, wavefronts of 32 x 32,
    // so that the channel tiles alone spread over more compute units, with a ring six stages deep
    if ((long long)a.N * a.P * a.Q <= 1024 && a.K > 64) {
        if (conv_fc_supports(a)) return launch_conv_fc(a, st);
        return launch_cfg<64, 64, 2, 2, 6, 2>(a, st);
    }
    // one weight format per output channel: the tile shapes for which that epilogue is built
    if (a.frac_w && a.K > 64) return launch_cfg<128, 128, 2, 2, 3, 3>(a, st);
    if (a.K <= 64) return pointwise ? launch_cfg<256, 64, 4, 1, 3, 2>(a, st) : launch_cfg<256, 64, 4, 1, 2, 3>(a, st);
    if (a.K % 256 == 0 && (pointwise || a.stride == 1)) {
        const long long M = (long long)a.N * a.P * a.Q;
        if ((M + 255) / 256 * (a.K / 256) >= 192) return launch_cfg<256, 256, 4, 2, 3, 1>(a, st);
    }
    // kernels larger than 1x1 whose 256 x 128 tiles would occupy at most half of the compute units: 128 x 128 tiles, twice as
    // many workgroups (7 x 7 x 512 -> 512, 3x3, at batch 128: 34.0 -> 28.5 us; at batch 256, with 196 such tiles, the
    // smaller tiles were slower, 39.7 -> 45.8 us)
    if (!pointwise && ((long long)a.N * a.P * a.Q + 255) / 256 * ((a.K + 127) / 128) <= kNumCU / 2)
        return launch_cfg<128, 128, 2, 2, 3, 3>(a, st);
    return pointwise ? launch_cfg<128, 128, 2, 2, 3, 3>(a, st) : launch_cfg<256, 128, 4, 2, 3, 2>(a, st);
}

}  // namespace dfq
