// Convolution with few input channels (the first layer of a network: C = 3) on the int8
// matrix cores.
//
// With NHWC and a small C, the S taps of one kernel row r are S*C CONTIGUOUS bytes of the
// input row (channels of pixel iw0, then of iw0+1, ...).  When S*C <= 32 that run is used as
// one 32-byte block of the reduction axis of Eq. 6: the block for (output pixel, r) is simply
// the 32 bytes starting at x[n, ih, iw0, 0]; the weight block for (k, r) is w[k, r, :, :]
// followed by zeros, so whatever the input bytes beyond S*C hold is multiplied by 0.  The
// reduction is then R blocks long (7 for a 7x7 kernel) instead of R*S*C padded tap by tap.
//
// The pixel operand is read straight from global memory in matrix-operand layout (each lane
// one unaligned 16-byte load per block; neighbouring output pixels overlap heavily, so these
// hit in L1/L2); only the small packed weight tensor lives in LDS, loaded once per workgroup,
// which then walks over pixel tiles (persistent grid).  A run that crosses the left or right
// image border is read from the nearest 16 bytes inside the row and shifted into place, which
// both zero-fills the padding and keeps every access inside the tensor.
//
// Neighbouring output pixels' runs overlap (they start stride*C bytes apart), and the memory
// pipeline does not merge overlapping unaligned 16-byte pieces: such a wavefront load costs one
// L1 access per lane.  The second kernel below (conv_smallc_rows_kernel) therefore fetches, per
// kernel row and 32-pixel group, the contiguous span of input bytes that the group's runs cover
// with ONE dword-per-lane load straight into LDS (aligned, coalesced, out-of-image dwords zero
// filled by the buffer range check) and lets every lane pick its 16 bytes out of LDS with five
// dword reads and a byte-funnel shift.  It needs rows of a multiple of 4 bytes, at least 32 output
// pixels per row, and spans that fit 64 dwords; the first kernel remains for the rest.
#include "conv_ring.hpp"

namespace dfq {

namespace {

constexpr int kThreads = 256;
constexpr int kTilePixels = 256;   // 4 wavefronts x 64 pixels

struct SmallCParams {
    ConvArgs a;
    int M;              // N*P*Q  (< 2^31)
    int tiles_p;
    int run;            // S*C, bytes of one kernel row
    int rowlen;         // W*C
    FastDiv div_pq, div_q;
};

template <int CT>   // channel tile = CT * 32
__global__ void __launch_bounds__(kThreads, 2) conv_smallc_kernel(SmallCParams prm)
{
    constexpr int BC = CT * 32;
    extern __shared__ uint4 wlds[];   // [R][BC][2] 16-byte pieces, piece index XOR-ed with bit 3 of k

    const ConvArgs &a = prm.a;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, lh = lane >> 5;
    const int k0 = blockIdx.y * BC;

    // ---- packed weights into LDS: block (r, k) = w[k][r][0 .. run) then zeros
    {
        int8_t *wb = (int8_t *)wlds;
        const int total = a.R * BC * 32;
        for (int i = tid; i < total; i += kThreads) {
            int j = i & 31;
            int kl = (i >> 5) % BC;
            int r = (i >> 5) / BC;
            int k = k0 + kl;
            int8_t v = 0;
            if (j < prm.run && k < a.K) v = a.w[((size_t)k * a.R + r) * prm.run + j];
            // LDS row of channel kl follows the same permutation as the dense kernel: a lane's
            // 16 accumulators are 16 consecutive channels
            int c32 = kl & 31;
            int row = (kl & ~31) + 8 * ((c32 & 15) >> 2) + 4 * (c32 >> 4) + (c32 & 3);
            int piece = (j >> 4) ^ ((row >> 3) & 1);
            wb[((r * BC + row) * 2 + piece) * 16 + (j & 15)] = v;
        }
    }
    __syncthreads();

    Requant rq;
    rq.init(a.shift, a.relu);
    const bool fast = epilogue_is_fast(a, rq, k0 + BC);
    // one weight format per output channel: a lane's channels are the same for every tile, so their
    // shifts are read once
    const bool pc_packed = epilogue_is_per_channel_packed(a, k0 + BC);
    __shared__ int pc_shift[CT * 32];
    if (pc_packed) {
        for (int i = threadIdx.x; i < CT * 32; i += blockDim.x) pc_shift[i] = a.shift + a.frac_w[k0 + i];
        __syncthreads();
    }
    const v4i *wl = (const v4i *)wlds;

    int bias[CT][16];
#pragma unroll
    for (int c = 0; c < CT; c++) load_bias16(a, k0 + c * 32 + 16 * lh, bias[c]);

    for (int tile = blockIdx.x; tile < prm.tiles_p; tile += gridDim.x) {
        const int mbase = tile * kTilePixels + wave * 64;
        const int8_t *rowptr[2];   // address of the lane's 16 bytes in kernel row r = 0
        int ih0[2], rb[2];         // first input row; byte offset of the run inside its row (may be < 0)
        bool any_border[2];
#pragma unroll
        for (int p = 0; p < 2; p++) {
            int m = mbase + p * 32 + l32;
            if (m >= prm.M) m = prm.M - 1;              // duplicate work for the ragged tail, never stored
            int n = fastdiv(m, prm.div_pq);
            int pq = m - n * (a.P * a.Q);
            int pp = fastdiv(pq, prm.div_q);
            int q = pq - pp * a.Q;
            ih0[p] = pp * a.stride - a.pad;
            rb[p] = (q * a.stride - a.pad) * a.C;
            rowptr[p] = a.x + ((long long)n * a.H + ih0[p]) * prm.rowlen + rb[p] + 16 * lh;
            any_border[p] = __any(rb[p] < 0 || rb[p] + 32 > prm.rowlen);   // uniform over the 32-pixel tile pair of lanes
        }

        v16i acc[CT][2];
#pragma unroll
        for (int c = 0; c < CT; c++)
#pragma unroll
            for (int p = 0; p < 2; p++)
#pragma unroll
                for (int r = 0; r < 16; r++) acc[c][p][r] = bias[c][r];

        for (int r = 0; r < a.R; r++) {
            v4i xf[2];
#pragma unroll
            for (int p = 0; p < 2; p++) {
                const int ih = ih0[p] + r;
                const bool row_ok = (unsigned)ih < (unsigned)a.H;
                const int8_t *src = rowptr[p] + (long long)r * prm.rowlen;
                v4i v = {0, 0, 0, 0};
                if (!any_border[p]) {
                    if (row_ok) __builtin_memcpy(&v, src, 16);
                } else if (row_ok) {
                    // piece covers row bytes [o, o+16); bytes outside [0, rowlen) are padding.  The
                    // 16 bytes are read from the nearest position that lies wholly inside the row
                    // and shifted into place, which zero-fills the padding.
                    const int o = rb[p] + 16 * lh;
                    const int oc = min(max(o, 0), prm.rowlen - 16);
                    unsigned __int128 t;
                    __builtin_memcpy(&t, src - o + oc, 16);
                    const int sh = o - oc;          // > 0: piece starts right of what was read
                    if (sh >= 16 || sh <= -16) t = 0;
                    else if (sh > 0) t >>= 8 * sh;
                    else if (sh < 0) t <<= 8 * (-sh);
                    __builtin_memcpy(&v, &t, 16);
                }
                xf[p] = v;
            }
#pragma unroll
            for (int c = 0; c < CT; c++) {
                const int row = c * 32 + l32;
                const v4i wf = wl[(r * BC + row) * 2 + (lh ^ ((row >> 3) & 1))];
#pragma unroll
                for (int p = 0; p < 2; p++)
                    acc[c][p] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf, xf[p], acc[c][p], 0, 0, 0);
            }
        }

        settle_accumulators<CT * 2>(&acc[0][0]);
#pragma unroll
        for (int c = 0; c < CT; c++) {
            const int kc = k0 + c * 32 + 16 * lh;
#pragma unroll
            for (int p = 0; p < 2; p++) {
                const int m = mbase + p * 32 + l32;
                if (m < prm.M) {
                    if (fast) store_tile_lane_fast(acc[c][p], a, rq, m, kc);
                    else if (pc_packed) {
                        int sh[16];
#pragma unroll
                        for (int r4 = 0; r4 < 4; r4++) {
                            const int4 t = *(const int4 *)(pc_shift + c * 32 + 16 * lh + 4 * r4);
                            sh[4 * r4] = t.x; sh[4 * r4 + 1] = t.y; sh[4 * r4 + 2] = t.z; sh[4 * r4 + 3] = t.w;
                        }
                        store_tile_lane_per_channel(acc[c][p], a, sh, a.relu, m, kc);
                    }
                    else if (kc < a.K) store_tile_lane_general(acc[c][p], a, a.shift, a.relu, m, kc);
                }
            }
        }
    }
}


// 4 bytes per lane straight into LDS: lane l's dword lands at lds_base + 4*l; out-of-range lanes give 0.
__device__ __forceinline__ void load_dword_to_lds(unsigned voffset, v4i rsrc, unsigned lds_base)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tbuffer_load_dword %0, %1, 0 offen lds" ::"v"(voffset), "s"(rsrc), "s"(lds_base)
                 : "memory", "m0");
}

struct SmallCRowsParams {
    SmallCParams p;
    unsigned x_bytes;
    int row_dwords;     // W*C / 4
};

constexpr int kGroupBytes = 256;   // LDS bytes one 32-pixel group's span of one kernel row occupies

template <int CT>   // channel tile = CT * 32
__global__ void __launch_bounds__(kThreads, 2) conv_smallc_rows_kernel(SmallCRowsParams rp)
{
    constexpr int BC = CT * 32;
    // [R][BC][2] packed weight pieces (as in the first kernel), then per wavefront
    // [2 tiles in flight][R][2 groups][kGroupBytes] span bytes, then 16 bytes of slack
    extern __shared__ uint4 wlds[];
    const SmallCParams &prm = rp.p;
    const ConvArgs &a = prm.a;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, lh = lane >> 5;
    const int k0 = blockIdx.y * BC;
    {
        int8_t *wb = (int8_t *)wlds;
        const int total = a.R * BC * 32;
        for (int i = tid; i < total; i += kThreads) {
            int j = i & 31;
            int kl = (i >> 5) % BC;
            int r = (i >> 5) / BC;
            int k = k0 + kl;
            int8_t v = 0;
            if (j < prm.run && k < a.K) v = a.w[((size_t)k * a.R + r) * prm.run + j];
            int c32 = kl & 31;
            int row = (kl & ~31) + 8 * ((c32 & 15) >> 2) + 4 * (c32 >> 4) + (c32 & 3);
            int piece = (j >> 4) ^ ((row >> 3) & 1);
            wb[((r * BC + row) * 2 + piece) * 16 + (j & 15)] = v;
        }
    }
    __syncthreads();

    Requant rq;
    rq.init(a.shift, a.relu);
    const bool fast = epilogue_is_fast(a, rq, k0 + BC);
    // one weight format per output channel: a lane's channels are the same for every tile, so their
    // shifts are read once
    const bool pc_packed = epilogue_is_per_channel_packed(a, k0 + BC);
    __shared__ int pc_shift[CT * 32];
    if (pc_packed) {
        for (int i = threadIdx.x; i < CT * 32; i += blockDim.x) pc_shift[i] = a.shift + a.frac_w[k0 + i];
        __syncthreads();
    }
    const v4i *wl = (const v4i *)wlds;
    const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) char *)(char *)&wlds[0];
    const unsigned span_base = (unsigned)(a.R * BC * 32) + (unsigned)wave * (unsigned)(2 * a.R * 2 * kGroupBytes);
    const char *span_lds = (const char *)wlds + span_base;
    const v4i xrsrc = make_rsrc(a.x, rp.x_bytes);

    int bias[CT][16];
#pragma unroll
    for (int c = 0; c < CT; c++) load_bias16(a, k0 + c * 32 + 16 * lh, bias[c]);

    // what a lane needs to know about one tile: for the loads, where its dword of each group's
    // span lies; for the reads, where its pixel's run starts inside the group's LDS bytes
    struct TileInfo {
        int off0[2];      // byte offset in x of the lane's span dword in kernel row 0 (meaningful for rows inside the image)
        int ih0[2];       // input row of kernel row 0 for the lane's span segment
        int rd[2];        // byte offset of the lane's 16 bytes inside the group's LDS block
    };
    auto describe = [&](int tile, TileInfo &ti) __attribute__((always_inline)) {
        const int mbase = tile * kTilePixels + wave * 64;
#pragma unroll
        for (int p = 0; p < 2; p++) {
            int m = min(mbase + p * 32 + l32, prm.M - 1);          // pixels past the end repeat the last one, never stored
            const int n = fastdiv(m, prm.div_pq);
            const int pq = m - n * (a.P * a.Q);
            const int pp = fastdiv(pq, prm.div_q);
            const int q = pq - pp * a.Q;
            const int rowid = n * a.P + pp;
            const int rb = (q * a.stride - a.pad) * a.C;            // run start inside the input row, may be < 0
            // segment A: pixels in the output row of the group's first pixel; segment B: the rest (the next
            // output row - a group of 32 spans at most two since Q >= 32)
            const int rowidA = __builtin_amdgcn_readlane(rowid, 0);
            const bool inB = rowid != rowidA;
            const unsigned long long maskB = __ballot(inB) & 0xffffffffull;
            const int firstB = maskB ? (int)__builtin_ctzll(maskB) : 32;
            const int rbA = __builtin_amdgcn_readlane(rb, 0);
            const int rbLastA = __builtin_amdgcn_readlane(rb, firstB - 1);
            const int d0A = rbA >> 2;                               // floor: rbA may be negative
            const int nA = (rbLastA + 32 - 4 * d0A + 3) >> 2;       // dwords of segment A
            const int fb = min(firstB, 31);
            const int rbB = __builtin_amdgcn_readlane(rb, fb);
            const int d0B = rbB >> 2;
            const int ihA = __builtin_amdgcn_readlane(pp, 0) * a.stride - a.pad;
            const int ihB = __builtin_amdgcn_readlane(pp, fb) * a.stride - a.pad;
            const int nImgA = __builtin_amdgcn_readlane(n, 0), nImgB = __builtin_amdgcn_readlane(n, fb);
            // loader view: lane = dword index of the span
            const bool ldB = lane >= nA;
            const int d = ldB ? d0B + (lane - nA) : d0A + lane;
            const bool dv = d >= 0 && d < rp.row_dwords && (!ldB || firstB < 32);
            // kernel row 0 may lie above the image (negative offset): used only for rows that pass the test below
            ti.off0[p] = ((ldB ? nImgB : nImgA) * a.H + (ldB ? ihB : ihA)) * prm.rowlen + 4 * d;
            ti.ih0[p] = dv ? (ldB ? ihB : ihA) : -0x40000000;       // a dword outside the row fails every row test
            // reader view: lane = (pixel l32, half lh)
            ti.rd[p] = (inB ? 4 * nA + (rb - 4 * d0B) : (rb - 4 * d0A)) + 16 * lh;
        }
    };
    auto issue_tile = [&](const TileInfo &ti, int buf) __attribute__((always_inline)) {
        for (int r = 0; r < a.R; r++) {
#pragma unroll
            for (int p = 0; p < 2; p++) {
                const bool ok = (unsigned)(ti.ih0[p] + r) < (unsigned)a.H;
                const unsigned off = ok ? (unsigned)ti.off0[p] + (unsigned)(r * prm.rowlen) : kOutOfRange;
                const unsigned dst = (unsigned)__builtin_amdgcn_readfirstlane(
                    (int)(lds_base + span_base + (unsigned)(((buf * a.R + r) * 2 + p) * kGroupBytes)));
                load_dword_to_lds(off, xrsrc, dst);
            }
        }
    };
    auto wait_tile = [&](bool next_in_flight) __attribute__((always_inline)) {
        if (!next_in_flight) { wait_loads<0>(); return; }
        switch (a.R) {          // 2 * R loads of the next tile may stay outstanding
            case 1: wait_loads<2>(); break;
            case 2: wait_loads<4>(); break;
            case 3: wait_loads<6>(); break;
            case 4: wait_loads<8>(); break;
            case 5: wait_loads<10>(); break;
            case 6: wait_loads<12>(); break;
            case 7: wait_loads<14>(); break;
            default: wait_loads<0>(); break;
        }
    };

    TileInfo cur, nxt;
    int tile = blockIdx.x;
    int buf = 0;
    if (tile < prm.tiles_p) {
        describe(tile, cur);
        issue_tile(cur, 0);
    }
    for (; tile < prm.tiles_p; tile += gridDim.x) {
        const int tile_next = tile + gridDim.x;
        const bool has_next = tile_next < prm.tiles_p;
        if (has_next) {
            describe(tile_next, nxt);
            issue_tile(nxt, buf ^ 1);
        }
        wait_tile(has_next);

        v16i acc[CT][2];
#pragma unroll
        for (int c = 0; c < CT; c++)
#pragma unroll
            for (int p = 0; p < 2; p++)
#pragma unroll
                for (int r = 0; r < 16; r++) acc[c][p][r] = bias[c][r];

        for (int r = 0; r < a.R; r++) {
            v4i xf[2];
#pragma unroll
            for (int p = 0; p < 2; p++) {
                const int at = ((buf * a.R + r) * 2 + p) * kGroupBytes + cur.rd[p];
                const uint32_t *src = (const uint32_t *)(span_lds + (at & ~3));
                const unsigned sh = (unsigned)(at & 3) * 8u;
                uint32_t w[5];
#pragma unroll
                for (int d = 0; d < 5; d++) w[d] = src[d];
#pragma unroll
                for (int d = 0; d < 4; d++)
                    xf[p][d] = (int)(uint32_t)((((unsigned long long)w[d + 1] << 32) | w[d]) >> sh);
            }
#pragma unroll
            for (int c = 0; c < CT; c++) {
                const int row = c * 32 + l32;
                const v4i wf = wl[(r * BC + row) * 2 + (lh ^ ((row >> 3) & 1))];
#pragma unroll
                for (int p = 0; p < 2; p++)
                    acc[c][p] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf, xf[p], acc[c][p], 0, 0, 0);
            }
        }

        const int mbase = tile * kTilePixels + wave * 64;
        settle_accumulators<CT * 2>(&acc[0][0]);
#pragma unroll
        for (int c = 0; c < CT; c++) {
            const int kc = k0 + c * 32 + 16 * lh;
#pragma unroll
            for (int p = 0; p < 2; p++) {
                const int m = mbase + p * 32 + l32;
                if (m < prm.M) {
                    if (fast) store_tile_lane_fast(acc[c][p], a, rq, m, kc);
                    else if (pc_packed) {
                        int sh[16];
#pragma unroll
                        for (int r4 = 0; r4 < 4; r4++) {
                            const int4 t = *(const int4 *)(pc_shift + c * 32 + 16 * lh + 4 * r4);
                            sh[4 * r4] = t.x; sh[4 * r4 + 1] = t.y; sh[4 * r4 + 2] = t.z; sh[4 * r4 + 3] = t.w;
                        }
                        store_tile_lane_per_channel(acc[c][p], a, sh, a.relu, m, kc);
                    }
                    else if (kc < a.K) store_tile_lane_general(acc[c][p], a, a.shift, a.relu, m, kc);
                }
            }
        }
        cur = nxt;
        buf ^= 1;
    }
}

}  // namespace

// the row-staging kernel's extra conditions (see the comment at the top)
static bool rows_kernel_ok(const ConvArgs &a)
{
    if ((a.W * a.C) % 4 || a.Q < 32 || a.R > 7) return false;
    if ((long long)a.N * a.H * a.W * a.C >= (1LL << 31)) return false;
    if ((uintptr_t)a.x & 3) return false;
    const int sc = a.stride * a.C;
    auto dw = [&](int k) { return k > 0 ? ((k - 1) * sc + 32 + 3 + 3) / 4 : 0; };   // dwords a segment of k pixels may need
    for (int k = 1; k <= 32; k++)
        if (dw(k) + dw(32 - k) > 64) return false;
    return true;
}

bool conv_smallc_supports(const ConvArgs &a)
{
    if (a.groups != 1) return false;
    if (a.S * a.C > 32) return false;
    if ((size_t)a.R * (a.K > 32 ? 64 : 32) * 32 > 64 * 1024) return false;   // the packed weights of a channel tile live in LDS
    if (a.W * a.C < 32) return false;                       // clamped border loads need a row of >= 16 bytes
    if ((long long)a.N * a.P * a.Q >= (1LL << 31) - 512) return false;
    if (a.acc_out && ((uintptr_t)a.acc_out & 15)) return false;
    return true;
}

hipError_t launch_conv_smallc(const ConvArgs &a, hipStream_t st)
{
    SmallCParams prm;
    prm.a = a;
    prm.M = (int)((long long)a.N * a.P * a.Q);
    prm.tiles_p = (prm.M + kTilePixels - 1) / kTilePixels;
    prm.run = a.S * a.C;
    prm.rowlen = a.W * a.C;
    prm.div_pq = make_fastdiv(a.P * a.Q);
    prm.div_q = make_fastdiv(a.Q);
    const bool wide = a.K > 32;
    const int BC = wide ? 64 : 32;
    dim3 grid((unsigned)min(prm.tiles_p, 256 * 4), (unsigned)((a.K + BC - 1) / BC));
    size_t lds = (size_t)a.R * BC * 32;
    if (lds > 64 * 1024) return hipErrorInvalidValue;
    if (rows_kernel_ok(a)) {
        SmallCRowsParams rp;
        rp.p = prm;
        rp.x_bytes = (unsigned)((long long)a.N * a.H * a.W * a.C);
        rp.row_dwords = prm.rowlen / 4;
        const size_t lds2 = lds + (size_t)(kThreads / 64) * 2 * a.R * 2 * kGroupBytes + 16;
        if (lds2 <= 64 * 1024) {
            if (wide) conv_smallc_rows_kernel<2><<<grid, kThreads, lds2, st>>>(rp);
            else conv_smallc_rows_kernel<1><<<grid, kThreads, lds2, st>>>(rp);
            return hipGetLastError();
        }
    }
    if (wide) conv_smallc_kernel<2><<<grid, kThreads, lds, st>>>(prm);
    else conv_smallc_kernel<1><<<grid, kThreads, lds, st>>>(prm);
    return hipGetLastError();
}

}  // namespace dfq
