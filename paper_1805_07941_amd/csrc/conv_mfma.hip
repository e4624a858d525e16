// Dense quantized convolution as an implicit GEMM on the gfx950 int8 matrix cores.
//
// The sum of Eq. 6 for groups == 1 is a matrix product  acc[k][m] = sum_j Wm[k][j] * Xm[j][m]
// with m running over the N*P*Q output pixels and j over the R*S*C (tap, input channel) pairs.
// In NHWC the C channels of one tap are contiguous, and a weight row [R][S][C] is contiguous
// in exactly the same (tap, channel) order, so both operands are fetched as 16-byte pieces
// that cover the same 16 values of j; taps outside the image are fetched as zeros (the code
// of the value 0).  Nothing is materialized: the im2col matrix exists only as LDS tiles.
//
// Per workgroup (256 lanes = 4 wavefronts): a BP-pixel x BC-channel output tile; the j range
// is walked in steps of 64 bytes through two LDS stages (one barrier per step; the global
// loads of step i+1 are in flight while step i is multiplied).  LDS rows are 64 bytes with
// the 16-byte piece index XOR-ed with bits of the row so that both the 128-bit stores and the
// 128-bit operand reads spread over all banks without padding.
//
// Matrix instruction: v_mfma_i32_32x32x32_i8.  Output channels take the role of the rows of
// the first operand and pixels the columns of the second, so a lane ends up holding, for one
// pixel, accumulators of several channels.  Weight rows are placed in LDS in a permuted order
// such that those channels are 16 consecutive ones; the epilogue (bias, ReLU, rounding shift,
// clamp: the rescale of Eq. 6 for power-of-two scales) then packs them into one 16-byte store.
// The 32-bit sums never leave registers unless the caller asks for them (acc_out).
#include "conv_epilogue.hpp"

namespace dfq {

namespace {

constexpr int kThreads = 256;
constexpr int kStepBytes = 64;   // bytes of the reduction axis per LDS stage
constexpr int kPieces = 4;       // 16-byte pieces per LDS row

struct MfmaParams {
    ConvArgs a;
    long long M;      // N*P*Q
    int Kgemm;        // R*S*C
    int nsteps;       // ceil(Kgemm / 64)
    int tiles_c;      // channel tiles
    long long tiles_p;
};

// position of (row, piece) inside a tile of 64-byte rows, in 16-byte units
__device__ __forceinline__ int lds_slot(int row, int piece) { return row * kPieces + (piece ^ ((row >> 2) & 3)); }

// LDS row (MFMA row index) of weight row c within a 32-channel group, chosen so that the
// accumulators a lane holds are those of 16 consecutive channels.
__device__ __forceinline__ int weight_row(int c)
{
    int c32 = c & 31;
    return (c & ~31) + 8 * ((c32 & 15) >> 2) + 4 * (c32 >> 4) + (c32 & 3);
}

template <int BP, int BC, int WAVES_P, int WAVES_C>
__global__ void __launch_bounds__(kThreads) conv_mfma_kernel(MfmaParams prm)
{
    static_assert(WAVES_P * WAVES_C == 4, "four wavefronts per workgroup");
    constexpr int WP = BP / WAVES_P, WC = BC / WAVES_C;   // wavefront tile
    constexpr int PT = WP / 32, CT = WC / 32;             // 32x32 MFMA tiles per wavefront
    constexpr int XI = BP / 64, WI = BC / 64 > 0 ? BC / 64 : 1;  // 16-byte loads per lane per step
    constexpr bool kHalfW = BC < 64;                      // BC == 32: only half the lanes load weights
    static_assert(WP % 32 == 0 && WC % 32 == 0, "tile shape");

    __shared__ uint4 lds[2][(BP + BC) * kPieces];

    const ConvArgs &a = prm.a;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;

    // ---- which tile: spread consecutive tile numbers over the 8 XCDs in contiguous runs, so
    // that workgroups sharing input rows (neighbouring pixel tiles, all channel tiles of one
    // pixel tile) meet in the same L2.
    long long nblk = (long long)gridDim.x;
    long long bid = blockIdx.x;
    {
        long long per = nblk / 8, rem = nblk % 8, xcd = bid % 8, idx = bid / 8;
        bid = (xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per) + idx;
    }
    const int tile_c = (int)(bid % prm.tiles_c);
    const long long tile_p = bid / prm.tiles_c;
    const long long m0 = tile_p * BP;
    const int k0 = tile_c * BC;

    // ---- per-lane load bookkeeping
    const int piece = tid & 3;      // which 16 bytes of the 64-byte step
    const int lrow = tid >> 2;      // 0..63
    const int8_t *ximg[XI];
    int ih0[XI], iw0[XI];
    const long long PQ = (long long)a.P * a.Q;
#pragma unroll
    for (int i = 0; i < XI; i++) {
        long long m = m0 + lrow + 64 * i;
        if (m < prm.M) {
            long long n = m / PQ;
            int pq = (int)(m - n * PQ);
            int p = pq / a.Q, q = pq - p * a.Q;
            ximg[i] = a.x + (size_t)n * a.H * a.W * a.C;
            ih0[i] = p * a.stride - a.pad;
            iw0[i] = q * a.stride - a.pad;
        } else {
            ximg[i] = a.x;
            ih0[i] = -(1 << 28);    // never inside the image
            iw0[i] = 0;
        }
    }
    const int8_t *wrow[WI];
    bool wok[WI];
#pragma unroll
    for (int i = 0; i < WI; i++) {
        int k = k0 + lrow + 64 * i;
        wok[i] = k < a.K && (!kHalfW || lrow < 32);
        wrow[i] = a.w + (size_t)(wok[i] ? k : 0) * prm.Kgemm;
    }
    // reduction-axis position of this lane's piece: byte kb = step*64 + piece*16 = (tap r,s; channel c)
    int kb = piece * 16;
    int tr, ts, tc;
    {
        int tap = kb / a.C;
        tc = kb - tap * a.C;
        tr = tap / a.S;
        ts = tap - tr * a.S;
    }

    uint4 xreg[XI], wreg[WI];
    auto load_global = [&]() {
        const bool kin = tr < a.R;   // kb < Kgemm
#pragma unroll
        for (int i = 0; i < XI; i++) {
            int ih = ih0[i] + tr, iw = iw0[i] + ts;
            bool ok = kin && (unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)a.W;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (ok) v = *(const uint4 *)(ximg[i] + ((size_t)ih * a.W + iw) * a.C + tc);
            xreg[i] = v;
        }
#pragma unroll
        for (int i = 0; i < WI; i++) {
            uint4 v = make_uint4(0, 0, 0, 0);
            if (wok[i] && kin) v = *(const uint4 *)(wrow[i] + kb);
            wreg[i] = v;
        }
    };
    auto advance = [&]() {
        kb += kStepBytes;
        tc += kStepBytes;
        while (tc >= a.C) {
            tc -= a.C;
            if (++ts == a.S) { ts = 0; ++tr; }
        }
    };
    auto store_lds = [&](int buf) {
        uint4 *xs = lds[buf];
        uint4 *ws = xs + BP * kPieces;
#pragma unroll
        for (int i = 0; i < XI; i++) xs[lds_slot(lrow + 64 * i, piece)] = xreg[i];
#pragma unroll
        for (int i = 0; i < WI; i++)
            if (!kHalfW || lrow < 32) ws[lds_slot(weight_row(lrow + 64 * i), piece)] = wreg[i];
    };

    const int wp0 = (wave % WAVES_P) * WP;
    const int wc0 = (wave / WAVES_P) * WC;
    const int l32 = lane & 31, lh = lane >> 5;
    const int swz = (l32 >> 2) & 3;

    // ---- accumulators start at the bias: register r of a lane belongs to channel kc + r
    v16i acc[CT][PT];
#pragma unroll
    for (int c = 0; c < CT; c++) {
        const int kc = k0 + wc0 + c * 32 + 16 * lh;
#pragma unroll
        for (int r = 0; r < 16; r++) {
            const int bv = (a.b && kc + r < a.K) ? a.b[kc + r] : 0;
#pragma unroll
            for (int p = 0; p < PT; p++) acc[c][p][r] = bv;
        }
    }

    load_global();
    store_lds(0);
    __syncthreads();

    for (int step = 0; step < prm.nsteps; step++) {
        const int buf = step & 1;
        const bool more = step + 1 < prm.nsteps;
        if (more) {
            advance();
            load_global();
        }
        const v4i *xs = (const v4i *)lds[buf];
        const v4i *ws = xs + BP * kPieces;
#pragma unroll
        for (int kk = 0; kk < 2; kk++) {
            const int g = (kk * 2 + lh) ^ swz;
            v4i wf[CT], xf[PT];
#pragma unroll
            for (int c = 0; c < CT; c++) wf[c] = ws[(wc0 + c * 32 + l32) * kPieces + g];
#pragma unroll
            for (int p = 0; p < PT; p++) xf[p] = xs[(wp0 + p * 32 + l32) * kPieces + g];
#pragma unroll
            for (int c = 0; c < CT; c++)
#pragma unroll
                for (int p = 0; p < PT; p++)
                    acc[c][p] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[c], xf[p], acc[c][p], 0, 0, 0);
        }
        if (more) store_lds(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: lane holds, per (c, p) tile, channels kc..kc+15 of pixel m
    Requant rq;
    rq.init(a.shift, a.relu);
    const bool vec_ok = ((a.ldy & 15) == 0) && (((uintptr_t)a.y & 15) == 0);
#pragma unroll
    for (int c = 0; c < CT; c++) {
        const int kc = k0 + wc0 + c * 32 + 16 * lh;
#pragma unroll
        for (int p = 0; p < PT; p++) {
            const long long m = m0 + wp0 + p * 32 + l32;
            if (m < prm.M && kc < a.K) store_tile_lane(acc[c][p], a, rq, m, kc, vec_ok);
        }
    }
}

template <int BP, int BC, int WAVES_P, int WAVES_C>
hipError_t launch_cfg(const ConvArgs &a, hipStream_t st)
{
    MfmaParams prm;
    prm.a = a;
    prm.M = (long long)a.N * a.P * a.Q;
    prm.Kgemm = a.R * a.S * a.C;
    prm.nsteps = (prm.Kgemm + kStepBytes - 1) / kStepBytes;
    prm.tiles_c = (a.K + BC - 1) / BC;
    prm.tiles_p = (prm.M + BP - 1) / BP;
    long long blocks = prm.tiles_p * prm.tiles_c;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    conv_mfma_kernel<BP, BC, WAVES_P, WAVES_C><<<(unsigned)blocks, kThreads, 0, st>>>(prm);
    return hipGetLastError();
}

}  // namespace

bool conv_mfma_supports(const ConvArgs &a)
{
    if (a.groups != 1) return false;
    if (a.C % 16) return false;
    if (((uintptr_t)a.x & 15) || ((uintptr_t)a.w & 15)) return false;
    if (a.acc_out && ((uintptr_t)a.acc_out & 15)) return false;
    return true;
}

hipError_t launch_conv_mfma(const ConvArgs &a, hipStream_t st)
{
    if (a.K <= 32) return launch_cfg<256, 32, 4, 1>(a, st);
    if (a.K <= 64) return launch_cfg<256, 64, 4, 1>(a, st);
    return launch_cfg<128, 128, 2, 2>(a, st);
}

}  // namespace dfq
