// Pieces shared by the matrix-core convolution kernels that feed the int8 matrix instructions from a
// ring of LDS stages filled by direct global -> LDS loads: the geometry constants, the buffer
// resource, the load / store primitives and the waits on the vector-memory counter.
#pragma once
#include "conv_epilogue.hpp"

namespace dfq {

constexpr int kStepBytes = 64;   // bytes of the reduction axis per LDS stage (the width of an LDS row)
constexpr int kPieces = 4;       // 16-byte pieces per LDS row
constexpr unsigned kOutOfRange = 0x80000000u;   // any offset with this bit set is past either buffer

constexpr int kNumCU = 256;
constexpr int kLdsBytes = 160 * 1024;

// Buffer resource for raw byte addressing with range checking (stride 0: offsets >= bytes read as 0).
__device__ __forceinline__ v4i make_rsrc(const void *base, unsigned bytes)
{
    const unsigned long long p = (unsigned long long)base;
    v4i r;
    r.x = __builtin_amdgcn_readfirstlane((int)(unsigned)(p & 0xffffffffu));
    r.y = __builtin_amdgcn_readfirstlane((int)(unsigned)((p >> 32) & 0xffffu));
    r.z = __builtin_amdgcn_readfirstlane((int)bytes);
    r.w = __builtin_amdgcn_readfirstlane(0x00020000);   // 32-bit raw data format
    return r;
}

// Direct global -> LDS load of 16 bytes per lane: lane l's data lands at lds_base + 16*l; a lane
// whose offset is outside the buffer gets zeros.  Issued through inline assembly so that the
// compiler's own wait-count bookkeeping does not serialize it against later LDS reads;
// completion is awaited explicitly with wait_loads<>().
__device__ __forceinline__ void load_piece_to_lds(unsigned voffset, v4i rsrc, unsigned lds_base)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tbuffer_load_dwordx4 %0, %1, 0 offen lds" ::"v"(voffset), "s"(rsrc), "s"(lds_base)
                 : "memory", "m0");
}

// 16-byte store through a buffer resource: a lane whose offset is outside the buffer stores
// nothing, so rows past the last pixel need no branch and every wavefront issues the same number
// of stores per tile (the pacing of the load ring counts them).
typedef unsigned v4u __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void store_piece(uint4 d, unsigned voffset, __amdgpu_buffer_rsrc_t rsrc)
{
    const v4u data = {d.x, d.y, d.z, d.w};
    __builtin_amdgcn_raw_buffer_store_b128(data, rsrc, (int)voffset, 0, 0);
}

// 16-byte load into registers through a buffer resource, outside the compiler's wait-count
// bookkeeping like the LDS loads: the data may be used only behind wait_loads_for<N>() on the same
// registers, and that wait must follow in the SAME block of straight-line code - the compiler
// believes the registers are written at once, so any register copy or spill it places between the
// load and the wait (loop boundaries, merges of branches) would read them too early.  A lane whose
// offset is outside the buffer gets zeros.
__device__ __forceinline__ void load_piece_to_regs(v4i &dst, unsigned voffset, v4i rsrc)
{
    asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen" : "=&v"(dst) : "v"(voffset), "s"(rsrc) : "memory");
}

// wait until at most N vector-memory operations are outstanding; the registers passed are marked as
// written here, so that no use of them can be scheduled ahead of the wait
template <int N>
__device__ __forceinline__ void wait_loads_for(v4i &a, v4i &b, v4i &c, v4i &d)
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt %4" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : "n"((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8)));
}

// wait until at most N vector-memory operations of this wavefront are outstanding
template <int N>
__device__ __forceinline__ void wait_loads()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// wait until only the loads of the next `ahead` (0..5) steps, LP loads each, are outstanding
template <int LP>
__device__ __forceinline__ void wait_ahead(int ahead)
{
    switch (ahead) {
        case 0: wait_loads<0>(); break;
        case 1: wait_loads<LP>(); break;
        case 2: wait_loads<2 * LP>(); break;
        case 3: wait_loads<3 * LP>(); break;
        case 4: wait_loads<4 * LP>(); break;
        default: wait_loads<5 * LP>(); break;
    }
}

// at most BASE + SP * cnt outstanding, for 0 <= cnt <= 5 (larger cnt waits as for 5)
template <int BASE, int SP>
__device__ __forceinline__ void wait_loads_plus(int cnt)
{
    static_assert(BASE + 5 * SP < 64, "vmcnt is a 6-bit counter");
    switch (cnt) {
        case 0: wait_loads<BASE>(); break;
        case 1: wait_loads<BASE + SP>(); break;
        case 2: wait_loads<BASE + 2 * SP>(); break;
        case 3: wait_loads<BASE + 3 * SP>(); break;
        case 4: wait_loads<BASE + 4 * SP>(); break;
        default: wait_loads<BASE + 5 * SP>(); break;
    }
}

}  // namespace dfq
