// Global memory straight to LDS, and the counted waits that go with it (gfx950).
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

namespace lpm {

#define LPM_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
// wait until at most n of this wavefront's vector-memory operations are outstanding
#define LPM_WAIT_VM(n) __builtin_amdgcn_s_waitcnt(0x0f70 | ((n) & 15) | (((n) >> 4) << 14))

// 16 bytes per lane from a buffer straight into LDS: lane l's data lands at LDS byte address dst + 16 l (dst
// wave-uniform, handed over in M0); an offset outside the buffer stores zeros.  Issued as assembly so that the
// compiler keeps no record of loads in flight that target LDS: its own bookkeeping would make every LDS
// transpose read wait for all of them, and the kernel orders the two sides itself (a count wait on the
// vector-memory counter, then a workgroup barrier, before a stage is read).
typedef unsigned int u32x4_ __attribute__((ext_vector_type(4)));
__device__ __forceinline__ u32x4_ buffer_words(const void* base, unsigned bytes) {
    const unsigned long long a = (unsigned long long)base;
    const u32x4_ r = {(unsigned)a, (unsigned)(a >> 32) & 0xffffu, bytes, 0x00020000u};
    return r;
}
__device__ __forceinline__ void load_to_lds16(u32x4_ rs, const unsigned char* dst, unsigned off) {
    const unsigned d = (unsigned)(uintptr_t)LPM_LDS_PTR(dst);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :
                 : "s"(d), "v"(off), "s"(rs)
                 : "memory");
    // M0 is not on the clobber list on purpose: the compiler treats it as a reserved register (it rejects the entry with
    // "clobber list contains reserved registers: m0"), which means it never keeps a value in M0 across statements and
    // writes M0 itself immediately before each instruction of its own that reads it.  Were that to change, the weight
    // gradients of the patch-based kernel would land in the wrong LDS stage: its layer-level parity tests compare every
    // output element with the fp64 result and would fail.
}

// wait until at most min(rem, MAXT) * LPT of this wavefront's loads are outstanding (the count is an immediate)
template <int LPT, int MAXT>
__device__ __forceinline__ void wait_tiles_behind(int rem) {
    static_assert(MAXT <= 6 && MAXT * LPT < 64, "six cases, 6-bit counter");
    if (rem >= MAXT) { LPM_WAIT_VM(MAXT * LPT); return; }
    switch (rem) {
        case 0: LPM_WAIT_VM(0); break;
        case 1: LPM_WAIT_VM(1 * LPT); break;
        case 2: LPM_WAIT_VM(2 * LPT); break;
        case 3: LPM_WAIT_VM(3 * LPT); break;
        case 4: LPM_WAIT_VM(4 * LPT); break;
        default: LPM_WAIT_VM(5 * LPT); break;
    }
}

}  // namespace lpm
