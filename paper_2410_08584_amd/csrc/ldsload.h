// Global -> LDS loads that do not pass through registers, shared by the attention and score kernels.
#pragma once
#include "common.h"

namespace zipvl {

// byte offset of logical 16-byte chunk `c` in a swizzled LDS row (sw = the row's swizzle): rows are unpadded, and
// the XOR makes consecutive rows read at the same logical chunk hit different bank groups
__device__ __forceinline__ int swz_chunk(int c, int sw) { return (c ^ sw) << 4; }

// Row swizzle of a tile whose rows are read 32 at a time at one logical chunk (key rows): the LDS
// serves a 16-byte-per-lane read 16 lanes per clock from 64 banks (256 bytes), so 16 consecutive rows must
// land on 16 different chunks of that period: rows of 256 bytes or more XOR the chunk index with (row & 15),
// rows of 128 bytes (two to a period, already apart by half of it) with ((row >> 1) & 7).
template <int RB>
__device__ __forceinline__ int k_row_swizzle(int row) { return RB >= 256 ? (row & 15) : ((row >> 1) & 7); }


__device__ __forceinline__ unsigned lds_address(const char* p) {
    return (unsigned)(uintptr_t)(const __attribute__((address_space(3))) char*)p;
}

#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
// One 1-KiB direct-to-LDS load of the wave: lane L's 16 bytes at gbase + goff land at LDS byte
// lds_base + 16 L (gbase and lds_base wave-uniform, goff a per-lane byte offset below 4 GiB).
// global_load_lds_dwordx4 takes the LDS base from M0 (named as clobbered on purpose: nothing else here
// uses M0).  The instruction is written out rather than taken from the builtin because the compiler,
// while such a load is pending, turns every LDS-read wait into a wait for ALL outstanding LDS reads,
// which stalls the matrix pipeline on each operand fetch; completion is awaited explicitly (vmcnt)
// before the barrier that hands the buffer to its readers.
__device__ __forceinline__ void load_kib_to_lds(const char* gbase, int goff, unsigned lds_base) {
    const unsigned m0v = __builtin_amdgcn_readfirstlane(lds_base);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(m0v), "v"(goff), "s"(gbase) : "memory", "m0");
}

// The same load, placed by data flow instead of by program order: it is tied to a register (`pin`, passed
// through unchanged) so that it issues after the instruction that produced `pin` and before the one that
// consumes it, without ordering the surrounding LDS reads the way a statement with side effects would.
// The buffers written must not be read before a barrier that is preceded by a wait for all of the wave's loads.
__device__ __forceinline__ void load_kib_to_lds_pinned(const char* gbase, int goff, unsigned lds_base, unsigned& pin) {
    const unsigned m0v = __builtin_amdgcn_readfirstlane(lds_base);
    asm("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3"
        : "+v"(pin) : "s"(m0v), "v"(goff), "s"(gbase) : "m0");
}
#pragma clang diagnostic pop

}  // namespace zipvl
