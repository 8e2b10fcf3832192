// Shared device-side helpers for the gfx950 kernels (64-wide wavefronts, MFMA).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "zipvl.h"
#include "zipvl_bench.h"

namespace zipvl {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));
typedef uint32_t uintx2 __attribute__((ext_vector_type(2)));

constexpr float kLog2e = 1.4426950408889634f;

int set_error(int code, const char* fmt, ...);
int check_launch(const char* what);

// One 16-byte operand fragment per lane.  A 32x32 MFMA tile is fed by 64 lanes:
// lane = (row or column index i = lane % 32, half h = lane / 32).
//   bf16: the fragment holds 8 consecutive elements  [16*c + 8*h, +8)  of row i
//         and feeds one v_mfma_f32_32x32x16_bf16.
//   fp32: the fragment holds 4 consecutive elements  [8*c + 4*h, +4)   of row i
//         and feeds four v_mfma_f32_32x32x2_f32 (element t in step t).  The
//         contraction order is permuted the same way for both operands, which
//         leaves the sum unchanged.
template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int kBytes = 4;
    static constexpr int kPerFrag = 4;     // elements per 16-byte fragment
    static constexpr int kPerChunk = 8;    // contraction elements covered by the two halves
};
template <> struct Elem<__bf16> {
    static constexpr int kBytes = 2;
    static constexpr int kPerFrag = 8;
    static constexpr int kPerChunk = 16;
};

template <typename T>
__device__ __forceinline__ floatx16 mma_frag(const uintx4& a, const uintx4& b, floatx16 acc);

template <>
__device__ __forceinline__ floatx16 mma_frag<__bf16>(const uintx4& a, const uintx4& b, floatx16 acc) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                   __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
}
template <>
__device__ __forceinline__ floatx16 mma_frag<float>(const uintx4& a, const uintx4& b, floatx16 acc) {
    floatx4 fa = __builtin_bit_cast(floatx4, a);
    floatx4 fb = __builtin_bit_cast(floatx4, b);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[0], fb[0], acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[1], fb[1], acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[2], fb[2], acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[3], fb[3], acc, 0, 0, 0);
    return acc;
}

// Row of the 32x32 accumulator held in register r of a lane with half h.
__device__ __forceinline__ int acc_row(int r, int h) { return 8 * (r >> 2) + 4 * h + (r & 3); }

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ uintx4 load16(const void* p) { return *reinterpret_cast<const uintx4*>(p); }
__device__ __forceinline__ void store16(void* p, const uintx4& v) { *reinterpret_cast<uintx4*>(p) = v; }

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    floatx2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// acc + lo + hi of a packed bf16 pair (the values as rounded to bf16, accumulated in fp32)
__device__ __forceinline__ float add_bf16x2(uint32_t packed, float acc) {
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, packed), ones, acc, false);
}

}  // namespace zipvl
