// Row-wise helpers shared by the decode kernels: 16 lanes cover one cached row, each lane holds
// EPL = d/16 consecutive elements as floats; online-softmax states are merged with the usual rule.
#pragma once
#include "common.h"

namespace zipvl {

template <typename T, int EPL> struct RowChunk;      // EPL consecutive elements of a row as floats
template <> struct RowChunk<__bf16, 8> {
    __device__ static __forceinline__ void load(const __bf16* p, float (&f)[8]) {
        const uintx4 v = load16(p);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            f[2 * e] = __uint_as_float(v[e] << 16);
            f[2 * e + 1] = __uint_as_float(v[e] & 0xFFFF0000u);
        }
    }
};
template <> struct RowChunk<__bf16, 4> {
    __device__ static __forceinline__ void load(const __bf16* p, float (&f)[4]) {
        const uintx2 v = *reinterpret_cast<const uintx2*>(p);
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            f[2 * e] = __uint_as_float(v[e] << 16);
            f[2 * e + 1] = __uint_as_float(v[e] & 0xFFFF0000u);
        }
    }
};
template <> struct RowChunk<float, 8> {
    __device__ static __forceinline__ void load(const float* p, float (&f)[8]) {
        const floatx4 a = *reinterpret_cast<const floatx4*>(p), b = *reinterpret_cast<const floatx4*>(p + 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) { f[e] = a[e]; f[4 + e] = b[e]; }
    }
};
template <> struct RowChunk<float, 4> {
    __device__ static __forceinline__ void load(const float* p, float (&f)[4]) {
        const floatx4 a = *reinterpret_cast<const floatx4*>(p);
#pragma unroll
        for (int e = 0; e < 4; ++e) f[e] = a[e];
    }
};

// merge (m2, l2, o2) into (m, l, o)
template <int EPL>
__device__ __forceinline__ void merge_state(float& m, float& l, float (&o)[EPL], float m2, float l2, const float (&o2)[EPL]) {
    const float M = fmaxf(m, m2);
    if (M == -INFINITY) return;
    const float a = fast_exp2(m - M), b = fast_exp2(m2 - M);
    l = l * a + l2 * b;
#pragma unroll
    for (int e = 0; e < EPL; ++e) o[e] = o[e] * a + o2[e] * b;
    m = M;
}

// Storage word of the codes of EPL consecutive elements at BITS bits each (element e in bits
// [e*BITS, e*BITS + BITS) of the little-endian word).
template <int EPL, int BITS> struct CodeWord;
template <> struct CodeWord<8, 4> { using type = uint32_t; };
template <> struct CodeWord<8, 2> { using type = uint16_t; };
template <> struct CodeWord<4, 4> { using type = uint16_t; };
template <> struct CodeWord<4, 2> { using type = uint8_t; };

}  // namespace zipvl
