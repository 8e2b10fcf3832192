// Decode-phase attention against the (evicted) KV cache (Eq. (5); Algorithm 2).
// Memory-bound: one query per head, every cached row read exactly once.
// Split-KV: grid = (splits, units); inside a workgroup 16 lanes cover one
// cached row (16 bytes each at d = 128 bf16), so a wave reads 4 rows per step
// as full 256-byte lines, reduces the dot product over the 16 lanes with
// shuffles and keeps an online-softmax state per row group; row groups, waves
// and finally splits are merged with the usual (max, sum, weighted output)
// rule.  All query heads of a KV group are served from the same read.
#include "launch.h"
#include "rowops.h"

namespace zipvl {

constexpr int kDecMaxSplit = 64;

// One cached row against the GT queries of the group: kf / vf are this lane's EPL elements of the row.
template <int EPL, int GT>
__device__ __forceinline__ void attend_row(bool valid, const float (&kf)[EPL], const float (&vf)[EPL],
                                           const float (&qv)[GT][EPL], float (&m)[GT], float (&l)[GT], float (&o)[GT][EPL]) {
#pragma unroll
    for (int t = 0; t < GT; ++t) {
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) s += qv[t][e] * kf[e];
        s += __shfl_xor(s, 1); s += __shfl_xor(s, 2); s += __shfl_xor(s, 4); s += __shfl_xor(s, 8);
        if (valid) {
            const float m_new = fmaxf(m[t], s);
            const float a = fast_exp2(m[t] - m_new), p = fast_exp2(s - m_new);
            l[t] = l[t] * a + p;
#pragma unroll
            for (int e = 0; e < EPL; ++e) o[t][e] = o[t][e] * a + p * vf[e];
            m[t] = m_new;
        }
    }
}

// this lane's EPL elements of the group's queries, pre-multiplied by the softmax scale (log2 domain)
template <typename T, int D, int GT>
__device__ __forceinline__ void load_queries(const T* q, int b, int g, int G, int Hq, int gbase, int sub, float c,
                                             float (&qv)[GT][D / 16]) {
    constexpr int EPL = D / 16;
#pragma unroll
    for (int t = 0; t < GT; ++t) {
        const int hh = gbase + t;
        if (hh < G) {
            RowChunk<T, EPL>::load(q + ((int64_t)(b * Hq + g * G + hh)) * D + sub * EPL, qv[t]);
#pragma unroll
            for (int e = 0; e < EPL; ++e) qv[t][e] *= c;
        } else {
#pragma unroll
            for (int e = 0; e < EPL; ++e) qv[t][e] = 0.f;
        }
    }
}

// Merge the 4 row groups of every wave, then the 4 waves, and write the workgroup's partial state.
// partial layout: [(unit*G + head_in_group) * nsplit + split][D + 2]  (o[D], m, l), log2 domain
template <int D, int GT>
__device__ __forceinline__ void write_partial(float (&m)[GT], float (&l)[GT], float (&o)[GT][D / 16], float (&red)[4][GT][D + 2],
                                              int u, int G, int gbase, int split, int nsplit, float* part) {
    constexpr int EPL = D / 16;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, sub = lane & 15, rg = lane >> 4;
#pragma unroll
    for (int t = 0; t < GT; ++t) {
#pragma unroll
        for (int off = 16; off <= 32; off <<= 1) {
            const float m2 = __shfl_xor(m[t], off), l2 = __shfl_xor(l[t], off);
            float o2[EPL];
#pragma unroll
            for (int e = 0; e < EPL; ++e) o2[e] = __shfl_xor(o[t][e], off);
            merge_state<EPL>(m[t], l[t], o[t], m2, l2, o2);
        }
        if (rg == 0) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) red[w][t][sub * EPL + e] = o[t][e];
            if (sub == 0) { red[w][t][D] = m[t]; red[w][t][D + 1] = l[t]; }
        }
    }
    __syncthreads();
    for (int wi = tid; wi < GT * D; wi += 256) {
        const int t = wi / D, dd = wi - t * D;
        if (gbase + t >= G) continue;
        float M = -INFINITY;
#pragma unroll
        for (int ww = 0; ww < 4; ++ww) M = fmaxf(M, red[ww][t][D]);
        float acc = 0.f, lsum = 0.f;
        if (M > -INFINITY) {
#pragma unroll
            for (int ww = 0; ww < 4; ++ww) {
                const float a = fast_exp2(red[ww][t][D] - M);
                acc += red[ww][t][dd] * a;
                lsum += red[ww][t][D + 1] * a;
            }
        }
        float* dst = part + (((int64_t)u * G + gbase + t) * nsplit + split) * (D + 2);
        dst[dd] = acc;
        if (dd == 0) { dst[D] = M; dst[D + 1] = lsum; }
    }
}

// rows [r_begin, r_end) of a segment of L rows that split `split` of nsplit handles (multiples of 16 rows)
__device__ __forceinline__ void split_range(int L, int split, int nsplit, int& r_begin, int& r_end) {
    int per = (L + nsplit - 1) / nsplit;
    per = (per + 15) & ~15;
    r_begin = split * per;
    r_end = min(L, r_begin + per);
}

template <typename T, int D, int GT>
__global__ __launch_bounds__(256) void decode_partial_kernel(
    const T* __restrict__ q, const T* __restrict__ Kc, const T* __restrict__ Vc,
    const int32_t* __restrict__ len, int cap, int Hq, int Hkv, int gbase, float c,
    float* __restrict__ part, int nsplit)
{
    constexpr int EPL = D / 16;
    __shared__ float red[4][GT][D + 2];
    const int G = Hq / Hkv;
    const int split = blockIdx.x, u = blockIdx.y, b = u / Hkv, g = u - b * Hkv;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, sub = lane & 15, rg = lane >> 4;
    int L = len[u];
    L = max(0, min(L, cap));
    int r_begin, r_end;
    split_range(L, split, nsplit, r_begin, r_end);

    float qv[GT][EPL];
    load_queries<T, D, GT>(q, b, g, G, Hq, gbase, sub, c, qv);
    float m[GT], l[GT], o[GT][EPL];
#pragma unroll
    for (int t = 0; t < GT; ++t) {
        m[t] = -INFINITY; l[t] = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) o[t][e] = 0.f;
    }
    const T* Kb = Kc + (int64_t)u * cap * D + sub * EPL;
    const T* Vb = Vc + (int64_t)u * cap * D + sub * EPL;
#pragma unroll 2
    for (int r = r_begin + w * 4 + rg; r - rg - w * 4 < r_end; r += 16) {
        const bool valid = r < r_end;
        const int rr = valid ? r : r_begin;                 // r_begin < r_end inside the loop
        float kf[EPL], vf[EPL];
        RowChunk<T, EPL>::load(Kb + (int64_t)rr * D, kf);
        RowChunk<T, EPL>::load(Vb + (int64_t)rr * D, vf);
        attend_row<EPL, GT>(valid, kf, vf, qv, m, l, o);
    }
    write_partial<D, GT>(m, l, o, red, u, G, gbase, split, nsplit, part);
}

// ---------------------------------------------------------------- mixed-precision cache
// Codes of EPL consecutive elements at BITS bits each (element e in bits [e*BITS, e*BITS+BITS) of the
// little-endian word) -> floats zero + scale * code.

template <int EPL, int BITS>
__device__ __forceinline__ void load_quantized(const uint8_t* codes, const uint32_t* params, int64_t row, int D, int sub,
                                               float (&f)[EPL]) {
    using W = typename CodeWord<EPL, BITS>::type;
    const uint32_t word = *reinterpret_cast<const W*>(codes + row * (D * BITS / 8) + sub * sizeof(W));
    const uint32_t par = params[row];                       // fp16 scale (low half), fp16 zero (high half)
    const float scale = (float)__builtin_bit_cast(_Float16, (uint16_t)(par & 0xFFFFu));
    const float zero = (float)__builtin_bit_cast(_Float16, (uint16_t)(par >> 16));
#pragma unroll
    for (int e = 0; e < EPL; ++e) f[e] = fmaf(scale, (float)((word >> (e * BITS)) & ((1u << BITS) - 1u)), zero);
}

struct QTensor {                 // device pointers of one mixed-precision tensor, by value in the kernel arguments
    const uint8_t* hi_codes; const uint32_t* hi_params;
    const uint8_t* lo_codes; const uint32_t* lo_params;
};

// Eq. (5) over [4-bit rows of T | 2-bit rows of the other tokens | rows appended during decoding].
template <typename T, int D, int GT>
__global__ __launch_bounds__(256) void decode_q_partial_kernel(
    const T* __restrict__ q, QTensor Kq, QTensor Vq, const int32_t* __restrict__ len_hi, const int32_t* __restrict__ len_lo,
    int cap_hi, int cap_lo, const T* __restrict__ Kt, const T* __restrict__ Vt, const int32_t* __restrict__ len_t, int cap_t,
    int Hq, int Hkv, int gbase, float c, float* __restrict__ part, int nsplit)
{
    constexpr int EPL = D / 16;
    __shared__ float red[4][GT][D + 2];
    const int G = Hq / Hkv;
    const int split = blockIdx.x, u = blockIdx.y, b = u / Hkv, g = u - b * Hkv;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, sub = lane & 15, rg = lane >> 4;
    float qv[GT][EPL];
    load_queries<T, D, GT>(q, b, g, G, Hq, gbase, sub, c, qv);
    float m[GT], l[GT], o[GT][EPL];
#pragma unroll
    for (int t = 0; t < GT; ++t) {
        m[t] = -INFINITY; l[t] = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) o[t][e] = 0.f;
    }
    int r_begin, r_end;
    {   // important tokens, 4 bits
        const int L = max(0, min(len_hi[u], cap_hi));
        split_range(L, split, nsplit, r_begin, r_end);
        const int64_t base = (int64_t)u * cap_hi;
#pragma unroll 2
        for (int r = r_begin + w * 4 + rg; r - rg - w * 4 < r_end; r += 16) {
            const bool valid = r < r_end;
            const int64_t row = base + (valid ? r : r_begin);
            float kf[EPL], vf[EPL];
            load_quantized<EPL, 4>(Kq.hi_codes, Kq.hi_params, row, D, sub, kf);
            load_quantized<EPL, 4>(Vq.hi_codes, Vq.hi_params, row, D, sub, vf);
            attend_row<EPL, GT>(valid, kf, vf, qv, m, l, o);
        }
    }
    {   // the other tokens, 2 bits
        const int L = max(0, min(len_lo[u], cap_lo));
        split_range(L, split, nsplit, r_begin, r_end);
        const int64_t base = (int64_t)u * cap_lo;
#pragma unroll 2
        for (int r = r_begin + w * 4 + rg; r - rg - w * 4 < r_end; r += 16) {
            const bool valid = r < r_end;
            const int64_t row = base + (valid ? r : r_begin);
            float kf[EPL], vf[EPL];
            load_quantized<EPL, 2>(Kq.lo_codes, Kq.lo_params, row, D, sub, kf);
            load_quantized<EPL, 2>(Vq.lo_codes, Vq.lo_params, row, D, sub, vf);
            attend_row<EPL, GT>(valid, kf, vf, qv, m, l, o);
        }
    }
    if (Kt) {   // rows appended during decoding, as stored
        const int L = max(0, min(len_t[u], cap_t));
        split_range(L, split, nsplit, r_begin, r_end);
        const T* Kb = Kt + (int64_t)u * cap_t * D + sub * EPL;
        const T* Vb = Vt + (int64_t)u * cap_t * D + sub * EPL;
        for (int r = r_begin + w * 4 + rg; r - rg - w * 4 < r_end; r += 16) {
            const bool valid = r < r_end;
            const int rr = valid ? r : r_begin;
            float kf[EPL], vf[EPL];
            RowChunk<T, EPL>::load(Kb + (int64_t)rr * D, kf);
            RowChunk<T, EPL>::load(Vb + (int64_t)rr * D, vf);
            attend_row<EPL, GT>(valid, kf, vf, qv, m, l, o);
        }
    }
    write_partial<D, GT>(m, l, o, red, u, G, gbase, split, nsplit, part);
}

template <typename T> __device__ __forceinline__ T to_out(float x);
template <> __device__ __forceinline__ float to_out<float>(float x) { return x; }
template <> __device__ __forceinline__ __bf16 to_out<__bf16>(float x) { return (__bf16)x; }

template <typename T, int D>
__global__ void decode_combine_kernel(const float* __restrict__ part, int nsplit, T* __restrict__ o)
{
    const int bh = blockIdx.x, dd = threadIdx.x;            // units*G + head_in_group == b*Hq + head
    const float* p = part + (int64_t)bh * nsplit * (D + 2);
    float M = -INFINITY;
    for (int s = 0; s < nsplit; ++s) M = fmaxf(M, p[s * (D + 2) + D]);
    float acc = 0.f, lsum = 0.f;
    if (M > -INFINITY)
        for (int s = 0; s < nsplit; ++s) {
            const float a = fast_exp2(p[s * (D + 2) + D] - M);
            acc += p[s * (D + 2) + dd] * a;
            lsum += p[s * (D + 2) + D + 1] * a;
        }
    o[(int64_t)bh * D + dd] = to_out<T>(lsum > 0.f ? acc / lsum : 0.f);
}

static int decode_splits(const zipvl_dims& d, int cap) {
    const int units = d.B * d.Hkv;
    int s = (1024 + units - 1) / units;
    const int by_len = (cap + 255) / 256;                   // at least 256 rows per split
    s = s < by_len ? s : by_len;
    return s < 1 ? 1 : (s > kDecMaxSplit ? kDecMaxSplit : s);
}

size_t decode_workspace_bytes(const zipvl_dims& d, int cap) {
    return (size_t)d.B * d.Hq * decode_splits(d, cap) * (d.d + 2) * sizeof(float);
}

template <typename T, int D>
static int launch_decode_t(const void* q, const void* Kc, const void* Vc, const int32_t* len, int32_t cap,
                           const zipvl_dims& d, float scale, void* o, void* ws, hipStream_t st)
{
    const int G = d.Hq / d.Hkv, units = d.B * d.Hkv, nsplit = decode_splits(d, cap);
    const float c = scale * kLog2e;
    dim3 grid(nsplit, units);
#define ZIPVL_DEC(GT, GB)                                                                            \
    hipLaunchKernelGGL((decode_partial_kernel<T, D, GT>), grid, dim3(256), 0, st, (const T*)q,       \
        (const T*)Kc, (const T*)Vc, len, cap, d.Hq, d.Hkv, GB, c, (float*)ws, nsplit)
    for (int gb = 0; gb < G; gb += 8) {
        const int rem = G - gb;
        KernelTimer tm(ZIPVL_K_DECODE_PARTIAL, st);
        if (rem >= 5) ZIPVL_DEC(8, gb);
        else if (rem >= 3) ZIPVL_DEC(4, gb);
        else if (rem == 2) ZIPVL_DEC(2, gb);
        else ZIPVL_DEC(1, gb);
        int rc = check_launch("decode_partial");
        if (rc) return rc;
    }
#undef ZIPVL_DEC
    KernelTimer tm(ZIPVL_K_DECODE_COMBINE, st);
    hipLaunchKernelGGL((decode_combine_kernel<T, D>), dim3(d.B * d.Hq), dim3(D), 0, st,
        (const float*)ws, nsplit, (T*)o);
    return check_launch("decode_combine");
}

template <typename T, int D>
static int launch_decode_q_t(const void* q, const zipvl_qtensor& Kq, const zipvl_qtensor& Vq, const int32_t* len_hi,
                             const int32_t* len_lo, int32_t cap_hi, int32_t cap_lo, const void* Kt, const void* Vt,
                             const int32_t* len_t, int32_t cap_t, const zipvl_dims& d, float scale, void* o, void* ws, hipStream_t st)
{
    const int G = d.Hq / d.Hkv, units = d.B * d.Hkv, nsplit = decode_splits(d, cap_hi + cap_lo + cap_t);
    const float c = scale * kLog2e;
    dim3 grid(nsplit, units);
    const QTensor kq{(const uint8_t*)Kq.hi_codes, (const uint32_t*)Kq.hi_params, (const uint8_t*)Kq.lo_codes, (const uint32_t*)Kq.lo_params};
    const QTensor vq{(const uint8_t*)Vq.hi_codes, (const uint32_t*)Vq.hi_params, (const uint8_t*)Vq.lo_codes, (const uint32_t*)Vq.lo_params};
#define ZIPVL_DECQ(GT, GB)                                                                           \
    hipLaunchKernelGGL((decode_q_partial_kernel<T, D, GT>), grid, dim3(256), 0, st, (const T*)q, kq, vq, \
        len_hi, len_lo, cap_hi, cap_lo, (const T*)Kt, (const T*)Vt, len_t, cap_t, d.Hq, d.Hkv, GB, c, (float*)ws, nsplit)
    for (int gb = 0; gb < G; gb += 8) {
        const int rem = G - gb;
        KernelTimer tm(ZIPVL_K_DECODE_Q_PARTIAL, st);
        if (rem >= 5) ZIPVL_DECQ(8, gb);
        else if (rem >= 3) ZIPVL_DECQ(4, gb);
        else if (rem == 2) ZIPVL_DECQ(2, gb);
        else ZIPVL_DECQ(1, gb);
        int rc = check_launch("decode_q_partial");
        if (rc) return rc;
    }
#undef ZIPVL_DECQ
    KernelTimer tm(ZIPVL_K_DECODE_COMBINE, st);
    hipLaunchKernelGGL((decode_combine_kernel<T, D>), dim3(d.B * d.Hq), dim3(D), 0, st,
        (const float*)ws, nsplit, (T*)o);
    return check_launch("decode_combine");
}

int launch_decode_attn_q(const void* q, const zipvl_qtensor& Kq, const zipvl_qtensor& Vq, const int32_t* len_hi,
                         const int32_t* len_lo, int32_t cap_hi, int32_t cap_lo, const void* Kt, const void* Vt,
                         const int32_t* len_t, int32_t cap_t, const zipvl_dims& d, float scale, void* o, void* ws, hipStream_t st)
{
#define ZIPVL_ARGS q, Kq, Vq, len_hi, len_lo, cap_hi, cap_lo, Kt, Vt, len_t, cap_t, d, scale, o, ws, st
    if (d.dtype == ZIPVL_BF16) {
        if (d.d == 128) return launch_decode_q_t<__bf16, 128>(ZIPVL_ARGS);
        return launch_decode_q_t<__bf16, 64>(ZIPVL_ARGS);
    }
    if (d.d == 128) return launch_decode_q_t<float, 128>(ZIPVL_ARGS);
    return launch_decode_q_t<float, 64>(ZIPVL_ARGS);
#undef ZIPVL_ARGS
}

int launch_decode_attn(const void* q, const void* Kc, const void* Vc, const int32_t* len, int32_t cap,
                       const zipvl_dims& d, float scale, void* o, void* ws, hipStream_t st)
{
    if (d.dtype == ZIPVL_BF16) {
        if (d.d == 128) return launch_decode_t<__bf16, 128>(q, Kc, Vc, len, cap, d, scale, o, ws, st);
        return launch_decode_t<__bf16, 64>(q, Kc, Vc, len, cap, d, scale, o, ws, st);
    }
    if (d.d == 128) return launch_decode_t<float, 128>(q, Kc, Vc, len, cap, d, scale, o, ws, st);
    return launch_decode_t<float, 64>(q, Kc, Vc, len, cap, d, scale, o, ws, st);
}

}  // namespace zipvl
