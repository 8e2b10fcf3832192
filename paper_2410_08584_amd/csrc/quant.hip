// Mixed-precision KV cache keyed by the important set (Section 5.3.1: important
// tokens at 4 bits, the others at 2 bits).  The quantiser the paper leaves open
// is taken as uniform asymmetric per row (one token of one KV head) with an
// fp16 (scale, zero) pair:
//   zero = fp16(min), scale = fp16((max - min) * fp32(1 / (2^bits - 1))),
//   code = clamp(rint((x - zero) / scale), 0, 2^bits - 1)   (0 when scale = 0), all in fp32.
// Two kernels: `token_slots` turns T (ascending positions) into, for every token,
// its row in the 4-bit group (rank among the kept tokens) or in the 2-bit group
// (rank among the others, Eq. (10)), with an LDS bitmap and a prefix count;
// `quantize_rows` then handles 16 rows per wave pass, 16 lanes per row like the
// decode kernels, so every code row is written as one contiguous store per lane.
#include <atomic>

#include "launch.h"
#include "rowops.h"

namespace zipvl {

constexpr int kQuantMaxTokens = 262144;      // bitmap + prefix counts of one unit fit in 64 KB of LDS
constexpr int kSlotThreads = 1024;
constexpr int kQuantRows = 64;               // rows per workgroup of quantize_rows

// slot[ut, j] = i >= 0: token j is T_i (4-bit row i);  slot = ~i < 0: token j is the i-th other token (2-bit row i)
__global__ __launch_bounds__(kSlotThreads) void token_slots_kernel(
    const int32_t* __restrict__ idx, const int32_t* __restrict__ kcnt, int n, int32_t* __restrict__ slot)
{
    extern __shared__ uint32_t lds[];
    const int nwords = (n + 31) >> 5;
    uint32_t* bm = lds;                      // [nwords] bit j set <=> token j is in T
    uint32_t* pre = lds + nwords;            // [nwords] number of kept tokens before word w
    __shared__ uint32_t wave_tot[kSlotThreads / 64];
    const int ut = blockIdx.x, tid = threadIdx.x;
    int kk = kcnt ? kcnt[ut] : n;
    kk = max(0, min(kk, n));
    for (int w = tid; w < nwords; w += kSlotThreads) bm[w] = 0u;
    __syncthreads();
    for (int i = tid; i < kk; i += kSlotThreads) {
        const int t = idx ? idx[(int64_t)ut * n + i] : i;
        if (t >= 0 && t < n) atomicOr(&bm[t >> 5], 1u << (t & 31));
    }
    __syncthreads();
    // exclusive prefix of the word popcounts: every thread owns a contiguous run of words
    const int per = (nwords + kSlotThreads - 1) / kSlotThreads;
    const int w0 = min(tid * per, nwords), w1 = min(w0 + per, nwords);
    uint32_t mine = 0;
    for (int w = w0; w < w1; ++w) mine += __popc(bm[w]);
    uint32_t incl = mine;                    // inclusive scan inside the wave
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t v = __shfl_up(incl, off);
        if ((tid & 63) >= off) incl += v;
    }
    if ((tid & 63) == 63) wave_tot[tid >> 6] = incl;
    __syncthreads();
    uint32_t before = incl - mine;
    for (int ww = 0; ww < (tid >> 6); ++ww) before += wave_tot[ww];
    for (int w = w0; w < w1; ++w) { pre[w] = before; before += __popc(bm[w]); }
    __syncthreads();
    for (int j = tid; j < n; j += kSlotThreads) {
        const uint32_t word = bm[j >> 5], bit = j & 31;
        const int kept_before = (int)(pre[j >> 5] + __popc(word & ((1u << bit) - 1u)));
        slot[(int64_t)ut * n + j] = ((word >> bit) & 1u) ? kept_before : ~(j - kept_before);
    }
}

template <int EPL, int BITS>
__device__ __forceinline__ void quantize_chunk(const float (&x)[EPL], uint8_t* codes, uint32_t* params, int64_t row, int D, int sub) {
    float lo = x[0], hi = x[0];
#pragma unroll
    for (int e = 1; e < EPL; ++e) { lo = fminf(lo, x[e]); hi = fmaxf(hi, x[e]); }
#pragma unroll
    for (int off = 1; off < 16; off <<= 1) {
        lo = fminf(lo, __shfl_xor(lo, off));
        hi = fmaxf(hi, __shfl_xor(hi, off));
    }
    constexpr float qmax = (float)((1 << BITS) - 1);
    const _Float16 zero_h = (_Float16)lo;
    float step = (hi - lo) * (float)(1.0 / (double)qmax);
    asm volatile("" : "+v"(step));            // the product is rounded to fp32 first: no fused multiply-convert
    const _Float16 scale_h = (_Float16)step;
    const float zero = (float)zero_h, scale = (float)scale_h;
    uint32_t word = 0;
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
        float t = scale > 0.f ? (x[e] - zero) / scale : 0.f;
        t = fminf(fmaxf(__builtin_rintf(t), 0.f), qmax);
        word |= (uint32_t)t << (e * BITS);
    }
    using W = typename CodeWord<EPL, BITS>::type;
    *reinterpret_cast<W*>(codes + row * (D * BITS / 8) + sub * sizeof(W)) = (W)word;
    if (sub == 0)
        params[row] = (uint32_t)__builtin_bit_cast(uint16_t, scale_h) | ((uint32_t)__builtin_bit_cast(uint16_t, zero_h) << 16);
}

struct QTensorOut {
    uint8_t* hi_codes; uint32_t* hi_params;
    uint8_t* lo_codes; uint32_t* lo_params;
};

template <typename T, int D>
__global__ __launch_bounds__(256) void quantize_rows_kernel(
    const T* __restrict__ K, const T* __restrict__ V,
    int64_t ks0, int64_t ks1, int64_t ks2, int64_t vs0, int64_t vs1, int64_t vs2,
    const int32_t* __restrict__ slot, const int32_t* __restrict__ kcnt,
    QTensorOut Kq, QTensorOut Vq, int cap_hi, int cap_lo, int32_t* __restrict__ len_hi, int32_t* __restrict__ len_lo,
    int n, int Hkv, int t_per_batch)
{
    constexpr int EPL = D / 16;
    const int u = blockIdx.y, b = u / Hkv, g = u - b * Hkv;
    const int ut = t_per_batch ? b : u;
    const int tid = threadIdx.x, sub = tid & 15, rl = tid >> 4;         // 16 rows per pass
    if (blockIdx.x == 0 && tid == 0) {
        int kk = kcnt ? kcnt[ut] : n;
        kk = max(0, min(kk, n));
        len_hi[u] = min(kk, cap_hi);
        len_lo[u] = min(n - kk, cap_lo);
    }
    const T* Kb = K + b * ks0 + g * ks1 + sub * EPL;
    const T* Vb = V + b * vs0 + g * vs1 + sub * EPL;
    const int j0 = blockIdx.x * kQuantRows;
#pragma unroll 1
    for (int p = 0; p < kQuantRows / 16; ++p) {
        const int j = j0 + p * 16 + rl;                                 // uniform over the 16 lanes of a row
        if (j >= n) continue;
        const int s = slot[(int64_t)ut * n + j];
        float kf[EPL], vf[EPL];
        RowChunk<T, EPL>::load(Kb + (int64_t)j * ks2, kf);
        RowChunk<T, EPL>::load(Vb + (int64_t)j * vs2, vf);
        if (s >= 0) {
            if (s < cap_hi) {
                const int64_t row = (int64_t)u * cap_hi + s;
                quantize_chunk<EPL, 4>(kf, Kq.hi_codes, Kq.hi_params, row, D, sub);
                quantize_chunk<EPL, 4>(vf, Vq.hi_codes, Vq.hi_params, row, D, sub);
            }
        } else if (~s < cap_lo) {
            const int64_t row = (int64_t)u * cap_lo + ~s;
            quantize_chunk<EPL, 2>(kf, Kq.lo_codes, Kq.lo_params, row, D, sub);
            quantize_chunk<EPL, 2>(vf, Vq.lo_codes, Vq.lo_params, row, D, sub);
        }
    }
}

size_t quantize_workspace_bytes(const zipvl_dims& d) { return (size_t)d.B * d.Hkv * d.n * sizeof(int32_t); }

template <typename T, int D>
static int launch_quantize_t(const void* K, const void* V, const zipvl_dims& d, const int32_t* idx, const int32_t* k,
                             const zipvl_qtensor& Kq, const zipvl_qtensor& Vq, int32_t cap_hi, int32_t cap_lo,
                             int32_t* len_hi, int32_t* len_lo, int flags, void* ws, hipStream_t st)
{
    const int units = d.B * d.Hkv;
    const int t_per_batch = (flags & ZIPVL_T_PER_BATCH) ? 1 : 0;
    int32_t* slot = (int32_t*)ws;
    const size_t lds = 2 * (size_t)((d.n + 31) / 32) * sizeof(uint32_t);
    static std::atomic<bool> attr_done{false};
    if (!attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(&token_slots_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024) != hipSuccess)
            return set_error(ZIPVL_EHIP, "quantize_kv: cannot reserve LDS for the token bitmap");
        attr_done = true;
    }
    {
        KernelTimer tm(ZIPVL_K_TOKEN_SLOTS, st);
        hipLaunchKernelGGL(token_slots_kernel, dim3(t_per_batch ? d.B : units), dim3(kSlotThreads), lds, st, idx, k, d.n, slot);
    }
    int rc = check_launch("token_slots");
    if (rc) return rc;
    const QTensorOut kq{(uint8_t*)Kq.hi_codes, (uint32_t*)Kq.hi_params, (uint8_t*)Kq.lo_codes, (uint32_t*)Kq.lo_params};
    const QTensorOut vq{(uint8_t*)Vq.hi_codes, (uint32_t*)Vq.hi_params, (uint8_t*)Vq.lo_codes, (uint32_t*)Vq.lo_params};
    KernelTimer tm(ZIPVL_K_QUANTIZE_ROWS, st);
    hipLaunchKernelGGL((quantize_rows_kernel<T, D>), dim3((d.n + kQuantRows - 1) / kQuantRows, units), dim3(256), 0, st,
        (const T*)K, (const T*)V, d.k_strides[0], d.k_strides[1], d.k_strides[2],
        d.v_strides[0], d.v_strides[1], d.v_strides[2], (const int32_t*)slot, k, kq, vq, cap_hi, cap_lo, len_hi, len_lo,
        d.n, d.Hkv, t_per_batch);
    return check_launch("quantize_rows");
}

int launch_quantize_kv(const void* K, const void* V, const zipvl_dims& d, const int32_t* idx, const int32_t* k,
                       const zipvl_qtensor& Kq, const zipvl_qtensor& Vq, int32_t cap_hi, int32_t cap_lo,
                       int32_t* len_hi, int32_t* len_lo, int flags, void* ws, hipStream_t st)
{
    if (d.n > kQuantMaxTokens) return set_error(ZIPVL_ESHAPE, "quantize_kv: n = %d exceeds %d", d.n, kQuantMaxTokens);
#define ZIPVL_ARGS K, V, d, idx, k, Kq, Vq, cap_hi, cap_lo, len_hi, len_lo, flags, ws, st
    if (d.dtype == ZIPVL_BF16) {
        if (d.d == 128) return launch_quantize_t<__bf16, 128>(ZIPVL_ARGS);
        return launch_quantize_t<__bf16, 64>(ZIPVL_ARGS);
    }
    if (d.d == 128) return launch_quantize_t<float, 128>(ZIPVL_ARGS);
    return launch_quantize_t<float, 64>(ZIPVL_ARGS);
#undef ZIPVL_ARGS
}

}  // namespace zipvl
