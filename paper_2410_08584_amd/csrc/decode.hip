// Decode-phase attention against the (evicted) KV cache (Eq. (5); Algorithm 2).
// Memory-bound: one query per head, every cached row read exactly once.
// Split-KV: grid = (splits, units).  A split is a fixed number of cached rows
// (chosen on the host from the capacity), and how many splits of a unit have
// work follows from the length that lives on the device: a short (evicted)
// cache occupies few workgroups, all of the same size, and the dispatcher
// balances them.  Inside a workgroup 16 lanes cover one cached row (16 bytes
// each at d = 128 bf16), so a wave reads 4 rows per step as full 256-byte
// lines (the rows of the next step are requested before the current ones are
// consumed), reduces the dot product over the 16 lanes with shuffles and keeps
// an online-softmax state per row group; row groups, waves and finally splits
// are merged with the usual (max, sum, weighted output) rule.  All query
// heads of a KV group are served from the same read.
#include <algorithm>
#include <mutex>

#include "launch.h"
#include "rowops.h"

namespace zipvl {

constexpr int kDecMaxSplit = 64;

template <typename T> __device__ __forceinline__ T to_out(float x);
template <> __device__ __forceinline__ float to_out<float>(float x) { return x; }
template <> __device__ __forceinline__ __bf16 to_out<__bf16>(float x) { return (__bf16)x; }

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

// The 4 waves' states in red[wave][head][o[D], m, l] -> the workgroup's partial state.
// partial layout: [(unit*G + head_in_group) * nsplit + split][D + 2]  (o[D], m, l), log2 domain
// COHERENT: the partial state is read by another workgroup of the same launch (possibly on another XCD,
// whose L2 is not coherent with this one's): written through with device-scope stores.
template <int D, int GT, bool COHERENT = false>
__device__ __forceinline__ void combine_waves(float (&red)[4][GT][D + 2], int u, int G, int gbase, int split, int nsplit, float* part) {
    auto put = [](float* p, float v) {
        if constexpr (COHERENT) __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else *p = v;
    };
    for (int wi = threadIdx.x; wi < GT * D; wi += 256) {
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
        put(dst + dd, acc);
        if (dd == 0) { put(dst + D, M); put(dst + D + 1, lsum); }
    }
}

// Merge the 4 row groups of every wave, then the 4 waves, and write the workgroup's partial state.
template <int D, int GT, bool COHERENT = false>
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
    combine_waves<D, GT, COHERENT>(red, u, G, gbase, split, nsplit, part);
}

// rows [r_begin, r_end) of a segment of L rows that split `split` of nsplit handles (multiples of 16 rows)
__device__ __forceinline__ void split_range(int L, int split, int nsplit, int& r_begin, int& r_end) {
    int per = (L + nsplit - 1) / nsplit;
    per = (per + 15) & ~15;
    r_begin = split * per;
    r_end = min(L, r_begin + per);
}

// the same in multiples of 64 rows (16 rows per wave step)
__device__ __forceinline__ void split_range64(int L, int split, int nsplit, int& r_begin, int& r_end) {
    int per = (L + nsplit - 1) / nsplit;
    per = (per + 63) & ~63;
    r_begin = split * per;
    r_end = min(L, r_begin + per);
}

// Rows per split for a cache of `cap` rows: 256 for short caches, more for long ones so that a unit never
// has more than kDecRowSplits splits (the merge reads one partial state per split).  A multiple of 16.
constexpr int kDecRowSplits = 16;
static inline int rows_per_split(int cap) {
    const int per = ((cap + kDecRowSplits - 1) / kDecRowSplits + 15) & ~15;
    return per < 256 ? 256 : per;        // 128 ... 512 rows measured within 5 % of each other on 2000-row caches
}

template <typename T, int EPL> struct alignas(sizeof(T) * EPL > 16 ? 16 : sizeof(T) * EPL) RawChunk { T v[EPL]; };

template <typename T, int EPL>
__device__ __forceinline__ void raw_to_floats(const RawChunk<T, EPL>& r, float (&f)[EPL]) {
    RowChunk<T, EPL>::load(r.v, f);
}

// Rows [r_begin, r_end) of one unit against the GT queries in qv.  Row r comes from the cache, except row
// `new_row` (>= 0 only in the fused step), which comes from k_new / v_new and is also written to the cache.
// The 16 row groups of the workgroup take rows r_begin + g, r_begin + g + 16, ...; the loads of a group's next
// row are in flight while the current one is consumed.
template <typename T, int D, int GT>
__device__ __forceinline__ void attend_rows(const T* Kb, const T* Vb, T* Kw, T* Vw, const T* kn, const T* vn, int new_row,
                                            int r_begin, int r_end, int group, const float (&qv)[GT][D / 16],
                                            float (&m)[GT], float (&l)[GT], float (&o)[GT][D / 16]) {
    constexpr int EPL = D / 16;
    using Raw = RawChunk<T, EPL>;
    auto fetch = [&](int r, Raw& kr, Raw& vr) {
        const int rr = r < r_end ? r : r_begin;             // clamped rows are loaded and ignored
        const bool fresh = rr == new_row;
        kr = *reinterpret_cast<const Raw*>(fresh ? kn : Kb + (int64_t)rr * D);
        vr = *reinterpret_cast<const Raw*>(fresh ? vn : Vb + (int64_t)rr * D);
    };
    if (r_begin >= r_end) return;
    Raw kc, vc;
    int r = r_begin + group;
    fetch(r, kc, vc);
    for (int base = r_begin; base < r_end; base += 16, r += 16) {   // workgroup-uniform trip count
        Raw kx = kc, vx = vc;
        if (base + 16 < r_end) fetch(r + 16, kx, vx);
        const bool valid = r < r_end;
        if (valid && r == new_row) {
            *reinterpret_cast<Raw*>(Kw + (int64_t)r * D) = kc;
            *reinterpret_cast<Raw*>(Vw + (int64_t)r * D) = vc;
        }
        float kf[EPL], vf[EPL];
        raw_to_floats<T, EPL>(kc, kf);
        raw_to_floats<T, EPL>(vc, vf);
        attend_row<EPL, GT>(valid, kf, vf, qv, m, l, o);
        kc = kx; vc = vx;
    }
}

template <typename T, int D, int GT>
__global__ __launch_bounds__(256) void decode_partial_kernel(
    const T* __restrict__ q, const T* __restrict__ Kc, const T* __restrict__ Vc,
    const int32_t* __restrict__ len, int cap, int Hq, int Hkv, int gbase, float c,
    float* __restrict__ part, int rows, int max_splits)
{
    constexpr int EPL = D / 16;
    __shared__ float red[4][GT][D + 2];
    const int G = Hq / Hkv;
    const int split = blockIdx.x, u = blockIdx.y, b = u / Hkv, g = u - b * Hkv;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, sub = lane & 15, rg = lane >> 4;
    const int L = max(0, min(len[u], cap));
    const int r_begin = split * rows, r_end = min(L, r_begin + rows);
    if (split > 0 && r_begin >= L) return;                  // split 0 always reports (an empty state when L = 0)

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
    attend_rows<T, D, GT>(Kb, Vb, nullptr, nullptr, nullptr, nullptr, -1, r_begin, r_end, w * 4 + rg, qv, m, l, o);
    write_partial<D, GT>(m, l, o, red, u, G, gbase, split, max_splits, part);
}

// The partial states of one unit's splits -> its output rows.  One wave per head first turns the splits'
// (max, sum) pairs into weights a_s / sum_s(a_s l_s), a_s = exp2(m_s - max), one split per lane; then every
// thread accumulates one output element over the splits, eight independent loads at a time.
// nsplit <= 64.  COHERENT: the states were written by other workgroups of the same launch.
template <typename T, int D, bool COHERENT>
__device__ __forceinline__ void merge_splits(const float* __restrict__ part, int u, int G, int nsplit, int max_splits,
                                             float (&wgt)[8][64], T* __restrict__ out) {
    auto get = [](const float* p) {
        if constexpr (COHERENT) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else return *p;
    };
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    for (int t0 = 0; t0 < G; t0 += 8) {                      // groups larger than 8 heads: 8 at a time
        const int gt = min(8, G - t0);
        __syncthreads();
        for (int t = w; t < gt; t += 4) {
            const float* p = part + ((int64_t)u * G + t0 + t) * max_splits * (D + 2);
            const float ms = lane < nsplit ? get(p + lane * (D + 2) + D) : -INFINITY;
            const float ls = lane < nsplit ? get(p + lane * (D + 2) + D + 1) : 0.f;
            float M = ms;
#pragma unroll
            for (int off = 32; off; off >>= 1) M = fmaxf(M, __shfl_xor(M, off));
            const float a = M > -INFINITY ? fast_exp2(ms - M) : 0.f;
            float tot = a * ls;
#pragma unroll
            for (int off = 32; off; off >>= 1) tot += __shfl_xor(tot, off);
            wgt[t][lane] = tot > 0.f ? a / tot : 0.f;
        }
        __syncthreads();
        for (int wi = tid; wi < gt * D; wi += 256) {
            const int t = wi / D, dd = wi - t * D;
            const float* p = part + ((int64_t)u * G + t0 + t) * max_splits * (D + 2) + dd;
            float acc = 0.f;
            for (int s0 = 0; s0 < nsplit; s0 += 8) {
                float v[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) v[j] = get(p + (int64_t)min(s0 + j, nsplit - 1) * (D + 2));
#pragma unroll
                for (int j = 0; j < 8; ++j) acc = fmaf(s0 + j < nsplit ? wgt[t][s0 + j] : 0.f, v[j], acc);
            }
            out[((int64_t)u * G + t0 + t) * D + dd] = to_out<T>(acc);
        }
    }
}

// Splits of unit u that hold rows: from the device-resident length when `len` is given, else `fixed`.
__device__ __forceinline__ int unit_splits(const int32_t* len, int u, int cap, int rows, int fixed) {
    if (!len) return fixed;
    const int L = max(0, min(len[u], cap));
    return max(1, (L + rows - 1) / rows);
}

template <typename T, int D>
__global__ __launch_bounds__(256) void decode_combine_kernel(const float* __restrict__ part, const int32_t* __restrict__ len,
                                                             int cap, int rows, int nsplit_fixed, int max_splits, int G,
                                                             T* __restrict__ o)
{
    __shared__ float wgt[8][64];
    const int u = blockIdx.x;
    merge_splits<T, D, false>(part, u, G, unit_splits(len, u, cap, rows, nsplit_fixed), max_splits, wgt, o);
}

// ---------------------------------------------------------------- one launch per decode step
// Append and attention of Algorithm 2 in one kernel.  The new row (k_new / v_new) becomes row len of the
// cache: the workgroup whose split contains that row takes it from k_new / v_new in its place in the row
// order (the arithmetic is that of the two separate calls) and stores it in the cache.  Every workgroup
// of a unit - those without rows too - reads len and then arrives at a per-unit counter; the one that
// arrives last merges the unit's partial states, writes the output, advances len and clears the counter.
// Since all workgroups have read len before the last one arrives, the update cannot be seen by a reader of
// the old value.
template <typename T, int D, int GT>
__global__ __launch_bounds__(256) void decode_step_kernel(
    const T* __restrict__ q, T* __restrict__ Kc, T* __restrict__ Vc, int32_t* __restrict__ len, int cap,
    const T* __restrict__ k_new, const T* __restrict__ v_new, int Hq, int Hkv, float c,
    float* __restrict__ part, int rows, int max_splits, unsigned* __restrict__ arrived, T* __restrict__ out)
{
    constexpr int EPL = D / 16;
    __shared__ float red[4][GT][D + 2];
    __shared__ float wgt[8][64];
    __shared__ int is_last;
    const int G = Hq / Hkv;
    const int split = blockIdx.x, u = blockIdx.y, b = u / Hkv, g = u - b * Hkv;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, sub = lane & 15, rg = lane >> 4;
    const int Lraw = len[u];
    const bool room = Lraw >= 0 && Lraw < cap;               // a full cache is left unchanged, as by the append call
    const int L0 = max(0, min(Lraw, cap));
    const int L = L0 + (room ? 1 : 0);                       // rows attended: the new one included
    const int r_begin = split * rows, r_end = min(L, r_begin + rows);
    const int nsplit = max(1, (L + rows - 1) / rows);

    if (split < nsplit) {
        float qv[GT][EPL];
        load_queries<T, D, GT>(q, b, g, G, Hq, 0, sub, c, qv);
        float m[GT], l[GT], o[GT][EPL];
#pragma unroll
        for (int t = 0; t < GT; ++t) {
            m[t] = -INFINITY; l[t] = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) o[t][e] = 0.f;
        }
        T* Kb = Kc + (int64_t)u * cap * D + sub * EPL;
        T* Vb = Vc + (int64_t)u * cap * D + sub * EPL;
        attend_rows<T, D, GT>(Kb, Vb, Kb, Vb, k_new + (int64_t)u * D + sub * EPL, v_new + (int64_t)u * D + sub * EPL,
                              room ? L0 : -1, r_begin, r_end, w * 4 + rg, qv, m, l, o);
        write_partial<D, GT, true>(m, l, o, red, u, G, 0, split, max_splits, part);
    }

    // The partial state went out with device-scope (write-through) stores: once they have completed
    // (vmcnt 0) it is visible to every XCD, and only then is this workgroup counted.  A release fence
    // would do the same by writing back the whole L2, 150 us per launch here.
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (tid == 0) is_last = atomicAdd(&arrived[u], 1u) == gridDim.x - 1u;
    __syncthreads();
    if (!is_last) return;
    merge_splits<T, D, true>(part, u, G, nsplit, max_splits, wgt, out);
    if (tid == 0) {
        if (room) len[u] = Lraw + 1;
        arrived[u] = 0u;                                     // ready for the next step
    }
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

// ---- the same, for small query groups (GT <= 2): 4 lanes per row.
// A 4-bit row of d = 128 is 64 bytes: with 16 lanes per row a lane would hold 4 bytes and the per-row work
// (cross-lane sums, softmax update) would dominate.  Here a lane holds d/4 consecutive elements (16 bytes of 4-bit
// codes, 8 bytes of 2-bit codes), a wave covers 16 rows per step, and the arithmetic runs on the codes:
//   q . (zero + scale * code) = zero * sum(q) + scale * (q . code),
//   sum_j p_j (zero_j + scale_j * code_j) = sum_j p_j zero_j + sum_j (p_j scale_j) code_j,
// i.e. one conversion and one FMA per element and side.  The softmax offset follows the running maximum lazily
// (moves only when exceeded by 2^kDecLazyLog2), so the accumulators are rescaled on few rows.
constexpr float kDecLazyLog2 = 8.f;

// sum over the 4 lanes of a quad (lanes 4i .. 4i+3), result in all four, by two in-register lane permutes
__device__ __forceinline__ float quad_sum(float v) {
    int x = __float_as_int(v);
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, x, 0xB1, 0xF, 0xF, true));    // quad_perm [1,0,3,2]
    x = __float_as_int(v);
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, x, 0x4E, 0xF, 0xF, true));    // quad_perm [2,3,0,1]
    return v;
}

// the NB-byte code string of one lane -> EPL = NB * 8 / BITS floats (codes as numbers), element e at bits [e*BITS, ..)
template <int BITS, int NW>
__device__ __forceinline__ void codes_to_floats(const uint32_t (&w)[NW], float (&f)[NW * 32 / BITS]) {
#pragma unroll
    for (int i = 0; i < NW; ++i) {
        if constexpr (BITS == 4) {
            const uint32_t ev = w[i] & 0x0F0F0F0Fu, od = (w[i] >> 4) & 0x0F0F0F0Fu;   // codes 0,2,4,6 / 1,3,5,7 as bytes
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                f[8 * i + 2 * b] = (float)((ev >> (8 * b)) & 0xFFu);
                f[8 * i + 2 * b + 1] = (float)((od >> (8 * b)) & 0xFFu);
            }
        } else {
#pragma unroll
            for (int sft = 0; sft < 4; ++sft) {
                const uint32_t t = (w[i] >> (2 * sft)) & 0x03030303u;                  // codes sft, sft+4, sft+8, sft+12 as bytes
#pragma unroll
                for (int b = 0; b < 4; ++b) f[16 * i + 4 * b + sft] = (float)((t >> (8 * b)) & 0xFFu);
            }
        }
    }
}

template <int NW> __device__ __forceinline__ void load_words(const uint8_t* p, uint32_t (&w)[NW]);
template <> __device__ __forceinline__ void load_words<4>(const uint8_t* p, uint32_t (&w)[4]) {
    const uintx4 v = load16(p); w[0] = v[0]; w[1] = v[1]; w[2] = v[2]; w[3] = v[3];
}
template <> __device__ __forceinline__ void load_words<2>(const uint8_t* p, uint32_t (&w)[2]) {
    const uintx2 v = *reinterpret_cast<const uintx2*>(p); w[0] = v[0]; w[1] = v[1];
}
template <> __device__ __forceinline__ void load_words<1>(const uint8_t* p, uint32_t (&w)[1]) {
    w[0] = *reinterpret_cast<const uint32_t*>(p);
}

template <typename T, int D, int GT>
__global__ __launch_bounds__(256) void decode_q4_partial_kernel(
    const T* __restrict__ q, QTensor Kq, QTensor Vq, const int32_t* __restrict__ len_hi, const int32_t* __restrict__ len_lo,
    int cap_hi, int cap_lo, const T* __restrict__ Kt, const T* __restrict__ Vt, const int32_t* __restrict__ len_t, int cap_t,
    int Hq, int Hkv, int gbase, float c, float* __restrict__ part, int nsplit)
{
    constexpr int EPL = D / 4;                               // elements per lane
    __shared__ float red[4][GT][D + 2];
    const int G = Hq / Hkv;
    const int split = blockIdx.x, u = blockIdx.y, b = u / Hkv, g = u - b * Hkv;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, sub = lane & 3, rg = lane >> 2;   // 16 rows per wave step
    float qv[GT][EPL], qsum[GT];
#pragma unroll
    for (int t = 0; t < GT; ++t) {
        const int hh = gbase + t;
        float part_sum = 0.f;
#pragma unroll
        for (int e8 = 0; e8 < EPL / 8; ++e8) {
            float f[8];
            if (hh < G) RowChunk<T, 8>::load(q + ((int64_t)(b * Hq + g * G + hh)) * D + sub * EPL + 8 * e8, f);
#pragma unroll
            for (int e = 0; e < 8; ++e) { qv[t][8 * e8 + e] = hh < G ? f[e] * c : 0.f; part_sum += qv[t][8 * e8 + e]; }
        }
        qsum[t] = quad_sum(part_sum);                        // sum over the whole row of the scaled query
    }
    float m[GT], l[GT], zacc[GT], o[GT][EPL];
#pragma unroll
    for (int t = 0; t < GT; ++t) {
        m[t] = -INFINITY; l[t] = 0.f; zacc[t] = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) o[t][e] = 0.f;
    }
    // one cached row: kd[t] = q_t . (this lane's K codes), score = kz * qsum + ks * sum over lanes of kd; then
    // o += (p * vs) * (V codes), zacc += p * vz
    auto attend = [&](bool valid, const float (&kc)[EPL], float ks, float kz, const float (&vc)[EPL], float vs, float vz) {
#pragma unroll
        for (int t = 0; t < GT; ++t) {
            float dsum = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) dsum = fmaf(qv[t][e], kc[e], dsum);
            dsum = quad_sum(dsum);
            const float sc = valid ? fmaf(ks, dsum, kz * qsum[t]) : -INFINITY;
            const bool grow = sc > m[t] + kDecLazyLog2;
            if (__any(grow)) {
                const float m_new = grow ? sc : m[t];
                const float a = grow ? fast_exp2(m[t] - m_new) : 1.f;   // 0 on a row group's first row (m = -inf)
                l[t] *= a; zacc[t] *= a;
#pragma unroll
                for (int e = 0; e < EPL; ++e) o[t][e] *= a;
                m[t] = m_new;
            }
            const float p = valid ? fast_exp2(sc - m[t]) : 0.f;
            l[t] += p;
            zacc[t] = fmaf(p, vz, zacc[t]);
            const float pv = p * vs;
#pragma unroll
            for (int e = 0; e < EPL; ++e) o[t][e] = fmaf(pv, vc[e], o[t][e]);
        }
    };
    auto unpack_params = [](uint32_t v, float& scale, float& zero) {
        scale = (float)__builtin_bit_cast(_Float16, (uint16_t)(v & 0xFFFFu));
        zero = (float)__builtin_bit_cast(_Float16, (uint16_t)(v >> 16));
    };
    int r_begin, r_end;
    {   // important tokens, 4 bits
        constexpr int NW = EPL * 4 / 32;
        const int L = max(0, min(len_hi[u], cap_hi));
        split_range64(L, split, nsplit, r_begin, r_end);
        const int64_t base = (int64_t)u * cap_hi;
        // the loads of the next 16 rows are issued before the current ones are consumed
        uint32_t kw[NW], vw[NW], kp, vp;
        auto fetch = [&](int r, uint32_t (&kw_)[NW], uint32_t (&vw_)[NW], uint32_t& kp_, uint32_t& vp_) {
            const int64_t row = base + (r < r_end ? r : r_begin);
            load_words<NW>(Kq.hi_codes + row * (D / 2) + sub * (NW * 4), kw_);
            load_words<NW>(Vq.hi_codes + row * (D / 2) + sub * (NW * 4), vw_);
            kp_ = Kq.hi_params[row];
            vp_ = Vq.hi_params[row];
        };
        int r = r_begin + w * 16 + rg;
        if (r - rg - w * 16 < r_end) fetch(r, kw, vw, kp, vp);
        for (; r - rg - w * 16 < r_end; r += 64) {
            const bool valid = r < r_end;
            uint32_t kw2[NW], vw2[NW], kp2 = 0, vp2 = 0;
            const bool more = r + 64 - rg - w * 16 < r_end;
            if (more) fetch(r + 64, kw2, vw2, kp2, vp2);
            float ks, kz, vs, vz, kc[EPL], vc[EPL];
            unpack_params(kp, ks, kz);
            unpack_params(vp, vs, vz);
            codes_to_floats<4, NW>(kw, kc);
            codes_to_floats<4, NW>(vw, vc);
            attend(valid, kc, ks, kz, vc, vs, vz);
            if (more) {
#pragma unroll
                for (int i = 0; i < NW; ++i) { kw[i] = kw2[i]; vw[i] = vw2[i]; }
                kp = kp2; vp = vp2;
            }
        }
    }
    {   // the other tokens, 2 bits
        constexpr int NW = EPL * 2 / 32;
        const int L = max(0, min(len_lo[u], cap_lo));
        split_range64(L, split, nsplit, r_begin, r_end);
        const int64_t base = (int64_t)u * cap_lo;
        // the loads of the next 16 rows are issued before the current ones are consumed
        uint32_t kw[NW], vw[NW], kp, vp;
        auto fetch = [&](int r, uint32_t (&kw_)[NW], uint32_t (&vw_)[NW], uint32_t& kp_, uint32_t& vp_) {
            const int64_t row = base + (r < r_end ? r : r_begin);
            load_words<NW>(Kq.lo_codes + row * (D / 4) + sub * (NW * 4), kw_);
            load_words<NW>(Vq.lo_codes + row * (D / 4) + sub * (NW * 4), vw_);
            kp_ = Kq.lo_params[row];
            vp_ = Vq.lo_params[row];
        };
        int r = r_begin + w * 16 + rg;
        if (r - rg - w * 16 < r_end) fetch(r, kw, vw, kp, vp);
        for (; r - rg - w * 16 < r_end; r += 64) {
            const bool valid = r < r_end;
            uint32_t kw2[NW], vw2[NW], kp2 = 0, vp2 = 0;
            const bool more = r + 64 - rg - w * 16 < r_end;
            if (more) fetch(r + 64, kw2, vw2, kp2, vp2);
            float ks, kz, vs, vz, kc[EPL], vc[EPL];
            unpack_params(kp, ks, kz);
            unpack_params(vp, vs, vz);
            codes_to_floats<2, NW>(kw, kc);
            codes_to_floats<2, NW>(vw, vc);
            attend(valid, kc, ks, kz, vc, vs, vz);
            if (more) {
#pragma unroll
                for (int i = 0; i < NW; ++i) { kw[i] = kw2[i]; vw[i] = vw2[i]; }
                kp = kp2; vp = vp2;
            }
        }
    }
    if (Kt) {   // rows appended during decoding, as stored: "codes" are the values, scale 1, zero 0
        const int L = max(0, min(len_t[u], cap_t));
        split_range64(L, split, nsplit, r_begin, r_end);
        const T* Kb = Kt + (int64_t)u * cap_t * D + sub * EPL;
        const T* Vb = Vt + (int64_t)u * cap_t * D + sub * EPL;
        for (int r = r_begin + w * 16 + rg; r - rg - w * 16 < r_end; r += 64) {
            const bool valid = r < r_end;
            const int rr = valid ? r : r_begin;
            float kc[EPL], vc[EPL];
#pragma unroll
            for (int e8 = 0; e8 < EPL / 8; ++e8) {
                float f[8];
                RowChunk<T, 8>::load(Kb + (int64_t)rr * D + 8 * e8, f);
#pragma unroll
                for (int e = 0; e < 8; ++e) kc[8 * e8 + e] = f[e];
                RowChunk<T, 8>::load(Vb + (int64_t)rr * D + 8 * e8, f);
#pragma unroll
                for (int e = 0; e < 8; ++e) vc[8 * e8 + e] = f[e];
            }
            attend(valid, kc, 1.f, 0.f, vc, 1.f, 0.f);
        }
    }
    // fold the zero-point sums into the outputs, merge the 16 row groups of the wave, then the 4 waves
#pragma unroll
    for (int t = 0; t < GT; ++t) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) o[t][e] += zacc[t];
#pragma unroll
        for (int off = 4; off <= 32; off <<= 1) {
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
    combine_waves<D, GT>(red, u, G, gbase, split, nsplit, part);
}

static int decode_splits(const zipvl_dims& d, int cap) {
    const int units = d.B * d.Hkv;
    int s = (1024 + units - 1) / units;
    const int by_len = (cap + 255) / 256;                   // at least 256 rows per split
    s = s < by_len ? s : by_len;
    return s < 1 ? 1 : (s > kDecMaxSplit ? kDecMaxSplit : s);
}

static int row_splits(int cap) { const int r = rows_per_split(cap); return (cap + r - 1) / r; }

size_t decode_workspace_bytes(const zipvl_dims& d, int cap) {
    const int s = std::max(decode_splits(d, cap), row_splits(cap));     // either split scheme fits
    return (size_t)d.B * d.Hq * s * (d.d + 2) * sizeof(float);
}

template <typename T, int D>
static int launch_decode_t(const void* q, const void* Kc, const void* Vc, const int32_t* len, int32_t cap,
                           const zipvl_dims& d, float scale, void* o, void* ws, hipStream_t st)
{
    const int G = d.Hq / d.Hkv, units = d.B * d.Hkv, rows = rows_per_split(cap), max_splits = row_splits(cap);
    const float c = scale * kLog2e;
    dim3 grid(max_splits, units);
#define ZIPVL_DEC(GT, GB)                                                                            \
    hipLaunchKernelGGL((decode_partial_kernel<T, D, GT>), grid, dim3(256), 0, st, (const T*)q,       \
        (const T*)Kc, (const T*)Vc, len, cap, d.Hq, d.Hkv, GB, c, (float*)ws, rows, max_splits)
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
    hipLaunchKernelGGL((decode_combine_kernel<T, D>), dim3(units), dim3(256), 0, st,
        (const float*)ws, len, cap, rows, 0, max_splits, G, (T*)o);
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
        if (G <= 2) {
            if (rem == 2)
                hipLaunchKernelGGL((decode_q4_partial_kernel<T, D, 2>), grid, dim3(256), 0, st, (const T*)q, kq, vq,
                    len_hi, len_lo, cap_hi, cap_lo, (const T*)Kt, (const T*)Vt, len_t, cap_t, d.Hq, d.Hkv, gb, c, (float*)ws, nsplit);
            else
                hipLaunchKernelGGL((decode_q4_partial_kernel<T, D, 1>), grid, dim3(256), 0, st, (const T*)q, kq, vq,
                    len_hi, len_lo, cap_hi, cap_lo, (const T*)Kt, (const T*)Vt, len_t, cap_t, d.Hq, d.Hkv, gb, c, (float*)ws, nsplit);
        }
        else if (rem >= 5) ZIPVL_DECQ(8, gb);
        else if (rem >= 3) ZIPVL_DECQ(4, gb);
        else if (rem == 2) ZIPVL_DECQ(2, gb);
        else ZIPVL_DECQ(1, gb);
        int rc = check_launch("decode_q_partial");
        if (rc) return rc;
    }
#undef ZIPVL_DECQ
    KernelTimer tm(ZIPVL_K_DECODE_COMBINE, st);
    hipLaunchKernelGGL((decode_combine_kernel<T, D>), dim3(units), dim3(256), 0, st,
        (const float*)ws, (const int32_t*)nullptr, 0, 1, nsplit, nsplit, G, (T*)o);
    return check_launch("decode_combine");
}

static size_t step_counter_bytes(const zipvl_dims& d) { return ((size_t)d.B * d.Hkv * sizeof(unsigned) + 255) / 256 * 256; }

size_t decode_step_workspace_bytes(const zipvl_dims& d, int cap) {
    return step_counter_bytes(d) + decode_workspace_bytes(d, cap);
}

template <typename T, int D>
static int launch_decode_step_t(const void* q, void* Kc, void* Vc, int32_t* len, int32_t cap, const void* k_new,
                                const void* v_new, const zipvl_dims& d, float scale, void* o, void* ws, hipStream_t st)
{
    const int G = d.Hq / d.Hkv, units = d.B * d.Hkv, rows = rows_per_split(cap), max_splits = row_splits(cap);
    unsigned* arrived = (unsigned*)ws;
    float* part = (float*)((char*)ws + step_counter_bytes(d));
    if (G > 8) {                                            // several passes over the cache per step: not fused
        int rc = launch_kv_append(Kc, Vc, len, cap, k_new, v_new, d, st);
        if (rc) return rc;
        return launch_decode_attn(q, Kc, Vc, len, cap, d, scale, o, part, st);
    }
    const float c = scale * kLog2e;
    dim3 grid(max_splits, units);
    KernelTimer tm(ZIPVL_K_DECODE_STEP, st);
#define ZIPVL_STEP(GT)                                                                               \
    hipLaunchKernelGGL((decode_step_kernel<T, D, GT>), grid, dim3(256), 0, st, (const T*)q, (T*)Kc, (T*)Vc, len, cap, \
        (const T*)k_new, (const T*)v_new, d.Hq, d.Hkv, c, part, rows, max_splits, arrived, (T*)o)
    if (G >= 5) ZIPVL_STEP(8);
    else if (G >= 3) ZIPVL_STEP(4);
    else if (G == 2) ZIPVL_STEP(2);
    else ZIPVL_STEP(1);
#undef ZIPVL_STEP
    return check_launch("decode_step");
}

int launch_decode_step(const void* q, void* Kc, void* Vc, int32_t* len, int32_t cap, const void* k_new,
                       const void* v_new, const zipvl_dims& d, float scale, void* o, void* ws, hipStream_t st)
{
    if (d.dtype == ZIPVL_BF16) {
        if (d.d == 128) return launch_decode_step_t<__bf16, 128>(q, Kc, Vc, len, cap, k_new, v_new, d, scale, o, ws, st);
        return launch_decode_step_t<__bf16, 64>(q, Kc, Vc, len, cap, k_new, v_new, d, scale, o, ws, st);
    }
    if (d.d == 128) return launch_decode_step_t<float, 128>(q, Kc, Vc, len, cap, k_new, v_new, d, scale, o, ws, st);
    return launch_decode_step_t<float, 64>(q, Kc, Vc, len, cap, k_new, v_new, d, scale, o, ws, st);
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

// ---------------------------------------------------------------- decode attention without a caller workspace
// The partial states of the split-KV kernels live in a fixed device array of this library instead of a
// workspace argument, for callers that cannot allocate.  Every GPU holds its own copy of the array at its
// own address: the address is looked up once per device (with that device current) and only that pointer
// is ever handed to kernels.  Nothing in the array has to start at zero: every (unit, head, split) slot is
// written by the partial kernel before the combine kernel of the same call reads it.
constexpr size_t kStaticScratchBytes = ZIPVL_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
static std::mutex g_scratch_mu;
static void* g_scratch_ptr[kMaxDevices] = {};

static int static_scratch(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return set_error(ZIPVL_EHIP, "decode_attn_static: hipGetDevice failed: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return set_error(ZIPVL_EUNSUPPORTED, "decode_attn_static: device ordinal %d is beyond %d", dev, kMaxDevices);
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return set_error(ZIPVL_EHIP, "decode_attn_static: no device address for the scratch array: %s", hipGetErrorString(e));
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return ZIPVL_OK;
}

int launch_decode_attn_static(const void* q, const void* Kc, const void* Vc, const int32_t* len, int32_t cap,
                              const zipvl_dims& d, float scale, void* o, hipStream_t st)
{
    const size_t need = decode_workspace_bytes(d, cap);
    if (need > kStaticScratchBytes)
        return set_error(ZIPVL_ESHAPE, "decode_attn_static: these dims need %zu bytes of partial states, the built-in scratch holds %zu "
                                       "(use zipvl_decode_attn with a workspace)", need, kStaticScratchBytes);
    void* ws = nullptr;
    const int rc = static_scratch(&ws);
    if (rc) return rc;
    return launch_decode_attn(q, Kc, Vc, len, cap, d, scale, o, ws, st);
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
