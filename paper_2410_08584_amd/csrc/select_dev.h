// Device code of the selection (Eq. (7), Eq. (9)) that is shared by the stand-alone select kernels and by
// the score kernel that ends with the selection of its unit.
//
// Two-level form of the radix descent.  The first digit is 12 bits wide (exponent byte and four mantissa
// bits of the order-preserving key: 4096 bins) and its histograms - element count packed over the exact
// integer score sum for the accumulated scores, plain counts for the normalised scores - are built by
// many workgroups in parallel (each in LDS over its own slice of positions, then added to a per-unit
// table in memory).  One workgroup per unit then finishes: it scans the table for the bin where the
// descending cumulative sum crosses the target, gathers that bin's few elements into a list in LDS, and
// runs the remaining 19 bits of the descent (7 + 6 + 6) on the list; the same for the k-th largest
// normalised score on counts; then the ascending emission.  Everything is integer arithmetic on exact
// values, so the result is the full sort's, whatever the order in which the table was accumulated.
#pragma once
#include "common.h"

namespace zipvl {

constexpr int kSelBins = 4096;              // first digit: the top 12 of the 31 key bits
constexpr int kSelBinShift = 19;
constexpr int kSelMaxCand = 2048;           // elements of one bin that are gathered into a list
constexpr int kSumBits = 41;                // a packed slot: count << 41 | integer score sum (sum of a unit < 2^41)

// Order-preserving 31-bit key of a non-negative fp32 score: its bit pattern.  Scores are >= 0 by
// contract; anything with the sign bit set (-0 included) is ordered and summed as zero.
__device__ __forceinline__ uint32_t orderable(float x) {
    const uint32_t b = __float_as_uint(x);
    return (b & 0x80000000u) ? 0u : b;
}

// floor(x * 2^40) for finite x in [0, 2^24), exact, integer-only.
__device__ __forceinline__ unsigned long long fixed40(float x) {
    const uint32_t b = __float_as_uint(x);
    const int e = (b >> 23) & 255;
    if ((b & 0x80000000u) || e == 0 || e == 255) return 0ull;
    const unsigned long long M = (b & 0x7FFFFFu) | 0x800000u;     // x = M * 2^(e-150)
    const int sh = e - 110;
    if (sh >= 0) return M << (sh > 40 ? 40 : sh);
    return (-sh >= 24) ? 0ull : (M >> (-sh));
}

__device__ __forceinline__ unsigned long long fixed40_of_key(uint32_t key) { return fixed40(__uint_as_float(key)); }

// Loads of data that other workgroups of the same launch may have written (COH): device-scope, so that they
// are served from the coherence point and not from this XCD's L2.
template <bool COH> __device__ __forceinline__ float sel_ld(const float* p) {
    if constexpr (COH) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else return *p;
}
template <bool COH> __device__ __forceinline__ uint32_t sel_ld(const uint32_t* p) {
    if constexpr (COH) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else return *p;
}
template <bool COH> __device__ __forceinline__ unsigned long long sel_ld(const unsigned long long* p) {
    if constexpr (COH) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else return *p;
}

struct TailShared {
    unsigned long long hist[128];            // histogram of one digit of the list descent (packed, or counts)
    uint32_t list[kSelMaxCand];              // the gathered elements of the crossing bin
    unsigned long long wsum[16];             // per-wave totals of a workgroup scan
    uint32_t wcnt[16];
    uint32_t wave_cnt[16], wave_eq[16];      // emission
    unsigned long long target, base_sum;
    uint32_t base_cnt, sel_digit, sel_cnt, sole_key;
    int k;
};

// Exclusive prefix (ec, es) of the per-thread pair (lc, ls) over the workgroup in thread order, and the totals.
template <int NTH>
__device__ __forceinline__ void block_scan(uint32_t lc, unsigned long long ls, TailShared& sh,
                                           uint32_t& ec, unsigned long long& es, uint32_t& tc, unsigned long long& ts) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t ic = lc;
    unsigned long long is = ls;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t c2 = __shfl_up(ic, o);
        const unsigned long long s2 = __shfl_up(is, o);
        if (lane >= o) { ic += c2; is += s2; }
    }
    if (lane == 63) { sh.wcnt[wave] = ic; sh.wsum[wave] = is; }
    __syncthreads();
    ec = ic - lc; es = is - ls; tc = 0; ts = 0;
#pragma unroll
    for (int w2 = 0; w2 < NTH / 64; ++w2) {
        const uint32_t c2 = sh.wcnt[w2];
        const unsigned long long s2 = sh.wsum[w2];
        if (w2 < wave) { ec += c2; es += s2; }
        tc += c2; ts += s2;
    }
    __syncthreads();
}

// Where the keys of the vector in use live: n order-preserving keys in LDS, or (longer vectors) the fp32
// values in memory, re-read by every sweep.
template <int NTH, bool COH>
struct KeySrc {
    const uint32_t* lds;
    const float* x;
    int n;
    template <typename F>
    __device__ __forceinline__ void for_each(F&& f) const {
        if (lds) {
#pragma unroll 4
            for (int j = threadIdx.x; j < n; j += NTH) f(lds[j]);
        } else {
#pragma unroll 4
            for (int j = threadIdx.x; j < n; j += NTH) f(orderable(sel_ld<COH>(x + j)));
        }
    }
};

template <int NTH>
struct ListSrc {
    const uint32_t* list;
    int n;
    template <typename F>
    __device__ __forceinline__ void for_each(F&& f) const {
        for (int j = threadIdx.x; j < n; j += NTH) f(list[j]);
    }
};

// First digit from the per-unit table.  Thread t owns the bins 4095 - t*BPT downwards: table_load fetches them
// (early, so that the memory latency overlaps the key loads), table_cross finds the bin where the descending
// cumulative sum (WITH_SUM) or count crosses the target and leaves sel_digit, base_cnt, base_sum, sel_cnt (and
// target, WITH_SUM) in sh.
template <int NTH> struct TableRegs {
    static constexpr int BPT = kSelBins / NTH;
    unsigned long long v[BPT];      // packed slots, or plain counts
};

template <int NTH, bool COH>
__device__ __forceinline__ void table_load(const unsigned long long* __restrict__ hm, const uint32_t* __restrict__ hr, TableRegs<NTH>& r) {
    constexpr int BPT = kSelBins / NTH;
#pragma unroll
    for (int t = 0; t < BPT; ++t) {
        const int bin = kSelBins - 1 - ((int)threadIdx.x * BPT + t);
        r.v[t] = hr ? (unsigned long long)sel_ld<COH>(hr + bin) : sel_ld<COH>(hm + bin);
    }
}

template <int NTH, bool WITH_SUM>
__device__ void table_cross(const TableRegs<NTH>& r, bool packed, double tau, uint32_t cnt_target, TailShared& sh) {
    constexpr int BPT = kSelBins / NTH;
    const int tid = threadIdx.x;
    uint32_t c[BPT], lc = 0;
    unsigned long long s[BPT], ls = 0;
#pragma unroll
    for (int t = 0; t < BPT; ++t) {
        c[t] = packed ? (uint32_t)(r.v[t] >> kSumBits) : (uint32_t)r.v[t];
        s[t] = WITH_SUM ? (r.v[t] & ((1ull << kSumBits) - 1ull)) : 0ull;
        lc += c[t]; ls += s[t];
    }
    uint32_t ec, tc;
    unsigned long long es, ts;
    block_scan<NTH>(lc, ls, sh, ec, es, tc, ts);
    unsigned long long target = cnt_target;
    if (WITH_SUM) {
        // ceil(tau * W): one IEEE double multiply, then ceil (W < 2^53)
        target = (unsigned long long)ceil(tau * (double)ts);
        if (tid == 0) sh.target = target;
    }
    uint32_t rc = ec;
    unsigned long long rs = es;
#pragma unroll
    for (int t = 0; t < BPT; ++t) {
        const bool cross = WITH_SUM ? (rs < target && target <= rs + s[t])
                                    : ((unsigned long long)rc < target && target <= (unsigned long long)rc + c[t]);
        if (cross) {
            sh.sel_digit = kSelBins - 1 - (tid * BPT + t);
            sh.base_cnt = rc;
            sh.base_sum = rs;
            sh.sel_cnt = c[t];
        }
        rc += c[t];
        rs += s[t];
    }
    __syncthreads();
}

// The elements whose first digit is `bin`, gathered into sh.list (any order); at most kSelMaxCand of them exist.
// cnt: how many of them this thread will meet in its sweep (counted by the caller, or -1: counted here).
template <int NTH, typename Src>
__device__ int gather_bin(const Src& src, uint32_t bin, int cnt_known, TailShared& sh) {
    uint32_t cnt = cnt_known >= 0 ? (uint32_t)cnt_known : 0u;
    if (cnt_known < 0) src.for_each([&](uint32_t key) { cnt += (key >> kSelBinShift) == bin ? 1u : 0u; });
    uint32_t ec, tc;
    unsigned long long es, ts;
    block_scan<NTH>(cnt, 0ull, sh, ec, es, tc, ts);
    uint32_t pos = ec;
    src.for_each([&](uint32_t key) {
        if ((key >> kSelBinShift) == bin && pos < (uint32_t)kSelMaxCand) sh.list[pos++] = key;
    });
    __syncthreads();
    return (int)min(tc, (uint32_t)kSelMaxCand);
}

// The remaining 19 bits (7 + 6 + 6) of the descent over the elements of `src` that match prefix under mask.
// On return prefix holds the key at which the cumulative sum / count crosses, base_cnt / base_sum what lies
// strictly above it.
template <int NTH, bool WITH_SUM, typename Src>
__device__ void descend_low(const Src& src, unsigned long long target, TailShared& sh,
                            uint32_t& prefix, uint32_t& base_cnt, unsigned long long& base_sum) {
    const int tid = threadIdx.x;
    uint32_t mask = (uint32_t)(kSelBins - 1) << kSelBinShift;
    for (int pass = 0; pass < 3; ++pass) {
        const int shift = pass == 0 ? 12 : pass == 1 ? 6 : 0;
        const int bits = pass == 0 ? 7 : 6;
        const uint32_t dmask = (1u << bits) - 1u;
        const int nb = 1 << bits;
        if (tid < nb) sh.hist[tid] = 0ull;
        __syncthreads();
        src.for_each([&](uint32_t key) {
            if ((key & mask) == prefix)
                atomicAdd(&sh.hist[(key >> shift) & dmask], WITH_SUM ? (1ull << kSumBits) + fixed40_of_key(key) : 1ull);
        });
        __syncthreads();
        if (tid < 64) {
            // lane l owns bins nb-1-2l and nb-2-2l (descending value order); only the first nb/2 lanes hold bins
            uint32_t c[2], lc = 0;
            unsigned long long s[2], ls = 0;
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int bin = nb - 1 - (2 * tid + t);
                const unsigned long long v = bin >= 0 ? sh.hist[bin] : 0ull;
                c[t] = WITH_SUM ? (uint32_t)(v >> kSumBits) : (uint32_t)v;
                s[t] = WITH_SUM ? (v & ((1ull << kSumBits) - 1ull)) : 0ull;
                lc += c[t]; ls += s[t];
            }
            uint32_t ic = lc;
            unsigned long long is = ls;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const uint32_t c2 = __shfl_up(ic, o);
                const unsigned long long s2 = __shfl_up(is, o);
                if (tid >= o) { ic += c2; is += s2; }
            }
            uint32_t rc = base_cnt + (ic - lc);
            unsigned long long rs = base_sum + (is - ls);
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const bool cross = WITH_SUM ? (rs < target && target <= rs + s[t])
                                            : ((unsigned long long)rc < target && target <= (unsigned long long)rc + c[t]);
                if (cross) {
                    sh.sel_digit = nb - 1 - (2 * tid + t);
                    sh.base_cnt = rc;
                    sh.base_sum = rs;
                    sh.sel_cnt = c[t];
                }
                rc += c[t];
                rs += s[t];
            }
        }
        __syncthreads();
        prefix |= sh.sel_digit << shift;
        mask |= dmask << shift;
        base_cnt = sh.base_cnt;
        base_sum = sh.base_sum;
        if (pass < 2 && sh.sel_cnt == 1u) {
            // one element left under this prefix: the remaining digits are its own
            src.for_each([&](uint32_t key) { if ((key & mask) == prefix) sh.sole_key = key; });
            __syncthreads();
            prefix = sh.sole_key;
            break;
        }
    }
}

// After table_cross: the key at which the descending cumulative sum (WITH_SUM) or count crosses the target, with the
// count / sum strictly above it.  my_cnt: elements of the crossing bin in this thread's sweep, or -1 if not counted.
// Returns false when all scores are zero (WITH_SUM only).
template <int NTH, bool COH, bool WITH_SUM>
__device__ bool crossing_key(const KeySrc<NTH, COH>& keys, uint32_t cnt_target, int my_cnt, TailShared& sh, uint32_t& key_out,
                             uint32_t& base_cnt, unsigned long long& base_sum, unsigned long long& target) {
    target = WITH_SUM ? sh.target : (unsigned long long)cnt_target;
    if (WITH_SUM && target == 0ull) return false;
    const uint32_t bin = sh.sel_digit, in_bin = sh.sel_cnt;
    uint32_t prefix = bin << kSelBinShift;
    base_cnt = sh.base_cnt;
    base_sum = sh.base_sum;
    __syncthreads();                                         // every thread has read sh before it is reused
    if (in_bin == 1u) {
        keys.for_each([&](uint32_t key) { if ((key >> kSelBinShift) == bin) sh.sole_key = key; });
        __syncthreads();
        prefix = sh.sole_key;
    } else if (in_bin <= (uint32_t)kSelMaxCand) {
        const int nl = gather_bin<NTH>(keys, bin, my_cnt, sh);
        descend_low<NTH, WITH_SUM>(ListSrc<NTH>{sh.list, nl}, target, sh, prefix, base_cnt, base_sum);
    } else {
        descend_low<NTH, WITH_SUM>(keys, target, sh, prefix, base_cnt, base_sum);
    }
    key_out = prefix;
    return true;
}

// Ascending emission of {key > vstar} plus the first need_eq positions with key == vstar.  Keys of positions
// [b0, b0 + bn) are at lds_keys[off .. off + bn): thread t classifies 32 consecutive positions into two bit
// masks, a workgroup scan of the populations gives its output offset, ties are cut by the scanned count.
template <int NTH>
__device__ void emit_block(const uint32_t* lds_keys, int b0, int bn, uint32_t vstar, uint32_t need_eq,
                           uint32_t& gt_run, uint32_t& eq_run, TailShared& sh, int32_t* __restrict__ idx) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int base = tid * 32;
    uint32_t gm = 0, em = 0;
    if (base < bn) {
        // all 32 reads are issued at once (index clamped, the mask bit predicated instead); the rotation by the
        // lane spreads the 64 reads of a wave over the banks
        uint32_t key[32];
#pragma unroll
        for (int cc = 0; cc < 32; ++cc) key[cc] = lds_keys[min(base + ((cc + lane) & 31), bn - 1)];
#pragma unroll
        for (int cc = 0; cc < 32; ++cc) {
            const int p = (cc + lane) & 31;
            const bool in = base + p < bn;
            gm |= (in && key[cc] > vstar ? 1u : 0u) << p;
            em |= (in && key[cc] == vstar ? 1u : 0u) << p;
        }
    }
    const uint32_t cg = __popc(gm), ce = __popc(em);
    uint32_t ig = cg, ie = ce;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t tg = __shfl_up(ig, o), te = __shfl_up(ie, o);
        if (lane >= o) { ig += tg; ie += te; }
    }
    if (lane == 63) { sh.wave_cnt[wave] = ig; sh.wave_eq[wave] = ie; }
    __syncthreads();
    uint32_t gt_before = gt_run + (ig - cg), eq_before = eq_run + (ie - ce), tot_g = 0, tot_e = 0;
#pragma unroll
    for (int w2 = 0; w2 < NTH / 64; ++w2) {
        const uint32_t wg = sh.wave_cnt[w2], we = sh.wave_eq[w2];
        if (w2 < wave) { gt_before += wg; eq_before += we; }
        tot_g += wg; tot_e += we;
    }
    __syncthreads();
    // of this thread's ties, the lowest-indexed `allow` are kept
    const uint32_t allow = need_eq > eq_before ? need_eq - eq_before : 0u;
    uint32_t ek = em;
    if (allow < ce) {
        ek = 0;
        uint32_t rest = em;
        for (uint32_t a2 = 0; a2 < allow; ++a2) {
            const uint32_t low = rest & (0u - rest);
            ek |= low;
            rest ^= low;
        }
    }
    uint32_t km = gm | ek;
    uint32_t out = gt_before + min(eq_before, need_eq);
    while (km) {
        const int p = __builtin_ctz(km);
        km &= km - 1;
        idx[out++] = b0 + base + p;
    }
    gt_run += tot_g;
    eq_run += tot_e;
}

// What the contract of the selection excludes, looked for in the inputs of one unit (one more pass over both
// vectors, only when the caller asks for the status word): bit 0 an entry with the sign bit set (ordered and summed as
// zero), bit 1 an infinity or NaN (ordered by its bits, summed as zero), bit 2 the integer sum of `mass` reaches
// 2^41 (it no longer fits its field of a histogram slot: k is unreliable).  scratch: one 64-bit and one 32-bit
// word of LDS.  Every thread returns the same flags.
template <int NTH>
__device__ uint32_t input_flags(const float* __restrict__ mass, const float* __restrict__ rank, int n,
                                unsigned long long* sum_scratch, uint32_t* flag_scratch) {
    if (threadIdx.x == 0) { *sum_scratch = 0ull; *flag_scratch = 0u; }
    __syncthreads();
    uint32_t f = 0;
    unsigned long long s = 0;
    for (int j = threadIdx.x; j < n; j += NTH) {
        const uint32_t bm = __float_as_uint(mass[j]);
        f |= (bm >> 31) | (((bm >> 23) & 255u) == 255u ? 2u : 0u);
        s += fixed40(mass[j]);
        if (rank != mass) {
            const uint32_t br = __float_as_uint(rank[j]);
            f |= (br >> 31) | (((br >> 23) & 255u) == 255u ? 2u : 0u);
        }
    }
    if (f) atomicOr(flag_scratch, f);
    if (s) atomicAdd(sum_scratch, s);
    __syncthreads();
    return *flag_scratch | (*sum_scratch >= (1ull << kSumBits) ? 4u : 0u);
}

// One unit, one workgroup of NTH threads: k from (mass, hm), T from (rank, hr) -> idx, k_out.
// lds_keys: key_cap words of LDS (key_cap a multiple of 32).  rank == mass (and hr null): one vector for both steps.
template <int NTH, bool COH>
__device__ void select_tail(const float* __restrict__ mass, const float* __restrict__ rank, int n, double tau,
                            const unsigned long long* __restrict__ hm, const uint32_t* __restrict__ hr,
                            int32_t* __restrict__ idx, int32_t* __restrict__ k_out, uint32_t* lds_keys, int key_cap,
                            TailShared& sh) {
    const int tid = threadIdx.x;
    if (tau >= 1.0) {
        if (tid == 0) *k_out = n;
        for (int j = tid; j < n; j += NTH) idx[j] = j;
        return;
    }
    const bool in_lds = n <= key_cap;
    const bool two = rank != mass;
    constexpr int kPre = 8;                                  // values of the second vector a thread holds while the first is in use
    const bool pre_rank = in_lds && two && n <= kPre * NTH;
    // everything the first step needs from memory is requested at once: both tables, the first vector, and (short
    // vectors) the second vector, which waits in registers
    TableRegs<NTH> tm, tr;
    table_load<NTH, COH>(hm, nullptr, tm);
    if (two) table_load<NTH, COH>(hm, hr, tr);
    float pre[kPre];
    if (pre_rank) {
#pragma unroll
        for (int q = 0; q < kPre; ++q) pre[q] = sel_ld<COH>(rank + min(tid + q * NTH, n - 1));
    }
    // ---- how many (Eq. (7)) ----
    table_cross<NTH, true>(tm, true, tau, 0u, sh);
    const uint32_t bin_m = sh.sel_digit;                     // garbage when every score is zero: unused then
    int my_cnt = -1;
    if (in_lds) {
        // keys into LDS; the elements of the crossing bin are counted on the way
        my_cnt = 0;
#pragma unroll 8
        for (int j = tid; j < n; j += NTH) {
            const uint32_t key = orderable(sel_ld<COH>(mass + j));
            lds_keys[j] = key;
            my_cnt += (key >> kSelBinShift) == bin_m ? 1 : 0;
        }
        __syncthreads();
    }
    int k = 1;
    {
        uint32_t key, base_cnt;
        unsigned long long base_sum, target;
        const KeySrc<NTH, COH> mk{in_lds ? lds_keys : nullptr, mass, n};
        if (crossing_key<NTH, COH, true>(mk, 0u, my_cnt, sh, key, base_cnt, base_sum, target)) {
            const unsigned long long qv = fixed40_of_key(key);
            const unsigned long long need = target - base_sum;              // >= 1
            k = (int)(base_cnt + (qv ? (need + qv - 1) / qv : 1ull));
        }
        k = max(1, min(k, n));
    }
    if (tid == 0) *k_out = k;
    if (k >= n) {
        for (int j = tid; j < n; j += NTH) idx[j] = j;
        return;
    }
    __syncthreads();
    // ---- which (Eq. (9)): k-th largest normalised score v*, ties to the lower index ----
    table_cross<NTH, false>(two ? tr : tm, !two, tau, (uint32_t)k, sh);
    const uint32_t bin_r = sh.sel_digit;
    if (in_lds && two) {
        my_cnt = 0;
        if (pre_rank) {
#pragma unroll
            for (int q = 0; q < kPre; ++q) {
                const int j = tid + q * NTH;
                if (j < n) {
                    const uint32_t key = orderable(pre[q]);
                    lds_keys[j] = key;
                    my_cnt += (key >> kSelBinShift) == bin_r ? 1 : 0;
                }
            }
        } else {
#pragma unroll 8
            for (int j = tid; j < n; j += NTH) {
                const uint32_t key = orderable(sel_ld<COH>(rank + j));
                lds_keys[j] = key;
                my_cnt += (key >> kSelBinShift) == bin_r ? 1 : 0;
            }
        }
        __syncthreads();
    } else {
        my_cnt = -1;                                         // one vector for both steps: other bin, counted in the gather
    }
    uint32_t vstar, cnt_gt;
    {
        unsigned long long unused, target;
        const KeySrc<NTH, COH> rk{in_lds ? lds_keys : nullptr, rank, n};
        crossing_key<NTH, COH, false>(rk, (uint32_t)k, my_cnt, sh, vstar, cnt_gt, unused, target);
    }
    const uint32_t need_eq = (uint32_t)k - cnt_gt;           // ties at v* that are kept (>= 1)
    __syncthreads();
    // ---- ascending emission, 32 NTH positions (or as many as LDS holds) at a time ----
    uint32_t gt_run = 0, eq_run = 0;
    const int blk = min(key_cap, 32 * NTH);
    for (int b0 = 0; b0 < n; b0 += blk) {
        const int bn = min(blk, n - b0);
        if (!in_lds) {
            __syncthreads();
#pragma unroll 8
            for (int j = tid; j < bn; j += NTH) lds_keys[j] = orderable(sel_ld<COH>(rank + b0 + j));
            __syncthreads();
        }
        emit_block<NTH>(in_lds ? lds_keys + b0 : lds_keys, b0, bn, vstar, need_eq, gt_run, eq_run, sh, idx);
    }
}

// A slice of positions of one unit -> the first-digit histograms, accumulated in LDS (lm: kSelBins packed slots,
// lr: kSelBins counts, both zero on entry) by the caller; this adds the non-empty bins to the unit's tables.
template <int NTH>
__device__ __forceinline__ void flush_tables(const unsigned long long* lm, const uint32_t* lr,
                                             unsigned long long* __restrict__ hm, uint32_t* __restrict__ hr) {
    for (int b = threadIdx.x; b < kSelBins; b += NTH) {
        const unsigned long long v = lm[b];
        if (v) __hip_atomic_fetch_add(hm + b, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (hr) {
            const uint32_t c = lr[b];
            if (c) __hip_atomic_fetch_add(hr + b, c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

}  // namespace zipvl
