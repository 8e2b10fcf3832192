// Adaptive count and important-token set (Eq. (7), Eq. (9); Algorithm 1 steps 3-5).
//
// The definition is "sort descending, cumulative sum, first crossing of
// tau * total, then top-k by the normalised score".  Neither step needs the
// sorted sequence itself:
//   * the first crossing of the sorted cumulative sum is found by a radix
//     descent over the 31-bit order-preserving image of the fp32 scores, in
//     8-bit digits: per digit, an LDS histogram of counts and of exact integer
//     sums (floor(x * 2^40), so the result is independent of summation order),
//     a descending wave-shuffle scan over the 256 bins, and the bin where the
//     running sum crosses the target; after four digits the remaining
//     candidates are equal and the count follows by one integer division;
//   * the top-k set is {score > v*} plus the lowest-indexed ties at v*, where
//     v* is the k-th largest value, found by the same descent on counts;
//   * the set is written in ascending position: every thread classifies 32
//     consecutive positions into two bit masks, a workgroup-wide scan of the
//     mask populations gives each thread its output offset.
// One 1024-thread workgroup per selection unit.  Up to n = 27648 the order-preserving keys of
// the vector in use are held in LDS (read from memory once, coalesced); longer vectors are
// re-read per digit and pass through LDS block by block for the emission.
#include <algorithm>
#include <atomic>

#include "launch.h"
#include "select_dev.h"

namespace zipvl {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kSelMaxLdsKeys = 27648;      // 108 KiB of keys beside the 32 KiB histogram
constexpr int kSelPre = kSelMaxLdsKeys / kSelThreads;   // keys per thread of a vector held in LDS
constexpr int kSelRep = 16, kSelRepStride = 257;    // histogram replicas and their spacing in slots

struct SelShared {
    unsigned long long hist[kSelRep * kSelRepStride];   // packed (count, integer sum) slots, or plain 32-bit counts
    unsigned long long folded[256];
    uint32_t wave_cnt[kSelWaves];
    uint32_t wave_eq[kSelWaves];
    unsigned long long target;
    unsigned long long base_sum;
    uint32_t base_cnt;
    uint32_t sel_digit;
    uint32_t sel_cnt;      // elements in the selected bin
    uint32_t sole_key;     // the key of a bin's only element
    int k;
};

// Where the keys of a unit live while the kernel runs: in LDS (filled once per vector with
// coalesced reads, then read conflict-free by every pass) when they fit, otherwise every pass
// re-reads the fp32 vector from global memory (any n).
struct Keys {
    const uint32_t* lds;      // n order-preserving keys, or nullptr
    const float* x;
    int n;
    template <typename F>
    __device__ __forceinline__ void for_each(F&& f) const {
        if (lds) {
#pragma unroll 4
            for (int j = threadIdx.x; j < n; j += kSelThreads) f(j, lds[j]);
        } else {
#pragma unroll 4
            for (int j = threadIdx.x; j < n; j += kSelThreads) f(j, orderable(x[j]));
        }
    }
};

__device__ __forceinline__ void fill_keys(uint32_t* dst, const float* __restrict__ x, int n) {
#pragma unroll 8
    for (int j = threadIdx.x; j < n; j += kSelThreads) dst[j] = orderable(x[j]);
}

// One descent over the 31 key bits in four digits, exponent byte first (8 + 8 + 8 + 7 bits).  The
// first two digits see many elements and spread them over kRep histogram replicas chosen by the
// lane (replica r of digit v sits at slot r * 257 + v: the lanes of a wave that share a digit hit
// different banks, and a fold over the replicas reads consecutive slots); later digits only see the
// few elements that share the prefix and use one replica.  WITH_SUM: a histogram slot packs the
// element count (bits 41..63) over the integer score sum (bits 0..40, sum of a unit < 2^41), one LDS
// atomic per element, and the descent crosses on the sum (target fixed after the first digit from
// the grand total); otherwise slots are plain counts and the descent crosses on cnt_target.
constexpr int kRep = kSelRep, kRepStride = kSelRepStride;

template <bool WITH_SUM>
__device__ void radix_descent(const Keys& keys, double tau, uint32_t cnt_target,
                              SelShared& sh, uint32_t& prefix_out, uint32_t& base_cnt_out,
                              unsigned long long& base_sum_out, bool& degenerate)
{
    const int tid = threadIdx.x;
    uint32_t* cnt_hist = reinterpret_cast<uint32_t*>(sh.hist);
    uint32_t prefix = 0, mask = 0, base_cnt = 0;
    unsigned long long base_sum = 0;
    degenerate = false;
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = pass < 3 ? 23 - 8 * pass : 0;
        const uint32_t dmask = pass < 3 ? 255u : 127u;
        const bool replicated = pass < 2;
        const int slots = replicated ? kRep * kRepStride : 256;
        const int rep_off = replicated ? (tid & (kRep - 1)) * kRepStride : 0;
        for (int i = tid; i < slots; i += kSelThreads) {
            if (WITH_SUM) sh.hist[i] = 0; else cnt_hist[i] = 0;
        }
        __syncthreads();
        keys.for_each([&](int, uint32_t key) {
            if ((key & mask) == prefix) {
                const int slot = rep_off + ((key >> shift) & dmask);
                if (WITH_SUM) atomicAdd(&sh.hist[slot], (1ull << kSumBits) + fixed40_of_key(key));
                else atomicAdd(&cnt_hist[slot], 1u);
            }
        });
        __syncthreads();
        if (replicated) {                                   // fold the replicas of bin `tid` into replica 0
            if (tid < 256) {
                uint32_t cc = 0;
                unsigned long long ss = 0;
#pragma unroll
                for (int r = 0; r < kRep; ++r) {
                    if (WITH_SUM) ss += sh.hist[r * kRepStride + tid];   // count and sum fields add without carry between them
                    else cc += cnt_hist[r * kRepStride + tid];
                }
                if (WITH_SUM) sh.folded[tid] = ss; else reinterpret_cast<uint32_t*>(sh.folded)[tid] = cc;
            }
            __syncthreads();
        }
        if (tid < 64) {
            // lane l owns bins 255-4l .. 252-4l (descending value order)
            const unsigned long long* h64 = replicated ? sh.folded : sh.hist;
            const uint32_t* h32 = reinterpret_cast<const uint32_t*>(h64);
            uint32_t c[4], lc = 0;
            unsigned long long s[4], ls = 0;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int bin = 255 - (4 * tid + t);
                if (WITH_SUM) {
                    const unsigned long long v = h64[bin];
                    c[t] = (uint32_t)(v >> kSumBits);
                    s[t] = v & ((1ull << kSumBits) - 1ull);
                } else {
                    c[t] = h32[bin];
                    s[t] = 0;
                }
                lc += c[t]; ls += s[t];
            }
            uint32_t ic = lc;
            unsigned long long is = ls;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const uint32_t tc = __shfl_up(ic, o);
                const unsigned long long ts = WITH_SUM ? __shfl_up(is, o) : 0ull;
                if (tid >= o) { ic += tc; is += ts; }
            }
            unsigned long long target;
            if (WITH_SUM) {
                if (pass == 0) {
                    const unsigned long long W = __shfl(is, 63);
                    // ceil(tau * W): one IEEE double multiply, then ceil (W < 2^53)
                    const double prod = tau * (double)W;
                    target = (unsigned long long)ceil(prod);
                    if (tid == 0) sh.target = target;
                } else {
                    target = sh.target;
                }
            } else {
                target = cnt_target;
            }
            uint32_t rc = base_cnt + (ic - lc);
            unsigned long long rs = base_sum + (is - ls);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const bool cross = WITH_SUM ? (rs < target && target <= rs + s[t])
                                            : ((unsigned long long)rc < target && target <= (unsigned long long)rc + c[t]);
                if (cross) {
                    sh.sel_digit = 255 - (4 * tid + t);
                    sh.base_cnt = rc;
                    sh.base_sum = rs;
                    sh.sel_cnt = c[t];
                }
                rc += c[t];
                rs += s[t];
            }
        }
        __syncthreads();
        if (WITH_SUM && sh.target == 0ull) { degenerate = true; break; }   // all scores zero
        prefix |= sh.sel_digit << shift;
        mask |= dmask << shift;
        base_cnt = sh.base_cnt;
        base_sum = sh.base_sum;
        if (pass < 3 && sh.sel_cnt == 1u) {
            // One element left under this prefix: the remaining digits are its own.  One sweep fetches the key
            // (the counts and sums above it are already final) instead of a histogram pass per digit.
            keys.for_each([&](int, uint32_t key) {
                if ((key & mask) == prefix) sh.sole_key = key;
            });
            __syncthreads();
            prefix = sh.sole_key;
            break;
        }
    }
    prefix_out = prefix;
    base_cnt_out = base_cnt;
    base_sum_out = base_sum;
}

__global__ __launch_bounds__(kSelThreads) void select_kernel(
    const float* __restrict__ mass_all, const float* __restrict__ rank_all, int n, double tau,
    int32_t* __restrict__ idx_all, int32_t* __restrict__ k_out, int keys_in_lds, int32_t* __restrict__ status)
{
    __shared__ SelShared sh;
    extern __shared__ uint32_t lds_keys[];             // kSelMaxLdsKeys entries
    const int u = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float* mass = mass_all + (int64_t)u * n;
    const float* rank = rank_all ? rank_all + (int64_t)u * n : mass;
    int32_t* idx = idx_all + (int64_t)u * n;
    if (status) {
        const uint32_t f = input_flags<kSelThreads>(mass, rank, n, &sh.base_sum, &sh.sel_cnt);
        if (tid == 0) status[u] = (int32_t)f;
        __syncthreads();
    }

    if (tau >= 1.0) {
        if (tid == 0) k_out[u] = n;
        for (int j = tid; j < n; j += kSelThreads) idx[j] = j;
        return;
    }

    // ---- how many (Eq. (7)) ----
    Keys mk{keys_in_lds ? lds_keys : nullptr, mass, n};
    if (keys_in_lds) { fill_keys(lds_keys, mass, n); __syncthreads(); }
    // the second vector is requested now and waits in registers while the first descent runs
    const bool second_vector = keys_in_lds && rank != mass;
    float pre[kSelPre];
    if (second_vector) {
#pragma unroll
        for (int q = 0; q < kSelPre; ++q) pre[q] = rank[min(tid + q * kSelThreads, n - 1)];   // independent loads
    }
    int k;
    {
        uint32_t prefix, base_cnt;
        unsigned long long base_sum;
        bool degenerate;
        radix_descent<true>(mk, tau, 0u, sh, prefix, base_cnt, base_sum, degenerate);
        if (tid == 0) {
            int kk = 1;
            if (!degenerate) {
                const unsigned long long qv = fixed40_of_key(prefix);
                const unsigned long long need = sh.target - base_sum;           // >= 1
                kk = (int)(base_cnt + (qv ? (need + qv - 1) / qv : 1ull));
            }
            sh.k = max(1, min(kk, n));
        }
        __syncthreads();
        k = sh.k;
    }
    if (tid == 0) k_out[u] = k;
    if (k >= n) {
        for (int j = tid; j < n; j += kSelThreads) idx[j] = j;
        return;
    }
    __syncthreads();

    // ---- which (Eq. (9)): k-th largest normalised score v*, ties to the lower index ----
    Keys rk{keys_in_lds ? lds_keys : nullptr, rank, n};
    if (second_vector) {
#pragma unroll
        for (int q = 0; q < kSelPre; ++q) {
            const int j = tid + q * kSelThreads;
            if (j < n) lds_keys[j] = orderable(pre[q]);
        }
        __syncthreads();
    }
    uint32_t vstar, cnt_gt;
    {
        unsigned long long unused;
        bool dg;
        radix_descent<false>(rk, tau, (uint32_t)k, sh, vstar, cnt_gt, unused, dg);
    }
    const uint32_t need_eq = (uint32_t)k - cnt_gt;     // ties at v* that are kept (>= 1)

    // ---- ascending emission, one block of positions (as many as LDS holds) at a time ----
    uint32_t gt_run = 0, eq_run = 0;                   // elements above / at v* in the blocks before
    for (int b0 = 0; b0 < n; b0 += kSelMaxLdsKeys) {
        const int bn = min(kSelMaxLdsKeys, n - b0);
        if (!keys_in_lds) {
            __syncthreads();
            fill_keys(lds_keys, rank + b0, bn);
            __syncthreads();
        }
        // thread t classifies positions [32 t, 32 t + 32) of the block; the rotation by the lane
        // spreads the 64 reads of a wave over the banks
        const int base = tid * 32;
        uint32_t gm = 0, em = 0;
        if (base < bn) {
            // all 32 reads are issued at once (index clamped, the mask bit predicated instead)
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
        for (int w2 = 0; w2 < kSelWaves; ++w2) {
            const uint32_t wg = sh.wave_cnt[w2], we = sh.wave_eq[w2];
            if (w2 < wave) { gt_before += wg; eq_before += we; }
            tot_g += wg; tot_e += we;
        }
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
}

// ---------------------------------------------------------------- two kernels: parallel first digit, then one workgroup per unit
// First-digit histograms of a slice of positions, built in LDS and added to the unit's tables.
__global__ __launch_bounds__(256) void select_hist_kernel(
    const float* __restrict__ mass_all, const float* __restrict__ rank_all, int n, int slice,
    unsigned long long* __restrict__ hm_all, uint32_t* __restrict__ hr_all)
{
    __shared__ unsigned long long lm[kSelBins];
    __shared__ uint32_t lr[kSelBins];
    const int u = blockIdx.y, tid = threadIdx.x;
    const int j0 = blockIdx.x * slice, j1 = min(n, j0 + slice);
    if (j0 >= j1) return;
    for (int b = tid; b < kSelBins; b += 256) { lm[b] = 0ull; lr[b] = 0u; }
    __syncthreads();
    const float* mass = mass_all + (int64_t)u * n;
    const float* rank = rank_all ? rank_all + (int64_t)u * n : nullptr;
    for (int j = j0 + tid; j < j1; j += 256) {
        const uint32_t key = orderable(mass[j]);
        atomicAdd(&lm[key >> kSelBinShift], (1ull << kSumBits) + fixed40_of_key(key));
        if (rank) atomicAdd(&lr[orderable(rank[j]) >> kSelBinShift], 1u);
    }
    __syncthreads();
    flush_tables<256>(lm, lr, hm_all + (int64_t)u * kSelBins, rank ? hr_all + (int64_t)u * kSelBins : nullptr);
}

// The rest of the selection of one unit; leaves the unit's tables zero for the next call.
__global__ __launch_bounds__(kSelThreads) void select_tail_kernel(
    const float* __restrict__ mass_all, const float* __restrict__ rank_all, int n, double tau,
    unsigned long long* __restrict__ hm_all, uint32_t* __restrict__ hr_all,
    int32_t* __restrict__ idx_all, int32_t* __restrict__ k_out, int key_cap, int32_t* __restrict__ status)
{
    __shared__ TailShared sh;
    extern __shared__ uint32_t lds_keys[];
    const int u = blockIdx.x;
    const float* mass = mass_all + (int64_t)u * n;
    if (status) {
        const uint32_t f = input_flags<kSelThreads>(mass, rank_all ? rank_all + (int64_t)u * n : mass, n, &sh.base_sum, &sh.sel_cnt);
        if (threadIdx.x == 0) status[u] = (int32_t)f;
        __syncthreads();
    }
    unsigned long long* hm = hm_all + (int64_t)u * kSelBins;
    uint32_t* hr = hr_all + (int64_t)u * kSelBins;
    select_tail<kSelThreads, false>(mass, rank_all ? rank_all + (int64_t)u * n : mass, n, tau, hm, rank_all ? hr : nullptr,
                                    idx_all + (int64_t)u * n, k_out + u, lds_keys, key_cap, sh);
    __syncthreads();
    for (int b = threadIdx.x; b < kSelBins; b += kSelThreads) { hm[b] = 0ull; hr[b] = 0u; }
}

size_t select_workspace_bytes(int units) {
    return (size_t)units * kSelBins * (sizeof(unsigned long long) + sizeof(uint32_t));
}

int launch_select(const float* mass, const float* rank, int units, int n, double tau,
                  int32_t* idx, int32_t* k, int32_t* status, void* ws, size_t ws_bytes, hipStream_t st)
{
    static std::atomic<bool> attr_done{false};
    if (!attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(&select_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                kSelMaxLdsKeys * (int)sizeof(uint32_t)) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void*>(&select_tail_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                kSelMaxLdsKeys * (int)sizeof(uint32_t)) != hipSuccess)
            return set_error(ZIPVL_EHIP, "select: cannot reserve LDS for the keys");
        attr_done = true;
    }
    const int in_lds = n <= kSelMaxLdsKeys ? 1 : 0;
    if (ws && ws_bytes >= select_workspace_bytes(units) && tau < 1.0) {
        // two kernels: the first digit of both descents from every CU, then one workgroup per unit
        unsigned long long* hm = (unsigned long long*)ws;
        uint32_t* hr = (uint32_t*)(hm + (size_t)units * kSelBins);
        const int slices = std::max(1, std::min((n + 255) / 256, (512 + units - 1) / units));
        const int slice = ((n + slices - 1) / slices + 63) / 64 * 64;
        {
            KernelTimer tm(ZIPVL_K_SELECT_HIST, st);
            hipLaunchKernelGGL(select_hist_kernel, dim3((n + slice - 1) / slice, units), dim3(256), 0, st, mass, rank, n, slice, hm, hr);
        }
        int rc = check_launch("select_hist");
        if (rc) return rc;
        const int key_cap = in_lds ? (n + 31) / 32 * 32 : kSelMaxLdsKeys;
        KernelTimer tm(ZIPVL_K_SELECT, st);
        hipLaunchKernelGGL(select_tail_kernel, dim3(units), dim3(kSelThreads), (size_t)key_cap * sizeof(uint32_t), st,
                           mass, rank, n, tau, hm, hr, idx, k, key_cap, status);
        return check_launch("select_tail");
    }
    // the key area also stages the blocks of a longer vector for the emission
    const size_t dyn = (size_t)(in_lds ? n : kSelMaxLdsKeys) * sizeof(uint32_t);
    KernelTimer tm(ZIPVL_K_SELECT, st);
    hipLaunchKernelGGL(select_kernel, dim3(units), dim3(kSelThreads), dyn, st, mass, rank, n, tau, idx, k, in_lds, status);
    return check_launch("select");
}

// ---------------------------------------------------------------- shared selection
// One important set per batch element: the per-unit scores are averaged over the Hkv units, units
// added in ascending order in fp32 and the sum multiplied by fp32(1/Hkv), so that the result is a
// fixed function of the inputs (the selection that follows is decided by these bits).
__global__ __launch_bounds__(256) void share_scores_kernel(
    const float* __restrict__ mass, const float* __restrict__ rank, int Hkv, int n, float inv,
    float* __restrict__ mass_b, float* __restrict__ rank_b)
{
    const int b = blockIdx.y;
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= n) return;
    const float* mp = mass + (int64_t)b * Hkv * n + j;
    float a = mp[0];
    for (int g = 1; g < Hkv; ++g) a += mp[(int64_t)g * n];
    mass_b[(int64_t)b * n + j] = a * inv;
    if (rank) {
        const float* rp = rank + (int64_t)b * Hkv * n + j;
        float r = rp[0];
        for (int g = 1; g < Hkv; ++g) r += rp[(int64_t)g * n];
        rank_b[(int64_t)b * n + j] = r * inv;
    }
}

int launch_share_scores(const float* mass, const float* rank, int B, int Hkv, int n,
                        float* mass_b, float* rank_b, hipStream_t st)
{
    KernelTimer tm(ZIPVL_K_SHARE_SCORES, st);
    hipLaunchKernelGGL(share_scores_kernel, dim3((n + 255) / 256, B), dim3(256), 0, st,
        mass, rank, Hkv, n, (float)(1.0 / Hkv), mass_b, rank_b);
    return check_launch("share_scores");
}

}  // namespace zipvl
