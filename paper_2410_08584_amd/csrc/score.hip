// Probe-token importance scores (supplementary Eq. (A); Eq. (6), Eq. (8);
// Algorithm 1 steps 2-4).  The m x n probe attention matrix is never stored:
//   pass 1  row statistics: for each (head, probe row) the maximum and the
//           exp-sum of the masked, scaled logits over a slice of 128 keys;
//           a small kernel merges the slices into one exponent offset per row;
//   pass 2  the logits are recomputed, normalised with that offset, summed
//           down the probe rows and over the query heads of the group, and
//           written as mass / rank.
// Both passes share one kernel body.  A workgroup (4 waves) owns 128 keys of
// one KV head: each wave keeps the fragments of its 32 keys in registers and
// walks over the group's query heads, whose probe rows pass through LDS a few
// heads at a time (small footprint, several workgroups per CU), so K is read
// from memory once per pass.  A 32-key x 32-probe tile is one 32x32 MFMA
// accumulator.  Pass 1 computes K Q^T (lane = probe column: row statistics
// stay in the lane); pass 2 computes Q K^T (lane = key column: column sums
// stay in the lane).  Same fragments, operands swapped.
#include <atomic>

#include "launch.h"

namespace zipvl {

// Probe rows are handled in blocks of 32 (NB = 2 for m <= 64, NB = 4 for m <= 128; rows beyond m are masked out).
constexpr int kMaxNB = ZIPVL_MAX_PROBES / 32;
constexpr int kMaxGroup = 16;
constexpr int kScoreWaves = 4;
constexpr int kScoreThreads = 64 * kScoreWaves;
constexpr int kScoreKeys = 32 * kScoreWaves;  // keys per workgroup

template <typename T, int D, int NB = 2>
struct ScoreCfg {
    static constexpr int kProbes = NB * 32;
    static constexpr int E = Elem<T>::kBytes;
    static constexpr int CH = D / Elem<T>::kPerChunk;      // fragments per row per lane
    static constexpr int QS = D * E + 16;                   // padded LDS row of a probe query (bytes)
    static constexpr int HEAD_BYTES = kProbes * QS;
    static constexpr int GC = (36 * 1024) / HEAD_BYTES > 0 ? (36 * 1024) / HEAD_BYTES : 1;   // heads staged in LDS at once
    static constexpr int CPR = D * E / 16;                  // 16-byte chunks per row
};

template <typename T, int D>
__device__ __forceinline__ void load_row_frags(const T* row, int h, uintx4 (&f)[ScoreCfg<T, D>::CH]) {
#pragma unroll
    for (int c = 0; c < ScoreCfg<T, D>::CH; ++c)
        f[c] = load16(row + c * Elem<T>::kPerChunk + h * Elem<T>::kPerFrag);
}

// PASS 1: partial[(bh * nsplit + split) * 64 + probe] = (raw-logit maximum, sum of exp2((s - max) * c))
// PASS 2: mass / rank of the workgroup's keys, from bias[bh * 64 + probe] = max * c + log2(sum)
// GCT = query heads whose probe rows are staged in LDS at once (1 when the group has a single head: fewer
// staging registers and a smaller LDS footprint, so more workgroups per CU hide the load latency)
// bf16: at least three workgroups per CU; the register budget that follows keeps the accumulators in architectural VGPRs,
// where the vector ALU reads them without copies.
template <typename T, int D, int PASS, int NB, int GCT>
__global__ __launch_bounds__(kScoreThreads, (Elem<T>::kBytes == 2 ? 3 : 1)) void score_pass_kernel(
    const T* __restrict__ Q, const T* __restrict__ K,
    int64_t qs0, int64_t qs1, int64_t qs2, int64_t ks0, int64_t ks1, int64_t ks2,
    ProbeList probes, int m, int n, int n_eff, float c, float2* __restrict__ partial, int nsplit,
    const float* __restrict__ bias, float* __restrict__ mass, float* __restrict__ rank, int Hq, int Hkv)
{
    using C = ScoreCfg<T, D, NB>;
    constexpr int CH = C::CH;
    constexpr int kProbes = NB * 32, kNB = NB;
    extern __shared__ __attribute__((aligned(16))) char smem[];     // [gc][64] padded probe rows
    __shared__ int sp[kProbes];
    __shared__ __attribute__((aligned(16))) float row_bias[kMaxGroup][kProbes];
    const int G = Hq / Hkv;
    const int u = blockIdx.y, b = u / Hkv, g = u - b * Hkv;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, i = lane & 31, h = lane >> 5;
    const int block_begin = blockIdx.x * kScoreKeys;

    if (PASS == 2 && block_begin >= n_eff) {          // no probe row sees these keys
        for (int j = block_begin + tid; j < min(n, block_begin + kScoreKeys); j += kScoreThreads) {
            mass[(int64_t)u * n + j] = 0.f;
            if (rank) rank[(int64_t)u * n + j] = 0.f;
        }
        return;
    }
    if (tid < kProbes) sp[tid] = probes.pos[tid];          // -1 beyond m
    if (PASS == 2)
        for (int t = tid; t < G * kProbes; t += kScoreThreads)
            (&row_bias[0][0])[t] = bias[(int64_t)(b * Hq + g * G) * kProbes + t];
    __syncthreads();
    const int Pmin = sp[0];
    const bool has_pad = m < kProbes;

    // this wave's 32 keys stay in registers for every head of the group
    const int jb = block_begin + w * 32;
    const bool live = jb < n_eff;                           // wave-uniform
    uintx4 kf[CH];
    load_row_frags<T, D>(K + b * ks0 + g * ks1 + (int64_t)min(jb + i, n - 1) * ks2, h, kf);
    const bool masked = has_pad || jb + 31 > Pmin;          // wave-uniform

    float colsum = 0.f;                                     // PASS 2
    float2* wstat = reinterpret_cast<float2*>(smem + GCT * C::HEAD_BYTES);   // PASS 1: [wave][head of chunk][nb][lane]

    // Probe rows travel global -> registers -> LDS one chunk of GC heads at a time; the next chunk
    // is requested before the current one is consumed, so its latency hides under the matrix work.
    constexpr int NPRE = GCT * kProbes * C::CPR / kScoreThreads;
    static_assert(NPRE * kScoreThreads == GCT * kProbes * C::CPR, "chunk must divide evenly over the threads");
    uintx4 pre[NPRE];
    // where this thread's NPRE chunks sit inside a chunk of heads: fixed for the whole kernel
    int pre_head[NPRE];
    int64_t pre_off[NPRE];
#pragma unroll
    for (int q = 0; q < NPRE; ++q) {
        const int t = tid + q * kScoreThreads;
        const int row = t / C::CPR, cc = t - row * C::CPR;
        pre_head[q] = row / kProbes;
        pre_off[q] = (int64_t)sp[min(row - pre_head[q] * kProbes, m - 1)] * qs2 + cc * Elem<T>::kPerFrag;
    }
    auto fetch_chunk = [&](int h0) {
        const T* base = Q + b * qs0 + (int64_t)(g * G + h0) * qs1;
        const int last = min(GCT, G - h0) - 1;               // heads beyond the chunk re-read its last head
#pragma unroll
        for (int q = 0; q < NPRE; ++q) pre[q] = load16(base + min(pre_head[q], last) * qs1 + pre_off[q]);
    };
    fetch_chunk(0);
    for (int h0 = 0; h0 < G; h0 += GCT) {
        const int gc = min(GCT, G - h0);
        if (h0) __syncthreads();                            // previous chunk fully consumed
#pragma unroll
        for (int q = 0; q < NPRE; ++q) {
            const int t = tid + q * kScoreThreads;
            const int row = t / C::CPR, cc = t - row * C::CPR;
            store16(smem + row * C::QS + cc * 16, pre[q]);  // rows beyond gc heads hold duplicates, never read
        }
        __syncthreads();
        if (h0 + GCT < G) fetch_chunk(h0 + GCT);
#pragma unroll 1
        for (int hh = 0; hh < gc; ++hh) {
            const char* qh = smem + hh * C::HEAD_BYTES;
#pragma unroll
            for (int nb = 0; nb < kNB; ++nb) {
                float2 stat = make_float2(-INFINITY, 0.f);
                if (live) {
                    uintx4 qf[CH];
#pragma unroll
                    for (int cc = 0; cc < CH; ++cc)
                        qf[cc] = *reinterpret_cast<const uintx4*>(qh + (nb * 32 + i) * C::QS + cc * 32 + h * 16);
                    floatx16 acc = {0};
                    if (PASS == 1) {
#pragma unroll
                        for (int cc = 0; cc < CH; ++cc) acc = mma_frag<T>(kf[cc], qf[cc], acc);
                        // acc[r]: key jb + acc_row(r, h), probe column nb*32 + i  (raw logit)
                        float sv[16], mx = -INFINITY;
#pragma unroll
                        for (int r = 0; r < 16; ++r) sv[r] = acc[r];
                        if (masked) {
                            const int Pm = sp[nb * 32 + i];
#pragma unroll
                            for (int r = 0; r < 16; ++r)
                                if (jb + acc_row(r, h) > Pm) sv[r] = -INFINITY;
                        }
#pragma unroll
                        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sv[r]);
                        float sum = 0.f;
                        if (mx > -INFINITY) {               // statistics of this lane's 16 keys only
                            const float mc = mx * c;
#pragma unroll
                            for (int r = 0; r < 16; ++r) sum += fast_exp2(fmaf(sv[r], c, -mc));
                        }
                        stat = make_float2(mx, sum);
                    } else {
#pragma unroll
                        for (int cc = 0; cc < CH; ++cc) acc = mma_frag<T>(qf[cc], kf[cc], acc);
                        // acc[r]: probe row nb*32 + acc_row(r, h), key column jb + i
                        float rb[16];
#pragma unroll
                        for (int a = 0; a < 4; ++a) {
                            const floatx4 v = *reinterpret_cast<const floatx4*>(&row_bias[h0 + hh][nb * 32 + 8 * a + 4 * h]);
                            rb[4 * a] = v[0]; rb[4 * a + 1] = v[1]; rb[4 * a + 2] = v[2]; rb[4 * a + 3] = v[3];
                        }
                        float sum = 0.f;
                        if (masked) {
#pragma unroll
                            for (int r = 0; r < 16; ++r) {
                                const float p = fast_exp2(fmaf(acc[r], c, -rb[r]));
                                sum += jb + i > sp[nb * 32 + acc_row(r, h)] ? 0.f : p;
                            }
                        } else {
#pragma unroll
                            for (int r = 0; r < 16; ++r) sum += fast_exp2(fmaf(acc[r], c, -rb[r]));
                        }
                        colsum += sum;
                    }
                }
                if (PASS == 1) wstat[((w * GCT + hh) * kNB + nb) * 64 + lane] = stat;
            }
        }
        if (PASS == 1) {
            // merge the 4 waves x 2 half-waves that saw each (head, probe row) and emit the slice partial
            __syncthreads();
            for (int t = tid; t < gc * kProbes; t += kScoreThreads) {
                const int hh = t / kProbes, pc = t - hh * kProbes, nb = pc >> 5, ii = pc & 31;
                float M = -INFINITY;
#pragma unroll
                for (int ww = 0; ww < kScoreWaves; ++ww)
#pragma unroll
                    for (int hf = 0; hf < 2; ++hf)
                        M = fmaxf(M, wstat[((ww * GCT + hh) * kNB + nb) * 64 + hf * 32 + ii].x);
                float L = 0.f;
                if (M > -INFINITY) {
#pragma unroll
                    for (int ww = 0; ww < kScoreWaves; ++ww)
#pragma unroll
                        for (int hf = 0; hf < 2; ++hf) {
                            const float2 v = wstat[((ww * GCT + hh) * kNB + nb) * 64 + hf * 32 + ii];
                            L += v.y * fast_exp2((v.x - M) * c);
                        }
                }
                partial[((int64_t)(b * Hq + g * G + h0 + hh) * nsplit + blockIdx.x) * kProbes + pc] = make_float2(M, L);
            }
        }
    }

    if (PASS == 2) {
        const float a = (colsum + __shfl_xor(colsum, 32)) / (float)G;
        const int j = jb + i;
        if (h == 0 && j < n) {
            int cnt = 0;
            if (j <= Pmin) cnt = m;
            else for (int t = 0; t < m; ++t) cnt += sp[t] >= j ? 1 : 0;
            mass[(int64_t)u * n + j] = a / (float)m;
            if (rank) rank[(int64_t)u * n + j] = cnt > 0 ? a / (float)cnt : 0.f;
        }
    }
}

// Merge the per-slice statistics of every (head, probe row) into one exponent offset
// bias = max * c + log2(sum), so that exp2(s * c - bias) is the normalised probability.
// Block = np probe rows x 8 slice groups.
__global__ __launch_bounds__(1024) void score_rowfinal_kernel(
    const float2* __restrict__ partial, int nsplit, int m, int np, float c, float* __restrict__ bias)
{
    __shared__ float2 red[8][ZIPVL_MAX_PROBES];
    const int bh = blockIdx.x, pc = threadIdx.x % np, sg = threadIdx.x / np;
    const float2* p = partial + (int64_t)bh * nsplit * np + pc;
    float M = -INFINITY, L = 0.f;
    for (int s0 = sg; s0 < nsplit; s0 += 32) {              // 4 independent loads per round
        float2 v[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int s = s0 + 8 * q;
            v[q] = s < nsplit ? p[(int64_t)s * np] : make_float2(-INFINITY, 0.f);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float Mn = fmaxf(M, v[q].x);
            if (Mn > -INFINITY) L = L * fast_exp2((M - Mn) * c) + v[q].y * fast_exp2((v[q].x - Mn) * c);
            M = Mn;
        }
    }
    red[sg][pc] = make_float2(M, L);
    __syncthreads();
    if (sg == 0) {
        float Mt = -INFINITY;
#pragma unroll
        for (int q = 0; q < 8; ++q) Mt = fmaxf(Mt, red[q][pc].x);
        float Lt = 0.f;
        if (Mt > -INFINITY) {
#pragma unroll
            for (int q = 0; q < 8; ++q) Lt += red[q][pc].y * fast_exp2((red[q][pc].x - Mt) * c);
        }
        bias[(int64_t)bh * np + pc] = (pc < m && Lt > 0.f) ? Mt * c + __log2f(Lt) : INFINITY;
    }
}

// ---------------------------------------------------------------- host side
static int score_splits(const zipvl_dims& d) { return (d.n + kScoreKeys - 1) / kScoreKeys; }
static int probe_rows(int m) { return m <= 64 ? 64 : 128; }

static size_t score_partial_bytes(const zipvl_dims& d, int m) {
    return (size_t)d.B * d.Hq * score_splits(d) * probe_rows(m) * sizeof(float2);
}

size_t score_workspace_bytes(const zipvl_dims& d, int m) {
    return score_partial_bytes(d, m) + (size_t)d.B * d.Hq * probe_rows(m) * sizeof(float);
}

template <typename T, int D, int NB, int GCT>
static int launch_score_g(const void* Q, const void* K, const zipvl_dims& d, const ProbeList& pl, int m,
                          int n_eff, float scale, float* mass, float* rank, void* ws, hipStream_t st)
{
    using C = ScoreCfg<T, D, NB>;
    const float c = scale * kLog2e;
    float2* partial = (float2*)ws;
    float* bias = (float*)((char*)ws + score_partial_bytes(d, m));
    const int units = d.B * d.Hkv;
    // probe rows of GC heads, then the per-wave statistics of pass 1
    const size_t lds = (size_t)GCT * C::HEAD_BYTES + (size_t)kScoreWaves * GCT * NB * 64 * sizeof(float2);
    static std::atomic<bool> attr_done{false};
    if (!attr_done) {
        const int cap = 96 * 1024;
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(&score_pass_kernel<T, D, 1, NB, GCT>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, cap) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void*>(&score_pass_kernel<T, D, 2, NB, GCT>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, cap) != hipSuccess)
            return set_error(ZIPVL_EHIP, "score: cannot reserve LDS for the probe rows");
        attr_done = true;
    }
    const int nsplit = (n_eff + kScoreKeys - 1) / kScoreKeys;
    {
        KernelTimer tm(ZIPVL_K_SCORE_ROWSTATS, st);
        hipLaunchKernelGGL((score_pass_kernel<T, D, 1, NB, GCT>), dim3(nsplit, units), dim3(kScoreThreads), lds, st,
            (const T*)Q, (const T*)K, d.q_strides[0], d.q_strides[1], d.q_strides[2],
            d.k_strides[0], d.k_strides[1], d.k_strides[2], pl, m, d.n, n_eff, c, partial, nsplit,
            (const float*)nullptr, (float*)nullptr, (float*)nullptr, d.Hq, d.Hkv);
    }
    int rc = check_launch("score_rowstats");
    if (rc) return rc;
    {
        KernelTimer tm(ZIPVL_K_SCORE_ROWFINAL, st);
        hipLaunchKernelGGL(score_rowfinal_kernel, dim3(d.B * d.Hq), dim3(NB * 32 * 8), 0, st,
            (const float2*)partial, nsplit, m, NB * 32, c, bias);
    }
    rc = check_launch("score_rowfinal");
    if (rc) return rc;
    KernelTimer tm(ZIPVL_K_SCORE_COLSUM, st);
    hipLaunchKernelGGL((score_pass_kernel<T, D, 2, NB, GCT>), dim3(score_splits(d), units), dim3(kScoreThreads), lds, st,
        (const T*)Q, (const T*)K, d.q_strides[0], d.q_strides[1], d.q_strides[2],
        d.k_strides[0], d.k_strides[1], d.k_strides[2], pl, m, d.n, n_eff, c, (float2*)nullptr, nsplit,
        (const float*)bias, mass, rank, d.Hq, d.Hkv);
    return check_launch("score_colsum");
}

template <typename T, int D, int NB>
static int launch_score_t(const void* Q, const void* K, const zipvl_dims& d, const ProbeList& pl, int m,
                          int n_eff, float scale, float* mass, float* rank, void* ws, hipStream_t st)
{
    constexpr int GC = ScoreCfg<T, D, NB>::GC;
    if constexpr (GC > 1) {
        if (d.Hq == d.Hkv) return launch_score_g<T, D, NB, 1>(Q, K, d, pl, m, n_eff, scale, mass, rank, ws, st);
    }
    return launch_score_g<T, D, NB, GC>(Q, K, d, pl, m, n_eff, scale, mass, rank, ws, st);
}

template <typename T, int D>
static int launch_score_nb(const void* Q, const void* K, const zipvl_dims& d, const ProbeList& pl, int m,
                           int n_eff, float scale, float* mass, float* rank, void* ws, hipStream_t st)
{
    if (m <= 64) return launch_score_t<T, D, 2>(Q, K, d, pl, m, n_eff, scale, mass, rank, ws, st);
    return launch_score_t<T, D, 4>(Q, K, d, pl, m, n_eff, scale, mass, rank, ws, st);
}

int launch_score(const void* Q, const void* K, const zipvl_dims& d, const int32_t* probe_pos, int m,
                 float scale, float* mass, float* rank, void* ws, hipStream_t st)
{
    if (d.Hq / d.Hkv > kMaxGroup) return set_error(ZIPVL_ESHAPE, "score: Hq/Hkv = %d exceeds %d", d.Hq / d.Hkv, kMaxGroup);
    ProbeList pl;
    for (int t = 0; t < ZIPVL_MAX_PROBES; ++t) pl.pos[t] = t < m ? probe_pos[t] : -1;
    const int n_eff = probe_pos[m - 1] + 1;
    if (d.dtype == ZIPVL_BF16) {
        if (d.d == 128) return launch_score_nb<__bf16, 128>(Q, K, d, pl, m, n_eff, scale, mass, rank, ws, st);
        return launch_score_nb<__bf16, 64>(Q, K, d, pl, m, n_eff, scale, mass, rank, ws, st);
    }
    if (d.d == 128) return launch_score_nb<float, 128>(Q, K, d, pl, m, n_eff, scale, mass, rank, ws, st);
    return launch_score_nb<float, 64>(Q, K, d, pl, m, n_eff, scale, mass, rank, ws, st);
}

}  // namespace zipvl
