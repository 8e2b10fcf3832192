// Probe-token importance scores (supplementary Eq. (A); Eq. (6), Eq. (8);
// Algorithm 1 steps 2-4).  The m x n probe attention matrix is never stored:
//   pass 1  row statistics: for each (head, probe row) the running maximum
//           and exp-sum of the masked, scaled logits over a slice of keys,
//           one partial per key slice;
//   pass 2  the logits are recomputed tile by tile, normalised with the merged
//           row statistics, summed down the probe rows and over the query
//           heads of the group, and written as mass / rank.
// Both passes take the logits on the matrix cores: a 32-key x 32-probe tile is
// one 32x32 MFMA accumulator, operands are read straight from global memory as
// 16-byte fragments (K rows are consumed whole by consecutive fragments).
// Pass 1 computes K Q^T (lane = probe column, so row statistics stay in the
// lane); pass 2 computes Q K^T (lane = key column, so column sums stay in the
// lane).  Same registers, operands swapped.
#include "launch.h"

namespace zipvl {

constexpr int kNB = ZIPVL_MAX_PROBES / 32;   // probe blocks of 32 (rows beyond m are masked out)
constexpr int kMaxSplit = 32;
constexpr int kMaxGroup = 16;

template <typename T, int D>
struct ScoreCfg {
    static constexpr int CH = D / Elem<T>::kPerChunk;      // fragments per row per lane
};

template <typename T, int D>
__device__ __forceinline__ void load_row_frags(const T* row, int h, uintx4 (&f)[ScoreCfg<T, D>::CH]) {
#pragma unroll
    for (int c = 0; c < ScoreCfg<T, D>::CH; ++c)
        f[c] = load16(row + c * Elem<T>::kPerChunk + h * Elem<T>::kPerFrag);
}

// ---------------------------------------------------------------- pass 1
template <typename T, int D>
__global__ __launch_bounds__(256) void score_rowstats_kernel(
    const T* __restrict__ Q, const T* __restrict__ K,
    int64_t qs0, int64_t qs1, int64_t qs2, int64_t ks0, int64_t ks1, int64_t ks2,
    ProbeList probes, int m, int n, int n_eff, float c, float2* __restrict__ partial,
    int nsplit, int keys_per_split, int Hq, int Hkv)
{
    constexpr int CH = ScoreCfg<T, D>::CH;
    __shared__ float2 wave_stats[4][kNB * 32];
    const int split = blockIdx.x;
    const int bh = blockIdx.y, b = bh / Hq, head = bh - b * Hq, g = head / (Hq / Hkv);
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, i = lane & 31, h = lane >> 5;

    uintx4 qf[kNB][CH];
    int Pm[kNB];
#pragma unroll
    for (int nb = 0; nb < kNB; ++nb) {
        const int pc = nb * 32 + i;
        const int P = probes.pos[min(pc, m - 1)];
        Pm[nb] = pc < m ? P : -1;
        load_row_frags<T, D>(Q + b * qs0 + head * qs1 + (int64_t)P * qs2, h, qf[nb]);
    }
    float m_run[kNB], l_run[kNB];
#pragma unroll
    for (int nb = 0; nb < kNB; ++nb) { m_run[nb] = -INFINITY; l_run[nb] = 0.f; }

    const T* Kb = K + b * ks0 + g * ks1;
    const int j_begin = split * keys_per_split;
    const int j_end = min(n_eff, j_begin + keys_per_split);
    for (int jb = j_begin + w * 32; jb < j_end; jb += 128) {
        uintx4 kf[CH];
        load_row_frags<T, D>(Kb + (int64_t)min(jb + i, n - 1) * ks2, h, kf);
#pragma unroll
        for (int nb = 0; nb < kNB; ++nb) {
            floatx16 acc = {0};
#pragma unroll
            for (int cc = 0; cc < CH; ++cc) acc = mma_frag<T>(kf[cc], qf[nb][cc], acc);
            // acc[r]: key jb + acc_row(r, h), probe column nb*32 + i
            float s[16], mx = -INFINITY;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = jb + acc_row(r, h);
                s[r] = key > Pm[nb] ? -INFINITY : acc[r] * c;
                mx = fmaxf(mx, s[r]);
            }
            const float m_new = fmaxf(m_run[nb], mx);
            if (m_new > -INFINITY) {
                float sum = 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) sum += fast_exp2(s[r] - m_new);
                l_run[nb] = l_run[nb] * fast_exp2(m_run[nb] - m_new) + sum;
                m_run[nb] = m_new;
            }
        }
    }
    // merge the two lanes that share a probe column, then the four waves
#pragma unroll
    for (int nb = 0; nb < kNB; ++nb) {
        const float m2 = __shfl_xor(m_run[nb], 32), l2 = __shfl_xor(l_run[nb], 32);
        const float M = fmaxf(m_run[nb], m2);
        float L = 0.f;
        if (M > -INFINITY) L = l_run[nb] * fast_exp2(m_run[nb] - M) + l2 * fast_exp2(m2 - M);
        if (h == 0) wave_stats[w][nb * 32 + i] = make_float2(M, L);
    }
    __syncthreads();
    if (tid < kNB * 32) {
        float M = -INFINITY;
#pragma unroll
        for (int ww = 0; ww < 4; ++ww) M = fmaxf(M, wave_stats[ww][tid].x);
        float L = 0.f;
        if (M > -INFINITY) {
#pragma unroll
            for (int ww = 0; ww < 4; ++ww) L += wave_stats[ww][tid].y * fast_exp2(wave_stats[ww][tid].x - M);
        }
        partial[((int64_t)bh * nsplit + split) * (kNB * 32) + tid] = make_float2(M, L);
    }
}

// ---------------------------------------------------------------- pass 2
template <typename T, int D, int KB>
__global__ __launch_bounds__(256) void score_colsum_kernel(
    const T* __restrict__ Q, const T* __restrict__ K,
    int64_t qs0, int64_t qs1, int64_t qs2, int64_t ks0, int64_t ks1, int64_t ks2,
    ProbeList probes, int m, int n, int n_eff, float c, const float2* __restrict__ partial,
    int nsplit, float* __restrict__ mass, float* __restrict__ rank, int Hq, int Hkv)
{
    constexpr int CH = ScoreCfg<T, D>::CH;
    __shared__ int sp[kNB * 32];
    __shared__ float row_bias[kMaxGroup][kNB * 32];    // log2 of the row's softmax denominator
    const int G = Hq / Hkv;
    const int u = blockIdx.y, b = u / Hkv, g = u - b * Hkv;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, i = lane & 31, h = lane >> 5;
    const int block_begin = blockIdx.x * (128 * KB);

    if (block_begin >= n_eff) {          // no probe row sees these keys
        for (int j = block_begin + tid; j < min(n, block_begin + 128 * KB); j += 256) {
            mass[(int64_t)u * n + j] = 0.f;
            if (rank) rank[(int64_t)u * n + j] = 0.f;
        }
        return;
    }
    if (tid < kNB * 32) sp[tid] = tid < m ? probes.pos[tid] : -1;
    for (int t = tid; t < G * kNB * 32; t += 256) {
        const int hh = t / (kNB * 32), pc = t - hh * (kNB * 32);
        const float2* p = partial + ((int64_t)(b * Hq + g * G + hh) * nsplit) * (kNB * 32) + pc;
        float M = -INFINITY;
        for (int s = 0; s < nsplit; ++s) M = fmaxf(M, p[(int64_t)s * (kNB * 32)].x);
        float L = 0.f;
        if (M > -INFINITY)
            for (int s = 0; s < nsplit; ++s) {
                const float2 v = p[(int64_t)s * (kNB * 32)];
                L += v.y * fast_exp2(v.x - M);
            }
        row_bias[hh][pc] = (pc < m && L > 0.f) ? M + __log2f(L) : INFINITY;
    }
    __syncthreads();
    const int Pmin = sp[0];

    float colsum[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) colsum[kb] = 0.f;

    const T* Kb = K + b * ks0 + g * ks1;
    for (int hh = 0; hh < G; ++hh) {
        const int head = g * G + hh;
        uintx4 qf[kNB][CH];
        float rb[kNB][16];
#pragma unroll
        for (int nb = 0; nb < kNB; ++nb) {
            const int P = sp[min(nb * 32 + i, m - 1)];
            load_row_frags<T, D>(Q + b * qs0 + head * qs1 + (int64_t)P * qs2, h, qf[nb]);
#pragma unroll
            for (int r = 0; r < 16; ++r) rb[nb][r] = row_bias[hh][nb * 32 + acc_row(r, h)];
        }
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            const int jb = block_begin + (w * KB + kb) * 32;
            if (jb >= n_eff) continue;
            const int j = jb + i;                       // this lane's key column
            uintx4 kf[CH];
            load_row_frags<T, D>(Kb + (int64_t)min(j, n - 1) * ks2, h, kf);
            const bool masked = jb + 31 > Pmin;
            float sum = 0.f;
#pragma unroll
            for (int nb = 0; nb < kNB; ++nb) {
                floatx16 acc = {0};
#pragma unroll
                for (int cc = 0; cc < CH; ++cc) acc = mma_frag<T>(qf[nb][cc], kf[cc], acc);
                // acc[r]: probe row nb*32 + acc_row(r, h), key column j
                if (masked) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float p = fast_exp2(acc[r] * c - rb[nb][r]);
                        sum += j > sp[nb * 32 + acc_row(r, h)] ? 0.f : p;
                    }
                } else {
#pragma unroll
                    for (int r = 0; r < 16; ++r) sum += fast_exp2(acc[r] * c - rb[nb][r]);
                }
            }
            colsum[kb] += sum;
        }
    }
    const float inv_g = 1.f / (float)G;
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
        const int jb = block_begin + (w * KB + kb) * 32;
        const float a = (colsum[kb] + __shfl_xor(colsum[kb], 32)) * inv_g;
        const int j = jb + i;
        if (h == 0 && j < n) {
            int cnt = 0;
            for (int t = 0; t < m; ++t) cnt += sp[t] >= j ? 1 : 0;
            mass[(int64_t)u * n + j] = a / (float)m;
            if (rank) rank[(int64_t)u * n + j] = cnt > 0 ? a / (float)cnt : 0.f;
        }
    }
}

// ---------------------------------------------------------------- host side
struct ScorePlan { int n_eff, nsplit, keys_per_split, KB; };

static ScorePlan plan_score(const zipvl_dims& d, const int32_t* probe_pos, int m) {
    ScorePlan p;
    p.n_eff = probe_pos ? probe_pos[m - 1] + 1 : d.n;
    const int heads = d.B * d.Hq;
    int want = (1024 + heads - 1) / heads;
    want = want < 1 ? 1 : (want > kMaxSplit ? kMaxSplit : want);
    int per = (p.n_eff + want - 1) / want;
    per = ((per + 127) / 128) * 128;
    p.keys_per_split = per;
    p.nsplit = (p.n_eff + per - 1) / per;
    const int units = d.B * d.Hkv;
    p.KB = 1;
    for (int kb = 4; kb >= 1; kb >>= 1)
        if ((int64_t)((d.n + 128 * kb - 1) / (128 * kb)) * units >= 512) { p.KB = kb; break; }
    return p;
}

size_t score_workspace_bytes(const zipvl_dims& d, int m) {
    (void)m;
    return (size_t)d.B * d.Hq * kMaxSplit * (kNB * 32) * sizeof(float2);
}

template <typename T, int D>
static int launch_score_t(const void* Q, const void* K, const zipvl_dims& d, const ProbeList& pl, int m,
                          const ScorePlan& p, float scale, float* mass, float* rank, void* ws, hipStream_t st)
{
    const float c = scale * kLog2e;
    float2* partial = (float2*)ws;
    {
        KernelTimer tm(ZIPVL_K_SCORE_ROWSTATS, st);
        hipLaunchKernelGGL((score_rowstats_kernel<T, D>), dim3(p.nsplit, d.B * d.Hq), dim3(256), 0, st,
            (const T*)Q, (const T*)K, d.q_strides[0], d.q_strides[1], d.q_strides[2],
            d.k_strides[0], d.k_strides[1], d.k_strides[2], pl, m, d.n, p.n_eff, c, partial,
            p.nsplit, p.keys_per_split, d.Hq, d.Hkv);
    }
    int rc = check_launch("score_rowstats");
    if (rc) return rc;
#define ZIPVL_COLSUM(KBV)                                                                          \
    hipLaunchKernelGGL((score_colsum_kernel<T, D, KBV>),                                           \
        dim3((d.n + 128 * KBV - 1) / (128 * KBV), d.B * d.Hkv), dim3(256), 0, st,                  \
        (const T*)Q, (const T*)K, d.q_strides[0], d.q_strides[1], d.q_strides[2],                  \
        d.k_strides[0], d.k_strides[1], d.k_strides[2], pl, m, d.n, p.n_eff, c,                    \
        (const float2*)partial, p.nsplit, mass, rank, d.Hq, d.Hkv)
    KernelTimer tm(ZIPVL_K_SCORE_COLSUM, st);
    if (p.KB == 4) ZIPVL_COLSUM(4);
    else if (p.KB == 2) ZIPVL_COLSUM(2);
    else ZIPVL_COLSUM(1);
#undef ZIPVL_COLSUM
    return check_launch("score_colsum");
}

int launch_score(const void* Q, const void* K, const zipvl_dims& d, const int32_t* probe_pos, int m,
                 float scale, float* mass, float* rank, void* ws, hipStream_t st)
{
    if (d.Hq / d.Hkv > kMaxGroup) return set_error(ZIPVL_ESHAPE, "score: Hq/Hkv = %d exceeds %d", d.Hq / d.Hkv, kMaxGroup);
    ProbeList pl;
    for (int t = 0; t < ZIPVL_MAX_PROBES; ++t) pl.pos[t] = t < m ? probe_pos[t] : -1;
    const ScorePlan p = plan_score(d, probe_pos, m);
    if (d.dtype == ZIPVL_BF16) {
        if (d.d == 128) return launch_score_t<__bf16, 128>(Q, K, d, pl, m, p, scale, mass, rank, ws, st);
        return launch_score_t<__bf16, 64>(Q, K, d, pl, m, p, scale, mass, rank, ws, st);
    }
    if (d.d == 128) return launch_score_t<float, 128>(Q, K, d, pl, m, p, scale, mass, rank, ws, st);
    return launch_score_t<float, 64>(Q, K, d, pl, m, p, scale, mass, rank, ws, st);
}

}  // namespace zipvl
