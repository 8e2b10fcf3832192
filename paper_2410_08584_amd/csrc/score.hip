// Probe-token importance scores (supplementary Eq. (A); Eq. (6), Eq. (8);
// Algorithm 1 steps 2-4).  The m x n probe attention matrix is never stored:
//   pass 1  row statistics: for each (head, probe row) the maximum and the
//           exp-sum of the masked, scaled logits over the chunk of keys a
//           workgroup owns (one partial pair per row and chunk);
//   pass 2  merges the partial pairs of its rows into one exponent offset per
//           row (in its prologue: no launch in between), recomputes the
//           logits, normalises them with that offset, sums them down the probe
//           rows and over the query heads of the group, and writes mass / rank.
// Both passes share one kernel body.  A workgroup owns a chunk of keys of one
// KV head and streams it through LDS in stages of 32 KiB, loaded straight from
// global memory (no staging registers), double buffered.  The work of a stage
// is a grid of 32-key x 32-probe tiles, one 32x32 MFMA accumulator each.  A
// wave owns one (query head, block of 32 probe rows) - its "task" - for the
// whole kernel: the probe rows' fragments stay in its registers, and the key
// fragments of a tile come from LDS.  With few tasks (one query head per KV
// head) several waves share a task and split the key blocks of a stage; with
// more tasks than waves the chunk is streamed once per round of tasks.
// Pass 1 computes K Q^T (lane = probe column: row statistics stay in the
// lane); pass 2 computes Q K^T (lane = key column: column sums stay in the
// lane, the tasks' sums of a stage meet in LDS and are added in task order, so
// the result does not depend on scheduling).
#include <algorithm>
#include <atomic>

#include "launch.h"
#include "ldsload.h"

namespace zipvl {

constexpr int kMaxGroup = 16;
constexpr int kStageBufs = 4;               // stage buffers in LDS: three stages are in flight while one is worked on

// NWV waves per workgroup.  16 waves (one workgroup per CU): stages of 32 KiB; 8 waves (two per CU): 16 KiB;
// never more than 128 keys (the column-sum buffers grow with the keys of a stage).
template <typename T, int D, int NWV>
struct ScoreCfg {
    static constexpr int E = Elem<T>::kBytes;
    static constexpr int CH = D / Elem<T>::kPerChunk;      // fragments per row per lane
    static constexpr int RB = D * E;                        // bytes per key row
    static constexpr int STG = NWV * 2048 < 128 * RB ? NWV * 2048 : 128 * RB;   // bytes per stage: two 1-KiB loads per wave, 128 keys at most
    static constexpr int SK = STG / RB;                     // keys per stage
    static constexpr int KBS = SK / 32;                     // 32-key blocks per stage
    static constexpr int NLD = STG / 1024 / NWV;            // 1-KiB loads per wave per stage
};

// The statistics (maximum m, exp-sum l relative to m, log2 domain scale c) of two disjoint key sets of one row.
__device__ __forceinline__ void merge_stats(float& m, float& l, float m2, float l2, float c) {
    const float M = fmaxf(m, m2);
    if (M > -INFINITY) l = l * fast_exp2((m - M) * c) + l2 * fast_exp2((m2 - M) * c);
    m = M;
}

// PASS 1: partial[((b*Hq + head) * nsplit + chunk) * np + probe] = (raw-logit maximum, sum of exp2((s - max) * c))
// PASS 2: mass / rank of the workgroup's keys; nsplit = chunks of pass 1
// np = probe rows rounded up to a multiple of 32 (NB blocks); rows beyond m are masked out.
// bpc = 32-key blocks per chunk of this pass.
template <typename T, int D, int PASS, int NWV>
__global__ __launch_bounds__(64 * NWV, (Elem<T>::kBytes == 4 && D == 128 && NWV == 8) ? 2 : 4) void score_kernel(
    const T* __restrict__ Q, const T* __restrict__ K,
    int64_t qs0, int64_t qs1, int64_t qs2, int64_t ks0, int64_t ks1, int64_t ks2,
    ProbeList probes, int m, int NB, int n, int n_eff, float c, float2* __restrict__ partial, int nsplit, int bpc,
    float* __restrict__ mass, float* __restrict__ rank, int Hq, int Hkv, int kv_div)
{
    using C = ScoreCfg<T, D, NWV>;
    constexpr int CH = C::CH, RB = C::RB, SK = C::SK, KBS = C::KBS, NLD = C::NLD, kStageBytes = C::STG;
    constexpr int kThreads = 64 * NWV;
    extern __shared__ __attribute__((aligned(16))) char kstage[];   // kStageBufs stage buffers
    __shared__ int sp[ZIPVL_MAX_PROBES];
    __shared__ float2 wstat[PASS == 1 ? NWV : 1][32];                // pass 1: per-wave row statistics
    __shared__ __attribute__((aligned(16))) float row_bias[PASS == 2 ? NWV : 1][32];
    __shared__ float colbuf[PASS == 2 ? 2 : 1][PASS == 2 ? NWV : 1][PASS == 2 ? SK : 1];

    const int G = Hq / Hkv, np = NB * 32, NT = G * NB;
    const int u = blockIdx.y, b = u / Hkv, g = u - b * Hkv;
    const int tid = threadIdx.x, lane = tid & 63, i = lane & 31, h = lane >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);          // wave-uniform: everything derived from it lives in scalar registers
    const int nblk = ((PASS == 1 ? n_eff : n) + 31) >> 5;
    const int blk0 = blockIdx.x * bpc, blk1 = min(blk0 + bpc, nblk);
    if (blk0 >= blk1) return;
    const int S = (blk1 - blk0 + KBS - 1) / KBS;                     // stages of this chunk

    if (tid < ZIPVL_MAX_PROBES) sp[tid] = probes.pos[tid];           // -1 beyond m
    __syncthreads();
    const int Pmin = sp[0];
    const bool has_pad = m < np;

    // waves -> tasks.  Fewer tasks than waves: KS waves share a task and take the key blocks slot, slot + KS, ...
    const bool few = NT < NWV;
    const int KS = few ? NWV / NT : 1;
    const int rounds = few ? 1 : (NT + NWV - 1) / NWV;
    const int ts = few ? w % NT : w;                                 // task slot inside a round
    const int slot = few ? w / NT : 0;

    // where this lane's NLD 16-byte pieces of a stage come from: row inside the stage and chunk under the row swizzle
    const char* Ku = reinterpret_cast<const char*>(K + b * ks0 + (g / kv_div) * ks1);   // kv_div > 1: every query head is its own unit
    const int row_stride = (int)ks2 * C::E;                          // bytes; a stage spans less than 2 GiB (checked on the host)
    const unsigned lds0 = lds_address(kstage);
    // where this lane's NLD 16-byte pieces of a stage come from: byte offset of (row inside the stage, chunk under the row swizzle)
    int ld_off[NLD];
#pragma unroll
    for (int q = 0; q < NLD; ++q) {
        const int o = (q * NWV + w) * 1024 + lane * 16;              // LDS byte of the piece: row r, position p of the row
        const int r = o / RB, p = (o % RB) >> 4;
        ld_off[q] = r * row_stride + ((p ^ k_row_swizzle<RB>(r)) << 4);
    }
    // Every wave issues exactly NLD loads per stage (pieces past the chunk's or the sequence's last row re-read
    // the stage's first row and are never used), so that "all but the newest p stages have landed" is a count.
    auto issue_stage = [&](int s) {
        const int row0 = (blk0 + s * KBS) * 32;
        const int rows = min(min(blk1 * 32, n) - row0, SK);           // rows of this stage that exist and belong to the chunk
        const char* gbase = Ku + (int64_t)row0 * row_stride;
        const unsigned dst = lds0 + (s % kStageBufs) * kStageBytes;
#pragma unroll
        for (int q = 0; q < NLD; ++q) {
            const int r = ((q * NWV + w) * 1024 + lane * 16) / RB;
            load_kib_to_lds(gbase, r < rows ? ld_off[q] : 0, dst + (q * NWV + w) * 1024);
        }
    };
    // wait until at most `pending` stages (NLD loads each) of this wave are still on their way
    auto wait_stages = [&](int pending) {
        if (pending >= 2) __builtin_amdgcn_s_waitcnt(0x0F70 | (2 * NLD));
        else if (pending == 1) __builtin_amdgcn_s_waitcnt(0x0F70 | NLD);
        else __builtin_amdgcn_s_waitcnt(0x0F70);
    };
    static_assert(2 * NLD < 16, "vmcnt immediate");

#pragma unroll 1
    for (int rd = 0; rd < rounds; ++rd) {
        const int task = rd * NWV + ts;
        const bool active = few ? w < NT * KS : task < NT;
        const int ntr = few ? NT : min(NWV, NT - rd * NWV);          // tasks of this round
        const int head = active ? task / NB : 0, nb = active ? task - (task / NB) * NB : 0;
        const int bh = b * Hq + g * G + head;

        if (rd) __syncthreads();                                     // the stage buffers of the previous round are free
#pragma unroll
        for (int s = 0; s < kStageBufs - 1; ++s)
            if (s < S) issue_stage(s);

        // this wave's probe rows: fragments of row nb*32 + i, held for the whole round
        uintx4 qf[CH];
        {
            const int prow = sp[min(nb * 32 + i, m - 1)];
            const T* qp = Q + b * qs0 + (int64_t)(g * G + head) * qs1 + (int64_t)prow * qs2 + h * Elem<T>::kPerFrag;
#pragma unroll
            for (int cc = 0; cc < CH; ++cc) qf[cc] = load16(qp + cc * Elem<T>::kPerChunk);
        }
        const int Pm = sp[nb * 32 + i];                              // PASS 1: position of this lane's probe (-1: padding)

        if (PASS == 2) {
            // merge the chunk statistics of this task's 32 rows: lane = (row, half of the chunks)
            float M = -INFINITY, L = 0.f;
            const float2* p = partial + (int64_t)bh * nsplit * np + nb * 32;     // wave-uniform base; the rest fits 32 bits (host check)
            for (int s0 = h; s0 < nsplit; s0 += 16) {                // 8 independent loads per lane and round
                float2 v[8];
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    const int s = s0 + 2 * q;
                    v[q] = s < nsplit ? p[s * np + i] : make_float2(-INFINITY, 0.f);
                }
#pragma unroll
                for (int q = 0; q < 8; ++q) merge_stats(M, L, v[q].x, v[q].y, c);
            }
            merge_stats(M, L, __shfl_xor(M, 32), __shfl_xor(L, 32), c);
            if (active && slot == 0 && h == 0)
                row_bias[ts][i] = (nb * 32 + i < m && L > 0.f) ? M * c + __log2f(L) : INFINITY;
            __syncthreads();
        }

        float m_run = -INFINITY, l_run = 0.f;                        // PASS 1
        // add the tasks' column sums of stage s (PASS 2) in task order and write the scores of its keys
        // (taken by the workgroup's last threads first: with more waves than tasks those waves are otherwise idle)
        auto reduce_stage = [&](int s) {
            const int buf = s & 1;
            const int row0 = (blk0 + s * KBS) * 32;
            const int keys = min(min(blk1 * 32, n) - row0, SK);
            for (int t = kThreads - 1 - tid; t < keys; t += kThreads) {
                const int j = row0 + t;
                float a = (rd && j < n_eff) ? mass[(int64_t)u * n + j] : 0.f;     // tasks of earlier rounds
                if (j < n_eff)
                    for (int q = 0; q < ntr; ++q) a += colbuf[buf][q][t];
                if (rd + 1 < rounds) {
                    mass[(int64_t)u * n + j] = a;
                } else {
                    a /= (float)G;
                    int cnt = 0;
                    if (j <= Pmin) cnt = m;
                    else for (int q = 0; q < m; ++q) cnt += sp[q] >= j ? 1 : 0;
                    mass[(int64_t)u * n + j] = a / (float)m;
                    if (rank) rank[(int64_t)u * n + j] = cnt > 0 ? a / (float)cnt : 0.f;
                }
            }
        };
#pragma unroll 1
        for (int s = 0; s < S; ++s) {
            // stage s has landed (this wave's pieces, then everyone's); everyone is done with stage s - 1, whose
            // buffer takes stage s + kStageBufs - 1 and whose column sums are complete
            wait_stages(min(kStageBufs - 2, S - 1 - s));
            __syncthreads();
            if (s + kStageBufs - 1 < S) issue_stage(s + kStageBufs - 1);
            if (PASS == 2 && s > 0) reduce_stage(s - 1);
            const int buf = s & 1;                                   // column-sum buffer of the stage
            const char* kb0 = kstage + (s % kStageBufs) * kStageBytes;
            const int sblk = blk0 + s * KBS;                         // first key block of the stage
            if (active) {
#pragma unroll 1
                for (int kb = slot; kb < KBS && sblk + kb < blk1; kb += KS) {
                    const int jb = (sblk + kb) * 32;
                    if (PASS == 2 && jb >= n_eff) {                  // no probe row sees these keys
                        if (h == 0) colbuf[buf][ts][kb * 32 + i] = 0.f;
                        continue;
                    }
                    const char* krow = kb0 + (kb * 32 + i) * RB;
                    auto kfrag = [&](int cc) { return *reinterpret_cast<const uintx4*>(krow + swz_chunk(2 * cc + h, k_row_swizzle<RB>(i))); };
                    floatx16 acc = {0};
                    const bool masked = has_pad || jb + 31 > Pmin;  // wave-uniform
                    if (PASS == 1) {
#pragma unroll
                        for (int cc = 0; cc < CH; ++cc) acc = mma_frag<T>(kfrag(cc), qf[cc], acc);
                        // acc[r]: key jb + acc_row(r, h), probe column nb*32 + i  (raw logit)
                        float sv[16], mx = -INFINITY;
#pragma unroll
                        for (int r = 0; r < 16; ++r) sv[r] = acc[r];
                        if (masked) {
#pragma unroll
                            for (int r = 0; r < 16; ++r)
                                if (jb + acc_row(r, h) > Pm) sv[r] = -INFINITY;
                        }
#pragma unroll
                        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sv[r]);
                        const float m_new = fmaxf(m_run, mx);
                        if (m_new > -INFINITY) {
                            const float mc = m_new * c;
                            float sum = l_run * fast_exp2(m_run * c - mc);      // 0 while m_run = -inf
#pragma unroll
                            for (int r = 0; r < 16; ++r) sum += fast_exp2(fmaf(sv[r], c, -mc));
                            l_run = sum;
                            m_run = m_new;
                        }
                    } else {
#pragma unroll
                        for (int cc = 0; cc < CH; ++cc) acc = mma_frag<T>(qf[cc], kfrag(cc), acc);
                        // acc[r]: probe row nb*32 + acc_row(r, h), key column jb + i; rb[r]: exponent offset of that row
                        float rb[16];
#pragma unroll
                        for (int a = 0; a < 4; ++a) {
                            const floatx4 v = *reinterpret_cast<const floatx4*>(&row_bias[ts][8 * a + 4 * h]);
                            rb[4 * a] = v[0]; rb[4 * a + 1] = v[1]; rb[4 * a + 2] = v[2]; rb[4 * a + 3] = v[3];
                        }
                        float sum = 0.f;
                        if (masked) {
#pragma unroll
                            for (int r = 0; r < 16; ++r) {
                                const float pr = fast_exp2(fmaf(acc[r], c, -rb[r]));
                                sum += jb + i > sp[nb * 32 + acc_row(r, h)] ? 0.f : pr;
                            }
                        } else {
#pragma unroll
                            for (int r = 0; r < 16; ++r) sum += fast_exp2(fmaf(acc[r], c, -rb[r]));
                        }
                        sum += __shfl_xor(sum, 32);
                        if (h == 0) colbuf[buf][ts][kb * 32 + i] = sum;
                    }
                }
            }
        }
        if (PASS == 2) {
            __syncthreads();                                         // the last stage's column sums are in LDS
            reduce_stage(S - 1);
        }

        if (PASS == 1) {
            // the two half-waves saw different keys of the same rows; waves that share a task saw different key blocks
            merge_stats(m_run, l_run, __shfl_xor(m_run, 32), __shfl_xor(l_run, 32), c);
            if (h == 0) wstat[w][i] = active ? make_float2(m_run, l_run) : make_float2(-INFINITY, 0.f);
            __syncthreads();
            for (int t = tid; t < ntr * 32; t += kThreads) {
                const int q = t >> 5, pc = t & 31;                   // task slot, probe row of its block
                float M = -INFINITY, L = 0.f;
                for (int sl = 0; sl < KS; ++sl) {
                    const float2 v = wstat[few ? sl * NT + q : q][pc];
                    merge_stats(M, L, v.x, v.y, c);
                }
                const int tk = rd * NWV + q, hd = tk / NB, nbk = tk - hd * NB;
                partial[((int64_t)(b * Hq + g * G + hd) * nsplit + blockIdx.x) * np + nbk * 32 + pc] = make_float2(M, L);
            }
        }
    }
}

// ---------------------------------------------------------------- host side
static int probe_rows(int m) { return (m + 31) / 32 * 32; }

// Workgroups that fit the chip at once with `waves` waves each (registers allow 16 waves per CU here).
static int resident_slots(int waves) {
    static std::atomic<int> cus{0};
    int c = cus.load();
    if (!c) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v < 1) v = 256;
        cus = c = v;
    }
    return c * (16 / waves);
}

// 32-key blocks per chunk so that about `slots` workgroups cover `units` x nblk blocks
static int blocks_per_chunk(int nblk, int units, int slots) {
    const int chunks = std::max(1, std::min(nblk, slots / units));
    return (nblk + chunks - 1) / chunks;
}

size_t score_workspace_bytes(const zipvl_dims& d, int m) {
    // one (max, sum) pair per head, probe row and pass-1 chunk; chunks per unit never exceed the resident slots
    const int max_chunks = std::max(1, resident_slots(8) / std::max(1, d.B * d.Hkv));
    return (size_t)d.B * d.Hq * max_chunks * probe_rows(m) * sizeof(float2);
}

template <typename T, int D, int NWV>
static int launch_score_w(const void* Q, const void* K, const zipvl_dims& d, const ProbeList& pl, int m,
                          int n_eff, float scale, float* mass, float* rank, void* ws, int kv_div, hipStream_t st)
{
    using C = ScoreCfg<T, D, NWV>;
    const float c = scale * kLog2e;
    float2* partial = (float2*)ws;
    const int units = d.B * d.Hkv, NB = probe_rows(m) / 32;
    const size_t lds = (size_t)kStageBufs * C::STG;
    static std::atomic<bool> attr_done{false};
    if (!attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(&score_kernel<T, D, 1, NWV>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void*>(&score_kernel<T, D, 2, NWV>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return set_error(ZIPVL_EHIP, "score: cannot reserve LDS for the key stages");
        attr_done = true;
    }
    const int slots = resident_slots(NWV);
    const int nblk1 = (n_eff + 31) / 32, bpc1 = blocks_per_chunk(nblk1, units, slots), nsplit = (nblk1 + bpc1 - 1) / bpc1;
    const int nblk2 = (d.n + 31) / 32, bpc2 = blocks_per_chunk(nblk2, units, slots), chunks2 = (nblk2 + bpc2 - 1) / bpc2;
    {
        KernelTimer tm(ZIPVL_K_SCORE_ROWSTATS, st);
        hipLaunchKernelGGL((score_kernel<T, D, 1, NWV>), dim3(nsplit, units), dim3(64 * NWV), lds, st,
            (const T*)Q, (const T*)K, d.q_strides[0], d.q_strides[1], d.q_strides[2],
            d.k_strides[0], d.k_strides[1], d.k_strides[2], pl, m, NB, d.n, n_eff, c, partial, nsplit, bpc1,
            (float*)nullptr, (float*)nullptr, d.Hq, d.Hkv, kv_div);
    }
    int rc = check_launch("score_rowstats");
    if (rc) return rc;
    KernelTimer tm(ZIPVL_K_SCORE_COLSUM, st);
    hipLaunchKernelGGL((score_kernel<T, D, 2, NWV>), dim3(chunks2, units), dim3(64 * NWV), lds, st,
        (const T*)Q, (const T*)K, d.q_strides[0], d.q_strides[1], d.q_strides[2],
        d.k_strides[0], d.k_strides[1], d.k_strides[2], pl, m, NB, d.n, n_eff, c, partial, nsplit, bpc2,
        mass, rank, d.Hq, d.Hkv, kv_div);
    return check_launch("score_colsum");
}

template <typename T, int D>
static int launch_score_t(const void* Q, const void* K, const zipvl_dims& d, const ProbeList& pl, int m,
                          int n_eff, float scale, float* mass, float* rank, void* ws, int kv_div, hipStream_t st)
{
    const int NT = (d.Hq / d.Hkv) * (probe_rows(m) / 32);            // (head, probe block) tasks per unit
    if (NT > 8) return launch_score_w<T, D, 16>(Q, K, d, pl, m, n_eff, scale, mass, rank, ws, kv_div, st);
    return launch_score_w<T, D, 8>(Q, K, d, pl, m, n_eff, scale, mass, rank, ws, kv_div, st);
}

int launch_score(const void* Q, const void* K, const zipvl_dims& d0, const int32_t* probe_pos, int m,
                 float scale, int flags, float* mass, float* rank, void* ws, hipStream_t st)
{
    // one row of scores per query head: the same kernels on dims in which every query head is a unit of its own
    // that reads the K of the KV head it belongs to
    zipvl_dims d = d0;
    int kv_div = 1;
    if ((flags & ZIPVL_SCORE_PER_QHEAD) && d0.Hq != d0.Hkv) {
        kv_div = d0.Hq / d0.Hkv;
        d.Hkv = d0.Hq;
    }
    if (d0.Hq / d0.Hkv > kMaxGroup) return set_error(ZIPVL_ESHAPE, "score: Hq/Hkv = %d exceeds %d", d0.Hq / d0.Hkv, kMaxGroup);
    if (d.k_strides[2] * (d.dtype == ZIPVL_BF16 ? 2 : 4) > (1 << 22))       // 256 staged rows must span less than 2 GiB
        return set_error(ZIPVL_ESHAPE, "score: K token stride of %lld elements is too large", (long long)d.k_strides[2]);
    ProbeList pl;
    for (int t = 0; t < ZIPVL_MAX_PROBES; ++t) pl.pos[t] = t < m ? probe_pos[t] : -1;
    const int n_eff = probe_pos[m - 1] + 1;
    if (d.dtype == ZIPVL_BF16) {
        if (d.d == 128) return launch_score_t<__bf16, 128>(Q, K, d, pl, m, n_eff, scale, mass, rank, ws, kv_div, st);
        return launch_score_t<__bf16, 64>(Q, K, d, pl, m, n_eff, scale, mass, rank, ws, kv_div, st);
    }
    if (d.d == 128) return launch_score_t<float, 128>(Q, K, d, pl, m, n_eff, scale, mass, rank, ws, kv_div, st);
    return launch_score_t<float, 64>(Q, K, d, pl, m, n_eff, scale, mass, rank, ws, kv_div, st);
}

}  // namespace zipvl
