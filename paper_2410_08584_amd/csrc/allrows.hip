// Exact token scores from EVERY row of the attention matrix (Eq. (6) and Eq. (8)
// as written, before the probe approximation of the supplementary material): the
// accuracy reference for the probe scores.  A is never stored.  Two passes of one
// kernel body over the causal half of Q K^T:
//   pass 1  per query row, the exponent offset lse = max * c + log2(sum exp2((s - max) c))
//           of its visible logits (c = softmax scale * log2 e);
//   pass 2  per query head and key column, sum over the rows that see it of exp2(s c - lse);
//           a small kernel then averages the query heads of a group (fixed order) and writes
//           mass = a / n and rank = a / (n - j)  (every row at or after j counts in Eq. (8)).
// A workgroup keeps 128 rows of one side in registers as MFMA fragments (32 per wave:
// queries in pass 1, keys in pass 2) and streams the other side through LDS in chunks
// of 64 rows (double buffered, one barrier per chunk).  The product is taken as
// (streamed rows) x (register rows)^T on 32x32 tiles, so a lane owns one register-side
// row and its statistic (running max / sum in pass 1, column sum in pass 2) never
// leaves the lane until the end.
#include <atomic>

#include "launch.h"

namespace zipvl {

constexpr int kArRows = 128;      // register-side rows per workgroup (4 waves x 32)
constexpr int kArChunk = 64;      // streamed rows per chunk

template <typename T, int D>
struct ArCfg {
    static constexpr int E = Elem<T>::kBytes;
    static constexpr int CH = D / Elem<T>::kPerChunk;       // fragments per row per lane
    static constexpr int RS = D * E + 16;                    // padded LDS row (bytes)
    static constexpr int CPR = D * E / 16;                   // 16-byte pieces per row
    static constexpr int NPRE = kArChunk * CPR / 256;        // pieces staged per thread
    static constexpr int BUF = kArChunk * RS;                // one chunk in LDS
};

template <typename T, int D, int PASS>
__global__ __launch_bounds__(256) void allrows_pass_kernel(
    const T* __restrict__ R, int64_t rs0, int64_t rs1, int64_t rs2,     // register side: Q (pass 1) / K (pass 2)
    const T* __restrict__ S, int64_t ss0, int64_t ss1, int64_t ss2,     // streamed side: K (pass 1) / Q (pass 2)
    int n, float c, float* __restrict__ lse, float* __restrict__ mass, float* __restrict__ rank, int Hq, int Hkv)
{
    using C = ArCfg<T, D>;
    extern __shared__ __attribute__((aligned(16))) char smem[];          // two chunk buffers, then two lse rows (pass 2)
    float* lse_lds = reinterpret_cast<float*>(smem + 2 * C::BUF);        // [2][kArChunk]
    const int G = Hq / Hkv;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, i = lane & 31, h = lane >> 5;
    const int nblk = (n + kArRows - 1) / kArRows;
    // heavy workgroups first: late query blocks in pass 1, early key blocks in pass 2
    const int blk = PASS == 1 ? nblk - 1 - (int)blockIdx.x : (int)blockIdx.x;
    const int row0 = blk * kArRows, wrow0 = row0 + 32 * w;              // first register-side row of the workgroup / wave
    const int bh = blockIdx.y, b = bh / Hq, head = bh - b * Hq, g = head / G;        // one query head per workgroup

    const int my = wrow0 + i;                                            // this lane's register-side row
    const int myc = min(my, n - 1);
    float colsum = 0.f;                                                  // pass 2
    {
        // register-side fragments: Q[b, head, my] in pass 1; K[b, g, my] in pass 2
        uintx4 rf[C::CH];
        {
            const T* rp = R + b * rs0 + (int64_t)(PASS == 1 ? head : g) * rs1 + (int64_t)myc * rs2;
#pragma unroll
            for (int cc = 0; cc < C::CH; ++cc) rf[cc] = load16(rp + cc * Elem<T>::kPerChunk + h * Elem<T>::kPerFrag);
        }
        const T* Sb = S + b * ss0 + (int64_t)(PASS == 1 ? g : head) * ss1;
        const float* lse_h = lse + (int64_t)(b * Hq + head) * n;
        // streamed chunks this workgroup needs: keys [0, last row] in pass 1; query rows [first key, n) in pass 2
        const int c_begin = PASS == 1 ? 0 : (row0 / kArChunk) * kArChunk;
        const int c_end = PASS == 1 ? min(n, row0 + kArRows) : n;
        float m_run = -INFINITY, l_run = 0.f;                            // pass 1

        uintx4 pre[C::NPRE];
        float pre_lse = 0.f;
        auto fetch = [&](int c0) {
#pragma unroll
            for (int q = 0; q < C::NPRE; ++q) {
                const int t = tid + q * 256, row = t / C::CPR, cc = t - row * C::CPR;
                pre[q] = load16(Sb + (int64_t)min(c0 + row, n - 1) * ss2 + cc * Elem<T>::kPerFrag);
            }
            if (PASS == 2 && tid < kArChunk) pre_lse = lse_h[min(c0 + tid, n - 1)];
        };
        auto stage = [&](int buf) {
#pragma unroll
            for (int q = 0; q < C::NPRE; ++q) {
                const int t = tid + q * 256, row = t / C::CPR, cc = t - row * C::CPR;
                store16(smem + buf * C::BUF + row * C::RS + cc * 16, pre[q]);
            }
            if (PASS == 2 && tid < kArChunk) lse_lds[buf * kArChunk + tid] = pre_lse;
        };
        fetch(c_begin);
        stage(0);
        __syncthreads();
        int buf = 0;
        for (int c0 = c_begin; c0 < c_end; c0 += kArChunk, buf ^= 1) {
            const bool more = c0 + kArChunk < c_end;
            if (more) fetch(c0 + kArChunk);                              // in flight while this chunk is multiplied
            // does this wave need the chunk at all?
            const bool live = PASS == 1 ? c0 <= wrow0 + 31 : c0 + kArChunk - 1 >= wrow0;
            if (live) {
                const char* sb = smem + buf * C::BUF;
                const bool masked = (PASS == 1 ? c0 + kArChunk - 1 > wrow0 : c0 < wrow0 + 31) || c0 + kArChunk > n;
#pragma unroll
                for (int nb = 0; nb < kArChunk / 32; ++nb) {
                    floatx16 acc = {0};
#pragma unroll
                    for (int cc = 0; cc < C::CH; ++cc) {
                        const uintx4 sf = *reinterpret_cast<const uintx4*>(sb + (nb * 32 + i) * C::RS + cc * 32 + h * 16);
                        acc = mma_frag<T>(sf, rf[cc], acc);
                    }
                    // acc[r]: streamed row c0 + nb*32 + acc_row(r, h), register-side row `my`
                    if (PASS == 1) {
                        float sv[16], mx = -INFINITY;
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int key = c0 + nb * 32 + acc_row(r, h);
                            sv[r] = (masked && (key > my || key >= n)) ? -INFINITY : acc[r];
                            mx = fmaxf(mx, sv[r]);
                        }
                        if (mx > -INFINITY) {
                            const float m_new = fmaxf(m_run, mx), mc = m_new * c;
                            float sum = 0.f;
#pragma unroll
                            for (int r = 0; r < 16; ++r) sum += fast_exp2(fmaf(sv[r], c, -mc));
                            l_run = l_run * fast_exp2(m_run * c - mc) + sum;
                            m_run = m_new;
                        }
                    } else {
                        float rb[16];
#pragma unroll
                        for (int a = 0; a < 4; ++a) {
                            const floatx4 v = *reinterpret_cast<const floatx4*>(&lse_lds[buf * kArChunk + nb * 32 + 8 * a + 4 * h]);
                            rb[4 * a] = v[0]; rb[4 * a + 1] = v[1]; rb[4 * a + 2] = v[2]; rb[4 * a + 3] = v[3];
                        }
                        float sum = 0.f;
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int qrow = c0 + nb * 32 + acc_row(r, h);
                            const float p = fast_exp2(fmaf(acc[r], c, -rb[r]));
                            sum += (masked && (qrow < my || qrow >= n)) ? 0.f : p;
                        }
                        colsum += sum;
                    }
                }
            }
            if (more) stage(buf ^ 1);                                    // the other buffer was consumed one chunk ago
            __syncthreads();
        }
        if (PASS == 1) {
            // the two half-waves saw different keys of the same query row: merge, then lse = max c + log2(sum)
            const unsigned um = __float_as_uint(m_run), ul = __float_as_uint(l_run);
            const auto pm = __builtin_amdgcn_permlane32_swap(um, um, false, false);
            const auto pl = __builtin_amdgcn_permlane32_swap(ul, ul, false, false);
            const float m0 = __uint_as_float(pm[0]), m1 = __uint_as_float(pm[1]);
            const float l0 = __uint_as_float(pl[0]), l1 = __uint_as_float(pl[1]);
            const float M = fmaxf(m0, m1);                               // finite: a row sees at least itself
            const float L = l0 * fast_exp2((m0 - M) * c) + l1 * fast_exp2((m1 - M) * c);
            if (h == 0 && my < n) lse[(int64_t)(b * Hq + head) * n + my] = M * c + __log2f(L);
        }
    }
    if (PASS == 2) {
        const unsigned uc = __float_as_uint(colsum);
        const auto pc = __builtin_amdgcn_permlane32_swap(uc, uc, false, false);
        if (h == 0 && my < n) mass[(int64_t)bh * n + my] = __uint_as_float(pc[0]) + __uint_as_float(pc[1]);   // per-head column sums
    }
}

// mass / rank of a unit from the per-head column sums: heads of the group added in ascending order
__global__ __launch_bounds__(256) void allrows_finish_kernel(
    const float* __restrict__ colsum, int n, int Hq, int Hkv, float* __restrict__ mass, float* __restrict__ rank)
{
    const int G = Hq / Hkv, u = blockIdx.y, b = u / Hkv, g = u - b * Hkv;
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= n) return;
    const float* p = colsum + (int64_t)(b * Hq + g * G) * n + j;
    float a = p[0];
    for (int hh = 1; hh < G; ++hh) a += p[(int64_t)hh * n];
    a /= (float)G;
    mass[(int64_t)u * n + j] = a / (float)n;
    if (rank) rank[(int64_t)u * n + j] = a / (float)(n - j);
}

size_t allrows_workspace_bytes(const zipvl_dims& d) { return 2 * (size_t)d.B * d.Hq * d.n * sizeof(float); }   // lse, per-head column sums

template <typename T, int D>
static int launch_allrows_t(const void* Q, const void* K, const zipvl_dims& d, float scale,
                            float* mass, float* rank, void* ws, hipStream_t st)
{
    using C = ArCfg<T, D>;
    const size_t lds = 2 * (size_t)C::BUF + 2 * kArChunk * sizeof(float);
    static std::atomic<bool> attr_done{false};
    if (!attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(&allrows_pass_kernel<T, D, 1>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void*>(&allrows_pass_kernel<T, D, 2>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return set_error(ZIPVL_EHIP, "score_all_rows: cannot reserve %zu bytes of LDS", lds);
        attr_done = true;
    }
    const float c = scale * kLog2e;
    const int nblk = (d.n + kArRows - 1) / kArRows;
    float* lse = (float*)ws;
    {
        KernelTimer tm(ZIPVL_K_ALLROWS_LSE, st);
        hipLaunchKernelGGL((allrows_pass_kernel<T, D, 1>), dim3(nblk, d.B * d.Hq), dim3(256), lds, st,
            (const T*)Q, d.q_strides[0], d.q_strides[1], d.q_strides[2],
            (const T*)K, d.k_strides[0], d.k_strides[1], d.k_strides[2],
            d.n, c, lse, (float*)nullptr, (float*)nullptr, d.Hq, d.Hkv);
    }
    int rc = check_launch("allrows_lse");
    if (rc) return rc;
    float* colsum = lse + (size_t)d.B * d.Hq * d.n;
    KernelTimer tm(ZIPVL_K_ALLROWS_COLSUM, st);
    hipLaunchKernelGGL((allrows_pass_kernel<T, D, 2>), dim3(nblk, d.B * d.Hq), dim3(256), lds, st,
        (const T*)K, d.k_strides[0], d.k_strides[1], d.k_strides[2],
        (const T*)Q, d.q_strides[0], d.q_strides[1], d.q_strides[2],
        d.n, c, lse, colsum, (float*)nullptr, d.Hq, d.Hkv);
    rc = check_launch("allrows_colsum");
    if (rc) return rc;
    hipLaunchKernelGGL(allrows_finish_kernel, dim3((d.n + 255) / 256, d.B * d.Hkv), dim3(256), 0, st,
        (const float*)colsum, d.n, d.Hq, d.Hkv, mass, rank);
    return check_launch("allrows_finish");
}

int launch_score_all_rows(const void* Q, const void* K, const zipvl_dims& d, float scale,
                          float* mass, float* rank, void* ws, hipStream_t st)
{
    if (d.dtype == ZIPVL_BF16) {
        if (d.d == 128) return launch_allrows_t<__bf16, 128>(Q, K, d, scale, mass, rank, ws, st);
        return launch_allrows_t<__bf16, 64>(Q, K, d, scale, mass, rank, ws, st);
    }
    if (d.d == 128) return launch_allrows_t<float, 128>(Q, K, d, scale, mass, rank, ws, st);
    return launch_allrows_t<float, 64>(Q, K, d, scale, mass, rank, ws, st);
}

}  // namespace zipvl
