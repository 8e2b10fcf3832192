// KV-cache eviction (Section 4.2; Algorithm 1, cache step) and the cache append
// of the decode phase (Eq. (4); Algorithm 2).  Pure data movement: every row
// is d*e contiguous bytes and moves as 16-byte vectors, 16 (or 8/32) lanes per
// row, so both the gathered reads and the packed writes are full-line accesses.
#include "launch.h"

namespace zipvl {

constexpr int kCompactRows = 64;   // kept rows handled by one workgroup

__global__ __launch_bounds__(256) void compact_kv_kernel(
    const char* __restrict__ K, const char* __restrict__ V,
    int64_t kb_stride, int64_t kh_stride, int64_t kt_stride,     // bytes
    int64_t vb_stride, int64_t vh_stride, int64_t vt_stride,
    const int32_t* __restrict__ idx, const int32_t* __restrict__ kcnt,
    char* __restrict__ Kc, char* __restrict__ Vc, int32_t* __restrict__ len,
    int n, int Hkv, int cap, int row_bytes, int t_per_batch)
{
    const int u = blockIdx.y;
    const int b = u / Hkv, g = u - b * Hkv;
    const int ut = t_per_batch ? b : u;                   // row of idx / k that holds this unit's T
    int kk = kcnt ? kcnt[ut] : n;
    kk = max(0, min(min(kk, n), cap));
    if (blockIdx.x == 0 && threadIdx.x == 0) len[u] = kk;
    const int r0 = blockIdx.x * kCompactRows;
    if (r0 >= kk) return;
    const int cpr = row_bytes >> 4;                       // 16-byte chunks per row
    const char* Kb = K + b * kb_stride + g * kh_stride;
    const char* Vb = V + b * vb_stride + g * vh_stride;
    const int64_t out_base = (int64_t)u * cap * row_bytes;
    for (int w = threadIdx.x; w < kCompactRows * cpr; w += 256) {
        const int r = r0 + w / cpr, c = w - (w / cpr) * cpr;
        if (r >= kk) break;
        const int src = idx ? idx[(int64_t)ut * n + r] : r;
        const int64_t o = out_base + (int64_t)r * row_bytes + c * 16;
        store16(Kc + o, load16(Kb + (int64_t)src * kt_stride + c * 16));
        store16(Vc + o, load16(Vb + (int64_t)src * vt_stride + c * 16));
    }
}

__global__ __launch_bounds__(64) void kv_append_kernel(
    char* __restrict__ Kc, char* __restrict__ Vc, int32_t* __restrict__ len, int cap,
    const char* __restrict__ k_new, const char* __restrict__ v_new, int row_bytes)
{
    const int u = blockIdx.x;
    const int L = len[u];
    if (L < 0 || L >= cap) return;
    const int cpr = row_bytes >> 4;
    const int64_t o = ((int64_t)u * cap + L) * row_bytes;
    for (int c = threadIdx.x; c < cpr; c += 64) {
        store16(Kc + o + c * 16, load16(k_new + (int64_t)u * row_bytes + c * 16));
        store16(Vc + o + c * 16, load16(v_new + (int64_t)u * row_bytes + c * 16));
    }
    __syncthreads();                 // every lane has read len[u] before it changes
    if (threadIdx.x == 0) len[u] = L + 1;
}

int launch_compact_kv(const void* K, const void* V, const zipvl_dims& d, const int32_t* idx,
                      const int32_t* k, void* Kc, void* Vc, int32_t cap, int32_t* len, int flags, hipStream_t st)
{
    const int e = d.dtype == ZIPVL_BF16 ? 2 : 4;
    const int units = d.B * d.Hkv;
    dim3 grid((min(d.n, cap) + kCompactRows - 1) / kCompactRows, units);
    KernelTimer tm(ZIPVL_K_COMPACT_KV, st);
    hipLaunchKernelGGL(compact_kv_kernel, grid, dim3(256), 0, st,
        (const char*)K, (const char*)V,
        d.k_strides[0] * e, d.k_strides[1] * e, d.k_strides[2] * e,
        d.v_strides[0] * e, d.v_strides[1] * e, d.v_strides[2] * e,
        idx, k, (char*)Kc, (char*)Vc, len, d.n, d.Hkv, cap, d.d * e, (flags & ZIPVL_T_PER_BATCH) ? 1 : 0);
    return check_launch("compact_kv");
}

int launch_kv_append(void* Kc, void* Vc, int32_t* len, int32_t cap, const void* k_new,
                     const void* v_new, const zipvl_dims& d, hipStream_t st)
{
    const int e = d.dtype == ZIPVL_BF16 ? 2 : 4;
    KernelTimer tm(ZIPVL_K_KV_APPEND, st);
    hipLaunchKernelGGL(kv_append_kernel, dim3(d.B * d.Hkv), dim3(64), 0, st,
        (char*)Kc, (char*)Vc, len, cap, (const char*)k_new, (const char*)v_new, d.d * e);
    return check_launch("kv_append");
}

}  // namespace zipvl
