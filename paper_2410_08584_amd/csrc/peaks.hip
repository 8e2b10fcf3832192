// Measurement aids (not part of the method): what this GPU actually sustains, for reading the
// roofline fractions of the benchmark.  `mfma_peak` issues nothing but independent bf16 32x32x16
// MFMAs from every SIMD (8 accumulator chains per wave, two waves per SIMD, operands held in
// registers); `stream_read` reads a buffer once with 16-byte loads and keeps a checksum.
#include "launch.h"

namespace zipvl {

constexpr int kPeakChains = 8;

__global__ __launch_bounds__(256, 2) void mfma_peak_kernel(int iters, float* __restrict__ out)
{
    const int lane = threadIdx.x & 63;
    bf16x8 a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(0.001f * (float)(lane + e)); b[e] = (__bf16)(0.002f * (float)(lane - e)); }
    floatx16 acc[kPeakChains];
#pragma unroll
    for (int c = 0; c < kPeakChains; ++c) acc[c] = floatx16{0};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int c = 0; c < kPeakChains; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[c], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < kPeakChains; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[c][r];
    out[(int64_t)blockIdx.x * blockDim.x + threadIdx.x] = s;     // keeps the chains alive
}

__global__ __launch_bounds__(256) void stream_read_kernel(const uintx4* __restrict__ src, int64_t n16, uint32_t* __restrict__ out)
{
    uint32_t s = 0;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
#pragma unroll 4
    for (int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; q < n16; q += stride) {
        const uintx4 v = src[q];
        s ^= v[0] ^ v[1] ^ v[2] ^ v[3];
    }
    out[(int64_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

int launch_probe_mfma(int iters, int workgroups, float* out, hipStream_t st)
{
    KernelTimer tm(ZIPVL_K_PROBE_MFMA, st);
    hipLaunchKernelGGL(mfma_peak_kernel, dim3(workgroups), dim3(256), 0, st, iters, out);
    return check_launch("mfma_peak");
}

int launch_probe_read(const void* src, size_t bytes, int workgroups, uint32_t* out, hipStream_t st)
{
    KernelTimer tm(ZIPVL_K_PROBE_READ, st);
    hipLaunchKernelGGL(stream_read_kernel, dim3(workgroups), dim3(256), 0, st, (const uintx4*)src, (int64_t)(bytes / 16), out);
    return check_launch("stream_read");
}

}  // namespace zipvl
