// Small memory-bound helpers: the backward pass's per-row dot products and fills.
#include "common.hpp"

namespace l2a {
namespace {

constexpr int kThreads = 256;

// delta_l[b,h,t] = <dO, S>, delta_g[b,h,t] = <dO, A>  (the "D" vector of the FlashAttention
// backward, one per branch; delta_g is also the task-loss part of the router-score gradient,
// Sec. 3.3 Eq. 7).  Sixteen lanes share one (b, t, h) row.
template <typename E, int DL>
__global__ __launch_bounds__(kThreads) void row_deltas_kernel(Geom gm, const E* __restrict__ dO,
                                                              const E* __restrict__ S, const E* __restrict__ A,
                                                              float* __restrict__ delta_l,
                                                              float* __restrict__ delta_g) {
    const long long row = (long long)blockIdx.x * (kThreads / 16) + (threadIdx.x >> 4);
    const int part = threadIdx.x & 15;
    const long long nrows = (long long)gm.B * gm.T * gm.Hq;
    if (row >= nrows) return;
    const size_t off = (size_t)row * gm.D + part * DL;
    float a = 0.f, c = 0.f;
#pragma unroll
    for (int i = 0; i < DL; ++i) {
        const float g = (float)dO[off + i];
        if (S) a += g * (float)S[off + i];
        if (A) c += g * (float)A[off + i];
    }
    for (int o = 8; o > 0; o >>= 1) {
        a += __shfl_xor(a, o);
        c += __shfl_xor(c, o);
    }
    if (part == 0) {
        const int h = (int)(row % gm.Hq);
        const long long bt = row / gm.Hq;
        const int t = (int)(bt % gm.T);
        const int b = (int)(bt / gm.T);
        const size_t so = ((size_t)b * gm.Hq + h) * gm.T + t;
        if (delta_l) delta_l[so] = a;
        if (delta_g) delta_g[so] = c;
    }
}

__global__ __launch_bounds__(kThreads) void fill_u32_kernel(uint32_t* p, size_t n, uint32_t value) {
    size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * kThreads;
    for (; i < n; i += stride) p[i] = value;
}

}  // namespace

int row_deltas(const Geom& g, int dtype, const void* dO, const void* S, const void* A, float* delta_l,
               float* delta_g, hipStream_t st) {
    const long long nrows = (long long)g.B * g.T * g.Hq;
    const dim3 grid((unsigned)((nrows + kThreads / 16 - 1) / (kThreads / 16)));
    KernelTimer kt("row_deltas", st);
    if (dtype == L2A_FP32 && g.D == 64)
        hipLaunchKernelGGL((row_deltas_kernel<float, 4>), grid, dim3(kThreads), 0, st, g, (const float*)dO, (const float*)S, (const float*)A, delta_l, delta_g);
    else if (dtype == L2A_FP32 && g.D == 128)
        hipLaunchKernelGGL((row_deltas_kernel<float, 8>), grid, dim3(kThreads), 0, st, g, (const float*)dO, (const float*)S, (const float*)A, delta_l, delta_g);
    else if (dtype == L2A_BF16 && g.D == 64)
        hipLaunchKernelGGL((row_deltas_kernel<__bf16, 4>), grid, dim3(kThreads), 0, st, g, (const __bf16*)dO, (const __bf16*)S, (const __bf16*)A, delta_l, delta_g);
    else if (dtype == L2A_BF16 && g.D == 128)
        hipLaunchKernelGGL((row_deltas_kernel<__bf16, 8>), grid, dim3(kThreads), 0, st, g, (const __bf16*)dO, (const __bf16*)S, (const __bf16*)A, delta_l, delta_g);
    else
        return L2A_ERR_UNSUPPORTED;
    return launch_status();
}

// bytes must be a multiple of 4 (every tensor here is)
int fill_zero(void* ptr, size_t bytes, hipStream_t st) {
    const size_t n = bytes / 4;
    if (n == 0) return L2A_OK;
    size_t blocks = (n + kThreads - 1) / kThreads;
    if (blocks > 65536) blocks = 65536;
    KernelTimer kt("fill", st);
    hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, st, (uint32_t*)ptr, n, 0u);
    return launch_status();
}

int fill_f32(float* ptr, size_t n, float value, hipStream_t st) {
    if (n == 0) return L2A_OK;
    size_t blocks = (n + kThreads - 1) / kThreads;
    if (blocks > 65536) blocks = 65536;
    uint32_t bits;
    __builtin_memcpy(&bits, &value, 4);
    KernelTimer kt("fill", st);
    hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, st, (uint32_t*)ptr, n, bits);
    return launch_status();
}

}  // namespace l2a
