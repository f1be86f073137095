// Small memory-bound helpers: the backward pass's per-row dot products and fills.
#include "common.hpp"

#include <algorithm>

namespace l2a {
namespace {

constexpr int kThreads = 256;

// delta_l[b,h,t] = <dO, S>, delta_g[b,h,t] = <dO, A>  (the "D" vector of the FlashAttention
// backward, one per branch; delta_g is also the task-loss part of the router-score gradient,
// Sec. 3.3 Eq. 7).  A workgroup takes `tok` consecutive tokens of one sequence -- a contiguous
// stretch of [t, h, D] rows, sixteen lanes per row -- and transposes its results through LDS, so
// that the [b, h, t] outputs are written in runs of consecutive t instead of one scattered float
// per row.
template <typename E, int DL>
__global__ __launch_bounds__(kThreads) void row_deltas_kernel(Geom gm, const E* __restrict__ dO,
                                                              const E* __restrict__ S, const E* __restrict__ A,
                                                              float* __restrict__ delta_l,
                                                              float* __restrict__ delta_g, int tok) {
    extern __shared__ float stage[];  // [2][Hq][tok]
    const int b = blockIdx.y, t0 = blockIdx.x * tok;
    const int ntok = min(tok, gm.T - t0);
    const int part = threadIdx.x & 15;
    float* sa = stage;
    float* sc = stage + gm.Hq * tok;
    const size_t row0 = ((size_t)b * gm.T + t0) * gm.Hq;
    for (int r = threadIdx.x >> 4; r < ntok * gm.Hq; r += kThreads / 16) {
        const size_t off = (row0 + r) * gm.D + part * DL;
        float a = 0.f, c = 0.f;
        // one 16- or 32-byte load per array and lane
        typedef E Vec __attribute__((ext_vector_type(DL)));
        const Vec gv = *reinterpret_cast<const Vec*>(dO + off);
        if (S) {
            const Vec sv = *reinterpret_cast<const Vec*>(S + off);
#pragma unroll
            for (int i = 0; i < DL; ++i) a += (float)gv[i] * (float)sv[i];
        }
        if (A) {
            const Vec av = *reinterpret_cast<const Vec*>(A + off);
#pragma unroll
            for (int i = 0; i < DL; ++i) c += (float)gv[i] * (float)av[i];
        }
        for (int o = 8; o > 0; o >>= 1) {
            a += __shfl_xor(a, o);
            c += __shfl_xor(c, o);
        }
        if (part == 0) {
            const int tt = r / gm.Hq, h = r - tt * gm.Hq;
            sa[h * tok + tt] = a;
            sc[h * tok + tt] = c;
        }
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < gm.Hq * tok; idx += kThreads) {
        const int h = idx / tok, tt = idx - h * tok;
        if (tt >= ntok) continue;
        const size_t so = ((size_t)b * gm.Hq + h) * gm.T + t0 + tt;
        if (delta_l) delta_l[so] = sa[idx];
        if (delta_g) delta_g[so] = sc[idx];
    }
}

// delta of the first tokens of a sequence, from its definition instead of from the saved outputs:
//     delta_t = sum_j p_tj <dO_t, v_j>,   p_tj = exp(scale <q_t, k_j> - lse_t)     (= <dO_t, out_t>).
// The saved outputs are bf16: <dO_t, out_t> then carries an error of about 2^-9 sqrt(D) |dO_t| |out_t|,
// which enters dq_t as  scale * error * sum_j p_tj k_j.  Both factors shrink like 1 / sqrt(keys) for
// rows that average many keys, but for the first few tokens they do not (token 2 with N(0,1) inputs:
// up to 1.2e-2 per branch, twice that when both branches read the same tensors, since s_t = a_t
// there), so the first kHeadTokens deltas are recomputed exactly.  One wavefront per (token, head);
// lane = key.  A row whose log-sum-exp is -inf (not routed: a_t = 0) gets delta = 0.
constexpr int kHeadTokens = 64;

__global__ __launch_bounds__(64) void head_deltas_kernel(Geom gm, const __bf16* __restrict__ q,
                                                         const __bf16* __restrict__ k, const __bf16* __restrict__ v,
                                                         const __bf16* __restrict__ dO, const float* __restrict__ lse,
                                                         float* __restrict__ delta, int local) {
    const int t = blockIdx.x, h = blockIdx.y, b = blockIdx.z, j = threadIdx.x;
    const int hk = h / gm.G;
    const size_t so = ((size_t)b * gm.Hq + h) * gm.T + t;
    const float l = lse[so];
    float term = 0.f;
    const bool in_reach = j <= t && (!local || t - j <= gm.W);
    if (in_reach && l != -INFINITY) {
        const __bf16* qr = q + (((size_t)b * gm.T + t) * gm.Hq + h) * gm.D;
        const __bf16* gr = dO + (((size_t)b * gm.T + t) * gm.Hq + h) * gm.D;
        const __bf16* kr = k + (((size_t)b * gm.T + j) * gm.Hkv + hk) * gm.D;
        const __bf16* vr = v + (((size_t)b * gm.T + j) * gm.Hkv + hk) * gm.D;
        float s = 0.f, dp = 0.f;
        for (int c = 0; c < gm.D; ++c) {
            s = fmaf((float)qr[c], (float)kr[c], s);
            dp = fmaf((float)gr[c], (float)vr[c], dp);
        }
        term = expf(s * gm.scale - l) * dp;
    }
    for (int o = 32; o > 0; o >>= 1) term += __shfl_xor(term, o);
    if (j == 0) delta[so] = term;
}

__global__ __launch_bounds__(kThreads) void fill_u32_kernel(uint32_t* p, size_t n, uint32_t value) {
    size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * kThreads;
    for (; i < n; i += stride) p[i] = value;
}

}  // namespace

int row_deltas(const Geom& g, int dtype, const void* dO, const void* S, const void* A, float* delta_l,
               float* delta_g, hipStream_t st) {
    int tok = 64;  // tokens per workgroup: as many as fit 64 KB of LDS with Hq heads
    while (tok > 1 && sizeof(float) * 2 * g.Hq * tok > 64 * 1024) tok /= 2;
    // short sequences: fewer tokens per workgroup rather than a grid that leaves most of the chip idle
    while (tok > 8 && (long long)((g.T + tok - 1) / tok) * g.B < 2048) tok /= 2;
    const size_t lds = sizeof(float) * 2 * g.Hq * tok;
    if (lds > 64 * 1024) return L2A_ERR_UNSUPPORTED;
    const dim3 grid((unsigned)((g.T + tok - 1) / tok), (unsigned)g.B);
    KernelTimer kt("row_deltas", st);
    if (dtype == L2A_FP32 && g.D == 64)
        hipLaunchKernelGGL((row_deltas_kernel<float, 4>), grid, dim3(kThreads), lds, st, g, (const float*)dO, (const float*)S, (const float*)A, delta_l, delta_g, tok);
    else if (dtype == L2A_FP32 && g.D == 128)
        hipLaunchKernelGGL((row_deltas_kernel<float, 8>), grid, dim3(kThreads), lds, st, g, (const float*)dO, (const float*)S, (const float*)A, delta_l, delta_g, tok);
    else if (dtype == L2A_BF16 && g.D == 64)
        hipLaunchKernelGGL((row_deltas_kernel<__bf16, 4>), grid, dim3(kThreads), lds, st, g, (const __bf16*)dO, (const __bf16*)S, (const __bf16*)A, delta_l, delta_g, tok);
    else if (dtype == L2A_BF16 && g.D == 128)
        hipLaunchKernelGGL((row_deltas_kernel<__bf16, 8>), grid, dim3(kThreads), lds, st, g, (const __bf16*)dO, (const __bf16*)S, (const __bf16*)A, delta_l, delta_g, tok);
    else
        return L2A_ERR_UNSUPPORTED;
    return launch_status();
}

int head_deltas(const Geom& g, const void* q, const void* k, const void* v, const void* dO, const float* lse,
                float* delta, int local, hipStream_t st) {
    static_assert(kHeadTokens <= 64, "one lane per key");
    const dim3 grid((unsigned)std::min(g.T, kHeadTokens), (unsigned)g.Hq, (unsigned)g.B);
    KernelTimer kt("head_deltas", st);
    hipLaunchKernelGGL(head_deltas_kernel, grid, dim3(64), 0, st, g, (const __bf16*)q, (const __bf16*)k,
                       (const __bf16*)v, (const __bf16*)dO, lse, delta, local);
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
