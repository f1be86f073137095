// Straightforward scalar-FMA kernels for both branches of the layer, fp32 arithmetic on fp32
// or bf16 storage.  They serve the fp32 element type (where no bf16 matrix core applies) and
// head sizes the MFMA kernels are not built for.  Four lanes share one query row (forward,
// dQ) or one key token (dK/dV); each lane keeps D/4 of the row's channels in registers and
// partial dot products are combined with two cross-lane exchanges.
//
// Forward: streaming softmax over the row's keys (App. C Alg. 1, with a key tile of one);
// backward: the standard softmax-attention gradient restricted to the routed rows (Sec. 3.2).
#include "common.hpp"

namespace l2a {
namespace {

constexpr int kThreads = 256;
constexpr int kRowsPerBlock = kThreads / 4;

template <typename E>
__device__ __forceinline__ float ld(const E* p) {
    return (float)*p;
}
template <typename E>
__device__ __forceinline__ void st(E* p, float x) {
    *p = (E)x;
}

__device__ __forceinline__ float quad_sum(float x) {
    x += __shfl_xor(x, 1);
    x += __shfl_xor(x, 2);
    return x;
}

struct Row {
    int pos, g;
};

// rows of one (b, KV head): how many, and the r-th one (device data: clamped into the valid ranges)
__device__ __forceinline__ int num_rows(const RowSet& rs, const Geom& gm, int bh) {
    return rs.count ? min(max(rs.count[bh], 0), gm.T * gm.G) : gm.T * gm.G;
}
__device__ __forceinline__ Row get_row(const RowSet& rs, const Geom& gm, int bh, int r) {
    const int code = rs.row_idx ? min(max(rs.row_idx[(size_t)bh * gm.T * gm.G + r], 0), gm.T * gm.G - 1) : r;
    Row x;
    x.pos = code / gm.G;
    x.g = code - x.pos * gm.G;
    return x;
}

template <typename E, int DL>
__global__ __launch_bounds__(kThreads) void simple_fwd_kernel(Geom gm, RowSet rs, const E* __restrict__ q,
                                                              const E* __restrict__ k, const E* __restrict__ v,
                                                              FwdOut out) {
    const int bh = blockIdx.y, b = bh / gm.Hkv, hk = bh % gm.Hkv;
    const int r = blockIdx.x * kRowsPerBlock + (threadIdx.x >> 2);
    const int part = threadIdx.x & 3;
    if (r >= num_rows(rs, gm, bh)) return;
    const Row row = get_row(rs, gm, bh, r);
    const int h = hk * gm.G + row.g;
    const size_t qoff = (((size_t)b * gm.T + row.pos) * gm.Hq + h) * gm.D + part * DL;

    float qr[DL], acc[DL];
#pragma unroll
    for (int i = 0; i < DL; ++i) {
        qr[i] = ld(q + qoff + i);
        acc[i] = 0.f;
    }
    float m = -INFINITY, l = 0.f;
    const int j0 = rs.local ? (row.pos - gm.W > 0 ? row.pos - gm.W : 0) : 0;
    for (int j = j0; j <= row.pos; ++j) {
        const size_t koff = (((size_t)b * gm.T + j) * gm.Hkv + hk) * gm.D + part * DL;
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < DL; ++i) s += qr[i] * ld(k + koff + i);
        s = quad_sum(s) * gm.scale;
        const float mn = fmaxf(m, s);
        const float alpha = expf(m - mn);
        const float p = expf(s - mn);
        l = l * alpha + p;
#pragma unroll
        for (int i = 0; i < DL; ++i) acc[i] = acc[i] * alpha + p * ld(v + koff + i);
        m = mn;
    }
    const float inv = 1.f / l;
    E* mo = (E*)out.main_out;
    E* co = (E*)out.copy_out;
    E* zf = (E*)out.zero_fill;
#pragma unroll
    for (int i = 0; i < DL; ++i) {
        const float x = acc[i] * inv;
        const float y = out.merge ? ld(mo + qoff + i) + x : x;
        st(mo + qoff + i, y);
        if (co) st(co + qoff + i, x);
        if (zf) st(zf + qoff + i, 0.f);
    }
    if (part == 0) {
        const size_t so = ((size_t)b * gm.Hq + h) * gm.T + row.pos;
        out.lse_out[so] = m + logf(l);
        if (out.lse_fill) out.lse_fill[so] = -INFINITY;
    }
}

template <typename E, int DL>
__global__ __launch_bounds__(kThreads) void simple_bwd_dq_kernel(Geom gm, RowSet rs, const E* __restrict__ q,
                                                                 const E* __restrict__ k, const E* __restrict__ v,
                                                                 const E* __restrict__ dO,
                                                                 const float* __restrict__ lse, float* delta,
                                                                 E* dq, int accumulate) {
    const int bh = blockIdx.y, b = bh / gm.Hkv, hk = bh % gm.Hkv;
    const int r = blockIdx.x * kRowsPerBlock + (threadIdx.x >> 2);
    const int part = threadIdx.x & 3;
    if (r >= num_rows(rs, gm, bh)) return;
    const Row row = get_row(rs, gm, bh, r);
    const int h = hk * gm.G + row.g;
    const size_t qoff = (((size_t)b * gm.T + row.pos) * gm.Hq + h) * gm.D + part * DL;
    const size_t so = ((size_t)b * gm.Hq + h) * gm.T + row.pos;

    float qr[DL], gr[DL], acc[DL];
#pragma unroll
    for (int i = 0; i < DL; ++i) {
        qr[i] = ld(q + qoff + i);
        gr[i] = ld(dO + qoff + i);
        acc[i] = 0.f;
    }
    const float L = lse[so], dl = delta[so];
    float dl_exact = 0.f;  // sum_j p_j dp_j: the same quantity without the rounding of the saved output
    const int j0 = rs.local ? (row.pos - gm.W > 0 ? row.pos - gm.W : 0) : 0;
    for (int j = j0; j <= row.pos; ++j) {
        const size_t koff = (((size_t)b * gm.T + j) * gm.Hkv + hk) * gm.D + part * DL;
        float s = 0.f, dp = 0.f;
#pragma unroll
        for (int i = 0; i < DL; ++i) {
            s += qr[i] * ld(k + koff + i);
            dp += gr[i] * ld(v + koff + i);
        }
        s = quad_sum(s) * gm.scale;
        dp = quad_sum(dp);
        const float p = expf(s - L);
        const float ds = p * (dp - dl);
        dl_exact += p * dp;
#pragma unroll
        for (int i = 0; i < DL; ++i) acc[i] += ds * ld(k + koff + i);
    }
    if (part == 0) delta[so] = dl_exact;
#pragma unroll
    for (int i = 0; i < DL; ++i) {
        float x = acc[i] * gm.scale;
        if (accumulate) x += ld(dq + qoff + i);
        st(dq + qoff + i, x);
    }
}

struct DkdvSets {
    RowSet rs[2];
    const float* lse[2];
    const float* delta[2];
    int n;
};

template <typename E, int DL>
__global__ __launch_bounds__(kThreads) void simple_bwd_dkdv_kernel(Geom gm, DkdvSets sets, const E* __restrict__ q,
                                                                   const E* __restrict__ k, const E* __restrict__ v,
                                                                   const E* __restrict__ dO, E* dk, E* dv) {
    const int bh = blockIdx.y, b = bh / gm.Hkv, hk = bh % gm.Hkv;
    const int j = blockIdx.x * kRowsPerBlock + (threadIdx.x >> 2);
    const int part = threadIdx.x & 3;
    if (j >= gm.T) return;
    const size_t koff = (((size_t)b * gm.T + j) * gm.Hkv + hk) * gm.D + part * DL;
    float kr[DL], vr[DL], ak[DL], av[DL];
#pragma unroll
    for (int i = 0; i < DL; ++i) {
        kr[i] = ld(k + koff + i);
        vr[i] = ld(v + koff + i);
        ak[i] = 0.f;
        av[i] = 0.f;
    }
    const int nkb = (gm.T + 63) / 64;
    for (int s = 0; s < sets.n; ++s) {
        const RowSet rs = sets.rs[s];
        int r0, r1;  // candidate rows [r0, r1)
        if (rs.local) {
            const int last = j + gm.W < gm.T - 1 ? j + gm.W : gm.T - 1;
            r0 = j * gm.G;
            r1 = (last + 1) * gm.G;
        } else {
            r0 = rs.kblk_first_row ? max(rs.kblk_first_row[(size_t)bh * (nkb + 1) + (j >> 6)], 0) : (j >> 6) * 64 * gm.G;
            r1 = num_rows(rs, gm, bh);
        }
        for (int r = r0; r < r1; ++r) {
            const Row row = get_row(rs, gm, bh, r);
            if (row.pos < j) continue;
            const int h = hk * gm.G + row.g;
            const size_t qoff = (((size_t)b * gm.T + row.pos) * gm.Hq + h) * gm.D + part * DL;
            const size_t so = ((size_t)b * gm.Hq + h) * gm.T + row.pos;
            float sc = 0.f, dp = 0.f;
#pragma unroll
            for (int i = 0; i < DL; ++i) {
                sc += ld(q + qoff + i) * kr[i];
                dp += ld(dO + qoff + i) * vr[i];
            }
            sc = quad_sum(sc) * gm.scale;
            dp = quad_sum(dp);
            const float p = expf(sc - sets.lse[s][so]);
            const float ds = p * (dp - sets.delta[s][so]);
#pragma unroll
            for (int i = 0; i < DL; ++i) {
                av[i] += p * ld(dO + qoff + i);
                ak[i] += ds * ld(q + qoff + i);
            }
        }
    }
#pragma unroll
    for (int i = 0; i < DL; ++i) {
        st(dk + koff + i, ak[i] * gm.scale);
        st(dv + koff + i, av[i]);
    }
}

inline dim3 row_grid(const Geom& g) {
    const long long rows = (long long)g.T * g.G;
    return dim3((unsigned)((rows + kRowsPerBlock - 1) / kRowsPerBlock), g.B * g.Hkv);
}

}  // namespace

template <typename T>
static const T* cp(const void* p) { return (const T*)p; }

int simple_fwd(const Geom& g, int dtype, const RowSet& rs, const void* q, const void* k, const void* v,
               const FwdOut& out, hipStream_t st) {
    const dim3 grid = row_grid(g);
    KernelTimer kt(rs.local ? "scalar_fwd_local" : "scalar_fwd_global", st);
    if (dtype == L2A_FP32 && g.D == 64)
        hipLaunchKernelGGL((simple_fwd_kernel<float, 16>), grid, dim3(kThreads), 0, st, g, rs, cp<float>(q), cp<float>(k), cp<float>(v), out);
    else if (dtype == L2A_FP32 && g.D == 128)
        hipLaunchKernelGGL((simple_fwd_kernel<float, 32>), grid, dim3(kThreads), 0, st, g, rs, cp<float>(q), cp<float>(k), cp<float>(v), out);
    else if (dtype == L2A_BF16 && g.D == 64)
        hipLaunchKernelGGL((simple_fwd_kernel<__bf16, 16>), grid, dim3(kThreads), 0, st, g, rs, cp<__bf16>(q), cp<__bf16>(k), cp<__bf16>(v), out);
    else if (dtype == L2A_BF16 && g.D == 128)
        hipLaunchKernelGGL((simple_fwd_kernel<__bf16, 32>), grid, dim3(kThreads), 0, st, g, rs, cp<__bf16>(q), cp<__bf16>(k), cp<__bf16>(v), out);
    else
        return L2A_ERR_UNSUPPORTED;
    return launch_status();
}

int simple_bwd_dq(const Geom& g, int dtype, const RowSet& rs, const void* q, const void* k, const void* v,
                  const void* dO, const float* lse, float* delta, void* dq, int accumulate, hipStream_t st) {
    const dim3 grid = row_grid(g);
    KernelTimer kt(rs.local ? "scalar_bwd_dq_local" : "scalar_bwd_dq_global", st);
    if (dtype == L2A_FP32 && g.D == 64)
        hipLaunchKernelGGL((simple_bwd_dq_kernel<float, 16>), grid, dim3(kThreads), 0, st, g, rs, cp<float>(q), cp<float>(k), cp<float>(v), cp<float>(dO), lse, delta, (float*)dq, accumulate);
    else if (dtype == L2A_FP32 && g.D == 128)
        hipLaunchKernelGGL((simple_bwd_dq_kernel<float, 32>), grid, dim3(kThreads), 0, st, g, rs, cp<float>(q), cp<float>(k), cp<float>(v), cp<float>(dO), lse, delta, (float*)dq, accumulate);
    else if (dtype == L2A_BF16 && g.D == 64)
        hipLaunchKernelGGL((simple_bwd_dq_kernel<__bf16, 16>), grid, dim3(kThreads), 0, st, g, rs, cp<__bf16>(q), cp<__bf16>(k), cp<__bf16>(v), cp<__bf16>(dO), lse, delta, (__bf16*)dq, accumulate);
    else if (dtype == L2A_BF16 && g.D == 128)
        hipLaunchKernelGGL((simple_bwd_dq_kernel<__bf16, 32>), grid, dim3(kThreads), 0, st, g, rs, cp<__bf16>(q), cp<__bf16>(k), cp<__bf16>(v), cp<__bf16>(dO), lse, delta, (__bf16*)dq, accumulate);
    else
        return L2A_ERR_UNSUPPORTED;
    return launch_status();
}

int simple_bwd_dkdv(const Geom& g, int dtype, const RowSet* sets, int nsets, const void* q, const void* k,
                    const void* v, const void* dO, const float* const* lse, const float* const* delta, void* dk,
                    void* dv, hipStream_t st) {
    DkdvSets s;
    s.n = nsets;
    for (int i = 0; i < nsets; ++i) {
        s.rs[i] = sets[i];
        s.lse[i] = lse[i];
        s.delta[i] = delta[i];
    }
    const dim3 grid((g.T + kRowsPerBlock - 1) / kRowsPerBlock, g.B * g.Hkv);
    KernelTimer kt("scalar_bwd_dkdv", st);
    if (dtype == L2A_FP32 && g.D == 64)
        hipLaunchKernelGGL((simple_bwd_dkdv_kernel<float, 16>), grid, dim3(kThreads), 0, st, g, s, cp<float>(q), cp<float>(k), cp<float>(v), cp<float>(dO), (float*)dk, (float*)dv);
    else if (dtype == L2A_FP32 && g.D == 128)
        hipLaunchKernelGGL((simple_bwd_dkdv_kernel<float, 32>), grid, dim3(kThreads), 0, st, g, s, cp<float>(q), cp<float>(k), cp<float>(v), cp<float>(dO), (float*)dk, (float*)dv);
    else if (dtype == L2A_BF16 && g.D == 64)
        hipLaunchKernelGGL((simple_bwd_dkdv_kernel<__bf16, 16>), grid, dim3(kThreads), 0, st, g, s, cp<__bf16>(q), cp<__bf16>(k), cp<__bf16>(v), cp<__bf16>(dO), (__bf16*)dk, (__bf16*)dv);
    else if (dtype == L2A_BF16 && g.D == 128)
        hipLaunchKernelGGL((simple_bwd_dkdv_kernel<__bf16, 32>), grid, dim3(kThreads), 0, st, g, s, cp<__bf16>(q), cp<__bf16>(k), cp<__bf16>(v), cp<__bf16>(dO), (__bf16*)dk, (__bf16*)dv);
    else
        return L2A_ERR_UNSUPPORTED;
    return launch_status();
}

}  // namespace l2a
