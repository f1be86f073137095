// Router front-end (Sec. 3.1 Eq. 3): score dhat_t = sigmoid(<w, x_t> + bias) and decision
// d_t = [dhat_t >= tau] of every token, written as the byte mask l2a_route_compact reads
// (mask_heads = 1: one decision per token, shared by all heads).  The decision is taken on the
// logit, logit >= ln(tau / (1 - tau)), the same comparison without the sigmoid's rounding.
//
// HBM-bound: x is read once (B T C elements), everything else is small.  A wavefront takes four
// tokens at a time so that a slice of w is loaded once per four rows of x; lanes own 8 adjacent
// channels (16-byte loads for bf16), partial sums are fp32 and meet in a butterfly.
#include "common.hpp"

#include <hip/hip_bf16.h>

namespace l2a {
namespace {

constexpr int kThreads = 256;
constexpr int kTok = 4;  // tokens per wavefront pass

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct RouterArgs {
    const void* x;
    const float* w;
    float bias, thr;
    float* dhat;
    float* logit;
    uint8_t* mask;
    long long ntok;
    int C;
};

template <typename E>
__device__ __forceinline__ void load8(const E* p, float (&v)[8]);
template <>
__device__ __forceinline__ void load8<float>(const float* p, float (&v)[8]) {
    const f32x4 a = *reinterpret_cast<const f32x4*>(p), b = *reinterpret_cast<const f32x4*>(p + 4);
    v[0] = a[0], v[1] = a[1], v[2] = a[2], v[3] = a[3], v[4] = b[0], v[5] = b[1], v[6] = b[2], v[7] = b[3];
}
template <>
__device__ __forceinline__ void load8<__bf16>(const __bf16* p, float (&v)[8]) {
    const bf16x8 a = *reinterpret_cast<const bf16x8*>(p);
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = (float)a[i];
}

template <typename E>
__global__ __launch_bounds__(kThreads) void router_kernel(RouterArgs a) {
    const int lane = threadIdx.x & 63;
    const long long wave = (long long)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    const long long t0 = wave * kTok;
    if (t0 >= a.ntok) return;
    const E* x = static_cast<const E*>(a.x);
    float acc[kTok];
#pragma unroll
    for (int i = 0; i < kTok; ++i) acc[i] = 0.f;
    for (int c = lane * 8; c < a.C; c += 64 * 8) {
        float wv[8];
        load8<float>(a.w + c, wv);
#pragma unroll
        for (int i = 0; i < kTok; ++i) {
            const long long t = t0 + i < a.ntok ? t0 + i : a.ntok - 1;  // a ragged last group repeats its last token
            float xv[8];
            load8<E>(x + (size_t)t * a.C + c, xv);
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[i] = fmaf(wv[j], xv[j], acc[i]);
        }
    }
#pragma unroll
    for (int i = 0; i < kTok; ++i)
        for (int o = 32; o > 0; o >>= 1) acc[i] += __shfl_xor(acc[i], o);
    if (lane < kTok && t0 + lane < a.ntok) {
        float lg = acc[0];
#pragma unroll
        for (int i = 1; i < kTok; ++i) lg = lane == i ? acc[i] : lg;
        lg += a.bias;
        a.mask[t0 + lane] = lg >= a.thr ? 1 : 0;
        if (a.dhat) a.dhat[t0 + lane] = 1.f / (1.f + __expf(-lg));
        if (a.logit) a.logit[t0 + lane] = lg;
    }
}

}  // namespace

int router_decide(const l2a_params& p, int C, const void* x, const float* w, float bias, float thr, float* logit,
                  float* dhat, uint8_t* mask, hipStream_t st) {
    RouterArgs a{x, w, bias, thr, dhat, logit, mask, (long long)p.B * p.T, C};
    const long long waves = (a.ntok + kTok - 1) / kTok;
    const dim3 grid((unsigned)((waves + kThreads / 64 - 1) / (kThreads / 64)));
    KernelTimer kt("router", st);
    if (p.dtype == L2A_FP32)
        hipLaunchKernelGGL((router_kernel<float>), grid, dim3(kThreads), 0, st, a);
    else
        hipLaunchKernelGGL((router_kernel<__bf16>), grid, dim3(kThreads), 0, st, a);
    return launch_status();
}

}  // namespace l2a
