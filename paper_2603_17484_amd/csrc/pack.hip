// Layout pre-passes of the matrix-core kernels (memory-bound, one pass over the tensor).
//
//   pack_token_minor : copies of a tensor whose rows are either the tokens of a KV head (V, for
//                      the forward kernel: the token-minor copy XT[b, kv head, channel, row], rows
//                      inside each group of 16 in the order the matrix-core operands want, see
//                      tiles.hpp) or the rows of a branch's row set (Q and dO, for the dK/dV
//                      kernel: compact row-major copies together with the rows' saved statistics
//                      -- for the Global branch this is the consolidation of the active queries
//                      into a contiguous buffer Q_c, App. C Alg. 1 step 1).
// The transpose itself is done by ds_read_b64_tr_b16: sixteen lanes hand in four rows of sixteen
// channels and each lane gets back four rows of one channel.
#include "tiles.hpp"

namespace l2a {
namespace {

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

struct PackArgs {
    Geom gm;
    RowSet rs;
    int kv_rows;  // 1: rows are the tokens of a KV head, tensors are [B,T,Hkv,D]; 0: rows of rs, tensors [B,T,Hq,D]
    const __bf16* x[2];   // up to two tensors share the row list (Q and dO); x[1] may be null
    __bf16* xt[2];        // optional token-minor copies [B*Hkv][128][cap]
    __bf16* xc[2];        // optional compact row-major copies [B*Hkv][cap][128]
    const float* lse;     // optional per-row statistics of the row set, [B,Hq,T]
    const float* delta;
    float* lse2_c;        // [B*Hkv][cap]: lse * log2(e)
    float* delta_c;
    int32_t* pos_c;       // position of the row, -1 for padding
    int cap;              // rows per (b, kv head) in the outputs; multiple of 64
};

__global__ __launch_bounds__(kThreads) void pack_token_minor_kernel(PackArgs a) {
    __shared__ __attribute__((aligned(16))) __bf16 lds[2][kTileRows * kRowPad];
    const Geom& gm = a.gm;
    const int bh = blockIdx.y, b = bh / gm.Hkv, hk = bh - b * gm.Hkv;
    const int r0 = blockIdx.x * 64;
    const int n_rows = a.kv_rows ? gm.T : rows_total(a.rs, gm, bh);
    if (r0 >= n_rows) return;

    // global element offset of row r's channel 0, or -1 for padding
    auto row_offset = [&](int r, int* pos_out, size_t* stat_out) -> long long {
        if (r >= n_rows) return -1;
        if (a.kv_rows) return (((long long)b * gm.T + r) * gm.Hkv + hk) * kD;
        const int code = row_code(a.rs, gm, bh, r);
        const int p = code / gm.G;
        const int head = hk * gm.G + (code - p * gm.G);
        if (pos_out) *pos_out = p;
        if (stat_out) *stat_out = ((size_t)b * gm.Hq + head) * gm.T + p;
        return (((long long)b * gm.T + p) * gm.Hq + head) * kD;
    };

    // ---- 64 rows -> LDS (row-major, padded), and the compact row-major copy
    const int r4 = (threadIdx.x >> 4) * 4, c8 = (threadIdx.x & 15) * 8;
    long long offs[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) offs[i] = row_offset(r0 + r4 + i, nullptr, nullptr);
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        if (!a.x[t]) continue;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            u32x4 v = {0u, 0u, 0u, 0u};
            if (offs[i] >= 0) v = *reinterpret_cast<const u32x4*>(a.x[t] + offs[i] + c8);
            if (a.xt[t]) *reinterpret_cast<u32x4*>(&lds[t][(r4 + i) * kRowPad + c8]) = v;
            if (a.xc[t])
                *reinterpret_cast<u32x4*>(a.xc[t] + ((size_t)bh * a.cap + r0 + r4 + i) * kD + c8) = v;
        }
    }
    if (a.lse2_c && threadIdx.x < 64) {
        int p = -1;
        size_t so = 0;
        const long long off = row_offset(r0 + (int)threadIdx.x, &p, &so);
        const size_t o = (size_t)bh * a.cap + r0 + threadIdx.x;
        a.lse2_c[o] = off >= 0 ? a.lse[so] * kLog2e : 0.f;
        a.delta_c[o] = off >= 0 ? -a.delta[so] : 0.f;  // stored negated: dP accumulators start from it
        a.pos_c[o] = off >= 0 ? p : -1;
    }
    __syncthreads();

    // ---- token-minor copy.  A group of 16 lanes transposes 4 rows x 16 channels at a time; two
    // such reads (rows R..R+3 and R+8..R+11) are one 16-byte chunk of a channel's row.
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j = lane & 15, gi = lane >> 4;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        if (!a.x[t] || !a.xt[t]) continue;
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
            const int combo = (wave * 4 + tt) * 4 + gi;
            const int cb = combo >> 3, lc = combo & 7;   // 16-channel block, chunk of the 64-token row
            const int grp = lc >> 1, hh = lc & 1;
            const int R = 16 * grp + 4 * hh;
            const __bf16* p1 = &lds[t][(R + (j >> 2)) * kRowPad + cb * 16 + 4 * (j & 3)];
            const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (s16x4 __attribute__((address_space(3)))*)(__attribute__((address_space(3))) const void*)p1);
            const s16x4 v2 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (s16x4 __attribute__((address_space(3)))*)(__attribute__((address_space(3))) const void*)(p1 + 8 * kRowPad));
            const s16x8 v = __builtin_shufflevector(v1, v2, 0, 1, 2, 3, 4, 5, 6, 7);
            __bf16* dst = a.xt[t] + ((size_t)bh * kD + cb * 16 + j) * a.cap + r0 + 16 * grp + 8 * hh;
            *reinterpret_cast<s16x8*>(dst) = v;
        }
    }
}

// O = S + A on the rows of a set (Sec. 3.2 Eq. 5), for the forward that runs both branches in one
// launch: O holds S, A the Global branch's rows in fp32, so that the sum is rounded once.  Sixteen
// lanes per row, sixteen rows per workgroup.
__global__ __launch_bounds__(kThreads) void merge_rows_kernel(Geom gm, RowSet rs, const float* __restrict__ A,
                                                              __bf16* __restrict__ O) {
    const int bh = blockIdx.y, b = bh / gm.Hkv, hk = bh - b * gm.Hkv;
    const int r = blockIdx.x * (kThreads / 16) + (threadIdx.x >> 4);
    if (r >= rows_total(rs, gm, bh)) return;
    const int code = row_code(rs, gm, bh, r);
    const int p = code / gm.G;
    const int head = hk * gm.G + (code - p * gm.G);
    const size_t off = (((size_t)b * gm.T + p) * gm.Hq + head) * kD + (threadIdx.x & 15) * 8;
    const f32x8 x = *reinterpret_cast<const f32x8*>(A + off);
    const bf16x8 y = *reinterpret_cast<const bf16x8*>(O + off);
    *reinterpret_cast<bf16x8*>(O + off) = __builtin_convertvector(x + __builtin_convertvector(y, f32x8), bf16x8);
}

}  // namespace

// rows = tokens of each KV head: x [B,T,Hkv,128] -> xt [B*Hkv][128][cap], cap = round_up(T, 64)
int pack_kv(const Geom& g, const void* x, void* xt, int cap, hipStream_t st) {
    PackArgs a{};
    a.gm = g;
    a.rs = RowSet{nullptr, nullptr, nullptr, 0};
    a.kv_rows = 1;
    a.x[0] = (const __bf16*)x;
    a.xt[0] = (__bf16*)xt;
    a.cap = cap;
    KernelTimer kt("pack_kv", st);
    hipLaunchKernelGGL(pack_token_minor_kernel, dim3(cap / 64, g.B * g.Hkv), dim3(kThreads), 0, st, a);
    return launch_status();
}

// rows of a branch: Q and dO -> compact row-major copies + per-row statistics
int pack_rows(const Geom& g, const RowSet& rs, const void* q, const void* dO, const float* lse, const float* delta,
              void* qc, void* gc, float* lse2_c, float* delta_c, int32_t* pos_c, int cap, hipStream_t st) {
    PackArgs a{};
    a.gm = g;
    a.rs = rs;
    a.kv_rows = 0;
    a.x[0] = (const __bf16*)q;
    a.x[1] = (const __bf16*)dO;
    a.xc[0] = (__bf16*)qc;
    a.xc[1] = (__bf16*)gc;
    a.lse = lse;
    a.delta = delta;
    a.lse2_c = lse2_c;
    a.delta_c = delta_c;
    a.pos_c = pos_c;
    a.cap = cap;
    KernelTimer kt(rs.local ? "pack_rows_local" : "pack_rows_global", st);
    hipLaunchKernelGGL(pack_token_minor_kernel, dim3(cap / 64, g.B * g.Hkv), dim3(kThreads), 0, st, a);
    return launch_status();
}

int merge_rows(const Geom& g, const RowSet& rs, const float* A, void* O, hipStream_t st) {
    if (g.D != kD) return L2A_ERR_UNSUPPORTED;
    const long long rows = (long long)g.T * g.G;
    KernelTimer kt("merge_rows", st);
    hipLaunchKernelGGL(merge_rows_kernel, dim3((unsigned)((rows + kThreads / 16 - 1) / (kThreads / 16)), g.B * g.Hkv),
                       dim3(kThreads), 0, st, g, rs, A, (__bf16*)O);
    return launch_status();
}

}  // namespace l2a
