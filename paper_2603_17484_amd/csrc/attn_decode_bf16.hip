// Decode step of the layer (Sec. 3.4): one new token per sequence attends to the KV cache --
// Local attention over the last W+1 keys for every token, Global attention over the whole prefix
// only if the token's router decision is 1, skipped entirely otherwise -- and the two are merged
// as o = s + d a (Sec. 3.1 Eq. 5).  HBM-bound: the cache is read once per branch that runs.
//
// Split-key scheme, two launches:
//   decode_partial_kernel  grid (chunks of 512 keys, branch, batch x KV head), one wavefront per
//       workgroup.  The G query heads of a KV group are the rows of one 32-row matrix tile (rows >= G
//       are padding), so K and V are read once for all of them.  The wavefront walks its chunk in
//       32-key sub-blocks: K and V rows go global -> LDS with direct loads into its one 16 KB buffer,
//       S^T = K Q^T and O^T += V^T P^T run on the matrix cores with the streaming softmax of App. C
//       Alg. 1 in between; V^T operands are transposed on the way out of LDS (ds_read_b64_tr_b16).
//       A wavefront does not overlap its own loads with its arithmetic: up to ten such workgroups
//       share a CU and overlap each other's, which keeps 160 KB of loads in flight per CU (measured
//       faster than double buffers in fewer, larger workgroups) and makes the units of work small
//       enough that a mix of routed and unrouted sequences still fills the chip evenly.
//       One partial (max, sum, O) per chunk, head and branch.
//   decode_combine_kernel  one workgroup per (batch, query head): merges the chunks of each
//       branch, writes S, A, the log-sum-exps and O = S + d A.
#include "tiles.hpp"

namespace l2a {
namespace {

constexpr int kChunk = 512;   // keys per workgroup
constexpr int kSub = 32;     // keys per wavefront step
constexpr int kWaves = 1;     // wavefronts per workgroup
constexpr int kBufs = 1;     // LDS buffers per wavefront (1: two workgroups per CU overlap each other's loads)
constexpr int kPart = kD + 4;  // floats per partial: max (log2 units), sum, 2 unused, O[128]


struct DecodeArgs {
    Geom gm;            // gm.T = capacity of the cache (tokens per sequence)
    const __bf16* q;    // [B, Hq, D]
    const __bf16* k;    // [B, T, Hkv, D]
    const __bf16* v;
    const int32_t* pos; // [B] position of the new token (keys 0..pos are valid)
    const uint8_t* mask;  // [B, mask_heads]; nullptr: every head routed
    int mask_heads;
    int do_local, do_global;
    int ring;           // the cache is a ring of gm.T slots: key j lies in slot j mod gm.T, pos is unbounded (Local only)
    float* part;        // [B*Hq][2][nchunks][kPart]
    int nchunks;        // chunks per sequence, = ceil(T / chunk)
    int chunk;
    __bf16* O;          // [B, Hq, D]
    __bf16* S;
    __bf16* A;
    float* lse_l;       // [B, Hq]
    float* lse_g;
};

__device__ __forceinline__ bool head_routed(const DecodeArgs& a, int b, int head) {
    if (!a.mask) return true;
    const int mh = a.mask_heads == 1 ? 0 : (a.mask_heads == a.gm.Hq ? head : head / a.gm.G);
    return a.mask[(size_t)b * a.mask_heads + mh] != 0;
}

template <bool RING>
__global__ __launch_bounds__(64 * kWaves) void decode_partial_kernel(DecodeArgs a) {
    // per wavefront: kBufs buffers of (K tile, V tile), 32 keys x 128 channels each
    __shared__ __attribute__((aligned(1024))) __bf16 lds[kWaves][kBufs][2][kSub * 128];

    const Geom& gm = a.gm;
    const int bh = blockIdx.z, b = bh / gm.Hkv, hk = bh - b * gm.Hkv;
    const int branch = blockIdx.y;  // 0 local, 1 global
    const int chunk = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 31, h = lane >> 5;

    // positions outside the cache are clamped, never followed; in a ring only negative ones are
    const int t_abs = max(a.pos[b], 0);
    const int t = min(t_abs, gm.T - 1);
    if (branch == 0 ? !a.do_local : !a.do_global) return;
    if (branch == 1) {  // Global attention is skipped entirely when no head of the group is routed
        bool any = false;
        for (int g = 0; g < gm.G; ++g) any = any || head_routed(a, b, hk * gm.G + g);
        if (!any) return;
    }
    // keys lo..hi; in a ring: slots 0..hi are written, which of them lie in the window is decided per key
    const int lo = (branch == 0 && !RING) ? max(t - gm.W, 0) : 0, hi = t;
    const int c0 = chunk * a.chunk;
    if (c0 > hi || c0 + a.chunk <= lo) return;
    const int kb = max(c0, lo) / kSub, ke = min(c0 + a.chunk - 1, hi) / kSub;  // sub-blocks kb..ke of this chunk
    // Which keys of a sub-block count is decided without branches (a basic-block boundary between
    // the score instructions and the code that reads their results costs the compiler its
    // bookkeeping of the wait between them).  Without a ring: lo <= key <= hi.  In a ring the token
    // in slot `key` is age = (t_ref - key) mod T positions back and counts if age <= W; a ring that
    // has not wrapped yet (t_abs < T) must not wrap either: its slots behind the new token are
    // unwritten.  (A wrapped ring has a multiple of 32 slots, so no sub-block reaches past its end.)
    const unsigned t_ref = RING ? t_abs % gm.T : 0;
    const unsigned wrap = (RING && t_abs >= gm.T) ? gm.T : 0;

    // Q of the group's heads as B operands: lane n = row (head in group), rows >= G repeat the last head
    const int head = hk * gm.G + min(n, gm.G - 1);
    bf16x8 qreg[8];
    {
        const __bf16* qp = a.q + ((size_t)b * gm.Hq + head) * kD + 8 * h;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qreg[ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
    }

    const unsigned kv_row_bytes = (unsigned)gm.Hkv * kD * 2;
    const char* kbase = (const char*)(a.k + ((size_t)b * gm.T * gm.Hkv + hk) * kD);
    const char* vbase = (const char*)(a.v + ((size_t)b * gm.T * gm.Hkv + hk) * kD);
    const RmDma<kSub, 1> off = rm_dma_setup<kSub, 1>(kv_row_bytes, 0);
    const RmDma<kSub, 1> off_tr = rm_tr_dma_setup<kSub, 1>(kv_row_bytes, 0);
    const unsigned lds0 = lds_offset(&lds[0][0][0][0]) + wave * (unsigned)sizeof(lds[0]);
    auto load = [&](int sb, int buf) __attribute__((always_inline)) {
        const size_t src = (size_t)sb * kSub * kv_row_bytes;
        const unsigned dst = lds0 + buf * (unsigned)sizeof(lds[0][0]);
        if ((sb + 1) * kSub <= hi + 1) {
            rm_dma_issue(off, kbase + src, dst, 0);
            rm_dma_issue(off_tr, vbase + src, dst + kSub * 256, 0);
        } else {  // the sub-block that holds the new token: the rows behind it are not written yet (or past
                  // the end of the cache) and may hold anything, NaN patterns included, which a zero
                  // weight would not keep out of the sums: they repeat the last valid row (always masked)
            rm_dma_issue_clamped<kSub, 1>(kv_row_bytes, hi + 1 - sb * kSub, kbase + src, dst, 0);
            const int valid = hi + 1 - sb * kSub;
#pragma unroll
            for (int i = 0; i < kSub / 4; ++i) {
                const int row = i * 4 + (lane >> 4);
                dma16_so(vbase + src, (unsigned)min(row, valid - 1) * kv_row_bytes +
                                          (unsigned)(((lane & 15) ^ rm_tr_swizzle(row)) * 16),
                         dst + kSub * 256 + i * 1024);
            }
        }
    };

    f32x16 oacc[4];
#pragma unroll
    for (int d = 0; d < 4; ++d)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[d][r] = 0.f;
    float m = -INFINITY, l = 0.f;
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

    // this wavefront's sub-blocks: kb + wave, kb + wave + 4, ...
    int sb = kb + wave;
    if (kBufs == 2 && sb <= ke) load(sb, 0);
    for (int it = 0; sb <= ke; sb += kWaves, ++it) {
        const int buf = kBufs == 2 ? (it & 1) : 0;
        if (kBufs == 2 && sb + kWaves <= ke) {
            load(sb + kWaves, buf ^ 1);
            asm volatile("s_waitcnt vmcnt(16)" ::: "memory");  // the 16 loads just issued may stay in flight
        } else {
            if (kBufs == 1) load(sb, 0);  // the previous step's LDS reads have all returned (their MFMAs were issued)
            dma_wait();
        }
        const __bf16* kt = &lds[wave][buf][0][0];
        const __bf16* vt = &lds[wave][buf][1][0];

        // S^T[key, row] = K Q^T
        f32x16 s = zero16;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) s = mfma32(rm_operand(kt, n, ks, h), qreg[ks], s);

        // streaming softmax, one row per lane (the lane 32 apart holds the row's other 16 keys)
        const int k0 = sb * kSub;
        float mx = -INFINITY;
        const int lo_l = lo - k0 - 4 * h, hi_l = hi - k0 - 4 * h;  // the lane's keys are k0 + 4 h + cr
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int cr = 8 * (r >> 2) + (r & 3);
            bool ok;
            if constexpr (RING) {
                const unsigned d = t_ref - (unsigned)(k0 + 4 * h + cr), age = min(d, d + wrap);  // d < 0 reads as a huge number
                ok = age <= (unsigned)gm.W;
            } else {
                ok = cr >= lo_l && cr <= hi_l;
            }
            s[r] = ok ? s[r] * gm.scale_log2 : -INFINITY;
            mx = fmaxf(mx, s[r]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        // a ring larger than the window has sub-blocks out of reach: while no key has been seen the
        // running maximum stays -inf and the exponentials take 0 as their reference (all of them are 0)
        const float mnew = fmaxf(m, mx);  // without a ring every sub-block of the range has a valid key: mnew is finite
        const float mref = (RING && mnew == -INFINITY) ? 0.f : mnew;
        const float alpha = fast_exp2(m - mref);  // exp2(-inf) = 0 on the first step
        m = mnew;
        float rsum = 0.f;
        uint32_t pw[2][4];
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
            const float p0 = fast_exp2(s[r] - mref), p1 = fast_exp2(s[r + 1] - mref);
            rsum += p0 + p1;
            f32x2 f = {p0, p1};
            pw[r >> 3][(r & 7) >> 1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
        }
        l = l * alpha + rsum;
        if (__any(alpha != 1.f)) {  // the running maximum of some row grew
#pragma unroll
            for (int d = 0; d < 4; ++d)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[d][r] *= alpha;
        }

        // O^T[ch, row] += V^T P^T
#pragma unroll
        for (int step = 0; step < 2; ++step) {
            const u32x4 pv = {pw[step][0], pw[step][1], pw[step][2], pw[step][3]};
#pragma unroll
            for (int d = 0; d < 4; ++d)
                oacc[d] = mfma32(rm_tr_col_operand(vt, d, step, lane), __builtin_bit_cast(bf16x8, pv), oacc[d]);
        }
    }
    l += __shfl_xor(l, 32);

    // ---- merge the four wavefronts in LDS (rows < G only), one partial per chunk
    __syncthreads();  // every wavefront is done with its tiles
    float* stage = reinterpret_cast<float*>(&lds[0][0][0][0]);  // [4 waves][G][kPart]
    if (n < gm.G) {
        float* dst = stage + ((size_t)wave * gm.G + n) * kPart;
        if (h == 0) {
            dst[0] = m;
            dst[1] = l;
        }
#pragma unroll
        for (int d = 0; d < 4; ++d)
#pragma unroll
            for (int r = 0; r < 16; ++r) dst[4 + d * 32 + c_row(r, h)] = oacc[d][r];
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < gm.G * kD; idx += 64 * kWaves) {
        const int g = idx / kD, c = idx - g * kD;
        float mm = -INFINITY;
        for (int w = 0; w < kWaves; ++w) mm = fmaxf(mm, stage[((size_t)w * gm.G + g) * kPart]);
        float ll = 0.f, oo = 0.f;
        for (int w = 0; w < kWaves; ++w) {
            const float* src = stage + ((size_t)w * gm.G + g) * kPart;
            const float sc = src[0] == -INFINITY ? 0.f : fast_exp2(src[0] - mm);
            ll += src[1] * sc;
            oo += src[4 + c] * sc;
        }
        float* out = a.part + ((((size_t)b * gm.Hq + hk * gm.G + g) * 2 + branch) * a.nchunks + chunk) * kPart;
        out[4 + c] = oo;
        if (c == 0) {
            out[0] = mm;
            out[1] = ll;
        }
    }
}

// Thread = (channel, slice): slice i of n (n = blockDim.x / 128 <= kSlices) takes every n-th chunk with a
// running maximum (loads of successive chunks are independent, the loop is unrolled); the slices meet in LDS.
constexpr int kSlices = 8;
__global__ __launch_bounds__(kSlices * kD) void decode_combine_kernel(DecodeArgs a) {
    const int nslices = blockDim.x >> 7;
    __shared__ float sm[kSlices][kD], sl[kSlices][kD], so[kSlices][kD];
    const Geom& gm = a.gm;
    const int bhq = blockIdx.x, b = bhq / gm.Hq, head = bhq - b * gm.Hq;
    const int c = threadIdx.x & (kD - 1), slice = threadIdx.x >> 7;
    const int t = min(max(a.pos[b], 0), gm.T - 1);  // ring: the last written slot while it fills up, then the last slot
    float out[2] = {0.f, 0.f};
    float lse[2] = {-INFINITY, -INFINITY};
    for (int branch = 0; branch < 2; ++branch) {
        const bool on = branch == 0 ? a.do_local != 0 : (a.do_global && head_routed(a, b, head));
        if (!on) continue;  // uniform over the workgroup
        const int lo = (branch == 0 && !a.ring) ? max(t - gm.W, 0) : 0;
        const int c_lo = lo / a.chunk, c_hi = t / a.chunk;
        const float* base = a.part + (((size_t)bhq * 2 + branch) * a.nchunks) * kPart;
        float mm = -INFINITY, ll = 0.f, oo = 0.f;
#pragma unroll 8
        for (int ch = c_lo + slice; ch <= c_hi; ch += nslices) {
            const float* src = base + (size_t)ch * kPart;
            const float m1 = src[0], l1 = src[1], o1 = src[4 + c];
            const float mn = fmaxf(mm, m1);
            // exp2(-inf) = 0 on the first chunk; a chunk of a ring may have no slot in the window (m1 = -inf):
            // while nothing has been seen the reference is 0 and both factors are 0
            const float mref = mn == -INFINITY ? 0.f : mn;
            const float s0 = fast_exp2(mm - mref), s1 = fast_exp2(m1 - mref);
            ll = ll * s0 + l1 * s1;
            oo = oo * s0 + o1 * s1;
            mm = mn;
        }
        __syncthreads();
        sm[slice][c] = mm, sl[slice][c] = ll, so[slice][c] = oo;
        __syncthreads();
        if (slice == 0) {  // slices that had no chunk hold (-inf, 0, 0); slice 0 always has one
            float mn = sm[0][c];
            for (int i = 1; i < nslices; ++i) mn = fmaxf(mn, sm[i][c]);
            float lsum = 0.f, osum = 0.f;
            for (int i = 0; i < nslices; ++i) {
                const float sc = sm[i][c] == -INFINITY ? 0.f : fast_exp2(sm[i][c] - mn);
                lsum += sl[i][c] * sc;
                osum += so[i][c] * sc;
            }
            out[branch] = osum / lsum;
            lse[branch] = (mn + __builtin_amdgcn_logf(lsum)) * kLn2;
        }
    }
    if (slice) return;
    const size_t o = (size_t)bhq * kD + c;
    a.O[o] = (__bf16)(out[0] + out[1]);
    if (a.S) a.S[o] = (__bf16)out[0];
    if (a.A) a.A[o] = (__bf16)out[1];
    if (c == 0) {
        if (a.lse_l) a.lse_l[bhq] = lse[0];
        if (a.lse_g) a.lse_g[bhq] = lse[1];
    }
}

}  // namespace

size_t decode_partial_floats(const Geom& g) {
    const int nchunks = (g.T + kChunk - 1) / kChunk;
    return (size_t)g.B * g.Hq * 2 * nchunks * kPart;
}

int mfma_decode(const Geom& g, const void* q, const void* k, const void* v, const int32_t* pos, const uint8_t* mask,
                int mask_heads, int do_local, int do_global, int ring, float* part, void* O, void* S, void* A, float* lse_l,
                float* lse_g, hipStream_t st) {
    if (g.D != kD || g.G > 16) return L2A_ERR_UNSUPPORTED;  // the merge stage holds kWaves x G partials in LDS
    DecodeArgs a{};
    a.gm = g;
    a.q = (const __bf16*)q;
    a.k = (const __bf16*)k;
    a.v = (const __bf16*)v;
    a.pos = pos;
    a.mask = mask;
    a.mask_heads = mask_heads;
    a.do_local = do_local;
    a.do_global = do_global;
    a.ring = ring;
    a.part = part;
    a.chunk = kChunk;
    a.nchunks = (g.T + a.chunk - 1) / a.chunk;
    a.O = (__bf16*)O;
    a.S = (__bf16*)S;
    a.A = (__bf16*)A;
    a.lse_l = lse_l;
    a.lse_g = lse_g;
    {
        KernelTimer kt("decode_partial", st);
        if (ring)
            hipLaunchKernelGGL(decode_partial_kernel<true>, dim3(a.nchunks, 2, g.B * g.Hkv), dim3(64 * kWaves), 0, st, a);
        else
            hipLaunchKernelGGL(decode_partial_kernel<false>, dim3(a.nchunks, 2, g.B * g.Hkv), dim3(64 * kWaves), 0, st, a);
    }
    {
        KernelTimer kt("decode_combine", st);
        const int slices = a.nchunks >= 128 ? 8 : (a.nchunks >= 32 ? 4 : 2);  // few chunks: few, short loops
        hipLaunchKernelGGL(decode_combine_kernel, dim3(g.B * g.Hq), dim3(slices * kD), 0, st, a);
    }
    return launch_status();
}

}  // namespace l2a
