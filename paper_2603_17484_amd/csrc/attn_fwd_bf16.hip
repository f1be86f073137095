// Forward attention kernel, bf16 on the matrix cores (gfx950), for both branches of the layer:
//   GLOBAL rows = compacted routed (position, head-in-group) pairs, keys 0..pos
//          (App. C Alg. 1: tiles of Q_c, causal mask with the original positions Q_idx, K/V tiles
//          beyond the tile's largest position skipped), or all rows in the dense mode;
//   LOCAL  rows = all (position, head) pairs, keys pos-W..pos (Sec. 2 sliding-window mask).
// The epilogue writes the log-sum-exp and merges into O (Sec. 3.1 Eq. 5), so the scatter of
// Alg. 1's last step costs no extra pass.
//
// Work decomposition.  One workgroup = 4 wavefronts = a tile of 4 * 32 * NQB consecutive rows
// of one (batch, KV head); rows of the G query heads of the group are interleaved, so every
// row of a tile reads the same K/V.  K/V are streamed through LDS in blocks of 64 keys
// (double buffered, one barrier per block); V is transposed on its way into LDS.
//
// Everything is computed transposed so that a lane owns a query row:
//   S^T[key, row]  = K Q^T     A = K tile (LDS, row-major), B = Q (registers, loaded once)
//   O^T[ch,  row] += V^T P^T   A = V tile (LDS, transposed), B = P^T = the S^T accumulators
// A lane then holds 32 scores of one row per K block (the lane 32 apart holds the other 32):
// row max / row sum are in-register reductions plus one cross-lane exchange, and the
// rescaling of O is a per-lane scalar.
#include "mfma.hpp"

namespace l2a {
namespace {

constexpr int kBK = 64;  // keys per LDS block

struct FwdArgs {
    Geom gm;
    RowSet rs;
    const __bf16* q;
    const __bf16* k;
    const __bf16* v;
    FwdOut out;
};

template <int NQB, bool LOCAL>
__global__ __launch_bounds__(kThreads) void fwd_kernel(FwdArgs a) {
    constexpr int RW = 32 * NQB;  // rows per wavefront
    constexpr int BQ = 4 * RW;    // rows per workgroup
    __shared__ __attribute__((aligned(16))) __bf16 lds_k[2][kTileRows * kRowPad];
    __shared__ __attribute__((aligned(16))) __bf16 lds_v[2][kD * kColPad];

    const Geom& gm = a.gm;
    const int bh = blockIdx.y, b = bh / gm.Hkv, hk = bh - b * gm.Hkv;
    const int n_rows = rows_total(a.rs, gm, bh);
    const int n_tiles = (n_rows + BQ - 1) / BQ;
    if ((int)blockIdx.x >= n_tiles) return;
    const int tile = n_tiles - 1 - (int)blockIdx.x;  // longest prefixes first

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 31, h = lane >> 5;

    // ---- rows of this workgroup / wavefront / lane
    const int wg_r0 = tile * BQ;
    const int wg_r1 = min(wg_r0 + BQ, n_rows);  // exclusive
    const int wg_pmin = row_code(a.rs, gm, bh, wg_r0) / gm.G;
    const int wg_pmax = row_code(a.rs, gm, bh, wg_r1 - 1) / gm.G;
    const int wv_r0 = wg_r0 + wave * RW;
    const bool wave_active = wv_r0 < n_rows;
    const int wv_r1 = min(wv_r0 + RW, n_rows);
    int wv_pmin = 0, wv_pmax = 0;
    if (wave_active) {
        wv_pmin = row_code(a.rs, gm, bh, wv_r0) / gm.G;
        wv_pmax = row_code(a.rs, gm, bh, wv_r1 - 1) / gm.G;
    }

    int pos[NQB], head[NQB];
    bool valid[NQB];
    bf16x8 qreg[NQB][8];
#pragma unroll
    for (int c = 0; c < NQB; ++c) {
        const int r = wv_r0 + c * 32 + n;
        valid[c] = r < n_rows;
        // rows past the end repeat the last row: computed, never written
        const int code = row_code(a.rs, gm, bh, min(r, n_rows - 1));
        pos[c] = code / gm.G;
        head[c] = hk * gm.G + (code - pos[c] * gm.G);
        const __bf16* qp = a.q + (((size_t)b * gm.T + pos[c]) * gm.Hq + head[c]) * kD + 8 * h;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qreg[c][ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
    }

    // ---- K/V block range of the workgroup
    const int jb0 = LOCAL ? max(wg_pmin - gm.W, 0) / kBK : 0;
    const int jb1 = wg_pmax / kBK;  // inclusive

    const size_t kv_row = (size_t)gm.Hkv * kD;
    const __bf16* kbase = a.k + ((size_t)b * gm.T * gm.Hkv + hk) * kD;
    const __bf16* vbase = a.v + ((size_t)b * gm.T * gm.Hkv + hk) * kD;
    const int r4 = (threadIdx.x >> 4) * 4;
    TileRegs kr, vr;
    auto load_block = [&](int jb) {
        const int k0 = jb * kBK + r4;
        // keys past the end of the sequence are clamped: always masked, never out of bounds
        tile_load(kr, [&](int i) { return kbase + (size_t)min(k0 + i, gm.T - 1) * kv_row; });
        tile_load(vr, [&](int i) { return vbase + (size_t)min(k0 + i, gm.T - 1) * kv_row; });
    };
    auto store_block = [&](int buf) {
        tile_store_rowmajor(kr, lds_k[buf]);
        tile_store_transposed(vr, lds_v[buf]);
    };

    f32x16 oacc[4][NQB];
    float m[NQB], l[NQB];
#pragma unroll
    for (int c = 0; c < NQB; ++c) {
        m[c] = -INFINITY;
        l[c] = 0.f;
#pragma unroll
        for (int d = 0; d < 4; ++d)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[d][c][r] = 0.f;
    }

    load_block(jb0);
    store_block(0);
    __syncthreads();

    for (int jb = jb0; jb <= jb1; ++jb) {
        const int cur = (jb - jb0) & 1;
        if (jb < jb1) load_block(jb + 1);

        const int k0 = jb * kBK;
        bool skip = !wave_active || k0 > wv_pmax;
        if (LOCAL) skip = skip || (k0 + kBK - 1 < wv_pmin - gm.W);
        if (!skip) {
            bool need_mask = k0 + kBK - 1 > wv_pmin;
            if (LOCAL) need_mask = need_mask || (k0 < wv_pmax - gm.W);
            const __bf16* ks_ = lds_k[cur];
            const __bf16* vs_ = lds_v[cur];

            // S^T = K Q^T
            f32x16 s[2][NQB];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int c = 0; c < NQB; ++c)
#pragma unroll
                    for (int r = 0; r < 16; ++r) s[kb][c][r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const bf16x8 a0 = lds_rowmajor(ks_, n, ks, h);
                const bf16x8 a1 = lds_rowmajor(ks_, 32 + n, ks, h);
#pragma unroll
                for (int c = 0; c < NQB; ++c) {
                    s[0][c] = mfma32(a0, qreg[c][ks], s[0][c]);
                    s[1][c] = mfma32(a1, qreg[c][ks], s[1][c]);
                }
            }

            // streaming softmax, one row per lane
            bf16x8 pb[NQB][4];
#pragma unroll
            for (int c = 0; c < NQB; ++c) {
                if (need_mask) {
#pragma unroll
                    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int key = k0 + kb * 32 + c_row(r, h);
                            bool ok = key <= pos[c];
                            if (LOCAL) ok = ok && (key >= pos[c] - gm.W);
                            s[kb][c][r] = ok ? s[kb][c][r] : -INFINITY;
                        }
                }
                float mx = s[0][c][0];
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kb][c][r]);
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                // A row may have seen only masked keys so far (sliding window): its running max is
                // then -inf and must not enter a subtraction.
                const float mnew = fmaxf(m[c], mx * gm.scale_log2);
                const bool grow = mnew > m[c];
                if (__any(grow)) {
                    const float alpha = grow ? fast_exp2(m[c] - mnew) : 1.f;
                    l[c] *= alpha;
#pragma unroll
                    for (int d = 0; d < 4; ++d)
#pragma unroll
                        for (int r = 0; r < 16; ++r) oacc[d][c][r] *= alpha;
                    m[c] = mnew;
                }
                const float negm = (m[c] == -INFINITY) ? 0.f : -m[c];
                float rsum = 0.f;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float p = fast_exp2(fmaf(s[kb][c][r], gm.scale_log2, negm));
                        s[kb][c][r] = p;
                        rsum += p;
                    }
                l[c] += rsum;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    pb[c][kb * 2 + 0] = pack8(s[kb][c], 0);
                    pb[c][kb * 2 + 1] = pack8(s[kb][c], 1);
                }
            }

            // O^T += V^T P^T
#pragma unroll
            for (int step = 0; step < 4; ++step)
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    const bf16x8 av = lds_transposed(vs_, d * 32 + n, step, h);
#pragma unroll
                    for (int c = 0; c < NQB; ++c) oacc[d][c] = mfma32(av, pb[c][step], oacc[d][c]);
                }
        }

        if (jb < jb1) store_block(cur ^ 1);
        __syncthreads();
    }

    // ---- epilogue: normalise, log-sum-exp, merge / scatter
    if (!wave_active) return;
    __bf16* mo = (__bf16*)a.out.main_out;
    __bf16* co = (__bf16*)a.out.copy_out;
    __bf16* zf = (__bf16*)a.out.zero_fill;
#pragma unroll
    for (int c = 0; c < NQB; ++c) {
        const float lt = l[c] + __shfl_xor(l[c], 32);
        if (!valid[c]) continue;
        const float inv = 1.f / lt;
        const size_t base = (((size_t)b * gm.T + pos[c]) * gm.Hq + head[c]) * kD + 4 * h;
#pragma unroll
        for (int d = 0; d < 4; ++d)
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                const size_t off = base + d * 32 + 8 * rg;
                f32x4 x = {oacc[d][c][4 * rg + 0] * inv, oacc[d][c][4 * rg + 1] * inv,
                           oacc[d][c][4 * rg + 2] * inv, oacc[d][c][4 * rg + 3] * inv};
                if (co) *reinterpret_cast<bf16x4*>(co + off) = __builtin_convertvector(x, bf16x4);
                if (a.out.merge) {
                    const bf16x4 old = *reinterpret_cast<const bf16x4*>(mo + off);
                    x += __builtin_convertvector(old, f32x4);
                }
                *reinterpret_cast<bf16x4*>(mo + off) = __builtin_convertvector(x, bf16x4);
                if (zf) {
                    const u32x2 z = {0u, 0u};
                    *reinterpret_cast<u32x2*>(zf + off) = z;
                }
            }
        if (h == 0) {
            const size_t so = ((size_t)b * gm.Hq + head[c]) * gm.T + pos[c];
            a.out.lse_out[so] = (m[c] + __builtin_amdgcn_logf(lt)) * kLn2;
            if (a.out.lse_fill) a.out.lse_fill[so] = -INFINITY;
        }
    }
}

int env_int(const char* name, int dflt) {
    const char* s = getenv(name);
    return s ? atoi(s) : dflt;
}

}  // namespace

int mfma_fwd(const Geom& g, const RowSet& rs, const void* q, const void* k, const void* v, const FwdOut& out,
             hipStream_t st) {
    if (g.D != kD) return L2A_ERR_UNSUPPORTED;
    static const int nqb = env_int("L2A_FWD_NQB", 2);
    FwdArgs a{g, rs, (const __bf16*)q, (const __bf16*)k, (const __bf16*)v, out};
    const long long rows = (long long)g.T * g.G;
    const int bq = 128 * (nqb == 1 ? 1 : 2);
    const dim3 grid((unsigned)((rows + bq - 1) / bq), g.B * g.Hkv);
    KernelTimer kt(rs.local ? "fwd_local" : "fwd_global", st);
    if (nqb == 1) {
        if (rs.local)
            hipLaunchKernelGGL((fwd_kernel<1, true>), grid, dim3(kThreads), 0, st, a);
        else
            hipLaunchKernelGGL((fwd_kernel<1, false>), grid, dim3(kThreads), 0, st, a);
    } else {
        if (rs.local)
            hipLaunchKernelGGL((fwd_kernel<2, true>), grid, dim3(kThreads), 0, st, a);
        else
            hipLaunchKernelGGL((fwd_kernel<2, false>), grid, dim3(kThreads), 0, st, a);
    }
    return launch_status();
}

}  // namespace l2a
