// Backward attention kernels, bf16 on the matrix cores (gfx950).  Gradients are taken only for
// the rows of a branch's row set -- the routed queries for the Global branch -- with the saved
// log-sum-exp and the compacted row list (Sec. 3.2).  The formulas are the standard gradient
// of softmax attention:
//     P = exp(scale Q K^T - lse),  dV = P^T dO,  dP = dO V^T,  dS = P o (dP - delta),
//     dQ = scale dS K,  dK = scale dS^T Q,       delta_t = <dO_t, out_t>.
// Two kernels, no atomics, bit-reproducible:
//   bwd_dq_kernel   : one workgroup per tile of rows (as the forward); streams K/V blocks.
//                     Also emits delta_t = sum_j P_tj dP_tj, which equals <dO_t, out_t> without
//                     the rounding of the saved bf16 output; the dK/dV kernel uses that value.
//   bwd_dkdv_kernel : one workgroup per block of 128 keys; streams tiles of 64 rows, first the
//                     Local rows that can see the block, then the compacted Global rows from
//                     kblk_first_row on.  The G heads of a KV group are rows of the same list,
//                     so the sum over heads needs no second pass.
#include "mfma.hpp"

namespace l2a {
namespace {

constexpr int kBK = 64;

// ======================================================================================
// dQ
// ======================================================================================
struct DqArgs {
    Geom gm;
    RowSet rs;
    const __bf16* q;
    const __bf16* k;
    const __bf16* v;
    const __bf16* dO;
    const float* lse;
    float* delta;  // in: <dO, saved out>; out: sum_j P dP
    __bf16* dq;
    int accumulate;
};

template <int NQB, bool LOCAL>
__global__ __launch_bounds__(kThreads) void bwd_dq_kernel(DqArgs a) {
    constexpr int RW = 32 * NQB;
    constexpr int BQ = 4 * RW;
    __shared__ __attribute__((aligned(16))) __bf16 lds_k[2][kTileRows * kRowPad];
    __shared__ __attribute__((aligned(16))) __bf16 lds_kt[2][kD * kColPad];
    __shared__ __attribute__((aligned(16))) __bf16 lds_v[2][kTileRows * kRowPad];

    const Geom& gm = a.gm;
    const int bh = blockIdx.y, b = bh / gm.Hkv, hk = bh - b * gm.Hkv;
    const int n_rows = rows_total(a.rs, gm, bh);
    const int n_tiles = (n_rows + BQ - 1) / BQ;
    if ((int)blockIdx.x >= n_tiles) return;
    const int tile = n_tiles - 1 - (int)blockIdx.x;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 31, h = lane >> 5;

    const int wg_r0 = tile * BQ;
    const int wg_r1 = min(wg_r0 + BQ, n_rows);
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
    float lse2[NQB], dlt[NQB], dlt_exact[NQB];
    bf16x8 qreg[NQB][8], greg[NQB][8];
#pragma unroll
    for (int c = 0; c < NQB; ++c) {
        const int r = wv_r0 + c * 32 + n;
        valid[c] = r < n_rows;
        const int code = row_code(a.rs, gm, bh, min(r, n_rows - 1));
        pos[c] = code / gm.G;
        head[c] = hk * gm.G + (code - pos[c] * gm.G);
        const size_t off = (((size_t)b * gm.T + pos[c]) * gm.Hq + head[c]) * kD + 8 * h;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            qreg[c][ks] = *reinterpret_cast<const bf16x8*>(a.q + off + ks * 16);
            greg[c][ks] = *reinterpret_cast<const bf16x8*>(a.dO + off + ks * 16);
        }
        const size_t so = ((size_t)b * gm.Hq + head[c]) * gm.T + pos[c];
        lse2[c] = a.lse[so] * kLog2e;
        dlt[c] = a.delta[so];
        dlt_exact[c] = 0.f;
    }

    const int jb0 = LOCAL ? max(wg_pmin - gm.W, 0) / kBK : 0;
    const int jb1 = wg_pmax / kBK;

    const size_t kv_row = (size_t)gm.Hkv * kD;
    const __bf16* kbase = a.k + ((size_t)b * gm.T * gm.Hkv + hk) * kD;
    const __bf16* vbase = a.v + ((size_t)b * gm.T * gm.Hkv + hk) * kD;
    const int r4 = (threadIdx.x >> 4) * 4;
    TileRegs kr, vr;
    auto load_block = [&](int jb) {
        const int k0 = jb * kBK + r4;
        tile_load(kr, [&](int i) { return kbase + (size_t)min(k0 + i, gm.T - 1) * kv_row; });
        tile_load(vr, [&](int i) { return vbase + (size_t)min(k0 + i, gm.T - 1) * kv_row; });
    };
    auto store_block = [&](int buf) {
        tile_store_rowmajor(kr, lds_k[buf]);
        tile_store_transposed(kr, lds_kt[buf]);
        tile_store_rowmajor(vr, lds_v[buf]);
    };

    f32x16 acc[4][NQB];
#pragma unroll
    for (int c = 0; c < NQB; ++c)
#pragma unroll
        for (int d = 0; d < 4; ++d)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[d][c][r] = 0.f;

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
            const __bf16* kt_ = lds_kt[cur];
            const __bf16* vs_ = lds_v[cur];

            bf16x8 dsb[NQB][4];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                // S^T = K Q^T and dP^T = V dO^T for 32 keys
                f32x16 s[NQB], dp[NQB];
#pragma unroll
                for (int c = 0; c < NQB; ++c)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        s[c][r] = 0.f;
                        dp[c][r] = 0.f;
                    }
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) {
                    const bf16x8 ak = lds_rowmajor(ks_, kb * 32 + n, ks, h);
                    const bf16x8 av = lds_rowmajor(vs_, kb * 32 + n, ks, h);
#pragma unroll
                    for (int c = 0; c < NQB; ++c) {
                        s[c] = mfma32(ak, qreg[c][ks], s[c]);
                        dp[c] = mfma32(av, greg[c][ks], dp[c]);
                    }
                }
#pragma unroll
                for (int c = 0; c < NQB; ++c) {
                    float dsum = 0.f;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        float p = fast_exp2(fmaf(s[c][r], gm.scale_log2, -lse2[c]));
                        if (need_mask) {
                            const int key = k0 + kb * 32 + c_row(r, h);
                            bool ok = key <= pos[c];
                            if (LOCAL) ok = ok && (key >= pos[c] - gm.W);
                            p = ok ? p : 0.f;
                        }
                        dsum = fmaf(p, dp[c][r], dsum);
                        s[c][r] = p * (dp[c][r] - dlt[c]);
                    }
                    dlt_exact[c] += dsum;
                    dsb[c][kb * 2 + 0] = pack8(s[c], 0);
                    dsb[c][kb * 2 + 1] = pack8(s[c], 1);
                }
            }
            // dQ^T += K^T dS^T
#pragma unroll
            for (int step = 0; step < 4; ++step)
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    const bf16x8 akt = lds_transposed(kt_, d * 32 + n, step, h);
#pragma unroll
                    for (int c = 0; c < NQB; ++c) acc[d][c] = mfma32(akt, dsb[c][step], acc[d][c]);
                }
        }

        if (jb < jb1) store_block(cur ^ 1);
        __syncthreads();
    }

    if (!wave_active) return;
#pragma unroll
    for (int c = 0; c < NQB; ++c) {
        const float de = dlt_exact[c] + __shfl_xor(dlt_exact[c], 32);
        if (!valid[c]) continue;
        const size_t base = (((size_t)b * gm.T + pos[c]) * gm.Hq + head[c]) * kD + 4 * h;
#pragma unroll
        for (int d = 0; d < 4; ++d)
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                const size_t off = base + d * 32 + 8 * rg;
                f32x4 x = {acc[d][c][4 * rg + 0] * gm.scale, acc[d][c][4 * rg + 1] * gm.scale,
                           acc[d][c][4 * rg + 2] * gm.scale, acc[d][c][4 * rg + 3] * gm.scale};
                if (a.accumulate) {
                    const bf16x4 old = *reinterpret_cast<const bf16x4*>(a.dq + off);
                    x += __builtin_convertvector(old, f32x4);
                }
                *reinterpret_cast<bf16x4*>(a.dq + off) = __builtin_convertvector(x, bf16x4);
            }
        if (h == 0) a.delta[((size_t)b * gm.Hq + head[c]) * gm.T + pos[c]] = de;
    }
}

// ======================================================================================
// dK, dV
// ======================================================================================
constexpr int kKeysPerWg = 128;  // 4 wavefronts x 32 keys
constexpr int kRT = 64;          // rows per streamed tile

struct DkdvArgs {
    Geom gm;
    RowSet rs[2];
    const float* lse[2];
    const float* delta[2];
    int nsets;
    const __bf16* q;
    const __bf16* k;
    const __bf16* v;
    const __bf16* dO;
    __bf16* dk;
    __bf16* dv;
};

struct RowTileLds {
    __bf16 q_rm[kTileRows * kRowPad];
    __bf16 q_t[kD * kColPad];
    __bf16 g_rm[kTileRows * kRowPad];
    __bf16 g_t[kD * kColPad];
    float lse2[kRT];
    float delta[kRT];
    int pos[kRT];
    int pad[kRT];  // keeps the struct a multiple of 16 bytes
};

__global__ __launch_bounds__(kThreads) void bwd_dkdv_kernel(DkdvArgs a) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    RowTileLds* lds = reinterpret_cast<RowTileLds*>(smem);  // [2]

    const Geom& gm = a.gm;
    const int bh = blockIdx.y, b = bh / gm.Hkv, hk = bh - b * gm.Hkv;
    const int k0 = blockIdx.x * kKeysPerWg;  // first key of the workgroup
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 31, h = lane >> 5;
    const int kw0 = k0 + wave * 32;  // first key of the wavefront
    const int key = kw0 + n;         // this lane's key (as a column of S)
    const int nkb = (gm.T + 63) / 64;

    // ---- the wavefront's 32 keys stay in registers as B operands (column = key, k-slots = channels)
    bf16x8 kreg[8], vreg[8];
    {
        const size_t off = (((size_t)b * gm.T + min(key, gm.T - 1)) * gm.Hkv + hk) * kD + 8 * h;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            kreg[ks] = *reinterpret_cast<const bf16x8*>(a.k + off + ks * 16);
            vreg[ks] = *reinterpret_cast<const bf16x8*>(a.v + off + ks * 16);
        }
    }

    // ---- row ranges of each set that can see this block of keys, as 64-row tiles
    int r_begin[2] = {0, 0}, r_end[2] = {0, 0}, ntile[2] = {0, 0};
    for (int s = 0; s < a.nsets; ++s) {
        const RowSet& rs = a.rs[s];
        if (rs.local) {
            r_begin[s] = k0 * gm.G;
            r_end[s] = min(gm.T, k0 + kKeysPerWg + gm.W) * gm.G;
        } else {
            r_begin[s] = rs.kblk_first_row ? rs.kblk_first_row[(size_t)bh * (nkb + 1) + (k0 >> 6)] : k0 * gm.G;
            r_end[s] = rows_total(rs, gm, bh);
        }
        ntile[s] = r_end[s] > r_begin[s] ? (r_end[s] - r_begin[s] + kRT - 1) / kRT : 0;
    }
    const int total_tiles = ntile[0] + ntile[1];

    const int r4 = (threadIdx.x >> 4) * 4;
    TileRegs qr, gr;
    float st_lse2 = 0.f, st_delta = 0.f;
    int st_pos = -1;
    // tile `it` of the concatenated list -> registers
    auto load_tile = [&](int it) {
        const int s = it < ntile[0] ? 0 : 1;
        const RowSet& rs = a.rs[s];
        const int rt0 = r_begin[s] + (it - (s ? ntile[0] : 0)) * kRT;
        const int last = r_end[s] - 1;
        size_t offs[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int code = row_code(rs, gm, bh, min(rt0 + r4 + i, last));
            const int p = code / gm.G;
            offs[i] = (((size_t)b * gm.T + p) * gm.Hq + hk * gm.G + (code - p * gm.G)) * kD;
        }
        tile_load(qr, [&](int i) { return a.q + offs[i]; });
        tile_load(gr, [&](int i) { return a.dO + offs[i]; });
        if (threadIdx.x < kRT) {
            const int r = rt0 + (int)threadIdx.x;
            if (r <= last) {
                const int code = row_code(rs, gm, bh, r);
                const int p = code / gm.G;
                const size_t so = ((size_t)b * gm.Hq + hk * gm.G + (code - p * gm.G)) * gm.T + p;
                st_pos = p;
                st_lse2 = a.lse[s][so] * kLog2e;
                st_delta = a.delta[s][so];
            } else {  // padding row: masked for every key
                st_pos = -1;
                st_lse2 = 0.f;
                st_delta = 0.f;
            }
        }
    };
    auto store_tile = [&](int buf) {
        RowTileLds& t = lds[buf];
        tile_store_rowmajor(qr, t.q_rm);
        tile_store_transposed(qr, t.q_t);
        tile_store_rowmajor(gr, t.g_rm);
        tile_store_transposed(gr, t.g_t);
        if (threadIdx.x < kRT) {
            t.lse2[threadIdx.x] = st_lse2;
            t.delta[threadIdx.x] = st_delta;
            t.pos[threadIdx.x] = st_pos;
        }
    };

    f32x16 dkacc[4], dvacc[4];
#pragma unroll
    for (int d = 0; d < 4; ++d)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            dkacc[d][r] = 0.f;
            dvacc[d][r] = 0.f;
        }

    if (total_tiles > 0) {
        load_tile(0);
        store_tile(0);
    }
    __syncthreads();

    for (int it = 0; it < total_tiles; ++it) {
        const int cur = it & 1;
        if (it + 1 < total_tiles) load_tile(it + 1);

        const int s_ = it < ntile[0] ? 0 : 1;
        const bool local = a.rs[s_].local != 0;
        const RowTileLds& t = lds[cur];

        // rows of a tile ascend in position: cheap bounds for skipping and for the mask
        const int rt0 = r_begin[s_] + (it - (s_ ? ntile[0] : 0)) * kRT;
        const int rt1 = min(rt0 + kRT, r_end[s_]);
        const int t_pmin = row_code(a.rs[s_], gm, bh, rt0) / gm.G;
        const int t_pmax = row_code(a.rs[s_], gm, bh, rt1 - 1) / gm.G;
        bool skip = t_pmax < kw0 || kw0 >= gm.T;
        if (local) skip = skip || (t_pmin - gm.W > kw0 + 31);
        if (!skip) {
            bool need_mask = (t_pmin < kw0 + 31) || (rt1 - rt0 < kRT) || (kw0 + 31 >= gm.T);
            if (local) need_mask = need_mask || (t_pmax - gm.W > kw0);

            bf16x8 pT[4], dsT[4];
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                // S = Q K^T and dP = dO V^T for 32 rows x this wavefront's 32 keys
                f32x16 s, dp;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    s[r] = 0.f;
                    dp[r] = 0.f;
                }
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) {
                    const bf16x8 aq = lds_rowmajor(t.q_rm, qb * 32 + n, ks, h);
                    const bf16x8 ag = lds_rowmajor(t.g_rm, qb * 32 + n, ks, h);
                    s = mfma32(aq, kreg[ks], s);
                    dp = mfma32(ag, vreg[ks], dp);
                }
#pragma unroll
                for (int rg = 0; rg < 4; ++rg) {
                    const int row0 = qb * 32 + 8 * rg + 4 * h;  // registers 4 rg .. 4 rg + 3 hold rows row0 .. row0 + 3
                    const f32x4 l2 = *reinterpret_cast<const f32x4*>(&t.lse2[row0]);
                    const f32x4 dl = *reinterpret_cast<const f32x4*>(&t.delta[row0]);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int r = 4 * rg + e;
                        float p = fast_exp2(fmaf(s[r], gm.scale_log2, -l2[e]));
                        if (need_mask) {
                            const int rp = t.pos[row0 + e];
                            bool ok = rp >= key && key < gm.T;
                            if (local) ok = ok && (rp - key <= gm.W);
                            p = ok ? p : 0.f;
                        }
                        s[r] = p;
                        dp[r] = p * (dp[r] - dl[e]);
                    }
                }
                pT[qb * 2 + 0] = pack8(s, 0);
                pT[qb * 2 + 1] = pack8(s, 1);
                dsT[qb * 2 + 0] = pack8(dp, 0);
                dsT[qb * 2 + 1] = pack8(dp, 1);
            }
            // dV += P^T dO,  dK += dS^T Q   (contract over the tile's 64 rows)
#pragma unroll
            for (int step = 0; step < 4; ++step)
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    const bf16x8 bg = lds_transposed(t.g_t, d * 32 + n, step, h);
                    const bf16x8 bq = lds_transposed(t.q_t, d * 32 + n, step, h);
                    dvacc[d] = mfma32(pT[step], bg, dvacc[d]);
                    dkacc[d] = mfma32(dsT[step], bq, dkacc[d]);
                }
        }

        if (it + 1 < total_tiles) store_tile(cur ^ 1);
        __syncthreads();
    }

    // ---- write dK, dV: lane = channel d*32+n, register r = key c_row(r, h)
#pragma unroll
    for (int d = 0; d < 4; ++d)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int kk = kw0 + c_row(r, h);
            if (kk < gm.T) {
                const size_t off = (((size_t)b * gm.T + kk) * gm.Hkv + hk) * kD + d * 32 + n;
                a.dk[off] = (__bf16)(dkacc[d][r] * gm.scale);
                a.dv[off] = (__bf16)dvacc[d][r];
            }
        }
}

int env_int(const char* name, int dflt) {
    const char* s = getenv(name);
    return s ? atoi(s) : dflt;
}

}  // namespace

int mfma_bwd_dq(const Geom& g, const RowSet& rs, const void* q, const void* k, const void* v, const void* dO,
                const float* lse, float* delta, void* dq, int accumulate, hipStream_t st) {
    if (g.D != kD) return L2A_ERR_UNSUPPORTED;
    static const int nqb = env_int("L2A_DQ_NQB", 1);
    DqArgs a{g, rs, (const __bf16*)q, (const __bf16*)k, (const __bf16*)v, (const __bf16*)dO, lse, delta,
             (__bf16*)dq, accumulate};
    const long long rows = (long long)g.T * g.G;
    const int bq = 128 * (nqb == 2 ? 2 : 1);
    const dim3 grid((unsigned)((rows + bq - 1) / bq), g.B * g.Hkv);
    KernelTimer kt(rs.local ? "bwd_dq_local" : "bwd_dq_global", st);
    if (nqb == 2) {
        if (rs.local)
            hipLaunchKernelGGL((bwd_dq_kernel<2, true>), grid, dim3(kThreads), 0, st, a);
        else
            hipLaunchKernelGGL((bwd_dq_kernel<2, false>), grid, dim3(kThreads), 0, st, a);
    } else {
        if (rs.local)
            hipLaunchKernelGGL((bwd_dq_kernel<1, true>), grid, dim3(kThreads), 0, st, a);
        else
            hipLaunchKernelGGL((bwd_dq_kernel<1, false>), grid, dim3(kThreads), 0, st, a);
    }
    return launch_status();
}

int mfma_bwd_dkdv(const Geom& g, const RowSet* sets, int nsets, const void* q, const void* k, const void* v,
                  const void* dO, const float* const* lse, const float* const* delta, void* dk, void* dv,
                  hipStream_t st) {
    if (g.D != kD) return L2A_ERR_UNSUPPORTED;
    DkdvArgs a;
    a.gm = g;
    a.nsets = nsets;
    for (int i = 0; i < 2; ++i) {
        a.rs[i] = sets[i < nsets ? i : 0];
        a.lse[i] = lse[i < nsets ? i : 0];
        a.delta[i] = delta[i < nsets ? i : 0];
    }
    a.q = (const __bf16*)q;
    a.k = (const __bf16*)k;
    a.v = (const __bf16*)v;
    a.dO = (const __bf16*)dO;
    a.dk = (__bf16*)dk;
    a.dv = (__bf16*)dv;
    const size_t smem = 2 * sizeof(RowTileLds);
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute((const void*)bwd_dkdv_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)smem) != hipSuccess)
            return L2A_ERR_LAUNCH;
        attr_set = true;
    }
    const dim3 grid((g.T + kKeysPerWg - 1) / kKeysPerWg, g.B * g.Hkv);
    KernelTimer kt("bwd_dkdv", st);
    hipLaunchKernelGGL(bwd_dkdv_kernel, grid, dim3(kThreads), smem, st, a);
    return launch_status();
}

}  // namespace l2a
