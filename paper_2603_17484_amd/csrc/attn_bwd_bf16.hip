// Backward attention kernels, bf16 on the matrix cores (gfx950).  Gradients are taken only for
// the rows of a branch's row set -- the routed queries for the Global branch -- with the saved
// log-sum-exp and the compacted row list (Sec. 3.2).  The formulas are the standard gradient
// of softmax attention:
//     P = exp(scale Q K^T - lse),  dV = P^T dO,  dP = dO V^T,  dS = P o (dP - delta),
//     dQ = scale dS K,  dK = scale dS^T Q,       delta_t = <dO_t, out_t>.
// dK and dV (the dQ kernel lives in attn_bwd_dq_bf16.hip); no atomics, bit-reproducible:
//   bwd_dkdv_kernel : one workgroup per block of 128 keys; streams tiles of 64 rows, first the
//                     Local rows that can see the block, then the compacted Global rows from
//                     kblk_first_row on.  The G heads of a KV group are rows of the same list,
//                     so the sum over heads needs no second pass.
#include <type_traits>

#include "mfma.hpp"

namespace l2a {
namespace {

constexpr int kBK = 64;

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

// One element of the backward softmax: register r of an S tile (row 8 (r/4) + 4 h + r%4, this
// lane's key).  s <- P, dp <- dS.
template <bool MASK>
__device__ __forceinline__ void bwd_softmax_elem(int r, f32x16& s, f32x16& dp, const f32x4 (&l2)[4],
                                                 const f32x4 (&dl)[4], const i32x4 (&ps)[4], float c, int key,
                                                 int T, int W, bool local) {
    const int rg = r >> 2, e = r & 3;
    float p = fast_exp2(fmaf(s[r], c, -l2[rg][e]));
    if (MASK) {
        const int rp = ps[rg][e];
        bool ok = rp >= key && key < T;
        if (local) ok = ok && (rp - key <= W);
        p = ok ? p : 0.f;
    }
    s[r] = p;
    dp[r] = p * (dp[r] - dl[rg][e]);
}

// Keeps the instruction scheduler from moving anything across this point: the tile body below
// is software-pipelined by hand (matrix-core instructions interleaved with the VALU work and
// the LDS traffic of the neighbouring stages), one wavefront per SIMD.
#define L2A_FENCE() __builtin_amdgcn_sched_barrier(0)

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
    int rb0 = 0, re0 = 0, rb1 = 0, re1 = 0;
    {
        const RowSet& rs = a.rs[0];
        if (rs.local) {
            rb0 = k0 * gm.G;
            re0 = min(gm.T, k0 + kKeysPerWg + gm.W) * gm.G;
        } else {
            rb0 = rs.kblk_first_row ? rs.kblk_first_row[(size_t)bh * (nkb + 1) + (k0 >> 6)] : k0 * gm.G;
            re0 = rows_total(rs, gm, bh);
        }
    }
    if (a.nsets > 1) {
        const RowSet& rs = a.rs[1];
        if (rs.local) {
            rb1 = k0 * gm.G;
            re1 = min(gm.T, k0 + kKeysPerWg + gm.W) * gm.G;
        } else {
            rb1 = rs.kblk_first_row ? rs.kblk_first_row[(size_t)bh * (nkb + 1) + (k0 >> 6)] : k0 * gm.G;
            re1 = rows_total(rs, gm, bh);
        }
    }
    const int nt0 = re0 > rb0 ? (re0 - rb0 + kRT - 1) / kRT : 0;
    const int nt1 = re1 > rb1 ? (re1 - rb1 + kRT - 1) / kRT : 0;
    const int total_tiles = nt0 + nt1;

    const int r4 = (threadIdx.x >> 4) * 4;
    const int c8 = (threadIdx.x & 15) * 8;
    TileRegs qr, gr;
    float st_lse2 = 0.f, st_delta = 0.f;
    int st_pos = -1;
    // tile `it` of the concatenated list -> registers
    auto load_tile = [&](int it) {
        const int s = it < nt0 ? 0 : 1;
        const RowSet& rs = a.rs[s];
        const int rt0 = (s ? rb1 : rb0) + (it - (s ? nt0 : 0)) * kRT;
        const int last = (s ? re1 : re0) - 1;
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
    // registers -> LDS in 16 pieces, so that the pieces can be spread between matrix-core instructions
    auto store_piece = [&](RowTileLds& t, auto ic) {
        constexpr int i = decltype(ic)::value;
        if constexpr (i < 4) {
            *reinterpret_cast<u32x4*>(t.q_rm + (r4 + i) * kRowPad + c8) = qr.x[i];
        } else if constexpr (i < 8) {
            *reinterpret_cast<u32x4*>(t.g_rm + (r4 + i - 4) * kRowPad + c8) = gr.x[i - 4];
        } else {
            const TileRegs& x = i < 12 ? qr : gr;
            __bf16* dst = i < 12 ? t.q_t : t.g_t;
            constexpr int p = i & 3;
            const uint32_t w0 = x.x[0][p], w1 = x.x[1][p], w2 = x.x[2][p], w3 = x.x[3][p];
            u32x2 even = {(w0 & 0xffffu) | (w1 << 16), (w2 & 0xffffu) | (w3 << 16)};
            u32x2 odd = {(w0 >> 16) | (w1 & 0xffff0000u), (w2 >> 16) | (w3 & 0xffff0000u)};
            *reinterpret_cast<u32x2*>(dst + (c8 + 2 * p) * kColPad + r4) = even;
            *reinterpret_cast<u32x2*>(dst + (c8 + 2 * p + 1) * kColPad + r4) = odd;
        }
        if constexpr (i == 0) {
            if (threadIdx.x < kRT) {
                t.lse2[threadIdx.x] = st_lse2;
                t.delta[threadIdx.x] = st_delta;
                t.pos[threadIdx.x] = st_pos;
            }
        }
    };
    auto store_all = [&](RowTileLds& t) { static_for<0, 16>([&](auto ic) { store_piece(t, ic); }); };

    f32x16 dkacc[4], dvacc[4];
#pragma unroll
    for (int d = 0; d < 4; ++d)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            dkacc[d][r] = 0.f;
            dvacc[d][r] = 0.f;
        }

    // One 64-row tile against this wavefront's 32 keys: 64 matrix-core instructions, issued as 64
    // slots.  Slot m issues instruction m, the LDS read of the operand of instruction m + kAhead,
    // and a share of the VALU / LDS-store work of the neighbouring stages:
    //   slots  0-15  S0, dP0 (rows 0-31)
    //   slots 16-31  S1, dP1 (rows 32-63)   | softmax-backward of rows 0-31
    //   slots 32-47  dV, dK from rows 0-31  | softmax-backward of rows 32-63
    //   slots 48-63  dV, dK from rows 32-63 | next tile: registers -> LDS
    // Only the operands of the next kAhead slots are live, so the register file also holds the
    // wavefront's K/V operands and the 128 accumulator registers.
    auto tile_body = [&](auto mask_tag, const RowTileLds& t, bool local, bool do_store, RowTileLds& tn) {
        constexpr bool MASK = decltype(mask_tag)::value;
        constexpr int kAhead = 4;
        const float c = gm.scale_log2;
        bf16x8 opnd[64 + kAhead];
        f32x4 l2a[4], dla[4], l2b[4], dlb[4];
        i32x4 psa[4], psb[4];
        f32x16 s0, dp0, s1, dp1;
        bf16x8 pT[4], dsT[4];
        // operand of instruction m, read from LDS
        auto read_operand = [&](auto mc) {
            constexpr int m = decltype(mc)::value;
            if constexpr (m < 64) {
                constexpr int i = m & 15, ks = i >> 1;
                if constexpr (m < 32) {
                    const int row = (m < 16 ? 0 : 32) + n;
                    if constexpr (i & 1) opnd[m] = lds_rowmajor(t.g_rm, row, ks, h);
                    else opnd[m] = lds_rowmajor(t.q_rm, row, ks, h);
                } else {
                    constexpr int step = (m - 32) >> 3, d = (i >> 1) & 3;
                    if constexpr (i & 1) opnd[m] = lds_transposed(t.q_t, d * 32 + n, step, h);
                    else opnd[m] = lds_transposed(t.g_t, d * 32 + n, step, h);
                }
            }
        };
        auto issue = [&](auto mc) {
            constexpr int m = decltype(mc)::value;
            constexpr int i = m & 15, ks = i >> 1, d = (i >> 1) & 3;
            if constexpr (m < 16) {
                if constexpr (i & 1) dp0 = mfma32(opnd[m], vreg[ks], dp0);
                else s0 = mfma32(opnd[m], kreg[ks], s0);
            } else if constexpr (m < 32) {
                if constexpr (i & 1) dp1 = mfma32(opnd[m], vreg[ks], dp1);
                else s1 = mfma32(opnd[m], kreg[ks], s1);
            } else {
                constexpr int step = (m - 32) >> 3;
                if constexpr (i & 1) dkacc[d] = mfma32(dsT[step], opnd[m], dkacc[d]);
                else dvacc[d] = mfma32(pT[step], opnd[m], dvacc[d]);
            }
        };
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            s0[r] = 0.f;
            dp0[r] = 0.f;
            s1[r] = 0.f;
            dp1[r] = 0.f;
        }
        static_for<0, kAhead>([&](auto mc) { read_operand(mc); });
        L2A_FENCE();
        static_for<0, 64>([&](auto mc) {
            constexpr int m = decltype(mc)::value;
            issue(mc);
            read_operand(std::integral_constant<int, m + kAhead>{});
            if constexpr (m >= 8 && m < 12) {  // per-row statistics of rows 0-31
                constexpr int rg = m - 8;
                l2a[rg] = *reinterpret_cast<const f32x4*>(&t.lse2[8 * rg + 4 * h]);
                dla[rg] = *reinterpret_cast<const f32x4*>(&t.delta[8 * rg + 4 * h]);
                if (MASK) psa[rg] = *reinterpret_cast<const i32x4*>(&t.pos[8 * rg + 4 * h]);
            }
            if constexpr (m >= 26 && m < 30) {  // ... of rows 32-63
                constexpr int rg = m - 26;
                l2b[rg] = *reinterpret_cast<const f32x4*>(&t.lse2[32 + 8 * rg + 4 * h]);
                dlb[rg] = *reinterpret_cast<const f32x4*>(&t.delta[32 + 8 * rg + 4 * h]);
                if (MASK) psb[rg] = *reinterpret_cast<const i32x4*>(&t.pos[32 + 8 * rg + 4 * h]);
            }
            if constexpr (m >= 16 && m < 32) {
                bwd_softmax_elem<MASK>(m - 16, s0, dp0, l2a, dla, psa, c, key, gm.T, gm.W, local);
                if constexpr (m == 31) {
                    pT[0] = pack8(s0, 0);
                    pT[1] = pack8(s0, 1);
                    dsT[0] = pack8(dp0, 0);
                    dsT[1] = pack8(dp0, 1);
                }
            } else if constexpr (m >= 32 && m < 48) {
                bwd_softmax_elem<MASK>(m - 32, s1, dp1, l2b, dlb, psb, c, key, gm.T, gm.W, local);
                if constexpr (m == 47) {
                    pT[2] = pack8(s1, 0);
                    pT[3] = pack8(s1, 1);
                    dsT[2] = pack8(dp1, 0);
                    dsT[3] = pack8(dp1, 1);
                }
            } else if constexpr (m >= 48) {
                if (do_store) store_piece(tn, std::integral_constant<int, m - 48>{});
            }
            L2A_FENCE();
        });
    };

    if (total_tiles > 0) {
        load_tile(0);
        store_all(lds[0]);
    }
    __syncthreads();

    // The tiles of a set form three runs: a head whose rows can lie before some key of the block
    // (causal mask), a middle that needs no mask at all, and a tail (sliding-window edge, ragged
    // last tile).  Each run gets its own loop so the common case is straight-line code.
    auto split = [&](const RowSet& rs, int rb, int re, int nt, int& head, int& tail_start) {
        if (nt == 0) {
            head = 0;
            tail_start = 0;
            return;
        }
        const int kend = k0 + kKeysPerWg;  // rows at positions >= kend see every key of the block
        int r_mid;
        if (kend > gm.T)
            r_mid = re;
        else if (rs.local || !rs.kblk_first_row)
            r_mid = kend * gm.G;
        else
            r_mid = rs.kblk_first_row[(size_t)bh * (nkb + 1) + (kend >> 6)];
        head = min(nt, max(0, (r_mid - rb + kRT - 1) / kRT));
        tail_start = ((re - rb) % kRT) ? nt - 1 : nt;
        if (rs.local) {
            const long long r_suf = (long long)(k0 + gm.W + 1) * gm.G;  // first row whose window starts after k0
            if (r_suf < re) tail_start = min(tail_start, (int)((r_suf - rb) / kRT));
        }
        tail_start = max(tail_start, head);
    };
    int head0, tail0, head1, tail1;
    split(a.rs[0], rb0, re0, nt0, head0, tail0);
    split(a.rs[1], rb1, re1, nt1, head1, tail1);

    for (int seg = 0; seg < 6; ++seg) {
        const int set = seg / 3, part = seg - 3 * set;
        const int base = set ? nt0 : 0;
        const int hd = set ? head1 : head0, tl = set ? tail1 : tail0, nt = set ? nt1 : nt0;
        const int it_begin = base + (part == 0 ? 0 : (part == 1 ? hd : tl));
        const int it_end = base + (part == 0 ? hd : (part == 1 ? tl : nt));
        if (it_begin >= it_end) continue;
        const RowSet& rs = a.rs[set];
        const bool local = rs.local != 0;
        const int rbs = set ? rb1 : rb0, res = set ? re1 : re0;
        if (part == 1) {
            for (int it = it_begin; it < it_end; ++it) {
                const int cur = it & 1;
                const bool more = it + 1 < total_tiles;
                if (more) load_tile(it + 1);
                if (kw0 < gm.T) tile_body(std::false_type{}, lds[cur], local, more, lds[cur ^ 1]);
                else if (more) store_all(lds[cur ^ 1]);
                __syncthreads();
            }
        } else {
            for (int it = it_begin; it < it_end; ++it) {
                const int cur = it & 1;
                const bool more = it + 1 < total_tiles;
                if (more) load_tile(it + 1);
                // rows of a tile ascend in position: cheap per-wavefront bounds for skipping
                const int rt0 = rbs + (it - base) * kRT;
                const int rt1 = min(rt0 + kRT, res);
                const int t_pmin = row_code(rs, gm, bh, rt0) / gm.G;
                const int t_pmax = row_code(rs, gm, bh, rt1 - 1) / gm.G;
                bool skip = t_pmax < kw0 || kw0 >= gm.T;
                if (local) skip = skip || (t_pmin - gm.W > kw0 + 31);
                if (!skip) tile_body(std::true_type{}, lds[cur], local, more, lds[cur ^ 1]);
                else if (more) store_all(lds[cur ^ 1]);
                __syncthreads();
            }
        }
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
