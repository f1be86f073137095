// Backward kernel for dQ, bf16 on the matrix cores (gfx950).  Gradients are taken only for the
// rows of a branch's row set -- the routed queries for the Global branch -- with the saved
// log-sum-exp (Sec. 3.2).  Standard softmax-attention gradient:
//     P = exp(scale Q K^T - lse),  dP = dO V^T,  dS = P o (dP - delta),  dQ = scale dS K.
// The kernel also emits delta_t = sum_j P_tj dP_tj, which equals <dO_t, out_t> without the
// rounding of the saved bf16 output; the dK/dV kernel uses that value.
//
// Same decomposition as the forward: a workgroup owns a tile of consecutive rows (4 wavefronts
// x 32 rows), a lane owns a row, everything is computed transposed:
//   S^T  = K Q^T        A = K block (LDS),            B = Q  (registers)
//   dP^T = V dO^T       A = V block (LDS),            B = dO (registers)
//   dQ^T += K^T dS^T    A = K block read transposed (LDS), B = dS^T = the accumulators above
// K and V stream through LDS by direct global->LDS loads; one K tile serves both orientations
// (ds_read_b64_tr_b16 for the second, with a chunk permutation that keeps both free of bank conflicts).
// Software pipeline per 32 keys (24 matrix-core instructions = 24 slots): the scores of the next
// half-block (slots 0-15) and the dQ update of this one (slots 16-23) run on the matrix cores
// while the VALU turns this half-block's S, dP into dS.
#include "tiles.hpp"

namespace l2a {
namespace {

constexpr int kBK = 64;
constexpr int kRW = 32;        // rows per wavefront
constexpr int kAhead = 3;      // operand look-ahead, in slots

#define L2A_FENCE() __builtin_amdgcn_sched_barrier(0)

template <int V>
using Int = std::integral_constant<int, V>;

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

struct SdP {
    f32x16 s, dp;  // 32 keys x 32 rows each
};

// NW wavefronts of 32 rows per workgroup.  With 8 the register budget is 256 per wavefront and two
// share a SIMD: the loop over unmasked blocks fits without spills and gains 14 %, the masked blocks
// spill -- so the Global rows (a handful of masked blocks out of hundreds per tile) run with 8
// wavefronts and the Local rows (every twentieth block masked) with 4.
template <bool LOCAL, int NW>
__global__ __launch_bounds__(64 * NW) void bwd_dq_kernel(DqArgs a) {
    constexpr int kNW = NW;
    constexpr int kBQ = NW * kRW;            // rows per workgroup
    constexpr int kNL = 16 / NW;             // 16-byte loads a wavefront issues per K, V or K^T block
    constexpr int kLoadSlot0 = 23 - 2 * kNL;  // the loads of later blocks go out in the last slots of a block's first half
    // K and V tiles in one array: a V tile lies a fixed 48 KB behind the K tile of the same buffer, so
    // the reads of both share their per-lane addresses (the distance goes into the offset field)
    __shared__ __attribute__((aligned(1024))) __bf16 lds_kv[2][3][kBK * 128];
    auto& lds_k = lds_kv[0];
    auto& lds_v = lds_kv[1];
    constexpr int kVBehindK = 3 * kBK * 128;  // elements

    const Geom& gm = a.gm;
    // Workgroups are dispatched in the order of their linear index and dealt round-robin to the 8 XCDs
    // (the grid's width is a multiple of 8).  Global rows: longest prefixes first; every tile starts
    // at key block 0, so the tiles resident on an XCD read the same K/V blocks at about the same time
    // whatever their order.  While the K and V of all heads together about fit the last-level cache, the
    // order runs over all (b, KV head) together (rotated, so that no XCD is tied to one head) -- with
    // a few hundred tiles in all, a head whose long tiles started last would set the kernel's time;
    // beyond that the heads go one after the other, so that the chip streams one head's K and V at a time.
    // Local rows: each XCD takes a contiguous range of a head's tiles, so that the tiles resident on it
    // have overlapping windows and share their K/V blocks through its L2 -- when the sequence is
    // several windows long, so that the ranges cost the same; otherwise the tiles' costs grow with
    // their position like the Global ones' and they are ordered the same way.
    int bh, rank;
    const bool by_range = LOCAL && gm.T / 4 > gm.W;
    const int nbh = gridDim.y;
    if (by_range) {
        bh = blockIdx.y;
        rank = ((int)blockIdx.x & 7) * ((int)gridDim.x >> 3) + ((int)blockIdx.x >> 3);
    } else if ((long long)nbh * gm.T <= kAllHeadsMaxTokens) {
        const int lin = (int)(blockIdx.y * gridDim.x + blockIdx.x);
        rank = lin / nbh;
        bh = (lin - rank * nbh + rank) % nbh;
    } else {
        bh = blockIdx.y;
        rank = blockIdx.x;
    }
    const int b = bh / gm.Hkv, hk = bh - b * gm.Hkv;
    const int n_rows = rows_total(a.rs, gm, bh);
    const int n_tiles = (n_rows + kBQ - 1) / kBQ;
    const int tile = by_range ? rank : n_tiles - 1 - rank;
    if (tile < 0 || tile >= n_tiles) return;

    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 31, h = lane >> 5;

    const int wg_r0 = tile * kBQ;
    const int wg_r1 = min(wg_r0 + kBQ, n_rows);
    const int wg_pmin = row_code(a.rs, gm, bh, wg_r0) / gm.G;
    const int wg_pmax = row_code(a.rs, gm, bh, wg_r1 - 1) / gm.G;
    const int wv_r0 = wg_r0 + wave * kRW;
    const bool wave_active = wv_r0 < n_rows;

    // ---- this lane's row: Q and dO stay in registers as B operands
    const int r = wv_r0 + n;
    const bool valid = r < n_rows;
    const int code = row_code(a.rs, gm, bh, min(r, n_rows - 1));  // rows past the end repeat the last one
    const int pos = code / gm.G;
    const int head = hk * gm.G + (code - pos * gm.G);
    const size_t row_off = (((size_t)b * gm.T + pos) * gm.Hq + head) * kD;
    const size_t so = ((size_t)b * gm.Hq + head) * gm.T + pos;
    bf16x8 qreg[8], greg[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
        qreg[ks] = *reinterpret_cast<const bf16x8*>(a.q + row_off + 8 * h + ks * 16);
        greg[ks] = *reinterpret_cast<const bf16x8*>(a.dO + row_off + 8 * h + ks * 16);
    }
    const float neg_lse2 = -a.lse[so] * kLog2e;
    // The dP accumulators start from -delta (delta = <dO, saved out>), so dS = P o dP' needs no
    // subtraction, and since every row's P sums to one, sum_j dS_j = (sum_j P dP) - delta: the
    // exact delta is the saved one plus the row sum of dS.
    const float dlt = a.delta[so];
    f32x16 ndl16;
#pragma unroll
    for (int e = 0; e < 16; ++e) ndl16[e] = -dlt;
    float dlt_exact = 0.f;

    // ---- block range and its three runs (window-start masks / no masks / causal diagonal)
    const int jb0 = LOCAL ? max(wg_pmin - gm.W, 0) / kBK : 0;
    const int jb1 = wg_pmax / kBK;
    int j_mid = jb0;
    if (LOCAL) j_mid = min(jb1 + 1, max(jb0, (max(wg_pmax - gm.W, 0) + kBK - 1) / kBK));
    const int j_diag = max(j_mid, min(jb1 + 1, (wg_pmin + 1) / kBK));

    // Loads: a wave-uniform base per block plus per-lane offsets fixed for the whole kernel.
    const unsigned kv_row_bytes = (unsigned)gm.Hkv * kD * 2;
    const size_t kv_head = ((size_t)b * gm.T * gm.Hkv + hk) * kD;
    const char* kbase = (const char*)(a.k + kv_head);
    const char* vbase = (const char*)(a.v + kv_head);
    const unsigned lds_k0 = lds_offset(&lds_k[0][0]), lds_v0 = lds_offset(&lds_v[0][0]);
    const RmDma<kBK, kNW> kv_off = rm_tr_dma_setup<kBK, kNW>(kv_row_bytes, wave);
    auto load_kv = [&](int jb, int buf) __attribute__((always_inline)) {
        const size_t src = (size_t)jb * kBK * kv_row_bytes;
        const unsigned dk_ = lds_k0 + buf * (kBK * 256), dv_ = lds_v0 + buf * (kBK * 256);
        if ((jb + 1) * kBK <= gm.T) {
            rm_dma_issue(kv_off, kbase + src, dk_, wave);
            rm_dma_issue(kv_off, vbase + src, dv_, wave);
        } else {  // keys past the end of the sequence are clamped: always masked, never out of bounds
            rm_dma_issue_clamped<kBK, kNW, true>(kv_row_bytes, gm.T - jb * kBK, kbase + src, dk_, wave);
            rm_dma_issue_clamped<kBK, kNW, true>(kv_row_bytes, gm.T - jb * kBK, vbase + src, dv_, wave);
        }
    };
    // In the main loop the loads of a block are issued one at a time between matrix instructions.
    // K and V rows are clamped to the end of the sequence on the fly (rows past it are always masked),
    // so that the ragged last block needs no code path of its own: lane l of load j fetches chunk
    // (l & 15) ^ rm_tr_swizzle(row) of row (NW j + wave) * 4 + (l >> 4); the permutation depends on
    // row & 15 only, which j does not change.
    const int k_lane_row = wave * 4 + (lane >> 4);
    const unsigned k_lane_chunk = (unsigned)(((lane & 15) ^ rm_tr_swizzle(k_lane_row)) * 16);
    struct BlockLoads {
        const char* ksrc;
        const char* vsrc;
        unsigned kdst, vdst;
        int krows;  // rows of the K, V block that exist
    };
    unsigned tr_off[4][2];  // this lane's part of the transposed reads' addresses
#pragma unroll
    for (int d = 0; d < 4; ++d) tr_off[d][0] = rm_tr_col_offset(d, 0, lane), tr_off[d][1] = rm_tr_col_offset(d, 1, lane);
    auto issue_block_load = [&](const BlockLoads& L, auto ic) __attribute__((always_inline)) {
        constexpr int i = decltype(ic)::value;
        constexpr int j = i % kNL;
        const unsigned row = (unsigned)min(k_lane_row + 4 * kNW * j, L.krows - 1);
        const unsigned voff = __umul24(row, kv_row_bytes) + k_lane_chunk;
        if constexpr (i < kNL) dma16_so(L.ksrc, voff, L.kdst + (j * kNW + wave) * 1024);
        else dma16_so(L.vsrc, voff, L.vdst + (j * kNW + wave) * 1024);
    };

    f32x16 acc[4];
#pragma unroll
    for (int d = 0; d < 4; ++d)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[d][e] = 0.f;
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

    // One half-block (32 keys k0..k0+31, half KB of its block): dS from `cur`, overlapped with S, dP
    // of the next half-block into `nxt` (rows krow0.. of K tile kt_ and the V tile behind it) and dQ += K^T dS (this block's K tile through trp).
    auto half_block = [&](auto mask_tag, auto kb_tag, SdP& cur, SdP& nxt, const __bf16* kt_,
                          int krow0, const lds_cptr (&trp)[4][2], int k0, auto&& side) __attribute__((always_inline)) {
        constexpr bool MASK = decltype(mask_tag)::value;
        constexpr int KB = decltype(kb_tag)::value;
        const float c2 = gm.scale_log2;
        bf16x8 opnd[24 + kAhead];
        uint32_t dsw[2][4];  // dS as packed bf16 pairs: [16-key group][dword]
        float dsum = 0.f;
        // operand of slot m: m < 16 -> K (even) / V (odd) rows of the next half-block, ks = m / 2;
        // else this block's K read transposed: (16-key group, channel block)
        auto read_operand = [&](auto mc) {
            constexpr int mm = decltype(mc)::value;
            if constexpr (mm < 16) {
                if constexpr ((mm & 1) == 0) opnd[mm] = rm_tr_row_operand(kt_, krow0 + n, mm >> 1, h);
                else opnd[mm] = rm_tr_row_operand(kt_ + kVBehindK, krow0 + n, mm >> 1, h);
            } else if constexpr (mm < 24) {  // this block's K tile read transposed: channel block, 16-key group
                constexpr int d = (mm - 16) & 3;
                opnd[mm] = rm_tr_col_operand_at(trp[d][0], trp[d][1], 2 * KB + ((mm - 16) >> 2), 0);
            }
        };
        auto issue = [&](auto mc) {
            constexpr int mm = decltype(mc)::value;
            if constexpr (mm < 16) {
                constexpr int ks = mm >> 1;
                if constexpr (ks == 0) {
                    if constexpr ((mm & 1) == 0) mfma32_vgpr_first(nxt.s, opnd[mm], qreg[ks]);
                    else mfma32_vgpr_from(nxt.dp, opnd[mm], greg[ks], ndl16);
                } else {
                    if constexpr ((mm & 1) == 0) mfma32_vgpr_acc(nxt.s, opnd[mm], qreg[ks]);
                    else mfma32_vgpr_acc(nxt.dp, opnd[mm], greg[ks]);
                }
            } else {
                constexpr int x = mm - 16, grp = x >> 2, d = x & 3;
                const u32x4 dv = {dsw[grp][0], dsw[grp][1], dsw[grp][2], dsw[grp][3]};
                acc[d] = mfma32(opnd[mm], __builtin_bit_cast(bf16x8, dv), acc[d]);
            }
        };
        auto ds_pair = [&](auto qc) {  // pair q in 0..7, in the order the dQ product consumes them
            constexpr int q = decltype(qc)::value;
            constexpr int grp = q >> 2, i2 = (q & 3) * 2, e = grp * 8 + i2;
            float p0 = fast_exp2(fmaf(cur.s[e], c2, neg_lse2));
            float p1 = fast_exp2(fmaf(cur.s[e + 1], c2, neg_lse2));
            if (MASK) {
                const int key0 = k0 + c_row(e, h), key1 = k0 + c_row(e + 1, h);
                bool ok0 = key0 <= pos, ok1 = key1 <= pos;
                if (LOCAL) {
                    ok0 = ok0 && (key0 >= pos - gm.W);
                    ok1 = ok1 && (key1 >= pos - gm.W);
                }
                p0 = ok0 ? p0 : 0.f;
                p1 = ok1 ? p1 : 0.f;
            }
            const float dp0 = cur.dp[e], dp1 = cur.dp[e + 1];
            f32x2 f = {p0 * dp0, p1 * dp1};  // dp already holds dP - delta
            dsum += f[0] + f[1];
            dsw[grp][i2 >> 1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
        };

        static_for<0, kAhead>([&](auto mc) { read_operand(mc); });
        L2A_FENCE();
        static_for<0, 24>([&](auto mc) {
            constexpr int mm = decltype(mc)::value;
            // Two wavefronts share a SIMD (the Global rows' shape): each is at high priority through the slots
            // that carry its S, dP instructions and the softmax arithmetic, so that the other's dQ slots fill the
            // gaps (Global rows -3.5 %; the same in the forward kernel changed nothing).
            if constexpr (mm == 0) __builtin_amdgcn_s_setprio(3);
            if constexpr (mm == 16) __builtin_amdgcn_s_setprio(0);
            issue(mc);
            read_operand(Int<mm + kAhead>{});
            static_for<0, 8>([&](auto qc) {
                constexpr int q = decltype(qc)::value;
                if constexpr ((q * 7) / 4 == mm) ds_pair(qc);
            });
            side(mc);
            L2A_FENCE();
        });
        dlt_exact += dsum;
    };

    // ---- prologue: K, V of the first two blocks; S, dP of the first half-block
    SdP Xa, Xb;
    load_kv(jb0, 0);
    if (jb0 < jb1) load_kv(jb0 + 1, 1);
    dma_wait();
    __syncthreads();
    {  // wavefronts whose rows all lie past the end compute on a repeated row and store nothing
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const bf16x8 ka = rm_tr_row_operand(&lds_k[0][0], n, ks, h), va = rm_tr_row_operand(&lds_v[0][0], n, ks, h);
            if (ks == 0) {
                mfma32_vgpr_first(Xa.s, ka, qreg[ks]);
                mfma32_vgpr_from(Xa.dp, va, greg[ks], ndl16);
            } else {
                mfma32_vgpr_acc(Xa.s, ka, qreg[ks]);
                mfma32_vgpr_acc(Xa.dp, va, greg[ks]);
            }
        }
        mfma_vgpr_settle();  // the first half-block reads Xa at once
    }

    // K, V blocks rotate through three buffers: block jb in buf, jb+1 in buf1, and the block loaded now, jb+2, in buf2
    int buf = 0, buf1 = 1, buf2 = 2;
    auto run = [&](auto mask_tag, int j_begin, int j_end) __attribute__((always_inline)) {
        for (int jb = j_begin; jb < j_end; ++jb) {
            // prefetch: K, V of block jb+2 (their buffer held block jb-1), issued in the slots of the first
            // half-block where the VALU has nothing to do.  Past the last block the last one is loaded again, into buffers nobody reads any more.
            const int jk = min(jb + 2, jb1);
            {  // wavefronts whose rows all lie past the end compute on a repeated row and store nothing
                // this block's K, read transposed for dQ += dS K: this lane's pieces of the reads, for both half-blocks
                lds_cptr trp[4][2];
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    trp[d][0] = (lds_cptr)(uintptr_t)(lds_offset(&lds_k[buf][0]) + tr_off[d][0]);
                    trp[d][1] = (lds_cptr)(uintptr_t)(lds_offset(&lds_k[buf][0]) + tr_off[d][1]);
                }
                BlockLoads L;
                half_block(mask_tag, Int<0>{}, Xa, Xb, &lds_k[buf][0], 32, trp, jb * kBK, [&](auto mc) {
                    constexpr int mm = decltype(mc)::value;
                    if constexpr (mm == kLoadSlot0 - 1) {
                        const size_t src = (size_t)jk * kBK * kv_row_bytes;
                        L.ksrc = kbase + src;
                        L.vsrc = vbase + src;
                        L.kdst = lds_k0 + buf2 * (kBK * 256);
                        L.vdst = lds_v0 + buf2 * (kBK * 256);
                        L.krows = min(kBK, gm.T - jk * kBK);
                    }
                    if constexpr (mm >= kLoadSlot0 && mm < kLoadSlot0 + 2 * kNL) issue_block_load(L, Int<mm - kLoadSlot0>{});
                });
                half_block(mask_tag, Int<1>{}, Xb, Xa, &lds_k[buf1][0], 0, trp, jb * kBK + 32,
                           [](auto) {});
            }
            dma_wait();
            __syncthreads();
            const int t = buf;
            buf = buf1, buf1 = buf2, buf2 = t;
        }
    };
    for (int seg = 0; seg < 3; ++seg) {
        const int j_begin = seg == 0 ? jb0 : (seg == 1 ? j_mid : j_diag);
        const int j_end = seg == 0 ? j_mid : (seg == 1 ? j_diag : jb1 + 1);
        if (seg == 1)
            run(std::false_type{}, j_begin, j_end);
        else
            run(std::true_type{}, j_begin, j_end);
    }

    // ---- epilogue
    if (!wave_active) return;
    const float de = dlt + dlt_exact + __shfl_xor(dlt_exact, 32);
    if (!valid) return;
#pragma unroll
    for (int d = 0; d < 4; ++d)
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
            const size_t off = row_off + 4 * h + d * 32 + 8 * rg;
            f32x4 x = {acc[d][4 * rg + 0] * gm.scale, acc[d][4 * rg + 1] * gm.scale, acc[d][4 * rg + 2] * gm.scale,
                       acc[d][4 * rg + 3] * gm.scale};
            if (a.accumulate) {
                const bf16x4 old = *reinterpret_cast<const bf16x4*>(a.dq + off);
                x += __builtin_convertvector(old, f32x4);
            }
            *reinterpret_cast<bf16x4*>(a.dq + off) = __builtin_convertvector(x, bf16x4);
        }
    if (h == 0) a.delta[so] = de;
}

}  // namespace

int mfma_bwd_dq(const Geom& g, const RowSet& rs, const void* q, const void* k, const void* v, const void* dO,
                const float* lse, float* delta, void* dq, int accumulate, hipStream_t st) {
    if (g.D != kD) return L2A_ERR_UNSUPPORTED;
    // per-lane load offsets are 32-bit: 64 rows of K or V
    if (64ull * g.Hkv * kD * 2ull > 0xffffffffull) return L2A_ERR_UNSUPPORTED;
    DqArgs a{g, rs, (const __bf16*)q, (const __bf16*)k, (const __bf16*)v, (const __bf16*)dO, lse, delta,
             (__bf16*)dq, accumulate};
    const long long rows = (long long)g.T * g.G;
    constexpr int kNwLocal = 4, kNwGlobal = 8;
    const int bq = (rs.local ? kNwLocal : kNwGlobal) * kRW;
    const dim3 grid((unsigned)(((rows + bq - 1) / bq + 7) / 8 * 8), g.B * g.Hkv);  // a multiple of 8: see the tile order
    KernelTimer kt_(rs.local ? "bwd_dq_local" : "bwd_dq_global", st);
    if (rs.local)
        hipLaunchKernelGGL((bwd_dq_kernel<true, kNwLocal>), grid, dim3(64 * kNwLocal), 0, st, a);
    else
        hipLaunchKernelGGL((bwd_dq_kernel<false, kNwGlobal>), grid, dim3(64 * kNwGlobal), 0, st, a);
    return launch_status();
}

}  // namespace l2a
