// Backward kernel for dK and dV, bf16 on the matrix cores (gfx950).  Gradients come only from
// the rows of each branch's row set -- the routed queries for the Global branch (Sec. 3.2).
//     P = exp(scale Q K^T - lse),  dV = P^T dO,  dP = dO V^T,  dS = P o (dP - delta),  dK = scale dS^T Q.
// No atomics, bit-reproducible: one workgroup owns a block of 128 keys (4 wavefronts x 32 keys)
// and streams tiles of 32 rows: first the Local rows that can see the block, then the compacted
// Global rows from kblk_first_row on.  The G heads of a KV group are rows of the same list, so
// the sum over the heads of a group needs no second pass.
//
// Rows are read from the compact row-major copies the pack pre-pass makes of each branch's Q and
// dO, together with the rows' log-sum-exp, -delta and position, by direct global->LDS loads.  One
// tile in LDS serves both orientations: S = Q K^T and dP = dO V^T read its rows, dV += P^T dO and
// dK += dS^T Q read it transposed (ds_read_b64_tr_b16; the tile's chunk permutation keeps both
// kinds of read free of bank conflicts).  The load path into LDS is the scarcer resource (64 B/clk
// per CU against 188 B/clk of LDS reads), so loading a second, token-minor copy of every tile
// costs more than the half-rate transposed reads do.  The dP accumulators start from -delta, so
// that dS = P o dP' needs no subtraction.
//   S  [row, key] = Q K^T     A = Q tile (LDS, rows),        B = K (registers, loaded once)
//   dP [row, key] = dO V^T    A = dO tile,                   B = V (registers)
//   dV [key, ch] += P^T dO    A = P^T  = the S accumulators,  B = dO tile (LDS, transposed reads)
//   dK [key, ch] += dS^T Q    A = dS^T = the dP accumulators, B = Q tile (LDS, transposed reads)
// Software pipeline per tile (32 matrix-core instructions = 32 slots): S, dP of the next tile
// (slots 0-15) and the dV, dK update of this tile (slots 16-31) run on the matrix cores while the
// VALU turns this tile's S, dP into P and dS.
#include "tiles.hpp"
#include "dkdv_walk.hpp"

namespace l2a {
namespace {

using walk::kKeysPerWg;
using walk::kRT;  // rows per tile
constexpr int kAhead = 3;   // operand look-ahead, in slots
constexpr int kNB = 8;              // LDS buffers: loads run kNB - 1 tiles ahead
constexpr int kDmaPerStep = 7;      // direct-to-LDS instructions a wavefront issues per tile step
constexpr int kLoadSlot0 = 1;       // ... in slots kLoadSlot0 + kLoadStride i of a step, i = 0 .. 6
constexpr int kLoadStride = 4;

#define L2A_FENCE() __builtin_amdgcn_sched_barrier(0)

template <int V>
using Int = std::integral_constant<int, V>;

struct PackedRows {   // compact copies of one branch's rows, per (b, kv head): cap rows
    const char* qc;      // [nbh][cap][128] bf16
    const char* gc;      // dO
    const char* lse2;    // [nbh][cap] f32  lse * log2(e)
    const char* ndelta;  // [nbh][cap] f32  -delta
    const char* pos;     // [nbh][cap] i32, -1 = padding
};

struct DkdvArgs {
    Geom gm;
    RowSet rs[2];
    PackedRows rows;        // set 0; every array of set 1 lies set_stride bytes further
    long long set_stride;
    int nsets;
    int cap;
    int chunk;              // key blocks handed to one XCD at a time
    const __bf16* k;
    const __bf16* v;
    __bf16* dk;
    __bf16* dv;
    int nsplit;             // workgroups per key block (grid.z): each takes a share of the row tiles
    float* part;            // nsplit > 1: partial sums [nsplit][2][B, T, Hkv, D] instead of dk, dv
};

struct RowTileLds {
    __bf16 q_rm[kRT * 128];
    __bf16 g_rm[kRT * 128];
    float ndelta[64];  // per-row statistics: 32 used; a whole wavefront writes 64 entries
    float lse2[64];
    int pos[64];
    int pad[64];
};

struct SdP {
    f32x16 s, dp;
};

__global__ __launch_bounds__(kThreads) void bwd_dkdv_kernel(DkdvArgs a) {
    __shared__ __attribute__((aligned(1024))) RowTileLds lds_rm[kNB];

    const Geom& gm = a.gm;
    const int bh = blockIdx.y, b = bh / gm.Hkv, hk = bh - b * gm.Hkv;
    const int kblk = walk::key_block((int)blockIdx.x, a.chunk);  // XCD-aware: chunks of neighbours, snake order
    const int k0 = kblk * kKeysPerWg;
    if (k0 >= a.gm.T) return;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 31, h = lane >> 5;
    const int kw0 = k0 + wave * 32;
    const int key = kw0 + n;  // this lane's key (a column of S)
    const int nkb = (gm.T + 63) / 64;

    // ---- the wavefront's 32 keys stay in registers as B operands
    bf16x8 kreg[8], vreg[8];
    {
        const size_t off = (((size_t)b * gm.T + min(key, gm.T - 1)) * gm.Hkv + hk) * kD + 8 * h;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            kreg[ks] = *reinterpret_cast<const bf16x8*>(a.k + off + ks * 16);
            vreg[ks] = *reinterpret_cast<const bf16x8*>(a.v + off + ks * 16);
        }
    }

    // ---- per set: the 32-row tiles that can see this block of keys, in three runs (causal-masked head,
    // unmasked middle, window / ragged tail), and the order they are walked in (dkdv_walk.hpp)
    auto tile_runs = [&](int s) __attribute__((always_inline)) {
        if (s >= a.nsets) return walk::Runs{0, 0, 0, 0};
        const RowSet& rs = a.rs[s];
        int kind = rs.local ? walk::kLocalRows : walk::kDenseRows, f_lo = 0, f_hi = 0, rows = gm.T * gm.G;
        if (!rs.local && rs.kblk_first_row) {
            const int32_t* first = rs.kblk_first_row + (size_t)bh * (nkb + 1);
            kind = walk::kListRows;
            rows = rows_total(rs, gm, bh);  // clamped like the entries of `first`: device data
            f_lo = first[k0 >> 6];
            f_hi = first[min((k0 + kKeysPerWg) >> 6, nkb)];
        }
        return walk::tile_runs(kind, k0, gm.T, gm.G, gm.W, f_lo, f_hi, rows, a.nsplit, (int)blockIdx.z);
    };
    const walk::Plan plan = walk::make_plan(a.nsets, tile_runs(0), a.rs[0].local != 0, tile_runs(1),
                                            a.nsets > 1 && a.rs[1].local != 0, kblk, a.chunk, gm.T, gm.G, a.set_stride);
    const int total = plan.total;

    // ---- loads.  A cursor names the tile of each step (advanced once per step, branch-free)
    const unsigned lds_rm0 = lds_offset(&lds_rm[0]);
    using Cursor = walk::Cursor;
    auto advance = [&](Cursor& c) __attribute__((always_inline)) { walk::cursor_advance(c, plan); };
    // Every load is a wave-uniform base plus a per-lane offset fixed for the whole kernel.
    const RmDma<kRT> rm_off = rm_tr_dma_setup<kRT>(kD * 2, wave);
    const unsigned stat_off = n * 4;
    const size_t rows_bh = (size_t)bh * a.cap;
    // The 7 loads of a step (the Q and dO rows of a tile, row-major, and three per-row statistics),
    // numbered so that the tile steps can issue them one at a time between matrix instructions.
    struct StepLoads {
        size_t rm256, rm4;  // byte offsets of the tile inside the packed arrays
        unsigned dst_rm;    // LDS buffer
    };
    auto stage_rm = [&](StepLoads& L, long long cset, int ct, int buf) __attribute__((always_inline)) {
        const size_t set = (size_t)cset, row0 = rows_bh + (size_t)ct * kRT;
        L.rm256 = set + row0 * (kD * 2);
        L.rm4 = set + row0 * 4;
        L.dst_rm = __builtin_amdgcn_readfirstlane(lds_rm0 + buf * (unsigned)sizeof(RowTileLds));
    };
    auto issue_load = [&](const StepLoads& L, auto kc) __attribute__((always_inline)) {
        constexpr int k = decltype(kc)::value;
        // per-row statistics (k >= 4): 32 rows, the upper half-wave repeats the lower one (every
        // wavefront issues them, identically, so that all have the same number of loads in flight)
        if constexpr (k < 2) dma16_so(a.rows.qc + L.rm256, rm_off.voff[k], L.dst_rm + (k * 4 + wave) * 1024);
        else if constexpr (k < 4)
            dma16_so(a.rows.gc + L.rm256, rm_off.voff[k - 2], L.dst_rm + kRT * 256 + ((k - 2) * 4 + wave) * 1024);
        else if constexpr (k == 4) dma4_so(a.rows.ndelta + L.rm4, stat_off, L.dst_rm + 2 * kRT * 256);
        else if constexpr (k == 5) dma4_so(a.rows.lse2 + L.rm4, stat_off, L.dst_rm + 2 * kRT * 256 + 256);
        else dma4_so(a.rows.pos + L.rm4, stat_off, L.dst_rm + 2 * kRT * 256 + 512);
    };

    unsigned tr_off[4][2];  // this lane's part of the transposed reads' addresses
#pragma unroll
    for (int d = 0; d < 4; ++d) tr_off[d][0] = rm_tr_col_offset(d, 0, lane), tr_off[d][1] = rm_tr_col_offset(d, 1, lane);
    f32x16 dkacc[4], dvacc[4];
#pragma unroll
    for (int d = 0; d < 4; ++d)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            dkacc[d][e] = 0.f;
            dvacc[d][e] = 0.f;
        }
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

    // One tile: P, dS from `cur` (tile it; its statistics and, read transposed, its rows in ct) overlapped with
    // S, dP of tile it+1 into `nxt` (row-major tiles rt) and the dV, dK update of tile it.
    auto tile_step = [&](auto mask_tag, SdP& cur, SdP& nxt, const RowTileLds& rt, const RowTileLds& ct, bool local,
                         auto&& stage_loads, auto&& loads_issued) __attribute__((always_inline)) {
        StepLoads L;
        constexpr bool MASK = decltype(mask_tag)::value;
        const float c2 = gm.scale_log2;
        lds_cptr trp[4][2];  // this lane's pieces of the transposed reads in tile ct
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            trp[d][0] = (lds_cptr)(uintptr_t)(lds_offset(&ct) + tr_off[d][0]);
            trp[d][1] = (lds_cptr)(uintptr_t)(lds_offset(&ct) + tr_off[d][1]);
        }
        bf16x8 opnd[32 + kAhead];
        uint32_t pw[2][4], dsw[2][4];  // P^T, dS^T as packed bf16 pairs: [16-row group][dword]
        f32x4 l2[4];
        i32x4 ps[4];
        f32x16 nd;  // -delta of the next tile's rows: the dP accumulators start from it
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {  // register 4 rg + e holds row 8 rg + 4 h + e
            l2[rg] = *reinterpret_cast<const f32x4*>(&ct.lse2[8 * rg + 4 * h]);
            const f32x4 x = *reinterpret_cast<const f32x4*>(&rt.ndelta[8 * rg + 4 * h]);
            nd[4 * rg] = x[0], nd[4 * rg + 1] = x[1], nd[4 * rg + 2] = x[2], nd[4 * rg + 3] = x[3];
            if (MASK) ps[rg] = *reinterpret_cast<const i32x4*>(&ct.pos[8 * rg + 4 * h]);
        }
        // operand of slot m: m < 16 -> Q (even) / dO (odd) rows of the next tile, ks = m / 2;
        // else dO (even) / Q (odd) of this tile read transposed: 16-row group (m - 16) / 8, channel block ((m - 16) / 2) % 4
        auto read_operand = [&](auto mc) {
            constexpr int mm = decltype(mc)::value;
            if constexpr (mm < 16) {
                if constexpr ((mm & 1) == 0) opnd[mm] = rm_tr_row_operand(rt.q_rm, n, mm >> 1, h);
                else opnd[mm] = rm_tr_row_operand(rt.g_rm, n, mm >> 1, h);
            } else if constexpr (mm < 32) {
                constexpr int x = mm - 16, step = x >> 3, d = (x >> 1) & 3;
                opnd[mm] = rm_tr_col_operand_at(trp[d][0], trp[d][1], step, (x & 1) == 0 ? kRT * 256 : 0);  // dO / Q tile
            }
        };
        auto issue = [&](auto mc) {
            constexpr int mm = decltype(mc)::value;
            if constexpr (mm < 16) {
                constexpr int ks = mm >> 1;
                if constexpr (ks == 0) {
                    if constexpr ((mm & 1) == 0) mfma32_vgpr_first(nxt.s, opnd[mm], kreg[ks]);
                    else mfma32_vgpr_from(nxt.dp, opnd[mm], vreg[ks], nd);
                } else {
                    if constexpr ((mm & 1) == 0) mfma32_vgpr_acc(nxt.s, opnd[mm], kreg[ks]);
                    else mfma32_vgpr_acc(nxt.dp, opnd[mm], vreg[ks]);
                }
            } else {
                constexpr int x = mm - 16, step = x >> 3, d = (x >> 1) & 3;
                if constexpr ((x & 1) == 0) {
                    const u32x4 pv = {pw[step][0], pw[step][1], pw[step][2], pw[step][3]};
                    dvacc[d] = mfma32(__builtin_bit_cast(bf16x8, pv), opnd[mm], dvacc[d]);
                } else {
                    const u32x4 dv = {dsw[step][0], dsw[step][1], dsw[step][2], dsw[step][3]};
                    dkacc[d] = mfma32(__builtin_bit_cast(bf16x8, dv), opnd[mm], dkacc[d]);
                }
            }
        };
        auto ds_pair = [&](auto qc) {  // pair q in 0..7, in the order the dV / dK products consume them
            constexpr int q = decltype(qc)::value;
            constexpr int step = q >> 2, i2 = (q & 3) * 2, e = step * 8 + i2, rg = e >> 2, el = e & 3;
            float p0 = fast_exp2(fmaf(cur.s[e], c2, -l2[rg][el]));
            float p1 = fast_exp2(fmaf(cur.s[e + 1], c2, -l2[rg][el + 1]));
            if (MASK) {
                const int rp0 = ps[rg][el], rp1 = ps[rg][el + 1];
                bool ok0 = rp0 >= key && key < gm.T, ok1 = rp1 >= key && key < gm.T;
                if (local) {
                    ok0 = ok0 && (rp0 - key <= gm.W);
                    ok1 = ok1 && (rp1 - key <= gm.W);
                }
                p0 = ok0 ? p0 : 0.f;
                p1 = ok1 ? p1 : 0.f;
            }
            f32x2 fp = {p0, p1};
            f32x2 fd = {p0 * cur.dp[e], p1 * cur.dp[e + 1]};  // dp already holds dP - delta
            pw[step][i2 >> 1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(fp, bf16x2));
            dsw[step][i2 >> 1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(fd, bf16x2));
        };

        static_for<0, kAhead>([&](auto mc) { read_operand(mc); });
        L2A_FENCE();
        static_for<0, 32>([&](auto mc) {
            constexpr int mm = decltype(mc)::value;
            issue(mc);
            read_operand(Int<mm + kAhead>{});
            static_for<0, 8>([&](auto qc) {
                constexpr int q = decltype(qc)::value;
                if constexpr ((q * 7) / 4 == mm) ds_pair(qc);
            });
            // the loads of later tiles go out spread over the step
            if constexpr (mm == kLoadSlot0 - 1) stage_loads(L);
            if constexpr (mm >= kLoadSlot0 && (mm - kLoadSlot0) % kLoadStride == 0 &&
                          (mm - kLoadSlot0) / kLoadStride < kDmaPerStep)
                issue_load(L, Int<(mm - kLoadSlot0) / kLoadStride>{});
            if constexpr (mm == kLoadSlot0 + kLoadStride * (kDmaPerStep - 1)) loads_issued();
            L2A_FENCE();
        });
    };

    if (total > 0) {
        // ---- prologue: tiles 0 .. kNB-2; S, dP of tile 0
        SdP Xa, Xb;
        Cursor lc = walk::cursor_begin(plan);
        static_for<0, kNB - 1>([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            StepLoads L;
            stage_rm(L, lc.set, lc.t, i);
            static_for<0, kDmaPerStep>([&](auto kc) { issue_load(L, kc); });
            advance(lc);
        });
        dma_wait();
        __syncthreads();
#pragma unroll
        for (int e = 0; e < 16; ++e) Xa.dp[e] = lds_rm[0].ndelta[c_row(e, h)];
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const bf16x8 qa = rm_tr_row_operand(lds_rm[0].q_rm, n, ks, h), ga = rm_tr_row_operand(lds_rm[0].g_rm, n, ks, h);
            if (ks == 0) mfma32_vgpr_first(Xa.s, qa, kreg[ks]);
            else mfma32_vgpr_acc(Xa.s, qa, kreg[ks]);
            mfma32_vgpr_acc(Xa.dp, ga, vreg[ks]);
        }
        mfma_vgpr_settle();  // the first tile step reads Xa at once

        // Step `it` reads the rows of tile it+1 and tile `it` transposed, and issues the loads of tile
        // it+kNB-1 (into the buffer tile it-1 left one step ago).  At its end only the loads of the last
        // kNB-3 steps may still be in flight: tile it+2 has landed.  Two tiles per trip so that the two
        // S/dP buffers swap roles without copies.
        auto one = [&](auto mask_tag, SdP& cur, SdP& nxt, int it, bool local) __attribute__((always_inline)) {
            static_assert((kNB & (kNB - 1)) == 0, "buffer indices are taken with a mask");
            tile_step(mask_tag, cur, nxt, lds_rm[(it + 1) & (kNB - 1)], lds_rm[it & (kNB - 1)], local,
                      [&](StepLoads& L) __attribute__((always_inline)) {
                          stage_rm(L, lc.set, lc.t, (it + kNB - 1) & (kNB - 1));
                      },
                      [&]() __attribute__((always_inline)) { advance(lc); });
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"((kNB - 3) * kDmaPerStep) : "memory");
            __syncthreads();
        };
        // The two S/dP buffers swap roles every tile; which one holds the current tile is carried
        // across runs in `flip` (no register copies): a leading single step restores the phase,
        // then steps come in pairs.
        bool flip = false;  // false: Xa holds the current tile
        auto run = [&](auto mask_tag, int it_begin, int it_end, bool local) __attribute__((always_inline)) {
            int it = it_begin;
            if (flip && it < it_end) {
                one(mask_tag, Xb, Xa, it, local);
                flip = false;
                ++it;
            }
            for (; it + 1 < it_end; it += 2) {
                one(mask_tag, Xa, Xb, it, local);
                one(mask_tag, Xb, Xa, it + 1, local);
            }
            if (it < it_end) {
                one(mask_tag, Xa, Xb, it, local);
                flip = true;
            }
        };
        // Segments in walking order; inside one the mask flag is constant.
        int it0 = 0;
        walk::for_each_segment(plan, [&](int s, bool masked, int count) __attribute__((always_inline)) {
            const bool local = (s ? a.rs[1].local : a.rs[0].local) != 0;
            if (masked)
                run(std::true_type{}, it0, it0 + count, local);
            else
                run(std::false_type{}, it0, it0 + count, local);
            it0 += count;
        });
        dma_wait();  // the last steps' loads (re-loads of the last tile) must land before the LDS is given up
    }

    // ---- write dK, dV: lane = channel d*32+n, register e = key c_row(e, h)
#pragma unroll
    for (int d = 0; d < 4; ++d)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int kk = kw0 + c_row(e, h);
            if (kk < gm.T) {
                const size_t off = (((size_t)b * gm.T + kk) * gm.Hkv + hk) * kD + d * 32 + n;
                if (a.nsplit > 1) {
                    const size_t elems = (size_t)gm.B * gm.T * gm.Hkv * kD;
                    float* pz = a.part + (size_t)blockIdx.z * 2 * elems;
                    pz[off] = dkacc[d][e] * gm.scale;
                    pz[elems + off] = dvacc[d][e];
                } else {
                    a.dk[off] = (__bf16)(dkacc[d][e] * gm.scale);
                    a.dv[off] = (__bf16)dvacc[d][e];
                }
            }
        }
}

// dk, dv = sum over the splits of their partial sums, rounded once
__global__ __launch_bounds__(kThreads) void dkdv_reduce_kernel(const float* __restrict__ part, int nsplit, size_t elems,
                                                               __bf16* __restrict__ dk, __bf16* __restrict__ dv) {
    const size_t i = ((size_t)blockIdx.x * kThreads + threadIdx.x) * 4;
    if (i >= elems) return;
    __bf16* out = blockIdx.y ? dv : dk;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int z = 0; z < nsplit; ++z)
        acc += *reinterpret_cast<const f32x4*>(part + ((size_t)z * 2 + blockIdx.y) * elems + i);
    *reinterpret_cast<bf16x4*>(out + i) = __builtin_convertvector(acc, bf16x4);
}

}  // namespace

// Workgroups per key block (short sequences share a key block's row tiles between several)
int dkdv_splits(const Geom& g) { return walk::launch_shape(g.T, (long long)g.B * g.Hkv).nsplit; }

// packed[s]: compact copies of set s made by pack_rows (5 pointers in the order of PackedRows).
// With two sets every array of the second must lie the same number of bytes after the first's.
// part: dkdv_splits(g) > 1: room for that many x 2 x (B T Hkv D) floats
int mfma_bwd_dkdv(const Geom& g, const RowSet* sets, int nsets, const void* const (*packed)[5], int cap,
                  const void* k, const void* v, void* dk, void* dv, float* part, hipStream_t st) {
    if (g.D != kD) return L2A_ERR_UNSUPPORTED;
    DkdvArgs a{};
    a.gm = g;
    a.nsets = nsets;
    a.cap = cap;
    for (int i = 0; i < nsets; ++i) a.rs[i] = sets[i];
    a.rows = PackedRows{(const char*)packed[0][0], (const char*)packed[0][1], (const char*)packed[0][2],
                        (const char*)packed[0][3], (const char*)packed[0][4]};
    if (nsets > 1) {
        a.set_stride = (const char*)packed[1][0] - (const char*)packed[0][0];
        for (int j = 1; j < 5; ++j)
            if ((const char*)packed[1][j] - (const char*)packed[0][j] != a.set_stride) return L2A_ERR_SHAPE;
    }
    a.k = (const __bf16*)k;
    a.v = (const __bf16*)v;
    a.dk = (__bf16*)dk;
    a.dv = (__bf16*)dv;
    const walk::LaunchShape shape = walk::launch_shape(g.T, (long long)g.B * g.Hkv);
    a.chunk = shape.chunk;
    a.nsplit = shape.nsplit;
    a.part = part;
    if (a.nsplit > 1 && !part) return L2A_ERR_WORKSPACE;
    const dim3 grid(shape.grid_x, g.B * g.Hkv, a.nsplit);
    {
        KernelTimer kt("bwd_dkdv", st);
        hipLaunchKernelGGL(bwd_dkdv_kernel, grid, dim3(kThreads), 0, st, a);
    }
    if (a.nsplit > 1) {
        const size_t elems = (size_t)g.B * g.T * g.Hkv * kD;
        KernelTimer kt("dkdv_reduce", st);
        hipLaunchKernelGGL(dkdv_reduce_kernel, dim3((unsigned)((elems / 4 + kThreads - 1) / kThreads), 2), dim3(kThreads), 0,
                           st, part, a.nsplit, elems, a.dk, a.dv);
    }
    return launch_status();
}

}  // namespace l2a
