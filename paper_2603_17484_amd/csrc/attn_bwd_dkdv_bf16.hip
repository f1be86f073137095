// Backward kernel for dK and dV, bf16 on the matrix cores (gfx950), two wavefronts per SIMD.
// Gradients come only from the rows of each branch's row set -- the routed queries for the Global
// branch (Sec. 3.2):
//     P = exp(scale Q K^T - lse),  dV = P^T dO,  dP = dO V^T,  dS = P o (dP - delta),  dK = scale dS^T Q.
// No atomics, bit-reproducible: a workgroup owns a block of 128 keys and streams tiles of 32 rows,
// first the Local rows that can see the block, then the compacted Global rows (the walk is the one
// of dkdv_walk.hpp).  The G heads of a KV group are rows of the same list, so the sum over the heads
// of a group needs no second pass.
//
// Eight wavefronts in two roles, so that each needs half the accumulators and two fit a SIMD (one
// wavefront's softmax arithmetic and LDS reads then run beside the other's matrix instructions):
//   wavefronts 0-3, one per 32 keys:  S = Q K^T (K in registers),  P = exp2(c S - lse'),  dV += P^T dO
//   wavefronts 4-7, the same keys:    dP = dO V^T - delta (V in registers),  dS = P o dP,  dK += dS^T Q
// P passes from the first to the second through LDS as packed bf16 -- the very operand registers of
// the P^T dO product, 2 KB per wavefront and tile -- and the second role runs one tile behind the
// first, so that one barrier per tile step serves the tile buffers and the hand-over alike.
//
// Rows are read from the compact row-major copies the pack pre-pass makes of each branch's Q and dO,
// together with the rows' log-sum-exp, -delta and position, by direct global->LDS loads issued by the
// second role's wavefronts.  One tile in LDS serves both orientations: the products over the channels
// read its rows, the products over the rows read it transposed (ds_read_b64_tr_b16; the tile's chunk
// permutation keeps both kinds of read free of bank conflicts).
#include "tiles.hpp"
#include "dkdv_walk.hpp"

namespace l2a {
namespace {

using walk::kKeysPerWg;
using walk::kRT;  // rows per tile
constexpr int kPairWaves = 8;
constexpr int kAhead = 3;           // operand look-ahead, in slots
constexpr int kNB = 8;              // LDS tile buffers
constexpr int kLook = kNB - 2;      // loads run kLook tiles ahead: a tile is read during two steps
constexpr int kDmaPerStep = 7;      // direct-to-LDS instructions a loading wavefront issues per tile step
constexpr int kLoadSlot0 = 1;       // ... in slots kLoadSlot0 + kLoadStride i of a step, i = 0 .. 6
constexpr int kLoadStride = 2;
constexpr int kSlots = 16;          // matrix instructions per wavefront and tile step

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

struct PairArgs {
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

__global__ __launch_bounds__(64 * kPairWaves) void bwd_dkdv_kernel(PairArgs a) {
    __shared__ __attribute__((aligned(1024))) RowTileLds lds_rm[kNB];
    // P^T of one tile as the first role packs it: [tile parity][key wavefront][16-row group][lane] x 16 bytes
    __shared__ __attribute__((aligned(16))) u32x4 lds_p[2][4][2][64];

    const Geom& gm = a.gm;
    const int bh = blockIdx.y, b = bh / gm.Hkv, hk = bh - b * gm.Hkv;
    const int kblk = walk::key_block((int)blockIdx.x, a.chunk);  // XCD-aware: chunks of neighbours, snake order
    const int k0 = kblk * kKeysPerWg;
    if (k0 >= a.gm.T) return;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int kw = wave & 3;          // which 32 keys
    const bool second = wave >= 4;    // role: dP, dS, dK (else S, P, dV)
    const int n = lane & 31, h = lane >> 5;
    const int kw0 = k0 + kw * 32;
    const int key = kw0 + n;  // this lane's key (a column of S)
    const int nkb = (gm.T + 63) / 64;

    // ---- the wavefront's 32 keys stay in registers as B operands: K for the first role, V for the second
    bf16x8 breg[8];
    {
        const __bf16* src = second ? a.v : a.k;
        const size_t off = (((size_t)b * gm.T + min(key, gm.T - 1)) * gm.Hkv + hk) * kD + 8 * h;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) breg[ks] = *reinterpret_cast<const bf16x8*>(src + off + ks * 16);
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

    // ---- loads (second role).  A cursor names the tile of each step (advanced once per step, branch-free);
    // every load is a wave-uniform base plus a per-lane offset fixed for the whole kernel.
    const unsigned lds_rm0 = lds_offset(&lds_rm[0]);
    using Cursor = walk::Cursor;
    const RmDma<kRT> rm_off = rm_tr_dma_setup<kRT>(kD * 2, kw);
    const unsigned stat_off = n * 4;
    const size_t rows_bh = (size_t)bh * a.cap;
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
    // The 7 loads of a step: the Q and dO rows of a tile (two instructions each: a loading wavefront takes a
    // quarter of each) and three per-row statistics (every loading wavefront issues them, identically, so
    // that all have the same number of loads in flight).
    auto issue_load = [&](const StepLoads& L, auto kc) __attribute__((always_inline)) {
        constexpr int k = decltype(kc)::value;
        if constexpr (k < 2) dma16_so(a.rows.qc + L.rm256, rm_off.voff[k], L.dst_rm + (k * 4 + kw) * 1024);
        else if constexpr (k < 4)
            dma16_so(a.rows.gc + L.rm256, rm_off.voff[k - 2], L.dst_rm + kRT * 256 + ((k - 2) * 4 + kw) * 1024);
        else if constexpr (k == 4) dma4_so(a.rows.ndelta + L.rm4, stat_off, L.dst_rm + 2 * kRT * 256);
        else if constexpr (k == 5) dma4_so(a.rows.lse2 + L.rm4, stat_off, L.dst_rm + 2 * kRT * 256 + 256);
        else dma4_so(a.rows.pos + L.rm4, stat_off, L.dst_rm + 2 * kRT * 256 + 512);
    };

    unsigned tr_off[4][2];  // this lane's part of the transposed reads' addresses
#pragma unroll
    for (int d = 0; d < 4; ++d) tr_off[d][0] = rm_tr_col_offset(d, 0, lane), tr_off[d][1] = rm_tr_col_offset(d, 1, lane);
    f32x16 acc[4];  // dV (first role) or dK (second role): lane = channel d*32+n, register e = key c_row(e, h)
#pragma unroll
    for (int d = 0; d < 4; ++d)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[d][e] = 0.f;

    // One tile step of a wavefront: 8 matrix instructions for X = S (first role) or dP (second) of tile
    // `rt`, under which the VALU turns an earlier tile's X into the packed operand P^T or dS^T, then
    // 8 that add that operand's product with the transposed tile `ct` to the accumulators.
    //   first role : xcur = S of tile `ct`, its statistics in ct; P^T goes to the accumulators' product
    //                and, packed, to `xp` for the second role
    //   second role: xcur = dP of tile `ct` (one step behind the first role), P^T of that tile from `xp`
    auto tile_step = [&](auto role_tag, auto mask_tag, const f32x16& xcur, f32x16& xnxt, const RowTileLds& rt,
                         const RowTileLds& ct, u32x4* xp, bool local, auto&& stage_loads,
                         auto&& loads_issued) __attribute__((always_inline)) {
        constexpr bool SECOND = decltype(role_tag)::value;
        constexpr bool MASK = decltype(mask_tag)::value;
        StepLoads L;
        const float c2 = gm.scale_log2;
        lds_cptr trp[4][2];  // this lane's pieces of the transposed reads in tile ct
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            trp[d][0] = (lds_cptr)(uintptr_t)(lds_offset(&ct) + tr_off[d][0]);
            trp[d][1] = (lds_cptr)(uintptr_t)(lds_offset(&ct) + tr_off[d][1]);
        }
        bf16x8 opnd[kSlots + kAhead];
        uint32_t pk[2][4];  // P^T or dS^T as packed bf16 pairs: [16-row group][dword]
        f32x4 l2[4];
        i32x4 ps[4];
        f32x16 nd;     // second role: -delta of the next tile's rows, the start value of its dP
        u32x4 pin[2];  // second role: P^T of tile ct as the first role packed it
        if constexpr (SECOND) {
            pin[0] = xp[lane];
            pin[1] = xp[64 + lane];
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {  // register 4 rg + e holds row 8 rg + 4 h + e
                const f32x4 x = *reinterpret_cast<const f32x4*>(&rt.ndelta[8 * rg + 4 * h]);
                nd[4 * rg] = x[0], nd[4 * rg + 1] = x[1], nd[4 * rg + 2] = x[2], nd[4 * rg + 3] = x[3];
            }
        } else {
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                l2[rg] = *reinterpret_cast<const f32x4*>(&ct.lse2[8 * rg + 4 * h]);
                if (MASK) ps[rg] = *reinterpret_cast<const i32x4*>(&ct.pos[8 * rg + 4 * h]);
            }
        }
        // slots 0-7: k-step m of the X tile (rows of tile rt: Q for the first role, dO for the second); slots 8-15: the
        // product (16-row group (m - 8) / 4, channel block (m - 8) % 4) with tile ct read transposed (dO / Q)
        auto is_x = [](int m) constexpr { return m < 8; };
        auto read_operand = [&](auto mc) {
            constexpr int mm = decltype(mc)::value;
            if constexpr (mm < kSlots) {
                constexpr int idx = mm & 7;
                if constexpr (is_x(mm)) {
                    opnd[mm] = rm_tr_row_operand(SECOND ? rt.g_rm : rt.q_rm, n, idx, h);
                } else {
                    constexpr int step = idx >> 2, d = idx & 3;
                    opnd[mm] = rm_tr_col_operand_at(trp[d][0], trp[d][1], step, SECOND ? 0 : kRT * 256);
                }
            }
        };
        auto issue = [&](auto mc) {
            constexpr int mm = decltype(mc)::value;
            constexpr int idx = mm & 7;
            if constexpr (is_x(mm)) {
                if constexpr (idx == 0) {
                    if constexpr (SECOND) mfma32_vgpr_from(xnxt, opnd[mm], breg[idx], nd);
                    else mfma32_vgpr_first(xnxt, opnd[mm], breg[idx]);
                } else {
                    mfma32_vgpr_acc(xnxt, opnd[mm], breg[idx]);
                }
            } else {
                constexpr int step = idx >> 2, d = idx & 3;
                const u32x4 pv = {pk[step][0], pk[step][1], pk[step][2], pk[step][3]};
                acc[d] = mfma32(__builtin_bit_cast(bf16x8, pv), opnd[mm], acc[d]);
            }
        };
        auto pair = [&](auto qc) {  // pair q in 0..7, in the order the accumulating products consume them
            constexpr int q = decltype(qc)::value;
            constexpr int step = q >> 2, i2 = (q & 3) * 2, e = step * 8 + i2, rg = e >> 2, el = e & 3;
            f32x2 f;
            if constexpr (SECOND) {
                const uint32_t w = pin[step][i2 >> 1];
                const float p0 = __builtin_bit_cast(float, w << 16), p1 = __builtin_bit_cast(float, w & 0xffff0000u);
                f = f32x2{p0 * xcur[e], p1 * xcur[e + 1]};  // dP already holds dP - delta
            } else {
                float p0 = fast_exp2(fmaf(xcur[e], c2, -l2[rg][el]));
                float p1 = fast_exp2(fmaf(xcur[e + 1], c2, -l2[rg][el + 1]));
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
                f = f32x2{p0, p1};
            }
            pk[step][i2 >> 1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
            if constexpr (!SECOND && (q & 3) == 3) {  // a 16-row group of P^T is complete: hand it over
                const u32x4 pv = {pk[step][0], pk[step][1], pk[step][2], pk[step][3]};
                xp[step * 64 + lane] = pv;
            }
        };

        static_for<0, kAhead>([&](auto mc) { read_operand(mc); });
        L2A_FENCE();
        static_for<0, kSlots>([&](auto mc) {
            constexpr int mm = decltype(mc)::value;
            // Both wavefronts of a SIMD take turns by priority: high while a wavefront is in the half of its step
            // that carries its VALU work, so that the other's accumulating half fills the gaps (measured: -2 %).
            if constexpr (mm == 0) __builtin_amdgcn_s_setprio(3);
            if constexpr (mm == 8) __builtin_amdgcn_s_setprio(0);
            issue(mc);
            read_operand(Int<mm + kAhead>{});
            if constexpr (is_x(mm)) pair(Int<(mm & 7)>{});
            if constexpr (SECOND) {  // the loads of later tiles go out spread over the step
                if constexpr (mm == kLoadSlot0 - 1) stage_loads(L);
                if constexpr (mm >= kLoadSlot0 && (mm - kLoadSlot0) % kLoadStride == 0 &&
                              (mm - kLoadSlot0) / kLoadStride < kDmaPerStep)
                    issue_load(L, Int<(mm - kLoadSlot0) / kLoadStride>{});
                if constexpr (mm == kLoadSlot0 + kLoadStride * (kDmaPerStep - 1)) loads_issued();
            }
            L2A_FENCE();
        });
    };

    if (total > 0) {
        static_assert((kNB & (kNB - 1)) == 0, "buffer indices are taken with a mask");
        auto buf = [&](int i) -> RowTileLds& { return lds_rm[i & (kNB - 1)]; };
        // ---- prologue.  Tiles 0 .. kLook-1 are loaded; the buffer the second role's first step reads as
        // "tile -1" and the P^T it pairs with are zeroed (0 x garbage could be NaN), so that step needs no
        // special case; X of tile 0 is computed.
        Cursor lc = walk::cursor_begin(plan);
        if (second) {
            static_for<0, kLook>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                StepLoads L;
                stage_rm(L, lc.set, lc.t, i);
                static_for<0, kDmaPerStep>([&](auto kc) { issue_load(L, kc); });
                walk::cursor_advance(lc, plan);
            });
        }
        {
            const u32x4 z = {0u, 0u, 0u, 0u};
            reinterpret_cast<u32x4*>(buf(-1).q_rm)[threadIdx.x] = z;  // 512 threads x 16 bytes = the 8 KB tile
            if (threadIdx.x < 256) (&lds_p[1][0][0][0])[threadIdx.x * 2] = z, (&lds_p[1][0][0][0])[threadIdx.x * 2 + 1] = z;
        }
        dma_wait();
        __syncthreads();
        // (each role declares its own X tiles inside its branch: merged variables made the compiler copy
        // them right behind the matrix instructions that write them)
        // At the end of a step only the loads of the last kLook - 2 steps may still be in flight: the tile
        // whose rows the next step reads has landed.
        auto step_end = [&]() __attribute__((always_inline)) {
            if (second) asm volatile("s_waitcnt vmcnt(%0)" ::"n"((kLook - 2) * kDmaPerStep) : "memory");
            __syncthreads();
        };
        if (!second) {
            // ---- first role: steps 0 .. total-1, S buffers swapping roles every step; which one holds the
            // current tile is carried across segments in `flip`.  Step i: S of tile i+1, P and dV of tile i.
            f32x16 X0, X1;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {   // S of tile 0
                const bf16x8 ra = rm_tr_row_operand(lds_rm[0].q_rm, n, ks, h);
                if (ks == 0) mfma32_vgpr_first(X0, ra, breg[ks]);
                else mfma32_vgpr_acc(X0, ra, breg[ks]);
            }
            mfma_vgpr_settle();  // the first tile step reads X0 at once
            auto one = [&](auto mask_tag, const f32x16& cur, f32x16& nxt, int i, bool local) __attribute__((always_inline)) {
                tile_step(std::false_type{}, mask_tag, cur, nxt, buf(i + 1), buf(i), &lds_p[i & 1][kw][0][0], local,
                          [](StepLoads&) {}, []() {});
                step_end();
            };
            bool flip = false;  // false: X0 holds the current tile
            auto run = [&](auto mask_tag, int it_begin, int it_end, bool local) __attribute__((always_inline)) {
                int it = it_begin;
                if (flip && it < it_end) {
                    one(mask_tag, X1, X0, it, local);
                    flip = false;
                    ++it;
                }
                for (; it + 1 < it_end; it += 2) {
                    one(mask_tag, X0, X1, it, local);
                    one(mask_tag, X1, X0, it + 1, local);
                }
                if (it < it_end) {
                    one(mask_tag, X0, X1, it, local);
                    flip = true;
                }
            };
            int it0 = 0;
            walk::for_each_segment(plan, [&](int s, bool masked, int count) __attribute__((always_inline)) {
                const bool local = (s ? a.rs[1].local : a.rs[0].local) != 0;
                if (masked)
                    run(std::true_type{}, it0, it0 + count, local);
                else
                    run(std::false_type{}, it0, it0 + count, local);
                it0 += count;
            });
            __syncthreads();  // the second role's last step
        } else {
            // ---- second role: steps 0 .. total.  Step i: dP of tile i+1 (kept for two steps: three buffers in
            // rotation), dS and dK of tile i-1, the loads of tile i+kLook.  Step 0 pairs the zeroed P^T with the
            // zeroed tile; past the last tile the cursor stays on it, so every step finds finite data.
            f32x16 X0, X1, X2;
#pragma unroll
            for (int e = 0; e < 16; ++e) X0[e] = 0.f, X1[e] = lds_rm[0].ndelta[c_row(e, h)];
#pragma unroll
            for (int ks = 0; ks < 8; ++ks)   // dP of tile 0, from -delta
                mfma32_vgpr_acc(X1, rm_tr_row_operand(lds_rm[0].g_rm, n, ks, h), breg[ks]);
            mfma_vgpr_settle();
            auto one = [&](const f32x16& cur, f32x16& nxt, int i) __attribute__((always_inline)) {
                tile_step(std::true_type{}, std::false_type{}, cur, nxt, buf(i + 1), buf(i - 1), &lds_p[(i - 1) & 1][kw][0][0],
                          false,
                          [&](StepLoads& L) __attribute__((always_inline)) { stage_rm(L, lc.set, lc.t, (i + kLook) & (kNB - 1)); },
                          [&]() __attribute__((always_inline)) { walk::cursor_advance(lc, plan); });
                step_end();
            };
            const int steps = total + 1;   // the last tile's dK is added one step after the first role's last step
            int i = 0;
            for (; i + 3 <= steps; i += 3) {
                one(X0, X2, i);
                one(X1, X0, i + 1);
                one(X2, X1, i + 2);
            }
            if (i < steps) one(X0, X2, i++);
            if (i < steps) one(X1, X0, i++);
            dma_wait();  // the last steps' loads (re-loads of the last tile) must land before the LDS is given up
        }
    }

    // ---- write dV (first role) or dK (second role): lane = channel d*32+n, register e = key c_row(e, h)
    const float out_scale = second ? gm.scale : 1.f;
#pragma unroll
    for (int d = 0; d < 4; ++d)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int kk = kw0 + c_row(e, h);
            if (kk < gm.T) {
                const size_t off = (((size_t)b * gm.T + kk) * gm.Hkv + hk) * kD + d * 32 + n;
                if (a.nsplit > 1) {
                    const size_t elems = (size_t)gm.B * gm.T * gm.Hkv * kD;
                    float* pz = a.part + (size_t)blockIdx.z * 2 * elems + (second ? 0 : elems);
                    pz[off] = acc[d][e] * out_scale;
                } else {
                    (second ? a.dk : a.dv)[off] = (__bf16)(acc[d][e] * out_scale);
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
    PairArgs a{};
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
        hipLaunchKernelGGL(bwd_dkdv_kernel, grid, dim3(64 * kPairWaves), 0, st, a);
    }
    if (a.nsplit > 1) {
        const size_t elems = (size_t)g.B * g.T * g.Hkv * kD;
        KernelTimer kt("dkdv_reduce", st);
        hipLaunchKernelGGL(dkdv_reduce_kernel, dim3((unsigned)((elems / 4 + kThreads - 1) / kThreads), 2), dim3(kThreads),
                           0, st, part, a.nsplit, elems, a.dk, a.dv);
    }
    return launch_status();
}

}  // namespace l2a
