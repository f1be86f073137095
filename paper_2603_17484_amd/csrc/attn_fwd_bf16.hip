// Forward attention kernel, bf16 on the matrix cores (gfx950), for both branches of the layer:
//   GLOBAL rows = compacted routed (position, head-in-group) pairs, keys 0..pos
//          (App. C Alg. 1: tiles of Q_c, causal mask with the original positions Q_idx, K/V tiles
//          beyond the tile's largest position skipped), or all rows in the dense mode;
//   LOCAL  rows = all (position, head) pairs, keys pos-W..pos (Sec. 2 sliding-window mask).
// The epilogue writes the log-sum-exp and merges into O (Sec. 3.1 Eq. 5), so the scatter of
// Alg. 1's last step costs no extra pass.
//
// Work decomposition.  One workgroup = 8 wavefronts of 32 rows = a tile of 256 consecutive rows of
// one (batch, KV head); the rows of the G query heads of the group are interleaved, so every row of
// a tile reads the same K/V.  K and the token-minor copy of V are streamed through LDS in blocks
// of 64 keys by direct global->LDS loads (three and two buffers, one barrier per block).  With 32 rows
// a wavefront needs 256 registers, so two share a SIMD (measured 2-5 % faster than 4 wavefronts of 64
// rows at 500 registers, which the kernel template still covers).
//
// Everything is computed transposed so that a lane owns a query row:
//   S^T[key, row]  = K Q^T     A = K block (LDS), B = Q (registers, loaded once)
//   O^T[ch,  row] += V^T P^T   A = V block (LDS, token-minor), B = P^T = the S^T accumulators
// A lane holds 32 scores of one row per block (the lane 32 apart holds the other 32): row max
// and row sum are in-register reductions plus one cross-lane exchange, and rescaling O is a
// per-lane scalar.
//
// Software pipeline (per wavefront and half-block of 32 keys: 16 matrix-core instructions per 32 rows,
// issued as numbered slots): while half-block j's scores go through the softmax on the VALU, the
// matrix cores first compute half-block j+1's scores and then accumulate P_j V_j (in the order the
// softmax finishes the 16-key groups).  LDS operand reads run a few slots ahead.
#include "tiles.hpp"

namespace l2a {
namespace {

constexpr int kBK = 64;  // keys per block
constexpr int kNQB = 2;  // 32-row blocks per wavefront (fix-up kernel)
constexpr int kFwdNQB = 1, kFwdNW = 8;  // the pipelined kernel's shape: see fwd_kernel
constexpr int kRW = 32 * kNQB;
constexpr int kBQ = 4 * kRW;
constexpr int kAhead = 2;  // operand look-ahead, in operands (each feeds two instructions)

#define L2A_FENCE() __builtin_amdgcn_sched_barrier(0)

struct FwdArgs {
    Geom gm;
    RowSet rs;
    const __bf16* q;
    const __bf16* k;
    const __bf16* v;   // V as given (fix-up kernel only)
    const __bf16* vt;  // token-minor copy of V: [B*Hkv][128][vt_cap]
    int vt_cap;
    int32_t* redo;  // [B*Hkv][width of the branch's grid]: set to 1 for a tile whose rows must be recomputed by the fix-up kernel
    FwdOut out;
};

template <int NQB>
struct ScoresT {
    f32x16 s[NQB];  // 32 keys x (NQB x 32) rows
};

template <int V>
using Int = std::integral_constant<int, V>;

// NW wavefronts of NQB x 32 rows each (NW * NQB = 8): 4 x 2 runs one wavefront per SIMD with 500 registers,
// 8 x 1 runs two per SIMD with 256 each, so that one wavefront's softmax arithmetic can overlap the
// other's matrix instructions.
// (bx, by) of (gx, nbh): the workgroup's index in its branch's part of the grid (a launch may carry both branches)
template <bool LOCAL, int NQB, int NW>
__device__ __forceinline__ void fwd_body(const FwdArgs& a, const int bx, const int by, const int gx, const int nbh,
                                         __bf16 (&lds_k)[3][kBK * 128], __bf16 (&lds_v)[2][kD * kBK]) {
    static_assert(NW * NQB * 32 == kBQ, "a workgroup covers kBQ rows");
    constexpr int RW = 32 * NQB;       // rows per wavefront
    constexpr int NS = 16 * NQB;       // slots (matrix instructions) per half-block: NS / 2 for S, NS / 2 for P V
    constexpr int NL = 16 / NW;        // 16-byte loads a wavefront issues per K or V block
    constexpr int kLoadSlot0 = NS - 1 - 2 * NL;  // the loads of later blocks go out in the last slots of a block's first half
    using Scores = ScoresT<NQB>;

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
    if (by_range) {
        bh = by;
        rank = (bx & 7) * (gx >> 3) + (bx >> 3);
    } else if ((long long)nbh * gm.T <= kAllHeadsMaxTokens) {
        const int lin = by * gx + bx;
        rank = lin / nbh;
        bh = (lin - rank * nbh + rank) % nbh;
    } else {
        bh = by;
        rank = bx;
    }
    const int b = bh / gm.Hkv, hk = bh - b * gm.Hkv;
    const int n_rows = rows_total(a.rs, gm, bh);
    const int n_tiles = (n_rows + kBQ - 1) / kBQ;
    const int tile = by_range ? rank : n_tiles - 1 - rank;
    if (tile < 0 || tile >= n_tiles) return;

    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 31, h = lane >> 5;

    // ---- rows of this workgroup / wavefront / lane
    const int wg_r0 = tile * kBQ;
    const int wg_r1 = min(wg_r0 + kBQ, n_rows);  // exclusive
    const int wg_pmin = row_code(a.rs, gm, bh, wg_r0) / gm.G;
    const int wg_pmax = row_code(a.rs, gm, bh, wg_r1 - 1) / gm.G;
    const int wv_r0 = wg_r0 + wave * RW;
    const bool wave_active = wv_r0 < n_rows;

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

    // ---- block range of the workgroup, and its three runs: blocks that need the window-start
    // mask (LOCAL only), blocks no row of the tile needs a mask for, blocks on the causal diagonal
    const int jb0 = LOCAL ? max(wg_pmin - gm.W, 0) / kBK : 0;
    const int jb1 = wg_pmax / kBK;  // inclusive
    int j_mid = jb0;                // first block without window-start masking
    if (LOCAL) j_mid = min(jb1 + 1, max(jb0, (max(wg_pmax - gm.W, 0) + kBK - 1) / kBK));
    const int j_diag = max(j_mid, min(jb1 + 1, (wg_pmin + 1) / kBK));  // first block with a key > some row

    // Loads: a wave-uniform base per block plus per-lane offsets fixed for the whole kernel.
    const unsigned kv_row_bytes = (unsigned)gm.Hkv * kD * 2;
    const char* kbase = (const char*)(a.k + ((size_t)b * gm.T * gm.Hkv + hk) * kD);
    const char* vtbase = (const char*)(a.vt + (size_t)bh * kD * a.vt_cap);
    const unsigned lds_k0 = lds_offset(&lds_k[0][0]), lds_v0 = lds_offset(&lds_v[0][0]);
    const RmDma<kBK, NW> k_off = rm_dma_setup<kBK, NW>(kv_row_bytes, wave);
    const TmDma<kBK, NW> v_off = tm_dma_setup<kBK, NW>((unsigned)a.vt_cap * 2u, wave);
    auto load_k = [&](int jb, int buf) __attribute__((always_inline)) {
        const char* src = kbase + (size_t)jb * kBK * kv_row_bytes;
        const unsigned dst = lds_k0 + buf * (kBK * 256);
        if ((jb + 1) * kBK <= gm.T) rm_dma_issue(k_off, src, dst, wave);
        else  // keys past the end of the sequence are clamped: always masked, never out of bounds
            rm_dma_issue_clamped<kBK, NW>(kv_row_bytes, gm.T - jb * kBK, src, dst, wave);
    };
    auto load_v = [&](int jb, int buf) __attribute__((always_inline)) {
        tm_dma_issue(v_off, vtbase + (size_t)jb * kBK * 2, lds_v0 + buf * (kD * kBK * 2), wave);
    };
    // In the main loop the 2 NL loads of a block are issued one at a time between matrix
    // instructions.  K rows are clamped to the end of the sequence on the fly (rows past it are always
    // masked), so that the ragged last block needs no code path of its own:
    // lane l of load i fetches chunk (l & 15) ^ (row & 15) of row (NW i + wave) * 4 + (l >> 4).
    const int k_lane_row = wave * 4 + (lane >> 4);
    const unsigned k_lane_chunk = (unsigned)(((lane & 15) ^ (k_lane_row & 15)) * 16);
    struct BlockLoads {
        const char* ksrc;
        const char* vsrc;
        unsigned kdst, vdst;
        int krows;  // rows of the K block that exist
    };
    auto issue_block_load = [&](const BlockLoads& L, auto ic) __attribute__((always_inline)) {
        constexpr int i = decltype(ic)::value;
        if constexpr (i < NL) {
            const unsigned row = (unsigned)min(k_lane_row + 4 * NW * i, L.krows - 1);
            dma16_so(L.ksrc, __umul24(row, kv_row_bytes) + k_lane_chunk, L.kdst + (i * NW + wave) * 1024);
        } else {
            dma16_so(L.vsrc, v_off.voff[i - NL], L.vdst + ((i - NL) * NW + wave) * 1024);
        }
    };

    f32x16 oacc[4][NQB];
    float mref[NQB], negm[NQB], l[NQB];
#pragma unroll
    for (int c = 0; c < NQB; ++c) {
        l[c] = 0.f;
#pragma unroll
        for (int d = 0; d < 4; ++d)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[d][c][r] = 0.f;
    }
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    auto key_ok = [&](int key, int c) __attribute__((always_inline)) {
        bool ok = key <= pos[c];
        if (LOCAL) ok = ok && (key >= pos[c] - gm.W);
        return ok;
    };

    // One half-block (32 keys, half KB of block jb; keys k0 .. k0+31): exp of `cur` against the
    // row's fixed reference, overlapped with the scores of the next half-block into `nxt` (K rows
    // krow0.. of tile kt) and with O += P V for this half-block (tile vt).  32 matrix-core
    // instructions = 32 slots:
    //   first half of the slots   next half-block's scores | exp, row sum, pack P  (pair q in slot 3 q / 2)
    //   second half               O += P V
    auto score = [&](float x) __attribute__((always_inline)) { return NQB == 2 ? acc_read(x) : x; };
    auto half_block = [&](auto mask_tag, auto kb_tag, Scores& cur, Scores& nxt, const __bf16* kt, int krow0,
                          const __bf16* vt, int k0, auto&& side) __attribute__((always_inline)) {
        constexpr bool MASK = decltype(mask_tag)::value;
        constexpr int KB = decltype(kb_tag)::value;
        const float c2 = gm.scale_log2;
        bf16x8 opnd[16 + kAhead];
        uint32_t pw[NQB][2][4];  // P as packed bf16 pairs: [row block][16-key group][dword]
        float rsum[NQB];
        const bf16x2 one2 = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
        for (int c = 0; c < NQB; ++c) rsum[c] = 0.f;
        // operand o: o < 8 -> K rows of the next half-block (ks = o); else V^T (16-key group, channel block)
        auto read_operand = [&](auto oc) {
            constexpr int o = decltype(oc)::value;
            if constexpr (o < 8) opnd[o] = rm_operand(kt, krow0 + n, o, h);
            else if constexpr (o < 16) opnd[o] = tm_operand<kBK>(vt, ((o - 8) & 3) * 32 + n, 2 * KB + ((o - 8) >> 2), h);
        };
        auto issue = [&](auto mc) {
            constexpr int mm = decltype(mc)::value;
            if constexpr (mm < NS / 2) {
                constexpr int ks = mm / NQB, c = mm % NQB;
                nxt.s[c] = mfma32(opnd[ks], qreg[c][ks], ks == 0 ? zero16 : nxt.s[c]);
            } else {
                constexpr int x = mm - NS / 2, grp = x / (4 * NQB), d = (x / NQB) & 3, c = x % NQB;
                const u32x4 pv = {pw[c][grp][0], pw[c][grp][1], pw[c][grp][2], pw[c][grp][3]};
                oacc[d][c] = mfma32(opnd[8 + x / NQB], __builtin_bit_cast(bf16x8, pv), oacc[d][c]);
            }
        };
        // exp of one pair of scores: pair q in 0 .. 8 NQB - 1, in the order the P V product consumes them
        auto exp_pair = [&](auto qc) {
            constexpr int q = decltype(qc)::value;
            constexpr int grp = q / (4 * NQB), c = (q >> 2) % NQB, i2 = (q & 3) * 2, r = grp * 8 + i2;
            float p0 = fast_exp2(fmaf(score(cur.s[c][r]), c2, negm[c]));
            float p1 = fast_exp2(fmaf(score(cur.s[c][r + 1]), c2, negm[c]));
            if (MASK) {
                p0 = key_ok(k0 + c_row(r, h), c) ? p0 : 0.f;
                p1 = key_ok(k0 + c_row(r + 1, h), c) ? p1 : 0.f;
            }
            f32x2 f = {p0, p1};
            const bf16x2 pb = __builtin_convertvector(f, bf16x2);
            pw[c][grp][i2 >> 1] = __builtin_bit_cast(uint32_t, pb);
            // row sum of the weights as the matrix cores will see them (rounded to bf16): one
            // v_dot2 per pair, and the normalisation is exact for the weights actually used
            rsum[c] = __builtin_amdgcn_fdot2_f32_bf16(pb, one2, rsum[c], false);
        };

        static_for<0, kAhead>([&](auto oc) { read_operand(oc); });
        L2A_FENCE();
        static_for<0, NS>([&](auto mc) {
            constexpr int mm = decltype(mc)::value;
            issue(mc);
            if constexpr (mm % NQB == 0) read_operand(Int<mm / NQB + kAhead>{});
            static_for<0, 8 * NQB>([&](auto qc) {
                constexpr int q = decltype(qc)::value;
                if constexpr ((3 * q) / 2 == mm) exp_pair(qc);
            });
            side(mc);
            L2A_FENCE();
        });
#pragma unroll
        for (int c = 0; c < NQB; ++c) l[c] += rsum[c];
        // With more than 256 registers both score buffers stay in AGPRs, where the matrix instructions
        // write them; the VALU side fetches each element with acc_read where it is consumed.
        if constexpr (NQB == 2) asm volatile("" : "+a"(nxt.s[0]), "+a"(nxt.s[1]));
    };

    // ---- prologue: K of the first two blocks, V of the first
    Scores Sa, Sb;
    load_k(jb0, 0);
    if (jb0 < jb1) load_k(jb0 + 1, 1);
    load_v(jb0, 0);
    dma_wait();
    __syncthreads();
    // Reference of every row's exponentials: the largest score among the row's keys in the first
    // two blocks (every row of the tile has a key there).  It is never updated: scores that come
    // later may exceed it, which costs no accuracy in floating point; the epilogue checks that the
    // row sums stayed far from overflow and otherwise leaves the tile to the fix-up kernel.
    {  // wavefronts whose rows all lie past the end compute on a repeated row and store nothing
#pragma unroll
        for (int c = 0; c < NQB; ++c) mref[c] = -INFINITY;
        const int nb = jb0 < jb1 ? 2 : 1;
        for (int bi = 0; bi < nb; ++bi) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                Scores S;
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) {
                    const bf16x8 op = rm_operand(&lds_k[bi][0], kb * 32 + n, ks, h);
#pragma unroll
                    for (int c = 0; c < NQB; ++c) S.s[c] = mfma32(op, qreg[c][ks], ks == 0 ? zero16 : S.s[c]);
                }
#pragma unroll
                for (int c = 0; c < NQB; ++c)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int key = (jb0 + bi) * kBK + kb * 32 + c_row(r, h);
                        mref[c] = fmaxf(mref[c], key_ok(key, c) ? S.s[c][r] : -INFINITY);
                    }
            }
        }
#pragma unroll
        for (int c = 0; c < NQB; ++c) {
            mref[c] = fmaxf(mref[c], __shfl_xor(mref[c], 32)) * gm.scale_log2;
            if (!(mref[c] > -INFINITY)) mref[c] = 0.f;  // no key in reach yet: any finite reference will do
            negm[c] = -mref[c];
        }
        // scores of the first half-block
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const bf16x8 op = rm_operand(&lds_k[0][0], n, ks, h);
#pragma unroll
            for (int c = 0; c < NQB; ++c) Sa.s[c] = mfma32(op, qreg[c][ks], ks == 0 ? zero16 : Sa.s[c]);
        }
    }

    // One block = two half-blocks; Sa holds the scores of a block's first half on entry and exit.
    // K blocks rotate through three buffers: block jb in kbuf, jb+1 in kbuf1, and the block loaded now, jb+2, in kbuf2
    int kbuf = 0, kbuf1 = 1, kbuf2 = 2;
    auto run = [&](auto mask_tag, int j_begin, int j_end) __attribute__((always_inline)) {
        for (int jb = j_begin; jb < j_end; ++jb) {
            const int rel = jb - jb0;
            // prefetch: K of block jb+2 (its buffer held block jb-1), V of block jb+1 (held block jb-1),
            // issued in the slots of the first half-block where the VALU has nothing to do.  Past the
            // last block the last one is loaded again, into buffers nobody reads any more.
            const int jk = min(jb + 2, jb1), jv = min(jb + 1, jb1);
            {  // wavefronts whose rows all lie past the end compute on a repeated row and store nothing
                const __bf16* vt = &lds_v[rel & 1][0];
                BlockLoads L;
                half_block(mask_tag, Int<0>{}, Sa, Sb, &lds_k[kbuf][0], 32, vt, jb * kBK, [&](auto mc) {
                    constexpr int mm = decltype(mc)::value;
                    if constexpr (mm == kLoadSlot0 - 1) {
                        L.ksrc = kbase + (size_t)jk * kBK * kv_row_bytes;
                        L.vsrc = vtbase + (size_t)jv * kBK * 2;
                        L.kdst = lds_k0 + kbuf2 * (kBK * 256);
                        L.vdst = lds_v0 + ((rel + 1) & 1) * (kD * kBK * 2);
                        L.krows = min(kBK, gm.T - jk * kBK);
                    }
                    if constexpr (mm >= kLoadSlot0 && mm < kLoadSlot0 + 2 * NL) issue_block_load(L, Int<mm - kLoadSlot0>{});
                });
                half_block(mask_tag, Int<1>{}, Sb, Sa, &lds_k[kbuf1][0], 0, vt, jb * kBK + 32, [](auto) {});
            }
            dma_wait();
            __syncthreads();
            const int t = kbuf;
            kbuf = kbuf1, kbuf1 = kbuf2, kbuf2 = t;
        }
    };
    // three runs: window-start masks (LOCAL), no masks, causal diagonal
    for (int seg = 0; seg < 3; ++seg) {
        const int j_begin = seg == 0 ? jb0 : (seg == 1 ? j_mid : j_diag);
        const int j_end = seg == 0 ? j_mid : (seg == 1 ? j_diag : jb1 + 1);
        if (seg == 1)
            run(std::false_type{}, j_begin, j_end);
        else
            run(std::true_type{}, j_begin, j_end);
    }

    // ---- did every row sum stay in range, and every accumulator finite?  (workgroup-wide vote; LDS is
    // free after the last barrier.)  A row sum below 1e30 bounds the weights, not the products with V:
    // values beyond ~3e8 can still overflow an accumulator, so those are checked themselves
    // (x * 0 is NaN exactly when x is infinite or NaN).
    float lt[NQB];
    bool bad = false;
#pragma unroll
    for (int c = 0; c < NQB; ++c) {
        lt[c] = l[c] + __shfl_xor(l[c], 32);
        float chk = 0.f;
#pragma unroll
        for (int d = 0; d < 4; ++d)
#pragma unroll
            for (int e = 0; e < 16; ++e) chk = fmaf(oacc[d][c][e], 0.f, chk);
        bad = bad || (wave_active && valid[c] && !(lt[c] > 0.f && lt[c] < 1.0e30f && chk == 0.f));
    }
    int* vote = reinterpret_cast<int*>(&lds_v[0][0]);
    if (threadIdx.x == 0) *vote = 0;
    __syncthreads();
    if (bad) *vote = 1;
    __syncthreads();
    if (*vote) {
        if (threadIdx.x == 0) a.redo[(size_t)bh * gx + tile] = 1;
        return;
    }

    // ---- epilogue: normalise, log-sum-exp, merge / scatter
    if (!wave_active) return;
    __bf16* mo = (__bf16*)a.out.main_out;
    __bf16* co = (__bf16*)a.out.copy_out;
    __bf16* zf = (__bf16*)a.out.zero_fill;
#pragma unroll
    for (int c = 0; c < NQB; ++c) {
        if (!valid[c]) continue;
        const float inv = 1.f / lt[c];
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
                if (a.out.wide_out) *reinterpret_cast<f32x4*>(a.out.wide_out + off) = x;
                else *reinterpret_cast<bf16x4*>(mo + off) = __builtin_convertvector(x, bf16x4);
                if (zf) {
                    const u32x2 z = {0u, 0u};
                    *reinterpret_cast<u32x2*>(zf + off) = z;
                }
            }
        if (h == 0) {
            const size_t so = ((size_t)b * gm.Hq + head[c]) * gm.T + pos[c];
            a.out.lse_out[so] = (mref[c] + __builtin_amdgcn_logf(lt[c])) * kLn2;
            if (a.out.lse_fill) a.out.lse_fill[so] = -INFINITY;
        }
    }
}

template <bool LOCAL, int NQB, int NW>
__global__ __launch_bounds__(64 * NW) void fwd_kernel(FwdArgs a) {
    __shared__ __attribute__((aligned(1024))) __bf16 lds_k[3][kBK * 128];
    __shared__ __attribute__((aligned(1024))) __bf16 lds_v[2][kD * kBK];
    fwd_body<LOCAL, NQB, NW>(a, (int)blockIdx.x, (int)blockIdx.y, (int)gridDim.x, (int)gridDim.y, lds_k, lds_v);
}

// Both branches in one launch, for sequences so short that the Global rows' tiles alone leave most
// compute units idle: the first gx_global workgroups (per b, KV head) take the Global rows' tiles,
// the others the Local rows'.  The branches then must not depend on each other: the Global one
// writes its rows of A only (in fp32, besides the caller's bf16 copy), and O = S + A is formed
// afterwards (merge_rows) with the one rounding the sequential order has.
template <int NQB, int NW>
__global__ __launch_bounds__(64 * NW) void fwd_pair_kernel(FwdArgs ag, FwdArgs al, int gx_global) {
    __shared__ __attribute__((aligned(1024))) __bf16 lds_k[3][kBK * 128];
    __shared__ __attribute__((aligned(1024))) __bf16 lds_v[2][kD * kBK];
    if ((int)blockIdx.x < gx_global)
        fwd_body<false, NQB, NW>(ag, (int)blockIdx.x, (int)blockIdx.y, gx_global, (int)gridDim.y, lds_k, lds_v);
    else
        fwd_body<true, NQB, NW>(al, (int)blockIdx.x - gx_global, (int)blockIdx.y, (int)gridDim.x - gx_global,
                                (int)gridDim.y, lds_k, lds_v);
}

// Fix-up kernel: recomputes the tiles the pipelined kernel gave up on (a later score exceeded a
// row's fixed reference by so much that a row sum left the safe range).  Same tiling, classical
// streaming softmax with a running maximum and rescaling (App. C Alg. 1 as printed, with the
// rescaling factor read as exp(m_old - m_new)); V is transposed on its way into LDS.
template <bool LOCAL>
__global__ __launch_bounds__(kThreads) void fwd_fixup_kernel(FwdArgs a) {
    constexpr int NQB = kNQB;
    constexpr int RW = 32 * NQB;
    constexpr int BQ = 4 * RW;
    __shared__ __attribute__((aligned(16))) __bf16 lds_k[2][kTileRows * kRowPad];
    __shared__ __attribute__((aligned(16))) __bf16 lds_v[2][kD * kColPad];

    const Geom& gm = a.gm;
    const int bh = blockIdx.y, b = bh / gm.Hkv, hk = bh - b * gm.Hkv;
    const int n_rows = rows_total(a.rs, gm, bh);
    const int n_tiles = (n_rows + BQ - 1) / BQ;
    if ((int)blockIdx.x >= n_tiles) return;
    const int tile = n_tiles - 1 - (int)blockIdx.x;
    if (!a.redo[(size_t)bh * gridDim.x + tile]) return;

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
                if (a.out.wide_out) *reinterpret_cast<f32x4*>(a.out.wide_out + off) = x;
                else *reinterpret_cast<bf16x4*>(mo + off) = __builtin_convertvector(x, bf16x4);
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


}  // namespace

int mfma_fwd(const Geom& g, const RowSet& rs, const void* q, const void* k, const void* v, const void* vt,
             int vt_cap, int32_t* redo, const FwdOut& out, hipStream_t st) {
    if (g.D != kD) return L2A_ERR_UNSUPPORTED;
    // per-lane load offsets are 32-bit
    if ((unsigned long long)vt_cap * 2ull * kD > 0xffffffffull) return L2A_ERR_UNSUPPORTED;
    FwdArgs a{g, rs, (const __bf16*)q, (const __bf16*)k, (const __bf16*)v, (const __bf16*)vt, vt_cap, redo, out};
    const long long rows = (long long)g.T * g.G;
    const dim3 grid((unsigned)(((rows + kBQ - 1) / kBQ + 7) / 8 * 8), g.B * g.Hkv);  // a multiple of 8: see the tile order
    int r = fill_zero(redo, sizeof(int32_t) * grid.x * grid.y, st);
    if (r != L2A_OK) return r;
    {
        KernelTimer kt(rs.local ? "fwd_local" : "fwd_global", st);
        if (rs.local)
            hipLaunchKernelGGL((fwd_kernel<true, kFwdNQB, kFwdNW>), grid, dim3(64 * kFwdNW), 0, st, a);
        else
            hipLaunchKernelGGL((fwd_kernel<false, kFwdNQB, kFwdNW>), grid, dim3(64 * kFwdNW), 0, st, a);
    }
    {
        KernelTimer kt(rs.local ? "fwd_local_fixup" : "fwd_global_fixup", st);
        if (rs.local)
            hipLaunchKernelGGL((fwd_fixup_kernel<true>), grid, dim3(kThreads), 0, st, a);
        else
            hipLaunchKernelGGL((fwd_fixup_kernel<false>), grid, dim3(kThreads), 0, st, a);
    }
    return launch_status();
}

// Both branches at once (fwd_pair_kernel): the Global branch's result goes to out_g.wide_out, and
// neither branch may write where the other does.  redo: 2 x mfma_fwd_redo_entries flags.
int mfma_fwd_pair(const Geom& g, const RowSet& rs_l, const void* q_l, const void* k_l, const void* v_l,
                  const void* vt_l, const FwdOut& out_l, const RowSet& rs_g, const void* q_g, const void* k_g,
                  const void* v_g, const void* vt_g, const FwdOut& out_g, int vt_cap, int32_t* redo, hipStream_t st) {
    if (g.D != kD || out_g.merge || !out_g.wide_out || out_l.wide_out) return L2A_ERR_UNSUPPORTED;
    if ((unsigned long long)vt_cap * 2ull * kD > 0xffffffffull) return L2A_ERR_UNSUPPORTED;
    const long long rows = (long long)g.T * g.G;
    const unsigned gx = (unsigned)(((rows + kBQ - 1) / kBQ + 7) / 8 * 8);  // per branch
    const size_t entries = (size_t)gx * g.B * g.Hkv;
    FwdArgs al{g, rs_l, (const __bf16*)q_l, (const __bf16*)k_l, (const __bf16*)v_l, (const __bf16*)vt_l, vt_cap, redo, out_l};
    FwdArgs ag{g, rs_g, (const __bf16*)q_g, (const __bf16*)k_g, (const __bf16*)v_g, (const __bf16*)vt_g, vt_cap,
               redo + entries, out_g};
    int r = fill_zero(redo, sizeof(int32_t) * 2 * entries, st);
    if (r != L2A_OK) return r;
    {
        KernelTimer kt("fwd_pair", st);
        hipLaunchKernelGGL((fwd_pair_kernel<kFwdNQB, kFwdNW>), dim3(2 * gx, g.B * g.Hkv), dim3(64 * kFwdNW), 0, st, ag, al,
                           (int)gx);
    }
    {
        KernelTimer kt("fwd_local_fixup", st);
        hipLaunchKernelGGL((fwd_fixup_kernel<true>), dim3(gx, g.B * g.Hkv), dim3(kThreads), 0, st, al);
    }
    {
        KernelTimer kt("fwd_global_fixup", st);
        hipLaunchKernelGGL((fwd_fixup_kernel<false>), dim3(gx, g.B * g.Hkv), dim3(kThreads), 0, st, ag);
    }
    return launch_status();
}

// number of redo flags mfma_fwd needs
size_t mfma_fwd_redo_entries(const Geom& g) {
    const long long rows = (long long)g.T * g.G;
    return (size_t)(((rows + kBQ - 1) / kBQ + 7) / 8 * 8) * g.B * g.Hkv;
}

}  // namespace l2a
