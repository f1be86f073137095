// C ABI of the L2A layer: argument checks and the launch sequence of each call.
// Every step of the layer runs in the kernels of this library; nothing here computes.
#include "common.hpp"

#include <cmath>

using namespace l2a;

namespace {

int check_params(const l2a_params* p) {
    if (!p) return L2A_ERR_NULL;
    if (p->B < 1 || p->T < 1 || p->Hq < 1 || p->Hkv < 1 || p->W < 0) return L2A_ERR_SHAPE;
    if (p->Hq % p->Hkv != 0) return L2A_ERR_SHAPE;
    const int G = p->Hq / p->Hkv;
    if (p->mask_heads != 1 && p->mask_heads != p->Hkv && p->mask_heads != p->Hq) return L2A_ERR_SHAPE;
    if ((long long)p->T * G > 0x7fffffffLL) return L2A_ERR_SHAPE;       // row codes pos*G+g are int32
    if ((long long)p->B * p->Hkv > 65535) return L2A_ERR_SHAPE;         // grid.y
    if ((long long)p->B * p->T * p->Hq * p->D > (1LL << 40)) return L2A_ERR_SHAPE;
    if (G > 16) return L2A_ERR_UNSUPPORTED;
    if (p->dtype != L2A_BF16 && p->dtype != L2A_FP32) return L2A_ERR_UNSUPPORTED;
    if (p->D != 64 && p->D != 128) return L2A_ERR_UNSUPPORTED;
    // bf16 runs on the matrix cores, built for D = 128; other head sizes only through the scalar kernels, on request
    if (p->dtype == L2A_BF16 && p->D != 128 && !(p->flags & L2A_FLAG_SCALAR)) return L2A_ERR_UNSUPPORTED;
    if ((p->flags & L2A_FLAG_SKIP_LOCAL) && (p->flags & L2A_FLAG_SKIP_GLOBAL)) return L2A_ERR_UNSUPPORTED;
    if (!(p->softmax_scale > 0.f)) return L2A_ERR_SHAPE;
    return L2A_OK;
}

bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

Geom make_geom(const l2a_params& p) {
    Geom g;
    g.B = p.B; g.T = p.T; g.Hq = p.Hq; g.Hkv = p.Hkv; g.G = p.Hq / p.Hkv; g.D = p.D;
    g.W = p.W < p.T ? p.W : p.T;  // a window reaching past token 0 is the whole prefix
    g.scale = p.softmax_scale;
    g.scale_log2 = p.softmax_scale * kLog2e;
    return g;
}

bool use_mfma(const l2a_params& p) { return p.dtype == L2A_BF16 && p.D == 128 && !(p.flags & L2A_FLAG_SCALAR); }

size_t elem_bytes(const l2a_params& p) { return p.dtype == L2A_BF16 ? 2 : 4; }
size_t q_elems(const l2a_params& p) { return (size_t)p.B * p.T * p.Hq * p.D; }
size_t stat_elems(const l2a_params& p) { return (size_t)p.B * p.Hq * p.T; }

// rows per (b, KV head) of a token-minor copy of K or V
int kv_cap(const l2a_params& p) { return (p.T + 63) / 64 * 64; }
size_t kv_copy_bytes(const l2a_params& p) { return (size_t)p.B * p.Hkv * p.D * kv_cap(p) * 2; }

size_t redo_bytes(const l2a_params& p) {
    const size_t n = mfma_fwd_redo_entries(make_geom(p)) * sizeof(int32_t);
    return (n + 255) / 256 * 256;
}
// Short sequences: the Global rows' tiles alone would leave most compute units idle, so both
// branches go out in one launch and O = S + A is formed afterwards.
constexpr size_t kPairMaxTiles = 2048;  // row tiles of one branch, all (b, KV head) together
bool pair_fwd(const l2a_params& p) {
    const int f = p.flags;
    return use_mfma(p) && !(f & (L2A_FLAG_DENSE | L2A_FLAG_SKIP_LOCAL | L2A_FLAG_SKIP_GLOBAL | L2A_FLAG_SEQUENTIAL)) &&
           mfma_fwd_redo_entries(make_geom(p)) <= kPairMaxTiles;
}
// two token-minor copies of V (one per branch) and the forward kernels' redo flags; short sequences:
// flags for both branches at once and room for A in fp32
size_t fwd_workspace_bytes(const l2a_params& p) {
    if (!use_mfma(p)) return 0;
    if (pair_fwd(p)) return 2 * kv_copy_bytes(p) + 2 * redo_bytes(p) + q_elems(p) * sizeof(float);
    return 2 * kv_copy_bytes(p) + redo_bytes(p);
}
// backward: delta of each branch; matrix-core path: + compact copies of each branch's rows
size_t delta_bytes(const l2a_params& p) { return (sizeof(float) * stat_elems(p) + 255) / 256 * 256; }
// compact copies of a branch's rows for the dK/dV kernel: Q, dO row-major, + 3 statistics
int rows_cap(const l2a_params& p) { return (int)(((long long)p.T * (p.Hq / p.Hkv) + 63) / 64 * 64); }
size_t rows_copy_bytes(const l2a_params& p) { return (size_t)p.B * p.Hkv * rows_cap(p) * p.D * 2; }
size_t rows_stat_bytes(const l2a_params& p) { return ((size_t)p.B * p.Hkv * rows_cap(p) * 4 + 255) / 256 * 256; }
size_t packed_set_bytes(const l2a_params& p) { return 2 * rows_copy_bytes(p) + 3 * rows_stat_bytes(p); }
// short sequences: partial dK, dV sums of the workgroups that share a key block
size_t dkdv_part_bytes(const l2a_params& p) {
    const int z = dkdv_splits(make_geom(p));
    return z > 1 ? (size_t)z * 2 * p.B * p.T * p.Hkv * p.D * sizeof(float) : 0;
}
size_t bwd_workspace_bytes(const l2a_params& p) {
    return 2 * delta_bytes(p) + (use_mfma(p) ? 2 * packed_set_bytes(p) + dkdv_part_bytes(p) : 0);
}



}  // namespace

extern "C" {

int l2a_version(void) { return 1; }

const char* l2a_strerror(int code) {
    switch (code) {
        case L2A_OK: return "ok";
        case L2A_ERR_NULL: return "a required pointer is NULL";
        case L2A_ERR_SHAPE: return "invalid shape, window, mask_heads or scale";
        case L2A_ERR_UNSUPPORTED: return "unsupported dtype / head size / flag or aliasing combination";
        case L2A_ERR_WORKSPACE: return "workspace missing or too small";
        case L2A_ERR_ALIGN: return "a data pointer is not 16-byte aligned";
        case L2A_ERR_LAUNCH: return "the HIP runtime refused a kernel launch";
        case L2A_ERR_STATIC_LIMIT:
            return "problem too large for the library's static scratch (l2a_route_compact_static: more than 65536 "
                   "chunk counters); use the entry point that takes a workspace";
        default: return "unknown error code";
    }
}

int32_t l2a_kblk_entries(int32_t T) { return (T + 63) / 64 + 1; }

size_t l2a_route_workspace_bytes(const l2a_params* p) {
    if (check_params(p) != L2A_OK) return 0;
    if (p->flags & L2A_FLAG_DENSE) return 0;
    return route_workspace_bytes(*p);
}

size_t l2a_attn_workspace_bytes(const l2a_params* p, int backward) {
    if (check_params(p) != L2A_OK) return 0;
    if (!backward) return fwd_workspace_bytes(*p);
    return bwd_workspace_bytes(*p);
}

int l2a_route_compact(const l2a_params* p, const uint8_t* mask, int32_t* row_idx, int32_t* count,
                      int32_t* kblk_first_row, void* workspace, size_t workspace_bytes, void* stream) {
    const int rc = check_params(p);
    if (rc != L2A_OK) return rc;
    if (p->flags & L2A_FLAG_DENSE) return L2A_OK;
    if (!mask || !row_idx || !count || !kblk_first_row) return L2A_ERR_NULL;
    if (!workspace || workspace_bytes < route_workspace_bytes(*p)) return L2A_ERR_WORKSPACE;
    if (misaligned(row_idx) || misaligned(workspace)) return L2A_ERR_ALIGN;
    return route_compact(*p, mask, row_idx, count, kblk_first_row, workspace, (hipStream_t)stream);
}

int l2a_route_compact_static(const l2a_params* p, const uint8_t* mask, int32_t* row_idx, int32_t* count,
                             int32_t* kblk_first_row, void* stream) {
    const int rc = check_params(p);
    if (rc != L2A_OK) return rc;
    if (p->flags & L2A_FLAG_DENSE) return L2A_OK;
    if (!mask || !row_idx || !count || !kblk_first_row) return L2A_ERR_NULL;
    if (misaligned(row_idx)) return L2A_ERR_ALIGN;
    return route_compact_static(*p, mask, row_idx, count, kblk_first_row, (hipStream_t)stream);
}

int l2a_router_decide(const l2a_params* p, int32_t C, const void* x, const float* w, float bias, float tau,
                      float* logit_opt, float* dhat_opt, uint8_t* mask, void* stream) {
    const int rc = check_params(p);
    if (rc != L2A_OK) return rc;
    if (C < 8 || C % 8 != 0 || !(tau > 0.f && tau < 1.f)) return L2A_ERR_SHAPE;
    if (!x || !w || !mask) return L2A_ERR_NULL;
    if (misaligned(x) || misaligned(w)) return L2A_ERR_ALIGN;
    const float thr = (float)std::log((double)tau / (1.0 - (double)tau));
    return router_decide(*p, C, x, w, bias, thr, logit_opt, dhat_opt, mask, (hipStream_t)stream);
}

size_t l2a_decode_workspace_bytes(const l2a_params* p) {
    if (check_params(p) != L2A_OK || !use_mfma(*p)) return 0;
    return decode_partial_floats(make_geom(*p)) * sizeof(float);
}

int l2a_attn_decode(const l2a_params* p, const void* q, const void* k_cache, const void* v_cache, const int32_t* pos,
                    const uint8_t* mask, void* O, float* lse_local, float* lse_global, void* S_opt, void* A_opt,
                    void* workspace, size_t workspace_bytes, void* stream) {
    const int rc = check_params(p);
    if (rc != L2A_OK) return rc;
    if (!use_mfma(*p)) return L2A_ERR_UNSUPPORTED;  // (check_params has already limited Hq / Hkv to 16)
    const bool dense = p->flags & L2A_FLAG_DENSE;
    if (!q || !k_cache || !v_cache || !pos || !O || (!dense && !mask)) return L2A_ERR_NULL;
    const void* ptrs[] = {q, k_cache, v_cache, O, S_opt, A_opt};
    for (const void* x : ptrs)
        if (x && misaligned(x)) return L2A_ERR_ALIGN;
    if (!workspace || workspace_bytes < l2a_decode_workspace_bytes(p)) return L2A_ERR_WORKSPACE;
    if (misaligned(workspace)) return L2A_ERR_ALIGN;
    const int ring = (p->flags & L2A_FLAG_RING_CACHE) ? 1 : 0;
    // a ring serves the Local branch alone, must hold the whole window, and is walked in whole sub-blocks of 32 slots
    if (ring && (!(p->flags & L2A_FLAG_SKIP_GLOBAL) || p->T < p->W + 1 || p->T % 32 != 0)) return L2A_ERR_UNSUPPORTED;
    return mfma_decode(make_geom(*p), q, k_cache, v_cache, pos, dense ? nullptr : mask, p->mask_heads,
                       !(p->flags & L2A_FLAG_SKIP_LOCAL), !(p->flags & L2A_FLAG_SKIP_GLOBAL), ring, (float*)workspace, O,
                       S_opt, A_opt, lse_local, lse_global, (hipStream_t)stream);
}

int l2a_attn_fwd(const l2a_params* p, const void* q_loc, const void* k_loc, const void* v_loc,
                 const void* q_glb, const void* k_glb, const void* v_glb, const int32_t* row_idx,
                 const int32_t* count, const int32_t* kblk_first_row, void* O, float* lse_local,
                 float* lse_global, void* S_opt, void* A_opt, void* workspace, size_t workspace_bytes,
                 void* stream) {
    (void)kblk_first_row;
    const int rc = check_params(p);
    if (rc != L2A_OK) return rc;
    const bool dense = p->flags & L2A_FLAG_DENSE;
    const bool do_local = !(p->flags & L2A_FLAG_SKIP_LOCAL);
    const bool do_global = !(p->flags & L2A_FLAG_SKIP_GLOBAL);
    if (!O) return L2A_ERR_NULL;
    if (do_local && (!q_loc || !k_loc || !v_loc || !lse_local)) return L2A_ERR_NULL;
    if (do_global && (!q_glb || !k_glb || !v_glb || !lse_global)) return L2A_ERR_NULL;
    if (do_global && !dense && (!row_idx || !count)) return L2A_ERR_NULL;
    const void* ptrs[] = {q_loc, k_loc, v_loc, q_glb, k_glb, v_glb, O, S_opt, A_opt};
    for (const void* x : ptrs)
        if (x && misaligned(x)) return L2A_ERR_ALIGN;
    const size_t need = fwd_workspace_bytes(*p);
    if (need && (!workspace || workspace_bytes < need)) return L2A_ERR_WORKSPACE;
    if (need && misaligned(workspace)) return L2A_ERR_ALIGN;

    hipStream_t st = (hipStream_t)stream;
    const Geom g = make_geom(*p);
    const bool mfma = use_mfma(*p);
    int r = L2A_OK;
    // matrix-core path: token-minor copy of each distinct V (layout pre-pass, one pass over V)
    char* vt_loc = (char*)workspace;
    char* vt_glb = vt_loc;
    if (mfma) {
        if (do_local && (r = pack_kv(g, v_loc, vt_loc, kv_cap(*p), st)) != L2A_OK) return r;
        if (do_global && (!do_local || v_glb != v_loc)) {
            vt_glb = (char*)workspace + kv_copy_bytes(*p);
            if ((r = pack_kv(g, v_glb, vt_glb, kv_cap(*p), st)) != L2A_OK) return r;
        }
    }
    if (pair_fwd(*p)) {
        char* after_v = (char*)workspace + 2 * kv_copy_bytes(*p);
        float* A32 = (float*)(after_v + 2 * redo_bytes(*p));
        // tokens the Global branch never visits
        if (A_opt && (r = fill_zero(A_opt, q_elems(*p) * elem_bytes(*p), st)) != L2A_OK) return r;
        if ((r = fill_f32(lse_global, stat_elems(*p), -INFINITY, st)) != L2A_OK) return r;
        const RowSet rs_l{nullptr, nullptr, nullptr, 1};
        const RowSet rs_g{row_idx, count, kblk_first_row, 0};
        const FwdOut out_l{O, S_opt, lse_local, nullptr, nullptr, 0};
        const FwdOut out_g{nullptr, A_opt, lse_global, nullptr, nullptr, 0, A32};
        if ((r = mfma_fwd_pair(g, rs_l, q_loc, k_loc, v_loc, vt_loc, out_l, rs_g, q_glb, k_glb, v_glb, vt_glb, out_g,
                               kv_cap(*p), (int32_t*)after_v, st)) != L2A_OK)
            return r;
        return merge_rows(g, rs_g, A32, O, st);
    }
    auto fwd_branch = [&](const RowSet& rs, const void* q, const void* k, const void* v, const void* vt,
                          const FwdOut& out) {
        int32_t* redo = (int32_t*)((char*)workspace + 2 * kv_copy_bytes(*p));
        return mfma ? mfma_fwd(g, rs, q, k, v, vt, kv_cap(*p), redo, out, st)
                    : simple_fwd(g, p->dtype, rs, q, k, v, out, st);
    };
    if (do_local) {
        const RowSet rs{nullptr, nullptr, nullptr, 1};
        FwdOut out{O, S_opt, lse_local, nullptr, nullptr, 0};
        if (do_global && !dense) {  // tokens the global branch never visits
            out.lse_fill = lse_global;
            out.zero_fill = A_opt;
        }
        if ((r = fwd_branch(rs, q_loc, k_loc, v_loc, vt_loc, out)) != L2A_OK) return r;
    }
    if (do_global) {
        if (!do_local && !dense) {
            if ((r = fill_zero(O, q_elems(*p) * elem_bytes(*p), st)) != L2A_OK) return r;
            if (A_opt && (r = fill_zero(A_opt, q_elems(*p) * elem_bytes(*p), st)) != L2A_OK) return r;
            if ((r = fill_f32(lse_global, stat_elems(*p), -INFINITY, st)) != L2A_OK) return r;
        }
        const RowSet rs = dense ? RowSet{nullptr, nullptr, nullptr, 0} : RowSet{row_idx, count, kblk_first_row, 0};
        const FwdOut out{O, A_opt, lse_global, nullptr, nullptr, do_local ? 1 : 0};
        if ((r = fwd_branch(rs, q_glb, k_glb, v_glb, vt_glb, out)) != L2A_OK) return r;
    }
    return L2A_OK;
}

int l2a_attn_bwd(const l2a_params* p, const void* dO, const void* q_loc, const void* k_loc,
                 const void* v_loc, const void* q_glb, const void* k_glb, const void* v_glb,
                 const int32_t* row_idx, const int32_t* count, const int32_t* kblk_first_row, const void* S,
                 const void* A, const float* lse_local, const float* lse_global, void* dq_loc, void* dk_loc,
                 void* dv_loc, void* dq_glb, void* dk_glb, void* dv_glb, float* delta_glb_opt,
                 void* workspace, size_t workspace_bytes, void* stream) {
    const int rc = check_params(p);
    if (rc != L2A_OK) return rc;
    const bool dense = p->flags & L2A_FLAG_DENSE;
    const bool do_local = !(p->flags & L2A_FLAG_SKIP_LOCAL);
    const bool do_global = !(p->flags & L2A_FLAG_SKIP_GLOBAL);
    if (!dO) return L2A_ERR_NULL;
    if (do_local && (!q_loc || !k_loc || !v_loc || !S || !lse_local || !dq_loc || !dk_loc || !dv_loc))
        return L2A_ERR_NULL;
    if (do_global && (!q_glb || !k_glb || !v_glb || !A || !lse_global || !dq_glb || !dk_glb || !dv_glb))
        return L2A_ERR_NULL;
    if (do_global && !dense && (!row_idx || !count || !kblk_first_row)) return L2A_ERR_NULL;
    if (!workspace || workspace_bytes < l2a_attn_workspace_bytes(p, 1)) return L2A_ERR_WORKSPACE;
    const void* ptrs[] = {dO, q_loc, k_loc, v_loc, q_glb, k_glb, v_glb, S, A, dq_loc, dk_loc, dv_loc,
                          dq_glb, dk_glb, dv_glb, workspace};
    for (const void* x : ptrs)
        if (x && misaligned(x)) return L2A_ERR_ALIGN;

    const bool both = do_local && do_global;
    const bool out_alias = both && dq_glb == dq_loc;
    if (both && ((dk_glb == dk_loc) != out_alias || (dv_glb == dv_loc) != out_alias)) return L2A_ERR_UNSUPPORTED;
    const bool in_alias = both && q_glb == q_loc && k_glb == k_loc && v_glb == v_loc;
    if (out_alias && !in_alias) return L2A_ERR_UNSUPPORTED;  // summed gradients need shared inputs

    hipStream_t st = (hipStream_t)stream;
    const Geom g = make_geom(*p);
    int r;
    float* delta_l = (float*)workspace;
    float* delta_g = delta_glb_opt ? delta_glb_opt : (float*)((char*)workspace + delta_bytes(*p));
    const bool mfma = use_mfma(*p);
    auto bwd_dq = [&](const RowSet& rs, const void* q, const void* k, const void* v, const float* lse, float* delta,
                      void* dq, int acc) {
        return mfma ? mfma_bwd_dq(g, rs, q, k, v, dO, lse, delta, dq, acc, st)
                    : simple_bwd_dq(g, p->dtype, rs, q, k, v, dO, lse, delta, dq, acc, st);
    };
    if ((r = row_deltas(g, p->dtype, dO, do_local ? S : nullptr, do_global ? A : nullptr, delta_l, delta_g, st)) !=
        L2A_OK)
        return r;
    if (p->dtype == L2A_BF16) {  // outputs saved in bf16: the first tokens' deltas come from the definition instead
        if (do_local && (r = head_deltas(g, q_loc, k_loc, v_loc, dO, lse_local, delta_l, 1, st)) != L2A_OK) return r;
        if (do_global && (r = head_deltas(g, q_glb, k_glb, v_glb, dO, lse_global, delta_g, 0, st)) != L2A_OK) return r;
    }

    const RowSet rs_l{nullptr, nullptr, nullptr, 1};
    const RowSet rs_g = dense ? RowSet{nullptr, nullptr, nullptr, 0} : RowSet{row_idx, count, kblk_first_row, 0};

    // dQ: one pass per branch over that branch's rows
    if (do_local && (r = bwd_dq(rs_l, q_loc, k_loc, v_loc, lse_local, delta_l, dq_loc, 0)) != L2A_OK) return r;
    if (do_global) {
        if (!out_alias && !dense && (r = fill_zero(dq_glb, q_elems(*p) * elem_bytes(*p), st)) != L2A_OK) return r;
        if ((r = bwd_dq(rs_g, q_glb, k_glb, v_glb, lse_global, delta_g, dq_glb, out_alias ? 1 : 0)) != L2A_OK)
            return r;
    }
    // dK, dV: one pass over the key tokens; with shared inputs both branches accumulate in registers.
    // The matrix-core kernel reads each branch's rows from compact copies (layout pre-pass).
    char* packed_base = (char*)workspace + 2 * delta_bytes(*p);
    const int cap = rows_cap(*p);
    auto dkdv = [&](const RowSet* sets, int n, const void* const* qs, const float* const* lses,
                    const float* const* deltas, const void* k, const void* v, void* dk, void* dv) -> int {
        if (!mfma) return simple_bwd_dkdv(g, p->dtype, sets, n, qs[0], k, v, dO, lses, deltas, dk, dv, st);
        const void* packed[2][5];
        for (int i = 0; i < n; ++i) {
            char* base = packed_base + (sets[i].local ? 0 : packed_set_bytes(*p));
            char* stat = base + 2 * rows_copy_bytes(*p);
            void* out[5] = {base, base + rows_copy_bytes(*p), stat, stat + rows_stat_bytes(*p),
                            stat + 2 * rows_stat_bytes(*p)};
            const int rc2 = pack_rows(g, sets[i], qs[i], dO, lses[i], deltas[i], out[0], out[1], (float*)out[2],
                                      (float*)out[3], (int32_t*)out[4], cap, st);
            if (rc2 != L2A_OK) return rc2;
            for (int j = 0; j < 5; ++j) packed[i][j] = out[j];
        }
        float* part = dkdv_part_bytes(*p) ? (float*)(packed_base + 2 * packed_set_bytes(*p)) : nullptr;
        return mfma_bwd_dkdv(g, sets, n, packed, cap, k, v, dk, dv, part, st);
    };
    if (out_alias) {
        const RowSet sets[2] = {rs_l, rs_g};
        const void* qs[2] = {q_loc, q_loc};
        const float* lses[2] = {lse_local, lse_global};
        const float* deltas[2] = {delta_l, delta_g};
        return dkdv(sets, 2, qs, lses, deltas, k_loc, v_loc, dk_loc, dv_loc);
    }
    if (do_local) {
        const void* qs[1] = {q_loc};
        const float* lses[1] = {lse_local};
        const float* deltas[1] = {delta_l};
        if ((r = dkdv(&rs_l, 1, qs, lses, deltas, k_loc, v_loc, dk_loc, dv_loc)) != L2A_OK) return r;
    }
    if (do_global) {
        const void* qs[1] = {q_glb};
        const float* lses[1] = {lse_global};
        const float* deltas[1] = {delta_g};
        if ((r = dkdv(&rs_g, 1, qs, lses, deltas, k_glb, v_glb, dk_glb, dv_glb)) != L2A_OK) return r;
    }
    return L2A_OK;
}

}  // extern "C"
