// Shared declarations of the L2A HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/l2a.h"

namespace l2a {

// Problem geometry handed to every kernel.
struct Geom {
    int B, T, Hq, Hkv, G, D, W;
    float scale;       // softmax scale
    float scale_log2;  // scale * log2(e)
};

// One branch of the layer as a kernel sees it.
//   LOCAL : rows are all (pos, g) pairs in identity order, keys pos-W..pos
//   GLOBAL: rows come from row_idx (or identity when dense), keys 0..pos
struct RowSet {
    const int32_t* row_idx;  // [B,Hkv,T*G] or nullptr = identity (dense / local)
    const int32_t* count;    // [B,Hkv]     or nullptr = T*G rows
    const int32_t* kblk_first_row;  // [B,Hkv,ceil(T/64)+1] or nullptr (identity: 64*k*G)
    int local;               // 1: sliding-window branch
};

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

inline int launch_status() { return hipGetLastError() == hipSuccess ? L2A_OK : L2A_ERR_LAUNCH; }

// Optional per-kernel timing (l2a_profile_enable / l2a_profile_read): when enabled, a KernelTimer
// around a launch records a HIP event on the launch stream before and after it.
bool profile_begin(const char* name, hipStream_t st);  // true: a record was opened (and must be closed)
void profile_end(hipStream_t st);
struct KernelTimer {
    hipStream_t st;
    bool open;
    KernelTimer(const char* name, hipStream_t s) : st(s), open(profile_begin(name, s)) {}
    ~KernelTimer() {
        if (open) profile_end(st);
    }
};

// ---- route_compact.hip
size_t route_workspace_bytes(const l2a_params& p);
int route_compact(const l2a_params& p, const uint8_t* mask, int32_t* row_idx, int32_t* count,
                  int32_t* kblk_first_row, void* ws, hipStream_t st);
// the same with the chunk counts in the library's static device array
int route_compact_static(const l2a_params& p, const uint8_t* mask, int32_t* row_idx, int32_t* count,
                         int32_t* kblk_first_row, hipStream_t st);

// A forward branch kernel computes x = attention(row) for every row of `rs` and then
//   main_out[row] = merge ? main_out[row] + x : x      (O)
//   copy_out[row] = x                                   (S_opt / A_opt, optional)
//   lse_out[row]  = log-sum-exp
//   lse_fill[row] = -inf, zero_fill[row] = 0            (optional: what the other branch leaves
//                                                        for tokens it never visits)
struct FwdOut {
    void* main_out;
    void* copy_out;
    float* lse_out;
    float* lse_fill;
    void* zero_fill;
    int merge;
    float* wide_out = nullptr;  // matrix-core kernels: the result goes here in fp32 instead of to main_out
};

// ---- attn_simple.hip : straightforward scalar-FMA kernels (fp32 arithmetic, any element type)
int simple_fwd(const Geom& g, int dtype, const RowSet& rs, const void* q, const void* k, const void* v,
               const FwdOut& out, hipStream_t st);
int simple_bwd_dq(const Geom& g, int dtype, const RowSet& rs, const void* q, const void* k, const void* v,
                  const void* dO, const float* lse, float* delta, void* dq, int accumulate, hipStream_t st);
// dk, dv of every key token; `sets` (1 or 2 row sets: local and/or global) accumulate into the same outputs
int simple_bwd_dkdv(const Geom& g, int dtype, const RowSet* sets, int nsets, const void* q, const void* k,
                    const void* v, const void* dO, const float* const* lse, const float* const* delta, void* dk,
                    void* dv, hipStream_t st);

// ---- router.hip : logit = <w, x_t> + bias; mask = [logit >= thr]; optional sigmoid score and logit
int router_decide(const l2a_params& p, int C, const void* x, const float* w, float bias, float thr, float* logit,
                  float* dhat, uint8_t* mask, hipStream_t st);

// ---- util.hip
int row_deltas(const Geom& g, int dtype, const void* dO, const void* S, const void* A, float* delta_l,
               float* delta_g, hipStream_t st);
// bf16: delta of the first 64 tokens of every sequence recomputed from its definition (one branch)
int head_deltas(const Geom& g, const void* q, const void* k, const void* v, const void* dO, const float* lse,
                float* delta, int local, hipStream_t st);
int fill_zero(void* ptr, size_t bytes, hipStream_t st);
int fill_f32(float* ptr, size_t n, float value, hipStream_t st);

// ---- attn_fwd_bf16.hip / attn_bwd_bf16.hip : MFMA kernels (bf16, D = 128)
// vt: token-minor copy of v from pack_kv, [B*Hkv][128][vt_cap]
// redo: mfma_fwd_redo_entries(g) int32 of scratch
int mfma_fwd(const Geom& g, const RowSet& rs, const void* q, const void* k, const void* v, const void* vt,
             int vt_cap, int32_t* redo, const FwdOut& out, hipStream_t st);
size_t mfma_fwd_redo_entries(const Geom& g);
// both branches in one launch; out_g must not merge; redo: 2 x mfma_fwd_redo_entries(g) int32
int mfma_fwd_pair(const Geom& g, const RowSet& rs_l, const void* q_l, const void* k_l, const void* v_l,
                  const void* vt_l, const FwdOut& out_l, const RowSet& rs_g, const void* q_g, const void* k_g,
                  const void* v_g, const void* vt_g, const FwdOut& out_g, int vt_cap, int32_t* redo, hipStream_t st);

// ---- attn_decode_bf16.hip : one new token per sequence against the KV cache (bf16, D = 128)
size_t decode_partial_floats(const Geom& g);
int mfma_decode(const Geom& g, const void* q, const void* k, const void* v, const int32_t* pos, const uint8_t* mask,
                int mask_heads, int do_local, int do_global, int ring, float* part, void* O, void* S, void* A, float* lse_l,
                float* lse_g, hipStream_t st);

// ---- pack.hip : layout pre-passes (token-minor copies for the matrix-core kernels)
int pack_kv(const Geom& g, const void* x, void* xt, int cap, hipStream_t st);
// O += A on the rows of rs (O bf16, A fp32, D = 128)
int merge_rows(const Geom& g, const RowSet& rs, const float* A, void* O, hipStream_t st);
int pack_rows(const Geom& g, const RowSet& rs, const void* q, const void* dO, const float* lse, const float* delta,
              void* qc, void* gc, float* lse2_c, float* delta_c, int32_t* pos_c, int cap, hipStream_t st);
int mfma_bwd_dq(const Geom& g, const RowSet& rs, const void* q, const void* k, const void* v, const void* dO,
                const float* lse, float* delta, void* dq, int accumulate, hipStream_t st);
// packed[s]: the five outputs of pack_rows for set s (qc, gc, lse2_c, delta_c, pos_c)
// part: scratch for dkdv_splits(g) x 2 x (B T Hkv D) floats when dkdv_splits(g) > 1 (short sequences)
int dkdv_splits(const Geom& g);
int mfma_bwd_dkdv(const Geom& g, const RowSet* sets, int nsets, const void* const (*packed)[5], int cap,
                  const void* k, const void* v, void* dk, void* dv, float* part, hipStream_t st);

}  // namespace l2a
