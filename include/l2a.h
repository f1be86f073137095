/*
 * l2a.h -- C ABI of the L2A token-wise conditional attention layer for MI355X (gfx950).
 *
 * The layer (paper Sec. 3.1): every token takes causal sliding-window (Local) attention
 *     s_t = softmax_j( scale <q_t, k_j> : 0 <= t - j <= W ) v_j            (Sec. 2, window mask)
 * and only tokens whose router decision d_t = 1 also take full-prefix causal (Global) attention
 *     a_t = softmax_j( scale <q_t, k_j> : j <= t ) v_j   if d_t = 1, else 0 (Sec. 2 Eq. Attn; Sec. 3.1 Eq. 4)
 * merged additively
 *     o_t = s_t + d_t a_t                                                    (Sec. 3.1 Eq. 5).
 * The window holds the token itself and the W tokens before it (W + 1 keys).
 *
 * How it is computed (Sec. 3.2; App. C Alg. 1): the routed queries are compacted into dense
 * tiles with their original positions kept (Q_idx); a tiled online-softmax kernel runs over
 * those tiles only, masks with the original positions, and skips K/V tiles beyond a tile's
 * largest position; outputs are scattered back.  The backward pass visits the routed
 * queries only, reusing the saved log-sum-exp and Q_idx.
 *
 * General conventions
 *   - Every pointer is a DEVICE pointer owned by the caller unless it is the l2a_params
 *     struct (host).  The library allocates no device memory and keeps no state between calls; all work is enqueued
 *     on the caller's stream (`stream` is a hipStream_t passed as void*; NULL = default
 *     stream) and no call synchronises with the host.
 *   - Tensors are contiguous, row-major:  q, O, dO, dq, S, A : [B, T, Hq, D];
 *     k, v, dk, dv : [B, T, Hkv, D];  lse_* : [B, Hq, T] float.  Element type is bf16
 *     (L2A_BF16, fp32 accumulation, D = 128; D = 64 only together with L2A_FLAG_SCALAR, otherwise
 *     L2A_ERR_UNSUPPORTED) or float (L2A_FP32, D = 64 or 128).  There are no stride arguments: the
 *     kernels fill their LDS tiles with direct global->LDS loads whose per-lane offsets are fixed
 *     for the whole kernel from these row sizes, and the pre-passes that would absorb another
 *     layout are exactly the copies a caller with strided views would otherwise make itself.
 *   - Hq / Hkv <= 16.
 *   - Grouped-query attention: query head h reads KV head h / G, G = Hq / Hkv.
 *   - Log-sum-exp values are natural logs of sum_j exp(scale <q,k_j>).
 *   - Return value: 0 on success, a negative L2A_ERR_* otherwise.  On an argument error
 *     nothing is launched and no output is touched.
 *   - Data pointers must be 16-byte aligned.
 */
#ifndef L2A_H_
#define L2A_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { L2A_BF16 = 0, L2A_FP32 = 1 };

enum {
    L2A_FLAG_DENSE = 1,       /* every token is routed (d = 1 everywhere): the in-house dense causal
                                 FlashAttention-style mode; mask and index arrays are ignored, may be NULL */
    L2A_FLAG_SKIP_LOCAL = 2,  /* run the Global branch only:  O = d a  */
    L2A_FLAG_SKIP_GLOBAL = 4, /* run the Local branch only:   O = s    */
    L2A_FLAG_SEQUENTIAL = 8,  /* forward: run the branches one after the other at every length (see
                                 l2a_attn_fwd: short sequences otherwise run them in one launch) */
    L2A_FLAG_RING_CACHE = 16, /* l2a_attn_decode with L2A_FLAG_SKIP_GLOBAL: the cache is a ring (see there) */
    L2A_FLAG_SCALAR = 1 << 16 /* bf16 only: use the scalar-FMA kernels instead of the matrix-core ones
                                 (slow; for cross-checking, and the only bf16 path for D = 64) */
};

enum {
    L2A_OK = 0,
    L2A_ERR_NULL = -1,        /* a required pointer is NULL */
    L2A_ERR_SHAPE = -2,       /* B, T < 1; Hq % Hkv != 0; W < 0; mask_heads not in {1, Hkv, Hq}; sizes overflow int32 rows */
    L2A_ERR_UNSUPPORTED = -3, /* dtype / D combination or flag combination not built */
    L2A_ERR_WORKSPACE = -4,   /* workspace NULL or smaller than l2a_*_workspace_bytes() */
    L2A_ERR_ALIGN = -5,       /* a data pointer is not 16-byte aligned */
    L2A_ERR_LAUNCH = -6,      /* the HIP runtime refused a launch (hipGetLastError) */
    L2A_ERR_STATIC_LIMIT = -7 /* the problem needs more scratch than a *_static entry point's fixed array holds */
};

typedef struct l2a_params {
    int32_t B, T, Hq, Hkv, D;
    int32_t W;           /* local window: keys j with 0 <= t - j <= W                  (Sec. 2) */
    int32_t mask_heads;  /* routing mask is [B, mask_heads, T]: 1 (shared by all heads, the paper's
                            router emits one decision per token, Sec. 3.1 Eq. 3), Hkv, or Hq   */
    int32_t dtype;       /* L2A_BF16 | L2A_FP32 */
    int32_t flags;       /* L2A_FLAG_* */
    float softmax_scale; /* multiplies <q,k>; the paper uses 1/sqrt(d) (Sec. 2 Eq. Attn) */
} l2a_params;

int l2a_version(void);
const char* l2a_strerror(int code);

/*
 * Host-only, pure: scratch bytes each call needs (0 is possible; then workspace may be NULL).
 * The workspace is device memory owned by the caller, 16-byte aligned (sub-buffers are laid out at
 * multiples of 256 bytes from its start), not preserved between
 * calls; calls that share one workspace must be ordered on one stream.  What it holds:
 *   route     one int32 count per (b, KV head, chunk of 2048 positions; of 256 for T <= 16384)
 *   forward   bf16, D = 128 without L2A_FLAG_SCALAR: a token-minor copy [B,Hkv,D,ceil64(T)] of
 *             each branch's V and one int32 flag per tile of 256 rows (tiles per (b, KV head)
 *             rounded up to a multiple of 8); when both branches run in one launch (see
 *             l2a_attn_fwd) the flags twice and a [B,T,Hq,D] float buffer for a; else nothing
 *   backward  delta_t of each branch, [B,Hq,T] float, twice; on the matrix-core path also, per
 *             branch, compact row-major copies of the rows' Q and dO (ceil64(T G) rows per
 *             (b, KV head)) with three per-row statistics; short sequences (fewer than 256
 *             blocks of 128 keys over all (b, KV head)): up to 8 x 2 float copies of [B,T,Hkv,D],
 *             partial sums of the workgroups that share a key block's rows
 */
size_t l2a_route_workspace_bytes(const l2a_params* p);
size_t l2a_attn_workspace_bytes(const l2a_params* p, int backward);

/* Number of int32 entries of kblk_first_row per (b, KV head): ceil(T / 64) + 1. */
int32_t l2a_kblk_entries(int32_t T);

/*
 * Routing compaction: the preprocessing step of the sparse kernel (Sec. 3.2; App. C Alg. 1
 * step 1; App. D.1 counts it in the kernel's time).  For each (b, KV head) builds the
 * ascending list of routed query rows.  A row is a (position, head-in-group) pair coded
 * pos * G + g, so the G query heads that share a KV head sit in the same dense tile.
 *
 *   mask            in  [B, mask_heads, T] uint8; any non-zero byte means d = 1
 *   row_idx         out [B, Hkv, T*G] int32, ascending; entries at index >= count are -1
 *   count           out [B, Hkv] int32, number of routed rows
 *   kblk_first_row  out [B, Hkv, ceil(T/64)+1] int32; entry k = number of rows with pos < 64 k
 *                       (so the last entry equals count); lets the backward pass find, for a
 *                       block of keys, the first compacted row that can see it
 * Results are bit-exact and unique.  With L2A_FLAG_DENSE the call is a no-op returning L2A_OK.
 */
int l2a_route_compact(const l2a_params* p, const uint8_t* mask, int32_t* row_idx, int32_t* count,
                      int32_t* kblk_first_row, void* workspace, size_t workspace_bytes, void* stream);

/*
 * l2a_route_compact for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same inputs, same
 * outputs, same bits as l2a_route_compact; the per-chunk counts live in a fixed array in the library's
 * device image instead of a caller workspace, and the call allocates nothing (no hipMalloc, no hipFree).
 *   Limit   B * Hkv * ceil(T / c) <= 65536 counters, c = 2048 positions (256 for T <= 16384) -- e.g.
 *           B * Hkv = 32 at T = 4M tokens; beyond it the call returns L2A_ERR_STATIC_LIMIT and
 *           launches nothing.  The array (256 KB) stays resident on every GPU the library runs on
 *           until the process ends.
 *   Sharing every call on a GPU uses that GPU's one array and overwrites what the last call left (no
 *           part of it has to start at zero: each counter is written before it is read).  Calls
 *           that overlap on one GPU -- different streams, or different threads -- race; order
 *           them on one stream or with events.
 *   Set-up  the first call on a device looks up the array's address on that device
 *           (hipGetSymbolAddress), so make it outside stream capture.  L2A_ERR_LAUNCH if that fails.
 */
int l2a_route_compact_static(const l2a_params* p, const uint8_t* mask, int32_t* row_idx, int32_t* count,
                             int32_t* kblk_first_row, void* stream);

/*
 * Router front-end (Sec. 3.1 Eq. 3; the threshold is 0.5 in training and a knob at test time):
 *     logit_t = <w, x_t> + bias,   dhat_t = sigmoid(logit_t),   d_t = 1 iff dhat_t >= tau,
 * the decision being taken on the logit (logit_t >= ln(tau / (1 - tau))).  The mask it writes is
 * the input of l2a_route_compact with mask_heads = 1.  Only B, T and dtype of `p` are used (the
 * other fields must still be valid).  fp32 accumulation; HBM-bound, x is read once.
 *
 *   C          channels of the router input, a multiple of 8
 *   x          in  [B,T,C] router input of every token, element type p->dtype (the Local module's
 *                  output; for a router that reads the raw local attention output, S viewed as
 *                  [B,T,Hq*D])
 *   w          in  [C] float
 *   logit_opt  out optional [B,T] float
 *   dhat_opt   out optional [B,T] float: the score, for the sparsity regulariser and the
 *                  straight-through gradient (Sec. 3.3 Eqs. 6, 7)
 *   mask       out [B,1,T] uint8, 0 or 1
 * Errors: L2A_ERR_SHAPE for C not a positive multiple of 8 or tau outside (0,1).
 */
int l2a_router_decide(const l2a_params* p, int32_t C, const void* x, const float* w, float bias, float tau,
                      float* logit_opt, float* dhat_opt, uint8_t* mask, void* stream);

/*
 * Forward (Sec. 3.1 Eqs. 2, 4, 5; App. C Alg. 1).
 *
 *   q_loc,k_loc,v_loc  in  inputs of the Local branch
 *   q_glb,k_glb,v_glb  in  inputs of the Global branch; may be the same pointers as *_loc (the
 *                          paper's shared-projection variant) or different tensors (separate
 *                          Local / Global modules)
 *   row_idx,count,kblk_first_row  in  from l2a_route_compact (NULL allowed with L2A_FLAG_DENSE
 *                          or L2A_FLAG_SKIP_GLOBAL)
 *   O           out [B,T,Hq,D]  o = s + d a
 *   lse_local   out [B,Hq,T]    (may be NULL with L2A_FLAG_SKIP_LOCAL)
 *   lse_global  out [B,Hq,T]    -inf where d = 0 (may be NULL with L2A_FLAG_SKIP_GLOBAL)
 *   S_opt       out optional [B,T,Hq,D]: s alone (needed by l2a_attn_bwd)
 *   A_opt       out optional [B,T,Hq,D]: d a alone, zero where d = 0 (needed by l2a_attn_bwd)
 *
 * Short sequences (bf16, D = 128, both branches, routing lists in use, at most 2048 tiles of 256
 * rows over all (b, KV head)): the Global rows' tiles alone would occupy a fraction of the chip, so
 * the two branches run in one launch, the Global one leaves a in fp32 in the workspace, and a
 * third, small kernel forms o = s + d a -- bit for bit the result of the sequential order, where
 * the Global kernel adds its fp32 result to the stored s.  L2A_FLAG_SEQUENTIAL keeps the sequential
 * order at every length.
 */
int l2a_attn_fwd(const l2a_params* p, const void* q_loc, const void* k_loc, const void* v_loc,
                 const void* q_glb, const void* k_glb, const void* v_glb, const int32_t* row_idx,
                 const int32_t* count, const int32_t* kblk_first_row, void* O, float* lse_local,
                 float* lse_global, void* S_opt, void* A_opt, void* workspace, size_t workspace_bytes,
                 void* stream);

/*
 * Decode step (Sec. 3.4): one new token per sequence against the KV cache.  Local attention over
 * the last W+1 keys for every token; Global attention over keys 0..pos only for heads whose
 * decision is 1 -- skipped entirely, cache not read, when no head of a KV group is routed; merged
 * as o = s + d a (Sec. 3.1 Eq. 5).  bf16, D = 128, Hq / Hkv <= 16; both branches read the same
 * q / cache (for separate Local and Global modules call twice with L2A_FLAG_SKIP_GLOBAL /
 * L2A_FLAG_SKIP_LOCAL).  HBM-bound: every cache row in reach is read once per branch.
 *
 *   p->T        capacity of the cache in tokens (the row stride of k_cache / v_cache)
 *   q           in  [B,Hq,D]      the new token's queries
 *   k_cache,v_cache  in  [B,T,Hkv,D]  rows 0..pos[b] valid (the new token's own K, V included); what
 *                   the rows behind pos[b] hold never enters the result
 *   pos         in  [B] int32, device memory: position of the new token, 0 <= pos[b] < T
 *                   (device data cannot be validated on the host: values outside are clamped into the range)
 *   mask        in  [B,mask_heads] uint8, device memory: the new token's decisions
 *                   (NULL allowed with L2A_FLAG_DENSE)
 *   O           out [B,Hq,D]
 *   lse_local, lse_global  out optional [B,Hq]; lse_global is -inf where d = 0
 *   S_opt, A_opt  out optional [B,Hq,D]; A is zero where d = 0
 *   workspace   l2a_decode_workspace_bytes(p): one partial (max, sum, O) per 512 keys, head and branch
 *
 * L2A_FLAG_RING_CACHE (with L2A_FLAG_SKIP_GLOBAL; a Local module of its own keeps only its window):
 * the cache is a ring of p->T >= W + 1 slots (a multiple of 32), the K, V of token j in slot j mod p->T, and pos[b] is the
 * new token's position in the sequence, however long (negative values are clamped to 0).  Slots not
 * yet written (pos[b] < p->T - 1) are never used.  Errors: L2A_ERR_UNSUPPORTED without
 * L2A_FLAG_SKIP_GLOBAL, with p->T < W + 1 or p->T not a multiple of 32.
 */
size_t l2a_decode_workspace_bytes(const l2a_params* p);
int l2a_attn_decode(const l2a_params* p, const void* q, const void* k_cache, const void* v_cache,
                    const int32_t* pos, const uint8_t* mask, void* O, float* lse_local, float* lse_global,
                    void* S_opt, void* A_opt, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Backward (Sec. 3.2: gradients only for the active queries, reusing the saved log-sum-exp
 * and Q_idx; the formulas are the standard softmax-attention gradient).  With g_t = dO_t for
 * the Local branch and d_t dO_t for the Global branch (from Eq. 5):
 *     p_tj = exp(scale <q_t,k_j> - lse(t)),  delta_t = <g_t, out_t>,
 *     dv_j += p_tj g_t,  ds_tj = p_tj (<g_t, v_j> - delta_t),
 *     dq_t += scale ds_tj k_j,  dk_j += scale ds_tj q_t      (dk, dv summed over the G heads of a group).
 *
 *   dO                in  [B,T,Hq,D]
 *   S, A              in  branch outputs saved by the forward (S_opt, A_opt)
 *   lse_local, lse_global  in  saved by the forward
 *   dq_loc,dk_loc,dv_loc   out gradients w.r.t. the Local branch's inputs
 *   dq_glb,dk_glb,dv_glb   out gradients w.r.t. the Global branch's inputs.  If a *_glb pointer
 *                          equals its *_loc partner the two gradients are summed into that one
 *                          buffer (shared projections); all three must then alias.
 *                          Rows of dq_glb for tokens with d = 0 are zero.
 *   delta_glb_opt     out optional [B,Hq,T] float: <dO_t, A_t>, the task-loss part of the
 *                          router-score gradient (Sec. 3.3 Eq. 7), for every token: zero where A is.
 *                          For the training steps that compute Global attention for all tokens
 *                          (Sec. 3.3), pass as A and lse_global the outputs of a Global-only
 *                          L2A_FLAG_DENSE forward together with the sparse row lists: the q/k/v
 *                          gradients still come from the routed rows only, delta_glb covers all.
 */
int l2a_attn_bwd(const l2a_params* p, const void* dO, const void* q_loc, const void* k_loc,
                 const void* v_loc, const void* q_glb, const void* k_glb, const void* v_glb,
                 const int32_t* row_idx, const int32_t* count, const int32_t* kblk_first_row, const void* S,
                 const void* A, const float* lse_local, const float* lse_global, void* dq_loc, void* dk_loc,
                 void* dv_loc, void* dq_glb, void* dk_glb, void* dv_glb, float* delta_glb_opt,
                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * Optional per-kernel timing, for benchmarks (off by default).  While enabled, every kernel the
 * library launches -- from any thread: the log is guarded by a mutex, and records of concurrent
 * callers interleave in launch order -- is bracketed by HIP events on its launch stream.
 * l2a_profile_read synchronises with those events, copies up to `max` records (launch order;
 * `name` points to a static string) into `out`, clears the log and returns the number of
 * records there were.  This log is the only state the library keeps between calls.
 */
typedef struct l2a_kernel_time {
    const char* name;
    float ms;
} l2a_kernel_time;
void l2a_profile_enable(int on);
int l2a_profile_read(l2a_kernel_time* out, int max);

#ifdef __cplusplus
}
#endif
#endif /* L2A_H_ */
