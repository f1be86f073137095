/*
 * CPU oracle for the L2A conditional-attention layer.  TEST INFRASTRUCTURE ONLY:
 * nothing on the product path may link, load or call this file; it exists so that the
 * tests, the smoke check and the benchmark's cpu_baseline leg have an independent
 * statement of what the layer computes.  It shares no code with the HIP path.
 *
 * Every function writes out the plain definition, one query token (or one key token) at
 * a time, in fp64: no tiling, no online softmax, no fusion.
 *
 *   Global attention         softmax(q k^T / sqrt(d) + M) v,  M_ij = 0 iff j <= i     (Sec. 2, Eq. Attn)
 *   Local (sliding window)   same with M_ij = 0 iff 0 <= i - j <= w: the token itself
 *                            and the w tokens before it                                (Sec. 2)
 *   Conditional global       a_t = GlobalAttn(...) if d_t = 1, else 0                  (Sec. 3.1, Eq. 4)
 *   Merge                    o_t = s_t + a_t * d_t                                     (Sec. 3.1, Eq. 5)
 *   Router                   dhat_t = sigmoid(<w, x_t> + bias), d_t = [dhat_t >= tau]   (Sec. 3.1, Eq. 3;
 *                            tau = 0.5 in training, a knob at test time)
 *   Compaction               ascending list of the active queries' positions (Q_idx)   (Sec. 3.2; App. C, Alg. 1 step 1)
 *   Backward                 the paper only says gradients are taken for active queries
 *                            with the saved log-sum-exp (Sec. 3.2); the formulas are the
 *                            textbook gradient of softmax attention.
 *
 * Conventions fixed here because the paper leaves them open:
 *   - tensors are row-major [B, T, H, D] (fp32 storage; all arithmetic in fp64);
 *   - grouped-query attention: query head h reads KV head h / G, G = Hq / Hkv;
 *   - the routing mask is [B, Hm, T] with Hm in {1, Hkv, Hq}: shared by all heads, per KV
 *     head, or per query head; any non-zero byte means d = 1;
 *   - log-sum-exp is the natural log of the sum of exp(scaled scores); it is -inf for the
 *     global branch of a token with d = 0;
 *   - compacted rows are (position, head-in-group) pairs coded pos * G + g, ascending,
 *     one list per (batch, KV head); kblk_first_row[k] counts rows with pos < 64 k.
 */
#include <math.h>
#include <omp.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t B, T, Hq, Hkv, D, W, Hm;
    double scale;
} oracle_dims;

static inline int mask_head(const oracle_dims* p, int h) {
    const int G = p->Hq / p->Hkv;
    if (p->Hm == 1) return 0;
    if (p->Hm == p->Hq) return h;
    return h / G; /* Hm == Hkv */
}

static inline int routed(const oracle_dims* p, const uint8_t* mask, int b, int h, int t) {
    return mask[((size_t)b * p->Hm + mask_head(p, h)) * p->T + t] != 0;
}

static inline const float* qrow(const oracle_dims* p, const float* q, int b, int t, int h) {
    return q + (((size_t)b * p->T + t) * p->Hq + h) * p->D;
}

static inline const float* kvrow(const oracle_dims* p, const float* x, int b, int t, int hk) {
    return x + (((size_t)b * p->T + t) * p->Hkv + hk) * p->D;
}

static inline double dotf(const float* a, const float* b, int D) {
    double s = 0.0;
    for (int i = 0; i < D; ++i) s += (double)a[i] * (double)b[i];
    return s;
}

/* Softmax attention of one query over keys j0..j1 (inclusive) of one KV head.
 * z_j = scale <q, k_j>;  m = max z;  l = sum exp(z - m);  out = sum (exp(z_j - m) / l) v_j;
 * lse = m + ln l.  `z` is scratch of length >= j1 - j0 + 1 and returns the probabilities. */
static void attend(const oracle_dims* p, const float* qv, const float* k, const float* v, int b, int hk,
                   int j0, int j1, double* z, double* out, double* lse) {
    const int D = p->D, n = j1 - j0 + 1;
    double m = -INFINITY;
    for (int j = 0; j < n; ++j) {
        z[j] = p->scale * dotf(qv, kvrow(p, k, b, j0 + j, hk), D);
        if (z[j] > m) m = z[j];
    }
    double l = 0.0;
    for (int j = 0; j < n; ++j) l += exp(z[j] - m);
    for (int i = 0; i < D; ++i) out[i] = 0.0;
    for (int j = 0; j < n; ++j) {
        const double pj = exp(z[j] - m) / l;
        z[j] = pj;
        const float* vj = kvrow(p, v, b, j0 + j, hk);
        for (int i = 0; i < D; ++i) out[i] += pj * (double)vj[i];
    }
    *lse = m + log(l);
}

/* ---------------------------------------------------------------------------------------
 * Router (Sec. 3.1 Eq. 3): score and decision of every token from its router input x_t [C].
 *   logit[b,t] = <w, x[b,t,:]> + bias;  dhat = 1 / (1 + exp(-logit));  d = 1 iff dhat >= tau,
 * taken on the logit: logit >= ln(tau / (1 - tau)), which is the same comparison without the
 * rounding of the sigmoid.  x is fp32 storage; everything else fp64.
 * ------------------------------------------------------------------------------------- */
void l2a_oracle_router(int32_t B, int32_t T, int32_t C, const float* x, const double* w, double bias, double tau,
                       double* logit, double* dhat, uint8_t* d) {
    const double thr = log(tau / (1.0 - tau));
#pragma omp parallel for schedule(static)
    for (long long i = 0; i < (long long)B * T; ++i) {
        const float* xi = x + (size_t)i * C;
        double acc = 0.0;
        for (int c = 0; c < C; ++c) acc += w[c] * (double)xi[c];
        acc += bias;
        logit[i] = acc;
        dhat[i] = 1.0 / (1.0 + exp(-acc));
        d[i] = acc >= thr ? 1 : 0;
    }
}

/* ---------------------------------------------------------------------------------------
 * Compaction (Sec. 3.2; App. C, Alg. 1 step 1): brute force over (pos, g).
 * row_idx [B, Hkv, T*G] (unused tail = -1), count [B, Hkv], kblk_first_row [B, Hkv, nkb+1]
 * with nkb = ceil(T / 64).
 * ------------------------------------------------------------------------------------- */
void l2a_oracle_route_compact(const oracle_dims* p, const uint8_t* mask, int32_t* row_idx, int32_t* count,
                              int32_t* kblk_first_row) {
    const int G = p->Hq / p->Hkv, T = p->T;
    const int nkb = (T + 63) / 64;
    for (int b = 0; b < p->B; ++b)
        for (int hk = 0; hk < p->Hkv; ++hk) {
            int32_t* rows = row_idx + ((size_t)b * p->Hkv + hk) * (size_t)T * G;
            int32_t* first = kblk_first_row + ((size_t)b * p->Hkv + hk) * (size_t)(nkb + 1);
            int n = 0;
            for (int pos = 0; pos < T; ++pos) {
                if (pos % 64 == 0) first[pos / 64] = n;
                for (int g = 0; g < G; ++g)
                    if (routed(p, mask, b, hk * G + g, pos)) rows[n++] = pos * G + g;
            }
            first[nkb] = n;
            count[b * p->Hkv + hk] = n;
            for (size_t i = n; i < (size_t)T * G; ++i) rows[i] = -1;
        }
}

/* ---------------------------------------------------------------------------------------
 * Forward for a list of query rows (b, h, t).  Outputs are [n, D] / [n]:
 *   S = local attention, A = global attention (0 if d = 0), O = S + d A,
 *   lse_l, lse_g (-inf if d = 0).
 * Local and global branches read their own q/k/v, which may be the same arrays.
 * ------------------------------------------------------------------------------------- */
void l2a_oracle_fwd_rows(const oracle_dims* p, const float* ql, const float* kl, const float* vl,
                         const float* qg, const float* kg, const float* vg, const uint8_t* mask,
                         int64_t n, const int32_t* rows, double* S, double* A, double* O, double* lse_l,
                         double* lse_g) {
    const int D = p->D, G = p->Hq / p->Hkv;
#pragma omp parallel
    {
        double* z = (double*)malloc(sizeof(double) * (size_t)p->T);
#pragma omp for schedule(dynamic, 4)
        for (int64_t r = 0; r < n; ++r) {
            const int b = rows[3 * r], h = rows[3 * r + 1], t = rows[3 * r + 2];
            const int hk = h / G;
            const int j0 = t - p->W > 0 ? t - p->W : 0;
            attend(p, qrow(p, ql, b, t, h), kl, vl, b, hk, j0, t, z, S + r * D, lse_l + r);
            if (routed(p, mask, b, h, t)) {
                attend(p, qrow(p, qg, b, t, h), kg, vg, b, hk, 0, t, z, A + r * D, lse_g + r);
            } else {
                for (int i = 0; i < D; ++i) A[r * D + i] = 0.0;
                lse_g[r] = -INFINITY;
            }
            for (int i = 0; i < D; ++i) O[r * D + i] = S[r * D + i] + A[r * D + i];
        }
        free(z);
    }
}

/* One branch's gradient w.r.t. one query row.  With g = dL/d(branch output):
 *   p_j = softmax probabilities, out = sum p_j v_j, delta = <g, out>, dp_j = <g, v_j>,
 *   ds_j = p_j (dp_j - delta),  dq = scale * sum_j ds_j k_j.                               */
static void dq_branch(const oracle_dims* p, const float* qv, const float* k, const float* v, int b, int hk,
                      int j0, int j1, const float* g, double* z, double* out, double* dq) {
    const int D = p->D;
    double lse;
    attend(p, qv, k, v, b, hk, j0, j1, z, out, &lse);
    double delta = 0.0;
    for (int i = 0; i < D; ++i) delta += (double)g[i] * out[i];
    for (int i = 0; i < D; ++i) dq[i] = 0.0;
    for (int j = j0; j <= j1; ++j) {
        const double dp = dotf(g, kvrow(p, v, b, j, hk), D);
        const double ds = z[j - j0] * (dp - delta);
        const float* kj = kvrow(p, k, b, j, hk);
        for (int i = 0; i < D; ++i) dq[i] += p->scale * ds * (double)kj[i];
    }
}

/* dQ for a list of query rows: dq_l (local branch) and dq_g (global branch, 0 if d = 0). */
void l2a_oracle_bwd_dq_rows(const oracle_dims* p, const float* ql, const float* kl, const float* vl,
                            const float* qg, const float* kg, const float* vg, const uint8_t* mask,
                            const float* dO, int64_t n, const int32_t* rows, double* dq_l, double* dq_g) {
    const int D = p->D, G = p->Hq / p->Hkv;
#pragma omp parallel
    {
        double* z = (double*)malloc(sizeof(double) * (size_t)p->T);
        double* out = (double*)malloc(sizeof(double) * (size_t)D);
#pragma omp for schedule(dynamic, 4)
        for (int64_t r = 0; r < n; ++r) {
            const int b = rows[3 * r], h = rows[3 * r + 1], t = rows[3 * r + 2];
            const int hk = h / G;
            const int j0 = t - p->W > 0 ? t - p->W : 0;
            const float* g = qrow(p, dO, b, t, h);
            dq_branch(p, qrow(p, ql, b, t, h), kl, vl, b, hk, j0, t, g, z, out, dq_l + r * D);
            if (routed(p, mask, b, h, t))
                dq_branch(p, qrow(p, qg, b, t, h), kg, vg, b, hk, 0, t, g, z, out, dq_g + r * D);
            else
                for (int i = 0; i < D; ++i) dq_g[r * D + i] = 0.0;
        }
        free(z);
        free(out);
    }
}

/* dK, dV for a list of key tokens (b, hk, j), per branch.  Needs each query row's saved
 * statistics lse_X[B,Hq,T] and delta_X[B,Hq,T] = <dO_t, X_t> (X = S or A) for every row that
 * can see key j (rows outside that set are not read):
 *   p_tj = exp(z_tj - lse_X(t)),  dv_j += p_tj dO_t,  dp_tj = <dO_t, v_j>,
 *   ds_tj = p_tj (dp_tj - delta_X(t)),  dk_j += scale ds_tj q_t,
 * summed over the G query heads of the KV head and over t in the branch's range:
 * local j <= t <= j + W, global t >= j with d_t = 1.                                       */
void l2a_oracle_bwd_dkdv_keys(const oracle_dims* p, const float* ql, const float* kl, const float* vl,
                              const float* qg, const float* kg, const float* vg, const uint8_t* mask,
                              const float* dO, const double* lse_l, const double* delta_l,
                              const double* lse_g, const double* delta_g, int64_t n, const int32_t* keys,
                              double* dk_l, double* dv_l, double* dk_g, double* dv_g) {
    const int D = p->D, G = p->Hq / p->Hkv, T = p->T;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t r = 0; r < n; ++r) {
        const int b = keys[3 * r], hk = keys[3 * r + 1], j = keys[3 * r + 2];
        double* out[4] = {dk_l + r * D, dv_l + r * D, dk_g + r * D, dv_g + r * D};
        for (int o = 0; o < 4; ++o)
            for (int i = 0; i < D; ++i) out[o][i] = 0.0;
        for (int g = 0; g < G; ++g) {
            const int h = hk * G + g;
            for (int t = j; t < T; ++t) {
                const size_t st = ((size_t)b * p->Hq + h) * T + t;
                const float* go = qrow(p, dO, b, t, h);
                if (t - j <= p->W) { /* local branch */
                    const float* qt = qrow(p, ql, b, t, h);
                    const double z = p->scale * dotf(qt, kvrow(p, kl, b, j, hk), D);
                    const double pt = exp(z - lse_l[st]);
                    const double ds = pt * (dotf(go, kvrow(p, vl, b, j, hk), D) - delta_l[st]);
                    for (int i = 0; i < D; ++i) {
                        dv_l[r * D + i] += pt * (double)go[i];
                        dk_l[r * D + i] += p->scale * ds * (double)qt[i];
                    }
                }
                if (routed(p, mask, b, h, t)) { /* global branch */
                    const float* qt = qrow(p, qg, b, t, h);
                    const double z = p->scale * dotf(qt, kvrow(p, kg, b, j, hk), D);
                    const double pt = exp(z - lse_g[st]);
                    const double ds = pt * (dotf(go, kvrow(p, vg, b, j, hk), D) - delta_g[st]);
                    for (int i = 0; i < D; ++i) {
                        dv_g[r * D + i] += pt * (double)go[i];
                        dk_g[r * D + i] += p->scale * ds * (double)qt[i];
                    }
                }
            }
        }
    }
}

int l2a_oracle_abi(void) { return 1; }

/* OpenMP threads the parallel loops above will use (for reporting timings). */
int l2a_oracle_threads(void) { return omp_get_max_threads(); }
