/*
 * CPU oracle for one FlowSpec verification stage.  TEST INFRASTRUCTURE ONLY:
 * imported by tests/, by __graft_entry__.smoke() and by bench.py's cpu_baseline
 * leg; the product path (the HIP library) shares no code with this file and
 * never calls it.
 *
 * Plain C, fp64 arithmetic, loops written in the order the method states them;
 * OpenMP is used only as "parallel for" over independent output features / rows.
 *
 * What it computes (paper, Sec. III):
 *   - orc_tree_ancestors : tree attention mask + tree position ids of a draft
 *     sequence S in descending-score order (Sec. III-A: a segment's position IDs and
 *     attention mask follow the tree; Sec. III-B: S is a topological order).
 *   - orc_verify_stage   : forward of a block of decoder layers (Appendix A:
 *     self-attention, FFN, residuals; LLaMA2/Qwen2 form) over one draft segment
 *     with the tree mask, appending the segment's K/V to the stage cache.
 *   - orc_lm_head / orc_argmax_rows : last stage's next-token scores.
 *   - orc_accept         : accepted tokens S_acc, x_new, continuous condition
 *     (Eq. 2) and retain set I_retain = I_acc U I_pr (Sec. III-C), greedy.
 *   - orc_kv_compact     : KV-cache pruning by I_incache (Sec. III-C).
 *   - orc_seg_prune      : draft-segment pruning by I_local (Sec. III-C).
 *   - orc_tree_remap     : T_pr / S_pr in original order (Sec. III-C).
 *
 * Pins (tests, "not gpu"): per-path sequential decoding with library routines,
 * chain / star / empty-prefix special cases, closed forms for RMSNorm / RoPE /
 * softmax, the pruning figure's index sets, brute force over all paths.  The
 * paper prints no numeric hidden states or logits, so numeric values are pinned
 * only through those identities ("parity unpinned" by the paper itself).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_OK 0
#define ORC_EINVAL (-1)
#define ORC_ETOPO (-2)
#define ORC_ECAP (-3)

typedef struct {
    int n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
    int wdtype; /* 0: weights are float32, 1: weights are bfloat16 bit patterns (uint16) */
    double rms_eps, rope_theta;
    int kv_capacity;
} orc_desc;

typedef struct {
    const void *rms_attn, *wq, *wk, *wv, *wo, *rms_ffn, *w_gate, *w_up, *w_down;
    const void *bq, *bk, *bv; /* may be NULL */
} orc_layer;

typedef struct {
    int32_t n_acc, x_new, n_new, continuous, n_retain, n_pr_verified;
} orc_accept_result;

static inline double wget(const void *w, int wdtype, size_t i) {
    if (wdtype == 0) return (double)((const float *)w)[i];
    uint32_t u = (uint32_t)((const uint16_t *)w)[i] << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* ---- tree structure -------------------------------------------------------------------- */

/* anc[i] (W = ceil(T/64) words) = ancestor-or-self set of node i; depth[i] = #edges to its root.
 * Recurrence in S order: anc[i] = anc[parent[i]] | bit(i). */
int orc_tree_ancestors(const int32_t *parent, int T, uint64_t *anc, int32_t *depth) {
    int W = (T + 63) / 64;
    for (int i = 0; i < T; ++i) {
        int p = parent[i];
        if (p < -1 || p >= i) return ORC_ETOPO;
        for (int w = 0; w < W; ++w) anc[(size_t)i * W + w] = (p >= 0) ? anc[(size_t)p * W + w] : 0;
        anc[(size_t)i * W + i / 64] |= (uint64_t)1 << (i % 64);
        depth[i] = (p >= 0) ? depth[p] + 1 : 0;
    }
    return ORC_OK;
}

/* ---- decoder-layer pieces -------------------------------------------------------------- */

/* out = x * rsqrt(mean(x^2) + eps) * g */
void orc_rmsnorm(const double *x, const void *g, int wdtype, int d, double eps, double *out) {
    double ss = 0.0;
    for (int i = 0; i < d; ++i) ss += x[i] * x[i];
    double r = 1.0 / sqrt(ss / d + eps);
    for (int i = 0; i < d; ++i) out[i] = x[i] * r * wget(g, wdtype, i);
}

/* Rotary embedding of one head vector at absolute position pos: element t pairs with t + hd/2,
 * angle = pos * theta^(-2t/hd). */
void orc_rope(double *v, int hd, double pos, double theta) {
    int h = hd / 2;
    for (int t = 0; t < h; ++t) {
        double ang = pos * pow(theta, -2.0 * t / hd);
        double c = cos(ang), s = sin(ang);
        double a = v[t], b = v[t + h];
        v[t] = a * c - b * s;
        v[t + h] = b * c + a * s;
    }
}

/* y[r][n] = sum_k x[r][k] * W[n][k] (+ bias[n]) for r < rows, n < N; W row-major [N][K]. */
static void matmul_wt(const double *x, int rows, int K, const void *W, const void *bias, int wdtype, int N, double *y) {
#pragma omp parallel
    {
        double *wrow = (double *)malloc(sizeof(double) * (size_t)K);
#pragma omp for schedule(static)
        for (int n = 0; n < N; ++n) {
            for (int k = 0; k < K; ++k) wrow[k] = wget(W, wdtype, (size_t)n * K + k);
            double b = bias ? wget(bias, wdtype, n) : 0.0;
            for (int r = 0; r < rows; ++r) {
                const double *xr = x + (size_t)r * K;
                double acc = 0.0;
                for (int k = 0; k < K; ++k) acc += xr[k] * wrow[k];
                y[(size_t)r * N + n] = acc + b;
            }
        }
        free(wrow);
    }
}

static inline size_t kv_index(const orc_desc *D, int layer, int which, int head, int slot) {
    return ((((size_t)layer * 2 + which) * D->n_kv_heads + head) * D->kv_capacity + slot) * (size_t)D->head_dim;
}

/*
 * Verify one segment S[seg_off, seg_off + l_s) through the stage's layers.
 *   kv         : double [n_layers][2][n_kv_heads][kv_capacity][head_dim]; slots [0, l_cache) valid on entry,
 *                slots [l_cache, l_cache + l_s) written (K stored after rotation).
 *   parent     : [seg_off + l_s] in S order; requires l_cache == l_glo + seg_off so that S index j lives at
 *                slot l_glo + j.
 *   visibility : row r (node g = seg_off + r) sees slot s iff s < l_glo or (s - l_glo) is an
 *                ancestor-or-self of g.
 */
int orc_verify_stage(const orc_desc *D, const orc_layer *L, double *kv, int l_glo, int l_cache, const double *hidden_in,
                     int seg_off, int l_s, const int32_t *parent, double *hidden_out) {
    if (l_s < 0 || seg_off < 0 || l_glo < 0 || l_cache != l_glo + seg_off) return ORC_EINVAL;
    if (l_cache + l_s > D->kv_capacity) return ORC_ECAP;
    if (D->n_q_heads % D->n_kv_heads != 0 || D->head_dim % 2 != 0) return ORC_EINVAL;
    if (l_s == 0) return ORC_OK;
    const int T = seg_off + l_s, W = (T + 63) / 64;
    const int d = D->d_model, hd = D->head_dim, Hq = D->n_q_heads, Hkv = D->n_kv_heads, F = D->d_ffn;
    const int G = Hq / Hkv, nq = Hq * hd, nkv = Hkv * hd, wd = D->wdtype;
    uint64_t *anc = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)T * W);
    int32_t *depth = (int32_t *)malloc(sizeof(int32_t) * (size_t)T);
    int rc = orc_tree_ancestors(parent, T, anc, depth);
    if (rc != ORC_OK) {
        free(anc);
        free(depth);
        return rc;
    }
    double *x = (double *)malloc(sizeof(double) * (size_t)l_s * d);
    double *nrm = (double *)malloc(sizeof(double) * (size_t)l_s * d);
    double *q = (double *)malloc(sizeof(double) * (size_t)l_s * nq);
    double *k = (double *)malloc(sizeof(double) * (size_t)l_s * nkv);
    double *v = (double *)malloc(sizeof(double) * (size_t)l_s * nkv);
    double *o = (double *)malloc(sizeof(double) * (size_t)l_s * nq);
    double *t1 = (double *)malloc(sizeof(double) * (size_t)l_s * (F > d ? F : d));
    double *t2 = (double *)malloc(sizeof(double) * (size_t)l_s * F);
    memcpy(x, hidden_in, sizeof(double) * (size_t)l_s * d);
    const int Ltot = l_cache + l_s;
    const double scale = 1.0 / sqrt((double)hd);

    for (int layer = 0; layer < D->n_layers; ++layer) {
        const orc_layer *w = &L[layer];
        /* attention block */
        for (int r = 0; r < l_s; ++r) orc_rmsnorm(x + (size_t)r * d, w->rms_attn, wd, d, D->rms_eps, nrm + (size_t)r * d);
        matmul_wt(nrm, l_s, d, w->wq, w->bq, wd, nq, q);
        matmul_wt(nrm, l_s, d, w->wk, w->bk, wd, nkv, k);
        matmul_wt(nrm, l_s, d, w->wv, w->bv, wd, nkv, v);
        for (int r = 0; r < l_s; ++r) {
            double pos = (double)(l_glo + depth[seg_off + r]);
            for (int h = 0; h < Hq; ++h) orc_rope(q + (size_t)r * nq + (size_t)h * hd, hd, pos, D->rope_theta);
            for (int h = 0; h < Hkv; ++h) {
                orc_rope(k + (size_t)r * nkv + (size_t)h * hd, hd, pos, D->rope_theta);
                memcpy(kv + kv_index(D, layer, 0, h, l_cache + r), k + (size_t)r * nkv + (size_t)h * hd, sizeof(double) * hd);
                memcpy(kv + kv_index(D, layer, 1, h, l_cache + r), v + (size_t)r * nkv + (size_t)h * hd, sizeof(double) * hd);
            }
        }
#pragma omp parallel
        {
            double *sc = (double *)malloc(sizeof(double) * (size_t)Ltot);
#pragma omp for collapse(2) schedule(static)
            for (int h = 0; h < Hq; ++h) {
                for (int r = 0; r < l_s; ++r) {
                    const int g = seg_off + r, hk = h / G;
                    const double *qv = q + (size_t)r * nq + (size_t)h * hd;
                    double mx = -INFINITY;
                    for (int s = 0; s < Ltot; ++s) {
                        int vis = (s < l_glo);
                        if (!vis) {
                            int j = s - l_glo;
                            vis = (j < T) && ((anc[(size_t)g * W + j / 64] >> (j % 64)) & 1);
                        }
                        if (!vis) {
                            sc[s] = -INFINITY;
                            continue;
                        }
                        const double *kr = kv + kv_index(D, layer, 0, hk, s);
                        double acc = 0.0;
                        for (int t = 0; t < hd; ++t) acc += qv[t] * kr[t];
                        sc[s] = acc * scale;
                        if (sc[s] > mx) mx = sc[s];
                    }
                    double den = 0.0;
                    for (int s = 0; s < Ltot; ++s) {
                        sc[s] = (sc[s] == -INFINITY) ? 0.0 : exp(sc[s] - mx);
                        den += sc[s];
                    }
                    double *ov = o + (size_t)r * nq + (size_t)h * hd;
                    for (int t = 0; t < hd; ++t) ov[t] = 0.0;
                    for (int s = 0; s < Ltot; ++s) {
                        if (sc[s] == 0.0) continue;
                        const double *vr = kv + kv_index(D, layer, 1, hk, s);
                        double p = sc[s] / den;
                        for (int t = 0; t < hd; ++t) ov[t] += p * vr[t];
                    }
                }
            }
            free(sc);
        }
        matmul_wt(o, l_s, nq, w->wo, NULL, wd, d, t1);
        for (size_t i = 0; i < (size_t)l_s * d; ++i) x[i] += t1[i];
        /* feed-forward block (SwiGLU) */
        for (int r = 0; r < l_s; ++r) orc_rmsnorm(x + (size_t)r * d, w->rms_ffn, wd, d, D->rms_eps, nrm + (size_t)r * d);
        matmul_wt(nrm, l_s, d, w->w_gate, NULL, wd, F, t1);
        matmul_wt(nrm, l_s, d, w->w_up, NULL, wd, F, t2);
        for (size_t i = 0; i < (size_t)l_s * F; ++i) {
            double gte = t1[i];
            t2[i] = (gte / (1.0 + exp(-gte))) * t2[i];
        }
        matmul_wt(t2, l_s, F, w->w_down, NULL, wd, d, t1);
        for (size_t i = 0; i < (size_t)l_s * d; ++i) x[i] += t1[i];
    }
    memcpy(hidden_out, x, sizeof(double) * (size_t)l_s * d);
    free(anc); free(depth); free(x); free(nrm); free(q); free(k); free(v); free(o); free(t1); free(t2);
    return ORC_OK;
}

/* Lowest index of the maximum; comparisons use '>' so NaN never wins; an all-NaN row gives 0. */
void orc_argmax_rows(const float *logits, int rows, int vocab, int32_t *amax) {
    for (int r = 0; r < rows; ++r) {
        const float *p = logits + (size_t)r * vocab;
        float best = -INFINITY;
        int bi = 0;
        for (int i = 0; i < vocab; ++i)
            if (p[i] > best) {
                best = p[i];
                bi = i;
            }
        amax[r] = bi;
    }
}

/* logits = RMSNorm_final(hidden) * E^T, rounded to float32; amax per row. */
int orc_lm_head(const orc_desc *D, const void *final_norm, const void *lm_head, const double *hidden, int rows, float *logits,
                int32_t *amax) {
    if (D->vocab <= 0) return ORC_EINVAL;
    const int d = D->d_model, V = D->vocab;
    double *nrm = (double *)malloc(sizeof(double) * (size_t)rows * d);
    double *lg = (double *)malloc(sizeof(double) * (size_t)rows * V);
    for (int r = 0; r < rows; ++r) orc_rmsnorm(hidden + (size_t)r * d, final_norm, D->wdtype, d, D->rms_eps, nrm + (size_t)r * d);
    matmul_wt(nrm, rows, d, lm_head, NULL, D->wdtype, V, lg);
    for (size_t i = 0; i < (size_t)rows * V; ++i) logits[i] = (float)lg[i];
    orc_argmax_rows(logits, rows, V, amax);
    free(nrm);
    free(lg);
    return ORC_OK;
}

/* ---- acceptance, continuous condition, retain set (Sec. III-C, greedy) ------------------ */
/*
 * Nodes [0, n_ver) of S have a verified next-token argmax amax[i].
 *   match[i] : i > 0, its parent is verified and token[i] == amax[parent[i]]
 *   ok[i]    : every node on path(root 0 -> i) below the root matches (ok[0] = true)
 *   e        : verified ok node of maximum depth, lowest S index among equals
 *   I_acc    : path(0 -> e);   x_new = amax[e]
 *   n_new    : lowest-index child of e whose token is x_new, else -1  (Eq. 2: continuous iff it exists)
 *   I_pr     : n_new and its descendants;   retain = I_acc || I_pr, ascending
 * n_ver == 0 (an emptied segment reached the last stage): nothing is accepted, the context is not
 * updated and every node is retained.
 */
int orc_accept(const int32_t *amax, const int32_t *token, const int32_t *parent, int T, int n_ver, orc_accept_result *res,
               int32_t *retain) {
    if (T <= 0 || n_ver < 0 || n_ver > T) return ORC_EINVAL;
    for (int i = 0; i < T; ++i)
        if (parent[i] < -1 || parent[i] >= i) return ORC_ETOPO;
    if (parent[0] != -1) return ORC_ETOPO;
    if (n_ver == 0) {
        for (int i = 0; i < T; ++i) retain[i] = i;
        res->n_acc = 0; res->x_new = -1; res->n_new = 0; res->continuous = 1; res->n_retain = T; res->n_pr_verified = 0;
        return ORC_OK;
    }
    char *ok = (char *)calloc((size_t)T, 1);
    char *keep = (char *)calloc((size_t)T, 1);
    int *depth = (int *)calloc((size_t)T, sizeof(int));
    ok[0] = 1;
    for (int i = 1; i < T; ++i) {
        int p = parent[i];
        depth[i] = (p >= 0) ? depth[p] + 1 : 0;
        int match = (p >= 0) && (p < n_ver) && (token[i] == amax[p]);
        ok[i] = (char)((p >= 0) && ok[p] && match);
    }
    int e = 0;
    for (int i = 1; i < n_ver; ++i)
        if (ok[i] && depth[i] > depth[e]) e = i;
    int n_acc = 0;
    for (int i = e; i >= 0; i = parent[i]) {
        keep[i] = 1;
        ++n_acc;
    }
    int x_new = amax[e], n_new = -1;
    for (int c = e + 1; c < T; ++c)
        if (parent[c] == e && token[c] == x_new) {
            n_new = c;
            break;
        }
    int n_prv = 0;
    if (n_new >= 0) {
        keep[n_new] = 2;
        for (int i = n_new + 1; i < T; ++i)
            if (parent[i] >= 0 && keep[parent[i]] == 2) keep[i] = 2;
        for (int i = 0; i < n_ver; ++i) n_prv += (keep[i] == 2);
    }
    int n = 0;
    for (int i = 0; i < T; ++i)
        if (keep[i] == 1) retain[n++] = i;
    for (int i = 0; i < T; ++i)
        if (keep[i] == 2) retain[n++] = i;
    res->n_acc = n_acc; res->x_new = x_new; res->n_new = n_new; res->continuous = (n_new >= 0);
    res->n_retain = n; res->n_pr_verified = n_prv;
    free(ok); free(keep); free(depth);
    return ORC_OK;
}

/* T_pr / S_pr: retained draft nodes keep their order; parents are renumbered by rank; new root has parent -1.
 * Returns the new tree size (0 when the round ends). */
int orc_tree_remap(const int32_t *parent, const int32_t *token, int T, const int32_t *retain, int n_acc, int n_retain,
                   int32_t *new_parent, int32_t *new_token) {
    int *rank = (int *)malloc(sizeof(int) * (size_t)T);
    for (int i = 0; i < T; ++i) rank[i] = -1;
    int n = 0;
    for (int j = n_acc; j < n_retain; ++j) rank[retain[j]] = n++;
    for (int j = n_acc; j < n_retain; ++j) {
        int i = retain[j], p = parent[i];
        new_parent[j - n_acc] = (j == n_acc || p < 0) ? -1 : rank[p];
        new_token[j - n_acc] = token[i];
    }
    free(rank);
    return n;
}

/* ---- KV-cache and segment pruning (Sec. III-C) ------------------------------------------ */
/*
 * Cache of any element type, layout [n_layers][2][n_kv_heads][cap][hd] (elem bytes each).
 * I_incache = { i in retain : l_glo + i < l_cache };  new slot l_glo + j <- old slot l_glo + I_incache[j];
 * slots below l_glo are not touched;  out[0] = l_glo + n_acc, out[1] = l_glo + |I_incache|.
 */
int orc_kv_compact(void *base, size_t elem, int n_layers, int n_kv_heads, int cap, int hd, int l_glo, int l_cache,
                   const int32_t *retain, int n_retain, int n_acc, int32_t *out) {
    if (l_glo < 0 || l_cache < l_glo || l_cache > cap || n_acc > n_retain) return ORC_EINVAL;
    int n_in = 0;
    for (int j = 0; j < n_retain; ++j) {
        if (retain[j] < 0 || (j > 0 && retain[j] <= retain[j - 1])) return ORC_EINVAL;
        if (l_glo + retain[j] < l_cache) ++n_in;
    }
    size_t row = elem * (size_t)hd;
    unsigned char *tmp = (unsigned char *)malloc(row * (size_t)(n_in > 0 ? n_in : 1));
    for (int l = 0; l < n_layers; ++l)
        for (int w = 0; w < 2; ++w)
            for (int h = 0; h < n_kv_heads; ++h) {
                unsigned char *head = (unsigned char *)base + ((((size_t)l * 2 + w) * n_kv_heads + h) * (size_t)cap) * row;
                int j = 0;
                for (int t = 0; t < n_retain; ++t)
                    if (l_glo + retain[t] < l_cache) memcpy(tmp + row * (size_t)(j++), head + row * (size_t)(l_glo + retain[t]), row);
                memcpy(head + row * (size_t)l_glo, tmp, row * (size_t)n_in);
            }
    free(tmp);
    out[0] = l_glo + n_acc;
    out[1] = l_glo + n_in;
    return ORC_OK;
}

/* I_local = { i - off : i in retain, 0 <= i - off < l_s } with off = l_cache - l_glo (the S index of the
 * segment's first row); rows are gathered in order.  Returns the pruned length. */
int orc_seg_prune(const void *seg_in, int l_s, size_t row_bytes, int off, const int32_t *retain, int n_retain, void *seg_out) {
    int n = 0;
    for (int t = 0; t < n_retain; ++t) {
        int loc = retain[t] - off;
        if (loc >= 0 && loc < l_s)
            memcpy((unsigned char *)seg_out + row_bytes * (size_t)(n++), (const unsigned char *)seg_in + row_bytes * (size_t)loc,
                   row_bytes);
    }
    return n;
}

/* Threads the "parallel for" loops above will use (reported beside CPU timings). */
#ifdef _OPENMP
#include <omp.h>
int orc_num_threads(void) { return omp_get_max_threads(); }
#else
int orc_num_threads(void) { return 1; }
#endif

/* ---- stochastic acceptance (temperature > 0) --------------------------------------------------------------------
 * The paper evaluates temperature 1 (Table I) with the acceptance rule of the speculative-decoding code base it
 * extends and prints no formula (Sec. III-C).  Reading taken: sequential candidate test.  At an accepted node u with
 * next-token distribution p_u = softmax(logits_u / temperature), the children of u are tried in S order; child c is
 * accepted with probability p_u(token[c]) / (mass still unrejected at u); a rejected token's mass is removed.  If no
 * child is accepted, x_new is drawn from the remaining distribution.  The emitted token is distributed exactly as p_u.
 *
 * To make every decision reproducible bit for bit on any machine, probabilities are integers:
 *   z_v = logits_v * inv_temp (fp32);  m = max_v z_v;  e_v = exp2_spec((z_v - m) * log2(e));  E_v = (uint64)(e_v * 2^32)
 *   Z = sum_v E_v (exact in 64-bit integers, any order)
 * and decisions compare integers: accept c iff r24 * R < E_c * 2^24, R the remaining mass; residual draw: the first v
 * whose running sum of unrejected E exceeds floor(u48 * R / 2^48).  Uniform numbers come from a counter-based
 * generator keyed by (seed, step, draw index).  exp2_spec is a fixed sequence of IEEE fp32 operations. */

static uint64_t orc_rng(uint64_t seed, uint64_t step, uint64_t k) {
    uint64_t z = seed ^ (step * 0x9E3779B97F4A7C15ull) ^ (k * 0xBF58476D1CE4E5B9ull);
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

static uint64_t orc_exp_weight(float z, float m) {
    const float t = (z - m) * 1.44269504088896341f;
    if (!(t >= -64.0f)) return 0;
    const float n = floorf(t), f = t - n;
    float p = 1.52527338e-5f;
    p = fmaf(p, f, 1.54035304e-4f);
    p = fmaf(p, f, 1.33335581e-3f);
    p = fmaf(p, f, 9.61812911e-3f);
    p = fmaf(p, f, 5.55041087e-2f);
    p = fmaf(p, f, 2.40226507e-1f);
    p = fmaf(p, f, 6.93147181e-1f);
    p = fmaf(p, f, 1.0f);
    return (uint64_t)(ldexpf(p, (int)n) * 4294967296.0f);
}

/* Probability weights of one row: E[v] for every v; returns Z.  (Used by the tests to check the distribution.) */
uint64_t orc_row_weights(const float *logits, int vocab, float inv_temp, uint64_t *E) {
    float m = -INFINITY;
    for (int v = 0; v < vocab; ++v) {
        float z = logits[v] * inv_temp;
        if (z > m) m = z;
    }
    uint64_t Z = 0;
    for (int v = 0; v < vocab; ++v) {
        uint64_t e = orc_exp_weight(logits[v] * inv_temp, m);
        if (E) E[v] = e;
        Z += e;
    }
    return Z;
}

int orc_accept_sample(const float *logits, int vocab, float inv_temp, const int32_t *token, const int32_t *parent, int T, int n_ver,
                      uint64_t seed, uint64_t step, orc_accept_result *res, int32_t *retain) {
    if (T <= 0 || n_ver < 0 || n_ver > T || vocab < 1 || !(inv_temp > 0.0f)) return ORC_EINVAL;
    for (int i = 0; i < T; ++i)
        if (parent[i] < -1 || parent[i] >= i) return ORC_ETOPO;
    if (parent[0] != -1) return ORC_ETOPO;
    if (n_ver == 0) {
        for (int i = 0; i < T; ++i) retain[i] = i;
        res->n_acc = 0; res->x_new = -1; res->n_new = 0; res->continuous = 1; res->n_retain = T; res->n_pr_verified = 0;
        return ORC_OK;
    }
    uint64_t *E = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)vocab);
    char *keep = (char *)calloc((size_t)T, 1);
    int32_t *rej = (int32_t *)malloc(sizeof(int32_t) * (size_t)T);
    uint64_t draw = 0;
    int u = 0, n_acc = 0, x_new = -1, n_new = -1;
    for (;;) {
        keep[u] = 1;
        ++n_acc;
        const float *row = logits + (size_t)u * vocab;
        uint64_t R = orc_row_weights(row, vocab, inv_temp, E);
        int n_rej = 0, next = -1;
        for (int c = u + 1; c < T && next < 0; ++c) {
            if (parent[c] != u) continue;
            int dup = 0;
            for (int k = 0; k < n_rej; ++k) dup |= (rej[k] == token[c]);
            if (dup || token[c] < 0 || token[c] >= vocab) continue;  /* already rejected here (or not a vocabulary id): no mass */
            const uint64_t Ec = E[token[c]];
            const uint64_t r24 = orc_rng(seed, step, draw++) >> 40;
            if ((unsigned __int128)r24 * R < ((unsigned __int128)Ec << 24)) {
                next = c;
            } else {
                R -= Ec;
                rej[n_rej++] = token[c];
            }
        }
        if (next >= 0 && next < n_ver) {  /* accepted and already verified: descend */
            u = next;
            continue;
        }
        if (next >= 0) {  /* accepted, not verified yet: it is the node n_new of the continuous condition */
            x_new = token[next];
            n_new = next;
        } else {          /* every candidate rejected: draw x_new from what is left */
            const uint64_t u48 = ((orc_rng(seed, step, draw) >> 40) << 24) | (orc_rng(seed, step, draw + 1) >> 40);
            draw += 2;
            const uint64_t target = (uint64_t)(((unsigned __int128)u48 * R) >> 48);
            uint64_t run = 0;
            x_new = vocab - 1;
            for (int v = 0; v < vocab; ++v) {
                int dup = 0;
                for (int k = 0; k < n_rej; ++k) dup |= (rej[k] == v);
                if (dup) continue;
                run += E[v];
                if (run > target) {
                    x_new = v;
                    break;
                }
            }
        }
        break;
    }
    int n_prv = 0;
    if (n_new >= 0) {
        keep[n_new] = 2;
        for (int i = n_new + 1; i < T; ++i)
            if (parent[i] >= 0 && keep[parent[i]] == 2) keep[i] = 2;
        for (int i = 0; i < n_ver; ++i) n_prv += (keep[i] == 2);
    }
    int n = 0;
    for (int i = 0; i < T; ++i)
        if (keep[i] == 1) retain[n++] = i;
    for (int i = 0; i < T; ++i)
        if (keep[i] == 2) retain[n++] = i;
    res->n_acc = n_acc; res->x_new = x_new; res->n_new = n_new; res->continuous = (n_new >= 0);
    res->n_retain = n; res->n_pr_verified = n_prv;
    free(E); free(keep); free(rej);
    return ORC_OK;
}
