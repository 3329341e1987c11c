/*
 * CPU oracle for the budgeted-KV decode + evict path of ForesightKV.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * path computes; the tests, the smoke check and the benchmark's cpu_baseline leg
 * call it, the product never does.  It shares no code, header, table or helper
 * with the HIP library.
 *
 * Everything floating point is evaluated in double precision from the stored
 * bits of the inputs (fp32 words or bf16 half-words, widened exactly).  There is
 * no blocking, fusion or reordering beyond what the definitions state.
 *
 * Cache layout (row major):
 *   K, V  [batch][n_kv_heads][capacity][head_dim]   storage type
 *   pos   [batch][n_kv_heads][capacity]             int32 absolute position ids
 *   len   [batch]                                   int32 retained count (same for all heads)
 *
 * What each function follows:
 *   ora_decode_attn   retained-set attention with renormalised softmax
 *                     (Appendix A, "Problem Setup": o_hat = sum_{i in S} a_hat_i v_i).
 *   ora_score_kv      MLP scorer phi = sigma(x W1 + b1) W2 + b2 on x = concat(k, v)
 *                     (Appendix B.1, Model Design; Section 3.1 Eq. 1 without the
 *                     attention features), sigma = exact erf GELU.
 *   ora_decode_attn_probs, ora_score_kv_feat
 *                     the same two with the paper's attention features: the attention weights
 *                     are returned per slot, and the scorer takes x = concat(k, v, a)
 *                     (Appendix B.1); the feature bookkeeping itself is in __init__.py.
 *   ora_select_keep   keep the most recent R pairs and the top (B - R) of the others by
 *                     importance (Section 3.1, eviction protocol; Top_{B-L} of Eq. 5;
 *                     deterministic Top-K variant of the sampling ablation).
 *   ora_select_keep_sampled
 *                     Top-K multinomial eviction (Section 3.1 Eq. 2, Appendix B.2): the n_cand
 *                     lowest-scored pairs are candidates, the evicted ones are drawn from them
 *                     without replacement with probabilities softmax(-phi); the draw is taken in
 *                     its Gumbel-top-k form on noise handed in by the caller.
 *   ora_compact       drop the evicted pairs, order preserved (Section 1: evicted pairs are
 *                     gone for good; the stable order is this build's definition).
 *   ora_append        one generated token joins every KV-head row (Section 3.1).
 *
 * Parity pins for every function live in tests/test_oracle_*.py; none is unpinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORA_F32 = 0, ORA_BF16 = 1 };

static int g_threads = 1;

void ora_set_threads(int n) { g_threads = n < 1 ? 1 : n; }

int ora_get_threads(void) { return g_threads; }

int ora_max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* widen one stored element to double (exact) */
static inline double ld(const void *p, int dtype, int64_t i) {
    if (dtype == ORA_F32) return (double)((const float *)p)[i];
    uint32_t u = ((uint32_t)((const uint16_t *)p)[i]) << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

static inline size_t esize(int dtype) { return dtype == ORA_F32 ? 4 : 2; }

/* ------------------------------------------------------------------------- */
/* append: slot len[b] of every KV-head row receives (k_new, v_new, pos_new)   */
/* ------------------------------------------------------------------------- */
int ora_append(int dtype, int batch, int n_kv, int D, int cap, void *K, void *V, int32_t *pos,
               int32_t *len, const void *k_new, const void *v_new, const int32_t *pos_new) {
    size_t es = esize(dtype);
    for (int b = 0; b < batch; ++b) {
        int n = len[b];
        if (n >= cap) return 1;
        for (int h = 0; h < n_kv; ++h) {
            int64_t row = (int64_t)b * n_kv + h;
            memcpy((char *)K + ((row * cap + n) * D) * es, (const char *)k_new + (row * D) * es, D * es);
            memcpy((char *)V + ((row * cap + n) * D) * es, (const char *)v_new + (row * D) * es, D * es);
            pos[row * cap + n] = pos_new[b];
        }
        len[b] = n + 1;
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* attention over the retained set                                            */
/*   s_i = scale <q, k_i>;  a_hat_i = exp(s_i) / sum_{k in S} exp(s_k);        */
/*   o_hat = sum_{i in S} a_hat_i v_i          (S = slots 0 .. len-1)          */
/* The maximum logit is subtracted before exp; that changes nothing in exact   */
/* arithmetic and keeps exp in range.                                          */
/* out: double [batch][n_q][D]; rows with len == 0 give zeros.                 */
/* ------------------------------------------------------------------------- */
void ora_decode_attn(int dtype, int batch, int n_q, int n_kv, int D, int cap, const void *q,
                     const void *K, const void *V, const int32_t *len, double scale, double *out) {
    int g = n_q / n_kv;
#pragma omp parallel for num_threads(g_threads) schedule(dynamic, 1)
    for (int bh = 0; bh < batch * n_q; ++bh) {
        int b = bh / n_q, hq = bh % n_q, hk = hq / g;
        int n = len[b];
        int64_t row = (int64_t)b * n_kv + hk;
        double *o = out + (int64_t)bh * D;
        for (int d = 0; d < D; ++d) o[d] = 0.0;
        if (n <= 0) continue;
        double *s = (double *)malloc(sizeof(double) * (size_t)n);
        double m = -INFINITY;
        for (int i = 0; i < n; ++i) {
            double acc = 0.0;
            for (int d = 0; d < D; ++d)
                acc += ld(q, dtype, (int64_t)bh * D + d) * ld(K, dtype, (row * cap + i) * D + d);
            s[i] = scale * acc;
            if (s[i] > m) m = s[i];
        }
        double z = 0.0;
        for (int i = 0; i < n; ++i) {
            s[i] = exp(s[i] - m);
            z += s[i];
        }
        for (int i = 0; i < n; ++i) {
            double a = s[i] / z;
            for (int d = 0; d < D; ++d) o[d] += a * ld(V, dtype, (row * cap + i) * D + d);
        }
        free(s);
    }
}

/* Same attention, also returning the weights a_hat (Appendix A) of every live slot:             */
/* probs double [batch][n_q][cap], slots >= len untouched.  They feed the attention features    */
/* of the scoring model (Appendix B.1, "Attention Features").                                   */
void ora_decode_attn_probs(int dtype, int batch, int n_q, int n_kv, int D, int cap, const void *q,
                           const void *K, const void *V, const int32_t *len, double scale,
                           double *out, double *probs) {
    int g = n_q / n_kv;
#pragma omp parallel for num_threads(g_threads) schedule(dynamic, 1)
    for (int bh = 0; bh < batch * n_q; ++bh) {
        int b = bh / n_q, hq = bh % n_q, hk = hq / g;
        int n = len[b];
        int64_t row = (int64_t)b * n_kv + hk;
        double *o = out + (int64_t)bh * D;
        double *pr = probs + (int64_t)bh * cap;
        for (int d = 0; d < D; ++d) o[d] = 0.0;
        if (n <= 0) continue;
        double m = -INFINITY;
        for (int i = 0; i < n; ++i) {
            double acc = 0.0;
            for (int d = 0; d < D; ++d)
                acc += ld(q, dtype, (int64_t)bh * D + d) * ld(K, dtype, (row * cap + i) * D + d);
            pr[i] = scale * acc;
            if (pr[i] > m) m = pr[i];
        }
        double z = 0.0;
        for (int i = 0; i < n; ++i) {
            pr[i] = exp(pr[i] - m);
            z += pr[i];
        }
        for (int i = 0; i < n; ++i) {
            pr[i] /= z;
            for (int d = 0; d < D; ++d) o[d] += pr[i] * ld(V, dtype, (row * cap + i) * D + d);
        }
    }
}

/* ------------------------------------------------------------------------- */
/* scorer: phi_n = sum_j gelu( sum_f x_{n,f} W1[f][j] + b1[j] ) W2[j] + b2,     */
/*         x_n = [k_n, v_n]  (F = 2D)                                          */
/* W1 [n_kv or 1][2D][H] storage type; b1, W2 [.][H] fp32; b2 [.] fp32.        */
/* shared != 0: one weight set for all KV heads.                               */
/* scores: double [batch][n_kv][cap]; slots >= len are left untouched.         */
/* ------------------------------------------------------------------------- */
static inline double gelu_erf(double x) { return 0.5 * x * (1.0 + erf(x / sqrt(2.0))); }

void ora_score_kv(int dtype, int batch, int n_kv, int D, int cap, const void *K, const void *V,
                  const int32_t *len, const void *W1, const float *b1, const float *W2,
                  const float *b2, int H, int shared, double *scores) {
    int F = 2 * D;
#pragma omp parallel for num_threads(g_threads) schedule(dynamic, 1)
    for (int row = 0; row < batch * n_kv; ++row) {
        int b = row / n_kv, h = row % n_kv;
        int hw = shared ? 0 : h;
        int n = len[b];
        double *x = (double *)malloc(sizeof(double) * (size_t)F);
        double *w = (double *)malloc(sizeof(double) * (size_t)F * H);
        /* private widened copy of this head's W1, stored hidden-major: w[j*F + f] = W1[f][j] */
        for (int f = 0; f < F; ++f)
            for (int j = 0; j < H; ++j)
                w[(int64_t)j * F + f] = ld(W1, dtype, ((int64_t)hw * F + f) * H + j);
        for (int i = 0; i < n; ++i) {
            int64_t base = ((int64_t)row * cap + i) * D;
            for (int d = 0; d < D; ++d) {
                x[d] = ld(K, dtype, base + d);
                x[D + d] = ld(V, dtype, base + d);
            }
            double phi = 0.0;
            for (int j = 0; j < H; ++j) {
                double z = 0.0;
                for (int f = 0; f < F; ++f) z += x[f] * w[(int64_t)j * F + f];
                z += (double)b1[(int64_t)hw * H + j];
                phi += gelu_erf(z) * (double)W2[(int64_t)hw * H + j];
            }
            scores[(int64_t)row * cap + i] = phi + (double)b2[hw];
        }
        free(x);
        free(w);
    }
}

/* Scorer on the paper's full input x_n = [k_n, v_n, a_n] (Section 3.1 Eq. 1, Appendix B.1):     */
/* a_n = the A attention features of the pair (fp64 here), W1 [.][2D + A][H] storage type with   */
/* the rows in the order k, v, a.                                                               */
void ora_score_kv_feat(int dtype, int batch, int n_kv, int D, int cap, const void *K, const void *V,
                       const double *feat /* [batch][n_kv][cap][A] */, int A, const int32_t *len,
                       const void *W1, const float *b1, const float *W2, const float *b2, int H,
                       int shared, double *scores) {
    int F = 2 * D + A;
#pragma omp parallel for num_threads(g_threads) schedule(dynamic, 1)
    for (int row = 0; row < batch * n_kv; ++row) {
        int b = row / n_kv, h = row % n_kv;
        int hw = shared ? 0 : h;
        int n = len[b];
        double *x = (double *)malloc(sizeof(double) * (size_t)F);
        double *w = (double *)malloc(sizeof(double) * (size_t)F * H);
        for (int f = 0; f < F; ++f)
            for (int j = 0; j < H; ++j)
                w[(int64_t)j * F + f] = ld(W1, dtype, ((int64_t)hw * F + f) * H + j);
        for (int i = 0; i < n; ++i) {
            int64_t base = ((int64_t)row * cap + i) * D;
            for (int d = 0; d < D; ++d) {
                x[d] = ld(K, dtype, base + d);
                x[D + d] = ld(V, dtype, base + d);
            }
            for (int a = 0; a < A; ++a) x[2 * D + a] = feat[((int64_t)row * cap + i) * A + a];
            double phi = 0.0;
            for (int j = 0; j < H; ++j) {
                double z = 0.0;
                for (int f = 0; f < F; ++f) z += x[f] * w[(int64_t)j * F + f];
                z += (double)b1[(int64_t)hw * H + j];
                phi += gelu_erf(z) * (double)W2[(int64_t)hw * H + j];
            }
            scores[(int64_t)row * cap + i] = phi + (double)b2[hw];
        }
        free(x);
        free(w);
    }
}

/* ------------------------------------------------------------------------- */
/* selection                                                                  */
/* Total order on the candidates of a row: a "beats" b when                    */
/*   score_a > score_b, or the scores are equal and pos_a < pos_b.             */
/* -0.0 equals +0.0; NaN ranks below -inf and NaNs are equal to each other.    */
/* Positions within a row are distinct, so the order is total.                 */
/* ------------------------------------------------------------------------- */
static inline int beats(float sa, int32_t pa, float sb, int32_t pb) {
    int na = isnan(sa), nb = isnan(sb);
    if (na || nb) {
        if (na && nb) return pa < pb;
        return nb; /* a is a number, b is NaN -> a beats b */
    }
    if (sa > sb) return 1;
    if (sa < sb) return 0;
    return pa < pb;
}

/* kept[] flags for one row by rank counting (O(n^2)). */
static void select_row_rank(int n, const float *sc, const int32_t *ps, int budget, int R,
                            uint8_t *kept) {
    /* protected: the R entries with the largest positions */
    for (int i = 0; i < n; ++i) {
        int newer = 0;
        for (int j = 0; j < n; ++j) newer += ps[j] > ps[i];
        kept[i] = newer < R ? 2 : 0;
    }
    int k = budget - R;
    for (int i = 0; i < n; ++i) {
        if (kept[i]) continue;
        int rank = 0;
        for (int j = 0; j < n; ++j)
            if (!(kept[j] & 2) && j != i) rank += beats(sc[j], ps[j], sc[i], ps[i]);
        if (rank < k) kept[i] = 1;
    }
}

typedef struct {
    float s;
    int32_t p;
    int32_t slot;
} cand_t;

static int cmp_pos_desc(const void *a, const void *b) {
    int32_t pa = ((const cand_t *)a)->p, pb = ((const cand_t *)b)->p;
    return pa > pb ? -1 : (pa < pb ? 1 : 0);
}

static int cmp_importance(const void *a, const void *b) {
    const cand_t *x = (const cand_t *)a, *y = (const cand_t *)b;
    if (beats(x->s, x->p, y->s, y->p)) return -1;
    if (beats(y->s, y->p, x->s, x->p)) return 1;
    return 0;
}

/* kept[] flags for one row by sorting (second, independent formulation). */
static void select_row_sort(int n, const float *sc, const int32_t *ps, int budget, int R,
                            uint8_t *kept) {
    cand_t *c = (cand_t *)malloc(sizeof(cand_t) * (size_t)n);
    for (int i = 0; i < n; ++i) {
        c[i].s = sc[i];
        c[i].p = ps[i];
        c[i].slot = i;
        kept[i] = 0;
    }
    qsort(c, (size_t)n, sizeof(cand_t), cmp_pos_desc);
    for (int i = 0; i < R; ++i) kept[c[i].slot] = 2;
    qsort(c + R, (size_t)(n - R), sizeof(cand_t), cmp_importance);
    for (int i = 0; i < budget - R; ++i) kept[c[R + i].slot] = 1;
    free(c);
}

/*
 * keep_idx [batch][n_kv][budget] int32: the kept slots of each row in ascending slot
 * order.  Rows with len <= budget keep everything: keep_idx[j] = j for j < len, the
 * rest of the row is left untouched.  method 0 = rank counting, 1 = sorting.
 * Returns 0, or 1 on bad arguments (R > budget, budget > cap).
 */
int ora_select_keep(int batch, int n_kv, int cap, const float *scores, const int32_t *pos,
                    const int32_t *len, int budget, int R, int method, int32_t *keep_idx) {
    if (R > budget || budget > cap || R < 0) return 1;
    int rc = 0;
#pragma omp parallel for num_threads(g_threads) schedule(dynamic, 1)
    for (int row = 0; row < batch * n_kv; ++row) {
        int b = row / n_kv;
        int n = len[b];
        int32_t *out = keep_idx + (int64_t)row * budget;
        if (n <= budget) {
            for (int j = 0; j < n; ++j) out[j] = j;
            continue;
        }
        uint8_t *kept = (uint8_t *)malloc((size_t)n);
        const float *sc = scores + (int64_t)row * cap;
        const int32_t *ps = pos + (int64_t)row * cap;
        if (method == 0)
            select_row_rank(n, sc, ps, budget, R, kept);
        else
            select_row_sort(n, sc, ps, budget, R, kept);
        int c = 0;
        for (int i = 0; i < n; ++i)
            if (kept[i]) {
                if (c < budget) out[c] = i;
                ++c;
            }
        if (c != budget) {
#pragma omp atomic write
            rc = 2;
        }
        free(kept);
    }
    return rc;
}

/* ------------------------------------------------------------------------- */
/* sampled selection (Top-K multinomial eviction, Section 3.1 Eq. 2 / Appendix B.2)           */
/* Row with n > budget entries, E = n - budget to evict, R newest protected:                  */
/*   1. order the other n - R pairs by importance (score desc, position asc);                 */
/*      the n_cand LAST of them (lowest scores) are the candidates (all, if fewer);            */
/*      n_cand is raised to E when it is smaller.  The rest are safe.                          */
/*   2. draw E of the candidates without replacement with probabilities softmax(-score).      */
/*      Sequential draws with renormalisation have the same law as taking the E largest of     */
/*      -score_i + g_i with g_i iid Gumbel(0,1) (Gumbel-top-k).  noise[] holds the g_i; the    */
/*      perturbed key is formed in fp32, t_i = score_i - noise_i (= -(-score_i + noise_i)      */
/*      exactly), so the E smallest t_i are evicted: the candidates are ordered by             */
/*      (t desc, position asc) and the first n_cand - E stay.                                  */
/* noise == 0 everywhere, or n_cand <= E, gives ora_select_keep's result.                      */
/* ------------------------------------------------------------------------- */
int ora_select_keep_sampled(int batch, int n_kv, int cap, const float *scores, const float *noise,
                            const int32_t *pos, const int32_t *len, int budget, int R, int n_cand,
                            int32_t *keep_idx) {
    if (R > budget || budget > cap || R < 0 || n_cand < 0) return 1;
    int rc = 0;
#pragma omp parallel for num_threads(g_threads) schedule(dynamic, 1)
    for (int row = 0; row < batch * n_kv; ++row) {
        int b = row / n_kv;
        int n = len[b];
        int32_t *out = keep_idx + (int64_t)row * budget;
        if (n <= budget) {
            for (int j = 0; j < n; ++j) out[j] = j;
            continue;
        }
        const float *sc = scores + (int64_t)row * cap;
        const float *nz = noise + (int64_t)row * cap;
        const int32_t *ps = pos + (int64_t)row * cap;
        uint8_t *kept = (uint8_t *)calloc((size_t)n, 1);
        cand_t *c = (cand_t *)malloc(sizeof(cand_t) * (size_t)n);
        for (int i = 0; i < n; ++i) {
            c[i].s = sc[i];
            c[i].p = ps[i];
            c[i].slot = i;
        }
        qsort(c, (size_t)n, sizeof(cand_t), cmp_pos_desc);
        for (int i = 0; i < R; ++i) kept[c[i].slot] = 1;
        int others = n - R, E = n - budget;
        int K = n_cand < E ? E : n_cand;
        if (K > others) K = others;
        qsort(c + R, (size_t)others, sizeof(cand_t), cmp_importance);
        for (int i = 0; i < others - K; ++i) kept[c[R + i].slot] = 1; /* safe */
        cand_t *cd = c + R + (others - K);                              /* the K candidates */
        for (int i = 0; i < K; ++i) cd[i].s = sc[cd[i].slot] - nz[cd[i].slot]; /* fp32 subtraction */
        qsort(cd, (size_t)K, sizeof(cand_t), cmp_importance);
        for (int i = 0; i < K - E; ++i) kept[cd[i].slot] = 1;
        int cnt = 0;
        for (int i = 0; i < n; ++i)
            if (kept[i]) {
                if (cnt < budget) out[cnt] = i;
                ++cnt;
            }
        if (cnt != budget) {
#pragma omp atomic write
            rc = 2;
        }
        free(c);
        free(kept);
    }
    return rc;
}

/* ------------------------------------------------------------------------- */
/* compaction: for rows with len > budget, slot j <- slot keep_idx[j],          */
/* j = 0 .. budget-1, for K, V and pos; then len = budget.  Written as a gather */
/* into a fresh copy of the row, then copied back.                             */
/* ------------------------------------------------------------------------- */
void ora_compact(int dtype, int batch, int n_kv, int D, int cap, void *K, void *V, int32_t *pos,
                 int32_t *len, const int32_t *keep_idx, int budget) {
    size_t rb = (size_t)D * esize(dtype);
#pragma omp parallel for num_threads(g_threads) schedule(dynamic, 1)
    for (int row = 0; row < batch * n_kv; ++row) {
        int b = row / n_kv;
        if (len[b] <= budget) continue;
        char *k = (char *)K + (size_t)row * cap * rb;
        char *v = (char *)V + (size_t)row * cap * rb;
        int32_t *p = pos + (int64_t)row * cap;
        const int32_t *idx = keep_idx + (int64_t)row * budget;
        char *nk = (char *)malloc(rb * (size_t)budget);
        char *nv = (char *)malloc(rb * (size_t)budget);
        int32_t *np_ = (int32_t *)malloc(sizeof(int32_t) * (size_t)budget);
        for (int j = 0; j < budget; ++j) {
            memcpy(nk + (size_t)j * rb, k + (size_t)idx[j] * rb, rb);
            memcpy(nv + (size_t)j * rb, v + (size_t)idx[j] * rb, rb);
            np_[j] = p[idx[j]];
        }
        memcpy(k, nk, rb * (size_t)budget);
        memcpy(v, nv, rb * (size_t)budget);
        memcpy(p, np_, sizeof(int32_t) * (size_t)budget);
        free(nk);
        free(nv);
        free(np_);
    }
    for (int b = 0; b < batch; ++b)
        if (len[b] > budget) len[b] = budget;
}
