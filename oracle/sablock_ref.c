/*
 * sablock_ref.c -- plain fp64 CPU oracle of the SABlock compression path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the parity reference for the HIP
 * library; it is slow on purpose, shares no code with it, and must never be
 * called from the product path (only tests, the smoke check and the benchmark's
 * cpu_baseline leg use it).
 *
 * Every function works on ONE KV head of ONE (sequence, layer): callers loop.
 * All arithmetic is double precision; inputs are the bf16/fp32 values widened
 * exactly to double by the caller.  Steps follow the paper's order and
 * notation (Sec. 3.2, Alg. 1, Eqs. barA/st/Ik/Dk/omegak/st_tilde; Sec. 3.3,
 * Alg. 2, Eqs. topk/implicit_budget/rk/gk_star/final_selection) with no
 * blocking, fusion or reordering.  Where the paper is silent the reading taken
 * is stated at the step.
 *
 * Pins (tests/test_oracle_pins.py): library softmax on the single-row case,
 * closed forms for Q == 0, column sums adding up to W, a one-hot construction,
 * hand-computed refinement and block-search examples, a library full sort for
 * the Top-B set, brute-force enumeration of every candidate block size, and
 * the invariants the paper states (|T*| = B, R_k(g) <= 1, g = 1 is token-level
 * top-k, blocks never leave their segment).  No function is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    double v;
    int32_t idx;
} ref_item;

/* order used everywhere a ranking is needed: value descending, index ascending
 * (the paper does not say how ties are broken; this is the reading taken) */
static int cmp_desc(const void *a, const void *b)
{
    const ref_item *x = (const ref_item *)a, *y = (const ref_item *)b;
    if (x->v > y->v) return -1;
    if (x->v < y->v) return 1;
    return (x->idx > y->idx) - (x->idx < y->idx);
}

/* ------------------------------------------------------------------------
 * Window scoring (Sec. 3.2; Eq. barA, Eq. st, inner sum of Eq. Dk).
 *
 * q [G][W][D] : window queries of the G query heads sharing this KV head;
 *               query i sits at absolute position T + i, T = L - W
 * k [L][D]    : all cached keys of this KV head
 * s [L], e[L] : outputs.
 *
 * A[h,i,t] is the softmax over the keys query i can see (t <= T + i, causal
 * inside the window, the SnapKV convention the paper cites) of
 * <q_hi, k_t>/sqrt(D) (Eq. 1).  Abar is the mean over the G heads (Eq. barA,
 * taken per KV head), s_t = sum_i Abar[i,t] (Eq. st) and
 * e_t = -sum_i Ahat[i,t] ln(Ahat[i,t] + eps), Ahat = Abar / s_t (the per-token
 * term that Eq. Dk averages over a segment; natural log).  Masked entries have
 * Abar = 0 and contribute 0; e_t = 0 if s_t = 0.
 * ---------------------------------------------------------------------- */
int sablock_ref_score(const double *q, const double *k, int32_t G, int32_t W, int32_t D, int32_t L,
                      double eps, double *s, double *e)
{
    if (!q || !k || !s || !e || G <= 0 || W <= 0 || D <= 0 || L <= W) return 1;
    const int32_t T = L - W;
    double *abar = (double *)calloc((size_t)W * (size_t)L, sizeof(double));
    double *x = (double *)malloc((size_t)L * sizeof(double));
    if (!abar || !x) { free(abar); free(x); return 2; }
    const double scale = 1.0 / sqrt((double)D);

    for (int32_t h = 0; h < G; ++h) {
        for (int32_t i = 0; i < W; ++i) {
            const double *qr = q + ((size_t)h * W + i) * D;
            const int32_t nvis = T + i + 1;
            double m = -INFINITY;
            for (int32_t t = 0; t < nvis; ++t) {
                const double *kr = k + (size_t)t * D;
                double dot = 0.0;
                for (int32_t d = 0; d < D; ++d) dot += qr[d] * kr[d];
                x[t] = dot * scale;
                if (x[t] > m) m = x[t];
            }
            double z = 0.0;
            for (int32_t t = 0; t < nvis; ++t) z += exp(x[t] - m);
            double *row = abar + (size_t)i * L;
            for (int32_t t = 0; t < nvis; ++t) row[t] += exp(x[t] - m) / z;
        }
    }
    for (size_t j = 0; j < (size_t)W * (size_t)L; ++j) abar[j] /= (double)G;

    for (int32_t t = 0; t < L; ++t) {
        double st = 0.0;
        for (int32_t i = 0; i < W; ++i) st += abar[(size_t)i * L + t];
        s[t] = st;
        double ent = 0.0;
        if (st > 0.0) {
            for (int32_t i = 0; i < W; ++i) {
                double ah = abar[(size_t)i * L + t] / st;
                ent -= ah * log(ah + eps);
            }
        }
        e[t] = ent;
    }
    free(abar);
    free(x);
    return 0;
}

/* ------------------------------------------------------------------------
 * Window scoring with the head mean taken literally (Eq. barA averages over
 * ALL H query heads of the layer): one score row per layer instead of one per
 * KV head.
 *
 * q [Hq][W][D] : window queries of every query head of the layer
 * k [Hkv][L][D]: keys of every KV head; query head h reads KV head h / (Hq/Hkv)
 * s [L], e [L] : outputs, defined as in sablock_ref_score with Abar the mean
 *                over the Hq heads.
 * ---------------------------------------------------------------------- */
int sablock_ref_score_layer(const double *q, const double *k, int32_t Hq, int32_t Hkv, int32_t W, int32_t D,
                            int32_t L, double eps, double *s, double *e)
{
    if (!q || !k || !s || !e || Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0 || W <= 0 || D <= 0 || L <= W) return 1;
    const int32_t T = L - W, G = Hq / Hkv;
    double *abar = (double *)calloc((size_t)W * (size_t)L, sizeof(double));
    double *x = (double *)malloc((size_t)L * sizeof(double));
    if (!abar || !x) { free(abar); free(x); return 2; }
    const double scale = 1.0 / sqrt((double)D);

    for (int32_t h = 0; h < Hq; ++h) {
        const double *kh = k + (size_t)(h / G) * (size_t)L * D;
        for (int32_t i = 0; i < W; ++i) {
            const double *qr = q + ((size_t)h * W + i) * D;
            const int32_t nvis = T + i + 1;
            double m = -INFINITY;
            for (int32_t t = 0; t < nvis; ++t) {
                const double *kr = kh + (size_t)t * D;
                double dot = 0.0;
                for (int32_t d = 0; d < D; ++d) dot += qr[d] * kr[d];
                x[t] = dot * scale;
                if (x[t] > m) m = x[t];
            }
            double z = 0.0;
            for (int32_t t = 0; t < nvis; ++t) z += exp(x[t] - m);
            double *row = abar + (size_t)i * L;
            for (int32_t t = 0; t < nvis; ++t) row[t] += exp(x[t] - m) / z;
        }
    }
    for (size_t j = 0; j < (size_t)W * (size_t)L; ++j) abar[j] /= (double)Hq;

    for (int32_t t = 0; t < L; ++t) {
        double st = 0.0;
        for (int32_t i = 0; i < W; ++i) st += abar[(size_t)i * L + t];
        s[t] = st;
        double ent = 0.0;
        if (st > 0.0) {
            for (int32_t i = 0; i < W; ++i) {
                double ah = abar[(size_t)i * L + t] / st;
                ent -= ah * log(ah + eps);
            }
        }
        e[t] = ent;
    }
    free(abar);
    free(x);
    return 0;
}

/* ------------------------------------------------------------------------
 * Segment-guided refinement (Alg. 1; Eqs. Ik, Dk, omegak, st_tilde).
 * seg_off[0..K]: 0 = o_0 < ... < o_K = T, segment k = [o_k, o_{k+1}).
 * ---------------------------------------------------------------------- */
int sablock_ref_refine(const double *s, const double *e, int32_t T, const int32_t *seg_off, int32_t K,
                       double alpha, double eta, double *s_tilde, double *omega /* nullable */)
{
    if (!s || !e || !seg_off || !s_tilde || T < 0 || K < 0) return 1;
    for (int32_t k = 0; k < K; ++k) {
        const int32_t a = seg_off[k], b = seg_off[k + 1];
        if (a < 0 || b > T || b <= a) return 1;
        double sum_s = 0.0, sum_e = 0.0;
        for (int32_t t = a; t < b; ++t) { sum_s += s[t]; sum_e += e[t]; }
        const double Ik = sum_s / (double)(b - a);        /* Eq. Ik */
        const double Dk = sum_e / (double)(b - a);        /* Eq. Dk */
        const double wk = Ik * (1.0 + eta * Dk);          /* Eq. omegak */
        if (omega) omega[k] = wk;
        for (int32_t t = a; t < b; ++t) s_tilde[t] = s[t] * (1.0 + alpha * wk); /* Eq. st_tilde */
    }
    return 0;
}

/* Top-B membership flags (Eq. topk): the first min(B,T) tokens under
 * (score descending, index ascending). */
static int topb_flags(const double *st, int32_t T, int32_t B, unsigned char *flag)
{
    memset(flag, 0, (size_t)T);
    if (T == 0 || B <= 0) return 0;
    ref_item *it = (ref_item *)malloc((size_t)T * sizeof(ref_item));
    if (!it) return 2;
    for (int32_t t = 0; t < T; ++t) { it[t].v = st[t]; it[t].idx = t; }
    qsort(it, (size_t)T, sizeof(ref_item), cmp_desc);
    const int32_t n = B < T ? B : T;
    for (int32_t r = 0; r < n; ++r) flag[it[r].idx] = 1;
    free(it);
    return 0;
}

/* ------------------------------------------------------------------------
 * One pass of Alg. 2's inner loop for segment [a,b) and block size g with
 * implicit budget bk: partition from the segment's first token (the last block
 * may be short), Phi = block sum, visit blocks by (Phi descending, block index
 * ascending); a block that still fits is taken whole, the first one that does
 * not is cut to its Top-(bk - n) tokens and the walk stops.
 * take[0..b-a) receives the membership of T_k(g); returns Score_k(g), summed
 * over the taken tokens in ascending index.
 * ---------------------------------------------------------------------- */
static double greedy_fill(const double *st, int32_t a, int32_t b, int32_t g, int32_t bk,
                          unsigned char *take)
{
    const int32_t len = b - a;
    const int32_t nb = (len + g - 1) / g;
    memset(take, 0, (size_t)len);
    ref_item *blk = (ref_item *)malloc((size_t)nb * sizeof(ref_item));
    ref_item *tok = (ref_item *)malloc((size_t)g * sizeof(ref_item));
    for (int32_t m = 0; m < nb; ++m) {
        const int32_t lo = a + m * g, hi = (lo + g < b) ? lo + g : b;
        double phi = 0.0;
        for (int32_t t = lo; t < hi; ++t) phi += st[t];
        blk[m].v = phi;
        blk[m].idx = m;
    }
    qsort(blk, (size_t)nb, sizeof(ref_item), cmp_desc);
    int32_t n = 0;
    for (int32_t r = 0; r < nb; ++r) {
        const int32_t m = blk[r].idx;
        const int32_t lo = a + m * g, hi = (lo + g < b) ? lo + g : b;
        const int32_t sz = hi - lo;
        if (n + sz <= bk) {
            for (int32_t t = lo; t < hi; ++t) take[t - a] = 1;
            n += sz;
        } else {
            const int32_t rem = bk - n;
            for (int32_t t = lo; t < hi; ++t) { tok[t - lo].v = st[t]; tok[t - lo].idx = t; }
            qsort(tok, (size_t)sz, sizeof(ref_item), cmp_desc);
            for (int32_t j = 0; j < rem; ++j) take[tok[j].idx - a] = 1;
            break;
        }
    }
    double score = 0.0;
    for (int32_t t = a; t < b; ++t) if (take[t - a]) score += st[t];
    free(blk);
    free(tok);
    return score;
}

/* ------------------------------------------------------------------------
 * Budget-driven block-size search (Alg. 2 up to the accept rule; Eqs. topk,
 * implicit_budget, rk, gk_star).
 *
 * cand[0..n_cand) ascending, cand[0] == 1 (the candidate list is an argument;
 * g_max = cand[n_cand-1]).  Outputs b_k (Eq. implicit_budget) and g_k*
 * (0 where b_k = 0: nothing is kept from that segment).  The accept test
 * R_k(g) >= tau is evaluated as Score_k(g) >= tau * Score_k^base; g = 1 is the
 * unconditional last resort (Sec. 3.3, the text after Eq. gk_star).
 * ---------------------------------------------------------------------- */
int sablock_ref_search_blocks(const double *st, int32_t T, const int32_t *seg_off, int32_t K,
                              const int32_t *cand, int32_t n_cand, int32_t B, double tau,
                              int32_t *b_out, int32_t *g_out)
{
    if (!st || !seg_off || !cand || !b_out || !g_out || n_cand <= 0 || cand[0] != 1 || B < 0) return 1;
    for (int32_t c = 1; c < n_cand; ++c) if (cand[c] <= cand[c - 1]) return 1;
    unsigned char *flag = (unsigned char *)malloc((size_t)(T > 0 ? T : 1));
    unsigned char *take = (unsigned char *)malloc((size_t)(T > 0 ? T : 1));
    if (!flag || !take) { free(flag); free(take); return 2; }
    int rc = topb_flags(st, T, B, flag);
    if (rc) { free(flag); free(take); return rc; }

    for (int32_t k = 0; k < K; ++k) {
        const int32_t a = seg_off[k], b = seg_off[k + 1];
        const int32_t len = b - a;
        int32_t bk = 0;
        double base = 0.0;                              /* Score_k^base */
        for (int32_t t = a; t < b; ++t) if (flag[t]) { ++bk; base += st[t]; }
        b_out[k] = bk;
        g_out[k] = 0;
        if (bk == 0) continue;
        const int32_t gcap = len < bk ? len : bk;       /* G_k: g <= min(|S_k|, b_k, g_max) */
        for (int32_t c = n_cand - 1; c >= 0; --c) {
            const int32_t g = cand[c];
            if (g > gcap) continue;
            if (g == 1) { g_out[k] = 1; break; }
            const double score = greedy_fill(st, a, b, g, bk, take);
            if (score >= tau * base) { g_out[k] = g; break; }
        }
    }
    free(flag);
    free(take);
    return 0;
}

/* ------------------------------------------------------------------------
 * Selection (Alg. 2's T_k* = T_k(g_k*) and Eq. final_selection): the union of
 * the per-segment sets, written in ascending token index.  idx_out has room
 * for B entries; entries past n_sel are set to -1.
 * ---------------------------------------------------------------------- */
int sablock_ref_select(const double *st, int32_t T, const int32_t *seg_off, int32_t K,
                       const int32_t *bk, const int32_t *gk, int32_t B,
                       int32_t *idx_out, int32_t *n_sel_out)
{
    if (!st || !seg_off || !bk || !gk || !idx_out || !n_sel_out || B < 0) return 1;
    unsigned char *take = (unsigned char *)malloc((size_t)(T > 0 ? T : 1));
    if (!take) return 2;
    int32_t n = 0;
    for (int32_t k = 0; k < K; ++k) {
        if (bk[k] <= 0 || gk[k] <= 0) continue;
        const int32_t a = seg_off[k], b = seg_off[k + 1];
        greedy_fill(st, a, b, gk[k], bk[k], take);
        for (int32_t t = a; t < b; ++t) {
            if (take[t - a]) {
                if (n >= B) { free(take); return 3; }
                idx_out[n++] = t;
            }
        }
    }
    for (int32_t j = n; j < B; ++j) idx_out[j] = -1;
    *n_sel_out = n;
    free(take);
    return 0;
}

/* ------------------------------------------------------------------------
 * Cache construction (end of Sec. 3.3): rows idx[0..n_sel) of K and V copied
 * bit for bit, rows n_sel..B-1 zero, then (append_window) the W most recent
 * rows T..L-1 in order.  row_bytes = D * element size.
 * ---------------------------------------------------------------------- */
int sablock_ref_compact(const void *k, const void *v, int32_t L, int32_t W, int64_t row_bytes,
                        const int32_t *idx, int32_t n_sel, int32_t B, int32_t append_window,
                        void *k_out, void *v_out)
{
    if (!k || !v || !idx || !k_out || !v_out || n_sel < 0 || n_sel > B) return 1;
    const char *src[2] = { (const char *)k, (const char *)v };
    char *dst[2] = { (char *)k_out, (char *)v_out };
    for (int w = 0; w < 2; ++w) {
        for (int32_t j = 0; j < B; ++j) {
            if (j < n_sel) {
                if (idx[j] < 0 || idx[j] >= L) return 1;
                memcpy(dst[w] + (size_t)j * row_bytes, src[w] + (size_t)idx[j] * row_bytes, (size_t)row_bytes);
            } else {
                memset(dst[w] + (size_t)j * row_bytes, 0, (size_t)row_bytes);
            }
        }
        if (append_window)
            memcpy(dst[w] + (size_t)B * row_bytes, src[w] + (size_t)(L - W) * row_bytes,
                   (size_t)W * (size_t)row_bytes);
    }
    return 0;
}

/* Diagnostic used by the pins: Score_k(g), and T_k(g) membership, for one
 * segment and one block size (exposes greedy_fill). */
double sablock_ref_segment_score(const double *st, int32_t a, int32_t b, int32_t g, int32_t bk,
                                 unsigned char *take)
{
    return greedy_fill(st, a, b, g, bk, take);
}
