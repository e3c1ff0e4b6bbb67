/*
 * lca_oracle.c — plain fp64 CPU oracle for Latent-Condensed Attention (LCA).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement of what the
 * GPU library must compute.  It shares no code with the HIP path and is never called by it;
 * only the tests, the smoke check and the benchmark's CPU-baseline leg may use it.
 *
 * Every function works on host arrays of double (inputs already rounded to the storage type
 * of the GPU run and widened exactly), takes the steps of the method in the order the paper
 * gives them, and applies no blocking, fusion or reordering beyond an OpenMP loop over
 * independent outputs (groups or query rows).
 *
 * Notation follows the paper (section 4): L tokens, group size g, local window w,
 * m = floor((L - w) / g) groups, k = L - m*g raw tokens.  Indices here are 0-based:
 * token i in [0, L), group j in [0, m) covers tokens [j*g, (j+1)*g).
 *
 * Two modes:
 *   MLA (mode 0): token i has a latent c_i (POOL, d_pool wide, shared by all heads) and a RoPE
 *                 key k^R_i (SEL, d_sel wide).  Absorbed form: key_i = [c_i ; k^R_i]
 *                 (d_qk = d_pool + d_sel), value_i = c_i (section 3, Eq. 2-5 with W^UK, W^UV
 *                 folded into the query and the output projection).
 *   GQA (mode 1): per KV head, key k_i (SEL) and value v_i (POOL); key_i = k_i, value_i = v_i
 *                 (section 5.4: max-selection on keys, weighted pooling on values).
 *
 * "Sets": S condensed sets per sequence; query head h uses set h / (H / S).  In MLA mode all
 * sets read the same C^KV / K^R; in GQA mode set s reads KV head s.
 *
 * Readings taken where the paper leaves a point open:
 *   - every query row t sees what a decode step at that position would see: representatives of
 *     the groups lying wholly inside tokens [0, t+1-w), then raw tokens up to and including t
 *     (appendix A.2 notation: recent window R, distant history H, per query t);
 *   - representatives are computed once, from the summary query at the end of the prompt
 *     (Algorithm 1, first step);
 *   - each representative enters the softmax once (Algorithm 1, last step; Z' in appendix A.2);
 *     rep_logit_bias = ln(g) gives the multiplicity-weighted variant used in the theorem's proof;
 *   - the anchor is the lowest index attaining the maximum score (Eq. 8; softmax is monotone,
 *     so arg-max of alpha = arg-max of s).
 *
 * Pins: tests/test_oracle_*.py (closed forms, invariants, brute force, degenerate cases).
 * The numeric values of c^rep and of the attention output on the benchmark configurations are
 * "parity unpinned" by the paper (it prints no worked example); they are pinned only through
 * those invariants and brute-force re-derivations.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t B, L, H, S;
    int32_t d_pool, d_sel;
    int32_t g, w, n_q;
    int32_t mode; /* 0 = MLA, 1 = GQA */
    double scale;
    double rep_logit_bias;
    int32_t pool_reduce; /* how a group's vectors become the representative's pooled component: 0 = the method */
    int32_t sel_reduce;  /* ... and its selected component (ablation of section 5.4, Table 5)                 */
} oracle_desc;

/* reduce strategies; 0 stands for the method's own: weighted pooling (Eq. 7) / max selection (Eq. 8) */
enum { RED_DEFAULT = 0, RED_WEIGHTED = 1, RED_MEAN = 2, RED_MAXSEL = 3, RED_MAXPOOL = 4 };

enum { ORACLE_OK = 0, ORACLE_BAD_ARG = 1 };

static int d_qk_of(const oracle_desc *d) { return d->mode == 0 ? d->d_pool + d->d_sel : d->d_sel; }
static int kv_heads_of(const oracle_desc *d) { return d->mode == 0 ? 1 : d->S; }
static int kv_head_of_set(const oracle_desc *d, int s) { return d->mode == 0 ? 0 : s; }

/* number of groups, section 4.2: m = floor((L - w) / g), none when L <= w */
static int num_groups(int L, int w, int g) { return L > w ? (L - w) / g : 0; }

/* groups visible to query row t: those wholly inside the distant history of the t+1 tokens seen */
static int groups_visible(int t, int w, int g) { return (t + 1 > w) ? (t + 1 - w) / g : 0; }

static int check_desc(const oracle_desc *d)
{
    if (!d) return ORACLE_BAD_ARG;
    if (d->B <= 0 || d->L <= 0 || d->H <= 0 || d->S <= 0 || d->g <= 0 || d->w < 0) return ORACLE_BAD_ARG;
    if (d->H % d->S != 0 || d->d_pool <= 0 || d->d_sel <= 0) return ORACLE_BAD_ARG;
    if (d->mode != 0 && d->mode != 1) return ORACLE_BAD_ARG;
    if (d->pool_reduce < 0 || d->pool_reduce > 4 || d->sel_reduce < 0 || d->sel_reduce > 4) return ORACLE_BAD_ARG;
    return ORACLE_OK;
}

/* row of token i in a [B, L, P, width] array, KV head p */
static const double *tok_row(const double *base, const oracle_desc *d, int b, int i, int p, int width)
{
    int P = kv_heads_of(d);
    return base + (((size_t)b * d->L + i) * P + p) * (size_t)width;
}

/* <q, key>: MLA key = [pool_row ; sel_row], GQA key = sel_row */
static double key_dot(const oracle_desc *d, const double *q, const double *pool_row, const double *sel_row)
{
    double acc = 0.0;
    if (d->mode == 0) {
        for (int x = 0; x < d->d_pool; ++x) acc += q[x] * pool_row[x];
        for (int x = 0; x < d->d_sel; ++x) acc += q[d->d_pool + x] * sel_row[x];
    } else {
        for (int x = 0; x < d->d_sel; ++x) acc += q[x] * sel_row[x];
    }
    return acc;
}

int oracle_num_groups(const oracle_desc *d) { return check_desc(d) ? -1 : num_groups(d->L, d->w, d->g); }

/*
 * Summary query (Algorithm 1, first step; section 4.2): the average of the last n_q queries.
 * With fewer sets than heads the average also runs over the heads of the set (the mean of the
 * per-head scores, by linearity).
 *   q_tail [B, n_q, H, d_qk]  the queries of tokens L-n_q .. L-1
 *   qbar   [B, S, d_qk]
 */
int oracle_summary_query(const oracle_desc *d, const double *q_tail, double *qbar)
{
    if (check_desc(d) || !q_tail || !qbar || d->n_q <= 0 || d->n_q > d->L) return ORACLE_BAD_ARG;
    const int dq = d_qk_of(d), hps = d->H / d->S;
    for (int b = 0; b < d->B; ++b)
        for (int s = 0; s < d->S; ++s)
            for (int x = 0; x < dq; ++x) {
                double acc = 0.0;
                for (int t = 0; t < d->n_q; ++t)
                    for (int h = s * hps; h < (s + 1) * hps; ++h)
                        acc += q_tail[(((size_t)b * d->n_q + t) * d->H + h) * dq + x];
                qbar[((size_t)b * d->S + s) * dq + x] = acc / ((double)d->n_q * hps);
            }
    return ORACLE_OK;
}

/*
 * Latent-space condensation (section 4.2; Algorithm 1, loop over groups).
 * For every group j of every set:
 *   s_i     = scale * <qbar, key_i>                       (importance score)
 *   alpha_i = exp(s_i) / sum_{k in G_j} exp(s_k)          (Eq. 6)
 *   c^rep_j = sum_i alpha_i * pool_i                      (Eq. 7)
 *   I_j     = lowest i with s_i = max                     (Eq. 8),  sel_rep_j = sel_{I_j}
 * With the ablation's other strategies (section 5.4, Table 5; appendix on alternative pooling) a component is
 * instead the plain mean, the alpha-weighted sum, the arg-max score token's vector, or ("max pooling", which the
 * appendix describes as keeping the vector with the highest norm) the group's vector of largest Euclidean norm.
 *   margin_j = gap between the largest and second-largest score (0 when g == 1 is reported as +inf)
 * Outputs: pool_rep [B,S,m,d_pool], sel_rep [B,S,m,d_sel], anchor [B,S,m] (absolute token
 * index), alpha [B,S,m*g] (nullable), margin [B,S,m] (nullable).
 */
int oracle_condense(const oracle_desc *d, const double *qbar, const double *POOL, const double *SEL,
                    double *pool_rep, double *sel_rep, int32_t *anchor, double *alpha, double *margin)
{
    if (check_desc(d) || !qbar || !POOL || !SEL) return ORACLE_BAD_ARG;
    const int m = num_groups(d->L, d->w, d->g), g = d->g, dq = d_qk_of(d);
    if (m > 0 && (!pool_rep || !sel_rep || !anchor)) return ORACLE_BAD_ARG;
    const long total = (long)d->B * d->S * m;
#pragma omp parallel for schedule(static)
    for (long u = 0; u < total; ++u) {
        const int j = (int)(u % m), s = (int)((u / m) % d->S), b = (int)(u / ((long)m * d->S));
        const int p = kv_head_of_set(d, s);
        const double *q = qbar + ((size_t)b * d->S + s) * dq;
        double *sc = (double *)malloc(sizeof(double) * g);
        double *al = (double *)malloc(sizeof(double) * g);
        /* scores */
        for (int r = 0; r < g; ++r) {
            const int i = j * g + r;
            sc[r] = d->scale * key_dot(d, q, tok_row(POOL, d, b, i, p, d->d_pool), tok_row(SEL, d, b, i, p, d->d_sel));
        }
        /* group softmax, Eq. 6 */
        double mx = sc[0];
        for (int r = 1; r < g; ++r) if (sc[r] > mx) mx = sc[r];
        double z = 0.0;
        for (int r = 0; r < g; ++r) { al[r] = exp(sc[r] - mx); z += al[r]; }
        for (int r = 0; r < g; ++r) al[r] /= z;
        /* anchor, Eq. 8: first index attaining the maximum */
        int best = 0;
        for (int r = 1; r < g; ++r) if (sc[r] > sc[best]) best = r;
        double second = -INFINITY;
        for (int r = 0; r < g; ++r) if (r != best && sc[r] > second) second = sc[r];
        anchor[u] = j * g + best;
        /* the two components of the representative: Eq. 7 and Eq. 8 unless the ablation asks otherwise */
        for (int comp = 0; comp < 2; ++comp) {
            const double *X = comp == 0 ? POOL : SEL;
            const int width = comp == 0 ? d->d_pool : d->d_sel;
            double *out = (comp == 0 ? pool_rep : sel_rep) + (size_t)u * width;
            int strat = comp == 0 ? d->pool_reduce : d->sel_reduce;
            if (strat == RED_DEFAULT) strat = comp == 0 ? RED_WEIGHTED : RED_MAXSEL;
            if (strat == RED_WEIGHTED || strat == RED_MEAN) {
                for (int x = 0; x < width; ++x) {
                    double acc = 0.0;
                    for (int r = 0; r < g; ++r) acc += (strat == RED_WEIGHTED ? al[r] : 1.0 / g) * tok_row(X, d, b, j * g + r, p, width)[x];
                    out[x] = acc;
                }
            } else {
                int pick = best;                                  /* max selection: the arg-max score token */
                if (strat == RED_MAXPOOL) {                       /* max pooling: the vector of largest Euclidean norm */
                    double nbest = -1.0;
                    for (int r = 0; r < g; ++r) {
                        const double *row = tok_row(X, d, b, j * g + r, p, width);
                        double n2 = 0.0;
                        for (int x = 0; x < width; ++x) n2 += row[x] * row[x];
                        if (n2 > nbest) { nbest = n2; pick = r; }
                    }
                }
                memcpy(out, tok_row(X, d, b, j * g + pick, p, width), sizeof(double) * width);
            }
        }
        if (margin) margin[u] = sc[best] - second;
        if (alpha) memcpy(alpha + (size_t)u * g, al, sizeof(double) * g);
        free(sc);
        free(al);
    }
    return ORACLE_OK;
}

/* softmax over n logits followed by the weighted sum of the n value rows vals[e] (each d_v wide) */
static void softmax_weighted_sum(int n, const double *logit, const double *const *vals, int d_v, double *out, double *lse)
{
    double mx = logit[0];
    for (int e = 1; e < n; ++e) if (logit[e] > mx) mx = logit[e];
    double z = 0.0;
    for (int e = 0; e < n; ++e) z += exp(logit[e] - mx);
    for (int x = 0; x < d_v; ++x) out[x] = 0.0;
    for (int e = 0; e < n; ++e) {
        const double p = exp(logit[e] - mx) / z;
        for (int x = 0; x < d_v; ++x) out[x] += p * vals[e][x];
    }
    if (lse) *lse = mx + log(z);
}

/*
 * Attention with condensed context for a list of query rows (section 4.3, Eq. 10; Algorithm 1,
 * last steps; appendix A.2 notation for a query at position t).
 * Row t of head h (set s) attends the entries
 *     E_t = { representative j : j < m_t }  U  { raw token i : m_t*g <= i <= t },
 *     m_t = max(0, floor((t + 1 - w) / g)),
 * with logit scale*<q, key_e> (+ rep_logit_bias for representatives), one softmax over E_t, and
 * output sum_e p_e value_e (value = c^rep_j or the raw pool row).  For t = L-1 this is
 * Algorithm 1 literally: m_t = m and the raw part is the last k = L - m*g tokens.
 *   rows   [n_rows]                token positions
 *   q_rows [B, n_rows, H, d_qk]    queries of those positions
 *   O      [B, n_rows, H, d_pool], lse [B, n_rows, H] (nullable)
 */
int oracle_lca_attn_rows(const oracle_desc *d, int n_rows, const int32_t *rows, const double *q_rows,
                         const double *POOL, const double *SEL, const double *pool_rep, const double *sel_rep,
                         double *O, double *lse)
{
    if (check_desc(d) || n_rows < 0 || (n_rows > 0 && (!rows || !q_rows || !O)) || !POOL || !SEL) return ORACLE_BAD_ARG;
    const int m = num_groups(d->L, d->w, d->g), g = d->g, dq = d_qk_of(d), hps = d->H / d->S;
    if (m > 0 && (!pool_rep || !sel_rep)) return ORACLE_BAD_ARG;
    for (int r = 0; r < n_rows; ++r) if (rows[r] < 0 || rows[r] >= d->L) return ORACLE_BAD_ARG;
    const long total = (long)d->B * n_rows * d->H;
#pragma omp parallel for schedule(dynamic, 1)
    for (long u = 0; u < total; ++u) {
        const int h = (int)(u % d->H), r = (int)((u / d->H) % n_rows), b = (int)(u / ((long)d->H * n_rows));
        const int t = rows[r], s = h / hps, p = kv_head_of_set(d, s);
        const int mt = groups_visible(t, d->w, g);
        const int n = mt + (t + 1 - mt * g);
        const double *q = q_rows + (size_t)u * dq;
        double *logit = (double *)malloc(sizeof(double) * n);
        const double **vals = (const double **)malloc(sizeof(double *) * n);
        int e = 0;
        for (int j = 0; j < mt; ++j, ++e) { /* representatives of the distant history */
            const size_t rep = ((size_t)b * d->S + s) * m + j;
            logit[e] = d->scale * key_dot(d, q, pool_rep + rep * d->d_pool, sel_rep + rep * d->d_sel) + d->rep_logit_bias;
            vals[e] = pool_rep + rep * d->d_pool;
        }
        for (int i = mt * g; i <= t; ++i, ++e) { /* raw local context */
            const double *pr = tok_row(POOL, d, b, i, p, d->d_pool);
            logit[e] = d->scale * key_dot(d, q, pr, tok_row(SEL, d, b, i, p, d->d_sel));
            vals[e] = pr;
        }
        softmax_weighted_sum(n, logit, vals, d->d_pool, O + (size_t)u * d->d_pool, lse ? lse + u : NULL);
        free(logit);
        free((void *)vals);
    }
    return ORACLE_OK;
}

/*
 * Dense causal attention for a list of query rows (section 3, Eq. 5, in absorbed form for MLA):
 * row t attends every token i <= t.  g, w, n_q and rep_logit_bias are ignored.
 */
int oracle_dense_attn_rows(const oracle_desc *d, int n_rows, const int32_t *rows, const double *q_rows,
                           const double *POOL, const double *SEL, double *O, double *lse)
{
    if (!d || d->B <= 0 || d->L <= 0 || d->H <= 0 || d->S <= 0 || d->H % d->S != 0 || d->d_pool <= 0 || d->d_sel <= 0 ||
        (d->mode != 0 && d->mode != 1))
        return ORACLE_BAD_ARG;
    if (n_rows < 0 || (n_rows > 0 && (!rows || !q_rows || !O)) || !POOL || !SEL) return ORACLE_BAD_ARG;
    for (int r = 0; r < n_rows; ++r) if (rows[r] < 0 || rows[r] >= d->L) return ORACLE_BAD_ARG;
    const int dq = d_qk_of(d), hps = d->H / d->S;
    const long total = (long)d->B * n_rows * d->H;
#pragma omp parallel for schedule(dynamic, 1)
    for (long u = 0; u < total; ++u) {
        const int h = (int)(u % d->H), r = (int)((u / d->H) % n_rows), b = (int)(u / ((long)d->H * n_rows));
        const int t = rows[r], p = kv_head_of_set(d, h / hps);
        const int n = t + 1;
        const double *q = q_rows + (size_t)u * dq;
        double *logit = (double *)malloc(sizeof(double) * n);
        const double **vals = (const double **)malloc(sizeof(double *) * n);
        for (int i = 0; i <= t; ++i) {
            const double *pr = tok_row(POOL, d, b, i, p, d->d_pool);
            logit[i] = d->scale * key_dot(d, q, pr, tok_row(SEL, d, b, i, p, d->d_sel));
            vals[i] = pr;
        }
        softmax_weighted_sum(n, logit, vals, d->d_pool, O + (size_t)u * d->d_pool, lse ? lse + u : NULL);
        free(logit);
        free((void *)vals);
    }
    return ORACLE_OK;
}

/*
 * One decode step over a condensed cache (section 4.3, decoding paragraph): the newest token of
 * each sequence (already appended to the raw tail, L counts it) attends the m cached
 * representatives and the k = L - m*g raw tail entries, m = floor((L - w) / g).
 *   q         [B, H, d_qk]
 *   pool_rep  [B, S, m, d_pool], sel_rep [B, S, m, d_sel]
 *   pool_tail [B, P, k, d_pool], sel_tail [B, P, k, d_sel]   (P = 1 for MLA, S for GQA)
 *   O         [B, H, d_pool]
 */
int oracle_decode_attn(const oracle_desc *d, const double *q, const double *pool_rep, const double *sel_rep,
                       const double *pool_tail, const double *sel_tail, double *O)
{
    if (check_desc(d) || !q || !pool_tail || !sel_tail || !O) return ORACLE_BAD_ARG;
    const int m = num_groups(d->L, d->w, d->g), k = d->L - m * d->g, dq = d_qk_of(d), hps = d->H / d->S;
    const int P = kv_heads_of(d);
    if (m > 0 && (!pool_rep || !sel_rep)) return ORACLE_BAD_ARG;
    const long total = (long)d->B * d->H;
#pragma omp parallel for schedule(dynamic, 1)
    for (long u = 0; u < total; ++u) {
        const int h = (int)(u % d->H), b = (int)(u / d->H), s = h / hps, p = kv_head_of_set(d, s);
        const int n = m + k;
        const double *qv = q + (size_t)u * dq;
        double *logit = (double *)malloc(sizeof(double) * n);
        const double **vals = (const double **)malloc(sizeof(double *) * n);
        int e = 0;
        for (int j = 0; j < m; ++j, ++e) {
            const size_t rep = ((size_t)b * d->S + s) * m + j;
            logit[e] = d->scale * key_dot(d, qv, pool_rep + rep * d->d_pool, sel_rep + rep * d->d_sel) + d->rep_logit_bias;
            vals[e] = pool_rep + rep * d->d_pool;
        }
        for (int i = 0; i < k; ++i, ++e) {
            const size_t row = ((size_t)b * P + p) * k + i;
            logit[e] = d->scale * key_dot(d, qv, pool_tail + row * d->d_pool, sel_tail + row * d->d_sel);
            vals[e] = pool_tail + row * d->d_pool;
        }
        softmax_weighted_sum(n, logit, vals, d->d_pool, O + (size_t)u * d->d_pool, NULL);
        free(logit);
        free((void *)vals);
    }
    return ORACLE_OK;
}

/*
 * Per-token deviations between the original keys / values and the representative that stands for them
 * (Theorem 1's delta_k, delta_v; measured in appendix "Empirical per-token deviations", Tables 9-10):
 * for every condensed token i of group j (i < m*g),
 *     dk_i = || key_i - key^rep_j ||_2,   dv_i = || value_i - value^rep_j ||_2,
 * with key = [pool ; sel] (MLA, absorbed space) or sel (GQA) and value = pool.
 * stats [B, S, 6] = mean dk, mean dk / ||key_i||, max dk, mean dv, mean dv / ||value_i||, max dv over those
 * tokens (a ratio with a zero denominator counts as 0; all zeros when m = 0).
 */
int oracle_deviation_stats(const oracle_desc *d, const double *POOL, const double *SEL, const double *pool_rep,
                           const double *sel_rep, double *stats)
{
    if (check_desc(d) || !POOL || !SEL || !stats) return ORACLE_BAD_ARG;
    const int m = num_groups(d->L, d->w, d->g), g = d->g;
    if (m > 0 && (!pool_rep || !sel_rep)) return ORACLE_BAD_ARG;
    for (int b = 0; b < d->B; ++b)
        for (int s = 0; s < d->S; ++s) {
            const int p = kv_head_of_set(d, s);
            double sum_dk = 0, sum_rk = 0, max_dk = 0, sum_dv = 0, sum_rv = 0, max_dv = 0;
            for (int i = 0; i < m * g; ++i) {
                const int j = i / g;
                const double *pr = tok_row(POOL, d, b, i, p, d->d_pool), *sr = tok_row(SEL, d, b, i, p, d->d_sel);
                const double *prr = pool_rep + (((size_t)b * d->S + s) * m + j) * d->d_pool;
                const double *srr = sel_rep + (((size_t)b * d->S + s) * m + j) * d->d_sel;
                double dp2 = 0, np2 = 0, ds2 = 0, ns2 = 0;
                for (int x = 0; x < d->d_pool; ++x) { dp2 += (pr[x] - prr[x]) * (pr[x] - prr[x]); np2 += pr[x] * pr[x]; }
                for (int x = 0; x < d->d_sel; ++x) { ds2 += (sr[x] - srr[x]) * (sr[x] - srr[x]); ns2 += sr[x] * sr[x]; }
                const double dk = d->mode == 0 ? sqrt(dp2 + ds2) : sqrt(ds2), nk = d->mode == 0 ? sqrt(np2 + ns2) : sqrt(ns2);
                const double dv = sqrt(dp2), nv = sqrt(np2);
                sum_dk += dk; sum_rk += nk > 0 ? dk / nk : 0; if (dk > max_dk) max_dk = dk;
                sum_dv += dv; sum_rv += nv > 0 ? dv / nv : 0; if (dv > max_dv) max_dv = dv;
            }
            double *o = stats + ((size_t)b * d->S + s) * 6;
            const double n = m * g > 0 ? (double)(m * g) : 1.0;
            o[0] = sum_dk / n; o[1] = sum_rk / n; o[2] = max_dk; o[3] = sum_dv / n; o[4] = sum_rv / n; o[5] = max_dv;
        }
    return ORACLE_OK;
}

/*
 * KV-cache footprint (section 4.3 decoding paragraph; appendix B): the dense cache holds one
 * (pool, sel) row per token and KV head; the condensed cache holds m representatives per set
 * plus the k raw tail tokens per KV head.
 */
int oracle_cache_bytes(const oracle_desc *d, int elt_bytes, uint64_t *dense_bytes, uint64_t *condensed_bytes)
{
    if (check_desc(d) || elt_bytes <= 0 || !dense_bytes || !condensed_bytes) return ORACLE_BAD_ARG;
    const uint64_t m = (uint64_t)num_groups(d->L, d->w, d->g), k = (uint64_t)d->L - m * d->g;
    const uint64_t row = (uint64_t)(d->d_pool + d->d_sel) * elt_bytes, P = (uint64_t)kv_heads_of(d);
    *dense_bytes = (uint64_t)d->B * d->L * P * row;
    *condensed_bytes = (uint64_t)d->B * ((uint64_t)d->S * m + P * k) * row;
    return ORACLE_OK;
}
