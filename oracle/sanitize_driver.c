/*
 * sanitize_driver.c — runs every entry point of the oracle (lca_oracle.c, included as source) on one case read from a
 * file, in buffers allocated to exactly the documented sizes, and writes every output to a second file.
 *
 * TEST INFRASTRUCTURE ONLY, like the oracle itself.  tests/test_sanitizers.py builds this file with
 * -fsanitize=address,undefined (any out-of-range access, signed overflow or misaligned access inside the oracle ends the
 * program with a report) and compares what it writes with the ordinary build of the oracle on the same case.
 *
 * Case file: oracle_desc (as laid out in lca_oracle.c), int32 n_rows, int32 rows[n_rows], then doubles:
 *   q_tail [B,n_q,H,d_qk], q_rows [B,n_rows,H,d_qk], POOL, SEL ([B,L,d] for MLA, [B,L,S,d] for GQA).
 * Output file, doubles unless said: qbar [B,S,d_qk]; pool_rep [B,S,m,d_pool]; sel_rep [B,S,m,d_sel]; anchor (int32)
 *   [B,S,m]; alpha [B,S,m*g]; margin [B,S,m]; O_lca [B,n_rows,H,d_pool]; lse_lca [B,n_rows,H]; O_dense, lse_dense likewise;
 *   O_decode [B,H,d_pool] (decode step for the last token over the condensed cache); stats [B,S,6];
 *   uint64 dense_bytes, condensed_bytes.
 */
#include "lca_oracle.c"

#include <stdio.h>

static void *exact(size_t n, size_t elt)
{
    void *p = malloc(n * elt ? n * elt : 1);      /* exactly the documented size: one element more would hide an overrun */
    if (!p) { fprintf(stderr, "out of memory\n"); exit(2); }
    return p;
}

static void rd(void *p, size_t elt, size_t n, FILE *f)
{
    if (n && fread(p, elt, n, f) != n) { fprintf(stderr, "short case file\n"); exit(2); }
}

static void wr(const void *p, size_t elt, size_t n, FILE *f)
{
    if (n && fwrite(p, elt, n, f) != n) { fprintf(stderr, "write failed\n"); exit(2); }
}

#define MUST(call) do { int rc_ = (call); if (rc_ != ORACLE_OK) { fprintf(stderr, "%s returned %d\n", #call, rc_); return 3; } } while (0)

int main(int argc, char **argv)
{
    if (argc != 3) { fprintf(stderr, "usage: %s case.bin out.bin\n", argv[0]); return 2; }
    FILE *in = fopen(argv[1], "rb"), *out = fopen(argv[2], "wb");
    if (!in || !out) { fprintf(stderr, "cannot open files\n"); return 2; }
    oracle_desc d;
    int32_t n_rows;
    rd(&d, sizeof d, 1, in);
    rd(&n_rows, sizeof n_rows, 1, in);
    if (check_desc(&d) || n_rows < 0) { fprintf(stderr, "bad case\n"); return 2; }
    const size_t B = d.B, L = d.L, H = d.H, S = d.S, P = kv_heads_of(&d), dq = d_qk_of(&d), dp = d.d_pool, ds = d.d_sel, g = d.g;
    const size_t m = num_groups(d.L, d.w, d.g), k = L - m * g, nq = d.n_q, nr = n_rows;

    int32_t *rows = exact(nr, sizeof *rows);
    double *q_tail = exact(B * nq * H * dq, 8), *q_rows = exact(B * nr * H * dq, 8);
    double *POOL = exact(B * L * P * dp, 8), *SEL = exact(B * L * P * ds, 8);
    rd(rows, sizeof *rows, nr, in);
    rd(q_tail, 8, B * nq * H * dq, in);
    rd(q_rows, 8, B * nr * H * dq, in);
    rd(POOL, 8, B * L * P * dp, in);
    rd(SEL, 8, B * L * P * ds, in);
    fclose(in);

    double *qbar = exact(B * S * dq, 8);
    MUST(oracle_summary_query(&d, q_tail, qbar));
    wr(qbar, 8, B * S * dq, out);

    double *pool_rep = exact(B * S * m * dp, 8), *sel_rep = exact(B * S * m * ds, 8), *alpha = exact(B * S * m * g, 8), *margin = exact(B * S * m, 8);
    int32_t *anchor = exact(B * S * m, sizeof *anchor);
    MUST(oracle_condense(&d, qbar, POOL, SEL, pool_rep, sel_rep, anchor, alpha, margin));
    if ((size_t)oracle_num_groups(&d) != m) return 3;
    wr(pool_rep, 8, B * S * m * dp, out);
    wr(sel_rep, 8, B * S * m * ds, out);
    wr(anchor, sizeof *anchor, B * S * m, out);
    wr(alpha, 8, B * S * m * g, out);
    wr(margin, 8, B * S * m, out);

    double *O = exact(B * nr * H * dp, 8), *lse = exact(B * nr * H, 8);
    MUST(oracle_lca_attn_rows(&d, n_rows, rows, q_rows, POOL, SEL, pool_rep, sel_rep, O, lse));
    wr(O, 8, B * nr * H * dp, out);
    wr(lse, 8, B * nr * H, out);
    MUST(oracle_dense_attn_rows(&d, n_rows, rows, q_rows, POOL, SEL, O, lse));
    wr(O, 8, B * nr * H * dp, out);
    wr(lse, 8, B * nr * H, out);

    /* decode step of the last token: its query is the last of the summary queries' rows; the tail is tokens [m g, L) per KV head */
    double *q_last = exact(B * H * dq, 8), *pool_tail = exact(B * P * k * dp, 8), *sel_tail = exact(B * P * k * ds, 8), *Od = exact(B * H * dp, 8);
    for (size_t b = 0; b < B; ++b) {
        memcpy(q_last + b * H * dq, q_tail + ((b * nq + (nq - 1)) * H) * dq, H * dq * 8);
        for (size_t p = 0; p < P; ++p)
            for (size_t i = 0; i < k; ++i) {
                memcpy(pool_tail + ((b * P + p) * k + i) * dp, POOL + ((b * L + m * g + i) * P + p) * dp, dp * 8);
                memcpy(sel_tail + ((b * P + p) * k + i) * ds, SEL + ((b * L + m * g + i) * P + p) * ds, ds * 8);
            }
    }
    MUST(oracle_decode_attn(&d, q_last, pool_rep, sel_rep, pool_tail, sel_tail, Od));
    wr(Od, 8, B * H * dp, out);

    double *stats = exact(B * S * 6, 8);
    MUST(oracle_deviation_stats(&d, POOL, SEL, pool_rep, sel_rep, stats));
    wr(stats, 8, B * S * 6, out);

    uint64_t cb[2];
    MUST(oracle_cache_bytes(&d, 2, &cb[0], &cb[1]));
    wr(cb, sizeof cb[0], 2, out);

    /* argument errors must come back as codes, not as accesses */
    if (oracle_condense(&d, NULL, POOL, SEL, pool_rep, sel_rep, anchor, alpha, margin) == ORACLE_OK) return 4;
    if (oracle_summary_query(NULL, q_tail, qbar) == ORACLE_OK) return 4;
    { oracle_desc bad = d; bad.g = 0; if (oracle_num_groups(&bad) != -1) return 4; }
    { oracle_desc bad = d; bad.H = d.S + 1; bad.S = d.S + 2; if (oracle_decode_attn(&bad, q_last, pool_rep, sel_rep, pool_tail, sel_tail, Od) == ORACLE_OK) return 4; }
    if (nr > 0) { int32_t off = d.L; if (oracle_dense_attn_rows(&d, 1, &off, q_rows, POOL, SEL, O, lse) == ORACLE_OK) return 4; }

    free(rows); free(q_tail); free(q_rows); free(POOL); free(SEL); free(qbar); free(pool_rep); free(sel_rep); free(alpha); free(margin);
    free(anchor); free(O); free(lse); free(q_last); free(pool_tail); free(sel_tail); free(Od); free(stats);
    if (fclose(out) != 0) return 2;
    return 0;
}
