/* Runs the five benchmark compositions of the CPU oracle at small sizes, every buffer sized exactly, so that a build
 * with -fsanitize=address,undefined reports any access out of bounds or undefined operation in oracle/dol_oracle.c.
 * TEST INFRASTRUCTURE: compiled and run by tests/test_oracle_sanitizers.py only.  Exit status 0 = clean. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int orc_set_threads(int n);
int orc_out_syms(int64_t n, const int32_t *tri_o, int32_t *out_syms);
int orc_damp_apply2_fwd(int B, int64_t n, const int32_t *ti, const int32_t *tj, const int32_t *to, int na, int nb, int S,
                        const int32_t *out_syms, const float *a, int64_t lda, const float *b, int64_t ldb, float *out,
                        int64_t ldo, float *pre32, double *pre64);
int orc_damp_apply2_bwd(int B, int64_t n, const int32_t *ti, const int32_t *tj, const int32_t *to, int na, int nb, int S,
                        const int32_t *out_syms, const float *a, int64_t lda, const float *b, int64_t ldb, const float *g,
                        int64_t ldg, float *ga, int64_t ldga, float *gb, int64_t ldgb);
int orc_filter_plan(int n, const int32_t *syms, const uint8_t *pred, int32_t *out_syms, int32_t *keep_idx);
int orc_damp_filter_fwd(int B, int n, const uint8_t *pred, const float *in, int64_t ldi, float *out, int64_t ldo);
int orc_damp_filter_bwd(int B, int n, const uint8_t *pred, const float *g, int64_t ldg, float *gin, int64_t ldgi);
int orc_union_plan(int na, const int32_t *sa, int nb, const int32_t *sb, int32_t *out_syms, int32_t *ia, int32_t *ib);
int orc_damp_union_fwd(int B, int S, const int32_t *ia, const int32_t *ib, const float *a, int64_t lda, const float *b,
                       int64_t ldb, float *out, int64_t ldo);
int orc_damp_union_bwd(int B, int S, const int32_t *ia, const int32_t *ib, const float *a, int64_t lda, const float *b,
                       int64_t ldb, const float *g, int64_t ldg, float *ga, int64_t ldga, float *gb, int64_t ldgb);
int orc_reach_fwd(int B, int n, int E, const int32_t *eu, const int32_t *ev, int src, int rounds, const float *p,
                  int64_t ldp, float *hist);
int orc_reach_bwd(int B, int n, int E, const int32_t *eu, const int32_t *ev, int rounds, const float *p, int64_t ldp,
                  const float *hist, const float *g, int64_t ldg, float *gp, int64_t ldgp);
int orc_dtkp_init(int B, int n, int k, int n_facts, const int32_t *fact_of_sym, const float *fact_prob, uint64_t *mask,
                  float *pprob, float *prob, int64_t ld);
int orc_dtkp_apply2(int B, int64_t n, const int32_t *ti, const int32_t *tj, const int32_t *to, int na, int nb, int S,
                    const int32_t *out_syms, int k, int n_facts, const int32_t *group, const float *fact_prob,
                    const uint64_t *am, const uint64_t *bm, uint64_t *om, float *op, float *oprob, int64_t ldo);
int orc_dtkp_prob_bwd(int B, int n, int k, int n_facts, const uint64_t *mask, const float *fact_prob, const float *g,
                      int64_t ldg, float *gfact);

static uint64_t rng_state = 12345;
static float unif(void)
{
    rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
    return (float)((rng_state >> 40) & 0xffffff) / 16777216.0f;
}
static float *rows(int B, int n, float scale)      /* B rows of n tags, each row summing to `scale` */
{
    float *x = malloc(sizeof(float) * (size_t)B * n);
    for (int s = 0; s < B; ++s) {
        float tot = 0;
        for (int i = 0; i < n; ++i) tot += x[s * n + i] = 0.05f + unif();
        for (int i = 0; i < n; ++i) x[s * n + i] *= scale / tot;
    }
    return x;
}
#define CHECK(call) do { int rc_ = (call); if (rc_) { fprintf(stderr, "%s -> %d\n", #call, rc_); exit(2); } } while (0)

/* all (i, j) -> f(i, j) of a dense table, ascending (i, j) */
typedef struct { int64_t n; int32_t *i, *j, *o; int na, nb, S; int32_t *syms; } table;
static table make_table(int na, int nb, int kind, int mod)
{
    table t;
    t.na = na; t.nb = nb; t.n = 0;
    t.i = malloc(sizeof(int32_t) * na * nb); t.j = malloc(sizeof(int32_t) * na * nb); t.o = malloc(sizeof(int32_t) * na * nb);
    for (int i = 0; i < na; ++i)
        for (int j = 0; j < nb; ++j) {
            int v = kind == 0 ? i + j : (int)((i * 2654435761u + j * 40503u + 17u) % (unsigned)mod);
            if (kind == 1 && (i * 7 + j) % 11 == 0) continue;            /* some tuples rejected */
            t.i[t.n] = i; t.j[t.n] = j; t.o[t.n] = v; ++t.n;
        }
    t.syms = malloc(sizeof(int32_t) * (t.n ? t.n : 1));
    t.S = orc_out_syms(t.n, t.o, t.syms);
    return t;
}
static void free_table(table *t) { free(t->i); free(t->j); free(t->o); free(t->syms); }

static void sum_chain(int B, int n_digits, float scale)
{
    float *p[8], *acc[8], *gacc, *g;
    table tabs[8];
    int m = 10;
    for (int t = 0; t < n_digits; ++t) p[t] = rows(B, 10, scale);
    acc[0] = p[0];
    for (int t = 1; t < n_digits; ++t) {
        tabs[t] = make_table(m, 10, 0, 0);
        acc[t] = malloc(sizeof(float) * B * tabs[t].S);
        float *pre32 = malloc(sizeof(float) * B * tabs[t].S);
        double *pre64 = malloc(sizeof(double) * B * tabs[t].S);
        CHECK(orc_damp_apply2_fwd(B, tabs[t].n, tabs[t].i, tabs[t].j, tabs[t].o, m, 10, tabs[t].S, tabs[t].syms, acc[t - 1], m, p[t], 10,
                                  acc[t], tabs[t].S, pre32, pre64));
        free(pre32); free(pre64);
        m = tabs[t].S;
    }
    g = rows(B, m, 1.0f);
    for (int t = n_digits - 1; t >= 1; --t) {
        const int ma = tabs[t].na;
        gacc = malloc(sizeof(float) * B * ma);
        float *gb = malloc(sizeof(float) * B * 10);
        CHECK(orc_damp_apply2_bwd(B, tabs[t].n, tabs[t].i, tabs[t].j, tabs[t].o, ma, 10, tabs[t].S, tabs[t].syms, acc[t - 1], ma, p[t], 10, g,
                                  tabs[t].S, gacc, ma, gb, 10));
        free(gb); free(g);
        g = gacc;
    }
    free(g);
    for (int t = 1; t < n_digits; ++t) { free(acc[t]); free_table(&tabs[t]); }
    for (int t = 0; t < n_digits; ++t) free(p[t]);
}

static void hashed_pipeline(int B, int na, int nb, int n_out, float scale)
{
    table T = make_table(na, nb, 1, n_out);
    float *a = rows(B, na, scale), *b = rows(B, nb, scale), *p2 = rows(B, n_out, scale), *g = rows(B, 2 * n_out, 1.0f);
    float *o1 = malloc(sizeof(float) * B * T.S);
    float *pre32 = malloc(sizeof(float) * B * T.S);
    double *pre64 = malloc(sizeof(double) * B * T.S);
    CHECK(orc_damp_apply2_fwd(B, T.n, T.i, T.j, T.o, na, nb, T.S, T.syms, a, na, b, nb, o1, T.S, pre32, pre64));
    uint8_t *pred = malloc(T.S);
    for (int c = 0; c < T.S; ++c) pred[c] = (uint8_t)((T.syms[c] * 5 + 1) % 3 != 0);
    int32_t *s2 = malloc(sizeof(int32_t) * T.S), *keep = malloc(sizeof(int32_t) * T.S);
    const int n2 = orc_filter_plan(T.S, T.syms, pred, s2, keep);
    float *o2 = malloc(sizeof(float) * B * (n2 ? n2 : 1));
    CHECK(orc_damp_filter_fwd(B, T.S, pred, o1, T.S, o2, n2));
    int32_t *all = malloc(sizeof(int32_t) * n_out), *s3 = malloc(sizeof(int32_t) * (n2 + n_out)), *ia = malloc(sizeof(int32_t) * (n2 + n_out)),
            *ib = malloc(sizeof(int32_t) * (n2 + n_out));
    for (int c = 0; c < n_out; ++c) all[c] = c;
    const int n3 = orc_union_plan(n2, s2, n_out, all, s3, ia, ib);
    float *o3 = malloc(sizeof(float) * B * n3), *g2 = malloc(sizeof(float) * B * (n2 ? n2 : 1)), *gp2 = malloc(sizeof(float) * B * n_out);
    CHECK(orc_damp_union_fwd(B, n3, ia, ib, o2, n2, p2, n_out, o3, n3));
    CHECK(orc_damp_union_bwd(B, n3, ia, ib, o2, n2, p2, n_out, g, 2 * n_out, g2, n2, gp2, n_out));
    float *g1 = malloc(sizeof(float) * B * T.S), *ga = malloc(sizeof(float) * B * na), *gb = malloc(sizeof(float) * B * nb);
    CHECK(orc_damp_filter_bwd(B, T.S, pred, g2, n2, g1, T.S));
    CHECK(orc_damp_apply2_bwd(B, T.n, T.i, T.j, T.o, na, nb, T.S, T.syms, a, na, b, nb, g1, T.S, ga, na, gb, nb));
    free(a); free(b); free(p2); free(g); free(o1); free(pre32); free(pre64); free(pred); free(s2); free(keep); free(o2); free(all);
    free(s3); free(ia); free(ib); free(o3); free(g2); free(gp2); free(g1); free(ga); free(gb);
    free_table(&T);
}

static void dtkp_chain(int B, int n_digits, int k)
{
    const int F = 10 * n_digits;
    float *fp = rows(B, F, (float)n_digits);                      /* about one unit of mass per digit */
    int32_t *group = malloc(sizeof(int32_t) * F), fos[10];
    for (int f = 0; f < F; ++f) group[f] = f / 10;
    for (int d = 0; d < 10; ++d) fos[d] = d;
    int m = 10;
    uint64_t *am = malloc(sizeof(uint64_t) * B * m * k);
    float *ap = malloc(sizeof(float) * B * m * k), *apr = malloc(sizeof(float) * B * m);
    CHECK(orc_dtkp_init(B, 10, k, F, fos, fp, am, ap, apr, m));
    for (int t = 1; t < n_digits; ++t) {
        table T = make_table(m, 10, 0, 0);
        for (int d = 0; d < 10; ++d) fos[d] = 10 * t + d;
        uint64_t *bm = malloc(sizeof(uint64_t) * B * 10 * k);
        float *bp = malloc(sizeof(float) * B * 10 * k), *bpr = malloc(sizeof(float) * B * 10);
        CHECK(orc_dtkp_init(B, 10, k, F, fos, fp, bm, bp, bpr, 10));
        uint64_t *om = malloc(sizeof(uint64_t) * B * T.S * k);
        float *op = malloc(sizeof(float) * B * T.S * k), *opr = malloc(sizeof(float) * B * T.S);
        CHECK(orc_dtkp_apply2(B, T.n, T.i, T.j, T.o, m, 10, T.S, T.syms, k, F, group, fp, am, bm, om, op, opr, T.S));
        free(am); free(ap); free(apr); free(bm); free(bp); free(bpr);
        am = om; ap = op; apr = opr; m = T.S;
        free_table(&T);
    }
    float *g = rows(B, m, 1.0f), *gf = malloc(sizeof(float) * B * F);
    CHECK(orc_dtkp_prob_bwd(B, m, k, F, am, fp, g, m, gf));
    free(am); free(ap); free(apr); free(g); free(gf); free(fp); free(group);
}

static void grid_reach(int B, int side, int rounds)
{
    const int n = side * side, E = 2 * side * (side - 1);
    int32_t *eu = malloc(sizeof(int32_t) * E), *ev = malloc(sizeof(int32_t) * E);
    int e = 0;
    for (int y = 0; y < side; ++y)
        for (int x = 0; x + 1 < side; ++x) { eu[e] = y * side + x; ev[e] = y * side + x + 1; ++e; }
    for (int y = 0; y + 1 < side; ++y)
        for (int x = 0; x < side; ++x) { eu[e] = y * side + x; ev[e] = (y + 1) * side + x; ++e; }
    float *p = malloc(sizeof(float) * B * E), *g = rows(B, n, 1.0f);
    for (int x = 0; x < B * E; ++x) p[x] = unif();
    float *hist = malloc(sizeof(float) * (size_t)(rounds + 1) * B * n), *gp = malloc(sizeof(float) * B * E);
    CHECK(orc_reach_fwd(B, n, E, eu, ev, 0, rounds, p, E, hist));
    CHECK(orc_reach_bwd(B, n, E, eu, ev, rounds, p, E, hist, g, n, gp, E));
    free(eu); free(ev); free(p); free(g); free(hist); free(gp);
}

int main(void)
{
    for (int threads = 1; threads <= 3; threads += 2) {
        orc_set_threads(threads);
        sum_chain(7, 2, 1.0f);                 /* workload 1: two digits */
        sum_chain(9, 5, 1.0f);                 /* workload 2: a chain, forward and backward */
        sum_chain(5, 4, 3.0f);                 /* ... with sums above the clamp */
        hashed_pipeline(11, 16, 12, 40, 1.0f); /* workload 3 */
        hashed_pipeline(6, 9, 5, 7, 4.0f);
        dtkp_chain(6, 3, 3);                   /* workload 4 */
        dtkp_chain(4, 2, 1);
        grid_reach(5, 4, 7);                   /* workload 5 */
        grid_reach(3, 2, 0);
    }
    puts("oracle sanitizer driver: clean");
    return 0;
}
