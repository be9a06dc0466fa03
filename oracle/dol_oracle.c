/*
 * dol_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, obviously-correct CPU statement of what the Dolphin hot path
 * computes (arXiv 2410.03348): the Distribution operators Apply / ApplyIf (two
 * operands, and any number K >= 1 of them at the end of the file), Filter and
 * Union (Sec. 3.1.2, Eq. 1-3) under the two provenances of Sec. 3.2 /
 * Table 1: DAMP (add-mult probabilities) with its vector-Jacobian products,
 * and DTKP-AM top-k proofs (App. A) in a fact-bitmask encoding.
 *
 * It shares no code with the HIP library and is only ever called by tests/,
 * by the smoke check, and by the bench's cpu_baseline leg.
 *
 * Conventions
 *   - A Distribution is a host list of ascending int32 symbol ids plus a
 *     row-major tag tensor [B, ld] (fp32), ld >= number of symbols.
 *   - The symbol side of Apply arrives as the list of admitted tuples
 *     (i, j, s): operand symbols with positions i and j produce symbol id s.
 *     The list is in ascending (i, j) order.  A dense user function is that
 *     list over all (i, j) pairs minus the tuples the condition rejects.
 *   - DAMP values are accumulated in double and rounded once to float.  The
 *     discontinuous clamp decision [pre <= 1] used by the backward pass is
 *     taken on `pre32`: the float sum built with one fused multiply-add per
 *     tuple in list order, starting from 0.  (Any fixed order is as good as
 *     another mathematically; fixing one makes the 0/1 decision reproducible.)
 *   - DTKP proofs are 64-bit masks over at most 63 input facts; the all-ones
 *     mask marks an absent proof slot.  A proof's probability is the float
 *     product of its facts' probabilities taken in ascending fact index,
 *     starting from 1 (Sec. 3.2, Pr(t_i) = prod_j norm(t_ij): absent symbols
 *     contribute 1).
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py
 * (worked examples of Ex. 3.1-3.3 and App. A.1, brute-force enumeration,
 * convolution and matrix-power closed forms, finite differences, invariants;
 * the K-operand routines also by agreement with the two-operand ones and by
 * composition through an injective pairing function).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_OK 0
#define ORC_EINVAL 1
#define ORC_ENOMEM 3

#define ABSENT UINT64_MAX

static int g_threads = 1;

/* Number of host threads the batch loops use (1 = sequential). Returns the value in force. */
int orc_set_threads(int n)
{
#ifdef _OPENMP
    if (n < 1) n = omp_get_num_procs();
    g_threads = n;
#else
    (void)n;
    g_threads = 1;
#endif
    return g_threads;
}

/* ------------------------------------------------------------------ symbol side */

static int cmp_i32(const void *x, const void *y)
{
    int32_t a = *(const int32_t *)x, b = *(const int32_t *)y;
    return (a > b) - (a < b);
}

/* Eq. 1-2, symbol half: the output Distribution's symbols are the distinct
 * results of f over the admitted tuples, listed in ascending id order.
 * out_syms has room for n entries; returns the count S (or -1). */
int orc_out_syms(int64_t n, const int32_t *tri_o, int32_t *out_syms)
{
    int64_t m = 0;
    for (int64_t t = 0; t < n; ++t)
        if (tri_o[t] >= 0) out_syms[m++] = tri_o[t];
    qsort(out_syms, (size_t)m, sizeof(int32_t), cmp_i32);
    int64_t s = 0;
    for (int64_t t = 0; t < m; ++t)
        if (s == 0 || out_syms[s - 1] != out_syms[t]) out_syms[s++] = out_syms[t];
    return (int)s;
}

static int find_col(int S, const int32_t *out_syms, int32_t id)
{
    int lo = 0, hi = S - 1;
    while (lo <= hi) {
        int mid = (lo + hi) / 2;
        if (out_syms[mid] == id) return mid;
        if (out_syms[mid] < id) lo = mid + 1; else hi = mid - 1;
    }
    return -1;
}

/* Shuffle stage (Eq. 2): column of the output Distribution each tuple lands in. */
static int *tuple_columns(int64_t n, const int32_t *ti, const int32_t *tj, const int32_t *to,
                          int na, int nb, int S, const int32_t *out_syms, int *err)
{
    int *col = (int *)malloc(sizeof(int) * (size_t)(n > 0 ? n : 1));
    *err = ORC_OK;
    if (!col) { *err = ORC_ENOMEM; return NULL; }
    for (int64_t t = 0; t < n; ++t) {
        if (ti[t] < 0 || ti[t] >= na || tj[t] < 0 || tj[t] >= nb) { *err = ORC_EINVAL; break; }
        if (t > 0 && !(ti[t - 1] < ti[t] || (ti[t - 1] == ti[t] && tj[t - 1] < tj[t]))) { *err = ORC_EINVAL; break; }
        col[t] = to[t] < 0 ? -1 : find_col(S, out_syms, to[t]);
        if (to[t] >= 0 && col[t] < 0) { *err = ORC_EINVAL; break; }
    }
    if (*err) { free(col); return NULL; }
    return col;
}

/* ------------------------------------------------------------------ DAMP apply */

/* Apply with K=2 under DAMP (Eq. 1-3 with Table 1: conjunction t*t', disjunction
 * clamp(t+t')).  For every sample and output symbol,
 *     pre = sum over admitted tuples (i,j) with f(i,j)=symbol of a[i]*b[j],
 *     out = min(1, pre).
 * For tags in [0,1] folding the pairwise clamped sum over a group equals
 * clamping the whole sum once, and the lower clamp never acts.
 * out [B,ldo] float; pre32 [B,S] float (decision quantity) and pre64 [B,S]
 * double are optional. */
int orc_damp_apply2_fwd(int B, int64_t n, const int32_t *ti, const int32_t *tj, const int32_t *to,
                        int na, int nb, int S, const int32_t *out_syms,
                        const float *a, int64_t lda, const float *b, int64_t ldb,
                        float *out, int64_t ldo, float *pre32, double *pre64)
{
    int err;
    int *col = tuple_columns(n, ti, tj, to, na, nb, S, out_syms, &err);
    if (!col) return err;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (int s = 0; s < B; ++s) {
        double *acc = (double *)calloc((size_t)(S > 0 ? S : 1), sizeof(double));
        float *accf = (float *)calloc((size_t)(S > 0 ? S : 1), sizeof(float));
        const float *ar = a + (int64_t)s * lda, *br = b + (int64_t)s * ldb;
        for (int64_t t = 0; t < n; ++t) {
            if (col[t] < 0) continue;
            acc[col[t]] += (double)ar[ti[t]] * (double)br[tj[t]];
            accf[col[t]] = fmaf(ar[ti[t]], br[tj[t]], accf[col[t]]);
        }
        for (int c = 0; c < S; ++c) {
            out[(int64_t)s * ldo + c] = (float)(acc[c] < 1.0 ? acc[c] : 1.0);
            if (pre32) pre32[(int64_t)s * S + c] = accf[c];
            if (pre64) pre64[(int64_t)s * S + c] = acc[c];
        }
        free(acc); free(accf);
    }
    free(col);
    return ORC_OK;
}

/* Vector-Jacobian product of the above.  With gh[c] = g[c] * [pre32[c] <= 1]
 * (the clamp passes gradient inside and on its boundary, App. A.2),
 *     ga[i] = sum_j gh[col(i,j)] * b[j],   gb[j] = sum_i gh[col(i,j)] * a[i],
 * over admitted tuples only.  ga [B,ldga], gb [B,ldgb] are overwritten. */
int orc_damp_apply2_bwd(int B, int64_t n, const int32_t *ti, const int32_t *tj, const int32_t *to,
                        int na, int nb, int S, const int32_t *out_syms,
                        const float *a, int64_t lda, const float *b, int64_t ldb,
                        const float *g, int64_t ldg,
                        float *ga, int64_t ldga, float *gb, int64_t ldgb)
{
    int err;
    int *col = tuple_columns(n, ti, tj, to, na, nb, S, out_syms, &err);
    if (!col) return err;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (int s = 0; s < B; ++s) {
        float *accf = (float *)calloc((size_t)(S > 0 ? S : 1), sizeof(float));
        double *da = (double *)calloc((size_t)(na > 0 ? na : 1), sizeof(double));
        double *db = (double *)calloc((size_t)(nb > 0 ? nb : 1), sizeof(double));
        const float *ar = a + (int64_t)s * lda, *br = b + (int64_t)s * ldb, *gr = g + (int64_t)s * ldg;
        for (int64_t t = 0; t < n; ++t)
            if (col[t] >= 0) accf[col[t]] = fmaf(ar[ti[t]], br[tj[t]], accf[col[t]]);
        for (int64_t t = 0; t < n; ++t) {
            if (col[t] < 0) continue;
            double gh = accf[col[t]] <= 1.0f ? (double)gr[col[t]] : 0.0;
            da[ti[t]] += gh * (double)br[tj[t]];
            db[tj[t]] += gh * (double)ar[ti[t]];
        }
        if (ga) for (int i = 0; i < na; ++i) ga[(int64_t)s * ldga + i] = (float)da[i];
        if (gb) for (int j = 0; j < nb; ++j) gb[(int64_t)s * ldgb + j] = (float)db[j];
        free(accf); free(da); free(db);
    }
    free(col);
    return ORC_OK;
}

/* ------------------------------------------------------------------ Filter */

/* Filter (Sec. 3.1.2, Ex. 3.3): symbols failing the predicate are removed, the
 * others keep their tags and their order.  Returns the kept count; out_syms and
 * keep_idx (position in the input) have room for n entries. */
int orc_filter_plan(int n, const int32_t *syms, const uint8_t *pred, int32_t *out_syms, int32_t *keep_idx)
{
    int m = 0;
    for (int i = 0; i < n; ++i)
        if (pred[i]) { if (out_syms) out_syms[m] = syms[i]; if (keep_idx) keep_idx[m] = i; ++m; }
    return m;
}

int orc_damp_filter_fwd(int B, int n, const uint8_t *pred, const float *in, int64_t ldi, float *out, int64_t ldo)
{
    for (int s = 0; s < B; ++s) {
        int m = 0;
        for (int i = 0; i < n; ++i)
            if (pred[i]) out[(int64_t)s * ldo + m++] = in[(int64_t)s * ldi + i];
    }
    return ORC_OK;
}

/* Its transpose: kept positions receive the gradient of their copy, removed ones 0. */
int orc_damp_filter_bwd(int B, int n, const uint8_t *pred, const float *g, int64_t ldg, float *gin, int64_t ldgi)
{
    for (int s = 0; s < B; ++s) {
        int m = 0;
        for (int i = 0; i < n; ++i)
            gin[(int64_t)s * ldgi + i] = pred[i] ? g[(int64_t)s * ldg + m++] : 0.0f;
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------ Union */

/* Union (Sec. 3.1.2): the symbol set is the union of both (ascending merge);
 * ia[c] / ib[c] give the position of output symbol c in each input, or -1. */
int orc_union_plan(int na, const int32_t *sa, int nb, const int32_t *sb, int32_t *out_syms, int32_t *ia, int32_t *ib)
{
    int i = 0, j = 0, m = 0;
    while (i < na || j < nb) {
        int32_t id; int pa = -1, pb = -1;
        if (j >= nb || (i < na && sa[i] < sb[j])) { id = sa[i]; pa = i++; }
        else if (i >= na || sb[j] < sa[i]) { id = sb[j]; pb = j++; }
        else { id = sa[i]; pa = i++; pb = j++; }
        if (out_syms) out_syms[m] = id;
        if (ia) ia[m] = pa;
        if (ib) ib[m] = pb;
        ++m;
    }
    return m;
}

/* Common symbols have their tags disjuncted, clamp(a+b) under DAMP (Table 1);
 * symbols of one side only are copied. */
int orc_damp_union_fwd(int B, int S, const int32_t *ia, const int32_t *ib,
                       const float *a, int64_t lda, const float *b, int64_t ldb, float *out, int64_t ldo)
{
    for (int s = 0; s < B; ++s)
        for (int c = 0; c < S; ++c) {
            float v;
            if (ia[c] >= 0 && ib[c] >= 0) {
                double t = (double)a[(int64_t)s * lda + ia[c]] + (double)b[(int64_t)s * ldb + ib[c]];
                v = (float)(t < 1.0 ? t : 1.0);
            } else if (ia[c] >= 0) v = a[(int64_t)s * lda + ia[c]];
            else v = b[(int64_t)s * ldb + ib[c]];
            out[(int64_t)s * ldo + c] = v;
        }
    return ORC_OK;
}

/* VJP: a common symbol passes g to both inputs iff the float sum a+b <= 1
 * (one rounded float addition: the decision quantity); one-sided symbols pass g.
 * Every position of ga [B,na] / gb [B,nb] appears in the union, so all are written. */
int orc_damp_union_bwd(int B, int S, const int32_t *ia, const int32_t *ib,
                       const float *a, int64_t lda, const float *b, int64_t ldb,
                       const float *g, int64_t ldg, float *ga, int64_t ldga, float *gb, int64_t ldgb)
{
    for (int s = 0; s < B; ++s)
        for (int c = 0; c < S; ++c) {
            float gv = g[(int64_t)s * ldg + c];
            if (ia[c] >= 0 && ib[c] >= 0) {
                float t = a[(int64_t)s * lda + ia[c]] + b[(int64_t)s * ldb + ib[c]];
                if (!(t <= 1.0f)) gv = 0.0f;
            }
            if (ia[c] >= 0 && ga) ga[(int64_t)s * ldga + ia[c]] = gv;
            if (ib[c] >= 0 && gb) gb[(int64_t)s * ldgb + ib[c]] = gv;
        }
    return ORC_OK;
}

/* ------------------------------------------------------------------ grid reachability */

/* Single-source reachability on an undirected graph by synchronous rounds
 *     r_{t+1}[v] = min(1, r_t[v] + sum_{u ~ v} r_t[u] * p(u,v)),   r_0 = e_src,
 * i.e. union(paths, apply_if(paths, edges)) of App. B with one clamp per node
 * per round.  eu/ev [E]: end nodes of edge e, p [B,E] its probability.
 * hist [rounds+1, B, n] receives r_0..r_rounds (r_rounds is the result).
 * The float decision quantity adds the terms in ascending source-node order
 * (the node itself, weight 1, takes its place in that order). */
static void reach_round(int n, int E, const int32_t *eu, const int32_t *ev, const float *p,
                        const float *r, float *rn, float *pre32, int **nbr, int **nbe, int *deg)
{
    (void)E; (void)eu; (void)ev;
    for (int v = 0; v < n; ++v) {
        double acc = (double)r[v];
        float accf = 0.0f;
        int self_done = 0;
        for (int q = 0; q < deg[v]; ++q) {
            int u = nbr[v][q];
            if (!self_done && u > v) { accf = fmaf(r[v], 1.0f, accf); self_done = 1; }
            acc += (double)r[u] * (double)p[nbe[v][q]];
            accf = fmaf(r[u], p[nbe[v][q]], accf);
        }
        if (!self_done) accf = fmaf(r[v], 1.0f, accf);
        rn[v] = (float)(acc < 1.0 ? acc : 1.0);
        if (pre32) pre32[v] = accf;
    }
}

static int build_adj(int n, int E, const int32_t *eu, const int32_t *ev, int ***nbr_, int ***nbe_, int **deg_)
{
    int *deg = (int *)calloc((size_t)n, sizeof(int));
    int **nbr = (int **)calloc((size_t)n, sizeof(int *)), **nbe = (int **)calloc((size_t)n, sizeof(int *));
    for (int e = 0; e < E; ++e) {
        if (eu[e] < 0 || eu[e] >= n || ev[e] < 0 || ev[e] >= n || eu[e] == ev[e]) return ORC_EINVAL;
        deg[eu[e]]++; deg[ev[e]]++;
    }
    for (int v = 0; v < n; ++v) { nbr[v] = (int *)malloc(sizeof(int) * (size_t)(deg[v] + 1)); nbe[v] = (int *)malloc(sizeof(int) * (size_t)(deg[v] + 1)); deg[v] = 0; }
    for (int e = 0; e < E; ++e) {
        int u = eu[e], v = ev[e];
        nbr[u][deg[u]] = v; nbe[u][deg[u]++] = e;
        nbr[v][deg[v]] = u; nbe[v][deg[v]++] = e;
    }
    /* neighbours in ascending node id (insertion sort, degrees are tiny) */
    for (int v = 0; v < n; ++v)
        for (int x = 1; x < deg[v]; ++x)
            for (int y = x; y > 0 && nbr[v][y - 1] > nbr[v][y]; --y) {
                int t = nbr[v][y]; nbr[v][y] = nbr[v][y - 1]; nbr[v][y - 1] = t;
                t = nbe[v][y]; nbe[v][y] = nbe[v][y - 1]; nbe[v][y - 1] = t;
            }
    *nbr_ = nbr; *nbe_ = nbe; *deg_ = deg;
    return ORC_OK;
}

static void free_adj(int n, int **nbr, int **nbe, int *deg)
{
    for (int v = 0; v < n; ++v) { free(nbr[v]); free(nbe[v]); }
    free(nbr); free(nbe); free(deg);
}

int orc_reach_fwd(int B, int n, int E, const int32_t *eu, const int32_t *ev, int src, int rounds,
                  const float *p, int64_t ldp, float *hist)
{
    int **nbr, **nbe, *deg;
    if (src < 0 || src >= n) return ORC_EINVAL;
    int err = build_adj(n, E, eu, ev, &nbr, &nbe, &deg);
    if (err) return err;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (int s = 0; s < B; ++s) {
        float *r0 = hist + (int64_t)s * n;
        for (int v = 0; v < n; ++v) r0[v] = v == src ? 1.0f : 0.0f;
        for (int t = 0; t < rounds; ++t)
            reach_round(n, E, eu, ev, p + (int64_t)s * ldp,
                        hist + ((int64_t)t * B + s) * n, hist + ((int64_t)(t + 1) * B + s) * n, NULL, nbr, nbe, deg);
    }
    free_adj(n, nbr, nbe, deg);
    return ORC_OK;
}

/* Reverse sweep: g [B,n] is the gradient w.r.t. r_rounds; gp [B,E] receives the
 * gradient w.r.t. every edge probability (both directions of an edge add up).
 * hist is the forward history. */
int orc_reach_bwd(int B, int n, int E, const int32_t *eu, const int32_t *ev, int rounds,
                  const float *p, int64_t ldp, const float *hist, const float *g, int64_t ldg,
                  float *gp, int64_t ldgp)
{
    int **nbr, **nbe, *deg;
    int err = build_adj(n, E, eu, ev, &nbr, &nbe, &deg);
    if (err) return err;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (int s = 0; s < B; ++s) {
        const float *ps = p + (int64_t)s * ldp;
        double *gr = (double *)calloc((size_t)n, sizeof(double)), *gn = (double *)calloc((size_t)n, sizeof(double));
        double *ge = (double *)calloc((size_t)(E > 0 ? E : 1), sizeof(double));
        float *pre = (float *)malloc(sizeof(float) * (size_t)n), *tmp = (float *)malloc(sizeof(float) * (size_t)n);
        for (int v = 0; v < n; ++v) gr[v] = (double)g[(int64_t)s * ldg + v];
        for (int t = rounds - 1; t >= 0; --t) {
            const float *r = hist + ((int64_t)t * B + s) * n;
            reach_round(n, E, eu, ev, ps, r, tmp, pre, nbr, nbe, deg);
            for (int v = 0; v < n; ++v) gn[v] = 0.0;
            for (int v = 0; v < n; ++v) {
                double gh = pre[v] <= 1.0f ? gr[v] : 0.0;
                gn[v] += gh;
                for (int q = 0; q < deg[v]; ++q) {
                    int u = nbr[v][q], e = nbe[v][q];
                    gn[u] += gh * (double)ps[e];
                    ge[e] += gh * (double)r[u];
                }
            }
            double *sw = gr; gr = gn; gn = sw;
        }
        for (int e = 0; e < E; ++e) gp[(int64_t)s * ldgp + e] = (float)ge[e];
        free(gr); free(gn); free(ge); free(pre); free(tmp);
    }
    free_adj(n, nbr, nbe, deg);
    return ORC_OK;
}

/* ------------------------------------------------------------------ DTKP-AM */

typedef struct { uint64_t mask; float prob; } proof_t;

/* Pr(t_i) = prod_j norm(t_ij) (Sec. 3.2): product of the probabilities of the
 * facts present, ascending fact index, float, starting from 1. */
static float proof_prob(uint64_t mask, const float *fact_prob, int n_facts)
{
    float pr = 1.0f;
    for (int j = 0; j < n_facts; ++j)
        if ((mask >> j) & 1u) pr = pr * fact_prob[j];
    return pr;
}

/* A proof is inconsistent when it holds two different facts of one exclusion
 * group (two values for one input slot). */
static int proof_conflict(uint64_t mask, int n_facts, const int32_t *group)
{
    if (!group) return 0;
    for (int x = 0; x < n_facts; ++x) {
        if (!((mask >> x) & 1u)) continue;
        for (int y = x + 1; y < n_facts; ++y)
            if (((mask >> y) & 1u) && group[x] == group[y]) return 1;
    }
    return 0;
}

/* top_k order: higher probability first, equal probabilities by smaller mask. */
static int cmp_proof(const void *x, const void *y)
{
    const proof_t *a = (const proof_t *)x, *b = (const proof_t *)y;
    if (a->prob > b->prob) return -1;
    if (a->prob < b->prob) return 1;
    return (a->mask > b->mask) - (a->mask < b->mask);
}

/* top_k with set semantics: order, drop repeated proofs (equal masks are one
 * proof), keep the first k; absent slots are (ABSENT, 0).  Also the tag's
 * probability min(1, sum of kept proof probabilities) added in rank order
 * (add-mult approximation of WMC, App. A.1). */
static float keep_top_k(proof_t *cand, int n, int k, uint64_t *om, float *op)
{
    qsort(cand, (size_t)n, sizeof(proof_t), cmp_proof);
    int m = 0;
    float sum = 0.0f;
    for (int x = 0; x < n && m < k; ++x) {
        int dup = 0;
        for (int y = 0; y < m; ++y) if (om[y] == cand[x].mask) dup = 1;
        if (dup) continue;
        om[m] = cand[x].mask; op[m] = cand[x].prob; sum = sum + cand[x].prob; ++m;
    }
    for (; m < k; ++m) { om[m] = ABSENT; op[m] = 0.0f; }
    return sum < 1.0f ? sum : 1.0f;
}

/* Natural initialisation (App. A.1): the tag of input symbol i is the single
 * proof {fact_of_sym[i]}.  mask/pprob [B,n,k], prob [B,ld]. */
int orc_dtkp_init(int B, int n, int k, int n_facts, const int32_t *fact_of_sym, const float *fact_prob,
                  uint64_t *mask, float *pprob, float *prob, int64_t ld)
{
    if (n_facts < 0 || n_facts > 63 || k < 1) return ORC_EINVAL;
    for (int i = 0; i < n; ++i) if (fact_of_sym[i] < 0 || fact_of_sym[i] >= n_facts) return ORC_EINVAL;
    for (int s = 0; s < B; ++s)
        for (int i = 0; i < n; ++i) {
            int64_t o = ((int64_t)s * n + i) * k;
            mask[o] = (uint64_t)1 << fact_of_sym[i];
            pprob[o] = proof_prob(mask[o], fact_prob + (int64_t)s * n_facts, n_facts);
            for (int x = 1; x < k; ++x) { mask[o + x] = ABSENT; pprob[o + x] = 0.0f; }
            if (prob) prob[(int64_t)s * ld + i] = pprob[o] < 1.0f ? pprob[o] : 1.0f;
        }
    return ORC_OK;
}

/* Apply with K=2 under DTKP-AM (Eq. 1-3 with Table 1): the conjunction of two
 * tags is top_k over all pairs of their proofs of the union of the two fact
 * sets (App. A.1), inconsistent unions dropped; the disjunction over all tuples
 * producing one symbol is top_k of everything gathered.  top_k of a union of
 * top_k's equals top_k of the union, so one top_k over all candidate proofs of
 * an output symbol is the same result.
 * am [B,na,k], bm [B,nb,k]; outputs om/op [B,S,k], oprob [B,ldo]. */
int orc_dtkp_apply2(int B, int64_t n, const int32_t *ti, const int32_t *tj, const int32_t *to,
                    int na, int nb, int S, const int32_t *out_syms,
                    int k, int n_facts, const int32_t *group, const float *fact_prob,
                    const uint64_t *am, const uint64_t *bm,
                    uint64_t *om, float *op, float *oprob, int64_t ldo)
{
    int err;
    if (n_facts < 0 || n_facts > 63 || k < 1) return ORC_EINVAL;
    int *col = tuple_columns(n, ti, tj, to, na, nb, S, out_syms, &err);
    if (!col) return err;
    /* tuples per column, to size the candidate lists */
    int64_t *cnt = (int64_t *)calloc((size_t)(S + 1), sizeof(int64_t));
    for (int64_t t = 0; t < n; ++t) if (col[t] >= 0) cnt[col[t] + 1]++;
    for (int c = 0; c < S; ++c) cnt[c + 1] += cnt[c];
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (int s = 0; s < B; ++s) {
        const float *fp = fact_prob + (int64_t)s * n_facts;
        proof_t *cand = (proof_t *)malloc(sizeof(proof_t) * (size_t)(cnt[S] > 0 ? cnt[S] : 1) * (size_t)k * (size_t)k);
        int64_t *fill = (int64_t *)calloc((size_t)(S > 0 ? S : 1), sizeof(int64_t));
        for (int64_t t = 0; t < n; ++t) {
            int c = col[t];
            if (c < 0) continue;
            for (int x = 0; x < k; ++x) {
                uint64_t ma = am[((int64_t)s * na + ti[t]) * k + x];
                if (ma == ABSENT) continue;
                for (int y = 0; y < k; ++y) {
                    uint64_t mb = bm[((int64_t)s * nb + tj[t]) * k + y];
                    if (mb == ABSENT) continue;
                    uint64_t m = ma | mb;
                    if (proof_conflict(m, n_facts, group)) continue;
                    proof_t *q = cand + cnt[c] * k * k + fill[c]++;
                    q->mask = m; q->prob = proof_prob(m, fp, n_facts);
                }
            }
        }
        for (int c = 0; c < S; ++c) {
            int64_t o = ((int64_t)s * S + c) * k;
            float pr = keep_top_k(cand + cnt[c] * k * k, (int)fill[c], k, om + o, op + o);
            if (oprob) oprob[(int64_t)s * ldo + c] = pr;
        }
        free(cand); free(fill);
    }
    free(cnt); free(col);
    return ORC_OK;
}

/* Union under DTKP-AM: common symbols get top_k(cat(t, t')) (Table 1) with
 * repeated proofs counted once; one-sided symbols are copied. */
int orc_dtkp_union(int B, int S, const int32_t *ia, const int32_t *ib, int na, int nb, int k,
                   const uint64_t *am, const float *ap, const uint64_t *bm, const float *bp,
                   uint64_t *om, float *op, float *oprob, int64_t ldo)
{
    proof_t *cand = (proof_t *)malloc(sizeof(proof_t) * 2 * (size_t)k);
    for (int s = 0; s < B; ++s)
        for (int c = 0; c < S; ++c) {
            int m = 0;
            if (ia[c] >= 0)
                for (int x = 0; x < k; ++x) {
                    int64_t o = ((int64_t)s * na + ia[c]) * k + x;
                    if (am[o] != ABSENT) { cand[m].mask = am[o]; cand[m++].prob = ap[o]; }
                }
            if (ib[c] >= 0)
                for (int x = 0; x < k; ++x) {
                    int64_t o = ((int64_t)s * nb + ib[c]) * k + x;
                    if (bm[o] != ABSENT) { cand[m].mask = bm[o]; cand[m++].prob = bp[o]; }
                }
            int64_t o = ((int64_t)s * S + c) * k;
            float pr = keep_top_k(cand, m, k, om + o, op + o);
            if (oprob) oprob[(int64_t)s * ldo + c] = pr;
        }
    free(cand);
    return ORC_OK;
}

/* Filter under DTKP-AM: kept symbols carry their whole tag over. */
int orc_dtkp_filter(int B, int n, int k, const uint8_t *pred, const uint64_t *im, const float *ip,
                    const float *iprob, int64_t ldi, uint64_t *om, float *op, float *oprob, int64_t ldo)
{
    int K = 0;
    for (int i = 0; i < n; ++i) K += pred[i] ? 1 : 0;
    for (int s = 0; s < B; ++s) {
        int m = 0;
        for (int i = 0; i < n; ++i) {
            if (!pred[i]) continue;
            for (int x = 0; x < k; ++x) {
                om[((int64_t)s * K + m) * k + x] = im[((int64_t)s * n + i) * k + x];
                op[((int64_t)s * K + m) * k + x] = ip[((int64_t)s * n + i) * k + x];
            }
            if (oprob) oprob[(int64_t)s * ldo + m] = iprob[(int64_t)s * ldi + i];
            ++m;
        }
    }
    return ORC_OK;
}

/* Gradient of the tag probabilities w.r.t. the probabilities of the input
 * facts (Sec. 3.2: Pr(t) = sum_i prod_j norm(t_ij), clamped at 1 as every
 * disjunction of probabilities is; App. A.2: the clamp passes gradient inside
 * and on its bounds).  Which proofs top_k kept is a constant of the
 * differentiation.  d Pr / d p_f = sum over the kept proofs that hold fact f of
 * the product of the proof's other facts.  The clamp decision is taken on the
 * float sum of the kept proofs' float probabilities in rank order, the quantity
 * the forward pass clamps.
 * mask [B,n,k]; g [B,ldg]; gfact [B,n_facts], overwritten. */
int orc_dtkp_prob_bwd(int B, int n, int k, int n_facts, const uint64_t *mask, const float *fact_prob,
                      const float *g, int64_t ldg, float *gfact)
{
    if (n_facts < 0 || n_facts > 63 || k < 1) return ORC_EINVAL;
    for (int s = 0; s < B; ++s) {
        const float *fp = fact_prob + (int64_t)s * n_facts;
        double acc[64];
        for (int f = 0; f < n_facts; ++f) acc[f] = 0.0;
        for (int i = 0; i < n; ++i) {
            const uint64_t *m = mask + ((int64_t)s * n + i) * k;
            float sum = 0.0f;
            for (int x = 0; x < k; ++x)
                if (m[x] != ABSENT) sum = sum + proof_prob(m[x], fp, n_facts);
            if (!(sum <= 1.0f)) continue;
            const double gi = (double)g[(int64_t)s * ldg + i];
            for (int x = 0; x < k; ++x) {
                if (m[x] == ABSENT) continue;
                for (int f = 0; f < n_facts; ++f) {
                    if (!((m[x] >> f) & 1u)) continue;
                    double others = 1.0;
                    for (int f2 = 0; f2 < n_facts; ++f2)
                        if (f2 != f && ((m[x] >> f2) & 1u)) others *= (double)fp[f2];
                    acc[f] += gi * others;
                }
            }
        }
        for (int f = 0; f < n_facts; ++f) gfact[(int64_t)s * n_facts + f] = (float)acc[f];
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------ Apply over K Distributions */

/* Symbol side of Apply / ApplyIf for any arity K >= 1 (Sec. 3.1.2, Eq. 1-2): the
 * admitted tuples arrive as idx[t*K + l] = position of the t-th tuple's symbol in
 * operand l, ascending lexicographically, each once; to[t] is the produced symbol
 * id (negative: the condition of ApplyIf rejects the tuple). */
static int *ktuple_columns(int K, int64_t n, const int32_t *idx, const int32_t *to, const int32_t *n_sym,
                           int S, const int32_t *out_syms, int *err)
{
    int *col = (int *)malloc(sizeof(int) * (size_t)(n > 0 ? n : 1));
    *err = ORC_OK;
    if (!col) { *err = ORC_ENOMEM; return NULL; }
    if (K < 1) *err = ORC_EINVAL;
    for (int64_t t = 0; t < n && !*err; ++t) {
        for (int l = 0; l < K; ++l)
            if (idx[t * K + l] < 0 || idx[t * K + l] >= n_sym[l]) *err = ORC_EINVAL;
        if (t > 0) {
            int order = 0;
            for (int l = 0; l < K && order == 0; ++l)
                order = (idx[t * K + l] > idx[(t - 1) * K + l]) - (idx[t * K + l] < idx[(t - 1) * K + l]);
            if (order <= 0) *err = ORC_EINVAL;
        }
        col[t] = to[t] < 0 ? -1 : find_col(S, out_syms, to[t]);
        if (to[t] >= 0 && col[t] < 0) *err = ORC_EINVAL;
    }
    if (*err) { free(col); return NULL; }
    return col;
}

/* Eq. 1-3 under DAMP for K operands: the tag of a tuple is the product of its K
 * input tags, the tag of an output symbol the clamped sum over the tuples that
 * produce it.  The decision quantity pre32 is the float sum in tuple order from 0
 * of one term per tuple: for K = 1 the tag itself is added; for K >= 2 the first
 * K-1 tags are multiplied left to right in float and the product enters through
 * one fused multiply-add with the last tag (K = 2 is then exactly the two-operand
 * rule above).
 * in[l] [B, ld[l]]; out [B,ldo]; pre32 / pre64 [B,S] optional. */
int orc_damp_applyk_fwd(int B, int K, int64_t n, const int32_t *idx, const int32_t *to, const int32_t *n_sym,
                        int S, const int32_t *out_syms, const float *const *in, const int64_t *ld,
                        float *out, int64_t ldo, float *pre32, double *pre64)
{
    int err;
    int *col = ktuple_columns(K, n, idx, to, n_sym, S, out_syms, &err);
    if (!col) return err;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (int s = 0; s < B; ++s) {
        double *acc = (double *)calloc((size_t)(S > 0 ? S : 1), sizeof(double));
        float *accf = (float *)calloc((size_t)(S > 0 ? S : 1), sizeof(float));
        for (int64_t t = 0; t < n; ++t) {
            if (col[t] < 0) continue;
            double prod = 1.0;
            for (int l = 0; l < K; ++l) prod *= (double)in[l][(int64_t)s * ld[l] + idx[t * K + l]];
            acc[col[t]] += prod;
            float head = in[0][(int64_t)s * ld[0] + idx[t * K]];
            for (int l = 1; l + 1 < K; ++l) head = head * in[l][(int64_t)s * ld[l] + idx[t * K + l]];
            if (K == 1) accf[col[t]] = accf[col[t]] + head;
            else accf[col[t]] = fmaf(head, in[K - 1][(int64_t)s * ld[K - 1] + idx[t * K + K - 1]], accf[col[t]]);
        }
        for (int c = 0; c < S; ++c) {
            out[(int64_t)s * ldo + c] = (float)(acc[c] < 1.0 ? acc[c] : 1.0);
            if (pre32) pre32[(int64_t)s * S + c] = accf[c];
            if (pre64) pre64[(int64_t)s * S + c] = acc[c];
        }
        free(acc); free(accf);
    }
    free(col);
    return ORC_OK;
}

/* Vector-Jacobian product of the above: with gh[c] = g[c] * [pre32[c] <= 1],
 *     gin_l[i] = sum over admitted tuples t with idx[t][l] = i of gh[col(t)] * prod_{m != l} in_m[idx[t][m]].
 * gin[l] [B, ldgi[l]] is overwritten (a NULL entry is skipped). */
int orc_damp_applyk_bwd(int B, int K, int64_t n, const int32_t *idx, const int32_t *to, const int32_t *n_sym,
                        int S, const int32_t *out_syms, const float *const *in, const int64_t *ld,
                        const float *g, int64_t ldg, float *const *gin, const int64_t *ldgi)
{
    int err;
    int *col = ktuple_columns(K, n, idx, to, n_sym, S, out_syms, &err);
    if (!col) return err;
    int total = 0;
    for (int l = 0; l < K; ++l) total += n_sym[l];
    float *pre32 = (float *)malloc(sizeof(float) * (size_t)(B > 0 ? B : 1) * (size_t)(S > 0 ? S : 1));
    float *tmp = (float *)malloc(sizeof(float) * (size_t)(B > 0 ? B : 1) * (size_t)(S > 0 ? S : 1));
    err = orc_damp_applyk_fwd(B, K, n, idx, to, n_sym, S, out_syms, in, ld, tmp, S, pre32, NULL);
    if (!err) {
#pragma omp parallel for schedule(static) num_threads(g_threads)
        for (int s = 0; s < B; ++s) {
            double *d = (double *)calloc((size_t)(total > 0 ? total : 1), sizeof(double));
            for (int64_t t = 0; t < n; ++t) {
                if (col[t] < 0) continue;
                if (!(pre32[(int64_t)s * S + col[t]] <= 1.0f)) continue;
                const double gh = (double)g[(int64_t)s * ldg + col[t]];
                int base = 0;
                for (int l = 0; l < K; ++l) {
                    double others = 1.0;
                    for (int m = 0; m < K; ++m)
                        if (m != l) others *= (double)in[m][(int64_t)s * ld[m] + idx[t * K + m]];
                    d[base + idx[t * K + l]] += gh * others;
                    base += n_sym[l];
                }
            }
            int base = 0;
            for (int l = 0; l < K; ++l) {
                if (gin[l])
                    for (int i = 0; i < n_sym[l]; ++i) gin[l][(int64_t)s * ldgi[l] + i] = (float)d[base + i];
                base += n_sym[l];
            }
            free(d);
        }
    }
    free(pre32); free(tmp); free(col);
    return err;
}

/* Eq. 1-3 under DTKP-AM for K operands.  Table 1 gives the conjunction as a
 * binary operation; the tag of a tuple is taken as that operation folded over the
 * operands left to right, every intermediate result pruned to its top k proofs
 * (K = 1: the operand's tag unchanged).  The disjunction over the tuples producing
 * one symbol is one top_k over all their proofs, as in the two-operand routine.
 * im[l] [B, n_sym[l], k]; outputs om/op [B,S,k], oprob [B,ldo]. */
int orc_dtkp_applyk(int B, int K, int64_t n, const int32_t *idx, const int32_t *to, const int32_t *n_sym,
                    int S, const int32_t *out_syms, int k, int n_facts, const int32_t *group,
                    const float *fact_prob, const uint64_t *const *im,
                    uint64_t *om, float *op, float *oprob, int64_t ldo)
{
    int err;
    if (n_facts < 0 || n_facts > 63 || k < 1) return ORC_EINVAL;
    int *col = ktuple_columns(K, n, idx, to, n_sym, S, out_syms, &err);
    if (!col) return err;
    int64_t *cnt = (int64_t *)calloc((size_t)(S + 1), sizeof(int64_t));
    for (int64_t t = 0; t < n; ++t) if (col[t] >= 0) cnt[col[t] + 1]++;
    for (int c = 0; c < S; ++c) cnt[c + 1] += cnt[c];
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (int s = 0; s < B; ++s) {
        const float *fp = fact_prob + (int64_t)s * n_facts;
        proof_t *cand = (proof_t *)malloc(sizeof(proof_t) * (size_t)(cnt[S] > 0 ? cnt[S] : 1) * (size_t)k);
        proof_t *pairs = (proof_t *)malloc(sizeof(proof_t) * (size_t)k * (size_t)k);
        uint64_t *cm = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)k);
        float *cp = (float *)malloc(sizeof(float) * (size_t)k);
        int64_t *fill = (int64_t *)calloc((size_t)(S > 0 ? S : 1), sizeof(int64_t));
        for (int64_t t = 0; t < n; ++t) {
            int c = col[t];
            if (c < 0) continue;
            for (int x = 0; x < k; ++x) {
                cm[x] = im[0][((int64_t)s * n_sym[0] + idx[t * K]) * k + x];
                cp[x] = cm[x] == ABSENT ? 0.0f : proof_prob(cm[x], fp, n_facts);
            }
            for (int l = 1; l < K; ++l) {
                int m = 0;
                for (int x = 0; x < k; ++x) {
                    if (cm[x] == ABSENT) continue;
                    for (int y = 0; y < k; ++y) {
                        uint64_t mb = im[l][((int64_t)s * n_sym[l] + idx[t * K + l]) * k + y];
                        if (mb == ABSENT) continue;
                        uint64_t u = cm[x] | mb;
                        if (proof_conflict(u, n_facts, group)) continue;
                        pairs[m].mask = u; pairs[m].prob = proof_prob(u, fp, n_facts); ++m;
                    }
                }
                keep_top_k(pairs, m, k, cm, cp);
            }
            for (int x = 0; x < k; ++x) {
                if (cm[x] == ABSENT) continue;
                proof_t *q = cand + cnt[c] * k + fill[c]++;
                q->mask = cm[x]; q->prob = cp[x];
            }
        }
        for (int c = 0; c < S; ++c) {
            int64_t o = ((int64_t)s * S + c) * k;
            float pr = keep_top_k(cand + cnt[c] * k, (int)fill[c], k, om + o, op + o);
            if (oprob) oprob[(int64_t)s * ldo + c] = pr;
        }
        free(cand); free(pairs); free(cm); free(cp); free(fill);
    }
    free(cnt); free(col);
    return ORC_OK;
}
