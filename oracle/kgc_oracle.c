/*
 * CPU oracle for the TransE knowledge-graph-completion join.  TEST INFRASTRUCTURE ONLY:
 * it is called by the tests, by the smoke check and by the benchmark's CPU-baseline leg,
 * never by the product path, and it shares no code with the GPU library.
 *
 * What it computes (Definition 1 and the straightforward algorithm of Section 3.1, with the
 * TransE distance of Section 4.3):  all (h, r, t) in E x R x E with
 *     dist_3(h, r, t) = || e_h + r - e_t ||_p  <=  delta,       p in {1, 2},
 * inclusive, self pairs h == t included, nothing filtered.  Arithmetic is IEEE double,
 * dimensions summed in ascending order.
 *
 * Modes (all must return the same set):
 *   0  brute force: the triple loop, every distance summed in full (this one is the definition);
 *   1  early abandon: the dimension loop stops once the partial sum of non-negative terms
 *      can no longer come back under the threshold; hits are still summed in full;
 *   2  pivot filter: the fast completion algorithm of Section 4.5 on the CPU -- connectors
 *      a = h + r, b = t, pivot distances distA, distB, sort, valid range [s_i, e_i] of
 *      Lemma 2, full test on the range only.  distB and its order are computed once because
 *      they do not depend on r (Section 5.2).
 *
 * Build:  gcc -O2 -fopenmp -shared -fPIC -o libkgc_oracle.so kgc_oracle.c -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- distance of one triple, Section 4.3: dist(connector_1(h,r), connector_2(t,r)) ---- */
static double triple_dist(const double *eh, const double *rv, const double *et, int32_t d, int32_t p)
{
    double s = 0.0;
    if (p == 2) {
        for (int32_t i = 0; i < d; ++i) {
            double x = eh[i] + rv[i] - et[i];
            s += x * x;
        }
        return sqrt(s);
    }
    for (int32_t i = 0; i < d; ++i) {
        double x = eh[i] + rv[i] - et[i];
        s += fabs(x);
    }
    return s;
}

/* Same sum, but gives up (returns +inf) once the partial sum exceeds `giveup`.  The terms are
 * non-negative, so partial sums never decrease in floating point either. */
static double triple_dist_abandon(const double *eh, const double *rv, const double *et, int32_t d, int32_t p,
                                  double giveup)
{
    double s = 0.0;
    if (p == 2) {
        for (int32_t i = 0; i < d; ++i) {
            double x = eh[i] + rv[i] - et[i];
            s += x * x;
            if (s > giveup) return INFINITY;
        }
        return sqrt(s);
    }
    for (int32_t i = 0; i < d; ++i) {
        double x = eh[i] + rv[i] - et[i];
        s += fabs(x);
        if (s > giveup) return INFINITY;
    }
    return s;
}

/* metric dist(x, y) = ||x - y||_p of Section 4.2, used for pivot distances */
static double metric_dist(const double *x, const double *y, int32_t d, int32_t p)
{
    double s = 0.0;
    for (int32_t i = 0; i < d; ++i) {
        double v = x[i] - y[i];
        s += (p == 2) ? v * v : fabs(v);
    }
    return (p == 2) ? sqrt(s) : s;
}

/* ---- growable per-thread result list ---- */
typedef struct {
    int32_t *h, *r, *t;
    double *dist;
    int64_t n, cap;
} hitlist;

static void hl_push(hitlist *L, int32_t h, int32_t r, int32_t t, double dist)
{
    if (L->n == L->cap) {
        int64_t nc = L->cap ? 2 * L->cap : 1024;
        L->h = (int32_t *)realloc(L->h, (size_t)nc * sizeof(int32_t));
        L->r = (int32_t *)realloc(L->r, (size_t)nc * sizeof(int32_t));
        L->t = (int32_t *)realloc(L->t, (size_t)nc * sizeof(int32_t));
        L->dist = (double *)realloc(L->dist, (size_t)nc * sizeof(double));
        L->cap = nc;
    }
    L->h[L->n] = h; L->r[L->n] = r; L->t[L->n] = t; L->dist[L->n] = dist;
    L->n++;
}

/* ---- Lemma 2: valid range of each a in the sorted order of b ----
 * sa[0..m), sb[0..n) ascending.  For each i, s[i] and e[i] are the first and last j with
 * |sa[i] - sb[j]| <= eps (eq. "condition"); an empty set is reported as e[i] = s[i] - 1.
 * impl 0: two pointers moving forward only, possible because s and e are non-decreasing
 *         in i (eq. "se2"); O(m + n).
 * impl 1: two binary searches per i; O(m log n).
 */
void kgco_compute_range(const double *sa, int64_t m, const double *sb, int64_t n, double eps, int32_t impl,
                        int64_t *s, int64_t *e)
{
    if (impl == 0) {
        int64_t j = 0;
        for (int64_t i = 0; i < m; ++i) {           /* first j with sb[j] >= sa[i] - eps */
            while (j < n && sb[j] < sa[i] - eps) ++j;
            s[i] = j;
        }
        j = 0;
        for (int64_t i = 0; i < m; ++i) {           /* last j with sb[j] <= sa[i] + eps */
            while (j < n && sb[j] <= sa[i] + eps) ++j;
            e[i] = j - 1;
        }
        return;
    }
    for (int64_t i = 0; i < m; ++i) {
        double lo_v = sa[i] - eps, hi_v = sa[i] + eps;
        int64_t lo = 0, hi = n;
        while (lo < hi) {                            /* lower bound of lo_v */
            int64_t mid = lo + (hi - lo) / 2;
            if (sb[mid] < lo_v) lo = mid + 1; else hi = mid;
        }
        s[i] = lo;
        lo = 0; hi = n;
        while (lo < hi) {                            /* upper bound of hi_v */
            int64_t mid = lo + (hi - lo) / 2;
            if (sb[mid] <= hi_v) lo = mid + 1; else hi = mid;
        }
        e[i] = lo - 1;
    }
}

typedef struct { double key; int64_t idx; } keyidx;
static int cmp_keyidx(const void *a, const void *b)
{
    const keyidx *x = (const keyidx *)a, *y = (const keyidx *)b;
    if (x->key < y->key) return -1;
    if (x->key > y->key) return 1;
    return (x->idx > y->idx) - (x->idx < y->idx);
}

/* ---- distances of listed triples (used to re-verify GPU output and to choose delta) ---- */
void kgco_dist_triples(const double *E, int32_t d, const double *Rv, int32_t p, const int32_t *h,
                       const int32_t *r, const int32_t *t, int64_t n, double *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < n; ++k)
        out[k] = triple_dist(E + (int64_t)h[k] * d, Rv + (int64_t)r[k] * d, E + (int64_t)t[k] * d, d, p);
}

/* ---- the join in its general form (Section 4.3): the caller supplies the connector outputs ----
 * A[R][N][d] holds a_{r,h} = connector_1(h, r); B[RB][N][d] holds b_{r,t} = connector_2(t, r), with RB = R when
 * connector_2 depends on the relation (b_per_rel != 0) and RB = 1 when it does not (TransE: b = t).  All
 * (h, r, t) with dist(a_{r,h}, b_{r,t}) = ||a - b||_p <= delta, by the plain triple loop in double, every
 * distance summed in full, dimensions ascending.  Same output convention as kgco_join. */
int64_t kgco_join_ab(const double *A, const double *B, int64_t N, int32_t d, int32_t R, int32_t b_per_rel, int32_t p,
                     double delta, int64_t cap, int32_t *oh, int32_t *or_, int32_t *ot, double *od)
{
    if ((p != 1 && p != 2) || N < 0 || R < 0 || d < 0) return -1;
    int64_t total = 0;
    for (int32_t r = 0; r < R; ++r) {
        const double *Ar = A + (int64_t)r * N * d;
        const double *Br = B + (b_per_rel ? (int64_t)r * N * d : 0);
        for (int64_t h = 0; h < N; ++h)
            for (int64_t t = 0; t < N; ++t) {
                double v = metric_dist(Ar + h * d, Br + t * d, d, p);
                if (v <= delta) {
                    if (total < cap) { oh[total] = (int32_t)h; or_[total] = r; ot[total] = (int32_t)t; od[total] = v; }
                    ++total;
                }
            }
    }
    return total;
}

/* ---- top-1: the smallest distance over all triples (the top-1 score of Section 3.3), optionally
 * leaving out the self pairs h == t (the second quantity that section looks at).  Plain triple loop,
 * every distance summed in full.  Among equal distances the smallest (r, h, t) wins.  Returns 1 and fills
 * the outputs, or 0 when no triple is eligible (N == 0, R == 0, or exclude_self with N == 1), or -1 on a
 * bad argument. */
int32_t kgco_top1(const double *E, int64_t N, int32_t d, const double *Rv, int32_t R, int32_t p, int32_t exclude_self,
                  int32_t *oh, int32_t *or_, int32_t *ot, double *od)
{
    if ((p != 1 && p != 2) || N < 0 || R < 0 || d < 0) return -1;
    int found = 0;
    double best = INFINITY;
    int32_t bh = -1, br = -1, bt = -1;
#pragma omp parallel
    {
        int lfound = 0;
        double lbest = INFINITY;
        int32_t lh = -1, lr = -1, lt = -1;
#pragma omp for schedule(static) collapse(2) nowait
        for (int32_t r = 0; r < R; ++r)
            for (int64_t h = 0; h < N; ++h)
                for (int64_t t = 0; t < N; ++t) {
                    if (exclude_self && h == t) continue;
                    double v = triple_dist(E + h * d, Rv + (int64_t)r * d, E + t * d, d, p);
                    /* within a thread (r, h, t) ascends, so '<' keeps the first of equal distances */
                    if (!lfound || v < lbest) { lfound = 1; lbest = v; lh = (int32_t)h; lr = r; lt = (int32_t)t; }
                }
#pragma omp critical
        {
            if (lfound) {
                int better = !found || lbest < best;
                if (!better && lbest == best)
                    better = (lr < br) || (lr == br && (lh < bh || (lh == bh && lt < bt)));
                if (better) { found = 1; best = lbest; bh = lh; br = lr; bt = lt; }
            }
        }
    }
    if (!found) return 0;
    *oh = bh; *or_ = br; *ot = bt; *od = best;
    return 1;
}

/* ---- top-k: the k smallest distances over all (eligible) triples, the plain definition: every distance
 * is computed in full and the k smallest by (distance, r, h, t) are kept (a bounded insertion per thread,
 * merged at the end).  Writes min(k, eligible) records in ascending (distance, r, h, t) order and returns
 * that number, or -1 on a bad argument. */
typedef struct { double v; int32_t r, h, t; } topk_rec;
static int topk_less(const topk_rec *a, const topk_rec *b)
{
    if (a->v != b->v) return a->v < b->v;
    if (a->r != b->r) return a->r < b->r;
    if (a->h != b->h) return a->h < b->h;
    return a->t < b->t;
}
static void topk_insert(topk_rec *best, int64_t *n, int64_t k, const topk_rec *x)
{
    if (*n == k && !topk_less(x, &best[k - 1])) return;
    int64_t i = (*n < k) ? (*n)++ : k - 1;
    while (i > 0 && topk_less(x, &best[i - 1])) { best[i] = best[i - 1]; --i; }
    best[i] = *x;
}
int64_t kgco_topk(const double *E, int64_t N, int32_t d, const double *Rv, int32_t R, int32_t p, int32_t exclude_self,
                  int64_t k, int32_t *oh, int32_t *or_, int32_t *ot, double *od)
{
    if ((p != 1 && p != 2) || N < 0 || R < 0 || d < 0 || k < 0) return -1;
    if (k == 0) return 0;
    topk_rec *all = (topk_rec *)malloc((size_t)k * sizeof(topk_rec));
    int64_t nall = 0;
#pragma omp parallel
    {
        topk_rec *best = (topk_rec *)malloc((size_t)k * sizeof(topk_rec));
        int64_t n = 0;
#pragma omp for schedule(static) collapse(2) nowait
        for (int32_t r = 0; r < R; ++r)
            for (int64_t h = 0; h < N; ++h)
                for (int64_t t = 0; t < N; ++t) {
                    if (exclude_self && h == t) continue;
                    topk_rec x;
                    x.v = triple_dist(E + h * d, Rv + (int64_t)r * d, E + t * d, d, p);
                    x.r = r; x.h = (int32_t)h; x.t = (int32_t)t;
                    topk_insert(best, &n, k, &x);
                }
#pragma omp critical
        for (int64_t i = 0; i < n; ++i) topk_insert(all, &nall, k, &best[i]);
        free(best);
    }
    for (int64_t i = 0; i < nall; ++i) { oh[i] = all[i].h; or_[i] = all[i].r; ot[i] = all[i].t; od[i] = all[i].v; }
    free(all);
    return nall;
}

/* ---- the join ----
 * E[N][d], Rv[R][d] row-major doubles.  pivot: d doubles or NULL for the zero vector (mode 2).
 * range_impl: see kgco_compute_range (mode 2).  Writes min(total, cap) hits to oh/or_/ot/od in an
 * unspecified order and returns the total.  *evaluated (may be NULL) receives the number of
 * triples whose distance was started.  Returns -1 on a bad argument.
 */
int64_t kgco_join(const double *E, int64_t N, int32_t d, const double *Rv, int32_t R, int32_t p, double delta,
                  int32_t mode, const double *pivot, int32_t range_impl, int64_t cap, int32_t *oh,
                  int32_t *or_, int32_t *ot, double *od, int64_t *evaluated)
{
    if ((p != 1 && p != 2) || N < 0 || R < 0 || d < 0 || mode < 0 || mode > 2) return -1;
    int nthreads = 1;
#ifdef _OPENMP
    nthreads = omp_get_max_threads();
#endif
    hitlist *lists = (hitlist *)calloc((size_t)nthreads, sizeof(hitlist));
    int64_t n_eval = 0;

    /* a partial sum above this can never give dist <= delta; two ulps of room keep the
     * decision identical to the full-sum test at the boundary */
    double giveup = (p == 2) ? delta * delta : delta;
    giveup = nextafter(nextafter(giveup, INFINITY), INFINITY);

    keyidx *kb = NULL, *ka = NULL;
    double *sa = NULL, *sb = NULL, *zero = NULL;
    int64_t *s = NULL, *e = NULL;
    if (mode == 2 && N > 0) {
        kb = (keyidx *)malloc((size_t)N * sizeof(keyidx));
        ka = (keyidx *)malloc((size_t)N * sizeof(keyidx));
        sa = (double *)malloc((size_t)N * sizeof(double));
        sb = (double *)malloc((size_t)N * sizeof(double));
        s = (int64_t *)malloc((size_t)N * sizeof(int64_t));
        e = (int64_t *)malloc((size_t)N * sizeof(int64_t));
        zero = (double *)calloc((size_t)(d > 0 ? d : 1), sizeof(double));
        const double *pv = pivot ? pivot : zero;
        /* B = Connector_2(E, r) = E for every r: distB and its order once */
        for (int64_t t = 0; t < N; ++t) { kb[t].key = metric_dist(pv, E + t * d, d, p); kb[t].idx = t; }
        qsort(kb, (size_t)N, sizeof(keyidx), cmp_keyidx);
        for (int64_t j = 0; j < N; ++j) sb[j] = kb[j].key;
    }

    for (int32_t r = 0; r < R; ++r) {
        const double *rv = Rv + (int64_t)r * d;
        if (mode != 2) {
#pragma omp parallel reduction(+ : n_eval)
            {
                int tid = 0;
#ifdef _OPENMP
                tid = omp_get_thread_num();
#endif
                hitlist *L = &lists[tid];
#pragma omp for schedule(static)
                for (int64_t h = 0; h < N; ++h) {
                    const double *eh = E + h * d;
                    for (int64_t t = 0; t < N; ++t) {
                        double dist = (mode == 0) ? triple_dist(eh, rv, E + t * d, d, p)
                                                  : triple_dist_abandon(eh, rv, E + t * d, d, p, giveup);
                        if (dist <= delta) hl_push(L, (int32_t)h, r, (int32_t)t, dist);
                    }
                    n_eval += N;
                }
            }
            continue;
        }
        if (N == 0) continue;
        /* A = Connector_1(E, r) = E + r; distA, sort, ranges */
        const double *pv = pivot ? pivot : zero;
#pragma omp parallel
        {
            double *a = (double *)malloc((size_t)(d > 0 ? d : 1) * sizeof(double));
#pragma omp for schedule(static)
            for (int64_t h = 0; h < N; ++h) {
                for (int32_t i = 0; i < d; ++i) a[i] = E[h * d + i] + rv[i];
                ka[h].key = metric_dist(pv, a, d, p);
                ka[h].idx = h;
            }
            free(a);
        }
        qsort(ka, (size_t)N, sizeof(keyidx), cmp_keyidx);
        for (int64_t i = 0; i < N; ++i) sa[i] = ka[i].key;
        /* the pivot distances carry rounding of their own; widen the window by a hair so the
         * filter stays a superset (extra candidates fail the full test) */
        double eps = delta + 1e-9 * (1.0 + fabs(delta));
        if (delta < 0) eps = delta;                  /* negative threshold: nothing qualifies */
        kgco_compute_range(sa, N, sb, N, eps, range_impl, s, e);
#pragma omp parallel reduction(+ : n_eval)
        {
            int tid = 0;
#ifdef _OPENMP
            tid = omp_get_thread_num();
#endif
            hitlist *L = &lists[tid];
#pragma omp for schedule(dynamic, 64)
            for (int64_t i = 0; i < N; ++i) {
                int64_t h = ka[i].idx;
                for (int64_t j = s[i]; j <= e[i]; ++j) {
                    int64_t t = kb[j].idx;
                    double dist = triple_dist(E + h * d, rv, E + t * d, d, p);
                    if (dist <= delta) hl_push(L, (int32_t)h, r, (int32_t)t, dist);
                }
                if (e[i] >= s[i]) n_eval += e[i] - s[i] + 1;
            }
        }
    }

    int64_t total = 0, w = 0;
    for (int k = 0; k < nthreads; ++k) total += lists[k].n;
    for (int k = 0; k < nthreads; ++k) {
        for (int64_t q = 0; q < lists[k].n && w < cap; ++q, ++w) {
            oh[w] = lists[k].h[q]; or_[w] = lists[k].r[q]; ot[w] = lists[k].t[q]; od[w] = lists[k].dist[q];
        }
        free(lists[k].h); free(lists[k].r); free(lists[k].t); free(lists[k].dist);
    }
    free(lists); free(kb); free(ka); free(sa); free(sb); free(s); free(e); free(zero);
    if (evaluated) *evaluated = n_eval;
    return total;
}

int32_t kgco_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void kgco_set_num_threads(int32_t n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}
