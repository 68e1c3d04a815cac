/* Test driver: runs every entry point of the CPU oracle on small seeded inputs, with tight output buffers, so that a
 * build with -fsanitize=address,undefined sees every loop and buffer of it.  Prints "ok" and the hit counts; any
 * sanitizer report makes the process fail.  Compiled together with oracle/kgc_oracle.c by tests/test_sanitizers.py. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

void kgco_compute_range(const double *sa, int64_t m, const double *sb, int64_t n, double eps, int32_t impl, int64_t *s, int64_t *e);
void kgco_dist_triples(const double *E, int32_t d, const double *Rv, int32_t p, const int32_t *h, const int32_t *r,
                       const int32_t *t, int64_t n, double *out);
int64_t kgco_join_ab(const double *A, const double *B, int64_t N, int32_t d, int32_t R, int32_t b_per_rel, int32_t p,
                     double delta, int64_t cap, int32_t *oh, int32_t *or_, int32_t *ot, double *od);
int32_t kgco_top1(const double *E, int64_t N, int32_t d, const double *Rv, int32_t R, int32_t p, int32_t exclude_self,
                  int32_t *oh, int32_t *or_, int32_t *ot, double *od);
int64_t kgco_topk(const double *E, int64_t N, int32_t d, const double *Rv, int32_t R, int32_t p, int32_t exclude_self,
                  int64_t k, int32_t *oh, int32_t *or_, int32_t *ot, double *od);
int64_t kgco_join(const double *E, int64_t N, int32_t d, const double *Rv, int32_t R, int32_t p, double delta,
                  int32_t mode, const double *pivot, int32_t range_impl, int64_t cap, int32_t *oh, int32_t *or_,
                  int32_t *ot, double *od, int64_t *evaluated);

static uint64_t state = 0x9e3779b97f4a7c15ull;
static double unif(void)
{
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return (double)(state >> 11) / 9007199254740992.0 - 0.5;
}

int main(void)
{
    const int64_t N = 157;
    const int32_t d = 13, R = 3;
    double *E = malloc(sizeof(double) * N * d), *Rv = malloc(sizeof(double) * R * d);
    for (int64_t i = 0; i < N * d; ++i) E[i] = unif() + (double)((i / d) % 5);       /* five loose clusters */
    for (int64_t i = 0; i < R * d; ++i) Rv[i] = 0.2 * unif();
    for (int p = 1; p <= 2; ++p) {
        const double delta = p == 2 ? 1.3 : 3.6;
        int64_t counts[4];
        for (int mode = 0; mode < 3; ++mode) {
            for (int impl = 0; impl < (mode == 2 ? 2 : 1); ++impl) {
                /* first with no room at all, then with exactly the room needed */
                int64_t ev = 0;
                const int64_t total = kgco_join(E, N, d, Rv, R, p, delta, mode, NULL, impl, 0, NULL, NULL, NULL, NULL, &ev);
                if (total < 0) return 2;
                int32_t *oh = malloc(sizeof(int32_t) * (total + 1)), *orr = malloc(sizeof(int32_t) * (total + 1)),
                        *ot = malloc(sizeof(int32_t) * (total + 1));
                double *od = malloc(sizeof(double) * (total + 1));
                const int64_t again = kgco_join(E, N, d, Rv, R, p, delta, mode, NULL, impl, total, oh, orr, ot, od, &ev);
                if (again != total) return 3;
                double *chk = malloc(sizeof(double) * (total + 1));
                kgco_dist_triples(E, d, Rv, p, oh, orr, ot, total, chk);
                for (int64_t i = 0; i < total; ++i)
                    if (fabs(chk[i] - od[i]) > 1e-12 * (1.0 + od[i]) || od[i] > delta) return 4;
                counts[mode + impl] = total;
                free(oh); free(orr); free(ot); free(od); free(chk);
            }
        }
        if (counts[0] != counts[1] || counts[0] != counts[2] || counts[0] != counts[3] || counts[0] < N) return 5;
        /* the general form on the same connectors: a = e + r, b = e */
        double *A = malloc(sizeof(double) * R * N * d);
        for (int32_t r = 0; r < R; ++r)
            for (int64_t i = 0; i < N * d; ++i) A[(int64_t)r * N * d + i] = E[i] + Rv[(int64_t)r * d + i % d];
        int32_t *oh = malloc(sizeof(int32_t) * counts[0]), *orr = malloc(sizeof(int32_t) * counts[0]), *ot = malloc(sizeof(int32_t) * counts[0]);
        double *od = malloc(sizeof(double) * counts[0]);
        if (kgco_join_ab(A, E, N, d, R, 0, p, delta, counts[0], oh, orr, ot, od) != counts[0]) return 6;
        if (kgco_join_ab(A, A, N, d, R, 1, p, delta, 7, oh, orr, ot, od) < 0) return 7;       /* short buffer */
        int32_t bh, br, bt;
        double bd;
        for (int ex = 0; ex < 2; ++ex) {
            if (kgco_top1(E, N, d, Rv, R, p, ex, &bh, &br, &bt, &bd) != 1) return 8;
            const int64_t k = 19;
            if (kgco_topk(E, N, d, Rv, R, p, ex, k, oh, orr, ot, od) != k) return 9;
            if (fabs(od[0] - bd) > 0.0 && od[0] < bd) return 10;
        }
        printf("p=%d hits=%lld\n", p, (long long)counts[0]);
        free(A); free(oh); free(orr); free(ot); free(od);
    }
    /* the range search on its own, with empty sides and ties */
    double sa[5] = {0.0, 1.0, 1.0, 2.5, 9.0}, sb[6] = {-1.0, 1.0, 1.0, 1.5, 3.0, 3.0};
    int64_t s[5], e[5];
    for (int impl = 0; impl < 2; ++impl) {
        kgco_compute_range(sa, 5, sb, 6, 0.5, impl, s, e);
        kgco_compute_range(sa, 0, sb, 6, 0.5, impl, s, e);
        kgco_compute_range(sa, 5, sb, 0, 0.5, impl, s, e);
    }
    free(E); free(Rv);
    puts("ok");
    return 0;
}
