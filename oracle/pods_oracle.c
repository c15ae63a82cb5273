/* CPU oracle, batched: max-variance down-sampling and advantages.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain C, one prompt group at a time, OpenMP over groups.  Used by the tests (for batch sizes
 * the Python oracle is too slow for) and as the timed CPU baseline of the benchmark.  It
 * shares no code with the HIP kernels and the product library never links it.
 *
 *   oracle_select     Alg. 2 evaluated the way Theorem 1's proof describes: sort by
 *                     (reward, index), running sums of r and r^2 in double, one O(1)
 *                     evaluation per split k, strict ">" starting from k = 0.  The quantity
 *                     compared is m*sum(x^2) - (sum x)^2 = m^2 * Var (same arg-max, no division).
 *                     A split k whose multiset equals that of k-1 (the reward entering at the top
 *                     equals the one leaving at the bottom) is passed over, so rounding cannot
 *                     break a tie between identical multisets.
 *   oracle_advantage  a = (r - mu_S) / (sigma_S + std_eps) over the kept rewards, population
 *                     sigma (Sec. 3.2); all-equal kept rewards give zeros.
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC pods_oracle.c -o libpods_oracle.so -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct { float r; int32_t i; } item_t;

static int item_cmp(const void *pa, const void *pb) {
    const item_t *a = (const item_t *)pa, *b = (const item_t *)pb;
    if (a->r < b->r) return -1;
    if (a->r > b->r) return 1;          /* -0.0f and +0.0f fall through: equal rewards */
    return (a->i > b->i) - (a->i < b->i);
}

static void select_one(const float *r, int n, int m, item_t *it, double *p1, double *p2,
                       int32_t *out, int32_t *kout) {
    for (int i = 0; i < n; ++i) { it[i].r = r[i]; it[i].i = i; }
    qsort(it, (size_t)n, sizeof(item_t), item_cmp);   /* total order, so stability is moot */
    p1[0] = 0.0; p2[0] = 0.0;
    for (int j = 0; j < m; ++j) {                      /* only the m lowest are ever needed */
        double s = (double)it[j].r;
        p1[j + 1] = p1[j] + s;
        p2[j + 1] = p2[j] + s * s;
    }
    int best_k = 0;
    double best = (double)m * p2[m] - p1[m] * p1[m];
    double u1 = 0.0, u2 = 0.0;                         /* sums over the k highest */
    for (int k = 1; k <= m; ++k) {
        double top = (double)it[n - k].r;
        u1 += top; u2 += top * top;
        if (it[n - k].r == it[m - k].r) continue;
        double S = p1[m - k] + u1, Q = p2[m - k] + u2;
        double D = (double)m * Q - S * S;
        if (D > best) { best = D; best_k = k; }
    }
    for (int j = 0; j < m - best_k; ++j) out[j] = it[j].i;
    for (int j = 0; j < best_k; ++j) out[m - best_k + j] = it[n - best_k + j].i;
    if (kout) *kout = best_k;
}

int oracle_select(const float *rewards, int32_t B, int32_t n, int32_t m, int32_t *sel_idx,
                  int32_t *sel_k, int32_t threads) {
    if (!rewards || !sel_idx || B <= 0 || n <= 0 || m <= 0 || m > n) return 1;
    int used = 1;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
#endif
#pragma omp parallel
    {
        item_t *it = (item_t *)malloc(sizeof(item_t) * (size_t)n);
        double *p1 = (double *)malloc(sizeof(double) * (size_t)(m + 1));
        double *p2 = (double *)malloc(sizeof(double) * (size_t)(m + 1));
#ifdef _OPENMP
#pragma omp single
        used = omp_get_num_threads();
#endif
#pragma omp for schedule(static)
        for (int32_t b = 0; b < B; ++b)
            select_one(rewards + (size_t)b * n, n, m, it, p1, p2, sel_idx + (size_t)b * m,
                       sel_k ? sel_k + b : 0);
        free(it); free(p1); free(p2);
    }
    return -used;   /* negative thread count actually used = success */
}

int oracle_advantage(const float *rewards, const int32_t *sel_idx, int32_t B, int32_t n,
                     int32_t m, double std_eps, double *adv) {
    if (!rewards || !sel_idx || !adv || B <= 0 || n <= 0 || m <= 0 || m > n) return 1;
#pragma omp parallel for schedule(static)
    for (int32_t b = 0; b < B; ++b) {
        const float *r = rewards + (size_t)b * n;
        const int32_t *s = sel_idx + (size_t)b * m;
        double *a = adv + (size_t)b * m;
        double lo = r[s[0]], hi = r[s[0]], sum = 0.0;
        for (int j = 0; j < m; ++j) {
            double x = r[s[j]];
            sum += x; if (x < lo) lo = x; if (x > hi) hi = x;
        }
        if (lo == hi) { for (int j = 0; j < m; ++j) a[j] = 0.0; continue; }
        double mu = sum / m, ss = 0.0;
        for (int j = 0; j < m; ++j) { double x = r[s[j]] - mu; ss += x * x; }
        double sigma = sqrt(ss / m);
        for (int j = 0; j < m; ++j) a[j] = (r[s[j]] - mu) / (sigma + std_eps);
    }
    return 0;
}
