/* Drives the C oracle (oracle/pods_oracle.c, compiled into this program) under AddressSanitizer and
 * UndefinedBehaviorSanitizer over a sweep of shapes, ties and degenerate groups, and checks what does not
 * need a second implementation: every index is in range, no index repeats, the kept set is the (m-k) lowest
 * plus the k highest of the (reward, index) order, and the advantages of each group sum to zero. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_select(const float *rewards, int32_t B, int32_t n, int32_t m, int32_t *sel_idx, int32_t *sel_k,
                  int32_t threads);
int oracle_advantage(const float *rewards, const int32_t *sel_idx, int32_t B, int32_t n, int32_t m,
                     double std_eps, double *adv);

static uint64_t state = 0x9E3779B97F4A7C15ull;
static uint32_t next_u32(void) {
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)(state >> 33);
}

static int before(const float *r, int a, int b) { return r[a] < r[b] || (r[a] == r[b] && a < b); }

static int check_case(int B, int n, int m, int kind) {
    float *r = (float *)malloc(sizeof(float) * (size_t)B * n);
    int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * (size_t)B * m);
    int32_t *k = (int32_t *)malloc(sizeof(int32_t) * (size_t)B);
    double *adv = (double *)malloc(sizeof(double) * (size_t)B * m);
    char *seen = (char *)malloc((size_t)n);
    for (long i = 0; i < (long)B * n; ++i) {
        uint32_t u = next_u32();
        r[i] = kind == 0 ? (float)(u % 2) : kind == 1 ? (float)(u % 5) * 0.25f - 0.5f
             : kind == 2 ? 0.1f : (float)u / 4294967296.0f - 0.5f;
    }
    int bad = 0;
    if (oracle_select(r, B, n, m, idx, k, 3) >= 0) bad = 1;
    if (oracle_advantage(r, idx, B, n, m, 0.0, adv) != 0) bad = 1;
    for (int b = 0; b < B && !bad; ++b) {
        const float *row = r + (size_t)b * n;
        const int32_t *s = idx + (size_t)b * m;
        for (int i = 0; i < n; ++i) seen[i] = 0;
        for (int j = 0; j < m; ++j) {
            if (s[j] < 0 || s[j] >= n || seen[s[j]]) { bad = 2; break; }
            seen[s[j]] = 1;
        }
        if (bad) break;
        if (k[b] < 0 || k[b] > m) { bad = 3; break; }
        /* ascending inside the low part and inside the high part */
        for (int j = 0; j + 1 < m - k[b]; ++j) if (!before(row, s[j], s[j + 1])) bad = 4;
        for (int j = m - k[b]; j + 1 < m; ++j) if (!before(row, s[j], s[j + 1])) bad = 4;
        /* nothing left out sits below the low part's last element or above the high part's first */
        for (int i = 0; i < n && !bad; ++i) {
            if (seen[i]) continue;
            if (m - k[b] > 0 && before(row, i, s[m - k[b] - 1])) bad = 5;
            if (k[b] > 0 && before(row, s[m - k[b]], i)) bad = 5;
        }
        double sum = 0.0;
        for (int j = 0; j < m; ++j) sum += adv[(size_t)b * m + j];
        if (!(fabs(sum) < 1e-9 * m)) bad = 6;
    }
    if (bad) fprintf(stderr, "oracle check failed: B=%d n=%d m=%d kind=%d code=%d\n", B, n, m, kind, bad);
    free(r); free(idx); free(k); free(adv); free(seen);
    return bad;
}

int main(void) {
    static const int shapes[][3] = {{3, 1, 1}, {5, 2, 1}, {9, 7, 3}, {4, 16, 16}, {11, 63, 17}, {64, 64, 16},
                                    {7, 65, 5}, {40, 256, 64}, {6, 255, 64}, {3, 1000, 333}, {2, 4096, 1024}};
    for (unsigned c = 0; c < sizeof(shapes) / sizeof(shapes[0]); ++c)
        for (int kind = 0; kind < 4; ++kind)
            if (check_case(shapes[c][0], shapes[c][1], shapes[c][2], kind)) return 1;
    /* rejected arguments must be rejected without touching the buffers */
    if (oracle_select(0, 1, 4, 2, 0, 0, 1) != 1) return 2;
    float one = 0.0f;
    int32_t out = 0;
    if (oracle_select(&one, 1, 1, 2, &out, 0, 1) != 1) return 2;   /* m > n */
    printf("oracle sanitizer run ok\n");
    return 0;
}
