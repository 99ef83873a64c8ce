/* Driver for the AddressSanitizer / UBSan build of the CPU oracle (tests/test_sanitizers.py).
 * Links oracle/lloyd_oracle.c directly, calls every entry on the hand-worked case whose
 * numbers come in on the command line (from tests/golden/handworked_2d.json) and on ragged,
 * degenerate and error-path inputs, and checks what can be checked without the oracle itself:
 * the golden values, counts that sum to N, member means, the error return of a bad id. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int fko_num_threads(void);
void fko_assign(const void* X, int x_is_f64, const double* C, int64_t N, int d, int K, int32_t* a,
                double* best, double* second, double* xnorm2);
int fko_update(const void* X, int x_is_f64, const int32_t* a, const double* C_prev, int64_t N, int d,
               int K, double* C_out, int64_t* counts, double* sums);
double fko_inertia(const void* X, int x_is_f64, const double* C, const int32_t* a, int64_t N, int d);
double fko_pair_dist(const void* X, int x_is_f64, const double* C, int64_t i, int k, int d);

static uint64_t rng = 88172645463325252ull;
static double rnd(void) {
    rng ^= rng << 13; rng ^= rng >> 7; rng ^= rng << 17;
    return (double)(rng >> 11) / 9007199254740992.0 - 0.5;
}

#define CHECK(c) do { if (!(c)) { fprintf(stderr, "CHECK failed line %d: %s\n", __LINE__, #c); return 1; } } while (0)

int main(int argc, char** argv) {
    /* argv: N d K, then X (N*d), C (K*d), assign (N), best (N) */
    CHECK(argc > 4);
    const int N = atoi(argv[1]), d = atoi(argv[2]), K = atoi(argv[3]);
    CHECK(argc == 4 + N * d + K * d + 2 * N);
    int p = 4;
    double* X = malloc(sizeof(double) * N * d);
    float* Xf = malloc(sizeof(float) * N * d);
    double* C = malloc(sizeof(double) * K * d);
    for (int i = 0; i < N * d; ++i) { X[i] = atof(argv[p++]); Xf[i] = (float)X[i]; }
    for (int i = 0; i < K * d; ++i) C[i] = atof(argv[p++]);
    int32_t* a = malloc(sizeof(int32_t) * N);
    double *best = malloc(sizeof(double) * N), *second = malloc(sizeof(double) * N), *xn = malloc(sizeof(double) * N);
    for (int f64 = 0; f64 < 2; ++f64) {
        fko_assign(f64 ? (void*)X : (void*)Xf, f64, C, N, d, K, a, best, second, xn);
        for (int i = 0; i < N; ++i) {
            CHECK(a[i] == atoi(argv[p + i]));
            CHECK(best[i] == atof(argv[p + N + i]));
            CHECK(fko_pair_dist(f64 ? (void*)X : (void*)Xf, f64, C, i, a[i], d) == best[i]);
        }
    }
    free(X); free(Xf); free(C); free(a); free(best); free(second); free(xn);

    /* ragged and degenerate shapes, exact-size buffers so that any overrun is caught */
    const int shapes[][3] = {{1, 1, 1}, {7, 3, 1}, {33, 5, 4}, {257, 17, 9}, {1000, 64, 31}, {64, 128, 200}, {5, 1, 8}};
    for (unsigned s = 0; s < sizeof(shapes) / sizeof(shapes[0]); ++s) {
        const int n = shapes[s][0], dd = shapes[s][1], k = shapes[s][2];
        float* x = malloc(sizeof(float) * n * dd);
        double* c = malloc(sizeof(double) * k * dd);
        for (int i = 0; i < n * dd; ++i) x[i] = (float)rnd();
        for (int i = 0; i < k * dd; ++i) c[i] = rnd();
        int32_t* as = malloc(sizeof(int32_t) * n);
        double *b1 = malloc(sizeof(double) * n), *b2 = malloc(sizeof(double) * n), *b3 = malloc(sizeof(double) * n);
        fko_assign(x, 0, c, n, dd, k, as, b1, b2, b3);
        double* co = malloc(sizeof(double) * k * dd);
        double* su = malloc(sizeof(double) * k * dd);
        int64_t* cnt = malloc(sizeof(int64_t) * k);
        CHECK(fko_update(x, 0, as, c, n, dd, k, co, cnt, su) == 0);
        int64_t tot = 0;
        for (int j = 0; j < k; ++j) {
            tot += cnt[j];
            if (cnt[j] == 0)
                for (int q = 0; q < dd; ++q) CHECK(co[j * dd + q] == c[j * dd + q]);   /* empty: kept */
        }
        CHECK(tot == n);
        /* member mean of the first point's cluster, feature 0, summed here in order */
        double m = 0; int64_t c0 = 0;
        for (int i = 0; i < n; ++i) if (as[i] == as[0]) { m += (double)x[i * dd]; ++c0; }
        CHECK(fabs(co[as[0] * dd] - m / (double)c0) <= 1e-12 * (1.0 + fabs(m)));
        const double J0 = fko_inertia(x, 0, c, as, n, dd), J1 = fko_inertia(x, 0, co, as, n, dd);
        CHECK(J1 <= J0 * (1.0 + 1e-12));
        /* an id outside [0, K) is an error, not a wild write */
        as[n - 1] = k;
        CHECK(fko_update(x, 0, as, c, n, dd, k, co, cnt, su) != 0);
        as[n - 1] = -1;
        CHECK(fko_update(x, 0, as, c, n, dd, k, co, cnt, su) != 0);
        free(x); free(c); free(as); free(b1); free(b2); free(b3); free(co); free(su); free(cnt);
    }
    CHECK(fko_num_threads() >= 1);
    printf("oracle sanitizer run ok\n");
    return 0;
}
