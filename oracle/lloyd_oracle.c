/*
 * Reference ("oracle") implementation of one exact Lloyd k-means iteration.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 definition that
 * the GPU library is checked against.  It shares no code with the GPU path and
 * the GPU path never calls it.  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg may load it.
 *
 * What it follows (Flash-KMeans paper, Section 3.1):
 *   Eq. (1)  objective      J = sum_i || x_i - c_{a_i} ||^2
 *   Eq. (2)  assignment     D_ik = || x_i - c_k ||^2 ,  a_i = argmin_k D_ik
 *   Eq. (3)  update         n_k = #{i : a_i = k},  s_k = sum_{a_i = k} x_i,
 *                           c_k <- s_k / n_k
 * The paper's kernels reach exactly these results (it states that neither the
 * formulation is changed nor an approximation introduced), so the oracle is the
 * definition itself, not the paper's tiling.
 *
 * Readings where the paper is silent:
 *   - ties in the argmin: the lowest centroid index wins;
 *   - a cluster that receives no point keeps its previous centroid;
 *   - indices are 0-based (the paper counts from 1);
 *   - D_ik is evaluated by direct differences, summed over the feature index in
 *     ascending order, in fp64.  The norm expansion of Section 3.1 is an
 *     implementation device with cancellation and is not used here.
 *
 * Inputs are the stored values (fp16 / bf16 / fp32 bits widened exactly to
 * fp32, or fp64 as is); all arithmetic is fp64.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_pins.py
 * (hand-worked integer cases, brute force written a second way, closed forms,
 * invariants, an independent library distance routine).  Nothing is unpinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static inline double load_x(const void* X, int x_is_f64, int64_t idx) {
    return x_is_f64 ? ((const double*)X)[idx] : (double)((const float*)X)[idx];
}

int fko_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Eq. (2).  X[N,d] row-major (float32 if x_is_f64 == 0, else float64),
 * C[K,d] row-major float64.
 * Outputs (each may be NULL except assign):
 *   assign[i]  argmin_k D_ik, lowest k on ties
 *   best[i]    D_{i,assign[i]}
 *   second[i]  smallest D_ik over k != assign[i]  (+inf when K == 1)
 *   xnorm2[i]  || x_i ||^2
 *
 * For each point the K distances are built up together, feature by feature:
 * acc[k] += (x_ij - c_kj)^2 for j = 0..d-1.  Every D_ik is therefore the plain
 * ascending-j sum; only the loop nesting (j outside, k inside) is chosen so the
 * compiler can vectorise over k without reassociating any sum.
 */
void fko_assign(const void* X, int x_is_f64, const double* C,
                int64_t N, int d, int K,
                int32_t* assign, double* best, double* second, double* xnorm2) {
    /* Ct[j*K + k] = C[k*d + j] : same numbers, transposed for contiguous k. */
    double* Ct = (double*)malloc(sizeof(double) * (size_t)K * (size_t)d);
    for (int k = 0; k < K; ++k)
        for (int j = 0; j < d; ++j) Ct[(size_t)j * K + k] = C[(size_t)k * d + j];

#pragma omp parallel
    {
        double* acc = (double*)malloc(sizeof(double) * (size_t)K);
#pragma omp for schedule(static)
        for (int64_t i = 0; i < N; ++i) {
            for (int k = 0; k < K; ++k) acc[k] = 0.0;
            double xn = 0.0;
            for (int j = 0; j < d; ++j) {
                const double x = load_x(X, x_is_f64, i * d + j);
                const double* row = Ct + (size_t)j * K;
                xn += x * x;
                for (int k = 0; k < K; ++k) {
                    const double diff = x - row[k];
                    acc[k] += diff * diff;
                }
            }
            /* ascending k with strict '<' : lowest index wins ties */
            int bk = 0;
            double bd = acc[0];
            for (int k = 1; k < K; ++k)
                if (acc[k] < bd) { bd = acc[k]; bk = k; }
            double sd = INFINITY;
            for (int k = 0; k < K; ++k)
                if (k != bk && acc[k] < sd) sd = acc[k];
            assign[i] = bk;
            if (best) best[i] = bd;
            if (second) second[i] = sd;
            if (xnorm2) xnorm2[i] = xn;
        }
        free(acc);
    }
    free(Ct);
}

/*
 * Eq. (3) with the empty-cluster reading.  assign[i] in [0,K).
 * Outputs: counts[K] (int64), sums[K,d] (fp64, may be NULL),
 *          C_new[K,d] = sums/counts, or C_prev row where counts == 0.
 * Serial over points, in index order: the sum s_k is the plain left-to-right
 * fp64 sum of the member rows.
 * Returns 0, or -1 if an assignment is out of range (outputs then undefined).
 */
int fko_update(const void* X, int x_is_f64, const int32_t* assign, const double* C_prev,
               int64_t N, int d, int K,
               double* C_new, int64_t* counts, double* sums) {
    double* s = sums ? sums : (double*)malloc(sizeof(double) * (size_t)K * (size_t)d);
    memset(s, 0, sizeof(double) * (size_t)K * (size_t)d);
    memset(counts, 0, sizeof(int64_t) * (size_t)K);
    int rc = 0;
    for (int64_t i = 0; i < N; ++i) {
        const int32_t k = assign[i];
        if (k < 0 || k >= K) { rc = -1; break; }
        counts[k] += 1;
        double* sk = s + (size_t)k * d;
        for (int j = 0; j < d; ++j) sk[j] += load_x(X, x_is_f64, i * d + j);
    }
    if (rc == 0) {
        for (int k = 0; k < K; ++k) {
            for (int j = 0; j < d; ++j) {
                const size_t o = (size_t)k * d + j;
                C_new[o] = counts[k] > 0 ? s[o] / (double)counts[k] : C_prev[o];
            }
        }
    }
    if (!sums) free(s);
    return rc;
}

/*
 * Eq. (1): J = sum_i || x_i - c_{a_i} ||^2, direct differences, fp64,
 * summed over points in index order.
 */
double fko_inertia(const void* X, int x_is_f64, const double* C, const int32_t* assign,
                   int64_t N, int d) {
    double J = 0.0;
    for (int64_t i = 0; i < N; ++i) {
        const double* c = C + (size_t)assign[i] * d;
        double D = 0.0;
        for (int j = 0; j < d; ++j) {
            const double diff = load_x(X, x_is_f64, i * d + j) - c[j];
            D += diff * diff;
        }
        J += D;
    }
    return J;
}

/*
 * D_ik for one (point, centroid) pair; used by the tests that sample single
 * outputs of full-size runs.
 */
double fko_pair_dist(const void* X, int x_is_f64, const double* C,
                     int64_t i, int k, int d) {
    double D = 0.0;
    for (int j = 0; j < d; ++j) {
        const double diff = load_x(X, x_is_f64, i * d + j) - C[(size_t)k * d + j];
        D += diff * diff;
    }
    return D;
}
