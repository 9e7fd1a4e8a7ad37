/*
 * TEST ORACLE -- not part of the product path.
 *
 * Double-precision cyclic Jacobi eigensolver for a batch of small real
 * symmetric matrices.  It computes, straight from the definition, what the
 * paper's solver is defined to return (Sec. 3.1 Eq. (1) together with the
 * "whole ED" equation at the end of Sec. 3.2.1):  A = V diag(lambda) V^T with
 * V orthogonal.  Eigenvalues are returned in ascending order, eigenvectors
 * are the columns of V.
 *
 * The algorithm is the textbook row-cyclic Jacobi method (Golub & Van Loan,
 * "Matrix Computations", Sec. 8.5): every off-diagonal entry is annihilated in
 * turn by a plane rotation whose angle is the smaller root of
 *     t^2 + 2*theta*t - 1 = 0,   theta = (a_qq - a_pp) / (2 a_pq),
 * which is the same "angle within 45 degrees" choice the paper makes for its
 * 2x2 solve in App. A.3.  It shares no code, no constants and no helper with
 * the GPU path (which uses Householder tridiagonalisation + shifted QR).
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call
 * this file.
 *
 * Input convention (same as the GPU library): row-major [batch][n][n] fp32,
 * only the LOWER triangle (i >= j) is read and mirrored.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_MAX_SWEEPS 64

/* One matrix.  W: n*n work copy (row-major), V: n*n output (row-major,
 * columns are eigenvectors), lam: n eigenvalues.  Returns sweeps used. */
static int jacobi_one(int n, double *W, double *V, double *lam, int *perm)
{
    int i, j, p, q, r, sweep;
    double normF2 = 0.0;

    for (i = 0; i < n; ++i)
        for (j = 0; j < n; ++j)
            V[i * n + j] = (i == j) ? 1.0 : 0.0;
    for (i = 0; i < n; ++i)
        for (j = 0; j < n; ++j)
            normF2 += W[i * n + j] * W[i * n + j];

    for (sweep = 0; sweep < ORACLE_MAX_SWEEPS; ++sweep) {
        double off2 = 0.0;
        for (p = 0; p < n; ++p)
            for (q = p + 1; q < n; ++q)
                off2 += W[p * n + q] * W[p * n + q];
        /* converged: off-diagonal mass is below 1e-17 of the matrix norm */
        if (off2 == 0.0 || off2 <= 1e-34 * normF2)
            break;

        for (p = 0; p < n - 1; ++p) {
            for (q = p + 1; q < n; ++q) {
                double apq = W[p * n + q];
                double app, aqq, theta, t, c, s;
                if (apq == 0.0 || fabs(apq) < 1e-300)
                    continue;
                app = W[p * n + p];
                aqq = W[q * n + q];
                theta = (aqq - app) / (2.0 * apq);
                if (isinf(theta)) {
                    /* a_pq utterly negligible against the diagonal gap */
                    t = 0.5 / theta;
                } else {
                    t = 1.0 / (fabs(theta) + sqrt(theta * theta + 1.0));
                    if (theta < 0.0)
                        t = -t;
                }
                c = 1.0 / sqrt(t * t + 1.0);
                s = t * c;

                W[p * n + p] = app - t * apq;
                W[q * n + q] = aqq + t * apq;
                W[p * n + q] = 0.0;
                W[q * n + p] = 0.0;
                for (r = 0; r < n; ++r) {
                    double arp, arq;
                    if (r == p || r == q)
                        continue;
                    arp = W[r * n + p];
                    arq = W[r * n + q];
                    W[r * n + p] = c * arp - s * arq;
                    W[r * n + q] = s * arp + c * arq;
                    W[p * n + r] = W[r * n + p];
                    W[q * n + r] = W[r * n + q];
                }
                for (r = 0; r < n; ++r) {
                    double vrp = V[r * n + p];
                    double vrq = V[r * n + q];
                    V[r * n + p] = c * vrp - s * vrq;
                    V[r * n + q] = s * vrp + c * vrq;
                }
            }
        }
    }

    /* ascending order, stable (insertion sort on an index permutation) */
    for (i = 0; i < n; ++i)
        perm[i] = i;
    for (i = 1; i < n; ++i) {
        int key = perm[i];
        double kv = W[key * n + key];
        j = i - 1;
        while (j >= 0 && W[perm[j] * n + perm[j]] > kv) {
            perm[j + 1] = perm[j];
            --j;
        }
        perm[j + 1] = key;
    }
    for (i = 0; i < n; ++i)
        lam[i] = W[perm[i] * n + perm[i]];
    /* permute columns of V; reuse the off-diagonal storage of W as scratch */
    for (r = 0; r < n; ++r) {
        for (i = 0; i < n; ++i)
            W[r * n + i] = V[r * n + perm[i]];
    }
    memcpy(V, W, (size_t)n * n * sizeof(double));
    return sweep;
}

/*
 * A      : host, [batch][n][n] fp32, lower triangle trusted
 * evals  : host, [batch][n]    fp64, ascending
 * evecs  : host, [batch][n][n] fp64, evecs[b][i][j] = component i of the
 *          eigenvector belonging to evals[b][j]
 * sweeps : host, [batch] or NULL, Jacobi sweeps used per matrix
 * threads: number of OpenMP threads; <= 0 means all available
 * returns the number of threads actually used, or -1 on bad arguments.
 */
int oracle_syevd_f64(const float *A, int batch, int n, double *evals,
                     double *evecs, int *sweeps, int threads)
{
    int used = 1;
    if (!A || !evals || !evecs || batch < 0 || n < 1)
        return -1;
#ifdef _OPENMP
    if (threads <= 0)
        threads = omp_get_max_threads();
    used = threads;
#else
    (void)threads;
#endif

#ifdef _OPENMP
#pragma omp parallel num_threads(threads)
#endif
    {
        double *W = (double *)malloc((size_t)n * n * sizeof(double));
        int *perm = (int *)malloc((size_t)n * sizeof(int));
        int b;
#ifdef _OPENMP
#pragma omp for schedule(static)
#endif
        for (b = 0; b < batch; ++b) {
            const float *Ab = A + (size_t)b * n * n;
            int i, j, sw;
            for (i = 0; i < n; ++i)
                for (j = 0; j <= i; ++j) {
                    double v = (double)Ab[i * n + j];
                    W[i * n + j] = v;
                    W[j * n + i] = v;
                }
            sw = jacobi_one(n, W, evecs + (size_t)b * n * n,
                            evals + (size_t)b * n, perm);
            if (sweeps)
                sweeps[b] = sw;
        }
        free(W);
        free(perm);
    }
    return used;
}

/* Same solver on fp64 input (used by the pins that need an exact-in-double
 * matrix, e.g. A = Q diag(lambda) Q^T with prescribed lambda). */
int oracle_syevd_f64_in64(const double *A, int batch, int n, double *evals,
                          double *evecs, int *sweeps, int threads)
{
    int used = 1;
    if (!A || !evals || !evecs || batch < 0 || n < 1)
        return -1;
#ifdef _OPENMP
    if (threads <= 0)
        threads = omp_get_max_threads();
    used = threads;
#else
    (void)threads;
#endif

#ifdef _OPENMP
#pragma omp parallel num_threads(threads)
#endif
    {
        double *W = (double *)malloc((size_t)n * n * sizeof(double));
        int *perm = (int *)malloc((size_t)n * sizeof(int));
        int b;
#ifdef _OPENMP
#pragma omp for schedule(static)
#endif
        for (b = 0; b < batch; ++b) {
            const double *Ab = A + (size_t)b * n * n;
            int i, j, sw;
            for (i = 0; i < n; ++i)
                for (j = 0; j <= i; ++j) {
                    W[i * n + j] = Ab[i * n + j];
                    W[j * n + i] = Ab[i * n + j];
                }
            sw = jacobi_one(n, W, evecs + (size_t)b * n * n,
                            evals + (size_t)b * n, perm);
            if (sweeps)
                sweeps[b] = sw;
        }
        free(W);
        free(perm);
    }
    return used;
}

int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
