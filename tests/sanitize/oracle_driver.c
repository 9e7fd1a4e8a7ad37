/* Host-only sanitizer driver for the CPU oracle (oracle/jacobi.c), built with
 * -fsanitize=address,undefined by tests/test_sanitizers.py.  It runs the oracle over the
 * shapes the pins use (every n up to 64, one and many threads, diagonal / zero / NaN inputs,
 * float and double entry points) with heap buffers of exactly the documented sizes, so that any
 * access outside [batch][n][n] / [batch][n] / [batch], any signed overflow or misaligned access is reported, and checks the
 * results against invariants of the definition (trace, residual, orthogonality). */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_syevd_f64(const float* A, int batch, int n, double* evals, double* evecs, int* sweeps, int threads);
int oracle_syevd_f64_in64(const double* A, int batch, int n, double* evals, double* evecs, int* sweeps, int threads);
int oracle_max_threads(void);

static unsigned long long state = 88172645463325252ull;
static double rnd(void) {               /* xorshift64: values in (-1, 1) */
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return (double)(state >> 11) / 4503599627370496.0 - 1.0;
}

static int check(const double* A, int n, const double* lam, const double* V, const char* what) {
    double tr = 0, fro = 0, res = 0, orth = 0;
    for (int i = 0; i < n; ++i) tr += A[i * n + i];
    for (int i = 0; i < n * n; ++i) fro += A[i] * A[i];
    double s = 0;
    for (int i = 0; i < n; ++i) s += lam[i];
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j) {
            double av = 0, g = 0;
            for (int k = 0; k < n; ++k) { av += A[i * n + k] * V[k * n + j]; g += V[k * n + i] * V[k * n + j]; }
            av -= V[i * n + j] * lam[j];
            res += av * av;
            g -= (i == j);
            orth += g * g;
        }
    for (int i = 1; i < n; ++i) if (lam[i] < lam[i - 1]) { fprintf(stderr, "%s n=%d: not ascending\n", what, n); return 1; }
    fro = sqrt(fro) + 1e-300;
    if (fabs(s - tr) > 1e-12 * n * fro || sqrt(res) > 1e-12 * n * fro || sqrt(orth) > 1e-12 * n) {
        fprintf(stderr, "%s n=%d: trace %g residual %g orth %g\n", what, n, fabs(s - tr), sqrt(res), sqrt(orth));
        return 1;
    }
    return 0;
}

int main(void) {
    int bad = 0;
    for (int n = 1; n <= 64; ++n) {
        const int batch = (n <= 8) ? 7 : 3;
        float* Af = malloc(sizeof(float) * batch * n * n);
        double* Ad = malloc(sizeof(double) * batch * n * n);
        double* lam = malloc(sizeof(double) * batch * n);
        double* V = malloc(sizeof(double) * batch * n * n);
        int* sw = malloc(sizeof(int) * batch);
        for (int b = 0; b < batch; ++b)
            for (int i = 0; i < n; ++i)
                for (int j = 0; j <= i; ++j) {
                    double x = (b == 0) ? (i == j ? rnd() : 0.0) : (b == 1 ? 0.0 : rnd());   /* diagonal, zero, dense */
                    Af[(b * n + i) * n + j] = (float)x;
                    Af[(b * n + j) * n + i] = (float)x;
                }
        for (int i = 0; i < batch * n * n; ++i) Ad[i] = (double)Af[i];
        for (int threads = 0; threads <= 2; ++threads) {
            if (oracle_syevd_f64(Af, batch, n, lam, V, sw, threads) < 0) { fprintf(stderr, "f32 entry refused n=%d\n", n); bad = 1; }
            for (int b = 0; b < batch; ++b) bad |= check(Ad + b * n * n, n, lam + b * n, V + b * n * n, "f32 entry");
            if (oracle_syevd_f64_in64(Ad, batch, n, lam, V, sw, threads) < 0) { fprintf(stderr, "f64 entry refused n=%d\n", n); bad = 1; }
            for (int b = 0; b < batch; ++b) bad |= check(Ad + b * n * n, n, lam + b * n, V + b * n * n, "f64 entry");
        }
        /* non-finite input must terminate and stay inside its buffers */
        Af[0] = NAN;
        Af[batch * n * n - 1] = INFINITY;
        oracle_syevd_f64(Af, batch, n, lam, V, sw, 1);
        /* sweeps pointer is optional */
        oracle_syevd_f64_in64(Ad, batch, n, lam, V, NULL, 1);
        free(Af); free(Ad); free(lam); free(V); free(sw);
    }
    /* argument errors are refused without touching the buffers */
    if (oracle_syevd_f64(NULL, 1, 4, NULL, NULL, NULL, 1) >= 0) { fprintf(stderr, "NULL accepted\n"); bad = 1; }
    { double one = 1.0; if (oracle_syevd_f64_in64(&one, -1, 1, &one, &one, NULL, 1) >= 0) { fprintf(stderr, "batch < 0 accepted\n"); bad = 1; } }
    if (oracle_max_threads() < 1) bad = 1;
    printf(bad ? "FAILED\n" : "oracle sanitizer driver OK\n");
    return bad;
}
