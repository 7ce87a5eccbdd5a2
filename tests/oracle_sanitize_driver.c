/* Driver for the sanitizer run of the CPU oracle (tests/test_oracle_sanitizers.py): calls every batch driver and the
 * entry points with (m, s) given on small seeded inputs, including the row-parallel branch (order >= 256).
 * Built together with oracle/expm_oracle.c under -fsanitize=address,undefined; prints a checksum so that the calls
 * cannot be optimised away. */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_expm_batch(const double *W, int n, int batch, double eps, double *X, int *m, int *s, double *n1, double *n2,
                      int *near, int threads);
int oracle_expm_ps_batch(const double *W, int n, int batch, double eps, double *X, int *m, int *s, double *norms, int *near,
                         int threads);
int oracle_expm_baseline_batch(const double *W, int n, int batch, double eps, double *X, int *m, int *s, double *n1, int *near,
                               int threads);
int oracle_lowrank_batch(const double *A1, const double *A2, int n, int t, int batch, double eps, double *X, int *m, int *flag,
                         double *v1, int *near, int threads);
int oracle_expm_forced(const double *W, int n, int m, int s, int plus16, double *X, int threads);
int oracle_lowrank_forced(const double *A1, const double *A2, int n, int t, int m, double *X);
int oracle_matmul_threads(const double *A, const double *B, double *C, int n, int threads);

static unsigned long long state = 88172645463325252ULL;
static double rnd(void)
{
    state ^= state << 13;
    state ^= state >> 7;
    state ^= state << 17;
    return (double)(state >> 11) / 9007199254740992.0 - 0.5;
}

int main(void)
{
    double sum = 0.0;
    const int sizes[4] = {1, 7, 33, 257};
    for (int c = 0; c < 4; ++c) {
        const int n = sizes[c], batch = n > 100 ? 2 : 5;
        const size_t nn = (size_t)n * n;
        double *W = malloc(sizeof(double) * nn * batch), *X = malloc(sizeof(double) * nn * batch);
        int *m = malloc(sizeof(int) * batch), *s = malloc(sizeof(int) * batch), *near = malloc(sizeof(int) * batch);
        double *n1 = malloc(sizeof(double) * batch), *n2 = malloc(sizeof(double) * batch), *n4 = malloc(sizeof(double) * 4 * batch);
        for (int b = 0; b < batch; ++b) {
            const double scale = b == 0 ? 0.0 : pow(10.0, -3.0 + 1.2 * b) / sqrt((double)n);
            for (size_t e = 0; e < nn; ++e)
                W[b * nn + e] = scale * rnd();
        }
        if (oracle_expm_batch(W, n, batch, ldexp(1.0, -53), X, m, s, n1, n2, near, 3) < 0) return 2;
        sum += X[nn * batch - 1] + m[batch - 1] + s[batch - 1];
        if (oracle_expm_ps_batch(W, n, batch, 1e-8, X, m, s, n4, near, 2) < 0) return 2;
        sum += X[0] + m[batch - 1];
        if (oracle_expm_forced(W + nn * (batch - 1), n, 15, 2, 1, X, 2) != 0) return 2;
        sum += X[nn - 1];
        if (oracle_expm_forced(W + nn * (batch - 1), n, 0, 0, 0, X, 1) != 0) return 2;
        if (n <= 33) {
            if (oracle_expm_baseline_batch(W, n, batch, 1e-8, X, m, s, n1, near, 3) < 0) return 2;
            sum += X[nn - 1] + m[batch - 1];
        }
        if (oracle_matmul_threads(W, W, X, n, 3) < 1) return 2;
        free(W); free(X); free(m); free(s); free(near); free(n1); free(n2); free(n4);
    }
    {
        const int n = 19, t = 4, batch = 3;
        double *A1 = malloc(sizeof(double) * n * t * batch), *A2 = malloc(sizeof(double) * n * t * batch);
        double *X = malloc(sizeof(double) * n * n * batch), v1[3];
        int m[3], flag[3], near[3];
        for (int e = 0; e < n * t * batch; ++e) { A1[e] = 0.3 * rnd(); A2[e] = 0.3 * rnd(); }
        if (oracle_lowrank_batch(A1, A2, n, t, batch, ldexp(1.0, -24), X, m, flag, v1, near, 2) < 0) return 2;
        sum += X[n * n * batch - 1] + m[0];
        if (oracle_lowrank_forced(A1, A2, n, t, 6, X) != 0) return 2;
        sum += X[5];
        free(A1); free(A2); free(X);
    }
    printf("checksum %.17g\n", sum);
    return isfinite(sum) ? 0 : 3;
}
