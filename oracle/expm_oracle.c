/*
 * CPU oracle for the Taylor scaling-and-squaring matrix exponential of
 * Sastre et al., "Improving Matrix Exponential for Generative AI Flows: A
 * Taylor-Based Approach Beyond Paterson-Stockmeyer" (arXiv 2512.20777).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a deliberately plain and slow reference
 * that the GPU library is checked against; it is not part of the product and
 * shares no code, header, table or helper with it.  Only the test-suite, the
 * smoke check and the benchmark's CPU-baseline leg may call it.
 *
 * What it computes, per matrix, all in IEEE double (fp32 inputs are widened
 * exactly by the caller):
 *   - the order m and scaling s of Algorithm 4 (Sec. 3.3), from ||W||_1 and
 *     the 1-norm of the explicitly formed W^2, with the bounds of the table
 *     that follows Algorithm 4;
 *   - the polynomial the evaluation formulas of Sec. 3.1 equal in exact
 *     arithmetic, by DIRECT summation of the Taylor series: T_m(A) for
 *     m in {1,2,4,8} (eq. for T_m(W) in Sec. 2.2) and T_15(A) + b16*A^16 for
 *     the 15+ approximant (Sec. 3.1, relation y22 = T15 + b16 A^16 with
 *     b16 = c1^4), A = W/2^s;
 *   - s repeated squarings (Algorithm 2).
 * Products are plain triple loops (row i, then k ascending, then column j),
 * no blocking, no BLAS.  Nothing here uses the evaluation formulas
 * y02/y12/y22 themselves, so agreement of the GPU path with this file also
 * checks those formulas against the definition.
 *
 * Readings of points the paper leaves open (also listed in the design notes):
 *   - norm: the 1-norm (max column abs sum), as in the printed algorithms;
 *   - acceptance test uses E1+E2 <= eps, the scaling uses each E_i separately
 *     and keeps the larger s (Algorithm 4 as printed);
 *   - s starts at 0 and is only raised, so a negative ceiling is ignored;
 *   - a non-finite E_i gives the cap s = 20;
 *   - m = 0 (zero matrix) returns the identity;
 *   - inputs are assumed finite (non-finite input is a host-side error path
 *     of the GPU library, not part of the method).
 *
 * The file also holds the Paterson-Stockmeyer variant of the paper (Algorithm 3 selection,
 * plain Taylor polynomial T_m, m in {1,2,4,6,9,12,16}) and the baseline of the paper's
 * comparison (its Algorithm 1); see further down.  Last comes the low-rank variant of Sec. 2.2
 * (W = A1 A2, the series in V = A2 A1, no scaling), pinned in tests/test_lowrank.py by the full-size
 * exponential of A1 A2, the rank-one closed form, a nilpotent pair and exact-rational checks of the order.
 *
 * Entry points that take (m, s) -- or the order of the low-rank series -- as given evaluate the same polynomial
 * through the same routine as the selecting calls (oracle_expm_forced, oracle_lowrank_forced); the parity tests use
 * them for matrices whose norms sit within 1e-6 of a switch point, where the device may take the other admissible
 * choice.  Pinned in tests/test_oracle_forced_pins.py: bit-equal to the selecting calls for the pair those select,
 * the closed form (sum_{k<=m} (x/2^s)^k/k! [+ b16 (x/2^s)^16])^(2^s) on 1 x 1 input in exact rationals, and the
 * rank-one closed form; the same file pins the row-parallel products of the batch drivers (order >= 256) by
 * bit-equality with the sequential ones, and the `near` flags of Algorithm 3 and of the baseline at hand-placed
 * switch points.
 *
 * Pins (tests/test_oracle_pins.py): the two worked selection examples of the
 * paper (Remark 1; Sec. 4.2, normal matrix of norm 12.8), closed forms
 * (diagonal, nilpotent, rotation, Remark-1 matrix), det/trace and inverse
 * identities, a brute-force long-double series, hand-computed products, and
 * closed-form switch points of the selection for W = x*I.
 */
#include <float.h>
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_S_CAP 20

/* ||W||_1 = max over columns j of sum_i |w_ij|  (Sec. 1, notation). */
double oracle_norm1(const double *W, int n)
{
    double best = 0.0;
    for (int j = 0; j < n; ++j) {
        double sum = 0.0;
        for (int i = 0; i < n; ++i)
            sum += fabs(W[(size_t)i * n + j]);
        if (sum > best)
            best = sum;
    }
    return best;
}

/* C = A*B, dense row-major n x n, plain triple loop.  Each c_ij is the sum
 * over k = 0..n-1 in ascending order.  `par` != 0 spreads rows over OpenMP
 * threads (used for large n only; the arithmetic per element is unchanged). */
static void matmul_impl(const double *A, const double *B, double *C, int n, int par)
{
#pragma omp parallel for schedule(static) if (par)
    for (int i = 0; i < n; ++i) {
        double *c = C + (size_t)i * n;
        for (int j = 0; j < n; ++j)
            c[j] = 0.0;
        for (int k = 0; k < n; ++k) {
            const double a = A[(size_t)i * n + k];
            const double *b = B + (size_t)k * n;
            for (int j = 0; j < n; ++j)
                c[j] += a * b[j];
        }
    }
}

void oracle_matmul(const double *A, const double *B, double *C, int n)
{
    matmul_impl(A, B, C, n, 0);
}

static double factorial(int k)
{
    double f = 1.0;
    for (int i = 2; i <= k; ++i)
        f *= (double)i;
    return f;
}

static double ipow(double x, int k)
{
    double p = 1.0;
    for (int i = 0; i < k; ++i)
        p *= x;
    return p;
}

/* b16 = c1^4 with c1 of the 15+ coefficient table (Sec. 3.1). */
double oracle_b16(void)
{
    const double c1 = 4.018761610201036e-4;
    return (c1 * c1) * (c1 * c1);
}

/*
 * Algorithm 4 on the two norms n1 = ||W||_1 and n2 = ||W^2||_1.
 * Orders M = [1,2,4,8,15]; bounds per order from the table after Algorithm 4:
 *   m=1 : E1 = n1^2/2!,            E2 = n1^3/3!
 *   m=2 : E1 = n2*n1/3!,           E2 = n2*n2/4!
 *   m=4 : E1 = n2^2*n1/5!,         E2 = n2^2*n2/6!
 *   m=8 : E1 = n2^4*n1/9!,         E2 = n2^4*n2/10!
 *   m=15: E1 = |1/16!-b16|*n2^8,   E2 = n2^8*n1/17!
 * First order with E1+E2 <= eps wins with s=0; otherwise m=15 and
 * s = max_i ceil(log2(E_i/eps)/(15+i)), i=1,2, capped at 20.
 * n2 is not looked at when n1 == 0 or the m=1 test passes.
 */
void oracle_select_from_norms(double n1, double n2, double eps, int *m_out, int *s_out)
{
    int m = 0, s = 0;
    double E1 = 0.0, E2 = 0.0;
    int found = 0;

    if (n1 == 0.0) {
        *m_out = 0;
        *s_out = 0;
        return;
    }
    /* m = 1 */
    m = 1;
    E1 = n1 * n1 / factorial(2);
    E2 = n1 * n1 * n1 / factorial(3);
    if (E1 + E2 <= eps)
        found = 1;

    if (!found) {
        const int Ms[3] = {2, 4, 8};
        for (int t = 0; t < 3 && !found; ++t) {
            m = Ms[t];
            const int k = m / 2;
            const double pk = ipow(n2, k);
            E1 = pk * n1 / factorial(m + 1);
            E2 = pk * n2 / factorial(m + 2);
            if (E1 + E2 <= eps)
                found = 1;
        }
    }
    if (!found) {
        m = 15;
        const double p8 = ipow(n2, 8);
        E1 = fabs(1.0 / factorial(16) - oracle_b16()) * p8;
        E2 = p8 * n1 / factorial(17);
        if (E1 + E2 <= eps)
            found = 1;
    }
    if (!found) {
        const double E[2] = {E1, E2};
        for (int i = 1; i <= 2; ++i) {
            int s1;
            if (!isfinite(E[i - 1])) {
                s1 = ORACLE_S_CAP;
            } else if (E[i - 1] <= 0.0) {
                s1 = 0;
            } else {
                const double q = ceil(log2(E[i - 1] / eps) / (double)(m + i));
                s1 = (q > (double)ORACLE_S_CAP) ? ORACLE_S_CAP : (q < 0.0 ? 0 : (int)q);
            }
            if (s1 > s)
                s = s1;
        }
    }
    if (s > ORACLE_S_CAP)
        s = ORACLE_S_CAP;
    *m_out = m;
    *s_out = s;
}

/*
 * Selection for one matrix.  Returns n1, n2 (n2 = -1 when W^2 was not needed)
 * and `near`: 1 when the choice changes if either norm moves by 1e-6 relative
 * (the four corners (n1(1+-1e-6), n2(1+-1e-6)) are re-run).  W2 (n*n doubles)
 * is scratch supplied by the caller.
 */
static void select_matrix(const double *W, int n, double eps, double *W2, int par,
                          int *m, int *s, double *n1_out, double *n2_out, int *near)
{
    const double n1 = oracle_norm1(W, n);
    double n2 = -1.0;
    int need_w2 = 0;
    if (n1 != 0.0) {
        /* W^2 is formed only once the m=1 test has failed (Algorithm 4).  The
         * corner re-runs below need it as soon as the test fails at the
         * upper corner, which (the bound is monotone in n1) is the first to
         * fail. */
        const double hi = n1 * (1.0 + 1e-6);
        const double worst = hi * hi / 2.0 + hi * hi * hi / 6.0;
        need_w2 = !(worst <= eps);
    }
    if (need_w2) {
        matmul_impl(W, W, W2, n, par);
        n2 = oracle_norm1(W2, n);
    }
    oracle_select_from_norms(n1, n2 < 0.0 ? 0.0 : n2, eps, m, s);
    *near = 0;
    if (n1 != 0.0) {
        for (int c = 0; c < 4; ++c) {
            const double f1 = (c & 1) ? 1.0 + 1e-6 : 1.0 - 1e-6;
            const double f2 = (c & 2) ? 1.0 + 1e-6 : 1.0 - 1e-6;
            int mc, sc;
            oracle_select_from_norms(n1 * f1, (n2 < 0.0 ? 0.0 : n2) * f2, eps, &mc, &sc);
            if (mc != *m || sc != *s)
                *near = 1;
        }
    }
    *n1_out = n1;
    *n2_out = n2;
}

int oracle_select(const double *W, int n, double eps, int *m, int *s,
                  double *n1, double *n2, int *near)
{
    double *W2 = (double *)malloc(sizeof(double) * (size_t)n * n + 8);
    if (!W2)
        return -3;
    select_matrix(W, n, eps, W2, 0, m, s, n1, n2, near);
    free(W2);
    return 0;
}

/* Threads the OpenMP runtime offered when the library was first asked: a batch call with an explicit thread count
 * changes the runtime's own default, so "all threads" must not be read back from it afterwards. */
static int all_threads(void)
{
#ifdef _OPENMP
    static int offered = 0;
    if (offered <= 0)
        offered = omp_get_max_threads();
    return offered;
#else
    return 1;
#endif
}

/*
 * Evaluation half of Algorithm 2 with the order and the scaling given: A = W/2^s,
 * X = sum_{k=0..m} A^k/k! by direct summation (term_k = term_{k-1} * A / k), plus
 * b16 * A^16 when `plus16` is set (the 15+ approximant, Sec. 3.1: y22 = T15 + b16 A^16),
 * then s squarings.  `work` holds 3*n*n doubles.
 */
static void taylor_then_square(const double *W, int n, int m, int s, int plus16, double *X, double *work, int par)
{
    const size_t nn = (size_t)n * n;
    double *A = work, *term = work + nn, *next = work + 2 * nn;

    const double scale = ldexp(1.0, -s); /* exact power of two */
    for (size_t t = 0; t < nn; ++t)
        A[t] = W[t] * scale;

    /* X = I, term = I */
    memset(X, 0, sizeof(double) * nn);
    memset(term, 0, sizeof(double) * nn);
    for (int i = 0; i < n; ++i) {
        X[(size_t)i * n + i] = 1.0;
        term[(size_t)i * n + i] = 1.0;
    }
    /* term_k = term_{k-1} * A / k = A^k / k!,  X += term_k  for k = 1..m */
    for (int k = 1; k <= m; ++k) {
        if (k == 1) {
            memcpy(term, A, sizeof(double) * nn);
        } else {
            matmul_impl(term, A, next, n, par);
            const double inv = (double)k;
            for (size_t t = 0; t < nn; ++t)
                term[t] = next[t] / inv;
        }
        for (size_t t = 0; t < nn; ++t)
            X[t] += term[t];
    }
    if (plus16) {
        /* 15+ : add b16 * A^16 = (b16 * 16!) * (A^16/16!); term holds A^15/15! here */
        matmul_impl(term, A, next, n, par);
        const double w = oracle_b16() * factorial(16);
        for (size_t t = 0; t < nn; ++t)
            X[t] += w * (next[t] / 16.0);
    }
    /* squaring phase */
    for (int q = 0; q < s; ++q) {
        matmul_impl(X, X, next, n, par);
        memcpy(X, next, sizeof(double) * nn);
    }
}

/*
 * Algorithm 2 for one matrix: select (m,s), A = W/2^s, X = polynomial by
 * direct summation, s squarings.  `work` holds 4*n*n doubles.
 */
static void expm_matrix(const double *W, int n, double eps, double *X, double *work, int par,
                        int *m_out, int *s_out, double *n1, double *n2, int *near)
{
    const size_t nn = (size_t)n * n;
    int m, s;
    select_matrix(W, n, eps, work + 3 * nn, par, &m, &s, n1, n2, near);
    *m_out = m;
    *s_out = s;
    taylor_then_square(W, n, m, s, m == 15, X, work, par);
}

/*
 * The same evaluation with (m, s) handed in instead of selected: what Algorithm 2 computes once
 * Algorithm 3 or 4 has returned this pair.  Used by the parity tests for matrices whose norms sit
 * within 1e-6 of a switch point, where the device may rightly take the neighbouring choice.
 * plus16 != 0 adds the b16 A^16 term of the 15+ approximant (only meaningful with m == 15).
 * threads <= 0: all; the rows of every product are spread over the threads when n >= 256.
 */
int oracle_expm_forced(const double *W, int n, int m, int s, int plus16, double *X, int threads)
{
    if (m < 0 || s < 0 || (plus16 && m != 15))
        return -1;
    double *work = (double *)malloc(sizeof(double) * 3 * (size_t)n * n + 8);
    if (!work)
        return -3;
#ifdef _OPENMP
    omp_set_num_threads(threads <= 0 ? all_threads() : threads);
#else
    (void)threads;
#endif
    taylor_then_square(W, n, m, s, plus16, X, work, n >= 256);
    free(work);
    return 0;
}

int oracle_expm(const double *W, int n, double eps, double *X, int *m, int *s,
                double *n1, double *n2, int *near)
{
    double *work = (double *)malloc(sizeof(double) * 4 * (size_t)n * n + 8);
    if (!work)
        return -3;
    expm_matrix(W, n, eps, X, work, 0, m, s, n1, n2, near);
    free(work);
    return 0;
}

/*
 * Batch driver, also the timed CPU baseline.  threads <= 0 means "all the
 * OpenMP runtime offers".  Matrices of order < 256 are spread over threads
 * one matrix each; larger ones run one after another with the rows of every
 * product spread over the threads.  Returns the thread count used, or a
 * negative value on allocation failure.
 */
int oracle_expm_batch(const double *W, int n, int batch, double eps, double *X,
                      int *m, int *s, double *n1, double *n2, int *near, int threads)
{
    const size_t nn = (size_t)n * n;
    int used = 1;
#ifdef _OPENMP
    if (threads <= 0)
        threads = all_threads();
    used = threads;
    omp_set_num_threads(threads);
#else
    (void)threads;
#endif
    int fail = 0;
    if (n < 256) {
#pragma omp parallel
        {
            double *work = (double *)malloc(sizeof(double) * 4 * nn + 8);
            if (!work) {
#pragma omp atomic write
                fail = 1;
            }
#pragma omp for schedule(dynamic, 1)
            for (int b = 0; b < batch; ++b) {
                if (work)
                    expm_matrix(W + (size_t)b * nn, n, eps, X + (size_t)b * nn, work, 0,
                                &m[b], &s[b], &n1[b], &n2[b], &near[b]);
            }
            free(work);
        }
    } else {
        double *work = (double *)malloc(sizeof(double) * 4 * nn + 8);
        if (!work)
            return -3;
        for (int b = 0; b < batch; ++b)
            expm_matrix(W + (size_t)b * nn, n, eps, X + (size_t)b * nn, work, 1,
                        &m[b], &s[b], &n1[b], &n2[b], &near[b]);
        free(work);
    }
    return fail ? -3 : used;
}

/* ------------------------------------------------------------------------------------------
 * Paterson-Stockmeyer variant (Algorithm 3 of Sec. 3.3 with Algorithm 2): orders
 * M = [1,2,4,6,9,12,16], powers W^j, j = ceil(sqrt(m)) in {1,2,2,3,3,4,4}, k = m/j.
 * Bounds from the table after Algorithm 3:
 *   m=1      : E1 = n1^2/2!,              E2 = n1^3/3!
 *   m=j*k>1  : E1 = nj^k * n1 / (m+1)!,   E2 = nj^k * n2 / (m+2)!,   nj = ||W^j||_1
 * First order with E1+E2 <= eps wins with s = 0; otherwise m = 16 and
 * s = max_i ceil(log2(E_i/eps)/(16+i)), i = 1,2, capped at 20.
 * The polynomial is the plain Taylor polynomial T_m (direct summation here; how it is
 * evaluated -- Paterson-Stockmeyer -- is the GPU side's business).
 * ------------------------------------------------------------------------------------------ */
void oracle_select_ps_from_norms(double n1, double n2, double n3, double n4, double eps, int *m_out, int *s_out)
{
    static const int M[7] = {1, 2, 4, 6, 9, 12, 16};
    static const int J[7] = {1, 2, 2, 3, 3, 4, 4};
    int m = 0, s = 0, found = 0;
    double E1 = 0.0, E2 = 0.0;
    if (n1 == 0.0) {
        *m_out = 0;
        *s_out = 0;
        return;
    }
    const double nj[5] = {0.0, n1, n2, n3, n4};
    for (int i = 0; i < 7 && !found; ++i) {
        m = M[i];
        const int j = J[i], k = m / j;
        if (m == 1) {
            E1 = n1 * n1 / factorial(2);
            E2 = n1 * n1 * n1 / factorial(3);
        } else {
            const double pk = ipow(nj[j], k);
            E1 = pk * n1 / factorial(m + 1);
            E2 = pk * n2 / factorial(m + 2);
        }
        if (E1 + E2 <= eps)
            found = 1;
    }
    if (!found) {
        const double E[2] = {E1, E2};
        for (int i = 1; i <= 2; ++i) {
            int s1;
            if (!isfinite(E[i - 1])) {
                s1 = ORACLE_S_CAP;
            } else if (E[i - 1] <= 0.0) {
                s1 = 0;
            } else {
                const double q = ceil(log2(E[i - 1] / eps) / (double)(m + i));
                s1 = (q > (double)ORACLE_S_CAP) ? ORACLE_S_CAP : (q < 0.0 ? 0 : (int)q);
            }
            if (s1 > s)
                s = s1;
        }
    }
    if (s > ORACLE_S_CAP)
        s = ORACLE_S_CAP;
    *m_out = m;
    *s_out = s;
}

/* Norms of W, W^2, W^3 = W^2*W, W^4 = W^3*W (powers by repeated multiplication, as in Algorithm 3),
 * the choice, and the near flag over the 16 corners of the four norms.  work: 3*n*n doubles. */
static void select_ps_matrix(const double *W, int n, double eps, double *work, int par,
                             int *m, int *s, double norms[4], int *near)
{
    const size_t nn = (size_t)n * n;
    double *W2 = work, *W3 = work + nn, *W4 = work + 2 * nn;
    norms[0] = oracle_norm1(W, n);
    norms[1] = norms[2] = norms[3] = 0.0;
    *near = 0;
    if (norms[0] == 0.0) {
        *m = 0;
        *s = 0;
        return;
    }
    const double hi = norms[0] * (1.0 + 1e-6);
    if (!(hi * hi / 2.0 + hi * hi * hi / 6.0 <= eps)) {
        matmul_impl(W, W, W2, n, par);
        matmul_impl(W2, W, W3, n, par);
        matmul_impl(W3, W, W4, n, par);
        norms[1] = oracle_norm1(W2, n);
        norms[2] = oracle_norm1(W3, n);
        norms[3] = oracle_norm1(W4, n);
    }
    oracle_select_ps_from_norms(norms[0], norms[1], norms[2], norms[3], eps, m, s);
    for (int c = 0; c < 16; ++c) {
        double f[4];
        for (int t = 0; t < 4; ++t)
            f[t] = (c >> t) & 1 ? 1.0 + 1e-6 : 1.0 - 1e-6;
        int mc, sc;
        oracle_select_ps_from_norms(norms[0] * f[0], norms[1] * f[1], norms[2] * f[2], norms[3] * f[3], eps, &mc, &sc);
        if (mc != *m || sc != *s)
            *near = 1;
    }
}

int oracle_select_ps(const double *W, int n, double eps, int *m, int *s, double *norms4, int *near)
{
    double *work = (double *)malloc(sizeof(double) * 3 * (size_t)n * n + 8);
    if (!work)
        return -3;
    select_ps_matrix(W, n, eps, work, 0, m, s, norms4, near);
    free(work);
    return 0;
}

/* Algorithm 2 with Algorithm 3: X = T_m(W/2^s) by direct summation, s squarings.  work: 6*n*n doubles. */
static void expm_ps_matrix(const double *W, int n, double eps, double *X, double *work, int par,
                           int *m_out, int *s_out, double norms[4], int *near)
{
    const size_t nn = (size_t)n * n;
    int m, s;
    select_ps_matrix(W, n, eps, work + 3 * nn, par, &m, &s, norms, near);
    *m_out = m;
    *s_out = s;
    taylor_then_square(W, n, m, s, 0, X, work, par);
}

/* Batch driver of the Paterson-Stockmeyer variant; norms is [batch][4]. */
int oracle_expm_ps_batch(const double *W, int n, int batch, double eps, double *X,
                         int *m, int *s, double *norms, int *near, int threads)
{
    const size_t nn = (size_t)n * n;
    int used = 1;
#ifdef _OPENMP
    if (threads <= 0)
        threads = all_threads();
    used = threads;
    omp_set_num_threads(threads);
#else
    (void)threads;
#endif
    int fail = 0;
    if (n < 256) {
#pragma omp parallel
        {
            double *work = (double *)malloc(sizeof(double) * 6 * nn + 8);
            if (!work) {
#pragma omp atomic write
                fail = 1;
            }
#pragma omp for schedule(dynamic, 1)
            for (int b = 0; b < batch; ++b) {
                if (work)
                    expm_ps_matrix(W + (size_t)b * nn, n, eps, X + (size_t)b * nn, work, 0,
                                   &m[b], &s[b], norms + 4 * (size_t)b, &near[b]);
            }
            free(work);
        }
    } else {
        double *work = (double *)malloc(sizeof(double) * 6 * nn + 8);
        if (!work)
            return -3;
        for (int b = 0; b < batch; ++b)
            expm_ps_matrix(W + (size_t)b * nn, n, eps, X + (size_t)b * nn, work, 1,
                           &m[b], &s[b], norms + 4 * (size_t)b, &near[b]);
        free(work);
    }
    return fail ? -3 : used;
}

/* ------------------------------------------------------------------------------------------
 * Baseline of the paper's comparison (its Algorithm 1, Sec. 2.2, after Xiao & Liu): smallest
 * s >= 0 with ||W||_1 / 2^s < 1/2; W <- W/2^s; X = I, Y = W, k = 2; while ||Y||_1 > eps:
 * X += Y, Y = W*Y/k, k++; then s squarings of X (the printed listing squares and returns Y,
 * which is a slip: Sec. 2.2 describes squaring the computed exponential).
 * m_out = number of terms added (the degree reached); the paper prices this at (m-1)+s products.
 * near = 1 if ||W||/2^s lies within 1e-6 relative of 1/2 or some ||Y|| within 1e-6 relative of eps.
 * work: 3*n*n doubles.
 * ------------------------------------------------------------------------------------------ */
static void expm_baseline_matrix(const double *W, int n, double eps, double *X, double *work,
                                 int *m_out, int *s_out, double *n1_out, int *near)
{
    const size_t nn = (size_t)n * n;
    double *A = work, *Y = work + nn, *next = work + 2 * nn;
    const double n1 = oracle_norm1(W, n);
    int s = 0, m = 0;
    *near = 0;
    *n1_out = n1;
    memset(X, 0, sizeof(double) * nn);
    for (int i = 0; i < n; ++i)
        X[(size_t)i * n + i] = 1.0;
    if (n1 == 0.0) {
        *m_out = 0;
        *s_out = 0;
        return;
    }
    while (!(ldexp(n1, -s) < 0.5))
        ++s;
    {
        const double r = ldexp(n1, -s) / 0.5, r2 = ldexp(n1, -s + 1) / 0.5;
        if (fabs(r - 1.0) < 1e-6 || (s > 0 && fabs(r2 - 1.0) < 1e-6))
            *near = 1;
    }
    const double scale = ldexp(1.0, -s);
    for (size_t t = 0; t < nn; ++t) {
        A[t] = W[t] * scale;
        Y[t] = A[t];
    }
    int k = 2;
    for (;;) {
        const double ny = oracle_norm1(Y, n);
        if (fabs(ny / eps - 1.0) < 1e-6)
            *near = 1;
        if (!(ny > eps))
            break;
        for (size_t t = 0; t < nn; ++t)
            X[t] += Y[t];
        ++m;
        matmul_impl(A, Y, next, n, 0);
        for (size_t t = 0; t < nn; ++t)
            Y[t] = next[t] / (double)k;
        ++k;
    }
    for (int q = 0; q < s; ++q) {
        matmul_impl(X, X, next, n, 0);
        memcpy(X, next, sizeof(double) * nn);
    }
    *m_out = m;
    *s_out = s;
}

int oracle_expm_baseline_batch(const double *W, int n, int batch, double eps, double *X,
                               int *m, int *s, double *n1, int *near, int threads)
{
    const size_t nn = (size_t)n * n;
    int used = 1;
#ifdef _OPENMP
    if (threads <= 0)
        threads = all_threads();
    used = threads;
    omp_set_num_threads(threads);
#else
    (void)threads;
#endif
    int fail = 0;
#pragma omp parallel
    {
        double *work = (double *)malloc(sizeof(double) * 3 * nn + 8);
        if (!work) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (int b = 0; b < batch; ++b) {
            if (work)
                expm_baseline_matrix(W + (size_t)b * nn, n, eps, X + (size_t)b * nn, work,
                                     &m[b], &s[b], &n1[b], &near[b]);
        }
        free(work);
    }
    return fail ? -3 : used;
}

/* ----------------------------------------------------------------------------------------------
 * Low-rank parameterisation W = A1 A2 (Sec. 2.2, the equation for e^W in terms of V = A2 A1):
 *     e^W ~ I + A1 ( sum_{i=0..m} V^i / (i+1)! ) A2,   A1: n x t, A2: t x n, V: t x t, no scaling (s = 0).
 * Order: the Paterson-Stockmeyer orders 1,2,4,6,9,12,16, the smallest whose truncation bound
 *     ||V||^(m+1) / (m+2)! / (1 - ||V|| / (m+3))          (the bound printed after that equation; Theorem 3 with p = 1)
 * is at most eps (it needs ||V|| < m+3).  ||V|| = 0 gives m = 0 (the sum is I and the result I + A1 A2 is exact);
 * if no order reaches eps the largest one is used and flag 2 says that the tolerance is not guaranteed
 * (this variant does not scale).  m = -1 for a non-finite norm.
 * ------------------------------------------------------------------------------------------ */
static double lowrank_bound(double v, int m)
{
    if (!(v < (double)(m + 3)))
        return INFINITY;
    return ipow(v, m + 1) / factorial(m + 2) / (1.0 - v / (double)(m + 3));
}

void oracle_lowrank_select_from_norm(double v1, double eps, int *m_out, int *flag_out)
{
    static const int M[7] = {1, 2, 4, 6, 9, 12, 16};
    *flag_out = 0;
    if (!(v1 <= DBL_MAX)) {
        *m_out = -1;
        *flag_out = 1;
        return;
    }
    if (v1 == 0.0) {
        *m_out = 0;
        return;
    }
    for (int i = 0; i < 7; ++i)
        if (lowrank_bound(v1, M[i]) <= eps) {
            *m_out = M[i];
            return;
        }
    *m_out = 16;
    *flag_out = 2;
}

/* plain rectangular product C (p x r) = A (p x q) * B (q x r), row-major, i-k-j loop order */
static void matmul_rect(const double *A, const double *B, double *C, int p, int q, int r)
{
    for (int i = 0; i < p; ++i) {
        double *c = C + (size_t)i * r;
        for (int j = 0; j < r; ++j)
            c[j] = 0.0;
        for (int k = 0; k < q; ++k) {
            const double a = A[(size_t)i * q + k];
            const double *b = B + (size_t)k * r;
            for (int j = 0; j < r; ++j)
                c[j] += a * b[j];
        }
    }
}

/* X = I + A1 (sum_{i=0..m} V^i/(i+1)!) A2 for a given order m >= 0; V = A2 A1 (t x t) is handed in.
 * work: 2*t*t + max(t*n, t*t) doubles. */
static void lowrank_eval(const double *A1, const double *A2, const double *V, int n, int t, int m, double *X, double *work)
{
    const size_t tt = (size_t)t * t;
    double *Phi = work, *term = work + tt, *PA2 = work + 2 * tt; /* PA2: t x n */
    /* Phi = sum_{i=0..m} V^i / (i+1)!, term by term: term_0 = I, term_i = term_{i-1} V / (i+1) */
    memset(Phi, 0, sizeof(double) * tt);
    memset(term, 0, sizeof(double) * tt);
    for (int i = 0; i < t; ++i) {
        Phi[(size_t)i * t + i] = 1.0;
        term[(size_t)i * t + i] = 1.0;
    }
    for (int i = 1; i <= m; ++i) {
        double *next = PA2; /* the last scratch area holds at least t*t doubles */
        matmul_rect(term, V, next, t, t, t);
        for (size_t e = 0; e < tt; ++e) {
            term[e] = next[e] / (double)(i + 1);
            Phi[e] += term[e];
        }
    }
    matmul_rect(Phi, A2, PA2, t, t, n);
    matmul_rect(A1, PA2, X, n, t, n);
    for (int i = 0; i < n; ++i)
        X[(size_t)i * n + i] += 1.0;
}

/* One pair (A1, A2).  work: 3*t*t + max(t*n, t*t) doubles.  X: n x n. */
static void lowrank_matrix(const double *A1, const double *A2, int n, int t, double eps, double *X, double *work,
                           int *m_out, int *flag_out, double *v1_out, int *near)
{
    const size_t tt = (size_t)t * t;
    double *V = work;
    matmul_rect(A2, A1, V, t, n, t);
    const double v1 = oracle_norm1(V, t);
    int m, flag;
    oracle_lowrank_select_from_norm(v1, eps, &m, &flag);
    *v1_out = v1;
    *m_out = m;
    *flag_out = flag;
    *near = 0;
    if (m >= 0) {
        int ma, mb, fa, fb;
        oracle_lowrank_select_from_norm(v1 * (1.0 - 1e-6), eps, &ma, &fa);
        oracle_lowrank_select_from_norm(v1 * (1.0 + 1e-6), eps, &mb, &fb);
        if (ma != m || mb != m)
            *near = 1;
    }
    if (m < 0) {
        for (size_t e = 0; e < (size_t)n * n; ++e)
            X[e] = NAN;
        return;
    }
    lowrank_eval(A1, A2, V, n, t, m, X, work + tt);
}

/* The same with the order handed in (for pairs whose ||V|| sits within 1e-6 of a switch point). */
int oracle_lowrank_forced(const double *A1, const double *A2, int n, int t, int m, double *X)
{
    if (m < 0)
        return -1;
    const size_t tt = (size_t)t * t, tn = (size_t)t * n;
    double *work = (double *)malloc(sizeof(double) * (3 * tt + (tn > tt ? tn : tt)) + 8);
    if (!work)
        return -3;
    matmul_rect(A2, A1, work, t, n, t);
    lowrank_eval(A1, A2, work, n, t, m, X, work + tt);
    free(work);
    return 0;
}

/* Batch: A1 [batch][n][t], A2 [batch][t][n], X [batch][n][n]; returns threads used or -3. */
int oracle_lowrank_batch(const double *A1, const double *A2, int n, int t, int batch, double eps, double *X,
                         int *m, int *flag, double *v1, int *near, int threads)
{
    int used = 1;
#ifdef _OPENMP
    if (threads <= 0)
        threads = all_threads();
    used = threads;
    omp_set_num_threads(threads);
#else
    (void)threads;
#endif
    int fail = 0;
    const size_t tt = (size_t)t * t, tn = (size_t)t * n;
#pragma omp parallel
    {
        double *work = (double *)malloc(sizeof(double) * (3 * tt + (tn > tt ? tn : tt)) + 8);
        if (!work) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (int b = 0; b < batch; ++b) {
            if (work)
                lowrank_matrix(A1 + (size_t)b * n * t, A2 + (size_t)b * tn, n, t, eps, X + (size_t)b * n * n, work,
                               &m[b], &flag[b], &v1[b], &near[b]);
        }
        free(work);
    }
    return fail ? -3 : used;
}

int oracle_max_threads(void)
{
    return all_threads();
}

/* One product with its rows spread over the threads, exactly as the batch drivers run products of matrices of
 * order >= 256 (same loop, same summation order per element).  Exported so that the benchmark can time a single
 * product at a size whose whole exponential takes many minutes.  Returns the thread count used. */
int oracle_matmul_threads(const double *A, const double *B, double *C, int n, int threads)
{
    int used = 1;
#ifdef _OPENMP
    if (threads <= 0)
        threads = all_threads();
    used = threads;
    omp_set_num_threads(threads);
#else
    (void)threads;
#endif
    matmul_impl(A, B, C, n, 1);
    return used;
}
