// Internal declarations shared by the HIP translation units of the gfx950 expm library.
// Not part of the public interface (that is include/expm_mi355x.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace expmk {

// ---------------------------------------------------------------------------------------------
// Coefficients of the evaluation formulas (Sec. 3.1 of arXiv 2512.20777, the two coefficient
// tables), as printed, in double.  The fp32 path rounds each (scaled) coefficient to float.
// ---------------------------------------------------------------------------------------------
// order 8:  y02 = A2 (c1 A2 + c2 A);  T8 = (y02 + c3 A2 + c4 A)(y02 + c5 A2) + c6 y02 + A2/2 + A + I
#define EXPM_T8_C1 4.980119205559973e-3
#define EXPM_T8_C2 1.992047682223989e-2
#define EXPM_T8_C3 7.665265321119147e-2
#define EXPM_T8_C4 8.765009801785554e-1
#define EXPM_T8_C5 1.225521150112075e-1
#define EXPM_T8_C6 2.974307204847627e0
// order 15+:  y02 = A2 (c1 A2 + c2 A)
//             y12 = (y02 + c3 A2 + c4 A)(y02 + c5 A2) + c6 y02 + c7 A2
//             y22 = (y12 + c8 A2 + c9 A)(y12 + c10 y02 + c11 A) + c12 y12 + c13 y02 + c14 A2 + c15 A + c16 I
#define EXPM_T15_C1 4.018761610201036e-4
#define EXPM_T15_C2 2.945531440279683e-3
#define EXPM_T15_C3 -8.709066576837676e-3
#define EXPM_T15_C4 4.017568440673568e-1
#define EXPM_T15_C5 3.230762888122312e-2
#define EXPM_T15_C6 5.768988513026145e0
#define EXPM_T15_C7 2.338576034271299e-2
#define EXPM_T15_C8 2.381070373870987e-1
#define EXPM_T15_C9 2.224209172496374e0
#define EXPM_T15_C10 -5.792361707073261e0
#define EXPM_T15_C11 -4.130276365929783e-2
#define EXPM_T15_C12 1.040801735231354e1
#define EXPM_T15_C13 -6.331712455883370e1
#define EXPM_T15_C14 3.484665863364574e-1
#define EXPM_T15_C15 1.0
#define EXPM_T15_C16 1.0

constexpr int kSCap = 20;          // cap on s (Algorithm 4, last lines)
constexpr int kMaxRounds = 3 + kSCap;  // product rounds after the W^2 round: 3 for 15+, one per squaring

// Per-matrix record produced by the selection stage.
struct MatInfo {
    int m;      // 0,1,2,4,8,15 ; -1 = non-finite input
    int s;      // 0..20        ; -1 = non-finite input
    int len;    // product rounds still to run after the W^2 round
    int flags;  // bit0 non-finite, bit1 s hit the cap
};

// Scaling that one error term asks for (last steps of Algorithms 3 and 4): the smallest s >= 0 with
// e / 2^(w s) <= eps, i.e. ceil(log2(e / eps) / w), or cap + 1 if that exceeds the cap (or e is not finite): the
// caller clips to the cap and flags the matrix.  Found from the binary exponents of e and eps and one exact
// comparison against eps * 2^(w s) instead of a division and a logarithm: with e = fe 2^xe and eps = fp 2^xp
// (fe, fp in [1/2, 1)) the ratio lies in (2^(d-1), 2^(d+1)), d = xe - xp, so s is floor((d-1)/w) + 1 or one more.
__host__ __device__ inline int scaling_for_term(double e, double eps, int w)
{
    if (!(e <= 1.7976931348623157e308)) return kSCap + 1;
    if (e <= eps) return 0;  // also e <= 0
    int xe, xp;
    (void)frexp(e, &xe);
    (void)frexp(eps, &xp);
    const int d = xe - xp;  // >= 0 here
    int s1 = d >= 1 ? (d - 1) / w + 1 : 0;
    if (s1 > kSCap) return kSCap + 1;
    if (e > ldexp(eps, w * s1)) ++s1;
    return s1 > kSCap ? kSCap + 1 : s1;
}

// ---------------------------------------------------------------------------------------------
// Algorithm 4 (Sec. 3.3) on the two norms n1 = ||W||_1, n2 = ||W^2||_1, tolerance eps.
// Bounds per order from the table that follows Algorithm 4.  All in double.
// ---------------------------------------------------------------------------------------------
__host__ __device__ inline void select_order_scaling(double n1, double n2, double eps, int &m, int &s, int &flags)
{
    flags = 0;
    if (!(n1 == n1) || !(n2 == n2) || n1 > 1.7976931348623157e308 || n2 > 1.7976931348623157e308) {
        m = -1; s = -1; flags = 1;
        return;
    }
    m = 0; s = 0;
    if (n1 == 0.0) return;
    // 1/(m+1)!, 1/(m+2)! for m = 1, 2, 4, 8 ; for 15+: |1/16! - b16|, 1/17!
    const double inv2 = 0.5, inv6 = 1.0 / 6.0, inv24 = 1.0 / 24.0, inv120 = 1.0 / 120.0, inv720 = 1.0 / 720.0;
    const double inv9f = 1.0 / 362880.0, inv10f = 1.0 / 3628800.0;
    const double c1 = EXPM_T15_C1;
    const double b16 = (c1 * c1) * (c1 * c1);
    const double inv16f = 1.0 / 20922789888000.0, inv17f = 1.0 / 355687428096000.0;
    double e1, e2;
    m = 1;
    e1 = inv2 * n1 * n1;
    e2 = inv6 * n1 * n1 * n1;
    if (e1 + e2 <= eps) return;
    m = 2;
    e1 = inv6 * n2 * n1;
    e2 = inv24 * n2 * n2;
    if (e1 + e2 <= eps) return;
    m = 4;
    const double p2 = n2 * n2;
    e1 = inv120 * p2 * n1;
    e2 = inv720 * p2 * n2;
    if (e1 + e2 <= eps) return;
    m = 8;
    const double p4 = p2 * p2;
    e1 = inv9f * p4 * n1;
    e2 = inv10f * p4 * n2;
    if (e1 + e2 <= eps) return;
    m = 15;
    const double p8 = p4 * p4;
    const double d16 = inv16f > b16 ? inv16f - b16 : b16 - inv16f;
    e1 = d16 * p8;
    e2 = inv17f * p8 * n1;
    if (e1 + e2 <= eps) return;
    // scaling from each of the two terms alone, the larger wins (Sec. 3.2, last paragraph)
    const int sa = scaling_for_term(e1, eps, 16), sb = scaling_for_term(e2, eps, 17);
    s = sa > sb ? sa : sb;
    if (s > kSCap) { s = kSCap; flags |= 2; }  // Algorithm clips only when more than the cap is asked for
}

// Rounds after the W^2 product: T4 needs 1 more product, T8 2, 15+ 3, plus one per squaring.
__host__ __device__ inline int chain_length(int m, int s)
{
    if (m == 4) return 1;
    if (m == 8) return 2;
    if (m == 15) return 3 + s;
    return 0;
}

// ---------------------------------------------------------------------------------------------
// Paterson-Stockmeyer variant (Algorithm 3, Sec. 3.3): orders M = [1,2,4,6,9,12,16], powers W^j with
// j = ceil(sqrt(m)), k = m/j; bounds of the table after Algorithm 3:
//   m = 1: E1 = n1^2/2!, E2 = n1^3/3! ;  m = j*k > 1: E1 = nj^k n1/(m+1)!, E2 = nj^k n2/(m+2)!.
// nrm[r-1] = ||W^r||_1 for r = 1..avail.  Orders that need a power above `avail` are not looked at:
// if none of the orders that can be judged is accepted, need_more is set and (m, s) are not final.
// ---------------------------------------------------------------------------------------------
__host__ __device__ inline int ps_j(int m) { return m <= 1 ? 1 : (m <= 4 ? 2 : (m <= 9 ? 3 : 4)); }
__host__ __device__ inline int ps_k(int m) { return m <= 0 ? 1 : m / ps_j(m); }

__host__ __device__ inline void select_ps_order_scaling(const double nrm[4], int avail, double eps, int &m, int &s,
                                                        int &flags, bool &need_more)
{
    flags = 0;
    need_more = false;
    for (int r = 0; r < avail; ++r)
        if (!(nrm[r] <= 1.7976931348623157e308)) {  // NaN or Inf
            m = -1; s = -1; flags = 1;
            return;
        }
    m = 0; s = 0;
    const double n1 = nrm[0];
    if (n1 == 0.0) return;
    // 1/(m+1)! and 1/(m+2)! for m = 1,2,4,6,9,12,16
    const double c1[7] = {1.0 / 2.0, 1.0 / 6.0, 1.0 / 120.0, 1.0 / 5040.0, 1.0 / 3628800.0, 1.0 / 6227020800.0,
                          1.0 / 355687428096000.0};
    const double c2[7] = {1.0 / 6.0, 1.0 / 24.0, 1.0 / 720.0, 1.0 / 40320.0, 1.0 / 39916800.0, 1.0 / 87178291200.0,
                          1.0 / 6402373705728000.0};
    const int M[7] = {1, 2, 4, 6, 9, 12, 16};
    double e1 = 0.0, e2 = 0.0;
    for (int i = 0; i < 7; ++i) {
        m = M[i];
        const int j = ps_j(m), k = m / j;
        if (j > avail) { need_more = true; return; }
        if (m == 1) {
            e1 = c1[0] * n1 * n1;
            e2 = c2[0] * n1 * n1 * n1;
        } else {
            double pk = 1.0;
            for (int q = 0; q < k; ++q) pk *= nrm[j - 1];
            e1 = c1[i] * pk * n1;
            e2 = c2[i] * pk * nrm[1];
        }
        if (e1 + e2 <= eps) return;
    }
    const int sa = scaling_for_term(e1, eps, 17), sb = scaling_for_term(e2, eps, 18);
    s = sa > sb ? sa : sb;
    if (s > kSCap) { s = kSCap; flags |= 2; }  // Algorithm clips only when more than the cap is asked for
}

// Products after the powers: k-1 Horner steps, plus one per squaring.
__host__ __device__ inline int chain_length_ps(int m, int s)
{
    if (m < 4) return 0;
    return ps_k(m) - 1 + s;
}

// 1/i!, i = 0..18 (i! is exact in double up to 18!, so this is the correctly rounded reciprocal)
__host__ __device__ inline double inv_factorial(int i)
{
    double f = 1.0;
    for (int q = 2; q <= i; ++q) f *= (double)q;
    return 1.0 / f;
}

// ---------------------------------------------------------------------------------------------
// Low-rank variant (Sec. 2.2): e^(A1 A2) = I + A1 (sum_{i<=m} V^i/(i+1)!) A2 with V = A2 A1 and no scaling.
// Order from v1 = ||V||_1: the smallest of the Paterson-Stockmeyer orders whose truncation bound
// v1^(m+1)/(m+2)!/(1 - v1/(m+3)) (printed after that equation; Theorem 3 with p = 1) is at most eps.
// v1 = 0: m = 0 (the sum is I, the result exact).  No order reaches eps: the largest, flag bit 1.
// ---------------------------------------------------------------------------------------------
__host__ __device__ inline void select_lowrank_order(double v1, double eps, int &m, int &flags)
{
    flags = 0;
    if (!(v1 <= 1.7976931348623157e308)) {
        m = -1; flags = 1;
        return;
    }
    m = 0;
    if (v1 == 0.0) return;
    const int M[7] = {1, 2, 4, 6, 9, 12, 16};
    for (int i = 0; i < 7; ++i) {
        m = M[i];
        if (v1 < (double)(m + 3)) {
            double pw = 1.0;
            for (int q = 0; q <= m; ++q) pw *= v1;
            if (pw * inv_factorial(m + 2) / (1.0 - v1 / (double)(m + 3)) <= eps) return;
        }
    }
    m = 16;
    flags |= 2;
}

// ---------------------------------------------------------------------------------------------
// MFMA wrappers.  Both dtypes use the 16x16x4 shape.  Operand layouts coincide:
//   A operand: lane l holds A[i = l%16][k = l/16]
//   B operand: lane l holds B[k = l/16][j = l%16]
// The result layouts differ in the row index (checked on the device with a probe):
//   f32: lane l, register v (0..3) holds C[i = 4*(l/16) + v][j = l%16]
//   f64: lane l, register v (0..3) holds C[i = 4*v + l/16][j = l%16]
// ---------------------------------------------------------------------------------------------
typedef double v4d __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));

template <typename T> struct Mfma;
template <> struct Mfma<double> {
    using acc_t = v4d;
    static __device__ __forceinline__ acc_t run(double a, double b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
    }
    // row inside the 16x16 tile held by register v of a lane in 16-lane group g
    static __device__ __forceinline__ int row(int g, int v) { return 4 * v + g; }
};
template <> struct Mfma<float> {
    using acc_t = v4f;
    static __device__ __forceinline__ acc_t run(float a, float b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int row(int g, int v) { return 4 * g + v; }
};

// ---------------------------------------------------------------------------------------------
// Buffers of the round-based (larger n) path, one [batch][n][n] array each.
// ---------------------------------------------------------------------------------------------
constexpr int kSchemeSastre = 0;  // evaluation formulas of Sec. 3.1 with Algorithm 4
constexpr int kSchemePS = 1;      // Paterson-Stockmeyer with Algorithm 3
constexpr int kSchemeBaseline = 2;  // the paper's comparison baseline (its Algorithm 1)
constexpr int kSchemePhi = 3;       // core series of the low-rank variant, sum_i V^i/(i+1)!, no scaling

enum Buf : int { BUF_W = 0, BUF_W2 = 1, BUF_T0 = 2, BUF_T1 = 3, BUF_T2 = 4, BUF_T3 = 5, BUF_T4 = 6, BUF_T5 = 7,
                 BUF_OUT = 8, BUF_COUNT = 9,
                 BUF_W3 = BUF_T3, BUF_W4 = BUF_T4 };  // the Paterson-Stockmeyer variant keeps W^3, W^4 there

// One product round for one matrix:
//   t      = acc_scale * (L*R) + sum_i g[i] * S_i
//   out_j  = a[j] * t + sum_i b[j][i] * S_i + d[j] * I
// S_i are up to four source matrices read element-wise, out_j up to four outputs.
template <typename T> struct Step {
    int L, R;
    T acc_scale;
    int nsrc;
    int src[4];
    T g[4];
    int nout;
    int dst[4];
    T a[4];
    T b[4][4];
    T d[4];
};

// Build the round `r` (1-based, after the W^2 round) of the chain for order m and scaling s.
// With sigma = 2^-s:  A = sigma W, A2 = sigma^2 W2.  The power-of-two factors are folded into
// the coefficients (exact), so W and W2 are never rescaled in memory.
template <typename T>
__device__ __forceinline__ Step<T> build_step(int m, int s, int r)
{
    Step<T> st;
    st.L = BUF_T0; st.R = BUF_T1; st.acc_scale = (T)1; st.nsrc = 0; st.nout = 1;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        st.src[i] = BUF_W; st.g[i] = (T)0; st.dst[i] = BUF_OUT; st.a[i] = (T)1; st.d[i] = (T)0;
#pragma unroll
        for (int j = 0; j < 4; ++j) st.b[i][j] = (T)0;
    }
    if (m == 4) {
        // T4 = L*R + A + I with L = (A2/4 + A)/3 + I, R = A2/2 prepared beforehand (s = 0 here)
        st.L = BUF_T0; st.R = BUF_T1;
        st.nsrc = 1; st.src[0] = BUF_W; st.g[0] = (T)1;
        st.nout = 1; st.dst[0] = BUF_OUT; st.a[0] = (T)1; st.d[0] = (T)1;
    } else if (m == 8) {
        if (r == 1) {
            // y02 = A2 * (c1 A2 + c2 A); emit both factors of T8 and its additive part
            st.L = BUF_W2; st.R = BUF_T0;
            st.nsrc = 2; st.src[0] = BUF_W2; st.src[1] = BUF_W;
            st.nout = 3;
            st.dst[0] = BUF_T1; st.a[0] = (T)1; st.b[0][0] = (T)EXPM_T8_C3; st.b[0][1] = (T)EXPM_T8_C4;
            st.dst[1] = BUF_T2; st.a[1] = (T)1; st.b[1][0] = (T)EXPM_T8_C5;
            st.dst[2] = BUF_T3; st.a[2] = (T)EXPM_T8_C6; st.b[2][0] = (T)0.5; st.b[2][1] = (T)1; st.d[2] = (T)1;
        } else {
            st.L = BUF_T1; st.R = BUF_T2;
            st.nsrc = 1; st.src[0] = BUF_T3; st.g[0] = (T)1;
            st.nout = 1; st.dst[0] = BUF_OUT; st.a[0] = (T)1;
        }
    } else {  // m == 15
        const double sg = __builtin_ldexp(1.0, -s), sg2 = __builtin_ldexp(1.0, -2 * s);
        const int poly_dst = (s & 1) ? BUF_T1 : BUF_OUT;  // so that s squarings later end in OUT
        if (r == 1) {
            st.L = BUF_W2; st.R = BUF_T0; st.acc_scale = (T)sg2;  // y02 = A2 * (c1 A2 + c2 A)
            st.nsrc = 2; st.src[0] = BUF_W2; st.src[1] = BUF_W;
            st.nout = 3;
            st.dst[0] = BUF_T1; st.b[0][0] = (T)(EXPM_T15_C3 * sg2); st.b[0][1] = (T)(EXPM_T15_C4 * sg);
            st.dst[1] = BUF_T2; st.b[1][0] = (T)(EXPM_T15_C5 * sg2);
            st.dst[2] = BUF_T4;  // y02 itself; the additive part c6 y02 + c7 A2 is re-formed in round 2
        } else if (r == 2) {
            st.L = BUF_T1; st.R = BUF_T2;  // y12 = L*R + (c6 y02 + c7 A2)
            st.nsrc = 3; st.src[0] = BUF_T4; st.src[1] = BUF_W2; st.src[2] = BUF_W;
            st.g[0] = (T)EXPM_T15_C6; st.g[1] = (T)(EXPM_T15_C7 * sg2);
            st.nout = 3;
            st.dst[0] = BUF_T0; st.b[0][1] = (T)(EXPM_T15_C8 * sg2); st.b[0][2] = (T)(EXPM_T15_C9 * sg);
            st.dst[1] = BUF_T5; st.b[1][0] = (T)EXPM_T15_C10; st.b[1][2] = (T)(EXPM_T15_C11 * sg);
            st.dst[2] = BUF_T3; st.a[2] = (T)EXPM_T15_C12; st.b[2][0] = (T)EXPM_T15_C13;
            st.b[2][1] = (T)(EXPM_T15_C14 * sg2); st.b[2][2] = (T)(EXPM_T15_C15 * sg); st.d[2] = (T)EXPM_T15_C16;
        } else if (r == 3) {
            st.L = BUF_T0; st.R = BUF_T5;  // y22 = L*R + additive part
            st.nsrc = 1; st.src[0] = BUF_T3; st.g[0] = (T)1;
            st.nout = 1; st.dst[0] = poly_dst;
        } else {
            // squaring q = r-3 of s: ping-pong between OUT and T1, arranged to finish in OUT
            const int q = r - 3;
            const bool cur_is_out = (((s - (q - 1)) & 1) == 0);
            st.L = st.R = cur_is_out ? BUF_OUT : BUF_T1;
            st.nsrc = 0; st.nout = 1; st.dst[0] = cur_is_out ? BUF_T1 : BUF_OUT;
        }
    }
    return st;
}

// Round r (1-based, after the power products) of the Paterson-Stockmeyer chain for order m = j*k and
// scaling s.  Horner in A^j:  H <- H * A^j + sum_{r'<j} c_{qj+r'} A^r',  q = k-2 .. 0, with the top block
// prepared beforehand in T0; intermediate H ping-pongs between T0 and T2; then the squarings.
// `shift` = 0: coefficients 1/i! (the Taylor polynomial); 1: coefficients 1/(i+1)! (core series of the low-rank
// variant, Sec. 2.2, which is never scaled: s = 0).
template <typename T>
__device__ __forceinline__ Step<T> build_step_ps(int m, int s, int r, int shift = 0)
{
    Step<T> st;
    st.L = BUF_T0; st.R = BUF_W2; st.acc_scale = (T)1; st.nsrc = 0; st.nout = 1;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        st.src[i] = BUF_W; st.g[i] = (T)0; st.dst[i] = BUF_OUT; st.a[i] = (T)1; st.d[i] = (T)0;
#pragma unroll
        for (int j = 0; j < 4; ++j) st.b[i][j] = (T)0;
    }
    const int j = ps_j(m), k = ps_k(m);
    const int horner = k - 1;
    const int poly_dst = (s & 1) ? BUF_T1 : BUF_OUT;
    if (r <= horner) {
        const int q = k - 1 - r;  // block whose coefficients are added in this step
        const double sg = __longlong_as_double((long long)(1023 - s) << 52);
        st.L = (r & 1) ? BUF_T0 : BUF_T2;
        st.R = j == 2 ? BUF_W2 : (j == 3 ? BUF_W3 : BUF_W4);
        double sgj = 1.0;
        for (int e = 0; e < j; ++e) sgj *= sg;
        st.acc_scale = (T)sgj;                       // H * A^j = sigma^j (H * W^j)
        st.nsrc = j - 1;                             // A, A^2, A^3 as far as the block reaches
        st.src[0] = BUF_W; st.src[1] = BUF_W2; st.src[2] = BUF_W3;
        st.g[0] = (T)(inv_factorial(q * j + 1 + shift) * sg);
        if (j >= 3) st.g[1] = (T)(inv_factorial(q * j + 2 + shift) * sg * sg);
        if (j >= 4) st.g[2] = (T)(inv_factorial(q * j + 3 + shift) * sg * sg * sg);
        st.nout = 1;
        st.dst[0] = r == horner ? poly_dst : ((r & 1) ? BUF_T2 : BUF_T0);
        st.a[0] = (T)1;
        st.d[0] = (T)inv_factorial(q * j + shift);
    } else {
        const int q = r - horner;  // squaring q of s
        const bool cur_is_out = (((s - (q - 1)) & 1) == 0);
        st.L = st.R = cur_is_out ? BUF_OUT : BUF_T1;
        st.nsrc = 0; st.nout = 1; st.dst[0] = cur_is_out ? BUF_T1 : BUF_OUT;
    }
    return st;
}

// ---------------------------------------------------------------------------------------------
// Baseline of the paper's comparison (its Algorithm 1, Sec. 2.2) on the round-based path.  Per matrix:
// s = smallest s >= 0 with ||W|| / 2^s < 1/2, A = W / 2^s; X = I, Y_1 = A; while ||Y_t|| > eps: X += Y_t,
// Y_(t+1) = A Y_t / (t + 1); then s squarings of X.  Term round t (t = 1, 2, ...) of a matrix that is still in the
// loop does both halves of one pass through the loop body: X += Y_t in its epilogue and the product for Y_(t+1),
// whose norm (taken in the same epilogue) decides whether the matrix takes part in round t + 1.
// MatInfo of this scheme: m = terms added once the coming round has run, s, len = 1 while the matrix is in the loop.
// Buffers: Y_1 is W itself (scaled through the coefficients), Y_t for t >= 2 alternates between T0 and T1, X
// accumulates in OUT when s = 0 and in T2 otherwise (or always in T2 when only (m, s) are wanted); squaring q reads
// T2 (q odd) or T3 (q even) and writes the other one, the last squaring writes OUT.
// ---------------------------------------------------------------------------------------------
constexpr int kBaselineSquareRound = 64;  // round numbers above this are squarings: q = round - kBaselineSquareRound

// Term rounds that can be needed at tolerance eps: ||Y_t|| <= (1/2)^t / t! (the norm of A is below 1/2), so the loop
// has ended once that bound is at most eps; two spare rounds for norms that rounding carries past the bound.
__host__ __device__ inline int baseline_max_terms(double eps)
{
    double bound = 0.5;
    int t = 1;
    while (bound > eps && t < 60) {
        ++t;
        bound *= 0.5 / (double)t;
    }
    return t + 1;
}

template <typename T>
__device__ __forceinline__ Step<T> build_step_baseline(int s, int round, bool keep_in_workspace)
{
    Step<T> st;
    st.acc_scale = (T)1; st.nsrc = 0; st.nout = 1;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        st.src[i] = BUF_W; st.g[i] = (T)0; st.dst[i] = BUF_OUT; st.a[i] = (T)1; st.d[i] = (T)0;
#pragma unroll
        for (int j = 0; j < 4; ++j) st.b[i][j] = (T)0;
    }
    const int xbuf = (s == 0 && !keep_in_workspace) ? BUF_OUT : BUF_T2;
    if (round <= kBaselineSquareRound) {
        const int t = round;
        const double sg = __longlong_as_double((long long)(1023 - s) << 52);   // 2^-s
        st.L = BUF_W;
        st.R = t == 1 ? BUF_W : ((t & 1) ? BUF_T0 : BUF_T1);                // Y_t
        // Y_(t+1) = A Y_t / (t+1) = 2^-s (W Y_t) / (t+1);  Y_1 = 2^-s W adds one more factor 2^-s in round 1
        st.acc_scale = (T)((t == 1 ? sg * sg : sg) / (double)(t + 1));
        st.nout = 2;
        st.dst[0] = ((t + 1) & 1) ? BUF_T0 : BUF_T1;                          // Y_(t+1)
        st.dst[1] = xbuf; st.a[1] = (T)0;
        if (t == 1) {
            st.nsrc = 1; st.src[0] = BUF_W;
            st.b[1][0] = (T)sg; st.d[1] = (T)1;                               // X = I + A
        } else {
            st.nsrc = 2; st.src[0] = xbuf; st.src[1] = st.R;
            st.b[1][0] = (T)1; st.b[1][1] = (T)1;                             // X += Y_t
        }
    } else {
        const int q = round - kBaselineSquareRound;                           // squaring q of s
        const int in = q == 1 ? BUF_T2 : ((q & 1) ? BUF_T2 : BUF_T3);
        st.L = st.R = in;
        st.dst[0] = q == s ? BUF_OUT : ((q & 1) ? BUF_T3 : BUF_T2);
    }
    return st;
}

// ---------------------------------------------------------------------------------------------
// Host-side launchers implemented by the kernel translation units.
// ---------------------------------------------------------------------------------------------
struct GeneralBuffers {
    void *base[BUF_COUNT];   // device pointers, [batch][n][n] each (BUF_W = input, BUF_OUT = output)
    double *colpart;         // [batch][chunks][n] column abs-sum partials of the power rounds (chunks: see the launchers)
    double *colpart_w;       // the same for W itself; a buffer of its own: that pass may run beside the W^2 round
    double *n1, *n2, *n3, *n4;  // [batch][colblocks] per-column-block maxima of the column sums of W .. W^4
    MatInfo *info;           // [batch]
    int *order;              // [batch] matrices sorted by chain length, longest first
    int *summary;            // [64] : [0] longest chain, [1] OR of flags, [2+r] matrices active in round r
    bool ptr_align16;        // input and output pointers are 16-byte aligned (vector loads allowed)
    int norm_inf;            // 0: 1-norm (column sums), 1: infinity-norm (row sums) in the selection
};

// Workgroup ids are handed to the 8 XCDs round-robin; remap so that every XCD works on a
// contiguous range of (matrix, tile) pairs and its L2 sees whole operand panels reused.
__device__ __forceinline__ int xcd_remap(int pid, int total)
{
    const int nx = 8;
    if (total < 2 * nx) return pid;
    const int per = (total + nx - 1) / nx;
    const int tall = total % nx == 0 ? nx : total % nx;  // XCDs that hold `per` ids; the rest hold per-1
    const int xcd = pid % nx, idx = pid / nx;
    return xcd < tall ? xcd * per + idx : tall * per + (xcd - tall) * (per - 1) + idx;
}

// A kernel's dynamic-LDS limit is an attribute of the (kernel, device) pair: run `set` once per device.
struct PerDeviceOnce {
    unsigned long long done = 0;  // bit d: set on device d
    template <class F> hipError_t operator()(F &&set)
    {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        if (dev >= 0 && dev < 64 && ((done >> dev) & 1ull)) return hipSuccess;
        e = set();
        if (e == hipSuccess && dev >= 0 && dev < 64) done |= 1ull << dev;
        return e;
    }
};

// small fused path
bool small_path_supported(int n, int dtype);
hipError_t launch_small(const void *A, void *out, int n, int batch, int dtype, double eps, int select_only,
                        int scheme, int norm_inf, MatInfo *info, hipStream_t stream);

// larger-n path
int general_colchunks(int n);   // row chunks of the column abs-sum pass over the input
int general_colblocks(int n);   // 256-column blocks: per-block maxima make up n1 / n2
int choose_tile_shape(int n, int matrices);  // 4 -> 128x128 tiles, 2 -> 64x64 tiles, 1 -> 32x32 tiles
hipError_t launch_colabs(const GeneralBuffers &gb, int n, int batch, int dtype, hipStream_t stream);
hipError_t launch_colmax(const GeneralBuffers &gb, int n, int batch, int which, int chunks, hipStream_t stream);
hipError_t launch_power_round(const GeneralBuffers &gb, int n, int batch, int dtype, int wt, int which,
                              hipStream_t stream);
hipError_t launch_select_plan(const GeneralBuffers &gb, int n, int batch, double eps, int scheme, hipStream_t stream);
hipError_t launch_prepare(const GeneralBuffers &gb, int n, int batch, int dtype, int scheme, hipStream_t stream);
hipError_t launch_rect_gemm(const void *A, const void *B, void *C, int M, int N, int K, int lda, int ldb, int ldc,
                            size_t stride_a, size_t stride_b, size_t stride_c, int batch, int dtype, int add_identity,
                            int slices, void *partials, hipStream_t stream);
int rect_gemm_slices(int M, int N, int K, int batch, int dtype);
bool first_round_is_self_contained(int n, int scheme);
hipError_t launch_first_round(const GeneralBuffers &gb, int n, int batch, int dtype, hipStream_t stream);
hipError_t launch_chain_round(const GeneralBuffers &gb, int n, int active, int round, int dtype, int wt, int scheme,
                              hipStream_t stream, int first = 0, int step = 1, bool device_plan = false);
// baseline (Algorithm 1) on the round-based path
hipError_t launch_baseline_round(const GeneralBuffers &gb, int n, int batch, int round, int dtype, int wt,
                                 bool keep_in_workspace, hipStream_t stream);
hipError_t launch_baseline_decide(const GeneralBuffers &gb, int n, int batch, double eps, int term, hipStream_t stream);

}  // namespace expmk
