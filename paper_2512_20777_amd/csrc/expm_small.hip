// Fused single-kernel path for small matrices, gfx950.
//
// One workgroup per matrix.  The matrix is loaded once into LDS, every step of Algorithm 2 and
// Algorithm 4 (Sec. 3.3 of arXiv 2512.20777) runs on LDS-resident data -- ||W||_1, W^2 and its
// norm, the choice of (m, s), the evaluation formulas of Sec. 3.1, the s squarings -- and the
// result is written once.  (m, s) is uniform over the workgroup, so no wavefront diverges.
// Products use MFMA 16x16x4 in the matrix dtype on 16x16 tiles of the zero-padded matrix.
#include "expm_internal.h"

namespace expmk {

namespace {

// LDS matrices are [NP][NP+1] elements (odd pitch: conflict-free row-strided operand reads).
template <typename T, int NT> struct SmallCfg {
    static constexpr int NP = 16 * NT;
    static constexpr int LP = NP + 1;
    static constexpr int kThreads = NT == 1 ? 64 : 256;
    static constexpr int kWaves = kThreads / 64;
    static constexpr int kTiles = NT * NT;
    static constexpr int kTilesPerWave = (kTiles + kWaves - 1) / kWaves;
    static constexpr int kMatBytes = NP * LP * (int)sizeof(T);
    static constexpr int kNumMats = 6;  // A, A2, Y (y02), P, Q, G
    static constexpr int kLds = kNumMats * kMatBytes + 64 * (int)sizeof(double) + 16;
};

__device__ __forceinline__ double pow2neg_small(int e)
{
    return __longlong_as_double((long long)(1023 - e) << 52);
}

template <typename T, int NT>
__global__ __launch_bounds__(NT == 1 ? 64 : 256) void small_expm_kernel(const T *__restrict__ Ain, T *__restrict__ Out,
                                                                               int n, double eps, int select_only,
                                                                               MatInfo *__restrict__ info)
{
    using C = SmallCfg<T, NT>;
    using acc_t = typename Mfma<T>::acc_t;
    constexpr int NP = C::NP, LP = C::LP, TPW = C::kTilesPerWave;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    T *mA = reinterpret_cast<T *>(smem_raw);
    T *mA2 = mA + NP * LP;
    T *mY = mA2 + NP * LP;
    T *mP = mY + NP * LP;
    T *mQ = mP + NP * LP;
    T *mG = mQ + NP * LP;
    double *red = reinterpret_cast<double *>(smem_raw + C::kNumMats * C::kMatBytes + ((16 - (C::kNumMats * C::kMatBytes) % 16) % 16));

    const int b = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lj = lane & 15, lg = lane >> 4;
    const size_t moff = (size_t)b * n * n;
    const T *W = Ain + moff;

    // ---- load W, zero padded --------------------------------------------------------------------
    for (int e = tid; e < NP * NP; e += C::kThreads) {
        const int r = e / NP, c = e - r * NP;
        mA[r * LP + c] = (r < n && c < n) ? W[(size_t)r * n + c] : (T)0;
    }
    __syncthreads();

    // ---- 1-norm of an LDS matrix: max column abs-sum, double accumulation, NaN if non-finite -------
    auto norm1 = [&](const T *M) -> double {
        double s = 0.0;
        if (tid < NP) {
            for (int r = 0; r < n; ++r) s += fabs((double)M[r * LP + tid]);
        }
        int bad = !(s <= 1.7976931348623157e308);
        // wave reduce (max, or)
        for (int off = 32; off > 0; off >>= 1) {
            const double o = __shfl_xor(s, off);
            const int ob = __shfl_xor(bad, off);
            s = o > s ? o : s;
            bad |= ob;
        }
        __syncthreads();  // red[] free to overwrite
        if (lane == 0) { red[wave] = s; red[8 + wave] = (double)bad; }
        __syncthreads();
        double mx = red[0];
        double anybad = red[8];
        for (int w = 1; w < C::kWaves; ++w) {
            mx = red[w] > mx ? red[w] : mx;
            anybad += red[8 + w];
        }
        return anybad != 0.0 ? __longlong_as_double(0x7ff8000000000000LL) : mx;
    };

    // ---- product of two LDS matrices into this wave's accumulator tiles ----------------------------
    // tile t = wave + kWaves*q -> (ti, tj) = (t / NT, t % NT)
    auto product = [&](const T *L, const T *R, acc_t *acc) {
#pragma unroll
        for (int q = 0; q < TPW; ++q) {
            const int t = wave + C::kWaves * q;
            acc[q] = (acc_t)(0);
            if (t < C::kTiles) {
                const int ti = t / NT, tj = t - ti * NT;
                const T *lp = L + (16 * ti + lj) * LP + lg;
                const T *rp = R + lg * LP + 16 * tj + lj;
#pragma unroll
                for (int kk = 0; kk < NP / 4; ++kk) acc[q] = Mfma<T>::run(lp[4 * kk], rp[4 * kk * LP], acc[q]);
            }
        }
    };
    // visit every element this lane owns: f(q, v, row, col)
    auto for_owned = [&](auto &&f) {
#pragma unroll
        for (int q = 0; q < TPW; ++q) {
            const int t = wave + C::kWaves * q;
            if (t < C::kTiles) {
                const int ti = t / NT, tj = t - ti * NT;
#pragma unroll
                for (int v = 0; v < 4; ++v) f(q, v, 16 * ti + Mfma<T>::row(lg, v), 16 * tj + lj);
            }
        }
    };

    acc_t acc[TPW];
    int m = 0, s = 0, flags = 0;

    const double n1 = norm1(mA);
    double n2 = 0.0;
    bool have_w2 = false;
    {
        // m = 0 and m = 1 need no product (Algorithm 4 forms W^2 only once the m = 1 test has failed)
        const bool finite1 = n1 == n1;
        const bool tiny = finite1 && (n1 == 0.0 || (0.5 * n1 * n1 + (1.0 / 6.0) * n1 * n1 * n1 <= eps));
        if (finite1 && !tiny) {
            product(mA, mA, acc);
            for_owned([&](int q, int v, int r, int c) { mA2[r * LP + c] = acc[q][v]; });
            __syncthreads();
            n2 = norm1(mA2);
            have_w2 = true;
        }
    }
    select_order_scaling(n1, n2, eps, m, s, flags);
    if (tid == 0) {
        MatInfo mi;
        mi.m = m; mi.s = s; mi.len = 0; mi.flags = flags;
        info[b] = mi;
    }
    if (select_only) return;
    T *O = Out + moff;

    if (m < 0) {
        const T qnan = (T)__longlong_as_double(0x7ff8000000000000LL);
        for (int e = tid; e < n * n; e += C::kThreads) O[e] = qnan;
        return;
    }

    // ---- scale: A = W / 2^s, A2 = W2 / 4^s (exact) ------------------------------------------------
    if (s > 0) {
        const T sg = (T)pow2neg_small(s), sg2 = (T)pow2neg_small(2 * s);
        for_owned([&](int, int, int r, int c) {
            mA[r * LP + c] *= sg;
            mA2[r * LP + c] *= sg2;
        });
    }
    (void)have_w2;
    T *X = mP;  // where the polynomial ends up
    auto dg = [&](int r, int c) -> T { return (r == c && r < n) ? (T)1 : (T)0; };

    if (m <= 2) {
        for_owned([&](int, int, int r, int c) {
            T x = dg(r, c);
            if (m >= 1) x += mA[r * LP + c];
            if (m == 2) x += mA2[r * LP + c] / (T)2;
            X[r * LP + c] = x;
        });
    } else if (m == 4) {
        // T4 = ((A2/4 + A)/3 + I) * (A2/2) + A + I
        for_owned([&](int, int, int r, int c) {
            const T a = mA[r * LP + c], a2 = mA2[r * LP + c];
            mP[r * LP + c] = (a2 / (T)4 + a) / (T)3 + dg(r, c);
            mQ[r * LP + c] = a2 / (T)2;
        });
        __syncthreads();
        product(mP, mQ, acc);
        __syncthreads();
        for_owned([&](int q, int v, int r, int c) { X[r * LP + c] = acc[q][v] + mA[r * LP + c] + dg(r, c); });
    } else if (m == 8) {
        const T c1 = (T)EXPM_T8_C1, c2 = (T)EXPM_T8_C2, c3 = (T)EXPM_T8_C3, c4 = (T)EXPM_T8_C4, c5 = (T)EXPM_T8_C5,
                c6 = (T)EXPM_T8_C6;
        for_owned([&](int, int, int r, int c) { mQ[r * LP + c] = c1 * mA2[r * LP + c] + c2 * mA[r * LP + c]; });
        __syncthreads();
        product(mA2, mQ, acc);  // y02
        __syncthreads();
        for_owned([&](int q, int v, int r, int c) {
            const T y = acc[q][v], a = mA[r * LP + c], a2 = mA2[r * LP + c];
            mP[r * LP + c] = y + c3 * a2 + c4 * a;
            mQ[r * LP + c] = y + c5 * a2;
            mG[r * LP + c] = c6 * y + a2 / (T)2 + a + dg(r, c);
        });
        __syncthreads();
        product(mP, mQ, acc);
        __syncthreads();
        for_owned([&](int q, int v, int r, int c) { X[r * LP + c] = acc[q][v] + mG[r * LP + c]; });
    } else {  // 15+
        const T c1 = (T)EXPM_T15_C1, c2 = (T)EXPM_T15_C2, c3 = (T)EXPM_T15_C3, c4 = (T)EXPM_T15_C4, c5 = (T)EXPM_T15_C5,
                c6 = (T)EXPM_T15_C6, c7 = (T)EXPM_T15_C7, c8 = (T)EXPM_T15_C8, c9 = (T)EXPM_T15_C9,
                c10 = (T)EXPM_T15_C10, c11 = (T)EXPM_T15_C11, c12 = (T)EXPM_T15_C12, c13 = (T)EXPM_T15_C13,
                c14 = (T)EXPM_T15_C14, c15 = (T)EXPM_T15_C15, c16 = (T)EXPM_T15_C16;
        for_owned([&](int, int, int r, int c) { mQ[r * LP + c] = c1 * mA2[r * LP + c] + c2 * mA[r * LP + c]; });
        __syncthreads();
        product(mA2, mQ, acc);  // y02
        __syncthreads();
        for_owned([&](int q, int v, int r, int c) {
            const T y = acc[q][v], a = mA[r * LP + c], a2 = mA2[r * LP + c];
            mY[r * LP + c] = y;
            mP[r * LP + c] = y + c3 * a2 + c4 * a;
            mQ[r * LP + c] = y + c5 * a2;
            mG[r * LP + c] = c6 * y + c7 * a2;
        });
        __syncthreads();
        product(mP, mQ, acc);
        __syncthreads();
        for_owned([&](int q, int v, int r, int c) {
            const T a = mA[r * LP + c], a2 = mA2[r * LP + c], y0 = mY[r * LP + c];
            const T y1 = acc[q][v] + mG[r * LP + c];  // y12
            mP[r * LP + c] = y1 + c8 * a2 + c9 * a;
            mQ[r * LP + c] = y1 + c10 * y0 + c11 * a;
            mG[r * LP + c] = c12 * y1 + c13 * y0 + c14 * a2 + c15 * a + c16 * dg(r, c);
        });
        __syncthreads();
        product(mP, mQ, acc);
        __syncthreads();
        for_owned([&](int q, int v, int r, int c) { X[r * LP + c] = acc[q][v] + mG[r * LP + c]; });
    }
    __syncthreads();

    // ---- squaring phase ------------------------------------------------------------------------------
    for (int q = 0; q < s; ++q) {
        product(X, X, acc);
        __syncthreads();
        for_owned([&](int qq, int v, int r, int c) { X[r * LP + c] = acc[qq][v]; });
        __syncthreads();
    }

    // ---- store -------------------------------------------------------------------------------------------
    for (int e = tid; e < n * n; e += C::kThreads) {
        const int r = e / n, c = e - r * n;
        O[e] = X[r * LP + c];
    }
}

template <typename T, int NT>
hipError_t launch_small_t(const void *A, void *out, int n, int batch, double eps, int select_only, MatInfo *info,
                          hipStream_t stream)
{
    using C = SmallCfg<T, NT>;
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(small_expm_kernel<T, NT>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, C::kLds);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    hipLaunchKernelGGL((small_expm_kernel<T, NT>), dim3(batch), dim3(C::kThreads), C::kLds, stream,
                       reinterpret_cast<const T *>(A), reinterpret_cast<T *>(out), n, eps, select_only, info);
    return hipGetLastError();
}

}  // namespace

bool small_path_supported(int n, int dtype)
{
    return dtype == 1 ? n <= 48 : n <= 64;
}

hipError_t launch_small(const void *A, void *out, int n, int batch, int dtype, double eps, int select_only,
                        MatInfo *info, hipStream_t stream)
{
    const int nt = (n + 15) / 16;
    if (dtype == 1) {
        switch (nt) {
        case 1: return launch_small_t<double, 1>(A, out, n, batch, eps, select_only, info, stream);
        case 2: return launch_small_t<double, 2>(A, out, n, batch, eps, select_only, info, stream);
        case 3: return launch_small_t<double, 3>(A, out, n, batch, eps, select_only, info, stream);
        default: return hipErrorInvalidValue;
        }
    }
    switch (nt) {
    case 1: return launch_small_t<float, 1>(A, out, n, batch, eps, select_only, info, stream);
    case 2: return launch_small_t<float, 2>(A, out, n, batch, eps, select_only, info, stream);
    case 3: return launch_small_t<float, 3>(A, out, n, batch, eps, select_only, info, stream);
    case 4: return launch_small_t<float, 4>(A, out, n, batch, eps, select_only, info, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace expmk
