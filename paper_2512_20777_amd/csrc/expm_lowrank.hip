// Rectangular batched products for the low-rank variant of Sec. 2.2 of arXiv 2512.20777, gfx950:
//     e^(A1 A2) = I + A1 phi(V) A2,   V = A2 A1 (t x t),   phi(V) = sum_{i<=m} V^i / (i+1)!
// Three products of this file frame the on-chip evaluation of phi (fused kernel, scheme kSchemePhi):
//     V = A2 A1 (t x n x t),   U = A1 phi (n x t x t),   out = U A2 + I (n x t x n).
// The last one writes n^2 outputs from an inner dimension of only t: it is bound by its output stream, so
// the kernel is kept simple -- 64x64 tile per workgroup, 2x2 waves of 2x2 MFMA 16x16x4 tiles, one LDS
// stage, element-wise bounds checks (any n, t and alignment).
#include "expm_internal.h"

namespace expmk {

namespace {

template <typename T>
__global__ __launch_bounds__(256) void rect_gemm_kernel(const T *__restrict__ A, const T *__restrict__ B, T *__restrict__ C,
                                                        int M, int N, int K, int lda, int ldb, int ldc, size_t sa, size_t sb,
                                                        size_t sc, int add_identity)
{
    using acc_t = typename Mfma<T>::acc_t;
    constexpr int BM = 64, BN = 64;
    constexpr int BK = sizeof(T) == 4 ? 32 : 16;
    constexpr int PA = BK + 4 / (int)(sizeof(T) / 4);  // words of padding keep the fragment reads off one bank
    constexpr int PB = BN + 16;
    __shared__ T As[BM * PA];
    __shared__ T Bs[BK * PB];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1, lj = lane & 15, lg = lane >> 4;
    const int row0 = blockIdx.y * BM, col0 = blockIdx.x * BN;
    A += (size_t)blockIdx.z * sa;
    B += (size_t)blockIdx.z * sb;
    C += (size_t)blockIdx.z * sc;

    acc_t acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = (acc_t)(0);

    for (int k0 = 0; k0 < K; k0 += BK) {
        // stage the A tile (BM x BK) and the B tile (BK x BN), zero beyond the matrix
#pragma unroll
        for (int e = tid; e < BM * BK; e += 256) {
            const int r = e / BK, c = e % BK;
            As[r * PA + c] = (row0 + r < M && k0 + c < K) ? A[(size_t)(row0 + r) * lda + k0 + c] : (T)0;
        }
#pragma unroll
        for (int e = tid; e < BK * BN; e += 256) {
            const int r = e / BN, c = e % BN;
            Bs[r * PB + c] = (k0 + r < K && col0 + c < N) ? B[(size_t)(k0 + r) * ldb + col0 + c] : (T)0;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < BK / 4; ++kk) {
            T a[2], b[2];
#pragma unroll
            for (int ti = 0; ti < 2; ++ti) a[ti] = As[(wm * 32 + 16 * ti + lj) * PA + 4 * kk + lg];
#pragma unroll
            for (int tj = 0; tj < 2; ++tj) b[tj] = Bs[(4 * kk + lg) * PB + wn * 32 + 16 * tj + lj];
#pragma unroll
            for (int ti = 0; ti < 2; ++ti)
#pragma unroll
                for (int tj = 0; tj < 2; ++tj) acc[ti][tj] = Mfma<T>::run(a[ti], b[tj], acc[ti][tj]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int ti = 0; ti < 2; ++ti)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int row = row0 + wm * 32 + 16 * ti + Mfma<T>::row(lg, v);
#pragma unroll
            for (int tj = 0; tj < 2; ++tj) {
                const int col = col0 + wn * 32 + 16 * tj + lj;
                if (row < M && col < N) {
                    T x = acc[ti][tj][v];
                    if (add_identity && row == col) x += (T)1;
                    C[(size_t)row * ldc + col] = x;
                }
            }
        }
}

}  // namespace

// C[b] (M x N, leading dimension ldc) = A[b] (M x K, lda) * B[b] (K x N, ldb) (+ I), b < batch; strides in elements
hipError_t launch_rect_gemm(const void *A, const void *B, void *C, int M, int N, int K, int lda, int ldb, int ldc,
                            size_t stride_a, size_t stride_b, size_t stride_c, int batch, int dtype, int add_identity,
                            hipStream_t stream)
{
    if (M <= 0 || N <= 0 || batch <= 0) return hipSuccess;
    const dim3 grid((unsigned)((N + 63) / 64), (unsigned)((M + 63) / 64), (unsigned)batch);
    if (dtype == 1)
        hipLaunchKernelGGL(rect_gemm_kernel<double>, grid, dim3(256), 0, stream, reinterpret_cast<const double *>(A),
                           reinterpret_cast<const double *>(B), reinterpret_cast<double *>(C), M, N, K, lda, ldb, ldc,
                           stride_a, stride_b, stride_c, add_identity);
    else
        hipLaunchKernelGGL(rect_gemm_kernel<float>, grid, dim3(256), 0, stream, reinterpret_cast<const float *>(A),
                           reinterpret_cast<const float *>(B), reinterpret_cast<float *>(C), M, N, K, lda, ldb, ldc,
                           stride_a, stride_b, stride_c, add_identity);
    return hipGetLastError();
}

}  // namespace expmk
