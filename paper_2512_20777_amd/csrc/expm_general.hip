// Round-based path for larger matrices (n above the fused-path limit), gfx950.
//
// Pipeline per call (Algorithm 2 with Algorithm 4, Sec. 3.3 of arXiv 2512.20777):
//   colabs + finalize        ||W||_1 per matrix
//   square round             W2 = W*W for every matrix, column abs-sums of W2 fused in the epilogue
//   finalize                 ||W2||_1
//   select_plan              (m, s) per matrix, chain length, order by chain length, active counts
//   prepare                  results of orders 0,1,2 ; first operand pair for orders 4, 8, 15+
//   chain rounds r = 1..R    one grouped MFMA product per still-active matrix, fused epilogue forming
//                            every linear combination the next round needs (Sec. 3.1 formulas)
//
// The product kernel computes 128x128 tiles with 256 threads (2x2 waves of 64x64), MFMA 16x16x4 in
// the matrix dtype, operands staged through double-buffered LDS in k-blocks of 128 bytes per row.
#include "expm_internal.h"

namespace expmk {

namespace {

constexpr int BM = 128, BN = 128;
constexpr int kThreads = 256;
constexpr int kAPitch = 144;  // bytes per A row in LDS: 128 data + 16 pad (conflict-free 16-byte reads)

template <typename T> struct Tile;
template <> struct Tile<double> {
    static constexpr int BK = 16;        // k-block: 128 bytes of a row
    static constexpr int VN = 2;         // elements per 16-byte vector
    static constexpr int BPitch = 1024 + 128;  // bytes per B row in LDS
    using vec_t = double2;
};
template <> struct Tile<float> {
    static constexpr int BK = 32;
    static constexpr int VN = 4;
    static constexpr int BPitch = 512 + 32;
    using vec_t = float4;
};

template <typename T> constexpr int stage_bytes() { return BM * kAPitch + Tile<T>::BK * Tile<T>::BPitch; }

struct GemmParams {
    void *base[BUF_COUNT];
    const MatInfo *info;
    const int *order;
    double *colpart;
    int n;
    int tiles;   // tiles per dimension
    int round;   // 0 = square round (W2 = W*W), >= 1 chain round
    int total;   // workgroups in the grid
};

__device__ __forceinline__ double pow2neg(int e)
{
    return __longlong_as_double((long long)(1023 - e) << 52);
}

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

template <typename T, bool ALIGNED>
__device__ __forceinline__ typename Tile<T>::vec_t load_vec(const T *__restrict__ p, int row, int col, int n)
{
    using V = typename Tile<T>::vec_t;
    constexpr int VN = Tile<T>::VN;
    V v;
    T *e = reinterpret_cast<T *>(&v);
    if (ALIGNED) {
        if (row < n && col < n) {
            v = *reinterpret_cast<const V *>(p + (size_t)row * n + col);
        } else {
#pragma unroll
            for (int i = 0; i < VN; ++i) e[i] = (T)0;
        }
    } else {
#pragma unroll
        for (int i = 0; i < VN; ++i) e[i] = (row < n && col + i < n) ? p[(size_t)row * n + col + i] : (T)0;
    }
    return v;
}

template <typename T, bool ALIGNED>
__global__ __launch_bounds__(kThreads, 2) void gemm_round_kernel(GemmParams p)
{
    using V = typename Tile<T>::vec_t;
    using acc_t = typename Mfma<T>::acc_t;
    constexpr int BK = Tile<T>::BK, VN = Tile<T>::VN, BPitch = Tile<T>::BPitch;
    constexpr int KQ = BK / 4;            // k values each 16-lane group owns per k-block
    constexpr int VPR = BN / VN;          // 16-byte vectors per B row
    constexpr int STAGE = stage_bytes<T>();
    extern __shared__ __align__(16) unsigned char smem[];

    const int n = p.n;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int lj = lane & 15, lg = lane >> 4;

    // ---- which (matrix, tile) ---------------------------------------------------------------
    const int tiles2 = p.tiles * p.tiles;
    const int wid = xcd_remap(blockIdx.x, p.total);
    const int slot = wid / tiles2;
    int tile = wid - slot * tiles2;
    int b;
    Step<T> st;
    if (p.round == 0) {
        b = slot;
        st.L = BUF_W; st.R = BUF_W; st.acc_scale = (T)1; st.nsrc = 0; st.nout = 1; st.dst[0] = BUF_W2;
    } else {
        b = p.order[slot];
        const MatInfo mi = p.info[b];
        if (p.round > mi.len) return;
        st = build_step<T>(mi.m, mi.s, p.round);
    }
    // grouped tile order: 8 tile-rows at a time, column by column
    int tm, tn;
    {
        const int GM = 8;
        const int per_group = GM * p.tiles;
        const int group = tile / per_group;
        const int first = group * GM;
        const int gsz = min(p.tiles - first, GM);
        const int rem = tile - group * per_group;
        tm = first + rem % gsz;
        tn = rem / gsz;
    }
    const size_t moff = (size_t)b * n * n;
    const T *Lp = reinterpret_cast<const T *>(p.base[st.L]) + moff;
    const T *Rp = reinterpret_cast<const T *>(p.base[st.R]) + moff;

    // ---- staging maps -----------------------------------------------------------------------
    // A tile: 128 rows x 8 vectors ; B tile: BK rows x VPR vectors ; 1024 vectors each, 4 per thread.
    // vector v = tid + 256*i: A row = tid/8 + 32*i, B row = tid/VPR + (256/VPR)*i.
    constexpr int BSTEP = kThreads / VPR;
    const int a_row0 = tid >> 3, a_col = (tid & 7) * VN;
    const int b_row0 = tid / VPR, b_col = (tid % VPR) * VN;
    const int a_lds = a_row0 * kAPitch + (tid & 7) * 16;
    const int b_lds = BM * kAPitch + b_row0 * BPitch + (tid % VPR) * 16;
    const int row0 = tm * BM, col0 = tn * BN;

    acc_t acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = (acc_t)(0);

    const int kblocks = (n + BK - 1) / BK;
    V ra[4], rb[4];
    // prologue: first k-block into stage 0
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        ra[i] = load_vec<T, ALIGNED>(Lp, row0 + a_row0 + 32 * i, a_col, n);
        rb[i] = load_vec<T, ALIGNED>(Rp, b_row0 + BSTEP * i, col0 + b_col, n);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        *reinterpret_cast<V *>(smem + a_lds + 32 * i * kAPitch) = ra[i];
        *reinterpret_cast<V *>(smem + b_lds + BSTEP * i * BPitch) = rb[i];
    }
    __syncthreads();

    // per-lane LDS read offsets (bytes) inside a stage
    //   A: row (wm*64 + 16*ti + lj), k values lg*KQ .. lg*KQ+KQ-1  -> two 16-byte reads
    //   B: row (lg*KQ + kk), column (wn*64 + 16*tj + lj)
    const int a_rd = (wm * 64 + lj) * kAPitch + lg * 32;
    const int b_rd = BM * kAPitch + (lg * KQ) * BPitch + (wn * 64 + lj) * (int)sizeof(T);

    for (int kb = 0; kb < kblocks; ++kb) {
        const unsigned char *cur = smem + (kb & 1) * STAGE;
        unsigned char *nxt = smem + ((kb + 1) & 1) * STAGE;
        const bool more = kb + 1 < kblocks;
        if (more) {
            const int k0 = (kb + 1) * BK;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                ra[i] = load_vec<T, ALIGNED>(Lp, row0 + a_row0 + 32 * i, k0 + a_col, n);
                rb[i] = load_vec<T, ALIGNED>(Rp, k0 + b_row0 + BSTEP * i, col0 + b_col, n);
            }
        }
        // A fragments of the whole k-block
        T af[4][KQ];
#pragma unroll
        for (int ti = 0; ti < 4; ++ti) {
            const V lo = *reinterpret_cast<const V *>(cur + a_rd + ti * 16 * kAPitch);
            const V hi = *reinterpret_cast<const V *>(cur + a_rd + ti * 16 * kAPitch + 16);
            const T *l = reinterpret_cast<const T *>(&lo);
            const T *h = reinterpret_cast<const T *>(&hi);
#pragma unroll
            for (int q = 0; q < VN; ++q) {
                af[ti][q] = l[q];
                af[ti][VN + q] = h[q];
            }
        }
#pragma unroll
        for (int kk = 0; kk < KQ; ++kk) {
            T bf[4];
#pragma unroll
            for (int tj = 0; tj < 4; ++tj)
                bf[tj] = *reinterpret_cast<const T *>(cur + b_rd + kk * BPitch + tj * 16 * (int)sizeof(T));
#pragma unroll
            for (int ti = 0; ti < 4; ++ti)
#pragma unroll
                for (int tj = 0; tj < 4; ++tj) acc[ti][tj] = Mfma<T>::run(af[ti][kk], bf[tj], acc[ti][tj]);
        }
        if (more) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                *reinterpret_cast<V *>(nxt + a_lds + 32 * i * kAPitch) = ra[i];
                *reinterpret_cast<V *>(nxt + b_lds + BSTEP * i * BPitch) = rb[i];
            }
        }
        __syncthreads();
    }

    // ---- epilogue -----------------------------------------------------------------------------
    // lane holds C[row0 + wm*64 + 16*ti + Mfma<T>::row(lg, v)][col0 + wn*64 + 16*tj + lj]
    const int er = row0 + wm * 64;
    const int ec = col0 + wn * 64 + lj;
    if (st.nsrc == 0 && st.nout == 1) {
        T *D = reinterpret_cast<T *>(p.base[st.dst[0]]) + moff;
#pragma unroll
        for (int ti = 0; ti < 4; ++ti)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = er + 16 * ti + Mfma<T>::row(lg, v);
#pragma unroll
                for (int tj = 0; tj < 4; ++tj) {
                    const int col = ec + 16 * tj;
                    if (row < n && col < n) D[(size_t)row * n + col] = acc[ti][tj][v];
                }
            }
    } else {
        const T *S[4];
        T *D[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            S[i] = reinterpret_cast<const T *>(p.base[st.src[i]]) + moff;
            D[i] = reinterpret_cast<T *>(p.base[st.dst[i]]) + moff;
        }
#pragma unroll
        for (int ti = 0; ti < 4; ++ti)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = er + 16 * ti + Mfma<T>::row(lg, v);
#pragma unroll
                for (int tj = 0; tj < 4; ++tj) {
                    const int col = ec + 16 * tj;
                    if (row < n && col < n) {
                        const size_t idx = (size_t)row * n + col;
                        T sv[4];
#pragma unroll
                        for (int i = 0; i < 4; ++i) sv[i] = i < st.nsrc ? S[i][idx] : (T)0;
                        T t = st.acc_scale * acc[ti][tj][v];
#pragma unroll
                        for (int i = 0; i < 4; ++i) t += st.g[i] * sv[i];
                        const T dg = row == col ? (T)1 : (T)0;
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            if (j < st.nout) {
                                T o = st.a[j] * t;
#pragma unroll
                                for (int i = 0; i < 4; ++i) o += st.b[j][i] * sv[i];
                                o += st.d[j] * dg;
                                D[j][idx] = o;
                            }
                        }
                    }
                }
            }
    }

    if (p.round == 0) {
        // column abs-sums of this tile of W2, in double: 64 rows per wave, then the two wave rows
        double *red = reinterpret_cast<double *>(smem);  // [2][128]; the k-loop's last barrier has passed
#pragma unroll
        for (int tj = 0; tj < 4; ++tj) {
            double cs = 0.0;
#pragma unroll
            for (int ti = 0; ti < 4; ++ti)
#pragma unroll
                for (int v = 0; v < 4; ++v) cs += fabs((double)acc[ti][tj][v]);
            cs += __shfl_xor(cs, 16);
            cs += __shfl_xor(cs, 32);
            if (lg == 0) red[wm * BN + wn * 64 + 16 * tj + lj] = cs;
        }
        __syncthreads();
        if (tid < BN) {
            const int col = col0 + tid;
            if (col < n) p.colpart[((size_t)b * p.tiles + tm) * n + col] = red[tid] + red[BN + tid];
        }
    }
}

// ---- ||.||_1 helpers ----------------------------------------------------------------------------
// Column abs-sums of W over row chunks of 128: colpart[b][chunk][col], accumulated in double.
template <typename T>
__global__ __launch_bounds__(256) void colabs_kernel(const T *__restrict__ W, double *__restrict__ colpart, int n, int chunks)
{
    const int col = blockIdx.x * 256 + threadIdx.x;
    const int chunk = blockIdx.y, b = blockIdx.z;
    if (col >= n) return;
    const T *p = W + (size_t)b * n * n;
    const int r0 = chunk * BM, r1 = min(n, r0 + BM);
    double s = 0.0;
    for (int r = r0; r < r1; ++r) s += fabs((double)p[(size_t)r * n + col]);
    colpart[((size_t)b * chunks + chunk) * n + col] = s;
}

// norm[b] = max over columns of (sum over chunks of colpart[b][chunk][col]); NaN if anything is non-finite.
__global__ __launch_bounds__(256) void norm_finalize_kernel(const double *__restrict__ colpart, double *__restrict__ norm,
                                                            int n, int chunks)
{
    __shared__ double smax[256];
    __shared__ int sbad[256];
    const int b = blockIdx.x, tid = threadIdx.x;
    double mx = 0.0;
    int bad = 0;
    for (int col = tid; col < n; col += 256) {
        double s = 0.0;
        for (int c = 0; c < chunks; ++c) s += colpart[((size_t)b * chunks + c) * n + col];
        if (!(s <= 1.7976931348623157e308)) bad = 1;  // NaN or Inf
        if (s > mx) mx = s;
    }
    smax[tid] = mx;
    sbad[tid] = bad;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if (tid < w) {
            if (smax[tid + w] > smax[tid]) smax[tid] = smax[tid + w];
            sbad[tid] |= sbad[tid + w];
        }
        __syncthreads();
    }
    if (tid == 0) norm[b] = sbad[0] ? __longlong_as_double(0x7ff8000000000000LL) : smax[0];
}

// ---- selection and plan ---------------------------------------------------------------------------
// One workgroup.  Writes info[b], the order (longest chain first) and the summary:
//   summary[0] = longest chain, summary[1] = OR of flags, summary[2 + r] = matrices active in round r.
__global__ __launch_bounds__(1024) void select_plan_kernel(const double *__restrict__ n1, const double *__restrict__ n2,
                                                           MatInfo *__restrict__ info, int *__restrict__ order,
                                                           int *__restrict__ summary, int batch, double eps)
{
    __shared__ int hist[kMaxRounds + 1];
    __shared__ int cursor[kMaxRounds + 1];
    __shared__ int flags_or;
    const int tid = threadIdx.x;
    if (tid <= kMaxRounds) hist[tid] = 0;
    if (tid == 0) flags_or = 0;
    __syncthreads();
    for (int b = tid; b < batch; b += blockDim.x) {
        MatInfo mi;
        select_order_scaling(n1[b], n2[b], eps, mi.m, mi.s, mi.flags);
        mi.len = chain_length(mi.m, mi.s);
        info[b] = mi;
        atomicAdd(&hist[mi.len], 1);
        if (mi.flags) atomicOr(&flags_or, mi.flags);
    }
    __syncthreads();
    if (tid == 0) {
        int run = 0, longest = 0;
        for (int len = kMaxRounds; len >= 0; --len) {
            cursor[len] = run;
            run += hist[len];
            if (hist[len] > 0 && len > longest) longest = len;
            if (len >= 1) summary[2 + len] = run;  // matrices with chain length >= len
        }
        summary[0] = longest;
        summary[1] = flags_or;
        summary[2] = batch;
    }
    __syncthreads();
    for (int b = tid; b < batch; b += blockDim.x) {
        const int len = info[b].len;
        order[atomicAdd(&cursor[len], 1)] = b;
    }
}

// ---- operand preparation --------------------------------------------------------------------------
// Orders 0, 1, 2 are finished here (no further product); orders 4, 8, 15+ get the operands of their
// first chain round.  One workgroup handles 1024 consecutive elements of one matrix.
template <typename T>
__global__ __launch_bounds__(256) void prepare_kernel(GemmParams p)
{
    const int b = blockIdx.y;
    const MatInfo mi = p.info[b];
    const int n = p.n;
    const size_t nn = (size_t)n * n, moff = (size_t)b * nn;
    const T *W = reinterpret_cast<const T *>(p.base[BUF_W]) + moff;
    const T *W2 = reinterpret_cast<const T *>(p.base[BUF_W2]) + moff;
    T *O = reinterpret_cast<T *>(p.base[BUF_OUT]) + moff;
    T *T0 = reinterpret_cast<T *>(p.base[BUF_T0]) + moff;
    T *T1 = reinterpret_cast<T *>(p.base[BUF_T1]) + moff;
    const double sg = mi.s > 0 ? pow2neg(mi.s) : 1.0, sg2 = mi.s > 0 ? pow2neg(2 * mi.s) : 1.0;
    const T c1_8 = (T)EXPM_T8_C1, c2_8 = (T)EXPM_T8_C2;
    const T c1_15 = (T)(EXPM_T15_C1 * sg2), c2_15 = (T)(EXPM_T15_C2 * sg);
    for (int e = 0; e < 4; ++e) {
        const size_t idx = ((size_t)blockIdx.x * 4 + e) * 256 + threadIdx.x;
        if (idx >= nn) break;
        const int row = (int)(idx / n), col = (int)(idx - (size_t)row * n);
        const T dg = row == col ? (T)1 : (T)0;
        if (mi.m < 0) {
            O[idx] = (T)__longlong_as_double(0x7ff8000000000000LL);
        } else if (mi.m == 0) {
            O[idx] = dg;                                         // P_0 = I
        } else if (mi.m == 1) {
            O[idx] = W[idx] + dg;                                // T_1 = A + I
        } else if (mi.m == 2) {
            O[idx] = W2[idx] / (T)2 + W[idx] + dg;               // T_2 = A^2/2 + A + I
        } else if (mi.m == 4) {
            const T a2 = W2[idx], a = W[idx];
            T0[idx] = (a2 / (T)4 + a) / (T)3 + dg;               // left factor of T_4
            T1[idx] = a2 / (T)2;                                 // right factor of T_4
        } else if (mi.m == 8) {
            T0[idx] = c1_8 * W2[idx] + c2_8 * W[idx];            // right factor of y02 (order 8)
        } else {
            T0[idx] = c1_15 * W2[idx] + c2_15 * W[idx];          // right factor of y02 (order 15+), scaled
        }
    }
}

template <typename T, bool ALIGNED>
hipError_t launch_gemm_t(const GemmParams &p, hipStream_t stream)
{
    static bool attr_done = false;
    const int lds = 2 * stage_bytes<T>();
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(gemm_round_kernel<T, ALIGNED>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    hipLaunchKernelGGL((gemm_round_kernel<T, ALIGNED>), dim3(p.total), dim3(kThreads), lds, stream, p);
    return hipGetLastError();
}

GemmParams make_params(const GeneralBuffers &gb, int n, int round, int matrices)
{
    GemmParams p;
    for (int i = 0; i < BUF_COUNT; ++i) p.base[i] = gb.base[i];
    p.info = gb.info;
    p.order = gb.order;
    p.colpart = gb.colpart;
    p.n = n;
    p.tiles = general_tiles(n);
    p.round = round;
    p.total = matrices * p.tiles * p.tiles;
    return p;
}

hipError_t launch_gemm(const GemmParams &p, int dtype, bool ptr_align16, hipStream_t stream)
{
    if (p.total <= 0) return hipSuccess;
    if (dtype == 1) {
        return (ptr_align16 && p.n % 2 == 0) ? launch_gemm_t<double, true>(p, stream)
                                             : launch_gemm_t<double, false>(p, stream);
    }
    return (ptr_align16 && p.n % 4 == 0) ? launch_gemm_t<float, true>(p, stream) : launch_gemm_t<float, false>(p, stream);
}

}  // namespace

int general_tiles(int n) { return (n + BM - 1) / BM; }

hipError_t launch_colabs(const GeneralBuffers &gb, int n, int batch, int dtype, hipStream_t stream)
{
    const int chunks = general_tiles(n);
    dim3 grid((n + 255) / 256, chunks, batch);
    if (dtype == 1)
        hipLaunchKernelGGL(colabs_kernel<double>, grid, dim3(256), 0, stream,
                           reinterpret_cast<const double *>(gb.base[BUF_W]), gb.colpart, n, chunks);
    else
        hipLaunchKernelGGL(colabs_kernel<float>, grid, dim3(256), 0, stream,
                           reinterpret_cast<const float *>(gb.base[BUF_W]), gb.colpart, n, chunks);
    return hipGetLastError();
}

hipError_t launch_norm_finalize(const GeneralBuffers &gb, int n, int batch, int which, hipStream_t stream)
{
    hipLaunchKernelGGL(norm_finalize_kernel, dim3(batch), dim3(256), 0, stream, gb.colpart, which == 1 ? gb.n1 : gb.n2, n,
                       general_tiles(n));
    return hipGetLastError();
}

hipError_t launch_square_round(const GeneralBuffers &gb, int n, int batch, int dtype, hipStream_t stream)
{
    return launch_gemm(make_params(gb, n, 0, batch), dtype, gb.ptr_align16, stream);
}

hipError_t launch_select_plan(const GeneralBuffers &gb, int n, int batch, double eps, hipStream_t stream)
{
    (void)n;
    hipLaunchKernelGGL(select_plan_kernel, dim3(1), dim3(1024), 0, stream, gb.n1, gb.n2, gb.info, gb.order, gb.summary,
                       batch, eps);
    return hipGetLastError();
}

hipError_t launch_prepare(const GeneralBuffers &gb, int n, int batch, int dtype, hipStream_t stream)
{
    const GemmParams p = make_params(gb, n, 0, batch);
    const size_t nn = (size_t)n * n;
    dim3 grid((unsigned)((nn + 1023) / 1024), batch);
    if (dtype == 1)
        hipLaunchKernelGGL(prepare_kernel<double>, grid, dim3(256), 0, stream, p);
    else
        hipLaunchKernelGGL(prepare_kernel<float>, grid, dim3(256), 0, stream, p);
    return hipGetLastError();
}

hipError_t launch_chain_round(const GeneralBuffers &gb, int n, int active, int round, int dtype, hipStream_t stream)
{
    return launch_gemm(make_params(gb, n, round, active), dtype, gb.ptr_align16, stream);
}

}  // namespace expmk
