// Rectangular batched products for the low-rank variant of Sec. 2.2 of arXiv 2512.20777, gfx950:
//     e^(A1 A2) = I + A1 phi(V) A2,   V = A2 A1 (t x t),   phi(V) = sum_{i<=m} V^i / (i+1)!
// Three products of this file frame the on-chip evaluation of phi (fused kernel, scheme kSchemePhi):
//     V = A2 A1 (t x n x t),   U = A1 phi (n x t x t),   out = U A2 + I (n x t x n).
// V has few outputs and a long inner dimension: its inner dimension is cut into slices that separate workgroups
// sum, and a second small kernel adds the slices in a fixed order.  The last product has 2t flops per output
// element: at t = 64 in fp32 its matrix-core time and the time to stream the n^2 outputs are about equal.
//
// One kernel serves all three: a 32*WT x 32*WT tile per workgroup, 2x2 waves of WT x WT MFMA 16x16x4 tiles, two
// LDS stages (the next k-block is fetched into registers while the current one is multiplied), left rows padded
// for 16-byte fragment reads, right rows rotated per k-group.  Operands are read as 16-byte vectors when the
// leading dimensions, sizes and addresses allow it and element by element otherwise; every access is bounds-checked.
#include "expm_internal.h"
#include "expm_tile.h"

namespace expmk {

namespace {

constexpr int kRectThreads = kTileThreads;
constexpr int kRectMinGroups = 1024;

// How the operands are fetched: element by element, as 16-byte vectors through registers (both bounds-checked),
// or -- every tile full, every slice a whole number of k-blocks -- as 16-byte vectors straight into LDS
// (global_load_lds: lane l of a wave writes its 16 bytes at a wave-uniform base + 16 l, so a tile is a sequence of
// 16-byte slots and the lane that owns a slot fetches the vector that belongs there).
constexpr int kRectScalar = 0, kRectVector = 1, kRectDma = 2;

struct RectParams {
    const void *A, *B;
    void *C;
    int M, N, K;
    int lda, ldb, ldc;
    size_t sa, sb, sc;   // strides between the matrices of the batch, in elements
    int slices;          // slices of the inner dimension (1: the product is written whole)
    int kslice;          // inner indices per slice, a multiple of the k-block
    size_t sslice;       // stride between the partial products of one matrix, in elements
    int add_identity;
    int ctiles;          // column tiles one workgroup goes through
    int groups;          // workgroups per tile row
    int per_matrix;      // workgroups per matrix and slice
    int total;           // workgroups in the grid
};

// VN elements of row `row` from column `col` of a rows x cols matrix; zero beyond it
template <typename T, bool VEC>
__device__ __forceinline__ typename Tile<T>::vec_t rect_load(const T *__restrict__ p, int row, int col, int rows, int cols,
                                                                 int ld)
{
    using V = typename Tile<T>::vec_t;
    constexpr int VN = Tile<T>::VN;
    V v;
    T *e = reinterpret_cast<T *>(&v);
    if constexpr (VEC) {
        if (row < rows && col < cols) {   // cols is a multiple of VN here: a vector is inside or outside as a whole
            v = *reinterpret_cast<const V *>(p + (size_t)row * ld + col);
        } else {
#pragma unroll
            for (int i = 0; i < VN; ++i) e[i] = (T)0;
        }
    } else {
#pragma unroll
        for (int i = 0; i < VN; ++i) e[i] = (row < rows && col + i < cols) ? p[(size_t)row * ld + col + i] : (T)0;
    }
    return v;
}

// RES (direct-to-LDS variant, inner dimension of at most kResBlocks k-blocks, several column tiles per workgroup):
// the workgroup's left panel is fetched once and stays in LDS, the stages hold right tiles only.
constexpr int kResBlocks = 2;
template <typename T, int WT, int MODE, bool RES = false>
__global__ __launch_bounds__(kRectThreads, WT == 4 ? 2 : 4) void rect_gemm_kernel(RectParams p)
{
    constexpr bool VEC = MODE >= kRectVector, DMA = MODE == kRectDma;
    static_assert(!RES || DMA, "the resident left panel belongs to the direct-to-LDS variant");
    using S = TileStaging<T, WT, DMA>;              // tile layouts in LDS and who stages what (expm_tile.h)
    using V = typename Tile<T>::vec_t;
    using acc_t = typename Mfma<T>::acc_t;
    constexpr int BM = S::BM, BN = S::BN, BK = S::BK, VN = S::VN;
    constexpr int APitch = S::APitch, BPitch = S::BPitch, BSTEP = S::BSTEP, kRot = S::kRot;
    constexpr int STAGE = RES ? S::kRightBytes : stage_bytes<T, WT>(DMA);
    constexpr int kRightAt = RES ? 0 : S::kLeftBytes;   // where the right tile starts in a stage
    // Two LDS stages; with the direct-to-LDS loads two separate LDS objects and a loop written out for both parities
    // (an LDS read is ordered behind every outstanding load into an LDS object it may alias: with one array for both
    // stages nothing would be fetched while a wave multiplies).
    extern __shared__ __align__(16) unsigned char smem_dyn[];
    __shared__ __align__(16) unsigned char stage_even[DMA ? STAGE : 16];
    __shared__ __align__(16) unsigned char stage_odd[DMA ? STAGE : 16];
    __shared__ __align__(16) unsigned char left_panel[RES ? kResBlocks * S::kLeftBytes : 16];
    unsigned char *const smem = DMA ? stage_even : smem_dyn;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1, lj = lane & 15, lg = lane >> 4;
    const int M = p.M, N = p.N;
    // workgroup -> (matrix and slice, tile row, group of column tiles); every XCD gets a contiguous range, so the
    // operand panels of a matrix stay within one L2
    const int wid = xcd_remap(blockIdx.x, p.total);
    const int bz = wid / p.per_matrix, rem = wid - bz * p.per_matrix;
    const int gy = rem / p.groups, gx = rem - gy * p.groups;
    const int b = bz / p.slices, slice = bz - b * p.slices;
    const int kbeg = slice * p.kslice, kend = min(p.K, kbeg + p.kslice);
    const int row0 = gy * BM;
    const int ct0 = gx * p.ctiles;                                    // first column tile of this workgroup
    const int nct = min(p.ctiles, (N + BN - 1) / BN - ct0);           // >= 1 by construction of the grid
    const T *Lp = reinterpret_cast<const T *>(p.A) + (size_t)b * p.sa;
    const T *Rp = reinterpret_cast<const T *>(p.B) + (size_t)b * p.sb;
    T *Cp = reinterpret_cast<T *>(p.C) + (size_t)b * p.sc + (size_t)slice * p.sslice;

    // staging maps (expm_tile.h)
    const S sg(tid);
    const int a_row0 = sg.a_row0, a_col = sg.a_col, b_row0 = sg.b_row0, b_col = sg.b_col;

    acc_t acc[WT][WT];
    auto clear = [&]() {
#pragma unroll
        for (int i = 0; i < WT; ++i)
#pragma unroll
            for (int j = 0; j < WT; ++j) acc[i][j] = (acc_t)(0);
    };
    clear();

    // The (column tile, k-block) pairs of this workgroup form one sequence of steps: the operands of step i + 1 are
    // fetched while step i is multiplied, across tile boundaries too, and a finished tile is stored at the start of
    // the next tile's first step (before that step's fetch: the fetched vectors need not stay live across the stores).
    const int kblocks = kend > kbeg ? (kend - kbeg + BK - 1) / BK : 0;
    const int steps = nct * kblocks;
    V ra[WT], rb[WT];
    int f_kb = 0, f_ct = ct0;  // step the next fetch belongs to
    auto fetch = [&]() __attribute__((always_inline)) {
        const int k0 = kbeg + f_kb * BK, col0 = f_ct * BN;
#pragma unroll
        for (int i = 0; i < WT; ++i) {
            ra[i] = rect_load<T, VEC>(Lp, row0 + a_row0 + 32 * i, k0 + a_col, M, kend, p.lda);
            rb[i] = rect_load<T, VEC>(Rp, k0 + b_row0 + BSTEP * i, col0 + b_col, kend, N, p.ldb);
        }
        if (++f_kb == kblocks) {
            f_kb = 0;
            ++f_ct;
        }
    };
    auto stash = [&](unsigned char *stage) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < WT; ++i) {
            *reinterpret_cast<V *>(stage + sg.left_write(i)) = ra[i];
            *reinterpret_cast<V *>(stage + sg.right_write(i)) = rb[i];
        }
    };
    // one k-block of the step the next fetch belongs to, straight into a stage (slot layout: expm_tile.h)
    auto dma = [&](unsigned char *stage) __attribute__((always_inline)) {
        if constexpr (DMA) {
            if constexpr (RES) sg.fetch_right_to_lds(Rp, (size_t)p.ldb, f_ct * BN, kbeg + f_kb * BK, stage);
            else sg.fetch_to_lds(Lp, (size_t)p.lda, row0, Rp, (size_t)p.ldb, f_ct * BN, kbeg + f_kb * BK, stage);
            if (++f_kb == kblocks) {
                f_kb = 0;
                ++f_ct;
            }
        }
    };
    // this wave's global-to-LDS loads have landed (vmcnt(0)); must hold before the barrier that lets others read them
    auto dma_done = [&]() {
        if constexpr (DMA) __builtin_amdgcn_s_waitcnt(0x0F70);
    };
    // lane holds C[row0 + wm*16*WT + 16*ti + Mfma<T>::row(lg, v)][ct*BN + wn*16*WT + 16*tj + lj]
    auto store_tile = [&](int ct) __attribute__((always_inline)) {
        int er = row0 + wm * 16 * WT;
        asm volatile("" : "+v"(er));  // offsets are formed here, next to the stores, not kept in registers across the loop
        int ec = wn * 16 * WT + lj;
        asm volatile("" : "+v"(ec));
        ec += ct * BN;
        // 32-bit element offsets inside one matrix (M * ldc < 2^31 for every row that is stored)
        const unsigned ldc = (unsigned)p.ldc;
        const bool inside = row0 + BM <= M && ct * BN + BN <= N;                                  // uniform
        const bool diagonal = p.add_identity && row0 < ct * BN + BN && ct * BN < row0 + BM;     // uniform
        if (inside && !diagonal) {
            // whole tile off the diagonal: one per-lane base, uniform row offsets, no predicates
            T *base = Cp + ((unsigned)(er + Mfma<T>::row(lg, 0)) * ldc + (unsigned)ec);
#pragma unroll
            for (int ti = 0; ti < WT; ++ti)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    T *r = base + (unsigned)(16 * ti + Mfma<T>::row(0, v)) * ldc;
#pragma unroll
                    for (int tj = 0; tj < WT; ++tj) r[16 * tj] = acc[ti][tj][v];
                }
            return;
        }
#pragma unroll
        for (int ti = 0; ti < WT; ++ti)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = er + 16 * ti + Mfma<T>::row(lg, v);
                const unsigned ro = (unsigned)row * ldc;
#pragma unroll
                for (int tj = 0; tj < WT; ++tj) {
                    const int col = ec + 16 * tj;
                    if (row < M && col < N) {
                        T x = acc[ti][tj][v];
                        if (p.add_identity && row == col) x += (T)1;
                        Cp[ro + (unsigned)col] = x;
                    }
                }
            }
    };
    if (steps == 0) {  // empty inner range: the tiles are zero (+ I)
        for (int i = 0; i < nct; ++i) store_tile(ct0 + i);
        return;
    }
    if constexpr (DMA) {
        if constexpr (RES) {
            for (int kb = 0; kb < kblocks; ++kb)   // kblocks <= kResBlocks: the launcher's condition for this variant
                sg.fetch_left_to_lds(Lp, (size_t)p.lda, row0, kbeg + kb * BK, left_panel + kb * S::kLeftBytes);
        }
        dma(smem);
        dma_done();
    } else {
        fetch();
        stash(smem);
    }
    __syncthreads();

    const int a_rd0 = S::left_read(wm, lj, lg, 0), a_rd1 = S::left_read(wm, lj, lg, 1);
    const int b_rd = S::right_read_base(lg) - S::kLeftBytes + lj * (int)sizeof(T);   // relative to the right tile
    const int b_rc0 = (wn * 16 * WT + 16 * lg) * (int)sizeof(T);

    auto multiply = [&](const unsigned char *left, const unsigned char *right) __attribute__((always_inline)) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            V af[WT];
#pragma unroll
            for (int ti = 0; ti < WT; ++ti) af[ti] = *reinterpret_cast<const V *>(left + (h ? a_rd1 : a_rd0) + ti * 16 * APitch);
#pragma unroll
            for (int q = 0; q < VN; ++q) {
                const int kk = h * VN + q;
                T bf[WT];
#pragma unroll
                for (int tj = 0; tj < WT; ++tj)
                    bf[tj] = *reinterpret_cast<const T *>(right + b_rd + kk * BPitch + ((b_rc0 + tj * kRot) & (BPitch - 1)));
#pragma unroll
                for (int ti = 0; ti < WT; ++ti) {
                    const T a = reinterpret_cast<const T *>(&af[ti])[q];
#pragma unroll
                    for (int tj = 0; tj < WT; ++tj) acc[ti][tj] = Mfma<T>::run(a, bf[tj], acc[ti][tj]);
                }
            }
        }
    };

    int c_kb = 0, c_ct = ct0;  // step being multiplied
    auto step = [&](const unsigned char *cur, unsigned char *nxt, int s) __attribute__((always_inline)) {
        const bool more = s + 1 < steps;
        if (c_kb == 0 && s > 0) {
            store_tile(c_ct - 1);
            clear();
        }
        if constexpr (DMA) {
            if (more) dma(nxt);
            if constexpr (RES) multiply(left_panel + c_kb * S::kLeftBytes, cur);
            else multiply(cur, cur + kRightAt);
            dma_done();
        } else {
            if (more) fetch();
            multiply(cur, cur + kRightAt);
            if (more) stash(nxt);
        }
        __syncthreads();
        if (++c_kb == kblocks) {
            c_kb = 0;
            ++c_ct;
        }
    };
    if constexpr (DMA) {
        int s = 0;
        for (; s + 1 < steps; s += 2) {
            step(stage_even, stage_odd, s);
            step(stage_odd, stage_even, s + 1);
        }
        if (s < steps) step(stage_even, stage_odd, s);
    } else {
        for (int s = 0; s < steps; ++s) step(smem + (s & 1) * STAGE, smem + ((s + 1) & 1) * STAGE, s);
    }
    store_tile(ct0 + nct - 1);
}

// C[b][e] = sum over the slices, in slice order, of P[b][slice][e]
template <typename T>
__global__ __launch_bounds__(256) void slice_sum_kernel(const T *__restrict__ P, T *__restrict__ C, size_t elems, int slices)
{
    const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= elems) return;
    const T *src = P + (size_t)blockIdx.y * slices * elems + e;
    T sum = (T)0;
    for (int s = 0; s < slices; ++s) sum += src[(size_t)s * elems];
    C[(size_t)blockIdx.y * elems + e] = sum;
}

template <typename T, int WT, int MODE>
hipError_t launch_rect_v(const RectParams &p, dim3 grid, hipStream_t stream)
{
    const int lds = 2 * stage_bytes<T, WT>(MODE == kRectDma);
    if constexpr (MODE == kRectDma) {
        // the direct-to-LDS variant holds its two stages in static LDS
        static_assert(2 * stage_bytes<T, WT>(true) <= 65536, "static LDS of the direct-to-LDS variant");
        // a short inner dimension walked over several column tiles: the left panel stays in LDS
        if (p.slices == 1 && p.K <= kResBlocks * Tile<T>::BK && p.ctiles > 1) {
            hipLaunchKernelGGL((rect_gemm_kernel<T, WT, MODE, true>), grid, dim3(kRectThreads), 0, stream, p);
            return hipGetLastError();
        }
        hipLaunchKernelGGL((rect_gemm_kernel<T, WT, MODE>), grid, dim3(kRectThreads), 0, stream, p);
        return hipGetLastError();
    }
    static PerDeviceOnce lds_limit;  // the 128x128 tile needs more dynamic LDS than the default limit
    hipError_t e = lds_limit([] {
        return hipFuncSetAttribute(reinterpret_cast<const void *>(rect_gemm_kernel<T, WT, MODE>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    });
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((rect_gemm_kernel<T, WT, MODE>), grid, dim3(kRectThreads), lds, stream, p);
    return hipGetLastError();
}

template <typename T, int WT>
hipError_t launch_rect_t(const RectParams &p, int batch, bool vec, hipStream_t stream)
{
    constexpr int BT = 32 * WT;
    // several column tiles per workgroup hide the first fetch and the last store of a tile behind its neighbours;
    // keep at least kRectMinGroups workgroups so that the chip stays covered and the last round stays short
    const int tn = (p.N + BT - 1) / BT, tm = (p.M + BT - 1) / BT;
    const long rows = (long)tm * batch * p.slices;
    int ct = 1;
    while (ct < 8 && ct < tn && rows * ((tn + 2 * ct - 1) / (2 * ct)) >= kRectMinGroups) ct *= 2;
    RectParams q = p;
    q.ctiles = ct;
    q.groups = (tn + ct - 1) / ct;
    q.per_matrix = q.groups * tm;
    const long total = (long)q.per_matrix * batch * p.slices;
    if (total > 0x7fffffffL) return hipErrorInvalidValue;
    q.total = (int)total;
    const dim3 grid((unsigned)total);
    constexpr int bk = Tile<T>::BK;
    if (vec && p.M % BT == 0 && p.N % BT == 0 && p.K % bk == 0) return launch_rect_v<T, WT, kRectDma>(q, grid, stream);
    if (vec) return launch_rect_v<T, WT, kRectVector>(q, grid, stream);
    return launch_rect_v<T, WT, kRectScalar>(q, grid, stream);
}

}  // namespace

// Slices of the inner dimension for a product with few output tiles: enough workgroups to cover the chip twice,
// every slice at least two k-blocks long (64 pairs of 64 x 1024 factors: 8 slices; 16 were 2 % slower for the call,
// 4 the same).  1 means no slicing (and no partial buffer).
int rect_gemm_slices(int M, int N, int K, int batch, int dtype)
{
    if (M <= 0 || N <= 0 || K <= 0 || batch <= 0) return 1;
    const int bt = (M <= 64 || N <= 64) ? 64 : 128;
    const int bk = dtype == 1 ? 16 : 32;
    const long tiles = (long)((M + bt - 1) / bt) * ((N + bt - 1) / bt) * batch;
    const long want = (512 + tiles - 1) / tiles;
    const long most = K / (2 * bk);
    long s = want < most ? want : most;
    if (s > 64) s = 64;
    return s < 2 ? 1 : (int)s;
}

// C[b] (M x N, leading dimension ldc) = A[b] (M x K, lda) * B[b] (K x N, ldb) (+ I), b < batch; strides in elements.
// slices > 1: `partials` holds batch * slices * M * N elements; the slices are summed into C (ldc = N, stride M * N).
hipError_t launch_rect_gemm(const void *A, const void *B, void *C, int M, int N, int K, int lda, int ldb, int ldc,
                            size_t stride_a, size_t stride_b, size_t stride_c, int batch, int dtype, int add_identity,
                            int slices, void *partials, hipStream_t stream)
{
    if (M <= 0 || N <= 0 || batch <= 0) return hipSuccess;
    const int w = dtype == 1 ? 8 : 4, vn = 16 / w, bk = dtype == 1 ? 16 : 32;
    if (slices < 1 || partials == nullptr) slices = 1;
    if (slices > 1 && (ldc != N || stride_c != (size_t)M * N || add_identity)) return hipErrorInvalidValue;
    RectParams p{};
    p.A = A; p.B = B;
    p.M = M; p.N = N; p.K = K;
    p.lda = lda; p.ldb = ldb;
    p.sa = stride_a; p.sb = stride_b;
    p.slices = slices;
    p.add_identity = add_identity;
    if (slices > 1) {
        const int blocks = (K + bk - 1) / bk;
        p.kslice = ((blocks + slices - 1) / slices) * bk;
        p.C = partials;
        p.ldc = N;
        p.sslice = (size_t)M * N;
        p.sc = (size_t)slices * M * N;
    } else {
        p.kslice = ((K + bk - 1) / bk) * bk;
        if (p.kslice == 0) p.kslice = bk;
        p.C = C;
        p.ldc = ldc;
        p.sslice = 0;
        p.sc = stride_c;
    }
    const bool vec = K % vn == 0 && N % vn == 0 && lda % vn == 0 && ldb % vn == 0 && stride_a % vn == 0 && stride_b % vn == 0 &&
                     (reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(B)) % 16 == 0;
    const bool small = M <= 64 || N <= 64;
    hipError_t e;
    if (dtype == 1) e = small ? launch_rect_t<double, 2>(p, batch, vec, stream) : launch_rect_t<double, 4>(p, batch, vec, stream);
    else e = small ? launch_rect_t<float, 2>(p, batch, vec, stream) : launch_rect_t<float, 4>(p, batch, vec, stream);
    if (e != hipSuccess || slices == 1) return e;
    const size_t elems = (size_t)M * N;
    const dim3 grid((unsigned)((elems + 255) / 256), (unsigned)batch);
    if (dtype == 1)
        hipLaunchKernelGGL(slice_sum_kernel<double>, grid, dim3(256), 0, stream, reinterpret_cast<const double *>(partials),
                           reinterpret_cast<double *>(C), elems, slices);
    else
        hipLaunchKernelGGL(slice_sum_kernel<float>, grid, dim3(256), 0, stream, reinterpret_cast<const float *>(partials),
                           reinterpret_cast<float *>(C), elems, slices);
    return hipGetLastError();
}

}  // namespace expmk
