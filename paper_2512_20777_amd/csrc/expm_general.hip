// Round-based path for larger matrices (n above the fused-path limit), gfx950.
//
// Pipeline per call (Algorithm 2 with Algorithm 4, Sec. 3.3 of arXiv 2512.20777):
//   colabs + colmax          ||W||_1 per matrix (per-column-block maxima, reduced by the selection)
//   square round             W2 = W*W for every matrix, column abs-sums of W2 fused in the epilogue
//   colmax                   ||W2||_1
//   select_plan              (m, s) per matrix, chain length, order by chain length, active counts
//   prepare                  results of orders 0,1,2 ; first operand pair for orders 4, 8, 15+
//   chain rounds r = 1..R    one grouped MFMA product per still-active matrix, fused epilogue forming
//                            every linear combination the next round needs (Sec. 3.1 formulas)
//
// The product kernel computes a (32*WT)x(32*WT) tile per workgroup of 256 threads (2x2 waves, each
// WT x WT MFMA 16x16x4 tiles in the matrix dtype); WT = 4 for large matrices, WT = 2 below n = 1024 and for
// launches with too few tiles to give every compute unit two workgroups, WT = 1 for thin launches.
// Operands are staged through double-buffered LDS in k-blocks of 128 bytes per row: straight from global
// memory into LDS when tiles are full and rows 16-byte aligned, through registers otherwise.
#include "expm_internal.h"
#include "expm_tile.h"

#include <utility>

#include <cstdlib>

namespace expmk {

namespace {

constexpr int kThreads = kTileThreads;
constexpr int kThinGroups = 384;    // launches of at most this many 64x64 tiles switch to 32x32 tiles
constexpr int kColChunk = 32;   // rows per column-abs-sum partial of the input matrix

// G neighbouring columns per lane: the 16 columns of MFMA tile tj of a wave do not stand for columns 16 tj .. 16 tj + 15
// of the wave's span but, in groups of G tiles, for columns (tj / G) * 16 G + G * lj + tj % G (lj = lane % 16).  A lane's
// right-operand fragments for the G tiles of a group are then G neighbouring elements of an LDS row (one 8- or 16-byte
// read instead of G reads), and its results for them are G neighbouring elements of an output row (one vector access
// per source and destination in the epilogue).  G = 16 bytes' worth of elements, at most the tiles per wave.
template <typename T, int WT> constexpr int col_group() { return WT < 16 / (int)sizeof(T) ? WT : 16 / (int)sizeof(T); }
template <typename T, int N> struct VecOfN { typedef T type __attribute__((ext_vector_type(N))); };

template <int... I, class F> __device__ __forceinline__ void static_for(std::integer_sequence<int, I...>, F &&f)
{
    (f(std::integral_constant<int, I>{}), ...);
}

struct GemmParams {
    void *base[BUF_COUNT];
    const MatInfo *info;
    const int *order;
    double *colpart;
    int n;
    int tiles;   // tiles per dimension
    int round;   // <= 0 power round (0: W2 = W*W, -1: W3 = W2*W, -2: W4 = W3*W), >= 1 chain round
    int total;   // workgroups in the grid
    int slot0, slot_step;  // chain rounds: this launch covers the sorted matrices slot0, slot0 + slot_step, ...
    int scheme;  // kSchemeSastre, kSchemePS, kSchemeBaseline or kSchemePhi
    int norm_inf;  // power rounds: emit row abs-sums (infinity-norm) instead of column abs-sums
    const int *active;  // rounds planned on the device: &summary[2], active[r] = matrices still active in round r; else null
    int keep;    // baseline scheme: accumulate X in the workspace even when s = 0 (only (m, s) are wanted)
};

__device__ __forceinline__ double pow2neg(int e)
{
    return __longlong_as_double((long long)(1023 - e) << 52);
}

// How a product kernel may touch its operands: element by element with bounds checks, 16-byte vectors with
// bounds checks, or 16-byte vectors with none (n a multiple of the tile and of the k-block: every tile full).
constexpr int kAccessScalar = 0, kAccessVector = 1, kAccessFull = 2, kAccessDma = 3;
// kAccessDma: as kAccessFull, and the operand tiles go from global memory straight into LDS (16 bytes per lane,
// global_load_lds): no staging registers, no LDS store instructions, and the loads of the next k-block stay in
// flight for the whole multiply phase.  A lane's 16 bytes land at (wave-uniform base) + 16 * lane, so the tile
// layouts are made of whole 16-byte slots in slot order and the permutation that keeps the fragment reads off
// one bank is applied on the global side: the lane that owns a slot fetches the vector that belongs there.

// grouped tile order: 8 tile-rows at a time, column by column
__device__ __forceinline__ void tile_position(int tile, int tiles, int &tm, int &tn)
{
    const int GM = 8;
    const int per_group = GM * tiles;
    const int group = tile / per_group;
    const int first = group * GM;
    const int gsz = min(tiles - first, GM);
    const int rem = tile - group * per_group;
    tm = first + rem % gsz;
    tn = rem / gsz;
}

template <typename T, int ALIGNED>
__device__ __forceinline__ typename Tile<T>::vec_t load_vec(const T *__restrict__ p, int row, int col, int n)
{
    using V = typename Tile<T>::vec_t;
    constexpr int VN = Tile<T>::VN;
    if constexpr (ALIGNED >= kAccessFull) return *reinterpret_cast<const V *>(p + (size_t)row * n + col);
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

// FIRST: chain round 1 of the main scheme without a preparation pass.  The operand that is a linear combination of
// W^2 and W (right factor c1 A^2 + c2 A of y02 for orders 8 and 15+, left factor A^2/12 + A/3 + I of T_4) is formed
// while its tile is staged (one more vector per staged vector, combined just before the LDS store), and the
// workgroups of matrices of order <= 2, which need no product, write their tile of the result and leave.
template <typename T, int WT, int ALIGNED, bool FIRST = false>
__global__ __launch_bounds__(kThreads, WT == 4 ? 2 : (FIRST && ALIGNED == kAccessDma ? 3 : 4)) void gemm_round_kernel(GemmParams p)
{
    using V = typename Tile<T>::vec_t;
    using acc_t = typename Mfma<T>::acc_t;
    constexpr bool DMA = ALIGNED == kAccessDma;
    using S = TileStaging<T, WT, DMA>;            // tile layouts in LDS and who stages what (expm_tile.h)
    constexpr int BM = S::BM, BN = S::BN, BK = S::BK, VN = S::VN;
    constexpr int APitch = S::APitch, BPitch = S::BPitch, BSTEP = S::BSTEP;
    constexpr int G = col_group<T, WT>();         // neighbouring columns per lane (see col_group)
    using GV = typename VecOfN<T, G>::type;
    constexpr bool kPipe = DMA && !FIRST && sizeof(T) == 4;  // fragment reads one k-step ahead (fp32: registers to spare; fp64 loses)
    // FIRST with the direct-to-LDS loads: a third tile per stage holds the part of W that goes into the combined
    // operand, in the layout of the side it belongs to (both tiles are 32*WT*128 bytes); the combination is formed
    // from the two fragments, on their way from LDS into the MFMAs.
    constexpr bool kFragComb = DMA && FIRST;
    constexpr int kXOff = BM * APitch + BK * BPitch;   // offset of that tile in a stage
    static_assert(!kFragComb || BM * APitch == BK * BPitch, "left and right tiles of equal size");
    constexpr int STAGE = stage_bytes<T, WT>(DMA) + (kFragComb ? BM * APitch : 0);
    // Two LDS stages.  With the direct-to-LDS loads they are two separate LDS objects and the k-loop below is written
    // out for both parities: the compiler orders every LDS read behind all outstanding loads into an LDS object the
    // read may alias, so with one array holding both stages a wave waited for the next k-block's loads before it
    // read the current k-block's fragments, and nothing was fetched while it multiplied.
    // The 32 x 32 tiles (a few workgroups per compute unit, launches of small batches and the tails of chains) wait
    // for memory most of the time with one k-block in flight; they keep three in flight in a ring of four stages.
    constexpr bool kRing = DMA && WT == 1;
    extern __shared__ __align__(16) unsigned char smem_dyn[];
    __shared__ __align__(16) unsigned char stage_even[DMA ? STAGE : 16];
    __shared__ __align__(16) unsigned char stage_odd[DMA ? STAGE : 16];
    __shared__ __align__(16) unsigned char stage_2[kRing ? STAGE : 16];
    __shared__ __align__(16) unsigned char stage_3[kRing ? STAGE : 16];
    unsigned char *const smem = DMA ? stage_even : smem_dyn;   // stage 0: prologue, and scratch of the epilogue

    const int n = p.n;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int lj = lane & 15, lg = lane >> 4;

    // ---- which (matrix, tile) ---------------------------------------------------------------
    const int tiles2 = p.tiles * p.tiles;
    // Rounds planned on the device are launched over the whole batch: the workgroups beyond this round's active
    // prefix of the sorted list leave, and the others spread over the XCDs as a launch of exactly that size would.
    int total = p.total;
    if (p.active != nullptr) {
        total = min(total, p.active[p.round] * tiles2);
        if ((int)blockIdx.x >= total) return;
    }
    const int wid = xcd_remap(blockIdx.x, total);
    const int slot = wid / tiles2;
    const int tile = wid - slot * tiles2;
    int b;
    Step<T> st;
    int first_m = 0;      // FIRST: order of this matrix (4: left operand combined, 8 / 15: right operand combined)
    T xa = (T)1, xb = (T)0;  // FIRST: coefficients of W^2 and W in the combined operand
    if (p.round <= 0) {
        b = slot;
        st.L = p.round == 0 ? BUF_W : (p.round == -1 ? BUF_W2 : BUF_W3);
        st.R = BUF_W;
        st.acc_scale = (T)1; st.nsrc = 0; st.nout = 1;
        st.dst[0] = p.round == 0 ? BUF_W2 : (p.round == -1 ? BUF_W3 : BUF_W4);
    } else if (p.scheme == kSchemeBaseline) {
        // Algorithm 1: matrices in input order; a matrix leaves the term rounds when the norm of its last term
        // has dropped to the tolerance, and takes part in squaring q only while q <= s
        b = slot;
        const MatInfo mi = p.info[b];
        if (p.round <= kBaselineSquareRound) {
            if (!mi.len) {
                if (p.round == 1) {
                    // never entered the loop (zero matrix, or ||A|| <= eps): X = I; not finite: NaN
                    int tm0, tn0;
                    tile_position(tile, p.tiles, tm0, tn0);
                    T *O = reinterpret_cast<T *>(p.base[(mi.s <= 0 && !p.keep) ? BUF_OUT : BUF_T2]) + (size_t)b * n * n;
                    for (int e = tid; e < BM * BN; e += kThreads) {
                        const int r = tm0 * BM + e / BN, c = tn0 * BN + e % BN;
                        if (r < n && c < n)
                            O[(size_t)r * n + c] = mi.m < 0 ? (T)__longlong_as_double(0x7ff8000000000000LL) : (r == c ? (T)1 : (T)0);
                    }
                }
                return;
            }
        } else if (p.round - kBaselineSquareRound > mi.s) {
            return;
        }
        st = build_step_baseline<T>(mi.s, p.round, p.keep != 0);
    } else {
        b = p.order[p.slot0 + slot * p.slot_step];
        const MatInfo mi = p.info[b];
        if constexpr (FIRST) {
            first_m = mi.m;
            if (mi.m <= 2) {
                // no product: P_0 = I, T_1 = A + I, T_2 = A^2/2 + A + I (s = 0 for these orders), NaN if not finite
                int tm0, tn0;
                tile_position(tile, p.tiles, tm0, tn0);
                const size_t mo = (size_t)b * n * n;
                const T *Wp = reinterpret_cast<const T *>(p.base[BUF_W]) + mo;
                const T *W2p = reinterpret_cast<const T *>(p.base[BUF_W2]) + mo;
                T *O = reinterpret_cast<T *>(p.base[BUF_OUT]) + mo;
                for (int e = tid; e < BM * BN; e += kThreads) {
                    const int r = tm0 * BM + e / BN, c = tn0 * BN + e % BN;
                    if (r < n && c < n) {
                        const size_t idx = (size_t)r * n + c;
                        const T dg = r == c ? (T)1 : (T)0;
                        T o;
                        if (mi.m < 0) o = (T)__longlong_as_double(0x7ff8000000000000LL);
                        else if (mi.m == 0) o = dg;
                        else if (mi.m == 1) o = Wp[idx] + dg;
                        else o = W2p[idx] / (T)2 + Wp[idx] + dg;
                        O[idx] = o;
                    }
                }
                return;
            }
            st = build_step<T>(mi.m, mi.s, 1);
            // both operands start from W^2; the combined side adds W
            st.L = BUF_W2; st.R = BUF_W2;
            if (mi.m == 4) {
                xa = (T)(1.0 / 12.0); xb = (T)(1.0 / 3.0);   // left factor A^2/12 + A/3 + I (s = 0)
                st.acc_scale = (T)0.5;                        // right factor A^2/2
            } else if (mi.m == 8) {
                xa = (T)EXPM_T8_C1; xb = (T)EXPM_T8_C2;       // right factor c1 A^2 + c2 A (s = 0)
            } else {
                const double sg = mi.s > 0 ? pow2neg(mi.s) : 1.0, sg2 = mi.s > 0 ? pow2neg(2 * mi.s) : 1.0;
                xa = (T)(EXPM_T15_C1 * sg2); xb = (T)(EXPM_T15_C2 * sg);
            }
        } else {
            if (p.round > mi.len) return;
            st = p.scheme == kSchemePS ? build_step_ps<T>(mi.m, mi.s, p.round)
                 : (p.scheme == kSchemePhi ? build_step_ps<T>(mi.m, 0, p.round, 1) : build_step<T>(mi.m, mi.s, p.round));
        }
    }
    int tm, tn;
    tile_position(tile, p.tiles, tm, tn);
    const size_t moff = (size_t)b * n * n;
    const T *Lp = reinterpret_cast<const T *>(p.base[st.L]) + moff;
    const T *Rp = reinterpret_cast<const T *>(p.base[st.R]) + moff;

    // ---- staging maps (expm_tile.h) -----------------------------------------------------------
    const S sg(tid);
    const int a_row0 = sg.a_row0, a_col = sg.a_col, b_row0 = sg.b_row0, b_col = sg.b_col;
    const int row0 = tm * BM, col0 = tn * BN;

    acc_t acc[WT][WT];
#pragma unroll
    for (int i = 0; i < WT; ++i)
#pragma unroll
        for (int j = 0; j < WT; ++j) acc[i][j] = (acc_t)(0);

    const int kblocks = (n + BK - 1) / BK;
    V ra[WT], rb[WT];
    // FIRST: the vectors of W that go into the combined operand, at the A positions (order 4) or the B positions
    V rx[FIRST ? WT : 1];
    const T *Xp = reinterpret_cast<const T *>(p.base[BUF_W]) + moff;
    const bool comb_a = FIRST && first_m == 4;  // uniform over the workgroup
    auto fetch_x = [&](int k0) {
        if constexpr (FIRST) {
#pragma unroll
            for (int i = 0; i < WT; ++i)
                rx[i] = comb_a ? load_vec<T, ALIGNED>(Xp, row0 + a_row0 + 32 * i, k0 + a_col, n)
                               : load_vec<T, ALIGNED>(Xp, k0 + b_row0 + BSTEP * i, col0 + b_col, n);
        }
    };
    // combined operand = xa * (vector of W^2) + xb * (vector of W) (+ I on the left side), element by element
    auto combine = [&](int k0) {
        if constexpr (FIRST) {
#pragma unroll
            for (int i = 0; i < WT; ++i) {
                T *dst = reinterpret_cast<T *>(comb_a ? &ra[i] : &rb[i]);
                const T *x = reinterpret_cast<const T *>(&rx[i]);
#pragma unroll
                for (int e = 0; e < VN; ++e) {
                    T v = xa * dst[e] + xb * x[e];
                    if (comb_a && row0 + a_row0 + 32 * i == k0 + a_col + e) v += (T)1;
                    dst[e] = v;
                }
            }
        }
    };
    // one k-block straight into a stage (slot layout: expm_tile.h)
    auto dma = [&](int k0, unsigned char *stage) {
        if constexpr (DMA) {
            sg.fetch_to_lds(Lp, (size_t)n, row0, Rp, (size_t)n, col0, k0, stage);
            if constexpr (kFragComb) {
                // W at the positions of the side that is combined (uniform over the workgroup)
#pragma unroll
                for (int i = 0; i < WT; ++i) {
                    const T *gx = comb_a ? Xp + (size_t)(row0 + sg.left_row(i)) * n + k0 + sg.a_kv
                                         : Xp + (size_t)(k0 + sg.right_row(i)) * n + col0 + sg.right_col(i);
                    S::to_lds(gx, stage + kXOff + sg.slot(i));
                }
            }
        }
    };
    // all of this wave's global-to-LDS loads have landed (vmcnt(0)): must hold before the barrier that lets the
    // other waves read them
    auto dma_done = [&]() {
        if constexpr (DMA) __builtin_amdgcn_s_waitcnt(0x0F70);
    };

    // prologue: first k-block into stage 0 (the ring of four stages has its own, below)
    const bool ring = kRing && kblocks >= 3;   // uniform over the launch
    if constexpr (DMA) {
        if (!ring) {
            dma(0, smem);
            dma_done();
        }
    } else {
#pragma unroll
        for (int i = 0; i < WT; ++i) {
            ra[i] = load_vec<T, ALIGNED>(Lp, row0 + a_row0 + 32 * i, a_col, n);
            rb[i] = load_vec<T, ALIGNED>(Rp, b_row0 + BSTEP * i, col0 + b_col, n);
        }
        fetch_x(0);
        combine(0);
#pragma unroll
        for (int i = 0; i < WT; ++i) {
            *reinterpret_cast<V *>(smem + sg.left_write(i)) = ra[i];
            *reinterpret_cast<V *>(smem + sg.right_write(i)) = rb[i];
        }
    }
    if (!ring) __syncthreads();

    // per-lane LDS read offsets (bytes) inside a stage: two 16-byte reads per left fragment (h = 0, 1), and the right
    // rows of this lane group; the rotated column of the lane's first group of G tiles follows below
    const int a_rd0 = S::left_read(wm, lj, lg, 0), a_rd1 = S::left_read(wm, lj, lg, 1);
    const int b_rd = S::right_read_base(lg);
    const int b_rc0 = (wn * 16 * WT + G * lj + 16 * lg) * (int)sizeof(T);  // rotated column of this lane's first group, before wrap

    // the products of one staged k-block
    auto multiply = [&](const unsigned char *cur, int kb) __attribute__((always_inline)) {
        // A fragments: each lane's KQ k-values of a row are two 16-byte halves (h = 0, 1), VN k-steps each.
        if constexpr (kPipe) {
            // Fragment registers in two sets: the reads for k-step kk + 1 (and, at the end of a half, for the next
            // half of the left rows) are issued ahead of the 16 MFMAs of k-step kk and land while those run.
            V af[2][WT];
            GV bv[2][WT / G];
            auto read_a = [&](int h) {
#pragma unroll
                for (int ti = 0; ti < WT; ++ti)
                    af[h & 1][ti] = *reinterpret_cast<const V *>(cur + (h ? a_rd1 : a_rd0) + ti * 16 * APitch);
            };
            auto read_b = [&](int kk) {
#pragma unroll
                for (int g = 0; g < WT / G; ++g)
                    bv[kk & 1][g] = *reinterpret_cast<const GV *>(cur + b_rd + kk * BPitch +
                                                                   ((b_rc0 + g * 16 * G * (int)sizeof(T)) & (BPitch - 1)));
            };
            read_a(0);
            read_b(0);
            static_for(std::make_integer_sequence<int, 2 * VN>{}, [&](auto KK) {
                constexpr int kk = decltype(KK)::value, h = kk / VN, q = kk % VN;
                constexpr bool more_b = kk + 1 < 2 * VN, more_a = more_b && q == VN - 1;
                if constexpr (more_b) read_b(kk + 1);
                if constexpr (more_a) read_a(h + 1);
#pragma unroll
                for (int ti = 0; ti < WT; ++ti) {
                    const T a = reinterpret_cast<const T *>(&af[h & 1][ti])[q];
#pragma unroll
                    for (int tj = 0; tj < WT; ++tj) acc[ti][tj] = Mfma<T>::run(a, bv[kk & 1][tj / G][tj % G], acc[ti][tj]);
                }
                // keep this order in the schedule: the reads first, then the MFMAs that do not depend on them
                if constexpr (more_b) __builtin_amdgcn_sched_group_barrier(0x100, WT / G + (more_a ? WT : 0), 0);
                __builtin_amdgcn_sched_group_barrier(0x008, WT * WT, 0);
            });
        } else {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                V af[WT];
#pragma unroll
                for (int ti = 0; ti < WT; ++ti)
                    af[ti] = *reinterpret_cast<const V *>(cur + (h ? a_rd1 : a_rd0) + ti * 16 * APitch);
                if constexpr (kFragComb) {
                    if (comb_a) {
                        // left factor of T_4: xa * (A^2 fragment) + xb * (A fragment) + I; the lane holds row
                        // (wave's first row + 16 ti + lj) at the k values lg * KQ + h * VN + q of this k-block
#pragma unroll
                        for (int ti = 0; ti < WT; ++ti) {
                            const V ax = *reinterpret_cast<const V *>(cur + kXOff + (h ? a_rd1 : a_rd0) + ti * 16 * APitch);
                            const int row = row0 + wm * 16 * WT + 16 * ti + lj;
#pragma unroll
                            for (int q = 0; q < VN; ++q) {
                                T v = xa * reinterpret_cast<const T *>(&af[ti])[q] + xb * reinterpret_cast<const T *>(&ax)[q];
                                if (row == kb * BK + lg * S::KQ + h * VN + q) v += (T)1;
                                reinterpret_cast<T *>(&af[ti])[q] = v;
                            }
                        }
                    }
                }
#pragma unroll
                for (int q = 0; q < VN; ++q) {
                    const int kk = h * VN + q;
                    T bf[WT];
#pragma unroll
                    for (int g = 0; g < WT / G; ++g) {
                        const int off = b_rd + kk * BPitch + ((b_rc0 + g * 16 * G * (int)sizeof(T)) & (BPitch - 1));
                        GV x = *reinterpret_cast<const GV *>(cur + off);
                        if constexpr (kFragComb) {
                            if (!comb_a) {
                                // right factor of y02: xa * (W^2 fragment) + xb * (W fragment)
                                const GV xw = *reinterpret_cast<const GV *>(cur + kXOff - BM * APitch + off);
                                x = xa * x + xb * xw;
                            }
                        }
#pragma unroll
                        for (int e = 0; e < G; ++e) bf[g * G + e] = x[e];
                    }
#pragma unroll
                    for (int ti = 0; ti < WT; ++ti) {
                        const T a = reinterpret_cast<const T *>(&af[ti])[q];
#pragma unroll
                        for (int tj = 0; tj < WT; ++tj) acc[ti][tj] = Mfma<T>::run(a, bf[tj], acc[ti][tj]);
                    }
                }
            }
        }
    };
    auto kstep = [&](const unsigned char *cur, unsigned char *nxt, int kb) __attribute__((always_inline)) {
        const bool more = kb + 1 < kblocks;
        if (more) {
            const int k0 = (kb + 1) * BK;
            if constexpr (DMA) {
                dma(k0, nxt);
            } else {
#pragma unroll
                for (int i = 0; i < WT; ++i) {
                    ra[i] = load_vec<T, ALIGNED>(Lp, row0 + a_row0 + 32 * i, k0 + a_col, n);
                    rb[i] = load_vec<T, ALIGNED>(Rp, k0 + b_row0 + BSTEP * i, col0 + b_col, n);
                }
                fetch_x(k0);
            }
        }
        multiply(cur, kb);
        if constexpr (DMA) {
            dma_done();
        } else if (more) {
            combine((kb + 1) * BK);
#pragma unroll
            for (int i = 0; i < WT; ++i) {
                *reinterpret_cast<V *>(nxt + sg.left_write(i)) = ra[i];
                *reinterpret_cast<V *>(nxt + sg.right_write(i)) = rb[i];
            }
        }
        __syncthreads();
    };
    // Ring of four stages: k-blocks kb + 1 .. kb + 3 are in flight while k-block kb is multiplied.  A wave's loads
    // complete in the order it issued them, and the loop holds no other vector memory operation, so "at most two
    // k-blocks' loads of this wave outstanding" means that its part of k-block kb + 1 has landed; the barrier after
    // that wait publishes it to the other waves and also says that every wave has finished reading the stage the
    // next step's loads overwrite.  The waits are counted by hand and the barrier is the bare instruction, because
    // the fences of __syncthreads() wait for every outstanding load into LDS; the scheduling barriers around it keep
    // the LDS reads on their side.  The stages are separate LDS objects for the reason given above.
    constexpr int kGroup = (kFragComb ? 3 : 2) * WT;   // loads per thread and k-block
    auto ring_barrier = [&]() __attribute__((always_inline)) {
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
        __builtin_amdgcn_sched_barrier(0);
    };
    auto ring_step = [&](const unsigned char *cur, unsigned char *pre, int kb) __attribute__((always_inline)) {
        dma((kb + 3) * BK, pre);
        multiply(cur, kb);
        __builtin_amdgcn_s_waitcnt(0x0F70 | (2 * kGroup));   // vmcnt: two k-blocks may stay outstanding
        ring_barrier();
    };
    // the last (at most six) k-blocks: loads only while there is a k-block left to fetch, and full waits
    auto ring_tail = [&](const unsigned char *cur, unsigned char *pre, int kb) __attribute__((always_inline)) {
        if (kb >= kblocks) return;
        if (kb + 3 < kblocks) dma((kb + 3) * BK, pre);
        multiply(cur, kb);
        __builtin_amdgcn_s_waitcnt(0x0F70);
        ring_barrier();
    };
    if (ring) {
        if constexpr (kRing) {
            static_assert(2 * kGroup <= 15, "wait count fits the low bits of the immediate");
            dma(0, stage_even);
            dma(BK, stage_odd);
            dma(2 * BK, stage_2);
            __builtin_amdgcn_s_waitcnt(0x0F70 | (2 * kGroup));
            ring_barrier();
            int kb = 0;
            for (; kb + 6 < kblocks; kb += 4) {   // every step of these fetches a k-block
                ring_step(stage_even, stage_3, kb);
                ring_step(stage_odd, stage_even, kb + 1);
                ring_step(stage_2, stage_odd, kb + 2);
                ring_step(stage_3, stage_2, kb + 3);
            }
            ring_tail(stage_even, stage_3, kb);
            ring_tail(stage_odd, stage_even, kb + 1);
            ring_tail(stage_2, stage_odd, kb + 2);
            ring_tail(stage_3, stage_2, kb + 3);
            ring_tail(stage_even, stage_3, kb + 4);
            ring_tail(stage_odd, stage_even, kb + 5);
        }
    } else if constexpr (DMA) {
        int kb = 0;
        for (; kb + 1 < kblocks; kb += 2) {
            kstep(stage_even, stage_odd, kb);
            kstep(stage_odd, stage_even, kb + 1);
        }
        if (kb < kblocks) kstep(stage_even, stage_odd, kb);
    } else {
        for (int kb = 0; kb < kblocks; ++kb) kstep(smem + (kb & 1) * STAGE, smem + ((kb + 1) & 1) * STAGE, kb);
    }

    // ---- epilogue -----------------------------------------------------------------------------
    // lane holds C[row0 + wm*16*WT + 16*ti + Mfma<T>::row(lg, v)][col0 + wn*16*WT + (tj/G)*16*G + G*lj + tj%G]:
    // for every (ti, v) and every group of G tiles, G neighbouring elements of one row
    const int er = row0 + wm * 16 * WT;
    const int ec = col0 + wn * 16 * WT + G * lj;
    constexpr bool kVecIO = ALIGNED != kAccessScalar;  // rows are 16-byte aligned and n is a multiple of G
    if (st.nsrc == 0 && st.nout == 1) {
        T *D = reinterpret_cast<T *>(p.base[st.dst[0]]) + moff;
#pragma unroll
        for (int ti = 0; ti < WT; ++ti)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = er + 16 * ti + Mfma<T>::row(lg, v);
#pragma unroll
                for (int g = 0; g < WT / G; ++g) {
                    const int col = ec + g * 16 * G;
                    if constexpr (kVecIO) {
                        if (ALIGNED >= kAccessFull || (row < n && col < n)) {
                            GV o;
#pragma unroll
                            for (int e = 0; e < G; ++e) o[e] = acc[ti][g * G + e][v];
                            *reinterpret_cast<GV *>(D + (size_t)row * n + col) = o;
                        }
                    } else {
#pragma unroll
                        for (int e = 0; e < G; ++e)
                            if (row < n && col + e < n) D[(size_t)row * n + col + e] = acc[ti][g * G + e][v];
                    }
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
        // A lane holds 4 * WT rows of the tile ((ti, v) pairs).  The source vectors of a batch of rows are all fetched
        // before the first result of the batch is stored: the memory counter of a wave counts loads and stores
        // together and in order, so a load issued behind a store is waited for together with that store, and row by
        // row the epilogue was 4 * WT memory round trips one after another.  The batch is as many rows as fit 32
        // registers (more and the 64 x 64 fp64 kernel spills; the 128 x 128 kernels have none to spare and go row by row).
        constexpr int kRows = 4 * WT;
        constexpr int kRegsPerRow = (WT / G) * 4 * (int)sizeof(GV) / 4;
        constexpr int NB = WT == 4 ? 1 : (32 / kRegsPerRow < kRows ? 32 / kRegsPerRow : kRows);
        static_assert(kRows % NB == 0, "whole batches");
#pragma unroll
        for (int it0 = 0; it0 < kRows; it0 += NB) {
            GV sv[NB][WT / G][4];
#pragma unroll
            for (int q = 0; q < NB; ++q) {
                const int row = er + 16 * ((it0 + q) / 4) + Mfma<T>::row(lg, (it0 + q) % 4);
#pragma unroll
                for (int g = 0; g < WT / G; ++g) {
                    const int col = ec + g * 16 * G;
                    const size_t idx = (size_t)row * n + col;
                    if (kVecIO ? (ALIGNED >= kAccessFull || (row < n && col < n)) : row < n) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            if constexpr (kVecIO) {
                                sv[q][g][i] = i < st.nsrc ? *reinterpret_cast<const GV *>(S[i] + idx) : (GV)(0);
                            } else {
#pragma unroll
                                for (int e = 0; e < G; ++e) sv[q][g][i][e] = (i < st.nsrc && col + e < n) ? S[i][idx + e] : (T)0;
                            }
                        }
                    }
                }
            }
#pragma unroll
            for (int q = 0; q < NB; ++q) {
                const int ti = (it0 + q) / 4, v = (it0 + q) % 4;
                const int row = er + 16 * ti + Mfma<T>::row(lg, v);
#pragma unroll
                for (int g = 0; g < WT / G; ++g) {
                    const int col = ec + g * 16 * G;
                    const size_t idx = (size_t)row * n + col;
                    if (kVecIO ? (ALIGNED >= kAccessFull || (row < n && col < n)) : row < n) {
                        GV t;
#pragma unroll
                        for (int e = 0; e < G; ++e) t[e] = st.acc_scale * acc[ti][g * G + e][v];
#pragma unroll
                        for (int i = 0; i < 4; ++i) t += st.g[i] * sv[q][g][i];
                        GV dg;
#pragma unroll
                        for (int e = 0; e < G; ++e) dg[e] = row == col + e ? (T)1 : (T)0;
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            if (j < st.nout) {
                                GV o = st.a[j] * t;
#pragma unroll
                                for (int i = 0; i < 4; ++i) o += st.b[j][i] * sv[q][g][i];
                                o += st.d[j] * dg;
                                if constexpr (kVecIO) {
                                    *reinterpret_cast<GV *>(D[j] + idx) = o;
                                } else {
#pragma unroll
                                    for (int e = 0; e < G; ++e)
                                        if (col + e < n) D[j][idx + e] = o[e];
                                }
                            }
                        }
                    }
                }
            }
        }
    }

    // norm partials of the product just formed: the power rounds (W^2, W^3, W^4) and the term rounds of the baseline
    // (whose term Y = acc_scale * product decides whether the matrix goes on)
    const bool term_round = p.scheme == kSchemeBaseline && p.round >= 1 && p.round <= kBaselineSquareRound;
    const bool emit_norm = p.round <= 0 || term_round;
    const T nscale = term_round ? st.acc_scale : (T)1;
    if (emit_norm && !p.norm_inf) {
        // column abs-sums of this tile of the new power, in double: 16*WT rows per wave, then the two wave rows
        double *red = reinterpret_cast<double *>(smem);  // [2][BN]; the k-loop's last barrier has passed
#pragma unroll
        for (int tj = 0; tj < WT; ++tj) {
            double cs = 0.0;
#pragma unroll
            for (int ti = 0; ti < WT; ++ti)
#pragma unroll
                for (int v = 0; v < 4; ++v) cs += fabs((double)(nscale * acc[ti][tj][v]));
            cs += __shfl_xor(cs, 16);
            cs += __shfl_xor(cs, 32);
            if (lg == 0) red[wm * BN + wn * 16 * WT + (tj / G) * 16 * G + G * lj + tj % G] = cs;
        }
        __syncthreads();
        if (tid < BN) {
            const int col = col0 + tid;
            if (col < n) p.colpart[((size_t)b * p.tiles + tm) * n + col] = red[tid] + red[BN + tid];
        }
    } else if (emit_norm) {
        // row abs-sums of this tile (infinity-norm): 16*WT columns per wave, then the two wave columns;
        // partials are indexed by tile column: colpart[b][tn][row]
        double *red = reinterpret_cast<double *>(smem);  // [2][BM]
#pragma unroll
        for (int ti = 0; ti < WT; ++ti)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                double rs = 0.0;
#pragma unroll
                for (int tj = 0; tj < WT; ++tj) rs += fabs((double)(nscale * acc[ti][tj][v]));
                rs += __shfl_xor(rs, 1);
                rs += __shfl_xor(rs, 2);
                rs += __shfl_xor(rs, 4);
                rs += __shfl_xor(rs, 8);
                if (lj == 0) red[wn * BM + wm * 16 * WT + 16 * ti + Mfma<T>::row(lg, v)] = rs;
            }
        __syncthreads();
        if (tid < BM) {
            const int row = row0 + tid;
            if (row < n) p.colpart[((size_t)b * p.tiles + tn) * n + row] = red[tid] + red[BM + tid];
        }
    }
}

// ---- ||.||_1 helpers ----------------------------------------------------------------------------
// Column abs-sums of W over row chunks of kColChunk rows: colpart[b][chunk][col], accumulated in double.
template <typename T>
__global__ __launch_bounds__(256) void colabs_kernel(const T *__restrict__ W, double *__restrict__ colpart, int n, int chunks)
{
    const int col = blockIdx.x * 256 + threadIdx.x;
    const int chunk = blockIdx.y, b = blockIdx.z;
    if (col >= n) return;
    const T *p = W + (size_t)b * n * n + col;
    const int r0 = chunk * kColChunk, r1 = min(n, r0 + kColChunk);
    double s = 0.0;
#pragma unroll 8
    for (int r = r0; r < r1; ++r) s += fabs((double)p[(size_t)r * n]);
    colpart[((size_t)b * chunks + chunk) * n + col] = s;
}

// Row abs-sums of W (infinity-norm): one wave per row, lanes stride over the columns, fixed-order wave
// reduction; written as a single chunk colpart[b][0][row].
template <typename T>
__global__ __launch_bounds__(256) void rowabs_kernel(const T *__restrict__ W, double *__restrict__ colpart, int n)
{
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63, b = blockIdx.y;
    if (row >= n) return;
    const T *p = W + ((size_t)b * n + row) * n;
    double s = 0.0;
#pragma unroll 4
    for (int c = lane; c < n; c += 64) s += fabs((double)p[c]);
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
    if (lane == 0) colpart[(size_t)b * n + row] = s;
}

// pmax[b][blk] = max over the 256 columns of block blk of (sum over chunks of colpart[b][chunk][col]),
// chunks added in ascending order; NaN if any column sum is non-finite.
__global__ __launch_bounds__(256) void colmax_kernel(const double *__restrict__ colpart, double *__restrict__ pmax,
                                                     int n, int chunks, int nblk)
{
    __shared__ double smax[4];
    __shared__ int sbad[4];
    const int blk = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const int col = blk * 256 + tid;
    double s = 0.0;
    if (col < n) {
        const double *p = colpart + (size_t)b * chunks * n + col;
#pragma unroll 4
        for (int c = 0; c < chunks; ++c) s += p[(size_t)c * n];
    }
    int bad = !(s <= 1.7976931348623157e308);  // NaN or Inf
    for (int off = 32; off > 0; off >>= 1) {
        const double o = __shfl_xor(s, off);
        const int ob = __shfl_xor(bad, off);
        s = o > s ? o : s;
        bad |= ob;
    }
    if ((tid & 63) == 0) { smax[tid >> 6] = s; sbad[tid >> 6] = bad; }
    __syncthreads();
    if (tid == 0) {
        double mx = smax[0];
        int anybad = sbad[0];
        for (int w = 1; w < 4; ++w) {
            mx = smax[w] > mx ? smax[w] : mx;
            anybad |= sbad[w];
        }
        pmax[(size_t)b * nblk + blk] = anybad ? __longlong_as_double(0x7ff8000000000000LL) : mx;
    }
}

// ---- selection and plan ---------------------------------------------------------------------------
// One workgroup.  Reduces the per-block maxima to n1, n2, runs Algorithm 4, writes info[b], the order
// (longest chain first) and the summary:
//   summary[0] = longest chain, summary[1] = OR of flags, summary[2 + r] = matrices active in round r.
__global__ __launch_bounds__(1024) void select_plan_kernel(const double *__restrict__ p1, const double *__restrict__ p2,
                                                           const double *__restrict__ p3, const double *__restrict__ p4,
                                                           int nblk, MatInfo *__restrict__ info, int *__restrict__ order,
                                                           int *__restrict__ summary, int batch, double eps, int scheme)
{
    __shared__ int hist[kMaxRounds + 1];
    __shared__ int cursor[kMaxRounds + 1];
    __shared__ int flags_or;
    const int tid = threadIdx.x;
    if (tid <= kMaxRounds) hist[tid] = 0;
    if (tid == 0) flags_or = 0;
    __syncthreads();
    for (int b = tid; b < batch; b += blockDim.x) {
        double nrm[4] = {0.0, 0.0, 0.0, 0.0};
        bool bad = false;
        const int used = scheme == kSchemePS ? 4 : (scheme == kSchemePhi ? 1 : 2);
        for (int q = 0; q < used; ++q) {
            const double *pq = q == 0 ? p1 : (q == 1 ? p2 : (q == 2 ? p3 : p4));
            for (int k = 0; k < nblk; ++k) {
                const double x = pq[(size_t)b * nblk + k];
                if (!(x == x)) bad = true;
                nrm[q] = x > nrm[q] ? x : nrm[q];
            }
        }
        if (bad) nrm[0] = __longlong_as_double(0x7ff8000000000000LL);
        MatInfo mi;
        if (scheme == kSchemePS) {
            bool need_more;
            select_ps_order_scaling(nrm, 4, eps, mi.m, mi.s, mi.flags, need_more);
            mi.len = chain_length_ps(mi.m, mi.s);
        } else if (scheme == kSchemePhi) {
            // core series of the low-rank variant: the order follows from the norm alone, no scaling
            select_lowrank_order(nrm[0], eps, mi.m, mi.flags);
            mi.s = mi.m < 0 ? -1 : 0;
            mi.len = mi.m < 0 ? 0 : chain_length_ps(mi.m, 0);
        } else {
            select_order_scaling(nrm[0], nrm[1], eps, mi.m, mi.s, mi.flags);
            mi.len = chain_length(mi.m, mi.s);
        }
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
    // Stable placement (matrices of one chain length keep their input order, so that the plan and with it every
    // launch's work list is the same from run to run): chunks of blockDim matrices in ascending order; inside a
    // chunk a matrix's rank among those of its length comes from wave ballots and per-wave counts.
    __shared__ int wave_count[16][kMaxRounds + 1];
    const int lane = tid & 63, wave = tid >> 6, waves = blockDim.x >> 6;
    for (int base = 0; base < batch; base += blockDim.x) {
        const int b = base + tid;
        const int len = b < batch ? info[b].len : -1;
        int my_rank = 0;
        for (int L = 0; L <= kMaxRounds; ++L) {
            const unsigned long long mask = __ballot(len == L);
            if (len == L) my_rank = __popcll(mask & ((1ull << lane) - 1ull));
            if (lane == 0) wave_count[wave][L] = __popcll(mask);
        }
        __syncthreads();
        if (len >= 0) {
            int pos = cursor[len] + my_rank;
            for (int w = 0; w < wave; ++w) pos += wave_count[w][len];
            order[pos] = b;
        }
        __syncthreads();
        if (tid <= kMaxRounds) {
            int add = 0;
            for (int w = 0; w < waves; ++w) add += wave_count[w][tid];
            cursor[tid] += add;
        }
        __syncthreads();
    }
}

// ---- baseline (Algorithm 1): who is still in the term loop ------------------------------------------------------
// One workgroup.  term = 0: from ||W|| (per-block maxima in p1) the scaling s = smallest s >= 0 with ||W|| / 2^s < 1/2
// and whether the first term A = W / 2^s exceeds the tolerance; summary[0] = largest s, summary[1] = OR of flags.
// term = t >= 1: from the norm of the term Y_(t+1) that round t formed (maxima in p2) whether the matrix goes on.
__global__ __launch_bounds__(1024) void baseline_decide_kernel(const double *__restrict__ p1, const double *__restrict__ p2,
                                                               int nblk, MatInfo *__restrict__ info, int *__restrict__ summary,
                                                               int batch, double eps, int term)
{
    __shared__ int smax, flags_or;
    const int tid = threadIdx.x;
    if (tid == 0) { smax = 0; flags_or = 0; }
    __syncthreads();
    for (int b = tid; b < batch; b += blockDim.x) {
        const double *pq = (term == 0 ? p1 : p2) + (size_t)b * nblk;
        double nrm = 0.0;
        bool bad = false;
        for (int k = 0; k < nblk; ++k) {
            const double x = pq[k];
            if (!(x <= 1.7976931348623157e308)) bad = true;
            nrm = x > nrm ? x : nrm;
        }
        if (term == 0) {
            MatInfo mi;
            mi.m = 0; mi.s = 0; mi.len = 0; mi.flags = 0;
            if (bad) {
                mi.m = -1; mi.s = -1; mi.flags = 1;
            } else {
                double t = nrm;
                while (!(t < 0.5)) { t *= 0.5; ++mi.s; }   // exact halvings: t = ||W|| / 2^s
                if (t > eps) { mi.m = 1; mi.len = 1; }
            }
            info[b] = mi;
            atomicMax(&smax, mi.s);
            if (mi.flags) atomicOr(&flags_or, mi.flags);
        } else {
            MatInfo mi = info[b];
            if (mi.len) {
                if (!bad && nrm > eps) mi.m = term + 1;
                else mi.len = 0;
                info[b] = mi;
            }
        }
    }
    __syncthreads();
    if (term == 0 && tid == 0) {
        summary[0] = smax;
        summary[1] = flags_or;
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
    const int shift = p.scheme == kSchemePhi ? 1 : 0;   // coefficients 1/(i+1)! instead of 1/i!
    if (shift && mi.m >= 0 && mi.m <= 2) {
        // core series of the low-rank variant, orders without a further product: I, I + V/2, I + V/2 + V^2/6
        for (int e = 0; e < 4; ++e) {
            const size_t idx = ((size_t)blockIdx.x * 4 + e) * 256 + threadIdx.x;
            if (idx >= nn) break;
            const int row = (int)(idx / n), col = (int)(idx - (size_t)row * n);
            T o = row == col ? (T)1 : (T)0;
            if (mi.m >= 1) o += W[idx] / (T)2;
            if (mi.m == 2) o += W2[idx] / (T)6;
            O[idx] = o;
        }
        return;
    }
    if ((p.scheme == kSchemePS || shift) && mi.m >= 4) {
        // top block of the Paterson-Stockmeyer form: H0 = sum_{r=0..j} c_{(k-1)j+r} A^r  ->  T0
        const T *W3 = reinterpret_cast<const T *>(p.base[BUF_W3]) + moff;
        const T *W4 = reinterpret_cast<const T *>(p.base[BUF_W4]) + moff;
        const int j = ps_j(mi.m), base = (ps_k(mi.m) - 1) * j + shift;
        const T h0 = (T)inv_factorial(base), h1 = (T)(inv_factorial(base + 1) * sg),
                h2 = (T)(inv_factorial(base + 2) * sg2), h3 = j >= 3 ? (T)(inv_factorial(base + 3) * sg2 * sg) : (T)0,
                h4 = j >= 4 ? (T)(inv_factorial(base + 4) * sg2 * sg2) : (T)0;
        for (int e = 0; e < 4; ++e) {
            const size_t idx = ((size_t)blockIdx.x * 4 + e) * 256 + threadIdx.x;
            if (idx >= nn) break;
            const int row = (int)(idx / n), col = (int)(idx - (size_t)row * n);
            T h = h1 * W[idx] + h2 * W2[idx] + (row == col ? h0 : (T)0);
            if (j >= 3) h += h3 * W3[idx];
            if (j >= 4) h += h4 * W4[idx];
            T0[idx] = h;
        }
        return;
    }
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

template <typename T, int WT, int ALIGNED, bool FIRST = false>
hipError_t launch_gemm_t(const GemmParams &p, hipStream_t stream)
{
    // the direct-to-LDS variants hold their stages (two, or the four of the 32x32 tiles' ring) in static LDS (at most
    // 64 KB); the others in dynamic LDS
    if constexpr (ALIGNED == kAccessDma) {
        static_assert((WT == 1 ? 4 : 2) * (stage_bytes<T, WT>(true) + (FIRST ? 32 * WT * 128 : 0)) <= 65536,
                      "static LDS of the direct-to-LDS variants");
        hipLaunchKernelGGL((gemm_round_kernel<T, WT, ALIGNED, FIRST>), dim3(p.total), dim3(kThreads), 0, stream, p);
        return hipGetLastError();
    }
    static PerDeviceOnce lds_limit;
    const int lds = 2 * stage_bytes<T, WT>(ALIGNED == kAccessDma);
    hipError_t e = lds_limit([] {
        return hipFuncSetAttribute(reinterpret_cast<const void *>(gemm_round_kernel<T, WT, ALIGNED, FIRST>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    });
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((gemm_round_kernel<T, WT, ALIGNED, FIRST>), dim3(p.total), dim3(kThreads), lds, stream, p);
    return hipGetLastError();
}

GemmParams make_params(const GeneralBuffers &gb, int n, int round, int matrices, int wt, int scheme)
{
    GemmParams p;
    p.scheme = scheme;
    p.norm_inf = gb.norm_inf;
    for (int i = 0; i < BUF_COUNT; ++i) p.base[i] = gb.base[i];
    p.info = gb.info;
    p.order = gb.order;
    p.colpart = gb.colpart;
    p.n = n;
    p.tiles = (n + 32 * wt - 1) / (32 * wt);
    p.round = round;
    p.total = matrices * p.tiles * p.tiles;
    p.slot0 = 0;
    p.slot_step = 1;
    p.active = nullptr;
    p.keep = 0;
    return p;
}

template <typename T, int WT>
hipError_t launch_gemm_a(const GemmParams &p, bool aligned, hipStream_t stream)
{
    // Full tiles and 16-byte aligned rows: operands go straight from global memory into LDS.  Measured against the
    // register-staged kernels: 4096x4096 fp64 products 6.5 % faster (the 128x128 fp64 kernel no longer spills),
    // fp32 1.7 %, 512x512 fp64 (64x64 tiles) 0.7 %.
    if (aligned && p.n % (32 * WT) == 0 && p.n % Tile<T>::BK == 0) return launch_gemm_t<T, WT, kAccessDma>(p, stream);
    return aligned ? launch_gemm_t<T, WT, kAccessVector>(p, stream) : launch_gemm_t<T, WT, kAccessScalar>(p, stream);
}

hipError_t launch_gemm(const GemmParams &p, int dtype, int wt, bool ptr_align16, hipStream_t stream)
{
    if (p.total <= 0) return hipSuccess;
    if (dtype == 1) {
        const bool al = ptr_align16 && p.n % 2 == 0;
        if (wt == 1) return launch_gemm_a<double, 1>(p, al, stream);
        return wt == 4 ? launch_gemm_a<double, 4>(p, al, stream) : launch_gemm_a<double, 2>(p, al, stream);
    }
    const bool al = ptr_align16 && p.n % 4 == 0;
    if (wt == 1) return launch_gemm_a<float, 1>(p, al, stream);
    return wt == 4 ? launch_gemm_a<float, 4>(p, al, stream) : launch_gemm_a<float, 2>(p, al, stream);
}

// chain round 1 with the operands formed on the fly (64x64 tiles, or 32x32 for thin launches)
template <typename T, int WT>
hipError_t launch_gemm_first(const GemmParams &p, bool aligned, hipStream_t stream)
{
    if (aligned && p.n % (32 * WT) == 0 && p.n % Tile<T>::BK == 0) return launch_gemm_t<T, WT, kAccessDma, true>(p, stream);
    return aligned ? launch_gemm_t<T, WT, kAccessVector, true>(p, stream) : launch_gemm_t<T, WT, kAccessScalar, true>(p, stream);
}

}  // namespace

// True when chain round 1 forms its operands itself and no preparation pass is needed: the main scheme on
// matrices below 1024, which always run on 64x64 tiles.  (Above, the pass is half a percent of a call and the
// register-bound 128x128 kernels have no room for the extra vectors.)
bool first_round_is_self_contained(int n, int scheme)
{
    return scheme == kSchemeSastre && n < 1024;  // the sizes whose first round (whole batch) runs in 64x64 tiles
}

hipError_t launch_first_round(const GeneralBuffers &gb, int n, int batch, int dtype, hipStream_t stream)
{
    const int wt = choose_tile_shape(n, batch) == 1 ? 1 : 2;
    const GemmParams p = make_params(gb, n, 1, batch, wt, kSchemeSastre);
    if (p.total <= 0) return hipSuccess;
    if (dtype == 1) {
        const bool al = gb.ptr_align16 && n % 2 == 0;
        return wt == 1 ? launch_gemm_first<double, 1>(p, al, stream) : launch_gemm_first<double, 2>(p, al, stream);
    }
    const bool al = gb.ptr_align16 && n % 4 == 0;
    return wt == 1 ? launch_gemm_first<float, 1>(p, al, stream) : launch_gemm_first<float, 2>(p, al, stream);
}

// Tile shape for a round with `matrices` active matrices of order n: 128x128 tiles (WT = 4) for large
// matrices unless they would leave compute units idle or poorly balanced, 64x64 tiles (WT = 2) otherwise,
// 32x32 tiles (WT = 1) for thin launches.
// Cost model for n >= 1024, in units of one 128x128 tile on one compute unit: a compute unit works
// through its tiles one after another (co-resident tiles share the matrix pipe); a 64x64 tile costs a
// quarter of the work at roughly 0.9 of the efficiency.
int choose_tile_shape(int n, int matrices)
{
    // debugging aid: EXPM_FORCE_WT=1|2|4 pins the shape (read once)
    static const int forced = [] {
        const char *e = getenv("EXPM_FORCE_WT");
        const int v = e ? atoi(e) : 0;
        return (v == 1 || v == 2 || v == 4) ? v : 0;
    }();
    if (forced) return forced;
    // Thin launches (late rounds with few matrices left, small batches): a compute unit that holds a single workgroup
    // runs one wave per SIMD and nothing covers its latencies; a smaller tile gives four times the workgroups.
    const long long t2 = (long long)matrices * ((n + 63) / 64) * ((n + 63) / 64);
    if (t2 <= kThinGroups) return 1;
    // Measured on MI355X: up to n of several hundred the 64x64 shape is as fast per product and, with
    // four workgroups per compute unit out of phase, hides the fused epilogues' memory traffic better.
    if (n < 1024) return 2;
    const long long cus = 256;
    const long long t4 = (long long)matrices * ((n + 127) / 128) * ((n + 127) / 128);
    if (t4 < 2 * cus) return 2;  // fewer than two 128x128 workgroups per compute unit: the same, one size up
    const double cost4 = (double)((t4 + cus - 1) / cus);
    const double cost2 = (double)((t2 + cus - 1) / cus) * 0.25 / 0.9;
    return cost2 < cost4 ? 2 : 4;
}

int general_colchunks(int n) { return (n + kColChunk - 1) / kColChunk; }
int general_colblocks(int n) { return (n + 255) / 256; }

hipError_t launch_colabs(const GeneralBuffers &gb, int n, int batch, int dtype, hipStream_t stream)
{
    if (gb.norm_inf) {
        dim3 grid((n + 3) / 4, batch);
        if (dtype == 1)
            hipLaunchKernelGGL(rowabs_kernel<double>, grid, dim3(256), 0, stream,
                               reinterpret_cast<const double *>(gb.base[BUF_W]), gb.colpart_w, n);
        else
            hipLaunchKernelGGL(rowabs_kernel<float>, grid, dim3(256), 0, stream,
                               reinterpret_cast<const float *>(gb.base[BUF_W]), gb.colpart_w, n);
        return hipGetLastError();
    }
    const int chunks = general_colchunks(n);
    dim3 grid((n + 255) / 256, chunks, batch);
    if (dtype == 1)
        hipLaunchKernelGGL(colabs_kernel<double>, grid, dim3(256), 0, stream,
                           reinterpret_cast<const double *>(gb.base[BUF_W]), gb.colpart_w, n, chunks);
    else
        hipLaunchKernelGGL(colabs_kernel<float>, grid, dim3(256), 0, stream,
                           reinterpret_cast<const float *>(gb.base[BUF_W]), gb.colpart_w, n, chunks);
    return hipGetLastError();
}

hipError_t launch_colmax(const GeneralBuffers &gb, int n, int batch, int which, int chunks, hipStream_t stream)
{
    const int nblk = general_colblocks(n);
    double *dst = which == 1 ? gb.n1 : (which == 2 ? gb.n2 : (which == 3 ? gb.n3 : gb.n4));
    hipLaunchKernelGGL(colmax_kernel, dim3(nblk, batch), dim3(256), 0, stream, which == 1 ? gb.colpart_w : gb.colpart, dst, n,
                       chunks, nblk);
    return hipGetLastError();
}

// power round `which` = 2, 3, 4: W^which = W^(which-1) * W with the column abs-sums of the result
hipError_t launch_power_round(const GeneralBuffers &gb, int n, int batch, int dtype, int wt, int which, hipStream_t stream)
{
    return launch_gemm(make_params(gb, n, 2 - which, batch, wt, kSchemeSastre), dtype, wt, gb.ptr_align16, stream);
}

hipError_t launch_select_plan(const GeneralBuffers &gb, int n, int batch, double eps, int scheme, hipStream_t stream)
{
    hipLaunchKernelGGL(select_plan_kernel, dim3(1), dim3(1024), 0, stream, gb.n1, gb.n2, gb.n3, gb.n4,
                       general_colblocks(n), gb.info, gb.order, gb.summary, batch, eps, scheme);
    return hipGetLastError();
}

hipError_t launch_prepare(const GeneralBuffers &gb, int n, int batch, int dtype, int scheme, hipStream_t stream)
{
    const GemmParams p = make_params(gb, n, 0, batch, 4, scheme);
    const size_t nn = (size_t)n * n;
    dim3 grid((unsigned)((nn + 1023) / 1024), batch);
    if (dtype == 1)
        hipLaunchKernelGGL(prepare_kernel<double>, grid, dim3(256), 0, stream, p);
    else
        hipLaunchKernelGGL(prepare_kernel<float>, grid, dim3(256), 0, stream, p);
    return hipGetLastError();
}

// `active` matrices of the sorted list, starting at `first` and `step` apart (1: a contiguous range)
hipError_t launch_chain_round(const GeneralBuffers &gb, int n, int active, int round, int dtype, int wt, int scheme,
                              hipStream_t stream, int first, int step, bool device_plan)
{
    GemmParams p = make_params(gb, n, round, active, wt, scheme);
    p.slot0 = first;
    p.slot_step = step;
    if (device_plan) p.active = gb.summary + 2;   // `active` is then the whole batch
    return launch_gemm(p, dtype, wt, gb.ptr_align16, stream);
}

// Round of the baseline (Algorithm 1) over the whole batch: term round `round` >= 1, or squaring
// round - kBaselineSquareRound; workgroups of matrices that do not take part leave at once.
hipError_t launch_baseline_round(const GeneralBuffers &gb, int n, int batch, int round, int dtype, int wt,
                                 bool keep_in_workspace, hipStream_t stream)
{
    GemmParams p = make_params(gb, n, round, batch, wt, kSchemeBaseline);
    p.keep = keep_in_workspace ? 1 : 0;
    return launch_gemm(p, dtype, wt, gb.ptr_align16, stream);
}

hipError_t launch_baseline_decide(const GeneralBuffers &gb, int n, int batch, double eps, int term, hipStream_t stream)
{
    hipLaunchKernelGGL(baseline_decide_kernel, dim3(1), dim3(1024), 0, stream, gb.n1, gb.n2, general_colblocks(n), gb.info,
                       gb.summary, batch, eps, term);
    return hipGetLastError();
}

}  // namespace expmk
