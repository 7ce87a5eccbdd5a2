// Fused single-kernel path for matrices that fit one compute unit's LDS, gfx950.
//
// One workgroup per matrix.  The matrix is read once, every step of Algorithm 2 and Algorithm 4
// (Sec. 3.3 of arXiv 2512.20777) runs on chip -- ||W||_1, W^2 and its norm, the choice of (m, s),
// the evaluation formulas of Sec. 3.1, the s squarings -- and the result is written once.
// (m, s) is uniform over the workgroup, so no wavefront diverges and nothing has to be bucketed.
//
// Layout on chip: two LDS buffers hold the current left and right operand of a product; everything that
// is only combined element-wise (A, A^2, y02, the additive part) lives in registers of the lane that owns
// the element in the MFMA result layout.  Products are 16x16 tiles of MFMA 16x16x4 in the matrix dtype on
// the zero-padded matrix; 1 wave for n <= 16, otherwise 2x2 waves, each owning a TH x TH block of tiles.
//
// fp32: the left operand is kept row-major and the right operand transposed, so that on both sides a lane
// fetches four consecutive k of its row or column with one 16-byte read (lane group g takes k = 16G + 4g + q
// in step q of group G); with a pitch of 4*odd words these reads, the 16-byte stores of a result tile into
// the transposed buffer and its 4-byte stores into the row-major buffer are all free of bank conflicts.
// Every wave computes its full block of tiles; the buffers are padded to 2*TH tiles per side.
// fp64: one 8-byte read per fragment, each buffer with the pitch that keeps its side conflict free.
#include "expm_internal.h"

namespace expmk {

namespace {

template <typename T, int NT> struct FusedCfg {
    static constexpr int NP = 16 * NT;
    static constexpr int WG = NT == 1 ? 1 : 2;          // waves per dimension
    static constexpr int TH = (NT + WG - 1) / WG;       // tiles per wave per dimension
    static constexpr int kThreads = 64 * WG * WG;
    static constexpr bool kF32 = sizeof(T) == 4;
    static constexpr bool kWide = kF32;                  // 16-byte fragment reads, right operand transposed
    static constexpr int NPP = 16 * WG * TH;             // rows and columns covered by the waves' tile blocks
    static constexpr int kRows = kWide ? NPP : NP;
    // fp64 left operand: 16 lanes read 16 consecutive rows at one k -> pitch = 2*odd words
    static constexpr int LPA = kWide ? NPP + 4 : NP + 2;
    // fp64 right operand: the four 16-lane groups read four k rows -> pitch = 16*odd elements
    static constexpr int LPB = kWide ? NPP + 4 : (NT % 2 == 0 ? NP + 16 : NP);
    static constexpr int kBytesP = kRows * LPA * (int)sizeof(T);
    static constexpr int kBytesQ = kRows * LPB * (int)sizeof(T);
    // Single-wave matrices are packed four to a workgroup (one wave each, nothing shared between them):
    // fewer, larger workgroups start faster than four times as many one-wave ones.
    static constexpr int kMPW = NT == 1 ? 4 : 1;
    static constexpr int kBlock = kThreads * kMPW;
    static constexpr int kLdsPer = kBytesP + kBytesQ + (kThreads + 16) * (int)sizeof(double);
    static constexpr int kLds = kLdsPer * kMPW;
    static_assert(kLdsPer % 16 == 0 && kLds <= 163840, "fused path exceeds the LDS of one compute unit");
};

template <typename T> struct VecOf;
template <> struct VecOf<float> { using type = float4; };
template <> struct VecOf<double> { using type = double2; };

// x of the lane that the DPP control CTRL pairs with this one (within rows of 16 lanes)
template <int CTRL> __device__ __forceinline__ double dpp_move(double x)
{
    // every lane is written (row and bank masks all ones, every source lane of these controls exists), so no
    // previous value has to be set up for the destination: the form without one saves two moves per call
    const int lo = __builtin_amdgcn_mov_dpp(__double2loint(x), CTRL, 0xf, 0xf, true);
    const int hi = __builtin_amdgcn_mov_dpp(__double2hiint(x), CTRL, 0xf, 0xf, true);
    return __hiloint2double(hi, lo);
}
// Reduction over the 16 lanes of a row, result in every lane: mirror the row, mirror its halves, then
// swap pairs of pairs and pairs -- four steps that each join two disjoint sets of lanes.
template <typename Op> __device__ __forceinline__ double row16_allreduce(double x, Op op)
{
    x = op(x, dpp_move<0x140>(x));  // row_mirror
    x = op(x, dpp_move<0x141>(x));  // row_half_mirror
    x = op(x, dpp_move<0x4e>(x));   // quad_perm [2,3,0,1]
    x = op(x, dpp_move<0xb1>(x));   // quad_perm [1,0,3,2]
    return x;
}

__device__ __forceinline__ double pow2neg_f(int e)
{
    return __longlong_as_double((long long)(1023 - e) << 52);
}

// FULL: n = 16 NT exactly and 16-byte aligned pointers (the launcher checks): the size is a compile-time constant, so
// the zero padding, the bounds of the load and store loops and their predicates fold away.
template <typename T, int NT, int SCHEME, bool FULL = false>
__global__ __launch_bounds__(256) void fused_expm_kernel(const T *__restrict__ Ain, T *__restrict__ Out, int n_arg, int batch,
                                                         double eps, int select_only, int norm_inf,
                                                         MatInfo *__restrict__ info)
{
    using C = FusedCfg<T, NT>;
    const int n = FULL ? C::NP : n_arg;
    using acc_t = typename Mfma<T>::acc_t;
    constexpr int NP = C::NP, LPA = C::LPA, LPB = C::LPB, TH = C::TH, WG = C::WG, NR = C::kRows;
    constexpr bool kWide = C::kWide;
    extern __shared__ __align__(16) unsigned char smem_all[];
    // matrix of this wave (packed single-wave case) or of this workgroup
    const int slot = C::kMPW > 1 ? __builtin_amdgcn_readfirstlane(threadIdx.x >> 6) : 0;
    const int b = blockIdx.x * C::kMPW + slot;
    if (b >= batch) return;  // a whole wave of a packed workgroup; those synchronise per wave only (sync below)
    unsigned char *smem_raw = smem_all + slot * C::kLdsPer;
    T *P = reinterpret_cast<T *>(smem_raw);                         // left operand layout
    T *Q = reinterpret_cast<T *>(smem_raw + C::kBytesP);            // right operand layout
    double *red = reinterpret_cast<double *>(smem_raw + C::kBytesP + C::kBytesQ);
    // Barrier between the phases of one matrix.  A single wave runs its LDS instructions in order, so it
    // only has to keep the compiler from moving accesses across this point.
    auto sync = [&]() {
        if constexpr (NT == 1) {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        } else {
            __syncthreads();
        }
    };

    __builtin_assume(n >= 1 && n <= NP);  // the launcher picks NT = ceil(n / 16); lets the copy loops below fold for small NT
    const int tid = C::kMPW > 1 ? (int)(threadIdx.x & 63) : (int)threadIdx.x, lane = tid & 63;
    const int wave = C::kMPW > 1 ? 0 : __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, in a scalar register
    const int wr = wave / WG, wc = wave % WG;
    constexpr bool kAllTiles = kWide || NT % WG == 0;  // every wave computes a full TH x TH block
    auto row_ok = [&](int ti) -> bool { return kAllTiles || wr * TH + ti < NT; };
    auto col_ok = [&](int tj) -> bool { return kAllTiles || wc * TH + tj < NT; };
    const int lj = lane & 15, lg = lane >> 4;
    const size_t moff = (size_t)b * n * n;
    const T *W = Ain + moff;
    // position of element (r, c) in the left-operand buffer P and in the right-operand buffer Q
    auto li = [&](int r, int c) -> int { return r * LPA + c; };
    auto ri = [&](int r, int c) -> int { return kWide ? c * LPB + r : r * LPB + c; };

    // ---- load W into both operand layouts, zero padded -------------------------------------------
    constexpr int VN = 16 / (int)sizeof(T);  // elements per 16-byte vector
    const bool vec_ok = FULL || ((n % VN == 0) && ((reinterpret_cast<uintptr_t>(Ain) | reinterpret_cast<uintptr_t>(Out)) % 16 == 0));
    if (n < NR) {
        for (int e = tid; e < NR * NR; e += C::kThreads) {
            const int r = e / NR, c = e - r * NR;
            if (r >= n || c >= n) {
                P[li(r, c)] = (T)0;
                if constexpr (!kWide) Q[ri(r, c)] = (T)0;
            }
        }
    }
    // (the transposed copy of the fp32 path is written further down, from registers)
    // Threads walk the padded rows (a compile-time width, so no division by n); columns past n are skipped.
    constexpr int CV = NR / VN;
    if (vec_ok) {
        using V = typename VecOf<T>::type;
#pragma unroll(NT >= 4 ? 16 : (NT >= 2 ? 4 : 1))  // all of a thread's loads in flight at once
        for (int e = tid; e < n * CV; e += C::kThreads) {
            const int r = e / CV, c = (e - r * CV) * VN;
            if (c < n) {
                const V x = *reinterpret_cast<const V *>(W + (size_t)r * n + c);
                *reinterpret_cast<V *>(P + li(r, c)) = x;
                if constexpr (!kWide) *reinterpret_cast<V *>(Q + ri(r, c)) = x;
            }
        }
    } else {
#pragma unroll 4
        for (int e = tid; e < n * NR; e += C::kThreads) {
            const int r = e / NR, c = e - r * NR;
            if (c < n) {
                const T x = W[(size_t)r * n + c];
                P[li(r, c)] = x;
                if constexpr (!kWide) Q[ri(r, c)] = x;
            }
        }
    }
    sync();

    // ---- norm of a matrix held in registers in the result layout, get(ti, tj, v) -> element: max column
    // abs-sum (1-norm) or, with norm_inf, max row abs-sum; sums in double, NaN if not finite.  Each wave adds
    // up its part of every line (column or row) with lane shuffles, the parts meet in LDS, and every wave
    // then takes the maximum over all lines itself, so that all lanes return the same bits.
    auto norm_regs = [&](auto &&get) -> double {
        constexpr int L = 16 * WG * TH;  // lines covered by the waves' tile blocks
        auto add = [](double a, double b2) { return a + b2; };
        auto mxop = [](double a, double b2) { return b2 > a ? b2 : a; };
        if constexpr (NT == 1) {
            // one wave, one tile: the shuffles alone finish the sums, nothing goes through LDS
            double line;
            if (!norm_inf) {
                line = 0.0;
#pragma unroll
                for (int v = 0; v < 4; ++v) line += fabs((double)get(0, 0, v));
                line += __shfl_xor(line, 16);
                line += __shfl_xor(line, 32);  // column lj, complete in every lane
            } else {
                double rs[4];
#pragma unroll
                for (int v = 0; v < 4; ++v) rs[v] = row16_allreduce(fabs((double)get(0, 0, v)), add);
                const int bad4 = !(rs[0] + rs[1] + rs[2] + rs[3] <= 1.7976931348623157e308);
                line = mxop(mxop(rs[0], rs[1]), mxop(rs[2], rs[3]));
                if (bad4) line = __longlong_as_double(0x7ff8000000000000LL);
            }
            const int bad = !(line <= 1.7976931348623157e308);
            double mx = bad ? 0.0 : line;
            if (!norm_inf) {
                // a column sum is the same in all four 16-lane groups: the maximum over one group is the norm
                mx = row16_allreduce(mx, mxop);
            } else {
                // a lane's maximum over its four rows is the same in all lanes of a group: combine the four groups
                mx = mxop(mx, __shfl_xor(mx, 16));
                mx = mxop(mx, __shfl_xor(mx, 32));
            }
            return __any(bad) ? __longlong_as_double(0x7ff8000000000000LL) : mx;
        }
        sync();  // red[] free to overwrite
        if (!norm_inf) {
#pragma unroll
            for (int tj = 0; tj < TH; ++tj) {
                double sum = 0.0;
#pragma unroll
                for (int ti = 0; ti < TH; ++ti)
                    if (row_ok(ti) && col_ok(tj)) {
#pragma unroll
                        for (int v = 0; v < 4; ++v) sum += fabs((double)get(ti, tj, v));
                    }
                sum += __shfl_xor(sum, 16);
                sum += __shfl_xor(sum, 32);
                if (lg == 0) red[wr * L + 16 * (wc * TH + tj) + lj] = sum;
            }
        } else {
#pragma unroll
            for (int ti = 0; ti < TH; ++ti)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    double sum = 0.0;
#pragma unroll
                    for (int tj = 0; tj < TH; ++tj)
                        if (row_ok(ti) && col_ok(tj)) sum += fabs((double)get(ti, tj, v));
                    sum = row16_allreduce(sum, add);
                    if (lj == 0) red[wc * L + 16 * (wr * TH + ti) + Mfma<T>::row(lg, v)] = sum;
                }
        }
        sync();
        double mx = 0.0;
        int bad = 0;
        for (int line = lane; line < L; line += 64) {
            double t = red[line];
            if (WG == 2) t += red[L + line];
            bad |= !(t <= 1.7976931348623157e308);
            mx = t > mx ? t : mx;
        }
        mx = row16_allreduce(mx, mxop);
        mx = mxop(mx, __shfl_xor(mx, 16));
        mx = mxop(mx, __shfl_xor(mx, 32));
        return __any(bad) ? __longlong_as_double(0x7ff8000000000000LL) : mx;
    };

    // ---- acc = L * R on this wave's block of tiles; L in left-operand layout, R in right-operand layout ----
    // Fragments of the next step are in flight while this one multiplies.  A prefetch past the end wraps to
    // step 0 (read, not used) so that the loop body has no branch and every wait is exact.
    acc_t acc[TH][TH];
    auto product = [&](const T *Lb, const T *Rb) {
        if constexpr (kWide) {
            // One group = four k-steps = one 16-byte fragment per tile row and per tile column.
            using V = typename VecOf<T>::type;
            constexpr int NG = NP / 16;
            const T *lp = Lb + (16 * (wr * TH) + lj) * LPA + 4 * lg;
            const T *rp = Rb + (16 * (wc * TH) + lj) * LPB + 4 * lg;
            V a0[TH], b0[TH], a1[TH], b1[TH];
            auto fetch = [&](V *a, V *bq, int g) {
#pragma unroll
                for (int t = 0; t < TH; ++t) a[t] = *reinterpret_cast<const V *>(lp + t * 16 * LPA + 16 * g);
#pragma unroll
                for (int t = 0; t < TH; ++t) bq[t] = *reinterpret_cast<const V *>(rp + t * 16 * LPB + 16 * g);
            };
            // 4*TH*TH MFMAs; the 2*TH fragment reads issued just before are spread between the first of them,
            // one read per TH MFMAs: a lone wave per SIMD loses matrix-core cycles to every other instruction
            // it has to issue in a row.
            auto fma_group = [&](const V *a, const V *bq, bool first, bool spread) {
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int ti = 0; ti < TH; ++ti)
#pragma unroll
                        for (int tj = 0; tj < TH; ++tj) {
                            const T av_ = reinterpret_cast<const T *>(&a[ti])[q], bv_ = reinterpret_cast<const T *>(&bq[tj])[q];
                            acc[ti][tj] = (first && q == 0) ? Mfma<T>::run(av_, bv_, (acc_t)(0))
                                                            : Mfma<T>::run(av_, bv_, acc[ti][tj]);
                        }
                if (spread) {
#pragma unroll
                    for (int i = 0; i < 2 * TH; ++i) {
                        __builtin_amdgcn_sched_group_barrier(0x008, TH, 0);  // MFMA
                        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // LDS read
                    }
                    __builtin_amdgcn_sched_group_barrier(0x008, 4 * TH * TH - 2 * TH * TH, 0);
                }
            };
            fetch(a0, b0, 0);
            if (NG > 1) fetch(a1, b1, 1);
            fma_group(a0, b0, true, false);  // group 0 starts the accumulators
#pragma unroll 1
            for (int g = 1; g + 1 < NG; g += 2) {
                fetch(a0, b0, g + 1);
                fma_group(a1, b1, false, true);
                fetch(a1, b1, g + 2 < NG ? g + 2 : 0);
                fma_group(a0, b0, false, true);
            }
            if ((NG - 1) % 2 == 1) fma_group(a1, b1, false, false);
        } else {
#pragma unroll
            for (int ti = 0; ti < TH; ++ti)
#pragma unroll
                for (int tj = 0; tj < TH; ++tj) acc[ti][tj] = (acc_t)(0);
            const T *lp = Lb + (16 * (wr * TH) + lj) * LPA + lg;
            const T *rp = Rb + lg * LPB + 16 * (wc * TH) + lj;
            constexpr int NK = NP / 4;  // k-steps; even
            T a0[TH], b0[TH], a1[TH], b1[TH];
            auto fetch = [&](T *a, T *bq, int kk) {
#pragma unroll
                for (int ti = 0; ti < TH; ++ti) a[ti] = row_ok(ti) ? lp[ti * 16 * LPA + 4 * kk] : (T)0;
#pragma unroll
                for (int tj = 0; tj < TH; ++tj) bq[tj] = col_ok(tj) ? rp[4 * kk * LPB + tj * 16] : (T)0;
            };
            auto fma_step = [&](const T *a, const T *bq) {
#pragma unroll
                for (int ti = 0; ti < TH; ++ti)
#pragma unroll
                    for (int tj = 0; tj < TH; ++tj)
                        if (row_ok(ti) && col_ok(tj)) acc[ti][tj] = Mfma<T>::run(a[ti], bq[tj], acc[ti][tj]);
            };
            fetch(a0, b0, 0);
#pragma unroll 1
            for (int kk = 0; kk < NK; kk += 2) {
                fetch(a1, b1, kk + 1);
                fma_step(a0, b0);
                fetch(a0, b0, kk + 2 < NK ? kk + 2 : 0);
                fma_step(a1, b1);
            }
        }
    };
    // visit every element this lane owns: f(ti, tj, v, row, col)
    auto for_owned = [&](auto &&f) {
#pragma unroll
        for (int ti = 0; ti < TH; ++ti)
#pragma unroll
            for (int tj = 0; tj < TH; ++tj)
                if (row_ok(ti) && col_ok(tj)) {
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        f(ti, tj, v, 16 * (wr * TH + ti) + Mfma<T>::row(lg, v), 16 * (wc * TH + tj) + lj);
                }
    };
    // identity term; it also lands on the diagonal of the zero padding, which is a block of its own
    // (padded rows and columns of every operand are zero) and is never stored
    auto dg = [&](int r, int c) -> T { return r == c ? (T)1 : (T)0; };
    // Q(r, c) = val(ti, tj, v, r, c) for every element this lane owns.  In the transposed fp32 buffer the four
    // rows a lane holds of one column are adjacent: one 16-byte store per tile.
    auto store_right = [&](auto &&val) {
#pragma unroll
        for (int ti = 0; ti < TH; ++ti)
#pragma unroll
            for (int tj = 0; tj < TH; ++tj)
                if (row_ok(ti) && col_ok(tj)) {
                    const int rb = 16 * (wr * TH + ti), c = 16 * (wc * TH + tj) + lj;
                    if constexpr (kWide) {
                        typename VecOf<T>::type x;
#pragma unroll
                        for (int v = 0; v < 4; ++v) reinterpret_cast<T *>(&x)[v] = val(ti, tj, v, rb + 4 * lg + v, c);
                        *reinterpret_cast<typename VecOf<T>::type *>(Q + c * LPB + rb + 4 * lg) = x;
                    } else {
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            const int r = rb + Mfma<T>::row(lg, v);
                            Q[ri(r, c)] = val(ti, tj, v, r, c);
                        }
                    }
                }
    };

    // element-wise state in registers: A, A^2, y02, additive part
    T av[TH][TH][4], a2v[TH][TH][4], yv[TH][TH][4], gv[TH][TH][4];
    for_owned([&](int ti, int tj, int v, int r, int c) {
        av[ti][tj][v] = P[li(r, c)];
        a2v[ti][tj][v] = (T)0;
    });
    // the transposed copy; visible after the barriers of the norm below
    if constexpr (kWide) store_right([&](int ti, int tj, int v, int, int) { return av[ti][tj][v]; });

    int m = 0, s = 0, flags = 0;
    // The polynomial X ends in registers xv (aliasing acc's storage is left to the compiler).
    T xv[TH][TH][4];
    const double n1 = norm_regs([&](int ti, int tj, int v) { return av[ti][tj][v]; });
    T a3v[TH][TH][4], a4v[TH][TH][4];  // W^3, W^4 of the Paterson-Stockmeyer variant
    if constexpr (SCHEME == kSchemePS) {
        // Algorithm 3: powers are formed one by one, only as far as the orders tried need them.
        // P holds the newest power (left operand), Q keeps W (right operand): W^j = W^(j-1) * W.
        double nrm[4] = {n1, 0.0, 0.0, 0.0};
        bool need_more = false;
        select_ps_order_scaling(nrm, 1, eps, m, s, flags, need_more);
        if (need_more) {
            product(P, Q);  // W * W
            sync();
            for_owned([&](int ti, int tj, int v, int r, int c) {
                a2v[ti][tj][v] = acc[ti][tj][v];
                P[li(r, c)] = acc[ti][tj][v];
            });
            sync();
            nrm[1] = norm_regs([&](int ti, int tj, int v) { return a2v[ti][tj][v]; });
            select_ps_order_scaling(nrm, 2, eps, m, s, flags, need_more);
        }
        if (need_more) {
            product(P, Q);  // W^2 * W
            sync();
            for_owned([&](int ti, int tj, int v, int r, int c) {
                a3v[ti][tj][v] = acc[ti][tj][v];
                P[li(r, c)] = acc[ti][tj][v];
            });
            sync();
            nrm[2] = norm_regs([&](int ti, int tj, int v) { return a3v[ti][tj][v]; });
            select_ps_order_scaling(nrm, 3, eps, m, s, flags, need_more);
        }
        if (need_more) {
            product(P, Q);  // W^3 * W
            sync();
            for_owned([&](int ti, int tj, int v, int r, int c) {
                a4v[ti][tj][v] = acc[ti][tj][v];
                P[li(r, c)] = acc[ti][tj][v];
            });
            sync();
            nrm[3] = norm_regs([&](int ti, int tj, int v) { return a4v[ti][tj][v]; });
            select_ps_order_scaling(nrm, 4, eps, m, s, flags, need_more);
        }
    } else if constexpr (SCHEME == kSchemePhi) {
        // Core series of the low-rank variant: the order follows from the norm alone, no scaling; the powers the
        // Paterson-Stockmeyer form of that order needs are formed as above (P: newest power, Q: the matrix).
        select_lowrank_order(n1, eps, m, flags);
        const int jn = m >= 0 ? ps_j(m) : 0;
        if (jn >= 2) {
            product(P, Q);
            sync();
            for_owned([&](int ti, int tj, int v, int r, int c) {
                a2v[ti][tj][v] = acc[ti][tj][v];
                P[li(r, c)] = acc[ti][tj][v];
            });
            sync();
        }
        if (jn >= 3) {
            product(P, Q);
            sync();
            for_owned([&](int ti, int tj, int v, int r, int c) {
                a3v[ti][tj][v] = acc[ti][tj][v];
                P[li(r, c)] = acc[ti][tj][v];
            });
            sync();
        }
        if (jn >= 4) {
            product(P, Q);
            sync();
            for_owned([&](int ti, int tj, int v, int r, int c) {
                a4v[ti][tj][v] = acc[ti][tj][v];
                P[li(r, c)] = acc[ti][tj][v];
            });
            sync();
        }
    } else if constexpr (SCHEME == kSchemeBaseline) {
        // The comparison baseline of the paper (its Algorithm 1): s from ||W|| / 2^s < 1/2, then Taylor terms
        // Y <- W Y / k are added while ||Y|| > eps.  The whole loop runs here because the degree reached
        // is only known at its end; xv holds X when it is done.
        for_owned([&](int ti, int tj, int v, int r, int c) { xv[ti][tj][v] = dg(r, c); });
        if (!(n1 <= 1.7976931348623157e308)) {
            m = -1; s = -1; flags = 1;
        } else if (n1 > 0.0) {
            double t = n1;
            while (!(t < 0.5)) { t *= 0.5; ++s; }
            const T sg = (T)ldexp(1.0, -s);
            sync();
            for_owned([&](int ti, int tj, int v, int r, int c) {
                av[ti][tj][v] *= sg;
                yv[ti][tj][v] = av[ti][tj][v];
                P[li(r, c)] = av[ti][tj][v];   // left operand: the scaled matrix, fixed
            });
            store_right([&](int ti, int tj, int v, int, int) { return av[ti][tj][v]; });  // right operand: the term Y
            sync();
            int k = 2;
            for (int it = 0; it < 256; ++it) {
                const double ny = norm_regs([&](int ti, int tj, int v) { return yv[ti][tj][v]; });
                if (!(ny > eps)) break;
                for_owned([&](int ti, int tj, int v, int, int) { xv[ti][tj][v] += yv[ti][tj][v]; });
                ++m;
                product(P, Q);
                const T kk = (T)k;
                for_owned([&](int ti, int tj, int v, int, int) { yv[ti][tj][v] = acc[ti][tj][v] / kk; });
                ++k;
                sync();
                store_right([&](int ti, int tj, int v, int, int) { return yv[ti][tj][v]; });
                sync();
            }
        }
    } else {
        double n2 = 0.0;
        // orders 0 and 1 need no product: Algorithm 4 forms W^2 only once the m = 1 test has failed
        const bool finite1 = n1 == n1;
        const bool tiny = finite1 && (n1 == 0.0 || (0.5 * n1 * n1 + (1.0 / 6.0) * n1 * n1 * n1 <= eps));
        if (finite1 && !tiny) {
            product(P, Q);  // W * W
            sync();
            for_owned([&](int ti, int tj, int v, int r, int c) {
                a2v[ti][tj][v] = acc[ti][tj][v];
                P[li(r, c)] = acc[ti][tj][v];
            });
            sync();
            n2 = norm_regs([&](int ti, int tj, int v) { return a2v[ti][tj][v]; });
        }
        select_order_scaling(n1, n2, eps, m, s, flags);
    }
    // (m, s) are the same in every lane (the norms are, bit for bit): say so, and everything that depends on them
    // -- which formulas, which coefficients, how many squarings -- becomes scalar control flow and scalar selects
    m = __builtin_amdgcn_readfirstlane(m);
    s = __builtin_amdgcn_readfirstlane(s);
    flags = __builtin_amdgcn_readfirstlane(flags);
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

    if constexpr (SCHEME == kSchemeBaseline) {
        // nothing left to evaluate: the term loop above produced X
    } else if constexpr (SCHEME == kSchemePS || SCHEME == kSchemePhi) {
        // ---- Paterson-Stockmeyer: sum_i c_i A^i = Horner in A^j with blocks of degree < j, m = j*k ----------
        // c_i = 1/i! (the Taylor polynomial T_m) or 1/(i+1)! (the series of the low-rank variant)
        constexpr int kShift = SCHEME == kSchemePhi ? 1 : 0;
        const int j = ps_j(m), k = ps_k(m);
        if (s > 0) {
            const T sg = (T)pow2neg_f(s), sg2 = (T)pow2neg_f(2 * s), sg3 = (T)pow2neg_f(3 * s), sg4 = (T)pow2neg_f(4 * s);
            for_owned([&](int ti, int tj, int v, int, int) {
                av[ti][tj][v] *= sg;
                if (j >= 2 || m == 2) a2v[ti][tj][v] *= sg2;
                if (j >= 3) a3v[ti][tj][v] *= sg3;
                if (j >= 4) a4v[ti][tj][v] *= sg4;
            });
        }
        auto pw = [&](int r, int ti, int tj, int v) -> T {
            return r == 1 ? av[ti][tj][v] : (r == 2 ? a2v[ti][tj][v] : (r == 3 ? a3v[ti][tj][v] : a4v[ti][tj][v]));
        };
        if (k == 1) {  // orders 0, 1, 2: no further product
            const T c1 = (T)inv_factorial(1 + kShift), c2 = (T)inv_factorial(2 + kShift);
            for_owned([&](int ti, int tj, int v, int r, int c) {
                T x = dg(r, c);
                if (m >= 1) x += c1 * av[ti][tj][v];
                if (m == 2) x += c2 * a2v[ti][tj][v];
                xv[ti][tj][v] = x;
            });
        } else {
            T cf[5];
#pragma unroll
            for (int r = 0; r <= 4; ++r) cf[r] = r <= j ? (T)inv_factorial((k - 1) * j + r + kShift) : (T)0;
            sync();  // every wave is done with P (norm) before it is overwritten
            for_owned([&](int ti, int tj, int v, int r, int c) {
                T h = cf[0] * dg(r, c) + cf[1] * av[ti][tj][v] + cf[2] * a2v[ti][tj][v];
                if (j >= 3) h += cf[3] * a3v[ti][tj][v];
                if (j >= 4) h += cf[4] * a4v[ti][tj][v];
                P[li(r, c)] = h;              // top block c_{(k-1)j} I + ... + c_m A^j
            });
            store_right([&](int ti, int tj, int v, int, int) { return pw(j, ti, tj, v); });  // right operand of every Horner step: A^j
            for (int q = k - 2; q >= 0; --q) {
#pragma unroll
                for (int r = 0; r <= 3; ++r) cf[r] = r < j ? (T)inv_factorial(q * j + r + kShift) : (T)0;
                sync();
                product(P, Q);
                for_owned([&](int ti, int tj, int v, int r, int c) {
                    T h = acc[ti][tj][v] + cf[0] * dg(r, c) + cf[1] * av[ti][tj][v];
                    if (j >= 3) h += cf[2] * a2v[ti][tj][v];
                    if (j >= 4) h += cf[3] * a3v[ti][tj][v];
                    xv[ti][tj][v] = h;
                });
                if (q > 0) {
                    sync();
                    for_owned([&](int ti, int tj, int v, int r, int c) { P[li(r, c)] = xv[ti][tj][v]; });
                }
            }
        }
    } else {
    // ---- scale: A = W / 2^s, A2 = W2 / 4^s (exact).  P holds W2 and becomes A2. ------------------------
    if (s > 0) {
        const T sg = (T)pow2neg_f(s), sg2 = (T)pow2neg_f(2 * s);
        for_owned([&](int ti, int tj, int v, int r, int c) {
            av[ti][tj][v] *= sg;
            a2v[ti][tj][v] *= sg2;
            P[li(r, c)] = a2v[ti][tj][v];
        });
    }

    if (m <= 2) {
        for_owned([&](int ti, int tj, int v, int r, int c) {
            T x = dg(r, c);
            if (m >= 1) x += av[ti][tj][v];
            if (m == 2) x += a2v[ti][tj][v] / (T)2;
            xv[ti][tj][v] = x;
        });
    } else if (m == 4) {
        // T4 = (A2/12 + A/3 + I) * (A2/2) + A + I
        sync();  // every wave is done with P (norm) before it is overwritten
        for_owned([&](int ti, int tj, int v, int r, int c) {
            const T a = av[ti][tj][v], a2 = a2v[ti][tj][v];
            P[li(r, c)] = a2 * (T)(1.0 / 12.0) + a * (T)(1.0 / 3.0) + dg(r, c);
        });
        store_right([&](int ti, int tj, int v, int, int) { return a2v[ti][tj][v] / (T)2; });
        sync();
        product(P, Q);
        for_owned([&](int ti, int tj, int v, int r, int c) { xv[ti][tj][v] = acc[ti][tj][v] + av[ti][tj][v] + dg(r, c); });
    } else {
        const bool hi = m == 15;
        const T c1 = (T)(hi ? EXPM_T15_C1 : EXPM_T8_C1), c2 = (T)(hi ? EXPM_T15_C2 : EXPM_T8_C2);
        const T c3 = (T)(hi ? EXPM_T15_C3 : EXPM_T8_C3), c4 = (T)(hi ? EXPM_T15_C4 : EXPM_T8_C4);
        const T c5 = (T)(hi ? EXPM_T15_C5 : EXPM_T8_C5), c6 = (T)(hi ? EXPM_T15_C6 : EXPM_T8_C6);
        // y02 = A2 * (c1 A2 + c2 A): left operand A2 is already in P
        store_right([&](int ti, int tj, int v, int, int) { return c1 * a2v[ti][tj][v] + c2 * av[ti][tj][v]; });
        sync();
        product(P, Q);
        sync();
        for_owned([&](int ti, int tj, int v, int r, int c) {
            const T y = acc[ti][tj][v], a = av[ti][tj][v], a2 = a2v[ti][tj][v];
            yv[ti][tj][v] = y;
            P[li(r, c)] = y + c3 * a2 + c4 * a;
            gv[ti][tj][v] = hi ? c6 * y + (T)EXPM_T15_C7 * a2 : c6 * y + a2 / (T)2 + a + dg(r, c);
        });
        store_right([&](int ti, int tj, int v, int, int) { return yv[ti][tj][v] + c5 * a2v[ti][tj][v]; });
        sync();
        product(P, Q);
        if (!hi) {
            for_owned([&](int ti, int tj, int v, int, int) { xv[ti][tj][v] = acc[ti][tj][v] + gv[ti][tj][v]; });
        } else {
            const T c8 = (T)EXPM_T15_C8, c9 = (T)EXPM_T15_C9, c10 = (T)EXPM_T15_C10, c11 = (T)EXPM_T15_C11,
                    c12 = (T)EXPM_T15_C12, c13 = (T)EXPM_T15_C13, c14 = (T)EXPM_T15_C14, c15 = (T)EXPM_T15_C15,
                    c16 = (T)EXPM_T15_C16;
            sync();
            store_right([&](int ti, int tj, int v, int, int) {
                const T y1 = acc[ti][tj][v] + gv[ti][tj][v];  // y12
                return y1 + c10 * yv[ti][tj][v] + c11 * av[ti][tj][v];
            });
            for_owned([&](int ti, int tj, int v, int r, int c) {
                const T a = av[ti][tj][v], a2 = a2v[ti][tj][v], y0 = yv[ti][tj][v];
                const T y1 = acc[ti][tj][v] + gv[ti][tj][v];  // y12
                P[li(r, c)] = y1 + c8 * a2 + c9 * a;
                gv[ti][tj][v] = c12 * y1 + c13 * y0 + c14 * a2 + c15 * a + c16 * dg(r, c);
            });
            sync();
            product(P, Q);
            for_owned([&](int ti, int tj, int v, int, int) { xv[ti][tj][v] = acc[ti][tj][v] + gv[ti][tj][v]; });
        }
    }

    }

    // ---- squaring phase: X in both operand layouts, product, repeat ------------------------------------
    for (int q = 0; q < s; ++q) {
        sync();
        for_owned([&](int ti, int tj, int v, int r, int c) { P[li(r, c)] = xv[ti][tj][v]; });
        store_right([&](int ti, int tj, int v, int, int) { return xv[ti][tj][v]; });
        sync();
        product(P, Q);
        for_owned([&](int ti, int tj, int v, int, int) { xv[ti][tj][v] = acc[ti][tj][v]; });
    }

    // ---- store through P so that global writes are whole rows -----------------------------------------
    sync();
    for_owned([&](int ti, int tj, int v, int r, int c) { P[li(r, c)] = xv[ti][tj][v]; });
    sync();
    if (vec_ok) {
        using V = typename VecOf<T>::type;
#pragma unroll 4
        for (int e = tid; e < n * CV; e += C::kThreads) {
            const int r = e / CV, c = (e - r * CV) * VN;
            if (c < n) *reinterpret_cast<V *>(O + (size_t)r * n + c) = *reinterpret_cast<const V *>(P + li(r, c));
        }
    } else {
#pragma unroll 4
        for (int e = tid; e < n * NR; e += C::kThreads) {
            const int r = e / NR, c = e - r * NR;
            if (c < n) O[(size_t)r * n + c] = P[li(r, c)];
        }
    }
}

// ---------------------------------------------------------------------------------------------------
// Matrices of at most one MFMA tile (n <= 16): one wave per matrix, everything in registers, no LDS.
//
// Every matrix M of the computation is held twice, in the MFMA result layout: h[v] = M(row(g,v), j) and
// t[v] = M(j, row(g,v)) = M^T in the same layout (lane = 16 g + j).  With the k index of step q of a
// product taken as row(g,q), t of the left factor is exactly the left-operand fragment and h of the right
// factor the right-operand fragment, so  D = L R  is  D.h = sum_q mfma(L.t[q], R.h[q])  and, because
// D^T = R^T L^T,  D.t = sum_q mfma(R.h[q], L.t[q]).  Both forms of the result come out of the matrix cores
// in the layout they are needed in next; nothing is transposed through memory.  The 1-norm is taken from
// h (column j is summed within the lane and across the four lane groups), the infinity norm from t.
// Four matrices share a workgroup (one wave each, nothing in common).
// ---------------------------------------------------------------------------------------------------
template <typename T> struct Pair {
    T h[4], t[4];
};

// (register budget of 128 per lane: the four workgroups a compute unit gets at a batch of 4096 are resident together)
// (FULL: n = 16 exactly, a compile-time constant for the index arithmetic and the bounds predicates)
template <typename T, int SCHEME, bool FULL = false>
__global__ __launch_bounds__(256, 4) void fused_tile_kernel(const T *__restrict__ Ain, T *__restrict__ Out, int n_arg, int batch,
                                                         double eps, int select_only, int norm_inf,
                                                         MatInfo *__restrict__ info)
{
    using acc_t = typename Mfma<T>::acc_t;
    const int n = FULL ? 16 : n_arg;
    using M = Pair<T>;
    const int b = blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (b >= batch) return;
    const int lane = threadIdx.x & 63, lj = lane & 15, lg = lane >> 4;
    const size_t moff = (size_t)b * n * n;
    const T *W = Ain + moff;
    int rw[4];
    bool in[4];  // element (rw[v], lj) -- and (lj, rw[v]) -- lies inside the n x n matrix
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        rw[v] = Mfma<T>::row(lg, v);
        in[v] = rw[v] < n && lj < n;
    }
    auto each = [&](auto &&f) {
#pragma unroll
        for (int v = 0; v < 4; ++v) f(v);
    };
    // D = L * R in both forms; the transposed form is skipped (left equal to h) when nothing multiplies D again
    auto mul = [&](const M &L, const M &R, bool both = true) -> M {
        acc_t dh = (acc_t)(0), dt = (acc_t)(0);
#pragma unroll
        for (int q = 0; q < 4; ++q) dh = Mfma<T>::run(L.t[q], R.h[q], dh);
        if (both) {
#pragma unroll
            for (int q = 0; q < 4; ++q) dt = Mfma<T>::run(R.h[q], L.t[q], dt);
        }
        M d;
        each([&](int v) { d.h[v] = dh[v]; d.t[v] = both ? dt[v] : dh[v]; });
        return d;
    };
    // e = f(x.., identity) applied to both forms; the identity is symmetric
    T dgv[4];
    each([&](int v) { dgv[v] = rw[v] == lj ? (T)1 : (T)0; });  // also on the padding's diagonal: a block of its own
    // max column abs-sum of the matrix whose result-layout registers are x (double sums, NaN if not finite)
    auto colnorm = [&](const T (&x)[4]) -> double {
        double sum = 0.0;
        each([&](int v) { sum += fabs((double)x[v]); });
        sum += __shfl_xor(sum, 16);
        sum += __shfl_xor(sum, 32);  // column lj, complete in every lane
        const int bad = !(sum <= 1.7976931348623157e308);
        double mx = bad ? 0.0 : sum;
        mx = row16_allreduce(mx, [](double a, double c) { return c > a ? c : a; });
        return __any(bad) ? __longlong_as_double(0x7ff8000000000000LL) : mx;
    };
    auto norm = [&](const M &x) -> double { return norm_inf ? colnorm(x.t) : colnorm(x.h); };

    // W is read once, in the form whose loads are whole row segments (rows rw[v], 16 consecutive columns);
    // indices past n are clamped and the value dropped, so no load is predicated.  The transposed form
    // comes from the matrix cores: with h as the left-operand fragment and the identity on the right,
    // sum_q mfma(h[q], I[q]) is W^T I in the result layout (exact: products with 1 and sums with 0).
    M w;
    {
        const int cj = lj < n ? lj : n - 1;
        T ld[4];
        each([&](int v) { ld[v] = W[(size_t)(rw[v] < n ? rw[v] : n - 1) * n + cj]; });
        each([&](int v) { w.h[v] = in[v] ? ld[v] : (T)0; });
        acc_t tt = (acc_t)(0);
#pragma unroll
        for (int q = 0; q < 4; ++q) tt = Mfma<T>::run(w.h[q], (rw[q] == lj ? (T)1 : (T)0), tt);
        each([&](int v) { w.t[v] = tt[v]; });
    }

    int m = 0, s = 0, flags = 0;
    M w2, w3, w4, x;
    each([&](int v) { w2.h[v] = w2.t[v] = w3.h[v] = w3.t[v] = w4.h[v] = w4.t[v] = (T)0; x.h[v] = x.t[v] = dgv[v]; });
    const double n1 = norm(w);
    if constexpr (SCHEME == kSchemePS) {
        // Algorithm 3: powers are formed one by one, only as far as the orders tried need them
        double nrm[4] = {n1, 0.0, 0.0, 0.0};
        bool need_more = false;
        select_ps_order_scaling(nrm, 1, eps, m, s, flags, need_more);
        if (need_more) {
            w2 = mul(w, w);
            nrm[1] = norm(w2);
            select_ps_order_scaling(nrm, 2, eps, m, s, flags, need_more);
        }
        if (need_more) {
            w3 = mul(w2, w);
            nrm[2] = norm(w3);
            select_ps_order_scaling(nrm, 3, eps, m, s, flags, need_more);
        }
        if (need_more) {
            w4 = mul(w3, w);
            nrm[3] = norm(w4);
            select_ps_order_scaling(nrm, 4, eps, m, s, flags, need_more);
        }
    } else if constexpr (SCHEME == kSchemeBaseline) {
        // The comparison baseline of the paper (its Algorithm 1): s from ||W|| / 2^s < 1/2, then Taylor terms
        // Y <- W Y / k are added while ||Y|| > eps; x holds X when the loop is done.
        if (!(n1 <= 1.7976931348623157e308)) {
            m = -1; s = -1; flags = 1;
        } else if (n1 > 0.0) {
            double tt = n1;
            while (!(tt < 0.5)) { tt *= 0.5; ++s; }
            const T sg = (T)ldexp(1.0, -s);
            each([&](int v) { w.h[v] *= sg; w.t[v] *= sg; });
            M y = w;
            int k = 2;
            for (int it = 0; it < 256; ++it) {
                const double ny = norm(y);
                if (!(ny > eps)) break;
                each([&](int v) { x.h[v] += y.h[v]; x.t[v] += y.t[v]; });
                ++m;
                const M p = mul(w, y);
                const T kk = (T)k;
                each([&](int v) { y.h[v] = p.h[v] / kk; y.t[v] = p.t[v] / kk; });
                ++k;
            }
        }
    } else {
        double n2 = 0.0;
        // orders 0 and 1 need no product: Algorithm 4 forms W^2 only once the m = 1 test has failed
        const bool finite1 = n1 == n1;
        const bool tiny = finite1 && (n1 == 0.0 || (0.5 * n1 * n1 + (1.0 / 6.0) * n1 * n1 * n1 <= eps));
        if (finite1 && !tiny) {
            w2 = mul(w, w);
            n2 = norm(w2);
        }
        select_order_scaling(n1, n2, eps, m, s, flags);
    }
    // (m, s) are the same in every lane: scalar control flow and scalar coefficient selects from here on
    m = __builtin_amdgcn_readfirstlane(m);
    s = __builtin_amdgcn_readfirstlane(s);
    flags = __builtin_amdgcn_readfirstlane(flags);
    if (lane == 0) {
        MatInfo mi;
        mi.m = m; mi.s = s; mi.len = 0; mi.flags = flags;
        info[b] = mi;
    }
    if (select_only) return;
    T *O = Out + moff;
    if (m < 0) {
        const T qnan = (T)__longlong_as_double(0x7ff8000000000000LL);
        each([&](int v) { if (in[v]) O[(size_t)rw[v] * n + lj] = qnan; });
        return;
    }

    // f(h-or-t registers...) on both forms
    if constexpr (SCHEME == kSchemeBaseline) {
        // nothing left to evaluate: the term loop above produced X
    } else if constexpr (SCHEME == kSchemePS) {
        // ---- Paterson-Stockmeyer: T_m(A) = Horner in A^j with blocks of degree < j, m = j*k -----------------
        const int j = ps_j(m), k = ps_k(m);
        if (s > 0) {
            const T sg = (T)pow2neg_f(s), sg2 = (T)pow2neg_f(2 * s), sg3 = (T)pow2neg_f(3 * s), sg4 = (T)pow2neg_f(4 * s);
            each([&](int v) {
                w.h[v] *= sg; w.t[v] *= sg;
                w2.h[v] *= sg2; w2.t[v] *= sg2;
                w3.h[v] *= sg3; w3.t[v] *= sg3;
                w4.h[v] *= sg4; w4.t[v] *= sg4;
            });
        }
        if (k == 1) {  // orders 0, 1, 2: no further product
            each([&](int v) {
                T xh = dgv[v], xt = dgv[v];
                if (m >= 1) { xh += w.h[v]; xt += w.t[v]; }
                if (m == 2) { xh += w2.h[v] / (T)2; xt += w2.t[v] / (T)2; }
                x.h[v] = xh; x.t[v] = xt;
            });
        } else {
            const M &aj = j == 2 ? w2 : (j == 3 ? w3 : w4);  // right operand of every Horner step: A^j
            T cf[5];
#pragma unroll
            for (int r = 0; r <= 4; ++r) cf[r] = r <= j ? (T)inv_factorial((k - 1) * j + r) : (T)0;
            M hcur;  // top block c_{(k-1)j} I + ... + c_m A^j
            each([&](int v) {
                hcur.h[v] = cf[0] * dgv[v] + cf[1] * w.h[v] + cf[2] * w2.h[v] + cf[3] * w3.h[v] + cf[4] * w4.h[v];
                hcur.t[v] = cf[0] * dgv[v] + cf[1] * w.t[v] + cf[2] * w2.t[v] + cf[3] * w3.t[v] + cf[4] * w4.t[v];
            });
            for (int q = k - 2; q >= 0; --q) {
#pragma unroll
                for (int r = 0; r <= 3; ++r) cf[r] = r < j ? (T)inv_factorial(q * j + r) : (T)0;
                const M p = mul(hcur, aj, q > 0 || s > 0);
                each([&](int v) {
                    hcur.h[v] = p.h[v] + cf[0] * dgv[v] + cf[1] * w.h[v] + cf[2] * w2.h[v] + cf[3] * w3.h[v];
                    hcur.t[v] = p.t[v] + cf[0] * dgv[v] + cf[1] * w.t[v] + cf[2] * w2.t[v] + cf[3] * w3.t[v];
                });
            }
            x = hcur;
        }
    } else {
        // ---- scale: A = W / 2^s, A2 = W2 / 4^s (exact) ---------------------------------------------------
        if (s > 0) {
            const T sg = (T)pow2neg_f(s), sg2 = (T)pow2neg_f(2 * s);
            each([&](int v) { w.h[v] *= sg; w.t[v] *= sg; w2.h[v] *= sg2; w2.t[v] *= sg2; });
        }
        const M &a = w, &a2 = w2;
        if (m <= 2) {
            each([&](int v) {
                T xh = dgv[v], xt = dgv[v];
                if (m >= 1) { xh += a.h[v]; xt += a.t[v]; }
                if (m == 2) { xh += a2.h[v] / (T)2; xt += a2.t[v] / (T)2; }
                x.h[v] = xh; x.t[v] = xt;
            });
        } else if (m == 4) {
            // T4 = (A2/12 + A/3 + I) * (A2/2) + A + I
            M L, R;
            each([&](int v) {
                L.h[v] = a2.h[v] * (T)(1.0 / 12.0) + a.h[v] * (T)(1.0 / 3.0) + dgv[v];
                L.t[v] = a2.t[v] * (T)(1.0 / 12.0) + a.t[v] * (T)(1.0 / 3.0) + dgv[v];
                R.h[v] = a2.h[v] / (T)2;
                R.t[v] = a2.t[v] / (T)2;
            });
            const M p = mul(L, R, s > 0);
            each([&](int v) { x.h[v] = p.h[v] + a.h[v] + dgv[v]; x.t[v] = p.t[v] + a.t[v] + dgv[v]; });
        } else {
            const bool hi = m == 15;
            const T c1 = (T)(hi ? EXPM_T15_C1 : EXPM_T8_C1), c2 = (T)(hi ? EXPM_T15_C2 : EXPM_T8_C2);
            const T c3 = (T)(hi ? EXPM_T15_C3 : EXPM_T8_C3), c4 = (T)(hi ? EXPM_T15_C4 : EXPM_T8_C4);
            const T c5 = (T)(hi ? EXPM_T15_C5 : EXPM_T8_C5), c6 = (T)(hi ? EXPM_T15_C6 : EXPM_T8_C6);
            // y02 = A2 * (c1 A2 + c2 A)
            M R;
            each([&](int v) { R.h[v] = c1 * a2.h[v] + c2 * a.h[v]; R.t[v] = c1 * a2.t[v] + c2 * a.t[v]; });
            const M y0 = mul(a2, R);
            M L, g;
            each([&](int v) {
                L.h[v] = y0.h[v] + c3 * a2.h[v] + c4 * a.h[v];
                L.t[v] = y0.t[v] + c3 * a2.t[v] + c4 * a.t[v];
                R.h[v] = y0.h[v] + c5 * a2.h[v];
                R.t[v] = y0.t[v] + c5 * a2.t[v];
                g.h[v] = hi ? c6 * y0.h[v] + (T)EXPM_T15_C7 * a2.h[v] : c6 * y0.h[v] + a2.h[v] / (T)2 + a.h[v] + dgv[v];
                g.t[v] = hi ? c6 * y0.t[v] + (T)EXPM_T15_C7 * a2.t[v] : c6 * y0.t[v] + a2.t[v] / (T)2 + a.t[v] + dgv[v];
            });
            const M p1 = mul(L, R, hi || s > 0);
            if (!hi) {
                each([&](int v) { x.h[v] = p1.h[v] + g.h[v]; x.t[v] = p1.t[v] + g.t[v]; });
            } else {
                const T c8 = (T)EXPM_T15_C8, c9 = (T)EXPM_T15_C9, c10 = (T)EXPM_T15_C10, c11 = (T)EXPM_T15_C11,
                        c12 = (T)EXPM_T15_C12, c13 = (T)EXPM_T15_C13, c14 = (T)EXPM_T15_C14, c15 = (T)EXPM_T15_C15,
                        c16 = (T)EXPM_T15_C16;
                each([&](int v) {
                    const T y1h = p1.h[v] + g.h[v], y1t = p1.t[v] + g.t[v];  // y12
                    L.h[v] = y1h + c8 * a2.h[v] + c9 * a.h[v];
                    L.t[v] = y1t + c8 * a2.t[v] + c9 * a.t[v];
                    R.h[v] = y1h + c10 * y0.h[v] + c11 * a.h[v];
                    R.t[v] = y1t + c10 * y0.t[v] + c11 * a.t[v];
                    g.h[v] = c12 * y1h + c13 * y0.h[v] + c14 * a2.h[v] + c15 * a.h[v] + c16 * dgv[v];
                    g.t[v] = c12 * y1t + c13 * y0.t[v] + c14 * a2.t[v] + c15 * a.t[v] + c16 * dgv[v];
                });
                const M p2 = mul(L, R, s > 0);
                each([&](int v) { x.h[v] = p2.h[v] + g.h[v]; x.t[v] = p2.t[v] + g.t[v]; });
            }
        }
    }

    // ---- squaring phase ----------------------------------------------------------------------------
    for (int q = 0; q < s; ++q) x = mul(x, x, q + 1 < s);

    each([&](int v) { if (in[v]) O[(size_t)rw[v] * n + lj] = x.h[v]; });
}

template <typename T, int SCHEME>
hipError_t launch_tile_t(const void *A, void *out, int n, int batch, double eps, int select_only, int norm_inf,
                         MatInfo *info, hipStream_t stream)
{
    if (SCHEME == kSchemeSastre && n == 16)
        hipLaunchKernelGGL((fused_tile_kernel<T, SCHEME, SCHEME == kSchemeSastre>), dim3((batch + 3) / 4), dim3(256), 0, stream,
                           reinterpret_cast<const T *>(A), reinterpret_cast<T *>(out), n, batch, eps, select_only, norm_inf, info);
    else
        hipLaunchKernelGGL((fused_tile_kernel<T, SCHEME>), dim3((batch + 3) / 4), dim3(256), 0, stream,
                           reinterpret_cast<const T *>(A), reinterpret_cast<T *>(out), n, batch, eps, select_only, norm_inf, info);
    return hipGetLastError();
}

template <typename T, int NT, int SCHEME>
hipError_t launch_fused_t(const void *A, void *out, int n, int batch, double eps, int select_only, int norm_inf,
                          MatInfo *info, hipStream_t stream)
{
    using C = FusedCfg<T, NT>;
    static PerDeviceOnce lds_limit;
    hipError_t e = lds_limit([] {
        return hipFuncSetAttribute(reinterpret_cast<const void *>(fused_expm_kernel<T, NT, SCHEME>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, C::kLds);
    });
    if (e != hipSuccess) return e;
    // one-tile matrices of exactly 16 x 16 at aligned addresses (the main scheme): the variant with the size folded in
    constexpr bool kHasFull = NT == 1 && SCHEME == kSchemeSastre;
    if (kHasFull && n == 16 && (reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(out)) % 16 == 0) {
        hipLaunchKernelGGL((fused_expm_kernel<T, NT, SCHEME, kHasFull>), dim3((batch + C::kMPW - 1) / C::kMPW), dim3(C::kBlock),
                           C::kLds, stream, reinterpret_cast<const T *>(A), reinterpret_cast<T *>(out), n, batch, eps,
                           select_only, norm_inf, info);
        return hipGetLastError();
    }
    hipLaunchKernelGGL((fused_expm_kernel<T, NT, SCHEME>), dim3((batch + C::kMPW - 1) / C::kMPW), dim3(C::kBlock), C::kLds,
                       stream, reinterpret_cast<const T *>(A), reinterpret_cast<T *>(out), n, batch, eps, select_only,
                       norm_inf, info);
    return hipGetLastError();
}

}  // namespace

bool small_path_supported(int n, int dtype)
{
    return dtype == 1 ? n <= 96 : n <= 128;
}

hipError_t launch_small(const void *A, void *out, int n, int batch, int dtype, double eps, int select_only,
                        int scheme, int norm_inf, MatInfo *info, hipStream_t stream)
{
    const int nt = (n + 15) / 16;
    if (nt == 1 && dtype == 1 && scheme != kSchemePhi) {
        // One tile in fp64: the register-resident kernel.  (In fp32 the doubled matrix-core work of that design
        // costs more than the LDS round trips of the general kernel save, so fp32 stays there.)
        return scheme == kSchemePS
                   ? launch_tile_t<double, kSchemePS>(A, out, n, batch, eps, select_only, norm_inf, info, stream)
                   : (scheme == kSchemeBaseline
                          ? launch_tile_t<double, kSchemeBaseline>(A, out, n, batch, eps, select_only, norm_inf, info, stream)
                          : launch_tile_t<double, kSchemeSastre>(A, out, n, batch, eps, select_only, norm_inf, info, stream));
    }
#define EXPM_FUSED_ARGS A, out, n, batch, eps, select_only, norm_inf, info, stream
#define EXPM_FUSED_CASE(TYPE, K)                                                               \
    case K:                                                                                    \
        switch (scheme) {                                                                      \
        case kSchemePS: return launch_fused_t<TYPE, K, kSchemePS>(EXPM_FUSED_ARGS);            \
        case kSchemeBaseline: return launch_fused_t<TYPE, K, kSchemeBaseline>(EXPM_FUSED_ARGS); \
        case kSchemePhi: return launch_fused_t<TYPE, K, kSchemePhi>(EXPM_FUSED_ARGS);          \
        default: return launch_fused_t<TYPE, K, kSchemeSastre>(EXPM_FUSED_ARGS);               \
        }
    if (dtype == 1) {
        switch (nt) {
        case 1: return launch_fused_t<double, 1, kSchemePhi>(EXPM_FUSED_ARGS);  // the other schemes: tile kernel above
            EXPM_FUSED_CASE(double, 2) EXPM_FUSED_CASE(double, 3)
            EXPM_FUSED_CASE(double, 4) EXPM_FUSED_CASE(double, 5) EXPM_FUSED_CASE(double, 6)
        default: return hipErrorInvalidValue;
        }
    }
    switch (nt) {
        EXPM_FUSED_CASE(float, 1) EXPM_FUSED_CASE(float, 2) EXPM_FUSED_CASE(float, 3) EXPM_FUSED_CASE(float, 4)
        EXPM_FUSED_CASE(float, 5) EXPM_FUSED_CASE(float, 6) EXPM_FUSED_CASE(float, 7) EXPM_FUSED_CASE(float, 8)
    default: return hipErrorInvalidValue;
    }
#undef EXPM_FUSED_CASE
#undef EXPM_FUSED_ARGS
}

}  // namespace expmk
