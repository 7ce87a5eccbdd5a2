/*
 * expm_mi355x.h -- C ABI of the MI355X (gfx950) batched matrix exponential.
 *
 * Method: Taylor scaling and squaring with dynamic choice of the order m and
 * the scaling s, and the evaluation formulas beyond Paterson-Stockmeyer, of
 * Sastre, Faronbi, Alonso, Traver, Ibanez, Lloret, "Improving Matrix
 * Exponential for Generative AI Flows: A Taylor-Based Approach Beyond
 * Paterson-Stockmeyer" (arXiv 2512.20777).  Per matrix W and tolerance eps:
 *   (m, s) by Algorithm 4 (Sec. 3.3) from ||W||_1 and ||W^2||_1;
 *   A = W / 2^s;  X = T_m(A) by the formulas of Sec. 3.1 (T_1, T_2, T_4, T_8,
 *   and y22 = T_15+);  X <- X*X  s times  (Algorithm 2).
 *
 * All matrices are real, dense, row-major and contiguous: a batch is
 * [batch][n][n] with element (b, i, j) at offset (b*n + i)*n + j.
 * Every pointer is labelled HOST or DEVICE below.  Nothing is thrown across
 * this boundary; every entry point returns a status code.
 *
 * Threading and streams: the library keeps one cached device workspace per device.  Entry points are
 * serialised by a lock, and a call on another stream than the previous call's is ordered on the device
 * behind everything queued on that stream so far, so calls from several host threads or on several
 * streams are safe; they run one after another, not side by side.  Exceptions: calls recorded into a HIP
 * graph and expm_noalloc() are not ordered against other calls (see there).
 */
#ifndef EXPM_MI355X_H
#define EXPM_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* dtype argument */
#define EXPM_DTYPE_F32 0
#define EXPM_DTYPE_F64 1

/* status codes: 0 success, > 0 warning (results delivered), < 0 error (nothing delivered) */
#define EXPM_OK                 0
#define EXPM_WARN_NONFINITE     1  /* some matrix holds NaN/Inf (or its square overflows): its (m,s) is (-1,-1), its result all NaN */
#define EXPM_WARN_SCALING_CAP   2  /* some matrix asked for more than the cap s = 20 of Algorithm 4 and was clipped to it: tolerance not guaranteed for it */
#define EXPM_ERR_INVALID_ARG   -1  /* null pointer, n < 0, batch < 0, unknown dtype, out overlapping A, size overflow */
#define EXPM_ERR_TOLERANCE     -2  /* tol negative, NaN, or 0 < tol < unit roundoff of dtype (Sec. 3.2 requires eps >= u) */
#define EXPM_ERR_ALLOC         -3  /* device or pinned-host allocation failed */
#define EXPM_ERR_HIP           -4  /* a HIP call failed; expm_last_hip_error() returns its hipError_t */
#define EXPM_ERR_UNSUPPORTED   -5  /* the scheme asked for is not available for this matrix size */
#define EXPM_ERR_WORKSPACE     -6  /* the workspace of this shape exceeds what the call may use: the static scratch of
                                      expm_noalloc(), or a cached workspace that would have to grow inside a stream capture */

#define EXPM_S_CAP 20  /* largest scaling Algorithm 4 returns */

/*
 * expm_select -- order and scaling of Algorithm 4 (Sec. 3.3) for every matrix.
 *
 *   A      DEVICE, const, [batch][n][n] of dtype; not modified; caller-owned.
 *   n      matrix order, >= 0.          batch  number of matrices, >= 0.
 *   dtype  EXPM_DTYPE_F32 or EXPM_DTYPE_F64.
 *          Limits: n <= 46340; for n above the fused-path limit (128 in fp32, 96 in fp64)
 *          batch <= 65535 and batch * ceil(n/128)^2 <= 2e9.
 *   tol    absolute tolerance eps of Algorithm 4; 0 means "unit roundoff of dtype"
 *          (2^-24 or 2^-53); otherwise must be >= that unit roundoff.
 *   m_out, s_out   HOST, int32[batch], written on return.  m is one of 0,1,2,4,8,15
 *          (15 stands for the 15+ approximant); 0 <= s <= 20; (-1,-1) marks a
 *          non-finite matrix.
 *
 * Runs on the null stream and is synchronous: the outputs are valid on return.
 * Uses the same kernels as expm(), so both always agree on (m, s).
 * Returns 0, a warning (> 0) or an error (< 0).  n == 0 or batch == 0: success, no work.
 */
int expm_select(const void *A, int n, int batch, int dtype, double tol,
                int32_t *m_out, int32_t *s_out);

/*
 * expm -- e^W for every matrix of the batch (Algorithm 2 with Algorithm 4, Sec. 3.3,
 * evaluation formulas of Sec. 3.1).
 *
 *   A      DEVICE, const, [batch][n][n] of dtype; not modified.
 *   out    DEVICE, [batch][n][n] of dtype, must not overlap A; fully overwritten
 *          (it also serves as scratch while the call is in flight).
 *   stream hipStream_t as void* (NULL = null stream).  All device work is ordered
 *          on this stream.
 *   other arguments as for expm_select.
 *
 * Ordering / blocking: for matrices that fit a compute unit's LDS (n <= 128 in fp32, n <= 96 in fp64) the
 * whole call is one fused kernel and returns without waiting for the device.  For
 * larger n the number of product rounds depends on the data.  By default the call waits on
 * `stream` until the selection stage has finished (one 256-byte read-back), enqueues
 * exactly the rounds needed and returns without waiting for them.  With EXPM_PLAN=device in the environment, and
 * always while `stream` is being captured, the rounds are planned on the device instead: the call enqueues the
 * selection and every round a matrix can need (3 + EXPM_S_CAP), workgroups of rounds a matrix does not need leave
 * at once, and nothing waits.
 *
 * Stream capture: while `stream` is being captured a call only enqueues kernels on that stream (no read-back, no
 * memset, no other stream) and may be recorded into a HIP graph for any n, provided the workspace was reserved
 * before the capture (expm_reserve, or an earlier call of the same size; otherwise EXPM_ERR_WORKSPACE) -- the
 * recorded kernels hold its address, so a later call that makes the workspace grow invalidates such graphs, and
 * replays must not overlap other calls of the library.
 *
 * Returns 0 or an error (< 0).  Warnings are returned when they are known at return
 * time (the larger-n path planned on the host); after any call expm_get_stats() reports them.
 * Ownership: caller owns A and out and must keep them alive until `stream` has
 * finished the call; the library owns its workspace (see expm_workspace_bytes).
 */
int expm(const void *A, int n, int batch, int dtype, double tol, void *out, void *stream);

/*
 * expm_noalloc -- expm() for callers that cannot allocate: code under HIP graph capture, tight serving loops,
 * harnesses that forbid allocation.  Same arguments, result and status codes as expm(); the differences:
 *
 *   - It calls no allocator of any kind (no hipMalloc / hipFree / hipHostMalloc, no stream or event creation, no
 *     host allocation).  Its workspace (per-matrix records, norm partials and, above the fused-path sizes, the seven
 *     matrix stacks) lives in a static device array of EXPM_NOALLOC_SCRATCH_BYTES that every GPU the library runs on
 *     holds from the moment the library is loaded until the process ends.  A shape whose
 *     expm_workspace_bytes(n, batch, dtype) exceeds that size is rejected with EXPM_ERR_WORKSPACE, nothing enqueued.
 *     (64 MiB: batches of on-chip sizes up to about a million matrices, 52 bytes each; e.g. 29 matrices of 200 x 200 or 4 of
 *     512 x 512 in fp64 on the round-based path.)
 *   - It only enqueues kernels on `stream` (rounds planned on the device, see expm()), never waits, and may be
 *     recorded into a HIP graph as it is.  It therefore returns 0 or an error; warnings surface through
 *     expm_get_stats().
 *   - All calls on one GPU share that GPU's array, which keeps the previous call's contents (every call rewrites what
 *     it reads; nothing needs clearing).  Calls that overlap in time on one GPU -- two streams, or a graph replay
 *     beside another call -- race on it: the caller orders them.  expm_noalloc does not touch the cached workspace
 *     of the other entry points, so it may run beside those.
 */
#define EXPM_NOALLOC_SCRATCH_BYTES (64u << 20)
int expm_noalloc(const void *A, int n, int batch, int dtype, double tol, void *out, void *stream);

/*
 * Variants of the two calls above that pick the evaluation scheme (Sec. 3.3, Algorithm 2 with either
 * selection algorithm):
 *   EXPM_SCHEME_SASTRE  Algorithm 4 + the evaluation formulas of Sec. 3.1, orders {1,2,4,8,15+}
 *                       (what expm / expm_select run; the paper's expm_flow_opt15);
 *   EXPM_SCHEME_PS      Algorithm 3 + Paterson-Stockmeyer evaluation of the Taylor polynomial,
 *                       orders {1,2,4,6,9,12,16}, powers up to W^4 (the paper's expm_flow_ps).  m_out then
 *                       holds one of 0,1,2,4,6,9,12,16.  On the round-based path W^2, W^3 = W^2 W and
 *                       W^4 = W^3 W are formed for the whole batch before the selection.
 *   EXPM_SCHEME_BASELINE  the comparison baseline of the paper (its Algorithm 1, Sec. 2.2, after Xiao & Liu):
 *                       smallest s with ||W||/2^s < 1/2, Taylor terms Y <- W Y/k added while ||Y|| > tol,
 *                       s squarings.  m_out holds the degree reached (it may exceed 16; the paper prices it at
 *                       (m-1)+s products), no cap on s.  Up to n = 128 (fp32) / 96 (fp64) the whole loop runs on
 *                       chip in the fused kernel; above, every term is a product round over the matrices still in
 *                       the loop (as many rounds as the tolerance can ask for are enqueued, a matrix leaves them when
 *                       its term has dropped to tol), and the largest s is read back once to size the squaring
 *                       rounds -- so for larger n this scheme waits on the stream like expm() does by default, and
 *                       returns EXPM_ERR_UNSUPPORTED under stream capture.  expm_select_scheme runs the term loop
 *                       as well, since the degree is only known at its end.
 * All other arguments, blocking behaviour, ownership and status codes are as for expm_select / expm.
 */
#define EXPM_SCHEME_SASTRE   0
#define EXPM_SCHEME_PS       1
#define EXPM_SCHEME_BASELINE 2
#define EXPM_SCHEME_LOWRANK_CORE 3  /* reported by expm_get_stats() after expm_lowrank(); not an argument value */
int expm_select_scheme(const void *A, int n, int batch, int dtype, double tol, int scheme,
                       int32_t *m_out, int32_t *s_out);
int expm_scheme(const void *A, int n, int batch, int dtype, double tol, int scheme, void *out, void *stream);

/*
 * Same again with the norm of the selection as an argument.  The printed algorithms use the 1-norm
 * (EXPM_NORM_ONE: largest column abs-sum, what every call above uses); the paper's PyTorch runs use the
 * infinity-norm, as their baseline does (Sec. 4.2): EXPM_NORM_INF takes the largest row abs-sum
 * of W and of its powers instead.  Only the selection changes; with EXPM_NORM_INF the result equals the
 * transpose of what EXPM_NORM_ONE gives for the transposed batch.
 */
#define EXPM_NORM_ONE 0
#define EXPM_NORM_INF 1
int expm_select_ex(const void *A, int n, int batch, int dtype, double tol, int scheme, int norm_kind,
                   int32_t *m_out, int32_t *s_out);
int expm_ex(const void *A, int n, int batch, int dtype, double tol, int scheme, int norm_kind, void *out,
            void *stream);

/*
 * Low-rank variant (Sec. 2.2): for W = A1 A2 with A1 n x t and A2 t x n,
 *     e^W = I + A1 (sum_{i=0..m} V^i / (i+1)!) A2,   V = A2 A1  (t x t),
 * evaluated without scaling (s = 0, as the paper prescribes for this variant).  The order m is the smallest of
 * 1, 2, 4, 6, 9, 12, 16 whose truncation bound ||V||_1^(m+1) / (m+2)! / (1 - ||V||_1/(m+3)) (the bound printed
 * with that equation; Theorem 3 with p = 1) is at most tol; the series is evaluated by Paterson-Stockmeyer
 * (powers up to V^j, Horner in V^j; the paper does not print optimised coefficients for this series).
 * ||V||_1 = 0 gives m = 0 and the exact result I + A1 A2.  If no order reaches tol (||V||_1 beyond about 1 at
 * tol = 2^-53, 2.9 at 1e-8) the largest order is used and EXPM_WARN_SCALING_CAP is reported: tolerance not
 * guaranteed.  A non-finite V gives m = -1 and an all-NaN result (EXPM_WARN_NONFINITE).
 *
 *   A1     DEVICE, const, [batch][n][t] row-major.      A2   DEVICE, const, [batch][t][n] row-major.
 *   n, t   >= 0; batch <= 65535.  Up to t = 128 (fp32) / 96 (fp64) the core series is evaluated on chip in one
 *          kernel; a larger core goes through the product rounds of expm() (powers V^2..V^4 for the whole batch,
 *          one round per Horner step; the call then waits once on the stream like expm(), unless captured).
 *   tol    as for expm_select.                           out  DEVICE, [batch][n][n], must not overlap A1, A2.
 *   m_out  HOST, int32[batch].
 * expm_lowrank_select is synchronous (null stream) and returns the warning; expm_lowrank is asynchronous on
 * `stream` and returns 0 or an error, its warnings surface through expm_get_stats() (n of the statistics is t,
 * products counts the t x t products of the core series).  Both use the cached workspace.  expm_lowrank only
 * enqueues kernels: once a call of the same shape has sized the workspace it may be recorded into a HIP graph
 * (same condition as for expm: the workspace must not grow while such a graph is in use).
 */
int expm_lowrank_select(const void *A1, const void *A2, int n, int t, int batch, int dtype, double tol,
                        int32_t *m_out);
int expm_lowrank(const void *A1, const void *A2, int n, int t, int batch, int dtype, double tol, void *out,
                 void *stream);

/*
 * Bytes of device workspace the library holds for a call of this shape (the fused
 * small-matrix path needs only the per-matrix records).  The workspace is allocated
 * on first use, grown when a larger shape arrives, reused otherwise, and released by
 * expm_shutdown().  Returns 0 for invalid arguments.
 */
size_t expm_workspace_bytes(int n, int batch, int dtype);

/* Grow the workspace now (so that later calls of this shape do not allocate). */
int expm_reserve(int n, int batch, int dtype);

/*
 * Statistics of the most recent expm()/expm_select() call.  Synchronises with the
 * stream of that call.  products = sum over matrices of pi(m)+s with pi = 0,0,1,2,3,4
 * for m = 0,1,2,4,8,15 (cost of the formulas of Sec. 3.1 plus one per squaring), resp.
 * pi = 0,0,1,2,3,4,5,6 for m = 0,1,2,4,6,9,12,16 with the Paterson-Stockmeyer scheme (Table 1).
 */
struct expm_stats {
    int64_t matrices;      /* batch of the call                                   */
    int64_t products;      /* matrix products the method asked for                */
    int32_t n;             /* matrix order                                        */
    int32_t dtype;
    int32_t rounds;        /* product rounds launched after the W^2 round (0 on the fused path) */
    int32_t warning;       /* 0, EXPM_WARN_NONFINITE or EXPM_WARN_SCALING_CAP (non-finite wins; warning_bits has both) */
    int32_t fused_path;    /* 1 if the single-kernel on-chip path ran             */
    int32_t scheme;        /* EXPM_SCHEME_* of the call                           */
    int64_t hist_m[17];    /* matrices with order m, indexed by m = 0..16 (baseline degrees above 16 in the last bin) */
    int64_t hist_s[21];    /* matrices with s = 0..20                             */
    int64_t nonfinite;     /* matrices flagged (-1,-1)                            */
    int32_t warning_bits;  /* bit 0: some matrix non-finite; bit 1: some matrix asked for more than the cap s = 20 */
    int32_t reserved;
};
int expm_get_stats(struct expm_stats *st /* HOST */);

/*
 * Kernel timing hooks for benchmarks.  With profiling enabled, expm() brackets every
 * kernel launch with HIP events on the caller's stream (this adds launch gaps: do not
 * time throughput with it on).  expm_profile_read() synchronises and returns, per
 * kernel class, the launch count, the summed event time in milliseconds and the summed
 * algorithmic FLOPs (2 n^3 per product actually launched) since the last reset.
 */
#define EXPM_KCLASS_NORM   0   /* column abs-sum passes and norm reductions */
#define EXPM_KCLASS_SELECT 1   /* selection / plan / operand preparation    */
#define EXPM_KCLASS_GEMM   2   /* grouped MFMA product rounds               */
#define EXPM_KCLASS_FUSED  3   /* single-kernel small-matrix path           */
#define EXPM_KCLASS_COUNT  4
struct expm_profile {
    int64_t launches[EXPM_KCLASS_COUNT];
    double  ms[EXPM_KCLASS_COUNT];
    double  flops[EXPM_KCLASS_COUNT];
    double  bytes[EXPM_KCLASS_COUNT];   /* algorithmic HBM bytes (compulsory reads + writes) */
};
int expm_profile_enable(int on);
int expm_profile_reset(void);
int expm_profile_read(struct expm_profile *p /* HOST */);

/* Release the workspace and cached events.  Safe to call repeatedly. */
int expm_shutdown(void);

/* hipError_t of the last failing HIP call (0 if none). */
int expm_last_hip_error(void);

/* Static, human-readable text for a status code. */
const char *expm_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* EXPM_MI355X_H */
