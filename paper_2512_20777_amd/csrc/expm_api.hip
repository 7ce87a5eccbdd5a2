// C ABI, workspace management and round dispatcher of the gfx950 expm library.
// Interface contract: include/expm_mi355x.h.
#include "../../include/expm_mi355x.h"
#include "expm_internal.h"

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <vector>

namespace {

using namespace expmk;

// Everything the library keeps between calls is kept per device: the cached workspace block, the pinned mirror of
// the plan summary, the side streams and events of the round-based path, and the address of that device's copy of
// the static scratch array.
constexpr int kMaxDevices = 16;
constexpr int kChains = 2;                        // chains of rounds that run side by side below n = 1024

struct DeviceState {
    void *dev = nullptr;      // one device block (workspace), grown on demand
    size_t bytes = 0;
    int *host_summary = nullptr;  // pinned, 64 ints
    hipEvent_t summary_ready = nullptr;
    hipStream_t side_stream = nullptr;          // norm of W beside the W^2 round (default priority)
    hipEvent_t fork = nullptr, join = nullptr;
    hipStream_t chain_stream[kChains] = {};     // [0] unused (the caller's stream), [1] = side_stream, rest their own
    hipEvent_t chain_join[kChains] = {};
    hipEvent_t order_event = nullptr;           // orders a call behind the previous one when the stream changes
    unsigned char *scratch_ptr = nullptr;       // device address of this device's copy of `scratch`
};

struct LastCall {
    bool valid = false;
    int n = 0, batch = 0, dtype = 0;
    int rounds = 0;           // -1: the rounds were planned on the device; the statistics derive them from the records
    int fused = 0;
    int scheme = 0;
    int device = 0;
    bool stream_usable = false;  // false after a call made under stream capture (the stream cannot be waited on)
    hipStream_t stream = nullptr;
    MatInfo *info_dev = nullptr;
    int *summary_dev = nullptr;
};

struct ProfEvent {
    hipEvent_t start, stop;
    int kclass;
    double flops, bytes;
};

// Scratch for the entry point that must not allocate (expm_noalloc): its control block and matrix stacks live here
// instead of in the cached workspace.  Every GPU the library runs on holds its own copy at its own address
// (hipGetSymbolAddress with that device current); in host code the name below is only a handle for that lookup.
constexpr size_t kStaticScratchBytes = (size_t)EXPM_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

DeviceState g_dev[kMaxDevices];
std::vector<MatInfo> g_host_info;   // pageable mirror of the per-matrix records for stats / select
std::mutex g_mutex;                 // entry points that touch the state above run one at a time
LastCall g_last;
int g_last_hip_error = 0;
bool g_profile = false;
bool g_brackets = false;            // per call: g_profile, except in calls that must not create events
std::vector<ProfEvent> g_events;
std::vector<hipEvent_t> g_event_pool;

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

int hip_fail(hipError_t e)
{
    g_last_hip_error = (int)e;
    (void)hipGetLastError();
    return EXPM_ERR_HIP;
}
#define EXPM_TRY(expr)                                  \
    do {                                                \
        hipError_t e__ = (expr);                        \
        if (e__ != hipSuccess) return hip_fail(e__);    \
    } while (0)

struct Layout {
    size_t info, order, summary, n1, n2, n3, n4, colpart, colpart_w, mats, total;
    size_t mat_bytes;
};

// Device workspace layout: control block first, then 7 matrix-stack buffers (W2, T0..T5) for the
// round-based path.  The fused path only needs the control block.
Layout make_layout(int n, int batch, int dtype)
{
    Layout L{};
    const size_t w = dtype == EXPM_DTYPE_F64 ? 8 : 4;
    size_t off = 0;
    L.summary = off; off = align_up(off + 64 * sizeof(int), 256);
    L.info = off;    off = align_up(off + (size_t)batch * sizeof(MatInfo), 256);
    L.order = off;   off = align_up(off + (size_t)batch * sizeof(int), 256);
    const size_t nblk = (size_t)general_colblocks(n);
    L.n1 = off;      off = align_up(off + (size_t)batch * nblk * sizeof(double), 256);
    L.n2 = off;      off = align_up(off + (size_t)batch * nblk * sizeof(double), 256);
    L.n3 = off;      off = align_up(off + (size_t)batch * nblk * sizeof(double), 256);
    L.n4 = off;      off = align_up(off + (size_t)batch * nblk * sizeof(double), 256);
    L.mat_bytes = 0;
    L.colpart = off;
    L.colpart_w = off;
    L.mats = off;
    if (!small_path_supported(n, dtype)) {
        // column-sum partials: 32-row chunks for W, one per tile row (>= 32 rows) for the powers
        off = align_up(off + (size_t)batch * general_colchunks(n) * n * sizeof(double), 256);
        L.colpart_w = off;
        off = align_up(off + (size_t)batch * general_colchunks(n) * n * sizeof(double), 256);
        L.mats = off;
        L.mat_bytes = align_up((size_t)batch * n * n * w, 256);
        off += 7 * L.mat_bytes;
    }
    L.total = off;
    return L;
}

// State of the device that is current on this thread.
int current_device(DeviceState **ds, int *index = nullptr)
{
    int dev = 0;
    EXPM_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return EXPM_ERR_INVALID_ARG;
    *ds = &g_dev[dev];
    if (index) *index = dev;
    return EXPM_OK;
}

int ensure_workspace(DeviceState *ds, size_t bytes)
{
    if (bytes <= ds->bytes) return EXPM_OK;
    if (ds->dev) {
        // earlier calls may still be using the old block
        hipError_t e = hipDeviceSynchronize();
        if (e != hipSuccess) return hip_fail(e);
        (void)hipFree(ds->dev);
        ds->dev = nullptr;
        ds->bytes = 0;
        g_last.valid = false;
    }
    void *p = nullptr;
    hipError_t e = hipMalloc(&p, bytes);
    if (e != hipSuccess) { g_last_hip_error = (int)e; (void)hipGetLastError(); return EXPM_ERR_ALLOC; }
    ds->dev = p;
    ds->bytes = bytes;
    return EXPM_OK;
}

int ensure_host_summary(DeviceState *ds)
{
    if (ds->host_summary) return EXPM_OK;
    hipError_t e = hipHostMalloc(reinterpret_cast<void **>(&ds->host_summary), 64 * sizeof(int), hipHostMallocDefault);
    if (e != hipSuccess) { g_last_hip_error = (int)e; (void)hipGetLastError(); return EXPM_ERR_ALLOC; }
    return EXPM_OK;
}

bool stream_is_capturing(hipStream_t stream)
{
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &cs) != hipSuccess) { (void)hipGetLastError(); return false; }
    return cs == hipStreamCaptureStatusActive;
}

// All calls on one device share that device's workspace.  A call on another stream than the previous call's is
// therefore ordered behind everything queued on that stream so far (an event recorded there now, waited for here):
// calls on several streams then run one after another instead of overwriting each other's intermediates.
int order_behind_last_call(DeviceState *ds, int dev, hipStream_t stream)
{
    if (!g_last.valid || !g_last.stream_usable || g_last.device != dev || g_last.stream == stream) return EXPM_OK;
    if (!ds->order_event) EXPM_TRY(hipEventCreateWithFlags(&ds->order_event, hipEventDisableTiming));
    if (hipEventRecord(ds->order_event, g_last.stream) != hipSuccess) {
        (void)hipGetLastError();   // the caller has destroyed that stream: its work was finished or abandoned with it
        return EXPM_OK;
    }
    EXPM_TRY(hipStreamWaitEvent(stream, ds->order_event, 0));
    return EXPM_OK;
}

int check_args(const void *A, int n, int batch, int dtype, double &tol)
{
    if (n < 0 || batch < 0) return EXPM_ERR_INVALID_ARG;
    if (dtype != EXPM_DTYPE_F32 && dtype != EXPM_DTYPE_F64) return EXPM_ERR_INVALID_ARG;
    if ((n > 0 && batch > 0) && A == nullptr) return EXPM_ERR_INVALID_ARG;
    if (n > 46340) return EXPM_ERR_INVALID_ARG;  // n*n must fit the kernels' int tile arithmetic
    if ((double)batch * (double)n * (double)n > 9.0e15) return EXPM_ERR_INVALID_ARG;
    if (!small_path_supported(n, dtype)) {
        // round-based path: the batch is a grid dimension and (matrices x tiles) must fit an int
        const double tiles = (double)((n + 31) / 32);
        if (batch > 65535 || (double)batch * tiles * tiles > 2.0e9) return EXPM_ERR_INVALID_ARG;
    }
    const double u = dtype == EXPM_DTYPE_F64 ? ldexp(1.0, -53) : ldexp(1.0, -24);
    if (!(tol == tol) || tol < 0.0) return EXPM_ERR_TOLERANCE;
    if (tol == 0.0) tol = u;
    if (tol < u) return EXPM_ERR_TOLERANCE;
    return EXPM_OK;
}

// ---- profiling brackets ---------------------------------------------------------------------------
hipEvent_t get_event()
{
    if (!g_event_pool.empty()) {
        hipEvent_t e = g_event_pool.back();
        g_event_pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

struct Bracket {
    hipStream_t stream;
    ProfEvent ev{};
    bool on;
    Bracket(hipStream_t s, int kclass, double flops, double bytes) : stream(s), on(g_brackets)
    {
        if (!on) return;
        ev.start = get_event();
        ev.stop = get_event();
        ev.kclass = kclass;
        ev.flops = flops;
        ev.bytes = bytes;
        if (!ev.start || !ev.stop) { on = false; return; }
        (void)hipEventRecord(ev.start, stream);
    }
    ~Bracket()
    {
        if (!on) return;
        (void)hipEventRecord(ev.stop, stream);
        g_events.push_back(ev);
    }
};

// Warnings are independent bits; the status code can carry one: a non-finite matrix (results missing) outranks a
// scaling that hit the cap (results delivered, tolerance not guaranteed).  expm_stats.warning_bits carries both.
int warning_from_flags(int flags)
{
    if (flags & 1) return EXPM_WARN_NONFINITE;
    if (flags & 2) return EXPM_WARN_SCALING_CAP;
    return EXPM_OK;
}

struct Bound {
    GeneralBuffers gb;
    Layout L;
};

Bound bind(unsigned char *base, const void *A, void *out, int n, int batch, int dtype, int norm_kind)
{
    Bound B;
    B.gb.norm_inf = norm_kind == EXPM_NORM_INF ? 1 : 0;
    B.L = make_layout(n, batch, dtype);
    B.gb.summary = reinterpret_cast<int *>(base + B.L.summary);
    B.gb.info = reinterpret_cast<MatInfo *>(base + B.L.info);
    B.gb.order = reinterpret_cast<int *>(base + B.L.order);
    B.gb.n1 = reinterpret_cast<double *>(base + B.L.n1);
    B.gb.n2 = reinterpret_cast<double *>(base + B.L.n2);
    B.gb.n3 = reinterpret_cast<double *>(base + B.L.n3);
    B.gb.n4 = reinterpret_cast<double *>(base + B.L.n4);
    B.gb.colpart = reinterpret_cast<double *>(base + B.L.colpart);
    B.gb.colpart_w = reinterpret_cast<double *>(base + B.L.colpart_w);
    B.gb.base[BUF_W] = const_cast<void *>(A);
    for (int i = 0; i < 7; ++i) B.gb.base[BUF_W2 + i] = base + B.L.mats + (size_t)i * B.L.mat_bytes;
    B.gb.base[BUF_OUT] = out;
    B.gb.ptr_align16 = (((uintptr_t)A | (uintptr_t)out) % 16) == 0;
    return B;
}

// Selection stage of the round-based path: norms, W2, (m,s), plan.  With `readback` the plan summary also travels
// to pinned host memory (the caller waits on summary_ready); without it the stage only enqueues kernels on `stream`.
int run_selection_general(DeviceState *ds, const Bound &B, int n, int batch, int dtype, double tol, int scheme,
                          hipStream_t stream, bool readback)
{
    const double w = dtype == EXPM_DTYPE_F64 ? 8.0 : 4.0;
    const double nn = (double)n * n;
    // The norm of W needs nothing but W: its two kernels run on a side stream beside the W^2 round (they fill
    // the compute units that round leaves idle towards its end) and join before the selection.  With the
    // per-class timers on, everything stays on the caller's stream so that each class is timed by itself.
    // (only for matrices below 1024: beyond that the pass is a fraction of a percent of the call, and its reads
    // beside the start of a long product round cost that round more than they save)
    const bool side = readback && !g_brackets && n < 1024;
    if (side) {
        if (!ds->side_stream) {
            EXPM_TRY(hipStreamCreateWithFlags(&ds->side_stream, hipStreamNonBlocking));
            EXPM_TRY(hipEventCreateWithFlags(&ds->fork, hipEventDisableTiming));
            EXPM_TRY(hipEventCreateWithFlags(&ds->join, hipEventDisableTiming));
        }
        EXPM_TRY(hipEventRecord(ds->fork, stream));
        EXPM_TRY(hipStreamWaitEvent(ds->side_stream, ds->fork, 0));
    }
    {
        hipStream_t ns = side ? ds->side_stream : stream;
        Bracket br(stream, EXPM_KCLASS_NORM, 0.0, batch * nn * w);
        EXPM_TRY(launch_colabs(B.gb, n, batch, dtype, ns));
        EXPM_TRY(launch_colmax(B.gb, n, batch, 1, B.gb.norm_inf ? 1 : general_colchunks(n), ns));
    }
    if (side) EXPM_TRY(hipEventRecord(ds->join, ds->side_stream));
    const int wt0 = choose_tile_shape(n, batch);
    {
        Bracket br(stream, EXPM_KCLASS_GEMM, 2.0 * nn * n * batch, 2.0 * batch * nn * w);
        EXPM_TRY(launch_power_round(B.gb, n, batch, dtype, wt0, 2, stream));
    }
    {
        Bracket br(stream, EXPM_KCLASS_NORM, 0.0, 0.0);
        EXPM_TRY(launch_colmax(B.gb, n, batch, 2, (n + 32 * wt0 - 1) / (32 * wt0), stream));
    }
    if (scheme == kSchemePS || scheme == kSchemePhi) {
        // Algorithm 3 looks at ||W^3|| and ||W^4|| as well: W^3 = W^2 W, W^4 = W^3 W for the whole batch
        // (the core series of the low-rank variant only needs the powers, formed here for all orders alike)
        for (int which = 3; which <= 4; ++which) {
            {
                Bracket br(stream, EXPM_KCLASS_GEMM, 2.0 * nn * n * batch, 2.0 * batch * nn * w);
                EXPM_TRY(launch_power_round(B.gb, n, batch, dtype, wt0, which, stream));
            }
            Bracket br(stream, EXPM_KCLASS_NORM, 0.0, 0.0);
            EXPM_TRY(launch_colmax(B.gb, n, batch, which, (n + 32 * wt0 - 1) / (32 * wt0), stream));
        }
    }
    if (side) EXPM_TRY(hipStreamWaitEvent(stream, ds->join, 0));
    {
        Bracket br(stream, EXPM_KCLASS_SELECT, 0.0, 0.0);
        EXPM_TRY(launch_select_plan(B.gb, n, batch, tol, scheme, stream));
    }
    if (readback) {
        // the plan summary travels to pinned host memory; summary_ready marks the copy, so that the
        // caller can queue more work behind it before waiting
        EXPM_TRY(hipMemcpyAsync(ds->host_summary, B.gb.summary, 64 * sizeof(int), hipMemcpyDeviceToHost, stream));
        if (!ds->summary_ready) EXPM_TRY(hipEventCreateWithFlags(&ds->summary_ready, hipEventDisableTiming));
        EXPM_TRY(hipEventRecord(ds->summary_ready, stream));
    }
    return EXPM_OK;
}

void remember(int n, int batch, int dtype, int rounds, int fused, int scheme, int dev, hipStream_t stream, bool usable,
              MatInfo *info, int *summary)
{
    g_last.valid = true;
    g_last.scheme = scheme;
    g_last.n = n; g_last.batch = batch; g_last.dtype = dtype;
    g_last.rounds = rounds; g_last.fused = fused; g_last.stream = stream;
    g_last.device = dev;
    g_last.stream_usable = usable;
    g_last.info_dev = info;
    g_last.summary_dev = summary;
}

constexpr long long kTwoChainTiles = 1024;  // 64 x 64 tiles in round 2 from which the rounds run as two chains

// Profiling aids read once from the environment: EXPM_CHAINS=1 keeps one chain of rounds (a kernel trace then
// shows launches that do not overlap); EXPM_PLAN=device|host forces where the rounds are planned.
int env_chain_limit()
{
    static const int v = [] {
        const char *e = getenv("EXPM_CHAINS");
        const int x = e ? atoi(e) : 0;
        return x >= 1 && x <= kChains ? x : kChains;
    }();
    return v;
}
int env_plan()   // 0: library's choice, 1: on the device, 2: on the host
{
    static const int v = [] {
        const char *e = getenv("EXPM_PLAN");
        if (!e) return 0;
        return strcmp(e, "device") == 0 ? 1 : (strcmp(e, "host") == 0 ? 2 : 0);
    }();
    return v;
}

// Where the rounds of a call on the round-based path are planned when the caller leaves the choice to the library.
// Planning on the device never blocks the host but launches every possible round (workgroups of rounds a matrix
// does not need leave at once: about 2.6 us per such launch); planning on the host waits once for 256 bytes and
// launches exactly the rounds needed, each with the tile shape that suits the matrices still active.
bool plan_on_device_by_default(int n, int batch)
{
    (void)n; (void)batch;
    return false;
}

// The rounds of one call on the round-based path.  plan_on_device: only kernels are enqueued, on `stream` alone.
int run_rounds(DeviceState *ds, const Bound &B, int n, int batch, int dtype, double tol, int scheme, hipStream_t stream,
               bool plan_on_device, int *rounds_out, int *warning_out)
{
    const double w = dtype == EXPM_DTYPE_F64 ? 8.0 : 4.0;
    const double nn = (double)n * n;
    *warning_out = EXPM_OK;
    if (!plan_on_device) {
        int rc = ensure_host_summary(ds);
        if (rc != EXPM_OK) return rc;
    }
    int rc = run_selection_general(ds, B, n, batch, dtype, tol, scheme, stream, !plan_on_device);
    if (rc != EXPM_OK) return rc;
    // Work that does not need the host's view of the plan is queued before the wait, so the device
    // stays busy while the summary is read: operand preparation, and the first chain round over the
    // whole batch (workgroups of matrices that need no product leave at once).
    if (first_round_is_self_contained(n, scheme)) {
        // no preparation pass: round 1 combines W^2 and W while it stages its tiles and finishes orders <= 2 itself
        Bracket br(stream, EXPM_KCLASS_GEMM, 0.0, 0.0);  // its work is filled in once the plan is known
        EXPM_TRY(launch_first_round(B.gb, n, batch, dtype, stream));
    } else {
        {
            Bracket br(stream, EXPM_KCLASS_SELECT, 0.0, 0.0);
            EXPM_TRY(launch_prepare(B.gb, n, batch, dtype, scheme, stream));
        }
        Bracket br(stream, EXPM_KCLASS_GEMM, 0.0, 0.0);  // its work is filled in once the plan is known
        EXPM_TRY(launch_chain_round(B.gb, n, batch, 1, dtype, choose_tile_shape(n, batch), scheme, stream));
    }
    if (plan_on_device) {
        // Every round a matrix can need (3 + 20 for both schemes), each over the whole sorted list: a workgroup looks
        // up its matrix's chain length and leaves if the round is beyond it.
        const int wt = choose_tile_shape(n, batch);
        for (int r = 2; r <= kMaxRounds; ++r)
            EXPM_TRY(launch_chain_round(B.gb, n, batch, r, dtype, wt, scheme, stream, 0, 1, true));
        *rounds_out = -1;
        return EXPM_OK;
    }
    const size_t round1_event = g_events.size();
    EXPM_TRY(hipEventSynchronize(ds->summary_ready));
    const int longest = ds->host_summary[0];
    const int flags = ds->host_summary[1];
    if (g_brackets && round1_event > 0) {
        const int active1 = longest >= 1 ? ds->host_summary[3] : 0;
        g_events[round1_event - 1].flops = 2.0 * nn * n * active1;
        g_events[round1_event - 1].bytes = 2.0 * active1 * nn * w;
    }
    // Rounds 2.. : a matrix's round r needs only its own round r-1.  Below n = 1024 the sorted matrices are dealt
    // alternately to kChains streams, each with its own chain of rounds: while one chain's launch runs out of
    // workgroups towards its end, the other's fills the compute units (a single chain leaves them idle there,
    // 8 % of the call for 32 matrices of 512 x 512).  With the per-class timers on, one chain on the caller's
    // stream, so that launches do not overlap and each is timed by itself.
    // A round that does not even give every compute unit four 64 x 64 tiles gains nothing from a second chain and
    // pays for the fork and the join (8 matrices of 256 x 256 fp64: 0.113 ms on one chain, 0.143 ms on two; 12 of
    // 512 x 512: 0.523 / 0.550; from 16 of 512 x 512 on two chains win).
    int chains = 1;
    const long long tiles64 = (long long)ds->host_summary[4] * ((n + 63) / 64) * ((n + 63) / 64);  // round 2
    if (!g_brackets && n < 1024 && longest >= 2 && tiles64 >= kTwoChainTiles && ds->side_stream != nullptr)
        chains = std::min(env_chain_limit(), ds->host_summary[4]);
    if (chains > 1) {
        EXPM_TRY(hipEventRecord(ds->fork, stream));
        for (int c = 1; c < chains; ++c) {
            if (!ds->chain_stream[c]) {
                if (c == 1) ds->chain_stream[c] = ds->side_stream;
                else EXPM_TRY(hipStreamCreateWithFlags(&ds->chain_stream[c], hipStreamNonBlocking));
                EXPM_TRY(hipEventCreateWithFlags(&ds->chain_join[c], hipEventDisableTiming));
            }
            EXPM_TRY(hipStreamWaitEvent(ds->chain_stream[c], ds->fork, 0));
        }
    }
    for (int r = 2; r <= longest && r <= kMaxRounds; ++r) {
        const int active = ds->host_summary[2 + r];
        if (active <= 0) break;
        if (chains > 1) {
            for (int c = 0; c < chains; ++c) {
                const int mine = (active - c + chains - 1) / chains;  // sorted matrices c, c + chains, ... below active
                if (mine <= 0) break;
                EXPM_TRY(launch_chain_round(B.gb, n, mine, r, dtype, choose_tile_shape(n, mine), scheme,
                                            c == 0 ? stream : ds->chain_stream[c], c, chains));
            }
            continue;
        }
        Bracket br(stream, EXPM_KCLASS_GEMM, 2.0 * nn * n * active, 2.0 * active * nn * w);
        EXPM_TRY(launch_chain_round(B.gb, n, active, r, dtype, choose_tile_shape(n, active), scheme, stream));
    }
    for (int c = 1; c < chains; ++c) {
        EXPM_TRY(hipEventRecord(ds->chain_join[c], ds->chain_stream[c]));
        EXPM_TRY(hipStreamWaitEvent(stream, ds->chain_join[c], 0));
    }
    *rounds_out = longest;
    *warning_out = warning_from_flags(flags);
    return EXPM_OK;
}

// Baseline of the paper's comparison (its Algorithm 1) on the round-based path.  The term rounds are planned on the
// device: as many as the tolerance can ask for are launched over the whole batch (a matrix whose last term has
// dropped to the tolerance leaves them), each followed by the norm reduction of the new term and the decision who
// goes on.  The scalings follow from ||W|| alone: the largest travels to the host while the term rounds run, and
// exactly that many squaring rounds follow (Algorithm 1 has no cap on s, so these cannot be launched blind).
int run_baseline_rounds(DeviceState *ds, const Bound &B, int n, int batch, int dtype, double tol, hipStream_t stream,
                        bool select_only, int *rounds_out, int *warning_out)
{
    const double w = dtype == EXPM_DTYPE_F64 ? 8.0 : 4.0;
    const double nn = (double)n * n;
    *warning_out = EXPM_OK;
    int rc = ensure_host_summary(ds);
    if (rc != EXPM_OK) return rc;
    {
        Bracket br(stream, EXPM_KCLASS_NORM, 0.0, batch * nn * w);
        EXPM_TRY(launch_colabs(B.gb, n, batch, dtype, stream));
        EXPM_TRY(launch_colmax(B.gb, n, batch, 1, B.gb.norm_inf ? 1 : general_colchunks(n), stream));
    }
    {
        Bracket br(stream, EXPM_KCLASS_SELECT, 0.0, 0.0);
        EXPM_TRY(launch_baseline_decide(B.gb, n, batch, tol, 0, stream));
    }
    EXPM_TRY(hipMemcpyAsync(ds->host_summary, B.gb.summary, 64 * sizeof(int), hipMemcpyDeviceToHost, stream));
    if (!ds->summary_ready) EXPM_TRY(hipEventCreateWithFlags(&ds->summary_ready, hipEventDisableTiming));
    EXPM_TRY(hipEventRecord(ds->summary_ready, stream));
    const int wt = choose_tile_shape(n, batch);
    const int terms = baseline_max_terms(tol);
    for (int t = 1; t <= terms; ++t) {
        {
            Bracket br(stream, EXPM_KCLASS_GEMM, 0.0, 0.0);   // how many matrices are still in the loop is known on the device only
            EXPM_TRY(launch_baseline_round(B.gb, n, batch, t, dtype, wt, select_only, stream));
        }
        Bracket br(stream, EXPM_KCLASS_SELECT, 0.0, 0.0);
        EXPM_TRY(launch_colmax(B.gb, n, batch, 2, (n + 32 * wt - 1) / (32 * wt), stream));
        EXPM_TRY(launch_baseline_decide(B.gb, n, batch, tol, t, stream));
    }
    EXPM_TRY(hipEventSynchronize(ds->summary_ready));
    const int smax = ds->host_summary[0];
    *warning_out = warning_from_flags(ds->host_summary[1]);
    if (!select_only) {
        for (int q = 1; q <= smax; ++q) {
            Bracket br(stream, EXPM_KCLASS_GEMM, 0.0, 0.0);
            EXPM_TRY(launch_baseline_round(B.gb, n, batch, kBaselineSquareRound + q, dtype, wt, false, stream));
        }
    }
    *rounds_out = terms + (select_only ? 0 : smax);
    return EXPM_OK;
}

constexpr int kModeCached = 0;   // workspace from the cached block (allocated and grown on demand)
constexpr int kModeStatic = 1;   // workspace in the static scratch array: no allocation of any kind

int expm_impl(const void *A, int n, int batch, int dtype, double tol, int scheme, int norm_kind, void *out, void *stream_v,
              int mode)
{
    if (scheme != EXPM_SCHEME_SASTRE && scheme != EXPM_SCHEME_PS && scheme != EXPM_SCHEME_BASELINE)
        return EXPM_ERR_INVALID_ARG;
    if (norm_kind != EXPM_NORM_ONE && norm_kind != EXPM_NORM_INF) return EXPM_ERR_INVALID_ARG;
    int rc = check_args(A, n, batch, dtype, tol);
    if (rc != EXPM_OK) return rc;
    if (n == 0 || batch == 0) return EXPM_OK;
    if (out == nullptr) return EXPM_ERR_INVALID_ARG;
    {
        const size_t bytes = (size_t)batch * n * n * (dtype == EXPM_DTYPE_F64 ? 8 : 4);
        const uintptr_t a0 = (uintptr_t)A, o0 = (uintptr_t)out;
        if (a0 < o0 + bytes && o0 < a0 + bytes) return EXPM_ERR_INVALID_ARG;  // overlap
        if ((a0 | o0) % (dtype == EXPM_DTYPE_F64 ? 8 : 4)) return EXPM_ERR_INVALID_ARG;
    }
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    const Layout L = make_layout(n, batch, dtype);
    if (mode == kModeStatic && L.total > kStaticScratchBytes) return EXPM_ERR_WORKSPACE;   // before any device work
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState *ds = nullptr;
    int dev = 0;
    rc = current_device(&ds, &dev);
    if (rc != EXPM_OK) return rc;
    const bool capturing = stream_is_capturing(stream);
    unsigned char *base = nullptr;
    if (mode == kModeStatic) {
        if (!ds->scratch_ptr) {
            // once per device, with that device current: where this device keeps its copy of the array
            void *p = nullptr;
            EXPM_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
            ds->scratch_ptr = static_cast<unsigned char *>(p);
        }
        base = ds->scratch_ptr;
    } else {
        if (capturing && L.total > ds->bytes) return EXPM_ERR_WORKSPACE;   // a capture cannot allocate: expm_reserve first
        rc = ensure_workspace(ds, L.total);
        if (rc != EXPM_OK) return rc;
        base = static_cast<unsigned char *>(ds->dev);
        if (!capturing) {
            rc = order_behind_last_call(ds, dev, stream);
            if (rc != EXPM_OK) return rc;
        }
    }
    g_brackets = g_profile && mode == kModeCached && !capturing;
    const Bound B = bind(base, A, out, n, batch, dtype, norm_kind);
    const double w = dtype == EXPM_DTYPE_F64 ? 8.0 : 4.0;
    const double nn = (double)n * n;

    if (small_path_supported(n, dtype)) {
        // one kernel, nothing read back: warnings of this path surface through expm_get_stats()
        {
            Bracket br(stream, EXPM_KCLASS_FUSED, 0.0, 2.0 * batch * nn * w);
            EXPM_TRY(launch_small(A, out, n, batch, dtype, tol, 0, scheme, B.gb.norm_inf, B.gb.info, stream));
        }
        remember(n, batch, dtype, 0, 1, scheme, dev, stream, !capturing, B.gb.info, B.gb.summary);
        return EXPM_OK;
    }
    bool on_device = mode == kModeStatic || capturing;
    int rounds = 0, warning = EXPM_OK;
    if (scheme == EXPM_SCHEME_BASELINE) {
        // its squarings have no cap, so their number has to be read back: not under capture
        if (on_device) return EXPM_ERR_UNSUPPORTED;
        rc = run_baseline_rounds(ds, B, n, batch, dtype, tol, stream, false, &rounds, &warning);
        if (rc != EXPM_OK) return rc;
        remember(n, batch, dtype, rounds, 0, scheme, dev, stream, true, B.gb.info, B.gb.summary);
        return warning;
    }
    if (!on_device) on_device = env_plan() == 1 || (env_plan() == 0 && plan_on_device_by_default(n, batch));
    rc = run_rounds(ds, B, n, batch, dtype, tol, scheme, stream, on_device, &rounds, &warning);
    if (rc != EXPM_OK) return rc;
    remember(n, batch, dtype, rounds, 0, scheme, dev, stream, !capturing, B.gb.info, B.gb.summary);
    return warning;
}

}  // namespace

extern "C" {

size_t expm_workspace_bytes(int n, int batch, int dtype)
{
    double tol = 0.0;
    int dummy = 0;
    if (check_args(&dummy, n, batch, dtype, tol) != EXPM_OK) return 0;
    if (n == 0 || batch == 0) return 0;
    return make_layout(n, batch, dtype).total;
}

int expm_reserve(int n, int batch, int dtype)
{
    double tol = 0.0;
    int dummy = 0;
    int rc = check_args(&dummy, n, batch, dtype, tol);
    if (rc != EXPM_OK) return rc;
    if (n == 0 || batch == 0) return EXPM_OK;
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState *ds = nullptr;
    rc = current_device(&ds);
    if (rc != EXPM_OK) return rc;
    return ensure_workspace(ds, make_layout(n, batch, dtype).total);
}

int expm_select(const void *A, int n, int batch, int dtype, double tol, int32_t *m_out, int32_t *s_out)
{
    return expm_select_scheme(A, n, batch, dtype, tol, EXPM_SCHEME_SASTRE, m_out, s_out);
}

int expm_select_scheme(const void *A, int n, int batch, int dtype, double tol, int scheme, int32_t *m_out, int32_t *s_out)
{
    return expm_select_ex(A, n, batch, dtype, tol, scheme, EXPM_NORM_ONE, m_out, s_out);
}

int expm_select_ex(const void *A, int n, int batch, int dtype, double tol, int scheme, int norm_kind, int32_t *m_out,
                   int32_t *s_out)
{
    if (scheme != EXPM_SCHEME_SASTRE && scheme != EXPM_SCHEME_PS && scheme != EXPM_SCHEME_BASELINE)
        return EXPM_ERR_INVALID_ARG;
    if (norm_kind != EXPM_NORM_ONE && norm_kind != EXPM_NORM_INF) return EXPM_ERR_INVALID_ARG;
    int rc = check_args(A, n, batch, dtype, tol);
    if (rc != EXPM_OK) return rc;
    if (batch > 0 && (m_out == nullptr || s_out == nullptr)) return EXPM_ERR_INVALID_ARG;
    if (batch == 0) return EXPM_OK;
    if (n == 0) {
        for (int b = 0; b < batch; ++b) { m_out[b] = 0; s_out[b] = 0; }
        return EXPM_OK;
    }
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState *ds = nullptr;
    int dev = 0;
    rc = current_device(&ds, &dev);
    if (rc != EXPM_OK) return rc;
    rc = ensure_workspace(ds, make_layout(n, batch, dtype).total);
    if (rc != EXPM_OK) return rc;
    hipStream_t stream = nullptr;
    rc = order_behind_last_call(ds, dev, stream);
    if (rc != EXPM_OK) return rc;
    g_brackets = false;
    const Bound B = bind(static_cast<unsigned char *>(ds->dev), A, nullptr, n, batch, dtype, norm_kind);
    int flags = 0;
    if (small_path_supported(n, dtype)) {
        EXPM_TRY(launch_small(A, nullptr, n, batch, dtype, tol, 1, scheme, B.gb.norm_inf, B.gb.info, stream));
        remember(n, batch, dtype, 0, 1, scheme, dev, stream, true, B.gb.info, B.gb.summary);
    } else if (scheme == EXPM_SCHEME_BASELINE) {
        // the degree is only known once the term loop has run: all of it, without the squarings
        int rounds = 0, warning = EXPM_OK;
        rc = run_baseline_rounds(ds, B, n, batch, dtype, tol, stream, true, &rounds, &warning);
        if (rc != EXPM_OK) return rc;
        remember(n, batch, dtype, rounds, 0, scheme, dev, stream, true, B.gb.info, B.gb.summary);
    } else {
        rc = run_selection_general(ds, B, n, batch, dtype, tol, scheme, stream, false);
        if (rc != EXPM_OK) return rc;
        remember(n, batch, dtype, 0, 0, scheme, dev, stream, true, B.gb.info, B.gb.summary);
    }
    g_host_info.resize((size_t)batch);
    EXPM_TRY(hipMemcpyAsync(g_host_info.data(), B.gb.info, (size_t)batch * sizeof(MatInfo), hipMemcpyDeviceToHost, stream));
    EXPM_TRY(hipStreamSynchronize(stream));
    for (int b = 0; b < batch; ++b) {
        m_out[b] = g_host_info[b].m;
        s_out[b] = g_host_info[b].s;
        flags |= g_host_info[b].flags;
    }
    return warning_from_flags(flags);
}

int expm(const void *A, int n, int batch, int dtype, double tol, void *out, void *stream_v)
{
    return expm_impl(A, n, batch, dtype, tol, EXPM_SCHEME_SASTRE, EXPM_NORM_ONE, out, stream_v, kModeCached);
}

int expm_scheme(const void *A, int n, int batch, int dtype, double tol, int scheme, void *out, void *stream_v)
{
    return expm_impl(A, n, batch, dtype, tol, scheme, EXPM_NORM_ONE, out, stream_v, kModeCached);
}

int expm_ex(const void *A, int n, int batch, int dtype, double tol, int scheme, int norm_kind, void *out, void *stream_v)
{
    return expm_impl(A, n, batch, dtype, tol, scheme, norm_kind, out, stream_v, kModeCached);
}

int expm_noalloc(const void *A, int n, int batch, int dtype, double tol, void *out, void *stream_v)
{
    return expm_impl(A, n, batch, dtype, tol, EXPM_SCHEME_SASTRE, EXPM_NORM_ONE, out, stream_v, kModeStatic);
}

// ---- low-rank variant (Sec. 2.2): e^(A1 A2) = I + A1 phi(A2 A1) A2 ------------------------------------------
namespace {

struct LowrankLayout {
    Layout ctl;
    size_t V, Vpart, Phi, U, total;
    int vslices;  // slices of the inner dimension of V = A2 A1
};

LowrankLayout make_lowrank_layout(int n, int t, int batch, int dtype)
{
    LowrankLayout L{};
    const size_t w = dtype == EXPM_DTYPE_F64 ? 8 : 4;
    L.ctl = make_layout(t, batch, dtype);  // control records; for a core beyond the on-chip sizes also the matrix stacks
    size_t off = align_up(L.ctl.total, 256);
    L.V = off;   off = align_up(off + (size_t)batch * t * t * w, 256);
    L.vslices = rect_gemm_slices(t, t, n, batch, dtype == EXPM_DTYPE_F64 ? 1 : 0);
    L.Vpart = off;
    if (L.vslices > 1) off = align_up(off + (size_t)batch * L.vslices * t * t * w, 256);
    L.Phi = off; off = align_up(off + (size_t)batch * t * t * w, 256);
    L.U = off;   off = align_up(off + (size_t)batch * n * t * w, 256);
    L.total = off;
    return L;
}

int check_lowrank_args(const void *A1, const void *A2, int n, int t, int batch, int dtype, double &tol)
{
    if (n < 0 || t < 0 || batch < 0) return EXPM_ERR_INVALID_ARG;
    if (dtype != EXPM_DTYPE_F32 && dtype != EXPM_DTYPE_F64) return EXPM_ERR_INVALID_ARG;
    if (n > 0 && t > 0 && batch > 0 && (A1 == nullptr || A2 == nullptr)) return EXPM_ERR_INVALID_ARG;
    if (n > 46340 || batch > 65535) return EXPM_ERR_INVALID_ARG;  // int index arithmetic; the batch is a grid dimension
    if ((double)batch * (double)n * (double)n > 9.0e15) return EXPM_ERR_INVALID_ARG;
    const double u = dtype == EXPM_DTYPE_F64 ? ldexp(1.0, -53) : ldexp(1.0, -24);
    if (!(tol == tol) || tol < 0.0) return EXPM_ERR_TOLERANCE;
    if (tol == 0.0) tol = u;
    if (tol < u) return EXPM_ERR_TOLERANCE;
    if (t > 0 && !small_path_supported(t, dtype)) {
        // the core series runs on the round-based path: the limits of that path, for t x t matrices
        const double tiles = (double)((t + 31) / 32);
        if ((double)batch * tiles * tiles > 2.0e9) return EXPM_ERR_INVALID_ARG;
    }
    return EXPM_OK;
}

// V = A2 A1 and, unless select_only, Phi = series of V; leaves the per-matrix records (m, flags) in the workspace.
// A core that fits a compute unit's LDS is evaluated on chip by the fused kernel; a larger one goes through the
// round-based path (powers V^2..V^4 for the whole batch, top Horner block, one product round per Horner step).
int run_lowrank_core(DeviceState *ds, unsigned char *base, const void *A1, const void *A2, int n, int t, int batch, int dtype,
                     double tol, int select_only, bool plan_on_device, const LowrankLayout &L, hipStream_t stream)
{
    const double w = dtype == EXPM_DTYPE_F64 ? 8.0 : 4.0;
    {
        Bracket br(stream, EXPM_KCLASS_GEMM, 2.0 * t * (double)t * n * batch, ((2.0 * n * t) + (double)t * t) * batch * w);
        EXPM_TRY(launch_rect_gemm(A2, A1, base + L.V, t, t, n, n, t, t, (size_t)t * n, (size_t)n * t, (size_t)t * t, batch,
                                  dtype, 0, L.vslices, L.vslices > 1 ? base + L.Vpart : nullptr, stream));
    }
    if (small_path_supported(t, dtype)) {
        Bracket br(stream, EXPM_KCLASS_FUSED, 0.0, 2.0 * batch * (double)t * t * w);
        EXPM_TRY(launch_small(base + L.V, base + L.Phi, t, batch, dtype, tol, select_only, kSchemePhi, 0,
                              reinterpret_cast<MatInfo *>(base + L.ctl.info), stream));
        return EXPM_OK;
    }
    const Bound B = bind(base, base + L.V, base + L.Phi, t, batch, dtype, EXPM_NORM_ONE);
    if (select_only) return run_selection_general(ds, B, t, batch, dtype, tol, kSchemePhi, stream, false);
    int rounds = 0, warning = EXPM_OK;
    return run_rounds(ds, B, t, batch, dtype, tol, kSchemePhi, stream, plan_on_device, &rounds, &warning);
}

void remember_lowrank(unsigned char *base, int t, int batch, int dtype, int dev, hipStream_t stream, bool usable,
                      const LowrankLayout &L)
{
    const int fused = small_path_supported(t, dtype) ? 1 : 0;
    remember(t, batch, dtype, fused ? 0 : -1, fused, kSchemePhi, dev, stream, usable,
             reinterpret_cast<MatInfo *>(base + L.ctl.info), reinterpret_cast<int *>(base + L.ctl.summary));
}

}  // namespace

int expm_lowrank_select(const void *A1, const void *A2, int n, int t, int batch, int dtype, double tol, int32_t *m_out)
{
    int rc = check_lowrank_args(A1, A2, n, t, batch, dtype, tol);
    if (rc != EXPM_OK) return rc;
    if (batch > 0 && m_out == nullptr) return EXPM_ERR_INVALID_ARG;
    if (batch == 0) return EXPM_OK;
    if (n == 0 || t == 0) {
        for (int b = 0; b < batch; ++b) m_out[b] = 0;
        return EXPM_OK;
    }
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState *ds = nullptr;
    int dev = 0;
    rc = current_device(&ds, &dev);
    if (rc != EXPM_OK) return rc;
    const LowrankLayout L = make_lowrank_layout(n, t, batch, dtype);
    rc = ensure_workspace(ds, L.total);
    if (rc != EXPM_OK) return rc;
    hipStream_t stream = nullptr;
    rc = order_behind_last_call(ds, dev, stream);
    if (rc != EXPM_OK) return rc;
    g_brackets = false;
    unsigned char *base = static_cast<unsigned char *>(ds->dev);
    rc = run_lowrank_core(ds, base, A1, A2, n, t, batch, dtype, tol, 1, false, L, stream);
    if (rc != EXPM_OK) return rc;
    remember_lowrank(base, t, batch, dtype, dev, stream, true, L);
    g_host_info.resize((size_t)batch);
    EXPM_TRY(hipMemcpyAsync(g_host_info.data(), g_last.info_dev, (size_t)batch * sizeof(MatInfo), hipMemcpyDeviceToHost, stream));
    EXPM_TRY(hipStreamSynchronize(stream));
    int flags = 0;
    for (int b = 0; b < batch; ++b) {
        m_out[b] = g_host_info[b].m;
        flags |= g_host_info[b].flags;
    }
    return warning_from_flags(flags);
}

int expm_lowrank(const void *A1, const void *A2, int n, int t, int batch, int dtype, double tol, void *out, void *stream_v)
{
    int rc = check_lowrank_args(A1, A2, n, t, batch, dtype, tol);
    if (rc != EXPM_OK) return rc;
    if (n == 0 || batch == 0) return EXPM_OK;
    if (out == nullptr) return EXPM_ERR_INVALID_ARG;
    const size_t w = dtype == EXPM_DTYPE_F64 ? 8 : 4;
    {
        const uintptr_t o0 = (uintptr_t)out, ob = (size_t)batch * n * n * w, ib = (size_t)batch * n * t * w;
        const uintptr_t a1 = (uintptr_t)A1, a2 = (uintptr_t)A2;
        if (t > 0 && ((a1 < o0 + ob && o0 < a1 + ib) || (a2 < o0 + ob && o0 < a2 + ib))) return EXPM_ERR_INVALID_ARG;
        if ((o0 | (t > 0 ? (a1 | a2) : 0)) % w) return EXPM_ERR_INVALID_ARG;
    }
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState *ds = nullptr;
    int dev = 0;
    rc = current_device(&ds, &dev);
    if (rc != EXPM_OK) return rc;
    const LowrankLayout L = make_lowrank_layout(n, t, batch, dtype);
    const bool capturing = stream_is_capturing(stream);
    if (capturing && L.total > ds->bytes) return EXPM_ERR_WORKSPACE;
    rc = ensure_workspace(ds, L.total);
    if (rc != EXPM_OK) return rc;
    if (!capturing) {
        rc = order_behind_last_call(ds, dev, stream);
        if (rc != EXPM_OK) return rc;
    }
    g_brackets = g_profile && !capturing;
    unsigned char *base = static_cast<unsigned char *>(ds->dev);
    if (t > 0) {
        const bool on_device = capturing || env_plan() == 1;
        rc = run_lowrank_core(ds, base, A1, A2, n, t, batch, dtype, tol, 0, on_device, L, stream);
        if (rc != EXPM_OK) return rc;
        // U = A1 Phi
        Bracket br(stream, EXPM_KCLASS_GEMM, 2.0 * n * (double)t * t * batch, (2.0 * n * t + (double)t * t) * batch * (double)w);
        EXPM_TRY(launch_rect_gemm(A1, base + L.Phi, base + L.U, n, t, t, t, t, t, (size_t)n * t, (size_t)t * t, (size_t)n * t,
                                  batch, dtype, 0, 1, nullptr, stream));
    }
    {
        // out = U A2 + I  (t = 0: the empty product, out = I)
        Bracket br(stream, EXPM_KCLASS_GEMM, 2.0 * n * (double)n * t * batch, ((double)n * n + 2.0 * n * t) * batch * (double)w);
        EXPM_TRY(launch_rect_gemm(base + L.U, A2, out, n, n, t, t, n, n, (size_t)n * t, (size_t)t * n, (size_t)n * n, batch,
                                  dtype, 1, 1, nullptr, stream));
    }
    if (t > 0) remember_lowrank(base, t, batch, dtype, dev, stream, !capturing, L);
    else g_last.valid = false;
    return EXPM_OK;
}

int expm_get_stats(struct expm_stats *st)
{
    if (!st) return EXPM_ERR_INVALID_ARG;
    std::memset(st, 0, sizeof(*st));
    std::lock_guard<std::mutex> lock(g_mutex);
    if (!g_last.valid) return EXPM_OK;
    // the records are read on the stream of the call (after a call recorded into a graph: on the null stream, which
    // waits for whatever replays of that graph have been launched so far on blocking streams)
    hipStream_t rs = g_last.stream_usable ? g_last.stream : nullptr;
    g_host_info.resize((size_t)g_last.batch);
    int prev = 0;
    EXPM_TRY(hipGetDevice(&prev));
    if (prev != g_last.device) EXPM_TRY(hipSetDevice(g_last.device));
    hipError_t e = hipMemcpyAsync(g_host_info.data(), g_last.info_dev, (size_t)g_last.batch * sizeof(MatInfo),
                                  hipMemcpyDeviceToHost, rs);
    if (e == hipSuccess) e = hipStreamSynchronize(rs);
    if (prev != g_last.device) (void)hipSetDevice(prev);
    if (e != hipSuccess) return hip_fail(e);
    st->matrices = g_last.batch;
    st->n = g_last.n;
    st->dtype = g_last.dtype;
    st->fused_path = g_last.fused;
    st->scheme = g_last.scheme;
    int flags = 0, longest = 0;
    for (int b = 0; b < g_last.batch; ++b) {
        const MatInfo &mi = g_host_info[b];
        flags |= mi.flags;
        if (mi.m < 0) { st->nonfinite++; continue; }
        // products the method spends: Sec. 3.1 formulas 0,0,1,2,3,4 for m = 0,1,2,4,8,15; Paterson-Stockmeyer
        // (powers up to W^j plus k-1 Horner steps) 0,0,1,2,3,4,5,6 for m = 0,1,2,4,6,9,12,16
        int pi = 0;
        if (g_last.scheme == kSchemePS) {
            pi = mi.m < 2 ? 0 : ps_j(mi.m) - 1 + ps_k(mi.m) - 1;
        } else if (g_last.scheme == kSchemePhi) {
            pi = mi.m < 2 ? 0 : ps_j(mi.m) - 1 + ps_k(mi.m) - 1;   // products of the t x t core series only
        } else if (g_last.scheme == kSchemeBaseline) {
            pi = mi.m < 1 ? 0 : mi.m - 1;   // the paper prices degree m at (m-1) products (its eq. for C_orig)
        } else {
            pi = mi.m < 2 ? 0 : (mi.m == 2 ? 1 : (mi.m == 4 ? 2 : (mi.m == 8 ? 3 : 4)));
        }
        st->hist_m[mi.m > 16 ? 16 : mi.m]++;   // the baseline may exceed degree 16: counted in the last bin
        if (mi.s >= 0 && mi.s <= EXPM_S_CAP) st->hist_s[mi.s]++;
        st->products += pi + mi.s;
        if (mi.len > longest) longest = mi.len;
    }
    // rounds planned on the device: the longest chain among the records is what the host would have launched
    st->rounds = g_last.rounds >= 0 ? g_last.rounds : longest;
    st->warning = warning_from_flags(flags);
    st->warning_bits = flags & 3;
    return EXPM_OK;
}

int expm_profile_enable(int on)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    g_profile = on != 0;
    return EXPM_OK;
}

int expm_profile_reset(void)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    for (auto &e : g_events) {
        g_event_pool.push_back(e.start);
        g_event_pool.push_back(e.stop);
    }
    g_events.clear();
    return EXPM_OK;
}

int expm_profile_read(struct expm_profile *p)
{
    if (!p) return EXPM_ERR_INVALID_ARG;
    std::memset(p, 0, sizeof(*p));
    std::lock_guard<std::mutex> lock(g_mutex);
    for (auto &e : g_events) {
        EXPM_TRY(hipEventSynchronize(e.stop));
        float ms = 0.f;
        EXPM_TRY(hipEventElapsedTime(&ms, e.start, e.stop));
        p->launches[e.kclass]++;
        p->ms[e.kclass] += ms;
        p->flops[e.kclass] += e.flops;
        p->bytes[e.kclass] += e.bytes;
    }
    return EXPM_OK;
}

int expm_shutdown(void)
{
    expm_profile_reset();
    std::lock_guard<std::mutex> lock(g_mutex);
    for (auto e : g_event_pool) (void)hipEventDestroy(e);
    g_event_pool.clear();
    int prev = 0;
    const bool have_prev = hipGetDevice(&prev) == hipSuccess;
    for (int d = 0; d < kMaxDevices; ++d) {
        DeviceState &ds = g_dev[d];
        const bool used = ds.dev || ds.host_summary || ds.summary_ready || ds.fork || ds.side_stream || ds.order_event;
        if (!used) { ds = DeviceState{}; continue; }
        (void)hipSetDevice(d);
        if (ds.dev) {
            (void)hipDeviceSynchronize();
            (void)hipFree(ds.dev);
        }
        if (ds.host_summary) (void)hipHostFree(ds.host_summary);
        if (ds.summary_ready) (void)hipEventDestroy(ds.summary_ready);
        if (ds.fork) (void)hipEventDestroy(ds.fork);
        if (ds.join) (void)hipEventDestroy(ds.join);
        if (ds.order_event) (void)hipEventDestroy(ds.order_event);
        for (int c = 1; c < kChains; ++c) {
            if (ds.chain_join[c]) (void)hipEventDestroy(ds.chain_join[c]);
            if (c > 1 && ds.chain_stream[c]) (void)hipStreamDestroy(ds.chain_stream[c]);
        }
        if (ds.side_stream) (void)hipStreamDestroy(ds.side_stream);
        ds = DeviceState{};   // the static scratch array stays with the device; its address is looked up again on demand
    }
    if (have_prev) (void)hipSetDevice(prev);
    (void)hipGetLastError();
    g_host_info.clear();
    g_host_info.shrink_to_fit();
    g_last = LastCall{};
    return EXPM_OK;
}

int expm_last_hip_error(void) { return g_last_hip_error; }

const char *expm_status_string(int status)
{
    switch (status) {
    case EXPM_OK: return "success";
    case EXPM_WARN_NONFINITE: return "warning: non-finite matrix in the batch (its result is NaN)";
    case EXPM_WARN_SCALING_CAP: return "warning: scaling parameter reached its cap of 20";
    case EXPM_ERR_INVALID_ARG: return "error: invalid argument";
    case EXPM_ERR_TOLERANCE: return "error: tolerance is negative, NaN or below the unit roundoff of dtype";
    case EXPM_ERR_ALLOC: return "error: allocation failed";
    case EXPM_ERR_HIP: return "error: a HIP call failed (see expm_last_hip_error)";
    case EXPM_ERR_UNSUPPORTED: return "error: this scheme is not available for this matrix size";
    case EXPM_ERR_WORKSPACE: return "error: the workspace this shape needs exceeds what the call may use (static scratch "
                                    "of expm_noalloc, or a workspace that would have to grow inside a stream capture)";
    default: return "unknown status";
    }
}

}  // extern "C"
