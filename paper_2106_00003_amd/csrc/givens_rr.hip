// C ABI of the round-robin Givens library (see include/givens_rr.h for the contract).
// Host side: argument checks, workspaces, kernel selection, launches, optional event timing.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <memory>
#include <mutex>
#include <new>
#include <type_traits>
#include <vector>

#include "../../include/givens_rr.h"
#include "carousel_host.hpp"
#include "coef_kernels.hpp"
#include "gram_kernels.hpp"
#include "lds_kernels.hpp"
#include "rr_index.h"
#include "unitary_kernels.hpp"

namespace givens {
namespace {

constexpr int kMaxDevices = 64;
constexpr int kMaxWorkspacesPerDevice = 8;                     // streams with a workspace of their own, per device
constexpr size_t kLdsBudgetBytes = 144 * 1024;                 // of the 160 KB per CU on gfx950
constexpr long long kReduceSplitMaxAngles = 1 << 18;           // below this the second stage splits the rows too
constexpr size_t kPartialCapBytes = size_t(24) << 30;          // cap on one chunk of strip partials
constexpr int kMaxRows = 36864;                                // largest n any kernel family takes (one float column in LDS)
constexpr size_t kFlagBytes = 256;                             // the flag words of a workspace

struct Buffer {
    void *ptr = nullptr;
    size_t bytes = 0;
};

// One sweep direction's coefficients.
struct CoefSet {
    Buffer table;   // N pairs in the rotation form the flag selects (standard: cos, sin)
    Buffer renorm;  // scaled / lifted forms: periods * n/2 pairs
    Buffer factor;  // reverse sweep: per-angle factor of the dtheta reduction
};

// What a prepared call needs to know about the tables givens_prepare left in a workspace.
struct Prepared {
    int64_t token = 0;       // 0: nothing prepared
    int rows = 0, m = 0;
    bool fwd = false, rev = false, mirrored = false;
    // whether each set was built with the device-side choice of the rotation form (float carousel kernels
    // only can read such a set; a set built without it holds the standard form, which every family reads)
    bool fwd_forms = false, rev_forms = false, mirrored_forms = false;
    float scaled_max = 0.f;
};

// Everything the library allocates for the calls made on one stream of one device.  Calls on different
// streams use different workspaces and may overlap; calls on one stream are ordered by the stream.
struct Workspace {
    hipStream_t stream = nullptr;
    uint64_t last_use = 0;
    Buffer flag;        // three words holding the bit pattern of max |theta|: [0], [1] take turns from call to
                        // call (each range check zeroes the other for the next call), [2] is givens_prepare's
    int flag_turn = 0;  // which of [0], [1] the next range check uses
    Buffer scale;       // scaled / lifted forms: row factors d, float [n-1][n] (scratch of the coefficient kernels)
    CoefSet fwd, rev;   // forward sweep, reverse sweep
    CoefSet mirrored;   // forward-type sweep that computes dX = U^T G in the Gram form
    Buffer partial;     // per-workgroup (carousel) or per-strip (LDS family) dtheta partial sums
    Buffer zeros;       // N floats that are zeroed when allocated and never written again
    Buffer sink;        // N + 8192 floats: where idle lanes of the carousel reverse sweep put their sums
    Buffer chain;       // reverse sweep's chained rows: XCD numbers and the error word (reset by every launch)
    Buffer chain_flags; // one cache line per workgroup and block: tag of the launch and pass that finished it;
                        // last word: the launch counter
    Buffer gram;        // Gram form: slices of C = Y G^T, rows x rows floats each
    Buffer map;         // restricted parametrisation / odd n: index in theta of every entry of E, or -1
    Buffer map_counts;  // free pairs per block (scratch of the map kernels)
    // unitary extension, carousel family: phase inputs and reduced phase angles (fixed point), rotation signs, the two
    // coefficient tables, the 0/1 table of the reverse sweep, final phase per row
    Buffer u_q, u_psi, u_sgn, u_rot, u_phs, u_orient, u_fin;
    int map_rows = 0, map_m = 0; // the (row count, m) the map was built for
    Prepared prepared;
    Buffer *all[25] = {&flag, &scale, &fwd.table, &fwd.renorm, &fwd.factor, &rev.table, &rev.renorm, &rev.factor,
                       &mirrored.table, &mirrored.renorm, &mirrored.factor, &partial, &zeros, &sink, &gram, &map,
                       &u_q, &u_psi, &u_sgn, &u_rot, &u_phs, &u_orient, &u_fin, &chain, &chain_flags};
};

// One call's problem: `rows` coordinates of which the first m may rotate with every other one
// (Section 5 of the paper; m = rows - 1 is the unrestricted case), run by the kernels on n = rows
// rounded up to even (end of Section 3: an added, inactive dimension).  map == nullptr when every
// pair of E is free, and then theta is indexed by E directly.
struct Problem {
    int n = 0, rows = 0, m = 0;
    const int *map = nullptr;
    long long free_angles = 0;
};

// Per-call choices.  The plain entry points take the process-wide defaults (givens_set_*); the _ex entry points
// take them from the caller.
struct CallOptions {
    int kernel = GIVENS_KERNEL_AUTO, form = GIVENS_FORM_AUTO, reduction = GIVENS_REDUCTION_AUTO;
};

std::mutex g_mutex;
std::vector<std::unique_ptr<Workspace>> g_ws[kMaxDevices];
uint64_t g_use_clock = 0;
int64_t g_next_token = 0;
int g_kernel_choice = GIVENS_KERNEL_AUTO;
int g_form_choice = GIVENS_FORM_AUTO;
int g_reduction_choice = GIVENS_REDUCTION_AUTO;
int g_timing_on = 0;

struct TimedSpan {
    int category;
    hipEvent_t start, stop;
};
struct ThreadState {
    int last_hip_error = 0;
    int last_kernel = 0;
    int last_reduction = 0;
    int last_chains = 0;                 // chains of workgroups in the last two-stage carousel reverse sweep (0: none)
    const unsigned *last_flag = nullptr; // device flag of the last call when the form was chosen on the device
    float last_scaled_max = 0.f;         // that call's threshold for the scaled form
    hipStream_t last_stream = nullptr;
    bool timing_valid = false;
    std::vector<TimedSpan> spans;
    std::vector<hipEvent_t> pool;
};
thread_local ThreadState t_state;

bool hip_ok(hipError_t e)
{
    if (e == hipSuccess) return true;
    t_state.last_hip_error = (int)e;
    return false;
}

#define GIVENS_HIP(call)                         \
    do {                                         \
        if (!hip_ok(call)) return GIVENS_ERR_HIP; \
    } while (0)

int grow(Buffer &b, size_t want)
{
    if (b.bytes >= want) return GIVENS_OK;
    if (b.ptr) {
        GIVENS_HIP(hipFree(b.ptr));                            // synchronises the device
        b.ptr = nullptr;
        b.bytes = 0;
    }
    GIVENS_HIP(hipMalloc(&b.ptr, want));
    b.bytes = want;
    return GIVENS_OK;
}

int free_workspace(Workspace &ws)
{
    int rc = GIVENS_OK;
    for (Buffer *b : ws.all) {
        if (b->ptr && !hip_ok(hipFree(b->ptr))) rc = GIVENS_ERR_HIP;
        *b = Buffer{};
    }
    if (ws.map_counts.ptr && !hip_ok(hipFree(ws.map_counts.ptr))) rc = GIVENS_ERR_HIP;
    ws.map_counts = Buffer{};
    ws.map_rows = ws.map_m = 0;
    ws.prepared = Prepared{};
    return rc;
}

// The workspace of (device, stream), created on first use.  When a device already has
// kMaxWorkspacesPerDevice of them, the one used longest ago is given up first (after a device-wide
// synchronisation: its stream may have work in flight that still reads it).
int workspace_for(int dev, hipStream_t stream, Workspace **out)
{
    auto &list = g_ws[dev];
    for (auto &w : list)
        if (w->stream == stream) {
            w->last_use = ++g_use_clock;
            *out = w.get();
            return GIVENS_OK;
        }
    if ((int)list.size() >= kMaxWorkspacesPerDevice) {
        size_t victim = 0;
        for (size_t i = 1; i < list.size(); ++i)
            if (list[i]->last_use < list[victim]->last_use) victim = i;
        GIVENS_HIP(hipDeviceSynchronize());
        if (int rc = free_workspace(*list[victim])) return rc;
        list.erase(list.begin() + (long)victim);
    }
    std::unique_ptr<Workspace> w(new (std::nothrow) Workspace);
    if (!w) return GIVENS_ERR_UNSUPPORTED;
    w->stream = stream;
    w->last_use = ++g_use_clock;
    try {
        list.push_back(std::move(w));   // no exception may cross the C boundary
    } catch (...) {
        return GIVENS_ERR_UNSUPPORTED;
    }
    *out = list.back().get();
    return GIVENS_OK;
}

hipEvent_t take_event()
{
    ThreadState &ts = t_state;
    if (!ts.pool.empty()) {
        hipEvent_t e = ts.pool.back();
        ts.pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (!hip_ok(hipEventCreate(&e))) return nullptr;
    return e;
}

void timing_begin_call()
{
    ThreadState &ts = t_state;
    try {
        for (auto &s : ts.spans) {
            ts.pool.push_back(s.start);
            ts.pool.push_back(s.stop);
        }
    } catch (...) {   // out of host memory: the events stay with their spans' records and are not reused
    }
    ts.spans.clear();
    ts.timing_valid = g_timing_on != 0;
}

// RAII: records an event pair around the launches made while it is alive.
struct Span {
    hipStream_t stream;
    bool on;
    TimedSpan rec{};
    Span(int category, hipStream_t s) : stream(s), on(t_state.timing_valid)
    {
        if (!on) return;
        rec.category = category;
        rec.start = take_event();
        rec.stop = take_event();
        if (!rec.start || !rec.stop) { on = false; return; }
        (void)hipEventRecord(rec.start, stream);
    }
    ~Span()
    {
        if (!on) return;
        (void)hipEventRecord(rec.stop, stream);
        try {
            t_state.spans.push_back(rec);
        } catch (...) {   // out of host memory: this span is not reported
        }
    }
};

int check_n(int n) { return (n < 2 || (n & 1)) ? GIVENS_ERR_BAD_N : GIVENS_OK; }

long long count_free_angles(int rows, int m) { return (long long)m * rows - (long long)m * (m + 1) / 2; }

int check_restricted(int rows, int m)
{
    if (rows < 2) return GIVENS_ERR_BAD_N;
    if (m < 1 || m > rows - 1) return GIVENS_ERR_BAD_M;
    return GIVENS_OK;
}

// Free pairs in E order: circle-method blocks on n = rows rounded up to even, leaving out the pairs
// with the added dimension (j >= rows) and the pairs inside m..rows-1 (i >= m).  `visit(e, i, j, free)`
// is called for every entry e of the full sequence.
template <typename F>
void walk_pairs(int rows, int m, F &&visit)
{
    const int n = rows + (rows & 1), H = n / 2;
    long long e = 0;
    for (int k = 0; k < n - 1; ++k)
        for (int p = 0; p < H; ++p, ++e) {
            const int a = rr_label(n, k, p), b = rr_label(n, k, n - 1 - p);
            const int i = a < b ? a : b, j = a < b ? b : a;
            visit(e, i, j, j < rows && i < m);
        }
}

// Fills in the padded size and, when some pair of E is bypassed, the device map: built by three small
// kernels on the caller's stream the first time this workspace sees (rows, m), and again when another
// (rows, m) has used the buffer in between (the stream orders the rebuild after the previous reader).
int resolve_problem(Workspace *ws, int rows, int m, hipStream_t stream, Problem *out)
{
    if (int rc = check_restricted(rows, m)) return rc;
    if (rows > kMaxRows) return GIVENS_ERR_UNSUPPORTED;      // before anything is allocated
    out->rows = rows;
    out->m = m;
    out->n = rows + (rows & 1);
    out->free_angles = count_free_angles(rows, m);
    out->map = nullptr;
    if (!(rows & 1) && m == rows - 1) return GIVENS_OK;
    if (!ws) return GIVENS_ERR_UNSUPPORTED;
    if (!(ws->map.ptr && ws->map_rows == rows && ws->map_m == m)) {
        const int n = out->n;
        const long long N = (long long)(n - 1) * (n / 2);
        ws->map_rows = 0;
        if (int rc = grow(ws->map, (size_t)N * sizeof(int))) return rc;
        if (int rc = grow(ws->map_counts, (size_t)n * sizeof(int))) return rc;
        int *map = reinterpret_cast<int *>(ws->map.ptr);
        int *counts = reinterpret_cast<int *>(ws->map_counts.ptr);
        hipLaunchKernelGGL(map_count_kernel, dim3(n - 1), dim3(kMapThreads), 0, stream, n, rows, m, counts);
        hipLaunchKernelGGL(map_scan_kernel, dim3(1), dim3(kMapThreads), 0, stream, n - 1, counts);
        hipLaunchKernelGGL(map_fill_kernel, dim3(n - 1), dim3(kMapThreads), 0, stream, n, rows, m, counts, map);
        GIVENS_HIP(hipGetLastError());
        ws->map_rows = rows;
        ws->map_m = m;
    }
    out->map = reinterpret_cast<const int *>(ws->map.ptr);
    return GIVENS_OK;
}

// Widest odd strip (<= 15 columns) whose `strips_in_lds` copies fit the LDS budget; narrower
// when that is needed to give every CU a few workgroups.
template <typename T>
int lds_strip_width(int n, long long B, int strips_in_lds)
{
    int w = 15;
    while (w > 1 && (size_t)n * lds_row_stride(w) * sizeof(T) * strips_in_lds > kLdsBudgetBytes) w -= 2;
    if ((size_t)n * lds_row_stride(w) * sizeof(T) * strips_in_lds > kLdsBudgetBytes) return 0;
    while (w > 1 && (B + w - 1) / w < 1024) w -= 2;
    return w;
}

// Everything the sweeps of one call read that depends on theta only.
template <typename T>
struct Coefs {
    const typename Pair2<T>::type *table = nullptr; // in the form the flag selects
    const T *factor = nullptr;                      // reverse sweep only
    const float2 *renorm = nullptr;                 // scaled / lifted forms
    const unsigned *flag = nullptr;                 // nullptr: standard form, no range check was made
    float scaled_max = 0.f;
    CarouselCoefs carousel() const
    {
        return CarouselCoefs{reinterpret_cast<const float2 *>(table), renorm, flag, scaled_max};
    }
};

// What the rotation-form choice means for a call on the float carousel path: whether the range check and
// the scaled / lifted tables are wanted, and the threshold of the scaled form.
struct FormPolicy {
    bool try_forms;
    float scaled_max;
};
// `updates`: pair-column updates of the sweep the coefficients are for.  The scaled and lifted forms cost a range
// check and a row-factor scan per direction (0.07 - 0.1 ms) and save arithmetic only where the sweep is bound by
// it: measured, they pay from about n = B = 2048 (4.3e9 updates; 2.97 against 3.08 ms per step) and lose below
// (n = B = 1024, 5.4e8: 0.98 against 0.92 ms; n = B = 256: 0.20 against 0.14 ms).
constexpr double kFormsMinUpdates = 1.0e9;
FormPolicy form_policy(bool float_carousel, int n, int form_choice, double updates)
{
    // a carousel shape with an odd number of slots per lane has the standard form only
    if (!float_carousel || !carousel_has_forms(n) || form_choice == GIVENS_FORM_STANDARD) return {false, 0.f};
    if (form_choice == GIVENS_FORM_LIFTED) return {true, -1.f};
    if (form_choice == GIVENS_FORM_AUTO && updates < kFormsMinUpdates) return {false, 0.f};
    return {true, kScaledMaxAbsTheta};
}
inline double sweep_updates(int n, long long B) { return 0.5 * (double)n * (double)(n - 1) * (double)B; }

// Where the coefficient kernels of one sweep direction write: buffers of the workspace (grown on demand) or
// pieces of the static scratch array of the entry point that may not allocate.
template <typename T>
struct CoefStorage {
    typename Pair2<T>::type *table = nullptr; // N pairs
    T *factor = nullptr;                      // reverse sweep only, N values
    unsigned *flag = nullptr;                 // this call's flag word (float carousel path), zero before the call
    unsigned *next_flag = nullptr;            // the word the next call will use (zeroed by this call), or nullptr
    float *scale = nullptr;                   // (n-1) * n row factors
    float *renorm = nullptr;                  // periods * n/2 pairs
};

inline int renorm_periods(int n) { return (n - 1 + kRenormPeriod - 1) / kRenormPeriod; }

template <typename T>
int workspace_coef_storage(Workspace &ws, CoefSet &set, int n, bool want_factor, bool try_forms, hipStream_t stream,
                           CoefStorage<T> *out, bool for_prepare)
{
    using P2 = typename Pair2<T>::type;
    const long long N = (long long)n * (n - 1) / 2;
    if (int rc = grow(set.table, (size_t)N * sizeof(P2))) return rc;
    out->table = reinterpret_cast<P2 *>(set.table.ptr);
    if (want_factor) {
        if (int rc = grow(set.factor, (size_t)N * sizeof(T))) return rc;
        out->factor = reinterpret_cast<T *>(set.factor.ptr);
    }
    if (try_forms) {
        if (!ws.flag.ptr) {
            if (int rc = grow(ws.flag, kFlagBytes)) return rc;
            GIVENS_HIP(hipMemsetAsync(ws.flag.ptr, 0, kFlagBytes, stream));   // every flag word starts at zero
        }
        if (int rc = grow(ws.scale, (size_t)(n - 1) * n * sizeof(float))) return rc;
        if (int rc = grow(set.renorm, (size_t)renorm_periods(n) * (n / 2) * sizeof(float2))) return rc;
        unsigned *words = reinterpret_cast<unsigned *>(ws.flag.ptr);
        if (for_prepare) {
            out->flag = words + 2;                              // reset by prepare_impl before the range check
            out->next_flag = nullptr;
        } else {
            out->flag = words + ws.flag_turn;
            out->next_flag = words + (ws.flag_turn ^ 1);
            ws.flag_turn ^= 1;
        }
        out->scale = reinterpret_cast<float *>(ws.scale.ptr);
        out->renorm = reinterpret_cast<float *>(set.renorm.ptr);
    }
    return GIVENS_OK;
}

// ---- the entry point that allocates nothing: its coefficient tables live in a static device array.
constexpr int kNoAllocMaxN = GIVENS_NOALLOC_MAX_N;
constexpr size_t round_up_256(size_t v) { return (v + 255) / 256 * 256; }
constexpr size_t noalloc_bytes(int n)
{
    const size_t N = (size_t)n * (n - 1) / 2;
    return round_up_256(N * sizeof(float2))                                                // the table
           + round_up_256((size_t)(n - 1) * n * sizeof(float))                             // row factors
           + round_up_256((size_t)((n - 1 + kRenormPeriod - 1) / kRenormPeriod) * (n / 2) * sizeof(float2))
           + kFlagBytes;                                                                   // flag words
}
constexpr size_t kNoAllocBytes = noalloc_bytes(kNoAllocMaxN);
static_assert(kNoAllocBytes == GIVENS_NOALLOC_BYTES, "the header states the size of the static array");
static __device__ __align__(256) unsigned char scratch[kNoAllocBytes];
// Address of `scratch` on each device (every GPU holds its own copy of the array): looked up once per
// device with that device current.  Host code uses these pointers, never the array's name.
unsigned char *g_scratch_ptr[kMaxDevices] = {};
int g_scratch_turn[kMaxDevices] = {};   // which of the array's two flag words the next call uses

int static_coef_storage(int dev, int n, CoefStorage<float> *out)
{
    if (n > kNoAllocMaxN) return GIVENS_ERR_UNSUPPORTED;
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        GIVENS_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        g_scratch_ptr[dev] = static_cast<unsigned char *>(p);
    }
    const size_t N = (size_t)n * (n - 1) / 2;
    unsigned char *at = g_scratch_ptr[dev];
    auto take = [&](size_t bytes) {
        unsigned char *here = at;
        at += round_up_256(bytes);
        return here;
    };
    // the flag words come first: their place must not depend on n, because the word a call uses has to be zero
    // when the call starts and it is the call before that puts it to zero (a fresh array is all zero)
    unsigned *words = reinterpret_cast<unsigned *>(take(kFlagBytes));
    out->flag = words + g_scratch_turn[dev];
    out->next_flag = words + (g_scratch_turn[dev] ^ 1);
    g_scratch_turn[dev] ^= 1;
    out->table = reinterpret_cast<float2 *>(take(N * sizeof(float2)));
    out->scale = reinterpret_cast<float *>(take((size_t)(n - 1) * n * sizeof(float)));
    out->renorm = reinterpret_cast<float *>(take((size_t)renorm_periods(n) * (n / 2) * sizeof(float2)));
    out->factor = nullptr;
    return (size_t)(at - g_scratch_ptr[dev]) <= kNoAllocBytes ? GIVENS_OK : GIVENS_ERR_UNSUPPORTED;
}

// Launches the coefficient kernels of one sweep direction.  `forward` picks the direction of the scaled /
// lifted forms' row factors; `policy.try_forms` adds those forms (range check unless `range_known`: the
// flag already holds max |theta| of this theta).
template <typename T>
int build_coefs(const CoefStorage<T> &st, const Problem &pb, const T *theta, bool forward, FormPolicy policy,
                hipStream_t stream, Coefs<T> *out, int mirror = 0, bool range_known = false)
{
    const int n = pb.n;
    const int *map = pb.map;
    const long long N = (long long)n * (n - 1) / 2;
    unsigned *flag = nullptr;
    const int threads = 256;
    const unsigned blocks = (unsigned)std::min<long long>((N + threads - 1) / threads, 8192);
    Span span(0, stream);
    if constexpr (std::is_same<T, float>::value) {
        if (policy.try_forms) {
            flag = st.flag;
            if (!range_known) {
                const unsigned range_blocks =
                    (unsigned)std::min<long long>(kRangeBlocks, (pb.free_angles + 4095) / 4096);
                hipLaunchKernelGGL(theta_range_kernel, dim3(range_blocks), dim3(512), 0, stream, pb.free_angles, theta,
                                   flag, st.next_flag);
            }
            const long long scan_threads = (long long)renorm_periods(n) * n;
            const unsigned scan_blocks = (unsigned)((scan_threads + threads - 1) / threads);
            if (forward)
                hipLaunchKernelGGL(scaled_scan_kernel<true>, dim3(scan_blocks), dim3(threads), 0, stream, n, theta, map,
                                   mirror, flag, policy.scaled_max, st.scale, st.renorm);
            else
                hipLaunchKernelGGL(scaled_scan_kernel<false>, dim3(scan_blocks), dim3(threads), 0, stream, n, theta, map,
                                   mirror, flag, policy.scaled_max, st.scale, st.renorm);
            out->renorm = reinterpret_cast<const float2 *>(st.renorm);
        }
    }
    hipLaunchKernelGGL(coef_table_kernel<T>, dim3(blocks), dim3(threads), 0, stream, n, theta, map, mirror,
                       static_cast<const unsigned *>(flag), policy.scaled_max, static_cast<const float *>(st.scale),
                       st.table, forward ? nullptr : st.factor);
    GIVENS_HIP(hipGetLastError());
    out->table = st.table;
    out->factor = forward ? nullptr : st.factor;
    out->flag = flag;
    out->scaled_max = policy.scaled_max;
    t_state.last_flag = flag;
    t_state.last_scaled_max = policy.scaled_max;
    t_state.last_stream = stream;
    return GIVENS_OK;
}

// the usual case: storage from a coefficient set of the workspace
// for_prepare: the tables are givens_prepare's: they read its own flag word, which only givens_prepare writes
// (range_known: an earlier build of the same givens_prepare call has made the range check already)
template <typename T>
int build_coefs(Workspace &ws, CoefSet &set, const Problem &pb, const T *theta, bool forward, FormPolicy policy,
                hipStream_t stream, Coefs<T> *out, int mirror = 0, bool range_known = false, bool for_prepare = false)
{
    CoefStorage<T> st;
    const bool forms = policy.try_forms && std::is_same<T, float>::value;
    if (int rc = workspace_coef_storage<T>(ws, set, pb.n, !forward, forms, stream, &st, for_prepare))
        return rc;
    return build_coefs<T>(st, pb, theta, forward, policy, stream, out, mirror, range_known);
}

// From n = 2048 on (four or more arcs per thread and block) the LDS-family kernels run the instance that fetches
// its coefficients a block ahead.  Measured, complex64 B = 2048: n = 2048 reverse sweep 15.5 -> 9.7 ms with it,
// n = 1024 (B = 4096) 5.97 -> 6.33 ms: below that a block is short enough, and the resident workgroups many
// enough, that the loads are hidden anyway and the prefetch only costs registers.
inline bool lds_wants_ahead(int n) { return n >= 2048; }

template <typename T>
int lds_forward(int n, int rows, long long B, const typename Pair2<T>::type *table, const T *X, T *Y,
                int identity, hipStream_t stream, int mirror = 0)
{
    const int w = lds_strip_width<T>(n, B, 1);
    if (w == 0) return GIVENS_ERR_UNSUPPORTED;
    const size_t smem = (size_t)n * lds_row_stride(w) * sizeof(T);
    auto kern = lds_wants_ahead(n) ? lds_forward_kernel<T, kLdsAhead> : lds_forward_kernel<T, 0>;
    GIVENS_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    const long long strips = (B + w - 1) / w;
    Span span(1, stream);
    hipLaunchKernelGGL(kern, dim3((unsigned)strips), dim3(kLdsThreads), smem, stream, n, rows, B, w, table, X,
                       Y, identity, mirror);
    GIVENS_HIP(hipGetLastError());
    return GIVENS_OK;
}

// Which kernel family a call takes.
struct Families {
    bool carousel = false, column = false;  // neither: LDS strip family
};
template <typename T>
int pick_forward_family(int n, long long B, int choice, Families *out)
{
    const bool can_carousel = carousel_supported<T>(n, B);
    const bool can_column = std::is_same<T, float>::value && n <= kColumnFamilyMaxN;
    if (choice == GIVENS_KERNEL_CAROUSEL && !can_carousel) return GIVENS_ERR_UNSUPPORTED;
    if (choice == GIVENS_KERNEL_COLUMN && !can_column) return GIVENS_ERR_UNSUPPORTED;
    out->carousel = can_carousel && (choice == GIVENS_KERNEL_AUTO || choice == GIVENS_KERNEL_CAROUSEL);
    out->column = !out->carousel && can_column && (choice == GIVENS_KERNEL_AUTO || choice == GIVENS_KERNEL_COLUMN);
    return GIVENS_OK;
}
template <typename T>
int pick_backward_family(int n, long long B, int choice, Families *out)
{
    const bool can_carousel = carousel_backward_supported<T>(n, B);
    const bool can_column = std::is_same<T, float>::value && n <= kColumnFamilyMaxN;
    if (choice == GIVENS_KERNEL_CAROUSEL && !can_carousel) return GIVENS_ERR_UNSUPPORTED;
    if (choice == GIVENS_KERNEL_COLUMN && !can_column) return GIVENS_ERR_UNSUPPORTED;
    // the family that sweeps (the n x n operand of the Gram form, or all B columns); the column family has
    // no reverse sweep of its own and borrows the LDS family's
    out->carousel = can_carousel && (choice == GIVENS_KERNEL_AUTO || choice == GIVENS_KERNEL_CAROUSEL);
    out->column = can_column && (choice == GIVENS_KERNEL_AUTO || choice == GIVENS_KERNEL_COLUMN);
    return GIVENS_OK;
}

// The forward-type sweep of one call, coefficients given.
template <typename T>
int run_forward_sweep(const Problem &pb, long long B, const Coefs<T> &coefs, Families fam, const T *X, T *Y,
                      int identity, int transpose, hipStream_t stream)
{
    const int n = pb.n, rows = pb.rows;
    int rc = GIVENS_OK;
    if (fam.carousel) {
        if constexpr (std::is_same<T, float>::value) {
            Span span(1, stream);
            rc = carousel_forward(n, rows, B, coefs.carousel(), X, Y, identity, transpose, stream);
            if (rc == GIVENS_OK && !hip_ok(hipGetLastError())) rc = GIVENS_ERR_HIP;
        } else {
            rc = GIVENS_ERR_UNSUPPORTED;
        }
        t_state.last_kernel = GIVENS_KERNEL_CAROUSEL;
    } else if (fam.column) {
        if constexpr (std::is_same<T, float>::value) {
            Span span(1, stream);
            rc = column_forward(n, rows, B, coefs.table, X, Y, identity, transpose, stream);
            if (rc == GIVENS_OK && !hip_ok(hipGetLastError())) rc = GIVENS_ERR_HIP;
        }
        t_state.last_kernel = GIVENS_KERNEL_COLUMN;
    } else {
        rc = lds_forward<T>(n, rows, B, coefs.table, X, Y, identity, stream, transpose);
        t_state.last_kernel = GIVENS_KERNEL_LDS;
    }
    return rc;
}

// Reverse sweep and the reduction of its partial sums into dtheta.  LDS family: chunks of strips, one
// partial sum per (strip, angle), folded into dtheta chunk by chunk.  Carousel family: persistent
// workgroups with one row of partial sums each.
template <typename T>
int backward_chunks(Workspace &ws, int dev, bool carousel, const Problem &pb, long long B, const Coefs<T> &coefs,
                    const T *Y, const T *G, T *dX, T *dtheta, hipStream_t stream, int g_identity = 0)
{
    const int n = pb.n, rows = pb.rows;
    const int *map = pb.map;
    const long long N = (long long)n * (n - 1) / 2;
    int w = 0;
    size_t smem = 0;
    auto kern = lds_backward_kernel<T, 0>;
    if (!carousel) {
        w = lds_strip_width<T>(n, B, 2);
        if (w == 0) return GIVENS_ERR_UNSUPPORTED;
        smem = (size_t)2 * n * lds_row_stride(w) * sizeof(T);
        if (lds_wants_ahead(n)) kern = lds_backward_kernel<T, kLdsAhead>;
        GIVENS_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    } else {
        w = carousel_bwd_width(n, B);
        if (w == 0) return GIVENS_ERR_UNSUPPORTED;
    }
    const long long strips = (B + w - 1) / w;
    int cus = 0;
    GIVENS_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    const float *zeros = nullptr;
    float *sink = nullptr;
    if constexpr (std::is_same<T, float>::value) {
        if (carousel) {
            const size_t want = (size_t)N * sizeof(float);
            if (ws.zeros.bytes < want) {
                if (int rc = grow(ws.zeros, want)) return rc;
                hipLaunchKernelGGL(fill_zero_kernel, dim3(2048), dim3(256), 0, stream, N,
                                   reinterpret_cast<float *>(ws.zeros.ptr));
                GIVENS_HIP(hipGetLastError());
            }
            zeros = reinterpret_cast<const float *>(ws.zeros.ptr);
            if (int rc = grow(ws.sink, ((size_t)N + 8192) * sizeof(float))) return rc;
            sink = reinterpret_cast<float *>(ws.sink.ptr);
        }
    }
    t_state.last_reduction = GIVENS_REDUCTION_TWO_STAGE;

    // Two-stage reduction.  LDS family: one row of partial sums per strip, in chunks of strips that fit
    // the workspace cap.  Carousel family: one row per persistent workgroup (at most what the chip
    // holds at once), whatever the number of strips.
    const long long rows_wanted = carousel ? carousel_bwd_groups(n, B, strips, cus) : strips;
    long long prows = (long long)(kPartialCapBytes / ((size_t)N * sizeof(T)));
    prows = std::max<long long>(1, std::min(prows, rows_wanted));
    // Large carousel sweeps link their persistent workgroups into chains that share rows (fewer rows, and rows
    // that stay in L2 while they are summed): needs the full grid and its rows within the cap
    int chains = 0;
    long long passes = 1;
    if constexpr (std::is_same<T, float>::value) {
        if (carousel && prows == rows_wanted) {
            chains = carousel_bwd_chains(n, B, strips, rows_wanted);
            passes = (strips + rows_wanted - 1) / rows_wanted;
            if (chains && passes * chains > prows) chains = 0;
        }
    }
    t_state.last_chains = chains;
    CarouselChainArgs chain{};
    if (chains) {
        // one flag line per workgroup and block, and the launch counter: zeroed when (re)allocated; after that
        // every launch writes tags larger than all earlier ones
        const size_t flag_words = (size_t)rows_wanted * (size_t)(n - 1) * kFlagStride + 1;
        if (ws.chain_flags.bytes < flag_words * sizeof(unsigned)) {
            if (int rc = grow(ws.chain_flags, flag_words * sizeof(unsigned))) return rc;
            hipLaunchKernelGGL(fill_zero_kernel, dim3(2048), dim3(256), 0, stream,
                               (long long)(ws.chain_flags.bytes / sizeof(float)),
                               reinterpret_cast<float *>(ws.chain_flags.ptr));
            GIVENS_HIP(hipGetLastError());
        }
        unsigned *flags = reinterpret_cast<unsigned *>(ws.chain_flags.ptr);
        unsigned *epoch = flags + (ws.chain_flags.bytes / sizeof(unsigned) - 1);    // the buffer's last word
        const int words = (int)rows_wanted + 1;               // xcd_of, error
        if (int rc = grow(ws.chain, (size_t)words * sizeof(unsigned))) return rc;
        unsigned *cw = reinterpret_cast<unsigned *>(ws.chain.ptr);
        hipLaunchKernelGGL(chain_flags_wrap_kernel, dim3(1024), dim3(256), 0, stream, epoch, flags,
                           (long long)(ws.chain_flags.bytes / sizeof(unsigned) - 1));
        hipLaunchKernelGGL(chain_reset_kernel, dim3((words + 255) / 256), dim3(256), 0, stream, cw, words, epoch);
        GIVENS_HIP(hipGetLastError());
        chain = CarouselChainArgs{flags, cw, cw + rows_wanted, epoch, chains};
    }
    if (int rc = grow(ws.partial, (size_t)prows * N * sizeof(T))) return rc;
    T *partial = reinterpret_cast<T *>(ws.partial.ptr);
    const long long chunk = carousel ? strips : prows;     // strips per launch
    for (long long s0 = 0; s0 < strips; s0 += chunk) {
        const long long ns = std::min(chunk, strips - s0);
        long long nrows = carousel ? std::min(prows, ns) : ns;
        {
            Span span(1, stream);
            if (!carousel) {
                hipLaunchKernelGGL(kern, dim3((unsigned)ns), dim3(kLdsThreads), smem, stream, n, rows, B, w, s0,
                                   coefs.table, Y, G, dX, partial, g_identity, map);
            } else if constexpr (std::is_same<T, float>::value) {
                if (int rc = carousel_backward_strips(n, rows, B, w, s0, ns, nrows, coefs.carousel(), Y, G, dX, partial,
                                                      zeros, sink, g_identity, stream, chains ? &chain : nullptr))
                    return rc;
                if (chains) {
                    // rows of the chains: all of them in every full pass, the heads that still had a strip in the last
                    const long long last = strips - (passes - 1) * rows_wanted;
                    nrows = (passes - 1) * chains + std::min<long long>(chains, last);
                }
            } else {
                return GIVENS_ERR_UNSUPPORTED;
            }
            GIVENS_HIP(hipGetLastError());
        }
        {
            Span span(2, stream);
            const int threads = 256;
            if (N <= kReduceSplitMaxAngles && nrows >= 4 * kReduceSplit)
                hipLaunchKernelGGL(reduce_partials_split_kernel<T>, dim3((unsigned)((N + 63) / 64)),
                                   dim3(64 * kReduceSplit), 0, stream, n, nrows, partial, coefs.factor, map, dtheta,
                                   s0 > 0 ? 1 : 0);
            else
                hipLaunchKernelGGL(reduce_partials_kernel<T>, dim3((unsigned)((N + threads - 1) / threads)),
                                   dim3(threads), 0, stream, n, nrows, partial, coefs.factor, map, dtheta,
                                   s0 > 0 ? 1 : 0, chains ? (const unsigned *)chain.error : nullptr);
            GIVENS_HIP(hipGetLastError());
        }
    }
    return GIVENS_OK;
}

int current_device(int *dev)
{
    GIVENS_HIP(hipGetDevice(dev));
    if (*dev < 0 || *dev >= kMaxDevices) return GIVENS_ERR_UNSUPPORTED;
    return GIVENS_OK;
}

CallOptions default_options() { return CallOptions{g_kernel_choice, g_form_choice, g_reduction_choice}; }

int options_from(const givens_options *o, CallOptions *out)
{
    *out = default_options();
    if (!o) return GIVENS_OK;
    auto in = [](int v, std::initializer_list<int> ok) { return std::find(ok.begin(), ok.end(), v) != ok.end(); };
    if (!in(o->kernel, {GIVENS_KERNEL_AUTO, GIVENS_KERNEL_LDS, GIVENS_KERNEL_CAROUSEL, GIVENS_KERNEL_COLUMN}) ||
        !in(o->rotation_form, {GIVENS_FORM_AUTO, GIVENS_FORM_STANDARD, GIVENS_FORM_LIFTED, GIVENS_FORM_RANGE}) ||
        !in(o->reduction, {GIVENS_REDUCTION_AUTO, GIVENS_REDUCTION_TWO_STAGE, GIVENS_REDUCTION_GRAM}))
        return GIVENS_ERR_UNSUPPORTED;
    *out = CallOptions{o->kernel, o->rotation_form, o->reduction};
    return GIVENS_OK;
}

// A call that writes a coefficient set of the workspace ends the validity of what givens_prepare left there.
void invalidate_prepared(Workspace &ws, bool fwd, bool rev)
{
    if (fwd) ws.prepared.fwd = false;
    if (rev) ws.prepared.rev = false;
    if (!ws.prepared.fwd && !ws.prepared.rev) ws.prepared.token = 0;
}

// rows, m: see Problem.  The unrestricted entry points pass an even rows and m = rows - 1.
template <typename T>
int forward_impl(int rows, int m, long long B, const T *theta, const T *X, T *Y, int identity, void *stream_v,
                 CallOptions opt, int transpose = 0, bool no_alloc = false)
{
    if (int rc = check_restricted(rows, m)) return rc;
    if (B < 1) return GIVENS_ERR_BAD_B;
    if (!theta || !Y || (!identity && !X)) return GIVENS_ERR_NULL;
    // the variant that may not allocate: float, every pair free (no index map), n within the static array
    if (no_alloc && (!std::is_same<T, float>::value || (rows & 1) || m != rows - 1 || rows > kNoAllocMaxN))
        return GIVENS_ERR_UNSUPPORTED;
    hipStream_t stream = reinterpret_cast<hipStream_t>(stream_v);
    std::lock_guard<std::mutex> lock(g_mutex);
    int dev = 0;
    if (int rc = current_device(&dev)) return rc;
    Workspace *ws = nullptr;
    if (!no_alloc)
        if (int rc = workspace_for(dev, stream, &ws)) return rc;
    Problem pb;
    if (int rc = resolve_problem(ws, rows, m, stream, &pb)) return rc;
    const int n = pb.n;
    timing_begin_call();
    if (no_alloc) t_state.timing_valid = false; // event pairs are created on demand: not here
    Families fam;
    if (int rc = pick_forward_family<T>(n, B, opt.kernel, &fam)) return rc;
    Coefs<T> coefs;
    const FormPolicy policy = form_policy(fam.carousel && std::is_same<T, float>::value, n, opt.form, sweep_updates(n, B));
    if (no_alloc) {
        if constexpr (std::is_same<T, float>::value) {
            CoefStorage<float> st;
            if (int rc = static_coef_storage(dev, n, &st)) return rc;
            if (int rc = build_coefs<float>(st, pb, theta, true, policy, stream, &coefs, transpose)) return rc;
        }
    } else {
        invalidate_prepared(*ws, true, false);
        if (int rc = build_coefs<T>(*ws, ws->fwd, pb, theta, true, policy, stream, &coefs, transpose)) return rc;
    }
    return run_forward_sweep<T>(pb, B, coefs, fam, X, Y, identity, transpose, stream);
}

// The reverse sweep of one call, reverse-direction coefficients given; `mirrored_for_dx` builds (or returns) the
// forward-type coefficients of the mirrored problem when the Gram form needs them for dX.
template <typename T, typename MirroredFn>
int run_backward(Workspace &ws, int dev, const Problem &pb, long long B, const Coefs<T> &coefs, Families fam,
                 CallOptions opt, const T *Y, const T *G, T *dX, T *dtheta, hipStream_t stream,
                 MirroredFn &&mirrored_for_dx)
{
    const int n = pb.n, rows = pb.rows;
    t_state.last_kernel = fam.carousel ? GIVENS_KERNEL_CAROUSEL : GIVENS_KERNEL_LDS;
    if constexpr (std::is_same<T, float>::value) {
        // Gram-matrix form for wide batches.  With C = Y G^T (rows x rows) the sums of the reverse sweep
        // are those of the same sweep run on the operand C with the identity as upstream gradient:
        // z_k gbar_k^T = A_k C A_k^T for the product A_k of the transposed blocks so far, and the sweep on
        // (C, I) carries A_k C and A_k.  So dtheta costs one contraction over B plus a rows-column sweep, and
        // dX = U^T G one forward-type sweep over B (mirrored tables), instead of a two-strip sweep over B.
        const bool wide = B >= 2LL * n;   // measured break-even is near B = 1.6 n
        const bool want_gram = opt.reduction == GIVENS_REDUCTION_GRAM || (opt.reduction == GIVENS_REDUCTION_AUTO && wide);
        if (want_gram) {
            int cus = 0;
            GIVENS_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
            const int slices = gram_slices(rows, B, cus);
            if (int rc = grow(ws.gram, (size_t)slices * rows * rows * sizeof(float))) return rc;
            float *C = reinterpret_cast<float *>(ws.gram.ptr);
            {
                Span span(3, stream);
                gram_matrix(rows, B, slices, Y, G, C, stream);
                GIVENS_HIP(hipGetLastError());
            }
            int rc = backward_chunks<T>(ws, dev, fam.carousel, pb, rows, coefs, C, nullptr, nullptr, dtheta, stream, 1);
            if (rc == GIVENS_OK && dX) {
                Coefs<T> mirrored;
                Families dx_fam;
                dx_fam.column = fam.column;
                dx_fam.carousel = !fam.column && fam.carousel;
                rc = mirrored_for_dx(dx_fam, &mirrored);
                if (rc == GIVENS_OK) rc = run_forward_sweep<T>(pb, B, mirrored, dx_fam, G, dX, 0, 1, stream);
            }
            t_state.last_reduction = GIVENS_REDUCTION_GRAM;
            if (fam.column) t_state.last_kernel = GIVENS_KERNEL_COLUMN;
            else t_state.last_kernel = fam.carousel ? GIVENS_KERNEL_CAROUSEL : GIVENS_KERNEL_LDS;
            return rc;
        }
    }
    return backward_chunks<T>(ws, dev, fam.carousel, pb, B, coefs, Y, G, dX, dtheta, stream);
}

template <typename T>
int backward_impl(int rows, int m, long long B, const T *theta, const T *Y, const T *G, T *dX, T *dtheta,
                  void *stream_v, CallOptions opt)
{
    if (int rc = check_restricted(rows, m)) return rc;
    if (B < 1) return GIVENS_ERR_BAD_B;
    if (!theta || !Y || !G || !dtheta) return GIVENS_ERR_NULL;
    if (dX && (const void *)dX == (const void *)Y) return GIVENS_ERR_ALIAS;
    hipStream_t stream = reinterpret_cast<hipStream_t>(stream_v);
    std::lock_guard<std::mutex> lock(g_mutex);
    int dev = 0;
    if (int rc = current_device(&dev)) return rc;
    Workspace *ws = nullptr;
    if (int rc = workspace_for(dev, stream, &ws)) return rc;
    Problem pb;
    if (int rc = resolve_problem(ws, rows, m, stream, &pb)) return rc;
    const int n = pb.n;
    timing_begin_call();
    Families fam;
    if (int rc = pick_backward_family<T>(n, B, opt.kernel, &fam)) return rc;
    invalidate_prepared(*ws, false, true);
    Coefs<T> coefs;
    if (int rc = build_coefs<T>(*ws, ws->rev, pb, theta, false,
                                form_policy(fam.carousel && std::is_same<T, float>::value, n, opt.form, sweep_updates(n, B)),
                                stream, &coefs))
        return rc;
    auto mirrored_for_dx = [&](Families dx_fam, Coefs<T> *out) {
        return build_coefs<T>(*ws, ws->mirrored, pb, theta, true,
                              form_policy(dx_fam.carousel && std::is_same<T, float>::value, n, opt.form, sweep_updates(n, B)),
                              stream, out, 1);
    };
    return run_backward<T>(*ws, dev, pb, B, coefs, fam, opt, Y, G, dX, dtheta, stream, mirrored_for_dx);
}

// ---- prepared coefficients (float): givens_prepare builds the tables of one theta once, in the workspace of
// the stream, and the *_prepared calls run the sweeps on them.
int64_t prepare_impl(int rows, int m, const float *theta, int directions, void *stream_v, CallOptions opt,
                     long long batch_hint = 0)
{
    if (int rc = check_restricted(rows, m)) return rc;
    if (!theta) return GIVENS_ERR_NULL;
    constexpr int kAll = GIVENS_PREPARE_FORWARD | GIVENS_PREPARE_BACKWARD | GIVENS_PREPARE_BACKWARD_WIDE;
    if (!(directions & kAll) || (directions & ~kAll)) return GIVENS_ERR_UNSUPPORTED;
    if (directions & GIVENS_PREPARE_BACKWARD_WIDE) directions |= GIVENS_PREPARE_BACKWARD;
    hipStream_t stream = reinterpret_cast<hipStream_t>(stream_v);
    std::lock_guard<std::mutex> lock(g_mutex);
    int dev = 0;
    if (int rc = current_device(&dev)) return rc;
    Workspace *ws = nullptr;
    if (int rc = workspace_for(dev, stream, &ws)) return rc;
    Problem pb;
    if (int rc = resolve_problem(ws, rows, m, stream, &pb)) return rc;
    const int n = pb.n;
    timing_begin_call();
    // the family does not depend on B (B >= 1 is all the shape checks look at)
    const bool fwd = (directions & GIVENS_PREPARE_FORWARD) != 0, rev = (directions & GIVENS_PREPARE_BACKWARD) != 0;
    Families ffam, bfam;
    if (fwd)
        if (int rc = pick_forward_family<float>(n, 1, opt.kernel, &ffam)) return rc;
    if (rev)
        if (int rc = pick_backward_family<float>(n, 1, opt.kernel, &bfam)) return rc;
    ws->prepared = Prepared{};
    Coefs<float> c;
    bool range_known = false, mirrored_forms = false;
    // without a hint the batch is not known here and AUTO means GIVENS_FORM_RANGE
    const double kAnyBatch = batch_hint > 0 ? sweep_updates(n, batch_hint) : 1.0e300;
    const FormPolicy fpol = form_policy(ffam.carousel, n, opt.form, kAnyBatch), bpol = form_policy(bfam.carousel, n, opt.form, kAnyBatch);
    // one range check for all the sets, into the flag word that belongs to givens_prepare
    auto build = [&](CoefSet &set, bool forward, FormPolicy pol, int mirror) {
        if (pol.try_forms && !range_known) {
            if (!ws->flag.ptr) {
                if (int rc = grow(ws->flag, kFlagBytes)) return rc;
                if (!hip_ok(hipMemsetAsync(ws->flag.ptr, 0, kFlagBytes, stream))) return (int)GIVENS_ERR_HIP;
            }
            hipLaunchKernelGGL(reset_flag_kernel, dim3(1), dim3(1), 0, stream, reinterpret_cast<unsigned *>(ws->flag.ptr) + 2);
        }
        const int rc = build_coefs<float>(*ws, set, pb, theta, forward, pol, stream, &c, mirror, range_known, true);
        range_known = range_known || pol.try_forms;
        return rc;
    };
    if (fwd)
        if (int rc = build(ws->fwd, true, fpol, 0)) return rc;
    if (rev) {
        if (int rc = build(ws->rev, false, bpol, 0)) return rc;
    }
    const bool wide = (directions & GIVENS_PREPARE_BACKWARD_WIDE) != 0;
    if (wide) {
        // the Gram form's dX sweep (wide batches) reads forward-type tables of the mirrored problem
        Families dx_fam;
        dx_fam.column = bfam.column;
        dx_fam.carousel = !bfam.column && bfam.carousel;
        const FormPolicy mpol = form_policy(dx_fam.carousel, n, opt.form, kAnyBatch);
        if (int rc = build(ws->mirrored, true, mpol, 1)) return rc;
        mirrored_forms = mpol.try_forms;
    }
    Prepared &p = ws->prepared;
    p.token = ++g_next_token;
    p.rows = rows;
    p.m = m;
    p.fwd = fwd;
    p.rev = rev;
    p.mirrored = wide;
    p.fwd_forms = fwd && fpol.try_forms;
    p.rev_forms = rev && bpol.try_forms;
    p.mirrored_forms = wide && mirrored_forms;
    p.scaled_max = form_policy(true, n, opt.form, kAnyBatch).scaled_max;
    return p.token;
}

// coefficients of a prepared set, as build_coefs would have returned them
Coefs<float> prepared_coefs(Workspace &ws, const CoefSet &set, bool reverse, bool forms, float scaled_max)
{
    Coefs<float> c;
    c.table = reinterpret_cast<const float2 *>(set.table.ptr);
    c.factor = reverse ? reinterpret_cast<const float *>(set.factor.ptr) : nullptr;
    if (forms) {
        c.renorm = reinterpret_cast<const float2 *>(set.renorm.ptr);
        c.flag = reinterpret_cast<const unsigned *>(ws.flag.ptr) + 2;
        c.scaled_max = scaled_max;
    }
    t_state.last_flag = c.flag;
    t_state.last_scaled_max = scaled_max;
    return c;
}

int prepared_workspace(int64_t token, hipStream_t stream, int *dev, Workspace **ws)
{
    if (token <= 0) return GIVENS_ERR_STALE;
    if (int rc = current_device(dev)) return rc;
    for (auto &w : g_ws[*dev])
        if (w->stream == stream && w->prepared.token == token) {
            w->last_use = ++g_use_clock;
            *ws = w.get();
            return GIVENS_OK;
        }
    return GIVENS_ERR_STALE;
}

int forward_prepared_impl(int64_t token, long long B, const float *X, float *Y, int identity, void *stream_v,
                          CallOptions opt)
{
    if (B < 1 && !identity) return GIVENS_ERR_BAD_B;
    if (!Y || (!identity && !X)) return GIVENS_ERR_NULL;
    hipStream_t stream = reinterpret_cast<hipStream_t>(stream_v);
    std::lock_guard<std::mutex> lock(g_mutex);
    int dev = 0;
    Workspace *ws = nullptr;
    if (int rc = prepared_workspace(token, stream, &dev, &ws)) return rc;
    if (!ws->prepared.fwd) return GIVENS_ERR_STALE;
    Problem pb;
    if (int rc = resolve_problem(ws, ws->prepared.rows, ws->prepared.m, stream, &pb)) return rc;
    if (identity) B = pb.rows;
    timing_begin_call();
    t_state.last_stream = stream;
    Families fam;
    if (int rc = pick_forward_family<float>(pb.n, B, opt.kernel, &fam)) return rc;
    if (ws->prepared.fwd_forms && !fam.carousel) return GIVENS_ERR_STALE; // another family than the one prepared for
    const Coefs<float> coefs = prepared_coefs(*ws, ws->fwd, false, ws->prepared.fwd_forms, ws->prepared.scaled_max);
    return run_forward_sweep<float>(pb, B, coefs, fam, X, Y, identity, 0, stream);
}

int backward_prepared_impl(int64_t token, long long B, const float *Y, const float *G, float *dX, float *dtheta,
                           void *stream_v, CallOptions opt)
{
    if (B < 1) return GIVENS_ERR_BAD_B;
    if (!Y || !G || !dtheta) return GIVENS_ERR_NULL;
    if (dX && (const void *)dX == (const void *)Y) return GIVENS_ERR_ALIAS;
    hipStream_t stream = reinterpret_cast<hipStream_t>(stream_v);
    std::lock_guard<std::mutex> lock(g_mutex);
    int dev = 0;
    Workspace *ws = nullptr;
    if (int rc = prepared_workspace(token, stream, &dev, &ws)) return rc;
    if (!ws->prepared.rev) return GIVENS_ERR_STALE;
    Problem pb;
    if (int rc = resolve_problem(ws, ws->prepared.rows, ws->prepared.m, stream, &pb)) return rc;
    timing_begin_call();
    t_state.last_stream = stream;
    Families fam;
    if (int rc = pick_backward_family<float>(pb.n, B, opt.kernel, &fam)) return rc;
    const Prepared prep = ws->prepared;
    if (prep.rev_forms && !fam.carousel) return GIVENS_ERR_STALE;         // another family than the one prepared for
    if (!prep.mirrored) {
        // no tables for the Gram form's dX sweep: the two-stage sweep over all B columns serves any B
        if (opt.reduction == GIVENS_REDUCTION_GRAM) return GIVENS_ERR_STALE;
        opt.reduction = GIVENS_REDUCTION_TWO_STAGE;
    }
    const Coefs<float> coefs = prepared_coefs(*ws, ws->rev, true, prep.rev_forms, prep.scaled_max);
    auto mirrored_for_dx = [&](Families dx_fam, Coefs<float> *out) {
        if (prep.mirrored_forms && !dx_fam.carousel) return (int)GIVENS_ERR_STALE;
        *out = prepared_coefs(*ws, ws->mirrored, false, prep.mirrored_forms, prep.scaled_max);
        return (int)GIVENS_OK;
    };
    return run_backward<float>(*ws, dev, pb, B, coefs, fam, opt, Y, G, dX, dtheta, stream, mirrored_for_dx);
}

// ---- unitary extension (appendix): complex operands, LDS strip kernels
template <typename T>
int unitary_strip_width(int n, long long B, int strips_in_lds)
{
    int w = 7;
    while (w > 1 && (size_t)n * w * 2 * sizeof(T) * strips_in_lds > kLdsBudgetBytes) --w;
    if ((size_t)n * w * 2 * sizeof(T) * strips_in_lds > kLdsBudgetBytes) return 0;
    while (w > 1 && (B + w - 1) / w < 1024) --w;
    return w;
}

template <typename T>
int unitary_table(Workspace &ws, int n, const T *theta, const T *phi, hipStream_t stream,
                  const typename Cplx<T>::quad **out)
{
    const long long N = (long long)n * (n - 1) / 2;
    invalidate_prepared(ws, true, false);
    if (int rc = grow(ws.fwd.table, (size_t)N * sizeof(typename Cplx<T>::quad))) return rc;
    auto *table = reinterpret_cast<typename Cplx<T>::quad *>(ws.fwd.table.ptr);
    Span span(0, stream);
    const int threads = 256;
    const unsigned blocks = (unsigned)std::min<long long>((N + threads - 1) / threads, 4096);
    hipLaunchKernelGGL(unitary_table_kernel<T>, dim3(blocks), dim3(threads), 0, stream, n, theta, phi, table);
    GIVENS_HIP(hipGetLastError());
    *out = table;
    return GIVENS_OK;
}

// Unitary extension in the carousel family (complex64, n a multiple of 16 from 128 to 4096): coefficients of one
// sweep direction into the workspace.
struct UnitaryCoefs {
    const float2 *rot, *phs, *fin;
    const float *orient, *sgn;
};
int unitary_carousel_coefs(Workspace &ws, int n, const float *theta, const float *phi, bool reverse,
                           hipStream_t stream, UnitaryCoefs *out)
{
    const size_t N = (size_t)n * (n - 1) / 2;
    if (int rc = grow(ws.u_q, N * sizeof(uint2))) return rc;
    if (int rc = grow(ws.u_psi, N * sizeof(int))) return rc;
    if (int rc = grow(ws.u_sgn, N * sizeof(float))) return rc;
    if (int rc = grow(ws.u_rot, N * sizeof(float2))) return rc;
    if (int rc = grow(ws.u_phs, N * sizeof(float2))) return rc;
    if (int rc = grow(ws.u_fin, (size_t)n * sizeof(float2))) return rc;
    if (reverse)
        if (int rc = grow(ws.u_orient, N * sizeof(float))) return rc;
    Span span(0, stream);
    auto *orient = reverse ? reinterpret_cast<float *>(ws.u_orient.ptr) : nullptr;
    if (int rc = unitary_carousel_coefficients(n, theta, phi, reverse ? 1 : 0,
                                               reinterpret_cast<uint2 *>(ws.u_q.ptr),
                                               reinterpret_cast<unsigned *>(ws.u_psi.ptr),
                                               reinterpret_cast<float *>(ws.u_sgn.ptr),
                                               reinterpret_cast<float2 *>(ws.u_rot.ptr),
                                               reinterpret_cast<float2 *>(ws.u_phs.ptr), orient,
                                               reinterpret_cast<float2 *>(ws.u_fin.ptr), stream))
        return rc;
    GIVENS_HIP(hipGetLastError());
    *out = UnitaryCoefs{reinterpret_cast<const float2 *>(ws.u_rot.ptr), reinterpret_cast<const float2 *>(ws.u_phs.ptr),
                        reinterpret_cast<const float2 *>(ws.u_fin.ptr), orient,
                        reinterpret_cast<const float *>(ws.u_sgn.ptr)};
    return GIVENS_OK;
}

bool unitary_wants_carousel(int n, int kernel_choice)
{
    return unitary_carousel_supported(n) && (kernel_choice == GIVENS_KERNEL_AUTO || kernel_choice == GIVENS_KERNEL_CAROUSEL);
}

int unitary_carousel_forward(Workspace &ws, int n, long long B, const float *theta, const float *phi, const float *X,
                             float *Y, int identity, hipStream_t stream)
{
    UnitaryCoefs c;
    if (int rc = unitary_carousel_coefs(ws, n, theta, phi, false, stream, &c)) return rc;
    const long long Breal = 2 * B;
    const int waves = (n / 16 + 63) / 64;
    int W = carousel_width(Breal, waves);
    if (W < 2) W = 2;
    const bool aligned = (Breal % 4 == 0) && (reinterpret_cast<uintptr_t>(Y) % 16 == 0) &&
                         (identity || reinterpret_cast<uintptr_t>(X) % 16 == 0);
    Span span(1, stream);
    const UnitaryCarouselFwdArgs a{n, Breal, c.rot, c.phs, c.fin, X, Y, identity, aligned ? 1 : 0, stream};
    if (int rc = unitary_carousel_forward_m8(a, waves, W)) return rc;
    GIVENS_HIP(hipGetLastError());
    t_state.last_kernel = GIVENS_KERNEL_CAROUSEL;
    return GIVENS_OK;
}

int unitary_carousel_backward(Workspace &ws, int dev, int n, long long B, const float *theta, const float *phi,
                              const float *Y, const float *G, float *dX, float *dtheta, float *dphi,
                              hipStream_t stream)
{
    UnitaryCoefs c;
    if (int rc = unitary_carousel_coefs(ws, n, theta, phi, true, stream, &c)) return rc;
    const long long N = (long long)n * (n - 1) / 2;
    const long long Breal = 2 * B;
    // Shape.  Two slots per lane with strips of 8 floats (four complex numbers) where n <= 2048 and the batch is
    // wide enough to keep the chip busy: half the rows of partial sums of the alternative, four slots per lane
    // with strips of 4 floats (or 2 for narrow batches), which a lane's registers limit to that width.
    // (measured at n = 2048, B = 2048: sweep 8.6 -> 5.2 ms, second stage 1.9 -> 1.0 ms.)
    const bool two_slots = n <= 2048 && ((Breal + 7) / 8) * ((n / 4 + 63) / 64) >= 512;
    const int M = two_slots ? 2 : 4;
    const int waves = (n / (2 * M) + 63) / 64;
    const int W = M == 2 ? 8 : ((((Breal + 3) / 4) * waves >= 512) ? 4 : 2);
    const long long strips = (Breal + W - 1) / W;
    int cus = 0;
    GIVENS_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    const long long resident = (long long)cus * (8 / waves > 0 ? 8 / waves : 1);
    long long groups = std::min(strips, resident);
    const long long cap_rows = (long long)(kPartialCapBytes / ((size_t)2 * N * sizeof(float)));
    groups = std::max<long long>(1, std::min(groups, cap_rows));
    if (int rc = grow(ws.partial, (size_t)2 * groups * N * sizeof(float))) return rc;
    const size_t want = (size_t)N * sizeof(float);
    if (ws.zeros.bytes < want) {
        if (int rc = grow(ws.zeros, want)) return rc;
        hipLaunchKernelGGL(fill_zero_kernel, dim3(2048), dim3(256), 0, stream, N, reinterpret_cast<float *>(ws.zeros.ptr));
        GIVENS_HIP(hipGetLastError());
    }
    if (int rc = grow(ws.sink, ((size_t)N + 8192) * sizeof(float))) return rc;
    float *partial = reinterpret_cast<float *>(ws.partial.ptr);
    const bool aligned = (Breal % 4 == 0) && (reinterpret_cast<uintptr_t>(Y) % 16 == 0) &&
                         (reinterpret_cast<uintptr_t>(G) % 16 == 0) && (!dX || reinterpret_cast<uintptr_t>(dX) % 16 == 0);
    {
        Span span(1, stream);
        const UnitaryCarouselBwdArgs a{n, Breal, 0, strips, groups, c.rot, c.phs, c.orient, c.fin, Y, G, dX, partial,
                                       reinterpret_cast<const float *>(ws.zeros.ptr),
                                       reinterpret_cast<float *>(ws.sink.ptr), aligned ? 1 : 0, stream};
        if (int rc = M == 2 ? unitary_carousel_backward_m2(a, waves, W) : unitary_carousel_backward_m4(a, waves, W))
            return rc;
        GIVENS_HIP(hipGetLastError());
    }
    {
        Span span(2, stream);
        const int threads = 256;
        const unsigned blocks = (unsigned)((N + threads - 1) / threads);
        hipLaunchKernelGGL(reduce_partials_kernel<float>, dim3(blocks), dim3(threads), 0, stream, n, groups, partial,
                           c.sgn, (const int *)nullptr, dtheta, 0);
        hipLaunchKernelGGL(reduce_partials_kernel<float>, dim3(blocks), dim3(threads), 0, stream, n, groups,
                           partial + groups * N, (const float *)nullptr, (const int *)nullptr, dphi, 0);
        GIVENS_HIP(hipGetLastError());
    }
    t_state.last_kernel = GIVENS_KERNEL_CAROUSEL;
    t_state.last_reduction = GIVENS_REDUCTION_TWO_STAGE;
    t_state.last_chains = 0;
    t_state.last_flag = nullptr;
    return GIVENS_OK;
}

template <typename T>
int unitary_forward_impl(int n, long long B, const T *theta, const T *phi, const T *X, T *Y, int identity,
                         void *stream_v)
{
    using C = typename Cplx<T>::type;
    if (int rc = check_n(n)) return rc;
    if (B < 1) return GIVENS_ERR_BAD_B;
    if (!theta || !phi || !Y || (!identity && !X)) return GIVENS_ERR_NULL;
    hipStream_t stream = reinterpret_cast<hipStream_t>(stream_v);
    std::lock_guard<std::mutex> lock(g_mutex);
    int dev = 0;
    if (int rc = current_device(&dev)) return rc;
    timing_begin_call();
    Workspace *ws = nullptr;
    if constexpr (std::is_same<T, float>::value) {
        if (unitary_wants_carousel(n, g_kernel_choice)) {
            if (int rc = workspace_for(dev, stream, &ws)) return rc;
            return unitary_carousel_forward(*ws, n, B, theta, phi, X, Y, identity, stream);
        }
    }
    if (g_kernel_choice == GIVENS_KERNEL_CAROUSEL || g_kernel_choice == GIVENS_KERNEL_COLUMN) return GIVENS_ERR_UNSUPPORTED;
    const int w = unitary_strip_width<T>(n, B, 1);
    if (w == 0) return GIVENS_ERR_UNSUPPORTED;
    const typename Cplx<T>::quad *table = nullptr;
    if (int rc = workspace_for(dev, stream, &ws)) return rc;
    if (int rc = unitary_table<T>(*ws, n, theta, phi, stream, &table)) return rc;
    const size_t smem = (size_t)n * w * sizeof(C);
    auto kern = lds_wants_ahead(n) ? unitary_forward_kernel<T, kUnitaryAhead> : unitary_forward_kernel<T, 0>;
    GIVENS_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    Span span(1, stream);
    hipLaunchKernelGGL(kern, dim3((unsigned)((B + w - 1) / w)), dim3(kUnitaryThreads), smem, stream, n, B, w, table,
                       reinterpret_cast<const C *>(X), reinterpret_cast<C *>(Y), identity);
    GIVENS_HIP(hipGetLastError());
    t_state.last_kernel = GIVENS_KERNEL_LDS;
    return GIVENS_OK;
}

template <typename T>
int unitary_backward_impl(int n, long long B, const T *theta, const T *phi, const T *Y, const T *G, T *dX,
                          T *dtheta, T *dphi, void *stream_v)
{
    using C = typename Cplx<T>::type;
    if (int rc = check_n(n)) return rc;
    if (B < 1) return GIVENS_ERR_BAD_B;
    if (!theta || !phi || !Y || !G || !dtheta || !dphi) return GIVENS_ERR_NULL;
    if (dX && (const void *)dX == (const void *)Y) return GIVENS_ERR_ALIAS;
    hipStream_t stream = reinterpret_cast<hipStream_t>(stream_v);
    std::lock_guard<std::mutex> lock(g_mutex);
    int dev = 0;
    if (int rc = current_device(&dev)) return rc;
    timing_begin_call();
    Workspace *wsp = nullptr;
    if constexpr (std::is_same<T, float>::value) {
        if (unitary_wants_carousel(n, g_kernel_choice)) {
            if (int rc = workspace_for(dev, stream, &wsp)) return rc;
            return unitary_carousel_backward(*wsp, dev, n, B, theta, phi, Y, G, dX, dtheta, dphi, stream);
        }
    }
    if (g_kernel_choice == GIVENS_KERNEL_CAROUSEL || g_kernel_choice == GIVENS_KERNEL_COLUMN) return GIVENS_ERR_UNSUPPORTED;
    const int w = unitary_strip_width<T>(n, B, 2);
    if (w == 0) return GIVENS_ERR_UNSUPPORTED;
    const typename Cplx<T>::quad *table = nullptr;
    if (int rc = workspace_for(dev, stream, &wsp)) return rc;
    Workspace &ws = *wsp;
    if (int rc = unitary_table<T>(ws, n, theta, phi, stream, &table)) return rc;
    const long long N = (long long)n * (n - 1) / 2;
    const long long strips = (B + w - 1) / w;
    long long rows = (long long)(kPartialCapBytes / ((size_t)2 * N * sizeof(T)));
    rows = std::max<long long>(1, std::min(rows, strips));
    if (int rc = grow(ws.partial, (size_t)rows * 2 * N * sizeof(T))) return rc;
    T *partial = reinterpret_cast<T *>(ws.partial.ptr);
    const size_t smem = (size_t)2 * n * w * sizeof(C);
    auto kern = lds_wants_ahead(n) ? unitary_backward_kernel<T, kUnitaryAhead> : unitary_backward_kernel<T, 0>;
    GIVENS_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    for (long long s0 = 0; s0 < strips; s0 += rows) {
        const long long ns = std::min(rows, strips - s0);
        {
            Span span(1, stream);
            hipLaunchKernelGGL(kern, dim3((unsigned)ns), dim3(kUnitaryThreads), smem, stream, n, B, w, s0, table,
                               reinterpret_cast<const C *>(Y), reinterpret_cast<const C *>(G),
                               reinterpret_cast<C *>(dX), partial);
            GIVENS_HIP(hipGetLastError());
        }
        {
            Span span(2, stream);
            const int threads = 256;
            const unsigned blocks = (unsigned)((N + threads - 1) / threads);
            hipLaunchKernelGGL(sum_rows_kernel<T>, dim3(blocks), dim3(threads), 0, stream, N, ns, 2 * N, partial,
                               dtheta, s0 > 0 ? 1 : 0);
            hipLaunchKernelGGL(sum_rows_kernel<T>, dim3(blocks), dim3(threads), 0, stream, N, ns, 2 * N, partial + N,
                               dphi, s0 > 0 ? 1 : 0);
            GIVENS_HIP(hipGetLastError());
        }
    }
    t_state.last_kernel = GIVENS_KERNEL_LDS;
    t_state.last_reduction = GIVENS_REDUCTION_TWO_STAGE;
    t_state.last_chains = 0;
    t_state.last_flag = nullptr;
    return GIVENS_OK;
}

} // namespace
} // namespace givens

extern "C" {

int rr_schedule(int n, int32_t *pairs)
{
    if (n < 2 || (n & 1)) return GIVENS_ERR_BAD_N;
    if (!pairs) return GIVENS_ERR_NULL;
    const int H = n / 2;
    for (int k = 0; k < n - 1; ++k) {
        for (int p = 0; p < H; ++p) {
            const int a = rr_label(n, k, p), b = rr_label(n, k, n - 1 - p);
            int32_t *out = pairs + ((size_t)k * H + p) * 2;
            out[0] = a < b ? a : b;
            out[1] = a < b ? b : a;
        }
    }
    return GIVENS_OK;
}

int givens_forward(int n, int64_t B, const float *theta, const float *X, float *Y, void *stream)
{
    if (int rc = givens::check_n(n)) return rc;
    return givens::forward_impl<float>(n, n - 1, B, theta, X, Y, 0, stream, givens::default_options());
}
int givens_build(int n, const float *theta, float *U, void *stream)
{
    if (int rc = givens::check_n(n)) return rc;
    return givens::forward_impl<float>(n, n - 1, n, theta, nullptr, U, 1, stream, givens::default_options());
}
int givens_backward(int n, int64_t B, const float *theta, const float *Y, const float *G, float *dX,
                    float *dtheta, void *stream)
{
    if (int rc = givens::check_n(n)) return rc;
    return givens::backward_impl<float>(n, n - 1, B, theta, Y, G, dX, dtheta, stream, givens::default_options());
}
int givens_forward_f64(int n, int64_t B, const double *theta, const double *X, double *Y, void *stream)
{
    if (int rc = givens::check_n(n)) return rc;
    return givens::forward_impl<double>(n, n - 1, B, theta, X, Y, 0, stream, givens::default_options());
}
int givens_build_f64(int n, const double *theta, double *U, void *stream)
{
    if (int rc = givens::check_n(n)) return rc;
    return givens::forward_impl<double>(n, n - 1, n, theta, nullptr, U, 1, stream, givens::default_options());
}
int givens_backward_f64(int n, int64_t B, const double *theta, const double *Y, const double *G,
                        double *dX, double *dtheta, void *stream)
{
    if (int rc = givens::check_n(n)) return rc;
    return givens::backward_impl<double>(n, n - 1, B, theta, Y, G, dX, dtheta, stream, givens::default_options());
}

int givens_forward_transposed(int n, int64_t B, const float *theta, const float *X, float *Y, void *stream)
{
    if (int rc = givens::check_n(n)) return rc;
    return givens::forward_impl<float>(n, n - 1, B, theta, X, Y, 0, stream, givens::default_options(), 1);
}
int givens_forward_transposed_f64(int n, int64_t B, const double *theta, const double *X, double *Y, void *stream)
{
    if (int rc = givens::check_n(n)) return rc;
    return givens::forward_impl<double>(n, n - 1, B, theta, X, Y, 0, stream, givens::default_options(), 1);
}

int givens_forward_noalloc(int n, int64_t B, const float *theta, const float *X, float *Y, void *stream)
{
    if (int rc = givens::check_n(n)) return rc;
    return givens::forward_impl<float>(n, n - 1, B, theta, X, Y, 0, stream, givens::default_options(), 0, true);
}

int givens_forward_ex(int n, int m, int64_t B, const float *theta, const float *X, float *Y, void *stream,
                      const givens_options *options)
{
    givens::CallOptions opt;
    if (int rc = givens::options_from(options, &opt)) return rc;
    if (!X && B != n) return GIVENS_ERR_BAD_B;   // X == NULL: the operand is I_n
    return givens::forward_impl<float>(n, m, B, theta, X, Y, X ? 0 : 1, stream, opt);
}
int givens_backward_ex(int n, int m, int64_t B, const float *theta, const float *Y, const float *G, float *dX,
                       float *dtheta, void *stream, const givens_options *options)
{
    givens::CallOptions opt;
    if (int rc = givens::options_from(options, &opt)) return rc;
    return givens::backward_impl<float>(n, m, B, theta, Y, G, dX, dtheta, stream, opt);
}

int64_t givens_prepare(int n, const float *theta, int directions, void *stream)
{
    if (int rc = givens::check_n(n)) return rc;
    return givens::prepare_impl(n, n - 1, theta, directions, stream, givens::default_options());
}
int64_t givens_prepare_restricted(int n, int m, const float *theta, int directions, void *stream)
{
    return givens::prepare_impl(n, m, theta, directions, stream, givens::default_options());
}
int64_t givens_prepare_ex(int n, int m, const float *theta, int directions, int64_t batch_hint, void *stream,
                          const givens_options *options)
{
    givens::CallOptions opt;
    if (int rc = givens::options_from(options, &opt)) return rc;
    if (batch_hint < 0) return GIVENS_ERR_BAD_B;
    return givens::prepare_impl(n, m, theta, directions, stream, opt, batch_hint);
}
int givens_forward_prepared(int64_t token, int64_t B, const float *X, float *Y, void *stream)
{
    return givens::forward_prepared_impl(token, B, X, Y, 0, stream, givens::default_options());
}
int givens_build_prepared(int64_t token, float *U, void *stream)
{
    return givens::forward_prepared_impl(token, 0, nullptr, U, 1, stream, givens::default_options());
}
int givens_backward_prepared(int64_t token, int64_t B, const float *Y, const float *G, float *dX, float *dtheta,
                             void *stream)
{
    return givens::backward_prepared_impl(token, B, Y, G, dX, dtheta, stream, givens::default_options());
}

int64_t givens_num_angles(int n, int m)
{
    if (int rc = givens::check_restricted(n, m)) return rc;
    return givens::count_free_angles(n, m);
}

int rr_schedule_restricted(int n, int m, int32_t *pairs)
{
    if (int rc = givens::check_restricted(n, m)) return rc;
    if (!pairs) return GIVENS_ERR_NULL;
    long long next = 0;
    givens::walk_pairs(n, m, [&](long long, int i, int j, bool is_free) {
        if (!is_free) return;
        pairs[2 * next] = i;
        pairs[2 * next + 1] = j;
        ++next;
    });
    return GIVENS_OK;
}

int givens_forward_restricted(int n, int m, int64_t B, const float *theta, const float *X, float *Y, void *stream)
{
    return givens::forward_impl<float>(n, m, B, theta, X, Y, 0, stream, givens::default_options());
}
int givens_build_restricted(int n, int m, const float *theta, float *U, void *stream)
{
    return givens::forward_impl<float>(n, m, n, theta, nullptr, U, 1, stream, givens::default_options());
}
int givens_backward_restricted(int n, int m, int64_t B, const float *theta, const float *Y, const float *G,
                               float *dX, float *dtheta, void *stream)
{
    return givens::backward_impl<float>(n, m, B, theta, Y, G, dX, dtheta, stream, givens::default_options());
}
int givens_forward_restricted_f64(int n, int m, int64_t B, const double *theta, const double *X, double *Y,
                                  void *stream)
{
    return givens::forward_impl<double>(n, m, B, theta, X, Y, 0, stream, givens::default_options());
}
int givens_build_restricted_f64(int n, int m, const double *theta, double *U, void *stream)
{
    return givens::forward_impl<double>(n, m, n, theta, nullptr, U, 1, stream, givens::default_options());
}
int givens_backward_restricted_f64(int n, int m, int64_t B, const double *theta, const double *Y, const double *G,
                                   double *dX, double *dtheta, void *stream)
{
    return givens::backward_impl<double>(n, m, B, theta, Y, G, dX, dtheta, stream, givens::default_options());
}

int givens_unitary_forward(int n, int64_t B, const float *theta, const float *phi, const float *X, float *Y,
                           void *stream)
{
    return givens::unitary_forward_impl<float>(n, B, theta, phi, X, Y, 0, stream);
}
int givens_unitary_build(int n, const float *theta, const float *phi, float *U, void *stream)
{
    return givens::unitary_forward_impl<float>(n, n, theta, phi, nullptr, U, 1, stream);
}
int givens_unitary_backward(int n, int64_t B, const float *theta, const float *phi, const float *Y, const float *G,
                            float *dX, float *dtheta, float *dphi, void *stream)
{
    return givens::unitary_backward_impl<float>(n, B, theta, phi, Y, G, dX, dtheta, dphi, stream);
}
int givens_unitary_forward_f64(int n, int64_t B, const double *theta, const double *phi, const double *X,
                               double *Y, void *stream)
{
    return givens::unitary_forward_impl<double>(n, B, theta, phi, X, Y, 0, stream);
}
int givens_unitary_build_f64(int n, const double *theta, const double *phi, double *U, void *stream)
{
    return givens::unitary_forward_impl<double>(n, n, theta, phi, nullptr, U, 1, stream);
}
int givens_unitary_backward_f64(int n, int64_t B, const double *theta, const double *phi, const double *Y,
                                const double *G, double *dX, double *dtheta, double *dphi, void *stream)
{
    return givens::unitary_backward_impl<double>(n, B, theta, phi, Y, G, dX, dtheta, dphi, stream);
}

int givens_release(void)
{
    using namespace givens;
    std::lock_guard<std::mutex> lock(g_mutex);
    int keep = 0;
    if (!hip_ok(hipGetDevice(&keep))) return GIVENS_ERR_HIP;
    int rc = GIVENS_OK;
    for (int d = 0; d < kMaxDevices; ++d) {
        if (g_ws[d].empty()) continue;
        if (!hip_ok(hipSetDevice(d))) { rc = GIVENS_ERR_HIP; continue; }
        if (!hip_ok(hipDeviceSynchronize())) rc = GIVENS_ERR_HIP;
        for (auto &w : g_ws[d])
            if (free_workspace(*w) != GIVENS_OK) rc = GIVENS_ERR_HIP;
        g_ws[d].clear();
    }
    (void)hipSetDevice(keep);
    return rc;
}

int givens_last_hip_error(void) { return givens::t_state.last_hip_error; }

const char *givens_error_string(int code)
{
    switch (code) {
    case GIVENS_OK: return "success";
    case GIVENS_ERR_BAD_N: return "n must be even and at least 2";
    case GIVENS_ERR_BAD_B: return "B must be at least 1";
    case GIVENS_ERR_NULL: return "a required pointer is NULL";
    case GIVENS_ERR_HIP: return "a HIP call failed (see givens_last_hip_error)";
    case GIVENS_ERR_UNSUPPORTED: return "shape or option not supported by the requested kernel";
    case GIVENS_ERR_ALIAS: return "forbidden aliasing between arguments";
    case GIVENS_ERR_BAD_M: return "m must satisfy 1 <= m <= n - 1";
    case GIVENS_ERR_STALE: return "the prepared coefficients are no longer in the stream's workspace";
    default: return "unknown error code";
    }
}

int givens_set_kernel(int which)
{
    if (which != GIVENS_KERNEL_AUTO && which != GIVENS_KERNEL_LDS && which != GIVENS_KERNEL_CAROUSEL &&
        which != GIVENS_KERNEL_COLUMN)
        return GIVENS_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(givens::g_mutex);
    const int prev = givens::g_kernel_choice;
    givens::g_kernel_choice = which;
    return prev;
}

int givens_last_kernel(void) { return givens::t_state.last_kernel; }

int givens_set_reduction(int which)
{
    if (which != GIVENS_REDUCTION_AUTO && which != GIVENS_REDUCTION_TWO_STAGE && which != GIVENS_REDUCTION_GRAM)
        return GIVENS_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(givens::g_mutex);
    const int prev = givens::g_reduction_choice;
    givens::g_reduction_choice = which;
    return prev;
}

int givens_last_reduction(void) { return givens::t_state.last_reduction; }
int givens_last_chains(void) { return givens::t_state.last_chains; }


int givens_set_rotation_form(int which)
{
    if (which != GIVENS_FORM_AUTO && which != GIVENS_FORM_STANDARD && which != GIVENS_FORM_LIFTED &&
        which != GIVENS_FORM_RANGE)
        return GIVENS_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(givens::g_mutex);
    const int prev = givens::g_form_choice;
    givens::g_form_choice = which;
    return prev;
}

int givens_last_rotation_form(void)
{
    using namespace givens;
    ThreadState &ts = t_state;
    if (!ts.last_flag) return GIVENS_FORM_STANDARD;
    unsigned bits = 0;
    if (!hip_ok(hipMemcpyAsync(&bits, ts.last_flag, sizeof(bits), hipMemcpyDeviceToHost, ts.last_stream)))
        return GIVENS_ERR_HIP;
    if (!hip_ok(hipStreamSynchronize(ts.last_stream))) return GIVENS_ERR_HIP;
    float max_abs;
    static_assert(sizeof(max_abs) == sizeof(bits), "");
    __builtin_memcpy(&max_abs, &bits, sizeof(bits));
    switch (form_for_range(max_abs, ts.last_scaled_max)) {
    case kFormScaled: return GIVENS_FORM_SCALED;
    case kFormLifted: return GIVENS_FORM_LIFTED;
    default: return GIVENS_FORM_STANDARD;
    }
}

int givens_set_timing(int on)
{
    std::lock_guard<std::mutex> lock(givens::g_mutex);
    const int prev = givens::g_timing_on;
    givens::g_timing_on = on ? 1 : 0;
    return prev;
}

int givens_last_timing(float ms[4])
{
    using namespace givens;
    if (!ms) return GIVENS_ERR_NULL;
    ThreadState &ts = t_state;
    if (!ts.timing_valid) return GIVENS_ERR_UNSUPPORTED;
    ms[0] = ms[1] = ms[2] = ms[3] = 0.f;
    for (auto &s : ts.spans) {
        if (!hip_ok(hipEventSynchronize(s.stop))) return GIVENS_ERR_HIP;
        float t = 0.f;
        if (!hip_ok(hipEventElapsedTime(&t, s.start, s.stop))) return GIVENS_ERR_HIP;
        if (s.category >= 0 && s.category < 4) ms[s.category] += t;
    }
    return GIVENS_OK;
}

} // extern "C"
