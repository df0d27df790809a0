// C ABI of the round-robin Givens library (see include/givens_rr.h for the contract).
// Host side: argument checks, workspace, kernel selection, launches, optional event timing.
#include <dlfcn.h>
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <mutex>
#include <type_traits>
#include <vector>

#include "../../include/givens_rr.h"
#include "carousel_host.hpp"
#include "coef_kernels.hpp"
#include "lds_kernels.hpp"
#include "rr_index.h"
#include "unitary_kernels.hpp"

namespace givens {
namespace {

constexpr int kMaxDevices = 64;
constexpr size_t kLdsBudgetBytes = 144 * 1024;                 // of the 160 KB per CU on gfx950
constexpr size_t kPartialCapBytes = size_t(24) << 30;          // cap on one chunk of strip partials
constexpr bool kAutoReductionIsAtomic = false;                 // GIVENS_REDUCTION_AUTO never picks the atomic variant

struct Buffer {
    void *ptr = nullptr;
    size_t bytes = 0;
};
struct Workspace {
    Buffer table;        // standard-form cos/sin table, E order
    Buffer table_scaled; // scaled-form (alpha, beta) table, E order
    Buffer scale;        // scaled form: float64 row factors d, [n-1][n]
    Buffer renorm;       // scaled form: renormalisation rows, float2 [periods][n/2]
    Buffer factor;       // per-angle factor of the dtheta reduction
    Buffer flag;         // device word: bit pattern of max |theta|
    Buffer partial;      // per-strip dtheta partial sums (two-stage reduction)
    Buffer acc;          // one accumulation buffer of N floats (accumulating reduction)
    Buffer zeros;        // N floats that are zeroed when allocated and never written again
    Buffer sink;         // N + 8192 floats: where idle lanes of the carousel reverse sweep put their sums
    Buffer gram;         // Gram-matrix reduction: C = Y G^T, n x n floats
    Buffer map;          // restricted parametrisation / odd n: index in theta of every entry of E, or -1
    int map_rows = 0, map_m = 0; // the (row count, m) the map was built for
    Buffer *all[12] = {&table, &table_scaled, &scale, &renorm, &factor, &flag,
                       &partial, &acc, &zeros, &sink, &gram, &map};
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

std::mutex g_mutex;
Workspace g_ws[kMaxDevices];
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
    const unsigned *last_flag = nullptr; // device flag of the last call when several forms were launched
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
    for (auto &s : ts.spans) {
        ts.pool.push_back(s.start);
        ts.pool.push_back(s.stop);
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
        t_state.spans.push_back(rec);
    }
};

int check_n(int n) { return (n < 2 || (n & 1)) ? GIVENS_ERR_BAD_N : GIVENS_OK; }

long long count_free_angles(int rows, int m) { return (long long)m * rows - (long long)m * (m + 1) / 2; }

int check_restricted(int rows, int m)
{
    if (rows < 2 || rows > (1 << 20)) return GIVENS_ERR_BAD_N;
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

// Fills in the padded size and, when some pair of E is bypassed, the device map (built on the host
// once per (rows, m) and kept in the workspace).
int resolve_problem(int dev, int rows, int m, Problem *out)
{
    if (int rc = check_restricted(rows, m)) return rc;
    out->rows = rows;
    out->m = m;
    out->n = rows + (rows & 1);
    out->free_angles = count_free_angles(rows, m);
    out->map = nullptr;
    if (!(rows & 1) && m == rows - 1) return GIVENS_OK;
    Workspace &ws = g_ws[dev];
    if (!(ws.map.ptr && ws.map_rows == rows && ws.map_m == m)) {
        const long long N = (long long)(out->n - 1) * (out->n / 2);
        std::vector<int> host((size_t)N);
        long long next = 0;
        walk_pairs(rows, m, [&](long long e, int, int, bool is_free) { host[(size_t)e] = is_free ? (int)next++ : -1; });
        if (next != out->free_angles) return GIVENS_ERR_UNSUPPORTED;
        ws.map_rows = 0;
        if (int rc = grow(ws.map, (size_t)N * sizeof(int))) return rc;
        GIVENS_HIP(hipMemcpy(ws.map.ptr, host.data(), (size_t)N * sizeof(int), hipMemcpyHostToDevice));
        ws.map_rows = rows;
        ws.map_m = m;
    }
    out->map = reinterpret_cast<const int *>(ws.map.ptr);
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
    const typename Pair2<T>::type *table = nullptr; // standard form
    const T *factor = nullptr;                      // reverse sweep only
    CarouselCoefs standard{kFormStandard, nullptr, nullptr, nullptr, 0.f};
    CarouselCoefs scaled{kFormScaled, nullptr, nullptr, nullptr, 0.f};
    CarouselCoefs lifted{kFormLifted, nullptr, nullptr, nullptr, 0.f};
    bool all_forms = false;                         // scaled- and lifted-form kernels were launched too
};

// What the process-wide form setting means for a call on the float carousel path: whether the range
// check and the scaled / lifted tables are wanted, and the threshold of the scaled form.
struct FormPolicy {
    bool try_forms;
    float scaled_max;
};
FormPolicy form_policy(bool float_carousel)
{
    if (!float_carousel || g_form_choice == GIVENS_FORM_STANDARD) return {false, 0.f};
    if (g_form_choice == GIVENS_FORM_LIFTED) return {true, -1.f};
    return {true, kScaledMaxAbsTheta};
}

// Where the coefficient kernels of one call write: either the per-device workspace (grown on demand) or
// the static scratch array of the entry point that may not allocate.
template <typename T>
struct CoefStorage {
    typename Pair2<T>::type *table = nullptr; // standard form, N pairs
    T *factor = nullptr;                      // reverse sweep only, N values
    unsigned *flag = nullptr;                 // float carousel path only, as are the following
    float2 *table_scaled = nullptr;           // N pairs
    double *scale = nullptr;                  // (n-1) * n row factors
    float *renorm = nullptr;                  // periods * n/2 pairs
};

inline int renorm_periods(int n) { return (n - 1 + kRenormPeriod - 1) / kRenormPeriod; }

template <typename T>
int workspace_coef_storage(int dev, int n, bool forward, bool try_forms, CoefStorage<T> *out)
{
    using P2 = typename Pair2<T>::type;
    const long long N = (long long)n * (n - 1) / 2;
    Workspace &ws = g_ws[dev];
    if (int rc = grow(ws.table, (size_t)N * sizeof(P2))) return rc;
    out->table = reinterpret_cast<P2 *>(ws.table.ptr);
    if (!forward) {
        if (int rc = grow(ws.factor, (size_t)N * sizeof(T))) return rc;
        out->factor = reinterpret_cast<T *>(ws.factor.ptr);
    }
    if (try_forms) {
        if (int rc = grow(ws.flag, 256)) return rc;
        if (int rc = grow(ws.table_scaled, (size_t)N * sizeof(float2))) return rc;
        if (int rc = grow(ws.scale, (size_t)(n - 1) * n * sizeof(double))) return rc;
        if (int rc = grow(ws.renorm, (size_t)renorm_periods(n) * (n / 2) * sizeof(float2))) return rc;
        out->flag = reinterpret_cast<unsigned *>(ws.flag.ptr);
        out->table_scaled = reinterpret_cast<float2 *>(ws.table_scaled.ptr);
        out->scale = reinterpret_cast<double *>(ws.scale.ptr);
        out->renorm = reinterpret_cast<float *>(ws.renorm.ptr);
    }
    return GIVENS_OK;
}

// ---- the entry point that allocates nothing: its coefficient tables live in a static device array.
constexpr int kNoAllocMaxN = GIVENS_NOALLOC_MAX_N;
constexpr size_t round_up_256(size_t v) { return (v + 255) / 256 * 256; }
constexpr size_t noalloc_bytes(int n)
{
    const size_t N = (size_t)n * (n - 1) / 2;
    return round_up_256(N * sizeof(float2)) * 2                                            // both tables
           + round_up_256((size_t)(n - 1) * n * sizeof(double))                            // row factors
           + round_up_256((size_t)((n - 1 + kRenormPeriod - 1) / kRenormPeriod) * (n / 2) * sizeof(float2))
           + 256;                                                                          // flag word
}
constexpr size_t kNoAllocBytes = noalloc_bytes(kNoAllocMaxN);
static_assert(kNoAllocBytes == GIVENS_NOALLOC_BYTES, "the header states the size of the static array");
static __device__ __align__(256) unsigned char scratch[kNoAllocBytes];
// Address of `scratch` on each device (every GPU holds its own copy of the array): looked up once per
// device with that device current.  Host code uses these pointers, never the array's name.
unsigned char *g_scratch_ptr[kMaxDevices] = {};

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
    out->table = reinterpret_cast<float2 *>(take(N * sizeof(float2)));
    out->table_scaled = reinterpret_cast<float2 *>(take(N * sizeof(float2)));
    out->scale = reinterpret_cast<double *>(take((size_t)(n - 1) * n * sizeof(double)));
    out->renorm = reinterpret_cast<float *>(take((size_t)renorm_periods(n) * (n / 2) * sizeof(float2)));
    out->flag = reinterpret_cast<unsigned *>(take(256));
    out->factor = nullptr;
    return (size_t)(at - g_scratch_ptr[dev]) <= kNoAllocBytes ? GIVENS_OK : GIVENS_ERR_UNSUPPORTED;
}

// Launches the coefficient kernels.  `forward` picks the sweep direction of the scaled / lifted
// forms' row factors; `policy.try_forms` adds the range check and those forms' tables.
template <typename T>
int prepare_coefs(const CoefStorage<T> &st, const Problem &pb, const T *theta, bool forward, FormPolicy policy,
                  hipStream_t stream, Coefs<T> *out, int mirror = 0)
{
    const bool try_scaled = policy.try_forms;
    const float scaled_max = policy.scaled_max;
    using P2 = typename Pair2<T>::type;
    const int n = pb.n;
    const int *map = pb.map;
    const long long N = (long long)n * (n - 1) / 2;
    P2 *table = st.table;
    T *factor = forward ? nullptr : st.factor;
    unsigned *flag = nullptr;
    const int threads = 256;
    const unsigned blocks = (unsigned)((N + threads - 1) / threads);
    Span span(0, stream);
    if constexpr (std::is_same<T, float>::value) {
        if (try_scaled) {
            const int periods = renorm_periods(n);
            flag = st.flag;
            float2 *tab_s = st.table_scaled;
            double *D = st.scale;
            float *rn = st.renorm;
            hipLaunchKernelGGL(reset_flag_kernel, dim3(1), dim3(1), 0, stream, flag);
            hipLaunchKernelGGL(theta_range_kernel, dim3(512), dim3(512), 0, stream, pb.free_angles, theta, flag);
            const long long scan_threads = (long long)periods * n;
            const unsigned scan_blocks = (unsigned)((scan_threads + threads - 1) / threads);
            if (forward) {
                hipLaunchKernelGGL(scaled_scan_kernel<true>, dim3(scan_blocks), dim3(threads), 0, stream, n, theta,
                                   map, mirror, flag, scaled_max, D, rn);
                hipLaunchKernelGGL(scaled_table_kernel<true>, dim3(blocks), dim3(threads), 0, stream, n, theta,
                                   map, mirror, flag, scaled_max, D, tab_s, factor);
            } else {
                hipLaunchKernelGGL(scaled_scan_kernel<false>, dim3(scan_blocks), dim3(threads), 0, stream, n, theta,
                                   map, mirror, flag, scaled_max, D, rn);
                hipLaunchKernelGGL(scaled_table_kernel<false>, dim3(blocks), dim3(threads), 0, stream, n, theta,
                                   map, mirror, flag, scaled_max, D, tab_s, factor);
            }
            out->scaled = CarouselCoefs{kFormScaled, tab_s, reinterpret_cast<const float2 *>(rn), flag, scaled_max};
            out->lifted = CarouselCoefs{kFormLifted, tab_s, reinterpret_cast<const float2 *>(rn), flag, scaled_max};
            out->all_forms = true;
        }
        out->standard = CarouselCoefs{kFormStandard, table, nullptr, flag, scaled_max};
    }
    hipLaunchKernelGGL(coef_table_kernel<T>, dim3(std::min(blocks, 4096u)), dim3(threads), 0, stream, n, theta,
                       map, mirror, static_cast<const unsigned *>(flag), scaled_max, table, factor);
    GIVENS_HIP(hipGetLastError());
    out->table = table;
    out->factor = factor;
    t_state.last_flag = flag;
    t_state.last_scaled_max = scaled_max;
    t_state.last_stream = stream;
    return GIVENS_OK;
}

// the usual case: storage from the per-device workspace
template <typename T>
int prepare_coefs(int dev, const Problem &pb, const T *theta, bool forward, FormPolicy policy, hipStream_t stream,
                  Coefs<T> *out, int mirror = 0)
{
    CoefStorage<T> st;
    if (int rc = workspace_coef_storage<T>(dev, pb.n, forward,
                                           policy.try_forms && std::is_same<T, float>::value, &st))
        return rc;
    return prepare_coefs<T>(st, pb, theta, forward, policy, stream, out, mirror);
}

template <typename T>
int lds_forward(int n, int rows, long long B, const typename Pair2<T>::type *table, const T *X, T *Y,
                int identity, hipStream_t stream, int mirror = 0)
{
    const int w = lds_strip_width<T>(n, B, 1);
    if (w == 0) return GIVENS_ERR_UNSUPPORTED;
    const size_t smem = (size_t)n * lds_row_stride(w) * sizeof(T);
    auto kern = lds_forward_kernel<T>;
    GIVENS_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    const long long strips = (B + w - 1) / w;
    Span span(1, stream);
    hipLaunchKernelGGL(kern, dim3((unsigned)strips), dim3(kLdsThreads), smem, stream, n, rows, B, w, table, X,
                       Y, identity, mirror);
    GIVENS_HIP(hipGetLastError());
    return GIVENS_OK;
}

// Reverse sweep and the reduction of its partial sums into dtheta.  LDS family: chunks of strips, one
// partial sum per (strip, angle), folded into dtheta chunk by chunk.  Carousel family: persistent
// workgroups with one row of partial sums each, or the accumulating variant.  `family` picks the kernel.
template <typename T>
int backward_chunks(int dev, int family, const Problem &pb, long long B, const Coefs<T> &coefs, const T *Y,
                    const T *G, T *dX, T *dtheta, hipStream_t stream, int g_identity = 0)
{
    const int n = pb.n, rows = pb.rows;
    const int *map = pb.map;
    const long long N = (long long)n * (n - 1) / 2;
    int w = 0;
    size_t smem = 0;
    auto kern = lds_backward_kernel<T>;
    if (family == GIVENS_KERNEL_LDS) {
        w = lds_strip_width<T>(n, B, 2);
        if (w == 0) return GIVENS_ERR_UNSUPPORTED;
        smem = (size_t)2 * n * lds_row_stride(w) * sizeof(T);
        GIVENS_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    } else {
        w = carousel_bwd_width(n, B);
        if (w == 0) return GIVENS_ERR_UNSUPPORTED;
    }
    const long long strips = (B + w - 1) / w;
    Workspace &ws = g_ws[dev];
    int cus = 0;
    GIVENS_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    const float *zeros = nullptr;
    float *sink = nullptr;
    if constexpr (std::is_same<T, float>::value) {
        if (family == GIVENS_KERNEL_CAROUSEL) {
            const size_t want = (size_t)N * sizeof(float);
            if (ws.zeros.bytes < want) {
                if (int rc = grow(ws.zeros, want)) return rc;
                hipLaunchKernelGGL(fill_zero_kernel, dim3(2048), dim3(256), 0, stream, N,
                                   reinterpret_cast<float *>(ws.zeros.ptr));
                GIVENS_HIP(hipGetLastError());
                // later calls may come on other streams and never write this buffer again
                GIVENS_HIP(hipStreamSynchronize(stream));
            }
            zeros = reinterpret_cast<const float *>(ws.zeros.ptr);
            if (int rc = grow(ws.sink, ((size_t)N + 8192) * sizeof(float))) return rc;
            sink = reinterpret_cast<float *>(ws.sink.ptr);
        }
    }

    if constexpr (std::is_same<T, float>::value) {
        // accumulating reduction (carousel family): every strip adds its sums into one zeroed buffer
        // with float atomics; no per-strip partials, no second pass over them
        const bool want_acc = g_reduction_choice == GIVENS_REDUCTION_ATOMIC ||
                              (g_reduction_choice == GIVENS_REDUCTION_AUTO && kAutoReductionIsAtomic);
        if (family == GIVENS_KERNEL_CAROUSEL && want_acc) {
            int lanes = 0, slots = 0;
            if (!carousel_bwd_layout(n, &lanes, &slots)) return GIVENS_ERR_UNSUPPORTED;
            if (int rc = grow(ws.acc, (size_t)N * sizeof(float))) return rc;
            float *acc = reinterpret_cast<float *>(ws.acc.ptr);
            const int threads = 256;
            {
                Span span(1, stream);
                hipLaunchKernelGGL(fill_zero_kernel, dim3(2048), dim3(threads), 0, stream, N, acc);
                const long long groups = carousel_bwd_groups(n, strips, cus);
                if (coefs.all_forms) {
                    if (int rc = carousel_backward_strips(n, rows, B, w, 0, strips, groups, coefs.scaled, Y, G, dX,
                                                          acc, zeros, sink, 1, g_identity, stream))
                        return rc;
                    if (int rc = carousel_backward_strips(n, rows, B, w, 0, strips, groups, coefs.lifted, Y, G, dX,
                                                          acc, zeros, sink, 1, g_identity, stream))
                        return rc;
                }
                if (int rc = carousel_backward_strips(n, rows, B, w, 0, strips, groups, coefs.standard, Y, G, dX,
                                                      acc, zeros, sink, 1, g_identity, stream))
                    return rc;
                GIVENS_HIP(hipGetLastError());
            }
            {
                Span span(2, stream);
                hipLaunchKernelGGL(finish_accumulated_kernel, dim3((unsigned)((N + threads - 1) / threads)),
                                   dim3(threads), 0, stream, n, lanes, slots, acc, coefs.factor, map, dtheta);
                GIVENS_HIP(hipGetLastError());
            }
            t_state.last_reduction = GIVENS_REDUCTION_ATOMIC;
            return GIVENS_OK;
        }
    }
    t_state.last_reduction = GIVENS_REDUCTION_TWO_STAGE;

    // Two-stage reduction.  LDS family: one row of partial sums per strip, in chunks of strips that fit
    // the workspace cap.  Carousel family: one row per persistent workgroup (at most what the chip
    // holds at once), whatever the number of strips.
    const bool persistent = family == GIVENS_KERNEL_CAROUSEL;
    const long long rows_wanted = persistent ? carousel_bwd_groups(n, strips, cus) : strips;
    long long prows = (long long)(kPartialCapBytes / ((size_t)N * sizeof(T)));
    prows = std::max<long long>(1, std::min(prows, rows_wanted));
    if (int rc = grow(ws.partial, (size_t)prows * N * sizeof(T))) return rc;
    T *partial = reinterpret_cast<T *>(ws.partial.ptr);
    const long long chunk = persistent ? strips : prows;     // strips per launch
    for (long long s0 = 0; s0 < strips; s0 += chunk) {
        const long long ns = std::min(chunk, strips - s0);
        const long long nrows = persistent ? std::min(prows, ns) : ns;
        {
            Span span(1, stream);
            if (family == GIVENS_KERNEL_LDS) {
                hipLaunchKernelGGL(kern, dim3((unsigned)ns), dim3(kLdsThreads), smem, stream, n, rows, B, w, s0,
                                   coefs.table, Y, G, dX, partial, g_identity);
            } else if constexpr (std::is_same<T, float>::value) {
                if (coefs.all_forms) {
                    if (int rc = carousel_backward_strips(n, rows, B, w, s0, ns, nrows, coefs.scaled, Y, G, dX,
                                                          partial, zeros, sink, 0, g_identity, stream))
                        return rc;
                    if (int rc = carousel_backward_strips(n, rows, B, w, s0, ns, nrows, coefs.lifted, Y, G, dX,
                                                          partial, zeros, sink, 0, g_identity, stream))
                        return rc;
                }
                if (int rc = carousel_backward_strips(n, rows, B, w, s0, ns, nrows, coefs.standard, Y, G, dX,
                                                      partial, zeros, sink, 0, g_identity, stream))
                    return rc;
            } else {
                return GIVENS_ERR_UNSUPPORTED;
            }
            GIVENS_HIP(hipGetLastError());
        }
        {
            Span span(2, stream);
            const int threads = 256;
            hipLaunchKernelGGL(reduce_partials_kernel<T>, dim3((unsigned)((N + threads - 1) / threads)),
                               dim3(threads), 0, stream, n, nrows, partial, coefs.factor, map, dtheta,
                               s0 > 0 ? 1 : 0);
            GIVENS_HIP(hipGetLastError());
        }
    }
    return GIVENS_OK;
}

// ---- rocBLAS, loaded on first use: only the Gram-matrix reduction needs it (one plain SGEMM), and the
// library must load and run without it.
struct RocblasApi {
    bool tried = false, ok = false;
    void *lib = nullptr;
    int (*create_handle)(void **) = nullptr;
    int (*destroy_handle)(void *) = nullptr;
    int (*set_stream)(void *, hipStream_t) = nullptr;
    int (*set_atomics_mode)(void *, int) = nullptr;
    int (*sgemm)(void *, int, int, int, int, int, const float *, const float *, int, const float *, int,
                 const float *, float *, int) = nullptr;
    int (*sgemm_strided_batched)(void *, int, int, int, int, int, const float *, const float *, int, long long,
                                 const float *, int, long long, const float *, float *, int, long long,
                                 int) = nullptr;
    void *handle[kMaxDevices] = {};
};
RocblasApi g_blas;
constexpr int kBlasOpNone = 111, kBlasOpTranspose = 112; // rocblas_operation values of the public API

bool rocblas_available()
{
    RocblasApi &b = g_blas;
    if (b.tried) return b.ok;
    b.tried = true;
    for (const char *name : {"librocblas.so.5", "librocblas.so", "/opt/rocm/lib/librocblas.so"}) {
        b.lib = dlopen(name, RTLD_NOW | RTLD_LOCAL);
        if (b.lib) break;
    }
    if (!b.lib) return false;
    b.create_handle = reinterpret_cast<decltype(b.create_handle)>(dlsym(b.lib, "rocblas_create_handle"));
    b.destroy_handle = reinterpret_cast<decltype(b.destroy_handle)>(dlsym(b.lib, "rocblas_destroy_handle"));
    b.set_stream = reinterpret_cast<decltype(b.set_stream)>(dlsym(b.lib, "rocblas_set_stream"));
    b.set_atomics_mode = reinterpret_cast<decltype(b.set_atomics_mode)>(dlsym(b.lib, "rocblas_set_atomics_mode"));
    b.sgemm = reinterpret_cast<decltype(b.sgemm)>(dlsym(b.lib, "rocblas_sgemm"));
    b.sgemm_strided_batched = reinterpret_cast<decltype(b.sgemm_strided_batched)>(
        dlsym(b.lib, "rocblas_sgemm_strided_batched"));
    b.ok = b.create_handle && b.destroy_handle && b.set_stream && b.set_atomics_mode && b.sgemm &&
           b.sgemm_strided_batched;
    return b.ok;
}

// How many slices of the contraction (batch) dimension the Gram matrix is computed in.  The library's
// SGEMM gives a 256 x 256 tile of C to one workgroup, so a 2048 x 2048 result alone would occupy 64
// of the 256 CUs; slicing B and summing the slices' results afterwards (fixed order) fills the chip.
int gram_slices(int rows, long long B)
{
    const long long tiles = (long long)((rows + 255) / 256) * ((rows + 255) / 256);
    long long s = (256 + tiles - 1) / tiles;
    s = std::min<long long>(s, 16);
    s = std::min<long long>(s, std::max<long long>(1, B / 1024));
    return (int)std::max<long long>(1, s);
}

__global__ void sum_slices_kernel(long long count, int slices, float *__restrict__ c)
{
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < count;
         i += (long long)gridDim.x * blockDim.x) {
        float acc = c[i];
        for (int s = 1; s < slices; ++s) acc += c[(long long)s * count + i];
        c[i] = acc;
    }
}

// C (rows x rows, row-major) = Y G^T for row-major rows x B operands: in the library's column-major
// terms C^T = G_cm^T Y_cm with G_cm, Y_cm the B x rows column-major views of the same memory.
// C has room for `slices` matrices; the result ends in the first.
int gram_matrix(int dev, int rows, long long B, int slices, const float *Y, const float *G, float *C,
                hipStream_t stream)
{
    RocblasApi &b = g_blas;
    if (!rocblas_available() || B > 0x7fffffffLL) return GIVENS_ERR_UNSUPPORTED;
    if (!b.handle[dev]) {
        if (b.create_handle(&b.handle[dev]) != 0) { b.handle[dev] = nullptr; return GIVENS_ERR_UNSUPPORTED; }
        (void)b.set_atomics_mode(b.handle[dev], 0); // no atomics: bit-identical results from run to run
    }
    if (b.set_stream(b.handle[dev], stream) != 0) return GIVENS_ERR_UNSUPPORTED;
    const float one = 1.f, zero = 0.f;
    const long long count = (long long)rows * rows;
    const long long kc = B / slices;            // columns per slice; the remainder goes to a last GEMM
    int st;
    if (slices > 1)
        st = b.sgemm_strided_batched(b.handle[dev], kBlasOpTranspose, kBlasOpNone, rows, rows, (int)kc, &one, G,
                                     (int)B, kc, Y, (int)B, kc, &zero, C, rows, count, slices);
    else
        st = b.sgemm(b.handle[dev], kBlasOpTranspose, kBlasOpNone, rows, rows, (int)kc, &one, G, (int)B, Y, (int)B,
                     &zero, C, rows);
    if (st != 0) return GIVENS_ERR_UNSUPPORTED;
    const long long tail = B - kc * slices;
    if (tail > 0) {
        st = b.sgemm(b.handle[dev], kBlasOpTranspose, kBlasOpNone, rows, rows, (int)tail, &one, G + kc * slices,
                     (int)B, Y + kc * slices, (int)B, &one, C, rows);
        if (st != 0) return GIVENS_ERR_UNSUPPORTED;
    }
    if (slices > 1) {
        hipLaunchKernelGGL(sum_slices_kernel, dim3(1024), dim3(256), 0, stream, count, slices, C);
        GIVENS_HIP(hipGetLastError());
    }
    return GIVENS_OK;
}

int current_device(int *dev)
{
    GIVENS_HIP(hipGetDevice(dev));
    if (*dev < 0 || *dev >= kMaxDevices) return GIVENS_ERR_UNSUPPORTED;
    return GIVENS_OK;
}

// rows, m: see Problem.  The unrestricted entry points pass an even rows and m = rows - 1.
template <typename T>
int forward_impl(int rows, int m, long long B, const T *theta, const T *X, T *Y, int identity, void *stream_v,
                 int transpose = 0, bool no_alloc = false)
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
    Problem pb;
    if (int rc = resolve_problem(dev, rows, m, &pb)) return rc;
    const int n = pb.n;
    timing_begin_call();
    if (no_alloc) t_state.timing_valid = false; // event pairs are created on demand: not here
    const int choice = g_kernel_choice;
    const bool can_carousel = carousel_supported<T>(n, B);
    const bool can_column = std::is_same<T, float>::value && n <= kColumnFamilyMaxN;
    if (choice == GIVENS_KERNEL_CAROUSEL && !can_carousel) return GIVENS_ERR_UNSUPPORTED;
    if (choice == GIVENS_KERNEL_COLUMN && !can_column) return GIVENS_ERR_UNSUPPORTED;
    const bool use_carousel = can_carousel && (choice == GIVENS_KERNEL_AUTO || choice == GIVENS_KERNEL_CAROUSEL);
    const bool use_column = can_column && (choice == GIVENS_KERNEL_AUTO || choice == GIVENS_KERNEL_COLUMN);
    Coefs<T> coefs;
    const FormPolicy policy = form_policy(use_carousel && std::is_same<T, float>::value);
    if (no_alloc) {
        if constexpr (std::is_same<T, float>::value) {
            CoefStorage<float> st;
            if (int rc = static_coef_storage(dev, n, &st)) return rc;
            if (int rc = prepare_coefs<float>(st, pb, theta, true, policy, stream, &coefs, transpose)) return rc;
        }
    } else if (int rc = prepare_coefs<T>(dev, pb, theta, true, policy, stream, &coefs, transpose)) {
        return rc;
    }
    int rc = GIVENS_OK;
    if (use_carousel) {
        if constexpr (std::is_same<T, float>::value) {
            Span span(1, stream);
            if (coefs.all_forms) {
                rc = carousel_forward(n, rows, B, coefs.scaled, X, Y, identity, transpose, stream);
                if (rc == GIVENS_OK) rc = carousel_forward(n, rows, B, coefs.lifted, X, Y, identity, transpose, stream);
            }
            if (rc == GIVENS_OK) rc = carousel_forward(n, rows, B, coefs.standard, X, Y, identity, transpose, stream);
            if (rc == GIVENS_OK && !hip_ok(hipGetLastError())) rc = GIVENS_ERR_HIP;
        } else {
            rc = GIVENS_ERR_UNSUPPORTED;
        }
        t_state.last_kernel = GIVENS_KERNEL_CAROUSEL;
    } else if (use_column) {
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

template <typename T>
int backward_impl(int rows, int m, long long B, const T *theta, const T *Y, const T *G, T *dX, T *dtheta,
                  void *stream_v)
{
    if (int rc = check_restricted(rows, m)) return rc;
    if (B < 1) return GIVENS_ERR_BAD_B;
    if (!theta || !Y || !G || !dtheta) return GIVENS_ERR_NULL;
    if (dX && (const void *)dX == (const void *)Y) return GIVENS_ERR_ALIAS;
    hipStream_t stream = reinterpret_cast<hipStream_t>(stream_v);
    std::lock_guard<std::mutex> lock(g_mutex);
    int dev = 0;
    if (int rc = current_device(&dev)) return rc;
    Problem pb;
    if (int rc = resolve_problem(dev, rows, m, &pb)) return rc;
    const int n = pb.n;
    timing_begin_call();
    const int choice = g_kernel_choice;
    const bool can_carousel = carousel_backward_supported<T>(n, B);
    const bool can_column = std::is_same<T, float>::value && n <= kColumnFamilyMaxN;
    if (choice == GIVENS_KERNEL_CAROUSEL && !can_carousel) return GIVENS_ERR_UNSUPPORTED;
    if (choice == GIVENS_KERNEL_COLUMN && !can_column) return GIVENS_ERR_UNSUPPORTED;
    // the family that sweeps (the n x n operand of the Gram form, or all B columns); the column family has
    // no reverse sweep of its own and borrows the LDS family's
    const int family = (can_carousel && (choice == GIVENS_KERNEL_AUTO || choice == GIVENS_KERNEL_CAROUSEL))
                           ? GIVENS_KERNEL_CAROUSEL
                           : GIVENS_KERNEL_LDS;
    const bool column = can_column && (choice == GIVENS_KERNEL_AUTO || choice == GIVENS_KERNEL_COLUMN);
    Coefs<T> coefs;
    if (int rc = prepare_coefs<T>(dev, pb, theta, false,
                                  form_policy(family == GIVENS_KERNEL_CAROUSEL && std::is_same<T, float>::value),
                                  stream, &coefs))
        return rc;
    t_state.last_kernel = family;
    if constexpr (std::is_same<T, float>::value) {
        // Gram-matrix form for wide batches.  With C = Y G^T (rows x rows) the sums of the reverse sweep
        // are those of the same sweep run on the operand C with the identity as upstream gradient:
        // z_k gbar_k^T = A_k C A_k^T for the product A_k of the transposed blocks so far, and the sweep on
        // (C, I) carries A_k C and A_k.  So dtheta costs one GEMM over B plus a rows-column sweep, and
        // dX = U^T G one forward-type sweep over B (mirrored tables), instead of a two-strip sweep over B.
        const bool wide = B >= 2LL * n;   // measured break-even is near B = 1.6 n
        const bool want_gram = (g_reduction_choice == GIVENS_REDUCTION_GRAM ||
                                (g_reduction_choice == GIVENS_REDUCTION_AUTO && wide));
        if (want_gram && rocblas_available()) {
            Workspace &ws = g_ws[dev];
            const int slices = gram_slices(rows, B);
            if (int rc = grow(ws.gram, (size_t)slices * rows * rows * sizeof(float))) return rc;
            float *C = reinterpret_cast<float *>(ws.gram.ptr);
            int rc;
            {
                Span span(1, stream);
                rc = gram_matrix(dev, rows, B, slices, Y, G, C, stream);
            }
            if (rc == GIVENS_OK) {
                rc = backward_chunks<T>(dev, family, pb, rows, coefs, C, nullptr, nullptr, dtheta, stream, 1);
                if (rc == GIVENS_OK && dX && column) {
                    Coefs<T> mirrored;
                    rc = prepare_coefs<T>(dev, pb, theta, true, form_policy(false), stream, &mirrored, 1);
                    Span span(1, stream);
                    if (rc == GIVENS_OK) rc = column_forward(n, rows, B, mirrored.table, G, dX, 0, 1, stream);
                    if (rc == GIVENS_OK && !hip_ok(hipGetLastError())) rc = GIVENS_ERR_HIP;
                } else if (rc == GIVENS_OK && dX && family == GIVENS_KERNEL_LDS) {
                    Coefs<T> mirrored;
                    rc = prepare_coefs<T>(dev, pb, theta, true, form_policy(false), stream, &mirrored, 1);
                    if (rc == GIVENS_OK) rc = lds_forward<T>(n, rows, B, mirrored.table, G, dX, 0, stream, 1);
                } else if (rc == GIVENS_OK && dX) {
                    Coefs<T> mirrored;
                    rc = prepare_coefs<T>(dev, pb, theta, true, form_policy(true), stream, &mirrored, 1);
                    Span span(1, stream);
                    if (rc == GIVENS_OK && mirrored.all_forms) {
                        rc = carousel_forward(n, rows, B, mirrored.scaled, G, dX, 0, 1, stream);
                        if (rc == GIVENS_OK) rc = carousel_forward(n, rows, B, mirrored.lifted, G, dX, 0, 1, stream);
                    }
                    if (rc == GIVENS_OK) rc = carousel_forward(n, rows, B, mirrored.standard, G, dX, 0, 1, stream);
                    if (rc == GIVENS_OK && !hip_ok(hipGetLastError())) rc = GIVENS_ERR_HIP;
                }
                t_state.last_reduction = GIVENS_REDUCTION_GRAM;
                if (column) t_state.last_kernel = GIVENS_KERNEL_COLUMN;
                return rc;
            }
            // the GEMM could not be run: fall through to the sweep over all B columns
        } else if (g_reduction_choice == GIVENS_REDUCTION_GRAM) {
            return GIVENS_ERR_UNSUPPORTED; // forced, but rocBLAS could not be loaded
        }
    }
    return backward_chunks<T>(dev, family, pb, B, coefs, Y, G, dX, dtheta, stream);
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
int unitary_table(int dev, int n, const T *theta, const T *phi, hipStream_t stream,
                  const typename Cplx<T>::quad **out)
{
    const long long N = (long long)n * (n - 1) / 2;
    Workspace &ws = g_ws[dev];
    if (int rc = grow(ws.table, (size_t)N * sizeof(typename Cplx<T>::quad))) return rc;
    auto *table = reinterpret_cast<typename Cplx<T>::quad *>(ws.table.ptr);
    Span span(0, stream);
    const int threads = 256;
    const unsigned blocks = (unsigned)std::min<long long>((N + threads - 1) / threads, 4096);
    hipLaunchKernelGGL(unitary_table_kernel<T>, dim3(blocks), dim3(threads), 0, stream, n, theta, phi, table);
    GIVENS_HIP(hipGetLastError());
    *out = table;
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
    const int w = unitary_strip_width<T>(n, B, 1);
    if (w == 0) return GIVENS_ERR_UNSUPPORTED;
    const typename Cplx<T>::quad *table = nullptr;
    if (int rc = unitary_table<T>(dev, n, theta, phi, stream, &table)) return rc;
    const size_t smem = (size_t)n * w * sizeof(C);
    auto kern = unitary_forward_kernel<T>;
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
    const int w = unitary_strip_width<T>(n, B, 2);
    if (w == 0) return GIVENS_ERR_UNSUPPORTED;
    const typename Cplx<T>::quad *table = nullptr;
    if (int rc = unitary_table<T>(dev, n, theta, phi, stream, &table)) return rc;
    const long long N = (long long)n * (n - 1) / 2;
    const long long strips = (B + w - 1) / w;
    long long rows = (long long)(kPartialCapBytes / ((size_t)2 * N * sizeof(T)));
    rows = std::max<long long>(1, std::min(rows, strips));
    Workspace &ws = g_ws[dev];
    if (int rc = grow(ws.partial, (size_t)rows * 2 * N * sizeof(T))) return rc;
    T *partial = reinterpret_cast<T *>(ws.partial.ptr);
    const size_t smem = (size_t)2 * n * w * sizeof(C);
    auto kern = unitary_backward_kernel<T>;
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
    return givens::forward_impl<float>(n, n - 1, B, theta, X, Y, 0, stream);
}
int givens_build(int n, const float *theta, float *U, void *stream)
{
    if (int rc = givens::check_n(n)) return rc;
    return givens::forward_impl<float>(n, n - 1, n, theta, nullptr, U, 1, stream);
}
int givens_backward(int n, int64_t B, const float *theta, const float *Y, const float *G, float *dX,
                    float *dtheta, void *stream)
{
    if (int rc = givens::check_n(n)) return rc;
    return givens::backward_impl<float>(n, n - 1, B, theta, Y, G, dX, dtheta, stream);
}
int givens_forward_f64(int n, int64_t B, const double *theta, const double *X, double *Y, void *stream)
{
    if (int rc = givens::check_n(n)) return rc;
    return givens::forward_impl<double>(n, n - 1, B, theta, X, Y, 0, stream);
}
int givens_build_f64(int n, const double *theta, double *U, void *stream)
{
    if (int rc = givens::check_n(n)) return rc;
    return givens::forward_impl<double>(n, n - 1, n, theta, nullptr, U, 1, stream);
}
int givens_backward_f64(int n, int64_t B, const double *theta, const double *Y, const double *G,
                        double *dX, double *dtheta, void *stream)
{
    if (int rc = givens::check_n(n)) return rc;
    return givens::backward_impl<double>(n, n - 1, B, theta, Y, G, dX, dtheta, stream);
}

int givens_forward_transposed(int n, int64_t B, const float *theta, const float *X, float *Y, void *stream)
{
    if (int rc = givens::check_n(n)) return rc;
    return givens::forward_impl<float>(n, n - 1, B, theta, X, Y, 0, stream, 1);
}
int givens_forward_transposed_f64(int n, int64_t B, const double *theta, const double *X, double *Y, void *stream)
{
    if (int rc = givens::check_n(n)) return rc;
    return givens::forward_impl<double>(n, n - 1, B, theta, X, Y, 0, stream, 1);
}

int givens_forward_noalloc(int n, int64_t B, const float *theta, const float *X, float *Y, void *stream)
{
    if (int rc = givens::check_n(n)) return rc;
    return givens::forward_impl<float>(n, n - 1, B, theta, X, Y, 0, stream, 0, true);
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
    return givens::forward_impl<float>(n, m, B, theta, X, Y, 0, stream);
}
int givens_build_restricted(int n, int m, const float *theta, float *U, void *stream)
{
    return givens::forward_impl<float>(n, m, n, theta, nullptr, U, 1, stream);
}
int givens_backward_restricted(int n, int m, int64_t B, const float *theta, const float *Y, const float *G,
                               float *dX, float *dtheta, void *stream)
{
    return givens::backward_impl<float>(n, m, B, theta, Y, G, dX, dtheta, stream);
}
int givens_forward_restricted_f64(int n, int m, int64_t B, const double *theta, const double *X, double *Y,
                                  void *stream)
{
    return givens::forward_impl<double>(n, m, B, theta, X, Y, 0, stream);
}
int givens_build_restricted_f64(int n, int m, const double *theta, double *U, void *stream)
{
    return givens::forward_impl<double>(n, m, n, theta, nullptr, U, 1, stream);
}
int givens_backward_restricted_f64(int n, int m, int64_t B, const double *theta, const double *Y, const double *G,
                                   double *dX, double *dtheta, void *stream)
{
    return givens::backward_impl<double>(n, m, B, theta, Y, G, dX, dtheta, stream);
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
        Workspace &ws = g_ws[d];
        bool any = false;
        for (Buffer *b : ws.all) any = any || b->ptr;
        if (!any) continue;
        if (!hip_ok(hipSetDevice(d))) { rc = GIVENS_ERR_HIP; continue; }
        for (Buffer *b : ws.all) {
            if (b->ptr && !hip_ok(hipFree(b->ptr))) rc = GIVENS_ERR_HIP;
            *b = Buffer{};
        }
        ws.map_rows = ws.map_m = 0;
        if (g_blas.handle[d]) {
            (void)g_blas.destroy_handle(g_blas.handle[d]);
            g_blas.handle[d] = nullptr;
        }
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
    if (which != GIVENS_REDUCTION_AUTO && which != GIVENS_REDUCTION_TWO_STAGE && which != GIVENS_REDUCTION_ATOMIC &&
        which != GIVENS_REDUCTION_GRAM)
        return GIVENS_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(givens::g_mutex);
    const int prev = givens::g_reduction_choice;
    givens::g_reduction_choice = which;
    return prev;
}

int givens_last_reduction(void) { return givens::t_state.last_reduction; }

int givens_set_rotation_form(int which)
{
    if (which != GIVENS_FORM_AUTO && which != GIVENS_FORM_STANDARD && which != GIVENS_FORM_LIFTED)
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

int givens_last_timing(float ms[3])
{
    using namespace givens;
    if (!ms) return GIVENS_ERR_NULL;
    ThreadState &ts = t_state;
    if (!ts.timing_valid) return GIVENS_ERR_UNSUPPORTED;
    ms[0] = ms[1] = ms[2] = 0.f;
    for (auto &s : ts.spans) {
        if (!hip_ok(hipEventSynchronize(s.stop))) return GIVENS_ERR_HIP;
        float t = 0.f;
        if (!hip_ok(hipEventElapsedTime(&t, s.start, s.stop))) return GIVENS_ERR_HIP;
        if (s.category >= 0 && s.category < 3) ms[s.category] += t;
    }
    return GIVENS_OK;
}

} // extern "C"
