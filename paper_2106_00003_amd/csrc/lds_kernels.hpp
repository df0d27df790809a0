// LDS strip kernels: the general-shape family (any even n whose strip fits in LDS, float or
// double).  One workgroup owns w columns of the operand, keeps the n x w strip in LDS for all
// n-1 blocks of Algorithm 2, and touches HBM once on the way in and once on the way out.
// Inside a block each thread owns whole pairs (arcs) and walks the strip's columns, so the
// per-pair gradient sum of the reverse sweep needs no cross-thread reduction.
//
// cos/sin come from the standard-form table of coef_kernels.hpp (orientation folded into the sine).
// `rows` is the operand's row count: n itself, or n - 1 when n is the padded size of an odd problem
// (end of Section 3: the added dimension is inactive; its row is zero in LDS and never stored).
#pragma once
#include <hip/hip_runtime.h>
#include "coef_kernels.hpp"
#include "rr_index.h"

namespace givens {

constexpr int kLdsThreads = 256;
// AHEAD (template argument of the sweep kernels): arcs per thread whose coefficients are fetched a block ahead, in
// registers.  It pays for large n (many arcs per thread, long tables); for small n the resident workgroups hide
// the loads and the prefetch only costs registers, so the launch picks 0 there.
constexpr int kLdsAhead = 10;   // n <= 5120: all of a thread's arcs

// row stride of the strip in LDS: odd, so that consecutive rows fall in different banks
__host__ __device__ inline int lds_row_stride(int w) { return w | 1; }

template <typename T, int AHEAD>
__global__ __launch_bounds__(kLdsThreads) void lds_forward_kernel(
    int n, int rows, long long B, int w, const typename Pair2<T>::type *__restrict__ table,
    const T *X, T *Y, int identity, int mirror)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    T *strip = reinterpret_cast<T *>(smem_raw);
    const int H = n >> 1;
    const int ldw = lds_row_stride(w);
    const long long b0 = (long long)blockIdx.x * w;
    const int wv = (B - b0) < w ? (int)(B - b0) : w;

    for (long long idx = threadIdx.x; idx < (long long)n * w; idx += blockDim.x) {
        // mirror: strip row q holds operand row n - q (q >= 1); with the mirrored table the launch applies U^T
        const int q = (int)(idx / w), c = (int)(idx % w);
        const int r = (mirror && q) ? n - q : q;
        T v = T(0);
        if (c < wv && r < rows)
            v = identity ? ((long long)r == b0 + c ? T(1) : T(0)) : X[(long long)r * B + b0 + c];
        strip[q * ldw + c] = v;
    }
    __syncthreads();

    // One arc: rotate its two rows over the strip's columns.  Section 5 / odd n: a pair that is not a free
    // parameter is bypassed, and its table entry is the identity.  Skipping every identity entry is exact (a free
    // angle of exactly 0 rotates nothing) and lets wavefronts whose 64 arcs are all bypassed move on.
    auto rotate = [&](int k, int p, typename Pair2<T>::type cs) {
        if (cs.x == T(1) && cs.y == T(0)) return;
        const int a = rr_label(n, k, p), b = rr_label(n, k, n - 1 - p);
        T *ra = strip + a * ldw;
        T *rb = strip + b * ldw;
        for (int c = 0; c < w; ++c) {
            const T va = ra[c], vb = rb[c];
            ra[c] = cs.x * va - cs.y * vb;
            rb[c] = cs.y * va + cs.x * vb;
        }
    };
    // A thread's first AHEAD arcs of a block get their cos/sin a block ahead, in registers: a block is short
    // (a few microseconds) and ends in a barrier, so a load issued inside it is waited for in full.
    typename Pair2<T>::type ahead[AHEAD > 0 ? AHEAD : 1];
    auto fetch = [&](int k) {
#pragma unroll
        for (int i = 0; i < AHEAD; ++i) {
            const int p = threadIdx.x + i * kLdsThreads;
            if (k >= 0 && p < H) ahead[i] = table[(long long)k * H + p];
        }
    };
    fetch(n - 2);
    for (int k = n - 2; k >= 0; --k) {                      // the blocks in reverse order (Algorithm 2)
        typename Pair2<T>::type cur[AHEAD > 0 ? AHEAD : 1];
#pragma unroll
        for (int i = 0; i < AHEAD; ++i) cur[i] = ahead[i];
        fetch(k - 1);
#pragma unroll
        for (int i = 0; i < AHEAD; ++i) {
            const int p = threadIdx.x + i * kLdsThreads;
            if (p < H) rotate(k, p, cur[i]);
        }
        for (int p = threadIdx.x + AHEAD * kLdsThreads; p < H; p += kLdsThreads)
            rotate(k, p, table[(long long)k * H + p]);
        __syncthreads();                                    // the next block pairs these rows differently
    }

    for (long long idx = threadIdx.x; idx < (long long)n * w; idx += blockDim.x) {
        const int q = (int)(idx / w), c = (int)(idx % w);
        const int r = (mirror && q) ? n - q : q;
        if (c < wv && r < rows) Y[(long long)r * B + b0 + c] = strip[q * ldw + c];
    }
}

// Reverse sweep on strips [strip0, strip0 + gridDim.x).  partial is [gridDim.x][N].  map: nullptr, or the index
// in theta of every entry of E (-1: bypassed pair).
template <typename T, int AHEAD>
__global__ __launch_bounds__(kLdsThreads) void lds_backward_kernel(
    int n, int rows, long long B, int w, long long strip0, const typename Pair2<T>::type *__restrict__ table,
    const T *Yin, const T *G, T *dX, T *__restrict__ partial, int g_identity, const int *__restrict__ map)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    const int H = n >> 1;
    const int ldw = lds_row_stride(w);
    T *z = reinterpret_cast<T *>(smem_raw);
    T *gb = z + (size_t)n * ldw;
    const long long b0 = (strip0 + blockIdx.x) * w;
    const int wv = (B - b0) < w ? (int)(B - b0) : w;
    const long long N = (long long)(n - 1) * H;
    T *mine = partial + (long long)blockIdx.x * N;

    for (long long idx = threadIdx.x; idx < (long long)n * w; idx += blockDim.x) {
        const int r = (int)(idx / w), c = (int)(idx % w);
        T vz = T(0), vg = T(0);
        if (c < wv && r < rows) {
            vz = Yin[(long long)r * B + b0 + c];
            vg = g_identity ? ((long long)r == b0 + c ? T(1) : T(0)) : G[(long long)r * B + b0 + c]; // G = I_n: not read
        }
        z[r * ldw + c] = vz;
        gb[r * ldw + c] = vg;
    }
    __syncthreads();

    // One arc: its share of dL/dtheta, then the transposed rotation of both strips' rows.  A bypassed pair
    // (bypass: Section 5, odd n) has no gradient component and rotates nothing; its entry of the partial sums
    // stays unwritten and the second stage drops it.  (A free angle of exactly 0 still needs its sum, so the
    // coefficient alone does not decide here.)
    auto undo = [&](int k, int p, typename Pair2<T>::type cs, bool bypass) {
        if (bypass) return;
        const int a = rr_label(n, k, p), b = rr_label(n, k, n - 1 - p);
        T *za = z + a * ldw, *zb = z + b * ldw;
        T *ga = gb + a * ldw, *gbb = gb + b * ldw;
        T sum = T(0);
        for (int c = 0; c < w; ++c) {
            const T va = za[c], vb = zb[c], ua = ga[c], ub = gbb[c];
            sum += ub * va - ua * vb;                   // gbar_bot z_top - gbar_top z_bot
            za[c] = cs.x * va + cs.y * vb;              // transposed rotation
            zb[c] = cs.x * vb - cs.y * va;
            ga[c] = cs.x * ua + cs.y * ub;
            gbb[c] = cs.x * ub - cs.y * ua;
        }
        // the orientation sign is applied by the second-stage reduction (factor array)
        mine[(long long)k * H + p] = sum;
    };
    // coefficients (and bypass marks) of a thread's first AHEAD arcs a block ahead, as in the forward kernel
    // (the marks are kept as loaded and compared when used: a comparison here would wait for the load)
    typename Pair2<T>::type ahead[AHEAD > 0 ? AHEAD : 1];
    int mark_ahead[AHEAD > 0 ? AHEAD : 1];
    auto fetch = [&](int k) {
#pragma unroll
        for (int i = 0; i < AHEAD; ++i) {
            const int p = threadIdx.x + i * kLdsThreads;
            if (k <= n - 2 && p < H) {
                ahead[i] = table[(long long)k * H + p];
                mark_ahead[i] = map ? map[(long long)k * H + p] : 0;
            }
        }
    };
    fetch(0);
    for (int k = 0; k <= n - 2; ++k) {                      // blocks b_1, b_2, ... in order
        typename Pair2<T>::type cur[AHEAD > 0 ? AHEAD : 1];
        int mark[AHEAD > 0 ? AHEAD : 1];
#pragma unroll
        for (int i = 0; i < AHEAD; ++i) { cur[i] = ahead[i]; mark[i] = mark_ahead[i]; }
        fetch(k + 1);
#pragma unroll
        for (int i = 0; i < AHEAD; ++i) {
            const int p = threadIdx.x + i * kLdsThreads;
            if (p < H) undo(k, p, cur[i], mark[i] < 0);
        }
        for (int p = threadIdx.x + AHEAD * kLdsThreads; p < H; p += kLdsThreads) {
            const bool bypass = map && map[(long long)k * H + p] < 0;
            if (!bypass) undo(k, p, table[(long long)k * H + p], false);
        }
        __syncthreads();
    }

    if (dX) {
        for (long long idx = threadIdx.x; idx < (long long)n * w; idx += blockDim.x) {
            const int r = (int)(idx / w), c = (int)(idx % w);
            if (c < wv && r < rows) dX[(long long)r * B + b0 + c] = gb[r * ldw + c];
        }
    }
}

} // namespace givens
