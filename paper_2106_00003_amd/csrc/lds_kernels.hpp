// LDS strip kernels: the general-shape family (any even n whose strip fits in LDS, float or
// double).  One workgroup owns w columns of the operand, keeps the n x w strip in LDS for all
// n-1 blocks of Algorithm 2, and touches HBM once on the way in and once on the way out.
// Inside a block each thread owns whole pairs (arcs) and walks the strip's columns, so the
// per-pair gradient sum of the reverse sweep needs no cross-thread reduction.
//
// The table holds, per (block k, arc p), cos(theta) and the sine with the orientation folded in:
// the strip is addressed by the labels at positions p ("top") and n-1-p ("bottom") of the
// circle-method sequence, and sin is negated when the top label is the larger one, so that
//     top' = c*top - s*bot,   bot' = s*top + c*bot
// is Algorithm 2's update (r_i = c U_i - s U_j, r_j = s U_i + c U_j with i < j) either way.
#pragma once
#include <hip/hip_runtime.h>
#include "rr_index.h"

namespace givens {

template <typename T> struct Pair2;
template <> struct Pair2<float> { using type = float2; };
template <> struct Pair2<double> { using type = double2; };

constexpr int kLdsThreads = 256;

// row stride of the strip in LDS: odd, so that consecutive rows fall in different banks
__host__ __device__ inline int lds_row_stride(int w) { return w | 1; }

template <typename T>
__global__ __launch_bounds__(kLdsThreads) void lds_forward_kernel(
    int n, long long B, int w, const typename Pair2<T>::type *__restrict__ table,
    const T *X, T *Y, int identity)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    T *strip = reinterpret_cast<T *>(smem_raw);
    const int H = n >> 1;
    const int ldw = lds_row_stride(w);
    const long long b0 = (long long)blockIdx.x * w;
    const int wv = (B - b0) < w ? (int)(B - b0) : w;

    for (long long idx = threadIdx.x; idx < (long long)n * w; idx += blockDim.x) {
        const int r = (int)(idx / w), c = (int)(idx % w);
        T v = T(0);
        if (c < wv) v = identity ? ((long long)r == b0 + c ? T(1) : T(0)) : X[(long long)r * B + b0 + c];
        strip[r * ldw + c] = v;
    }
    __syncthreads();

    for (int k = n - 2; k >= 0; --k) {                      // reversed(B)
        for (int p = threadIdx.x; p < H; p += blockDim.x) { // the block's arcs: disjoint rows
            const int a = rr_label(n, k, p), b = rr_label(n, k, n - 1 - p);
            const auto cs = table[(long long)k * H + p];
            T *ra = strip + a * ldw;
            T *rb = strip + b * ldw;
            for (int c = 0; c < w; ++c) {
                const T va = ra[c], vb = rb[c];
                ra[c] = cs.x * va - cs.y * vb;
                rb[c] = cs.y * va + cs.x * vb;
            }
        }
        __syncthreads();                                    // "Synchronize parallel operations"
    }

    for (long long idx = threadIdx.x; idx < (long long)n * w; idx += blockDim.x) {
        const int r = (int)(idx / w), c = (int)(idx % w);
        if (c < wv) Y[(long long)r * B + b0 + c] = strip[r * ldw + c];
    }
}

// Reverse sweep on strips [strip0, strip0 + gridDim.x).  partial is [gridDim.x][N].
template <typename T>
__global__ __launch_bounds__(kLdsThreads) void lds_backward_kernel(
    int n, long long B, int w, long long strip0, const typename Pair2<T>::type *__restrict__ table,
    const T *Yin, const T *G, T *dX, T *__restrict__ partial)
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
        if (c < wv) {
            vz = Yin[(long long)r * B + b0 + c];
            vg = G[(long long)r * B + b0 + c];
        }
        z[r * ldw + c] = vz;
        gb[r * ldw + c] = vg;
    }
    __syncthreads();

    for (int k = 0; k <= n - 2; ++k) {                      // blocks b_1, b_2, ... in order
        for (int p = threadIdx.x; p < H; p += blockDim.x) {
            const int a = rr_label(n, k, p), b = rr_label(n, k, n - 1 - p);
            const auto cs = table[(long long)k * H + p];
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
            // orientation sign (top holds the larger label <=> negate) is applied by the reduction
            mine[(long long)k * H + p] = sum;
        }
        __syncthreads();
    }

    if (dX) {
        for (long long idx = threadIdx.x; idx < (long long)n * w; idx += blockDim.x) {
            const int r = (int)(idx / w), c = (int)(idx % w);
            if (c < wv) dX[(long long)r * B + b0 + c] = gb[r * ldw + c];
        }
    }
}

// Second stage of the gradient reduction: dtheta[e] (+)= sign(e) * sum over strips s of
// partial[s][e], in strip order (fixed order: reproducible).  The sweeps store
// sum_b (gbar_bot z_top - gbar_top z_bot); with i < j the paper's term is gbar_j z_i - gbar_i z_j,
// so the sum is negated for the pairs whose top position holds the larger label.
template <typename T>
__global__ void reduce_partials_kernel(int n, long long nstrips, const T *__restrict__ partial,
                                       T *dtheta, int accumulate)
{
    const int H = n >> 1;
    const long long N = (long long)(n - 1) * H;
    const long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= N) return;
    T a0 = T(0), a1 = T(0), a2 = T(0), a3 = T(0);
    long long s = 0;
    for (; s + 4 <= nstrips; s += 4) {          // four loads in flight; the order of additions is fixed
        a0 += partial[s * N + e];
        a1 += partial[(s + 1) * N + e];
        a2 += partial[(s + 2) * N + e];
        a3 += partial[(s + 3) * N + e];
    }
    for (; s < nstrips; ++s) a0 += partial[s * N + e];
    T acc = (a0 + a1) + (a2 + a3);
    const int k = (int)(e / H), p = (int)(e % H);
    if (rr_label(n, k, p) > rr_label(n, k, n - 1 - p)) acc = -acc;
    dtheta[e] = accumulate ? dtheta[e] + acc : acc;
}

// cos/sin table in E order, evaluated in double whatever T is, with the orientation sign folded
// into the sine (see the header comment).
template <typename T>
__global__ void coef_table_kernel(int n, const T *__restrict__ theta,
                                  typename Pair2<T>::type *__restrict__ table)
{
    const int H = n >> 1;
    const long long N = (long long)(n - 1) * H;
    const long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= N) return;
    const int k = (int)(e / H), p = (int)(e % H);
    const int a = rr_label(n, k, p), b = rr_label(n, k, n - 1 - p);
    double s, c;
    sincos((double)theta[e], &s, &c);
    if (a > b) s = -s;
    typename Pair2<T>::type out;
    out.x = (T)c;
    out.y = (T)s;
    table[e] = out;
}

} // namespace givens
