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

// row stride of the strip in LDS: odd, so that consecutive rows fall in different banks
__host__ __device__ inline int lds_row_stride(int w) { return w | 1; }

template <typename T>
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
        __syncthreads();                                    // the next block pairs these rows differently
    }

    for (long long idx = threadIdx.x; idx < (long long)n * w; idx += blockDim.x) {
        const int q = (int)(idx / w), c = (int)(idx % w);
        const int r = (mirror && q) ? n - q : q;
        if (c < wv && r < rows) Y[(long long)r * B + b0 + c] = strip[q * ldw + c];
    }
}

// Reverse sweep on strips [strip0, strip0 + gridDim.x).  partial is [gridDim.x][N].
template <typename T>
__global__ __launch_bounds__(kLdsThreads) void lds_backward_kernel(
    int n, int rows, long long B, int w, long long strip0, const typename Pair2<T>::type *__restrict__ table,
    const T *Yin, const T *G, T *dX, T *__restrict__ partial, int g_identity)
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
            // the orientation sign is applied by the second-stage reduction (factor array)
            mine[(long long)k * H + p] = sum;
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
