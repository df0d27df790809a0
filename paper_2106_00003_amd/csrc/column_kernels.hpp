// Column kernels (float): the forward family for small n (n <= 128).
//
// One lane owns one column of the operand and keeps all n of its rows in VGPRs, so a block of
// Algorithm 2 (Section 3: n/2 disjoint pairs) is n/2 rotations inside the lane with no exchange at
// all, and cos/sin are the same for every lane: they come through scalar loads from the
// standard-form table of coef_kernels.hpp (orientation folded into the sine).  As in the carousel
// kernels the rows are kept in circle-method *position* order: block k pairs position p with position
// n-1-p, and going from block k to block k-1 the ring of positions 1..n-1 turns by one.  Inside an
// unrolled group of kGroup blocks the turn is a renaming of registers; after the group the ring is
// turned physically (n-1 register moves per kGroup blocks).
//
// The reverse sweep of this family is not a kernel of its own: for the wide batches small n comes
// with, the gradient goes through the Gram matrix (C = Y G^T by one GEMM, the reverse sweep on the
// n x n operand C in the LDS family, dX by this forward kernel on the mirrored problem).
#pragma once
#include <hip/hip_runtime.h>

#include <utility>

#include "rr_index.h"

namespace givens {

constexpr int kColumnThreads = 256;
constexpr int kColumnMaxN = 128;

template <int N>
struct ColumnFwd {
    static constexpr int kRing = N - 1;
    static constexpr int kGroup = (N - 1 >= 4) ? 4 : 1; // blocks per physical turn of the ring
    float pos[N];                                        // pos[0]: position 0; pos[1 + i]: ring index i

    // register that holds logical position q when the ring has been turned u times by renaming
    template <int U>
    static constexpr int reg(int q)
    {
        return q == 0 ? 0 : 1 + (q - 1 + U) % kRing;
    }

    template <int U, int... Ps>
    __device__ __forceinline__ void block(const float2 *__restrict__ t, std::integer_sequence<int, Ps...>)
    {
        (rotate<reg<U>(Ps), reg<U>(N - 1 - Ps)>(t[Ps]), ...);
    }
    template <int A, int B>
    __device__ __forceinline__ void rotate(float2 cs)
    {
        const float a = pos[A], b = pos[B];
        pos[A] = fmaf(cs.x, a, -(cs.y * b)); // r_i = cos U_i - sin U_j (sign of sin already oriented)
        pos[B] = fmaf(cs.x, b, cs.y * a);    // r_j = sin U_i + cos U_j
    }
    // kGroup blocks k, k-1, ..., then the physical turn by kGroup
    template <int... Us>
    __device__ __forceinline__ void group(const float2 *__restrict__ table, int k, std::integer_sequence<int, Us...>)
    {
        (block<Us>(table + (long long)(k - Us) * (N / 2), std::make_integer_sequence<int, N / 2>{}), ...);
        turn<sizeof...(Us)>();
    }
    static constexpr int gcd(int a, int b) { return b == 0 ? a : gcd(b, a % b); }
    // ring[i] <- ring[(i + S) mod kRing], in place: one temporary per cycle of the permutation
    template <int S>
    __device__ __forceinline__ void turn()
    {
        constexpr int g = gcd(kRing, S % kRing);
        if constexpr (S % kRing != 0) {
#pragma unroll
            for (int c = 0; c < g; ++c) {
                const float first = pos[1 + c];
                int i = c;
#pragma unroll
                for (int step = 0; step < kRing / g - 1; ++step) {
                    const int j = (i + S) % kRing;
                    pos[1 + i] = pos[1 + j];
                    i = j;
                }
                pos[1 + i] = first;
            }
        }
    }
};

// table: standard-form (cos, sin) per angle of the n-dimensional problem in E order (of the mirrored
// problem when `mirror` is set, see carousel_forward_kernel).  rows: the operand's row count (n, or
// n - 1 when n pads an odd problem).
// launch bound: three wavefronts per SIMD for 64 < n <= 112 (the scheduler otherwise spends registers on
// overlapping more rotations than the issue rate can use)
template <int N>
__global__ __launch_bounds__(kColumnThreads, N > 112 ? 2 : (N > 64 ? 3 : 4)) void column_forward_kernel(
    int rows, long long B, const float2 *__restrict__ table, const float *X, float *Y, int identity, int mirror)
{
    using State = ColumnFwd<N>;
    State st;
    const long long col = (long long)blockIdx.x * kColumnThreads + threadIdx.x;
    const bool live = col < B;
    // strip in the position order of block n-1 (k = n-2)
#pragma unroll
    for (int q = 0; q < N; ++q) {
        const int label = rr_label(N, N - 2, q);
        const int r = (mirror && label) ? N - label : label;
        float v = 0.f;
        if (live && r < rows) v = identity ? ((long long)r == col ? 1.f : 0.f) : X[(long long)r * B + col];
        st.pos[q] = v;
    }
    constexpr int G = State::kGroup;
    int k = N - 2;
    for (; k >= G - 1; k -= G) st.group(table, k, std::make_integer_sequence<int, G>{});
    for (; k >= 0; --k) st.group(table, k, std::make_integer_sequence<int, 1>{});
    // all turns done: the ring is in the order that follows block 1, one turn past the identity order
    // of block 1 itself, i.e. position q holds the row that block "0" would pair: undo that last turn
    // by reading the registers one ring step back.
#pragma unroll
    for (int q = 0; q < N; ++q) {
        const int src = q == 0 ? 0 : 1 + (q - 1 + State::kRing - 1) % State::kRing;
        const int r = (mirror && q) ? N - q : q;
        if (live && r < rows) Y[(long long)r * B + col] = st.pos[src];
    }
}

} // namespace givens
