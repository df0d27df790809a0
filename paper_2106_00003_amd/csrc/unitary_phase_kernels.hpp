// Coefficients of the unitary carousel kernels (unitary_carousel_kernels.hpp explains the carried phases):
// the parallel conversion of phi to fixed point, the sequential pass over the blocks that produces the phase
// every pair's top row is turned by, and the parallel kernel that writes the coefficient tables.
#pragma once
#include <hip/hip_runtime.h>

#include "rr_index.h"

namespace givens {

constexpr int kUnitaryCarouselMaxN = 4096;   // phases of all rows in LDS, two buffers of 4 bytes each: 32 KB
constexpr int kPhaseScanThreads = 1024;

// x = r + m * pi with |r| <= pi/2; returns m's parity.  Two-piece pi, like the lifted form's reduction.
__device__ __forceinline__ int reduce_by_pi(double x, double *r)
{
    const double m = rint(x * 0.31830988618379067154);
    *r = fma(-m, 1.2246467991473532e-16, fma(-m, 3.141592653589793116, x));
    return (int)((long long)m & 1);
}

// Phases in the sequential pass are fixed-point numbers: an unsigned 32-bit integer x stands for the angle
// 2 pi x / 2^32, so that sums and differences wrap round modulo 2 pi by themselves and the pass needs integer
// additions only.  Rounding phi to 2 pi / 2^32 = 1.5e-9 rad is a perturbation of the parameter far below
// float32's resolution of the result.
//
// The pass is one workgroup on one compute unit and is bound by the number of instructions it issues, so
// everything that does not depend on the carried phases is prepared here, in parallel.  With f = phi in fixed
// point, F2 = pi if reducing the rotation angle by a multiple of pi negates both rows (rint(theta / pi) odd)
// and "i on top" = the top position holds the pair's smaller label, per pair (see the pass for their use):
//   forward:  q.x = (i on top ? f : -f) + pi/2,   q.y = (i on top ? 0 : f) + F2
//   reverse:  q.x = (i on top ? -f : 0) + F2,     q.y = (i on top ? 0 : -f) + F2
constexpr unsigned kFixedQuarterTurn = 1u << 30, kFixedHalfTurn = 1u << 31;

template <bool REVERSE>
__global__ void unitary_phase_input_kernel(int n, const float *__restrict__ theta, const float *__restrict__ phi,
                                           uint2 *__restrict__ q)
{
    const int H = n >> 1;
    const long long N = (long long)(n - 1) * H;
    for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < N;
         e += (long long)gridDim.x * blockDim.x) {
        double x = (double)phi[e] * 0.31830988618379067154;     // in units of pi
        x -= 2.0 * rint(0.5 * x);                                 // [-1, 1]
        const unsigned f = (unsigned)(long long)llrint(x * 2147483648.0);   // pi = 2^31; +-pi wrap to one value
        double unused;
        const unsigned f2 = reduce_by_pi((double)theta[e], &unused) ? kFixedHalfTurn : 0u;
        const int k = (int)(e / H), p = (int)(e % H);
        const bool i_on_top = rr_label(n, k, p) < rr_label(n, k, n - 1 - p);
        if (!REVERSE)
            q[e] = make_uint2((i_on_top ? f : 0u - f) + kFixedQuarterTurn, (i_on_top ? 0u : f) + f2);
        else
            q[e] = make_uint2((i_on_top ? 0u - f : 0u) + f2, (i_on_top ? 0u : 0u - f) + f2);
    }
}

// The sequential pass.  REVERSE = false: blocks n-2 .. 0 (forward sweep); true: blocks 0 .. n-2 (reverse sweep).
// One workgroup; blockDim.x * PER >= n/2.  q: unitary_phase_input_kernel<REVERSE>'s output.
// The carried phases live in LDS indexed by circle-method *position*, in two buffers that take turns: thread p
// owns the pair of positions (p, n-1-p) in every block, reads its two phases from one buffer and writes the
// new ones to the places the two rows take in the next block of the pass, in the other buffer -- all four
// addresses are fixed per thread.  One barrier per block and five or six integer operations per pair:
//   forward (r_i = w c y_i - s y_j, r_j = w s y_i + c y_j: row i enters with w, both rows leave with the bottom
//   row's phase, plus phi when the bottom row is row i):
//       u = top - bottom + q.x        new bottom = bottom + q.y       new top = new bottom + (u's top bit)
//   reverse (z_i' = conj(w) (c z_i + s z_j), z_j' = -s z_i + c z_j: the rows meet at the bottom row's phase and
//   row i leaves with -phi on top of it):
//       u = top - bottom + pi/2       new bottom = bottom + q.y       new top = bottom + q.x + (u's top bit)
// u - pi/2 is the angle the top row is short of; written as r + flip * pi with r in [-pi/2, pi/2), the top bit of
// u is flip (the turned top row counts as negated) and its low 31 bits are r + pi/2.  turn[e] = u is all the pass
// stores; the table kernel takes it apart.  After the last block the rows have made one more move, which the
// final loop undoes when it writes fin[r], (cos, sin) of the phase row r ends with.
// Inputs are fetched kDepth blocks ahead (a block of the pass is far shorter than a trip to memory).
template <bool REVERSE, int PER>
__global__ __launch_bounds__(kPhaseScanThreads) void unitary_phase_scan_kernel(int n, const uint2 *__restrict__ q,
                                                                               unsigned *__restrict__ turn,
                                                                               float2 *__restrict__ fin)
{
    __shared__ unsigned a[2][kUnitaryCarouselMaxN];
    constexpr int kDepth = 16 / PER;
    static_assert(kDepth % 2 == 0, "the buffer a block reads is its index modulo 2");
    const int H = n >> 1;
    const int tid = threadIdx.x, threads = blockDim.x;
    for (int r = tid; r < n; r += threads) a[0][r] = 0u;

    // fixed places: read (top, bottom), write (where the two rows sit in the next block of the pass)
    int rt[PER], rb[PER], wt[PER], wb[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const int p = tid + i * threads, b = n - 1 - p;
        rt[i] = p;
        rb[i] = b;
        if (!REVERSE) {   // towards block k-1: position x -> x-1, position 1 -> n-1, position 0 held
            wt[i] = p == 0 ? 0 : (p == 1 ? n - 1 : p - 1);
            wb[i] = b - 1;
        } else {          // towards block k+1: position x -> x+1, position n-1 -> 1, position 0 held
            wt[i] = p == 0 ? 0 : p + 1;
            wb[i] = b == n - 1 ? 1 : b + 1;
        }
    }
    __syncthreads();

    uint2 ring[kDepth][PER];
    auto fetch = [&](int step, uint2 (&dst)[PER]) {
        const int k = REVERSE ? step : n - 2 - step;
        const uint2 *row = q + (long long)k * H;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const unsigned p = tid + i * threads;
            dst[i] = (step < n - 1 && p < (unsigned)H) ? row[p] : make_uint2(0u, 0u);
        }
    };
#pragma unroll
    for (int d = 0; d < kDepth; ++d) fetch(d, ring[d]);

    for (int step0 = 0; step0 < n - 1; step0 += kDepth) {
#pragma unroll
        for (int d = 0; d < kDepth; ++d) {
            const int step = step0 + d;
            if (step < n - 1) {                                   // uniform over the workgroup
                const int k = REVERSE ? step : n - 2 - step;
                const unsigned *cur = a[d & 1];
                unsigned *nxt = a[(d & 1) ^ 1];
                unsigned *out = turn + (long long)k * H;
#pragma unroll
                for (int i = 0; i < PER; ++i) {
                    const unsigned p = tid + i * threads;
                    if (p < (unsigned)H) {
                        const unsigned at = cur[rt[i]], ab = cur[rb[i]];
                        unsigned u, nt, nb;
                        if (!REVERSE) {
                            u = at - ab + ring[d][i].x;
                            nb = ab + ring[d][i].y;
                            nt = nb ^ (u & kFixedHalfTurn);
                        } else {
                            u = at - ab + kFixedQuarterTurn;
                            nb = ab + ring[d][i].y;
                            nt = (ab + ring[d][i].x) ^ (u & kFixedHalfTurn);
                        }
                        nxt[wt[i]] = nt;
                        nxt[wb[i]] = nb;
                        out[p] = u;
                    }
                }
                fetch(step + kDepth, ring[d]);
                __syncthreads();
            }
        }
    }
    // the phases are in the buffer the last block wrote, one move past the position order of that block
    const unsigned *final_phase = a[(n - 1) & 1];
    for (int pos = tid; pos < n; pos += threads) {
        double s, c;
        sincos((double)(int)final_phase[pos] * 1.4629180792671596e-09, &s, &c);   // 2 pi / 2^32
        int row;
        if (!REVERSE) {   // block 1's order is the identity; one move further position x holds row x+1
            row = pos == 0 ? 0 : (pos == n - 1 ? 1 : pos + 1);
        } else {          // block n-1's order, one move further
            row = rr_label(n, n - 2, pos == 0 ? 0 : (pos == 1 ? n - 1 : pos - 1));
        }
        fin[row] = make_float2((float)c, (float)s);
    }
}

// rot[e] = (tan(theta'/2), sin theta') and phs[e] = (tan(psi'/2), sin psi') from the pass's turn[e]; sgn[e] = +-1:
// the real rotation uses the angle sgn[e] * theta[e], reduced by a multiple of pi to theta' (and in the reverse
// sweep sgn[e] is also the sign of the pair's dL/dtheta sum); with ORIENT, orient[e] = 1 when the top position of
// the pair holds its smaller label (reverse sweep).
template <bool ORIENT>
__global__ void unitary_carousel_table_kernel(int n, const float *__restrict__ theta, const unsigned *__restrict__ turn,
                                              float *__restrict__ sgn, float2 *__restrict__ rot,
                                              float2 *__restrict__ phs, float *__restrict__ orient)
{
    const int H = n >> 1;
    const long long N = (long long)(n - 1) * H;
    for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < N;
         e += (long long)gridDim.x * blockDim.x) {
        const int k = (int)(e / H), p = (int)(e % H);
        const bool i_on_top = rr_label(n, k, p) < rr_label(n, k, n - 1 - p);
        const unsigned u = turn[e];
        const bool flip = (u >> 31) != 0;
        const double psi = (double)((int)(u & (kFixedHalfTurn - 1)) - (int)kFixedQuarterTurn) * 1.4629180792671596e-09;
        const float sg = (i_on_top != flip) ? 1.f : -1.f;
        double r;
        reduce_by_pi((double)sg * (double)theta[e], &r);
        double s, c;
        sincos(0.5 * r, &s, &c);
        rot[e] = make_float2((float)(s / c), (float)(2.0 * s * c));
        sincos(0.5 * psi, &s, &c);
        phs[e] = make_float2((float)(s / c), (float)(2.0 * s * c));
        sgn[e] = sg;
        if constexpr (ORIENT) orient[e] = i_on_top ? 1.f : 0.f;
    }
}

} // namespace givens
