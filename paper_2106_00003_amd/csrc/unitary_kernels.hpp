// Unitary extension (the paper's appendix "Adaptations to U(n)"): LDS strip kernels on complex operands.
//
// Factor of pair e = (i, j), i < j:  G_ii = w cos, G_ij = -sin, G_ji = w sin, G_jj = cos, w = exp(i phi)
// (the appendix's forward algorithm: r_i = w cos U_i - sin U_j, r_j = w sin U_i + cos U_j).  Operands are
// row-major n x B arrays of interleaved (re, im) pairs.  Same structure as lds_kernels.hpp: one
// workgroup keeps an n x w strip in LDS for all n-1 blocks, each thread owns whole pairs of a block.
// The table holds (cos theta, sin theta, cos phi, sin phi) per angle in E order, unoriented: these
// kernels look the labels up themselves and put the smaller one first.
#pragma once
#include <hip/hip_runtime.h>

#include "rr_index.h"

namespace givens {

template <typename T> struct Cplx;
template <> struct Cplx<float> { using type = float2; using quad = float4; };
template <> struct Cplx<double> { using type = double2; using quad = double4; };

constexpr int kUnitaryThreads = 256;
constexpr int kUnitaryAhead = 8;   // AHEAD of the large-strip instances (see lds_kernels.hpp): n <= 4096: all pairs

template <typename T>
__global__ void unitary_table_kernel(int n, const T *__restrict__ theta, const T *__restrict__ phi,
                                     typename Cplx<T>::quad *__restrict__ table)
{
    const long long N = (long long)(n - 1) * (n >> 1);
    for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < N;
         e += (long long)gridDim.x * blockDim.x) {
        double s, c, sp, cp;
        sincos((double)theta[e], &s, &c);
        sincos((double)phi[e], &sp, &cp);
        typename Cplx<T>::quad out;
        out.x = (T)c; out.y = (T)s; out.z = (T)cp; out.w = (T)sp;
        table[e] = out;
    }
}

template <typename T>
__device__ __forceinline__ typename Cplx<T>::type cmul(T wr, T wi, typename Cplx<T>::type v)
{
    typename Cplx<T>::type r;
    r.x = wr * v.x - wi * v.y;
    r.y = wr * v.y + wi * v.x;
    return r;
}

template <typename T, int AHEAD>
__global__ __launch_bounds__(kUnitaryThreads) void unitary_forward_kernel(
    int n, long long B, int w, const typename Cplx<T>::quad *__restrict__ table,
    const typename Cplx<T>::type *X, typename Cplx<T>::type *Y, int identity)
{
    using C = typename Cplx<T>::type;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    C *strip = reinterpret_cast<C *>(smem_raw);
    const int H = n >> 1;
    const long long b0 = (long long)blockIdx.x * w;
    const int wv = (B - b0) < w ? (int)(B - b0) : w;

    for (long long idx = threadIdx.x; idx < (long long)n * w; idx += blockDim.x) {
        const int r = (int)(idx / w), c = (int)(idx % w);
        C v;
        v.x = T(0); v.y = T(0);
        if (c < wv) {
            if (identity) v.x = ((long long)r == b0 + c) ? T(1) : T(0);
            else v = X[(long long)r * B + b0 + c];
        }
        strip[r * w + c] = v;
    }
    __syncthreads();

    auto update = [&](int k, int p, typename Cplx<T>::quad q) {
        const int a = rr_label(n, k, p), b = rr_label(n, k, n - 1 - p);
        const int i = a < b ? a : b, j = a < b ? b : a;
        C *ri = strip + i * w, *rj = strip + j * w;
        for (int c = 0; c < w; ++c) {
            const C ui = cmul<T>(q.z, q.w, ri[c]);      // exp(i phi) U_i
            const C uj = rj[c];
            C ni, nj;
            ni.x = q.x * ui.x - q.y * uj.x; ni.y = q.x * ui.y - q.y * uj.y;
            nj.x = q.y * ui.x + q.x * uj.x; nj.y = q.y * ui.y + q.x * uj.y;
            ri[c] = ni;
            rj[c] = nj;
        }
    };
    // a thread's first kUnitaryAhead pairs of a block get their coefficients a block ahead, in registers (a block
    // is short and ends in a barrier, so a load issued inside it is waited for in full)
    typename Cplx<T>::quad ahead[AHEAD > 0 ? AHEAD : 1];
    auto fetch = [&](int k) {
#pragma unroll
        for (int i = 0; i < AHEAD; ++i) {
            const int p = threadIdx.x + i * kUnitaryThreads;
            if (k >= 0 && p < H) ahead[i] = table[(long long)k * H + p];
        }
    };
    fetch(n - 2);
    for (int k = n - 2; k >= 0; --k) {                       // the blocks in reverse order (appendix, forward algorithm)
        typename Cplx<T>::quad cur[AHEAD > 0 ? AHEAD : 1];
#pragma unroll
        for (int i = 0; i < AHEAD; ++i) cur[i] = ahead[i];
        fetch(k - 1);
#pragma unroll
        for (int i = 0; i < AHEAD; ++i) {
            const int p = threadIdx.x + i * kUnitaryThreads;
            if (p < H) update(k, p, cur[i]);
        }
        for (int p = threadIdx.x + AHEAD * kUnitaryThreads; p < H; p += kUnitaryThreads)
            update(k, p, table[(long long)k * H + p]);
        __syncthreads();
    }

    for (long long idx = threadIdx.x; idx < (long long)n * w; idx += blockDim.x) {
        const int r = (int)(idx / w), c = (int)(idx % w);
        if (c < wv) Y[(long long)r * B + b0 + c] = strip[r * w + c];
    }
}

// Reverse sweep on strips [strip0, strip0 + gridDim.x).  partial is [gridDim.x][2 N]: the strip's share
// of dL/dtheta in the first N entries of a row, of dL/dphi in the last N.  With z and gbar the carried
// strips, per pair (i, j) of block k:
//   dtheta = Re sum_b ( conj(gbar_j) z_i - conj(gbar_i) z_j )            (before the block is undone)
//   z, gbar <- G^dagger z, G^dagger gbar:  row i <- conj(w) (c row_i + s row_j),  row j <- -s row_i + c row_j
//   dphi   = -Im sum_b conj(gbar_i) z_i                                   (after: P_e z = i (c, s)^T (c z_i + s z_j)
//            and c z_i + s z_j = w z_i', c gbar_i + s gbar_j = w gbar_i', so the phases cancel)
template <typename T, int AHEAD>
__global__ __launch_bounds__(kUnitaryThreads) void unitary_backward_kernel(
    int n, long long B, int w, long long strip0, const typename Cplx<T>::quad *__restrict__ table,
    const typename Cplx<T>::type *Yin, const typename Cplx<T>::type *G, typename Cplx<T>::type *dX,
    T *__restrict__ partial)
{
    using C = typename Cplx<T>::type;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    const int H = n >> 1;
    C *z = reinterpret_cast<C *>(smem_raw);
    C *gb = z + (size_t)n * w;
    const long long b0 = (strip0 + blockIdx.x) * w;
    const int wv = (B - b0) < w ? (int)(B - b0) : w;
    const long long N = (long long)(n - 1) * H;
    T *mine = partial + (long long)blockIdx.x * 2 * N;

    for (long long idx = threadIdx.x; idx < (long long)n * w; idx += blockDim.x) {
        const int r = (int)(idx / w), c = (int)(idx % w);
        C vz, vg;
        vz.x = vz.y = vg.x = vg.y = T(0);
        if (c < wv) {
            vz = Yin[(long long)r * B + b0 + c];
            vg = G[(long long)r * B + b0 + c];
        }
        z[r * w + c] = vz;
        gb[r * w + c] = vg;
    }
    __syncthreads();

    auto undo = [&](int k, int p, typename Cplx<T>::quad q) {
        const int a = rr_label(n, k, p), b = rr_label(n, k, n - 1 - p);
        const int i = a < b ? a : b, j = a < b ? b : a;
        C *zi = z + i * w, *zj = z + j * w, *gi = gb + i * w, *gj = gb + j * w;
        T sum_t = T(0), sum_p = T(0);
        for (int c = 0; c < w; ++c) {
            const C a_i = zi[c], a_j = zj[c], u_i = gi[c], u_j = gj[c];
            sum_t += (u_j.x * a_i.x + u_j.y * a_i.y) - (u_i.x * a_j.x + u_i.y * a_j.y);
            C t;
            t.x = q.x * a_i.x + q.y * a_j.x; t.y = q.x * a_i.y + q.y * a_j.y;
            const C nz_i = cmul<T>(q.z, -q.w, t);       // conj(w) (c z_i + s z_j)
            C nz_j;
            nz_j.x = q.x * a_j.x - q.y * a_i.x; nz_j.y = q.x * a_j.y - q.y * a_i.y;
            t.x = q.x * u_i.x + q.y * u_j.x; t.y = q.x * u_i.y + q.y * u_j.y;
            const C ng_i = cmul<T>(q.z, -q.w, t);
            C ng_j;
            ng_j.x = q.x * u_j.x - q.y * u_i.x; ng_j.y = q.x * u_j.y - q.y * u_i.y;
            sum_p += ng_i.y * nz_i.x - ng_i.x * nz_i.y; // -Im( conj(gbar_i') z_i' )
            zi[c] = nz_i; zj[c] = nz_j; gi[c] = ng_i; gj[c] = ng_j;
        }
        mine[(long long)k * H + p] = sum_t;
        mine[N + (long long)k * H + p] = sum_p;
    };
    typename Cplx<T>::quad ahead[AHEAD > 0 ? AHEAD : 1];   // coefficients a block ahead, as in the forward kernel
    auto fetch = [&](int k) {
#pragma unroll
        for (int i = 0; i < AHEAD; ++i) {
            const int p = threadIdx.x + i * kUnitaryThreads;
            if (k <= n - 2 && p < H) ahead[i] = table[(long long)k * H + p];
        }
    };
    fetch(0);
    for (int k = 0; k <= n - 2; ++k) {
        typename Cplx<T>::quad cur[AHEAD > 0 ? AHEAD : 1];
#pragma unroll
        for (int i = 0; i < AHEAD; ++i) cur[i] = ahead[i];
        fetch(k + 1);
#pragma unroll
        for (int i = 0; i < AHEAD; ++i) {
            const int p = threadIdx.x + i * kUnitaryThreads;
            if (p < H) undo(k, p, cur[i]);
        }
        for (int p = threadIdx.x + AHEAD * kUnitaryThreads; p < H; p += kUnitaryThreads)
            undo(k, p, table[(long long)k * H + p]);
        __syncthreads();
    }

    if (dX) {
        for (long long idx = threadIdx.x; idx < (long long)n * w; idx += blockDim.x) {
            const int r = (int)(idx / w), c = (int)(idx % w);
            if (c < wv) dX[(long long)r * B + b0 + c] = gb[r * w + c];
        }
    }
}

// out[e] (+)= sum over rows r of partial[r * stride + e], rows in order (fixed order: reproducible)
template <typename T>
__global__ void sum_rows_kernel(long long count, long long rows, long long stride, const T *__restrict__ partial,
                                T *out, int accumulate)
{
    const long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= count) return;
    T a0 = T(0), a1 = T(0), a2 = T(0), a3 = T(0);
    long long r = 0;
    for (; r + 4 <= rows; r += 4) {             // four loads in flight; the order of additions is fixed
        a0 += partial[r * stride + e];
        a1 += partial[(r + 1) * stride + e];
        a2 += partial[(r + 2) * stride + e];
        a3 += partial[(r + 3) * stride + e];
    }
    for (; r < rows; ++r) a0 += partial[r * stride + e];
    const T acc = (a0 + a1) + (a2 + a3);
    out[e] = accumulate ? out[e] + acc : acc;
}

} // namespace givens
