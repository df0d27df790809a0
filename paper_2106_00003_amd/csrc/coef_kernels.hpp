// Coefficient kernels: everything the sweeps need that depends on theta only.
//
// Standard form.  Per (block k, arc p): cos(theta) and the sine with the orientation folded in (the
// sweeps address the strip by circle-method position: "top" = position p, "bottom" = position
// n-1-p; the sine is negated when the top position holds the larger label), so that
//     top' = c*top - s*bot,   bot' = s*top + c*bot
// is Algorithm 2's update (r_i = c U_i - s U_j, r_j = s U_i + c U_j with i < j) either way.
//
// Scaled form (float, near-identity angles only: max |theta| <= kScaledMaxAbsTheta).  Each row r is
// kept as a stored value y~_r = y_r / d_r, where d_r is the product of the cosines of the rotations
// the row has been through since the last renormalisation.  Dividing a rotation of rows (a, b) by
// its cosine turns it into two FMAs on the stored values,
//     a~' = a~ - alpha * b~,   b~' = b~ + beta * a~,
//     alpha = tan(theta) * d_b / d_a,   beta = tan(theta) * d_a / d_b,   d_a' = c d_a,  d_b' = c d_b,
// and every kRenormPeriod blocks (and after the last one) the stored values are multiplied by d_r and
// d_r restarts at 1.  The factors d depend on theta alone, so they are produced here, in float64: a
// scan walks each row's trajectory through the circle-method positions for one renormalisation
// period (scaled_scan_kernel), and the table kernel turns (theta, d_a, d_b) into (alpha, beta).
// The result is the same product of Givens rotations (Eq. (2)); only the rounding differs (one
// rounding per output instead of two).
//
// Lifted form (float, any finite angles up to kLiftedMaxAbsTheta).  A rotation is three shears,
//     a -= t b,   b += s a,   a -= t b,       t = tan(theta/2),  s = sin(theta),
// i.e. three dependent FMAs instead of 2 MUL + 2 FMA.  To keep |t| <= 1 the angle is first reduced
// by a multiple of pi, theta = theta' + m*pi with |theta'| <= pi/2, R(theta) = (-1)^m R(theta'), and
// the signs (-1)^m are carried exactly like the scaled form's cosines: a row's stored value is
// y_r / d_r with d_r = +-1, the shear coefficients are multiplied by d_a d_b, and the rows are
// multiplied back by d_r at the same points.  Same scan, same table layout, same sweeps.
//
// The choice between the forms is made on the device: theta_range_kernel leaves the bit pattern of
// max |theta| in a flag word, and every kernel of a form returns at once when the flag says another
// form is the one to run (form_for_range).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "forms.hpp"
#include "rr_index.h"

namespace givens {

template <typename T> struct Pair2;
template <> struct Pair2<float> { using type = float2; };
template <> struct Pair2<double> { using type = double2; };

// flag <- bit pattern of max |theta| (non-negative floats order like unsigned integers; NaN sorts last).
// theta is read as float4 where alignment allows; N is tiny next to the sweeps but this kernel sits
// in front of every call, so it should run at memory speed.  Atomics on one word serialise (some 10 ns
// each: thousands of them cost more than reading theta), so the wavefronts of a workgroup combine
// through LDS first and send one atomicMax per workgroup.  `flag` must be zero when the kernel starts: the
// host alternates between two flag words from call to call, and each launch zeroes the word the next one
// will use (`next_flag`; nothing reads that word any more: the call that used it is earlier in the stream).
constexpr int kRangeBlocks = 512;
__global__ __launch_bounds__(512) void theta_range_kernel(long long N, const float *__restrict__ theta,
                                                          unsigned *flag, unsigned *next_flag)
{
    if (next_flag && blockIdx.x == 0 && threadIdx.x == 0) *next_flag = 0u;
    unsigned m = 0u;
    const long long tid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long nthreads = (long long)gridDim.x * blockDim.x;
    const bool aligned = (reinterpret_cast<uintptr_t>(theta) & 15u) == 0;
    const long long n4 = aligned ? N / 4 : 0;
    const uint4 *t4 = reinterpret_cast<const uint4 *>(theta);
    for (long long i = tid; i < n4; i += nthreads) {
        const uint4 v = t4[i];
        const unsigned a = v.x & 0x7fffffffu, b = v.y & 0x7fffffffu, c = v.z & 0x7fffffffu, d = v.w & 0x7fffffffu;
        const unsigned ab = a > b ? a : b, cd = c > d ? c : d;
        const unsigned q = ab > cd ? ab : cd;
        m = q > m ? q : m;
    }
    for (long long e = n4 * 4 + tid; e < N; e += nthreads) {
        const unsigned bits = __float_as_uint(theta[e]) & 0x7fffffffu;
        m = bits > m ? bits : m;
    }
    for (int off = 32; off > 0; off >>= 1) {
        const unsigned other = (unsigned)__shfl_xor((int)m, off, 64);
        m = other > m ? other : m;
    }
    __shared__ unsigned wave_max[16];
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) wave_max[wave] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        const int waves = (blockDim.x + 63) >> 6;
        for (int w = 1; w < waves; ++w) m = wave_max[w] > m ? wave_max[w] : m;
        atomicMax(flag, m);
    }
}
// puts one flag word to zero (before the range check of givens_prepare, whose flag word is its own)
__global__ void reset_flag_kernel(unsigned *flag) { *flag = 0u; }

// sin and cos in float64 for |x| <= pi/4 (the only arguments the scaled form ever sees): plain
// Taylor polynomials, no range reduction.  Truncation error below 1e-17 relative on that interval.
__device__ __forceinline__ double cos_small(double x)
{
    const double z = x * x;
    double p = 1.0 / 20922789888000.0;                 // 1/16!
    p = fma(p, z, -1.0 / 87178291200.0);               // 1/14!
    p = fma(p, z, 1.0 / 479001600.0);                  // 1/12!
    p = fma(p, z, -1.0 / 3628800.0);                   // 1/10!
    p = fma(p, z, 1.0 / 40320.0);                      // 1/8!
    p = fma(p, z, -1.0 / 720.0);                       // 1/6!
    p = fma(p, z, 1.0 / 24.0);                         // 1/4!
    p = fma(p, z, -0.5);
    return fma(p, z, 1.0);
}
__device__ __forceinline__ double sin_small(double x)
{
    const double z = x * x;
    double p = 1.0 / 355687428096000.0;                // 1/17!
    p = fma(p, z, -1.0 / 1307674368000.0);             // 1/15!
    p = fma(p, z, 1.0 / 6227020800.0);                 // 1/13!
    p = fma(p, z, -1.0 / 39916800.0);                  // 1/11!
    p = fma(p, z, 1.0 / 362880.0);                     // 1/9!
    p = fma(p, z, -1.0 / 5040.0);                      // 1/7!
    p = fma(p, z, 1.0 / 120.0);                        // 1/5!
    p = fma(p, z, -1.0 / 6.0);
    return fma(p * z, x, x);
}

// Lifted form: theta = theta' + m*pi with |theta'| <= pi/2, so that R(theta) = (-1)^m R(theta') and
// the three shears of R(theta') have coefficients tan(theta'/2), sin(theta') of magnitude <= 1.
// Returns theta'; *odd = m is odd.  Used by the scan (signs) and the table (coefficients) alike.
__device__ __forceinline__ double lift_reduce(double th, bool *odd)
{
    const double m = rint(th * 0.31830988618379067154);            // |th| <= 1e6: exact integer
    *odd = ((long long)m & 1LL) != 0;
    return fma(-m, 1.2246467991473532e-16, fma(-m, 3.141592653589793116, th)); // pi in two pieces
}

// Angle of entry e of the full sequence E.  With a restricted parametrisation or odd n (Section 5 of
// the paper; end of Section 3) theta lists only the free pairs: `map` (nullptr: every pair is free)
// gives each entry of E its index in theta, or -1 for a bypassed pair, which is run as a rotation
// by zero.
//
// `mirror`: the tables are wanted for the mirrored problem, whose forward product equals the
// transposed product of the original one up to a relabelling of the rows.  Relabel row r >= 1 as
// n - r and keep row 0: the pairs of block k become the pairs of block n-2-k, arc by arc, and
//     U(theta)^T = P^T U(theta') P,   theta'[k][p] = -theta[n-2-k][p] for p = 0 (pairs with row 0,
//     whose order i < j survives the relabelling) and +theta[n-2-k][p] otherwise (order reversed:
//     the sign change of the transpose and that of the swap cancel),
// with P the relabelling.  So entry e = (k, p) of the mirrored problem reads the original entry
// (n-2-k, p) with that sign.
template <typename T>
__device__ __forceinline__ T theta_at(const T *__restrict__ theta, const int *__restrict__ map, int mirror, int n,
                                      long long e)
{
    T sign = T(1);
    if (mirror) {
        const int H = n >> 1;
        const long long k = e / H;
        const int p = (int)(e - k * H);
        e = (long long)(n - 2 - k) * H + p;
        if (p == 0) sign = T(-1);
    }
    if (!map) return sign * theta[e];
    const int c = map[e];
    return c < 0 ? T(0) : sign * theta[c];
}

// Scaled and lifted forms, step 1.  One thread per (renormalisation period g, row r): walks the row
// through the period's blocks in sweep order (FWD: k = n-2, n-3, ...; reverse sweep: k = 0, 1, ...),
// records the row's factor d *before* each block at D[k][position], and leaves the factor after the
// period's last block in renorm[g][arc] (.x for the arc's top position, .y for its bottom position).
// A rotation multiplies the factor of both its rows by cos(theta) (scaled form) or by the sign
// (-1)^m of theta = theta' + m*pi (lifted form).  The product is carried in float64; D keeps it rounded
// to float32 (a relative 6e-8 on a coefficient that is itself rounded to float32 afterwards).  The
// angles of kScanAhead blocks are fetched before the dependent chain of multiplications starts, so the
// thread waits for memory once per kScanAhead blocks instead of once per block.
constexpr int kScanAhead = 16;
template <bool FWD>
__global__ void scaled_scan_kernel(int n, const float *__restrict__ theta, const int *__restrict__ map,
                                   int mirror, const unsigned *flag, float scaled_max, float *__restrict__ D,
                                   float *__restrict__ renorm)
{
    const int form = selected_form(flag, scaled_max);
    if (form == kFormStandard) return;
    const int H = n >> 1;
    const int nseg = (n - 1 + kRenormPeriod - 1) / kRenormPeriod;
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (long long)nseg * n) return;
    const int g = (int)(idx / n), r = (int)(idx % n);
    const int t0 = g * kRenormPeriod;
    const int t1 = (t0 + kRenormPeriod < n - 1) ? t0 + kRenormPeriod : n - 1;
    double d = 1.0;
    int q = 0, p = 0;
    // position of label r in the sequence of block k: 0 for r = 0, else 1 + (r - 1 + k) mod (n - 1); from one
    // block of the sweep to the next it moves by one place round the ring of positions 1 .. n-1
    const int k_first = FWD ? n - 2 - t0 : t0;
    int q_load = (r == 0) ? 0 : 1 + (r - 1 + k_first) % (n - 1);
    int q_use = q_load;
    auto advance = [&](int pos) {
        if (r == 0) return 0;
        if (FWD) return pos == 1 ? n - 1 : pos - 1;      // k goes down
        return pos == n - 1 ? 1 : pos + 1;               // k goes up
    };
    for (int tb = t0; tb < t1; tb += kScanAhead) {
        float th[kScanAhead];
#pragma unroll
        for (int u = 0; u < kScanAhead; ++u) {
            const int t = tb + u < t1 ? tb + u : t1 - 1;
            const int k = FWD ? n - 2 - t : t;
            const int pp = (q_load < H) ? q_load : n - 1 - q_load;
            th[u] = theta_at(theta, map, mirror, n, (long long)k * H + pp);
            if (tb + u < t1 - 1) q_load = advance(q_load);
        }
#pragma unroll
        for (int u = 0; u < kScanAhead; ++u) {
            const int t = tb + u;
            if (t < t1) {
                const int k = FWD ? n - 2 - t : t;
                q = q_use;
                p = (q < H) ? q : n - 1 - q;
                D[(long long)k * n + q] = (float)d;
                if (form == kFormScaled) {
                    d *= cos_small((double)th[u]);
                } else {
                    bool odd;
                    (void)lift_reduce((double)th[u], &odd);
                    d = odd ? -d : d;
                }
                q_use = advance(q_use);
            }
        }
        q_load = q_use;
    }
    renorm[2 * ((long long)g * H + p) + (q < H ? 0 : 1)] = (float)d;
}

// Step 2, and the only step of the standard form: the table of one sweep direction in E order, in the form
// the flag selects (flag == nullptr: standard).
//   standard: (cos, sin) with the orientation folded into the sine; `factor` (reverse sweep only) receives the
//     orientation sign (+1 when the top position holds the smaller label) that the dtheta reduction
//     multiplies its sums by.
//   scaled: (alpha, beta).  The same magnitudes serve both sweeps; the sweeps apply the signs (forward:
//     a - alpha b, b + beta a; reverse: a + alpha b, b - beta a), but the factors d differ between the two
//     directions, hence one scan per direction.  factor = orientation sign * d_top * d_bot: the sweep sums
//     stored values, and gbar_j z_i - gbar_i z_j = d_i d_j (g~_j z~_i - g~_i z~_j).
//   lifted: (T, S) = (tan(theta'/2), sin(theta')) * orientation * d_top * d_bot (the factors are +-1 here):
//     the forward sweep does a -= T b, b += S a, a -= T b on the stored values, the reverse sweep the same
//     with the signs flipped.
template <typename T>
__global__ void coef_table_kernel(int n, const T *__restrict__ theta, const int *__restrict__ map, int mirror,
                                  const unsigned *flag, float scaled_max, const float *__restrict__ D,
                                  typename Pair2<T>::type *__restrict__ table, T *__restrict__ factor)
{
    const int form = selected_form(flag, scaled_max);
    const int H = n >> 1;
    const long long N = (long long)(n - 1) * H;
    for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < N;
         e += (long long)gridDim.x * blockDim.x) {
        const int k = (int)(e / H), p = (int)(e % H);
        const int a = rr_label(n, k, p), b = rr_label(n, k, n - 1 - p);
        const double th = (double)theta_at(theta, map, mirror, n, e);
        const double orient = (a < b) ? 1.0 : -1.0;
        typename Pair2<T>::type out;
        double fac = orient;
        if (form == kFormStandard) {
            double s, c;
            sincos(th, &s, &c);
            out.x = (T)c;
            out.y = (T)(orient * s);
        } else {
            const double da = (double)D[(long long)k * n + p], db = (double)D[(long long)k * n + (n - 1 - p)]; // before this block
            fac = orient * da * db;
            if (form == kFormScaled) {
                const double s = orient * sin_small(th);
                const double c = cos_small(th);
                const double inv = s / (c * da * db);        // tan(theta) / (d_top d_bot)
                out.x = (T)(inv * db * db);
                out.y = (T)(inv * da * da);
            } else {
                bool odd;
                const double red = lift_reduce(th, &odd);
                double s, c;
                sincos(red, &s, &c);
                out.x = (T)(fac * s / (1.0 + c));            // tan(x/2) = sin x / (1 + cos x)
                out.y = (T)(fac * s);
            }
        }
        table[e] = out;
        if (factor) factor[e] = (T)fac;
    }
}

// ---- index map of a restricted parametrisation / odd n (Section 5; end of Section 3), built on the device.
// map[e] = index in theta of entry e of the full sequence E when its pair (i, j) is free (i < m and
// j < rows), else -1.  Three small kernels on the caller's stream: free pairs per block, exclusive scan
// over the blocks, then the positions inside each block.
__device__ __forceinline__ bool pair_is_free(int n, int rows, int m, int k, int p)
{
    const int a = rr_label(n, k, p), b = rr_label(n, k, n - 1 - p);
    const int i = a < b ? a : b, j = a < b ? b : a;
    return j < rows && i < m;
}
constexpr int kMapThreads = 256;
__global__ __launch_bounds__(kMapThreads) void map_count_kernel(int n, int rows, int m, int *__restrict__ counts)
{
    const int k = blockIdx.x, H = n >> 1;
    int c = 0;
    for (int p = threadIdx.x; p < H; p += kMapThreads) c += pair_is_free(n, rows, m, k, p) ? 1 : 0;
    for (int off = 32; off > 0; off >>= 1) c += __shfl_xor(c, off, 64);
    __shared__ int part[kMapThreads / 64];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = c;
    __syncthreads();
    if (threadIdx.x == 0) {
        int t = 0;
        for (int w = 0; w < kMapThreads / 64; ++w) t += part[w];
        counts[k] = t;
    }
}
// exclusive scan of counts[0 .. blocks) in place, one workgroup (blocks is at most a few ten thousand)
__global__ __launch_bounds__(kMapThreads) void map_scan_kernel(int blocks, int *__restrict__ counts)
{
    __shared__ int buf[kMapThreads];
    __shared__ int carry;
    if (threadIdx.x == 0) carry = 0;
    __syncthreads();
    for (int base = 0; base < blocks; base += kMapThreads) {
        const int i = base + threadIdx.x;
        const int v = i < blocks ? counts[i] : 0;
        buf[threadIdx.x] = v;
        __syncthreads();
        for (int off = 1; off < kMapThreads; off <<= 1) {  // inclusive scan of the chunk
            const int add = threadIdx.x >= off ? buf[threadIdx.x - off] : 0;
            __syncthreads();
            buf[threadIdx.x] += add;
            __syncthreads();
        }
        const int incl = buf[threadIdx.x], before = carry;
        if (i < blocks) counts[i] = before + incl - v;
        __syncthreads();
        if (threadIdx.x == kMapThreads - 1) carry = before + incl;
        __syncthreads();
    }
}
__global__ __launch_bounds__(kMapThreads) void map_fill_kernel(int n, int rows, int m, const int *__restrict__ offsets,
                                                               int *__restrict__ map)
{
    const int k = blockIdx.x, H = n >> 1;
    __shared__ int wave_count[kMapThreads / 64];
    __shared__ int carry;
    if (threadIdx.x == 0) carry = offsets[k];
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int base = 0; base < H; base += kMapThreads) {
        const int p = base + threadIdx.x;
        const bool is_free = p < H && pair_is_free(n, rows, m, k, p);
        const unsigned long long votes = __ballot(is_free);
        const int before_in_wave = __popcll(votes & ((1ull << lane) - 1ull));
        if (lane == 0) wave_count[wave] = __popcll(votes);
        __syncthreads();
        int before = carry;
        for (int w = 0; w < wave; ++w) before += wave_count[w];
        if (p < H) map[(long long)k * H + p] = is_free ? before + before_in_wave : -1;
        __syncthreads();
        if (threadIdx.x == 0) {
            int t = carry;
            for (int w = 0; w < kMapThreads / 64; ++w) t += wave_count[w];
            carry = t;
        }
        __syncthreads();
    }
}

// Second stage of the gradient reduction: dtheta[e] (+)= factor[e] * sum over strips s of
// partial[s][e], in strip order (fixed order: reproducible).  The sweeps store
// sum_b (g_bot z_top - g_top z_bot) of their stored values; `factor` carries the orientation sign
// (with i < j the paper's term is gbar_j z_i - gbar_i z_j) and, in the scaled form, d_top * d_bot.
// (factor == nullptr: 1).  `map` (see theta_at): dtheta lists the free angles only; sums of bypassed pairs are dropped.
// `poison` (may be null): a word the sweep sets when its chained rows could not be trusted; the result is then NaN.
template <typename T>
__global__ void reduce_partials_kernel(int n, long long nstrips, const T *__restrict__ partial,
                                       const T *__restrict__ factor, const int *__restrict__ map, T *dtheta,
                                       int accumulate, const unsigned *__restrict__ poison = nullptr)
{
    const int H = n >> 1;
    const long long N = (long long)(n - 1) * H;
    const long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= N) return;
    const long long out = map ? (long long)map[e] : e;
    if (out < 0) return;
    T a0 = T(0), a1 = T(0), a2 = T(0), a3 = T(0);
    long long s = 0;
    for (; s + 4 <= nstrips; s += 4) {          // four loads in flight; the order of additions is fixed
        a0 += partial[s * N + e];
        a1 += partial[(s + 1) * N + e];
        a2 += partial[(s + 2) * N + e];
        a3 += partial[(s + 3) * N + e];
    }
    for (; s < nstrips; ++s) a0 += partial[s * N + e];
    T acc = ((a0 + a1) + (a2 + a3)) * (factor ? factor[e] : T(1));
    if (poison && *poison) acc = T(__builtin_nanf(""));
    dtheta[out] = accumulate ? dtheta[out] + acc : acc;
}

// Before a reverse sweep with chained rows: the launch counter goes up by one and the per-launch words (XCD
// numbers, error word) go to zero.  kChainEpochLimit launches after the flags were last cleared the counter starts
// again at 1 and chain_flags_wrap_kernel, which runs just before, clears the flags (their tags would wrap).
constexpr unsigned kChainEpochLimit = 1u << 27;
__global__ void chain_flags_wrap_kernel(const unsigned *__restrict__ epoch, unsigned *__restrict__ flags, long long words)
{
    if (*epoch < kChainEpochLimit) return;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < words;
         i += (long long)gridDim.x * blockDim.x)
        flags[i] = 0u;
}
__global__ void chain_reset_kernel(unsigned *words, int count, unsigned *epoch)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) words[i] = 0u;
    if (i == 0) *epoch = (*epoch >= kChainEpochLimit) ? 1u : *epoch + 1u;
}

// The same sum for small problems, where one thread per angle leaves most of the chip idle behind a long chain of
// dependent loads (n = 256: 128 workgroups, 256 rows each): a workgroup takes 64 angles, its kReduceSplit groups of
// 64 threads each sum every kReduceSplit-th row, and the first group adds the group sums in a fixed order.
constexpr int kReduceSplit = 8;
template <typename T>
__global__ __launch_bounds__(64 * kReduceSplit) void reduce_partials_split_kernel(
    int n, long long nstrips, const T *__restrict__ partial, const T *__restrict__ factor,
    const int *__restrict__ map, T *dtheta, int accumulate)
{
    __shared__ T sums[kReduceSplit][64];
    const int H = n >> 1;
    const long long N = (long long)(n - 1) * H;
    const int lane = threadIdx.x & 63, group = threadIdx.x >> 6;
    const long long e = (long long)blockIdx.x * 64 + lane;
    T a0 = T(0), a1 = T(0);
    if (e < N) {
        long long s = group;
        for (; s + kReduceSplit < nstrips; s += 2 * kReduceSplit) {
            a0 += partial[s * N + e];
            a1 += partial[(s + kReduceSplit) * N + e];
        }
        if (s < nstrips) a0 += partial[s * N + e];
    }
    sums[group][lane] = a0 + a1;
    __syncthreads();
    if (group != 0 || e >= N) return;
    const long long out = map ? (long long)map[e] : e;
    if (out < 0) return;
    T acc = sums[0][lane];
#pragma unroll
    for (int g = 1; g < kReduceSplit; ++g) acc += sums[g][lane];
    acc *= factor ? factor[e] : T(1);
    dtheta[out] = accumulate ? dtheta[out] + acc : acc;
}

__global__ void fill_zero_kernel(long long count, float *__restrict__ dst)
{
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < count;
         i += (long long)gridDim.x * blockDim.x)
        dst[i] = 0.f;
}

} // namespace givens
