// Unitary extension (the paper's appendix "Adaptations to U(n)") in the register-carousel family, complex64.
//
// Factor of pair e = (i, j), i < j:  G_ii = w cos, G_ij = -sin, G_ji = w sin, G_jj = cos, w = exp(i phi), i.e.
// the real rotation of the pair times diag(w, 1).  A complex n x B operand with interleaved (re, im) is a real
// n x 2B operand, and the real rotation acts on re and im alike, so the real carousel kernel's data movement
// (carousel_kernels.hpp) serves unchanged; what is new is the phase.
//
// Carried phases.  Every row r is kept as y_r = exp(i a_r) * stored_r with a real angle a_r that depends on the
// angles alone, never on the data.  A real rotation may only mix two rows whose carried phases agree up to a
// sign, so before the rotation of a pair the kernel multiplies the row in the *top* position by
// exp(i psi'), where psi = (phase the top row must take on) - (phase it has), reduced to psi' in [-pi/2, pi/2]
// by a multiple of pi whose sign is folded into the rotation angle.  That multiply is itself a rotation of
// (re, im) and is done as three shears (3 FMA, like the lifted form of the real kernels); the real rotation
// follows as three shears on re and three on im: 9 FMA per (pair, complex column) in the forward sweep, against
// 12 for a rotation with complex coefficients.  Afterwards both rows carry the phase of the bottom row (plus
// phi when the bottom row is row i of the pair): the phase factor w never touches the data.  The signs (-1)^m
// of all angle reductions go into the carried phases too, so there is no renormalisation.  At the end every
// row is multiplied once by exp(i a_r).  Which row sits on top does not matter to the kernel: the choice to
// multiply the top row is free (it fixes which phase the pair inherits), which is what keeps the block body
// free of orientation-dependent code.
//
// The carried phases of a block depend on those of the block before through the partner row, so they are
// produced by a sequential pass over the n-1 blocks (unitary_phase_kernels.hpp): one workgroup, phases in LDS as
// 64-bit fixed-point fractions of a turn, one barrier per block; it writes psi' and the sign of the effective
// rotation angle per pair, and a parallel kernel turns these into the coefficient tables
//     rot[e] = (tan(theta'/2), sin theta'),   phs[e] = (tan(psi'/2), sin psi')
// with theta' the effective rotation angle reduced by a multiple of pi.
//
// Reverse sweep (gradients; operand-side form of the appendix's derivative entries, see unitary_kernels.hpp for
// the formulas on uncarried rows): two strips z (from Y) and g (from G) share the carried phases.  Per pair:
// multiply both top rows by exp(i psi'); the pair's share of dL/dtheta is then the real kernel's expression
// sum (g_bot z_top - g_top z_bot) over re and im (the common phase cancels), up to the sign the second stage
// applies; undo the real rotation; the share of dL/dphi is -Im sum conj(g_i) z_i on the un-rotated row i, which
// is the top or the bottom row -- both sums are formed and a per-pair 0/1 table picks one.  26 FMA per
// (pair, complex column).
#pragma once
#include <hip/hip_runtime.h>

#include <utility>

#include "carousel_kernels.hpp"

namespace givens {

// (a, b) <- rotation by the angle whose (tan(x/2), sin x) is (t, s), as three shears
__device__ __forceinline__ void shear3(float &a, float &b, float t, float s)
{
    a = fmaf(-t, b, a);
    b = fmaf(s, a, b);
    a = fmaf(-t, b, a);
}
// the transposed rotation
__device__ __forceinline__ void shear3_t(float &a, float &b, float t, float s)
{
    a = fmaf(t, b, a);
    b = fmaf(-s, a, b);
    a = fmaf(t, b, a);
}

// a row of W floats = W/2 complex numbers times (c, s) = exp(i a)
template <int W>
__device__ __forceinline__ void phase_row(float (&v)[W], float2 cs)
{
#pragma unroll
    for (int x = 0; x < W; x += 2) {
        const float re = v[x], im = v[x + 1];
        v[x] = fmaf(cs.x, re, -(cs.y * im));
        v[x + 1] = fmaf(cs.x, im, cs.y * re);
    }
}

// load_row of the real kernels with the complex identity: real column b0 + x of row `row` is 1 when it is
// the real part of complex column `row`
template <int W>
__device__ __forceinline__ void unitary_load_row(float (&dst)[W], const float *X, long long B, int row, int rows,
                                                 long long b0, int wv, bool vec, int identity)
{
    if (identity && (unsigned)row < (unsigned)rows) {
#pragma unroll
        for (int x = 0; x < W; ++x) dst[x] = (x < wv && b0 + x == 2 * (long long)row) ? 1.f : 0.f;
        return;
    }
    load_row<W>(dst, X, B, row, rows, b0, wv, vec, 0);
}

// ---------------------------------------------------------------------------------------------
// forward sweep: the structure of CarouselFwd (carousel_kernels.hpp) with two coefficient pairs per slot
// ---------------------------------------------------------------------------------------------
template <int M, int W, int WAVES>
struct UnitaryCarouselFwd {
    static_assert(W % 2 == 0, "a lane holds whole complex numbers");
    static constexpr int kLastU = (2 * M - 2) % M;

    float top[M][W];
    float bot[M][W];
    float2 rot[2][M], phs[2][M];
    int n, H, lane, wave, tid;
    const float2 *rot_lane, *phs_lane; // tables + tid*M
    float *out_top, *out_bot, *turn;
    const float *in_top, *in_bot;
    static constexpr int kBufFloats = (int)(sizeof(typename CarouselExchange<W, WAVES>::Buf) / sizeof(float));

    __device__ __forceinline__ void load_pairs(const float2 *base, int k, float2 (&dst)[M])
    {
        const float2 *src = base + (long long)k * H;
        if constexpr (M % 2 == 0) {
            const float4 *s4 = reinterpret_cast<const float4 *>(src);
#pragma unroll
            for (int r = 0; r < M / 2; ++r) {
                const float4 v = s4[r];
                dst[2 * r] = make_float2(v.x, v.y);
                dst[2 * r + 1] = make_float2(v.z, v.w);
            }
        } else {
#pragma unroll
            for (int r = 0; r < M; ++r) dst[r] = src[r];
        }
    }
    __device__ __forceinline__ void load_coefs(int k, int buf)
    {
        load_pairs(rot_lane, k, rot[buf]);
        load_pairs(phs_lane, k, phs[buf]);
    }

    // logical slot R under the register map of unrolled copy U: phase turn of the top row, then the rotation
    template <int U, int R>
    __device__ __forceinline__ void rotate_slot(const float2 (&cr)[M], const float2 (&cp)[M])
    {
        constexpr int it = (R + U) % M, ib = (R - U + M) % M;
        const float t = cr[R].x, s = cr[R].y, pt = cp[R].x, ps = cp[R].y;
#pragma unroll
        for (int x = 0; x < W; x += 2) {
            float re = top[it][x], im = top[it][x + 1];
            shear3(re, im, pt, ps);
            shear3(re, bot[ib][x], t, s);
            shear3(im, bot[ib][x + 1], t, s);
            top[it][x] = re;
            top[it][x + 1] = im;
        }
#pragma unroll
        for (int x = 0; x < W; ++x) asm volatile("" : "+v"(top[it][x]), "+v"(bot[ib][x]));
    }
    template <int U, int FIRST, int... Rs>
    __device__ __forceinline__ void rotate_inner(const float2 (&cr)[M], const float2 (&cp)[M],
                                                 std::integer_sequence<int, Rs...>)
    {
        (rotate_slot<U, FIRST + Rs>(cr, cp), ...);
    }

    template <int U, bool LAST>
    __device__ __forceinline__ void step(int k)
    {
        float2(&cr)[M] = rot[U & 1];
        float2(&cp)[M] = phs[U & 1];
        if constexpr (!LAST) load_coefs(k - 1, (U + 1) & 1);

        constexpr int kInner = M > 3 ? M - 3 : 0;
        constexpr int kInnerA = (kInner + 1) / 2;
        if constexpr (kInnerA > 0) rotate_inner<U, 2>(cr, cp, std::make_integer_sequence<int, kInnerA>{});

        __builtin_amdgcn_s_setprio(2);
        rotate_slot<U, 0>(cr, cp);
        if constexpr (M > 1) rotate_slot<U, M - 1>(cr, cp);
        if constexpr (M > 2) rotate_slot<U, 1>(cr, cp);

        constexpr int q = U % M;
        constexpr int qb = (M - 1 - U + M) % M;
        constexpr int q1 = (1 + U) % M;
        constexpr int par = U & 1;
        if constexpr (!LAST) {
            lds_store_row<W, WAVES>(out_top + par * kBufFloats, top[q]);
            lds_store_row<W, WAVES>(out_bot + par * kBufFloats, bot[qb]);
            if (wave == 0) {
                if (lane == 0) lds_store_row<W, WAVES>(turn + par * kBufFloats, top[q1]);
#pragma unroll
                for (int x = 0; x < W; ++x) {
                    const float held = top[q][x], other = top[q1][x];
                    top[q1][x] = (lane == 0) ? held : other;
                }
            }
        }
        __builtin_amdgcn_s_setprio(0);
        if constexpr (kInner - kInnerA > 0)
            rotate_inner<U, 2 + kInnerA>(cr, cp, std::make_integer_sequence<int, kInner - kInnerA>{});

        if constexpr (!LAST) {
            __syncthreads();
            lds_load_row<W, WAVES>(top[q], in_top + par * kBufFloats);
            lds_load_row<W, WAVES>(bot[qb], in_bot + par * kBufFloats);
        }
    }

    template <int... Us>
    __device__ __forceinline__ void full_group(int k_first, std::integer_sequence<int, Us...>)
    {
        (step<Us, false>(k_first - Us), ...);
    }
    template <int... Us>
    __device__ __forceinline__ void tail_group(std::integer_sequence<int, Us...>)
    {
        (step<Us, Us == M - 2>(M - 2 - Us), ...);
    }
    __device__ __forceinline__ void sweep()
    {
        constexpr auto seq = std::make_integer_sequence<int, M>{};
        int k = n - 2;
        for (; k >= M - 1; k -= M) full_group(k, seq);
        tail_group(std::make_integer_sequence<int, M - 1>{});
    }
};

// X, Y: the complex operand as floats (row stride Breal = 2 B floats); fin: final phase per row.
template <int M, int W, int WAVES>
__global__ __launch_bounds__(64 * WAVES, 2) void unitary_carousel_forward_kernel(
    int n, long long Breal, const float2 *__restrict__ rot, const float2 *__restrict__ phs,
    const float2 *__restrict__ fin, const float *X, float *Y, int identity, int vec_ok)
{
    __shared__ CarouselExchange<W, WAVES> sh;
    using State = UnitaryCarouselFwd<M, W, WAVES>;
    State st;
    const int L = n / (2 * M);
    const bool idle = (int)threadIdx.x >= L;
    const int coef_lane = idle ? 0 : (int)threadIdx.x;
    const int my_rows = idle ? 0 : n;
    st.n = n;
    st.H = n >> 1;
    st.tid = threadIdx.x;
    st.lane = threadIdx.x & 63;
    st.wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    st.rot_lane = rot + (long long)coef_lane * M;
    st.phs_lane = phs + (long long)coef_lane * M;
    {
        constexpr int LMAX = 64 * WAVES;
        auto &b = sh.buf[0];
        const int t = threadIdx.x;
        st.out_top = b.top_out.lane(t);
        st.out_bot = b.bot_out.lane(t);
        st.turn = b.top_out.lane(LMAX);
        st.in_top = (t < L - 1) ? b.top_out.lane(t + 1) : b.bot_out.lane(L - 1);
        st.in_bot = (t > 0) ? b.bot_out.lane(t - 1) : b.top_out.lane(LMAX);
    }
    const long long b0 = (long long)blockIdx.x * W;
    const int wv = (Breal - b0) < W ? (int)(Breal - b0) : W;
    const bool vec = vec_ok && wv == W;

#pragma unroll
    for (int r = 0; r < M; ++r) {
        const int p = st.tid * M + r;
        unitary_load_row<W>(st.top[r], X, Breal, rr_label(n, n - 2, p), my_rows, b0, wv, vec, identity);
        unitary_load_row<W>(st.bot[r], X, Breal, rr_label(n, n - 2, n - 1 - p), my_rows, b0, wv, vec, identity);
    }
    st.load_coefs(n - 2, 0);

    st.sweep();

    // identity position order now: position p holds row p; give every row its carried phase back
    constexpr int UL = State::kLastU;
#pragma unroll
    for (int r = 0; r < M; ++r) {
        const int p = st.tid * M + r;
        if (!idle) {
            phase_row<W>(st.top[(r + UL) % M], fin[p]);
            phase_row<W>(st.bot[(r - UL + M) % M], fin[n - 1 - p]);
        }
        store_row<W>(st.top[(r + UL) % M], Y, Breal, p, my_rows, b0, wv, vec);
        store_row<W>(st.bot[(r - UL + M) % M], Y, Breal, n - 1 - p, my_rows, b0, wv, vec);
    }
}

// ---------------------------------------------------------------------------------------------
// reverse sweep: the structure of CarouselBwd with two coefficient pairs, a 0/1 and two sums per slot
// ---------------------------------------------------------------------------------------------
template <int M, int W, int WAVES>
struct UnitaryCarouselBwd {
    static_assert(W % 2 == 0, "a lane holds whole complex numbers");
    static constexpr int kLastU = (2 * M - 2) % M;

    float zt[M][W], zb[M][W], gt[M][W], gb[M][W];
    float2 rot[2][M], phs[2][M];
    float ori[2][M];
    float prior_t[2][M], prior_p[2][M]; // sums of this workgroup's earlier strips (dtheta, dphi), current / next block
    int n, H, lane, wave, tid;
    const float2 *rot_lane, *phs_lane;
    const float *ori_lane;
    float *part_t, *part_p;             // this workgroup's rows of partial sums + tid*M (idle lanes: the sink)
    const float *prior_t_lane, *prior_p_lane;
    float *out_top, *out_bot, *hold;
    const float *in_top, *in_bot;
    static constexpr int kStripFloats = (int)(sizeof(typename CarouselExchangeBwd<W, WAVES>::Strip) / sizeof(float));
    static constexpr int kBufFloats = (int)(sizeof(typename CarouselExchangeBwd<W, WAVES>::Buf) / sizeof(float));

    __device__ __forceinline__ void load_pairs(const float2 *base, int k, float2 (&dst)[M])
    {
        const float2 *src = base + (long long)k * H;
        if constexpr (M % 2 == 0) {
            const float4 *s4 = reinterpret_cast<const float4 *>(src);
#pragma unroll
            for (int r = 0; r < M / 2; ++r) {
                const float4 v = s4[r];
                dst[2 * r] = make_float2(v.x, v.y);
                dst[2 * r + 1] = make_float2(v.z, v.w);
            }
        } else {
#pragma unroll
            for (int r = 0; r < M; ++r) dst[r] = src[r];
        }
    }
    __device__ __forceinline__ void load_floats(const float *base, int k, float (&dst)[M])
    {
        const float *src = base + (long long)k * H;
        if constexpr (M % 4 == 0) {
#pragma unroll
            for (int r = 0; r < M / 4; ++r) {
                const float4 v = reinterpret_cast<const float4 *>(src)[r];
                dst[4 * r] = v.x; dst[4 * r + 1] = v.y; dst[4 * r + 2] = v.z; dst[4 * r + 3] = v.w;
            }
        } else if constexpr (M % 2 == 0) {
#pragma unroll
            for (int r = 0; r < M / 2; ++r) {
                const float2 v = reinterpret_cast<const float2 *>(src)[r];
                dst[2 * r] = v.x; dst[2 * r + 1] = v.y;
            }
        } else {
#pragma unroll
            for (int r = 0; r < M; ++r) dst[r] = src[r];
        }
    }
    __device__ __forceinline__ void store_floats(float *base, int k, const float (&src)[M])
    {
        float *dst = base + (long long)k * H;
        if constexpr (M % 4 == 0) {
#pragma unroll
            for (int r = 0; r < M / 4; ++r)
                reinterpret_cast<float4 *>(dst)[r] = make_float4(src[4 * r], src[4 * r + 1], src[4 * r + 2], src[4 * r + 3]);
        } else if constexpr (M % 2 == 0) {
#pragma unroll
            for (int r = 0; r < M / 2; ++r) reinterpret_cast<float2 *>(dst)[r] = make_float2(src[2 * r], src[2 * r + 1]);
        } else {
#pragma unroll
            for (int r = 0; r < M; ++r) dst[r] = src[r];
        }
    }
    __device__ __forceinline__ void load_coefs(int k, int buf)
    {
        load_pairs(rot_lane, k, rot[buf]);
        load_pairs(phs_lane, k, phs[buf]);
        load_floats(ori_lane, k, ori[buf]);
    }
    __device__ __forceinline__ void load_prior(int k, int buf)
    {
        load_floats(prior_t_lane, k, prior_t[buf]);
        load_floats(prior_p_lane, k, prior_p[buf]);
    }

    template <int U, int WHICH>
    __device__ __forceinline__ void publish(float (&t)[M][W], float (&b)[M][W])
    {
        constexpr int qt = (M - 1 - U + M) % M;
        constexpr int qb = U % M;
        constexpr int pf = (M - U) % M;
        constexpr int off = (U & 1) * kBufFloats + WHICH * kStripFloats;
        lds_store_row<W, WAVES>(out_top + off, t[qt]);
        lds_store_row<W, WAVES>(out_bot + off, b[qb]);
        if (wave == 0 && lane == 0) lds_store_row<W, WAVES>(hold + off, t[pf]);
    }
    template <int U, int WHICH>
    __device__ __forceinline__ void receive(float (&t)[M][W], float (&b)[M][W])
    {
        constexpr int qt = (M - 1 - U + M) % M;
        constexpr int qb = U % M;
        constexpr int pf = (M - U) % M;
        constexpr int off = (U & 1) * kBufFloats + WHICH * kStripFloats;
        if (wave == 0) {
#pragma unroll
            for (int x = 0; x < W; ++x) {
                const float turn = b[qb][x], keep = t[pf][x];
                t[pf][x] = (lane == 0) ? turn : keep;
            }
        }
        lds_load_row<W, WAVES>(t[qt], in_top + off);
        lds_load_row<W, WAVES>(b[qb], in_bot + off);
    }

    // logical slot R of one block; returns the strip's share of the pair's dtheta (up to its sign) and dphi
    template <int U, int R>
    __device__ __forceinline__ void sweep_slot(const float2 (&cr)[M], const float2 (&cp)[M], const float (&co)[M],
                                               float &sum_t, float &sum_p)
    {
        constexpr int it = (R - U + M) % M, ib = (R + U) % M;
        const float t = cr[R].x, s = cr[R].y, pt = cp[R].x, ps = cp[R].y;
        float acc = 0.f, dtop = 0.f, dbot = 0.f;
#pragma unroll
        for (int x = 0; x < W; x += 2) {
            float zr = zt[it][x], zi = zt[it][x + 1], gr = gt[it][x], gi = gt[it][x + 1];
            float zvr = zb[ib][x], zvi = zb[ib][x + 1], gvr = gb[ib][x], gvi = gb[ib][x + 1];
            shear3(zr, zi, pt, ps);
            shear3(gr, gi, pt, ps);
            acc = fmaf(gvr, zr, acc);
            acc = fmaf(-gr, zvr, acc);
            acc = fmaf(gvi, zi, acc);
            acc = fmaf(-gi, zvi, acc);
            shear3_t(zr, zvr, t, s);
            shear3_t(zi, zvi, t, s);
            shear3_t(gr, gvr, t, s);
            shear3_t(gi, gvi, t, s);
            dtop = fmaf(gi, zr, dtop);     // -Im conj(g) z = g.im z.re - g.re z.im
            dtop = fmaf(-gr, zi, dtop);
            dbot = fmaf(gvi, zvr, dbot);
            dbot = fmaf(-gvr, zvi, dbot);
            zt[it][x] = zr; zt[it][x + 1] = zi; gt[it][x] = gr; gt[it][x + 1] = gi;
            zb[ib][x] = zvr; zb[ib][x + 1] = zvi; gb[ib][x] = gvr; gb[ib][x + 1] = gvi;
            if ((x & 3) == 2 || x == W - 2) {
#pragma unroll
                for (int y = x & ~3; y <= x + 1; ++y)
                    asm volatile("" : "+v"(zt[it][y]), "+v"(zb[ib][y]), "+v"(gt[it][y]), "+v"(gb[ib][y]), "+v"(acc),
                                 "+v"(dtop), "+v"(dbot));
            }
        }
        sum_t = acc;
        sum_p = fmaf(co[R], dtop - dbot, dbot);   // co is 1 (row i on top) or 0
    }
    template <int U, int FIRST, int... Rs>
    __device__ __forceinline__ void sweep_inner(const float2 (&cr)[M], const float2 (&cp)[M], const float (&co)[M],
                                                float (&st)[M], float (&sp)[M], std::integer_sequence<int, Rs...>)
    {
        (sweep_slot<U, FIRST + Rs>(cr, cp, co, st[FIRST + Rs], sp[FIRST + Rs]), ...);
    }

    template <int U, bool LAST>
    __device__ __forceinline__ void step(int k)
    {
        float2(&cr)[M] = rot[U & 1];
        float2(&cp)[M] = phs[U & 1];
        float(&co)[M] = ori[U & 1];
        if constexpr (!LAST) load_coefs(k + 1, (U + 1) & 1);
        float(&earlier_t)[M] = prior_t[U & 1];
        float(&earlier_p)[M] = prior_p[U & 1];
        if constexpr (!LAST) load_prior(k + 1, (U + 1) & 1);

        float st[M], sp[M];
        constexpr int kInner = M > 2 ? M - 2 : 0;
        __builtin_amdgcn_s_setprio(2);
        sweep_slot<U, 0>(cr, cp, co, st[0], sp[0]);
        if constexpr (M > 1) sweep_slot<U, M - 1>(cr, cp, co, st[M - 1], sp[M - 1]);
        if constexpr (!LAST) {
            publish<U, 0>(zt, zb);
            publish<U, 1>(gt, gb);
        }
        __builtin_amdgcn_s_setprio(0);
        if constexpr (kInner > 0) sweep_inner<U, 1>(cr, cp, co, st, sp, std::make_integer_sequence<int, kInner>{});
#pragma unroll
        for (int r = 0; r < M; ++r) {
            st[r] += earlier_t[r];
            sp[r] += earlier_p[r];
        }
        store_floats(part_t, k, st);
        store_floats(part_p, k, sp);
        if constexpr (!LAST) {
            __syncthreads();
            receive<U, 0>(zt, zb);
            receive<U, 1>(gt, gb);
        }
    }

    template <int... Us>
    __device__ __forceinline__ void full_group(int k_first, std::integer_sequence<int, Us...>)
    {
        (step<Us, false>(k_first + Us), ...);
    }
    template <int... Us>
    __device__ __forceinline__ void tail_group(int k_first, std::integer_sequence<int, Us...>)
    {
        (step<Us, Us == M - 2>(k_first + Us), ...);
    }
    __device__ __forceinline__ void sweep()
    {
        constexpr auto seq = std::make_integer_sequence<int, M>{};
        load_prior(0, 0);
        int k = 0;
        for (; k + M <= n - 1; k += M) full_group(k, seq);
        tail_group(k, std::make_integer_sequence<int, M - 1>{});
    }
};

// partial: [2][gridDim.x][N] floats: the dtheta rows of the persistent workgroups, then their dphi rows.
template <int M, int W, int WAVES>
__global__ __launch_bounds__(64 * WAVES, 2) void unitary_carousel_backward_kernel(
    int n, long long Breal, long long strip0, long long nstrips, const float2 *__restrict__ rot,
    const float2 *__restrict__ phs, const float *__restrict__ orient, const float2 *__restrict__ fin, const float *Yin,
    const float *G, float *dX, float *partial, const float *__restrict__ zeros, float *sink, int vec_ok)
{
    __shared__ CarouselExchangeBwd<W, WAVES> sh;
    using State = UnitaryCarouselBwd<M, W, WAVES>;
    State st;
    const int L = n / (2 * M);
    const bool idle = (int)threadIdx.x >= L;
    const int coef_lane = idle ? 0 : (int)threadIdx.x;
    const int my_rows = idle ? 0 : n;
    const long long N = (long long)(n - 1) * (n >> 1);
    st.n = n;
    st.H = n >> 1;
    st.tid = threadIdx.x;
    st.lane = threadIdx.x & 63;
    st.wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    st.rot_lane = rot + (long long)coef_lane * M;
    st.phs_lane = phs + (long long)coef_lane * M;
    st.ori_lane = orient + (long long)coef_lane * M;
    st.part_t = idle ? sink + (long long)threadIdx.x * M : partial + (long long)blockIdx.x * N + (long long)threadIdx.x * M;
    st.part_p = idle ? st.part_t : st.part_t + (long long)gridDim.x * N;
    {
        constexpr int LMAX = 64 * WAVES;
        auto &z = sh.buf[0].strip[0];
        const int t = threadIdx.x;
        st.out_top = z.top_out.lane(t);
        st.out_bot = z.bot_out.lane(t);
        st.hold = z.top_out.lane(LMAX);
        st.in_top = (t > 0) ? z.top_out.lane(t - 1) : z.top_out.lane(LMAX);
        st.in_bot = (t < L - 1) ? z.bot_out.lane(t + 1) : z.top_out.lane(L - 1);
    }

    for (long long s = blockIdx.x; s < nstrips; s += gridDim.x) {
        const bool first_strip = (s == (long long)blockIdx.x);
        st.prior_t_lane = first_strip ? zeros + (long long)coef_lane * M : st.part_t;
        st.prior_p_lane = first_strip ? zeros + (long long)coef_lane * M : st.part_p;
        const long long b0 = (strip0 + s) * W;
        const int wv = (Breal - b0) < W ? (int)(Breal - b0) : W;
        const bool vec = vec_ok && wv == W;
#pragma unroll
        for (int r = 0; r < M; ++r) {
            const int p = st.tid * M + r;
            load_row<W>(st.zt[r], Yin, Breal, p, my_rows, b0, wv, vec, 0);
            load_row<W>(st.zb[r], Yin, Breal, n - 1 - p, my_rows, b0, wv, vec, 0);
            load_row<W>(st.gt[r], G, Breal, p, my_rows, b0, wv, vec, 0);
            load_row<W>(st.gb[r], G, Breal, n - 1 - p, my_rows, b0, wv, vec, 0);
        }
        st.load_coefs(0, 0);

        st.sweep();

        if (dX) {
            constexpr int UL = State::kLastU;
#pragma unroll
            for (int r = 0; r < M; ++r) {
                const int p = st.tid * M + r;
                const int row_t = rr_label(n, n - 2, p), row_b = rr_label(n, n - 2, n - 1 - p);
                if (!idle) {
                    phase_row<W>(st.gt[(r - UL + M) % M], fin[row_t]);
                    phase_row<W>(st.gb[(r + UL) % M], fin[row_b]);
                }
                store_row<W>(st.gt[(r - UL + M) % M], dX, Breal, row_t, my_rows, b0, wv, vec);
                store_row<W>(st.gb[(r + UL) % M], dX, Breal, row_b, my_rows, b0, wv, vec);
            }
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------------------------
// launches (instantiated by unitary_carousel_fwd.hip / unitary_carousel_bwd.hip)
// ---------------------------------------------------------------------------------------------
template <int M, int W, int WAVES>
inline void unitary_carousel_launch_fwd(const UnitaryCarouselFwdArgs &a)
{
    const long long strips = (a.Breal + W - 1) / W;
    hipLaunchKernelGGL((unitary_carousel_forward_kernel<M, W, WAVES>), dim3((unsigned)strips), dim3(64 * WAVES), 0,
                       a.stream, a.n, a.Breal, a.rot, a.phs, a.fin, a.X, a.Y, a.identity, a.vec_ok);
}
template <int M, int WAVES>
inline int unitary_carousel_fwd_widths(int W, const UnitaryCarouselFwdArgs &a)
{
    switch (W) {
    case 8: unitary_carousel_launch_fwd<M, 8, WAVES>(a); return GIVENS_OK;
    case 4: unitary_carousel_launch_fwd<M, 4, WAVES>(a); return GIVENS_OK;
    case 2: unitary_carousel_launch_fwd<M, 2, WAVES>(a); return GIVENS_OK;
    default: return GIVENS_ERR_UNSUPPORTED;
    }
}
template <int M>
inline int unitary_carousel_forward_slots(const UnitaryCarouselFwdArgs &a, int waves, int W)
{
    switch (waves) {
    case 1: return unitary_carousel_fwd_widths<M, 1>(W, a);
    case 2: return unitary_carousel_fwd_widths<M, 2>(W, a);
    case 3: return unitary_carousel_fwd_widths<M, 3>(W, a);
    case 4: return unitary_carousel_fwd_widths<M, 4>(W, a);
    case 5: return unitary_carousel_fwd_widths<M, 5>(W, a);
    case 6: return unitary_carousel_fwd_widths<M, 6>(W, a);
    case 7: return unitary_carousel_fwd_widths<M, 7>(W, a);
    case 8: return unitary_carousel_fwd_widths<M, 8>(W, a);
    default: return GIVENS_ERR_UNSUPPORTED;
    }
}

template <int M, int W, int WAVES>
inline void unitary_carousel_launch_bwd(const UnitaryCarouselBwdArgs &a)
{
    hipLaunchKernelGGL((unitary_carousel_backward_kernel<M, W, WAVES>), dim3((unsigned)a.groups), dim3(64 * WAVES), 0,
                       a.stream, a.n, a.Breal, a.strip0, a.nstrips, a.rot, a.phs, a.orient, a.fin, a.Y, a.G, a.dX,
                       a.partial, a.zeros, a.sink, a.vec_ok);
}
template <int M, int WAVES>
inline int unitary_carousel_bwd_widths(int W, const UnitaryCarouselBwdArgs &a)
{
    // with 4 slots per lane, 8 floats per slot and strip would need more registers than a lane has (it compiles
    // with 340 bytes of scratch); with 2 slots they fit
    if constexpr (M == 2)
        if (W == 8) {
            unitary_carousel_launch_bwd<M, 8, WAVES>(a);
            return GIVENS_OK;
        }
    switch (W) {
    case 4: unitary_carousel_launch_bwd<M, 4, WAVES>(a); return GIVENS_OK;
    case 2: unitary_carousel_launch_bwd<M, 2, WAVES>(a); return GIVENS_OK;
    default: return GIVENS_ERR_UNSUPPORTED;
    }
}
template <int M>
inline int unitary_carousel_backward_slots(const UnitaryCarouselBwdArgs &a, int waves, int W)
{
    switch (waves) {
    case 1: return unitary_carousel_bwd_widths<M, 1>(W, a);
    case 2: return unitary_carousel_bwd_widths<M, 2>(W, a);
    case 3: return unitary_carousel_bwd_widths<M, 3>(W, a);
    case 4: return unitary_carousel_bwd_widths<M, 4>(W, a);
    case 5: return unitary_carousel_bwd_widths<M, 5>(W, a);
    case 6: return unitary_carousel_bwd_widths<M, 6>(W, a);
    case 7: return unitary_carousel_bwd_widths<M, 7>(W, a);
    case 8: return unitary_carousel_bwd_widths<M, 8>(W, a);
    default: return GIVENS_ERR_UNSUPPORTED;
    }
}

} // namespace givens
