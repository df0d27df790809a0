// Register-carousel kernels (float): the fast family for n = 2 * M * L with M slots per lane and L lanes,
// L <= 64 * WAVES (when L is not a multiple of 64 the last wavefront's spare lanes idle: they carry
// zeros, read lane 0's coefficients and write their sums to a sink).
//
// Idea.  The circle method (paper Section 3, Figure 1) keeps a line of n positions; block k
// pairs position p with position n-1-p, and between blocks the labels move one position along
// a ring of n-1 positions while position 0 is held.  So instead of moving pairings around, the
// kernel keeps the strip of the operand *in position order* and folded in two:
//
//     top[p] = row sitting at position p,      bot[p] = row sitting at position n-1-p,
//
// p = 0..n/2-1.  Every block then rotates (top[p], bot[p]) for all p -- the partner is always in
// the same lane -- and the step to the next block is a carousel move: the top line shifts by one
// slot in one direction, the bottom line by one slot in the other direction, with a turn-around at
// the far end (top[n/2-1] <-> bot[n/2-1]) and at the near end (top[1] <-> bot[0]); top[0] stays.
//
// Mapping.  A workgroup of L = 64*WAVES lanes owns W columns of the operand for all n-1 blocks
// (one HBM read, one HBM write).  Lane l holds slots p = l*M .. l*M+M-1 of both lines, W columns
// each, in VGPRs: 2*M*W floats.  The carousel move only changes one slot per lane per line: the
// slot that leaves goes to the neighbouring lane through LDS, and the other M-1 slots are "moved"
// by renaming: the round loop is unrolled M times so that the slot <-> register map is static in
// every copy of the body.
// cos/sin come from the table written by coef_table_kernel, M pairs per lane per block, reused
// for the W columns the lane holds and prefetched one block ahead.
//
// Forward (Algorithm 2 from operand X) walks blocks k = n-2 .. 0, so the strip is loaded in the
// position order of block n-1 and ends in the order of block 1, which is the identity order.
#pragma once
#include <hip/hip_runtime.h>

#include <type_traits>
#include <utility>

#include "../../include/givens_rr.h"
#include "carousel_host.hpp"
#include "forms.hpp"
#include "rr_index.h"

namespace givens {

// How the slots that leave a lane reach the neighbouring lane.
//   kExchangeLds:  through LDS, for every lane (any number of wavefronts); one barrier per block.
//   kExchangeWave: with DPP wavefront shifts, for workgroups of one wavefront.  No LDS, no barrier, and a chain of
//                  a few cycles from one block to the next instead of an LDS write, a barrier and an LDS read.
//                  Each move costs VALU issue slots (two shifts and one or two selects per column), so it is
//                  the choice where a sweep is bound by that chain and not by arithmetic: few, narrow strips.
enum { kExchangeLds = 0, kExchangeWave = 1 };
// Coefficients (and the reverse sweep's earlier sums) are fetched ahead into a ring of registers: one block ahead
// where the LDS exchange sets the pace of a block anyway, three or seven blocks ahead with the wavefront exchange,
// whose blocks are shorter than a load's latency (a ring of 2 left those sweeps at one L2 latency per block: n = 256,
// 64 columns, forward 38 us; ring of 4: 22 us; ring of 8: 15 us).
// (ring slots are static, so the unrolled group has lcm(M, depth) copies and n must be a multiple of that: 8 here)
constexpr int wave_ring_depth_fwd(int M) { return M == 8 ? 4 : 8; }
constexpr int wave_ring_depth_bwd(int M) { return M == 2 ? 8 : 4; }
constexpr int carousel_lcm(int a, int b)
{
    int x = a, y = b;
    while (y) { const int t = x % y; x = y; y = t; }
    return a / x * b;
}

// lane l receives the value of lane l+1; lane 63 (no source) keeps `incoming`
__device__ __forceinline__ float lane_from_next(float incoming, float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(incoming), __float_as_int(v),
                                                      0x130 /* wave_shl:1 */, 0xf, 0xf, false));
}
// lane l receives the value of lane l-1; lane 0 (no source) keeps `incoming`
__device__ __forceinline__ float lane_from_prev(float incoming, float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(incoming), __float_as_int(v),
                                                      0x138 /* wave_shr:1 */, 0xf, 0xf, false));
}

// The carousel move goes through LDS for every lane: each lane writes the slot that leaves its top
// line and the slot that leaves its bottom line, and after the barrier reads its neighbours'.  This
// costs LDS bandwidth (2*W floats written and read per lane per block), which is otherwise idle,
// instead of VALU issue slots (DPP moves), which are the bottleneck, and it needs no special case at
// wavefront boundaries.  One buffer per block parity, so one barrier per block is enough.
//
// Layout of one exchange line (L lanes plus one extra row for the element that turns round at the
// near end): when W is a multiple of 4 a lane's W floats are split into 16-byte chunks and chunk c of
// lane l sits at float offset (c*(L+1) + l)*4, so that a wavefront's ds_*_b128 touches consecutive
// 16-byte words (no bank conflicts; a [lane][W] layout with W = 8 had two-way conflicts on every
// access).  Otherwise the W floats of a lane are contiguous.
template <int W, int WAVES>
struct CarouselLine {
    static constexpr int kLanes = 64 * WAVES;
    static constexpr int kLaneStride = (W % 4 == 0) ? 4 : W;   // floats between neighbouring lanes
    static constexpr int kChunkStride = (kLanes + 1) * 4;      // floats between a lane's chunks
    alignas(16) float data[(kLanes + 1) * W];
    __device__ __forceinline__ float *lane(int l) { return data + l * kLaneStride; }
};
template <int W, int WAVES>
struct CarouselExchange {
    struct Buf {
        CarouselLine<W, WAVES> top_out; // per lane: the top slot that leaves; extra row: the near-end turn
        CarouselLine<W, WAVES> bot_out; // per lane: the bottom slot that leaves
    };
    Buf buf[2];
};

// a lane's W floats to / from its place in an exchange line
template <int W, int WAVES>
__device__ __forceinline__ void lds_store_row(float *dst, const float (&src)[W])
{
    if constexpr (W % 4 == 0) {
#pragma unroll
        for (int c = 0; c < W / 4; ++c)
            *reinterpret_cast<float4 *>(dst + c * CarouselLine<W, WAVES>::kChunkStride) =
                make_float4(src[4 * c], src[4 * c + 1], src[4 * c + 2], src[4 * c + 3]);
    } else if constexpr (W % 2 == 0) {
#pragma unroll
        for (int x = 0; x < W / 2; ++x) reinterpret_cast<float2 *>(dst)[x] = make_float2(src[2 * x], src[2 * x + 1]);
    } else {
#pragma unroll
        for (int x = 0; x < W; ++x) dst[x] = src[x];
    }
}
template <int W, int WAVES>
__device__ __forceinline__ void lds_load_row(float (&dst)[W], const float *src)
{
    if constexpr (W % 4 == 0) {
#pragma unroll
        for (int c = 0; c < W / 4; ++c) {
            const float4 v = *reinterpret_cast<const float4 *>(src + c * CarouselLine<W, WAVES>::kChunkStride);
            dst[4 * c] = v.x; dst[4 * c + 1] = v.y; dst[4 * c + 2] = v.z; dst[4 * c + 3] = v.w;
        }
    } else if constexpr (W % 2 == 0) {
#pragma unroll
        for (int x = 0; x < W / 2; ++x) {
            const float2 v = reinterpret_cast<const float2 *>(src)[x];
            dst[2 * x] = v.x; dst[2 * x + 1] = v.y;
        }
    } else {
#pragma unroll
        for (int x = 0; x < W; ++x) dst[x] = src[x];
    }
}

// FORM 0: standard rotation (2 MUL + 2 FMA per update, table holds cos and sin).
// FORM 1: scaled rotation (2 FMA per update on values kept divided by their accumulated cosines,
//         table holds alpha and beta, renormalisation every kRenormPeriod blocks; coef_kernels.hpp).
// FORM 2: lifted rotation (3 dependent FMA per update: three shears; table holds tan(theta'/2) and
//         sin(theta') with the carried signs folded in; same renormalisation points, factors +-1).
template <int M, int W, int WAVES, int FORM, int EX = kExchangeLds>
struct CarouselFwd {
    static_assert(EX == kExchangeLds || WAVES == 1, "the DPP exchange stays inside one wavefront");
    // copies of the block body in one unrolled group: a multiple of M (static register map) and of the ring depth
    // (static ring slot; the LDS exchange buffers alternate by block parity), so an odd M unrolls 2 M times
    static constexpr int kDepth = EX == kExchangeWave ? wave_ring_depth_fwd(M) : 2;
    static constexpr int kUnroll = carousel_lcm(M, kDepth);
    static_assert(FORM == 0 || kRenormPeriod % kUnroll == 0,
                  "renormalisation must fall on the last copy of an unrolled group");
    static constexpr int kLastU = (2 * M - 2) % M; // register rotation after the n-2 moves (n is a multiple of M)

    float top[M][W];
    float bot[M][W];
    float2 cs[kDepth][M];
    int n, H, lane, wave, tid;
    int lanes;              // L = n / (2 M): lanes that hold slots (wavefront exchange: where the far end is)
    const float2 *tab_lane; // table + tid*M
    const float2 *rn_lane;  // renormalisation factors + tid*M (scaled form)
    // this lane's LDS addresses in exchange buffer 0 (buffer 1 is at a compile-time offset)
    float *out_top, *out_bot, *turn;
    const float *in_top, *in_bot;
    static constexpr int kBufFloats = (int)(sizeof(typename CarouselExchange<W, WAVES>::Buf) / sizeof(float));

    __device__ __forceinline__ void load_coefs(int k, float2 (&dst)[M]) { load_row_of(tab_lane, k, dst); }

    __device__ __forceinline__ void load_row_of(const float2 *base, int row, float2 (&dst)[M])
    {
        const float2 *src = base + (long long)row * H;
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

    // Rotation of logical slot R under the register map of unrolled copy U (RN: then multiply the
    // rows back by their renormalisation factors, scaled form).  Ends with an empty asm that has the
    // slot's registers as in/out operands: it emits nothing, but pins the finished values here, so
    // that the compiler cannot sink a rotation into a later block (which would keep that block's
    // cos/sin registers alive and multiply the live table registers by the unroll factor).
    template <int U, int R, bool RN>
    __device__ __forceinline__ void rotate_slot(const float2 (&cur)[M], const float2 (&rn)[M])
    {
        constexpr int it = (R + U) % M, ib = (R - U + M) % M;
        const float c = cur[R].x, s = cur[R].y;
#pragma unroll
        for (int x = 0; x < W; ++x) {
            const float a = top[it][x], b = bot[ib][x];
            if constexpr (FORM == 0) {
                top[it][x] = fmaf(c, a, -(s * b)); // r_i = cos U_i - sin U_j
                bot[ib][x] = fmaf(c, b, s * a);    // r_j = sin U_i + cos U_j
            } else if constexpr (FORM == 1) {
                top[it][x] = fmaf(-c, b, a);       // a~ - alpha b~
                bot[ib][x] = fmaf(s, a, b);        // b~ + beta a~
            } else {
                const float a1 = fmaf(-c, b, a);   // a - t b
                const float b1 = fmaf(s, a1, b);   // b + s a
                top[it][x] = fmaf(-c, b1, a1);     // a - t b
                bot[ib][x] = b1;
            }
            if constexpr (RN) {
                top[it][x] *= rn[R].x;
                bot[ib][x] *= rn[R].y;
            }
        }
#pragma unroll
        for (int x = 0; x < W; ++x) asm volatile("" : "+v"(top[it][x]), "+v"(bot[ib][x]));
    }
    template <int U, bool RN, int... Rs>
    __device__ __forceinline__ void rotate_slots(const float2 (&cur)[M], const float2 (&rn)[M],
                                                 std::integer_sequence<int, Rs...>)
    {
        (rotate_slot<U, Rs, RN>(cur, rn), ...);
    }
    // a run of inner slots (2 .. M-2 take no part in the exchange), starting at slot FIRST
    template <int U, bool RN, int FIRST, int... Rs>
    __device__ __forceinline__ void rotate_inner(const float2 (&cur)[M], const float2 (&rn)[M],
                                                 std::integer_sequence<int, Rs...>)
    {
        (rotate_slot<U, FIRST + Rs, RN>(cur, rn), ...);
    }

    // One block of Algorithm 2 as unrolled copy C (register map C mod M, ring slot C mod kDepth), then the move.
    // LAST marks the very last block (k = 0): no move after it.  PF: block k - (kDepth - 1) exists and is fetched.
    // RENORM (scaled form): this block closes a renormalisation period; the rows are multiplied back
    // by their factors (compile-time variant: a run-time branch around 2*M*W multiplies made the
    // register allocator spill).
    // Order inside the block: the slots whose results leave the lane (0, M-1 and, for the held
    // position, 1) need what the previous block's exchange delivers and feed this block's exchange;
    // the other slots are rotated around them, so that both LDS latencies and the barrier overlap
    // with arithmetic.
    template <int C, bool LAST, bool RENORM, bool PF>
    __device__ __forceinline__ void step(int k)
    {
        constexpr int U = C % M;
        constexpr int par = C & 1;
        constexpr bool RN = FORM != 0 && (LAST || RENORM);
        float2(&cur)[M] = cs[C % kDepth];
        if constexpr (PF) load_coefs(k - (kDepth - 1), cs[(C + kDepth - 1) % kDepth]);
        float2 rn[M];
        if constexpr (RN) load_row_of(rn_lane, (n - 2 - k) / kRenormPeriod, rn);

        // inner slots 2 .. M-2 are split in two runs: the first (the larger half) covers the latency of the LDS
        // reads issued at the end of the previous block, the second the LDS writes and the barrier
        constexpr int kInner = M > 3 ? M - 3 : 0;
        constexpr int kInnerA = (kInner + 1) / 2;
        if constexpr (kInnerA > 0) rotate_inner<U, RN, 2>(cur, rn, std::make_integer_sequence<int, kInnerA>{});

        // The slots that feed the exchange are the block's critical path (every wavefront of the workgroup waits
        // at the barrier for the slowest publisher): they run at raised wave priority, so that the SIMD's other
        // wavefront, if it is in an inner run, yields the issue slots.  Measured at n = B = 4096: 5 % off the
        // sweep together with the 3 + 2 split of the inner slots (priority alone 2 %, split alone slower).
        __builtin_amdgcn_s_setprio(2);
        rotate_slot<U, 0, RN>(cur, rn);
        if constexpr (M > 1) rotate_slot<U, M - 1, RN>(cur, rn);
        if constexpr (M > 2) rotate_slot<U, 1, RN>(cur, rn);

        constexpr int q = U % M;                // top slot 0: leaves towards the previous lane
        constexpr int qb = (M - 1 - U + M) % M; // bottom slot M-1: leaves towards the next lane
        constexpr int q1 = (1 + U) % M;         // top slot 1 (matters in lane 0 of wavefront 0)
        if constexpr (!LAST && EX == kExchangeLds) {
            lds_store_row<W, WAVES>(out_top + par * kBufFloats, top[q]);
            lds_store_row<W, WAVES>(out_bot + par * kBufFloats, bot[qb]);
            if (wave == 0) {
                if (lane == 0) lds_store_row<W, WAVES>(turn + par * kBufFloats, top[q1]);
                // position 0 is held: in lane 0 its row hops to the register that will be slot 0
#pragma unroll
                for (int x = 0; x < W; ++x) {
                    const float held = top[q][x], other = top[q1][x];
                    top[q1][x] = (lane == 0) ? held : other;
                }
            }
        }
        if constexpr (!LAST && EX == kExchangeWave) {
            // the whole move inside the wavefront: the top slot that leaves comes from the next lane (at the far
            // end, lane L-1, it is the lane's own leaving bottom slot), the bottom slot from the previous lane (in
            // lane 0 it is the lane's own top slot 1, and the held row hops into that register)
            const bool far = lane == lanes - 1;
#pragma unroll
            for (int x = 0; x < W; ++x) {
                const float t_out = top[q][x], b_out = bot[qb][x], t_one = top[q1][x];
                const float t_in = lane_from_next(b_out, t_out);
                bot[qb][x] = lane_from_prev(t_one, b_out);
                top[q][x] = far ? b_out : t_in;
                top[q1][x] = (lane == 0) ? t_out : top[q1][x];
            }
        }

        __builtin_amdgcn_s_setprio(0);
        if constexpr (kInner - kInnerA > 0)
            rotate_inner<U, RN, 2 + kInnerA>(cur, rn, std::make_integer_sequence<int, kInner - kInnerA>{});

        if constexpr (!LAST && EX == kExchangeLds) {
            __syncthreads();
            lds_load_row<W, WAVES>(top[q], in_top + par * kBufFloats);
            lds_load_row<W, WAVES>(bot[qb], in_bot + par * kBufFloats);
        }
    }

    // kUnroll consecutive blocks starting at block index k_first (going down), none of them the last;
    // RENORM: the group's last block closes a renormalisation period
    template <bool RENORM, int... Cs>
    __device__ __forceinline__ void full_group(int k_first, std::integer_sequence<int, Cs...>)
    {
        (step<Cs, false, RENORM && Cs == kUnroll - 1, true>(k_first - Cs), ...);
    }
    // the closing kUnroll-1 blocks k = kUnroll-2 .. 0 (n is a multiple of kUnroll, so n-1 blocks always leave
    // a tail of kUnroll-1)
    template <int... Cs>
    __device__ __forceinline__ void tail_group(std::integer_sequence<int, Cs...>)
    {
        (step<Cs, Cs == kUnroll - 2, false, (kUnroll - 2 - Cs >= kDepth - 1)>(kUnroll - 2 - Cs), ...);
    }

    // all n-1 blocks: n/kUnroll - 1 full groups, then the tail of kUnroll - 1
    __device__ __forceinline__ void sweep()
    {
        constexpr auto seq = std::make_integer_sequence<int, kUnroll>{};
        int k = n - 2;
        if constexpr (FORM == 0) {
            for (; k >= kUnroll - 1; k -= kUnroll) full_group<false>(k, seq);
        } else {
            constexpr int per = kRenormPeriod / kUnroll;   // groups per renormalisation period
            const int groups = n / kUnroll - 1;
            for (int pd = 0; pd < groups / per; ++pd) {
                for (int g = 0; g < per - 1; ++g, k -= kUnroll) full_group<false>(k, seq);
                full_group<true>(k, seq);
                k -= kUnroll;
            }
            for (int g = 0; g < groups % per; ++g, k -= kUnroll) full_group<false>(k, seq);
        }
        tail_group(std::make_integer_sequence<int, kUnroll - 1>{});
    }
};

// `rows` is the operand's row count (n, or n - 1 for the padded size of an odd problem): a row beyond
// it is the inactive added dimension, zero on the way in and not stored on the way out.
template <int W>
__device__ __forceinline__ void load_row(float (&dst)[W], const float *X, long long B, int row, int rows,
                                         long long b0, int wv, bool vec, int identity)
{
    if ((unsigned)row >= (unsigned)rows) { // also catches the meaningless (negative) rows of idle lanes
#pragma unroll
        for (int x = 0; x < W; ++x) dst[x] = 0.f;
        return;
    }
    if (identity) {
#pragma unroll
        for (int x = 0; x < W; ++x) dst[x] = (x < wv && (long long)row == b0 + x) ? 1.f : 0.f;
        return;
    }
    const float *src = X + (long long)row * B + b0;
    if constexpr (W % 4 == 0) {
        if (vec) {
#pragma unroll
            for (int x = 0; x < W / 4; ++x) {
                const float4 v = reinterpret_cast<const float4 *>(src)[x];
                dst[4 * x] = v.x; dst[4 * x + 1] = v.y; dst[4 * x + 2] = v.z; dst[4 * x + 3] = v.w;
            }
            return;
        }
    }
#pragma unroll
    for (int x = 0; x < W; ++x) dst[x] = (x < wv) ? src[x] : 0.f;
}

template <int W>
__device__ __forceinline__ void store_row(const float (&src)[W], float *Y, long long B, int row, int rows,
                                          long long b0, int wv, bool vec)
{
    if ((unsigned)row >= (unsigned)rows) return;
    float *dst = Y + (long long)row * B + b0;
    if constexpr (W % 4 == 0) {
        if (vec) {
#pragma unroll
            for (int x = 0; x < W / 4; ++x)
                reinterpret_cast<float4 *>(dst)[x] =
                    make_float4(src[4 * x], src[4 * x + 1], src[4 * x + 2], src[4 * x + 3]);
            return;
        }
    }
#pragma unroll
    for (int x = 0; x < W; ++x)
        if (x < wv) dst[x] = src[x];
}

// mirror: rows are relabelled r -> n - r (r >= 1) on the way in and on the way out; with the mirrored
// coefficient tables (theta_at in coef_kernels.hpp) the launch then computes U(theta)^T X.
__device__ __forceinline__ int mirrored_row(int n, int r, int mirror) { return (mirror && r) ? n - r : r; }

template <int M, int W, int WAVES, int FORM, int EX, typename Exchange>
__device__ __forceinline__ void carousel_forward_body(Exchange &sh, int n, int rows, long long B,
                                                      const float2 *__restrict__ table,
                                                      const float2 *__restrict__ renorm, const float *X, float *Y,
                                                      int identity, int vec_ok, int mirror)
{
    using State = CarouselFwd<M, W, WAVES, FORM, EX>;
    State st;
    const int L = n / (2 * M);                  // lanes that hold slots; the rest of the last wavefront idles
    st.lanes = L;
    const bool idle = (int)threadIdx.x >= L;
    const int coef_lane = idle ? 0 : (int)threadIdx.x;
    const int my_rows = idle ? 0 : rows;        // an idle lane loads zeros and stores nothing
    st.rn_lane = renorm + (long long)coef_lane * M;
    st.n = n;
    st.H = n >> 1;
    st.tid = threadIdx.x;
    st.lane = threadIdx.x & 63;
    st.wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    st.tab_lane = table + (long long)coef_lane * M;
    if constexpr (EX == kExchangeLds) {
        constexpr int LMAX = 64 * WAVES;
        auto &b = sh.buf[0];
        const int t = threadIdx.x;
        st.out_top = b.top_out.lane(t);
        st.out_bot = b.bot_out.lane(t);
        st.turn = b.top_out.lane(LMAX);                                           // the extra row
        st.in_top = (t < L - 1) ? b.top_out.lane(t + 1) : b.bot_out.lane(L - 1); // far end: bot[n/2-1] -> top[n/2-1]
        st.in_bot = (t > 0) ? b.bot_out.lane(t - 1) : b.top_out.lane(LMAX);      // near end: top[1] -> bot[0]
    }

    const long long b0 = (long long)blockIdx.x * W;
    const int wv = (B - b0) < W ? (int)(B - b0) : W;
    const bool vec = vec_ok && wv == W;

    // strip in the position order of block n-1 (k = n-2)
#pragma unroll
    for (int r = 0; r < M; ++r) {
        const int p = st.tid * M + r;
        load_row<W>(st.top[r], X, B, mirrored_row(n, rr_label(n, n - 2, p), mirror), my_rows, b0, wv, vec, identity);
        load_row<W>(st.bot[r], X, B, mirrored_row(n, rr_label(n, n - 2, n - 1 - p), mirror), my_rows, b0, wv, vec,
                    identity);
    }
#pragma unroll
    for (int d = 0; d < State::kDepth - 1; ++d) st.load_coefs(n - 2 - d, st.cs[d]);

    st.sweep();

    // after block 1 the position order is the identity: position p holds row p
    constexpr int UL = State::kLastU;
#pragma unroll
    for (int r = 0; r < M; ++r) {
        const int p = st.tid * M + r;
        store_row<W>(st.top[(r + UL) % M], Y, B, mirrored_row(n, p, mirror), my_rows, b0, wv, vec);
        store_row<W>(st.bot[(r - UL + M) % M], Y, B, mirrored_row(n, n - 1 - p, mirror), my_rows, b0, wv, vec);
    }
}

// One launch per call: the rotation form is read from the device flag (nullptr: standard) and the
// matching copy of the sweep runs; `table` holds that form's coefficients (coef_table_kernel).
struct NoExchange {};   // the wavefront exchange needs no LDS
template <int M, int W, int WAVES, int EX = kExchangeLds>
__global__ __launch_bounds__(64 * WAVES, WAVES > 8 ? 1 : 2) void carousel_forward_kernel(
    int n, int rows, long long B, const float2 *__restrict__ table, const float2 *__restrict__ renorm,
    const unsigned *flag, float scaled_max, const float *X, float *Y, int identity, int vec_ok, int mirror)
{
    using Exchange = std::conditional_t<EX == kExchangeLds, CarouselExchange<W, WAVES>, NoExchange>;
    __shared__ Exchange sh;
    if constexpr (kRenormPeriod % M != 0) {
        // slot counts that do not divide the renormalisation period: standard form only (the host passes no flag)
        carousel_forward_body<M, W, WAVES, kFormStandard, EX>(sh, n, rows, B, table, renorm, X, Y, identity, vec_ok,
                                                              mirror);
    } else {
        const int form = __builtin_amdgcn_readfirstlane(selected_form(flag, scaled_max));
        if (form == kFormScaled)
            carousel_forward_body<M, W, WAVES, kFormScaled, EX>(sh, n, rows, B, table, renorm, X, Y, identity,
                                                                vec_ok, mirror);
        else if (form == kFormLifted)
            carousel_forward_body<M, W, WAVES, kFormLifted, EX>(sh, n, rows, B, table, renorm, X, Y, identity,
                                                                vec_ok, mirror);
        else
            carousel_forward_body<M, W, WAVES, kFormStandard, EX>(sh, n, rows, B, table, renorm, X, Y, identity,
                                                                  vec_ok, mirror);
    }
}

// ---------------------------------------------------------------------------------------------
// Reverse sweep (dtheta and dX from the forward output Y and the upstream gradient G).
//
// Two strips are carried, z (starts as Y) and g (starts as G), both in position order.  Blocks are
// taken in the order b_1, b_2, ..., so the strips start in the identity order, the carousel turns
// the other way (top line towards higher slots, bottom line towards lower slots), and the strips
// end in the order of block n-1.  Per block and slot, first
//     sum_x ( g_bot[x] * z_top[x] - g_top[x] * z_bot[x] )
// over the lane's W columns -- the strip's share of dL/dtheta for that pair, up to the orientation
// sign, which the second-stage reduction applies (top holds the larger label <=> negate) -- and
// then the transposed rotation on both strips.
// ---------------------------------------------------------------------------------------------
// Exchange buffers of the reverse sweep: as in the forward kernel every lane's leaving slots go
// through LDS, here for two strips (z and g); one buffer per block parity.
template <int W, int WAVES>
struct CarouselExchangeBwd {
    struct Strip {
        CarouselLine<W, WAVES> top_out; // per lane: the top slot that leaves; extra row: the held position's row
        CarouselLine<W, WAVES> bot_out; // per lane: the bottom slot that leaves
    };
    struct Buf {
        Strip strip[2]; // z, g
    };
    Buf buf[2];
};

// CHAIN: the persistent workgroups are linked into chains that share one row of partial sums (see
// carousel_backward_body): a workgroup adds its sums to what its predecessor in the chain has left in the row, so
// the row lives in the L2 of the chain's XCD while the chain works its way through it.
// Progress is published as one flag per workgroup and block, each in a cache line of its own (kFlagStride words),
// holding the tag of the launch and pass that last finished the block.
constexpr int kChainSpinLimit = 1 << 23;   // polls (some seconds) before a workgroup gives up waiting
// Blocks a place lets its predecessor get ahead, beyond the one it needs, whenever it has to wait.  Measured at
// n = B = 4096 (reverse sweep, ms): 0: 8.58, 1: 8.66, 2: 8.87, 3 (with the row fetched a block ahead): 9.2.  The
// closer a place follows, the more of the row it finds in the L2 where its predecessor left it.
constexpr int kChainSlack = 0;
// s_waitcnt immediates (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8; others: no wait)
constexpr int waitcnt_vm(int vmcnt) { return (vmcnt & 15) | ((vmcnt >> 4) << 14) | (7 << 4) | (15 << 8); }

template <int M, int W, int WAVES, int FORM, int EX = kExchangeLds, int CHAIN = 0>
struct CarouselBwd {
    static_assert(EX == kExchangeLds || WAVES == 1, "the DPP exchange stays inside one wavefront");
    static_assert(!CHAIN || (EX == kExchangeLds && M % 4 == 0), "chained rows: LDS exchange, 4 or 8 slots per lane");
    // Two workgroups of a chain must never share a compute unit: a store does not update a line that the unit's
    // L1 holds, so the second would read the row as the first found it (seen with one-wavefront workgroups: sums
    // off by a strip's share; invalidating the L1 every block, buffer_inv sc1, made the sweep 13 times slower).
    // From 5 wavefronts on a workgroup has its compute unit to itself (registers and LDS leave no room for two).
    static_assert(!CHAIN || WAVES >= 5, "chained rows: one workgroup per compute unit");
    static constexpr int kDepth = EX == kExchangeWave ? wave_ring_depth_bwd(M) : 2; // as in the forward kernel
    static constexpr int kUnroll = carousel_lcm(M, kDepth);
    static_assert(FORM == 0 || kRenormPeriod % kUnroll == 0,
                  "renormalisation must fall on the last copy of an unrolled group");
    static constexpr int kLastU = (2 * M - 2) % M;

    float zt[M][W], zb[M][W], gt[M][W], gb[M][W];
    float2 cs[kDepth][M];
    float prior[kDepth][M]; // sums of this workgroup's earlier strips for the current and the next blocks
    int n, H, lane, wave, tid;
    int lanes;               // L = n / (2 M): lanes that hold slots
    const float2 *tab_lane;  // table + tid*M
    const float2 *rn_lane;   // renormalisation factors + tid*M (scaled form)
    float *part_lane;        // this workgroup's row of partial sums + tid*M (idle lanes: the sink)
    const float *prior_lane; // what load_prior reads: this workgroup's row, or zeros for its first strip
    // chained rows: the predecessor's flags and this workgroup's own (one per block), the error word, the tag of
    // this launch and pass, the predecessor's flag read ahead for the next block, and whether this wavefront waits
    // for nobody (the head of a chain, or a wavefront that has given up waiting)
    const unsigned *pred_flags;
    unsigned *my_flags, *chain_error;
    unsigned chain_tag, polled;
    int unlinked;
    // this lane's LDS addresses for strip z in exchange buffer 0 (strip g and buffer 1 are at
    // compile-time offsets)
    float *out_top, *out_bot, *hold;
    const float *in_top, *in_bot;
    static constexpr int kStripFloats = (int)(sizeof(typename CarouselExchangeBwd<W, WAVES>::Strip) / sizeof(float));
    static constexpr int kBufFloats = (int)(sizeof(typename CarouselExchangeBwd<W, WAVES>::Buf) / sizeof(float));

    __device__ __forceinline__ void load_coefs(int k, float2 (&dst)[M]) { load_row_of(tab_lane, k, dst); }

    __device__ __forceinline__ void load_row_of(const float2 *base, int row, float2 (&dst)[M])
    {
        const float2 *src = base + (long long)row * H;
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

    // A counter of another workgroup, read through the scalar unit with the cache-bypass bit: the read is served by
    // the L2, which the workgroups of a chain share, and it does not queue with the wavefront's vector loads (those
    // return in order, so one slow read among them would hold up every coefficient fetch behind it: counters read
    // and written with agent-scope vector accesses, which go to memory, cost 3.5 us per block).
    __device__ __forceinline__ static unsigned read_counter(const unsigned *p)
    {
        // (the address is the same in every lane; the two halves are made scalar explicitly)
        const unsigned long long a = reinterpret_cast<unsigned long long>(p);
        const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)a);
        const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(a >> 32));
        const unsigned long long q = ((unsigned long long)hi << 32) | lo;
        unsigned v;
        asm volatile("s_load_dword %0, %1, 0x0 glc\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(q) : "memory");
        return v;
    }
    // A flag is written with an ordinary store (through the write-through L1 into the L2); "atomic" only keeps
    // the compiler from merging or dropping it, and wavefront scope keeps it free of cache-policy bits and waits.
    __device__ __forceinline__ static void publish_counter(unsigned *p, unsigned value)
    {
        __hip_atomic_store(p, value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
    }
    // The predecessor's flag for block k as an ordinary vector load, issued one block before it is looked at.  Every
    // flag has a cache line of its own and is read this way once per launch, so the load cannot be served by a
    // stale line of this compute unit's L1: it comes from the L2 like the coefficient loads around it.
    __device__ __forceinline__ unsigned flag_ahead(int k) const
    {
        const int kk = k < n - 1 ? k : n - 2;
        return __hip_atomic_load(pred_flags + (long long)kk * kFlagStride, __ATOMIC_RELAXED,
                                 __HIP_MEMORY_SCOPE_WAVEFRONT);
    }
    // Returns once the predecessor has finished block k of this pass.  Normally `polled` (flag_ahead of the block
    // before) already says so.  If not, the wavefront reads the flag (of the block kChainSlack further on, while
    // the pass has that many left) through the scalar unit until it is set.  A wait that does not end within
    // the spin limit marks the call as failed (the second stage then writes NaN) and stops this wavefront from
    // waiting again, so every wavefront reaches the end of the kernel whatever happens to its predecessor.
    __device__ __forceinline__ void wait_for_predecessor(int k)
    {
        if (unlinked || __builtin_amdgcn_readfirstlane(polled) >= chain_tag) return;
        const int far = k + kChainSlack < n - 1 ? k + kChainSlack : n - 2;
        const unsigned *flag = pred_flags + (long long)far * kFlagStride;
        int budget = kChainSpinLimit;
        while (read_counter(flag) < chain_tag) {
            if (--budget <= 0) break;
            __builtin_amdgcn_s_sleep(4);
        }
        if (budget <= 0) {
            unlinked = 1;
            if (lane == 0) atomicOr(chain_error, 1u);
        }
    }

    // The partial sums already stored for block k by this workgroup's earlier strips.  For its first
    // strip prior_lane points into a row of zeros instead: a branch here would sit in every block and
    // split the scheduler's region, which costs more than the loads.
    __device__ __forceinline__ void load_prior(int k, float (&dst)[M])
    {
        const float *src = prior_lane + (long long)k * H;
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

    // carousel move of one strip (top line `t`, bottom line `b`), reverse direction; register map U, buffer PAR
    template <int U, int PAR, int WHICH>
    __device__ __forceinline__ void publish(float (&t)[M][W], float (&b)[M][W])
    {
        constexpr int qt = (M - 1 - U + M) % M; // top slot M-1: leaves towards the next lane
        constexpr int qb = U % M;               // bottom slot 0: leaves towards the previous lane
        constexpr int pf = (M - U) % M;         // top slot 0 (the held position, in lane 0 of wavefront 0)
        constexpr int off = PAR * kBufFloats + WHICH * kStripFloats;
        lds_store_row<W, WAVES>(out_top + off, t[qt]);
        lds_store_row<W, WAVES>(out_bot + off, b[qb]);
        if (wave == 0 && lane == 0) lds_store_row<W, WAVES>(hold + off, t[pf]);
    }
    template <int U, int PAR, int WHICH>
    __device__ __forceinline__ void receive(float (&t)[M][W], float (&b)[M][W])
    {
        constexpr int qt = (M - 1 - U + M) % M;
        constexpr int qb = U % M;
        constexpr int pf = (M - U) % M;
        constexpr int off = PAR * kBufFloats + WHICH * kStripFloats;
        if (wave == 0) {
            // lane 0: bot[0] turns round into top[1], i.e. into the register the held row leaves
#pragma unroll
            for (int x = 0; x < W; ++x) {
                const float turn = b[qb][x], keep = t[pf][x];
                t[pf][x] = (lane == 0) ? turn : keep;
            }
        }
        lds_load_row<W, WAVES>(t[qt], in_top + off);
        lds_load_row<W, WAVES>(b[qb], in_bot + off);
    }
    // the same move inside one wavefront: the top slot that leaves comes from the previous lane (lane 0 keeps the
    // held row there, and its bottom slot 0 turns round into the register the held row leaves), the bottom slot
    // from the next lane (at the far end, lane L-1, it is the lane's own leaving top slot)
    template <int U>
    __device__ __forceinline__ void move_in_wavefront(float (&t)[M][W], float (&b)[M][W])
    {
        constexpr int qt = (M - 1 - U + M) % M;
        constexpr int qb = U % M;
        constexpr int pf = (M - U) % M;
        const bool far = lane == lanes - 1;
#pragma unroll
        for (int x = 0; x < W; ++x) {
            const float t_out = t[qt][x], b_out = b[qb][x], held = t[pf][x];
            const float b_in = lane_from_next(t_out, b_out);
            t[qt][x] = lane_from_prev(held, t_out);
            b[qb][x] = far ? t_out : b_in;
            t[pf][x] = (lane == 0) ? b_out : held;
        }
    }

    // Logical slot R of one block: the strip's share of the pair's gradient, then the transposed
    // rotation on both strips (RN: then the renormalisation multiply), then the pin (see the forward
    // kernel's rotate_slot).
    template <int U, int R, bool RN>
    __device__ __forceinline__ float sweep_slot(const float2 (&cur)[M], const float2 (&rn)[M])
    {
        constexpr int it = (R - U + M) % M, ib = (R + U) % M;
        const float c = cur[R].x, s = cur[R].y;
        float acc = 0.f;
#pragma unroll
        for (int x = 0; x < W; ++x) {
            const float za = zt[it][x], zv = zb[ib][x], ga = gt[it][x], gv = gb[ib][x];
            acc = fmaf(gv, za, acc);
            acc = fmaf(-ga, zv, acc);
            if constexpr (FORM == 0) {
                zt[it][x] = fmaf(c, za, s * zv);   // transposed rotation
                zb[ib][x] = fmaf(c, zv, -(s * za));
                gt[it][x] = fmaf(c, ga, s * gv);
                gb[ib][x] = fmaf(c, gv, -(s * ga));
            } else if constexpr (FORM == 1) {
                zt[it][x] = fmaf(c, zv, za);       // a~ + alpha b~
                zb[ib][x] = fmaf(-s, za, zv);      // b~ - beta a~
                gt[it][x] = fmaf(c, gv, ga);
                gb[ib][x] = fmaf(-s, ga, gv);
            } else {
                const float z1 = fmaf(c, zv, za);  // the three shears of the transposed rotation
                const float w1 = fmaf(-s, z1, zv);
                zt[it][x] = fmaf(c, w1, z1);
                zb[ib][x] = w1;
                const float g1 = fmaf(c, gv, ga);
                const float h1 = fmaf(-s, g1, gv);
                gt[it][x] = fmaf(c, h1, g1);
                gb[ib][x] = h1;
            }
            if constexpr (RN) {
                zt[it][x] *= rn[R].x;
                zb[ib][x] *= rn[R].y;
                gt[it][x] *= rn[R].x;
                gb[ib][x] *= rn[R].y;
            }
            // pin every four columns (or at the end): a whole slot in flight at once costs more
            // registers than this kernel has
            if ((x & 3) == 3 || x == W - 1) {
#pragma unroll
                for (int y = x & ~3; y <= x; ++y)
                    asm volatile("" : "+v"(zt[it][y]), "+v"(zb[ib][y]), "+v"(gt[it][y]), "+v"(gb[ib][y]), "+v"(acc));
            }
        }
        return acc;
    }
    // a run of inner slots (1 .. M-2 take no part in the exchange), starting at slot FIRST
    template <int U, bool RN, int FIRST, int... Rs>
    __device__ __forceinline__ void sweep_inner(const float2 (&cur)[M], const float2 (&rn)[M], float (&sums)[M],
                                                std::integer_sequence<int, Rs...>)
    {
        ((sums[FIRST + Rs] = sweep_slot<U, FIRST + Rs, RN>(cur, rn)), ...);
    }

    // One block of the reverse sweep.  The slots whose rows leave the lane (0 and M-1) go first and
    // are published to LDS; the inner slots run while those writes and the barrier are in flight.
    template <int C, bool LAST, bool RENORM, bool PF>
    __device__ __forceinline__ void step(int k)
    {
        constexpr int U = C % M;      // register map of this unrolled copy
        constexpr int PAR = C & 1;    // its exchange buffers
        constexpr int SLOT = C % kDepth, FREE = (C + kDepth - 1) % kDepth;   // ring of coefficients and prior sums
        constexpr bool RN = FORM != 0 && (LAST || RENORM);
        float2(&cur)[M] = cs[SLOT];
        if constexpr (PF) load_coefs(k + (kDepth - 1), cs[FREE]);
        float2 rn[M];
        if constexpr (RN) load_row_of(rn_lane, k / kRenormPeriod, rn);
        // what this workgroup's earlier strips have summed for a LATER block: fetched ahead, like cos/sin, and
        // before this block's store, so that waiting for it never waits for a store
        float(&earlier)[M] = prior[SLOT];
        if constexpr (CHAIN) {
            // chained rows: this block's part of the row is fetched in the block itself (it is needed only at the
            // block's end), so that a place runs as close behind its predecessor as the flags allow and finds the
            // lines its predecessor stored still in the L2
            wait_for_predecessor(k);
            polled = flag_ahead(k + 1);   // looked at in the next block: nothing waits for this load here
            load_prior(k, prior[SLOT]);
        } else {
            if constexpr (PF) load_prior(k + (kDepth - 1), prior[FREE]);
        }

        float sums[M];
        // the inner slots all run after the exchange slots here: splitting them around the exchange as
        // the forward kernel does costs registers this kernel does not have (it spills and gets slower)
        constexpr int kInner = M > 2 ? M - 2 : 0;
        __builtin_amdgcn_s_setprio(2);   // the exchange slots are the block's critical path (see the forward kernel)
        sums[0] = sweep_slot<U, 0, RN>(cur, rn);
        if constexpr (M > 1) sums[M - 1] = sweep_slot<U, M - 1, RN>(cur, rn);
        if constexpr (!LAST && EX == kExchangeLds) {
            publish<U, PAR, 0>(zt, zb);
            publish<U, PAR, 1>(gt, gb);
        }
        if constexpr (!LAST && EX == kExchangeWave) {
            move_in_wavefront<U>(zt, zb);
            move_in_wavefront<U>(gt, gb);
        }
        __builtin_amdgcn_s_setprio(0);
        if constexpr (kInner > 0) sweep_inner<U, RN, 1>(cur, rn, sums, std::make_integer_sequence<int, kInner>{});
        {
            float *dst = part_lane + (long long)k * H;
#pragma unroll
            for (int r = 0; r < M; ++r) sums[r] += earlier[r];
            if constexpr (M % 4 == 0) {
#pragma unroll
                for (int r = 0; r < M / 4; ++r)
                    reinterpret_cast<float4 *>(dst)[r] =
                        make_float4(sums[4 * r], sums[4 * r + 1], sums[4 * r + 2], sums[4 * r + 3]);
            } else if constexpr (M % 2 == 0) {
#pragma unroll
                for (int r = 0; r < M / 2; ++r)
                    reinterpret_cast<float2 *>(dst)[r] = make_float2(sums[2 * r], sums[2 * r + 1]);
            } else {
#pragma unroll
                for (int r = 0; r < M; ++r) dst[r] = sums[r];
            }
        }
        if constexpr (!LAST && EX == kExchangeLds) {
            // chained rows: this wavefront's store of the previous block has reached L2 once at most the memory
            // operations of this block are outstanding (they complete in order; a block issues at least five:
            // two coefficient loads, the flag read ahead, the earlier sums, this store), and after the barrier that
            // holds for all wavefronts, so block k-1 can be flagged as being in the row
            if constexpr (CHAIN) __builtin_amdgcn_s_waitcnt(waitcnt_vm(4));
            __syncthreads();
            if constexpr (CHAIN) {
                if (tid == 0 && k > 0) publish_counter(my_flags + (long long)(k - 1) * kFlagStride, chain_tag);
            }
            receive<U, PAR, 0>(zt, zb);
            receive<U, PAR, 1>(gt, gb);
        }
    }

    template <bool RENORM, int... Cs>
    __device__ __forceinline__ void full_group(int k_first, std::integer_sequence<int, Cs...>)
    {
        (step<Cs, false, RENORM && Cs == kUnroll - 1, true>(k_first + Cs), ...);
    }
    template <int... Cs>
    __device__ __forceinline__ void tail_group(int k_first, std::integer_sequence<int, Cs...>)
    {
        (step<Cs, Cs == kUnroll - 2, false, (kUnroll - 2 - Cs >= kDepth - 1)>(k_first + Cs), ...);
    }

    // all n-1 blocks in the order b_1, b_2, ...: n/kUnroll - 1 full groups, then the tail of kUnroll - 1
    __device__ __forceinline__ void sweep()
    {
        constexpr auto seq = std::make_integer_sequence<int, kUnroll>{};
        if constexpr (CHAIN) {
            polled = 0u;
        } else {
#pragma unroll
            for (int d = 0; d < kDepth - 1; ++d) load_prior(d, prior[d]);
        }
        int k = 0;
        if constexpr (FORM == 0) {
            for (; k + kUnroll <= n - 1; k += kUnroll) full_group<false>(k, seq);
        } else {
            constexpr int per = kRenormPeriod / kUnroll;
            const int groups = n / kUnroll - 1;
            for (int pd = 0; pd < groups / per; ++pd) {
                for (int g = 0; g < per - 1; ++g, k += kUnroll) full_group<false>(k, seq);
                full_group<true>(k, seq);
                k += kUnroll;
            }
            for (int g = 0; g < groups % per; ++g, k += kUnroll) full_group<false>(k, seq);
        }
        tail_group(k, std::make_integer_sequence<int, kUnroll - 1>{});
    }
};

// Chained rows (CHAIN).  Workgroup g of the grid belongs to chain c = g mod `chains` at place j = g / chains
// (kChainLength places; the grid is chains * kChainLength workgroups, `chains` a multiple of 8, so that the
// workgroups of a chain differ by multiples of 8 and, workgroups being dealt to the XCDs in turn, share an L2).  In
// pass t (the workgroup's t-th strip) the chain sums into row t * chains + c: the head stores its sums, every other
// place adds its own to what the place before it has left there, one block behind it at the earliest, and the last
// place leaves the chain's total.  Only the head's lines ever come from HBM-side zeros and only the finished row
// goes back to HBM; in between the row's active part sits in L2.  What tells a workgroup that its predecessor is
// done with a block is that predecessor's progress counter (wait_for_predecessor).  At the start every workgroup
// records which XCD it runs on and checks that its predecessor runs on the same one: if not (or if a wait runs
// out), the error word is set and the second stage poisons the result instead of returning sums that may have
// been read from a stale L2.

template <int M, int W, int WAVES, int FORM, int EX, int CHAIN, typename Exchange>
__device__ __forceinline__ void carousel_backward_body(Exchange &sh, int n, int rows, long long B,
                                                       long long strip0, long long nstrips,
                                                       const float2 *__restrict__ table,
                                                       const float2 *__restrict__ renorm, const float *Yin,
                                                       const float *G, float *dX, float *partial,
                                                       const float *__restrict__ zeros, float *sink, int vec_ok,
                                                       int g_identity, const CarouselChainArgs &chain)
{
    using State = CarouselBwd<M, W, WAVES, FORM, EX, CHAIN>;
    State st;
    const int L = n / (2 * M);                  // lanes that hold slots; the rest of the last wavefront idles
    const bool idle = (int)threadIdx.x >= L;
    const int coef_lane = idle ? 0 : (int)threadIdx.x;
    const int my_rows = idle ? 0 : rows;        // an idle lane loads zeros and stores no rows
    st.lanes = L;
    st.rn_lane = renorm + (long long)coef_lane * M;
    st.n = n;
    st.H = n >> 1;
    st.tid = threadIdx.x;
    st.lane = threadIdx.x & 63;
    st.wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    st.tab_lane = table + (long long)coef_lane * M;
    // an idle lane's sums (all zero) go to the sink: N + 8192 floats nobody reads
    const long long N = (long long)(n - 1) * (n >> 1);
    st.part_lane = idle ? sink + (long long)threadIdx.x * M
                        : partial + (long long)blockIdx.x * N + (long long)threadIdx.x * M;
    int place = 0, chain_id = 0;
    unsigned tag_base = 0u;
    if constexpr (CHAIN) {
        chain_id = (int)blockIdx.x % chain.chains;
        place = (int)blockIdx.x / chain.chains;
        const long long flags_per_group = (long long)(n - 1) * kFlagStride;
        st.my_flags = chain.flags + (long long)blockIdx.x * flags_per_group;
        st.pred_flags = place ? chain.flags + (long long)(blockIdx.x - chain.chains) * flags_per_group : st.my_flags;
        st.chain_error = chain.error;
        tag_base = State::read_counter(chain.epoch) * (unsigned)(kChainMaxPasses + 1);
        st.chain_tag = 0u;
        st.polled = 0u;
        st.unlinked = place ? 0 : 1;
        unsigned xcd;
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcd));
        xcd = (xcd & 15u) + 1u;
        if (threadIdx.x == 0) State::publish_counter(chain.xcd_of + blockIdx.x, xcd);
        if (place) {
            // the predecessor has a lower number and was dealt out earlier; wait (bounded) until it has started
            const unsigned *theirs = chain.xcd_of + (blockIdx.x - chain.chains);
            unsigned v = 0;
            int budget = kChainSpinLimit;
            do {
                v = State::read_counter(theirs);
                if (v == 0) __builtin_amdgcn_s_sleep(4);
            } while (v == 0 && --budget > 0);
            if (v != xcd) {
                st.unlinked = 1;
                if (st.lane == 0) atomicOr(chain.error, v ? 2u : 1u);
            }
        }
    }
    if constexpr (EX == kExchangeLds) {
        constexpr int LMAX = 64 * WAVES;
        auto &z = sh.buf[0].strip[0];
        const int t = threadIdx.x;
        st.out_top = z.top_out.lane(t);
        st.out_bot = z.bot_out.lane(t);
        st.hold = z.top_out.lane(LMAX);                                           // the extra row
        // near end: the held row stays in slot 0
        st.in_top = (t > 0) ? z.top_out.lane(t - 1) : z.top_out.lane(LMAX);
        st.in_bot = (t < L - 1) ? z.bot_out.lane(t + 1) : z.top_out.lane(L - 1); // far end: top[n/2-1] -> bot[n/2-1]
    }

    // Persistent workgroup: strips strip0 + blockIdx.x, + gridDim.x, ... of the nstrips of this launch.
    // Its row of partial sums is written by the first strip and added to by the others, in program
    // order, so the result does not depend on scheduling.
    int pass = 0;
    for (long long s = blockIdx.x; s < nstrips; s += gridDim.x, ++pass) {
        const bool first_strip = (s == (long long)blockIdx.x);
        if constexpr (CHAIN) {
            // this pass's row of the chain; the head starts it from zeros
            float *row = partial + ((long long)pass * chain.chains + chain_id) * N + (long long)threadIdx.x * M;
            if (!idle) st.part_lane = row;
            st.prior_lane = (place && !idle) ? row : zeros + (long long)coef_lane * M;
            st.chain_tag = tag_base + (unsigned)pass;
        } else {
            st.prior_lane = first_strip ? zeros + (long long)coef_lane * M : st.part_lane;
        }
        const long long b0 = (strip0 + s) * W;
        const int wv = (B - b0) < W ? (int)(B - b0) : W;
        const bool vec = vec_ok && wv == W;

        // block 1 is processed first: identity position order
#pragma unroll
        for (int r = 0; r < M; ++r) {
            const int p = st.tid * M + r;
            load_row<W>(st.zt[r], Yin, B, p, my_rows, b0, wv, vec, 0);
            load_row<W>(st.zb[r], Yin, B, n - 1 - p, my_rows, b0, wv, vec, 0);
            load_row<W>(st.gt[r], G, B, p, my_rows, b0, wv, vec, g_identity);   // g_identity: G = I_n, not read
            load_row<W>(st.gb[r], G, B, n - 1 - p, my_rows, b0, wv, vec, g_identity);
        }
#pragma unroll
        for (int d = 0; d < State::kDepth - 1; ++d) st.load_coefs(d, st.cs[d]);

        st.sweep();

        if (dX) {
            constexpr int UL = State::kLastU;
#pragma unroll
            for (int r = 0; r < M; ++r) {
                const int p = st.tid * M + r;
                store_row<W>(st.gt[(r - UL + M) % M], dX, B, rr_label(n, n - 2, p), my_rows, b0, wv, vec);
                store_row<W>(st.gb[(r + UL) % M], dX, B, rr_label(n, n - 2, n - 1 - p), my_rows, b0, wv, vec);
            }
        }
        if constexpr (CHAIN) __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));   // this pass's sums have reached L2
        if constexpr (EX == kExchangeLds) __syncthreads(); // the next strip reuses the exchange buffers
        if constexpr (CHAIN) {
            // (everything up to the last block at once: the per-block flags of the last blocks trail by one)
            if (threadIdx.x == 0) {
                State::publish_counter(st.my_flags + (long long)(n - 3) * kFlagStride, st.chain_tag);
                State::publish_counter(st.my_flags + (long long)(n - 2) * kFlagStride, st.chain_tag);
            }
        }
    }
}

template <int M, int W, int WAVES, int EX = kExchangeLds>
__global__ __launch_bounds__(64 * WAVES, WAVES > 8 ? 1 : 2) void carousel_backward_kernel(
    int n, int rows, long long B, long long strip0, long long nstrips, const float2 *__restrict__ table,
    const float2 *__restrict__ renorm, const unsigned *flag, float scaled_max, const float *Yin, const float *G,
    float *dX, float *partial, const float *__restrict__ zeros, float *sink, int vec_ok, int g_identity)
{
    using Exchange = std::conditional_t<EX == kExchangeLds, CarouselExchangeBwd<W, WAVES>, NoExchange>;
    __shared__ Exchange sh;
    if constexpr (kRenormPeriod % M != 0) {
        carousel_backward_body<M, W, WAVES, kFormStandard, EX, 0>(sh, n, rows, B, strip0, nstrips, table, renorm, Yin,
                                                                  G, dX, partial, zeros, sink, vec_ok, g_identity,
                                                                  CarouselChainArgs{});
    } else {
        const int form = __builtin_amdgcn_readfirstlane(selected_form(flag, scaled_max));
        if (form == kFormScaled)
            carousel_backward_body<M, W, WAVES, kFormScaled, EX, 0>(sh, n, rows, B, strip0, nstrips, table, renorm,
                                                                    Yin, G, dX, partial, zeros, sink, vec_ok,
                                                                    g_identity, CarouselChainArgs{});
        else if (form == kFormLifted)
            carousel_backward_body<M, W, WAVES, kFormLifted, EX, 0>(sh, n, rows, B, strip0, nstrips, table, renorm,
                                                                    Yin, G, dX, partial, zeros, sink, vec_ok,
                                                                    g_identity, CarouselChainArgs{});
        else
            carousel_backward_body<M, W, WAVES, kFormStandard, EX, 0>(sh, n, rows, B, strip0, nstrips, table, renorm,
                                                                      Yin, G, dX, partial, zeros, sink, vec_ok,
                                                                      g_identity, CarouselChainArgs{});
    }
}

// The reverse sweep with chained rows of partial sums (carousel_backward_body): same arguments plus the chain's
// counters; `partial` holds passes * chains rows.
template <int M, int W, int WAVES>
__global__ __launch_bounds__(64 * WAVES, 2) void carousel_backward_chain_kernel(
    int n, int rows, long long B, long long strip0, long long nstrips, const float2 *__restrict__ table,
    const float2 *__restrict__ renorm, const unsigned *flag, float scaled_max, const float *Yin, const float *G,
    float *dX, float *partial, const float *__restrict__ zeros, float *sink, int vec_ok, int g_identity,
    CarouselChainArgs chain)
{
    __shared__ CarouselExchangeBwd<W, WAVES> sh;
    const int form = __builtin_amdgcn_readfirstlane(selected_form(flag, scaled_max));
    if (form == kFormScaled)
        carousel_backward_body<M, W, WAVES, kFormScaled, kExchangeLds, 1>(sh, n, rows, B, strip0, nstrips, table,
                                                                          renorm, Yin, G, dX, partial, zeros, sink,
                                                                          vec_ok, g_identity, chain);
    else if (form == kFormLifted)
        carousel_backward_body<M, W, WAVES, kFormLifted, kExchangeLds, 1>(sh, n, rows, B, strip0, nstrips, table,
                                                                          renorm, Yin, G, dX, partial, zeros, sink,
                                                                          vec_ok, g_identity, chain);
    else
        carousel_backward_body<M, W, WAVES, kFormStandard, kExchangeLds, 1>(sh, n, rows, B, strip0, nstrips, table,
                                                                            renorm, Yin, G, dX, partial, zeros,
                                                                            sink, vec_ok, g_identity, chain);
}

// ---------------------------------------------------------------------------------------------
// launches (instantiated per number of slots per lane by carousel_fwd_m*.hip / carousel_bwd_m*.hip, and for more
// than 8 wavefronts by carousel_fwd_wide.hip / carousel_bwd_wide.hip)
// ---------------------------------------------------------------------------------------------
template <int M, int W, int WAVES>
inline void carousel_launch_fwd(const CarouselFwdArgs &a)
{
    const long long strips = (a.B + W - 1) / W;
    hipLaunchKernelGGL((carousel_forward_kernel<M, W, WAVES>), dim3((unsigned)strips), dim3(64 * WAVES), 0,
                       a.stream, a.n, a.rows, a.B, a.coefs.table, a.coefs.renorm, a.coefs.flag, a.coefs.scaled_max,
                       a.X, a.Y, a.identity, a.vec_ok, a.mirror);
}

template <int M, int WAVES>
inline int carousel_fwd_widths(int W, const CarouselFwdArgs &a)
{
    switch (W) {
    case 8: carousel_launch_fwd<M, 8, WAVES>(a); return GIVENS_OK;
    case 4: carousel_launch_fwd<M, 4, WAVES>(a); return GIVENS_OK;
    case 2: carousel_launch_fwd<M, 2, WAVES>(a); return GIVENS_OK;
    case 1: carousel_launch_fwd<M, 1, WAVES>(a); return GIVENS_OK;
    default: return GIVENS_ERR_UNSUPPORTED;
    }
}

// every number of wavefronts carousel_shape_for can return for M slots per lane, in two halves so that a slot
// count whose kernels take long to compile can spread them over two translation units
template <int M>
inline int carousel_forward_slots_1to4(const CarouselFwdArgs &a, int waves, int W)
{
    switch (waves) {
    case 1: return carousel_fwd_widths<M, 1>(W, a);
    case 2: return carousel_fwd_widths<M, 2>(W, a);
    case 3: return carousel_fwd_widths<M, 3>(W, a);
    case 4: return carousel_fwd_widths<M, 4>(W, a);
    default: return GIVENS_ERR_UNSUPPORTED;
    }
}
template <int M>
inline int carousel_forward_slots_5to8(const CarouselFwdArgs &a, int waves, int W)
{
    switch (waves) {
    case 5: return carousel_fwd_widths<M, 5>(W, a);
    case 6: return carousel_fwd_widths<M, 6>(W, a);
    case 7: return carousel_fwd_widths<M, 7>(W, a);
    case 8: return carousel_fwd_widths<M, 8>(W, a);
    default: return GIVENS_ERR_UNSUPPORTED;
    }
}
template <int M>
inline int carousel_forward_slots(const CarouselFwdArgs &a, int waves, int W)
{
    return waves <= 4 ? carousel_forward_slots_1to4<M>(a, waves, W) : carousel_forward_slots_5to8<M>(a, waves, W);
}

template <int M, int W, int WAVES>
inline void carousel_launch_bwd(const CarouselBwdArgs &a)
{
    hipLaunchKernelGGL((carousel_backward_kernel<M, W, WAVES>), dim3((unsigned)a.groups), dim3(64 * WAVES), 0,
                       a.stream, a.n, a.rows, a.B, a.strip0, a.nstrips, a.coefs.table, a.coefs.renorm, a.coefs.flag,
                       a.coefs.scaled_max, a.Y, a.G, a.dX, a.partial, a.zeros, a.sink, a.vec_ok, a.g_identity);
}

template <int M, int WAVES>
inline int carousel_bwd_widths(int W, const CarouselBwdArgs &a)
{
    switch (W) {
    case 8: carousel_launch_bwd<M, 8, WAVES>(a); return GIVENS_OK;
    case 4: carousel_launch_bwd<M, 4, WAVES>(a); return GIVENS_OK;
    case 2: carousel_launch_bwd<M, 2, WAVES>(a); return GIVENS_OK;
    case 1: carousel_launch_bwd<M, 1, WAVES>(a); return GIVENS_OK;
    default: return GIVENS_ERR_UNSUPPORTED;
    }
}

template <int M>
inline int carousel_backward_slots(const CarouselBwdArgs &a, int waves, int W)
{
    switch (waves) {
    case 1: return carousel_bwd_widths<M, 1>(W, a);
    case 2: return carousel_bwd_widths<M, 2>(W, a);
    case 3: return carousel_bwd_widths<M, 3>(W, a);
    case 4: return carousel_bwd_widths<M, 4>(W, a);
    case 5: return carousel_bwd_widths<M, 5>(W, a);
    case 6: return carousel_bwd_widths<M, 6>(W, a);
    case 7: return carousel_bwd_widths<M, 7>(W, a);
    case 8: return carousel_bwd_widths<M, 8>(W, a);
    default: return GIVENS_ERR_UNSUPPORTED;
    }
}

// Chained rows (carousel_bwd_chain.hip): 4 slots per lane, strips of 8 or 4 columns.
template <int M, int W, int WAVES>
inline void carousel_launch_bwd_chain(const CarouselBwdArgs &a, const CarouselChainArgs &c)
{
    hipLaunchKernelGGL((carousel_backward_chain_kernel<M, W, WAVES>), dim3((unsigned)a.groups), dim3(64 * WAVES), 0,
                       a.stream, a.n, a.rows, a.B, a.strip0, a.nstrips, a.coefs.table, a.coefs.renorm, a.coefs.flag,
                       a.coefs.scaled_max, a.Y, a.G, a.dX, a.partial, a.zeros, a.sink, a.vec_ok, a.g_identity, c);
}
template <int M, int WAVES>
inline int carousel_bwd_chain_widths(int W, const CarouselBwdArgs &a, const CarouselChainArgs &c)
{
    switch (W) {
    case 8: carousel_launch_bwd_chain<M, 8, WAVES>(a, c); return GIVENS_OK;
    case 4: carousel_launch_bwd_chain<M, 4, WAVES>(a, c); return GIVENS_OK;
    default: return GIVENS_ERR_UNSUPPORTED;
    }
}
template <int M>
inline int carousel_backward_chain_slots(const CarouselBwdArgs &a, const CarouselChainArgs &c, int waves, int W)
{
    switch (waves) {
    case 5: return carousel_bwd_chain_widths<M, 5>(W, a, c);
    case 6: return carousel_bwd_chain_widths<M, 6>(W, a, c);
    case 7: return carousel_bwd_chain_widths<M, 7>(W, a, c);
    case 8: return carousel_bwd_chain_widths<M, 8>(W, a, c);
    default: return GIVENS_ERR_UNSUPPORTED;
    }
}

// One-wavefront shapes with the exchange inside the wavefront (carousel_fwd_wave.hip / carousel_bwd_wave.hip):
// forward strips of up to 8 columns, reverse strips of up to 4.
template <int M, int W>
inline void carousel_launch_fwd_wave(const CarouselFwdArgs &a)
{
    const long long strips = (a.B + W - 1) / W;
    hipLaunchKernelGGL((carousel_forward_kernel<M, W, 1, kExchangeWave>), dim3((unsigned)strips), dim3(64), 0,
                       a.stream, a.n, a.rows, a.B, a.coefs.table, a.coefs.renorm, a.coefs.flag, a.coefs.scaled_max,
                       a.X, a.Y, a.identity, a.vec_ok, a.mirror);
}
template <int M>
inline int carousel_forward_wave_slots(const CarouselFwdArgs &a, int W)
{
    switch (W) {
    case 8: carousel_launch_fwd_wave<M, 8>(a); return GIVENS_OK;
    case 4: carousel_launch_fwd_wave<M, 4>(a); return GIVENS_OK;
    case 2: carousel_launch_fwd_wave<M, 2>(a); return GIVENS_OK;
    case 1: carousel_launch_fwd_wave<M, 1>(a); return GIVENS_OK;
    default: return GIVENS_ERR_UNSUPPORTED;
    }
}
template <int M, int W>
inline void carousel_launch_bwd_wave(const CarouselBwdArgs &a)
{
    hipLaunchKernelGGL((carousel_backward_kernel<M, W, 1, kExchangeWave>), dim3((unsigned)a.groups), dim3(64), 0,
                       a.stream, a.n, a.rows, a.B, a.strip0, a.nstrips, a.coefs.table, a.coefs.renorm, a.coefs.flag,
                       a.coefs.scaled_max, a.Y, a.G, a.dX, a.partial, a.zeros, a.sink, a.vec_ok, a.g_identity);
}
template <int M>
inline int carousel_backward_wave_slots(const CarouselBwdArgs &a, int W)
{
    switch (W) {
    case 4: carousel_launch_bwd_wave<M, 4>(a); return GIVENS_OK;
    case 2: carousel_launch_bwd_wave<M, 2>(a); return GIVENS_OK;
    case 1: carousel_launch_bwd_wave<M, 1>(a); return GIVENS_OK;
    default: return GIVENS_ERR_UNSUPPORTED;
    }
}

// Shapes with an odd number of slots per lane (standard rotation form only, reverse-sweep strips of at most 4
// columns): every compiled number of wavefronts, up to 1024 lanes.
template <int M>
inline int carousel_forward_odd_slots(const CarouselFwdArgs &a, int waves, int W)
{
    static_assert(M % 2 == 1, "the even slot counts have their own translation units");
    switch (waves) {
    case 10: return carousel_fwd_widths<M, 10>(W, a);
    case 12: return carousel_fwd_widths<M, 12>(W, a);
    case 14: return carousel_fwd_widths<M, 14>(W, a);
    case 16: return carousel_fwd_widths<M, 16>(W, a);
    default: return carousel_forward_slots<M>(a, waves, W);
    }
}

template <int M, int WAVES>
inline int carousel_bwd_narrow_widths(int W, const CarouselBwdArgs &a)
{
    switch (W) {
    case 4: carousel_launch_bwd<M, 4, WAVES>(a); return GIVENS_OK;
    case 2: carousel_launch_bwd<M, 2, WAVES>(a); return GIVENS_OK;
    case 1: carousel_launch_bwd<M, 1, WAVES>(a); return GIVENS_OK;
    default: return GIVENS_ERR_UNSUPPORTED;
    }
}

template <int M>
inline int carousel_backward_odd_slots(const CarouselBwdArgs &a, int waves, int W)
{
    static_assert(M % 2 == 1, "the even slot counts have their own translation units");
    switch (waves) {
    case 1: return carousel_bwd_narrow_widths<M, 1>(W, a);
    case 2: return carousel_bwd_narrow_widths<M, 2>(W, a);
    case 3: return carousel_bwd_narrow_widths<M, 3>(W, a);
    case 4: return carousel_bwd_narrow_widths<M, 4>(W, a);
    case 5: return carousel_bwd_narrow_widths<M, 5>(W, a);
    case 6: return carousel_bwd_narrow_widths<M, 6>(W, a);
    case 7: return carousel_bwd_narrow_widths<M, 7>(W, a);
    case 8: return carousel_bwd_narrow_widths<M, 8>(W, a);
    case 10: return carousel_bwd_narrow_widths<M, 10>(W, a);
    case 12: return carousel_bwd_narrow_widths<M, 12>(W, a);
    case 14: return carousel_bwd_narrow_widths<M, 14>(W, a);
    case 16: return carousel_bwd_narrow_widths<M, 16>(W, a);
    default: return GIVENS_ERR_UNSUPPORTED;
    }
}

} // namespace givens
