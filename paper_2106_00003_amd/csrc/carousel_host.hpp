// Host side of the register-carousel kernels: shapes, launch arguments and the entry points of the
// translation units that instantiate the kernels (one per sweep direction and number of slots per lane,
// so that they compile in parallel).  No device code here.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>
#include <initializer_list>
#include <type_traits>

#include "../../include/givens_rr.h"
#include "forms.hpp"

namespace givens {

struct CarouselShape {
    int M, WAVES;
};

// What a sweep reads: the table of the rotation form the device flag selects, the renormalisation rows
// (scaled and lifted forms) and that flag (nullptr: standard form).
struct CarouselCoefs {
    const float2 *table;
    const float2 *renorm;
    const unsigned *flag;
    float scaled_max; // threshold of the scaled form (negative: never), see form_for_range
};

// n = 2 * M * L: M slots per lane in {8, 4, 2} (the scaled and lifted forms need a slot count that divides the
// renormalisation period) and
// L <= 512 lanes, run by a workgroup of WAVES = ceil(L / 64) wavefronts whose spare lanes idle.  So the
// family takes every n that is a multiple of 4 from kCarouselMinN up to 2048 (M = 2), of 8 up to 4096 and
// of 16 up to 8192.  The most slots per lane that fit are preferred: fewer of a lane's slots take part in
// the exchange.  Below kCarouselMinN a workgroup would be mostly idle lanes.
// The remaining multiples of 4 up to 4096 and of 8 up to 8192 run with 513 to 1024 lanes (2 or 4 slots per lane,
// an even number of wavefronts from 10 to 16, one workgroup per compute unit): slower per update than the shapes
// above, but several times faster than the LDS family they would otherwise fall to.
constexpr int kCarouselMinN = 132;
inline bool carousel_shape_with(int n, std::initializer_list<int> slots, CarouselShape *out, int max_lanes = 512)
{
    if (n < kCarouselMinN) return false;
    for (int m : slots)
        if (n % (2 * m) == 0 && n / (2 * m) <= max_lanes) {
            int waves = (n / (2 * m) + 63) / 64;
            if (waves > 8) waves += waves & 1;      // compiled: 10, 12, 14, 16
            *out = {m, waves};
            return true;
        }
    return false;
}
// What is left of the even n (n = 2 (mod 4), and multiples of 4 or 8 too large for the shapes above) runs with
// 7, 5 or 3 slots per lane where n / 2 has such a factor and n / (2 M) <= 1024: about half of those sizes, among
// them the padded sizes of half of the odd n.  Standard rotation form only (carousel_has_forms).
inline bool carousel_odd_shape_for(int n, CarouselShape *out)
{
    return carousel_shape_with(n, {7, 5, 3}, out) || carousel_shape_with(n, {7, 5, 3}, out, 1024);
}
inline bool carousel_shape_for(int n, CarouselShape *out)
{
    return carousel_shape_with(n, {8, 4, 2}, out) || carousel_shape_with(n, {4, 2}, out, 1024) ||
           carousel_odd_shape_for(n, out);
}

template <typename T>
inline bool carousel_supported(int n, long long B)
{
    (void)B;
    CarouselShape s;
    return std::is_same<T, float>::value && carousel_shape_for(n, &s);
}

// shapes of the reverse sweep: two strips per lane, so 4 slots per lane where that covers n (multiples of 8 up
// to 4096), 2 for the other multiples of 4 up to 2048, and 8 slots per lane with narrower strips for the
// multiples of 16 beyond 4096, up to 8192
inline bool carousel_bwd_shape_for(int n, CarouselShape *out)
{
    if (carousel_shape_with(n, {4, 2}, out)) return true;
    if (n > 4096 && carousel_shape_with(n, {8}, out)) return true;
    return carousel_shape_with(n, {4, 2}, out, 1024) || carousel_odd_shape_for(n, out);
}
// The scaled and lifted rotation forms renormalise on the last copy of an unrolled group of blocks, which needs a
// slot count that divides the renormalisation period: the shapes with 2, 4 or 8 slots per lane.
inline bool carousel_has_forms(int n)
{
    CarouselShape f, b;
    return carousel_shape_for(n, &f) && carousel_bwd_shape_for(n, &b) && f.M % 2 == 0 && b.M % 2 == 0;
}

// One-wavefront shapes whose exchange stays inside the wavefront (DPP shifts, no LDS, no barrier): the fewest slots
// per lane in {2, 4, 8} with at most 64 lanes, so multiples of 8 up to 256, 512 and 1024.  A lane then has the least
// work per block, and the block-to-block chain is what bounds the small sweeps these shapes are for.  max_slots: 8
// for the forward sweep, 4 for the reverse sweep (with 8 slots and two strips per lane it does not beat the LDS
// exchange).
inline bool carousel_wave_shape_for(int n, int max_slots, CarouselShape *out)
{
    if (n < kCarouselMinN) return false;
    if (n % 8) return false;   // the kernels unroll 8 blocks (ring of prefetched coefficients)
    for (int m : {2, 4, 8})
        if (m <= max_slots && n % (2 * m) == 0 && n / (2 * m) <= 64) {
            *out = {m, 1};
            return true;
        }
    return false;
}

// What a sweep runs with: shape, columns per lane, and whether the exchange stays inside the wavefront.
struct CarouselPlan {
    CarouselShape s;
    int W;
    bool wave;
};
template <typename T>
inline bool carousel_backward_supported(int n, long long B)
{
    (void)B;
    CarouselShape s;
    return std::is_same<T, float>::value && carousel_bwd_shape_for(n, &s);
}

// Columns per lane of the forward sweep: the widest of {8,4,2,1} that still gives the chip about one wavefront
// per SIMD (measured at n = 256 .. 2048, B = 256 .. 2048: at two per SIMD, the earlier rule, n = 2048 ran
// 1.4 to 1.9 times slower; large batches reach 8 columns either way).
// `widest`: what the shape's registers allow (carousel_fwd_widest).
inline int carousel_width(long long B, int waves, int widest = 8)
{
    const long long want_waves = 1024; // 256 CUs x 4 SIMDs
    for (int w = widest; w > 1; w >>= 1)
        if (((B + w - 1) / w) * waves >= want_waves) return w;
    return 1;
}
// Widest strips whose block loop compiles without register spills.  Workgroups of more than 8 wavefronts have
// 168 (10, 12) or 128 (14, 16) registers per lane instead of 256, which the 7- and 5-slot shapes feel first.
inline int carousel_fwd_widest(const CarouselShape &s)
{
    if (s.M == 7 && s.WAVES > 8) return 4;
    if (s.M == 5 && s.WAVES > 12) return 4;
    return 8;
}
inline int carousel_bwd_widest(const CarouselShape &s)
{
    if (s.M == 7 && s.WAVES > 8) return 2;
    if (s.M == 5 && s.WAVES > 12) return 2;
    // 5 or more slots per lane, an odd number of them, or more than 8 wavefronts: strips of at most 4 columns
    return (s.M > 4 || s.M % 2 || s.WAVES > 8) ? 4 : 8;
}

struct CarouselFwdArgs {
    int n, rows; // rows: the operand's row count (n, or n - 1 when n pads an odd problem)
    long long B;
    CarouselCoefs coefs;
    const float *X;
    float *Y;
    int identity, vec_ok;
    int mirror; // rows relabelled r -> n - r: with mirrored tables the launch applies U^T
    hipStream_t stream;
};

struct CarouselBwdArgs {
    int n, rows;
    long long B, strip0, nstrips, groups;
    CarouselCoefs coefs;
    const float *Y, *G;
    float *dX, *partial;
    const float *zeros; // N floats that are always zero
    float *sink;        // N + 8192 floats that idle lanes write to and nobody reads
    int vec_ok;
    int g_identity; // G is I_n (generated on chip, the pointer is not read)
    hipStream_t stream;
};

// Chained rows of partial sums in the reverse sweep (see carousel_backward_body for what the kernel does).
constexpr int kChainLength = 8;      // workgroups per chain (measured at n = B = 4096, step in ms: 4: 11.97, 8: 11.57, 16: 11.67)
constexpr int kChainMaxPasses = 8;   // strips per workgroup beyond which the rows would outgrow their use
constexpr int kFlagStride = 32;      // words between progress flags: a 128-byte cache line each
struct CarouselChainArgs {
    unsigned *flags;      // [grid][n-1] cache lines of 32 words: word 0 = tag of the launch and pass that finished the block
    unsigned *xcd_of;     // [grid], zero at launch; 1 + XCD number once the workgroup has started
    unsigned *error;      // one word, zero at launch
    const unsigned *epoch; // one word: number of this launch (counted on the device, so that a replayed graph counts
                           // too); the tags of a launch are epoch * (kChainMaxPasses + 1) + pass
    int chains;
};
// Number of chains the reverse sweep of (n, B) links its `groups` persistent workgroups into, or 0 for separate
// rows.  Chains need: the 4-slot LDS-exchange shape with 5 to 8 wavefronts (n from 2112 to 4096) and strips of 8 or 4
// columns; n a multiple of 64; a grid that is a multiple of
// 8 chains of kChainLength (chain members then differ by multiples of 8 and share an XCD); a first pass in which
// every workgroup has a strip; and enough partial sums for their traffic to matter (0.5 GB of separate rows).
inline int carousel_bwd_chains(int n, long long B, long long nstrips, long long groups);
int carousel_backward_chain(const CarouselBwdArgs &a, const CarouselChainArgs &c, int M, int waves, int W);

// Unitary extension in the carousel family (unitary_carousel_kernels.hpp): complex64 operands seen as real
// n x Breal arrays (Breal = 2 B), W real columns per lane (even).  Even n that is a multiple of 16, from
// kUnitaryCarouselMinN up to 4096 (8 slots per lane forward, 4 reverse; the phase pass keeps n float64 in LDS).
constexpr int kUnitaryCarouselMinN = 128;
inline bool unitary_carousel_supported(int n) { return n >= kUnitaryCarouselMinN && n <= 4096 && n % 16 == 0; }

struct UnitaryCarouselFwdArgs {
    int n;
    long long Breal;
    const float2 *rot, *phs, *fin;
    const float *X;
    float *Y;
    int identity, vec_ok;
    hipStream_t stream;
};
struct UnitaryCarouselBwdArgs {
    int n;
    long long Breal, strip0, nstrips, groups;
    const float2 *rot, *phs;
    const float *orient;
    const float2 *fin;
    const float *Y, *G;
    float *dX, *partial; // partial: [2][groups][N]
    const float *zeros;
    float *sink;
    int vec_ok;
    hipStream_t stream;
};
// Defined in unitary_carousel_fwd.hip / unitary_carousel_bwd.hip.  unitary_carousel_coefficients runs the
// phase pass and the table kernel for one sweep direction (q: N 8-byte words, turn: N 4-byte words of scratch; orient may be
// null for the forward direction).
int unitary_carousel_coefficients(int n, const float *theta, const float *phi, int reverse, uint2 *q, unsigned *turn,
                                  float *sgn, float2 *rot, float2 *phs, float *orient, float2 *fin, hipStream_t stream);
int unitary_carousel_forward_m8(const UnitaryCarouselFwdArgs &a, int waves, int W);
int unitary_carousel_backward_m4(const UnitaryCarouselBwdArgs &a, int waves, int W);
int unitary_carousel_backward_m2(const UnitaryCarouselBwdArgs &a, int waves, int W);

// Column family (column_fwd.hip): forward sweep for even n <= 128, one lane per column, standard-form
// table.  GIVENS_ERR_UNSUPPORTED for other n.
constexpr int kColumnFamilyMaxN = 128;
int column_forward(int n, int rows, long long B, const float2 *table, const float *X, float *Y, int identity,
                   int mirror, hipStream_t stream);

// Defined in carousel_fwd_m<M>.hip / carousel_bwd_m<M>.hip: launch the kernel with M slots per lane, `waves`
// wavefronts per workgroup and W columns per lane; GIVENS_ERR_UNSUPPORTED for a combination that is not compiled.
int carousel_forward_m8(const CarouselFwdArgs &a, int waves, int W);
int carousel_forward_m4(const CarouselFwdArgs &a, int waves, int W);
int carousel_forward_m2(const CarouselFwdArgs &a, int waves, int W);
int carousel_backward_m4(const CarouselBwdArgs &a, int waves, int W);
int carousel_backward_m2(const CarouselBwdArgs &a, int waves, int W);
int carousel_backward_m8(const CarouselBwdArgs &a, int waves, int W);
// carousel_fwd_wide.hip / carousel_bwd_wide.hip: more than 8 wavefronts (M in {4, 2})
int carousel_forward_wide(const CarouselFwdArgs &a, int M, int waves, int W);
int carousel_backward_wide(const CarouselBwdArgs &a, int M, int waves, int W);
// odd slot counts: any compiled number of wavefronts, 1 to 8 and 10 to 16
int carousel_forward_m7(const CarouselFwdArgs &a, int waves, int W);
int carousel_forward_m5(const CarouselFwdArgs &a, int waves, int W);
int carousel_forward_m3(const CarouselFwdArgs &a, int waves, int W);
int carousel_backward_m7(const CarouselBwdArgs &a, int waves, int W);
int carousel_backward_m5(const CarouselBwdArgs &a, int waves, int W);
int carousel_backward_m3(const CarouselBwdArgs &a, int waves, int W);

int carousel_forward_wave(const CarouselFwdArgs &a, int M, int W);
int carousel_backward_wave(const CarouselBwdArgs &a, int M, int W);

// Forward sweep.  A size with a one-wavefront shape always takes the wavefront exchange: measured against the LDS
// exchange over n = 256 .. 1024 and B = 64 .. 262144 it is 1.5 to 3.2 times faster with 2 or 4 slots per lane (the
// LDS shapes of those n leave lanes idle) and 1.0 to 1.7 times with 8.  Its strips are single columns while the
// batch gives each SIMD at most one wavefront, then 2, 4 and 8 columns: every wavefront reads the whole coefficient
// table, and beyond about a thousand wavefronts that traffic (L2) sets the time.
inline bool carousel_fwd_plan(int n, long long B, CarouselPlan *p)
{
    if (!carousel_shape_for(n, &p->s)) return false;
    p->W = carousel_width(B, p->s.WAVES, carousel_fwd_widest(p->s));
    p->wave = false;
    CarouselShape ws;
    if (carousel_wave_shape_for(n, 8, &ws)) {
        const long long single = ws.M == 8 ? 512 : 1024;     // widest batch of single-column strips
        *p = {ws, B <= single ? 1 : B <= 4 * single ? 2 : B <= 16 * single ? 4 : 8, true};
    }
    return true;
}

inline int carousel_forward(int n, int rows, long long B, const CarouselCoefs &coefs, const float *X, float *Y,
                            int identity, int mirror, hipStream_t stream)
{
    CarouselPlan plan;
    if (!carousel_fwd_plan(n, B, &plan)) return GIVENS_ERR_UNSUPPORTED;
    const CarouselShape s = plan.s;
    const int W = plan.W;
    const bool aligned = (B % 4 == 0) && (reinterpret_cast<uintptr_t>(Y) % 16 == 0) &&
                         (identity || reinterpret_cast<uintptr_t>(X) % 16 == 0);
    const CarouselFwdArgs a{n, rows, B, coefs, X, Y, identity, aligned ? 1 : 0, mirror, stream};
    if (plan.wave) return carousel_forward_wave(a, s.M, W);
    switch (s.M) {
    case 7: return carousel_forward_m7(a, s.WAVES, W);
    case 5: return carousel_forward_m5(a, s.WAVES, W);
    case 3: return carousel_forward_m3(a, s.WAVES, W);
    default: break;
    }
    if (s.WAVES > 8) return carousel_forward_wide(a, s.M, s.WAVES, W);
    switch (s.M) {
    case 8: return carousel_forward_m8(a, s.WAVES, W);
    case 4: return carousel_forward_m4(a, s.WAVES, W);
    case 2: return carousel_forward_m2(a, s.WAVES, W);
    default: return GIVENS_ERR_UNSUPPORTED;
    }
}

// Columns per workgroup of the reverse sweep.  Fewer, wider strips mean fewer rows of partial sums to write,
// add to and reduce, and a workgroup's time per block grows slowly with its width (a lone workgroup is bound
// by the latency of its exchange, not by arithmetic): the widest of {8, 4, 2} that still gives the chip 512
// wavefronts, and 2 below that (measured at n = 256 .. 2048, B = 256 .. 2048: 1.1 to 1.8 times faster than
// the forward sweep's rule).
inline bool carousel_bwd_plan(int n, long long B, CarouselPlan *p)
{
    if (!carousel_bwd_shape_for(n, &p->s)) return false;
    p->wave = false;
    p->W = B > 1 ? 2 : 1;
    for (int w = carousel_bwd_widest(p->s); w > 2; w >>= 1)
        if (((B + w - 1) / w) * p->s.WAVES >= 512) {
            p->W = w;
            break;
        }
    // wavefront exchange: n up to 512 and batches up to 4096 columns (measured 1.2 to 2.1 times faster, sweep and
    // second stage together; each strip costs a row of partial sums, hence wider strips sooner than forward)
    CarouselShape ws;
    if (B <= 4096 && carousel_wave_shape_for(n, 4, &ws)) *p = {ws, B <= 256 ? 1 : B <= 1024 ? 2 : 4, true};
    return true;
}
inline int carousel_bwd_width(int n, long long B)
{
    CarouselPlan p;
    return carousel_bwd_plan(n, B, &p) ? p.W : 0;
}

// Number of persistent workgroups the reverse sweep runs with: what the chip holds at once (the
// kernel is limited to two wavefronts per SIMD by its registers), or one per strip if that is fewer.
inline long long carousel_bwd_groups(int n, long long B, long long nstrips, int compute_units)
{
    CarouselPlan p;
    if (!carousel_bwd_plan(n, B, &p)) return 0;
    const CarouselShape s = p.s;
    const long long resident = (long long)compute_units * (8 / s.WAVES > 0 ? 8 / s.WAVES : 1);
    return nstrips < resident ? nstrips : resident;
}

inline int carousel_bwd_chains(int n, long long B, long long nstrips, long long groups)
{
    CarouselPlan p;
    if (!carousel_bwd_plan(n, B, &p) || p.wave || p.s.M != 4 || (p.W != 8 && p.W != 4)) return 0;
    if (p.s.WAVES < 5 || p.s.WAVES > 8) return 0;   // one workgroup per compute unit (see CarouselBwd)
    // (a row's blocks must start on cache-line boundaries: a line that straddles two blocks could be read into a
    // successor's L1 before the predecessor has written its second half)
    if (n % 64 != 0 || groups % (8 * kChainLength) != 0 || nstrips < groups) return 0;
    if ((nstrips + groups - 1) / groups > kChainMaxPasses) return 0;
    const long long N = (long long)n * (n - 1) / 2;
    if (N * groups * 4 < (512ll << 20)) return 0;
    return (int)(groups / kChainLength);
}

// Launches the reverse sweep on strips [strip0, strip0 + nstrips) with `groups` persistent workgroups.
// partial is [groups][N]: workgroup g stores the sums of its first strip in row g and adds those of its later
// strips to them.  zeros: N floats that stay zero.
inline int carousel_backward_strips(int n, int rows, long long B, int W, long long strip0, long long nstrips,
                                    long long groups, const CarouselCoefs &coefs, const float *Y, const float *G,
                                    float *dX, float *partial, const float *zeros, float *sink, int g_identity,
                                    hipStream_t stream, const CarouselChainArgs *chain = nullptr)
{
    CarouselPlan plan;
    if (!carousel_bwd_plan(n, B, &plan) || plan.W != W) return GIVENS_ERR_UNSUPPORTED;
    const CarouselShape s = plan.s;
    const bool aligned = (B % 4 == 0) && (reinterpret_cast<uintptr_t>(Y) % 16 == 0) &&
                         (g_identity || reinterpret_cast<uintptr_t>(G) % 16 == 0) &&
                         (!dX || reinterpret_cast<uintptr_t>(dX) % 16 == 0);
    const CarouselBwdArgs a{n,  rows,    B,     strip0, nstrips,         groups,     coefs, Y, G,
                            dX, partial, zeros, sink,   aligned ? 1 : 0, g_identity, stream};
    if (chain) return carousel_backward_chain(a, *chain, s.M, s.WAVES, W);
    if (plan.wave) return carousel_backward_wave(a, s.M, W);
    switch (s.M) {
    case 7: return carousel_backward_m7(a, s.WAVES, W);
    case 5: return carousel_backward_m5(a, s.WAVES, W);
    case 3: return carousel_backward_m3(a, s.WAVES, W);
    default: break;
    }
    if (s.WAVES > 8) return carousel_backward_wide(a, s.M, s.WAVES, W);
    switch (s.M) {
    case 8: return carousel_backward_m8(a, s.WAVES, W);
    case 4: return carousel_backward_m4(a, s.WAVES, W);
    case 2: return carousel_backward_m2(a, s.WAVES, W);
    default: return GIVENS_ERR_UNSUPPORTED;
    }
}

} // namespace givens
