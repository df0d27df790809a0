/*
 * givens_rr.h -- C ABI of the round-robin Givens library for MI355X (gfx950).
 *
 * The library applies an angle-parametrised special orthogonal matrix
 *
 *     U(theta) = G^{e_1}(theta_{e_1}) G^{e_2}(theta_{e_2}) ... G^{e_N}(theta_{e_N}),   N = n(n-1)/2,
 *
 * (paper Section 2, Eq. (2); G^{e_N} is applied first) to an n x B operand, where the pair
 * sequence E is the round-robin sequence produced by the circle method (Section 3, Figure 1):
 * n-1 blocks b_1..b_{n-1} of n/2 disjoint pairs, so that each block is one parallel step
 * (Algorithm 2).  It also runs the reverse sweep that yields dL/dtheta (the quantity
 * Algorithm 3 computes) and dL/dX without stored activations.
 *
 * Conventions shared by every entry point
 *   - n is even, n >= 2.  Coordinates are 0..n-1.  A pair is written (i, j) with i < j and
 *     G^e has G_ii = G_jj = cos, G_ij = -sin, G_ji = +sin (Section 2).
 *   - theta and dtheta have N entries in E order: entry k*(n/2)+p belongs to arc p of block
 *     b_{k+1}, i.e. to rr_schedule's pairs[k][p].
 *   - Matrices are row-major n x B with leading dimension B: a row is a coordinate that gets
 *     rotated, a column is one vector of the batch.
 *   - Unless marked "host", pointers are DEVICE pointers owned by the caller; the library
 *     neither frees nor retains them.  `stream` is a hipStream_t passed as void* (NULL = the
 *     default stream).  Calls are asynchronous on that stream.
 *   - The library owns one workspace per (device, stream) it has been called on (coefficient tables,
 *     partial gradients), grown on demand with hipMalloc and released by givens_release().  Calls on
 *     different streams use different workspaces and may overlap; calls on one stream are ordered by
 *     that stream.  At most 8 streams per device keep a workspace: a ninth gives up the one used
 *     longest ago (after a device-wide synchronisation).
 *   - Return value: 0 on success, a negative GIVENS_ERR_* code otherwise.  Nothing is launched
 *     when an argument check fails.  No exceptions, no aborts.
 */
#ifndef GIVENS_RR_H
#define GIVENS_RR_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define GIVENS_OK 0
#define GIVENS_ERR_BAD_N (-1)       /* n < 2 or n odd                                   */
#define GIVENS_ERR_BAD_B (-2)       /* B < 1                                            */
#define GIVENS_ERR_NULL (-3)        /* a required pointer is NULL                       */
#define GIVENS_ERR_HIP (-4)         /* a HIP call failed; see givens_last_hip_error()   */
#define GIVENS_ERR_UNSUPPORTED (-5) /* shape not supported by the requested kernel      */
#define GIVENS_ERR_ALIAS (-6)       /* forbidden aliasing between arguments             */
#define GIVENS_ERR_BAD_M (-7)       /* restricted entry points: m outside 1..n-1        */
#define GIVENS_ERR_STALE (-8)       /* prepared calls: the token's tables are gone      */

/* Kernel families (givens_set_kernel). */
#define GIVENS_KERNEL_AUTO 0     /* column kernels for n <= 128, register carousel where the  */
                                 /* shape allows, else LDS strip                              */
#define GIVENS_KERNEL_LDS 1      /* strip of the operand held in LDS; any even n that fits   */
#define GIVENS_KERNEL_CAROUSEL 2 /* strip held in VGPRs in circle-method position order: float, */
                                 /* n from 132, a multiple of 4 up to 4096 or of 8 up to 8192,  */
                                 /* or n = 2 M L with M in {7, 5, 3} and L <= 1024 (standard    */
                                 /* rotation form only, whatever givens_set_rotation_form says) */
#define GIVENS_KERNEL_COLUMN 3   /* float, n <= 128: one lane per column, all rows in its VGPRs */

/* Rotation forms of the float carousel kernels (givens_set_rotation_form). */
#define GIVENS_FORM_AUTO 0     /* GIVENS_FORM_RANGE where the sweeps are long enough to pay for its extra       */
                               /* coefficient work (n (n-1)/2 * B >= 1e9 updates; always in givens_prepare),    */
                               /* GIVENS_FORM_STANDARD below that                                               */
#define GIVENS_FORM_STANDARD 1 /* r_i = c U_i - s U_j, r_j = s U_i + c U_j exactly as in Algorithm 1         */
#define GIVENS_FORM_SCALED 2   /* same rotations on rows kept divided by their accumulated cosines (2 FMAs)  */
#define GIVENS_FORM_LIFTED 3   /* same rotations as three shears (3 FMAs), angles reduced modulo pi           */
#define GIVENS_FORM_RANGE 4    /* decided on the device from max |theta|: scaled if <= pi/4, lifted if <= 1e6,  */
                               /* standard otherwise (including NaN)                                          */

/* How givens_backward sums the per-strip shares of dtheta (givens_set_reduction). */
#define GIVENS_REDUCTION_AUTO 0      /* the library's default for the kernel family in use                     */
#define GIVENS_REDUCTION_TWO_STAGE 1 /* one partial sum per (strip, angle), then a fixed-order pass: reproducible */
                                     /* (large float sweeps, n = 2112 .. 4096: the sweep's persistent workgroups */
                                     /* are chained and add their sums into shared rows, in a fixed order too;   */
                                     /* should a workgroup's bounded wait for its predecessor ever run out, the  */
                                     /* call cannot report it, being asynchronous: dtheta is then all NaN)       */
#define GIVENS_REDUCTION_GRAM 3      /* C = Y G^T by the library's float32 MFMA kernel, then the sweep on the    */
                                     /* n x n operand C; dX by a forward-type sweep (float entry points)        */

/*
 * rr_schedule -- the round-robin sequence by the circle method (Section 3; the worked n = 6
 * example is Eq. (3), the dimension sequences are the left column of Figure 1).
 * Start from (0, 1, ..., n-1); block k pairs position p with position n-1-p of the current sequence,
 * p = 0 (the outermost arc) first; then element 0 is held and the last element moves to position 1.
 *   pairs : HOST buffer of (n-1)*(n/2)*2 int32, written as pairs[k][p][0] = i, pairs[k][p][1] = j.
 * Pure host integer work; bit-exact by definition.
 */
int rr_schedule(int n, int32_t *pairs);

/*
 * givens_forward -- Y = U(theta) X  (Algorithm 2 started from X instead of I_n).
 *   theta : N floats.   X : n x B.   Y : n x B, may be the same buffer as X (in place).
 *   Partial overlap of X and Y is not checked and not allowed.
 */
int givens_forward(int n, int64_t B, const float *theta, const float *X, float *Y, void *stream);

/*
 * givens_build -- U = U(theta), n x n  (Algorithm 2 as printed: the operand is I_n, which is
 * generated on chip and never read from memory).
 */
int givens_build(int n, const float *theta, float *U, void *stream);

/*
 * givens_backward -- reverse sweep for L with upstream gradient G = dL/dY.
 * Takes the forward OUTPUT Y (not X): the state before each block is recovered by applying the
 * block's transposed rotations, so no activation is stored.  For block k = 1..n-1 in order and
 * every pair e = (i, j) of the block:
 *     dtheta_e = sum_b ( gbar_{j,b} z_{i,b} - gbar_{i,b} z_{j,b} ),
 * then z <- G^{b_k}^T z and gbar <- G^{b_k}^T gbar, with z = Y and gbar = G at the start
 * (Section 4.1: dU/dtheta_e = U^{1:k-1} Q_e U^{k:n-1}; this is the quantity of Algorithm 3
 * with dL/dU = G X^T).  At the end gbar = dL/dX = U^T G.
 *   Y, G : n x B.   dX : n x B, may be the same buffer as G.   dtheta : N floats, overwritten.
 *   dX may be NULL (only dtheta is wanted).
 */
int givens_backward(int n, int64_t B, const float *theta, const float *Y, const float *G,
                    float *dX, float *dtheta, void *stream);

/*
 * givens_forward_transposed -- Y = U(theta)^T X, i.e. the inverse transform (U is orthogonal): the
 * transposed rotations applied in E order, which is also what givens_backward computes for dX.  Run as
 * the forward sweep of the mirrored problem: relabelling row r >= 1 as n - r maps the pairs of block k
 * onto those of block n-2-k (Section 3's circle method is symmetric under this reflection), so
 * U(theta)^T = P^T U(theta') P with theta'[k][p] = -/+ theta[n-2-k][p].  Same arguments as givens_forward.
 */
int givens_forward_transposed(int n, int64_t B, const float *theta, const float *X, float *Y, void *stream);
int givens_forward_transposed_f64(int n, int64_t B, const double *theta, const double *X, double *Y, void *stream);

/*
 * givens_forward_noalloc -- givens_forward for callers that cannot allocate device memory: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels
 * and bit-identical results, but the coefficient tables (cos/sin or scaled / lifted coefficients, row
 * factors, renormalisation rows, the range-check flag) are written to a static device array of
 * GIVENS_NOALLOC_BYTES bytes inside the library instead of the hipMalloc'ed workspace, so the call makes
 * no hipMalloc, hipFree or other allocating call.  Every GPU the library runs on holds that array until
 * the process ends.
 *   n even, 2 <= n <= GIVENS_NOALLOC_MAX_N (larger n: GIVENS_ERR_UNSUPPORTED, nothing launched); any B >= 1.
 *   All calls on one GPU share the array: calls that overlap on one GPU (two streams, two threads) race.
 *   Nothing in it needs clearing between calls: every word a call reads it has written first, except the
 *   flag word of the range check, which must start at zero: two words take turns, the array starts all zero,
 *   and each call's range kernel zeroes the word the next call will use.
 *   Per-kernel timing (givens_set_timing) is not recorded for this call.
 */
#define GIVENS_NOALLOC_MAX_N 1024
#define GIVENS_NOALLOC_BYTES 8446208 /* flag words, table, row factors, renormalisation rows at n = 1024 */
int givens_forward_noalloc(int n, int64_t B, const float *theta, const float *X, float *Y, void *stream);

/*
 * Per-call choices.  givens_forward_ex / givens_backward_ex are givens_forward_restricted /
 * givens_backward_restricted (any n >= 2, m = n - 1 for the unrestricted parametrisation) with the kernel
 * family, rotation form and reduction taken from `options` instead of the process-wide givens_set_* settings
 * (options == NULL: those settings).  givens_forward_ex with X == NULL builds U (B must equal n).
 * An unknown value in `options` returns GIVENS_ERR_UNSUPPORTED.
 */
typedef struct givens_options {
    int kernel;        /* GIVENS_KERNEL_*    */
    int rotation_form; /* GIVENS_FORM_AUTO, _STANDARD or _LIFTED */
    int reduction;     /* GIVENS_REDUCTION_* */
} givens_options;
int givens_forward_ex(int n, int m, int64_t B, const float *theta, const float *X, float *Y, void *stream,
                      const givens_options *options);
int givens_backward_ex(int n, int m, int64_t B, const float *theta, const float *Y, const float *G, float *dX,
                       float *dtheta, void *stream, const givens_options *options);

/*
 * Prepared coefficients (float).  Everything the sweeps need that depends on theta alone -- the range check
 * that picks the rotation form and the coefficient tables of Algorithm 2's blocks, for the forward sweep, the
 * reverse sweep (Section 4.1) or both -- is built once by givens_prepare in the workspace of `stream`, and
 * the *_prepared calls then run only the sweeps: a layer calls givens_prepare in its forward pass and reuses
 * the tables in its backward pass (theta cannot change in between), and a model that is only evaluated
 * prepares once per change of theta.  givens_prepare returns a positive token (or a negative error code).
 * The tables stay valid until another call on the same stream writes the same coefficient set: a plain
 * forward / build call replaces the forward set, a plain backward call the reverse set, givens_prepare
 * both; givens_release drops everything.  A *_prepared call whose token is no longer the workspace's, whose
 * direction was not prepared or lost, or which asks (through givens_set_kernel) for another kernel family
 * than the tables were built for returns GIVENS_ERR_STALE and launches nothing: call the plain entry point
 * instead.  The token must be used on the stream it was prepared on.
 *   directions : GIVENS_PREPARE_FORWARD, GIVENS_PREPARE_BACKWARD or both (or-ed).  GIVENS_PREPARE_BACKWARD_WIDE
 *     (implies _BACKWARD) also builds the tables of the forward-type sweep that computes dX in the Gram form,
 *     which the backward call takes for B >= 2 n; without it givens_backward_prepared runs the two-stage sweep
 *     over all B columns whatever B is (and returns GIVENS_ERR_STALE if the Gram form is forced).
 *   n, m, B, X, Y, U, G, dX, dtheta : as for the plain calls; n and m are those of givens_prepare.
 */
#define GIVENS_PREPARE_FORWARD 1
#define GIVENS_PREPARE_BACKWARD 2
#define GIVENS_PREPARE_BACKWARD_WIDE 4
int64_t givens_prepare(int n, const float *theta, int directions, void *stream);
int64_t givens_prepare_restricted(int n, int m, const float *theta, int directions, void *stream);
/* The same with per-call options (NULL: the process-wide defaults) and the batch the tables will be used with
 * (batch_hint >= 1; 0: not known), which GIVENS_FORM_AUTO needs for its size rule; m = n - 1: unrestricted. */
int64_t givens_prepare_ex(int n, int m, const float *theta, int directions, int64_t batch_hint, void *stream,
                          const givens_options *options);
int givens_forward_prepared(int64_t token, int64_t B, const float *X, float *Y, void *stream);
int givens_build_prepared(int64_t token, float *U, void *stream);
int givens_backward_prepared(int64_t token, int64_t B, const float *Y, const float *G, float *dX, float *dtheta,
                             void *stream);

/* float64 variants: same semantics, all arrays double. */
int givens_forward_f64(int n, int64_t B, const double *theta, const double *X, double *Y, void *stream);
int givens_build_f64(int n, const double *theta, double *U, void *stream);
int givens_backward_f64(int n, int64_t B, const double *theta, const double *Y, const double *G,
                        double *dX, double *dtheta, void *stream);

/*
 * Restricted parametrisation and odd n.
 *
 * Section 5 of the paper ("Restricting the Parametrization"): for an integer 1 <= m <= n-1 no
 * rotation is performed among the coordinates m..n-1, i.e. of the pairs (i, j), i < j, only those
 * with i < m are free: N(n, m) = m n - m (m + 1) / 2 angles (n = 8, m = 4: 22).  The blocks are still
 * the n-1 blocks of the circle method; the pairs that are not free are bypassed.  m = n-1 is the
 * unrestricted case.  End of Section 3 (and of Section 4.2 for the gradient): odd n is run on the
 * circle method's sequence for n+1 dimensions, bypassing every pair that contains the added one, so
 * there are n blocks of at most (n-1)/2 pairs.  Both conditions combine.
 *
 * These entry points accept any n >= 2, odd or even.  theta and dtheta have N(n, m) entries: the
 * free pairs in the order in which the sequence E lists them (rr_schedule_restricted).  The kernels
 * run a bypassed pair as a rotation by zero, so the cost is that of the unrestricted problem of
 * n (or n+1) dimensions.  Everything else -- layouts, aliasing, streams, errors -- is as for the
 * unrestricted entry points; m outside 1..n-1 returns GIVENS_ERR_BAD_M; n beyond what any kernel
 * family takes (36864) returns GIVENS_ERR_UNSUPPORTED before anything is allocated.  The map from the
 * entries of E to the indices in theta is built on the device, by kernels on the caller's stream, the
 * first time a workspace sees (n, m) and whenever another (n, m) has used it in between.
 */
int64_t givens_num_angles(int n, int m);                         /* N(n, m), or a negative error code  */
int rr_schedule_restricted(int n, int m, int32_t *pairs);        /* HOST buffer of N(n, m) * 2 int32   */
int givens_forward_restricted(int n, int m, int64_t B, const float *theta, const float *X, float *Y,
                              void *stream);
int givens_build_restricted(int n, int m, const float *theta, float *U, void *stream);
int givens_backward_restricted(int n, int m, int64_t B, const float *theta, const float *Y, const float *G,
                               float *dX, float *dtheta, void *stream);
int givens_forward_restricted_f64(int n, int m, int64_t B, const double *theta, const double *X, double *Y,
                                  void *stream);
int givens_build_restricted_f64(int n, int m, const double *theta, double *U, void *stream);
int givens_backward_restricted_f64(int n, int m, int64_t B, const double *theta, const double *Y,
                                   const double *G, double *dX, double *dtheta, void *stream);

/*
 * Unitary extension (the paper's appendix "Adaptations to U(n)").  Every pair e = (i, j), i < j, has a
 * rotation angle theta_e and a phase angle phi_e, and its factor is the identity except for
 *     G_ii = exp(i phi) cos(theta),  G_ij = -sin(theta),  G_ji = exp(i phi) sin(theta),  G_jj = cos(theta)
 * (the appendix's forward algorithm: r_i = exp(i phi) cos U_i - sin U_j, r_j = exp(i phi) sin U_i + cos U_j);
 * U = G^{e_1} ... G^{e_N} over the same round-robin sequence E, n even.
 *   theta, phi, dtheta, dphi : N reals in E order.
 *   X, Y, U, G, dX : complex, row-major n x B (n x n for U), each element stored as (re, im): 2 n B reals.
 * givens_unitary_backward takes the forward output Y and the upstream gradient G = dL/dRe(Y) + i dL/dIm(Y)
 * of a real loss L (dL = Re sum conj(G) dY) and returns dL/dtheta, dL/dphi and dX = U^dagger G (dX may be
 * NULL, may be the buffer of G).  Per pair of block k, with z and gbar the carried strips:
 *     dtheta_e = Re sum_b ( conj(gbar_j) z_i - conj(gbar_i) z_j ),  dphi_e = Re <gbar, P_e z>
 * (Q_e and P_e of the appendix), then the block is undone with the adjoint factors.
 * Kernel families: the float entry points run in the register-carousel family when n is a multiple of 16 from
 * 128 to 4096 (the phases are then carried as per-row angles, prepared by a sequential pass over the blocks, and phi
 * is rounded to 2 pi / 2^32 on the way), otherwise and for float64 in the LDS strip family; givens_set_kernel
 * (GIVENS_KERNEL_LDS / GIVENS_KERNEL_CAROUSEL) forces one, and GIVENS_ERR_UNSUPPORTED is returned for a shape the
 * forced family does not cover.  Aliasing, streams and errors as elsewhere.
 */
int givens_unitary_forward(int n, int64_t B, const float *theta, const float *phi, const float *X, float *Y,
                           void *stream);
int givens_unitary_build(int n, const float *theta, const float *phi, float *U, void *stream);
int givens_unitary_backward(int n, int64_t B, const float *theta, const float *phi, const float *Y, const float *G,
                            float *dX, float *dtheta, float *dphi, void *stream);
int givens_unitary_forward_f64(int n, int64_t B, const double *theta, const double *phi, const double *X,
                               double *Y, void *stream);
int givens_unitary_build_f64(int n, const double *theta, const double *phi, double *U, void *stream);
int givens_unitary_backward_f64(int n, int64_t B, const double *theta, const double *phi, const double *Y,
                                const double *G, double *dX, double *dtheta, double *dphi, void *stream);

/* Frees every workspace the library holds (all devices).  Synchronises the devices it touches. */
int givens_release(void);

/* hipError_t value of the last failed HIP call made by the library on this thread (0 if none). */
int givens_last_hip_error(void);

/* Static, human-readable text for a GIVENS_ERR_* code. */
const char *givens_error_string(int code);

/* Selects the kernel family for subsequent calls (process-wide).  Returns the previous value,
 * or GIVENS_ERR_UNSUPPORTED for an unknown value.  With GIVENS_KERNEL_CAROUSEL or GIVENS_KERNEL_COLUMN a
 * call whose shape those kernels do not cover returns GIVENS_ERR_UNSUPPORTED instead of falling back.
 * The column family has a forward kernel only: its backward call uses the Gram-matrix reduction (see
 * givens_set_reduction) with the sweep on the n x n Gram matrix done by the LDS family, and the LDS
 * family outright when that reduction is not available or not selected. */
int givens_set_kernel(int which);

/* Which family the last successful forward/build/backward call on this thread used
 * (GIVENS_KERNEL_LDS, GIVENS_KERNEL_CAROUSEL or GIVENS_KERNEL_COLUMN; 0 before any call). */
int givens_last_kernel(void);

/*
 * The float carousel kernels have three arithmetically equivalent forms of the same Givens update
 * (Algorithm 1's loop body).  The scaled form keeps every row divided by the product of the cosines it
 * has met, which turns an update into two FMAs, and multiplies the rows back every 64 blocks; it is
 * used only when every |theta| <= pi/4.  The lifted form writes the rotation as three shears (three
 * FMAs) after reducing the angle modulo pi, carrying the resulting signs the same way; it is used for
 * larger finite angles.  A device-side check of theta decides per call.
 * givens_set_rotation_form(GIVENS_FORM_STANDARD) switches the check and both other forms off,
 * GIVENS_FORM_LIFTED keeps the check but never picks the scaled form (process-wide; GIVENS_FORM_SCALED
 * cannot be forced); returns the previous setting.  givens_last_rotation_form() reports which form the
 * last forward/build/backward call on this thread ran (it reads the device flag back and waits for
 * that call's stream).  Other kernel families and the f64 entry points always use the standard form.
 */
int givens_set_rotation_form(int which);
int givens_last_rotation_form(void);

/*
 * Selects how the reverse sweep reduces over strips (process-wide); returns the previous setting.
 * TWO_STAGE keeps one row of 4*N bytes of partial sums per resident workgroup of the carousel sweep
 * (at most 256 rows on this chip: 8.6 GB at n = 4096, whatever B is) or per strip of the LDS family,
 * capped at 24 GiB per chunk, and gives bit-identical dtheta from run to run.  GRAM replaces the sweep
 * over B columns by the Gram matrix C = Y G^T (the sums of the sweep are those of the same sweep on the
 * operand C with upstream gradient I_n), contracted over B by the library's own float32 MFMA kernel in a
 * fixed order (reproducible as well), and computes dX = U^T G by a forward-type sweep.  AUTO means GRAM for
 * every float kernel family when B >= 2 n, TWO_STAGE otherwise; the f64 entry points always use TWO_STAGE.
 * givens_last_reduction() reports what the last backward call on this thread did.
 */
int givens_set_reduction(int which);
int givens_last_reduction(void);

/*
 * givens_last_chains() -- how the last two-stage reverse sweep on this thread laid out its partial sums: the number
 * of chains its persistent workgroups were linked into (each chain sums into one shared row per pass; the kernel is
 * then carousel_backward_chain_kernel), or 0 when every workgroup or strip kept a row of its own.  Section 4.2
 * (the row sums across columns); reporting only.
 */
int givens_last_chains(void);

/*
 * Per-kernel timing.  givens_set_timing(1) makes every subsequent call record HIP events on the
 * caller's stream around each group of kernels it launches.  givens_last_timing() waits for the events of
 * the last call on this thread and writes milliseconds: ms[0] = coefficient kernels (range check, tables),
 * ms[1] = sweep kernel(s), ms[2] = dtheta second-stage reduction, ms[3] = Gram-matrix contraction and its
 * slice sum (ms[2], ms[3]: 0 for forward/build).  Returns GIVENS_ERR_UNSUPPORTED if timing was off for that call.
 */
int givens_set_timing(int on);
int givens_last_timing(float ms[4]);

#ifdef __cplusplus
}
#endif
#endif /* GIVENS_RR_H */
