/*
 * CPU oracle (plain C, float64) for full-size checks and for the benchmark's CPU baseline.
 *
 * TEST INFRASTRUCTURE ONLY: nothing in the product path links or loads this file.
 * It shares no code with the HIP kernels and never sees a value they computed.
 *
 * What it computes is exactly what oracle/givens_oracle.py computes, for sizes where
 * NumPy is too slow.  The arithmetic per matrix column is the paper's, in the paper's
 * order; the only arrangement added is that columns are taken in groups of CB and the
 * groups are shared among threads.  Columns never interact in any of these algorithms
 * (a Givens factor only mixes two rows of the multiplicand, Section 2), so this changes
 * no floating-point operation and no order of operations within a column.  The one
 * exception is the final sum over columns in the two gradient routines, which is taken
 * group by group, then thread by thread in thread-index order.
 *
 *   oracle_schedule          Section 3, circle method (Figure 1): blocks b_1..b_{n-1}
 *   oracle_forward           Algorithm 1 over reversed(E), started from X (or I_n)
 *   oracle_grad_operand      dL/dX = U^T G: transposed rotations in E order
 *   oracle_reverse_sweep     operand-side gradient: for block k = 1..n-1, first
 *                            dtheta_e = sum_b (gbar_j z_i - gbar_i z_j), then z, gbar <- G^{b_k}^T z, gbar
 *                            (Section 4.1: dU/dtheta_e = U^{1:k-1} Q_e U^{k:n-1})
 *   oracle_*_pairs           the three routines above for any sequence E of pairs and any n >= 2:
 *                            the free pairs of a restricted parametrisation (Section 5) or of
 *                            odd n (end of Section 3), listed by oracle/restricted_oracle.py
 *   oracle_grad_theta_alg3   Algorithm 3 with the (parallel) index l taken outermost:
 *                            per l, row l of U^fwd and column l of M are rotated for the
 *                            block, then A[m(e), l] = M[i,l] u[l,j] - M[j,l] u[l,i];
 *                            the row sums of A are accumulated over l
 *
 * Pins: tests/test_oracle_c.py compares every routine with the NumPy oracle (itself
 * pinned to the paper's worked example, closed forms and finite differences) and
 * re-checks orthogonality and the zero-gradient case at sizes NumPy cannot reach.
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC (see oracle/build_oracle.py).  No -ffast-math:
 * the compiler must not reassociate.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define CB 32 /* columns per group */

static int bad_n(int n) { return n < 2 || (n & 1); }

/* Section 3 / Figure 1: hold seq[0], move the last element to position 1 at each shift;
 * block k pairs seq[p] with seq[n-1-p], written smaller index first. */
int oracle_schedule(int n, int32_t *pairs)
{
    if (bad_n(n) || !pairs) return -1;
    int32_t *seq = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
    if (!seq) return -2;
    for (int p = 0; p < n; ++p) seq[p] = p;
    int half = n / 2;
    for (int k = 0; k < n - 1; ++k) {
        for (int p = 0; p < half; ++p) {
            int32_t a = seq[p], b = seq[n - 1 - p];
            pairs[((size_t)k * half + p) * 2 + 0] = a < b ? a : b;
            pairs[((size_t)k * half + p) * 2 + 1] = a < b ? b : a;
        }
        int32_t last = seq[n - 1];
        memmove(seq + 2, seq + 1, sizeof(int32_t) * (size_t)(n - 2));
        seq[1] = last;
    }
    free(seq);
    return 0;
}

static void set_threads(int nthreads)
{
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#else
    (void)nthreads;
#endif
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static int make_cs(long count, const double *theta, double **c, double **s)
{
    *c = (double *)malloc(sizeof(double) * (size_t)count);
    *s = (double *)malloc(sizeof(double) * (size_t)count);
    if (!*c || !*s) { free(*c); free(*s); return -2; }
    for (long e = 0; e < count; ++e) { (*c)[e] = cos(theta[e]); (*s)[e] = sin(theta[e]); }
    return 0;
}

/* copy columns [b0, b0+w) of an n x B matrix into an n x CB buffer (and back) */
static void load_group(int n, long B, const double *src, long b0, int w, double *buf)
{
    for (int r = 0; r < n; ++r)
        for (int x = 0; x < w; ++x) buf[(size_t)r * CB + x] = src[(size_t)r * B + b0 + x];
}
static void store_group(int n, long B, double *dst, long b0, int w, const double *buf)
{
    for (int r = 0; r < n; ++r)
        for (int x = 0; x < w; ++x) dst[(size_t)r * B + b0 + x] = buf[(size_t)r * CB + x];
}

/* Algorithm 1 over a given sequence E of `count` pairs.  X == NULL means the operand is I_n (then B
 * must equal n). */
static int forward_impl(int n, long B, long count, const double *theta, const int32_t *pairs,
                        const double *X, double *Y, int nthreads)
{
    if (n < 2 || count < 0 || B < 1 || !theta || !pairs || !Y) return -1;
    if (!X && B != n) return -1;
    double *c, *s;
    if (make_cs(count, theta, &c, &s)) return -2;
    set_threads(nthreads);
    long groups = (B + CB - 1) / CB;
    int fail = 0;
#pragma omp parallel
    {
        double *u = (double *)malloc(sizeof(double) * (size_t)n * CB);
        if (!u) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (long g = 0; g < groups; ++g) {
            if (!u) continue;
            long b0 = g * CB;
            int w = (int)((B - b0) < CB ? (B - b0) : CB);
            memset(u, 0, sizeof(double) * (size_t)n * CB);
            if (X) load_group(n, B, X, b0, w, u);
            else {
                for (int x = 0; x < w; ++x) u[(size_t)(b0 + x) * CB + x] = 1.0;
            }
            for (long e = count - 1; e >= 0; --e) {          /* reversed(E) */
                double *ui = u + (size_t)pairs[2 * e] * CB;
                double *uj = u + (size_t)pairs[2 * e + 1] * CB;
                double ce = c[e], se = s[e];
                for (int x = 0; x < CB; ++x) {
                    double ri = ce * ui[x] - se * uj[x];
                    double rj = se * ui[x] + ce * uj[x];
                    ui[x] = ri;
                    uj[x] = rj;
                }
            }
            store_group(n, B, Y, b0, w, u);
        }
        free(u);
    }
    free(c); free(s);
    return fail ? -2 : 0;
}

int oracle_forward(int n, long B, const double *theta, const int32_t *pairs,
                   const double *X, double *Y, int nthreads)
{
    if (bad_n(n)) return -1;
    return forward_impl(n, B, (long)n * (n - 1) / 2, theta, pairs, X, Y, nthreads);
}

/* The same for the free pairs of a restricted parametrisation or of odd n (Section 5; end of
 * Section 3): E is whatever sequence of pairs the caller lists, any n >= 2. */
int oracle_forward_pairs(int n, long B, long count, const double *theta, const int32_t *pairs,
                         const double *X, double *Y, int nthreads)
{
    return forward_impl(n, B, count, theta, pairs, X, Y, nthreads);
}

/* dL/dX = U^T G: G^{e_1}^T applies first, so the loop runs over E in order. */
static int grad_operand_impl(int n, long B, long count, const double *theta, const int32_t *pairs,
                             const double *G, double *dX, int nthreads)
{
    if (n < 2 || count < 0 || B < 1 || !theta || !pairs || !G || !dX) return -1;
    double *c, *s;
    if (make_cs(count, theta, &c, &s)) return -2;
    set_threads(nthreads);
    long groups = (B + CB - 1) / CB;
    int fail = 0;
#pragma omp parallel
    {
        double *u = (double *)malloc(sizeof(double) * (size_t)n * CB);
        if (!u) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (long g = 0; g < groups; ++g) {
            if (!u) continue;
            long b0 = g * CB;
            int w = (int)((B - b0) < CB ? (B - b0) : CB);
            memset(u, 0, sizeof(double) * (size_t)n * CB);
            load_group(n, B, G, b0, w, u);
            for (long e = 0; e < count; ++e) {
                double *ui = u + (size_t)pairs[2 * e] * CB;
                double *uj = u + (size_t)pairs[2 * e + 1] * CB;
                double ce = c[e], se = s[e];
                for (int x = 0; x < CB; ++x) {
                    double ri = ce * ui[x] + se * uj[x];
                    double rj = -se * ui[x] + ce * uj[x];
                    ui[x] = ri;
                    uj[x] = rj;
                }
            }
            store_group(n, B, dX, b0, w, u);
        }
        free(u);
    }
    free(c); free(s);
    return fail ? -2 : 0;
}

int oracle_grad_operand(int n, long B, const double *theta, const int32_t *pairs,
                        const double *G, double *dX, int nthreads)
{
    if (bad_n(n)) return -1;
    return grad_operand_impl(n, B, (long)n * (n - 1) / 2, theta, pairs, G, dX, nthreads);
}

int oracle_grad_operand_pairs(int n, long B, long count, const double *theta, const int32_t *pairs,
                              const double *G, double *dX, int nthreads)
{
    return grad_operand_impl(n, B, count, theta, pairs, G, dX, nthreads);
}

/* Operand-side gradient sweep over a sequence E of `count` pairs.  dX and Xrec may be NULL. */
static int reverse_sweep_impl(int n, long B, long count, const double *theta, const int32_t *pairs,
                              const double *Y, const double *G, double *dtheta,
                              double *dX, double *Xrec, int nthreads)
{
    if (n < 2 || count < 0 || B < 1 || !theta || !pairs || !Y || !G || !dtheta) return -1;
    double *c, *s;
    if (make_cs(count, theta, &c, &s)) return -2;
    set_threads(nthreads);
    int nt = oracle_num_threads();
    double *acc = (double *)calloc((size_t)nt * (size_t)count, sizeof(double));
    if (!acc) { free(c); free(s); return -2; }
    long groups = (B + CB - 1) / CB;
    int fail = 0;
#pragma omp parallel num_threads(nt)
    {
        int tid = 0;
#ifdef _OPENMP
        tid = omp_get_thread_num();
#endif
        double *mine = acc + (size_t)tid * (size_t)count;
        double *z = (double *)malloc(sizeof(double) * (size_t)n * CB);
        double *gb = (double *)malloc(sizeof(double) * (size_t)n * CB);
        if (!z || !gb) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(static)
        for (long g = 0; g < groups; ++g) {
            if (!z || !gb) continue;
            long b0 = g * CB;
            int w = (int)((B - b0) < CB ? (B - b0) : CB);
            memset(z, 0, sizeof(double) * (size_t)n * CB);
            memset(gb, 0, sizeof(double) * (size_t)n * CB);
            load_group(n, B, Y, b0, w, z);
            load_group(n, B, G, b0, w, gb);
            for (long e = 0; e < count; ++e) {               /* blocks b_1, b_2, ... in order */
                double *zi = z + (size_t)pairs[2 * e] * CB;
                double *zj = z + (size_t)pairs[2 * e + 1] * CB;
                double *gi = gb + (size_t)pairs[2 * e] * CB;
                double *gj = gb + (size_t)pairs[2 * e + 1] * CB;
                double ce = c[e], se = s[e];
                double sum = 0.0;
                for (int x = 0; x < CB; ++x) sum += gj[x] * zi[x] - gi[x] * zj[x];
                mine[e] += sum;
                for (int x = 0; x < CB; ++x) {
                    double a = ce * zi[x] + se * zj[x];
                    double b = -se * zi[x] + ce * zj[x];
                    zi[x] = a;
                    zj[x] = b;
                    a = ce * gi[x] + se * gj[x];
                    b = -se * gi[x] + ce * gj[x];
                    gi[x] = a;
                    gj[x] = b;
                }
            }
            if (dX) store_group(n, B, dX, b0, w, gb);
            if (Xrec) store_group(n, B, Xrec, b0, w, z);
        }
        free(z); free(gb);
    }
    for (long e = 0; e < count; ++e) {
        double t = 0.0;
        for (int k = 0; k < nt; ++k) t += acc[(size_t)k * (size_t)count + e];
        dtheta[e] = t;
    }
    free(acc); free(c); free(s);
    return fail ? -2 : 0;
}

/* dtheta has n(n-1)/2 entries. */
int oracle_reverse_sweep(int n, long B, const double *theta, const int32_t *pairs,
                         const double *Y, const double *G, double *dtheta,
                         double *dX, double *Xrec, int nthreads)
{
    if (bad_n(n)) return -1;
    return reverse_sweep_impl(n, B, (long)n * (n - 1) / 2, theta, pairs, Y, G, dtheta, dX, Xrec, nthreads);
}

/* dtheta has `count` entries, one per listed pair. */
int oracle_reverse_sweep_pairs(int n, long B, long count, const double *theta, const int32_t *pairs,
                               const double *Y, const double *G, double *dtheta,
                               double *dX, double *Xrec, int nthreads)
{
    return reverse_sweep_impl(n, B, count, theta, pairs, Y, G, dtheta, dX, Xrec, nthreads);
}

/* Algorithm 3.  U and Gamma are n x n row-major.  For a fixed l the algorithm touches
 * only row l of U^fwd (entries (l,i), (l,j)) and column l of M = (row l of Gamma, at the
 * start), so a group of CB values of l is carried as two n x CB buffers. */
int oracle_grad_theta_alg3(int n, const double *theta, const int32_t *pairs,
                           const double *U, const double *Gamma, double *dtheta, int nthreads)
{
    if (bad_n(n) || !theta || !pairs || !U || !Gamma || !dtheta) return -1;
    long count = (long)n * (n - 1) / 2;
    int half = n / 2;
    double *c, *s;
    if (make_cs(count, theta, &c, &s)) return -2;
    set_threads(nthreads);
    int nt = oracle_num_threads();
    double *acc = (double *)calloc((size_t)nt * (size_t)count, sizeof(double));
    if (!acc) { free(c); free(s); return -2; }
    long groups = ((long)n + CB - 1) / CB;
    int fail = 0;
#pragma omp parallel num_threads(nt)
    {
        int tid = 0;
#ifdef _OPENMP
        tid = omp_get_thread_num();
#endif
        double *mine = acc + (size_t)tid * (size_t)count;
        double *uf = (double *)malloc(sizeof(double) * (size_t)n * CB); /* uf[r][x] = U^fwd[l0+x, r] */
        double *mm = (double *)malloc(sizeof(double) * (size_t)n * CB); /* mm[r][x] = M[r, l0+x]     */
        if (!uf || !mm) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(static)
        for (long g = 0; g < groups; ++g) {
            if (!uf || !mm) continue;
            long l0 = g * CB;
            int w = (int)(((long)n - l0) < CB ? ((long)n - l0) : CB);
            memset(uf, 0, sizeof(double) * (size_t)n * CB);
            memset(mm, 0, sizeof(double) * (size_t)n * CB);
            for (int r = 0; r < n; ++r)
                for (int x = 0; x < w; ++x) {
                    uf[(size_t)r * CB + x] = U[(size_t)(l0 + x) * n + r];      /* U^fwd <- U       */
                    mm[(size_t)r * CB + x] = Gamma[(size_t)(l0 + x) * n + r];  /* M <- Gamma^T     */
                }
            for (int k = n - 2; k >= 0; --k) {               /* reversed(B) */
                for (int p = 0; p < half; ++p) {
                    long e = (long)k * half + p;
                    double *ui = uf + (size_t)pairs[2 * e] * CB;
                    double *uj = uf + (size_t)pairs[2 * e + 1] * CB;
                    double *mi = mm + (size_t)pairs[2 * e] * CB;
                    double *mj = mm + (size_t)pairs[2 * e + 1] * CB;
                    double ce = c[e], se = s[e];
                    double sum = 0.0;
                    for (int x = 0; x < CB; ++x) {
                        double a = ce * ui[x] - se * uj[x];   /* column update of U^fwd */
                        double b = se * ui[x] + ce * uj[x];
                        ui[x] = a;
                        uj[x] = b;
                        a = ce * mi[x] - se * mj[x];          /* row update of M */
                        b = se * mi[x] + ce * mj[x];
                        mi[x] = a;
                        mj[x] = b;
                        sum += mi[x] * uj[x] - mj[x] * ui[x]; /* A[m(e), l] */
                    }
                    mine[e] += sum;
                }
            }
        }
        free(uf); free(mm);
    }
    for (long e = 0; e < count; ++e) {
        double t = 0.0;
        for (int k = 0; k < nt; ++k) t += acc[(size_t)k * (size_t)count + e];
        dtheta[e] = t;
    }
    free(acc); free(c); free(s);
    return fail ? -2 : 0;
}
