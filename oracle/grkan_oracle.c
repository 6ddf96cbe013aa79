/*
 * GR-KAN group-wise rational function: fp64 CPU oracle.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * GPU library is checked against.  It shares no code with the HIP path and is
 * never called by it; only tests, the smoke check and the bench's CPU-baseline
 * leg may use it.
 *
 * What it computes (FlashKAT paper, Sec. "Kolmogorov-Arnold Transformer",
 * Eq. "pade"; Sec. "Gradient Computations", Eq. "grad_a", "grad_b", "grad_x",
 * "accum", "accum2"), one element at a time in double precision:
 *
 *   channel c of a row belongs to group g = c div d_g, d_g = D / G
 *   P(x)    = a_{g,0} + a_{g,1} x + ... + a_{g,m} x^m
 *   Aden(x) = b_{g,1} x + ... + b_{g,n} x^n          (the paper calls it A(x))
 *   Q(x)    = 1 + |Aden(x)|
 *   y       = P / Q
 *   dL/dx   = dy * ( P'/Q - s * Aden' * P / Q^2 ),  s = sign(Aden), s(0) = 0
 *   dL/da_{g,i} = sum over rows and the group's channels of  dy * x^i / Q
 *   dL/db_{g,j} = sum over the same elements of             -dy * x^j * s * P / Q^2
 *
 * Readings where the paper is silent: sign(0) = 0 (sub-gradient of |.|);
 * groups are 0-based contiguous channel blocks; B[g][0] multiplies x^1 (there
 * is no b_0); dA and dB are overwritten with the sums.
 *
 * Further down: the GR-KAN layer itself, out = W F(x) (Eq. "GR_KAN"), and its
 * backward pass by the chain rule.
 *
 * Layout: x, dy, y, dx are row-major [rows][D]; A is [G][m+1], B is [G][n].
 * The coefficient sums use Neumaier-compensated double accumulation.
 *
 * `threads` <= 1 runs the plain sequential loop (the definition).  With
 * threads > 1 the rows are cut into `threads` contiguous ranges, each range is
 * summed exactly as above into its own compensated accumulator, and the ranges
 * are added in index order; the per-element arithmetic is the same function.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define GRKAN_ORACLE_MAXDEG 16

/* Neumaier compensated accumulator. */
typedef struct {
    double sum;
    double comp;
} nacc_t;

static void nacc_add(nacc_t *a, double v)
{
    double t = a->sum + v;
    if (fabs(a->sum) >= fabs(v))
        a->comp += (a->sum - t) + v;
    else
        a->comp += (v - t) + a->sum;
    a->sum = t;
}

static double nacc_value(const nacc_t *a) { return a->sum + a->comp; }

/* Everything the equations need at one element. */
typedef struct {
    double xp[GRKAN_ORACLE_MAXDEG + 1]; /* x^0 .. x^max(m,n) */
    double P, dP, Aden, dAden, Q, s;
} elem_t;

static void eval_elem(double x, const double *a, int m, const double *b, int n, elem_t *e)
{
    int top = m > n ? m : n;
    e->xp[0] = 1.0;
    for (int i = 1; i <= top; ++i)
        e->xp[i] = e->xp[i - 1] * x;

    e->P = 0.0;
    for (int i = 0; i <= m; ++i)
        e->P += a[i] * e->xp[i];
    e->dP = 0.0;
    for (int i = 1; i <= m; ++i)
        e->dP += (double)i * a[i] * e->xp[i - 1];

    /* b[j-1] is b_j: it multiplies x^j, j = 1..n */
    e->Aden = 0.0;
    for (int j = 1; j <= n; ++j)
        e->Aden += b[j - 1] * e->xp[j];
    e->dAden = 0.0;
    for (int j = 1; j <= n; ++j)
        e->dAden += (double)j * b[j - 1] * e->xp[j - 1];

    e->Q = 1.0 + fabs(e->Aden);
    e->s = (e->Aden > 0.0) ? 1.0 : ((e->Aden < 0.0) ? -1.0 : 0.0);
}

static int check_args(int64_t rows, int D, int G, int m, int n)
{
    if (rows < 0 || D <= 0 || G <= 0 || D % G != 0)
        return 2;
    if (m < 0 || n < 0 || m > GRKAN_ORACLE_MAXDEG || n > GRKAN_ORACLE_MAXDEG)
        return 3;
    return 0;
}

static int pick_threads(int threads, int64_t rows)
{
    if (threads < 1)
        threads = 1;
#ifndef _OPENMP
    threads = 1;
#endif
    if ((int64_t)threads > rows)
        threads = rows > 0 ? (int)rows : 1;
    return threads;
}

/* y = P/Q.  Returns 0 on success, 2 for a bad shape, 3 for a bad degree. */
int grkan_oracle_fwd(const double *x, const double *A, const double *B, double *y,
                     int64_t rows, int D, int G, int m, int n, int threads)
{
    int rc = check_args(rows, D, G, m, n);
    if (rc)
        return rc;
    const int dg = D / G;
    threads = pick_threads(threads, rows);
#ifdef _OPENMP
#pragma omp parallel for num_threads(threads) schedule(static) if (threads > 1)
#endif
    for (int64_t r = 0; r < rows; ++r) {
        for (int c = 0; c < D; ++c) {
            const int g = c / dg;
            elem_t e;
            eval_elem(x[r * D + c], A + (size_t)g * (m + 1), m, B + (size_t)g * n, n, &e);
            y[r * D + c] = e.P / e.Q;
        }
    }
    return 0;
}

/* One contiguous row range of the backward pass; acc is [G][m+1+n]. */
static void bwd_rows(const double *x, const double *dy, const double *A, const double *B,
                     double *dx, nacc_t *acc, int64_t r0, int64_t r1, int D, int G, int m, int n)
{
    const int dg = D / G;
    const int nc = m + 1 + n;
    for (int64_t r = r0; r < r1; ++r) {
        for (int c = 0; c < D; ++c) {
            const int g = c / dg;
            const double xv = x[r * D + c];
            const double d = dy[r * D + c];
            elem_t e;
            eval_elem(xv, A + (size_t)g * (m + 1), m, B + (size_t)g * n, n, &e);

            dx[r * D + c] = d * (e.dP / e.Q - e.s * e.dAden * e.P / (e.Q * e.Q));

            nacc_t *ag = acc + (size_t)g * nc;
            for (int i = 0; i <= m; ++i)
                nacc_add(&ag[i], d * e.xp[i] / e.Q);
            for (int j = 1; j <= n; ++j)
                nacc_add(&ag[m + j], -d * e.xp[j] * e.s * e.P / (e.Q * e.Q));
        }
    }
}

/* dx, dA[G][m+1], dB[G][n] (both overwritten). */
int grkan_oracle_bwd(const double *x, const double *dy, const double *A, const double *B,
                     double *dx, double *dA, double *dB,
                     int64_t rows, int D, int G, int m, int n, int threads)
{
    int rc = check_args(rows, D, G, m, n);
    if (rc)
        return rc;
    const int nc = m + 1 + n;
    threads = pick_threads(threads, rows);

    nacc_t *acc = (nacc_t *)calloc((size_t)threads * G * nc, sizeof(nacc_t));
    if (!acc)
        return 9;

    if (threads == 1) {
        bwd_rows(x, dy, A, B, dx, acc, 0, rows, D, G, m, n);
    } else {
#ifdef _OPENMP
#pragma omp parallel num_threads(threads)
        {
            const int t = omp_get_thread_num();
            const int nt = omp_get_num_threads();
            /* nt can be smaller than asked for; ranges follow the real count and
               unused accumulator slots stay zero */
            const int64_t r0 = rows * t / nt;
            const int64_t r1 = rows * (t + 1) / nt;
            bwd_rows(x, dy, A, B, dx, acc + (size_t)t * G * nc, r0, r1, D, G, m, n);
        }
#endif
    }

    for (int g = 0; g < G; ++g) {
        for (int k = 0; k < nc; ++k) {
            nacc_t total = {0.0, 0.0};
            for (int t = 0; t < threads; ++t) {
                const nacc_t *p = &acc[((size_t)t * G + g) * nc + k];
                nacc_add(&total, p->sum);
                nacc_add(&total, p->comp);
            }
            const double v = nacc_value(&total);
            if (k <= m)
                dA[(size_t)g * (m + 1) + k] = v;
            else
                dB[(size_t)g * n + (k - m - 1)] = v;
        }
    }
    free(acc);
    return 0;
}

/*
 * Condition scales for the error metric used by the parity tests (not part of
 * the method).
 *
 * Elementwise results: the paper's expressions with every monomial of P, P'
 * and Aden' replaced by its magnitude, i.e. the size the result would have if
 * nothing cancelled inside those polynomials.  Q itself is taken as exact (the
 * GPU kernels evaluate Aden in double for float32 I/O precisely so that it is).
 *
 *   Sy  = Pm / Q
 *   Sdx = |dy| ( dPm / Q + dAm Pm / Q^2 )
 *
 * with Pm = sum |a_i||x|^i, dPm = sum i|a_i||x|^(i-1), dAm = sum j|b_j||x|^(j-1).
 * Where nothing cancels, Sy = |y| and Sdx >= |dx| within a factor 2.
 *
 * Coefficient gradients: the root-sum-square of the very terms that
 * Eq. "accum" and "accum2" add up, with the actual P (no magnitude
 * replacement), which is the scale of the rounding error of any summation
 * order:
 *
 *   RA[g][i]   = sqrt( sum (dy x^i / Q)^2 )
 *   RB[g][j-1] = sqrt( sum (dy x^j s P / Q^2)^2 )
 *
 * Any of the output pointers may be NULL.  dy may be NULL when only Sy is wanted.
 * The root-sum-squares are plain (uncompensated) double sums: they only scale a tolerance.
 */
int grkan_oracle_scales(const double *x, const double *dy, const double *A, const double *B,
                        double *Sy, double *Sdx, double *RA, double *RB,
                        int64_t rows, int D, int G, int m, int n, int threads)
{
    int rc = check_args(rows, D, G, m, n);
    if (rc)
        return rc;
    const int dg = D / G;
    const int nc = m + 1 + n;
    const int nsq = G * nc;
    double *sq = (double *)calloc((size_t)nsq, sizeof(double));
    if (!sq)
        return 9;
    threads = pick_threads(threads, rows);
#ifdef _OPENMP
#pragma omp parallel for num_threads(threads) schedule(static) reduction(+ : sq[:nsq]) if (threads > 1)
#endif
    for (int64_t r = 0; r < rows; ++r) {
        for (int c = 0; c < D; ++c) {
            const int g = c / dg;
            const double *a = A + (size_t)g * (m + 1);
            const double *b = B + (size_t)g * n;
            const double xv = x[r * D + c];
            const double ax = fabs(xv);
            const double d = dy ? fabs(dy[r * D + c]) : 0.0;
            elem_t e;
            eval_elem(xv, a, m, b, n, &e);

            double axp[GRKAN_ORACLE_MAXDEG + 1];
            int top = m > n ? m : n;
            axp[0] = 1.0;
            for (int i = 1; i <= top; ++i)
                axp[i] = axp[i - 1] * ax;
            double Pm = 0.0, dPm = 0.0, dAm = 0.0;
            for (int i = 0; i <= m; ++i)
                Pm += fabs(a[i]) * axp[i];
            for (int i = 1; i <= m; ++i)
                dPm += (double)i * fabs(a[i]) * axp[i - 1];
            for (int j = 1; j <= n; ++j)
                dAm += (double)j * fabs(b[j - 1]) * axp[j - 1];

            const double Q = e.Q, Q2 = Q * Q;
            if (Sy)
                Sy[r * D + c] = Pm / Q;
            if (Sdx)
                Sdx[r * D + c] = d * (dPm / Q + dAm * Pm / Q2);
            for (int i = 0; i <= m; ++i) {
                double t = d * axp[i] / Q;
                sq[(size_t)g * nc + i] += t * t;
            }
            for (int j = 1; j <= n; ++j) {
                double t = d * axp[j] * fabs(e.s) * fabs(e.P) / Q2;
                sq[(size_t)g * nc + m + j] += t * t;
            }
        }
    }
    for (int g = 0; g < G; ++g) {
        for (int i = 0; i <= m; ++i)
            if (RA)
                RA[(size_t)g * (m + 1) + i] = sqrt(sq[(size_t)g * nc + i]);
        for (int j = 1; j <= n; ++j)
            if (RB)
                RB[(size_t)g * n + (j - 1)] = sqrt(sq[(size_t)g * nc + m + j]);
    }
    free(sq);
    return 0;
}

/*
 * GR-KAN layer (Sec. "Kolmogorov-Arnold Transformer", Eq. "GR_KAN"): the
 * group-wise rational function followed by the weighted summation,
 *
 *   out[r][o] = sum_c W[o][c] * F_{g(c)}(x[r][c])   (+ bias[o] if bias != NULL)
 *
 * W is [D_out][D_in] row-major (the paper's W in R^{d_out x d_in}); the
 * equation has no bias term, which is an optional addition of this build
 * (bias == NULL gives the equation itself).  Plain loops, double precision,
 * Neumaier-compensated sum over c.
 *
 * round_operand: 0 = the definition.  1 = F is rounded to bfloat16 (8
 * significant bits, round to nearest, ties to even) before it is multiplied,
 * which is the quantised operand a bfloat16 matrix unit is fed; used by the
 * parity tests to check the contraction apart from that rounding.
 */
static double round_to_bf16(double v)
{
    if (v == 0.0 || !isfinite(v))
        return v;
    int e;
    const double mant = frexp(v, &e);    /* v = mant * 2^e, 0.5 <= |mant| < 1 */
    return ldexp(rint(ldexp(mant, 8)), e - 8); /* 8 significant bits; rint rounds ties to even */
}

int grkan_oracle_linear_fwd(const double *x, const double *A, const double *B, const double *W,
                            const double *bias, double *out,
                            int64_t rows, int D_in, int D_out, int G, int m, int n,
                            int round_operand, int threads)
{
    int rc = check_args(rows, D_in, G, m, n);
    if (rc)
        return rc;
    if (D_out <= 0)
        return 2;
    const int dg = D_in / G;
    threads = pick_threads(threads, rows);
#ifdef _OPENMP
#pragma omp parallel num_threads(threads) if (threads > 1)
#endif
    {
        double *f = (double *)malloc((size_t)D_in * sizeof(double));
#ifdef _OPENMP
#pragma omp for schedule(static)
#endif
        for (int64_t r = 0; r < rows; ++r) {
            if (!f)
                continue;
            for (int c = 0; c < D_in; ++c) {
                const int g = c / dg;
                elem_t e;
                eval_elem(x[r * D_in + c], A + (size_t)g * (m + 1), m, B + (size_t)g * n, n, &e);
                const double v = e.P / e.Q;
                f[c] = round_operand ? round_to_bf16(v) : v;
            }
            for (int o = 0; o < D_out; ++o) {
                nacc_t acc = {0.0, 0.0};
                for (int c = 0; c < D_in; ++c)
                    nacc_add(&acc, W[(size_t)o * D_in + c] * f[c]);
                out[r * D_out + o] = nacc_value(&acc) + (bias ? bias[o] : 0.0);
            }
        }
        free(f);
    }
    return 0;
}

/*
 * Backward of the GR-KAN layer for an upstream gradient dOut [rows][D_out]
 * (chain rule through Eq. "GR_KAN", then Eq. "grad_x", "grad_a", "grad_b",
 * "accum", "accum2" with dy = dF):
 *
 *   dF[r][c]   = sum_o dOut[r][o] * W[o][c]
 *   dW[o][c]   = sum_r dOut[r][o] * F_{g(c)}(x[r][c])
 *   dbias[o]   = sum_r dOut[r][o]
 *   dx, dA, dB = backward of the rational function for the upstream gradient dF
 *
 * dF is returned too (the tests use it).  Sequential; small cases only.
 */
int grkan_oracle_linear_bwd(const double *x, const double *dOut, const double *A, const double *B,
                            const double *W, double *dF, double *dx, double *dA, double *dB,
                            double *dW, double *dbias,
                            int64_t rows, int D_in, int D_out, int G, int m, int n)
{
    int rc = check_args(rows, D_in, G, m, n);
    if (rc)
        return rc;
    if (D_out <= 0)
        return 2;
    const int dg = D_in / G;
    for (int64_t r = 0; r < rows; ++r)
        for (int c = 0; c < D_in; ++c) {
            nacc_t acc = {0.0, 0.0};
            for (int o = 0; o < D_out; ++o)
                nacc_add(&acc, dOut[r * D_out + o] * W[(size_t)o * D_in + c]);
            dF[r * D_in + c] = nacc_value(&acc);
        }
    for (int o = 0; o < D_out; ++o) {
        nacc_t b = {0.0, 0.0};
        for (int64_t r = 0; r < rows; ++r)
            nacc_add(&b, dOut[r * D_out + o]);
        dbias[o] = nacc_value(&b);
        for (int c = 0; c < D_in; ++c) {
            const int g = c / dg;
            nacc_t acc = {0.0, 0.0};
            for (int64_t r = 0; r < rows; ++r) {
                elem_t e;
                eval_elem(x[r * D_in + c], A + (size_t)g * (m + 1), m, B + (size_t)g * n, n, &e);
                nacc_add(&acc, dOut[r * D_out + o] * (e.P / e.Q));
            }
            dW[(size_t)o * D_in + c] = nacc_value(&acc);
        }
    }
    return grkan_oracle_bwd(x, dF, A, B, dx, dA, dB, rows, D_in, G, m, n, 1);
}

/* Number of OpenMP threads the oracle would use when asked for `threads`. */
int grkan_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
