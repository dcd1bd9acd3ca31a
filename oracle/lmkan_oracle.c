/*
 * CPU oracle for the 2-D lmKAN layer ("Lookup multivariate Kolmogorov-Arnold
 * Networks", arXiv 2509.07103).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, double-precision
 * restatement of what the paper defines, kept deliberately free of blocking,
 * fusion, SIMD or any other optimisation so that it can be checked against
 * the paper by eye.  It shares no code with the GPU library and must only be
 * used by the tests, the smoke check and the benchmark's CPU-baseline leg.
 *
 * Parity status: every function below is pinned by CPU tests against facts
 * the paper or the mathematics fix (grid = percentile levels of sigma, weights
 * summing to one, node interpolation, exact bilinear / ReLU reproduction,
 * brute-force evaluation of every basis function, finite differences, a
 * hand-worked example).  Nothing here is "parity unpinned".
 *
 * Conventions (Sec. 3.1, Alg. 1, App. B):
 *   G        number of grid intervals per axis (G >= 3)
 *   E[0..G]  extended grid: E[1..G-1] are the G-1 real grid points, E[0] and
 *            E[G] are the left and right ghost points of App. B.
 *   cell i   (0 <= i <= G-1) is [E[i], E[i+1]); cell 0 also holds everything
 *            left of the left ghost, cell G-1 everything right of the right
 *            ghost.
 *   P        coefficient tensor [G+1][G+1][K][N_out], K = N_in/2, last index
 *            fastest (Alg. 1 "Require").  P[a][b][k][j] multiplies
 *            B_a(x_{2k}) * B_b(x_{2k+1}) in output j (Eq. 2, Eq. 3).
 *
 * Readings of the paper taken here:
 *   - Edge intervals.  Alg. 1 / Alg. 3 leave them out "for brevity".  The same
 *     two formulas are used in the edge cells, with the ghost point as the
 *     outer grid value and no clipping, so every function is linear on the
 *     two infinite intervals (App. B, last paragraph of "Edge cases" and the
 *     paragraph on linear asymptotes) and w*ReLU(x) is reproduced exactly for
 *     even G (App. F.1).  Compiling with -DORACLE_CLIP_EDGE selects the other
 *     reading (edge hat functions cut to zero beyond the ghost); it exists
 *     only so a test can show that it breaks the ReLU statement.
 *   - The cell index is defined on the float32-rounded grid: i = number of
 *     real grid points E32[k] (k = 1..G-1) that are <= x.  In exact
 *     arithmetic this equals floor(sigma(x) * G) (Sec. 3.1 "Sigma grid");
 *     defining it by comparison makes it an exact integer function of the
 *     float32 input.  A point on a grid point belongs to the cell on its right.
 *   - Weights use the float32-rounded grid promoted to double, so that this
 *     file and a float32 implementation evaluate the same function.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------ */
/* sigma(x) and the grid                                                     */
/* ------------------------------------------------------------------------ */

/* App. B, Eq. 5 evaluated the way Alg. 2 does it: one exponential of -|x|. */
double oracle_sigma(double x)
{
    double t = exp(-fabs(x));
    if (x > 0.0)
        return 1.0 - 0.5 * t;
    return 0.5 * t;
}

/* Solve sigma(x) = p on the lower branch of Eq. 5 (0 < p <= 1/2): 0.5 e^x = p. */
static double sigma_inverse_lower(double p)
{
    return log(2.0 * p);
}

/*
 * Extended grid in double (Sec. 3.1 "Sigma grid" + App. B "Edge cases").
 * Real points: where sigma crosses the G-1 equispaced levels k/G.
 * Ghost points: mirror the second real point about the first one on each side.
 * Levels above 1/2 use sigma(-x) = 1 - sigma(x): the point for level k/G is
 * minus the point for level (G-k)/G, which keeps the two halves exact mirror
 * images of each other.
 */
int oracle_grid(int G, double *E)
{
    if (G < 3 || E == NULL)
        return 1;
    for (int k = 1; k <= G - 1; ++k) {
        if (2 * k <= G)
            E[k] = sigma_inverse_lower((double)k / (double)G);
        else
            E[k] = -sigma_inverse_lower((double)(G - k) / (double)G);
    }
    E[0] = E[1] - (E[2] - E[1]);
    E[G] = E[G - 1] + (E[G - 1] - E[G - 2]);
    return 0;
}

/* The grid table as a float32 implementation sees it: round each entry once. */
int oracle_grid_f32(int G, float *E32)
{
    double *E = (double *)malloc((size_t)(G + 1) * sizeof(double));
    if (E == NULL || oracle_grid(G, E) != 0) {
        free(E);
        return 1;
    }
    for (int k = 0; k <= G; ++k)
        E32[k] = (float)E[k];
    free(E);
    return 0;
}

/* Cell index by comparison against the real grid points (see header). */
int oracle_locate(int G, const float *E32, float x)
{
    int i = 0;
    for (int k = 1; k <= G - 1; ++k)
        if (E32[k] <= x)
            ++i;
    return i;
}

/* Cell index the way Sec. 3.1 states it, in double: floor(sigma(x) G), kept in range. */
int oracle_locate_sigma(int G, double x)
{
    int i = (int)floor(oracle_sigma(x) * (double)G);
    if (i < 0)
        i = 0;
    if (i > G - 1)
        i = G - 1;
    return i;
}

/* ------------------------------------------------------------------------ */
/* Basis functions from their description (no cell lookup)                   */
/* ------------------------------------------------------------------------ */

/*
 * Value of the a-th one-dimensional basis function (0 <= a <= G) at x, on an
 * arbitrary extended grid E, written from Sec. 3.1 "B-splines" and App. B
 * "Edge cases":
 *   a = 0, a = G : linear functions on the infinite intervals, zero at the
 *                  outermost real grid point, one at the ghost point, same
 *                  slope all the way to infinity, zero on the other side.
 *   1 <= a <= G-1: hat centred on real point E[a]: rises 0 -> 1 from E[a-1]
 *                  to E[a], falls 1 -> 0 from E[a] to E[a+1], zero elsewhere.
 *                  For a = 1 the left neighbour is the left ghost, for
 *                  a = G-1 the right neighbour is the right ghost, and under
 *                  the reading taken here the outer branch keeps its slope
 *                  past the ghost.
 */
double oracle_basis(int G, const double *E, int a, double x)
{
    if (a == 0)
        return (x < E[1]) ? (E[1] - x) / (E[1] - E[0]) : 0.0;
    if (a == G)
        return (x >= E[G - 1]) ? (x - E[G - 1]) / (E[G] - E[G - 1]) : 0.0;

    if (x < E[a]) {
        /* rising branch */
        int unbounded = (a == 1);
#ifdef ORACLE_CLIP_EDGE
        unbounded = 0;
#endif
        if (!unbounded && x < E[a - 1])
            return 0.0;
        return (x - E[a - 1]) / (E[a] - E[a - 1]);
    } else {
        /* falling branch */
        int unbounded = (a == G - 1);
#ifdef ORACLE_CLIP_EDGE
        unbounded = 0;
#endif
        if (!unbounded && x >= E[a + 1])
            return 0.0;
        return (E[a + 1] - x) / (E[a + 1] - E[a]);
    }
}

/*
 * One two-dimensional function straight from Eq. 3: the full double sum over
 * all (G+1)^2 products of one-dimensional basis functions.
 * P2 is [G+1][G+1] row-major, first index belongs to x1.
 */
double oracle_eval2d_def(int G, const double *E, const double *P2, double x1, double x2)
{
    double f = 0.0;
    for (int a = 0; a <= G; ++a) {
        double Ba = oracle_basis(G, E, a, x1);
        for (int b = 0; b <= G; ++b) {
            double Bb = oracle_basis(G, E, b, x2);
            f += P2[a * (G + 1) + b] * Ba * Bb;
        }
    }
    return f;
}

/* ------------------------------------------------------------------------ */
/* Preamble of Alg. 1 and the O(1) evaluation of Alg. 3                      */
/* ------------------------------------------------------------------------ */

typedef struct {
    int i1, i2;         /* cell indices                                    */
    double B00;         /* B_{i1,   i2  }(x1, x2)                           */
    double B10;         /* B_{i1+1, i2  }(x1, x2)                           */
    double B01;         /* B_{i1,   i2+1}(x1, x2)                           */
    double B11;         /* B_{i1+1, i2+1}(x1, x2)                           */
} preamble_t;

/* The four non-zero terms of Eq. 3 at (x1, x2).  Sec. 3.1: on each axis exactly two of the
 * one-dimensional functions are non-zero at a point, the ones attached to the two ends of the
 * interval the point falls in, and a two-dimensional function is the product of one function of
 * x1 and one of x2.  So: find the interval on each axis, evaluate those two functions with the
 * definition above (oracle_basis, which also carries the reading of the edge cells), and
 * multiply.  The grid is the float32-rounded one, promoted to double. */
static preamble_t preamble(int G, const float *E32, float x1f, float x2f)
{
    preamble_t r;
    double E[G + 1]; /* (a few hundred bytes: G is at most a few dozen) */
    for (int a = 0; a <= G; ++a)
        E[a] = (double)E32[a];
    const double x1 = (double)x1f, x2 = (double)x2f;
    r.i1 = oracle_locate(G, E32, x1f);
    r.i2 = oracle_locate(G, E32, x2f);
    const double first_lo = oracle_basis(G, E, r.i1, x1), first_hi = oracle_basis(G, E, r.i1 + 1, x1);
    const double second_lo = oracle_basis(G, E, r.i2, x2), second_hi = oracle_basis(G, E, r.i2 + 1, x2);
    r.B00 = first_lo * second_lo;
    r.B10 = first_hi * second_lo;
    r.B01 = first_lo * second_hi;
    r.B11 = first_hi * second_hi;
    return r;
}

/* Expose the preamble to tests: out = {B00, B10, B01, B11}, returns i1*G+i2. */
int oracle_preamble(int G, const float *E32, float x1, float x2, double *out)
{
    preamble_t r = preamble(G, E32, x1, x2);
    out[0] = r.B00;
    out[1] = r.B10;
    out[2] = r.B01;
    out[3] = r.B11;
    return r.i1 * G + r.i2;
}

/* Alg. 3: one standalone 2-D function with four terms.  P2 is [G+1][G+1]. */
double oracle_eval2d(int G, const float *E32, const double *P2, float x1, float x2)
{
    preamble_t r = preamble(G, E32, x1, x2);
    int W = G + 1;
    double y = 0.0;
    y += r.B00 * P2[r.i1 * W + r.i2];
    y += r.B10 * P2[(r.i1 + 1) * W + r.i2];
    y += r.B01 * P2[r.i1 * W + (r.i2 + 1)];
    y += r.B11 * P2[(r.i1 + 1) * W + (r.i2 + 1)];
    return y;
}

/* ------------------------------------------------------------------------ */
/* Stored coefficient formats                                                */
/* ------------------------------------------------------------------------ */

enum { ORACLE_F32 = 0, ORACLE_F16 = 1, ORACLE_BF16 = 2 };

/* IEEE binary16 bit pattern -> double, exactly. */
double oracle_half_bits_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int m = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)m, -24);                 /* zero and subnormals */
    else if (e == 31)
        v = (m == 0) ? INFINITY : NAN;
    else
        v = ldexp((double)(m + 1024), e - 25);     /* (1 + m/1024) 2^(e-15) */
    return sign ? -v : v;
}

/* bfloat16 bit pattern -> double: it is the upper half of a float32. */
double oracle_bf16_bits_to_double(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static double coef_at(const void *P, int dtype, size_t idx)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)P)[idx];
    if (dtype == ORACLE_F16)
        return oracle_half_bits_to_double(((const uint16_t *)P)[idx]);
    return oracle_bf16_bits_to_double(((const uint16_t *)P)[idx]);
}

/* Offset of P[a][b][k][j] in the layout of Alg. 1. */
static size_t p_index(int G, int K, int N_out, int a, int b, int k, int j)
{
    return (((size_t)a * (size_t)(G + 1) + (size_t)b) * (size_t)K + (size_t)k) * (size_t)N_out +
           (size_t)j;
}

/* ------------------------------------------------------------------------ */
/* Layer forward                                                             */
/* ------------------------------------------------------------------------ */

/*
 * Alg. 1 for a batch: for every row, for every input pair run the preamble
 * once, then four multiply-adds per output.
 *   x  [B][N_in]  float32 (the same bits a GPU run reads)
 *   P  [G+1][G+1][N_in/2][N_out] in `dtype` storage, decoded exactly
 *   y  [B][N_out] double
 * `threads` > 1 splits the rows over OpenMP threads (rows are independent).
 */
int oracle_forward(int64_t B, int N_in, int N_out, int G, const float *x, const void *P, int dtype,
                   double *y, int threads)
{
    if (N_in < 2 || (N_in & 1) || N_out < 1 || G < 3)
        return 1;
    int K = N_in / 2;
    float *E32 = (float *)malloc((size_t)(G + 1) * sizeof(float));
    if (E32 == NULL || oracle_grid_f32(G, E32) != 0) {
        free(E32);
        return 1;
    }
    if (threads < 1)
        threads = 1;
#pragma omp parallel for num_threads(threads) schedule(static)
    for (int64_t n = 0; n < B; ++n) {
        const float *xr = x + n * N_in;
        double *yr = y + n * N_out;
        for (int j = 0; j < N_out; ++j)
            yr[j] = 0.0;
        for (int k = 0; k < K; ++k) {
            preamble_t r = preamble(G, E32, xr[2 * k], xr[2 * k + 1]);
            for (int j = 0; j < N_out; ++j) {
                yr[j] += r.B00 * coef_at(P, dtype, p_index(G, K, N_out, r.i1, r.i2, k, j));
                yr[j] += r.B10 * coef_at(P, dtype, p_index(G, K, N_out, r.i1 + 1, r.i2, k, j));
                yr[j] += r.B01 * coef_at(P, dtype, p_index(G, K, N_out, r.i1, r.i2 + 1, k, j));
                yr[j] += r.B11 * coef_at(P, dtype, p_index(G, K, N_out, r.i1 + 1, r.i2 + 1, k, j));
            }
        }
    }
    free(E32);
    return 0;
}

/*
 * The same layer straight from its definition (Eq. 2 with Eq. 3 for every
 * f_qp): all (G+1)^2 basis products per function, no cell lookup.  Uses the
 * float32-rounded grid promoted to double so it describes the same function
 * as oracle_forward.  Meant for tiny layers only.
 */
int oracle_forward_def(int64_t B, int N_in, int N_out, int G, const float *x, const void *P,
                       int dtype, double *y)
{
    if (N_in < 2 || (N_in & 1) || N_out < 1 || G < 3)
        return 1;
    int K = N_in / 2;
    float *E32 = (float *)malloc((size_t)(G + 1) * sizeof(float));
    double *E = (double *)malloc((size_t)(G + 1) * sizeof(double));
    double *P2 = (double *)malloc((size_t)(G + 1) * (size_t)(G + 1) * sizeof(double));
    if (!E32 || !E || !P2 || oracle_grid_f32(G, E32) != 0) {
        free(E32);
        free(E);
        free(P2);
        return 1;
    }
    for (int a = 0; a <= G; ++a)
        E[a] = (double)E32[a];
    for (int64_t n = 0; n < B; ++n) {
        for (int q = 0; q < N_out; ++q) {
            double acc = 0.0;
            for (int p = 0; p < K; ++p) {
                for (int a = 0; a <= G; ++a)
                    for (int b = 0; b <= G; ++b)
                        P2[a * (G + 1) + b] = coef_at(P, dtype, p_index(G, K, N_out, a, b, p, q));
                acc += oracle_eval2d_def(G, E, P2, (double)x[n * N_in + 2 * p],
                                         (double)x[n * N_in + 2 * p + 1]);
            }
            y[n * N_out + q] = acc;
        }
    }
    free(E32);
    free(E);
    free(P2);
    return 0;
}

/* Cell index of every (row, pair): cell[n][k] = i1 * G + i2. */
int oracle_locate_batch(int64_t B, int N_in, int G, const float *x, int32_t *cell)
{
    if (N_in < 2 || (N_in & 1) || G < 3)
        return 1;
    int K = N_in / 2;
    float *E32 = (float *)malloc((size_t)(G + 1) * sizeof(float));
    if (E32 == NULL || oracle_grid_f32(G, E32) != 0) {
        free(E32);
        return 1;
    }
    for (int64_t n = 0; n < B; ++n)
        for (int k = 0; k < K; ++k) {
            int i1 = oracle_locate(G, E32, x[n * N_in + 2 * k]);
            int i2 = oracle_locate(G, E32, x[n * N_in + 2 * k + 1]);
            cell[n * K + k] = i1 * G + i2;
        }
    free(E32);
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Layer backward (the paper trains with its kernels but prints no formulas; */
/* these are the derivatives of Alg. 1's four-term sum)                      */
/* ------------------------------------------------------------------------ */

/*
 * Gradient with respect to the inputs for a batch.
 * Inside a cell the four weights are products of one factor in x1 and one in
 * x2, each linear, so
 *   dB00/dx1 = -(E[i2+1]-x2) Ainv,  dB10/dx1 = +(E[i2+1]-x2) Ainv,
 *   dB01/dx1 = -(x2-E[i2])  Ainv,  dB11/dx1 = +(x2-E[i2])  Ainv,
 * and symmetrically for x2.  On a grid point the derivative of the cell chosen
 * by the locate rule (the one on the right) is returned.
 *   gy [B][N_out] float32, gx [B][N_in] double.
 */
int oracle_backward_input(int64_t B, int N_in, int N_out, int G, const float *x, const void *P,
                          int dtype, const float *gy, double *gx, int threads)
{
    if (N_in < 2 || (N_in & 1) || N_out < 1 || G < 3)
        return 1;
    int K = N_in / 2;
    float *E32 = (float *)malloc((size_t)(G + 1) * sizeof(float));
    if (E32 == NULL || oracle_grid_f32(G, E32) != 0) {
        free(E32);
        return 1;
    }
    if (threads < 1)
        threads = 1;
#pragma omp parallel for num_threads(threads) schedule(static)
    for (int64_t n = 0; n < B; ++n) {
        const float *xr = x + n * N_in;
        const float *gyr = gy + n * N_out;
        for (int k = 0; k < K; ++k) {
            double x1 = (double)xr[2 * k], x2 = (double)xr[2 * k + 1];
            int i1 = oracle_locate(G, E32, xr[2 * k]);
            int i2 = oracle_locate(G, E32, xr[2 * k + 1]);
            double g1lo = (double)E32[i1], g1hi = (double)E32[i1 + 1];
            double g2lo = (double)E32[i2], g2hi = (double)E32[i2 + 1];
            double Ainv = 1.0 / ((g1hi - g1lo) * (g2hi - g2lo));
            double d1 = 0.0, d2 = 0.0;
            for (int j = 0; j < N_out; ++j) {
                double c00 = coef_at(P, dtype, p_index(G, K, N_out, i1, i2, k, j));
                double c10 = coef_at(P, dtype, p_index(G, K, N_out, i1 + 1, i2, k, j));
                double c01 = coef_at(P, dtype, p_index(G, K, N_out, i1, i2 + 1, k, j));
                double c11 = coef_at(P, dtype, p_index(G, K, N_out, i1 + 1, i2 + 1, k, j));
                double g = (double)gyr[j];
                d1 += g * ((c10 - c00) * (g2hi - x2) + (c11 - c01) * (x2 - g2lo)) * Ainv;
                d2 += g * ((c01 - c00) * (g1hi - x1) + (c11 - c10) * (x1 - g1lo)) * Ainv;
            }
            gx[n * N_in + 2 * k] = d1;
            gx[n * N_in + 2 * k + 1] = d2;
        }
    }
    free(E32);
    return 0;
}

/*
 * Gradient with respect to the coefficients of ONE input pair k:
 *   gPk[a][b][j] = sum_n B_{ab}(x_n) gy[n][j]  over the four (a,b) of row n's cell.
 * y is linear in P, so this is exact; nodes no row touches stay exactly zero
 * (Sec. 3.5 notes that only active B-splines receive gradient).
 * gPk is [G+1][G+1][N_out] double and is overwritten.
 */
int oracle_backward_coef_pair(int64_t B, int N_in, int N_out, int G, int k, const float *x,
                              const float *gy, double *gPk)
{
    if (N_in < 2 || (N_in & 1) || N_out < 1 || G < 3 || k < 0 || k >= N_in / 2)
        return 1;
    float *E32 = (float *)malloc((size_t)(G + 1) * sizeof(float));
    if (E32 == NULL || oracle_grid_f32(G, E32) != 0) {
        free(E32);
        return 1;
    }
    int W = G + 1;
    memset(gPk, 0, (size_t)W * (size_t)W * (size_t)N_out * sizeof(double));
    for (int64_t n = 0; n < B; ++n) {
        preamble_t r = preamble(G, E32, x[n * N_in + 2 * k], x[n * N_in + 2 * k + 1]);
        const float *gyr = gy + n * N_out;
        double *r00 = gPk + ((size_t)r.i1 * W + r.i2) * N_out;
        double *r10 = gPk + ((size_t)(r.i1 + 1) * W + r.i2) * N_out;
        double *r01 = gPk + ((size_t)r.i1 * W + (r.i2 + 1)) * N_out;
        double *r11 = gPk + ((size_t)(r.i1 + 1) * W + (r.i2 + 1)) * N_out;
        for (int j = 0; j < N_out; ++j) {
            double g = (double)gyr[j];
            r00[j] += r.B00 * g;
            r10[j] += r.B10 * g;
            r01[j] += r.B01 * g;
            r11[j] += r.B11 * g;
        }
    }
    free(E32);
    return 0;
}

/* ------------------------------------------------------------------------
 * Off-diagonal Hessian regulariser (Sec. 3.5, App. C).
 *
 * For one 2-D function with table p[a][b] on the grid E[0..G], at every node
 * that has all its neighbours (a, b in [1, G-1]; the values at the ghost
 * nodes enter as neighbours) the three finite-difference second derivatives
 * of App. C are formed with the non-uniform spacings
 *   hl = E[a] - E[a-1], hr = E[a+1] - E[a]   (and hb, hu along the second axis)
 *   D11 = 2 (hl p[a+1][b] - (hl + hr) p[a][b] + hr p[a-1][b]) / (hl hr (hl + hr))
 *   D22 = the same along b
 *   D12 = (p[a+1][b+1] - p[a+1][b-1] - p[a-1][b+1] + p[a-1][b-1]) / ((hl + hr)(hb + hu))
 *   H   = D11^2 + 2 D12^2 + D22^2
 * and the function's term is the mean of H over those (G-1)^2 nodes.  The
 * paper is silent on which nodes "all the grid points" are; this reading takes
 * every node where the stencil exists.
 *
 * Returns the mean; if grad != NULL adds d(mean)/dp[a][b] into grad[a*(G+1)+b]
 * (scatter form: each centre adds 2 D dD/dp to the nodes of its stencil).
 * --------------------------------------------------------------------- */
double oracle_hessian_reg_2d(int G, const double *E, const double *p, double *grad)
{
    const int W = G + 1;
    const double inv_n = 1.0 / ((double)(G - 1) * (double)(G - 1));
    double sum = 0.0;
    for (int a = 1; a <= G - 1; ++a) {
        const double hl = E[a] - E[a - 1], hr = E[a + 1] - E[a];
        for (int b = 1; b <= G - 1; ++b) {
            const double hb = E[b] - E[b - 1], hu = E[b + 1] - E[b];
            const double d11 = 2.0 * (hl * p[(a + 1) * W + b] - (hl + hr) * p[a * W + b] + hr * p[(a - 1) * W + b]) /
                               (hl * hr * (hl + hr));
            const double d22 = 2.0 * (hb * p[a * W + b + 1] - (hb + hu) * p[a * W + b] + hu * p[a * W + b - 1]) /
                               (hb * hu * (hb + hu));
            const double d12 = (p[(a + 1) * W + b + 1] - p[(a + 1) * W + b - 1] - p[(a - 1) * W + b + 1] +
                                p[(a - 1) * W + b - 1]) /
                               ((hl + hr) * (hb + hu));
            sum += d11 * d11 + 2.0 * d12 * d12 + d22 * d22;
            if (grad != NULL) {
                const double c11 = 2.0 * d11 * 2.0 / (hl * hr * (hl + hr)) * inv_n;
                grad[(a + 1) * W + b] += c11 * hl;
                grad[a * W + b] -= c11 * (hl + hr);
                grad[(a - 1) * W + b] += c11 * hr;
                const double c22 = 2.0 * d22 * 2.0 / (hb * hu * (hb + hu)) * inv_n;
                grad[a * W + b + 1] += c22 * hb;
                grad[a * W + b] -= c22 * (hb + hu);
                grad[a * W + b - 1] += c22 * hu;
                const double c12 = 4.0 * d12 / ((hl + hr) * (hb + hu)) * inv_n;
                grad[(a + 1) * W + b + 1] += c12;
                grad[(a + 1) * W + b - 1] -= c12;
                grad[(a - 1) * W + b + 1] -= c12;
                grad[(a - 1) * W + b - 1] += c12;
            }
        }
    }
    return sum * inv_n;
}

/* The regulariser of a whole layer: the sum of the 2-D terms over all pairs and outputs
 * (App. C, last paragraph), on the float32-rounded sigma grid promoted to double (the grid
 * every other function here uses).  P in the layout of Alg. 1, stored as `dtype`;
 * grad, if not NULL, is [G+1][G+1][K][N_out] in double and is overwritten. */
int oracle_hessian_reg(int N_in, int N_out, int G, const void *P, int dtype, double *value, double *grad)
{
    if (N_in < 2 || (N_in & 1) || N_out < 1 || G < 3) return 1;
    const int K = N_in / 2, W = G + 1;
    float *E32 = (float *)malloc((size_t)W * sizeof(float));
    double *E = (double *)malloc((size_t)W * sizeof(double));
    double *p = (double *)malloc((size_t)W * W * sizeof(double));
    double *g = (double *)malloc((size_t)W * W * sizeof(double));
    if (!E32 || !E || !p || !g || oracle_grid_f32(G, E32) != 0) {
        free(E32); free(E); free(p); free(g);
        return 1;
    }
    for (int a = 0; a < W; ++a) E[a] = (double)E32[a];
    double total = 0.0;
    for (int k = 0; k < K; ++k) {
        for (int j = 0; j < N_out; ++j) {
            for (int n = 0; n < W * W; ++n) p[n] = coef_at(P, dtype, ((size_t)n * K + k) * N_out + j);
            if (grad != NULL) memset(g, 0, (size_t)W * W * sizeof(double));
            total += oracle_hessian_reg_2d(G, E, p, grad != NULL ? g : NULL);
            if (grad != NULL)
                for (int n = 0; n < W * W; ++n) grad[((size_t)n * K + k) * N_out + j] = g[n];
        }
    }
    *value = total;
    free(E32); free(E); free(p); free(g);
    return 0;
}

/* ------------------------------------------------------------------------
 * Inference-time folds (App. E "Preconditioning", Eq. 4b; App. F.1).
 *
 * A ReLU-first preconditioned layer  y = gamma lmKAN(x) + Linear(ReLU(x))  followed by an
 * evaluation-mode batch normalisation  y' = s_j y_j + t_j  is again one lmKAN layer:
 *   f_kj <- gamma f_kj + Wl[j][2k] ReLU(x1) + Wl[j][2k+1] ReLU(x2)
 * is exact when 0 is a grid point (G even), because a piecewise-linear table with a node at
 * the kink reproduces ReLU, and a per-output constant c_j can be added to the table of any
 * one pair (here pair 0) because the four weights of a cell sum to one.  In coefficients:
 *   P'[a][b][k][j] = s_j (gamma P[a][b][k][j] + Wl[j][2k] max(E[a],0) + Wl[j][2k+1] max(E[b],0))
 *                    + [k == 0] (s_j bias_j + t_j)
 * on the float32-rounded grid E (the grid the layer is evaluated on).  lin_w is
 * [N_out][N_in] row-major, any of lin_w / lin_b / scale / shift may be NULL (absent
 * term; scale defaults to 1).  P and P_out are float32 / double in the layout of Alg. 1.
 * --------------------------------------------------------------------- */
int oracle_fold(int N_in, int N_out, int G, const float *P, double gamma, const double *lin_w,
                const double *lin_b, const double *scale, const double *shift, double *P_out)
{
    if (N_in < 2 || (N_in & 1) || N_out < 1 || G < 3) return 1;
    const int K = N_in / 2, W = G + 1;
    float *E32 = (float *)malloc((size_t)W * sizeof(float));
    if (E32 == NULL || oracle_grid_f32(G, E32) != 0) {
        free(E32);
        return 1;
    }
    for (int a = 0; a < W; ++a) {
        const double ra = E32[a] > 0.0f ? (double)E32[a] : 0.0;
        for (int b = 0; b < W; ++b) {
            const double rb = E32[b] > 0.0f ? (double)E32[b] : 0.0;
            for (int k = 0; k < K; ++k) {
                for (int j = 0; j < N_out; ++j) {
                    const size_t idx = p_index(G, K, N_out, a, b, k, j);
                    double v = gamma * (double)P[idx];
                    if (lin_w != NULL) v += lin_w[(size_t)j * N_in + 2 * k] * ra + lin_w[(size_t)j * N_in + 2 * k + 1] * rb;
                    const double s = scale != NULL ? scale[j] : 1.0;
                    v *= s;
                    if (k == 0) v += s * (lin_b != NULL ? lin_b[j] : 0.0) + (shift != NULL ? shift[j] : 0.0);
                    P_out[idx] = v;
                }
            }
        }
    }
    free(E32);
    return 0;
}

/* ---------------------------------------------------------------------------------------------
 * Convolution as a fully connected layer on patches (Sec. 5, "lmKAN-based Convolutional Neural
 * Networks": a kh x kw convolution is the map R^{kh kw C_in} -> R^{C_out} applied to every window;
 * the paper casts it to a fully connected layer by memory reshaping).  The oracle does exactly
 * that reshaping, written out, and then calls the fully connected functions above.
 *
 * Reading: channels-last image x[N][H][W][C]; no padding; window (oy, ox) covers rows
 * oy*stride .. oy*stride + kh - 1 and columns ox*stride .. ox*stride + kw - 1; OH = (H - kh) / stride + 1
 * (floor), likewise OW; patch row r = (img*OH + oy)*OW + ox; patch column e = (ky*kw + kx)*C + c.
 * With C even, consecutive columns 2k, 2k+1 (one lmKAN pair) are two channels of one pixel.
 * ------------------------------------------------------------------------------------------- */

/* patches[r][e] = x[img][oy*stride + ky][ox*stride + kx][c] */
int oracle_conv2d_patches(int N, int H, int W, int C, int kh, int kw, int stride, const float *x,
                          float *patches)
{
    if (N < 0 || H < kh || W < kw || C < 1 || kh < 1 || kw < 1 || stride < 1) return 1;
    const int OH = (H - kh) / stride + 1, OW = (W - kw) / stride + 1;
    const size_t E = (size_t)kh * kw * C;
    for (int img = 0; img < N; ++img)
        for (int oy = 0; oy < OH; ++oy)
            for (int ox = 0; ox < OW; ++ox) {
                const size_t r = ((size_t)img * OH + oy) * OW + ox;
                for (int ky = 0; ky < kh; ++ky)
                    for (int kx = 0; kx < kw; ++kx)
                        for (int c = 0; c < C; ++c) {
                            const size_t e = ((size_t)ky * kw + kx) * C + c;
                            const size_t src = (((size_t)img * H + (oy * stride + ky)) * W + (ox * stride + kx)) * C + c;
                            patches[r * E + e] = x[src];
                        }
            }
    return 0;
}

/* The chain rule through the reshaping above: every image element receives the sum of the patch
 * gradients of all windows that contain it; elements outside every window receive zero. */
int oracle_conv2d_patches_adjoint(int N, int H, int W, int C, int kh, int kw, int stride,
                                  const double *g_patches, double *gx)
{
    if (N < 0 || H < kh || W < kw || C < 1 || kh < 1 || kw < 1 || stride < 1) return 1;
    const int OH = (H - kh) / stride + 1, OW = (W - kw) / stride + 1;
    const size_t E = (size_t)kh * kw * C;
    for (size_t i = 0; i < (size_t)N * H * W * C; ++i) gx[i] = 0.0;
    for (int img = 0; img < N; ++img)
        for (int oy = 0; oy < OH; ++oy)
            for (int ox = 0; ox < OW; ++ox) {
                const size_t r = ((size_t)img * OH + oy) * OW + ox;
                for (int ky = 0; ky < kh; ++ky)
                    for (int kx = 0; kx < kw; ++kx)
                        for (int c = 0; c < C; ++c) {
                            const size_t e = ((size_t)ky * kw + kx) * C + c;
                            const size_t dst = (((size_t)img * H + (oy * stride + ky)) * W + (ox * stride + kx)) * C + c;
                            gx[dst] += g_patches[r * E + e];
                        }
            }
    return 0;
}
