/*
 * CPU oracle for the singular values of a dense real matrix.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path (the HIP library and
 * its Python binding) may include, link or call this file; only the tests, the
 * smoke check and the benchmark's cpu_baseline leg do.  It shares no code with
 * the HIP path.
 *
 * What it computes (paper, Section 3, equation (1)): the singular values
 * sigma_1 >= ... >= sigma_n >= 0 of A, i.e. the diagonal of Sigma in
 * A = U Sigma V^T.  The paper's method reaches exactly these values (up to
 * rounding) through orthogonal transformations only (Section 3: dense -> band
 * -> bidiagonal -> diagonal), so the oracle is the textbook route to the same
 * definition, always in fp64:
 *
 *   1. unblocked Golub-Kahan Householder bidiagonalisation (one column
 *      reflector from the left, one row reflector from the right, per step);
 *      this is the classic, untiled Householder algorithm that the tiled
 *      algorithm of Section 3.2 restructures, with the 8/3 n^3 flop count
 *      the benchmark credits;
 *   2. the singular values of the bidiagonal by bisection with Sturm counts
 *      on the Golub-Kahan tridiagonal (zero diagonal, off-diagonals
 *      |d_1|,|e_1|,|d_2|,...), whose eigenvalues are +-sigma_i.  (The paper
 *      calls LAPACK here, Section 3; for values only any accurate bidiagonal
 *      solver is the same function.)
 *
 * The Householder reflector uses the normalised form of Algorithm 3
 * (H = I - tau v v^T with v_1 = 1 and a sign chosen to avoid cancellation),
 * with the degenerate case handled by tau = 0 (H = I) when the tail is zero
 * instead of the paper's absolute 10*eps threshold.
 *
 * OpenMP is used only to split independent columns / rows / singular values
 * across threads; the arithmetic per entry is the plain algorithm's.
 *
 * Pins (tests/test_oracle.py): closed forms for the reflector (Algorithm 3),
 * for the bidiagonal solver (2 cos(k pi/(2n+1)) spectrum, 2x2 closed form,
 * diagonal input), and for the whole (diagonal, rank one, prescribed spectrum,
 * Frobenius norm, determinant, Jacobi brute force on A^T A, library SVD).
 */
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define A_(i, j) a[(size_t)(i) + (size_t)(j) * (size_t)lda]

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Euclidean norm with scaling against overflow / underflow. */
static double scaled_norm(int64_t n, const double *x, int64_t incx)
{
    double big = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        double t = fabs(x[i * incx]);
        if (t > big) big = t;
    }
    if (big == 0.0 || !isfinite(big)) return big;
    double s = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        double t = x[i * incx] / big;
        s += t * t;
    }
    return big * sqrt(s);
}

/*
 * Householder reflector for the vector (alpha, x[0..n-2]) of length n:
 * H = I - tau v v^T, v = (1, x_out), H (alpha, x)^T = (beta, 0)^T with
 * beta = -sign(alpha) * norm.  On return *alpha = beta and x holds the tail
 * of v.  tau = 0 when the tail is already zero.
 */
void orc_householder(int64_t n, double *alpha, double *x, int64_t incx, double *tau)
{
    if (n <= 1) { *tau = 0.0; return; }
    double xnorm = scaled_norm(n - 1, x, incx);
    if (xnorm == 0.0) { *tau = 0.0; return; }
    double al = *alpha;
    double nrm = hypot(al, xnorm);
    double beta = (al >= 0.0) ? -nrm : nrm;
    *tau = (beta - al) / beta;
    double inv = 1.0 / (al - beta);
    for (int64_t i = 0; i < n - 1; ++i) x[i * incx] *= inv;
    *alpha = beta;
}

/*
 * Golub-Kahan bidiagonalisation of the m x n (m >= n) column-major matrix a.
 * On return d[0..n-1] and e[0..n-2] hold the upper bidiagonal; a holds the
 * reflector tails (column reflectors below the diagonal, row reflectors to
 * the right of the superdiagonal) and tauq / taup their scalars, so that a
 * test can rebuild U and V.  Returns 0, or -1 on bad arguments.
 */
int orc_bidiagonalize(int64_t m, int64_t n, double *a, int64_t lda,
                      double *d, double *e, double *tauq, double *taup)
{
    if (m < n || n < 0 || lda < (m > 1 ? m : 1)) return -1;
    double *w = (double *)malloc(sizeof(double) * (size_t)(m > 0 ? m : 1));
    if (!w) return -2;
    for (int64_t k = 0; k < n; ++k) {
        /* column reflector: zero A[k+1:m, k] */
        double tq;
        orc_householder(m - k, &A_(k, k), &A_(k + (k + 1 < m ? 1 : 0), k), 1, &tq);
        tauq[k] = tq;
        d[k] = A_(k, k);
        if (tq != 0.0) {
            const double *v = &A_(k, k); /* v[0] is treated as 1 */
#pragma omp parallel for schedule(static)
            for (int64_t j = k + 1; j < n; ++j) {
                double *c = &A_(k, j);
                double s = c[0];
                for (int64_t i = 1; i < m - k; ++i) s += v[i] * c[i];
                s *= tq;
                c[0] -= s;
                for (int64_t i = 1; i < m - k; ++i) c[i] -= s * v[i];
            }
        }
        if (k >= n - 1) break;
        /* row reflector: zero A[k, k+2:n] */
        double tp = 0.0;
        if (k < n - 2) orc_householder(n - k - 1, &A_(k, k + 1), &A_(k, k + 2), lda, &tp);
        taup[k] = tp;
        e[k] = A_(k, k + 1);
        if (tp != 0.0) {
            int64_t rows = m - k - 1;
            int64_t cols = n - k - 1; /* u[0] = 1, u[j] = A[k, k+1+j] */
#pragma omp parallel
            {
                int nt = 1, id = 0;
#ifdef _OPENMP
                nt = omp_get_num_threads();
                id = omp_get_thread_num();
#endif
                int64_t chunk = (rows + nt - 1) / nt;
                int64_t r0 = id * chunk, r1 = r0 + chunk;
                if (r1 > rows) r1 = rows;
                if (r0 < r1) {
                    double *wi = w + r0;
                    const double *c0 = &A_(k + 1 + r0, k + 1);
                    for (int64_t i = 0; i < r1 - r0; ++i) wi[i] = c0[i];
                    for (int64_t j = 1; j < cols; ++j) {
                        double uj = A_(k, k + 1 + j);
                        const double *c = &A_(k + 1 + r0, k + 1 + j);
                        for (int64_t i = 0; i < r1 - r0; ++i) wi[i] += uj * c[i];
                    }
                    for (int64_t i = 0; i < r1 - r0; ++i) wi[i] *= tp;
                    double *c00 = &A_(k + 1 + r0, k + 1);
                    for (int64_t i = 0; i < r1 - r0; ++i) c00[i] -= wi[i];
                    for (int64_t j = 1; j < cols; ++j) {
                        double uj = A_(k, k + 1 + j);
                        double *c = &A_(k + 1 + r0, k + 1 + j);
                        for (int64_t i = 0; i < r1 - r0; ++i) c[i] -= wi[i] * uj;
                    }
                }
            }
        }
    }
    free(w);
    return 0;
}

/* Number of eigenvalues smaller than x of the symmetric tridiagonal matrix of
 * order nz+1 with zero diagonal and off-diagonals z[0..nz-1] (squares in z2). */
static int64_t sturm_count(int64_t nz, const double *z2, double x, double pivmin)
{
    int64_t cnt = 0;
    double q = -x;
    if (fabs(q) < pivmin) q = -pivmin;
    if (q < 0.0) ++cnt;
    for (int64_t j = 0; j < nz; ++j) {
        q = -x - z2[j] / q;
        if (fabs(q) < pivmin) q = -pivmin;
        if (q < 0.0) ++cnt;
    }
    return cnt;
}

/*
 * Singular values of the n x n upper bidiagonal (d, e) by bisection, written
 * to sigma in descending order.  Returns 0, -1 on bad arguments, -3 if an
 * entry is not finite.
 */
int orc_bdsvals(int64_t n, const double *d, const double *e, double *sigma)
{
    if (n < 0) return -1;
    if (n == 0) return 0;
    int64_t nz = 2 * n - 1;
    double *z2 = (double *)malloc(sizeof(double) * (size_t)nz);
    if (!z2) return -2;
    double zmax = 0.0, bound = 0.0, prev = 0.0;
    for (int64_t j = 0; j < nz; ++j) {
        double z = fabs((j & 1) ? e[j / 2] : d[j / 2]);
        if (!isfinite(z)) { free(z2); return -3; }
        if (z > zmax) zmax = z;
        if (prev + z > bound) bound = prev + z; /* Gershgorin row sums */
        prev = z;
        z2[j] = z;
    }
    if (prev > bound) bound = prev;
    if (zmax == 0.0) {
        for (int64_t k = 0; k < n; ++k) sigma[k] = 0.0;
        free(z2);
        return 0;
    }
    /* work on the matrix scaled to max entry 1 so that squares cannot overflow */
    double scale = zmax;
    for (int64_t j = 0; j < nz; ++j) {
        double z = z2[j] / scale;
        z2[j] = z * z;
    }
    double hi0 = bound / scale * (1.0 + 4.0 * DBL_EPSILON) + DBL_MIN;
    double pivmin = DBL_MIN;
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t k = 0; k < n; ++k) {
        /* k-th smallest singular value = eigenvalue number n+k (0-based) */
        double lo = 0.0, hi = hi0;
        /* relative width 2 eps, with an absolute floor of 1e-38 sigma_max so
         * that exactly singular input does not bisect down to denormals */
        for (int it = 0; it < 256; ++it) {
            double mid = 0.5 * (lo + hi);
            if (mid <= lo || mid >= hi) break;
            if (hi - lo <= 2.0 * DBL_EPSILON * hi + 1e-38) break;
            if (sturm_count(nz, z2, mid, pivmin) >= n + k + 1) hi = mid;
            else lo = mid;
        }
        sigma[n - 1 - k] = 0.5 * (lo + hi) * scale;
    }
    free(z2);
    return 0;
}

/*
 * All singular values of the m x n (m >= n) column-major matrix a (destroyed),
 * descending, into sigma[0..n-1].
 */
int orc_svdvals(int64_t m, int64_t n, double *a, int64_t lda, double *sigma)
{
    if (m < n || n < 0) return -1;
    if (n == 0) return 0;
    double *buf = (double *)malloc(sizeof(double) * (size_t)(4 * n));
    if (!buf) return -2;
    double *d = buf, *e = buf + n, *tq = buf + 2 * n, *tp = buf + 3 * n;
    int rc = orc_bidiagonalize(m, n, a, lda, d, e, tq, tp);
    if (rc == 0) rc = orc_bdsvals(n, d, e, sigma);
    free(buf);
    return rc;
}
