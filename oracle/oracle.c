/*
 * oracle.c - TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, fp64 CPU statement of what the batched Cholesky operator family
 * of "Auto-Differentiating Linear Algebra" (arXiv 1710.08717) computes.  It exists
 * to check the HIP library; it shares no code with it.  Only tests, the smoke
 * check and the benchmark's cpu_baseline leg may load it.
 *
 * Conventions (section 4, "BLAS and LAPACK" paragraph): every matrix is a full
 * square / rectangle in ROW-MAJOR order; a batch is the same-shape matrices laid
 * one after another ("batch mode").  All arithmetic is double precision.
 *
 * Every result here is exactly defined (the factor with positive diagonal is
 * unique; the rest are closed-form matrix expressions), so each routine is the
 * definition written as loops.  The only liberties taken are the order of the loop
 * nest (so that inner loops walk along rows) and, for one big matrix, handing its
 * independent vectors (right-hand sides, rows of a product) to the threads in
 * chunks; every sum keeps its terms and their order.  There is no tiling of the
 * sums and no fusion of steps.
 *
 * Pins: every function below is pinned by tests/test_oracle_*.py against closed
 * forms, brute-force determinants / inverses, finite differences and the adjoint
 * identity.  Nothing here is "parity unpinned".
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_OK 0
#define ORC_ERR_INVALID_ARG 1

/* Entry (i,k) of the triangular operand as the operator sees it.
 * M is stored row-major n x n.  lower!=0: M is lower triangular, entries above
 * the diagonal are taken to be zero whatever the memory holds.  lower==0: M is
 * upper triangular.  trans!=0 gives the entry of the transpose, t(M) = M^T
 * (operator table of section 4). */
static inline double tri_at(const double *M, int n, int lower, int trans, int i, int k)
{
    int r = trans ? k : i;
    int c = trans ? i : k;
    if (lower ? (r < c) : (r > c))
        return 0.0;
    return M[(size_t)r * n + c];
}

/* ------------------------------------------------------------------------- */
/* potrf forward: A = L L^T, l_ij = 0 for i < j, positive diagonal
 * (operator table row "potrf"; section 4.2 first paragraph).
 * lower == 0 gives the upper factor R with A = R^T R (appendix, potrf, last
 * paragraph).  Only the named triangle of A is read.  info[b] = 0, or the
 * 1-based index of the first pivot that is not > 0 (then that matrix's factor
 * is unspecified from that column/row on).  L may be the same memory as A. */
static void potrf_one_lower(int n, const double *A, double *L, int32_t *info)
{
    int fail = 0;
    for (int j = 0; j < n; ++j) {
        const double *Lj = L + (size_t)j * n;
        double d = A[(size_t)j * n + j];
        for (int k = 0; k < j; ++k)
            d -= Lj[k] * Lj[k];
        if (!(d > 0.0)) {
            fail = j + 1;
            break;
        }
        double ljj = sqrt(d);
        L[(size_t)j * n + j] = ljj;
#pragma omp parallel for schedule(static) if (n >= 1024)
        for (int i = j + 1; i < n; ++i) {
            const double *Li = L + (size_t)i * n;
            double s = A[(size_t)i * n + j];
            for (int k = 0; k < j; ++k)
                s -= Li[k] * Lj[k];
            L[(size_t)i * n + j] = s / ljj;
        }
    }
    for (int i = 0; i < n; ++i)
        for (int j = i + 1; j < n; ++j)
            L[(size_t)i * n + j] = 0.0;
    if (info)
        *info = fail;
}

static void potrf_one_upper(int n, const double *A, double *R, int32_t *info)
{
    /* Row i of R needs rows 0..i-1 of R: r_ij = (a_ij - sum_{k<i} r_ki r_kj) / r_ii. */
    int fail = 0;
    for (int i = 0; i < n; ++i) {
        double d = A[(size_t)i * n + i];
        for (int k = 0; k < i; ++k)
            d -= R[(size_t)k * n + i] * R[(size_t)k * n + i];
        if (!(d > 0.0)) {
            fail = i + 1;
            break;
        }
        double rii = sqrt(d);
        R[(size_t)i * n + i] = rii;
#pragma omp parallel for schedule(static) if (n >= 1024)
        for (int j = i + 1; j < n; ++j) {
            double s = A[(size_t)i * n + j];
            for (int k = 0; k < i; ++k)
                s -= R[(size_t)k * n + i] * R[(size_t)k * n + j];
            R[(size_t)i * n + j] = s / rii;
        }
    }
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < i; ++j)
            R[(size_t)i * n + j] = 0.0;
    if (info)
        *info = fail;
}

int orc_potrf(int lower, int64_t batch, int n, const double *A, double *L, int32_t *info)
{
    if (batch < 0 || n < 0)
        return ORC_ERR_INVALID_ARG;
    if (batch == 0 || n == 0)
        return ORC_OK;
    if (!A || !L)
        return ORC_ERR_INVALID_ARG;
    size_t nn = (size_t)n * n;
#pragma omp parallel for schedule(dynamic) if (batch > 1)
    for (int64_t b = 0; b < batch; ++b) {
        int32_t *ib = info ? info + b : NULL;
        if (lower)
            potrf_one_lower(n, A + b * nn, L + b * nn, ib);
        else
            potrf_one_upper(n, A + b * nn, L + b * nn, ib);
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* trmm forward (section 4.2, "trmm"):
 *   rightside == 0:  B = alpha * t(L) A,   A and B are n x m
 *   rightside != 0:  B = alpha * A t(L),   A and B are m x n
 * alpha is not in the paper's statement (alpha = 1 reproduces it); it scales the
 * result the way it does for gemm2 and syrk.  B may be the same memory as A. */
/* Entries of t(L) laid out with the FIRST index contiguous: Tc[c * n + k] = T(k,c).  The sums of
 * the right-side operators run over k for a fixed c, i.e. down a column of t(L); reading them
 * from this copy (made from n = 64 on) keeps those sums on consecutive addresses.  The terms and
 * their order are those of the plain loop.  NULL if not made. */
static double *first_index_contiguous(int lower, int trans, int n, const double *L, int parallel)
{
    if (n < 64)
        return NULL;
    double *Tc = (double *)malloc((size_t)n * n * sizeof(double));
    if (!Tc)
        return NULL;
#pragma omp parallel for schedule(static) if (parallel)
    for (int c = 0; c < n; ++c)
        for (int k = 0; k < n; ++k)
            Tc[(size_t)c * n + k] = tri_at(L, n, lower, trans, k, c);
    return Tc;
}

/* The m vectors a triangular operator acts on (columns of A for a left operator, rows for a
 * right one) are independent.  For one big matrix they are handed to the threads in chunks of
 * VCHUNK, and a chunk walks through t(L) once for all its vectors; below that size a single
 * chunk holds all of them.  Every sum keeps its terms and their order. */
#define VCHUNK 64

static void trmm_one(int lower, int trans, int rightside, double alpha, int n, int m,
                     const double *L, const double *A, double *B, double *tmp)
{
    /* t(L) is effectively lower triangular when exactly one of (upper, trans) holds;
     * entries on the other side of the diagonal are structural zeros and take no
     * part in the sums (so nothing stored there, or paired with it, is touched). */
    int eff_lower = (lower != 0) != (trans != 0);
    int big = ((double)n * n * m > 5e7);
    int chunk = big ? VCHUNK : m;
    int nchunk = (m + chunk - 1) / chunk;
    if (!rightside) {
        /* row i of the product = sum_k T(i,k) * row k of A, on the columns of one chunk */
#pragma omp parallel for schedule(dynamic) if (big)
        for (int q = 0; q < nchunk; ++q) {
            int c0 = q * chunk, c1 = c0 + chunk < m ? c0 + chunk : m;
            for (int i = 0; i < n; ++i) {
                double *ti = tmp + (size_t)i * m;
                for (int c = c0; c < c1; ++c)
                    ti[c] = 0.0;
                int k0 = eff_lower ? 0 : i;
                int k1 = eff_lower ? i + 1 : n;
                for (int k = k0; k < k1; ++k) {
                    double t = tri_at(L, n, lower, trans, i, k);
                    const double *ak = A + (size_t)k * m;
                    for (int c = c0; c < c1; ++c)
                        ti[c] += t * ak[c];
                }
            }
        }
    } else {
        /* entry (r,c) of the product = sum_k a_rk T(k,c), for the rows r of one chunk */
        double *Tc = first_index_contiguous(lower, trans, n, L, big);
#pragma omp parallel for schedule(dynamic) if (big)
        for (int q = 0; q < nchunk; ++q) {
            int r0 = q * chunk, r1 = r0 + chunk < m ? r0 + chunk : m;
            for (int c = 0; c < n; ++c) {
                int k0 = eff_lower ? c : 0;
                int k1 = eff_lower ? n : c + 1;
                for (int r = r0; r < r1; ++r) {
                    const double *ar = A + (size_t)r * n;
                    double s = 0.0;
                    if (Tc) {
                        const double *tc = Tc + (size_t)c * n;
                        for (int k = k0; k < k1; ++k)
                            s += ar[k] * tc[k];
                    } else {
                        for (int k = k0; k < k1; ++k)
                            s += ar[k] * tri_at(L, n, lower, trans, k, c);
                    }
                    tmp[(size_t)r * n + c] = s;
                }
            }
        }
        free(Tc);
    }
    for (size_t e = 0; e < (size_t)n * m; ++e)
        B[e] = alpha * tmp[e];
}

int orc_trmm(int lower, int trans, int rightside, double alpha, int64_t batch, int n, int m,
             const double *L, const double *A, double *B)
{
    if (batch < 0 || n < 0 || m < 0)
        return ORC_ERR_INVALID_ARG;
    if (batch == 0 || n == 0 || m == 0)
        return ORC_OK;
    if (!L || !A || !B)
        return ORC_ERR_INVALID_ARG;
    size_t nn = (size_t)n * n, nm = (size_t)n * m;
    int fail = 0;
#pragma omp parallel for schedule(dynamic) if (batch > 1)
    for (int64_t b = 0; b < batch; ++b) {
        double *tmp = (double *)malloc(nm * sizeof(double));
        if (!tmp) {
            fail = 1;
            continue;
        }
        trmm_one(lower, trans, rightside, alpha, n, m, L + b * nn, A + b * nm, B + b * nm, tmp);
        free(tmp);
    }
    return fail ? ORC_ERR_INVALID_ARG : ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* trsm forward (section 4.2, "trsm"):
 *   rightside == 0:  B = alpha * t(L)^{-1} A,   A and B are n x m
 *   rightside != 0:  B = alpha * A t(L)^{-1},   A and B are m x n
 * Plain substitution.  B may be the same memory as A. */
static void trsm_left_cols(int lower, int trans, double alpha, int n, int m, const double *L,
                           const double *A, double *B, int c0, int c1)
{
    /* t(L) X = alpha A on columns [c0, c1).  Row i of X =
     * (alpha * row i of A - sum_k T(i,k) row k of X) / T(i,i), with k < i for a lower T
     * (rows top to bottom) and k > i for an upper T (rows bottom to top). */
    int eff_lower = (lower != 0) != (trans != 0);
    for (int step = 0; step < n; ++step) {
        int i = eff_lower ? step : n - 1 - step;
        double *xi = B + (size_t)i * m;
        const double *ai = A + (size_t)i * m;
        for (int c = c0; c < c1; ++c)
            xi[c] = alpha * ai[c];
        int k0 = eff_lower ? 0 : i + 1;
        int k1 = eff_lower ? i : n;
        for (int k = k0; k < k1; ++k) {
            double t = tri_at(L, n, lower, trans, i, k);
            const double *xk = B + (size_t)k * m;
            for (int c = c0; c < c1; ++c)
                xi[c] -= t * xk[c];
        }
        double d = tri_at(L, n, lower, trans, i, i);
        for (int c = c0; c < c1; ++c)
            xi[c] /= d;
    }
}

static void trsm_right_rows(int lower, int trans, double alpha, int n, const double *L,
                            const double *Tc, const double *A, double *B, int r0, int r1)
{
    /* x t(L) = alpha a for the rows [r0, r1): sum_k x_k T(k,c) = alpha a_c.  Lower T: T(k,c) != 0
     * for k >= c, so c runs n-1 .. 0; upper T: c runs 0 .. n-1.
     * Tc, if given, holds T with the summation index contiguous (first_index_contiguous). */
    int eff_lower = (lower != 0) != (trans != 0);
    for (int step = 0; step < n; ++step) {
        int c = eff_lower ? n - 1 - step : step;
        int k0 = eff_lower ? c + 1 : 0;
        int k1 = eff_lower ? n : c;
        for (int r = r0; r < r1; ++r) {
            const double *a = A + (size_t)r * n;
            double *x = B + (size_t)r * n;
            double s = alpha * a[c];
            if (Tc) {
                const double *tc = Tc + (size_t)c * n;
                for (int k = k0; k < k1; ++k)
                    s -= x[k] * tc[k];
                x[c] = s / tc[c];
            } else {
                for (int k = k0; k < k1; ++k)
                    s -= x[k] * tri_at(L, n, lower, trans, k, c);
                x[c] = s / tri_at(L, n, lower, trans, c, c);
            }
        }
    }
}

/* The right-hand sides (columns for a left solve, rows for a right solve) are
 * independent; for one big matrix they are shared out over threads in chunks, nothing else. */
static void trsm_one(int lower, int trans, int rightside, double alpha, int n, int m,
                     const double *L, const double *A, double *B)
{
    int big = ((double)n * n * m > 5e7);
    if (!rightside) {
        const int chunk = VCHUNK;
        int nchunk = (m + chunk - 1) / chunk;
#pragma omp parallel for schedule(dynamic) if (big)
        for (int q = 0; q < nchunk; ++q) {
            int c0 = q * chunk, c1 = c0 + chunk < m ? c0 + chunk : m;
            trsm_left_cols(lower, trans, alpha, n, m, L, A, B, c0, c1);
        }
    } else {
        double *Tc = first_index_contiguous(lower, trans, n, L, big);
        int chunk = big ? 8 : m;  /* rows that share one pass over t(L) */
        int nchunk = (m + chunk - 1) / chunk;
#pragma omp parallel for schedule(dynamic) if (big)
        for (int q = 0; q < nchunk; ++q) {
            int r0 = q * chunk, r1 = r0 + chunk < m ? r0 + chunk : m;
            trsm_right_rows(lower, trans, alpha, n, L, Tc, A, B, r0, r1);
        }
        free(Tc);
    }
}

int orc_trsm(int lower, int trans, int rightside, double alpha, int64_t batch, int n, int m,
             const double *L, const double *A, double *B)
{
    if (batch < 0 || n < 0 || m < 0)
        return ORC_ERR_INVALID_ARG;
    if (batch == 0 || n == 0 || m == 0)
        return ORC_OK;
    if (!L || !A || !B)
        return ORC_ERR_INVALID_ARG;
    size_t nn = (size_t)n * n, nm = (size_t)n * m;
#pragma omp parallel for schedule(dynamic) if (batch > 1)
    for (int64_t b = 0; b < batch; ++b)
        trsm_one(lower, trans, rightside, alpha, n, m, L + b * nn, A + b * nm, B + b * nm);
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* syrk forward (section 4.2, "syrk"):
 *   trans == 0:  B = alpha A A^T,  A is n x k, B is n x n
 *   trans != 0:  B = alpha A^T A,  A is k x n, B is n x n
 * Both triangles of B are written.  B must not overlap A. */
int orc_syrk(int trans, double alpha, int64_t batch, int n, int k, const double *A, double *B)
{
    if (batch < 0 || n < 0 || k < 0)
        return ORC_ERR_INVALID_ARG;
    if (batch == 0 || n == 0)
        return ORC_OK;
    if (!B || (k > 0 && !A))
        return ORC_ERR_INVALID_ARG;
    size_t nn = (size_t)n * n, nk = (size_t)n * k;
#pragma omp parallel for schedule(dynamic) collapse(2)
    for (int64_t b = 0; b < batch; ++b) {
        for (int i = 0; i < n; ++i) {
            const double *Ab = A + b * nk;
            double *Bb = B + b * nn;
            for (int j = 0; j < n; ++j) {
                double s = 0.0;
                if (!trans)
                    for (int p = 0; p < k; ++p)
                        s += Ab[(size_t)i * k + p] * Ab[(size_t)j * k + p];
                else
                    for (int p = 0; p < k; ++p)
                        s += Ab[(size_t)p * n + i] * Ab[(size_t)p * n + j];
                Bb[(size_t)i * n + j] = alpha * s;
            }
        }
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Outer product that carries the gradient of the triangular operand in the trmm and
 * trsm backward rules (section 4.2; appendix "trsm", "trmm", also for an upper
 * factor): with P, Q of the shape of A (n x m for a left-side operator, m x n for a
 * right-side one) and (X1, X2) = (P, Q) without transposition, (Q, P) with it,
 *   left:  G = X1 X2^T,     right:  G = X2^T X1     (n x n),
 * of which the triangle of the factor is kept (tril for a lower factor, triu for an
 * upper one), scaled by `scale`; the other triangle of out is set to zero. */
static void tri_outer(int lower, int trans, int rightside, double scale, int n, int m, const double *P,
                      const double *Q, double *out)
{
    const double *X1 = trans ? Q : P, *X2 = trans ? P : Q;
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j) {
            double s = 0.0;
            int keep = lower ? (i >= j) : (i <= j);
            if (keep) {
                if (!rightside)
                    for (int c = 0; c < m; ++c)
                        s += X1[(size_t)i * m + c] * X2[(size_t)j * m + c];
                else
                    for (int r = 0; r < m; ++r)
                        s += X2[(size_t)r * n + i] * X1[(size_t)r * n + j];
                s *= scale;
            }
            out[(size_t)i * n + j] = s;
        }
}

/* trmm backward (section 4.2, "trmm"; appendix "trmm"): for B = alpha t(L) A (left) or
 * B = alpha A t(L) (right),
 *   Abar = alpha t(L)^T Bbar  resp.  alpha Bbar t(L)^T,
 *   Lbar = alpha tri( Bbar A^T | A Bbar^T | A^T Bbar | Bbar^T A )   for (left, t=no | left, t=yes |
 *          right, t=no | right, t=yes), tri = tril for a lower factor, triu for an upper one.
 * Lbar is computed first, so Abar may be the same memory as Bbar. */
int orc_trmm_backward(int lower, int trans, int rightside, double alpha, int64_t batch, int n, int m,
                      const double *L, const double *A, const double *Bbar, double *Abar, double *Lbar)
{
    if (batch < 0 || n < 0 || m < 0)
        return ORC_ERR_INVALID_ARG;
    if (batch == 0 || n == 0)
        return ORC_OK;
    if (!L || !Lbar || (m > 0 && (!A || !Bbar || !Abar)))
        return ORC_ERR_INVALID_ARG;
    size_t nn = (size_t)n * n, nm = (size_t)n * m;
    for (int64_t b = 0; b < batch; ++b)
        tri_outer(lower, trans, rightside, alpha, n, m, Bbar + b * nm, A + b * nm, Lbar + b * nn);
    if (m == 0)
        return ORC_OK;
    return orc_trmm(lower, !trans, rightside, alpha, batch, n, m, L, Bbar, Abar);
}

/* trsm backward (section 4.2, "trsm"; appendix "trsm"): for B = alpha t(L)^-1 A (left) or
 * B = alpha A t(L)^-1 (right), with Y = t(L)^-T Bbar resp. Bbar t(L)^-T,
 *   Abar = alpha Y,
 *   Lbar = -tri( Y B^T | B Y^T | B^T Y | Y^T B )   (same four cases as above).
 * For alpha = 1 this is the paper's rule with Abar in place of Y.  Needs the forward OUTPUT B,
 * not A.  Abar may be the same memory as Bbar. */
int orc_trsm_backward(int lower, int trans, int rightside, double alpha, int64_t batch, int n, int m,
                      const double *L, const double *B, const double *Bbar, double *Abar, double *Lbar)
{
    if (batch < 0 || n < 0 || m < 0)
        return ORC_ERR_INVALID_ARG;
    if (batch == 0 || n == 0)
        return ORC_OK;
    if (!L || !Lbar || (m > 0 && (!B || !Bbar || !Abar)))
        return ORC_ERR_INVALID_ARG;
    size_t nn = (size_t)n * n, nm = (size_t)n * m;
    if (m > 0) {
        int rc = orc_trsm(lower, !trans, rightside, 1.0, batch, n, m, L, Bbar, Abar); /* Y */
        if (rc != ORC_OK)
            return rc;
    }
    for (int64_t b = 0; b < batch; ++b)
        tri_outer(lower, trans, rightside, -1.0, n, m, Abar + b * nm, B + b * nm, Lbar + b * nn);
    for (size_t e = 0; e < (size_t)batch * nm; ++e)
        Abar[e] *= alpha;
    return ORC_OK;
}

/* syrk backward (section 4.2, "syrk"): Bbar need not be symmetric;
 *   B = alpha A A^T  (A n x k):  Abar = 2 alpha sym(Bbar) A = alpha (Bbar + Bbar^T) A
 *   B = alpha A^T A  (A k x n):  Abar = alpha A (Bbar + Bbar^T) */
int orc_syrk_backward(int trans, double alpha, int64_t batch, int n, int k, const double *A,
                      const double *Bbar, double *Abar)
{
    if (batch < 0 || n < 0 || k < 0)
        return ORC_ERR_INVALID_ARG;
    if (batch == 0 || n == 0 || k == 0)
        return ORC_OK;
    if (!A || !Bbar || !Abar)
        return ORC_ERR_INVALID_ARG;
    size_t nn = (size_t)n * n, nk = (size_t)n * k;
    for (int64_t b = 0; b < batch; ++b) {
        const double *Ab = A + b * nk, *G = Bbar + b * nn;
        double *O = Abar + b * nk;
        /* every entry of the result is its own sum: rows are shared out over the threads */
        if (!trans) {
#pragma omp parallel for schedule(dynamic, 4) if ((double)n * n * k > 5e7)
            for (int i = 0; i < n; ++i)
                for (int p = 0; p < k; ++p) {
                    double s = 0.0;
                    for (int j = 0; j < n; ++j)
                        s += (G[(size_t)i * n + j] + G[(size_t)j * n + i]) * Ab[(size_t)j * k + p];
                    O[(size_t)i * k + p] = alpha * s;
                }
        } else {
#pragma omp parallel for schedule(dynamic, 4) if ((double)n * n * k > 5e7)
            for (int p = 0; p < k; ++p)
                for (int j = 0; j < n; ++j) {
                    double s = 0.0;
                    for (int i = 0; i < n; ++i)
                        s += Ab[(size_t)p * n + i] * (G[(size_t)i * n + j] + G[(size_t)j * n + i]);
                    O[(size_t)p * n + j] = alpha * s;
                }
        }
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* gemm2 forward (section 4.2, "gemm2"): C = alpha * t_a(A) t_b(B).
 * t_a(A) is m x k, t_b(B) is k x n, C is m x n; A is stored m x k (ta == 0) or k x m (ta != 0),
 * B is stored k x n (tb == 0) or n x k (tb != 0).  C must not overlap A or B. */
int orc_gemm2(int ta, int tb, double alpha, int64_t batch, int m, int n, int k, const double *A,
              const double *B, double *C)
{
    if (batch < 0 || m < 0 || n < 0 || k < 0)
        return ORC_ERR_INVALID_ARG;
    if (batch == 0 || m == 0 || n == 0)
        return ORC_OK;
    if (!C || (k > 0 && (!A || !B)))
        return ORC_ERR_INVALID_ARG;
    size_t sa = (size_t)m * k, sb = (size_t)k * n, sc = (size_t)m * n;
#pragma omp parallel for schedule(dynamic) collapse(2)
    for (int64_t b = 0; b < batch; ++b)
        for (int i = 0; i < m; ++i) {
            const double *Ab = A + b * sa, *Bb = B + b * sb;
            double *Cb = C + b * sc;
            for (int j = 0; j < n; ++j) {
                double s = 0.0;
                for (int p = 0; p < k; ++p) {
                    double a = ta ? Ab[(size_t)p * m + i] : Ab[(size_t)i * k + p];
                    double bb = tb ? Bb[(size_t)j * k + p] : Bb[(size_t)p * n + j];
                    s += a * bb;
                }
                Cb[(size_t)i * n + j] = alpha * s;
            }
        }
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* gemm2 backward (section 4.2, "gemm2"): for C = alpha t_a(A) t_b(B),
 *   Abar = alpha Cbar t_b(B)^T      (ta == 0)     or  alpha t_b(B) Cbar^T   (ta != 0),
 *   Bbar = alpha t_a(A)^T Cbar      (tb == 0)     or  alpha Cbar^T t_a(A)   (tb != 0),
 * each in the storage shape of its operand, written as sums over the definition. */
int orc_gemm2_backward(int ta, int tb, double alpha, int64_t batch, int m, int n, int k, const double *A,
                       const double *B, const double *Cbar, double *Abar, double *Bbar)
{
    if (batch < 0 || m < 0 || n < 0 || k < 0)
        return ORC_ERR_INVALID_ARG;
    if (batch == 0)
        return ORC_OK;
    size_t sa = (size_t)m * k, sb = (size_t)k * n, sc = (size_t)m * n;
    if ((sa && (!A || !Abar)) || (sb && (!B || !Bbar)) || (sc && !Cbar))
        return ORC_ERR_INVALID_ARG;
    for (int64_t b = 0; b < batch; ++b) {
        const double *Ab = A + b * sa, *Bb = B + b * sb, *G = Cbar + b * sc;
        double *Ao = Abar + b * sa, *Bo = Bbar + b * sb;
        /* d phi / d t_a(A)(i,p) = alpha sum_j Cbar(i,j) t_b(B)(p,j) */
        for (int i = 0; i < m; ++i)
            for (int p = 0; p < k; ++p) {
                double s = 0.0;
                for (int j = 0; j < n; ++j)
                    s += G[(size_t)i * n + j] * (tb ? Bb[(size_t)j * k + p] : Bb[(size_t)p * n + j]);
                if (ta)
                    Ao[(size_t)p * m + i] = alpha * s;
                else
                    Ao[(size_t)i * k + p] = alpha * s;
            }
        /* d phi / d t_b(B)(p,j) = alpha sum_i t_a(A)(i,p) Cbar(i,j) */
        for (int p = 0; p < k; ++p)
            for (int j = 0; j < n; ++j) {
                double s = 0.0;
                for (int i = 0; i < m; ++i)
                    s += (ta ? Ab[(size_t)p * m + i] : Ab[(size_t)i * k + p]) * G[(size_t)i * n + j];
                if (tb)
                    Bo[(size_t)j * k + p] = alpha * s;
                else
                    Bo[(size_t)p * n + j] = alpha * s;
            }
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* potri (section 4.2, "potri"): B = A^-1 from the Cholesky factor of A.
 *   lower != 0: A = L L^T, B = L^-T L^-1;   lower == 0: A = R^T R, B = R^-1 R^-T.
 * Column j of B solves A b = e_j: two substitutions with the factor per column.
 * Both triangles of B are written. */
int orc_potri(int lower, int64_t batch, int n, const double *L, double *B)
{
    if (batch < 0 || n < 0)
        return ORC_ERR_INVALID_ARG;
    if (batch == 0 || n == 0)
        return ORC_OK;
    if (!L || !B)
        return ORC_ERR_INVALID_ARG;
    size_t nn = (size_t)n * n;
    int fail = 0;
#pragma omp parallel for schedule(dynamic) if (batch > 1)
    for (int64_t b = 0; b < batch; ++b) {
        double *E = (double *)malloc(nn * sizeof(double));
        if (!E) {
            fail = 1;
            continue;
        }
        for (size_t e = 0; e < nn; ++e)
            E[e] = 0.0;
        for (int i = 0; i < n; ++i)
            E[(size_t)i * n + i] = 1.0;
        /* A = F F^T with F = L (lower) or F = R^T (upper, i.e. t(R) with trans):
         * F Y = I, then F^T X = Y */
        trsm_one(lower, lower ? 0 : 1, 0, 1.0, n, n, L + b * nn, E, E);
        trsm_one(lower, lower ? 1 : 0, 0, 1.0, n, n, L + b * nn, E, B + b * nn);
        free(E);
    }
    return fail ? ORC_ERR_INVALID_ARG : ORC_OK;
}

/* potri backward (section 4.2, "potri"; appendix "potri"; Bbar need not be symmetric):
 *   lower != 0:  Lbar = -2 tril( B sym(Bbar) L^-T )
 *   lower == 0:  Rbar = -2 triu( R^-T sym(Bbar) B )
 * with B = A^-1 the forward output.  The other triangle of the result is zero. */
int orc_potri_backward(int lower, int64_t batch, int n, const double *L, const double *B, const double *Bbar,
                       double *Lbar)
{
    if (batch < 0 || n < 0)
        return ORC_ERR_INVALID_ARG;
    if (batch == 0 || n == 0)
        return ORC_OK;
    if (!L || !B || !Bbar || !Lbar)
        return ORC_ERR_INVALID_ARG;
    size_t nn = (size_t)n * n;
    int fail = 0;
#pragma omp parallel for schedule(dynamic) if (batch > 1)
    for (int64_t b = 0; b < batch; ++b) {
        double *M = (double *)malloc(nn * sizeof(double));
        if (!M) {
            fail = 1;
            continue;
        }
        const double *Bb = B + b * nn, *G = Bbar + b * nn;
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j) {
                double s = 0.0;
                if (lower) /* 2 B sym(Bbar) */
                    for (int p = 0; p < n; ++p)
                        s += Bb[(size_t)i * n + p] * (G[(size_t)p * n + j] + G[(size_t)j * n + p]);
                else /* 2 sym(Bbar) B */
                    for (int p = 0; p < n; ++p)
                        s += (G[(size_t)i * n + p] + G[(size_t)p * n + i]) * Bb[(size_t)p * n + j];
                M[(size_t)i * n + j] = s;
            }
        /* lower: X = M L^-T (right solve with the transpose); upper: X = R^-T M (left solve) */
        double *X = Lbar + b * nn;
        if (lower)
            trsm_one(1, 1, 1, -1.0, n, n, L + b * nn, M, X);
        else
            trsm_one(0, 1, 0, -1.0, n, n, L + b * nn, M, X);
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j)
                if (lower ? (i < j) : (i > j))
                    X[(size_t)i * n + j] = 0.0;
        free(M);
    }
    return fail ? ORC_ERR_INVALID_ARG : ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* log|L| = sum_i log l_ii (section 3.1, the identity below the GP code).
 * Plain log: a non-positive diagonal gives NaN / -inf as IEEE says. */
int orc_sumlogdiag(int64_t batch, int n, const double *L, double *out)
{
    if (batch < 0 || n < 0)
        return ORC_ERR_INVALID_ARG;
    if (batch == 0)
        return ORC_OK;
    if (!out || (n > 0 && !L))
        return ORC_ERR_INVALID_ARG;
    size_t nn = (size_t)n * n;
    for (int64_t b = 0; b < batch; ++b) {
        double s = 0.0;
        for (int i = 0; i < n; ++i)
            s += log(L[b * nn + (size_t)i * n + i]);
        out[b] = s;
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* copyltu / copyutl (section 4.1 "Simple Matrix Functions"; appendix potrf). */
static void copyltu(int n, double *X)
{
    for (int i = 0; i < n; ++i)
        for (int j = i + 1; j < n; ++j)
            X[(size_t)i * n + j] = X[(size_t)j * n + i];
}
static void copyutl(int n, double *X)
{
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < i; ++j)
            X[(size_t)i * n + j] = X[(size_t)j * n + i];
}

/* potrf backward in the order section 4.2 gives it:
 *   Abar = 1/2 L^{-T} copyltu(L^T Lbar) L^{-1}
 * carried out the way the paragraph after it describes: copy Lbar to Abar,
 * multiply by L^T from the left (trmm), copyltu, back-substitute from the left
 * with L^T and from the right with L (two trsm), halve.
 * lower == 0: Abar = 1/2 R^{-1} copyutl(Rbar R^T) R^{-T} (appendix, potrf). */
static void potrf_backward_one(int lower, int n, const double *L, const double *Lbar, double *Abar,
                               double *tmp)
{
    size_t nn = (size_t)n * n;
    if (Abar != Lbar)
        memcpy(Abar, Lbar, nn * sizeof(double));
    if (lower) {
        trmm_one(1, 1, 0, 1.0, n, n, L, Abar, Abar, tmp); /* L^T Lbar */
        copyltu(n, Abar);
        trsm_one(1, 1, 0, 1.0, n, n, L, Abar, Abar); /* L^{-T} (.) */
        trsm_one(1, 0, 1, 1.0, n, n, L, Abar, Abar); /* (.) L^{-1} */
    } else {
        trmm_one(0, 1, 1, 1.0, n, n, L, Abar, Abar, tmp); /* Rbar R^T */
        copyutl(n, Abar);
        trsm_one(0, 0, 0, 1.0, n, n, L, Abar, Abar); /* R^{-1} (.) */
        trsm_one(0, 1, 1, 1.0, n, n, L, Abar, Abar); /* (.) R^{-T} */
    }
    for (size_t e = 0; e < nn; ++e)
        Abar[e] *= 0.5;
}

int orc_potrf_backward(int lower, int64_t batch, int n, const double *L, const double *Lbar,
                       double *Abar)
{
    if (batch < 0 || n < 0)
        return ORC_ERR_INVALID_ARG;
    if (batch == 0 || n == 0)
        return ORC_OK;
    if (!L || !Lbar || !Abar)
        return ORC_ERR_INVALID_ARG;
    size_t nn = (size_t)n * n;
    int fail = 0;
#pragma omp parallel for schedule(dynamic) if (batch > 1)
    for (int64_t b = 0; b < batch; ++b) {
        double *tmp = (double *)malloc(nn * sizeof(double));
        if (!tmp) {
            fail = 1;
            continue;
        }
        potrf_backward_one(lower, n, L + b * nn, Lbar + b * nn, Abar + b * nn, tmp);
        free(tmp);
    }
    return fail ? ORC_ERR_INVALID_ARG : ORC_OK;
}

/* The same quantity through the masking matrix E of the appendix (e_ij = 0, 1, 2
 * for i <, =, > j): with Phi(X) = 1/2 (X o E) (lower triangle, halved diagonal),
 * copyltu(X) = Phi(X) + Phi(X)^T, hence
 *   Abar = sym( L^{-T} Phi(L^T Lbar) L^{-1} ).
 * Written with its own loops (dense inverse of L by substitution, dense
 * products) so that it cross-checks the routine above.  Lower factor only. */
int orc_potrf_backward_phi(int64_t batch, int n, const double *L, const double *Lbar, double *Abar)
{
    if (batch < 0 || n < 0)
        return ORC_ERR_INVALID_ARG;
    if (batch == 0 || n == 0)
        return ORC_OK;
    if (!L || !Lbar || !Abar)
        return ORC_ERR_INVALID_ARG;
    size_t nn = (size_t)n * n;
    double *Li = (double *)malloc(nn * sizeof(double));  /* L^{-1} */
    double *Ph = (double *)malloc(nn * sizeof(double));  /* Phi(L^T Lbar) */
    double *W = (double *)malloc(nn * sizeof(double));
    if (!Li || !Ph || !W) {
        free(Li);
        free(Ph);
        free(W);
        return ORC_ERR_INVALID_ARG;
    }
    for (int64_t b = 0; b < batch; ++b) {
        const double *Lb = L + b * nn, *Gb = Lbar + b * nn;
        double *Ab = Abar + b * nn;
        /* inverse of L, column c: solve L x = e_c */
        for (int c = 0; c < n; ++c)
            for (int i = 0; i < n; ++i) {
                double s = (i == c) ? 1.0 : 0.0;
                for (int k = c; k < i; ++k)
                    s -= Lb[(size_t)i * n + k] * Li[(size_t)k * n + c];
                Li[(size_t)i * n + c] = (i < c) ? 0.0 : s / Lb[(size_t)i * n + i];
            }
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j) {
                double s = 0.0;
                if (i >= j) {
                    for (int k = i; k < n; ++k) /* l_ki = 0 for k < i; lbar_kj needs k >= j */
                        s += Lb[(size_t)k * n + i] * Gb[(size_t)k * n + j];
                    if (i == j)
                        s *= 0.5;
                }
                Ph[(size_t)i * n + j] = s;
            }
        /* W = L^{-T} Ph : w_ij = sum_k linv_ki ph_kj */
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j) {
                double s = 0.0;
                for (int k = 0; k < n; ++k)
                    s += Li[(size_t)k * n + i] * Ph[(size_t)k * n + j];
                W[(size_t)i * n + j] = s;
            }
        /* Ph <- W L^{-1} */
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j) {
                double s = 0.0;
                for (int k = 0; k < n; ++k)
                    s += W[(size_t)i * n + k] * Li[(size_t)k * n + j];
                Ph[(size_t)i * n + j] = s;
            }
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j)
                Ab[(size_t)i * n + j] = 0.5 * (Ph[(size_t)i * n + j] + Ph[(size_t)j * n + i]);
    }
    free(Li);
    free(Ph);
    free(W);
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Variational sparse Gaussian-process criterion (section 3.2) and its gradient, from the
 * DEFINITION of the criterion rather than from the section's efficient evaluation: with the
 * Nystrom matrix Q = Kuf^T Kuu^-1 Kuf (n x n, formed densely here) and S = Q + lam I,
 *   phi = -log N(y | 0, S) + tr(Kff - Q) / (2 lam)
 *       = 1/2 log det S + 1/2 y^T S^-1 y + n/2 log 2 pi + (sum Kff_diag - tr Q) / (2 lam).
 * Its derivatives by matrix calculus, with a = S^-1 y and W = Kuu^-1 Kuf:
 *   d phi / dQ = M = 1/2 (S^-1 - a a^T) - I / (2 lam)          (symmetric),
 *   Kuf_bar = 2 W M,   Kuu_bar = -W M W^T   (symmetric: d phi = <Kuu_bar, dKuu> for symmetric dKuu),
 *   y_bar = a,   Kff_diag_bar = 1 / (2 lam),
 *   lam_bar = 1/2 tr S^-1 - 1/2 a^T a - (sum Kff_diag - tr Q) / (2 lam^2).
 * Inputs: Kuu (U x U, symmetric positive definite, lower triangle read), Kuf (U x n),
 * Kff_diag (n), y (n), noise variance lam.  Costs O(n^3): for checking only. */
/* Plain dense products for it (rows of the result shared out over the threads; every entry is
 * the sum over p = 0, 1, ... in that order):  Z = X^T Y,  Z = X Y,  Z = X Y^T. */
static void dense_tn(int m, int n, int k, const double *X, const double *Y, double *Z) /* X: k x m, Y: k x n */
{
#pragma omp parallel for schedule(static)
    for (int i = 0; i < m; ++i) {
        double *zi = Z + (size_t)i * n;
        for (int j = 0; j < n; ++j)
            zi[j] = 0.0;
        for (int p = 0; p < k; ++p) {
            const double x = X[(size_t)p * m + i];
            const double *yp = Y + (size_t)p * n;
            for (int j = 0; j < n; ++j)
                zi[j] += x * yp[j];
        }
    }
}
static void dense_nn(int m, int n, int k, const double *X, const double *Y, double *Z) /* X: m x k, Y: k x n */
{
#pragma omp parallel for schedule(static)
    for (int i = 0; i < m; ++i) {
        double *zi = Z + (size_t)i * n;
        for (int j = 0; j < n; ++j)
            zi[j] = 0.0;
        for (int p = 0; p < k; ++p) {
            const double x = X[(size_t)i * k + p];
            const double *yp = Y + (size_t)p * n;
            for (int j = 0; j < n; ++j)
                zi[j] += x * yp[j];
        }
    }
}
static void dense_nt(int m, int n, int k, const double *X, const double *Y, double *Z) /* X: m x k, Y: n x k */
{
#pragma omp parallel for schedule(static)
    for (int i = 0; i < m; ++i)
        for (int j = 0; j < n; ++j) {
            double t = 0.0;
            for (int p = 0; p < k; ++p)
                t += X[(size_t)i * k + p] * Y[(size_t)j * k + p];
            Z[(size_t)i * n + j] = t;
        }
}

int orc_sgp_criterion(int U, int n, const double *Kuu, const double *Kuf, const double *Kff_diag, const double *y,
                      double lam, double *phi, double *Kuu_bar, double *Kuf_bar, double *Kff_diag_bar, double *y_bar,
                      double *lam_bar)
{
    if (U <= 0 || n <= 0 || !Kuu || !Kuf || !Kff_diag || !y || !phi || !Kuu_bar || !Kuf_bar || !Kff_diag_bar ||
        !y_bar || !lam_bar || !(lam > 0.0))
        return ORC_ERR_INVALID_ARG;
    size_t uu = (size_t)U * U, un = (size_t)U * n, nn = (size_t)n * n;
    double *Lu = malloc(uu * sizeof(double)), *Ki = malloc(uu * sizeof(double)), *W = malloc(un * sizeof(double));
    double *S = malloc(nn * sizeof(double)), *Ls = malloc(nn * sizeof(double)), *Si = malloc(nn * sizeof(double));
    double *a = malloc(n * sizeof(double)), *T = malloc(un * sizeof(double));
    int rc = ORC_ERR_INVALID_ARG;
    if (!Lu || !Ki || !W || !S || !Ls || !Si || !a || !T)
        goto done;
    /* W = Kuu^-1 Kuf through the explicit inverse of Kuu;  Q = Kuf^T W */
    if (orc_potrf(1, 1, U, Kuu, Lu, NULL) || orc_potri(1, 1, U, Lu, Ki))
        goto done;
    dense_nn(U, n, U, Ki, Kuf, W);
    dense_tn(n, n, U, Kuf, W, S);
    double trq = 0.0, kk = 0.0;
    for (int i = 0; i < n; ++i) {
        trq += S[(size_t)i * n + i];
        kk += Kff_diag[i];
        S[(size_t)i * n + i] += lam;
    }
    /* S = Ls Ls^T:  log det S = 2 sum log Ls_ii,  a = S^-1 y by two substitutions,  S^-1 explicitly */
    if (orc_potrf(1, 1, n, S, Ls, NULL) || orc_trsm(1, 0, 0, 1.0, 1, n, 1, Ls, y, a) ||
        orc_trsm(1, 1, 0, 1.0, 1, n, 1, Ls, a, a) || orc_potri(1, 1, n, Ls, Si))
        goto done;
    double logdet = 0.0, ya = 0.0, aa = 0.0, tri = 0.0;
    for (int i = 0; i < n; ++i) {
        logdet += 2.0 * log(Ls[(size_t)i * n + i]);
        ya += y[i] * a[i];
        aa += a[i] * a[i];
        tri += Si[(size_t)i * n + i];
    }
    const double l2pi = 1.8378770664093454835606594728112; /* log(2 pi) */
    *phi = 0.5 * logdet + 0.5 * ya + 0.5 * n * l2pi + (kk - trq) / (2.0 * lam);
    *lam_bar = 0.5 * tri - 0.5 * aa - (kk - trq) / (2.0 * lam * lam);
    for (int i = 0; i < n; ++i) {
        y_bar[i] = a[i];
        Kff_diag_bar[i] = 1.0 / (2.0 * lam);
    }
    /* M = 1/2 (S^-1 - a a^T) - I / (2 lam), into Si */
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j)
            Si[(size_t)i * n + j] = 0.5 * (Si[(size_t)i * n + j] - a[i] * a[j]) - (i == j ? 1.0 / (2.0 * lam) : 0.0);
    /* T = W M;  Kuf_bar = 2 T;  Kuu_bar = -T W^T, symmetrised against rounding */
    dense_nn(U, n, n, W, Si, T);
    dense_nt(U, U, n, T, W, Lu);
    for (size_t e = 0; e < un; ++e)
        Kuf_bar[e] = 2.0 * T[e];
    for (int i = 0; i < U; ++i)
        for (int j = 0; j < U; ++j)
            Kuu_bar[(size_t)i * U + j] = -0.5 * (Lu[(size_t)i * U + j] + Lu[(size_t)j * U + i]);
    rc = ORC_OK;
done:
    free(Lu); free(Ki); free(W); free(S); free(Ls); free(Si); free(a); free(T);
    return rc;
}

/* ------------------------------------------------------------------------- */
/* Gaussian-process criterion pieces (section 3.1) for one noisy kernel matrix
 * A = L L^T and targets y:
 *   z = L^{-1} y, alpha = L^{-T} z,
 *   loss = 1/2 y^T alpha + sum_i log l_ii          (= phi - n/2 log 2 pi)
 * and the gradient that reaches potrf's output: the trsm backward case
 * B = L^{-1} A gives -tril(abar b^T) with bbar = z, abar = alpha, b = z
 * (section 4.2 "trsm", first case), and d/dl_ii sum log l_ii = 1 / l_ii:
 *   Lbar = -tril(alpha z^T) + diag(1 / l_ii).
 * z and alpha are inputs here (they come from two trsm calls). */
int orc_gp_glue(int64_t batch, int n, const double *L, const double *y, const double *z,
                const double *alpha, double *loss, double *Lbar)
{
    if (batch < 0 || n < 0)
        return ORC_ERR_INVALID_ARG;
    if (batch == 0)
        return ORC_OK;
    if (!loss || (n > 0 && (!L || !y || !z || !alpha || !Lbar)))
        return ORC_ERR_INVALID_ARG;
    size_t nn = (size_t)n * n;
    for (int64_t b = 0; b < batch; ++b) {
        const double *Lb = L + b * nn, *yb = y + b * n, *zb = z + b * n, *ab = alpha + b * n;
        double *Gb = Lbar + b * nn;
        double q = 0.0, ld = 0.0;
        for (int i = 0; i < n; ++i) {
            q += yb[i] * ab[i];
            ld += log(Lb[(size_t)i * n + i]);
        }
        loss[b] = 0.5 * q + ld;
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j) {
                double g = 0.0;
                if (i >= j)
                    g = -ab[i] * zb[j];
                if (i == j)
                    g += 1.0 / Lb[(size_t)i * n + i];
                Gb[(size_t)i * n + j] = g;
            }
    }
    return ORC_OK;
}

/* One entry of L L^T (lower != 0) or R^T R (lower == 0): lets a test compare a
 * huge factor against A on sampled positions without forming the product. */
double orc_llt_entry(int lower, int n, const double *L, int i, int j)
{
    double s = 0.0;
    int kmax = (i < j ? i : j);
    if (lower)
        for (int k = 0; k <= kmax; ++k)
            s += L[(size_t)i * n + k] * L[(size_t)j * n + k];
    else
        for (int k = 0; k <= kmax; ++k)
            s += L[(size_t)k * n + i] * L[(size_t)k * n + j];
    return s;
}

/* One entry of L^T X L for a lower factor L and a dense X: the defining relation
 * 2 L^T Abar L = copyltu(L^T Lbar) of the backward expression can be sampled with
 * it at sizes where the full backward is too slow on the CPU.  O(n^2) per entry. */
double orc_ltxl_entry(int n, const double *L, const double *X, int i, int j)
{
    double s = 0.0;
#pragma omp parallel for reduction(+ : s) schedule(static)
    for (int p = i; p < n; ++p) {
        double lpi = L[(size_t)p * n + i];
        const double *xp = X + (size_t)p * n;
        double t = 0.0;
        for (int q = j; q < n; ++q)
            t += xp[q] * L[(size_t)q * n + j];
        s += lpi * t;
    }
    return s;
}

/* One entry of L^T Lbar, lower triangles only (k >= max(i, j)). */
double orc_ltlbar_entry(int n, const double *L, const double *Lbar, int i, int j)
{
    double s = 0.0;
    int k0 = i > j ? i : j;
    for (int k = k0; k < n; ++k)
        s += L[(size_t)k * n + i] * Lbar[(size_t)k * n + j];
    return s;
}

/* Number of threads the batch loops above will use. */
/* ------------------------------------------------------------------------- */
/* Kalman filter (section 3.4, "Kalman Filtering").  Gaussian linear dynamical system
 *   h_t ~ N(A h_{t-1}, S_h),   v_t ~ N(B h_t, S_v),   h_0 ~ N(mu_0, S_0),
 * h of dimension dh, v of dimension dv.  For t = 0 the predicted state is the prior
 * (mu_h = mu_0, S_hh = S_0); for t > 0
 *   mu_h = A f_{t-1},  S_hh = A F_{t-1} A^T + S_h.
 * Then, in the order of the section's equations:
 *   mu_v = B mu_h,  S_vv = B S_hh B^T + S_v = L L^T (potrf),
 *   K = (S_hh B^T) L^{-T} L^{-1}   (two right-side trsm),
 *   f_t = mu_h + K (v_t - mu_v),
 *   F_t = (I - K B) S_hh (I - K B)^T + K S_v K^T.
 * The negative log likelihood the section speaks of is the sum over t of
 * -log N(v_t | mu_v, S_vv) = dv/2 log(2 pi) + sum_i log L_ii + 1/2 |L^{-1}(v_t - mu_v)|^2
 * (the formula is not printed there; it is the density of the predicted observation).
 *
 * Parameters: one set for every sequence (shared != 0) or one per sequence.
 * v: [batch, T, dv].  f: [batch, T, dh] or NULL.  F: [batch, T, dh, dh] or NULL.
 * nll: [batch].  info: [batch] or NULL; 0, or 1 + the first t whose S_vv has a pivot <= 0. */
static void matmul_nn(int m, int n, int k, const double *X, const double *Y, double *Z)
{
    for (int i = 0; i < m; ++i)
        for (int j = 0; j < n; ++j) {
            double s = 0.0;
            for (int p = 0; p < k; ++p)
                s += X[i * k + p] * Y[p * n + j];
            Z[i * n + j] = s;
        }
}
static void matmul_nt(int m, int n, int k, const double *X, const double *Y, double *Z)
{
    /* Z = X Y^T, X is m x k, Y is n x k */
    for (int i = 0; i < m; ++i)
        for (int j = 0; j < n; ++j) {
            double s = 0.0;
            for (int p = 0; p < k; ++p)
                s += X[i * k + p] * Y[j * k + p];
            Z[i * n + j] = s;
        }
}

static void kalman_one(int T, int dh, int dv, const double *A, const double *B, const double *Sh,
                       const double *Sv, const double *mu0, const double *S0, const double *v, double *f,
                       double *F, double *nll, int32_t *info, double *w)
{
    /* work space: all dh x dh unless noted */
    double *fcur = w, *Fcur = fcur + dh, *muh = Fcur + dh * dh, *Shh = muh + dh, *T1 = Shh + dh * dh;
    double *muv = T1 + dh * dh;                 /* dv */
    double *M = muv + dv;                       /* dh x dv: S_hh B^T */
    double *Svv = M + dh * dv, *L = Svv + dv * dv; /* dv x dv */
    double *K = L + dv * dv;                    /* dh x dv */
    double *delta = K + dh * dv, *z = delta + dv; /* dv */
    double *G = z + dv, *T2 = G + dh * dh;      /* dh x dh */
    double *T3 = T2 + dh * dh;                  /* dv x dh: S_v K^T */
    double total = 0.0;
    int32_t bad = 0;
    for (int t = 0; t < T; ++t) {
        if (t == 0) {
            memcpy(muh, mu0, sizeof(double) * dh);
            memcpy(Shh, S0, sizeof(double) * dh * dh);
        } else {
            matmul_nn(dh, 1, dh, A, fcur, muh);
            matmul_nt(dh, dh, dh, Fcur, A, T1);  /* F A^T */
            matmul_nn(dh, dh, dh, A, T1, Shh);
            for (int i = 0; i < dh * dh; ++i)
                Shh[i] += Sh[i];
        }
        matmul_nn(dv, 1, dh, B, muh, muv);
        matmul_nt(dh, dv, dh, Shh, B, M);
        matmul_nn(dv, dv, dh, B, M, Svv);
        for (int i = 0; i < dv * dv; ++i)
            Svv[i] += Sv[i];
        int32_t inf = 0;
        potrf_one_lower(dv, Svv, L, &inf);
        if (inf != 0 && bad == 0)
            bad = t + 1;
        /* K = M L^-T L^-1: X L^T = M, then K L = X */
        trsm_one(1, 1, 1, 1.0, dv, dh, L, M, K);
        trsm_one(1, 0, 1, 1.0, dv, dh, L, K, K);
        for (int i = 0; i < dv; ++i)
            delta[i] = v[(size_t)t * dv + i] - muv[i];
        for (int i = 0; i < dh; ++i) {
            double s = muh[i];
            for (int j = 0; j < dv; ++j)
                s += K[i * dv + j] * delta[j];
            fcur[i] = s;
        }
        matmul_nn(dh, dh, dv, K, B, G);
        for (int i = 0; i < dh; ++i)
            for (int j = 0; j < dh; ++j)
                G[i * dh + j] = (i == j ? 1.0 : 0.0) - G[i * dh + j];
        matmul_nt(dh, dh, dh, Shh, G, T2);   /* S_hh (I - K B)^T */
        matmul_nn(dh, dh, dh, G, T2, Fcur);
        matmul_nt(dv, dh, dv, Sv, K, T3);    /* S_v K^T */
        matmul_nn(dh, dh, dv, K, T3, T2);
        for (int i = 0; i < dh * dh; ++i)
            Fcur[i] += T2[i];
        /* likelihood term */
        trsm_one(1, 0, 0, 1.0, dv, 1, L, delta, z);
        double q = 0.0, ld = 0.0;
        for (int i = 0; i < dv; ++i) {
            q += z[i] * z[i];
            ld += log(L[i * dv + i]);
        }
        total += 0.5 * dv * log(2.0 * M_PI) + ld + 0.5 * q;
        if (f)
            memcpy(f + (size_t)t * dh, fcur, sizeof(double) * dh);
        if (F)
            memcpy(F + (size_t)t * dh * dh, Fcur, sizeof(double) * dh * dh);
    }
    *nll = total;
    if (info)
        *info = bad;
}

int orc_kalman_filter(int64_t batch, int T, int dh, int dv, int shared, const double *A, const double *B,
                      const double *Sh, const double *Sv, const double *mu0, const double *S0, const double *v,
                      double *f, double *F, double *nll, int32_t *info)
{
    if (batch < 0 || T < 0 || dh < 1 || dv < 1)
        return ORC_ERR_INVALID_ARG;
    if (batch == 0)
        return ORC_OK;
    if (!A || !B || !Sh || !Sv || !mu0 || !S0 || !nll || (T > 0 && !v))
        return ORC_ERR_INVALID_ARG;
    size_t words = (size_t)dh * 2 + (size_t)dh * dh * 6 + (size_t)dv * 3 + (size_t)dh * dv * 3 + (size_t)dv * dv * 2;
    int fail = 0;
#pragma omp parallel
    {
        double *w = (double *)malloc(sizeof(double) * words);
        if (!w) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(static)
        for (int64_t b = 0; b < batch; ++b) {
            if (!w)
                continue;
            size_t pb = shared ? 0 : (size_t)b;
            kalman_one(T, dh, dv, A + pb * dh * dh, B + pb * dv * dh, Sh + pb * dh * dh, Sv + pb * dv * dv,
                       mu0 + pb * dh, S0 + pb * dh * dh, v + (size_t)b * T * dv, f ? f + (size_t)b * T * dh : NULL,
                       F ? F + (size_t)b * T * dh * dh : NULL, nll + b, info ? info + b : NULL, w);
        }
        free(w);
    }
    return fail ? ORC_ERR_INVALID_ARG : ORC_OK;
}

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
