/*
 * Body of the CPU oracle, included once per precision by oracle_blas.c with
 *   T    element type (float or double)
 *   FN() name-mangling macro (oracle_s... / oracle_d...)
 * defined.  TEST INFRASTRUCTURE ONLY: a plain, slow, obviously correct statement of what each
 * routine computes.  Every sum is accumulated in x87 80-bit long double (64-bit significand), in
 * ascending index order, with exactly one rounding to T when the result is stored.  No blocking,
 * no reordering, no vectorisation, no code shared with the GPU library.
 *
 * Each routine follows the loop nest the paper gives as object code (Sec. 2 for gemv, Fig. 4a for
 * axpy, Fig. 7c for transposed gemv, Sec. 6.2.1/6.2.2 for the kernel families) completed with the
 * standard BLAS meaning of alpha, beta, trans, uplo, diag, lda and the increments, which the
 * paper says its kernels handle but leaves out of its listings (Sec. 6.2.2, skinny-matrix
 * paragraph).
 *
 * Every routine can also return, per output element, the "condition denominator" D (in double):
 * the sum of the absolute values of the terms that make up that output.  Tests divide the
 * GPU-vs-oracle difference by D, which keeps a relative-error bound meaningful under cancellation.
 * D pointers may be NULL.
 */

/* Position of logical element k of an n-vector with BLAS increment inc (inc != 0):
 * forward from the base for inc > 0, backwards from element (n-1)*|inc| for inc < 0. */
static int64_t FN(pos)(int64_t k, int64_t n, int64_t inc)
{
    return inc > 0 ? k * inc : (n - 1 - k) * (-inc);
}

/* Element (i, j) of a matrix stored with leading dimension lda in the given layout. */
static T FN(elem)(const T* A, int64_t lda, int layout, int64_t i, int64_t j)
{
    return layout == ORACLE_ROW_MAJOR ? A[i * lda + j] : A[j * lda + i];
}

/* axpy, Fig. 4a: y[i] += a * x[i].  alpha == 0 or n <= 0 leaves y untouched. */
void FN(axpy)(int64_t n, T alpha, const T* x, int64_t incx, T* y, int64_t incy, double* D)
{
    if (n <= 0 || alpha == (T)0) return;
    for (int64_t k = 0; k < n; ++k) {
        const T xv = x[FN(pos)(k, n, incx)];
        T* yp = &y[FN(pos)(k, n, incy)];
        if (D) D[k] = fabs((double)alpha * (double)xv) + fabs((double)*yp);
        *yp = (T)((acc_t)alpha * (acc_t)xv + (acc_t)*yp);
    }
}

/* scal, Sec. 6.2.1: x[i] = alpha * x[i].  Always multiplies.  n <= 0 or incx <= 0: no-op. */
void FN(scal)(int64_t n, T alpha, T* x, int64_t incx, double* D)
{
    if (n <= 0 || incx <= 0) return;
    for (int64_t k = 0; k < n; ++k) {
        T* xp = &x[k * incx];
        if (D) D[k] = fabs((double)alpha * (double)*xp);
        *xp = (T)((acc_t)alpha * (acc_t)*xp);
    }
}

/* dot, Sec. 6.2.1: r = sum_i x[i] * y[i]. */
T FN(dot)(int64_t n, const T* x, int64_t incx, const T* y, int64_t incy, double* D)
{
    acc_t acc = 0;
    double d = 0;
    for (int64_t k = 0; k < n; ++k) {
        const T xv = x[FN(pos)(k, n, incx)];
        const T yv = y[FN(pos)(k, n, incy)];
        acc += (acc_t)xv * (acc_t)yv;
        d += fabs((double)xv * (double)yv);
    }
    if (D) *D = d;
    return (T)acc;
}

/* asum, Sec. 6.2.1: r = sum_i |x[i]|.  n <= 0 or incx <= 0 gives 0. */
T FN(asum)(int64_t n, const T* x, int64_t incx, double* D)
{
    acc_t acc = 0;
    if (n > 0 && incx > 0)
        for (int64_t k = 0; k < n; ++k) acc += fabsl((acc_t)x[k * incx]);
    if (D) *D = (double)acc;
    return (T)acc;
}

/* nrm2: r = sqrt(sum_i x[i]^2).  The paper leaves this one out (Sec. 6.2.1), so this is the plain
 * definition.  The long double exponent range (15 bits) holds the square of any finite double, so
 * no scaling is needed here. */
T FN(nrm2)(int64_t n, const T* x, int64_t incx, double* D)
{
    acc_t acc = 0;
    if (n > 0 && incx > 0)
        for (int64_t k = 0; k < n; ++k) {
            const acc_t v = (acc_t)x[k * incx];
            acc += v * v;
        }
    const acc_t r = sqrtl(acc);
    if (D) *D = (double)r;
    return (T)r;
}

/* gemv, Sec. 2 (no transpose: y[i] += A[i,j] * x[j]) and Fig. 7c (transpose:
 * y[j] += x[i] * A[i,j]), with y = alpha * op(A) x + beta * y.
 * A is m x n.  beta == 0 overwrites y without reading it; alpha == 0 reads neither A nor x. */
void FN(gemv)(int layout, int trans, int64_t m, int64_t n, T alpha, const T* A, int64_t lda,
              const T* x, int64_t incx, T beta, T* y, int64_t incy, double* D)
{
    if (m <= 0 || n <= 0) return;
    if (alpha == (T)0 && beta == (T)1) return;
    const int64_t leny = trans == ORACLE_NO_TRANS ? m : n;
    const int64_t lenx = trans == ORACLE_NO_TRANS ? n : m;
    for (int64_t o = 0; o < leny; ++o) {
        acc_t acc = 0;
        double d = 0;
        if (alpha != (T)0)
            for (int64_t k = 0; k < lenx; ++k) {
                const T a = trans == ORACLE_NO_TRANS ? FN(elem)(A, lda, layout, o, k)
                                                     : FN(elem)(A, lda, layout, k, o);
                const T xv = x[FN(pos)(k, lenx, incx)];
                acc += (acc_t)a * (acc_t)xv;
                d += fabs((double)a * (double)xv);
            }
        T* yp = &y[FN(pos)(o, leny, incy)];
        acc_t r = (acc_t)alpha * acc;
        d = fabs((double)alpha) * d;
        if (beta != (T)0) {
            r += (acc_t)beta * (acc_t)*yp;
            d += fabs((double)beta * (double)*yp);
        }
        if (D) D[o] = d;
        *yp = (T)r;
    }
}

/* A batch of independent gemv calls on operands that lie at fixed distances in memory (Sec. 6.2.2
 * times the standard strided-batch convention): problem b uses A + b*strideA, x + b*stridex and
 * y + b*stridey (element counts; 0 shares an operand among all problems).  D, if given, holds
 * len(y) denominators per problem, one problem after the other. */
void FN(gemv_batched)(int layout, int trans, int64_t m, int64_t n, T alpha, const T* A, int64_t lda,
                      int64_t strideA, const T* x, int64_t incx, int64_t stridex, T beta, T* y,
                      int64_t incy, int64_t stridey, int64_t batch, double* D)
{
    const int64_t leny = trans == ORACLE_NO_TRANS ? m : n;
    for (int64_t b = 0; b < batch; ++b)
        FN(gemv)(layout, trans, m, n, alpha, A + b * strideA, lda, x + b * stridex, incx, beta,
                 y + b * stridey, incy, D ? D + b * leny : 0);
}

/* Is (i, j) inside the stored triangle? */
static int FN(in_tri)(int uplo, int64_t i, int64_t j)
{
    return uplo == ORACLE_UPPER ? j >= i : j <= i;
}

/* trmv, Sec. 6.2.2 (triangular matrices): x := op(T) x with T the uplo triangle of the n x n
 * matrix A; with a unit diagonal the diagonal is taken as 1 and never read.  Elements outside
 * the triangle are never read.  The product uses the x that was passed in. */
void FN(trmv)(int layout, int uplo, int trans, int diag, int64_t n, const T* A, int64_t lda,
              T* x, int64_t incx, double* D)
{
    if (n <= 0) return;
    T* x0 = (T*)malloc((size_t)n * sizeof(T));
    for (int64_t k = 0; k < n; ++k) x0[k] = x[FN(pos)(k, n, incx)];
    for (int64_t o = 0; o < n; ++o) {
        acc_t acc = 0;
        double d = 0;
        for (int64_t k = 0; k < n; ++k) {
            /* op(T)[o][k] = T[o][k] (no transpose) or T[k][o] (transpose) */
            const int64_t i = trans == ORACLE_NO_TRANS ? o : k;
            const int64_t j = trans == ORACLE_NO_TRANS ? k : o;
            if (!FN(in_tri)(uplo, i, j)) continue;
            if (i == j && diag == ORACLE_UNIT) {
                acc += (acc_t)x0[k];
                d += fabs((double)x0[k]);
            } else {
                const T a = FN(elem)(A, lda, layout, i, j);
                acc += (acc_t)a * (acc_t)x0[k];
                d += fabs((double)a * (double)x0[k]);
            }
        }
        if (D) D[o] = d;
        x[FN(pos)(o, n, incx)] = (T)acc;
    }
    free(x0);
}

/* symv, Sec. 6.2.2: y = alpha * S x + beta * y, S symmetric n x n of which only the uplo
 * triangle of A is ever read: S[i][j] = A[i][j] inside the triangle, A[j][i] outside. */
void FN(symv)(int layout, int uplo, int64_t n, T alpha, const T* A, int64_t lda,
              const T* x, int64_t incx, T beta, T* y, int64_t incy, double* D)
{
    if (n <= 0) return;
    if (alpha == (T)0 && beta == (T)1) return;
    for (int64_t i = 0; i < n; ++i) {
        acc_t acc = 0;
        double d = 0;
        if (alpha != (T)0)
            for (int64_t j = 0; j < n; ++j) {
                const T a = FN(in_tri)(uplo, i, j) ? FN(elem)(A, lda, layout, i, j)
                                                   : FN(elem)(A, lda, layout, j, i);
                const T xv = x[FN(pos)(j, n, incx)];
                acc += (acc_t)a * (acc_t)xv;
                d += fabs((double)a * (double)xv);
            }
        T* yp = &y[FN(pos)(i, n, incy)];
        acc_t r = (acc_t)alpha * acc;
        d = fabs((double)alpha) * d;
        if (beta != (T)0) {
            r += (acc_t)beta * (acc_t)*yp;
            d += fabs((double)beta * (double)*yp);
        }
        if (D) D[i] = d;
        *yp = (T)r;
    }
}

/* ger, Sec. 6.2.2: A[i][j] += alpha * x[i] * y[j], A m x n.  D (if given) is m*n, row index
 * major: D[i*n + j]. */
void FN(ger)(int layout, int64_t m, int64_t n, T alpha, const T* x, int64_t incx,
             const T* y, int64_t incy, T* A, int64_t lda, double* D)
{
    if (m <= 0 || n <= 0 || alpha == (T)0) return;
    for (int64_t i = 0; i < m; ++i) {
        const T xv = x[FN(pos)(i, m, incx)];
        for (int64_t j = 0; j < n; ++j) {
            const T yv = y[FN(pos)(j, n, incy)];
            T* ap = layout == ORACLE_ROW_MAJOR ? &A[i * lda + j] : &A[j * lda + i];
            const acc_t t = (acc_t)alpha * (acc_t)xv * (acc_t)yv;
            if (D) D[i * n + j] = fabs((double)*ap) + fabs((double)t);
            *ap = (T)((acc_t)*ap + t);
        }
    }
}

/* ---- rest of the level-2 set of Sec. 6.2.2 (syr, syr2, trsv) ---------------------------------- */

/* syr: A[i][j] += alpha * x[i] * x[j] for (i, j) in the uplo triangle of the n x n matrix A;
 * nothing outside the triangle is read or written.  D (if given) is n*n, D[i*n + j], 0 outside. */
void FN(syr)(int layout, int uplo, int64_t n, T alpha, const T* x, int64_t incx, T* A, int64_t lda,
             double* D)
{
    if (n <= 0 || alpha == (T)0) return;
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = 0; j < n; ++j) {
            if (D) D[i * n + j] = 0;
            if (!FN(in_tri)(uplo, i, j)) continue;
            const T xi = x[FN(pos)(i, n, incx)], xj = x[FN(pos)(j, n, incx)];
            T* ap = layout == ORACLE_ROW_MAJOR ? &A[i * lda + j] : &A[j * lda + i];
            const acc_t t = (acc_t)alpha * (acc_t)xi * (acc_t)xj;
            if (D) D[i * n + j] = fabs((double)*ap) + fabs((double)t);
            *ap = (T)((acc_t)*ap + t);
        }
}

/* syr2: A[i][j] += alpha * x[i] * y[j] + alpha * y[i] * x[j] for (i, j) in the uplo triangle. */
void FN(syr2)(int layout, int uplo, int64_t n, T alpha, const T* x, int64_t incx, const T* y,
              int64_t incy, T* A, int64_t lda, double* D)
{
    if (n <= 0 || alpha == (T)0) return;
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = 0; j < n; ++j) {
            if (D) D[i * n + j] = 0;
            if (!FN(in_tri)(uplo, i, j)) continue;
            const T xi = x[FN(pos)(i, n, incx)], xj = x[FN(pos)(j, n, incx)];
            const T yi = y[FN(pos)(i, n, incy)], yj = y[FN(pos)(j, n, incy)];
            T* ap = layout == ORACLE_ROW_MAJOR ? &A[i * lda + j] : &A[j * lda + i];
            const acc_t t1 = (acc_t)alpha * (acc_t)xi * (acc_t)yj;
            const acc_t t2 = (acc_t)alpha * (acc_t)yi * (acc_t)xj;
            if (D) D[i * n + j] = fabs((double)*ap) + fabs((double)t1) + fabs((double)t2);
            *ap = (T)((acc_t)*ap + t1 + t2);
        }
}

/* trsv: solve op(T) z = b for z, where T is the uplo triangle of the n x n matrix A (unit: the
 * diagonal is taken as 1 and never read) and b is the x passed in; z overwrites x.  Plain
 * substitution in the order the dependences impose (first unknown first), every unknown kept in
 * the accumulator's precision until the end and rounded to T once.  No test for singularity.
 * D[o] (if given) = (|b_o| + sum_{k != o} |op(T)[o][k] z_k|) / |op(T)[o][o]|. */
void FN(trsv)(int layout, int uplo, int trans, int diag, int64_t n, const T* A, int64_t lda, T* x,
              int64_t incx, double* D)
{
    if (n <= 0) return;
    acc_t* z = (acc_t*)malloc((size_t)n * sizeof(acc_t));
    /* op(T) is lower triangular iff (uplo == lower) != (trans == transpose): then the first
     * unknown is z_0 and unknown o depends on k < o; otherwise the last one and k > o. */
    const int op_lower = (uplo == ORACLE_LOWER) != (trans == ORACLE_TRANS);
    for (int64_t step = 0; step < n; ++step) {
        const int64_t o = op_lower ? step : n - 1 - step;
        acc_t acc = (acc_t)x[FN(pos)(o, n, incx)];
        double d = fabs((double)acc);
        const int64_t k0 = op_lower ? 0 : o + 1, k1 = op_lower ? o : n;
        for (int64_t k = k0; k < k1; ++k) {
            /* op(T)[o][k] = T[o][k] (no transpose) or T[k][o] (transpose) */
            const int64_t i = trans == ORACLE_NO_TRANS ? o : k;
            const int64_t j = trans == ORACLE_NO_TRANS ? k : o;
            const T a = FN(elem)(A, lda, layout, i, j);
            acc -= (acc_t)a * z[k];
            d += fabs((double)((acc_t)a * z[k]));
        }
        if (diag == ORACLE_NON_UNIT) {
            const T a = FN(elem)(A, lda, layout, o, o);
            acc /= (acc_t)a;
            d /= fabs((double)a);
        }
        z[o] = acc;
        if (D) D[o] = d;
    }
    for (int64_t o = 0; o < n; ++o) x[FN(pos)(o, n, incx)] = (T)z[o];
    free(z);
}

/* ---- rest of the level-1 set of Sec. 6.2.1 (copy, swap, rot, rotm) and iamax (which, like nrm2,
 *      the paper could not express; plain definition) ------------------------------------------ */

/* copy: y[i] = x[i]. */
void FN(copy)(int64_t n, const T* x, int64_t incx, T* y, int64_t incy)
{
    for (int64_t k = 0; k < n; ++k) y[FN(pos)(k, n, incy)] = x[FN(pos)(k, n, incx)];
}

/* swap: x[i] <-> y[i]. */
void FN(swap)(int64_t n, T* x, int64_t incx, T* y, int64_t incy)
{
    for (int64_t k = 0; k < n; ++k) {
        T* xp = &x[FN(pos)(k, n, incx)];
        T* yp = &y[FN(pos)(k, n, incy)];
        const T t = *xp;
        *xp = *yp;
        *yp = t;
    }
}

/* rot: (x[i], y[i]) := (c*x[i] + s*y[i], c*y[i] - s*x[i]).  D (if given) holds 2n entries:
 * D[2k] for the new x, D[2k+1] for the new y. */
void FN(rot)(int64_t n, T* x, int64_t incx, T* y, int64_t incy, T c, T s, double* D)
{
    for (int64_t k = 0; k < n; ++k) {
        T* xp = &x[FN(pos)(k, n, incx)];
        T* yp = &y[FN(pos)(k, n, incy)];
        const acc_t xv = *xp, yv = *yp;
        if (D) {
            D[2 * k] = fabs((double)c * (double)*xp) + fabs((double)s * (double)*yp);
            D[2 * k + 1] = fabs((double)c * (double)*yp) + fabs((double)s * (double)*xp);
        }
        *xp = (T)((acc_t)c * xv + (acc_t)s * yv);
        *yp = (T)((acc_t)c * yv - (acc_t)s * xv);
    }
}

/* rotm: (x[i], y[i]) := H (x[i], y[i]) with H given by param[0] = flag and param[1..4] =
 * h11, h21, h12, h22:  flag -1: H = [h11 h12; h21 h22];  flag 0: H = [1 h12; h21 1];
 * flag 1: H = [h11 1; -1 h22];  flag -2: H = identity (nothing is touched). */
void FN(rotm)(int64_t n, T* x, int64_t incx, T* y, int64_t incy, const T* param, double* D)
{
    const T flag = param[0];
    if (n <= 0 || flag == (T)-2) return;
    acc_t h11, h12, h21, h22;
    if (flag < (T)0) { h11 = param[1]; h21 = param[2]; h12 = param[3]; h22 = param[4]; }
    else if (flag == (T)0) { h11 = 1; h21 = param[2]; h12 = param[3]; h22 = 1; }
    else { h11 = param[1]; h21 = -1; h12 = 1; h22 = param[4]; }
    for (int64_t k = 0; k < n; ++k) {
        T* xp = &x[FN(pos)(k, n, incx)];
        T* yp = &y[FN(pos)(k, n, incy)];
        const acc_t xv = *xp, yv = *yp;
        if (D) {
            D[2 * k] = fabs((double)(h11 * xv)) + fabs((double)(h12 * yv));
            D[2 * k + 1] = fabs((double)(h21 * xv)) + fabs((double)(h22 * yv));
        }
        *xp = (T)(h11 * xv + h12 * yv);
        *yp = (T)(h21 * xv + h22 * yv);
    }
}

/* iamax: 0-based index of the first element of largest absolute value, found by the sequential
 * scan "best = |x[0]|; for k >= 1: if |x[k]| > best, take k" (so a NaN is never taken, and a NaN
 * in x[0] wins by default).  n <= 0 or incx <= 0 gives 0. */
int64_t FN(iamax)(int64_t n, const T* x, int64_t incx)
{
    if (n <= 0 || incx <= 0) return 0;
    int64_t best = 0;
    T bv = (T)fabs((double)x[0]);
    for (int64_t k = 1; k < n; ++k) {
        const T v = (T)fabs((double)x[k * incx]);
        if (v > bv) { bv = v; best = k; }
    }
    return best;
}

