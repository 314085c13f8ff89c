/*
 * CPU oracle for the BLAS level-1 / level-2 kernel family of Sec. 6.2.1 and 6.2.2.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is linked by nothing but the test-suite, the smoke check
 * and the benchmark's cpu-baseline leg.  It shares no code, header, table or constant with the
 * GPU library and the GPU library never calls it.
 *
 * Host pointers everywhere.  Precision: accumulation in 80-bit long double, one rounding to the
 * element type on store.  See oracle_blas_impl.h for the per-routine statements.
 *
 * Pins (tests/test_oracle_pins.py) tie every routine to closed forms, exact small-integer brute
 * force in int64, hand-worked 2x2/3x3 cases and an independent fp64 library routine, so no
 * routine here is "parity unpinned".
 */
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

#if LDBL_MANT_DIG < 64
#error "the oracle needs a long double with a 64-bit significand (x86-64 gcc)"
#endif

typedef long double acc_t;

enum { ORACLE_ROW_MAJOR = 101, ORACLE_COL_MAJOR = 102 };
enum { ORACLE_NO_TRANS = 111, ORACLE_TRANS = 112 };
enum { ORACLE_UPPER = 121, ORACLE_LOWER = 122 };
enum { ORACLE_NON_UNIT = 131, ORACLE_UNIT = 132 };

#define T float
#define FN(name) oracle_s##name
#include "oracle_blas_impl.h"
#undef T
#undef FN

#define T double
#define FN(name) oracle_d##name
#include "oracle_blas_impl.h"
#undef T
#undef FN

/* dsdot, Sec. 6.2.1: fp32 inputs, products and sum in (at least) double, double result. */
double oracle_dsdot(int64_t n, const float* x, int64_t incx, const float* y, int64_t incy, double* D)
{
    acc_t acc = 0;
    double d = 0;
    for (int64_t k = 0; k < n; ++k) {
        const float xv = x[oracle_spos(k, n, incx)], yv = y[oracle_spos(k, n, incy)];
        acc += (acc_t)xv * (acc_t)yv;
        d += fabs((double)xv * (double)yv);
    }
    if (D) *D = d;
    return (double)acc;
}

