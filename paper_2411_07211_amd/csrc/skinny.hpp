// Skinny matrices (Sec. 6.2.2, skinny matrix): gemv in both orientations and ger for row-major
// matrices with very short rows.  Entry points; the kernels live in skinny.hip.
#pragma once
#include "common.hpp"

namespace mxb {

enum SkinnyOp { SKINNY_GEMV_N, SKINNY_GEMV_T, SKINNY_GER };

// Does the skinny path take this operation on a rows x cols row-major matrix with this base and
// pitch?  The limits are where the skinny kernels measured faster than the general ones: rows of
// up to 12 vectors of 16 bytes in fp32 (48 columns; in fp64 only the rank-1 update, up to 20
// vectors = 40 columns), at least one vector per row, and enough rows that the run is not
// launch-bound (the transposed product also has to pay for its second kernel).
template <typename T>
inline bool skinny_takes(SkinnyOp op, int64_t rows, int64_t cols, const T* A, int64_t lda)
{
    const int64_t fv = 16 / (int64_t)sizeof(T);
    (void)A; (void)lda;                       // any base and pitch: matrix accesses need element alignment only
    if (cols < fv) return false;
    const int64_t nv = (cols + fv - 1) / fv;  // a ragged last vector is moved back to end at the last column
    if (sizeof(T) == 8) return op == SKINNY_GER && nv <= 20 && rows >= 100000;
    return nv <= 12 && rows >= (op == SKINNY_GEMV_T ? 500000 : 100000);
}

// y = alpha*A*x + beta*y (A rows x cols, x has cols elements).  Pointers at logical element 0.
template <typename T>
int skinny_gemv_n(mxb_handle_t h, int64_t rows, int64_t cols, T alpha, const T* A, int64_t lda, const T* x0, int64_t incx, T beta,
                  T* y0, int64_t incy);
// y = alpha*A^t*x + beta*y (x has rows elements, y has cols).  Uses the handle's workspace.
template <typename T>
int skinny_gemv_t(mxb_handle_t h, int64_t rows, int64_t cols, T alpha, const T* A, int64_t lda, const T* x0, int64_t incx, T beta,
                  T* y0, int64_t incy);
// A += alpha*x*y^t (x has rows elements, y has cols).
template <typename T>
int skinny_ger(mxb_handle_t h, int64_t rows, int64_t cols, T alpha, const T* x0, int64_t incx, const T* y0, int64_t incy, T* A,
               int64_t lda);
// Workspace bytes skinny_gemv_t needs.
size_t skinny_workspace_bytes(int64_t cols, int elem_size);

}  // namespace mxb
