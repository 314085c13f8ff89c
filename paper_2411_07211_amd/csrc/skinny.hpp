// Skinny matrices (Sec. 6.2.2, skinny matrix): gemv in both orientations and ger for row-major
// matrices with very short rows.  Entry points; the kernels live in skinny.hip.
#pragma once
#include "common.hpp"

namespace mxb {

enum SkinnyOp { SKINNY_GEMV_N, SKINNY_GEMV_T, SKINNY_GER };

// Does the skinny path take this operation on a rows x cols row-major matrix with this base and
// pitch?  The limits are where the skinny kernels measured faster than the general ones: in fp32
// rows of up to 12 vectors of 16 bytes (48 columns); in fp64 up to 23 vectors (46 columns; 20 transposed) for
// the products when there are a million rows (half a million transposed), up to 16 (8) columns from
// 100000 rows, and up to 20 vectors (40 columns) for the rank-1 update; at least one vector per
// row, and enough rows that the run is not launch-bound (the transposed product also has to pay
// for its second kernel).  With 4194304 rows of 2 .. 16 doubles the general kernels take 136-183
// us whatever the width, the skinny ones 21-101 us.
template <typename T>
inline bool skinny_takes(SkinnyOp op, int64_t rows, int64_t cols, const T* A, int64_t lda)
{
    const int64_t fv = 16 / (int64_t)sizeof(T);
    (void)A; (void)lda;                       // any base and pitch: matrix accesses need element alignment only
    if (cols < fv) return false;
    const int64_t nv = (cols + fv - 1) / fv;  // a ragged last vector is moved back to end at the last column
    if (sizeof(T) == 8) {
        if (op == SKINNY_GER) return nv <= 20 && rows >= 100000;
        if (op == SKINNY_GEMV_N) return (nv <= 8 && rows >= 100000) || (nv <= 23 && rows >= 1000000);
        return (nv <= 4 && rows >= 100000) || (nv <= 20 && rows >= 500000);
    }
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
