// Batches of matrices with very short rows (at most 16 vectors of 16 bytes): both products of
// gemv_batched (Sec. 6.2.2 gemv, many small problems in one call).  Entry points; the kernels
// live in tiny.hip.
#pragma once
#include "common.hpp"

namespace mxb {

// Does the tiny path take `batch` products with rows x cols row-major matrices?  Rows narrower
// than one vector run with one element per lane (8 x 1 x 32768 problems: 105 us per call with the
// general kernels).  Transposed, a wavefront works through whole problems, so the batch has to
// fill the device or the problems have to be short: per call 2048 x 40 in a batch of 8 takes 104 us
// that way and 7.3 through the general kernels, in a batch of 2048 it is 47 against 72 for
// 700 x 40 and 33 against 120 for 2048 x 8.
template <typename T>
inline bool tiny_takes(bool no_trans, int64_t rows, int64_t cols, int64_t batch)
{
    const int64_t fv = 16 / (int64_t)sizeof(T);
    if (batch <= 1 || cols > 16 * fv || rows * batch >= ((int64_t)1 << 31)) return false;
    return no_trans || batch >= 2048 || rows <= 32 || (batch >= 512 && cols <= 4 * fv);
}

// y_b = alpha*A_b*x_b + beta*y_b for b < batch (A_b rows x cols, problems sA, sx, sy elements apart).
// Pointers at logical element 0 of problem 0.  No workspace.
template <typename T>
int tiny_gemv_n(mxb_handle_t h, int64_t rows, int64_t cols, T alpha, const T* A, int64_t lda, int64_t sA, const T* x0, int64_t incx,
                int64_t sx, T beta, T* y0, int64_t incy, int64_t sy, int64_t batch);

// y_b = alpha*A_b^t*x_b + beta*y_b (x_b has rows elements, y_b has cols).
template <typename T>
int tiny_gemv_t(mxb_handle_t h, int64_t rows, int64_t cols, T alpha, const T* A, int64_t lda, int64_t sA, const T* x0, int64_t incx,
                int64_t sx, T beta, T* y0, int64_t incy, int64_t sy, int64_t batch);

}  // namespace mxb
