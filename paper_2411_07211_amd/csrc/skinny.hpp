// Skinny matrices (Sec. 6.2.2, skinny matrix): gemv in both orientations and ger for row-major
// matrices with very short rows.  Entry points; the kernels live in skinny.hip.
#pragma once
#include "common.hpp"

namespace mxb {

enum SkinnyOp { SKINNY_GEMV_N, SKINNY_GEMV_T, SKINNY_GER };

// Does the skinny path take this operation on a rows x cols row-major matrix with this base and
// pitch?  The limits are where the skinny kernels measured faster than the general ones (nv =
// 16-byte vectors per row, the last one moved back when the width is ragged):
//   fp32  A*x     nv <= 32 (128 columns), and 48 <= nv <= 64 where a row fills most of a wavefront
//                 (2097152 x 127: 49 -> 80 % of peak, x 100: 55 -> 78 %, x 255: 59 -> 80 %; 1048576 x 256:
//                 161-166 us against the row-dot kernel's 167-172 on the same machine); 37 <= nv <= 47
//                 unless the width is a multiple of 32 (x 170: 305 -> 248 us, x 188: 308 -> 254 us, but
//                 x 160: 217 against 240 us; below, x 129 .. 140: 215-243 against 250-278 us);
//         A^t*x   nv <= 17 (68 columns), from 2049 rows (up to 2048 the single kernel for cache-sized matrices
//                 takes them; per call 177147 x 40: 8.4 against 12.9 us, 65536 x 64: 7.0 against 9.3, x 16: 5.7
//                 against 7.8; 19683 x 40 is the one loss, 6.8 against 6.5);
//         x*y^t   nv <= 12, and up to 20 for whole vectors (x 64: 52 -> 70 %, x 72: 273 -> 236 us, x 80:
//                 282 -> 249 us; x 96 ties; ragged rows lose);
//   fp64  A*x     nv <= 8 from 65536 rows; from a million nv <= 31, and 32 for the odd width
//                 (2097152 x 42: 167 -> 126 us, x 50: 205 -> 155 us, x 63: 258 -> 182 us; x 64 ties; one
//                 row per wavefront, x 65 .. 96, loses: 230-270 against 314-325 us) (4194304 rows of
//                 2 .. 16 doubles: the general kernels take 136-183 us whatever the width, these
//                 21-101 us);
//         A^t*x   nv <= 8 from 2049 rows (177147 x 16: 10.4 against 14.2 us), nv <= 20 from 500000 (x 40 loses
//                 below: 65536 rows 10.1 against 7.8 us);   x*y^t   nv <= 20, from 16384 rows.
// Enough rows that the run is not launch-bound.
template <typename T>
inline bool skinny_takes(SkinnyOp op, int64_t rows, int64_t cols, const T* A, int64_t lda)
{
    const int64_t fv = 16 / (int64_t)sizeof(T);
    (void)A; (void)lda;                       // any base and pitch: matrix accesses need element alignment only
    // rows narrower than one vector (1 to 3 floats, 1 double): the same kernels with one element per lane.  The
    // general kernels give such a row a lane (per call: 8388608 x 1 A*x 186 -> 20 us, A^t*x 211 -> 20, x*y^t
    // 535 -> 20; x 3: 186 -> 36, 212 -> 26, 536 -> 41; 65536 x 1: 4.5 -> 4.2, 6.9 against 8.8, 7.8 -> 4.1)
    if (cols < fv) return rows >= (op == SKINNY_GER ? 16384 : (op == SKINNY_GEMV_N ? 65536 : 200000));
    const int64_t nv = (cols + fv - 1) / fv;  // a ragged last vector is moved back to end at the last column
    if (sizeof(T) == 8) {
        // (per call, 65536 rows: x*y^t of 2 / 16 / 40 doubles 9.2 / 10.1 / 11.2 -> 4.5 / 5.5 / 8.0 us, A*x of 2 / 16: 5.1 / 5.9 -> 4.4 / 5.2)
        if (op == SKINNY_GER) return nv <= 20 && rows >= 16384;
        if (op == SKINNY_GEMV_N) return (nv <= 8 && rows >= 65536) || ((nv <= 31 || (nv == 32 && cols % 2 == 1)) && rows >= 1000000);
        return (nv <= 8 && rows > 2048) || (nv <= 20 && rows >= 500000);
    }
    // rows from which these kernels win (per call, 65536 rows: x*y^t of 40 columns 5.6 against 9.0 us, A*x of
    // 128 columns 6.9 against 14.5, of 64 columns 5.4 against 6.2; 8192 rows: 4.0 against 3.5, 5.1 against 3.9)
    if (op == SKINNY_GER) return (nv <= 12 || (nv <= 20 && cols % fv == 0)) && rows >= 16384;
    if (op == SKINNY_GEMV_N)
        return (nv <= 32 || (nv >= 37 && nv <= 47 && cols % 32 != 0) || (nv >= 48 && nv <= 64)) &&
               rows >= (nv >= 32 ? 16384 : (nv >= 16 ? 65536 : 100000));
    return nv <= 17 && rows > 2048;
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
