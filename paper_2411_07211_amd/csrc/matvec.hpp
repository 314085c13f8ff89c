// The two matrix-vector kernels (row-dot, column-accumulate) as the other level-2 routines use
// them: argument blocks and launchers.  The kernels live in matvec.hip.
#pragma once
#include "common.hpp"

namespace mxb {

enum { MODE_GENERAL = 0, MODE_UPPER = 1, MODE_LOWER = 2 };

template <typename T>
struct RowdotArgs {
    int64_t M, N;        // rows and columns of the row-major matrix
    const T* A;
    int64_t lda;
    const T* x;          // logical element 0
    int64_t incx;        // signed
    T* y;                // logical element 0
    int64_t incy;
    T alpha, beta;
    int xchunk;          // elements of x staged per chunk (multiple of 256)
    int x_contig;        // x has unit increment and is 16-byte aligned: stage it with 128-bit loads
    // a batch of problems of this shape: problem b uses A + b*sA, x + b*sx, y + b*sy
    int64_t batch = 1, sA = 0, sx = 0, sy = 0;
};

template <typename T>
struct ColaccArgs {
    int64_t M, N;
    const T* A;
    int64_t lda;
    const T* x;          // logical element 0 (length M)
    int64_t incx;
    T* y;                // logical element 0 (length N); written directly when there is one row group
    int64_t incy;
    T alpha, beta;
    T* partials;         // [row groups][ppitch] when there are several row groups
    int64_t ppitch;      // N rounded up to whole vectors
    int64_t rows_per_block;   // WR == 4 only: rows of one slab
    // a batch of problems of this shape (blockIdx.z): problem b uses A + b*sA, x + b*sx, y + b*sy
    // and the partials at partials + b*spart
    int64_t sA = 0, sx = 0, sy = 0, spart = 0;
};

// Launches the row-dot kernel.  mode: MODE_*, unit: trmv with unit diagonal.  Checks nothing;
// a.xchunk / a.x_contig are filled here.
template <typename T>
int launch_rowdot(mxb_handle_t h, RowdotArgs<T> a, int mode, bool unit);

// Launches the column-accumulate kernel and, where the rows are split, the combine pass, for
// `batch` problems of one shape (a.sA, a.sx, a.sy apart).  Uses the handle's workspace.
template <typename T>
int launch_colacc(mxb_handle_t h, ColaccArgs<T> a, int64_t batch = 1);

}  // namespace mxb
