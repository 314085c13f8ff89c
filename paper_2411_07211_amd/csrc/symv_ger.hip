// symv and ger (Sec. 6.2.2) on a row-major matrix.
//
// symv reads the stored triangle exactly once with the triangle sweep of trisweep.hip: every
// stored element A[i,j] is used twice, A[i,j]*x[j] for row i and, off the diagonal, A[i,j]*x[i]
// for column j.  This file holds its argument checks and the alpha == 0 case.
//
// ger is a streaming read-modify-write of A with the y slice of every lane held in registers.
#include "common.hpp"
#include "options.hpp"
#include "plan.hpp"
#include "trisweep.hpp"

namespace mxb {
namespace {

__device__ __forceinline__ int64_t imin(int64_t a, int64_t b) { return a < b ? a : b; }

constexpr int kThreads = 256;

template <typename T>
__global__ void __launch_bounds__(256) scale_y_kernel(int64_t n, T beta, T* __restrict__ y, int64_t incy)
{
    const int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (k < n) y[k * incy] = beta == T(0) ? T(0) : beta * y[k * incy];
}

// ---------------------------------------------------------------------------------------------
// ger

template <typename T>
struct GerArgs {
    int64_t M, N;
    T* A;
    int64_t lda;
    const T* x;
    int64_t incx;
    const T* y;
    int64_t incy;
    T alpha;
    int64_t rows_per_block;
};

template <typename T, int VEC>
__global__ void __launch_bounds__(kThreads) ger_kernel(const GerArgs<T> p)
{
    typedef typename VecOf<T, VEC>::type V;
    constexpr int U = 8;
    const int64_t c = ((int64_t)blockIdx.x * kThreads + threadIdx.x) * VEC;
    if (c + VEC > p.N) return;
    T yj[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) yj[k] = p.y[(c + k) * p.incy];
    const int64_t rlo = (int64_t)blockIdx.y * p.rows_per_block, rhi = imin(p.M, rlo + p.rows_per_block);
    T* acol = p.A + c;
    int64_t i0 = rlo;
    for (; i0 + U <= rhi; i0 += U) {
        V a[U];
        T ax[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            a[u] = ld_stream(reinterpret_cast<const V*>(acol + (i0 + u) * p.lda));
            ax[u] = p.alpha * p.x[(i0 + u) * p.incx];
        }
        __builtin_amdgcn_sched_barrier(0);   // all loads of the batch are in flight before the first store
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int k = 0; k < VEC; ++k) a[u][k] = fmad(ax[u], yj[k], a[u][k]);
            st_stream(reinterpret_cast<V*>(acol + (i0 + u) * p.lda), a[u]);
        }
    }
    for (; i0 < rhi; ++i0) {
        V a = ld_stream(reinterpret_cast<const V*>(acol + i0 * p.lda));
        const T ax = p.alpha * p.x[i0 * p.incx];
#pragma unroll
        for (int k = 0; k < VEC; ++k) a[k] = fmad(ax, yj[k], a[k]);
        st_stream(reinterpret_cast<V*>(acol + i0 * p.lda), a);
    }
}

// ---------------------------------------------------------------------------------------------
// launchers

inline bool layout_ok(int v) { return v == MXB_ROW_MAJOR || v == MXB_COL_MAJOR; }
inline bool uplo_ok(int v) { return v == MXB_UPPER || v == MXB_LOWER; }

template <typename T>
int symv(mxb_handle_t h, int layout, int uplo, int64_t n, T alpha, const T* A, int64_t lda, const T* x, int64_t incx, T beta,
         T* y, int64_t incy)
{
    if (!handle_ok(h)) return MXB_ERR_HANDLE;
    if (!layout_ok(layout)) return -1;
    if (!uplo_ok(uplo)) return -2;
    if (n < 0) return -3;
    if (lda < (n > 1 ? n : 1)) return -6;
    if (incx == 0) return -8;
    if (incy == 0) return -11;
    if (n == 0 || (alpha == T(0) && beta == T(1))) return MXB_OK;
    if (!y) return -10;
    T* y0 = vec_base(y, n, incy);
    if (alpha == T(0)) {
        hipLaunchKernelGGL(scale_y_kernel<T>, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, h->stream, n, beta, y0, incy);
        return launch_status();
    }
    if (!A) return -5;
    if (!x) return -7;
    // the column-major upper triangle occupies the bytes of the row-major lower triangle
    const bool upper = (uplo == MXB_UPPER) == (layout == MXB_ROW_MAJOR);
    const T* x0 = vec_base(x, n, incx);
    return trisweep_symv<T>(h, upper, n, alpha, A, lda, x0, incx, beta, y0, incy);
}

template <typename T>
int ger(mxb_handle_t h, int layout, int64_t m, int64_t n, T alpha, const T* x, int64_t incx, const T* y, int64_t incy, T* A,
        int64_t lda)
{
    if (!handle_ok(h)) return MXB_ERR_HANDLE;
    if (!layout_ok(layout)) return -1;
    if (m < 0) return -2;
    if (n < 0) return -3;
    if (incx == 0) return -6;
    if (incy == 0) return -8;
    const int64_t minor = layout == MXB_ROW_MAJOR ? n : m;
    if (lda < (minor > 1 ? minor : 1)) return -10;
    if (m == 0 || n == 0 || alpha == T(0)) return MXB_OK;
    if (!x) return -5;
    if (!y) return -7;
    if (!A) return -9;
    // column-major A (m x n) is the row-major n x m matrix: A^T += alpha * y x^T
    GerArgs<T> a;
    if (layout == MXB_ROW_MAJOR) a = GerArgs<T>{m, n, A, lda, vec_base(x, m, incx), incx, vec_base(y, n, incy), incy, alpha, 0};
    else a = GerArgs<T>{n, m, A, lda, vec_base(y, n, incy), incy, vec_base(x, m, incx), incx, alpha, 0};
    a.rows_per_block = option(h, MXB_OPT_GER_ROWS_PER_BLOCK);
    constexpr int FV = Full<T>::vec;
    const bool vec = aligned16(A) && (lda % FV) == 0 && (a.N % FV) == 0;
    const int v = vec ? FV : 1;
    const dim3 grid((unsigned)ceil_div(a.N, (int64_t)kThreads * v), (unsigned)ceil_div(a.M, a.rows_per_block));
    if (vec) hipLaunchKernelGGL((ger_kernel<T, FV>), grid, dim3(kThreads), 0, h->stream, a);
    else hipLaunchKernelGGL((ger_kernel<T, 1>), grid, dim3(kThreads), 0, h->stream, a);
    return launch_status();
}

}  // namespace
}  // namespace mxb

extern "C" {
int mxb_ssymv(mxb_handle_t h, mxb_layout_t layout, mxb_uplo_t uplo, int64_t n, float alpha, const float* A, int64_t lda,
              const float* x, int64_t incx, float beta, float* y, int64_t incy)
{ return mxb::symv<float>(h, layout, uplo, n, alpha, A, lda, x, incx, beta, y, incy); }
int mxb_dsymv(mxb_handle_t h, mxb_layout_t layout, mxb_uplo_t uplo, int64_t n, double alpha, const double* A, int64_t lda,
              const double* x, int64_t incx, double beta, double* y, int64_t incy)
{ return mxb::symv<double>(h, layout, uplo, n, alpha, A, lda, x, incx, beta, y, incy); }
int mxb_sger(mxb_handle_t h, mxb_layout_t layout, int64_t m, int64_t n, float alpha, const float* x, int64_t incx,
             const float* y, int64_t incy, float* A, int64_t lda)
{ return mxb::ger<float>(h, layout, m, n, alpha, x, incx, y, incy, A, lda); }
int mxb_dger(mxb_handle_t h, mxb_layout_t layout, int64_t m, int64_t n, double alpha, const double* x, int64_t incx,
             const double* y, int64_t incy, double* A, int64_t lda)
{ return mxb::ger<double>(h, layout, m, n, alpha, x, incx, y, incy, A, lda); }
}
