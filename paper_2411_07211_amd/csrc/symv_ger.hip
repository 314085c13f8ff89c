// symv and ger (Sec. 6.2.2) on a row-major matrix.
//
// symv reads the stored triangle once.  The triangle is cut into tiles of TR rows by 256*VEC
// columns (tile-granular triangular bounds, as in the paper's bound rounding; elements of a
// diagonal tile that fall outside the triangle are discarded with a select).  Every stored
// element A[i,j] is used twice: A[i,j]*x[j] goes to row i (folded across the wavefront with DPP,
// across the block through LDS) and, off the diagonal, A[i,j]*x[i] goes to column j (a register
// of the lane that owns the column).  Each tile hands a partial row-sum vector and a partial
// column-sum vector to a second kernel, which adds them in tile order and applies alpha/beta.
//
// ger is a streaming read-modify-write of A with the y slice of every lane held in registers.
#include "common.hpp"
#include "options.hpp"
#include "plan.hpp"

namespace mxb {
namespace {

__device__ __forceinline__ int64_t imin(int64_t a, int64_t b) { return a < b ? a : b; }
__device__ __forceinline__ int64_t imax(int64_t a, int64_t b) { return a > b ? a : b; }

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kMaxTileRows = 256;

template <typename T>
struct SymvArgs {
    int64_t n;
    const T* A;
    int64_t lda;
    const T* x;        // logical element 0
    int64_t incx;
    T* rowpart;        // [ncol_tiles][n]
    T* colpart;        // [nrow_tiles][n]
    int tile_rows;
};

// Is tile (row tile rt, column tile ct) touched by the stored triangle?
__host__ __device__ __forceinline__ bool symv_tile_active(bool upper, int64_t rt, int64_t ct, int64_t TR, int64_t TC)
{
    return upper ? ct * TC + TC - 1 >= rt * TR : rt * TR + TR - 1 >= ct * TC;
}

template <typename T, int VEC, bool UPPER>
__global__ void __launch_bounds__(kThreads) symv_tile_kernel(const SymvArgs<T> p)
{
    typedef typename VecOf<T, VEC>::type V;
    constexpr int U = 4;
    constexpr int TC = kThreads * VEC;
    __shared__ T rowsum[kMaxTileRows][kWaves];

    const int64_t ct = blockIdx.x, rt = blockIdx.y;
    const int64_t TR = p.tile_rows;
    if (!symv_tile_active(UPPER, rt, ct, TR, TC)) return;

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t cb0 = ct * TC, rb0 = rt * TR;
    const int64_t c = cb0 + (int64_t)threadIdx.x * VEC;
    const bool col_ok = c + VEC <= p.n;
    const int64_t cb1 = imin(p.n, cb0 + TC);
    // rows of this tile that have stored elements in these columns
    int64_t rlo = rb0, rhi = imin(p.n, rb0 + TR);
    if (UPPER) rhi = imin(rhi, cb1);       // i <= j
    else rlo = imax(rlo, cb0);             // i >= j

    T xj[VEC], cacc[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) {
        xj[k] = col_ok ? p.x[(c + k) * p.incx] : T(0);
        cacc[k] = T(0);
    }
    const T* acol = p.A + (col_ok ? c : 0);

    for (int64_t i0 = rlo; i0 < rhi; i0 += U) {
        V a[U];
        T xi[U], rsum[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = imin(i0 + u, rhi - 1);           // clamp: the load stays in bounds
            a[u] = V(T(0));
            if (col_ok) a[u] = ld_stream(reinterpret_cast<const V*>(acol + i * p.lda));
            xi[u] = p.x[i * p.incx];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = i0 + u;
            const bool row_ok = i < rhi;
            T rs = T(0);
#pragma unroll
            for (int k = 0; k < VEC; ++k) {
                const int64_t j = c + k;
                const bool stored = row_ok && col_ok && (UPPER ? j >= i : j <= i);
                const T v = stored ? a[u][k] : T(0);
                rs = __builtin_fma(v, xj[k], rs);
                cacc[k] = __builtin_fma((i != j) ? v : T(0), xi[u], cacc[k]);
            }
            rsum[u] = rs;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const T s = wave_sum(rsum[u]);
            if (lane == 0 && i0 + u < rhi) rowsum[i0 + u - rb0][wave] = s;
        }
    }
    __syncthreads();
    for (int64_t i = rlo + threadIdx.x; i < rhi; i += kThreads) {
        T s = rowsum[i - rb0][0];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) s += rowsum[i - rb0][w];
        p.rowpart[ct * p.n + i] = s;
    }
    if (col_ok) {
        V v;
#pragma unroll
        for (int k = 0; k < VEC; ++k) v[k] = cacc[k];
        *reinterpret_cast<V*>(p.colpart + rt * p.n + c) = v;
    }
}

constexpr int kCombineGroups = 16;

// y[i] = alpha*(sum over active column tiles of rowpart + sum over active row tiles of colpart)
//        + beta*y[i], each list in ascending tile order.
template <typename T, bool UPPER>
__global__ void __launch_bounds__(kCombineGroups* kWave) symv_combine_kernel(int64_t n, int64_t TR, int64_t TC, int64_t nrt, int64_t nct,
                                                                             const T* __restrict__ rowpart,
                                                                             const T* __restrict__ colpart, T alpha, T beta,
                                                                             T* __restrict__ y, int64_t incy)
{
    __shared__ T red[kCombineGroups][kWave];
    const int tx = threadIdx.x & (kWave - 1), ty = threadIdx.x >> 6;
    const int64_t i = (int64_t)blockIdx.x * kWave + tx;
    T s = T(0);
    if (i < n) {
        const int64_t rt = i / TR, ct = i / TC;
        // A row tile rt wrote rowpart[q][i] for its active column tiles q with a non-empty row
        // range containing i; column tile ct wrote colpart[q][i] for its active row tiles q.
        // Rows of a tile outside the clipped range [rlo, rhi) were not written: skip them.
        for (int64_t q = ty; q < nct; q += kCombineGroups) {
            if (!symv_tile_active(UPPER, rt, q, TR, TC)) continue;
            const int64_t cb0 = q * TC, cb1 = (q + 1) * TC < n ? (q + 1) * TC : n;
            const bool wrote = UPPER ? i < cb1 : i >= cb0;
            if (wrote) s += rowpart[q * n + i];
        }
        for (int64_t q = ty; q < nrt; q += kCombineGroups)
            if (symv_tile_active(UPPER, q, ct, TR, TC)) s += colpart[q * n + i];
    }
    red[ty][tx] = s;
    __syncthreads();
    if (ty != 0 || i >= n) return;
    T tot = red[0][tx];
#pragma unroll
    for (int k = 1; k < kCombineGroups; ++k) tot += red[k][tx];
    T* yp = y + i * incy;
    T v = alpha * tot;
    if (beta != T(0)) v = __builtin_fma(beta, *yp, v);
    *yp = v;
}

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
            for (int k = 0; k < VEC; ++k) a[u][k] = __builtin_fma(ax[u], yj[k], a[u][k]);
            st_stream(reinterpret_cast<V*>(acol + (i0 + u) * p.lda), a[u]);
        }
    }
    for (; i0 < rhi; ++i0) {
        V a = ld_stream(reinterpret_cast<const V*>(acol + i0 * p.lda));
        const T ax = p.alpha * p.x[i0 * p.incx];
#pragma unroll
        for (int k = 0; k < VEC; ++k) a[k] = __builtin_fma(ax, yj[k], a[k]);
        st_stream(reinterpret_cast<V*>(acol + i0 * p.lda), a);
    }
}

// ---------------------------------------------------------------------------------------------
// launchers

inline bool layout_ok(int v) { return v == MXB_ROW_MAJOR || v == MXB_COL_MAJOR; }
inline bool uplo_ok(int v) { return v == MXB_UPPER || v == MXB_LOWER; }

template <typename T, int VEC>
int symv_launch(mxb_handle_t h, bool upper, int64_t n, T alpha, const T* A, int64_t lda, const T* x0, int64_t incx, T beta,
                T* y0, int64_t incy)
{
    const SymvPlan pl = symv_plan(n, VEC, option(h, MXB_OPT_SYMV_TILE_ROWS));
    const size_t need = (size_t)(pl.ncol_tiles + pl.nrow_tiles) * (size_t)n * sizeof(T);
    if (!h->ws || h->ws_bytes < need) return MXB_ERR_WORKSPACE;
    T* rowpart = static_cast<T*>(h->ws);
    T* colpart = rowpart + pl.ncol_tiles * n;
    SymvArgs<T> a{n, A, lda, x0, incx, rowpart, colpart, (int)pl.tile_rows};
    const dim3 grid((unsigned)pl.ncol_tiles, (unsigned)pl.nrow_tiles);
    if (upper) hipLaunchKernelGGL((symv_tile_kernel<T, VEC, true>), grid, dim3(kThreads), 0, h->stream, a);
    else hipLaunchKernelGGL((symv_tile_kernel<T, VEC, false>), grid, dim3(kThreads), 0, h->stream, a);
    int st = launch_status();
    if (st != MXB_OK) return st;
    const dim3 cgrid((unsigned)ceil_div(n, kWave));
    if (upper)
        hipLaunchKernelGGL((symv_combine_kernel<T, true>), cgrid, dim3(kCombineGroups * kWave), 0, h->stream, n, pl.tile_rows,
                           pl.tile_cols, pl.nrow_tiles, pl.ncol_tiles, rowpart, colpart, alpha, beta, y0, incy);
    else
        hipLaunchKernelGGL((symv_combine_kernel<T, false>), cgrid, dim3(kCombineGroups * kWave), 0, h->stream, n, pl.tile_rows,
                           pl.tile_cols, pl.nrow_tiles, pl.ncol_tiles, rowpart, colpart, alpha, beta, y0, incy);
    return launch_status();
}

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
    constexpr int FV = Full<T>::vec;
    const bool vec = aligned16(A) && (lda % FV) == 0 && (n % FV) == 0;
    return vec ? symv_launch<T, FV>(h, upper, n, alpha, A, lda, x0, incx, beta, y0, incy)
               : symv_launch<T, 1>(h, upper, n, alpha, A, lda, x0, incx, beta, y0, incy);
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
