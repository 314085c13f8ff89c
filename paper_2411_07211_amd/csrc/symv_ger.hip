// symv and ger (Sec. 6.2.2) on a row-major matrix.
//
// symv reads the stored triangle exactly once, as one front-to-back sweep.  The triangle is cut
// into column tiles (tile-granular triangular bounds, as in the paper's bound rounding); a block
// owns one tile and takes batches of adjacent rows cyclically with the other blocks of the tile.
// Every stored element A[i,j] is used twice: A[i,j]*x[j] goes to row i (folded across the
// wavefront with DPP, one partial per wavefront) and, off the diagonal, A[i,j]*x[i] goes to
// column j (a register of the lane that owns the column).  In the rows that cross the diagonal,
// elements outside the triangle are discarded with a select, and a 128-bit load that would lie
// wholly outside the triangle is redirected to the vector that holds the diagonal element (a line
// the neighbouring lanes fetch anyway), so no byte outside the triangle is pulled from HBM.
// A second kernel adds the partials in a fixed order and applies alpha/beta.
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

template <typename T>
struct SymvArgs {
    int64_t n;
    const T* A;
    int64_t lda;
    const T* x;        // logical element 0
    int64_t incx;
    T* rowpart;        // [ntiles * 4 wavefronts][n]
    T* colpart;        // [max_groups][n]
    int ntiles;
    int first_block[kSymvMaxTiles + 1];
};

// One batch: U adjacent rows starting at rb, CV vectors per lane.  Rows and columns are below
// 2^31 (the tile table caps n), so the index arithmetic is 32-bit; only addresses are 64-bit.
template <typename T, int VEC, int CV, bool UPPER, bool MASKED>
__device__ __forceinline__ void symv_batch(const SymvArgs<T>& p, int rb, int rlo, int rend, int c, const T* const (&acol)[CV],
                                           const bool (&col_ok)[CV], const T (&xj)[CV][VEC], T (&cacc)[CV][VEC], T* rowpart_wave,
                                           int lane)
{
    typedef typename VecOf<T, VEC>::type V;
    constexpr int U = CV == 4 ? 4 : 8;
    constexpr int SPAN = kThreads * VEC;
    V a[U][CV];
    T xi[U];
    // Masked batches: a vector index whose 64 lanes all lie outside the triangle for every row of
    // the batch is skipped by the whole wavefront (a scalar branch): no loads, no arithmetic.
    bool dead[CV];
#pragma unroll
    for (int v = 0; v < CV; ++v) {
        const int cw = __builtin_amdgcn_readfirstlane(c - lane * VEC) + v * SPAN;      // first column of the wavefront's vector v
        dead[v] = MASKED && (UPPER ? cw + kWave * VEC - 1 < rb : cw > rb + U - 1);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        int i = rb + u;
        if (MASKED) i = min(max(i, rlo), rend - 1);              // clamp: the load stays inside the tile's rows
        const T* arow = p.A + (int64_t)i * p.lda;
#pragma unroll
        for (int v = 0; v < CV; ++v) {
            if (MASKED && dead[v]) {
                a[u][v] = V(T(0));
            } else if (MASKED) {
                int cc = c + v * SPAN;
                const int diag = i / VEC * VEC;                  // vector that holds the diagonal element of row i
                cc = UPPER ? max(cc, diag) : min(cc, diag);      // wholly outside the triangle: read that one instead
                cc = min(cc, (int)p.n - VEC);                    // lanes past the last column
                a[u][v] = ld_stream(reinterpret_cast<const V*>(arow + cc));
            } else {
                a[u][v] = ld_stream(reinterpret_cast<const V*>(acol[v] + (int64_t)i * p.lda));
            }
        }
        xi[u] = p.x[(int64_t)i * p.incx];
    }
    __builtin_amdgcn_sched_barrier(0);   // keep every load of the batch ahead of the first FMA
    T rs[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int i = rb + u;
        T r = T(0);
#pragma unroll
        for (int v = 0; v < CV; ++v) {
            // d = position of the diagonal inside this vector: element k is stored iff k <= d (lower) / k >= d (upper)
            if (MASKED && dead[v]) continue;
            const int d = i - (c + v * SPAN);
            const bool live = MASKED ? (i >= rlo && i < rend && col_ok[v]) : true;
#pragma unroll
            for (int k = 0; k < VEC; ++k) {
                T val = a[u][v][k];
                if (MASKED) {
                    const T in_row = (live && (UPPER ? k >= d : k <= d)) ? val : T(0);
                    const T in_col = (live && (UPPER ? k > d : k < d)) ? val : T(0);
                    r = fmad(in_row, xj[v][k], r);
                    cacc[v][k] = fmad(in_col, xi[u], cacc[v][k]);
                } else {
                    r = fmad(val, xj[v][k], r);
                    cacc[v][k] = fmad(val, xi[u], cacc[v][k]);
                }
            }
        }
        rs[u] = r;
    }
    // fold each row over the wavefront; lane u then stores row u's partial
    T out = T(0);
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const T sum = wave_sum(rs[u]);
        out = lane == u ? sum : out;
    }
    const int i = rb + lane;
    if (lane < U && i >= rlo && i < rend) rowpart_wave[i] = out;
}

template <typename T, int VEC, int CV, bool UPPER>
__global__ void __launch_bounds__(kThreads) symv_sweep_kernel(const SymvArgs<T> p)
{
    constexpr int U = CV == 4 ? 4 : 8;
    constexpr int SPAN = kThreads * VEC;
    constexpr int TC = CV * SPAN;

    int t = 0;
    while (t + 1 < p.ntiles && (int)blockIdx.x >= p.first_block[t + 1]) ++t;
    const int64_t s = (int)blockIdx.x - p.first_block[t];
    const int64_t S = p.first_block[t + 1] - p.first_block[t];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = (int)p.n;
    const int cb0 = t * TC, cb1 = min(n, cb0 + TC);
    const int c = cb0 + (int)threadIdx.x * VEC;
    const int rlo = UPPER ? 0 : cb0, rend = UPPER ? cb1 : n;     // rows with stored elements in these columns
    const bool full_tile = cb0 + TC <= n;

    bool col_ok[CV];
    const T* acol[CV];
    T xj[CV][VEC], cacc[CV][VEC];
#pragma unroll
    for (int v = 0; v < CV; ++v) {
        col_ok[v] = c + v * SPAN + VEC <= n;
        acol[v] = p.A + (col_ok[v] ? c + v * SPAN : cb0);
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            xj[v][k] = col_ok[v] ? p.x[(int64_t)(c + v * SPAN + k) * p.incx] : T(0);
            cacc[v][k] = T(0);
        }
    }
    T* rowpart_wave = p.rowpart + ((int64_t)t * kWaves + wave) * p.n;

    // batches of U adjacent rows, dealt cyclically to the S blocks of this tile
    const int rbase = rlo / U * U;
    for (int64_t rb64 = rbase + s * U; rb64 < rend; rb64 += S * U) {
        const int rb = (int)rb64;
        // no element of the batch touches the diagonal or the ragged edges: no masks needed
        const bool interior = full_tile && rb + U <= rend && (UPPER ? rb + U <= cb0 : rb >= cb1);
        if (interior) symv_batch<T, VEC, CV, UPPER, false>(p, rb, rlo, rend, c, acol, col_ok, xj, cacc, rowpart_wave, lane);
        else symv_batch<T, VEC, CV, UPPER, true>(p, rb, rlo, rend, c, acol, col_ok, xj, cacc, rowpart_wave, lane);
    }

    typedef typename VecOf<T, VEC>::type V;
#pragma unroll
    for (int v = 0; v < CV; ++v) {
        if (!col_ok[v]) continue;
        V val;
#pragma unroll
        for (int k = 0; k < VEC; ++k) val[k] = cacc[v][k];
        *reinterpret_cast<V*>(p.colpart + s * p.n + c + v * SPAN) = val;
    }
}

constexpr int kCombineGroups = 16;

// y[i] = alpha*(column partials of i's tile, then the row partials of every tile whose rows
//        include i, each list in ascending order) + beta*y[i].
template <typename T, bool UPPER>
__global__ void __launch_bounds__(kCombineGroups* kWave) symv_combine_kernel(const SymvArgs<T> p, int64_t TC, T alpha, T beta,
                                                                             T* __restrict__ y, int64_t incy)
{
    __shared__ T red[kCombineGroups][kWave];
    const int tx = threadIdx.x & (kWave - 1), ty = threadIdx.x >> 6;
    const int64_t i = (int64_t)blockIdx.x * kWave + tx;
    T s = T(0);
    if (i < p.n) {
        const int64_t t = i / TC;
        const int64_t ngroups = p.first_block[t + 1] - p.first_block[t];
        for (int64_t q = ty; q < ngroups; q += kCombineGroups) s += p.colpart[q * p.n + i];
        // tile q visited row i iff i >= its first column (lower) / i < its end column (upper)
        const int64_t q0 = UPPER ? t : 0, q1 = UPPER ? p.ntiles : t + 1;
        for (int64_t e = q0 * kWaves + ty; e < q1 * kWaves; e += kCombineGroups) s += p.rowpart[e * p.n + i];
    }
    red[ty][tx] = s;
    __syncthreads();
    if (ty != 0 || i >= p.n) return;
    T tot = red[0][tx];
#pragma unroll
    for (int k = 1; k < kCombineGroups; ++k) tot += red[k][tx];
    T* yp = y + i * incy;
    T v = alpha * tot;
    if (beta != T(0)) v = fmad(beta, *yp, v);
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

template <typename T, int VEC, int CV>
void symv_launch_inst(mxb_handle_t h, bool upper, const SymvArgs<T>& a, int blocks)
{
    if (upper) hipLaunchKernelGGL((symv_sweep_kernel<T, VEC, CV, true>), dim3((unsigned)blocks), dim3(kThreads), 0, h->stream, a);
    else hipLaunchKernelGGL((symv_sweep_kernel<T, VEC, CV, false>), dim3((unsigned)blocks), dim3(kThreads), 0, h->stream, a);
}

template <typename T, int VEC>
int symv_launch(mxb_handle_t h, bool upper, int64_t n, T alpha, const T* A, int64_t lda, const T* x0, int64_t incx, T beta,
                T* y0, int64_t incy)
{
    if (n > 0x7fffffff - 4096) return MXB_ERR_NOT_IMPLEMENTED;
    const SymvPlan pl = symv_plan(n, VEC, upper, option(h, MXB_OPT_SYMV_TARGET_BLOCKS), option(h, MXB_OPT_SYMV_TILE_VECTORS));
    if (!pl.ok) return MXB_ERR_NOT_IMPLEMENTED;
    const size_t need = ((size_t)pl.ntiles * kWaves + (size_t)pl.max_groups) * (size_t)n * sizeof(T);
    if (!h->ws || h->ws_bytes < need) return MXB_ERR_WORKSPACE;
    SymvArgs<T> a;
    a.n = n; a.A = A; a.lda = lda; a.x = x0; a.incx = incx;
    a.rowpart = static_cast<T*>(h->ws);
    a.colpart = a.rowpart + (int64_t)pl.ntiles * kWaves * n;
    a.ntiles = pl.ntiles;
    for (int t = 0; t <= pl.ntiles; ++t) a.first_block[t] = pl.first_block[t];
    const int blocks = pl.first_block[pl.ntiles];
    if (pl.cv == 4) symv_launch_inst<T, VEC, 4>(h, upper, a, blocks);
    else if (pl.cv == 2) symv_launch_inst<T, VEC, 2>(h, upper, a, blocks);
    else symv_launch_inst<T, VEC, 1>(h, upper, a, blocks);
    int st = launch_status();
    if (st != MXB_OK) return st;
    const dim3 cgrid((unsigned)ceil_div(n, kWave)), cblock(kCombineGroups * kWave);
    if (upper) hipLaunchKernelGGL((symv_combine_kernel<T, true>), cgrid, cblock, 0, h->stream, a, pl.tile_cols, alpha, beta, y0, incy);
    else hipLaunchKernelGGL((symv_combine_kernel<T, false>), cgrid, cblock, 0, h->stream, a, pl.tile_cols, alpha, beta, y0, incy);
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
