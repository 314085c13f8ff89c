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
#include "skinny.hpp"
#include "trisweep.hpp"

namespace mxb {
namespace {

__device__ __forceinline__ int64_t imin(int64_t a, int64_t b) { return a < b ? a : b; }

constexpr int kThreads = 256;

// ---------------------------------------------------------------------------------------------
// ger

constexpr int64_t kMaxGerBlocks = 1 << 23;          // x 256 threads: below the 2^32 threads a launch may have
constexpr int64_t kGerWideRowBytes = 1 << 20;      // rows from this size on are updated one by one, as long vectors
constexpr int kGerWideRows = 4;                    // ... in groups of this many per block

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
    uint32_t col_tiles;    // blocks side by side along a row; the grid is col_tiles x row groups, flattened
};

// A vector that would run past column N is moved back so that it ends at N (the host makes sure
// that N >= VEC; element alignment is all a matrix access needs): its first `shift` elements are
// the neighbouring lane's columns, they are updated in registers like the rest and not stored.
template <typename T, int VEC>
__device__ __forceinline__ void st_matrix_from(T* p, typename VecOf<T, VEC>::type v, int shift)
{
    if (shift == 0) {
        st_matrix<T, VEC>(p, v);
    } else {
#pragma unroll
        for (int k = 1; k < VEC; ++k)
            if (k >= shift) p[k] = v[k];
    }
}

template <typename T, int VEC, bool KEEP>
__global__ void __launch_bounds__(kThreads) ger_kernel(const GerArgs<T> p)
{
    typedef typename VecOf<T, VEC>::type V;
    constexpr int U = 8;
    const int64_t bx = blockIdx.x % p.col_tiles, by = blockIdx.x / p.col_tiles;   // 32-bit division
    int64_t c = (bx * kThreads + threadIdx.x) * VEC;
    if (c >= p.N) return;
    const int shift = c + VEC > p.N ? (int)(c + VEC - p.N) : 0;
    c -= shift;
    T yj[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) yj[k] = p.y[(c + k) * p.incy];
    const int64_t rlo = by * p.rows_per_block, rhi = imin(p.M, rlo + p.rows_per_block);
    T* acol = p.A + c;
    int64_t i0 = rlo;
    for (; i0 + U <= rhi; i0 += U) {
        V a[U];
        T ax[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            a[u] = ld_matrix_as<T, VEC, KEEP>(acol + (i0 + u) * p.lda);
            ax[u] = p.alpha * p.x[(i0 + u) * p.incx];
        }
        __builtin_amdgcn_sched_barrier(0);   // all loads of the batch are in flight before the first store
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int k = 0; k < VEC; ++k) a[u][k] = fmad(ax[u], yj[k], a[u][k]);
            st_matrix_from<T, VEC>(acol + (i0 + u) * p.lda, a[u], shift);
        }
    }
    for (; i0 < rhi; ++i0) {
        V a = ld_matrix_as<T, VEC, KEEP>(acol + i0 * p.lda);
        const T ax = p.alpha * p.x[i0 * p.incx];
#pragma unroll
        for (int k = 0; k < VEC; ++k) a[k] = fmad(ax, yj[k], a[k]);
        st_matrix_from<T, VEC>(acol + i0 * p.lda, a, shift);
    }
}

// Rows of a megabyte and more: every row is updated like one long vector, A[i][:] += (alpha*x[i])*y,
// in the tiles of the streaming level-1 kernels (8 runs of 4 KiB that lie 64 KiB apart inside
// the row).  The tile of the kernel above stacks 8 rows, which lie a whole pitch apart: with a
// pitch of several megabytes, and worst a power of two, all 8 runs fall into the same memory
// channels (1024 x 4194304 floats: 51 % of peak at pitch 4194304, 73 % at pitch 4194304 + 1024).
// blockIdx.y = group of 4 rows (one tile of y in registers serves them all: a y that does not fit
// the caches would otherwise be fetched once per row), blockIdx.x = tile of the row; y has unit increment.
template <typename T>
__global__ void __launch_bounds__(kThreads) ger_wide_kernel(const GerArgs<T> p, int64_t row0, int64_t nvec, int64_t nfull, int64_t n2d,
                                                            int tail)
{
    constexpr int VEC = Full<T>::vec;
    constexpr int U = 8, R = kGerWideRows;
    typedef typename VecOf<T, VEC>::type V;
    typedef V LooseV __attribute__((aligned(sizeof(T))));
    const int64_t i0 = row0 + (int64_t)blockIdx.y * R;
    const int nr = (int)imin((int64_t)R, p.M - i0);
    for (int64_t t = blockIdx.x; t < nfull; t += gridDim.x) {
        int64_t base, step;
        stream_tile<U>(t, n2d, base, step);
        V b[U];
#pragma unroll
        for (int u = 0; u < U; ++u) b[u] = *reinterpret_cast<const LooseV*>(p.y + (base + u * step) * VEC);
        for (int r = 0; r < nr; ++r) {       // the tile of y serves R rows
            T* arow = p.A + (i0 + r) * p.lda;
            const T ax = p.alpha * p.x[(i0 + r) * p.incx];
            V a[U];
#pragma unroll
            for (int u = 0; u < U; ++u) a[u] = ld_matrix<T, VEC>(arow + (base + u * step) * VEC);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int k = 0; k < VEC; ++k) a[u][k] = fmad(ax, b[u][k], a[u][k]);
                st_matrix<T, VEC>(arow + (base + u * step) * VEC, a[u]);
            }
        }
    }
    if (blockIdx.x != gridDim.x - 1) return;
    for (int r = 0; r < nr; ++r) {
        T* arow = p.A + (i0 + r) * p.lda;
        const T ax = p.alpha * p.x[(i0 + r) * p.incx];
        for (int64_t v = nfull * (kThreads * U) + threadIdx.x; v < nvec; v += kThreads) {
            V a = ld_matrix<T, VEC>(arow + v * VEC);
#pragma unroll
            for (int k = 0; k < VEC; ++k) a[k] = fmad(ax, p.y[v * VEC + k], a[k]);
            st_matrix<T, VEC>(arow + v * VEC, a);
        }
        if ((int)threadIdx.x < tail) {
            const int64_t j = nvec * VEC + threadIdx.x;
            arow[j] = fmad(ax, p.y[j], arow[j]);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// syr / syr2: the same streaming read-modify-write restricted to the stored triangle

template <typename T>
struct SyrArgs {
    int64_t n;
    T* A;
    int64_t lda;
    const T* x;        // logical element 0
    int64_t incx;
    const T* y;        // syr2 only
    int64_t incy;
    T alpha;
    uint32_t ntiles;       // tiles of kThreads*VEC columns across the matrix
};

// One block: 8 adjacent rows x kThreads*VEC columns (a tile).  Only tiles that hold stored
// elements are launched: the rows are cut into bands of one tile width, band q holds q+1 tiles
// per batch of rows if lower (ntiles-q if upper), and bands q and ntiles-1-q are enumerated
// together, so that every batch index of a pair owns exactly ntiles+1 blocks and a block finds its
// tile with two 32-bit divisions.  Tiles wholly inside the triangle run the unpredicated ger code;
// in the tiles that straddle the diagonal every lane decides per row whether its vector lies
// inside (vector access), outside (nothing is loaded or stored) or across the diagonal (loaded
// whole, stored element by element).
template <typename T, int VEC, bool UPPER, bool TWO, bool KEEP>
__global__ void __launch_bounds__(kThreads) syr_kernel(const SyrArgs<T> p)
{
    typedef typename VecOf<T, VEC>::type V;
    constexpr int U = 8;
    constexpr uint32_t W = kThreads * VEC, BPB = W / U;     // tile width; batches of rows per band
    const uint32_t nt = p.ntiles, per_pair = (nt + 1) * BPB, pairs = nt / 2;
    uint32_t band, tile, batch;
    if (blockIdx.x < pairs * per_pair) {
        const uint32_t q = blockIdx.x / per_pair, rest = blockIdx.x % per_pair, j = rest % (nt + 1);
        batch = rest / (nt + 1);
        const uint32_t first = UPPER ? nt - q : q + 1;     // tiles of band q; the rest belong to band nt-1-q
        band = j < first ? q : nt - 1 - q;
        tile = UPPER ? band + (j < first ? j : j - first) : (j < first ? j : j - first);
    } else {                                               // the middle band of an odd number of bands
        const uint32_t rest = blockIdx.x - pairs * per_pair, m = pairs;
        band = m;
        batch = rest / (m + 1);
        tile = (UPPER ? m : 0) + rest % (m + 1);
    }
    const int64_t c0 = (int64_t)tile * W, r0 = (int64_t)band * W + (int64_t)batch * U;
    if (r0 >= p.n) return;                                  // the last band may be short
    const int64_t r1 = imin(p.n, r0 + U);   // exclusive
    int64_t c = c0 + (int64_t)threadIdx.x * VEC;
    const bool col_ok = c < p.n;
    // ragged last vector of a row: moved back to end at n, its first `shift` elements not stored
    const int shift = col_ok && c + VEC > p.n ? (int)(c + VEC - p.n) : 0;
    c -= shift;
    T xj[VEC], yj[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) {
        xj[k] = col_ok ? p.x[(c + k) * p.incx] : T(0);
        yj[k] = (TWO && col_ok) ? p.y[(c + k) * p.incy] : T(0);
    }
    T* acol = p.A + c;
    const bool inside = tile != band && r0 + U <= p.n && c0 + W <= p.n;
    V a[U];
    T ax[U], ay[U];
    if (inside) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            a[u] = ld_matrix_as<T, VEC, KEEP>(acol + (r0 + u) * p.lda);
            ax[u] = p.alpha * p.x[(r0 + u) * p.incx];
            ay[u] = TWO ? p.alpha * p.y[(r0 + u) * p.incy] : T(0);
        }
        __builtin_amdgcn_sched_barrier(0);   // all loads of the batch are in flight before the first store
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int k = 0; k < VEC; ++k) {
                if (TWO) a[u][k] = fmad(ax[u], yj[k], fmad(ay[u], xj[k], a[u][k]));
                else a[u][k] = fmad(ax[u], xj[k], a[u][k]);
            }
            st_matrix<T, VEC>(acol + (r0 + u) * p.lda, a[u]);
        }
        return;
    }
    if (!col_ok) return;
    // d = position of the diagonal inside the lane's vector in row i: element k is stored iff
    // k <= d (lower) / k >= d (upper)
    // (no load is predicated, so that all of them are in flight together: a lane whose vector lies
    // outside the triangle, or whose row is past the end, reads the vector that holds the diagonal
    // element of the last valid row instead and drops it; one conditional load per row had the
    // batch wait for each in turn, n = 256 .. 1024: 5.7 us per call against ger's 3)
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t i = imin(r0 + u, r1 - 1), d = i - c;
        const bool none = UPPER ? d > VEC - 1 : d < 0;
        a[u] = ld_matrix_as<T, VEC, KEEP>(p.A + i * p.lda + (none ? imin(i / VEC * VEC, p.n - VEC) : c));
        ax[u] = p.alpha * p.x[i * p.incx];
        ay[u] = TWO ? p.alpha * p.y[i * p.incy] : T(0);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t i = r0 + u, d = i - c;
        if (i >= r1) break;
        const bool all = UPPER ? d <= 0 : d >= VEC - 1;
        const bool none = UPPER ? d > VEC - 1 : d < 0;
        if (none) continue;
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            if (TWO) a[u][k] = fmad(ax[u], yj[k], fmad(ay[u], xj[k], a[u][k]));
            else a[u][k] = fmad(ax[u], xj[k], a[u][k]);
        }
        T* ap = acol + i * p.lda;
        if (all && shift == 0) {
            st_matrix<T, VEC>(ap, a[u]);
        } else {
#pragma unroll
            for (int k = 0; k < VEC; ++k)
                if (k >= shift && (UPPER ? k >= d : k <= d)) ap[k] = a[u][k];
        }
    }
}

// ---------------------------------------------------------------------------------------------
// symv of a small matrix in one kernel (no workspace, no second pass): a call on a few thousand
// unknowns is bound by launches and latency, not by bytes, so every stored element is read twice
// instead of once.  Block b owns the 16 unknowns I = [16b, 16b + 16) and forms both halves of
// their results itself:
//   row part     sum over the stored part of rows I (columns <= i if lower, >= i if upper): each
//                wavefront takes 4 rows, its lanes stride across the columns with 128-bit loads;
//   column part  sum over the stored part of columns I in the other rows (rows > j if lower,
//                < j if upper), i.e. the mirrored elements: 16 columns = CL lanes, 64 / CL rows
//                side by side per wavefront load, column sums in registers, folded through LDS.
// Every block reads about 16 n elements, whatever b is.  The order of all sums is fixed.
// (unknowns per block, measured per call: 8 / 16 / 32 at n = 256 4.1 / 3.7 / 4.0 us, 1024 5.0 / 4.8 / 6.0, 1536 5.8 / 5.4 / 7.2,
// 2048 9.1 / 7.6 / 8.5; double precision 1024 5.3 / 5.6 / 8.0, 1536 8.1 / 8.5 / 10.4)
constexpr int kSmallTile = 16;

template <typename T, int VEC, bool UPPER, int TILE>
__global__ void __launch_bounds__(kThreads) symv_small_kernel(int n, T alpha, const T* __restrict__ A, int64_t lda,
                                                              const T* __restrict__ x, int64_t incx, T beta, T* __restrict__ y,
                                                              int64_t incy)
{
    typedef typename VecOf<T, VEC>::type V;
    constexpr int NW = kThreads / kWave, RPW = TILE / NW;   // wavefronts; rows of the row part per wavefront
    constexpr int CL = TILE / VEC, RL = kWave / CL;         // column part: lanes per row, rows per wavefront load
    constexpr int UB = 4;                                         // column part: loads in flight per lane
    __shared__ T ya[TILE];
    __shared__ T red[NW][kWave][VEC];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int i0 = (int)blockIdx.x * TILE, i1 = min(n, i0 + TILE);

    // ---- row part: rows i0 + wave*RPW + u, columns [ca, cb)
    {
        const int ca = UPPER ? i0 / (kWave * VEC) * (kWave * VEC) : 0, cb = UPPER ? n : i1;
        T acc[RPW];
#pragma unroll
        for (int u = 0; u < RPW; ++u) acc[u] = T(0);
        for (int c0 = ca; c0 < cb; c0 += kWave * VEC) {
            const int c = c0 + lane * VEC;                 // my columns: [c, c + VEC)
            const int cl = min(c, n - VEC);                // a vector past the end is moved back into the row
            V a[RPW];
            T xv[VEC];
#pragma unroll
            for (int u = 0; u < RPW; ++u) a[u] = ld_resident<T, VEC>(A + (int64_t)min(i0 + wave * RPW + u, n - 1) * lda + cl);
#pragma unroll
            for (int k = 0; k < VEC; ++k) xv[k] = x[(int64_t)(cl + k) * incx];
#pragma unroll
            for (int u = 0; u < RPW; ++u) {
                const int i = i0 + wave * RPW + u;
#pragma unroll
                for (int k = 0; k < VEC; ++k) {
                    const int j = cl + k;
                    const bool use = j >= c && j < cb && (UPPER ? j >= i : j <= i);
                    acc[u] = use ? fmad(a[u][k], xv[k], acc[u]) : acc[u];
                }
            }
        }
#pragma unroll
        for (int u = 0; u < RPW; ++u) {
            const T s = wave_sum(acc[u]);
            if (lane == 0) ya[wave * RPW + u] = s;
        }
    }

    // ---- column part: columns i0 + [0, 32), rows [ra, rb) in groups of RL, the groups dealt to the wavefronts
    {
        const int ra = UPPER ? 0 : i0, rb = UPPER ? i1 : n;
        const int cq = lane % CL, rl = lane / CL;
        const int c = i0 + cq * VEC;                        // my columns: [c, c + VEC)
        const int cl = max(min(c, n - VEC), 0);
        T acc[VEC];
#pragma unroll
        for (int k = 0; k < VEC; ++k) acc[k] = T(0);
        for (int r0 = ra + wave * RL; r0 < rb; r0 += NW * RL * UB) {
            V a[UB];
            T xr[UB];
#pragma unroll
            for (int u = 0; u < UB; ++u) {
                const int r = min(r0 + u * NW * RL + rl, n - 1);
                a[u] = ld_resident<T, VEC>(A + (int64_t)r * lda + cl);
                xr[u] = x[(int64_t)r * incx];
            }
#pragma unroll
            for (int u = 0; u < UB; ++u) {
                const int r = r0 + u * NW * RL + rl;
#pragma unroll
                for (int k = 0; k < VEC; ++k) {
                    const int j = cl + k;
                    const bool use = j >= c && j < i1 && r < rb && (UPPER ? r < j : r > j);
                    acc[k] = use ? fmad(a[u][k], xr[u], acc[k]) : acc[k];
                }
            }
        }
#pragma unroll
        for (int k = 0; k < VEC; ++k) red[wave][lane][k] = acc[k];
    }
    __syncthreads();
    const int t = threadIdx.x;
    if (t < TILE && i0 + t < n) {
        // column i0 + t sits in element k of the vector of lanes cq + CL*rl (rl = 0..RL-1)
        const int cq = t / VEC, cl = max(min(i0 + cq * VEC, n - VEC), 0), k = i0 + t - cl;
        T s = ya[t];
        for (int w = 0; w < NW; ++w)
            for (int rl = 0; rl < RL; ++rl) s += red[w][cq + CL * rl][k];
        T* yp = y + (int64_t)(i0 + t) * incy;
        T v = alpha * s;
        if (beta != T(0)) v = fmad(beta, *yp, v);
        *yp = v;
    }
}

// ---------------------------------------------------------------------------------------------
// launchers


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
        hipLaunchKernelGGL(scale_y_kernel<T>, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, h->stream, n, beta, y0, incy, (int64_t)0);
        return launch_status();
    }
    if (!A) return -5;
    if (!x) return -7;
    // the column-major upper triangle occupies the bytes of the row-major lower triangle
    const bool upper = (uplo == MXB_UPPER) == (layout == MXB_ROW_MAJOR);
    const T* x0 = vec_base(x, n, incx);
    constexpr int FV = Full<T>::vec;
    // (in double precision a lane walks twice the rows: the sweep is ahead from two thirds of the limit on, n = 1536: 12 against 19 us)
    if (n >= FV && n <= option(h, MXB_OPT_SYMV_SMALL_MAX) * (sizeof(T) == 8 ? 2 : 3) / 3) {
        const dim3 grid((unsigned)ceil_div(n, (int64_t)kSmallTile));
        if (upper) hipLaunchKernelGGL((symv_small_kernel<T, FV, true, kSmallTile>), grid, dim3(kThreads), 0, h->stream, (int)n, alpha, A, lda, x0, incx, beta, y0, incy);
        else hipLaunchKernelGGL((symv_small_kernel<T, FV, false, kSmallTile>), grid, dim3(kThreads), 0, h->stream, (int)n, alpha, A, lda, x0, incx, beta, y0, incy);
        return launch_status();
    }
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
    if (layout == MXB_ROW_MAJOR) a = GerArgs<T>{m, n, A, lda, vec_base(x, m, incx), incx, vec_base(y, n, incy), incy, alpha, 0, 0};
    else a = GerArgs<T>{n, m, A, lda, vec_base(y, n, incy), incy, vec_base(x, m, incx), incx, alpha, 0, 0};
    if (skinny_takes(SKINNY_GER, a.M, a.N, a.A, a.lda))   // very short rows: several rows side by side per wavefront
        return skinny_ger<T>(h, a.M, a.N, alpha, a.x, a.incx, a.y, a.incy, a.A, a.lda);
    a.rows_per_block = option(h, MXB_OPT_GER_ROWS_PER_BLOCK);
    constexpr int FV = Full<T>::vec;
    if (a.incy == 1 && a.N * (int64_t)sizeof(T) >= kGerWideRowBytes) {      // very long rows: row by row, as long vectors
        const int64_t nvec = a.N / FV, nfull = nvec / (kThreads * 8);
        if (nfull <= 0x7fffffff) {
            constexpr int64_t kRowsPerLaunch = (int64_t)65535 * kGerWideRows;
            for (int64_t r0 = 0; r0 < a.M; r0 += kRowsPerLaunch) {
                const int64_t nr = ceil_div(a.M - r0 < kRowsPerLaunch ? a.M - r0 : kRowsPerLaunch, (int64_t)kGerWideRows);
                hipLaunchKernelGGL(ger_wide_kernel<T>, dim3((unsigned)nfull, (unsigned)nr), dim3(kThreads), 0, h->stream, a, r0, nvec, nfull,
                                   stream_tiles_2d(nvec, 8), (int)(a.N % FV));
                const int st = launch_status();
                if (st != MXB_OK) return st;
            }
            return MXB_OK;
        }
    }
    // Any pitch, any base address and any width of at least one vector: matrix accesses need element
    // alignment only and the kernel moves the last vector of a ragged row back.
    // (a short ragged row keeps more lanes busy with one element per lane)
    const bool vec = a.N % FV == 0 || a.N >= 2 * kWave;
    a.col_tiles = (uint32_t)ceil_div(a.N, (int64_t)kThreads * (vec ? FV : 1));
    // a launch cannot have 2^32 threads or more: a very tall matrix gets more rows per block
    while ((int64_t)a.col_tiles * ceil_div(a.M, a.rows_per_block) > kMaxGerBlocks) a.rows_per_block *= 2;
    const int64_t blocks = (int64_t)a.col_tiles * ceil_div(a.M, a.rows_per_block);
    const dim3 grid((unsigned)blocks);
    if (!vec) hipLaunchKernelGGL((ger_kernel<T, 1, false>), grid, dim3(kThreads), 0, h->stream, a);
    else if (keeps_update(a.M * a.N * (int64_t)sizeof(T))) hipLaunchKernelGGL((ger_kernel<T, FV, true>), grid, dim3(kThreads), 0, h->stream, a);
    else hipLaunchKernelGGL((ger_kernel<T, FV, false>), grid, dim3(kThreads), 0, h->stream, a);
    return launch_status();
}

// syr (y == nullptr) and syr2.  Both updates are symmetric, so the column-major uplo triangle is
// the row-major opposite triangle of the same bytes.
template <typename T, bool TWO>
int syr(mxb_handle_t h, int layout, int uplo, int64_t n, T alpha, const T* x, int64_t incx, const T* y, int64_t incy, T* A,
        int64_t lda)
{
    if (!handle_ok(h)) return MXB_ERR_HANDLE;
    if (!layout_ok(layout)) return -1;
    if (!uplo_ok(uplo)) return -2;
    if (n < 0) return -3;
    if (incx == 0) return -6;
    if (TWO && incy == 0) return -8;
    if (lda < (n > 1 ? n : 1)) return TWO ? -10 : -8;
    if (n == 0 || alpha == T(0)) return MXB_OK;
    if (!x) return -5;
    if (TWO && !y) return -7;
    if (!A) return TWO ? -9 : -7;
    const bool upper = (uplo == MXB_UPPER) == (layout == MXB_ROW_MAJOR);
    SyrArgs<T> a{n, A, lda, vec_base(x, n, incx), incx, TWO ? vec_base(y, n, incy) : nullptr, incy, alpha, 0};
    constexpr int FV = Full<T>::vec;
    // Any pitch, any base address and any n of at least one vector: matrix accesses need element
    // alignment only and the kernel moves the last vector of a ragged row back.
    const bool vec = n >= FV;
    const int64_t w = (int64_t)kThreads * (vec ? FV : 1), nt = ceil_div(n, w);
    a.ntiles = (uint32_t)nt;
    // pairs of bands with nt+1 tiles per batch of 8 rows, plus the middle band of an odd count
    const int64_t blocks = (nt / 2) * (nt + 1) * (w / 8) + (nt % 2) * (nt / 2 + 1) * (w / 8);
    if (blocks > 0x7fffffff) return MXB_ERR_NOT_IMPLEMENTED;
    const dim3 grid((unsigned)blocks);
#define MXB_SYR(VEC_, KEEP_)                                                                                        \
    if (upper) hipLaunchKernelGGL((syr_kernel<T, VEC_, true, TWO, KEEP_>), grid, dim3(kThreads), 0, h->stream, a);  \
    else hipLaunchKernelGGL((syr_kernel<T, VEC_, false, TWO, KEEP_>), grid, dim3(kThreads), 0, h->stream, a);
    if (!vec) { MXB_SYR(1, true) }        // narrower than one vector
    else if (keeps_matrix(n * (n + 1) / 2 * (int64_t)sizeof(T))) { MXB_SYR(FV, true) }
    else { MXB_SYR(FV, false) }
#undef MXB_SYR
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
int mxb_ssyr(mxb_handle_t h, mxb_layout_t layout, mxb_uplo_t uplo, int64_t n, float alpha, const float* x, int64_t incx, float* A,
             int64_t lda)
{ return mxb::syr<float, false>(h, layout, uplo, n, alpha, x, incx, nullptr, 1, A, lda); }
int mxb_dsyr(mxb_handle_t h, mxb_layout_t layout, mxb_uplo_t uplo, int64_t n, double alpha, const double* x, int64_t incx, double* A,
             int64_t lda)
{ return mxb::syr<double, false>(h, layout, uplo, n, alpha, x, incx, nullptr, 1, A, lda); }
int mxb_ssyr2(mxb_handle_t h, mxb_layout_t layout, mxb_uplo_t uplo, int64_t n, float alpha, const float* x, int64_t incx,
              const float* y, int64_t incy, float* A, int64_t lda)
{ return mxb::syr<float, true>(h, layout, uplo, n, alpha, x, incx, y, incy, A, lda); }
int mxb_dsyr2(mxb_handle_t h, mxb_layout_t layout, mxb_uplo_t uplo, int64_t n, double alpha, const double* x, int64_t incx,
              const double* y, int64_t incy, double* A, int64_t lda)
{ return mxb::syr<double, true>(h, layout, uplo, n, alpha, x, incx, y, incy, A, lda); }
}
