// Triangle sweep (Sec. 6.2.2, triangular and symmetric matrices): one pass over the stored
// triangle of a row-major matrix that produces column sums (transposed trmv) or row sums and
// column sums at once (symv), reading every stored element exactly once.
//
// The paper rounds triangular loop bounds to the vector width and predicates the edge; here the
// same idea works at tile granularity.  The triangle is cut into column tiles of TC columns.  A
// block of 8 wavefronts owns one tile for its whole life: a lane owns CV vectors of VEC adjacent
// columns and keeps their column sums in registers, and the block walks down the rows that have
// stored elements in the tile, taking batches of adjacent rows cyclically with the other blocks
// of the tile, so that the blocks of a tile read one compact, moving window of rows.  Tiles get
// blocks in proportion to their work.  Row sums (symv): the 8 or 16 sums of a batch are folded
// across the wavefront together (lane swaps and DPP, common.hpp) and written once per row and
// wavefront; column sums are written once, at the end.  A second
// kernel adds the partials in a fixed order (no atomics) and applies alpha/beta.
//
// Rows that lie wholly off the diagonal run without any mask.  In the TC rows of a tile that
// cross the diagonal every vector of a wavefront (64 lanes x VEC columns) is classified once per
// batch, wave-uniformly: wholly outside the triangle (skipped: no loads, no arithmetic), wholly
// inside (plain arithmetic), or straddling the diagonal (element-wise selects, never a
// multiplication by zero; a lane whose vector lies wholly outside redirects its load to the
// vector that holds the diagonal element, which its neighbours fetch anyway).  About half of the
// vectors are skipped there, so those batches take twice the rows.
#include "trisweep.hpp"

#include "options.hpp"

namespace mxb {

enum { TRI_SYMV = 0, TRI_TRMV_T = 1 };

struct TriArgs {
    int n, ntiles, tile_cols, blocks;
    int64_t lda, incx;
    int first_block[kTriMaxTiles + 1];   // blocks of tile t: [first_block[t], first_block[t+1])
};

namespace {

// One batch: U adjacent rows starting at rb (of the rows [.., r1) the caller walks), CV vectors per lane.
// Rows and columns are below 2^31, so index arithmetic is 32-bit; only addresses are 64-bit.
// In a masked batch every vector of the wavefront (64 lanes x VEC columns) is classified once,
// wave-uniformly: wholly outside the triangle for every row of the batch (skipped: no loads, no
// arithmetic), wholly and strictly inside (plain arithmetic), or straddling the diagonal or a
// ragged edge (element-wise selects).
// MODE: TRI_PLAIN, a whole tile and rows wholly off the diagonal, nothing is masked; TRI_MASKED, as
// above; TRI_EDGE, rows wholly off the diagonal in the ragged last tile: a vector is outside (past
// column n), inside, or straddles column n, and the lane's column is the same for every row.
enum { TRI_PLAIN = 0, TRI_MASKED = 1, TRI_EDGE = 2 };

template <typename T, int VEC, int CV, int U, bool UPPER, int KIND, bool UNIT, int MODE, bool RES>
__device__ __forceinline__ void tri_batch(const TriArgs& p, const T* __restrict__ A, const T* __restrict__ x, int rb, int r1, const int (&cfull)[CV],
                                          const int (&col)[CV], const int (&kmin)[CV], const bool (&col_ok)[CV], const T (&xj)[CV][VEC], T (&cacc)[CV][VEC],
                                          T* __restrict__ rowpart_wave, int lane)
{
    typedef typename VecOf<T, VEC>::type V;
    constexpr int WSPAN = kWave * VEC;          // columns one wavefront covers with one vector
    constexpr bool ROWS = KIND == TRI_SYMV;
    V a[U][CV];
    T xi[U];
    constexpr bool MASKED = MODE == TRI_MASKED, EDGE = MODE == TRI_EDGE;
    bool dead[CV], plain[CV];
#pragma unroll
    for (int v = 0; v < CV; ++v) {
        const int cw = __builtin_amdgcn_readfirstlane(cfull[v] - lane * VEC);       // first column of the wavefront's vector v
        dead[v] = (MASKED && (UPPER ? cw + WSPAN - 1 < rb : cw > rb + U - 1)) || (EDGE && cw >= p.n);
        plain[v] = MODE == TRI_PLAIN || (EDGE && cw + WSPAN <= p.n) ||
                   (MASKED && (UPPER ? cw > rb + U - 1 : cw + WSPAN - 1 < rb) && rb + U <= r1 && cw + WSPAN <= p.n);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        int i = rb + u;
        if (MASKED) i = min(i, r1 - 1);                      // clamp: the load stays inside the matrix
        const T* arow = A + (int64_t)i * p.lda;
#pragma unroll
        for (int v = 0; v < CV; ++v) {
            if (dead[v]) {
                a[u][v] = V(T(0));
            } else if (EDGE) {
                a[u][v] = ld_matrix_as<T, VEC, RES>(arow + min(col[v], p.n - VEC));   // lanes past the last column stay in bounds
            } else if (MASKED) {
                int cc = col[v];
                const int diag = i / VEC * VEC;              // vector that holds the diagonal element of row i
                // wholly outside the triangle: read that one instead (a vector moved back from the
                // ragged end is not on the vector grid and stays where it is)
                if (kmin[v] == 0) cc = UPPER ? max(cc, diag) : min(cc, diag);
                cc = min(cc, p.n - VEC);                     // lanes past the last column
                a[u][v] = ld_matrix_as<T, VEC, RES>(arow + cc);
            } else {
                a[u][v] = ld_matrix_as<T, VEC, RES>(arow + cfull[v]);
            }
        }
        xi[u] = x[(int64_t)i * p.incx];
    }
    __builtin_amdgcn_sched_barrier(0);   // keep every load of the batch ahead of the first FMA
    T rs[U];
#pragma unroll
    for (int u = 0; u < U; ++u) rs[u] = T(0);
#pragma unroll
    for (int v = 0; v < CV; ++v) {
        if (dead[v]) continue;
        if (plain[v]) {
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int k = 0; k < VEC; ++k) {
                    if (ROWS) rs[u] = fmad(a[u][v][k], xj[v][k], rs[u]);
                    cacc[v][k] = fmad(a[u][v][k], xi[u], cacc[v][k]);
                }
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = rb + u;
                // d = position of the diagonal inside this vector: element k lies strictly inside the
                // triangle iff k < d (lower) / k > d (upper) and on the diagonal iff k == d
                const int d = i - col[v];
                const bool live = (EDGE || i < r1) && col_ok[v];
#pragma unroll
                for (int k = 0; k < VEC; ++k) {
                    const T val = a[u][v][k];
                    const bool mine = live && k >= kmin[v];
                    // rows off the diagonal: every column below n is inside the triangle
                    const bool off = mine && (EDGE || (UPPER ? k > d : k < d));
                    const bool on = !EDGE && mine && k == d;
                    if (ROWS) {
                        // symv: the diagonal goes to the row sum only
                        rs[u] = (off || on) ? fmad(val, xj[v][k], rs[u]) : rs[u];
                        cacc[v][k] = off ? fmad(val, xi[u], cacc[v][k]) : cacc[v][k];
                    } else {
                        // trmv: the diagonal (1 if unit, and then never used) goes to the column sum
                        const T dv = UNIT ? T(1) : val;
                        cacc[v][k] = off ? fmad(val, xi[u], cacc[v][k]) : (on ? fmad(dv, xi[u], cacc[v][k]) : cacc[v][k]);
                    }
                }
            }
        }
    }
    if (ROWS) {
        // fold all rows of the batch over the wavefront at once; a lane ends up with one row's sum
        int mine;
        const bool writer = rows_fold_lane<U>(lane, mine);
        const T out = rows_fold<U>(rs, lane);
        const int i = rb + mine;
        if (writer && i < r1) rowpart_wave[i] = out;
    }
}

// x: logical element 0.  rowpart: [ntiles * 8 wavefronts][n] (symv).  colpart: [blocks][TC].
template <typename T, int VEC, int CV, int UB, bool UPPER, int KIND, bool UNIT>
__global__ void __launch_bounds__(kTriThreads) trisweep_kernel(const TriArgs p, const T* __restrict__ A, const T* __restrict__ x,
                                                               T* __restrict__ rowpart, T* __restrict__ colpart)
{
    typedef typename VecOf<T, VEC>::type V;
    constexpr int U = UB / CV, UD = 2 * U;   // rows per batch: off the diagonal / across it
    constexpr int SPAN = kTriThreads * VEC;
    constexpr int TC = CV * SPAN;
    constexpr bool ROWS = KIND == TRI_SYMV;
    // The short batches serve the triangles that fit the last-level cache: loads without the
    // streaming hint, so that the triangle stays there for the next call.
    constexpr bool RES = UB < 16;

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = p.n;
    const int g = blockIdx.x;

    // my tile, my index s among its S blocks
    int t = 0;
    while (t + 1 < p.ntiles && g >= p.first_block[t + 1]) ++t;
    const int s = g - p.first_block[t], S = p.first_block[t + 1] - p.first_block[t];
    const int cb0 = t * TC, cb1 = min(n, cb0 + TC);
    const bool full_tile = cb0 + TC <= n;
    int cfull[CV];       // first column of the lane's vector v, before a ragged end moves it back
#pragma unroll
    for (int v = 0; v < CV; ++v) cfull[v] = cb0 + ((v * kTriWaves + wave) * kWave + lane) * VEC;

    // col[v]: first column of the lane's vector v.  A vector that would run past column n is moved
    // back so that it ends at n (n >= VEC here; element alignment is all a matrix load needs); its
    // first kmin[v] elements are the neighbouring lane's columns and never count.
    int col[CV], kmin[CV];
    bool col_ok[CV];
    T xj[CV][VEC], cacc[CV][VEC];
#pragma unroll
    for (int v = 0; v < CV; ++v) {
        const int cv = cfull[v];
        col_ok[v] = cv < n;
        kmin[v] = (VEC > 1 && col_ok[v] && cv + VEC > n) ? cv + VEC - n : 0;
        col[v] = cv - kmin[v];
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            xj[v][k] = (ROWS && col_ok[v]) ? x[(int64_t)(col[v] + k) * p.incx] : T(0);
            cacc[v][k] = T(0);
        }
    }
    T* rowpart_wave = ROWS ? rowpart + ((int64_t)t * kTriWaves + wave) * n : nullptr;

    // Rows with stored elements in this tile, in ascending order: the rows that cross the
    // diagonal [cb0, cb1) and the rows wholly inside the triangle (below them if lower, above if
    // upper).  Each range is dealt in batches of adjacent rows cyclically to the S blocks.
    // Lower: down from the diagonal, so that all tiles reach the last rows together and the kernel
    // ends in unmasked batches that span whole matrix rows.  Upper mirrors that: the same batches
    // taken from the bottom of each range upwards, the diagonal first, so that all tiles reach row
    // 0 together (taken top-down it would end in the masked, half-empty batches on the diagonal:
    // transposed trmv 89.7 -> 86.0 us at n = 16384, symv 92.6 -> 91.1).
    const int f0 = UPPER ? 0 : cb1, f1 = UPPER ? cb0 : n;
    auto diagonal_rows = [&]() {
        const int64_t nb = ((int64_t)(cb1 - cb0) + UD - 1) / UD;
        for (int64_t k = s; k < nb; k += S) {
            const int64_t rb = cb0 + (UPPER ? nb - 1 - k : k) * UD;
            tri_batch<T, VEC, CV, UD, UPPER, KIND, UNIT, TRI_MASKED, RES>(p, A, x, (int)rb, cb1, cfull, col, kmin, col_ok, xj, cacc, rowpart_wave, lane);
        }
    };
    auto inside_rows = [&]() {
        const int64_t nb = ((int64_t)(f1 - f0) + U - 1) / U;
        for (int64_t k = s; k < nb; k += S) {
            const int rb = (int)(f0 + (UPPER ? nb - 1 - k : k) * U);
            if (rb + U > f1)
                tri_batch<T, VEC, CV, U, UPPER, KIND, UNIT, TRI_MASKED, RES>(p, A, x, rb, f1, cfull, col, kmin, col_ok, xj, cacc, rowpart_wave, lane);
            else if (full_tile)
                tri_batch<T, VEC, CV, U, UPPER, KIND, UNIT, TRI_PLAIN, RES>(p, A, x, rb, f1, cfull, col, kmin, col_ok, xj, cacc, rowpart_wave, lane);
            else
                tri_batch<T, VEC, CV, U, UPPER, KIND, UNIT, TRI_EDGE, RES>(p, A, x, rb, f1, cfull, col, kmin, col_ok, xj, cacc, rowpart_wave, lane);
        }
    };
    diagonal_rows();
    inside_rows();

    // column sums of this block over its tile
    T* slot = colpart + (int64_t)g * TC - cb0;
#pragma unroll
    for (int v = 0; v < CV; ++v) {
        if (kmin[v] == 0) {
            V val;
#pragma unroll
            for (int k = 0; k < VEC; ++k) val[k] = cacc[v][k];
            *reinterpret_cast<V*>(slot + col[v]) = val;
        } else {
#pragma unroll
            for (int k = 0; k < VEC; ++k)
                if (k >= kmin[v]) slot[col[v] + k] = cacc[v][k];
        }
    }
}

constexpr int kCombineGroups = 16;

// out[i] = alpha * (column partials of column i: every block of i's tile; then, for symv, the
//          row partials of row i: every tile with stored elements in row i, every wavefront)
//          + beta*out[i], each list in ascending order, folded over 16 wavefronts through LDS in
//          wave order.  (Four loads of a list in flight: 1.3 us less per call than one at a time.
//          A block of 16 columns x 64 groups, a quarter of the loads per lane in four times the
//          blocks, changes nothing: +-0.3 us up to n = 12000, 2 us slower at 16384.)
template <typename T, bool UPPER, int KIND>
__global__ void __launch_bounds__(kCombineGroups* kWave) trisweep_combine_kernel(const TriArgs p, const T* __restrict__ rowpart,
                                                                                 const T* __restrict__ colpart, T alpha, T beta,
                                                                                 T* __restrict__ out, int64_t inco)
{
    __shared__ T red[kCombineGroups][kWave];
    const int tx = threadIdx.x & (kWave - 1), ty = threadIdx.x >> 6;
    const int i = (int)blockIdx.x * kWave + tx;
    const int TC = p.tile_cols;
    T s = T(0);
    if (i < p.n) {
        const int t = i / TC;
        const T* base = colpart + (i - t * TC);
#pragma unroll 4
        for (int g = p.first_block[t] + ty; g < p.first_block[t + 1]; g += kCombineGroups) s += base[(int64_t)g * TC];
        if (KIND == TRI_SYMV) {
            const int q0 = UPPER ? t : 0, q1 = UPPER ? p.ntiles : t + 1;
#pragma unroll 4
            for (int e = q0 * kTriWaves + ty; e < q1 * kTriWaves; e += kCombineGroups) s += rowpart[(int64_t)e * p.n + i];
        }
    }
    red[ty][tx] = s;
    __syncthreads();
    if (ty != 0 || i >= p.n) return;
    T tot = red[0][tx];
#pragma unroll
    for (int k = 1; k < kCombineGroups; ++k) tot += red[k][tx];
    T* op = out + (int64_t)i * inco;
    T v = alpha * tot;
    if (beta != T(0)) v = fmad(beta, *op, v);
    *op = v;
}

template <typename T, int VEC, int CV, int UB, int KIND>
void launch_sweep(mxb_handle_t h, bool upper, bool unit, const TriArgs& a, const T* A, const T* x, T* rowpart, T* colpart)
{
    const dim3 grid((unsigned)a.blocks), block(kTriThreads);
#define MXB_TRI(UP_, KIND_, UNIT_) \
    hipLaunchKernelGGL((trisweep_kernel<T, VEC, CV, UB, UP_, KIND_, UNIT_>), grid, block, 0, h->stream, a, A, x, rowpart, colpart)
    if (KIND == TRI_SYMV) {
        if (upper) MXB_TRI(true, TRI_SYMV, false); else MXB_TRI(false, TRI_SYMV, false);
    } else if (upper) {
        if (unit) MXB_TRI(true, TRI_TRMV_T, true); else MXB_TRI(true, TRI_TRMV_T, false);
    } else {
        if (unit) MXB_TRI(false, TRI_TRMV_T, true); else MXB_TRI(false, TRI_TRMV_T, false);
    }
#undef MXB_TRI
}

template <typename T, int KIND>
int trisweep(mxb_handle_t h, bool upper, bool unit, int64_t n, T alpha, const T* A, int64_t lda, const T* x0, int64_t incx, T beta,
             T* out, int64_t inco)
{
    constexpr int FV = Full<T>::vec;
    if (n > 0x7fffffff - 65536) return MXB_ERR_NOT_IMPLEMENTED;
    // Any pitch, any base address and any n of at least one vector: matrix loads need element
    // alignment only and the kernel moves the last vector of a ragged row back.
    const bool vec = n >= FV;
    const TriPlan pl = tri_plan(n, vec ? FV : 1, (int)sizeof(T), upper, h->opt[MXB_OPT_SYMV_TARGET_BLOCKS],
                                h->opt[MXB_OPT_SYMV_TILE_VECTORS], option(h, MXB_OPT_TRI_DIAG_WEIGHT));
    if (!pl.ok) return MXB_ERR_NOT_IMPLEMENTED;
    const size_t need = tri_workspace_elems(n, pl, KIND == TRI_SYMV) * sizeof(T);
    T* rowpart = static_cast<T*>(take_workspace(h, need));
    if (!rowpart) return MXB_ERR_WORKSPACE;
    TriArgs a;
    a.n = (int)n; a.ntiles = pl.ntiles; a.tile_cols = pl.tile_cols; a.blocks = pl.blocks;
    a.lda = lda; a.incx = incx;
    for (int t = 0; t <= kTriMaxTiles; ++t) a.first_block[t] = pl.first_block[t <= pl.ntiles ? t : pl.ntiles];
    T* colpart = rowpart + (KIND == TRI_SYMV ? (int64_t)pl.ntiles * kTriWaves * n : 0);
    if (!vec) launch_sweep<T, 1, 1, 4, KIND>(h, upper, unit, a, A, x0, rowpart, colpart);
    else if (pl.cv == 4) launch_sweep<T, FV, 4, 16, KIND>(h, upper, unit, a, A, x0, rowpart, colpart);
    else if (pl.cv == 2) launch_sweep<T, FV, 2, 16, KIND>(h, upper, unit, a, A, x0, rowpart, colpart);
    else if (pl.ub == 16) launch_sweep<T, FV, 1, 16, KIND>(h, upper, unit, a, A, x0, rowpart, colpart);
    else if (pl.ub == 8) launch_sweep<T, FV, 1, 8, KIND>(h, upper, unit, a, A, x0, rowpart, colpart);
    else launch_sweep<T, FV, 1, 4, KIND>(h, upper, unit, a, A, x0, rowpart, colpart);
    const int st = launch_status();
    if (st != MXB_OK) return st;
    const dim3 cgrid((unsigned)ceil_div(n, kWave)), cblock(kCombineGroups * kWave);
    if (upper)
        hipLaunchKernelGGL((trisweep_combine_kernel<T, true, KIND>), cgrid, cblock, 0, h->stream, a, rowpart, colpart, alpha, beta, out, inco);
    else
        hipLaunchKernelGGL((trisweep_combine_kernel<T, false, KIND>), cgrid, cblock, 0, h->stream, a, rowpart, colpart, alpha, beta, out, inco);
    return launch_status();
}

}  // namespace

template <typename T>
int trisweep_symv(mxb_handle_t h, bool upper, int64_t n, T alpha, const T* A, int64_t lda, const T* x0, int64_t incx, T beta,
                  T* y0, int64_t incy)
{
    return trisweep<T, TRI_SYMV>(h, upper, false, n, alpha, A, lda, x0, incx, beta, y0, incy);
}

template <typename T>
int trisweep_trmv_t(mxb_handle_t h, bool upper, bool unit, int64_t n, const T* A, int64_t lda, T* x0, int64_t incx)
{
    return trisweep<T, TRI_TRMV_T>(h, upper, unit, n, T(1), A, lda, x0, incx, T(0), x0, incx);
}

template int trisweep_symv<float>(mxb_handle_t, bool, int64_t, float, const float*, int64_t, const float*, int64_t, float, float*, int64_t);
template int trisweep_symv<double>(mxb_handle_t, bool, int64_t, double, const double*, int64_t, const double*, int64_t, double, double*,
                                   int64_t);
template int trisweep_trmv_t<float>(mxb_handle_t, bool, bool, int64_t, const float*, int64_t, float*, int64_t);
template int trisweep_trmv_t<double>(mxb_handle_t, bool, bool, int64_t, const double*, int64_t, double*, int64_t);

}  // namespace mxb
