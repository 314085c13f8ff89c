// gemv and trmv (Sec. 6.2.2) on a row-major matrix.
//
// Two kernels cover gemv and trmv in both orientations, and the off-diagonal part of trsv (trsv.hip):
//
//  * row-dot (no transpose; Sec. 2: y[i] += A[i,j]*x[j]).  The paper batches r rows so that each
//    x[j] is loaded once for all of them (unroll-and-jam).  Here a group of LPR lanes walks R
//    rows at once with 128-bit loads of A; x is staged in LDS once per block and chunk and read
//    from there by every row of the tile; the R sums are folded across the lane group with DPP
//    and written with one store per wavefront.
//
//  * column-accumulate (transpose; Fig. 7c: y[j] += x[i]*A[i,j]).  Every lane owns VEC adjacent
//    columns and keeps their sums in registers while the block walks down a slab of rows; x[i]
//    is wave-uniform and comes through the scalar path.  Slabs are combined by a second kernel
//    that adds the per-slab partial vectors in slab order and applies alpha/beta (no atomics).
//
// trmv without transposition runs the row-dot kernel with MODE = upper/lower: the column range
// of every tile is clipped to the triangle at tile granularity (the paper's bound rounding) and
// the elements of a straddling 128-bit load that lie outside the triangle are discarded with a
// select, never by multiplying with zero, so that NaN/Inf stored there cannot leak into the
// result.  Transposed trmv is the triangle sweep of trisweep.hip.
#include "matvec.hpp"

#include <mutex>

#include "options.hpp"
#include "plan.hpp"
#include "skinny.hpp"
#include "tiny.hpp"
#include "trisweep.hpp"

namespace mxb {
namespace {


__device__ __forceinline__ int64_t imin(int64_t a, int64_t b) { return a < b ? a : b; }
__device__ __forceinline__ int64_t imax(int64_t a, int64_t b) { return a > b ? a : b; }

// Value that matrix element (i, j), loaded as `a`, contributes in a triangular mode.
template <typename T, int MODE, bool UNIT>
__device__ __forceinline__ T tri_value(T a, int64_t i, int64_t j)
{
    if constexpr (MODE == MODE_GENERAL) return a;
    const bool inside = MODE == MODE_UPPER ? j >= i : j <= i;
    a = inside ? a : T(0);
    if constexpr (UNIT) a = (i == j) ? T(1) : a;
    return a;
}

// ---------------------------------------------------------------------------------------------
// row-dot


constexpr int kRowdotWaves = 8;
constexpr int kRowdotThreads = kRowdotWaves * kWave;

// One batch of the row-dot inner loop: U column steps of R rows, all loads issued before the FMAs.
template <typename T, int VEC, int R, int U, int STEP, int MODE, bool UNIT>
__device__ __forceinline__ void rowdot_batch(const T* const (&arow)[R], const T* xs_at_c, int64_t c, int64_t grow0, T (&acc)[R])
{
    typedef typename VecOf<T, VEC>::type V;
    V av[U][R], xv[U];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int r = 0; r < R; ++r) av[u][r] = ld_matrix<T, VEC>(arow[r] + c + u * STEP);
#pragma unroll
    for (int u = 0; u < U; ++u) xv[u] = *reinterpret_cast<const V*>(xs_at_c + u * STEP);
    __builtin_amdgcn_sched_barrier(0);   // keep every load of the batch ahead of the first FMA
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int k = 0; k < VEC; ++k)
                acc[r] = fmad(tri_value<T, MODE, UNIT>(av[u][r][k], grow0 + r, c + u * STEP + k), xv[u][k], acc[r]);
}

template <typename T, int VEC, int LPR, int R, int U, int MODE, bool UNIT>
__global__ void __launch_bounds__(kRowdotThreads, 4) rowdot_kernel(const RowdotArgs<T> p)
{
    constexpr int FV = Full<T>::vec;
    typedef typename VecOf<T, FV>::type XV;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    T* xs = reinterpret_cast<T*>(smem_raw);

    constexpr int GPW = kWave / LPR;          // lane groups (= concurrent rows) per wavefront
    constexpr int RW = GPW * R;               // rows per wavefront tile
    constexpr int RB = kRowdotWaves * RW;     // rows per block tile
    constexpr int STEP = LPR * VEC;           // columns a lane group covers per load
    constexpr int SUPER = U * STEP;           // columns per batch of U loads

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane / LPR, l = lane % LPR;
    const int64_t ntiles = (p.M + RB - 1) / RB;
    const int64_t Nv = p.N - p.N % VEC;       // columns that whole vectors cover
    const int64_t xc = p.xchunk;
    const int64_t total = ntiles * p.batch;   // tiles of all problems, one problem after the other
    int64_t staged = -1, staged_b = -1;

    for (int64_t pass = 0; pass * gridDim.x < total; ++pass) {
        // Triangular modes: rows get shorter (upper) or longer (lower) down the matrix, so the
        // passes alternate direction: the block that took the heaviest tile of one pass takes the
        // lightest of the next and every block ends up with about the same number of elements.
        const int64_t slot = (MODE != MODE_GENERAL && (pass & 1)) ? (int64_t)gridDim.x - 1 - blockIdx.x : blockIdx.x;
        int64_t t = pass * gridDim.x + slot;
        if (t >= total) continue;
        int64_t b = 0;
        if (p.batch > 1) { b = t / ntiles; t -= b * ntiles; }
        const T* __restrict__ A = p.A + b * p.sA;
        const T* __restrict__ x = p.x + b * p.sx;
        T* __restrict__ y = p.y + b * p.sy;
        const int64_t tile = MODE == MODE_LOWER ? ntiles - 1 - t : t;
        const int64_t brow0 = tile * RB;
        const int64_t wrow0 = brow0 + (int64_t)wave * RW;
        const int64_t grow0 = wrow0 + g * R;

        // column range the block / the wavefront has to visit
        int64_t bclo = 0, bchi = p.N, wclo = 0, wchi = Nv;
        if (MODE == MODE_UPPER) { bclo = imin(brow0, p.N); wclo = wrow0; }
        if (MODE == MODE_LOWER) { bchi = imin(p.N, brow0 + RB); wchi = imin(Nv, wrow0 + RW); }

        const T* arow[R];
#pragma unroll
        for (int r = 0; r < R; ++r) arow[r] = A + imin(grow0 + r, p.M - 1) * p.lda;   // clamp: loads stay in bounds
        T acc[R];
#pragma unroll
        for (int r = 0; r < R; ++r) acc[r] = T(0);

        for (int64_t c0 = bclo / xc * xc; c0 < bchi; c0 += xc) {
            const int64_t c1 = imin(c0 + xc, p.N);
            if (c0 != staged || b != staged_b) {
                __syncthreads();
                const int cnt = (int)(c1 - c0);
                if (p.x_contig) {
                    const XV* src = reinterpret_cast<const XV*>(x + c0);
                    XV* dst = reinterpret_cast<XV*>(xs);
                    const int nv = cnt / FV;
#pragma unroll 4
                    for (int j = threadIdx.x; j < nv; j += kRowdotThreads) dst[j] = src[j];
                    for (int j = nv * FV + threadIdx.x; j < cnt; j += kRowdotThreads) xs[j] = x[c0 + j];
                } else {
#pragma unroll 4
                    for (int j = threadIdx.x; j < cnt; j += kRowdotThreads) xs[j] = x[(c0 + j) * p.incx];
                }
                __syncthreads();
                staged = c0;
                staged_b = b;
            }
            const int64_t lo = imax(wclo, c0), hi = imin(wchi, imin(c0 + xc, Nv));
            if (lo < hi) {
                // Whole batches first.  Every wavefront starts at a different batch and wraps
                // around, so that the wavefronts that run side by side are not all pulling the
                // same column range (= the same HBM channels) of their rows at once.
                const int64_t base = c0 + (lo - c0) / STEP * STEP;
                const int64_t nfull = (hi - base) / SUPER;
                if (nfull > 0) {
                    int64_t s = ((tile * kRowdotWaves + wave) * 3) % nfull;
                    for (int64_t k = 0; k < nfull; ++k) {
                        const int64_t cw = base + s * SUPER;     // first column of the batch (wave-uniform)
                        const int64_t c = cw + l * VEC;
                        s = s + 1 == nfull ? 0 : s + 1;
                        // a batch that lies wholly inside the triangle for every row of the wavefront needs no masks
                        const bool inside = MODE == MODE_GENERAL || (MODE == MODE_UPPER ? cw > wrow0 + RW - 1 : cw + SUPER <= wrow0);
                        if (inside) rowdot_batch<T, VEC, R, U, STEP, MODE_GENERAL, false>(arow, xs + (c - c0), c, grow0, acc);
                        else rowdot_batch<T, VEC, R, U, STEP, MODE, UNIT>(arow, xs + (c - c0), c, grow0, acc);
                    }
                }
                for (int64_t c = base + nfull * SUPER + l * VEC; c < hi; c += STEP)
                    rowdot_batch<T, VEC, R, 1, STEP, MODE, UNIT>(arow, xs + (c - c0), c, grow0, acc);
            }
        }
        // columns past the last whole vector (N not a multiple of VEC): one lane each
        if (VEC > 1 && Nv < p.N) {
            const int64_t j = Nv + l;
            const bool visit = MODE == MODE_LOWER ? wrow0 + RW > Nv : true;
            if (visit && j < p.N) {
                const T xj = x[j * p.incx];
#pragma unroll
                for (int r = 0; r < R; ++r)
                    acc[r] = fmad(tri_value<T, MODE, UNIT>(arow[r][j], grow0 + r, j), xj, acc[r]);
            }
        }

        // fold the lane group, then lane r of the group stores row r
        T out = T(0);
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const T s = lanes_sum<LPR>(acc[r]);
            out = (l == r) ? s : out;
        }
        const int64_t i = grow0 + l;
        if (l < R && i < p.M) {
            T* yp = y + i * p.incy;
            T v = p.alpha * out;
            if (p.beta != T(0)) v = fmad(p.beta, *yp, v);
            *yp = v;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// row-dot for a matrix that comes from the caches

// A product this small is bound by launches and latency, not by bytes: the persistent row-dot
// grid gives a 1024 x 1024 matrix 128 blocks, each of which first stages x in LDS behind two
// barriers.  Here a wavefront takes R rows from end to end on its own: x comes straight from
// the second-level cache (a few KiB that every wavefront reads), up to U loads of 16 bytes per
// row are in flight per lane, no LDS, no barrier, two wavefronts per block so that a matrix of
// 1024 rows already makes 512 blocks.
constexpr int kRowSmallThreads = 128;

// WC == 1: the block's two wavefronts take R rows each.  WC > 1 (few, long rows): the block's WC
// wavefronts share one row, batch b of its columns goes to wavefront b % WC, LDS folds them in
// wave order.
// MODE upper / lower (trmv): a wavefront's columns start at the vector that holds the diagonal
// of its first row, resp. end with the one of its last row, and what a load brings from outside
// the triangle is discarded by a select.
// BATCH: the rows of all problems of a batch as one list (problems of fewer rows than a tile of the
// persistent grid, which that grid would fill to a sixteenth and re-stage x for).
template <typename T, int VEC, int R, int U, int WC, int MODE = MODE_GENERAL, bool UNIT = false, bool BATCH = false>
__global__ void __launch_bounds__(WC == 1 ? kRowSmallThreads : WC * kWave) rowsmall_kernel(const RowdotArgs<T> pin)
{
    static_assert(!BATCH || (R == 1 && WC == 1 && MODE == MODE_GENERAL), "batched: one row per wavefront");
    RowdotArgs<T> p = pin;
    if (BATCH) {
        const int64_t id = (int64_t)blockIdx.x * (kRowSmallThreads / kWave) + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        if (id >= pin.M * pin.batch) return;
        const int64_t b = id / pin.M, r = id - b * pin.M;
        p.A = pin.A + b * pin.sA + r * pin.lda;
        p.x = pin.x + b * pin.sx;
        p.y = pin.y + b * pin.sy + r * pin.incy;
        p.M = 1;                               // my row is row 0 of what p now describes
    }
    typedef typename VecOf<T, VEC>::type V;
    static_assert(WC == 1 || R == 1, "wavefronts that share a row take one row");
    static_assert(WC == 1 || MODE == MODE_GENERAL, "triangular rows are not shared");
    constexpr int SPANV = kWave * VEC;             // columns a wavefront covers with one load
    __shared__ T part[WC];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // (the rows of a lower triangle grow towards the end: the last blocks first, so that the long rows start early)
    const int64_t blk = MODE == MODE_LOWER ? (int64_t)gridDim.x - 1 - blockIdx.x : (int64_t)blockIdx.x;
    const int64_t row0 = BATCH ? 0 : (WC == 1 ? (blk * (kRowSmallThreads / kWave) + wave) * R : blk);
    if (row0 >= p.M) return;
    const T* arow[R];
#pragma unroll
    for (int r = 0; r < R; ++r) arow[r] = p.A + imin(row0 + r, p.M - 1) * p.lda;      // clamp: loads stay in bounds
    T acc[R];
#pragma unroll
    for (int r = 0; r < R; ++r) acc[r] = T(0);
    // Batches of U loads per row, all in flight before the first use and none predicated: a vector
    // that would start past column N, or run past it, is moved back to end at N (N >= VEC), and
    // the elements that are not its own (a neighbour's, or all of them) meet a zero of x.
    const int64_t cbeg = MODE == MODE_UPPER ? row0 / VEC * VEC : 0, cend = MODE == MODE_LOWER ? imin(p.N, row0 + R) : p.N;
    for (int64_t c0 = cbeg + (int64_t)lane * VEC + (WC == 1 ? 0 : wave * (SPANV * U)); c0 - lane * VEC < cend; c0 += (int64_t)SPANV * U * WC) {
        V a[U][R], xv[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t cu = c0 + u * SPANV, c = imin(cu, p.N - VEC);
#pragma unroll
            for (int r = 0; r < R; ++r) a[u][r] = ld_resident<T, VEC>(arow[r] + c);
            if (p.incx == 1) {
                xv[u] = *reinterpret_cast<const V __attribute__((aligned(sizeof(T))))*>(p.x + c);
            } else {
#pragma unroll
                for (int k = 0; k < VEC; ++k) xv[u][k] = p.x[(c + k) * p.incx];
            }
#pragma unroll
            for (int k = 0; k < VEC; ++k) xv[u][k] = (c + k >= cu && cu < p.N) ? xv[u][k] : T(0);
        }
        __builtin_amdgcn_sched_barrier(0);   // keep every load of the batch ahead of the first FMA
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int k = 0; k < VEC; ++k) {
                    const int64_t j = imin(c0 + u * SPANV, p.N - VEC) + k;
                    acc[r] = fmad(tri_value<T, MODE, UNIT>(a[u][r][k], row0 + r, j), xv[u][k], acc[r]);
                }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
        T s = wave_sum(acc[r]);
        if (WC > 1) {
            if (lane == 0) part[wave] = s;
            __syncthreads();
            if (wave != 0) return;
            s = part[0];
#pragma unroll
            for (int w = 1; w < WC; ++w) s += part[w];
        }
        const int64_t i = row0 + r;
        if (lane == 0 && i < p.M) {
            T* yp = p.y + i * p.incy;
            T v = p.alpha * s;
            if (p.beta != T(0)) v = fmad(p.beta, *yp, v);
            *yp = v;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// column-accumulate


constexpr int kColaccThreads = 256;

// Two shapes:
//  WR == 1 (wide matrices): the 4 wavefronts of a block sit side by side and every lane owns CV
//    vectors of VEC adjacent columns, 256*VEC columns apart, so that a block reads runs of
//    CV*4 KiB from each row.  Rows are taken in batches of U adjacent rows and the batches are
//    dealt to the gridDim.y row groups cyclically: at any moment the whole grid is reading one
//    narrow band of adjacent rows, i.e. the matrix is swept front to back like a single
//    sequential stream, which is what HBM serves fastest.
//  WR == 4 (narrow matrices, CV == 1): one wavefront spans the row, the 4 wavefronts of a block
//    interleave over the rows of a contiguous slab and are folded through LDS.
template <typename T, int VEC, int CV, int WR, bool KEEP>
__global__ void __launch_bounds__(kColaccThreads) colacc_kernel(const ColaccArgs<T> p)
{
    const T* __restrict__ A = p.A + (int64_t)blockIdx.z * p.sA;
    const T* __restrict__ x = p.x + (int64_t)blockIdx.z * p.sx;
    T* __restrict__ y = p.y + (int64_t)blockIdx.z * p.sy;
    T* __restrict__ partials = p.partials + (int64_t)blockIdx.z * p.spart;
    typedef typename VecOf<T, VEC>::type V;
    static_assert(WR == 1 || CV == 1, "narrow shape has one vector per lane");
    constexpr int NW = kColaccThreads / kWave, WC = NW / WR;
    constexpr int U = 16 / CV > 8 ? 8 : 16 / CV;          // rows in flight: 16 loads per lane (8 when CV == 1)
    constexpr int SPAN = WC * kWave * VEC;                // columns one vector index covers across the block
    __shared__ T red[WR > 1 ? (WR - 1) * WC * kWave * VEC : 1];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wc = wave % WC, wr = wave / WC;
    const int64_t cblock0 = (int64_t)blockIdx.x * (CV * SPAN);
    const int64_t c = cblock0 + (int64_t)(wc * kWave + lane) * VEC;
    // A vector that would run past column N is moved back so that it ends at N (the host makes sure
    // that N >= VEC; element alignment is all a matrix load needs): its first `shift` elements are
    // the neighbouring lane's columns and are dropped when the sums are written.
    bool col_ok[CV];
    int shift[CV];
#pragma unroll
    for (int v = 0; v < CV; ++v) {
        const int64_t cv = c + v * SPAN;
        col_ok[v] = cv < p.N;
        shift[v] = (VEC > 1 && col_ok[v] && cv + VEC > p.N) ? (int)(cv + VEC - p.N) : 0;
    }

    // Rows are visited in batches of U: rows r0 + u*rstep (u < U), then r0 += radvance.
    int64_t r0, rstep, radvance, rend = p.M;
    if (WR == 1) {
        // wide shape: batch = U adjacent rows; the batches are dealt to the row groups cyclically
        rstep = 1;
        radvance = (int64_t)gridDim.y * U;
        r0 = (int64_t)blockIdx.y * U;
    } else {
        // narrow shape: a contiguous slab per block, its rows interleaved over the 4 wavefronts
        int64_t rlo = (int64_t)blockIdx.y * p.rows_per_block;
        rend = imin(rend, rlo + p.rows_per_block);
        rstep = WR;
        radvance = (int64_t)U * WR;
        r0 = rlo + wr;
    }

    T acc[CV][VEC];
#pragma unroll
    for (int v = 0; v < CV; ++v)
#pragma unroll
        for (int k = 0; k < VEC; ++k) acc[v][k] = T(0);

    // Lanes past the last column load the block's first vector instead (in bounds, never stored),
    // so that the loads below carry no predicate and can all be issued back to back.
    const T* acol[CV];
#pragma unroll
    for (int v = 0; v < CV; ++v) acol[v] = A + (col_ok[v] ? c + v * SPAN - shift[v] : imin(cblock0, p.N - VEC));
    for (; r0 + (int64_t)(U - 1) * rstep < rend; r0 += radvance) {
        V a[U][CV];
        T xi[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = r0 + (int64_t)u * rstep;
#pragma unroll
            for (int v = 0; v < CV; ++v) a[u][v] = ld_matrix_as<T, VEC, KEEP>(acol[v] + i * p.lda);
            xi[u] = x[i * p.incx];
        }
        __builtin_amdgcn_sched_barrier(0);   // keep every load of the batch ahead of the first FMA
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int v = 0; v < CV; ++v)
#pragma unroll
                for (int k = 0; k < VEC; ++k)
                    acc[v][k] = fmad(a[u][v][k], xi[u], acc[v][k]);
    }
    for (; r0 < rend; r0 += rstep) {   // the one ragged batch
        const T xi = x[r0 * p.incx];
#pragma unroll
        for (int v = 0; v < CV; ++v) {
            const V a = ld_matrix_as<T, VEC, KEEP>(acol[v] + r0 * p.lda);
#pragma unroll
            for (int k = 0; k < VEC; ++k) acc[v][k] = fmad(a[k], xi, acc[v][k]);
        }
    }

    if (WR > 1) {   // fold the wavefronts that split the rows, in wave order
        T* mine = red + ((int64_t)((wr - 1) * WC + wc) * kWave + lane) * VEC;
        if (wr > 0)
#pragma unroll
            for (int k = 0; k < VEC; ++k) mine[k] = acc[0][k];
        __syncthreads();
        if (wr > 0) return;
#pragma unroll
        for (int w = 1; w < WR; ++w)
#pragma unroll
            for (int k = 0; k < VEC; ++k) acc[0][k] += red[((int64_t)((w - 1) * WC + wc) * kWave + lane) * VEC + k];
    }

#pragma unroll
    for (int v = 0; v < CV; ++v) {
        if (!col_ok[v]) continue;
        const int64_t cv = c + v * SPAN - shift[v];      // column of element 0 of the vector
        if (gridDim.y == 1) {
#pragma unroll
            for (int k = 0; k < VEC; ++k) {
                if (k < shift[v]) continue;
                T* yp = y + (cv + k) * p.incy;
                T val = p.alpha * acc[v][k];
                if (p.beta != T(0)) val = fmad(p.beta, *yp, val);
                *yp = val;
            }
        } else if (shift[v] == 0) {
            V val;
#pragma unroll
            for (int k = 0; k < VEC; ++k) val[k] = acc[v][k];
            *reinterpret_cast<V*>(partials + (int64_t)blockIdx.y * p.ppitch + cv) = val;
        } else {
#pragma unroll
            for (int k = 0; k < VEC; ++k)
                if (k >= shift[v]) partials[(int64_t)blockIdx.y * p.ppitch + cv + k] = acc[v][k];
        }
    }
}

// ---------------------------------------------------------------------------------------------
// few long rows, not transposed

constexpr int kFewThreads = 256;

// A*x for at most MR rows of any length: the result is a handful of dot products that share x.
// The columns are dealt to the blocks in tiles of U runs of 256 vectors; a lane keeps its vector
// of x and the matching vector of every row in flight, so x is read once whatever the number of
// rows, and sums one partial result per row.  Block b writes its M sums to partials[b][0..M);
// the pass that combines partial vectors adds them in block order.
template <typename T, int VEC, int MR, bool KEEP>
__global__ void __launch_bounds__(kFewThreads) fewrows_kernel(int M, int64_t N, const T* __restrict__ A, int64_t lda,
                                                              const T* __restrict__ x, int64_t incx, T* __restrict__ partials)
{
    typedef typename VecOf<T, VEC>::type V;
    constexpr int U = MR <= 2 ? 8 : (MR <= 4 ? 4 : (MR <= 8 ? 2 : 1));   // 16 to 33 loads in flight per lane
    constexpr int NW = kFewThreads / kWave;
    __shared__ T red[NW][MR];
    const int64_t nvec = N / VEC, tile = (int64_t)kFewThreads * U, nfull = nvec / tile;
    T acc[MR];
#pragma unroll
    for (int i = 0; i < MR; ++i) acc[i] = T(0);

    auto load_x = [&](int64_t v) -> V {
        if (incx == 1) return ld_matrix_as<T, VEC, KEEP>(x + v * VEC);
        V r;
#pragma unroll
        for (int k = 0; k < VEC; ++k) r[k] = x[(v * VEC + k) * incx];
        return r;
    };
    for (int64_t t = blockIdx.x; t < nfull; t += gridDim.x) {
        const int64_t v0 = t * tile + threadIdx.x;
        V xv[U], a[U][MR];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            xv[u] = load_x(v0 + u * kFewThreads);
            // one pointer walks down the rows, its step hidden from the compiler, which would
            // otherwise keep every row's offset in scalar registers and spill them
            const T* at = A + (v0 + u * kFewThreads) * VEC;
#pragma unroll
            for (int i = 0; i < MR; ++i)
                if (i < M) {                                                         // wave-uniform
                    a[u][i] = ld_matrix_as<T, VEC, KEEP>(at);
                    int64_t step = lda;
                    asm volatile("" : "+s"(step));
                    at += step;
                }
        }
        __builtin_amdgcn_sched_barrier(0);   // every load of the tile is in flight before the first FMA
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int i = 0; i < MR; ++i)
                if (i < M)
#pragma unroll
                    for (int k = 0; k < VEC; ++k) acc[i] = fmad(a[u][i][k], xv[u][k], acc[i]);
    }
    // the vectors after the last whole tile go to the block whose turn it is; the elements after
    // the last whole vector to that block's first lane
    if ((int64_t)blockIdx.x == nfull % gridDim.x) {
        for (int64_t v = nfull * tile + threadIdx.x; v < nvec; v += kFewThreads) {
            const V xv = load_x(v);
            const T* at = A + v * VEC;
#pragma unroll
            for (int i = 0; i < MR; ++i)
                if (i < M) {
                    const V a = ld_matrix_as<T, VEC, KEEP>(at);
#pragma unroll
                    for (int k = 0; k < VEC; ++k) acc[i] = fmad(a[k], xv[k], acc[i]);
                    int64_t step = lda;
                    asm volatile("" : "+s"(step));
                    at += step;
                }
        }
        if (threadIdx.x == 0)
            for (int64_t j = nvec * VEC; j < N; ++j) {
                const T xj = x[j * incx];
                const T* at = A + j;
#pragma unroll
                for (int i = 0; i < MR; ++i)
                    if (i < M) {
                        acc[i] = fmad(*at, xj, acc[i]);
                        int64_t step = lda;
                        asm volatile("" : "+s"(step));
                        at += step;
                    }
            }
    }
    const int wave = threadIdx.x >> 6;
#pragma unroll
    for (int i = 0; i < MR; ++i) {
        const T w = wave_sum(acc[i]);
        if ((threadIdx.x & (kWave - 1)) == 0) red[wave][i] = w;
    }
    __syncthreads();
    if ((int)threadIdx.x < M) {
        T tot = red[0][threadIdx.x];
#pragma unroll
        for (int w = 1; w < NW; ++w) tot += red[w][threadIdx.x];
        partials[(int64_t)blockIdx.x * M + threadIdx.x] = tot;
    }
}

// The transposed product for at most MR rows: y = alpha * sum_i x[i] * row i + beta * y, a stream
// over the columns.  A lane keeps the matching vector of every row in flight for U vectors of y
// (tiles of U runs of 256 vectors, one or a few tiles per block), x[i] in registers; no partial
// results.
template <typename T, int VEC, int MR, bool BETA, bool KEEP>
__global__ void __launch_bounds__(kFewThreads) fewrows_t_kernel(int M, int64_t N, const T* __restrict__ A, int64_t lda,
                                                                const T* __restrict__ x, int64_t incx, T alpha, T beta,
                                                                T* __restrict__ y, int64_t incy)
{
    typedef typename VecOf<T, VEC>::type V;
    constexpr int U = MR <= 2 ? 8 : (MR <= 4 ? 4 : (MR <= 8 ? 2 : 1));
    const int64_t nvec = N / VEC, tile = (int64_t)kFewThreads * U, nfull = nvec / tile;
    T xr[MR];
#pragma unroll
    for (int i = 0; i < MR; ++i) xr[i] = i < M ? x[i * incx] : T(0);

    auto load_y = [&](int64_t v) -> V {
        if (incy == 1) return ld_matrix_as<T, VEC, KEEP>(y + v * VEC);
        V r;
#pragma unroll
        for (int k = 0; k < VEC; ++k) r[k] = y[(v * VEC + k) * incy];
        return r;
    };
    auto finish = [&](int64_t v, V acc, V yo) {
        V out;
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            out[k] = alpha * acc[k];
            if (BETA) out[k] = fmad(beta, yo[k], out[k]);
        }
        if (incy == 1) st_matrix<T, VEC>(y + v * VEC, out);
        else
#pragma unroll
            for (int k = 0; k < VEC; ++k) y[(v * VEC + k) * incy] = out[k];
    };
    for (int64_t t = blockIdx.x; t < nfull; t += gridDim.x) {
        const int64_t v0 = t * tile + threadIdx.x;
        V a[U][MR], yo[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int i = 0; i < MR; ++i)
                if (i < M) a[u][i] = ld_matrix_as<T, VEC, KEEP>(A + i * lda + (v0 + u * kFewThreads) * VEC);     // wave-uniform
            if (BETA) yo[u] = load_y(v0 + u * kFewThreads);
        }
        __builtin_amdgcn_sched_barrier(0);   // every load of the tile is in flight before the first FMA
#pragma unroll
        for (int u = 0; u < U; ++u) {
            V acc = V(T(0));
#pragma unroll
            for (int i = 0; i < MR; ++i)
                if (i < M)
#pragma unroll
                    for (int k = 0; k < VEC; ++k) acc[k] = fmad(a[u][i][k], xr[i], acc[k]);
            finish(v0 + u * kFewThreads, acc, yo[u]);
        }
    }
    // the vectors after the last whole tile go to the block whose turn it is; the elements after
    // the last whole vector to that block's first lane
    if ((int64_t)blockIdx.x == nfull % gridDim.x) {
        for (int64_t v = nfull * tile + threadIdx.x; v < nvec; v += kFewThreads) {
            V acc = V(T(0)), yo = V(T(0));
            if (BETA) yo = load_y(v);
#pragma unroll
            for (int i = 0; i < MR; ++i)
                if (i < M) {
                    const V a = ld_matrix_as<T, VEC, KEEP>(A + i * lda + v * VEC);
#pragma unroll
                    for (int k = 0; k < VEC; ++k) acc[k] = fmad(a[k], xr[i], acc[k]);
                }
            finish(v, acc, yo);
        }
        if (threadIdx.x == 0)
            for (int64_t j = nvec * VEC; j < N; ++j) {
                T acc = T(0);
#pragma unroll
                for (int i = 0; i < MR; ++i)
                    if (i < M) acc = fmad(A[i * lda + j], xr[i], acc);
                T out = alpha * acc;
                if (BETA) out = fmad(beta, y[j * incy], out);
                y[j * incy] = out;
            }
    }
}

constexpr int kCombineGroups = 16;
constexpr int64_t kMaxCombineBlocks = 1 << 21;      // x 1024 threads: below the 2^32 threads a launch may have

// y[j] = alpha * sum_p partials[p][j] + beta*y[j], p ascending.  64 columns per block; the 16
// wavefronts of the block each take every 16th slab, LDS folds them in wave order.
template <typename T>
__global__ void __launch_bounds__(kCombineGroups* kWave) colacc_combine_kernel(int64_t nparts, int64_t N, int64_t ppitch,
                                                                               const T* __restrict__ partials, T alpha, T beta,
                                                                               T* __restrict__ y, int64_t incy, int64_t spart,
                                                                               int64_t sy)
{
    partials += (int64_t)blockIdx.y * spart;   // blockIdx.y: problem of a batch
    y += (int64_t)blockIdx.y * sy;
    __shared__ T red[kCombineGroups][kWave];
    const int tx = threadIdx.x & (kWave - 1), ty = threadIdx.x >> 6;
    // (a loop: the grid is capped, a launch cannot have 2^32 threads or more)
    for (int64_t jb = blockIdx.x; jb * kWave < N; jb += gridDim.x) {
        const int64_t j = jb * kWave + tx;
        T s = T(0);
        if (j < N) {
#pragma unroll 4
            for (int64_t q = ty; q < nparts; q += kCombineGroups) s += partials[q * ppitch + j];
        }
        red[ty][tx] = s;
        __syncthreads();
        if (ty == 0 && j < N) {
            T tot = red[0][tx];
#pragma unroll
            for (int k = 1; k < kCombineGroups; ++k) tot += red[k][tx];
            T* yp = y + j * incy;
            T v = alpha * tot;
            if (beta != T(0)) v = fmad(beta, *yp, v);
            *yp = v;
        }
        __syncthreads();
    }
}

// dense copy of a strided vector (trmv's snapshot of x)
template <typename T>
__global__ void __launch_bounds__(256) gather_kernel(int64_t n, const T* __restrict__ x, int64_t incx, T* __restrict__ dst)
{
    const int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (k < n) dst[k] = x[k * incx];
}

// ---------------------------------------------------------------------------------------------
// launchers

template <typename T, int VEC, int LPR, int R, int U, int MODE, bool UNIT>
void launch_rowdot_inst(mxb_handle_t h, const RowdotArgs<T>& a)
{
    constexpr int RB = kRowdotWaves * (kWave / LPR) * R;
    const int64_t ntiles = ceil_div(a.M, RB) * a.batch;
    const int64_t cap = kCUs * option(h, MXB_OPT_ROWDOT_BLOCKS_PER_CU);
    const int64_t grid = ntiles < cap ? ntiles : cap;
    const size_t lds = (size_t)a.xchunk * sizeof(T);
    hipLaunchKernelGGL((rowdot_kernel<T, VEC, LPR, R, U, MODE, UNIT>), dim3((unsigned)grid), dim3(kRowdotThreads), lds, h->stream, a);
}

template <typename T, int VEC, int MODE, bool UNIT>
void launch_rowdot_shape(mxb_handle_t h, const RowdotArgs<T>& a)
{
    // R x U = rows x column steps a lane group keeps in flight (8 loads of 16 bytes per lane).
    //  * narrow rows (up to 16 vectors): 16 lanes per row, four rows side by side per wavefront;
    //  * long rows: 2 rows x 4 steps, so that a wavefront reads 4 KiB runs of each row;
    //  * few rows: one row per wavefront so that the grid still fills the device.
    const int64_t allrows = a.M * a.batch;   // rows of all problems of a batch
    if (MODE == MODE_GENERAL && a.N <= 16 * 16 * VEC) {
        if (allrows >= (int64_t)kCUs * kRowdotWaves * 4 * 4) launch_rowdot_inst<T, VEC, 16, 4, 2, MODE_GENERAL, false>(h, a);
        else launch_rowdot_inst<T, VEC, 16, 1, 2, MODE_GENERAL, false>(h, a);
    } else if (allrows >= (int64_t)kCUs * kRowdotWaves * 2) {
        launch_rowdot_inst<T, VEC, 64, 2, 4, MODE, UNIT>(h, a);
    } else {
        launch_rowdot_inst<T, VEC, 64, 1, 4, MODE, UNIT>(h, a);
    }
}

}  // namespace

template <typename T>
int launch_rowdot(mxb_handle_t h, RowdotArgs<T> a, int mode, bool unit)
{
    constexpr int FV = Full<T>::vec;
    const int64_t max_chunk = (int64_t)(64 * 1024 / sizeof(T));
    int64_t xc = option(h, MXB_OPT_ROWDOT_XCHUNK);
    const int64_t ncols = ceil_div(a.N, 256) * 256;
    if (xc > ncols) xc = ncols;
    if (xc > max_chunk) xc = max_chunk;
    xc = ceil_div(xc, 256) * 256;
    a.xchunk = (int)xc;
    a.x_contig = a.incx == 1 && aligned16(a.x);
#define MXB_ROWDOT(VEC_)                                                                                   \
    switch (mode) {                                                                                        \
        case MODE_GENERAL: launch_rowdot_shape<T, VEC_, MODE_GENERAL, false>(h, a); break;                  \
        case MODE_UPPER:                                                                                   \
            if (unit) launch_rowdot_shape<T, VEC_, MODE_UPPER, true>(h, a);                                 \
            else launch_rowdot_shape<T, VEC_, MODE_UPPER, false>(h, a);                                     \
            break;                                                                                         \
        default:                                                                                           \
            if (unit) launch_rowdot_shape<T, VEC_, MODE_LOWER, true>(h, a);                                 \
            else launch_rowdot_shape<T, VEC_, MODE_LOWER, false>(h, a);                                     \
    }
    MXB_ROWDOT(FV)   // rows may start at any element: the loads need element alignment only, and the kernel
                     // takes the columns past the last whole vector one by one
#undef MXB_ROWDOT
    return launch_status();
}

namespace {

// y = alpha*A^t*x + beta*y for a matrix small enough to come from the caches, in one kernel and
// without partial vectors: a block owns 8 vectors of columns (32 in single precision) and all
// the rows; its 256 lanes are 8 column lanes x 32 row lanes, a lane walks down every 32nd row
// with 8 loads in flight, the 32 row lanes of a column are folded through LDS in a fixed order.
// The general kernel gives a block at least 1024 columns, which for such a matrix leaves a
// handful of blocks or forces many row groups whose partial vectors weigh as much as the matrix.
constexpr int kSmallUnroll = 8;

// CL column lanes (CL vectors of columns per block) x RL row lanes; a lane walks down every RL-th
// row.  The RL partial sums of a column are folded through LDS in two fixed stages: groups of
// RL / 8 adjacent row lanes first, then the 8 group sums.
// MODE upper / lower (transposed trmv): a block's rows end with, resp. start at, the rows that
// cross the diagonal in its columns, and what a load brings from outside the triangle is
// discarded by a select.
template <typename T, int VEC, int CL, int RL, int MODE = MODE_GENERAL, bool UNIT = false>
__global__ void __launch_bounds__(CL* RL) colsum_small_kernel(const ColaccArgs<T> p)
{
    typedef typename VecOf<T, VEC>::type V;
    constexpr int U = kSmallUnroll, W = CL * VEC, G = 8, PER = RL / G;
    static_assert(RL % G == 0 && CL * RL >= G * W, "two-stage fold");
    __shared__ T red[RL][W + 1];
    __shared__ T red2[G][W + 1];
    const int cl = threadIdx.x % CL, rl = threadIdx.x / CL;
    // my vector of columns; the last vector of a ragged width is moved back to end at the last
    // column and its first `shift` elements, which the lane before it owns, are dropped at the end
    auto place = [&](int lane_c, int64_t& c, int& shift) {
        c = (int64_t)blockIdx.x * W + lane_c * VEC;
        shift = 0;
        if (c >= p.N) return false;
        if (c + VEC > p.N) {
            shift = (int)(c + VEC - p.N);
            c = p.N - VEC;
        }
        return true;
    };
    int64_t c;
    int shift;
    const bool live = place(cl, c, shift);
    if (!live) c = 0;
    const T* col = p.A + c;
    V acc = V(T(0));
    const int64_t rbeg = MODE == MODE_LOWER ? imin((int64_t)blockIdx.x * W, p.M) : 0;
    const int64_t rend = MODE == MODE_UPPER ? imin(p.M, (int64_t)(blockIdx.x + 1) * W) : p.M;
    for (int64_t r0 = rbeg + rl; r0 < rend; r0 += (int64_t)RL * U) {
        V a[U];
        T xr[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {        // rows past the end: the last row again, times zero
            const int64_t r = r0 + (int64_t)u * RL;
            const int64_t rc = r < rend ? r : rend - 1;
            a[u] = ld_resident<T, VEC>(col + rc * p.lda);
            xr[u] = r < rend ? p.x[rc * p.incx] : T(0);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int k = 0; k < VEC; ++k) {
                const int64_t r = r0 + (int64_t)u * RL;
                acc[k] = fmad(tri_value<T, MODE, UNIT>(a[u][k], r < rend ? r : rend - 1, c + k), xr[u], acc[k]);
            }
    }
#pragma unroll
    for (int k = 0; k < VEC; ++k) red[rl][cl * VEC + k] = acc[k];
    __syncthreads();
    if (threadIdx.x < G * W) {
        const int g = threadIdx.x / W, w = threadIdx.x % W;
        T tot = T(0);
#pragma unroll
        for (int q = 0; q < PER; ++q) tot += red[g * PER + q][w];
        red2[g][w] = tot;
    }
    __syncthreads();
    if (threadIdx.x < W) {
        const int lane_c = threadIdx.x / VEC, k = threadIdx.x % VEC;
        int64_t c2;
        int shift2;
        if (place(lane_c, c2, shift2) && k >= shift2) {
            T tot = T(0);
#pragma unroll
            for (int g = 0; g < G; ++g) tot += red2[g][threadIdx.x];
            T* out = p.y + (c2 + k) * p.incy;
            *out = p.beta == T(0) ? p.alpha * tot : fmad(p.alpha, tot, p.beta * *out);
        }
    }
}

// Shape of the kernel above for an M x N matrix, as column lanes * 100 + row lanes: row lanes so
// that a lane has one or two rounds of loads (per call in a replayed graph, 8 x 32 / 8 x 64 /
// 4 x 128 / 8 x 128 lanes: 256^2 2.7 / 2.8 / 3.1 / 3.2 us, 512^2 3.3 / 2.9 / 3.2 / 3.4, 1024^2 4.4 /
// 3.6 / 3.3 / 3.5, 1536^2 5.6 / 4.3 / 3.9 / 4.6, 2048^2 6.8 / 5.0 / 6.5 / 4.8; the general kernels:
// 4.5, 6.1, 6.3, 6.6, 8.1).  From 2049 rows on the general kernels win (2500^2: 8.8 against 9.7 us at
// best, 4096 x 2048: 8.9 against 9.9, 8192 x 512: 7.0 against 11.9; 4096 x 512 is the exception, 6.6
// against 4.9).
// 0: not taken.
constexpr int64_t kSmallMaxRows = 2048;
template <typename T>
int colsum_small_shape(mxb_handle_t h, int64_t M, int64_t N)
{
    constexpr int FV = Full<T>::vec;
    if (N < FV || M > kSmallMaxRows || M * N * (int64_t)sizeof(T) > option(h, MXB_OPT_GEMVT_SMALL_MAX)) return 0;
    return M <= 256 ? 832 : (M <= 512 ? 864 : (M <= 1536 ? 428 : 928));
}

template <typename T, int VEC, int CL, int RL, int MODE = MODE_GENERAL, bool UNIT = false>
void launch_colsum_small(mxb_handle_t h, const ColaccArgs<T>& a)
{
    hipLaunchKernelGGL((colsum_small_kernel<T, VEC, CL, RL, MODE, UNIT>), dim3((unsigned)ceil_div(a.N, (int64_t)CL * VEC)), dim3(CL * RL), 0, h->stream, a);
}

template <typename T, int VEC>
void launch_colacc_inst(mxb_handle_t h, const ColaccArgs<T>& a, const ColaccPlan& pl, int64_t batch)
{
    const dim3 grid((unsigned)pl.col_tiles, (unsigned)pl.nparts, (unsigned)batch);
    const dim3 block(kColaccThreads);
#define MXB_COLACC(KEEP_)                                                                                       \
    if (pl.wr == 4) hipLaunchKernelGGL((colacc_kernel<T, VEC, 1, 4, KEEP_>), grid, block, 0, h->stream, a);         \
    else if (pl.cv == 4) hipLaunchKernelGGL((colacc_kernel<T, VEC, 4, 1, KEEP_>), grid, block, 0, h->stream, a);    \
    else if (pl.cv == 2) hipLaunchKernelGGL((colacc_kernel<T, VEC, 2, 1, KEEP_>), grid, block, 0, h->stream, a);    \
    else hipLaunchKernelGGL((colacc_kernel<T, VEC, 1, 1, KEEP_>), grid, block, 0, h->stream, a)
    if (keeps_matrix(batch * a.M * a.N * (int64_t)sizeof(T))) { MXB_COLACC(true); } else { MXB_COLACC(false); }
#undef MXB_COLACC
}

constexpr int64_t kMaxGridZ = 65535;
constexpr int64_t kRowSmallOneRow = 2048;      // up to here a wavefront takes one row, beyond two
constexpr int64_t kRowSmallBatchRows = 32;     // batched problems of up to this many rows: the rows of all problems as one list

}  // namespace

// `batch` problems of one shape (a.sA, a.sx, a.sy apart); the blocks the plan aims at are shared
// among them, so that a large batch of small matrices runs one block per column tile and problem
// and needs neither partial vectors nor the second kernel.
template <typename T>
int launch_colacc(mxb_handle_t h, ColaccArgs<T> a, int64_t batch)
{
    constexpr int FV = Full<T>::vec;
    // Any pitch, any base address and any width of at least one vector: matrix loads need element
    // alignment only and the kernel moves the last vector of a ragged row back.
    // (a ragged row of up to 64 elements keeps more lanes busy with one element per lane)
    const bool vec = a.N % FV == 0 || a.N > kWave;
    if (batch == 1) {
        switch (colsum_small_shape<T>(h, a.M, a.N)) {
            case 832: launch_colsum_small<T, FV, 8, 32>(h, a); return launch_status();
            case 864: launch_colsum_small<T, FV, 8, 64>(h, a); return launch_status();
            case 428: launch_colsum_small<T, FV, 4, 128>(h, a); return launch_status();
            case 928: launch_colsum_small<T, FV, 8, 128>(h, a); return launch_status();
            default: break;
        }
    }
    auto share = [&](int64_t blocks) { return blocks / batch > 1 ? blocks / batch : 1; };
    const ColaccPlan pl = colacc_plan(a.M, a.N, (int)sizeof(T), vec ? FV : 1, share(option(h, MXB_OPT_COLACC_TARGET_BLOCKS)),
                                      share(colacc_narrow_target(h)), option(h, MXB_OPT_COLACC_MIN_ROWS));
    a.rows_per_block = pl.rows_per_block;
    a.partials = nullptr;
    a.ppitch = ceil_div(a.N, FV) * FV;
    a.spart = pl.nparts * a.ppitch;
    if (pl.nparts > 1) {
        a.partials = static_cast<T*>(take_workspace(h, (size_t)batch * (size_t)a.spart * sizeof(T)));
        if (!a.partials) return MXB_ERR_WORKSPACE;
    }
    for (int64_t b0 = 0; b0 < batch; b0 += kMaxGridZ) {       // the grid's z extent is limited
        const int64_t nb = batch - b0 < kMaxGridZ ? batch - b0 : kMaxGridZ;
        ColaccArgs<T> c = a;
        c.A += b0 * a.sA; c.x += b0 * a.sx; c.y += b0 * a.sy;
        if (c.partials) c.partials += b0 * a.spart;
        if (vec) launch_colacc_inst<T, FV>(h, c, pl, nb);
        else launch_colacc_inst<T, 1>(h, c, pl, nb);
        int st = launch_status();
        if (st != MXB_OK) return st;
        if (pl.nparts == 1) continue;
        hipLaunchKernelGGL(colacc_combine_kernel<T>, dim3((unsigned)(ceil_div(a.N, kWave) < kMaxCombineBlocks ? ceil_div(a.N, kWave) : kMaxCombineBlocks), (unsigned)nb),
                           dim3(kCombineGroups * kWave),
                           0, h->stream, pl.nparts, a.N, a.ppitch, c.partials, a.alpha, a.beta, c.y, a.incy, a.spart, a.sy);
        st = launch_status();
        if (st != MXB_OK) return st;
    }
    return MXB_OK;
}


template int launch_rowdot<float>(mxb_handle_t, RowdotArgs<float>, int, bool);
template int launch_rowdot<double>(mxb_handle_t, RowdotArgs<double>, int, bool);
template int launch_colacc<float>(mxb_handle_t, ColaccArgs<float>, int64_t);
template int launch_colacc<double>(mxb_handle_t, ColaccArgs<double>, int64_t);

namespace {

// gemv on a row-major rows x cols matrix, arguments validated, x0 / y0 at logical element 0;
// `batch` problems of this shape lie sA, sx, sy elements apart.
template <typename T>
int gemv_rows(mxb_handle_t h, bool no_trans, int64_t rows, int64_t cols, T alpha, const T* A, int64_t lda, int64_t sA, const T* x0,
              int64_t incx, int64_t sx, T beta, T* y0, int64_t incy, int64_t sy, int64_t batch)
{
    const int64_t leny = no_trans ? rows : cols;
    if (alpha == T(0)) {
        for (int64_t b0 = 0; b0 < batch; b0 += kMaxGridZ) {
            const int64_t nb = batch - b0 < kMaxGridZ ? batch - b0 : kMaxGridZ;
            hipLaunchKernelGGL(scale_y_kernel<T>, dim3((unsigned)ceil_div(leny, 256), (unsigned)nb), dim3(256), 0, h->stream, leny,
                               beta, y0 + b0 * sy, incy, sy);
            const int st = launch_status();
            if (st != MXB_OK) return st;
        }
        return MXB_OK;
    }
    if (batch == 1) {
        // very short rows: several rows side by side per wavefront
        if (no_trans && skinny_takes(SKINNY_GEMV_N, rows, cols, A, lda))
            return skinny_gemv_n<T>(h, rows, cols, alpha, A, lda, x0, incx, beta, y0, incy);
        if (!no_trans && skinny_takes(SKINNY_GEMV_T, rows, cols, A, lda))
            return skinny_gemv_t<T>(h, rows, cols, alpha, A, lda, x0, incx, beta, y0, incy);
    }
    // a batch of matrices with very short rows: the rows of all problems as one list
    if (tiny_takes<T>(no_trans, rows, cols, batch))
        return no_trans ? tiny_gemv_n<T>(h, rows, cols, alpha, A, lda, sA, x0, incx, sx, beta, y0, incy, sy, batch)
                        : tiny_gemv_t<T>(h, rows, cols, alpha, A, lda, sA, x0, incx, sx, beta, y0, incy, sy, batch);
    if (no_trans && batch == 1 && cols >= kWideMinCols && (rows <= kFewRows || (rows <= kFewMaxRows && cols >= kFewManyMinCols))) {
        // A handful of very long rows: dot products that share x, one partial result per row and block.
        constexpr int FV = Full<T>::vec;
        const int mr = rows <= 1 ? 1 : (rows <= 2 ? 2 : (rows <= 4 ? 4 : (rows <= 8 ? 8 : (rows <= 16 ? 16 : 32))));
        const int u = mr <= 2 ? 8 : (mr <= 4 ? 4 : (mr <= 8 ? 2 : 1));          // as in the kernel
        const int64_t tiles = cols / FV / ((int64_t)kFewThreads * u);
        const int64_t cap = mr >= 16 ? kFewBlocks / 2 : kFewBlocks;     // 16 rows and more: one block per compute unit (measured)
        const int64_t grid = tiles < 1 ? 1 : (tiles < cap ? tiles : cap);
        T* partials = static_cast<T*>(take_workspace(h, (size_t)grid * (size_t)rows * sizeof(T)));
        if (!partials) return MXB_ERR_WORKSPACE;
        const bool keep = keeps_matrix((rows + 1) * cols * (int64_t)sizeof(T));
#define MXB_FEW(MR_)                                                                                                          \
    if (keep)                                                                                                                 \
        hipLaunchKernelGGL((fewrows_kernel<T, FV, MR_, true>), dim3((unsigned)grid), dim3(kFewThreads), 0, h->stream, (int)rows, cols, A, lda, \
                           x0, incx, partials);                                                                               \
    else                                                                                                                      \
        hipLaunchKernelGGL((fewrows_kernel<T, FV, MR_, false>), dim3((unsigned)grid), dim3(kFewThreads), 0, h->stream, (int)rows, cols, A, lda, \
                           x0, incx, partials)
        switch (mr) {
            case 1: MXB_FEW(1); break;
            case 2: MXB_FEW(2); break;
            case 4: MXB_FEW(4); break;
            case 8: MXB_FEW(8); break;
            case 16: MXB_FEW(16); break;
            default: MXB_FEW(32); break;
        }
#undef MXB_FEW
        const int st = launch_status();
        if (st != MXB_OK) return st;
        hipLaunchKernelGGL(colacc_combine_kernel<T>, dim3(1u, 1u), dim3(kCombineGroups * kWave), 0, h->stream, grid, rows, rows, partials,
                           alpha, beta, y0, incy, (int64_t)0, (int64_t)0);
        return launch_status();
    }
    if (!no_trans && batch == 1 && cols >= kFewStreamMinCols &&
        (rows <= kFewStreamRows || (rows <= 2 * kFewStreamRows && rows * cols * (int64_t)sizeof(T) <= kFewStreamManyMaxBytes))) {
        // The transposed product of a handful of very long rows: a stream over the columns.
        constexpr int FV = Full<T>::vec;
        const int mr = rows <= 1 ? 1 : (rows <= 2 ? 2 : (rows <= 4 ? 4 : (rows <= 8 ? 8 : 16)));
        const int u = mr <= 2 ? 8 : (mr <= 4 ? 4 : (mr <= 8 ? 2 : 1));           // as in the kernel
        const int64_t tiles = cols / FV / ((int64_t)kFewThreads * u);
        const int64_t grid = tiles < 1 ? 1 : (tiles < kFewStreamBlocks ? tiles : kFewStreamBlocks);
#define MXB_FEW_T2(MR_, BETA_)                                                                                               \
    if (keep)                                                                                                                \
        hipLaunchKernelGGL((fewrows_t_kernel<T, FV, MR_, BETA_, true>), dim3((unsigned)grid), dim3(kFewThreads), 0, h->stream, (int)rows, \
                           cols, A, lda, x0, incx, alpha, beta, y0, incy);                                                   \
    else                                                                                                                     \
        hipLaunchKernelGGL((fewrows_t_kernel<T, FV, MR_, BETA_, false>), dim3((unsigned)grid), dim3(kFewThreads), 0, h->stream, (int)rows, \
                           cols, A, lda, x0, incx, alpha, beta, y0, incy)
#define MXB_FEW_T(MR_)                                                                                                       \
    if (beta != T(0)) { MXB_FEW_T2(MR_, true); } else { MXB_FEW_T2(MR_, false); }
        const bool keep = keeps_matrix((rows + 1) * cols * (int64_t)sizeof(T));
        switch (mr) {
            case 1: MXB_FEW_T(1); break;
            case 2: MXB_FEW_T(2); break;
            case 4: MXB_FEW_T(4); break;
            case 8: MXB_FEW_T(8); break;
            default: MXB_FEW_T(16); break;
        }
#undef MXB_FEW_T
#undef MXB_FEW_T2
        return launch_status();
    }
    if (no_trans && batch == 1 && rows <= kWideMaxRows && cols >= kWideMinCols) {
        // Few, very long rows: the row-dot grid wants some 8192 rows to be busy.  The columns are cut
        // into chunks, the chunks run as a batch of rows x chunk problems that write partial results
        // (a shorter last chunk in a launch of its own), and the pass that combines the partial
        // vectors of the transposed product adds them up, in chunk order, with alpha and beta.
        int64_t parts = ceil_div(kWideFillRows, rows);
        if (parts > cols / kWideMinChunk) parts = cols / kWideMinChunk;
        const int64_t chunk = ceil_div(ceil_div(cols, parts), (int64_t)256) * 256;
        const int64_t nfull = cols / chunk, tail = cols - nfull * chunk, nparts = nfull + (tail > 0 ? 1 : 0);
        T* partials = static_cast<T*>(take_workspace(h, (size_t)nparts * (size_t)rows * sizeof(T)));
        if (!partials) return MXB_ERR_WORKSPACE;
        RowdotArgs<T> a{rows, chunk, A, lda, x0, incx, partials, 1, T(1), T(0), 0, 0, nfull, chunk, chunk * incx, rows};
        int st = launch_rowdot(h, a, MODE_GENERAL, false);
        if (st != MXB_OK) return st;
        if (tail > 0) {
            RowdotArgs<T> b{rows, tail, A + nfull * chunk, lda, x0 + nfull * chunk * incx, incx, partials + nfull * rows, 1, T(1), T(0),
                            0, 0, 1, 0, 0, 0};
            st = launch_rowdot(h, b, MODE_GENERAL, false);
            if (st != MXB_OK) return st;
        }
        hipLaunchKernelGGL(colacc_combine_kernel<T>, dim3((unsigned)ceil_div(rows, (int64_t)kWave), 1u), dim3(kCombineGroups * kWave), 0,
                           h->stream, nparts, rows, rows, partials, alpha, beta, y0, incy, (int64_t)0, (int64_t)0);
        return launch_status();
    }
    if (no_trans && batch == 1 && cols >= kWave * Full<T>::vec / 2 && rows * cols * (int64_t)sizeof(T) <= option(h, MXB_OPT_GEMVN_SMALL_MAX)) {
        // a matrix that comes from the caches, rows of at least half a wavefront of vectors: one or two
        // rows per wavefront, no LDS, no barrier
        constexpr int FV = Full<T>::vec;
        RowdotArgs<T> a{rows, cols, A, lda, x0, incx, y0, incy, alpha, beta, 0, 0};
        constexpr int WPB = kRowSmallThreads / kWave;
        const int64_t loads = ceil_div(cols, (int64_t)kWave * FV);          // loads that cover a row
        const dim3 g1((unsigned)ceil_div(rows, (int64_t)WPB)), g2((unsigned)ceil_div(rows, (int64_t)WPB * 2)), blk(kRowSmallThreads);
        if (rows > kRowSmallOneRow) hipLaunchKernelGGL((rowsmall_kernel<T, FV, 2, 4, 1>), g2, blk, 0, h->stream, a);
        else if (rows <= 256 && loads >= 32) hipLaunchKernelGGL((rowsmall_kernel<T, FV, 1, 4, 8>), dim3((unsigned)rows), dim3(8 * kWave), 0, h->stream, a);
        else if (rows <= 512 && loads >= 16) hipLaunchKernelGGL((rowsmall_kernel<T, FV, 1, 4, 4>), dim3((unsigned)rows), dim3(4 * kWave), 0, h->stream, a);
        else if (loads <= 2) hipLaunchKernelGGL((rowsmall_kernel<T, FV, 1, 2, 1>), g1, blk, 0, h->stream, a);
        else if (loads <= 4) hipLaunchKernelGGL((rowsmall_kernel<T, FV, 1, 4, 1>), g1, blk, 0, h->stream, a);
        else hipLaunchKernelGGL((rowsmall_kernel<T, FV, 1, 8, 1>), g1, blk, 0, h->stream, a);
        return launch_status();
    }
    if (no_trans && batch > 1 && rows <= kRowSmallBatchRows && rows * batch < ((int64_t)1 << 31) * (kRowSmallThreads / kWave)) {
        // a batch of problems of a few rows each: one wavefront per row, the rows of all problems as one list
        // (per call, 1 x 100 in 167772 problems: 909 -> 41 us; 1 x 256 in 65536: 417 -> 27; 8 x 100 in 20971: 118 -> 40)
        constexpr int FV = Full<T>::vec;
        RowdotArgs<T> a{rows, cols, A, lda, x0, incx, y0, incy, alpha, beta, 0, 0, batch, sA, sx, sy};
        const int64_t loads = ceil_div(cols, (int64_t)kWave * FV);
        const dim3 g((unsigned)ceil_div(rows * batch, (int64_t)(kRowSmallThreads / kWave))), blk(kRowSmallThreads);
        if (loads <= 2) hipLaunchKernelGGL((rowsmall_kernel<T, FV, 1, 2, 1, MODE_GENERAL, false, true>), g, blk, 0, h->stream, a);
        else if (loads <= 4) hipLaunchKernelGGL((rowsmall_kernel<T, FV, 1, 4, 1, MODE_GENERAL, false, true>), g, blk, 0, h->stream, a);
        else hipLaunchKernelGGL((rowsmall_kernel<T, FV, 1, 8, 1, MODE_GENERAL, false, true>), g, blk, 0, h->stream, a);
        return launch_status();
    }
    if (no_trans) {
        RowdotArgs<T> a{rows, cols, A, lda, x0, incx, y0, incy, alpha, beta, 0, 0, batch, sA, sx, sy};
        return launch_rowdot(h, a, MODE_GENERAL, false);
    }
    ColaccArgs<T> a{rows, cols, A, lda, x0, incx, y0, incy, alpha, beta, nullptr, 0, 0, sA, sx, sy, 0};
    return launch_colacc(h, a, batch);
}

// Argument checks of gemv.  Returns the status to hand back, or kProceed when there is work to launch.
constexpr int kProceed = 1 << 30;
template <typename T>
int gemv_check(mxb_handle_t h, int layout, int trans, int64_t m, int64_t n, T alpha, const T* A, int64_t lda, const T* x,
               int64_t incx, T beta, T* y, int64_t incy)
{
    if (!handle_ok(h)) return MXB_ERR_HANDLE;
    if (!layout_ok(layout)) return -1;
    if (!trans_ok(trans)) return -2;
    if (m < 0) return -3;
    if (n < 0) return -4;
    const int64_t minor = layout == MXB_ROW_MAJOR ? n : m;
    if (lda < (minor > 1 ? minor : 1)) return -7;
    if (incx == 0) return -9;
    if (incy == 0) return -12;
    if (m == 0 || n == 0 || (alpha == T(0) && beta == T(1))) return MXB_OK;
    if (!y) return -11;
    if (alpha != T(0)) {
        if (!A) return -6;
        if (!x) return -8;
    }
    return kProceed;
}

template <typename T>
int gemv(mxb_handle_t h, int layout, int trans, int64_t m, int64_t n, T alpha, const T* A, int64_t lda, const T* x,
         int64_t incx, T beta, T* y, int64_t incy)
{
    const int chk = gemv_check<T>(h, layout, trans, m, n, alpha, A, lda, x, incx, beta, y, incy);
    if (chk != kProceed) return chk;
    // a column-major m x n matrix is the row-major n x m matrix of the transposed problem
    const bool row_major = layout == MXB_ROW_MAJOR;
    const int64_t rows = row_major ? m : n, cols = row_major ? n : m;
    const bool no_trans = (trans == MXB_NO_TRANS) == row_major;
    const int64_t lenx = no_trans ? cols : rows, leny = no_trans ? rows : cols;
    return gemv_rows<T>(h, no_trans, rows, cols, alpha, A, lda, 0, x ? vec_base(x, lenx, incx) : x, incx, 0, beta,
                        vec_base(y, leny, incy), incy, 0, 1);
}

// ---------------------------------------------------------------------------------------------
// gemv without a caller's workspace

// Scratch memory of mxb_sgemv_static: the partial vectors that the handle's workspace holds for
// mxb_sgemv.  One copy per GPU, there from the moment the library is loaded until the process
// ends.  In host code the array's name stands for the symbol, not for device memory: its address
// on a GPU comes from hipGetSymbolAddress, asked for once per device with that device current.
static __device__ __align__(256) unsigned char scratch[MXB_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];      // per device; null until the first call on it

// Device address of `scratch` on the current GPU, or null with a status in `st`.
void* static_scratch(int& st)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { st = MXB_ERR_HIP_BASE + (int)e; return nullptr; }
    if (dev < 0 || dev >= kMaxDevices) { st = MXB_ERR_NOT_IMPLEMENTED; return nullptr; }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) { st = MXB_ERR_HIP_BASE + (int)e; return nullptr; }
        g_scratch_ptr[dev] = p;
    }
    st = MXB_OK;
    return g_scratch_ptr[dev];
}

int sgemv_static(mxb_handle_t h, int layout, int trans, int64_t m, int64_t n, float alpha, const float* A, int64_t lda,
                 const float* x, int64_t incx, float beta, float* y, int64_t incy)
{
    // the argument checks first: they touch no device state
    const int chk = gemv_check<float>(h, layout, trans, m, n, alpha, A, lda, x, incx, beta, y, incy);
    if (chk != kProceed) return chk;
    int st;
    void* ptr = static_scratch(st);
    if (!ptr) return st;
    // The same launchers as mxb_sgemv, with the static array standing in for the handle's
    // workspace for the length of this call.  Every kernel that reads partial results reads only
    // what this call's first pass wrote, so nothing has to be cleared between calls.
    void* const ws = h->ws;
    const size_t ws_bytes = h->ws_bytes;
    const int* const status = h->device_status;
    h->ws = ptr;
    h->ws_bytes = MXB_STATIC_SCRATCH_BYTES;
    st = gemv<float>(h, layout, trans, m, n, alpha, A, lda, x, incx, beta, y, incy);
    h->ws = ws;
    h->ws_bytes = ws_bytes;
    h->device_status = status;
    // every launcher asks for its partial vectors before it launches anything
    return st == MXB_ERR_WORKSPACE ? MXB_ERR_STATIC_LIMIT : st;
}

// `batch` gemv problems of one shape; problem b uses A + b*strideA, x + b*stridex, y + b*stridey.
template <typename T>
int gemv_batched(mxb_handle_t h, int layout, int trans, int64_t m, int64_t n, T alpha, const T* A, int64_t lda, int64_t strideA,
                 const T* x, int64_t incx, int64_t stridex, T beta, T* y, int64_t incy, int64_t stridey, int64_t batch)
{
    if (!handle_ok(h)) return MXB_ERR_HANDLE;
    if (!layout_ok(layout)) return -1;
    if (!trans_ok(trans)) return -2;
    if (m < 0) return -3;
    if (n < 0) return -4;
    const int64_t minor = layout == MXB_ROW_MAJOR ? n : m;
    if (lda < (minor > 1 ? minor : 1)) return -7;
    if (strideA < 0) return -8;
    if (incx == 0) return -10;
    if (stridex < 0) return -11;
    if (incy == 0) return -14;
    if (batch < 0) return -16;
    if (stridey < 0 || (stridey == 0 && batch > 1)) return -15;      // the results of two problems would collide
    if (m == 0 || n == 0 || batch == 0 || (alpha == T(0) && beta == T(1))) return MXB_OK;
    if (!y) return -13;
    const bool row_major = layout == MXB_ROW_MAJOR;
    const int64_t rows = row_major ? m : n, cols = row_major ? n : m;
    const bool no_trans = (trans == MXB_NO_TRANS) == row_major;
    const int64_t lenx = no_trans ? cols : rows, leny = no_trans ? rows : cols;
    if (alpha != T(0)) {
        if (!A) return -6;
        if (!x) return -9;
    }
    return gemv_rows<T>(h, no_trans, rows, cols, alpha, A, lda, strideA, x ? vec_base(x, lenx, incx) : x, incx, stridex, beta,
                        vec_base(y, leny, incy), incy, stridey, batch);
}

template <typename T>
int trmv(mxb_handle_t h, int layout, int uplo, int trans, int diag, int64_t n, const T* A, int64_t lda, T* x, int64_t incx)
{
    if (!handle_ok(h)) return MXB_ERR_HANDLE;
    if (!layout_ok(layout)) return -1;
    if (!uplo_ok(uplo)) return -2;
    if (!trans_ok(trans)) return -3;
    if (!diag_ok(diag)) return -4;
    if (n < 0) return -5;
    if (lda < (n > 1 ? n : 1)) return -7;
    if (incx == 0) return -9;
    if (n == 0) return MXB_OK;
    if (!A) return -6;
    if (!x) return -8;
    // column-major: the same bytes are the row-major transpose, whose stored triangle is the other one
    const bool row_major = layout == MXB_ROW_MAJOR;
    const bool upper = (uplo == MXB_UPPER) == row_major;
    const bool no_trans = (trans == MXB_NO_TRANS) == row_major;
    const int mode = upper ? MODE_UPPER : MODE_LOWER;
    const bool unit = diag == MXB_UNIT;

    T* x0 = vec_base(x, n, incx);
    if (!no_trans && n >= Full<T>::vec && n <= kSmallMaxRows) {
        // transposed, a small triangle: a snapshot of x, then the single-kernel column sums of a small
        // transposed gemv in triangular mode (no partial vectors)
        T* snap = static_cast<T*>(take_workspace(h, align_up((size_t)n * sizeof(T), 256)));
        if (!snap) return MXB_ERR_WORKSPACE;
        hipLaunchKernelGGL(gather_kernel<T>, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, h->stream, n, x0, incx, snap);
        const int st = launch_status();
        if (st != MXB_OK) return st;
        constexpr int FV = Full<T>::vec;
        ColaccArgs<T> a{n, n, A, lda, snap, 1, x0, incx, T(1), T(0), nullptr, 0, 0};
#define MXB_COLSUM_TRI(CL_, RL_)                                                                     \
    if (upper) {                                                                                     \
        if (unit) launch_colsum_small<T, FV, CL_, RL_, MODE_UPPER, true>(h, a);                       \
        else launch_colsum_small<T, FV, CL_, RL_, MODE_UPPER, false>(h, a);                           \
    } else {                                                                                         \
        if (unit) launch_colsum_small<T, FV, CL_, RL_, MODE_LOWER, true>(h, a);                       \
        else launch_colsum_small<T, FV, CL_, RL_, MODE_LOWER, false>(h, a);                           \
    }
        if (n <= 256) { MXB_COLSUM_TRI(8, 32) }
        else if (n <= 512) { MXB_COLSUM_TRI(8, 64) }
        else if (n <= 1536) { MXB_COLSUM_TRI(4, 128) }
        else { MXB_COLSUM_TRI(8, 128) }
#undef MXB_COLSUM_TRI
        return launch_status();
    }
    // transposed: the triangle sweep reads x, its combine pass writes x afterwards: no copy needed
    if (!no_trans) return trisweep_trmv_t<T>(h, upper, unit, n, A, lda, x0, incx);

    // not transposed: rows are written while other blocks still read x, so work from a snapshot
    const size_t snap_bytes = align_up((size_t)n * sizeof(T), 256);
    T* snap = static_cast<T*>(take_workspace(h, snap_bytes));
    if (!snap) return MXB_ERR_WORKSPACE;
    hipLaunchKernelGGL(gather_kernel<T>, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, h->stream, n, x0, incx, snap);
    int st = launch_status();
    if (st != MXB_OK) return st;
    RowdotArgs<T> a{n, n, A, lda, snap, 1, x0, incx, T(1), T(0), 0, 0};
    constexpr int FV = Full<T>::vec;
    if (n >= kWave * FV / 2 && n * (n + 1) / 2 * (int64_t)sizeof(T) <= option(h, MXB_OPT_GEMVN_SMALL_MAX)) {
        // a triangle that comes from the caches: one or two rows per wavefront, as for gemv
        constexpr int WPB = kRowSmallThreads / kWave;
        const int64_t loads = ceil_div(n, (int64_t)kWave * FV);
        const dim3 g1((unsigned)ceil_div(n, (int64_t)WPB)), g2((unsigned)ceil_div(n, (int64_t)WPB * 2)), blk(kRowSmallThreads);
#define MXB_ROWSMALL_TRI(R_, U_, G_)                                                                                         \
    if (mode == MODE_UPPER) {                                                                                                \
        if (unit) hipLaunchKernelGGL((rowsmall_kernel<T, FV, R_, U_, 1, MODE_UPPER, true>), G_, blk, 0, h->stream, a);        \
        else hipLaunchKernelGGL((rowsmall_kernel<T, FV, R_, U_, 1, MODE_UPPER, false>), G_, blk, 0, h->stream, a);            \
    } else {                                                                                                                 \
        if (unit) hipLaunchKernelGGL((rowsmall_kernel<T, FV, R_, U_, 1, MODE_LOWER, true>), G_, blk, 0, h->stream, a);        \
        else hipLaunchKernelGGL((rowsmall_kernel<T, FV, R_, U_, 1, MODE_LOWER, false>), G_, blk, 0, h->stream, a);            \
    }
        if (n > kRowSmallOneRow) { MXB_ROWSMALL_TRI(2, 4, g2) }
        else if (loads <= 2) { MXB_ROWSMALL_TRI(1, 2, g1) }
        else if (loads <= 4) { MXB_ROWSMALL_TRI(1, 4, g1) }
        else { MXB_ROWSMALL_TRI(1, 8, g1) }
#undef MXB_ROWSMALL_TRI
        return launch_status();
    }
    return launch_rowdot(h, a, mode, unit);
}

}  // namespace
}  // namespace mxb

extern "C" {
int mxb_sgemv(mxb_handle_t h, mxb_layout_t layout, mxb_trans_t trans, int64_t m, int64_t n, float alpha, const float* A,
              int64_t lda, const float* x, int64_t incx, float beta, float* y, int64_t incy)
{ return mxb::gemv<float>(h, layout, trans, m, n, alpha, A, lda, x, incx, beta, y, incy); }
int mxb_dgemv(mxb_handle_t h, mxb_layout_t layout, mxb_trans_t trans, int64_t m, int64_t n, double alpha, const double* A,
              int64_t lda, const double* x, int64_t incx, double beta, double* y, int64_t incy)
{ return mxb::gemv<double>(h, layout, trans, m, n, alpha, A, lda, x, incx, beta, y, incy); }
int mxb_sgemv_static(mxb_handle_t h, mxb_layout_t layout, mxb_trans_t trans, int64_t m, int64_t n, float alpha, const float* A,
                     int64_t lda, const float* x, int64_t incx, float beta, float* y, int64_t incy)
{ return mxb::sgemv_static(h, layout, trans, m, n, alpha, A, lda, x, incx, beta, y, incy); }
int mxb_sgemv_batched(mxb_handle_t h, mxb_layout_t layout, mxb_trans_t trans, int64_t m, int64_t n, float alpha,
                      const float* A, int64_t lda, int64_t strideA, const float* x, int64_t incx, int64_t stridex,
                      float beta, float* y, int64_t incy, int64_t stridey, int64_t batch)
{ return mxb::gemv_batched<float>(h, layout, trans, m, n, alpha, A, lda, strideA, x, incx, stridex, beta, y, incy, stridey, batch); }
int mxb_dgemv_batched(mxb_handle_t h, mxb_layout_t layout, mxb_trans_t trans, int64_t m, int64_t n, double alpha,
                      const double* A, int64_t lda, int64_t strideA, const double* x, int64_t incx, int64_t stridex,
                      double beta, double* y, int64_t incy, int64_t stridey, int64_t batch)
{ return mxb::gemv_batched<double>(h, layout, trans, m, n, alpha, A, lda, strideA, x, incx, stridex, beta, y, incy, stridey, batch); }
int mxb_strmv(mxb_handle_t h, mxb_layout_t layout, mxb_uplo_t uplo, mxb_trans_t trans, mxb_diag_t diag, int64_t n,
              const float* A, int64_t lda, float* x, int64_t incx)
{ return mxb::trmv<float>(h, layout, uplo, trans, diag, n, A, lda, x, incx); }
int mxb_dtrmv(mxb_handle_t h, mxb_layout_t layout, mxb_uplo_t uplo, mxb_trans_t trans, mxb_diag_t diag, int64_t n,
              const double* A, int64_t lda, double* x, int64_t incx)
{ return mxb::trmv<double>(h, layout, uplo, trans, diag, n, A, lda, x, incx); }
}
