// Triangle sweep: the kernel behind symv and transposed trmv (Sec. 6.2.2).  Host-side plan and
// entry points; the kernels live in trisweep.hip.
#pragma once
#include "common.hpp"

namespace mxb {

// The stored triangle of an n x n row-major matrix is cut into column tiles of `tile_cols`
// columns.  Tile t owns the rows that have stored elements in its columns: the tile_cols rows
// that cross the diagonal there and the rows wholly inside the triangle (below them if lower,
// above if upper).  It gets a share of the blocks in proportion to its work, so that all blocks
// finish together; a row that crosses the diagonal counts diag_weight/4 of a row that does not
// (fewer bytes, but masked code).
constexpr int kTriThreads = 512;
constexpr int kTriWaves = kTriThreads / kWave;
constexpr int kTriMaxTiles = 128;
constexpr int64_t kTriDefaultBlocks = 192, kTriCachedBlocks = 256;

struct TriPlan {
    int vec;         // elements per load (16-byte vectors; 1 only for matrices narrower than one vector)
    int cv;          // vectors per lane and row
    int ub;          // loads a lane keeps in flight in a batch of rows off the diagonal: 4, 8 or 16
    int tile_cols;   // cv * 512 * vec
    int ntiles;
    int blocks;      // grid size; at least ntiles
    int first_block[kTriMaxTiles + 1];   // blocks of tile t: [first_block[t], first_block[t+1])
    bool ok;         // false: n needs more than kTriMaxTiles tiles
};

inline TriPlan tri_plan(int64_t n, int vec, int elem_size, bool upper, int64_t want_blocks, int64_t force_cv, int64_t diag_weight)
{
    TriPlan p;
    n = n > 0 ? n : 1;
    p.vec = vec;
    const int64_t span = (int64_t)kTriThreads * vec;
    // two vectors per lane once that still leaves four tiles: wide tiles read long runs of every
    // row, but the rows that cross the diagonal run masked code and should stay a small part
    p.cv = n >= 4 * 2 * span ? 2 : 1;
    if (force_cv == 1 || force_cv == 2 || force_cv == 4) p.cv = (int)force_cv;
    if (vec == 1) p.cv = 1;      // scalar loads serve only matrices narrower than one vector
    while (p.cv < 4 && ceil_div(n, p.cv * span) > kTriMaxTiles) p.cv *= 2;
    // Long batches (16 loads in flight per lane) sweep a triangle that streams from HBM fastest; a
    // triangle that fits the last-level cache is bound by the latency of its few batches per
    // block and wants short ones (measured: 4 loads below 72 MiB, 8 below 288 MiB).
    const int64_t tri_bytes = n * (n + 1) / 2 * elem_size;
    p.ub = (p.cv > 1 || tri_bytes >= ((int64_t)288 << 20)) ? 16 : tri_bytes >= ((int64_t)72 << 20) ? 8 : 4;
    if (vec == 1) p.ub = 4;
    p.tile_cols = (int)(p.cv * span);
    const int64_t nt = ceil_div(n, p.tile_cols);
    p.ok = nt <= kTriMaxTiles;
    p.ntiles = (int)(p.ok ? nt : kTriMaxTiles);
    const int64_t dw = diag_weight < 1 ? 1 : (diag_weight > 8 ? 8 : diag_weight);
    // work of a tile in quarter rows
    int64_t work[kTriMaxTiles], total = 0;
    for (int t = 0; t < p.ntiles; ++t) {
        const int64_t c0 = (int64_t)t * p.tile_cols, c1 = c0 + p.tile_cols < n ? c0 + p.tile_cols : n;
        const int64_t inside = upper ? c0 : n - c1, across = c1 - c0;
        // (a narrow last tile saves bytes, but a batch of its rows takes as long as a full one)
        work[t] = 4 * inside + dw * across;
        total += work[t];
    }
    // (a triangle that comes from the last-level cache wants a block per compute unit, one that streams
    // from HBM fewer: per call 4096 12.2 against 13.3 us, 6001 18.2 against 19.7, 12000 49.3 against 52.8)
    int64_t g = want_blocks > 0 ? want_blocks : (p.ub < 16 ? kTriCachedBlocks : kTriDefaultBlocks);
    const int64_t batches = ceil_div(n, p.ub / p.cv);
    if (g > batches * p.ntiles) g = batches * p.ntiles;      // more blocks than batches of rows are of no use
    if (g < p.ntiles) g = p.ntiles;
    p.blocks = (int)g;
    // one block each, the rest in proportion to the work (double: the products exceed 64 bits for large n)
    const int64_t spare = g - p.ntiles;
    double before = 0;
    p.first_block[0] = 0;
    for (int t = 0; t < p.ntiles; ++t) {
        before += (double)work[t];
        int64_t hi = t + 1 + (int64_t)(before / (double)total * (double)spare);
        if (hi > g - (p.ntiles - 1 - t)) hi = g - (p.ntiles - 1 - t);
        if (hi <= p.first_block[t]) hi = p.first_block[t] + 1;
        p.first_block[t + 1] = (int)hi;
    }
    p.first_block[p.ntiles] = (int)g;
    return p;
}

// Workspace of a sweep: per-wavefront row partials [ntiles * 8][n] (symv only) followed by the
// column partials [blocks][tile_cols].
inline size_t tri_workspace_elems(int64_t n, const TriPlan& p, bool row_sums)
{
    const size_t rows = row_sums ? (size_t)p.ntiles * kTriWaves * (size_t)n : 0;
    return rows + (size_t)p.blocks * (size_t)p.tile_cols;
}

// Upper bound over both vector widths and both triangles for the given options (0: default).
inline size_t tri_workspace_bound(int64_t n, int elem_size, int64_t want_blocks = 0, int64_t force_cv = 0, int64_t diag_weight = 3)
{
    size_t b = 0;
    for (int vec : {1, 16 / elem_size})
        for (bool upper : {false, true}) {
            const TriPlan p = tri_plan(n, vec, elem_size, upper, want_blocks, force_cv, diag_weight);
            const size_t need = tri_workspace_elems(n, p, true) * (size_t)elem_size;
            b = need > b ? need : b;
        }
    return align_up(b, 256);
}

// y = alpha*S*x + beta*y with S given by the `upper` or lower triangle of the row-major A.
// x0 / y0 point at logical element 0.  Arguments are already validated; uses h's workspace.
template <typename T>
int trisweep_symv(mxb_handle_t h, bool upper, int64_t n, T alpha, const T* A, int64_t lda, const T* x0, int64_t incx, T beta,
                  T* y0, int64_t incy);

// x := T^t x with T the `upper` or lower triangle of the row-major A (unit: diagonal taken as 1).
// The sweep only reads x and the combine pass writes it, so no copy of x is needed.
template <typename T>
int trisweep_trmv_t(mxb_handle_t h, bool upper, bool unit, int64_t n, const T* A, int64_t lda, T* x0, int64_t incx);

}  // namespace mxb
