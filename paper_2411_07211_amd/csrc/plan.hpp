// Host-side launch plans shared by the level-2 launchers and by mxb_workspace_bytes.
#pragma once
#include "common.hpp"

namespace mxb {

// Column-accumulate kernels (transposed gemv / trmv on a row-major matrix): a block of 4
// wavefronts covers `cols_per_block` columns and one of `nparts` row groups and produces one
// partial vector; the partial vectors of a column are combined by a second kernel (none if 1).
struct ColaccPlan {
    int wr;                  // wavefronts of a block that split the rows (1: wide shape, 4: narrow shape)
    int cv;                  // column vectors per lane (wide shape)
    int64_t cols_per_block;
    int64_t col_tiles;
    int64_t rows_per_block;  // narrow shape: rows of one slab
    int64_t nparts;          // row groups = partial vectors per column
};

inline ColaccPlan colacc_plan(int64_t rows, int64_t cols, int elem_size, int vec, bool triangular, int64_t target_blocks,
                              int64_t narrow_blocks, int64_t min_rows)
{
    ColaccPlan p;
    rows = rows > 0 ? rows : 1;
    cols = cols > 0 ? cols : 1;
    p.wr = cols <= 2 * kWave * vec ? 4 : 1;
    p.cv = 1;
    const int64_t span = (int64_t)(4 / p.wr) * kWave * vec;
    // A matrix that fits the 256 MiB last-level cache is not an HBM stream: it wants many small
    // blocks (latency), not a few long sweeping ones.
    const bool cache_sized = rows * cols * elem_size <= ((int64_t)128 << 20);
    if (p.wr == 1 && !triangular && !cache_sized) {
        // widest lane footprint that wastes under an eighth of the lanes on the ragged last tile;
        // triangular shapes keep one vector per lane: more, smaller tiles balance the load better
        for (int cv : {4, 2}) {
            const int64_t padded = ceil_div(cols, cv * span) * cv * span;
            if ((padded - cols) * 8 <= padded) { p.cv = cv; break; }
        }
    }
    p.cols_per_block = p.cv * span;
    p.col_tiles = ceil_div(cols, p.cols_per_block);
    if (triangular || cache_sized) target_blocks *= 4;
    if (p.wr == 4) target_blocks = narrow_blocks;
    int64_t parts = ceil_div(target_blocks, p.col_tiles);
    const int64_t max_parts = ceil_div(rows, min_rows * p.wr);
    if (parts > max_parts) parts = max_parts;
    if (parts < 1) parts = 1;
    if (p.wr == 1) {
        p.rows_per_block = ceil_div(rows, parts);
        p.nparts = parts;
    } else {
        const int64_t quantum = 8 * p.wr;
        p.rows_per_block = ceil_div(ceil_div(rows, parts), quantum) * quantum;
        p.nparts = ceil_div(rows, p.rows_per_block);
    }
    return p;
}

// symv: the stored triangle is cut into column tiles of cv*256*vec columns.  Tile t owns the
// rows that have stored elements in its columns (lower: from its first column down; upper: from
// the top to its last column) and gets a share of the blocks proportional to that row count, so
// that all blocks stream about the same number of bytes.  Block s of a tile takes batches of
// adjacent rows cyclically.  Every block yields one partial column-sum vector over its tile
// (colpart[s]) and every wavefront one partial row sum per row it visits (rowpart[4*t + wave]).
constexpr int kSymvMaxTiles = 128;

struct SymvPlan {
    int cv;                              // column vectors per lane
    int64_t tile_cols;
    int ntiles;
    int first_block[kSymvMaxTiles + 1];  // blocks of tile t: [first_block[t], first_block[t+1])
    int max_groups;                      // largest number of blocks any tile has
    bool ok;                             // false: n needs more than kSymvMaxTiles tiles
};

inline SymvPlan symv_plan(int64_t n, int vec, bool upper, int64_t target_blocks, int64_t force_cv = 0)
{
    SymvPlan p;
    n = n > 0 ? n : 1;
    const int64_t span = 256 * (int64_t)vec;
    // two vectors per lane unless that wastes over an eighth of the lanes on the ragged last tile
    // (wider tiles spend more of their batches in the masked code along the diagonal)
    p.cv = 1;
    {
        const int64_t padded = ceil_div(n, 2 * span) * 2 * span;
        if ((padded - n) * 8 <= padded) p.cv = 2;
    }
    if (force_cv == 1 || force_cv == 2 || force_cv == 4) p.cv = (int)force_cv;
    while (p.cv < 4 && ceil_div(n, p.cv * span) > kSymvMaxTiles) p.cv *= 2;
    p.tile_cols = p.cv * span;
    const int64_t nt = ceil_div(n, p.tile_cols);
    p.ok = nt <= kSymvMaxTiles;
    p.ntiles = (int)(p.ok ? nt : kSymvMaxTiles);
    const int batch = p.cv == 4 ? 4 : 8;
    int64_t total_rows = 0;
    for (int t = 0; t < p.ntiles; ++t) {
        const int64_t c0 = t * p.tile_cols, c1 = c0 + p.tile_cols < n ? c0 + p.tile_cols : n;
        total_rows += upper ? c1 : n - c0;
    }
    p.first_block[0] = 0;
    p.max_groups = 1;
    for (int t = 0; t < p.ntiles; ++t) {
        const int64_t c0 = t * p.tile_cols, c1 = c0 + p.tile_cols < n ? c0 + p.tile_cols : n;
        const int64_t rows = upper ? c1 : n - c0;
        int64_t g = (target_blocks * rows + total_rows / 2) / total_rows;
        const int64_t cap = ceil_div(rows, batch);
        if (g > cap) g = cap;
        if (g < 1) g = 1;
        p.first_block[t + 1] = p.first_block[t] + (int)g;
        if (g > p.max_groups) p.max_groups = (int)g;
    }
    return p;
}

}  // namespace mxb
