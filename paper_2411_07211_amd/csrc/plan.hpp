// Host-side launch plans shared by the level-2 launchers and by mxb_workspace_bytes.
#pragma once
#include "common.hpp"

namespace mxb {

// Column-accumulate kernels (transposed gemv on a row-major matrix): a block of 4
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

// gemv, not transposed, few and very long rows: up to kWideMaxRows rows of at least kWideMinCols
// columns, the columns are split into chunks of at least kWideMinChunk so that rows x chunks
// reaches kWideFillRows (what keeps the row-dot grid busy); the chunks' partial results take at
// most kWideFillRows + 2 rows' worth of elements of workspace.
constexpr int64_t kWideMaxRows = 4096, kWideMinCols = 32768, kWideMinChunk = 2048, kWideFillRows = 8192;
// Up to kFewRows rows of that length (up to kFewMaxRows rows of at least kFewManyMinCols columns)
// are a handful of dot products sharing x: at most kFewBlocks blocks (two per compute unit read
// fastest, measured from 256 to 4096), each with one partial result per row.
constexpr int64_t kFewRows = 16, kFewMaxRows = 32, kFewManyMinCols = (int64_t)1 << 21, kFewBlocks = 512;
// The transposed product of up to kFewStreamRows rows of at least kFewStreamMinCols columns is a
// read-and-write stream over the columns: one tile per block, as in the level-1 kernels (the cap
// keeps a launch below 2^32 threads); up to twice as many rows while the matrix is small.  The
// column-accumulate kernel keeps 16 rows in flight and falls back to one load at a time when there
// are fewer (per call, repeated: 1 x 4194304 69 -> 5.9 us, 2 x 4194304 81 -> 11.6, 4 x 1048576 20.1 ->
// 4.0, 8 x 1048576 23.2 -> 8.1, 8 x 16777216 122 -> 112, 16 x 262144 8.0 -> 4.0, but 16 x 1048576 14.9
// against 17.1; at 65536 columns the column-accumulate kernels are 0.2 us faster).
constexpr int64_t kFewStreamRows = 8, kFewStreamBlocks = (int64_t)1 << 22, kFewStreamMinCols = (int64_t)1 << 17,
                  kFewStreamManyMaxBytes = (int64_t)32 << 20;

inline ColaccPlan colacc_plan(int64_t rows, int64_t cols, int elem_size, int vec, int64_t target_blocks,
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
    if (p.wr == 1 && !cache_sized) {
        // widest lane footprint that wastes under an eighth of the lanes on the ragged last tile
        for (int cv : {4, 2}) {
            const int64_t padded = ceil_div(cols, cv * span) * cv * span;
            if ((padded - cols) * 8 <= padded) { p.cv = cv; break; }
        }
    }
    p.cols_per_block = p.cv * span;
    p.col_tiles = ceil_div(cols, p.cols_per_block);
    if (cache_sized) target_blocks *= 4;
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

}  // namespace mxb
