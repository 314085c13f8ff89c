// Default launch geometry and per-handle overrides.
#pragma once
#include "common.hpp"

namespace mxb {

inline int64_t option_default(int o)
{
    switch (o) {
        case MXB_OPT_L1_BLOCKS_PER_CU: return 1 << 20;   // in effect one 16 KiB tile per block: read+write streams run best unthrottled
        case MXB_OPT_REDUCE_BLOCKS: return 256;
        case MXB_OPT_ROWDOT_XCHUNK: return 4096;       // elements; capped to 64 KiB of LDS by the launcher
        case MXB_OPT_ROWDOT_BLOCKS_PER_CU: return 2;
        case MXB_OPT_COLACC_TARGET_BLOCKS: return 192;
        case MXB_OPT_COLACC_MIN_ROWS: return 64;
        case MXB_OPT_SYMV_TARGET_BLOCKS: return 192;   // grid of the triangle sweep (symv, transposed trmv)
        case MXB_OPT_GER_ROWS_PER_BLOCK: return 8;     // one batch of 8 rows per block: short read-then-write bursts stream best
        case MXB_OPT_SYMV_TILE_VECTORS: return 0;     // 0: chosen from n
        case MXB_OPT_TRI_DIAG_WEIGHT: return 3;
        case MXB_OPT_GEMVT_SMALL_MAX: return 32 << 20;   // and at most 2048 rows; larger matrices stream better through the general kernels
        case MXB_OPT_GEMVN_SMALL_MAX: return kKeepMatrixBytes;   // what stays in the last-level cache; beyond, the persistent row-dot grid with x in LDS and streaming loads (per call, repeated: 5000^2 16.9 against 22.6 us, 7000^2 29.0 against 33.3, 8192^2 39.4 against 40.5, 10000^2 71.5 against 65.6)
        case MXB_OPT_TRSV_SPIN_LIMIT: return 1 << 24;  // polls of one hand-over word before a wavefront gives up: tens of seconds
        case MXB_OPT_TRSV_CHAIN_MIN: return 129;       // from here the chained kernel is faster than a launch per block
        case MXB_OPT_SYMV_SMALL_MAX: return 2400;      // beyond this the triangle sweep is faster (measured per call: 2048 7.6 against 8.7 us, 2500 9.8 against 10.2, 3000 12.1 against 10.6; double precision, two thirds of it: 1536 8.5 against 9.4, 2048 11.6 against 10.4)
        default: return 0;
    }
}

inline int64_t option(mxb_handle_t h, int o) { return h->opt[o] > 0 ? h->opt[o] : option_default(o); }

// Blocks the narrow column-accumulate shape aims for: two per compute unit, or twice the
// caller's MXB_OPT_COLACC_TARGET_BLOCKS when that option is set.
constexpr int64_t kColaccNarrowBlocks = 2 * kCUs;
constexpr int64_t kStridedBlocksFactor = 8;   // first-pass blocks of a strided one-operand reduction per MXB_OPT_REDUCE_BLOCKS
constexpr int64_t kProbeReadBlocks = 2048;    // the read probe keeps 8 loads in flight per lane and needs many blocks
inline int64_t colacc_narrow_target(mxb_handle_t h)
{
    return h->opt[MXB_OPT_COLACC_TARGET_BLOCKS] > 0 ? 2 * h->opt[MXB_OPT_COLACC_TARGET_BLOCKS] : kColaccNarrowBlocks;
}

}  // namespace mxb
