// Handle management, workspace sizing and the two bandwidth probes.
#include <new>

#include "common.hpp"
#include "options.hpp"
#include "plan.hpp"
#include "skinny.hpp"
#include "trisweep.hpp"

namespace mxb {
namespace {

constexpr int kThreads = 256;
constexpr int kUnroll = 4;
typedef float f4 __attribute__((ext_vector_type(4)));

__global__ void __launch_bounds__(kThreads) probe_copy_kernel(int64_t nvec, int64_t ntiles, int64_t n2d, const f4* __restrict__ src,
                                                              f4* __restrict__ dst)
{
    for (int64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        int64_t base, step;
        stream_tile<kUnroll>(t, n2d, base, step);
        f4 a[kUnroll];
        if (t < n2d) {      // whole tiles of the 2-D part: no predicate
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) a[u] = ld_stream(src + base + u * step);
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) st_stream(dst + base + u * step, a[u]);
        } else {
#pragma unroll
            for (int u = 0; u < kUnroll; ++u)
                if (base + u * step < nvec) a[u] = ld_stream(src + base + u * step);
#pragma unroll
            for (int u = 0; u < kUnroll; ++u)
                if (base + u * step < nvec) st_stream(dst + base + u * step, a[u]);
        }
    }
}

__global__ void __launch_bounds__(kThreads) probe_read_kernel(int64_t nvec, int64_t ntiles, const f4* __restrict__ src,
                                                              double* __restrict__ out)
{
    __shared__ double slots[kThreads / kWave];
    f4 s = f4(0.f);
    for (int64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const int64_t base = t * (kThreads * kUnroll) + threadIdx.x;
        f4 a[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            a[u] = f4(0.f);
            if (base + u * kThreads < nvec) a[u] = ld_stream(src + base + u * kThreads);
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) s += a[u];
    }
    const double tot = block_sum<kThreads / kWave>((double)(s[0] + s[1] + s[2] + s[3]), slots);
    if (threadIdx.x == 0) out[blockIdx.x] = tot;
}

}  // namespace
}  // namespace mxb

extern "C" {

int mxb_create(mxb_handle_t* h)
{
    if (!h) return -1;
    mxb_ctx* c = new (std::nothrow) mxb_ctx;
    if (!c) return MXB_ERR_HANDLE;
    c->magic = mxb::kMagic;
    c->stream = nullptr;
    c->ws = nullptr;
    c->ws_bytes = 0;
    for (int o = 0; o < MXB_OPT_COUNT; ++o) c->opt[o] = 0;
    c->device_status = nullptr;
    *h = c;
    return MXB_OK;
}

int mxb_destroy(mxb_handle_t h)
{
    if (!mxb::handle_ok(h)) return MXB_ERR_HANDLE;
    h->magic = 0;
    delete h;
    return MXB_OK;
}

int mxb_set_stream(mxb_handle_t h, void* hip_stream)
{
    if (!mxb::handle_ok(h)) return MXB_ERR_HANDLE;
    h->stream = static_cast<hipStream_t>(hip_stream);
    return MXB_OK;
}

int mxb_set_workspace(mxb_handle_t h, void* dev_ptr, size_t bytes)
{
    if (!mxb::handle_ok(h)) return MXB_ERR_HANDLE;
    if ((reinterpret_cast<uintptr_t>(dev_ptr) & 255u) != 0) return -1;
    if (!dev_ptr && bytes != 0) return -2;
    h->ws = dev_ptr;
    h->ws_bytes = bytes;
    h->device_status = nullptr;
    return MXB_OK;
}

int mxb_set_option(mxb_handle_t h, int option, int64_t value)
{
    if (!mxb::handle_ok(h)) return MXB_ERR_HANDLE;
    if (option < 0 || option >= MXB_OPT_COUNT) return -1;
    h->opt[option] = value > 0 ? value : 0;
    return MXB_OK;
}

int64_t mxb_get_option(mxb_handle_t h, int option)
{
    if (!mxb::handle_ok(h) || option < 0 || option >= MXB_OPT_COUNT) return 0;
    return mxb::option(h, option);
}

int mxb_last_status(mxb_handle_t h)
{
    if (!mxb::handle_ok(h)) return MXB_ERR_HANDLE;
    int word = 0;
    hipError_t e = hipSuccess;
    if (h->device_status) e = hipMemcpyAsync(&word, h->device_status, sizeof(int), hipMemcpyDeviceToHost, h->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(h->stream);
    if (e != hipSuccess) return MXB_ERR_HIP_BASE + (int)e;
    return word != 0 ? MXB_ERR_TIMEOUT : MXB_OK;
}

size_t mxb_workspace_bytes(int routine, int elem_size, int64_t m, int64_t n)
{
    return mxb_workspace_bytes_for(nullptr, routine, elem_size, m, n);
}

size_t mxb_workspace_bytes_for(mxb_handle_t h, int routine, int elem_size, int64_t m, int64_t n)
{
    using namespace mxb;
    if ((elem_size != 4 && elem_size != 8) || m < 0 || n < 0) return 0;
    if (h && !handle_ok(h)) return 0;
    // the launch-geometry options that size partial results: the handle's, or the defaults
    auto opt = [&](int o) { return h ? option(h, o) : option_default(o); };
    auto raw = [&](int o) { return h ? h->opt[o] : (int64_t)0; };
    const int full = 16 / elem_size;
    auto colacc_bound = [&](int64_t rows, int64_t cols) {
        size_t b = 0;
        for (int vec : {1, full}) {
            const ColaccPlan p = colacc_plan(rows, cols, elem_size, vec, opt(MXB_OPT_COLACC_TARGET_BLOCKS),
                                             raw(MXB_OPT_COLACC_TARGET_BLOCKS) > 0 ? 2 * raw(MXB_OPT_COLACC_TARGET_BLOCKS) : kColaccNarrowBlocks,
                                             opt(MXB_OPT_COLACC_MIN_ROWS));
            const size_t need = p.nparts > 1 ? (size_t)p.nparts * (size_t)(ceil_div(cols, full) * full) * (size_t)elem_size : 0;
            b = need > b ? need : b;
        }
        return align_up(b, 256);
    };
    switch (routine) {
        case MXB_AXPY: case MXB_SCAL: case MXB_GER: return 0;
        case MXB_DOT: case MXB_ASUM: case MXB_NRM2:
            return (size_t)opt(MXB_OPT_REDUCE_BLOCKS) * kStridedBlocksFactor * 3 * sizeof(double);
        case MXB_GEMV: {
            size_t a = colacc_bound(m, n), b = colacc_bound(n, m);
            a = a > b ? a : b;
            // the skinny transposed product keeps one partial vector per block
            const int64_t narrow = m < n ? m : n;
            b = narrow <= 68 ? skinny_workspace_bytes(narrow, elem_size) : 0;
            a = a > b ? a : b;
            // few long rows, not transposed: partial results of the column chunks
            b = align_up((size_t)(kWideFillRows + 2 * kWideMaxRows) * (size_t)elem_size, 256);
            a = a > b ? a : b;
            b = align_up((size_t)(kFewBlocks * kFewMaxRows) * (size_t)elem_size, 256);     // a handful of rows
            a = a > b ? a : b;
            return a;
        }
        case MXB_GEMV_BATCHED: {
            // the blocks a plan aims at are shared among the problems: over all problems there are at most
            // one and a half times as many partial vectors as the largest target
            int64_t t = 4 * opt(MXB_OPT_COLACC_TARGET_BLOCKS);
            if (raw(MXB_OPT_COLACC_TARGET_BLOCKS) > 0 && 2 * raw(MXB_OPT_COLACC_TARGET_BLOCKS) > t) t = 2 * raw(MXB_OPT_COLACC_TARGET_BLOCKS);
            if (t < kColaccNarrowBlocks) t = kColaccNarrowBlocks;
            const int64_t len = ceil_div(m > n ? m : n, (int64_t)full) * full;
            return align_up((size_t)(t + t / 2) * (size_t)len * (size_t)elem_size, 256);
        }
        case MXB_TRMV: {
            const size_t a = align_up((size_t)n * elem_size, 256),
                         b = tri_workspace_bound(n, elem_size, raw(MXB_OPT_SYMV_TARGET_BLOCKS), raw(MXB_OPT_SYMV_TILE_VECTORS), opt(MXB_OPT_TRI_DIAG_WEIGHT));
            return a > b ? a : b;
        }
        case MXB_SYMV:
            return tri_workspace_bound(n, elem_size, raw(MXB_OPT_SYMV_TARGET_BLOCKS), raw(MXB_OPT_SYMV_TILE_VECTORS), opt(MXB_OPT_TRI_DIAG_WEIGHT));
        case MXB_TRSV: {
            // blocked: the transposed product's partial vectors; chained: 8 (fp32) or 16 (fp64) bytes per
            // unknown of whole sub-blocks of 64, and two counters
            const size_t a = colacc_bound(n, n), b = align_up((size_t)ceil_div(n, (int64_t)64) * 64 * 16 + 8, 256);
            return a > b ? a : b;
        }
        default: return 0;
    }
}

int mxb_probe_copy(mxb_handle_t h, size_t bytes, const void* src, void* dst)
{
    using namespace mxb;
    if (!handle_ok(h)) return MXB_ERR_HANDLE;
    if (bytes % 16 != 0 || !aligned16(src) || !aligned16(dst)) return -1;
    if (bytes == 0) return MXB_OK;
    if (!src) return -2;
    if (!dst) return -3;
    const int64_t nvec = (int64_t)(bytes / 16), ntiles = ceil_div(nvec, kThreads * kUnroll);
    const int64_t cap = kCUs * option(h, MXB_OPT_L1_BLOCKS_PER_CU);
    hipLaunchKernelGGL(probe_copy_kernel, dim3((unsigned)(ntiles < cap ? ntiles : cap)), dim3(kThreads), 0, h->stream, nvec,
                       ntiles, stream_tiles_2d(nvec, kUnroll), static_cast<const f4*>(src), static_cast<f4*>(dst));
    return launch_status();
}

int mxb_probe_read(mxb_handle_t h, size_t bytes, const void* src)
{
    using namespace mxb;
    if (!handle_ok(h)) return MXB_ERR_HANDLE;
    if (bytes % 16 != 0 || !aligned16(src)) return -1;
    if (bytes == 0) return MXB_OK;
    if (!src) return -2;
    const int64_t nvec = (int64_t)(bytes / 16), ntiles = ceil_div(nvec, kThreads * kUnroll);
    const int64_t grid = ntiles < kProbeReadBlocks ? ntiles : kProbeReadBlocks;
    double* sums = static_cast<double*>(take_workspace(h, (size_t)grid * sizeof(double)));
    if (!sums) return MXB_ERR_WORKSPACE;
    hipLaunchKernelGGL(probe_read_kernel, dim3((unsigned)grid), dim3(kThreads), 0, h->stream, nvec, ntiles,
                       static_cast<const f4*>(src), sums);
    return launch_status();
}
}
