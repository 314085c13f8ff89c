// Level-1 kernels (Sec. 6.2.1): axpy, scal (streaming) and dot, asum, nrm2 (reductions).
//
// The paper's recipe for these single-loop kernels is vector lanes plus loop interleaving, with
// per-lane partial sums for the reductions.  On gfx950 the same idea reads: every lane moves
// 128 bits per load, each thread keeps kUnroll independent loads in flight (the interleave
// factor), reductions keep per-lane partial sums in registers, fold them across the wavefront
// with DPP, across the block through LDS, and across blocks in a second, single-block kernel
// that adds the per-block partials in a fixed order (no atomics).
#include "common.hpp"
#include "options.hpp"

namespace mxb {
namespace {

constexpr int kThreads = 256;
constexpr int kUnroll = 4;      // independent 128-bit loads per thread and array
constexpr int kScalUnroll = 2;  // scal reads and writes the same lines: shorter batches stream better

// ---------------------------------------------------------------------------------------------
// streaming: axpy / scal on contiguous data (any base address: 128-bit accesses at element alignment)

// Tiles of kThreads*U vectors (shaped by stream_tile).  Whole tiles carry no predicate, so that
// all loads of a tile are issued back to back; the ragged rest (fewer than one tile of vectors,
// then fewer than VEC elements) is handled by the last block, one vector resp. one element per thread.
template <typename T, bool KEEP>
__global__ void __launch_bounds__(kThreads) axpy_vec_kernel(int64_t nvec, int64_t nfull, int64_t n2d, int tail, T alpha,
                                                            const T* __restrict__ x, T* __restrict__ y)
{
    constexpr int VEC = Full<T>::vec;
    constexpr int U = kUnroll;
    typedef typename VecOf<T, VEC>::type V;
    for (int64_t t = blockIdx.x; t < nfull; t += gridDim.x) {
        int64_t base, step;
        stream_tile<U>(t, n2d, base, step);
        V a[U], b[U];
#pragma unroll
        for (int u = 0; u < U; ++u) a[u] = ld_matrix_as<T, VEC, KEEP>(x + (base + u * step) * VEC);
#pragma unroll
        for (int u = 0; u < U; ++u) b[u] = ld_matrix_as<T, VEC, KEEP>(y + (base + u * step) * VEC);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int k = 0; k < VEC; ++k) b[u][k] = fmad(alpha, a[u][k], b[u][k]);
            st_matrix<T, VEC>(y + (base + u * step) * VEC, b[u]);
        }
    }
    if (blockIdx.x != gridDim.x - 1) return;
    for (int64_t i = nfull * (kThreads * U) + threadIdx.x; i < nvec; i += kThreads) {
        V b = ld_matrix_as<T, VEC, KEEP>(y + i * VEC);
        const V a = ld_matrix_as<T, VEC, KEEP>(x + i * VEC);
#pragma unroll
        for (int k = 0; k < VEC; ++k) b[k] = fmad(alpha, a[k], b[k]);
        st_matrix<T, VEC>(y + i * VEC, b);
    }
    if ((int)threadIdx.x < tail) {
        const int64_t i = nvec * VEC + threadIdx.x;
        y[i] = fmad(alpha, x[i], y[i]);
    }
}

template <typename T, bool KEEP>
__global__ void __launch_bounds__(kThreads) scal_vec_kernel(int64_t nvec, int64_t nfull, int64_t n2d, int tail, T alpha,
                                                            T* __restrict__ x)
{
    constexpr int VEC = Full<T>::vec;
    constexpr int U = kScalUnroll;
    typedef typename VecOf<T, VEC>::type V;
    for (int64_t t = blockIdx.x; t < nfull; t += gridDim.x) {
        int64_t base, step;
        stream_tile<U>(t, n2d, base, step);
        V a[U];
#pragma unroll
        for (int u = 0; u < U; ++u) a[u] = ld_matrix_as<T, VEC, KEEP>(x + (base + u * step) * VEC);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int k = 0; k < VEC; ++k) a[u][k] = alpha * a[u][k];
            st_matrix<T, VEC>(x + (base + u * step) * VEC, a[u]);
        }
    }
    if (blockIdx.x != gridDim.x - 1) return;
    for (int64_t i = nfull * (kThreads * U) + threadIdx.x; i < nvec; i += kThreads) {
        V a = ld_matrix_as<T, VEC, KEEP>(x + i * VEC);
#pragma unroll
        for (int k = 0; k < VEC; ++k) a[k] = alpha * a[k];
        st_matrix<T, VEC>(x + i * VEC, a);
    }
    if ((int)threadIdx.x < tail) {
        const int64_t i = nvec * VEC + threadIdx.x;
        x[i] = alpha * x[i];
    }
}

// streaming with arbitrary increments: one element per lane and load,
// 64-bit offsets because a strided fp64 vector of 2^28 elements spans more than 4 GiB.  Tiles of
// kThreads*kStridedUnroll logical elements; whole tiles carry no predicate, the last block takes
// the ragged rest.
constexpr int kStridedUnroll = 8;

template <typename T>
__global__ void __launch_bounds__(kThreads) axpy_strided_kernel(int64_t n, int64_t nfull, T alpha, const T* __restrict__ x,
                                                                int64_t incx, T* __restrict__ y, int64_t incy)
{
    constexpr int U = kStridedUnroll;
    for (int64_t t = blockIdx.x; t < nfull; t += gridDim.x) {
        const int64_t base = t * (kThreads * U) + threadIdx.x;
        T a[U], b[U];
#pragma unroll
        for (int u = 0; u < U; ++u) a[u] = ld_stream(x + (base + u * kThreads) * incx);
#pragma unroll
        for (int u = 0; u < U; ++u) b[u] = y[(base + u * kThreads) * incy];   // plain load: the line is written next and should stay in L2
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < U; ++u) y[(base + u * kThreads) * incy] = fmad(alpha, a[u], b[u]);
    }
    if (blockIdx.x != gridDim.x - 1) return;
    for (int64_t i = nfull * (kThreads * U) + threadIdx.x; i < n; i += kThreads) y[i * incy] = fmad(alpha, x[i * incx], y[i * incy]);
}

template <typename T>
__global__ void __launch_bounds__(kThreads) scal_strided_kernel(int64_t n, int64_t nfull, T alpha, T* __restrict__ x, int64_t incx)
{
    constexpr int U = kStridedUnroll;
    for (int64_t t = blockIdx.x; t < nfull; t += gridDim.x) {
        const int64_t base = t * (kThreads * U) + threadIdx.x;
        T a[U];
#pragma unroll
        for (int u = 0; u < U; ++u) a[u] = x[(base + u * kThreads) * incx];   // plain load: the line is written next and should stay in L2
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < U; ++u) x[(base + u * kThreads) * incx] = alpha * a[u];
    }
    if (blockIdx.x != gridDim.x - 1) return;
    for (int64_t i = nfull * (kThreads * U) + threadIdx.x; i < n; i += kThreads) x[i * incx] = alpha * x[i * incx];
}

// ---------------------------------------------------------------------------------------------
// reductions

enum { OP_DOT = 0, OP_ASUM = 1, OP_NRM2 = 2, OP_DSDOT = 3 };

// Up to this many tiles one block does everything (a second launch costs more than a few tiles).
constexpr int64_t kSingleBlockTiles = 4;

// Constants of Blue's scaled sum of squares for fp64 (as restated by Anderson, "Safe scaling in
// the level 1 BLAS", 2017): values above kBig are scaled down, values below kSmall are scaled up,
// so that no square overflows or underflows; the rest is summed as is.
constexpr double kTSmall = 0x1p-511, kTBig = 0x1p+486, kSSmall = 0x1p+537, kSBig = 0x1p-538;

// Per-thread running sums.  K = number of doubles a block hands to the second pass.
template <typename T, int OP> struct Acc;

template <> struct Acc<float, OP_DOT> {
    static constexpr int K = 1;
    float s = 0.f;
    __device__ __forceinline__ void add(float x, float y) { s = __builtin_fmaf(x, y, s); }
    __device__ __forceinline__ void get(double* o) const { o[0] = (double)s; }
};
template <> struct Acc<double, OP_DOT> {
    static constexpr int K = 1;
    double s = 0.0;
    __device__ __forceinline__ void add(double x, double y) { s = fmad(x, y, s); }
    __device__ __forceinline__ void get(double* o) const { o[0] = s; }
};
template <> struct Acc<float, OP_DSDOT> {   // fp32 inputs, exact fp64 products, fp64 sum
    static constexpr int K = 1;
    double s = 0.0;
    __device__ __forceinline__ void add(float x, float y) { s = fmad((double)x, (double)y, s); }
    __device__ __forceinline__ void get(double* o) const { o[0] = s; }
};
template <> struct Acc<float, OP_ASUM> {
    static constexpr int K = 1;
    float s = 0.f;
    __device__ __forceinline__ void add(float x, float) { s += __builtin_fabsf(x); }
    __device__ __forceinline__ void get(double* o) const { o[0] = (double)s; }
};
template <> struct Acc<double, OP_ASUM> {
    static constexpr int K = 1;
    double s = 0.0;
    __device__ __forceinline__ void add(double x, double) { s += __builtin_fabs(x); }
    __device__ __forceinline__ void get(double* o) const { o[0] = s; }
};
template <> struct Acc<float, OP_NRM2> {   // squares of floats are exact and cannot overflow in fp64
    static constexpr int K = 1;
    double s = 0.0;
    __device__ __forceinline__ void add(float x, float) { const double d = (double)x; s = fmad(d, d, s); }
    __device__ __forceinline__ void get(double* o) const { o[0] = s; }
};
template <> struct Acc<double, OP_NRM2> {
    static constexpr int K = 3;
    double med = 0.0, big = 0.0, sml = 0.0;
    __device__ __forceinline__ void add(double x, double)
    {
        const double ax = __builtin_fabs(x);
        const bool is_big = ax > kTBig, is_sml = ax < kTSmall;
        const double m = (is_big || is_sml) ? 0.0 : ax;   // NaN compares false twice: goes to med
        const double b = is_big ? ax * kSBig : 0.0;
        const double s = is_sml ? ax * kSSmall : 0.0;
        med = fmad(m, m, med);
        big = fmad(b, b, big);
        sml = fmad(s, s, sml);
    }
    __device__ __forceinline__ void get(double* o) const { o[0] = med; o[1] = big; o[2] = sml; }
};

template <typename T, int OP, typename RES> __device__ __forceinline__ void finish(const double* v, RES* __restrict__ result);

// Folds the block's running sums.  A grid of several blocks hands them to the second pass; a
// grid of one block (short vectors, where a second launch would double the latency) finishes
// the result itself.
template <typename T, int OP, typename RES>
__device__ __forceinline__ void block_partial(const Acc<T, OP>* acc, int nacc, double* __restrict__ partials, RES* __restrict__ result)
{
    constexpr int K = Acc<T, OP>::K;
    __shared__ double slots[kThreads / kWave];
    double v[K];
#pragma unroll
    for (int k = 0; k < K; ++k) v[k] = 0.0;
    for (int a = 0; a < nacc; ++a) {
        double t[K];
        acc[a].get(t);
#pragma unroll
        for (int k = 0; k < K; ++k) v[k] += t[k];
    }
#pragma unroll
    for (int k = 0; k < K; ++k) v[k] = block_sum<kThreads / kWave>(v[k], slots);
    if (threadIdx.x != 0) return;
    if (gridDim.x == 1) {
        finish<T, OP, RES>(v, result);
    } else {
#pragma unroll
        for (int k = 0; k < K; ++k) partials[(int64_t)blockIdx.x * K + k] = v[k];
    }
}

// pass 1 on contiguous data: whole tiles without predicates, the ragged rest by the
// last block.
template <typename T, int OP, typename RES, bool KEEP>
__global__ void __launch_bounds__(kThreads) reduce_vec_kernel(int64_t nvec, int64_t nfull, int tail,
                                                              const T* __restrict__ x, const T* __restrict__ y,
                                                              double* __restrict__ partials, RES* __restrict__ result)
{
    constexpr int VEC = Full<T>::vec;
    constexpr bool TWO = OP == OP_DOT || OP == OP_DSDOT;
    constexpr int U = TWO ? kUnroll : 2 * kUnroll;      // 8 loads in flight per thread either way
    typedef typename VecOf<T, VEC>::type V;
    Acc<T, OP> acc[VEC];
    for (int64_t t = blockIdx.x; t < nfull; t += gridDim.x) {
        const int64_t base = t * (kThreads * U) + threadIdx.x;
        V a[U], b[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            a[u] = ld_matrix_as<T, VEC, KEEP>(x + (base + u * kThreads) * VEC);
            b[u] = TWO ? ld_matrix_as<T, VEC, KEEP>(y + (base + u * kThreads) * VEC) : V(T(0));
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int k = 0; k < VEC; ++k) acc[k].add(a[u][k], b[u][k]);
    }
    if (blockIdx.x == gridDim.x - 1) {
        for (int64_t i = nfull * (kThreads * U) + threadIdx.x; i < nvec; i += kThreads) {
            const V a = ld_matrix_as<T, VEC, KEEP>(x + i * VEC);
            const V b = TWO ? ld_matrix_as<T, VEC, KEEP>(y + i * VEC) : V(T(0));
#pragma unroll
            for (int k = 0; k < VEC; ++k) acc[k].add(a[k], b[k]);
        }
        if ((int)threadIdx.x < tail) {
            const int64_t i = nvec * VEC + threadIdx.x;
            acc[0].add(x[i], TWO ? y[i] : T(0));
        }
    }
    block_partial<T, OP, RES>(acc, VEC, partials, result);
}

// pass 1 with arbitrary increments
template <typename T, int OP, typename RES>
__global__ void __launch_bounds__(kThreads) reduce_strided_kernel(int64_t n, int64_t nfull, const T* __restrict__ x, int64_t incx,
                                                                  const T* __restrict__ y, int64_t incy,
                                                                  double* __restrict__ partials, RES* __restrict__ result)
{
    constexpr bool TWO = OP == OP_DOT || OP == OP_DSDOT;
    constexpr int U = kStridedUnroll;
    constexpr int NACC = 4;
    Acc<T, OP> acc[NACC];
    for (int64_t t = blockIdx.x; t < nfull; t += gridDim.x) {
        const int64_t base = t * (kThreads * U) + threadIdx.x;
        T a[U], b[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            a[u] = ld_stream(x + (base + u * kThreads) * incx);
            b[u] = TWO ? ld_stream(y + (base + u * kThreads) * incy) : T(0);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < U; ++u) acc[u % NACC].add(a[u], b[u]);
    }
    if (blockIdx.x == gridDim.x - 1)
        for (int64_t i = nfull * (kThreads * U) + threadIdx.x; i < n; i += kThreads) acc[0].add(x[i * incx], TWO ? y[i * incy] : T(0));
    block_partial<T, OP, RES>(acc, NACC, partials, result);
}

// Turns the K sums of a reduction into its result (thread 0 of the last pass).
template <typename T, int OP, typename RES>
__device__ __forceinline__ void finish(const double* v, RES* __restrict__ result)
{
    constexpr int K = Acc<T, OP>::K;
    if constexpr (OP != OP_NRM2) {
        *result = (RES)v[0];
    } else if constexpr (K == 1) {
        *result = (RES)__builtin_sqrt(v[0]);
    } else {
        double med = v[0], big = v[1], sml = v[2], r;
        if (big > 0.0) {
            // fold the mid-range sum into the scaled-down one (also carries a NaN across)
            if (med > 0.0 || med != med) big += (med * kSBig) * kSBig;
            r = __builtin_sqrt(big) / kSBig;
        } else if (sml > 0.0) {
            if (med > 0.0 || med != med) {
                const double a = __builtin_sqrt(med), b = __builtin_sqrt(sml) / kSSmall;
                const double lo = a < b ? a : b, hi = a < b ? b : a;
                r = hi * __builtin_sqrt(1.0 + (lo / hi) * (lo / hi));
            } else {
                r = __builtin_sqrt(sml) / kSSmall;
            }
        } else {
            r = __builtin_sqrt(med);
        }
        *result = r;
    }
}

// pass 2: one block adds the per-block partials in a fixed order and finishes the result.
template <typename T, int OP, typename RES>
__global__ void __launch_bounds__(kThreads) reduce_final_kernel(int nparts, const double* __restrict__ partials,
                                                                RES* __restrict__ result)
{
    constexpr int K = Acc<T, OP>::K;
    __shared__ double slots[kThreads / kWave];
    double v[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        double s = 0.0;
        for (int p = threadIdx.x; p < nparts; p += kThreads) s += partials[(int64_t)p * K + k];
        v[k] = block_sum<kThreads / kWave>(s, slots);
    }
    if (threadIdx.x == 0) finish<T, OP, RES>(v, result);
}

template <typename T>
__global__ void store_scalar_kernel(T* p, T v) { *p = v; }

// ---------------------------------------------------------------------------------------------
// host side

template <typename T>
int axpy(mxb_handle_t h, int64_t n, T alpha, const T* x, int64_t incx, T* y, int64_t incy)
{
    if (!handle_ok(h)) return MXB_ERR_HANDLE;
    if (n < 0) return -1;
    if (n == 0 || alpha == T(0)) return MXB_OK;
    if (!x) return -3;
    if (incx == 0) return -4;
    if (!y) return -5;
    if (incy == 0) return -6;
    constexpr int VEC = Full<T>::vec;
    const int64_t bpc = option(h, MXB_OPT_L1_BLOCKS_PER_CU);
    if (incx == 1 && incy == 1) {   // any base address: the vector accesses need element alignment only
        const int64_t nvec = n / VEC;
        const int64_t nfull = nvec / (kThreads * kUnroll);
        const int64_t grid = nfull < 1 ? 1 : (nfull < kCUs * bpc ? nfull : kCUs * bpc);
        if (keeps_vectors(2 * n * (int64_t)sizeof(T)))
            hipLaunchKernelGGL((axpy_vec_kernel<T, true>), dim3((unsigned)grid), dim3(kThreads), 0, h->stream, nvec, nfull,
                               stream_tiles_2d(nvec, kUnroll), (int)(n % VEC), alpha, x, y);
        else
            hipLaunchKernelGGL((axpy_vec_kernel<T, false>), dim3((unsigned)grid), dim3(kThreads), 0, h->stream, nvec, nfull,
                               stream_tiles_2d(nvec, kUnroll), (int)(n % VEC), alpha, x, y);
    } else {
        const int64_t nfull = n / (kThreads * kStridedUnroll);
        const int64_t grid = nfull < 1 ? 1 : (nfull < kCUs * bpc ? nfull : kCUs * bpc);
        hipLaunchKernelGGL(axpy_strided_kernel<T>, dim3((unsigned)grid), dim3(kThreads), 0, h->stream, n, nfull, alpha,
                           vec_base(x, n, incx), incx, vec_base(y, n, incy), incy);
    }
    return launch_status();
}

template <typename T>
int scal(mxb_handle_t h, int64_t n, T alpha, T* x, int64_t incx)
{
    if (!handle_ok(h)) return MXB_ERR_HANDLE;
    if (n < 0) return -1;
    if (n == 0 || incx <= 0) return MXB_OK;
    if (!x) return -3;
    constexpr int VEC = Full<T>::vec;
    const int64_t bpc = option(h, MXB_OPT_L1_BLOCKS_PER_CU);
    if (incx == 1) {   // any base address: the vector accesses need element alignment only
        const int64_t nvec = n / VEC;
        const int64_t nfull = nvec / (kThreads * kScalUnroll);
        const int64_t grid = nfull < 1 ? 1 : (nfull < kCUs * bpc ? nfull : kCUs * bpc);
        if (keeps_vectors(n * (int64_t)sizeof(T)))
            hipLaunchKernelGGL((scal_vec_kernel<T, true>), dim3((unsigned)grid), dim3(kThreads), 0, h->stream, nvec, nfull,
                               stream_tiles_2d(nvec, kScalUnroll), (int)(n % VEC), alpha, x);
        else
            hipLaunchKernelGGL((scal_vec_kernel<T, false>), dim3((unsigned)grid), dim3(kThreads), 0, h->stream, nvec, nfull,
                               stream_tiles_2d(nvec, kScalUnroll), (int)(n % VEC), alpha, x);
    } else {
        const int64_t nfull = n / (kThreads * kStridedUnroll);
        const int64_t grid = nfull < 1 ? 1 : (nfull < kCUs * bpc ? nfull : kCUs * bpc);
        hipLaunchKernelGGL(scal_strided_kernel<T>, dim3((unsigned)grid), dim3(kThreads), 0, h->stream, n, nfull, alpha, x, incx);
    }
    return launch_status();
}

// x, y already checked.  y == nullptr for the one-vector ops.
template <typename T, int OP, typename RES = T>
int reduce(mxb_handle_t h, int64_t n, const T* x, int64_t incx, const T* y, int64_t incy, RES* result)
{
    constexpr bool TWO = OP == OP_DOT || OP == OP_DSDOT;
    constexpr int VEC = Full<T>::vec;
    constexpr int K = Acc<T, OP>::K;
    const bool empty = n == 0 || (!TWO && incx <= 0);
    if (empty) {
        hipLaunchKernelGGL(store_scalar_kernel<RES>, dim3(1), dim3(1), 0, h->stream, result, RES(0));
        return launch_status();
    }
    const bool contiguous = incx == 1 && (!TWO || incy == 1);   // any base address: element alignment suffices
    // One block per compute unit with 16 vector loads in flight per lane reads fastest; a single
    // strided operand, one element per lane and load, wants eight times as many blocks (measured).
    const int64_t max_blocks = option(h, MXB_OPT_REDUCE_BLOCKS) * ((contiguous || TWO) ? 1 : kStridedBlocksFactor);
    double* partials = static_cast<double*>(take_workspace(h, (size_t)max_blocks * K * sizeof(double)));
    if (!partials) return MXB_ERR_WORKSPACE;
    int64_t grid;
    if (contiguous) {
        const int64_t nvec = n / VEC;
        const int64_t nfull = nvec / (kThreads * (TWO ? kUnroll : 2 * kUnroll));
        grid = nfull <= kSingleBlockTiles ? 1 : (nfull < max_blocks ? nfull : max_blocks);
        if (keeps_vectors((TWO ? 2 : 1) * n * (int64_t)sizeof(T)))
            hipLaunchKernelGGL((reduce_vec_kernel<T, OP, RES, true>), dim3((unsigned)grid), dim3(kThreads), 0, h->stream, nvec, nfull,
                               (int)(n % VEC), x, y, partials, result);
        else
            hipLaunchKernelGGL((reduce_vec_kernel<T, OP, RES, false>), dim3((unsigned)grid), dim3(kThreads), 0, h->stream, nvec, nfull,
                               (int)(n % VEC), x, y, partials, result);
    } else {
        const int64_t nfull = n / (kThreads * kStridedUnroll);
        grid = nfull <= kSingleBlockTiles ? 1 : (nfull < max_blocks ? nfull : max_blocks);
        hipLaunchKernelGGL((reduce_strided_kernel<T, OP, RES>), dim3((unsigned)grid), dim3(kThreads), 0, h->stream, n, nfull,
                           vec_base(x, n, incx), incx, y ? vec_base(y, n, incy) : nullptr, incy, partials, result);
    }
    int st = launch_status();
    if (st != MXB_OK || grid == 1) return st;      // a single block has written the result itself
    hipLaunchKernelGGL((reduce_final_kernel<T, OP, RES>), dim3(1), dim3(kThreads), 0, h->stream, (int)grid, partials, result);
    return launch_status();
}

template <typename T, int OP = OP_DOT, typename RES = T>
int dot(mxb_handle_t h, int64_t n, const T* x, int64_t incx, const T* y, int64_t incy, RES* result)
{
    if (!handle_ok(h)) return MXB_ERR_HANDLE;
    if (n < 0) return -1;
    if (!result) return -6;
    if (n > 0) {
        if (!x) return -2;
        if (incx == 0) return -3;
        if (!y) return -4;
        if (incy == 0) return -5;
    }
    return reduce<T, OP, RES>(h, n, x, incx, y, incy, result);
}

template <typename T, int OP>
int one_vector(mxb_handle_t h, int64_t n, const T* x, int64_t incx, T* result)
{
    if (!handle_ok(h)) return MXB_ERR_HANDLE;
    if (n < 0) return -1;
    if (!result) return -4;
    if (n > 0 && incx > 0 && !x) return -2;
    return reduce<T, OP>(h, n, x, incx, nullptr, 0, result);
}


// ---------------------------------------------------------------------------------------------
// iamax: index of the first element of largest magnitude.  A candidate is (|x|, index); the
// better of two has the larger magnitude or, at equal magnitude, the smaller index, which makes
// the result independent of how the elements are split over lanes and blocks.  NaN never compares
// greater, so it is mapped to -1 (below every magnitude); the reference scan keeps index 0 when
// x[0] is NaN, and the final kernel restores exactly that.
struct Cand {
    double v;
    int64_t i;
};
__device__ __forceinline__ Cand better(Cand a, Cand b) { return (b.v > a.v || (b.v == a.v && b.i < a.i)) ? b : a; }

template <typename T>
__device__ __forceinline__ Cand cand_of(T x, int64_t i)
{
    const double a = (double)(x < T(0) ? -x : x);
    return Cand{a == a ? a : -1.0, i};
}

__device__ __forceinline__ Cand block_best(Cand c, Cand* slots)
{
    // One barrier: every lane of the first wavefront takes the candidates of its own lane number in all
    // wavefronts, then the wavefront folds its 64 through shuffles.  `better` is a total order, so the
    // result does not depend on the shape of the tree.  Valid in the first wavefront only.
    // (a tree through LDS with a barrier per level: 65536 elements 6.5 us per call instead of 5.4, 100 elements
    // 3.5 instead of 2.8)
    slots[threadIdx.x] = c;
    __syncthreads();
    if (threadIdx.x >= kWave) return c;
#pragma unroll
    for (int w = 1; w < kThreads / kWave; ++w) c = better(c, slots[w * kWave + threadIdx.x]);
#pragma unroll
    for (int m = kWave / 2; m > 0; m >>= 1) {
        Cand o;
        o.v = __shfl_xor(c.v, m);
        o.i = (int64_t)__shfl_xor((long long)c.i, m);
        c = better(c, o);
    }
    return c;
}

template <typename T>
__global__ void __launch_bounds__(kThreads) iamax_kernel(int64_t n, int64_t nfull, const T* __restrict__ x, int64_t incx,
                                                         Cand* __restrict__ partials, int64_t* __restrict__ result)
{
    constexpr int U = kStridedUnroll;
    __shared__ Cand slots[kThreads];
    Cand best{-2.0, 0};
    for (int64_t t = blockIdx.x; t < nfull; t += gridDim.x) {
        const int64_t base = t * (kThreads * U) + threadIdx.x;
        T a[U];
#pragma unroll
        for (int u = 0; u < U; ++u) a[u] = ld_stream(x + (base + u * kThreads) * incx);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < U; ++u) best = better(best, cand_of(a[u], base + u * kThreads));
    }
    if (blockIdx.x == gridDim.x - 1)
        for (int64_t i = nfull * (kThreads * U) + threadIdx.x; i < n; i += kThreads) best = better(best, cand_of(x[i * incx], i));
    const Cand b = block_best(best, slots);
    if (threadIdx.x == 0) {
        if (result) {                      // the only block: no second pass
            const T x0 = x[0];
            *result = (x0 != x0) ? 0 : b.i;
        } else {
            partials[blockIdx.x] = b;
        }
    }
}

// The same on contiguous data: 128-bit loads at element alignment, whole tiles without predicates,
// the vectors after the last whole tile and the elements after the last whole vector by the last
// block (one element per lane and load moves 32 MiB at 1.6 TB/s).
template <typename T, bool KEEP>
__global__ void __launch_bounds__(kThreads) iamax_vec_kernel(int64_t n, int64_t nvec, int64_t nfull, const T* __restrict__ x,
                                                             Cand* __restrict__ partials, int64_t* __restrict__ result)
{
    constexpr int VEC = Full<T>::vec;
    constexpr int U = 2 * kUnroll;
    typedef typename VecOf<T, VEC>::type V;
    __shared__ Cand slots[kThreads];
    // One running best per vector element and parity of the load, in the element's own type: 2 * VEC
    // independent chains instead of one chain of 64-bit candidates through every element.  Inside a
    // chain the indices only grow, so "strictly greater" keeps the first of equal magnitudes.
    T bv[2][VEC];
    int64_t bi[2][VEC];
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int k = 0; k < VEC; ++k) { bv[c][k] = T(-2); bi[c][k] = 0; }
    auto take = [&](int c, int k, T v, int64_t i) {
        T a = v < T(0) ? -v : v;
        a = a == a ? a : T(-1);          // NaN never wins
        const bool up = a > bv[c][k];
        bv[c][k] = up ? a : bv[c][k];
        bi[c][k] = up ? i : bi[c][k];
    };
    for (int64_t t = blockIdx.x; t < nfull; t += gridDim.x) {
        const int64_t base = t * (kThreads * U) + threadIdx.x;
        V a[U];
#pragma unroll
        for (int u = 0; u < U; ++u) a[u] = ld_matrix_as<T, VEC, KEEP>(x + (base + u * kThreads) * VEC);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int k = 0; k < VEC; ++k) take(u & 1, k, a[u][k], (base + u * kThreads) * VEC + k);
    }
    if (blockIdx.x == gridDim.x - 1) {
        for (int64_t v = nfull * (kThreads * U) + threadIdx.x; v < nvec; v += kThreads) {
            const V a = ld_matrix_as<T, VEC, KEEP>(x + v * VEC);
#pragma unroll
            for (int k = 0; k < VEC; ++k) take(0, k, a[k], v * VEC + k);
        }
        const int64_t i = nvec * VEC + threadIdx.x;
        if (i < n) take(0, 0, x[i], i);
    }
    Cand best{-2.0, 0};
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int k = 0; k < VEC; ++k) best = better(best, Cand{(double)bv[c][k], bi[c][k]});
    const Cand b = block_best(best, slots);
    if (threadIdx.x == 0) {
        if (result) {                      // the only block: no second pass
            const T x0 = x[0];
            *result = (x0 != x0) ? 0 : b.i;
        } else {
            partials[blockIdx.x] = b;
        }
    }
}

template <typename T>
__global__ void __launch_bounds__(kThreads) iamax_final_kernel(int nparts, const Cand* __restrict__ partials,
                                                               const T* __restrict__ x, int64_t* __restrict__ result)
{
    __shared__ Cand slots[kThreads];
    Cand best{-2.0, 0};
    for (int p = threadIdx.x; p < nparts; p += kThreads) best = better(best, partials[p]);
    const Cand b = block_best(best, slots);
    if (threadIdx.x == 0) {
        const T x0 = x[0];
        *result = (x0 != x0) ? 0 : b.i;      // a NaN in front wins the reference scan by default
    }
}

template <typename T>
int iamax(mxb_handle_t h, int64_t n, const T* x, int64_t incx, int64_t* result)
{
    if (!handle_ok(h)) return MXB_ERR_HANDLE;
    if (n < 0) return -1;
    if (!result) return -4;
    if (n == 0 || incx <= 0) {
        hipLaunchKernelGGL(store_scalar_kernel<int64_t>, dim3(1), dim3(1), 0, h->stream, result, (int64_t)0);
        return launch_status();
    }
    if (!x) return -2;
    const int64_t max_blocks = option(h, MXB_OPT_REDUCE_BLOCKS);
    // (the contiguous kernel wants two blocks per compute unit: its comparisons take a wavefront long enough that a
    // second one has to keep the loads going meanwhile; n = 2^28: 5.8 -> 6.7 TB/s)
    Cand* partials = static_cast<Cand*>(take_workspace(h, (size_t)(2 * max_blocks) * sizeof(Cand)));
    if (!partials) return MXB_ERR_WORKSPACE;
    int64_t grid;
    if (incx == 1) {   // any base address: element alignment suffices
        constexpr int VEC = Full<T>::vec;
        const int64_t nvec = n / VEC, nfull = nvec / (kThreads * 2 * kUnroll);
        grid = nfull <= kSingleBlockTiles ? 1 : (nfull < 2 * max_blocks ? nfull : 2 * max_blocks);
        if (keeps_vectors(n * (int64_t)sizeof(T)))
            hipLaunchKernelGGL((iamax_vec_kernel<T, true>), dim3((unsigned)grid), dim3(kThreads), 0, h->stream, n, nvec, nfull, x, partials, grid == 1 ? result : nullptr);
        else
            hipLaunchKernelGGL((iamax_vec_kernel<T, false>), dim3((unsigned)grid), dim3(kThreads), 0, h->stream, n, nvec, nfull, x, partials, grid == 1 ? result : nullptr);
    } else {
        const int64_t nfull = n / (kThreads * kStridedUnroll);
        grid = nfull <= kSingleBlockTiles ? 1 : (nfull < max_blocks ? nfull : max_blocks);
        hipLaunchKernelGGL(iamax_kernel<T>, dim3((unsigned)grid), dim3(kThreads), 0, h->stream, n, nfull, x, incx, partials, grid == 1 ? result : nullptr);
    }
    int st = launch_status();
    if (st != MXB_OK || grid == 1) return st;      // a single block has written the result itself
    hipLaunchKernelGGL(iamax_final_kernel<T>, dim3(1), dim3(kThreads), 0, h->stream, (int)grid, partials, x, result);
    return launch_status();
}

}  // namespace
}  // namespace mxb

extern "C" {
int mxb_saxpy(mxb_handle_t h, int64_t n, float alpha, const float* x, int64_t incx, float* y, int64_t incy)
{ return mxb::axpy<float>(h, n, alpha, x, incx, y, incy); }
int mxb_daxpy(mxb_handle_t h, int64_t n, double alpha, const double* x, int64_t incx, double* y, int64_t incy)
{ return mxb::axpy<double>(h, n, alpha, x, incx, y, incy); }
int mxb_sscal(mxb_handle_t h, int64_t n, float alpha, float* x, int64_t incx) { return mxb::scal<float>(h, n, alpha, x, incx); }
int mxb_dscal(mxb_handle_t h, int64_t n, double alpha, double* x, int64_t incx) { return mxb::scal<double>(h, n, alpha, x, incx); }
int mxb_sdot(mxb_handle_t h, int64_t n, const float* x, int64_t incx, const float* y, int64_t incy, float* r)
{ return mxb::dot<float>(h, n, x, incx, y, incy, r); }
int mxb_ddot(mxb_handle_t h, int64_t n, const double* x, int64_t incx, const double* y, int64_t incy, double* r)
{ return mxb::dot<double>(h, n, x, incx, y, incy, r); }
int mxb_sasum(mxb_handle_t h, int64_t n, const float* x, int64_t incx, float* r)
{ return mxb::one_vector<float, mxb::OP_ASUM>(h, n, x, incx, r); }
int mxb_dasum(mxb_handle_t h, int64_t n, const double* x, int64_t incx, double* r)
{ return mxb::one_vector<double, mxb::OP_ASUM>(h, n, x, incx, r); }
int mxb_snrm2(mxb_handle_t h, int64_t n, const float* x, int64_t incx, float* r)
{ return mxb::one_vector<float, mxb::OP_NRM2>(h, n, x, incx, r); }
int mxb_dnrm2(mxb_handle_t h, int64_t n, const double* x, int64_t incx, double* r)
{ return mxb::one_vector<double, mxb::OP_NRM2>(h, n, x, incx, r); }
int mxb_dsdot(mxb_handle_t h, int64_t n, const float* x, int64_t incx, const float* y, int64_t incy, double* r)
{ return mxb::dot<float, mxb::OP_DSDOT, double>(h, n, x, incx, y, incy, r); }
int mxb_isamax(mxb_handle_t h, int64_t n, const float* x, int64_t incx, int64_t* r) { return mxb::iamax<float>(h, n, x, incx, r); }
int mxb_idamax(mxb_handle_t h, int64_t n, const double* x, int64_t incx, int64_t* r) { return mxb::iamax<double>(h, n, x, incx, r); }
}
