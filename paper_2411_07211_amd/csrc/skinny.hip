// Skinny matrices (Sec. 6.2.2, skinny matrix).  The paper loads the whole short vector into
// registers before the quadratic loop and specialises the code for each register count.  Here a
// row is so short (nv <= 20 vectors of 16 bytes) that a wavefront takes
// G = 64 / nv rows side by side: lane l works on vector k = l % nv of row g = l / nv of the
// wavefront's current G rows, so that the lanes read one contiguous run of G rows (the lanes past
// G*nv idle), and every lane needs just ONE vector of the short operand, which it keeps in
// registers for its whole life.  U such slots are in flight per lane.
//   A*x:      per slot a 4-term dot, then a sum over the nv lanes of each row (ds_bpermute
//             shuffles; the groups are not powers of two, so DPP rows do not fit); a row of more
//             than 32 vectors has the wavefront to itself, and the 8 sums of a tile are folded
//             over all 64 lanes at once (rows_fold);
//   A^t*x:    per lane one running sum per owned column; at the end the G lanes that own the same
//             columns and then the wavefronts of the block are folded through LDS, and a second
//             kernel adds the per-block partial vectors in a fixed order;
//   x*y^t:    a read-modify-write with y's vector in registers.
#include "skinny.hpp"

#include "options.hpp"

namespace mxb {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kSlots = 8;                     // rows in flight per lane
constexpr int64_t kSkinnyBlocksT = 512;       // blocks (= partial vectors) of the transposed product: 256 to 512 measure alike, 128 and 1024 and
                                              // more slower (524288 x 40: 22.0, 18.3, 18.3, 19.6, 22.1 us per call for 128 ... 2048; blocks of 16
                                              // wavefronts: 25 to 43 us)

template <typename T>
struct SkinnyArgs {
    int64_t M;           // rows
    int N;               // columns
    int nv;              // vectors per row = ceil(N / VEC); the last one is moved back to end at N
    int64_t lda;
    int64_t incs, incl;  // increments of the short (length N) and the long (length M) vector
    T alpha, beta;
};

__device__ __forceinline__ float shfl_down(float v, int lane, int off)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute((lane + off) << 2, __builtin_bit_cast(int, v)));
}
__device__ __forceinline__ double shfl_down(double v, int lane, int off)
{
    const uint64_t b = __builtin_bit_cast(uint64_t, v);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_ds_bpermute((lane + off) << 2, (int)(uint32_t)b);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_ds_bpermute((lane + off) << 2, (int)(uint32_t)(b >> 32));
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}

// What a lane works on: vector k of row g (of the wavefront's G rows per slot).  The vector
// starts at column c; when N is not a whole number of vectors the last vector of a row is moved
// back so that it ends at N (rows may start at any element: a matrix access needs element
// alignment only) and its first kmin elements, which the lane before it owns, do not count.
struct LaneMap {
    int lane, G, g, k, c, kmin;
    bool active;
};
__device__ __forceinline__ LaneMap lane_map(int nv, int N, int vec)
{
    LaneMap m;
    m.lane = threadIdx.x & (kWave - 1);
    m.G = kWave / nv;
    m.g = m.lane / nv;
    m.k = m.lane - m.g * nv;
    m.active = m.g < m.G;
    if (!m.active) m.g = m.k = 0;      // idle lanes shadow lane 0: their loads stay in bounds and are discarded
    m.c = m.k * vec < N - vec ? m.k * vec : N - vec;
    m.kmin = m.k * vec - m.c;
    return m;
}

// Rows are dealt in tiles of kSlots*G adjacent rows per wavefront, tiles cyclically to all
// wavefronts of the grid: slot u of a tile holds rows tile*kSlots*G + u*G + g.
// Rows that take more than half a wavefront (33 to 64 vectors): one row per wavefront load, SLOTS
// rows in flight, the lanes past the row idle.  The SLOTS sums of a tile are folded over the
// wavefront all at once and leave one row's sum in each of SLOTS lanes, which load the old y of
// their row with the tile and store the new one: SLOTS adjacent elements of y per tile.
template <typename T, int VEC, bool BETA, int SLOTS, bool KEEP>
__global__ void __launch_bounds__(kThreads) skinny_gemv_n_onerow_kernel(const SkinnyArgs<T> p, const T* __restrict__ A,
                                                                        const T* __restrict__ x, T* __restrict__ y)
{
    typedef typename VecOf<T, VEC>::type V;
    const LaneMap m = lane_map(p.nv, p.N, VEC);
    T xr[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) xr[e] = (m.active && e >= m.kmin) ? x[(int64_t)(m.c + e) * p.incs] : T(0);
    int mine;
    const bool writer = rows_fold_lane<SLOTS>(m.lane, mine);
    const int64_t ntiles = (p.M + SLOTS - 1) / SLOTS;
    const int64_t wave0 = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6), nwaves = (int64_t)gridDim.x * kWaves;
    for (int64_t t = wave0; t < ntiles; t += nwaves) {
        const int64_t tile0 = t * SLOTS;
        V a[SLOTS];
        if (tile0 + SLOTS <= p.M) {      // whole tile: no predicate, so that all loads issue back to back
#pragma unroll
            for (int u = 0; u < SLOTS; ++u) a[u] = ld_matrix_as<T, VEC, KEEP>(A + (tile0 + u) * p.lda + m.c);
        } else {
#pragma unroll
            for (int u = 0; u < SLOTS; ++u) {
                a[u] = V(T(0));
                if (tile0 + u < p.M) a[u] = ld_matrix_as<T, VEC, KEEP>(A + (tile0 + u) * p.lda + m.c);
            }
        }
        const int64_t i = tile0 + mine;
        T yo = T(0);
        if (BETA && writer && i < p.M) yo = y[i * p.incl];
        __builtin_amdgcn_sched_barrier(0);   // every load of the tile is in flight before the first FMA
        T s[SLOTS];
#pragma unroll
        for (int u = 0; u < SLOTS; ++u) {
            s[u] = T(0);
#pragma unroll
            for (int e = 0; e < VEC; ++e) s[u] = fmad(a[u][e], xr[e], s[u]);     // xr is zero where the element does not count
        }
        T v = p.alpha * rows_fold<SLOTS>(s, m.lane);
        if (writer && i < p.M) {
            if (BETA) v = fmad(p.beta, yo, v);
            y[i * p.incl] = v;
        }
    }
}

template <typename T, int VEC, bool BETA, bool KEEP>
__global__ void __launch_bounds__(kThreads) skinny_gemv_n_kernel(const SkinnyArgs<T> p, const T* __restrict__ A,
                                                                 const T* __restrict__ x, T* __restrict__ y)
{
    typedef typename VecOf<T, VEC>::type V;
    // the sums of a tile, in row order: written by the first lane of each row, read back one row per
    // lane, so that y is read and written in whole runs of adjacent elements
    __shared__ T sums[kWaves][kSlots * kWave];
    const LaneMap m = lane_map(p.nv, p.N, VEC);
    T* const mine = sums[threadIdx.x >> 6];
    T xr[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) xr[e] = m.active ? x[(int64_t)(m.c + e) * p.incs] : T(0);
    const int rows_per_tile = kSlots * m.G;
    const int64_t ntiles = (p.M + rows_per_tile - 1) / rows_per_tile;
    const int64_t wave0 = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6), nwaves = (int64_t)gridDim.x * kWaves;
    for (int64_t t = wave0; t < ntiles; t += nwaves) {
        const int64_t tile0 = t * rows_per_tile, row0 = tile0 + m.g;
        V a[kSlots];
        if ((t + 1) * rows_per_tile <= p.M) {      // whole tile: no predicate, so that all loads issue back to back
#pragma unroll
            for (int u = 0; u < kSlots; ++u) a[u] = ld_matrix_as<T, VEC, KEEP>(A + (row0 + (int64_t)u * m.G) * p.lda + m.c);
        } else {
#pragma unroll
            for (int u = 0; u < kSlots; ++u) {
                const int64_t i = row0 + (int64_t)u * m.G;
                a[u] = V(T(0));
                if (i < p.M) a[u] = ld_matrix_as<T, VEC, KEEP>(A + i * p.lda + m.c);
            }
        }
        // the old y of the tile's rows travels with the matrix, 64 adjacent rows per load: read after
        // the sums it would cost a round trip of its own
        T yo[kSlots];
        if (BETA) {
#pragma unroll
            for (int q = 0; q < kSlots; ++q) {
                const int r = q * kWave + m.lane;
                const int64_t i = tile0 + r;
                if (r < rows_per_tile && i < p.M) yo[q] = y[i * p.incl];
            }
        }
        __builtin_amdgcn_sched_barrier(0);   // every load of the tile is in flight before the first FMA
#pragma unroll
        for (int u = 0; u < kSlots; ++u) {
            T s = T(0);
#pragma unroll
            for (int e = 0; e < VEC; ++e) s = e >= m.kmin ? fmad(a[u][e], xr[e], s) : s;
            // sum over the nv lanes of the row: lane k adds lane k+off while that is still in the row
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) {
                if (off < p.nv) {            // wave-uniform
                    const T o = shfl_down(s, m.lane, off);
                    s += (m.k + off < p.nv) ? o : T(0);
                }
            }
            if (m.active && m.k == 0) mine[u * m.G + m.g] = s;
        }
        // the wavefront's own LDS traffic runs in order: only the compiler has to keep it so
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront", "local");
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int q = 0; q < kSlots; ++q) {
            const int r = q * kWave + m.lane;
            const int64_t i = tile0 + r;
            if (r < rows_per_tile && i < p.M) {
                T v = p.alpha * mine[r];
                if (BETA) v = fmad(p.beta, yo[q], v);
                y[i * p.incl] = v;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront", "local");
        __builtin_amdgcn_wave_barrier();
    }
}

template <typename T, int VEC, bool KEEP>
__global__ void __launch_bounds__(kThreads) skinny_gemv_t_kernel(const SkinnyArgs<T> p, const T* __restrict__ A,
                                                                 const T* __restrict__ x, T* __restrict__ partials)
{
    typedef typename VecOf<T, VEC>::type V;
    __shared__ T red[kWaves][kWave][VEC];
    const LaneMap m = lane_map(p.nv, p.N, VEC);
    const int wave = threadIdx.x >> 6;
    T acc[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] = T(0);
    const int64_t rows_per_tile = (int64_t)kSlots * m.G;
    const int64_t ntiles = (p.M + rows_per_tile - 1) / rows_per_tile;
    const int64_t wave0 = (int64_t)blockIdx.x * kWaves + wave, nwaves = (int64_t)gridDim.x * kWaves;
    for (int64_t t = wave0; t < ntiles; t += nwaves) {
        const int64_t row0 = t * rows_per_tile + m.g;
        V a[kSlots];
        T xi[kSlots];
        if ((t + 1) * rows_per_tile <= p.M) {      // whole tile: no predicate
#pragma unroll
            for (int u = 0; u < kSlots; ++u) {
                const int64_t i = row0 + (int64_t)u * m.G;
                a[u] = ld_matrix_as<T, VEC, KEEP>(A + i * p.lda + m.c);
                xi[u] = x[i * p.incl];
            }
        } else {
#pragma unroll
            for (int u = 0; u < kSlots; ++u) {
                const int64_t i = row0 + (int64_t)u * m.G;
                a[u] = V(T(0));
                xi[u] = T(0);
                if (i < p.M) {
                    a[u] = ld_matrix_as<T, VEC, KEEP>(A + i * p.lda + m.c);
                    xi[u] = x[i * p.incl];
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < kSlots; ++u)
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[e] = fmad(a[u][e], xi[u], acc[e]);
    }
    // fold the lanes that own the same columns (g = 0..G-1, in that order), then the wavefronts
#pragma unroll
    for (int e = 0; e < VEC; ++e) red[wave][m.lane][e] = m.active ? acc[e] : T(0);
    __syncthreads();
    for (int j = threadIdx.x; j < p.N; j += kThreads) {
        int k = j / VEC;
        k = k < p.nv - 1 ? k : p.nv - 1;
        const int c = k * VEC < p.N - VEC ? k * VEC : p.N - VEC, e = j - c;     // as in lane_map
        T s = T(0);
        for (int w = 0; w < kWaves; ++w)
            for (int g = 0; g < m.G; ++g) s += red[w][g * p.nv + k][e];
        partials[(int64_t)blockIdx.x * p.N + j] = s;
    }
}

constexpr int kCombineGroups = 16;

// y[j] = alpha * sum_b partials[b][j] + beta*y[j], b ascending; 64 columns per block, 16
// wavefronts each take every 16th partial vector, LDS folds them in wave order.
template <typename T>
__global__ void __launch_bounds__(kCombineGroups* kWave) skinny_combine_kernel(int64_t nparts, int N, const T* __restrict__ partials,
                                                                               T alpha, T beta, T* __restrict__ y, int64_t incy)
{
    __shared__ T red[kCombineGroups][kWave];
    const int tx = threadIdx.x & (kWave - 1), ty = threadIdx.x >> 6;
    const int j = (int)blockIdx.x * kWave + tx;
    T s = T(0);
    if (j < N) {
#pragma unroll 8
        for (int64_t q = ty; q < nparts; q += kCombineGroups) s += partials[q * N + j];
    }
    red[ty][tx] = s;
    __syncthreads();
    if (ty != 0 || j >= N) return;
    T tot = red[0][tx];
#pragma unroll
    for (int k = 1; k < kCombineGroups; ++k) tot += red[k][tx];
    T* yp = y + (int64_t)j * incy;
    T v = alpha * tot;
    if (beta != T(0)) v = fmad(beta, *yp, v);
    *yp = v;
}

template <typename T, int VEC, bool KEEP>
__global__ void __launch_bounds__(kThreads) skinny_ger_kernel(const SkinnyArgs<T> p, T* __restrict__ A, const T* __restrict__ x,
                                                              const T* __restrict__ y)
{
    typedef typename VecOf<T, VEC>::type V;
    const LaneMap m = lane_map(p.nv, p.N, VEC);
    if (!m.active) return;               // no barrier below: idle lanes can leave
    T yr[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) yr[e] = y[(int64_t)(m.c + e) * p.incs];
    const int64_t rows_per_tile = (int64_t)kSlots * m.G;
    const int64_t ntiles = (p.M + rows_per_tile - 1) / rows_per_tile;
    const int64_t wave0 = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6), nwaves = (int64_t)gridDim.x * kWaves;
    for (int64_t t = wave0; t < ntiles; t += nwaves) {
        const int64_t row0 = t * rows_per_tile + m.g;
        V a[kSlots];
        T ax[kSlots];
        if ((t + 1) * rows_per_tile <= p.M) {      // whole tile: no predicate
#pragma unroll
            for (int u = 0; u < kSlots; ++u) {
                const int64_t i = row0 + (int64_t)u * m.G;
                a[u] = ld_matrix_as<T, VEC, KEEP>(A + i * p.lda + m.c);
                ax[u] = p.alpha * x[i * p.incl];
            }
        } else {
#pragma unroll
            for (int u = 0; u < kSlots; ++u) {
                const int64_t i = row0 + (int64_t)u * m.G;
                a[u] = V(T(0));
                ax[u] = T(0);
                if (i < p.M) {
                    a[u] = ld_matrix_as<T, VEC, KEEP>(A + i * p.lda + m.c);
                    ax[u] = p.alpha * x[i * p.incl];
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);   // all loads of the tile are in flight before the first store
#pragma unroll
        for (int u = 0; u < kSlots; ++u) {
            const int64_t i = row0 + (int64_t)u * m.G;
            if (i < p.M) {
#pragma unroll
                for (int e = 0; e < VEC; ++e) a[u][e] = fmad(ax[u], yr[e], a[u][e]);
                T* ap = A + i * p.lda + m.c;
                if (m.kmin == 0) {
                    st_matrix<T, VEC>(ap, a[u]);
                } else {
#pragma unroll
                    for (int e = 1; e < VEC; ++e)
                        if (e >= m.kmin) ap[e] = a[u][e];
                }
            }
        }
    }
}

template <typename T>
SkinnyArgs<T> make_args(int64_t rows, int64_t cols, int vec, int64_t lda, int64_t incs, int64_t incl, T alpha, T beta)
{
    SkinnyArgs<T> a;
    a.M = rows; a.N = (int)cols; a.nv = (int)ceil_div(cols, (int64_t)vec); a.lda = lda; a.incs = incs; a.incl = incl; a.alpha = alpha; a.beta = beta;
    return a;
}

// Grid: one wavefront per tile of kSlots * (64 / nv) rows, capped.
inline int64_t tile_blocks(int64_t rows, int nv, int64_t cap)
{
    const int64_t tiles = ceil_div(rows, (int64_t)kSlots * (kWave / nv));
    const int64_t b = ceil_div(tiles, kWaves);
    return b < cap ? b : cap;
}

// Rows narrower than one 16-byte vector (1 to 3 floats, 1 double) take the same kernels with
// one element per lane: 64, 32 or 21 rows side by side per wavefront load.
#define MXB_SKINNY_DISPATCH_VEC(KERNEL, VEC_, GRID, ...)                                                                         \
    if (keeps_matrix(rows * cols * (int64_t)sizeof(T)))                                                                          \
        hipLaunchKernelGGL((KERNEL<T, VEC_, true>), dim3((unsigned)(GRID)), dim3(kThreads), 0, h->stream, a, __VA_ARGS__);       \
    else                                                                                                                         \
        hipLaunchKernelGGL((KERNEL<T, VEC_, false>), dim3((unsigned)(GRID)), dim3(kThreads), 0, h->stream, a, __VA_ARGS__)
#define MXB_SKINNY_DISPATCH(KERNEL, GRID, ...)                                              \
    if (cols < Full<T>::vec) { MXB_SKINNY_DISPATCH_VEC(KERNEL, 1, GRID, __VA_ARGS__); }     \
    else { MXB_SKINNY_DISPATCH_VEC(KERNEL, Full<T>::vec, GRID, __VA_ARGS__); }

template <typename T>
inline int vec_for(int64_t cols) { return cols < Full<T>::vec ? 1 : Full<T>::vec; }

}  // namespace

size_t skinny_workspace_bytes(int64_t cols, int elem_size)
{
    return align_up((size_t)kSkinnyBlocksT * (size_t)cols * (size_t)elem_size, 256);
}

template <typename T>
int skinny_gemv_n(mxb_handle_t h, int64_t rows, int64_t cols, T alpha, const T* A, int64_t lda, const T* x0, int64_t incx, T beta,
                  T* y0, int64_t incy)
{
    const SkinnyArgs<T> a = make_args<T>(rows, cols, vec_for<T>(cols), lda, incx, incy, alpha, beta);
    if (a.nv > kWave / 2) {
        // one tile of 8 rows per wavefront, or two: many short-lived blocks read this flat stream
        // fastest (1048576 x 256: 2 to 16 blocks per compute unit 166-170 us, 64 and more 160-164)
        constexpr int SLOTS = 8;
        const int64_t blocks = ceil_div(ceil_div(rows, (int64_t)SLOTS), (int64_t)kWaves), cap = (int64_t)kCUs * 64;
        const dim3 g1((unsigned)(blocks < cap ? blocks : cap));
#define MXB_SKINNY_ONEROW(BETA_)                                                                                                              \
    if (keeps_matrix(rows * cols * (int64_t)sizeof(T)))                                                                                       \
        hipLaunchKernelGGL((skinny_gemv_n_onerow_kernel<T, Full<T>::vec, BETA_, SLOTS, true>), g1, dim3(kThreads), 0, h->stream, a, A, x0, y0);  \
    else                                                                                                                                      \
        hipLaunchKernelGGL((skinny_gemv_n_onerow_kernel<T, Full<T>::vec, BETA_, SLOTS, false>), g1, dim3(kThreads), 0, h->stream, a, A, x0, y0)
        if (beta != T(0)) { MXB_SKINNY_ONEROW(true); } else { MXB_SKINNY_ONEROW(false); }
#undef MXB_SKINNY_ONEROW
        return launch_status();
    }
    const dim3 grid((unsigned)tile_blocks(rows, a.nv, (int64_t)kCUs * 16));
#define MXB_SKINNY_N(VEC_, BETA_)                                                                                       \
    if (keeps_matrix(rows * cols * (int64_t)sizeof(T)))                                                                     \
        hipLaunchKernelGGL((skinny_gemv_n_kernel<T, VEC_, BETA_, true>), grid, dim3(kThreads), 0, h->stream, a, A, x0, y0); \
    else                                                                                                                    \
        hipLaunchKernelGGL((skinny_gemv_n_kernel<T, VEC_, BETA_, false>), grid, dim3(kThreads), 0, h->stream, a, A, x0, y0)
    if (cols < Full<T>::vec) {
        if (beta != T(0)) { MXB_SKINNY_N(1, true); } else { MXB_SKINNY_N(1, false); }
    } else {
        if (beta != T(0)) { MXB_SKINNY_N(Full<T>::vec, true); } else { MXB_SKINNY_N(Full<T>::vec, false); }
    }
#undef MXB_SKINNY_N
    return launch_status();
}

template <typename T>
int skinny_gemv_t(mxb_handle_t h, int64_t rows, int64_t cols, T alpha, const T* A, int64_t lda, const T* x0, int64_t incx, T beta,
                  T* y0, int64_t incy)
{
    const SkinnyArgs<T> a = make_args<T>(rows, cols, vec_for<T>(cols), lda, incy, incx, alpha, beta);
    const int64_t blocks = tile_blocks(rows, a.nv, kSkinnyBlocksT);
    T* partials = static_cast<T*>(take_workspace(h, (size_t)blocks * (size_t)cols * sizeof(T)));
    if (!partials) return MXB_ERR_WORKSPACE;
    MXB_SKINNY_DISPATCH(skinny_gemv_t_kernel, blocks, A, x0, partials);
    const int st = launch_status();
    if (st != MXB_OK) return st;
    hipLaunchKernelGGL(skinny_combine_kernel<T>, dim3((unsigned)ceil_div(cols, kWave)), dim3(kCombineGroups * kWave), 0, h->stream, blocks,
                       (int)cols, partials, alpha, beta, y0, incy);
    return launch_status();
}

template <typename T>
int skinny_ger(mxb_handle_t h, int64_t rows, int64_t cols, T alpha, const T* x0, int64_t incx, const T* y0, int64_t incy, T* A,
               int64_t lda)
{
    const SkinnyArgs<T> a = make_args<T>(rows, cols, vec_for<T>(cols), lda, incy, incx, alpha, T(0));
    MXB_SKINNY_DISPATCH(skinny_ger_kernel, tile_blocks(rows, a.nv, (int64_t)kCUs * 16), A, x0, y0);
    return launch_status();
}

#define MXB_SKINNY_INST(T)                                                                                                        \
    template int skinny_gemv_n<T>(mxb_handle_t, int64_t, int64_t, T, const T*, int64_t, const T*, int64_t, T, T*, int64_t);       \
    template int skinny_gemv_t<T>(mxb_handle_t, int64_t, int64_t, T, const T*, int64_t, const T*, int64_t, T, T*, int64_t);       \
    template int skinny_ger<T>(mxb_handle_t, int64_t, int64_t, T, const T*, int64_t, const T*, int64_t, T*, int64_t);
MXB_SKINNY_INST(float)
MXB_SKINNY_INST(double)
#undef MXB_SKINNY_INST

}  // namespace mxb
