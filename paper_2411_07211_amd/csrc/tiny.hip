// Batches of matrices with very short rows (see tiny.hpp).  Not transposed: the row-dot kernel
// gives every problem a block tile of its own and stages x in LDS per tile, which leaves most of a
// block idle when a matrix has a few dozen rows.  Here the rows of all problems form one long
// list: a group of LPR lanes (4, 8 or 16: one DPP quad, half row or row) takes one row with one
// 128-bit load per lane, 64 / LPR rows side by side per wavefront load and U such loads in
// flight; the matching vector of the row's own x comes straight from memory (every x is re-read
// once per row, from cache), the group folds its 4-term dots with DPP and one lane writes y.
#include "tiny.hpp"

namespace mxb {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kSlots = 8;                     // rows in flight per lane group
constexpr int kTinyFewRows = 16;              // transposed: problems of up to this many rows take the lane-per-column-vector kernel

template <typename T>
struct TinyArgs {
    int M, N;            // rows and columns of one problem
    uint32_t total;      // rows of all problems
    const T* A;
    int64_t lda, sA;
    const T* x;
    int64_t incx, sx;
    T* y;
    int64_t incy, sy;
    T alpha, beta;
};

// Sum over a group of LPR adjacent lanes; every lane of the group receives it.
template <int LPR, typename T>
__device__ __forceinline__ T group_sum(T v)
{
    v += dpp_mov<kDppXor1>(v);
    v += dpp_mov<kDppXor2>(v);
    if (LPR >= 8) v += dpp_mov<kDppHalfMirror>(v);
    if (LPR >= 16) v += dpp_mov<kDppMirror>(v);
    return v;
}

template <typename T, int VEC, int LPR, bool BETA>
__global__ void __launch_bounds__(kThreads) tiny_gemv_n_kernel(const TinyArgs<T> p)
{
    typedef typename VecOf<T, VEC>::type V;
    constexpr int G = kWave / LPR;            // rows per wavefront load
    const int lane = threadIdx.x & (kWave - 1);
    const int g = lane / LPR, l = lane % LPR;
    // my columns [c, c + VEC); a vector past the end of the row is moved back to end at N, and only
    // the elements from column c on are mine (none if the row ends before c)
    const int c = l * VEC, cl = min(c, p.N - VEC);
    const uint32_t rows_per_tile = kSlots * G;
    const uint32_t ntiles = (p.total + rows_per_tile - 1) / rows_per_tile;
    const uint32_t wave0 = blockIdx.x * kWaves + (threadIdx.x >> 6), nwaves = gridDim.x * kWaves;
    for (uint32_t t = wave0; t < ntiles; t += nwaves) {
        V a[kSlots], xv[kSlots];
        T yo[kSlots];
        uint32_t b[kSlots], i[kSlots];
#pragma unroll
        for (int u = 0; u < kSlots; ++u) {
            const uint32_t row = min(t * rows_per_tile + u * G + g, p.total - 1);     // clamp: loads stay in bounds
            b[u] = row / (uint32_t)p.M;
            i[u] = row - b[u] * (uint32_t)p.M;
            a[u] = ld_matrix<T, VEC>(p.A + (int64_t)b[u] * p.sA + (int64_t)i[u] * p.lda + cl);
            // the old y travels with the tile: read after the sums, each would cost a round trip of its own
            if (BETA) yo[u] = p.y[(int64_t)b[u] * p.sy + (int64_t)i[u] * p.incy];
            const T* xb = p.x + (int64_t)b[u] * p.sx;
            if (p.incx == 1) {
                xv[u] = ld_matrix<T, VEC>(xb + cl);
            } else {
#pragma unroll
                for (int k = 0; k < VEC; ++k) xv[u][k] = xb[(int64_t)(cl + k) * p.incx];
            }
        }
        __builtin_amdgcn_sched_barrier(0);   // every load of the tile is in flight before the first FMA
#pragma unroll
        for (int u = 0; u < kSlots; ++u) {
            T s = T(0);
#pragma unroll
            for (int k = 0; k < VEC; ++k) s = (cl + k >= c) ? fmad(a[u][k], xv[u][k], s) : s;
            s = group_sum<LPR>(s);
            const uint32_t row = t * rows_per_tile + u * G + g;
            if (l == 0 && row < p.total) {
                T* yp = p.y + (int64_t)b[u] * p.sy + (int64_t)i[u] * p.incy;
                T v = p.alpha * s;
                if (BETA) v = fmad(p.beta, yo[u], v);
                *yp = v;
            }
        }
    }
}

// Transposed: y_b[j] = sum_i A_b[i][j] x_b[i].  A lane owns one vector of columns (l = lane % LPR)
// and one of the 64 / LPR rows that a wavefront load covers; a wavefront works through whole
// problems, one after the other: the (problem, group of rows) pairs form a list that is taken
// kSlots at a time, column sums run in registers while the problem stays the same and are folded
// over the lanes that own the same columns when it ends (DPP rotations inside a row of 16 lanes,
// shuffles across rows), after which the first LPR lanes write y.
constexpr int kDppRor4 = 0x124, kDppRor8 = 0x128;     // row_ror:4, row_ror:8

__device__ __forceinline__ float shfl_xor(float v, int lane, int mask)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute((lane ^ mask) << 2, __builtin_bit_cast(int, v)));
}
__device__ __forceinline__ double shfl_xor(double v, int lane, int mask)
{
    const uint64_t b = __builtin_bit_cast(uint64_t, v);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_ds_bpermute((lane ^ mask) << 2, (int)(uint32_t)b);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_ds_bpermute((lane ^ mask) << 2, (int)(uint32_t)(b >> 32));
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}

// Sum over the lanes lane % LPR == const of a wavefront; every such lane receives it.
template <int LPR, typename T>
__device__ __forceinline__ T strided_sum(T v, int lane)
{
    if (LPR <= 4) v += dpp_mov<kDppRor4>(v);      // lanes 4 apart: i, i-4 ...
    if (LPR <= 8) v += dpp_mov<kDppRor8>(v);      // ... then 8 apart: all lanes of the row with the same lane % LPR
    v += shfl_xor(v, lane, 16);
    v += shfl_xor(v, lane, 32);
    return v;
}

template <typename T, int VEC, int LPR, bool BETA>
__global__ void __launch_bounds__(kThreads) tiny_gemv_t_kernel(const TinyArgs<T> p, uint32_t batch)
{
    typedef typename VecOf<T, VEC>::type V;
    constexpr int G = kWave / LPR;            // rows per wavefront load
    const int lane = threadIdx.x & (kWave - 1);
    const int g = lane / LPR, l = lane % LPR;
    const int c = l * VEC, cl = min(c, p.N - VEC);      // as in the not-transposed kernel
    const uint32_t groups = ((uint32_t)p.M + G - 1) / G;                 // groups of G rows per problem
    const uint32_t wave0 = blockIdx.x * kWaves + (threadIdx.x >> 6), nwaves = gridDim.x * kWaves;
    // problems are dealt to the wavefronts in contiguous runs, so that a wavefront reads one stream
    const uint32_t per = (batch + nwaves - 1) / nwaves;
    const uint32_t b0 = min(wave0 * per, batch), b1 = min(b0 + per, batch);
    const uint64_t items = (uint64_t)(b1 - b0) * groups;
    T acc[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) acc[k] = T(0);
    uint32_t b = b0, s = 0;                   // the (problem, group) of the next item
    for (uint64_t it = 0; it < items; it += kSlots) {
        V a[kSlots];
        T xi[kSlots];
        T yo[kSlots][VEC];
        uint32_t bb = b, ss = s;
#pragma unroll
        for (int u = 0; u < kSlots; ++u) {
            const uint32_t bu = min(bb, b1 - 1);                          // items past the end repeat the last problem; unused
            const uint32_t i = min(ss * G + g, (uint32_t)p.M - 1);        // clamp: loads stay in bounds
            a[u] = ld_matrix<T, VEC>(p.A + (int64_t)bu * p.sA + (int64_t)i * p.lda + cl);
            xi[u] = p.x[(int64_t)bu * p.sx + (int64_t)i * p.incx];
            if (++ss == groups) {             // this slot completes a problem: its old y travels with the tile
                if (BETA && g == 0) {
#pragma unroll
                    for (int k = 0; k < VEC; ++k) yo[u][k] = p.y[(int64_t)bu * p.sy + (int64_t)(cl + k) * p.incy];
                }
                ss = 0;
                ++bb;
            }
        }
        __builtin_amdgcn_sched_barrier(0);   // every load of the batch is in flight before the first FMA
#pragma unroll
        for (int u = 0; u < kSlots; ++u) {
            if (b < b1) {                     // the same for the whole wavefront
                const bool row_ok = s * G + g < (uint32_t)p.M;
#pragma unroll
                for (int k = 0; k < VEC; ++k) acc[k] = row_ok ? fmad(a[u][k], xi[u], acc[k]) : acc[k];
                if (++s == groups) {          // the problem is complete: fold and write
#pragma unroll
                    for (int k = 0; k < VEC; ++k) {
                        const T tot = strided_sum<LPR>(acc[k], lane);
                        if (g == 0 && cl + k >= c) {
                            T* yp = p.y + (int64_t)b * p.sy + (int64_t)(cl + k) * p.incy;
                            T v = p.alpha * tot;
                            if (BETA) v = fmad(p.beta, yo[u][k], v);
                            *yp = v;
                        }
                        acc[k] = T(0);
                    }
                    s = 0;
                    ++b;
                }
            }
        }
    }
}

// Transposed, problems of at most MR rows: a lane owns one vector of columns of one problem (the
// (problem, vector) pairs of the whole batch as one list, so that adjacent lanes read adjacent
// memory when the problems are packed) and walks down the problem's rows, all of them in flight
// at once; no folding across lanes.  The kernel above gives such a problem a group of 64 / LPR
// rows that it fills to a fraction and folds after every problem.
template <typename T, int VEC, int MR, bool BETA>
__global__ void __launch_bounds__(kThreads) tiny_fewrows_t_kernel(const TinyArgs<T> p, int nv, int64_t items)
{
    typedef typename VecOf<T, VEC>::type V;
    const int64_t id = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (id >= items) return;
    const int64_t b = id / nv;
    const int l = (int)(id - b * nv);
    const int c = l * VEC, cl = min(c, p.N - VEC);        // a vector past the end of the row is moved back; its first elements are the neighbour's
    const T* Ab = p.A + b * p.sA + cl;
    const T* xb = p.x + b * p.sx;
    V a[MR];
    T xi[MR];
#pragma unroll
    for (int i = 0; i < MR; ++i) {
        const int ic = min(i, p.M - 1);                   // clamp: loads stay in bounds, rows past the end meet a zero
        a[i] = ld_matrix<T, VEC>(Ab + (int64_t)ic * p.lda);
        xi[i] = i < p.M ? xb[(int64_t)ic * p.incx] : T(0);
    }
    T yo[VEC];
    if (BETA) {
#pragma unroll
        for (int k = 0; k < VEC; ++k) yo[k] = p.y[b * p.sy + (int64_t)(cl + k) * p.incy];
    }
    __builtin_amdgcn_sched_barrier(0);
    T acc[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) acc[k] = T(0);
#pragma unroll
    for (int i = 0; i < MR; ++i)
#pragma unroll
        for (int k = 0; k < VEC; ++k) acc[k] = fmad(a[i][k], xi[i], acc[k]);
#pragma unroll
    for (int k = 0; k < VEC; ++k) {
        if (cl + k >= c) {
            T v = p.alpha * acc[k];
            if (BETA) v = fmad(p.beta, yo[k], v);
            p.y[b * p.sy + (int64_t)(cl + k) * p.incy] = v;
        }
    }
}

}  // namespace

template <typename T>
int tiny_gemv_n(mxb_handle_t h, int64_t rows, int64_t cols, T alpha, const T* A, int64_t lda, int64_t sA, const T* x0, int64_t incx,
                int64_t sx, T beta, T* y0, int64_t incy, int64_t sy, int64_t batch)
{
    constexpr int VEC = Full<T>::vec;
    TinyArgs<T> a{(int)rows, (int)cols, (uint32_t)(rows * batch), A, lda, sA, x0, incx, sx, y0, incy, sy, alpha, beta};
    const int64_t nv = ceil_div(cols, (int64_t)VEC);
    const int lpr = nv <= 4 ? 4 : nv <= 8 ? 8 : 16;
    const int64_t tiles = ceil_div((int64_t)a.total, (int64_t)kSlots * (kWave / lpr));
    int64_t grid = ceil_div(tiles, (int64_t)kWaves);
    if (grid > (int64_t)kCUs * 16) grid = (int64_t)kCUs * 16;
    const dim3 g((unsigned)grid), blk(kThreads);
#define MXB_TINY_N(LPR_)                                                                                   \
    if (beta != T(0)) hipLaunchKernelGGL((tiny_gemv_n_kernel<T, VEC, LPR_, true>), g, blk, 0, h->stream, a); \
    else hipLaunchKernelGGL((tiny_gemv_n_kernel<T, VEC, LPR_, false>), g, blk, 0, h->stream, a)
    if (cols < VEC) {
        // rows narrower than one vector: one element per lane, a quad of lanes per row
        if (beta != T(0)) hipLaunchKernelGGL((tiny_gemv_n_kernel<T, 1, 4, true>), g, blk, 0, h->stream, a);
        else hipLaunchKernelGGL((tiny_gemv_n_kernel<T, 1, 4, false>), g, blk, 0, h->stream, a);
    }
    else if (lpr == 4) { MXB_TINY_N(4); }
    else if (lpr == 8) { MXB_TINY_N(8); }
    else { MXB_TINY_N(16); }
#undef MXB_TINY_N
    return launch_status();
}

template <typename T>
int tiny_gemv_t(mxb_handle_t h, int64_t rows, int64_t cols, T alpha, const T* A, int64_t lda, int64_t sA, const T* x0, int64_t incx,
                int64_t sx, T beta, T* y0, int64_t incy, int64_t sy, int64_t batch)
{
    constexpr int VEC = Full<T>::vec;
    TinyArgs<T> a{(int)rows, (int)cols, (uint32_t)(rows * batch), A, lda, sA, x0, incx, sx, y0, incy, sy, alpha, beta};
    if (rows <= kTinyFewRows) {
        const int vec = cols < VEC ? 1 : VEC;
        const int64_t nvf = ceil_div(cols, (int64_t)vec), items = batch * nvf;
        const dim3 gf((unsigned)ceil_div(items, (int64_t)kThreads)), bf(kThreads);
#define MXB_TINY_FEW2(VEC_, MR_)                                                                                                       \
    if (beta != T(0)) hipLaunchKernelGGL((tiny_fewrows_t_kernel<T, VEC_, MR_, true>), gf, bf, 0, h->stream, a, (int)nvf, items);       \
    else hipLaunchKernelGGL((tiny_fewrows_t_kernel<T, VEC_, MR_, false>), gf, bf, 0, h->stream, a, (int)nvf, items)
#define MXB_TINY_FEW(VEC_)                                   \
    if (rows <= 1) { MXB_TINY_FEW2(VEC_, 1); }               \
    else if (rows <= 2) { MXB_TINY_FEW2(VEC_, 2); }          \
    else if (rows <= 4) { MXB_TINY_FEW2(VEC_, 4); }          \
    else if (rows <= 8) { MXB_TINY_FEW2(VEC_, 8); }          \
    else { MXB_TINY_FEW2(VEC_, 16); }
        if (vec == 1) { MXB_TINY_FEW(1) } else { MXB_TINY_FEW(VEC) }
#undef MXB_TINY_FEW
#undef MXB_TINY_FEW2
        return launch_status();
    }
    const int64_t nv = ceil_div(cols, (int64_t)VEC);
    const int lpr = nv <= 4 ? 4 : nv <= 8 ? 8 : 16;
    // enough wavefronts to fill the device, but whole problems per wavefront
    int64_t waves = (int64_t)kCUs * 16 * kWaves;
    if (waves > batch) waves = batch;
    const dim3 g((unsigned)ceil_div(waves, (int64_t)kWaves)), blk(kThreads);
#define MXB_TINY_T(LPR_)                                                                                                      \
    if (beta != T(0)) hipLaunchKernelGGL((tiny_gemv_t_kernel<T, VEC, LPR_, true>), g, blk, 0, h->stream, a, (uint32_t)batch); \
    else hipLaunchKernelGGL((tiny_gemv_t_kernel<T, VEC, LPR_, false>), g, blk, 0, h->stream, a, (uint32_t)batch)
    if (cols < VEC) {
        if (beta != T(0)) hipLaunchKernelGGL((tiny_gemv_t_kernel<T, 1, 4, true>), g, blk, 0, h->stream, a, (uint32_t)batch);
        else hipLaunchKernelGGL((tiny_gemv_t_kernel<T, 1, 4, false>), g, blk, 0, h->stream, a, (uint32_t)batch);
    }
    else if (lpr == 4) { MXB_TINY_T(4); }
    else if (lpr == 8) { MXB_TINY_T(8); }
    else { MXB_TINY_T(16); }
#undef MXB_TINY_T
    return launch_status();
}

template int tiny_gemv_t<float>(mxb_handle_t, int64_t, int64_t, float, const float*, int64_t, int64_t, const float*, int64_t, int64_t,
                                float, float*, int64_t, int64_t, int64_t);
template int tiny_gemv_t<double>(mxb_handle_t, int64_t, int64_t, double, const double*, int64_t, int64_t, const double*, int64_t,
                                 int64_t, double, double*, int64_t, int64_t, int64_t);
template int tiny_gemv_n<float>(mxb_handle_t, int64_t, int64_t, float, const float*, int64_t, int64_t, const float*, int64_t, int64_t,
                                float, float*, int64_t, int64_t, int64_t);
template int tiny_gemv_n<double>(mxb_handle_t, int64_t, int64_t, double, const double*, int64_t, int64_t, const double*, int64_t,
                                 int64_t, double, double*, int64_t, int64_t, int64_t);

}  // namespace mxb
