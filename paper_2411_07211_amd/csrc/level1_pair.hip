// The element-wise two-vector routines of the level-1 set (Sec. 6.2.1): copy, swap, rot, rotm.
// One streaming kernel per access shape, parameterised by the operation applied to each (x, y)
// pair: 128-bit non-temporal loads and stores, whole tiles without predicates (all loads of a
// tile are issued before the first store), the ragged rest by the last block.
#include "common.hpp"
#include "options.hpp"

namespace mxb {
namespace {

constexpr int kThreads = 256;
constexpr int kUnroll = 4;          // 128-bit loads per thread and array (contiguous shape)
constexpr int kStridedUnroll = 8;   // elements per thread and array (strided shape)

template <typename T> struct OpCopy {
    static constexpr bool kReadY = false, kWriteX = false;
    __device__ __forceinline__ void operator()(T& x, T& y) const { y = x; }
};
template <typename T> struct OpSwap {
    static constexpr bool kReadY = true, kWriteX = true;
    __device__ __forceinline__ void operator()(T& x, T& y) const { const T t = x; x = y; y = t; }
};
// (x, y) := (h11*x + h12*y, h21*x + h22*y); rot is the case h11 = h22 = c, h12 = s, h21 = -s
template <typename T> struct OpLinear {
    static constexpr bool kReadY = true, kWriteX = true;
    T h11, h12, h21, h22;
    __device__ __forceinline__ void operator()(T& x, T& y) const
    {
        const T nx = fmad(h11, x, h12 * y);
        const T ny = fmad(h22, y, h21 * x);
        x = nx;
        y = ny;
    }
};

template <typename T, typename Op, bool KEEP>
__global__ void __launch_bounds__(kThreads) pair_vec_kernel(int64_t nvec, int64_t nfull, int64_t n2d, int tail, T* __restrict__ x,
                                                            T* __restrict__ y, const Op op)
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
        for (int u = 0; u < U; ++u) b[u] = Op::kReadY ? ld_matrix_as<T, VEC, KEEP>(y + (base + u * step) * VEC) : V(T(0));
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int k = 0; k < VEC; ++k) {
                T p = a[u][k], q = b[u][k];
                op(p, q);
                a[u][k] = p;
                b[u][k] = q;
            }
            if (Op::kWriteX) st_matrix<T, VEC>(x + (base + u * step) * VEC, a[u]);
            st_matrix<T, VEC>(y + (base + u * step) * VEC, b[u]);
        }
    }
    if (blockIdx.x != gridDim.x - 1) return;
    const int64_t first = nfull * (kThreads * U) * VEC;                 // first element of the ragged rest
    const int64_t n = nvec * VEC + tail;
    for (int64_t i = first + threadIdx.x; i < n; i += kThreads) {
        T p = x[i], q = Op::kReadY ? y[i] : T(0);
        op(p, q);
        if (Op::kWriteX) x[i] = p;
        y[i] = q;
    }
}

template <typename T, typename Op>
__global__ void __launch_bounds__(kThreads) pair_strided_kernel(int64_t n, int64_t nfull, T* __restrict__ x, int64_t incx,
                                                                T* __restrict__ y, int64_t incy, const Op op)
{
    constexpr int U = kStridedUnroll;
    for (int64_t t = blockIdx.x; t < nfull; t += gridDim.x) {
        const int64_t base = t * (kThreads * U) + threadIdx.x;
        T a[U], b[U];
#pragma unroll
        for (int u = 0; u < U; ++u) a[u] = x[(base + u * kThreads) * incx];
#pragma unroll
        for (int u = 0; u < U; ++u) b[u] = Op::kReadY ? y[(base + u * kThreads) * incy] : T(0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            op(a[u], b[u]);
            if (Op::kWriteX) x[(base + u * kThreads) * incx] = a[u];
            y[(base + u * kThreads) * incy] = b[u];
        }
    }
    if (blockIdx.x != gridDim.x - 1) return;
    for (int64_t i = nfull * (kThreads * U) + threadIdx.x; i < n; i += kThreads) {
        T p = x[i * incx], q = Op::kReadY ? y[i * incy] : T(0);
        op(p, q);
        if (Op::kWriteX) x[i * incx] = p;
        y[i * incy] = q;
    }
}

// Errors: n < 0 (-1), x NULL (-2), incx == 0 (-3), y NULL (-4), incy == 0 (-5).
template <typename T, typename Op>
int pair_op(mxb_handle_t h, int64_t n, T* x, int64_t incx, T* y, int64_t incy, const Op& op)
{
    if (!handle_ok(h)) return MXB_ERR_HANDLE;
    if (n < 0) return -1;
    if (n == 0) return MXB_OK;
    if (!x) return -2;
    if (incx == 0) return -3;
    if (!y) return -4;
    if (incy == 0) return -5;
    constexpr int VEC = Full<T>::vec;
    const int64_t cap = kCUs * option(h, MXB_OPT_L1_BLOCKS_PER_CU);
    if (incx == 1 && incy == 1) {   // any base address: the vector accesses need element alignment only
        const int64_t nvec = n / VEC, nfull = nvec / (kThreads * kUnroll);
        const int64_t grid = nfull < 1 ? 1 : (nfull < cap ? nfull : cap);
        if (keeps_vectors((Op::kReadY ? 2 : 1) * n * (int64_t)sizeof(T)))
            hipLaunchKernelGGL((pair_vec_kernel<T, Op, true>), dim3((unsigned)grid), dim3(kThreads), 0, h->stream, nvec, nfull,
                               stream_tiles_2d(nvec, kUnroll), (int)(n % VEC), x, y, op);
        else
            hipLaunchKernelGGL((pair_vec_kernel<T, Op, false>), dim3((unsigned)grid), dim3(kThreads), 0, h->stream, nvec, nfull,
                               stream_tiles_2d(nvec, kUnroll), (int)(n % VEC), x, y, op);
    } else {
        const int64_t nfull = n / (kThreads * kStridedUnroll);
        const int64_t grid = nfull < 1 ? 1 : (nfull < cap ? nfull : cap);
        hipLaunchKernelGGL((pair_strided_kernel<T, Op>), dim3((unsigned)grid), dim3(kThreads), 0, h->stream, n, nfull,
                           vec_base(x, n, incx), incx, vec_base(y, n, incy), incy, op);
    }
    return launch_status();
}

template <typename T>
int rotm(mxb_handle_t h, int64_t n, T* x, int64_t incx, T* y, int64_t incy, const T* param)
{
    if (!handle_ok(h)) return MXB_ERR_HANDLE;
    if (n < 0) return -1;
    if (!param) return -6;
    const T flag = param[0];
    if (n == 0 || flag == T(-2)) return MXB_OK;
    OpLinear<T> op;
    if (flag < T(0)) op = OpLinear<T>{param[1], param[3], param[2], param[4]};
    else if (flag == T(0)) op = OpLinear<T>{T(1), param[3], param[2], T(1)};
    else op = OpLinear<T>{param[1], T(1), T(-1), param[4]};
    return pair_op<T>(h, n, x, incx, y, incy, op);
}

}  // namespace
}  // namespace mxb

extern "C" {
int mxb_scopy(mxb_handle_t h, int64_t n, const float* x, int64_t incx, float* y, int64_t incy)
{ return mxb::pair_op<float>(h, n, const_cast<float*>(x), incx, y, incy, mxb::OpCopy<float>{}); }
int mxb_dcopy(mxb_handle_t h, int64_t n, const double* x, int64_t incx, double* y, int64_t incy)
{ return mxb::pair_op<double>(h, n, const_cast<double*>(x), incx, y, incy, mxb::OpCopy<double>{}); }
int mxb_sswap(mxb_handle_t h, int64_t n, float* x, int64_t incx, float* y, int64_t incy)
{ return mxb::pair_op<float>(h, n, x, incx, y, incy, mxb::OpSwap<float>{}); }
int mxb_dswap(mxb_handle_t h, int64_t n, double* x, int64_t incx, double* y, int64_t incy)
{ return mxb::pair_op<double>(h, n, x, incx, y, incy, mxb::OpSwap<double>{}); }
int mxb_srot(mxb_handle_t h, int64_t n, float* x, int64_t incx, float* y, int64_t incy, float c, float s)
{ return mxb::pair_op<float>(h, n, x, incx, y, incy, mxb::OpLinear<float>{c, s, -s, c}); }
int mxb_drot(mxb_handle_t h, int64_t n, double* x, int64_t incx, double* y, int64_t incy, double c, double s)
{ return mxb::pair_op<double>(h, n, x, incx, y, incy, mxb::OpLinear<double>{c, s, -s, c}); }
int mxb_srotm(mxb_handle_t h, int64_t n, float* x, int64_t incx, float* y, int64_t incy, const float* param)
{ return mxb::rotm<float>(h, n, x, incx, y, incy, param); }
int mxb_drotm(mxb_handle_t h, int64_t n, double* x, int64_t incx, double* y, int64_t incy, const double* param)
{ return mxb::rotm<double>(h, n, x, incx, y, incy, param); }
}
