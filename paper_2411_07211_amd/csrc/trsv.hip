// trsv (Sec. 6.2.2, triangular solve) on a row-major matrix: blocked substitution.  The part of
// a block's right-hand side that depends on unknowns solved earlier is subtracted with the
// matrix-vector kernels of matvec.hip; the block on the diagonal is solved by one workgroup.
#include "matvec.hpp"

#include "options.hpp"

namespace mxb {
namespace {

// op(T) z = b by blocked substitution.
//
// The unknowns are cut into blocks of NB = 64*NW.  For every block, in the order the
// dependences impose, (1) the contributions of all unknowns solved so far are subtracted from
// the block's right-hand side by the gemv kernels (row-dot if not transposed,
// column-accumulate if transposed: both read rows of the row-major matrix), and (2) one
// workgroup solves the NB x NB triangle on the diagonal.  Everything is enqueued on one stream,
// so the steps run in order; the chain of dependences makes the routine latency-bound, not
// bandwidth-bound.
//
// In the diagonal kernel lane l of wavefront w owns unknown i = 64*w + l.  Every wavefront keeps
// its row of the 64 x 64 triangle on the diagonal in registers (zero outside the triangle, so the
// substitution needs no predicate) and solves it in 64 unrolled steps, broadcasting each new
// unknown with readlane; the 64 results go to LDS, from where the wavefronts that come later
// subtract their 64 x 64 block's contribution (its elements were fetched while the solver ran).
template <typename T>
struct TrsvArgs {
    int nb;              // unknowns of this block (<= 64*NW)
    const T* A;          // element (0, 0) of the diagonal block
    int64_t lda;
    T* x;                // logical element 0 of the block's part of x
    int64_t incx;
};

__device__ __forceinline__ float lane_bcast(float v, int j)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), j));
}
__device__ __forceinline__ double lane_bcast(double v, int j)
{
    const uint64_t b = __builtin_bit_cast(uint64_t, v);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)b, j);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(b >> 32), j);
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}

// OPLOWER: op(T) is lower triangular (unknown 0 first); TRANS: op(T)[i][j] is stored at (j, i).
template <typename T, int NW, bool OPLOWER, bool TRANS, bool UNIT>
__global__ void __launch_bounds__(NW* kWave) trsv_diag_kernel(const TrsvArgs<T> p)
{
    __shared__ T xs[NW * kWave];
    __shared__ T tile[TRANS ? 1 : NW][TRANS ? 1 : kWave][TRANS ? 1 : kWave + 1];   // per-wavefront transposition buffer
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int i = wave * kWave + lane;
    const bool active = i < p.nb;
    const int nsub = (p.nb + kWave - 1) / kWave;

    // out[j] = op(T)[i][c0 + j], j < 64, for my unknown i (0 where i or the column is past the
    // block).  Transposed: row c0 + j of the matrix holds these values for 64 adjacent unknowns,
    // one coalesced load per j.  Not transposed: a lane's values are its own row, so the
    // wavefront reads the 64 x 64 tile row by row (coalesced) and turns it through LDS.
    auto fetch = [&](int c0, T (&out)[kWave]) {
        // Addresses are clamped into the block, so that every load is unconditional and all 64 are
        // in flight at once; what lies past the block is replaced by zero afterwards.  (The empty
        // asm pins each loaded value: without it the compiler moves every load under the
        // condition of its select and waits for each one in turn.)
        const int last = p.nb - 1;
        T raw[kWave];
        if (TRANS) {
            const int ic = min(i, last);
#pragma unroll
            for (int j = 0; j < kWave; ++j) {
                const T* rowp = p.A + (int64_t)min(c0 + j, last) * p.lda;      // wave-uniform: scalar base, lane offset
                raw[j] = rowp[ic];
            }
#pragma unroll
            for (int j = 0; j < kWave; ++j) asm volatile("" : "+v"(raw[j]));
#pragma unroll
            for (int j = 0; j < kWave; ++j) out[j] = (active && c0 + j < p.nb) ? raw[j] : T(0);
        } else {
            T tmp[kWave];
            const int cc = min(c0 + lane, last);
#pragma unroll
            for (int r = 0; r < kWave; ++r) {
                const T* rowp = p.A + (int64_t)min(wave * kWave + r, last) * p.lda;   // wave-uniform: scalar base, lane offset
                raw[r] = rowp[cc];
            }
#pragma unroll
            for (int r = 0; r < kWave; ++r) asm volatile("" : "+v"(raw[r]));
#pragma unroll
            for (int r = 0; r < kWave; ++r) tmp[r] = (wave * kWave + r < p.nb && c0 + lane < p.nb) ? raw[r] : T(0);
            __builtin_amdgcn_wave_barrier();      // earlier reads of the buffer by this wavefront come first
#pragma unroll
            for (int r = 0; r < kWave; ++r) tile[TRANS ? 0 : wave][TRANS ? 0 : r][TRANS ? 0 : lane] = tmp[r];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int j = 0; j < kWave; ++j) out[j] = tile[TRANS ? 0 : wave][TRANS ? 0 : lane][TRANS ? 0 : j];
        }
    };

    T b = active ? p.x[(int64_t)i * p.incx] : T(0);
    // my row of the triangle on the diagonal: zero on and outside the diagonal
    T e[kWave];
    fetch(wave * kWave, e);
    T dv = T(1);
#pragma unroll
    for (int j = 0; j < kWave; ++j) {
        dv = (!UNIT && active && j == lane) ? e[j] : dv;
        const bool inside = OPLOWER ? j < lane : j > lane;
        e[j] = inside ? e[j] : T(0);
    }
    const T rinv = T(1) / dv;      // 1 in the lanes past the block: their zeros stay zeros

    for (int step = 0; step < nsub; ++step) {
        const int s = OPLOWER ? step : nsub - 1 - step;
        const bool later = OPLOWER ? wave > s : wave < s;
        T ev[kWave];
        if (wave == s) {
            T xv = T(0);
#pragma unroll
            for (int jj = 0; jj < kWave; ++jj) {
                const int j = OPLOWER ? jj : kWave - 1 - jj;
                const T xj = lane_bcast(UNIT ? b : b * rinv, j);
                xv = lane == j ? xj : xv;
                b = fmad(-e[j], xj, b);
            }
            xs[i] = xv;
            if (active) p.x[(int64_t)i * p.incx] = xv;
        } else if (later) {
            fetch(s * kWave, ev);
        }
        __syncthreads();
        if (later) {
#pragma unroll
            for (int j = 0; j < kWave; ++j) b = fmad(-ev[j], xs[s * kWave + j], b);
        }
    }
}

template <typename T, int NW, bool TRANS>
void launch_trsv_diag(mxb_handle_t h, bool op_lower, bool unit, const TrsvArgs<T>& a)
{
    const dim3 grid(1), block(NW * kWave);
    if (op_lower) {
        if (unit) hipLaunchKernelGGL((trsv_diag_kernel<T, NW, true, TRANS, true>), grid, block, 0, h->stream, a);
        else hipLaunchKernelGGL((trsv_diag_kernel<T, NW, true, TRANS, false>), grid, block, 0, h->stream, a);
    } else {
        if (unit) hipLaunchKernelGGL((trsv_diag_kernel<T, NW, false, TRANS, true>), grid, block, 0, h->stream, a);
        else hipLaunchKernelGGL((trsv_diag_kernel<T, NW, false, TRANS, false>), grid, block, 0, h->stream, a);
    }
}

template <typename T>
int trsv(mxb_handle_t h, int layout, int uplo, int trans, int diag, int64_t n, const T* A, int64_t lda, T* x, int64_t incx)
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
    const bool unit = diag == MXB_UNIT;
    const bool op_lower = upper != no_trans;          // lower and not transposed, or upper and transposed
    constexpr int NW = sizeof(T) == 4 ? 8 : 4;        // 64 registers of triangle + 64 of prefetch per lane: 512 / 256 unknowns
    constexpr int64_t NB = NW * kWave;
    T* x0 = vec_base(x, n, incx);
    const int64_t nblocks = ceil_div(n, NB);
    for (int64_t step = 0; step < nblocks; ++step) {
        const int64_t k = op_lower ? step : nblocks - 1 - step;
        const int64_t r0 = k * NB, nb = r0 + NB < n ? NB : n - r0;
        // unknowns solved so far: [0, r0) if op(T) is lower, [r0 + nb, n) if upper
        const int64_t s0 = op_lower ? 0 : r0 + nb, ns = op_lower ? r0 : n - s0;
        if (ns > 0) {
            int st;
            if (no_trans) {   // b_k -= T[block rows, solved columns] * z[solved]
                RowdotArgs<T> a{nb, ns, A + r0 * lda + s0, lda, x0 + s0 * incx, incx, x0 + r0 * incx, incx, T(-1), T(1), 0, 0};
                st = launch_rowdot(h, a, MODE_GENERAL, false);
            } else {          // b_k -= T[solved rows, block columns]^t * z[solved]
                ColaccArgs<T> a{ns, nb, A + s0 * lda + r0, lda, x0 + s0 * incx, incx, x0 + r0 * incx, incx, T(-1), T(1), nullptr, 0, 0};
                st = launch_colacc(h, a);
            }
            if (st != MXB_OK) return st;
        }
        const TrsvArgs<T> d{(int)nb, A + r0 * lda + r0, lda, x0 + r0 * incx, incx};
        if (no_trans) launch_trsv_diag<T, NW, false>(h, op_lower, unit, d);
        else launch_trsv_diag<T, NW, true>(h, op_lower, unit, d);
        const int st = launch_status();
        if (st != MXB_OK) return st;
    }
    return MXB_OK;
}

}  // namespace
}  // namespace mxb

extern "C" {
int mxb_strsv(mxb_handle_t h, mxb_layout_t layout, mxb_uplo_t uplo, mxb_trans_t trans, mxb_diag_t diag, int64_t n,
              const float* A, int64_t lda, float* x, int64_t incx)
{ return mxb::trsv<float>(h, layout, uplo, trans, diag, n, A, lda, x, incx); }
int mxb_dtrsv(mxb_handle_t h, mxb_layout_t layout, mxb_uplo_t uplo, mxb_trans_t trans, mxb_diag_t diag, int64_t n,
              const double* A, int64_t lda, double* x, int64_t incx)
{ return mxb::trsv<double>(h, layout, uplo, trans, diag, n, A, lda, x, incx); }
}
