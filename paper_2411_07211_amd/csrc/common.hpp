// Shared host/device helpers of libmxblas: the handle, argument checks, launch geometry, 128-bit
// vector types, streaming loads and wavefront (64-lane) reductions on DPP.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/mxblas.h"

struct mxb_ctx {
    uint32_t magic;
    hipStream_t stream;
    void* ws;
    size_t ws_bytes;
    int64_t opt[MXB_OPT_COUNT];
    const int* device_status;   // error word of the last call that can fail on the device (in the workspace), or null
};

namespace mxb {

constexpr uint32_t kMagic = 0x6d786231u;   // "mxb1"
constexpr int kWave = 64;                  // CDNA wavefront width
constexpr int kCUs = 256;                  // MI355X compute units (8 XCDs x 32)

inline bool handle_ok(mxb_handle_t h) { return h != nullptr && h->magic == kMagic; }

// The handle's workspace if it holds at least `bytes`, else null.  What the last call left there
// for mxb_last_status is about to be overwritten, so that is forgotten.
inline void* take_workspace(mxb_handle_t h, size_t bytes)
{
    if (!h->ws || h->ws_bytes < bytes) return nullptr;
    h->device_status = nullptr;
    return h->ws;
}

inline int launch_status()
{
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? MXB_OK : MXB_ERR_HIP_BASE + (int)e;
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Pointer to logical element 0 of a strided vector: for a negative increment BLAS stores the
// vector backwards, so element 0 sits at (n-1)*|inc| and the signed increment walks down.
template <typename T>
inline T* vec_base(T* p, int64_t n, int64_t inc)
{
    return inc >= 0 ? p : p + (n - 1) * (-inc);
}

// Fused multiply-add in the element type (the bare builtin is the fp64 one and would silently
// promote floats to double and back).
__device__ __forceinline__ float fmad(float a, float b, float c) { return __builtin_fmaf(a, b, c); }
__device__ __forceinline__ double fmad(double a, double b, double c) { return __builtin_fma(a, b, c); }

// ------------------------------------------------------------------------------------------------
// 128-bit vectors: 4 floats or 2 doubles per lane and load, so that one wavefront load moves 1 KiB.
template <typename T, int VEC> struct VecOf;
template <> struct VecOf<float, 4> { typedef float type __attribute__((ext_vector_type(4))); };
template <> struct VecOf<double, 2> { typedef double type __attribute__((ext_vector_type(2))); };
template <> struct VecOf<float, 1> { typedef float type __attribute__((ext_vector_type(1))); };
template <> struct VecOf<double, 1> { typedef double type __attribute__((ext_vector_type(1))); };

template <typename T> struct Full { static constexpr int vec = 16 / sizeof(T); };

// Streaming (read-once) load / store: the non-temporal hint keeps a matrix that is touched exactly
// once from pushing the reused vectors out of L2.
template <typename V> __device__ __forceinline__ V ld_stream(const V* p) { return __builtin_nontemporal_load(p); }
template <typename V> __device__ __forceinline__ void st_stream(V* p, V v) { __builtin_nontemporal_store(v, p); }

// The same for VEC adjacent elements of a matrix row or of a contiguous vector.  A 128-bit global load or store needs the alignment
// of one element only, so the rows of a matrix may start anywhere (any pitch, any base address):
// the vector is declared with element alignment and still moves as one 128-bit access.
template <typename T, int VEC>
__device__ __forceinline__ typename VecOf<T, VEC>::type ld_matrix(const T* p)
{
    typedef typename VecOf<T, VEC>::type Loose __attribute__((aligned(sizeof(T))));
    return __builtin_nontemporal_load(reinterpret_cast<const Loose*>(p));
}
// The same load without the hint, for the kernels that take a matrix small enough to stay in the
// caches from one call to the next: a line that a hinted load misses is not kept, so a matrix read
// only through hinted loads comes from wherever earlier traffic happened to leave it.
template <typename T, int VEC>
__device__ __forceinline__ typename VecOf<T, VEC>::type ld_resident(const T* p)
{
    typedef typename VecOf<T, VEC>::type Loose __attribute__((aligned(sizeof(T))));
    return *reinterpret_cast<const Loose*>(p);
}
template <typename T, int VEC, bool RESIDENT>
__device__ __forceinline__ typename VecOf<T, VEC>::type ld_matrix_as(const T* p)
{
    return RESIDENT ? ld_resident<T, VEC>(p) : ld_matrix<T, VEC>(p);
}

// Which calls load without the hint (measured, per call when the same call is repeated): vectors
// that together fit the L2 caches (8 x 4 MiB) stay there between calls, 15 to 45 % faster at 16 to
// 32 MiB and no slower below; a matrix of up to 192 MiB stays in the last-level cache, 3 to 25 %
// faster, and one that has to come from HBM all the same takes 4 to 9 % longer than with the hint.
// Beyond these sizes the hint is worth up to 45 % (A*x at 16384^2: 158 against 230 us).
constexpr int64_t kKeepVectorBytes = (int64_t)32 << 20;
constexpr int64_t kKeepMatrixBytes = (int64_t)192 << 20;
constexpr int64_t kKeepUpdateBytes = (int64_t)512 << 20;   // rank-1 update, per call: 8192^2 75.9 against 85.3 us, 16384^2 the same either way
inline bool keeps_vectors(int64_t bytes) { return bytes <= kKeepVectorBytes; }
inline bool keeps_matrix(int64_t bytes) { return bytes <= kKeepMatrixBytes; }
inline bool keeps_update(int64_t bytes) { return bytes <= kKeepUpdateBytes; }
template <typename T, int VEC>
__device__ __forceinline__ void st_matrix(T* p, typename VecOf<T, VEC>::type v)
{
    typedef typename VecOf<T, VEC>::type Loose __attribute__((aligned(sizeof(T))));
    __builtin_nontemporal_store(v, reinterpret_cast<Loose*>(p));
}

// ------------------------------------------------------------------------------------------------
// Tiles of a flat, contiguous stream of 16-byte vectors for 256-thread blocks that keep U vectors
// per thread in flight.  Where whole groups of U*64 KiB are left, a tile is U runs of 4 KiB that
// lie 64 KiB apart (the stream seen as rows of 64 KiB, 16 tiles side by side, as in the rank-1
// update of a 16384-column matrix): read-modify-write streams run 4-9 points closer to the HBM
// peak in this shape than in contiguous tiles of U*4 KiB.  The rest of the stream is cut into
// contiguous tiles.  t: tile index; n2d: tiles in the 2-D part = (vectors / (U*4096)) * 16.
constexpr int kPitchVec = 4096;
template <int U>
__device__ __forceinline__ void stream_tile(int64_t t, int64_t n2d, int64_t& base, int64_t& step)
{
    if (t < n2d) {
        base = (t >> 4) * (int64_t)(U * kPitchVec) + (t & 15) * 256 + threadIdx.x;
        step = kPitchVec;
    } else {
        base = t * (int64_t)(256 * U) + threadIdx.x;
        step = 256;
    }
}
inline int64_t stream_tiles_2d(int64_t nvec, int u) { return nvec / ((int64_t)u * kPitchVec) * 16; }

// ------------------------------------------------------------------------------------------------
// Wavefront reductions.  Lanes are organised as 4 DPP rows of 16.  Within a row: two quad
// permutes (xor 1, xor 2), then row_half_mirror and row_mirror fold 4 -> 8 -> 16 lanes, after
// which every lane of a row holds the row's sum.  Across rows: row_bcast15 adds row r into row
// r+1 (rows 1 and 3), row_bcast31 adds lane 31 into rows 2 and 3, leaving the wavefront total in
// lane 63, which readlane returns as a wave-uniform value.  The order of additions is fixed, so
// results are reproducible.
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ float dpp_mov(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xF, false));
}
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ double dpp_mov(double v)
{
    const uint64_t b = __builtin_bit_cast(uint64_t, v);
    const int lo = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)b, CTRL, ROW_MASK, 0xF, false);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)(b >> 32), CTRL, ROW_MASK, 0xF, false);
    return __builtin_bit_cast(double, ((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
}

constexpr int kDppXor1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141; // row_half_mirror
constexpr int kDppMirror = 0x140;     // row_mirror
constexpr int kDppBcast15 = 0x142;    // row_bcast:15
constexpr int kDppBcast31 = 0x143;    // row_bcast:31

// Sum over each DPP row (16 adjacent lanes); every lane of the row receives the row sum.
template <typename A>
__device__ __forceinline__ A row16_sum(A v)
{
    v += dpp_mov<kDppXor1>(v);
    v += dpp_mov<kDppXor2>(v);
    v += dpp_mov<kDppHalfMirror>(v);
    v += dpp_mov<kDppMirror>(v);
    return v;
}

__device__ __forceinline__ float read_lane63(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}
__device__ __forceinline__ double read_lane63(double v)
{
    const uint64_t b = __builtin_bit_cast(uint64_t, v);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)b, 63);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(b >> 32), 63);
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}

// Sum over the whole wavefront, returned wave-uniform.
template <typename A>
__device__ __forceinline__ A wave_sum(A v)
{
    v = row16_sum(v);
    v += dpp_mov<kDppBcast15, 0xA>(v);
    v += dpp_mov<kDppBcast31, 0xC>(v);
    return read_lane63(v);
}

// Sum over the lanes that share one matrix row: 64 (whole wavefront) or 16 (one DPP row).
template <int LANES, typename A>
__device__ __forceinline__ A lanes_sum(A v)
{
    static_assert(LANES == 64 || LANES == 16, "lane group is a wavefront or a DPP row");
    if constexpr (LANES == 64) return wave_sum(v);
    else return row16_sum(v);
}

// ------------------------------------------------------------------------------------------------
// NR sums at once (NR = 4, 8, 16 or 32 per lane, each to be added up over the 64 lanes): instead of
// NR full folds, the values are folded pairwise so that every step halves the number of live
// values.  gfx950's lane-swap instructions do the two cross-row steps: permlane32_swap exchanges
// the upper half of one register with the lower half of another, so that a + b afterwards holds
// value 0's sum over both halves in lanes 0-31 and value 1's in lanes 32-63; permlane16_swap does
// the same with odd and even rows of 16.  Inside a row, quad permutes pair lanes l and l^1, l^2
// the same way (the lane's bit picks which value it keeps and which it hands over).  What is left
// of the 64 lanes per value is folded plainly: l^1, l^2 by quad permutes, then the four lanes
// l, l+4, l+8, l+12 by two row rotations.  NR = 8 costs 18 instructions instead of 64.
// Fixed order, so results are reproducible.  The lane's value belongs to row rows_fold_lane().
constexpr int kDppRor4 = 0x124, kDppRor8 = 0x128;   // row_ror: lane l reads lane (l - n) mod 16 of its row

__device__ __forceinline__ void lane_swap32(float& a, float& b)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(unsigned, a), __builtin_bit_cast(unsigned, b), false, false);
    const unsigned r0 = r[0], r1 = r[1];     // (a bit cast straight from r[1] reads r[0] with this compiler)
    a = __builtin_bit_cast(float, r0);
    b = __builtin_bit_cast(float, r1);
}
__device__ __forceinline__ void lane_swap16(float& a, float& b)
{
    const auto r = __builtin_amdgcn_permlane16_swap(__builtin_bit_cast(unsigned, a), __builtin_bit_cast(unsigned, b), false, false);
    const unsigned r0 = r[0], r1 = r[1];     // (a bit cast straight from r[1] reads r[0] with this compiler)
    a = __builtin_bit_cast(float, r0);
    b = __builtin_bit_cast(float, r1);
}
__device__ __forceinline__ void lane_swap32(double& a, double& b)
{
    const uint64_t x = __builtin_bit_cast(uint64_t, a), y = __builtin_bit_cast(uint64_t, b);
    const auto lo = __builtin_amdgcn_permlane32_swap((unsigned)x, (unsigned)y, false, false);
    const auto hi = __builtin_amdgcn_permlane32_swap((unsigned)(x >> 32), (unsigned)(y >> 32), false, false);
    a = __builtin_bit_cast(double, ((uint64_t)hi[0] << 32) | lo[0]);
    b = __builtin_bit_cast(double, ((uint64_t)hi[1] << 32) | lo[1]);
}
__device__ __forceinline__ void lane_swap16(double& a, double& b)
{
    const uint64_t x = __builtin_bit_cast(uint64_t, a), y = __builtin_bit_cast(uint64_t, b);
    const auto lo = __builtin_amdgcn_permlane16_swap((unsigned)x, (unsigned)y, false, false);
    const auto hi = __builtin_amdgcn_permlane16_swap((unsigned)(x >> 32), (unsigned)(y >> 32), false, false);
    a = __builtin_bit_cast(double, ((uint64_t)hi[0] << 32) | lo[0]);
    b = __builtin_bit_cast(double, ((uint64_t)hi[1] << 32) | lo[1]);
}

// Row whose sum rows_fold<NR> leaves in this lane; true for the one lane per row that should write it.
template <int NR>
__device__ __forceinline__ bool rows_fold_lane(int lane, int& row)
{
    static_assert(NR == 4 || NR == 8 || NR == 16 || NR == 32, "rows per batch");
    row = ((lane >> 5) & 1) | (((lane >> 4) & 1) << 1);
    int used = 0x30;
    if (NR >= 8) { row |= (lane & 1) << 2; used |= 1; }
    if (NR >= 16) { row |= ((lane >> 1) & 1) << 3; used |= 2; }
    if (NR >= 32) { row |= ((lane >> 3) & 1) << 4; used |= 8; }
    return (lane & ~used & 63) == 0;
}

template <int NR, typename A>
__device__ __forceinline__ A rows_fold(const A (&v)[NR], int lane)
{
    static_assert(NR == 4 || NR == 8 || NR == 16 || NR == 32, "rows per batch");
    A w[NR / 2];
#pragma unroll
    for (int i = 0; i < NR / 2; ++i) {        // lanes 0-31: row 2i, lanes 32-63: row 2i + 1
        A a = v[2 * i], b = v[2 * i + 1];
        lane_swap32(a, b);
        w[i] = a + b;
    }
    A z[NR / 4];
#pragma unroll
    for (int i = 0; i < NR / 4; ++i) {        // even rows of 16 lanes: w[2i], odd rows: w[2i + 1]
        A a = w[2 * i], b = w[2 * i + 1];
        lane_swap16(a, b);
        z[i] = a + b;
    }
    if constexpr (NR == 4) {
        A s = z[0];
        s += dpp_mov<kDppXor1>(s);
        s += dpp_mov<kDppXor2>(s);
        s += dpp_mov<kDppRor8>(s);
        s += dpp_mov<kDppRor4>(s);
        return s;
    } else {
        const bool b0 = lane & 1;
        A y[NR / 8];
#pragma unroll
        for (int i = 0; i < NR / 8; ++i) {    // even lanes: z[2i], odd lanes: z[2i + 1]
            const A keep = b0 ? z[2 * i + 1] : z[2 * i], give = b0 ? z[2 * i] : z[2 * i + 1];
            y[i] = keep + dpp_mov<kDppXor1>(give);
        }
        if constexpr (NR == 8) {
            A s = y[0];
            s += dpp_mov<kDppXor2>(s);
            s += dpp_mov<kDppRor8>(s);
            s += dpp_mov<kDppRor4>(s);
            return s;
        } else {
            const bool b1 = lane & 2;
            A t[NR / 16];
#pragma unroll
            for (int i = 0; i < NR / 16; ++i) {   // lanes with bit 1 clear: y[2i], set: y[2i + 1]
                const A keep = b1 ? y[2 * i + 1] : y[2 * i], give = b1 ? y[2 * i] : y[2 * i + 1];
                t[i] = keep + dpp_mov<kDppXor2>(give);
            }
#pragma unroll
            for (int i = 0; i < NR / 16; ++i) {   // lanes l, l+4, l+8, l+12 of a row of 16
                t[i] += dpp_mov<kDppRor8>(t[i]);
                t[i] += dpp_mov<kDppRor4>(t[i]);
            }
            if constexpr (NR == 16) return t[0];
            else return (lane & 8) ? t[1] : t[0];
        }
    }
}

// Sum over a thread block of NW wavefronts in fixed wave order; every thread gets the result.
// `slots` is LDS room for NW values and may be reused after the call returns.
template <int NW, typename A>
__device__ __forceinline__ A block_sum(A v, A* slots)
{
    const A w = wave_sum(v);
    const int wave = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) slots[wave] = w;
    __syncthreads();
    A s = slots[0];
#pragma unroll
    for (int k = 1; k < NW; ++k) s += slots[k];
    return s;
}

// ------------------------------------------------------------------------------------------------
// Argument checks and the alpha == 0 case shared by the level-2 routines.
inline bool layout_ok(int v) { return v == MXB_ROW_MAJOR || v == MXB_COL_MAJOR; }
inline bool trans_ok(int v) { return v == MXB_NO_TRANS || v == MXB_TRANS; }
inline bool uplo_ok(int v) { return v == MXB_UPPER || v == MXB_LOWER; }
inline bool diag_ok(int v) { return v == MXB_NON_UNIT || v == MXB_UNIT; }

// y[k] = beta*y[k] (zeros when beta == 0, without reading y): what gemv and symv leave of y when
// alpha == 0.  blockIdx.y: problem of a batch, sy elements apart.
template <typename T>
__global__ void __launch_bounds__(256) scale_y_kernel(int64_t n, T beta, T* __restrict__ y, int64_t incy, int64_t sy)
{
    y += (int64_t)blockIdx.y * sy;
    const int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (k < n) y[k * incy] = beta == T(0) ? T(0) : beta * y[k * incy];
}

}  // namespace mxb
