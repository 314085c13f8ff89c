// trsv (Sec. 6.2.2, triangular solve) on a row-major matrix: blocked substitution.  The part of
// a block's right-hand side that depends on unknowns solved earlier is subtracted with the
// matrix-vector kernels of matvec.hip; the block on the diagonal is solved by one workgroup.
#include <type_traits>

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
    __shared__ __attribute__((aligned(16))) T xs[NW * kWave];
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
    // Row i is scaled by 1 / T[i][i] once, so that the chain of 64 dependent steps below is one
    // broadcast and one FMA per step: with c = b / T[i][i] the unknown j is c of lane j when its
    // turn comes, and c no longer changes after a lane's own turn (its row is zero from there).
    T dv = T(1);
#pragma unroll
    for (int j = 0; j < kWave; ++j) dv = (!UNIT && active && j == lane) ? e[j] : dv;
    const T rinv = T(1) / dv;      // 1 in the lanes past the block: their zeros stay zeros
#pragma unroll
    for (int j = 0; j < kWave; ++j) {
        const bool inside = OPLOWER ? j < lane : j > lane;
        e[j] = inside ? (UNIT ? e[j] : e[j] * rinv) : T(0);
    }
    // (The chained kernel's four unknowns per step do not pay here: the premultiplication of the rows, which
    // that kernel does while it waits, costs one solve more than it saves: n = 64 in 9.2 us instead of 6.8.)

    for (int step = 0; step < nsub; ++step) {
        const int s = OPLOWER ? step : nsub - 1 - step;
        const bool later = OPLOWER ? wave > s : wave < s;
        T ev[kWave];
        if (wave == s) {
            T c = UNIT ? b : b * rinv;
#pragma unroll
            for (int jj = 0; jj < kWave; ++jj) {
                const int j = OPLOWER ? jj : kWave - 1 - jj;
                c = fmad(-e[j], lane_bcast(c, j), c);
            }
            xs[i] = c;
            if (active) p.x[(int64_t)i * p.incx] = c;
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
    // only the wavefronts that own unknowns: the others would still fetch and turn their (empty) tiles
    const dim3 grid(1), block((unsigned)(ceil_div((int64_t)a.nb, (int64_t)kWave) * kWave));
    if (op_lower) {
        if (unit) hipLaunchKernelGGL((trsv_diag_kernel<T, NW, true, TRANS, true>), grid, block, 0, h->stream, a);
        else hipLaunchKernelGGL((trsv_diag_kernel<T, NW, true, TRANS, false>), grid, block, 0, h->stream, a);
    } else {
        if (unit) hipLaunchKernelGGL((trsv_diag_kernel<T, NW, false, TRANS, true>), grid, block, 0, h->stream, a);
        else hipLaunchKernelGGL((trsv_diag_kernel<T, NW, false, TRANS, false>), grid, block, 0, h->stream, a);
    }
}

// ---------------------------------------------------------------------------------------------
// The same substitution in ONE kernel: no launch per block, and the off-diagonal work of a block
// of rows overlaps the solves of the blocks before it.
//
// A workgroup of 2 wavefronts owns 128 consecutive unknowns, one sub-block of 64 per wavefront,
// in solving order.  Workgroups number themselves with a ticket when they start, so that every
// workgroup with a smaller number is already running or done.  A wavefront first subtracts,
// sub-block by sub-block, the part of its rows that multiplies unknowns owned by earlier
// workgroups: the 64 x 64 tile is fetched while the wavefront waits for that sub-block's
// solutions.  The sub-blocks of the workgroup itself are then solved as in the blocked kernel
// above (LDS and barriers), each one handed on as soon as it is solved.
//
// Every wavefront has to take one tile per sub-block that the chain solves, so the chain runs
// no faster than the slowest wavefront gets through a tile.  That, not the hand-over, was the
// limit while a tile was 64 loads of one element per lane (per tile: 0.8 to 1.2 us to issue the
// loads, 0.3 to 0.6 us of polls queued behind them, since loads return in order, and 0.5 us of
// broadcasts and multiply-adds when transposed; the wavefront that a workgroup's first solve
// waits for began to look for the last solutions 3 us after they were there).  The streamed tiles
// are therefore read with 128-bit loads, 16 per tile, whatever the pitch and the base address
// (a matrix load needs element alignment only; rows that begin off a 16-byte boundary cost nothing
// measurable: n = 8192, lda = 8193 against 8196: 144.5 / 130.7 against 145.2 / 129.8 us, and the
// element-wise loads that used to serve them took 226 / 185).
//
// Solutions travel between workgroups in words that validate themselves: the solver stores
// {value bits, tag} as one 64-bit device-scope atomic (two words, one per half, for a double), a
// reader loads the word the same way and takes the value once the tag is there.  No fence is
// needed on either side, so no cache is written back or invalidated on the way (the compute
// dies have a second-level cache each, and a device-scope fence has to reach through it); the
// solutions go to x as well, with plain stores, for the caller.  Waits are bounded: a wavefront
// that polls longer than the limit, or sees the error word set, sets the error word and goes on
// without waiting, so the kernel always drains (the result is then wrong; it cannot happen while
// every workgroup makes progress, because a workgroup only ever waits for workgroups that
// started before it).
template <typename T>
struct Handover;
template <>
struct Handover<float> {
    static constexpr int kWords = 1;
    static __device__ __forceinline__ void put(unsigned long long* w, float v)
    {
        __hip_atomic_store(w, (1ull << 32) | __float_as_uint(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    // the load and the reading of what came back are apart, so that a caller can ask, do other
    // things, and only then wait for the answer
    struct Raw { unsigned long long u; };
    static __device__ __forceinline__ Raw ask(unsigned long long* w)
    {
        return Raw{__hip_atomic_load(w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)};
    }
    static __device__ __forceinline__ bool read(const Raw& r, float& v)
    {
        v = __uint_as_float((unsigned)r.u);
        return (r.u >> 32) != 0;
    }
    static __device__ __forceinline__ bool get(unsigned long long* w, float& v) { return read(ask(w), v); }
};
template <>
struct Handover<double> {
    static constexpr int kWords = 2;
    static __device__ __forceinline__ void put(unsigned long long* w, double v)
    {
        const unsigned long long bits = (unsigned long long)__double_as_longlong(v);
        __hip_atomic_store(w, (1ull << 32) | (bits & 0xffffffffull), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(w + 1, (1ull << 32) | (bits >> 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    struct Raw { unsigned long long lo, hi; };
    static __device__ __forceinline__ Raw ask(unsigned long long* w)
    {
        return Raw{__hip_atomic_load(w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT),
                   __hip_atomic_load(w + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)};
    }
    static __device__ __forceinline__ bool read(const Raw& r, double& v)
    {
        v = __longlong_as_double((long long)((r.hi << 32) | (r.lo & 0xffffffffull)));
        return (r.lo >> 32) != 0 && (r.hi >> 32) != 0;
    }
    static __device__ __forceinline__ bool get(unsigned long long* w, double& v) { return read(ask(w), v); }
};

// the value of lane s of each lane's group of four
template <typename T>
__device__ __forceinline__ T quad_bcast(T v, int s)
{
    switch (s) {
        case 0: return dpp_mov<0x00>(v);
        case 1: return dpp_mov<0x55>(v);
        case 2: return dpp_mov<0xAA>(v);
        default: return dpp_mov<0xFF>(v);
    }
}

template <typename T>
struct ChainArgs {
    int n, nsub;         // unknowns; sub-blocks of 64
    const T* A;
    int64_t lda;
    T* x;                // logical element 0
    int64_t incx;
    unsigned long long* solved;   // [nsub * 64 * Handover<T>::kWords] hand-over words in solving order; all zero at the start
    int* control;        // the ticket counter and the error word; zero at the start
    int spin_limit;
};


__global__ void __launch_bounds__(256) trsv_chain_init_kernel(int* words, int count)
{
    const int k = (int)blockIdx.x * 256 + threadIdx.x;
    if (k < count) words[k] = 0;
}

// raw[k] = A[min(first + k, last)][col], k < COUNT; first is the same for the whole wavefront.
// Buffer loads: the descriptor holds the address of row `first`, the lane's column is the vector
// offset (the same for every row) and the row is a scalar offset that grows by one pitch per
// load, so a load costs one scalar addition beside itself (with flat addresses: a 64-bit vector
// addition and half a dozen scalar instructions, and a wavefront alone on its SIMD unit issues
// one instruction every four or five cycles: asking for a tile then took 1.4 to 1.7 us, more than
// the solve of a sub-block).  All addresses are clamped into the matrix, so the descriptor's own
// range check is left wide open.  The scalar offset is 32 bits: the caller makes sure that COUNT
// rows are less than 2^31 bytes apart.  The empty asm keeps the compiler from forming all COUNT
// offsets ahead of the loops around the call and holding them in scalar registers.
__device__ __forceinline__ float buffer_load(__amdgpu_buffer_rsrc_t r, int voff, int soff, float)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0));
}
__device__ __forceinline__ double buffer_load(__amdgpu_buffer_rsrc_t r, int voff, int soff, double)
{
    return __builtin_bit_cast(double, __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, 0));
}
constexpr int kBufferRawDword3 = 0x00020000;      // 32-bit raw data, no swizzle
template <typename T, int COUNT>
__device__ __forceinline__ void load_rows(const T* A, int64_t lda, int first, int last, int col, T (&raw)[COUNT])
{
    asm volatile("" : "+s"(first));
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(A + (int64_t)min(first, last) * lda), 0, -1, kBufferRawDword3);
    const int voff = col * (int)sizeof(T), pitch = (int)lda * (int)sizeof(T);
    int soff = 0;
    if (first + COUNT - 1 <= last) {
#pragma unroll
        for (int k = 0; k < COUNT; ++k) {
            raw[k] = buffer_load(rsrc, voff, soff, T());
            soff += pitch;
            asm volatile("" : "+s"(soff));
        }
    } else {
#pragma unroll
        for (int k = 0; k < COUNT; ++k) {
            raw[k] = buffer_load(rsrc, voff, soff, T());
            soff += first + k < last ? pitch : 0;
            asm volatile("" : "+s"(soff));
        }
    }
}

// Wavefronts per workgroup of the chained kernel.  A step from one sub-block to the next costs
// 0.45 us inside a workgroup (LDS, one barrier) and 1.3 us between workgroups, beside 0.6 us of
// solve, which speaks for large workgroups; but the wavefronts of a workgroup share a compute unit
// and its path to memory, all of them ask for a tile at the same moment, and the other compute
// units idle.  Measured at n = 16384, single precision, not transposed / transposed, element-wise
// loads: 4 wavefronts 615 / 502 us, 2: 531 / 455, 1: 554 / 486; 128-bit loads: 4: 425 / 449, 2: 401 /
// 364, 1: 457 / 423.  (8 wavefronts are two per SIMD unit, 256 registers each: the kernel then spills
// 260 to 620 of them.  Handing the unknowns on through LDS in groups of 16 as they become final,
// with the others polling instead of a barrier, or one LDS flag per sub-block in place of the
// barrier, were both slower than the barrier.)
template <typename T, bool TRANS>
constexpr int chain_waves() { return 2; }

template <typename T, bool OPLOWER, bool TRANS, bool UNIT, bool AHEAD>
__global__ void __launch_bounds__((chain_waves<T, TRANS>() * kWave)) trsv_chain_kernel(const ChainArgs<T> p)
{
    constexpr int NW = chain_waves<T, TRANS>();
    constexpr int V = 16 / (int)sizeof(T);       // elements of a 128-bit load
    __shared__ __attribute__((aligned(16))) T xs[NW * kWave];
    __shared__ __attribute__((aligned(16))) T fold[TRANS ? NW : 1][TRANS ? V * kWave : 1];
    // Per-wavefront buffers.  tile: turns a tile when not transposed (row-wise loads, a lane wants its row).
    // park: in double precision, where the registers are short, the wavefront's finished diagonal rows.
    // near_park: transposed, the tile next to the workgroup's own while the others stream; not transposed
    // that tile waits in tile[] (double precision) or in registers (single; transposed, the single
    // precision kernel would spill 4 to 23 registers with it, and 14 are enough to take n = 4096 from
    // 72 to 105 us).  fold / foldn: the partial sums on their way from lane = column to lane = unknown.
    constexpr bool kPark = sizeof(T) == 8;
    constexpr bool kParkNear = TRANS || sizeof(T) == 8;      // single precision, not transposed: it stays in registers
    __shared__ __attribute__((aligned(16))) T tile[TRANS ? 1 : NW][TRANS ? 1 : kWave][TRANS ? 1 : kWave + 1];
    __shared__ T park[kPark ? NW : 1][kPark ? kWave : 1][kPark ? kWave + 1 : 1];
    __shared__ T near_park[TRANS ? NW : 1][TRANS ? kWave : 1][TRANS ? kWave + 1 : 1];      // (not transposed: in tile[])
    constexpr int kFoldRows = sizeof(T) == 4 ? kWave : kWave / 2;       // unknowns folded in one pass (a piece of a tile)
    __shared__ __attribute__((aligned(16))) T foldn[TRANS ? 1 : NW][TRANS ? 1 : (kWave / V) * (kFoldRows + V)];
    __shared__ int my_ticket;
    constexpr int HW = Handover<T>::kWords;
    int* const ticket = p.control;
    int* const error = p.control + 1;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (threadIdx.x == 0) my_ticket = atomicAdd(ticket, 1);
    __syncthreads();
    const int q0 = my_ticket * NW;       // my workgroup's sub-blocks q0 .. q0 + NW - 1, counted in solving order
    const int q = q0 + wave;
    const bool have = q < p.nsub;        // false: a wavefront past the last sub-block only keeps the barriers company
    auto actual = [&](int qq) { return OPLOWER ? qq : p.nsub - 1 - qq; };      // sub-block number in the matrix
    const int r0 = actual(have ? q : p.nsub - 1) * kWave;                       // my rows: r0 .. r0 + 63
    const int i = r0 + lane, last = p.n - 1;
    const bool active = have && i < p.n;

    // raw[j] = op(T)[r0 + lane][c0 + j], in two halves as the tile is in flight between them:
    // issue() starts the 64 loads (addresses clamped into the matrix: no predicate), finish() pins
    // them, zeroes what lies outside the matrix and, if not transposed, turns the tile through LDS.
    auto issue = [&](int c0, T (&raw)[kWave]) {
        if (TRANS) load_rows(p.A, p.lda, c0, last, min(i, last), raw);
        else load_rows(p.A, p.lda, r0, last, min(c0 + lane, last), raw);
    };
    auto finish = [&](int c0, T (&raw)[kWave]) {
#pragma unroll
        for (int j = 0; j < kWave; ++j) asm volatile("" : "+v"(raw[j]));
        if (TRANS) {
#pragma unroll
            for (int j = 0; j < kWave; ++j) raw[j] = (active && c0 + j < p.n) ? raw[j] : T(0);
        } else {
            __builtin_amdgcn_wave_barrier();      // earlier reads of the buffer by this wavefront come first
#pragma unroll
            for (int r = 0; r < kWave; ++r)
                tile[TRANS ? 0 : wave][TRANS ? 0 : r][TRANS ? 0 : lane] = (have && r0 + r < p.n && c0 + lane < p.n) ? raw[r] : T(0);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int j = 0; j < kWave; ++j) raw[j] = tile[TRANS ? 0 : wave][TRANS ? 0 : lane][TRANS ? 0 : j];
        }
    };

    T b = active ? p.x[(int64_t)i * p.incx] : T(0);
    T e[kWave];
    issue(r0, e);                        // my tile on the diagonal

    // Tile s of my own workgroup (s = 0 .. wave - 1) multiplies the sub-block solved in step s.
    // Two of them are in flight at any time, in pa and pb by turns: the first two are asked for
    // right away and travel during the whole first phase, tile s + 2 is asked for when tile s has
    // been used, so that a tile has two steps to arrive.
    T pa[kWave], pb[kWave];
    auto own_c0 = [&](int s) { return actual(q0 + s) * kWave; };
    auto wants = [&](int s) { return s < NW - 1 && have && wave > s && q0 + s < p.nsub; };
    if (wants(0)) issue(own_c0(0), pa);
    if (wants(1)) issue(own_c0(1), pb);
    // The last tile before my workgroup's own, the one whose solutions arrive last and that the first
    // solve of the workgroup waits for, is taken like a tile of my own workgroup: fetched now, turned
    // so that a lane holds its row, and applied from LDS when the solutions are there.  Except in
    // single precision when not transposed, where the registers hold it, it waits in LDS while the
    // other tiles stream (not transposed: in the turning buffer, which nothing else needs until then).
    T pc[kWave];
    const bool near_tile = have && q0 > 0;
    if (near_tile) issue(actual(q0 - 1) * kWave, pc);

    // My row of the diagonal tile, scaled by 1 / T[i][i] as in the blocked kernel.  Before the
    // wait for the earlier workgroups, which is where a workgroup has time to spare: in single
    // precision it stays in registers; in double precision it would not (the compiler would fetch
    // it back from scratch memory one element at a time inside the solve), so it is parked in LDS.
    finish(r0, e);
    T dv = T(1);
#pragma unroll
    for (int j = 0; j < kWave; ++j) dv = (!UNIT && active && j == lane) ? e[j] : dv;
    const T rinv = T(1) / dv;            // 1 in the lanes past the end: their zeros stay zeros
#pragma unroll
    for (int j = 0; j < kWave; ++j) {
        const bool inside = OPLOWER ? j < lane : j > lane;
        e[j] = inside ? (UNIT ? e[j] : e[j] * rinv) : T(0);
    }
    // Four unknowns per step of the substitution: the rows of every group of four lanes are
    // multiplied by the inverse of the group's own 4 x 4 unit triangle (held by the group itself:
    // quad permutes), which makes that triangle the identity.  The four unknowns of a group then no
    // longer depend on each other, and a step is four independent broadcasts and four multiply-adds
    // instead of four rounds of broadcast-then-multiply-add, each waiting for the one before.  The
    // right-hand side takes the same 4 x 4 product when the solve begins (qinv).
    T qinv[4];
    {
        const int r = lane & 3;
        T nq[4] = {T(0), T(0), T(0), T(0)};      // my row of my group's triangle, without the diagonal
#pragma unroll
        for (int j = 0; j < kWave; ++j) nq[j & 3] = (j >> 2) == (lane >> 2) ? e[j] : nq[j & 3];
#pragma unroll
        for (int k = 0; k < 4; ++k) qinv[k] = k == r ? T(1) : T(0);
        // row r of the inverse: unit vector r minus the earlier (lower) or later (upper) rows, each final in its turn
#pragma unroll
        for (int ss = 0; ss < 3; ++ss) {
            const int sidx = OPLOWER ? ss : 3 - ss;
            const T coef = (OPLOWER ? r > sidx : r < sidx) ? nq[sidx] : T(0);
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (OPLOWER ? k <= sidx : k >= sidx) qinv[k] = fmad(-coef, quad_bcast(qinv[k], sidx), qinv[k]);
        }
#pragma unroll
        for (int j = 0; j < kWave; ++j) {
            const bool beyond = OPLOWER ? j < (lane & ~3) : j > (lane | 3);      // outside my group's triangle
            T v = qinv[0] * quad_bcast(e[j], 0);
#pragma unroll
            for (int k = 1; k < 4; ++k) v = fmad(qinv[k], quad_bcast(e[j], k), v);
            e[j] = beyond ? v : T(0);
            if constexpr (kPark) park[wave][j][lane] = e[j];      // read back by this lane only
            else asm volatile("" : "+v"(e[j]));                   // here, not when the solve needs it
        }
    }
    // the first two tiles of my own workgroup are made ready now as well: turning a tile through LDS
    // between two steps takes a wavefront longer than the solving wavefront needs for its step
    if (wants(0)) finish(own_c0(0), pa);
    if (wants(1)) finish(own_c0(1), pb);
    {
        if (near_tile) {
            finish(actual(q0 - 1) * kWave, pc);
            if constexpr (kParkNear) {            // read back by this lane only
                if constexpr (!TRANS) __builtin_amdgcn_wave_barrier();      // finish() has read the turning buffer
#pragma unroll
                for (int j = 0; j < kWave; ++j) {
                    if constexpr (TRANS) near_park[TRANS ? wave : 0][TRANS ? j : 0][TRANS ? lane : 0] = pc[j];
                    else tile[TRANS ? 0 : wave][TRANS ? 0 : j][TRANS ? 0 : lane] = pc[j];
                }
            }
        }
    }

    // ---- the unknowns of earlier workgroups: tiles 0 .. q0 - 1 of my block row, in solving order.
    // A tile travels in pieces of RH memory rows, two pieces in flight by turns; the 64 solutions a
    // tile multiplies are waited for when its first piece is used.
    bool ok = true;
    auto look = [&](int qq, T& xv) { return Handover<T>::get(p.solved + ((int64_t)qq * kWave + lane) * HW, xv); };
    auto wait_x = [&](int qq, T& xv, bool got) {
        for (int spins = 0; ok && __ballot(got) != ~0ull;) {
            // (the error word every 64th round only: a round would otherwise be two trips to memory, one after the
            // other; from the last solution of a workgroup to the first of the next: 4.3 -> 3.4 us)
            if (++spins > p.spin_limit || (spins % 64 == 0 && __hip_atomic_load(error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)) {
                ok = false;
                if (lane == 0) __hip_atomic_store(error, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                break;
            }
            __builtin_amdgcn_s_sleep(1);
            got = look(qq, xv);
        }
    };
    {
      const int nstream = q0 - 1;                 // tiles taken by the streaming loop: all but the near one
      if (have && nstream > 0) {
        // 128-bit loads: lane (g, m), g = lane / CG, m = lane % CG, fetches for t < NL the V elements
        // at memory row row0 + g * NL + t, columns col0 + m * V .., of a piece of RH = V * NL rows, so
        // a piece is NL loads instead of RH (a wavefront alone on its SIMD unit issues slowly, and
        // asking for the tiles is what the streaming wavefronts spend their time on).  Transposed,
        // the rows of the piece are solved unknowns and the columns mine: a lane keeps V partial
        // sums, for unknowns m * V .., over the rows it loads.  Not transposed, the rows are my
        // unknowns: a lane keeps one partial sum per row it loads, over its V columns.  Either way
        // the partial sums are folded over the lanes once, through LDS, after the last tile, and
        // the 64 solutions a tile multiplies reach the lanes that need them through LDS.
        constexpr int CG = kWave / V;
        constexpr int RH = sizeof(T) == 4 ? kWave : kWave / 2;
        constexpr int CPT = kWave / RH, NL = RH / V;
        typedef T vec_t __attribute__((ext_vector_type(V)));
        const int m = lane % CG, g = lane / CG;
        const int pitch = (int)p.lda * (int)sizeof(T);
        const int lastvec = last / V * V;
        const int voff_inside = g * NL * pitch + m * V * (int)sizeof(T);
        T* const xb = xs + wave * kWave;          // my slot of xs is free until my own solve
        auto startv = [&](int ch, vec_t (&raw)[NL]) {
            const int cblk = actual(ch / CPT) * kWave, h0 = (ch % CPT) * RH;
            int row0 = (TRANS ? cblk : r0) + h0;
            const int col0 = TRANS ? r0 : cblk;
            asm volatile("" : "+s"(row0));
            const int rowb = min(row0, last);
            const __amdgpu_buffer_rsrc_t rsrc =
                __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(p.A + (int64_t)rowb * p.lda + col0), 0, -1, kBufferRawDword3);
            if (row0 + RH <= p.n && col0 + kWave <= p.n) {
                int soff = 0;
#pragma unroll
                for (int t = 0; t < NL; ++t) {
                    raw[t] = __builtin_bit_cast(vec_t, __builtin_amdgcn_raw_buffer_load_b128(rsrc, voff_inside, soff, 0));
                    soff += pitch;
                    asm volatile("" : "+s"(soff));
                }
            } else {      // the last rows or columns of the matrix: addresses clamped into it, lane by lane
                const int cofs = (min(col0 + m * V, lastvec) - col0) * (int)sizeof(T);
#pragma unroll
                for (int t = 0; t < NL; ++t) {
                    const int r = min(row0 + g * NL + t, last) - rowb;
                    raw[t] = __builtin_bit_cast(vec_t, __builtin_amdgcn_raw_buffer_load_b128(rsrc, r * pitch + cofs, 0, 0));
                }
            }
        };
        T pv[V];
        T acc[TRANS ? 1 : CG];
        vec_t xmine;                              // not transposed: the V solutions my columns multiply
#pragma unroll
        for (int v = 0; v < V; ++v) { pv[v] = T(0); xmine[v] = T(0); }
        if (!TRANS) {
#pragma unroll
            for (int k = 0; k < CG; ++k) acc[TRANS ? 0 : k] = T(0);
        }
        // Where memory is slow to answer (AHEAD: a matrix larger than the last-level cache), the
        // solutions of the next tile are asked for once before the next piece is, and the answer is
        // read after.  Loads return in order, so a poll behind a piece just asked for comes back when
        // the piece does, and a wavefront that has fallen behind the chain, whose solutions are there
        // already, would wait for the piece for nothing; a wait for the answer before the next piece
        // is asked for would wait for the piece before it, leaving one piece in flight instead of
        // two.  (n = 16384, transposed: 361 -> 340 us, double precision 700 -> 636 and 698 -> 665; smaller
        // matrices lose: n = 4096 transposed 73 -> 77 us.)
        auto ask_x = [&](int qq) { return Handover<T>::ask(p.solved + ((int64_t)qq * kWave + lane) * HW); };
        typename Handover<T>::Raw ahead;
        if (AHEAD) ahead = ask_x(0);

        auto usev = [&](auto piece, int ch, vec_t (&raw)[NL]) {
            constexpr int PIECE = decltype(piece)::value, H0 = PIECE * RH;
            const int qq = ch / CPT, cblk = actual(qq) * kWave;
            const int row0 = (TRANS ? cblk : r0) + H0, col0 = TRANS ? r0 : cblk;
            if (PIECE == 0) {
                T xv;
                const bool got = AHEAD ? Handover<T>::read(ahead, xv) : look(qq, xv);
                wait_x(qq, xv, got);
                __builtin_amdgcn_wave_barrier();      // my earlier reads of the buffer come first
                xb[lane] = xv;
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                if (!TRANS) xmine = *reinterpret_cast<const vec_t*>(xb + m * V);
            }
#pragma unroll
            for (int t = 0; t < NL; ++t) asm volatile("" : "+v"(raw[t]));
            if (row0 + RH > p.n || col0 + kWave > p.n) {
#pragma unroll
                for (int t = 0; t < NL; ++t)
#pragma unroll
                    for (int v = 0; v < V; ++v)
                        raw[t][v] = (row0 + g * NL + t < p.n && col0 + m * V + v < p.n) ? raw[t][v] : T(0);
            }
            if (TRANS) {
#pragma unroll
                for (int t = 0; t < NL; t += V) {
                    const vec_t xq = *reinterpret_cast<const vec_t*>(xb + H0 + g * NL + t);
#pragma unroll
                    for (int u = 0; u < V; ++u)
#pragma unroll
                        for (int v = 0; v < V; ++v) pv[v] = fmad(raw[t + u][v], xq[u], pv[v]);
                }
            } else {
#pragma unroll
                for (int t = 0; t < NL; ++t) {
                    T sum = acc[TRANS ? 0 : PIECE * NL + t];
#pragma unroll
                    for (int v = 0; v < V; ++v) sum = fmad(raw[t][v], xmine[v], sum);
                    acc[TRANS ? 0 : PIECE * NL + t] = sum;
                }
            }
            if (AHEAD && PIECE == CPT - 1 && qq + 1 < nstream) ahead = ask_x(qq + 1);
        };
        const int nch = nstream * CPT;
        vec_t t0[NL], t1[NL];
        startv(0, t0);
        if (nch > 1) startv(1, t1);
        int ch = 0;
        for (; ch + 1 < nch; ch += 2) {
            usev(std::integral_constant<int, 0>(), ch, t0);
            if (ch + 2 < nch) startv(ch + 2, t0);
            usev(std::integral_constant<int, CPT - 1>(), ch + 1, t1);
            if (ch + 3 < nch) startv(ch + 3, t1);
        }
        if (ch < nch) usev(std::integral_constant<int, 0>(), ch, t0);
        // the partial sums, folded over the lanes: lane = unknown from here on
        __builtin_amdgcn_wave_barrier();
        if (TRANS) {
            T* const red = &fold[TRANS ? wave : 0][0];
            vec_t out;
#pragma unroll
            for (int v = 0; v < V; ++v) out[v] = pv[v];
            *reinterpret_cast<vec_t*>(red + (TRANS ? g * kWave + m * V : 0)) = out;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            T sum = T(0);
#pragma unroll
            for (int gg = 0; gg < V; ++gg) sum += red[TRANS ? gg * kWave + lane : 0];
            b -= sum;
        } else {
            // unknown h * RH + g * NL + t is acc[h * NL + t] of the lanes (g, 0 .. CG - 1): one pass per piece h of
            // a tile (the buffer is small because the turning buffer may hold the near tile meanwhile); rows of
            // the buffer V apart from a power of two, so that the 128-bit stores spread over the banks
            static_assert(RH == kFoldRows, "a pass folds the unknowns of one piece");
            constexpr int STRIDE = RH + V;
            T* const red = &foldn[TRANS ? 0 : wave][0];
#pragma unroll
            for (int h = 0; h < CPT; ++h) {
                __builtin_amdgcn_wave_barrier();      // the pass before has read the buffer
#pragma unroll
                for (int t = 0; t < NL; t += V) {
                    vec_t out;
#pragma unroll
                    for (int v = 0; v < V; ++v) out[v] = acc[TRANS ? 0 : h * NL + t + v];
                    *reinterpret_cast<vec_t*>(red + (TRANS ? 0 : m * STRIDE + g * NL + t)) = out;
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                const int u = lane - h * RH;
                if (u >= 0 && u < RH) {
                    T part[4] = {T(0), T(0), T(0), T(0)};
#pragma unroll
                    for (int mm = 0; mm < CG; ++mm) part[mm & 3] += red[TRANS ? 0 : mm * STRIDE + u];
                    b -= (part[0] + part[1]) + (part[2] + part[3]);
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
      }
      {
        if (near_tile) {
            T* const xb = xs + wave * kWave;
            if constexpr (kParkNear) {            // back into the registers that the streamed tiles have left
#pragma unroll
                for (int j = 0; j < kWave; ++j) {
                    if constexpr (TRANS) pc[j] = near_park[TRANS ? wave : 0][TRANS ? j : 0][TRANS ? lane : 0];
                    else pc[j] = tile[TRANS ? 0 : wave][TRANS ? 0 : j][TRANS ? 0 : lane];
                }
#pragma unroll
                for (int j = 0; j < kWave; ++j) asm volatile("" : "+v"(pc[j]));
            }
            T xv;
            const bool got = look(q0 - 1, xv);
            wait_x(q0 - 1, xv, got);
            __builtin_amdgcn_wave_barrier();
            xb[lane] = xv;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            T part[4] = {T(0), T(0), T(0), T(0)};
#pragma unroll
            for (int j = 0; j < kWave; ++j) part[j & 3] = fmad(pc[j], xb[j], part[j & 3]);
            b -= (part[0] + part[1]) + (part[2] + part[3]);
        }
      }
    }

    // ---- my workgroup's own sub-blocks.  One step: sub-block q0 + s is solved by wavefront s and
    // handed on at once, while the wavefronts after it get their tile ready; after the barrier
    // they subtract its part.  Only LDS traffic is fenced around the barrier: the tiles still in
    // flight from global memory must not be waited for there.
    auto step = [&](int s, T (&tile_s)[kWave]) {
        if (q0 + s >= p.nsub) return;    // the same for the whole workgroup
        if (wave == s) {
            T c = UNIT ? b : b * rinv;
            {
                T t = qinv[0] * quad_bcast(c, 0);
#pragma unroll
                for (int k = 1; k < 4; ++k) t = fmad(qinv[k], quad_bcast(c, k), t);
                c = t;
            }
            auto column = [](int jj) { return OPLOWER ? jj : kWave - 1 - jj; };
            if constexpr (kPark) {
                // the parked row comes back in groups of kGroup, each asked for one group ahead of the
                // steps that use it (left to itself the compiler reads each element right before its
                // step, and the chain of dependent steps waits for LDS every time)
                constexpr int kGroup = 8;
                T eb[2][kGroup];
#pragma unroll
                for (int k = 0; k < kGroup; ++k) eb[0][k] = park[wave][column(k)][lane];
#pragma unroll
                for (int j0 = 0; j0 < kWave; j0 += kGroup) {
                    if (j0 + kGroup < kWave) {
#pragma unroll
                        for (int k = 0; k < kGroup; ++k) eb[(j0 / kGroup + 1) & 1][k] = park[wave][column(j0 + kGroup + k)][lane];
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int k0 = 0; k0 < kGroup; k0 += 4) {
                        T xq[4];
#pragma unroll
                        for (int k = 0; k < 4; ++k) xq[k] = lane_bcast(c, column(j0 + k0 + k));
#pragma unroll
                        for (int k = 0; k < 4; ++k) c = fmad(-eb[(j0 / kGroup) & 1][k0 + k], xq[k], c);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else {
#pragma unroll
                for (int j0 = 0; j0 < kWave; j0 += 4) {
                    T xq[4];
#pragma unroll
                    for (int k = 0; k < 4; ++k) xq[k] = lane_bcast(c, column(j0 + k));
#pragma unroll
                    for (int k = 0; k < 4; ++k) c = fmad(-e[column(j0 + k)], xq[k], c);
                }
            }
            xs[wave * kWave + lane] = c;
            Handover<T>::put(p.solved + ((int64_t)q * kWave + lane) * HW, c);     // all 64, zeros past the end
            if (active) p.x[(int64_t)i * p.incx] = c;
        } else if (s >= 2 && wants(s)) {
            finish(own_c0(s), tile_s);       // tiles 0 and 1 were made ready at the start
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
        if (wants(s)) {
            T part[4] = {T(0), T(0), T(0), T(0)};
#pragma unroll
            for (int j = 0; j < kWave; ++j) part[j & 3] = fmad(tile_s[j], xs[s * kWave + j], part[j & 3]);
            b -= (part[0] + part[1]) + (part[2] + part[3]);
            if (wants(s + 2)) issue(own_c0(s + 2), tile_s);
        }
    };
    static_assert(NW == 1 || NW == 2 || NW == 4, "two tile buffers by turns");
    step(0, pa);
    if constexpr (NW >= 2) step(1, pb);
    if constexpr (NW == 4) {
        step(2, pa);
        step(3, pb);
    }
}

// Workspace of the one-kernel solve: the hand-over words of every sub-block, then the ticket and
// the error word.
// From where asking ahead pays (see the kernel), MiB of matrix, [double precision][transposed]; per call, without
// against with: single precision not transposed (a tile follows the last one along the same rows, memory answers
// sooner) n = 2048 49.2 / 46.7 against 46.8 / 47.0 us (lower / upper), 8192 153 / 143 against 144 / 143; transposed 8192
// 131 against 141, 12288 263 against 232; double precision not transposed 6144 195 against 205, 8192 335 against
// 306; transposed 2048 70.8 against 70.5, 4096 129 against 126, 8192 309 against 274.
constexpr int kChainAskAheadMiB[2][2] = {{16, 384}, {384, 128}};

template <typename T>
inline size_t chain_bytes(int64_t n) { return (size_t)ceil_div(n, (int64_t)kWave) * kWave * Handover<T>::kWords * 8 + 2 * sizeof(int); }

template <typename T>
int trsv_chain(mxb_handle_t h, bool op_lower, bool no_trans, bool unit, int64_t n, const T* A, int64_t lda, T* x0, int64_t incx)
{
    const size_t bytes = chain_bytes<T>(n);
    void* ws = take_workspace(h, bytes);
    if (!ws) return MXB_ERR_WORKSPACE;
    const int64_t words = (int64_t)(bytes / sizeof(int));
    unsigned long long* solved = static_cast<unsigned long long*>(ws);
    int* control = static_cast<int*>(ws) + (words - 2);
    hipLaunchKernelGGL(trsv_chain_init_kernel, dim3((unsigned)ceil_div(words, (int64_t)256)), dim3(256), 0, h->stream,
                       static_cast<int*>(ws), (int)words);
    int st = launch_status();
    if (st != MXB_OK) return st;
    h->device_status = control + 1;
    int64_t spin_limit = option(h, MXB_OPT_TRSV_SPIN_LIMIT);
    if (spin_limit > (1 << 30)) spin_limit = 1 << 30;
    const bool ask_ahead = n * n * (int64_t)sizeof(T) >= ((int64_t)kChainAskAheadMiB[sizeof(T) == 8][!no_trans] << 20);
    const ChainArgs<T> a{(int)n, (int)ceil_div(n, (int64_t)kWave), A, lda, x0, incx, solved, control, (int)spin_limit};
#define MXB_CHAIN(LOW_, TR_)                                                                                          \
    {                                                                                                                 \
        constexpr int NW = chain_waves<T, TR_>();                                                                     \
        const dim3 grid((unsigned)ceil_div((int64_t)a.nsub, (int64_t)NW)), block(NW * kWave);                         \
        if (ask_ahead) {                                                                                              \
            if (unit) hipLaunchKernelGGL((trsv_chain_kernel<T, LOW_, TR_, true, true>), grid, block, 0, h->stream, a);        \
            else hipLaunchKernelGGL((trsv_chain_kernel<T, LOW_, TR_, false, true>), grid, block, 0, h->stream, a);            \
        } else {                                                                                                      \
            if (unit) hipLaunchKernelGGL((trsv_chain_kernel<T, LOW_, TR_, true, false>), grid, block, 0, h->stream, a);       \
            else hipLaunchKernelGGL((trsv_chain_kernel<T, LOW_, TR_, false, false>), grid, block, 0, h->stream, a);           \
        }                                                                                                             \
    }
    if (op_lower) { if (no_trans) { MXB_CHAIN(true, false) } else { MXB_CHAIN(true, true) } }
    else { if (no_trans) { MXB_CHAIN(false, false) } else { MXB_CHAIN(false, true) } }
#undef MXB_CHAIN
    return launch_status();
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
    // From where the chained kernel is faster than one launch per block (per call, 20 calls back to
    // back: n = 128 9.3 against 9.5 us in single precision, 8.5 against 8.0 transposed, 11.7 against 12.0
    // and 10.7 against 10.1 in double precision; n = 192: 10.8 / 9.9 / 13.8 / 12.4 against 12.3 / 10.9 / 16.9 /
    // 14.9; n = 512: 17.8 against 29.7).
    const int64_t chain_min = option(h, MXB_OPT_TRSV_CHAIN_MIN);
    // 32-bit counts in the chained kernel, and 64 rows of a tile within 2^31 bytes of each other; no such matrix fits the device anyway
    if (n >= chain_min && n < ((int64_t)1 << 24) && lda <= (((int64_t)1 << 25) / (int64_t)sizeof(T)))
        return trsv_chain<T>(h, op_lower, no_trans, unit, n, A, lda, x0, incx);
    h->device_status = nullptr;                      // nothing in the blocked path waits on the device
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
