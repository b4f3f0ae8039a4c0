// Conversion kernels for SMALL problems (Algorithm 1 lines 1-5; the scale vectors of Section 4.2).
// Below about 2048^3 a call is bound by the latency of its dependent kernel launches, not by
// memory or arithmetic: the general path takes seven launches for the conversion (row shifts;
// clear, column maxima, column sums, column finish; residues of A; residues of B).  Here it
// takes two, each covering both factors:
//   k_small_shifts    every workgroup owns whole vectors (one row, or a strip of 8 or 16
//                     columns), so the maximum and the integer sum of squares need neither
//                     atomics nor a buffer that has to be cleared first; the two passes read
//                     the operand twice, which at these sizes comes from the caches;
//   k_small_residues  the row-form and column-form workgroups of the general kernels, dealt
//                     to the two factors by workgroup index.
// Accurate mode uses the same two shapes for what precedes its product Cbar: k_small_maxbits
// (the first half of k_small_shifts) and k_small_residues in its "magnitude" form (Abar, Bbar).
// Results are identical to the general kernels': the shifts are exact integer functions of
// the data and the residues use the same device code.
#include <algorithm>

#include "oz2_convert.hpp"
#include "oz2_kernels.hpp"

namespace oz2 {
namespace {

using namespace dev;

// One factor: `vecs` vectors of `len` elements get one shift each; element h of vector v is
// X[v * ld + h] (k_contiguous) or X[h * ld + v].
template <typename T>
struct SmallSide {
    const T *X;
    int64_t ld, vecs, len;
    int32_t *t;                 // [vecs] shifts: written by k_small_shifts, read by k_small_residues
    unsigned long long *maxbits;   // [vecs] accurate mode: bits of max |x|, written by k_small_maxbits
    int8_t *out;                // residue slices [N][len_pad/64][vecs_pad][64]
    int64_t vecs_pad, len_pad;
    int k_contiguous;
    unsigned blocks;            // workgroups of this side in the launch at hand
};

template <typename T>
constexpr int strip_cols() { return 64 / (int)sizeof(T); }          // 64-byte row segments

__device__ inline int shift_from(uint64_t T_, int e, const ShiftArgs &sa) {
    int j = 0;
    while (j < sa.levels - 1 && T_ > sa.theta[j]) ++j;
    return (sa.f_max - j) - e;
}

#ifndef OZ2_SPLIT_MODULI_BELOW
#define OZ2_SPLIT_MODULI_BELOW 600
#endif
constexpr unsigned kSplitModuliBelow = OZ2_SPLIT_MODULI_BELOW;   // residue launches with fewer workgroups split the moduli

constexpr int kShiftThreads = 256;      // (1024 threads per workgroup were measured: slower at every size)
constexpr int kShiftWaves = kShiftThreads / kWave;

// Bits of max |x| over one contiguous vector (a row), by the whole workgroup; every thread
// receives the result.
template <typename T>
__device__ uint64_t row_max(const T *__restrict__ x, int64_t len, uint64_t *red) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint64_t mx = 0;
    for (int64_t h = threadIdx.x; h < len; h += kShiftThreads) {
        const uint64_t b = (uint64_t)__double_as_longlong(fabs((double)x[h]));
        mx = b > mx ? b : mx;
    }
    mx = wave_max(mx);
    if (lane == 0) red[wave] = mx;
    __syncthreads();
    mx = 0;
    for (int w = 0; w < kShiftWaves; ++w) mx = red[w] > mx ? red[w] : mx;
    __syncthreads();                                                  // red[] may be reused
    return mx;
}

// Shift of one row.
template <typename T>
__device__ void row_shift(const T *__restrict__ x, int64_t len, const ShiftArgs &sa, int32_t *t_out,
                          uint64_t *red) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t mx = row_max<T>(x, len, red);
    if (mx == 0) {                                                    // all-zero vector
        if (threadIdx.x == 0) *t_out = 0;
        return;
    }
    const int e = floor_log2_of_bits(mx);
    uint64_t sum = 0;
    for (int64_t h = threadIdx.x; h < len; h += kShiftThreads) {
        const uint64_t q = (uint64_t)ceil(ldexp(fabs((double)x[h]), 15 - e));
        sum += q * q;
    }
    sum = wave_sum(sum);
    if (lane == 0) red[wave] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint64_t T_ = 0;
        for (int w = 0; w < kShiftWaves; ++w) T_ += red[w];
        *t_out = shift_from(T_, e, sa);
    }
}

// A strip of COLS columns: thread -> (column, row lane); a wavefront reads 64-byte segments of
// 64 / COLS consecutive rows.  Partial results are combined across the row lanes of a wavefront
// by shuffles, across wavefronts through LDS (red: kShiftWaves x COLS entries).
// col_strip_max: every thread receives the bits of max |x| over its column (0 beyond `cols`).
template <typename T>
__device__ uint64_t col_strip_max(int64_t strip, const T *__restrict__ X, int64_t ld, int64_t cols,
                                  int64_t rows, uint64_t *red) {
    constexpr int COLS = strip_cols<T>(), LANES = kShiftThreads / COLS;
    const int cl = threadIdx.x % COLS, rl = threadIdx.x / COLS;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t c = strip * COLS + cl;
    const T *x = X + c;
    uint64_t mx = 0;
    if (c < cols) {
#pragma unroll 8
        for (int64_t r = rl; r < rows; r += LANES) {
            const uint64_t b = (uint64_t)__double_as_longlong(fabs((double)x[r * ld]));
            mx = b > mx ? b : mx;
        }
    }
    for (int off = COLS; off < kWave; off <<= 1) {                    // lanes with the same column
        const uint64_t o = __shfl_xor(mx, off, kWave);
        mx = o > mx ? o : mx;
    }
    if (lane < COLS) red[wave * COLS + cl] = mx;
    __syncthreads();
    mx = 0;
    for (int w = 0; w < kShiftWaves; ++w) {
        const uint64_t o = red[w * COLS + cl];
        mx = o > mx ? o : mx;
    }
    __syncthreads();                                                  // red[] may be reused
    return mx;
}

template <typename T>
__device__ void col_strip_shifts(int64_t strip, const T *__restrict__ X, int64_t ld, int64_t cols,
                                 int64_t rows, const ShiftArgs &sa, int32_t *t, uint64_t *red) {
    constexpr int COLS = strip_cols<T>(), LANES = kShiftThreads / COLS;
    const int cl = threadIdx.x % COLS, rl = threadIdx.x / COLS;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t c = strip * COLS + cl;
    const bool live = c < cols;
    const T *x = X + c;
    const uint64_t mx = col_strip_max<T>(strip, X, ld, cols, rows, red);
    const int e = mx ? floor_log2_of_bits(mx) : 0;
    uint64_t sum = 0;
    if (live && mx) {
#pragma unroll 8
        for (int64_t r = rl; r < rows; r += LANES) {
            const uint64_t q = (uint64_t)ceil(ldexp(fabs((double)x[r * ld]), 15 - e));
            sum += q * q;
        }
    }
    for (int off = COLS; off < kWave; off <<= 1) sum += __shfl_xor(sum, off, kWave);
    if (lane < COLS) red[wave * COLS + cl] = sum;
    __syncthreads();
    if (rl == 0 && live) {
        uint64_t T_ = 0;
        for (int w = 0; w < kShiftWaves; ++w) T_ += red[w * COLS + cl];
        t[c] = mx ? shift_from(T_, e, sa) : 0;                        // all-zero column: shift 0
    }
}

template <typename T>
__global__ __launch_bounds__(kShiftThreads) void k_small_shifts(SmallSide<T> a, SmallSide<T> b, ShiftArgs sa) {
    __shared__ uint64_t red[kShiftWaves * 16];
    const bool first = blockIdx.x < a.blocks;
    const SmallSide<T> s = first ? a : b;
    const int64_t blk = first ? blockIdx.x : blockIdx.x - a.blocks;
    if (s.k_contiguous) row_shift<T>(s.X + blk * s.ld, s.len, sa, s.t + blk, red);
    else col_strip_shifts<T>(blk, s.X, s.ld, s.vecs, s.len, sa, s.t, red);
}

// Accurate mode: only the bits of max |x| per vector (its pre-shift 5 - e follows from them).
template <typename T>
__global__ __launch_bounds__(kShiftThreads) void k_small_maxbits(SmallSide<T> a, SmallSide<T> b) {
    __shared__ uint64_t red[kShiftWaves * 16];
    const bool first = blockIdx.x < a.blocks;
    const SmallSide<T> s = first ? a : b;
    const int64_t blk = first ? blockIdx.x : blockIdx.x - a.blocks;
    if (s.k_contiguous) {
        const uint64_t mx = row_max<T>(s.X + blk * s.ld, s.len, red);
        if (threadIdx.x == 0) s.maxbits[blk] = mx;
    } else {
        constexpr int COLS = strip_cols<T>();
        const uint64_t mx = col_strip_max<T>(blk, s.X, s.ld, s.vecs, s.len, red);
        const int64_t c = blk * COLS + threadIdx.x;
        if (threadIdx.x < COLS && c < s.vecs) s.maxbits[c] = mx;
    }
}

// KIND 0: residues for all moduli; KIND 1 (accurate mode): the 7-bit magnitudes ceil(|x| 2^t).
// gridDim.y > 1: workgroup row y produces the moduli of group y only (groups of kModGroup), so
// that the smallest problems, whose few workgroups would each walk through all N moduli one after
// the other, fill more of the chip; the operand is then read once per group, from the caches.
template <typename T, int ROUNDS, int KIND>
__global__ __launch_bounds__(256) void k_small_residues(SmallSide<T> a, SmallSide<T> b, ModArgs ma) {
    const bool first = blockIdx.x < a.blocks;
    const SmallSide<T> s = first ? a : b;
    const int64_t blk = first ? blockIdx.x : blockIdx.x - a.blocks;
    const int g_lo = gridDim.y > 1 ? (int)blockIdx.y : 0, g_hi = gridDim.y > 1 ? (int)blockIdx.y + 1 : 1 << 30;
    if (s.k_contiguous) {
        residues_block<T, ROUNDS, KIND>(blk, s.X, s.ld, s.vecs, s.len, s.t, ma, s.out, s.vecs_pad, s.len_pad,
                                     s.vecs_pad, g_lo, g_hi);
    } else {
        const int64_t strips = s.vecs_pad / kColStrip;
        residues_cols_block<T, ROUNDS, KIND>(blk % strips, blk / strips, s.X, s.ld, s.len, s.vecs, s.t, ma, s.out,
                                          s.vecs_pad, s.len_pad, s.vecs_pad, g_lo, g_hi);
    }
}

template <typename T>
SmallSide<T> side_of(const T *X, int64_t ld, bool k_contiguous, int64_t vecs, int64_t len, int32_t *t,
                     int8_t *out, int64_t vecs_pad, int64_t len_pad) {
    return SmallSide<T>{X, ld, vecs, len, t, nullptr, out, vecs_pad, len_pad, k_contiguous ? 1 : 0, 0u};
}

// Workgroups one side contributes to the shift / maximum launch and to the residue launch.
template <typename T>
unsigned shift_blocks(const SmallSide<T> &s) {
    return (unsigned)(s.k_contiguous ? s.vecs : (s.vecs + strip_cols<T>() - 1) / strip_cols<T>());
}
template <typename T>
unsigned residue_blocks(const SmallSide<T> &s) {
    return (unsigned)(s.k_contiguous ? (s.vecs_pad * (s.len_pad / kResPerThread) + 255) / 256
                                     : (s.vecs_pad / kColStrip) * (s.len_pad / kBlockK));
}

}  // namespace

template <typename T>
hipError_t launch_small_shifts(const T *A, int64_t lda, bool a_k_contiguous, const T *B, int64_t ldb,
                               bool b_k_contiguous, int64_t m, int64_t n, int64_t k, const ShiftArgs &sa,
                               int32_t *tA, int32_t *tB, hipStream_t stream) {
    SmallSide<T> a = side_of<T>(A, lda, a_k_contiguous, m, k, tA, nullptr, 0, 0);
    SmallSide<T> b = side_of<T>(B, ldb, b_k_contiguous, n, k, tB, nullptr, 0, 0);
    a.blocks = shift_blocks(a);
    b.blocks = shift_blocks(b);
    hipLaunchKernelGGL((k_small_shifts<T>), dim3(a.blocks + b.blocks), dim3(kShiftThreads), 0, stream, a, b,
                       sa);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_small_residues(const T *A, int64_t lda, bool a_k_contiguous, const T *B, int64_t ldb,
                                 bool b_k_contiguous, int64_t m, int64_t n, int64_t k, const ModArgs &ma,
                                 const int32_t *tA, const int32_t *tB, int8_t *rA, int8_t *rB, int64_t Mp,
                                 int64_t Np, int64_t Kp, hipStream_t stream) {
    SmallSide<T> a = side_of<T>(A, lda, a_k_contiguous, m, k, const_cast<int32_t *>(tA), rA, Mp, Kp);
    SmallSide<T> b = side_of<T>(B, ldb, b_k_contiguous, n, k, const_cast<int32_t *>(tB), rB, Np, Kp);
    a.blocks = residue_blocks(a);
    b.blocks = residue_blocks(b);
    // few workgroups: one row of workgroups per group of moduli (see k_small_residues)
    const unsigned groups = (unsigned)((ma.n + kModGroup - 1) / kModGroup);
    const unsigned rows = (a.blocks + b.blocks) < kSplitModuliBelow ? groups : 1u;
    if (ma.rounds == 1)
        hipLaunchKernelGGL((k_small_residues<T, 1, 0>), dim3(a.blocks + b.blocks, rows), dim3(256), 0, stream, a, b, ma);
    else
        hipLaunchKernelGGL((k_small_residues<T, 2, 0>), dim3(a.blocks + b.blocks, rows), dim3(256), 0, stream, a, b, ma);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_small_maxbits(const T *A, int64_t lda, bool a_k_contiguous, const T *B, int64_t ldb,
                                bool b_k_contiguous, int64_t m, int64_t n, int64_t k,
                                unsigned long long *amax, unsigned long long *bmax, hipStream_t stream) {
    SmallSide<T> a = side_of<T>(A, lda, a_k_contiguous, m, k, nullptr, nullptr, 0, 0);
    SmallSide<T> b = side_of<T>(B, ldb, b_k_contiguous, n, k, nullptr, nullptr, 0, 0);
    a.maxbits = amax;
    b.maxbits = bmax;
    a.blocks = shift_blocks(a);
    b.blocks = shift_blocks(b);
    hipLaunchKernelGGL((k_small_maxbits<T>), dim3(a.blocks + b.blocks), dim3(kShiftThreads), 0, stream, a, b);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_small_magnitudes(const T *A, int64_t lda, bool a_k_contiguous, const T *B, int64_t ldb,
                                   bool b_k_contiguous, int64_t m, int64_t n, int64_t k, const int32_t *preA,
                                   const int32_t *preB, int8_t *Abar, int8_t *Bbar, int64_t Mp, int64_t Np,
                                   int64_t Kp, hipStream_t stream) {
    SmallSide<T> a = side_of<T>(A, lda, a_k_contiguous, m, k, const_cast<int32_t *>(preA), Abar, Mp, Kp);
    SmallSide<T> b = side_of<T>(B, ldb, b_k_contiguous, n, k, const_cast<int32_t *>(preB), Bbar, Np, Kp);
    a.blocks = residue_blocks(a);
    b.blocks = residue_blocks(b);
    ModArgs none{};
    hipLaunchKernelGGL((k_small_residues<T, 1, 1>), dim3(a.blocks + b.blocks), dim3(256), 0, stream, a, b, none);
    return hipGetLastError();
}

#define OZ2_INSTANTIATE_SMALL(T)                                                                        \
    template hipError_t launch_small_shifts<T>(const T *, int64_t, bool, const T *, int64_t, bool,      \
                                               int64_t, int64_t, int64_t, const ShiftArgs &, int32_t *, \
                                               int32_t *, hipStream_t);                                 \
    template hipError_t launch_small_residues<T>(const T *, int64_t, bool, const T *, int64_t, bool,    \
                                                 int64_t, int64_t, int64_t, const ModArgs &,            \
                                                 const int32_t *, const int32_t *, int8_t *, int8_t *,  \
                                                 int64_t, int64_t, int64_t, hipStream_t);              \
    template hipError_t launch_small_maxbits<T>(const T *, int64_t, bool, const T *, int64_t, bool,     \
                                                int64_t, int64_t, int64_t, unsigned long long *,        \
                                                unsigned long long *, hipStream_t);                     \
    template hipError_t launch_small_magnitudes<T>(const T *, int64_t, bool, const T *, int64_t, bool,  \
                                                   int64_t, int64_t, int64_t, const int32_t *,          \
                                                   const int32_t *, int8_t *, int8_t *, int64_t,        \
                                                   int64_t, int64_t, hipStream_t);
OZ2_INSTANTIATE_SMALL(double)
OZ2_INSTANTIATE_SMALL(float)

}  // namespace oz2
