// Column-side kernels: B is row-major k x n, its scale vector runs over COLUMNS
// (Algorithm 1 line 1: nu in F^n) and its residue slices are wanted K-contiguous
// (transposed).  These kernels read B in place, coalesced along its rows, so no transposed
// copy of B is ever written:
//   k_col_max, k_col_sumsq, k_col_finish  -- the fast-mode shift of Section 4.2 per column;
//       partial maxima / partial integer sums per (column strip, row chunk) combined with
//       64-bit integer atomics, which is exact and order-independent;
//   k_residues_cols -- Algorithm 1 lines 3 and 5 for B: a 64 x 64 tile of B is read row-wise,
//       each thread reduces 8 consecutive k of one column modulo all N moduli, and the int8
//       results go through LDS so that every modulus' 4 KiB piece of the K-blocked output
//       [Kp/64][Np][64] is written as one contiguous run.
#include <algorithm>

#include "oz2_kernels.hpp"

namespace oz2 {
namespace {

constexpr int kColStrip = 64;        // columns per workgroup (one per lane)
constexpr int kRowChunk = 512;       // rows per workgroup in the shift kernels

__global__ __launch_bounds__(256) void k_fill_u64(uint64_t *p, int64_t count, uint64_t v) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < count) p[i] = v;
}

// colmax[c] = max_h bits(|X[h][c]|)
template <typename T>
__global__ __launch_bounds__(256) void k_col_max(const T *__restrict__ X, int64_t ld, int64_t rows,
                                                 int64_t cols, unsigned long long *colmax) {
    __shared__ uint64_t part[4][kColStrip];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t c = (int64_t)blockIdx.x * kColStrip + lane;
    const int64_t r0 = (int64_t)blockIdx.y * kRowChunk;
    const int64_t r1 = r0 + kRowChunk < rows ? r0 + kRowChunk : rows;
    uint64_t mx = 0;
    if (c < cols) {
#pragma unroll 8
        for (int64_t r = r0 + wave; r < r1; r += 4) {
            uint64_t b = (uint64_t)__double_as_longlong(fabs((double)X[r * ld + c]));
            mx = b > mx ? b : mx;
        }
    }
    part[wave][lane] = mx;
    __syncthreads();
    if (wave == 0 && c < cols) {
        for (int w = 1; w < 4; ++w) mx = part[w][lane] > mx ? part[w][lane] : mx;
        if (mx) atomicMax(&colmax[c], (unsigned long long)mx);
    }
}

// colsum[c] = sum_h ceil(|X[h][c]| 2^(15-e_c))^2 with e_c from colmax[c]
template <typename T>
__global__ __launch_bounds__(256) void k_col_sumsq(const T *__restrict__ X, int64_t ld,
                                                   int64_t rows, int64_t cols,
                                                   const unsigned long long *__restrict__ colmax,
                                                   unsigned long long *colsum) {
    __shared__ uint64_t part[4][kColStrip];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t c = (int64_t)blockIdx.x * kColStrip + lane;
    const int64_t r0 = (int64_t)blockIdx.y * kRowChunk;
    const int64_t r1 = r0 + kRowChunk < rows ? r0 + kRowChunk : rows;
    uint64_t sum = 0;
    const uint64_t mx = c < cols ? (uint64_t)colmax[c] : 0;
    if (mx) {
        const int sh = 15 - floor_log2_of_bits(mx);
#pragma unroll 8
        for (int64_t r = r0 + wave; r < r1; r += 4) {
            uint64_t q = (uint64_t)ceil(ldexp(fabs((double)X[r * ld + c]), sh));
            sum += q * q;
        }
    }
    part[wave][lane] = sum;
    __syncthreads();
    if (wave == 0 && mx) {
        sum += part[1][lane] + part[2][lane] + part[3][lane];
        atomicAdd(&colsum[c], (unsigned long long)sum);
    }
}

__global__ __launch_bounds__(256) void k_col_finish(const unsigned long long *__restrict__ colmax,
                                                    const unsigned long long *__restrict__ colsum,
                                                    int64_t cols, ShiftArgs sa,
                                                    int32_t *__restrict__ t) {
    const int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (c >= cols) return;
    const uint64_t mx = colmax[c];
    if (mx == 0) { t[c] = 0; return; }                                // all-zero column
    const uint64_t T_ = colsum[c];
    int j = 0;
    while (j < sa.levels - 1 && T_ > sa.theta[j]) ++j;
    t[c] = (sa.f_max - j) - floor_log2_of_bits(mx);
}

// Same reduction as in the row kernel (see oz2_prepost.hip for why it is exact).
__device__ inline double group_reduce(double x, double M, double Minv) {
    return fma(-rint(x * Minv), M, x);
}
__device__ inline int residue_of(double y, double p, double pinv) {
    return (int)fma(-rint(y * pinv), p, y);
}

// KIND as in the row kernel: 0 = residues for all moduli, 1 = the 7-bit magnitudes (slice 0).
template <typename T, int ROUNDS, int KIND>
__device__ __forceinline__ void residues_cols_block(int64_t block_x, int64_t block_y,
                                                    const T *__restrict__ X, int64_t ld, int64_t rows,
                                                    int64_t cols, const int32_t *__restrict__ t,
                                                    const ModArgs &ma, int8_t *__restrict__ out,
                                                    int64_t cols_pad, int64_t rows_pad,
                                                    int64_t cols_stride) {
    // cols_pad columns are written (the grid covers them); cols_stride >= cols_pad is the number
    // of rows of the whole transposed slice, of which this launch may fill a block.
    // LDS: per modulus 8 pieces x 64 columns x 8 bytes, piece-major so that the writes of a
    // wavefront (one piece, 64 columns) are contiguous; 8 bytes of padding per piece row.
    // Moduli are processed kGroup at a time to keep the LDS footprint (and so the number of
    // resident workgroups) independent of N; a group is also what shares the first reduction
    // round when two are needed.
    constexpr int kGroup = kModGroup;
    __shared__ uint2 stage[kGroup][8][65];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t c = block_x * kColStrip + lane;                     // column of X = row of the output
    const int64_t kb = block_y;                                       // K block
    const int sh = c < cols ? t[c] : 0;

    double v[2][8];                                                   // pieces wave and wave + 4
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        const int64_t h0 = kb * kBlockK + (wave + 4 * half) * 8;
#pragma unroll
        for (int i = 0; i < 8; ++i)
            v[half][i] = !(c < cols && h0 + i < rows) ? 0.0
                         : KIND == 0 ? trunc(ldexp((double)X[(h0 + i) * ld + c], sh))
                                     : ceil(ldexp(fabs((double)X[(h0 + i) * ld + c]), sh));
    }

    // Write-out: per modulus the 64 columns x 64 bytes of this tile are contiguous in
    // out[s][kb][c0 .. c0+63][64]; thread -> (column, 16-byte quarter).
    const int64_t plane = cols_stride * rows_pad;
    const int col = threadIdx.x >> 2, quarter = threadIdx.x & 3;
    int8_t *dst = out + (kb * cols_stride + block_x * kColStrip) * kBlockK + threadIdx.x * 16;

    const int n_slices = KIND == 0 ? ma.n : 1;
    for (int s0 = 0; s0 < n_slices; s0 += kGroup) {
        const int ns = n_slices - s0 < kGroup ? n_slices - s0 : kGroup;
        double y[2][8];
#pragma unroll
        for (int half = 0; half < 2; ++half)
#pragma unroll
            for (int i = 0; i < 8; ++i)
                y[half][i] = (KIND == 0 && ROUNDS == 2)
                                 ? group_reduce(v[half][i], ma.group_mod[s0 / kGroup], ma.group_inv[s0 / kGroup])
                                 : v[half][i];
        for (int g = 0; g < ns; ++g) {
            const double p = (double)ma.p[s0 + g], pinv = ma.pinv[s0 + g];
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                uint32_t w[2] = {0u, 0u};
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    uint32_t b = (KIND == 0 ? (uint32_t)residue_of(y[half][i], p, pinv)
                                            : (uint32_t)(int)y[half][i]) & 0xffu;
                    w[i >> 2] |= b << (8 * (i & 3));
                }
                stage[g][wave + 4 * half][lane] = make_uint2(w[0], w[1]);
            }
        }
        __syncthreads();
        for (int g = 0; g < ns; ++g) {
            const uint2 lo = stage[g][2 * quarter][col];
            const uint2 hi = stage[g][2 * quarter + 1][col];
            *reinterpret_cast<uint4 *>(dst + (int64_t)(s0 + g) * plane) = make_uint4(lo.x, lo.y, hi.x, hi.y);
        }
        __syncthreads();
    }
}

template <typename T, int ROUNDS, int KIND>
__global__ __launch_bounds__(256) void k_residues_cols(const T *__restrict__ X, int64_t ld,
                                                       int64_t rows, int64_t cols,
                                                       const int32_t *__restrict__ t, ModArgs ma,
                                                       int8_t *__restrict__ out, int64_t cols_pad,
                                                       int64_t rows_pad, int64_t cols_stride) {
    residues_cols_block<T, ROUNDS, KIND>(blockIdx.x, blockIdx.y, X, ld, rows, cols, t, ma, out, cols_pad,
                                         rows_pad, cols_stride);
}

}  // namespace

size_t column_scratch_bytes(int64_t cols) { return (size_t)cols * 16; }

template <typename T>
hipError_t launch_shifts_cols(const T *X, int64_t ld, int64_t rows, int64_t cols,
                              const ShiftArgs &sa, void *scratch, int32_t *t, hipStream_t stream) {
    unsigned long long *colmax = static_cast<unsigned long long *>(scratch);
    unsigned long long *colsum = colmax + cols;
    // A fill kernel, not hipMemsetAsync: the call may be captured into a HIP graph.
    hipLaunchKernelGGL(k_fill_u64, dim3((unsigned)((2 * cols + 255) / 256)), dim3(256), 0, stream,
                       reinterpret_cast<uint64_t *>(colmax), 2 * cols, 0ull);
    dim3 grid((unsigned)((cols + kColStrip - 1) / kColStrip), (unsigned)((rows + kRowChunk - 1) / kRowChunk));
    hipLaunchKernelGGL((k_col_max<T>), grid, dim3(256), 0, stream, X, ld, rows, cols, colmax);
    hipLaunchKernelGGL((k_col_sumsq<T>), grid, dim3(256), 0, stream, X, ld, rows, cols, colmax, colsum);
    hipLaunchKernelGGL(k_col_finish, dim3((unsigned)((cols + 255) / 256)), dim3(256), 0, stream, colmax,
                       colsum, cols, sa, t);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_residues_cols(const T *X, int64_t ld, int64_t rows, int64_t cols, const int32_t *t,
                                const ModArgs &ma, int8_t *out, int64_t cols_pad, int64_t rows_pad,
                                hipStream_t stream, int64_t cols_stride) {
    if (cols_stride == 0) cols_stride = cols_pad;
    dim3 grid((unsigned)(cols_pad / kColStrip), (unsigned)(rows_pad / kBlockK));
    if (ma.rounds == 1)
        hipLaunchKernelGGL((k_residues_cols<T, 1, 0>), grid, dim3(256), 0, stream, X, ld, rows, cols, t,
                           ma, out, cols_pad, rows_pad, cols_stride);
    else
        hipLaunchKernelGGL((k_residues_cols<T, 2, 0>), grid, dim3(256), 0, stream, X, ld, rows, cols, t,
                           ma, out, cols_pad, rows_pad, cols_stride);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_magnitudes_cols(const T *X, int64_t ld, int64_t rows, int64_t cols,
                                  const int32_t *pre, int8_t *out, int64_t cols_pad,
                                  int64_t rows_pad, hipStream_t stream) {
    dim3 grid((unsigned)(cols_pad / kColStrip), (unsigned)(rows_pad / kBlockK));
    ModArgs none{};
    hipLaunchKernelGGL((k_residues_cols<T, 1, 1>), grid, dim3(256), 0, stream, X, ld, rows, cols, pre,
                       none, out, cols_pad, rows_pad, cols_pad);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_col_maxbits(const T *X, int64_t ld, int64_t rows, int64_t cols,
                              unsigned long long *colmax, hipStream_t stream) {
    hipLaunchKernelGGL(k_fill_u64, dim3((unsigned)((cols + 255) / 256)), dim3(256), 0, stream,
                       reinterpret_cast<uint64_t *>(colmax), cols, 0ull);
    dim3 grid((unsigned)((cols + kColStrip - 1) / kColStrip), (unsigned)((rows + kRowChunk - 1) / kRowChunk));
    hipLaunchKernelGGL((k_col_max<T>), grid, dim3(256), 0, stream, X, ld, rows, cols, colmax);
    return hipGetLastError();
}

#define OZ2_INSTANTIATE_COLS(T)                                                                   \
    template hipError_t launch_shifts_cols<T>(const T *, int64_t, int64_t, int64_t,               \
                                              const ShiftArgs &, void *, int32_t *, hipStream_t); \
    template hipError_t launch_magnitudes_cols<T>(const T *, int64_t, int64_t, int64_t,           \
                                                  const int32_t *, int8_t *, int64_t, int64_t,    \
                                                  hipStream_t);                                   \
    template hipError_t launch_col_maxbits<T>(const T *, int64_t, int64_t, int64_t,               \
                                              unsigned long long *, hipStream_t);                 \
    template hipError_t launch_residues_cols<T>(const T *, int64_t, int64_t, int64_t,             \
                                                const int32_t *, const ModArgs &, int8_t *,       \
                                                int64_t, int64_t, hipStream_t, int64_t);
OZ2_INSTANTIATE_COLS(double)
OZ2_INSTANTIATE_COLS(float)

}  // namespace oz2
