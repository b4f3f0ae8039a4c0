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

#include "oz2_convert.hpp"
#include "oz2_kernels.hpp"

namespace oz2 {
namespace {

using namespace dev;

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
