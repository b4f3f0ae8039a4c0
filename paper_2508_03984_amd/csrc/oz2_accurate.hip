// Accurate mode of Section 4.2: the scale vectors come from the row and column maxima of
// Cbar = Abar * Bbar, where Abar = ceil(mu' |A|) and Bbar = ceil(|B| nu') are 7-bit
// matrices (mu'_i = 2^(5 - floor(log2 max_h |a_ih|)), likewise nu'_j) and the product runs
// on the INT8 matrix cores like every other slice.  Everything here is integer or exact
// power-of-two arithmetic, so the shifts are bit-reproducible; the floor(P'_accu - 0.51 log2 c)
// of the paper is a table lookup on the integer maximum c (built on the host from that
// formula, see oz2_constants.cpp).
#include "oz2_kernels.hpp"

namespace oz2 {
namespace {

__device__ inline uint64_t wave_max_u64(uint64_t v) {
    for (int off = 32; off > 0; off >>= 1) {
        uint64_t o = __shfl_xor(v, off, 64);
        v = o > v ? o : v;
    }
    return v;
}

// rowmax[r] = max_h bits(|X[r][h]|): one workgroup per row.
template <typename T>
__global__ __launch_bounds__(256) void k_row_maxbits(const T *__restrict__ X, int64_t ld,
                                                     int64_t len, unsigned long long *rowmax) {
    __shared__ uint64_t part[4];
    const T *x = X + (int64_t)blockIdx.x * ld;
    uint64_t mx = 0;
    for (int64_t h = threadIdx.x; h < len; h += 256) {
        uint64_t b = (uint64_t)__double_as_longlong(fabs((double)x[h]));
        mx = b > mx ? b : mx;
    }
    mx = wave_max_u64(mx);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = mx;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 4; ++w) mx = part[w] > mx ? part[w] : mx;
        rowmax[blockIdx.x] = mx;
    }
}

// pre[v] = 5 - floor(log2 max) (0 for an all-zero vector: its magnitudes are all 0 anyway), for
// the rows of A and the columns of B in one go (their arrays adjoin); also clears the maxima of
// Cbar for every K range (a kernel, not a memset: the call may be captured into a HIP graph).
__global__ __launch_bounds__(256) void k_preshift(const unsigned long long *__restrict__ maxbits,
                                                  int64_t count, int ranges, int32_t *__restrict__ pre,
                                                  int32_t *__restrict__ cmax) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= count) return;
    const uint64_t b = maxbits[i];
    pre[i] = b ? 5 - floor_log2_of_bits(b) : 0;
    for (int r = 0; r < ranges; ++r) cmax[r * count + i] = 0;
}

// t[v] = (5 - e_v) + floor(P'_accu - 0.51 log2 max(c_v, 1)) with c_v the sum over the K ranges of
// the maxima of Cbar_r (Section 4.2; for a contraction of more than 2^17 the sum bounds the
// maximum of the whole Cbar from above, Section 4.3); an all-zero vector gets 0.
// Entries [0, m) are the rows of A, [m, count) the columns of B (the arrays adjoin).
__global__ __launch_bounds__(256) void k_accu_finish(const unsigned long long *__restrict__ maxbits,
                                                     const int32_t *__restrict__ cmax, int64_t m,
                                                     int64_t count, int ranges, ShiftArgs sa,
                                                     int32_t *__restrict__ tA, int32_t *__restrict__ tB) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= count) return;
    int32_t *t = i < m ? tA + i : tB + (i - m);
    const uint64_t b = maxbits[i];
    if (b == 0) { *t = 0; return; }
    uint64_t c = 0;
    for (int r = 0; r < ranges; ++r) c += (uint64_t)cmax[r * count + i];   // each in [0, 2^29]
    if (c == 0) c = 1;
    int j = 0;
    while (j < sa.levels - 1 && c > sa.theta[j]) ++j;
    *t = (5 - floor_log2_of_bits(b)) + (sa.f_max - j);
}

struct Scratch {
    unsigned long long *amax, *bmax;     // bits of max |.| per row of A / column of B
    int32_t *preA, *preB;                // 5 - e
    int32_t *cmax;                       // maxima of Cbar_r: [range][m row maxima | n column maxima]
};

Scratch carve(void *scratch, int64_t m, int64_t n) {
    Scratch s;
    s.amax = static_cast<unsigned long long *>(scratch);
    s.bmax = s.amax + m;
    s.preA = reinterpret_cast<int32_t *>(s.bmax + n);
    s.preB = s.preA + m;
    s.cmax = s.preB + n;
    return s;
}

inline unsigned blocks_for(int64_t threads) { return (unsigned)((threads + 255) / 256); }

}  // namespace

template <typename T>
hipError_t launch_accurate_prescale(const T *A, int64_t lda, bool a_k_contiguous, const T *B,
                                    int64_t ldb, bool b_k_contiguous, int64_t m, int64_t n,
                                    int64_t k, int ranges, void *scratch, int8_t *Abar, int8_t *Bbar,
                                    int64_t Mp, int64_t Np, int64_t Kp, bool small, hipStream_t stream) {
    if (ranges < 1 || ranges > kMaxKRanges) return hipErrorInvalidValue;
    const Scratch s = carve(scratch, m, n);
    if (small) {                                          // both factors per launch
        if (hipError_t e = launch_small_maxbits<T>(A, lda, a_k_contiguous, B, ldb, b_k_contiguous, m, n, k,
                                                   s.amax, s.bmax, stream))
            return e;
        hipLaunchKernelGGL(k_preshift, dim3(blocks_for(m + n)), dim3(256), 0, stream, s.amax, m + n, ranges,
                           s.preA, s.cmax);
        return launch_small_magnitudes<T>(A, lda, a_k_contiguous, B, ldb, b_k_contiguous, m, n, k, s.preA,
                                          s.preB, Abar, Bbar, Mp, Np, Kp, stream);
    }
    // A vector of the product (a row of op(A), a column of op(B)) is either contiguous in
    // memory (one workgroup per vector) or strided by the leading dimension (column kernels).
    if (a_k_contiguous)
        hipLaunchKernelGGL((k_row_maxbits<T>), dim3((unsigned)m), dim3(256), 0, stream, A, lda, k, s.amax);
    else if (hipError_t e = launch_col_maxbits<T>(A, lda, k, m, s.amax, stream)) return e;
    if (b_k_contiguous)
        hipLaunchKernelGGL((k_row_maxbits<T>), dim3((unsigned)n), dim3(256), 0, stream, B, ldb, k, s.bmax);
    else if (hipError_t e = launch_col_maxbits<T>(B, ldb, k, n, s.bmax, stream)) return e;
    // amax | bmax, preA | preB and the row | column maxima adjoin: one launch for both factors
    hipLaunchKernelGGL(k_preshift, dim3(blocks_for(m + n)), dim3(256), 0, stream, s.amax, m + n, ranges, s.preA,
                       s.cmax);
    if (hipError_t e = a_k_contiguous ? launch_magnitudes<T>(A, lda, m, k, s.preA, Abar, Mp, Kp, stream)
                                      : launch_magnitudes_cols<T>(A, lda, k, m, s.preA, Abar, Mp, Kp, stream))
        return e;
    return b_k_contiguous ? launch_magnitudes<T>(B, ldb, n, k, s.preB, Bbar, Np, Kp, stream)
                          : launch_magnitudes_cols<T>(B, ldb, k, n, s.preB, Bbar, Np, Kp, stream);
}

void accurate_maxima(void *scratch, int64_t m, int64_t n, int range, int **row_max, int **col_max) {
    const Scratch s = carve(scratch, m, n);
    *row_max = s.cmax + (int64_t)range * (m + n);
    *col_max = *row_max + m;
}

hipError_t launch_accurate_finish(int64_t m, int64_t n, int ranges, const ShiftArgs &sa, void *scratch,
                                  int32_t *tA, int32_t *tB, hipStream_t stream) {
    if (ranges < 1 || ranges > kMaxKRanges) return hipErrorInvalidValue;
    const Scratch s = carve(scratch, m, n);
    hipLaunchKernelGGL(k_accu_finish, dim3(blocks_for(m + n)), dim3(256), 0, stream, s.amax, s.cmax, m, m + n,
                       ranges, sa, tA, tB);
    return hipGetLastError();
}

template hipError_t launch_accurate_prescale<double>(const double *, int64_t, bool, const double *, int64_t,
                                                     bool, int64_t, int64_t, int64_t, int, void *, int8_t *,
                                                     int8_t *, int64_t, int64_t, int64_t, bool, hipStream_t);
template hipError_t launch_accurate_prescale<float>(const float *, int64_t, bool, const float *, int64_t,
                                                    bool, int64_t, int64_t, int64_t, int, void *, int8_t *,
                                                    int8_t *, int64_t, int64_t, int64_t, bool, hipStream_t);

}  // namespace oz2
