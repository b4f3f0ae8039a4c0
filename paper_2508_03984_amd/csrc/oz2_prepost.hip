// Bandwidth-bound kernels of the emulation for gfx950 (row side: A, and the output):
// fast-mode shifts (Algorithm 1 line 1), residue slices (lines 2-5) and the fused
// mod-reduce + CRT + unscale epilogue (lines 7-12).  64-wide wavefronts throughout.
#include <algorithm>
#include <type_traits>

#include "oz2_convert.hpp"
#include "oz2_kernels.hpp"

namespace oz2 {

int residue_rounds(const Table &t, bool accurate) {
    // One reduction round gives the canonical residue while |x'| < 2^46 (see residue_of).
    // Fast mode: |x| < 2^(e+1) and t = f - e with f <= f_max, so |x'| < 2^(f_max+1).
    // Accurate mode: mu' brings |x| below 2^6 and the second factor is at most 2^accu_f_max
    // (reached when the maximum of Cbar is 0 or 1), so |x'| < 2^(accu_f_max+6).
    const int bits = accurate ? t.accu_f_max + 6 : t.f_max + 1;
    return bits <= 46 ? 1 : 2;
}

ModArgs make_mod_args(const Table &t, bool accurate) {
    ModArgs a{};
    a.n = t.n;
    a.rounds = residue_rounds(t, accurate);
    for (int i = 0; i < t.n; ++i) {
        a.p[i] = t.p[i];
        a.pinv_prime[i] = t.pinv_prime[i];
        a.pinv[i] = t.pinv[i];
        a.s1[i] = t.s1[i];
        a.s2[i] = t.s2[i];
    }
    for (int g = 0; g * kModGroup < t.n; ++g) {
        double M = 1.0;                                  // exact: an integer below 2^40
        for (int i = g * kModGroup; i < t.n && i < (g + 1) * kModGroup; ++i) M *= (double)t.p[i];
        a.group_mod[g] = M;
        a.group_inv[g] = 1.0 / M;
    }
    a.P1 = t.P1; a.P2 = t.P2; a.Pinv = t.Pinv;
    return a;
}

ShiftArgs make_shift_args(const Table &t) {
    ShiftArgs s{};
    s.f_max = t.f_max;
    s.levels = t.levels;
    for (int j = 0; j < kMaxLevels; ++j) s.theta[j] = j < t.levels ? t.theta[j] : ~0ull;
    return s;
}

ShiftArgs make_accu_shift_args(const Table &t) {
    ShiftArgs s{};
    s.f_max = t.accu_f_max;
    s.levels = t.accu_levels;
    for (int j = 0; j < kMaxLevels; ++j) s.theta[j] = j < t.accu_levels ? t.accu_theta[j] : ~0ull;
    return s;
}

namespace {

using namespace dev;

// ----------------------------------------------------------------------------------------
// Shifts.  One workgroup per row: pass 1 finds max|x| (as an integer compare of the FP64
// bit patterns), pass 2 sums q^2 with q = ceil(|x| 2^(15-e)) <= 2^16 in 64-bit integers, which
// is exact and independent of the order of summation.  f comes from the threshold table,
// t = f - e.  k_shifts re-reads the row for pass 2 (rows of any length); k_shifts_cached
// further down keeps rows of up to 16384 elements in registers between the passes.
// ----------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_shifts(const T *__restrict__ X, int64_t ld, int64_t len,
                                                ShiftArgs sa, int32_t *__restrict__ t) {
    __shared__ uint64_t part[4];
    __shared__ uint64_t bcast;
    const T *x = X + (int64_t)blockIdx.x * ld;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

    uint64_t mx = 0;
    for (int64_t h = threadIdx.x; h < len; h += 256) {
        uint64_t b = (uint64_t)__double_as_longlong(fabs((double)x[h]));
        mx = b > mx ? b : mx;
    }
    mx = wave_max(mx);
    if (lane == 0) part[wave] = mx;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint64_t m = part[0];
        for (int w = 1; w < 4; ++w) m = part[w] > m ? part[w] : m;
        bcast = m;
    }
    __syncthreads();
    mx = bcast;
    if (mx == 0) {                                                    // all-zero row
        if (threadIdx.x == 0) t[blockIdx.x] = 0;
        return;
    }
    const int e = floor_log2_of_bits(mx);

    uint64_t sum = 0;
    for (int64_t h = threadIdx.x; h < len; h += 256) {
        double q = ceil(ldexp(fabs((double)x[h]), 15 - e));
        uint64_t qi = (uint64_t)q;
        sum += qi * qi;
    }
    sum = wave_sum(sum);
    __syncthreads();                                                  // part[] is reused
    if (lane == 0) part[wave] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint64_t T_ = part[0] + part[1] + part[2] + part[3];
        int j = 0;
        while (j < sa.levels - 1 && T_ > sa.theta[j]) ++j;
        t[blockIdx.x] = (sa.f_max - j) - e;
    }
}

template <typename T, int ROUNDS, int KIND>
__global__ __launch_bounds__(256) void k_residues(const T *__restrict__ X, int64_t ld,
                                                  int64_t rows, int64_t len,
                                                  const int32_t *__restrict__ t, ModArgs ma,
                                                  int8_t *__restrict__ out, int64_t rows_pad,
                                                  int64_t len_pad, int64_t rows_stride) {
    residues_block<T, ROUNDS, KIND>(blockIdx.x, X, ld, rows, len, t, ma, out, rows_pad, len_pad, rows_stride);
}

// ----------------------------------------------------------------------------------------
// Shifts of rows of up to 16384 elements, reading each row once: the row is held in registers
// (CH pieces of 8 elements per thread, 8 threads per 64 elements), its maximum and then its
// integer sum of squares come from two workgroup reductions.  Same result as k_shifts, half
// its memory traffic (0.34 against 0.67 ms at 16384^2 FP64).  (Computing the residues from
// the same registers as well was measured: no faster than the separate residue kernel, because
// a workgroup that owns one row writes 64-byte pieces 1 MiB apart.)
// ----------------------------------------------------------------------------------------
template <typename T, int THREADS, int CH>
__global__ __launch_bounds__(THREADS) void k_shifts_cached(const T *__restrict__ X, int64_t ld,
                                                           int64_t len, ShiftArgs sa,
                                                           int32_t *__restrict__ t_out) {
    constexpr int kPer = 8;                                           // elements per piece
    constexpr int kWaves = THREADS / kWave;
    __shared__ uint64_t part[kWaves];
    __shared__ uint64_t bcast;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const T *x = X + (int64_t)blockIdx.x * ld;
    const bool aligned = (reinterpret_cast<uintptr_t>(x) & 15) == 0;

    double v[CH][kPer];
    uint64_t mx = 0;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const int64_t h0 = ((int64_t)c * THREADS + threadIdx.x) * kPer;
        if (h0 + kPer <= len && aligned) {
            constexpr int kVec = 16 / sizeof(T);
            typedef T vec_t __attribute__((ext_vector_type(kVec)));
#pragma unroll
            for (int i = 0; i < kPer / kVec; ++i) {
                const vec_t q = reinterpret_cast<const vec_t *>(x + h0)[i];
#pragma unroll
                for (int e = 0; e < kVec; ++e) v[c][i * kVec + e] = (double)q[e];
            }
        } else {
#pragma unroll
            for (int i = 0; i < kPer; ++i) v[c][i] = (h0 + i < len) ? (double)x[h0 + i] : 0.0;
        }
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            const uint64_t bits = (uint64_t)__double_as_longlong(fabs(v[c][i]));
            mx = bits > mx ? bits : mx;
        }
    }
    mx = wave_max(mx);
    if (lane == 0) part[wave] = mx;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint64_t m = part[0];
        for (int w = 1; w < kWaves; ++w) m = part[w] > m ? part[w] : m;
        bcast = m;
    }
    __syncthreads();
    mx = bcast;
    if (mx == 0) {                                                    // all-zero row
        if (threadIdx.x == 0) t_out[blockIdx.x] = 0;
        return;
    }
    const int e = floor_log2_of_bits(mx);
    uint64_t sum = 0;
#pragma unroll
    for (int c = 0; c < CH; ++c)
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            const uint64_t qi = (uint64_t)ceil(ldexp(fabs(v[c][i]), 15 - e));
            sum += qi * qi;
        }
    sum = wave_sum(sum);
    __syncthreads();                                                  // part[] is reused
    if (lane == 0) part[wave] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint64_t T_ = 0;
        for (int w = 0; w < kWaves; ++w) T_ += part[w];
        int j = 0;
        while (j < sa.levels - 1 && T_ > sa.theta[j]) ++j;
        t_out[blockIdx.x] = (sa.f_max - j) - e;
    }
}

// ----------------------------------------------------------------------------------------
// Epilogue: for each (i, j) read the N int32 products once, U_s = mod(C'_s, p_s) by the
// mulhi reduction of Section 4.3, C1 += s_s1 U_s, C2 += s_s2 U_s (s = 1..N, one FMA each),
// Q = rint(P_inv C1), C'' = fma(-P2, Q, fma(-P1, Q, C1) + C2), c = C'' 2^-(tA_i + tB_j).
// One thread per 4 consecutive columns (16-byte loads of the int32 planes).
// ----------------------------------------------------------------------------------------

template <typename OutT>
__device__ inline OutT finish(double c, double alpha, double beta, const OutT *Cin) {
    double r;
    if (beta == 0.0) r = (alpha == 1.0) ? c : alpha * c;
    else r = fma(alpha, c, beta * (double)*Cin);
    return (OutT)r;
}

// IN_U8: the GEMM already reduced its sums (prod holds U_s as uint8, 4 bytes per thread and
// modulus); otherwise prod holds int32 sums (possibly folded partial sums) reduced here.
template <typename OutT, bool IN_U8>
__device__ __forceinline__ void epilogue_block(int64_t block, const void *__restrict__ prod_, int64_t Mp,
                                               int64_t Np, int64_t m, int64_t n,
                                               const int32_t *__restrict__ tA,
                                               const int32_t *__restrict__ tB, const ModArgs &ma,
                                               double alpha, double beta, OutT *C, int64_t ldc) {
    // 4 consecutive columns per thread: one 4-byte (uint8 input) or 16-byte (int32 input) load
    // per modulus; 8 columns per thread measured slower (2.4 against 1.9 ms at 16384^2, N = 16).
    // Np is a multiple of 256.
    constexpr int W = 4;
    const int64_t groups = (n + W - 1) / W;
    const int64_t idx = block * 256 + threadIdx.x;
    if (idx >= m * groups) return;
    const int64_t i = idx / groups, j0 = (idx % groups) * W;

    const int64_t plane = Mp * Np;
    const int64_t at = i * Np + j0;
    double C1[W], C2[W];
#pragma unroll
    for (int c = 0; c < W; ++c) C1[c] = C2[c] = 0.0;
    // Moduli s0 .. s0 + CNT - 1: all loads first (CNT of them in flight), then the FMAs in
    // ascending order of s, which is the order the accumulation of C'(2) is defined in.
    auto group = [&](int s0, auto cnt) {
        constexpr int CNT = decltype(cnt)::value;
        int us[CNT][W];
#pragma unroll
        for (int g = 0; g < CNT; ++g) {
            const int s = s0 + g;
            if (IN_U8) {
                const uint32_t x = *reinterpret_cast<const uint32_t *>(
                    static_cast<const uint8_t *>(prod_) + (int64_t)s * plane + at);
#pragma unroll
                for (int c = 0; c < 4; ++c) us[g][c] = (int)((x >> (8 * c)) & 0xffu);
            } else {
                const int4 x = *reinterpret_cast<const int4 *>(
                    static_cast<const int32_t *>(prod_) + (int64_t)s * plane + at);
                const int p = ma.p[s], pv = (int)ma.pinv_prime[s];
                us[g][0] = mod_small(x.x, p, pv); us[g][1] = mod_small(x.y, p, pv);
                us[g][2] = mod_small(x.z, p, pv); us[g][3] = mod_small(x.w, p, pv);
            }
        }
#pragma unroll
        for (int g = 0; g < CNT; ++g) {
            const double s1 = ma.s1[s0 + g], s2 = ma.s2[s0 + g];
#pragma unroll
            for (int c = 0; c < W; ++c) {
                const double u = (double)us[g][c];
                C1[c] = fma(s1, u, C1[c]);
                C2[c] = fma(s2, u, C2[c]);
            }
        }
    };
    // groups of 8, then 4, 2, 1: a count that is not a multiple of 8 costs at most three more
    // rounds of load latency (a plain remainder loop cost 0.15 ms at 16384^2 for N = 14, 15)
    int s = 0;
    for (; s + 8 <= ma.n; s += 8) group(s, std::integral_constant<int, 8>{});
    if (s + 4 <= ma.n) { group(s, std::integral_constant<int, 4>{}); s += 4; }
    if (s + 2 <= ma.n) { group(s, std::integral_constant<int, 2>{}); s += 2; }
    if (s < ma.n) group(s, std::integral_constant<int, 1>{});
    const int ta = tA[i];
    OutT *dst = C + i * ldc + j0;
    OutT res[W];
#pragma unroll
    for (int c = 0; c < W; ++c) {
        if (j0 + c < n) {
            double Q = rint(ma.Pinv * C1[c]);
            double T_ = fma(-ma.P1, Q, C1[c]);
            double Cpp = fma(-ma.P2, Q, T_ + C2[c]);
            double val = ldexp(Cpp, -(ta + tB[j0 + c]));
            res[c] = finish<OutT>(val, alpha, beta, dst + c);
        }
    }
    if (j0 + W <= n && (reinterpret_cast<uintptr_t>(dst) & 15) == 0) {      // 16-byte stores
        constexpr int kVec = 16 / sizeof(OutT);
        typedef OutT vec_t __attribute__((ext_vector_type(kVec)));
#pragma unroll
        for (int q = 0; q < W / kVec; ++q) {
            vec_t v;
#pragma unroll
            for (int c = 0; c < kVec; ++c) v[c] = res[q * kVec + c];
            reinterpret_cast<vec_t *>(dst)[q] = v;
        }
    } else {
#pragma unroll
        for (int c = 0; c < W; ++c)
            if (j0 + c < n) dst[c] = res[c];
    }
}

template <typename OutT, bool IN_U8>
__global__ __launch_bounds__(256) void k_epilogue(const void *__restrict__ prod_, int64_t Mp,
                                                  int64_t Np, int64_t m, int64_t n,
                                                  const int32_t *__restrict__ tA,
                                                  const int32_t *__restrict__ tB, ModArgs ma,
                                                  double alpha, double beta, OutT *C,
                                                  int64_t ldc) {
    epilogue_block<OutT, IN_U8>(blockIdx.x, prod_, Mp, Np, m, n, tA, tB, ma, alpha, beta, C, ldc);
}

template <typename OutT>
__global__ __launch_bounds__(256) void k_scale_c(OutT *C, int64_t ldc, int64_t m, int64_t n,
                                                 double beta) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= m * n) return;
    OutT *dst = C + (idx / n) * ldc + idx % n;
    *dst = (beta == 0.0) ? OutT(0) : (OutT)(beta * (double)*dst);
}

inline unsigned blocks_for(int64_t threads) { return (unsigned)((threads + 255) / 256); }

}  // namespace

template <typename T>
hipError_t launch_shifts(const T *X, int64_t ld, int64_t rows, int64_t len, const ShiftArgs &sa,
                         int32_t *t, hipStream_t stream) {
    // rows of up to 16384 elements are read once (pieces of 8 elements: 128 threads hold 1024
    // elements per piece, 512 threads 4096); longer rows are read twice
    auto cached = [&](auto threads, auto ch) {
        hipLaunchKernelGGL((k_shifts_cached<T, decltype(threads)::value, decltype(ch)::value>), dim3((unsigned)rows),
                           dim3(decltype(threads)::value), 0, stream, X, ld, len, sa, t);
    };
    using std::integral_constant;
    if (len <= 1024) cached(integral_constant<int, 128>{}, integral_constant<int, 1>{});
    else if (len <= 2048) cached(integral_constant<int, 128>{}, integral_constant<int, 2>{});
    else if (len <= 4096) cached(integral_constant<int, 512>{}, integral_constant<int, 1>{});
    else if (len <= 8192) cached(integral_constant<int, 512>{}, integral_constant<int, 2>{});
    else if (len <= 12288) cached(integral_constant<int, 512>{}, integral_constant<int, 3>{});
    else if (len <= 16384) cached(integral_constant<int, 512>{}, integral_constant<int, 4>{});
    else hipLaunchKernelGGL((k_shifts<T>), dim3((unsigned)rows), dim3(256), 0, stream, X, ld, len, sa, t);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_residues(const T *X, int64_t ld, int64_t rows, int64_t len, const int32_t *t,
                           const ModArgs &ma, int8_t *out, int64_t rows_pad, int64_t len_pad,
                           hipStream_t stream, int64_t rows_stride) {
    if (rows_stride == 0) rows_stride = rows_pad;
    const int64_t threads = rows_pad * (len_pad / kResPerThread);
    if (ma.rounds == 1)
        hipLaunchKernelGGL((k_residues<T, 1, 0>), dim3(blocks_for(threads)), dim3(256), 0, stream, X,
                           ld, rows, len, t, ma, out, rows_pad, len_pad, rows_stride);
    else
        hipLaunchKernelGGL((k_residues<T, 2, 0>), dim3(blocks_for(threads)), dim3(256), 0, stream, X,
                           ld, rows, len, t, ma, out, rows_pad, len_pad, rows_stride);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_magnitudes(const T *X, int64_t ld, int64_t rows, int64_t len, const int32_t *pre,
                             int8_t *out, int64_t rows_pad, int64_t len_pad, hipStream_t stream) {
    const int64_t threads = rows_pad * (len_pad / kResPerThread);
    ModArgs none{};
    hipLaunchKernelGGL((k_residues<T, 1, 1>), dim3(blocks_for(threads)), dim3(256), 0, stream, X, ld,
                       rows, len, pre, none, out, rows_pad, len_pad, rows_pad);
    return hipGetLastError();
}

template <typename OutT>
hipError_t launch_epilogue(const void *prod, bool prod_is_u8, int64_t Mp, int64_t Np, int64_t m,
                           int64_t n, const int32_t *tA, const int32_t *tB, const ModArgs &ma,
                           double alpha, double beta, OutT *C, int64_t ldc, hipStream_t stream) {
    const int64_t threads = m * ((n + 3) / 4);
    if (prod_is_u8)
        hipLaunchKernelGGL((k_epilogue<OutT, true>), dim3(blocks_for(threads)), dim3(256), 0, stream,
                           prod, Mp, Np, m, n, tA, tB, ma, alpha, beta, C, ldc);
    else
        hipLaunchKernelGGL((k_epilogue<OutT, false>), dim3(blocks_for(threads)), dim3(256), 0, stream,
                           prod, Mp, Np, m, n, tA, tB, ma, alpha, beta, C, ldc);
    return hipGetLastError();
}

template <typename OutT>
hipError_t launch_scale_c(OutT *C, int64_t ldc, int64_t m, int64_t n, double beta,
                          hipStream_t stream) {
    hipLaunchKernelGGL((k_scale_c<OutT>), dim3(blocks_for(m * n)), dim3(256), 0, stream, C, ldc, m,
                       n, beta);
    return hipGetLastError();
}

#define OZ2_INSTANTIATE(T)                                                                        \
    template hipError_t launch_shifts<T>(const T *, int64_t, int64_t, int64_t, const ShiftArgs &, \
                                         int32_t *, hipStream_t);                                 \
    template hipError_t launch_magnitudes<T>(const T *, int64_t, int64_t, int64_t,               \
                                             const int32_t *, int8_t *, int64_t, int64_t,        \
                                             hipStream_t);                                        \
    template hipError_t launch_residues<T>(const T *, int64_t, int64_t, int64_t, const int32_t *, \
                                           const ModArgs &, int8_t *, int64_t, int64_t,           \
                                           hipStream_t, int64_t);                                 \
    template hipError_t launch_epilogue<T>(const void *, bool, int64_t, int64_t, int64_t,        \
                                           int64_t, const int32_t *, const int32_t *,             \
                                           const ModArgs &, double, double, T *, int64_t,         \
                                           hipStream_t);                                          \
    template hipError_t launch_scale_c<T>(T *, int64_t, int64_t, int64_t, double, hipStream_t);
OZ2_INSTANTIATE(double)
OZ2_INSTANTIATE(float)

}  // namespace oz2
