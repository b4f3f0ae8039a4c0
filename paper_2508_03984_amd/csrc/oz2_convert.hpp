// Device code of the conversion to INT8 residues (Algorithm 1 lines 2-5) shared by the row
// kernels, the column kernels and the fused kernels for small problems: the reduction of an
// integer-valued FP64 number modulo the moduli of Section 4.1, and the work of one workgroup
// of the row form (residues_block) and of the column form (residues_cols_block).
#pragma once
#include "oz2_kernels.hpp"

namespace oz2 {
namespace dev {

constexpr int kWave = 64;
constexpr int kColStrip = 64;        // columns per workgroup of the column form (one per lane)

__device__ inline uint64_t wave_max(uint64_t v) {
    for (int off = kWave / 2; off > 0; off >>= 1) {
        uint64_t o = __shfl_xor(v, off, kWave);
        v = o > v ? o : v;
    }
    return v;
}
__device__ inline uint64_t wave_sum(uint64_t v) {
    for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

// ----------------------------------------------------------------------------------------
// Residues.  x' = trunc(x 2^t) is an integer-valued FP64 number below 2^77.  Its
// symmetric residue modulo p comes from rounds of  y <- fma(-rint(y * (1/p)), p, y),
// the reduction of Section 4.2 kept in FP64 throughout (FP64 and FP32 FMA run at the
// same rate on this chip, so there is nothing to gain from dropping to FP32):
//   the first round is exact (the difference is an integer below 2^26 in magnitude) and leaves
//   |y| <= p/2 + 2^-52 |x'|;  for |x'| < 2^46 the quotient estimate is within 2^-13 of
//   x'/p, closer than any integer/p can be to a half-integer for odd p, so rint returns
//   round(x'/p) and y is already the residue in [-(p-1)/2, (p-1)/2];
//   otherwise two rounds.  The first one is shared by up to five moduli: it reduces
//   modulo their product M < 2^40 (group_reduce), which is exact for the same reason (the
//   difference is an integer, |y| <= M/2 + 2^-51 |x'| < 2^45) and y = x' (mod M) implies
//   y = x' (mod p) for every p that divides M; the second round, on |y| < 2^46, is the
//   one-round case above for each of these p.
// p = 256: 1/p is exact, y lands in [-128, 128] and the int8 cast wraps 128 to -128,
// which is the same class (Section 4.1).
// ----------------------------------------------------------------------------------------
__device__ inline double group_reduce(double x, double M, double Minv) {
    return fma(-rint(x * Minv), M, x);
}
__device__ inline int residue_of(double y, double p, double pinv) {
    return (int)fma(-rint(y * pinv), p, y);
}

constexpr int kResPerThread = 8;     // consecutive elements per thread -> 8-byte stores

// KIND 0: residues of trunc(x 2^t) for all moduli.  KIND 1 (accurate mode): the single
// 7-bit magnitude matrix ceil(|x| 2^t), written as slice 0.
template <typename T, int ROUNDS, int KIND>
__device__ __forceinline__ void residues_block(int64_t block, const T *__restrict__ X, int64_t ld,
                                               int64_t rows, int64_t len,
                                               const int32_t *__restrict__ t, const ModArgs &ma,
                                               int8_t *__restrict__ out, int64_t rows_pad,
                                               int64_t len_pad, int64_t rows_stride, int group_lo = 0,
                                               int group_hi = 1 << 30) {
    // Only the moduli of the groups [group_lo, group_hi) (groups of kModGroup) are produced: small
    // problems spread the groups over several workgroups (see oz2_small.hip).
    // rows_pad rows are written (zeros beyond `rows`); rows_stride >= rows_pad is the number of
    // rows of the whole slice, of which this launch may fill a block.
    // Thread -> (K block, row, 8-element piece of the 64-wide block), piece fastest: a
    // wavefront writes 8 rows x 64 B = 512 contiguous bytes of the blocked output and reads
    // 512 contiguous bytes of each of 8 input rows.
    constexpr int kPieces = kBlockK / kResPerThread;
    const int64_t idx = block * 256 + threadIdx.x;
    if (idx >= rows_pad * (len_pad / kResPerThread)) return;
    const int64_t kb = idx / (rows_pad * kPieces);
    const int64_t r = (idx / kPieces) % rows_pad;
    const int64_t h0 = kb * kBlockK + (idx % kPieces) * kResPerThread;

    double v[kResPerThread];
    if (r < rows) {
        const int sh = t[r];
        const T *x = X + r * ld + h0;
        T raw[kResPerThread];
        if (h0 + kResPerThread <= len && (reinterpret_cast<uintptr_t>(x) & 15) == 0) {
            // whole piece in range and 16-byte aligned: 16-byte loads (1.9 -> 1.3 ms at 16384^2)
            constexpr int kVec = 16 / sizeof(T);
            typedef T vec_t __attribute__((ext_vector_type(kVec)));
#pragma unroll
            for (int i = 0; i < kResPerThread / kVec; ++i) {
                const vec_t q = reinterpret_cast<const vec_t *>(x)[i];
#pragma unroll
                for (int c = 0; c < kVec; ++c) raw[i * kVec + c] = q[c];
            }
        } else {
#pragma unroll
            for (int i = 0; i < kResPerThread; ++i) raw[i] = (h0 + i < len) ? x[i] : T(0);
        }
#pragma unroll
        for (int i = 0; i < kResPerThread; ++i)
            v[i] = KIND == 0 ? trunc(ldexp((double)raw[i], sh)) : ceil(ldexp(fabs((double)raw[i]), sh));
    } else {
#pragma unroll
        for (int i = 0; i < kResPerThread; ++i) v[i] = 0.0;
    }

    const int64_t plane = rows_stride * len_pad;
    int8_t *o = out + (kb * rows_stride + r) * kBlockK + (h0 - kb * kBlockK);
    if (KIND == 1) {
        uint32_t w[2] = {0u, 0u};
#pragma unroll
        for (int i = 0; i < kResPerThread; ++i) w[i >> 2] |= ((uint32_t)(int)v[i] & 0xffu) << (8 * (i & 3));
        *reinterpret_cast<uint2 *>(o) = make_uint2(w[0], w[1]);
        return;
    }
    const int s_end = group_hi < (ma.n + kModGroup - 1) / kModGroup ? group_hi * kModGroup : ma.n;
    for (int s0 = group_lo * kModGroup; s0 < s_end; s0 += kModGroup) {
        double y[kResPerThread];
#pragma unroll
        for (int i = 0; i < kResPerThread; ++i)
            y[i] = ROUNDS == 2 ? group_reduce(v[i], ma.group_mod[s0 / kModGroup], ma.group_inv[s0 / kModGroup]) : v[i];
        const int s1 = s0 + kModGroup < ma.n ? s0 + kModGroup : ma.n;
        for (int s = s0; s < s1; ++s) {
            const double p = (double)ma.p[s], pinv = ma.pinv[s];
            uint32_t w[2] = {0u, 0u};
#pragma unroll
            for (int i = 0; i < kResPerThread; ++i) {
                uint32_t b = (uint32_t)residue_of(y[i], p, pinv) & 0xffu;
                w[i >> 2] |= b << (8 * (i & 3));
            }
            *reinterpret_cast<uint2 *>(o + (int64_t)s * plane) = make_uint2(w[0], w[1]);
        }
    }
}

// KIND as in the row kernel: 0 = residues for all moduli, 1 = the 7-bit magnitudes (slice 0).
template <typename T, int ROUNDS, int KIND>
__device__ __forceinline__ void residues_cols_block(int64_t block_x, int64_t block_y,
                                                    const T *__restrict__ X, int64_t ld, int64_t rows,
                                                    int64_t cols, const int32_t *__restrict__ t,
                                                    const ModArgs &ma, int8_t *__restrict__ out,
                                                    int64_t cols_pad, int64_t rows_pad,
                                                    int64_t cols_stride, int group_lo = 0,
                                                    int group_hi = 1 << 30) {
    // Only the moduli of the groups [group_lo, group_hi) are produced (as in residues_block).
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

    const int n_all = KIND == 0 ? ma.n : 1;
    const int n_slices = group_hi < (n_all + kGroup - 1) / kGroup ? group_hi * kGroup : n_all;
    for (int s0 = group_lo * kGroup; s0 < n_slices; s0 += kGroup) {
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

}  // namespace dev
}  // namespace oz2
