// Launchers of the gfx950 kernels behind oz2_dgemm / oz2_sgemm.  Every launcher
// enqueues on `stream`, checks nothing but its own launch, and returns the HIP
// error of that launch.  Buffer shapes are stated per launcher; all pointers
// are device pointers.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "oz2_constants.hpp"
#include "oz2_plan.hpp"           // padding granularity, scratch sizes (host-only header)

namespace oz2 {

// Per-modulus constants handed to kernels by value (Section 4.1).
constexpr int kModGroup = 5;             // moduli per pre-reduction group: 256^5 = 2^40 < 2^45
struct ModArgs {
    int32_t n;
    int32_t rounds;                      // 1 or 2 reduction rounds in the residue kernel
    // rounds == 2: the product of the moduli of group g = moduli [5g, 5g+5) and double(1/product);
    // the first round reduces modulo the group's product once for all its members.
    double group_mod[(kMaxModuli + kModGroup - 1) / kModGroup], group_inv[(kMaxModuli + kModGroup - 1) / kModGroup];
    int32_t p[kMaxModuli];
    uint32_t pinv_prime[kMaxModuli];
    double pinv[kMaxModuli];
    double s1[kMaxModuli], s2[kMaxModuli];
    double P1, P2, Pinv;
};

// Shift table of Section 4.2 (see oz2_constants.hpp); the same shape serves fast mode
// (argument: sum of squares T) and accurate mode (argument: maximum c of Abar*Bbar).
struct ShiftArgs {
    int32_t f_max, levels;
    uint64_t theta[kMaxLevels];
};

// accurate: the scale vectors come from accurate mode, whose scaled integers can be larger than
// fast mode's for the same number of moduli (it decides the number of reduction rounds).
int residue_rounds(const Table &t, bool accurate);
ModArgs make_mod_args(const Table &t, bool accurate);
ShiftArgs make_shift_args(const Table &t);
ShiftArgs make_accu_shift_args(const Table &t);

#if defined(__HIPCC__)
// floor(log2 |x|) from the bit pattern of a finite FP64 |x| > 0 (subnormals included).
__device__ inline int floor_log2_of_bits(uint64_t bits) {
    int ex = (int)(bits >> 52);
    if (ex) return ex - 1023;
    return (63 - __clzll((long long)bits)) - 1074;
}

// mod(x, p) in [0, p) for any int32 x and the moduli of Section 4.1, by the mulhi reduction
// of Section 4.3: y = x - mulhi(x, pinv') p lies in (-p, 2p), then one conditional addition and
// one conditional subtraction.  Both are written as unsigned minima (a negative y is a huge
// unsigned number and y + p wraps into [0, p); for y < p, y - p wraps to a huge one): two
// instructions each instead of compare, select and add.
__device__ inline int mod_small(int x, int p, int pinv_prime) {
    unsigned y = (unsigned)x - (unsigned)__mulhi(x, pinv_prime) * (unsigned)p;
    y = min(y, y + (unsigned)p);
    y = min(y, y - (unsigned)p);
    return (int)y;
}
#endif

// Algorithm 1 line 1 (fast mode): one shift per row of X (rows x len, leading dimension ld).
template <typename T>
hipError_t launch_shifts(const T *X, int64_t ld, int64_t rows, int64_t len, const ShiftArgs &sa,
                         int32_t *t, hipStream_t stream);

// Algorithm 1 lines 2-5: rmod(trunc(X[r][h] * 2^t[r]), p_s) as int8 for s < n,
// r < rows_pad, h < len_pad, stored K-blocked: out[s][h / 64][r][h % 64]; entries with
// r >= rows or h >= len are written as 0.  rows_stride (0: rows_pad) is the number of rows of
// the whole slice when the launch fills only a block of it: X, t and out then point at the
// block's first row (out + first_row * 64), and rows / rows_pad describe the block.
template <typename T>
hipError_t launch_residues(const T *X, int64_t ld, int64_t rows, int64_t len, const int32_t *t,
                           const ModArgs &ma, int8_t *out, int64_t rows_pad, int64_t len_pad,
                           hipStream_t stream, int64_t rows_stride = 0);

// The same two stages for the COLUMNS of X (rows x cols, leading dimension ld), reading X in
// place: one shift per column, and residue slices of X transposed, K-blocked:
// out[s][h / 64][c][h % 64] for c < cols_pad, h < rows_pad (zero beyond cols / rows).
// scratch: column_scratch_bytes(cols) bytes of device memory, overwritten.
template <typename T>
hipError_t launch_shifts_cols(const T *X, int64_t ld, int64_t rows, int64_t cols,
                              const ShiftArgs &sa, void *scratch, int32_t *t, hipStream_t stream);
template <typename T>
hipError_t launch_residues_cols(const T *X, int64_t ld, int64_t rows, int64_t cols, const int32_t *t,
                                const ModArgs &ma, int8_t *out, int64_t cols_pad, int64_t rows_pad,
                                hipStream_t stream, int64_t cols_stride = 0);   // stride: as in launch_residues

// Algorithm 1 lines 1-5 (fast mode) for SMALL problems, where the number of dependent launches
// sets the time: one launch for the shifts of both factors and one for their residues, with the
// results of the launchers above.  A is the left factor (m vectors of k elements: its rows when
// a_k_contiguous, else its columns), B the right one (n vectors); slices as in launch_residues.
// small_conversion_applies (oz2_plan.hpp) says for which shapes these launchers may be used.
template <typename T>
hipError_t launch_small_shifts(const T *A, int64_t lda, bool a_k_contiguous, const T *B, int64_t ldb,
                               bool b_k_contiguous, int64_t m, int64_t n, int64_t k, const ShiftArgs &sa,
                               int32_t *tA, int32_t *tB, hipStream_t stream);
template <typename T>
hipError_t launch_small_residues(const T *A, int64_t lda, bool a_k_contiguous, const T *B, int64_t ldb,
                                 bool b_k_contiguous, int64_t m, int64_t n, int64_t k, const ModArgs &ma,
                                 const int32_t *tA, const int32_t *tB, int8_t *rA, int8_t *rB, int64_t Mp,
                                 int64_t Np, int64_t Kp, hipStream_t stream);

// The same for accurate mode: the bits of max |.| per vector of both factors in one launch, and
// the 7-bit magnitude matrices ceil(|x| 2^pre) of both (slice 0 of the residue buffers) in one.
template <typename T>
hipError_t launch_small_maxbits(const T *A, int64_t lda, bool a_k_contiguous, const T *B, int64_t ldb,
                                bool b_k_contiguous, int64_t m, int64_t n, int64_t k,
                                unsigned long long *amax, unsigned long long *bmax, hipStream_t stream);
template <typename T>
hipError_t launch_small_magnitudes(const T *A, int64_t lda, bool a_k_contiguous, const T *B, int64_t ldb,
                                   bool b_k_contiguous, int64_t m, int64_t n, int64_t k, const int32_t *preA,
                                   const int32_t *preB, int8_t *Abar, int8_t *Bbar, int64_t Mp, int64_t Np,
                                   int64_t Kp, hipStream_t stream);

// Accurate mode (Section 4.2, second half).  All vectors live in `scratch`
// (accurate_scratch_bytes(m, n) bytes); the 7-bit matrices go to slice 0 of the residue
// buffers (same K-blocked layout); Cbar itself is never stored:
//   launch_accurate_prescale   max|.| per row of A / column of B, mu' = 2^(5-e), nu', and
//                              Abar = ceil(mu' |A|), Bbar = ceil(|B| nu') as int8; clears the
//                              maxima of Cbar for `ranges` K ranges.  small: with the fused
//                              launches for small problems
//   (the caller then runs launch_int8_gemm_maxima on Cbar_r = Abar * Bbar over each K range r)
//   launch_accurate_finish     t = (5 - e) + floor(P'_accu - 0.51 log2 c), c = the sum over the
//                              ranges of the maxima of Cbar_r (one range: the maximum of Cbar, the
//                              paper's formula; more: an upper bound of it); zero vectors -> 0
template <typename T>
hipError_t launch_accurate_prescale(const T *A, int64_t lda, bool a_k_contiguous, const T *B,
                                    int64_t ldb, bool b_k_contiguous, int64_t m, int64_t n,
                                    int64_t k, int ranges, void *scratch, int8_t *Abar, int8_t *Bbar,
                                    int64_t Mp, int64_t Np, int64_t Kp, bool small, hipStream_t stream);
// Where the maxima of Cbar_r live in `scratch` (m row maxima, then n column maxima; the caller
// fills them with launch_int8_gemm_maxima); _finish turns them into the shifts.
void accurate_maxima(void *scratch, int64_t m, int64_t n, int range, int **row_max, int **col_max);
hipError_t launch_accurate_finish(int64_t m, int64_t n, int ranges, const ShiftArgs &sa, void *scratch,
                                  int32_t *tA, int32_t *tB, hipStream_t stream);

// Row / column kernels in "magnitude" form, used by accurate mode:
// out[h / 64][r][h % 64] = ceil(|X[r][h]| * 2^pre[r]) (int8), zero beyond rows / len.
template <typename T>
hipError_t launch_magnitudes(const T *X, int64_t ld, int64_t rows, int64_t len, const int32_t *pre,
                             int8_t *out, int64_t rows_pad, int64_t len_pad, hipStream_t stream);
template <typename T>
hipError_t launch_magnitudes_cols(const T *X, int64_t ld, int64_t rows, int64_t cols,
                                  const int32_t *pre, int8_t *out, int64_t cols_pad,
                                  int64_t rows_pad, hipStream_t stream);
// colmax[c] = max_h bits(|X[h][c]|) as uint64 (fills colmax with 0 first).
template <typename T>
hipError_t launch_col_maxbits(const T *X, int64_t ld, int64_t rows, int64_t cols,
                              unsigned long long *colmax, hipStream_t stream);

// Algorithm 1 lines 6-7: for b < batch, the contraction of A[b] and B[b]^T over the K range
// [k_begin, k_begin + k_len) (multiples of kPadK), int8 in, wrapping int32 accumulation.
// A: [batch][Kp/64][Mp][64], B: [batch][Kp/64][Np][64] (K-blocked, see launch_residues);
// Mp, Np multiples of kPadMN.  C is [batch][Mp][Np] and receives
//   as_u8 = false, fold = false   the int32 sums C'_b
//   as_u8 = true,  fold = false   U_b = mod(C'_b, p_b) as uint8
//   fold = true                   the same combined with what C already holds, for the
//                                 second and later K ranges of a product with k > 2^17:
//                                 int32: mod(old) + mod(new);  uint8: (old + mod(new)) mod p_b
// ma supplies the moduli (slice b uses p_b); it may be NULL for the plain int32 form.
// The part of the product that one launch computes and where it goes: rows [row0, row0+rows)
// of the A slices times rows [col0, col0+cols) of the B slices (all multiples of 256), written
// to C[slice * c_plane + (row - row0) * c_ld + (column - col0)].
struct GemmPanel {
    int64_t row0, rows, col0, cols;
    int64_t c_ld, c_plane;              // in elements; multiples of 16
};

// panel == nullptr: the whole product, C = [batch][Mp][Np].
hipError_t launch_int8_gemm(const int8_t *A, const int8_t *B, void *C, int batch, int64_t Mp,
                            int64_t Np, int64_t Kp, int64_t k_begin, int64_t k_len, bool as_u8,
                            bool fold, const ModArgs *ma, hipStream_t stream,
                            const GemmPanel *panel = nullptr);

// Accurate mode (Section 4.2): the contraction of slice 0 of A and B over the K range
// [k_begin, k_begin + k_len) (k_len <= 2^17) for one panel (as above), of which only the maxima
// are kept: row_max[i] = max(row_max[i], max_j c_ij) for the panel's rows i < valid_rows,
// col_max[j] likewise for its columns j < valid_cols (entries are sums of products of
// non-negative numbers).  Both arrays are indexed from the panel's first row / column and are
// updated with integer atomic maxima.
hipError_t launch_int8_gemm_maxima(const int8_t *A, const int8_t *B, int64_t Mp, int64_t Np, int64_t Kp,
                                   int64_t k_begin, int64_t k_len, const GemmPanel &panel,
                                   int64_t valid_rows, int64_t valid_cols, int *row_max, int *col_max,
                                   hipStream_t stream);

// Algorithm 1 lines 7-12 and the alpha/beta update, fused:
// C[i][j] = alpha * ldexp(C''(i,j), -(tA[i]+tB[j])) + beta * C[i][j]   (OutT = double or float)
// prod: [n_mod][Mp][Np], int32 sums (prod_is_u8 = false; reduced here) or uint8 residues U_s.
template <typename OutT>
hipError_t launch_epilogue(const void *prod, bool prod_is_u8, int64_t Mp, int64_t Np, int64_t m, int64_t n,
                           const int32_t *tA, const int32_t *tB, const ModArgs &ma, double alpha,
                           double beta, OutT *C, int64_t ldc, hipStream_t stream);

// C <- beta * C (the k == 0 case).
template <typename OutT>
hipError_t launch_scale_c(OutT *C, int64_t ldc, int64_t m, int64_t n, double beta,
                          hipStream_t stream);

}  // namespace oz2
