/*
 * CPU oracle for Ozaki scheme II (DGEMM / SGEMM emulation through the Chinese
 * Remainder Theorem on an INT8 matrix engine with INT32 accumulation).
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, written from the paper so that it
 * can be checked against it by eye.  It shares no code, header, table or
 * constant generator with the HIP library and must never be reachable from
 * the product path: only tests/, __graft_entry__.smoke() and bench.py's
 * cpu_baseline leg may load it.
 *
 * Stages (numbering of Algorithm 1, Section 4):
 *   line 1      oz2o_shifts            fast-mode scale vectors (Section 4.2)
 *               oz2o_accu_prescale /   accurate-mode scale vectors (Section 4.2)
 *               oz2o_accu_shifts
 *   lines 2-5   oz2o_residues          trunc(scaled) and rmod(., p_s) as int8
 *   line 6      oz2o_int8_gemm_rows /  int8 x int8 products, wrapping int32 sums
 *               oz2o_int8_gemm_entries
 *   line 7      oz2o_mod_reduce        U_s = mod(C'_s, p_s) in [0, p_s)
 *   lines 8-11  oz2o_crt_fold          C'(1), C'(2), Q, C''      (Section 4.3)
 *   line 12     oz2o_unscale_*         C = diag(mu^-1) C'' diag(nu^-1), then
 *                                      alpha / beta as in BLAS (not in the paper)
 * plus oz2o_dd_rows, a double-double product used only to measure error.
 *
 * Readings taken where the paper is silent or garbled (each also listed in the
 * design notes of the repository):
 *   - scale vectors are carried as integer shifts t (mu = 2^t), never as floats;
 *   - the sum of squares in the scale formula is taken on the row divided by
 *     2^floor(log2 max|a|), and is made an exact upper bound by rounding every
 *     normalised magnitude up to a multiple of 2^-15 before squaring (the paper
 *     asks for a round-up-mode sum; this is an order-independent way to get
 *     one);
 *   - an all-zero row or column gets shift 0;
 *   - fma(x,y,z) means x*y+z;
 *   - rmod returns the representative in [-(p-1)/2, (p-1)/2] for odd p and in
 *     [-128, 127] for p = 256 (128 wraps to -128, Section 4.1).
 *
 * All vectors of a matrix are addressed through two strides, so that the same
 * routine serves rows of A (stride_v = lda, stride_h = 1) and columns of B
 * (stride_v = 1, stride_h = ldb).  Residue slices are stored vector-major:
 * slice s, vector v, position h at out[(s*nv + v)*len + h]; for B this is the
 * transposed orientation, a storage choice only.
 *
 * Build: gcc -O2 -fopenmp -ffp-contract=off -shared -fPIC oz2_oracle.c -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------- */
/* Algorithm 1 line 1, fast mode (Section 4.2, the formula for mu_i, nu_j).   */
/*                                                                           */
/* For vector v:  e = floor(log2 max_h |x_h|)                                 */
/*                q_h = ceil(|x_h| * 2^(15-e))      (an integer <= 2^16)       */
/*                T = sum_h q_h^2                   (exact: T <= 2^49)         */
/*                S = T * 2^-30  >= sum_h (x_h 2^-e)^2                        */
/*                f = floor(P'_fast - max(1, 0.51*log2 S))                    */
/*                t = f - e                         (mu = 2^t)                */
/* e_out and T_out may be NULL.                                               */
/* ------------------------------------------------------------------------- */
void oz2o_shifts(const double *X, int64_t nv, int64_t len, int64_t stride_v,
                 int64_t stride_h, double Pfast, int32_t *t, int32_t *e_out,
                 double *T_out)
{
#pragma omp parallel for schedule(static)
    for (int64_t v = 0; v < nv; ++v) {
        const double *x = X + v * stride_v;
        double amax = 0.0;
        for (int64_t h = 0; h < len; ++h) {
            double a = fabs(x[h * stride_h]);
            if (a > amax) amax = a;
        }
        if (amax == 0.0) {
            t[v] = 0;
            if (e_out) e_out[v] = 0;
            if (T_out) T_out[v] = 0.0;
            continue;
        }
        int ex;
        (void)frexp(amax, &ex);          /* amax = m * 2^ex, 0.5 <= m < 1 */
        int e = ex - 1;                  /* floor(log2 amax)              */
        double T = 0.0;
        for (int64_t h = 0; h < len; ++h) {
            double q = ceil(ldexp(fabs(x[h * stride_h]), 15 - e));
            T += q * q;                  /* exact: integers below 2^53    */
        }
        double S = ldexp(T, -30);
        double f = floor(Pfast - fmax(1.0, 0.51 * log2(S)));
        t[v] = (int32_t)f - e;
        if (e_out) e_out[v] = e;
        if (T_out) T_out[v] = T;
    }
}


/* ------------------------------------------------------------------------- */
/* Accurate mode (Section 4.2, second half).                                  */
/*   mu'_i = 2^(5 - floor(log2 max_h |a_ih|)),  abar_ih = ceil(mu'_i |a_ih|)   */
/* (an integer in [0, 64], so it fits INT8), likewise nu'_j and bbar for the   */
/* columns of B.  oz2o_accu_prescale writes e = floor(log2 max) per vector    */
/* (0 for an all-zero vector) and the 7-bit matrix, vector-major [nv][len].   */
/* ------------------------------------------------------------------------- */
void oz2o_accu_prescale(const double *X, int64_t nv, int64_t len, int64_t stride_v,
                        int64_t stride_h, int32_t *e_out, int8_t *bar)
{
#pragma omp parallel for schedule(static)
    for (int64_t v = 0; v < nv; ++v) {
        const double *x = X + v * stride_v;
        double amax = 0.0;
        for (int64_t h = 0; h < len; ++h) {
            double a = fabs(x[h * stride_h]);
            if (a > amax) amax = a;
        }
        int e = 0;
        if (amax != 0.0) {
            int ex;
            (void)frexp(amax, &ex);
            e = ex - 1;
        }
        e_out[v] = e;
        for (int64_t h = 0; h < len; ++h)
            bar[v * len + h] = (int8_t)ceil(ldexp(fabs(x[h * stride_h]), 5 - e));
    }
}

/* ------------------------------------------------------------------------- */
/* Accurate-mode shifts from the row (column) maxima of Cbar = Abar * Bbar:    */
/*   mu_i = mu'_i * 2^floor(P'_accu - 0.51 log2 max_h cbar_ih)                 */
/* i.e. t_i = (5 - e_i) + floor(P'_accu - 0.51 log2 cmax_i).  A vector whose   */
/* own entries are all zero gets shift 0; a maximum of 0 that comes from the  */
/* OTHER matrix being zero is taken as 1 (any shift is valid then).           */
/* ------------------------------------------------------------------------- */
void oz2o_accu_shifts(const int32_t *e, const int64_t *cmax, const uint8_t *is_zero,
                      int64_t nv, double Paccu, int32_t *t)
{
    for (int64_t v = 0; v < nv; ++v) {
        if (is_zero[v]) { t[v] = 0; continue; }
        double c = cmax[v] > 0 ? (double)cmax[v] : 1.0;
        t[v] = (5 - e[v]) + (int32_t)floor(Paccu - 0.51 * log2(c));
    }
}

/* ------------------------------------------------------------------------- */
/* Algorithm 1 lines 2-5.                                                     */
/* x' = trunc(x * 2^t) is an integer of up to ~77 bits; it is never formed:   */
/* with x = sign * M * 2^(ex-53) (M a 53-bit integer) and s = ex - 53 + t,    */
/*     s >= 0:  x' = sign * M * 2^s,   x' mod p = (M mod p)(2^s mod p) mod p   */
/*     s <  0:  x' = sign * (M >> -s)  (truncation toward zero)               */
/* rmod(x', p) = x' - p*round(x'/p)  (Section 3) is then the representative   */
/* of x' mod p nearest to zero.                                               */
/* ------------------------------------------------------------------------- */
static int8_t symmetric_residue(uint64_t mag_mod_p, int negative, int p)
{
    int u = (int)mag_mod_p;                    /* |x'| mod p in [0,p)      */
    if (negative && u != 0) u = p - u;         /* x' mod p in [0,p)        */
    int r = (2 * u < p) ? u : u - p;           /* nearest representative;  */
                                               /* p=256, u=128 -> -128     */
    return (int8_t)r;
}

#define OZ2O_POW_TABLE 128

void oz2o_residues(const double *X, int64_t nv, int64_t len, int64_t stride_v,
                   int64_t stride_h, const int32_t *t, const int32_t *p, int N,
                   int8_t *out)
{
    /* pw[i][b] = 2^b mod p_i by repeated doubling (table lookup instead of a
       loop per element; larger exponents fall back to the loop). */
    uint64_t (*pw)[OZ2O_POW_TABLE] = malloc(sizeof(uint64_t[OZ2O_POW_TABLE]) * (size_t)N);
    for (int i = 0; i < N; ++i) {
        uint64_t pi = (uint64_t)p[i];
        pw[i][0] = 1 % pi;
        for (int b = 1; b < OZ2O_POW_TABLE; ++b) pw[i][b] = (pw[i][b - 1] * 2) % pi;
    }
#pragma omp parallel for schedule(static)
    for (int64_t v = 0; v < nv; ++v) {
        for (int64_t h = 0; h < len; ++h) {
            double x = X[v * stride_v + h * stride_h];
            int ex;
            double mant = frexp(fabs(x), &ex);
            uint64_t M = (uint64_t)ldexp(mant, 53);   /* exact, < 2^53 */
            int64_t s = (int64_t)ex - 53 + t[v];
            for (int i = 0; i < N; ++i) {
                uint64_t pi = (uint64_t)p[i];
                uint64_t u;
                if (M == 0 || s <= -64) {
                    u = 0;
                } else if (s < 0) {
                    u = (M >> (-s)) % pi;
                } else {
                    uint64_t pow2;
                    if (s < OZ2O_POW_TABLE) {
                        pow2 = pw[i][s];
                    } else {
                        pow2 = pw[i][OZ2O_POW_TABLE - 1];
                        for (int64_t b = OZ2O_POW_TABLE - 1; b < s; ++b)
                            pow2 = (pow2 * 2) % pi;
                    }
                    u = ((M % pi) * pow2) % pi;
                }
                out[((int64_t)i * nv + v) * len + h] =
                    symmetric_residue(u, x < 0.0, p[i]);
            }
        }
    }
    free(pw);
}

/* ------------------------------------------------------------------------- */
/* Algorithm 1 line 6: C'_s = A'_s B'_s with INT32 accumulation that wraps    */
/* (Section 4.3: exact for k < 2^17).  Ares is [N][m][k], Bres is [N][n][k].  */
/* Only the rows listed in `rows` are produced: out is [N][nrows][n].         */
/* ------------------------------------------------------------------------- */
void oz2o_int8_gemm_rows(const int8_t *Ares, const int8_t *Bres, int N,
                         int64_t m, int64_t n, int64_t k, const int64_t *rows,
                         int64_t nrows, int32_t *out)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int s = 0; s < N; ++s) {
        for (int64_t r = 0; r < nrows; ++r) {
            const int8_t *a = Ares + ((int64_t)s * m + rows[r]) * k;
            for (int64_t j = 0; j < n; ++j) {
                const int8_t *b = Bres + ((int64_t)s * n + j) * k;
                uint32_t acc = 0;                     /* wraps modulo 2^32 */
                for (int64_t h = 0; h < k; ++h)
                    acc += (uint32_t)((int32_t)a[h] * (int32_t)b[h]);
                out[((int64_t)s * nrows + r) * n + j] = (int32_t)acc;
            }
        }
    }
}

/* ------------------------------------------------------------------------- */
/* k > 2^17 ("it is possible to apply block matrix multiplication",           */
/* Section 4.3): the contraction is cut into ranges of `kblock` <= 2^17, each  */
/* range is accumulated in wrapping INT32 like above, and the range results    */
/* are added as integers; out is [N][nrows][n] int64.  With kblock >= k this   */
/* is the plain product.                                                       */
/* ------------------------------------------------------------------------- */
void oz2o_int8_gemm_rows_blocked(const int8_t *Ares, const int8_t *Bres, int N,
                                 int64_t m, int64_t n, int64_t k, int64_t kblock,
                                 const int64_t *rows, int64_t nrows, int64_t *out)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int s = 0; s < N; ++s) {
        for (int64_t r = 0; r < nrows; ++r) {
            const int8_t *a = Ares + ((int64_t)s * m + rows[r]) * k;
            for (int64_t j = 0; j < n; ++j) {
                const int8_t *b = Bres + ((int64_t)s * n + j) * k;
                int64_t total = 0;
                for (int64_t h0 = 0; h0 < k; h0 += kblock) {
                    int64_t h1 = h0 + kblock < k ? h0 + kblock : k;
                    uint32_t acc = 0;
                    for (int64_t h = h0; h < h1; ++h)
                        acc += (uint32_t)((int32_t)a[h] * (int32_t)b[h]);
                    total += (int32_t)acc;
                }
                out[((int64_t)s * nrows + r) * n + j] = total;
            }
        }
    }
}

/* mod for the int64 sums of the blocked product. */
void oz2o_mod_reduce64(const int64_t *prod, int N, int64_t count,
                       const int32_t *p, uint8_t *U)
{
    for (int s = 0; s < N; ++s) {
#pragma omp parallel for schedule(static)
        for (int64_t c = 0; c < count; ++c) {
            int64_t r = prod[(int64_t)s * count + c] % p[s];
            if (r < 0) r += p[s];
            U[(int64_t)s * count + c] = (uint8_t)r;
        }
    }
}

/* Same product for scattered entries (ii[c], jj[c]); out is [N][count]. */
void oz2o_int8_gemm_entries(const int8_t *Ares, const int8_t *Bres, int N,
                            int64_t m, int64_t n, int64_t k, const int64_t *ii,
                            const int64_t *jj, int64_t count, int32_t *out)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int s = 0; s < N; ++s) {
        for (int64_t c = 0; c < count; ++c) {
            const int8_t *a = Ares + ((int64_t)s * m + ii[c]) * k;
            const int8_t *b = Bres + ((int64_t)s * n + jj[c]) * k;
            uint32_t acc = 0;
            for (int64_t h = 0; h < k; ++h)
                acc += (uint32_t)((int32_t)a[h] * (int32_t)b[h]);
            out[(int64_t)s * count + c] = (int32_t)acc;
        }
    }
}

/* ------------------------------------------------------------------------- */
/* Algorithm 1 line 7: U_s = mod(C'_s, p_s) = C'_s - p_s*floor(C'_s/p_s).      */
/* prod and U are [N][count].                                                 */
/* ------------------------------------------------------------------------- */
void oz2o_mod_reduce(const int32_t *prod, int N, int64_t count,
                     const int32_t *p, uint8_t *U)
{
    for (int s = 0; s < N; ++s) {
#pragma omp parallel for schedule(static)
        for (int64_t c = 0; c < count; ++c) {
            int64_t x = prod[(int64_t)s * count + c];
            int64_t r = x % p[s];
            if (r < 0) r += p[s];
            U[(int64_t)s * count + c] = (uint8_t)r;
        }
    }
}

/* ------------------------------------------------------------------------- */
/* Algorithm 1 lines 8-11 (Section 4.3):                                      */
/*   C1 = sum_s s_s1 U_s   (exact in FP64),   C2 = sum_s s_s2 U_s             */
/*   Q  = round(P_inv * C1)                                                   */
/*   C'' = fma(-P2, Q, fma(-P1, Q, C1) + C2)                                  */
/* Sums run s = 1..N with one FMA each.  For SGEMM emulation s2 and P2 are    */
/* all zero, which makes the same code compute C'' = fma(-P1, Q, C1).         */
/* ------------------------------------------------------------------------- */
void oz2o_crt_fold(const uint8_t *U, int N, int64_t count, const double *s1,
                   const double *s2, double P1, double P2, double Pinv,
                   double *Cpp)
{
#pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < count; ++c) {
        double C1 = 0.0, C2 = 0.0;
        for (int s = 0; s < N; ++s) {
            double u = (double)U[(int64_t)s * count + c];
            C1 = fma(s1[s], u, C1);
            C2 = fma(s2[s], u, C2);
        }
        double Q = rint(Pinv * C1);
        double T = fma(-P1, Q, C1);
        Cpp[c] = fma(-P2, Q, T + C2);
    }
}

/* ------------------------------------------------------------------------- */
/* Algorithm 1 line 12 and the BLAS-style update.                             */
/*   c = C'' * 2^-(tA_i + tB_j);  out = alpha*c + beta*C_in                   */
/* with the conventions: alpha==1 and beta==0 -> c;  beta==0 -> alpha*c       */
/* (C_in is not read);  otherwise fma(alpha, c, beta*C_in).                   */
/* tsum[c] holds tA_i + tB_j of entry c.                                      */
/* ------------------------------------------------------------------------- */
static double update(double c, double alpha, double beta, const double *Cin,
                     int64_t idx)
{
    if (beta == 0.0) return (alpha == 1.0) ? c : alpha * c;
    return fma(alpha, c, beta * Cin[idx]);
}

void oz2o_unscale_entries(const double *Cpp, const int32_t *tsum,
                          int64_t count, double alpha, double beta,
                          const double *Cin, double *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < count; ++c)
        out[c] = update(ldexp(Cpp[c], -tsum[c]), alpha, beta, Cin, c);
}

/* Row form: Cpp, Cin, out are [nrows][n]; tA has one shift per listed row. */
void oz2o_unscale_rows(const double *Cpp, const int32_t *tA, const int32_t *tB,
                       int64_t nrows, int64_t n, double alpha, double beta,
                       const double *Cin, double *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < nrows; ++r)
        for (int64_t j = 0; j < n; ++j) {
            int64_t c = r * n + j;
            out[c] = update(ldexp(Cpp[c], -(tA[r] + tB[j])), alpha, beta, Cin, c);
        }
}

/* SGEMM emulation rounds the FP64 result to FP32 once, at the very end. */
void oz2o_round_to_f32(const double *x, int64_t count, float *out)
{
    for (int64_t c = 0; c < count; ++c) out[c] = (float)x[c];
}

/* ------------------------------------------------------------------------- */
/* Error measurement only: rows of A*B in double-double arithmetic (TwoProd   */
/* through fma, TwoSum), and of |A|*|B| in plain FP64.  A is m x k (lda),     */
/* B is k x n (ldb), both row-major.  hi, lo, absprod are [nrows][n].         */
/* ------------------------------------------------------------------------- */
void oz2o_dd_rows(const double *A, int64_t lda, const double *B, int64_t ldb,
                  int64_t n, int64_t k, const int64_t *rows, int64_t nrows,
                  double *hi, double *lo, double *absprod)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t r = 0; r < nrows; ++r) {
        for (int64_t j = 0; j < n; ++j) {
            const double *a = A + rows[r] * lda;
            double sh = 0.0, sl = 0.0, sa = 0.0;
            for (int64_t h = 0; h < k; ++h) {
                double x = a[h], y = B[h * ldb + j];
                double ph = x * y;
                double pl = fma(x, y, -ph);          /* x*y = ph + pl exactly */
                double th = sh + ph;                 /* TwoSum(sh, ph)        */
                double z = th - sh;
                double tl = (sh - (th - z)) + (ph - z);
                tl += sl + pl;
                sh = th + tl;                        /* renormalise           */
                sl = tl - (sh - th);
                sa += fabs(x) * fabs(y);
            }
            hi[r * n + j] = sh;
            lo[r * n + j] = sl;
            absprod[r * n + j] = sa;
        }
    }
}
