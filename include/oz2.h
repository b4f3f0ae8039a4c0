/*
 * oz2 -- DGEMM / SGEMM emulation on the INT8 matrix cores of AMD MI355X
 * (gfx950) by Ozaki scheme II: the Chinese Remainder Theorem over N pairwise
 * coprime moduli <= 256, N INT8 GEMMs with exact INT32 accumulation and an
 * FP64 reconstruction (Sections 3 and 4 and Algorithm 1 of the paper "High-
 * Performance and Power-Efficient Emulation of Matrix Multiplication using
 * INT8 Matrix Engines", Uchino, Ozaki, Imamura, SC'25).
 *
 * C ABI.  Conventions shared by every entry point:
 *   - matrices are ROW-MAJOR; oz2_dgemm / oz2_sgemm take them as they are, the
 *     oz2_*gemm_op entry points take an optional transposition of each.  A
 *     column-major caller obtains C = A*B by passing (B, A) and (n, m), since
 *     C^T = B^T A^T;
 *   - pointers named A, B, C, dev_* are DEVICE pointers owned by the caller;
 *     A and B are only read; host pointers are marked "host";
 *   - calls are asynchronous on `stream`; the returned status reports argument
 *     and launch errors only;
 *   - state (the workspace, the options, the diagnostics of the last call) lives in a
 *     CONTEXT (oz2_create / oz2_destroy; the oz2_ctx_* entry points).  The product calls
 *     of one context share its workspace: the caller orders them (one stream, or events
 *     between streams).  Calls on different contexts are independent and may run
 *     concurrently, from several host threads and on several streams.  Every entry
 *     point without a context argument (oz2_dgemm, oz2_set_workspace, ...) is the
 *     oz2_ctx_* one applied to the process's DEFAULT context, which a NULL context
 *     argument also denotes;
 *   - a product call whose workspace already exists (a caller-owned one, or the
 *     library's own after a call of at least the same size on the same device)
 *     allocates nothing and clears its scratch with kernels, not memsets, so it may be
 *     recorded into a HIP graph while profiling is off.  A call that has to grow the
 *     library's own workspace (or move it to another device) waits for the device,
 *     frees the old buffer and allocates the new one with hipMalloc before it
 *     launches anything;
 *   - inputs must be finite.  Inf/NaN inputs give an unspecified (but memory
 *     safe) result: the paper does not define them;
 *   - no entry point throws; besides the workspace growth above only oz2_destroy,
 *     oz2_release, oz2_set_workspace and oz2_last_stage_times_ms (and their oz2_ctx_
 *     forms) synchronise the device.
 */
#ifndef OZ2_H
#define OZ2_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ihipStream_t *hipStream_t;   /* same declaration as the HIP runtime's */

typedef enum {
    OZ2_OK = 0,
    OZ2_INVALID_ARG = 1,   /* null pointer, negative size, leading dimension too small  */
    OZ2_UNSUPPORTED = 2,   /* num_moduli outside 2..20, k > 2^20 (accurate mode: 2^17)  */
    OZ2_WORKSPACE = 3,     /* caller-provided workspace too small / allocation failed    */
    OZ2_HIP_ERROR = 4      /* a HIP runtime call or a kernel launch failed               */
} oz2_status;

#define OZ2_MIN_MODULI 2
#define OZ2_MAX_MODULI 20           /* Section 4.1: the table is kept to N <= 20        */
#define OZ2_MAX_K (1 << 17)         /* Section 4.3: INT32 accumulation is exact up to it */
#define OZ2_MAX_K_BLOCKED (1 << 20) /* longer contractions are cut into ranges of OZ2_MAX_K */

/*
 * C <- alpha * (A*B) + beta * C,  A: m x k (lda >= k), B: k x n (ldb >= n),
 * C: m x n (ldc >= n), with A*B evaluated by Algorithm 1 in fast mode
 * (Section 4.2) with `num_moduli` moduli: power-of-two row scaling of A and
 * column scaling of B, truncation, residues modulo the first num_moduli members
 * of the modulus set of Section 4.1 as INT8, num_moduli INT8 GEMMs accumulated
 * in INT32, reduction modulo p_s, CRT accumulation and fold in FP64
 * (Section 4.3) and inverse scaling.  More moduli give more accuracy: 14-17
 * reach native FP64 level for well-scaled data, 7-9 reach FP32 level (Section 5.1).
 *
 * alpha, beta are host values.  beta == 0: C is not read (NaNs in it do not
 * propagate).  m == 0 or n == 0: nothing is done.  k == 0: C <- beta * C.
 * OZ2_MAX_K < k <= OZ2_MAX_K_BLOCKED: the contraction is cut into ranges of at most
 * OZ2_MAX_K ("block matrix multiplication", Section 4.3) whose residues are added
 * modulo p_s; k > OZ2_MAX_K_BLOCKED returns OZ2_UNSUPPORTED (the exact integer sum of
 * squares behind the scale vectors needs k * 2^32 < 2^53).
 * oz2_sgemm takes FP32 data; its reconstruction still runs in FP64 and the
 * result is rounded to FP32 once.
 */
oz2_status oz2_dgemm(int64_t m, int64_t n, int64_t k, double alpha,
                     const double *A, int64_t lda, const double *B, int64_t ldb,
                     double beta, double *C, int64_t ldc, int num_moduli,
                     hipStream_t stream);

oz2_status oz2_sgemm(int64_t m, int64_t n, int64_t k, float alpha,
                     const float *A, int64_t lda, const float *B, int64_t ldb,
                     float beta, float *C, int64_t ldc, int num_moduli,
                     hipStream_t stream);

/*
 * oz2_dgemm for callers that cannot allocate device memory at the time of the call: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * result (bit for bit) and errors as oz2_dgemm, but the workspace is a fixed array of
 * OZ2_NOALLOC_WORKSPACE_BYTES in the library's device image (each GPU the library runs on holds
 * its copy until the process ends; the first call on a GPU looks its address up there), so the
 * call neither allocates nor frees anything, on the device or through any library.  A product whose workspace (oz2_workspace_bytes) exceeds that
 * size returns OZ2_WORKSPACE and does nothing: with 16 moduli the limit is reached at about
 * m = n = k = 1100.  All calls on one GPU share that GPU's array: the caller orders them (one
 * stream, or events); calls that overlap on one GPU race.  Nothing is assumed about what an
 * earlier call left in the array.  Contexts, options and the diagnostics (oz2_stage_ptr, stage
 * times) do not apply to this entry point.
 */
#define OZ2_NOALLOC_WORKSPACE_BYTES (64 * 1024 * 1024)
oz2_status oz2_dgemm_noalloc(int64_t m, int64_t n, int64_t k, double alpha,
                             const double *A, int64_t lda, const double *B, int64_t ldb,
                             double beta, double *C, int64_t ldc, int num_moduli,
                             hipStream_t stream);

/*
 * The same product with the scale vectors of ACCURATE mode (Section 4.2, second half):
 * A and B are first reduced to 7-bit matrices Abar = ceil(mu' |A|), Bbar = ceil(|B| nu')
 * (mu', nu' powers of two that bring each row / column maximum into [32, 64)), their
 * product Cbar is formed on the INT8 matrix cores, and its row and column maxima bound
 * sum_h |a_ih||b_hj| directly instead of through the Cauchy-Schwarz inequality.  This costs
 * one more INT8 GEMM and gives larger scale factors, i.e. a smaller truncation error for
 * the same number of moduli (it matters for inputs with a wide exponent range).
 * Arguments, conventions and errors are those of oz2_dgemm / oz2_sgemm.  For
 * OZ2_MAX_K < k <= OZ2_MAX_K_BLOCKED Cbar is cut into the same K ranges as the products
 * (Section 4.3, last sentence), each an exact INT32 product of which the row and column
 * maxima are kept; the maxima of the whole Cbar are then replaced by the sums of the ranges'
 * maxima, an upper bound of them, which is all the inequalities of Section 4.2 need (the
 * scale factors can come out one binary step smaller than with the exact maxima).
 */
oz2_status oz2_dgemm_accurate(int64_t m, int64_t n, int64_t k, double alpha,
                              const double *A, int64_t lda, const double *B, int64_t ldb,
                              double beta, double *C, int64_t ldc, int num_moduli,
                              hipStream_t stream);

oz2_status oz2_sgemm_accurate(int64_t m, int64_t n, int64_t k, float alpha,
                              const float *A, int64_t lda, const float *B, int64_t ldb,
                              float beta, float *C, int64_t ldc, int num_moduli,
                              hipStream_t stream);

/*
 * General form: C <- alpha * op(A) * op(B) + beta * C with op(X) = X (OZ2_OP_N) or X^T
 * (OZ2_OP_T), in fast (accurate = 0) or accurate (accurate != 0) mode of Section 4.2.
 * op(A) is m x k and op(B) is k x n; the stored A is m x k (lda >= k) or, transposed,
 * k x m (lda >= m); the stored B is k x n (ldb >= n) or n x k (ldb >= k).  Nothing is
 * transposed in memory: the scale vectors and residues of Algorithm 1 lines 1-5 are taken
 * along rows or along columns of the stored matrix as needed.  Everything else is as for
 * oz2_dgemm / oz2_sgemm, which are the (OZ2_OP_N, OZ2_OP_N, accurate = 0) case.
 */
typedef enum { OZ2_OP_N = 0, OZ2_OP_T = 1 } oz2_op;

oz2_status oz2_dgemm_op(oz2_op opA, oz2_op opB, int accurate, int64_t m, int64_t n, int64_t k,
                        double alpha, const double *A, int64_t lda, const double *B, int64_t ldb,
                        double beta, double *C, int64_t ldc, int num_moduli, hipStream_t stream);

oz2_status oz2_sgemm_op(oz2_op opA, oz2_op opB, int accurate, int64_t m, int64_t n, int64_t k,
                        float alpha, const float *A, int64_t lda, const float *B, int64_t ldb,
                        float beta, float *C, int64_t ldc, int num_moduli, hipStream_t stream);

/*
 * The same product for COLUMN-MAJOR callers (the BLAS convention): C <- alpha * op(A) * op(B)
 * + beta * C with every matrix stored column-major, op(A) m x k and op(B) k x n; the stored A is
 * m x k (lda >= m) or, transposed, k x m (lda >= k); the stored B is k x n (ldb >= k) or n x k
 * (ldb >= n); C is m x n (ldc >= m).  A column-major matrix is the row-major storage of its
 * transpose and C^T = op(B)^T op(A)^T, so this is oz2_*gemm_op with the operands exchanged:
 * (opA, opB, m, n, A, lda, B, ldb) -> (opB, opA, n, m, B, ldb, A, lda); nothing is copied, and the
 * result is the one that call gives, bit for bit.
 */
oz2_status oz2_dgemm_colmajor(oz2_op opA, oz2_op opB, int accurate, int64_t m, int64_t n, int64_t k,
                              double alpha, const double *A, int64_t lda, const double *B,
                              int64_t ldb, double beta, double *C, int64_t ldc, int num_moduli,
                              hipStream_t stream);

oz2_status oz2_sgemm_colmajor(oz2_op opA, oz2_op opB, int accurate, int64_t m, int64_t n, int64_t k,
                              float alpha, const float *A, int64_t lda, const float *B, int64_t ldb,
                              float beta, float *C, int64_t ldc, int num_moduli, hipStream_t stream);

/*
 * Contexts, for callers that run several products at once (host threads, streams) or want
 * options and workspaces of their own (the callers that cannot share the process-wide state).
 * oz2_create makes an empty context (no device memory yet; *out is written on success only);
 * oz2_destroy waits for the device, frees what the context owns (its workspace, events, second
 * stream) and the context itself; the caller makes sure none of its calls is still being issued.
 * A context may be used on any device: its own workspace lives on the device that is current
 * when a product call needs it (see oz2_set_workspace).  NULL stands for the default context.
 *
 * oz2_ctx_dgemm / oz2_ctx_sgemm are oz2_dgemm_op / oz2_sgemm_op on a context, i.e. the general
 * form C <- alpha * op(A) * op(B) + beta * C of Algorithm 1 in fast (accurate = 0) or accurate
 * mode (Section 4.2); arguments, conventions and errors as described there.  The other oz2_ctx_*
 * functions are the context forms of the functions of the same name without "ctx_", described
 * further down.  Options (oz2_ctx_set_option; value 0 = off, otherwise on):
 *   OZ2_OPT_INT32_PRODUCTS    see oz2_set_int32_products     (default off)
 *   OZ2_OPT_OVERLAP           see oz2_set_overlap            (default off)
 *   OZ2_OPT_SMALL_CONVERSION  see oz2_set_small_conversion   (default on)
 *   OZ2_OPT_PROFILING         see oz2_set_profiling          (default off)
 *   OZ2_OPT_CUT_LAUNCHES      the INT8 GEMMs of a large product run as several launches (see
 *                             oz2_last_gemm_launches); off = one launch per panel and K range of
 *                             2^17, for comparison.  Bit-identical.  (default on)
 */
typedef struct oz2_context oz2_context;
typedef enum { OZ2_OPT_INT32_PRODUCTS = 0, OZ2_OPT_OVERLAP = 1, OZ2_OPT_SMALL_CONVERSION = 2,
               OZ2_OPT_PROFILING = 3, OZ2_OPT_CUT_LAUNCHES = 4 } oz2_option;

oz2_status oz2_create(oz2_context **out);
oz2_status oz2_destroy(oz2_context *ctx);
oz2_status oz2_ctx_set_option(oz2_context *ctx, oz2_option option, int value);
oz2_status oz2_ctx_dgemm(oz2_context *ctx, oz2_op opA, oz2_op opB, int accurate, int64_t m, int64_t n,
                         int64_t k, double alpha, const double *A, int64_t lda, const double *B,
                         int64_t ldb, double beta, double *C, int64_t ldc, int num_moduli,
                         hipStream_t stream);
oz2_status oz2_ctx_sgemm(oz2_context *ctx, oz2_op opA, oz2_op opB, int accurate, int64_t m, int64_t n,
                         int64_t k, float alpha, const float *A, int64_t lda, const float *B,
                         int64_t ldb, float beta, float *C, int64_t ldc, int num_moduli,
                         hipStream_t stream);

/*
 * Prepared operands: Algorithm 1 lines 1-5 (fast mode) for ONE matrix, kept for reuse.
 * In fast mode the scale vector and the residues of A do not depend on B and vice versa,
 * so a matrix that enters many products (the panel of a blocked factorisation, a fixed
 * weight matrix) needs them only once.  oz2_prepare_* computes, on `stream`, the shifts
 * and the num_moduli INT8 residue slices of
 *     side = 0: the LEFT factor  op(X), rows x k   (its rows are scaled);
 *     side = 1: the RIGHT factor op(X), k x rows   (its columns are scaled; "rows" is then n);
 * X is stored as for oz2_dgemm_op.  The handle owns its device memory (allocated with
 * hipMalloc in the call: about num_moduli * rows * k bytes, rounded up to whole tiles);
 * oz2_operand_free releases it (the caller makes sure no product that uses it is still
 * running).  *out is written only on success.  X may be changed or freed once the work
 * queued on `stream` by the call has run.
 * oz2_*gemm_prepared: C <- alpha * L * R + beta * C for a left and a right operand prepared
 * with the same k, num_moduli and element type (OZ2_INVALID_ARG otherwise); C is
 * L.rows x R.rows with ldc >= R.rows.  The result is bit-identical to the oz2_*gemm_op call
 * on the original matrices in fast mode.  The stream of the product must be ordered after
 * the streams of the two preparations by the caller.
 */
typedef struct oz2_operand oz2_operand;

oz2_status oz2_prepare_d(int side, oz2_op op, int64_t rows, int64_t k, const double *X, int64_t ld,
                         int num_moduli, hipStream_t stream, oz2_operand **out);
oz2_status oz2_prepare_s(int side, oz2_op op, int64_t rows, int64_t k, const float *X, int64_t ld,
                         int num_moduli, hipStream_t stream, oz2_operand **out);
void oz2_operand_free(oz2_operand *operand);
size_t oz2_operand_bytes(const oz2_operand *operand);      /* device bytes it holds; 0 for NULL */

oz2_status oz2_dgemm_prepared(const oz2_operand *left, const oz2_operand *right, double alpha,
                              double beta, double *C, int64_t ldc, hipStream_t stream);
oz2_status oz2_sgemm_prepared(const oz2_operand *left, const oz2_operand *right, float alpha,
                              float beta, float *C, int64_t ldc, hipStream_t stream);
oz2_status oz2_ctx_dgemm_prepared(oz2_context *ctx, const oz2_operand *left, const oz2_operand *right,
                                  double alpha, double beta, double *C, int64_t ldc, hipStream_t stream);
oz2_status oz2_ctx_sgemm_prepared(oz2_context *ctx, const oz2_operand *left, const oz2_operand *right,
                                  float alpha, float beta, float *C, int64_t ldc, hipStream_t stream);

/*
 * Workspace.  A call needs device scratch for the shift vectors (and the
 * per-column partial results behind them), the INT8 residue slices of A and B (Algorithm 1 lines 4-5)
 * and the reduced products U_s (line 7; or the INT32 products of line 6 after
 * oz2_set_int32_products(1)): oz2_workspace_bytes gives the size for a
 * problem (0 if the arguments are unsupported).  oz2_set_workspace hands the
 * library a caller-owned device buffer (kept, not freed, must stay valid until
 * replaced; 256-byte aligned); with (NULL, 0) the library goes back to
 * allocating its own buffer with hipMalloc (on the device that is current at the
 * call; a call made with another device current allocates anew there), growing it on
 * demand and keeping it until oz2_release.  The library's own buffer is sized for
 * oz2_workspace_bytes, except for calls that take the overlapped form described under
 * oz2_set_overlap (an option): those work through C in panels of at most 4096 x 4096
 * anyway, so their buffer holds the products of one such panel beside the residues (at
 * m = n = k = 16384 and 16 moduli 8.9 GB instead of 12.9 GB).
 *
 * Bounded workspace ("block matrix multiplication" over the rows and columns of C): the
 * products U_s are the largest part (num_moduli * m * n bytes).  When the workspace may
 * not hold them all -- a caller-owned buffer smaller than oz2_workspace_bytes, or a limit
 * set with oz2_set_workspace_limit for the library's own buffer (0 = no limit) -- the call
 * computes C panel by panel: the shifts and residues of the whole of A and B once, then
 * for each (row panel, column panel) the INT8 GEMMs and the accumulation of that panel
 * only.  The result is bit-identical.  oz2_workspace_min_bytes is the smallest workspace
 * such a call can run in (one 256 x 256 panel); below it the call returns OZ2_WORKSPACE.
 * Accurate mode never stores its Cbar (only the row and column maxima are kept), so it needs
 * no workspace of its own.  oz2_plan_panels says, without touching the GPU, how a product of this
 * shape is cut in a workspace of `workspace_bytes` (host pointers, may be NULL: rows and
 * columns of a panel, multiples of 256, the last panels of a row or column may be smaller;
 * and the number of panels); oz2_last_panels reports the same for the most recent product
 * (OZ2_INVALID_ARG if there was none).  A product whose planes all fit the workspace (one
 * panel) may still run its INT8 GEMMs as several launches, each writing its part of the whole
 * product in place (a launch over all of a large C loses cache locality as its workgroups drift
 * apart); oz2_last_gemm_launches reports the number of INT8 GEMM launches that produced the
 * products of the most recent call (host pointer; accurate mode's launches for Cbar are not
 * counted).
 */
size_t oz2_workspace_bytes(int64_t m, int64_t n, int64_t k, int num_moduli, int is_double);
size_t oz2_workspace_min_bytes(int64_t m, int64_t n, int64_t k, int num_moduli, int is_double);
oz2_status oz2_set_workspace(void *dev_ptr, size_t bytes);
void oz2_set_workspace_limit(size_t bytes);
oz2_status oz2_plan_panels(int64_t m, int64_t n, int64_t k, int num_moduli, size_t workspace_bytes,
                           int64_t *panel_rows, int64_t *panel_cols, int64_t *count);
oz2_status oz2_last_panels(int64_t *panel_rows, int64_t *panel_cols, int64_t *count);
oz2_status oz2_last_gemm_launches(int64_t *launches);
void oz2_release(void);
size_t oz2_ctx_workspace_bytes(oz2_context *ctx, int64_t m, int64_t n, int64_t k, int num_moduli);
size_t oz2_ctx_workspace_min_bytes(oz2_context *ctx, int64_t m, int64_t n, int64_t k, int num_moduli);
oz2_status oz2_ctx_set_workspace(oz2_context *ctx, void *dev_ptr, size_t bytes);
oz2_status oz2_ctx_set_workspace_limit(oz2_context *ctx, size_t bytes);
oz2_status oz2_ctx_plan_panels(oz2_context *ctx, int64_t m, int64_t n, int64_t k, int num_moduli,
                               size_t workspace_bytes, int64_t *panel_rows, int64_t *panel_cols,
                               int64_t *count);
oz2_status oz2_ctx_last_panels(oz2_context *ctx, int64_t *panel_rows, int64_t *panel_cols, int64_t *count);
oz2_status oz2_ctx_last_gemm_launches(oz2_context *ctx, int64_t *launches);
oz2_status oz2_ctx_release(oz2_context *ctx);    /* frees what the context owns on the device, keeps the context */

/*
 * Constants of Section 4.1 for `num_moduli` moduli, written to HOST arrays of
 * at least num_moduli entries (any of them may be NULL):
 *   p           moduli p_i
 *   pinv_prime  floor(2^32/p_i - 1), the multiplier of the mulhi reduction (Section 4.3)
 *   s1, s2      the two-term split of (P/p_i) q_i  (is_double) or double(.) and 0 (single)
 *   P1P2Pinv    { P1, P2, P_inv }
 *   Pfast       P'_fast as a binary32 value
 */
oz2_status oz2_constants(int num_moduli, int is_double, int32_t *p, uint32_t *pinv_prime,
                         double *s1, double *s2, double *P1P2Pinv, float *Pfast);

/*
 * The fast-mode shift of Section 4.2 as the kernels evaluate it.  For a row
 * (column) with e = floor(log2 max|x|) and the exact integer
 * T = sum_h ceil(|x_h| 2^(15-e))^2, the scaled row has exponent
 * f = floor(P'_fast - max(1, 0.51 log2(T 2^-30))) and shift t = f - e.  The
 * kernels find f by comparing T with a table: f = f_max - min{ j : T <= theta[j] }.
 * This call writes f_max, the number of levels (<= 20) and theta[] to HOST memory.
 */
oz2_status oz2_shift_table(int num_moduli, int32_t *f_max, int32_t *levels, uint64_t *theta);

/*
 * The accurate-mode counterpart: P'_accu (binary32) and the table for
 * f = floor(P'_accu - 0.51 log2 c) over the integer c = maximum of a row or column of Cbar
 * (1 <= c <= 2^32: up to eight K ranges of at most 2^29 each): f = f_max - min{ j : c <= theta[j] };
 * the shift is t = (5 - e) + f.
 * Writes to HOST memory; theta needs room for 20 entries.
 */
oz2_status oz2_shift_table_accurate(int num_moduli, float *Paccu, int32_t *f_max, int32_t *levels,
                                    uint64_t *theta);

/*
 * How many rounds of the floating-point reduction y <- fma(-round(y / p), p, y) of Section 4.2
 * the residue kernels run for this number of moduli (1 or 2; 0 if num_moduli is out of range).
 * One round gives the symmetric residue only while the scaled integers stay below 2^46; fast
 * mode keeps them below 2^(f_max + 1) and accurate mode below 2^(f_max + 6) with f_max from
 * oz2_shift_table / oz2_shift_table_accurate, so accurate mode needs the second round earlier
 * (from 11 moduli on instead of 13, the threshold N_1 = 13 of Section 4.2 being fast mode's).
 */
int oz2_residue_rounds(int num_moduli, int accurate);

/*
 * Diagnostics: where the stages of the most recent oz2_dgemm / oz2_sgemm call
 * live in the workspace.  dims (host, 4 entries) describes the layout:
 *   OZ2_STAGE_SHIFT_A  int32 [m]                 dims = { m, 0, 0, 0 }
 *   OZ2_STAGE_SHIFT_B  int32 [n]                 dims = { n, 0, 0, 0 }
 *   OZ2_STAGE_RES_A    int8  [N][Kp/64][Mp][64]  dims = { N, Mp, Kp, m }   rows >= m, k-index >= k are 0
 *   OZ2_STAGE_RES_B    int8  [N][Kp/64][Np][64]  dims = { N, Np, Kp, n }   (B slices are stored transposed)
 *   OZ2_STAGE_U        uint8 [N][Mp][Np]         dims = { N, Mp, Np, 0 }   U_s = mod(C'_s, p_s) (Alg. 1 line 7)
 *   OZ2_STAGE_PROD     int32 [N][Mp][Np]         dims = { N, Mp, Np, 0 }   C'_s (Alg. 1 line 6)
 * By default the INT8 GEMM reduces its sums itself and only OZ2_STAGE_U exists; after
 * oz2_set_int32_products(1) calls keep the int32 sums instead (4x the workspace and the
 * traffic; for k > OZ2_MAX_K the planes hold sums of reduced partial results, congruent to
 * C'_s modulo p_s) and only OZ2_STAGE_PROD exists.  Asking for the other one returns
 * OZ2_INVALID_ARG.
 * The residue slices are K-blocked: residue (row r, k-index h) of slice s is at
 * ((s * Kp/64 + h/64) * rows + r) * 64 + h%64, so that a (rows x 64) tile is contiguous.
 * Valid until the next call or workspace change; the caller synchronises.  After a call
 * that was cut into panels the product planes hold the last panel only and the two product
 * stages return OZ2_INVALID_ARG; after a product of prepared operands no stage is available.
 */
enum { OZ2_STAGE_SHIFT_A = 0, OZ2_STAGE_SHIFT_B = 1, OZ2_STAGE_RES_A = 2,
       OZ2_STAGE_RES_B = 3, OZ2_STAGE_PROD = 4, OZ2_STAGE_U = 5 };
oz2_status oz2_stage_ptr(int stage, void **dev_ptr, int64_t *dims);
oz2_status oz2_ctx_stage_ptr(oz2_context *ctx, int stage, void **dev_ptr, int64_t *dims);
void oz2_set_int32_products(int on);

/*
 * Diagnostics: the batched INT8 GEMM of Algorithm 1 line 6 on its own.
 * dev_A: int8 [batch][Kp/64][Mp][64], dev_B: int8 [batch][Kp/64][Np][64] (the K-blocked
 * layout of the residue slices, see oz2_stage_ptr), dev_C: int32 [batch][Mp][Np];
 * C_b = A_b * B_b^T with wrapping INT32 sums.
 * Mp and Np must be multiples of 256, Kp a multiple of 128 (OZ2_INVALID_ARG otherwise) and
 * at most OZ2_MAX_K (OZ2_UNSUPPORTED otherwise).
 */
oz2_status oz2_int8_gemm(const int8_t *dev_A, const int8_t *dev_B, int32_t *dev_C,
                         int batch, int64_t Mp, int64_t Np, int64_t Kp, hipStream_t stream);

/*
 * Diagnostics: the rate of the INT8 matrix cores on their own (the instruction of the
 * GEMM of Algorithm 1 line 6, v_mfma_i32_32x32x32_i8, issued back to back from registers by
 * two wavefronts per SIMD, no memory traffic), sustained over about `seconds` (0 < seconds
 * <= 5) on the current device's default stream; blocks until done.
 * random_operands = 0: constant operands; 1: pseudo-random bytes, which is what residues
 * look like -- the sustained clock depends on it.
 * Outputs (HOST pointers): *tops in 1e12 INT8 operations per second (a multiply-add
 * counts as two), and, if not NULL, the device's compute-unit count and its nominal
 * maximum clock in MHz.  Allocates and frees a small device buffer of its own.
 */
oz2_status oz2_mfma_probe(int random_operands, double seconds, double *tops, int *compute_units,
                          int *clock_mhz);

/*
 * Overlap (an option, off by default).  With it, a product with a long contraction and a large C
 * (k >= 8192, at least four panels of at most 4096 x 4096, k times the number of panels at
 * least 9 x 8192) is computed panel by panel: the INT8 GEMMs and the accumulation
 * of the panels run one after the other on `stream`, while a second stream owned by the
 * context (default priority, created at the first such call, destroyed by oz2_release)
 * computes the residues of the blocks of A and B that the coming panels need.  The second
 * stream forks from `stream` after the shifts and has joined it again when the last panel
 * starts, so for the caller the call is ordered on `stream` as always (it can also be captured
 * into a graph once the second stream exists).  The result is bit-identical.  The product
 * stages of oz2_stage_ptr are not available after such a call (shifts and residues are).
 * Whether it pays depends on the device: the matrix cores run against the board's power limit,
 * and work beside the GEMMs takes clock from them (measured between -2 % and +1 % of the call).
 */
void oz2_set_overlap(int on);

/*
 * Small problems (on by default).  Below about 2048^3 a call is bound by the latency of its
 * dependent kernel launches.  For calls with k <= 4096, m, n <= 8192 and
 * (m + n) * k <= 2 * 2048^2 the conversion of Algorithm 1 lines 1-5 therefore runs as two
 * launches that cover both factors (the shifts; the residues) instead of seven, and in
 * accurate mode the passes that precede Cbar (maxima; Abar and Bbar) likewise.  The result
 * and every stage are bit-identical.  oz2_set_small_conversion(0) uses the general kernels
 * at every size.
 */
void oz2_set_small_conversion(int on);

/*
 * Per-stage timing.  With profiling on, each call records HIP events around its
 * stages on the call's stream; oz2_last_stage_times_ms waits for the last call
 * and writes { scale+exponent, residues, INT8 GEMM, epilogue } in milliseconds
 * to a HOST array.  Off by default (no events are recorded then).  For an overlapped call
 * (see oz2_set_overlap) the four numbers are: the shifts; the part of the residues that
 * precedes the first GEMM; the sum of the GEMM launches of all panels (events on `stream`
 * around each); the rest of the call (the accumulations, waits for residues).
 */
void oz2_set_profiling(int on);
oz2_status oz2_last_stage_times_ms(float *out4);
oz2_status oz2_ctx_last_stage_times_ms(oz2_context *ctx, float *out4);

/* Static text for a status code. */
const char *oz2_status_string(oz2_status s);

#ifdef __cplusplus
}
#endif
#endif /* OZ2_H */
