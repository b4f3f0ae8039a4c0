// C ABI of the library (declared in include/oz2.h): argument checks, workspace
// carving and the launch sequence of Algorithm 1 on the caller's stream.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <mutex>

#include "../../include/oz2.h"
#include "oz2_constants.hpp"
#include "oz2_kernels.hpp"

namespace {

using namespace oz2;

inline int64_t round_up(int64_t x, int64_t to) { return (x + to - 1) / to * to; }
inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

struct Layout {
    int64_t m, n, k, Mp, Np, Kp;
    int N;
    bool prod_u8;
    size_t off_bt, off_ta, off_tb, off_ra, off_rb, off_prod, total;
};

Layout make_layout(int64_t m, int64_t n, int64_t k, int N, bool prod_u8) {
    Layout L{};
    L.m = m; L.n = n; L.k = k; L.N = N; L.prod_u8 = prod_u8;
    L.Mp = round_up(m, kPadMN); L.Np = round_up(n, kPadMN); L.Kp = round_up(k, kPadK);
    size_t o = 0;
    L.off_bt = o;   o += align256(std::max(column_scratch_bytes(n), accurate_scratch_bytes(m, n)));
    L.off_ta = o;   o += align256((size_t)m * 4);
    L.off_tb = o;   o += align256((size_t)n * 4);
    L.off_ra = o;   o += align256((size_t)N * L.Mp * L.Kp);
    L.off_rb = o;   o += align256((size_t)N * L.Np * L.Kp);
    // products: N planes of uint8, or of int32 (diagnostic form; accurate mode also keeps
    // its int32 Cbar in plane 0, hence at least one int32 plane)
    L.off_prod = o; o += align256(std::max((size_t)N * L.Mp * L.Np * (prod_u8 ? 1 : 4), (size_t)L.Mp * L.Np * 4));
    L.total = o;
    return L;
}

struct State {
    std::mutex mu;
    char *ws = nullptr;
    size_t ws_bytes = 0;
    bool ws_owned = false;
    Layout last{};
    bool have_last = false;
    bool profiling = false;
    bool int32_products = false;           // diagnostic form: keep C'_s as int32
    hipEvent_t ev[5] = {nullptr, nullptr, nullptr, nullptr, nullptr};
    bool ev_recorded = false;
};
State g;

bool supported(int64_t k, int N) {
    return N >= OZ2_MIN_MODULI && N <= OZ2_MAX_MODULI && k <= OZ2_MAX_K_BLOCKED;
}

oz2_status ensure_workspace(size_t need) {
    if (g.ws && g.ws_bytes >= need) return OZ2_OK;
    if (g.ws && !g.ws_owned) return OZ2_WORKSPACE;            // caller-owned and too small
    if (g.ws) {
        if (hipDeviceSynchronize() != hipSuccess) return OZ2_HIP_ERROR;
        (void)hipFree(g.ws);
        g.ws = nullptr; g.ws_bytes = 0;
    }
    void *p = nullptr;
    if (hipMalloc(&p, need) != hipSuccess) { (void)hipGetLastError(); return OZ2_WORKSPACE; }
    g.ws = static_cast<char *>(p); g.ws_bytes = need; g.ws_owned = true;
    return OZ2_OK;
}

#define OZ2_TRY(expr) do { if ((expr) != hipSuccess) return OZ2_HIP_ERROR; } while (0)

oz2_status mark(int i, hipStream_t stream) {
    if (!g.profiling) return OZ2_OK;
    if (!g.ev[i]) OZ2_TRY(hipEventCreate(&g.ev[i]));
    OZ2_TRY(hipEventRecord(g.ev[i], stream));
    return OZ2_OK;
}

template <typename T>
oz2_status gemm_impl(int64_t m, int64_t n, int64_t k, double alpha, const T *A, int64_t lda,
                     const T *B, int64_t ldb, double beta, T *C, int64_t ldc, int N,
                     hipStream_t stream, bool accurate) {
    if (m < 0 || n < 0 || k < 0) return OZ2_INVALID_ARG;
    if (!supported(k, N) || (accurate && k > OZ2_MAX_K)) return OZ2_UNSUPPORTED;
    if (m == 0 || n == 0) return OZ2_OK;
    if (!C || ldc < n) return OZ2_INVALID_ARG;
    if (k == 0) {
        OZ2_TRY(launch_scale_c<T>(C, ldc, m, n, beta, stream));
        return OZ2_OK;
    }
    if (!A || !B || lda < k || ldb < n) return OZ2_INVALID_ARG;

    std::lock_guard<std::mutex> lock(g.mu);
    const bool is_double = sizeof(T) == 8;
    const Table &tab = table(N, is_double);
    const ModArgs ma = make_mod_args(tab);
    const ShiftArgs sa = make_shift_args(tab);
    const Layout L = make_layout(m, n, k, N, !g.int32_products);
    if (oz2_status st = ensure_workspace(L.total)) return st;
    g.last = L; g.have_last = true; g.ev_recorded = false;

    void *col_scratch = g.ws + L.off_bt;
    int32_t *tA = reinterpret_cast<int32_t *>(g.ws + L.off_ta);
    int32_t *tB = reinterpret_cast<int32_t *>(g.ws + L.off_tb);
    int8_t *rA = reinterpret_cast<int8_t *>(g.ws + L.off_ra);
    int8_t *rB = reinterpret_cast<int8_t *>(g.ws + L.off_rb);
    void *prod = g.ws + L.off_prod;

    if (oz2_status st = mark(0, stream)) return st;
    if (accurate) {
        // Section 4.2, accurate mode: 7-bit matrices into slice 0, Cbar into plane 0.
        OZ2_TRY(launch_accurate_prescale<T>(A, lda, B, ldb, m, n, k, col_scratch, rA, rB, L.Mp, L.Np,
                                            L.Kp, stream));
        OZ2_TRY(launch_int8_gemm(rA, rB, prod, 1, L.Mp, L.Np, L.Kp, 0, L.Kp, false, false, nullptr,
                                 stream));
        OZ2_TRY(launch_accurate_shifts(static_cast<const int32_t *>(prod), L.Np, m, n,
                                       make_accu_shift_args(tab), col_scratch, tA, tB, stream));
    } else {
        OZ2_TRY(launch_shifts<T>(A, lda, m, k, sa, tA, stream));
        OZ2_TRY(launch_shifts_cols<T>(B, ldb, k, n, sa, col_scratch, tB, stream));
    }
    if (oz2_status st = mark(1, stream)) return st;
    OZ2_TRY(launch_residues<T>(A, lda, m, k, tA, ma, rA, L.Mp, L.Kp, stream));
    OZ2_TRY(launch_residues_cols<T>(B, ldb, k, n, tB, ma, rB, L.Np, L.Kp, stream));
    if (oz2_status st = mark(2, stream)) return st;
    // Section 4.3: INT32 accumulation is exact for k <= 2^17; a longer contraction is cut into
    // K ranges of at most 2^17 whose reduced results are folded together modulo p_s.
    for (int64_t k0 = 0; k0 < L.Kp; k0 += OZ2_MAX_K) {
        const int64_t len = std::min<int64_t>(OZ2_MAX_K, L.Kp - k0);
        OZ2_TRY(launch_int8_gemm(rA, rB, prod, N, L.Mp, L.Np, L.Kp, k0, len, L.prod_u8, k0 > 0, &ma,
                                 stream));
    }
    if (oz2_status st = mark(3, stream)) return st;
    OZ2_TRY(launch_epilogue<T>(prod, L.prod_u8, L.Mp, L.Np, m, n, tA, tB, ma, alpha, beta, C, ldc,
                               stream));
    if (oz2_status st = mark(4, stream)) return st;
    g.ev_recorded = g.profiling;
    return OZ2_OK;
}

}  // namespace

extern "C" {

oz2_status oz2_dgemm(int64_t m, int64_t n, int64_t k, double alpha, const double *A, int64_t lda,
                     const double *B, int64_t ldb, double beta, double *C, int64_t ldc,
                     int num_moduli, hipStream_t stream) {
    return gemm_impl<double>(m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, num_moduli, stream, false);
}

oz2_status oz2_dgemm_accurate(int64_t m, int64_t n, int64_t k, double alpha, const double *A,
                              int64_t lda, const double *B, int64_t ldb, double beta, double *C,
                              int64_t ldc, int num_moduli, hipStream_t stream) {
    return gemm_impl<double>(m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, num_moduli, stream, true);
}

oz2_status oz2_sgemm_accurate(int64_t m, int64_t n, int64_t k, float alpha, const float *A,
                              int64_t lda, const float *B, int64_t ldb, float beta, float *C,
                              int64_t ldc, int num_moduli, hipStream_t stream) {
    return gemm_impl<float>(m, n, k, (double)alpha, A, lda, B, ldb, (double)beta, C, ldc,
                            num_moduli, stream, true);
}

oz2_status oz2_sgemm(int64_t m, int64_t n, int64_t k, float alpha, const float *A, int64_t lda,
                     const float *B, int64_t ldb, float beta, float *C, int64_t ldc,
                     int num_moduli, hipStream_t stream) {
    return gemm_impl<float>(m, n, k, (double)alpha, A, lda, B, ldb, (double)beta, C, ldc,
                            num_moduli, stream, false);
}

size_t oz2_workspace_bytes(int64_t m, int64_t n, int64_t k, int num_moduli, int is_double) {
    if (m <= 0 || n <= 0 || k <= 0 || !supported(k, num_moduli)) return 0;
    (void)is_double;                                          // the workspace holds no input-typed data
    return make_layout(m, n, k, num_moduli, !g.int32_products).total;
}

oz2_status oz2_set_workspace(void *dev_ptr, size_t bytes) {
    std::lock_guard<std::mutex> lock(g.mu);
    if (dev_ptr && (reinterpret_cast<uintptr_t>(dev_ptr) & 255)) return OZ2_INVALID_ARG;
    if (g.ws && g.ws_owned) {
        if (hipDeviceSynchronize() != hipSuccess) return OZ2_HIP_ERROR;
        (void)hipFree(g.ws);
    }
    g.ws = static_cast<char *>(dev_ptr);
    g.ws_bytes = dev_ptr ? bytes : 0;
    g.ws_owned = false;
    g.have_last = false;
    return OZ2_OK;
}

void oz2_release(void) {
    std::lock_guard<std::mutex> lock(g.mu);
    if (g.ws && g.ws_owned) {
        (void)hipDeviceSynchronize();
        (void)hipFree(g.ws);
    }
    g.ws = nullptr; g.ws_bytes = 0; g.ws_owned = false; g.have_last = false;
    for (auto &e : g.ev) if (e) { (void)hipEventDestroy(e); e = nullptr; }
    g.ev_recorded = false;
}

oz2_status oz2_constants(int num_moduli, int is_double, int32_t *p, uint32_t *pinv_prime,
                         double *s1, double *s2, double *P1P2Pinv, float *Pfast) {
    if (num_moduli < OZ2_MIN_MODULI || num_moduli > OZ2_MAX_MODULI) return OZ2_UNSUPPORTED;
    const Table &t = table(num_moduli, is_double != 0);
    for (int i = 0; i < t.n; ++i) {
        if (p) p[i] = t.p[i];
        if (pinv_prime) pinv_prime[i] = t.pinv_prime[i];
        if (s1) s1[i] = t.s1[i];
        if (s2) s2[i] = t.s2[i];
    }
    if (P1P2Pinv) { P1P2Pinv[0] = t.P1; P1P2Pinv[1] = t.P2; P1P2Pinv[2] = t.Pinv; }
    if (Pfast) *Pfast = t.Pfast;
    return OZ2_OK;
}

oz2_status oz2_shift_table(int num_moduli, int32_t *f_max, int32_t *levels, uint64_t *theta) {
    if (num_moduli < OZ2_MIN_MODULI || num_moduli > OZ2_MAX_MODULI) return OZ2_UNSUPPORTED;
    const Table &t = table(num_moduli, true);                 // P'_fast is the same for both widths
    if (t.levels < 1) return OZ2_UNSUPPORTED;
    if (f_max) *f_max = t.f_max;
    if (levels) *levels = t.levels;
    if (theta) for (int j = 0; j < t.levels; ++j) theta[j] = t.theta[j];
    return OZ2_OK;
}

oz2_status oz2_shift_table_accurate(int num_moduli, float *Paccu, int32_t *f_max, int32_t *levels,
                                    uint64_t *theta) {
    if (num_moduli < OZ2_MIN_MODULI || num_moduli > OZ2_MAX_MODULI) return OZ2_UNSUPPORTED;
    const Table &t = table(num_moduli, true);
    if (t.accu_levels < 1) return OZ2_UNSUPPORTED;
    if (Paccu) *Paccu = t.Paccu;
    if (f_max) *f_max = t.accu_f_max;
    if (levels) *levels = t.accu_levels;
    if (theta) for (int j = 0; j < t.accu_levels; ++j) theta[j] = t.accu_theta[j];
    return OZ2_OK;
}

oz2_status oz2_stage_ptr(int stage, void **dev_ptr, int64_t *dims) {
    std::lock_guard<std::mutex> lock(g.mu);
    if (!g.have_last || !dev_ptr || !dims) return OZ2_INVALID_ARG;
    const Layout &L = g.last;
    switch (stage) {
    case OZ2_STAGE_SHIFT_A: *dev_ptr = g.ws + L.off_ta; dims[0] = L.m; dims[1] = dims[2] = dims[3] = 0; break;
    case OZ2_STAGE_SHIFT_B: *dev_ptr = g.ws + L.off_tb; dims[0] = L.n; dims[1] = dims[2] = dims[3] = 0; break;
    case OZ2_STAGE_RES_A: *dev_ptr = g.ws + L.off_ra; dims[0] = L.N; dims[1] = L.Mp; dims[2] = L.Kp; dims[3] = L.m; break;
    case OZ2_STAGE_RES_B: *dev_ptr = g.ws + L.off_rb; dims[0] = L.N; dims[1] = L.Np; dims[2] = L.Kp; dims[3] = L.n; break;
    case OZ2_STAGE_PROD:
        if (L.prod_u8) return OZ2_INVALID_ARG;                // not kept in this form: see oz2_set_int32_products
        *dev_ptr = g.ws + L.off_prod; dims[0] = L.N; dims[1] = L.Mp; dims[2] = L.Np; dims[3] = 0; break;
    case OZ2_STAGE_U:
        if (!L.prod_u8) return OZ2_INVALID_ARG;
        *dev_ptr = g.ws + L.off_prod; dims[0] = L.N; dims[1] = L.Mp; dims[2] = L.Np; dims[3] = 0; break;
    default: return OZ2_INVALID_ARG;
    }
    return OZ2_OK;
}

oz2_status oz2_int8_gemm(const int8_t *dev_A, const int8_t *dev_B, int32_t *dev_C, int batch,
                         int64_t Mp, int64_t Np, int64_t Kp, hipStream_t stream) {
    if (!dev_A || !dev_B || !dev_C || batch < 1 || batch > 65535 || Mp < kPadMN || Np < kPadMN ||
        Kp < kPadK || Mp % kPadMN || Np % kPadMN || Kp % kPadK)
        return OZ2_INVALID_ARG;
    if (Kp > OZ2_MAX_K) return OZ2_UNSUPPORTED;
    OZ2_TRY(launch_int8_gemm(dev_A, dev_B, dev_C, batch, Mp, Np, Kp, 0, Kp, false, false, nullptr, stream));
    return OZ2_OK;
}

void oz2_set_int32_products(int on) {
    std::lock_guard<std::mutex> lock(g.mu);
    g.int32_products = on != 0;
}

void oz2_set_profiling(int on) {
    std::lock_guard<std::mutex> lock(g.mu);
    g.profiling = on != 0;
    if (!g.profiling) g.ev_recorded = false;
}

oz2_status oz2_last_stage_times_ms(float *out4) {
    std::lock_guard<std::mutex> lock(g.mu);
    if (!out4 || !g.ev_recorded) return OZ2_INVALID_ARG;
    OZ2_TRY(hipEventSynchronize(g.ev[4]));
    for (int i = 0; i < 4; ++i) OZ2_TRY(hipEventElapsedTime(&out4[i], g.ev[i], g.ev[i + 1]));
    return OZ2_OK;
}

const char *oz2_status_string(oz2_status s) {
    switch (s) {
    case OZ2_OK: return "ok";
    case OZ2_INVALID_ARG: return "invalid argument";
    case OZ2_UNSUPPORTED: return "unsupported number of moduli or k > 2^17";
    case OZ2_WORKSPACE: return "workspace too small or allocation failed";
    case OZ2_HIP_ERROR: return "HIP runtime error";
    }
    return "unknown status";
}

}  // extern "C"
