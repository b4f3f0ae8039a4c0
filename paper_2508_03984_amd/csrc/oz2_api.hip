// C ABI of the library (declared in include/oz2.h): argument checks, workspace
// carving and the launch sequence of Algorithm 1 on the caller's stream.  All state lives in
// contexts (oz2_context); the entry points without a context use the process's default one.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <cstdlib>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/oz2.h"
#include "oz2_constants.hpp"
#include "oz2_kernels.hpp"
#include "oz2_plan.hpp"

// Everything a product call keeps between its launches and for the diagnostics that follow it:
// one workspace, the options, the events of the per-stage timing and the second stream of the
// overlapped form.  Calls on one context share its workspace, so they must be ordered by the
// caller (one stream, or events); calls on different contexts are independent.
struct oz2_context {
    std::mutex mu;                         // guards the host-side fields below, not the device buffers
    char *ws = nullptr;
    size_t ws_bytes = 0;
    bool ws_owned = false;
    int ws_device = -1;                    // device of the library's own buffer
    size_t ws_limit = 0;                   // for the library's own buffer; 0 = none
    oz2::Layout last{};
    oz2::Panels last_panels{0, 0, 0};
    int64_t last_gemm_launches = 0;        // INT8 GEMM launches of the products of the last call
    bool have_last = false;                // shifts and residues of the last call are in the workspace
    bool have_last_prod = false;           // ... and so are all its products
    bool have_panels = false;
    bool profiling = false;
    bool int32_products = false;           // diagnostic form: keep C'_s as int32
    bool overlap = false;                  // conversion of later panels beside the GEMMs (run_overlapped)
    bool small_conversion = true;          // fused conversion launches for small problems (oz2_small.hip)
    bool cut_launches = true;              // GEMM launches of a large product cut into parts (launch_panels)
    hipEvent_t ev[5] = {nullptr, nullptr, nullptr, nullptr, nullptr};
    bool ev_recorded = false;
    // overlapped form: a second stream, ordering events, and with profiling one pair of timing
    // events per panel around its INT8 GEMMs
    hipStream_t aux = nullptr;
    std::vector<hipEvent_t> sync_ev, time_ev;
    int64_t last_overlapped_panels = 0;    // > 0: the last call ran overlapped, with this many panels
    int res_device = -1;                   // device the events and the second stream belong to
};

namespace {

using namespace oz2;
typedef oz2_context Ctx;

// The context behind the entry points that take none.  It is never destroyed: at process exit the
// HIP runtime may already be gone, and the driver reclaims the device memory anyway.
Ctx &default_context() {
    static Ctx *c = new Ctx();
    return *c;
}
inline Ctx &resolve(oz2_context *c) { return c ? *c : default_context(); }

// Makes at least `need_min` bytes of workspace available, `need_whole` if nothing limits it;
// *have receives the bytes the call may use.  Growing the library's own buffer (or moving it to
// another device) waits for the device, frees and allocates: the only synchronising step of a
// product call, and only when the buffer is too small.
oz2_status ensure_workspace(Ctx &g, size_t need_whole, size_t need_min, size_t *have) {
    if (g.ws && !g.ws_owned) {                                // caller-owned: take it as it is
        if (g.ws_bytes < need_min) return OZ2_WORKSPACE;
        *have = g.ws_bytes;
        return OZ2_OK;
    }
    size_t want = need_whole;
    if (g.ws_limit && want > g.ws_limit) want = g.ws_limit;
    if (want < need_min) return OZ2_WORKSPACE;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return OZ2_HIP_ERROR;
    if (!g.ws || g.ws_bytes < want || g.ws_device != dev) {   // the buffer lives on the current device
        if (g.ws) {                                           // wait on the device that may still use it
            const bool elsewhere = g.ws_device != dev;
            if (elsewhere && hipSetDevice(g.ws_device) != hipSuccess) return OZ2_HIP_ERROR;
            const hipError_t e = hipDeviceSynchronize();
            (void)hipFree(g.ws);
            g.ws = nullptr; g.ws_bytes = 0;
            if (elsewhere && hipSetDevice(dev) != hipSuccess) return OZ2_HIP_ERROR;
            if (e != hipSuccess) return OZ2_HIP_ERROR;
        }
        void *p = nullptr;
        if (hipMalloc(&p, want) != hipSuccess) { (void)hipGetLastError(); return OZ2_WORKSPACE; }
        g.ws = static_cast<char *>(p); g.ws_bytes = want; g.ws_owned = true; g.ws_device = dev;
    }
    *have = g.ws_limit ? std::min(g.ws_bytes, std::max(g.ws_limit, need_min)) : g.ws_bytes;
    return OZ2_OK;
}

#define OZ2_TRY(expr) do { if ((expr) != hipSuccess) return OZ2_HIP_ERROR; } while (0)

// Events and the second stream belong to one device: a call made with another device current
// drops them (they are created again when needed).
void drop_device_resources(Ctx &g) {
    for (auto &e : g.ev) if (e) { (void)hipEventDestroy(e); e = nullptr; }
    for (auto &e : g.sync_ev) (void)hipEventDestroy(e);
    for (auto &e : g.time_ev) (void)hipEventDestroy(e);
    g.sync_ev.clear(); g.time_ev.clear();
    if (g.aux) { (void)hipStreamDestroy(g.aux); g.aux = nullptr; }
    g.ev_recorded = false; g.last_overlapped_panels = 0;
}

oz2_status bind_device_resources(Ctx &g) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return OZ2_HIP_ERROR;
    if (g.res_device != dev) {
        drop_device_resources(g);
        g.res_device = dev;
    }
    return OZ2_OK;
}

oz2_status mark(Ctx &g, int i, hipStream_t stream) {
    if (!g.profiling) return OZ2_OK;
    if (!g.ev[i]) OZ2_TRY(hipEventCreate(&g.ev[i]));
    OZ2_TRY(hipEventRecord(g.ev[i], stream));
    return OZ2_OK;
}

// Algorithm 1 lines 1-5 (fast mode) for one factor: its shifts and its residue slices.  The
// vectors that get a scale factor (rows of op(A), columns of op(B)) are either contiguous in the
// stored matrix (row kernels) or strided by its leading dimension (column kernels).
template <typename T>
hipError_t launch_fast_shifts(const T *X, int64_t ld, bool k_contiguous, int64_t rows, int64_t k,
                              const ShiftArgs &sa, void *scratch, int32_t *t, hipStream_t stream) {
    return k_contiguous ? launch_shifts<T>(X, ld, rows, k, sa, t, stream)
                        : launch_shifts_cols<T>(X, ld, k, rows, sa, scratch, t, stream);
}

template <typename T>
hipError_t launch_any_residues(const T *X, int64_t ld, bool k_contiguous, int64_t rows, int64_t k,
                               const int32_t *t, const ModArgs &ma, int8_t *out, int64_t rows_pad,
                               int64_t Kp, hipStream_t stream) {
    return k_contiguous ? launch_residues<T>(X, ld, rows, k, t, ma, out, rows_pad, Kp, stream)
                        : launch_residues_cols<T>(X, ld, k, rows, t, ma, out, rows_pad, Kp, stream);
}

// The same for the block of vectors [v0, v0 + block) of a factor with `rows` vectors
// (block a multiple of 256): only that part of the slices is written.
template <typename T>
hipError_t launch_block_residues(const T *X, int64_t ld, bool k_contiguous, int64_t rows, int64_t k,
                                 const int32_t *t, const ModArgs &ma, int8_t *out, int64_t rows_pad,
                                 int64_t Kp, int64_t v0, int64_t block, hipStream_t stream) {
    const int64_t valid = std::min(rows - v0, block);          // >= 1: v0 < rows
    const T *Xb = X + (k_contiguous ? v0 * ld : v0);
    return k_contiguous
               ? launch_residues<T>(Xb, ld, valid, k, t + v0, ma, out + v0 * kBlockK, block, Kp, stream, rows_pad)
               : launch_residues_cols<T>(Xb, ld, k, valid, t + v0, ma, out + v0 * kBlockK, block, Kp, stream,
                                         rows_pad);
}

// Algorithm 1 lines 6-12 panel by panel: the INT8 GEMMs of one panel of C (Section 4.3: exact
// INT32 accumulation for k <= 2^17; a longer contraction is cut into K ranges of at most 2^17
// whose reduced results are folded together modulo p_s), then its accumulation and unscaling.
template <typename T>
oz2_status run_products(Ctx &g, const Layout &L, const Panels &P, const int8_t *rA, const int8_t *rB,
                        const int32_t *tA, const int32_t *tB, void *prod, const ModArgs &ma,
                        double alpha, double beta, T *C, int64_t ldc, hipStream_t stream) {
    // The product buffer holds one panel of C at a time: [N][rows][cols] (all of C if P.count is 1).
    // The GEMM launches of a panel are cut further (launch_panels, launch_k_len), each writing its
    // part of the buffer in place.  (The diagnostic int32 form keeps the raw sums C'_s of a whole
    // contraction up to 2^17.)
    const size_t entry = L.prod_u8 ? 1 : 4;
    int64_t done = 0;
    for (int64_t row0 = 0; row0 < L.Mp; row0 += P.pr)
        for (int64_t col0 = 0; col0 < L.Np; col0 += P.pc) {
            const int64_t rows = std::min(P.pr, L.Mp - row0), cols = std::min(P.pc, L.Np - col0);
            const Panels Q = g.cut_launches ? launch_panels(rows, cols, L.Kp) : Panels{rows, cols, 1};
            const int64_t k_len = g.cut_launches && L.prod_u8 ? launch_k_len(L.Kp, L.N, Q) : std::min<int64_t>(L.Kp, OZ2_MAX_K);
            for (int64_t r1 = 0; r1 < rows; r1 += Q.pr)
                for (int64_t c1 = 0; c1 < cols; c1 += Q.pc) {
                    const GemmPanel pn{row0 + r1, std::min(Q.pr, rows - r1), col0 + c1, std::min(Q.pc, cols - c1), cols,
                                       rows * cols};
                    void *dst = static_cast<char *>(prod) + (size_t)(r1 * cols + c1) * entry;
                    for (int64_t k0 = 0; k0 < L.Kp; k0 += k_len) {
                        ++g.last_gemm_launches;
                        OZ2_TRY(launch_int8_gemm(rA, rB, dst, L.N, L.Mp, L.Np, L.Kp, k0, std::min<int64_t>(k_len, L.Kp - k0),
                                                 L.prod_u8, k0 > 0, &ma, stream, &pn));
                    }
                }
            if (++done == P.count)                            // stage times: the last accumulation only
                if (oz2_status st = mark(g, 3, stream)) return st;
            OZ2_TRY(launch_epilogue<T>(prod, L.prod_u8, rows, cols, std::min(L.m - row0, rows),
                                       std::min(L.n - col0, cols), tA + row0, tB + col0, ma, alpha, beta,
                                       C + row0 * ldc + col0, ldc, stream));
        }
    return mark(g, 4, stream);
}

oz2_status overlap_resources(Ctx &g, size_t n_sync, size_t n_time) {
    if (!g.aux) OZ2_TRY(hipStreamCreateWithFlags(&g.aux, hipStreamNonBlocking));   // default priority
    while (g.sync_ev.size() < n_sync) {
        hipEvent_t e = nullptr;
        OZ2_TRY(hipEventCreateWithFlags(&e, hipEventDisableTiming));
        g.sync_ev.push_back(e);
    }
    while (g.time_ev.size() < n_time) {
        hipEvent_t e = nullptr;
        OZ2_TRY(hipEventCreate(&e));
        g.time_ev.push_back(e);
    }
    return OZ2_OK;
}

// Algorithm 1 lines 2-12 with the conversion to residues hidden behind the INT8 GEMMs.  The
// shifts are known.  C is cut into panels; on the caller's stream the GEMMs and the accumulation
// of one panel after the other; on a second stream, while they run, the residues of the row
// block of A and the column block of B that the NEXT panel needs (each block once, the first
// time a panel needs it).  Every dependency is an event; the second stream forks from the
// caller's after the shifts and has nothing left to do when the last panel starts, so the call
// as a whole is ordered on the caller's stream like any other (and can be captured into a
// graph).  Measured at 16 x 16384^3 on one device: 61.2 ms against 62.2 ms on one stream; also
// moving the accumulations to the second stream (two product buffers) was slower (61.7 ms: the
// GEMMs lose more to the accumulations beside them than those take on their own), and so were
// launches made "thin" for the registers a resident GEMM workgroup leaves free (64.6 ms).
template <typename T>
oz2_status run_overlapped(Ctx &g, const Layout &L, const Panels &P, const T *A, int64_t lda, bool a_kc, const T *B,
                          int64_t ldb, bool b_kc, const int32_t *tA, const int32_t *tB, int8_t *rA,
                          int8_t *rB, void *prod, const ModArgs &ma, double alpha, double beta, T *C,
                          int64_t ldc, hipStream_t stream) {
    const int64_t nR = (L.Mp + P.pr - 1) / P.pr, nC = (L.Np + P.pc - 1) / P.pc, count = nR * nC;
    // events: [0] fork, [1 .. nR] residues of the A blocks, then nC for the B blocks
    const size_t eA = 1, eB = eA + (size_t)nR;
    if (oz2_status st = overlap_resources(g, eB + (size_t)nC, g.profiling ? 2 * (size_t)count : 0)) return st;
    hipEvent_t *ev = g.sync_ev.data();
    hipStream_t aux = g.aux;
    OZ2_TRY(hipEventRecord(ev[0], stream));
    OZ2_TRY(hipStreamWaitEvent(aux, ev[0], 0));

    auto residues_a = [&](int64_t i) -> hipError_t {
        if (hipError_t e = launch_block_residues<T>(A, lda, a_kc, L.m, L.k, tA, ma, rA, L.Mp, L.Kp, i * P.pr,
                                                    std::min(P.pr, L.Mp - i * P.pr), aux))
            return e;
        return hipEventRecord(ev[eA + i], aux);
    };
    auto residues_b = [&](int64_t j) -> hipError_t {
        if (hipError_t e = launch_block_residues<T>(B, ldb, b_kc, L.n, L.k, tB, ma, rB, L.Np, L.Kp, j * P.pc,
                                                    std::min(P.pc, L.Np - j * P.pc), aux))
            return e;
        return hipEventRecord(ev[eB + j], aux);
    };
    // The second stream's program: the blocks in the order in which the panels (row by row)
    // first need them.  It runs ahead of the GEMMs as far as it can.
    OZ2_TRY(residues_a(0));
    for (int64_t j = 0; j < nC; ++j) OZ2_TRY(residues_b(j));
    for (int64_t i = 1; i < nR; ++i) OZ2_TRY(residues_a(i));

    for (int64_t p = 0; p < count; ++p) {
        const int64_t i = p / nC, j = p % nC;
        const int64_t row0 = i * P.pr, col0 = j * P.pc;
        const int64_t rows = std::min(P.pr, L.Mp - row0), cols = std::min(P.pc, L.Np - col0);
        if (j == 0) OZ2_TRY(hipStreamWaitEvent(stream, ev[eA + i], 0));
        if (i == 0) OZ2_TRY(hipStreamWaitEvent(stream, ev[eB + j], 0));
        if (g.profiling) OZ2_TRY(hipEventRecord(g.time_ev[2 * p], stream));
        const GemmPanel pn{row0, rows, col0, cols, cols, rows * cols};
        for (int64_t k0 = 0; k0 < L.Kp; k0 += OZ2_MAX_K) {
            const int64_t len = std::min<int64_t>(OZ2_MAX_K, L.Kp - k0);
            ++g.last_gemm_launches;
            OZ2_TRY(launch_int8_gemm(rA, rB, prod, L.N, L.Mp, L.Np, L.Kp, k0, len, L.prod_u8, k0 > 0, &ma, stream,
                                     &pn));
        }
        if (g.profiling) OZ2_TRY(hipEventRecord(g.time_ev[2 * p + 1], stream));
        OZ2_TRY(launch_epilogue<T>(prod, L.prod_u8, rows, cols, std::min(L.m - row0, rows),
                                   std::min(L.n - col0, cols), tA + row0, tB + col0, ma, alpha, beta,
                                   C + row0 * ldc + col0, ldc, stream));
    }
    // The caller's stream has waited for every event of the second one: the two have joined.
    g.last_overlapped_panels = count;
    return mark(g, 4, stream);
}

template <typename T>
oz2_status gemm_impl(Ctx &g, int opA, int opB, int64_t m, int64_t n, int64_t k, double alpha, const T *A,
                     int64_t lda, const T *B, int64_t ldb, double beta, T *C, int64_t ldc, int N,
                     hipStream_t stream, bool accurate) {
    Action action;
    if (oz2_status st = check_gemm_args(opA, opB, m, n, k, A, lda, B, ldb, C, ldc, N, &action)) return st;
    if (action == Action::kNothing) return OZ2_OK;
    if (action == Action::kScaleC) {
        OZ2_TRY(launch_scale_c<T>(C, ldc, m, n, beta, stream));
        return OZ2_OK;
    }
    const bool a_kc = opA == OZ2_OP_N, b_kc = opB == OZ2_OP_T;   // is k the contiguous index?

    std::lock_guard<std::mutex> lock(g.mu);
    if (oz2_status st = bind_device_resources(g)) return st;
    const bool is_double = sizeof(T) == 8;
    const Table &tab = table(N, is_double);
    const ModArgs ma = make_mod_args(tab, accurate);
    const ShiftArgs sa = make_shift_args(tab);
    const Layout L = make_layout(m, n, k, N, !g.int32_products);
    // The overlapped form (an option, see run_overlapped) works through C in panels of at most
    // 4096 x 4096 whatever the workspace could hold, so the library's own buffer is then sized for
    // the products of one such panel.
    const int64_t side_r = std::min(L.Mp, kOverlapPanel), side_c = std::min(L.Np, kOverlapPanel);
    const int64_t panels_4096 = ((L.Mp + side_r - 1) / side_r) * ((L.Np + side_c - 1) / side_c);
    const size_t prod_want = g.overlap && overlap_applies(L.Kp, panels_4096)
                                 ? align256((size_t)side_r * side_c * bytes_per_entry(N, L.prod_u8))
                                 : L.prod_whole;
    size_t have = 0;
    Panels P{};
    if (oz2_status st = ensure_workspace(g, L.off_prod + prod_want, L.off_prod + L.prod_min, &have)) return st;
    if (!plan_panels(L, have - L.off_prod, &P)) return OZ2_WORKSPACE;
    const Panels Po = overlap_panels(L, P);                // a workspace limit may have made the panels smaller
    const bool overlapped = g.overlap && overlap_applies(L.Kp, Po.count);
    if (overlapped) P = Po;
    g.last = L; g.last_panels = P; g.have_panels = true; g.last_overlapped_panels = 0; g.last_gemm_launches = 0;
    g.have_last = true; g.have_last_prod = P.count == 1; g.ev_recorded = false;

    void *scratch = g.ws + L.off_bt;
    int32_t *tA = reinterpret_cast<int32_t *>(g.ws + L.off_ta);
    int32_t *tB = reinterpret_cast<int32_t *>(g.ws + L.off_tb);
    int8_t *rA = reinterpret_cast<int8_t *>(g.ws + L.off_ra);
    int8_t *rB = reinterpret_cast<int8_t *>(g.ws + L.off_rb);
    void *prod = g.ws + L.off_prod;

    // Small problems: the conversion of both factors in two launches instead of seven (and
    // likewise the passes of accurate mode that precede Cbar).
    const bool small = g.small_conversion && small_conversion_applies(m, n, k);
    if (oz2_status st = mark(g, 0, stream)) return st;
    if (accurate) {
        // Section 4.2, accurate mode: 7-bit matrices into slice 0; of Cbar only the row and
        // column maxima are kept (it is never stored).  A contraction beyond 2^17 is cut into K
        // ranges (Section 4.3, last sentence), each an exact INT32 product with maxima of its own;
        // their sum bounds the maxima of the whole Cbar from above, which is all that the chain of
        // inequalities behind the scale vectors needs.
        const int ranges = (int)((L.Kp + OZ2_MAX_K - 1) / OZ2_MAX_K);
        OZ2_TRY(launch_accurate_prescale<T>(A, lda, a_kc, B, ldb, b_kc, m, n, k, ranges, scratch, rA, rB, L.Mp,
                                            L.Np, L.Kp, small, stream));
        const GemmPanel all{0, L.Mp, 0, L.Np, L.Np, L.Mp * L.Np};      // nothing is stored: no panels needed
        for (int r = 0; r < ranges; ++r) {
            int *row_max = nullptr, *col_max = nullptr;
            accurate_maxima(scratch, m, n, r, &row_max, &col_max);
            const int64_t k0 = (int64_t)r * OZ2_MAX_K;
            OZ2_TRY(launch_int8_gemm_maxima(rA, rB, L.Mp, L.Np, L.Kp, k0, std::min<int64_t>(OZ2_MAX_K, L.Kp - k0),
                                            all, m, n, row_max, col_max, stream));
        }
        OZ2_TRY(launch_accurate_finish(m, n, ranges, make_accu_shift_args(tab), scratch, tA, tB, stream));
    } else if (small) {
        OZ2_TRY(launch_small_shifts<T>(A, lda, a_kc, B, ldb, b_kc, m, n, k, sa, tA, tB, stream));
    } else {
        OZ2_TRY(launch_fast_shifts<T>(A, lda, a_kc, m, k, sa, scratch, tA, stream));
        OZ2_TRY(launch_fast_shifts<T>(B, ldb, b_kc, n, k, sa, scratch, tB, stream));
    }
    if (oz2_status st = mark(g, 1, stream)) return st;
    if (overlapped) {
        if (oz2_status st = run_overlapped<T>(g, L, P, A, lda, a_kc, B, ldb, b_kc, tA, tB, rA, rB, prod, ma, alpha,
                                              beta, C, ldc, stream))
            return st;
        g.ev_recorded = g.profiling;
        return OZ2_OK;
    }
    if (small) {
        OZ2_TRY(launch_small_residues<T>(A, lda, a_kc, B, ldb, b_kc, m, n, k, ma, tA, tB, rA, rB, L.Mp, L.Np,
                                         L.Kp, stream));
    } else {
        OZ2_TRY(launch_any_residues<T>(A, lda, a_kc, m, k, tA, ma, rA, L.Mp, L.Kp, stream));
        OZ2_TRY(launch_any_residues<T>(B, ldb, b_kc, n, k, tB, ma, rB, L.Np, L.Kp, stream));
    }
    if (oz2_status st = mark(g, 2, stream)) return st;
    if (oz2_status st = run_products<T>(g, L, P, rA, rB, tA, tB, prod, ma, alpha, beta, C, ldc, stream)) return st;
    g.ev_recorded = g.profiling;
    return OZ2_OK;
}

}  // namespace

// A prepared factor (oz2_prepare_*): the shifts and residue slices of Algorithm 1 lines 1-5.
struct oz2_operand {
    int side;                              // 0 = left factor, 1 = right factor
    bool is_double;
    int N;
    int64_t rows, k, rows_pad, Kp;
    char *mem;                             // one device allocation: [t | residues | scratch]
    size_t bytes;
    int32_t *t;
    int8_t *res;
};

namespace {

template <typename T>
oz2_status prepare_impl(int side, int op, int64_t rows, int64_t k, const T *X, int64_t ld, int N,
                        hipStream_t stream, oz2_operand **out) {
    if (!out || (side != 0 && side != 1) || (op != OZ2_OP_N && op != OZ2_OP_T) || rows < 1 || k < 1 || !X)
        return OZ2_INVALID_ARG;
    if (!supported(k, N)) return OZ2_UNSUPPORTED;
    const bool k_contiguous = (side == 0) == (op == OZ2_OP_N);
    if (ld < (k_contiguous ? k : rows)) return OZ2_INVALID_ARG;

    const bool is_double = sizeof(T) == 8;
    const Table &tab = table(N, is_double);
    oz2_operand *o = new (std::nothrow) oz2_operand{};
    if (!o) return OZ2_WORKSPACE;
    o->side = side; o->is_double = is_double; o->N = N; o->rows = rows; o->k = k;
    o->rows_pad = round_up(rows, kPadMN); o->Kp = round_up(k, kPadK);
    const size_t off_res = align256((size_t)rows * 4);
    const size_t off_scratch = off_res + align256((size_t)N * o->rows_pad * o->Kp);
    o->bytes = off_scratch + align256(column_scratch_bytes(rows));
    void *p = nullptr;
    if (hipMalloc(&p, o->bytes) != hipSuccess) { (void)hipGetLastError(); delete o; return OZ2_WORKSPACE; }
    o->mem = static_cast<char *>(p);
    o->t = reinterpret_cast<int32_t *>(o->mem);
    o->res = reinterpret_cast<int8_t *>(o->mem + off_res);
    hipError_t e = launch_fast_shifts<T>(X, ld, k_contiguous, rows, k, make_shift_args(tab),
                                         o->mem + off_scratch, o->t, stream);
    if (e == hipSuccess)
        e = launch_any_residues<T>(X, ld, k_contiguous, rows, k, o->t, make_mod_args(tab, false), o->res,
                                   o->rows_pad, o->Kp, stream);
    if (e != hipSuccess) { (void)hipFree(o->mem); delete o; return OZ2_HIP_ERROR; }
    *out = o;
    return OZ2_OK;
}

template <typename T>
oz2_status prepared_impl(Ctx &g, const oz2_operand *l, const oz2_operand *r, double alpha, double beta, T *C,
                         int64_t ldc, hipStream_t stream) {
    const bool is_double = sizeof(T) == 8;
    if (!l || !r || l->side != 0 || r->side != 1 || l->k != r->k || l->N != r->N ||
        l->is_double != is_double || r->is_double != is_double || !C || ldc < r->rows)
        return OZ2_INVALID_ARG;
    std::lock_guard<std::mutex> lock(g.mu);
    if (oz2_status st = bind_device_resources(g)) return st;
    const ModArgs ma = make_mod_args(table(l->N, is_double), false);
    const Layout L = make_layout(l->rows, r->rows, l->k, l->N, !g.int32_products, false);
    size_t have = 0;
    Panels P{};
    if (oz2_status st = ensure_workspace(g, L.prod_whole, L.prod_min, &have)) return st;
    if (!plan_panels(L, have, &P)) return OZ2_WORKSPACE;
    g.last_panels = P; g.have_panels = true; g.last_overlapped_panels = 0; g.last_gemm_launches = 0;
    g.have_last = g.have_last_prod = false; g.ev_recorded = false;
    for (int i = 0; i < 3; ++i)
        if (oz2_status st = mark(g, i, stream)) return st;
    if (oz2_status st = run_products<T>(g, L, P, l->res, r->res, l->t, r->t, g.ws, ma, alpha, beta, C, ldc, stream))
        return st;
    g.ev_recorded = g.profiling;
    return OZ2_OK;
}

void release_workspace(Ctx &g) {                           // g.mu is held
    if (g.ws && g.ws_owned) {
        (void)hipDeviceSynchronize();
        (void)hipFree(g.ws);
    }
    g.ws = nullptr; g.ws_bytes = 0; g.ws_owned = false; g.have_last = g.have_last_prod = false;
    drop_device_resources(g);
    g.res_device = -1;
}

}  // namespace

extern "C" {

// ------------------------------------------------------------------ contexts
oz2_status oz2_create(oz2_context **out) {
    if (!out) return OZ2_INVALID_ARG;
    oz2_context *c = new (std::nothrow) oz2_context();
    if (!c) return OZ2_WORKSPACE;
    *out = c;
    return OZ2_OK;
}

oz2_status oz2_destroy(oz2_context *ctx) {
    if (!ctx) return OZ2_INVALID_ARG;
    {
        std::lock_guard<std::mutex> lock(ctx->mu);
        release_workspace(*ctx);
    }
    delete ctx;
    return OZ2_OK;
}

oz2_status oz2_ctx_set_option(oz2_context *ctx, oz2_option option, int value) {
    Ctx &g = resolve(ctx);
    std::lock_guard<std::mutex> lock(g.mu);
    const bool on = value != 0;
    switch (option) {
    case OZ2_OPT_INT32_PRODUCTS: g.int32_products = on; break;
    case OZ2_OPT_OVERLAP: g.overlap = on; break;
    case OZ2_OPT_SMALL_CONVERSION: g.small_conversion = on; break;
    case OZ2_OPT_CUT_LAUNCHES: g.cut_launches = on; break;
    case OZ2_OPT_PROFILING: g.profiling = on; if (!on) g.ev_recorded = false; break;
    default: return OZ2_INVALID_ARG;
    }
    return OZ2_OK;
}

oz2_status oz2_ctx_dgemm(oz2_context *ctx, oz2_op opA, oz2_op opB, int accurate, int64_t m, int64_t n, int64_t k,
                         double alpha, const double *A, int64_t lda, const double *B, int64_t ldb,
                         double beta, double *C, int64_t ldc, int num_moduli, hipStream_t stream) {
    return gemm_impl<double>(resolve(ctx), opA, opB, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, num_moduli,
                             stream, accurate != 0);
}

oz2_status oz2_ctx_sgemm(oz2_context *ctx, oz2_op opA, oz2_op opB, int accurate, int64_t m, int64_t n, int64_t k,
                         float alpha, const float *A, int64_t lda, const float *B, int64_t ldb, float beta,
                         float *C, int64_t ldc, int num_moduli, hipStream_t stream) {
    return gemm_impl<float>(resolve(ctx), opA, opB, m, n, k, (double)alpha, A, lda, B, ldb, (double)beta, C, ldc,
                            num_moduli, stream, accurate != 0);
}

oz2_status oz2_ctx_dgemm_prepared(oz2_context *ctx, const oz2_operand *left, const oz2_operand *right,
                                  double alpha, double beta, double *C, int64_t ldc, hipStream_t stream) {
    return prepared_impl<double>(resolve(ctx), left, right, alpha, beta, C, ldc, stream);
}

oz2_status oz2_ctx_sgemm_prepared(oz2_context *ctx, const oz2_operand *left, const oz2_operand *right,
                                  float alpha, float beta, float *C, int64_t ldc, hipStream_t stream) {
    return prepared_impl<float>(resolve(ctx), left, right, (double)alpha, (double)beta, C, ldc, stream);
}

size_t oz2_ctx_workspace_bytes(oz2_context *ctx, int64_t m, int64_t n, int64_t k, int num_moduli) {
    if (m <= 0 || n <= 0 || k <= 0 || !supported(k, num_moduli)) return 0;
    Ctx &g = resolve(ctx);
    std::lock_guard<std::mutex> lock(g.mu);
    const Layout L = make_layout(m, n, k, num_moduli, !g.int32_products);
    return L.off_prod + L.prod_whole;
}

size_t oz2_ctx_workspace_min_bytes(oz2_context *ctx, int64_t m, int64_t n, int64_t k, int num_moduli) {
    if (m <= 0 || n <= 0 || k <= 0 || !supported(k, num_moduli)) return 0;
    Ctx &g = resolve(ctx);
    std::lock_guard<std::mutex> lock(g.mu);
    const Layout L = make_layout(m, n, k, num_moduli, !g.int32_products);
    return L.off_prod + L.prod_min;
}

oz2_status oz2_ctx_set_workspace(oz2_context *ctx, void *dev_ptr, size_t bytes) {
    Ctx &g = resolve(ctx);
    std::lock_guard<std::mutex> lock(g.mu);
    if (dev_ptr && (reinterpret_cast<uintptr_t>(dev_ptr) & 255)) return OZ2_INVALID_ARG;
    if (g.ws && g.ws_owned) {
        if (hipDeviceSynchronize() != hipSuccess) return OZ2_HIP_ERROR;
        (void)hipFree(g.ws);
    }
    g.ws = static_cast<char *>(dev_ptr);
    g.ws_bytes = dev_ptr ? bytes : 0;
    g.ws_owned = false;
    g.have_last = g.have_last_prod = false;
    return OZ2_OK;
}

oz2_status oz2_ctx_set_workspace_limit(oz2_context *ctx, size_t bytes) {
    Ctx &g = resolve(ctx);
    std::lock_guard<std::mutex> lock(g.mu);
    g.ws_limit = bytes;
    return OZ2_OK;
}

oz2_status oz2_ctx_release(oz2_context *ctx) {
    Ctx &g = resolve(ctx);
    std::lock_guard<std::mutex> lock(g.mu);
    release_workspace(g);
    return OZ2_OK;
}

oz2_status oz2_ctx_plan_panels(oz2_context *ctx, int64_t m, int64_t n, int64_t k, int num_moduli,
                               size_t workspace_bytes, int64_t *panel_rows, int64_t *panel_cols, int64_t *count) {
    if (m <= 0 || n <= 0 || k <= 0) return OZ2_INVALID_ARG;
    if (!supported(k, num_moduli)) return OZ2_UNSUPPORTED;
    Ctx &g = resolve(ctx);
    std::lock_guard<std::mutex> lock(g.mu);
    const Layout L = make_layout(m, n, k, num_moduli, !g.int32_products);
    Panels P{};
    if (workspace_bytes < L.off_prod || !plan_panels(L, workspace_bytes - L.off_prod, &P)) return OZ2_WORKSPACE;
    if (panel_rows) *panel_rows = P.pr;
    if (panel_cols) *panel_cols = P.pc;
    if (count) *count = P.count;
    return OZ2_OK;
}

oz2_status oz2_ctx_last_panels(oz2_context *ctx, int64_t *panel_rows, int64_t *panel_cols, int64_t *count) {
    Ctx &g = resolve(ctx);
    std::lock_guard<std::mutex> lock(g.mu);
    if (!g.have_panels) return OZ2_INVALID_ARG;
    if (panel_rows) *panel_rows = g.last_panels.pr;
    if (panel_cols) *panel_cols = g.last_panels.pc;
    if (count) *count = g.last_panels.count;
    return OZ2_OK;
}

oz2_status oz2_ctx_last_gemm_launches(oz2_context *ctx, int64_t *launches) {
    Ctx &g = resolve(ctx);
    std::lock_guard<std::mutex> lock(g.mu);
    if (!g.have_panels || !launches) return OZ2_INVALID_ARG;
    *launches = g.last_gemm_launches;
    return OZ2_OK;
}

oz2_status oz2_ctx_stage_ptr(oz2_context *ctx, int stage, void **dev_ptr, int64_t *dims) {
    Ctx &g = resolve(ctx);
    std::lock_guard<std::mutex> lock(g.mu);
    if (!g.have_last || !dev_ptr || !dims) return OZ2_INVALID_ARG;
    const Layout &L = g.last;
    switch (stage) {
    case OZ2_STAGE_SHIFT_A: *dev_ptr = g.ws + L.off_ta; dims[0] = L.m; dims[1] = dims[2] = dims[3] = 0; break;
    case OZ2_STAGE_SHIFT_B: *dev_ptr = g.ws + L.off_tb; dims[0] = L.n; dims[1] = dims[2] = dims[3] = 0; break;
    case OZ2_STAGE_RES_A: *dev_ptr = g.ws + L.off_ra; dims[0] = L.N; dims[1] = L.Mp; dims[2] = L.Kp; dims[3] = L.m; break;
    case OZ2_STAGE_RES_B: *dev_ptr = g.ws + L.off_rb; dims[0] = L.N; dims[1] = L.Np; dims[2] = L.Kp; dims[3] = L.n; break;
    case OZ2_STAGE_PROD:
        if (L.prod_u8 || !g.have_last_prod) return OZ2_INVALID_ARG;                // not kept in this form: see OZ2_OPT_INT32_PRODUCTS
        *dev_ptr = g.ws + L.off_prod; dims[0] = L.N; dims[1] = L.Mp; dims[2] = L.Np; dims[3] = 0; break;
    case OZ2_STAGE_U:
        if (!L.prod_u8 || !g.have_last_prod) return OZ2_INVALID_ARG;
        *dev_ptr = g.ws + L.off_prod; dims[0] = L.N; dims[1] = L.Mp; dims[2] = L.Np; dims[3] = 0; break;
    default: return OZ2_INVALID_ARG;
    }
    return OZ2_OK;
}

oz2_status oz2_ctx_last_stage_times_ms(oz2_context *ctx, float *out4) {
    Ctx &g = resolve(ctx);
    std::lock_guard<std::mutex> lock(g.mu);
    if (!out4 || !g.ev_recorded) return OZ2_INVALID_ARG;
    OZ2_TRY(hipEventSynchronize(g.ev[4]));
    if (g.last_overlapped_panels > 0) {
        // overlapped call: shifts; what of the residues was exposed before the first GEMM; the
        // sum of the panels' GEMM launches; the rest (gaps between them, the last accumulation)
        float after_shifts = 0.f, gemm = 0.f;
        OZ2_TRY(hipEventElapsedTime(&out4[0], g.ev[0], g.ev[1]));
        OZ2_TRY(hipEventElapsedTime(&out4[1], g.ev[1], g.time_ev[0]));
        OZ2_TRY(hipEventElapsedTime(&after_shifts, g.ev[1], g.ev[4]));
        for (int64_t p = 0; p < g.last_overlapped_panels; ++p) {
            float t = 0.f;
            OZ2_TRY(hipEventElapsedTime(&t, g.time_ev[2 * p], g.time_ev[2 * p + 1]));
            gemm += t;
        }
        out4[2] = gemm;
        out4[3] = after_shifts - out4[1] - gemm;
        return OZ2_OK;
    }
    for (int i = 0; i < 4; ++i) OZ2_TRY(hipEventElapsedTime(&out4[i], g.ev[i], g.ev[i + 1]));
    return OZ2_OK;
}

// ------------------------------------------------------------------ the same on the default context
oz2_status oz2_dgemm(int64_t m, int64_t n, int64_t k, double alpha, const double *A, int64_t lda,
                     const double *B, int64_t ldb, double beta, double *C, int64_t ldc,
                     int num_moduli, hipStream_t stream) {
    return oz2_ctx_dgemm(nullptr, OZ2_OP_N, OZ2_OP_N, 0, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, num_moduli, stream);
}

oz2_status oz2_sgemm(int64_t m, int64_t n, int64_t k, float alpha, const float *A, int64_t lda,
                     const float *B, int64_t ldb, float beta, float *C, int64_t ldc,
                     int num_moduli, hipStream_t stream) {
    return oz2_ctx_sgemm(nullptr, OZ2_OP_N, OZ2_OP_N, 0, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, num_moduli, stream);
}

oz2_status oz2_dgemm_accurate(int64_t m, int64_t n, int64_t k, double alpha, const double *A,
                              int64_t lda, const double *B, int64_t ldb, double beta, double *C,
                              int64_t ldc, int num_moduli, hipStream_t stream) {
    return oz2_ctx_dgemm(nullptr, OZ2_OP_N, OZ2_OP_N, 1, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, num_moduli, stream);
}

oz2_status oz2_sgemm_accurate(int64_t m, int64_t n, int64_t k, float alpha, const float *A,
                              int64_t lda, const float *B, int64_t ldb, float beta, float *C,
                              int64_t ldc, int num_moduli, hipStream_t stream) {
    return oz2_ctx_sgemm(nullptr, OZ2_OP_N, OZ2_OP_N, 1, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, num_moduli, stream);
}

oz2_status oz2_dgemm_op(oz2_op opA, oz2_op opB, int accurate, int64_t m, int64_t n, int64_t k,
                        double alpha, const double *A, int64_t lda, const double *B, int64_t ldb,
                        double beta, double *C, int64_t ldc, int num_moduli, hipStream_t stream) {
    return oz2_ctx_dgemm(nullptr, opA, opB, accurate, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, num_moduli, stream);
}

oz2_status oz2_sgemm_op(oz2_op opA, oz2_op opB, int accurate, int64_t m, int64_t n, int64_t k,
                        float alpha, const float *A, int64_t lda, const float *B, int64_t ldb,
                        float beta, float *C, int64_t ldc, int num_moduli, hipStream_t stream) {
    return oz2_ctx_sgemm(nullptr, opA, opB, accurate, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, num_moduli, stream);
}

// Column-major callers: C^T = op(B)^T op(A)^T in row-major terms (see include/oz2.h).
oz2_status oz2_dgemm_colmajor(oz2_op opA, oz2_op opB, int accurate, int64_t m, int64_t n, int64_t k,
                              double alpha, const double *A, int64_t lda, const double *B,
                              int64_t ldb, double beta, double *C, int64_t ldc, int num_moduli,
                              hipStream_t stream) {
    return oz2_ctx_dgemm(nullptr, opB, opA, accurate, n, m, k, alpha, B, ldb, A, lda, beta, C, ldc, num_moduli, stream);
}

oz2_status oz2_sgemm_colmajor(oz2_op opA, oz2_op opB, int accurate, int64_t m, int64_t n, int64_t k,
                              float alpha, const float *A, int64_t lda, const float *B, int64_t ldb,
                              float beta, float *C, int64_t ldc, int num_moduli, hipStream_t stream) {
    return oz2_ctx_sgemm(nullptr, opB, opA, accurate, n, m, k, alpha, B, ldb, A, lda, beta, C, ldc, num_moduli, stream);
}

oz2_status oz2_prepare_d(int side, oz2_op op, int64_t rows, int64_t k, const double *X, int64_t ld,
                         int num_moduli, hipStream_t stream, oz2_operand **out) {
    return prepare_impl<double>(side, op, rows, k, X, ld, num_moduli, stream, out);
}

oz2_status oz2_prepare_s(int side, oz2_op op, int64_t rows, int64_t k, const float *X, int64_t ld,
                         int num_moduli, hipStream_t stream, oz2_operand **out) {
    return prepare_impl<float>(side, op, rows, k, X, ld, num_moduli, stream, out);
}

void oz2_operand_free(oz2_operand *operand) {
    if (!operand) return;
    (void)hipFree(operand->mem);
    delete operand;
}

size_t oz2_operand_bytes(const oz2_operand *operand) { return operand ? operand->bytes : 0; }

oz2_status oz2_dgemm_prepared(const oz2_operand *left, const oz2_operand *right, double alpha,
                              double beta, double *C, int64_t ldc, hipStream_t stream) {
    return oz2_ctx_dgemm_prepared(nullptr, left, right, alpha, beta, C, ldc, stream);
}

oz2_status oz2_sgemm_prepared(const oz2_operand *left, const oz2_operand *right, float alpha,
                              float beta, float *C, int64_t ldc, hipStream_t stream) {
    return oz2_ctx_sgemm_prepared(nullptr, left, right, alpha, beta, C, ldc, stream);
}

size_t oz2_workspace_bytes(int64_t m, int64_t n, int64_t k, int num_moduli, int is_double) {
    (void)is_double;                                          // the workspace holds no input-typed data
    return oz2_ctx_workspace_bytes(nullptr, m, n, k, num_moduli);
}

size_t oz2_workspace_min_bytes(int64_t m, int64_t n, int64_t k, int num_moduli, int is_double) {
    (void)is_double;
    return oz2_ctx_workspace_min_bytes(nullptr, m, n, k, num_moduli);
}

void oz2_set_workspace_limit(size_t bytes) { (void)oz2_ctx_set_workspace_limit(nullptr, bytes); }

oz2_status oz2_plan_panels(int64_t m, int64_t n, int64_t k, int num_moduli, size_t workspace_bytes,
                           int64_t *panel_rows, int64_t *panel_cols, int64_t *count) {
    return oz2_ctx_plan_panels(nullptr, m, n, k, num_moduli, workspace_bytes, panel_rows, panel_cols, count);
}

oz2_status oz2_last_panels(int64_t *panel_rows, int64_t *panel_cols, int64_t *count) {
    return oz2_ctx_last_panels(nullptr, panel_rows, panel_cols, count);
}
oz2_status oz2_last_gemm_launches(int64_t *launches) { return oz2_ctx_last_gemm_launches(nullptr, launches); }

oz2_status oz2_set_workspace(void *dev_ptr, size_t bytes) { return oz2_ctx_set_workspace(nullptr, dev_ptr, bytes); }

void oz2_release(void) { (void)oz2_ctx_release(nullptr); }

oz2_status oz2_stage_ptr(int stage, void **dev_ptr, int64_t *dims) { return oz2_ctx_stage_ptr(nullptr, stage, dev_ptr, dims); }

void oz2_set_int32_products(int on) { (void)oz2_ctx_set_option(nullptr, OZ2_OPT_INT32_PRODUCTS, on); }
void oz2_set_overlap(int on) { (void)oz2_ctx_set_option(nullptr, OZ2_OPT_OVERLAP, on); }
void oz2_set_small_conversion(int on) { (void)oz2_ctx_set_option(nullptr, OZ2_OPT_SMALL_CONVERSION, on); }
void oz2_set_profiling(int on) { (void)oz2_ctx_set_option(nullptr, OZ2_OPT_PROFILING, on); }

oz2_status oz2_last_stage_times_ms(float *out4) { return oz2_ctx_last_stage_times_ms(nullptr, out4); }

// ------------------------------------------------------------------ allocation-free entry point
}  // extern "C"

namespace {

// The workspace of oz2_dgemm_noalloc: a fixed array in the library's device image, one copy per
// GPU, held from the moment the image is loaded on that GPU until the process ends.
static __device__ __align__(256) unsigned char scratch[OZ2_NOALLOC_WORKSPACE_BYTES];

constexpr int kMaxNoallocDevices = 64;
struct NoallocSlot {
    void *ptr = nullptr;                   // device address of `scratch` on this GPU (hipGetSymbolAddress)
    Ctx ctx;                               // a context whose workspace is that array, for good
};
NoallocSlot noalloc_slots[kMaxNoallocDevices];
std::mutex noalloc_mu;                     // guards the set-up of the slots

}  // namespace

extern "C" {

oz2_status oz2_dgemm_noalloc(int64_t m, int64_t n, int64_t k, double alpha, const double *A, int64_t lda,
                             const double *B, int64_t ldb, double beta, double *C, int64_t ldc,
                             int num_moduli, hipStream_t stream) {
    Action action;
    if (oz2_status st = check_gemm_args(OZ2_OP_N, OZ2_OP_N, m, n, k, A, lda, B, ldb, C, ldc, num_moduli, &action))
        return st;
    if (action == Action::kProduct) {                      // sizes beyond the fixed array are refused
        const Layout L = make_layout(m, n, k, num_moduli, true);
        if (L.off_prod + L.prod_whole > (size_t)OZ2_NOALLOC_WORKSPACE_BYTES) return OZ2_WORKSPACE;
    }
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return OZ2_HIP_ERROR;
    if (dev < 0 || dev >= kMaxNoallocDevices) return OZ2_UNSUPPORTED;
    NoallocSlot &slot = noalloc_slots[dev];
    {
        std::lock_guard<std::mutex> lock(noalloc_mu);
        if (!slot.ptr) {
            // Once per device, with that device current: each GPU holds its own copy of the array
            // at its own address.  In host code the array's name is not that address.
            void *p = nullptr;
            if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
                (void)hipGetLastError();
                return OZ2_HIP_ERROR;
            }
            slot.ptr = p;
            slot.ctx.ws = static_cast<char *>(p);          // a caller-owned workspace in the context's terms:
            slot.ctx.ws_bytes = OZ2_NOALLOC_WORKSPACE_BYTES;   // never grown, never freed
            slot.ctx.ws_owned = false;
        }
    }
    // Profiling and the overlapped form stay off in this context (they would create events and a
    // stream); what is left of the call path only launches kernels on `stream`.
    return gemm_impl<double>(slot.ctx, OZ2_OP_N, OZ2_OP_N, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, num_moduli,
                             stream, false);
}

// ------------------------------------------------------------------ stateless entry points
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

int oz2_residue_rounds(int num_moduli, int accurate) {
    if (num_moduli < OZ2_MIN_MODULI || num_moduli > OZ2_MAX_MODULI) return 0;
    return residue_rounds(table(num_moduli, true), accurate != 0);
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

const char *oz2_status_string(oz2_status s) {
    switch (s) {
    case OZ2_OK: return "ok";
    case OZ2_INVALID_ARG: return "invalid argument";
    case OZ2_UNSUPPORTED: return "unsupported number of moduli, or k > 2^20";
    case OZ2_WORKSPACE: return "workspace too small or allocation failed";
    case OZ2_HIP_ERROR: return "HIP runtime error";
    }
    return "unknown status";
}

}  // extern "C"
