// Host-side planning of a product call: argument checks, the workspace layout, how C is cut
// into panels when the workspace is bounded, and the rules that pick a form of the call.
// Plain C++ with no dependency on the HIP runtime, so that it can be built and exercised on the
// CPU (also under sanitizers); the entry points in oz2_api.hip apply it unchanged.
#pragma once
#include <algorithm>
#include <cstddef>
#include <cstdint>

#include "../../include/oz2.h"

namespace oz2 {

// Tile granularity the INT8 GEMM assumes for its padded operands.
constexpr int64_t kPadMN = 256;   // rows of the A slices, rows of the B^T slices
constexpr int64_t kPadK = 128;    // contraction length
constexpr int kBlockK = 64;       // K block of the residue-slice layout [Kp/64][rows][64]
// K ranges of a blocked contraction (Section 4.3, last sentence): at most this many of OZ2_MAX_K.
constexpr int kMaxKRanges = OZ2_MAX_K_BLOCKED / OZ2_MAX_K;

inline int64_t round_up(int64_t x, int64_t to) { return (x + to - 1) / to * to; }
inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

// Scratch of the column kernels: per column a 64-bit maximum and a 64-bit sum of squares.
inline size_t column_scratch_bytes(int64_t cols) { return (size_t)cols * 16; }
// Scratch of accurate mode: per row of A and column of B the bits of max |.| (8 bytes), the
// pre-shift (4) and one maximum of Cbar per K range (4 each).
inline size_t accurate_scratch_bytes(int64_t m, int64_t n) { return (size_t)(m + n) * (12 + 4 * kMaxKRanges); }

// Shapes whose conversion (Algorithm 1 lines 1-5) runs as two fused launches: both operands
// within 2 x 2048^2 elements (they and their slices then sit in the caches) and columns short
// enough for one workgroup per strip.
inline bool small_conversion_applies(int64_t m, int64_t n, int64_t k) {
    return k <= 4096 && m <= 8192 && n <= 8192 && (m + n) * k <= (int64_t)2 * 2048 * 2048;
}

inline bool supported(int64_t k, int N) {
    return N >= OZ2_MIN_MODULI && N <= OZ2_MAX_MODULI && k <= OZ2_MAX_K_BLOCKED;
}

// What a product call has to do once its arguments have passed the checks.
enum class Action { kNothing, kScaleC, kProduct };

// The argument checks of the product entry points, in the order their documentation states:
// sizes and ops, then the supported range, then empty products, then pointers and leading
// dimensions.  op(A) is m x k and op(B) is k x n (row-major storage).
inline oz2_status check_gemm_args(int opA, int opB, int64_t m, int64_t n, int64_t k, const void *A, int64_t lda,
                                  const void *B, int64_t ldb, const void *C, int64_t ldc, int N, Action *action) {
    *action = Action::kNothing;
    if (m < 0 || n < 0 || k < 0 || (opA != OZ2_OP_N && opA != OZ2_OP_T) || (opB != OZ2_OP_N && opB != OZ2_OP_T))
        return OZ2_INVALID_ARG;
    if (!supported(k, N)) return OZ2_UNSUPPORTED;
    if (m == 0 || n == 0) return OZ2_OK;
    if (!C || ldc < n) return OZ2_INVALID_ARG;
    if (k == 0) { *action = Action::kScaleC; return OZ2_OK; }
    const bool a_kc = opA == OZ2_OP_N, b_kc = opB == OZ2_OP_T;   // is k the contiguous index?
    if (!A || !B || lda < (a_kc ? k : m) || ldb < (b_kc ? k : n)) return OZ2_INVALID_ARG;
    *action = Action::kProduct;
    return OZ2_OK;
}

// Workspace: [scratch | tA | tB | residues of A | residues of B | products].  A product of
// prepared operands uses the product part only (its shifts and residues live in the operands).
struct Layout {
    int64_t m, n, k, Mp, Np, Kp;
    int N;
    bool prod_u8;
    size_t off_bt, off_ta, off_tb, off_ra, off_rb, off_prod;
    size_t prod_whole, prod_min;           // product part: all of C at once / one 256 x 256 panel
};

// Bytes of product workspace per entry of C: N planes of uint8, or of int32 (diagnostic form).
inline size_t bytes_per_entry(int N, bool prod_u8) { return (size_t)N * (prod_u8 ? 1 : 4); }

inline Layout make_layout(int64_t m, int64_t n, int64_t k, int N, bool prod_u8, bool with_operands = true) {
    Layout L{};
    L.m = m; L.n = n; L.k = k; L.N = N; L.prod_u8 = prod_u8;
    L.Mp = round_up(m, kPadMN); L.Np = round_up(n, kPadMN); L.Kp = round_up(k, kPadK);
    size_t o = 0;
    if (with_operands) {
        L.off_bt = o;   o += align256(std::max(column_scratch_bytes(std::max(m, n)), accurate_scratch_bytes(m, n)));
        L.off_ta = o;   o += align256((size_t)m * 4);
        L.off_tb = o;   o += align256((size_t)n * 4);
        L.off_ra = o;   o += align256((size_t)N * L.Mp * L.Kp);
        L.off_rb = o;   o += align256((size_t)N * L.Np * L.Kp);
    }
    L.off_prod = o;
    L.prod_whole = align256((size_t)L.Mp * L.Np * bytes_per_entry(N, prod_u8));
    L.prod_min = align256((size_t)kPadMN * kPadMN * bytes_per_entry(N, prod_u8));
    return L;
}

// How C is cut: panels of (pr x pc) entries (multiples of 256; the last ones may be smaller).
struct Panels {
    int64_t pr, pc, count;
};

// Panels whose N product planes fit into `avail` bytes: all of C if possible, otherwise as
// square as the shape allows (the INT8 GEMM re-reads a row panel of the A slices once per
// column panel and vice versa).  Panel sides below the full side are 256 times a power of two
// up to 4096 and multiples of 4096 beyond: then the workgroups of a launch (tiles x moduli) fill
// the 256 compute units evenly and the GEMM's tile map stays XCD-aware (measured at 16384^3,
// N = 16: panels of 2816^2 72 ms against 67.8 ms for 2048^2 and 62.9 ms for 4096^2).
inline int64_t panel_side(int64_t w) {
    if (w >= 4096) return w / 4096 * 4096;
    int64_t s = kPadMN;
    while (2 * s <= w) s *= 2;
    return s;
}

inline bool plan_panels(const Layout &L, size_t avail, Panels *out) {
    const size_t per = bytes_per_entry(L.N, L.prod_u8);
    if (avail >= L.prod_whole) { *out = Panels{L.Mp, L.Np, 1}; return true; }
    const int64_t entries = (int64_t)(avail / per);
    if (entries < kPadMN * kPadMN) return false;
    int64_t s = kPadMN;
    while ((s + kPadMN) * (s + kPadMN) <= entries) s += kPadMN;
    s = panel_side(s);
    int64_t pr = std::min(L.Mp, s), pc = std::min(L.Np, s);
    auto widen = [&](int64_t other, int64_t now, int64_t limit) {   // what fits beside `other`
        const int64_t w = entries / other / kPadMN * kPadMN;
        return std::max(now, w >= limit ? limit : panel_side(w));
    };
    pc = widen(pr, pc, L.Np);
    pr = widen(pc, pr, L.Mp);
    *out = Panels{pr, pc, ((L.Mp + pr - 1) / pr) * ((L.Np + pc - 1) / pc)};
    return true;
}

// How the INT8 GEMM launches of a product (of each workspace panel, if C is worked through in
// panels) are cut: into launches of at most kLaunchPanelRows x kLaunchPanelCols entries of C per
// modulus, each writing its part of the product buffer in place.  A launch over all of a large C
// runs hundreds of rounds of 256 workgroups; over such a launch the workgroups of a round drift
// apart, the operand tiles that an XCD's L2 holds are shared by fewer of its workgroups and the
// launch fetches a quarter more through the fabric.  A launch boundary every 32 rounds or so
// keeps them together.  Measured back to back on three devices, whole launch against these
// panels: 16384^3 1.2 to 4.6 % of the call (the slower the device, the more), 10000 x 9000 x
// 20000 4.5 %, 8192 x 8192 x 65536 1 to 3 %; no difference at 8192^3 or for k <= 4096, hence the
// limit on k.  (4096 x 4096 is as good at k = 16384 and 1 % worse at 8192^3; 2048-wide panels lose
// the XCD-aware tile order and are worse except for the longest contractions.)
#ifndef OZ2_LAUNCH_PANEL_ROWS
#define OZ2_LAUNCH_PANEL_ROWS 4096
#endif
#ifndef OZ2_LAUNCH_PANEL_COLS
#define OZ2_LAUNCH_PANEL_COLS 8192
#endif
#ifndef OZ2_LAUNCH_PANEL_MIN_K
#define OZ2_LAUNCH_PANEL_MIN_K 8192
#endif
constexpr int64_t kLaunchPanelRows = OZ2_LAUNCH_PANEL_ROWS, kLaunchPanelCols = OZ2_LAUNCH_PANEL_COLS;
constexpr int64_t kLaunchPanelMinK = OZ2_LAUNCH_PANEL_MIN_K;

// rows x cols: the padded extent of what the launches cover (all of C, or one workspace panel).
inline Panels launch_panels(int64_t rows, int64_t cols, int64_t Kp) {
    Panels Q{rows, cols, 1};
    if (kLaunchPanelRows <= 0 || Kp < kLaunchPanelMinK) return Q;
    Q.pr = std::min(rows, kLaunchPanelRows); Q.pc = std::min(cols, kLaunchPanelCols);
    Q.count = ((rows + Q.pr - 1) / Q.pr) * ((cols + Q.pc - 1) / Q.pc);
    return Q;
}

// ... and along k: a launch of such a panel is kept to about kLaunchMs of matrix-core work (a
// round of 256 tiles takes about 13.4 ns per element of k), in equal K ranges that are multiples
// of 8192; the results of the ranges are folded modulo p_s in the GEMM's store phase like the
// ranges of 2^17 that exactness requires (Section 4.3).  Returns the length of a K range: Kp
// itself when one launch is short enough, never more than OZ2_MAX_K.  Measured: 8192 x 8192 x
// 65536, N = 18: 74.3 -> 72.3 ms; 4096 x 4096 x 131072, N = 16: 38.4 -> 36.6 ms.
#ifndef OZ2_LAUNCH_MS
#define OZ2_LAUNCH_MS 7.0
#endif
constexpr double kLaunchMs = OZ2_LAUNCH_MS, kRoundNsPerK = 13.4;
constexpr int64_t kLaunchKStep = 8192;

inline int64_t launch_k_len(int64_t Kp, int N, const Panels &Q) {
    const int64_t whole = std::min<int64_t>(Kp, OZ2_MAX_K);
    if (kLaunchPanelRows <= 0 || Kp < 2 * kLaunchPanelMinK) return whole;
    const int64_t tiles = (Q.pr / kPadMN) * (Q.pc / kPadMN) * N;
    const int64_t rounds = (tiles + 255) / 256;
    const double want = kLaunchMs * 1e6 / (kRoundNsPerK * (double)rounds);      // elements of k per launch
    int64_t len = std::max<int64_t>(kLaunchKStep, (int64_t)(want / kLaunchKStep + 0.5) * kLaunchKStep);
    if (2 * Kp < 3 * len) return whole;                    // less than one and a half launches: leave it whole
    const int64_t n = (Kp + len - 1) / len;
    len = round_up((Kp + n - 1) / n, kLaunchKStep);
    return std::min<int64_t>(len, OZ2_MAX_K);
}

// Side of a panel of the overlapped form: the INT8 GEMM loses nothing down to 4096 x 4096.
constexpr int64_t kOverlapPanel = 4096;

// The overlapped form (conversion of later panels beside the GEMMs of earlier ones) needs a long
// contraction and enough panels to hide something behind: panels of at most 4096 x 4096, at
// least four of them, k >= 8192 and k x panels >= 9 x 8192 (measured: with less, the conversion
// that precedes the first GEMM, or what the shorter GEMM launches lose, outweighs what is hidden).
inline bool overlap_applies(int64_t Kp, int64_t panels) {
    return panels >= 4 && panels <= 4096 && Kp >= 8192 && Kp * panels >= (int64_t)9 * 8192;
}

// Panels of the overlapped form for a layout: P capped at kOverlapPanel per side.
inline Panels overlap_panels(const Layout &L, Panels P) {
    P.pr = std::min(P.pr, kOverlapPanel); P.pc = std::min(P.pc, kOverlapPanel);
    P.count = ((L.Mp + P.pr - 1) / P.pr) * ((L.Np + P.pc - 1) / P.pc);
    return P;
}

}  // namespace oz2
