"""CPU-only checks of the C-ABI library: it loads, exports every symbol that
include/oz2.h declares, its host-side constants equal the oracle's bit for bit,
its shift table reproduces the oracle's formula at every threshold, and its
argument checks reject bad calls before anything touches a GPU."""
import ctypes as C
import math
import os
import re

import numpy as np
import pytest

from oracle import constants as K

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def oz():
    import paper_2508_03984_amd as oz
    if not os.path.exists(oz.lib_path()):
        from paper_2508_03984_amd.build import build_library
        build_library()
    oz.load()
    return oz


def test_library_exports_every_declared_symbol(oz):
    header = open(os.path.join(ROOT, "include", "oz2.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(oz2_[a-z0-9_]+)\s*\(", header))
    assert {"oz2_dgemm", "oz2_sgemm", "oz2_dgemm_accurate", "oz2_sgemm_accurate", "oz2_workspace_bytes", "oz2_set_workspace", "oz2_release",
            "oz2_constants", "oz2_stage_ptr", "oz2_int8_gemm"} <= declared
    lib = C.CDLL(oz.lib_path())
    for name in declared:
        assert hasattr(lib, name), name
    from paper_2508_03984_amd import binding
    assert set(binding.EXPORTS) == declared
    for name in declared:
        assert hasattr(oz, name), f"binding lacks {name}"


@pytest.mark.parametrize("n", range(2, 21))
@pytest.mark.parametrize("is_double", [True, False])
def test_constants_equal_the_oracles(oz, n, is_double):
    """Two independent derivations (fixed-width integers in C++, Python integers)."""
    got = oz.oz2_constants(n, is_double)
    ref = K.constants(n, is_double)
    assert got["p"].tolist() == ref.p
    assert got["pinv_prime"].tolist() == ref.pinv_prime
    assert got["s1"].tolist() == ref.s1 and got["s2"].tolist() == ref.s2
    assert (got["P1"], got["P2"], got["Pinv"]) == (ref.P1, ref.P2, ref.Pinv)
    assert got["Pfast"] == ref.Pfast


@pytest.mark.parametrize("n", range(2, 21))
def test_shift_table_matches_the_formula_at_every_threshold(oz, oracle, n):
    """The kernels look f up by comparing the integer T with theta[]; the oracle
    evaluates floor(P'_fast - max(1, 0.51 log2(T 2^-30))).  f is monotone in T, so
    the two agree everywhere iff they agree on both sides of every threshold."""
    tab = oz.oz2_shift_table(n)
    c = K.constants(n)
    theta = [int(x) for x in tab["theta"]]
    assert theta == sorted(theta) and theta[-1] == 2 ** 52 and theta[0] >= 2 ** 30
    probes = [2 ** 30]
    for th in theta:
        probes += [th - 1, th, th + 1]
    probes = [T for T in probes if 2 ** 30 <= T <= 2 ** 52]
    # rows whose integer sum T is exactly a probe: one entry 1.0 (q = 2^15) plus filler
    # entries are not needed -- the oracle's formula is evaluated through its own C code
    # by building vectors with a prescribed T: q values are free integers in [0, 2^16].
    for T in probes:
        q = []
        rest = T - 2 ** 30                     # first entry fixes e = 0 and contributes 2^30
        while rest > 0:
            r = min(math.isqrt(rest), 2 ** 16 - 1)
            q.append(r)
            rest -= r * r
        x = np.array([[1.0] + [v / 2 ** 15 for v in q]])
        t, e, Tor = oracle.shifts(x, 0, c.Pfast)
        assert e[0] == 0 and int(Tor[0]) == T
        j = next(i for i, th in enumerate(theta) if T <= th)
        assert t[0] == tab["f_max"] - j, (n, T)


@pytest.mark.parametrize("n", range(2, 21))
def test_accurate_shift_table_matches_the_formula_at_every_threshold(oz, oracle, n):
    """Accurate mode: f = floor(P'_accu - 0.51 log2 c) is monotone in the integer c, so the
    kernels' table lookup equals the oracle's formula iff they agree around every threshold."""
    tab = oz.oz2_shift_table_accurate(n)
    c = K.constants(n)
    assert tab["Paccu"] == c.Paccu
    theta = [int(x) for x in tab["theta"]]
    assert theta == sorted(theta) and theta[-1] == 2 ** 32 and theta[0] >= 1
    probes = sorted({1, 2, 2 ** 29, 2 ** 32} | {v for th in theta for v in (th - 1, th, th + 1) if 1 <= v <= 2 ** 32})
    e = np.full(len(probes), 3, np.int32)
    t = oracle.accu_shift_from_max(e, np.array(probes, np.int64), c.Paccu)
    for cm, tv in zip(probes, t):
        j = next(i for i, th in enumerate(theta) if cm <= th)
        assert tv == (5 - 3) + tab["f_max"] - j, (n, cm)
    # a maximum of 0 (the other matrix is zero) is treated as 1
    assert oracle.accu_shift_from_max([3], [0], c.Paccu)[0] == 2 + tab["f_max"]


def test_argument_checks_need_no_gpu(oz):
    lib = oz.load()
    null = C.c_void_p(0)
    one = C.c_void_p(256)
    call = lambda m, n, k, N, A=one, B=one, Cc=one, lda=None, ldb=None, ldc=None: lib.oz2_dgemm(
        m, n, k, 1.0, A, k if lda is None else lda, B, n if ldb is None else ldb, 0.0, Cc,
        n if ldc is None else ldc, N, null)
    assert call(4, 4, 4, 1) == 2 and call(4, 4, 4, 21) == 2          # unsupported N
    assert call(4, 4, 2 ** 20 + 1, 14) == 2                           # k too large
    assert call(-1, 4, 4, 14) == 1
    assert call(4, 4, 4, 14, A=null) == 1 and call(4, 4, 4, 14, Cc=null) == 1
    assert call(4, 4, 4, 14, lda=3) == 1 and call(4, 4, 4, 14, ldb=3) == 1 and call(4, 4, 4, 14, ldc=3) == 1
    assert call(0, 4, 4, 14) == 0 and call(4, 0, 4, 14) == 0          # empty: no-op
    assert oz.oz2_workspace_bytes(4, 4, 4, 1) == 0
    assert oz.oz2_workspace_bytes(256, 256, 256, 14) >= 14 * (2 * 256 * 256 + 256 * 256)
    lib.oz2_set_int32_products(1)
    assert oz.oz2_workspace_bytes(256, 256, 256, 14) >= 14 * (2 * 256 * 256 + 4 * 256 * 256)
    lib.oz2_set_int32_products(0)
    assert lib.oz2_int8_gemm(one, one, one, 1, 256, 256, 2 ** 17 + 128, null) == 2
    assert lib.oz2_int8_gemm(one, one, one, 1, 100, 256, 128, null) == 1
    t = C.c_double()
    assert lib.oz2_mfma_probe(1, 0.0, C.byref(t), None, None) == 1    # no duration
    assert lib.oz2_mfma_probe(1, 60.0, C.byref(t), None, None) == 1   # longer than the limit
    assert lib.oz2_mfma_probe(1, 0.1, None, None, None) == 1
    assert "moduli" in oz.oz2_status_string(2)


def test_general_entry_points_check_their_arguments_without_a_gpu(oz):
    lib = oz.load()
    null, one = C.c_void_p(0), C.c_void_p(256)
    op = lambda opA, opB, m, n, k, lda, ldb, ldc, N=14, acc=0: lib.oz2_dgemm_op(
        opA, opB, acc, m, n, k, 1.0, one, lda, one, ldb, 0.0, one, ldc, N, null)
    assert op(2, 0, 4, 4, 4, 4, 4, 4) == 1 and op(0, 3, 4, 4, 4, 4, 4, 4) == 1
    assert op(1, 0, 4, 6, 5, 3, 6, 6) == 1                    # A^T is stored 5 x 4: lda >= 4
    assert op(0, 1, 4, 6, 5, 5, 4, 6) == 1                    # B^T is stored 6 x 5: ldb >= 5
    assert op(1, 1, 0, 6, 5, 1, 5, 6) == 0                    # empty: no-op
    assert op(1, 1, 4, 6, 2 ** 20 + 1, 4, 2 ** 20 + 1, 6, acc=1) == 2   # either mode: k <= 2^20
    # column-major form: A (m x k) needs lda >= m, A^T (k x m) lda >= k, C ldc >= m
    cm = lambda opA, opB, m, n, k, lda, ldb, ldc: lib.oz2_dgemm_colmajor(
        opA, opB, 0, m, n, k, 1.0, one, lda, one, ldb, 0.0, one, ldc, 14, null)
    assert cm(0, 0, 4, 6, 5, 3, 5, 4) == 1 and cm(1, 0, 4, 6, 5, 4, 5, 4) == 1      # lda
    assert cm(0, 0, 4, 6, 5, 4, 4, 4) == 1 and cm(0, 1, 4, 6, 5, 4, 5, 4) == 1      # ldb
    assert cm(0, 0, 4, 6, 5, 4, 5, 3) == 1 and cm(2, 0, 4, 6, 5, 4, 5, 4) == 1      # ldc, op
    assert cm(0, 0, 0, 6, 5, 1, 5, 1) == 0                                          # empty: no-op
    out = C.c_void_p(0)
    prep = lambda side, o, rows, k, ld, N=14, X=one: lib.oz2_prepare_d(side, o, rows, k, X, ld, N, null,
                                                                      C.byref(out))
    assert prep(2, 0, 4, 4, 4) == 1 and prep(0, 2, 4, 4, 4) == 1 and prep(0, 0, 0, 4, 4) == 1
    assert prep(0, 0, 4, 0, 4) == 1 and prep(0, 0, 4, 4, 4, X=null) == 1
    assert prep(0, 0, 4, 8, 7) == 1 and prep(0, 1, 4, 8, 3) == 1      # left: ld >= k, or >= rows if stored transposed
    assert prep(1, 0, 4, 8, 3) == 1 and prep(1, 1, 4, 8, 7) == 1      # right: ld >= rows, or >= k if stored transposed
    assert prep(0, 0, 4, 4, 4, N=21) == 2 and prep(0, 0, 4, 2 ** 20 + 1, 2 ** 20 + 1) == 2
    assert out.value is None                                  # written only on success
    assert lib.oz2_dgemm_prepared(null, null, 1.0, 0.0, one, 4, null) == 1
    assert lib.oz2_operand_bytes(null) == 0
    lib.oz2_operand_free(null)
    assert lib.oz2_last_panels(None, None, None) in (0, 1)


@pytest.mark.parametrize("m,n,k,N", [(700, 1100, 200, 15), (16384, 16384, 16384, 16), (8192, 300, 1000, 20),
                                     (256, 40000, 512, 2), (100000, 5000, 128, 12)])
def test_panel_plan_covers_c_within_the_workspace(oz, m, n, k, N):
    """Host logic of the bounded workspace: every plan fits, covers C, and uses whole tiles."""
    need = oz.oz2_workspace_bytes(m, n, k, N)
    least = oz.oz2_workspace_min_bytes(m, n, k, N)
    Mp, Np = -(-m // 256) * 256, -(-n // 256) * 256
    per = N
    fixed = need - Mp * Np * per
    assert fixed == least - 256 * 256 * per and fixed >= N * (Mp + Np) * k
    assert oz.oz2_plan_panels(m, n, k, N, need) == (Mp, Np, 1)
    assert oz.oz2_plan_panels(m, n, k, N, need + 12345) == (Mp, Np, 1)
    with pytest.raises(oz.OZ2Error) as e:
        oz.oz2_plan_panels(m, n, k, N, least - 1)
    assert e.value.status == 3
    rng = np.random.default_rng(m + n)
    sizes = [least, least + 1, need - 1] + [int(x) for x in rng.integers(least, need, 40)]
    last = 0
    for ws in sorted(sizes):
        pr, pc, count = oz.oz2_plan_panels(m, n, k, N, ws)
        assert pr % 256 == 0 and pc % 256 == 0 and 256 <= pr <= Mp and 256 <= pc <= Np
        assert fixed + pr * pc * per <= ws                     # fits
        assert count == -(-Mp // pr) * -(-Np // pc) and (count > 1 or ws >= need)
        assert pr * pc * 8 > min((ws - fixed) // per, Mp * Np) or pr * pc >= 4096 * 4096 // 4   # not wasteful
        for side, full in ((pr, Mp), (pc, Np)):               # full, 256 * 2^i, or a multiple of 4096
            assert side == full or side % 4096 == 0 or (side // 256) & (side // 256 - 1) == 0
        assert pr * pc >= last or pr * pc >= 4096 * 256       # more room never shrinks small panels
        last = pr * pc
    with pytest.raises(oz.OZ2Error):
        oz.oz2_plan_panels(m, n, 2 ** 20 + 1, N, need)


def test_binding_layout_helpers_on_the_host():
    """Argument marshalling that involves no device: the K-blocked slice layout and the
    detection of transposed views."""
    import torch
    from paper_2508_03984_amd import binding as b
    t = torch.arange(3 * 5 * 128, dtype=torch.int32).reshape(3, 5, 128)
    blocked = b.block_slices(t)
    assert blocked.shape == (3, 2, 5, 64)
    assert blocked[1, 1, 4, 7] == t[1, 4, 64 + 7]             # [s][k / 64][row][k % 64]
    assert torch.equal(b.unblock_slices(blocked), t)
    X = torch.zeros((6, 9))
    assert b._ld(X) == (False, 9) and b._ld(X.t()) == (True, 9)
    assert b._ld(X[:, :4]) == (False, 9) and b._ld(X[:, :4].t()) == (True, 9)
    assert b._ld(X[:1]) == (False, 9) and b._ld(X[:, :1]) == (False, 9)
    assert b._ld(X[:, :1].t()) == (True, 9)                   # 1 x 6 view of a column: stored 6 x 1, ld 9
    assert b._ld(torch.zeros((1, 1))) == (False, 1)
    with pytest.raises(ValueError):
        b._ld(X[:, ::2])                                      # neither row-major nor a transposed view
    with pytest.raises(ValueError):
        b.matmul(X, torch.zeros((8, 3)), 14)                  # inner dimensions differ


# AddressSanitizer + UBSan for host code built by the host compiler; the runtime is linked
# statically so that it comes first whatever else the environment loads into the process.
SANITIZE = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan"]
SAN_ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:verify_asan_link_order=0")


def test_host_constants_code_is_clean_under_sanitizers(tmp_path):
    """The library's only non-trivial host code (the wide-integer arithmetic behind the
    constants and the threshold tables) built with AddressSanitizer and UBSan by the host
    compiler, every table built once; the checksums equal those of a plain optimised build."""
    import subprocess
    src = os.path.join(ROOT, "paper_2508_03984_amd", "csrc")
    main = tmp_path / "main.cpp"
    main.write_text(r'''
#include <cstdio>
#include "oz2_constants.hpp"
int main() {
    for (int d = 0; d < 2; ++d)
        for (int n = oz2::kMinModuli; n <= oz2::kMaxModuli; ++n) {
            const oz2::Table &t = oz2::table(n, d != 0);
            double s = t.P1 + t.P2 + t.Pinv + t.Pfast + t.Paccu;
            unsigned long long x = (unsigned long long)t.f_max * 131 + t.levels * 17 + t.accu_f_max * 7 + t.accu_levels;
            for (int i = 0; i < t.n; ++i) { s += t.s1[i] * 1e-30 + t.s2[i] * 1e-20 + t.pinv[i]; x = x * 31 + t.p[i] + t.pinv_prime[i]; }
            for (int j = 0; j < t.levels; ++j) x = x * 33 + t.theta[j];
            for (int j = 0; j < t.accu_levels; ++j) x = x * 35 + t.accu_theta[j];
            std::printf("%d %d %.17g %llu\n", d, n, s, x);
        }
    return 0;
}
''')
    exe = tmp_path / "consts_san"
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-g"] + SANITIZE + ["-I", src, str(main),
                           os.path.join(src, "oz2_constants.cpp"), "-o", str(exe)])
    out = subprocess.run([str(exe)], env=SAN_ENV, capture_output=True, text=True)
    assert out.returncode == 0, out.stderr[-2000:]
    lines = out.stdout.strip().splitlines()
    assert len(lines) == 2 * 19
    plain = tmp_path / "consts_plain"
    subprocess.check_call(["g++", "-std=c++17", "-O2", "-I", src, str(main),
                           os.path.join(src, "oz2_constants.cpp"), "-o", str(plain)])
    assert subprocess.run([str(plain)], capture_output=True, text=True).stdout.strip().splitlines() == lines


def _one_round(x: int, p: int) -> int:
    """y = fma(-rint(x * double(1/p)), p, x) as the residue kernels evaluate it: the product is
    rounded to FP64, rint is to nearest-even, the FMA is exact here (Python integers)."""
    q = int(np.rint(np.float64(x) * (np.float64(1.0) / np.float64(p))))
    return x - q * p


def _adversarial(p: int, bits: int, rng):
    """Integers below 2^bits next to half-integer multiples of p, where a quotient estimate
    that is slightly off rounds to the wrong side."""
    top = (1 << bits) - 1
    if top // p < 4000:                                       # few enough to try every multiple
        return [c * s for j in range(top // p + 1) for c in ((2 * j + 1) * p // 2 + d for d in (-1, 0, 1, 2))
                for s in (1, -1) if c <= top]
    out = []
    for _ in range(400):
        j = int(rng.integers(top // p // 2, top // p))
        centre = (2 * j + 1) * p // 2
        out += [centre - 1, centre, centre + 1, centre + 2, -centre, -centre - 1]
    return [x for x in out if abs(x) <= top and float(x) == x]       # representable in FP64


@pytest.mark.parametrize("n", range(2, 21))
def test_residue_rounds_are_enough_for_the_largest_scaled_integer(oz, n):
    """Where the library takes ONE reduction round, that round must give the symmetric residue for
    every integer the mode can produce: |x'| < 2^(f_max+1) in fast mode, < 2^(f_max+6) in accurate
    mode (Section 4.2: mu' brings a row maximum into [32, 64), the second factor is at most
    2^floor(P'_accu)).  Checked at adversarial integers of that size for the moduli of this N."""
    rng = np.random.default_rng(n)
    fast_bits = oz.oz2_shift_table(n)["f_max"] + 1
    accu_bits = oz.oz2_shift_table_accurate(n)["f_max"] + 6
    assert accu_bits > fast_bits
    for accurate, bits in ((False, fast_bits), (True, accu_bits)):
        rounds = oz.oz2_residue_rounds(n, accurate)
        assert rounds in (1, 2)
        if rounds == 2 or bits > 52:
            continue
        for p in K.moduli(n):
            for x in _adversarial(p, bits, rng):
                y = _one_round(x, p)
                assert (y - x) % p == 0
                assert 2 * abs(y) < p or (p == 256 and abs(y) == 128), (n, accurate, p, x, y)


def test_one_round_is_not_enough_at_the_accurate_mode_bound_of_12_moduli():
    """Why accurate mode with 11 and 12 moduli takes two rounds although fast mode takes one:
    its scaled integers reach 2^52, and there a single round misses the symmetric residue."""
    rng = np.random.default_rng(0)
    misses = 0
    for p in K.moduli(12)[1:]:
        for x in _adversarial(p, 52, rng):
            misses += 2 * abs(_one_round(x, p)) > p
    assert misses > 0


def test_host_planning_is_clean_under_sanitizers_and_is_what_the_library_runs(oz, tmp_path):
    """The host logic of a product call that needs no GPU -- argument checks, workspace layout,
    the panel plan, the rules that pick a form of the call (csrc/oz2_plan.hpp) -- built by the host
    compiler with AddressSanitizer and UBSan and driven over many shapes and workspace sizes; the
    plans it prints equal the ones the library returns through the ABI for the same inputs."""
    import subprocess
    src = os.path.join(ROOT, "paper_2508_03984_amd", "csrc")
    main = tmp_path / "plan_main.cpp"
    main.write_text(r'''
#include <cstdio>
#include <cstdlib>
#include "oz2_plan.hpp"
using namespace oz2;
int main(int argc, char **argv) {
    // 1. argument checks: every combination of a few good and bad values
    const int64_t sizes[] = {-1, 0, 1, 300, (int64_t)1 << 20, ((int64_t)1 << 20) + 1};
    const int ops[] = {0, 1, 2}, mods[] = {1, 2, 14, 20, 21};
    char mem[8];
    unsigned long long h = 0;
    for (int64_t m : sizes) for (int64_t n : sizes) for (int64_t k : sizes)
        for (int oa : ops) for (int ob : ops) for (int N : mods)
            for (int nulls = 0; nulls < 8; ++nulls) for (int64_t dl : {(int64_t)-1, (int64_t)0}) {
                Action a;
                const int64_t lda = (oa == 0 ? k : m) + dl, ldb = (ob == 1 ? k : n) + dl, ldc = n + dl;
                oz2_status st = check_gemm_args(oa, ob, m, n, k, (nulls & 1) ? nullptr : mem, lda,
                                                (nulls & 2) ? nullptr : mem, ldb, (nulls & 4) ? nullptr : mem, ldc, N, &a);
                h = h * 31 + (unsigned)st * 5 + (unsigned)a;
            }
    std::printf("checks %llu\n", h);
    // 2. layouts and panel plans for the shapes and workspace sizes on the command line
    for (int i = 1; i + 5 <= argc; i += 5) {
        const int64_t m = atoll(argv[i]), n = atoll(argv[i + 1]), k = atoll(argv[i + 2]);
        const int N = atoi(argv[i + 3]);
        const size_t ws = strtoull(argv[i + 4], nullptr, 10);
        for (int u8 = 0; u8 < 2; ++u8) {
            const Layout L = make_layout(m, n, k, N, u8 != 0);
            Panels P{0, 0, 0};
            const bool ok = ws >= L.off_prod && plan_panels(L, ws - L.off_prod, &P);
            const Panels Po = ok ? overlap_panels(L, P) : P;
            // the cut of the GEMM launches of an unbounded product: whole panels that tile C exactly
            const Panels Q = launch_panels(L.Mp, L.Np, L.Kp);
            int64_t covered = 0, launches = 0;
            for (int64_t r0 = 0; r0 < L.Mp; r0 += Q.pr)
                for (int64_t c0 = 0; c0 < L.Np; c0 += Q.pc) {
                    const int64_t rows = std::min(Q.pr, L.Mp - r0), cols = std::min(Q.pc, L.Np - c0);
                    if (rows <= 0 || cols <= 0 || rows % kPadMN || cols % kPadMN || r0 % kPadMN || c0 % kPadMN) return 3;
                    covered += rows * cols; ++launches;
                }
            if (covered != L.Mp * L.Np || launches != Q.count || Q.pr > L.Mp || Q.pc > L.Np) return 4;
            if (L.Kp < kLaunchPanelMinK && Q.count != 1) return 5;
            const int64_t kl = launch_k_len(L.Kp, L.N, Q);
            if (kl <= 0 || kl > OZ2_MAX_K || kl % kPadK || (kl < L.Kp && kl % kLaunchKStep)) return 6;
            if (L.Kp <= OZ2_MAX_K && L.Kp < 2 * kLaunchPanelMinK && kl != L.Kp) return 7;
            std::printf("%lld %lld %lld %d %zu %d : %zu %zu %d %lld %lld %lld | %lld %lld %lld %d %d\n", (long long)m,
                        (long long)n, (long long)k, N, ws, u8, L.off_prod + L.prod_whole, L.off_prod + L.prod_min, (int)ok,
                        (long long)P.pr, (long long)P.pc, (long long)P.count, (long long)Po.pr, (long long)Po.pc,
                        (long long)Po.count, (int)(ok && overlap_applies(L.Kp, Po.count)), (int)small_conversion_applies(m, n, k));
        }
    }
    return 0;
}
''')
    exe = tmp_path / "plan_san"
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-g"] + SANITIZE + ["-I", src, str(main), "-o", str(exe)])
    rng = np.random.default_rng(5)
    cases = []
    for m, n, k, N in [(700, 1100, 200, 15), (16384, 16384, 16384, 16), (8192, 300, 1000, 20), (256, 40000, 512, 2),
                       (100000, 5000, 128, 12), (1, 1, 1, 2), (8192, 8192, 65536, 18), (5000, 7000, 2 ** 20, 9)]:
        need, least = oz.oz2_workspace_bytes(m, n, k, N), oz.oz2_workspace_min_bytes(m, n, k, N)
        for ws in [0, least - 1, least, need - 1, need, need * 2] + [int(x) for x in rng.integers(least, need + 1, 6)]:
            cases.append((m, n, k, N, ws))
    args = [str(v) for c in cases for v in c]
    out = subprocess.run([str(exe)] + args, env=SAN_ENV, capture_output=True, text=True)
    assert out.returncode == 0, out.stderr[-3000:]
    lines = out.stdout.strip().splitlines()
    assert lines[0].startswith("checks ") and len(lines) == 1 + 2 * len(cases)
    lib = oz.load()
    try:
        for (m, n, k, N, ws), (line_i32, line_u8) in zip(cases, zip(lines[1::2], lines[2::2])):
            for int32, line in ((True, line_i32), (False, line_u8)):
                lib.oz2_set_int32_products(int(int32))
                f = line.split(":")[1].split("|")[0].split()
                assert int(f[0]) == oz.oz2_workspace_bytes(m, n, k, N) and int(f[1]) == oz.oz2_workspace_min_bytes(m, n, k, N)
                try:
                    plan = oz.oz2_plan_panels(m, n, k, N, ws)
                    assert f[2] == "1" and tuple(int(x) for x in f[3:6]) == plan, (m, n, k, N, ws, int32)
                except oz.OZ2Error as e:
                    assert e.status == 3 and f[2] == "0"
    finally:
        lib.oz2_set_int32_products(0)


def test_header_is_c99_and_a_c_caller_links(oz, tmp_path):
    """include/oz2.h is a C header: a C99 translation unit that uses every kind of declaration in
    it compiles without warnings, links against the library and runs (host-side calls only)."""
    import subprocess
    main = tmp_path / "caller.c"
    main.write_text(r'''
#include <stdio.h>
#include "oz2.h"
int main(void) {
    int64_t pr = 0, pc = 0, cnt = 0;
    oz2_context *ctx = NULL;
    oz2_operand *none = NULL;
    double c3[3];
    int32_t p[OZ2_MAX_MODULI];
    if (oz2_create(&ctx) != OZ2_OK) return 1;
    if (oz2_ctx_set_option(ctx, OZ2_OPT_INT32_PRODUCTS, 1) != OZ2_OK) return 2;
    if (oz2_ctx_workspace_bytes(ctx, 256, 256, 256, 14) <= oz2_workspace_bytes(256, 256, 256, 14, 1)) return 3;
    if (oz2_ctx_plan_panels(ctx, 700, 1100, 200, 15, (size_t)1 << 40, &pr, &pc, &cnt) != OZ2_OK || cnt != 1) return 4;
    if (oz2_ctx_dgemm(ctx, OZ2_OP_N, OZ2_OP_T, 0, 4, 4, 4, 1.0, NULL, 4, NULL, 4, 0.0, NULL, 4, 14, NULL) != OZ2_INVALID_ARG) return 5;
    if (oz2_dgemm(4, 4, 4, 1.0, NULL, 4, NULL, 4, 0.0, NULL, 4, 99, NULL) != OZ2_UNSUPPORTED) return 6;
    if (oz2_constants(14, 1, p, NULL, NULL, NULL, c3, NULL) != OZ2_OK || p[0] != 256) return 7;
    if (oz2_operand_bytes(none) != 0 || oz2_residue_rounds(12, 1) != 2 || oz2_residue_rounds(12, 0) != 1) return 8;
    if (oz2_ctx_stage_ptr(ctx, OZ2_STAGE_U, NULL, NULL) != OZ2_INVALID_ARG) return 9;
    if (oz2_destroy(ctx) != OZ2_OK) return 10;
    printf("%s\n", oz2_status_string(OZ2_WORKSPACE));
    return 0;
}
''')
    exe = tmp_path / "caller"
    libdir = os.path.dirname(oz.lib_path())
    subprocess.check_call(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
                           str(main), "-L", libdir, "-l:liboz2.so", "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib",
                           "-Wl,--allow-shlib-undefined", "-o", str(exe)])
    out = subprocess.run([str(exe)], capture_output=True, text=True)
    assert out.returncode == 0, (out.returncode, out.stderr[-2000:])
    assert "workspace" in out.stdout
