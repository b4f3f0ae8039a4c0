"""Pins for the oracle's stages (oracle/oz2_oracle.c) against exact arithmetic
with Python integers and Fractions, closed forms and library routines (CPU only).

Everything "expected" here is derived from the definitions in Sections 3 and 4
of the paper with unbounded integers; nothing is taken from the oracle itself.
"""
import math
from fractions import Fraction

import mpmath
import numpy as np
import pytest

import synth_inputs as S
from oracle import constants as K

mpmath.mp.prec = 200


# --------------------------------------------------------------------------- exact helpers
def floor_log2(x: Fraction) -> int:
    assert x > 0
    e = x.numerator.bit_length() - x.denominator.bit_length()
    while Fraction(2) ** e > x:
        e -= 1
    while Fraction(2) ** (e + 1) <= x:
        e += 1
    return e


def exact_shift(vec, Pfast):
    """Fast-mode shift of Section 4.2 for one vector, in exact/high precision.
    Returns (t, distance of the floor argument from the nearest integer)."""
    fr = [abs(Fraction(float(v))) for v in vec]
    mx = max(fr)
    if mx == 0:
        return 0, 1.0
    e = floor_log2(mx)
    T = 0
    for a in fr:
        T += math.ceil(a * Fraction(2) ** (15 - e)) ** 2
    S = mpmath.mpf(T) / mpmath.mpf(2) ** 30
    arg = mpmath.mpf(Pfast) - max(mpmath.mpf(1), mpmath.mpf("0.51") * mpmath.log(S, 2))
    f = int(mpmath.floor(arg))
    return f - e, float(min(arg - f, f + 1 - arg))


def trunc_scaled(x: float, t: int) -> int:
    return int(Fraction(float(x)) * Fraction(2) ** int(t))      # int() truncates toward zero


def rmod(x: int, p: int) -> int:
    """rmod(x,p) = x - p*round(x/p) of Section 3; the tie of p=256 goes to -128."""
    u = x % p
    return u if 2 * u < p else u - p


def exact_scaled_matrices(A, B, tA, tB):
    Ap = [[trunc_scaled(A[i, h], tA[i]) for h in range(A.shape[1])] for i in range(A.shape[0])]
    Bp = [[trunc_scaled(B[h, j], tB[j]) for j in range(B.shape[1])] for h in range(B.shape[0])]
    return Ap, Bp


def exact_product(Ap, Bp):
    m, k, n = len(Ap), len(Bp), len(Bp[0])
    return [[sum(Ap[i][h] * Bp[h][j] for h in range(k)) for j in range(n)] for i in range(m)]


# --------------------------------------------------------------------------- line 1: shifts
@pytest.mark.parametrize("n_mod", [2, 7, 14, 20])
@pytest.mark.parametrize("phi", [0.5, 2.0])
def test_shifts_against_exact_formula(oracle, n_mod, phi):
    c = K.constants(n_mod)
    A, B = S.gemm_inputs(12, 10, 40, phi, seed=5)
    tA, eA, TA = oracle.shifts(A, 0, c.Pfast)
    tB, eB, TB = oracle.shifts(B, 1, c.Pfast)
    for i in range(A.shape[0]):
        t, margin = exact_shift(A[i, :], c.Pfast)
        assert margin > 1e-9
        assert tA[i] == t
        assert eA[i] == floor_log2(max(abs(Fraction(float(v))) for v in A[i, :]))
    for j in range(B.shape[1]):
        t, margin = exact_shift(B[:, j], c.Pfast)
        assert margin > 1e-9
        assert tB[j] == t


def test_sum_of_squares_is_a_tight_upper_bound(oracle):
    """S >= sum of squares of the normalised vector (the round-up requirement of
    Section 4.2), and overshoots by at most sum(2^-14 |x| + 2^-30)."""
    A = S.matrix(16, 300, 1.0, seed=9)
    _, e, T = oracle.shifts(A, 0, 50.0)
    for i in range(A.shape[0]):
        norm = [abs(Fraction(float(v))) * Fraction(2) ** int(-e[i]) for v in A[i, :]]
        true = sum(x * x for x in norm)
        S_or = Fraction(float(T[i])) / 2 ** 30
        assert Fraction(float(T[i])).denominator == 1
        assert 1 <= max(norm) < 2
        assert true <= S_or <= true + sum(norm) / 2 ** 14 + Fraction(300, 2 ** 30)


@pytest.mark.parametrize("n_mod", list(range(2, 21)))
def test_uniqueness_condition_eq3(oracle, n_mod):
    """Eq. 3: 2 * sum_h |a'_ih||b'_hj| < P for every (i, j), with exact integers."""
    c = K.constants(n_mod)
    for phi, seed in ((0.5, 1), (2.0, 2), (4.0, 3)):
        A, B = S.gemm_inputs(6, 5, 64, phi, seed)
        A[0, :] = np.abs(A[0, :]).max()                    # worst case for Cauchy-Schwarz:
        B[:, 0] = np.abs(B[:, 0]).max()                    # parallel constant vectors
        tA, _, _ = oracle.shifts(A, 0, c.Pfast)
        tB, _, _ = oracle.shifts(B, 1, c.Pfast)
        Ap, Bp = exact_scaled_matrices(A, B, tA, tB)
        for i in range(6):
            for j in range(5):
                assert 2 * sum(abs(Ap[i][h]) * abs(Bp[h][j]) for h in range(64)) < c.P


def test_shift_special_rows(oracle):
    c = K.constants(14)
    A = S.matrix(6, 32, 0.5, seed=11)
    A[1, :] = 0.0                                          # zero row -> shift 0
    A[2, :] *= 2.0 ** -1060                                # subnormal row
    A[3, :] = 0.0
    A[3, 7] = -3.0                                         # single entry
    A[4, :] = np.ldexp(A[0, :], 37)                        # power-of-two multiple of row 0
    t, e, T = oracle.shifts(A, 0, c.Pfast)
    assert t[1] == 0 and T[1] == 0
    assert e[2] < -1022 and t[2] == exact_shift(A[2, :], c.Pfast)[0]
    assert e[3] == 1 and t[3] == exact_shift(A[3, :], c.Pfast)[0]
    assert t[4] == t[0] - 37 and T[4] == T[0]


# --------------------------------------------------------------------------- lines 2-5: residues
@pytest.mark.parametrize("n_mod", [2, 5, 13, 20])
def test_residues_against_definition(oracle, n_mod):
    c = K.constants(n_mod)
    A, B = S.gemm_inputs(9, 11, 33, 1.5, seed=21)
    A[0, 0] = 0.0
    A[1, :] *= 2.0 ** -1050
    tA, _, _ = oracle.shifts(A, 0, c.Pfast)
    tB, _, _ = oracle.shifts(B, 1, c.Pfast)
    RA = oracle.residues(A, 0, tA, c.p)
    RB = oracle.residues(B, 1, tB, c.p)
    assert RA.shape == (n_mod, 9, 33) and RB.shape == (n_mod, 11, 33)
    for s, p in enumerate(c.p):
        for i in range(9):
            for h in range(33):
                assert RA[s, i, h] == rmod(trunc_scaled(A[i, h], tA[i]), p)
        for j in range(11):
            for h in range(33):
                assert RB[s, j, h] == rmod(trunc_scaled(B[h, j], tB[j]), p)


def test_residue_ranges_and_the_128_wrap(oracle):
    """Section 4.1: residues fit INT8; only p = 256 reaches -128 (128 wrapped)."""
    c = K.constants(20)
    X = np.arange(-700.0, 700.0).reshape(1, -1)            # already integers; shift 0
    R = oracle.residues(X, 0, np.zeros(1, np.int32), c.p)
    for s, p in enumerate(c.p):
        r = R[s, 0].astype(int)
        assert np.all((X[0].astype(int) - r) % p == 0)
        if p == 256:
            assert r.min() == -128 and r.max() == 127
            assert np.all(r[X[0].astype(int) % 256 == 128] == -128)
        else:
            assert r.min() == -(p - 1) // 2 and r.max() == (p - 1) // 2


def test_truncation_is_toward_zero(oracle):
    X = np.array([[2.75, -2.75, 0.99, -0.99, 255.5, -255.5, 1e-300, -1e-300]])
    R = oracle.residues(X, 0, np.zeros(1, np.int32), [251])
    assert R[0, 0].tolist() == [2, -2, 0, 0, 4, -4, 0, 0]
    R = oracle.residues(X, 0, np.array([2], np.int32), [251])      # x * 4 first
    assert R[0, 0].tolist() == [11, -11, 3, -3, 1022 - 4 * 251, 4 * 251 - 1022, 0, 0]


def test_residues_determine_scaled_integers(oracle):
    """CRT on the residues gives back trunc(2^t a) exactly, since |a'| < P/2."""
    c = K.constants(16)
    A = S.matrix(4, 20, 2.0, seed=4)
    tA, _, _ = oracle.shifts(A, 0, c.Pfast)
    R = oracle.residues(A, 0, tA, c.p)
    for i in range(4):
        for h in range(20):
            x = sum(w * int(R[s, i, h]) for s, w in enumerate(c.w)) % c.P
            if x > c.P // 2:
                x -= c.P
            assert x == trunc_scaled(A[i, h], tA[i])


# --------------------------------------------------------------------------- line 6: int8 GEMM
def test_int8_gemm_against_int64_matmul(oracle):
    rng = np.random.default_rng(0)
    Ares = rng.integers(-128, 128, (3, 17, 200), dtype=np.int8)
    Bres = rng.integers(-128, 128, (3, 13, 200), dtype=np.int8)
    rows = np.array([16, 0, 5, 5])
    out = oracle.int8_gemm_rows(Ares, Bres, rows)
    for s in range(3):
        ref = Ares[s].astype(np.int64) @ Bres[s].astype(np.int64).T
        assert np.array_equal(out[s], ref[rows].astype(np.int32))
    ii = np.array([0, 16, 3]); jj = np.array([12, 0, 7])
    ent = oracle.int8_gemm_entries(Ares, Bres, ii, jj)
    full = oracle.int8_gemm_rows(Ares, Bres, np.arange(17))
    assert np.array_equal(ent, full[:, ii, jj])


def test_int32_wraps_only_at_k_2_pow_17_and_harmlessly(oracle):
    """Section 4.3: k = 2^17, all residues -128: the sum 2^31 wraps to -2^31 and
    mod 256 is still 0; one element fewer does not wrap."""
    k = 2 ** 17
    a = np.full((1, 1, k), -128, np.int8)
    prod = oracle.int8_gemm_rows(a, a, np.array([0]))
    assert prod[0, 0, 0] == -2 ** 31
    assert oracle.mod_reduce(prod, [256])[0, 0, 0] == 0
    prod = oracle.int8_gemm_rows(a[:, :, :-1], a[:, :, :-1], np.array([0]))
    assert prod[0, 0, 0] == 2 ** 31 - 128 * 128


def test_blocked_product_for_k_beyond_2_pow_17(oracle):
    """Section 4.3, last sentence: block matrix multiplication.  Range sums wrap like the
    INT32 engine, their integer sum is congruent to the exact product modulo every p_s."""
    rng = np.random.default_rng(3)
    k = 2 ** 17 + 640
    A = rng.integers(-128, 128, (2, 2, k), dtype=np.int8)
    B = rng.integers(-128, 128, (2, 3, k), dtype=np.int8)
    A[0, 0, :] = -128; B[0, 0, :] = -128                   # range 1 sums to 2^31 and wraps
    got = oracle.int8_gemm_rows_blocked(A, B, np.arange(2))
    exact = np.einsum("sik,sjk->sij", A.astype(np.int64), B.astype(np.int64))
    assert got[0, 0, 0] == -2 ** 31 + 640 * 128 * 128 and exact[0, 0, 0] == 2 ** 31 + 640 * 128 * 128
    got[0, 0, 0] += 2 ** 32
    assert np.array_equal(got, exact)
    for p in (256, 255, 173):
        U = oracle.mod_reduce64(oracle.int8_gemm_rows_blocked(A, B, np.arange(2)), [p, p])
        if p == 256:                                     # the wrap by 2^32 is invisible modulo 256
            assert np.array_equal(U, np.mod(exact, p))
        else:                                            # -128 residues only occur for p = 256
            assert np.array_equal(U[1], np.mod(exact[1], p))
    small = oracle.int8_gemm_rows_blocked(A[:, :, :1000], B[:, :, :1000], np.arange(2), kblock=300)
    assert np.array_equal(small, np.einsum("sik,sjk->sij", A[:, :, :1000].astype(np.int64),
                                           B[:, :, :1000].astype(np.int64)))


# --------------------------------------------------------------------------- line 7: mod
def test_mod_reduce_against_floor_definition(oracle):
    c = K.constants(20)
    rng = np.random.default_rng(1)
    x = rng.integers(-2 ** 31, 2 ** 31, (20, 5000)).astype(np.int32)
    x[:, :4] = np.array([0, -1, 2 ** 31 - 1, -2 ** 31], np.int32)
    U = oracle.mod_reduce(x, c.p)
    for s, p in enumerate(c.p):
        expect = [int(v) - p * math.floor(Fraction(int(v), p)) for v in x[s, :300]]
        assert U[s, :300].tolist() == expect
        assert np.array_equal(U[s], np.mod(x[s].astype(np.int64), p))


# --------------------------------------------------------------------------- lines 8-11: CRT fold
@pytest.mark.parametrize("n_mod", list(range(2, 21)))
def test_crt_fold_reproduces_the_exact_integer_product(oracle, n_mod):
    """C'' must equal A'B' (Step 3): exactly as integers before the FP64 fold,
    and to FP64 rounding after it."""
    c = K.constants(n_mod)
    A, B = S.gemm_inputs(8, 7, 96, 1.0, seed=100 + n_mod)
    prep = oracle.prepare(A, B, n_mod)
    fin = oracle.finish_rows(prep, np.arange(8))
    Ap, Bp = exact_scaled_matrices(A, B, prep["tA"], prep["tB"])
    exact = exact_product(Ap, Bp)
    half = c.P // 2
    for i in range(8):
        for j in range(7):
            # integer CRT from the oracle's U reproduces A'B' (Eq. 4-5)
            x = sum(w * int(fin["U"][s, i, j]) for s, w in enumerate(c.w)) % c.P
            if x > half:
                x -= c.P
            assert x == exact[i][j]
            # and the FP64 evaluation of Section 4.3 is that integer up to rounding
            err = abs(Fraction(float(fin["Cpp"][i, j])) - exact[i][j])
            assert err <= abs(exact[i][j]) * Fraction(1, 2 ** 51) + Fraction(c.P, 2 ** 66)


def test_crt_fold_sgemm_constants(oracle):
    """SGEMM emulation: s_i1 = double(w_i), s_i2 = P2 = 0; the fold then loses
    about 2^-53 * N * 255 * P absolutely, far below the FP32 target."""
    for n_mod in (2, 5, 8, 10):
        c = K.constants(n_mod, is_double=False)
        A, B = S.gemm_inputs(6, 6, 64, 0.5, seed=n_mod, dtype=np.float32)
        prep = oracle.prepare(A, B, n_mod, is_double=False)
        fin = oracle.finish_rows(prep, np.arange(6))
        Ap, Bp = exact_scaled_matrices(A.astype(np.float64), B.astype(np.float64),
                                       prep["tA"], prep["tB"])
        exact = exact_product(Ap, Bp)
        for i in range(6):
            for j in range(6):
                err = abs(Fraction(float(fin["Cpp"][i, j])) - exact[i][j])
                assert err <= Fraction(c.P * n_mod * 256, 2 ** 52)


# --------------------------------------------------------------------------- line 12 + alpha/beta
def test_unscale_and_alpha_beta(oracle):
    Cpp = np.array([[3.0, -5.0], [7.0, 1.0]])
    tA = np.array([2, -1], np.int32); tB = np.array([0, 3], np.int32)
    base = np.array([[3 / 4, -5 / 32], [14.0, 1 / 4]])
    assert np.array_equal(oracle.unscale_rows(Cpp, tA, tB), base)
    assert np.array_equal(oracle.unscale_rows(Cpp, tA, tB, alpha=-2.0), -2.0 * base)
    Cin = np.array([[1.0, 2.0], [3.0, 4.0]])
    assert np.array_equal(oracle.unscale_rows(Cpp, tA, tB, 0.5, 2.0, Cin), 0.5 * base + 2.0 * Cin)
    nanC = np.full((2, 2), np.nan)
    assert np.array_equal(oracle.unscale_rows(Cpp, tA, tB, 1.0, 0.0, nanC), base)   # beta=0: C not read
    ent = oracle.unscale_entries(Cpp.ravel(), np.array([2, 5, -1, 2], np.int32))
    assert np.array_equal(ent, base.ravel())


# --------------------------------------------------------------------------- whole pipeline: invariances
def test_power_of_two_scale_invariance(oracle):
    """Scaling rows of A / columns of B by powers of two changes only the shifts:
    residues identical, C scaled exactly."""
    A, B = S.gemm_inputs(10, 9, 50, 1.0, seed=77)
    sa = np.array([0, 3, -7, 40, -100, 1, 2, 0, -1, 5])
    sb = np.array([5, -5, 0, 0, 17, -30, 2, 2, 1])
    r0 = oracle.gemm(A, B, 15)
    r1 = oracle.gemm(np.ldexp(A, sa[:, None]), np.ldexp(B, sb[None, :]), 15)
    assert np.array_equal(r1["tA"], r0["tA"] - sa) and np.array_equal(r1["tB"], r0["tB"] - sb)
    assert np.array_equal(r1["Ares"], r0["Ares"]) and np.array_equal(r1["Bres"], r0["Bres"])
    assert np.array_equal(r1["C"], np.ldexp(np.ldexp(r0["C"], sa[:, None]), sb[None, :]))


def test_zero_rows_columns_and_matrices(oracle):
    A, B = S.gemm_inputs(5, 6, 20, 0.5, seed=8)
    A[2, :] = 0.0
    B[:, 4] = 0.0
    r = oracle.gemm(A, B, 12)
    assert np.all(r["C"][2, :] == 0.0) and np.all(r["C"][:, 4] == 0.0)
    r = oracle.gemm(np.zeros((3, 4)), np.zeros((4, 2)), 12)
    assert np.all(r["C"] == 0.0)
