"""Pins for the oracle's accurate mode (Section 4.2, second half): the 7-bit
matrices, the bound chain that justifies the scale vectors, Eq. 3 with exact
integers, and the accuracy statements of Section 5.1.  CPU only."""
import math
import os
from fractions import Fraction

import mpmath
import numpy as np
import pytest

import synth_inputs as S
from oracle import constants as K
from test_oracle_accuracy import anchors, dd_error
from test_oracle_stages import exact_scaled_matrices, floor_log2

mpmath.mp.prec = 200


def test_Paccu_constant():
    for n in range(2, 21):
        c = K.constants(n)
        assert abs(c.Paccu - (0.5 * math.log2(c.P - 1) - 0.5)) <= 2.0 ** -17
        assert c.Paccu == np.float32(c.Paccu)
        assert abs((c.Paccu - c.Pfast) - 1.0) <= 2.0 ** -16
        assert 2 * c.Paccu + 1 <= math.log2(c.P) + 2.0 ** -15     # 2 * 2^(2P') <= P - 1 up to rounding


def test_prescale_is_the_ceiling_of_the_definition(oracle):
    A = S.matrix(9, 40, 2.0, seed=3)
    A[4, :] = 0.0
    A[5, :] *= 2.0 ** -1040
    for axis in (0, 1):
        e, bar = oracle.accu_prescale(A, axis)
        X = A if axis == 0 else A.T
        for v in range(X.shape[0]):
            fr = [abs(Fraction(float(x))) for x in X[v]]
            if max(fr) == 0:
                assert e[v] == 0 and not bar[v].any()
                continue
            assert e[v] == floor_log2(max(fr))
            want = [math.ceil(x * Fraction(2) ** int(5 - e[v])) for x in fr]
            assert bar[v].tolist() == want
            assert 32 <= max(want) <= 64                               # fits 7 bits (Section 4.2)


def test_bound_chain_of_accurate_mode(oracle):
    """sum_h |a_ih||b_hj| <= (mu'_i nu'_j)^-1 (Abar Bbar)_ij, exactly."""
    A, B = S.gemm_inputs(7, 6, 50, 1.5, seed=4)
    r = oracle.accu_shifts(A, B, 40.0)
    Cbar = r["Abar"].astype(np.int64) @ r["Bbar"].astype(np.int64).T
    assert np.array_equal(Cbar.max(axis=1), r["rmax"]) and np.array_equal(Cbar.max(axis=0), r["cmax"])
    for i in range(7):
        for j in range(6):
            lhs = sum(abs(Fraction(float(A[i, h])) * Fraction(float(B[h, j]))) for h in range(50))
            rhs = Fraction(int(Cbar[i, j])) / (Fraction(2) ** int(5 - r["eA"][i]) * Fraction(2) ** int(5 - r["eB"][j]))
            assert lhs <= rhs


@pytest.mark.parametrize("n_mod", [2, 7, 14, 20])
def test_accurate_shifts_against_exact_formula(oracle, n_mod):
    c = K.constants(n_mod)
    A, B = S.gemm_inputs(10, 8, 64, 1.0, seed=6)
    r = oracle.accu_shifts(A, B, c.Paccu)
    for t, e, cm in ((r["tA"], r["eA"], r["rmax"]), (r["tB"], r["eB"], r["cmax"])):
        for v in range(t.size):
            arg = mpmath.mpf(c.Paccu) - mpmath.mpf("0.51") * mpmath.log(int(cm[v]), 2)
            f = int(mpmath.floor(arg))
            assert min(arg - f, f + 1 - arg) > 1e-9
            assert t[v] == (5 - e[v]) + f


@pytest.mark.parametrize("n_mod", list(range(2, 21)))
def test_uniqueness_condition_eq3_accurate(oracle, n_mod):
    c = K.constants(n_mod)
    for phi, seed in ((0.5, 1), (2.0, 2), (4.0, 3)):
        A, B = S.gemm_inputs(6, 5, 64, phi, seed)
        A[0, :] = np.abs(A[0, :]).max()
        B[:, 0] = np.abs(B[:, 0]).max()
        prep = oracle.prepare(A, B, n_mod, accurate=True)
        Ap, Bp = exact_scaled_matrices(A, B, prep["tA"], prep["tB"])
        for i in range(6):
            for j in range(5):
                assert 2 * sum(abs(Ap[i][h]) * abs(Bp[h][j]) for h in range(64)) < c.P


def test_blocked_bound_for_long_contractions(oracle):
    """k beyond one INT32 product (Section 4.3, last sentence; here with a block of 16 instead of
    2^17 so that exact integers stay cheap): the row bound is sum_r max_j (Cbar_r)_ij, computed
    here from the definition with Python integers; it is at least the true row maximum of the
    whole Cbar, equals the paper's formula when one block holds all of k, and the bound chain of
    Section 4.2 still holds entry by entry."""
    A, B = S.gemm_inputs(6, 5, 70, 1.5, seed=12)
    r = oracle.accu_shifts(A, B, 40.0, kblock=16)
    Ab = [[int(v) for v in row] for row in r["Abar"]]
    Bb = [[int(v) for v in row] for row in r["Bbar"]]          # vector-major: Bb[j][h]
    blocks = [(k0, min(k0 + 16, 70)) for k0 in range(0, 70, 16)]
    cb = lambda i, j, k0, k1: sum(Ab[i][h] * Bb[j][h] for h in range(k0, k1))
    rmax = [sum(max(cb(i, j, *b) for j in range(5)) for b in blocks) for i in range(6)]
    cmax = [sum(max(cb(i, j, *b) for i in range(6)) for b in blocks) for j in range(5)]
    assert r["rmax"].tolist() == rmax and r["cmax"].tolist() == cmax
    whole = oracle.accu_shifts(A, B, 40.0, kblock=70)
    assert whole["rmax"].tolist() == [max(cb(i, j, 0, 70) for j in range(5)) for i in range(6)]
    assert np.all(r["rmax"] >= whole["rmax"]) and np.all(r["cmax"] >= whole["cmax"])
    assert np.any(r["rmax"] > whole["rmax"])                      # the bound is really coarser here
    assert np.all(r["tA"] <= whole["tA"]) and np.all(r["tB"] <= whole["tB"])
    for i in range(6):
        for j in range(5):
            lhs = sum(abs(Fraction(float(A[i, h])) * Fraction(float(B[h, j]))) for h in range(70))
            scale = Fraction(2) ** int(5 - r["eA"][i]) * Fraction(2) ** int(5 - r["eB"][j])
            assert lhs <= Fraction(rmax[i]) / scale and lhs <= Fraction(cmax[j]) / scale


@pytest.mark.parametrize("n_mod", [2, 9, 14, 20])
def test_uniqueness_condition_eq3_accurate_blocked(oracle, n_mod):
    """Eq. 3 with exact integers when the contraction spans several blocks, including the case in
    which every bound of the chain is attained (constant parallel vectors)."""
    c = K.constants(n_mod)
    for phi, seed in ((0.5, 1), (4.0, 3)):
        A, B = S.gemm_inputs(6, 5, 100, phi, seed)
        A[0, :] = np.abs(A[0, :]).max()
        B[:, 0] = np.abs(B[:, 0]).max()
        prep = oracle.prepare(A, B, n_mod, accurate=True, kblock=32)
        Ap, Bp = exact_scaled_matrices(A, B, prep["tA"], prep["tB"])
        for i in range(6):
            for j in range(5):
                assert 2 * sum(abs(Ap[i][h]) * abs(Bp[h][j]) for h in range(100)) < c.P


def test_blocked_accurate_mode_end_to_end(oracle):
    """The whole of Algorithm 1 with the blocked bound: the result is as accurate as with the
    unblocked bound up to the (at most 0.51 log2(blocks)-bit) smaller shifts."""
    A, B = S.gemm_inputs(24, 20, 512, 1.0, seed=5)
    rows = np.arange(24)
    err = {}
    for kb in (512, 64):
        prep = oracle.prepare(A, B, 13, accurate=True, kblock=kb)
        err[kb] = dd_error(oracle, oracle.finish_rows(prep, rows)["C"], A, B)
    assert err[512] <= 2 * err[64] and err[64] < 64 * err[512]


def test_accurate_special_cases(oracle):
    A, B = S.gemm_inputs(6, 7, 30, 0.5, seed=9)
    A[2, :] = 0.0
    B[:, 3] = 0.0
    r = oracle.gemm(A, B, 14, accurate=True)
    assert r["tA"][2] == 0 and r["tB"][3] == 0
    assert np.all(r["C"][2] == 0) and np.all(r["C"][:, 3] == 0)
    # B = 0: every row maximum of Cbar is 0 and is taken as 1; the product is exactly 0
    r = oracle.gemm(A, np.zeros_like(B), 14, accurate=True)
    assert np.all(r["C"] == 0)
    # power-of-two scaling of rows / columns only moves the shifts
    sa = np.array([3, -40, 0, 7, 1, -2]); sb = np.array([0, 5, -9, 0, 2, 2, -1])
    r0 = oracle.gemm(A, B, 15, accurate=True)
    r1 = oracle.gemm(np.ldexp(A, sa[:, None]), np.ldexp(B, sb[None, :]), 15, accurate=True)
    assert np.array_equal(r1["tA"], r0["tA"] - sa) and np.array_equal(r1["tB"], r0["tB"] - sb)
    assert np.array_equal(r1["Ares"], r0["Ares"]) and np.array_equal(r1["Bres"], r0["Bres"])


def test_accurate_mode_is_at_least_as_accurate_as_fast_mode(oracle):
    """Section 4.2: the direct product bounds sum |a||b| more tightly than Cauchy-Schwarz,
    so the shifts are never smaller... measured: the error is smaller at every N below the floor."""
    for phi in (0.5, 2.0, 4.0):
        A, B = S.gemm_inputs(64, 64, 512, phi, seed=2)
        pf = oracle.prepare(A, B, 13); pa = oracle.prepare(A, B, 13, accurate=True)
        assert np.all(pa["tA"][:, None] + pa["tB"][None, :] >= pf["tA"][:, None] + pf["tB"][None, :])
        for N in (10, 12, 14):
            ef = dd_error(oracle, oracle.gemm(A, B, N)["C"], A, B)
            ea = dd_error(oracle, oracle.gemm(A, B, N, accurate=True)["C"], A, B)
            assert ea < ef


def test_accurate_dgemm_and_sgemm_anchors(oracle):
    a = anchors()
    A, B = S.gemm_inputs(96, 96, 1024, 0.5, seed=0)
    native = dd_error(oracle, A @ B, A, B)
    e14 = dd_error(oracle, oracle.gemm(A, B, a["accu_dgemm_comparable"][0], accurate=True)["C"], A, B)
    e15 = dd_error(oracle, oracle.gemm(A, B, a["accu_dgemm_better"][0], accurate=True)["C"], A, B)
    f14 = dd_error(oracle, oracle.gemm(A, B, 14)["C"], A, B)
    assert e14 < 4 * native and e14 < f14          # comparable to DGEMM, better than fast-14
    assert e15 < native
    for phi in (0.5, 1.5):
        A, B = S.gemm_inputs(64, 64, 1024, phi, seed=3, dtype=np.float32)
        A64, B64 = A.astype(np.float64), B.astype(np.float64)
        native = dd_error(oracle, (A @ B).astype(np.float64), A64, B64)
        errs = {n: dd_error(oracle, oracle.gemm(A, B, n, is_double=False, accurate=True)["C"]
                            .astype(np.float64), A64, B64) for n in a["accu_sgemm_level"]}
        assert errs[7] < 2 * native and errs[8] < native and errs[6] < 40 * native
