"""End-to-end pins of the oracle: the final C against the exact rational
product and a double-double product, and the accuracy statements of
Section 5.1 (tests/golden/accuracy_anchors_section_5_1.txt).  CPU only.

The paper's accuracy figure itself is not available (only its discussion in
the text), and the text does not define the error measure: max over entries
of |c - exact| / (|A||B|)_ij is used here, for the emulation and for the
native product alike, and only orderings are compared.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

import synth_inputs as S

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "accuracy_anchors_section_5_1.txt")


def anchors():
    out = {}
    with open(GOLDEN) as f:
        for ln in f:
            if "=" in ln and not ln.startswith("#"):
                k, v = ln.split("=")
                out[k.strip()] = [int(x) for x in v.split()]
    return out


def exact_error(C, A, B):
    """max_ij |C_ij - (AB)_ij| / (|A||B|)_ij with the product in exact rationals."""
    fa = [[Fraction(float(v)) for v in row] for row in A]
    fb = [[Fraction(float(v)) for v in row] for row in B]
    worst = Fraction(0)
    for i in range(A.shape[0]):
        for j in range(B.shape[1]):
            ex = sum(fa[i][h] * fb[h][j] for h in range(A.shape[1]))
            ab = sum(abs(fa[i][h] * fb[h][j]) for h in range(A.shape[1]))
            worst = max(worst, abs(Fraction(float(C[i, j])) - ex) / ab)
    return float(worst)


def dd_error(oracle, C, A, B):
    rows = np.arange(A.shape[0])
    hi, lo, ab = oracle.dd_rows(A, B, rows)
    return float(np.max(np.abs((C - hi) - lo) / ab))


def test_error_against_exact_product_decreases_with_moduli(oracle):
    A, B = S.gemm_inputs(8, 8, 48, 0.5, seed=0)
    errs = {n: exact_error(oracle.gemm(A, B, n)["C"], A, B) for n in range(4, 21)}
    for n in range(4, 15):                       # each modulus buys ~8 bits: 2^-4 per side, squared
        assert errs[n + 1] < errs[n] / 4
    assert errs[4] < 2.0 ** -8 and errs[14] < 2.0 ** -48
    for n in range(16, 21):                      # FP64 floor: half an ulp of the result
        assert errs[n] <= 2.0 ** -53
    # truncation error model of Step 2: each factor is off by < 1 unit of its scaled grid
    native = exact_error(A @ B, A, B)
    assert errs[20] <= native


def test_double_double_reference_matches_exact(oracle):
    A, B = S.gemm_inputs(5, 4, 30, 1.0, seed=2)
    hi, lo, ab = oracle.dd_rows(A, B, np.arange(5))
    for i in range(5):
        for j in range(4):
            ex = sum(Fraction(float(A[i, h])) * Fraction(float(B[h, j])) for h in range(30))
            assert abs(Fraction(float(hi[i, j])) + Fraction(float(lo[i, j])) - ex) <= abs(ex) * Fraction(1, 2 ** 98)
            assert abs(ab[i, j] - float(sum(abs(Fraction(float(A[i, h])) * Fraction(float(B[h, j]))) for h in range(30)))) <= 1e-14 * ab[i, j]


def test_dgemm_level_anchors(oracle):
    """phi = 0.5: fast-14 slightly less accurate than native DGEMM, fast-15 at
    least on par (Section 5.1)."""
    a = anchors()
    A, B = S.gemm_inputs(96, 96, 1024, 0.5, seed=0)
    native = dd_error(oracle, A @ B, A, B)
    below = dd_error(oracle, oracle.gemm(A, B, a["dgemm_slightly_below"][0])["C"], A, B)
    par = dd_error(oracle, oracle.gemm(A, B, a["dgemm_on_par"][0])["C"], A, B)
    assert native < below < 16 * native
    assert par <= native


def test_fast_mode_limiting_accuracy_worsens_with_phi(oracle):
    errs = []
    for phi in (0.5, 2.0, 4.0):
        A, B = S.gemm_inputs(64, 64, 512, phi, seed=1)
        errs.append(dd_error(oracle, oracle.gemm(A, B, 12)["C"], A, B))
    assert errs[0] < errs[1] < errs[2]


def test_sgemm_level_anchors(oracle):
    """phi <= 1: fast-7 and fast-8 reach the accuracy level of native SGEMM."""
    a = anchors()
    for phi in (0.5, 1.0):
        A, B = S.gemm_inputs(64, 64, 1024, phi, seed=3, dtype=np.float32)
        A64, B64 = A.astype(np.float64), B.astype(np.float64)
        native = dd_error(oracle, (A @ B).astype(np.float64), A64, B64)
        for n in a["sgemm_level"]:
            r = oracle.gemm(A, B, n, is_double=False)
            assert r["C"].dtype == np.float32
            assert dd_error(oracle, r["C"].astype(np.float64), A64, B64) < 2 * native
        worse = oracle.gemm(A, B, 5, is_double=False)["C"].astype(np.float64)
        assert dd_error(oracle, worse, A64, B64) > 20 * native


def test_sgemm_rounds_once(oracle):
    """The FP32 result is the FP64 pipeline's value rounded once to FP32."""
    A, B = S.gemm_inputs(7, 9, 40, 0.5, seed=5, dtype=np.float32)
    r = oracle.gemm(A, B, 8, alpha=1.5, beta=0.0, is_double=False)
    c64 = oracle.unscale_rows(r["Cpp"], r["tA"], r["tB"], 1.5, 0.0)
    assert np.array_equal(r["C"], c64.astype(np.float32))
