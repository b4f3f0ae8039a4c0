"""Which reading of the fast-mode scale formula (Section 4.2) do the paper's own statements fix?

The printed formula  mu_i = 2^(floor(P'_fast - max(1, 0.51 log2 sum_j a_ij^2)) - floor(log2 max|a_i|))
with  P'_fast = single(log2(P - 1) - 1.5)  (Section 4.1) cannot be taken literally (Eq. 3 fails by
dozens of binary orders), so the oracle adopts a reading.  This file evaluates EVERY combination of
the three places where a reading is possible

    P'        "printed"  log2(P-1) - 1.5          | "halved"      0.5 log2(P-1) - 1.5
    sum       "raw"      sum_j a_ij^2             | "normalised"  sum_j (a_ij 2^-e_i)^2, e_i = floor(log2 max|a_i|)
    max(1,.)  kept                                | dropped

against the three things the paper states about fast mode:

    E3   the uniqueness condition, Eq. 3 (Section 3): 2 sum_h |a'_ih||b'_hj| < P -- for the inputs of
         Section 5 AND for the same inputs times a power of two (the method takes any FP input);
    A    Section 5.1, DGEMM at phi = 0.5: 14 moduli slightly less accurate than the native product, 15
         on par (evaluated through the oracle's own residue / product / fold stages);
    Z2   Section 5.1, SGEMM at phi in {0.5, 1, 1.5}: with 2 moduli fast mode gives A' = O and B' = O.

Result (asserted below, printed with `pytest -s`): exactly the readings with the halved P' and the
normalised sum satisfy E3 and A (with or without the max(1, .), which never acts on these inputs), and
NO reading satisfies Z2 together with E3 -- for a normalised sum Z2 is even impossible for k = 1024 by
a closed-form argument (test_fast_2_cannot_be_zero_with_a_normalised_sum).  The oracle's reading is the
only admissible one; the Z2 statement is not reproduced by any.

Everything here is computed independently of oracle/ (numpy and Python integers) except the stages
that follow the scale vectors in the accuracy check.  CPU only.
"""
import itertools
import math

import numpy as np
import pytest

import synth_inputs as S
from oracle import constants as K

READINGS = list(itertools.product(("printed", "halved"), ("raw", "normalised"), (True, False)))
ADOPTED = ("halved", "normalised", True)


def p_prime(P: int, which: str) -> float:
    v = math.log2(P - 1) - 1.5 if which == "printed" else 0.5 * math.log2(P - 1) - 1.5
    return float(np.float32(v))


def shifts(X: np.ndarray, axis: int, P: int, reading) -> np.ndarray:
    """Shift exponents t (mu = 2^t) of the vectors of X along `axis` under a reading."""
    which, summed, keep_max = reading
    X = np.asarray(X, np.float64)
    if axis == 1:
        X = X.T
    mx = np.abs(X).max(axis=1)
    e = np.frexp(mx)[1] - 1                                  # floor(log2 max|x|), exact
    Y = X if summed == "raw" else np.ldexp(X, -e[:, None])
    ssq = np.nextafter((Y * Y).sum(axis=1), np.inf)           # "round-up mode", to first order
    g = 0.51 * np.log2(ssq)
    if keep_max:
        g = np.maximum(1.0, g)
    return (np.floor(p_prime(P, which) - g) - e).astype(np.int64)


def scaled(X, axis, t):
    return np.trunc(np.ldexp(np.asarray(X, np.float64), t[:, None] if axis == 0 else t[None, :]))


def eq3_ratio(A, B, P, reading) -> float:
    """max_ij 2 sum_h |a'_ih||b'_hj| / P, in FP64 (ratios are never within 1e-6 of 1 here)."""
    Ap = np.abs(scaled(A, 0, shifts(A, 0, P, reading)))
    Bp = np.abs(scaled(B, 1, shifts(B, 1, P, reading)))
    return float(2.0 * (Ap @ Bp).max() / float(P))


def holds_eq3(reading) -> bool:
    """E3 on the inputs of Section 5 (FP32 and FP64, phi = 0.5 and 1.5; one row of A and one column
    of B made constant) and on power-of-two multiples of A."""
    for N, dtype in ((2, np.float32), (8, np.float32), (14, np.float64)):
        P = K.constants(N).P
        for phi in (0.5, 1.5):
            A, B = S.gemm_inputs(48, 40, 1024, phi, seed=3, dtype=dtype)
            A[0, :] = np.abs(A[0, :]).max()                  # parallel constant vectors: the case in
            B[:, 0] = np.abs(B[:, 0]).max()                  # which Cauchy-Schwarz is an equality
            for s in (0, -20, 12):
                r = eq3_ratio(np.ldexp(A.astype(np.float64), s), B.astype(np.float64), P, reading)
                assert abs(r - 1.0) > 1e-6
                if r >= 1.0:
                    return False
    return True


def zeroes_fast_2(reading) -> bool:
    """Z2 in the setting of the accuracy figure (m = n = 1024, k = 1024; 256 vectors for k = 16384)."""
    P = K.constants(2).P
    for phi in (0.5, 1.0, 1.5):
        for m, k in ((1024, 1024), (256, 16384)):
            A, B = S.gemm_inputs(m, m, k, phi, seed=0, dtype=np.float32)
            if scaled(A, 0, shifts(A, 0, P, reading)).any() or scaled(B, 1, shifts(B, 1, P, reading)).any():
                return False
    return True


def dgemm_anchor(oracle, reading) -> bool:
    """A: with the reading's scale vectors and the oracle's later stages, error(14) slightly above
    the native product's and error(15) at or below it (phi = 0.5; error relative to |A||B|)."""
    A, B = S.gemm_inputs(96, 96, 1024, 0.5, seed=0)
    rows = np.arange(96)
    hi, lo, ab = oracle.dd_rows(A, B, rows)

    def err(C):
        return float(np.max(np.abs((C - hi) - lo) / ab))

    native = err(A @ B)
    e = {}
    for N in (14, 15):
        c = K.constants(N)
        tA = shifts(A, 0, c.P, reading).astype(np.int32)
        tB = shifts(B, 1, c.P, reading).astype(np.int32)
        prep = dict(consts=c, tA=tA, tB=tB, Ares=oracle.residues(A, 0, tA, c.p),
                    Bres=oracle.residues(B, 1, tB, c.p))
        e[N] = err(oracle.finish_rows(prep, rows)["C"])
    return native < e[14] < 16 * native and e[15] <= native


def test_candidate_readings_table(oracle):
    rows = []
    for reading in READINGS:
        e3 = holds_eq3(reading)
        z2 = zeroes_fast_2(reading)
        anchor = dgemm_anchor(oracle, reading) if e3 else None      # without Eq. 3 the result is garbage
        rows.append((reading, e3, anchor, z2))
    print("\nP'       sum         max(1,.)  Eq.3   fast-14/15 anchor  fast-2 gives O")
    for (which, summed, keep_max), e3, anchor, z2 in rows:
        print(f"{which:8s} {summed:11s} {'kept' if keep_max else 'dropped':9s} {str(e3):6s} "
              f"{'n/a' if anchor is None else str(anchor):18s} {z2}")
    table = {r: (e3, anchor, z2) for r, e3, anchor, z2 in rows}
    # no reading reproduces the fast-2 statement without violating Eq. 3
    assert not any(e3 and z2 for e3, _, z2 in table.values())
    # Eq. 3 needs the halved P' and the normalised sum; those readings also meet the DGEMM anchor
    for reading, (e3, anchor, _) in table.items():
        assert e3 == (reading[0] == "halved" and reading[1] == "normalised"), reading
        if e3:
            assert anchor, reading
    assert table[ADOPTED] == (True, True, False)


def test_adopted_reading_here_is_the_oracles(oracle):
    """The numpy evaluation above and the oracle's exact-integer evaluation give the same shifts."""
    for N, dtype in ((2, np.float32), (14, np.float64)):
        c = K.constants(N)
        A, B = S.gemm_inputs(64, 48, 1024, 0.5, seed=4, dtype=dtype)
        tA, _, _ = oracle.shifts(A.astype(np.float64), 0, c.Pfast)
        tB, _, _ = oracle.shifts(B.astype(np.float64), 1, c.Pfast)
        # the oracle's sum is an upper bound that overshoots by < 2^-13 relative: a shift can differ
        # only when the floor argument is that close to an integer, which these inputs are not
        assert np.array_equal(tA, shifts(A, 0, c.P, ADOPTED))
        assert np.array_equal(tB, shifts(B, 1, c.P, ADOPTED))


@pytest.mark.parametrize("which", ["printed", "halved"])
def test_fast_2_cannot_be_zero_with_a_normalised_sum(which):
    """Closed form: a normalised vector has 1 <= max < 2, so its sum of squares is below 4k and
    f = floor(P' - 0.51 log2 S) >= floor(P' - 0.51 (2 + log2 k)).  For N = 2 (P = 256 * 255) and
    k = 1024 that is >= 0, hence the largest entry of every non-zero row scales to |a'| >= 1: A' = O
    is impossible whatever the data, and the fast-2 statement of Section 5.1 cannot come from any
    reading with a normalised sum."""
    P = 256 * 255
    assert K.constants(2).P == P
    worst = math.floor(p_prime(P, which) - max(1.0, 0.51 * (2 + math.log2(1024))))
    assert worst >= 0
    x = np.full((1, 1024), 1.9999, np.float32)               # the largest normalised sum there is
    for keep_max in (True, False):
        t = shifts(x, 0, P, (which, "normalised", keep_max))
        assert scaled(x, 0, t).all()
