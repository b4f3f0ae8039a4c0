"""Pins for oracle/constants.py: the constants of Section 4.1 against what the
paper prints and what number theory fixes (CPU only)."""
import math
import os
import random
import struct
from fractions import Fraction

import numpy as np
import pytest

from oracle import constants as K

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
ALL_N = list(range(2, 21))


def _golden_lines(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [ln.strip() for ln in f if ln.strip() and not ln.startswith("#")]


def test_moduli_match_printed_head_and_tail():
    head, tail = _golden_lines("moduli_section_4_1.txt")
    g = K.greedy_moduli()
    assert g[:4] == [int(x) for x in head.split()]
    assert g[-3:] == [int(x) for x in tail.split()]
    assert len(g) >= K.MAX_MODULI


def test_moduli_pairwise_coprime_and_int8_range():
    g = K.greedy_moduli()
    for i, a in enumerate(g):
        assert 2 <= a <= 256
        for b in g[i + 1:]:
            assert math.gcd(a, b) == 1
    # the greedy rule is maximal: no skipped value is coprime to all larger picks
    for c in range(2, 257):
        if c not in g:
            assert any(math.gcd(c, p) != 1 for p in g if p > c)


@pytest.mark.parametrize("n", ALL_N)
def test_crt_weights(n):
    c = K.constants(n)
    assert c.P == math.prod(c.p)
    for i, (pi, wi) in enumerate(zip(c.p, c.w)):
        assert wi % pi == 1
        assert 1 <= c.q[i] < pi
        for j, pj in enumerate(c.p):
            if j != i:
                assert wi % pj == 0


@pytest.mark.parametrize("n", ALL_N)
def test_crt_identity_random_integers(n):
    """Theorem 1 / Eq. 2: x = rmod(sum w_i y_i, P) for |x| < P/2."""
    c = K.constants(n)
    rnd = random.Random(n)
    half = (c.P - 1) // 2
    for x in [0, 1, -1, half, -half] + [rnd.randint(-half, half) for _ in range(200)]:
        acc = sum(wi * (x % pi) for wi, pi in zip(c.w, c.p))
        r = acc % c.P
        if r > half:
            r -= c.P
        assert r == x


def _ulp(x: float) -> Fraction:
    m, e = math.frexp(abs(x))
    return Fraction(2) ** (e - 53)


@pytest.mark.parametrize("n", ALL_N)
def test_P_double_double_and_Pinv(n):
    c = K.constants(n)
    # P1 is the double nearest to P, P2 the double nearest to P - P1
    assert abs(Fraction(c.P1) - c.P) <= _ulp(c.P1) / 2
    rest = c.P - Fraction(c.P1)
    if rest == 0:
        assert c.P2 == 0.0
    else:
        assert abs(Fraction(c.P2) - rest) <= _ulp(c.P2) / 2
    assert abs(Fraction(c.Pinv) * c.P - 1) <= Fraction(1, 2 ** 53)
    cs = K.constants(n, is_double=False)
    assert cs.P2 == 0.0 and all(v == 0.0 for v in cs.s2)
    for wi, s in zip(cs.w, cs.s1):
        assert abs(Fraction(s) - wi) <= _ulp(s) / 2


@pytest.mark.parametrize("n", ALL_N)
def test_s1_s2_split(n):
    c = K.constants(n)
    wmax = max(c.w).bit_length() - 1
    for wi, b, a1, a2 in zip(c.w, c.beta, c.s1, c.s2):
        assert b == 53 - 8 - math.ceil(math.log2(n)) + (wi.bit_length() - 1) - wmax
        hi = int(a1)
        assert Fraction(a1) == hi and 0 < hi <= wi
        # s1 keeps exactly the leading beta bits: the cut part is below one unit of them
        unit = 1 << max(wi.bit_length() - b, 0)
        assert hi % unit == 0 and wi - hi < unit
        rest = wi - hi
        if rest == 0:
            assert a2 == 0.0
        else:
            assert abs(Fraction(a2) - rest) <= _ulp(a2) / 2


@pytest.mark.parametrize("n", ALL_N)
def test_s1_accumulation_is_exact_in_fp64(n):
    """Section 4.3: no rounding error occurs in sum_i s_i1 U_i, in any order."""
    c = K.constants(n)
    rng = np.random.default_rng(n)
    cases = [[pi - 1 for pi in c.p]] + [[int(rng.integers(0, pi)) for pi in c.p] for _ in range(50)]
    for U in cases:
        exact = sum(int(s) * u for s, u in zip(c.s1, U))
        for order in (range(n), reversed(range(n)), rng.permutation(n)):
            acc = 0.0
            for i in order:
                acc = acc + c.s1[i] * float(U[i])      # plain mul + add, each rounded
            assert Fraction(acc) == exact


@pytest.mark.parametrize("n", ALL_N)
def test_Pfast_is_single_and_leaves_room_for_eq3(n):
    c = K.constants(n)
    assert struct.unpack("<f", struct.pack("<f", c.Pfast))[0] == c.Pfast
    assert abs(c.Pfast - (0.5 * math.log2(c.P - 1) - 1.5)) <= 2.0 ** -17
    # Cauchy-Schwarz chain of Section 4.2: 2 * (2^P')^2 must stay below P ...
    assert 2 * c.Pfast + 1 < math.log2(c.P) - 1.99
    # ... which the formula as printed (without the factor 1/2) cannot give
    printed = math.log2(c.P - 1) - 1.5
    assert 2 * 2.0 ** (2 * printed) > c.P


def _mulhi(x, y):
    return (x.astype(np.int64) * np.int64(y)) >> 32


@pytest.mark.parametrize("p", K.greedy_moduli()[:20])
def test_mulhi_reduction_of_section_4_3_is_exact(p):
    """y = x - mulhi(x, pinv')*p; y -= (y>=p)*p; y += (y<0)*p  equals x mod p."""
    pinv = (1 << 32) // p - 1
    assert pinv == math.floor(Fraction(2 ** 32, p) - 1)
    rng = np.random.default_rng(p)
    edge = np.array([0, 1, -1, p, -p, p - 1, 1 - p, 2 ** 31 - 1, -2 ** 31, 2 ** 31 - p,
                     -2 ** 31 + p], np.int64)
    near = (np.arange(-300, 300)[:, None] + np.array([0, 2 ** 30, -2 ** 30, 2 ** 31 - 301,
                                                      -2 ** 31 + 300])[None, :]).ravel()
    x = np.concatenate([edge, near, rng.integers(-2 ** 31, 2 ** 31, 400000)])
    x = x[(x >= -2 ** 31) & (x < 2 ** 31)].astype(np.int64)
    y = x - _mulhi(x, pinv) * p
    assert y.min() >= -p and y.max() < 2 * p + p      # stays tiny: int32 is enough
    y = y - (y >= p) * p
    y = y + (y < 0) * p
    assert np.array_equal(y, np.mod(x, p))


def test_int32_accumulation_bound():
    """Section 4.3: k*128^2 <= 2^31 for k <= 2^17, with equality only at k = 2^17
    for p = 256 (the only modulus whose residues reach -128)."""
    assert (2 ** 17 - 1) * 128 * 128 < 2 ** 31
    assert 2 ** 17 * 128 * 128 == 2 ** 31
    for p in K.greedy_moduli()[1:20]:
        assert 2 ** 17 * ((p - 1) // 2) ** 2 < 2 ** 31
