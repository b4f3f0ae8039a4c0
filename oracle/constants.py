"""Constants of Ozaki scheme II, computed with Python's unbounded integers.

TEST INFRASTRUCTURE ONLY.  This module is part of the CPU oracle: it may be
imported from tests/, from __graft_entry__.smoke() and from bench.py's
cpu_baseline leg, never from the product path.  It shares no code with the HIP
library, which derives its own table with its own fixed-width integer class.

Every quantity follows Section 4.1 ("Determination of Constants") of the paper:

* moduli          greedy descending pairwise-coprime picks starting at 256
                  (the set printed in Section 4.1, whose tail is 41, 37, 29);
                  for a given N the first N of that list are used.
* P               product of the N moduli                       (Step 1, Sec. 3)
* q_i             inverse of P/p_i modulo p_i                   (Theorem 1)
* w_i             (P/p_i) * q_i, the CRT weight                 (Eq. 2)
* P1, P2          double(P), double(P - P1)                     (Sec. 4.1)
* beta_i          53 - 8 - ceil(log2 N) + floor(log2 w_i) - floor(log2 max_j w_j)
* s_i1            w_i with everything below its top beta_i bits cleared
* s_i2            double(w_i - s_i1)
* P_inv           double(1/P)
* P'_fast         single(0.5*log2(P-1) - 1.5); the printed formula lacks the
                  factor 0.5, without which Eq. 3 cannot hold (the bound
                  2*mu*|a|*nu*|b| <= 2*2^(2P') must stay below P)
* P'_accu         single(0.5*log2(P-1) - 0.5), with the same factor 0.5: it makes the
                  accurate-mode bound exactly 2*2^(2P') = P-1 < P
* pinv'_i         floor(2^32/p_i - 1), the multiplier of the mulhi reduction
                  (Section 4.3)

For SGEMM emulation s_i1 = double(w_i) and s_i2 = P2 = 0 (Sec. 4.1).
"""
from __future__ import annotations

import math
import struct
from dataclasses import dataclass
from fractions import Fraction
from typing import List

MAX_MODULI = 20


def greedy_moduli(limit: int = 256) -> List[int]:
    """Every modulus the greedy rule of Section 4.1 can pick, in pick order.

    Walk c = limit, limit-1, ..., 2 and keep c when it is coprime to every
    modulus kept so far.
    """
    picked: List[int] = []
    for c in range(limit, 1, -1):
        if all(math.gcd(c, p) == 1 for p in picked):
            picked.append(c)
    return picked


def moduli(n: int) -> List[int]:
    if not 2 <= n <= MAX_MODULI:
        raise ValueError("number of moduli must be in 2..20")
    return greedy_moduli()[:n]


def _to_f32(x: float) -> float:
    """Round a double to the nearest binary32 value (returned as a double)."""
    return struct.unpack("<f", struct.pack("<f", x))[0]


def _ceil_log2(n: int) -> int:
    return (n - 1).bit_length()


@dataclass(frozen=True)
class Constants:
    n: int
    is_double: bool
    p: List[int]          # moduli
    P: int                # product
    q: List[int]          # modular inverses of P/p_i
    w: List[int]          # CRT weights (P/p_i)*q_i
    beta: List[int]       # bits kept in s_i1 (fp64 path only)
    s1: List[float]
    s2: List[float]
    P1: float
    P2: float
    Pinv: float
    Pfast: float          # binary32 value widened to double
    Paccu: float          # single(0.5*log2(P-1) - 0.5), same reading as P'_fast
    pinv_prime: List[int]


def constants(n: int, is_double: bool = True) -> Constants:
    p = moduli(n)
    P = 1
    for pi in p:
        P *= pi
    q = [pow(P // pi, -1, pi) for pi in p]
    w = [(P // pi) * qi for pi, qi in zip(p, q)]

    P1 = float(P)                       # int -> float is correctly rounded
    Pinv = float(Fraction(1, P))        # Fraction -> float is correctly rounded
    Pfast = _to_f32(0.5 * math.log2(P - 1) - 1.5)
    Paccu = _to_f32(0.5 * math.log2(P - 1) - 0.5)
    pinv_prime = [(1 << 32) // pi - 1 for pi in p]

    if is_double:
        P2 = float(P - int(P1))
        wmax_log = max(w).bit_length() - 1
        beta, s1, s2 = [], [], []
        for wi in w:
            b = 53 - 8 - _ceil_log2(n) + (wi.bit_length() - 1) - wmax_log
            cut = wi.bit_length() - b
            hi = (wi >> cut) << cut if cut > 0 else wi
            beta.append(b)
            s1.append(float(hi))        # exact: at most beta_i <= 45 significant bits
            assert int(s1[-1]) == hi
            s2.append(float(wi - hi))
    else:
        P2 = 0.0
        beta = [0] * n
        s1 = [float(wi) for wi in w]
        s2 = [0.0] * n
    return Constants(n, is_double, p, P, q, w, beta, s1, s2, P1, P2, Pinv,
                     Pfast, Paccu, pinv_prime)
