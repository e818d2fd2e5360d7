"""Oracle for the key-verification step.  TEST INFRASTRUCTURE ONLY (same rules as oracle/__init__.py).

What it follows: Section 4.3 (the RS-corrected output c_s is compared with the predetermined key g
"for statistical verification"), Listing of Section 6 (`verify(recovered_key, secret_key)` returns the
accuracy) and Table 2 (the false-positive rate is controlled, at 1e-6, and the true-positive rate
reported).  The paper prints no formula for the test; the reading taken here is the standard one for
multi-bit watermarks: under the null hypothesis (an image that carries no watermark) the K recovered
message bits are independent fair coin flips, so the number of bits that agree with the key is
Binomial(K, 1/2), and an image is declared watermarked when that number reaches the smallest tau with
P(Binomial(K, 1/2) >= tau) <= FPR.

Everything is exact: integers and rationals, no floating point.

Pins (tests/test_oracle_keycheck.py): exhaustive enumeration of all 2^K messages for small K (the
fraction that passes is <= FPR and would exceed it at tau - 1), hand-computed tails for K = 4, an
independent library's binomial survival function and regularised incomplete beta function, and
flipping a known number of bits of the key.
"""
from __future__ import annotations

from fractions import Fraction
from math import comb

import numpy as np


def binomial_tail(K: int, tau: int) -> Fraction:
    """P(Binomial(K, 1/2) >= tau), exactly."""
    if tau <= 0:
        return Fraction(1)
    return Fraction(sum(comb(K, j) for j in range(tau, K + 1)), 2 ** K)


def key_threshold(K: int, fpr) -> int:
    """Smallest tau in 0..K+1 with P(Binomial(K, 1/2) >= tau) <= fpr (K+1: no image ever passes)."""
    fpr = Fraction(fpr)
    for tau in range(0, K + 2):
        if binomial_tail(K, tau) <= fpr:
            return tau
    raise AssertionError("unreachable: the tail at K+1 is zero")


def verify_key(msg, key, m: int, tau: int):
    """msg u8 [N,k] (one m-bit symbol per byte), key u8 [k] -> (matches i32 [N], detected u8 [N]).

    matches = number of the k*m message bits equal to the key's; detected = (matches >= tau).
    Bits of a byte above the low m are not part of the symbol.
    """
    msg = np.asarray(msg, dtype=np.uint8)
    key = np.asarray(key, dtype=np.uint8).reshape(-1)
    N, k = msg.shape
    assert key.shape[0] == k
    matches = np.zeros(N, dtype=np.int32)
    for i in range(N):
        cnt = 0
        for j in range(k):
            for b in range(m):
                if ((int(msg[i, j]) >> b) & 1) == ((int(key[j]) >> b) & 1):
                    cnt += 1
        matches[i] = cnt
    return matches, (matches >= tau).astype(np.uint8)
