"""Pins for the key-verification oracle (oracle/keycheck.py).

Paper anchors: Section 4.3 (the RS-corrected message is compared with the predetermined key for
statistical verification), Table 2 (false-positive rate controlled at 1e-6).  What the oracle is
compared with: exhaustive enumeration over every possible message, tails worked out by hand, an
independent library (scipy) for the binomial survival function and the regularised incomplete beta
function, and messages built by flipping a known number of key bits.
"""
import itertools
from fractions import Fraction

import numpy as np
import pytest
from scipy import special, stats

from oracle import keycheck


def test_tail_of_four_coin_flips_by_hand():
    # 16 outcomes: 1 with four heads, 4 with three, 6 with two, 4 with one, 1 with none
    assert keycheck.binomial_tail(4, 4) == Fraction(1, 16)
    assert keycheck.binomial_tail(4, 3) == Fraction(5, 16)
    assert keycheck.binomial_tail(4, 2) == Fraction(11, 16)
    assert keycheck.binomial_tail(4, 1) == Fraction(15, 16)
    assert keycheck.binomial_tail(4, 0) == 1
    assert keycheck.binomial_tail(4, 5) == 0


def test_threshold_of_four_coin_flips_by_hand():
    assert keycheck.key_threshold(4, Fraction(1, 16)) == 4      # equality counts as controlled
    assert keycheck.key_threshold(4, Fraction(6, 100)) == 5     # 1/16 > 0.06: nothing may pass
    assert keycheck.key_threshold(4, Fraction(32, 100)) == 3
    assert keycheck.key_threshold(4, Fraction(7, 10)) == 2
    assert keycheck.key_threshold(4, 1) == 0


def test_threshold_for_48_and_32_bits_at_one_in_a_million():
    # C(48,0..7) = 1, 48, 1128, 17296, 194580, 1712304, 12271512, 73629072 sum to 87825941;
    # 87825941 / 2^48 = 3.12e-7 <= 1e-6, and adding C(48,8) = 377348994 gives 1.65e-6 > 1e-6.
    assert sum([1, 48, 1128, 17296, 194580, 1712304, 12271512, 73629072]) == 87825941
    assert keycheck.binomial_tail(48, 41) == Fraction(87825941, 2 ** 48)
    assert keycheck.key_threshold(48, Fraction(1, 10 ** 6)) == 41
    # 32 message bits of RS(12,8) over GF(16): 1 + 32 + 496 = 529 -> 1.2e-7; + 4960 -> 1.28e-6
    assert keycheck.key_threshold(32, Fraction(1, 10 ** 6)) == 30


@pytest.mark.parametrize("K", [1, 8, 32, 48, 64, 96, 256])
@pytest.mark.parametrize("fpr", [1e-2, 1e-4, 1e-6, 1e-9])
def test_threshold_against_library_survival_function(K, fpr):
    tau = keycheck.key_threshold(K, Fraction(fpr))
    assert 0 <= tau <= K + 1
    # survival function sf(x) = P(X > x); the regularised incomplete beta function gives the same tail
    if tau <= K:
        assert stats.binom.sf(tau - 1, K, 0.5) <= fpr * (1 + 1e-9)
        if tau >= 1:
            assert special.betainc(tau, K - tau + 1, 0.5) <= fpr * (1 + 1e-9)
    else:
        assert 0.5 ** K > fpr
    if tau >= 1:
        assert stats.binom.sf(tau - 2, K, 0.5) > fpr * (1 - 1e-9)


def test_threshold_is_monotone_in_the_rate():
    last = None
    for e in range(1, 15):
        tau = keycheck.key_threshold(40, Fraction(1, 10 ** e))
        assert last is None or tau >= last
        last = tau
    assert last == 41  # 2^-40 = 9.1e-13 > 1e-14: impossible, nothing passes


@pytest.mark.parametrize("k,m", [(3, 4), (2, 5), (1, 8), (4, 3)])
def test_exhaustive_false_positive_rate(k, m):
    """Every possible message against a fixed key: the passing fraction is the binomial tail."""
    rng = np.random.default_rng(7 + k * 16 + m)
    key = rng.integers(0, 1 << m, size=k, dtype=np.uint8)
    K = k * m
    msgs = np.array(list(itertools.product(range(1 << m), repeat=k)), dtype=np.uint8)
    assert msgs.shape[0] == 1 << K
    for fpr in (Fraction(1, 3), Fraction(1, 20), Fraction(1, 500)):
        tau = keycheck.key_threshold(K, fpr)
        matches, det = keycheck.verify_key(msgs, key, m, tau)
        assert Fraction(int(det.sum()), 1 << K) <= fpr
        assert Fraction(int((matches >= tau - 1).sum()), 1 << K) > fpr
        # the count of agreeing bits is binomial: C(K, j) messages agree in exactly j places
        hist = np.bincount(matches, minlength=K + 1)
        from math import comb
        assert [int(x) for x in hist] == [comb(K, j) for j in range(K + 1)]


def test_flipping_j_bits_loses_j_matches():
    rng = np.random.default_rng(11)
    for m, k in ((4, 8), (8, 8), (5, 7)):
        K = k * m
        key = rng.integers(0, 1 << m, size=k, dtype=np.uint8)
        msgs = np.zeros((K + 1, k), dtype=np.uint8)
        for j in range(K + 1):
            bits = rng.choice(K, size=j, replace=False)
            w = key.copy()
            for b in bits:
                w[b // m] ^= np.uint8(1 << (b % m))
            msgs[j] = w
        matches, det = keycheck.verify_key(msgs, key, m, K - 2)
        assert matches.tolist() == [K - j for j in range(K + 1)]
        assert det.tolist() == [1, 1, 1] + [0] * (K - 2)


def test_bits_above_the_symbol_width_are_ignored():
    key = np.array([0x3, 0xA], dtype=np.uint8)
    msg = np.array([[0xF3, 0x5A], [0x03, 0x0A]], dtype=np.uint8)
    matches, _ = keycheck.verify_key(msg, key, 4, 0)
    assert matches.tolist() == [8, 8]
