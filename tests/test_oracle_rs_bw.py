"""The paper's own decoder (Appendix B: evaluation-based encoding, Berlekamp-Welch with Gaussian elimination), written
out in oracle/berlekamp_welch.py with its own field arithmetic, against the syndrome-based oracle that the GPU kernels
are compared with.  On the full-length codes X_i = alpha^i makes the evaluation code and the oracle's code the same
set of words (C_i = coefficient of x^i; the oracle lists the highest power first), so the two must return the same
code word, the same number of corrected symbols and the same failures on every received word."""
import numpy as np
import pytest

import oracle
from oracle import berlekamp_welch as bw

CODES = [(4, 0x13, 15, 11), (4, 0x13, 15, 7), (3, 0xB, 7, 3), (5, 0x25, 31, 27), (4, 0x13, 15, 13)]


@pytest.mark.parametrize("m,poly,n,k", CODES)
def test_encoding_is_systematic_and_lands_in_the_oracle_code(m, poly, n, k):
    F = bw.Field(m, poly)
    X = bw.evaluation_points(F, n)
    assert len(set(X)) == n
    rng = np.random.default_rng(m * 100 + k)
    for _ in range(10):
        msg = rng.integers(0, 1 << m, size=k).tolist()
        cw = bw.encode(F, X, k, msg)
        assert cw[:k] == msg
        assert not oracle.rs_syndromes(np.array(cw[::-1], dtype=np.uint8)[None, :], m, poly, n, k).any()


@pytest.mark.parametrize("m,poly,n,k", CODES)
def test_berlekamp_welch_agrees_with_the_syndrome_decoder(m, poly, n, k):
    F = bw.Field(m, poly)
    X = bw.evaluation_points(F, n)
    t = (n - k) // 2
    rng = np.random.default_rng(m * 1000 + n * 10 + k)
    words = []
    for trial in range(60):
        cw = bw.encode(F, X, k, rng.integers(0, 1 << m, size=k).tolist())
        ne = int(rng.integers(0, t + 3))                     # up to two errors too many
        for p in rng.choice(n, size=ne, replace=False):
            cw[p] ^= int(rng.integers(1, 1 << m))
        words.append(cw)
    for trial in range(20):
        words.append(rng.integers(0, 1 << m, size=n).tolist())   # arbitrary words: mostly failures
    high_first = np.array([w[::-1] for w in words], dtype=np.uint8)
    _, ocw, onerr = oracle.rs_decode(high_first, m, poly, n, k)
    fails = 0
    for w, oc, oe in zip(words, ocw, onerr):
        got = bw.decode(F, X, k, w)
        if oe < 0:
            assert got is None
            fails += 1
        else:
            assert got is not None
            msg, cw, nerr = got
            assert cw == oc[::-1].tolist() and nerr == int(oe) and msg == cw[:k]
    assert 0 < fails < len(words)


def test_one_error_by_hand_gf8():
    """RS(7,3) over GF(8), message (1, 0, 0) at X = (1, 2, 4): P is the Lagrange basis polynomial of X_0."""
    F = bw.Field(3, 0xB)
    X = bw.evaluation_points(F, 7)
    assert X == [1, 2, 4, 3, 6, 7, 5]                        # powers of alpha = x modulo x^3 + x + 1
    cw = bw.encode(F, X, 3, [1, 0, 0])
    assert cw[:3] == [1, 0, 0]
    hit = cw[:]
    hit[5] ^= 6
    hit[1] ^= 3
    msg, fixed, nerr = bw.decode(F, X, 3, hit)
    assert (msg, fixed, nerr) == ([1, 0, 0], cw, 2)
    hit[2] ^= 1                                              # a third error: beyond t = 2
    out = bw.decode(F, X, 3, hit)
    assert out is None or out[1] != cw
