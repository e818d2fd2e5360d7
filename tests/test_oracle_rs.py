"""Pins for the Reed-Solomon half of the CPU oracle.

Everything the oracle is compared with here is computed by code in THIS file that
uses its own bit-wise field arithmetic (shift-and-reduce multiplication, no tables),
by closed forms, or by exhaustive search, so that a wrong sign, index, table entry or
dropped term in the oracle fails at least one test.

Paper anchors: Appendix B "Notation" ((n,k,t), t = floor((n-k)/2), n_max = 2^m - 1),
"Systematic Evaluation-Based Encoding" (message symbols appear unchanged in the first
k places; Lagrange interpolation through (X_i, M_i) and evaluation on all X_i),
"Berlekamp-Welch Decoding" (any received word within t symbol errors is restored; the
decoder reports message, codeword and number of corrected symbols).
"""
import itertools
import os

import numpy as np
import pytest

import oracle
import synth

CODES = {
    "rs15_11_gf16": dict(m=4, prim_poly=0x13, n=15, k=11),
    "rs12_8_gf16": dict(m=4, prim_poly=0x13, n=12, k=8),
    "rs12_8_gf256": dict(m=8, prim_poly=0x11D, n=12, k=8),
}


# ---------------------------------------------------------------- independent arithmetic

def bmul(a: int, b: int, m: int, poly: int) -> int:
    """Carry-less multiply then reduce modulo the primitive polynomial (no tables)."""
    r = 0
    for i in range(m):
        if (b >> i) & 1:
            r ^= a << i
    for i in range(2 * m - 2, m - 1, -1):
        if (r >> i) & 1:
            r ^= poly << (i - m)
    return r


def bpow(a: int, e: int, m: int, poly: int) -> int:
    r = 1
    for _ in range(e):
        r = bmul(r, a, m, poly)
    return r


def binv(a: int, m: int, poly: int) -> int:
    return bpow(a, (1 << m) - 2, m, poly)


def gen_poly(m, poly, two_t, fcr=1):
    """Coefficients, x^0 first, of prod (x + alpha^(fcr+j))."""
    g = [1]
    for j in range(two_t):
        root = bpow(2, fcr + j, m, poly)
        ng = [0] * (len(g) + 1)
        for i, c in enumerate(g):
            ng[i + 1] ^= c
            ng[i] ^= bmul(c, root, m, poly)
        g = ng
    return g


def poly_rem_high_first(word, g_low_first, m, poly):
    """Remainder of word(x) (word[0] = highest power) modulo monic g; returns 2t symbols, high first."""
    two_t = len(g_low_first) - 1
    w = list(int(x) for x in word)
    for i in range(len(w) - two_t):
        lead = w[i]
        if lead:
            for j in range(two_t + 1):
                w[i + j] ^= bmul(lead, g_low_first[two_t - j], m, poly)
    return w[len(w) - two_t:]


def golden():
    path = os.path.join(os.path.dirname(__file__), "golden", "gf16_rs15_11.txt")
    out = {}
    for line in open(path):
        if line.startswith("#") or ":" not in line:
            continue
        key, vals = line.split(":")
        out[key.strip()] = [int(v) for v in vals.split()]
    return out


# ---------------------------------------------------------------- field

@pytest.mark.parametrize("m,poly", [(4, 0x13), (8, 0x11D)])
def test_field_tables(m, poly):
    q = 1 << m
    e, l = oracle.gf_tables(m, poly)
    # alpha = 2 generates the whole multiplicative group and alpha^(q-1) = 1
    assert sorted(e.tolist()) == list(range(1, q))
    assert bmul(int(e[q - 2]), 2, m, poly) == 1
    x = 1
    for i in range(q - 1):
        assert e[i] == x and l[x] == i
        x = bmul(x, 2, m, poly)


def test_field_golden_gf16():
    g = golden()
    e, _ = oracle.gf_tables(4, 0x13)
    assert e.tolist() == g["exp"]


def test_field_known_values_gf256():
    # widely published values of the 0x11D field (the one QR codes use): alpha^8 = 29, log 3 = 25
    e, l = oracle.gf_tables(8, 0x11D)
    assert e[8] == 29 and l[3] == 25 and l[5] == 50 and l[7] == 198 and e[255 - 1] == 142


@pytest.mark.parametrize("m,poly", [(4, 0x13), (8, 0x11D)])
def test_field_mul_matches_bitwise(m, poly):
    q = 1 << m
    rng = np.random.default_rng(1)
    pairs = itertools.product(range(q), range(q)) if m == 4 else rng.integers(0, q, size=(3000, 2))
    for a, b in pairs:
        assert oracle.gf_mul(m, poly, int(a), int(b)) == bmul(int(a), int(b), m, poly)


def test_rejects_bad_parameters():
    with pytest.raises(ValueError):
        oracle.rs_encode(np.zeros((1, 11), np.uint8), 4, 0x13, 16, 11)       # n > 2^m - 1
    with pytest.raises(ValueError):
        oracle.rs_encode(np.zeros((1, 12), np.uint8), 4, 0x13, 15, 12)       # odd n - k
    with pytest.raises(ValueError):
        oracle.gf_tables(4, 0x1F)                                            # x^4+x^3+x^2+x+1: alpha not primitive


# ---------------------------------------------------------------- encoder

def test_generator_golden_gf16():
    g = oracle.rs_generator(4, 0x13, 15, 11)
    assert g.tolist() == golden()["g"]


@pytest.mark.parametrize("name", list(CODES))
def test_generator_matches_definition(name):
    c = CODES[name]
    g = oracle.rs_generator(c["m"], c["prim_poly"], c["n"], c["k"])
    assert g.tolist() == gen_poly(c["m"], c["prim_poly"], c["n"] - c["k"])
    # the roots are alpha^1..alpha^2t
    for j in range(1, c["n"] - c["k"] + 1):
        x = bpow(2, j, c["m"], c["prim_poly"])
        y = 0
        for coef in reversed(g.tolist()):
            y = bmul(y, x, c["m"], c["prim_poly"]) ^ coef
        assert y == 0


@pytest.mark.parametrize("name", list(CODES))
def test_encode_systematic_divisible_linear(name):
    c = CODES[name]
    m, poly, n, k = c["m"], c["prim_poly"], c["n"], c["k"]
    msgs, _, _ = synth.rs_cases(7, 200, n, k, m)
    cws = oracle.rs_encode(msgs, m, poly, n, k)
    assert np.array_equal(cws[:, :k], msgs)                       # first k symbols unchanged
    g = gen_poly(m, poly, n - k)
    for w in cws[:60]:
        assert not any(poly_rem_high_first(w, g, m, poly))        # g(x) divides every codeword
    assert not oracle.rs_syndromes(cws, m, poly, n, k).any()      # clean codeword => zero syndromes
    # linear over GF(2^m): sum of codewords is the codeword of the sum
    s = oracle.rs_encode(msgs[:100] ^ msgs[100:], m, poly, n, k)
    assert np.array_equal(s, cws[:100] ^ cws[100:])
    # zero message -> zero codeword; unit message -> non-zero parity
    assert not oracle.rs_encode(np.zeros((1, k), np.uint8), m, poly, n, k).any()


def test_syndrome_definition_single_error():
    # r = e * x^p  =>  S_j = e * alpha^(j p)
    m, poly, n, k = 4, 0x13, 15, 11
    for p in range(n):
        for e in (1, 7, 15):
            w = np.zeros((1, n), np.uint8)
            w[0, n - 1 - p] = e
            S = oracle.rs_syndromes(w, m, poly, n, k)[0]
            for j in range(1, 5):
                assert S[j - 1] == bmul(e, bpow(2, (j * p) % 15, m, poly), m, poly)


def lagrange_encode(msg, n, k, m, poly):
    """Evaluation-based systematic encoder of Appendix B with X_i = alpha^i (own arithmetic)."""
    X = [bpow(2, i, m, poly) for i in range(n)]

    def P(x):
        tot = 0
        for i in range(k):
            num, den = 1, 1
            for j in range(k):
                if j != i:
                    num = bmul(num, x ^ X[j], m, poly)
                    den = bmul(den, X[i] ^ X[j], m, poly)
            tot ^= bmul(msg[i], bmul(num, binv(den, m, poly), m, poly), m, poly)
        return tot
    return [P(x) for x in X]


def test_paper_evaluation_code_is_the_same_code():
    """With X_i = alpha^i and n = 2^m - 1 the evaluation code of the paper is the set of
    polynomials (C_i = coefficient of x^i) that vanish at alpha^1..alpha^(n-k): its words have
    zero oracle syndromes once written highest power first."""
    m, poly, n, k = 4, 0x13, 15, 11
    rng = np.random.default_rng(5)
    for _ in range(40):
        msg = rng.integers(0, 16, size=k).tolist()
        cw = lagrange_encode(msg, n, k, m, poly)
        assert cw[:k] == msg
        as_high_first = np.array(cw[::-1], dtype=np.uint8)[None, :]
        assert not oracle.rs_syndromes(as_high_first, m, poly, n, k).any()


# ---------------------------------------------------------------- decoder vs exhaustive search

class NearestCodeword:
    """Exhaustive bounded-distance decoder: tabulates x^(n-k)-remainders of every error pattern of
    weight <= t; a received word decodes to r - e iff rem(r) == rem(e).  Uses only bmul."""

    def __init__(self, m, prim_poly, n, k):
        self.m, self.poly, self.n, self.k = m, prim_poly, n, k
        q = 1 << m
        two_t = n - k
        assert two_t == 4
        self.g = gen_poly(m, prim_poly, two_t)
        bits = m * two_t
        # R1[p][v] = packed remainder of v * x^p (p = power; symbol index n-1-p)
        R1 = np.zeros((n, q), dtype=np.uint64)
        for p in range(n):
            unit = [0] * n
            unit[n - 1 - p] = 1
            base = poly_rem_high_first(unit, self.g, m, prim_poly)
            for v in range(1, q):
                rem = [bmul(v, b, m, prim_poly) for b in base]
                R1[p, v] = self._pack(rem)
        self.R1 = R1
        keys = [np.zeros(1, np.uint64)]
        pats = [np.zeros((1, 4), np.int32)]                     # (p1, v1, p2, v2), v = 0 unused
        vs = np.arange(1, q)
        for p in range(n):
            keys.append(R1[p, 1:])
            pats.append(np.stack([np.full(q - 1, p), vs, np.zeros(q - 1, int), np.zeros(q - 1, int)], 1).astype(np.int32))
        v1, v2 = np.meshgrid(vs, vs, indexing="ij")
        v1, v2 = v1.ravel(), v2.ravel()
        for p1 in range(n):
            for p2 in range(p1 + 1, n):
                keys.append(R1[p1, v1] ^ R1[p2, v2])
                pats.append(np.stack([np.full(v1.size, p1), v1, np.full(v1.size, p2), v2], 1).astype(np.int32))
        keys = np.concatenate(keys)
        pats = np.concatenate(pats)
        order = np.argsort(keys, kind="stable")
        self.keys, self.pats = keys[order], pats[order]
        self.count = keys.size
        # minimum distance 2t+1: no two patterns of weight <= t share a remainder
        assert np.all(self.keys[1:] != self.keys[:-1])
        assert bits <= 64

    def _pack(self, rem):
        x = 0
        for s in rem:
            x = (x << self.m) | int(s)
        return x

    def decode(self, word):
        key = np.uint64(self._pack(poly_rem_high_first(word, self.g, self.m, self.poly)))
        i = int(np.searchsorted(self.keys, key))
        if i >= self.count or self.keys[i] != key:
            return None, -1
        p1, v1, p2, v2 = (int(x) for x in self.pats[i])
        out = np.array(word, dtype=np.uint8).copy()
        nerr = 0
        if v1:
            out[self.n - 1 - p1] ^= v1
            nerr += 1
        if v2:
            out[self.n - 1 - p2] ^= v2
            nerr += 1
        return out, nerr


_NC = {}


def nearest(name):
    if name not in _NC:
        _NC[name] = NearestCodeword(**CODES[name])
    return _NC[name]


def test_sphere_sizes():
    # number of words within distance 2 of a codeword (closed form: sum C(n,i)(q-1)^i)
    assert nearest("rs15_11_gf16").count == 23851
    assert nearest("rs12_8_gf16").count == 15031
    assert nearest("rs12_8_gf256").count == 4294711


def _check_against_exhaustive(name, words):
    c = CODES[name]
    nc = nearest(name)
    msg, cw, nerr = oracle.rs_decode(words, c["m"], c["prim_poly"], c["n"], c["k"])
    for i, w in enumerate(words):
        ref, ne = nc.decode(w)
        assert nerr[i] == ne, (i, w, nerr[i], ne)
        if ne < 0:                                   # failure: received word passed through
            assert np.array_equal(cw[i], w) and np.array_equal(msg[i], w[:c["k"]])
        else:
            assert np.array_equal(cw[i], ref) and np.array_equal(msg[i], ref[:c["k"]])
            assert int(np.count_nonzero(cw[i] != w)) == ne
    return nerr


@pytest.mark.parametrize("name,cfg,count", [("rs15_11_gf16", 0, 1024), ("rs12_8_gf16", 1, 1024),
                                            ("rs12_8_gf256", 3, 600)])
def test_decode_equals_nearest_codeword_on_error_sets(name, cfg, count):
    """0..3 injected errors (t = 2): exact recovery up to t, flagged or legally miscorrected beyond."""
    c = CODES[name]
    msgs, err, ninj = synth.rs_cases(cfg, count, c["n"], c["k"], c["m"])
    clean = oracle.rs_encode(msgs, c["m"], c["prim_poly"], c["n"], c["k"])
    words = clean ^ err
    nerr = _check_against_exhaustive(name, words)
    msg, cw, _ = oracle.rs_decode(words, c["m"], c["prim_poly"], c["n"], c["k"])
    ok = ninj <= 2
    assert np.array_equal(nerr[ok], ninj[ok].astype(np.int8))      # number corrected = number injected
    assert np.array_equal(msg[ok], msgs[ok]) and np.array_equal(cw[ok], clean[ok])
    # beyond t: never silently returns the transmitted codeword
    bad = ~ok
    assert bad.sum() > 100
    assert not np.any(np.all(cw[bad] == clean[bad], axis=1))
    # corrected words are codewords
    good = nerr >= 0
    assert not oracle.rs_syndromes(cw[good], c["m"], c["prim_poly"], c["n"], c["k"]).any()


@pytest.mark.parametrize("name,cfg", [("rs15_11_gf16", 0), ("rs12_8_gf16", 1), ("rs12_8_gf256", 3)])
def test_decode_equals_nearest_codeword_on_random_words(name, cfg):
    c = CODES[name]
    words = synth.random_words(cfg, 1500, c["n"], c["m"])
    _check_against_exhaustive(name, words)


@pytest.mark.parametrize("name,cfg,p", [("rs15_11_gf16", 0, 23851 / 65536), ("rs12_8_gf16", 1, 15031 / 65536),
                                        ("rs12_8_gf256", 3, 4294711 / 2 ** 32)])
def test_random_word_acceptance_rate(name, cfg, p):
    """A uniformly random word lies in some decoding sphere with probability V(n,t)/q^(n-k)."""
    c = CODES[name]
    N = 200000
    words = synth.random_words(cfg, N, c["n"], c["m"], block=2000)
    _, _, nerr = oracle.rs_decode(words, c["m"], c["prim_poly"], c["n"], c["k"])
    acc = np.count_nonzero(nerr >= 0)
    sigma = np.sqrt(N * p * (1 - p))
    assert abs(acc - N * p) < 5 * sigma + 1, (acc, N * p, sigma)


def test_all_single_and_double_errors_rs15_11():
    """Every error pattern of weight <= 2 on one codeword is corrected exactly (exhaustive)."""
    m, poly, n, k = 4, 0x13, 15, 11
    msg = np.arange(1, 12, dtype=np.uint8)[None, :]
    cw = oracle.rs_encode(msg, m, poly, n, k)[0]
    words, counts = [], []
    for p in range(n):
        for v in range(1, 16):
            w = cw.copy(); w[p] ^= v
            words.append(w); counts.append(1)
    for p1, p2 in itertools.combinations(range(n), 2):
        for v1 in range(1, 16):
            for v2 in (1, 6, 11, 15):
                w = cw.copy(); w[p1] ^= v1; w[p2] ^= v2
                words.append(w); counts.append(2)
    words = np.array(words, dtype=np.uint8)
    dm, dc, ne = oracle.rs_decode(words, m, poly, n, k)
    assert np.array_equal(ne, np.array(counts, dtype=np.int8))
    assert np.all(dc == cw[None, :]) and np.all(dm == msg)


def test_shortened_code_is_the_full_code_with_leading_zeros():
    m, poly = 4, 0x13
    msgs, err, _ = synth.rs_cases(1, 300, 12, 8, m)
    cw12 = oracle.rs_encode(msgs, m, poly, 12, 8)
    full_msgs = np.concatenate([np.zeros((300, 3), np.uint8), msgs], axis=1)
    cw15 = oracle.rs_encode(full_msgs, m, poly, 15, 11)
    assert np.array_equal(cw15[:, 3:], cw12) and not cw15[:, :3].any()
    # a correction the full code would place in the removed positions is a failure for the short code
    w12 = cw12 ^ err
    w15 = np.concatenate([np.zeros((300, 3), np.uint8), w12], axis=1)
    _, c12, n12 = oracle.rs_decode(w12, m, poly, 12, 8)
    _, c15, n15 = oracle.rs_decode(w15, m, poly, 15, 11)
    for i in range(300):
        if n15[i] >= 0 and not c15[i, :3].any():
            assert n12[i] == n15[i] and np.array_equal(c12[i], c15[i, 3:])
        else:
            assert n12[i] == -1


def test_other_first_consecutive_root():
    # fcr = 0 (the convention QR codes use): same guarantees
    m, poly, n, k = 8, 0x11D, 20, 14
    msgs, err, ninj = synth.rs_cases(9, 400, n, k, m, max_err=3)
    cws = oracle.rs_encode(msgs, m, poly, n, k, fcr=0)
    assert not oracle.rs_syndromes(cws, m, poly, n, k, fcr=0).any()
    dm, dc, ne = oracle.rs_decode(cws ^ err, m, poly, n, k, fcr=0)
    assert np.array_equal(ne, ninj.astype(np.int8))               # t = 3 here: all corrected
    assert np.array_equal(dm, msgs) and np.array_equal(dc, cws)


def test_symbols_above_field_size_are_masked():
    m, poly, n, k = 4, 0x13, 15, 11
    msgs, err, _ = synth.rs_cases(0, 50, n, k, m)
    w = oracle.rs_encode(msgs, m, poly, n, k) ^ err
    a = oracle.rs_decode(w, m, poly, n, k)
    b = oracle.rs_decode(w | 0xA0, m, poly, n, k)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
