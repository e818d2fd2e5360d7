"""A second oracle for the Reed-Solomon stage: the decoder the paper itself describes.  TEST INFRASTRUCTURE ONLY.

What it follows, step by step, in the paper's notation (Appendix B):
  * "Systematic Evaluation-Based Encoding": evaluation points X_0..X_{n-1}, the message symbols M_i are the values of
    a polynomial P of degree < k at the first k points (Lagrange interpolation), the code word is C_i = P(X_i);
  * "Berlekamp-Welch Decoding": find Q (degree <= t, not zero) and N (degree <= t + k - 1) with
    N(X_i) = R_i Q(X_i) at all n points - a homogeneous linear system solved by Gaussian elimination over GF(2^m) -,
    accept when Q divides N with a quotient of degree < k, P = N / Q, and read the symbols back by evaluation.
A word for which no such pair exists (no code word within t symbol errors) is reported as a failure.

The field arithmetic here is its own (shift-and-reduce products, brute-force inverses): nothing is shared with
oracle/qrm_oracle.c, whose syndrome-based decoder this one is held against in tests/test_oracle_rs_bw.py on the full
length codes, where X_i = alpha^i makes the two descriptions the same code (C_i = coefficient of x^i).
"""
from __future__ import annotations

from typing import List, Optional, Tuple


class Field:
    def __init__(self, m: int, prim_poly: int):
        self.m, self.poly, self.q = m, prim_poly, 1 << m

    def mul(self, a: int, b: int) -> int:
        r = 0
        for i in range(self.m):
            if (b >> i) & 1:
                r ^= a << i
        for i in range(2 * self.m - 2, self.m - 1, -1):
            if (r >> i) & 1:
                r ^= self.poly << (i - self.m)
        return r

    def inv(self, a: int) -> int:
        assert a != 0
        for b in range(1, self.q):
            if self.mul(a, b) == 1:
                return b
        raise ArithmeticError("no inverse")

    def power(self, a: int, e: int) -> int:
        r = 1
        for _ in range(e):
            r = self.mul(r, a)
        return r

    def poly_eval(self, p: List[int], x: int) -> int:     # p[j] = coefficient of x^j
        r = 0
        for c in reversed(p):
            r = self.mul(r, x) ^ c
        return r


def evaluation_points(F: Field, n: int) -> List[int]:
    """X_i = alpha^i with alpha = x (the element 2): pairwise distinct for n <= 2^m - 1."""
    return [F.power(2, i) for i in range(n)]


def encode(F: Field, X: List[int], k: int, msg: List[int]) -> List[int]:
    """C_i = P(X_i), P the interpolation polynomial through (X_i, M_i), i < k."""
    def P(x):
        tot = 0
        for i in range(k):
            num, den = 1, 1
            for j in range(k):
                if j != i:
                    num = F.mul(num, x ^ X[j])
                    den = F.mul(den, X[i] ^ X[j])
            tot ^= F.mul(msg[i], F.mul(num, F.inv(den)))
        return tot
    return [P(x) for x in X]


def _nullspace_vector(F: Field, rows: List[List[int]], n_unknowns: int) -> Optional[List[int]]:
    """One non-zero solution of rows * v = 0 (Gauss-Jordan elimination), or None if only v = 0 solves it."""
    A = [r[:] for r in rows]
    pivots = []            # (row, column)
    r = 0
    for c in range(n_unknowns):
        p = next((i for i in range(r, len(A)) if A[i][c]), None)
        if p is None:
            continue
        A[r], A[p] = A[p], A[r]
        s = F.inv(A[r][c])
        A[r] = [F.mul(s, v) for v in A[r]]
        for i in range(len(A)):
            if i != r and A[i][c]:
                f = A[i][c]
                A[i] = [a ^ F.mul(f, b) for a, b in zip(A[i], A[r])]
        pivots.append((r, c))
        r += 1
        if r == len(A):
            break
    pivot_cols = {c for _, c in pivots}
    free = [c for c in range(n_unknowns) if c not in pivot_cols]
    if not free:
        return None
    v = [0] * n_unknowns
    v[free[0]] = 1
    for row, c in pivots:
        v[c] = A[row][free[0]]          # characteristic 2: minus is plus
    return v


def _poly_divmod(F: Field, num: List[int], den: List[int]) -> Tuple[List[int], List[int]]:
    num = num[:]
    while den and den[-1] == 0:
        den = den[:-1]
    dq = len(den) - 1
    quo = [0] * max(1, len(num) - dq)
    s = F.inv(den[-1])
    for i in range(len(num) - 1, dq - 1, -1):
        if num[i]:
            f = F.mul(num[i], s)
            quo[i - dq] = f
            for j, d in enumerate(den):
                num[i - dq + j] ^= F.mul(f, d)
    return quo, num


def decode(F: Field, X: List[int], k: int, R: List[int]):
    """-> (message, code word, number of corrected symbols) or None when no code word lies within t errors."""
    n = len(X)
    t = (n - k) // 2
    nq, nn = t + 1, t + k                                   # unknown coefficients of Q and of N
    rows = []
    for i in range(n):
        pw = [F.power(X[i], j) for j in range(max(nq, nn))]
        rows.append([F.mul(R[i], pw[j]) for j in range(nq)] + [pw[j] for j in range(nn)])   # R_i Q(X_i) + N(X_i) = 0
    v = _nullspace_vector(F, rows, nq + nn)
    if v is None:
        return None
    Q, N = v[:nq], v[nq:]
    if not any(Q):
        return None
    quo, rem = _poly_divmod(F, N, Q)
    if any(rem) or any(quo[k:]):
        return None                                          # Q does not divide N, or the quotient is too long
    P = (quo + [0] * k)[:k]
    C = [F.poly_eval(P, x) for x in X]
    nerr = sum(1 for a, b in zip(C, R) if a != b)
    if nerr > t:
        return None
    return C[:k], C, nerr
