"""Miss-probability model of the near-lossless selector (Appendix A) -- oracle
side, TEST INFRASTRUCTURE ONLY.

Setting (Appendix A): C candidates split evenly over T = C / I threads, each
thread keeps a priority queue of length 1, and the N relevant items are placed
uniformly at random among the C slots.  M = number of threads holding at least
one relevant item; L = N - M relevant items are lost.

Eq. 16:  P(M) = C(T, M) * S / C(C, N),  where S sums, over every way of
writing N as an ordered sum of M parts n_j >= 1, the product of C(I, n_j).
S is evaluated here exactly (Python integers) as the coefficient of x^N in
(sum_{n>=1} C(I, n) x^n)^M, which is the same sum grouped by polynomial
multiplication; the brute-force enumeration of the compositions lives in the
tests as a pin.
"""
from __future__ import annotations

from fractions import Fraction
from math import comb


def _series_power_coeff(I: int, M: int, L: int) -> int:
    """Coefficient of x^L in g(x)^M with g(x) = sum_{m>=0} C(I, m+1) x^m,
    i.e. the coefficient of x^(M+L) in (sum_{n>=1} C(I, n) x^n)^M."""
    base = [comb(I, m + 1) for m in range(L + 1)]

    def mul(a, b):
        out = [0] * (L + 1)
        for i, ai in enumerate(a):
            if ai == 0:
                continue
            for j, bj in enumerate(b):
                if i + j > L:
                    break
                out[i + j] += ai * bj
        return out

    result = [1] + [0] * L
    e = M
    while e:
        if e & 1:
            result = mul(result, base)
        base = mul(base, base)
        e >>= 1
    return result[L]


def prob_threads_hit(M: int, N: int, C: int, I: int) -> Fraction:
    """P(M) of Eq. 16 as an exact fraction.  Requires I | C."""
    if C % I:
        raise ValueError("Appendix A assumes T = C / I is an integer")
    T = C // I
    if M < 0 or M > N or M > T:
        return Fraction(0)
    if M == 0:
        return Fraction(1 if N == 0 else 0)
    S = _series_power_coeff(I, M, N - M)
    return Fraction(comb(T, M) * S, comb(C, N))


def miss_probability(l: int, N: int, C: int, I: int) -> float:
    """P(L <= l): probability of losing at most l of the N relevant items."""
    return float(sum(prob_threads_hit(N - m, N, C, I) for m in range(l + 1)))


def expected_recall(N: int, C: int, I: int, queue_len: int = 1) -> float:
    """Expected fraction of the N relevant items that survive the local selection.

    Queue length 1 (Appendix A): E[M] / N; a thread is hit unless all N relevant items avoid
    its I slots, so E[M] = T * (1 - C(C - I, N) / C(C, N)).
    Queue length p in general (same placement model): a thread holding n relevant items keeps
    min(n, p) of them, and n is hypergeometric, P(n) = C(I, n) C(C - I, N - n) / C(C, N); by
    linearity the expected number kept is T * sum_n min(n, p) P(n)."""
    if C % I:
        raise ValueError("Appendix A assumes T = C / I is an integer")
    T = C // I
    if queue_len == 1:
        p_empty = Fraction(comb(C - I, N), comb(C, N))
        return float(T * (1 - p_empty) / N)
    total = comb(C, N)
    kept = Fraction(0)
    # P(n) falls off like (N I / C)^n: far beyond 40 terms nothing is left in double precision
    for n in range(1, min(I, N) + 1):
        pn = Fraction(comb(I, n) * comb(C - I, N - n), total)
        kept += min(n, queue_len) * pn
        if n > queue_len + 40 and pn < Fraction(1, 10 ** 40):
            break
    return float(T * kept / N)
