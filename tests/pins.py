"""Independent yardsticks for the oracle: brute force, closed forms and the ordering that defines
the enumeration.  Nothing here calls the oracle or the GPU library, and none of it uses the
recurrence the oracle builds its table with."""
from __future__ import annotations

import itertools
from fractions import Fraction
from math import comb


def enumerate_pyramid(D: int, K: int):
    """All integer points with sum |p_d| = K (the set P(D,K) of arXiv 2410.16926, Sec. 2.4),
    by filtering the full cube; only for tiny D, K."""
    return [p for p in itertools.product(range(-K, K + 1), repeat=D)
            if sum(abs(v) for v in p) == K]


def n_hypergeometric(D: int, K: int) -> int:
    """N(D,K) = 2 D 2F1(1-D, 1-K; 2; 2) (Sec. 2.4), the series written out; it terminates
    because 1-D and 1-K are non-positive integers.  D, K >= 1."""
    def poch(a, n):
        r = Fraction(1)
        for i in range(n):
            r *= a + i
        return r
    s = Fraction(0)
    for n in range(0, min(D, K)):
        s += poch(Fraction(1 - D), n) * poch(Fraction(1 - K), n) / (poch(Fraction(2), n) * poch(Fraction(1), n)) * Fraction(2) ** n
    v = 2 * D * s
    assert v.denominator == 1
    return int(v)


def n_binomial(D: int, K: int) -> int:
    """Counting argument: choose the i non-zero coordinates, their signs, and a composition of
    K into i positive parts."""
    if K == 0:
        return 1
    return sum((2 ** i) * comb(D, i) * comb(K - 1, i - 1) for i in range(1, min(D, K) + 1))


def coordinate_order(v: int) -> int:
    """Position of a coordinate value in the order the enumeration visits them:
    0, +1, -1, +2, -2, ...  (App. B.2/B.3: the block of x_i = 0 comes first, then for each
    magnitude j the block of +j followed by the block of -j)."""
    return 0 if v == 0 else (2 * v - 1 if v > 0 else -2 * v)


def order_key(p):
    return tuple(coordinate_order(v) for v in p)


def count_before(p, K: int) -> int:
    """Number of points of P(D,K) that precede p in the lexicographic order of order_key:
    the index of p, obtained by counting rather than by the encoding routine.  Uses only the
    binomial count for the sizes of the sets skipped."""
    D = len(p)
    k = K
    total = 0
    for i, v in enumerate(p):
        rest = D - i - 1
        for u in sorted(range(-k, k + 1), key=coordinate_order):
            if coordinate_order(u) >= coordinate_order(v):
                break
            total += n_binomial(rest, k - abs(u)) if rest > 0 else (1 if abs(u) == k else 0)
        k -= abs(v)
    return total
