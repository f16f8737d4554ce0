"""Pins for the oracle's pyramid encoding (point -> index) and decoding (index -> point)."""
import json
import os
import random

import numpy as np
import pytest

from oracle import pvq_oracle as o
from tests import pins

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_values.json")))
TINY = [(1, 1), (1, 4), (2, 1), (2, 7), (3, 1), (3, 5), (4, 4), (4, 6), (5, 4), (6, 3)]


@pytest.mark.parametrize("D,K", TINY)
def test_rank_is_a_bijection_onto_0_N(D, K):
    pts = pins.enumerate_pyramid(D, K)
    idx = o.rank(pts, K)
    assert sorted(idx) == list(range(len(pts)))


@pytest.mark.parametrize("D,K", TINY)
def test_rank_is_the_position_in_the_defining_order(D, K):
    # sorting the brute-force point set by the visiting order 0,+1,-1,+2,-2,... per coordinate
    # must give index 0,1,2,...: checks every term of the encoding sum, not only bijectivity
    pts = sorted(pins.enumerate_pyramid(D, K), key=pins.order_key)
    assert o.rank(pts, K) == list(range(len(pts)))


@pytest.mark.parametrize("D,K", TINY)
def test_unrank_inverts_rank_everywhere(D, K):
    pts = sorted(pins.enumerate_pyramid(D, K), key=pins.order_key)
    got = o.unrank(range(len(pts)), D, K)
    assert got.tolist() == [list(p) for p in pts]


def test_paper_worked_example_codes():
    g = GOLD["pyramid_2_7"]
    pts = pins.enumerate_pyramid(g["D"], g["K"])
    idx = o.rank(pts, g["K"])
    assert min(idx) == g["first_code"] and max(idx) == g["last_code"]
    # the order on P(2,7): (0,7),(0,-7),(1,6),(1,-6),(-1,6),(-1,-6),(2,5),...,(7,0),(-7,0)
    assert o.unrank([0, 1, 2, 3, 4, 5, 6, 26, 27], 2, 7).tolist() == [
        [0, 7], [0, -7], [1, 6], [1, -6], [-1, 6], [-1, -6], [2, 5], [7, 0], [-7, 0]]


@pytest.mark.parametrize("D,K", [(8, 16), (16, 33), (32, 60)])
def test_extreme_points(D, K):
    N = pins.n_binomial(D, K)
    first = [0] * (D - 1) + [K]
    second = [0] * (D - 1) + [-K]
    last = [-K] + [0] * (D - 1)
    assert o.rank([first, second, last], K) == [0, 1, N - 1]
    assert o.unrank([0, 1, N - 1], D, K).tolist() == [first, second, last]


def _random_point(rng, D, K):
    cuts = sorted(rng.randint(0, K) for _ in range(D - 1))
    mags = [b - a for a, b in zip([0] + cuts, cuts + [K])]
    return [m if rng.random() < 0.5 else -m for m in mags]


@pytest.mark.parametrize("D,K", [(8, 16), (16, 33), (32, 60), (7, 11), (64, 40), (128, 187)])
def test_wide_indices_against_counting_with_python_integers(D, K):
    rng = random.Random(D * 1000 + K)
    pts = [_random_point(rng, D, K) for _ in range(150 if D <= 32 else 24)]
    want = [pins.count_before(p, K) for p in pts]
    assert o.rank(pts, K) == want
    assert o.unrank(want, D, K).tolist() == pts
    assert max(want) < pins.n_binomial(D, K)
    if D == 32:
        assert max(want).bit_length() > 96      # the 4-word path is really exercised
    if D == 128:
        # the large-group setting of on-the-fly activation quantisation: 3 bits per value
        assert o.index_bits(D, K) <= 384 < o.index_bits(D, K + 1)
        assert max(want).bit_length() > 352     # twelve words


def test_counting_yardstick_agrees_with_sorting():
    # the yardstick itself, against brute force
    for D, K in [(2, 7), (3, 5), (4, 4)]:
        pts = sorted(pins.enumerate_pyramid(D, K), key=pins.order_key)
        assert [pins.count_before(p, K) for p in pts] == list(range(len(pts)))


@pytest.mark.parametrize("D,K", [(3, 5), (4, 4), (5, 4)])
def test_the_1986_decoding_mistake_is_caught(D, K):
    # Sec. 2.5 / App. B.3: without the update of z after x_i = -j, points with a negative entry
    # that is not the last one decode wrongly; points whose only negative entry is the last one
    # still decode correctly.  Planted in the oracle (CPU) to show the checks above would fail.
    pts = sorted(pins.enumerate_pyramid(D, K), key=pins.order_key)
    bad = o.unrank(range(len(pts)), D, K, omit_negative_update=True).tolist()
    wrong = [p for p, b in zip(pts, bad) if list(p) != b]
    assert wrong, "the planted mistake went unnoticed"
    assert all(any(v < 0 for v in p[:-1]) for p in wrong)
    ok_last_negative = [p for p, b in zip(pts, bad) if all(v >= 0 for v in p[:-1])]
    assert all(list(p) == b for p, b in zip(pts, bad) if all(v >= 0 for v in p[:-1]))
    assert ok_last_negative


def test_rank_rejects_points_off_the_pyramid():
    with pytest.raises(ValueError):
        o.rank([[1, 2, 3]], 7)
    with pytest.raises(ValueError):
        o.unrank([pins.n_binomial(3, 5)], 3, 5)
