"""Pins for the oracle's size table N(D,K), index width and choice of K."""
import json
import os

import pytest

from oracle import pvq_oracle as o
from tests import pins

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_values.json")))


def test_paper_worked_example_size():
    g = GOLD["pyramid_2_7"]
    assert o.size_table(g["D"], g["K"])[g["D"]][g["K"]] == g["size"]
    # codes run over [first_code, last_code] -> the index needs bit_length(last_code) bits
    assert o.index_bits(g["D"], g["K"]) == g["last_code"].bit_length()


@pytest.mark.parametrize("D,K", [(1, 1), (1, 5), (2, 3), (2, 7), (3, 4), (4, 3), (4, 5), (5, 3), (6, 2)])
def test_table_equals_brute_force_count(D, K):
    tab = o.size_table(D, K)
    for d in range(1, D + 1):
        for k in range(0, K + 1):
            if (2 * k + 1) ** d > 400000:
                continue
            assert tab[d][k] == len(pins.enumerate_pyramid(d, k)), (d, k)


def test_boundary_values():
    tab = o.size_table(6, 9)
    assert all(tab[d][0] == 1 for d in range(7))          # N(D,0) = 1 for all D >= 0
    assert all(tab[0][k] == 0 for k in range(1, 10))      # N(0,K) = 0 for K >= 1


@pytest.mark.parametrize("D,K", [(8, 16), (16, 33), (32, 60), (12, 40), (64, 20)])
def test_table_equals_closed_forms(D, K):
    tab = o.size_table(D, K)
    for d in range(1, D + 1):
        for k in range(1, K + 1):
            assert tab[d][k] == pins.n_binomial(d, k), (d, k)
    for d in (1, 2, 3, D // 2, D - 1, D):
        for k in (1, 2, K // 2, K - 1, K):
            assert tab[d][k] == pins.n_hypergeometric(d, k), (d, k)


def test_small_closed_forms_and_asymmetry():
    tab = o.size_table(9, 12)
    for k in range(1, 13):
        assert tab[1][k] == 2
        assert tab[2][k] == 4 * k
        assert tab[3][k] == 4 * k * k + 2
    for d in range(1, 10):
        assert tab[d][1] == 2 * d
        assert tab[d][2] == 2 * d * d
    assert tab[3][5] != tab[5][3]                          # N is not symmetric in (D,K)


@pytest.mark.parametrize("D,budget", [(8, 24), (16, 52), (32, 104), (8, 16), (16, 40), (4, 13)])
def test_max_k_is_largest_that_fits(D, budget):
    K = o.max_k(D, budget)
    assert (pins.n_binomial(D, K) - 1).bit_length() <= budget
    assert (pins.n_binomial(D, K + 1) - 1).bit_length() > budget
    assert o.index_bits(D, K) == (pins.n_binomial(D, K) - 1).bit_length()


def test_index_bits_exact_at_power_of_two_sizes():
    # N(2,8) = 32 is a power of two: codes 0..31 need 5 bits, not 6 (a float log2 or an
    # off-by-one in the width would fail here); N(1,k) = 2 needs 1 bit.
    assert o.index_bits(2, 8) == 5
    assert o.index_bits(1, 9) == 1
    assert o.index_bits(2, 16) == 6


def test_oracle_integer_width_overflow_is_reported():
    with pytest.raises(OverflowError):
        o.size_table(200, 400)
