"""The C library loads, exports every symbol its header declares, and its host-only entry points
(no GPU needed) agree with independent arithmetic.  No kernel is launched here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2410_16926_amd as pvq
from tests import pins

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "pvq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pvq_[a-z0-9_]+)\s*\(", text)))


def test_header_and_library_agree_on_the_exports():
    names = declared_functions()
    assert sorted(pvq.EXPORTS) == names
    L = pvq.lib()
    for n in names:
        assert getattr(L, n) is not None


def test_diagnostics_are_declared_apart_from_the_public_header():
    text = open(os.path.join(ROOT, "paper_2410_16926_amd", "csrc", "pvq_diagnostics.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    assert sorted(set(re.findall(r"\b(pvq_[a-z0-9_]+)\s*\(", text))) == sorted(pvq.DIAGNOSTICS)
    assert not set(pvq.DIAGNOSTICS) & set(declared_functions())
    for n in pvq.DIAGNOSTICS:
        assert getattr(pvq.lib(), n) is not None


def test_process_wide_settings_of_the_diagnostics():
    # the two setters keep their number in host memory: they run without a GPU
    for setter, default in ((pvq.pvq_correct_set_front_tiles, 1536), (pvq.pvq_decode_set_table_decoder_min_groups, 1572864)):
        assert setter(7) == default
        assert setter(default) == 7
        with pytest.raises(pvq.PvqError):
            setter(-1)
        assert setter(default) == default              # a refused value changes nothing


def test_status_strings():
    L = pvq.lib()
    for code in (0, -1, -2, -3, -4, -5):
        assert L.pvq_strerror(code)
    assert L.pvq_strerror(-99) == b"unknown status"


@pytest.mark.parametrize("D,K", [(2, 7), (8, 16), (16, 33), (32, 60), (64, 40), (3, 1), (5, 0), (128, 187), (128, 382)])
def test_pvq_count(D, K):
    n, bits = pvq.pvq_count(D, K)
    assert n == pins.n_binomial(D, K)
    assert bits == (n - 1).bit_length()


def test_pvq_count_rejects_what_it_cannot_hold():
    with pytest.raises(pvq.PvqError) as e:
        pvq.pvq_count(256, 1024)
    assert e.value.status == -2
    with pytest.raises(pvq.PvqError) as e:
        pvq.pvq_count(0, 3)
    assert e.value.status == -1


@pytest.mark.parametrize("D,budget,K", [(8, 24, 16), (16, 52, 33), (32, 104, 60), (128, 384, 187), (64, 192, 96)])
def test_pvq_max_k_on_the_measured_settings(D, budget, K):
    assert pvq.pvq_max_k(D, budget) == K


@pytest.mark.parametrize("D,budget", [(4, 13), (8, 16), (16, 40), (24, 77), (128, 255), (256, 255), (128, 511), (64, 300)])
def test_pvq_max_k_is_the_largest_that_fits(D, budget):
    K = pvq.pvq_max_k(D, budget)
    assert (pins.n_binomial(D, K) - 1).bit_length() <= budget < (pins.n_binomial(D, K + 1) - 1).bit_length()


def test_pvq_max_k_errors():
    with pytest.raises(pvq.PvqError):
        pvq.pvq_max_k(8, 0)
    with pytest.raises(pvq.PvqError) as e:
        pvq.pvq_max_k(8, 3)          # N(8,1) = 16 needs 4 bits
    assert e.value.status == -2


@pytest.mark.parametrize("D,G,bits", [(4, 4, 2), (8, 512, 8), (8, 1024, 2), (16, 256, 4)])
def test_pvq_beta_tables_hit_their_quantiles(D, G, bits):
    from fractions import Fraction
    from math import comb
    edges, centers = pvq.pvq_beta_tables(D, G, bits)
    n = 1 << bits
    a, b = D // 2, D * (G - 1) // 2

    def cdf(x):  # binomial tail, exact rationals (not the series the library sums)
        m = a + b - 1
        xf = Fraction(float(x))
        return float(1 - sum(comb(m, j) * xf ** j * (1 - xf) ** (m - j) for j in range(a)))

    assert np.all(np.diff(edges) > 0)
    for j in sorted({0, n // 2 - 1, n - 2} & set(range(n - 1))):
        assert abs(cdf(edges[j]) - (j + 1) / n) < 1e-10
    for q in sorted({0, n // 2, n - 1}):
        assert abs(cdf(centers[q]) - (q + 0.5) / n) < 1e-10


def test_pvq_beta_tables_errors():
    with pytest.raises(pvq.PvqError):
        pvq.pvq_beta_tables(7, 16, 2)     # odd D
    with pytest.raises(pvq.PvqError):
        pvq.pvq_beta_tables(8, 16, 3)     # unsupported width
    with pytest.raises(pvq.PvqError):
        pvq.pvq_beta_tables(8, 1, 2)      # a single group has no distribution


@pytest.mark.parametrize("K", [1, 2, 5, 9, 13, 16, 17])
def test_table_driven_decoder_tables_replay_every_index(K):
    # host logic: the pair/bucket tables the D=8 kernels walk, replayed on the CPU over ALL indices
    # of P(8,K) against the plain coordinate-by-coordinate decoding
    assert pvq.pvq_fast_tables_selftest(K) == 0


def test_table_driven_decoder_limits():
    with pytest.raises(pvq.PvqError) as e:
        pvq.pvq_fast_tables_selftest(40)
    assert e.value.status == -2


def test_pvq_correct_work_bytes():
    # host-only helper: two buffers of 128 float32 per row (the t values of a panel), errors for what cannot be
    import ctypes as C
    n = C.c_size_t(0)
    assert pvq.lib().pvq_correct_work_bytes(1000, C.byref(n)) == 0 and n.value == 1000 * 256 * 4
    assert pvq.lib().pvq_correct_work_bytes(0, C.byref(n)) == 0 and n.value == 0
    assert pvq.lib().pvq_correct_work_bytes(-1, C.byref(n)) == -1
    assert pvq.lib().pvq_correct_work_bytes(5, None) == -1


@pytest.mark.parametrize("D,K,schedule", [(16, 33, (8, 0)), (32, 60, (15, 6)), (16, 16, (8, 0)), (8, 40, (0, 0)),
                                          (32, 9, (12, 0)), (32, 25, (15, 6)), (16, 60, (0, 0)), (8, 127, (0, 0)),
                                          (16, 1, (0, 0)), (32, 2, (0, 0)), (8, 3, (0, 0))])
def test_one_probe_per_coordinate_decoder_replays_sampled_indices(D, K, schedule):
    # host logic: the cumulative rows and guess tables the D = 16 / 32 kernels walk, replayed on the CPU over the
    # ends of the index range and seeded random indices against the magnitude-by-magnitude decoding; the width
    # schedule (64-bit integers down to 9 dimensions and 32-bit ones from 8 on, for the 52-bit setting)
    bad, sched, nbytes = pvq.pvq_walk_tables_selftest(D, K, seed=D * 1000 + K, count=60000)
    assert bad == 0
    assert sched == schedule
    assert 0 < nbytes and nbytes % 16 == 0


def test_one_probe_per_coordinate_decoder_limits():
    with pytest.raises(pvq.PvqError) as e:
        pvq.pvq_walk_tables_selftest(64, 10)
    assert e.value.status == -2
    with pytest.raises(pvq.PvqError) as e:
        pvq.pvq_walk_tables_selftest(32, 127)       # index beyond 128 bits
    assert e.value.status == -2
