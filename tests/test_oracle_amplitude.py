"""Pins for the oracle's amplitude path: Beta quantile tables, codes, dequantised amplitudes."""
import json
import os
from fractions import Fraction
from math import comb

import numpy as np
import pytest

import synth_inputs as si
from oracle import pvq_oracle as o

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_values.json")))


def beta_cdf_integer(x: float, a: int, b: int) -> float:
    """CDF of Beta(a,b) for integer a, b as the binomial tail  P[Bin(a+b-1, x) >= a], summed
    exactly in rationals.  Independent of scipy's incomplete-beta routine."""
    n = a + b - 1
    xf = Fraction(x)
    lower = sum(comb(n, j) * xf ** j * (1 - xf) ** (n - j) for j in range(a))
    return float(1 - lower)


def test_beta_2_6_example_of_the_paper():
    g = GOLD["beta_example"]
    assert (g["D"] / 2, g["D"] * (g["G"] - 1) / 2) == (g["a"], g["b"])
    for bits in (1, 2, 3, 4):
        edges, centers = o.beta_tables(g["D"], g["G"], bits)
        n = 1 << bits
        # closed form for Beta(2,6): CDF(x) = 1 - (1-x)^7 - 7 x (1-x)^6
        cdf = lambda x: 1 - (1 - x) ** 7 - 7 * x * (1 - x) ** 6
        assert np.allclose([cdf(e) for e in edges], np.arange(1, n) / n, atol=1e-12)
        assert np.allclose([cdf(c) for c in centers], (np.arange(n) + 0.5) / n, atol=1e-12)


@pytest.mark.parametrize("D,G,bits", [(8, 64, 2), (8, 512, 8), (8, 1024, 2), (16, 256, 4), (8, 3584, 2)])
def test_tables_hit_their_quantiles_exactly(D, G, bits):
    edges, centers = o.beta_tables(D, G, bits)
    n = 1 << bits
    a, b = D // 2, D * (G - 1) // 2
    assert np.all(np.diff(edges) > 0) and np.all(np.diff(centers) > 0)
    assert np.all(centers[:-1] < edges) and np.all(edges < centers[1:])
    pick = sorted(set([0, 1, n // 2 - 1, n - 2]) & set(range(n - 1)))
    for j in pick:
        assert abs(beta_cdf_integer(float(edges[j]), a, b) - (j + 1) / n) < 1e-9
    for q in sorted(set([0, n // 2, n - 1])):
        assert abs(beta_cdf_integer(float(centers[q]), a, b) - (q + 0.5) / n) < 1e-9


def test_codes_are_floor_cdf_times_levels_and_uniform_on_gaussian_rows():
    D, K, bits = 8, 16, 2
    rows, cols = 64, 4096
    G = cols // D
    W = si.gaussian_weights(rows, cols, 0.015, seed=si.BASE_SEED + 31)
    edges, centers = o.beta_tables(D, G, bits)
    enc = o.encode(W, D, K, bits, edges)
    codes = np.array(o.unpack_fields(enc.scale, G, bits))
    # the definition: floor(CDF(u) 2^b) with u = ||w_g||^2 / ||w_row||^2, here in float64
    W64 = W.astype(np.float64).reshape(rows, G, D)
    ss = (W64 ** 2).sum(axis=2)
    u = ss / ss.sum(axis=1, keepdims=True)
    from scipy.stats import beta
    want = np.minimum(np.floor(beta.cdf(u, D / 2, D * (G - 1) / 2) * 4), 3).astype(int)
    # float32 vs float64 u may disagree only within rounding distance of an edge
    near_edge = np.min(np.abs(u[:, :, None] - edges[None, None, :]), axis=2) < 1e-6 * u
    assert np.all((codes == want) | near_edge)
    assert np.mean(codes != want) < 1e-3
    # under the model every code is equally likely (Sec. 3.4)
    occ = np.bincount(codes.ravel(), minlength=4) / codes.size
    assert np.all(np.abs(occ - 0.25) < 0.01), occ
    # the stored row normaliser is the row's sum of squares
    assert np.allclose(enc.rowss, ss.sum(axis=1), rtol=1e-5)


def test_extreme_amplitudes_take_the_end_codes():
    D, K, bits, G = 8, 16, 2, 32
    rng = np.random.default_rng(5)
    W = rng.standard_normal((1, G * D)).astype(np.float32)
    W[0, :D] *= 1e-4          # a vanishing group -> code 0
    W[0, D:2 * D] *= 50       # a dominating group -> top code
    edges, _ = o.beta_tables(D, G, bits)
    enc = o.encode(W, D, K, bits, edges)
    codes = o.unpack_fields(enc.scale, G, bits)[0]
    assert codes[0] == 0 and codes[1] == 3


def test_dequantised_amplitude_is_sqrt_center_times_row_normaliser():
    D, K, bits = 8, 16, 4
    rows, cols = 8, 512
    G = cols // D
    W = si.gaussian_weights(rows, cols, 0.02, seed=si.BASE_SEED + 32)
    edges, centers = o.beta_tables(D, G, bits)
    enc = o.encode(W, D, K, bits, edges)
    Wd, _, _ = o.decode(enc, centers)
    codes = np.array(o.unpack_fields(enc.scale, G, bits))
    amp = np.sqrt((Wd.reshape(rows, G, D) ** 2).sum(axis=2))
    want = np.sqrt(centers[codes] * enc.rowss.astype(np.float64)[:, None])
    assert np.allclose(amp, want, rtol=1e-12)
    # and it approximates the true group norm to within the bin width
    true = np.sqrt((W.astype(np.float64).reshape(rows, G, D) ** 2).sum(axis=2))
    assert np.median(np.abs(amp - true) / true) < 0.08


# ---- least-squares amplitude (Sec. 3.3 Step 4) ------------------------------------------------

def _groups(n, D, seed):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((n, D)) * 0.02).astype(np.float32)


@pytest.mark.parametrize("D,K", [(8, 16), (16, 33), (32, 60), (4, 3)])
def test_ls_amplitude_is_the_least_squares_solution(D, K):
    # s minimises ||w - s d||_2 for the unit direction d = y/||y||_2: compare with a least-squares solve
    for w in _groups(200, D, seed=11 + D):
        y, _ = o.quantize_group(w, K)
        d = y.astype(np.float64) / np.linalg.norm(y.astype(np.float64))
        s_ref = np.linalg.lstsq(d[:, None], w.astype(np.float64), rcond=None)[0][0]
        s = o.ls_amplitude(w, y)
        assert abs(s - s_ref) <= 2e-6 * abs(s_ref) + 1e-12
        # it is the norm times the cosine of the angle between w and y, hence never above the norm
        wn = np.linalg.norm(w.astype(np.float64))
        assert s <= wn * (1 + 1e-6)
        assert abs(s - wn * float(d @ w.astype(np.float64)) / wn) <= 2e-6 * wn
        # and no other amplitude rebuilds the group better: not the norm, not the printed (inverted) ratio
        err = lambda a: np.linalg.norm(w.astype(np.float64) - a * d)
        assert err(s) <= err(wn) + 1e-12
        printed = float(y.astype(np.float64) @ y.astype(np.float64)) / float(y.astype(np.float64) @ w.astype(np.float64))
        assert err(s) <= err(printed * np.linalg.norm(y.astype(np.float64))) + 1e-12


def test_ls_amplitude_special_cases():
    # a group that lies exactly along a pyramid point: the amplitude is its norm
    y = np.array([3, -2, 0, 1, 0, -4, 5, 1], dtype=np.int32)
    w = (0.125 * y).astype(np.float32)
    yq, _ = o.quantize_group(w, int(np.abs(y).sum()))
    assert np.array_equal(yq, y)
    assert o.ls_amplitude(w, yq) == pytest.approx(float(np.linalg.norm(w.astype(np.float64))), rel=1e-6)
    # one-hot direction: the amplitude is that coordinate of the group
    w = np.array([0.5, 0.01, -0.02, 0.0, 0.0, 0.0, 0.0, 0.0], dtype=np.float32)
    y = np.array([1, 0, 0, 0, 0, 0, 0, 0], dtype=np.int32)
    assert o.ls_amplitude(w, y) == np.float32(0.5)
    # zero group -> point (0,...,0,+K), amplitude 0
    z = np.zeros(8, dtype=np.float32)
    yz, _ = o.quantize_group(z, 16)
    assert o.ls_amplitude(z, yz) == 0.0


@pytest.mark.parametrize("bits", [0, 2])
def test_ls_amplitude_in_the_matrix_encoder(bits):
    # the matrix encoder stores exactly the per-group values, and decoding with them rebuilds the
    # matrix at least as well as with the norms
    D, K = 8, 16
    W = si.gaussian_weights(24, 512, 0.02, seed=5)
    G = W.shape[1] // D
    edges, centers = o.beta_tables(D, G, bits) if bits else (None, None)
    e_ls = o.encode(W, D, K, bits, edges, amplitude="ls")
    e_l2 = o.encode(W, D, K, bits, edges, amplitude="l2")
    assert np.array_equal(e_ls.index, e_l2.index) and np.array_equal(e_ls.pulses, e_l2.pulses)
    amps = np.array([[o.ls_amplitude(W[r, g * D:(g + 1) * D], e_ls.pulses[r, g * D:(g + 1) * D].astype(np.int32))
                      for g in range(G)] for r in range(W.shape[0])], dtype=np.float32)
    if bits == 0:
        assert np.array_equal(e_ls.scale, amps)
        d_ls, _, _ = o.decode(e_ls)
        d_l2, _, _ = o.decode(e_l2)
        assert np.linalg.norm(W - d_ls) < np.linalg.norm(W - d_l2)
    else:
        ss = amps * amps
        # row normaliser = pair-level sum of the squared amplitudes; codes count the edges below ss/rowss
        for r in range(W.shape[0]):
            buf = ss[r].copy()
            n = buf.size
            while n > 1:
                half = n // 2
                nxt = buf[0:2 * half:2] + buf[1:2 * half:2]
                if n % 2:
                    nxt = np.append(nxt, buf[n - 1])
                buf = nxt.astype(np.float32)
                n = buf.size
            assert e_ls.rowss[r] == buf[0]
            u = (ss[r] / e_ls.rowss[r]).astype(np.float32)
            want = (np.asarray(edges, dtype=np.float64).astype(np.float32)[None, :] <= u[:, None]).sum(axis=1)
            got = o.unpack_fields(e_ls.scale[r:r + 1], G, bits)[0]
            assert np.array_equal(np.array(got), want)
