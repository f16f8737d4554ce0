"""Pins for the oracle's direction quantiser (projection to the l1 ball, rounding, +-1 repair)."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import pvq_oracle as o
from tests import pins


def _objective(w, p, K):
    """Squared Euclidean distance from the projected point t = K w / ||w||_1 to p, float64."""
    w = np.asarray(w, dtype=np.float64)
    t = K * w / np.abs(w).sum()
    return float(((t - np.asarray(p, dtype=np.float64)) ** 2).sum())


@pytest.mark.parametrize("D,K", [(2, 7), (3, 5), (4, 4), (4, 6), (5, 4), (6, 3)])
def test_quantiser_is_the_exhaustive_nearest_point(D, K):
    rng = np.random.default_rng(D * 100 + K)
    P = np.array(pins.enumerate_pyramid(D, K), dtype=np.float64)
    for trial in range(120):
        if trial % 3 == 0:
            w = rng.standard_normal(D)
        elif trial % 3 == 1:
            w = rng.laplace(size=D)
        else:
            w = rng.standard_normal(D) * (rng.random(D) < 0.6)
            if not np.any(w):
                w[0] = 1.0
        w = w.astype(np.float32)
        y, _ = o.quantize_group(w, K)
        t = K * w.astype(np.float64) / np.abs(w.astype(np.float64)).sum()
        best = ((P - t[None, :]) ** 2).sum(axis=1).min()
        assert _objective(w, y, K) <= best + 1e-5, (w, y)


def test_stated_tie_breaks():
    # rounding: to nearest, ties to even; repair: biggest deviation, lowest coordinate on ties
    cases = [
        ([1, 1, 1, 1], 2, [1, 1, 0, 0]),            # t = .5 each -> 0; raise two, lowest first
        ([3, 3, 3, 3], 6, [1, 1, 2, 2]),            # t = 1.5 each -> 2; lower two, lowest first
        ([2.5, 2.5, 1, 0], 6, [3, 2, 1, 0]),        # t = 2.5 -> 2 (even); raise coordinate 0
        ([-2.5, 2.5, -1, 0], 6, [-3, 2, -1, 0]),    # signs follow w
        ([0.5, 1.5, 2.5, 3.5], 8, [0, 2, 2, 4]),    # already sums to K after half-even rounding
        ([1, 0, 0, 0], 5, [5, 0, 0, 0]),
        ([0, 0, 0, -1], 5, [0, 0, 0, -5]),
    ]
    for w, K, want in cases:
        y, _ = o.quantize_group(np.array(w, dtype=np.float32), K)
        assert y.tolist() == want, (w, K, y)


def test_zero_and_vanishing_groups_go_to_index_zero():
    for D, K in [(8, 16), (16, 33)]:
        y, ss = o.quantize_group(np.zeros(D, dtype=np.float32), K)
        assert y.tolist() == [0] * (D - 1) + [K] and ss == 0.0
        assert o.rank([y], K) == [0]
        y, _ = o.quantize_group(np.full(D, -0.0, dtype=np.float32), K)
        assert y.tolist() == [0] * (D - 1) + [K]
        tiny = np.zeros(D, dtype=np.float32)
        tiny[2] = np.float32(1e-45)                  # K / ||w||_1 overflows
        y, _ = o.quantize_group(tiny, K)
        assert y.tolist() == [0] * (D - 1) + [K]


@pytest.mark.parametrize("D,K", [(16, 33), (64, 40), (128, 187)])
def test_no_single_pulse_move_comes_closer(D, K):
    """The objective sum (y_i - t_i)^2 is separable and convex and the constraint is one sum, so a
    point that no move of one pulse from a coordinate to another improves is the nearest point of the
    pyramid (exchange optimality).  Checked in float64 on the projected point the quantiser uses."""
    rng = np.random.default_rng(41 + D)
    groups = np.concatenate([
        rng.standard_normal((120, D)).astype(np.float32),
        rng.standard_t(2.5, (60, D)).astype(np.float32),          # heavy tails, as activations have
        si.adversarial_groups(60, D, seed=5 + D),
    ])
    for w in groups:
        y, _ = o.quantize_group(w, K)
        a = np.abs(w)
        buf = a.copy()
        n = D
        while n > 1:                       # the float32 pair-level sum the projection divides by
            buf[: n // 2] = buf[0:n:2] + buf[1:n:2]
            n //= 2
        l1 = buf[0]
        if not l1 > 0 or not np.isfinite(np.float32(K) / l1):
            continue
        t = (a * (np.float32(K) / l1)).astype(np.float64)
        m = np.abs(y).astype(np.float64)
        assert m.sum() == K
        gain_take = np.where(m > 0, (m - t) ** 2 - (m - 1 - t) ** 2, -np.inf)   # improvement from removing a pulse
        cost_give = (m + 1 - t) ** 2 - (m - t) ** 2                               # cost of adding one
        i = int(np.argmax(gain_take))
        cg = cost_give.copy()
        cg[i] = np.inf
        assert gain_take[i] - cg.min() <= 1e-9, (i, gain_take[i], cg.min())


@pytest.mark.parametrize("D,K", [(8, 16), (16, 33), (32, 60), (128, 187)])
def test_invariants_on_gaussian_and_adversarial_groups(D, K):
    rng = np.random.default_rng(7 + D)
    groups = np.concatenate([
        rng.standard_normal((600 if D <= 32 else 150, D)).astype(np.float32) * np.float32(0.02),
        si.adversarial_groups(400 if D <= 32 else 100, D, seed=11 + D),
    ])
    for w in groups:
        y, ss = o.quantize_group(w, K)
        assert np.abs(y).sum() == K
        l1 = np.abs(w.astype(np.float64)).sum()
        if l1 == 0:
            continue
        assert np.all((y == 0) | (np.sign(y) == np.sign(w))), (w, y)
        t = K * np.abs(w.astype(np.float64)) / l1
        assert np.all(np.abs(np.abs(y) - t) < 1.5 + 1e-5)
        assert abs(float(ss) - float((w.astype(np.float64) ** 2).sum())) <= 1e-6 * float(ss) + 1e-37


@pytest.mark.parametrize("D,K", [(8, 16), (32, 60)])
def test_power_of_two_scaling_leaves_the_point_unchanged(D, K):
    # float32 products and quotients scale exactly by powers of two (away from under/overflow),
    # so the direction must not depend on the group's scale
    rng = np.random.default_rng(3)
    for _ in range(200):
        w = rng.standard_normal(D).astype(np.float32)
        y0, _ = o.quantize_group(w, K)
        for e in (-30, -7, 9, 40):
            y1, _ = o.quantize_group(w * np.float32(2.0 ** e), K)
            assert y0.tolist() == y1.tolist()


def test_sum_of_squares_follows_the_pairwise_order():
    # ((a0+a1)+(a2+a3)) with each square rounded first: distinguishable from a left-to-right sum
    w = np.array([1.0, 2.0 ** -12, 2.0 ** -12, 2.0 ** -12], dtype=np.float32)
    _, ss = o.quantize_group(w, 4)
    sq = (w * w).astype(np.float32)
    want = np.float32(np.float32(sq[0] + sq[1]) + np.float32(sq[2] + sq[3]))
    left = np.float32(np.float32(np.float32(sq[0] + sq[1]) + sq[2]) + sq[3])
    assert ss == want
    assert want != left      # the case does tell the two orders apart


@pytest.mark.parametrize("D,K", [(8, 16), (16, 33), (32, 60)])
def test_repair_equals_adjusting_the_m_largest_deviations(D, K):
    """Host-logic check behind the GPU kernel's selection: no coordinate is adjusted twice, so the
    sequential repair is the same as adjusting the m = |sum - K| coordinates of largest deviation
    (lowest coordinate first on ties).  Restated here in numpy float32 and compared with the oracle."""
    rng = np.random.default_rng(5 + D)
    groups = np.concatenate([
        rng.standard_normal((1500, D)).astype(np.float32),
        si.bf16_bits_to_f32(si.f32_to_bf16_bits(rng.standard_normal((1500, D)).astype(np.float32))),
        si.adversarial_groups(800, D, seed=23 + D),
    ])
    for w in groups:
        a = np.abs(w)
        buf = a.copy()
        n = D
        while n > 1:
            buf[: n // 2] = buf[0:n:2] + buf[1:n:2]
            n //= 2
        l1 = buf[0]
        if not l1 > 0:
            continue
        g = np.float32(K) / l1
        if not np.isfinite(g):
            continue
        t = a * g
        y = np.rint(t).astype(np.int64)
        m = int(y.sum()) - K
        if m > 0:
            dev = np.where(y > 0, y.astype(np.float32) - t, -np.inf)
            order = np.lexsort((np.arange(D), -dev))
            y[order[:m]] -= 1
        elif m < 0:
            dev = t - y.astype(np.float32)
            order = np.lexsort((np.arange(D), -dev))
            y[order[:-m]] += 1
        y = np.where(w < 0, -y, y)
        got, _ = o.quantize_group(w, K)
        assert got.tolist() == y.tolist(), (w, got, y)
        assert abs(m) <= D // 2
