"""Pins for the oracle's error correction (Sec. 3.3 Step 6): the update it applies is checked against the
section's equation evaluated with explicit inverses of Hessian sub-matrices in float64, against the
stationarity of the proxy loss (Sec. 2.1) that defines it, and on the cases where it must do nothing."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import pvq_oracle as oracle


def make_case(rows, cols, seed, sigma=0.02):
    W = si.gaussian_weights(rows, cols, sigma, seed=seed, rotate=False, bf16=False)
    H, U = si.calibration_hessian(cols, 4 * cols, seed + 1)
    return np.asarray(W, dtype=np.float32), H, U


@pytest.mark.parametrize("D,K,cols", [(8, 16, 64), (4, 6, 24), (16, 33, 64), (8, 5, 40)])
@pytest.mark.parametrize("amplitude", ["l2", "ls"])
def test_update_is_the_sections_equation(D, K, cols, amplitude):
    # Given the errors e_g = (values quantised at step g) - (their quantised values), the procedure is
    # linear: a column of a later group h ends as its original value minus, for every g < h,
    # e_g (A_gg)^-1 A_g,h with A the inverse of the Hessian restricted to the columns from g on.
    W0, H, U = make_case(5, cols, 300 + D + K)
    Wq, Q = oracle.correct(W0, U, D, K, amplitude=amplitude)
    G = cols // D
    E = Wq.astype(np.float64) - Q.astype(np.float64)
    expect = W0.astype(np.float64).copy()
    for g in range(G - 1):
        A = np.linalg.inv(H[g * D:, g * D:])
        M = np.linalg.solve(A[:D, :D], A[:D, D:])          # D x remaining columns
        expect[:, (g + 1) * D:] -= E[:, g * D:(g + 1) * D] @ M
    scale = np.abs(W0).max()
    assert np.abs(Wq - expect).max() <= 2e-5 * scale * G


def test_update_makes_the_proxy_loss_stationary():
    # two groups: after the first is quantised, the change d of the second must make the gradient of
    # Tr(Delta H Delta^T) with respect to d vanish, Delta = [q_0 - w_0, d]   (Sec. 2.1, Sec. 3.3 Step 6)
    D, K = 8, 16
    W0, H, U = make_case(7, 2 * D, 411)
    Wq, Q = oracle.correct(W0, U, D, K)
    delta = np.concatenate([Q[:, :D].astype(np.float64) - W0[:, :D], Wq[:, D:].astype(np.float64) - W0[:, D:]], axis=1)
    grad = (delta @ H)[:, D:]
    ref = np.abs(delta[:, :D] @ H[:D, D:]).max()            # what the gradient would be without the update
    assert ref > 0 and np.abs(grad).max() <= 1e-4 * ref
    # and any other change of the second group is worse
    rng = np.random.default_rng(5)
    base = np.einsum("ri,ij,rj->", delta, H, delta)
    for _ in range(20):
        other = delta.copy()
        other[:, D:] += 1e-3 * np.abs(delta).max() * rng.standard_normal((7, D))
        assert np.einsum("ri,ij,rj->", other, H, other) > base


def test_uncorrelated_inputs_leave_the_weights_alone():
    # a diagonal Hessian couples no columns: nothing is handed on, bit for bit, and the quantised values are
    # those of plain encoding and decoding
    D, K, cols = 8, 16, 64
    W0, _, _ = make_case(6, cols, 512)
    rng = np.random.default_rng(9)
    U = np.diag(rng.uniform(0.5, 2.0, cols)).astype(np.float32)
    Wq, Q = oracle.correct(W0, U, D, K)
    assert np.array_equal(Wq.view(np.uint32), W0.view(np.uint32))
    ref, _, _ = oracle.decode(oracle.encode(W0, D, K), None)
    assert np.abs(Q - ref).max() <= 1e-6 * np.abs(ref).max()


@pytest.mark.parametrize("amplitude", ["l2", "ls"])
def test_encoding_the_result_gives_the_values_used_in_the_errors(amplitude):
    # the returned matrix holds what was quantised at every step: encoding and decoding it gives Q
    D, K, cols = 8, 16, 128
    W0, _, U = make_case(9, cols, 613)
    Wq, Q = oracle.correct(W0, U, D, K, amplitude=amplitude)
    ref, _, _ = oracle.decode(oracle.encode(Wq, D, K, amplitude=amplitude), None)
    assert np.abs(Q - ref).max() <= 1e-6 * np.abs(ref).max()


def test_correction_lowers_the_proxy_loss():
    # Sec. 2.1's loss Tr((W - W_hat) H (W - W_hat)^T) of the corrected quantisation against plain
    # quantisation of the same matrix, on strongly correlated inputs
    D, K, cols = 8, 16, 256
    W0, H, U = make_case(24, cols, 714)
    _, Q = oracle.correct(W0, U, D, K)
    plain, _, _ = oracle.decode(oracle.encode(W0, D, K), None)

    def loss(What):
        d = W0.astype(np.float64) - What
        return np.einsum("ri,ij,rj->", d, H, d)

    assert loss(Q.astype(np.float64)) < 0.7 * loss(plain)


def test_threads_do_not_change_the_result():
    D, K, cols = 8, 16, 64
    W0, _, U = make_case(11, cols, 815)
    a, qa = oracle.correct(W0, U, D, K, nthreads=1)
    b, qb = oracle.correct(W0, U, D, K, nthreads=4)
    assert np.array_equal(a.view(np.uint32), b.view(np.uint32)) and np.array_equal(qa.view(np.uint32), qb.view(np.uint32))


def test_the_synthetic_hessian_and_its_factor():
    # the input recipe: H symmetric positive definite with strongly coupled neighbouring channels, U upper
    # triangular with a positive diagonal and U^T U = H^-1 (up to its rounding to float32)
    H, U = si.calibration_hessian(96, 400, 916)
    assert np.allclose(H, H.T) and np.linalg.eigvalsh(H).min() > 0
    corr = H[np.arange(95), np.arange(1, 96)] / np.sqrt(np.diag(H)[:-1] * np.diag(H)[1:])
    assert np.median(corr) > 0.7
    assert U.dtype == np.float32 and np.array_equal(U, np.triu(U)) and np.diag(U).min() > 0
    U64 = U.astype(np.float64)
    assert np.abs(U64.T @ U64 @ H - np.eye(96)).max() < 1e-4
