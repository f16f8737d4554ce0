"""Seeded synthetic inputs, shared by the tests, the smoke check and the benchmark.

Holds none of the quantiser's arithmetic: only random weight matrices with the shapes and
statistics of the workloads (arXiv 2410.16926 quantises LLM weight matrices after a random
Hadamard rotation, Sec. 2.3 "Hadamard coherence processing" and Sec. 3.3 Step 1; trained
weights are not available here, so i.i.d. Gaussian matrices followed by that rotation stand in,
which is also the paper's own model of rotated weights, Theorem 3.1), activations, and the
float32 <-> bf16 bit conversions numpy lacks.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 20241016

# name -> (rows, cols) of a Llama-3-70B decoder layer's weight matrices (out x in)
LLAMA3_70B_SHAPES = {
    "q": (8192, 8192), "k": (1024, 8192), "v": (1024, 8192), "o": (8192, 8192),
    "gate": (28672, 8192), "up": (28672, 8192), "down": (8192, 28672),
}
LLAMA3_8B_UP = (14336, 4096)


def f32_to_bf16_bits(a) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u >> 16) & 1            # finite inputs only: the uint32 sum below cannot wrap for them
    r += np.uint32(0x7FFF)
    r += u
    r >>= 16
    return r.astype(np.uint16)


def bf16_bits_to_f32(b) -> np.ndarray:
    """bf16 bit patterns -> float32 with the same value."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def _fwht_rows(a: np.ndarray, n: int) -> None:
    """In-place unnormalised Walsh-Hadamard transform of every length-n block of each row."""
    rows, cols = a.shape
    h = 1
    while h < n:
        v = a.reshape(rows, cols // (2 * h), 2, h)
        x = v[:, :, 0, :].copy()
        v[:, :, 0, :] += v[:, :, 1, :]
        v[:, :, 1, :] = x - v[:, :, 1, :]
        h *= 2


def hadamard_rotate_rows(a: np.ndarray, seed: int) -> np.ndarray:
    """Randomised Hadamard rotation along the input dimension: x -> H diag(+-1) x / sqrt(n),
    applied to every row.  For a length that is not a power of two (28672 = 7 * 4096) the
    rotation is block diagonal with the largest power-of-two block that divides the length."""
    a = np.ascontiguousarray(a, dtype=np.float32).copy()
    cols = a.shape[1]
    n = cols & (-cols)  # largest power of two dividing cols
    signs = np.random.default_rng(seed).integers(0, 2, size=cols).astype(np.float32) * 2 - 1
    a *= signs[None, :]
    step = max(1, (1 << 26) // cols)  # bound the temporaries
    for r0 in range(0, a.shape[0], step):
        blk = a[r0:r0 + step]
        _fwht_rows(blk, n)
    a *= np.float32(1.0 / np.sqrt(n))
    return a


def gaussian_weights(rows: int, cols: int, sigma: float, seed: int, rotate: bool = True,
                     bf16: bool = False):
    """i.i.d. N(0, sigma^2) float32, then the randomised Hadamard rotation along each row.
    Returns float32 values; with bf16=True also rounds to bf16 and returns
    (float32 values equal to the bf16 numbers, uint16 bit patterns)."""
    rng = np.random.default_rng(seed)
    w = rng.standard_normal((rows, cols), dtype=np.float32) * np.float32(sigma)
    if rotate:
        w = hadamard_rotate_rows(w, seed + 100)
    if bf16:
        bits = f32_to_bf16_bits(w)
        return bf16_bits_to_f32(bits), bits
    return w


def activations(batch: int, cols: int, seed: int):
    """x ~ N(0,1) rounded to bf16: (float32 values, uint16 bit patterns), [batch][cols]."""
    rng = np.random.default_rng(seed + 200)
    x = rng.standard_normal((batch, cols), dtype=np.float32)
    bits = f32_to_bf16_bits(x)
    return bf16_bits_to_f32(bits), bits


def activation_matrix(tokens: int, hidden: int, seed: int, rotate: bool = True, bf16: bool = True):
    """Stand-in for a batch of transformer activations [tokens][hidden]: i.i.d. N(0,1) with a few
    channels (1 in 128, the same for every token) carrying 20x the magnitude and a per-token scale,
    log-normal over tokens; then, as the method does before quantising (Sec. 3.3 Step 1), the randomised
    Hadamard rotation along each row, which spreads the outlier channels.  With bf16=True returns
    (float32 values equal to the bf16 numbers, uint16 bit patterns), else float32."""
    rng = np.random.default_rng(seed + 300)
    x = rng.standard_normal((tokens, hidden), dtype=np.float32)
    outliers = rng.choice(hidden, size=max(1, hidden // 128), replace=False)
    x[:, outliers] *= np.float32(20.0)
    x *= np.exp(rng.standard_normal((tokens, 1)) * 0.5).astype(np.float32)
    if rotate:
        x = hadamard_rotate_rows(x, seed + 400)
    if bf16:
        bits = f32_to_bf16_bits(x)
        return bf16_bits_to_f32(bits), bits
    return x


def calibration_hessian(cols: int, samples: int, seed: int, damp: float = 0.01):
    """A layer-wise Hessian H = X^T X / samples of synthetic calibration activations (Sec. 2.1: the
    expectation of x x^T over a calibration set, which is not available here), float64 [cols][cols], and
    the factor that the error correction of Sec. 3.3 Step 6 takes as its input: U upper triangular with
    U^T U = H^-1, rounded once to float32.  The activations are Gaussian with correlated neighbouring
    channels (a first-order autoregression along the channel axis, coefficient 0.9) and a few channels of
    ten times the scale, a rough picture of the feature statistics of a transformer layer; `damp` times the
    mean diagonal is added to the diagonal, as is usual before factorising.  The factor comes from LAPACK
    routines (inverse, then Cholesky), as a caller of the library would make it."""
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((samples, cols))
    for c in range(1, cols):
        X[:, c] = 0.9 * X[:, c - 1] + np.sqrt(1.0 - 0.81) * X[:, c]
    loud = rng.choice(cols, size=max(1, cols // 64), replace=False)
    X[:, loud] *= 10.0
    H = X.T @ X / samples
    H[np.diag_indices(cols)] += damp * np.mean(np.diag(H))
    U = np.linalg.cholesky(np.linalg.inv(H)).T          # inv(H) = L L^T = U^T U with U = L^T
    return H, np.ascontiguousarray(U, dtype=np.float32)


def adversarial_groups(n_groups: int, D: int, seed: int) -> np.ndarray:
    """Groups built to sit on rounding ties and fix-up ties: small-integer and half-integer
    multiples of a power of two, repeated magnitudes, zeros, mixed signs, one-hot and all-zero
    groups.  float32 [n_groups][D]."""
    rng = np.random.default_rng(seed)
    out = np.zeros((n_groups, D), dtype=np.float32)
    for g in range(n_groups):
        kind = g % 8
        if kind == 0:      # half-integers: many exact .5 after projection
            v = rng.integers(0, 8, size=D) * 0.5
        elif kind == 1:    # few distinct magnitudes -> ties between coordinates
            v = rng.choice([0.25, 0.5, 1.0], size=D)
        elif kind == 2:    # all equal
            v = np.full(D, rng.choice([0.125, 1.0, 3.0]))
        elif kind == 3:    # one-hot
            v = np.zeros(D)
            v[rng.integers(0, D)] = rng.choice([1e-3, 1.0, 100.0])
        elif kind == 4:    # all zero
            v = np.zeros(D)
        elif kind == 5:    # bf16-rounded Gaussians (coarse mantissas -> exact ties happen)
            v = bf16_bits_to_f32(f32_to_bf16_bits(rng.standard_normal(D).astype(np.float32)))
        elif kind == 6:    # sparse
            v = rng.standard_normal(D) * (rng.random(D) < 0.3)
        else:              # wide dynamic range
            v = rng.standard_normal(D) * np.exp2(rng.integers(-20, 20, size=D))
        s = rng.integers(0, 2, size=D) * 2 - 1
        out[g] = (np.asarray(v, dtype=np.float64) * s).astype(np.float32)
    return out


def gaussian_weights_device(rows: int, cols: int, sigma: float, seed: int, device):
    """The same recipe as gaussian_weights(bf16=True), generated on a torch device (for matrices
    too large to build quickly with numpy): i.i.d. N(0, sigma^2), random signs and a block
    Walsh-Hadamard transform along each row, scaled by 1/sqrt(block), rounded to bf16.
    Returns a bfloat16 tensor [rows][cols].  The random stream differs from the numpy recipe."""
    import torch

    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    w = torch.randn((rows, cols), generator=gen, device=device, dtype=torch.float32) * sigma
    signs = torch.randint(0, 2, (cols,), generator=gen, device=device, dtype=torch.int32)
    w *= (signs * 2 - 1).to(torch.float32)[None, :]
    n = cols & (-cols)
    h = 1
    while h < n:
        v = w.view(rows, cols // (2 * h), 2, h)
        a, b = v[:, :, 0, :], v[:, :, 1, :]
        w = torch.stack((a + b, a - b), dim=2).reshape(rows, cols)
        h *= 2
    w *= 1.0 / float(np.sqrt(n))
    return w.to(torch.bfloat16)
