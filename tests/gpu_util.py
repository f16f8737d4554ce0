"""Helpers shared by the GPU parity tests: move seeded inputs to the device, run the library
through its binding, fetch results as numpy, compare with the oracle."""
from __future__ import annotations

import contextlib

import numpy as np

import paper_2410_16926_amd as pvq
from oracle import pvq_oracle as oracle


def to_dev_f32(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def to_dev_bf16(bits):
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits, dtype=np.uint16).view(np.int16)).cuda().view(torch.bfloat16)


def words(t) -> np.ndarray:
    return t.cpu().numpy().view(np.uint32)


def bf16_tensor_bits(t) -> np.ndarray:
    import torch
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def make_ctx(D, K, scale_bits, G):
    """Library context with the library's own tables, and the oracle's tables beside it; the two
    table sets must agree bit for bit once rounded as each side uses them."""
    if scale_bits == 0:
        return pvq.pvq_ctx_create(D, K), None, None
    e, c = pvq.pvq_beta_tables(D, G, scale_bits)
    oe, oc = oracle.beta_tables(D, G, scale_bits)
    assert np.array_equal(e.astype(np.float32), oe.astype(np.float32))
    assert np.array_equal(np.sqrt(c).astype(np.float32), np.sqrt(oc).astype(np.float32))
    return pvq.pvq_ctx_create(D, K, scale_bits, e, c), oe, oc


def assert_encode_equal(packed, enc, check_pulses=True):
    """Bit-exact: packed indices, pulse vectors, amplitudes / codes and row normalisers."""
    got = words(packed.index)
    bad = np.argwhere(got != enc.index)
    assert bad.size == 0, f"{bad.shape[0]} index words differ, first at {bad[0]}"
    if check_pulses and packed.pulses is not None:
        gp = packed.pulses.cpu().numpy()
        bad = np.argwhere(gp != enc.pulses)
        assert bad.size == 0, f"{bad.shape[0]} pulses differ, first at {bad[0]}"
    if enc.scale_bits == 0:
        gs = packed.scale.cpu().numpy()
        assert np.array_equal(gs.view(np.uint32), enc.scale.view(np.uint32)), "float32 amplitudes differ"
    else:
        assert np.array_equal(words(packed.scale), enc.scale), "amplitude codes differ"
        assert np.array_equal(packed.rownorm.cpu().numpy().view(np.uint32), enc.rowss.view(np.uint32)), \
            "row normalisers differ"


def ulp_f16(ref_bits: np.ndarray, got_bits: np.ndarray) -> int:
    """Largest distance in units in the last place between two arrays of 16-bit float patterns
    (works for binary16 and bf16: sign-magnitude patterns mapped to a monotone integer line)."""
    def line(b):
        b = b.astype(np.int32)
        return np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)
    return int(np.abs(line(ref_bits) - line(got_bits)).max()) if ref_bits.size else 0


def decoder_settings(D):
    """Values for pvq_decode_set_table_decoder_min_groups that force either decoder for groups of 8 (for other
    group sizes the setting has no effect: one pass with the default)."""
    return (0, 1 << 62) if D == 8 else (None,)


@contextlib.contextmanager
def decoder_setting(min_groups):
    if min_groups is None:
        yield
        return
    old = pvq.pvq_decode_set_table_decoder_min_groups(min_groups)
    try:
        yield
    finally:
        pvq.pvq_decode_set_table_decoder_min_groups(old)


def assert_decode_close(got_f32: np.ndarray, ref64: np.ndarray, rel=1e-6):
    """float32 output against the float64 oracle: relative 1e-6, zeros exactly zero."""
    got = got_f32.astype(np.float64)
    err = np.abs(got - ref64)
    ok = err <= rel * np.abs(ref64)
    assert ok.all(), f"{(~ok).sum()} weights off, worst rel {np.max(err / np.maximum(np.abs(ref64), 1e-300)):.3e}"


def assert_gemv_close(y: np.ndarray, ref: np.ndarray, scale: np.ndarray = None, rel=1e-3, rel_terms=1e-5):
    """Per activation vector b, against ref = float64 matmul of the oracle's weights:
      (1) ||y - ref||_2 <= rel * ||ref||_2
      (2) |y_i - ref_i| <= rel * (|ref_i| + rms(ref))                      (1e-3 relative, config 4)
      (3) |y_i - ref_i| <= rel_terms * s_i,  s_i = sqrt(sum_c (w_ic x_c)^2)  (with `scale` = s)
    Every kernel behind pvq_decode_gemv works with the float32 gain and the exact pulses (products of pulses
    with bf16 activations are exact in float32, on the vector ALUs and on the matrix cores alike) and
    accumulates in float32, so its error is rounding of sums and of the gain's multiplication: a few 2^-24 of
    the partial sums, about 1e-7 * s_i.  (3) pins that with a margin of 100; an error of 1e-4 in a gain or an amplitude, or a
    weight cut to fewer than 17 significant bits, fails it.  (1) and (2) are the tolerance the workload
    states; an output whose terms cancel to below 1e-3 of their size could fail (2) with correct arithmetic,
    which none of the seeded cases does."""
    y = y.astype(np.float64)
    for b in range(ref.shape[0]):
        nrm = np.linalg.norm(ref[b])
        rms = nrm / np.sqrt(ref.shape[1])
        d = np.abs(y[b] - ref[b])
        assert np.linalg.norm(y[b] - ref[b]) <= rel * nrm, (b, np.linalg.norm(y[b] - ref[b]) / nrm)
        assert np.all(d <= rel * (np.abs(ref[b]) + rms)), (b, float(np.max(d / (np.abs(ref[b]) + rms))))
        if scale is not None:
            worst = float(np.max(d / np.maximum(scale[b], 1e-300)))
            assert np.all(d <= rel_terms * scale[b]), (b, worst)


def product_scale(xf: np.ndarray, ref_weights: np.ndarray) -> np.ndarray:
    """[batch][rows]: root sum of squares of the terms of every output of x @ W^T (float64)."""
    x2 = xf.astype(np.float64) ** 2
    out = np.empty((xf.shape[0], ref_weights.shape[0]))
    step = 2048                                  # bound the temporaries
    for r0 in range(0, ref_weights.shape[0], step):
        out[:, r0:r0 + step] = np.sqrt(x2 @ (ref_weights[r0:r0 + step] ** 2).T)
    return out
