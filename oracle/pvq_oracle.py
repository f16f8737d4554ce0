"""numpy front end of the CPU oracle (``pvq_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the benchmark's
CPU-baseline leg.  The GPU library never imports or calls anything here.

The C file holds every step of the method (size table, quantisation, rank, unrank, packing,
amplitude codes, dequantisation, reference product).  This module only marshals numpy arrays
into it, and computes the Beta-quantile tables of the amplitude quantiser with
``scipy.stats.beta.ppf`` (arXiv 2410.16926, Sec. 3.4: quantize(x) = floor(CDF(x) 2^b),
dequantize(q) = PPF((q + 0.5) / 2^b), with Beta(D/2, D(G-1)/2) from Theorem 3.1).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pvq_oracle.c")
_LIB = os.path.join(_HERE, "libpvq_oracle.so")

# -ffp-contract=off: the float32 evaluation order of the encoder is part of its definition.
_CFLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
           "-Wall", "-Wextra", "-pthread"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (if the library is missing or older than its source)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        subprocess.check_call(["gcc", *_CFLAGS, "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        i32, i64, vp = C.c_int, C.c_int64, C.c_void_p
        L.pvqo_table.argtypes = [i32, i32, vp]
        L.pvqo_index_bits.argtypes = [i32, i32]
        L.pvqo_max_k.argtypes = [i32, i32]
        L.pvqo_row_words.argtypes = [i64, i32]
        L.pvqo_row_words.restype = i64
        L.pvqo_quantize_group.argtypes = [vp, i32, i32, vp, vp]
        L.pvqo_quantize_group.restype = None
        L.pvqo_rank_many.argtypes = [i32, i32, i64, vp, vp]
        L.pvqo_unrank_many.argtypes = [i32, i32, i64, vp, vp, i32]
        L.pvqo_encode.argtypes = [vp, i64, i64, i32, i32, i32, i32, vp, vp, vp, vp, vp, i32]
        L.pvqo_hadamard_rows.argtypes = [vp, i64, i64, i64, vp, i32, vp]
        L.pvqo_correct.argtypes = [vp, i64, i64, i32, i32, i32, vp, vp, i32]
        L.pvqo_ls_amplitude.argtypes = [vp, vp, i32]
        L.pvqo_ls_amplitude.restype = C.c_float
        L.pvqo_decode.argtypes = [vp, vp, vp, i64, i64, i32, i32, i32, vp, vp, vp, vp, i32,
                                  vp, i32]
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


NW = 16  # 32-bit words per integer inside the oracle


def words_to_int(words) -> int:
    """Little-endian 32-bit words -> Python int."""
    v = 0
    for i, w in enumerate(np.asarray(words).tolist()):
        v |= int(w) << (32 * i)
    return v


def int_to_words(v: int, nw: int = NW) -> np.ndarray:
    return np.array([(v >> (32 * i)) & 0xFFFFFFFF for i in range(nw)], dtype=np.uint32)


# ---------------------------------------------------------------- size table, K


def size_table(D: int, K: int):
    """N(d,k) for 0<=d<=D, 0<=k<=K as a list of lists of Python ints."""
    out = np.zeros(((D + 1) * (K + 1), NW), dtype=np.uint32)
    if lib().pvqo_table(D, K, _p(out)) != 0:
        raise OverflowError("N(D,K) exceeds the oracle's integer width")
    return [[words_to_int(out[d * (K + 1) + k]) for k in range(K + 1)] for d in range(D + 1)]


def index_bits(D: int, K: int) -> int:
    b = lib().pvqo_index_bits(D, K)
    if b < 0:
        raise ValueError("bad (D,K)")
    return b


def max_k(D: int, bit_budget: int) -> int:
    k = lib().pvqo_max_k(D, bit_budget)
    if k < 0:
        raise ValueError("no K fits")
    return k


def row_words(groups: int, bits: int) -> int:
    return int(lib().pvqo_row_words(groups, bits))


# ---------------------------------------------------------------- per-point routines


def quantize_group(w, K: int):
    """One group (float32) -> (pulse vector int32[D], float32 sum of squares)."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    y = np.zeros(w.size, dtype=np.int32)
    ss = np.zeros(1, dtype=np.float32)
    lib().pvqo_quantize_group(_p(w), w.size, K, _p(y), _p(ss))
    return y, ss[0]


def ls_amplitude(w, y) -> float:
    """Least-squares amplitude of one group w (float32) for its quantised point y (Sec. 3.3 Step 4)."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    y = np.ascontiguousarray(y, dtype=np.int32)
    assert w.shape == y.shape and w.ndim == 1
    return float(lib().pvqo_ls_amplitude(_p(w), _p(y), int(w.size)))


def rank(points, K: int):
    """points int [n][D] on P(D,K) -> list of Python-int indices."""
    x = np.ascontiguousarray(np.atleast_2d(points), dtype=np.int32)
    n, D = x.shape
    c = np.zeros((n, NW), dtype=np.uint32)
    if lib().pvqo_rank_many(D, K, n, _p(x), _p(c)) != 0:
        raise ValueError("a point is not on P(D,K)")
    return [words_to_int(c[i]) for i in range(n)]


def unrank(indices, D: int, K: int, omit_negative_update: bool = False) -> np.ndarray:
    """Python-int indices -> int32 [n][D].  ``omit_negative_update`` plants the decoding
    mistake of the original PVQ description (see the C file); tests only."""
    idx = list(indices)
    c = np.stack([int_to_words(int(v)) for v in idx]) if idx else np.zeros((0, NW), np.uint32)
    c = np.ascontiguousarray(c, dtype=np.uint32)
    x = np.zeros((len(idx), D), dtype=np.int32)
    if lib().pvqo_unrank_many(D, K, len(idx), _p(c), _p(x), int(omit_negative_update)) != 0:
        raise ValueError("an index is not below N(D,K)")
    return x


# ---------------------------------------------------------------- amplitude tables


def beta_tables(D: int, G: int, bits: int):
    """Quantile tables of Beta(D/2, D(G-1)/2) for a ``bits``-bit amplitude code.

    edges[j-1] = PPF(j / 2^b), j = 1 .. 2^b - 1   (so that #{edges <= u} = floor(CDF(u) 2^b))
    centers[q] = PPF((q + 0.5) / 2^b), q = 0 .. 2^b - 1
    Both float64.  The encoder compares against edges rounded once to float32.
    """
    from scipy.stats import beta

    a, b = D / 2.0, D * (G - 1) / 2.0
    n = 1 << bits
    edges = beta.ppf(np.arange(1, n, dtype=np.float64) / n, a, b)
    centers = beta.ppf((np.arange(n, dtype=np.float64) + 0.5) / n, a, b)
    return np.ascontiguousarray(edges), np.ascontiguousarray(centers)


# ---------------------------------------------------------------- whole matrices


def bf16_bits_to_f32(bits) -> np.ndarray:
    """uint16 bf16 bit patterns -> the same values as float32 (exact)."""
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


class Encoded:
    """What the encoder stores for one matrix."""

    def __init__(self, rows, cols, D, K, scale_bits, index, scale, rowss, pulses):
        self.rows, self.cols, self.D, self.K, self.scale_bits = rows, cols, D, K, scale_bits
        self.index = index      # uint32 [rows][row_words(G, index_bits)]
        self.scale = scale      # float32 [rows][G]  or  uint32 [rows][row_words(G, scale_bits)]
        self.rowss = rowss      # float32 [rows]
        self.pulses = pulses    # int8 [rows][cols] or None
        self.index_bits = index_bits(D, K)


def encode(W, D: int, K: int, scale_bits: int = 0, edges=None, want_pulses: bool = True,
           nthreads: int = 1, amplitude: str = "l2") -> Encoded:
    """W: float32 [rows][cols] (widen bf16 with bf16_bits_to_f32 first).
    amplitude: "l2" = the group's norm (Sec. 2.3), "ls" = least-squares amplitude (Sec. 3.3 Step 4)."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    rows, cols = W.shape
    G = cols // D
    ib = index_bits(D, K)
    index = np.zeros((rows, row_words(G, ib)), dtype=np.uint32)
    rowss = np.zeros(rows, dtype=np.float32)
    if scale_bits == 0:
        scale = np.zeros((rows, G), dtype=np.float32)
        e32 = None
    else:
        scale = np.zeros((rows, row_words(G, scale_bits)), dtype=np.uint32)
        e32 = np.ascontiguousarray(np.asarray(edges, dtype=np.float64).astype(np.float32))
        assert e32.size == (1 << scale_bits) - 1
    pulses = np.zeros((rows, cols), dtype=np.int8) if want_pulses and K <= 127 else None   # int8 plane
    rc = lib().pvqo_encode(_p(W), rows, cols, D, K, scale_bits, {"l2": 0, "ls": 1}[amplitude], _p(e32),
                           _p(index), _p(scale), _p(rowss), _p(pulses), nthreads)
    if rc != 0:
        raise ValueError("pvqo_encode rejected its arguments")
    return Encoded(rows, cols, D, K, scale_bits, index, scale, rowss, pulses)


def decode(enc: Encoded, centers=None, x=None, want_weights: bool = True,
           want_pulses: bool = False, nthreads: int = 1):
    """Returns (W_hat float64 [rows][cols] or None, pulses int8 or None,
    out float64 [batch][rows] or None).  x: float64 [batch][cols]."""
    rows, cols = enc.rows, enc.cols
    Wd = np.zeros((rows, cols), dtype=np.float64) if want_weights else None
    pulses = np.zeros((rows, cols), dtype=np.int8) if want_pulses else None
    cen = None
    if enc.scale_bits:
        cen = np.ascontiguousarray(centers, dtype=np.float64)
        assert cen.size == 1 << enc.scale_bits
    batch, out, xx = 0, None, None
    if x is not None:
        xx = np.ascontiguousarray(x, dtype=np.float64)
        batch = xx.shape[0]
        assert xx.shape[1] == cols
        out = np.zeros((batch, rows), dtype=np.float64)
    index = np.ascontiguousarray(enc.index, dtype=np.uint32)
    scale = np.ascontiguousarray(enc.scale)
    rowss = np.ascontiguousarray(enc.rowss, dtype=np.float32)
    rc = lib().pvqo_decode(_p(index), _p(scale), _p(rowss), rows, cols, enc.D, enc.K,
                           enc.scale_bits, _p(cen), _p(Wd), _p(pulses), _p(xx), batch, _p(out),
                           nthreads)
    if rc != 0:
        raise ValueError("pvqo_decode rejected its arguments")
    return Wd, pulses, out


def hadamard_rows(X, block: int, signs=None, signs_after: bool = False) -> np.ndarray:
    """Block-diagonal randomised Hadamard rotation of every row (float32), or its inverse
    (signs_after=True).  signs: uint8 [cols], non-zero = -1."""
    X = np.ascontiguousarray(X, dtype=np.float32)
    rows, cols = X.shape
    sg = None if signs is None else np.ascontiguousarray(signs, dtype=np.uint8)
    assert sg is None or sg.size == cols
    Y = np.empty_like(X)
    if lib().pvqo_hadamard_rows(_p(X), rows, cols, int(block), _p(sg), 1 if signs_after else 0, _p(Y)) != 0:
        raise ValueError("pvqo_hadamard_rows rejected its arguments")
    return Y


def correct(W, U, D: int, K: int, amplitude: str = "l2", nthreads: int = 1):
    """Sec. 3.3 Step 6: the rows of W (float32) taken through the groups in order, every group's
    quantisation error handed on to the columns behind it through U (float32 [cols][cols], upper
    triangular, U^T U = inverse Hessian).  Returns (the values that were quantised, their quantised
    values), both float32 [rows][cols]."""
    Wc = np.array(W, dtype=np.float32, order="C", copy=True)
    U32 = np.ascontiguousarray(U, dtype=np.float32)
    rows, cols = Wc.shape
    assert U32.shape == (cols, cols)
    Q = np.zeros_like(Wc)
    rc = lib().pvqo_correct(_p(Wc), rows, cols, D, K, {"l2": 0, "ls": 1}[amplitude], _p(U32), _p(Q), nthreads)
    if rc != 0:
        raise ValueError("pvqo_correct rejected its arguments")
    return Wc, Q


def unpack_fields(words, groups: int, bits: int):
    """Row bit streams uint32 [rows][row_words] -> list (per row) of lists of Python ints.
    A plain restatement of the layout, used by tests to look inside packed planes."""
    words = np.asarray(words, dtype=np.uint32)
    out = []
    for r in range(words.shape[0]):
        stream = words_to_int(words[r])
        out.append([(stream >> (g * bits)) & ((1 << bits) - 1) for g in range(groups)])
    return out


def to_f16(Wd) -> np.ndarray:
    """float64 -> IEEE binary16, round to nearest even."""
    return np.asarray(Wd, dtype=np.float64).astype(np.float16)


def to_bf16_bits(Wd) -> np.ndarray:
    """float64 -> bf16 bit patterns (uint16), rounded once to nearest, ties to even.

    bf16 is the upper half of an IEEE binary32: 8 significant bits for normal numbers (exponents
    -126..127), multiples of 2^-133 below 2^-126, overflow to infinity.  The value is divided by the
    spacing of bf16 numbers at its magnitude (a power of two: exact), rounded to an integer with
    ties to even, and multiplied back (exact); the result is a bf16 number, so its binary32 pattern
    has zero low bits and the upper half is the answer.  No intermediate rounding to binary32."""
    v = np.asarray(Wd, dtype=np.float64)
    out = np.empty(v.shape, dtype=np.uint16)
    finite = np.isfinite(v)
    a = np.abs(np.where(finite, v, 0.0))
    _, e = np.frexp(a)                      # a = m * 2^e with 0.5 <= m < 1, so floor(log2 a) = e - 1
    e = np.maximum(e - 1, -126)             # below the normal range the spacing stays 2^-133
    spacing = np.ldexp(1.0, e - 7)
    r = np.rint(a / spacing) * spacing      # np.rint rounds half-way cases to even
    with np.errstate(over="ignore"):
        r32 = np.where(r >= 2.0 ** 128, np.inf, r).astype(np.float32)   # exact, or overflow
    bits = (r32.view(np.uint32) >> 16).astype(np.uint16)
    bits = bits | np.where(np.signbit(v), 0x8000, 0).astype(np.uint16)
    out[...] = bits
    # infinities and NaN keep their class (a NaN's payload is not specified)
    nf = ~finite
    if nf.any():
        out[nf] = (np.asarray(v[nf], dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)
        out[nf & np.isnan(v)] |= 0x0040
    return out
