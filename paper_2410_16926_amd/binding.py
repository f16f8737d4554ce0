"""Thin ctypes binding of libpvq (see include/pvq.h).  Argument marshalling only: every step of
encode / decode / decode_gemv runs in the library's kernels.  PyTorch supplies device memory and
the stream."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

PVQ_F32, PVQ_F16, PVQ_BF16 = 0, 1, 2

EXPORTS = [
    "pvq_strerror", "pvq_last_hip_error", "pvq_count", "pvq_max_k", "pvq_beta_tables", "pvq_rotate_encode", "pvq_correct", "pvq_correct_work_bytes",
    "pvq_correct_static", "pvq_correct_static_max_rows",
    "pvq_size_table_device", "pvq_hadamard",
    "pvq_ctx_create", "pvq_ctx_destroy", "pvq_ctx_info", "pvq_ctx_set_amplitude", "pvq_packed_sizes",
    "pvq_encode", "pvq_decode", "pvq_decode_gemv",
]

# host-only diagnostics declared in csrc/pvq_diagnostics.h, exported for the tests
DIAGNOSTICS = ["pvq_fast_tables_selftest", "pvq_walk_tables_selftest", "pvq_decode_gemv_plan", "pvq_correct_set_front_tiles",
               "pvq_decode_set_table_decoder_min_groups"]


class PvqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().pvq_strerror(status).decode()
        if status == -4:
            msg += f" [hipError {lib().pvq_last_hip_error()}]"
        super().__init__(f"{where}: {msg} ({status})")


_lib = None


def lib():
    """The loaded library.  Builds it only if no built library exists; a missing or broken
    library is an error (there is no fallback path)."""
    global _lib
    if _lib is None:
        path = _build.LIB_PATH
        if not os.path.exists(path):
            _build.build()
        # PyTorch ships its own HIP runtime; load it first so that the process holds one runtime
        # and the library's streams and pointers are the ones torch hands out.
        import torch  # noqa: F401
        L = C.CDLL(path)
        i32, i64, vp = C.c_int, C.c_int64, C.c_void_p
        L.pvq_strerror.restype = C.c_char_p
        L.pvq_strerror.argtypes = [i32]
        L.pvq_last_hip_error.argtypes = []
        L.pvq_count.argtypes = [i32, i32, vp, vp]
        L.pvq_max_k.argtypes = [i32, i32, vp]
        L.pvq_beta_tables.argtypes = [i32, i64, i32, vp, vp]
        L.pvq_fast_tables_selftest.argtypes = [i32, C.c_uint64, C.c_uint64, vp]
        L.pvq_walk_tables_selftest.argtypes = [i32, i32, C.c_uint64, C.c_uint64, vp, vp, vp]
        L.pvq_decode_gemv_plan.argtypes = [vp, i64, i64, i32, vp, vp, i32, vp]
        L.pvq_size_table_device.argtypes = [i32, i32, i32, vp, vp, vp]
        L.pvq_hadamard.argtypes = [vp, i32, i64, i64, i64, i32, vp, i32, vp, i32, i64, vp]
        L.pvq_ctx_create.argtypes = [vp, i32, i32, i32, vp, vp]
        L.pvq_ctx_destroy.argtypes = [vp]
        L.pvq_ctx_info.argtypes = [vp, vp, vp, vp, vp]
        L.pvq_ctx_set_amplitude.argtypes = [vp, i32]
        L.pvq_packed_sizes.argtypes = [vp, i64, i64, vp, vp, vp]
        L.pvq_encode.argtypes = [vp, vp, i32, i64, i64, i64, vp, vp, vp, vp, vp]
        L.pvq_rotate_encode.argtypes = [vp, vp, i32, i64, i64, i64, i32, vp, vp, vp, vp, vp]
        L.pvq_correct_work_bytes.argtypes = [i64, vp]
        L.pvq_correct.argtypes = [vp, vp, i64, i64, i64, vp, i64, vp, C.c_size_t, vp]
        L.pvq_correct_static_max_rows.argtypes = [vp]
        L.pvq_correct_set_front_tiles.argtypes = [i64, vp]
        L.pvq_decode_set_table_decoder_min_groups.argtypes = [i64, vp]
        L.pvq_correct_static.argtypes = [vp, vp, i64, i64, i64, vp, i64, vp]
        L.pvq_decode.argtypes = [vp, vp, vp, vp, i64, i64, vp, i32, i64, vp]
        L.pvq_decode_gemv.argtypes = [vp, vp, vp, vp, i64, i64, vp, i32, i64, vp, i64, vp]
        _lib = L
    return _lib


def _check(status: int, where: str):
    if status != 0:
        raise PvqError(status, where)


# ------------------------------------------------------------------ host helpers


def pvq_count(D: int, K: int):
    """(N(D,K) as a Python int, index_bits)."""
    words = (C.c_uint32 * 16)()
    bits = C.c_int()
    _check(lib().pvq_count(D, K, words, C.byref(bits)), "pvq_count")
    n = 0
    for i in range(16):
        n |= int(words[i]) << (32 * i)
    return n, bits.value


def pvq_max_k(D: int, bit_budget: int) -> int:
    k = C.c_int()
    _check(lib().pvq_max_k(D, bit_budget, C.byref(k)), "pvq_max_k")
    return k.value


def pvq_beta_tables(D: int, G: int, scale_bits: int):
    """(edges float64[2^b - 1], centers float64[2^b])."""
    n = 1 << max(scale_bits, 0)
    edges = np.zeros(max(n - 1, 1), dtype=np.float64)
    centers = np.zeros(n, dtype=np.float64)
    _check(lib().pvq_beta_tables(D, G, scale_bits, edges.ctypes.data, centers.ctypes.data),
           "pvq_beta_tables")
    return edges[: n - 1], centers


def pvq_fast_tables_selftest(K: int, first: int = 0, count: int = 1 << 40) -> int:
    """Number of indices in [first, first+count) that the table-driven D=8 decoder gets wrong
    (host replay).  Raises PvqError(-2) if (8, K) has no such tables."""
    bad = C.c_uint64()
    _check(lib().pvq_fast_tables_selftest(K, first, count, C.byref(bad)), "pvq_fast_tables_selftest")
    return bad.value


def pvq_walk_tables_selftest(D: int, K: int, seed: int = 1, count: int = 100000):
    """(mismatches, (dA, dB), table bytes) of the host replay of the coordinate-by-coordinate decoder's tables."""
    bad, sched, nbytes = C.c_uint64(), (C.c_int * 2)(), C.c_uint32()
    _check(lib().pvq_walk_tables_selftest(D, K, seed, count, C.byref(bad), sched, C.byref(nbytes)),
           "pvq_walk_tables_selftest")
    return bad.value, (sched[0], sched[1]), nbytes.value


PASS_KINDS = {0: "valu_fp32_generic", 1: "valu_fp32", 2: "valu_fp32_rows", 3: "valu_fp32_16", 4: "mfma_bf16"}


def pvq_decode_gemv_plan(ctx, rows: int, cols: int, batch: int):
    """[(kind name, vectors)] per pass that pvq_decode_gemv would launch (nothing is launched)."""
    kinds, nvecs, n = (C.c_int * 16)(), (C.c_int * 16)(), C.c_int()
    _check(lib().pvq_decode_gemv_plan(ctx.handle, rows, cols, batch, kinds, nvecs, 16, C.byref(n)),
           "pvq_decode_gemv_plan")
    return [(PASS_KINDS[kinds[i]], nvecs[i]) for i in range(n.value)]


def pvq_size_table_device(D: int, K: int, words: int, device=None):
    """The size table computed on the GPU: (int32 tensor [(D+1)][(K+1)][words] holding the unsigned
    little-endian words, int32 tensor [1] = overflow flag), both on `device`; asynchronous."""
    import torch
    device = device or torch.device("cuda", torch.cuda.current_device())
    table = torch.empty((D + 1, K + 1, words), dtype=torch.int32, device=device)
    flag = torch.empty(1, dtype=torch.int32, device=device)
    _check(lib().pvq_size_table_device(D, K, words, C.c_void_p(table.data_ptr()), C.c_void_p(flag.data_ptr()),
                                       _stream_ptr()), "pvq_size_table_device")
    return table, flag


def pvq_hadamard(X, block: int, signs=None, inverse: bool = False, out=None, out_dtype=None):
    """Randomised Hadamard rotation of every row of the 2-D device tensor X (float32 or bfloat16) in
    blocks of `block` columns, or its inverse.  signs: uint8 device tensor [cols] (non-zero = -1) or None."""
    import torch
    rows, cols = X.shape
    if out is None:
        out = torch.empty((rows, cols), dtype=out_dtype or X.dtype, device=X.device)
    _check(lib().pvq_hadamard(_ptr(X), _dtype_code(X), rows, cols, X.stride(0) if rows > 1 else cols, block,
                              _ptr(signs), 1 if inverse else 0, _ptr(out), _dtype_code(out),
                              out.stride(0) if rows > 1 else cols, _stream_ptr()), "pvq_hadamard")
    return out


# ------------------------------------------------------------------ context


class PvqContext:
    """Owns a pvq_ctx*.  Create it with the wanted torch device current."""

    def __init__(self, D: int, K: int, scale_bits: int = 0, edges=None, centers=None):
        self._h = C.c_void_p()
        e = c = None
        if scale_bits:
            e = np.ascontiguousarray(edges, dtype=np.float64)
            c = np.ascontiguousarray(centers, dtype=np.float64)
            if e.size != (1 << scale_bits) - 1 or c.size != (1 << scale_bits):
                raise ValueError("edges/centers have the wrong length")
        _check(lib().pvq_ctx_create(C.byref(self._h), D, K, scale_bits,
                                    None if e is None else e.ctypes.data,
                                    None if c is None else c.ctypes.data), "pvq_ctx_create")
        d, k, b, s = C.c_int(), C.c_int(), C.c_int(), C.c_int()
        _check(lib().pvq_ctx_info(self._h, C.byref(d), C.byref(k), C.byref(b), C.byref(s)),
               "pvq_ctx_info")
        self.D, self.K, self.index_bits, self.scale_bits = d.value, k.value, b.value, s.value

    @property
    def handle(self):
        return self._h

    def set_amplitude(self, kind: str):
        """"norm": group norms (default); "ls": least-squares amplitudes (pvq_ctx_set_amplitude)."""
        _check(lib().pvq_ctx_set_amplitude(self._h, {"norm": 0, "ls": 1}[kind]), "pvq_ctx_set_amplitude")

    def close(self):
        if self._h:
            h, self._h = self._h, C.c_void_p()
            _check(lib().pvq_ctx_destroy(h), "pvq_ctx_destroy")

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def pvq_ctx_create(D, K, scale_bits=0, edges=None, centers=None) -> PvqContext:
    return PvqContext(D, K, scale_bits, edges, centers)


def pvq_ctx_destroy(ctx: PvqContext):
    ctx.close()


def pvq_ctx_set_amplitude(ctx: PvqContext, kind: str):
    ctx.set_amplitude(kind)


def pvq_packed_sizes(ctx: PvqContext, rows: int, cols: int):
    """(index_bytes, scale_bytes, rownorm_bytes)."""
    a, b, c = C.c_size_t(), C.c_size_t(), C.c_size_t()
    _check(lib().pvq_packed_sizes(ctx.handle, rows, cols, C.byref(a), C.byref(b), C.byref(c)),
           "pvq_packed_sizes")
    return a.value, b.value, c.value


# ------------------------------------------------------------------ hot path (torch tensors)


def _stream_ptr():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dtype_code(t):
    import torch
    return {torch.float32: PVQ_F32, torch.float16: PVQ_F16, torch.bfloat16: PVQ_BF16}[t.dtype]


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


class Packed:
    """The three planes of an encoded matrix (device tensors) and its shape."""

    def __init__(self, rows, cols, index, scale, rownorm, pulses=None):
        self.rows, self.cols = rows, cols
        self.index, self.scale, self.rownorm, self.pulses = index, scale, rownorm, pulses


def alloc_packed(ctx: PvqContext, rows: int, cols: int, device, want_pulses=False) -> Packed:
    import torch
    ib, sb, rb = pvq_packed_sizes(ctx, rows, cols)
    G = cols // ctx.D
    index = torch.empty((rows, ib // 4 // max(rows, 1)), dtype=torch.int32, device=device)
    if ctx.scale_bits == 0:
        scale = torch.empty((rows, G), dtype=torch.float32, device=device)
    else:
        scale = torch.empty((rows, sb // 4 // max(rows, 1)), dtype=torch.int32, device=device)
    rownorm = torch.empty((rows,), dtype=torch.float32, device=device)
    pulses = torch.empty((rows, cols), dtype=torch.int8, device=device) if want_pulses else None
    return Packed(rows, cols, index, scale, rownorm, pulses)


def pvq_encode(ctx: PvqContext, W, out: Packed = None, want_pulses: bool = False) -> Packed:
    """W: 2-D float32 or bfloat16 device tensor with unit column stride."""
    rows, cols = W.shape
    assert W.stride(1) == 1 or cols <= 1
    if out is None:
        out = alloc_packed(ctx, rows, cols, W.device, want_pulses)
    ld = W.stride(0) if rows > 1 else max(cols, 1)
    _check(lib().pvq_encode(ctx.handle, _ptr(W), _dtype_code(W), rows, cols, ld, _ptr(out.index),
                            _ptr(out.scale), _ptr(out.rownorm), _ptr(out.pulses), _stream_ptr()),
           "pvq_encode")
    return out


def pvq_rotate_encode(ctx: PvqContext, X, block: int, signs=None, out: Packed = None) -> Packed:
    """Randomised Hadamard rotation of the rows of X (blocks of `block` columns) and encoding of the rotated
    values, in one kernel.  X: 2-D float32 or bfloat16 device tensor; signs: uint8 device tensor [cols] or None."""
    rows, cols = X.shape
    if out is None:
        out = alloc_packed(ctx, rows, cols, X.device)
    ld = X.stride(0) if rows > 1 else max(cols, 1)
    _check(lib().pvq_rotate_encode(ctx.handle, _ptr(X), _dtype_code(X), rows, cols, ld, block, _ptr(signs),
                                   _ptr(out.index), _ptr(out.scale), _ptr(out.rownorm), _stream_ptr()), "pvq_rotate_encode")
    return out


def pvq_correct(ctx: PvqContext, W, U, work=None):
    """Error correction group after group, in place.  W: float32 [rows][cols] device tensor (overwritten
    with the values to encode), U: float32 [cols][cols] upper triangular device tensor, U^T U = inverse
    Hessian; work: optional uint8 device tensor of pvq_correct_work_bytes(rows) bytes.  Returns W."""
    import torch
    rows, cols = W.shape
    assert W.dtype == torch.float32 and U.dtype == torch.float32 and tuple(U.shape) == (cols, cols)
    if work is None:
        nbytes = C.c_size_t(0)
        _check(lib().pvq_correct_work_bytes(rows, C.byref(nbytes)), "pvq_correct_work_bytes")
        work = torch.empty((max(int(nbytes.value), 16),), dtype=torch.uint8, device=W.device)
    ldw = W.stride(0) if rows > 1 else max(cols, 1)
    ldu = U.stride(0) if cols > 1 else 1
    _check(lib().pvq_correct(ctx.handle, _ptr(W), rows, cols, ldw, _ptr(U), ldu, _ptr(work), work.numel(),
                             _stream_ptr()), "pvq_correct")
    return W


def pvq_correct_set_front_tiles(tiles: int) -> int:
    """Diagnostics: from how many update tiles on a launch of pvq_correct does the narrow update inside its panel
    workgroups (process-wide; results do not depend on it).  Returns the number in force before."""
    old = C.c_int64(0)
    _check(lib().pvq_correct_set_front_tiles(int(tiles), C.byref(old)), "pvq_correct_set_front_tiles")
    return old.value


def pvq_decode_set_table_decoder_min_groups(groups: int) -> int:
    """Diagnostics: matrices of fewer groups of 8 than this are decoded coordinate by coordinate instead of through
    the tables (process-wide).  Returns the number in force before."""
    old = C.c_int64(0)
    _check(lib().pvq_decode_set_table_decoder_min_groups(int(groups), C.byref(old)),
           "pvq_decode_set_table_decoder_min_groups")
    return old.value


def pvq_correct_static_max_rows() -> int:
    n = C.c_int64(0)
    _check(lib().pvq_correct_static_max_rows(C.byref(n)), "pvq_correct_static_max_rows")
    return n.value


def pvq_correct_static(ctx: PvqContext, W, U):
    """pvq_correct with the library's static work buffer: no allocation, the caller's stream only, at most
    pvq_correct_static_max_rows() rows.  Returns W."""
    import torch
    rows, cols = W.shape
    assert W.dtype == torch.float32 and U.dtype == torch.float32 and tuple(U.shape) == (cols, cols)
    ldw = W.stride(0) if rows > 1 else max(cols, 1)
    ldu = U.stride(0) if cols > 1 else 1
    _check(lib().pvq_correct_static(ctx.handle, _ptr(W), rows, cols, ldw, _ptr(U), ldu, _stream_ptr()),
           "pvq_correct_static")
    return W


def pvq_decode(ctx: PvqContext, packed: Packed, out_dtype=None, out=None):
    """Returns the decoded [rows][cols] tensor of out_dtype (torch.float32/float16/bfloat16)."""
    import torch
    if out is None:
        out = torch.empty((packed.rows, packed.cols), dtype=out_dtype or torch.float32,
                          device=packed.index.device)
    ld = out.stride(0) if packed.rows > 1 else max(packed.cols, 1)
    _check(lib().pvq_decode(ctx.handle, _ptr(packed.index), _ptr(packed.scale), _ptr(packed.rownorm),
                            packed.rows, packed.cols, _ptr(out), _dtype_code(out), ld, _stream_ptr()),
           "pvq_decode")
    return out


def pvq_decode_gemv(ctx: PvqContext, packed: Packed, x, out=None):
    """x: bfloat16 [batch][cols] device tensor; returns float32 [batch][rows]."""
    import torch
    batch = x.shape[0]
    assert x.dtype == torch.bfloat16 and x.shape[1] == packed.cols
    if out is None:
        out = torch.empty((batch, packed.rows), dtype=torch.float32, device=x.device)
    ldx = x.stride(0) if batch > 1 else max(packed.cols, 1)
    ldy = out.stride(0) if batch > 1 else max(packed.rows, 1)
    _check(lib().pvq_decode_gemv(ctx.handle, _ptr(packed.index), _ptr(packed.scale),
                                 _ptr(packed.rownorm), packed.rows, packed.cols, _ptr(x), batch, ldx,
                                 _ptr(out), ldy, _stream_ptr()), "pvq_decode_gemv")
    return out
