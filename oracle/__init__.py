"""CPU oracle of the quantized-linear hot path — TEST INFRASTRUCTURE ONLY.

Thin ctypes access to oracle/libqpo.so (plain C, binary64; see qpo.c for the
definitions and the list of pins).  Nothing in the product package may import
this module; only tests/, the smoke check and the benchmark's cpu_baseline leg do.
"""
from __future__ import annotations

import ctypes as C

import numpy as np

from . import build as _build

_lib = None

_u8p = np.ctypeslib.ndpointer(dtype=np.uint8, flags="C_CONTIGUOUS")
_u16p = np.ctypeslib.ndpointer(dtype=np.uint16, flags="C_CONTIGUOUS")
_i8p = np.ctypeslib.ndpointer(dtype=np.int8, flags="C_CONTIGUOUS")
_f64p = np.ctypeslib.ndpointer(dtype=np.float64, flags="C_CONTIGUOUS")
_i32p = np.ctypeslib.ndpointer(dtype=np.int32, flags="C_CONTIGUOUS")
_i64p = np.ctypeslib.ndpointer(dtype=np.int64, flags="C_CONTIGUOUS")


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(_build.build(force=False))
        L.qpo_half_to_double.restype = C.c_double
        L.qpo_half_to_double.argtypes = [C.c_uint16]
        L.qpo_half_to_double_array.argtypes = [_u16p, C.c_int64, _f64p]
        L.qpo_bit.restype = C.c_int
        L.qpo_bit.argtypes = [_u8p, C.c_int64]
        L.qpo_code.restype = C.c_uint32
        L.qpo_code.argtypes = [_u8p, C.c_int64, C.c_int]
        L.qpo_window.restype = C.c_uint32
        L.qpo_window.argtypes = [_u8p, C.c_int64, C.c_int, C.c_int64]
        L.qpo_decode.restype = C.c_int
        L.qpo_decode.argtypes = [C.c_int, _u8p, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_int,
                                 C.c_int, C.c_int, _u16p, _u16p]
        L.qpo_decode_row_tcq.argtypes = [_u8p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, _u16p, _u16p]
        L.qpo_decode_row_tcq_recurrence.argtypes = L.qpo_decode_row_tcq.argtypes
        L.qpo_decode_row_sq.argtypes = [_u8p, C.c_int, C.c_int, _u16p, _u16p]
        L.qpo_decode_row_vq.argtypes = [_u8p, C.c_int, C.c_int, C.c_int, _u16p, _u16p]
        L.qpo_hadamard_entry.restype = C.c_int
        L.qpo_hadamard_entry.argtypes = [C.c_uint32, C.c_uint32]
        for f in (L.qpo_hadamard_dense, L.qpo_hadamard_fast):
            f.argtypes = [_u16p, _i8p, C.c_int, C.c_int, C.c_int, C.c_int64, _f64p]
        L.qpo_matmul_scaled.argtypes = [_f64p, _u16p, _u16p, C.c_int, C.c_int, C.c_int, _f64p]
        L.qpo_linear_rows.restype = C.c_int
        L.qpo_linear_rows.argtypes = [C.c_int, _u8p, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_int,
                                      C.c_int, C.c_int, _u16p, _u16p, _f64p, C.c_int, C.c_int,
                                      C.c_int, _f64p, C.c_int]
        L.qpo_hybrid_lut.argtypes = [_u16p, C.c_int, _u16p]
        L.qpo_kmeans_assign.restype = C.c_double
        L.qpo_kmeans_assign.argtypes = [_f64p, C.c_int64, C.c_int, _f64p, C.c_int, _i32p]
        L.qpo_kmeans_update.restype = C.c_double
        L.qpo_kmeans_update.argtypes = [_f64p, C.c_int64, C.c_int, _i32p, _f64p, C.c_int, _f64p, _i64p]
        L.qpo_kmeans.restype = C.c_int
        L.qpo_kmeans.argtypes = [_f64p, C.c_int64, C.c_int, _f64p, C.c_int, C.c_int, C.c_double,
                                 C.POINTER(C.c_double)]
        L.qpo_num_threads.restype = C.c_int
        L.qpo_rtn_sq.argtypes = [_f64p, C.c_int64, C.c_int, _u16p, _u8p]
        L.qpo_rtn_vq.argtypes = [_f64p, C.c_int64, C.c_int, C.c_int, _u16p, _u8p]
        for f in (L.qpo_tcq_encode_brute, L.qpo_tcq_encode_viterbi_exact, L.qpo_tcq_encode_viterbi):
            f.restype = C.c_double
            f.argtypes = [_f64p, C.c_int, C.c_int, C.c_int, C.c_int, _u16p, _u8p]
        L.qpo_tcq_encode_tiles.argtypes = [_f64p, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_int,
                                           _u16p, _u8p, _f64p]
        L.qpo_tcq_encode_constrained.restype = C.c_double
        L.qpo_tcq_encode_constrained.argtypes = [_f64p, C.c_int, C.c_int, C.c_int, C.c_int, _u16p, C.c_uint32, _u8p]
        L.qpo_tcq_tile_error.restype = C.c_double
        L.qpo_tcq_tile_error.argtypes = [_f64p, _u8p, C.c_int, C.c_int, C.c_int, C.c_int, _u16p]
        _lib = L
    return _lib


def _u16(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    assert a.dtype == np.uint16
    return a


def half_to_double(a) -> np.ndarray:
    """Exact binary64 values of an fp16 (or uint16-pattern) array."""
    h = _u16(a)
    out = np.empty(h.size, dtype=np.float64)
    lib().qpo_half_to_double_array(h.reshape(-1), h.size, out)
    return out.reshape(h.shape)


TCQH = 3   # trellis with the hybrid computed code book: expanded here, then decoded as a trellis
TCQHH = 4  # half-TCQ: first half of the input channels at code_bits per step, second half at code_bits + 1


def hybrid_lut(tlut16, tlut_bits: int) -> np.ndarray:
    """Expanded 2^16 x 2 table (uint16 fp16 patterns) of the hybrid code book."""
    t = _u16(tlut16).reshape(-1)
    assert t.size == (1 << tlut_bits) * 2
    out = np.empty(65536 * 2, dtype=np.uint16)
    lib().qpo_hybrid_lut(t, tlut_bits, out)
    return out.reshape(65536, 2)


def _scheme_and_lut(layer):
    if layer.scheme == TCQH:
        return 2, hybrid_lut(layer.lut, layer.tlut_bits).reshape(-1)
    if layer.scheme == TCQHH:
        return 3, hybrid_lut(layer.lut, layer.tlut_bits).reshape(-1)
    return layer.scheme, _u16(layer.lut)


def decode(layer) -> np.ndarray:
    """Unscaled W^ as uint16 fp16 patterns [M, N] of a synth.Layer-like object."""
    out = np.empty((layer.M, layer.N), dtype=np.uint16)
    codes = np.ascontiguousarray(layer.codes)
    scheme, lut = _scheme_and_lut(layer)
    rc = lib().qpo_decode(scheme, codes.reshape(-1), codes.shape[1], layer.M, layer.N,
                          layer.code_bits, layer.vec, layer.window_bits, layer.tile,
                          lut, out.reshape(-1))
    assert rc == 0
    return out


def hadamard(x16, signs, block: int, *, fast: bool = False) -> np.ndarray:
    """Rotated activations in binary64 [B, n] from fp16 x [B, n]."""
    x = _u16(x16)
    B, n = x.shape
    out = np.empty((B, n), dtype=np.float64)
    f = lib().qpo_hadamard_fast if fast else lib().qpo_hadamard_dense
    f(x.reshape(-1), np.ascontiguousarray(signs, dtype=np.int8), B, n, block, n, out.reshape(-1))
    return out


def matmul_scaled(x64, W16, s16) -> np.ndarray:
    x = np.ascontiguousarray(x64, dtype=np.float64)
    W = _u16(W16)
    B, N = x.shape
    M = W.shape[0]
    y = np.empty((B, M), dtype=np.float64)
    lib().qpo_matmul_scaled(x.reshape(-1), W.reshape(-1), _u16(s16), B, M, N, y.reshape(-1))
    return y


def linear(layer, x, *, rows=None, threads: bool = False) -> np.ndarray:
    """y = (x W^T) diag(s) in binary64, [B, M].  x: fp16 [B,N] (exact values taken)
    or float64 [B,N].  rows=(begin,end) computes only those output rows (others 0)."""
    if x.dtype == np.float16 or x.dtype == np.uint16:
        x = half_to_double(x)
    x = np.ascontiguousarray(x, dtype=np.float64)
    B = x.shape[0]
    y = np.zeros((B, layer.M), dtype=np.float64)
    r0, r1 = rows if rows is not None else (0, layer.M)
    codes = np.ascontiguousarray(layer.codes)
    scheme, lut = _scheme_and_lut(layer)
    rc = lib().qpo_linear_rows(scheme, codes.reshape(-1), codes.shape[1], layer.M, layer.N,
                               layer.code_bits, layer.vec, layer.window_bits, layer.tile,
                               lut, _u16(layer.scales), x.reshape(-1), B, r0, r1,
                               y.reshape(-1), 1 if threads else 0)
    assert rc == 0
    return y


def num_threads() -> int:
    return lib().qpo_num_threads()


def rtn_sq(v, bits, lut16) -> np.ndarray:
    v = np.ascontiguousarray(v, dtype=np.float64).reshape(-1)
    out = np.zeros((v.size * bits + 7) // 8, dtype=np.uint8)
    lib().qpo_rtn_sq(v, v.size, bits, _u16(lut16), out)
    return out


def rtn_vq(v, cbits, V, lut16) -> np.ndarray:
    v = np.ascontiguousarray(v, dtype=np.float64).reshape(-1)
    out = np.zeros((v.size // V * cbits + 7) // 8, dtype=np.uint8)
    lib().qpo_rtn_vq(v, v.size, cbits, V, _u16(lut16).reshape(-1), out)
    return out


def tcq_encode(v, s, L, T, V, lut16, *, method="viterbi"):
    """One tile.  Returns (stream bytes, squared error)."""
    v = np.ascontiguousarray(v, dtype=np.float64).reshape(-1)
    assert v.size == T
    out = np.zeros((s * T // V + 7) // 8 + 4, dtype=np.uint8)
    f = {"viterbi": lib().qpo_tcq_encode_viterbi, "exact": lib().qpo_tcq_encode_viterbi_exact,
         "brute": lib().qpo_tcq_encode_brute}[method]
    e = f(v, s, L, T, V, _u16(lut16).reshape(-1), out)
    return out[: (s * T // V + 7) // 8], e


def tcq_encode_tiles(v, s, L, T, V, lut16):
    """Many tiles (threads over tiles).  v: [ntiles, T].  Returns (streams [ntiles, bytes], errs)."""
    v = np.ascontiguousarray(v, dtype=np.float64)
    nt = v.shape[0]
    tb = s * T // V // 8
    streams = np.zeros((nt, tb), dtype=np.uint8)
    errs = np.zeros(nt, dtype=np.float64)
    lib().qpo_tcq_encode_tiles(v.reshape(-1), nt, s, L, T, V, _u16(lut16).reshape(-1),
                               streams.reshape(-1), errs)
    return streams, errs


def tcq_encode_constrained(v, s, L, T, V, lut16, overlap: int):
    """One tile, the first L - s stream bits fixed to `overlap`: exact optimum for that value.
    Returns (stream bytes, squared error)."""
    v = np.ascontiguousarray(v, dtype=np.float64).reshape(-1)
    assert v.size == T
    nb = (s * T // V + 7) // 8
    out = np.zeros(nb + 4, dtype=np.uint8)
    e = lib().qpo_tcq_encode_constrained(v, s, L, T, V, _u16(lut16).reshape(-1), int(overlap), out)
    return out[:nb], e


def tcq_tile_error(v, stream, s, L, T, V, lut16) -> float:
    """Squared error between v and the tail-biting decode of one tile's stream."""
    v = np.ascontiguousarray(v, dtype=np.float64).reshape(-1)
    st = np.ascontiguousarray(stream, dtype=np.uint8)
    return lib().qpo_tcq_tile_error(v, st, s, L, T, V, _u16(lut16).reshape(-1))


def _samples(x) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float64)
    return x.reshape(-1, 1) if x.ndim == 1 else x


def kmeans_assign(x, centres):
    """(assignment int32 [n], inertia) of one assignment step (ties: the lowest index)."""
    x = _samples(x)
    m = np.ascontiguousarray(_samples(centres))
    a = np.empty(x.shape[0], dtype=np.int32)
    inertia = lib().qpo_kmeans_assign(x, x.shape[0], x.shape[1], m, m.shape[0], a)
    return a, float(inertia)


def kmeans_update(x, assign, centres):
    """(new centres, counts, total squared movement) of one update step."""
    x = _samples(x)
    m = np.ascontiguousarray(_samples(centres))
    out = np.empty_like(m)
    count = np.empty(m.shape[0], dtype=np.int64)
    moved = lib().qpo_kmeans_update(x, x.shape[0], x.shape[1], np.ascontiguousarray(assign, dtype=np.int32), m,
                                    m.shape[0], out, count)
    return out, count, float(moved)


def kmeans(x, init, max_iter: int = 300, tol: float = 1e-6):
    """Lloyd's algorithm from `init`: (centres, updates made, inertia of the last assignment)."""
    x = _samples(x)
    m = np.array(_samples(init), dtype=np.float64, order="C", copy=True)
    inertia = C.c_double(0.0)
    it = lib().qpo_kmeans(x, x.shape[0], x.shape[1], m, m.shape[0], int(max_iter), float(tol), C.byref(inertia))
    return m, int(it), float(inertia.value)
