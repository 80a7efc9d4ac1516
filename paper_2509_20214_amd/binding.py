"""ctypes binding of libqp.so.  Argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libqp.so")

QP_SQ, QP_VQ, QP_TCQ, QP_TCQH, QP_TCQHH = 0, 1, 2, 3, 4
QP_LAYOUT_CANONICAL, QP_LAYOUT_NATIVE = 0, 1
QP_OK = 0

EXPORTS = ["qp_linear", "qp_dequant", "qp_hadamard", "qp_repack", "qp_native_bytes",
           "qp_linear_workspace_bytes", "qp_validate", "qp_status_string", "qp_version",
           "qp_rotate_linear", "qp_rotate_linear_workspace_bytes", "qp_rotate_linear_launches", "qp_encode", "qp_encode_workspace_bytes",
           "qp_row_normalize", "qp_msq_solve", "qp_kmeans", "qp_kmeans_workspace_bytes",
           "qp_set_option", "qp_get_option", "qp_reset_options", "qp_rotate_linear_static",
           "qp_rotate_linear_static_max_bytes", "qp_bench_stream_read", "qp_bench_empty_launch", "qp_msq_solve_fused",
           "qp_block_workspace_bytes", "qp_block_enqueue", "qp_block_create", "qp_block_run", "qp_block_destroy"]

# qp_option (include/qp.h)
QP_OPT_LINEAR_KERNEL, QP_OPT_DEQUANT_KERNEL, QP_OPT_ROTATE_SPLIT, QP_OPT_LINEAR_PACK = 0, 1, 2, 3
QP_OPT_LINEAR_SPLIT, QP_OPT_WG_PER_CU, QP_OPT_NW, QP_OPT_TABLE_LATE_MAX = 4, 5, 6, 7
QP_KERNEL_AUTO, QP_KERNEL_ROW, QP_KERNEL_BLOCK = 0, 1, 2            # values of QP_OPT_LINEAR_KERNEL
QP_DEQUANT_AUTO, QP_DEQUANT_GENERIC, QP_DEQUANT_BLOCKS = 0, 1, 2    # values of QP_OPT_DEQUANT_KERNEL


class qp_weight(C.Structure):
    _fields_ = [("scheme", C.c_int32), ("M", C.c_int32), ("N", C.c_int32), ("code_bits", C.c_int32),
                ("vec", C.c_int32), ("window_bits", C.c_int32), ("tile", C.c_int32), ("layout", C.c_int32),
                ("row_stride", C.c_int64), ("codes", C.c_void_p), ("lut", C.c_void_p), ("scales", C.c_void_p),
                ("tlut_bits", C.c_int32), ("reserved", C.c_int32)]


class qp_block_item(C.Structure):
    _fields_ = [("w", C.POINTER(qp_weight)), ("x", C.c_void_p), ("signs", C.c_void_p), ("block", C.c_int32),
                ("B", C.c_int32), ("ldx", C.c_int64), ("y", C.c_void_p), ("ldy", C.c_int64)]


class QpError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: qp_status {code} ({qp_status_string(code)})")
        self.code = code


_lib = None


def load_library(build_if_missing: bool = True):
    """Load libqp.so (building it with hipcc first if it is not there).  Raises if
    neither works: there is no fallback implementation."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        if not build_if_missing:
            raise FileNotFoundError(LIB_PATH)
        from . import build as _b
        _b.build()
    # PyTorch ships its own copy of the HIP runtime.  It must be the one already in the
    # process when libqp.so resolves libamdhip64: with two runtimes loaded, kernels registered
    # in one cannot be launched on device pointers and streams that belong to the other.
    import torch  # noqa: F401
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    wp = C.POINTER(qp_weight)
    L.qp_linear.restype = C.c_int
    L.qp_linear.argtypes = [wp, vp, i32, i64, vp, i64, vp, sz, vp]
    L.qp_rotate_linear.restype = C.c_int
    L.qp_rotate_linear.argtypes = [wp, vp, vp, i32, i32, i64, vp, i64, vp, sz, vp]
    L.qp_rotate_linear_static.restype = C.c_int
    L.qp_rotate_linear_static.argtypes = [wp, vp, vp, i32, i32, i64, vp, i64, vp]
    L.qp_rotate_linear_static_max_bytes.restype = sz
    L.qp_rotate_linear_static_max_bytes.argtypes = []
    bp = C.POINTER(qp_block_item)
    L.qp_block_workspace_bytes.restype = sz
    L.qp_block_workspace_bytes.argtypes = [bp, i32]
    L.qp_block_enqueue.restype = C.c_int
    L.qp_block_enqueue.argtypes = [bp, i32, vp, sz, vp]
    L.qp_block_create.restype = C.c_int
    L.qp_block_create.argtypes = [bp, i32, vp, sz, C.POINTER(vp)]
    L.qp_block_run.restype = C.c_int
    L.qp_block_run.argtypes = [vp, vp]
    L.qp_block_destroy.restype = C.c_int
    L.qp_block_destroy.argtypes = [vp]
    L.qp_bench_stream_read.restype = C.c_int
    L.qp_bench_stream_read.argtypes = [vp, sz, vp, vp]
    L.qp_bench_empty_launch.restype = C.c_int
    L.qp_bench_empty_launch.argtypes = [vp]
    L.qp_rotate_linear_workspace_bytes.restype = sz
    L.qp_rotate_linear_workspace_bytes.argtypes = [wp, i32]
    L.qp_rotate_linear_launches.restype = i32
    L.qp_rotate_linear_launches.argtypes = [wp, i32, i32]
    L.qp_dequant.restype = C.c_int
    L.qp_dequant.argtypes = [wp, vp, vp]
    L.qp_encode.restype = C.c_int
    L.qp_encode.argtypes = [wp, vp, i64, vp, vp, vp, sz, vp]
    L.qp_row_normalize.restype = C.c_int
    L.qp_row_normalize.argtypes = [vp, i64, i32, i32, vp, vp]
    L.qp_msq_solve.restype = C.c_int
    L.qp_msq_solve.argtypes = [i32, C.POINTER(C.c_int32), C.POINTER(C.c_double), C.POINTER(C.c_double), C.c_double,
                               i32, C.POINTER(C.c_int32), C.POINTER(C.c_double), C.POINTER(C.c_double)]
    L.qp_msq_solve_fused.restype = C.c_int
    L.qp_msq_solve_fused.argtypes = [i32, i32, C.POINTER(C.c_double), C.POINTER(C.c_double), C.c_double, i32, i32,
                                     C.POINTER(C.c_int32), C.POINTER(C.c_double), C.POINTER(C.c_double)]
    L.qp_encode_workspace_bytes.restype = sz
    L.qp_encode_workspace_bytes.argtypes = [wp]
    L.qp_kmeans.restype = C.c_int
    L.qp_kmeans.argtypes = [vp, i64, i32, vp, i32, i32, C.c_float, vp, sz, vp, vp, vp, vp]
    L.qp_kmeans_workspace_bytes.restype = sz
    L.qp_kmeans_workspace_bytes.argtypes = [i32, i32]
    L.qp_hadamard.restype = C.c_int
    L.qp_hadamard.argtypes = [vp, vp, i32, i32, i32, i64, vp, i64, vp]
    L.qp_repack.restype = C.c_int
    L.qp_repack.argtypes = [wp, wp, vp, sz, vp]
    L.qp_native_bytes.restype = sz
    L.qp_native_bytes.argtypes = [wp]
    L.qp_linear_workspace_bytes.restype = sz
    L.qp_linear_workspace_bytes.argtypes = [wp, i32]
    L.qp_validate.restype = C.c_int
    L.qp_validate.argtypes = [wp]
    L.qp_status_string.restype = C.c_char_p
    L.qp_status_string.argtypes = [C.c_int]
    L.qp_version.restype = i32
    L.qp_version.argtypes = []
    L.qp_set_option.restype = C.c_int
    L.qp_set_option.argtypes = [i32, i32]
    L.qp_get_option.restype = i32
    L.qp_get_option.argtypes = [i32]
    L.qp_reset_options.restype = None
    L.qp_reset_options.argtypes = []
    _lib = L
    return L


def qp_status_string(code: int) -> str:
    return load_library().qp_status_string(int(code)).decode()


def qp_version() -> int:
    return int(load_library().qp_version())


def qp_set_option(option: int, value: int) -> None:
    _check(load_library().qp_set_option(int(option), int(value)), "qp_set_option")


def qp_get_option(option: int) -> int:
    return int(load_library().qp_get_option(int(option)))


def qp_reset_options() -> None:
    load_library().qp_reset_options()


def _stream_ptr(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _scratch(nbytes: int, device, stream):
    """A temporary workspace that this module allocates itself.  It comes from torch's caching
    allocator, which would hand the block out again as soon as the tensor is dropped as far as the
    CURRENT stream is concerned; the kernels run on `stream`, so the block is tied to that one too."""
    import torch
    t = torch.empty(nbytes, dtype=torch.uint8, device=device)
    if stream is not None:
        t.record_stream(stream)
    return t


def _check(code: int, what: str):
    if code != QP_OK:
        raise QpError(code, what)


class Weight:
    """A quantized layer resident on the device: torch tensors (owned here) plus the
    C descriptor that points at them."""

    def __init__(self, scheme, M, N, code_bits, vec, window_bits, tile, codes, lut, scales,
                 layout=QP_LAYOUT_CANONICAL, row_stride=None, tlut_bits=0):
        self.codes, self.lut, self.scales = codes, lut, scales
        if row_stride is None:
            row_stride = codes.shape[1] if (layout == QP_LAYOUT_CANONICAL and codes.dim() == 2) else 0
        self.desc = qp_weight(scheme, M, N, code_bits, vec, window_bits, tile, layout, row_stride,
                              codes.data_ptr(), lut.data_ptr(), scales.data_ptr(), tlut_bits, 0)

    @classmethod
    def from_layer(cls, layer, device="cuda"):
        """Upload a synth.Layer-like object (numpy arrays, canonical layout)."""
        import numpy as np
        import torch
        codes = torch.from_numpy(np.ascontiguousarray(layer.codes)).to(device)
        lut = torch.from_numpy(np.ascontiguousarray(layer.lut).view(np.int16)).to(device)
        scales = torch.from_numpy(np.ascontiguousarray(layer.scales).view(np.int16)).to(device)
        return cls(layer.scheme, layer.M, layer.N, layer.code_bits, layer.vec, layer.window_bits,
                   layer.tile, codes, lut, scales, tlut_bits=getattr(layer, "tlut_bits", 0))

    def with_codes(self, codes):
        """Same layer (table and scales shared) over another buffer of codes in the same layout."""
        d = self.desc
        return Weight(d.scheme, d.M, d.N, d.code_bits, d.vec, d.window_bits, d.tile, codes, self.lut, self.scales,
                      layout=d.layout, row_stride=d.row_stride, tlut_bits=d.tlut_bits)

    @property
    def M(self):
        return self.desc.M

    @property
    def N(self):
        return self.desc.N

    @property
    def code_bytes(self) -> int:
        d = self.desc
        if d.scheme == QP_TCQHH:   # code_bits per step on the first half of the columns, one more on the second
            return d.M * (d.N // 4 * (2 * d.code_bits + 1) // 8)
        return d.M * ((d.N // d.vec * d.code_bits + 7) // 8)


def qp_validate(w: Weight) -> int:
    return int(load_library().qp_validate(C.byref(w.desc)))


def qp_native_bytes(w: Weight) -> int:
    return int(load_library().qp_native_bytes(C.byref(w.desc)))


def qp_linear_workspace_bytes(w: Weight, B: int) -> int:
    return int(load_library().qp_linear_workspace_bytes(C.byref(w.desc), B))


def qp_repack(w: Weight, stream=None) -> Weight:
    """Canonical -> native copy of the codes (LUT and scales are shared)."""
    import torch
    nbytes = qp_native_bytes(w)
    if nbytes == 0:
        raise QpError(5, "qp_repack")
    out = torch.empty(nbytes, dtype=torch.uint8, device=w.codes.device)
    d = w.desc
    nw = Weight(d.scheme, d.M, d.N, d.code_bits, d.vec, d.window_bits, d.tile, out, w.lut, w.scales,
                layout=QP_LAYOUT_NATIVE, row_stride=0, tlut_bits=d.tlut_bits)
    tmp = qp_weight()
    _check(load_library().qp_repack(C.byref(w.desc), C.byref(tmp), out.data_ptr(), nbytes,
                                    _stream_ptr(stream)), "qp_repack")
    nw.desc = tmp
    return nw


def qp_encode(w: Weight, W, tile_err: bool = False, workspace=None, stream=None):
    """Quantize the fp16 targets W [M, N] into w's own code buffer (canonical layout; the buffer's
    previous contents are replaced).  Returns the fp32 [M, N/256] tile errors when asked for
    (trellis schemes), else None."""
    import torch
    d = w.desc
    need = int(load_library().qp_encode_workspace_bytes(C.byref(d)))
    if workspace is None and need:
        workspace = _scratch(need, W.device, stream)
    err = torch.zeros((d.M, d.N // 256), dtype=torch.float32, device=W.device) if tile_err else None
    _check(load_library().qp_encode(C.byref(d), W.data_ptr(), W.stride(0), w.codes.data_ptr(),
                                    err.data_ptr() if err is not None else None,
                                    workspace.data_ptr() if workspace is not None else None,
                                    workspace.numel() if workspace is not None else 0, _stream_ptr(stream)),
           "qp_encode")
    return err


def qp_row_normalize(W, scales=None, stream=None):
    """In place: every row of the fp16 matrix W divided by its root mean square; returns the
    fp16 scales [M]."""
    import torch
    M, N = W.shape
    if scales is None:
        scales = torch.empty(M, dtype=torch.float16, device=W.device)
    _check(load_library().qp_row_normalize(W.data_ptr(), W.stride(0), M, N, scales.data_ptr(), _stream_ptr(stream)),
           "qp_row_normalize")
    return scales


def qp_kmeans_workspace_bytes(k: int, d: int) -> int:
    return int(load_library().qp_kmeans_workspace_bytes(k, d))


def qp_kmeans(samples, centres, max_iter: int = 300, tol: float = 1e-6, assign=None, centres_f16=None,
              stats=None, workspace=None, stream=None):
    """Lloyd's algorithm on the device.  samples: fp32 [n] or [n, d]; centres: fp32 [k] or [k, d], start
    on entry, result on return (in place).  Optional device outputs: assign int32 [n], centres_f16
    fp16 like centres, stats float64 [3] (inertia of the last assignment, updates made, last
    movement).  Returns centres; nothing is synchronised."""
    import torch
    n = samples.shape[0]
    d = 1 if samples.dim() == 1 else samples.shape[1]
    k = centres.shape[0]
    if not (samples.is_contiguous() and centres.is_contiguous()):
        raise ValueError("samples and centres must be contiguous")
    if samples.dtype != torch.float32 or centres.dtype != torch.float32:
        raise ValueError("samples and centres must be float32")
    nbytes = qp_kmeans_workspace_bytes(k, d)
    if workspace is None:
        workspace = _scratch(max(nbytes, 16), samples.device, stream)
    _check(load_library().qp_kmeans(samples.data_ptr(), n, d, centres.data_ptr(), k, int(max_iter), float(tol),
                                    workspace.data_ptr(), workspace.numel(),
                                    assign.data_ptr() if assign is not None else None,
                                    centres_f16.data_ptr() if centres_f16 is not None else None,
                                    stats.data_ptr() if stats is not None else None, _stream_ptr(stream)),
           "qp_kmeans")
    return centres


def qp_msq_solve(classes, budget: float, resolution: int = 20000):
    """classes: list of lists of (loss, cost).  Returns (choices, total_loss, total_cost)."""
    n = len(classes)
    begin = (C.c_int32 * (n + 1))()
    flat = [oc for cl in classes for oc in cl]
    for i, cl in enumerate(classes):
        begin[i + 1] = begin[i] + len(cl)
    loss = (C.c_double * len(flat))(*[float(l) for l, _ in flat])
    cost = (C.c_double * len(flat))(*[float(c) for _, c in flat])
    choice = (C.c_int32 * n)()
    tl, tc = C.c_double(), C.c_double()
    _check(load_library().qp_msq_solve(n, begin, loss, cost, float(budget), int(resolution), choice,
                                       C.byref(tl), C.byref(tc)), "qp_msq_solve")
    return list(choice), tl.value, tc.value


def qp_encode_workspace_bytes(w: Weight) -> int:
    return int(load_library().qp_encode_workspace_bytes(C.byref(w.desc)))


def qp_linear(w: Weight, x, y=None, workspace=None, stream=None):
    """y[b, j] = s[j] * sum_i x[b, i] W^[j, i].  x: fp16 [B, N] (row stride = x.stride(0)).
    workspace: uint8 tensor of qp_linear_workspace_bytes(w, B) bytes, None (allocated here when the
    layer wants one) or False (none: the layer reads x in place; same result)."""
    import torch
    B = x.shape[0]
    if y is None:
        y = torch.empty((B, w.M), dtype=torch.float16, device=x.device)
    if workspace is None:   # allocate what the layer asks for (usually nothing); workspace=False: none
        need = qp_linear_workspace_bytes(w, B)
        workspace = _scratch(need, x.device, stream) if need else False
    ws_ptr, ws_bytes = (None, 0) if workspace is False else (workspace.data_ptr(), workspace.numel() * workspace.element_size())
    _check(load_library().qp_linear(C.byref(w.desc), x.data_ptr(), B, x.stride(0), y.data_ptr(), y.stride(0),
                                    ws_ptr, ws_bytes, _stream_ptr(stream)), "qp_linear")
    return y


def qp_dequant(w: Weight, out=None, stream=None):
    import torch
    if out is None:
        out = torch.empty((w.M, w.N), dtype=torch.float16, device=w.codes.device)
    _check(load_library().qp_dequant(C.byref(w.desc), out.data_ptr(), _stream_ptr(stream)), "qp_dequant")
    return out


def qp_hadamard(x, signs, block: int, out=None, stream=None):
    """xr = H_block (signs .* x) / sqrt(block) per contiguous block of each row."""
    import torch
    B, n = x.shape
    if out is None:
        out = torch.empty_like(x)
    _check(load_library().qp_hadamard(x.data_ptr(), signs.data_ptr(), B, n, block, x.stride(0),
                                      out.data_ptr(), out.stride(0), _stream_ptr(stream)), "qp_hadamard")
    return out


def qp_rotate_linear_workspace_bytes(w: Weight, B: int) -> int:
    return int(load_library().qp_rotate_linear_workspace_bytes(C.byref(w.desc), B))


def qp_rotate_linear_launches(w: Weight, B: int, block: int) -> int:
    return int(load_library().qp_rotate_linear_launches(C.byref(w.desc), B, block))


def qp_rotate_linear(w: Weight, x, signs, block: int, y=None, workspace=None, stream=None):
    """y = (H_block(signs .* x) / sqrt(block)) W^T diag(s), rotation and layer in one call.
    workspace: uint8 tensor of qp_rotate_linear_workspace_bytes(w, B) bytes (allocated here
    when None; pass one in to reuse it)."""
    import torch
    B = x.shape[0]
    if y is None:
        y = torch.empty((B, w.M), dtype=torch.float16, device=x.device)
    if workspace is None:
        workspace = _scratch(qp_rotate_linear_workspace_bytes(w, B), x.device, stream)
    _check(load_library().qp_rotate_linear(C.byref(w.desc), x.data_ptr(), signs.data_ptr(), block, B, x.stride(0),
                                           y.data_ptr(), y.stride(0), workspace.data_ptr(),
                                           workspace.numel(), _stream_ptr(stream)), "qp_rotate_linear")
    return y


def qp_rotate_linear_static_max_bytes() -> int:
    return int(load_library().qp_rotate_linear_static_max_bytes())


def qp_rotate_linear_static(w: Weight, x, signs, block: int, y, stream=None):
    """qp_rotate_linear through the library's own fixed scratch array: nothing is allocated, so the
    output y (fp16 [B, M]) must be passed in."""
    B = x.shape[0]
    _check(load_library().qp_rotate_linear_static(C.byref(w.desc), x.data_ptr(), signs.data_ptr(), block, B,
                                                  x.stride(0), y.data_ptr(), y.stride(0), _stream_ptr(stream)),
           "qp_rotate_linear_static")
    return y


class Block:
    """A decoder block's rotations and layers as one unit: `items` is a list of (Weight, x, signs, block, y)
    with x fp16 [B, N] unrotated and y fp16 [B, M]; the tensors (and the workspace made here) are kept alive
    by this object.  enqueue() launches the sequence, graph() captures it once into a graph that the
    library owns and run() replays it."""

    def __init__(self, items):
        import torch
        self.items = list(items)
        self._arr = (qp_block_item * len(self.items))()
        for a, (w, x, signs, block, y) in zip(self._arr, self.items):
            a.w, a.x, a.signs, a.block = C.pointer(w.desc), x.data_ptr(), signs.data_ptr(), block
            a.B, a.ldx, a.y, a.ldy = x.shape[0], x.stride(0), y.data_ptr(), y.stride(0)
        need = qp_block_workspace_bytes(self)
        self.workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=self.items[0][1].device)
        self._handle = None

    def enqueue(self, stream=None):
        qp_block_enqueue(self, stream)

    def graph(self):
        if self._handle is None:
            self._handle = qp_block_create(self)
        return self

    def run(self, stream=None):
        qp_block_run(self.graph()._handle, stream)

    def close(self):
        if self._handle is not None:
            qp_block_destroy(self._handle)
            self._handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def qp_block_workspace_bytes(blk: "Block") -> int:
    return int(load_library().qp_block_workspace_bytes(blk._arr, len(blk._arr)))


def qp_block_enqueue(blk: "Block", stream=None):
    _check(load_library().qp_block_enqueue(blk._arr, len(blk._arr), blk.workspace.data_ptr(), blk.workspace.numel(),
                                           _stream_ptr(stream)), "qp_block_enqueue")


def qp_block_create(blk: "Block"):
    h = C.c_void_p()
    _check(load_library().qp_block_create(blk._arr, len(blk._arr), blk.workspace.data_ptr(), blk.workspace.numel(),
                                          C.byref(h)), "qp_block_create")
    return h


def qp_block_run(handle, stream=None):
    _check(load_library().qp_block_run(handle, _stream_ptr(stream)), "qp_block_run")


def qp_block_destroy(handle):
    _check(load_library().qp_block_destroy(handle), "qp_block_destroy")


def qp_bench_stream_read(data, sink, stream=None):
    """Enqueue the read-only streaming kernel over the bytes of the tensor `data` (a yardstick, see qp.h)."""
    _check(load_library().qp_bench_stream_read(data.data_ptr(), data.numel() * data.element_size(), sink.data_ptr(),
                                               _stream_ptr(stream)), "qp_bench_stream_read")


def qp_bench_empty_launch(stream=None):
    _check(load_library().qp_bench_empty_launch(_stream_ptr(stream)), "qp_bench_empty_launch")
