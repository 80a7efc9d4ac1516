"""Host-side checks of the C-ABI library: it loads, exports every symbol the header
declares, and turns bad arguments into QP_ERR_* codes without touching a device
(no compute call is made here)."""
import ctypes as C
import os
import re

import pytest

import paper_2509_20214_amd as qp
from paper_2509_20214_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_symbols():
    src = open(os.path.join(ROOT, "include", "qp.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(qp_[a-z_]+)\s*\(", src)))


def test_library_loads_and_exports_every_declared_symbol():
    L = qp.load_library()
    syms = header_symbols()
    assert set(syms) == set(binding.EXPORTS)
    for s in syms:
        assert hasattr(L, s), s
    assert qp.qp_version() >= 200
    assert qp.qp_status_string(0) == "ok"
    for code in range(1, 8):
        assert qp.qp_status_string(code) not in ("ok", "unknown status")


def desc(**kw):
    d = dict(scheme=qp.QP_SQ, M=16, N=1024, code_bits=4, vec=1, window_bits=0, tile=0,
             layout=qp.QP_LAYOUT_CANONICAL, row_stride=512, codes=0x1000, lut=0x2000, scales=0x3000)
    d.update(kw)
    return binding.qp_weight(**d)


@pytest.mark.parametrize("kw,code", [
    (dict(), 0),
    (dict(scheme=7), 3),
    (dict(code_bits=3), 3),
    (dict(scheme=qp.QP_VQ, vec=2, code_bits=6), 3),
    (dict(scheme=qp.QP_VQ, vec=2, code_bits=5, row_stride=320), 0),
    (dict(scheme=qp.QP_TCQ, code_bits=2, window_bits=16, tile=256, row_stride=256), 0),
    # a row of 52 codes of 5 bits = 260 bits ends inside its 33rd byte: 32 bytes are one too few
    (dict(scheme=qp.QP_VQ, vec=2, code_bits=5, N=104, row_stride=32), 2),
    (dict(scheme=qp.QP_VQ, vec=2, code_bits=5, N=104, row_stride=48), 0),
    (dict(scheme=qp.QP_VQ, vec=2, code_bits=7, N=120, row_stride=48), 2),   # 420 bits = 52.5 bytes
    (dict(scheme=qp.QP_VQ, vec=2, code_bits=7, N=120, row_stride=64), 0),
    (dict(scheme=qp.QP_TCQ, code_bits=2, window_bits=12, tile=256, row_stride=256), 3),
    (dict(scheme=qp.QP_TCQ, code_bits=3, window_bits=16, tile=256, N=1000, row_stride=384), 2),
    (dict(scheme=qp.QP_TCQH, vec=2, code_bits=5, window_bits=16, tile=256, tlut_bits=9, row_stride=320), 0),
    (dict(scheme=qp.QP_TCQH, vec=2, code_bits=5, window_bits=16, tile=256, tlut_bits=10, row_stride=320), 3),
    (dict(scheme=qp.QP_TCQH, vec=2, code_bits=9, window_bits=16, tile=256, tlut_bits=9, row_stride=576), 3),
    (dict(scheme=qp.QP_TCQH, vec=2, code_bits=9, window_bits=16, tile=256, tlut_bits=10, row_stride=576), 0),
    (dict(scheme=qp.QP_TCQH, vec=2, code_bits=10, window_bits=16, tile=256, tlut_bits=11, row_stride=640), 0),
    (dict(scheme=qp.QP_TCQH, vec=2, code_bits=10, window_bits=16, tile=256, tlut_bits=10, row_stride=640), 3),
    (dict(scheme=qp.QP_TCQH, vec=2, code_bits=11, window_bits=16, tile=256, tlut_bits=11, row_stride=704), 3),
    (dict(scheme=qp.QP_TCQH, vec=1, code_bits=4, window_bits=16, tile=256, tlut_bits=9, row_stride=512), 3),
    # half-TCQ: s = 4 and 5 bits per step -> 1024/4 * 9/8 = 288 bytes per row; table of s + 1
    (dict(scheme=qp.QP_TCQHH, vec=2, code_bits=4, window_bits=16, tile=256, tlut_bits=9, row_stride=288), 0),
    (dict(scheme=qp.QP_TCQHH, vec=2, code_bits=8, window_bits=16, tile=256, tlut_bits=10, row_stride=544), 0),
    (dict(scheme=qp.QP_TCQHH, vec=2, code_bits=8, window_bits=16, tile=256, tlut_bits=9, row_stride=544), 3),
    (dict(scheme=qp.QP_TCQHH, vec=2, code_bits=10, window_bits=16, tile=256, tlut_bits=11, row_stride=672), 3),
    (dict(scheme=qp.QP_TCQHH, vec=2, code_bits=4, window_bits=16, tile=256, tlut_bits=9, row_stride=272), 2),
    (dict(scheme=qp.QP_TCQHH, vec=2, code_bits=4, window_bits=16, tile=256, tlut_bits=9, N=768, row_stride=224), 2),
    (dict(scheme=qp.QP_TCQHH, vec=2, code_bits=4, window_bits=16, tile=256, tlut_bits=9, row_stride=288,
          layout=qp.QP_LAYOUT_NATIVE), 5),
    (dict(scheme=qp.QP_TCQHH, vec=2, code_bits=4, window_bits=16, tile=256, tlut_bits=9, N=2048, row_stride=576,
          layout=qp.QP_LAYOUT_NATIVE), 0),
    (dict(M=0), 2),
    (dict(N=1020), 2),
    (dict(codes=0), 1),
    (dict(lut=0), 1),
    (dict(scales=0), 1),
    (dict(row_stride=500), 4),
    (dict(row_stride=256), 2),
    (dict(codes=0x1004), 4),
    (dict(layout=5), 5),
    (dict(layout=qp.QP_LAYOUT_NATIVE, M=24), 5),
    (dict(layout=qp.QP_LAYOUT_NATIVE, N=1024 + 256, row_stride=640), 0),   # a last column block cut short: whole spans of 256
    (dict(layout=qp.QP_LAYOUT_NATIVE, N=1024 + 128, row_stride=640), 5),
])
def test_descriptor_validation(kw, code):
    d = desc(**kw)
    assert qp.load_library().qp_validate(C.byref(d)) == code


def test_null_descriptor():
    L = qp.load_library()
    assert L.qp_validate(None) == 1
    assert L.qp_native_bytes(None) == 0


def test_linear_argument_errors_do_not_launch():
    L = qp.load_library()
    d = desc()
    call = lambda x, B, ldx, y, ldy: L.qp_linear(C.byref(d), x, B, ldx, y, ldy, None, 0, None)
    assert call(None, 1, 1024, 0x5000, 16) == 1
    assert call(0x4000, 1, 1024, None, 16) == 1
    assert call(0x4000, 0, 1024, 0x5000, 16) == 2
    assert call(0x4000, 17, 1024, 0x5000, 16) == 2
    assert call(0x4000, 1, 1000, 0x5000, 16) == 2
    assert call(0x4000, 1, 1028, 0x5000, 16) == 2
    assert call(0x4000, 1, (1 << 26) + 8, 0x5000, 16) == 2      # row stride beyond QP_MAX_LDX
    assert call(0x4000, 1, 1024, 0x5000, 8) == 2
    assert call(0x4008, 1, 1024, 0x5000, 16) == 4
    assert L.qp_dequant(C.byref(d), None, None) == 1
    assert L.qp_dequant(C.byref(d), 0x5004, None) == 4


def test_linear_workspace_sizes():
    """Host logic only: which layers and batch sizes want the optional workspace, and how much."""
    L = qp.load_library()
    big = desc(scheme=qp.QP_VQ, vec=2, code_bits=7, M=8192, N=16384, row_stride=7168)       # 2^27 weights
    mid = desc(scheme=qp.QP_VQ, vec=2, code_bits=5, M=8192, N=4096, row_stride=1280)        # 2^25
    small = desc(scheme=qp.QP_VQ, vec=2, code_bits=5, M=4096, N=4096, row_stride=1280)      # 2^24
    tcq = desc(scheme=qp.QP_TCQ, code_bits=3, window_bits=16, tile=256, M=8192, N=16384, row_stride=6144)
    tiny = desc()                                                                            # row kernel
    ws = lambda d, B: L.qp_linear_workspace_bytes(C.byref(d), B)
    assert [ws(big, B) for B in (1, 4, 5, 8, 9, 16)] == [0, 0, 8 * 16384 * 2, 8 * 16384 * 2, 16 * 16384 * 2, 16 * 16384 * 2]
    assert [ws(mid, B) for B in (1, 8, 9, 16)] == [0, 0, 16 * 4096 * 2, 16 * 4096 * 2]
    assert [ws(small, B) for B in (8, 16)] == [0, 0]
    assert [ws(tcq, B) for B in (5, 8, 9)] == [0, 0, 16 * 16384 * 2]
    assert [ws(tiny, B) for B in (1, 16)] == [0, 0]
    assert ws(big, 0) == 0 and ws(big, 17) == 0 and L.qp_linear_workspace_bytes(None, 8) == 0


def test_hadamard_argument_errors_do_not_launch():
    L = qp.load_library()
    call = lambda x, s, B, n, blk, ldx, xr, ldxr: L.qp_hadamard(x, s, B, n, blk, ldx, xr, ldxr, None)
    ok = (0x4000, 0x5000, 1, 1024, 1024, 1024, 0x8000, 1024)
    assert call(None, *ok[1:]) == 1
    assert call(0x4000, None, *ok[2:]) == 1
    assert call(*ok[:6], None, 1024) == 1
    assert call(0x4000, 0x5000, 0, 1024, 1024, 1024, 0x8000, 1024) == 2
    assert call(0x4000, 0x5000, 1, 1024, 768, 1024, 0x8000, 1024) == 2      # not a power of two
    assert call(0x4000, 0x5000, 1, 1024, 1, 1024, 0x8000, 1024) == 2
    assert call(0x4000, 0x5000, 1, 1536, 1024, 1536, 0x8000, 1536) == 2     # block does not divide n
    assert call(0x4000, 0x5000, 1, 1024, 1024, 512, 0x8000, 1024) == 2
    assert call(0x4000, 0x5000, 1, 1024, 1024, 1024, 0x4400, 1024) == 4     # partial overlap


def test_rotate_linear_argument_errors_do_not_launch():
    L = qp.load_library()
    d = desc()
    need = L.qp_rotate_linear_workspace_bytes(C.byref(d), 1)
    assert need == 2048
    call = lambda x, s, blk, B, ldx, y, ldy, ws, n: L.qp_rotate_linear(C.byref(d), x, s, blk, B, ldx, y, ldy, ws, n, None)
    ok = (0x4000, 0x5000, 1024, 1, 1024, 0x6000, 16, 0x10000, need)
    assert call(None, *ok[1:]) == 1
    assert call(0x4000, None, *ok[2:]) == 1
    assert call(*ok[:7], None, need) == 1
    assert call(*ok[:8], need - 1) == 7
    assert call(0x4000, 0x5000, 768, 1, 1024, 0x6000, 16, 0x10000, need) == 2
    assert call(0x4000, 0x5000, 1024, 0, 1024, 0x6000, 16, 0x10000, need) == 2
    assert call(0x4000, 0x5000, 1024, 1, 1024, 0x6000, 16, 0x10010, need) == 4
    assert L.qp_rotate_linear_workspace_bytes(None, 1) == 0
    assert L.qp_rotate_linear_launches(None, 1, 1024) == 0
    assert L.qp_rotate_linear_launches(C.byref(d), 2, 1024) == 2


def test_repack_argument_errors_do_not_launch():
    L = qp.load_library()
    out = binding.qp_weight()
    d = desc()
    assert L.qp_native_bytes(C.byref(d)) == 16 * 512
    assert L.qp_native_bytes(C.byref(desc(M=24))) == 0
    # N = 1280: two column blocks, the second padded from 256 to 1024 columns; N = 1152: no native form
    assert L.qp_native_bytes(C.byref(desc(N=1280, row_stride=640))) == 16 * 1024
    assert L.qp_native_bytes(C.byref(desc(N=1152, row_stride=640))) == 0
    assert L.qp_repack(C.byref(desc(N=1280, row_stride=640)), C.byref(out), 0x100000, 16 * 640, None) == 2   # room for the padding too
    assert L.qp_repack(C.byref(d), C.byref(out), None, 16 * 512, None) == 1
    assert L.qp_repack(C.byref(d), C.byref(out), 0x100000, 100, None) == 2
    assert L.qp_repack(C.byref(desc(M=24)), C.byref(out), 0x100000, 1 << 20, None) == 5
    assert L.qp_repack(C.byref(desc(layout=qp.QP_LAYOUT_NATIVE)), C.byref(out), 0x100000, 1 << 20, None) == 5
    assert L.qp_repack(C.byref(d), C.byref(out), 0x1100, 1 << 20, None) == 4   # overlaps the source
    sizes = {(qp.QP_VQ, 5, 2): 16 * 320, (qp.QP_VQ, 7, 2): 16 * 448, (qp.QP_TCQ, 3, 1): 16 * 384}
    for (s, cb, v), want in sizes.items():
        dd = desc(scheme=s, code_bits=cb, vec=v, window_bits=16 if s == qp.QP_TCQ else 0,
                  tile=256 if s == qp.QP_TCQ else 0, row_stride=1024)
        assert L.qp_native_bytes(C.byref(dd)) == want


def test_encode_argument_errors_do_not_launch():
    L = qp.load_library()
    d = desc(codes=0, scales=0, lut=0x2000)       # codes and scales are not read by the encoder
    call = lambda dd, W, ldw, out, ws, n: L.qp_encode(C.byref(dd), W, ldw, out, None, ws, n, None)
    assert L.qp_encode_workspace_bytes(C.byref(d)) == 0          # scalar quantizer: no workspace
    assert call(d, None, 1024, 0x9000, None, 0) == 1
    assert call(d, 0x4000, 1024, None, None, 0) == 1
    assert call(d, 0x4000, 1000, 0x9000, None, 0) == 2
    assert call(d, 0x4008, 1024, 0x9000, None, 0) == 4
    assert call(desc(lut=0), 0x4000, 1024, 0x9000, None, 0) == 1
    assert call(desc(layout=qp.QP_LAYOUT_NATIVE), 0x4000, 1024, 0x9000, None, 0) == 5
    t = desc(scheme=qp.QP_TCQH, vec=2, code_bits=4, window_bits=16, tile=256, tlut_bits=9, row_stride=256)
    per_wg = 128 * 4096                                          # 128 steps x 2^12 groups, one byte each
    assert L.qp_encode_workspace_bytes(C.byref(t)) == per_wg * 64   # 16 rows x 4 tiles
    assert call(t, 0x4000, 1024, 0x9000, None, 0) == 7
    assert call(t, 0x4000, 1024, 0x9000, 0x100000, per_wg - 1) == 7
    assert call(t, 0x4000, 1024, 0x9000, 0x100004, per_wg) == 4
    t10 = desc(scheme=qp.QP_TCQH, vec=2, code_bits=10, window_bits=16, tile=256, tlut_bits=11, row_stride=640)
    assert L.qp_encode_workspace_bytes(C.byref(t10)) == 128 * 64 * 2 * 64   # two bytes per decision from s = 9 on
    t11 = desc(scheme=qp.QP_TCQH, vec=2, code_bits=11, window_bits=16, tile=256, tlut_bits=11, row_stride=704)
    assert call(t11, 0x4000, 1024, 0x9000, 0x100000, 1 << 30) == 3
    assert L.qp_encode_workspace_bytes(C.byref(t11)) == 0
    assert L.qp_encode_workspace_bytes(None) == 0


def test_row_normalize_argument_errors_do_not_launch():
    L = qp.load_library()
    assert L.qp_row_normalize(None, 1024, 4, 1024, 0x5000, None) == 1
    assert L.qp_row_normalize(0x4000, 1024, 4, 1024, None, None) == 1
    assert L.qp_row_normalize(0x4000, 1024, 0, 1024, 0x5000, None) == 2
    assert L.qp_row_normalize(0x4000, 1024, 4, 1020, 0x5000, None) == 2
    assert L.qp_row_normalize(0x4000, 512, 4, 1024, 0x5000, None) == 2
    assert L.qp_row_normalize(0x4004, 1024, 4, 1024, 0x5000, None) == 4


def test_kmeans_rejects_bad_arguments_on_the_host():
    L = qp.load_library()
    ws = qp.qp_kmeans_workspace_bytes(16, 2)
    assert ws > 0 and qp.qp_kmeans_workspace_bytes(0, 2) == 0 and qp.qp_kmeans_workspace_bytes(16, 3) == 0
    assert qp.qp_kmeans_workspace_bytes(4097, 1) == 0
    call = lambda **kw: L.qp_kmeans(*[kw.get(k, v) for k, v in dict(
        samples=0x1000, n=100, d=2, centres=0x2000, k=16, max_iter=10, tol=1e-6, workspace=0x3000, workspace_bytes=ws,
        assign=None, c16=None, stats=None, stream=None).items()])
    assert call(samples=None) == 1 and call(centres=None) == 1 and call(workspace=None) == 1
    assert call(d=3) == 3 and call(k=0) == 3 and call(k=5000) == 3
    assert call(n=0) == 2 and call(max_iter=0) == 2 and call(tol=-1.0) == 2
    assert call(samples=0x1004) == 4 and call(workspace=0x3008) == 4 and call(stats=0x4004) == 4
    assert call(workspace_bytes=ws - 1) == 7


def test_options_are_plain_integers_with_ranges():
    """qp_set_option / qp_get_option / qp_reset_options: host state only, no device needed."""
    L = qp.load_library()
    defaults = [L.qp_get_option(o) for o in range(8)]
    assert defaults == [0, 0, 0, -1, -1, 1, 0, -1]
    try:
        assert L.qp_set_option(qp.QP_OPT_LINEAR_KERNEL, 2) == 0 and L.qp_get_option(qp.QP_OPT_LINEAR_KERNEL) == 2
        assert L.qp_set_option(qp.QP_OPT_LINEAR_KERNEL, 3) == 2          # out of range: QP_ERR_SHAPE, value kept
        assert L.qp_get_option(qp.QP_OPT_LINEAR_KERNEL) == 2
        assert L.qp_set_option(qp.QP_OPT_NW, 2) == 2 and L.qp_set_option(qp.QP_OPT_NW, 8) == 0
        assert L.qp_set_option(99, 0) == 3 and L.qp_set_option(-1, 0) == 3  # QP_ERR_UNSUPPORTED
        assert L.qp_get_option(99) == -2 ** 31
        # the forced kernel shows in what qp_linear_workspace_bytes answers (block kernel + always pack)
        w = desc(M=16, N=1024)
        assert L.qp_linear_workspace_bytes(C.byref(w), 16) == 0
        L.qp_set_option(qp.QP_OPT_LINEAR_PACK, 1)
        assert L.qp_linear_workspace_bytes(C.byref(w), 16) == 16 * 1024 * 2
    finally:
        L.qp_reset_options()
    assert [L.qp_get_option(o) for o in range(8)] == defaults


def test_bench_aids_reject_bad_arguments_on_the_host():
    L = qp.load_library()
    assert L.qp_bench_stream_read(None, 1024, 0x1000, None) == 1
    assert L.qp_bench_stream_read(0x1000, 1024, None, None) == 1
    assert L.qp_bench_stream_read(0x1000, 0, 0x2000, None) == 2
    assert L.qp_bench_stream_read(0x1000, 1000, 0x2000, None) == 2      # not a multiple of 16
    assert L.qp_bench_stream_read(0x1008, 1024, 0x2000, None) == 4
    assert L.qp_bench_stream_read(0x1000, 1024, 0x2002, None) == 4


def test_block_argument_errors_do_not_launch():
    """qp_block_*: every refusal comes before any device call (this test runs without a GPU)."""
    L = qp.load_library()
    from paper_2509_20214_amd.binding import qp_block_item
    items = (qp_block_item * 2)()
    h = C.c_void_p()
    assert L.qp_block_enqueue(None, 1, C.c_void_p(256), 1024, None) == 1
    assert L.qp_block_enqueue(items, 0, C.c_void_p(256), 1024, None) == 2
    assert L.qp_block_enqueue(items, 5000, C.c_void_p(256), 1024, None) == 2
    assert L.qp_block_enqueue(items, 2, C.c_void_p(256), 1024, None) == 1        # items[0].w is NULL
    assert L.qp_block_create(items, 2, C.c_void_p(256), 1024, None) == 1
    assert L.qp_block_create(items, 2, C.c_void_p(256), 1024, C.byref(h)) == 1 and not h.value
    assert L.qp_block_workspace_bytes(items, 2) == 0
    assert L.qp_block_run(None, None) == 1
    assert L.qp_block_destroy(None) == 1
