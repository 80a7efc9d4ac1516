"""The entry point that allocates nothing (qp_rotate_linear_static): called through the C ABI with raw
pointers, its output must equal qp_rotate_linear's bit for bit (same kernels, the rotated
activations in the library's fixed array instead of a caller's workspace) and the oracle's fp64
chain within tolerance - on two calls in a row, the second with a smaller input, so that what the
first call left in the array is there when the second runs."""
import ctypes as C

import numpy as np
import pytest

import oracle
import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
TOL = 1e-2


def dev(a):
    if a.dtype == np.float16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.float16)
    return torch.from_numpy(a).cuda()


def run_static(qp, L, w, x, sg, block, B):
    y = torch.full((B, w.M), 9.0, dtype=torch.float16, device="cuda")
    code = L.qp_rotate_linear_static(C.byref(w.desc), C.c_void_p(x.data_ptr()), C.c_void_p(sg.data_ptr()), block, B,
                                     x.stride(0), C.c_void_p(y.data_ptr()), y.stride(0),
                                     C.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert code == 0, qp.qp_status_string(code)
    return y


@pytest.mark.parametrize("scheme,cb", [(synth.VQ, 5), (synth.SQ, 4), (synth.TCQ, 3), (synth.TCQH, 6), (synth.TCQHH, 4)],
                         ids=["vq5", "sq4", "tcq3", "tcqh3", "tcqhh2.25"])
def test_static_entry_matches_workspace_entry_twice(qp, scheme, cb):
    L = qp.load_library()
    assert L.qp_rotate_linear_static_max_bytes() == 16 * 32768 * 2
    qp.qp_set_option(qp.QP_OPT_LINEAR_KERNEL, qp.QP_KERNEL_BLOCK)
    # first call: 4 column blocks at batch 13 (padded to 16 rows in the array); second call: a
    # smaller layer at batch 3 - it finds the first call's activations in the array around its own
    for (M, N, B, block) in [(272, 4096, 13, 1024), (48, 2048, 3, 1024)]:
        lay = synth.make_layer(90, scheme * 10 + cb, scheme, M, N, cb)
        x = synth.make_x(90, B, B, N)
        sg = synth.make_signs(90, B, N)
        want = oracle.linear(lay, oracle.hadamard(x, sg, block), threads=True)
        w = qp.qp_repack(qp.Weight.from_layer(lay))
        xd, sd = dev(x), dev(sg)
        y_ws = qp.qp_rotate_linear(w, xd, sd, block)
        y_st = run_static(qp, L, w, xd, sd, block, B)
        torch.cuda.synchronize()
        assert torch.equal(y_st, y_ws)
        got = y_st.cpu().numpy().astype(np.float64)
        assert np.max(np.abs(got - want)) / np.max(np.abs(want)) <= TOL


def test_static_entry_single_launch_and_row_kernel_paths(qp):
    """Batch 1 with one rotation block (the layer's kernel rotates; the array is not touched) and a
    ragged layer on the row kernel (row-major activations in the array)."""
    L = qp.load_library()
    for (scheme, cb, M, N, B, block, native) in [(synth.VQ, 7, 64, 2048, 1, 2048, True), (synth.VQ, 5, 40, 1280, 5, 256, False)]:
        lay = synth.make_layer(91, cb, scheme, M, N, cb)
        x = synth.make_x(91, B, B, N)
        sg = synth.make_signs(91, B, N)
        want = oracle.linear(lay, oracle.hadamard(x, sg, block), threads=True)
        w = qp.Weight.from_layer(lay)
        if native:
            w = qp.qp_repack(w)
            qp.qp_set_option(qp.QP_OPT_LINEAR_KERNEL, qp.QP_KERNEL_BLOCK)
        else:
            qp.qp_reset_options()
        xd, sd = dev(x), dev(sg)
        y_ws = qp.qp_rotate_linear(w, xd, sd, block)
        y_st = run_static(qp, L, w, xd, sd, block, B)
        torch.cuda.synchronize()
        assert torch.equal(y_st, y_ws)
        got = y_st.cpu().numpy().astype(np.float64)
        assert np.max(np.abs(got - want)) / np.max(np.abs(want)) <= TOL


def test_static_entry_rejects_what_does_not_fit(qp):
    """No launch for bad arguments: a batch beyond the maximum, a null pointer."""
    L = qp.load_library()
    lay = synth.make_layer(92, 0, synth.VQ, 16, 1024, 5)
    w = qp.Weight.from_layer(lay)
    x = dev(synth.make_x(92, 0, 1, 1024))
    sg = dev(synth.make_signs(92, 0, 1024))
    y = torch.zeros((1, 16), dtype=torch.float16, device="cuda")
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    call = lambda xp, B: L.qp_rotate_linear_static(C.byref(w.desc), C.c_void_p(xp), C.c_void_p(sg.data_ptr()), 1024, B,
                                                   1024, C.c_void_p(y.data_ptr()), 16, st)
    assert call(x.data_ptr(), 17) == 2      # QP_ERR_SHAPE
    assert call(None, 1) == 1               # QP_ERR_NULL
    assert call(x.data_ptr(), 1) == 0
    # a layer whose rotated activations do not fit the array: N = 40960 at batch 16 needs 1.25 MiB
    wide = synth.make_layer(92, 1, synth.VQ, 8, 40960, 5)
    ww = qp.Weight.from_layer(wide)
    xw = dev(synth.make_x(92, 1, 16, 40960))
    sw = dev(synth.make_signs(92, 1, 40960))
    yw = torch.zeros((16, 8), dtype=torch.float16, device="cuda")
    callw = lambda B: L.qp_rotate_linear_static(C.byref(ww.desc), C.c_void_p(xw.data_ptr()), C.c_void_p(sw.data_ptr()),
                                                1024, B, 40960, C.c_void_p(yw.data_ptr()), 8, st)
    assert callw(16) == 7                   # QP_ERR_WORKSPACE
    assert callw(8) == 0                    # 640 KiB: fits
    torch.cuda.synchronize()
    want = oracle.linear(wide, oracle.hadamard(synth.make_x(92, 1, 16, 40960)[:8], synth.make_signs(92, 1, 40960), 1024))
    got = yw[:8].cpu().numpy().astype(np.float64)
    assert np.max(np.abs(got - want)) / np.max(np.abs(want)) <= TOL
