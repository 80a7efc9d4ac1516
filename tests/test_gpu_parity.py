"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by
element on the same seeded inputs.  Decode must be bit-exact; outputs must be within
1e-2 of the fp64 reference, relative to its infinity norm (fp16 inputs, fp32
accumulation, one fp16 rounding at the end)."""
import numpy as np
import pytest

import oracle
import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

SCHEMES = [(synth.SQ, 4), (synth.VQ, 5), (synth.VQ, 7), (synth.TCQ, 2), (synth.TCQ, 3), (synth.TCQ, 4),
           (synth.TCQH, 3), (synth.TCQH, 4), (synth.TCQH, 5), (synth.TCQH, 6), (synth.TCQH, 7), (synth.TCQH, 8),
           (synth.TCQH, 9), (synth.TCQH, 10)]
IDS = ["sq4", "vq5", "vq7", "tcq2", "tcq3", "tcq4", "tcqh1.5", "tcqh2", "tcqh2.5", "tcqh3", "tcqh3.5", "tcqh4",
       "tcqh4.5", "tcqh5"]
TOL = 1e-2          # the stated bound on max |y - y_ref| / max |y_ref|
# One rounding of the result to fp16 (at most 2^-11 of |y|, so of max |y_ref|); fp32 accumulation of exact
# fp16 x fp16 products adds errors orders of magnitude below that at these sizes.  Twice 2^-11:
TOL_SHARP = 1e-3


def dev(a):
    if a.dtype == np.float16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.float16)
    return torch.from_numpy(a).cuda()


def host16(t):
    return t.detach().cpu().view(torch.int16).numpy().view(np.uint16)


def rel_err(y_gpu_u16, y_ref):
    y = y_gpu_u16.view(np.float16).astype(np.float64)
    return float(np.max(np.abs(y - y_ref)) / np.max(np.abs(y_ref)))


# ----------------------------------------------------------------- decode
@pytest.mark.parametrize("scheme,cb", SCHEMES, ids=IDS)
@pytest.mark.parametrize("layout,M,N", [("canonical", 40, 1280), ("canonical", 33, 256), ("native", 48, 3072),
                                        ("native-generic", 48, 3072), ("native", 4128, 2048)])
def test_dequant_bit_exact(qp, scheme, cb, layout, M, N):
    """canonical -> the layout-agnostic kernel; native -> one block per wavefront with the fused
    kernel's decoders (M = 4128: 516 blocks, more than one per wavefront of the grid and a ragged
    last round); native-generic -> the layout-agnostic kernel reading the native layout."""
    lay = synth.make_layer(70, scheme * 10 + cb, scheme, M, N, cb)
    want = oracle.decode(lay)
    w = qp.Weight.from_layer(lay)
    if layout.startswith("native"):
        w = qp.qp_repack(w)
    qp.qp_set_option(qp.QP_OPT_DEQUANT_KERNEL, qp.QP_DEQUANT_GENERIC if layout == "native-generic" else qp.QP_DEQUANT_BLOCKS)
    got = host16(qp.qp_dequant(w))
    assert np.array_equal(got, want)


@pytest.mark.parametrize("cb,N", [(5, 40), (5, 104), (7, 56), (7, 120), (5, 1288), (7, 2104)])
def test_vq_rows_that_end_inside_a_byte(qp, cb, N):
    """5- and 7-bit codes: N / 2 codes need not fill whole bytes (N = 40: 100 bits).  The last code
    pair of a row then sits in a dword whose upper bytes lie beyond the row's last whole byte."""
    M = 37
    lay = synth.make_layer(69, cb * 1000 + N, synth.VQ, M, N, cb)
    # canonical stride: a multiple of 16 that holds the row's bytes, the padding filled with other
    # values so that a read beyond the row would show
    rb = lay.codes.shape[1]
    stride = (rb + 15) // 16 * 16
    padded = np.full((M, stride), 0xA5, dtype=np.uint8)
    padded[:, :rb] = lay.codes
    w = qp.Weight(lay.scheme, M, N, cb, 2, 0, 0, dev(padded), dev(lay.lut), dev(lay.scales), row_stride=stride)
    assert qp.qp_validate(w) == 0
    assert np.array_equal(host16(qp.qp_dequant(w)), oracle.decode(lay))
    for B in (1, 3, 16):
        x = synth.make_x(69, B, B, N)
        assert rel_err(host16(qp.qp_linear(w, dev(x))), oracle.linear(lay, x)) <= TOL
        # one-hot on the last column: the product is the row's last weight, exact to one rounding
    e = np.zeros((1, N), dtype=np.float16)
    e[0, N - 1] = 1.0
    want = oracle.linear(lay, e)
    y = host16(qp.qp_linear(w, dev(e))).view(np.float16).astype(np.float64)
    assert np.all(np.abs(y - want) <= np.abs(want) * 2.0 ** -11 + 1e-7)


def test_repack_layout_is_as_documented(qp):
    """Piece p of lane l = 16 g + i of block (R, C) holds canonical bytes
    [(4C+g)*span + 16p, +16) of row 16R+i."""
    lay = synth.make_layer(71, 0, synth.VQ, 32, 2048, 5)
    w = qp.Weight.from_layer(lay)
    nat = qp.qp_repack(w).codes.cpu().numpy()
    span, P, nbc = 80, 5, 2
    want = np.empty_like(nat)
    for R in range(2):
        for C_ in range(nbc):
            base = (R * nbc + C_) * 64 * span
            for p in range(P):
                for l in range(64):
                    g, i = l >> 4, l & 15
                    src = lay.codes[16 * R + i, (4 * C_ + g) * span + 16 * p:(4 * C_ + g) * span + 16 * p + 16]
                    want[base + (p * 64 + l) * 16: base + (p * 64 + l) * 16 + 16] = src
    assert np.array_equal(nat, want)


# ----------------------------------------------------------------- linear
@pytest.mark.parametrize("scheme,cb", SCHEMES, ids=IDS)
@pytest.mark.parametrize("layout,M,N", [("canonical", 40, 1280), ("native", 48, 3072), ("native-rowwave", 48, 3072),
                                        ("native", 1040, 2048), ("native", 16, 14336)])
@pytest.mark.parametrize("B", [1, 2, 3, 4, 5, 8, 13, 16])
def test_linear_matches_oracle(qp, scheme, cb, layout, M, N, B):
    """canonical -> one wavefront per row; native -> the matrix-core kernel (several row
    blocks per workgroup at M=1040, 14 column blocks at N=14336); native-rowwave -> the
    row kernel reading the native layout."""
    lay = synth.make_layer(72, scheme * 10 + cb, scheme, M, N, cb)
    x = synth.make_x(72, B, B, N)
    want = oracle.linear(lay, x, threads=True)
    w = qp.Weight.from_layer(lay)
    if layout.startswith("native"):
        w = qp.qp_repack(w)
    # small test layers would be routed to the row kernel by size: force the one under test
    qp.qp_set_option(qp.QP_OPT_LINEAR_KERNEL, qp.QP_KERNEL_ROW if layout == "native-rowwave" else qp.QP_KERNEL_BLOCK)
    y = qp.qp_linear(w, dev(x))
    torch.cuda.synchronize()
    err = rel_err(host16(y), want)
    assert err <= TOL
    assert err <= TOL_SHARP, err


def test_linear_with_leading_dimensions(qp):
    lay = synth.make_layer(73, 0, synth.VQ, 32, 1024, 5)
    B, ldx, ldy = 3, 1024 + 64, 32 + 5
    x = synth.make_x(73, 0, B, 1024)
    xd = torch.zeros((B, ldx), dtype=torch.float16, device="cuda")
    xd[:, :1024] = dev(x)
    yd = torch.full((B, ldy), 7.0, dtype=torch.float16, device="cuda")
    w = qp.Weight.from_layer(lay)
    qp.qp_linear(w, xd[:, :1024], y=yd[:, :32])
    torch.cuda.synchronize()
    want = oracle.linear(lay, x)
    got = yd.cpu().numpy()
    assert np.all(got[:, 32:] == 7.0)          # nothing written outside [B, M]
    assert rel_err(np.ascontiguousarray(got[:, :32]).view(np.uint16), want) <= TOL


ALL_SCHEMES = SCHEMES + [(synth.TCQHH, s_) for s_ in range(3, 10)]
ALL_IDS = IDS + [f"tcqhh{s_ / 2 + 0.25}" for s_ in range(3, 10)]


@pytest.mark.parametrize("scheme,cb", ALL_SCHEMES, ids=ALL_IDS)
@pytest.mark.parametrize("layout", ["native", "canonical"])
def test_block_kernel_one_hot_sweep_is_exact(qp, scheme, cb, layout):
    """Every weight of a layer, one by one, through the block kernel: 16 one-hot activation rows per
    call (row b = e_{c0 + b}) sweep all columns of both column blocks - for half-TCQ one block of
    either half - and both row blocks.  With x = e_i the fp32 sum is the single product 1 * W^[j, i]
    plus zeros, s[j] W^[j, i] is exact in fp32 (two 11-bit significands), so y[b, j] must EQUAL
    fp16(s[j] * W^[j, c0 + b]): any dropped or misplaced step, column mask, fold lane or partial sum
    shows as a wrong value, not as a tolerance."""
    M, N = 32, 2048
    lay = synth.make_layer(68, scheme * 10 + cb, scheme, M, N, cb)
    W = oracle.decode(lay).view(np.float16).astype(np.float32)                       # [M, N], exact
    want = (lay.scales.astype(np.float32)[:, None] * W).astype(np.float16)          # one rounding
    w = qp.Weight.from_layer(lay)
    if layout == "native":
        w = qp.qp_repack(w)
    qp.qp_set_option(qp.QP_OPT_LINEAR_KERNEL, qp.QP_KERNEL_BLOCK)
    eye = torch.zeros((N, N), dtype=torch.float16, device="cuda")
    eye.fill_diagonal_(1.0)
    got = torch.empty((N, M), dtype=torch.float16, device="cuda")
    for c0 in range(0, N, 16):
        qp.qp_linear(w, eye[c0:c0 + 16], y=got[c0:c0 + 16])
    torch.cuda.synchronize()
    got = got.cpu().numpy().T                                                       # [M, N]
    assert np.array_equal(got.astype(np.float32), want.astype(np.float32))          # (-0 == +0)
    # other batch sizes take other instances of the kernel: one call each at a ragged column offset
    for B in (1, 2, 3, 4, 7, 8, 11):
        c0 = 1024 - B // 2 - 1 if B > 1 else 1999                                   # straddles the two column blocks
        y = qp.qp_linear(w, eye[c0:c0 + B]).cpu().numpy()
        assert np.array_equal(y.astype(np.float32), want.T[c0:c0 + B].astype(np.float32)), B
    if (scheme, cb) == (synth.VQ, 5):
        # the forms of this kernel that large layers (batch 1 - 2: sixteen-copy table of code pairs) and some
        # small ones (batch 3 - 4: per-wavefront table) take by shape, forced here: every column, then
        # ragged offsets at the other batch sizes
        qp.qp_set_option(qp.QP_OPT_LINEAR_SPLIT, 1)
        alt = torch.empty((N, M), dtype=torch.float16, device="cuda")
        for c0 in range(0, N, 2):
            qp.qp_linear(w, eye[c0:c0 + 2], y=alt[c0:c0 + 2])
        torch.cuda.synchronize()
        assert np.array_equal(alt.cpu().numpy().T.astype(np.float32), want.astype(np.float32))
        for B, c0 in ((1, 0), (1, 1023), (1, 2047), (2, 1023), (3, 1022), (4, 1021)):
            y = qp.qp_linear(w, eye[c0:c0 + B]).cpu().numpy()
            assert np.array_equal(y.astype(np.float32), want.T[c0:c0 + B].astype(np.float32)), (B, c0)


def test_linear_one_hot_picks_single_weights(qp):
    """x = e_i makes y[j] = s[j] W^[j, i]: exact up to one fp16 rounding."""
    for scheme, cb in SCHEMES:
        lay = synth.make_layer(74, scheme * 10 + cb, scheme, 16, 1024, cb)
        e = np.zeros((1, 1024), dtype=np.float16)
        e[0, 777] = 1.0
        want = oracle.linear(lay, e)
        y = host16(qp.qp_linear(qp.Weight.from_layer(lay), dev(e))).view(np.float16).astype(np.float64)
        assert np.all(np.abs(y - want) <= np.abs(want) * 2.0 ** -11 + 1e-7)


# --------------------------------------------------------------- Hadamard
@pytest.mark.parametrize("B,n,block", [(1, 1024, 1024), (3, 4096, 4096), (2, 8192, 8192), (1, 14336, 1024),
                                       (4, 14336, 1024), (16, 28672, 1024), (5, 64, 8), (1, 2, 2),
                                       (2, 16384, 16384), (7, 1536, 512)])
def test_hadamard_matches_oracle(qp, B, n, block):
    x = synth.make_x(75, n % 97, B, n)
    sg = synth.make_signs(75, n % 97, n)
    want = oracle.hadamard(x, sg, block, fast=(block > 2048))
    got = host16(qp.qp_hadamard(dev(x), dev(sg), block)).view(np.float16).astype(np.float64)
    # fp32 butterflies then one fp16 rounding: half an fp16 ulp plus the fp32 error
    # of log2(block) additions of O(sqrt(block))-sized numbers
    tol = np.abs(want) * 2.0 ** -11 + np.max(np.abs(want)) * 2.0 ** -20 + 2.0 ** -24
    assert np.all(np.abs(got - want) <= tol)


def test_hadamard_in_place_and_strided(qp):
    B, n, block, ld = 3, 2048, 1024, 2048 + 8
    x = synth.make_x(76, 0, B, n)
    sg = synth.make_signs(76, 0, n)
    buf = torch.zeros((B, ld), dtype=torch.float16, device="cuda")
    buf[:, :n] = dev(x)
    view = buf[:, :n]
    qp.qp_hadamard(view, dev(sg), block, out=view)
    torch.cuda.synchronize()
    want = oracle.hadamard(x, sg, block)
    got = view.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - want) <= np.abs(want) * 2.0 ** -11 + 1e-5)
    assert torch.all(buf[:, n:] == 0)


# ---------------------------------------------------------------- chained
@pytest.mark.parametrize("scheme,cb", SCHEMES, ids=IDS)
def test_rotation_then_linear_matches_fp64_chain(qp, scheme, cb):
    """Whole hot path: rotate x on the GPU, multiply on the GPU; the oracle stays in
    fp64 from the fp16 x to the end."""
    M, N, B = 64, 2048, 2
    block = 1024
    lay = synth.make_layer(77, scheme * 10 + cb, scheme, M, N, cb)
    x = synth.make_x(77, 1, B, N)
    sg = synth.make_signs(77, 1, N)
    want = oracle.linear(lay, oracle.hadamard(x, sg, block))
    w = qp.qp_repack(qp.Weight.from_layer(lay))
    xr = qp.qp_hadamard(dev(x), dev(sg), block)
    for kernel in (qp.QP_KERNEL_BLOCK, qp.QP_KERNEL_ROW):
        qp.qp_set_option(qp.QP_OPT_LINEAR_KERNEL, kernel)
        y = qp.qp_linear(w, xr)
        assert rel_err(host16(y), want) <= TOL


# ---------------------------------------------------- rotation fused into the launch
@pytest.mark.parametrize("scheme,cb", SCHEMES, ids=IDS)
@pytest.mark.parametrize("B", [1, 2, 3, 4, 8, 13, 16])
def test_rotate_linear_matches_oracle_and_unfused(qp, scheme, cb, B):
    """One call = rotation + layer; the rotated activations pass through the workspace in the
    block kernel's own fragment order.  Must equal the two-call sequence (row-major
    activations) bit for bit - same arithmetic, fp16 rotated activations in between - and
    the fp64 chain within tolerance; repeated calls reuse the workspace."""
    M, N, block = 272, 3072, 1024      # 17 row blocks, 3 column blocks: several units per wavefront
    lay = synth.make_layer(78, scheme * 10 + cb, scheme, M, N, cb)
    x = synth.make_x(78, B, B, N)
    sg = synth.make_signs(78, 1, N)
    want = oracle.linear(lay, oracle.hadamard(x, sg, block), threads=True)
    w = qp.qp_repack(qp.Weight.from_layer(lay))
    qp.qp_set_option(qp.QP_OPT_LINEAR_KERNEL, qp.QP_KERNEL_BLOCK)
    xd, sd = dev(x), dev(sg)
    y2 = qp.qp_linear(w, qp.qp_hadamard(xd, sd, block))
    ws = torch.empty(qp.qp_rotate_linear_workspace_bytes(w, B), dtype=torch.uint8, device="cuda")
    for rep in range(2):
        y1 = qp.qp_rotate_linear(w, xd, sd, block, workspace=ws)
        torch.cuda.synchronize()
        assert rel_err(host16(y1), want) <= TOL
        assert torch.equal(y1, y2)


def test_rotate_linear_strided_x(qp):
    lay = synth.make_layer(79, 2, synth.VQ, 256, 2048, 5)
    B, ldx = 2, 2048 + 64
    x = synth.make_x(79, 2, B, 2048)
    sg = synth.make_signs(79, 2, 2048)
    want = oracle.linear(lay, oracle.hadamard(x, sg, 1024))
    buf = torch.zeros((B, ldx), dtype=torch.float16, device="cuda")
    buf[:, :2048] = dev(x)
    qp.qp_set_option(qp.QP_OPT_LINEAR_KERNEL, qp.QP_KERNEL_BLOCK)
    y = qp.qp_rotate_linear(qp.qp_repack(qp.Weight.from_layer(lay)), buf[:, :2048], dev(sg), 1024)
    assert rel_err(host16(y), want) <= TOL


def test_rotate_linear_other_shapes_fall_back_to_two_launches(qp):
    lay = synth.make_layer(79, 0, synth.VQ, 64, 4096, 5)
    x = synth.make_x(79, 0, 2, 4096)
    sg = synth.make_signs(79, 0, 4096)
    want = oracle.linear(lay, oracle.hadamard(x, sg, 4096, fast=True))
    for layout in ("canonical", "native"):
        w = qp.Weight.from_layer(lay)
        if layout == "native":
            w = qp.qp_repack(w)
        y = qp.qp_rotate_linear(w, dev(x), dev(sg), 4096)
        assert rel_err(host16(y), want) <= TOL


# ----------------------------------------------------------------- half-TCQ
HH = [(synth.TCQHH, s) for s in range(3, 10)]
HH_IDS = [f"tcqhh{s / 2 + 0.25}" for s in range(3, 10)]


@pytest.mark.parametrize("scheme,cb", HH, ids=HH_IDS)
@pytest.mark.parametrize("layout,M,N", [("canonical", 40, 1536), ("canonical", 33, 512), ("native", 48, 4096),
                                        ("native-generic", 48, 4096), ("native", 4128, 2048)])
def test_half_tcq_dequant_bit_exact(qp, scheme, cb, layout, M, N):
    lay = synth.make_layer(80, cb, scheme, M, N, cb)
    want = oracle.decode(lay)
    w = qp.Weight.from_layer(lay)
    if layout.startswith("native"):
        w = qp.qp_repack(w)
    qp.qp_set_option(qp.QP_OPT_DEQUANT_KERNEL, qp.QP_DEQUANT_GENERIC if layout == "native-generic" else qp.QP_DEQUANT_BLOCKS)
    assert np.array_equal(host16(qp.qp_dequant(w)), want)


def test_half_tcq_repack_layout_is_as_documented(qp):
    """Per block row: the column blocks of the first half (cb pieces per lane), then those of
    the second (cb + 1 pieces); inside a block as for every other scheme."""
    cb, M, N = 4, 32, 4096
    lay = synth.make_layer(81, 0, synth.TCQHH, M, N, cb)
    nat = qp.qp_repack(qp.Weight.from_layer(lay)).codes.cpu().numpy()
    h = N // 2048
    lo_row = N // 512 * 16 * cb
    want = np.empty_like(nat)
    pos = 0
    for R in range(M // 16):
        for half in range(2):
            P = cb + half
            span = 16 * P
            for C_ in range(h):
                for p in range(P):
                    for l in range(64):
                        g, i = l >> 4, l & 15
                        off = half * lo_row + (4 * C_ + g) * span + 16 * p
                        want[pos + (p * 64 + l) * 16: pos + (p * 64 + l) * 16 + 16] = lay.codes[16 * R + i, off:off + 16]
                pos += 64 * span
    assert pos == nat.size
    assert np.array_equal(nat, want)


@pytest.mark.parametrize("scheme,cb", HH, ids=HH_IDS)
@pytest.mark.parametrize("layout,M,N", [("canonical", 40, 1536), ("native", 48, 4096), ("native-rowwave", 48, 4096),
                                        ("native", 1040, 2048), ("native", 16, 14336)])
@pytest.mark.parametrize("B", [1, 2, 3, 8, 16])
def test_half_tcq_linear_matches_oracle(qp, scheme, cb, layout, M, N, B):
    lay = synth.make_layer(82, cb, scheme, M, N, cb)
    x = synth.make_x(82, B, B, N)
    want = oracle.linear(lay, x, threads=True)
    w = qp.Weight.from_layer(lay)
    if layout.startswith("native"):
        w = qp.qp_repack(w)
    qp.qp_set_option(qp.QP_OPT_LINEAR_KERNEL, qp.QP_KERNEL_ROW if layout == "native-rowwave" else qp.QP_KERNEL_BLOCK)
    y = qp.qp_linear(w, dev(x))
    torch.cuda.synchronize()
    assert rel_err(host16(y), want) <= TOL_SHARP    # (and so within the stated TOL)


@pytest.mark.parametrize("scheme,cb", HH, ids=HH_IDS)
@pytest.mark.parametrize("B", [1, 4, 13])
def test_half_tcq_rotate_linear(qp, scheme, cb, B):
    M, N, block = 272, 4096, 1024
    lay = synth.make_layer(83, cb, scheme, M, N, cb)
    x = synth.make_x(83, B, B, N)
    sg = synth.make_signs(83, 1, N)
    want = oracle.linear(lay, oracle.hadamard(x, sg, block), threads=True)
    w = qp.qp_repack(qp.Weight.from_layer(lay))
    qp.qp_set_option(qp.QP_OPT_LINEAR_KERNEL, qp.QP_KERNEL_BLOCK)
    xd, sd = dev(x), dev(sg)
    y2 = qp.qp_linear(w, qp.qp_hadamard(xd, sd, block))
    y1 = qp.qp_rotate_linear(w, xd, sd, block)
    torch.cuda.synchronize()
    assert rel_err(host16(y1), want) <= TOL
    assert torch.equal(y1, y2)


# ------------------------------------------- rotation inside the layer's kernel (batch 1, one block)
ALL = SCHEMES + HH
ALL_IDS = IDS + HH_IDS


@pytest.mark.parametrize("scheme,cb", ALL, ids=ALL_IDS)
@pytest.mark.parametrize("M,N", [(272, 2048), (48, 4096), (1040, 4096), (32, 8192)])
def test_rotate_linear_in_kernel_rotation(qp, scheme, cb, M, N):
    """Batch 1 and one Hadamard block: qp_rotate_linear is a single launch whose workgroups
    rotate the activations themselves.  Same bits as rotation kernel + layer kernel, and the
    fp64 chain within tolerance; the split path stays available (QP_OPT_ROTATE_SPLIT)."""
    lay = synth.make_layer(84, scheme * 10 + cb, scheme, M, N, cb)
    x = synth.make_x(84, N, 1, N)
    sg = synth.make_signs(84, N, N)
    want = oracle.linear(lay, oracle.hadamard(x, sg, N, fast=True), threads=True)
    w = qp.qp_repack(qp.Weight.from_layer(lay))
    qp.qp_set_option(qp.QP_OPT_LINEAR_KERNEL, qp.QP_KERNEL_BLOCK)
    xd, sd = dev(x), dev(sg)
    y_two = qp.qp_linear(w, qp.qp_hadamard(xd, sd, N))
    y_one = qp.qp_rotate_linear(w, xd, sd, N)
    qp.qp_set_option(qp.QP_OPT_ROTATE_SPLIT, 1)
    y_split = qp.qp_rotate_linear(w, xd, sd, N)
    torch.cuda.synchronize()
    assert rel_err(host16(y_one), want) <= TOL
    assert torch.equal(y_one, y_two)
    assert torch.equal(y_split, y_two)


def test_rotate_linear_in_kernel_rotation_block_1024(qp):
    lay = synth.make_layer(85, 0, synth.VQ, 4096, 1024, 5)
    x = synth.make_x(85, 0, 1, 1024)
    sg = synth.make_signs(85, 0, 1024)
    w = qp.qp_repack(qp.Weight.from_layer(lay))
    qp.qp_set_option(qp.QP_OPT_LINEAR_KERNEL, qp.QP_KERNEL_BLOCK)
    y = qp.qp_rotate_linear(w, dev(x), dev(sg), 1024)
    assert rel_err(host16(y), oracle.linear(lay, oracle.hadamard(x, sg, 1024), threads=True)) <= TOL
    assert torch.equal(y, qp.qp_linear(w, qp.qp_hadamard(dev(x), dev(sg), 1024)))


@pytest.mark.parametrize("scheme,cb,M,N", [(synth.VQ, 5, 4096, 14336), (synth.SQ, 4, 48, 16384), (synth.VQ, 7, 1040, 2048),
                                           (synth.TCQH, 4, 512, 14336), (synth.TCQH, 9, 64, 3072), (synth.TCQH, 10, 4096, 2048),
                                           (synth.TCQHH, 4, 256, 4096 + 2048), (synth.TCQ, 3, 64, 3072),
                                           (synth.VQ, 5, 4112, 3072), (synth.SQ, 4, 32, 17408)],
                         ids=["vq5-4096x14336", "sq4-48x16384", "vq7-1040x2048", "tcqh2-512x14336", "tcqh4.5-64x3072",
                              "tcqh5-4096x2048", "tcqhh2.25-256x6144", "tcq3-two-launches", "vq5-4112-rows-two-launches",
                              "sq4-17-blocks-two-launches"])
def test_rotate_linear_rotates_blocks_of_1024_in_kernel(qp, scheme, cb, M, N):
    """Batch 1, blocks of 1024, a layer of at most 4096 x 16384 (not the V = 1 trellis): one launch, every
    wavefront transforms the block of its own unit on the matrix cores.  Same bits as rotation kernel +
    layer kernel - which the larger layers and the V = 1 trellis still take - and the fp64 chain within
    tolerance."""
    lay = synth.make_layer(86, scheme * 10 + cb, scheme, M, N, cb)
    x = synth.make_x(86, N % 89, 1, N)
    sg = synth.make_signs(86, N % 89, N)
    want = oracle.linear(lay, oracle.hadamard(x, sg, 1024, fast=True), threads=True)
    w = qp.qp_repack(qp.Weight.from_layer(lay))
    qp.qp_set_option(qp.QP_OPT_LINEAR_KERNEL, qp.QP_KERNEL_BLOCK)
    one_launch = scheme != synth.TCQ and M <= 4096 and N <= 16384
    assert qp.qp_rotate_linear_launches(w, 1, 1024) == (1 if one_launch else 2)
    assert qp.qp_rotate_linear_launches(w, 2, 1024) == 2
    xd, sd = dev(x), dev(sg)
    y_two = qp.qp_linear(w, qp.qp_hadamard(xd, sd, 1024))
    y_one = qp.qp_rotate_linear(w, xd, sd, 1024)
    y_again = qp.qp_rotate_linear(w, xd, sd, 1024)
    qp.qp_set_option(qp.QP_OPT_ROTATE_SPLIT, 1)
    y_split = qp.qp_rotate_linear(w, xd, sd, 1024)
    torch.cuda.synchronize()
    assert rel_err(host16(y_one), want) <= TOL_SHARP
    assert torch.equal(y_one, y_two)
    assert torch.equal(y_again, y_two)
    assert torch.equal(y_split, y_two)
    if scheme == synth.TCQH:
        # two wavefronts per unit: a wavefront's half units lie in other column blocks than the one it transformed
        qp.qp_reset_options()
        qp.qp_set_option(qp.QP_OPT_LINEAR_KERNEL, qp.QP_KERNEL_BLOCK)
        qp.qp_set_option(qp.QP_OPT_LINEAR_SPLIT, 1)
        y_two = qp.qp_linear(w, qp.qp_hadamard(xd, sd, 1024))
        y_one = qp.qp_rotate_linear(w, xd, sd, 1024)
        torch.cuda.synchronize()
        assert rel_err(host16(y_one), want) <= TOL_SHARP
        assert torch.equal(y_one, y_two)


RAGGED_SCHEMES = [(synth.SQ, 4), (synth.VQ, 5), (synth.VQ, 7), (synth.TCQ, 2), (synth.TCQ, 3), (synth.TCQ, 4),
                  (synth.TCQH, 3), (synth.TCQH, 6), (synth.TCQH, 9), (synth.TCQH, 10)]
RAGGED_IDS = ["sq4", "vq5", "vq7", "tcq2", "tcq3", "tcq4", "tcqh1.5", "tcqh3", "tcqh4.5", "tcqh5"]


@pytest.mark.parametrize("scheme,cb", RAGGED_SCHEMES, ids=RAGGED_IDS)
@pytest.mark.parametrize("M,N", [(48, 768), (272, 1280), (32, 2816), (16, 256)])
def test_last_column_block_cut_short(qp, scheme, cb, M, N):
    """N a multiple of 256 but not of 1024 (the 11008 and 13824 input channels of the 7B- and 13B-shaped
    models): the native layout pads the last column block with zero bytes and the block kernel multiplies
    the padding with zeros.  Decode bit-exact through both dequantization kernels; the layer against the
    oracle from either layout, with row-major and fragment-order activations, at every batch size class;
    rotation + layer the same bits as the two calls; one-hot activations on the last real columns exact."""
    lay = synth.make_layer(90, scheme * 10 + cb + N, scheme, M, N, cb)
    wc = qp.Weight.from_layer(lay)
    wn = qp.qp_repack(wc)
    assert wn.codes.numel() == M * ((N + 1023) // 1024 * 1024 // 256) * (32 * cb // (1 if scheme in (synth.SQ, synth.TCQ) else 2))
    want_w = oracle.decode(lay)
    for kern in (qp.QP_DEQUANT_GENERIC, qp.QP_DEQUANT_BLOCKS):
        qp.qp_set_option(qp.QP_OPT_DEQUANT_KERNEL, kern)
        assert np.array_equal(host16(qp.qp_dequant(wn)), want_w)
    block = synth.hadamard_block(N)
    sg = synth.make_signs(90, N, N)
    for B in (1, 2, 3, 8, 13):
        x = synth.make_x(90, B, B, N)
        xd = dev(x)
        want = oracle.linear(lay, x, threads=True)
        for w in (wn, wc):
            for pack in (0, 1):
                qp.qp_reset_options()
                qp.qp_set_option(qp.QP_OPT_LINEAR_KERNEL, qp.QP_KERNEL_BLOCK)
                qp.qp_set_option(qp.QP_OPT_LINEAR_PACK, pack)
                assert rel_err(host16(qp.qp_linear(w, xd)), want) <= TOL_SHARP, (B, w.layout, pack)
        qp.qp_reset_options()
        qp.qp_set_option(qp.QP_OPT_LINEAR_KERNEL, qp.QP_KERNEL_ROW)
        assert rel_err(host16(qp.qp_linear(wn, xd)), want) <= TOL_SHARP   # the row kernel on the padded native layout
        qp.qp_set_option(qp.QP_OPT_LINEAR_KERNEL, qp.QP_KERNEL_BLOCK)
        y = qp.qp_rotate_linear(wn, xd, dev(sg), block)
        assert torch.equal(y, qp.qp_linear(wn, qp.qp_hadamard(xd, dev(sg), block), workspace=False))
        assert rel_err(host16(y), oracle.linear(lay, oracle.hadamard(x, sg, block, fast=True), threads=True)) <= TOL_SHARP
    qp.qp_reset_options()
    qp.qp_set_option(qp.QP_OPT_LINEAR_KERNEL, qp.QP_KERNEL_BLOCK)
    cols = sorted({N - 1, N - 8, N - 256, max(N - 257, 0), 0})
    e = np.zeros((len(cols), N), dtype=np.float16)
    for r, c in enumerate(cols):
        e[r, c] = 1.0
    want = oracle.linear(lay, e)
    y = host16(qp.qp_linear(wn, dev(e))).view(np.float16).astype(np.float64)
    assert np.all(np.abs(y - want) <= np.abs(want) * 2.0 ** -11 + 1e-7)


def test_last_column_block_cut_short_at_full_size(qp):
    """4096 x 11008 at 2.5 bits: taken by the block kernel by default (not the row kernel), batch 1 and 8."""
    lay = synth.make_layer(91, 0, synth.VQ, 4096, 11008, 5)
    wn = qp.qp_repack(qp.Weight.from_layer(lay))
    sg = synth.make_signs(91, 0, 11008)
    for B in (1, 8):
        x = synth.make_x(91, B, B, 11008)
        want = oracle.linear(lay, oracle.hadamard(x, sg, 256, fast=True), threads=True)
        y = qp.qp_rotate_linear(wn, dev(x), dev(sg), 256)
        assert rel_err(host16(y), want) <= TOL_SHARP
        qp.qp_set_option(qp.QP_OPT_LINEAR_KERNEL, qp.QP_KERNEL_BLOCK)
        assert torch.equal(y, qp.qp_rotate_linear(wn, dev(x), dev(sg), 256))   # the default was the block kernel
        qp.qp_reset_options()


@pytest.mark.parametrize("scheme,cb,M,N,block,one", [
    (synth.SQ, 4, 1024, 1024, 1024, True), (synth.VQ, 5, 37, 3072, 1024, True), (synth.VQ, 7, 1000, 2048, 2048, True),
    (synth.TCQ, 3, 48, 2048, 1024, True), (synth.TCQ, 2, 64, 2048, 2048, False), (synth.TCQH, 6, 5, 8192, 8192, True),
    (synth.TCQH, 10, 130, 7168, 1024, True), (synth.TCQHH, 4, 256, 4096, 4096, True), (synth.SQ, 4, 16, 9216, 1024, False),
    (synth.VQ, 5, 64, 2048, 512, False)],
    ids=["sq4-1024x1024", "vq5-37x3072", "vq7-1000x2048-one-block", "tcq3-48x2048", "tcq2-one-block-two-launches",
         "tcqh3-5x8192-one-block", "tcqh5-130x7168", "tcqhh2.25-256x4096-one-block", "sq4-9-blocks-two-launches",
         "vq5-blocks-of-512-two-launches"])
def test_rotate_linear_row_kernel_rotates_in_kernel(qp, scheme, cb, M, N, block, one):
    """Tiny and ragged layers (the row kernel) at batch 1, N <= 8192, blocks of 1024 or one block of up to 8192:
    one launch, the workgroup rotates the row into LDS itself.  Same bits as rotation kernel + layer kernel;
    the fp64 chain within tolerance.  Beside the V = 1 trellis' table only blocks of 1024."""
    lay = synth.make_layer(89, scheme * 10 + cb, scheme, M, N, cb)
    x = synth.make_x(89, N % 89, 1, N)
    sg = synth.make_signs(89, N % 89, N)
    want = oracle.linear(lay, oracle.hadamard(x, sg, block, fast=True), threads=True)
    w = qp.Weight.from_layer(lay)
    if M % 16 == 0 and scheme != synth.VQ: w = qp.qp_repack(w)
    qp.qp_set_option(qp.QP_OPT_LINEAR_KERNEL, qp.QP_KERNEL_ROW)
    assert qp.qp_rotate_linear_launches(w, 1, block) == (1 if one else 2)
    assert qp.qp_rotate_linear_launches(w, 2, block) == 2
    xd, sd = dev(x), dev(sg)
    y_two = qp.qp_linear(w, qp.qp_hadamard(xd, sd, block))
    y_one = qp.qp_rotate_linear(w, xd, sd, block)
    y_again = qp.qp_rotate_linear(w, xd, sd, block)
    qp.qp_set_option(qp.QP_OPT_ROTATE_SPLIT, 1)
    assert qp.qp_rotate_linear_launches(w, 1, block) == 2
    y_split = qp.qp_rotate_linear(w, xd, sd, block)
    torch.cuda.synchronize()
    assert rel_err(host16(y_one), want) <= TOL_SHARP
    assert torch.equal(y_one, y_two)
    assert torch.equal(y_again, y_two)
    assert torch.equal(y_split, y_two)


@pytest.mark.parametrize("scheme,cb,M,N,block", [(synth.VQ, 5, 256, 3072, 1024), (synth.TCQH, 6, 512, 5120, 1024),
                                                 (synth.SQ, 4, 4096, 2048, 2048), (synth.TCQHH, 4, 256, 4096, 4096)],
                         ids=["vq5-3-blocks", "tcqh3-5-blocks", "sq4-one-block-2048", "tcqhh2.25-one-block-4096"])
def test_rotate_linear_in_kernel_rotation_canonical_layout(qp, scheme, cb, M, N, block):
    """The one-launch forms on weights that were not repacked (the block kernel reads the canonical layout too)."""
    lay = synth.make_layer(88, scheme * 10 + cb, scheme, M, N, cb)
    x = synth.make_x(88, N % 89, 1, N)
    sg = synth.make_signs(88, N % 89, N)
    want = oracle.linear(lay, oracle.hadamard(x, sg, block, fast=True), threads=True)
    w = qp.Weight.from_layer(lay)
    qp.qp_set_option(qp.QP_OPT_LINEAR_KERNEL, qp.QP_KERNEL_BLOCK)
    assert qp.qp_rotate_linear_launches(w, 1, block) == 1
    xd, sd = dev(x), dev(sg)
    y_two = qp.qp_linear(w, qp.qp_hadamard(xd, sd, block))
    y_one = qp.qp_rotate_linear(w, xd, sd, block)
    torch.cuda.synchronize()
    assert rel_err(host16(y_one), want) <= TOL_SHARP
    assert torch.equal(y_one, y_two)


@pytest.mark.parametrize("block", [1024, 2048, 4096, 8192])
def test_hadamard_matrix_core_and_butterfly_kernels(qp, block):
    """Blocks of 1024 .. 8192 run on the matrix cores when the output is 8-byte aligned, as butterfly stages
    otherwise; both against the oracle, and against each other to neighbouring fp16 numbers."""
    B, n = 3, (5 * 1024 if block == 1024 else 2 * block)
    x = synth.make_x(87, 0, B, n)
    sg = synth.make_signs(87, 0, n)
    want = oracle.hadamard(x, sg, block, fast=True)
    tol = np.abs(want) * 2.0 ** -11 + np.max(np.abs(want)) * 2.0 ** -20 + 2.0 ** -24
    xd, sd = dev(x), dev(sg)
    a = qp.qp_hadamard(xd, sd, block)
    buf = torch.zeros(B * n + 8, dtype=torch.float16, device="cuda")
    out = buf[1:1 + B * n].view(B, n)          # 2 bytes off an 8-byte boundary
    qp.qp_hadamard(xd, sd, block, out=out)
    torch.cuda.synchronize()
    for got in (a, out):
        assert np.all(np.abs(host16(got).view(np.float16).astype(np.float64) - want) <= tol)
    assert float(buf[0]) == 0 and torch.all(buf[1 + B * n:] == 0)
    ga, gb = host16(a).view(np.float16).astype(np.float64), host16(out).view(np.float16).astype(np.float64)
    # (neighbouring fp16 numbers; across a power of two the larger of the two spacings applies)
    assert np.all(np.abs(ga - gb) <= 2.0 * np.spacing(np.abs(want).astype(np.float16)).astype(np.float64) + 2.0 ** -24)


@pytest.mark.parametrize("scheme,cb", [(synth.TCQ, 2), (synth.TCQ, 3), (synth.TCQ, 4)] +
                         [(synth.TCQH, s) for s in range(3, 11)],
                         ids=["tcq2", "tcq3", "tcq4"] + [f"tcqh{s / 2}" for s in range(3, 11)])
@pytest.mark.parametrize("M,N,B", [(48, 4096, 1), (1040, 2048, 2), (16, 14336, 1), (272, 3072, 2)])
@pytest.mark.parametrize("split", ["0", "1"])
def test_linear_two_wavefronts_per_unit(qp, scheme, cb, M, N, B, split):
    """The trellis kernels at batch <= 2 exist in two forms: one wavefront per 16 x 1024 unit, or
    two, each decoding half of its steps from only the pieces it needs.  Both forms, at unit
    counts on either side of the automatic choice."""
    lay = synth.make_layer(86, scheme * 10 + cb, scheme, M, N, cb)
    x = synth.make_x(86, B, B, N)
    want = oracle.linear(lay, x, threads=True)
    w = qp.qp_repack(qp.Weight.from_layer(lay))
    qp.qp_set_option(qp.QP_OPT_LINEAR_KERNEL, qp.QP_KERNEL_BLOCK)
    qp.qp_set_option(qp.QP_OPT_LINEAR_SPLIT, int(split))
    y = qp.qp_linear(w, dev(x))
    torch.cuda.synchronize()
    assert rel_err(host16(y), want) <= TOL_SHARP    # (and so within the stated TOL)


@pytest.mark.parametrize("M,N,B", [(48, 4096, 1), (1040, 2048, 2), (16, 14336, 1), (4112, 3072, 2), (272, 3072, 1)])
@pytest.mark.parametrize("split", [0, 1])
def test_vq5_tables_of_code_pairs(qp, M, N, B, split):
    """The 2.5-bit vector quantizer at batch <= 2 decodes two codes per lookup from a table of pairs held
    eight times (64 KiB) or sixteen times (128 KiB, taken by shape from 20 units per workgroup on, and at 7 - 8); both
    forms on layers of one and of several passes, same bits from both (the decoded weights are the same
    and so is the order of the sums)."""
    lay = synth.make_layer(85, M + B, synth.VQ, M, N, 5)
    x = synth.make_x(85, B, B, N)
    want = oracle.linear(lay, x, threads=True)
    w = qp.qp_repack(qp.Weight.from_layer(lay))
    qp.qp_set_option(qp.QP_OPT_LINEAR_KERNEL, qp.QP_KERNEL_BLOCK)
    qp.qp_set_option(qp.QP_OPT_LINEAR_SPLIT, split)
    y = qp.qp_linear(w, dev(x))
    qp.qp_set_option(qp.QP_OPT_LINEAR_SPLIT, 1 - split)
    y_other = qp.qp_linear(w, dev(x))
    torch.cuda.synchronize()
    assert rel_err(host16(y), want) <= TOL_SHARP
    assert torch.equal(y, y_other)


def test_calls_captured_in_a_hip_graph_replay_identically(qp):
    """The library only enqueues kernels (no allocation, no memset, no synchronisation), so a
    sequence of its calls can be captured once and replayed: three replays, with eager work in
    between, each equal to the eager results."""
    qp.qp_set_option(qp.QP_OPT_LINEAR_KERNEL, qp.QP_KERNEL_BLOCK)
    lay_a = synth.make_layer(87, 0, synth.TCQH, 272, 4096, 5)
    lay_b = synth.make_layer(87, 1, synth.VQ, 4096, 3072, 5)
    wa, wb = qp.qp_repack(qp.Weight.from_layer(lay_a)), qp.qp_repack(qp.Weight.from_layer(lay_b))
    sga, sgb = dev(synth.make_signs(87, 0, 4096)), dev(synth.make_signs(87, 1, 3072))
    xa, xb = dev(synth.make_x(87, 0, 1, 4096)), dev(synth.make_x(87, 1, 3, 3072))
    ya = torch.empty((1, 272), dtype=torch.float16, device="cuda")
    yb = torch.empty((3, 4096), dtype=torch.float16, device="cuda")
    ws = torch.empty(max(qp.qp_rotate_linear_workspace_bytes(wa, 1), qp.qp_rotate_linear_workspace_bytes(wb, 3)),
                     dtype=torch.uint8, device="cuda")
    W = torch.empty((272, 4096), dtype=torch.float16, device="cuda")

    def work():
        qp.qp_rotate_linear(wa, xa, sga, 4096, y=ya, workspace=ws)      # one launch (in-kernel rotation)
        qp.qp_rotate_linear(wb, xb, sgb, 1024, y=yb, workspace=ws)      # two launches through the workspace
        qp.qp_dequant(wa, out=W)

    work()
    torch.cuda.synchronize()
    want = (ya.clone(), yb.clone(), W.clone())
    g = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        with torch.cuda.graph(g, stream=s):
            work()
    torch.cuda.current_stream().wait_stream(s)
    for rep in range(3):
        ya.zero_(); yb.zero_(); W.zero_(); ws.fill_(rep)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(ya, want[0]) and torch.equal(yb, want[1]) and torch.equal(W, want[2]), rep
        _ = qp.qp_linear(wb, xb)          # eager work between the replays
        torch.cuda.synchronize()


@pytest.mark.parametrize("scheme,cb", ALL, ids=ALL_IDS)
@pytest.mark.parametrize("M,N,B", [(48, 4096, 1), (1040, 2048, 3), (16, 14336, 8), (272, 6144, 16)])
def test_block_kernel_on_canonical_layout(qp, scheme, cb, M, N, B):
    """The matrix-core kernel reads whole 16 x 1024 blocks straight from the canonical bitstream
    (no repack; a padded row stride included) with the same result as from the native layout."""
    lay = synth.make_layer(89, scheme * 10 + cb, scheme, M, N, cb)
    x = synth.make_x(89, B, B, N)
    want = oracle.linear(lay, x, threads=True)
    qp.qp_set_option(qp.QP_OPT_LINEAR_KERNEL, qp.QP_KERNEL_BLOCK)
    w = qp.Weight.from_layer(lay)
    y = qp.qp_linear(w, dev(x))
    y_nat = qp.qp_linear(qp.qp_repack(w), dev(x))
    # the same codes in a buffer with 48 bytes of padding per row
    rb = lay.codes.shape[1]
    padded = torch.zeros((M, rb + 48), dtype=torch.uint8, device="cuda")
    padded[:, :rb] = dev(lay.codes)
    wp = qp.Weight(scheme, M, N, cb, lay.vec, lay.window_bits, lay.tile, padded, w.lut, w.scales,
                   row_stride=rb + 48, tlut_bits=lay.tlut_bits)
    y_pad = qp.qp_linear(wp, dev(x))
    torch.cuda.synchronize()
    assert rel_err(host16(y), want) <= TOL_SHARP    # (and so within the stated TOL)
    assert torch.equal(y, y_nat) and torch.equal(y_pad, y_nat)
