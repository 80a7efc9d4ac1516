"""The GPU encoders against the CPU oracle.  Encoders have several correct answers (ties, and
the two-pass trellis heuristic depends on a choice of shared bits), so what is compared is what is
unique: the error a stream decodes to (recomputed by the oracle in fp64 from the GPU's bytes),
optimality for the shared bits the GPU chose (the oracle's constrained pass is exact for them),
and agreement of the choice itself with the oracle's two-pass encoder on most tiles."""
import numpy as np
import pytest

import oracle
import synth

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def dev16(a):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda().view(torch.float16)


def targets(seed, M, N):
    return np.random.default_rng(seed).standard_normal((M, N)).astype(np.float16)


@pytest.mark.parametrize("scheme,cb", [(synth.SQ, 4), (synth.VQ, 5), (synth.VQ, 7)])
@pytest.mark.parametrize("M,N", [(8, 256), (37, 1280)])
def test_nearest_entry_encoders(qp, scheme, cb, M, N):
    """Every weight (pair) gets an entry that is as close as the oracle's choice up to fp32
    rounding of the distances; almost all codes are identical."""
    lay = synth.make_layer(90, cb, scheme, M, N, cb)
    Wt = targets(90 + cb, M, N)
    w = qp.Weight.from_layer(lay)
    w.codes.fill_(0xAA)
    qp.qp_encode(w, dev16(Wt))
    torch.cuda.synchronize()
    got_codes = w.codes.cpu().numpy()
    lay_g = synth.Layer(**{**lay.__dict__, "codes": got_codes})
    dec_g = oracle.half_to_double(oracle.decode(lay_g))
    v = oracle.half_to_double(Wt)
    want_codes = np.stack([(oracle.rtn_sq(v[j], cb, lay.lut) if scheme == synth.SQ else
                            oracle.rtn_vq(v[j], cb, 2, lay.lut)) for j in range(M)])
    lay_c = synth.Layer(**{**lay.__dict__, "codes": want_codes})
    dec_c = oracle.half_to_double(oracle.decode(lay_c))
    if scheme == synth.SQ:
        dg, dc = np.abs(dec_g - v), np.abs(dec_c - v)
    else:
        dg = ((dec_g - v) ** 2).reshape(M, -1, 2).sum(-1)
        dc = ((dec_c - v) ** 2).reshape(M, -1, 2).sum(-1)
    assert np.all(dg <= dc * (1 + 1e-3) + 1e-6)
    assert np.mean(got_codes == want_codes) > 0.995


TRELLIS = [(synth.TCQ, 2), (synth.TCQ, 3), (synth.TCQ, 4), (synth.TCQH, 3), (synth.TCQH, 4), (synth.TCQH, 5),
           (synth.TCQH, 6), (synth.TCQH, 7), (synth.TCQH, 8), (synth.TCQH, 9), (synth.TCQH, 10)]


def full_table(lay):
    if lay.scheme == synth.TCQ:
        return lay.lut
    return oracle.hybrid_lut(lay.lut, lay.tlut_bits).view(np.float16).reshape(-1)


def check_tiles(v_tiles, streams, errs_gpu, s, V, table, agree_min, two_pass=True):
    """v_tiles [nt, 256] fp64, streams [nt, bytes] from the GPU.  two_pass=False skips the
    comparison with the oracle's own two-pass encoder (its cost grows with 2^s per state)."""
    nt = v_tiles.shape[0]
    same = 0
    e_true = np.empty(nt)
    e_two = np.empty(nt)
    for i in range(nt):
        e_true[i] = oracle.tcq_tile_error(v_tiles[i], streams[i], s, 16, 256, V, table)
        ov = int.from_bytes(streams[i, :2].tobytes(), "little") & ((1 << (16 - s)) - 1)
        _, e_con = oracle.tcq_encode_constrained(v_tiles[i], s, 16, 256, V, table, ov)
        # optimal for the shared bits it chose: not better than the exact optimum, and no worse
        # than fp32 rounding of path costs allows
        assert e_true[i] >= e_con - 1e-9
        assert e_true[i] <= e_con * (1 + 2e-4) + 1e-4, (i, e_true[i], e_con)
        if two_pass:
            st2, e_two[i] = oracle.tcq_encode(v_tiles[i], s, 16, 256, V, table)
            ov2 = int.from_bytes(st2[:2].tobytes(), "little") & ((1 << (16 - s)) - 1)
            same += ov == ov2
    if errs_gpu is not None:   # what the kernel reports is the error of what it wrote
        assert np.allclose(errs_gpu, e_true, rtol=2e-3, atol=1e-3)
    if not two_pass:
        return
    assert same >= agree_min * nt, (same, nt)
    # on the tiles where the shared bits differ the two answers are of the same quality
    assert abs(e_true.mean() - e_two.mean()) <= 0.01 * e_two.mean()


@pytest.mark.parametrize("scheme,s", TRELLIS)
def test_trellis_encoder(qp, scheme, s):
    # 10 tiles, two per row; fewer where the oracle's passes get slow (2^s predecessors per state)
    M, N = (5 if s <= 6 else 2 if s <= 8 else 1), 512
    V = 1 if scheme == synth.TCQ else 2
    lay = synth.make_layer(91, s, scheme, M, N, s)
    Wt = targets(91 * 7 + s, M, N)
    w = qp.Weight.from_layer(lay)
    w.codes.fill_(0x55)
    err = qp.qp_encode(w, dev16(Wt), tile_err=True)
    torch.cuda.synchronize()
    codes = w.codes.cpu().numpy()
    tb = codes.shape[1] // (N // 256)
    v = oracle.half_to_double(Wt).reshape(M * (N // 256), 256)
    check_tiles(v, codes.reshape(M * (N // 256), tb), err.cpu().numpy().reshape(-1), s, V, full_table(lay), 0.8,
                two_pass=s <= 7)
    # the GPU decodes its own codes to what the oracle decodes them to, and the distortion is that
    # of a trellis quantizer at this rate (between the rate-distortion bound and twice it)
    lay_g = synth.Layer(**{**lay.__dict__, "codes": codes})
    assert np.array_equal(qp.qp_dequant(w).cpu().view(torch.int16).numpy().view(np.uint16), oracle.decode(lay_g))
    if scheme == synth.TCQH:   # random Gaussian code book of 2^9..2^11 pairs: a sane quantizer at s/2 bits
        mse = ((oracle.half_to_double(oracle.decode(lay_g)) - oracle.half_to_double(Wt)) ** 2).mean()
        assert 2.0 ** (-s) < mse < 3.0 * 2.0 ** (-s), mse


def test_trellis_encoder_small_workspace_and_many_tiles(qp):
    """Workspace for three workgroups only: each encodes several tiles one after the other."""
    s, M, N = 4, 4, 1024
    lay = synth.make_layer(92, 0, synth.TCQH, M, N, s)
    Wt = targets(920, M, N)
    w = qp.Weight.from_layer(lay)
    per_wg = qp.qp_encode_workspace_bytes(w) // (M * N // 256)
    ws = torch.empty(3 * per_wg, dtype=torch.uint8, device="cuda")
    err = qp.qp_encode(w, dev16(Wt), tile_err=True, workspace=ws)
    torch.cuda.synchronize()
    codes = w.codes.cpu().numpy()
    v = oracle.half_to_double(Wt).reshape(-1, 256)
    check_tiles(v, codes.reshape(v.shape[0], -1), err.cpu().numpy().reshape(-1), s, 2, full_table(lay), 0.75)
    with pytest.raises(qp.QpError):
        qp.qp_encode(w, dev16(Wt), workspace=ws[: per_wg - 16])


@pytest.mark.parametrize("s", [3, 4, 5, 8])
def test_half_tcq_encoder(qp, s):
    """First half of the input channels at s bits per step, second half at s + 1 (App. C.3.2)."""
    M, N = (3 if s <= 5 else 1), 1024
    lay = synth.make_layer(93, s, synth.TCQHH, M, N, s)
    Wt = targets(930 + s, M, N)
    w = qp.Weight.from_layer(lay)
    err = qp.qp_encode(w, dev16(Wt), tile_err=True)
    torch.cuda.synchronize()
    codes = w.codes.cpu().numpy()
    nb0 = N // 4 * s // 8
    v = oracle.half_to_double(Wt)
    e = err.cpu().numpy()
    table = full_table(lay)
    check_tiles(v[:, : N // 2].reshape(-1, 256), np.ascontiguousarray(codes[:, :nb0]).reshape(M * 2, -1),
                e[:, :2].reshape(-1), s, 2, table, 0.7, two_pass=s <= 5)
    check_tiles(v[:, N // 2:].reshape(-1, 256), np.ascontiguousarray(codes[:, nb0:]).reshape(M * 2, -1),
                e[:, 2:].reshape(-1), s + 1, 2, table, 0.7, two_pass=s <= 5)


def test_encode_then_linear_end_to_end(qp):
    """Quantize a Gaussian matrix on the GPU, repack, multiply: the product differs from the
    product with the unquantized matrix by what the quantizer's distortion predicts."""
    s, M, N, B = 6, 48, 2048, 4
    lay = synth.make_layer(94, 0, synth.TCQH, M, N, s)
    Wt = targets(94, M, N)
    w = qp.Weight.from_layer(lay)
    w.scales.fill_(0x3C00)   # fp16 1.0: the check is about W^, not the scales
    qp.qp_encode(w, dev16(Wt))
    x = synth.make_x(94, 0, B, N)
    qp.qp_set_option(qp.QP_OPT_LINEAR_KERNEL, qp.QP_KERNEL_BLOCK)
    y = qp.qp_linear(qp.qp_repack(w), dev16(x)).cpu().numpy().astype(np.float64)
    lay_g = synth.Layer(**{**lay.__dict__, "codes": w.codes.cpu().numpy(), "scales": np.ones(M, dtype=np.float16)})
    want = oracle.linear(lay_g, x)
    assert np.max(np.abs(y - want)) / np.max(np.abs(want)) <= 1e-2
    exact = oracle.half_to_double(x) @ oracle.half_to_double(Wt).T
    rel = np.linalg.norm(want - exact) / np.linalg.norm(exact)
    assert 0.05 < rel < 0.25, rel     # sqrt(MSE) at 3 bits is about 2^-3 .. 1.5 * 2^-3


def test_row_normalize(qp):
    M, N = 37, 1280
    W = (np.random.default_rng(96).standard_normal((M, N)) * np.linspace(0.01, 30, M)[:, None]).astype(np.float16)
    W[5] = 0
    Wd = torch.zeros((M, N + 64), dtype=torch.float16, device="cuda")
    Wd[:, :N] = dev16(W)
    sc = qp.qp_row_normalize(Wd[:, :N])
    torch.cuda.synchronize()
    w64 = oracle.half_to_double(W)
    s_ref = np.sqrt((w64 ** 2).mean(1))
    s_ref[5] = 1.0
    s_got = sc.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(s_got - s_ref) <= 2.0 ** -10 * s_ref)          # fp16 rounding of the scale
    out = Wd[:, :N].cpu().numpy().astype(np.float64)
    want = w64 / s_got[:, None]
    assert np.all(np.abs(out - want) <= 2.0 ** -10 * np.abs(want) + 1e-7)
    assert np.all(Wd[:, N:].cpu().numpy() == 0)                         # nothing written past the row
    assert np.allclose((out ** 2).mean(1)[np.arange(M) != 5], 1.0, atol=3e-3)


def test_offline_path_then_online_path(qp):
    """A dense weight matrix through the whole offline path (rotate rows, scale, encode, repack),
    then the online path on unrotated activations: y approximates x W^T as closely as the
    quantizer's distortion allows (Section 3.3: X W = (X R)(R^T W))."""
    s, M, N, B, block = 6, 64, 2048, 3, 1024
    g = np.random.default_rng(97)
    Wfull = (g.standard_normal((M, N)) * g.uniform(0.5, 2.0, M)[:, None]).astype(np.float16)
    Wfull[:, 7] *= 20.0       # an outlier column: what the rotation is there to spread
    x = synth.make_x(97, 0, B, N)
    sg = synth.make_signs(97, 0, N)
    lay = synth.make_layer(97, 0, synth.TCQH, M, N, s)
    w = qp.Weight.from_layer(lay)
    sgd = torch.from_numpy(sg).cuda()
    Wr = qp.qp_hadamard(dev16(Wfull), sgd, block)
    w.scales.copy_(qp.qp_row_normalize(Wr).view(torch.int16))
    qp.qp_encode(w, Wr)
    qp.qp_set_option(qp.QP_OPT_LINEAR_KERNEL, qp.QP_KERNEL_BLOCK)
    y = qp.qp_rotate_linear(qp.qp_repack(w), dev16(x), sgd, block).cpu().numpy().astype(np.float64)
    exact = oracle.half_to_double(x) @ oracle.half_to_double(Wfull).T
    rel = np.linalg.norm(y - exact) / np.linalg.norm(exact)
    assert rel < 0.2, rel          # 3 bits: relative error about sqrt(0.021) = 0.145
    # and the fp64 chain on the GPU's own codes and scales agrees with the GPU's product
    lay_g = synth.Layer(**{**lay.__dict__, "codes": w.codes.cpu().numpy(),
                           "scales": w.scales.cpu().numpy().view(np.float16)})
    want = oracle.linear(lay_g, oracle.hadamard(x, sg, block))
    assert np.max(np.abs(y - want)) / np.max(np.abs(want)) <= 1e-2
