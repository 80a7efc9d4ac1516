"""qp_linear with and without its optional workspace: large layers at batch > 4 copy the activations
into the matrix-core kernel's fragment order when they are given one.  Both ways must give the same
bits, and sampled output rows must match the oracle; a workspace that is too small or misaligned is
ignored, not an error."""
import numpy as np
import pytest

import oracle
import synth

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

# scheme, code bits, M, N, batch: all of them ask for a workspace
CASES = [(synth.SQ, 4, 4096, 8192, 9), (synth.VQ, 5, 4096, 8192, 16), (synth.VQ, 7, 4096, 14336, 13),
         (synth.TCQ, 3, 4096, 8192, 16), (synth.TCQH, 6, 2048, 28672, 11), (synth.TCQHH, 5, 4096, 10240, 10),
         (synth.VQ, 7, 8192, 16384, 8), (synth.SQ, 4, 16384, 8192, 5), (synth.TCQH, 5, 8192, 16384, 7)]


def dev(a):
    if a.dtype == np.float16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.float16)
    return torch.from_numpy(a).cuda()


@pytest.mark.parametrize("scheme,cb,M,N,B", CASES,
                         ids=[f"{synth.SCHEME_NAMES[s]}{cb}-{M}x{N}-b{B}" for s, cb, M, N, B in CASES])
def test_workspace_or_not(qp, scheme, cb, M, N, B):
    lay = synth.make_layer(91, cb, scheme, M, N, cb)
    x = synth.make_x(91, cb, B, N)
    w = qp.qp_repack(qp.Weight.from_layer(lay))
    need = qp.qp_linear_workspace_bytes(w, B)
    assert need >= 2 * B * N
    xd = dev(x)
    ws = torch.full((need,), 0xFF, dtype=torch.uint8, device="cuda")   # NaN patterns in the unused batch columns
    y_ws = qp.qp_linear(w, xd, workspace=ws)
    y_auto = qp.qp_linear(w, xd)
    y_plain = qp.qp_linear(w, xd, workspace=False)
    y_small = qp.qp_linear(w, xd, workspace=ws[: need - 256])
    y_odd = qp.qp_linear(w, xd, workspace=torch.empty(need + 64, dtype=torch.uint8, device="cuda")[64:])
    torch.cuda.synchronize()
    for other in (y_auto, y_plain, y_small, y_odd):
        assert torch.equal(y_ws, other)
    assert torch.isfinite(y_ws.float()).all()
    g = np.random.default_rng(cb + B)
    rows = sorted(set(int(r) for r in g.integers(0, M, size=12)) | {0, M - 1})
    sub = synth.Layer(**{**lay.__dict__, "codes": lay.codes[rows], "scales": lay.scales[rows], "M": len(rows)})
    want = oracle.linear(sub, x.view(np.uint16))
    got = y_ws[:, torch.tensor(rows, device="cuda")].cpu().numpy().astype(np.float64)
    err = np.max(np.abs(got - want)) / np.max(np.abs(want))
    assert err <= 1e-2      # the stated bound
    assert err <= 1e-3, err  # one fp16 rounding (2^-11) plus fp32 accumulation: twice 2^-11


def test_strided_activations(qp):
    """Row stride larger than N: the copy follows it."""
    scheme, cb, M, N, B = synth.VQ, 5, 4096, 8192, 12
    lay = synth.make_layer(92, 0, scheme, M, N, cb)
    w = qp.qp_repack(qp.Weight.from_layer(lay))
    x = dev(synth.make_x(92, 0, B, N))
    wide = torch.zeros((B, N + 512), dtype=torch.float16, device="cuda")
    wide[:, :N] = x
    y0 = qp.qp_linear(w, x)
    y1 = qp.qp_linear(w, wide[:, :N])
    torch.cuda.synchronize()
    assert torch.equal(y0, y1)


def test_no_workspace_wanted(qp):
    """Small layers, small batches and the V = 1 trellis at batch <= 8 ask for none."""
    lay = synth.make_layer(93, 0, synth.VQ, 4096, 8192, 5)
    w = qp.qp_repack(qp.Weight.from_layer(lay))
    for B in (1, 2, 4, 8):
        assert qp.qp_linear_workspace_bytes(w, B) == 0
    assert qp.qp_linear_workspace_bytes(w, 9) == 16 * 8192 * 2
