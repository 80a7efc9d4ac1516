"""Seeded random shapes for the fused layer on the native layout: column-block counts from 1 to 32
(and a few that end inside a column block),
row-block counts on both sides of the workgroup count (one row block per workgroup, several with a
ragged last pass, fewer than 256 in all), every batch size, every scheme; checked on sampled output
rows against the oracle, through qp_linear and through the single-call step."""
import numpy as np
import pytest

import oracle
import synth

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

SCHEMES = [(synth.SQ, 4), (synth.VQ, 5), (synth.VQ, 7), (synth.TCQ, 2), (synth.TCQ, 3), (synth.TCQ, 4)] + \
          [(synth.TCQH, s) for s in range(3, 11)] + [(synth.TCQHH, s) for s in range(3, 10)]


def cases():
    g = np.random.default_rng(2024)
    out = []
    for k in range(60):
        scheme, cb = SCHEMES[k % len(SCHEMES)]
        nbc = int(g.choice([1, 2, 3, 4, 5, 6, 7, 8, 11, 14, 16, 24, 28, 32]))
        if scheme == synth.TCQHH and nbc % 2:
            nbc += 1
        rbk = int(g.choice([1, 3, 17, 100, 255, 256, 257, 300, 511, 700, 1500]))
        if rbk * nbc > 60000:       # keep the layer below ~1 G weights
            rbk = max(1, 60000 // nbc)
        B = int(g.integers(1, 17))
        out.append((k, scheme, cb, rbk * 16, nbc * 1024, B))
    # Chosen by hand: many units per workgroup, i.e. the workgroup-wide byte-window table of VQ 5 bit
    # (small layers use a per-wavefront table instead) and passes of more than 32 units at small batch.
    extra = [(synth.VQ, 5, 40, 20, 1), (synth.VQ, 5, 600, 8, 2), (synth.VQ, 5, 1100, 28, 5), (synth.VQ, 5, 300, 24, 16),
             (synth.SQ, 4, 2000, 8, 1), (synth.VQ, 7, 1300, 32, 1), (synth.TCQH, 6, 2600, 8, 1),
             (synth.TCQ, 3, 3000, 16, 2), (synth.TCQHH, 5, 1000, 14, 1), (synth.SQ, 4, 900, 28, 4),
             # VQ 5 bit at batch 1 - 2 from 20 units per workgroup on: the sixteen-copy table of code pairs
             (synth.VQ, 5, 1500, 8, 1), (synth.VQ, 5, 700, 28, 2), (synth.VQ, 5, 513, 16, 1)]
    for j, (scheme, cb, rbk, nbc, B) in enumerate(extra):
        out.append((100 + j, scheme, cb, rbk * 16, nbc * 1024, B))
    # Input channels that are a multiple of 256 but not of 1024: the last column block is cut short.
    ragged = [(synth.VQ, 5, 256, 11008, 1), (synth.SQ, 4, 100, 13824, 8), (synth.TCQ, 3, 300, 2816, 2),
              (synth.TCQH, 7, 257, 6912, 16), (synth.VQ, 7, 700, 29440, 5), (synth.TCQH, 10, 17, 1280, 3),
              (synth.TCQ, 2, 1500, 768, 13), (synth.SQ, 4, 511, 256, 1)]
    for j, (scheme, cb, rbk, N, B) in enumerate(ragged):
        out.append((200 + j, scheme, cb, rbk * 16, N, B))
    return out


def dev(a):
    if a.dtype == np.float16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.float16)
    return torch.from_numpy(a).cuda()


@pytest.mark.parametrize("k,scheme,cb,M,N,B", cases(),
                         ids=[f"{k}-{synth.SCHEME_NAMES[s]}{cb}-{M}x{N}-b{B}" for k, s, cb, M, N, B in cases()])
def test_random_shape(qp, k, scheme, cb, M, N, B):
    lay = synth.make_layer(88, k, scheme, M, N, cb)
    x = synth.make_x(88, k, B, N)
    block = synth.hadamard_block(N)
    if block > 16384:       # the rotation supports blocks up to 16384
        block = 1024
    sg = synth.make_signs(88, k, N)
    w = qp.qp_repack(qp.Weight.from_layer(lay))
    qp.qp_set_option(qp.QP_OPT_LINEAR_KERNEL, qp.QP_KERNEL_BLOCK)
    xd, sd = dev(x), dev(sg)
    xr = qp.qp_hadamard(xd, sd, block)
    y = qp.qp_linear(w, xr)
    y_step = qp.qp_rotate_linear(w, xd, sd, block)
    torch.cuda.synchronize()
    assert torch.equal(y, y_step)
    g = np.random.default_rng(k)
    rows = sorted(set(int(r) for r in g.integers(0, M, size=20)) | {0, M - 1, min(M - 1, 16 * (M // 32))})
    sub = synth.Layer(**{**lay.__dict__, "codes": lay.codes[rows], "scales": lay.scales[rows], "M": len(rows)})
    want = oracle.linear(sub, xr.cpu().view(torch.int16).numpy().view(np.uint16))
    got = y[:, torch.tensor(rows, device="cuda")].cpu().numpy().astype(np.float64)
    err = np.max(np.abs(got - want)) / np.max(np.abs(want))
    assert err <= 1e-2      # the stated bound
    assert err <= 1e-3, err  # one fp16 rounding (2^-11) plus fp32 accumulation: twice 2^-11
    assert torch.isfinite(y.float()).all()
