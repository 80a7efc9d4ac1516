"""Parity at the benchmark's full sizes and launch configuration: the GPU output of a
whole layer is checked on sampled output rows that the oracle computes one by one, and
the dequantized matrix on sampled rows bit for bit."""
import numpy as np
import pytest

import oracle
import synth

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

CASES = [  # (cfg, layer index, batches)
    (1, 0, [1]),
    (2, 0, [1]),
    (3, 0, [1, 4, 8]),
    (4, 0, [1, 16]),
    (4, 1, [1, 4]),
    (4, 2, [1, 8]),
    (4, 3, [1, 2, 8]),
    (5, 0, [1]),
    (5, 1, [1]),
    (5, 2, [1, 8]),
    (5, 3, [1, 8]),
    (6, 1, [1, 8]),
    (6, 6, [1]),
    (6, 8, [1, 8]),
]


def sample_rows(M, k=24, seed=0):
    g = np.random.default_rng(seed)
    rows = set(int(r) for r in g.integers(0, M, size=k))
    rows.update([0, 15, 16, M - 17, M - 1])
    return sorted(rows)


@pytest.mark.parametrize("cfg,li,batches", CASES)
def test_full_size_layer_on_sampled_rows(qp, cfg, li, batches):
    desc = synth.config_layers(cfg)[li]
    lay = synth.build(desc)
    w_can = qp.Weight.from_layer(lay)
    w = qp.qp_repack(w_can)
    rows = sample_rows(lay.M, seed=cfg * 10 + li)
    # decode, sampled rows, both layouts
    Wd = qp.qp_dequant(w)
    Wc = qp.qp_dequant(w_can)
    sub = synth.Layer(**{**lay.__dict__, "codes": lay.codes[rows], "scales": lay.scales[rows], "M": len(rows)})
    want_W = oracle.decode(sub)
    idx = torch.tensor(rows, device="cuda")
    for Wg in (Wd, Wc):
        got = Wg[idx].cpu().view(torch.int16).numpy().view(np.uint16)
        assert np.array_equal(got, want_W)
    del Wd, Wc
    block = synth.hadamard_block(lay.N)
    sg = synth.make_signs(cfg, li, lay.N)
    for B in batches:
        x = synth.make_x(cfg, li, B, lay.N)
        xd = torch.from_numpy(x.view(np.int16)).cuda().view(torch.float16)
        sgd = torch.from_numpy(sg).cuda()
        xr = qp.qp_hadamard(xd, sgd, block)
        y = qp.qp_linear(w, xr)
        # the single-call step that bench.py times: same numbers, bit for bit
        y_step = qp.qp_rotate_linear(w, xd, sgd, block)
        torch.cuda.synchronize()
        assert torch.equal(y_step, y)
        xr_host = xr.cpu().view(torch.int16).numpy().view(np.uint16)
        # isolated check: the oracle multiplies the very fp16 xr the kernel received
        want = oracle.linear(sub, xr_host)
        got = y[:, idx].cpu().numpy().astype(np.float64)
        scale = np.max(np.abs(want))
        assert np.max(np.abs(got - want)) / scale <= 1e-2
        # chained check against fp64 rotation
        want2 = oracle.linear(sub, oracle.hadamard(x, sg, block, fast=True))
        assert np.max(np.abs(got - want2)) / np.max(np.abs(want2)) <= 1e-2
        assert torch.isfinite(y.float()).all()
