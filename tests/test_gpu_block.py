"""A decoder block's rotations and layers as one unit (qp_block_*): the same numbers, bit for bit, as one
qp_rotate_linear call per layer - enqueued directly and as the library's own graph, replayed with the
program's own eager work between the replays and with new activations in the same buffers."""
import numpy as np
import pytest
import torch

import oracle
import synth

pytestmark = pytest.mark.gpu


def dev(a):
    if a.dtype == np.float16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.float16)
    return torch.from_numpy(a).cuda()


# (name, scheme, code_bits, M, N): an 8B-shaped block in miniature - q, k, v read one input, gate and up another
LAYERS = [("q", synth.VQ, 5, 512, 2048), ("k", synth.TCQH, 4, 128, 2048), ("v", synth.SQ, 4, 128, 2048),
          ("o", synth.TCQ, 3, 512, 2048), ("gate", synth.TCQH, 6, 1024, 2048), ("up", synth.VQ, 7, 1024, 2048),
          ("down", synth.TCQHH, 4, 2048, 6144)]
INPUT_OF = {"q": 0, "k": 0, "v": 0, "o": 1, "gate": 2, "up": 2, "down": 3}


@pytest.mark.parametrize("B", [1, 2, 5, 16])
def test_block_equals_one_call_per_layer(qp, B):
    qp.qp_set_option(qp.QP_OPT_LINEAR_KERNEL, qp.QP_KERNEL_BLOCK)
    ws, want_layers = {}, {}
    for i, (name, scheme, cb, M, N) in enumerate(LAYERS):
        lay = synth.make_layer(90, i, scheme, M, N, cb)
        ws[name] = qp.qp_repack(qp.Weight.from_layer(lay))
        want_layers[name] = lay
    xs_host = {k: synth.make_x(90, k, B, 6144 if k == 3 else 2048) for k in range(4)}
    sg_host = {k: synth.make_signs(90, k, 6144 if k == 3 else 2048) for k in range(4)}
    xs = {k: dev(v) for k, v in xs_host.items()}
    sg = {k: dev(v) for k, v in sg_host.items()}
    ys = {name: torch.zeros((B, M), dtype=torch.float16, device="cuda") for name, _, _, M, _ in LAYERS}
    rot = {name: (2048 if N == 2048 else 1024) for name, _, _, _, N in LAYERS}
    items = [(ws[name], xs[INPUT_OF[name]], sg[INPUT_OF[name]], rot[name], ys[name]) for name, *_ in LAYERS]
    blk = qp.Block(items)

    def reference():
        return {name: qp.qp_rotate_linear(ws[name], xs[INPUT_OF[name]], sg[INPUT_OF[name]], rot[name]) for name, *_ in LAYERS}

    ref = reference()
    torch.cuda.synchronize()
    # against the oracle once (the fp64 chain), then bit for bit against the per-layer calls
    for name, *_ in LAYERS:
        k = INPUT_OF[name]
        want = oracle.linear(want_layers[name], oracle.hadamard(xs_host[k], sg_host[k], rot[name], fast=True), threads=True)
        got = ref[name].cpu().numpy().astype(np.float64)
        assert np.max(np.abs(got - want)) / np.max(np.abs(want)) <= 1e-2
    blk.enqueue()
    torch.cuda.synchronize()
    for name, *_ in LAYERS:
        assert torch.equal(ys[name], ref[name]), name
    # the graph, replayed three times with new activations in the same buffers and eager work in between
    for rep in range(3):
        for k in xs:
            xs[k].copy_(dev(synth.make_x(91 + rep, k, B, xs[k].shape[1])))
        for y in ys.values():
            y.zero_()
        ref = reference()
        torch.cuda.synchronize()
        blk.run()
        torch.cuda.synchronize()
        for name, *_ in LAYERS:
            assert torch.equal(ys[name], ref[name]), (rep, name)
    blk.close()


@pytest.mark.parametrize("B", [1, 8])
def test_block_with_a_down_projection_whose_last_column_block_is_cut_short(qp, B):
    """A 7B-shaped block in miniature: the down projection reads 2816 = 11 x 256 input channels (rotation in
    blocks of 256), two of them share that input; default kernel choice."""
    shapes = [("gate", synth.VQ, 5, 2816, 2048), ("up", synth.TCQH, 6, 2816, 2048), ("down", synth.SQ, 4, 2048, 2816),
              ("down2", synth.TCQ, 3, 512, 2816)]
    inp = {"gate": 0, "up": 0, "down": 1, "down2": 1}
    width = {0: 2048, 1: 2816}
    rot = {0: 2048, 1: 256}
    lays = {name: synth.make_layer(93, i, scheme, M, N, cb) for i, (name, scheme, cb, M, N) in enumerate(shapes)}
    ws = {name: qp.qp_repack(qp.Weight.from_layer(lays[name])) for name in lays}
    xs_host = {k: synth.make_x(93, k, B, width[k]) for k in width}
    sg_host = {k: synth.make_signs(93, k, width[k]) for k in width}
    xs = {k: dev(v) for k, v in xs_host.items()}
    sg = {k: dev(v) for k, v in sg_host.items()}
    ys = {name: torch.zeros((B, M), dtype=torch.float16, device="cuda") for name, _, _, M, _ in shapes}
    blk = qp.Block([(ws[name], xs[inp[name]], sg[inp[name]], rot[inp[name]], ys[name]) for name, *_ in shapes])
    ref = {name: qp.qp_rotate_linear(ws[name], xs[inp[name]], sg[inp[name]], rot[inp[name]]) for name, *_ in shapes}
    torch.cuda.synchronize()
    for name, *_ in shapes:
        k = inp[name]
        want = oracle.linear(lays[name], oracle.hadamard(xs_host[k], sg_host[k], rot[k], fast=True), threads=True)
        got = ref[name].cpu().numpy().astype(np.float64)
        assert np.max(np.abs(got - want)) / np.max(np.abs(want)) <= 1e-3, name
    for rep in range(2):
        for y in ys.values():
            y.zero_()
        (blk.enqueue if rep == 0 else blk.run)()
        torch.cuda.synchronize()
        for name, *_ in shapes:
            assert torch.equal(ys[name], ref[name]), (rep, name)
    blk.close()


def test_block_rejects_a_bad_item_before_launching(qp):
    lay = synth.make_layer(92, 0, synth.VQ, 64, 2048, 5)
    w = qp.qp_repack(qp.Weight.from_layer(lay))
    x = dev(synth.make_x(92, 0, 1, 2048))
    sg = dev(synth.make_signs(92, 0, 2048))
    y = torch.full((1, 64), 7.0, dtype=torch.float16, device="cuda")
    y_short = torch.zeros((1, 32), dtype=torch.float16, device="cuda")       # ldy < M
    blk = qp.Block([(w, x, sg, 1024, y), (w, x, sg, 1024, y_short)])
    with pytest.raises(qp.QpError) as e:
        blk.enqueue()
    assert e.value.code == 2
    with pytest.raises(qp.QpError):
        blk.graph()
    torch.cuda.synchronize()
    assert torch.all(y == 7.0)     # the first, valid item was not launched either
