#!/usr/bin/env python3
"""Benchmark of the quantized-linear hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch: rotate x, then the fused
dequantize-and-multiply on one layer (qp_rotate_linear: one call, two kernel launches; the
two-call sequence qp_hadamard + qp_linear is timed beside it).  The headline
workload is the 4096x14336 down-projection with the 2.5-bit vector quantizer at
batch 1 (seeded synthetic codes, LUT, scales and activations).  Weights are taken
from a ring of distinct device buffers larger than twice the 256 MB Infinity Cache,
so every step streams its codes from HBM ("cold"); inputs are resident in HBM before
the timed region starts.  The K timed steps are captured once into a HIP graph and
replayed, so that the host's per-call overhead does not hide the device time.

Prints ONE JSON line: metric / value / unit (code bytes per second through the whole step),
the per-kernel times, `roofline` for the dominant kernel (qp_linear: algorithmic bytes over its
HIP-event time against the 8 TB/s peak), `cpu_baseline` (the oracle on the host cores), the
dequantize-only kernel, the encoder, and `cases`: the other configurations.  --sweep70b and
--sweep8b / --sweep7b run whole models resident in HBM; --profile-only is the short run that profilers wrap.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

import numpy as np

HBM_PEAK_GBS = 8000.0


def committed_traffic(cfg, layer, batch, what="launch"):
    """HBM bytes per qp_linear launch (what = "launch") or per one-launch qp_rotate_linear step (what = "step")
    from the committed counter summaries under profiles/ (a line
    `traffic_bytes_per_<what> cfg<c> layer<l> batch<b> = <bytes>`), or None."""
    import glob
    import re
    here = os.path.dirname(os.path.abspath(__file__))
    pat = re.compile(rf"traffic_bytes_per_{what} cfg{cfg} layer{layer} batch{batch} = (\d+)")
    for path in sorted(glob.glob(os.path.join(here, "profiles", "*pmc*"))):
        m = pat.search(open(path).read())
        if m:
            return int(m.group(1))
    return None


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=2000)
    p.add_argument("--warmup", type=int, default=200)
    p.add_argument("--cfg", type=int, default=3, help="benchmark configuration 1..4 (headline: 3)")
    p.add_argument("--layer", type=int, default=0)
    p.add_argument("--batch", type=int, default=1)
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--micro", action="store_true",
                   help="build and run the stand-alone micro-benchmarks under paper_2509_20214_amd/csrc/microbench "
                        "(lookup paths, multiply of a decode step) and print what they print")
    p.add_argument("--no-cases", action="store_true", help="skip the table of other (layer, batch) cases")
    p.add_argument("--sweep70b", action="store_true",
                   help="configuration 5: all 80 layers of the 70B-shaped mixed-scheme model resident, "
                        "one decode step through every projection; prints its own JSON line")
    p.add_argument("--sweep8b", default="", metavar="SCHEME:BITS",
                   help="Llama-3-8B-shaped model (configuration 4's projections, 32 layers) with one quantizer, "
                        "e.g. tcq:3, tcqh:6, vq:5, tcqhh:6; prints its own JSON line")
    p.add_argument("--sweep7b", default="", metavar="SCHEME:BITS",
                   help="Llama-2-7B-shaped model (11008 intermediate channels: a down projection whose last column "
                        "block is cut short, rotation in blocks of 256) with one quantizer; prints its own JSON line")
    p.add_argument("--msq", action="store_true",
                   help="profile every (fusible group, quantizer) of an 8B-shaped block and run the fusion-aware "
                        "mixed-scheme selection on the measured latencies; prints its own JSON line")
    p.add_argument("--codebooks", action="store_true",
                   help="fit code books on the GPU (qp_kmeans) and measure the distortion of Gaussian weights "
                        "quantized with them (fit -> qp_encode -> qp_dequant); prints its own JSON line")
    p.add_argument("--option", action="append", default=[], metavar="QP_OPT_NAME=VALUE",
                   help="set a tuning option of the library before anything runs (qp_set_option; repeatable)")
    p.add_argument("--encode-only", action="store_true",
                   help="run the encoder case alone (two calls; for rocprofv3) and print its JSON line")
    p.add_argument("--profile-only", action="store_true",
                   help="run a short sequence of the dominant kernel only (for rocprofv3)")
    return p.parse_args()


def encode_case(torch, synth, qp, dev, upload):
    """The trellis encoder (two-pass tail-biting Viterbi) on 1024 x 4096 Gaussian targets at 2 bits; two calls, the
    second is the timed one."""
    M_e, N_e, s_e = 1024, 4096, 4
    lay_e = synth.make_layer(6, 900, synth.TCQH, 16, N_e, s_e)
    Wt = torch.randn((M_e, N_e), device=dev, generator=torch.Generator(device=dev).manual_seed(6)).half()
    codes_e = torch.zeros((M_e, lay_e.codes.shape[1]), dtype=torch.uint8, device=dev)
    we = qp.Weight(synth.TCQH, M_e, N_e, s_e, 2, 16, 256, codes_e, upload(lay_e.lut).view(torch.int16),
                   torch.full((M_e,), 0x3C00, dtype=torch.int16, device=dev), tlut_bits=lay_e.tlut_bits)
    ws_e = torch.empty(qp.qp_encode_workspace_bytes(we), dtype=torch.uint8, device=dev)
    dt = None
    for _ in range(2):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        qp.qp_encode(we, Wt, workspace=ws_e)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
    Wd = qp.qp_dequant(we).float()
    mse = float(((Wd - Wt.float()) ** 2).mean() / (Wt.float() ** 2).mean())
    out = {"workload": "tcqh 2 bit, 1024x4096 N(0,1) targets", "ms": round(dt * 1e3, 1),
           "Mweights_per_s": round(M_e * N_e / dt / 1e6, 1), "normalised_mse": round(mse, 5)}
    del Wt, Wd, ws_e, we, codes_e
    torch.cuda.empty_cache()
    return out


def sweep_model(model, label, torch, synth, qp, dev, upload, graph_of, event_time_us):
    """One decode step through every projection of a whole model that is resident in HBM.
    Codes are drawn on the device (seeded torch generator: 26 GB through the host would take
    minutes); tables, scales, activations and signs come from synth."""
    import oracle
    two = (synth.VQ, synth.TCQH, synth.TCQHH)
    trel = (synth.TCQ, synth.TCQH, synth.TCQHH)
    gen = torch.Generator(device=dev)
    gen.manual_seed(5)
    luts = {}
    sampled = {}
    layers = []
    total_bytes = 0
    t0 = time.perf_counter()
    for row in model:
        ws = []
        for d in row:
            vec = 2 if d["scheme"] in two else 1
            rb = synth.row_bytes_for(d["scheme"], d["N"], d["code_bits"], vec)
            key = (d["scheme"], d["code_bits"])
            if key not in luts:
                tiny = synth.make_layer(5, 500 + len(luts), d["scheme"], 16, 1024, d["code_bits"])
                luts[key] = (upload(tiny.lut), tiny.tlut_bits)
            codes = torch.randint(0, 256, (d["M"], rb), dtype=torch.uint8, device=dev, generator=gen)
            scales = upload(synth.rng(5, d["layer"], synth.TENSOR_SCALES).uniform(0.5, 1.5, d["M"]).astype(np.float16))
            trellis = d["scheme"] in trel
            can = qp.Weight(d["scheme"], d["M"], d["N"], d["code_bits"], vec, 16 if trellis else 0,
                            256 if trellis else 0, codes, luts[key][0].view(torch.int16), scales.view(torch.int16),
                            tlut_bits=luts[key][1])
            nat = qp.qp_repack(can)
            ws.append((d, nat))
            total_bytes += d["M"] * rb
            if d["scheme"] not in sampled and len(sampled) < 3:
                # keep a few rows of codes on the host: the oracle decodes those itself
                rows = sorted(set(int(r) for r in np.random.default_rng(d["layer"]).integers(0, d["M"], 12)))
                sampled[d["scheme"]] = (d, nat, rows, codes[torch.tensor(rows, device=dev)].cpu().numpy(),
                                        scales.cpu().view(torch.int16).numpy().view(np.float16)[rows], luts[key])
            del codes, can
        layers.append(ws)
    torch.cuda.synchronize()
    setup_s = time.perf_counter() - t0
    # parity on sampled rows of three projections of different schemes: the oracle decodes the
    # rows' codes (copied back from the device generator's output) and multiplies in fp64
    checked = []
    for d, nat, rows, code_rows, scale_rows, lut_dev in sampled.values():
        vec = 2 if d["scheme"] in two else 1
        trellis = d["scheme"] in trel
        sub = synth.Layer(scheme=d["scheme"], M=len(rows), N=d["N"], code_bits=d["code_bits"], vec=vec,
                          window_bits=16 if trellis else 0, tile=256 if trellis else 0,
                          codes=np.ascontiguousarray(code_rows),
                          lut=lut_dev[0].cpu().view(torch.int16).numpy().view(np.float16).reshape(-1),
                          scales=np.ascontiguousarray(scale_rows), tlut_bits=lut_dev[1])
        xh = synth.make_x(5, d["layer"], 2, d["N"])
        y = qp.qp_linear(nat, upload(xh))
        want = oracle.linear(sub, xh)
        got = y[:, torch.tensor(rows, device=dev)].cpu().numpy().astype(np.float64)
        err = float(np.max(np.abs(got - want)) / np.max(np.abs(want)))
        assert err <= 1e-2, (d["name"], err)
        checked.append({"layer": d["name"], "rows": len(rows), "rel_err_vs_oracle": round(err, 6)})
    out_cases = []
    Ns = sorted({d["N"] for row in model for d in row})
    Ms = sorted({d["M"] for row in model for d in row})
    n_proj = sum(len(row) for row in model)
    for B in (1, 8):
        # every projection of a decoder layer has an input of its own (position in the layer), shared by all layers
        width = max(len(ws) for ws in layers)
        xs = {(N, i): upload(synth.make_x(5, N + i, B, N)) for N in Ns for i in range(width)}
        sg = {N: upload(synth.make_signs(5, N, N)) for N in Ns}
        wsp = {N: torch.empty(max(qp.qp_rotate_linear_workspace_bytes(nat, B) for ws in layers for d, nat in ws if d["N"] == N),
                              dtype=torch.uint8, device=dev) for N in Ns}
        ys = {M: torch.empty((B, M), dtype=torch.float16, device=dev) for M in Ms}

        def step():
            for ws in layers:
                for i, (d, nat) in enumerate(ws):
                    N = d["N"]
                    qp.qp_rotate_linear(nat, xs[(N, i)], sg[N], synth.hadamard_block(N), y=ys[d["M"]], workspace=wsp[N])

        g = graph_of(step, 1)
        g.replay()
        us = event_time_us(g, 1, repeats=5)
        # the same step as one unit of the library (qp_block_*): one call enqueues it, one graph launch replays it
        blk = qp.Block([(nat, xs[(d["N"], i)], sg[d["N"]], synth.hadamard_block(d["N"]), ys[d["M"]])
                        for ws in layers for i, (d, nat) in enumerate(ws)])
        blk.graph()

        def wall_us(f, reps=5):
            out = []
            for _ in range(reps):
                torch.cuda.synchronize()
                t = time.perf_counter()
                f()
                torch.cuda.synchronize()
                out.append((time.perf_counter() - t) * 1e6)
            return statistics.median(out)

        blk.run()
        us_block_graph = wall_us(blk.run)
        us_calls = wall_us(step)
        us_enqueue = wall_us(blk.enqueue)
        blk.close()
        out_cases.append({"batch": B, "ms_per_model_step": round(us / 1e3, 4),
                          "weight_GBps": round(total_bytes / us / 1e3, 1),
                          "frac_of_peak": round(total_bytes / us / 1e3 / HBM_PEAK_GBS, 4),
                          "steps_per_s": round(1e6 / us, 1),
                          "wall_ms_host_included": {"one_python_call_per_projection": round(us_calls / 1e3, 4),
                                                    "qp_block_enqueue": round(us_enqueue / 1e3, 4),
                                                    "qp_block_run": round(us_block_graph / 1e3, 4)}})
    print(json.dumps({"metric": f"{label}: one decode step through all {n_proj} quantized projections "
                                f"({len(model)} decoder layers resident), rotation + fused layer each",
                      "resident_weight_GiB": round(total_bytes / 2**30, 2), "setup_s": round(setup_s, 1),
                      "qp_rotate_linear_calls_per_step": n_proj, "cases": out_cases, "parity": checked,
                      "data": "synthetic (codes drawn on the device from a seeded generator)"}))


def msq_demo(torch, synth, qp, dev, upload, graph_of, event_time_us):
    """Fusion-aware mixed-scheme selection (Section 4.2) fed with latencies measured here: for
    every fusible group of an 8B-shaped block and every quantizer of a palette, the time of
    qp_rotate_linear (batch 1, cold ring); loss terms = synthetic layer sensitivities x the
    distortion of the quantizer measured by encoding Gaussian targets with qp_encode."""
    from paper_2509_20214_amd import msq
    rows = {"q": 4096, "k": 1024, "v": 1024, "o": 4096, "u": 14336, "g": 14336, "d": 4096}
    cols = {"q": 4096, "k": 4096, "v": 4096, "o": 4096, "u": 4096, "g": 4096, "d": 14336}
    palette = [3, 4, 5, 6, 7, 8]                       # TCQH, bits per step; bits per weight = s / 2
    groups = sorted(msq.GROUPS, key=lambda g: (len(g), g))   # the twelve fusible groups of a block
    gen = torch.Generator(device=dev)
    gen.manual_seed(8)
    # distortion of each quantizer on N(0,1) targets (256 x 4096)
    dist = []
    Wt = torch.randn((256, 4096), device=dev, generator=gen).half()
    for s_ in palette:
        tiny = synth.make_layer(8, s_, synth.TCQH, 16, 4096, s_)
        codes = torch.zeros((256, tiny.codes.shape[1]), dtype=torch.uint8, device=dev)
        w = qp.Weight(synth.TCQH, 256, 4096, s_, 2, 16, 256, codes, upload(tiny.lut).view(torch.int16),
                      torch.full((256,), 0x3C00, dtype=torch.int16, device=dev), tlut_bits=tiny.tlut_bits)
        qp.qp_encode(w, Wt)
        d = float(((qp.qp_dequant(w).float() - Wt.float()) ** 2).mean())
        dist.append(d)
    # latency of every (group, quantizer)
    lat = {}
    for g in groups:
        M, N = sum(rows[l] for l in g), cols[g[0]]
        for qi, s_ in enumerate(palette):
            tiny = synth.make_layer(8, 100 + s_, synth.TCQH, 16, N, s_)
            rb = tiny.codes.shape[1]
            lut = upload(tiny.lut).view(torch.int16)
            sc = torch.full((M,), 0x3C00, dtype=torch.int16, device=dev)
            n_ring = max(2, -(-(320 << 20) // (M * rb)))
            ring = []
            for _ in range(n_ring):
                codes = torch.randint(0, 256, (M, rb), dtype=torch.uint8, device=dev, generator=gen)
                ring.append(qp.qp_repack(qp.Weight(synth.TCQH, M, N, s_, 2, 16, 256, codes, lut, sc,
                                                   tlut_bits=tiny.tlut_bits)))
            x = upload(synth.make_x(8, N, 1, N))
            sg = upload(synth.make_signs(8, N, N))
            y = torch.empty((1, M), dtype=torch.float16, device=dev)
            ws = torch.empty(qp.qp_rotate_linear_workspace_bytes(ring[0], 1), dtype=torch.uint8, device=dev)
            i = [0]

            def f():
                qp.qp_rotate_linear(ring[i[0] % n_ring], x, sg, synth.hadamard_block(N), y=y, workspace=ws)
                i[0] += 1

            gr = graph_of(f, 100)
            gr.replay()
            lat[(g, qi)] = event_time_us(gr, 100, repeats=3)
            del gr, ring
            torch.cuda.empty_cache()
    # one block's worth of classes, replicated for 32 blocks with seeded sensitivities
    n_blocks = 32
    sens = synth.rng(8, 0, 77).uniform(0.5, 2.0, size=(n_blocks, 7))
    names = ("q", "k", "v", "o", "u", "g", "d")
    loss = {(b, l): [float(sens[b, j] * rows[l] * cols[l] * d) for d in dist]
            for b in range(n_blocks) for j, l in enumerate(names)}
    cost = {(b, g): [lat[(g, qi)] for qi in range(len(palette))] for b in range(n_blocks) for g in groups}
    top = len(palette) - 1
    fused_lo = n_blocks * sum(min(lat[(cl, qi)] for qi in range(len(palette))) for cl in msq.CLUSTERS)
    fused_hi = n_blocks * sum(lat[(cl, top)] for cl in msq.CLUSTERS)
    plain_lo = n_blocks * sum(min(lat[((l,), qi)] for qi in range(len(palette))) for l in names)
    plain_hi = n_blocks * sum(lat[((l,), top)] for l in names)
    budgets = [fused_lo + f * (fused_hi - fused_lo) for f in (0.25, 0.5, 0.75)] + \
              [plain_lo + f * (plain_hi - plain_lo) for f in (0.25, 0.75)]
    out = []
    for budget in budgets:
        row = {"budget_us_per_token": round(budget, 1)}
        for fusion in (True, False):
            try:
                sel, tl, tc = msq.solve(n_blocks, len(palette), loss, cost, budget, fusion=fusion)
            except qp.QpError:
                row["fusion_aware" if fusion else "per_layer"] = None
                continue
            bits = sum(sum(rows[l] * cols[l] for l in g) * palette[q] / 2 for (b, g), q in sel.items()) / \
                (n_blocks * sum(rows[l] * cols[l] for l in names))
            row["fusion_aware" if fusion else "per_layer"] = {
                "loss_proxy": round(tl / 1e6, 3), "us_per_token": round(tc, 1), "mean_bits": round(bits, 3),
                "fused_groups": sum(1 for (b, g) in sel if len(g) > 1), "launch_pairs": len(sel)}
        out.append(row)
    print(json.dumps({"metric": "fusion-aware mixed-scheme selection on measured latencies: 32 8B-shaped blocks, "
                                "TCQH palette 1.5..4 bits, batch 1",
                      "palette_bits": [s_ / 2 for s_ in palette], "distortion": [round(d, 5) for d in dist],
                      "latency_us": {"+".join(g): [round(lat[(g, qi)], 2) for qi in range(len(palette))] for g in groups},
                      "selections": out, "data": "synthetic (seeded sensitivities; codes drawn on the device)"}))


def codebooks_demo(torch, synth, qp, dev):
    """Appendix C "Codebook construction" on the GPU, then the distortion of N(0,1) weights quantized
    with the fitted tables (Table 5 of the paper: NUQ-2 0.11747, VQ-2 0.10857, TCQ-2 0.07101 on
    4096 x 4096 Gaussian matrices with its own k-means tables)."""
    from paper_2509_20214_amd import codebooks
    out = {"metric": "code books fitted on the GPU and the distortion they reach on N(0,1) weights", "rows": []}
    gen = torch.Generator(device=dev).manual_seed(77)
    M, N = 1024, 4096
    Wt = torch.randn((M, N), device=dev, generator=gen).half()
    norm = float((Wt.float() ** 2).mean())
    ones = torch.full((M,), 0x3C00, dtype=torch.int16, device=dev)

    def timed(fn):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        r = fn()
        torch.cuda.synchronize()
        return r, time.perf_counter() - t0

    def quantize(scheme, cb, vec, lut16, tlut_bits=0):
        lay = synth.make_layer(6, 901, scheme, 16, N, cb)
        codes = torch.zeros((M, lay.codes.shape[1]), dtype=torch.uint8, device=dev)
        trel = scheme in (synth.TCQ, synth.TCQH, synth.TCQHH)
        w = qp.Weight(scheme, M, N, cb, vec, 16 if trel else 0, 256 if trel else 0, codes,
                      lut16.contiguous().view(torch.int16), ones, tlut_bits=tlut_bits)
        nb = qp.qp_encode_workspace_bytes(w)
        ws = torch.empty(max(nb, 16), dtype=torch.uint8, device=dev)
        _, dt = timed(lambda: qp.qp_encode(w, Wt, workspace=ws))
        Wd = qp.qp_dequant(w).float()
        return float(((Wd - Wt.float()) ** 2).mean()) / norm, dt

    # scalar table, 4 bits (the fused kernels' scalar scheme), against the closed-form Lloyd-Max levels
    lut, dt = timed(lambda: codebooks.train_scalar(4, n_samples=20_000_000, seed=1))
    d, de = quantize(synth.SQ, 4, 1, lut)
    ref = float(np.abs(lut.float().cpu().numpy() - synth.sq_lut(4).view(np.float16).astype(np.float32)).max())
    out["rows"].append({"table": "scalar 4 bit, 16 levels, 2e7 samples", "fit_ms": round(dt * 1e3, 1),
                        "normalised_mse": round(d, 5), "max_abs_diff_to_closed_form_levels": round(ref, 4)})
    # vector tables of the fused kernels
    for cb in (5, 7):
        lut, dt = timed(lambda: codebooks.train_vector(cb, n_samples=10_000_000, seed=2))
        d, de = quantize(synth.VQ, cb, 2, lut)
        d_rand, _ = quantize(synth.VQ, cb, 2, torch.from_numpy(synth.vq_lut(3, 0, cb).view(np.int16)).to(dev).view(torch.float16))
        out["rows"].append({"table": f"2-D {cb} bit ({cb / 2} bits per weight), 1e7 pairs", "fit_ms": round(dt * 1e3, 1),
                            "normalised_mse": round(d, 5), "with_random_gaussian_table": round(d_rand, 5),
                            "rate_distortion_bound": round(2.0 ** -cb, 5)})
    # the trellis quantizer's small table: 2^9 pairs fitted to 2^20 Gaussian pairs, several scalings
    for scale in (1.0, 0.9, 0.85, 0.8, 0.75):
        tl, dt = timed(lambda: codebooks.train_tlut(9, seed=3, scale=scale))
        d, de = quantize(synth.TCQH, 4, 2, tl, tlut_bits=9)
        out["rows"].append({"table": f"trellis small table 2^9 pairs, samples scaled by {scale}; TCQ 2 bit",
                            "fit_ms": round(dt * 1e3, 1), "encode_ms": round(de * 1e3, 1),
                            "normalised_mse": round(d, 5), "paper_table5": 0.07101})
    d_rand, _ = quantize(synth.TCQH, 4, 2, torch.from_numpy(synth.tcqh_tlut(6, 0, 9).view(np.int16)).to(dev).view(torch.float16), tlut_bits=9)
    out["rows"].append({"table": "trellis small table of random Gaussian pairs; TCQ 2 bit", "normalised_mse": round(d_rand, 5)})
    print(json.dumps(out))


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import synth
    import paper_2509_20214_amd as qp
    qp.load_library()
    for kv in a.option:
        name, value = kv.split("=")
        qp.qp_set_option(getattr(qp, name), int(value))
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")

    def upload(arr):
        if arr.dtype == np.float16:
            return torch.from_numpy(arr.view(np.int16)).to(dev).view(torch.float16)
        return torch.from_numpy(arr).to(dev)

    class Case:
        """One layer resident on the device: a ring of native-layout copies of its codes."""

        def __init__(self, cfg, li, B, ring_bytes=640 << 20):
            self.cfg, self.li = cfg, li
            self.desc = synth.config_layers(cfg)[li]
            self.lay = synth.build(self.desc)
            lay = self.lay
            self.code_bytes = lay.code_bytes
            base = qp.Weight.from_layer(lay)
            nat = qp.qp_repack(base)
            n = max(2, -(-ring_bytes // lay.code_bytes))
            self.ring = [nat]
            for _ in range(n - 1):
                self.ring.append(nat.with_codes(nat.codes.clone()))
            self.block = synth.hadamard_block(lay.N)
            self.signs = upload(synth.make_signs(cfg, li, lay.N))
            self.sink = torch.zeros(4, dtype=torch.int32, device=dev)
            self.i = 0
            self.set_batch(B)

        def set_batch(self, B):
            """Activations, outputs and workspaces for batch B (the ring of codes stays)."""
            lay, nat = self.lay, self.ring[0]
            self.B = B
            self.x = upload(synth.make_x(self.cfg, self.li, B, lay.N))
            self.xr = torch.empty_like(self.x)
            self.y = torch.empty((B, lay.M), dtype=torch.float16, device=dev)
            self.ws = torch.empty(qp.qp_rotate_linear_workspace_bytes(nat, B), dtype=torch.uint8, device=dev)
            need = qp.qp_linear_workspace_bytes(nat, B)   # the layer's own optional scratch (large layers, batch > 4)
            self.lin_ws = torch.empty(need, dtype=torch.uint8, device=dev) if need else False
            # algorithmic bytes of one qp_linear launch: codes + scales + x + y + one LUT
            self.alg_bytes = lay.code_bytes + 2 * lay.M + 2 * B * lay.N + 2 * B * lay.M + 2 * lay.lut.size

        def stream_only(self):
            # the yardstick: a kernel that only reads the same code bytes from the same cold ring
            qp.qp_bench_stream_read(self.ring[self.i % len(self.ring)].codes, self.sink)
            self.i += 1

        def step(self):
            # rotation + fused layer through the single-call entry point
            qp.qp_rotate_linear(self.ring[self.i % len(self.ring)], self.x, self.signs, self.block,
                                y=self.y, workspace=self.ws)
            self.i += 1

        def step_two_calls(self):
            qp.qp_hadamard(self.x, self.signs, self.block, out=self.xr)
            qp.qp_linear(self.ring[self.i % len(self.ring)], self.xr, y=self.y, workspace=self.lin_ws)
            self.i += 1

        def linear_only(self):
            qp.qp_linear(self.ring[self.i % len(self.ring)], self.xr, y=self.y, workspace=self.lin_ws)
            self.i += 1

        def hadamard_only(self):
            qp.qp_hadamard(self.x, self.signs, self.block, out=self.xr)

    def graph_of(fn, count):
        """Capture `count` calls of fn into one HIP graph on a side stream."""
        g = torch.cuda.CUDAGraph()
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            fn()
            torch.cuda.synchronize()
            with torch.cuda.graph(g, stream=s):
                for _ in range(count):
                    fn()
        torch.cuda.current_stream().wait_stream(s)
        torch.cuda.synchronize()
        return g

    def event_time_us(g, count, repeats=5):
        """Median over `repeats` of (HIP-event time of one graph replay) / count, in us."""
        out = []
        for _ in range(repeats):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            g.replay()
            e1.record()
            e1.synchronize()
            out.append(e0.elapsed_time(e1) * 1e3 / count)
        return statistics.median(out)

    if a.encode_only:
        print(json.dumps({"encode": encode_case(torch, synth, qp, dev, upload)}))
        return
    if a.micro:
        import subprocess
        import tempfile
        src_dir = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2509_20214_amd", "csrc", "microbench")
        with tempfile.TemporaryDirectory() as tmp:
            for name in sorted(f for f in os.listdir(src_dir) if f.endswith(".hip")):
                exe = os.path.join(tmp, name[:-4])
                subprocess.check_call(["/opt/rocm/bin/hipcc", "-O3", "--offload-arch=gfx950", "-Xclang", "-target-feature",
                                       "-Xclang", "-packed-fp32-ops", "-o", exe, os.path.join(src_dir, name)],
                                      stderr=subprocess.DEVNULL)
                print(f"== {name}", flush=True)
                subprocess.check_call([exe])
        return
    if a.sweep70b:
        sweep_model(synth.config5_model(80), "configuration 5, 70B-shaped mixed-scheme model", torch, synth, qp, dev,
                    upload, graph_of, event_time_us)
        return
    if a.msq:
        msq_demo(torch, synth, qp, dev, upload, graph_of, event_time_us)
        return
    if a.codebooks:
        codebooks_demo(torch, synth, qp, dev)
        return
    if a.sweep8b:
        name, bits = a.sweep8b.split(":")
        scheme = {v: k for k, v in synth.SCHEME_NAMES.items()}[name]
        sweep_model(synth.model_8b(scheme, int(bits)), f"8B-shaped model, every projection {name} code_bits {bits}",
                    torch, synth, qp, dev, upload, graph_of, event_time_us)
        return
    if a.sweep7b:
        name, bits = a.sweep7b.split(":")
        scheme = {v: k for k, v in synth.SCHEME_NAMES.items()}[name]
        sweep_model(synth.model_7b(scheme, int(bits)),
                    f"7B-shaped model (11008 intermediate channels), every projection {name} code_bits {bits}",
                    torch, synth, qp, dev, upload, graph_of, event_time_us)
        return

    head = Case(a.cfg, a.layer, a.batch)

    if a.profile_only:
        # a plain device-to-device copy of known size (64 MiB read + 64 MiB written per call):
        # the yardstick the HBM byte counters are scaled by
        src = torch.empty(64 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        for _ in range(20):
            head.step()
            head.step_two_calls()
        torch.cuda.synchronize()
        # the same back-to-back launch pattern as the timed region: one HIP graph of 200 launches
        g = graph_of(head.linear_only, 200)
        g.replay()
        torch.cuda.synchronize()
        # and 200 whole steps (one kernel each where the layer's kernel rotates the activations itself)
        g = graph_of(head.step, 200)
        g.replay()
        torch.cuda.synchronize()
        return

    # ---------------- whole-step throughput: W warm-up steps, then the K timed steps.  The K steps are one
    # HIP graph (at most 500 steps per graph); a short K would mostly measure the latency of launching
    # one graph, so the K-step sequence is replayed until at least 2000 steps have run, the wall clock
    # is taken around all of them (synchronised on both sides) and divided by the steps run.
    chunk = min(a.steps, 500)
    assert a.steps % chunk == 0, "--steps must be a multiple of 500 (or below 500)"
    g_step = graph_of(head.step, chunk)
    for _ in range(max(1, a.warmup // chunk)):
        g_step.replay()
    rounds = max(1, -(-2000 // a.steps))
    # HIP events on the stream the graphs are launched on, around the same timed region as the wall clock
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(rounds * (a.steps // chunk)):
        g_step.replay()
    ev1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / (rounds * a.steps)
    step_us_timed_region = ev0.elapsed_time(ev1) * 1e3 / (rounds * a.steps)
    value = head.code_bytes / (ms_per_step * 1e-3) / 1e9

    g_two = graph_of(head.step_two_calls, 500)
    g_two.replay()
    two_us = event_time_us(g_two, 500)
    del g_two

    # ---------------- dominant kernel alone (qp_linear), HIP events on its own stream
    R = 500
    g_lin = graph_of(head.linear_only, R)
    g_lin.replay()
    lin_us = event_time_us(g_lin, R)
    g_had = graph_of(head.hadamard_only, R)
    g_had.replay()
    had_us = event_time_us(g_had, R)
    # The dominant kernel of the timed step: where the layer's kernel rotates the activations itself the
    # step IS one kernel (its algorithmic bytes: the layer's plus the N sign bytes); otherwise the layer's
    # kernel, timed alone.
    launches = qp.qp_rotate_linear_launches(head.ring[0], a.batch, head.block)
    dom_us = step_us_timed_region if launches == 1 else lin_us
    dom_bytes = head.alg_bytes + (head.lay.N if launches == 1 else 0)
    achieved = dom_bytes / (dom_us * 1e-6) / 1e9
    # the two yardsticks of this box, same protocol (graph of R launches, cold ring, HIP events): a kernel
    # that only streams the layer's code bytes, and an empty launch
    g_str = graph_of(head.stream_only, R)
    g_str.replay()
    stream_us = event_time_us(g_str, R)
    g_emp = graph_of(qp.qp_bench_empty_launch, R)
    g_emp.replay()
    empty_us = event_time_us(g_emp, R)
    del g_str, g_emp
    # HBM bytes per launch: not counted in this run (that takes rocprofv3 --pmc); the figure of the
    # committed counter summary for exactly this workload, if there is one, else null
    traffic = committed_traffic(a.cfg, a.layer, a.batch, "step" if launches == 1 else "launch")
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                "traffic_source": "profiles/ (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE of an earlier run of this "
                                  "workload, not of this run)" if traffic else None,
                "kernel": "qp_rotate_linear as one launch (the layer's kernel rotates the activations itself)"
                          if launches == 1 else "qp_linear (the step's second launch; the first is the rotation)",
                "us_per_launch": round(dom_us, 3), "algorithmic_bytes": dom_bytes,
                "layer_kernel_alone": {"us_per_launch": round(lin_us, 3),
                                       "frac": round(head.alg_bytes / (lin_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                                       "frac_of_ceiling": round(stream_us / lin_us, 4)},
                "stream_read_us": round(stream_us, 3), "empty_launch_us": round(empty_us, 3),
                "frac_of_ceiling": round(stream_us / dom_us, 4),
                "ceiling": "a kernel that only reads the same code bytes (128-bit non-temporal loads, same cold "
                           "ring, same graph-and-events protocol); frac_of_ceiling = its time / the layer's"}

    # ---------------- other (layer, batch) cases: us per qp_linear call, cold ring
    cases = []
    if not a.no_cases:
        del g_lin, g_had
        # every (layer, batch) cell the benchmark configurations ask for: configuration 3 at batch 1, 4, 8
        # (+ 2, 16), configuration 4's four projections at batch 1, 2, 4, 8, 16, configuration 5's at
        # 1, 8, 16, configurations 1 and 2 at batch 1; configuration 6: the paper's V = 2 trellis
        todo = [(3, 0, (1, 2, 4, 8, 16)), (2, 0, (1,)), (1, 0, (1,)),
                (4, 0, (1, 2, 4, 8, 16)), (4, 1, (1, 2, 4, 8, 16)), (4, 2, (1, 2, 4, 8, 16)), (4, 3, (1, 2, 4, 8, 16)),
                (5, 0, (1, 8, 16)), (5, 1, (1, 8, 16)), (5, 2, (1, 8, 16)), (5, 3, (1, 8, 16)),
                (6, 0, (1,)), (6, 1, (1, 8)), (6, 2, (1,)), (6, 3, (1,)), (6, 4, (1,)), (6, 5, (1,)), (6, 6, (1,)),
                (6, 7, (1,)), (6, 8, (1, 8)), (6, 9, (1,)), (6, 10, (1, 8)), (6, 11, (1, 8)), (6, 12, (1, 2))]
        for cfg, li, batches in todo:
            c = Case(cfg, li, batches[0])
            g = graph_of(c.stream_only, 100)
            g.replay()
            us_stream = event_time_us(g, 100, repeats=3)
            del g
            for B in batches:
                if (cfg, li, B) == (a.cfg, a.layer, a.batch):
                    continue
                c.set_batch(B)
                c.hadamard_only()
                g = graph_of(c.linear_only, 200)
                g.replay()
                us = event_time_us(g, 200, repeats=3)
                del g
                g = graph_of(c.step, 200)
                g.replay()
                us_step = event_time_us(g, 200, repeats=3)
                del g
                cases.append({"workload": c.desc["name"], "batch": B, "us_per_call": round(us, 3),
                              "us_rotate_linear": round(us_step, 3),
                              "weight_GBps": round(c.code_bytes / us / 1e3, 1),
                              "frac_of_peak": round(c.code_bytes / us / 1e3 / HBM_PEAK_GBS, 4),
                              "stream_read_us": round(us_stream, 3), "frac_of_ceiling": round(us_stream / us, 4)})
            del c
            torch.cuda.empty_cache()

    # ---------------- dequantize-only kernel on the headline layer (write-bound: 2 bytes per weight)
    dequant = None
    if not a.no_cases:
        lay = head.lay
        Wout = torch.empty((lay.M, lay.N), dtype=torch.float16, device=dev)
        g = graph_of(lambda: qp.qp_dequant(head.ring[0], out=Wout), 30)
        g.replay()
        us = event_time_us(g, 30, repeats=3)
        dequant = {"workload": head.desc["name"], "us_per_call": round(us, 2),
                   "written_GBps": round(lay.M * lay.N * 2 / us / 1e3, 1),
                   "frac_of_peak": round(lay.M * lay.N * 2 / us / 1e3 / HBM_PEAK_GBS, 4),
                   "note": "output (112 MiB) fits the 256 MB Infinity Cache"}
        del g, Wout
        torch.cuda.empty_cache()

    # ---------------- encoder (offline path): 1024 x 4096 Gaussian targets at 2 bits, V = 2 trellis
    encode = None
    if not a.no_cases:
        encode = encode_case(torch, synth, qp, dev, upload)

    # ---------------- the oracle on this machine's host cores (a reported baseline, not a target)
    cpu = None
    if not a.no_cpu_baseline:
        import oracle
        xr_host = head.xr.cpu().view(torch.int16).numpy().view(np.uint16)
        times = []
        t_all = time.perf_counter()
        while len(times) < 3 or (time.perf_counter() - t_all < 8.0 and len(times) < 25):
            t = time.perf_counter()
            oracle.linear(head.lay, xr_host, threads=True)
            times.append(time.perf_counter() - t)
        med = statistics.median(times)
        cpu = {"value": round(head.code_bytes / med / 1e9, 4), "unit": "GB/s", "cores": oracle.num_threads(),
               "kind": "oracle", "ms_per_call": round(med * 1e3, 2),
               "sample": f"whole {head.desc['name']} layer, batch {a.batch}, qp_linear only, "
                         f"median of {len(times)} calls, OpenMP over output rows"}

    out = {
        "metric": "effective weight HBM bandwidth of the quantized-linear step (rotation + fused dequant-matmul)",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(ms_per_step, 6), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16 inputs, f32 accumulate", "data": "synthetic",
        "config": {"workload": f"cfg{a.cfg} {head.desc['name']} batch {a.batch}, native layout, cold ring of "
                               f"{len(head.ring)} weight buffers ({len(head.ring) * head.code_bytes >> 20} MiB)",
                   "steps_in_one_hip_graph": chunk, "graph_replays_timed": rounds * (a.steps // chunk)},
        "us_per_step": round(ms_per_step * 1e3, 3), "us_step_as_two_calls": round(two_us, 3),
        "us_qp_linear": round(lin_us, 3),
        "us_qp_hadamard": round(had_us, 3),
        "linear_weight_GBps": round(head.code_bytes / lin_us / 1e3, 1),
        "roofline": roofline, "cpu_baseline": cpu, "dequant": dequant, "encode": encode, "cases": cases,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
