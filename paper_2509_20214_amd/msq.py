"""Fusion-aware mixed-scheme quantization (Section 4.2): argument marshalling for qp_msq_solve_fused.
The class construction of eq. (4) - the splits of every cluster of layers into fused groups, one
quantizer per group, dominated options dropped - and the knapsack run inside the library."""
from __future__ import annotations

import ctypes as C

from .binding import _check, load_library

# order of the layers and of the twelve fusible groups of a block in the library's arrays (qp.h)
LAYERS = ("q", "k", "v", "o", "u", "g", "d")
GROUPS = (("q",), ("k",), ("v",), ("q", "k"), ("q", "v"), ("k", "v"), ("q", "k", "v"),
          ("o",), ("u",), ("g",), ("u", "g"), ("d",))
CLUSTERS = (("q", "k", "v"), ("o",), ("u", "g"), ("d",))


def solve(n_blocks, n_quant, loss, cost, budget, fusion=True, resolution=20000):
    """loss[(b, layer)][q], cost[(b, group)][q] with group one of GROUPS.
    Returns (assignment {(b, group): q} of the active groups, total loss, total cost)."""
    fl = (C.c_double * (n_blocks * len(LAYERS) * n_quant))()
    fc = (C.c_double * (n_blocks * len(GROUPS) * n_quant))()
    for b in range(n_blocks):
        for i, layer in enumerate(LAYERS):
            for q in range(n_quant):
                fl[(b * len(LAYERS) + i) * n_quant + q] = float(loss[(b, layer)][q])
        for i, group in enumerate(GROUPS):
            for q in range(n_quant):
                fc[(b * len(GROUPS) + i) * n_quant + q] = float(cost[(b, group)][q])
    assign = (C.c_int32 * (n_blocks * len(GROUPS)))()
    tl, tc = C.c_double(), C.c_double()
    _check(load_library().qp_msq_solve_fused(n_blocks, n_quant, fl, fc, float(budget), int(resolution),
                                             1 if fusion else 0, assign, C.byref(tl), C.byref(tc)), "qp_msq_solve_fused")
    out = {(b, GROUPS[i]): assign[b * len(GROUPS) + i] for b in range(n_blocks) for i in range(len(GROUPS))
           if assign[b * len(GROUPS) + i] >= 0}
    return out, tl.value, tc.value
