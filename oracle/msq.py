"""Brute-force statement of the mixed-scheme selection problems, for tiny instances only.
Test infrastructure: only tests may import this.

Section 4.1 eq. (3): one quantizer per layer, least summed loss, summed cost within the budget.
Section 4.2 eq. (4): binary P[g, q] over the fusible groups of every Transformer block
    G_b = {q},{k},{v},{q,k},{q,v},{k,v},{q,k,v},{o},{u},{g},{u,g},{d}
and the quantizers; (C1) every layer lies in exactly one active (group, quantizer) pair;
(C2) the summed profiled cost of the active pairs stays within C; the objective sums the loss
terms of the layers of every active pair.
"""
from __future__ import annotations

import itertools

LAYERS = ("q", "k", "v", "o", "u", "g", "d")
GROUPS = (("q",), ("k",), ("v",), ("q", "k"), ("q", "v"), ("k", "v"), ("q", "k", "v"),
          ("o",), ("u",), ("g",), ("u", "g"), ("d",))


def mckp_brute(classes, budget):
    """classes: list of lists of (loss, cost).  Returns (best loss, choices) or (None, None)."""
    best, arg = None, None
    for sel in itertools.product(*[range(len(c)) for c in classes]):
        cost = sum(classes[i][o][1] for i, o in enumerate(sel))
        if cost > budget:
            continue
        loss = sum(classes[i][o][0] for i, o in enumerate(sel))
        if best is None or loss < best:
            best, arg = loss, sel
    return best, arg


def fusion_aware_brute(n_blocks, n_quant, loss, cost, budget):
    """loss[(b, layer)][q], cost[(b, group)][q].  Enumerates every P that satisfies (C1), keeps
    those within (C2), returns (least loss, {(b, group): q}) or (None, None)."""
    per_block = []
    for b in range(n_blocks):
        sols = []
        # every subset of G_b that covers each of the seven layers exactly once
        for r in range(1, len(GROUPS) + 1):
            for sub in itertools.combinations(GROUPS, r):
                covered = [l for g in sub for l in g]
                if sorted(covered) != sorted(LAYERS):
                    continue
                for qs in itertools.product(range(n_quant), repeat=len(sub)):
                    l = sum(loss[(b, layer)][q] for g, q in zip(sub, qs) for layer in g)
                    c = sum(cost[(b, g)][q] for g, q in zip(sub, qs))
                    sols.append((l, c, {(b, g): q for g, q in zip(sub, qs)}))
        per_block.append(sols)
    best, arg = None, None
    for combo in itertools.product(*per_block):
        c = sum(x[1] for x in combo)
        if c > budget:
            continue
        l = sum(x[0] for x in combo)
        if best is None or l < best:
            best = l
            arg = {}
            for x in combo:
                arg.update(x[2])
    return best, arg
