"""Fusion-aware mixed-scheme quantization (Section 4.2) on top of qp_msq_solve: turns per-layer
loss terms and per-group profiled costs into the classes of a multiple-choice knapsack and maps
the solution back to (fused group -> quantizer)."""
from __future__ import annotations

import itertools

from .binding import qp_msq_solve

# layers of a Transformer block that share their input form a cluster; a cluster may be split
# into fused groups in any way (Section 4.2: the fusible groups G_b are all non-empty subsets of
# {q, k, v}, of {u, g}, and the single layers o and d)
CLUSTERS = (("q", "k", "v"), ("o",), ("u", "g"), ("d",))


def set_partitions(items):
    """All ways of cutting a tuple into non-empty groups (order inside a group kept)."""
    items = tuple(items)
    if not items:
        yield ()
        return
    first, rest = items[0], items[1:]
    for r in range(len(rest) + 1):
        for others in itertools.combinations(rest, r):
            group = (first,) + others
            remaining = tuple(x for x in rest if x not in others)
            for tail in set_partitions(remaining):
                yield (group,) + tail


def build_classes(n_blocks, n_quant, loss, cost, fusion=True):
    """loss[(b, layer)][q], cost[(b, group)][q] with group a tuple of layer names in cluster order.
    Returns (classes, meta): classes[i] = [(loss, cost), ...]; meta[i][o] = {(b, group): q}.
    fusion=False restricts every cluster to single-layer groups (plain mixed-scheme selection).
    Options that another option of the same class beats in both loss and cost are dropped."""
    classes, meta = [], []
    for b in range(n_blocks):
        for cluster in CLUSTERS:
            opts = []
            for part in set_partitions(cluster):
                if not fusion and any(len(g) > 1 for g in part):
                    continue
                for qs in itertools.product(range(n_quant), repeat=len(part)):
                    l = sum(loss[(b, layer)][q] for g, q in zip(part, qs) for layer in g)
                    c = sum(cost[(b, g)][q] for g, q in zip(part, qs))
                    opts.append((l, c, {(b, g): q for g, q in zip(part, qs)}))
            opts.sort(key=lambda x: (x[1], x[0]))
            kept, best_loss = [], float("inf")
            for l, c, m in opts:          # ascending cost: keep only strictly better losses
                if l < best_loss:
                    kept.append((l, c, m))
                    best_loss = l
            classes.append([(l, c) for l, c, _ in kept])
            meta.append([m for _, _, m in kept])
    return classes, meta


def solve(n_blocks, n_quant, loss, cost, budget, fusion=True, resolution=20000):
    """Returns (assignment {(b, group): q}, total loss, total cost)."""
    classes, meta = build_classes(n_blocks, n_quant, loss, cost, fusion)
    choice, tl, tc = qp_msq_solve(classes, budget, resolution)
    out = {}
    for i, o in enumerate(choice):
        out.update(meta[i][o])
    return out, tl, tc
