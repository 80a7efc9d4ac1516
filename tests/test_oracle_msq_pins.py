"""Pins of oracle/msq.py (the brute-force statements of eq. (3) and eq. (4)) against instances
worked by hand and the structural facts of Section 4.2.  None of them involves the library."""
import itertools

from oracle import msq as omsq


# --------------------------------------------------------------------- eq. (3), by hand
# Three layers, two quantizers each, (loss, cost):
#   layer 0: (5, 1) (1, 3)     layer 1: (4, 1) (2, 2)     layer 2: (3, 2) (0.5, 4)
# The eight selections, as (choice per layer): cost, loss
#   000: 4, 12     001: 6, 9.5    010: 5, 10     011: 7, 7.5
#   100: 6, 8      101: 8, 5.5    110: 7, 6      111: 9, 3.5
EQ3 = [[(5.0, 1.0), (1.0, 3.0)], [(4.0, 1.0), (2.0, 2.0)], [(3.0, 2.0), (0.5, 4.0)]]


def test_eq3_hand_worked_budgets():
    # budget 7 is met with equality by 110 (loss 6) and 011 (loss 7.5): "cost <= C", not "<"
    assert omsq.mckp_brute(EQ3, 7.0) == (6.0, (1, 1, 0))
    # a hair below 7: 110 and 011 drop out, 100 (cost 6, loss 8) beats 001 (cost 6, loss 9.5)
    assert omsq.mckp_brute(EQ3, 6.999) == (8.0, (1, 0, 0))
    assert omsq.mckp_brute(EQ3, 8.0) == (5.5, (1, 0, 1))
    assert omsq.mckp_brute(EQ3, 9.0) == (3.5, (1, 1, 1))
    assert omsq.mckp_brute(EQ3, 100.0) == (3.5, (1, 1, 1))
    assert omsq.mckp_brute(EQ3, 4.0) == (12.0, (0, 0, 0))       # the cheapest selection, exactly affordable
    assert omsq.mckp_brute(EQ3, 3.999) == (None, None)          # nothing fits


def test_eq3_every_layer_gets_exactly_one_quantizer():
    """A class with a single option must take it whatever it costs; a selection never skips a layer."""
    classes = [[(1.0, 5.0)], [(2.0, 1.0), (0.0, 2.0)]]
    assert omsq.mckp_brute(classes, 7.0) == (1.0, (0, 1))
    assert omsq.mckp_brute(classes, 6.5) == (3.0, (0, 0))
    assert omsq.mckp_brute(classes, 5.5) == (None, None)


# --------------------------------------------------------------------- eq. (4), by hand
# One block, two quantizers (0: few bits, 1: more bits).  Loss terms per layer (quantizer 0, 1):
LOSS = {"q": (4.0, 1.0), "k": (2.0, 0.5), "v": (2.0, 0.5), "o": (3.0, 1.0), "u": (5.0, 1.0), "g": (5.0, 1.0),
        "d": (6.0, 2.0)}
# Profiled cost per group (quantizer 0, 1): a fused group is cheaper than its members one by one
COST_FUSING_PAYS = {("q",): (3, 4), ("k",): (2, 3), ("v",): (2, 3), ("q", "k"): (4, 6), ("q", "v"): (4, 6),
                    ("k", "v"): (3, 4), ("q", "k", "v"): (5, 7), ("o",): (3, 4), ("u",): (4, 6), ("g",): (4, 6),
                    ("u", "g"): (6, 9), ("d",): (4, 6)}


def as_inputs(cost_table):
    loss = {(0, l): [float(x) for x in v] for l, v in LOSS.items()}
    cost = {(0, g): [float(x) for x in v] for g, v in cost_table.items()}
    return loss, cost


def test_eq4_fusing_wins():
    """All seven layers at quantizer 1 is the least loss there is: 1 + .5 + .5 + 1 + 1 + 1 + 2 = 7.  The
    cheapest way to have it is {q,k,v} {o} {u,g} {d}: 7 + 4 + 9 + 6 = 26 (one by one: 4+3+3+4+6+6+6 = 32)."""
    loss, cost = as_inputs(COST_FUSING_PAYS)
    best, arg = omsq.fusion_aware_brute(1, 2, loss, cost, 26.0)
    assert best == 7.0
    assert arg == {(0, ("q", "k", "v")): 1, (0, ("o",)): 1, (0, ("u", "g")): 1, (0, ("d",)): 1}
    # budget 25.5: one cluster must step down; the cheapest step in loss is o -> quantizer 0
    # (loss + 2, cost - 1; d: + 4, - 2; {u,g}: + 8, - 3; {q,k,v}: + 6, - 2; splitting {q,k,v} only costs more)
    best, arg = omsq.fusion_aware_brute(1, 2, loss, cost, 25.5)
    assert best == 9.0 and arg[(0, ("o",))] == 0 and arg[(0, ("q", "k", "v"))] == 1
    # the per-layer problem (single-layer groups only) at the same budget of 26: everything at
    # quantizer 0 costs 3+2+2+3+4+4+4 = 22 with loss 27; four cost units buy q -> 1 (- 3, + 1),
    # o -> 1 (- 2, + 1) and one of u, g, d -> 1 (- 4, + 2): loss 18
    singles = {g: c for g, c in COST_FUSING_PAYS.items() if len(g) == 1}
    classes = [[(LOSS[g[0]][q], float(singles[g][q])) for q in range(2)] for g in singles]
    assert omsq.mckp_brute(classes, 26.0)[0] == 18.0


def test_eq4_fusing_loses():
    """Fused groups that cost one unit more than their members together are never active: the
    fusion-aware optimum is the per-layer optimum (18 at budget 26, see above)."""
    table = dict(COST_FUSING_PAYS)
    for g in table:
        if len(g) > 1:
            table[g] = tuple(sum(COST_FUSING_PAYS[(l,)][q] for l in g) + 1 for q in range(2))
    loss, cost = as_inputs(table)
    best, arg = omsq.fusion_aware_brute(1, 2, loss, cost, 26.0)
    assert best == 18.0
    assert all(len(g) == 1 for (_, g) in arg) and len(arg) == 7


def test_eq4_every_one_of_the_twelve_groups_can_be_chosen():
    """{q,v} is the group a careless enumeration forgets (its layers are not neighbours): made
    almost free, it must be taken.  {q,v}@1 + {k}@1 = loss 2 at cost 1 + 3 = 4, against 7 for {q,k,v}@1:
    all layers at quantizer 1 then cost 4 + 4 + 9 + 6 = 23."""
    table = dict(COST_FUSING_PAYS)
    table[("q", "v")] = (1, 1)
    loss, cost = as_inputs(table)
    best, arg = omsq.fusion_aware_brute(1, 2, loss, cost, 23.0)
    assert best == 7.0 and arg[(0, ("q", "v"))] == 1 and arg[(0, ("k",))] == 1
    for group in omsq.GROUPS:       # the same with every group in turn: the free group is always active
        table = {g: (50, 50) for g in omsq.GROUPS}
        # single layers stay affordable so that a cover exists around the free group
        for g in omsq.GROUPS:
            if len(g) == 1:
                table[g] = (10, 10)
        table[group] = (0, 0)
        loss, cost = as_inputs(table)
        _, arg = omsq.fusion_aware_brute(1, 2, loss, cost, 70.0)
        assert (0, group) in arg, group


def test_eq4_constraint_c1_every_layer_exactly_once():
    loss, cost = as_inputs(COST_FUSING_PAYS)
    for budget in (22.0, 24.0, 26.0, 30.0, 40.0):
        _, arg = omsq.fusion_aware_brute(1, 2, loss, cost, budget)
        covered = sorted(l for (_, g) in arg for l in g)
        assert covered == sorted(omsq.LAYERS)
    # below the cheapest cover ({q,k,v} {o} {u,g} {d} at quantizer 0: 5 + 3 + 6 + 4 = 18) nothing fits
    assert omsq.fusion_aware_brute(1, 2, loss, cost, 17.9) == (None, None)
    assert omsq.fusion_aware_brute(1, 2, loss, cost, 18.0)[0] == 27.0


# --------------------------------------------------------------------- structure (Section 4.2)
def test_group_structure_of_a_block():
    assert len(omsq.LAYERS) == 7 and len(omsq.GROUPS) == 12 and len(set(omsq.GROUPS)) == 12
    # the groups are exactly the non-empty subsets of {q,k,v} and of {u,g} plus o and d
    want = set()
    for cluster in (("q", "k", "v"), ("u", "g"), ("o",), ("d",)):
        for r in range(1, len(cluster) + 1):
            want |= set(itertools.combinations(cluster, r))
    assert set(omsq.GROUPS) == want
    # twelve group variables per block against seven layer variables: the 1.71 x the paper states
    assert round(len(omsq.GROUPS) / len(omsq.LAYERS), 2) == 1.71
    # ways of covering every layer of a block exactly once: 5 splits of {q,k,v} x 2 splits of {u,g}
    covers = [sub for r in range(1, 13) for sub in itertools.combinations(omsq.GROUPS, r)
              if sorted(l for g in sub for l in g) == sorted(omsq.LAYERS)]
    assert len(covers) == 10


def test_eq4_two_blocks_share_one_budget():
    """Two copies of the hand-worked block under one budget of 26 + 25 = 51: one block keeps everything
    at quantizer 1 (26), the other steps o down (25): loss 7 + 9 = 16; at 52 both keep everything: 14."""
    l1, c1 = as_inputs(COST_FUSING_PAYS)
    loss = {**l1, **{(1, l): v for (_, l), v in l1.items()}}
    cost = {**c1, **{(1, g): v for (_, g), v in c1.items()}}
    assert omsq.fusion_aware_brute(2, 2, loss, cost, 52.0)[0] == 14.0
    assert omsq.fusion_aware_brute(2, 2, loss, cost, 51.0)[0] == 16.0
