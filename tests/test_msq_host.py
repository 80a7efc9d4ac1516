"""Host-side mixed-scheme selection (qp_msq_solve and the fusion-aware builder) against a
brute-force statement of the paper's problems on tiny instances."""
import ctypes as C

import numpy as np
import pytest

import paper_2509_20214_amd as qp
from oracle import msq as omsq
from paper_2509_20214_amd import msq


def random_classes(g, n_classes, max_opts, cost_hi):
    out = []
    for _ in range(n_classes):
        k = int(g.integers(1, max_opts + 1))
        out.append([(float(g.uniform(0, 10)), float(g.integers(0, cost_hi + 1))) for _ in range(k)])
    return out


@pytest.mark.parametrize("seed", range(12))
def test_mckp_exact_on_integer_costs(seed):
    """Costs are whole cells of the cost axis: the dynamic programme is exact."""
    g = np.random.default_rng(seed)
    classes = random_classes(g, int(g.integers(2, 7)), 4, 9)
    budget = float(g.integers(5, 30))
    want, arg = omsq.mckp_brute(classes, budget)
    if want is None:
        with pytest.raises(qp.QpError) as e:
            qp.qp_msq_solve(classes, budget, int(budget))
        assert e.value.code == 3
        return
    choice, tl, tc = qp.qp_msq_solve(classes, budget, int(budget))     # one cell = one cost unit
    assert tc <= budget
    assert abs(tl - want) < 1e-12
    assert abs(sum(classes[i][o][0] for i, o in enumerate(choice)) - tl) < 1e-12


def test_mckp_limits_and_monotonicity():
    g = np.random.default_rng(100)
    classes = random_classes(g, 6, 5, 20)
    big, tl, tc = qp.qp_msq_solve(classes, 1e6, 1000)
    assert big == [int(np.argmin([l for l, _ in c])) for c in classes]   # no constraint: least loss per class
    least = sum(min(c for _, c in cl) for cl in classes)
    with pytest.raises(qp.QpError):
        qp.qp_msq_solve(classes, least - 1, 1000)
    prev = np.inf
    for budget in range(int(least), int(least) + 40, 3):
        _, tl, tc = qp.qp_msq_solve(classes, float(budget), budget)
        assert tc <= budget and tl <= prev + 1e-12      # more budget never hurts
        prev = tl


def test_mckp_real_costs_feasible_and_near_optimal():
    """Costs that are not multiples of the cell: always feasible, never better than the optimum,
    and no worse than the optimum for the budget reduced by one cell per class."""
    g = np.random.default_rng(7)
    for _ in range(10):
        classes = [[(float(g.uniform(0, 10)), float(g.uniform(0, 5))) for _ in range(int(g.integers(2, 5)))]
                   for _ in range(5)]
        budget, R = 12.0, 600
        opt, _ = omsq.mckp_brute(classes, budget)
        low, _ = omsq.mckp_brute(classes, budget - len(classes) * budget / R)
        if low is None:
            continue
        _, tl, tc = qp.qp_msq_solve(classes, budget, R)
        assert tc <= budget + 1e-12
        assert opt - 1e-12 <= tl <= low + 1e-12


def test_mckp_argument_errors():
    L = qp.load_library()
    beg = (C.c_int32 * 3)(0, 2, 3)
    loss = (C.c_double * 3)(1, 2, 3)
    cost = (C.c_double * 3)(1, 2, 3)
    ch = (C.c_int32 * 2)()
    call = lambda n, b, l, c, bud, r, out: L.qp_msq_solve(n, b, l, c, bud, r, out, None, None)
    assert call(2, beg, loss, cost, 10.0, 100, ch) == 0
    assert call(2, None, loss, cost, 10.0, 100, ch) == 1
    assert call(2, beg, loss, cost, 10.0, 100, None) == 1
    assert call(0, beg, loss, cost, 10.0, 100, ch) == 2
    assert call(2, beg, loss, cost, -1.0, 100, ch) == 2
    assert call(2, beg, loss, cost, 10.0, 0, ch) == 2
    assert call(2, (C.c_int32 * 3)(0, 0, 3), loss, cost, 10.0, 100, ch) == 2      # empty class
    assert call(2, beg, loss, (C.c_double * 3)(1, -2, 3), 10.0, 100, ch) == 2       # negative cost
    assert call(2, beg, loss, cost, 2.0, 100, ch) == 3                             # nothing fits


def test_group_order_is_the_headers():
    """The binding's layer / group order is the one qp.h documents (and the paper's twelve groups)."""
    assert msq.LAYERS == omsq.LAYERS and set(msq.GROUPS) == set(omsq.GROUPS) and len(msq.GROUPS) == 12
    assert msq.GROUPS == (("q",), ("k",), ("v",), ("q", "k"), ("q", "v"), ("k", "v"), ("q", "k", "v"),
                          ("o",), ("u",), ("g",), ("u", "g"), ("d",))


def test_fused_solver_argument_errors():
    L = qp.load_library()
    loss = (C.c_double * 14)(*([1.0] * 14))
    cost = (C.c_double * 24)(*([1.0] * 24))
    out = (C.c_int32 * 12)()
    call = lambda nb, nq, l, c, bud, r, o: L.qp_msq_solve_fused(nb, nq, l, c, bud, r, 1, o, None, None)
    assert call(1, 2, loss, cost, 10.0, 100, out) == 0
    assert sorted(i for i in range(12) if out[i] >= 0) == [6, 7, 10, 11]      # equal costs: the fewest groups
    assert call(1, 2, None, cost, 10.0, 100, out) == 1
    assert call(1, 2, loss, cost, 10.0, 100, None) == 1
    assert call(0, 2, loss, cost, 10.0, 100, out) == 2
    assert call(1, 17, loss, cost, 10.0, 100, out) == 2
    assert call(1, 2, loss, cost, 3.0, 100, out) == 3                         # four clusters cost at least 4
    bad = (C.c_double * 24)(*([1.0] * 23 + [-1.0]))
    assert call(1, 2, loss, bad, 10.0, 100, out) == 2


@pytest.mark.gpu
def test_fusion_aware_selection_runs_in_the_gpu_suite_too():
    """The selection is host code; this one instance is also collected by `-m gpu`, so that the run on
    the GPU machine exercises the same library build."""
    check_fusion_aware(5, 1, 2)


@pytest.mark.parametrize("seed,n_blocks,n_quant", [(0, 1, 2), (1, 1, 3), (2, 2, 2), (3, 1, 2), (4, 2, 2)])
def test_fusion_aware_selection_against_brute_force(seed, n_blocks, n_quant):
    check_fusion_aware(seed, n_blocks, n_quant)


def check_fusion_aware(seed, n_blocks, n_quant):
    """Integer costs in which a fused group is cheaper than its members one by one (as profiled
    latencies are): the class construction + knapsack equals brute force over all P[g, q] that
    satisfy (C1) and (C2); without fusion the optimum can only be worse."""
    g = np.random.default_rng(200 + seed)
    loss, cost = {}, {}
    for b in range(n_blocks):
        for layer in omsq.LAYERS:
            base = g.uniform(0.5, 2.0)
            loss[(b, layer)] = [float(base * 4.0 ** -(q + 1) * g.uniform(0.8, 1.2)) for q in range(n_quant)]
        for grp in omsq.GROUPS:
            cost[(b, grp)] = [float(int(3 + 2 * len(grp) + 2 * q + g.integers(0, 3))) for q in range(n_quant)]
    lo = sum(min(cost[(b, grp)][q] for q in range(n_quant)) for b in range(n_blocks)
             for grp in (("q", "k", "v"), ("o",), ("u", "g"), ("d",)))
    for budget in (lo + 2, lo + 7, lo + 15):
        want, arg = omsq.fusion_aware_brute(n_blocks, n_quant, loss, cost, budget)
        got, tl, tc = msq.solve(n_blocks, n_quant, loss, cost, budget, resolution=int(budget))
        assert tc <= budget
        assert abs(tl - want) < 1e-12
        # a valid P: every layer in exactly one active group
        for b in range(n_blocks):
            covered = sorted(l for (bb, grp) in got if bb == b for l in grp)
            assert covered == sorted(omsq.LAYERS)
        try:
            _, tl_plain, _ = msq.solve(n_blocks, n_quant, loss, cost, budget, fusion=False, resolution=int(budget))
            assert tl_plain >= tl - 1e-12
        except qp.QpError as e:
            assert e.code == 3        # unfused layers alone do not fit this budget
