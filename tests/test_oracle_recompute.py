"""Pins of the oracle's recomputation path (section IV-D of the paper,
"Recomputation Scheduling", and the recomputation branch of the complete
scheduling algorithm, Alg. 3): candidate savings are exact peak reductions over
the whole gap, only tensors the plan never released are candidates, the value
MSPS = saving / recomputation time orders them, and the phase runs only after
swapping has ended and only while the peak is above the budget."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import oracle as O
from workloads import make_config_plans, make_plans, plans_from_lists, small_random_tas, tas_from_lists
from workloads.plans import Plans

from helpers import touch_points


def _augment(pl: Plans, b: int, i: int, o: int, r: int) -> Plans:
    t, oo, rr, k = pl.plan(b)
    return plans_from_lists([list(zip(t.tolist(), oo.tolist(), rr.tolist())) + [(i, o, r)]])


def _numpy_recompute(tas, plan, MF, P, tstar):
    """The definition with searchsorted and slice maxima (different primitives from the oracle's loops)."""
    N = tas.N
    score = np.zeros(N, dtype=np.int64); wo = np.full(N, -1, dtype=np.int32); wi = np.full(N, -1, dtype=np.int32)
    it, io, ir = plan
    ok = (it >= 0) & (it < N) & (io >= 0) & (ir <= tas.T) & (ir > io)
    released = set(it[ok].tolist())
    for i in range(N):
        p = touch_points(tas, i)
        j = int(np.searchsorted(p, tstar, side="left"))
        if j == 0 or j == len(p) or p[j] == tstar or i in released:
            continue
        pg, pg1 = int(p[j - 1]), int(p[j])
        score[i] = P - max(int(MF[:pg + 1].max()), int(MF[pg1:].max()), P - int(tas.size_bytes[i]))
        wo[i], wi[i] = pg, pg1
    return score, wo, wi


@pytest.mark.parametrize("seed,timed", [(1, True), (2, False), (3, True)])
def test_against_numpy_statement(seed, timed):
    tas = small_random_tas(300 + seed, N=40, T=60, max_acc=5, timed=timed, link_bytes_per_us=400_000)
    pl = make_plans(tas, 12, seed, p_swap=0.15)
    res, peak, arg, mn = O.eval_plans(tas, pl)
    sc, wo, wi = O.score_recompute_plans(tas, pl, res, peak, arg)
    hits = 0
    for b in range(pl.B):
        s2, o2, i2 = _numpy_recompute(tas, pl.plan(b)[:3], res[b], int(peak[b]), int(arg[b]))
        assert np.array_equal(sc[b], s2) and np.array_equal(wo[b], o2) and np.array_equal(wi[b], i2)
        hits += int((o2 >= 0).sum())
    assert hits > 10


@pytest.mark.parametrize("idx,rows", [(0, range(6)), (1, range(2))])
def test_saving_is_exact_peak_reduction(idx, rows, configs_small):
    """saving == P - peak(plan + the whole-gap window), for every candidate; 0 <= saving <= size."""
    tas = configs_small[idx]
    pl = make_config_plans(idx, tas, B=8)
    res, peak, arg, mn = O.eval_plans(tas, pl)
    sc, wo, wi = O.score_recompute_plans(tas, pl, res, peak, arg, rows=rows)
    n_checked = 0
    for n, b in enumerate(rows):
        assert np.all(sc[n][wo[n] < 0] == 0)
        for i in np.nonzero(wo[n] >= 0)[0][:60]:
            _, p2, _, _ = O.eval_plans(tas, _augment(pl, b, int(i), int(wo[n][i]), int(wi[n][i])), want_resident=False)
            assert sc[n][i] == peak[b] - p2[0]
            n_checked += 1
        assert np.all(sc[n] >= 0) and np.all(sc[n] <= tas.size_bytes)
    assert n_checked > 20


def test_equals_swap_score_without_timing_on_an_empty_plan(configs_small):
    """No latencies => the swap window is the whole gap too, and an empty plan released nothing."""
    tas = configs_small[0]
    pl = plans_from_lists([[]])
    res, peak, arg, mn = O.eval_plans(tas, pl)
    a = O.score_plans(tas, pl, res, peak, arg)
    b = O.score_recompute_plans(tas, pl, res, peak, arg)
    assert (a[1] >= 0).sum() > 5
    for u, v in zip(a, b):
        assert np.array_equal(u, v)


def test_any_interval_of_the_tensor_excludes_it():
    # tensor 0: touches 0, 4, 9; tensor 1 makes the peak at step 6
    tas = tas_from_lists(10, [10, 3], [0, 6], [[4, 9], [7]])
    empty = plans_from_lists([[]])
    res, peak, arg, mn = O.eval_plans(tas, empty)
    sc, wo, wi = O.score_recompute_plans(tas, empty, res, peak, arg)
    assert arg[0] == 6 and sc[0].tolist() == [3, 0] and (wo[0][0], wi[0][0]) == (4, 9)
    other_gap = plans_from_lists([[(0, 1, 3)]])          # an interval in the other gap (0,4): a swap candidate still,
    res, peak, arg, mn = O.eval_plans(tas, other_gap)    # but the tensor has been released once
    assert O.score_plans(tas, other_gap, res, peak, arg)[0][0][0] == 3
    sc, wo, wi = O.score_recompute_plans(tas, other_gap, res, peak, arg)
    assert sc[0].tolist() == [0, 0] and wo[0][0] == -1
    inapplicable = plans_from_lists([[(0, 5, 5), (0, -1, 3), (7, 1, 3)]])     # skipped everywhere: releases nothing
    res, peak, arg, mn = O.eval_plans(tas, inapplicable)
    assert O.score_recompute_plans(tas, inapplicable, res, peak, arg)[0][0].tolist() == [3, 0]


def _swap_free_case(step_ns):
    """Link so slow that nothing can be swapped: the planner goes straight to recomputation.
    Tensors 0..2 (sizes 8, 8, 5) are generated at steps 0, 1, 2 and used at 9, 8, 7; tensor 3 peaks at step 5."""
    return tas_from_lists(10, [8, 8, 5, 4], [0, 1, 2, 5], [[9], [8], [7], [6]], None, step_ns, 0, 1)


def test_msps_orders_by_saving_over_generation_time():
    # equal savings for tensors 0 and 1 (8 each): the one whose generating operator is quicker goes first
    sn = [50, 20, 10, 10, 10, 10, 10, 10, 10, 10]
    tas = _swap_free_case(sn)
    g = O.greedy(tas, 0, recompute=True)
    assert g["iv_kind"].tolist() == [1, 1, 1]
    assert g["iv_tensor"].tolist() == [1, 0, 2] or g["iv_tensor"].tolist()[:1] == [1]
    first = list(zip(g["iv_tensor"].tolist(), g["iv_out"].tolist(), g["iv_in"].tolist()))[0]
    assert first == (1, 1, 8)
    # a smaller saving wins when it is cheap enough: 5/10 > 8/20 > 8/50
    sn2 = [50, 20, 10, 10, 10, 10, 10, 10, 10, 10]
    sn2[2] = 10
    tas2 = _swap_free_case(sn2)
    pl = plans_from_lists([[]])
    res, peak, arg, mn = O.eval_plans(tas2, pl)
    sc, wo, wi = O.score_recompute_plans(tas2, pl, res, peak, arg)
    value = {i: Fraction(int(sc[0][i]), sn2[int(tas2.alloc_step[i])]) for i in range(4) if wo[0][i] >= 0 and sc[0][i] > 0}
    best = max(value, key=lambda i: (value[i], int(sc[0][i]), int(tas2.size_bytes[i]), -i))
    assert O.greedy(tas2, 0, recompute=True, max_iters=1)["iv_tensor"].tolist() == [best]


def test_cross_multiplication_is_exact_for_large_operands():
    """Savings near 2^40 and latencies near 2^40: the products need more than 64 bits."""
    big = 1 << 40
    sn = [big + 1, big, 7, 7, 7, 7, 7, 7, 7, 7]
    tas = tas_from_lists(10, [big, big + 1, 5, 4], [0, 1, 2, 5], [[9], [8], [7], [6]], None, sn, 0, 1)
    # tensor 0: saving big, time big+1; tensor 1: saving big+1 (capped by what the peak allows), time big
    pl = plans_from_lists([[]])
    res, peak, arg, mn = O.eval_plans(tas, pl)
    sc, wo, wi = O.score_recompute_plans(tas, pl, res, peak, arg)
    value = {i: Fraction(int(sc[0][i]), sn[int(tas.alloc_step[i])]) for i in range(4) if wo[0][i] >= 0 and sc[0][i] > 0}
    best = max(value, key=lambda i: (value[i], int(sc[0][i]), int(tas.size_bytes[i]), -i))
    assert O.greedy(tas, 0, recompute=True, max_iters=1)["iv_tensor"].tolist() == [best]


@pytest.mark.parametrize("seed,link", [(11, 200_000), (12, 60_000)])
def test_phase_order_budget_and_validity(seed, link):
    # (the stall rule of Alg. 3 ends the whole algorithm, so it is switched off here: the swap phase
    # must end because no swap is accepted any more)
    tas = small_random_tas(400 + seed, N=150, T=240, max_acc=4, timed=True, link_bytes_per_us=link)
    no_stall = dict(min_iters=1 << 30)
    swap_only = O.greedy(tas, 0, **no_stall)
    assert np.all(swap_only["iv_kind"] == 0) and len(swap_only["iv_tensor"]) > 3
    # budget 0 can never be met: recomputation continues until nothing saves memory any more
    both = O.greedy(tas, 0, recompute=True, **no_stall)
    n_swap = len(swap_only["iv_tensor"])
    k = both["iv_kind"]
    assert np.array_equal(both["iv_tensor"][:n_swap], swap_only["iv_tensor"]) and np.all(k[:n_swap] == 0)
    assert len(k) > n_swap and np.all(k[n_swap:] == 1), "recomputation follows the swap phase and never returns to it"
    tr = both["peak_trace"]
    assert np.all(np.diff(tr) <= 0) and np.all(np.diff(tr[n_swap:]) < 0), "every recomputation lowers the peak"
    assert both["final_peak"] < swap_only["final_peak"]
    # every recomputed tensor had no other interval; its window is one whole gap around that iteration's peak
    tensors = both["iv_tensor"].tolist()
    for n in range(n_swap, len(k)):
        i = tensors[n]
        assert tensors.count(i) == 1
        p = touch_points(tas, i).tolist()
        assert both["iv_out"][n] in p and p[p.index(both["iv_out"][n]) + 1] == both["iv_in"][n]
    # the trace is what the evaluator says about the prefixes
    ivs = list(zip(tensors, both["iv_out"].tolist(), both["iv_in"].tolist()))
    _, peak, _, mn = O.eval_plans(tas, plans_from_lists([ivs[:n_swap], ivs[:n_swap + 1], ivs]), want_resident=False)
    assert peak.tolist() == [tr[n_swap], tr[n_swap + 1], tr[-1]] and np.all(mn >= 0)
    # a budget between the two final peaks stops the phase as soon as it is met
    budget = int(tr[n_swap + 1])
    some = O.greedy(tas, budget, recompute=True, **no_stall)
    assert len(some["iv_tensor"]) == n_swap + 1 and some["final_peak"] <= budget
    # a budget the swap phase already meets: no recomputation at all
    none = O.greedy(tas, int(swap_only["final_peak"]), recompute=True, **no_stall)
    assert np.array_equal(none["iv_tensor"], swap_only["iv_tensor"]) and np.all(none["iv_kind"] == 0)


def test_stall_rule_ends_both_phases(configs_small):
    """Alg. 3 leaves its loop when the peak has stalled, whichever phase it is in."""
    tas = configs_small[1]
    a = O.greedy(tas, 0)
    b = O.greedy(tas, 0, recompute=True)
    assert len(a["iv_tensor"]) > 100 and np.array_equal(a["iv_tensor"], b["iv_tensor"]) and np.all(b["iv_kind"] == 0)


def test_each_choice_maximises_msps():
    """Re-derive every recomputation choice of a run from the scores, with exact rationals."""
    tas = small_random_tas(321, N=60, T=80, max_acc=4, timed=True, link_bytes_per_us=2)     # nearly nothing swappable
    g = O.greedy(tas, 0, recompute=True)
    kinds = g["iv_kind"].tolist()
    assert kinds.count(1) >= 3
    ivs = list(zip(g["iv_tensor"].tolist(), g["iv_out"].tolist(), g["iv_in"].tolist()))
    for n, kind in enumerate(kinds):
        if kind != 1:
            continue
        pl = plans_from_lists([ivs[:n]])
        res, peak, arg, mn = O.eval_plans(tas, pl)
        sc, wo, wi = O.score_recompute_plans(tas, pl, res, peak, arg)
        cands = [i for i in range(tas.N) if wo[0][i] >= 0 and sc[0][i] > 0]
        best = max(cands, key=lambda i: (Fraction(int(sc[0][i]), int(tas.step_ns[tas.alloc_step[i]])), int(sc[0][i]),
                                         int(tas.size_bytes[i]), -i))
        assert ivs[n] == (best, int(wo[0][best]), int(wi[0][best]))
