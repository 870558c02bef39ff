"""Pins of the oracle's candidate scores (candidate choice and feasible windows of
the paper's swap scheduling, section IV-C)."""
import os

import numpy as np
import pytest

from oracle import oracle as O
from workloads import CONFIGS, make_config_plans, make_plans, plans_from_lists, small_random_tas, tas_from_lists
from workloads.plans import Plans

from helpers import numpy_scores, parse_fixture_lines, touch_points
from test_oracle_eval import _hand


def _augment(pl: Plans, b: int, i: int, o: int, r: int) -> Plans:
    t, oo, rr, k = pl.plan(b)
    return plans_from_lists([list(zip(t.tolist(), oo.tolist(), rr.tolist())) + [(i, o, r)]])


def test_hand_example_scores():
    tas, get = _hand()
    pl = plans_from_lists([[]])
    res, peak, arg, mn = O.eval_plans(tas, pl)
    sc, wo, wi = O.score_plans(tas, pl, res, peak, arg)
    assert sc[0].tolist() == get("score") and wo[0].tolist() == get("window_out") and wi[0].tolist() == get("window_in")


@pytest.mark.parametrize("idx,rows", [(0, range(8)), (1, range(2))])
def test_score_is_exact_peak_reduction(idx, rows, configs_small):
    """score == P - peak(plan + the reported window), for every candidate."""
    tas = configs_small[idx]
    pl = make_config_plans(idx, tas, B=8)
    res, peak, arg, mn = O.eval_plans(tas, pl)
    sc, wo, wi = O.score_plans(tas, pl, res, peak, arg, rows=rows)
    n_checked = 0
    for n, b in enumerate(rows):
        cand = np.nonzero(wo[n] >= 0)[0]
        assert np.all(sc[n][wo[n] < 0] == 0)
        for i in cand:
            _, p2, _, _ = O.eval_plans(tas, _augment(pl, b, int(i), int(wo[n][i]), int(wi[n][i])), want_resident=False)
            assert sc[n][i] == peak[b] - p2[0]
            n_checked += 1
        assert np.all(sc[n] >= 0) and np.all(sc[n] <= tas.size_bytes)
    assert n_checked > 20


@pytest.mark.parametrize("seed,timed", [(1, True), (2, True), (3, False), (4, True), (5, False)])
def test_against_numpy_statement(seed, timed):
    tas = small_random_tas(200 + seed, N=40, T=60, max_acc=5, timed=timed, link_bytes_per_us=400_000)
    pl = make_plans(tas, 12, seed, p_swap=0.25)
    res, peak, arg, mn = O.eval_plans(tas, pl)
    sc, wo, wi = O.score_plans(tas, pl, res, peak, arg)
    hits = 0
    for b in range(pl.B):
        s2, o2, i2 = numpy_scores(tas, pl.plan(b)[:3], res[b], int(peak[b]), int(arg[b]))
        assert np.array_equal(sc[b], s2) and np.array_equal(wo[b], o2) and np.array_equal(wi[b], i2)
        hits += int((o2 >= 0).sum())
    assert hits > 10


def test_medium_against_numpy_statement(configs_small):
    tas = configs_small[1]
    pl = make_config_plans(1, tas, B=3)
    res, peak, arg, mn = O.eval_plans(tas, pl)
    sc, wo, wi = O.score_plans(tas, pl, res, peak, arg)
    for b in range(pl.B):
        s2, o2, i2 = numpy_scores(tas, pl.plan(b)[:3], res[b], int(peak[b]), int(arg[b]))
        assert np.array_equal(sc[b], s2) and np.array_equal(wo[b], o2) and np.array_equal(wi[b], i2)
    assert (wo >= 0).sum() > 300 and (sc > 0).sum() > 100
    # some candidates must be limited by transfer time (window narrower than the gap)
    narrowed = 0
    for i in np.nonzero(wo[0] >= 0)[0]:
        p = touch_points(tas, int(i))
        narrowed += int(wo[0][i] not in p)
    assert narrowed > 0


def test_no_timing_means_whole_gap(configs_small):
    tas = configs_small[0]
    assert tas.step_ns is None
    pl = make_config_plans(0, tas, B=4)
    res, peak, arg, mn = O.eval_plans(tas, pl)
    sc, wo, wi = O.score_plans(tas, pl, res, peak, arg)
    for b in range(4):
        for i in np.nonzero(wo[b] >= 0)[0]:
            p = touch_points(tas, int(i))
            j = int(np.searchsorted(p, arg[b]))
            assert wo[b][i] == p[j - 1] and wi[b][i] == p[j]


def test_slow_link_leaves_no_candidate(configs_small):
    tas = configs_small[1]
    import copy
    slow = copy.copy(tas)
    slow.link_bytes_per_us = 1                        # one byte per microsecond
    pl = make_config_plans(1, tas, B=1)
    res, peak, arg, mn = O.eval_plans(slow, pl)
    sc, wo, wi = O.score_plans(slow, pl, res, peak, arg)
    big = tas.size_bytes > 1 << 20
    assert np.all(sc[0][big] == 0) and np.all(wo[0][big] == -1)


def test_blocked_only_by_interval_in_the_same_gap():
    # tensor 0: touches 0, 4, 9; tensor 1 makes the peak at step 6
    tas = tas_from_lists(10, [10, 3], [0, 6], [[4, 9], [7]])
    empty = plans_from_lists([[]])
    res, peak, arg, mn = O.eval_plans(tas, empty)
    assert arg[0] == 6 and peak[0] == 13
    sc, wo, wi = O.score_plans(tas, empty, res, peak, arg)
    assert sc[0].tolist() == [3, 0] and wo[0][0] == 4 and wi[0][0] == 9     # new peak 10 at step 0
    other_gap = plans_from_lists([[(0, 1, 3)]])                             # interval in gap (0,4): not blocking
    res, peak, arg, mn = O.eval_plans(tas, other_gap)
    sc, wo, wi = O.score_plans(tas, other_gap, res, peak, arg)
    assert arg[0] == 6 and sc[0][0] == 3
    same_gap = plans_from_lists([[(0, 7, 9)]])                              # interval inside gap (4,9): blocks
    res, peak, arg, mn = O.eval_plans(tas, same_gap)
    sc, wo, wi = O.score_plans(tas, same_gap, res, peak, arg)
    assert arg[0] == 6 and sc[0].tolist() == [0, 0] and wo[0][0] == -1


def test_feasibility_boundaries():
    """x exactly fits / misses by one ns; swap-out must end before the peak step."""
    # tensor 0 (size 6 -> x = 6 ns at 1000 B/us): touches 0 and 5; tensor 1 peaks at step 3
    def run(step_ns):
        tas = tas_from_lists(6, [6, 1], [0, 3], [[5], [4]], step_ns=step_ns, link_bytes_per_us=1000)
        pl = plans_from_lists([[]])
        res, peak, arg, mn = O.eval_plans(tas, pl)
        assert arg[0] == 3
        sc, wo, wi = O.score_plans(tas, pl, res, peak, arg)
        return int(sc[0][0]), int(wo[0][0]), int(wi[0][0])
    # steps 1,2 give 6 ns -> o = 2 < 3; swap-in needs C[5]-C[3] = 6 >= 6
    assert run([1, 3, 3, 3, 3, 1]) == (1, 2, 5)    # score 1: the peak moves to 6 at the plateau's edge
    # swap-out needs steps 1..3 -> o = 3 == tstar: infeasible
    assert run([1, 3, 2, 3, 3, 1]) == (0, -1, -1)
    # swap-in one ns short: C[o+1] + x > C[r]
    assert run([1, 3, 3, 3, 2, 1]) == (0, -1, -1)
