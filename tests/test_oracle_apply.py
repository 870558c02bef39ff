"""Pins of the oracle's windowed update: one more interval per plan applied to existing footprint rows
(Alg. 3 of the paper runs the peak analysis again after every scheduled tensor; only the steps between
the new interval's endpoints change)."""
import numpy as np
import pytest

from oracle import oracle as O
from workloads import make_plans, plans_from_lists, small_random_tas, tas_from_lists
from workloads.plans import eligible_gaps


def _extended(pl, extra):
    lists = []
    for b in range(pl.B):
        t, o, r, k = pl.plan(b)
        lists.append([(int(t[j]), int(o[j]), int(r[j]), int(k[j])) for j in range(len(t))] + [extra[b]])
    return plans_from_lists(lists)


def test_hand_worked():
    # two tensors of 5 and 3 bytes, both alive during steps 0..5: the row is 8 everywhere
    tas = tas_from_lists(6, [5, 3], [0, 0], [[5], [5]])
    rows = np.full((3, 6), 8, dtype=np.int64)
    pk, arg, mn = O.apply_intervals(tas, [0, 1, 0], [1, 0, 3], [4, 5, 3], rows)
    assert rows[0].tolist() == [8, 8, 3, 3, 8, 8] and (pk[0], arg[0], mn[0]) == (8, 0, 3)
    assert rows[1].tolist() == [8, 5, 5, 5, 5, 8] and (pk[1], arg[1], mn[1]) == (8, 0, 5)
    assert rows[2].tolist() == [8] * 6 and (pk[2], arg[2], mn[2]) == (8, 0, 8)      # r <= o: not applied
    # the peak moves when the window covers it
    rows = np.array([[1, 9, 9, 2, 7, 7]], dtype=np.int64)
    pk, arg, mn = O.apply_intervals(tas, [0], [0], [3], rows)
    assert rows[0].tolist() == [1, 4, 4, 2, 7, 7] and (pk[0], arg[0], mn[0]) == (7, 4, 1)


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_equals_the_evaluation_of_the_extended_plan(seed):
    tas = small_random_tas(800 + seed, N=50, T=140, max_acc=5, timed=False, base_bytes=17)
    pl = make_plans(tas, 12, seed, p_swap=0.3)
    eoff, ep, eq = eligible_gaps(tas)
    rng = np.random.default_rng(seed)
    extra = []
    for b in range(pl.B):
        if b % 4 == 3:       # something that cannot be applied
            extra.append([(tas.N + 3, 2, 9, 0), (1, -1, 5, 0), (2, 7, 7, 0), (3, 5, tas.T + 1, 0)][(b // 4) % 4])
            continue
        g = int(rng.integers(0, len(ep)))
        i = int(np.searchsorted(eoff, g, side="right") - 1)
        o = int(rng.integers(ep[g], eq[g] - 1))
        r = int(rng.integers(o + 2, eq[g] + 1))
        extra.append((i, o, r, int(b % 2)))
    rows, p0, a0, m0 = O.eval_plans(tas, pl)
    before = rows.copy()
    pk, arg, mn = O.apply_intervals(tas, [e[0] for e in extra], [e[1] for e in extra], [e[2] for e in extra], rows)
    want, p1, a1, m1 = O.eval_plans(tas, _extended(pl, extra))
    assert np.array_equal(rows, want) and np.array_equal(pk, p1) and np.array_equal(arg, a1) and np.array_equal(mn, m1)
    for b in range(3, pl.B, 4):
        assert np.array_equal(rows[b], before[b]) and pk[b] == p0[b] and arg[b] == a0[b] and mn[b] == m0[b]


def test_a_chain_of_updates_is_the_whole_plan():
    """Starting from the unscheduled timeline and applying a plan's intervals one by one gives that plan's rows."""
    tas = small_random_tas(810, N=40, T=100, max_acc=4, timed=False)
    pl = make_plans(tas, 1, 4, p_swap=0.6)
    t, o, r, _ = pl.plan(0)
    row = O.base_timeline(tas)[None, :].copy()
    for j in range(len(t)):
        pk, arg, mn = O.apply_intervals(tas, [t[j]], [o[j]], [r[j]], row)
    want, p1, a1, m1 = O.eval_plans(tas, pl)
    assert len(t) > 5 and np.array_equal(row, want) and pk[0] == p1[0] and arg[0] == a1[0] and mn[0] == m1[0]
