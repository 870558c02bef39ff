"""Pins of the oracle's link-occupancy timeline (section IV-C of the paper: transfers use the PCIe
channel exclusively, one tensor at a time; section III-C: the host copy stays until the tensor's last
access, so a repeated swap-out costs no transfer)."""
import numpy as np
import pytest

from oracle import oracle as O
from workloads import make_plans, plans_from_lists, small_random_tas, tas_from_lists
from workloads.plans import Plans


def _merge(a: Plans, b: Plans) -> Plans:
    """Plan by plan, the intervals of a followed by those of b (tensors may then repeat inside a plan)."""
    lists = []
    for p in range(a.B):
        cur = []
        for pl in (a, b):
            t, o, r, k = pl.plan(p)
            cur += [(int(t[j]), int(o[j]), int(r[j]), int(k[j])) for j in range(len(t))]
        lists.append(cur)
    return plans_from_lists(lists)


def _membership(tas, pl, reuse):
    """Continuous-time statement, step by step: a transfer that ends at time e and lasts x occupies
    step t iff the step ends after the transfer starts, C[t+1] > e - x, and is not later than its last step."""
    C = np.concatenate(([0], np.cumsum(tas.step_ns))).astype(np.int64)
    x = -((-tas.size_bytes * 1000) // tas.link_bytes_per_us)
    t_ax = np.arange(tas.T)
    out = np.zeros((pl.B, tas.T), dtype=np.int64)
    for b in range(pl.B):
        t, o, r, k = pl.plan(b)
        ok = (t >= 0) & (t < tas.N) & (o >= 0) & (r <= tas.T) & (r > o) & (k == 0)
        t, o, r = t[ok].astype(np.int64), o[ok].astype(np.int64), r[ok].astype(np.int64)
        charged = np.ones(len(t), dtype=bool)
        if reuse:
            for j in range(len(t)):
                charged[j] = o[j] == o[t == t[j]].min()
        for j in range(len(t)):
            xi = x[t[j]]
            if charged[j]:
                out[b] += (t_ax <= o[j]) & (C[t_ax + 1] > C[o[j] + 1] - xi)
            out[b] += (t_ax <= r[j] - 1) & (C[t_ax + 1] > C[r[j]] - xi)
    return out


def test_hand_worked_uniform_steps():
    # 8 steps of 10 ns; 1000 bytes/us = 1 byte/ns, so x = size in ns
    tas = tas_from_lists(8, [25, 10], [0, 0], [[7], [5]], step_ns=[10] * 8, link_bytes_per_us=1000)
    one = plans_from_lists([[(0, 3, 7, 0)]])
    rows, pk, arg, over = O.link_occupancy(tas, one)
    # out ends with step 3 (t=40): 25 ns back is t=15, inside step 1 -> steps 1..3; in ends at t=70: from t=45 -> steps 4..6
    assert rows[0].tolist() == [0, 1, 1, 1, 1, 1, 1, 0]
    assert (pk[0], arg[0], over[0]) == (1, 1, 0)
    two = plans_from_lists([[(0, 3, 7, 0), (1, 2, 5, 0)]])
    rows, pk, arg, over = O.link_occupancy(tas, two)
    # tensor 1 (10 ns): out = step 2 alone, in = step 4 alone
    assert rows[0].tolist() == [0, 1, 2, 1, 2, 1, 1, 0]
    assert (pk[0], arg[0], over[0]) == (2, 2, 2)
    # a recomputation interval uses no link
    rec = plans_from_lists([[(0, 3, 7, 1), (1, 2, 5, 0)]])
    rows, pk, _, over = O.link_occupancy(tas, rec)
    assert rows[0].tolist() == [0, 0, 1, 0, 1, 0, 0, 0] and pk[0] == 1 and over[0] == 0


def test_hand_worked_ragged_steps_and_a_transfer_longer_than_the_past():
    ns = [5, 20, 1, 1, 30, 2, 7, 4]          # C = 0 5 25 26 27 57 59 66 70
    tas = tas_from_lists(8, [22], [0], [[7]], step_ns=ns, link_bytes_per_us=1000)
    rows, pk, arg, over = O.link_occupancy(tas, plans_from_lists([[(0, 3, 7, 0)]]))
    # out ends at C[4]=27, starts at 5 = C[1] exactly -> steps 1..3; in ends at C[7]=66, starts at 44, inside step 4 -> 4..6
    assert rows[0].tolist() == [0, 1, 1, 1, 1, 1, 1, 0]
    # the swap-out would have to start before time 0: it occupies everything from step 0 (and o = 0 is one step)
    rows, _, _, _ = O.link_occupancy(tas, plans_from_lists([[(0, 0, 7, 0)]]))
    assert rows[0].tolist() == [1, 0, 0, 0, 1, 1, 1, 0]
    # a window shorter than the two transfers: they overlap and the steps in the middle are booked twice
    rows, pk, arg, over = O.link_occupancy(tas, plans_from_lists([[(0, 4, 6, 0)]]))
    # out: ends C[5]=57, from 35 (inside step 4) -> step 4; in: ends C[6]=59, from 37 (inside step 4) -> steps 4..5
    assert rows[0].tolist() == [0, 0, 0, 0, 2, 1, 0, 0] and (pk[0], arg[0], over[0]) == (2, 4, 1)


@pytest.mark.parametrize("seed,reuse", [(1, False), (2, True), (3, False), (4, True)])
def test_against_the_continuous_time_statement(seed, reuse):
    tas = small_random_tas(700 + seed, N=40, T=120, max_acc=5, timed=True)
    pl = _merge(make_plans(tas, 6, seed, p_swap=0.5), make_plans(tas, 6, seed + 100, p_swap=0.5))
    rows, pk, arg, over = O.link_occupancy(tas, pl, reuse=reuse)
    want = _membership(tas, pl, reuse)
    assert np.array_equal(rows, want)
    assert np.array_equal(pk, want.max(axis=1)) and np.array_equal(arg, want.argmax(axis=1))
    assert np.array_equal(over, (want >= 2).sum(axis=1))
    _, pk2, arg2, over2 = O.link_occupancy(tas, pl, reuse=reuse, want_rows=False)
    assert np.array_equal(pk, pk2) and np.array_equal(arg, arg2) and np.array_equal(over, over2)


def test_host_copy_reuse_only_drops_repeated_swap_outs():
    tas = small_random_tas(710, N=30, T=100, max_acc=6, timed=True)
    single = make_plans(tas, 8, 5, p_swap=0.6)                 # at most one interval per tensor and plan
    a, *_ = O.link_occupancy(tas, single, reuse=False)
    b, *_ = O.link_occupancy(tas, single, reuse=True)
    assert np.array_equal(a, b)
    twice = _merge(single, make_plans(tas, 8, 6, p_swap=0.6))
    a, *_ = O.link_occupancy(tas, twice, reuse=False)
    b, *_ = O.link_occupancy(tas, twice, reuse=True)
    assert np.all(b <= a) and np.any(b < a)
    # the same swap listed twice: without reuse both copies are charged, with reuse both are "the earliest"
    tas2 = tas_from_lists(8, [25], [0], [[7]], step_ns=[10] * 8, link_bytes_per_us=1000)
    dup = plans_from_lists([[(0, 3, 7, 0), (0, 3, 7, 0)], [(0, 1, 4, 0), (0, 5, 7, 0)]])
    a, *_ = O.link_occupancy(tas2, dup, reuse=False)
    b, *_ = O.link_occupancy(tas2, dup, reuse=True)
    assert a[0].tolist() == [0, 2, 2, 2, 2, 2, 2, 0] and np.array_equal(a[0], b[0])
    # second plan: out 0..1 (C[2]=20, from -5 -> step 0), in 1..3 (C[4]=40 from 15); second out 3..5, in 4..6
    assert a[1].tolist() == [1, 2, 1, 2, 2, 2, 1, 0]
    assert b[1].tolist() == [1, 2, 1, 1, 1, 1, 1, 0]


def test_no_latencies_no_occupancy_and_a_faster_link_occupies_less():
    tas = small_random_tas(720, N=30, T=80, max_acc=4, timed=False)
    pl = make_plans(tas, 5, 7, p_swap=0.5)
    rows, pk, arg, over = O.link_occupancy(tas, pl)
    assert not rows.any() and not pk.any() and not arg.any() and not over.any()
    tas = small_random_tas(721, N=30, T=80, max_acc=4, timed=True)
    slow, *_ = O.link_occupancy(tas, pl)
    tas.link_bytes_per_us *= 3
    fast, *_ = O.link_occupancy(tas, pl)
    assert np.all(fast <= slow) and np.any(fast < slow)
    # every transfer occupies at least its last step
    t, o, r, k = pl.plan(0)
    ok = (k == 0) & (r <= tas.T)
    assert np.all(fast[0][o[ok]] >= 1) and np.all(fast[0][r[ok] - 1] >= 1)


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_greedy_plans_never_book_the_link_twice(seed):
    """Alg. 2 places one transfer at a time; the canonical transfers of its plan lie inside the runs it
    reported, so the occupancy of a greedy plan never exceeds one."""
    tas = small_random_tas(730 + seed, N=150, T=240, max_acc=4, timed=True, link_bytes_per_us=200_000)
    g = O.greedy(tas, budget=0, min_iters=1 << 30)
    n = len(g["iv_tensor"])
    assert n > 3
    pl = plans_from_lists([[(int(g["iv_tensor"][k]), int(g["iv_out"][k]), int(g["iv_in"][k]), int(g["iv_kind"][k]))
                           for k in range(n)]])
    rows, pk, _, over = O.link_occupancy(tas, pl)
    assert pk[0] == 1 and over[0] == 0
    booked = np.zeros(tas.T, dtype=np.int64)
    for k in range(n):
        booked[g["xfer_out_start"][k]:g["iv_out"][k] + 1] += 1
        booked[g["xfer_in_start"][k]:g["iv_in"][k]] += 1
    assert booked.max() == 1 and np.all(rows[0] <= booked)
