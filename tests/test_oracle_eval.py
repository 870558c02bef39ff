"""Pins of the oracle's footprint evaluation (Eq. 1, Eq. 2, Alg. 1 of the paper)
against things other than itself."""
import os

import numpy as np
import pytest

from oracle import oracle as O
from workloads import (CONFIGS, make_config_plans, make_plans, plans_from_lists, small_random_tas, tas_from_lists)
from workloads.plans import Plans

from helpers import membership_footprint, parse_fixture_lines

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _hand():
    rows = parse_fixture_lines(os.path.join(GOLDEN, "hand_example.txt"))
    tens = [r for r in rows if r[0] == "tensor"]
    tas = tas_from_lists(6, [int(r[2]) for r in tens], [int(r[3]) for r in tens], [[int(v) for v in r[4:]] for r in tens])
    get = lambda key: [int(v) for v in next(r for r in rows if r[0] == key)[1:]]
    return tas, get


def test_hand_example():
    tas, get = _hand()
    assert O.base_timeline(tas).tolist() == get("mf0")
    pl = plans_from_lists([[], [(0, 1, 5)]])
    res, peak, arg, mn = O.eval_plans(tas, pl)
    assert res[0].tolist() == get("mf0") and [peak[0], arg[0]] == get("peak0")
    assert res[1].tolist() == get("mf") and [peak[1], arg[1]] == get("peak") and [mn[1]] == get("min")


def test_five_situations():
    rows = parse_fixture_lines(os.path.join(GOLDEN, "five_situations.txt"))
    cases, cur = [], None
    for r in rows:
        if r[0] == "case":
            cur = dict(name=r[1], tensors=[], intervals=[])
            cases.append(cur)
        elif r[0] in ("T", "base"):
            cur[r[0]] = int(r[1])
        elif r[0] == "tensor":
            cur["tensors"].append([int(v) for v in r[1:]])
        elif r[0] == "interval":
            cur["intervals"].append(tuple(int(v) for v in r[1:]))
        elif r[0] == "mf":
            cur["mf"] = [int(v) for v in r[1:]]
    assert len(cases) == 5
    for c in cases:
        tas = tas_from_lists(c["T"], [t[0] for t in c["tensors"]], [t[1] for t in c["tensors"]],
                             [t[2:] for t in c["tensors"]], base_bytes=c["base"])
        res, peak, arg, mn = O.eval_plans(tas, plans_from_lists([c["intervals"]]))
        assert res[0].tolist() == c["mf"], c["name"]
        assert peak[0] == max(c["mf"]) and arg[0] == c["mf"].index(max(c["mf"])) and mn[0] == min(c["mf"])


@pytest.mark.parametrize("seed", range(6))
def test_literal_membership_sum(seed):
    """Brute-force membership evaluation of every (tensor, step) pair on tiny inputs."""
    tas = small_random_tas(100 + seed, N=14, T=37, base_bytes=seed * 11)
    pl = make_plans(tas, 9, seed, p_swap=0.6)
    res, peak, arg, mn = O.eval_plans(tas, pl)
    assert np.array_equal(O.base_timeline(tas), membership_footprint(tas, []))
    for b in range(pl.B):
        t, o, r, k = pl.plan(b)
        want = membership_footprint(tas, list(zip(t.tolist(), o.tolist(), r.tolist())))
        assert np.array_equal(res[b], want)
        assert peak[b] == want.max() and arg[b] == int(np.argmax(want)) and mn[b] == want.min()


def test_staircase_closed_form():
    """N tensors of size s, tensor i generated at step i, all read at the last step:
    MF[t] = (min(t, N-1) + 1) * s."""
    N, T, s = 9, 15, 1000
    tas = tas_from_lists(T, [s] * N, list(range(N)), [[T - 1]] * N)
    t = np.arange(T)
    assert np.array_equal(O.base_timeline(tas), (np.minimum(t, N - 1) + 1) * s)
    res, peak, arg, mn = O.eval_plans(tas, plans_from_lists([[]]))
    assert peak[0] == N * s and arg[0] == N - 1 and mn[0] == s      # earliest step of the plateau
    # evict tensor 0 over (0, T-1): every interior step drops by s
    res, peak, arg, mn = O.eval_plans(tas, plans_from_lists([[(0, 0, T - 1)]]))
    want = (np.minimum(t, N - 1) + 1) * s - s * ((t > 0) & (t < T - 1))
    assert np.array_equal(res[0], want) and peak[0] == N * s and arg[0] == T - 1


@pytest.mark.parametrize("idx", [0, 1])
def test_difference_array_vs_numpy_cumsum(idx, configs_small):
    """MF - MF0 is the inclusive prefix sum of the plan's difference array."""
    tas = configs_small[idx]
    pl = make_config_plans(idx, tas, B=6)
    res, *_ = O.eval_plans(tas, pl)
    MF0 = O.base_timeline(tas)
    for b in range(pl.B):
        t, o, r, _ = pl.plan(b)
        D = np.zeros(tas.T + 1, dtype=np.int64)
        np.subtract.at(D, o + 1, tas.size_bytes[t])
        np.add.at(D, r, tas.size_bytes[t])
        assert np.array_equal(res[b] - MF0, np.cumsum(D)[:tas.T])


@pytest.mark.parametrize("idx", [0, 1, 2])
def test_invariants(idx, configs_small):
    tas = configs_small[idx]
    pl = make_config_plans(idx, tas, B=16)
    res, peak, arg, mn = O.eval_plans(tas, pl)
    MF0 = O.base_timeline(tas)
    assert np.all(res >= 0) and np.all(mn >= 0)                       # never negative
    assert np.all(res <= MF0[None, :]) and np.all(peak <= MF0.max())   # scheduling never adds bytes
    assert np.array_equal(res[:, -1], np.full(pl.B, MF0[-1]))          # bytes conserved: all swapped back
    assert np.array_equal(arg, np.argmax(res, axis=1)) and np.array_equal(peak, res.max(axis=1))
    assert np.array_equal(mn, res.min(axis=1))
    for b in range(4):                                                 # unchanged outside every window
        t, o, r, _ = pl.plan(b)
        covered = np.zeros(tas.T, dtype=bool)
        for oo, rr in zip(o, r):
            covered[oo + 1:rr] = True
        assert np.array_equal(res[b][~covered], MF0[~covered])
    # peak-only mode agrees with the full mode
    _, p2, a2, m2 = O.eval_plans(tas, pl, want_resident=False)
    assert np.array_equal(p2, peak) and np.array_equal(a2, arg) and np.array_equal(m2, mn)


def test_empty_plan_is_base_timeline(configs_small):
    tas = configs_small[1]
    res, peak, arg, mn = O.eval_plans(tas, plans_from_lists([[], []]))
    MF0 = O.base_timeline(tas)
    assert np.array_equal(res[0], MF0) and np.array_equal(res[1], MF0)
    assert peak[0] == MF0.max() and arg[0] == int(np.argmax(MF0))


def test_order_and_duplicates_do_not_matter(configs_small):
    tas = configs_small[1]
    pl = make_config_plans(1, tas, B=2)
    t, o, r, k = pl.plan(0)
    perm = np.argsort(np.asarray([(int(v) * 2654435761) % 1000003 for v in range(len(t))]))
    shuffled = plans_from_lists([list(zip(t[perm].tolist(), o[perm].tolist(), r[perm].tolist())),
                                 list(zip(t.tolist(), o.tolist(), r.tolist())),
                                 list(zip(t.tolist(), o.tolist(), r.tolist()))])
    res, peak, arg, mn = O.eval_plans(tas, shuffled)
    assert np.array_equal(res[0], res[1]) and np.array_equal(res[1], res[2])
    assert peak[0] == peak[1] == peak[2] and arg[0] == arg[1] == arg[2]


def test_inapplicable_intervals_are_skipped_and_offsets_clamped():
    tas = tas_from_lists(8, [5, 7], [0, 1], [[6], [7]])
    good = [(0, 1, 5, 0)]
    bad = [(2, 1, 5, 0), (-1, 1, 5, 0), (0, -1, 5, 0), (0, 1, 9, 0), (0, 5, 5, 0), (0, 5, 3, 0)]
    a, *_ = O.eval_plans(tas, plans_from_lists([good]))
    b, *_ = O.eval_plans(tas, plans_from_lists([good + bad]))
    assert np.array_equal(a, b)
    # r == o + 1 is an empty window; r == T drops the '+' (nothing comes back inside the horizon)
    c, *_ = O.eval_plans(tas, plans_from_lists([[(0, 2, 3, 0)], [(1, 3, 8, 0)]]))
    assert np.array_equal(c[0], O.base_timeline(tas))
    assert c[1].tolist() == [5, 12, 12, 12, 5, 5, 5, 0]
    pl = plans_from_lists([good, good])
    pl = Plans(2, np.array([-5, 1, 99], dtype=np.int64), pl.iv_tensor, pl.iv_out, pl.iv_in, pl.iv_kind)
    d, *_ = O.eval_plans(tas, pl)
    assert np.array_equal(d[0], a[0]) and np.array_equal(d[1], a[0])


def test_times():
    tas = tas_from_lists(4, [64000, 1, 64001], [0, 0, 0], [[3], [3], [3]], step_ns=[5, 6, 7, 8], link_bytes_per_us=64000)
    C, x = O.times(tas)
    assert C.tolist() == [0, 5, 11, 18, 26] and x.tolist() == [1000, 1, 1001]
    tas.step_ns = None
    C, x = O.times(tas)
    assert not C.any() and not x.any()
