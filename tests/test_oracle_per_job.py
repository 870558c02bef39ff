"""Pins of the oracle's per-workload peaks (section III-A of the paper: MP_j is the
maximum of workload W_j's own footprint, and the global peak of asynchronously
running workloads is the sum of the MP_j)."""
import numpy as np
import pytest

from oracle import oracle as O
from workloads import make_config_plans, make_plans, plans_from_lists, prng, small_random_tas, tas_from_lists

from helpers import membership_footprint


def _job_view(tas, pl, j):
    """The sequence and the plans as workload j alone would see them: its tensors renumbered, no base bytes."""
    keep = np.nonzero(tas.job_id == j)[0]
    new_id = np.full(tas.N, -1, dtype=np.int64)
    new_id[keep] = np.arange(len(keep))
    accs = [tas.access_steps[tas.access_offsets[i]:tas.access_offsets[i + 1]].tolist() for i in keep]
    sub = tas_from_lists(tas.T, tas.size_bytes[keep].tolist(), tas.alloc_step[keep].tolist(), accs)
    plans = []
    for b in range(pl.B):
        t, o, r, _ = pl.plan(b)
        ok = (t >= 0) & (t < tas.N)
        ok[ok] &= new_id[t[ok]] >= 0
        plans.append([(int(new_id[a]), int(bb), int(c)) for a, bb, c in zip(t[ok], o[ok], r[ok])])
    return sub, plans_from_lists(plans)


def _with_jobs(tas, seed, J):
    tas.job_id = prng.randint(seed, 9, np.arange(tas.N), 0, J - 1).astype(np.int32)
    tas.J = J
    return tas


@pytest.mark.parametrize("seed,J", [(1, 2), (2, 3), (3, 5)])
def test_each_job_alone(seed, J):
    """Job j's peak and peak step are what the (pinned) single-timeline evaluation gives for job j's tensors alone."""
    tas = _with_jobs(small_random_tas(600 + seed, N=60, T=90, max_acc=4, timed=False, base_bytes=1000), seed, J)
    pl = make_plans(tas, 10, seed, p_swap=0.3)
    jp, ja, total = O.eval_per_job(tas, pl)
    for j in range(J):
        sub, sub_pl = _job_view(tas, pl, j)
        if sub.N == 0:
            assert np.all(jp[j] == 0) and np.all(ja[j] == 0)
            continue
        _, p, a, _ = O.eval_plans(sub, sub_pl, want_resident=False)
        assert np.array_equal(jp[j], p) and np.array_equal(ja[j], a)
    assert np.array_equal(total, jp.sum(axis=0) + 1000)


def test_one_job_is_the_merged_timeline(configs_small):
    tas = configs_small[0]
    assert tas.J == 1
    pl = make_config_plans(0, tas, B=16)
    _, peak, arg, _ = O.eval_plans(tas, pl, want_resident=False)
    jp, ja, total = O.eval_per_job(tas, pl)
    assert np.array_equal(total, peak) and np.array_equal(ja[0], arg)


def test_sum_of_job_peaks_bounds_the_merged_peak():
    tas = _with_jobs(small_random_tas(777, N=200, T=300, max_acc=4, timed=False, base_bytes=12345), 5, 4)
    pl = make_plans(tas, 20, 3, p_swap=0.3)
    res, peak, arg, _ = O.eval_plans(tas, pl)
    jp, ja, total = O.eval_per_job(tas, pl)
    assert np.all(total >= peak) and np.any(total > peak)
    # the job timelines add up to the merged one: at every job's own peak step the merged footprint
    # is at least that job's peak plus the base bytes
    for b in range(pl.B):
        for j in range(4):
            assert res[b][ja[j][b]] >= jp[j][b] + tas.base_bytes
    # literal membership sums per job on one plan
    for j in range(4):
        sub, sub_pl = _job_view(tas, pl, j)
        t, o, r, _ = sub_pl.plan(7)
        mf = membership_footprint(sub, list(zip(t.tolist(), o.tolist(), r.tolist())))
        assert mf.max() == jp[j][7] and int(np.argmax(mf)) == ja[j][7]


def test_hand_example_two_jobs():
    # job 0: A (size 4, steps 0..3), B (size 2, steps 1..2)       -> own timeline 4 6 6 4 0 0 0 0, peak 6 at step 1
    # job 1: C (size 5, steps 4..7), D (size 3, steps 5..6)       -> own timeline 0 0 0 0 5 8 8 5, peak 8 at step 5
    tas = tas_from_lists(8, [4, 2, 5, 3], [0, 1, 4, 5], [[3], [2], [7], [6]], jobs=[0, 0, 1, 1], base_bytes=10)
    pl = plans_from_lists([[], [(2, 4, 7)], [(0, 0, 3), (2, 4, 7)]])
    jp, ja, total = O.eval_per_job(tas, pl)
    assert jp.tolist() == [[6, 6, 4], [8, 5, 5]]         # evicting C over 5..6 leaves 5 (step 4), then D: 3 -> 5 at step 4
    assert ja.tolist() == [[1, 1, 0], [5, 4, 4]]
    assert total.tolist() == [24, 21, 19]
    _, peak, _, _ = O.eval_plans(tas, pl, want_resident=False)
    assert peak.tolist() == [18, 16, 15]                 # the jobs do not overlap in time: merged peak = base + the larger of the two
