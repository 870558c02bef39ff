"""Independent numpy statements of the definitions, used to pin the oracle.

These deliberately use different primitives from the oracle's C loops
(broadcast membership tests, ``numpy.cumsum``, ``searchsorted``, slice maxima)
so that a slip in either shows up as a disagreement.
"""
from __future__ import annotations

import numpy as np


def membership_footprint(tas, intervals):
    """MF[t] = base + sum_i size_i * [alloc_i <= t <= free_i] * [no window of i has out < t < in],
    evaluated literally for every (tensor, step) pair."""
    T, N = tas.T, tas.N
    t = np.arange(T)[None, :]
    alive = (tas.alloc_step[:, None] <= t) & (t <= tas.free_step[:, None])
    for (i, o, r, *_k) in intervals:
        if not (0 <= i < N and o >= 0 and r <= T and r > o):
            continue
        alive[i] &= ~((o < t[0]) & (t[0] < r))
    # a tensor hit by two overlapping windows would be subtracted twice by the
    # difference-array form; the membership form is only used with disjoint windows
    return tas.base_bytes + (alive * tas.size_bytes[:, None]).sum(axis=0)


def parse_fixture_lines(path):
    rows = []
    with open(path) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                rows.append(line.split())
    return rows


def touch_points(tas, i):
    a, b = int(tas.access_offsets[i]), int(tas.access_offsets[i + 1])
    return np.concatenate(([int(tas.alloc_step[i])], tas.access_steps[a:b].astype(np.int64)))


def numpy_scores(tas, plan, MF, P, tstar):
    """Scores and windows of one plan from the definition, with searchsorted for
    the gap and the earliest swap-out step and slice maxima for the peak outside
    the window.  plan = (iv_tensor, iv_out, iv_in)."""
    T, N = tas.T, tas.N
    if tas.step_ns is None:
        C = np.zeros(T + 1, dtype=np.int64)
        x = np.zeros(N, dtype=np.int64)
    else:
        C = np.concatenate(([0], np.cumsum(tas.step_ns)))
        x = -((-tas.size_bytes * 1000) // tas.link_bytes_per_us)
    score = np.zeros(N, dtype=np.int64); wo = np.full(N, -1, dtype=np.int32); wi = np.full(N, -1, dtype=np.int32)
    it, io, ir = plan
    for i in range(N):
        p = touch_points(tas, i)
        j = int(np.searchsorted(p, tstar, side="left"))      # first touch >= tstar
        if j == 0 or j == len(p) or p[j] == tstar:
            continue
        pg, pg1 = int(p[j - 1]), int(p[j])
        own = (it == i) & (io >= 0) & (ir <= T) & (ir > io)
        if np.any(own & (io >= pg) & (ir <= pg1)):
            continue
        # earliest o >= pg with C[o+1] >= C[pg+1] + x
        o = int(np.searchsorted(C[1:], C[pg + 1] + x[i], side="left"))
        o = max(o, pg)
        if o > T - 1:
            continue
        r = pg1
        if C[o + 1] + x[i] > C[r] or not (o < tstar < r):
            continue
        outside = max(int(MF[:o + 1].max()), int(MF[r:].max()))
        score[i] = P - max(outside, P - int(tas.size_bytes[i]))
        wo[i], wi[i] = o, r
    return score, wo, wi
