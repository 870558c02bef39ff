"""HIP path vs the CPU oracle, bit-exact (all quantities are integers), through
the C ABI.  Small cases compare every element; the full-size configurations run
in the launch configuration the benchmark times and compare sampled plans row
by row plus the per-plan reductions."""
import os
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("needs a GPU", allow_module_level=True)

import paper_2105_13336_amd as P  # noqa: E402
from oracle import oracle as O  # noqa: E402
from workloads import (CONFIGS, make_config_plans, make_plans, make_tas, plans_from_lists, small_random_tas,  # noqa: E402
                       tas_from_lists)
from workloads import prng  # noqa: E402
from workloads.plans import Plans, eligible_gaps  # noqa: E402


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def upload(pl: Plans) -> P.DevicePlans:
    return P.DevicePlans.from_numpy(pl.plan_offsets, pl.iv_tensor, pl.iv_out, pl.iv_in, pl.iv_kind)


def gpu_eval(h, dp, want_resident=True, want_min=True):
    B = dp.B
    res = torch.empty((B, h.T), dtype=torch.int64, device="cuda") if want_resident else None
    peak = torch.empty(B, dtype=torch.int64, device="cuda")
    arg = torch.empty(B, dtype=torch.int32, device="cuda")
    mn = torch.empty(B, dtype=torch.int64, device="cuda") if want_min else None
    P.tensile_eval_plans(h, dp, res, peak, arg, mn)
    torch.cuda.synchronize()
    return res, peak, arg, mn


def gpu_score(h, dp, res, peak, arg):
    B, N = dp.B, h.N
    sc = torch.empty((B, N), dtype=torch.int64, device="cuda")
    wo = torch.empty((B, N), dtype=torch.int32, device="cuda")
    wi = torch.empty((B, N), dtype=torch.int32, device="cuda")
    P.tensile_score_candidates(h, dp, res, peak, arg, sc, wo, wi)
    torch.cuda.synchronize()
    return sc, wo, wi


def check_eval(tas, pl, h=None, rows=None, label=""):
    """Full comparison of the batch ``pl`` (or of the plan rows ``rows`` of it)."""
    own = h is None
    h = h or P.tas_load(tas)
    res, peak, arg, mn = gpu_eval(h, upload(pl))
    sel = pl if rows is None else pl.select(rows)
    r0, p0, a0, m0 = O.eval_plans(tas, sel)
    idx = slice(None) if rows is None else torch.as_tensor(np.asarray(rows), device="cuda")
    assert np.array_equal(peak[idx].cpu().numpy(), p0), label + " peak"
    assert np.array_equal(arg[idx].cpu().numpy(), a0), label + " argmax"
    assert np.array_equal(mn[idx].cpu().numpy(), m0), label + " min"
    assert np.array_equal(res[idx].cpu().numpy(), r0), label + " resident"
    if own:
        h.close()
    return res, peak, arg, mn


# ------------------------------------------------------------------ tas_load

@pytest.mark.parametrize("idx", [0, 1, 2])
def test_tas_load_tables(idx, configs_small):
    tas = configs_small[idx]
    say(f"tas_load config {idx}")
    h = P.tas_load(tas)
    MF0 = O.base_timeline(tas)
    assert np.array_equal(P.tensile_tas_base_timeline(h), MF0)
    assert P.tensile_tas_info(h) == (int(MF0.max()), int(np.argmax(MF0)))
    h.close()


def test_tas_load_base_bytes_and_many_tiles():
    tas = small_random_tas(11, N=300, T=20011, max_acc=3, base_bytes=12345)
    say("tas_load T=20011")
    h = P.tas_load(tas)
    assert np.array_equal(P.tensile_tas_base_timeline(h), O.base_timeline(tas))
    h.close()


# ---------------------------------------------------------------------- eval

@pytest.mark.parametrize("idx,B", [(0, None), (1, 512), (2, 96)])
def test_eval_elementwise(idx, B, configs_small):
    tas = configs_small[idx]
    pl = make_config_plans(idx, tas, B=B)
    say(f"eval config {idx} B={pl.B} K={pl.n_intervals}")
    check_eval(tas, pl, label=f"c{idx}")


@pytest.mark.parametrize("T,B,segs", [(1, 3, 0), (2, 2, 0), (7, 5, 0), (4095, 4, 0), (4096, 4, 0), (4097, 4, 0),
                                      (12289, 9, 0), (12291, 2, 0), (20011, 3, 3), (20011, 17, 2), (50001, 2, 0)])
def test_eval_shapes_and_segments(T, B, segs, tuning):
    """Odd and even T (8- and 16-byte stores), ragged tails, one tile, tile edges, several
    tiles per segment and several segments per plan (finalize kernel)."""
    if segs:
        tuning("eval_segments", segs)
    N = max(1, min(400, T // 2))
    tas = small_random_tas(1000 + T, N=N, T=T, max_acc=4 if T > 8 else 1, base_bytes=7)
    pl = make_plans(tas, B, 5, p_swap=0.7)
    say(f"eval T={T} B={B} segs={segs} K={pl.n_intervals}")
    check_eval(tas, pl, label=f"T={T}")


@pytest.mark.parametrize("threads,binned,T,segs", [(512, 0, 20011, 0), (1024, 0, 4097, 0), (512, 1, 12291, 0),
                                                    (1024, 1, 20011, 2), (512, 1, 7, 0), (1024, 1, 50001, 3),
                                                    (256, 0, 20011, 0), (256, 0, 4097, 2), (256, 0, 2048, 0), (256, 0, 7, 0),
                                                    (256, 0, 12291, 4),
                                                    # binned rows of 4 ... 10 tiles: the tile loop takes groups of four
                                                    # and then the rest, so every remainder, with and without a group
                                                    (1024, 1, 24581, 0), (1024, 1, 32868, 0), (1024, 1, 40961, 0),
                                                    (1024, 1, 57347, 0), (1024, 1, 65545, 0), (1024, 1, 73730, 0),
                                                    (512, 1, 40962, 0), (512, 1, 36865, 2)])
def test_eval_geometries_and_binning(threads, binned, T, segs, tuning):
    """The workgroup geometries on rows they would not get by default, and the binned path (endpoints
    sorted by tile first) on short and ragged rows, with and without several segments per plan."""
    tuning("eval_threads", threads)
    tuning("eval_binned", binned)
    if segs:
        tuning("eval_segments", segs)
    N = max(1, min(400, T // 2))
    tas = small_random_tas(2000 + T, N=N, T=T, max_acc=4 if T > 8 else 1, base_bytes=11)
    pl = make_plans(tas, 6, 7, p_swap=0.7)
    say(f"eval threads={threads} binned={binned} T={T} segs={segs}")
    check_eval(tas, pl, label=f"threads={threads} binned={binned}")


@pytest.mark.parametrize("threads,binned,persistent,most,T", [(1024, 0, 0, 9000, 50001), (512, 0, 0, 5000, 20011),
                                                               (1024, 1, 0, 17000, 50001), (1024, 0, 1, 30000, 29999),
                                                               (256, 0, 0, 2048, 12291)])
def test_eval_rows_cut_by_the_segment_limit(threads, binned, persistent, most, T, tuning):
    """The kernels keep endpoints as 32-bit byte offsets into a segment's cells, so the host cuts rows into segments of
    at most 2^28 steps whatever else it chose; here the limit is lowered (tuning knob) so that the rule, and endpoints
    before, inside, at the edge of and after a segment, are exercised on rows a test can hold.  Where a persistent
    grid is asked for, the cut wins (that grid takes whole rows only)."""
    tuning("eval_threads", threads)
    tuning("eval_binned", binned)
    tuning("eval_persistent", persistent)
    tuning("eval_seg_steps", most)
    tas = small_random_tas(2300 + T, N=min(400, T // 2), T=T, max_acc=4, base_bytes=17)
    pl = make_plans(tas, 7, 11, p_swap=0.7)
    say(f"eval segment limit: threads={threads} binned={binned} persistent={persistent} most={most} T={T}")
    check_eval(tas, pl, label=f"segment limit {most}")


@pytest.mark.parametrize("threads,T,segs", [(512, 4097, 0), (1024, 20011, 2), (1024, 8192, 0)])
def test_eval_binned_tiles_with_many_records(threads, T, segs, tuning):
    """The binned path takes a tile's records two per thread, requested ahead of the tile; plans with a tile that
    holds more go through its general form.  One batch with plans of both kinds, with empty plans, and with every
    endpoint of a plan in one tile."""
    tuning("eval_threads", threads)
    tuning("eval_binned", 1)
    if segs:
        tuning("eval_segments", segs)
    tas = small_random_tas(2100 + T, N=400, T=T, max_acc=4, base_bytes=5)
    base = make_plans(tas, 8, 9, p_swap=0.8)
    lists = []
    for b in range(8):
        t, o, r, k = base.plan(b)
        one = [(int(t[j]), int(o[j]), int(r[j]), int(k[j])) for j in range(len(t))]
        reps = (0, 1, 4, 9, 1, 20, 0, 3)[b]           # x 250-300 intervals: up to ~6000 intervals, 12000 records
        lists.append(one * reps)
    # all endpoints of one plan at two steps of the first tile
    lists.append([(0, int(tas.alloc_step[0]), int(tas.alloc_step[0]) + 2, 0)] * 3000)
    pl = plans_from_lists(lists)
    say(f"eval binned, crowded tiles: threads={threads} T={T} segs={segs} lengths={[len(x) for x in lists]}")
    check_eval(tas, pl, label=f"binned crowded threads={threads}")


@pytest.mark.parametrize("threads,binned,T,segs,r", [(1024, 0, 20012, 0, 0), (1024, 0, 8192, 0, 2), (1024, 0, 16390, 2, 8), (1024, 1, 20012, 0, 0),
                                                      (1024, 1, 50002, 3, 0), (512, 1, 12292, 0, 0), (512, 1, 20012, 2, 0)])
def test_eval_rows_written_with_nontemporal_stores(threads, binned, T, segs, r, tuning):
    """Long rows are written with nontemporal stores (a kernel variant of its own); forced here on rows of a few
    tiles: the common kernel with several register capacities and the tail kernel behind it (one plan is longer
    than the registers hold), several segments per plan, and the binned kernels in both geometries."""
    tuning("eval_nt", 1)
    tuning("eval_threads", threads)
    tuning("eval_binned", binned)
    if segs:
        tuning("eval_segments", segs)
    if r:
        tuning("eval_r", r)
    tas = small_random_tas(2300 + T, N=400, T=T, max_acc=4, base_bytes=3)
    base = make_plans(tas, 7, 11, p_swap=0.8)
    lists = []
    for b in range(7):
        t, o, rr, k = base.plan(b)
        one = [(int(t[j]), int(o[j]), int(rr[j]), int(k[j])) for j in range(len(t))]
        lists.append(one * (1, 0, 2, 1, 40, 1, 3)[b])      # (x 40: more than 8192 intervals, the tail kernel's plan)
    pl = plans_from_lists(lists)
    say(f"eval nontemporal rows: threads={threads} binned={binned} T={T} segs={segs} r={r} lengths={[len(x) for x in lists]}")
    check_eval(tas, pl, label=f"nontemporal threads={threads} binned={binned}")


def test_eval_long_rows_take_nontemporal_stores_by_default():
    """A row of more than 131,072 steps (its unscheduled timeline exceeds 1 MiB) with short plans: the default
    path, which writes such rows with nontemporal stores, against the oracle; ragged last tile."""
    T = 150_002
    tas = small_random_tas(2400, N=300, T=T, max_acc=4, base_bytes=9)
    pl = make_plans(tas, 5, 13, p_swap=0.7)
    say(f"eval long rows: T={T} K={pl.n_intervals}")
    check_eval(tas, pl, label="long rows")


@pytest.mark.parametrize("threads,T,B,slots,tail", [(1024, 20011, 23, 3, False), (512, 12291, 40, 7, False), (1024, 4097, 9, 2, False),
                                                     (512, 7, 33, 4, False), (1024, 8192, 12, 5, False), (512, 20012, 21, 2, True),
                                                     (1024, 50001, 11, 3, True), (512, 4096, 5, 8, False),
                                                     (1024, 16384, 10, 3, False), (1024, 8193, 14, 4, True), (512, 8191, 17, 3, False)])
def test_eval_persistent_grid(threads, T, B, slots, tail, tuning):
    """The persistent kernel (several plans per workgroup, the next plan's intervals requested during the
    current plan's first tile and their sizes during its last) with a grid forced small: ragged and whole last
    tiles, one, two and more tiles per row, plans without intervals in the middle and at the end of a workgroup's
    walk, more workgroups than plans, and (tail) plans too long for the registers, which it must leave to the
    tail kernel."""
    tuning("eval_threads", threads)
    tuning("eval_persistent", 1)
    tuning("eval_segments", 1)
    tuning("eval_slots", slots)
    N = max(1, min(400, T // 2))
    tas = small_random_tas(3000 + T, N=N, T=T, max_acc=4 if T > 8 else 1, base_bytes=13)
    base = make_plans(tas, B, 9, p_swap=0.7)
    lists = [[(int(base.iv_tensor[k]), int(base.iv_out[k]), int(base.iv_in[k]), int(base.iv_kind[k]))
              for k in range(int(base.plan_offsets[b]), int(base.plan_offsets[b + 1]))] for b in range(B)]
    for b in (1, B // 2, B - 1):
        lists[b] = []
    if tail:   # repeat a plan's intervals until they exceed the smallest register capacity (2048)
        for b in (0, B // 3, B - 2):
            if lists[b]:
                lists[b] = (lists[b] * (2100 // len(lists[b]) + 1))[:2100 + b]
    pl = plans_from_lists(lists)
    say(f"eval persistent threads={threads} T={T} B={B} slots={slots} tail={tail} K={pl.n_intervals}")
    check_eval(tas, pl, label=f"persistent threads={threads} T={T}")


def test_eval_smallest_geometry_with_long_plans(tuning):
    """256-thread workgroups hold 2048 intervals of a plan; longer plans of the batch go to the tail kernel,
    empty ones stay; rows and peaks-only; ragged and whole last tiles."""
    tuning("eval_threads", 256)
    for T in (6000, 4096, 2049):
        tas = small_random_tas(4100 + T, N=300, T=T, max_acc=4, base_bytes=5)
        B = 19
        base = make_plans(tas, B, 11, p_swap=0.7)
        lists = [[(int(base.iv_tensor[k]), int(base.iv_out[k]), int(base.iv_in[k]), int(base.iv_kind[k]))
                  for k in range(int(base.plan_offsets[b]), int(base.plan_offsets[b + 1]))] for b in range(B)]
        lists[1] = []
        lists[B - 1] = []
        for b in (0, 7, B - 2):
            lists[b] = (lists[b] * (2100 // len(lists[b]) + 1))[:2100 + 40 * b]
        pl = plans_from_lists(lists)
        say(f"eval 256 threads with long plans T={T} K={pl.n_intervals}")
        h = P.tas_load(tas)
        check_eval(tas, pl, h=h, label=f"256 threads T={T}")
        _, p0, a0, _ = O.eval_plans(tas, pl, want_resident=False)
        _, peak, arg, _ = gpu_eval(h, upload(pl), want_resident=False, want_min=False)
        assert np.array_equal(peak.cpu().numpy(), p0) and np.array_equal(arg.cpu().numpy(), a0)
        h.close()


def repeated(base, b, length):
    t, o, r, k = base.plan(b)
    one = [(int(t[j]), int(o[j]), int(r[j]), int(k[j])) for j in range(len(t))]
    return (one * (length // max(1, len(one)) + 1))[:length]


@pytest.mark.parametrize("T", [20012, 50001])
def test_eval_mixed_batch_of_short_and_long_plans(T):
    """A batch of short plans in which every seventh plan is long (7,000 to 20,000 intervals: beyond what the
    common kernel keeps in registers, and beyond the 8192 of the kernel that takes the long ones, which then reads the
    rest again per tile), under the library's own launch choices."""
    tas = small_random_tas(4500 + T, N=400, T=T, max_acc=5, base_bytes=3)
    B = 300
    base = make_plans(tas, B, 23, p_swap=0.7)
    lists = [repeated(base, b, 7000 + 331 * (b % 41)) if b % 7 == 3 else repeated(base, b, len(base.plan(b)[0]))
             for b in range(B)]
    pl = plans_from_lists(lists)
    lens = np.diff(pl.plan_offsets)
    say(f"eval mixed batch T={T}: {int((lens > 6144).sum())} of {B} plans longer than 6144 (longest {int(lens.max())})")
    assert (lens > 6144).sum() >= B // 10 and lens.max() > 8192
    check_eval(tas, pl, label=f"mixed T={T}")


def test_eval_batch_of_plans_that_just_fit_eight_per_thread():
    """Average plan between 6144 and 8192 intervals: the common kernel's largest register capacity, with a few
    plans beyond it."""
    tas = small_random_tas(4600, N=400, T=33001, max_acc=5, base_bytes=3)
    B = 40
    base = make_plans(tas, B, 29, p_swap=0.7)
    lists = [repeated(base, b, 6500 + 37 * b if b % 9 else 8192 + 5 * b) for b in range(B)]
    lists[7] = []
    pl = plans_from_lists(lists)
    say(f"eval plans of 6500-8400 intervals: average {pl.n_intervals // B}")
    check_eval(tas, pl, label="eight per thread")


# ---- seeded sweep over shapes and launch variants ----------------------------------------------

@pytest.mark.parametrize("case", range(30))
def test_random_shapes_and_variants(case, tuning):
    """Every entry point on a seeded random shape (row length, batch, density, odd/even T) under a random
    choice of the evaluator's launch variants (geometry, segments, binning, persistent grid)."""
    rng = np.random.default_rng(9000 + case)
    T = int(rng.choice([3, 17, 255, 256, 1000, 4095, 4097, 8190, 9001, 16385, 23456, 33333]))
    B = int(rng.integers(1, 24))
    N = max(1, min(int(rng.integers(1, 500)), T // 2))
    timed = bool(rng.integers(0, 2))
    threads = int(rng.choice([0, 512, 1024])) if case < 24 else 256
    segs = int(rng.choice([0, 0, 1, 2, 3]))
    binned = int(rng.choice([-1, -1, 0, 1]))
    pers = int(rng.choice([-1, 0, 1]))
    if threads:
        tuning("eval_threads", threads)
    if segs:
        tuning("eval_segments", segs)
    if binned >= 0:
        tuning("eval_binned", binned)
    if pers >= 0:
        tuning("eval_persistent", pers)
        tuning("eval_slots", int(rng.integers(1, 6)))
    tas = small_random_tas(9100 + case, N=N, T=T, max_acc=int(rng.integers(1, 7)) if T > 8 else 1, timed=timed,
                           base_bytes=int(rng.integers(0, 1000)))
    pl = merged_plans(tas, B, 50 + case, p_swap=float(rng.uniform(0.05, 0.95))) if T > 2 else plans_from_lists([[]] * B)
    say(f"sweep {case}: T={T} B={B} N={N} K={pl.n_intervals} timed={timed} threads={threads} segs={segs} binned={binned} persistent={pers}")
    h = P.tas_load(tas)
    dp = upload(pl)
    res, peak, arg, mn = gpu_eval(h, dp)
    r0, p0, a0, m0 = O.eval_plans(tas, pl)
    assert np.array_equal(res.cpu().numpy(), r0) and np.array_equal(peak.cpu().numpy(), p0)
    assert np.array_equal(arg.cpu().numpy(), a0) and np.array_equal(mn.cpu().numpy(), m0)
    _, peak2, arg2, _ = gpu_eval(h, dp, want_resident=False, want_min=False)
    assert torch.equal(peak, peak2) and torch.equal(arg, arg2)
    sc, wo, wi = gpu_score(h, dp, res, peak, arg)
    s0, o0, i0 = O.score_plans(tas, pl, r0, p0, a0)
    assert np.array_equal(sc.cpu().numpy(), s0) and np.array_equal(wo.cpu().numpy(), o0) and np.array_equal(wi.cpu().numpy(), i0)
    P.tensile_score_recompute(h, dp, res, peak, arg, sc, wo, wi)
    torch.cuda.synchronize()
    s1, o1, i1 = O.score_recompute_plans(tas, pl, r0, p0, a0)
    assert np.array_equal(sc.cpu().numpy(), s1) and np.array_equal(wo.cpu().numpy(), o1) and np.array_equal(wi.cpu().numpy(), i1)
    reuse = bool(rng.integers(0, 2))
    rows, lpk, larg, lover = gpu_link(h, dp, reuse)
    l0, lp0, la0, lo0 = O.link_occupancy(tas, pl, reuse=reuse)
    assert np.array_equal(rows.cpu().numpy(), l0) and np.array_equal(lpk.cpu().numpy(), lp0)
    assert np.array_equal(larg.cpu().numpy(), la0) and np.array_equal(lover.cpu().numpy(), lo0)
    if T > 2:
        t, o, r = extra_intervals(tas, B, 70 + case)
        P.tensile_apply_intervals(h, torch.from_numpy(t).cuda(), torch.from_numpy(o).cuda(), torch.from_numpy(r).cuda(), res, peak, arg, mn)
        torch.cuda.synchronize()
        p1, a1, m1 = O.apply_intervals(tas, t, o, r, r0)
        assert np.array_equal(res.cpu().numpy(), r0) and np.array_equal(peak.cpu().numpy(), p1)
        assert np.array_equal(arg.cpu().numpy(), a1) and np.array_equal(mn.cpu().numpy(), m1)
    h.close()


# ---- windowed update ------------------------------------------------------------------------

def extra_intervals(tas, B, seed):
    """One new interval per plan inside a random gap; every fifth one cannot be applied."""
    eoff, ep, eq = eligible_gaps(tas)
    rng = np.random.default_rng(seed)
    bad = [(tas.N + 3, 2, 9), (1, -1, 5), (2, 7, 7), (0, 5, tas.T + 1)]
    t, o, r = [], [], []
    for b in range(B):
        if b % 5 == 4 or len(ep) == 0:
            i, oo, rr = bad[(b // 5) % 4]
        else:
            g = int(rng.integers(0, len(ep)))
            i = int(np.searchsorted(eoff, g, side="right") - 1)
            oo = int(rng.integers(ep[g], eq[g] - 1))
            rr = int(rng.integers(oo + 2, eq[g] + 1))
        t.append(i); o.append(oo); r.append(rr)
    return np.array(t, dtype=np.int32), np.array(o, dtype=np.int32), np.array(r, dtype=np.int32)


@pytest.mark.parametrize("T,B", [(1, 2), (7, 6), (8191, 5), (8192, 5), (8193, 6), (20011, 7), (20012, 11), (300, 400)])
def test_apply_intervals(T, B):
    """One more interval per plan on rows that exist: odd and even T (8- and 16-byte accesses), one chunk,
    chunk edges, several chunks (finalize kernel), windows across chunk borders, inapplicable intervals."""
    N = max(1, min(300, T // 2))
    tas = small_random_tas(5000 + T, N=N, T=T, max_acc=5 if T > 8 else 1, timed=False, base_bytes=9)
    pl = make_plans(tas, B, 13, p_swap=0.4)
    say(f"apply T={T} B={B}")
    h = P.tas_load(tas)
    res, peak, arg, mn = gpu_eval(h, upload(pl))
    r0, _, _, _ = O.eval_plans(tas, pl)
    t, o, r = extra_intervals(tas, B, 7 + T)
    up = lambda a: torch.from_numpy(a).cuda()
    P.tensile_apply_intervals(h, up(t), up(o), up(r), res, peak, arg, mn)
    torch.cuda.synchronize()
    p1, a1, m1 = O.apply_intervals(tas, t, o, r, r0)
    assert np.array_equal(res.cpu().numpy(), r0) and np.array_equal(peak.cpu().numpy(), p1)
    assert np.array_equal(arg.cpu().numpy(), a1) and np.array_equal(mn.cpu().numpy(), m1)
    # the same as evaluating the extended plans from scratch
    lists = []
    for b in range(B):
        pt, po, pr, pk = pl.plan(b)
        lists.append([(int(pt[j]), int(po[j]), int(pr[j]), int(pk[j])) for j in range(len(pt))] + [(int(t[b]), int(o[b]), int(r[b]), 0)])
    res2, peak2, arg2, mn2 = gpu_eval(h, upload(plans_from_lists(lists)))
    assert torch.equal(res, res2) and torch.equal(peak, peak2) and torch.equal(arg, arg2) and torch.equal(mn, mn2)
    # without the optional minimum
    P.tensile_apply_intervals(h, up(np.full(B, -1, dtype=np.int32)), up(o), up(r), res, peak, arg, None)
    torch.cuda.synchronize()
    assert torch.equal(res, res2) and torch.equal(peak, peak2) and torch.equal(arg, arg2)
    h.close()


# ---- link occupancy -----------------------------------------------------------------------

def gpu_link(h, dp, reuse=False, want_rows=True, want_all=True):
    B = dp.B
    rows = torch.full((B, h.T), -7, dtype=torch.int32, device="cuda") if want_rows else None
    pk = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    arg = torch.full((B,), -7, dtype=torch.int32, device="cuda") if want_all else None
    over = torch.full((B,), -7, dtype=torch.int32, device="cuda") if want_all else None
    P.tensile_eval_link(h, dp, pk, rows, arg, over, reuse_host_copies=reuse)
    torch.cuda.synchronize()
    return rows, pk, arg, over


def check_link(tas, pl, reuse, h=None, label=""):
    own = h is None
    h = h or P.tas_load(tas)
    dp = upload(pl)
    rows, pk, arg, over = gpu_link(h, dp, reuse)
    r0, p0, a0, o0 = O.link_occupancy(tas, pl, reuse=reuse)
    assert np.array_equal(pk.cpu().numpy(), p0), label + " peak"
    assert np.array_equal(arg.cpu().numpy(), a0), label + " argmax"
    assert np.array_equal(over.cpu().numpy(), o0), label + " overbooked"
    assert np.array_equal(rows.cpu().numpy(), r0), label + " rows"
    # peaks only (no rows, no optional outputs)
    _, pk2, _, _ = gpu_link(h, dp, reuse, want_rows=False, want_all=False)
    assert np.array_equal(pk2.cpu().numpy(), p0), label + " peak without rows"
    if own:
        h.close()


def merged_plans(tas, B, seed, p_swap=0.5):
    """Two batches merged plan by plan: tensors repeat inside a plan (several swaps of one tensor)."""
    a, b = make_plans(tas, B, seed, p_swap=p_swap), make_plans(tas, B, seed + 1000, p_swap=p_swap)
    lists = []
    for p in range(B):
        cur = []
        for src in (a, b):
            t, o, r, k = src.plan(p)
            cur += [(int(t[j]), int(o[j]), int(r[j]), int(k[j])) for j in range(len(t))]
        lists.append(cur)
    return plans_from_lists(lists)


@pytest.mark.parametrize("T,B,reuse", [(1, 2, False), (7, 5, True), (8191, 3, False), (8192, 3, True), (8193, 4, False),
                                        (20011, 6, True), (20012, 5, False), (300, 700, True)])
def test_link_occupancy_shapes(T, B, reuse):
    """One tile, tile edges, ragged last tiles, odd and even T (8- and 16-byte aligned rows), several
    swaps of one tensor in a plan, recomputation intervals in between, and more plans than workgroups."""
    N = max(1, min(300, T // 2))
    tas = small_random_tas(4000 + T, N=N, T=T, max_acc=5 if T > 8 else 1, timed=True)
    pl = merged_plans(tas, B, 11) if T > 1 else plans_from_lists([[], []])
    say(f"link T={T} B={B} reuse={reuse} K={pl.n_intervals}")
    check_link(tas, pl, reuse, label=f"link T={T}")


@pytest.mark.parametrize("T,B,packed", [(32767, 3, 1), (32768, 3, 1), (32769, 4, 1), (50168, 3, 1), (50169, 3, 1), (65537, 3, 1),
                                         (120001, 2, 1), (32769, 3, 0), (120001, 2, 0)])
def test_link_occupancy_long_rows(T, B, packed, tuning):
    """Edges of the 32768-step tile, rows whose table of C covers every block of seven steps (up to 50,168
    steps) and rows where it skips blocks, with the packed differences of C and with the probe search."""
    tuning("link_packed", packed)
    tas = small_random_tas(4300 + T, N=200, T=T, max_acc=6, timed=True)
    pl = merged_plans(tas, B, 31, p_swap=0.8)
    say(f"link long rows T={T} B={B} packed={packed} K={pl.n_intervals}")
    check_link(tas, pl, bool(T & 1), label=f"link T={T} packed={packed}")


def test_link_occupancy_with_latencies_too_long_to_pack():
    """Operator latencies of 2^21 ns and more cannot be packed: the probe search runs, also after an update
    of the latencies of a loaded sequence switched the handle from one form to the other."""
    tas = small_random_tas(4400, N=120, T=9001, max_acc=5, timed=True)
    pl = merged_plans(tas, 5, 41, p_swap=0.7)
    h = P.tas_load(tas)
    check_link(tas, pl, False, h=h, label="link short latencies")
    slow = tas.step_ns * 3000                      # up to 3 ms per step
    assert slow.max() >= 1 << 21
    P.tensile_tas_update_latencies(h, slow, tas.link_bytes_per_us // 3000 + 1)
    tas.step_ns, tas.link_bytes_per_us = slow, tas.link_bytes_per_us // 3000 + 1
    say("link: latencies updated to >= 2^21 ns")
    check_link(tas, pl, True, h=h, label="link long latencies")
    fast = np.minimum(slow // 3000 + 1, (1 << 21) - 1)
    P.tensile_tas_update_latencies(h, fast, 50_000)
    tas.step_ns, tas.link_bytes_per_us = fast, 50_000
    say("link: latencies updated back")
    check_link(tas, pl, False, h=h, label="link short latencies again")
    # exactly at the limit of the packed form: 2^21 - 1 fits, 2^21 does not
    for top in ((1 << 21) - 1, 1 << 21):
        edge = fast.copy()
        edge[::97] = top
        P.tensile_tas_update_latencies(h, edge, 50_000)
        tas.step_ns = edge
        check_link(tas, pl, True, h=h, label=f"link latency {top}")
    h.close()


def test_link_occupancy_long_plans_take_several_passes():
    """Plans of more than 6144 intervals (the registers of one pass), with and without rows."""
    tas = small_random_tas(4100, N=400, T=9000, max_acc=6, timed=True)
    base = merged_plans(tas, 4, 21, p_swap=0.9)
    lists = []
    for b in range(4):
        t, o, r, k = base.plan(b)
        one = [(int(t[j]), int(o[j]), int(r[j]), int(k[j])) for j in range(len(t))]
        lists.append((one * (14000 // max(1, len(one)) + 1))[:6144 * b + 5 + 6140 * (b % 2)])
    pl = plans_from_lists(lists)
    say(f"link long plans: {[len(x) for x in lists]}")
    for reuse in (False, True):
        check_link(tas, pl, reuse, label=f"link long reuse={reuse}")


def test_link_occupancy_edge_cases(configs_small):
    # no latencies: nothing is occupied
    tas = small_random_tas(4200, N=50, T=100, max_acc=4, timed=False)
    pl = make_plans(tas, 5, 3, p_swap=0.5)
    check_link(tas, pl, False, label="link untimed")
    # kinds omitted: every interval is a swap; inapplicable intervals are skipped; B == 0
    tas = small_random_tas(4201, N=50, T=100, max_acc=4, timed=True)
    pl = plans_from_lists([[(0, 3, 9, 0), (70, 1, 5, 0), (1, -1, 5, 0), (2, 5, 101, 0), (3, 9, 9, 0), (4, 20, 100, 0)], []])
    h = P.tas_load(tas)
    dp = P.DevicePlans.from_numpy(pl.plan_offsets, pl.iv_tensor, pl.iv_out, pl.iv_in, None)
    rows, pk, arg, over = gpu_link(h, dp)
    r0, p0, a0, o0 = O.link_occupancy(tas, pl)
    assert np.array_equal(rows.cpu().numpy(), r0) and np.array_equal(pk.cpu().numpy(), p0)
    assert np.array_equal(arg.cpu().numpy(), a0) and np.array_equal(over.cpu().numpy(), o0)
    empty = upload(plans_from_lists([]))
    P.tensile_eval_link(h, empty, pk, None)
    h.close()
    # a workload-shaped sequence
    tas = configs_small[1]
    pl = make_config_plans(1, tas, B=24)
    check_link(tas, pl, True, label="link c1")


def test_link_of_a_greedy_plan_is_exclusive(configs_small):
    """The plan that tensile_greedy_plan builds never books the link twice."""
    tas = configs_small[1]
    h = P.tas_load(tas)
    g = P.tensile_greedy_plan(h, budget_bytes=0, max_iters=150, min_iters=1 << 30)
    n = len(g["iv_tensor"])
    assert n > 20
    offs = np.array([0, n], dtype=np.int64)
    dp = P.DevicePlans.from_numpy(offs, g["iv_tensor"], g["iv_out"], g["iv_in"], g["iv_kind"])
    rows, pk, arg, over = gpu_link(h, dp)
    assert int(pk[0]) == 1 and int(over[0]) == 0 and int(rows.max()) == 1
    h.close()


def test_eval_binned_config(configs_small, tuning):
    tuning("eval_binned", 1)
    tas = configs_small[2]
    pl = make_config_plans(2, tas, B=64)
    say("eval binned config 2")
    check_eval(tas, pl, rows=range(0, 64, 9), label="c2 binned")


def test_eval_optional_outputs_and_empty_batches(configs_small):
    tas = configs_small[1]
    h = P.tas_load(tas)
    pl = make_config_plans(1, tas, B=16)
    dp = upload(pl)
    say("eval optional outputs")
    _, p0, a0, m0 = O.eval_plans(tas, pl, want_resident=False)
    res, peak, arg, mn = gpu_eval(h, dp, want_resident=False, want_min=False)
    assert res is None and mn is None
    assert np.array_equal(peak.cpu().numpy(), p0) and np.array_equal(arg.cpu().numpy(), a0)
    # B == 0: nothing happens
    empty = upload(plans_from_lists([]))
    P.tensile_eval_plans(h, empty, None, peak, arg, None)
    # plans without any interval
    none = upload(plans_from_lists([[], [], []]))
    res, peak, arg, mn = gpu_eval(h, none)
    MF0 = O.base_timeline(tas)
    assert np.array_equal(res.cpu().numpy(), np.tile(MF0, (3, 1)))
    assert peak.tolist() == [int(MF0.max())] * 3 and arg.tolist() == [int(np.argmax(MF0))] * 3
    h.close()


@pytest.mark.parametrize("binned,segs", [(-1, 0), (1, 0), (1, 2)])
def test_eval_inapplicable_intervals_and_clamped_offsets(binned, segs, tuning):
    """Intervals that cannot be applied are skipped, offsets outside the arrays are clamped: on the default path and
    on the binned one, whose counting pass looks at the steps alone when the rows are not cut into segments (an
    interval with a tensor index out of range then gets records of size zero)."""
    tuning("eval_binned", binned)
    if segs:
        tuning("eval_segments", segs)
    tas = tas_from_lists(8, [5, 7], [0, 1], [[6], [7]])
    good = [(0, 1, 5, 0)]
    bad = [(2, 1, 5, 0), (-1, 1, 5, 0), (0, -1, 5, 0), (0, 1, 9, 0), (0, 5, 5, 0), (0, 5, 3, 0), (1, 3, 8, 0), (0, 2, 3, 0)]
    pl = plans_from_lists([good, good + bad, bad])
    say(f"eval inapplicable intervals binned={binned} segs={segs}")
    check_eval(tas, pl)
    pl2 = plans_from_lists([good, good])
    pl2 = Plans(2, np.array([-5, 1, 99], dtype=np.int64), pl2.iv_tensor, pl2.iv_out, pl2.iv_in, pl2.iv_kind)
    check_eval(tas, pl2)
    # the same on rows of several tiles, many intervals, a third of them with a tensor index out of range
    tas2 = small_random_tas(2500, N=300, T=20012, max_acc=4, base_bytes=3)
    base = make_plans(tas2, 5, 17, p_swap=0.8)
    lists = []
    for b in range(5):
        t, o, r, k = base.plan(b)
        lists.append([((int(t[j]) if j % 3 else tas2.N + j), int(o[j]), int(r[j]), int(k[j])) for j in range(len(t))] * (1 + 3 * b))
    check_eval(tas2, plans_from_lists(lists), label="out-of-range tensors")


def test_eval_order_invariance(configs_small):
    """Permuting the intervals of a plan changes nothing (the scatter uses atomics)."""
    tas = configs_small[1]
    pl = make_config_plans(1, tas, B=1)
    t, o, r, k = pl.plan(0)
    rng = np.random.default_rng(3)
    plans = []
    for _ in range(6):
        perm = rng.permutation(len(t))
        plans.append(list(zip(t[perm].tolist(), o[perm].tolist(), r[perm].tolist())))
    say("eval order invariance")
    res, peak, arg, mn = check_eval(tas, plans_from_lists(plans))
    assert torch.equal(res[0], res[5]) and len(set(peak.tolist())) == 1


def test_eval_heavy_collisions():
    """Many intervals sharing the same endpoints (LDS atomic contention) and giant sizes."""
    N, T = 3000, 5000
    tas = tas_from_lists(T, [(1 << 31) - (i % 7) for i in range(N)], [0] * N, [[T - 1]] * N)
    ivs = [(i, 10 + (i % 3), 4000 + (i % 2)) for i in range(N)]
    say("eval collisions")
    check_eval(tas, plans_from_lists([ivs, ivs[:1500], []]))


@pytest.mark.parametrize("T,B", [(5000, 9), (20011, 6)])
def test_sizes_beyond_32_bits(T, B):
    """Tensors of up to 64 GiB with odd byte counts: no common power of two brings the sizes into 32 bits, so
    every kernel keeps them as int64 (both workgroup geometries; evaluation, scoring, the windowed update)."""
    tas = small_random_tas(5100 + T, N=300, T=T, max_acc=5, timed=True, max_size=1 << 36, link_bytes_per_us=1 << 24)
    assert int(tas.size_bytes.max()) > 1 << 33 and int((tas.size_bytes & 1).sum()) > 0
    pl = make_plans(tas, B, 3, p_swap=0.6)
    say(f"wide sizes T={T} B={B}")
    h = P.tas_load(tas)
    check_eval(tas, pl, h=h, label="wide sizes")
    assert check_score(tas, pl, h=h, label="wide sizes") > 0
    # one more interval per plan on the rows just evaluated
    res, peak, arg, mn = gpu_eval(h, upload(pl))
    r0 = res.cpu().numpy().copy()
    t, o, r = extra_intervals(tas, B, 17)
    P.tensile_apply_intervals(h, *(torch.from_numpy(x).cuda() for x in (t, o, r)), res, peak, arg, mn)
    torch.cuda.synchronize()
    p1, a1, m1 = O.apply_intervals(tas, t, o, r, r0)
    assert np.array_equal(res.cpu().numpy(), r0) and np.array_equal(peak.cpu().numpy(), p1)
    assert np.array_equal(arg.cpu().numpy(), a1) and np.array_equal(mn.cpu().numpy(), m1)
    h.close()


# --------------------------------------------------------------------- score

def check_score(tas, pl, rows=None, h=None, label=""):
    own = h is None
    h = h or P.tas_load(tas)
    dp = upload(pl)
    res, peak, arg, mn = gpu_eval(h, dp)
    sc, wo, wi = gpu_score(h, dp, res, peak, arg)
    rows = list(range(pl.B)) if rows is None else list(rows)
    r0, p0, a0, m0 = O.eval_plans(tas, pl.select(rows))
    s0, o0, i0 = O.score_plans(tas, pl.select(rows), r0, p0, a0)
    idx = torch.as_tensor(np.asarray(rows), device="cuda")
    assert np.array_equal(sc[idx].cpu().numpy(), s0), label + " score"
    assert np.array_equal(wo[idx].cpu().numpy(), o0), label + " win_out"
    assert np.array_equal(wi[idx].cpu().numpy(), i0), label + " win_in"
    if own:
        h.close()
    return int((o0 >= 0).sum())


@pytest.mark.parametrize("blocks", [1, 7, 100000])
def test_score_grid_sizes(blocks, configs_small, tuning):
    """The scoring grid deals the plans round-robin over any number of workgroups: one for all plans, a few
    with several plans each (lists and filters carried from plan to plan), one per plan."""
    tuning("score_blocks", blocks)
    tas = configs_small[1]
    pl = make_config_plans(1, tas, B=60)
    say(f"score with a grid of {blocks}")
    assert check_score(tas, pl, label=f"grid {blocks}") > 10


@pytest.mark.parametrize("blocks,B", [(2, 97), (5, 64), (0, 1100)])
def test_score_given_peak_steps(blocks, B, configs_small, tuning):
    """Scoring takes the peak and its step as inputs, so any step may be given: both sides then apply the
    definition to that step.  Peak steps spread over the whole sequence (consecutive plans of a workgroup
    then look at different parts of the candidate index), some of them outside [0, T) = no candidate."""
    if blocks:
        tuning("score_blocks", blocks)
    tas = configs_small[1]
    pl = make_config_plans(1, tas, B=B)
    say(f"score with given peak steps, grid {blocks or 'default'}, B={B}")
    h = P.tas_load(tas)
    dp = upload(pl)
    res, peak, arg, mn = gpu_eval(h, dp)
    steps = prng.randint(4242, 1, np.arange(B), 0, tas.T - 1).astype(np.int32)
    keep = np.arange(B) % 5 == 0                      # every fifth plan keeps its own peak step
    a_host = np.where(keep, arg.cpu().numpy(), steps).astype(np.int32)
    outside = np.arange(B) % 11 == 3
    a_host[outside] = np.where(np.arange(B)[outside] % 2 == 0, -1, tas.T + 7)
    arg2 = torch.from_numpy(a_host).cuda()
    sc, wo, wi = gpu_score(h, dp, res, peak, arg2)
    rows = [b for b in range(B) if not outside[b]][:: max(1, B // 120)]
    r0, p0, _, _ = O.eval_plans(tas, pl.select(rows))
    s0, o0, i0 = O.score_plans(tas, pl.select(rows), r0, p0, a_host[rows])
    idx = torch.as_tensor(np.asarray(rows), device="cuda")
    assert np.array_equal(sc[idx].cpu().numpy(), s0) and np.array_equal(wo[idx].cpu().numpy(), o0)
    assert np.array_equal(wi[idx].cpu().numpy(), i0)
    assert (o0 >= 0).sum() > 100 and len(np.unique(a_host[rows] >> 8)) > 8
    out_idx = torch.as_tensor(np.flatnonzero(outside), device="cuda")
    assert int(sc[out_idx].abs().sum()) == 0 and bool((wo[out_idx] == -1).all()) and bool((wi[out_idx] == -1).all())
    h.close()


@pytest.mark.parametrize("idx,B,rows", [(0, None, None), (1, 300, range(0, 300, 7)), (2, 40, range(0, 40, 5))])
def test_score_configs(idx, B, rows, configs_small):
    tas = configs_small[idx]
    pl = make_config_plans(idx, tas, B=B)
    say(f"score config {idx} B={pl.B}")
    assert check_score(tas, pl, rows, label=f"c{idx}") > 10


@pytest.mark.parametrize("seed,timed,T", [(1, True, 60), (2, False, 60), (3, True, 3000), (4, True, 9001)])
def test_score_random(seed, timed, T):
    tas = small_random_tas(200 + seed, N=min(500, T // 2), T=T, max_acc=5, timed=timed, link_bytes_per_us=400_000)
    pl = make_plans(tas, 24, seed, p_swap=0.25)
    say(f"score random seed={seed} T={T}")
    assert check_score(tas, pl) > 0


@pytest.mark.parametrize("timed", [False, True])
def test_score_crowded_bucket(timed):
    """More candidate gaps around the peak than one pass of the scoring kernel holds, many of
    them with the same swap-out step: every tensor is generated early and read late."""
    T, N = 600, 9000
    i = np.arange(N)
    alloc = prng.randint(77, 1, i, 0, 249)
    first = prng.randint(77, 2, i, 350, 598)
    sizes = prng.randint(77, 3, i, 1, 1 << 16)
    accs = [[int(first[k])] + ([int(first[k]) + 1] if k % 3 == 0 else []) for k in range(N)]
    sn = prng.randint(77, 4, np.arange(T), 1, 1000).astype(np.int64) if timed else None
    tas = tas_from_lists(T, [int(x) for x in sizes], [int(x) for x in alloc], accs, None, sn, 0, 4000 if timed else 0)
    pl = make_plans(tas, 6, 5, p_swap=0.2)
    say(f"score crowded bucket timed={timed}")
    assert check_score(tas, pl) > 4096


def test_score_optional_windows_and_blocking():
    tas = tas_from_lists(10, [10, 3], [0, 6], [[4, 9], [7]])
    pl = plans_from_lists([[], [(0, 1, 3)], [(0, 7, 9)], [(0, 4, 9)], [(5, 1, 2), (0, -3, 2)]])
    say("score blocking")
    check_score(tas, pl)
    h = P.tas_load(tas)
    dp = upload(pl)
    res, peak, arg, mn = gpu_eval(h, dp)
    sc = torch.empty((pl.B, 2), dtype=torch.int64, device="cuda")
    P.tensile_score_candidates(h, dp, res, peak, arg, sc, None, None)
    torch.cuda.synchronize()
    assert sc.tolist() == [[3, 0], [3, 0], [0, 0], [0, 0], [3, 0]]
    h.close()


# -------------------------------------------------------------------- evaluation + scoring in one call

def gpu_step(h, dp):
    B, N = dp.B, h.N
    res = torch.full((B, h.T), -3, dtype=torch.int64, device="cuda")
    peak = torch.full((B,), -3, dtype=torch.int64, device="cuda")
    arg = torch.full((B,), -3, dtype=torch.int32, device="cuda")
    mn = torch.full((B,), -3, dtype=torch.int64, device="cuda")
    sc = torch.full((B, N), -3, dtype=torch.int64, device="cuda")
    wo = torch.full((B, N), -3, dtype=torch.int32, device="cuda")
    wi = torch.full((B, N), -3, dtype=torch.int32, device="cuda")
    P.tensile_eval_score_plans(h, dp, res, peak, arg, mn, sc, wo, wi)
    torch.cuda.synchronize()
    return res, peak, arg, mn, sc, wo, wi


def check_step(tas, pl, h=None, label=""):
    own = h is None
    h = h or P.tas_load(tas)
    got = gpu_step(h, upload(pl))
    r0, p0, a0, m0 = O.eval_plans(tas, pl)
    s0, o0, i0 = O.score_plans(tas, pl, r0, p0, a0)
    for name, g, w in zip(("resident", "peak", "argmax", "min", "score", "win_out", "win_in"), got, (r0, p0, a0, m0, s0, o0, i0)):
        assert np.array_equal(g.cpu().numpy(), w), f"{label}: {name}"
    if own:
        h.close()
    return int((o0 >= 0).sum())


@pytest.mark.parametrize("fused", [1, 0, -1])
@pytest.mark.parametrize("T,B,timed", [(8, 3, False), (4096, 5, True), (8192, 300, False), (8194, 7, True), (20012, 9, True),
                                       (50000, 4, True), (33334, 600, True)])
def test_eval_score_in_one_call(T, B, timed, fused, tuning):
    """The fused kernel forced onto every shape it is compiled for (one tile, tile edges, ragged last tiles,
    fewer plans than workgroups and several plans per workgroup), the two kernels one after the other, and the
    library's own choice: the same outputs as the oracle's evaluation followed by its scores."""
    tuning("step_fused", fused)
    N = max(2, min(400, T // 2))
    tas = small_random_tas(6000 + T, N=N, T=T, max_acc=5 if T > 8 else 1, timed=timed, base_bytes=21, link_bytes_per_us=400_000)
    pl = make_plans(tas, B, 17, p_swap=0.5)
    say(f"eval+score T={T} B={B} timed={timed} fused={fused} K={pl.n_intervals}")
    n = check_step(tas, pl, label=f"T={T} fused={fused}")
    assert n > 0 or T <= 8


def test_eval_score_in_one_call_long_and_empty_plans(tuning):
    """Plans that do not fit the registers of the evaluation phase (it takes them through the form that re-reads
    its list per tile), empty plans, and peaks in different buckets of the candidate index from plan to plan."""
    tuning("step_fused", 1)
    tas = small_random_tas(6100, N=400, T=24576, max_acc=6, timed=True, link_bytes_per_us=400_000)
    base = make_plans(tas, 14, 19, p_swap=0.6)
    lists = []
    for b in range(base.B):
        t, o, r, k = base.plan(b)
        one = [(int(t[j]), int(o[j]), int(r[j]), int(k[j])) for j in range(len(t))]
        if b in (2, 9):
            one = (one * (9000 // len(one) + 1))[:2100 + 700 * b]      # 3500 and 8400 intervals
        if b in (0, 5, 13):
            one = []
        lists.append(one)
    pl = plans_from_lists(lists)
    say(f"eval+score fused, long and empty plans: {[len(x) for x in lists]}")
    assert check_step(tas, pl, label="long and empty") > 0


def test_eval_score_in_one_call_falls_back(tuning):
    """Shapes the fused kernel is not compiled for (odd T, sizes beyond 32 bits) run the two kernels even when the
    fused one is asked for; the scoring-only outputs may be left out."""
    tuning("step_fused", 1)
    tas = small_random_tas(6200, N=300, T=20011, max_acc=5, timed=True, link_bytes_per_us=400_000)
    check_step(tas, make_plans(tas, 6, 3, p_swap=0.5), label="odd T")
    tas = small_random_tas(6201, N=300, T=20012, max_acc=5, timed=True, max_size=1 << 36, link_bytes_per_us=1 << 24)
    check_step(tas, make_plans(tas, 6, 3, p_swap=0.5), label="wide sizes")
    tas = small_random_tas(6202, N=300, T=20012, max_acc=5, timed=True, link_bytes_per_us=400_000)
    pl = make_plans(tas, 5, 4, p_swap=0.5)
    h = P.tas_load(tas)
    dp = upload(pl)
    res, peak, arg, mn, sc, wo, wi = gpu_step(h, dp)
    sc2 = torch.full_like(sc, -3)
    P.tensile_eval_score_plans(h, dp, res, peak, arg, None, sc2, None, None)
    torch.cuda.synchronize()
    assert torch.equal(sc, sc2)
    h.close()


# -------------------------------------------------------------------- latency updates

def test_update_latencies_rescoring_and_greedy():
    """After new latencies only the scores, windows and the greedy's choices change; footprints
    evaluated before stay valid.  Everything must equal what a freshly loaded sequence gives."""
    import copy
    tas = small_random_tas(901, N=300, T=3000, max_acc=4, timed=True, link_bytes_per_us=300_000)
    pl = make_plans(tas, 16, 3, p_swap=0.25)
    h = P.tas_load(tas)
    dp = upload(pl)
    res, peak, arg, mn = gpu_eval(h, dp)
    say("update latencies")
    r0, p0, a0, m0 = O.eval_plans(tas, pl)
    variants = [
        (prng.randint(5, 1, np.arange(tas.T), 1, 5000).astype(np.int64), 300_000),     # drifted latencies
        (tas.step_ns, 40_000),                                                           # slower link
        (None, 0),                                                                        # no latencies at all
        (tas.step_ns, 300_000),                                                          # back to the start
    ]
    for step_ns, link in variants:
        t2 = copy.copy(tas)
        t2.step_ns, t2.link_bytes_per_us = step_ns, link
        P.tensile_tas_update_latencies(h, step_ns, link)
        sc, wo, wi = gpu_score(h, dp, res, peak, arg)            # footprints from before the update
        s0, o0, i0 = O.score_plans(t2, pl, r0, p0, a0)
        assert np.array_equal(sc.cpu().numpy(), s0) and np.array_equal(wo.cpu().numpy(), o0)
        assert np.array_equal(wi.cpu().numpy(), i0)
        same_greedy(P.tensile_greedy_plan(h, 0, max_iters=25, capacity=64, recompute=True),
                    O.greedy(t2, 0, max_iters=25, recompute=True))
        res2, peak2, arg2, mn2 = gpu_eval(h, dp)
        assert torch.equal(res2, res) and torch.equal(peak2, peak) and torch.equal(arg2, arg)
    with pytest.raises(P.TensileError):
        P.tensile_tas_update_latencies(h, np.zeros(tas.T, dtype=np.int64), 1000)       # latencies must be positive
    with pytest.raises(P.TensileError):
        P.tensile_tas_update_latencies(h, tas.step_ns, 0)
    h.close()


# -------------------------------------------------------------------- per-job peaks

def check_per_job(tas, pl, label=""):
    h = P.tas_load(tas)
    dp = upload(pl)
    J, B = int(tas.J), pl.B
    jp = torch.empty((J, B), dtype=torch.int64, device="cuda")
    ja = torch.empty((J, B), dtype=torch.int32, device="cuda")
    tot = torch.empty(B, dtype=torch.int64, device="cuda")
    P.tensile_eval_plans_per_job(h, dp, jp, ja, tot)
    torch.cuda.synchronize()
    p0, a0, t0 = O.eval_per_job(tas, pl)
    assert np.array_equal(jp.cpu().numpy(), p0), label + " job_peak"
    assert np.array_equal(ja.cpu().numpy(), a0), label + " job_argmax"
    assert np.array_equal(tot.cpu().numpy(), t0), label + " sum_peak"
    # optional outputs left out; the merged evaluation of the same handle is unaffected
    jp2 = torch.empty((J, B), dtype=torch.int64, device="cuda")
    P.tensile_eval_plans_per_job(h, dp, jp2)
    res, peak, arg, mn = gpu_eval(h, dp)
    assert torch.equal(jp2, jp) and bool((tot >= peak).all())
    _, p1, a1, _ = O.eval_plans(tas, pl, want_resident=False)
    assert np.array_equal(peak.cpu().numpy(), p1) and np.array_equal(arg.cpu().numpy(), a1)
    h.close()


@pytest.mark.parametrize("seed,J,T", [(1, 2, 90), (2, 3, 5000), (3, 7, 20001)])
def test_per_job_random(seed, J, T):
    tas = small_random_tas(600 + seed, N=min(400, T // 2), T=T, max_acc=4, timed=False, base_bytes=1000 * seed)
    tas.job_id = prng.randint(seed, 9, np.arange(tas.N), 0, J - 1).astype(np.int32)
    tas.J = J
    pl = make_plans(tas, 20, seed, p_swap=0.3)
    say(f"per-job random seed={seed} J={J} T={T}")
    check_per_job(tas, pl)


def test_per_job_configs(configs_small):
    say("per-job config 0 (one job) and hand example")
    tas = configs_small[0]
    check_per_job(tas, make_config_plans(0, tas, B=16), "c0")
    tas = tas_from_lists(8, [4, 2, 5, 3], [0, 1, 4, 5], [[3], [2], [7], [6]], jobs=[0, 0, 1, 1], base_bytes=10)
    check_per_job(tas, plans_from_lists([[], [(2, 4, 7)], [(0, 0, 3), (2, 4, 7)], [(9, 1, 2), (0, -1, 2)]]), "hand")


# -------------------------------------------------------------------- recomputation scores

def gpu_score_recompute(h, dp, res, peak, arg):
    B, N = dp.B, h.N
    sc = torch.empty((B, N), dtype=torch.int64, device="cuda")
    wo = torch.empty((B, N), dtype=torch.int32, device="cuda")
    wi = torch.empty((B, N), dtype=torch.int32, device="cuda")
    P.tensile_score_recompute(h, dp, res, peak, arg, sc, wo, wi)
    torch.cuda.synchronize()
    return sc, wo, wi


def check_score_recompute(tas, pl, rows=None, label=""):
    h = P.tas_load(tas)
    dp = upload(pl)
    res, peak, arg, mn = gpu_eval(h, dp)
    sc, wo, wi = gpu_score_recompute(h, dp, res, peak, arg)
    # the swap scores of the same handle are untouched by the second index
    s1, o1, i1 = gpu_score(h, dp, res, peak, arg)
    rows = list(range(pl.B)) if rows is None else list(rows)
    r0, p0, a0, m0 = O.eval_plans(tas, pl.select(rows))
    s0, o0, i0 = O.score_recompute_plans(tas, pl.select(rows), r0, p0, a0)
    idx = torch.as_tensor(np.asarray(rows), device="cuda")
    assert np.array_equal(sc[idx].cpu().numpy(), s0), label + " saving"
    assert np.array_equal(wo[idx].cpu().numpy(), o0), label + " win_out"
    assert np.array_equal(wi[idx].cpu().numpy(), i0), label + " win_in"
    s2, o2, i2 = O.score_plans(tas, pl.select(rows), r0, p0, a0)
    assert np.array_equal(s1[idx].cpu().numpy(), s2) and np.array_equal(o1[idx].cpu().numpy(), o2)
    h.close()
    return int((o0 >= 0).sum())


@pytest.mark.parametrize("idx,B,rows", [(0, None, None), (1, 300, range(0, 300, 7)), (2, 40, range(0, 40, 5))])
def test_score_recompute_configs(idx, B, rows, configs_small):
    tas = configs_small[idx]
    pl = make_config_plans(idx, tas, B=B)
    say(f"score recompute config {idx} B={pl.B}")
    assert check_score_recompute(tas, pl, rows, label=f"c{idx}") > 10


@pytest.mark.parametrize("seed,timed,T", [(1, True, 60), (2, False, 60), (3, True, 3000), (4, True, 9001)])
def test_score_recompute_random(seed, timed, T):
    tas = small_random_tas(500 + seed, N=min(500, T // 2), T=T, max_acc=5, timed=timed, link_bytes_per_us=400_000)
    pl = make_plans(tas, 24, seed, p_swap=0.1)
    say(f"score recompute random seed={seed} T={T}")
    assert check_score_recompute(tas, pl) > 0


def test_score_recompute_any_interval_excludes():
    tas = tas_from_lists(10, [10, 3], [0, 6], [[4, 9], [7]])
    pl = plans_from_lists([[], [(0, 1, 3)], [(0, 7, 9)], [(5, 1, 2), (0, -3, 2)]])
    say("score recompute exclusion")
    check_score_recompute(tas, pl)


# -------------------------------------------------------------------- greedy

def same_greedy(g, o):
    for f in ("iv_tensor", "iv_out", "iv_in", "iv_kind", "peak_trace"):
        assert np.array_equal(g[f], o[f]), f
    assert g["final_peak"] == o["final_peak"]


@pytest.mark.parametrize("idx", [0, 1])
def test_greedy_matches_oracle(idx, configs_small):
    tas = configs_small[idx]
    say(f"greedy config {idx}")
    h = P.tas_load(tas)
    o = O.greedy(tas, 0)
    g = P.tensile_greedy_plan(h, 0, capacity=len(o["iv_tensor"]) + 8)
    same_greedy(g, o)
    # the emitted plan passes the semantic validator
    dp = P.DevicePlans.from_numpy(np.array([0, len(g["iv_tensor"])]), g["iv_tensor"], g["iv_out"], g["iv_in"], g["iv_kind"])
    assert P.tensile_validate_plans(h, dp) == (-1, 0)
    h.close()


def test_greedy_options(configs_small):
    tas = configs_small[1]
    h = P.tas_load(tas)
    say("greedy options")
    same_greedy(P.tensile_greedy_plan(h, 0, max_iters=7, capacity=64), O.greedy(tas, 0, max_iters=7))
    budget = int(P.tensile_tas_info(h)[0] * 60 // 100)
    same_greedy(P.tensile_greedy_plan(h, budget, stop_at_budget=True, capacity=4096),
                O.greedy(tas, budget, stop_at_budget=True))
    same_greedy(P.tensile_greedy_plan(h, 0, min_iters=0, capacity=4096), O.greedy(tas, 0, min_iters=0))
    # capacity reached
    g = P.tensile_greedy_plan(h, 0, capacity=5)
    assert len(g["iv_tensor"]) == 5
    # extend an existing plan
    first = O.greedy(tas, 0, max_iters=4)
    init = (first["iv_tensor"], first["iv_out"], first["iv_in"], first["iv_kind"])
    same_greedy(P.tensile_greedy_plan(h, 0, max_iters=6, capacity=64, initial=init),
                O.greedy(tas, 0, max_iters=6, initial=init))
    h.close()


@pytest.mark.parametrize("seed,link", [(11, 200_000), (12, 60_000), (13, 2)])
def test_greedy_recompute_phase(seed, link):
    tas = small_random_tas(400 + seed, N=150, T=240, max_acc=4, timed=True, link_bytes_per_us=link)
    say(f"greedy recompute seed={seed}")
    h = P.tas_load(tas)
    o = O.greedy(tas, 0, recompute=True, min_iters=1 << 30)
    assert (o["iv_kind"] == 1).sum() >= 2
    g = P.tensile_greedy_plan(h, 0, recompute=True, min_iters=1 << 30, capacity=len(o["iv_tensor"]) + 8)
    same_greedy(g, o)
    # a budget in the middle of the recomputation phase, and one the swap phase already meets
    n_swap = int((o["iv_kind"] == 0).sum())
    for budget in (int(o["peak_trace"][n_swap + 1]), int(o["peak_trace"][n_swap])):
        same_greedy(P.tensile_greedy_plan(h, budget, recompute=True, min_iters=1 << 30, capacity=512),
                    O.greedy(tas, budget, recompute=True, min_iters=1 << 30))
    # the paper's stall rule and a cap on the iterations cut through both phases alike
    same_greedy(P.tensile_greedy_plan(h, 0, recompute=True, min_iters=2, capacity=512),
                O.greedy(tas, 0, recompute=True, min_iters=2))
    same_greedy(P.tensile_greedy_plan(h, 0, recompute=True, min_iters=1 << 30, max_iters=n_swap + 1, capacity=512),
                O.greedy(tas, 0, recompute=True, min_iters=1 << 30, max_iters=n_swap + 1))
    h.close()


@pytest.mark.parametrize("idx", [0, 1])
def test_greedy_recompute_config(idx, configs_small):
    tas = configs_small[idx]        # (config 0 has no latencies: recomputation time 1 for every tensor)
    say(f"greedy recompute config {idx}")
    h = P.tas_load(tas)
    o = O.greedy(tas, 0, recompute=True, min_iters=1 << 30)
    g = P.tensile_greedy_plan(h, 0, recompute=True, min_iters=1 << 30, capacity=len(o["iv_tensor"]) + 8)
    same_greedy(g, o)
    if idx == 1:
        assert (g["iv_kind"] == 1).sum() > 100 and (g["iv_kind"] == 0).sum() > 100
    h.close()


def test_greedy_rate_limit_and_link():
    tas = tas_from_lists(8, [50, 40, 100, 30], [1, 2, 4, 2], [[7], [6], [5], [6]], jobs=[0, 1, 0, 1])
    tas.J = 2
    h = P.tas_load(tas)
    say("greedy rate limit")
    for num, den in (([1, 0], 1), ([1, 1], 2)):
        same_greedy(P.tensile_greedy_plan(h, 0, msr_num=num, msr_den=den, capacity=16),
                    O.greedy(tas, 0, msr_num=np.array(num), msr_den=den))
    h.close()
    tas = tas_from_lists(12, [20, 20, 100], [0, 0, 5], [[11], [11], [6]], step_ns=[10] * 12, link_bytes_per_us=1000)
    h = P.tas_load(tas)
    g = P.tensile_greedy_plan(h, 0, capacity=16)
    same_greedy(g, O.greedy(tas, 0))
    assert list(zip(g["iv_tensor"].tolist(), g["iv_out"].tolist(), g["iv_in"].tolist())) == [(0, 2, 11), (1, 4, 9)]
    h.close()


def test_greedy_random_timed():
    for seed in range(4):
        tas = small_random_tas(500 + seed, N=120, T=400, max_acc=5, timed=True, link_bytes_per_us=300_000)
        say(f"greedy random {seed}")
        h = P.tas_load(tas)
        same_greedy(P.tensile_greedy_plan(h, 0, capacity=2048), O.greedy(tas, 0))
        h.close()


# ------------------------------------------------------------------ validate

def test_validate_plans(configs_small):
    tas = configs_small[1]
    h = P.tas_load(tas)
    pl = make_config_plans(1, tas, B=8)
    say("validate")
    assert P.tensile_validate_plans(h, upload(pl)) == (-1, 0)
    k = int(pl.plan_offsets[3]) + 2
    bad = Plans(pl.B, pl.plan_offsets, pl.iv_tensor.copy(), pl.iv_out.copy(), pl.iv_in.copy(), pl.iv_kind)
    bad.iv_in[k] = bad.iv_out[k]                    # empty or reversed window
    assert P.tensile_validate_plans(h, upload(bad)) == (k, 1)
    bad.iv_in[k] = tas.T                            # reaches past the next access
    assert P.tensile_validate_plans(h, upload(bad)) == (k, 2)
    dup = Plans(pl.B, pl.plan_offsets, pl.iv_tensor.copy(), pl.iv_out.copy(), pl.iv_in.copy(), pl.iv_kind)
    dup.iv_tensor[k], dup.iv_out[k], dup.iv_in[k] = dup.iv_tensor[k - 1], dup.iv_out[k - 1], dup.iv_in[k - 1]
    assert P.tensile_validate_plans(h, upload(dup)) == (k, 3)
    h.close()


def test_argument_errors(configs_small):
    tas = configs_small[0]
    h = P.tas_load(tas)
    dp = upload(make_config_plans(0, tas, B=4))
    peak = torch.empty(4, dtype=torch.int64, device="cuda")
    arg = torch.empty(4, dtype=torch.int32, device="cuda")
    with pytest.raises(P.TensileError):
        P.tensile_eval_plans(h, dp, None, peak.cpu(), arg)                  # host tensor
    with pytest.raises(P.TensileError):
        P.tensile_eval_plans(h, dp, None, peak[:2], arg)                    # too short
    with pytest.raises(P.TensileError):
        P.tensile_eval_plans(h, dp, None, None, arg)                        # required output missing
    h.close()
    with pytest.raises(P.TensileError):
        P.tensile_tas_info(h)                                               # freed handle


# ------------------------------------------------- full-size configurations

N_THREADS = min(16, os.cpu_count() or 1)      # the oracle's C loops release the interpreter lock: plans split over threads


def plan_range(pl: Plans, b0: int, b1: int) -> Plans:
    """Plans b0 .. b1-1 of the batch as views (no copies)."""
    k0, k1 = int(pl.plan_offsets[b0]), int(pl.plan_offsets[b1])
    return Plans(b1 - b0, pl.plan_offsets[b0:b1 + 1] - k0, pl.iv_tensor[k0:k1], pl.iv_out[k0:k1], pl.iv_in[k0:k1], pl.iv_kind[k0:k1])


def in_threads(fn, pieces):
    """fn(piece) for every piece, on N_THREADS threads; results in order."""
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=N_THREADS) as pool:
        return list(pool.map(fn, pieces))


def cuts(b0, b1, n):
    edges = np.linspace(b0, b1, min(n, b1 - b0) + 1).astype(np.int64)
    return [(int(edges[k]), int(edges[k + 1])) for k in range(len(edges) - 1) if edges[k + 1] > edges[k]]


@pytest.mark.parametrize("idx,n_score", [(1, 4096), (2, 8192), (3, 2048), (4, 128)])
def test_full_size_config(idx, n_score):
    """The whole batch on the GPU in the launch configuration the benchmark times, and EVERY plan of it
    against the oracle: peak, peak step, minimum and the full footprint rows (rows downloaded in chunks of at
    most 1 GB), the same for the windowed update of every row and the per-job peaks; scores, recomputation
    savings and link occupancy on `n_score` plans spread over the batch (all of them on configuration 1)."""
    cfg = CONFIGS[idx]
    say(f"full-size config {idx}: building TAS and {cfg.B} plans")
    tas = make_tas(idx)
    pl = make_config_plans(idx, tas)
    B, T, N = cfg.B, tas.T, tas.N
    say(f"  N={N} T={T} K={pl.n_intervals}; uploading")
    h = P.tas_load(tas)
    dp = upload(pl)
    res, peak, arg, mn = gpu_eval(h, dp)
    MF0 = O.base_timeline(tas)

    say("  peak, peak step and minimum of every plan")
    parts = in_threads(lambda c: O.eval_plans(tas, plan_range(pl, *c), want_resident=False, MF0=MF0), cuts(0, B, 4 * N_THREADS))
    p_all, a_all, m_all = (np.concatenate([x[k] for x in parts]) for k in (1, 2, 3))
    assert np.array_equal(peak.cpu().numpy(), p_all) and np.array_equal(arg.cpu().numpy(), a_all)
    assert np.array_equal(mn.cpu().numpy(), m_all)
    # the same through the peaks-only launch (another kernel variant)
    _, peak2, arg2, _ = gpu_eval(h, dp, want_resident=False, want_min=False)
    assert np.array_equal(peak2.cpu().numpy(), p_all) and np.array_equal(arg2.cpu().numpy(), a_all)
    del peak2, arg2

    # one more interval per plan on a copy of the rows (windowed update), then both sets of rows in chunks
    t1, o1, r1 = extra_intervals(tas, B, 99)
    res_up = res.clone()
    peak_up, arg_up, mn_up = torch.empty_like(peak), torch.empty_like(arg), torch.empty_like(mn)
    P.tensile_apply_intervals(h, torch.from_numpy(t1).cuda(), torch.from_numpy(o1).cuda(), torch.from_numpy(r1).cuda(),
                              res_up, peak_up, arg_up, mn_up)
    torch.cuda.synchronize()
    chunk = max(1, (1 << 30) // (8 * T))
    say(f"  every footprint row, and every row after the windowed update, in chunks of {chunk} plans")
    pu, au, mu = peak_up.cpu().numpy(), arg_up.cpu().numpy(), mn_up.cpu().numpy()
    for b0 in range(0, B, chunk):
        b1 = min(B, b0 + chunk)
        want = np.empty((b1 - b0, T), dtype=np.int64)

        def rows_of(c, want=want, b0=b0):
            r, _, _, _ = O.eval_plans(tas, plan_range(pl, *c), MF0=MF0)
            want[c[0] - b0:c[1] - b0] = r
            # the windowed update of these rows by the oracle, in place on its own copy
            r2 = r.copy()
            pa, aa, ma = O.apply_intervals(tas, t1[c[0]:c[1]], o1[c[0]:c[1]], r1[c[0]:c[1]], r2)
            return c, r2, pa, aa, ma
        pieces = in_threads(rows_of, cuts(b0, b1, N_THREADS))
        got = res[b0:b1].cpu().numpy()
        assert np.array_equal(got, want), f"rows of plans {b0}..{b1}"
        got = res_up[b0:b1].cpu().numpy()
        for c, r2, pa, aa, ma in pieces:
            assert np.array_equal(got[c[0] - b0:c[1] - b0], r2), f"updated rows of plans {c[0]}..{c[1]}"
            assert np.array_equal(pu[c[0]:c[1]], pa) and np.array_equal(au[c[0]:c[1]], aa) and np.array_equal(mu[c[0]:c[1]], ma)
        del got, want, pieces
        say(f"    plans {b0}..{b1} ok")
    del res_up, peak_up, arg_up, mn_up

    if tas.J > 1 and tas.J <= 8:
        say(f"  per-job peaks of every plan ({tas.J} jobs)")
        jp = torch.empty((int(tas.J), B), dtype=torch.int64, device="cuda")
        ja = torch.empty((int(tas.J), B), dtype=torch.int32, device="cuda")
        tot = torch.empty(B, dtype=torch.int64, device="cuda")
        P.tensile_eval_plans_per_job(h, dp, jp, ja, tot)
        torch.cuda.synchronize()
        parts = in_threads(lambda c: O.eval_per_job(tas, plan_range(pl, *c)), cuts(0, B, 4 * N_THREADS))
        assert np.array_equal(jp.cpu().numpy(), np.concatenate([x[0] for x in parts], axis=1))
        assert np.array_equal(ja.cpu().numpy(), np.concatenate([x[1] for x in parts], axis=1))
        assert np.array_equal(tot.cpu().numpy(), np.concatenate([x[2] for x in parts]))
        del jp, ja, tot

    # scores, recomputation savings, link occupancy: the whole batch on the GPU, n_score plans by the oracle
    rows = np.unique(np.linspace(0, B - 1, min(n_score, B)).astype(np.int64))
    sidx = torch.as_tensor(rows, device="cuda")
    say(f"  scoring the whole batch; the oracle scores {len(rows)} plans")
    sc = torch.empty((B, N), dtype=torch.int64, device="cuda")
    wo = torch.empty((B, N), dtype=torch.int32, device="cuda")
    wi = torch.empty((B, N), dtype=torch.int32, device="cuda")
    P.tensile_score_candidates(h, dp, res, peak, arg, sc, wo, wi)
    torch.cuda.synchronize()
    got_s = [x[sidx].cpu().numpy() for x in (sc, wo, wi)]
    say("  the same batch through tensile_eval_score_plans")
    one_call = gpu_step(h, dp)
    for name, g, w in zip(("resident", "peak", "argmax", "min", "score", "win_out", "win_in"), one_call, (res, peak, arg, mn, sc, wo, wi)):
        assert torch.equal(g, w), f"one call: {name}"
    del one_call
    size = torch.from_numpy(tas.size_bytes).cuda()
    assert bool((sc >= 0).all()) and bool((sc <= size[None, :]).all()) and bool(((wo >= 0) | (sc == 0)).all())
    P.tensile_score_recompute(h, dp, res, peak, arg, sc, wo, wi)
    torch.cuda.synchronize()
    got_r = [x[sidx].cpu().numpy() for x in (sc, wo, wi)]
    assert bool((sc >= 0).all()) and bool((sc <= size[None, :]).all()) and bool(((wo >= 0) | (sc == 0)).all())
    del sc, wo, wi

    def scores_of(c):
        sel = pl.select(rows[c[0]:c[1]])
        r0, p0, a0, _ = O.eval_plans(tas, sel, MF0=MF0)
        return O.score_plans(tas, sel, r0, p0, a0), O.score_recompute_plans(tas, sel, r0, p0, a0)
    pieces = cuts(0, len(rows), 2 * N_THREADS)
    for c, (swap, rec) in zip(pieces, in_threads(scores_of, pieces)):
        for k, name in enumerate(("score", "win_out", "win_in")):
            assert np.array_equal(got_s[k][c[0]:c[1]], swap[k]), f"{name} of sampled plans {c}"
            assert np.array_equal(got_r[k][c[0]:c[1]], rec[k]), f"recomputation {name} of sampled plans {c}"
    assert int((got_s[1] >= 0).sum()) > len(rows)

    if tas.step_ns is not None:
        say("  link occupancy of the whole batch")
        lrows = torch.empty((B, T), dtype=torch.int32, device="cuda")
        lpk = torch.empty(B, dtype=torch.int32, device="cuda")
        larg = torch.empty(B, dtype=torch.int32, device="cuda")
        lover = torch.empty(B, dtype=torch.int32, device="cuda")
        P.tensile_eval_link(h, dp, lpk, lrows, larg, lover, reuse_host_copies=True)
        torch.cuda.synchronize()
        got_l = [x[sidx].cpu().numpy() for x in (lrows, lpk, larg, lover)]
        for c, want_l in zip(pieces, in_threads(lambda c: O.link_occupancy(tas, pl.select(rows[c[0]:c[1]]), reuse=True), pieces)):
            for k, name in enumerate(("link rows", "link peak", "link peak step", "overbooked")):
                assert np.array_equal(got_l[k][c[0]:c[1]], want_l[k]), f"{name} of sampled plans {c}"
        assert torch.equal(lrows.max(dim=1).values, lpk) and bool((lrows >= 0).all())
        assert torch.equal((lrows >= 2).sum(dim=1).to(torch.int32), lover)
        del lrows
    h.close()


@pytest.mark.parametrize("idx", [2, 3])
def test_greedy_on_large_configs(idx):
    """The planner on the two-iteration transformer and on the four merged jobs, capped at 64 iterations:
    from nothing, and - with a swapping rate of zero per job, so that swapping ends after each job's first
    swap - through the recomputation phase on top of an existing plan (the batch's first)."""
    tas = make_tas(idx)
    say(f"greedy on config {idx}: N={tas.N} T={tas.T}")
    h = P.tas_load(tas)
    same_greedy(P.tensile_greedy_plan(h, 0, max_iters=64, capacity=64), O.greedy(tas, 0, max_iters=64))
    first = make_config_plans(idx, tas, B=1)
    init = tuple(np.ascontiguousarray(x) for x in first.plan(0))
    n0 = len(init[0])
    zero = np.zeros(int(tas.J), dtype=np.int64)
    o = O.greedy(tas, 0, max_iters=64, initial=init, recompute=True, msr_num=zero, msr_den=1, capacity=n0 + 64)
    g = P.tensile_greedy_plan(h, 0, max_iters=64, initial=init, recompute=True, msr_num=zero, msr_den=1, capacity=n0 + 64)
    same_greedy(g, o)
    kinds = g["iv_kind"][n0:]
    say(f"  on top of {n0} intervals: {int((kinds == 0).sum())} swaps, {int((kinds == 1).sum())} recomputations")
    assert len(kinds) == 64 and (kinds == 1).sum() >= 32
    h.close()
