"""The entry point that allocates nothing (tensile_eval_plans_static) against tensile_eval_plans, bit for
bit, through the C ABI: two calls in a row on the same GPU, the second on a smaller input, in the shapes
that use the preallocated scratch (several segments per plan, batches sorted by tile first)."""
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("needs a GPU", allow_module_level=True)

import paper_2105_13336_amd as P  # noqa: E402
from workloads import make_plans, plans_from_lists, small_random_tas  # noqa: E402


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def outputs(B, T, fill):
    return (torch.full((B, T), fill, dtype=torch.int64, device="cuda"), torch.full((B,), fill, dtype=torch.int64, device="cuda"),
            torch.full((B,), fill, dtype=torch.int32, device="cuda"), torch.full((B,), fill, dtype=torch.int64, device="cuda"))


def long_plans(tas, B, seed, length):
    base = make_plans(tas, B, seed, p_swap=0.8)
    lists = []
    for b in range(B):
        t, o, r, k = base.plan(b)
        one = [(int(t[j]), int(o[j]), int(r[j]), int(k[j])) for j in range(len(t))]
        lists.append((one * (length // max(1, len(one)) + 1))[:length + 7 * b])
    return plans_from_lists(lists)


def compare(h, pl, label):
    dp = P.DevicePlans.from_numpy(pl.plan_offsets, pl.iv_tensor, pl.iv_out, pl.iv_in, pl.iv_kind)
    want = outputs(pl.B, h.T, -5)
    got = outputs(pl.B, h.T, -9)
    P.tensile_eval_plans(h, dp, *want)
    P.tensile_eval_plans_static(h, dp, *got)
    torch.cuda.synchronize()
    for name, g, w in zip(("resident", "peak", "argmax", "min_resident"), got, want):
        assert torch.equal(g, w), f"{label}: {name}"
    # peaks only
    P.tensile_eval_plans_static(h, dp, None, got[1].fill_(-1), got[2].fill_(-1), None)
    torch.cuda.synchronize()
    assert torch.equal(got[1], want[1]) and torch.equal(got[2], want[2]), f"{label}: peaks only"


def test_static_scratch_two_calls_second_smaller():
    tas = small_random_tas(8101, N=400, T=50001, max_acc=5, base_bytes=3)
    h = P.tas_load(tas)
    # few plans of many tiles: the host splits every plan into segments, whose partials live in the scratch
    say("no-alloc: 9 plans of 50001 steps, then 4")
    compare(h, make_plans(tas, 9, 3, p_swap=0.7), "segments, first call")
    compare(h, make_plans(tas, 4, 4, p_swap=0.3), "segments, second (smaller) call")
    # plans too long for the registers: sorted by tile first, records and tile tables in the scratch
    say("no-alloc: 12 plans of 7000 intervals, then 5 of 6500")
    compare(h, long_plans(tas, 12, 5, 7000), "binned, first call")
    compare(h, long_plans(tas, 5, 6, 6500), "binned, second (smaller) call")
    # ... and a batch whose records do not fit the scratch: evaluated from the lists as they are
    say("no-alloc: 200 plans of 7000 intervals (records beyond the scratch)")
    compare(h, long_plans(tas, 200, 7, 7000), "long plans without binning")
    compare(h, make_plans(tas, 3, 8, p_swap=0.5), "after it, a small call")
    h.close()


def test_static_scratch_short_rows_and_empty_batches():
    tas = small_random_tas(8102, N=60, T=777, max_acc=4, base_bytes=0)
    h = P.tas_load(tas)
    say("no-alloc: short rows")
    compare(h, make_plans(tas, 700, 9, p_swap=0.5), "short rows, many plans")
    compare(h, make_plans(tas, 2, 10, p_swap=0.5), "short rows, two plans")
    empty = plans_from_lists([])
    dp = P.DevicePlans.from_numpy(empty.plan_offsets, empty.iv_tensor, empty.iv_out, empty.iv_in, empty.iv_kind)
    P.tensile_eval_plans_static(h, dp, None, torch.empty(0, dtype=torch.int64, device="cuda"),
                                torch.empty(0, dtype=torch.int32, device="cuda"), None)
    h.close()


def test_static_scratch_rejects_what_does_not_fit(tuning):
    """More per-segment partials than the array holds: a clear error, nothing enqueued."""
    tuning("eval_segments", 3)
    tas = small_random_tas(8103, N=50, T=20011, max_acc=3)
    h = P.tas_load(tas)
    B = 300_000                          # x 3 segments x 20 bytes > 16 MiB
    offs = torch.zeros(B + 1, dtype=torch.int64, device="cuda")
    none32 = torch.zeros(0, dtype=torch.int32, device="cuda")
    dp = P.DevicePlans(offs, none32, none32, none32, None)
    peak = torch.zeros(B, dtype=torch.int64, device="cuda")
    arg = torch.zeros(B, dtype=torch.int32, device="cuda")
    say("no-alloc: over capacity")
    with pytest.raises(P.TensileError) as e:
        P.tensile_eval_plans_static(h, dp, None, peak, arg, None)
    assert e.value.code == P.binding.TENSILE_E_CAPACITY and "scratch" in str(e.value)
    P.tensile_tuning_reset()
    P.tensile_eval_plans_static(h, dp, None, peak, arg, None)      # one segment per plan: no partials, fits
    torch.cuda.synchronize()
    mf0 = P.tensile_tas_base_timeline(h)
    assert int(peak.min()) == int(peak.max()) == int(mf0.max()) and int(arg[0]) == int(np.argmax(mf0))
    h.close()
