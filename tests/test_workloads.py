"""Seeded generators: determinism, agreement of the C and numpy recipes, shapes."""
import numpy as np
import pytest

from workloads import (CONFIGS, eligible_gaps, make_config_plans, make_plans, make_plans_numpy, make_tas, plans_hash,
                       small_random_tas, tas_hash)
from workloads import plans as plans_mod
from workloads import prng


def test_c_and_numpy_mixers_agree():
    lib = plans_mod._lib()
    for seed, stream, idx in [(0, 0, 0), (210513336, 3, 12345), (2**63 + 5, 2**40, 2**62 + 1)]:
        assert int(prng.u64(seed, stream, idx)) == lib.plangen_u64(seed, stream, idx)


def test_uniform_and_randint_ranges():
    u = prng.uniform01(7, 1, np.arange(100000))
    assert 0.0 <= u.min() and u.max() < 1.0 and abs(u.mean() - 0.5) < 0.01
    r = prng.randint(7, 2, np.arange(100000), -3, 4)
    assert r.min() == -3 and r.max() == 4


@pytest.mark.parametrize("idx", [0, 1])
def test_plan_generators_agree(idx, configs_small):
    tas = configs_small[idx]
    a = make_plans(tas, 5, CONFIGS[idx].seed, b0=3)
    b = make_plans_numpy(tas, 5, CONFIGS[idx].seed, b0=3)
    for f in ("plan_offsets", "iv_tensor", "iv_out", "iv_in", "iv_kind"):
        assert np.array_equal(getattr(a, f), getattr(b, f)), f


def test_plan_chunks_concatenate(configs_small):
    tas = configs_small[0]
    whole = make_plans(tas, 8, 99)
    lo, hi = make_plans(tas, 3, 99, b0=0), make_plans(tas, 5, 99, b0=3)
    assert np.array_equal(whole.iv_out, np.concatenate([lo.iv_out, hi.iv_out]))
    assert np.array_equal(whole.plan_offsets[4:] - whole.plan_offsets[3], hi.plan_offsets[1:])


@pytest.mark.parametrize("idx", [0, 1, 2])
def test_generated_plans_are_valid(idx, configs_small):
    """Every interval lies inside one gap of its tensor and is non-empty; at most one per tensor."""
    tas = configs_small[idx]
    pl = make_config_plans(idx, tas, B=4)
    eoff, ep, eq = eligible_gaps(tas)
    for b in range(4):
        t, o, r, k = pl.plan(b)
        assert len(set(t.tolist())) == len(t) and np.all(k == 0)
        for i, oo, rr in zip(t, o, r):
            gaps = list(zip(ep[eoff[i]:eoff[i + 1]], eq[eoff[i]:eoff[i + 1]]))
            assert any(p <= oo and rr <= q for p, q in gaps) and rr >= oo + 2
    frac = pl.n_intervals / 4 / np.count_nonzero(np.diff(eoff))
    assert 0.2 < frac < 0.4


def test_config_shapes(configs_small):
    want = {0: (60, 200), 1: (3000, 6000), 2: (10000, 24000)}
    for idx, (n, t) in want.items():
        tas = configs_small[idx]
        tas.check()
        assert tas.T == t
        assert tas.N == n if idx == 0 else abs(tas.N - n) <= 0.1 * n
    assert configs_small[0].step_ns is None and configs_small[1].step_ns is not None
    assert configs_small[1].step_ns.min() >= 50_000 and configs_small[1].step_ns.max() <= 2_000_000


def test_across_iteration_reads(configs_small):
    """In the two-iteration trace the parameters written by the first optimizer
    phase are read again in the second iteration (section IV-C of the paper)."""
    tas = configs_small[2]
    idx = [i for i, n in enumerate(tas.names) if n.startswith("j0.i0.") and n.endswith(".new")]
    assert len(idx) > 100
    cnt = np.diff(tas.access_offsets)[idx]
    assert np.all(cnt >= 1)


@pytest.mark.slow
def test_big_config_shapes():
    for idx, (n, t) in {3: (20000, 50000), 4: (200000, 1000000)}.items():
        tas = make_tas(idx)
        tas.check()
        assert tas.T == t and abs(tas.N - n) <= 0.1 * n
        if idx == 4:
            assert tas.N == n and tas.size_bytes.max() <= 1 << 31 and tas.size_bytes.min() >= 256
            k = np.diff(tas.access_offsets)
            assert k.min() >= 2 and k.max() <= 20
            assert 0.5 < np.median(tas.size_bytes) / (1 << 20) < 2.0


def test_determinism():
    a, b = make_tas(0), make_tas(0)
    assert tas_hash(a) == tas_hash(b)
    assert plans_hash(make_config_plans(0, a)) == plans_hash(make_config_plans(0, b))
    assert tas_hash(small_random_tas(1, 10, 30)) != tas_hash(small_random_tas(2, 10, 30))
