"""The C-ABI library loads and exports every symbol that include/tensile.h declares, and its host-side
argument checks work without a GPU (no compute call is made here)."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "tensile.h")
LIB = os.path.join(ROOT, "paper_2105_13336_amd", "libtensile.so")


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(tensile_[a-z_]+)\s*\(", src)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2105_13336_amd.build import build_library
        build_library()
    return ctypes.CDLL(LIB)


def test_header_declares_the_four_entry_points():
    names = declared_functions()
    for required in ("tensile_tas_load", "tensile_eval_plans", "tensile_score_candidates", "tensile_greedy_plan"):
        assert required in names


def test_every_declared_symbol_is_exported(lib):
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_binding_lists_the_same_names():
    from paper_2105_13336_amd import binding
    assert sorted(binding.EXPORTS) == declared_functions()
    for name in ("tensile_tas_load", "tensile_eval_plans", "tensile_eval_plans_per_job", "tensile_eval_link", "tensile_apply_intervals", "tensile_score_candidates",
                 "tensile_score_recompute",
                 "tensile_greedy_plan", "tensile_validate_plans", "tensile_tas_info", "tensile_tas_base_timeline", "tensile_tas_free",
                 "tensile_version"):
        assert callable(getattr(binding, name))


def test_version_and_error_string(lib):
    lib.tensile_last_error.restype = ctypes.c_char_p
    assert lib.tensile_version() >= 100
    assert isinstance(lib.tensile_last_error(), bytes)


def _load(**kw):
    import paper_2105_13336_amd as P
    base = dict(T=8, size_bytes=[5, 7], alloc_step=[0, 1], free_step=[6, 7], access_offsets=[0, 1, 2],
                access_steps=[6, 7])
    base.update(kw)
    return P.tensile_tas_load(**base)


@pytest.mark.parametrize("kw,code", [
    (dict(T=0), -1),                                         # no steps
    (dict(size_bytes=[5, 0]), -1),                           # empty tensor
    (dict(alloc_step=[0, 8]), -2),                           # allocation outside the horizon
    (dict(free_step=[6, 6]), -2),                            # free step is not the last access
    (dict(access_steps=[6, 1]), -2),                         # access not after the allocation
    (dict(access_steps=[6, 8]), -2),                         # access outside the horizon
    (dict(access_offsets=[0, 1, 0]), -1),                    # offsets not monotone
    (dict(job_id=[0, 3], J=2), -2),                          # job outside [0, J)
    (dict(step_ns=[1] * 8, link_bytes_per_us=0), -1),        # timing without a link speed
    (dict(step_ns=[1, 1, 1, 0, 1, 1, 1, 1], link_bytes_per_us=10), -1),   # non-positive latency
    (dict(base_bytes=-1), -1),
])
def test_tas_load_rejects_bad_descriptions(kw, code):
    import paper_2105_13336_amd as P
    with pytest.raises(P.TensileError) as e:
        _load(**kw)
    assert e.value.code == code and "tas_load" in str(e.value)


def test_null_arguments_are_errors_not_crashes(lib):
    lib.tensile_last_error.restype = ctypes.c_char_p
    assert lib.tensile_tas_load(None, None) == -1
    out = ctypes.c_void_p()
    assert lib.tensile_tas_load(None, ctypes.byref(out)) == -1 and out.value is None
    assert lib.tensile_tas_info(None, None, None) == -1
    assert lib.tensile_eval_plans(None, None, None, None, None, None, None) == -1
    assert lib.tensile_score_candidates(None, None, None, None, None, None, None, None, None) == -1
    assert lib.tensile_score_recompute(None, None, None, None, None, None, None, None, None) == -1
    assert lib.tensile_eval_plans_per_job(None, None, None, None, None, None) == -1
    assert lib.tensile_eval_link(None, None, 0, None, None, None, None, None) == -1
    assert lib.tensile_apply_intervals(None, 0, None, None, None, None, None, None, None, None) == -1
    assert lib.tensile_validate_plans(None, None, None, None) == -1
    assert lib.tensile_greedy_plan(None, ctypes.c_int64(0), None, 0, 0, None, None, None, None, None, None, None) == -1
    assert b"NULL" in lib.tensile_last_error()
    assert lib.tensile_eval_plans_static(None, None, None, None, None, None, None) == -1
    assert lib.tensile_eval_score_plans(None, None, None, None, None, None, None, None, None, None) == -1
    lib.tensile_tas_free.restype = None
    lib.tensile_tas_free(None)     # allowed


def test_tuning_knobs(lib):
    lib.tensile_tuning_set.argtypes = [ctypes.c_char_p, ctypes.c_int]
    for name in (b"eval_threads", b"eval_segments", b"eval_binned", b"eval_persistent", b"eval_slots", b"eval_r",
                 b"score_blocks", b"link_packed", b"step_fused", b"eval_nt", b"eval_seg_steps"):
        assert lib.tensile_tuning_set(name, 1) == 0
    assert lib.tensile_tuning_set(b"no_such_knob", 1) == -1 and lib.tensile_tuning_set(None, 1) == -1
    lib.tensile_tuning_reset.restype = None
    lib.tensile_tuning_reset()
