"""TEST INFRASTRUCTURE - ctypes front end of the CPU oracle (tensile_oracle.c).

Only tests, the smoke check and the benchmark's cpu_baseline leg import this.
It imports nothing from the product package and the product imports nothing
from here.  The C file is compiled with gcc on first use (``build()``).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tensile_oracle.c")
_SO = os.path.join(_HERE, "libtensile_oracle.so")
_LIB = None


def build() -> str:
    subprocess.check_call(["gcc", "-O2", "-std=c11", "-Wall", "-shared", "-fPIC", "-o", _SO, _SRC])
    return _SO


def _lib():
    global _LIB
    if _LIB is None:
        if not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
            build()
        _LIB = ctypes.CDLL(_SO)
    return _LIB


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _chk(rc: int, what: str) -> None:
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


i32, i64 = ctypes.c_int32, ctypes.c_int64


def base_timeline(tas) -> np.ndarray:
    MF0 = np.empty(tas.T, dtype=np.int64)
    _chk(_lib().oracle_base_timeline(i32(tas.T), i32(tas.N), _p(tas.size_bytes), _p(tas.alloc_step),
                                     _p(tas.free_step), i64(tas.base_bytes), _p(MF0)), "base_timeline")
    return MF0


def eval_plans(tas, plans, want_resident: bool = True, MF0: Optional[np.ndarray] = None):
    """-> (resident [B,T] or None, peak [B], argmax [B], min_resident [B])"""
    if MF0 is None:
        MF0 = base_timeline(tas)
    B = plans.B
    resident = np.empty((B, tas.T), dtype=np.int64) if want_resident else None
    peak = np.empty(B, dtype=np.int64); arg = np.empty(B, dtype=np.int32); mn = np.empty(B, dtype=np.int64)
    _chk(_lib().oracle_eval(i32(tas.T), i32(tas.N), _p(tas.size_bytes), _p(MF0), i64(B), _p(plans.plan_offsets),
                            i64(plans.n_intervals), _p(plans.iv_tensor), _p(plans.iv_out), _p(plans.iv_in),
                            _p(resident), _p(peak), _p(arg), _p(mn)), "eval")
    return resident, peak, arg, mn


def eval_per_job(tas, plans):
    """-> (job_peak [J,B], job_argmax [J,B], sum_peak [B] = base_bytes + sum over jobs of their peaks)"""
    B, J = plans.B, int(tas.J)
    jp = np.empty((J, B), dtype=np.int64); ja = np.empty((J, B), dtype=np.int32)
    job = np.ascontiguousarray(tas.job_id, dtype=np.int32)
    _chk(_lib().oracle_eval_per_job(i32(tas.T), i32(tas.N), i32(J), _p(tas.size_bytes), _p(tas.alloc_step),
                                    _p(tas.free_step), _p(job), i64(B), _p(plans.plan_offsets), i64(plans.n_intervals),
                                    _p(plans.iv_tensor), _p(plans.iv_out), _p(plans.iv_in), _p(jp), _p(ja)), "eval_per_job")
    return jp, ja, jp.sum(axis=0) + int(tas.base_bytes)


def apply_intervals(tas, tensor, out, in_, resident: np.ndarray):
    """One more interval per plan on existing rows (in place) -> (peak [B], argmax [B], min [B])"""
    B = resident.shape[0]
    assert resident.dtype == np.int64 and resident.flags.c_contiguous and resident.shape == (B, tas.T)
    t = np.ascontiguousarray(tensor, dtype=np.int32); o = np.ascontiguousarray(out, dtype=np.int32)
    r = np.ascontiguousarray(in_, dtype=np.int32)
    pk = np.empty(B, dtype=np.int64); arg = np.empty(B, dtype=np.int32); mn = np.empty(B, dtype=np.int64)
    _chk(_lib().oracle_apply_intervals(i32(tas.T), i32(tas.N), _p(tas.size_bytes), i64(B), _p(t), _p(o), _p(r),
                                       _p(resident), _p(pk), _p(arg), _p(mn)), "apply_intervals")
    return pk, arg, mn


def link_occupancy(tas, plans, reuse: bool = False, want_rows: bool = True):
    """-> (link [B,T] int32 or None, peak [B], argmax [B], overbooked [B]): steps of the host link that the
    plans' transfers occupy (canonical placement, see oracle_link_occupancy)"""
    B, T = plans.B, tas.T
    rows = np.empty((B, T), dtype=np.int32) if want_rows else None
    pk = np.empty(B, dtype=np.int32); arg = np.empty(B, dtype=np.int32); over = np.empty(B, dtype=np.int32)
    kind = np.ascontiguousarray(plans.iv_kind, dtype=np.uint8)
    _chk(_lib().oracle_link_occupancy(i32(T), i32(tas.N), _p(tas.size_bytes), _p(tas.step_ns), i64(tas.link_bytes_per_us),
                                      i64(B), _p(plans.plan_offsets), i64(plans.n_intervals), _p(plans.iv_tensor),
                                      _p(plans.iv_out), _p(plans.iv_in), _p(kind), i32(1 if reuse else 0),
                                      _p(rows), _p(pk), _p(arg), _p(over)), "link_occupancy")
    return rows, pk, arg, over


def times(tas):
    """-> (C [T+1], x [N]) cumulative step time and per-tensor transfer time, ns"""
    C = np.empty(tas.T + 1, dtype=np.int64); x = np.empty(tas.N, dtype=np.int64)
    _chk(_lib().oracle_times(i32(tas.T), i32(tas.N), _p(tas.size_bytes), _p(tas.step_ns),
                             i64(tas.link_bytes_per_us), _p(C), _p(x)), "times")
    return C, x


def score_plans(tas, plans, resident: np.ndarray, peak: np.ndarray, argmax: np.ndarray, rows: Optional[Sequence[int]] = None):
    """Scores of the plans in ``rows`` (default all): -> score [R,N], win_out [R,N], win_in [R,N]"""
    C, x = times(tas)
    rows = list(range(plans.B)) if rows is None else list(rows)
    R, N = len(rows), tas.N
    score = np.zeros((R, N), dtype=np.int64); wo = np.zeros((R, N), dtype=np.int32); wi = np.zeros((R, N), dtype=np.int32)
    lib = _lib()
    for n, b in enumerate(rows):
        a, e = int(plans.plan_offsets[b]), int(plans.plan_offsets[b + 1])
        t, o, r = (np.ascontiguousarray(v[a:e]) for v in (plans.iv_tensor, plans.iv_out, plans.iv_in))
        MF = np.ascontiguousarray(resident[b])
        _chk(lib.oracle_score_plan(i32(tas.T), i32(N), _p(tas.size_bytes), _p(tas.alloc_step), _p(tas.access_offsets),
                                   _p(tas.access_steps), _p(C), _p(x), i64(e - a), _p(t), _p(o), _p(r), _p(MF),
                                   i64(int(peak[b])), i32(int(argmax[b])), _p(score[n]), _p(wo[n]), _p(wi[n])), "score")
    return score, wo, wi


def score_recompute_plans(tas, plans, resident: np.ndarray, peak: np.ndarray, argmax: np.ndarray,
                          rows: Optional[Sequence[int]] = None):
    """Recomputation savings of the plans in ``rows`` (default all): -> score [R,N], win_out [R,N], win_in [R,N]"""
    rows = list(range(plans.B)) if rows is None else list(rows)
    R, N = len(rows), tas.N
    score = np.zeros((R, N), dtype=np.int64); wo = np.zeros((R, N), dtype=np.int32); wi = np.zeros((R, N), dtype=np.int32)
    lib = _lib()
    for n, b in enumerate(rows):
        a, e = int(plans.plan_offsets[b]), int(plans.plan_offsets[b + 1])
        t, o, r = (np.ascontiguousarray(v[a:e]) for v in (plans.iv_tensor, plans.iv_out, plans.iv_in))
        MF = np.ascontiguousarray(resident[b])
        _chk(lib.oracle_score_recompute_plan(i32(tas.T), i32(N), _p(tas.size_bytes), _p(tas.alloc_step),
                                             _p(tas.access_offsets), _p(tas.access_steps), i64(e - a), _p(t), _p(o), _p(r),
                                             _p(MF), i64(int(peak[b])), i32(int(argmax[b])), _p(score[n]), _p(wo[n]),
                                             _p(wi[n])), "score_recompute")
    return score, wo, wi


class _GreedyOpts(ctypes.Structure):
    _fields_ = [("max_iters", i32), ("min_iters", i32), ("stop_at_budget", i32), ("J", i32),
                ("job_id", ctypes.c_void_p), ("msr_num", ctypes.c_void_p), ("msr_den", i64), ("recompute", i32)]


def greedy(tas, budget: int, max_iters: int = 1 << 30, min_iters: int = 100, stop_at_budget: bool = False,
           msr_num: Optional[np.ndarray] = None, msr_den: int = 1, capacity: Optional[int] = None, initial=None,
           recompute: bool = False):
    """-> dict(iv_tensor, iv_out, iv_in, iv_kind, peak_trace, final_peak, xfer_out_start, xfer_in_start);
    ``initial`` = (iv_tensor, iv_out, iv_in, iv_kind) of a plan to extend."""
    n0 = 0 if initial is None else len(initial[0])
    if capacity is None:
        capacity = int(tas.access_steps.shape[0]) + n0
    cap = max(capacity, 1)
    t = np.zeros(cap, dtype=np.int32); o = np.zeros(cap, dtype=np.int32); r = np.zeros(cap, dtype=np.int32)
    k = np.zeros(cap, dtype=np.uint8); trace = np.zeros(cap + 1, dtype=np.int64)
    xo = np.full(cap, -1, dtype=np.int32); xi = np.full(cap, -1, dtype=np.int32)
    if n0:
        t[:n0], o[:n0], r[:n0], k[:n0] = initial
    n = i32(0); fp = i64(0)
    job = np.ascontiguousarray(tas.job_id, dtype=np.int32)
    num = None if msr_num is None else np.ascontiguousarray(msr_num, dtype=np.int64)
    opts = _GreedyOpts(min(max_iters, 1 << 30), min_iters, int(stop_at_budget), tas.J if num is not None else 0,
                       job.ctypes.data, None if num is None else num.ctypes.data, msr_den, int(recompute))
    _chk(_lib().oracle_greedy(i32(tas.T), i32(tas.N), _p(tas.size_bytes), _p(tas.alloc_step), _p(tas.free_step),
                              _p(tas.access_offsets), _p(tas.access_steps), _p(tas.step_ns), i64(tas.base_bytes),
                              i64(tas.link_bytes_per_us), i64(budget), ctypes.byref(opts), i32(capacity), i32(n0),
                              _p(t), _p(o), _p(r), _p(k), ctypes.byref(n), _p(trace), ctypes.byref(fp), _p(xo), _p(xi)),
         "greedy")
    m = n.value
    return dict(iv_tensor=t[:m].copy(), iv_out=o[:m].copy(), iv_in=r[:m].copy(), iv_kind=k[:m].copy(),
                peak_trace=trace[:m - n0 + 1].copy(), final_peak=fp.value, xfer_out_start=xo[:m].copy(),
                xfer_in_start=xi[:m].copy(), n_initial=n0)
