"""Thin ctypes binding of libtensile.so: argument marshalling only.

Function names are those of ``include/tensile.h``.  Device buffers are torch
tensors on the GPU (torch is used for device memory and streams, nothing
else); every step of the computation runs in the library's HIP kernels.  There
is no CPU fallback: if the library is missing, importing fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np
import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libtensile.so")

TENSILE_OK, TENSILE_E_INVAL, TENSILE_E_RANGE, TENSILE_E_NOMEM, TENSILE_E_HIP, TENSILE_E_CAPACITY = 0, -1, -2, -3, -4, -5

EXPORTS = ["tensile_last_error", "tensile_version", "tensile_tas_load", "tensile_tas_free", "tensile_tas_info",
           "tensile_tas_update_latencies",
           "tensile_tas_base_timeline", "tensile_eval_plans", "tensile_eval_plans_per_job", "tensile_eval_link", "tensile_apply_intervals", "tensile_score_candidates", "tensile_score_recompute",
           "tensile_validate_plans",
           "tensile_greedy_plan", "tensile_eval_plans_static", "tensile_eval_score_plans", "tensile_tuning_set", "tensile_tuning_reset"]


class TensileError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"tensile error {code}: {message}")
        self.code = code


class _TasDesc(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int32), ("N", ctypes.c_int32), ("J", ctypes.c_int32),
                ("size_bytes", ctypes.c_void_p), ("alloc_step", ctypes.c_void_p), ("free_step", ctypes.c_void_p),
                ("access_offsets", ctypes.c_void_p), ("access_steps", ctypes.c_void_p), ("job_id", ctypes.c_void_p),
                ("step_ns", ctypes.c_void_p), ("base_bytes", ctypes.c_int64), ("link_bytes_per_us", ctypes.c_int64)]


class _Plans(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("n_intervals", ctypes.c_int64), ("plan_offsets", ctypes.c_void_p),
                ("iv_tensor", ctypes.c_void_p), ("iv_out", ctypes.c_void_p), ("iv_in", ctypes.c_void_p),
                ("iv_kind", ctypes.c_void_p)]


class _GreedyOpts(ctypes.Structure):
    _fields_ = [("max_iters", ctypes.c_int32), ("min_iters", ctypes.c_int32), ("stop_at_budget", ctypes.c_int32),
                ("msr_num", ctypes.c_void_p), ("msr_den", ctypes.c_int64), ("recompute", ctypes.c_int32)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2105_13336_amd.build` "
                          "(there is no CPU fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    lib.tensile_last_error.restype = ctypes.c_char_p
    lib.tensile_tas_free.restype = None
    lib.tensile_tas_free.argtypes = [ctypes.c_void_p]
    lib.tensile_tuning_reset.restype = None
    lib.tensile_tuning_set.argtypes = [ctypes.c_char_p, ctypes.c_int]
    return lib


_lib = _load()


def _check(rc: int) -> None:
    if rc != TENSILE_OK:
        raise TensileError(rc, _lib.tensile_last_error().decode())


def _np(a, dtype):
    if a is None:
        return None
    return np.ascontiguousarray(a, dtype=dtype)


def _hp(a: Optional[np.ndarray]):
    return None if a is None else ctypes.c_void_p(a.ctypes.data)


def _dp(t: Optional[torch.Tensor], dtype, n: int, name: str):
    if t is None:
        return None
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous() or t.numel() < n:
        raise TensileError(TENSILE_E_INVAL, f"{name}: need a contiguous CUDA tensor of {dtype} with >= {n} elements")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def tensile_version() -> int:
    return _lib.tensile_version()


class TasHandle:
    """Owner of a ``tensile_tas*``; freed on ``close()`` / garbage collection."""

    def __init__(self, ptr: int, T: int, N: int, J: int):
        self._ptr, self.T, self.N, self.J = ptr, T, N, J

    @property
    def ptr(self) -> ctypes.c_void_p:
        if not self._ptr:
            raise TensileError(TENSILE_E_INVAL, "TAS handle already freed")
        return ctypes.c_void_p(self._ptr)

    def close(self) -> None:
        if self._ptr:
            _lib.tensile_tas_free(ctypes.c_void_p(self._ptr))
            self._ptr = 0

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def tensile_tas_load(T, size_bytes, alloc_step, free_step, access_offsets, access_steps, job_id=None, step_ns=None,
                     base_bytes: int = 0, link_bytes_per_us: int = 0, J: int = 1, N: Optional[int] = None) -> TasHandle:
    size = _np(size_bytes, np.int64); alloc = _np(alloc_step, np.int32); free = _np(free_step, np.int32)
    offs = _np(access_offsets, np.int64); acc = _np(access_steps, np.int32)
    job = _np(job_id, np.int32); sn = _np(step_ns, np.int64)
    n = int(size.shape[0]) if N is None else int(N)
    desc = _TasDesc(int(T), n, int(J), _hp(size), _hp(alloc), _hp(free), _hp(offs), _hp(acc), _hp(job), _hp(sn),
                    int(base_bytes), int(link_bytes_per_us))
    out = ctypes.c_void_p()
    _check(_lib.tensile_tas_load(ctypes.byref(desc), ctypes.byref(out)))
    return TasHandle(out.value, int(T), n, int(J))


def tas_load(tas) -> TasHandle:
    """Load from an object with the attributes of the description (e.g. workloads.TAS)."""
    return tensile_tas_load(tas.T, tas.size_bytes, tas.alloc_step, tas.free_step, tas.access_offsets, tas.access_steps,
                            tas.job_id, tas.step_ns, tas.base_bytes, tas.link_bytes_per_us, tas.J)


def tensile_tas_free(h: TasHandle) -> None:
    h.close()


def tensile_tas_update_latencies(h: TasHandle, step_ns, link_bytes_per_us: int = 0) -> None:
    """New operator latencies (HOST array of T values, or None) and link speed for a loaded sequence."""
    sn = None if step_ns is None else np.ascontiguousarray(step_ns, dtype=np.int64)
    if sn is not None and sn.shape[0] != h.T:
        raise TensileError(TENSILE_E_INVAL, "step_ns must have T entries")
    _check(_lib.tensile_tas_update_latencies(h.ptr, _hp(sn), ctypes.c_int64(int(link_bytes_per_us))))


def tensile_tas_info(h: TasHandle):
    peak, arg = ctypes.c_int64(), ctypes.c_int32()
    _check(_lib.tensile_tas_info(h.ptr, ctypes.byref(peak), ctypes.byref(arg)))
    return peak.value, arg.value


def tensile_tas_base_timeline(h: TasHandle) -> np.ndarray:
    out = np.empty(h.T, dtype=np.int64)
    _check(_lib.tensile_tas_base_timeline(h.ptr, _hp(out)))
    return out


class DevicePlans:
    """A batch of plans resident on the GPU (torch tensors), CSR layout of ``tensile_plans``."""

    def __init__(self, plan_offsets: torch.Tensor, iv_tensor: torch.Tensor, iv_out: torch.Tensor, iv_in: torch.Tensor,
                 iv_kind: Optional[torch.Tensor] = None):
        self.B = int(plan_offsets.numel()) - 1
        self.n_intervals = int(iv_tensor.numel())
        self.plan_offsets, self.iv_tensor, self.iv_out, self.iv_in, self.iv_kind = plan_offsets, iv_tensor, iv_out, iv_in, iv_kind

    @classmethod
    def from_numpy(cls, plan_offsets, iv_tensor, iv_out, iv_in, iv_kind=None, device="cuda") -> "DevicePlans":
        up = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a, dtype=dt)).to(device)
        return cls(up(plan_offsets, np.int64), up(iv_tensor, np.int32), up(iv_out, np.int32), up(iv_in, np.int32),
                   None if iv_kind is None else up(iv_kind, np.uint8))

    def struct(self) -> _Plans:
        K = self.n_intervals
        return _Plans(self.B, K, _dp(self.plan_offsets, torch.int64, self.B + 1, "plan_offsets"),
                      _dp(self.iv_tensor, torch.int32, K, "iv_tensor"), _dp(self.iv_out, torch.int32, K, "iv_out"),
                      _dp(self.iv_in, torch.int32, K, "iv_in"), _dp(self.iv_kind, torch.uint8, K, "iv_kind"))


def tensile_eval_plans(h: TasHandle, plans: DevicePlans, resident: Optional[torch.Tensor], peak: torch.Tensor,
                       argmax: torch.Tensor, min_resident: Optional[torch.Tensor] = None, stream=None) -> None:
    B = plans.B
    st = plans.struct()
    _check(_lib.tensile_eval_plans(h.ptr, ctypes.byref(st), _dp(resident, torch.int64, B * h.T, "resident"),
                                   _dp(peak, torch.int64, B, "peak"), _dp(argmax, torch.int32, B, "argmax"),
                                   _dp(min_resident, torch.int64, B, "min_resident"), _stream(stream)))


def tensile_eval_plans_static(h: TasHandle, plans: DevicePlans, resident: Optional[torch.Tensor], peak: torch.Tensor,
                              argmax: torch.Tensor, min_resident: Optional[torch.Tensor] = None, stream=None) -> None:
    """tensile_eval_plans with its scratch in the library's preallocated device array (allocates nothing)."""
    B = plans.B
    st = plans.struct()
    _check(_lib.tensile_eval_plans_static(h.ptr, ctypes.byref(st), _dp(resident, torch.int64, B * h.T, "resident"),
                                          _dp(peak, torch.int64, B, "peak"), _dp(argmax, torch.int32, B, "argmax"),
                                          _dp(min_resident, torch.int64, B, "min_resident"), _stream(stream)))


def tensile_tuning_set(knob: str, value: int) -> None:
    _check(_lib.tensile_tuning_set(knob.encode(), ctypes.c_int(int(value))))


def tensile_tuning_reset() -> None:
    _lib.tensile_tuning_reset()


def tensile_eval_plans_per_job(h: TasHandle, plans: DevicePlans, job_peak: torch.Tensor,
                               job_argmax: Optional[torch.Tensor] = None, sum_peak: Optional[torch.Tensor] = None,
                               stream=None) -> None:
    """job_peak / job_argmax: [J, B] (job-major), sum_peak: [B]"""
    B, J = plans.B, h.J
    st = plans.struct()
    _check(_lib.tensile_eval_plans_per_job(h.ptr, ctypes.byref(st), _dp(job_peak, torch.int64, J * B, "job_peak"),
                                           _dp(job_argmax, torch.int32, J * B, "job_argmax"),
                                           _dp(sum_peak, torch.int64, B, "sum_peak"), _stream(stream)))


def tensile_apply_intervals(h: TasHandle, tensor: torch.Tensor, out_step: torch.Tensor, in_step: torch.Tensor,
                            resident: torch.Tensor, peak: torch.Tensor, argmax: torch.Tensor,
                            min_resident: Optional[torch.Tensor] = None, stream=None) -> None:
    """tensor / out_step / in_step: [B] int32 (one new interval per plan), resident: [B, T] int64 in/out"""
    B = int(tensor.numel())
    _check(_lib.tensile_apply_intervals(h.ptr, ctypes.c_int32(B), _dp(tensor, torch.int32, B, "tensor"),
                                        _dp(out_step, torch.int32, B, "out_step"), _dp(in_step, torch.int32, B, "in_step"),
                                        _dp(resident, torch.int64, B * h.T, "resident"), _dp(peak, torch.int64, B, "peak"),
                                        _dp(argmax, torch.int32, B, "argmax"), _dp(min_resident, torch.int64, B, "min_resident"),
                                        _stream(stream)))


def tensile_eval_link(h: TasHandle, plans: DevicePlans, link_peak: torch.Tensor, link: Optional[torch.Tensor] = None,
                      link_argmax: Optional[torch.Tensor] = None, overbooked: Optional[torch.Tensor] = None,
                      reuse_host_copies: bool = False, stream=None) -> None:
    """link: [B, T] int32, link_peak / link_argmax / overbooked: [B] int32"""
    B = plans.B
    st = plans.struct()
    _check(_lib.tensile_eval_link(h.ptr, ctypes.byref(st), ctypes.c_int32(1 if reuse_host_copies else 0),
                                  _dp(link, torch.int32, B * h.T, "link"), _dp(link_peak, torch.int32, B, "link_peak"),
                                  _dp(link_argmax, torch.int32, B, "link_argmax"), _dp(overbooked, torch.int32, B, "overbooked"),
                                  _stream(stream)))


def tensile_score_candidates(h: TasHandle, plans: DevicePlans, resident: torch.Tensor, peak: torch.Tensor,
                             argmax: torch.Tensor, score: torch.Tensor, win_out: Optional[torch.Tensor] = None,
                             win_in: Optional[torch.Tensor] = None, stream=None) -> None:
    B, N = plans.B, h.N
    st = plans.struct()
    _check(_lib.tensile_score_candidates(h.ptr, ctypes.byref(st), _dp(resident, torch.int64, B * h.T, "resident"),
                                         _dp(peak, torch.int64, B, "peak"), _dp(argmax, torch.int32, B, "argmax"),
                                         _dp(score, torch.int64, B * N, "score"), _dp(win_out, torch.int32, B * N, "win_out"),
                                         _dp(win_in, torch.int32, B * N, "win_in"), _stream(stream)))


def tensile_eval_score_plans(h: TasHandle, plans: DevicePlans, resident: torch.Tensor, peak: torch.Tensor, argmax: torch.Tensor,
                             min_resident: Optional[torch.Tensor], score: torch.Tensor, win_out: Optional[torch.Tensor] = None,
                             win_in: Optional[torch.Tensor] = None, stream=None) -> None:
    """tensile_eval_plans followed by tensile_score_candidates on the same batch, in one call (one kernel when possible)."""
    B, N = plans.B, h.N
    st = plans.struct()
    _check(_lib.tensile_eval_score_plans(h.ptr, ctypes.byref(st), _dp(resident, torch.int64, B * h.T, "resident"),
                                         _dp(peak, torch.int64, B, "peak"), _dp(argmax, torch.int32, B, "argmax"),
                                         _dp(min_resident, torch.int64, B, "min_resident"),
                                         _dp(score, torch.int64, B * N, "score"), _dp(win_out, torch.int32, B * N, "win_out"),
                                         _dp(win_in, torch.int32, B * N, "win_in"), _stream(stream)))


def tensile_score_recompute(h: TasHandle, plans: DevicePlans, resident: torch.Tensor, peak: torch.Tensor,
                             argmax: torch.Tensor, score: torch.Tensor, win_out: Optional[torch.Tensor] = None,
                             win_in: Optional[torch.Tensor] = None, stream=None) -> None:
    B, N = plans.B, h.N
    st = plans.struct()
    _check(_lib.tensile_score_recompute(h.ptr, ctypes.byref(st), _dp(resident, torch.int64, B * h.T, "resident"),
                                         _dp(peak, torch.int64, B, "peak"), _dp(argmax, torch.int32, B, "argmax"),
                                         _dp(score, torch.int64, B * N, "score"), _dp(win_out, torch.int32, B * N, "win_out"),
                                         _dp(win_in, torch.int32, B * N, "win_in"), _stream(stream)))


def tensile_validate_plans(h: TasHandle, plans: DevicePlans):
    """-> (index of the first invalid interval or -1, reason code)"""
    bad, why = ctypes.c_int64(), ctypes.c_int32()
    st = plans.struct()
    _check(_lib.tensile_validate_plans(h.ptr, ctypes.byref(st), ctypes.byref(bad), ctypes.byref(why)))
    return bad.value, why.value


def tensile_greedy_plan(h: TasHandle, budget_bytes: int = 0, max_iters: int = 0, min_iters: int = 100,
                        stop_at_budget: bool = False, msr_num=None, msr_den: int = 1, capacity: Optional[int] = None,
                        initial=None, recompute: bool = False) -> dict:
    """-> dict(iv_tensor, iv_out, iv_in, iv_kind, peak_trace, final_peak, n_initial)"""
    n0 = 0 if initial is None else len(initial[0])
    cap = int(capacity) if capacity is not None else n0 + (max_iters if max_iters > 0 else 1 << 20)
    t = np.zeros(max(cap, 1), dtype=np.int32); o = np.zeros_like(t); r = np.zeros_like(t)
    k = np.zeros(max(cap, 1), dtype=np.uint8)
    if n0:
        t[:n0], o[:n0], r[:n0], k[:n0] = initial
    trace = np.zeros(cap - n0 + 1, dtype=np.int64)
    num = _np(msr_num, np.int64)
    if num is not None and num.shape != (h.J,):
        raise TensileError(TENSILE_E_INVAL, f"msr_num: need one entry per job ({h.J})")
    opts = _GreedyOpts(int(max_iters), int(min_iters), int(bool(stop_at_budget)), _hp(num), int(msr_den), int(bool(recompute)))
    n, fp = ctypes.c_int32(), ctypes.c_int64()
    _check(_lib.tensile_greedy_plan(h.ptr, ctypes.c_int64(int(budget_bytes)), ctypes.byref(opts), ctypes.c_int32(cap),
                                    ctypes.c_int32(n0), _hp(t), _hp(o), _hp(r), _hp(k), ctypes.byref(n), _hp(trace),
                                    ctypes.byref(fp)))
    m = n.value
    return dict(iv_tensor=t[:m].copy(), iv_out=o[:m].copy(), iv_in=r[:m].copy(), iv_kind=k[:m].copy(),
                peak_trace=trace[:m - n0 + 1].copy(), final_peak=fp.value, n_initial=n0)
