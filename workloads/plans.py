"""Batches of candidate plans in CSR form, and the seeded generator for them.

A plan is a set of intervals (tensor, out, in, kind): the tensor is not resident
during steps out+1 .. in-1 (kind 0 = swap, 1 = recompute).  The fast generator
is ``plangen.c`` (built on first use with gcc); ``make_plans_numpy`` is the same
recipe written with ``prng.py`` and is used to cross-check it on small cases.

No arithmetic of the scheduling method lives here.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

from . import prng
from .tas import TAS, hash64

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


@dataclass
class Plans:
    B: int
    plan_offsets: np.ndarray   # int64 [B+1]
    iv_tensor: np.ndarray      # int32 [K]
    iv_out: np.ndarray         # int32 [K]
    iv_in: np.ndarray          # int32 [K]
    iv_kind: np.ndarray        # uint8 [K]

    @property
    def n_intervals(self) -> int:
        return int(self.iv_tensor.shape[0])

    def plan(self, b: int):
        a, e = int(self.plan_offsets[b]), int(self.plan_offsets[b + 1])
        return self.iv_tensor[a:e], self.iv_out[a:e], self.iv_in[a:e], self.iv_kind[a:e]

    def select(self, rows) -> "Plans":
        """The sub-batch made of the given plan rows, in that order."""
        rows = np.asarray(rows, dtype=np.int64)
        lens = self.plan_offsets[rows + 1] - self.plan_offsets[rows]
        offs = np.zeros(rows.shape[0] + 1, dtype=np.int64)
        np.cumsum(lens, out=offs[1:])
        idx = np.concatenate([np.arange(self.plan_offsets[r], self.plan_offsets[r + 1]) for r in rows]) \
            if rows.size else np.zeros(0, dtype=np.int64)
        idx = idx.astype(np.int64)
        return Plans(int(rows.shape[0]), offs, self.iv_tensor[idx], self.iv_out[idx], self.iv_in[idx], self.iv_kind[idx])


def plans_from_lists(plans) -> Plans:
    """``plans`` is a list (one entry per plan) of lists of (tensor, out, in[, kind])."""
    offs = np.zeros(len(plans) + 1, dtype=np.int64)
    t, o, r, k = [], [], [], []
    for b, pl in enumerate(plans):
        offs[b + 1] = offs[b] + len(pl)
        for iv in pl:
            t.append(iv[0]); o.append(iv[1]); r.append(iv[2]); k.append(iv[3] if len(iv) > 3 else 0)
    return Plans(len(plans), offs, np.array(t, dtype=np.int32).reshape(-1), np.array(o, dtype=np.int32).reshape(-1),
                 np.array(r, dtype=np.int32).reshape(-1), np.array(k, dtype=np.uint8).reshape(-1))


def plans_hash(pl: Plans) -> int:
    return hash64([pl.plan_offsets, pl.iv_tensor, pl.iv_out, pl.iv_in, pl.iv_kind])


def eligible_gaps(tas: TAS):
    """CSR over tensors of the gaps (p_g, p_{g+1}) between consecutive touch
    points that are at least two steps long."""
    N = tas.N
    cnt = np.diff(tas.access_offsets)
    # touch array: alloc followed by accesses, per tensor
    toff = tas.access_offsets + np.arange(N + 1, dtype=np.int64)
    touch = np.empty(int(toff[N]), dtype=np.int64)
    touch[toff[:-1]] = tas.alloc_step
    mask = np.ones(touch.shape[0], dtype=bool)
    mask[toff[:-1]] = False
    touch[mask] = tas.access_steps
    owner = np.repeat(np.arange(N, dtype=np.int64), cnt + 1)
    is_last = np.zeros(touch.shape[0], dtype=bool)
    is_last[toff[1:] - 1] = True
    p = touch[:-1][~is_last[:-1]] if touch.shape[0] > 1 else np.zeros(0, dtype=np.int64)
    q = touch[1:][~is_last[:-1]] if touch.shape[0] > 1 else np.zeros(0, dtype=np.int64)
    own = owner[:-1][~is_last[:-1]] if touch.shape[0] > 1 else np.zeros(0, dtype=np.int64)
    keep = (q - p) >= 2
    p, q, own = p[keep], q[keep], own[keep]
    eoff = np.zeros(N + 1, dtype=np.int64)
    np.cumsum(np.bincount(own, minlength=N), out=eoff[1:])
    return eoff, p.astype(np.int32), q.astype(np.int32)


def _lib():
    global _LIB
    if _LIB is None:
        src, so = os.path.join(_HERE, "plangen.c"), os.path.join(_HERE, "libplangen.so")
        if not os.path.exists(so) or os.path.getmtime(so) < os.path.getmtime(src):
            build()
        _LIB = ctypes.CDLL(so)
        _LIB.plangen_u64.restype = ctypes.c_uint64
        _LIB.plangen_u64.argtypes = [ctypes.c_uint64] * 3
    return _LIB


def build() -> str:
    """Compile plangen.c next to its source."""
    src, so = os.path.join(_HERE, "plangen.c"), os.path.join(_HERE, "libplangen.so")
    subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-shared", "-fPIC", "-o", so, src])
    return so


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def make_plans(tas: TAS, B: int, seed: int, p_swap: float = 0.3, b0: int = 0) -> Plans:
    """Plans b0 .. b0+B-1 of the batch defined by (tas, seed, p_swap)."""
    lib = _lib()
    eoff, ep, eq = eligible_gaps(tas)
    thr = int(p_swap * (1 << 53))
    counts = np.zeros(B, dtype=np.int64)
    u64, i64 = ctypes.c_uint64, ctypes.c_int64
    lib.plangen_count(u64(seed), i64(b0), i64(B), i64(tas.N), _p(eoff), u64(thr), _p(counts))
    offs = np.zeros(B + 1, dtype=np.int64)
    np.cumsum(counts, out=offs[1:])
    K = int(offs[B])
    t = np.empty(K, dtype=np.int32); o = np.empty(K, dtype=np.int32); r = np.empty(K, dtype=np.int32)
    k = np.empty(K, dtype=np.uint8)
    lib.plangen_fill(u64(seed), i64(b0), i64(B), i64(tas.N), _p(eoff), _p(ep), _p(eq), u64(thr), _p(offs),
                     _p(t), _p(o), _p(r), _p(k))
    return Plans(B, offs, t, o, r, k)


def make_plans_numpy(tas: TAS, B: int, seed: int, p_swap: float = 0.3, b0: int = 0) -> Plans:
    """Same recipe with prng.py (slow; for cross-checks on small batches)."""
    eoff, ep, eq = eligible_gaps(tas)
    N = tas.N
    thr = np.uint64(int(p_swap * (1 << 53)))
    ne = np.diff(eoff)
    plans = []
    for b in range(b0, b0 + B):
        idx = np.uint64(b) * np.uint64(N) + np.arange(N, dtype=np.uint64)
        sel = ((prng.u64(seed, 1, idx) >> np.uint64(11)) < thr) & (ne > 0)
        ii = np.nonzero(sel)[0]
        g = eoff[ii] + (prng.u64(seed, 2, idx[ii]) % ne[ii].astype(np.uint64)).astype(np.int64)
        p, q = ep[g].astype(np.int64), eq[g].astype(np.int64)
        o = p + (prng.u64(seed, 3, idx[ii]) % (q - 2 - p + 1).astype(np.uint64)).astype(np.int64)
        r = o + 2 + (prng.u64(seed, 4, idx[ii]) % (q - (o + 2) + 1).astype(np.uint64)).astype(np.int64)
        plans.append(list(zip(ii.tolist(), o.tolist(), r.tolist())))
    return plans_from_lists(plans)
