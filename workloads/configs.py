"""The five benchmark configurations: seeded synthetic TAS and plan batches.

They stand in for the workloads the paper measures (CNN training jobs, one to
several at a time): the traces below reproduce the structure such a job has —
forward, backward and optimizer phases, activations kept for the backward
sweep, Adam state, several jobs interleaved on one timeline — with tensor sizes
taken from the layer shapes, not the paper's op traces or latencies.

Seeds are ``SEED0 + config index``.  Nothing here evaluates a plan.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np

from . import models as M
from . import prng
from .plans import Plans, make_plans
from .tas import TAS, Trace, even_grid, merge_traces, tas_from_lists

SEED0 = 210513336
STEP_NS_LO, STEP_NS_HI = 50_000, 2_000_000
LINK_BYTES_PER_US = 64_000          # 64 GB/s host link


@dataclass
class Config:
    index: int
    name: str
    T: int
    B: int
    budget_pct: int
    timed: bool                     # has per-step compute times (transfer feasibility)
    p_swap: float = 0.3

    @property
    def seed(self) -> int:
        return SEED0 + self.index


CONFIGS = [
    Config(0, "c0-mlp", 200, 64, 60, False),
    Config(1, "c1-resnet50", 6_000, 4_096, 60, True),
    Config(2, "c2-bert-2iter", 24_000, 8_192, 50, True),
    Config(3, "c3-4jobs", 50_000, 16_384, 50, True),
    Config(4, "c4-stress", 1_000_000, 1_024, 40, True),
]


def _step_ns(cfg: Config, T: int) -> Optional[np.ndarray]:
    if not cfg.timed:
        return None
    return prng.randint(cfg.seed, 10, np.arange(T), STEP_NS_LO, STEP_NS_HI).astype(np.int64)


def _single_job(cfg: Config, shapes, iteration, iters: int, **kw) -> TAS:
    tr = Trace()
    ps = M.placeholder(tr, shapes)
    for it in range(iters):
        ps = iteration(tr, ps, it=it, **kw)
    M.finish(tr, ps)
    return merge_traces(cfg.T, [tr], [even_grid(tr.n_ops, cfg.T)], _step_ns(cfg, cfg.T), 0,
                        LINK_BYTES_PER_US if cfg.timed else 0)


def _poisson_steps(seed: int, stream: int, n_ops: int, start: int, T: int) -> np.ndarray:
    """Operator arrival times of one job: exponential gaps whose mean makes the
    job end near the horizon, floored to steps, forced strictly increasing and
    kept two steps clear of the end (room for the last in-place output)."""
    mean = (T - 2 - start) / n_ops
    assert mean >= 2.0
    u = prng.uniform01(seed, stream, np.arange(n_ops))
    arrive = start + np.cumsum(-np.log1p(-u) * mean)
    raw = np.floor(arrive).astype(np.int64)
    steps = np.empty(n_ops, dtype=np.int64)
    prev = start - 1
    for k in range(n_ops):
        s = max(prev + 1, int(raw[k]))
        s = min(s, T - 2 - (n_ops - 1 - k))
        steps[k] = s
        prev = s
    assert steps[0] >= start and np.all(np.diff(steps) > 0) and steps[-1] <= T - 2
    return steps


def _four_jobs(cfg: Config) -> TAS:
    jobs = [("mlp", M.mlp_shapes(), M.mlp_iteration, dict(batch=32), 20),
            ("resnet50", M.resnet50_shapes(), M.resnet50_iteration, dict(batch=64), 3),
            ("vgg16", M.vgg16_shapes(), M.vgg16_iteration, dict(batch=32), 6),
            ("bert", M.bert_shapes(), M.bert_iteration, dict(batch=16), 2)]
    traces, steps = [], []
    for j, (_, shapes, iteration, kw, iters) in enumerate(jobs):
        tr = Trace()
        ps = M.placeholder(tr, shapes)
        for it in range(iters):
            ps = iteration(tr, ps, it=it, **kw)
        M.finish(tr, ps)
        start = int(prng.randint(cfg.seed, 20, j, 0, 5000))
        traces.append(tr)
        steps.append(_poisson_steps(cfg.seed, 21 + j, tr.n_ops, start, cfg.T))
    return merge_traces(cfg.T, traces, steps, _step_ns(cfg, cfg.T), 0, LINK_BYTES_PER_US)


def _stress(cfg: Config, N: int = 200_000, n_jobs: int = 64) -> TAS:
    """Statistical TAS: log-normal sizes (median 1 MiB, sigma 2 in natural log,
    clamped to [256 B, 2 GiB], multiples of 256 B), 2-20 accesses per tensor,
    geometric gaps of mean 40 steps; tensor i belongs to job i mod n_jobs."""
    T, seed = cfg.T, cfg.seed
    i = np.arange(N)
    u1, u2 = prng.uniform01(seed, 30, i), prng.uniform01(seed, 31, i)
    z = np.sqrt(-2.0 * np.log1p(-u1)) * np.cos(2.0 * np.pi * u2)          # Box-Muller
    size = np.exp(np.log(float(1 << 20)) + 2.0 * z)
    size = np.clip(np.rint(size / 256.0), 1, (1 << 31) // 256).astype(np.int64) * 256
    k = prng.randint(seed, 32, i, 2, 20)
    kmax = 20
    ug = prng.uniform01(seed, 33, (i[:, None] * kmax + np.arange(kmax)[None, :]).reshape(-1)).reshape(N, kmax)
    gaps = 1 + np.floor(np.log1p(-ug) / np.log(1.0 - 1.0 / 40.0)).astype(np.int64)     # geometric on {1,2,..}, mean 40
    gaps = np.where(np.arange(kmax)[None, :] < k[:, None], gaps, 0)
    span = gaps.sum(axis=1)
    alloc = prng.randint(seed, 34, i, 0, T - 1 - span)
    acc = alloc[:, None] + np.cumsum(gaps, axis=1)
    order = np.lexsort((i, alloc))
    size, k, alloc, acc = size[order], k[order], alloc[order], acc[order]
    offs = np.zeros(N + 1, dtype=np.int64)
    np.cumsum(k, out=offs[1:])
    flat = acc[np.arange(kmax)[None, :] < k[:, None]]
    free = acc[np.arange(N), k - 1]
    return TAS(T=T, size_bytes=size, alloc_step=alloc.astype(np.int32), free_step=free.astype(np.int32),
               access_offsets=offs, access_steps=flat.astype(np.int32), job_id=(order % n_jobs).astype(np.int32),
               step_ns=_step_ns(cfg, T), base_bytes=0, link_bytes_per_us=LINK_BYTES_PER_US, J=n_jobs)


def make_tas(index: int) -> TAS:
    cfg = CONFIGS[index]
    if index == 0:
        tas = _single_job(cfg, M.mlp_shapes(), M.mlp_iteration, 1, batch=32)
    elif index == 1:
        tas = _single_job(cfg, M.resnet50_shapes(), M.resnet50_iteration, 1, batch=64)
    elif index == 2:
        tas = _single_job(cfg, M.bert_shapes(), M.bert_iteration, 2, batch=16)
    elif index == 3:
        tas = _four_jobs(cfg)
    elif index == 4:
        tas = _stress(cfg)
    else:
        raise IndexError(index)
    return tas


def make_config_plans(index: int, tas: TAS, B: Optional[int] = None, b0: int = 0) -> Plans:
    """The first ``B`` plans (default: all) of configuration ``index``, from plan ``b0``."""
    cfg = CONFIGS[index]
    return make_plans(tas, cfg.B if B is None else B, cfg.seed, cfg.p_swap, b0)


def small_random_tas(seed: int, N: int, T: int, max_acc: int = 4, timed: bool = True, base_bytes: int = 0,
                     max_size: int = 1 << 20, link_bytes_per_us: int = 64) -> TAS:
    """Small unstructured TAS for tests: uniform sizes, allocation steps and gaps."""
    i = np.arange(N)
    size = prng.randint(seed, 40, i, 1, max_size)
    k = prng.randint(seed, 41, i, 0, max_acc)
    alloc = prng.randint(seed, 42, i, 0, T - 1)
    sizes, allocs, accs = [], [], []
    for t in range(N):
        room = T - 1 - int(alloc[t])
        kk = min(int(k[t]), room)
        if kk > 0:
            pick = np.argsort(prng.u64(seed, 44, t * 4096 + np.arange(room)), kind="stable")[:kk]
            acc = np.sort(int(alloc[t]) + 1 + pick)
        else:
            acc = np.zeros(0, dtype=np.int64)
        sizes.append(int(size[t])); allocs.append(int(alloc[t])); accs.append([int(a) for a in acc])
    sn = prng.randint(seed, 45, np.arange(T), 1, 1000).astype(np.int64) if timed else None
    return tas_from_lists(T, sizes, allocs, accs, None, sn, base_bytes, link_bytes_per_us if timed else 0)
