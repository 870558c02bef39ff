#!/usr/bin/env python3
"""Benchmark of the batched plan evaluator on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic plans:
``tensile_eval_plans`` (difference-array scatter, prefix scan, max/argmax/min,
footprint rows written) followed by ``tensile_score_candidates`` on the same
batch, inputs already resident in HBM.  The workload is configuration 3 (four
jobs merged on one timeline, 16,384 plans), the one the bandwidth target is
stated for.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3] [--no-cpu] [--no-greedy] [--no-extras]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
TRAFFIC_FILES = {"eval": os.path.join(ROOT, "profiles", "eval_stream_kernel_c3_hbm_traffic.txt"),
                 "score": os.path.join(ROOT, "profiles", "score_kernel_c3_hbm_traffic.txt"),
                 "step": os.path.join(ROOT, "profiles", "step_kernel_c3_hbm_traffic.txt")}
KERNEL_SOURCES = ("eval.hip", "eval_body.h", "score.hip", "score_body.h", "step.hip", "common.h", "wave_ops.h")


def kernel_sources_hash() -> str:
    """SHA-256 over the kernel sources: a counter summary under profiles/ is tied to the code it was measured on."""
    import hashlib
    hsh = hashlib.sha256()
    for name in KERNEL_SOURCES:
        path = os.path.join(ROOT, "paper_2105_13336_amd", "csrc", name)
        if os.path.exists(path):
            with open(path, "rb") as f:
                hsh.update(name.encode() + b"\0" + f.read())
    return hsh.hexdigest()[:16]


def measured_traffic(which: str, config: int):
    """(HBM bytes per launch, note): FETCH_SIZE + WRITE_SIZE of two rocprofv3 --pmc runs on this workload, as
    recorded in the summary under profiles/ (which gives the commands and the calibration).  The number is
    REPLAYED from that file, not measured in this run, so it is reported only while the file says it was taken on
    the kernel sources as they are now; otherwise None with the reason."""
    path = TRAFFIC_FILES[which]
    if config != 3:
        return None, "counter runs exist for configs[3] only"
    if not os.path.exists(path):
        return None, "no counter summary for this kernel"
    vals, stamp = {}, None
    with open(path) as f:
        for line in f:
            if "=" in line and not line.startswith("#"):
                k, v = line.split("=", 1)
                if k.strip() == "kernel_sources_sha256":
                    stamp = v.split()[0]
                else:
                    try:
                        vals[k.strip()] = float(v.split()[0])
                    except ValueError:
                        pass
    if stamp != kernel_sources_hash():
        return None, f"stale: {os.path.basename(path)} was measured on kernel sources {stamp}, these are {kernel_sources_hash()}"
    if "fetch_bytes_per_launch" in vals and "write_bytes_per_launch" in vals:
        return vals["fetch_bytes_per_launch"] + vals["write_bytes_per_launch"], f"replayed from profiles/{os.path.basename(path)} (kernel sources {stamp})"
    return None, "summary holds no byte counts"


def cpu_model() -> str:
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def log(msg: str) -> None:
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def ceilings() -> int:
    """What plain library kernels reach on this machine over a buffer of the size of configs[3]'s footprint rows
    (the practical ceilings the kernels are held against next to the 8 TB/s of the data sheet)."""
    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    n = 16384 * 50000
    a = torch.empty(n, dtype=torch.int64, device="cuda")
    b = torch.empty(n, dtype=torch.int64, device="cuda")

    def timed(f, reps=10):
        f()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            f()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    gb = n * 8 / 1e9
    out = {"buffer_GB": gb}
    for name, f, moved in (("fill", lambda: a.fill_(3), gb), ("copy", lambda: b.copy_(a), 2 * gb),
                           ("max_reduction", lambda: a.max(), gb), ("add_one_out_of_place", lambda: torch.add(a, 1, out=b), 2 * gb),
                           ("add_one_in_place", lambda: a.add_(1), 2 * gb)):
        ms = timed(f)
        out[name] = {"ms": ms, "GBps_moved": moved / ms * 1e3}
    print(json.dumps(out))
    return 0


def main() -> int:
    if "--ceilings" in sys.argv[1:]:
        return ceilings()
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle baseline leg")
    ap.add_argument("--cpu-plans", type=int, default=16384, help="plans in the oracle's sample on all threads (a quarter of them on one thread)")
    ap.add_argument("--cpu-threads", type=int, default=0, help="threads of the oracle's second leg (default: min(16, cores))")
    ap.add_argument("--print-sources-hash", action="store_true", help="print the hash that ties a counter summary to the kernel sources and exit")
    ap.add_argument("--no-greedy", action="store_true", help="skip the greedy-planner leg")
    ap.add_argument("--eval-only", action="store_true", help="steps run tensile_eval_plans alone (profiling aid)")
    ap.add_argument("--fused", action="store_true", help="the one-call row forces the fused evaluation + scoring kernel (profiling aid)")
    ap.add_argument("--no-extras", action="store_true", help="skip the per-job and recomputation rows (profiling aid)")
    ap.add_argument("--ceilings", action="store_true",
                    help="instead of the benchmark: time plain fill / copy / reduction kernels over 6.55 GB and print them")
    ap.add_argument("--calibrate", action="store_true",
                    help="before the steps, launch one plain elementwise kernel (out = in + 1) that reads 2 GiB and writes "
                         "2 GiB: the dispatch of known size that FETCH_SIZE / WRITE_SIZE of a counter run are scaled by")
    args = ap.parse_args()
    if args.print_sources_hash:
        print(kernel_sources_hash())
        return 0
    if args.gpus != 1:
        print("bench.py: this build evaluates plans on ONE GPU (plans are independent; no multi-GPU path is built); "
              "run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2105_13336_amd as P
    from workloads import CONFIGS, make_config_plans, make_tas, plans_hash, tas_hash

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = CONFIGS[args.config]
    t0 = time.time()
    tas = make_tas(args.config)
    pl = make_config_plans(args.config, tas)
    B, T, N, K = pl.B, tas.T, tas.N, pl.n_intervals
    log(f"{cfg.name}: B={B} T={T} N={N} intervals={K} tas_hash={tas_hash(tas):016x} plans_hash={plans_hash(pl):016x} "
        f"(generated in {time.time() - t0:.1f}s)")

    if args.calibrate:      # caches are far smaller than 2 GiB, so every byte comes from and goes to HBM
        cal_in = torch.zeros(1 << 28, dtype=torch.int64, device="cuda")
        cal_out = torch.empty_like(cal_in)
        torch.add(cal_in, 1, out=cal_out)
        torch.cuda.synchronize()
        del cal_in, cal_out

    h = P.tas_load(tas)
    dp = P.DevicePlans.from_numpy(pl.plan_offsets, pl.iv_tensor, pl.iv_out, pl.iv_in, pl.iv_kind)
    res = torch.empty((B, T), dtype=torch.int64, device="cuda")
    peak = torch.empty(B, dtype=torch.int64, device="cuda")
    arg = torch.empty(B, dtype=torch.int32, device="cuda")
    mn = torch.empty(B, dtype=torch.int64, device="cuda")
    sc = torch.empty((B, N), dtype=torch.int64, device="cuda")
    wo = torch.empty((B, N), dtype=torch.int32, device="cuda")
    wi = torch.empty((B, N), dtype=torch.int32, device="cuda")

    def step(events=None):
        if events is not None:
            events[0].record()
        P.tensile_eval_plans(h, dp, res, peak, arg, mn)
        if events is not None:
            events[1].record()
        if not args.eval_only:
            P.tensile_score_candidates(h, dp, res, peak, arg, sc, wo, wi)
            if events is not None:
                events[2].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for k in range(args.steps):
        step(evs[k])
    torch.cuda.synchronize()
    t_end = time.perf_counter()
    ms_per_step = (t_end - t_start) * 1e3 / args.steps
    eval_ms = [e[0].elapsed_time(e[1]) for e in evs]
    score_ms = [e[1].elapsed_time(e[2]) for e in evs] if not args.eval_only else [0.0]
    eval_avg, score_avg = float(np.mean(eval_ms)), float(np.mean(score_ms))
    plan_timesteps = float(B) * float(T)
    value = plan_timesteps / (ms_per_step * 1e-3)

    # algorithmic bytes of one eval launch: footprint rows out, intervals in (tensor, out, in: 12 B each;
    # the kind byte does not enter the footprint), offsets in, per-plan results out, MF0 and sizes once
    eval_bytes = 8.0 * B * T + 12.0 * K + 8.0 * (B + 1) + 20.0 * B + 8.0 * T + 8.0 * N
    achieved = eval_bytes / (eval_avg * 1e-3) / 1e9
    # scoring: footprint rows in, scores and windows out, intervals in
    score_bytes = 8.0 * B * T + 16.0 * B * N + 12.0 * K + 12.0 * B

    eval_traffic, eval_note = measured_traffic("eval", args.config)
    score_traffic, score_note = measured_traffic("score", args.config)
    out = {
        "metric": "plan-timesteps evaluated/sec (eval_plans + score_candidates per step) and % of peak HBM GB/s",
        "value": value, "unit": "plan-timesteps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int64", "data": "synthetic",
        "config": {"workload": f"configs[{args.config}] {cfg.name}", "B": B, "T": T, "N": N, "intervals": K,
                   "step": "eval_plans" if args.eval_only else "eval_plans+score_candidates"},
        "roofline": {"kernel": "eval_stream_kernel (tensile_eval_plans)" if args.config == 3 else "evaluation kernel (tensile_eval_plans)", "bound": "hbm", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": eval_traffic,
                     "traffic_note": eval_note, "algorithmic_bytes": eval_bytes, "avg_launch_ms": eval_avg},
        # the longest kernel of the step has its own block
        "roofline_score": {"kernel": "score_kernel (tensile_score_candidates)", "bound": "hbm",
                           "achieved": score_bytes / max(score_avg, 1e-9) / 1e6, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                           "frac": score_bytes / max(score_avg, 1e-9) / 1e6 / HBM_PEAK_GBS, "traffic": score_traffic,
                           "traffic_note": score_note, "algorithmic_bytes": score_bytes, "avg_launch_ms": score_avg},
        "kernel_sources": kernel_sources_hash(),
        "rows": {
            "eval_plans": {"ms": eval_avg, "ms_min": float(np.min(eval_ms)),
                           "plan_timesteps_per_s": plan_timesteps / (eval_avg * 1e-3)},
            "score_candidates": {"ms": score_avg, "algorithmic_GBps": score_bytes / max(score_avg, 1e-9) / 1e6,
                                 "frac_of_hbm_peak": score_bytes / max(score_avg, 1e-9) / 1e6 / HBM_PEAK_GBS},
        },
    }

    if not args.eval_only:
        # the same step through the one-call entry point
        if args.fused:
            P.tensile_tuning_set("step_fused", 1)
        sc1, wo1, wi1 = torch.empty_like(sc), torch.empty_like(wo), torch.empty_like(wi)
        pk1, ar1, mn1 = torch.empty_like(peak), torch.empty_like(arg), torch.empty_like(mn)
        res1 = torch.empty_like(res)
        P.tensile_eval_score_plans(h, dp, res1, pk1, ar1, mn1, sc1, wo1, wi1)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            P.tensile_eval_score_plans(h, dp, res1, pk1, ar1, mn1, sc1, wo1, wi1)
        e1.record()
        torch.cuda.synchronize()
        ms1 = e0.elapsed_time(e1) / 10
        for x, y in ((res1, res), (pk1, peak), (ar1, arg), (mn1, mn), (sc1, sc), (wo1, wo), (wi1, wi)):
            assert torch.equal(x, y)
        out["rows"]["eval_score_plans"] = {"ms": ms1, "plan_timesteps_per_s": plan_timesteps / (ms1 * 1e-3),
                                           "kernels": "one fused kernel (forced)" if args.fused else "evaluation, then scoring"}
        P.tensile_tuning_reset()
        del sc1, wo1, wi1, pk1, ar1, mn1, res1

    if not args.no_extras:
        # The same batch with the intervals of every plan in random order (seeded): the kernel lets a wavefront skip
        # the tiles its 384 consecutive intervals cannot touch, which a list in tensor / time order favours; a caller
        # that appends intervals in any other order (the greedy planner does) gets this number instead.
        gen = torch.Generator(device="cuda")
        gen.manual_seed(210513336)
        lens = dp.plan_offsets[1:] - dp.plan_offsets[:-1]
        owner = torch.repeat_interleave(torch.arange(B, device="cuda", dtype=torch.int64), lens)
        keys = (owner << 32) | torch.randint(0, 1 << 31, (K,), generator=gen, device="cuda", dtype=torch.int64)
        perm = torch.argsort(keys)
        del keys, owner
        dps = P.DevicePlans(dp.plan_offsets, dp.iv_tensor[perm].contiguous(), dp.iv_out[perm].contiguous(),
                            dp.iv_in[perm].contiguous(), None if dp.iv_kind is None else dp.iv_kind[perm].contiguous())
        del perm
        pk_s, ar_s, mn_s = torch.empty_like(peak), torch.empty_like(arg), torch.empty_like(mn)
        res_s = torch.empty_like(res)
        P.tensile_eval_plans(h, dps, res_s, pk_s, ar_s, mn_s)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            P.tensile_eval_plans(h, dps, res_s, pk_s, ar_s, mn_s)
        e1.record()
        torch.cuda.synchronize()
        ms_s = e0.elapsed_time(e1) / 5
        assert torch.equal(pk_s, peak) and torch.equal(ar_s, arg) and torch.equal(mn_s, mn) and torch.equal(res_s, res)
        out["rows"]["eval_plans_shuffled"] = {"ms": ms_s, "frac_of_hbm_peak": eval_bytes / (ms_s * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                              "note": "intervals of every plan in random order; results identical"}
        del dps, res_s, pk_s, ar_s, mn_s

    if not args.eval_only and not args.no_extras and tas.J > 1:
        # per-job peaks and their sum (one pass of the evaluation kernel per job, no rows written)
        jp = torch.empty((int(tas.J), B), dtype=torch.int64, device="cuda")
        tot = torch.empty(B, dtype=torch.int64, device="cuda")
        P.tensile_eval_plans_per_job(h, dp, jp, None, tot)                 # first call builds the per-job tables
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(3):
            P.tensile_eval_plans_per_job(h, dp, jp, None, tot)
        e1.record()
        torch.cuda.synchronize()
        out["rows"]["eval_plans_per_job"] = {"ms": e0.elapsed_time(e1) / 3, "jobs": int(tas.J)}
        del jp, tot

    if not args.eval_only and not args.no_extras:
        # the recomputation savings of the same batch (second scoring mode; not part of the step)
        P.tensile_score_recompute(h, dp, res, peak, arg, sc, wo, wi)       # first call builds its index
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(3):
            P.tensile_score_recompute(h, dp, res, peak, arg, sc, wo, wi)
        e1.record()
        torch.cuda.synchronize()
        out["rows"]["score_recompute"] = {"ms": e0.elapsed_time(e1) / 3}
        P.tensile_score_candidates(h, dp, res, peak, arg, sc, wo, wi)      # the outputs the checks below expect
        torch.cuda.synchronize()

    if not args.eval_only and not args.no_extras and tas.step_ns is not None:
        # occupancy of the host link by the same batch's transfers (second evaluated channel; not part of the step)
        lrows = torch.empty((B, T), dtype=torch.int32, device="cuda")
        lpk = torch.empty(B, dtype=torch.int32, device="cuda")
        larg = torch.empty(B, dtype=torch.int32, device="cuda")
        lover = torch.empty(B, dtype=torch.int32, device="cuda")
        link_ms = {}
        for name, rows_out, reuse in (("reuse", lrows, True), ("peaks_only", None, False), ("rows", lrows, False)):
            P.tensile_eval_link(h, dp, lpk, rows_out, larg, lover, reuse_host_copies=reuse)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(3):
                P.tensile_eval_link(h, dp, lpk, rows_out, larg, lover, reuse_host_copies=reuse)
            e1.record()
            torch.cuda.synchronize()
            link_ms[name] = e0.elapsed_time(e1) / 3
        out["rows"]["eval_link"] = {"ms": link_ms["rows"], "ms_peaks_only": link_ms["peaks_only"],
                                    "ms_with_host_copy_reuse": link_ms["reuse"],
                                    "max_link_peak": int(lpk.max()), "plans_within_one": int((lpk <= 1).sum())}
        del lrows, lpk, larg, lover

    if not args.eval_only and not args.no_extras:
        # windowed update: one more interval per plan on the rows that exist (a random gap of a random tensor each)
        from workloads.plans import eligible_gaps
        eoff, ep, eq = eligible_gaps(tas)
        rng = np.random.default_rng(2105_13336)
        g = rng.integers(0, len(ep), size=B)
        ti = (np.searchsorted(eoff, g, side="right") - 1).astype(np.int32)
        oi = (ep[g] + rng.integers(0, 1 << 30, size=B) % (eq[g] - 1 - ep[g])).astype(np.int32)
        ri = (oi + 2 + rng.integers(0, 1 << 30, size=B) % (eq[g] - oi - 1)).astype(np.int32)
        d_ti, d_oi, d_ri = (torch.from_numpy(x).cuda() for x in (ti, oi, ri))
        res2 = res.clone()
        pk2, ar2, mn2 = torch.empty_like(peak), torch.empty_like(arg), torch.empty_like(mn)
        P.tensile_apply_intervals(h, d_ti, d_oi, d_ri, res2, pk2, ar2, mn2)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(3):      # (each call takes the window out once more: the timing is what matters here)
            P.tensile_apply_intervals(h, d_ti, d_oi, d_ri, res2, pk2, ar2, mn2)
        e1.record()
        torch.cuda.synchronize()
        out["rows"]["apply_intervals"] = {"ms": e0.elapsed_time(e1) / 3, "mean_window_steps": float((ri - oi - 1).mean())}
        del res2, pk2, ar2, mn2

    if not args.no_greedy:
        iters = 48
        P.tensile_greedy_plan(h, 0, max_iters=4, capacity=8192)      # warm-up: the planner's buffers are allocated once per handle
        torch.cuda.synchronize()
        tg = time.perf_counter()
        g = P.tensile_greedy_plan(h, 0, max_iters=iters, capacity=iters)
        tg = time.perf_counter() - tg
        out["rows"]["greedy_plan"] = {"iterations": int(len(g["iv_tensor"])), "s": tg,
                                      "iterations_per_s": len(g["iv_tensor"]) / tg,
                                      "peak_before": int(g["peak_trace"][0]), "peak_after": int(g["final_peak"])}
        # both phases of the complete algorithm: swaps until none is accepted, then recomputation towards 10 %
        budget = int(g["peak_trace"][0]) // 10
        torch.cuda.synchronize()
        tg = time.perf_counter()
        g2 = P.tensile_greedy_plan(h, budget, min_iters=1 << 30, recompute=True, capacity=8192)
        tg = time.perf_counter() - tg
        out["rows"]["greedy_plan_with_recompute"] = {
            "iterations": int(len(g2["iv_tensor"])), "swaps": int((g2["iv_kind"] == 0).sum()),
            "recomputations": int((g2["iv_kind"] == 1).sum()), "s": tg, "iterations_per_s": len(g2["iv_tensor"]) / tg,
            "budget": budget, "peak_after": int(g2["final_peak"])}

    if not args.no_cpu:
        # The oracle as it stands on this machine's host cores, on a bounded sample of the same batch and the same
        # step: once on one thread, once with the plans split evenly over P threads (the C loops release the
        # interpreter lock).  A baseline, not a target.
        from concurrent.futures import ThreadPoolExecutor
        from oracle import oracle as O
        n_thr = args.cpu_threads if args.cpu_threads > 0 else min(16, os.cpu_count() or 1)
        ns = min(B, args.cpu_plans)
        ns1 = max(1, ns // 4)
        MF0 = O.base_timeline(tas)

        def leg(b0, b1):
            sample = pl.select(np.arange(b0, b1))
            t_a = time.perf_counter()
            r0, p0, a0, m0 = O.eval_plans(tas, sample, MF0=MF0)
            t_b = time.perf_counter()
            sco = None if args.eval_only else O.score_plans(tas, sample, r0, p0, a0)
            return (b0, b1), t_b - t_a, time.perf_counter() - t_b, (r0[:8].copy() if b0 == 0 else None, p0, a0, sco)

        log(f"cpu baseline: oracle on the first {ns1} plans, one thread")
        tc0 = time.perf_counter()
        one = leg(0, ns1)
        t_one = time.perf_counter() - tc0
        log(f"cpu baseline: oracle on the first {ns} plans, {n_thr} threads")
        edges = np.linspace(0, ns, n_thr + 1).astype(int)
        tc0 = time.perf_counter()
        with ThreadPoolExecutor(max_workers=n_thr) as pool:
            parts = list(pool.map(lambda k: leg(int(edges[k]), int(edges[k + 1])), range(n_thr)))
        t_all = time.perf_counter() - tc0
        what = "eval" if args.eval_only else "eval + score"
        out["cpu_baseline"] = {"value": ns * float(T) / t_all, "unit": "plan-timesteps/s", "cores": n_thr, "kind": "oracle",
                               "sample": f"first {ns} of {B} plans of the same batch, same step ({what}), plans split evenly "
                                         f"over {n_thr} threads; single thread: first {ns1} plans",
                               "seconds": t_all, "cpu_model": cpu_model(), "host_cores": os.cpu_count(),
                               "single_thread": {"value": ns1 * float(T) / t_one, "cores": 1, "plans": ns1, "seconds": t_one,
                                                 "eval_only_value": ns1 * float(T) / one[1]}}
        # the GPU results for the sample agree with what the oracle just computed
        for (b0, b1), _, _, (r8, p0, a0, sco) in parts + [one]:
            assert np.array_equal(peak[b0:b1].cpu().numpy(), p0) and np.array_equal(arg[b0:b1].cpu().numpy(), a0)
            if r8 is not None:
                assert np.array_equal(res[:8].cpu().numpy(), r8)
            if sco is not None:
                assert np.array_equal(sc[b0:b1].cpu().numpy(), sco[0]) and np.array_equal(wo[b0:b1].cpu().numpy(), sco[1])
    h.close()
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
