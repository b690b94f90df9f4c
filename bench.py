#!/usr/bin/env python3
"""Benchmark of the ONES evolutionary search on one MI355X.

A step is one generation of the whole hot path (compose the pool from the survivors, repair
every candidate to the cluster capacity, score it, select the best quarter) on the stress
cluster: 4096 GPUs, 2048 jobs, pool of 65536 candidates.  Prints one JSON line.

Protocol: the search is created from the same seed --reps + 1 times (initial population and
W warm-up generations untimed, then exactly K timed generations between two synchronisations);
the first repetition is a warm-up run, the reported figures are those of the repetition with
the median time of the others.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--reps 3] [--workload stress|large|paper_scale|tiny|online]
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import platform
import statistics
import subprocess
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published peak

# HBM bytes per evolve launch on the stress workload from rocprofv3 --pmc FETCH_SIZE and
# WRITE_SIZE (see profiles/), valid only for the kernel source with this hash.
MEASURED_TRAFFIC = {"source_sha256": "0b6ef20e102acdea716dafa2501ee9f1b0e5340947bc7b4bf13a3ae8b2a30dbe", "bytes_per_launch": 802626465}


def evolve_source_hash() -> str:
    h = hashlib.sha256()
    for f in ("ones_evolve.hip", "ones_candidate.h", "ones_device.h"):
        h.update(open(os.path.join(ROOT, "paper_2108_03645_amd", "csrc", f), "rb").read())
    return h.hexdigest()


def device_copy_gbps(torch) -> float:
    """Read + write rate of a plain 1 GiB device-to-device copy (best of 5), HIP events on the current stream."""
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0").fill_(1)
    dst = torch.empty_like(src)
    dst.copy_(src)
    best = float("inf")
    for _ in range(5):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(); dst.copy_(src); e1.record()
        e1.synchronize()
        best = min(best, e0.elapsed_time(e1))
    del src, dst
    return 2 * (1 << 30) / (best * 1e-3) / 1e9


def host_info():
    model = ""
    try:
        for line in open("/proc/cpuinfo"):
            if line.lower().startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    try:
        gcc = subprocess.run(["gcc", "--version"], capture_output=True, text=True).stdout.splitlines()[0]
    except (OSError, IndexError):
        gcc = ""
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = os.cpu_count() or 1
    return {"cpu_model": model or platform.processor(), "nproc": os.cpu_count() or 1, "usable_cpus": usable,
            "compiler": gcc}


def cpu_baseline(workload: str, sampled: bool = False):
    """The CPU oracle, as it stands, on a bounded sample of the same workload: a leg on the
    host's share of cores (at most 16 threads, the share of a one-GPU machine) and a single-thread
    leg, both from the same initial population."""
    from oracle import ones_ref
    from paper_2108_03645_amd import workloads as W
    info = host_info()
    threads = max(1, min(16, info["usable_cpus"]))
    if workload == "stress":
        cl, jobs = W.stress()
        gens_all, gens_one = 10, 2
    else:
        cl, jobs = W.CONFIGS[workload]()
        gens_all = max(10, min(cl.generations, int(1.5e9 / (cl.population * max(cl.n_slots, 1)))))
        gens_one = max(2, gens_all // 8)
    active = int(jobs.active.sum())
    legs = {}
    for name, n_threads, gens in (("all", threads, gens_all), ("one", 1, gens_one)):
        ones_ref.set_threads(n_threads)
        s = ones_ref.RefSearch(cl, jobs)              # initial population, not timed
        if sampled:
            s.set_progress(*W.progress(cl.n_slots, seed=cl.seed))
        t0 = time.perf_counter()
        s.generation(gens)
        dt = time.perf_counter() - t0
        s.close()
        legs[name] = {"value": cl.population * active * gens / dt, "generations_per_s": gens / dt, "seconds": dt,
                      "generations": gens, "threads": n_threads}
    ones_ref.set_threads(1)
    out = {"value": legs["all"]["value"], "unit": "evals/s", "cores": threads, "kind": "oracle",
           "sample": f"{workload} at full size (pool {cl.population}, {active} jobs): {gens_all} generations after the initial "
                     f"population on {threads} threads; single-thread leg: {gens_one} generations",
           "generations_per_s": legs["all"]["generations_per_s"], "seconds": legs["all"]["seconds"],
           "single_thread": {k: legs["one"][k] for k in ("value", "generations_per_s", "seconds", "generations")},
           "flags": "gcc -O2 -ffp-contract=off -fopenmp"}
    out.update(info)
    return out


def online_loop(make_search, sim, args, limits_clock, synchronize):
    """One run of the online sequence with any implementation of the search; returns the per-leg times."""
    cl = sim.cluster
    search = make_search(cl, sim.jobs)
    search.set_new_jobs_first(args.policies)
    search.set_crossover(per_gpu=args.crossover == "gpus")
    if args.sampled:
        search.set_progress(*sim.progress())
    gens = cl.generations
    t_set = t_gen = t_best = 0.0
    evals = 0
    for epoch in range(args.warmup + args.steps):
        timed = epoch >= args.warmup
        t0 = time.perf_counter()
        search.generation(gens)
        synchronize(search)
        t1 = time.perf_counter()
        batch, _, _ = search.best()
        t2 = time.perf_counter()
        limits_clock[1] = timed
        sim.advance(batch)
        t3 = time.perf_counter()
        search.set_jobs(sim.jobs)
        if args.policies:
            search.set_processed_time(sim.elapsed)
        if args.sampled:
            search.set_progress(*sim.progress())
        t4 = time.perf_counter()
        if timed:
            t_gen += t1 - t0; t_best += t2 - t1; t_set += t4 - t3
            evals += cl.population * int(sim.jobs.active.sum()) * gens
    search.close()
    return {"generations": t_gen, "ones_best": t_best, "ones_set_jobs": t_set, "ones_update_limits": limits_clock[0],
            "evals": evals, "completed": sim.completed, "last_batch": batch.tolist()}


def online(args, torch, ones, W) -> int:
    """The online sequence: every scheduling epoch replaces the job table (ones_set_jobs), runs
    20 warm-started generations and reads the winner (ones_best), which drives the simulated
    cluster.  A step is one epoch; --steps counts epochs.  Median of --reps repetitions of the
    whole sequence from the same seed after a warm-up repetition."""
    torch.cuda.set_device(0)

    def one_run(update_limits, make_search, synchronize):
        clock = [0.0, False]

        def timed_limits(*a, **k):
            t = time.perf_counter()
            out = update_limits(*a, **k)
            if clock[1]:
                clock[0] += time.perf_counter() - t
            return out

        sim = W.OnlineSequence(epochs=args.steps + args.warmup, limits=timed_limits if args.policies else None)
        return sim.cluster, online_loop(make_search, sim, args, clock, synchronize)

    def gpu_run():
        return one_run(ones.update_limits, lambda cl, jobs: ones.Search(cl, jobs, device="cuda:0"), lambda s: s.synchronize())

    legs = ("generations", "ones_best", "ones_set_jobs", "ones_update_limits")
    runs = [gpu_run() for _ in range(args.reps + 1)][1:] if args.reps > 0 else [gpu_run()]
    cl = runs[0][0]
    totals = sorted(sum(r[1][k] for k in legs) for r in runs)
    res = next(r[1] for r in runs if sum(r[1][k] for k in legs) == totals[(len(totals) - 1) // 2])
    assert all(r[1]["last_batch"] == res["last_batch"] for r in runs), "repetitions from one seed must end in one state"
    dt = sum(res[k] for k in legs)
    gens = cl.generations
    out = {"metric": "candidate-job fitness evals/sec", "value": res["evals"] / dt, "unit": "evals/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt * 1e3 / args.steps,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "i32 genes, f64 fitness", "data": "synthetic",
           "config": {"workload": "online", "n_gpus_cluster": cl.n_gpus, "slots": cl.n_slots,
                      "population": cl.population, "generations_per_epoch": gens, "seed": cl.seed,
                      "limit_policies": bool(args.policies), "crossover": "over " + args.crossover,
                      "remaining_work": "sampled per generation" if args.sampled else "fixed",
                      "jobs_completed": res["completed"]},
           "repetitions": {"timed": len(runs), "warmup_runs": 1 if args.reps > 0 else 0, "reported": "median",
                           "ms_per_step_all": [sum(r[1][k] for k in legs) * 1e3 / args.steps for r in runs]},
           "generations_per_s": gens * args.steps / dt,
           "per_epoch_ms": {k: res[k] * 1e3 / args.steps for k in legs}}
    if not args.no_cpu_baseline:
        # the oracle through the same loop, on the host's share of cores and on one
        from oracle import ones_ref
        info = host_info()
        threads = max(1, min(16, info["usable_cpus"]))
        cpu = {}
        for name, n_threads in (("all", threads), ("one", 1)):
            ones_ref.set_threads(n_threads)
            _, r = one_run(ones_ref.update_limits, lambda c, jobs: ones_ref.RefSearch(c, jobs), lambda s: None)
            t = sum(r[k] for k in legs)
            cpu[name] = {"value": r["evals"] / t, "ms_per_epoch": t * 1e3 / args.steps, "threads": n_threads}
            assert r["last_batch"] == res["last_batch"], "the oracle's sequence must end where the library's does"
        ones_ref.set_threads(1)
        out["cpu_baseline"] = {"value": cpu["all"]["value"], "unit": "evals/s", "cores": threads, "kind": "oracle",
                               "sample": f"the same {args.warmup} + {args.steps} epochs", "ms_per_epoch": cpu["all"]["ms_per_epoch"],
                               "single_thread": {"value": cpu["one"]["value"], "ms_per_epoch": cpu["one"]["ms_per_epoch"]},
                               "flags": "gcc -O2 -ffp-contract=off -fopenmp", **info}
    print(json.dumps(out))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--reps", type=int, default=3,
                    help="timed repetitions from the same seed after one warm-up repetition; the median is reported "
                         "(0: a single run, for profilers)")
    ap.add_argument("--workload", default="stress", choices=["stress", "large", "paper_scale", "tiny", "online"])
    ap.add_argument("--sampled", action="store_true",
                    help="probability sampling of the remaining work (Alg. 1): every generation draws it anew "
                         "and scores the survivors again; not the headline configuration")
    ap.add_argument("--crossover", default="jobs", choices=["jobs", "gpus"],
                    help="positions the uniform crossover scans: the jobs (headline configuration) or the GPUs of "
                         "the paper's encoding (Eq. 1)")
    ap.add_argument("--policies", action="store_true",
                    help="online workload only: batch-size limits from the policies of Section 3.3.2 "
                         "(ones_update_limits, timed as a leg of its own) and new jobs served first")
    ap.add_argument("--table-changes", type=int, default=0,
                    help="replace the job table (remaining work shrunk by 1 %%) this many times, evenly spread over the "
                         "timed generations: exercises the refresh of the survivors under a new table and the "
                         "selection that follows it; not the headline configuration")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-events", action="store_true", help="do not bracket kernels with HIP events")
    ap.add_argument("--copy-reference", action="store_true",
                    help="also run plain device copies of 1 GiB (2 GiB of traffic each), the yardstick "
                         "the rocprofv3 FETCH_SIZE / WRITE_SIZE counters are scaled by")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: the search runs on one GPU; --gpus above 1 is not supported "
              "(the pool would shard by candidates; only the selection couples them)", file=sys.stderr)
        return 2

    import torch
    from paper_2108_03645_amd import ones, workloads as W

    if args.workload == "online":
        return online(args, torch, ones, W)
    cl, jobs = W.CONFIGS[args.workload]()
    active = int(jobs.active.sum())
    jp = ones.padded_jobs(cl.n_slots)
    torch.cuda.set_device(0)

    def one_run():
        search = ones.Search(cl, jobs, device="cuda:0")       # initial population, not timed
        if args.sampled:
            search.set_progress(*W.progress(cl.n_slots, seed=cl.seed))
        search.set_crossover(per_gpu=args.crossover == "gpus")
        search.generation(args.warmup)
        search.synchronize()
        torch.cuda.synchronize()
        search.profile_enable(0 if args.no_events else 4)     # events on every 4th generation
        t0 = time.perf_counter()
        if args.table_changes > 0:
            table = jobs.copy()
            done = 0
            for k in range(args.table_changes + 1):
                upto = args.steps * (k + 1) // (args.table_changes + 1)
                search.generation(upto - done)
                done = upto
                if k < args.table_changes:
                    table.remaining = table.remaining * 0.99
                    search.set_jobs(table)
        else:
            search.generation(args.steps)
        search.synchronize()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        prof = search.profile_read()
        _, _, best_fit = search.best()
        search.close()
        return {"dt": dt, "prof": prof, "best_fit": best_fit}

    runs = [one_run() for _ in range(args.reps + 1)][1:] if args.reps > 0 else [one_run()]
    times = sorted(r["dt"] for r in runs)
    median = next(r for r in runs if r["dt"] == times[(len(times) - 1) // 2])
    dt, prof, best_fit = median["dt"], median["prof"], median["best_fit"]
    assert all(r["best_fit"] == best_fit for r in runs), "repetitions from one seed must end in one state"

    single_launch = prof["select_launches"] == 0 and prof["evolve_launches"] > 0   # small pool: one launch per call
    if args.no_events:
        prof = {"evolve_ms": float("nan"), "evolve_launches": 1, "select_ms": float("nan"), "select_launches": 1}
    evolve_ms = prof["evolve_ms"] / max(1, prof["evolve_launches"])
    select_ms = prof["select_ms"] / max(1, prof["select_launches"])
    if single_launch:
        evolve_ms, select_ms = evolve_ms / args.steps, 0.0    # the launch runs all timed generations
    # Bytes one evolve launch has to move for what it computes: it composes the 3P/4 children and
    # mutants (the P/4 survivors stay where they are), each gene of them read once from a parent
    # row and written once (int32), plus one fp64 score per candidate composed.
    composed = cl.population * 3 // 4
    alg_bytes = composed * cl.n_slots * 8 + composed * 8
    if args.sampled:      # the survivors are read once more to be scored again
        alg_bytes += (cl.population // 4) * (cl.n_slots * 4 + 8)
    pool_bytes = cl.population * cl.n_slots * 8 + cl.population * 8   # every candidate of the pool counted as read and written
    achieved = alg_bytes / (evolve_ms * 1e-3) / 1e9
    traffic = None
    if MEASURED_TRAFFIC["source_sha256"] == evolve_source_hash() and args.workload == "stress" and not args.sampled \
            and args.crossover == "jobs":
        traffic = MEASURED_TRAFFIC["bytes_per_launch"]
    copy_gbps = device_copy_gbps(torch)

    out = {
        "metric": "candidate-job fitness evals/sec",
        "value": cl.population * active * args.steps / dt,
        "unit": "evals/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt * 1e3 / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "i32 genes, f64 fitness", "data": "synthetic",
        "config": {"workload": args.workload, "n_gpus_cluster": cl.n_gpus, "jobs": active,
                   "slots_padded": jp, "population": cl.population, "survivors": cl.population // 4,
                   "mutation_rate": cl.mutation_rate, "crossover_rate": cl.crossover_rate,
                   "seed": cl.seed, "jobs_sha256": jobs.sha256()[:16],
                   "remaining_work": "sampled per generation" if args.sampled else "fixed",
                   "crossover": "over " + args.crossover, "table_changes": args.table_changes},
        "repetitions": {"timed": len(runs), "warmup_runs": 1 if args.reps > 0 else 0, "reported": "median",
                        "ms_per_step_all": [r["dt"] * 1e3 / args.steps for r in runs]},
        "generations_per_s": args.steps / dt,
        "best_fitness": best_fit,
        "kernels": {"evolve_ms": evolve_ms, "select_ms": select_ms,
                    "launches_per_generation": "one launch for all timed generations" if single_launch else "evolve + select"},
        "roofline": {"bound": "hbm", "kernel": "fused_kernel" if single_launch else "evolve_kernel",
                     "achieved": achieved, "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic,
                     "algorithmic_bytes_per_launch": alg_bytes,
                     "units_per_launch": f"{composed} candidates composed x {cl.n_slots} job slots, 8 B each, + 8 B per candidate",
                     # measured traffic over the same duration (None once the kernel has changed since the counters were read)
                     "physical_gbps": None if traffic is None else traffic / (evolve_ms * 1e-3) / 1e9,
                     "physical_frac": None if traffic is None else traffic / (evolve_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                     # a plain device-to-device copy of 1 GiB on this machine, read + write: the practical ceiling
                     "device_copy_gbps": copy_gbps, "frac_of_device_copy": achieved / copy_gbps,
                     # the whole pool counted as read and written, survivors included (what a ping-pong layout would move)
                     "pool_equivalent_gbps": pool_bytes / (evolve_ms * 1e-3) / 1e9},
    }
    if args.copy_reference:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.workload, args.sampled)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
