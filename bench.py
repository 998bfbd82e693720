#!/usr/bin/env python3
"""Benchmark of one scheduling tick (prepare -> fit -> select -> resolve) on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input that
is already resident in HBM.  Prints ONE JSON line: gap-job fit evaluations per
second for the whole step, the fit kernel's roofline figures, and the CPU
oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published peak HBM3E bandwidth


def algorithmic_fit_bytes(wl, n_atoms_total):
    """Bytes the pair-evaluation kernel must move: 4 B of cut per pair, one 12-byte atom
    record (running duration, running peak, boundary) per safe cut after the progress
    point, 8 B per gap.  The interest rows (1 bit per pair) are written by a kernel of
    their own and are not counted here."""
    G, J = wl.n_gaps, wl.n_jobs
    return 4 * G * J + 12 * n_atoms_total + 8 * G


def secondary_rates(wl, n_atoms_total, call_ms, rounds):
    """Algorithmic bytes and rates of the other calls (whole calls, HIP events): prepare moves 9 B in
    and 12 B out per segment after the progress point plus 16 B per atom and 20 B per job; select
    reads the 4-byte cut of every pair and writes 16 B per gap; the rounds of resolve are bound by
    latency, so they are reported per round."""
    import numpy as np
    G, J = wl.n_gaps, wl.n_jobs
    remaining = int((np.diff(wl.seg_off) - wl.progress).clip(min=0).sum())
    out = {}
    for name, nbytes in (("prepare", 21 * remaining + 16 * n_atoms_total + 20 * J), ("select", 4 * G * J + 16 * G)):
        gbs = nbytes / (call_ms[name] * 1e-3) / 1e9
        out[name] = {"algorithmic_bytes": nbytes, "achieved_GBs": gbs, "frac": gbs / HBM_PEAK_GBS,
                     "evals_per_s": G * J / (call_ms[name] * 1e-3)}
    out["resolve"] = {"us_per_round": 1e3 * call_ms["resolve"] / max(rounds, 1), "rounds": rounds,
                      "evals_per_s": G * J / (call_ms["resolve"] * 1e-3)}
    return out


# HBM traffic of one k_fit_main launch from two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE, KiB
# per dispatch), each scaled by what the same counter reads for a plain 1 GiB device copy
# (profiles/fit_main_stress_pmc.md).  It belongs to one kernel source and one workload: the
# sources are hashed, and a different hash means the counters are stale.
FIT_TRAFFIC = {
    "workload": ("stress", 0),
    "sources_sha256": "c8e03b40c653190bbaddc66b9dce349b1f4f729e9d9c9efb8aebfc76fe43d981",
    "fetch_kib": 51530.1, "fetch_scale": 2.0,
    "write_kib": 8391936.0, "write_scale": 1.0,
}


def fit_kernel_sources_sha256():
    """Hash of what defines k_fit_main: its source file and the tile constants it is built with."""
    import hashlib
    csrc = os.path.join(ROOT, "paper_2509_19086_amd", "csrc")
    h = hashlib.sha256()
    with open(os.path.join(csrc, "k_fit.h"), "rb") as f:
        h.update(f.read())
    with open(os.path.join(csrc, "sja_internal.h"), "rb") as f:
        for line in f.read().splitlines():
            if line.startswith(b"constexpr int kFit"):
                h.update(line)
    return h.hexdigest()


def measured_fit_traffic(workload, seed):
    """Bytes per launch, or None when the counters were taken for another kernel or workload."""
    t = FIT_TRAFFIC
    if t["workload"] != (workload, seed) or t["sources_sha256"] != fit_kernel_sources_sha256():
        return None
    return int((t["fetch_kib"] * t["fetch_scale"] + t["write_kib"] * t["write_scale"]) * 1024)


def count_atoms(wl):
    """Safe boundaries after each job's progress point (the end always counts)."""
    import numpy as np
    flags = wl.safe.astype(np.int64).copy()
    flags[wl.seg_off[1:] - 1] = 1
    cs = np.concatenate(([0], np.cumsum(flags)))
    start = wl.seg_off[:-1] + wl.progress
    return int((cs[wl.seg_off[1:]] - cs[start]).sum())


def cpu_baseline(wl, sample_gaps):
    """The oracle as it stands, whole hot path, on the first `sample_gaps` gaps x all jobs.
    Its resolve settles conflicts among the sampled gaps only (far fewer rounds than the full
    batch needs), so `value` is the oracle's rate on that smaller problem and must not be divided
    into the GPU's whole-tick `value`; `fit_only_value` (the per-pair walk alone) is like for like
    with `fit_evals_per_s`."""
    import numpy as np
    import oracle as O
    O.build()
    n = min(sample_gaps, wl.n_gaps)
    W = np.ascontiguousarray(wl.W[:n])
    C = np.ascontiguousarray(wl.C[:n])
    par = O.Params.make(wl.policy, wl.wait_scale, wl.sla_weight, wl.class0_override, wl.max_rounds)
    t0 = time.perf_counter()
    pd, pp, _ = O.prepare(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress)
    t1 = time.perf_counter()
    cut, _ = O.fit(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress, W, C)
    t2 = time.perf_counter()
    O.select(cut, wl.seg_off, pd, pp, par, wl.wait, wl.sla_class)
    t3 = time.perf_counter()
    res = O.resolve(cut, wl.seg_off, pd, pp, par, wl.wait, wl.sla_class)
    t4 = time.perf_counter()
    total = t4 - t0
    # one core, for scale: the per-pair walk on a slice of the same batch (about a second of work)
    one = {}
    threads = O.num_threads()
    try:
        O.set_num_threads(1)
        n1 = max(1, min(n, 64))
        t5 = time.perf_counter()
        O.fit(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress, np.ascontiguousarray(wl.W[:n1]),
              np.ascontiguousarray(wl.C[:n1]), False)
        t6 = time.perf_counter()
        one = {"fit_only_value_one_core": n1 * wl.n_jobs / (t6 - t5), "one_core_sample_gaps": n1}
    finally:
        O.set_num_threads(threads)
    return {
        **one,
        "value": n * wl.n_jobs / total,
        "unit": "fit evaluations/s",
        "cores": O.num_threads(),
        "kind": "oracle",
        "sample": f"first {n} of {wl.n_gaps} gaps x all {wl.n_jobs} jobs, whole tick "
                  f"(prepare {t1 - t0:.2f}s, fit {t2 - t1:.2f}s, select {t3 - t2:.2f}s, "
                  f"resolve {t4 - t3:.2f}s, {res[4]} rounds)",
        "fit_only_value": n * wl.n_jobs / (t2 - t1),
        "fit_seconds_sample": t2 - t1,
        "fit_seconds_full_extrapolated": (t2 - t1) * wl.n_gaps / n,
        "note": "resolve ran on the sampled gaps only (fewer conflicts, fewer rounds than the GPU's step): "
                "compare fit_only_value with fit_evals_per_s, not value with value",
        "seconds": total,
    }


def run_statistics(wl, tick):
    """What one tick produced, for comparing runs: interest density, mean walk length (cut - progress
    over the interested pairs) and plain int64 sums of the outputs.  Computed after the timed steps,
    a slab of gap rows at a time so that the temporaries stay small."""
    import torch
    G, J = wl.n_gaps, wl.n_jobs
    interested = 0
    cut_sum = 0
    walk_sum = 0
    prog = tick.progress.to(torch.int64)
    rows = max(1, (1 << 28) // max(J, 1))
    for g0 in range(0, G, rows):
        slab = tick.cut[g0:g0 + rows]
        m = slab >= 0
        per_job = m.sum(dim=0, dtype=torch.int64)
        interested += int(per_job.sum().item())
        cut_sum += int(slab.sum(dtype=torch.int64).item())
        walk_sum += int((torch.where(m, slab, torch.zeros_like(slab)).sum(dtype=torch.int64)
                         - (per_job * prog).sum()).item())
    i64 = lambda t: int(t.sum(dtype=torch.int64).item())
    return {"interest_density": interested / (G * J) if G * J else None,
            "mean_walk_segments": walk_sum / interested if interested else None,
            "checksums": {"cut": cut_sum, "interest_bits": i64(tick.bits.view(torch.uint8)) if tick.bits is not None else None,
                          "pre_dur": i64(tick.pre_dur), "cand_job": i64(tick.cand_job), "cand_score": i64(tick.cand_score),
                          "grant_job": i64(tick.grant_job), "grant_cut": i64(tick.grant_cut),
                          "grant_score": i64(tick.grant_score), "job_gap": i64(tick.job_gap)}}


def bandwidth_reference(eng, tick):
    """What this GPU does on plain kernels, measured in the same process: a linear fill of the cut
    matrix, the pair-evaluation kernel's own store stream with nothing computed
    (sja_store_reference: same launch shape, same row pieces in the same order) and a 1 GiB device
    copy (read + write counted).  Run after the timed steps: the first two overwrite the matrix."""
    import torch
    def timed(fn, reps=5):
        fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record(); e1.synchronize()
        return e0.elapsed_time(e1) / reps
    out = {}
    if tick.cut is not None and tick.cut.numel():
        ms = timed(lambda: tick.cut.fill_(-1))
        out["fill_cut_matrix_GBs"] = tick.cut.numel() * 4 / (ms * 1e-3) / 1e9
        ms = timed(lambda: eng.sja_store_reference(tick.cut))
        out["store_stream_ms"] = ms
        out["store_stream_GBs"] = tick.cut.numel() * 4 / (ms * 1e-3) / 1e9
    src = torch.empty(2**28, dtype=torch.int32, device="cuda:0")
    dst = torch.empty_like(src)
    ms = timed(lambda: dst.copy_(src))
    out["copy_1GiB_GBs"] = 2 * src.numel() * 4 / (ms * 1e-3) / 1e9
    return out


def large_fit(args):
    """The pair-evaluation kernel on the Large config as well (the second-largest; 2^28 pairs)."""
    import torch
    import paper_2509_19086_amd as P
    from gen import make_workload
    wl = make_workload("large", args.seed)
    eng = P.Engine(0)
    eng.sja_enable_timing(True)
    t = P.DeviceTick(eng, wl)
    t.prepare()
    ms, call = [], []
    for i in range(6):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(); t.fit(); e1.record(); e1.synchronize()
        if i:
            ms.append(eng.sja_last_fit_kernel_ms())
            call.append(e0.elapsed_time(e1))
    alg = algorithmic_fit_bytes(wl, count_atoms(wl))
    k = sum(ms) / len(ms)
    return {"workload": f"large seed {wl.seed}: {wl.n_gaps} gaps x {wl.n_jobs} jobs", "kernel_ms": k,
            "call_ms": sum(call) / len(call), "algorithmic_bytes": alg,
            "achieved_GBs": alg / (k * 1e-3) / 1e9, "frac": alg / (k * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "evals_per_s": wl.n_gaps * wl.n_jobs / (k * 1e-3)}


def measure_extras(args, wl, eng, tick, par):
    """Measured after the timed steps, never part of them: the fused fit-select call, a chain of
    ticks with sja_advance, and the tick's front half under admission limits with sja_cover."""
    import numpy as np
    import torch
    import paper_2509_19086_amd as P
    from gen import make_channels, make_gaps
    pairs = wl.n_gaps * wl.n_jobs

    # the fused fit -> select call (same candidates, no pair matrix)
    fused_ms, fused_kernel_ms = [], []
    reps = 3
    for i in range(reps + 1):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(); tick.fit_select(par); e1.record(); e1.synchronize()
        if i:
            fused_ms.append(e0.elapsed_time(e1))
            fused_kernel_ms.append(eng.sja_last_fit_kernel_ms())

    # a chain of ticks with fresh gaps each tick (fused fit-select,
    # grants, advance), the job tables carried over instead of prepared again
    chain_gaps = [(tick.W, tick.C)] + [tuple(torch.from_numpy(a).cuda() for a in
                                             make_gaps(args.workload, args.seed, k)) for k in range(1, args.chain_ticks)]
    chain = {"tick_ms": [], "advance_ms": [], "grants": [], "rejected_gaps": [], "finished_jobs": [], "rounds": [],
             "utilisation": [], "mean_wait_of_unfinished_jobs": []}
    lens = torch.from_numpy(np.diff(wl.seg_off).astype(np.int32)).cuda()
    tick.prepare()
    for W_k, C_k in chain_gaps:
        tick.W, tick.C = W_k, C_k
        e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        e[0].record(); tick.fit_select(par); tick.resolve(par)
        e[1].record(); tick.advance(1000)
        e[2].record(); e[2].synchronize()
        m = tick.metrics.cpu().tolist()
        chain["tick_ms"].append(e[0].elapsed_time(e[2]))
        chain["advance_ms"].append(e[1].elapsed_time(e[2]))
        chain["grants"].append(m[2])
        chain["rejected_gaps"].append(wl.n_gaps - m[2])
        chain["finished_jobs"].append(m[3])
        open_jobs = tick.progress < lens
        chain["mean_wait_of_unfinished_jobs"].append(
            float(tick.wait[open_jobs].double().mean().item()) if bool(open_jobs.any()) else None)
        chain["rounds"].append(tick.rounds.cpu().tolist()[0])
        chain["utilisation"].append(m[0] / m[1] if m[1] else None)
    # the tick's front half under admission limits, and the covering-capacity map
    power, deadline = make_channels(wl, args.seed)
    lim_kw = dict(tau_min=int(wl.W.max()) // 14, tau_max=(2 * int(wl.W.max())) // 3,
                  power_cap=int(np.percentile(power, 85)), now=7)
    d_power, d_deadline = torch.from_numpy(power).cuda(), torch.from_numpy(deadline).cuda()
    cap_set = torch.from_numpy(np.unique(wl.C)).cuda()
    cover = torch.empty(wl.n_gaps, dtype=torch.int32, device="cuda:0")
    slack = torch.empty_like(cover)
    tick.W, tick.C = chain_gaps[0]
    tick.progress.copy_(torch.from_numpy(wl.progress))
    tick.wait.copy_(torch.from_numpy(wl.wait))
    limited = {"prepare_ms": [], "fit_select_ms": [], "cover_ms": []}
    eng.sja_set_limits(P.Limits.make(**lim_kw), d_power, d_deadline)
    try:
        for i in range(reps + 1):
            e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
            e[0].record(); tick.prepare()
            e[1].record(); tick.fit_select(par)
            e[2].record(); e[2].synchronize()
            if i:
                limited["prepare_ms"].append(e[0].elapsed_time(e[1]))
                limited["fit_select_ms"].append(e[1].elapsed_time(e[2]))
        tick.resolve(par)
        for i in range(reps + 1):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(); eng.sja_cover(tick.C, tick.grant_job, tick.grant_cut, cap_set, cover, slack)
            e1.record(); e1.synchronize()
            if i:
                limited["cover_ms"].append(e0.elapsed_time(e1))
        limited = {k: sum(v) / len(v) for k, v in limited.items()}
        limited.update({"limits": lim_kw, "interested_candidates": int((tick.cand_job >= 0).sum().item()),
                        "grants": int((tick.grant_job >= 0).sum().item()),
                        "rounds": tick.rounds.cpu().tolist()[0],
                        "mean_slack_of_grants": float(slack[tick.grant_job >= 0].float().mean().item()),
                        "note": "power trace under a cap, per-job deadlines, min / max subjob duration "
                                "(sja_set_limits) and sja_cover over the gaps' own capacity set; "
                                "not part of the timed step"})
    finally:
        eng.sja_set_limits(None)
    chain["note"] = ("sja_fit_select + sja_resolve + sja_advance per tick, new gaps every tick, no prepare "
                     "after the first; not part of the timed step")

    # the same front half with the area-under-the-envelope score
    tick.progress.copy_(torch.from_numpy(wl.progress))
    tick.wait.copy_(torch.from_numpy(wl.wait))
    by_area = {"prepare_ms": [], "fit_select_ms": []}
    eng.sja_set_score(1)
    try:
        for i in range(reps + 1):
            e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
            e[0].record(); tick.prepare()
            e[1].record(); tick.fit_select(par)
            e[2].record(); e[2].synchronize()
            if i:
                by_area["prepare_ms"].append(e[0].elapsed_time(e[1]))
                by_area["fit_select_ms"].append(e[1].elapsed_time(e[2]))
        tick.resolve(par)
        by_area = {k: sum(v) / len(v) for k, v in by_area.items()}
        by_area.update({"rounds": tick.rounds.cpu().tolist()[0], "grants": int((tick.grant_job >= 0).sum().item()),
                        "note": "sja_set_score(SJA_SCORE_AREA): F = area under the envelope; not part of the timed step"})
    finally:
        eng.sja_set_score(0)
    return {
        "area_score": by_area,
        "fused_fit_select": {"call_ms": sum(fused_ms) / len(fused_ms),
                             "kernel_ms": sum(fused_kernel_ms) / len(fused_kernel_ms),
                             "evals_per_s": pairs / (sum(fused_ms) / len(fused_ms) * 1e-3),
                             "note": "sja_fit_select: the candidates of fit + select without the pair matrix; "
                                     "not part of the timed step"},
        "tick_chain": chain,
        "admission_limits": limited,
        "large_fit": large_fit(args) if wl.name != "large" else None,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="stress",
                    help="named config (default: stress, the largest single-GPU config)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--cpu-sample-gaps", type=int, default=4096)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--max-rounds", type=int, default=None,
                    help="override the config's resolve round cap (0 = until stable)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 1 GiB device copy three times (reference reading for "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE) and exit")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip what is measured after the timed steps (fused call, chain of ticks, limits)")
    ap.add_argument("--chain-ticks", type=int, default=4,
                    help="ticks in the carried-over chain measured after the timed steps")
    args = ap.parse_args()
    if args.copy_calibration:
        import torch
        src = torch.arange(2**28, dtype=torch.int32, device="cuda:0")      # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": src.numel() * 4, "copy_bytes_written": src.numel() * 4}))
        return
    if args.gpus != 1:
        print("bench.py measures one GPU: this path uses no second GPU, run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2509_19086_amd as P
    from gen import make_workload

    if not torch.cuda.is_available():
        print("bench.py needs the GPU (no CPU fallback exists)", file=sys.stderr)
        sys.exit(2)

    t_gen = time.perf_counter()
    wl = make_workload(args.workload, args.seed)
    if args.max_rounds is not None:
        wl.max_rounds = args.max_rounds
    n_atoms = count_atoms(wl)
    t_gen = time.perf_counter() - t_gen

    eng = P.Engine(0)
    tick = P.DeviceTick(eng, wl)
    par = P.Params.make(wl.policy, wl.wait_scale, wl.sla_weight, wl.class0_override, wl.max_rounds)
    eng.sja_enable_timing(True)
    torch.cuda.synchronize()

    def step(record=None):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(5)]
        ev[0].record(); tick.prepare()
        ev[1].record(); tick.fit()
        ev[2].record(); tick.select(par)
        ev[3].record(); tick.resolve(par)
        ev[4].record()
        if record is not None:
            ev[4].synchronize()
            record["prepare"].append(ev[0].elapsed_time(ev[1]))
            record["fit"].append(ev[1].elapsed_time(ev[2]))
            record["select"].append(ev[2].elapsed_time(ev[3]))
            record["resolve"].append(ev[3].elapsed_time(ev[4]))
            record["fit_kernel"].append(eng.sja_last_fit_kernel_ms())

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    rec = {k: [] for k in ("prepare", "fit", "select", "resolve", "fit_kernel")}
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(rec)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    pairs = wl.n_gaps * wl.n_jobs
    ms_per_step = 1e3 * elapsed / args.steps
    mean = lambda xs: sum(xs) / len(xs)
    fit_kernel_ms = mean(rec["fit_kernel"])
    alg_bytes = algorithmic_fit_bytes(wl, n_atoms)
    achieved = alg_bytes / (fit_kernel_ms * 1e-3) / 1e9
    rounds, stable = tick.rounds.cpu().tolist()
    grants = int((tick.grant_job >= 0).sum().item())
    stats = run_statistics(wl, tick)
    reference = bandwidth_reference(eng, tick)

    extras = {} if args.no_extras else measure_extras(args, wl, eng, tick, par)

    out = {
        "metric": "gap-job fit evaluations/sec: `value` = G*J / one whole tick (prepare+fit+select+resolve until "
                  "stable); `fit_evals_per_s` = G*J / t(sja_fit), the call the HBM roofline is quoted on; 1 GPU",
        "value": pairs / (elapsed / args.steps),
        "unit": "fit evaluations/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int32",
        "data": "synthetic",
        "config": {"workload": f"{wl.name} seed {wl.seed}: {wl.n_gaps} gaps x {wl.n_jobs} jobs, "
                               f"{wl.n_segments} segments, policy {wl.policy}, "
                               f"max_rounds {wl.max_rounds}",
                   "pairs": pairs, "atoms": n_atoms},
        "call_ms": {k: mean(v) for k, v in rec.items()},
        "call_ms_median": {k: sorted(v)[len(v) // 2] for k, v in rec.items()},
        "call_ms_min": {k: min(v) for k, v in rec.items()},
        "secondary": secondary_rates(wl, n_atoms, {k: mean(v) for k, v in rec.items()}, rounds),
        "fit_evals_per_s": pairs / (mean(rec["fit"]) * 1e-3),
        "fit_kernel_evals_per_s": pairs / (fit_kernel_ms * 1e-3),
        **extras,
        "resolve": {"rounds": rounds, "stable": stable, "grants": grants},
        "run": stats,
        "bandwidth_reference": reference,
        "roofline": {"kernel": "k_fit_main", "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "frac_of_fill": (achieved / reference["fill_cut_matrix_GBs"]
                                      if "fill_cut_matrix_GBs" in reference else None),
                     "frac_of_store_stream": (achieved / reference["store_stream_GBs"]
                                              if "store_stream_GBs" in reference else None),
                     "traffic": measured_fit_traffic(args.workload, args.seed),
                     "algorithmic_bytes": alg_bytes, "kernel_ms": fit_kernel_ms},
        "gen_seconds": t_gen,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, args.cpu_sample_gaps)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
