#!/usr/bin/env python3
"""Benchmark of the DuHL hot path on one MI355X.

A step is one round of the scheme over one synthetic problem: full gap evaluation -> top-m
selection -> (column swap) -> one asynchronous coordinate-descent pass over the working set.
Prints ONE JSON line: whole-step coordinate updates/s as `value`, the per-phase figures, the
roofline of the dominant kernel (the dense gap pass, HBM-bound) and the CPU oracle timed beside.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg5] [--no-cpu] [--no-ttg]

The default workload is the fully HBM-resident dense Lasso (50,000 x 500,000 fp32, 100 GB): the
largest single-GPU configuration and the one the bandwidth targets are quoted on.
"""
import argparse
import json

import numpy as np
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E peak


def log(msg):
    """Progress lines go to stderr; stdout carries the one JSON line."""
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)

# HBM bytes per launch of the dominant kernels as the hardware counters see them: measured by the
# profiling step (pmc_traffic.py, two rocprofv3 --pmc runs of this file) and kept in a tracked file.
TRAFFIC_FILE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "traffic.json")


def counter_traffic(workload, which, kernels):
    """Counter-measured bytes of `which` ("gap": per launch, "cd_pass": per pass) for the workload,
    or None if it was not profiled.  The file names the kernels it was made for: if those are no
    longer the kernels this benchmark measures, the figure is stale and the run stops."""
    if not os.path.exists(TRAFFIC_FILE):
        return None
    with open(TRAFFIC_FILE) as f:
        entry = json.load(f).get(workload, {}).get(which)
    if entry is None:
        return None
    if list(entry["kernels"]) != list(kernels):
        raise SystemExit(f"profiles/traffic.json holds {which} traffic of {entry['kernels']} for {workload}, but "
                         f"bench.py measures {kernels}: run the profiling step again (pmc_traffic.py)")
    return entry["bytes_per_launch" if which == "gap" else "bytes_per_pass"]


def dominant_kernels(prob, cd_mode):
    """Names of the kernels behind the two roofline objects, as the profiler prints them."""
    if "cols" in prob:
        # (columns of more than 25,600 entries and at most 49,152 of them per pass: the gap pass that
        # keeps v on chip, in parts of 100 KB)
        count = 2 * prob["m"] if prob["host_resident"] else prob["n"]
        lds = prob["d"] * 4 > 102400 and count <= 49152
        gap = ["gap_dense_lds_kernel", "gap_lds_finish_kernel"] if lds else ["gap_dense_kernel"]
        return gap, (["cd_dense_worker_kernel", "merge_workers_kernel"] if cd_mode == "async"
                     else ["cd_dense_atomic_kernel"])
    return ["csr_sliced_dot_kernel", "csr_blocked_finish_kernel"], ["cd_csr_plan_kernel", "cd_csr_async_kernel"]


def build_problem(name, device, scale, piece_gib=8.0, host_memory="pageable"):
    import torch
    from paper_1708_05357_amd import synth
    cfg = synth.CONFIGS[name]
    out = None
    if cfg.get("host_resident"):
        n = max(8, int(cfg["n"] * scale)) if scale != 1.0 else cfg["n"]
        if host_memory == "pageable":
            # unit A's memory: ordinary host memory, as large as the workload says (80 GB); the
            # library stages what crosses the link through its own pinned buffers
            out = torch.empty((n, cfg["d"]), dtype=torch.float32)
        else:
            # pinned, device-readable host memory in pieces of at most piece_gib (the test machines
            # pin at most 64 GiB in all and about 32 GB in one allocation)
            per = max(1, min(n, int(piece_gib * (1 << 30)) // (4 * cfg["d"])))
            out = [torch.empty((min(per, n - first), cfg["d"]), dtype=torch.float32, pin_memory=True)
                   for first in range(0, n, per)]
    t0 = time.time()
    prob = synth.make(name, seed=0, device=device, scale=scale, out=out)
    torch.cuda.synchronize()
    prob["gen_s"] = time.time() - t0
    prob["host_resident"] = bool(cfg.get("host_resident"))
    prob["pageable"] = prob["host_resident"] and host_memory == "pageable"
    return prob


def make_ctx(prob, budget):
    from paper_1708_05357_amd import duhl
    model = duhl.LASSO if prob["model"] == "lasso" else duhl.SVM
    g = duhl.Duhl(model, prob["d"], prob["n"], budget)
    def set_data():
        if "cols" in prob and isinstance(prob["cols"], list):
            g.set_data_dense_chunks(prob["cols"], prob["target"], prob["lam"])
        elif "cols" in prob:
            g.set_data_dense(prob["cols"], prob["target"], prob["lam"],
                             (duhl.RESIDENT_HOST_PAGEABLE if prob["pageable"] else duhl.RESIDENT_HOST)
                             if prob["host_resident"] else duhl.RESIDENT_DEVICE)
        else:
            g.set_data_csr(prob["rowptr"], prob["colidx"], prob["val"], prob["target"], prob["lam"])
    set_data()
    # A full duhl_gap right after set_data would return the sum of set_data's own pass without
    # computing anything; every gap call timed here must do its work, so the shortcut is switched
    # off for this context (the library drops it once a device pointer to z has been handed out).
    g.device_view(duhl.Z)
    return g, set_data


def make_samples(prob, gap_sample=1.0):
    """The coordinates whose gap-memory entries a round refreshes beside the working set, when not
    all are: 5 % of the columns per round with host residency (Section 5.1) -- a window that slides
    over one random permutation, so every column is refreshed once in 20 rounds -- or the fraction
    asked for with device residency.  Returns (windows as device lists, the same list for unit A's
    host threads), or (None, None) when every gap is refreshed every round."""
    import torch
    if not (prob["host_resident"] or gap_sample < 1.0):
        return None, None
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1)
    windows = 20 if prob["host_resident"] else max(1, int(round(1.0 / max(gap_sample, 1e-6))))
    k = max(1, prob["n"] // windows)
    perm = torch.randperm(prob["n"], generator=gen, device="cuda").to(torch.int32)
    perm = torch.cat([perm, perm[:k]]).contiguous()
    sample_idx = [perm[(r * k) % prob["n"]:(r * k) % prob["n"] + k] for r in range(windows)]
    hp = perm[:prob["n"]].cpu().numpy()
    return sample_idx, {"perm": np.concatenate([hp, hp[:k]]), "cursor": 0, "k": k, "n": prob["n"]}


def measure_brief(name, rounds=10, host_threads=12):
    """One of the other workloads in the same process, with its default settings: a few timed rounds
    from alpha = 0 (per-phase times from events on the compute stream) and the time to total gap 1e-3."""
    import gc
    import torch
    from paper_1708_05357_amd import duhl
    prob = build_problem(name, "cuda", 1.0)
    m, host = prob["m"], prob["host_resident"]
    if not host:
        rounds = 2 * rounds      # (short rounds: enough of them that the median is past the halved bound of the start)
    g, set_data = make_ctx(prob, 2 * m if host else m)
    passes = 8 if host else 1
    threads = host_threads if host else 0
    sample_idx, sample_host = make_samples(prob)
    for s in range(2):
        one_step(g, prob, m, s, sample_idx=sample_idx, passes=passes, host_threads=threads, sample_host=sample_host)
    auto = None
    if host:
        # as `--workload cfg4` does: at least 8 passes per round, more while the round's copies run
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(g.compute_stream)
        g.cd_epoch(duhl.CD_ASYNC, seed=99)
        e1.record(g.compute_stream)
        torch.cuda.synchronize()
        auto = {"cd_ms": e0.elapsed_time(e1), "link_GBps": 55.0, "max_passes": 96, "passes": [], "min_passes": passes}
    set_data()
    if sample_host is not None:
        sample_host["cursor"] = 0
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(rounds)]
    swap_log = [] if host else None
    t0 = time.time()
    for s in range(rounds):
        one_step(g, prob, m, s, evs[s], sample_idx, passes=0 if host else passes, swap_log=swap_log,
                 host_threads=threads, sample_host=sample_host, auto=auto)
    torch.cuda.synchronize()
    elapsed = time.time() - t0
    steps_kept = g.cd_stats()[2]
    med = lambda x: sorted(x)[len(x) // 2]
    gap_ms = med([e[0].elapsed_time(e[1]) for e in evs])
    per_round = auto["passes"] if host else [passes] * rounds
    cd_ms = med([e[2].elapsed_time(e[3]) / k for e, k in zip(evs, per_round)])
    gap_bytes, cd_bytes = algorithmic_bytes(prob, m)
    if host:
        gap_bytes = 4.0 * prob["d"] * g.resident_columns()
    out = {"workload": f"{prob['model']} d={prob['d']} n={prob['n']} m={m}"
                       + (" host-resident (pageable memory)" if host else ""),
           "rounds": rounds, "passes_per_round": per_round if host else passes, "updates_per_s": steps_kept / elapsed,
           "steps_kept": steps_kept, "steps_enqueued": m * sum(per_round),
           "ms_per_round": elapsed / rounds * 1e3, "gap_ms": gap_ms, "cd_pass_ms": cd_ms,
           "gap_GBps": gap_bytes / (gap_ms * 1e-3) / 1e9, "gap_frac": gap_bytes / (gap_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
           "cd_updates_per_s": m / (cd_ms * 1e-3), "cd_GBps": cd_bytes / (cd_ms * 1e-3) / 1e9,
           "cd_frac": cd_bytes / (cd_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS}
    if "val" in prob:
        nnz_pass = float(prob["val"].numel()) / prob["n"] * (steps_kept / sum(per_round))
        rate = g.probe_scatter_add(20_000_000, reps=3)
        out["cd_scatter_add_bound"] = {"adds_per_pass": nnz_pass, "adds_per_s_measured_peak": rate,
                                       "floor_ms": nnz_pass / rate * 1e3, "frac": nnz_pass / rate * 1e3 / cd_ms}
    if host:
        sw = [x for x in swap_log if "columns" in x]
        out["columns_swapped_per_round"] = [x["columns"] for x in sw]
        out["copy_ms_per_round"] = [round(x["copy_ms"], 3) for x in sw]
        out["hidden_frac_per_round"] = [round(min(x["copy_ms"], e[2].elapsed_time(e[3])) / x["copy_ms"], 3)
                                        if x["overlapped"] and x["copy_ms"] > 0 else 0.0 for x, e in zip(sw, evs)]
    if sample_host is not None:
        sample_host["cursor"] = 0
    if auto is not None:
        auto["passes"] = []
    ttg = time_to_gap(g, set_data, prob, m, 1e-3, 400, passes=0 if host else passes, sample_idx=sample_idx,
                      host_threads=threads, sample_host=sample_host, auto=auto)
    out["cd_guard"] = dict(zip(("passes_damped", "max_inflight_now"), g.cd_stats()[:2]))
    out["time_to_gap_s"] = ttg["abs_1e-3_s"]
    out["time_to_gap_rounds"] = ttg["rounds"]
    out["time_to_rel_gap_s"] = ttg["rel_1e-3_s"]
    g.close()
    del g, set_data, prob, sample_idx, sample_host
    gc.collect()
    torch.cuda.empty_cache()
    if hasattr(torch._C, "_host_emptyCache"):
        torch._C._host_emptyCache()
    return out


def algorithmic_bytes(prob, m):
    """Bytes one launch must move at least: the matrix once per gap pass (plus alpha, z), the
    working set once per CD pass."""
    d, n = prob["d"], prob["n"]
    if "cols" in prob:
        return 4.0 * d * n + 8.0 * n, 4.0 * d * m
    nnz = int(prob["val"].numel())
    per = 8.0 * nnz / n
    return 8.0 * nnz + 8.0 * (n + 1) + 12.0 * n, per * m + 8.0 * m


def one_step(g, prob, m, step, ev=None, sample_idx=None, mode=1, inflight=0, swap_log=None,
             rule=0, passes=1, host_threads=0, sample_host=None, auto=None):
    """gap -> select -> commit -> epoch.  With host residency the gaps are refreshed for the
    resident columns plus a sample of the others (stale gap memory, Section 4.1), and the copies
    of the next working set run on the side stream while the pass works on the current one."""
    if ev:
        ev[0].record()
    on_host = prob["host_resident"] and host_threads > 0 and sample_host is not None
    if not prob["host_resident"] and sample_idx is not None:
        # device-resident matrix with a gap memory kept stale on purpose (--gap-sample): only the
        # working set just updated and this round's sample are refreshed
        refreshed = g.working_set_size()
        if refreshed > 0:
            from paper_1708_05357_amd import duhl
            g.gap(g.device_view(duhl.P), want_sum=False)
    else:
        refreshed = g.working_set_size() if prob["host_resident"] else prob["n"]
        g.gap(want_sum=False)
    if sample_idx is not None and not on_host:
        g.gap(sample_idx[step % len(sample_idx)], want_sum=False)
        if not prob["host_resident"]:           # (host residency: the sample crosses the link and is
            refreshed += sample_idx[step % len(sample_idx)].numel()   # not part of the HBM figure)
    if ev:
        ev[1].record()
    stats = g.select(m, want_stats=swap_log is not None or passes == 0, rule=rule, arg=step)
    overlapped = prob["host_resident"] and g.working_set_size() > 0
    if passes == 0:
        # theta chosen per round so that the passes take about as long as the column copies they
        # run beside (Section 5.2): copy time from the number of columns the selection replaces
        passes = auto["min_passes"] if auto is not None else 1
        if auto is not None and overlapped and stats[0] > 0:
            copy_ms = stats[0] * 4.0 * prob["d"] / (auto["link_GBps"] * 1e6)
            passes = int(min(auto["max_passes"], max(passes, round(copy_ms / auto["cd_ms"]))))
        if auto is not None:
            auto["passes"].append(passes)
    if not overlapped:
        g.commit_swap()
    if ev:
        ev[2].record()
    if on_host:                                 # unit A samples gaps while unit B runs the pass
        # the list continues where the previous round was stopped, so that every column is
        # refreshed once per sweep of the permutation however long the rounds are
        perm, cur, k = sample_host["perm"], sample_host["cursor"], sample_host["k"]
        g.host_sample_begin(perm[cur:cur + k], host_threads)
    for k in range(passes):                     # passes per round: the accuracy knob theta (Section 5.2)
        g.cd_epoch(mode, seed=step * (passes if auto is None else 1000) + k, max_inflight=inflight)
    if ev:
        ev[3].record()
    if on_host:
        g.compute_stream.synchronize()          # unit A samples while unit B works: the pass and the copies
        g.copy_stream.synchronize()
        done = g.host_sample_end(wait_all=False)
        sample_host["cursor"] = (cur + max(done - 2 * host_threads, 0)) % sample_host["n"]
        if swap_log is not None:
            swap_log.append({"host_sampled": done})
    if overlapped:
        g.commit_swap()
    if swap_log is not None:
        copy_ms = g.swap_stats()[1] if prob["host_resident"] else 0.0    # the library's own clock of the copies
        swap_log.append({"columns": stats[0], "rho": stats[1], "overlapped": bool(overlapped), "copy_ms": copy_ms})
    return refreshed                            # gaps evaluated by the GPU from HBM in this round


def time_to_gap(g, set_data, prob, m, target, max_rounds, mode=1, inflight=0, sample_idx=None,
                rule=0, passes=1, host_threads=0, sample_host=None, auto=None):
    """Time of the rounds, from alpha = 0, until the total duality gap of a fresh full pass is
    <= target (absolute, with the paper's 1/d or 1/n normalisation) and <= target * O(alpha=0)
    (target * gap(alpha=0) for the SVM dual, whose objective is 0 at alpha = 0).
    Device residency: the round's own full gap pass is the check.  Host residency, or a gap
    memory kept stale on purpose: the rounds use stale gaps (working set + sample); the check
    is an extra full pass that is not part of the scheme, so it is left out of the clock and z
    is restored after it."""
    import torch
    from paper_1708_05357_amd import duhl
    set_data()
    o0 = g.objective()
    host = prob["host_resident"] or sample_idx is not None     # rounds run on a stale gap memory
    all_idx = torch.arange(prob["n"], dtype=torch.int32, device="cuda") if prob["host_resident"] else None
    torch.cuda.synchronize()
    t_abs = t_rel = None
    clock = 0.0
    rounds = 0
    gap0 = None
    gap = float("inf")
    check_every = 4 if prob["host_resident"] else 1   # host: each check is a pass over host memory
    if prob["host_resident"]:
        max_rounds = min(max_rounds, 160)
    for rnd in range(max_rounds):
        t0 = time.time()
        if host:
            if rnd > 0:
                one_step(g, prob, m, rnd, sample_idx=sample_idx, mode=mode, inflight=inflight, rule=rule,
                         passes=passes, host_threads=host_threads, sample_host=sample_host, auto=auto)
            torch.cuda.synchronize()
            clock += time.time() - t0
            if rnd % check_every != 0:
                rounds = rnd + 1
                continue
            keep = g.get(duhl.Z)
            gap = g.gap(all_idx) if all_idx is not None else g.gap()
            g.set(duhl.Z, keep)
            log(f"time-to-gap: round {rnd} total gap {gap:.3e} clock {clock:.3f}s")
        else:
            gap = g.gap()
            clock += time.time() - t0
        if gap0 is None:
            gap0 = gap
        if t_abs is None and gap <= target:
            t_abs = clock
        if t_rel is None and gap <= target * (abs(o0) if o0 != 0.0 else gap0):
            t_rel = clock
        if t_abs is not None and t_rel is not None:
            break
        if not host:
            t0 = time.time()
            g.select(m, want_stats=False, rule=rule, arg=rnd)
            g.commit_swap()
            for k in range(max(passes, 1)):
                g.cd_epoch(mode, seed=1000 + rnd * passes + k, max_inflight=inflight)
            clock += time.time() - t0
        elif rnd == 0:
            t0 = time.time()
            one_step(g, prob, m, 0, sample_idx=sample_idx, mode=mode, inflight=inflight, rule=rule, passes=passes,
                     host_threads=host_threads, sample_host=sample_host, auto=auto)
            torch.cuda.synchronize()
            clock += time.time() - t0
        rounds = rnd + 1
    return {"abs_1e-3_s": t_abs, "rel_1e-3_s": t_rel, "rounds": rounds, "final_gap": gap,
            "gap_at_zero": gap0, "objective_at_zero": o0, "final_objective": g.objective(),
            "passes_per_round": passes if passes > 0 else auto["passes"]}


def time_to_gap_native(g, set_data, prob, m, target, mode, inflight, rule, passes, sample_perm, host_threads,
                       extra_passes=0):
    """The same measurement with the round loop run by the library (duhl_run): no interpreter
    between the steps, one read-back of the gap-memory sum per round as the stopping test.  With
    a device-resident matrix that sum is the total gap of a fresh full pass.  With host residency
    it is built from stale entries (working set + 5 % window per round) and only an estimate, so
    the loop confirms it with a full refresh over the host link before it stops -- inside the
    clock, unlike the checks of time_to_gap above."""
    import torch
    out = {}
    passes = max(passes, 1)
    for name in ("abs", "rel"):
        set_data()
        o0 = g.objective()
        tol = target if name == "abs" else target * (abs(o0) if o0 != 0.0 else g.gap())
        torch.cuda.synchronize()
        kw = {}
        if prob["host_resident"]:
            kw = dict(sample=sample_perm, sample_per_round=max(1, prob["n"] // 20), host_threads=host_threads,
                      confirm=True, max_extra_passes=extra_passes)
        st = g.run(m, 400, passes=passes, mode=mode, gap_tol=tol, max_inflight=inflight, rule=rule,
                   seed=1000, **kw)
        out[f"{name}_1e-3_s"] = st["seconds"] if st["converged"] else None
        out[f"{name}_rounds"] = st["rounds"]
        out[f"{name}_passes"] = st["passes"]
        out[f"{name}_gap_memory_sum"] = st["gap_memory_sum"]
        out[f"{name}_confirmations"] = st["confirmations"]
        if prob["host_resident"]:
            all_idx = torch.arange(prob["n"], dtype=torch.int32, device="cuda")
            out[f"{name}_true_total_gap"] = g.gap(all_idx)
        else:
            out[f"{name}_true_total_gap"] = g.gap()
    out["passes_per_round"] = passes
    if not prob["host_resident"]:
        # the same loop choosing its own passes per round (options passes = 0: one pass in the first
        # round, then round(sqrt(refresh time / pass time)) + 1)
        set_data()
        torch.cuda.synchronize()
        st = g.run(m, 400, passes=0, mode=mode, gap_tol=target, max_inflight=inflight, rule=rule, seed=1000)
        out["auto_passes"] = {"abs_1e-3_s": st["seconds"] if st["converged"] else None, "rounds": st["rounds"],
                              "passes": st["passes"], "passes_per_round": st["passes_per_round"],
                              "true_total_gap": g.gap()}
    return out


def host_description():
    """CPU model, logical CPUs and memory of the machine the baseline ran on."""
    model, mem_gb = "unknown", None
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
        with open("/proc/meminfo") as f:
            mem_gb = round(int(f.readline().split()[1]) / 1e6)
    except OSError:
        pass
    return {"cpu": model, "logical_cpus": os.cpu_count(), "memory_GB": mem_gb}


def cpu_baseline(prob, m, budget_s=20.0):
    """The oracle as it stands, single thread, on the same inputs: rounds of full gap pass,
    selection and one CD pass from alpha = 0, for about budget_s seconds (at least one round;
    on a column subsample when a round would not fit)."""
    import numpy as np
    from oracle import duhl_oracle as orc
    model = orc.LASSO if prob["model"] == "lasso" else orc.SVM
    n, d = prob["n"], prob["d"]
    sample = "full workload"
    frac = 1.0
    if "cols" in prob:
        bytes_total = 4.0 * n * d
        if bytes_total > 8e9:                       # too large for the host: column subsample
            frac = 8e9 / bytes_total
        ns = int(n * frac)
        if isinstance(prob["cols"], list):          # host matrix in pieces: the first ns columns
            import torch
            cols = torch.cat([t[:max(0, ns - k * prob["cols"][0].shape[0])] for k, t in enumerate(prob["cols"])
                              if ns > k * prob["cols"][0].shape[0]]).numpy()
        else:
            cols = prob["cols"][:ns].cpu().numpy()
        o = orc.Oracle(model, prob["target"].cpu().numpy(), prob["lam"], cols=cols)
    else:
        ns = n
        o = orc.Oracle(model, prob["target"].cpu().numpy(), prob["lam"],
                       csr=(prob["rowptr"].cpu().numpy(), prob["colidx"].cpu().numpy(),
                            prob["val"].cpu().numpy()), d=d)
    ms = max(1, int(m * frac))
    if frac < 1.0:
        sample = f"first {ns} of {n} columns at full length, m scaled to {ms}; rate is per update"
    rng = np.random.default_rng(0)
    t_gap = t_cd = 0.0
    rounds = 0
    t_start = time.time()
    while True:
        t0 = time.time()
        o.gaps()
        t1 = time.time()
        P = o.select(ms)
        order = P[rng.permutation(P.size)]
        t2 = time.time()
        o.cd_pass(order)
        t3 = time.time()
        t_gap += t1 - t0
        t_cd += t3 - t2
        rounds += 1
        if time.time() - t_start > budget_s or rounds >= 50:
            break
    total = time.time() - t_start
    gap_bytes = 4.0 * d * ns if "cols" in prob else 8.0 * prob["val"].numel()
    # The gap pass alone on several host cores: the same oracle routine called from a thread per
    # slice of the coordinates (the calls release the interpreter lock and write disjoint entries of
    # z).  The coordinate-descent pass is sequential by definition and stays on one core.
    from concurrent.futures import ThreadPoolExecutor
    threads = 12                                    # a one-GPU share of the host's cores
    slices = [s.astype(np.int32) for s in np.array_split(np.arange(ns), threads)]
    with ThreadPoolExecutor(threads) as ex:
        list(ex.map(o.gaps, slices))                # warm
        t0 = time.time()
        list(ex.map(o.gaps, slices))
        t_par = time.time() - t0
    return {"value": ms * rounds / total, "unit": "coordinate updates/s", "cores": 1, "kind": "oracle",
            "sample": f"{sample}; {rounds} rounds of gap pass + top-m + one CD pass, fp64, 1 thread",
            "gap_pass_s": t_gap / rounds, "cd_pass_s": t_cd / rounds,
            "gap_GBps": gap_bytes / (t_gap / rounds) / 1e9,
            "cd_updates_per_s": ms / (t_cd / rounds),
            "gap_pass_threads": threads, "gap_pass_s_threads": t_par, "gap_GBps_threads": gap_bytes / t_par / 1e9,
            "host": host_description()}


def cpu_time_to_gap(prob, m, target, budget_s):
    """The paper's CPU reference point (Section 5.3: one thread of coordinate descent over all
    coordinates) and the oracle's own DuHL rounds, each from alpha = 0 until the total gap of a
    full pass is <= target or budget_s seconds have gone by.  Whole workload only.  Coordinate
    descent over everything does not need gaps, so its gap passes (one per pass, the stopping
    test) stay out of its clock; a DuHL round's gap pass drives the selection and stays in."""
    import numpy as np
    from oracle import duhl_oracle as orc
    model = orc.LASSO if prob["model"] == "lasso" else orc.SVM
    n = prob["n"]

    def fresh():
        if "cols" in prob:
            return orc.Oracle(model, prob["target"].cpu().numpy(), prob["lam"], cols=prob["cols"].cpu().numpy())
        return orc.Oracle(model, prob["target"].cpu().numpy(), prob["lam"],
                          csr=(prob["rowptr"].cpu().numpy(), prob["colidx"].cpu().numpy(),
                               prob["val"].cpu().numpy()), d=prob["d"])
    out = {"target_total_gap": target, "cores": 1, "kind": "oracle"}
    o = fresh()
    rng = np.random.default_rng(0)
    clock, rounds, gap = 0.0, 0, float("inf")
    while clock < budget_s:
        t0 = time.time()
        gap = o.gaps()
        if gap <= target:
            clock += time.time() - t0
            break
        P = o.select(m)
        o.cd_pass(P[rng.permutation(P.size)])
        clock += time.time() - t0
        rounds += 1
        log(f"cpu time-to-gap: DuHL round {rounds}, {clock:.2f}s, gap before it {gap:.3e}")
    out["duhl_rounds_of_one_pass"] = {"seconds": clock if gap <= target else None, "rounds": rounds,
                                      "total_gap": gap}
    log(f"cpu time-to-gap: DuHL rounds {rounds}, {clock:.2f}s, gap {gap:.3e}")
    o = fresh()
    rng = np.random.default_rng(0)
    clock, passes, gap = 0.0, 0, float("inf")
    while clock < budget_s:
        gap = o.gaps()                              # stopping test, not part of the solver
        if gap <= target:
            break
        t0 = time.time()
        o.cd_pass(rng.permutation(n).astype(np.int32))
        clock += time.time() - t0
        passes += 1
        log(f"cpu time-to-gap: CD pass {passes}, {clock:.2f}s, gap before it {gap:.3e}")
    out["coordinate_descent_over_all"] = {"seconds": clock if gap <= target else None, "passes": passes,
                                          "total_gap": gap}
    log(f"cpu time-to-gap: CD over all coordinates, passes {passes}, {clock:.2f}s, gap {gap:.3e}")
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg5", choices=["cfg1", "cfg2", "cfg2clustered", "cfg3", "cfg4", "cfg5", "cfg5clustered", "fig5svm", "sec51lasso",
                                                            "sec51svm"])
    ap.add_argument("--scale", type=float, default=1.0, help="shrink n (and m) at fixed d")
    ap.add_argument("--host-memory", default="pageable", choices=["pageable", "pinned"],
                    help="host residency (cfg4): the matrix in ordinary host memory, staged by the library "
                         "through pinned buffers (any size), or in pinned device-readable memory (the test "
                         "machines pin at most 64 GiB: --scale 0.8 or less)")
    ap.add_argument("--budget-factor", type=float, default=2.0,
                    help="device slots per working-set column (host residency)")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-ttg", action="store_true")
    ap.add_argument("--no-others", action="store_true",
                    help="default workload only: leave out the short runs of the other workloads")
    ap.add_argument("--cpu-ttg", type=float, default=0.0,
                    help="also time the oracle to total gap 1e-3 on one host core, for at most this many "
                         "seconds per scheme (whole workload in host memory: cfg1-cfg3 only)")
    ap.add_argument("--copy-calibration-gib", type=float, default=0.0,
                    help="also run plain device copies of this size (GiB), as a yardstick for the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run")
    ap.add_argument("--cd-mode", default="async", choices=["async", "atomic"],
                    help="concurrent CD scheme: the library's default, or per-update atomics")
    ap.add_argument("--inflight", type=int, default=0, help="max_inflight of duhl_cd_epoch (0 = default)")
    ap.add_argument("--select-rule", default="gap", choices=["gap", "random", "block"],
                    help="working-set rule: eq. (13), or one of the paper's reference schemes")
    ap.add_argument("--passes", type=int, default=None,
                    help="CD passes per round (theta of Section 5.2); 0 with host residency: as many, "
                         "up to 8, as fit beside the round's column copies; default 1, and 8 with host "
                         "residency, where the passes are also the time unit A's sampler has per round")
    ap.add_argument("--min-passes", type=int, default=1, help="lower bound for --passes 0")
    ap.add_argument("--max-passes", type=int, default=8, help="upper bound for --passes 0")
    ap.add_argument("--gap-sample", type=float, default=1.0,
                    help="device residency: refresh only the working set and this fraction of all "
                         "coordinates per round (stale gap memory, Section 4.1) instead of every gap")
    ap.add_argument("--host-sampler-threads", type=int, default=-1,
                    help="host residency: refresh the gap sample with this many host threads while the "
                         "GPU runs the pass (unit A's loop of Algorithm 2); 0: the GPU evaluates the sample "
                         "over the host link instead; default 12 (a one-GPU share of the host's cores)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures the single-GPU hot path; this build has no multi-GPU path "
              "(--gpus must be 1)", file=sys.stderr)
        sys.exit(2)

    if args.host_sampler_threads < 0:
        args.host_sampler_threads = 12
    if args.passes is None:
        # host residency: at least 8 passes per round, and as many more as fit beside the round's column
        # copies (theta sized to the copy, Section 5.2) -- the device would otherwise wait for the link
        args.passes = 0 if args.workload == "cfg4" else 1
        if args.workload == "cfg4":
            args.min_passes, args.max_passes = max(args.min_passes, 8), max(args.max_passes, 96)
    import torch
    from paper_1708_05357_amd import duhl
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    log(f"generating {args.workload} (scale {args.scale})")
    prob = build_problem(args.workload, "cuda", args.scale, host_memory=args.host_memory)
    log(f"generated in {prob['gen_s']:.1f}s; setting data")
    m = prob["m"]
    budget = int(m * args.budget_factor) if prob["host_resident"] else m
    g, set_data = make_ctx(prob, budget)
    mode = duhl.CD_ASYNC if args.cd_mode == "async" else duhl.CD_ATOMIC
    rule = {"gap": duhl.SELECT_GAP, "random": duhl.SELECT_RANDOM, "block": duhl.SELECT_BLOCK}[args.select_rule]
    sample_idx, sample_host = make_samples(prob, args.gap_sample)
    log(f"warm-up: {args.warmup} rounds")
    for s in range(args.warmup):
        one_step(g, prob, m, s, sample_idx=sample_idx, mode=mode, inflight=args.inflight, rule=rule,
                 passes=max(args.passes, 1), host_threads=args.host_sampler_threads, sample_host=sample_host)
    torch.cuda.synchronize()
    auto = None
    if args.passes == 0:
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(g.compute_stream)
        g.cd_epoch(mode, seed=99, max_inflight=args.inflight)
        e1.record(g.compute_stream)
        torch.cuda.synchronize()
        # 55 GB/s: what the copy kernel sustains on the host link of the test machines
        auto = {"cd_ms": e0.elapsed_time(e1), "link_GBps": 55.0, "max_passes": args.max_passes, "passes": [],
                "min_passes": args.min_passes}
    set_data()                                  # back to alpha = 0: the timed rounds are rounds 1..K
    torch.cuda.synchronize()

    host = prob["host_resident"]
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    swap_log = [] if host else None
    torch.cuda.synchronize()
    t0 = time.time()
    refreshed = 0
    for s in range(args.steps):
        refreshed += one_step(g, prob, m, s, evs[s], sample_idx, mode, args.inflight, swap_log, rule, args.passes,
                              args.host_sampler_threads, sample_host, auto)
    total_passes = args.passes * args.steps if auto is None else sum(auto["passes"])
    # Coordinate steps that count: those of the passes the guard let stand, as the device counted them
    # (a pass undone because the objective rose is work thrown away, and a pass enqueued before the
    # host knew of a halving solves only part of its working set).  Per-update atomics are unguarded.
    guard_undone, guard_inflight, steps_kept, _ = g.cd_stats()
    steps_done = steps_kept if args.cd_mode == "async" and os.environ.get("DUHL_CD_GUARD", "1") != "0" \
        else m * total_passes
    passes_timed = None if auto is None else list(auto["passes"])
    torch.cuda.synchronize()
    elapsed = time.time() - t0
    log(f"timed {args.steps} rounds in {elapsed:.3f}s")

    gap_ms = [e[0].elapsed_time(e[1]) for e in evs]
    sel_ms = [e[1].elapsed_time(e[2]) for e in evs]
    cd_ms = [e[2].elapsed_time(e[3]) for e in evs]
    avg = lambda x: sum(x) / len(x)
    gap_bytes, cd_bytes = algorithmic_bytes(prob, m)
    if prob["host_resident"]:
        # The pass refreshes every column held in a device slot: the working set and whatever
        # earlier members have not been evicted yet, counted after the timed rounds (the number
        # settles once the slots are full).  The sample of the other columns is link- or
        # host-bound and not part of this figure.
        resident = g.resident_columns()
        gap_bytes = 4.0 * prob["d"] * resident
    elif sample_idx is not None:
        gap_bytes *= refreshed / args.steps / prob["n"]        # working set + sample, as refreshed
    # (host residency: the slots fill up over the first rounds, so the settled count of resident
    # columns goes with the median pass time, not the mean)
    gap_time = sorted(gap_ms)[len(gap_ms) // 2] if prob["host_resident"] else avg(gap_ms)
    gap_gbps = gap_bytes / (gap_time * 1e-3) / 1e9
    cd_gbps = cd_bytes * (steps_done / m) / args.steps / (avg(cd_ms) * 1e-3) / 1e9
    final_gap = g.gap() if not prob["host_resident"] else None   # (fresh z; rounds are over)
    # yardstick: a plain read-only streaming kernel over the same device memory the gap pass reads
    stream_gbps = None
    if "cols" in prob and not prob["host_resident"] and prob["cols"].is_contiguous():
        stream_gbps = prob["cols"].numel() * 4.0 / (g.probe_stream_read(prob["cols"], reps=3) * 1e-3) / 1e9
    final_obj = g.objective()
    gap_kernels, cd_kernels = dominant_kernels(prob, args.cd_mode)
    # yardstick of the CSR pass: one fp32 atomic add to v per non-zero of every row stepped on; the
    # device performs such adds at a fixed rate, measured here on this problem's own v
    scatter = None
    if "val" in prob:
        nnz_pass = float(prob["val"].numel()) / prob["n"] * m * (steps_done / (m * total_passes))
        rate = g.probe_scatter_add(20_000_000, reps=3)
        pass_ms = avg(cd_ms) / (total_passes / args.steps)
        scatter = {"adds_per_pass": nnz_pass, "adds_per_s_measured_peak": rate, "floor_ms": nnz_pass / rate * 1e3,
                   "achieved_adds_per_s": nnz_pass / (pass_ms * 1e-3), "frac": nnz_pass / rate * 1e3 / pass_ms}

    out = {
        "metric": "coordinate updates/s (whole round: gap pass + top-m + CD pass)",
        "value": steps_done / elapsed,
        "unit": "coordinate updates/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {prob['model']} d={prob['d']} n={prob['n']} m={m}"
                               + (f" host-resident ({args.host_memory} memory), {budget} device slots"
                                  if prob["host_resident"] else ""),
                   "scale": args.scale, "rounds_timed": args.steps, "passes_per_round": args.passes if auto is None else passes_timed,
                   "cd_scheme": args.cd_mode, "max_inflight": args.inflight, "select_rule": args.select_rule,
                   "gap_sample": args.gap_sample,
                   "host_sampler_threads": args.host_sampler_threads if prob["host_resident"] else None,
                   "resident_columns": g.resident_columns() if prob["host_resident"] else None},
        "phases": {"gap_ms": avg(gap_ms), "select_ms": avg(sel_ms), "cd_ms": avg(cd_ms),
                   "gap_GBps": gap_gbps, "gap_frac_of_hbm_peak": gap_gbps / HBM_PEAK_GBPS,
                   "cd_updates_per_s": steps_done / args.steps / (avg(cd_ms) * 1e-3), "cd_GBps": cd_gbps,
                   "cd_frac_of_hbm_peak": cd_gbps / HBM_PEAK_GBPS,
                   "gap_ms_min": min(gap_ms), "cd_ms_min": min(cd_ms), "cd_ms_max": max(cd_ms),
                   "gap_ms_median": sorted(gap_ms)[len(gap_ms) // 2], "cd_ms_median": sorted(cd_ms)[len(cd_ms) // 2],
                   # host residency: the first round's selection waits for the whole working set to
                   # arrive over the link, which dominates the mean
                   "select_ms_median": sorted(sel_ms)[len(sel_ms) // 2]},
        "roofline": {"kernel": " + ".join(gap_kernels),
                     "bound": "hbm", "achieved": gap_gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": gap_gbps / HBM_PEAK_GBPS,
                     "traffic": counter_traffic(args.workload, "gap", gap_kernels)
                     if args.scale == 1.0 and sample_idx is None else None,
                     "algorithmic_bytes": gap_bytes, "avg_launch_ms": gap_time,
                     "stream_read_GBps": stream_gbps,
                     "frac_of_stream_read": gap_gbps / stream_gbps if stream_gbps else None},
        "roofline_cd": {"kernel": " + ".join(cd_kernels) + " (one pass)",
                        "bound": "hbm", "achieved": cd_gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                        "frac": cd_gbps / HBM_PEAK_GBPS,
                        "traffic": counter_traffic(args.workload, "cd_pass", cd_kernels)
                        if args.scale == 1.0 and args.cd_mode == "async" and args.inflight == 0 else None,
                        "algorithmic_bytes": cd_bytes, "avg_launch_ms": avg(cd_ms),
                        "frac_of_stream_read": cd_gbps / stream_gbps if stream_gbps else None,
                        "scatter_add_bound": scatter},
        "after_timed_rounds": {"total_gap": final_gap, "objective": final_obj},
        # the device-side guard of the concurrent passes: passes undone because the objective had risen
        # (since the data were set for the timed rounds), and the bound on concurrent steps now
        "cd_guard": {"passes_damped": guard_undone, "max_inflight_now": guard_inflight, "steps_kept": steps_kept,
                     "steps_enqueued": m * total_passes},
        "gen_s": prob["gen_s"],
    }
    if host:
        # column swap (Algorithm 2, the step that refreshes the memory of unit B): copies start after the selection and run
        # on the side stream; how much of them the concurrent pass hides
        rows = []
        sampled = [x["host_sampled"] for x in swap_log if "host_sampled" in x]
        swap_log = [x for x in swap_log if "columns" in x]
        for e, sw in zip(evs, swap_log):
            copy_ms = sw["copy_ms"]
            cd = e[2].elapsed_time(e[3])
            rows.append({"columns": sw["columns"], "copy_ms": copy_ms, "cd_ms": cd,
                         "overlapped": sw["overlapped"], "rho": sw["rho"],
                         "hidden_frac": (min(copy_ms, cd) / copy_ms) if sw["overlapped"] and copy_ms > 0 else 0.0})
        moved = sum(r["columns"] for r in rows if r["overlapped"])
        busy = sum(r["copy_ms"] for r in rows if r["overlapped"] and r["columns"] > 0)
        out["swap"] = {"columns_per_round": [r["columns"] for r in rows],
                       "copy_ms_per_round": [round(r["copy_ms"], 3) for r in rows],
                       "host_link_GBps": (moved * 4.0 * prob["d"] / (busy * 1e-3) / 1e9) if busy > 0 else None,
                       "hidden_frac_per_round": [round(r["hidden_frac"], 3) for r in rows],
                       "rho_per_round": [round(r["rho"], 2) for r in rows],
                       "host_sampled_per_round": sampled}
    if not args.no_ttg:
        log("time to gap 1e-3")
        if auto is not None:
            auto["passes"] = []
        out["time_to_gap"] = time_to_gap(g, set_data, prob, m, 1e-3, 400, mode, args.inflight, sample_idx, rule, args.passes,
                                         args.host_sampler_threads, sample_host, auto)
    if not args.no_ttg and args.passes == 1 and not prob["host_resident"] and args.gap_sample >= 1.0:
        # theta is the method's own knob (Section 5.2): with the matrix in HBM a gap pass costs
        # several CD passes, so more than one pass per round reaches the gap sooner
        log("time to gap 1e-3 with 4 passes per round")
        out["time_to_gap_4_passes"] = time_to_gap(g, set_data, prob, m, 1e-3, 400, mode, args.inflight, None, rule, 4)
    if not args.no_ttg and args.gap_sample >= 1.0:
        log("time to gap 1e-3, native round loop")
        perm_dev = None
        if prob["host_resident"]:
            perm_dev = torch.as_tensor(sample_host["perm"][:prob["n"]], device="cuda").contiguous()
        out["time_to_gap_native"] = time_to_gap_native(g, set_data, prob, m, 1e-3, mode, args.inflight, rule,
                                                       args.passes if args.passes > 0 else args.min_passes, perm_dev,
                                                       args.host_sampler_threads,
                                                       extra_passes=(args.max_passes - args.min_passes) if args.passes == 0 else 0)
    if not args.no_cpu:
        log("CPU baseline (oracle, one thread, about 20 s)")
        out["cpu_baseline"] = cpu_baseline(prob, m)
    else:
        out["cpu_baseline"] = None
    if args.cpu_ttg > 0:
        if prob["host_resident"] or 4.0 * prob["n"] * prob["d"] > 8e9 and "cols" in prob:
            log("--cpu-ttg: the workload does not fit the oracle whole; skipped")
        else:
            out["cpu_time_to_gap"] = cpu_time_to_gap(prob, m, 1e-3, args.cpu_ttg)
    g.close()
    if args.workload == "cfg5" and not args.no_others and args.scale == 1.0:
        # the other workloads of the method, each with its default settings, in the same process
        import gc
        del g, set_data, prob, sample_idx, sample_host, evs
        gc.collect()
        torch.cuda.empty_cache()
        out["other_workloads"] = {}
        for name in ("cfg1", "cfg2", "cfg2clustered", "cfg3", "cfg4"):
            log(f"other workloads: {name}")
            try:
                out["other_workloads"][name] = measure_brief(name, host_threads=args.host_sampler_threads)
            except (RuntimeError, MemoryError) as e:         # e.g. not enough host memory for the 80 GB matrix
                out["other_workloads"][name] = {"skipped": str(e)[:200]}
    if args.copy_calibration_gib > 0:
        nfl = int(args.copy_calibration_gib * (1 << 30) / 4)
        src = torch.ones(nfl, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        out["copy_calibration"] = {"bytes_read": nfl * 4, "bytes_written": nfl * 4, "copies": 3}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
