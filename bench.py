#!/usr/bin/env python3
"""Benchmark of the batched execution simulator on one MI355X.

A step is one pass of the whole hot path (task-graph construction + full simulation, one
ff_sim_batch call) over one batch of seeded synthetic candidate strategies that is already
resident in HBM.  The headline workload is the largest configuration, configs[4] (NMT-shaped
graph of 2321 ops, 16x4 simulated devices, 1024 candidates per step); the other four
configurations, the delta chains of configs[4], the search loop and the refinements are
measured the same way and reported beside it.

Prints ONE JSON line.  python bench.py --gpus 1 --steps K --warmup W
       python bench.py --long-chain 10000    (the configuration's 10000-step mutation chain alone)
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X HBM3E, published
HEADLINE = 4
# the chip's vector issue peak: 256 CUs x 4 SIMDs x 2.4 GHz / 4 cycles per 64-lane instruction
VALU_PEAK_G_PER_S = 256 * 4 * 2.4e9 / 4 / 1e9
# rocprofv3 counter readings per launch (HBM traffic from FETCH_SIZE / WRITE_SIZE, instruction
# counts from SQ_INSTS_*), one line per workload with the kernel instantiation they were read for
COUNTER_FILE = os.path.join(ROOT, "profiles", "k_sim_batch_pmc_counters.txt")


def profiled_counters():
    """{config id: {"kernel": name, "B": .., "traffic_bytes": .., "insts_valu": ..}} from the
    tracked summary of the counter runs; {} if there is none."""
    out = {}
    try:
        for line in open(COUNTER_FILE):
            if not line.startswith("counters "):
                continue
            f = dict(kv.split("=", 1) for kv in line.split()[1:] if "=" in kv)
            name = line.split('kernel="', 1)[1].split('"', 1)[0]
            out[int(f["config"])] = {"kernel": name, "B": int(f["B"]), "traffic_bytes": float(f["traffic_bytes"]),
                                     "insts_valu": float(f["insts_valu"])}
    except OSError:
        pass
    return out


def alg_bytes(n_ops, tc, npairs):
    """bytes the method moves per strategy if the task graph is written once and read once:
    strategy in, 40 B per compute task, 28 B per producer/consumer pair, result out."""
    return 8.0 * n_ops + 40.0 * tc + 28.0 * npairs + 8.0


def time_batches(sim, d_strat, B, steps, warmup):
    """wall ms per step over exactly `steps` launches back to back (the timed region of the
    contract), then, in a second pass of as many launches, the per-launch duration (ms) from HIP
    events on the launch stream."""
    import torch
    for _ in range(warmup):
        sim.batch(d_strat, B)
    out = torch.empty(B, dtype=torch.int64, device="cuda")
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        sim.batch(d_strat, B, d_out=out)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for a, b in ev:
        a.record()
        sim.batch(d_strat, B, d_out=out)
        b.record()
    torch.cuda.synchronize()
    kern_ms = [a.elapsed_time(b) for a, b in ev]
    return sum(kern_ms) / len(kern_ms), wall_ms, out


def copy_bandwidth_gbps():
    """what a plain device-to-device copy of 256 MiB reaches on this machine (read + write bytes per
    second): the achievable figure to hold beside the published HBM peak."""
    import torch
    n = 256 * 2 ** 20
    src = torch.empty(n, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(2):
        dst.copy_(src)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(5):
        dst.copy_(src)
    b.record()
    torch.cuda.synchronize()
    return 5 * 2 * n / (a.elapsed_time(b) * 1e-3) / 1e9


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def host_cores():
    """(threads the oracle is run on, logical CPUs of the box, CPUs this process may use)"""
    logical = os.cpu_count() or 1
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = logical
    # a one-GPU machine's CPU share is 16 cores, whatever the host shows
    return max(1, min(usable, 16)), logical, usable


def oracle_build_share(w, cfgs):
    """seconds the oracle spends building task graphs vs. building + simulating, one thread."""
    import oracle
    t0 = time.perf_counter()
    for c in cfgs:
        oracle.build_and_discard(w.ops, w.edges, w.machine, w.cost, c)
    t_build = time.perf_counter() - t0
    t0 = time.perf_counter()
    oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cfgs, n_threads=1)
    t_both = time.perf_counter() - t0
    return t_build, t_both


def timeline_items(w, cfg):
    """the oracle's timeline of one strategy as {task key: (ready, start, end)}; a compute task's
    key is (op, part), a transfer's is (key of its producer task, key of its consumer task)."""
    import numpy as np
    import oracle
    tg = oracle.build_task_graph(w.ops, w.edges, w.machine, w.cost, cfg)
    _, r, s_, e = tg.simulate()
    parts = cfg["deg"].astype(np.int64).prod(axis=1)
    op_of = np.repeat(np.arange(len(parts)), parts)
    part_of = np.concatenate([np.arange(p) for p in parts])
    ckey = op_of * 64 + part_of                                   # compute tasks, in id order
    pred = np.full(tg.n_tasks, -1, np.int64)
    succ = np.full(tg.n_tasks, -1, np.int64)
    comm_dst = tg.dep_dst >= tg.n_compute
    pred[tg.dep_dst[comm_dst]] = tg.dep_src[comm_dst]
    comm_src = tg.dep_src >= tg.n_compute
    succ[tg.dep_src[comm_src]] = tg.dep_dst[comm_src]
    keys = np.empty(tg.n_tasks, np.int64)
    keys[:tg.n_compute] = ckey
    c = np.arange(tg.n_compute, tg.n_tasks)
    keys[c] = (1 << 40) + ckey[pred[c]] * (1 << 19) + ckey[succ[c]]
    return keys, np.stack([r, s_, e], axis=1)


def changed_items(items_a, items_b):
    """Section 5.3's work: tasks removed + tasks inserted + tasks whose ready/start/end differ
    between the timelines of two strategies (counted by the oracle, nothing from the GPU)."""
    import numpy as np
    ka, ta = items_a
    kb, tb = items_b
    oa, ob = np.argsort(ka), np.argsort(kb)
    ka, ta, kb, tb = ka[oa], ta[oa], kb[ob], tb[ob]
    common, ia, ib = np.intersect1d(ka, kb, assume_unique=True, return_indices=True)
    moved = int((ta[ia] != tb[ib]).any(axis=1).sum())
    return {"removed": int(len(ka) - len(common)), "inserted": int(len(kb) - len(common)), "moved": moved,
            "tasks_after": int(len(kb))}


def delta_work_model(w, cfg0, muts, steps):
    """what an exact delta algorithm has to touch on the given steps of a chain: per step the
    oracle's timelines before and after the mutation are diffed."""
    import numpy as np
    want = sorted(int(s) for s in steps)
    cur = np.array(cfg0, copy=True)
    work = []
    for s in range(want[-1] + 1):
        nxt = cur.copy()
        nxt[int(muts[s]["op"])] = muts[s]["cfg"]
        if s in want:
            work.append(changed_items(timeline_items(w, cur), timeline_items(w, nxt)))
        cur = nxt
    return work


def oracle_rate(w, cfgs, threads):
    import oracle
    t0 = time.perf_counter()
    res = oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cfgs, n_threads=threads)
    return len(cfgs) / (time.perf_counter() - t0), res


def oracle_chain_steps(w, cfg0, muts, steps, threads):
    """the oracle's times after the given steps of a mutation chain (full re-simulation of each)"""
    import numpy as np
    import oracle
    want = set(int(s) for s in steps)
    cur = np.array(cfg0, copy=True)
    snaps = []
    for s in range(max(want) + 1):
        cur[int(muts[s]["op"])] = muts[s]["cfg"]
        if s in want:
            snaps.append(cur.copy())
    return oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, np.stack(snaps), n_threads=threads)


def long_chain(n_steps, check, threads):
    """the mutation chain of configs[4] at its full length: n_steps cumulative single-op mutations on
    one chain with delta simulation, in calls of 250 steps (a progress line each), `check` steps
    spread over the chain compared with the oracle."""
    import numpy as np
    import torch
    from paper_1807_05358_amd import binding, workloads as W
    w = W.workload(4)
    cfg0 = w.strategies(1)
    muts = w.mutations(n_steps, 1)
    sim = binding.Simulator(w.ops, w.edges, w.machine, w.cost)
    ch = binding.Chains(sim, cfg0)
    got, gpu_ms = [], 0.0
    t0 = time.perf_counter()
    for a in range(0, n_steps, 250):
        n = min(250, n_steps - a)
        d_m = ch.upload_mutations(muts[a:a + n])
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        out = ch.delta(d_m, n)
        e1.record()
        torch.cuda.synchronize()
        gpu_ms += e0.elapsed_time(e1)
        got.append(out.cpu().numpy().view("<u8")[:, 0])
        print(f"long chain: {a + n} of {n_steps} steps, {gpu_ms / (a + n):.2f} ms per step", file=sys.stderr, flush=True)
    wall = time.perf_counter() - t0
    got = np.concatenate(got)
    st = ch.stats()
    sel = sorted(set(np.linspace(0, n_steps - 1, check).astype(int).tolist()) | {0, n_steps - 1})
    want = oracle_chain_steps(w, cfg0[0], muts[:, 0], sel, threads)
    bad = [s for s, v in zip(sel, want) if got[s] != v]
    full = float(st["n_events_full"][0])
    line = {"metric": "delta-sims/sec", "workload": "configs[4] nmt: one chain of cumulative single-op mutations (delta simulation)",
            "steps": n_steps, "gpu_ms": gpu_ms, "ms_per_step": gpu_ms / n_steps, "delta_sims_per_s": n_steps / (gpu_ms * 1e-3),
            "wall_s_including_uploads": wall,
            "steps_resumed_from_snapshot": int(st["n_resumed"][0]), "steps_rejoined_previous_timeline": int(st["n_converged"][0]),
            "mean_events_per_step": float(st["n_events"][0]) / max(1, int(st["n_steps"][0])),
            "events_of_a_full_simulation": full,
            "share_of_a_full_simulation_per_step": float(st["n_events"][0]) / max(1, int(st["n_steps"][0])) / max(1.0, full),
            "oracle_checked_steps": len(sel), "first_mismatching_step": (bad[0] if bad else None), "bit_exact_on_checked_steps": not bad,
            "min_ns": int(got.min()), "max_ns": int(got[got < 2 ** 63].max()), "input_sha256_first_candidate": w.sha256(1)}
    ch.close()
    sim.close()
    print(json.dumps(line))
    return 0 if not bad else 1


SECTIONS = ["set-up (validate, initial state, kept per-edge set-up)", "queue pop", "wait for the popped op's words",
            "dequeue of READY tasks", "release: before the loop over producer parts", "wait for the edge's loads",
            "release: loop over producer parts", "consumer words and queue update"]


def sections():
    """Where the time of one wavefront (= one candidate) goes: the diagnostic build of the library accumulates shader
    clock ticks per section of the event loop (Algorithm 1) and returns them in the optional per-candidate record."""
    import numpy as np
    from paper_1807_05358_amd import binding, build, workloads as W
    if not os.path.exists(build.SECTIONS_LIB):
        print(f"bench.py --sections: {build.SECTIONS_LIB} is missing; build it with "
              "`python -m paper_1807_05358_amd.build --sections`", file=sys.stderr)
        return 2
    # queue steps per candidate come from the ordinary library (the diagnostic build reuses that field)
    steps = {}
    for c in range(5):
        w = W.workload(c)
        sim = binding.Simulator(w.ops, w.edges, w.machine, w.cost)
        steps[c] = float(sim.simulate(w.strategies(w.n_candidates), stats=True)[1]["n_events"].mean())
        sim.close()
    binding.load_library(build.SECTIONS_LIB)
    fields = ["n_compute", "n_pairs", "n_comm", "sum_comm_ns", "n_events", "exit_code", "n_stuck", "reserved"]
    for c in range(5):
        w = W.workload(c)
        sim = binding.Simulator(w.ops, w.edges, w.machine, w.cost)
        st = sim.simulate(w.strategies(w.n_candidates), stats=True)[1]
        sim.close()
        t = np.array([st[f] for f in fields], dtype=np.float64).mean(1)
        print(f"configs[{c}] {w.name}: B = {w.n_candidates}, {steps[c]:.0f} queue steps and {t.sum():.0f} clock ticks per candidate")
        for name, v in zip(SECTIONS, t):
            print(f"    {name:58s} {v:12.0f}  {100 * v / t.sum():5.1f} %  {v / steps[c]:8.1f} per queue step")
    return 0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--only-headline", action="store_true", help="skip the other workloads and the delta chain")
    ap.add_argument("--workloads", default="", help="comma-separated config ids to run instead of all five (profiling runs)")
    ap.add_argument("--no-delta", action="store_true", help="skip the delta chains, the search and the refinements")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="first run three device-to-device copies of 256 MiB (a kernel of known traffic, to scale "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE readings)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    ap.add_argument("--long-chain", type=int, default=0, metavar="N",
                    help="run only the N-step mutation chain of configs[4] (10000 in the configuration list)")
    ap.add_argument("--check", type=int, default=200, help="with --long-chain: steps compared with the oracle")
    ap.add_argument("--sections", action="store_true",
                    help="print where a wavefront's time goes inside the batch kernel (clock ticks per section of the "
                         "event loop, mean per candidate) for the five workloads; needs the diagnostic build "
                         "(python -m paper_1807_05358_amd.build --sections)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (candidates are independent: several GPUs would each take a "
              "contiguous share of the batch). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_1807_05358_amd import binding, workloads as W

    if args.sections:
        sys.exit(sections())
    threads, logical_cpus, usable_cpus = host_cores()
    if args.long_chain:
        sys.exit(long_chain(args.long_chain, args.check, threads))

    if args.calibration_copy:
        src = torch.empty(256 * 2 ** 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    prof = profiled_counters()
    results = {}
    order = [HEADLINE] if args.only_headline else [HEADLINE, 0, 1, 2, 3]
    if args.workloads:
        order = [HEADLINE] + [int(x) for x in args.workloads.split(",") if int(x) != HEADLINE]
    for c in order:
        w = W.workload(c)
        B = w.n_candidates
        cfgs = w.strategies(B)
        sim = binding.Simulator(w.ops, w.edges, w.machine, w.cost)
        d_strat = sim.upload_strategies(cfgs)
        _, st = sim.simulate(cfgs, stats=True)          # untimed: counters for the byte model
        sim.batch(d_strat, B)                            # back to the kernel without counters
        kernel = binding.ff_sim_batch_kernel_name(sim.handle, B)
        if c == HEADLINE:
            steps, warmup = args.steps, args.warmup
        else:
            steps, warmup = (20, 3) if c < 2 else (5, 1)
        kern_ms, wall_ms, out = time_batches(sim, d_strat, B, steps, warmup)
        got = out.cpu().numpy().view("<u8")
        tc, npairs = float(st["n_compute"].mean()), float(st["n_pairs"].mean())
        ab = alg_bytes(w.n_ops, tc, npairs)
        # counter readings only count if they were taken for the instantiation launched here
        pc = prof.get(c)
        if pc is not None and (pc["kernel"] != kernel or pc["B"] != B):
            pc = None
        traffic = pc["traffic_bytes"] if pc else None
        valu = pc["insts_valu"] if pc else None
        r = {
            "workload": f"configs[{c}] {w.name}", "B": B, "n_ops": w.n_ops, "n_edges": int(len(w.edges)),
            "simulated_devices": w.machine.n_devices, "steps": steps, "warmup": warmup,
            "ms_per_step": wall_ms, "kernel_ms": kern_ms, "strategies_per_s": B / (wall_ms * 1e-3),
            "mean_compute_tasks": tc, "mean_pairs": npairs, "mean_comm_tasks": float(st["n_comm"].mean()),
            "mean_events": float(st["n_events"].mean()),
            "roofline": {"bound": "hbm", "achieved": ab * B / (kern_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                         "frac": ab * B / (kern_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, "traffic": traffic,
                         "kernel": kernel, "alg_bytes_per_strategy": ab, "alg_bytes_per_launch": ab * B, "kernel_ms": kern_ms,
                         "traffic_GBps": (traffic / (kern_ms * 1e-3) / 1e9 if traffic else None),
                         "irreducible_io_bytes_per_launch": (8 * w.n_ops + 8) * B},
            "roofline_alu": ({"bound": "alu", "achieved": valu / (kern_ms * 1e-3) / 1e9, "peak": VALU_PEAK_G_PER_S,
                              "unit": "G wavefront-instructions/s", "frac": valu / (kern_ms * 1e-3) / 1e9 / VALU_PEAK_G_PER_S,
                              "insts_valu_per_strategy": valu / B,
                              "note": "instruction count per launch from rocprofv3 SQ_INSTS_VALU (profiles/), kernel time live"}
                             if valu else None),
            "wavefronts_per_simd": min(B, 1024 * 8) / 1024.0,
            "input_sha256": w.sha256(B),
        }
        if not args.workloads and not args.only_headline:
            # saturation: the same graph with four times as many candidates per launch
            cfgs4x = w.strategies(4 * B)
            d4 = sim.upload_strategies(cfgs4x)
            k4, w4ms, _ = time_batches(sim, d4, 4 * B, 2, 1)
            r["saturation_B"] = 4 * B
            r["saturation_strategies_per_s"] = 4 * B / (w4ms * 1e-3)
            del d4
        if not args.no_cpu:
            n_s = {0: 64, 1: 1024, 2: 128, 3: 64, 4: 128}[c]
            idx = np.linspace(0, B - 1, n_s).astype(np.int64)
            rate_t, ref = oracle_rate(w, cfgs[idx], threads)
            r["oracle_strategies_per_s"] = rate_t
            r["oracle_threads"] = threads
            r["oracle_sample"] = n_s
            r["bit_exact_on_sample"] = bool(np.array_equal(got[idx], ref))
        results[c] = (r, sim, w, cfgs)

    head, sim, w, cfgs = results[HEADLINE]
    copy_gbps = copy_bandwidth_gbps()
    roof = dict(head["roofline"])
    roof["achievable_copy_GBps"] = copy_gbps
    roof["frac_of_copy"] = roof["achieved"] / copy_gbps
    line = {
        "metric": "simulated strategies/sec (build + full simulation)",
        "value": head["strategies_per_s"],
        "unit": "strategies/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u64", "data": "synthetic",
        "config": {"workload": f"configs[{HEADLINE}]: NMT-shaped graph ({w.n_ops} ops, {len(w.edges)} tensor edges: 2+2 LSTM layers "
                               "unrolled 40 steps, attention, vocabulary 32768), batch 64, 16 nodes x 4 simulated devices, "
                               f"{head['B']} seeded candidate strategies per step", "B": head["B"],
                   "candidates_per_step": head["B"]},
        "roofline": roof,
        "roofline_alu": head["roofline_alu"],
    }
    if not args.no_cpu:
        # the oracle as it stands on the host cores, on a bounded sample of the same batch: every
        # 8th candidate (about 20 s of CPU time), and its single-thread rate on 8 of them
        idx = np.arange(0, head["B"], 8)
        multi, _ = oracle_rate(w, cfgs[idx], threads)
        one, _ = oracle_rate(w, cfgs[idx[:8]], 1)
        line["cpu_baseline"] = {"value": multi, "unit": "strategies/s", "cores": threads, "kind": "oracle",
                                "sample": f"every 8th of the {head['B']} candidates of configs[{HEADLINE}] ({len(idx)} strategies), "
                                          f"{threads} threads (static split); single thread on 8 of them: {one:.2f} strategies/s",
                                "single_thread_value": one, "cpu_model": cpu_model(),
                                "logical_cpus_of_the_box": logical_cpus, "cpus_usable_by_this_process": usable_cpus}
        tb, tt = oracle_build_share(w, cfgs[:4])
        line["cpu_baseline"]["one_thread_build_seconds_per_strategy"] = tb / 4
        line["cpu_baseline"]["one_thread_build_plus_simulate_seconds_per_strategy"] = tt / 4
    if not args.only_headline and not args.no_delta:
        # delta simulation on configs[4]: one chain, and 256 independent chains
        r4, sim4, w4, cfgs4 = results[4]
        delta = []
        # (the last: as many chains as the device holds at once -- three per compute unit, by the LDS a chain needs)
        for C, n_steps in ((1, 256), (256, 32), (768, 32)):
            muts = w4.mutations(n_steps, C)
            ch = binding.Chains(sim4, cfgs4[:C])
            d_m = ch.upload_mutations(muts)
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            out = ch.delta(d_m, n_steps)
            b.record()
            torch.cuda.synchronize()
            ms = a.elapsed_time(b)
            st = ch.stats()
            d = {"workload": "configs[4] nmt", "chains": C, "steps": n_steps, "ms": ms,
                 "delta_sims_per_s": C * n_steps / (ms * 1e-3),
                 "steps_resumed_from_snapshot": int(st["n_resumed"].sum()), "steps_total": int(st["n_steps"].sum()),
                 "mean_events_per_step": float(st["n_events"].sum() / max(1, st["n_steps"].sum())),
                 "events_of_a_full_simulation": float(st["n_events_full"].mean()),
                 "full_chain_length_in_the_configuration_list": 10000,
                 "note": "python bench.py --long-chain 10000 runs the full chain (profiles/)"}
            got = out.cpu().numpy().view("<u8")
            if not args.no_cpu and C == 1:
                sel = sorted(set(np.linspace(0, n_steps - 1, 16).astype(int).tolist()))
                ref = oracle_chain_steps(w4, cfgs4[0], muts[:, 0], sel, threads)
                d["oracle_checked_steps"] = len(sel)
                d["bit_exact_on_checked_steps"] = bool(np.array_equal(got[sel, 0], ref))
                # what Algorithm 2 would have to touch, counted by diffing the oracle's timelines of
                # consecutive strategies on 16 steps spread over the chain: removed + inserted + moved tasks
                work = delta_work_model(w4, cfgs4[0], muts[:, 0], sel)
                d["oracle_changed_tasks_on_sampled_steps"] = work
                items = float(np.mean([x["removed"] + x["inserted"] + x["moved"] for x in work]))
                d["mean_changed_share_of_tasks"] = float(np.mean([(x["removed"] + x["inserted"] + x["moved"]) / x["tasks_after"] for x in work]))
                d["algorithmic_bytes_per_step"] = items * 34.0   # 20 B per task written + read, 14 B per record, as in the byte model
                d["algorithmic_GBps"] = items * 34.0 * n_steps / (ms * 1e-3) / 1e9
            if not args.no_cpu and C > 1:
                chains_checked = [0, 31, 64, 100, 127, 200, 254, 255] if C == 256 else [0, 383, 767]
                ok = True
                for cc in chains_checked:
                    ref = oracle_chain_steps(w4, cfgs4[cc], muts[:, cc], [n_steps // 2, n_steps - 1], threads)
                    ok = ok and bool(np.array_equal(got[[n_steps // 2, n_steps - 1], cc], ref))
                d["oracle_checked_chains"] = len(chains_checked)
                d["bit_exact_on_checked_chains"] = ok
            delta.append(d)
            if C == 1:
                # proposals evaluated side by side against the chain's stored timeline (not committed)
                M = 1024
                props = w4.mutations(n_steps + M, 1)[n_steps:]
                d_p = ch.upload_mutations(props)
                ch.try_mutations(d_p, 8)
                torch.cuda.synchronize()
                a.record()
                tried = ch.try_mutations(d_p, M)
                b.record()
                torch.cuda.synchronize()
                ms = a.elapsed_time(b)
                t = {"workload": "configs[4] nmt", "chains": 1, "proposals": M, "ms": ms,
                     "kind": "trial mutations (ff_sim_delta_try), all against the same current strategy",
                     "delta_sims_per_s": M / (ms * 1e-3)}
                if not args.no_cpu:
                    import oracle
                    cur = cfgs4[0].copy()
                    for s_ in range(n_steps):
                        cur[int(muts[s_, 0]["op"])] = muts[s_, 0]["cfg"]
                    sel = [0, M // 4, M // 2, M - 1]
                    cand = np.repeat(cur[None], len(sel), 0)
                    for q, p_ in enumerate(sel):
                        cand[q, int(props[p_, 0]["op"])] = props[p_, 0]["cfg"]
                    ref = oracle.simulate_batch(w4.ops, w4.edges, w4.machine, w4.cost, cand, n_threads=threads)
                    t["bit_exact_on_sampled_proposals"] = bool(np.array_equal(tried.cpu().numpy().view("<u8")[sel, 0], ref))
                delta.append(t)
                # with one proposal per wavefront the launch lasts as long as its slowest proposal (one that has to
                # start from time 0); with several per wavefront, handed out from a counter, the launch follows the
                # MEAN cost of a proposal, which is where the kept timeline shows
                M8 = 8192
                props8 = w4.mutations(n_steps + M8, 1)[n_steps:]
                d_p8 = ch.upload_mutations(props8)
                ch.try_mutations(d_p8, 8)
                torch.cuda.synchronize()
                a.record()
                ch.try_mutations(d_p8, M8)
                b.record()
                torch.cuda.synchronize()
                ms8 = a.elapsed_time(b)
                delta.append({"workload": "configs[4] nmt", "chains": 1, "proposals": M8, "ms": ms8,
                              "kind": "trial mutations (ff_sim_delta_try), eight times as many as wavefronts fit",
                              "delta_sims_per_s": M8 / (ms8 * 1e-3),
                              "against_full_simulations_per_s": (M8 / (ms8 * 1e-3)) / line["value"]})
            ch.close()
        line["delta"] = delta
        # the search loop on the device (ff_sim_search): independent Metropolis chains
        search = []
        for cid, C, n_steps in ((4, 256, 8), (2, 1024, 16)):
            if cid not in results:
                continue
            _, sim_s, w_s, cfgs_s = results[cid]
            C = min(C, len(cfgs_s))
            ch = binding.Chains(sim_s, cfgs_s[:C])
            start = ch.start_ns().copy()
            bucket = max(1, int(np.median(start)) // 256)
            tp, tu = w_s.search_space()
            ch.search_setup(tp, tu, binding.ff_sim_accept_table(50.0 / float(np.median(start)), bucket, 256), bucket, 1807)
            ch.search(1)
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            trace = ch.search(n_steps)
            b.record()
            torch.cuda.synchronize()
            ms = a.elapsed_time(b)
            best_ns, _ = ch.best()
            tr = trace.cpu().numpy().view("<u8")
            search.append({"workload": f"configs[{cid}] {w_s.name}", "chains": C, "steps": n_steps, "ms": ms,
                           "proposals_per_s": C * n_steps / (ms * 1e-3),
                           "steps_that_changed_the_time": int((np.diff(tr.astype(np.int64), axis=0) != 0).sum()),
                           "median_start_ns": float(np.median(start)), "median_best_ns": float(np.median(best_ns))})
            ch.close()
        line["search"] = search
        # one chain is one wavefront in ff_sim_search; ff_sim_search_ahead simulates the proposals of the coming
        # steps side by side (the same chain, step for step).  It pays when few proposals are accepted.
        few = []
        for cid, n_steps, start_kind in ((1, 4000, "data parallelism"), (1, 2000, "random strategy"), (2, 600, "data parallelism")):
            if cid not in results:
                continue
            _, sim_s, w_s, cfgs_s = results[cid]
            cfg0 = cfgs_s[:1].copy()
            if start_kind == "data parallelism":
                cfg0[0] = W.data_parallel_strategy(w_s.ops, w_s.machine.n_devices, w_s.max_parts)
            tp, tu = w_s.search_space()
            rec = {"workload": f"configs[{cid}] {w_s.name}", "chains": 1, "steps": n_steps, "start": start_kind}
            traces = []
            for ahead in (0, 4096):
                ch = binding.Chains(sim_s, cfg0)
                t_start = float(ch.start_ns()[0])
                scale = 0.25 / len(w_s.ops)            # the search driver's default tolerance
                bucket = max(1, int(t_start * scale * 8 / 256))
                ch.search_setup(tp, tu, binding.ff_sim_accept_table(1.0 / (t_start * scale), bucket, 256), bucket, 1807)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                tr = ch.search(n_steps, ahead=ahead)
                torch.cuda.synchronize()
                dt = time.perf_counter() - t0
                traces.append(tr.cpu().numpy().view("<u8"))
                if ahead:
                    rec["ahead_steps_per_s"] = n_steps / dt
                    rec["ahead_rounds"], rec["ahead_proposals_simulated"] = int(ch.ahead_stats[0]), int(ch.ahead_stats[1])
                    rec["proposals_accepted"] = int(ch.ahead_stats[3])
                else:
                    rec["one_by_one_steps_per_s"] = n_steps / dt
                ch.close()
            rec["same_trace"] = bool(np.array_equal(traces[0], traces[1]))
            rec["steps_that_changed_the_time"] = int((np.diff(np.concatenate([[t_start], traces[0][:, 0].astype(np.float64)])) != 0).sum())
            rec["speedup"] = rec["ahead_steps_per_s"] / rec["one_by_one_steps_per_s"]
            few.append(rec)
        line["search_with_one_chain"] = few
        # the whole search with parameter-synchronisation traffic simulated (ff_sim_set_params): can it
        # beat data parallelism, as Section 8 reports?  (a simulator of its own, the timed kernels above
        # never see the refinement)
        if 1 in results:
            from paper_1807_05358_amd import search as driver
            w_p = results[1][2]
            sim_p = binding.Simulator(w_p.ops, w_p.edges, w_p.machine, w_p.cost, params=w_p.param_table())
            C, n_steps = 256, 1024
            cfg0 = driver.starting_strategies(w_p.ops, w_p.machine, w_p.max_parts, w_p.choices, C, 1807)
            cfg0[:C // 2] = W.data_parallel_strategy(w_p.ops, w_p.machine.n_devices, w_p.max_parts)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            res = driver.find_strategy(sim_p, w_p.ops, w_p.machine, w_p.max_parts, w_p.choices, steps=n_steps, accept_scale=0.005,
                                       seed=1807, start=cfg0)
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            line["search_with_parameter_traffic"] = {
                "workload": f"configs[1] {w_p.name}, parameters of conv / fc ops synchronised among replicas",
                "chains": C, "steps": n_steps, "wall_s": dt, "proposals_per_s": C * n_steps / dt,
                "data_parallel_ns": int(res.start_ns[0]), "best_found_ns": res.best_ns,
                "speedup_over_data_parallel": int(res.start_ns[0]) / res.best_ns,
                "best_degrees_per_op": res.best["deg"].tolist()}
            if not args.no_cpu:
                import oracle
                line["search_with_parameter_traffic"]["best_confirmed_by_oracle"] = bool(int(oracle.simulate_batch(
                    w_p.ops, w_p.edges, w_p.machine, w_p.cost, res.best[None], params=w_p.param_table())[0]) == res.best_ns)
            sim_p.close()
        # the refinements of the inputs on configs[1]: what each costs per launch
        if 1 in results:
            import dataclasses
            w_r = results[1][2]
            cfgs_r = w_r.strategies(1024)
            lbw, llat = W.paired_links(w_r.machine.gpus_per_node, 20, 6, 100, 900)
            variants = {
                "plain": (w_r.machine, None, None),
                "unequal_links": (dataclasses.replace(w_r.machine, link_Bpns=lbw, link_lat_ns=llat), None, None),
                "parameter_traffic": (w_r.machine, w_r.param_table(), None),
                "explicit_devices": (w_r.machine, None, W.device_maps(cfgs_r, w_r.machine.n_devices, 1807)),
            }
            ref = {}
            for name, (mach_r, params_r, maps_r) in variants.items():
                sim_r = binding.Simulator(w_r.ops, w_r.edges, mach_r, w_r.cost, params=params_r)
                d_r = sim_r.upload_strategies(cfgs_r)
                dm_r = None if maps_r is None else binding.to_device(maps_r)
                out_r = sim_r.batch(d_r, 1024, d_devmaps=dm_r)
                torch.cuda.synchronize()
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                for _ in range(5):
                    sim_r.batch(d_r, 1024, d_out=out_r, d_devmaps=dm_r)
                b.record()
                torch.cuda.synchronize()
                ms = a.elapsed_time(b) / 5
                ref[name] = {"kernel_ms": ms, "strategies_per_s": 1024 / (ms * 1e-3)}
                if not args.no_cpu:
                    import oracle
                    want = oracle.simulate_batch(w_r.ops, w_r.edges, mach_r, w_r.cost, cfgs_r[:64], params=params_r,
                                                 devmaps=None if maps_r is None else maps_r[:64])
                    ref[name]["bit_exact_on_sample"] = bool(np.array_equal(out_r.cpu().numpy().view("<u8")[:64], want))
                sim_r.close()
            line["refinements_on_configs1"] = ref
        # whole training iterations: forward and backward ops, gradient edges, tied configurations, parameter traffic
        train = []
        for cid in (1, 2):
            if cid not in results:
                continue
            w_t = results[cid][2]
            t_ops, t_edges, t_flops, leader, t_params = W.training_graph(w_t.ops, w_t.edges, w_t.flops)
            t_cost = np.ascontiguousarray(W.cost_table(cid, t_flops, w_t.seed)[:, :w_t.max_parts])
            sim_t = binding.Simulator(t_ops, t_edges, w_t.machine, t_cost, params=t_params, ties=leader)
            n_t = w_t.n_candidates
            cfgs_t = W.strategies(t_ops, n_t, w_t.seed, w_t.machine.n_devices, w_t.max_parts, w_t.choices)
            d_t = sim_t.upload_strategies(cfgs_t)
            k_ms, w_ms, out_t = time_batches(sim_t, d_t, n_t, 5, 1)
            t = {"workload": f"configs[{cid}] {w_t.name}: training iteration ({len(t_ops)} ops, {len(t_edges)} edges, "
                             "backward ops tied to their forward ops, gradients of conv / fc parameters synchronised)",
                 "B": n_t, "kernel_ms": k_ms, "strategies_per_s": n_t / (w_ms * 1e-3),
                 "kernel": binding.ff_sim_batch_kernel_name(sim_t.handle, n_t)}
            if not args.no_cpu:
                import oracle
                idx = np.linspace(0, n_t - 1, 64).astype(np.int64)
                want = oracle.simulate_batch(t_ops, t_edges, w_t.machine, t_cost, cfgs_t[idx], n_threads=threads, ties=leader, params=t_params)
                t["bit_exact_on_sample"] = bool(np.array_equal(out_t.cpu().numpy().view("<u8")[idx], want))
            if cid == 1:
                from paper_1807_05358_amd import search as driver
                C, n_steps = 256, 512
                cfg0 = driver.starting_strategies(t_ops, w_t.machine, w_t.max_parts, w_t.choices, C, 1807)
                cfg0[:C // 2] = W.data_parallel_strategy(t_ops, w_t.machine.n_devices, w_t.max_parts)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                res = driver.find_strategy(sim_t, t_ops, w_t.machine, w_t.max_parts, w_t.choices, steps=n_steps, accept_scale=0.005,
                                           seed=1807, start=cfg0)
                torch.cuda.synchronize()
                dt = time.perf_counter() - t0
                t["search"] = {"chains": C, "steps": n_steps, "wall_s": dt, "proposals_per_s": C * n_steps / dt,
                               "data_parallel_ns": int(res.start_ns[0]), "best_found_ns": res.best_ns,
                               "speedup_over_data_parallel": int(res.start_ns[0]) / res.best_ns,
                               "best_degrees_per_forward_op": res.best["deg"][:len(w_t.ops)].tolist()}
                if not args.no_cpu:
                    t["search"]["best_confirmed_by_oracle"] = bool(int(oracle.simulate_batch(
                        t_ops, t_edges, w_t.machine, t_cost, res.best[None], ties=leader, params=t_params)[0]) == res.best_ns)
            sim_t.close()
            train.append(t)
        line["training_iteration"] = train
        # neighbour sweep (local-optimality check): all single-op neighbours of one strategy
        if 1 in results:
            _, sim_n, w_n, cfgs_n = results[1]
            ch = binding.Chains(sim_n, cfgs_n[:1])
            tp, tu = w_n.search_space()
            t0 = time.perf_counter()
            muts_n, ns_n, best_n, idx_n = ch.neighbours(tp, tu)
            dt = time.perf_counter() - t0
            line["neighbour_sweep"] = {"workload": f"configs[1] {w_n.name}", "neighbours": int(ns_n.shape[0]),
                                       "wall_ms_including_copies_back": dt * 1e3,
                                       "neighbours_per_s": ns_n.shape[0] / dt,
                                       "start_ns": int(ch.start_ns()[0]), "best_neighbour_ns": int(best_n[0])}
            ch.close()
    if not args.only_headline:
        line["workloads"] = [results[c][0] for c in sorted(results)]
    print(json.dumps(line))


if __name__ == "__main__":
    main()
