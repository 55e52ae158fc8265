"""Randomized parity over everything at once: random graphs and machines with any combination of the refinements
(link tables inside and between nodes, parameter traffic, explicit devices), regular or general strategies; batch
simulation with and without counters, mutation chains in two calls, trial proposals against the state in between --
all against the CPU oracle, bit for bit (Sections 5.1-5.3).  And the look-ahead search against the plain one on
random graphs, temperatures, chain counts and depths (Section 6).
The number of cases per test follows FFSIM_SWEEP (default 8; a wide sweep, e.g. FFSIM_SWEEP=2000, takes minutes)."""
import dataclasses
import os

import numpy as np
import pytest

import oracle
from helpers import random_graph
from paper_1807_05358_amd import workloads as W

pytestmark = pytest.mark.gpu
N_CASES = int(os.environ.get("FFSIM_SWEEP", "8"))


@pytest.fixture(scope="module")
def B():
    from paper_1807_05358_amd import binding
    return binding


def _machine(rng, gpn_choices):
    n_nodes, gpn = int(rng.integers(1, 6)), int(rng.choice(gpn_choices))
    return W.Machine(n_nodes, gpn, int(rng.integers(1, 30)), int(rng.integers(1, 30)), int(rng.integers(0, 50)),
                     int(rng.integers(0, 50)), int(rng.choice([1, 2, 4, 8])))


@pytest.mark.parametrize("seed", range(N_CASES))
def test_all_refinements_together(B, seed):
    rng = np.random.default_rng(55000 + seed)
    big = seed % 8 == 7                                   # every eighth graph is too large for LDS-resident task words
    n_ops = int(rng.integers(65, 500)) if big else int(rng.integers(3, 90))
    ops, edges, _ = random_graph(rng, n_ops)
    mach = _machine(rng, [1, 2, 3, 4, 4, 4, 5, 8])
    n_nodes, gpn, D = mach.n_nodes, mach.gpus_per_node, mach.n_devices
    use_links, use_node, use_params, use_maps = (rng.random(4) < 0.5)
    if use_links:
        mach = dataclasses.replace(mach, link_Bpns=rng.integers(1, 40, size=(gpn, gpn)).astype("<u4"),
                                   link_lat_ns=rng.integers(0, 300, size=(gpn, gpn)).astype("<u4"))
    if use_node:
        mach = dataclasses.replace(mach, node_Bpns=rng.integers(1, 40, size=(n_nodes, n_nodes)).astype("<u4"),
                                   node_lat_ns=rng.integers(0, 300, size=(n_nodes, n_nodes)).astype("<u4"))
    params = None
    if use_params:
        pb = rng.integers(0, 200000, size=n_ops).astype("<u4")
        pb[rng.random(n_ops) < 0.4] = 0
        params = (pb, rng.integers(0, 16, size=n_ops).astype(np.uint8))
    cost = rng.integers(1, 3000, size=(n_ops, 64)).astype("<u4")
    n = 96
    regular = rng.random() < 0.5
    max_parts = min(64, D) if regular else 64
    cfgs = np.zeros((n, n_ops), W.CFG_DT)
    for i in range(n_ops):
        t = W.valid_degree_tuples(ops[i], max_parts, (1, 2, 3, 4, 5, 7, 8, 16, 32, 64))
        cfgs["deg"][:, i] = t[rng.integers(len(t), size=n)]
    cfgs["dev_offset"] = rng.integers(0, D, size=(n, n_ops))
    cfgs["dev_stride"] = 1 if regular else rng.integers(0, 4, size=(n, n_ops))
    print(f"seed {seed}: {n_ops} ops, {len(edges)} edges, machine {mach.as_tuple()}, links {use_links}, node links {use_node}, "
          f"parameters {use_params}, device maps {use_maps}, regular {regular}", flush=True)
    sim = B.Simulator(ops, edges, mach, cost, params=params)
    want = oracle.simulate_batch(ops, edges, mach, cost, cfgs, n_threads=8, params=params)
    got, st = sim.simulate(cfgs, stats=True)
    assert np.array_equal(got, want), f"batch: {np.nonzero(got != want)[0][:5]}"
    assert np.array_equal(sim.simulate(cfgs), want), "batch without counters"
    if use_maps:
        maps = W.device_maps(cfgs, D, seed)
        want_m = oracle.simulate_batch(ops, edges, mach, cost, cfgs, n_threads=8, devmaps=maps, params=params)
        assert np.array_equal(sim.simulate(cfgs, devmaps=maps), want_m), "explicit devices"
    steps, C = 30, 3
    ok = np.nonzero(want != oracle.INVALID)[0]
    if len(ok) >= C:
        muts = np.zeros((steps, C), W.MUT_DT)
        muts["op"] = rng.integers(0, n_ops, size=(steps, C))
        for s in range(steps):
            for c in range(C):
                i = int(muts[s, c]["op"])
                t = W.valid_degree_tuples(ops[i], max_parts, (1, 2, 3, 4, 8, 16))
                muts[s, c]["cfg"]["deg"] = t[rng.integers(len(t))]
                muts[s, c]["cfg"]["dev_offset"] = rng.integers(0, D)
                muts[s, c]["cfg"]["dev_stride"] = 1 if (regular and rng.random() < 0.95) else rng.integers(0, 3)
        start = ok[:C]
        half = steps // 2
        ch = B.Chains(sim, cfgs[start])
        d1 = ch.delta(ch.upload_mutations(muts[:half]), half).cpu().numpy().view("<u8")
        tried = ch.try_mutations(ch.upload_mutations(muts[half:]), steps - half).cpu().numpy().view("<u8")
        d2 = ch.delta(ch.upload_mutations(muts[half:]), steps - half).cpu().numpy().view("<u8")
        d = np.concatenate([d1, d2])
        for c in range(C):
            ref = oracle.simulate_delta_chain(ops, edges, mach, cost, cfgs[start[c]], muts[:, c], params=params)
            assert np.array_equal(d[:, c], ref), f"chain {c}: steps {np.nonzero(d[:, c] != ref)[0][:5]}"
            cur = cfgs[start[c]].copy()
            for s in range(half):
                cur[int(muts[s, c]["op"])] = muts[s, c]["cfg"]
            props = np.repeat(cur[None], steps - half, 0)
            for s in range(half, steps):
                props[s - half, int(muts[s, c]["op"])] = muts[s, c]["cfg"]
            assert np.array_equal(tried[:, c], oracle.simulate_batch(ops, edges, mach, cost, props, n_threads=8, params=params)), \
                f"trial proposals of chain {c}"
        ch.close()
    sim.close()


@pytest.mark.parametrize("seed", range(N_CASES))
def test_look_ahead_search_equals_the_plain_search(B, seed):
    rng = np.random.default_rng(880000 + seed)
    n_ops = int(rng.integers(3, 120))
    ops, edges, _ = random_graph(rng, n_ops)
    mach = _machine(rng, [1, 2, 4, 4, 4, 8])
    D = mach.n_devices
    params = None
    if rng.random() < 0.3:
        pb = rng.integers(0, 200000, size=n_ops).astype("<u4")
        pb[rng.random(n_ops) < 0.4] = 0
        params = (pb, rng.integers(0, 16, size=n_ops).astype(np.uint8))
    cost = rng.integers(1, 3000, size=(n_ops, 64)).astype("<u4")
    C = int(rng.choice([1, 1, 2, 5, 17]))
    choices = (1, 2, 4, 8, 16)
    cfgs = np.zeros((C, n_ops), W.CFG_DT)
    for i in range(n_ops):
        t = W.valid_degree_tuples(ops[i], min(64, D), choices)
        cfgs["deg"][:, i] = t[rng.integers(len(t), size=C)]
    cfgs["dev_offset"] = rng.integers(0, D, size=(C, n_ops))
    cfgs["dev_stride"] = 1
    tp, tu = W.search_space(ops, min(64, D), choices)
    steps = int(rng.integers(20, 300))
    temp = float(rng.choice([0.0005, 0.005, 0.02, 0.2]))
    patience = int(rng.choice([0, 0, 15, 60]))
    ahead = int(rng.choice([1, 2, 5, 33, 1000])) | (B.FF_AHEAD_ALWAYS if rng.random() < 0.6 else 0)
    print(f"seed {seed}: {n_ops} ops, {C} chains, {steps} steps, tolerance {temp}, patience {patience}, "
          f"look-ahead {ahead & 0xffff}{' always' if ahead >> 31 else ''}", flush=True)
    sim = B.Simulator(ops, edges, mach, cost, params=params)
    res = []
    for a in (0, ahead):
        ch = B.Chains(sim, cfgs)
        start = ch.start_ns()
        ok = start[start < B.FF_OVERFLOW_NS]
        ref = float(np.median(ok)) if len(ok) else 1000.0
        bucket = max(1, int(ref * temp * 8 / 64))
        ch.search_setup(tp, tu, B.ff_sim_accept_table(1.0 / max(1.0, ref * temp), bucket, 64), bucket, seed, patience=patience)
        n1 = steps // 3
        trace = np.concatenate([ch.search(n1, ahead=a).cpu().numpy().view("<u8"),
                                ch.search(steps - n1, ahead=a).cpu().numpy().view("<u8")])
        best_ns, best = ch.best()
        res.append((trace, best_ns.copy(), best.copy()))
        ch.close()
    sim.close()
    assert np.array_equal(res[0][0], res[1][0]), "traces"
    assert np.array_equal(res[0][1], res[1][1]) and np.array_equal(res[0][2], res[1][2]), "best times and strategies"
