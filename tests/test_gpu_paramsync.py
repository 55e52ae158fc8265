"""GPU parity of the parameter-synchronisation refinement (ff_sim_set_params) against the oracle,
bit for bit: batch simulation, counters, delta chains, the search loop, with explicit devices and
with unequal links."""
import dataclasses

import numpy as np
import pytest

import oracle
from oracle import search as osearch
from paper_1807_05358_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_1807_05358_amd import binding
    return binding


def _mixed(w, n, seed):
    cfgs = w.strategies(n)
    rng = np.random.default_rng(seed)
    irregular = rng.random(n) < 0.35
    cfgs["dev_stride"][irregular] = rng.integers(0, 6, size=(int(irregular.sum()), cfgs.shape[1]))
    return cfgs


@pytest.mark.parametrize("config_id,n", [(0, 64), (1, 320), (2, 40), (4, 2)])
def test_parameter_traffic_matches_the_oracle(B, config_id, n):
    w = W.workload(config_id)
    params = w.param_table()
    assert params[0].any()
    cfgs = _mixed(w, n, 60 + config_id)
    cfgs[0] = W.data_parallel_strategy(w.ops, w.machine.n_devices, w.max_parts)
    want = oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cfgs, n_threads=8, params=params)
    plain = oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cfgs, n_threads=8)
    assert config_id == 0 or (want != plain).mean() > 0.5        # (config 0's parameters are tiny)
    sim = B.Simulator(w.ops, w.edges, w.machine, w.cost, params=params)
    got, st = sim.simulate(cfgs, stats=True)
    assert not st["exit_code"].any() and not st["n_stuck"].any()
    bad = np.nonzero(got != want)[0]
    assert len(bad) == 0, f"{len(bad)} differ, first {bad[:5]}: gpu {got[bad[:5]]} oracle {want[bad[:5]]}"
    for b in range(min(n, 3)):
        tg = oracle.build_task_graph(w.ops, w.edges, w.machine, w.cost, cfgs[b], params=params)
        assert int(st["n_comm"][b]) == tg.n_tasks - tg.n_compute
        assert int(st["sum_comm_ns"][b]) == int(tg.exe[tg.n_compute:].sum())
    B.ff_sim_set_params(sim.handle, w.n_ops)                     # off again
    assert np.array_equal(sim.simulate(cfgs), plain)
    sim.close()


def test_parameter_dims_and_sizes_of_all_kinds_on_random_graphs(B):
    from helpers import random_graph
    for seed in range(5):
        rng = np.random.default_rng(9100 + seed)
        n_ops = int(rng.integers(3, 80))
        ops, edges, _ = random_graph(rng, n_ops)
        n_nodes, gpn = int(rng.integers(1, 5)), int(rng.choice([1, 2, 3, 4, 4, 8]))
        mach = W.Machine(n_nodes, gpn, int(rng.integers(1, 30)), int(rng.integers(1, 30)),
                         int(rng.integers(0, 50)), int(rng.integers(0, 50)), int(rng.choice([1, 2, 4, 8])))
        if seed % 2:
            mach = dataclasses.replace(mach, link_Bpns=rng.integers(1, 40, size=(gpn, gpn)).astype("<u4"),
                                       link_lat_ns=rng.integers(0, 300, size=(gpn, gpn)).astype("<u4"))
        if seed >= 2:                                           # network links per node pair as well
            mach = dataclasses.replace(mach, node_Bpns=rng.integers(1, 40, size=(n_nodes, n_nodes)).astype("<u4"),
                                       node_lat_ns=rng.integers(0, 300, size=(n_nodes, n_nodes)).astype("<u4"))
        cost = rng.integers(1, 3000, size=(n_ops, 64)).astype("<u4")
        pb = rng.integers(0, 200000, size=n_ops).astype("<u4")
        pb[rng.random(n_ops) < 0.4] = 0
        pb[0] = 2 ** 32 - 1                                     # the largest size the table can hold
        pd = rng.integers(0, 16, size=n_ops).astype(np.uint8)
        n = 96
        cfgs = np.zeros((n, n_ops), W.CFG_DT)
        for i in range(n_ops):
            t = W.valid_degree_tuples(ops[i], 64, (1, 2, 3, 4, 5, 7, 8, 16, 32, 64))
            cfgs["deg"][:, i] = t[rng.integers(len(t), size=n)]
        cfgs["dev_offset"] = rng.integers(0, mach.n_devices, size=(n, n_ops))
        cfgs["dev_stride"] = 1
        cfgs["dev_stride"][n // 2:] = rng.integers(0, 3, size=(n - n // 2, n_ops))
        # dims beyond an op's ndim never index anything (their degree is 1)
        print(f"seed {seed}: {n_ops} ops, {len(edges)} edges, machine {mach.as_tuple()}", flush=True)
        sim = B.Simulator(ops, edges, mach, cost, params=(pb, pd))
        got = sim.simulate(cfgs)
        want = oracle.simulate_batch(ops, edges, mach, cost, cfgs, n_threads=8, params=(pb, pd))
        assert np.array_equal(got, want), f"seed {seed}: {np.nonzero(got != want)[0][:5]}"
        maps = W.device_maps(cfgs, mach.n_devices, seed)
        got = sim.simulate(cfgs, devmaps=maps)
        want = oracle.simulate_batch(ops, edges, mach, cost, cfgs, n_threads=8, devmaps=maps, params=(pb, pd))
        assert np.array_equal(got, want), f"seed {seed} maps: {np.nonzero(got != want)[0][:5]}"
        sim.close()


@pytest.mark.parametrize("config_id,C,steps", [(1, 3, 40), (2, 2, 16)])
def test_delta_and_search_with_parameter_traffic(B, config_id, C, steps):
    w = W.workload(config_id)
    params = w.param_table()
    sim = B.Simulator(w.ops, w.edges, w.machine, w.cost, params=params)
    cfg0 = w.strategies(C)
    cfg0[0] = W.data_parallel_strategy(w.ops, w.machine.n_devices, w.max_parts)
    muts = w.mutations(steps, C)
    ch = B.Chains(sim, cfg0)
    assert np.array_equal(ch.start_ns(), oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cfg0, params=params))
    got = ch.delta(ch.upload_mutations(muts), steps).cpu().numpy().view("<u8")
    for c in range(C):
        assert np.array_equal(got[:, c], oracle.simulate_delta_chain(w.ops, w.edges, w.machine, w.cost, cfg0[c], muts[:, c],
                                                                      params=params)), f"chain {c}"
    # trial mutations against the chains' current strategies
    trial = w.mutations(8, C)[::-1].copy()
    tr = ch.try_mutations(ch.upload_mutations(trial), 8).cpu().numpy().view("<u8")
    cur = cfg0.copy()
    for s in range(steps):
        for c in range(C):
            cur[c, int(muts[s, c]["op"])] = muts[s, c]["cfg"]
    for c in range(C):
        for k in range(8):
            cand = cur[c].copy()
            cand[int(trial[k, c]["op"])] = trial[k, c]["cfg"]
            assert int(tr[k, c]) == int(oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cand[None], params=params)[0])
    ch.close()
    ptr, tup = w.search_space()
    n_steps = 10 if config_id == 1 else 5
    t0 = int(oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cfg0[:1], params=params)[0])
    bucket = max(1, t0 // 256)
    accept = B.ff_sim_accept_table(20.0 / t0, bucket, 64)
    ch = B.Chains(sim, cfg0)
    ch.search_setup(ptr, tup, accept, bucket, seed=31)
    trace = ch.search(n_steps).cpu().numpy().view("<u8")
    for c in range(C):
        want = osearch.metropolis_chain(w.ops, w.edges, w.machine, w.cost, cfg0[c], ptr, tup, accept, bucket, 31, c, 0, n_steps,
                                        params=params)
        assert np.array_equal(trace[:, c], want[0]), f"chain {c}"
    ch.close()
    sim.close()


def test_parameter_table_argument_errors(B):
    w = W.workload(1)
    sim = B.Simulator(w.ops, w.edges, w.machine, w.cost)
    pb, pd = w.param_table()
    with pytest.raises(B.FFSimError) as e:
        B._check(B.lib().ff_sim_set_params(sim.handle, pb.ctypes.data, None), "ff_sim_set_params")
    assert e.value.code == B.FF_EINVAL
    ch = B.Chains(sim, w.strategies(2))
    muts = ch.upload_mutations(w.mutations(2, 2))
    ch.delta(muts, 1)
    B.ff_sim_set_params(sim.handle, w.n_ops, pb, pd)             # the chains' timelines were made without the traffic
    with pytest.raises(B.FFSimError) as e:
        ch.delta(muts, 1)
    assert e.value.code == B.FF_EINVAL
    ch.close()
    sim.close()
