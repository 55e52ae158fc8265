"""GPU parity: the HIP path (through the C boundary) against the CPU oracle, bit for bit,
on the same seeded inputs.  Everything here needs an MI355X."""
import numpy as np
import pytest

import oracle
from helpers import graph_from_golden, load_golden, random_graph
from paper_1807_05358_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_1807_05358_amd import binding
    return binding


_sims = {}


def sim_for(B, config_id):
    if config_id not in _sims:
        w = W.workload(config_id)
        _sims[config_id] = B.Simulator(w.ops, w.edges, w.machine, w.cost)
    return _sims[config_id]


def oracle_stats(w, cfg):
    tg = oracle.build_task_graph(w.ops, w.edges, w.machine, w.cost, cfg)
    n_comm = tg.n_tasks - tg.n_compute
    return dict(n_compute=tg.n_compute, n_pairs=tg.n_deps - n_comm, n_comm=n_comm,
                sum_comm_ns=int(tg.exe[tg.n_compute:].sum()))


@pytest.mark.parametrize("name", ["build_two_ops_two_gpus.json", "build_shared_internode_link.json",
                                  "build_part_order_row_major.json", "build_link_latency.json",
                                  "build_intranode_latency.json", "build_uneven_split_7_by_3.json",
                                  "build_uneven_split_35_by_4.json", "build_strided_window_uneven_split.json",
                                  "build_pair_order_on_shared_link.json"])
def test_hand_computed_fixtures(B, golden_dir, name):
    g = load_golden(golden_dir, name)
    ops, edges, mach, cost, cfg = graph_from_golden(g)
    sim = B.Simulator(ops, edges, mach, cost)
    out, st = sim.simulate(cfg[None], stats=True)
    assert int(out[0]) == g["makespan"]
    n_comm = sum(1 for d in g["dev"] if d >= mach.n_devices)
    assert int(st[0]["n_comm"]) == n_comm and int(st[0]["n_compute"]) == len(g["dev"]) - n_comm
    sim.close()


# (config, number of candidates compared element by element, how many get their task-graph counters compared)
CASES = [(0, 64, 64), (1, 1024, 32), (2, 96, 4), (3, 48, 2), (4, 10, 1)]


@pytest.mark.parametrize("config_id,n,n_stats", CASES)
def test_batch_matches_oracle(B, config_id, n, n_stats):
    w = W.workload(config_id)
    cfgs = w.strategies(n)
    print(f"config {config_id} ({w.name}): {n} candidates, sha256 {w.sha256(n)[:16]}", flush=True)
    want = oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cfgs, n_threads=8)
    got, st = sim_for(B, config_id).simulate(cfgs, stats=True)
    assert not st["exit_code"].any() and not st["n_stuck"].any(), (st["exit_code"][:8], st["n_stuck"][:8], st["n_events"][:8])
    for b in range(n_stats):   # localise a builder mismatch before a timeline mismatch
        o = oracle_stats(w, cfgs[b])
        for k, v in o.items():
            assert int(st[b][k]) == v, f"candidate {b}: {k} gpu {int(st[b][k])} oracle {v}"
    bad = np.nonzero(got != want)[0]
    assert len(bad) == 0, f"{len(bad)} of {n} differ, first {bad[:5]}: gpu {got[bad[:5]]} oracle {want[bad[:5]]}"


def test_full_size_batches_run_in_bench_configuration(B):
    """every configuration at its full B, launch shape and kernel variant as in the bench (no
    per-candidate counters): every candidate of every configuration is compared with the oracle, and
    all results must respect a bound that holds for any strategy (some task runs from start to end)."""
    for config_id, n in ((0, 64), (1, 1024), (2, 4096), (3, 4096), (4, 1024)):
        w = W.workload(config_id)
        cfgs = w.strategies(n)
        print(f"config {config_id} ({w.name}): all {n} candidates", flush=True)
        got = sim_for(B, config_id).simulate(cfgs)
        want = oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cfgs, n_threads=16)
        bad = np.nonzero(got != want)[0]
        assert len(bad) == 0, f"config {config_id}: {len(bad)} of {n} differ, first {bad[:5]}: gpu {got[bad[:5]]} oracle {want[bad[:5]]}"
        parts = cfgs["deg"].astype(np.int64).prod(-1)
        task_ns = np.take_along_axis(np.broadcast_to(w.cost[None], (n,) + w.cost.shape), (parts - 1)[..., None], 2)[..., 0]
        assert (got >= task_ns.max(1)).all()
        assert (got < 2 ** 63).all()


def test_repeat_is_deterministic(B):
    w = W.workload(2)
    cfgs = w.strategies(256)
    sim = sim_for(B, 2)
    a = sim.simulate(cfgs)
    b = sim.simulate(cfgs)
    assert np.array_equal(a, b)
    # a different grid shape (fewer candidates per launch) gives the same bits
    c = np.concatenate([sim.simulate(cfgs[:100]), sim.simulate(cfgs[100:])])
    assert np.array_equal(a, c)


def test_invalid_candidates_are_flagged_not_fatal(B):
    w = W.workload(0)
    cfgs = w.strategies(8).copy()
    cfgs[1][5]["deg"] = (1, 2, 1, 1)     # softmax split in a non-parallelizable dim
    cfgs[3][0]["deg"] = (0, 1, 1, 1)
    cfgs[4][0]["deg"] = (8, 8, 2, 1)     # 128 parts
    cfgs[6][2]["dev_offset"] = 4         # device 4 of 4
    want = oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cfgs)
    got = sim_for(B, 0).simulate(cfgs)
    assert np.array_equal(got, want)
    assert (got[[1, 3, 4, 6]] == B.FF_INVALID_NS).all() and (got[[0, 2, 5, 7]] != B.FF_INVALID_NS).all()


def test_empty_batch_and_argument_errors(B):
    sim = sim_for(B, 0)
    assert B.lib().ff_sim_batch(sim.handle, None, 0, None, None) == B.FF_OK
    assert B.lib().ff_sim_batch(sim.handle, None, 4, None, None) == B.FF_EINVAL
    w = W.workload(0)
    bad_edges = w.edges[::-1].copy()     # not sorted by producer
    with pytest.raises(B.FFSimError):
        B.ff_sim_create(w.ops, bad_edges, w.machine, w.cost)
    zero_cost = w.cost.copy(); zero_cost[0, 0] = 0
    with pytest.raises(B.FFSimError):
        B.ff_sim_create(w.ops, w.edges, w.machine, zero_cost)


def test_general_degrees_strides_and_small_machines(B):
    """beyond the benchmark distribution: non-power-of-two degrees, device strides other
    than 1 (several parts per device), more parts than devices, link latency."""
    rng = np.random.default_rng(5)
    w = W.workload(1)
    mach = W.Machine(3, 2, 7, 3, 5, 9, 4)      # 6 devices
    choices = (1, 2, 3, 4, 5, 6, 7, 12)
    n = 200
    cfgs = np.zeros((n, w.n_ops), W.CFG_DT)
    for i in range(w.n_ops):
        t = W.valid_degree_tuples(w.ops[i], 64, choices)
        cfgs["deg"][:, i] = t[rng.integers(len(t), size=n)]
    cfgs["dev_offset"] = rng.integers(0, 6, size=(n, w.n_ops))
    cfgs["dev_stride"] = rng.integers(0, 9, size=(n, w.n_ops))
    want = oracle.simulate_batch(w.ops, w.edges, mach, w.cost, cfgs, n_threads=8)
    sim = B.Simulator(w.ops, w.edges, mach, w.cost)
    got = sim.simulate(cfgs)
    sim.close()
    bad = np.nonzero(got != want)[0]
    assert len(bad) == 0, f"{len(bad)} differ, first {bad[:5]}: gpu {got[bad[:5]]} oracle {want[bad[:5]]}"


def test_wide_tensors_take_the_64_bit_path(B):
    """a tensor of more than 2^32 bytes: element counts and transfer sizes need 64 bits."""
    g = W.GraphBuilder()
    a = g.op(W.T_ELEM, (1 << 12, 1 << 12, 1 << 9), (0, 1, 2), 1)     # 2^33 elements
    b = g.elementwise([a])
    g.elementwise([b])
    ops, edges, _ = g.finish()
    cost = np.full((3, 64), 1000, "<u4")
    mach = W.Machine(2, 4, 20, 12, 0, 3, 4)
    rng = np.random.default_rng(11)
    n = 64
    cfgs = np.zeros((n, 3), W.CFG_DT)
    t = W.valid_degree_tuples(ops[0], 64, (1, 2, 4, 8))
    for i in range(3):
        cfgs["deg"][:, i] = t[rng.integers(len(t), size=n)]
    cfgs["dev_offset"] = rng.integers(0, 8, size=(n, 3))
    cfgs["dev_stride"] = 1
    cfgs["deg"][0] = 1                      # candidate 0: whole tensors, 2^35 bytes per transfer,
    cfgs["dev_offset"][0] = [0, 1, 4]       # once inside a node and once between nodes
    want = oracle.simulate_batch(ops, edges, mach, cost, cfgs)
    sim = B.Simulator(ops, edges, mach, cost)
    got = sim.simulate(cfgs)
    sim.close()
    assert want[0] == 3 * 1000 + 2 ** 35 // 20 + 1 + (-(-2 ** 35 // 12) + 3)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("config_id,C,steps", [(0, 8, 60), (1, 4, 80), (2, 3, 40), (3, 2, 12), (4, 1, 6)])
def test_delta_chain_matches_resimulation(B, config_id, C, steps):
    """Section 5.3: after every single-op mutation the delta result equals a full
    simulation of the mutated strategy (here: the oracle's)."""
    w = W.workload(config_id)
    cfg0 = w.strategies(C)
    muts = w.mutations(steps, C)
    print(f"delta: config {config_id}, {C} chains x {steps} steps", flush=True)
    sim = sim_for(B, config_id)
    ch = B.Chains(sim, cfg0)
    assert np.array_equal(ch.start_ns(), oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cfg0))
    d_m = ch.upload_mutations(muts)
    got = ch.delta(d_m, steps).cpu().numpy().view("<u8")
    for c in range(C):
        want = oracle.simulate_delta_chain(w.ops, w.edges, w.machine, w.cost, cfg0[c], muts[:, c])
        bad = np.nonzero(got[:, c] != want)[0]
        assert len(bad) == 0, f"chain {c}: first differing step {bad[0]} (op {int(muts[bad[0], c]['op'])}): gpu {got[bad[0], c]} oracle {want[bad[0]]}"
    st = ch.stats()
    print(f"resumed {int(st['n_resumed'].sum())} of {int(st['n_steps'].sum())} steps, {int(st['n_converged'].sum())} re-joined the previous timeline", flush=True)
    if config_id == 2:
        # this case is known to contain steps whose timeline re-joins the previous one: the early stop is exercised
        assert st["n_converged"].sum() > 0
    ch.close()


def test_delta_in_several_calls_and_inverse_mutation(B):
    """the chain state survives between ff_sim_delta calls; a mutation followed by its
    inverse restores the previous value; mutating the first and the last op works."""
    w = W.workload(2)
    cfg0 = w.strategies(2)
    sim = sim_for(B, 2)
    ch = B.Chains(sim, cfg0)
    start = ch.start_ns().copy()
    m = w.mutations(6, 2)
    m["op"][0] = 0
    m["op"][2] = w.n_ops - 1
    fwd = np.zeros((12, 2), W.MUT_DT)
    fwd[0::2] = m
    for s in range(6):           # odd steps undo the even ones
        prev = cfg0.copy()
        fwd[2 * s + 1]["op"] = m[s]["op"]
        for c in range(2):
            fwd[2 * s + 1, c]["cfg"] = prev[c, int(m[s, c]["op"])]
    got = np.concatenate([ch.delta(ch.upload_mutations(fwd[a:b]), b - a).cpu().numpy().view("<u8")
                          for a, b in ((0, 5), (5, 6), (6, 12))])
    for c in range(2):
        want = oracle.simulate_delta_chain(w.ops, w.edges, w.machine, w.cost, cfg0[c], fwd[:, c])
        assert np.array_equal(got[:, c], want)
        assert (got[1::2, c] == start[c]).all()
    ch.close()


def test_delta_invalid_mutations(B):
    """an invalid configuration gives FF_INVALID_NS until a later mutation repairs it; a
    mutation naming an op outside the graph poisons the chain for good."""
    w = W.workload(1)
    cfg0 = w.strategies(2)
    sim = sim_for(B, 1)
    ch = B.Chains(sim, cfg0)
    muts = w.mutations(6, 2)
    muts[1, 0]["cfg"]["deg"] = (64, 64, 1, 1)          # chain 0: too many parts at step 1
    muts[2, 0]["op"] = muts[1, 0]["op"]                # ... repaired at step 2
    muts[3, 1]["op"] = w.n_ops + 5                     # chain 1: poisoned from step 3 on
    got = ch.delta(ch.upload_mutations(muts), 6).cpu().numpy().view("<u8")
    want0 = oracle.simulate_delta_chain(w.ops, w.edges, w.machine, w.cost, cfg0[0], muts[:, 0])
    assert want0[1] == oracle.INVALID and want0[2] != oracle.INVALID
    assert np.array_equal(got[:, 0], want0)
    want1 = oracle.simulate_delta_chain(w.ops, w.edges, w.machine, w.cost, cfg0[1], muts[:3, 1])
    assert np.array_equal(got[:3, 1], want1)
    assert (got[3:, 1] == B.FF_INVALID_NS).all()
    ch.close()


def test_more_candidates_than_resident_wavefronts(B):
    """B larger than the number of wavefronts the device holds at once: wavefronts stride
    over the batch and reuse their state."""
    w = W.workload(1)
    n = 9000
    cfgs = w.strategies(n)
    want = oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cfgs, n_threads=8)
    got = sim_for(B, 1).simulate(cfgs)
    assert np.array_equal(got, want)
    w = W.workload(2)            # task words in HBM: one workspace slot per resident wavefront
    sim = sim_for(B, 2)
    n = 9000
    cfgs = w.strategies(n)
    got = sim.simulate(cfgs)
    idx = np.arange(0, n, 150)
    want = oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cfgs[idx], n_threads=8)
    assert B.ff_sim_workspace_bytes(sim.handle, n) < n * B.ff_sim_workspace_bytes(sim.handle, 1)   # fewer slots than candidates
    assert np.array_equal(got[idx], want)


def test_advertised_workspace_is_enough_for_any_batch_size(B):
    """ff_sim_batch must accept exactly ff_sim_workspace_bytes(B) bytes, also for batches larger than
    the number of wavefronts either kernel variant keeps resident."""
    import torch
    w = W.workload(2)
    h = B.ff_sim_create(w.ops, w.edges, w.machine, w.cost)
    L = B.lib()
    for n in (1, 700, 5000, 20000):
        cfgs = w.strategies(n if n <= 5000 else 5000)
        if n > 5000:
            cfgs = np.concatenate([cfgs] * 4)
        d = B.to_device(cfgs)
        out = torch.empty(n, dtype=torch.int64, device="cuda")
        need = B.ff_sim_workspace_bytes(h, n)
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        assert L.ff_sim_set_workspace(h, ws.data_ptr(), need) == B.FF_OK
        assert L.ff_sim_batch(h, d.data_ptr(), n, out.data_ptr(), None) == B.FF_OK
        torch.cuda.synchronize()
        if n == 700:
            assert np.array_equal(out.cpu().numpy().view("<u8")[::100], oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cfgs[::100], n_threads=8))
        assert L.ff_sim_set_workspace(h, ws.data_ptr(), need - 256) == B.FF_OK
        assert L.ff_sim_batch(h, d.data_ptr(), n, out.data_ptr(), None) == B.FF_EWORKSPACE
    torch.cuda.synchronize()
    B.ff_sim_destroy(h)


def test_graphs_without_edges_and_single_op(B):
    g = W.GraphBuilder()
    for _ in range(5):
        g.op(W.T_ELEM, (64, 32), (0, 1), 1)
    ops, edges, _ = g.finish()
    cost = np.tile(np.arange(100, 164, dtype="<u4"), (5, 1))
    mach = W.Machine(2, 2)
    cfgs = W.strategies(ops, 40, 3, 4, 16, (1, 2, 4, 8, 16))
    sim = B.Simulator(ops, edges, mach, cost)
    assert np.array_equal(sim.simulate(cfgs), oracle.simulate_batch(ops, edges, mach, cost, cfgs))
    sim.close()
    sim = B.Simulator(ops[:1], edges, mach, cost[:1])
    assert np.array_equal(sim.simulate(cfgs[:, :1]), oracle.simulate_batch(ops[:1], edges, mach, cost[:1], cfgs[:, :1]))
    sim.close()


def test_many_parts_on_few_devices_and_wide_fan_in(B):
    """64 parts per op on a 1x2 machine (32 tasks per device queue up in id order) and an op
    with 40 producers."""
    g = W.GraphBuilder()
    srcs = [g.op(W.T_ELEM, (64, 64), (0, 1), 1) for _ in range(40)]
    mids = [g.elementwise([s]) for s in srcs]
    top = g.op(W.T_STACK, (64, 40, 64), (0, 2), 1)
    for m in mids:
        g.edge(m, top, [W.ident(0), W.ident(2)])
    g.softmax(top)
    ops, edges, _ = g.finish()
    rng = np.random.default_rng(2)
    cost = rng.integers(1, 5000, size=(len(ops), 64)).astype("<u4")
    for mach in (W.Machine(1, 2, 5, 3, 1, 2, 4), W.Machine(16, 4)):
        cfgs = W.strategies(ops, 48, 9, mach.n_devices, 64, (1, 2, 4, 8, 16, 32, 64))
        cfgs["dev_stride"] = rng.integers(0, 4, size=cfgs.shape)
        sim = B.Simulator(ops, edges, mach, cost)
        got, st = sim.simulate(cfgs, stats=True)
        want = oracle.simulate_batch(ops, edges, mach, cost, cfgs, n_threads=8)
        assert not st["exit_code"].any() and not st["n_stuck"].any()
        assert np.array_equal(got, want)
        sim.close()


def test_time_limit_is_reported_not_wrapped(B):
    """simulated times are limited to 2^48 ns; a candidate that gets there returns
    FF_OVERFLOW_NS (the oracle, with full 64-bit times, confirms the true value is beyond)."""
    g = W.GraphBuilder()
    x = g.op(W.T_ELEM, (64, 64), (0, 1), 1)
    for _ in range(1099):
        x = g.elementwise([x])
    ops, edges, _ = g.finish()
    cost = np.full((1100, 64), 2 ** 32 - 1, "<u4")
    cost[:, 0] = 1000
    mach = W.Machine(1, 2)
    cfgs = np.zeros((2, 1100), W.CFG_DT)
    cfgs["deg"] = 1
    cfgs["deg"][1, :, 0] = 64          # candidate 1: 64 parts per op, all on device 0, 2^32-1 ns each
    cfgs["dev_stride"] = 0
    want = oracle.simulate_batch(ops, edges, mach, cost, cfgs)
    sim = B.Simulator(ops, edges, mach, cost)
    got = sim.simulate(cfgs)
    sim.close()
    assert want[0] == 1100 * 1000 and got[0] == want[0]
    assert want[1] >= 2 ** 48 and got[1] == 2 ** 64 - 3


def test_workspace_errors_and_other_stream(B):
    import torch
    w = W.workload(2)
    h = B.ff_sim_create(w.ops, w.edges, w.machine, w.cost)
    cfgs = w.strategies(16)
    d = B.to_device(cfgs)
    out = torch.empty(16, dtype=torch.int64, device="cuda")
    L = B.lib()
    assert L.ff_sim_batch(h, d.data_ptr(), 16, out.data_ptr(), None) == B.FF_EWORKSPACE     # none set
    need = B.ff_sim_workspace_bytes(h, 16)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    assert L.ff_sim_set_workspace(h, ws.data_ptr() + 8, need - 8) == B.FF_EINVAL             # misaligned
    assert L.ff_sim_set_workspace(h, ws.data_ptr(), need // 2) == B.FF_OK
    assert L.ff_sim_batch(h, d.data_ptr(), 16, out.data_ptr(), None) == B.FF_EWORKSPACE     # too small
    assert L.ff_sim_set_workspace(h, ws.data_ptr(), need) == B.FF_OK
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        assert L.ff_sim_batch(h, d.data_ptr(), 16, out.data_ptr(), s.cuda_stream) == B.FF_OK
    s.synchronize()
    want = oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cfgs)
    assert np.array_equal(out.cpu().numpy().view("<u8"), want)
    B.ff_sim_destroy(h)
    # limits are reported at creation
    big = w.ops.copy(); big[0]["extent"][2] = 2 ** 21
    with pytest.raises(B.FFSimError) as e:
        B.ff_sim_create(big, w.edges, w.machine, w.cost)
    assert e.value.code == B.FF_ERANGE


@pytest.mark.parametrize("seed", range(6))
def test_random_graphs_machines_and_strategies(B, seed):
    rng = np.random.default_rng(1000 + seed)
    n_ops = int(rng.integers(3, 90))
    ops, edges, _ = random_graph(rng, n_ops)
    n_nodes, gpn = int(rng.integers(1, 6)), int(rng.integers(1, 5))
    mach = W.Machine(n_nodes, gpn, int(rng.integers(1, 30)), int(rng.integers(1, 30)),
                     int(rng.integers(0, 50)), int(rng.integers(0, 50)), int(rng.choice([1, 2, 4, 8])))
    cost = rng.integers(1, 3000, size=(n_ops, 64)).astype("<u4")
    n = 160
    cfgs = np.zeros((n, n_ops), W.CFG_DT)
    for i in range(n_ops):
        t = W.valid_degree_tuples(ops[i], 64, (1, 2, 3, 4, 5, 7, 8, 16, 32, 64))
        cfgs["deg"][:, i] = t[rng.integers(len(t), size=n)]
    cfgs["dev_offset"] = rng.integers(0, mach.n_devices, size=(n, n_ops))
    cfgs["dev_stride"] = rng.integers(0, 5, size=(n, n_ops))
    print(f"seed {seed}: {n_ops} ops, {len(edges)} edges, machine {mach.as_tuple()}", flush=True)
    want = oracle.simulate_batch(ops, edges, mach, cost, cfgs, n_threads=8)
    sim = B.Simulator(ops, edges, mach, cost)
    got, st = sim.simulate(cfgs, stats=True)
    assert not st["exit_code"].any() and not st["n_stuck"].any()
    bad = np.nonzero(got != want)[0]
    assert len(bad) == 0, f"{len(bad)} differ, first {bad[:5]}: gpu {got[bad[:5]]} oracle {want[bad[:5]]}"
    # and a mutation chain on the same graph
    muts = np.zeros((30, 2), W.MUT_DT)
    muts["op"] = rng.integers(0, n_ops, size=(30, 2))
    for s in range(30):
        for c in range(2):
            i = int(muts[s, c]["op"])
            t = W.valid_degree_tuples(ops[i], 64, (1, 2, 3, 4, 8, 16))
            muts[s, c]["cfg"]["deg"] = t[rng.integers(len(t))]
            muts[s, c]["cfg"]["dev_offset"] = rng.integers(0, mach.n_devices)
            muts[s, c]["cfg"]["dev_stride"] = rng.integers(0, 3)
    ch = B.Chains(sim, cfgs[:2])
    d = ch.delta(ch.upload_mutations(muts), 30).cpu().numpy().view("<u8")
    for c in range(2):
        ref = oracle.simulate_delta_chain(ops, edges, mach, cost, cfgs[c], muts[:, c])
        assert np.array_equal(d[:, c], ref), f"chain {c}: steps {np.nonzero(d[:, c] != ref)[0][:5]}"
    ch.close()
    sim.close()


@pytest.mark.parametrize("config_id,C,M", [(1, 3, 40), (2, 2, 24), (4, 1, 6)])
def test_trial_mutations_do_not_change_the_chain(B, config_id, C, M):
    """ff_sim_delta_try: M proposals per chain, each equal to a full simulation of the
    chain's current strategy with that one op changed; the chains continue afterwards as
    if nothing had been tried."""
    w = W.workload(config_id)
    sim = sim_for(B, config_id)
    cfg0 = w.strategies(C)
    ch = B.Chains(sim, cfg0)
    warm = w.mutations(5, C)
    ch.delta(ch.upload_mutations(warm), 5)
    cur = cfg0.copy()
    for s in range(5):
        for c in range(C):
            cur[c, int(warm[s, c]["op"])] = warm[s, c]["cfg"]
    props = w.mutations(5 + M, C)[5:]
    props["op"][0] = 0                       # a source op: nothing of the old timeline can be kept
    props["op"][1] = w.n_ops - 1
    props[2, 0]["cfg"]["deg"] = (64, 64, 1, 1)   # an invalid proposal
    got = ch.try_mutations(ch.upload_mutations(props), M).cpu().numpy().view("<u8")
    for c in range(C):
        cand = np.repeat(cur[c][None], M, 0)
        for p in range(M):
            cand[p, int(props[p, c]["op"])] = props[p, c]["cfg"]
        want = oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cand, n_threads=8)
        bad = np.nonzero(got[:, c] != want)[0]
        assert len(bad) == 0, f"chain {c}: proposals {bad[:5]} gpu {got[bad[:5], c]} oracle {want[bad[:5]]}"
    assert got[2, 0] == B.FF_INVALID_NS
    more = w.mutations(9, C)[5:]
    after = ch.delta(ch.upload_mutations(more), 4).cpu().numpy().view("<u8")
    for c in range(C):
        ref = oracle.simulate_delta_chain(w.ops, w.edges, w.machine, w.cost, cur[c], more[:, c])
        assert np.array_equal(after[:, c], ref)
    ch.close()


def test_delta_respaces_snapshots_when_the_timeline_shrinks(B):
    """a chain that starts unsplit on one device (long timeline) and is then mutated op by op
    to 16-way splits: the makespan falls by an order of magnitude; results stay exact."""
    w = W.workload(1)
    sim = sim_for(B, 1)
    cfg0 = np.zeros((1, w.n_ops), W.CFG_DT)
    cfg0["deg"] = 1
    cfg0["dev_stride"] = 1
    P = 16
    muts = np.zeros((3 * w.n_ops, 1), W.MUT_DT)
    for s in range(3 * w.n_ops):
        i = s % w.n_ops
        muts[s, 0]["op"] = i
        muts[s, 0]["cfg"]["deg"] = (min(P, int(w.ops[i]["extent"][0])) if s < 2 * w.n_ops else 1, 1, 1, 1)
        muts[s, 0]["cfg"]["dev_offset"] = s % 3
        muts[s, 0]["cfg"]["dev_stride"] = 1
    ch = B.Chains(sim, cfg0)
    got = ch.delta(ch.upload_mutations(muts), len(muts)).cpu().numpy().view("<u8")
    want = oracle.simulate_delta_chain(w.ops, w.edges, w.machine, w.cost, cfg0[0], muts[:, 0])
    assert want.max() > 4 * want.min()
    assert np.array_equal(got[:, 0], want)
    ch.close()


def test_trial_mutations_need_a_workspace(B):
    import torch
    w = W.workload(0)
    h = B.ff_sim_create(w.ops, w.edges, w.machine, w.cost)
    cfg0 = w.strategies(2)
    d = B.to_device(cfg0)
    out0 = torch.empty(2, dtype=torch.int64, device="cuda")
    ch = B.ff_sim_chains_create(h, d.data_ptr(), 2, out0.data_ptr())
    props = B.to_device(w.mutations(4, 2))
    out = torch.empty((4, 2), dtype=torch.int64, device="cuda")
    L = B.lib()
    assert L.ff_sim_delta_try(ch, props.data_ptr(), 4, out.data_ptr(), None) == B.FF_EWORKSPACE
    need = B.ff_sim_delta_try_workspace_bytes(ch, 4)
    assert need > 0
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    B.ff_sim_set_workspace(h, ws.data_ptr(), need)
    assert L.ff_sim_delta_try(ch, props.data_ptr(), 4, out.data_ptr(), None) == B.FF_OK
    assert L.ff_sim_delta_try(ch, None, 0, None, None) == B.FF_OK
    torch.cuda.synchronize()
    B.ff_sim_chains_destroy(ch)
    B.ff_sim_destroy(h)


@pytest.mark.parametrize("seed,n_nodes,gpn", [(0, 1, 4), (1, 3, 1), (2, 2, 2), (3, 5, 3), (4, 4, 4), (5, 3, 5),
                                               (6, 2, 8), (7, 7, 8), (8, 2, 9), (9, 6, 2)])
def test_random_graphs_with_regular_strategies(B, seed, n_nodes, gpn):
    """every op on consecutive, distinct devices (stride 1, parts <= devices): the form of the
    event loop that serialises transfers on shared link rows with a running sum along the lanes.
    Machine shapes cover one GPU per node, non-powers of two, eight and nine GPUs per node (nine
    is beyond that form's limit) and offsets that make the device numbers wrap around."""
    rng = np.random.default_rng(7000 + seed)
    n_ops = int(rng.integers(3, 70))
    ops, edges, _ = random_graph(rng, n_ops)
    mach = W.Machine(n_nodes, gpn, int(rng.integers(1, 30)), int(rng.integers(1, 30)),
                     int(rng.integers(0, 50)), int(rng.integers(0, 50)), int(rng.choice([1, 2, 4, 8])))
    D = mach.n_devices
    cost = rng.integers(1, 3000, size=(n_ops, 64)).astype("<u4")
    n = 200
    cfgs = np.zeros((n, n_ops), W.CFG_DT)
    for i in range(n_ops):
        t = W.valid_degree_tuples(ops[i], min(64, D), (1, 2, 3, 4, 5, 6, 7, 8, 16, 32, 64))
        cfgs["deg"][:, i] = t[rng.integers(len(t), size=n)]
    cfgs["dev_offset"] = rng.integers(0, D, size=(n, n_ops))
    cfgs["dev_offset"][: n // 4] = D - 1          # many wrap-arounds
    cfgs["dev_stride"] = 1
    cfgs["dev_stride"][-1, 0] = 2                 # one candidate that needs the general form
    print(f"seed {seed}: {n_ops} ops, {len(edges)} edges, machine {mach.as_tuple()}", flush=True)
    want = oracle.simulate_batch(ops, edges, mach, cost, cfgs, n_threads=8)
    sim = B.Simulator(ops, edges, mach, cost)
    got, st = sim.simulate(cfgs, stats=True)
    assert not st["exit_code"].any() and not st["n_stuck"].any()
    bad = np.nonzero(got != want)[0]
    assert len(bad) == 0, f"{len(bad)} differ, first {bad[:5]}: gpu {got[bad[:5]]} oracle {want[bad[:5]]}"
    assert np.array_equal(sim.simulate(cfgs), want)          # and the kernel without the counters
    # chains that stay regular, with one irregular mutation in the middle
    muts = np.zeros((24, 2), W.MUT_DT)
    muts["op"] = rng.integers(0, n_ops, size=(24, 2))
    for s in range(24):
        for c in range(2):
            i = int(muts[s, c]["op"])
            t = W.valid_degree_tuples(ops[i], min(64, D), (1, 2, 3, 4, 8, 16))
            muts[s, c]["cfg"]["deg"] = t[rng.integers(len(t))]
            muts[s, c]["cfg"]["dev_offset"] = rng.integers(0, D)
            muts[s, c]["cfg"]["dev_stride"] = 1
    muts[11, 0]["cfg"]["dev_stride"] = 3
    ch = B.Chains(sim, cfgs[:2])
    d = ch.delta(ch.upload_mutations(muts), 24).cpu().numpy().view("<u8")
    for c in range(2):
        ref = oracle.simulate_delta_chain(ops, edges, mach, cost, cfgs[c], muts[:, c])
        assert np.array_equal(d[:, c], ref), f"chain {c}: steps {np.nonzero(d[:, c] != ref)[0][:5]}"
    ch.close()
    sim.close()


@pytest.mark.parametrize("config_id,n", [(0, 64), (1, 256), (2, 48)])
def test_costs_keyed_by_degree_tuple(B, config_id, n):
    """the second cost model (ff_sim_create_tuplecost): batch, invalid because a tuple is not
    listed, delta chain, trial proposals and search, all against the oracle with the same lists"""
    from oracle import search as S
    w = W.workload(config_id)
    tc = w.tuple_costs()
    sim = B.Simulator(w.ops, w.edges, w.machine, tc)
    cfgs = w.strategies(n).copy()
    cfgs[3, 0]["deg"] = (3, 1, 1, 1)       # a valid configuration of op 0 (extent >= 3) that the list does not hold
    want = oracle.simulate_batch(w.ops, w.edges, w.machine, tc, cfgs, n_threads=8)
    assert want[3] == oracle.INVALID and (want != oracle.INVALID).sum() == n - 1
    got = sim.simulate(cfgs)
    bad = np.nonzero(got != want)[0]
    assert len(bad) == 0, f"{len(bad)} differ, first {bad[:5]}: gpu {got[bad[:5]]} oracle {want[bad[:5]]}"
    assert (got != oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cfgs, n_threads=8)).any()   # the surcharges matter
    C = 2
    muts = w.mutations(12, C)
    ch = B.Chains(sim, cfgs[:C])
    d = ch.delta(ch.upload_mutations(muts), 12).cpu().numpy().view("<u8")
    cur = cfgs[:C].copy()
    for c in range(C):
        assert np.array_equal(d[:, c], oracle.simulate_delta_chain(w.ops, w.edges, w.machine, tc, cfgs[c], muts[:, c]))
        for s in range(12):
            cur[c, int(muts[s, c]["op"])] = muts[s, c]["cfg"]
    tp, tu = w.search_space()
    t0 = int(oracle.simulate_batch(w.ops, w.edges, w.machine, tc, cur[:1])[0])
    table = S.metropolis_table(30.0 / t0, max(1, t0 // 256), 64)
    ch.search_setup(tp, tu, table, max(1, t0 // 256), 5)
    tr = ch.search(20).cpu().numpy().view("<u8")
    for c in range(C):
        ref = S.metropolis_chain(w.ops, w.edges, w.machine, tc, cur[c], tp, tu, table, max(1, t0 // 256), 5, c, 0, 20)[0]
        assert np.array_equal(tr[:, c], ref)
    ch.close()
    sim.close()


def test_costs_from_the_measurement_cache(B):
    """cost lists built through the (operation type, output size) cache of Section 5.1 (costcache.tuple_costs) on the
    Inception-shaped graph: batch and a mutation chain against the oracle with the same lists"""
    from paper_1807_05358_amd import costcache
    w = W.workload(2)
    tc = costcache.tuple_costs(w.ops, w.max_parts, w.choices, costcache.ExeTimeCache(costcache.model_measure))
    sim = B.Simulator(w.ops, w.edges, w.machine, tc)
    cfgs = w.strategies(96)
    want = oracle.simulate_batch(w.ops, w.edges, w.machine, tc, cfgs, n_threads=8)
    assert (want != oracle.INVALID).all()
    assert np.array_equal(sim.simulate(cfgs), want)
    muts = w.mutations(16, 2)
    ch = B.Chains(sim, cfgs[:2])
    d = ch.delta(ch.upload_mutations(muts), 16).cpu().numpy().view("<u8")
    for c in range(2):
        assert np.array_equal(d[:, c], oracle.simulate_delta_chain(w.ops, w.edges, w.machine, tc, cfgs[c], muts[:, c]))
    ch.close()
    sim.close()


def test_tuple_cost_argument_errors(B):
    w = W.workload(0)
    ptr, tup, ns = w.tuple_costs()
    with pytest.raises(B.FFSimError):                 # not ascending
        B.ff_sim_create_tuplecost(w.ops, w.edges, w.machine, ptr, tup[::-1].copy(), ns)
    z = ns.copy(); z[1] = 0
    with pytest.raises(B.FFSimError):                 # a zero exeTime
        B.ff_sim_create_tuplecost(w.ops, w.edges, w.machine, ptr, tup, z)
    p2 = ptr.copy(); p2[0] = 1
    with pytest.raises(B.FFSimError):
        B.ff_sim_create_tuplecost(w.ops, w.edges, w.machine, p2, tup, ns)
    h = B.ff_sim_create_tuplecost(w.ops, w.edges, w.machine, ptr, tup, ns)
    B.ff_sim_destroy(h)


def test_largest_graph_and_largest_machines(B):
    """the limits of the boundary: FF_MAX_OPS ops (64 groups in the queue's upper level), extents of
    FF_MAX_EXTENT (too large for the kept per-edge set-up), a machine whose device rows nearly
    fill a workgroup's 160 KB of LDS, a node with more GPUs than the regular event loop handles;
    and machines beyond the limit are refused."""
    rng = np.random.default_rng(77)
    ops, edges, _ = random_graph(rng, 4096)
    assert len(ops) == 4096
    mach = W.Machine(16, 4, 7, 3, 11, 29, 2)
    cost = rng.integers(1, 3000, size=(4096, 64)).astype("<u4")
    n = 6
    cfgs = np.zeros((n, 4096), W.CFG_DT)
    for i in range(4096):
        t = W.valid_degree_tuples(ops[i], 64, (1, 2, 3, 4, 8, 16, 64))
        cfgs["deg"][:, i] = t[rng.integers(len(t), size=n)]
    cfgs["dev_offset"] = rng.integers(0, mach.n_devices, size=(n, 4096))
    cfgs["dev_stride"] = 1
    cfgs["dev_stride"][n // 2:] = rng.integers(0, 4, size=(n - n // 2, 4096))
    sim = B.Simulator(ops, edges, mach, cost)
    got, st = sim.simulate(cfgs, stats=True)
    assert not st["exit_code"].any() and not st["n_stuck"].any()
    assert np.array_equal(got, oracle.simulate_batch(ops, edges, mach, cost, cfgs, n_threads=8))
    muts = np.zeros((4, 1), W.MUT_DT)
    muts["op"][:, 0] = [4095, 0, 2048, 4095]
    for s in range(4):
        i = int(muts[s, 0]["op"])
        t = W.valid_degree_tuples(ops[i], 64, (1, 2, 4, 8))
        muts[s, 0]["cfg"]["deg"] = t[rng.integers(len(t))]
        muts[s, 0]["cfg"]["dev_offset"] = rng.integers(0, mach.n_devices)
        muts[s, 0]["cfg"]["dev_stride"] = 1
    ch = B.Chains(sim, cfgs[:1])
    d = ch.delta(ch.upload_mutations(muts), 4).cpu().numpy().view("<u8")
    assert np.array_equal(d[:, 0], oracle.simulate_delta_chain(ops, edges, mach, cost, cfgs[0], muts[:, 0]))
    ch.close()
    sim.close()

    # extents at the limit on a 64 x 4 machine (5376 device rows), on 2 x 32 (general loop only)
    # and on 120 x 1 (14640 device rows: 130 KB of LDS per candidate)
    g = W.GraphBuilder()
    a = g.op(W.T_ELEM, (1 << 20, 64), (0, 1), 1)
    b = g.elementwise([a])
    c = g.op(W.T_ELEM, (64, 1 << 20), (0, 1), 1)
    g.edge(b, c, [W.ALL, W.ident(0)])
    g.elementwise([c])
    ops, edges, _ = g.finish()
    cost = rng.integers(1, 100000, size=(len(ops), 64)).astype("<u4")
    for mach in (W.Machine(64, 4, 20, 12, 0, 5, 4), W.Machine(2, 32, 3, 1, 2, 0, 8), W.Machine(120, 1)):
        cfgs = W.strategies(ops, 64, 5, mach.n_devices, 64, (1, 2, 4, 8, 16, 32, 64))
        sim = B.Simulator(ops, edges, mach, cost)
        got = sim.simulate(cfgs)
        want = oracle.simulate_batch(ops, edges, mach, cost, cfgs, n_threads=8)
        assert np.array_equal(got, want), f"machine {mach.as_tuple()}: {np.nonzero(got != want)[0][:5]}"
        sim.close()
    for mach in (W.Machine(256, 4), W.Machine(1, 1024), W.Machine(1024, 1)):
        with pytest.raises(B.FFSimError) as e:
            B.ff_sim_create(ops, edges, mach, cost)
        assert e.value.code == B.FF_ERANGE
    with pytest.raises(B.FFSimError) as e:
        B.ff_sim_create(ops, edges, W.Machine(1025, 1), cost)
    assert e.value.code == B.FF_ERANGE
