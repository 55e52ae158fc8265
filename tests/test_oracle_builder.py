"""Pins for the oracle's task-graph construction (Section 5.1) and for build + simulate:
hand-computed fixtures, task/pair counts, the shared-volume identity, closed forms,
symmetries, invalid strategies, and the definition of the delta result."""
import numpy as np
import pytest

import oracle
from helpers import check_timeline, critical_path, graph_from_golden, load_golden
from paper_1807_05358_amd import workloads as W


def cfgs_all(ops, deg=(1, 1, 1, 1), off=0, stride=1):
    cfg = np.zeros(len(ops), W.CFG_DT)
    cfg["deg"] = deg
    cfg["dev_offset"] = off
    cfg["dev_stride"] = stride
    return cfg


@pytest.mark.parametrize("name", ["build_two_ops_two_gpus.json", "build_shared_internode_link.json",
                                  "build_part_order_row_major.json", "build_link_latency.json",
                                  "build_intranode_latency.json", "build_uneven_split_7_by_3.json",
                                  "build_uneven_split_35_by_4.json", "build_strided_window_uneven_split.json",
                                  "build_pair_order_on_shared_link.json"])
def test_hand_computed_build_and_timeline(golden_dir, name):
    g = load_golden(golden_dir, name)
    tg = oracle.build_task_graph(*graph_from_golden(g))
    assert tg.exe.tolist() == g["exe"]
    assert tg.dev.tolist() == g["dev"]
    assert sorted(zip(tg.dep_src.tolist(), tg.dep_dst.tolist())) == sorted(map(tuple, g["deps"]))
    mk, ready, start, end = tg.simulate()
    assert start.tolist() == g["start"] and end.tolist() == g["end"] and mk == g["makespan"]


@pytest.mark.parametrize("name", ["build_conv_window_pairs.json", "build_strided_window_uneven_split.json"])
def test_hand_computed_window_pairs(golden_dir, name):
    g = load_golden(golden_dir, name)
    tg = oracle.build_task_graph(*graph_from_golden(g))
    comm = []
    for c in range(tg.n_compute, tg.n_tasks):
        (p,) = tg.dep_src[tg.dep_dst == c]
        (q,) = tg.dep_dst[tg.dep_src == c]
        comm.append([int(p), int(q), int(tg.exe[c])])
    assert comm == g["comm"]


def part_bounds(E, deg):
    return [(p * E) // deg for p in range(deg + 1)]


def needed_volume(w, e, cfg):
    """sum over consumer parts of the volume of the producer sub-tensor each one reads
    (independent of how the producer is split)."""
    edge = w.edges[e]
    prod, cons = w.ops[edge["src_op"]], w.ops[edge["dst_op"]]
    cdeg = cfg[edge["dst_op"]]["deg"]
    total = 0
    for idx in np.ndindex(*[int(d) for d in cdeg]):
        vol = 1
        for d in range(prod["ndim"]):
            m = edge["map"][d]
            E = int(prod["extent"][d])
            if m["src_dim"] < 0:
                vol *= E
                continue
            c = int(m["src_dim"])
            b = part_bounds(int(cons["extent"][c]) if c < cons["ndim"] else 1, int(cdeg[c]))
            lo, hi = b[idx[c]], b[idx[c] + 1]
            nlo = max(0, lo * int(m["stride"]) + int(m["a"]))
            nhi = min(E, (hi - 1) * int(m["stride"]) + int(m["b"]) + 1)
            vol *= max(0, nhi - nlo)
        total += vol
    return total


@pytest.mark.parametrize("config_id", [0, 1, 2])
def test_shared_volume_identity(config_id):
    """With 4-byte elements on 4 B/ns links the transfer time equals the shared element
    count; with producers and consumers on disjoint device sets every pair is a transfer.
    Then, per edge, the transfer times must add up to the volume the consumer parts read,
    because the producer parts tile the producer tensor."""
    w = W.workload(config_id)
    mach = W.Machine(1, 128, 4, 4, 0, 0, 4)
    rng = np.random.default_rng(config_id)
    cfg = w.strategies(8)[int(rng.integers(8))].copy()
    ops = w.ops
    # ops alternate between device halves so that neighbours never share a device;
    # for non-chain graphs fall back to checking only edges whose ends are in different halves
    half = np.zeros(len(ops), int)
    for e in w.edges:
        half[e["dst_op"]] = 1 - half[e["src_op"]]
    cfg["dev_offset"] = half * 64
    tg = oracle.build_task_graph(ops, w.edges, mach, w.cost, cfg)
    parts = cfg["deg"].astype(int).prod(1)
    first = np.concatenate(([0], np.cumsum(parts)))
    assert tg.n_compute == parts.sum()                     # step 1: |c_i| tasks per op
    op_of = np.repeat(np.arange(len(ops)), parts)
    # per edge sums of transfer times; transfers are created in edge order
    comm = np.arange(tg.n_compute, tg.n_tasks)
    src_of = np.zeros(tg.n_tasks, int)
    dst_of = np.zeros(tg.n_tasks, int)
    is_comm_dst = tg.dep_dst >= tg.n_compute
    src_of[tg.dep_dst[is_comm_dst]] = tg.dep_src[is_comm_dst]
    is_comm_src = tg.dep_src >= tg.n_compute
    dst_of[tg.dep_src[is_comm_src]] = tg.dep_dst[is_comm_src]
    checked = 0
    for e, edge in enumerate(w.edges):
        i, j = int(edge["src_op"]), int(edge["dst_op"])
        if half[i] == half[j]:
            continue
        sel = comm[(op_of[src_of[comm]] == i) & (op_of[dst_of[comm]] == j)]
        # several edges between the same op pair do not occur in these graphs
        assert tg.exe[sel].sum() == needed_volume(w, e, cfg), f"edge {e}"
        checked += 1
    assert checked >= len(w.edges) // 2


def test_pair_count_for_aligned_identity_edges():
    """elementwise edge, power-of-two splits of power-of-two extents: the number of
    overlapping pairs is prod_d max(deg_producer[d], deg_consumer[d])."""
    g = W.GraphBuilder()
    a = g.op(W.T_ELEM, (64, 32, 16, 8), (0, 1, 2, 3), 1)
    g.elementwise([a])
    ops, edges, _ = g.finish()
    cost = np.full((2, 64), 10, "<u4")
    mach = W.Machine(16, 4)
    rng = np.random.default_rng(3)
    for _ in range(40):
        cfg = np.zeros(2, W.CFG_DT)
        for i in range(2):
            t = W.valid_degree_tuples(ops[i], 64, (1, 2, 4, 8))
            cfg[i]["deg"] = t[rng.integers(len(t))]
        cfg["dev_offset"] = [0, 0]
        cfg["dev_stride"] = [0, 0]            # everything on device 0: pairs are plain dependencies
        tg = oracle.build_task_graph(ops, edges, mach, cost, cfg)
        assert tg.n_tasks == tg.n_compute
        assert tg.n_deps == np.maximum(cfg[0]["deg"], cfg[1]["deg"]).astype(int).prod()
        cfg["dev_offset"] = [0, 1]            # producer on device 0, consumer on 1: all transfers
        tg = oracle.build_task_graph(ops, edges, mach, cost, cfg)
        assert tg.n_tasks - tg.n_compute == np.maximum(cfg[0]["deg"], cfg[1]["deg"]).astype(int).prod()


@pytest.mark.parametrize("config_id", [0, 1, 2, 3])
def test_unsplit_on_one_device_is_sum_of_costs(config_id):
    w = W.workload(config_id)
    cfg = cfgs_all(w.ops, off=w.machine.n_devices - 1)
    tg = oracle.build_task_graph(w.ops, w.edges, w.machine, w.cost, cfg)
    assert tg.n_tasks == tg.n_compute == w.n_ops                 # same device => no transfers
    assert tg.n_deps == len(w.edges)
    assert tg.simulate()[0] == w.cost[:, 0].astype(np.int64).sum()


@pytest.mark.parametrize("config_id", [0, 1])
def test_unsplit_chain_one_op_per_device(config_id):
    """chain, every op unsplit, op i on device i mod D: makespan = sum of op times plus the
    transfer time of every tensor (each consumer reads its whole input here)."""
    w = W.workload(config_id)
    m = w.machine
    cfg = cfgs_all(w.ops)
    cfg["dev_offset"] = np.arange(w.n_ops) % m.n_devices
    expect = int(w.cost[:, 0].astype(np.int64).sum())
    for e in w.edges:
        i, j = int(e["src_op"]), int(e["dst_op"])
        nbytes = int(w.ops[i]["extent"].astype(np.int64).prod()) * m.elem_bytes
        same_node = (i % m.n_devices) // m.gpus_per_node == (j % m.n_devices) // m.gpus_per_node
        bw = m.intra_Bpns if same_node else m.inter_Bpns
        expect += -(-nbytes // bw)
    got = oracle.simulate_batch(w.ops, w.edges, m, w.cost, cfg[None])[0]
    assert got == expect


@pytest.mark.parametrize("config_id", [0, 1])
def test_pure_sample_split_has_no_transfers(config_id):
    """every op split P ways in the sample dim with the same device offset: every map is
    one-to-one in the sample dim, so part k only meets part k, on the same device."""
    w = W.workload(config_id)
    P = w.max_parts
    cfg = cfgs_all(w.ops, deg=(P, 1, 1, 1), off=1)
    tg = oracle.build_task_graph(w.ops, w.edges, w.machine, w.cost, cfg)
    assert tg.n_tasks == tg.n_compute == P * w.n_ops
    assert tg.simulate()[0] == w.cost[:, P - 1].astype(np.int64).sum()


@pytest.mark.parametrize("config_id", [0, 1, 2, 3, 4])
def test_built_graph_timeline_is_a_fixed_point_with_bounds(config_id):
    w = W.workload(config_id)
    cfg = w.strategies(4)[3]
    tg = oracle.build_task_graph(w.ops, w.edges, w.machine, w.cost, cfg)
    mk, ready, start, end = tg.simulate()
    check_timeline(tg.exe, tg.dev, tg.dep_src.astype(np.int64), tg.dep_dst.astype(np.int64), ready, start, end)
    assert mk == end.max() == end[:tg.n_compute].max()
    assert mk >= np.bincount(tg.dev, weights=tg.exe.astype(np.float64)).max()
    assert mk <= int(tg.exe.sum())
    if config_id <= 3:
        assert mk >= critical_path(tg.exe, tg.dep_src.astype(np.int64), tg.dep_dst.astype(np.int64))
    # every transfer has exactly one predecessor and one successor, both compute tasks
    comm = np.arange(tg.n_compute, tg.n_tasks)
    assert np.array_equal(np.bincount(tg.dep_dst, minlength=tg.n_tasks)[comm], np.ones(len(comm)))
    assert np.array_equal(np.bincount(tg.dep_src, minlength=tg.n_tasks)[comm], np.ones(len(comm)))
    assert (tg.dev[comm] >= w.machine.n_devices).all() and (tg.dev[:tg.n_compute] < w.machine.n_devices).all()


@pytest.mark.parametrize("config_id", [0, 1, 2])
def test_shifting_all_offsets_by_whole_nodes_changes_nothing(config_id):
    w = W.workload(config_id)
    m = w.machine
    cfgs = w.strategies(6).copy()
    base = oracle.simulate_batch(w.ops, w.edges, m, w.cost, cfgs)
    shifted = cfgs.copy()
    shifted["dev_offset"] = (cfgs["dev_offset"] + m.gpus_per_node * (3 if m.n_nodes > 1 else 1)) % m.n_devices
    if m.n_nodes == 1:   # a single node: any rotation keeps co-location and link sharing
        shifted["dev_offset"] = (cfgs["dev_offset"] + 1) % m.n_devices
    assert np.array_equal(base, oracle.simulate_batch(w.ops, w.edges, m, w.cost, shifted))


def test_invalid_strategies_are_flagged():
    w = W.workload(0)
    good = w.strategies(1)[0]
    def run(c):
        return int(oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, c[None])[0])
    assert run(good) != oracle.INVALID
    bad = good.copy(); bad[5]["deg"] = (1, 2, 1, 1)      # softmax: only the sample dim is parallelizable
    assert run(bad) == oracle.INVALID
    bad = good.copy(); bad[4]["deg"] = (1, 1, 2, 1)      # fc output has extent 1 in dim 2
    assert run(bad) == oracle.INVALID
    bad = good.copy(); bad[0]["deg"] = (0, 1, 1, 1)
    assert run(bad) == oracle.INVALID
    bad = good.copy(); bad[0]["deg"] = (8, 8, 2, 1)      # 128 parts > 64
    assert run(bad) == oracle.INVALID
    bad = good.copy(); bad[2]["dev_offset"] = 4          # device 4 of 4
    assert run(bad) == oracle.INVALID


def test_delta_oracle_is_resimulation_and_inverse_restores():
    w = W.workload(1)
    cfg0 = w.strategies(1)[0]
    muts = w.mutations(12)[:, 0]
    out = oracle.simulate_delta_chain(w.ops, w.edges, w.machine, w.cost, cfg0, muts)
    cur = cfg0.copy()
    for s, m in enumerate(muts):
        cur[int(m["op"])] = m["cfg"]
        assert out[s] == oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cur[None])[0]
    # a mutation followed by its inverse gives the starting value back
    inv = np.zeros(2, W.MUT_DT)
    inv[0] = muts[0]
    inv[1]["op"] = muts[0]["op"]
    inv[1]["cfg"] = cfg0[int(muts[0]["op"])]
    back = oracle.simulate_delta_chain(w.ops, w.edges, w.machine, w.cost, cfg0, inv)
    assert back[1] == oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cfg0[None])[0]


def test_edge_lists_not_grouped_by_producer_are_refused():
    """task ids follow (edge, producer part, consumer part) and, with parameter traffic, op by op: the two
    agree only for an edge list that is grouped by producer, so the oracle refuses any other"""
    w = W.workload(2)
    cfg = w.strategies(1)
    bad = w.edges.copy()
    k = int(np.nonzero(np.diff(bad["src_op"]) > 0)[0][0])
    bad[[k, k + 1]] = bad[[k + 1, k]]
    with pytest.raises(ValueError):
        oracle.simulate_batch(w.ops, bad, w.machine, w.cost, cfg)
    with pytest.raises(ValueError):
        oracle.build_task_graph(w.ops, bad, w.machine, w.cost, cfg[0])
    back = bad.copy()
    back[0]["src_op"], back[0]["dst_op"] = back[0]["dst_op"], back[0]["src_op"]     # an edge from a later to an earlier op
    with pytest.raises(ValueError):
        oracle.simulate_batch(w.ops, back, w.machine, w.cost, cfg)


def test_batch_threads_agree():
    w = W.workload(1)
    c = w.strategies(64)
    assert np.array_equal(oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, c, 1),
                          oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, c, 4))
