"""Pins of the oracle's parameter-synchronisation tasks (the reading is stated in the oracle,
at `Extras`): replicas of a parameter shard send their gradient to the shard's owner when their
task has finished; Section 8 discusses this traffic, Section 5.1 has no construction for it."""
import numpy as np

import oracle
from paper_1807_05358_amd import workloads as W


def _one_op(extent=(8, 8, 1, 1)):
    ops = np.zeros(1, W.OP_DT)
    ops[0]["ndim"], ops[0]["par_mask"] = 2, 3
    ops[0]["extent"] = extent
    return ops, np.zeros(0, W.EDGE_DT)


def _cfg(n_ops, degs, offs, stride=1):
    cfg = np.zeros((1, n_ops), W.CFG_DT)
    cfg["deg"] = 1
    for i, d in enumerate(degs):
        cfg["deg"][0, i, :len(d)] = d
    cfg["dev_offset"][0] = offs
    cfg["dev_stride"] = stride
    return cfg


COST = np.tile(np.array([1000, 600, 0, 400] + [0] * 60, np.uint32), (2, 1))
CHANNEL = np.array([2], np.uint8)          # parameters indexed by output dim 1


def test_replicas_send_their_gradient_to_the_owner():
    ops, edges = _one_op()
    P = np.array([1001], np.uint32)
    # four replicas of the one shard on the four GPUs of a node: three transfers on private links
    mach = W.Machine(1, 4, intra_Bpns=7, inter_Bpns=3, intra_lat_ns=11, inter_lat_ns=5)
    got = oracle.simulate_batch(ops, edges, mach, COST[:1], _cfg(1, [(4, 1)], [0]), params=(P, CHANNEL))
    assert int(got[0]) == 400 + (1001 + 6) // 7 + 11
    tg = oracle.build_task_graph(ops, edges, mach, COST[:1], _cfg(1, [(4, 1)], [0])[0], params=(P, CHANNEL))
    assert tg.n_compute == 4 and tg.n_tasks == 7
    assert list(tg.dev[4:]) == [4 + 1 * 4 + 0, 4 + 2 * 4 + 0, 4 + 3 * 4 + 0]        # rows of dev k -> dev 0
    assert list(tg.dep_src) == [1, 2, 3] and list(tg.dep_dst) == [4, 5, 6]           # one predecessor, no successor
    # two nodes of two GPUs: the replicas on node 1 share the link between the nodes
    mach = W.Machine(2, 2, intra_Bpns=7, inter_Bpns=3, intra_lat_ns=11, inter_lat_ns=5)
    t_in, t_out = (1001 + 6) // 7 + 11, (1001 + 2) // 3 + 5
    got = oracle.simulate_batch(ops, edges, mach, COST[:1], _cfg(1, [(4, 1)], [0]), params=(P, CHANNEL))
    assert int(got[0]) == 400 + max(t_in, 2 * t_out)
    # the owner is the replica with index 0, wherever it sits: offset 3 puts it on node 1
    got = oracle.simulate_batch(ops, edges, mach, COST[:1], _cfg(1, [(4, 1)], [3]), params=(P, CHANNEL))
    assert int(got[0]) == 400 + max(t_in, 2 * t_out)       # devices 3,0,1,2: 0 and 1 cross nodes, 2 is local
    # replicas on the owner's device send nothing
    got = oracle.simulate_batch(ops, edges, mach, COST[:1], _cfg(1, [(4, 1)], [0], stride=0), params=(P, CHANNEL))
    assert int(got[0]) == 4 * 400


def test_shards_have_no_replicas_to_synchronise():
    ops, edges = _one_op()
    P = np.array([1001], np.uint32)
    mach = W.Machine(1, 4, intra_Bpns=7)
    got = oracle.simulate_batch(ops, edges, mach, COST[:1], _cfg(1, [(1, 4)], [0]), params=(P, CHANNEL))
    assert int(got[0]) == 400
    # two shards with two replicas each: part (s, c) sends to part (0, c); a shard is ceil(P / 2) bytes
    tg = oracle.build_task_graph(ops, edges, mach, COST[:1], _cfg(1, [(2, 2)], [0])[0], params=(P, CHANNEL))
    assert tg.n_tasks == 6
    assert list(tg.dep_src) == [2, 3] and list(tg.dev[4:]) == [4 + 2 * 4 + 0, 4 + 3 * 4 + 1]
    assert list(tg.exe[4:]) == [(501 + 6) // 7] * 2
    tg = oracle.build_task_graph(ops, edges, W.Machine(1, 4, intra_Bpns=1), COST[:1], _cfg(1, [(2, 2)], [0])[0], params=(P, CHANNEL))
    assert list(tg.exe[4:]) == [501, 501]           # half of 1001 bytes, rounded up
    # parameters indexed by both dims: every part is a shard of its own
    got = oracle.simulate_batch(ops, edges, mach, COST[:1], _cfg(1, [(2, 2)], [0]), params=(P, np.array([3], np.uint8)))
    assert int(got[0]) == 400
    # no dims index the parameters: every part is a replica of the whole
    tg = oracle.build_task_graph(ops, edges, mach, COST[:1], _cfg(1, [(2, 2)], [0])[0], params=(P, np.array([0], np.uint8)))
    assert tg.n_tasks == 7 and list(tg.exe[4:]) == [(1001 + 6) // 7] * 3


def test_no_parameters_is_the_plain_graph():
    w = W.workload(1)
    cfgs = w.strategies(32)
    zero = (np.zeros(w.n_ops, np.uint32), np.full(w.n_ops, 2, np.uint8))
    assert np.array_equal(oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cfgs, params=zero),
                          oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cfgs))


def test_gradient_volume_and_task_shape_on_a_real_graph():
    """1 B/ns links without latency: the transfer times add up to the bytes sent, (replicas - 1) x
    shards x ceil(P / shards) per op when all parts sit on different devices"""
    w = W.workload(1)
    params = w.param_table()
    assert params[0].sum() > 200_000_000 and (params[0] > 0).sum() == 8          # AlexNet: 5 conv + 3 fc
    mach = W.Machine(4, 4, intra_Bpns=1, inter_Bpns=1)
    cfgs = w.strategies(24)
    for cfg in cfgs:
        plain = oracle.build_task_graph(w.ops, w.edges, mach, w.cost, cfg)
        tg = oracle.build_task_graph(w.ops, w.edges, mach, w.cost, cfg, params=params)
        deg = cfg["deg"].astype(np.int64)
        parts = deg.prod(axis=1)
        shards = np.array([np.prod([deg[i, d] for d in range(4) if (params[1][i] >> d) & 1]) for i in range(w.n_ops)])
        want = sum((int(parts[i]) - int(shards[i])) * (-(-int(params[0][i]) // int(shards[i]))) for i in range(w.n_ops) if params[0][i])
        n_sync = tg.n_tasks - plain.n_tasks
        assert n_sync == sum(int(parts[i] - shards[i]) for i in range(w.n_ops) if params[0][i])
        # sync tasks: the tasks that have no successor and are not compute tasks
        has_succ = np.zeros(tg.n_tasks, bool)
        has_succ[tg.dep_src] = True
        sync = np.nonzero(~has_succ & (np.arange(tg.n_tasks) >= tg.n_compute))[0]
        assert len(sync) == n_sync and int(tg.exe[sync].sum()) == want
        n_pred = np.bincount(tg.dep_dst, minlength=tg.n_tasks)
        assert (n_pred[sync] == 1).all()
        mk, r, s_, e = tg.simulate()
        assert mk == int(e.max()) >= plain.simulate()[0]


def test_an_ops_gradients_queue_behind_its_activations_on_a_shared_link():
    """two parts of op 0 on GPUs 0 and 1; op 1 unsplit on GPU 0.  Part 1 sends its activations and its
    gradient over the same link at the same time: the activation transfer has the lower id and goes first"""
    ops = np.zeros(2, W.OP_DT)
    for o in ops:
        o["ndim"], o["par_mask"] = 2, 3
        o["extent"] = (8, 8, 1, 1)
    edges = np.zeros(1, W.EDGE_DT)
    edges[0]["src_op"], edges[0]["dst_op"] = 0, 1
    for d in range(4):
        edges[0]["map"][d]["src_dim"] = d if d < 2 else -1
        edges[0]["map"][d]["stride"] = 1
    mach = W.Machine(1, 2, intra_Bpns=1, elem_bytes=1)
    params = (np.array([5000, 0], np.uint32), np.array([2, 2], np.uint8))
    cfg = _cfg(2, [(2, 1), (1, 1)], [0, 0])
    t_act = 4 * 8                        # half of the 8 x 8 tensor, one byte per element
    got = int(oracle.simulate_batch(ops, edges, mach, COST, cfg, params=params)[0])
    assert got == max(600 + t_act + 1000, 600 + t_act + 5000)
    tg = oracle.build_task_graph(ops, edges, mach, COST, cfg[0], params=params)
    mk, ready, start, end = tg.simulate()
    assert tg.n_tasks == 5 and list(tg.dev[3:]) == [2 + 1 * 2 + 0] * 2
    assert (int(start[3]), int(end[3]), int(start[4]), int(end[4])) == (600, 600 + t_act, 600 + t_act, 600 + t_act + 5000)
    # the consumer's own gradient traffic comes after every task op 0 created
    params2 = (np.array([5000, 7000], np.uint32), np.array([2, 2], np.uint8))
    cfg2 = _cfg(2, [(2, 1), (2, 1)], [0, 0])
    tg = oracle.build_task_graph(ops, edges, mach, COST, cfg2[0], params=params2)
    kinds = [int(tg.exe[t]) for t in range(tg.n_compute, tg.n_tasks)]
    assert kinds == [5000, 7000]         # (aligned parts: no activation transfers) op 0's gradient, then op 1's


def test_renaming_devices_keeps_times_with_parameter_traffic():
    w = W.workload(1)
    params = w.param_table()
    N, G = w.machine.n_nodes, w.machine.gpus_per_node
    cfgs = w.strategies(16)
    maps = W.device_maps(cfgs, N * G, 21)
    want = oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cfgs, devmaps=maps, params=params)
    assert not np.array_equal(want, oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cfgs, devmaps=maps))
    rng = np.random.default_rng(2)
    s, t = rng.permutation(N), rng.permutation(G)
    table = np.array([s[d // G] * G + t[d % G] for d in range(N * G)] + [0] * (65536 - N * G), np.uint16)
    table[0xFFFF] = 0xFFFF
    assert np.array_equal(oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cfgs, devmaps=table[maps], params=params), want)
