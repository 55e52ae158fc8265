"""Pins of the oracle's second cost model: exeTime keyed by the whole degree tuple (the time of
a task depends on which dims are split, Section 5.1 / 8.1)."""
import numpy as np

import oracle
from paper_1807_05358_amd import workloads as W


def _pack(t):
    t = np.asarray(t, np.uint32)
    return t[..., 0] | (t[..., 1] << 8) | (t[..., 2] << 16) | (t[..., 3] << 24)


def test_tuple_costs_without_surcharge_reduce_to_the_table_by_parts():
    """a tuple list that repeats the parts table must give the timelines of the (pinned) parts model"""
    for c in (0, 1):
        w = W.workload(c)
        ptr = np.zeros(w.n_ops + 1, np.uint32)
        tups, ns = [], []
        for i, o in enumerate(w.ops):
            t = W.valid_degree_tuples(o, w.max_parts, w.choices).astype(np.uint32)
            p = _pack(t)
            order = np.argsort(p)
            parts = t.prod(axis=1)
            tups.append(p[order])
            ns.append(w.cost[i, parts[order] - 1])
            ptr[i + 1] = ptr[i] + len(t)
        tc = (ptr, np.concatenate(tups), np.concatenate(ns))
        cfgs = w.strategies(48)
        assert np.array_equal(oracle.simulate_batch(w.ops, w.edges, w.machine, tc, cfgs),
                              oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cfgs))


def test_same_number_of_parts_different_tuples_different_times():
    ops = np.zeros(1, W.OP_DT)
    ops[0]["ndim"], ops[0]["par_mask"] = 2, 3
    ops[0]["extent"] = (4, 4, 1, 1)
    edges = np.zeros(0, W.EDGE_DT)
    mach = W.Machine(1, 2)
    tc = (np.array([0, 3], np.uint32), np.array([0x01010101, 0x01010102, 0x01010201], np.uint32),
          np.array([1000, 500, 900], np.uint32))
    cfg = np.zeros((4, 1), W.CFG_DT)
    cfg["deg"] = 1
    cfg["dev_stride"] = 1
    cfg["deg"][1, 0] = (2, 1, 1, 1)        # two parts by dim 0, one per device: 500
    cfg["deg"][2, 0] = (1, 2, 1, 1)        # two parts by dim 1: 900
    cfg["deg"][3, 0] = (2, 2, 1, 1)        # not in the list: no cost, invalid
    got = oracle.simulate_batch(ops, edges, mach, tc, cfg)
    assert list(got[:3]) == [1000, 500, 900] and got[3] == oracle.INVALID
    cfg["dev_stride"] = 0                  # both parts on one device: twice the time
    assert list(oracle.simulate_batch(ops, edges, mach, tc, cfg)[:3]) == [1000, 1000, 1800]


def test_unsplit_single_device_is_the_sum_of_the_unsplit_tuples():
    w = W.workload(2)
    ptr, tup, ns = w.tuple_costs()
    cfg = np.zeros((1, w.n_ops), W.CFG_DT)
    cfg["deg"] = 1
    cfg["dev_stride"] = 1
    want = 0
    for i in range(w.n_ops):
        seg = tup[ptr[i]:ptr[i + 1]]
        assert np.all(np.diff(seg.astype(np.int64)) > 0)          # ascending, as the boundary requires
        k = int(np.nonzero(seg == 0x01010101)[0][0])
        want += int(ns[ptr[i] + k])
        assert int(ns[ptr[i] + k]) == int(w.cost[i, 0])            # no split dim, no surcharge
    assert int(oracle.simulate_batch(w.ops, w.edges, w.machine, (ptr, tup, ns), cfg)[0]) == want


def test_generated_tuple_costs_only_add_to_the_parts_table():
    w = W.workload(1)
    ptr, tup, ns = w.tuple_costs()
    for i in range(w.n_ops):
        for k in range(ptr[i], ptr[i + 1]):
            d = [(int(tup[k]) >> (8 * j)) & 0xFF for j in range(4)]
            parts = d[0] * d[1] * d[2] * d[3]
            base = int(w.cost[i, parts - 1])
            assert base <= int(ns[k]) <= base + 3 * (base * 25 // 100)
            if d[1] == d[2] == d[3] == 1:
                assert int(ns[k]) == base
