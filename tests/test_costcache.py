"""Section 5.1: a task's exeTime is measured once and kept per (operation type, output size).  The cache in front
of the measurement, and the cost lists built through it (host side, no GPU)."""
import numpy as np

import oracle
from paper_1807_05358_amd import costcache, workloads as W


def test_one_measurement_per_type_and_shape():
    calls = []

    def measure(op_type, shape):
        calls.append((op_type, shape))
        return 1000 + 7 * op_type + sum(shape)

    cache = costcache.ExeTimeCache(measure)
    assert cache.exe_time(W.T_CONV, (4, 8)) == cache.exe_time(W.T_CONV, (4, 8)) == 1000 + 12
    assert cache.exe_time(W.T_POOL, (4, 8)) == 1000 + 7 + 12               # same shape, other type: its own entry
    assert cache.exe_time(W.T_CONV, (8, 4)) == 1000 + 12                    # other shape: its own entry
    assert calls == [(W.T_CONV, (4, 8)), (W.T_POOL, (4, 8)), (W.T_CONV, (8, 4))]
    assert (cache.hits, cache.misses) == (1, 3)


def test_task_shape_is_the_largest_part():
    op = np.zeros((), W.OP_DT)
    op["ndim"], op["extent"] = 3, (7, 35, 4, 1)
    assert costcache.task_shape(op, (3, 4, 1, 1)) == (3, 9, 4)               # parts of 2,2,3 and 8,9,9,9 elements
    assert costcache.task_shape(op, (1, 1, 4, 1)) == (7, 35, 1)


def test_lists_of_the_inception_graph_reuse_measurements():
    """the Inception-shaped graph repeats its blocks: far fewer measurements than list entries, ops of equal type
    and shape get equal lists, and the oracle takes the lists as they are"""
    w = W.workload(2)
    cache = costcache.ExeTimeCache(costcache.model_measure)
    ptr, tuples, ns = costcache.tuple_costs(w.ops, w.max_parts, w.choices, cache)
    assert ptr[0] == 0 and ptr[-1] == len(tuples) == len(ns) == cache.hits + cache.misses
    assert cache.misses == len(cache.kept) < len(tuples) // 2
    for i in range(len(w.ops)):
        t = tuples[ptr[i]:ptr[i + 1]]
        assert np.all(np.diff(t.astype(np.int64)) > 0)                          # ascending, no duplicates
    key = lambda o: (int(o["type"]), int(o["ndim"]), int(o["par_mask"]), tuple(int(x) for x in o["extent"]))
    seen = {}
    for i, o in enumerate(w.ops):
        j = seen.setdefault(key(o), i)
        if j != i:
            assert np.array_equal(ns[ptr[i]:ptr[i + 1]], ns[ptr[j]:ptr[j + 1]])
    assert len(seen) < len(w.ops)
    # more parts never make the largest task larger: the unsplit entry is the slowest of an op's list
    for i in range(len(w.ops)):
        t, v = tuples[ptr[i]:ptr[i + 1]], ns[ptr[i]:ptr[i + 1]]
        assert v[t == 0x01010101][0] == v.max()
    cfgs = w.strategies(4)
    got = oracle.simulate_batch(w.ops, w.edges, w.machine, (ptr, tuples, ns), cfgs)
    assert (got != oracle.INVALID).all() and len(set(got.tolist())) > 1
