"""Where the cost lists of ff_sim_create_tuplecost come from in the paper's set-up (Section 5.1, task properties):
the exeTime of a compute task is measured once and kept, and every later task of the same operation type and output
size takes the kept value.  This module is that bookkeeping on the host: a cache keyed by (operation type, shape of
one task's output) in front of any function that can time a task, and the per-op lists of (degree tuple, exeTime)
built through it.  Nothing here runs on the GPU or decides anything about a simulation; on the synthetic workloads the
"measurement" is a model (model_measure).

Reading taken where Section 4's equal-size partitions do not divide evenly: the parts of an op then differ by at most
one element per dim, and one time is kept per configuration -- that of the largest part, ceil(extent / degree) per dim.
"""
from __future__ import annotations

import numpy as np

from . import workloads as W


class ExeTimeCache:
    """measure(op_type, shape) -> exeTime in ns (an integer >= 1) is called once per distinct (type, shape)."""

    def __init__(self, measure):
        self.measure = measure
        self.kept = {}
        self.hits = 0
        self.misses = 0

    def exe_time(self, op_type, shape):
        key = (int(op_type), tuple(int(x) for x in shape))
        t = self.kept.get(key)
        if t is None:
            self.misses += 1
            t = int(self.measure(*key))
            if not 1 <= t < 2 ** 32:
                raise ValueError(f"measured time {t} ns of {key} does not fit the cost lists (1 .. 2^32-1)")
            self.kept[key] = t
        else:
            self.hits += 1
        return t


def task_shape(op, degrees):
    """output shape of the largest task of `op` under the degree tuple: ceil(extent / degree) per dim"""
    return tuple(-(-int(op["extent"][d]) // int(degrees[d])) for d in range(int(op["ndim"])))


def tuple_costs(ops, max_parts, choices, cache: ExeTimeCache):
    """(tuple_ptr [n_ops+1], tuples ascending per op, ns): for every op the valid degree tuples (workloads.
    valid_degree_tuples) with the exeTime of one of its tasks, every (type, shape) timed once through `cache`."""
    ptr = np.zeros(len(ops) + 1, np.uint32)
    tup_all, ns_all = [], []
    for i, o in enumerate(ops):
        t = W.valid_degree_tuples(o, max_parts, choices).astype(np.uint64)
        packed = t[:, 0] | (t[:, 1] << np.uint64(8)) | (t[:, 2] << np.uint64(16)) | (t[:, 3] << np.uint64(24))
        ns = np.array([cache.exe_time(o["type"], task_shape(o, row)) for row in t], dtype=np.uint64)
        order = np.argsort(packed, kind="stable")
        tup_all.append(packed[order].astype(np.uint32))
        ns_all.append(ns[order].astype(np.uint32))
        ptr[i + 1] = ptr[i] + len(t)
    return ptr, np.concatenate(tup_all), np.concatenate(ns_all)


# work per output element by operation type, in units of 0.1 ns (a stand-in for running the task on a device)
_WORK = {W.T_CONV: 900, W.T_POOL: 9, W.T_FC: 2000, W.T_SOFTMAX: 30, W.T_ELEM: 2, W.T_CONCAT: 2, W.T_EMBED: 4,
         W.T_ATTN: 400, W.T_SLICE: 2, W.T_STACK: 2}


def model_measure(op_type, shape):
    """a synthetic measurement: a launch overhead plus work proportional to the task's output elements"""
    elems = 1
    for x in shape:
        elems *= int(x)
    return min(2 ** 32 - 1, 5000 + (elems * _WORK.get(int(op_type), 2) + 9) // 10)
