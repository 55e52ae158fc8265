"""Test-side helpers: golden-fixture loading and checks that do not re-run the algorithm."""
import json
import os

import numpy as np

from paper_1807_05358_amd import workloads as W


def load_golden(golden_dir, name):
    with open(os.path.join(golden_dir, name)) as f:
        return json.load(f)


def graph_from_golden(g):
    """(ops, edges, machine, cost, cfg) arrays from a 'build_*' fixture."""
    ops = np.zeros(len(g["ops"]), W.OP_DT)
    for i, o in enumerate(g["ops"]):
        ext = list(o["extent"])
        ops[i]["ndim"] = len(ext)
        ops[i]["extent"] = ext + [1] * (4 - len(ext))
        ops[i]["par_mask"] = sum(1 << d for d in o["par"])
    edges = np.zeros(len(g["edges"]), W.EDGE_DT)
    for k, e in enumerate(g["edges"]):
        edges[k]["src_op"], edges[k]["dst_op"] = e["src"], e["dst"]
        kind = 1 if e.get("contributes") else 0      # a gradient edge: the producer contributes to the consumer's tensor
        for d in range(4):
            if d < len(e["map"]):
                c, st, a, b = e["map"][d]
                edges[k]["map"][d] = (c, kind, st, a, b)
            else:
                edges[k]["map"][d] = (-1, kind, 1, 0, 0)
    cost = np.full((len(ops), W.MAX_PARTS), 1, "<u4")
    for i, row in g["cost"].items():
        for p, v in row.items():
            cost[int(i), int(p) - 1] = v
    cfg = np.zeros(len(ops), W.CFG_DT)
    for i, s in enumerate(g["strategy"]):
        cfg[i]["deg"] = list(s["deg"]) + [1] * (4 - len(s["deg"]))
        cfg[i]["dev_offset"], cfg[i]["dev_stride"] = s["off"], s["stride"]
    return ops, edges, W.Machine(*g["machine"]), cost, cfg


def check_timeline(exe, dev, dep_src, dep_dst, ready, start, end):
    """Fixed-point check of a timeline against what Algorithm 1 and assumptions A3/A4
    require, without running the algorithm: readyTime = max end of predecessors; on each
    device, in (readyTime, id) order, start = max(readyTime, end of the previous task);
    end = start + exeTime."""
    n = len(exe)
    want_ready = np.zeros(n, np.uint64)
    np.maximum.at(want_ready, dep_dst, end[dep_src])
    assert np.array_equal(want_ready, ready), "readyTime != max end of predecessors"
    assert np.array_equal(end, start + exe), "end != start + exeTime"
    order = np.lexsort((np.arange(n), ready, dev))   # by device, then readyTime, then id
    d, r, s, e = dev[order], ready[order], start[order], end[order]
    prev_end = np.concatenate(([0], e[:-1]))
    first = np.concatenate(([True], d[1:] != d[:-1]))
    prev_end[first] = 0
    assert np.array_equal(s, np.maximum(r, prev_end)), "device order is not FIFO by (readyTime, id)"


def critical_path(exe, dep_src, dep_dst):
    """longest exeTime path (deps go from lower to higher topological position is NOT
    assumed: uses Kahn order)."""
    n = len(exe)
    indeg = np.zeros(n, np.int64)
    np.add.at(indeg, dep_dst, 1)
    order = np.argsort(dep_src, kind="stable")
    src_sorted, dst_sorted = dep_src[order], dep_dst[order]
    ptr = np.searchsorted(src_sorted, np.arange(n + 1))
    dist = exe.astype(np.int64).copy()
    stack = [t for t in range(n) if indeg[t] == 0]
    while stack:
        t = stack.pop()
        for s in dst_sorted[ptr[t]:ptr[t + 1]]:
            dist[s] = max(dist[s], dist[t] + int(exe[s]))
            indeg[s] -= 1
            if indeg[s] == 0:
                stack.append(s)
    return int(dist.max())


def random_graph(rng, n_ops):
    """random DAG with random shapes and random affine input maps (not a DNN: it only has to
    be a valid input of the boundary)."""
    g = W.GraphBuilder()
    for i in range(n_ops):
        ndim = int(rng.integers(1, 5))
        ext = [int(rng.choice([1, 2, 3, 5, 8, 12, 17, 32, 64, 100])) for _ in range(ndim)]
        par = [d for d in range(ndim) if rng.random() < 0.8] or [0]
        g.op(W.T_ELEM, ext, par, 1)
        n_in = 0 if i == 0 else int(rng.integers(0, min(i, 3) + 1))
        for src in sorted(rng.choice(i, size=n_in, replace=False).tolist()) if n_in else []:
            sext = g.extent(src)
            maps = []
            for d in range(len(sext)):
                if rng.random() < 0.3:
                    maps.append(W.ALL)
                else:
                    c = int(rng.integers(0, ndim))
                    stride = int(rng.choice([1, 1, 1, 2, 3]))
                    a = int(rng.integers(-3, 4))
                    b = a + int(rng.integers(0, 4))
                    maps.append((c, stride, a, b))
            g.edge(src, i, maps)
    return g.finish()
