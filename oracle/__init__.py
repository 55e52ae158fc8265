"""ctypes access to the CPU oracle (oracle/ff_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the bench's
cpu_baseline leg.  The product package never imports this module.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ff_oracle.cpp")
# FF_ORACLE_LIB: tests that plant a mistake in a copy of the source point the pins at the copy's library
_LIB = os.environ.get("FF_ORACLE_LIB") or os.path.join(_HERE, "libff_oracle.so")
INVALID = 2 ** 64 - 1
_lib = None


def build(force: bool = False) -> str:
    """compile the oracle with g++ (plain -O2, no vector tricks)."""
    if os.environ.get("FF_ORACLE_LIB"):
        return _LIB                       # someone else's build
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        compile_oracle(_SRC, _LIB)
    return _LIB


def compile_oracle(src: str, lib_path: str) -> None:
    subprocess.check_call(["g++", "-std=c++17", "-O2", "-fPIC", "-shared", "-pthread", "-Wall", "-o", lib_path, src])


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        vp, u32, u64p, u32p = C.c_void_p, C.c_uint32, C.POINTER(C.c_uint64), C.POINTER(C.c_uint32)
        L.ffo_build.restype = vp
        L.ffo_build.argtypes = [u32, vp, u32, vp, vp, vp, u32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.ffo_graph_ok.restype = C.c_int
        L.ffo_graph_ok.argtypes = [u32, u32, vp]
        L.ffo_from_arrays.restype = vp
        L.ffo_from_arrays.argtypes = [u32, vp, vp, u32, u32, vp, vp]
        L.ffo_counts.restype = None
        L.ffo_counts.argtypes = [vp, u32p, u32p, u32p, u32p]
        L.ffo_export.restype = None
        L.ffo_export.argtypes = [vp, vp, vp, vp, vp]
        L.ffo_simulate.restype = C.c_uint64
        L.ffo_simulate.argtypes = [vp, vp, vp, vp]
        L.ffo_free.restype = None
        L.ffo_free.argtypes = [vp]
        L.ffo_batch.restype = None
        L.ffo_batch.argtypes = [u32, vp, u32, vp, vp, vp, u32, vp, vp, vp, vp, u32, vp, u32, vp, vp, vp, vp, vp, vp, vp, vp]
        _lib = L
    return _lib


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p)


def _check_graph(ops, edges):
    """the oracle's readings of task ids need the tensor edges listed producer by producer"""
    if not lib().ffo_graph_ok(len(ops), len(edges), _ptr(edges)):
        raise ValueError("oracle: edges must go from a lower to a higher op index and be listed producer by producer")


def _cost_args(cost):
    """cost: [n_ops][n_cols] uint32 (exeTime by number of parts), or a triple
    (tuple_ptr [n_ops+1], tuples, ns): exeTime keyed by the packed degree tuple.
    Returns (keep-alive arrays, the five C arguments)."""
    if isinstance(cost, (tuple, list)):
        ptr, tup, ns = (np.ascontiguousarray(a, "<u4") for a in cost)
        return (ptr, tup, ns), (None, 0, _ptr(ptr), _ptr(tup), _ptr(ns))
    cost = np.ascontiguousarray(cost, "<u4")
    return (cost,), (_ptr(cost), cost.shape[1], None, None, None)


def _machine(m):
    return np.array(m.as_tuple() if hasattr(m, "as_tuple") else tuple(m), dtype="<u4")


def _link_args(m):
    """optional per-pair links inside a node: attributes link_Bpns / link_lat_ns of the machine,
    [gpus_per_node][gpus_per_node] (from local GPU, to local GPU); latency defaults to the
    machine's intra-node latency.  Returns (keep-alive arrays, the two C arguments)."""
    bw = getattr(m, "link_Bpns", None)
    if bw is None:
        return (), (None, None)
    G = int(m.gpus_per_node)
    bw = np.ascontiguousarray(bw, "<u4")
    lat = getattr(m, "link_lat_ns", None)
    lat = np.full((G, G), m.intra_lat_ns, "<u4") if lat is None else np.ascontiguousarray(lat, "<u4")
    assert bw.shape == (G, G) and lat.shape == (G, G)
    return (bw, lat), (_ptr(bw), _ptr(lat))


def _node_link_args(m):
    """optional per-pair links between nodes: attributes node_Bpns / node_lat_ns of the machine,
    [n_nodes][n_nodes] (from node, to node); latency defaults to the machine's inter-node latency.
    Returns (keep-alive arrays, the two C arguments)."""
    bw = getattr(m, "node_Bpns", None)
    if bw is None:
        return (), (None, None)
    N = int(m.n_nodes)
    bw = np.ascontiguousarray(bw, "<u4")
    lat = getattr(m, "node_lat_ns", None)
    lat = np.full((N, N), m.inter_lat_ns, "<u4") if lat is None else np.ascontiguousarray(lat, "<u4")
    assert bw.shape == (N, N) and lat.shape == (N, N)
    return (bw, lat), (_ptr(bw), _ptr(lat))


def _param_args(params, n_ops):
    """params: None, or (param_bytes [n_ops] uint32, param_dims [n_ops] uint8): bytes of parameters
    of every op (0 = none) and the output dims that index them (bit d).  Returns (keep-alive
    arrays, the two C arguments)."""
    if params is None:
        return (), (None, None)
    pb = np.ascontiguousarray(params[0], "<u4")
    pd = np.ascontiguousarray(params[1], np.uint8)
    assert pb.shape == (n_ops,) and pd.shape == (n_ops,)
    return (pb, pd), (_ptr(pb), _ptr(pd))


class TaskGraph:
    """a built task graph: exe[t], dev[t], deps (src, dst); the first n_compute tasks are
    compute tasks in (op, part) order, the rest communication tasks in creation order."""

    def __init__(self, handle):
        self._h = handle
        nt, nc, nd, nr = C.c_uint32(), C.c_uint32(), C.c_uint32(), C.c_uint32()
        lib().ffo_counts(handle, C.byref(nt), C.byref(nc), C.byref(nd), C.byref(nr))
        self.n_tasks, self.n_compute, self.n_deps, self.n_rows = nt.value, nc.value, nd.value, nr.value
        self.exe = np.zeros(self.n_tasks, "<u8")
        self.dev = np.zeros(self.n_tasks, "<u4")
        self.dep_src = np.zeros(self.n_deps, "<u4")
        self.dep_dst = np.zeros(self.n_deps, "<u4")
        lib().ffo_export(handle, _ptr(self.exe), _ptr(self.dev), _ptr(self.dep_src), _ptr(self.dep_dst))

    def simulate(self):
        """Algorithm 1 -> (makespan, ready[], start[], end[])."""
        r = np.zeros(self.n_tasks, "<u8")
        s = np.zeros(self.n_tasks, "<u8")
        e = np.zeros(self.n_tasks, "<u8")
        mk = lib().ffo_simulate(self._h, _ptr(r), _ptr(s), _ptr(e))
        return int(mk), r, s, e

    def __del__(self):
        if getattr(self, "_h", None):
            lib().ffo_free(self._h)
            self._h = None


def _tie_args(ties, n_ops):
    """ties: None, or leader [n_ops] uint32: op i takes the configuration of op leader[i]."""
    if ties is None:
        return (), (None,)
    t = np.ascontiguousarray(ties, "<u4")
    assert t.shape == (n_ops,)
    return (t,), (_ptr(t),)


def build_task_graph(ops, edges, machine, cost, cfg, devmap=None, params=None, ties=None):
    """Section 5.1 for one strategy (cfg: [n_ops] configs). None if the strategy is invalid.
    devmap [n_ops][64] uint16: the device of every part given explicitly (the configs' offset
    and stride are then not used)."""
    ops, edges, cfg = map(np.ascontiguousarray, (ops, edges, cfg))
    _check_graph(ops, edges)
    m = _machine(machine)
    keep, cargs = _cost_args(cost)
    keep_l, largs = _link_args(machine)
    if devmap is not None:
        devmap = np.ascontiguousarray(devmap, "<u2")
        assert devmap.shape == (len(ops), 64)
    keep_p, pargs = _param_args(params, len(ops))
    keep_n, nargs = _node_link_args(machine)
    keep_t, targs = _tie_args(ties, len(ops))
    h = lib().ffo_build(len(ops), _ptr(ops), len(edges), _ptr(edges), _ptr(m), *cargs, _ptr(cfg), *largs,
                        None if devmap is None else _ptr(devmap), *pargs, *nargs, *targs)
    return TaskGraph(h) if h else None


def build_and_discard(ops, edges, machine, cost, cfg):
    """Section 5.1 for one strategy, the task graph dropped at once (for timing the construction
    alone).  False if the strategy is invalid."""
    ops, edges, cfg = map(np.ascontiguousarray, (ops, edges, cfg))
    m = _machine(machine)
    keep, cargs = _cost_args(cost)
    keep_l, largs = _link_args(machine)
    keep_n, nargs = _node_link_args(machine)
    h = lib().ffo_build(len(ops), _ptr(ops), len(edges), _ptr(edges), _ptr(m), *cargs, _ptr(cfg), *largs, None, None, None, *nargs, None)
    if h:
        lib().ffo_free(h)
    return bool(h)


def task_graph_from_arrays(exe, dev, n_rows, dep_src, dep_dst):
    exe = np.ascontiguousarray(exe, "<u8")
    dev = np.ascontiguousarray(dev, "<u4")
    ds = np.ascontiguousarray(dep_src, "<u4")
    dd = np.ascontiguousarray(dep_dst, "<u4")
    return TaskGraph(lib().ffo_from_arrays(len(exe), _ptr(exe), _ptr(dev), n_rows, len(ds), _ptr(ds), _ptr(dd)))


def simulate_batch(ops, edges, machine, cost, cfgs, n_threads=1, devmaps=None, params=None, ties=None):
    """makespan (ns) of every strategy in cfgs [B][n_ops]; 2^64-1 for an invalid one.
    devmaps [B][n_ops][64] uint16: explicit devices of all parts (see build_task_graph)."""
    ops, edges, cfgs = map(np.ascontiguousarray, (ops, edges, cfgs))
    assert cfgs.ndim == 2 and cfgs.shape[1] == len(ops)
    _check_graph(ops, edges)
    m = _machine(machine)
    out = np.zeros(cfgs.shape[0], "<u8")
    keep, cargs = _cost_args(cost)
    keep_l, largs = _link_args(machine)
    if devmaps is not None:
        devmaps = np.ascontiguousarray(devmaps, "<u2")
        assert devmaps.shape == (cfgs.shape[0], len(ops), 64)
    keep_p, pargs = _param_args(params, len(ops))
    keep_n, nargs = _node_link_args(machine)
    keep_t, targs = _tie_args(ties, len(ops))
    lib().ffo_batch(len(ops), _ptr(ops), len(edges), _ptr(edges), _ptr(m), *cargs,
                    _ptr(cfgs), cfgs.shape[0], _ptr(out), n_threads, *largs,
                    None if devmaps is None else _ptr(devmaps), *pargs, *nargs, *targs)
    return out


def simulate_delta_chain(ops, edges, machine, cost, cfg0, mutations, steps=None, params=None, ties=None):
    """oracle for delta simulation: apply the single-op mutations cumulatively and fully
    re-simulate (the definition of the delta result, Section 5.3).  mutations: [n_steps]
    records (op, cfg).  `steps` selects which steps (0-based) to evaluate; returns their
    makespans in order."""
    cur = np.array(cfg0, copy=True)
    want = set(range(len(mutations))) if steps is None else set(int(s) for s in steps)
    last = max(want) if want else -1
    snaps = []
    for s in range(last + 1):
        cur[int(mutations[s]["op"])] = mutations[s]["cfg"]
        if s in want:
            snaps.append(cur.copy())
    if not snaps:
        return np.zeros(0, "<u8")
    return simulate_batch(ops, edges, machine, cost, np.stack(snaps), params=params, ties=ties)
