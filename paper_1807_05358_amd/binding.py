"""Thin ctypes binding of the C boundary in include/ff_sim.h (same names, argument
marshalling only).  torch is used for device memory and streams, nothing else.  There is
no CPU fallback: if libffsim.so is missing the import of the library fails loudly."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import workloads as W

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libffsim.so")

FF_OK, FF_EINVAL, FF_ENOMEM, FF_EWORKSPACE, FF_ERANGE, FF_EHIP = 0, -1, -2, -3, -4, -5
FF_AHEAD_ALWAYS = 0x80000000
FF_INVALID_NS = 2 ** 64 - 1
FF_INTERNAL_NS = 2 ** 64 - 2
FF_OVERFLOW_NS = 2 ** 64 - 3
STATS_DT = np.dtype([("n_compute", "<u8"), ("n_pairs", "<u8"), ("n_comm", "<u8"), ("sum_comm_ns", "<u8"),
                     ("n_events", "<u8"), ("exit_code", "<u8"), ("n_stuck", "<u8"), ("reserved", "<u8")])


class ff_opgraph_t(C.Structure):
    _fields_ = [("n_ops", C.c_uint32), ("n_edges", C.c_uint32), ("ops", C.c_void_p), ("edges", C.c_void_p)]


class ff_machine_t(C.Structure):
    _fields_ = [(n, C.c_uint32) for n in ("n_nodes", "gpus_per_node", "intra_Bpns", "inter_Bpns",
                                          "intra_lat_ns", "inter_lat_ns", "elem_bytes")]


class ff_costtable_t(C.Structure):
    _fields_ = [("n_ops", C.c_uint32), ("n_cols", C.c_uint32), ("ns", C.c_void_p)]


EXPORTS = ["ff_sim_create", "ff_sim_create_tuplecost", "ff_sim_destroy", "ff_sim_set_links", "ff_sim_set_node_links", "ff_sim_set_ties", "ff_sim_set_params",
           "ff_sim_workspace_bytes", "ff_sim_set_workspace", "ff_sim_set_stats",
           "ff_sim_batch", "ff_sim_batch_devmaps", "ff_sim_chains_create", "ff_sim_delta", "ff_sim_chains_destroy", "ff_sim_chains_get_stats",
           "ff_sim_delta_try", "ff_sim_delta_try_workspace_bytes", "ff_sim_search", "ff_sim_search_ahead", "ff_sim_accept_table",
           "ff_sim_batch_kernel_name",
           "ff_sim_neighbour_count", "ff_sim_neighbours", "ff_sim_neighbours_noalloc",
           "ff_sim_strerror"]
CHAIN_STATS_DT = np.dtype([("n_steps", "<u8"), ("n_resumed", "<u8"), ("n_events", "<u8"), ("n_events_full", "<u8"),
                           ("n_converged", "<u8")])



class ff_ahead_stats_t(C.Structure):
    _fields_ = [("rounds", C.c_uint64), ("proposals_simulated", C.c_uint64), ("steps", C.c_uint64), ("accepted", C.c_uint64)]


class ff_linktable_t(C.Structure):
    _fields_ = [("gpus_per_node", C.c_uint32), ("Bpns", C.c_void_p), ("lat_ns", C.c_void_p)]


class ff_tuplecost_t(C.Structure):
    _fields_ = [("n_ops", C.c_uint32), ("tuple_ptr", C.c_void_p), ("tuples", C.c_void_p), ("ns", C.c_void_p)]


class ff_search_t(C.Structure):
    _fields_ = [("seed", C.c_uint64), ("first_step", C.c_uint64), ("bucket_ns", C.c_uint64), ("patience", C.c_uint64),
                ("n_buckets", C.c_uint32), ("n_tuples", C.c_uint32),
                ("d_accept", C.c_void_p), ("d_tuple_ptr", C.c_void_p), ("d_tuples", C.c_void_p),
                ("d_best_ns", C.c_void_p), ("d_best", C.c_void_p)]


_lib = None


def load_library(path):
    """use another build of the library (the diagnostic build with section timers) for everything created from now
    on; handles made with the previous one must have been closed."""
    global _lib, LIB_PATH
    LIB_PATH = path
    _lib = None


def lib():
    """the loaded library; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            # nothing built yet: build once (hipcc); there is no other implementation to fall back to
            try:
                from . import build as _build
                _build.build_library(force=True)
            except Exception as exc:
                raise RuntimeError(f"{LIB_PATH} is missing and could not be built with hipcc "
                                   "(`python -m paper_1807_05358_amd.build`): " + str(exc)) from exc
        L = C.CDLL(LIB_PATH)
        vp, u32 = C.c_void_p, C.c_uint32
        L.ff_sim_create.restype = C.c_int
        L.ff_sim_create.argtypes = [C.POINTER(ff_opgraph_t), C.POINTER(ff_machine_t), C.POINTER(ff_costtable_t),
                                    C.POINTER(vp)]
        L.ff_sim_create_tuplecost.restype = C.c_int
        L.ff_sim_create_tuplecost.argtypes = [C.POINTER(ff_opgraph_t), C.POINTER(ff_machine_t), C.POINTER(ff_tuplecost_t),
                                              C.POINTER(vp)]
        L.ff_sim_destroy.restype = None
        L.ff_sim_destroy.argtypes = [vp]
        L.ff_sim_workspace_bytes.restype = C.c_size_t
        L.ff_sim_workspace_bytes.argtypes = [vp, u32]
        L.ff_sim_set_workspace.restype = C.c_int
        L.ff_sim_set_workspace.argtypes = [vp, vp, C.c_size_t]
        L.ff_sim_set_stats.restype = C.c_int
        L.ff_sim_set_stats.argtypes = [vp, vp]
        L.ff_sim_batch.restype = C.c_int
        L.ff_sim_batch.argtypes = [vp, vp, u32, vp, vp]
        L.ff_sim_batch_devmaps.restype = C.c_int
        L.ff_sim_batch_devmaps.argtypes = [vp, vp, vp, u32, vp, vp]
        L.ff_sim_set_links.restype = C.c_int
        L.ff_sim_set_links.argtypes = [vp, vp]
        L.ff_sim_set_node_links.restype = C.c_int
        L.ff_sim_set_node_links.argtypes = [vp, vp]
        L.ff_sim_set_ties.restype = C.c_int
        L.ff_sim_set_ties.argtypes = [vp, vp]
        L.ff_sim_set_params.restype = C.c_int
        L.ff_sim_set_params.argtypes = [vp, vp, vp]
        L.ff_sim_chains_create.restype = C.c_int
        L.ff_sim_chains_create.argtypes = [vp, vp, u32, vp, vp, C.POINTER(vp)]
        L.ff_sim_delta.restype = C.c_int
        L.ff_sim_delta.argtypes = [vp, vp, u32, vp, vp]
        L.ff_sim_chains_destroy.restype = None
        L.ff_sim_chains_destroy.argtypes = [vp]
        L.ff_sim_delta_try.restype = C.c_int
        L.ff_sim_delta_try.argtypes = [vp, vp, u32, vp, vp]
        L.ff_sim_delta_try_workspace_bytes.restype = C.c_size_t
        L.ff_sim_delta_try_workspace_bytes.argtypes = [vp, u32]
        L.ff_sim_search.restype = C.c_int
        L.ff_sim_search.argtypes = [vp, C.POINTER(ff_search_t), u32, vp, vp]
        L.ff_sim_search_ahead.restype = C.c_int
        L.ff_sim_search_ahead.argtypes = [vp, C.POINTER(ff_search_t), u32, u32, vp, vp, C.POINTER(ff_ahead_stats_t)]
        L.ff_sim_accept_table.restype = C.c_int
        L.ff_sim_accept_table.argtypes = [C.c_double, C.c_uint64, u32, vp]
        L.ff_sim_batch_kernel_name.restype = C.c_int
        L.ff_sim_batch_kernel_name.argtypes = [vp, u32, C.c_char_p, C.c_size_t]
        L.ff_sim_neighbour_count.restype = C.c_int
        L.ff_sim_neighbour_count.argtypes = [vp, vp, u32, u32, u32, C.POINTER(u32)]
        L.ff_sim_neighbours.restype = C.c_int
        L.ff_sim_neighbours.argtypes = [vp, vp, vp, u32, u32, u32, vp, vp, vp, vp, vp]
        L.ff_sim_neighbours_noalloc.restype = C.c_int
        L.ff_sim_neighbours_noalloc.argtypes = [vp, vp, vp, u32, u32, u32, u32, vp, vp, vp, vp, vp]
        L.ff_sim_chains_get_stats.restype = C.c_int
        L.ff_sim_chains_get_stats.argtypes = [vp, vp]
        L.ff_sim_strerror.restype = C.c_char_p
        L.ff_sim_strerror.argtypes = [C.c_int]
        _lib = L
    return _lib


class FFSimError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__(f"{where}: {lib().ff_sim_strerror(code).decode()} ({code})")


def _check(code, where):
    if code != FF_OK:
        raise FFSimError(code, where)


def ff_sim_create(ops, edges, machine, cost):
    """ops / edges: numpy arrays of workloads.OP_DT / EDGE_DT; machine: 7-tuple or
    workloads.Machine; cost: [n_ops][n_cols] uint32.  Returns an opaque handle (int)."""
    ops = np.ascontiguousarray(ops, W.OP_DT)
    edges = np.ascontiguousarray(edges, W.EDGE_DT)
    cost = np.ascontiguousarray(cost, "<u4")
    g = ff_opgraph_t(len(ops), len(edges), ops.ctypes.data, edges.ctypes.data)
    m = ff_machine_t(*(machine.as_tuple() if hasattr(machine, "as_tuple") else tuple(machine)))
    ct = ff_costtable_t(cost.shape[0], cost.shape[1], cost.ctypes.data)
    h = C.c_void_p()
    _check(lib().ff_sim_create(C.byref(g), C.byref(m), C.byref(ct), C.byref(h)), "ff_sim_create")
    return h.value


def ff_sim_create_tuplecost(ops, edges, machine, tuple_ptr, tuples, ns):
    """costs keyed by the degree tuple: op i's entries tuples[tuple_ptr[i]:tuple_ptr[i+1]] (packed,
    ascending) with exeTimes ns[] at the same index."""
    ops = np.ascontiguousarray(ops, W.OP_DT)
    edges = np.ascontiguousarray(edges, W.EDGE_DT)
    tuple_ptr, tuples, ns = (np.ascontiguousarray(a, "<u4") for a in (tuple_ptr, tuples, ns))
    g = ff_opgraph_t(len(ops), len(edges), ops.ctypes.data, edges.ctypes.data)
    m = ff_machine_t(*(machine.as_tuple() if hasattr(machine, "as_tuple") else tuple(machine)))
    tc = ff_tuplecost_t(len(ops), tuple_ptr.ctypes.data, tuples.ctypes.data, ns.ctypes.data)
    h = C.c_void_p()
    _check(lib().ff_sim_create_tuplecost(C.byref(g), C.byref(m), C.byref(tc), C.byref(h)), "ff_sim_create_tuplecost")
    return h.value


def ff_sim_destroy(sim):
    lib().ff_sim_destroy(sim)


def ff_sim_set_links(sim, gpus_per_node=0, Bpns=None, lat_ns=None):
    """Bpns / lat_ns: [gpus_per_node][gpus_per_node] (from local GPU, to local GPU); Bpns None:
    back to the machine's single intra-node figures."""
    if Bpns is None:
        _check(lib().ff_sim_set_links(sim, None), "ff_sim_set_links")
        return
    Bpns = np.ascontiguousarray(Bpns, "<u4")
    lat = None if lat_ns is None else np.ascontiguousarray(lat_ns, "<u4")
    if Bpns.size != gpus_per_node * gpus_per_node or (lat is not None and lat.size != Bpns.size):
        raise ValueError("link tables must be [gpus_per_node][gpus_per_node]")
    lt = ff_linktable_t(gpus_per_node, Bpns.ctypes.data, None if lat is None else lat.ctypes.data)
    _check(lib().ff_sim_set_links(sim, C.byref(lt)), "ff_sim_set_links")


def ff_sim_set_node_links(sim, n_nodes=0, Bpns=None, lat_ns=None):
    """Bpns / lat_ns: [n_nodes][n_nodes] (from node, to node); Bpns None: back to the machine's single
    inter-node figures."""
    if Bpns is None:
        _check(lib().ff_sim_set_node_links(sim, None), "ff_sim_set_node_links")
        return
    Bpns = np.ascontiguousarray(Bpns, "<u4")
    lat = None if lat_ns is None else np.ascontiguousarray(lat_ns, "<u4")
    if Bpns.size != n_nodes * n_nodes or (lat is not None and lat.size != Bpns.size):
        raise ValueError("node link tables must be [n_nodes][n_nodes]")
    lt = ff_linktable_t(n_nodes, Bpns.ctypes.data, None if lat is None else lat.ctypes.data)   # same layout as ff_nodelinks_t
    _check(lib().ff_sim_set_node_links(sim, C.byref(lt)), "ff_sim_set_node_links")


def ff_sim_set_ties(sim, n_ops, leader=None):
    """leader [n_ops] uint32: op i takes the configuration of op leader[i]; None: every op its own."""
    if leader is None:
        _check(lib().ff_sim_set_ties(sim, None), "ff_sim_set_ties")
        return
    t = np.ascontiguousarray(leader, "<u4")
    if t.shape != (n_ops,):
        raise ValueError("one leader per op")
    _check(lib().ff_sim_set_ties(sim, t.ctypes.data), "ff_sim_set_ties")


def ff_sim_set_params(sim, n_ops, param_bytes=None, param_dims=None):
    """param_bytes [n_ops] uint32 / param_dims [n_ops] uint8 (bit d: output dim d indexes the
    parameters); param_bytes None switches parameter synchronisation off."""
    if param_bytes is None:
        _check(lib().ff_sim_set_params(sim, None, None), "ff_sim_set_params")
        return
    pb = np.ascontiguousarray(param_bytes, "<u4")
    pd = np.ascontiguousarray(param_dims, np.uint8)
    if pb.shape != (n_ops,) or pd.shape != (n_ops,):
        raise ValueError("parameter tables must have one entry per op")
    _check(lib().ff_sim_set_params(sim, pb.ctypes.data, pd.ctypes.data), "ff_sim_set_params")


def ff_sim_workspace_bytes(sim, B):
    return lib().ff_sim_workspace_bytes(sim, B)


def ff_sim_set_workspace(sim, d_ws, nbytes):
    _check(lib().ff_sim_set_workspace(sim, d_ws, nbytes), "ff_sim_set_workspace")


def ff_sim_set_stats(sim, d_stats):
    _check(lib().ff_sim_set_stats(sim, d_stats), "ff_sim_set_stats")


def ff_sim_batch(sim, d_strategies, B, d_out_ns, stream=None):
    _check(lib().ff_sim_batch(sim, d_strategies, B, d_out_ns, stream), "ff_sim_batch")


def ff_sim_batch_devmaps(sim, d_strategies, d_devmaps, B, d_out_ns, stream=None):
    _check(lib().ff_sim_batch_devmaps(sim, d_strategies, d_devmaps, B, d_out_ns, stream), "ff_sim_batch_devmaps")


def ff_sim_chains_create(sim, d_strategies, C_, d_out_ns0, stream=None):
    h = C.c_void_p()
    _check(lib().ff_sim_chains_create(sim, d_strategies, C_, d_out_ns0, stream, C.byref(h)), "ff_sim_chains_create")
    return h.value


def ff_sim_delta(chains, d_muts, n_steps, d_out_ns, stream=None):
    _check(lib().ff_sim_delta(chains, d_muts, n_steps, d_out_ns, stream), "ff_sim_delta")


def ff_sim_chains_destroy(chains):
    lib().ff_sim_chains_destroy(chains)


def ff_sim_delta_try_workspace_bytes(chains, M):
    return lib().ff_sim_delta_try_workspace_bytes(chains, M)


def ff_sim_delta_try(chains, d_muts, M, d_out_ns, stream=None):
    _check(lib().ff_sim_delta_try(chains, d_muts, M, d_out_ns, stream), "ff_sim_delta_try")


def ff_sim_search(chains, params, n_steps, d_trace_ns, stream=None):
    _check(lib().ff_sim_search(chains, C.byref(params), n_steps, d_trace_ns, stream), "ff_sim_search")


def ff_sim_search_ahead(chains, params, n_steps, max_ahead, d_trace_ns, stream=None):
    """returns (rounds, proposals simulated ahead, steps made, proposals accepted; the last is not counted when the call
    runs as plain ff_sim_search because no look-ahead fits)"""
    st = ff_ahead_stats_t()
    _check(lib().ff_sim_search_ahead(chains, C.byref(params), n_steps, max_ahead, d_trace_ns, stream, C.byref(st)), "ff_sim_search_ahead")
    return st.rounds, st.proposals_simulated, st.steps, st.accepted


def ff_sim_neighbour_count(chains, d_tuple_ptr, n_tuples, op_begin, op_end):
    n = C.c_uint32()
    _check(lib().ff_sim_neighbour_count(chains, d_tuple_ptr, n_tuples, op_begin, op_end, C.byref(n)), "ff_sim_neighbour_count")
    return n.value


def ff_sim_neighbours(chains, d_tuple_ptr, d_tuples, n_tuples, op_begin, op_end, d_muts, d_out_ns, d_best_ns,
                      d_best_index, stream=None):
    _check(lib().ff_sim_neighbours(chains, d_tuple_ptr, d_tuples, n_tuples, op_begin, op_end, d_muts, d_out_ns,
                                   d_best_ns, d_best_index, stream), "ff_sim_neighbours")


def ff_sim_neighbours_noalloc(chains, d_tuple_ptr, d_tuples, n_tuples, op_begin, op_end, M, d_muts, d_out_ns, d_best_ns,
                              d_best_index, stream=None):
    _check(lib().ff_sim_neighbours_noalloc(chains, d_tuple_ptr, d_tuples, n_tuples, op_begin, op_end, M, d_muts, d_out_ns,
                                           d_best_ns, d_best_index, stream), "ff_sim_neighbours_noalloc")


def ff_sim_chains_get_stats(chains, n_chains):
    out = np.zeros(n_chains, CHAIN_STATS_DT)
    _check(lib().ff_sim_chains_get_stats(chains, out.ctypes.data), "ff_sim_chains_get_stats")
    return out


# ---- convenience on top of the boundary: torch tensors for device memory -----------------

def _torch():
    import torch
    if not torch.cuda.is_available():
        raise RuntimeError("no GPU visible: the simulator has no CPU path")
    return torch


def to_device(arr):
    """numpy (any dtype, incl. structured) -> uint8 torch tensor on cuda:0 holding its bytes."""
    torch = _torch()
    a = np.ascontiguousarray(arr)
    return torch.from_numpy(a.view(np.uint8).reshape(-1).copy()).cuda()


def ff_sim_accept_table(beta_per_ns, bucket_ns, n_buckets):
    """the acceptance table of ff_sim_search for a given beta (computed by the library)."""
    out = np.zeros(int(n_buckets), "<u4")
    _check(lib().ff_sim_accept_table(float(beta_per_ns), int(bucket_ns), int(n_buckets), out.ctypes.data), "ff_sim_accept_table")
    return out


def ff_sim_batch_kernel_name(sim, B):
    buf = C.create_string_buffer(256)
    _check(lib().ff_sim_batch_kernel_name(sim, B, buf, len(buf)), "ff_sim_batch_kernel_name")
    return buf.value.decode()


class Simulator:
    """owns a handle, its workspace and result buffers (all torch-allocated)."""

    def __init__(self, ops, edges, machine, cost, params=None, ties=None):
        """cost: [n_ops][n_cols] table by number of parts, or a triple (tuple_ptr, tuples, ns)
        keyed by the degree tuple.  params: (param_bytes, param_dims) per op, to simulate the
        parameter-synchronisation transfers as well."""
        _torch()
        self.n_ops = len(ops)
        if isinstance(cost, (tuple, list)):
            self.handle = ff_sim_create_tuplecost(ops, edges, machine, *cost)
        else:
            self.handle = ff_sim_create(ops, edges, machine, cost)
        if getattr(machine, "link_Bpns", None) is not None:
            lat = machine.link_lat_ns
            if lat is None:
                lat = np.full((machine.gpus_per_node,) * 2, machine.intra_lat_ns, "<u4")
            ff_sim_set_links(self.handle, machine.gpus_per_node, machine.link_Bpns, lat)
        if getattr(machine, "node_Bpns", None) is not None:
            lat = machine.node_lat_ns
            if lat is None:
                lat = np.full((machine.n_nodes,) * 2, machine.inter_lat_ns, "<u4")
            ff_sim_set_node_links(self.handle, machine.n_nodes, machine.node_Bpns, lat)
        if params is not None:
            ff_sim_set_params(self.handle, self.n_ops, params[0], params[1])
        if ties is not None:
            ff_sim_set_ties(self.handle, self.n_ops, ties)
        self._ws = None
        self._stats = None

    def close(self):
        if self.handle:
            ff_sim_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _ensure_workspace(self, B):
        torch = _torch()
        need = ff_sim_workspace_bytes(self.handle, B)
        if self._ws is None or self._ws.numel() < need:
            self._ws = None
            self._ws = torch.empty(need, dtype=torch.uint8, device="cuda")
            ff_sim_set_workspace(self.handle, self._ws.data_ptr(), self._ws.numel())

    def upload_strategies(self, cfgs):
        cfgs = np.ascontiguousarray(cfgs, W.CFG_DT)
        assert cfgs.ndim == 2 and cfgs.shape[1] == self.n_ops
        return to_device(cfgs)

    def batch(self, d_strategies, B, d_out=None, stats=False, d_devmaps=None):
        """d_strategies: device tensor from upload_strategies.  Returns the device tensor of
        B int64 (bit pattern of uint64 ns); asynchronous on the current stream.
        d_devmaps: device tensor of [B][n_ops][64] uint16, the device of every part given explicitly."""
        torch = _torch()
        self._ensure_workspace(B)
        if d_out is None:
            d_out = torch.empty(B, dtype=torch.int64, device="cuda")
        if stats:
            self._stats = torch.zeros(B * STATS_DT.itemsize, dtype=torch.uint8, device="cuda")
            ff_sim_set_stats(self.handle, self._stats.data_ptr())
        else:
            ff_sim_set_stats(self.handle, None)
        if d_devmaps is not None:
            ff_sim_batch_devmaps(self.handle, d_strategies.data_ptr(), d_devmaps.data_ptr(), B, d_out.data_ptr(),
                                 torch.cuda.current_stream().cuda_stream)
        else:
            ff_sim_batch(self.handle, d_strategies.data_ptr(), B, d_out.data_ptr(),
                         torch.cuda.current_stream().cuda_stream)
        return d_out

    def simulate(self, cfgs, stats=False, devmaps=None):
        """host convenience: numpy configs [B][n_ops] -> numpy uint64 [B] (and stats).
        devmaps: numpy [B][n_ops][64] uint16 (optional explicit devices)."""
        d = self.upload_strategies(cfgs)
        dm = None
        if devmaps is not None:
            devmaps = np.ascontiguousarray(devmaps, "<u2")
            assert devmaps.shape == (len(cfgs), self.n_ops, 64)
            dm = to_device(devmaps)
        out = self.batch(d, len(cfgs), stats=stats, d_devmaps=dm)
        res = out.cpu().numpy().view("<u8")
        if stats:
            return res, self._stats.cpu().numpy().view(STATS_DT)
        return res


class Chains:
    """C chains of cumulative single-op mutations (delta simulation)."""

    def __init__(self, sim: Simulator, cfgs0):
        torch = _torch()
        self.sim = sim
        cfgs0 = np.ascontiguousarray(cfgs0, W.CFG_DT)
        self.C = len(cfgs0)
        d = to_device(cfgs0)
        self.out0 = torch.empty(self.C, dtype=torch.int64, device="cuda")
        self.handle = ff_sim_chains_create(sim.handle, d.data_ptr(), self.C, self.out0.data_ptr(),
                                           torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()

    def start_ns(self):
        return self.out0.cpu().numpy().view("<u8")

    def upload_mutations(self, muts):
        muts = np.ascontiguousarray(muts, W.MUT_DT)
        assert muts.ndim == 2 and muts.shape[1] == self.C
        return to_device(muts)

    def delta(self, d_muts, n_steps, d_out=None):
        torch = _torch()
        if d_out is None:
            d_out = torch.empty((n_steps, self.C), dtype=torch.int64, device="cuda")
        ff_sim_delta(self.handle, d_muts.data_ptr(), n_steps, d_out.data_ptr(),
                     torch.cuda.current_stream().cuda_stream)
        return d_out

    def _ensure_try_workspace(self, M):
        """the trial kernel's slots live in the simulator's workspace"""
        torch = _torch()
        need = ff_sim_delta_try_workspace_bytes(self.handle, M)
        sim = self.sim
        if sim._ws is None or sim._ws.numel() < need:
            sim._ws = None
            sim._ws = torch.empty(need, dtype=torch.uint8, device="cuda")
            ff_sim_set_workspace(sim.handle, sim._ws.data_ptr(), sim._ws.numel())

    def try_mutations(self, d_muts, M, d_out=None):
        """evaluate M proposals per chain ([M][C] mutations) without changing the chains."""
        torch = _torch()
        self._ensure_try_workspace(M)
        if d_out is None:
            d_out = torch.empty((M, self.C), dtype=torch.int64, device="cuda")
        ff_sim_delta_try(self.handle, d_muts.data_ptr(), M, d_out.data_ptr(), torch.cuda.current_stream().cuda_stream)
        return d_out

    def search_setup(self, tuple_ptr, tuples, accept, bucket_ns, seed, patience=0):
        """uploads the proposal lists (workloads.search_space) and the acceptance table
        (probabilities scaled by 2^32, one per bucket of bucket_ns) and resets the best-so-far
        record.  Steps are numbered from 0 across the search() calls that follow."""
        torch = _torch()
        self._sp = dict(
            tuple_ptr=to_device(np.ascontiguousarray(tuple_ptr, "<u4")),
            tuples=to_device(np.ascontiguousarray(tuples, "<u4")),
            accept=to_device(np.ascontiguousarray(accept, "<u4")),
            best_ns=torch.full((self.C,), -1, dtype=torch.int64, device="cuda"),
            best=torch.zeros(self.C * self.sim.n_ops * W.CFG_DT.itemsize, dtype=torch.uint8, device="cuda"),
            n_tuples=len(tuples), n_buckets=len(accept), bucket_ns=int(bucket_ns), seed=int(seed), step=0,
            patience=int(patience))

    def search(self, n_steps, d_trace=None, ahead=0):
        """n_steps Metropolis steps on every chain; returns the device tensor [n_steps][C] of the
        chains' times after each step (asynchronous apart from the argument check).
        ahead > 0: ff_sim_search_ahead with up to that many proposals per chain simulated side by side (same
        results; synchronous; self.ahead_stats then holds (rounds, proposals simulated, steps))."""
        torch = _torch()
        sp = self._sp
        if d_trace is None:
            d_trace = torch.empty((n_steps, self.C), dtype=torch.int64, device="cuda")
        p = ff_search_t(sp["seed"], sp["step"], sp["bucket_ns"], sp["patience"], sp["n_buckets"], sp["n_tuples"],
                        sp["accept"].data_ptr(), sp["tuple_ptr"].data_ptr(), sp["tuples"].data_ptr(),
                        sp["best_ns"].data_ptr(), sp["best"].data_ptr())
        stream = torch.cuda.current_stream().cuda_stream
        if ahead:
            self._ensure_try_workspace(ahead & ~FF_AHEAD_ALWAYS)
            self.ahead_stats = ff_sim_search_ahead(self.handle, p, n_steps, ahead, d_trace.data_ptr(), stream)
        else:
            ff_sim_search(self.handle, p, n_steps, d_trace.data_ptr(), stream)
        sp["step"] += n_steps
        return d_trace

    def best(self):
        """(best times [C] uint64, best strategies [C][n_ops] of workloads.CFG_DT) so far."""
        sp = self._sp
        return (sp["best_ns"].cpu().numpy().view("<u8"),
                sp["best"].cpu().numpy().view(W.CFG_DT).reshape(self.C, self.sim.n_ops))

    def neighbours(self, tuple_ptr, tuples, op_begin=0, op_end=None):
        """every single-op neighbour of every chain's strategy for ops [op_begin, op_end).
        Returns (mutations [M][C] MUT_DT, times [M][C] uint64, best time [C], best index [C])."""
        torch = _torch()
        op_end = self.sim.n_ops if op_end is None else op_end
        d_ptr = to_device(np.ascontiguousarray(tuple_ptr, "<u4"))
        d_tup = to_device(np.ascontiguousarray(tuples, "<u4"))
        M = ff_sim_neighbour_count(self.handle, d_ptr.data_ptr(), len(tuples), op_begin, op_end)
        self._ensure_try_workspace(M)
        d_muts = torch.empty(M * self.C * W.MUT_DT.itemsize, dtype=torch.uint8, device="cuda")
        d_out = torch.empty((M, self.C), dtype=torch.int64, device="cuda")
        d_best = torch.empty(self.C, dtype=torch.int64, device="cuda")
        d_idx = torch.empty(self.C, dtype=torch.int32, device="cuda")
        ff_sim_neighbours(self.handle, d_ptr.data_ptr(), d_tup.data_ptr(), len(tuples), op_begin, op_end, d_muts.data_ptr(),
                          d_out.data_ptr(), d_best.data_ptr(), d_idx.data_ptr(), torch.cuda.current_stream().cuda_stream)
        return (d_muts.cpu().numpy().view(W.MUT_DT).reshape(M, self.C), d_out.cpu().numpy().view("<u8"),
                d_best.cpu().numpy().view("<u8"), d_idx.cpu().numpy().view("<u4"))

    def stats(self):
        return ff_sim_chains_get_stats(self.handle, self.C)

    def close(self):
        if self.handle:
            _torch().cuda.synchronize()
            ff_sim_chains_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
