"""Seeded synthetic inputs for the execution simulator: operator graphs, simulated
machines, cost tables, candidate strategies and single-op mutation chains.

This module only *describes inputs* (shapes, FLOP counts, random draws).  It holds none
of the simulator's arithmetic (no task-graph construction, no timeline), so both the CPU
oracle's tests and the GPU path's tests/bench may use it.

The five workloads stand in for the paper's benchmark DNNs (Table 3 and Section 8.1 give
only layer shapes; datasets and trained weights are not needed by the simulator).

Record layouts (numpy structured dtypes, little-endian, packed exactly like the C structs
of the library boundary):

  OP_DT    ndim u8 | par_mask u8 | type u16 | extent u32[4]
  EDGE_DT  src_op u32 | dst_op u32 | map[4] of {src_dim i8, pad u8, stride u16, a i32, b i32}
           map[] is indexed by the PRODUCER dim d.  src_dim = consumer output dim that
           drives producer dim d (-1: every consumer part needs the whole extent of d).
           For a consumer part covering [lo, hi) along src_dim the needed producer range is
           [lo*stride + a, (hi-1)*stride + b + 1) clamped to [0, extent_d].
           pad = 1 on all four maps marks a CONTRIBUTING edge (gradients flowing back along a forward
           edge): map[] is then indexed by the CONSUMER dim d, src_dim names a PRODUCER dim, and a
           producer part covering [lo, hi) along src_dim contributes to that range of the consumer's dim d.
  CFG_DT   deg u8[4] | dev_offset u16 | dev_stride u16       (one per op = a configuration c_i, Section 4)
  MUT_DT   op u32 | cfg CFG_DT
"""
from __future__ import annotations

import hashlib
from dataclasses import dataclass, field

import numpy as np

DIMMAP_DT = np.dtype([("src_dim", "i1"), ("pad", "u1"), ("stride", "<u2"), ("a", "<i4"), ("b", "<i4")])
OP_DT = np.dtype([("ndim", "u1"), ("par_mask", "u1"), ("type", "<u2"), ("extent", "<u4", (4,))])
EDGE_DT = np.dtype([("src_op", "<u4"), ("dst_op", "<u4"), ("map", DIMMAP_DT, (4,))])
CFG_DT = np.dtype([("deg", "u1", (4,)), ("dev_offset", "<u2"), ("dev_stride", "<u2")])
MUT_DT = np.dtype([("op", "<u4"), ("cfg", CFG_DT)])
assert DIMMAP_DT.itemsize == 12 and OP_DT.itemsize == 20 and EDGE_DT.itemsize == 56
assert CFG_DT.itemsize == 8 and MUT_DT.itemsize == 12

MAX_PARTS = 64          # largest |c_i| the boundary accepts
BASE_SEED = 1807053580

# informational op type codes
T_CONV, T_POOL, T_FC, T_SOFTMAX, T_ELEM, T_CONCAT, T_EMBED, T_ATTN, T_SLICE, T_STACK = range(10)

ALL = None  # marker for "whole extent needed"


def ident(c):
    """producer dim follows consumer dim c one-to-one."""
    return (c, 1, 0, 0)


def window(c, stride, pad, k):
    """sliding window of size k, given stride and padding, along consumer dim c."""
    return (c, stride, -pad, -pad + k - 1)


def shifted(c, off):
    """producer index = consumer index + off (slices, concat inputs)."""
    return (c, 1, off, off)


@dataclass
class Machine:
    n_nodes: int
    gpus_per_node: int
    intra_Bpns: int = 20
    inter_Bpns: int = 12
    intra_lat_ns: int = 0
    inter_lat_ns: int = 0
    elem_bytes: int = 4
    # optional [gpus_per_node][gpus_per_node] tables (from local GPU, to local GPU): links inside
    # a node that are not all alike; None = intra_Bpns / intra_lat_ns for every pair
    link_Bpns: object = None
    link_lat_ns: object = None
    # optional [n_nodes][n_nodes] tables (from node, to node): network links between nodes that are not
    # all alike; None = inter_Bpns / inter_lat_ns for every pair
    node_Bpns: object = None
    node_lat_ns: object = None

    @property
    def n_devices(self) -> int:
        return self.n_nodes * self.gpus_per_node

    def as_tuple(self):
        return (self.n_nodes, self.gpus_per_node, self.intra_Bpns, self.inter_Bpns,
                self.intra_lat_ns, self.inter_lat_ns, self.elem_bytes)


class GraphBuilder:
    """Collects ops (in topological order) and tensor edges of an operator graph."""

    def __init__(self):
        self.ops = []     # (ndim, par_mask, type, extent[4], flops)
        self.edges = []   # (src, dst, [map per producer dim])
        self.group_of = {}   # op -> label of the parameters it shares with other ops (unrolled steps of a layer)

    def shares(self, op, label):
        """op uses the parameters named `label` (every op with that label uses the same ones)."""
        self.group_of[op] = label
        return op

    def op(self, typ, extent, par_dims, flops):
        extent = list(extent)
        ndim = len(extent)
        assert 1 <= ndim <= 4
        mask = 0
        for d in par_dims:
            assert 0 <= d < ndim
            mask |= 1 << d
        self.ops.append((ndim, mask, typ, extent + [1] * (4 - ndim), int(flops)))
        return len(self.ops) - 1

    def extent(self, o):
        nd = self.ops[o][0]
        return self.ops[o][3][:nd]

    def edge(self, src, dst, maps):
        assert src < dst, "ops must be created in topological order"
        assert len(maps) == self.ops[src][0]
        self.edges.append((src, dst, list(maps)))

    def finish(self):
        ops = np.zeros(len(self.ops), OP_DT)
        flops = np.zeros(len(self.ops), np.int64)
        for i, (nd, mask, typ, ext, fl) in enumerate(self.ops):
            ops[i]["ndim"], ops[i]["par_mask"], ops[i]["type"] = nd, mask, typ
            ops[i]["extent"] = ext
            flops[i] = fl
        # canonical edge order: by producer op, then consumer op, then creation order
        order = sorted(range(len(self.edges)), key=lambda k: (self.edges[k][0], self.edges[k][1], k))
        edges = np.zeros(len(order), EDGE_DT)
        for n, k in enumerate(order):
            s, d, maps = self.edges[k]
            edges[n]["src_op"], edges[n]["dst_op"] = s, d
            for pd in range(4):
                m = maps[pd] if pd < len(maps) else ALL
                if m is ALL:
                    edges[n]["map"][pd] = (-1, 0, 1, 0, 0)
                else:
                    c, st, a, b = m
                    edges[n]["map"][pd] = (c, 0, st, a, b)
        return ops, edges, flops

    # ---- CNN helpers: tensors are (sample, channel, h, w) -------------------------------
    def conv(self, src, co, kh, kw=None, stride=1, ph=0, pw=None, src_extent=None):
        kw = kh if kw is None else kw
        pw = ph if pw is None else pw
        n, ci, h, w = self.extent(src) if src is not None else src_extent
        ho = (h + 2 * ph - kh) // stride + 1
        wo = (w + 2 * pw - kw) // stride + 1
        o = self.op(T_CONV, (n, co, ho, wo), (0, 1, 2, 3), 2 * n * co * ho * wo * ci * kh * kw)
        if src is not None:
            self.edge(src, o, [ident(0), ALL, window(2, stride, ph, kh), window(3, stride, pw, kw)])
        return o

    def pool(self, src, k, stride, pad=0):
        n, c, h, w = self.extent(src)
        ho = (h + 2 * pad - k) // stride + 1
        wo = (w + 2 * pad - k) // stride + 1
        o = self.op(T_POOL, (n, c, ho, wo), (0, 1, 2, 3), n * c * ho * wo * k * k)
        self.edge(src, o, [ident(0), ident(1), window(2, stride, pad, k), window(3, stride, pad, k)])
        return o

    def fc(self, src, co):
        ext = self.extent(src)
        n = ext[0]
        ci = int(np.prod(ext[1:]))
        o = self.op(T_FC, (n, co, 1, 1), (0, 1), 2 * n * ci * co)
        self.edge(src, o, [ident(0)] + [ALL] * (len(ext) - 1))
        return o

    def softmax(self, src):
        ext = self.extent(src)
        o = self.op(T_SOFTMAX, ext, (0,), 5 * int(np.prod(ext)))
        self.edge(src, o, [ident(0)] + [ALL] * (len(ext) - 1))
        return o

    def elementwise(self, srcs):
        ext = self.extent(srcs[0])
        o = self.op(T_ELEM, ext, tuple(range(len(ext))), int(np.prod(ext)))
        for s in srcs:
            assert self.extent(s) == ext
            self.edge(s, o, [ident(d) for d in range(len(ext))])
        return o

    def concat(self, srcs, axis=1):
        exts = [self.extent(s) for s in srcs]
        out = list(exts[0])
        out[axis] = sum(e[axis] for e in exts)
        o = self.op(T_CONCAT, out, tuple(range(len(out))), int(np.prod(out)))
        off = 0
        for s, e in zip(srcs, exts):
            maps = [ident(d) for d in range(len(out))]
            maps[axis] = shifted(axis, -off)
            self.edge(s, o, maps)
            off += e[axis]
        return o


# ---------------------------------------------------------------------------------------
# operator graphs
# ---------------------------------------------------------------------------------------

def graph_tiny_chain():
    """configs[0]: conv, pool, conv, pool, fc, softmax on (64, ., 32, 32) inputs."""
    g = GraphBuilder()
    c1 = g.conv(None, 16, 3, ph=1, src_extent=(64, 3, 32, 32))
    p1 = g.pool(c1, 2, 2)
    c2 = g.conv(p1, 32, 3, ph=1)
    p2 = g.pool(c2, 2, 2)
    f = g.fc(p2, 128)
    g.softmax(f)
    return g.finish()


def graph_alexnet(batch=256):
    """configs[1]: AlexNet-shaped 12-op chain (Table 3)."""
    g = GraphBuilder()
    x = g.conv(None, 96, 11, stride=4, ph=2, src_extent=(batch, 3, 224, 224))
    x = g.pool(x, 3, 2)
    x = g.conv(x, 256, 5, ph=2)
    x = g.pool(x, 3, 2)
    x = g.conv(x, 384, 3, ph=1)
    x = g.conv(x, 384, 3, ph=1)
    x = g.conv(x, 256, 3, ph=1)
    x = g.pool(x, 3, 2)
    x = g.fc(x, 4096)
    x = g.fc(x, 4096)
    x = g.fc(x, 1000)
    g.softmax(x)
    return g.finish()


def graph_inception_v3(batch=64):
    """configs[2]: Inception-v3-shaped DAG (stem, 3xA, reduce, 4xB, reduce, 2xC, tail);
    conv+bn+relu count as one op."""
    g = GraphBuilder()
    x = g.conv(None, 32, 3, stride=2, src_extent=(batch, 3, 299, 299))
    x = g.conv(x, 32, 3)
    x = g.conv(x, 64, 3, ph=1)
    x = g.pool(x, 3, 2)
    x = g.conv(x, 80, 1)
    x = g.conv(x, 192, 3)
    x = g.pool(x, 3, 2)                       # 192 @ 35x35
    for pool_ch in (32, 64, 64):              # three "A" blocks
        b0 = g.conv(x, 64, 1)
        b1 = g.conv(g.conv(x, 48, 1), 64, 5, ph=2)
        b2 = g.conv(g.conv(g.conv(x, 64, 1), 96, 3, ph=1), 96, 3, ph=1)
        b3 = g.conv(g.pool(x, 3, 1, 1), pool_ch, 1)
        x = g.concat([b0, b1, b2, b3])
    b0 = g.conv(x, 384, 3, stride=2)          # grid reduction 35 -> 17
    b1 = g.conv(g.conv(g.conv(x, 64, 1), 96, 3, ph=1), 96, 3, stride=2)
    b2 = g.pool(x, 3, 2)
    x = g.concat([b0, b1, b2])
    for c7 in (128, 160, 160, 192):           # four "B" blocks with factorised 7x7
        b0 = g.conv(x, 192, 1)
        b1 = g.conv(g.conv(g.conv(x, c7, 1), c7, 1, 7, ph=0, pw=3), 192, 7, 1, ph=3, pw=0)
        t = g.conv(x, c7, 1)
        t = g.conv(t, c7, 7, 1, ph=3, pw=0)
        t = g.conv(t, c7, 1, 7, ph=0, pw=3)
        t = g.conv(t, c7, 7, 1, ph=3, pw=0)
        b2 = g.conv(t, 192, 1, 7, ph=0, pw=3)
        b3 = g.conv(g.pool(x, 3, 1, 1), 192, 1)
        x = g.concat([b0, b1, b2, b3])
    b0 = g.conv(g.conv(x, 192, 1), 320, 3, stride=2)   # grid reduction 17 -> 8
    t = g.conv(x, 192, 1)
    t = g.conv(t, 192, 1, 7, ph=0, pw=3)
    t = g.conv(t, 192, 7, 1, ph=3, pw=0)
    b1 = g.conv(t, 192, 3, stride=2)
    b2 = g.pool(x, 3, 2)
    x = g.concat([b0, b1, b2])
    for _ in range(2):                        # two "C" blocks with split 1x3 / 3x1 heads
        b0 = g.conv(x, 320, 1)
        t = g.conv(x, 384, 1)
        b1a = g.conv(t, 384, 1, 3, ph=0, pw=1)
        b1b = g.conv(t, 384, 3, 1, ph=1, pw=0)
        t = g.conv(g.conv(x, 448, 1), 384, 3, ph=1)
        b2a = g.conv(t, 384, 1, 3, ph=0, pw=1)
        b2b = g.conv(t, 384, 3, 1, ph=1, pw=0)
        b3 = g.conv(g.pool(x, 3, 1, 1), 192, 1)
        x = g.concat([b0, b1a, b1b, b2a, b2b, b3])
    x = g.pool(x, 8, 1)
    x = g.fc(x, 1000)
    g.softmax(x)
    return g.finish()


def graph_resnet101(batch=64):
    """configs[3]: ResNet-101-shaped DAG: 33 bottleneck blocks (3, 4, 23, 3), conv / bn /
    relu / add as separate ops."""
    g = GraphBuilder()
    x = g.conv(None, 64, 7, stride=2, ph=3, src_extent=(batch, 3, 224, 224))
    x = g.elementwise([x])   # bn
    x = g.elementwise([x])   # relu
    x = g.pool(x, 3, 2, 1)   # 64 @ 56x56
    for stage, (blocks, width) in enumerate(((3, 64), (4, 128), (23, 256), (3, 512))):
        for blk in range(blocks):
            stride = 2 if (blk == 0 and stage > 0) else 1
            t = g.conv(x, width, 1)
            t = g.elementwise([t])
            t = g.elementwise([t])
            t = g.conv(t, width, 3, stride=stride, ph=1)
            t = g.elementwise([t])
            t = g.elementwise([t])
            t = g.conv(t, width * 4, 1)
            t = g.elementwise([t])
            if blk == 0:
                sc = g.conv(x, width * 4, 1, stride=stride)
                sc = g.elementwise([sc])
            else:
                sc = x
            t = g.elementwise([t, sc])   # residual add
            x = g.elementwise([t])       # relu
    x = g.pool(x, 7, 1)
    x = g.fc(x, 1000)
    g.softmax(x)
    return g.finish()


def graph_nmt(batch=64, hidden=1024, steps=40, vocab=32768, with_groups=False):
    """configs[4]: NMT-shaped graph: 2-layer LSTM encoder and decoder unrolled `steps`
    times, attention over the stacked encoder states at every decoder step, output
    projection and softmax over the vocabulary.  Tensors are (sample, channel); the
    stacked encoder state is (sample, length, channel)."""
    g = GraphBuilder()
    N, H = batch, hidden

    def matmul(src, co):
        ext = g.extent(src)
        o = g.op(T_FC, (N, co), (0, 1), 2 * N * int(np.prod(ext[1:])) * co)
        g.edge(src, o, [ident(0)] + [ALL] * (len(ext) - 1))
        return o

    def lstm_cell(x, h_prev, c_prev, tag=None):
        mx = g.shares(matmul(x, 4 * H), (tag, "x"))
        if h_prev is not None:
            mh = matmul(h_prev, 4 * H)
        else:   # first step: the recurrent product has no tensor input
            mh = g.op(T_FC, (N, 4 * H), (0, 1), 2 * N * H * 4 * H)
        g.shares(mh, (tag, "h"))
        s = g.elementwise([mx, mh])
        gates = []
        for k in range(4):
            o = g.op(T_SLICE, (N, H), (0, 1), N * H)
            g.edge(s, o, [ident(0), shifted(1, k * H)])
            gates.append(o)
        gi, gf, gg, go = gates
        fc_ = g.elementwise([gf, c_prev]) if c_prev is not None else g.elementwise([gf])
        ig = g.elementwise([gi, gg])
        c = g.elementwise([fc_, ig])
        tc = g.elementwise([c])
        h = g.elementwise([go, tc])
        return h, c

    def embed(tag=None):
        return g.shares(g.op(T_EMBED, (N, H), (0, 1), N * H), (tag, "embed"))

    enc_state = [(None, None), (None, None)]
    enc_top = []
    for _ in range(steps):
        x = embed("enc")
        for layer in range(2):
            h, c = lstm_cell(x, *enc_state[layer], tag=("enc", layer))
            enc_state[layer] = (h, c)
            x = h
        enc_top.append(x)
    stack = g.op(T_STACK, (N, steps, H), (0, 2), N * steps * H)
    for t, h in enumerate(enc_top):
        # every part of the stacked tensor needs step t (the length dim is not partitioned)
        g.edge(h, stack, [ident(0), ident(2)])
    dec_state = list(enc_state)
    for _ in range(steps):
        x = embed("dec")
        for layer in range(2):
            h, c = lstm_cell(x, *dec_state[layer], tag=("dec", layer))
            dec_state[layer] = (h, c)
            x = h
        score = g.op(T_ATTN, (N, steps), (0,), 2 * N * steps * H)
        g.edge(stack, score, [ident(0), ALL, ALL])
        g.edge(x, score, [ident(0), ALL])
        prob = g.softmax(score)
        ctx = g.op(T_ATTN, (N, H), (0, 1), 2 * N * steps * H)
        g.edge(prob, ctx, [ident(0), ALL])
        g.edge(stack, ctx, [ident(0), ALL, ident(1)])
        cat = g.concat([ctx, x], axis=1)
        lin = g.shares(matmul(cat, H), ("dec", "attention-out"))
        th = g.elementwise([lin])
        out = g.shares(matmul(th, vocab), ("dec", "vocabulary"))
        g.softmax(out)
    if with_groups:
        return g.finish() + (dict(g.group_of),)
    return g.finish()


# ---------------------------------------------------------------------------------------
# costs
# ---------------------------------------------------------------------------------------

def _mix64(x):
    """SplitMix64 finaliser on uint64 arrays (the one documented generator of this module)."""
    x = np.asarray(x, dtype=np.uint64)
    with np.errstate(over="ignore"):
        x = (x + np.uint64(0x9E3779B97F4A7C15))
        x = (x ^ (x >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        x = (x ^ (x >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        x = x ^ (x >> np.uint64(31))
    return x


def _draw(seed, *counters):
    """counter-based draw: hash of (seed, counters...) -> uint64 array (broadcast)."""
    h = _mix64(np.uint64(seed))
    for c in counters:
        with np.errstate(over="ignore"):
            h = _mix64(h ^ (np.asarray(c, dtype=np.uint64) * np.uint64(0xD6E8FEB86659FD93)))
    return h


def _ceil_div(a, b):
    return -(-a // b)


def cost_table(config_id, flops, seed):
    """exeTime of a compute task of op i when the op is split into p parts, p = 1..64:
    table[i][p-1] (the cached per-(op, size) measurement of Section 5.1, replaced by a model)."""
    n = len(flops)
    parts = np.arange(1, MAX_PARTS + 1, dtype=np.int64)[None, :]
    fl = flops.astype(np.int64)[:, None]
    if config_id == 0:
        base = (50000 + (_draw(seed, 7, np.arange(n)) % np.uint64(1950001)).astype(np.int64))[:, None]
        t = _ceil_div(base, parts) + 5000
    elif config_id == 1:
        base = 50000 + (1950000 * fl) // fl.max()
        t = _ceil_div(base, parts) + 5000
    else:
        # the largest convolutions exceed 2^32 ns when unsplit: saturate (the table is u32)
        t = np.minimum(_ceil_div(fl, 10 * parts) + 5000, 2 ** 32 - 1)
    assert t.min() >= 1 and t.max() < 2 ** 32
    return np.ascontiguousarray(t.astype(np.uint32))


# ---------------------------------------------------------------------------------------
# strategies and mutation chains
# ---------------------------------------------------------------------------------------

def valid_degree_tuples(op, max_parts, choices):
    """all degree tuples allowed for one op: degree from `choices` on parallelizable dims,
    1 elsewhere, product <= max_parts, degree <= extent."""
    per_dim = []
    for d in range(4):
        if d < op["ndim"] and (op["par_mask"] >> d) & 1:
            per_dim.append([c for c in choices if c <= op["extent"][d]])
        else:
            per_dim.append([1])
    out = []
    for a in per_dim[0]:
        for b in per_dim[1]:
            for c in per_dim[2]:
                for e in per_dim[3]:
                    if a * b * c * e <= max_parts:
                        out.append((a, b, c, e))
    return np.array(out, dtype=np.uint8)


def _draw_cfgs(ops, op_idx, cand_idx, step_idx, seed, n_dev, max_parts, choices):
    """configs for (op, candidate, step) triples; uniform over the op's valid tuples,
    device offset uniform in [0, n_dev), stride 1."""
    op_idx = np.asarray(op_idx, dtype=np.int64)
    out = np.zeros(op_idx.shape, CFG_DT)
    r_deg = _draw(seed, 1, cand_idx, op_idx, step_idx)
    r_off = _draw(seed, 2, cand_idx, op_idx, step_idx)
    # ops with the same (ndim, par_mask, extent) share one list of valid tuples
    sig_of, lists = {}, []
    sig = np.zeros(len(ops), np.int64)
    for i, o in enumerate(ops):
        key = (int(o["ndim"]), int(o["par_mask"]), tuple(int(e) for e in o["extent"]))
        if key not in sig_of:
            sig_of[key] = len(lists)
            lists.append(valid_degree_tuples(o, max_parts, choices))
        sig[i] = sig_of[key]
    n_valid = np.array([len(t) for t in lists], dtype=np.uint64)
    table = np.ones((len(lists), int(n_valid.max()), 4), np.uint8)
    for k, t in enumerate(lists):
        table[k, :len(t)] = t
    s_idx = sig[op_idx]
    out["deg"] = table[s_idx, (r_deg % n_valid[s_idx]).astype(np.int64)]
    out["dev_offset"] = (r_off % np.uint64(n_dev)).astype(np.uint16)
    out["dev_stride"] = 1
    return out


def strategies(ops, n_cand, seed, n_dev, max_parts, choices):
    n_ops = len(ops)
    op_idx = np.broadcast_to(np.arange(n_ops)[None, :], (n_cand, n_ops))
    cand = np.broadcast_to(np.arange(n_cand)[:, None], (n_cand, n_ops))
    return _draw_cfgs(ops, op_idx, cand, 0, seed, n_dev, max_parts, choices)


def mutation_chains(ops, n_steps, n_chains, seed, n_dev, max_parts, choices):
    """[n_steps][n_chains] single-op mutations: op uniform, new config from the strategy
    distribution (the proposal of Section 6.2, with every proposal accepted)."""
    step = np.broadcast_to(np.arange(1, n_steps + 1)[:, None], (n_steps, n_chains))
    chain = np.broadcast_to(np.arange(n_chains)[None, :], (n_steps, n_chains))
    op = (_draw(seed, 3, chain, step) % np.uint64(len(ops))).astype(np.int64)
    out = np.zeros((n_steps, n_chains), MUT_DT)
    out["op"] = op
    out["cfg"] = _draw_cfgs(ops, op, chain, step, seed, n_dev, max_parts, choices)
    return out


def search_space(ops, max_parts, choices):
    """the proposal lists of a search: (tuple_ptr [n_ops+1] uint32, tuples uint32), the valid
    degree tuples of every op, four bytes each (degree of dim 0 in the lowest byte)."""
    ptr = np.zeros(len(ops) + 1, np.uint32)
    chunks = []
    for i, o in enumerate(ops):
        t = valid_degree_tuples(o, max_parts, choices).astype(np.uint32)
        chunks.append(t[:, 0] | (t[:, 1] << 8) | (t[:, 2] << 16) | (t[:, 3] << 24))
        ptr[i + 1] = ptr[i] + len(t)
    return ptr, np.concatenate(chunks).astype(np.uint32)


def tuple_cost_table(ops, cost, max_parts, choices, seed):
    """costs keyed by the whole degree tuple, derived from a table by number of parts: the
    entry for `parts` plus, per split dim other than the sample dim, a seeded surcharge of
    0-25 % (splitting channels or pixels makes tasks less efficient than splitting samples).
    Returns (tuple_ptr, tuples ascending per op, ns)."""
    ptr = np.zeros(len(ops) + 1, np.uint32)
    tup_all, ns_all = [], []
    for i, o in enumerate(ops):
        t = valid_degree_tuples(o, max_parts, choices).astype(np.uint64)
        packed = (t[:, 0] | (t[:, 1] << np.uint64(8)) | (t[:, 2] << np.uint64(16)) | (t[:, 3] << np.uint64(24)))
        parts = t[:, 0] * t[:, 1] * t[:, 2] * t[:, 3]
        base = cost[i, parts.astype(np.int64) - 1].astype(np.uint64)
        extra = np.zeros(len(t), np.uint64)
        for d in (1, 2, 3):
            pct = _draw(seed, 7, i, d) % np.uint64(26)
            extra += np.where(t[:, d] > 1, base * pct // np.uint64(100), np.uint64(0))
        ns = np.minimum(base + extra, np.uint64(2 ** 32 - 1))
        order = np.argsort(packed, kind="stable")
        tup_all.append(packed[order].astype(np.uint32))
        ns_all.append(ns[order].astype(np.uint32))
        ptr[i + 1] = ptr[i] + len(t)
    return ptr, np.concatenate(tup_all), np.concatenate(ns_all)


def paired_links(gpus_per_node, fast_Bpns, slow_Bpns, fast_lat_ns=0, slow_lat_ns=0):
    """link tables [G][G] of a node whose GPUs sit in pairs (2k, 2k+1) behind a common switch:
    the two GPUs of a pair talk over the fast link, any other two over the slow one (the shape
    of the dual-GPU boards of the paper's older cluster, Section 8.1)."""
    G = gpus_per_node
    a = np.arange(G)
    same = (a[:, None] // 2) == (a[None, :] // 2)
    return (np.where(same, fast_Bpns, slow_Bpns).astype("<u4"),
            np.where(same, fast_lat_ns, slow_lat_ns).astype("<u4"))


def ring_node_links(n_nodes, near_Bpns, far_Bpns, hop_lat_ns=0):
    """link tables [N][N] of nodes on a ring: neighbours talk at near_Bpns, any other two nodes at
    far_Bpns; latency hop_lat_ns per hop of the shorter way round (a network whose connections are not
    all alike, as the device topology of Section 3 allows)."""
    a = np.arange(n_nodes)
    d = np.abs(a[:, None] - a[None, :])
    hops = np.minimum(d, n_nodes - d)
    return (np.where(hops <= 1, near_Bpns, far_Bpns).astype("<u4"), (hops * hop_lat_ns).astype("<u4"))


def device_maps(cfgs, n_dev, seed, spread=None):
    """a seeded explicit device for every part of every op of cfgs [B][n_ops]: [B][n_ops][64]
    uint16; entries beyond an op's parts hold 0xffff (they must be ignored).  spread: devices are
    drawn from the first `spread` devices only (more sharing)."""
    B, n_ops = cfgs.shape
    hi = n_dev if spread is None else min(n_dev, spread)
    rng = np.random.Generator(np.random.PCG64(seed))
    maps = rng.integers(0, hi, size=(B, n_ops, MAX_PARTS), dtype=np.uint16)
    parts = cfgs["deg"].astype(np.uint32).prod(axis=2)
    maps[np.arange(MAX_PARTS)[None, None, :] >= parts[:, :, None]] = 0xFFFF
    return maps


def param_table(ops, flops, bytes_per_param=4):
    """parameters of every op for the parameter-synchronisation refinement: (param_bytes [n_ops]
    uint32, param_dims [n_ops] uint8).  Convolutions and matrix products hold
    out_channels x (inputs per output element) parameters, recovered from the op's FLOPs
    (2 x outputs x inputs per output element) and indexed by the output's channel dim (bit 1); all
    other ops hold none.  Every op owns its parameters (unrolled steps of a recurrent layer are not
    tied together)."""
    pb = np.zeros(len(ops), "<u4")
    pd = np.zeros(len(ops), np.uint8)
    for i, o in enumerate(ops):
        if o["type"] in (T_CONV, T_FC):
            e = [int(x) for x in o["extent"]]
            n_params = int(flops[i]) // (2 * e[0] * e[2] * e[3])
            pb[i] = min(n_params * bytes_per_param, 2 ** 32 - 1)
            pd[i] = 2
    return pb, pd


def training_graph(ops, edges, flops, groups=None, backward_cost=2):
    """The graph of a whole training iteration, from a forward graph: every forward op i gets a backward op
    i' (same tensor shape, same parallelizable dims, `backward_cost` times the forward FLOPs), created in reverse
    order behind the forward ops (i' = 2n - 1 - i).  Edges: the forward edges; i -> i' (the backward computation
    needs what the forward one kept: one-to-one); and for every forward edge p -> i the CONTRIBUTING edge i' -> p'
    with the forward edge's maps (the part of i' that belongs to an output part of i produces gradient for exactly
    the input range that part read).  An operation is one thing to the strategy (Section 4): i' takes the
    configuration of i (`leader`).  `groups`: {forward op: label}; ops with the same label share their parameters:
    they all take the configuration of the first of them, and the parameters are synchronised once, after the
    backward op that runs last (that of the first forward op).  Parameters (param_table's model) sit on the
    backward op of every convolution / matrix product that owns some, or on the group's last backward op.
    Returns (ops, edges, flops, leader [2n] uint32, (param_bytes [2n] uint32, param_dims [2n] uint8))."""
    n = len(ops)
    bwd = lambda i: 2 * n - 1 - i
    ops2 = np.zeros(2 * n, OP_DT)
    ops2[:n] = ops
    flops2 = np.zeros(2 * n, np.int64)
    flops2[:n] = flops
    leader = np.arange(2 * n, dtype=np.uint32)
    first_of = {}
    for i in range(n):
        ops2[bwd(i)] = ops[i]
        flops2[bwd(i)] = backward_cost * int(flops[i])
        lead = i
        if groups and i in groups:
            lead = first_of.setdefault(groups[i], i)
            if tuple(ops[lead]["extent"]) != tuple(ops[i]["extent"]) or ops[lead]["par_mask"] != ops[i]["par_mask"]:
                lead = i                         # (shares parameters but not its shape: keeps its own configuration)
        leader[i] = leader[bwd(i)] = lead
    rows = []
    for e in edges:
        rows.append((int(e["src_op"]), int(e["dst_op"]), e["map"].copy()))
        m = e["map"].copy()
        m["pad"] = 1
        rows.append((bwd(int(e["dst_op"])), bwd(int(e["src_op"])), m))
    for i in range(n):
        m = np.zeros(4, DIMMAP_DT)
        for d in range(4):
            m[d] = (d, 0, 1, 0, 0) if d < ops[i]["ndim"] else (-1, 0, 1, 0, 0)
        rows.append((i, bwd(i), m))
    rows.sort(key=lambda r: (r[0], r[1]))
    edges2 = np.zeros(len(rows), EDGE_DT)
    for k, (a, b, m) in enumerate(rows):
        assert a < b
        edges2[k]["src_op"], edges2[k]["dst_op"], edges2[k]["map"] = a, b, m
    pb_f, pd_f = param_table(ops, flops)
    pb = np.zeros(2 * n, "<u4")
    pd = np.zeros(2 * n, np.uint8)
    for i in range(n):
        if pb_f[i]:
            if groups and i in groups and leader[i] != i:
                continue                         # the group's parameters are synchronised by its first op's backward op
            pb[bwd(i)], pd[bwd(i)] = pb_f[i], pd_f[i]
    return ops2, edges2, flops2, leader, (pb, pd)


def data_parallel_strategy(ops, n_dev, max_parts=MAX_PARTS):
    """every op split in the sample dim only, as far as the device count allows."""
    cfg = np.zeros(len(ops), CFG_DT)
    cfg["deg"] = 1
    p = 1
    while p * 2 <= min(n_dev, max_parts):
        p *= 2
    cfg["deg"][:, 0] = np.minimum(p, ops["extent"][:, 0])
    cfg["dev_stride"] = 1
    return cfg


# ---------------------------------------------------------------------------------------
# the five configurations
# ---------------------------------------------------------------------------------------

@dataclass
class Workload:
    config_id: int
    name: str
    ops: np.ndarray
    edges: np.ndarray
    flops: np.ndarray
    machine: Machine
    cost: np.ndarray            # [n_ops][max_parts] uint32 ns
    n_candidates: int
    max_parts: int
    choices: tuple
    seed: int
    _strategies: np.ndarray = field(default=None, repr=False)

    @property
    def n_ops(self):
        return len(self.ops)

    def strategies(self, n=None):
        n = self.n_candidates if n is None else n
        if self._strategies is None or len(self._strategies) < n:
            self._strategies = strategies(self.ops, n, self.seed, self.machine.n_devices,
                                          self.max_parts, self.choices)
        return self._strategies[:n].copy()      # callers may edit their batch

    def mutations(self, n_steps, n_chains=1):
        return mutation_chains(self.ops, n_steps, n_chains, self.seed, self.machine.n_devices,
                               self.max_parts, self.choices)

    def tuple_costs(self):
        """the same costs keyed by degree tuple (see tuple_cost_table)"""
        return tuple_cost_table(self.ops, self.cost, self.max_parts, self.choices, self.seed)

    def search_space(self):
        return search_space(self.ops, self.max_parts, self.choices)

    def param_table(self):
        return param_table(self.ops, self.flops)

    def sha256(self, n=None):
        h = hashlib.sha256()
        for a in (self.ops, self.edges, self.cost, self.strategies(n)):
            h.update(np.ascontiguousarray(a).tobytes())
        h.update(repr(self.machine.as_tuple()).encode())
        return h.hexdigest()


_SPECS = {
    0: ("tiny_chain", graph_tiny_chain, Machine(1, 4), 64, 4, (1, 2, 4)),
    1: ("alexnet", graph_alexnet, Machine(4, 4), 1024, 16, (1, 2, 4, 8, 16)),
    2: ("inception_v3", graph_inception_v3, Machine(16, 4), 4096, 64, (1, 2, 4, 8, 16, 32, 64)),
    3: ("resnet101", graph_resnet101, Machine(16, 4), 4096, 64, (1, 2, 4, 8, 16, 32, 64)),
    4: ("nmt", graph_nmt, Machine(16, 4), 1024, 64, (1, 2, 4, 8, 16, 32, 64)),
}

_cache = {}


def workload(config_id: int) -> Workload:
    """the config_id-th configuration of the benchmark list (0 tiny chain .. 4 NMT)."""
    if config_id not in _cache:
        name, fn, mach, n_cand, max_parts, choices = _SPECS[config_id]
        ops, edges, flops = fn()
        seed = BASE_SEED + config_id
        # one column per possible number of parts of the configuration (configs[0]: 4, [1]: 16, others 64)
        cost = np.ascontiguousarray(cost_table(config_id, flops, seed)[:, :max_parts])
        _cache[config_id] = Workload(config_id, name, ops, edges, flops, mach, cost, n_cand, max_parts,
                                     choices, seed)
    return _cache[config_id]
