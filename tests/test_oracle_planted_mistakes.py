"""Do the pins pin?  Every plausible mistake in the oracle must make at least one pin fail.

Each case below is a textual change to a COPY of oracle/ff_oracle.cpp (a wrong rounding of the
partition bounds, a transposed link row, a dropped term ...).  The copy is compiled, and the pin
tests -- hand-computed fixtures, closed forms, invariants, brute force; nothing that compares the
oracle with itself -- are run in a child process against the copy's library.  The child must
fail.  The unchanged source, run the same way, must pass.  All of this is CPU work."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "ff_oracle.cpp")
PIN_FILES = ["test_oracle_builder.py", "test_oracle_simulator.py", "test_oracle_links_devmap.py",
             "test_oracle_paramsync.py", "test_oracle_tuplecost.py", "test_oracle_training_graph.py"]

# (name, text in the source, replacement); every `text` occurs exactly once
MISTAKES = [
    ("partition bounds rounded up instead of down (Section 4, equal-size partitions)",
     "b.lo[d] = (int64_t)idx[d] * E / c.deg[d];\n        b.hi[d] = (int64_t)(idx[d] + 1) * E / c.deg[d];",
     "b.lo[d] = ((int64_t)idx[d] * E + c.deg[d] - 1) / c.deg[d];\n        b.hi[d] = ((int64_t)(idx[d] + 1) * E + c.deg[d] - 1) / c.deg[d];"),
    ("partition bounds rounded to nearest",
     "b.lo[d] = (int64_t)idx[d] * E / c.deg[d];\n        b.hi[d] = (int64_t)(idx[d] + 1) * E / c.deg[d];",
     "b.lo[d] = ((int64_t)idx[d] * E + c.deg[d] / 2) / c.deg[d];\n        b.hi[d] = ((int64_t)(idx[d] + 1) * E + c.deg[d] / 2) / c.deg[d];"),
    ("part index with dim 0 fastest instead of slowest",
     "for (int d = 3; d >= 0; d--) { idx[d] = rem % c.deg[d]; rem /= c.deg[d]; }\n    for (int d = 0; d < 4; d++) {\n        int64_t E",
     "for (int d = 0; d < 4; d++) { idx[d] = rem % c.deg[d]; rem /= c.deg[d]; }\n    for (int d = 0; d < 4; d++) {\n        int64_t E"),
    ("window offsets a and b swapped",
     "need_lo = driving.lo[m.src_dim] * (int64_t)m.stride + m.a;\n            need_hi = (driving.hi[m.src_dim] - 1) * (int64_t)m.stride + m.b + 1;",
     "need_lo = driving.lo[m.src_dim] * (int64_t)m.stride + m.b;\n            need_hi = (driving.hi[m.src_dim] - 1) * (int64_t)m.stride + m.a + 1;"),
    ("window end without its + 1",
     "(int64_t)m.stride + m.b + 1;", "(int64_t)m.stride + m.b;"),
    ("window stride dropped",
     "need_lo = driving.lo[m.src_dim] * (int64_t)m.stride + m.a;\n            need_hi = (driving.hi[m.src_dim] - 1) * (int64_t)m.stride + m.b + 1;",
     "need_lo = driving.lo[m.src_dim] + m.a;\n            need_hi = (driving.hi[m.src_dim] - 1) + m.b + 1;"),
    ("needed range not clamped to the producer's extent, shared volume counted outside the producer part",
     "int64_t lo = std::max(need_lo, owning.lo[d]), hi = std::min(need_hi, owning.hi[d]);",
     "int64_t lo = std::max(need_lo, owning.lo[d]), hi = need_hi;"),
    ("pairs enumerated consumer part first",
     "for (uint32_t kp = 0; kp < np[i]; kp++) {\n                Box pb = part_box(ops[i], cfg[i], kp);\n                for (uint32_t kc = 0; kc < np[j]; kc++) {\n                    Box cb = part_box(ops[j], cfg[j], kc);",
     "for (uint32_t kc = 0; kc < np[j]; kc++) {\n                Box cb = part_box(ops[j], cfg[j], kc);\n                for (uint32_t kp = 0; kp < np[i]; kp++) {\n                    Box pb = part_box(ops[i], cfg[i], kp);"),
    ("link row inside a node transposed",
     "return D + na * G * G + (from % G) * G + (to % G);", "return D + na * G * G + (to % G) * G + (from % G);"),
    ("link row between nodes transposed",
     "return D + N * G * G + na * N + nb;", "return D + N * G * G + nb * N + na;"),
    ("one link per GPU pair between nodes instead of one per node pair",
     "return D + N * G * G + na * N + nb;", "return D + N * G * G + (na * N + nb + from + to) % (N * N);"),
    ("bandwidth classes swapped",
     "uint64_t bw = same_node ? m.intra_Bpns : m.inter_Bpns;", "uint64_t bw = same_node ? m.inter_Bpns : m.intra_Bpns;"),
    ("latency classes swapped",
     "uint64_t lat = same_node ? m.intra_lat_ns : m.inter_lat_ns;", "uint64_t lat = same_node ? m.inter_lat_ns : m.intra_lat_ns;"),
    ("transfer time rounded down",
     "return (bytes + bw - 1) / bw + lat;", "return bytes / bw + lat;"),
    ("latency dropped",
     "return (bytes + bw - 1) / bw + lat;", "return (bytes + bw - 1) / bw;"),
    ("element size dropped",
     "transfer_ns(m, x, tg.dev[tp], tg.dev[tc], elems * m.elem_bytes)", "transfer_ns(m, x, tg.dev[tp], tg.dev[tc], elems)"),
    ("cost column off by one",
     "*out = cm.table[(size_t)i * cm.n_cols + (parts - 1)];", "*out = cm.table[(size_t)i * cm.n_cols + (parts > 1 ? parts - 2 : 0)];"),
    ("device stride dropped",
     "(cfg[i].dev_offset + (uint64_t)k * cfg[i].dev_stride) % D", "(cfg[i].dev_offset + (uint64_t)k) % D"),
    ("device index not wrapped around",
     "(cfg[i].dev_offset + (uint64_t)k * cfg[i].dev_stride) % D", "std::min<uint64_t>(cfg[i].dev_offset + (uint64_t)k * cfg[i].dev_stride, D - 1)"),
    ("tasks on one device still get a transfer",
     "if (tg.dev[tp] == tg.dev[tc]) { tg.add_dep(tp, tc); continue; }", "if (false) { tg.add_dep(tp, tc); continue; }"),
    ("transfers never created",
     "if (tg.dev[tp] == tg.dev[tc]) { tg.add_dep(tp, tc); continue; }", "if (true) { tg.add_dep(tp, tc); continue; }"),
    ("equal readyTimes dequeued highest id first",
     "const uint32_t t = ready_queue.begin()->second;\n        ready_queue.erase(ready_queue.begin());",
     "auto head = ready_queue.begin();\n        while (std::next(head) != ready_queue.end() && std::next(head)->first == ready_queue.begin()->first) ++head;\n"
     "        const uint32_t t = head->second;\n        ready_queue.erase(head);"),
    ("queue ordered by id alone",
     "ready_queue.emplace(ready_time[succ], succ);", "ready_queue.emplace(0, succ);"),
    ("readyTime is the last predecessor's end, not the largest",
     "ready_time[succ] = std::max(ready_time[succ], end_time[t]);", "ready_time[succ] = end_time[t];"),
    ("a task starts without waiting for its device",
     "start_time[t] = std::max(ready_time[t], busy_until);", "start_time[t] = ready_time[t];"),
    ("a task starts without waiting for its inputs",
     "start_time[t] = std::max(ready_time[t], busy_until);", "start_time[t] = busy_until;"),
    ("a task becomes READY after its first predecessor",
     "if (++complete_preds[succ] == tg.n_in[succ]) {", "if (++complete_preds[succ] == 1) {"),
    ("parameter shards rounded down",
     "const uint64_t shard_bytes = ((uint64_t)x.param_bytes[i] + shards - 1) / shards;", "const uint64_t shard_bytes = (uint64_t)x.param_bytes[i] / shards;"),
    ("shard owner taken along the wrong dims",
     "owner = owner * c.deg[d] + (((x.param_dims[i] >> d) & 1) ? idx[d] : 0);", "owner = owner * c.deg[d] + (((x.param_dims[i] >> d) & 1) ? 0 : idx[d]);"),
    ("link table indexed by (to, from)",
     "const size_t pair = (size_t)(from % G) * G + to % G;", "const size_t pair = (size_t)(to % G) * G + from % G;"),
    ("node link table indexed by (to, from)",
     "const size_t pair = (size_t)(from / G) * m.n_nodes + to / G;", "const size_t pair = (size_t)(to / G) * m.n_nodes + from / G;"),
    ("node link table ignored",
     "if (!same_node && x.node_bw) {", "if (false && x.node_bw) {"),
    ("node link table used inside a node as well",
     "if (!same_node && x.node_bw) {", "if (x.node_bw) {"),
    ("a contributing edge treated as a reading edge",
     "const bool contributes = e.map[0].kind != 0;", "const bool contributes = false;"),
    ("a contributing edge with the boxes of a reading edge",
     "const Box& owning = contributes ? cb : pb;", "const Box& owning = pb;"),
    ("a contributing edge whose ranges are taken in the producer's tensor",
     "const Op& space = contributes ? cons : prod;", "const Op& space = prod;"),
    ("tied configurations ignored",
     "tied[i] = cfg[x.leader[i]];", "tied[i] = cfg[i];"),
    ("explicit device map ignored",
     "dev = x.devmap[(size_t)i * MAX_PARTS + k];", "dev = dev;"),
    ("tuple cost list: first entry of the op instead of the matching one",
     "if (cm.tuples[t] == key) { *out = cm.tuple_ns[t]; return true; }", "{ *out = cm.tuple_ns[t]; return true; }"),
]


def run_pins(lib_path):
    """the pin tests in a child process against the given oracle library; returns the exit status"""
    env = dict(os.environ, FF_ORACLE_LIB=lib_path)
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + [os.path.join(ROOT, "tests", f) for f in PIN_FILES]
    try:
        return subprocess.run(cmd, env=env, cwd=ROOT, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL, timeout=300).returncode
    except subprocess.TimeoutExpired:
        return -1          # a mistake that makes the oracle spin is caught as well


def test_every_mistake_text_occurs_exactly_once():
    src = open(SRC).read()
    for name, old, new in MISTAKES:
        assert src.count(old) == 1, name
        assert old != new


def test_the_unchanged_oracle_passes_its_pins_in_a_child_process(tmp_path):
    lib = str(tmp_path / "libunchanged.so")
    oracle.compile_oracle(SRC, lib)
    assert run_pins(lib) == 0


def test_every_planted_mistake_fails_a_pin(tmp_path):
    src = open(SRC).read()

    def one(k):
        name, old, new = MISTAKES[k]
        path = str(tmp_path / f"mistake_{k}.cpp")
        lib = str(tmp_path / f"libmistake_{k}.so")
        with open(path, "w") as f:
            f.write(src.replace(old, new))
        oracle.compile_oracle(path, lib)
        return name, run_pins(lib)

    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(one, range(len(MISTAKES))))
    survived = [name for name, rc in results if rc == 0]
    assert not survived, "no pin notices: " + "; ".join(survived)
