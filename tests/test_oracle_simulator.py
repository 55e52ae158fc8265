"""Pins for the oracle's Algorithm 1 (full simulation) on hand-made task graphs:
hand-computed fixtures, brute force over processing orders, bounds, closed forms."""
import itertools

import numpy as np
import pytest

import oracle
from helpers import check_timeline, critical_path, load_golden


@pytest.mark.parametrize("name", ["sim_tie_by_id.json", "sim_fifo_by_ready.json"])
def test_hand_computed_timelines(golden_dir, name):
    g = load_golden(golden_dir, name)
    exe = [t[0] for t in g["tasks"]]
    dev = [t[1] for t in g["tasks"]]
    tg = oracle.task_graph_from_arrays(exe, dev, g["n_rows"], [d[0] for d in g["deps"]], [d[1] for d in g["deps"]])
    mk, ready, start, end = tg.simulate()
    assert mk == g["makespan"]
    assert ready.tolist() == g["ready"]
    assert start.tolist() == g["start"]
    assert end.tolist() == g["end"]


def random_dag(rng, n, n_rows, p_edge, max_exe):
    exe = rng.integers(1, max_exe + 1, n)
    dev = rng.integers(0, n_rows, n)
    src, dst = [], []
    for a in range(n):
        for b in range(a + 1, n):
            if rng.random() < p_edge:
                src.append(a)
                dst.append(b)
    perm = rng.permutation(n)   # ids are not topologically sorted in general
    src = [int(perm[a]) for a in src]
    dst = [int(perm[b]) for b in dst]
    return exe, dev, np.array(src, dtype=np.int64), np.array(dst, dtype=np.int64)


def run_in_order(order, exe, dev, n_rows, preds, succs):
    """apply Algorithm 1's per-task update (start/end/device, successors' readyTime) in a
    given global order; return (ready, start, end) or None if the order does not respect
    dependencies."""
    n = len(exe)
    ready = [0] * n
    start = [0] * n
    end = [0] * n
    done = [False] * n
    last = [0] * n_rows
    for t in order:
        if any(not done[p] for p in preds[t]):
            return None
        start[t] = max(ready[t], last[dev[t]])
        end[t] = start[t] + int(exe[t])
        last[dev[t]] = end[t]
        done[t] = True
        for s in succs[t]:
            ready[s] = max(ready[s], end[t])
    return ready, start, end


@pytest.mark.parametrize("seed", range(12))
def test_brute_force_over_processing_orders(seed):
    """every dependency-respecting global order whose (readyTime, id) sequence turns out
    non-decreasing is a legal run of Algorithm 1's queue; all of them must give the
    oracle's timeline.  Small exeTimes force many ties."""
    rng = np.random.default_rng(seed)
    n = 7
    exe, dev, src, dst = random_dag(rng, n, 3, 0.3, 3 if seed % 2 else 9)
    preds = [[int(a) for a, b in zip(src, dst) if b == t] for t in range(n)]
    succs = [[int(b) for a, b in zip(src, dst) if a == t] for t in range(n)]
    tg = oracle.task_graph_from_arrays(exe, dev, 3, src, dst)
    mk, ready, start, end = tg.simulate()
    kept = 0
    for order in itertools.permutations(range(n)):
        res = run_in_order(order, exe, dev, 3, preds, succs)
        if res is None:
            continue
        r, s, e = res
        keys = [(r[t], t) for t in order]
        if keys != sorted(keys):
            continue
        kept += 1
        assert r == ready.tolist() and s == start.tolist() and e == end.tolist()
        assert max(e) == mk
    assert kept >= 1


@pytest.mark.parametrize("seed", range(6))
def test_bounds_and_fixed_point_on_random_graphs(seed):
    rng = np.random.default_rng(100 + seed)
    n, rows = 400, 9
    exe, dev, src, dst = random_dag(rng, n, rows, 0.01, 50)
    tg = oracle.task_graph_from_arrays(exe, dev, rows, src, dst)
    mk, ready, start, end = tg.simulate()
    check_timeline(exe.astype(np.uint64), dev, src, dst, ready, start, end)
    assert mk == end.max()
    assert mk >= critical_path(exe, src, dst)                      # ready = max end of preds
    assert mk >= np.bincount(dev, weights=exe, minlength=rows).max()  # one task at a time per device
    assert mk <= exe.sum()                                         # A4: some device is always busy
    # scaling every exeTime by k scales the whole timeline by k
    mk3, r3, s3, e3 = oracle.task_graph_from_arrays(exe * 3, dev, rows, src, dst).simulate()
    assert mk3 == 3 * mk and np.array_equal(e3, 3 * end) and np.array_equal(s3, 3 * start)


def test_single_device_any_dag_is_sum_of_times():
    rng = np.random.default_rng(7)
    exe, dev, src, dst = random_dag(rng, 200, 1, 0.03, 1000)
    mk, *_ = oracle.task_graph_from_arrays(exe, np.zeros(200, int), 1, src, dst).simulate()
    assert mk == exe.sum()


def test_chain_across_devices_is_sum_of_times():
    exe = np.arange(1, 51) * 7
    src = np.arange(49)
    mk, ready, start, end = oracle.task_graph_from_arrays(exe, np.arange(50) % 5, 5, src, src + 1).simulate()
    assert mk == exe.sum()
    assert np.array_equal(start[1:], end[:-1])


def test_independent_tasks_fill_devices_in_id_order():
    # 6 source tasks, 2 devices, all ready at 0: each device runs its tasks in id order
    exe = np.array([5, 7, 11, 13, 17, 19])
    dev = np.array([0, 1, 0, 1, 0, 1])
    mk, ready, start, end = oracle.task_graph_from_arrays(exe, dev, 2, [], []).simulate()
    assert start.tolist() == [0, 0, 5, 7, 16, 20]
    assert mk == 39
