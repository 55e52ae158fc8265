"""GPU parity of the on-device search loop (ff_sim_search) against the search oracle: the same
proposals, the same acceptance decisions, the same times after every step, bit for bit."""
import numpy as np
import pytest

import oracle
from oracle import search as S
from paper_1807_05358_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_1807_05358_amd import binding
    return binding


def _run_both(B, config_id, C, calls, beta_rel, seed, n_buckets=64, ahead=0):
    """beta_rel: beta * (start time of chain 0); the bucket is 1/256 of that time."""
    w = W.workload(config_id)
    sim = B.Simulator(w.ops, w.edges, w.machine, w.cost)
    cfg0 = w.strategies(C)
    tp, tu = w.search_space()
    t0 = int(oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cfg0[:1])[0])
    bucket = max(1, t0 // 256)
    table = S.metropolis_table(beta_rel / t0, bucket, n_buckets)
    ch = B.Chains(sim, cfg0)
    ch.search_setup(tp, tu, table, bucket, seed)
    got = np.concatenate([ch.search(n, ahead=ahead).cpu().numpy().view("<u8") for n in calls])
    best_ns, best = ch.best()
    n_acc_total = 0
    for c in range(C):
        print(f"search: config {config_id} chain {c}", flush=True)
        tr, cur, want_best_ns, want_best, n_acc = S.metropolis_chain(
            w.ops, w.edges, w.machine, w.cost, cfg0[c], tp, tu, table, bucket, seed, c, 0, sum(calls))
        bad = np.nonzero(got[:, c] != tr)[0]
        assert len(bad) == 0, f"chain {c}: first differing step {bad[0]}: gpu {got[bad[0], c]} oracle {tr[bad[0]]}"
        assert int(best_ns[c]) == want_best_ns
        assert np.array_equal(best[c], want_best)
        n_acc_total += n_acc
    st = ch.stats()
    ch.close()
    sim.close()
    return got, n_acc_total, st


@pytest.mark.parametrize("config_id,C,calls,beta_rel", [
    (0, 4, (40, 25), 20.0),
    (1, 6, (50, 30), 40.0),
    (2, 3, (14, 10), 60.0),
    (3, 2, (12,), 60.0),
    (4, 1, (6,), 100.0),
])
def test_search_matches_oracle(B, config_id, C, calls, beta_rel):
    got, n_acc, st = _run_both(B, config_id, C, calls, beta_rel, seed=4242 + config_id)
    n = sum(calls) * C
    print(f"accepted {n_acc} of {n} proposals; resumed {int(st['n_resumed'].sum())} recorded runs", flush=True)
    assert n_acc > 0
    if n >= 24:
        assert n_acc < n      # the case exercises both outcomes


@pytest.mark.parametrize("config_id,C,calls,beta_rel,ahead", [
    (0, 4, (40, 25), 20.0, 1),
    (0, 4, (40, 25), 20.0, 7),
    (1, 6, (50, 30), 40.0, 3),
    (1, 2, (81,), 40.0, 500),
    (2, 3, (14, 10), 60.0, 5),
    (3, 2, (12,), 60.0, 16),
    (4, 1, (6,), 100.0, 4),
])
def test_search_ahead_matches_oracle(B, config_id, C, calls, beta_rel, ahead):
    """ff_sim_search_ahead: proposals of the coming steps simulated side by side, the same chain step for step
    (Sections 6.1, 6.2: a proposal does not depend on the current strategy, a rejection leaves it unchanged)"""
    got, n_acc, st = _run_both(B, config_id, C, calls, beta_rel, seed=4242 + config_id, ahead=ahead | B.FF_AHEAD_ALWAYS)
    assert n_acc > 0
    if config_id <= 2:      # and with the call deciding by itself when to simulate ahead
        again, _, _ = _run_both(B, config_id, C, calls, beta_rel, seed=4242 + config_id, ahead=ahead)
        assert np.array_equal(got, again)


def test_search_ahead_equals_search_over_a_long_run(B):
    """the two entry points on 600 steps with a stopping rule that strikes on the way, continued by 40 steps of the
    other kind: traces, best times and best strategies agree"""
    w = W.workload(1)
    sim = B.Simulator(w.ops, w.edges, w.machine, w.cost)
    cfg0 = w.strategies(3)
    tp, tu = w.search_space()
    t0 = int(oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cfg0[:1])[0])
    bucket = max(1, t0 // 256)
    table = B.ff_sim_accept_table(120.0 / t0, bucket, 64)
    out = []
    for first, second in ((0, 200), (200, 0)):
        ch = B.Chains(sim, cfg0)
        ch.search_setup(tp, tu, table, bucket, 77, patience=150)
        a = ch.search(600, ahead=first).cpu().numpy().view("<u8")
        if first:
            rounds, simulated, steps, accepted = ch.ahead_stats
            assert steps == 600 * 3 and rounds < 600 and simulated >= steps
            print(f"look-ahead: {rounds} rounds, {simulated} proposals simulated for {steps} steps", flush=True)
        b = ch.search(40, ahead=second).cpu().numpy().view("<u8")
        out.append((np.concatenate([a, b]),) + ch.best())
        ch.close()
    assert np.array_equal(out[0][0], out[1][0])
    assert np.array_equal(out[0][1], out[1][1]) and np.array_equal(out[0][2], out[1][2])
    assert len(np.unique(out[0][0][:, 0])) > 5                        # the chains did move
    sim.close()


def test_search_ahead_argument_errors(B):
    torch = pytest.importorskip("torch")
    w = W.workload(1)
    sim = B.Simulator(w.ops, w.edges, w.machine, w.cost)
    ch = B.Chains(sim, w.strategies(2))
    tp, tu = w.search_space()
    ch.search_setup(tp, tu, np.full(4, 1000, np.uint32), 1000, 5)
    sp = ch._sp
    p = B.ff_search_t(sp["seed"], 0, sp["bucket_ns"], 0, sp["n_buckets"], sp["n_tuples"], sp["accept"].data_ptr(),
                      sp["tuple_ptr"].data_ptr(), sp["tuples"].data_ptr(), sp["best_ns"].data_ptr(), sp["best"].data_ptr())
    trace = torch.empty((8, 2), dtype=torch.int64, device="cuda")
    with pytest.raises(B.FFSimError) as e:
        B.ff_sim_search_ahead(ch.handle, p, 8, 0, trace.data_ptr())
    assert e.value.code == B.FF_EINVAL
    B.ff_sim_set_workspace(sim.handle, None, 0)
    with pytest.raises(B.FFSimError) as e:
        B.ff_sim_search_ahead(ch.handle, p, 8, 4, trace.data_ptr())
    assert e.value.code == B.FF_EWORKSPACE
    assert B.ff_sim_search_ahead(ch.handle, p, 0, 4, None) == (0, 0, 0, 0)
    ch.close()
    sim.close()


def test_pure_descent_and_always_accept(B):
    w = W.workload(1)
    sim = B.Simulator(w.ops, w.edges, w.machine, w.cost)
    cfg0 = w.strategies(3)
    tp, tu = w.search_space()
    for table in (np.zeros(2, np.uint32), np.full(2, 2 ** 32 - 1, np.uint32)):
        ch = B.Chains(sim, cfg0)
        ch.search_setup(tp, tu, table, 1000, 11)
        got = ch.search(40).cpu().numpy().view("<u8")
        for c in range(3):
            tr = S.metropolis_chain(w.ops, w.edges, w.machine, w.cost, cfg0[c], tp, tu, table, 1000, 11, c, 0, 40)[0]
            assert np.array_equal(got[:, c], tr)
        if table[0] == 0:
            assert np.all(np.diff(got.astype(np.int64), axis=0) <= 0)
        ch.close()
    sim.close()


def test_search_then_forced_mutations_then_search(B):
    """the three ways of stepping a chain share its state: a search, forced mutations
    (ff_sim_delta), trial proposals (ff_sim_delta_try) and a search again."""
    w = W.workload(2)
    sim = B.Simulator(w.ops, w.edges, w.machine, w.cost)
    cfg0 = w.strategies(2)
    tp, tu = w.search_space()
    t0 = int(oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cfg0[:1])[0])
    bucket = t0 // 128
    table = S.metropolis_table(30.0 / t0, bucket, 32)
    ch = B.Chains(sim, cfg0)
    ch.search_setup(tp, tu, table, bucket, 99)
    got1 = ch.search(8).cpu().numpy().view("<u8")
    muts = w.mutations(3, 2)
    got2 = ch.delta(ch.upload_mutations(muts), 3).cpu().numpy().view("<u8")
    props = w.mutations(7, 2)[3:]
    got3 = ch.try_mutations(ch.upload_mutations(props), 4).cpu().numpy().view("<u8")
    got4 = ch.search(6).cpu().numpy().view("<u8")
    for c in range(2):
        a = S.metropolis_chain(w.ops, w.edges, w.machine, w.cost, cfg0[c], tp, tu, table, bucket, 99, c, 0, 8)
        assert np.array_equal(got1[:, c], a[0])
        cur = a[1].copy()
        want2 = oracle.simulate_delta_chain(w.ops, w.edges, w.machine, w.cost, cur, muts[:, c])
        assert np.array_equal(got2[:, c], want2)
        for s in range(3):
            cur[int(muts[s, c]["op"])] = muts[s, c]["cfg"]
        cand = np.repeat(cur[None], 4, 0)
        for p in range(4):
            cand[p, int(props[p, c]["op"])] = props[p, c]["cfg"]
        assert np.array_equal(got3[:, c], oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cand))
        b = S.metropolis_chain(w.ops, w.edges, w.machine, w.cost, cur, tp, tu, table, bucket, 99, c, 8, 6)
        assert np.array_equal(got4[:, c], b[0])
    ch.close()
    sim.close()


def test_search_argument_errors(B):
    import torch
    w = W.workload(0)
    sim = B.Simulator(w.ops, w.edges, w.machine, w.cost)
    ch = B.Chains(sim, w.strategies(2))
    tp, tu = w.search_space()
    ch.search_setup(tp, tu, np.zeros(2, np.uint32), 10, 1)
    L = B.lib()
    sp = ch._sp
    out = torch.empty((2, 2), dtype=torch.int64, device="cuda")

    def params(**kw):
        d = dict(seed=1, first_step=0, bucket_ns=10, n_buckets=2, n_tuples=len(tu), d_accept=sp["accept"].data_ptr(),
                 d_tuple_ptr=sp["tuple_ptr"].data_ptr(), d_tuples=sp["tuples"].data_ptr(),
                 d_best_ns=sp["best_ns"].data_ptr(), d_best=sp["best"].data_ptr())
        d.update(kw)
        return B.ff_search_t(**d)

    import ctypes
    assert L.ff_sim_search(ch.handle, None, 2, out.data_ptr(), None) == B.FF_EINVAL
    assert L.ff_sim_search(None, ctypes.byref(params()), 2, out.data_ptr(), None) == B.FF_EINVAL
    assert L.ff_sim_search(ch.handle, ctypes.byref(params()), 2, None, None) == B.FF_EINVAL
    assert L.ff_sim_search(ch.handle, ctypes.byref(params(bucket_ns=0)), 2, out.data_ptr(), None) == B.FF_EINVAL
    assert L.ff_sim_search(ch.handle, ctypes.byref(params(n_buckets=0)), 2, out.data_ptr(), None) == B.FF_EINVAL
    assert L.ff_sim_search(ch.handle, ctypes.byref(params(d_accept=None)), 2, out.data_ptr(), None) == B.FF_EINVAL
    # a list that reaches beyond the tuples handed over is refused before anything is launched
    assert L.ff_sim_search(ch.handle, ctypes.byref(params(n_tuples=len(tu) - 1)), 2, out.data_ptr(), None) == B.FF_EINVAL
    assert L.ff_sim_search(ch.handle, ctypes.byref(params()), 0, None, None) == B.FF_OK
    assert L.ff_sim_search(ch.handle, ctypes.byref(params()), 2, out.data_ptr(), None) == B.FF_OK
    torch.cuda.synchronize()
    ch.close()
    sim.close()


@pytest.mark.parametrize("config_id,C,ops_range", [(0, 3, None), (1, 2, None), (2, 1, (118, 121))])
def test_neighbour_sweep_matches_oracle(B, config_id, C, ops_range):
    """Section 8.4's local-optimality check: every strategy that differs from the chain's in one
    op's configuration, each equal to a full simulation by the oracle; the list is enumerated
    here independently (ops, then tuples in list order, then device offsets)."""
    w = W.workload(config_id)
    sim = B.Simulator(w.ops, w.edges, w.machine, w.cost)
    cfg0 = w.strategies(C)
    ch = B.Chains(sim, cfg0)
    warm = w.mutations(3, C)
    ch.delta(ch.upload_mutations(warm), 3)
    cur = cfg0.copy()
    for s in range(3):
        for c in range(C):
            cur[c, int(warm[s, c]["op"])] = warm[s, c]["cfg"]
    tp, tu = w.search_space()
    ob, oe = ops_range if ops_range else (0, w.n_ops)
    muts, got, best_ns, best_idx = ch.neighbours(tp, tu, ob, oe)
    want_list = [(op, int(tu[t]), off) for op in range(ob, oe) for t in range(tp[op], tp[op + 1])
                 for off in range(w.machine.n_devices)]
    M = len(want_list)
    assert muts.shape == (M, C) and got.shape == (M, C)
    print(f"neighbours: config {config_id}, {M} per chain", flush=True)
    for c in range(C):
        assert [int(x) for x in muts[:, c]["op"]] == [m[0] for m in want_list]
        deg = muts[:, c]["cfg"]["deg"].astype(np.uint32)
        assert np.array_equal(deg[:, 0] | (deg[:, 1] << 8) | (deg[:, 2] << 16) | (deg[:, 3] << 24),
                              np.array([m[1] for m in want_list], np.uint32))
        assert [int(x) for x in muts[:, c]["cfg"]["dev_offset"]] == [m[2] for m in want_list]
        assert np.all(muts[:, c]["cfg"]["dev_stride"] == 1)
        cand = np.repeat(cur[c][None], M, 0)
        for k in range(M):
            cand[k, int(muts[k, c]["op"])] = muts[k, c]["cfg"]
        want = oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cand, n_threads=8)
        bad = np.nonzero(got[:, c] != want)[0]
        assert len(bad) == 0, f"chain {c}: neighbours {bad[:5]} gpu {got[bad[:5], c]} oracle {want[bad[:5]]}"
        assert int(best_ns[c]) == int(want.min()) and int(best_idx[c]) == int(np.argmin(want))
        # the current strategy is its own neighbour: never better than the best
        own = int(oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cur[c][None])[0])
        assert int(best_ns[c]) <= own
    # the chains were only read
    more = w.mutations(5, C)[3:]
    after = ch.delta(ch.upload_mutations(more), 2).cpu().numpy().view("<u8")
    for c in range(C):
        assert np.array_equal(after[:, c], oracle.simulate_delta_chain(w.ops, w.edges, w.machine, w.cost, cur[c], more[:, c]))
    ch.close()
    sim.close()


def test_neighbour_sweep_argument_errors(B):
    import torch
    w = W.workload(0)
    sim = B.Simulator(w.ops, w.edges, w.machine, w.cost)
    ch = B.Chains(sim, w.strategies(1))
    tp, tu = w.search_space()
    d_ptr, d_tu = B.to_device(tp), B.to_device(tu)
    assert B.ff_sim_neighbour_count(ch.handle, d_ptr.data_ptr(), len(tu), 0, w.n_ops) == len(tu) * w.machine.n_devices
    assert B.ff_sim_neighbour_count(ch.handle, d_ptr.data_ptr(), len(tu), 2, 2) == 0
    import ctypes
    n = ctypes.c_uint32()
    L = B.lib()
    assert L.ff_sim_neighbour_count(ch.handle, d_ptr.data_ptr(), len(tu), 3, 2, ctypes.byref(n)) == B.FF_EINVAL
    assert L.ff_sim_neighbour_count(ch.handle, d_ptr.data_ptr(), len(tu), 0, w.n_ops + 1, ctypes.byref(n)) == B.FF_EINVAL
    assert L.ff_sim_neighbour_count(ch.handle, d_ptr.data_ptr(), len(tu) - 1, 0, w.n_ops, ctypes.byref(n)) == B.FF_EINVAL
    assert L.ff_sim_neighbour_count(ch.handle, None, len(tu), 0, w.n_ops, ctypes.byref(n)) == B.FF_EINVAL
    assert L.ff_sim_neighbours(ch.handle, d_ptr.data_ptr(), d_tu.data_ptr(), len(tu), 0, w.n_ops, None, None, None, None, None) == B.FF_EINVAL
    torch.cuda.synchronize()
    ch.close()
    sim.close()


def test_search_stopping_rule(B):
    """patience: chains stop proposing after that many steps without a new best; the count and
    the best so far carry over between calls."""
    w = W.workload(1)
    sim = B.Simulator(w.ops, w.edges, w.machine, w.cost)
    C = 5
    cfg0 = w.strategies(C)
    tp, tu = w.search_space()
    table = S.metropolis_table(40.0 / 4.0e7, 150000, 64)
    ch = B.Chains(sim, cfg0)
    ch.search_setup(tp, tu, table, 150000, 21, patience=7)
    got = np.concatenate([ch.search(n).cpu().numpy().view("<u8") for n in (30, 50)])
    stopped = 0
    for c in range(C):
        a = S.metropolis_chain(w.ops, w.edges, w.machine, w.cost, cfg0[c], tp, tu, table, 150000, 21, c, 0, 80, patience=7)
        assert np.array_equal(got[:, c], a[0]), f"chain {c}: step {np.nonzero(got[:, c] != a[0])[0][:3]}"
        stopped += int(np.all(a[0][-8:] == a[0][-1]))
    assert stopped == C           # with patience 7 every chain has come to rest within 80 steps
    best_ns, _ = ch.best()
    assert np.array_equal(best_ns, got.min(axis=0).clip(max=ch.start_ns()))
    ch.close()
    sim.close()


def test_search_driver_matches_the_oracle_chain_by_chain(B):
    """paper_1807_05358_amd.search.find_strategy: starting points, table and budget rule are its own;
    every chain it runs must be the oracle's chain for the same inputs, and the result the best of them"""
    from paper_1807_05358_amd import search as driver
    w = W.workload(1)
    sim = B.Simulator(w.ops, w.edges, w.machine, w.cost)
    C, steps, seed = 6, 24, 5
    res = driver.find_strategy(sim, w.ops, w.machine, w.max_parts, w.choices, n_chains=C, steps=steps, steps_per_call=10, seed=seed)
    cfg0 = driver.starting_strategies(w.ops, w.machine, w.max_parts, w.choices, C, seed)
    assert np.array_equal(cfg0[0], W.data_parallel_strategy(w.ops, w.machine.n_devices, w.max_parts))
    start = oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cfg0)
    assert np.array_equal(res.start_ns, start)
    ref = float(np.median(start))
    scale = 0.25 / len(w.ops)                      # the driver's default tolerance: a quarter of one op's share of the time
    bucket = max(1, int(ref * scale * 8 / 256))
    table = S.metropolis_table(1.0 / (ref * scale), bucket, 256)
    assert np.array_equal(table, B.ff_sim_accept_table(1.0 / (ref * scale), bucket, 256))
    tp, tu = w.search_space()
    best = []
    for c in range(C):
        trace, _, best_ns, best_cfg, _ = S.metropolis_chain(w.ops, w.edges, w.machine, w.cost, cfg0[c], tp, tu, table, bucket,
                                                                  seed, c, 0, steps, patience=steps // 2)
        assert np.array_equal(res.trace_ns[:, c], trace), f"chain {c}"
        assert int(res.chain_best_ns[c]) == best_ns
        best.append(best_ns)
    assert res.best_ns == min(best) <= int(start.min())
    assert int(oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, res.best[None])[0]) == res.best_ns
    sim.close()
