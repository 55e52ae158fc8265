"""Pins of the search oracle (oracle/search.py): the generator against published SplitMix64
outputs and against the input generators' own implementation, the acceptance table against
the closed form, and the Metropolis rule of Section 6.1 against the stationary distribution
it must produce on a two-state problem."""
import math

import numpy as np

import oracle
from oracle import search as S
from paper_1807_05358_amd import workloads as W


def test_mix64_is_the_splitmix64_output_function():
    # first two outputs of SplitMix64 seeded with 0 (the generator's published test values)
    assert S.mix64(0) == 0xE220A8397B1DCDAF
    assert S.mix64(0x9E3779B97F4A7C15) == 0x6E789E6AA1B965F4


def test_draw_agrees_with_the_input_generators():
    rng = np.random.default_rng(5)
    for _ in range(50):
        seed, p, c, s = (int(x) for x in rng.integers(0, 2 ** 62, 4))
        assert S.draw(seed, p, c, s) == int(W._draw(seed, p, c, s))


def test_metropolis_table_closed_form():
    t = S.metropolis_table(1e-3, 100, 64)
    assert t[0] == 2 ** 32 - 1
    assert all(t[i] >= t[i + 1] for i in range(63))
    for b in (1, 7, 40):
        assert abs(int(t[b]) / 2 ** 32 - math.exp(-0.1 * b)) < 1e-9
    assert np.all(S.metropolis_table(0.0, 100, 4) == 2 ** 32 - 1)


def _two_state():
    """one op (extent 4, splittable), one device: 1 part costs 1000 ns; 2 parts run one after
    the other on the only device and cost 2 * 700 = 1400 ns."""
    ops = np.zeros(1, W.OP_DT)
    ops[0]["ndim"], ops[0]["par_mask"] = 1, 1
    ops[0]["extent"] = (4, 1, 1, 1)
    edges = np.zeros(0, W.EDGE_DT)
    mach = W.Machine(1, 1)
    cost = np.full((1, 2), 1000, np.uint32)
    cost[0, 1] = 700
    cfg = np.zeros(1, W.CFG_DT)
    cfg["deg"] = 1
    cfg["dev_stride"] = 1
    tuple_ptr = np.array([0, 2], np.uint32)
    tuples = np.array([0x01010101, 0x01010102], np.uint32)
    return ops, edges, mach, cost, cfg, tuple_ptr, tuples


def test_two_state_costs():
    ops, edges, mach, cost, cfg, _, _ = _two_state()
    two = cfg.copy()
    two["deg"][0, 0] = 2
    assert list(oracle.simulate_batch(ops, edges, mach, cost, np.stack([cfg, two]))) == [1000, 1400]


def test_metropolis_rule_reaches_its_stationary_distribution():
    """symmetric proposals + acceptance min(1, exp(-beta*delta)) => the chain visits the slow
    state exp(-beta*delta) times as often as the fast one (detailed balance)."""
    ops, edges, mach, cost, cfg, tp, tu = _two_state()
    beta = math.log(4.0) / 400.0                  # exp(-beta * 400 ns) = 1/4
    table = S.metropolis_table(beta, 100, 8)
    assert abs(int(table[4]) / 2 ** 32 - 0.25) < 1e-9
    n = 6000
    trace, _, best_ns, best, n_acc = S.metropolis_chain(ops, edges, mach, cost, cfg, tp, tu, table, 100, 77, 0, 0, n)
    slow = float(np.mean(trace == 1400))
    assert set(np.unique(trace)) == {1000, 1400}
    assert abs(slow - 0.2) < 0.03, slow           # pi_slow = 0.25 / (1 + 0.25)
    assert best_ns == 1000 and best[0]["deg"][0] == 1
    # the same chain with the sign of the exponent flipped would sit in the slow state 80 % of
    # the time; with always-accept, 50 %
    always = np.full(8, 2 ** 32 - 1, np.uint32)
    t2 = S.metropolis_chain(ops, edges, mach, cost, cfg, tp, tu, always, 100, 77, 0, 0, n)[0]
    assert abs(float(np.mean(t2 == 1400)) - 0.5) < 0.03


def test_zero_table_is_descent_and_full_table_accepts_every_valid_proposal():
    w = W.workload(1)
    tp, tu = w.search_space()
    cfg0 = w.strategies(1)[0]
    never = np.zeros(4, np.uint32)
    tr, cur, best_ns, best, _ = S.metropolis_chain(w.ops, w.edges, w.machine, w.cost, cfg0, tp, tu, never, 1000, 3, 0, 0, 60)
    assert np.all(np.diff(tr.astype(np.int64)) <= 0)
    assert best_ns == tr[-1] and np.array_equal(best, cur)
    assert int(oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cur[None])[0]) == tr[-1]
    always = np.full(4, 2 ** 32 - 1, np.uint32)
    tr2, cur2, best2, _, n_acc = S.metropolis_chain(w.ops, w.edges, w.machine, w.cost, cfg0, tp, tu, always, 1000, 3, 0, 0, 60)
    assert n_acc == 60            # every proposal from the op's own list is valid
    assert int(oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cur2[None])[0]) == tr2[-1]
    assert best2 == min(int(tr2.min()), int(oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cfg0[None])[0]))


def test_steps_continue_across_calls():
    w = W.workload(0)
    tp, tu = w.search_space()
    cfg0 = w.strategies(1)[0]
    table = S.metropolis_table(1e-5, 1000, 32)
    whole = S.metropolis_chain(w.ops, w.edges, w.machine, w.cost, cfg0, tp, tu, table, 1000, 9, 2, 0, 30)
    a = S.metropolis_chain(w.ops, w.edges, w.machine, w.cost, cfg0, tp, tu, table, 1000, 9, 2, 0, 12)
    b = S.metropolis_chain(w.ops, w.edges, w.machine, w.cost, a[1], tp, tu, table, 1000, 9, 2, 12, 18)
    assert np.array_equal(whole[0], np.concatenate([a[0], b[0]]))
    assert np.array_equal(whole[1], b[1])


def test_stopping_rule_freezes_the_chain_after_patience_steps_without_a_new_best():
    """Section 6.2: the search from one initial strategy ends when the best strategy has not
    improved for the given number of steps; until then it is the same chain."""
    w = W.workload(1)
    tp, tu = w.search_space()
    cfg0 = w.strategies(1)[0]
    table = S.metropolis_table(40.0 / 4.0e7, 150000, 64)
    free = S.metropolis_chain(w.ops, w.edges, w.machine, w.cost, cfg0, tp, tu, table, 150000, 21, 0, 0, 300)[0]
    for patience in (3, 10, 40):
        tr = S.metropolis_chain(w.ops, w.edges, w.machine, w.cost, cfg0, tp, tu, table, 150000, 21, 0, 0, 300,
                                patience=patience)[0]
        # running best of the unrestricted chain, with the start strategy counted
        start = int(oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cfg0[None])[0])
        best, idle, stop = start, 0, None
        for s in range(300):
            if idle >= patience:
                stop = s
                break
            idle += 1
            if free[s] < best:
                best, idle = int(free[s]), 0
        assert stop is not None and stop < 300
        assert np.array_equal(tr[:stop], free[:stop])
        assert np.all(tr[stop:] == tr[stop - 1])
