"""Long mutation chains (Section 5.3: after every change the delta result equals a full simulation of
the changed strategy).  The search of Section 6 runs chains of thousands of proposals: here the chain
state is driven through what only long chains reach -- the per-run tags of recorded endTimes starting
over after 65535 runs, snapshot places flipping thousands of times, repeated re-spacing of the
snapshots -- and checked against the oracle's full re-simulation."""
import numpy as np
import pytest

import oracle
from paper_1807_05358_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_1807_05358_amd import binding
    return binding


def oracle_steps(w, cfg0, muts, steps):
    """the oracle's times after the given steps of one chain (full re-simulation of each)."""
    cur = np.array(cfg0, copy=True)
    want = set(int(s) for s in steps)
    snaps = []
    for s in range(max(want) + 1):
        cur[int(muts[s]["op"])] = muts[s]["cfg"]
        if s in want:
            snaps.append(cur.copy())
    return oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, np.stack(snaps), n_threads=16)


def test_nmt_chain_of_1000_steps(B):
    """configs[4]: one chain, 1000 cumulative single-op mutations in four calls; 64 steps spread over
    the chain, the first, and the last are compared with the oracle."""
    w = W.workload(4)
    n_steps = 1000
    cfg0 = w.strategies(1)
    muts = w.mutations(n_steps, 1)
    sim = B.Simulator(w.ops, w.edges, w.machine, w.cost)
    ch = B.Chains(sim, cfg0)
    got = []
    for a in range(0, n_steps, 250):
        got.append(ch.delta(ch.upload_mutations(muts[a:a + 250]), 250).cpu().numpy().view("<u8"))
        print(f"nmt chain: {a + 250} steps done", flush=True)
    got = np.concatenate(got)[:, 0]
    sel = sorted(set(np.linspace(0, n_steps - 1, 64).astype(int).tolist()) | {0, 1, n_steps - 1})
    want = oracle_steps(w, cfg0[0], muts[:, 0], sel)
    bad = [s for s, v in zip(sel, want) if got[s] != v]
    assert not bad, f"first differing step {bad[0]} (op {int(muts[bad[0], 0]['op'])}): gpu {got[bad[0]]}"
    st = ch.stats()
    assert int(st["n_steps"][0]) == n_steps and int(st["n_resumed"][0]) > n_steps // 2
    ch.close()
    sim.close()


def test_nmt_256_chains_of_32_steps(B):
    """configs[4]: 256 independent chains side by side (the search starts from several initial
    strategies); every step of 8 of them, and the last step of 64 of them, is compared with the oracle."""
    w = W.workload(4)
    C, n_steps = 256, 32
    cfg0 = w.strategies(C)
    muts = w.mutations(n_steps, C)
    sim = B.Simulator(w.ops, w.edges, w.machine, w.cost)
    ch = B.Chains(sim, cfg0)
    assert np.array_equal(ch.start_ns()[::32], oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cfg0[::32], n_threads=16))
    got = ch.delta(ch.upload_mutations(muts), n_steps).cpu().numpy().view("<u8")
    for c in (0, 1, 37, 100, 128, 200, 254, 255):
        want = oracle_steps(w, cfg0[c], muts[:, c], range(n_steps))
        bad = np.nonzero(got[:, c] != want)[0]
        assert len(bad) == 0, f"chain {c}: first differing step {bad[0]}"
    last = np.array([oracle_steps(w, cfg0[c], muts[:, c], [n_steps - 1])[0] for c in range(0, C, 4)])
    assert np.array_equal(got[n_steps - 1, ::4], last)
    ch.close()
    sim.close()


@pytest.mark.parametrize("config_id,C,n_steps", [(0, 2, 70000), (1, 2, 66000)])
def test_run_tags_start_over(B, config_id, C, n_steps):
    """more recorded runs than the 16-bit tag of a recorded endTime can count: the tags start over
    (and what earlier runs wrote is forgotten) without a wrong endTime ever being taken for a
    current one.  Every step of every chain is compared with the oracle."""
    w = W.workload(config_id)
    cfg0 = w.strategies(C)
    muts = w.mutations(n_steps, C)
    sim = B.Simulator(w.ops, w.edges, w.machine, w.cost)
    ch = B.Chains(sim, cfg0)
    got = []
    for a in range(0, n_steps, 10000):
        n = min(10000, n_steps - a)
        got.append(ch.delta(ch.upload_mutations(muts[a:a + n]), n).cpu().numpy().view("<u8"))
    got = np.concatenate(got)
    for c in range(C):
        want = oracle_steps(w, cfg0[c], muts[:, c], range(n_steps))
        bad = np.nonzero(got[:, c] != want)[0]
        assert len(bad) == 0, f"chain {c}: first differing step {bad[0]} of {n_steps}"
    st = ch.stats()
    assert int(st["n_steps"].min()) == n_steps
    ch.close()
    sim.close()
