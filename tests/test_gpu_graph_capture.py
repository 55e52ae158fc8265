"""The launch paths of the boundary allocate nothing and clear their scratch with kernels, so a
caller can record them into a HIP graph: every replay must give what the eager calls give."""
import numpy as np
import pytest

import oracle
from paper_1807_05358_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_1807_05358_amd import binding
    return binding


@pytest.mark.parametrize("config_id,n", [(1, 256), (2, 64)])
def test_batch_in_a_graph(B, config_id, n):
    import torch
    w = W.workload(config_id)
    sim = B.Simulator(w.ops, w.edges, w.machine, w.cost)
    cfgs = w.strategies(2 * n)
    want = oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cfgs, n_threads=8)
    d_in = sim.upload_strategies(cfgs[:n])
    d_other = sim.upload_strategies(cfgs[n:])
    out = torch.zeros(n, dtype=torch.int64, device="cuda")
    sim.batch(d_in, n, d_out=out)                        # eager once: sizes the workspace outside the capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        sim.batch(d_in, n, d_out=out)
    for replay in range(3):
        out.zero_()
        d_in.copy_(d_other if replay == 1 else sim.upload_strategies(cfgs[:n]))     # the graph reads the buffer, not a copy
        g.replay()
        torch.cuda.synchronize()
        got = out.cpu().numpy().view("<u8")
        assert np.array_equal(got, want[n:] if replay == 1 else want[:n]), f"replay {replay}"
        # eager work of the program between the replays
        assert np.array_equal(sim.simulate(cfgs[n:n + 8]), want[n:n + 8])
    sim.close()


def test_delta_and_trial_mutations_in_a_graph(B):
    import torch
    w = W.workload(1)
    sim = B.Simulator(w.ops, w.edges, w.machine, w.cost)
    C, steps, M = 3, 4, 6
    cfg0 = w.strategies(C)
    muts = w.mutations(3 * steps, C)
    trial = w.mutations(M, C)[::-1].copy()
    eager = B.Chains(sim, cfg0)
    ch = B.Chains(sim, cfg0)
    d_m = ch.upload_mutations(muts[:steps])
    d_t = ch.upload_mutations(trial)
    out = torch.zeros((steps, C), dtype=torch.int64, device="cuda")
    tried = torch.zeros((M, C), dtype=torch.int64, device="cuda")
    ch.try_mutations(d_t, M, d_out=tried)                # eager once: sizes the workspace
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        ch.delta(d_m, steps, d_out=out)
        ch.try_mutations(d_t, M, d_out=tried)
    for replay in range(3):
        d_m.copy_(ch.upload_mutations(muts[replay * steps:(replay + 1) * steps]))
        g.replay()
        torch.cuda.synchronize()
        want = eager.delta(eager.upload_mutations(muts[replay * steps:(replay + 1) * steps]), steps).cpu().numpy().view("<u8")
        want_try = eager.try_mutations(eager.upload_mutations(trial), M).cpu().numpy().view("<u8")
        assert np.array_equal(out.cpu().numpy().view("<u8"), want), f"replay {replay}"
        assert np.array_equal(tried.cpu().numpy().view("<u8"), want_try), f"replay {replay} (trial mutations)"
    # and the eager chains agree with the oracle
    ref = oracle.simulate_delta_chain(w.ops, w.edges, w.machine, w.cost, cfg0[0], muts[:, 0], steps=[3 * steps - 1])
    assert int(want[-1, 0]) == int(ref[0])
    ch.close()
    eager.close()
    sim.close()


def test_search_steps_in_a_graph(B):
    """after one eager call (which checks the proposal lists) ff_sim_search only launches: a graph of
    search steps, replayed, continues the chains exactly as eager calls do"""
    import torch
    from oracle import search as S
    w = W.workload(1)
    sim = B.Simulator(w.ops, w.edges, w.machine, w.cost)
    C, n = 3, 5
    cfg0 = w.strategies(C)
    tp, tu = w.search_space()
    t0 = int(oracle.simulate_batch(w.ops, w.edges, w.machine, w.cost, cfg0[:1])[0])
    bucket = max(1, t0 // 256)
    table = B.ff_sim_accept_table(20.0 / t0, bucket, 64)
    ch = B.Chains(sim, cfg0)
    ch.search_setup(tp, tu, table, bucket, seed=4)
    trace = torch.zeros((n, C), dtype=torch.int64, device="cuda")
    got = [ch.search(n, d_trace=trace).cpu().numpy().view("<u8").copy()]      # eager: steps 0..n-1
    sp = ch._sp
    # the graph holds the call for steps n..2n-1; step numbers are an argument, so each replay repeats those draws:
    # the second replay proposes the same ops again from where the first one left the chains
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        ch.search(n, d_trace=trace)
    for replay in range(2):
        g.replay()
        torch.cuda.synchronize()
        got.append(trace.cpu().numpy().view("<u8").copy())
    for c in range(C):
        a = S.metropolis_chain(w.ops, w.edges, w.machine, w.cost, cfg0[c], tp, tu, table, bucket, 4, c, 0, n)
        assert np.array_equal(got[0][:, c], a[0])
        b1 = S.metropolis_chain(w.ops, w.edges, w.machine, w.cost, a[1], tp, tu, table, bucket, 4, c, n, n, best_so_far=a[2])
        assert np.array_equal(got[1][:, c], b1[0]), f"chain {c}, first replay"
        b2 = S.metropolis_chain(w.ops, w.edges, w.machine, w.cost, b1[1], tp, tu, table, bucket, 4, c, n, n,
                                best_so_far=min(a[2], b1[2]))
        assert np.array_equal(got[2][:, c], b2[0]), f"chain {c}, second replay"
    assert sp["step"] == 2 * n
    ch.close()
    sim.close()
