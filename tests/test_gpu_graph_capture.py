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
