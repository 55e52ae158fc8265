"""Driver of the strategy search (Section 6) on top of the device-side search loop.

Everything that decides anything runs in the kernels behind ff_sim_search (proposal, delta
simulation, acceptance, best-so-far, stopping rule); this module only prepares the inputs the
way Section 6.2 describes them and calls it until the budget is spent:

* starting candidates: data parallelism and seeded random strategies, one per chain;
* budget: a number of steps per chain; a chain stops proposing once it has gone half of the
  budget without improving on its best strategy;
* acceptance: the Metropolis rule of Section 6.1 with beta chosen relative to the starting
  time (a proposal that is slower by `accept_scale` times the starting time is accepted with
  probability 1/e; default 0.25 / number of ops), tabulated for the integer rule the kernel applies.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

from . import binding as B
from . import workloads as W


@dataclass
class SearchResult:
    best_ns: int                 # simulated time of the best strategy found
    best: np.ndarray             # [n_ops] configurations (workloads.CFG_DT)
    start_ns: np.ndarray         # [C] time of every chain's starting strategy
    chain_best_ns: np.ndarray    # [C] best time per chain
    trace_ns: np.ndarray         # [steps][C] time of every chain's current strategy after each step
    steps: int
    seed: int


def starting_strategies(ops, machine, max_parts, choices, n_chains, seed):
    """chain 0 starts from data parallelism, the others from seeded random strategies."""
    cfgs = W.strategies(ops, n_chains, seed, machine.n_devices, max_parts, choices)
    cfgs[0] = W.data_parallel_strategy(ops, machine.n_devices, max_parts)
    return cfgs


def find_strategy(sim: B.Simulator, ops, machine, max_parts, choices, n_chains=64, steps=256, steps_per_call=64,
                  accept_scale=None, n_buckets=256, seed=1, start=None, ahead=0) -> SearchResult:
    """runs n_chains independent Markov chains for `steps` steps each and returns the best
    strategy any of them has seen.  `start`: [n_chains][n_ops] starting strategies (default: see
    starting_strategies).  `ahead`: with few chains, let ff_sim_search_ahead simulate up to that many
    proposals per chain side by side (the same chains, step for step; only faster)."""
    if accept_scale is None:
        # one op moves the iteration time by about its share of it: the tolerance follows the number of ops
        accept_scale = 0.25 / max(1, len(ops))
    cfg0 = starting_strategies(ops, machine, max_parts, choices, n_chains, seed) if start is None else np.ascontiguousarray(start, W.CFG_DT)
    n_chains = len(cfg0)
    chains = B.Chains(sim, cfg0)
    try:
        start_ns = chains.start_ns().copy()
        valid = start_ns[start_ns < B.FF_OVERFLOW_NS]
        if len(valid) == 0:
            raise ValueError("no valid starting strategy")
        ref = float(np.median(valid))
        bucket = max(1, int(ref * accept_scale * 8 / n_buckets))          # the table spans 8 / beta
        beta = 1.0 / (ref * accept_scale)
        ptr, tuples = W.search_space(ops, max_parts, choices)
        chains.search_setup(ptr, tuples, B.ff_sim_accept_table(beta, bucket, n_buckets), bucket, seed, patience=max(1, steps // 2))
        traces = []
        done = 0
        while done < steps:
            n = min(steps_per_call, steps - done)
            traces.append(chains.search(n, ahead=ahead).cpu().numpy().view("<u8"))
            done += n
        best_ns, best = chains.best()
    finally:
        chains.close()
    k = int(np.argmin(best_ns))
    return SearchResult(int(best_ns[k]), best[k].copy(), start_ns, best_ns.copy(), np.concatenate(traces), steps, seed)
