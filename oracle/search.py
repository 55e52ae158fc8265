"""CPU oracle of the search loop (Section 6): one Markov chain of single-op proposals
(Section 6.2) accepted by the Metropolis rule (Section 6.1), each candidate priced by a
full simulation with the oracle simulator.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).  Plain Python integers throughout.

The rule of Section 6.1 accepts a proposal S* from S with probability
min(1, exp(beta * (cost(S) - cost(S*)))).  To make every decision reproducible bit for bit,
the probabilities are an input: `accept[b]` is the probability, scaled by 2^32, for a proposal
that is slower by delta ns with b = min(delta // bucket_ns, len(accept) - 1); a proposal that
is not slower is always accepted.  metropolis_table() writes the table for a given beta.

Random numbers come from a counter-based generator that both this file and the GPU kernel
implement independently: the SplitMix64 finaliser chained over (seed, purpose, chain, step).
"""
from __future__ import annotations

import math

import numpy as np

from . import INVALID, simulate_batch

_M = (1 << 64) - 1
_K = 0xD6E8FEB86659FD93
OP, TUPLE, OFFSET, ACCEPT = 10, 11, 12, 13     # the `purpose` of a draw


def mix64(x: int) -> int:
    x = (x + 0x9E3779B97F4A7C15) & _M
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & _M
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & _M
    return x ^ (x >> 31)


def draw(seed: int, purpose: int, chain: int, step: int) -> int:
    h = mix64(seed & _M)
    for c in (purpose, chain, step):
        h = mix64(h ^ ((c * _K) & _M))
    return h


def metropolis_table(beta_per_ns: float, bucket_ns: int, n_buckets: int) -> np.ndarray:
    """accept[b] = floor(2^32 * exp(-beta * b * bucket_ns)) (the bucket's lower edge), capped
    at 2^32 - 1."""
    out = np.zeros(n_buckets, np.uint32)
    for b in range(n_buckets):
        out[b] = min((1 << 32) - 1, int(math.floor(math.exp(-beta_per_ns * b * bucket_ns) * 4294967296.0)))
    return out


def metropolis_chain(ops, edges, machine, cost, cfg0, tuple_ptr, tuples, accept, bucket_ns, seed,
                     chain, first_step, n_steps, patience=0, idle_steps=0, best_so_far=None, params=None):
    """runs n_steps of one chain starting from the valid strategy cfg0.  patience > 0: the
    stopping rule of Section 6.2 -- after `patience` steps without a new best the chain makes
    no further proposals (idle_steps / best_so_far carry the state of an earlier call over).
    Returns (trace [n_steps] of the chain's time after each step, final strategy, best time,
    best strategy, number of accepted proposals)."""
    n_ops = len(ops)
    n_dev = int(machine.n_devices)
    cur = np.array(cfg0, copy=True)
    cur_ns = int(simulate_batch(ops, edges, machine, cost, cur[None], params=params)[0])
    assert cur_ns != INVALID, "the chain must start from a valid strategy"
    best_ns, best = cur_ns, cur.copy()
    if best_so_far is not None and best_so_far < best_ns:
        best_ns, best = best_so_far, None
    idle = idle_steps
    trace = np.zeros(n_steps, "<u8")
    n_acc = 0
    for s in range(n_steps):
        st = first_step + s
        op = draw(seed, OP, chain, st) % n_ops
        t0, t1 = int(tuple_ptr[op]), int(tuple_ptr[op + 1])
        if t1 > t0 and not (patience and idle >= patience):
            word = int(tuples[t0 + draw(seed, TUPLE, chain, st) % (t1 - t0)])
            prop = cur.copy()
            prop[op]["deg"] = [(word >> (8 * d)) & 0xFF for d in range(4)]
            prop[op]["dev_offset"] = draw(seed, OFFSET, chain, st) % n_dev
            prop[op]["dev_stride"] = 1
            new_ns = int(simulate_batch(ops, edges, machine, cost, prop[None], params=params)[0])
            ok = False
            if new_ns < INVALID - 2:            # a time, not a result code
                if new_ns <= cur_ns:
                    ok = True
                else:
                    b = min((new_ns - cur_ns) // int(bucket_ns), len(accept) - 1)
                    ok = (draw(seed, ACCEPT, chain, st) >> 32) < int(accept[b])
            if ok:
                cur, cur_ns = prop, new_ns
                n_acc += 1
        trace[s] = cur_ns
        idle += 1
        if cur_ns < best_ns:
            best_ns, best = cur_ns, cur.copy()
            idle = 0
    return trace, cur, best_ns, best, n_acc
