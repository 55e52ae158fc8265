"""CPU-side checks of the boundary: the built library loads and exports every symbol the
header declares; record layouts match the header's structs."""
import os
import re

import numpy as np

from paper_1807_05358_amd import binding, workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "ff_sim.h")).read()
    declared = set(re.findall(r"\b(ff_sim_\w+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    L = binding.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert L.ff_sim_strerror(0) == b"ok"
    assert L.ff_sim_strerror(-3) == b"workspace missing or too small"


def test_record_layouts_match_header():
    assert W.DIMMAP_DT.itemsize == 12 and W.OP_DT.itemsize == 20 and W.EDGE_DT.itemsize == 56
    assert W.CFG_DT.itemsize == 8 and W.MUT_DT.itemsize == 12
    assert W.EDGE_DT.fields["map"][1] == 8 and W.OP_DT.fields["extent"][1] == 4
    assert W.MUT_DT.fields["cfg"][1] == 4 and W.CFG_DT.fields["dev_offset"][1] == 4
    assert binding.STATS_DT.itemsize == 64


def test_null_arguments_are_rejected_without_a_gpu():
    L = binding.lib()
    assert L.ff_sim_create(None, None, None, None) == binding.FF_EINVAL
    assert L.ff_sim_workspace_bytes(None, 8) == 0
    assert L.ff_sim_set_workspace(None, None, 0) == binding.FF_EINVAL
    assert L.ff_sim_batch(None, None, 1, None, None) == binding.FF_EINVAL
    assert L.ff_sim_delta(None, None, 1, None, None) == binding.FF_EINVAL


def test_exact_division_tricks_used_by_the_kernels():
    """host replica of the kernels' multiply-high divisions, checked against // on the
    ranges the library admits (degrees 1..64, numerators up to 64 * 2^20; any 32-bit
    numerator for the bandwidth division with its one fix-up step)."""
    rng = np.random.default_rng(0)
    n = np.concatenate([np.arange(0, 5000), rng.integers(0, 2 ** 26 + 1, 200000), [2 ** 26 - 1, 2 ** 26]]).astype(np.uint64)
    for d in range(2, 65):
        magic = np.uint64(2 ** 32 // d + 1)
        assert np.array_equal((n * magic) >> np.uint64(32), n // np.uint64(d)), d
    x = np.concatenate([np.arange(0, 3000), rng.integers(0, 2 ** 32, 200000), [2 ** 32 - 1]]).astype(np.uint64)
    for bw in [1, 2, 3, 7, 12, 20, 1000, 65535, 2 ** 31, 2 ** 32 - 1]:
        m = np.uint64(2 ** 32 - 1 if bw == 1 else 2 ** 32 // bw)
        q = (x * m) >> np.uint64(32)
        r = x - q * np.uint64(bw)
        q = q + (r >= bw)
        assert np.array_equal(q, x // np.uint64(bw)), bw
    # device index modulo: numerators below 2^22, divisors up to 1024
    n = rng.integers(0, 2 ** 22, 200000).astype(np.uint64)
    for d in [2, 3, 4, 6, 16, 64, 100, 1000, 1024]:
        magic = np.uint64(2 ** 32 // d + 1)
        assert np.array_equal((n * magic) >> np.uint64(32), n // np.uint64(d)), d
    # owner of coordinate x among deg balanced parts of extent E
    for E, deg in [(10, 3), (299, 64), (35, 4), (17, 16), (1000, 7), (64, 64), (5, 1)]:
        bounds = [(p * E) // deg for p in range(deg + 1)]
        for xx in range(E):
            p = ((xx + 1) * deg - 1) // E
            assert bounds[p] <= xx < bounds[p + 1], (E, deg, xx)


def test_accept_table_matches_the_search_oracle_entry_by_entry():
    """ff_sim_accept_table is host arithmetic (Section 6.1's exp(-beta * delta) at the lower edge of every
    bucket): the oracle's table, written independently, must agree in every entry."""
    from oracle import search as S
    for beta, bucket, n in [(1e-3, 100, 64), (0.0, 7, 5), (2.5e-7, 50_000, 256), (3.1e-9, 123_457, 1024), (0.5, 1, 80)]:
        got = binding.ff_sim_accept_table(beta, bucket, n)
        want = S.metropolis_table(beta, bucket, n)
        assert np.array_equal(got, want), (beta, bucket, n, np.nonzero(got != want)[0][:5])
    L = binding.lib()
    out = np.zeros(4, "<u4")
    assert L.ff_sim_accept_table(-1.0, 10, 4, out.ctypes.data) == binding.FF_EINVAL
    assert L.ff_sim_accept_table(float("nan"), 10, 4, out.ctypes.data) == binding.FF_EINVAL
    assert L.ff_sim_accept_table(1.0, 0, 4, out.ctypes.data) == binding.FF_EINVAL
    assert L.ff_sim_accept_table(1.0, 10, 0, out.ctypes.data) == binding.FF_EINVAL
    assert L.ff_sim_accept_table(1.0, 10, 4, None) == binding.FF_EINVAL
