"""ff_sim_neighbours_noalloc (the neighbour sweep for callers that cannot allocate: its scratch is a fixed
device array of the library) against ff_sim_neighbours, through the C boundary: same mutation list, same
times, same best neighbour, bit for bit, on two calls in a row, the second over a smaller range of ops."""
import numpy as np
import pytest

from paper_1807_05358_amd import workloads as W

pytestmark = pytest.mark.gpu


def _sweep_both(B, ch, d_ptr, d_tup, n_tuples, op_begin, op_end):
    import torch
    C = ch.C
    M = B.ff_sim_neighbour_count(ch.handle, d_ptr.data_ptr(), n_tuples, op_begin, op_end)
    ch._ensure_try_workspace(M)
    out = []
    for which in ("alloc", "noalloc"):
        d_muts = torch.zeros(M * C * W.MUT_DT.itemsize, dtype=torch.uint8, device="cuda")
        d_out = torch.zeros((M, C), dtype=torch.int64, device="cuda")
        d_best = torch.zeros(C, dtype=torch.int64, device="cuda")
        d_idx = torch.zeros(C, dtype=torch.int32, device="cuda")
        st = torch.cuda.current_stream().cuda_stream
        if which == "alloc":
            B.ff_sim_neighbours(ch.handle, d_ptr.data_ptr(), d_tup.data_ptr(), n_tuples, op_begin, op_end, d_muts.data_ptr(),
                                d_out.data_ptr(), d_best.data_ptr(), d_idx.data_ptr(), st)
        else:
            B.ff_sim_neighbours_noalloc(ch.handle, d_ptr.data_ptr(), d_tup.data_ptr(), n_tuples, op_begin, op_end, M, d_muts.data_ptr(),
                                        d_out.data_ptr(), d_best.data_ptr(), d_idx.data_ptr(), st)
        torch.cuda.synchronize()
        out.append((d_muts.cpu().numpy().view(W.MUT_DT).reshape(M, C), d_out.cpu().numpy().view("<u8"),
                    d_best.cpu().numpy().view("<u8"), d_idx.cpu().numpy().view("<u4")))
    return M, out


def test_noalloc_neighbour_sweep_equals_the_allocating_one():
    import torch
    from paper_1807_05358_amd import binding as B
    w = W.workload(1)
    sim = B.Simulator(w.ops, w.edges, w.machine, w.cost)
    ch = B.Chains(sim, w.strategies(2))
    tp, tu = w.search_space()
    d_ptr, d_tup = B.to_device(np.ascontiguousarray(tp, "<u4")), B.to_device(np.ascontiguousarray(tu, "<u4"))
    sizes = []
    for op_begin, op_end in ((0, w.n_ops), (3, 7)):          # the second call is the smaller one
        M, (a, b) = _sweep_both(B, ch, d_ptr, d_tup, len(tu), op_begin, op_end)
        sizes.append(M)
        assert np.array_equal(a[0], b[0]), "mutation lists differ"
        assert np.array_equal(a[1], b[1]), f"times differ at {np.argwhere(a[1] != b[1])[:4]}"
        assert np.array_equal(a[2], b[2]) and np.array_equal(a[3], b[3])
        assert (b[1] < B.FF_OVERFLOW_NS).any()
    assert sizes[1] < sizes[0]
    # a count that does not match the ranges is noticed on the device: every result is "invalid"
    M = sizes[1]
    d_muts = torch.zeros(M * 2 * W.MUT_DT.itemsize, dtype=torch.uint8, device="cuda")
    d_out = torch.zeros((M, 2), dtype=torch.int64, device="cuda")
    d_best = torch.zeros(2, dtype=torch.int64, device="cuda")
    d_idx = torch.zeros(2, dtype=torch.int32, device="cuda")
    B.ff_sim_neighbours_noalloc(ch.handle, d_ptr.data_ptr(), d_tup.data_ptr(), len(tu), 2, 7, M, d_muts.data_ptr(), d_out.data_ptr(),
                                d_best.data_ptr(), d_idx.data_ptr(), torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert (d_out.cpu().numpy().view("<u8") == B.FF_INVALID_NS).all() and (d_best.cpu().numpy().view("<u8") == B.FF_INVALID_NS).all()
    # argument errors come back as codes
    L = B.lib()
    assert L.ff_sim_neighbours_noalloc(ch.handle, d_ptr.data_ptr(), d_tup.data_ptr(), len(tu), 5, 5, M, d_muts.data_ptr(), d_out.data_ptr(),
                                       d_best.data_ptr(), d_idx.data_ptr(), None) == B.FF_EINVAL
    assert L.ff_sim_neighbours_noalloc(ch.handle, d_ptr.data_ptr(), d_tup.data_ptr(), len(tu), 0, w.n_ops + 1, M, d_muts.data_ptr(),
                                       d_out.data_ptr(), d_best.data_ptr(), d_idx.data_ptr(), None) == B.FF_EINVAL
    assert L.ff_sim_neighbours_noalloc(ch.handle, None, d_tup.data_ptr(), len(tu), 0, 2, M, d_muts.data_ptr(), d_out.data_ptr(),
                                       d_best.data_ptr(), d_idx.data_ptr(), None) == B.FF_EINVAL
    torch.cuda.synchronize()
    ch.close()
    sim.close()
