"""The entry point that allocates nothing, qv_sample_hop_noalloc, against qv_sample_hop.

Both go through the C ABI on the same inputs; outputs must be bit-equal (integer work).  Two
calls in a row share the library's fixed device scratch, the second with a smaller frontier, so
anything the first call left behind would show.  The oracle checks the first call as well.
"""
import ctypes as C

import numpy as np
import pytest

import oracle
import qvgen

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _hop(qv, ctx, g, frontier, fanout, seed, hop, noalloc):
    F = frontier.numel()
    nbr = torch.full((max(F * fanout, 1),), -7, dtype=torch.int32, device="cuda")
    off = torch.full((F + 1,), -7, dtype=torch.int64, device="cuda")
    qv.qv_sample_hop(ctx, g, frontier, fanout, seed, hop, out=(nbr, off), noalloc=noalloc)
    ctx.sync()
    off = off.cpu().numpy()
    return nbr[:off[-1]].cpu().numpy(), off


def test_noalloc_hop_matches_allocating_hop_twice_in_a_row():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2305_10863_amd as qv
    qv.lib()
    w = qvgen.workload("tiny")
    rowptr, col = w.graph()
    ctx = qv.Context(0)
    g = qv.Graph(ctx, torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda())
    rng = np.random.default_rng(77)
    hubs = np.argsort(-np.diff(rowptr))[:50]
    big = np.concatenate([rng.integers(0, w.n, 200_000), hubs]).astype(np.int32)      # several scan tiles, ragged tail
    small = np.concatenate([rng.integers(0, w.n, 777), hubs[:9]]).astype(np.int32)
    for fanout, seed, hop in ((5, 0xABCDEF0123, 1), (40, 2 ** 63 + 99, 3), (100, 12345, 2)):
        for frontier in (big, small):                       # the second call is the smaller one
            d_f = torch.from_numpy(frontier).cuda()
            want_nbr, want_off = _hop(qv, ctx, g, d_f, fanout, seed, hop, noalloc=False)
            got_nbr, got_off = _hop(qv, ctx, g, d_f, fanout, seed, hop, noalloc=True)
            assert np.array_equal(got_off, want_off), (fanout, len(frontier))
            assert np.array_equal(got_nbr, want_nbr), (fanout, len(frontier))
        o_nbr, o_off = oracle.sample_hop(rowptr, col, small, fanout, seed, hop)
        assert np.array_equal(got_off, o_off) and np.array_equal(got_nbr, o_nbr)
    # empty frontier, and a frontier beyond the fixed scratch
    e_nbr, e_off = _hop(qv, ctx, g, torch.zeros(0, dtype=torch.int32, device="cuda"), 5, 1, 1, noalloc=True)
    assert len(e_nbr) == 0 and e_off.tolist() == [0]
    too_many = qv.QV_NOALLOC_MAX_FRONTIER + 1
    d_f = torch.zeros(too_many, dtype=torch.int32, device="cuda")
    nbr = torch.empty(1, dtype=torch.int32, device="cuda")
    off = torch.empty(too_many + 1, dtype=torch.int64, device="cuda")
    rc = qv.lib().qv_sample_hop_noalloc(ctx.h, g.h, C.c_void_p(d_f.data_ptr()), too_many, 1, C.c_uint64(1), 1,
                                        C.c_void_p(nbr.data_ptr()), 1, C.c_void_p(off.data_ptr()))
    assert rc == qv.QV_EINVAL and b"fixed scratch" in qv.lib().qv_last_error(ctx.h)
    ctx.sync()
    g = None
    ctx.close()
