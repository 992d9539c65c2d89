"""The entry point that allocates nothing (xbq_search_static) against xbq_search.

Called through the C ABI on two calls in a row, the second with a smaller input, so that
whatever the first call left in the library's built-in scratch buffer is still there when
the second one runs.  Both the threshold schedule (many queries) and the histogram
selection (few queries) go through the buffer.  Results must be identical to xbq_search's,
which the parity tests tie to the oracle.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from paper_2008_02002_amd import workloads as wl
from paper_2008_02002_amd import xbq


def _both(Xdb, Xq, bits, k, scale):
    import torch
    n, d = Xdb.shape
    m = Xq.shape[0]
    db = xbq.xbq_encode(torch.from_numpy(Xdb).cuda(), bits, scale, xbq.BUNDLE64)
    q = xbq.xbq_encode(torch.from_numpy(Xq).cuda(), bits, scale, xbq.ROWS)
    want_idx, want_score = xbq.xbq_search(db, n, q, m, d, bits, k)
    idx = torch.full((m, k), -7, dtype=torch.int32, device="cuda")
    score = torch.full((m, k), -7, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    xbq.xbq_search_static(db, n, q, m, d, bits, k, idx, score)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before           # nothing came from torch's allocator either
    assert torch.equal(idx, want_idx), "rows differ from xbq_search"
    assert torch.equal(score, want_score), "scores differ from xbq_search"
    return idx.cpu().numpy(), score.cpu().numpy()


@pytest.mark.parametrize("m_first,m_second", [(300, 37), (8, 1)])
def test_static_scratch_matches_xbq_search_on_two_calls_in_a_row(m_first, m_second):
    w = wl.scaled_down(wl.WORKLOADS["C2"], n=70_003, m=m_first)
    Xdb, Xq, scale = wl.database(w), wl.queries(w), wl.workload_scale(w)
    _both(Xdb, Xq, 4, 100, scale)
    # second call: fewer rows (a ragged last bundle), fewer queries, smaller k, same buffer
    _both(Xdb[:9_990], Xq[:m_second], 4, 10, scale)


def test_static_scratch_against_the_oracle():
    from oracle import scale as oc
    w = wl.WORKLOADS["C1"]
    Xdb, Xq, scale = wl.database(w), wl.queries(w), wl.workload_scale(w)
    got = _both(Xdb, Xq, 4, 10, scale)
    want = oc.search(oc.encode(Xdb, 4, scale), oc.encode(Xq, 4, scale), w.d, 10)
    assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1])


def test_request_beyond_the_buffer_is_refused():
    import ctypes
    import torch
    L = xbq.lib()
    n, m, d, bits, k = 1_000_000, 10_000, 128, 4, 100
    assert L.xbq_search_workspace_bytes(n, m, d, bits, k) > xbq.STATIC_SCRATCH_BYTES
    t = torch.zeros(64, dtype=torch.int32, device="cuda")     # never touched: the size check comes first
    p = ctypes.c_void_p(t.data_ptr())
    assert L.xbq_search_static(p, n, p, m, d, bits, k, p, p, None) == xbq.ESTATIC
    assert b"built-in" in L.xbq_strerror(xbq.ESTATIC)
