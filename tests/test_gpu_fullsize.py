"""Parity at the full benchmark sizes, in the launch configuration the benchmark times.

Every query of every workload is searched by the C oracle over the whole database and the
GPU result is compared with it bit for bit (rows and scores), and every plane word of the
encoded database and queries is compared as well.  Where a workload is run at two values of K
the oracle searches once at the larger one: its result is the head of one total order
(score descending, row ascending), so its first K entries are the top-K for any smaller K.
"""
import functools
import sys
import time

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import scale as oc
from paper_2008_02002_amd import workloads as wl
from paper_2008_02002_amd import xbq
from tests import gpu_util as gu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@functools.lru_cache(maxsize=1)
def _prepared(name, bits):
    """Database and queries of one workload encoded on both sides, every plane word compared.
    Kept for the tests of the same workload that follow (one workload at a time)."""
    import torch
    w = wl.WORKLOADS[name]
    t0 = time.time()
    Xq = wl.queries(w)
    scale = wl.workload_scale(w)
    # encode the database in slabs so the fp32 rows never sit in memory all at once
    slab = 1 << 20
    nb = xbq.xbq_code_bytes(w.n, w.d, bits, xbq.BUNDLE64)
    db = torch.empty(nb // 4, dtype=torch.int32, device="cuda")
    W = (w.d + 31) // 32
    planes = np.empty((w.n, bits, (w.d + 63) // 64), dtype=np.uint64)
    for lo in range(0, w.n, slab):
        hi = min(w.n, lo + slab)
        X = wl.database(w, lo, hi)
        xbq.xbq_encode(torch.from_numpy(X).cuda(), bits, scale, xbq.BUNDLE64,
                       out=db[lo // 64 * 64 * bits * W:])
        planes[lo:hi] = oc.encode(X, bits, scale)
    _say(f"{name}: {w.n} rows generated and encoded on both sides ({time.time() - t0:.0f}s)")
    q = xbq.xbq_encode(torch.from_numpy(Xq).cuda(), bits, scale, xbq.ROWS)
    qplanes = oc.encode(Xq, bits, scale)
    assert np.array_equal(q.cpu().numpy().view(np.uint32).reshape(w.m, bits, W), oc.planes_as_u32(qplanes, w.d))
    # every plane word of the database codes, bundle layout against the oracle's rows
    got = db.cpu().numpy().view(np.uint32).reshape(-1, bits, W, 64)
    per = slab // 64
    for b0 in range(0, got.shape[0], per):
        b1 = min(got.shape[0], b0 + per)
        rows = got[b0:b1].transpose(0, 3, 1, 2).reshape(-1, bits, W)
        have = min(w.n, b1 * 64) - b0 * 64
        assert np.array_equal(rows[:have], oc.planes_as_u32(planes[b0 * 64:b0 * 64 + have], w.d)), f"bundles {b0}..{b1}"
        assert not rows[have:].any(), "rows past n in the last bundle must be zero words"
    del got
    _say(f"{name}: all code words equal ({time.time() - t0:.0f}s)")
    return db, q, planes, qplanes


def _run(name, bits, ks, part=0, parts=1):
    """The GPU searches all queries of the workload, as the benchmark does; the oracle searches
    the queries of this part (all of them when parts == 1; the long workload is split over
    several tests so that each stays short) and the two are compared whole."""
    import torch
    w = wl.WORKLOADS[name]
    t0 = time.time()
    db, q, planes, qplanes = _prepared(name, bits)
    lo, hi = w.m * part // parts, w.m * (part + 1) // parts
    kmax = max(ks)
    ridx, rscore = oc.search(planes, qplanes[lo:hi], w.d, kmax)
    _say(f"{name}: oracle searched queries {lo}..{hi} at K={kmax} ({time.time() - t0:.0f}s)")
    for k in ks:
        idx, score = xbq.xbq_search(db, w.n, q, w.m, w.d, bits, k)
        torch.cuda.synchronize()
        idx, score = idx.cpu().numpy(), score.cpu().numpy()
        gu.assert_same((idx[lo:hi], score[lo:hi]), (ridx[:, :k], rscore[:, :k]), f"{name} bits={bits} k={k}")
        _say(f"{name}: bits={bits} k={k}: queries {lo}..{hi} of {w.m} identical to the oracle ({time.time() - t0:.0f}s)")


def _run_few_queries(name, bits, k, m):
    """The few-query (histogram selection) path at full database size, every query checked."""
    import torch
    w = wl.WORKLOADS[name]
    db, q, planes, qplanes = _prepared(name, bits)
    W = (w.d + 31) // 32
    idx, score = xbq.xbq_search(db, w.n, q[:m * bits * W], m, w.d, bits, k)
    torch.cuda.synchronize()
    _say(f"{name}: {m} queries searched on the GPU")
    gu.assert_same((idx.cpu().numpy(), score.cpu().numpy()), oc.search(planes, qplanes[:m], w.d, k),
                   f"{name} few queries")


def test_c2_full_size_single_query_mode():
    _run_few_queries("C2", 4, 100, 1)
    _run_few_queries("C2", 4, 100, 8)


def test_c2_full_size():
    _run("C2", 4, (100,))


def test_c3_full_size_few_queries_long_codes():
    _run_few_queries("C3", 3, 10, 3)


def test_c3_full_size_3bit():
    _run("C3", 3, (10,))


def test_c3_full_size_4bit():
    _run("C3", 4, (10,))


def test_c4_full_size():
    _run("C4", 3, (10, 100))


def test_c5_full_size_few_queries():
    # 10 M rows of short codes: several passes of the local selection, not stored distances
    _run_few_queries("C5", 4, 100, 5)
    _run_few_queries("C5", 4, 100, 16)


@pytest.mark.parametrize("part", range(4))
def test_c5_full_size(part):
    _run("C5", 4, (100,), part, 4)


def test_release_the_prepared_workload():
    _prepared.cache_clear()


def test_c2_full_size_refine_4x3():
    """Algorithm 1 end to end at full size: 4-bit queries, 3-bit rows, extra distance, fp32
    refine.  The oracle runs a subset of queries over the whole database."""
    import torch
    from oracle import definition as od
    w = wl.WORKLOADS["C2"]
    k, extra, qb, db_bits = 100, 100, 4, 3
    X, Xq, scale = wl.database(w), wl.queries(w), wl.workload_scale(w)
    xd, xq = torch.from_numpy(X).cuda(), torch.from_numpy(Xq).cuda()
    db = xbq.xbq_encode(xd, db_bits, scale, xbq.BUNDLE64)
    q = xbq.xbq_encode(xq, qb, scale, xbq.ROWS)
    idx, sim, cand = xbq.xbq_search_refine(xd, db, db_bits, xq, q, qb, k, extra)
    torch.cuda.synchronize()
    idx, sim, cand = idx.cpu().numpy(), sim.cpu().numpy(), cand.cpu().numpy()
    _say("C2 refine: searched on the GPU")
    sub = np.concatenate([np.arange(40), w.m - 1 - np.arange(40)])
    S = oc.scores(oc.encode(X, db_bits, scale), oc.encode(Xq[sub], qb, scale), w.d)
    D = od.distance_from_score(S, w.d, qb, db_bits)
    _say("C2 refine: oracle distances done")
    gu.assert_refined_matches((idx[sub], sim[sub], cand[sub]), X, Xq[sub], D, k, extra, xbq.REFINE_MAX_CANDIDATES)
    real, _ = od.exact_cosine_topk(X, Xq[sub[:16]], k)
    assert od.precision_at_k(idx[sub[:16]], real) > 0.9


def test_c5_full_size_refine_hits_the_candidate_bound():
    """Algorithm 1 on the largest workload: 3.84 GB of fp32 rows (row offsets beyond 2^31
    bytes in the refine gather) and candidate lists that reach the documented bound."""
    import torch
    from oracle import definition as od
    w = wl.WORKLOADS["C5"]
    k, extra, bits = 100, 200, 4
    X, scale = wl.database(w), wl.workload_scale(w)
    Xq = wl.queries(w)
    xd, xq = torch.from_numpy(X).cuda(), torch.from_numpy(Xq).cuda()
    db = xbq.xbq_encode(xd, bits, scale, xbq.BUNDLE64)
    q = xbq.xbq_encode(xq, bits, scale, xbq.ROWS)
    idx, sim, cand = xbq.xbq_search_refine(xd, db, bits, xq, q, bits, k, extra)
    torch.cuda.synchronize()
    idx, sim, cand = idx.cpu().numpy(), sim.cpu().numpy(), cand.cpu().numpy()
    del xd, db
    _say("C5 refine: searched on the GPU")
    assert cand.max() == xbq.REFINE_MAX_CANDIDATES
    sub = np.concatenate([np.arange(8), w.m - 1 - np.arange(8)])
    S = oc.scores(oc.encode(X, bits, scale), oc.encode(Xq[sub], bits, scale), w.d)
    D = od.distance_from_score(S, w.d, bits, bits)
    del S
    _say("C5 refine: oracle distances done")
    gu.assert_refined_matches((idx[sub], sim[sub], cand[sub]), X, Xq[sub], D, k, extra, xbq.REFINE_MAX_CANDIDATES)
    real, _ = od.exact_cosine_topk(X, Xq[sub], k)
    assert od.precision_at_k(idx[sub], real) > 0.95


def test_c4_full_size_k_select_long_lists():
    """Algorithm 1 with the whole candidate list on the clustered workload: lists of tens of
    thousands of rows, some cut back to whole distance levels, five batches of queries."""
    import torch
    from oracle import definition as od
    w = wl.WORKLOADS["C4"]
    k, extra, bits, limit = 10, 120, 3, 1 << 17
    X, scale = wl.database(w), wl.workload_scale(w)
    Xq = wl.queries(w)
    xd, xq = torch.from_numpy(X).cuda(), torch.from_numpy(Xq).cuda()
    db = xbq.xbq_encode(xd, bits, scale, xbq.BUNDLE64)
    q = xbq.xbq_encode(xq, bits, scale, xbq.ROWS)
    idx, sim, cand = xbq.xbq_k_select(xd, db, bits, xq, q, bits, k, extra, limit)
    torch.cuda.synchronize()
    idx, sim, cand = idx.cpu().numpy(), sim.cpu().numpy(), cand.cpu().numpy()
    del xd, db
    _say(f"C4 k_select: searched on the GPU, lists of {cand.min()} .. {cand.max()} rows")
    assert cand.max() > 100_000 and cand.max() <= limit
    # the queries with the longest lists (cut or nearly so), the shortest, and both ends of the batch order
    order = np.argsort(cand)
    sub = np.unique(np.concatenate([order[:3], order[-5:], np.arange(3), w.m - 1 - np.arange(3), [2047, 2048]]))
    S = oc.scores(oc.encode(X, bits, scale), oc.encode(Xq[sub], bits, scale), w.d)
    D = od.distance_from_score(S, w.d, bits, bits)
    del S
    _say("C4 k_select: oracle distances done")
    gu.assert_refined_matches((idx[sub], sim[sub], cand[sub]), X, Xq[sub], D, k, extra, limit, by_levels=True)
    printed = np.array([(D[i] <= np.sort(D[i])[k - 1] + extra).sum() for i in range(len(sub))])
    _say(f"C4 k_select: rows within the printed boundary {printed.tolist()}, lists {cand[sub].tolist()}")
    assert (printed > limit).any(), "no sampled query had its list cut"


def test_input_of_more_than_2_31_elements():
    """One encode call and one search over 2.3 M x 960 fp32 values (2.2e9 elements, 8.8 GB; the
    codes alone pass 2^30 bytes): every offset in the path has to be 64-bit."""
    import torch
    w = wl.scaled_down(wl.WORKLOADS["C3"], n=2_300_000, m=6)
    assert w.n * w.d > 2**31
    bits, k = 4, 10
    X, Xq, scale = wl.database(w), wl.queries(w), wl.workload_scale(w)
    xd = torch.from_numpy(X).cuda()
    db = xbq.xbq_encode(xd, bits, scale, xbq.BUNDLE64)             # one call over the whole array
    torch.cuda.synchronize()
    _say("large input: encoded on the GPU")
    planes = oc.encode(X, bits, scale)
    W = (w.d + 31) // 32
    tail = slice(w.n - 70_000, w.n)                                 # rows whose fp32 offsets lie beyond 2^31 elements
    got = gu.bundle_as_rows(db.cpu().numpy().view(np.uint32), w.n, bits, W)[tail]
    assert np.array_equal(got, oc.planes_as_u32(planes[tail], w.d))
    head = gu.bundle_as_rows(db[:1024 * bits * W].cpu().numpy().view(np.uint32), 1024, bits, W)
    assert np.array_equal(head, oc.planes_as_u32(planes[:1024], w.d))
    q = xbq.xbq_encode(torch.from_numpy(Xq).cuda(), bits, scale, xbq.ROWS)
    for sel in (1, 2):                                              # threshold schedule, then histogram selection
        xbq.xbq_set_option("selector", sel)
        try:
            idx, score = xbq.xbq_search(db, w.n, q, w.m, w.d, bits, k)
            torch.cuda.synchronize()
        finally:
            xbq.xbq_set_option("selector", 0)
        _say(f"large input: searched, selector {sel}")
        gu.assert_same((idx.cpu().numpy(), score.cpu().numpy()), oc.search(planes, oc.encode(Xq, bits, scale), w.d, k),
                       f"large input selector {sel}")
    ridx, rsim, rc = xbq.xbq_search_refine(xd, db, bits, torch.from_numpy(Xq).cuda(), q, bits, k, 50)
    torch.cuda.synchronize()
    exact = np.einsum("qkd,qd->qk", X[ridx.cpu().numpy()].astype(np.float64), Xq.astype(np.float64))
    assert np.abs(exact - rsim.cpu().numpy()).max() <= 2e-6        # the refine gathered the right rows
