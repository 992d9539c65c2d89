"""Helpers for the GPU parity tests: run the HIP path through the C-ABI binding and the
oracle on the same inputs.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np

from oracle import scale as oc
from paper_2008_02002_amd import xbq


def to_dev(a: np.ndarray):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def gpu_encode(X: np.ndarray, bits: int, scale: float, layout: int) -> np.ndarray:
    """uint32 plane words as the library wrote them (flat)."""
    import torch
    codes = xbq.xbq_encode(to_dev(X.astype(np.float32)), bits, scale, layout)
    torch.cuda.synchronize()
    return codes.cpu().numpy().view(np.uint32)


def bundle_as_rows(flat: np.ndarray, n: int, bits: int, W: int) -> np.ndarray:
    """[ceil(n/64)][bits][W][64] -> [ceil(n/64)*64][bits][W] (pure re-indexing)."""
    nb = (n + 63) // 64
    return np.ascontiguousarray(flat.reshape(nb, bits, W, 64).transpose(0, 3, 1, 2).reshape(nb * 64, bits, W))


def oracle_rows(X: np.ndarray, bits: int, scale: float) -> np.ndarray:
    return oc.planes_as_u32(oc.encode(X, bits, scale), X.shape[1])


def gpu_search(Xdb: np.ndarray, Xq: np.ndarray, bits: int, k: int, scale: float):
    """Encode both sides on the GPU and search; returns numpy (idx, score) and the device codes."""
    import torch
    n, d = Xdb.shape
    m = Xq.shape[0]
    db = xbq.xbq_encode(to_dev(Xdb), bits, scale, xbq.BUNDLE64)
    q = xbq.xbq_encode(to_dev(Xq), bits, scale, xbq.ROWS)
    idx, score = xbq.xbq_search(db, n, q, m, d, bits, k)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), score.cpu().numpy()


def oracle_search(Xdb: np.ndarray, Xq: np.ndarray, bits: int, k: int, scale: float):
    d = Xdb.shape[1]
    return oc.search(oc.encode(Xdb, bits, scale), oc.encode(Xq, bits, scale), d, k)


def assert_same(got, want, what=""):
    gi, gs = got
    wi, ws = want
    if not np.array_equal(gs, ws):
        bad = np.argwhere(gs != ws)
        raise AssertionError(f"{what}: {len(bad)} score mismatches, first at {bad[0]}: "
                             f"gpu {gs[tuple(bad[0])]} oracle {ws[tuple(bad[0])]}")
    if not np.array_equal(gi, wi):
        bad = np.argwhere(gi != wi)
        raise AssertionError(f"{what}: {len(bad)} index mismatches, first at {bad[0]}: "
                             f"gpu {gi[tuple(bad[0])]} oracle {wi[tuple(bad[0])]}")


def check_order_properties(idx: np.ndarray, score: np.ndarray, n: int):
    """What holds at any size: rows in range and distinct, (score desc, idx asc) order."""
    assert idx.min() >= 0 and idx.max() < n
    srt = np.sort(idx, axis=1)
    assert (srt[:, 1:] != srt[:, :-1]).all(), "duplicate row in a result"
    ds = np.diff(score.astype(np.int64), axis=1)
    assert (ds <= 0).all(), "scores not descending"
    di = np.diff(idx.astype(np.int64), axis=1)
    assert (di[ds == 0] > 0).all(), "tie not broken by lower index"


def gpu_search_asym(Xdb, Xq, db_bits: int, q_bits: int, k: int, scale: float):
    import torch
    n, d = Xdb.shape
    m = Xq.shape[0]
    db = xbq.xbq_encode(to_dev(Xdb), db_bits, scale, xbq.BUNDLE64)
    q = xbq.xbq_encode(to_dev(Xq), q_bits, scale, xbq.ROWS)
    idx, score = xbq.xbq_search_asym(db, n, db_bits, q, m, q_bits, d, k)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), score.cpu().numpy()


def oracle_search_asym(Xdb, Xq, db_bits: int, q_bits: int, k: int, scale: float):
    d = Xdb.shape[1]
    return oc.search(oc.encode(Xdb, db_bits, scale), oc.encode(Xq, q_bits, scale), d, k)


def gpu_search_refine(Xdb, Xq, db_bits: int, q_bits: int, k: int, extra: int, scale: float):
    import torch
    xd, xq = to_dev(Xdb), to_dev(Xq)
    db = xbq.xbq_encode(xd, db_bits, scale, xbq.BUNDLE64)
    q = xbq.xbq_encode(xq, q_bits, scale, xbq.ROWS)
    idx, sim, cand = xbq.xbq_search_refine(xd, db, db_bits, xq, q, q_bits, k, extra)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), sim.cpu().numpy(), cand.cpu().numpy()


def oracle_distances(Xdb, Xq, db_bits: int, q_bits: int, scale: float):
    """Integer distances D[m, n] from the C oracle's scores."""
    from oracle import definition as od
    d = Xdb.shape[1]
    S = oc.scores(oc.encode(Xdb, db_bits, scale), oc.encode(Xq, q_bits, scale), d)
    return od.distance_from_score(S, d, q_bits, db_bits)


def gpu_k_select(Xdb, Xq, db_bits: int, q_bits: int, k: int, extra: int, max_candidates: int, scale: float):
    import torch
    xd, xq = to_dev(Xdb), to_dev(Xq)
    db = xbq.xbq_encode(xd, db_bits, scale, xbq.BUNDLE64)
    q = xbq.xbq_encode(xq, q_bits, scale, xbq.ROWS)
    idx, sim, cand = xbq.xbq_k_select(xd, db, db_bits, xq, q, q_bits, k, extra, max_candidates)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), sim.cpu().numpy(), cand.cpu().numpy()


def assert_refined_matches(got, Xdb, Xq, D, k, extra, limit, tol=2e-6, by_levels=False):
    """Compare with Algorithm 1 run by the oracle.  The candidate count is an integer and
    must match exactly.  Similarities are fp32 sums on the GPU and float64 in the oracle:
    they must agree within tol, and a returned row may differ from the oracle's row at the
    same rank only if their exact similarities are within tol (a tie at fp32 resolution)."""
    from oracle import definition as od
    gi, gs, gc = got
    select = od.k_select_by_levels if by_levels else od.k_select
    candidates = od.k_select_candidates_by_levels if by_levels else od.k_select_candidates
    ridx, rsim, rcount = select(D, Xdb, Xq, k, extra, limit)
    assert np.array_equal(gc, rcount), "candidate counts differ"
    X64 = Xdb.astype(np.float64)
    for q in range(Xq.shape[0]):
        exact = X64[gi[q]] @ Xq[q].astype(np.float64)
        assert np.abs(exact - gs[q]).max() <= tol, "similarity is not the inner product of the returned row"
        assert len(set(gi[q].tolist())) == k
        L = set(candidates(D[q], k, extra, limit).tolist())
        assert set(gi[q].tolist()) <= L, "a returned row is not a candidate"
        diff = gi[q] != ridx[q]
        assert (np.abs(exact[diff] - rsim[q][diff]) <= tol).all(), "rank differs beyond fp32 resolution"
