"""The plain-C oracle, pinned to the definition-level oracle and to brute force."""
import numpy as np
import pytest

from oracle import definition as od
from oracle import scale as oc


def _rand(n, d, seed, lo=-0.5, hi=0.5):
    rng = np.random.default_rng(seed)
    return rng.uniform(lo, hi, size=(n, d)).astype(np.float32)


@pytest.mark.parametrize("B", [1, 2, 3, 4, 5, 8])
@pytest.mark.parametrize("d", [1, 31, 32, 33, 63, 64, 65, 96, 128, 200])
def test_codes_and_planes_match_definition(B, d):
    X = _rand(23, d, seed=B * 1000 + d)
    for scale in (1.0, 2.95):
        codes = oc.quantize(X, B, scale)
        assert np.array_equal(codes, od.encode(X, B, scale))
        planes = oc.pack(codes, B)
        assert np.array_equal(oc.planes_as_u32(planes, d), od.pack_planes(codes, B))


def test_quantize_at_every_cell_boundary():
    for B in (3, 4):
        pts = []
        for k in range(-(1 << B) - 2, (1 << B) + 3):
            c = np.float32(k / float(1 << B))
            pts += [c, np.nextafter(c, np.float32(9)), np.nextafter(c, np.float32(-9))]
        pts += [np.float32(0.0), np.float32(-0.0), np.float32(1e-45), np.float32(-1e-45),
                np.float32(3e38), np.float32(-3e38), np.float32(np.inf), np.float32(-np.inf)]
        X = np.array([pts], dtype=np.float32)
        got = oc.quantize(X, B, 1.0)
        want = [od.quantize_code(float(p), B) for p in pts]
        assert got[0].tolist() == want


@pytest.mark.parametrize("d,Bq,Bd", [(128, 4, 4), (200, 3, 3), (96, 4, 4), (70, 4, 3), (960, 3, 3), (33, 1, 2)])
def test_scores_match_definition(d, Bq, Bd):
    Xd = _rand(57, d, 1)
    Xq = _rand(6, d, 2)
    pd_, pq = oc.encode(Xd, Bd, 2.0), oc.encode(Xq, Bq, 2.0)
    S = oc.scores(pd_, pq, d)
    ref = od.score_matrix(od.pack_planes(od.encode(Xq, Bq, 2.0), Bq),
                          od.pack_planes(od.encode(Xd, Bd, 2.0), Bd), d, Bq, Bd)
    assert np.array_equal(S, ref)
    # and the integer dot product of decoded vectors, computed as an exact float64 GEMM
    G = od.decode(oc.quantize(Xq, Bq, 2.0), Bq).astype(np.float64) @ \
        od.decode(oc.quantize(Xd, Bd, 2.0), Bd).astype(np.float64).T
    assert np.array_equal(S, G.astype(np.int64))
    qi = np.array([0, 5, 3, 3]); ri = np.array([56, 0, 17, 18])
    assert np.array_equal(oc.scores_at(pd_, pq, d, qi, ri), S[qi, ri])


@pytest.mark.parametrize("n,d,B,K", [(300, 64, 4, 1), (300, 64, 4, 17), (300, 64, 4, 300),
                                     (1000, 200, 3, 100), (129, 96, 4, 64), (50, 5, 2, 50)])
def test_search_matches_definition(n, d, B, K):
    Xd = _rand(n, d, 3)
    Xq = _rand(9, d, 4)
    idx, sc = oc.search(oc.encode(Xd, B, 2.5), oc.encode(Xq, B, 2.5), d, K)
    ridx, rsc = od.search(Xd, Xq, B, K, 2.5)
    assert np.array_equal(idx, ridx)
    assert np.array_equal(sc, rsc)


def test_search_heavy_ties_and_duplicates():
    # low dimension and one bit: only a handful of distinct scores, so the tie rule decides
    Xd = np.tile(_rand(40, 6, 5), (5, 1))
    Xq = _rand(4, 6, 6)
    idx, sc = oc.search(oc.encode(Xd, 1), oc.encode(Xq, 1), 6, 120)
    ridx, rsc = od.search(Xd, Xq, 1, 120)
    assert np.array_equal(idx, ridx) and np.array_equal(sc, rsc)
    # all rows identical: every score equal, result must be 0..K-1
    Xs = np.tile(_rand(1, 16, 7), (70, 1))
    idx, _ = oc.search(oc.encode(Xs, 4), oc.encode(Xq[:, :6].repeat(3, axis=1)[:, :16].copy(), 4), 16, 9)
    assert idx.tolist() == [list(range(9))] * 4


def test_search_rejects_bad_k():
    Xd = _rand(10, 8, 8)
    p = oc.encode(Xd, 4)
    with pytest.raises(ValueError):
        oc.search(p, p, 8, 11)
    with pytest.raises(ValueError):
        oc.search(p, p, 8, 0)


def test_threads_reported():
    assert oc.threads() >= 1
