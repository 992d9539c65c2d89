"""Input recipes: determinism, shapes, distributions, random access by row range."""
import numpy as np
import pytest

from paper_2008_02002_amd import workloads as wl
from paper_2008_02002_amd import costmodel as cm


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_rows_are_normalised_deterministic_and_sliceable(name):
    w = wl.WORKLOADS[name]
    a = wl.database(w, 0, 300)
    assert a.shape == (300, w.d) and a.dtype == np.float32
    assert np.allclose(np.linalg.norm(a.astype(np.float64), axis=1), 1.0, atol=1e-5)
    assert np.array_equal(a, wl.database(w, 0, 300))
    assert np.array_equal(a[100:250], wl.database(w, 100, 250))
    q = wl.queries(w, 0, 50)
    assert q.shape == (50, w.d) and not np.array_equal(q, a[:50])
    if w.kind == "absgauss":
        assert (a >= 0).all()


def test_block_boundary_slicing():
    w = wl.scaled_down(wl.WORKLOADS["C2"], n=wl.BLOCK + 500)
    full = wl.database(w)
    part = wl.database(w, wl.BLOCK - 10, wl.BLOCK + 10)
    assert np.array_equal(part, full[wl.BLOCK - 10:wl.BLOCK + 10])


def test_mixture_has_cluster_structure():
    w = wl.WORKLOADS["C5"]
    a = wl.database(w, 0, 2000).astype(np.float64)
    sims = a @ a.T
    np.fill_diagonal(sims, -1)
    # std 0.25 around N(0,1) centres: rows of one cluster are nearly parallel
    assert (sims.max(axis=1) > 0.7).mean() > 0.2
    z = wl.WORKLOADS["C4"]
    b = wl.database(z, 0, 3000).astype(np.float64)
    s2 = b @ b.T
    np.fill_diagonal(s2, -1)
    assert (s2.max(axis=1) > 0.6).mean() > 0.5          # Zipf: most rows share a big cluster


def test_choose_scale():
    x = np.linspace(-0.5, 0.5, 1001).reshape(1, -1)
    assert wl.choose_scale(x, 1.0) == pytest.approx(2.0)
    assert wl.choose_scale(x, 0.98) == pytest.approx(1 / 0.49, rel=1e-6)
    s = wl.workload_scale(wl.WORKLOADS["C1"])
    assert np.float32(s) == s and 3.0 < s < 6.0         # 1/q98 of |N(0,1)|/sqrt(128)


def test_cost_model_reproduces_printed_ratios(golden_dir):
    import os
    for line in open(os.path.join(golden_dir, "cost_ratios.txt")):
        line = line.split("#")[0].split()
        if not line:
            continue
        bd, bq, ops, space = int(line[0]), int(line[1]), float(line[2]), float(line[3])
        for d in (64 * 16, 64 * 100):                   # ratios are asymptotic in d
            assert round(cm.table1_ops(d, bd, bq) / cm.table1_fp32_ops(d), 2) == pytest.approx(ops, abs=0.011)
            assert round(cm.table1_bytes(d, bd, bq) / cm.table1_fp32_bytes(d), 2) == pytest.approx(space, abs=0.011)
    assert cm.credited_lane_ops_per_pair(128, 4, 4) == 128
    assert cm.credited_lane_ops_per_pair(32, 3, 3) == 18         # 9 XOR + 9 POPCNT (Section 3.3 example)
    assert cm.code_bytes_per_row(200, 3) == 84 and cm.code_bytes_per_row(128, 4) == 64
    assert abs(cm.VALU_INT_LANE_OPS_PER_S - 39.3e12) < 0.05e12


def test_clustered_rows_are_seeded_normalised_and_ordered_on_request():
    X1, Q1 = wl.clustered_rows(5000, 32, 7, 20, 0.25, 3, True)
    X2, Q2 = wl.clustered_rows(5000, 32, 7, 20, 0.25, 3, True)
    assert np.array_equal(X1, X2) and np.array_equal(Q1, Q2)
    assert X1.dtype == np.float32 and X1.shape == (5000, 32) and Q1.shape == (7, 32)
    assert np.allclose(np.linalg.norm(X1, axis=1), 1.0, atol=1e-5)
    assert np.allclose(np.linalg.norm(Q1, axis=1), 1.0, atol=1e-5)
    # ordered: neighbouring rows mostly belong to one cluster, so they are far more alike than
    # rows of the shuffled variant
    Xs, _ = wl.clustered_rows(5000, 32, 7, 20, 0.25, 3, False)
    near = lambda X: float(np.mean(np.sum(X[:-1] * X[1:], axis=1)))
    assert near(X1) > 0.4 and near(Xs) < 0.2
