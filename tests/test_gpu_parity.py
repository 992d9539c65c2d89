"""GPU parity: the HIP path (through the C-ABI binding) against the CPU oracle, bit-exact.

Codes, integer scores and top-K rows must be identical; ties go to the lower row.
"""
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import definition as od
from oracle import scale as oc
from paper_2008_02002_amd import workloads as wl
from paper_2008_02002_amd import xbq
from tests import gpu_util as gu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    xbq.lib()
    yield


@pytest.fixture(params=[1, 2, 3], ids=["threshold", "histogram", "local"])
def selector(request):
    """Run a test once with each top-K selector forced."""
    xbq.xbq_set_option("selector", request.param)
    yield request.param
    xbq.xbq_set_option("selector", 0)


def _rand(n, d, seed, lo=-0.5, hi=0.5):
    return np.random.default_rng(seed).uniform(lo, hi, size=(n, d)).astype(np.float32)


# ----------------------------------------------------------------------------- encode
@pytest.mark.parametrize("bits", [1, 2, 3, 4])
@pytest.mark.parametrize("n,d", [(1, 1), (5, 31), (64, 32), (65, 33), (130, 64), (257, 65), (300, 96),
                                 (1000, 128), (513, 200), (200, 960), (70, 2048), (3, 1000)])
def test_encode_matches_oracle(bits, n, d):
    _say(f"encode bits={bits} n={n} d={d}")
    X = _rand(n, d, seed=bits * 7919 + n * 31 + d)
    for scale in (1.0, 2.95):
        want = gu.oracle_rows(X, bits, scale)
        W = (d + 31) // 32
        got_rows = gu.gpu_encode(X, bits, scale, xbq.ROWS).reshape(n, bits, W)
        assert np.array_equal(got_rows, want)
        got_b = gu.bundle_as_rows(gu.gpu_encode(X, bits, scale, xbq.BUNDLE64), n, bits, W)
        assert np.array_equal(got_b[:n], want)
        assert (got_b[n:] == 0).all()                      # rows past n in the last bundle are zero words


def test_encode_bit_order_against_hand_typed_words(golden_dir):
    """Both code layouts of the library against the plane words typed by hand in the golden file
    (coordinate 0 at the least significant end of a plane; Section 3.3)."""
    from tests.test_oracle_pins import _read_bit_order_golden
    d, B, row, want, _ = _read_bit_order_golden(golden_dir)
    x = ((7 - 2 * row.astype(np.int64)) / 8.0).astype(np.float32)
    X = np.stack([x, x[::-1], x])                      # the hand-typed row first and last, another one between
    W = (d + 31) // 32
    rows = gu.gpu_encode(X, B, 1.0, xbq.ROWS).reshape(3, B, W)
    assert np.array_equal(rows[0], want) and np.array_equal(rows[2], want)
    assert not np.array_equal(rows[1], want)
    bundle = gu.gpu_encode(X, B, 1.0, xbq.BUNDLE64).reshape(1, B, W, 64)
    assert np.array_equal(bundle[0, :, :, 0], want) and np.array_equal(bundle[0, :, :, 2], want)
    assert np.array_equal(bundle[0, :, :, 1], rows[1]) and not bundle[0, :, :, 3:].any()


@pytest.mark.parametrize("bits", [1, 2, 3, 4])
def test_encode_cell_boundaries_denormals_and_saturation(bits):
    pts = []
    for k in range(-(1 << bits) - 2, (1 << bits) + 3):
        c = np.float32(k / float(1 << bits))
        pts += [c, np.nextafter(c, np.float32(9)), np.nextafter(c, np.float32(-9))]
    pts += [0.0, -0.0, 1e-45, -1e-45, 1e-39, -1e-39, 1.1754944e-38, -1.1754944e-38, 3e38, -3e38,
            np.inf, -np.inf, 0.99999994, -0.99999994, 123.0, -123.0]
    X = np.array(pts, dtype=np.float32)
    X = np.concatenate([X, np.zeros((-len(X)) % 8, np.float32)]).reshape(-1, 8)
    for scale in (1.0, 1.0000001, 3.0, 0.33333334, 2.95):
        want = gu.oracle_rows(X, bits, scale)
        got = gu.gpu_encode(X, bits, scale, xbq.ROWS).reshape(want.shape)
        assert np.array_equal(got, want), (bits, scale)
    # a product that only lands on the cell boundary after rounding to binary32
    x = np.full((4, 16), np.float32(0.083333336))
    assert np.array_equal(gu.gpu_encode(x, bits, 3.0, xbq.ROWS).reshape(4, bits, 1), gu.oracle_rows(x, bits, 3.0))


def test_encode_random_bits_sweep():
    # every fp32 bit pattern class: random words reinterpreted as floats (NaN removed)
    rng = np.random.default_rng(99)
    raw = rng.integers(0, 1 << 32, size=200_000, dtype=np.uint64).astype(np.uint32).view(np.float32)
    raw = raw[np.isfinite(raw)][:160_000].reshape(-1, 160)
    small = (rng.standard_normal((500, 160)) * 0.3).astype(np.float32)
    X = np.concatenate([raw, small])
    for bits in (3, 4):
        want = gu.oracle_rows(X, bits, 1.7)
        got = gu.gpu_encode(X, bits, 1.7, xbq.ROWS).reshape(want.shape)
        assert np.array_equal(got, want)


# ----------------------------------------------------------------------------- search
SMALL = [
    # n, d, m, bits, k
    (1, 8, 3, 4, 1),
    (63, 16, 5, 4, 10),
    (64, 128, 7, 4, 64),
    (65, 128, 7, 3, 65),
    (1000, 128, 33, 4, 10),
    (1024, 128, 9, 4, 100),
    (1025, 128, 9, 4, 100),
    (4097, 128, 17, 4, 100),
    (5000, 96, 40, 4, 100),
    (5000, 200, 40, 3, 10),
    (5000, 200, 40, 3, 100),
    (20000, 128, 100, 4, 1),
    (20000, 128, 50, 4, 1024),
    (9000, 64, 30, 2, 50),
    (9000, 32, 30, 1, 50),
    (7000, 256, 20, 4, 10),
    (7000, 250, 20, 3, 10),
    (3000, 960, 24, 3, 10),
    (3000, 960, 24, 4, 10),
    (3000, 300, 50, 4, 33),
    (2000, 2048, 18, 4, 5),
    (2000, 1000, 18, 2, 5),
    (2500, 320, 17, 1, 7),
]


@pytest.mark.parametrize("n,d,m,bits,k", SMALL)
def test_search_matches_oracle_small(n, d, m, bits, k, selector):
    _say(f"search n={n} d={d} m={m} bits={bits} k={k}")
    Xdb = _rand(n, d, seed=n + d)
    Xq = _rand(m, d, seed=n + d + 1)
    scale = 1.9
    gu.assert_same(gu.gpu_search(Xdb, Xq, bits, k, scale), gu.oracle_search(Xdb, Xq, bits, k, scale),
                   f"n={n} d={d} bits={bits} k={k}")


def test_config_c1_full(selector):
    w = wl.WORKLOADS["C1"]
    _say("C1 full")
    Xdb, Xq, scale = wl.database(w), wl.queries(w), wl.workload_scale(w)
    got = gu.gpu_search(Xdb, Xq, 4, 10, scale)
    gu.assert_same(got, gu.oracle_search(Xdb, Xq, 4, 10, scale), "C1")
    # and against the definition-level oracle directly
    ridx, rsc = od.search(Xdb, Xq, 4, 10, scale)
    assert np.array_equal(got[0], ridx) and np.array_equal(got[1], rsc)


@pytest.mark.parametrize("name,n,m", [("C2", 150_000, 200), ("C3", 40_000, 64), ("C4", 200_000, 150),
                                      ("C5", 300_000, 150)])
def test_configs_scaled_down(name, n, m, selector):
    w = wl.scaled_down(wl.WORKLOADS[name], n=n, m=m)
    Xdb, Xq, scale = wl.database(w), wl.queries(w), wl.workload_scale(w)
    for bits in w.bits:
        for k in w.ks:
            _say(f"{name} scaled n={n} m={m} bits={bits} k={k}")
            got = gu.gpu_search(Xdb, Xq, bits, k, scale)
            gu.assert_same(got, gu.oracle_search(Xdb, Xq, bits, k, scale), f"{name} bits={bits} k={k}")
            gu.check_order_properties(got[0], got[1], n)


ASYM = [
    # n, d, m, q_bits, db_bits, k
    (5000, 128, 40, 4, 3, 10),
    (5000, 200, 40, 4, 3, 100),
    (20000, 96, 64, 4, 3, 100),
    (9000, 64, 30, 3, 2, 50),
    (9000, 40, 30, 2, 1, 20),
    (3000, 960, 24, 4, 3, 10),
    (2500, 300, 17, 3, 2, 7),
    (300, 256, 5, 4, 3, 300),
]


@pytest.mark.parametrize("n,d,m,qb,db,k", ASYM)
def test_search_asymmetric_bits(n, d, m, qb, db, k, selector):
    # 4-bit queries against 3-bit documents is the setting of Sections 3.6 and 5
    _say(f"asym n={n} d={d} m={m} q_bits={qb} db_bits={db} k={k}")
    Xdb = _rand(n, d, seed=n + d + qb)
    Xq = _rand(m, d, seed=n + d + qb + 1)
    gu.assert_same(gu.gpu_search_asym(Xdb, Xq, db, qb, k, 2.2), gu.oracle_search_asym(Xdb, Xq, db, qb, k, 2.2),
                   f"asym {qb}x{db}")


def test_asymmetric_on_word_embedding_stand_in():
    w = wl.scaled_down(wl.WORKLOADS["C4"], n=150_000, m=100)
    Xdb, Xq, scale = wl.database(w), wl.queries(w), wl.workload_scale(w)
    got = gu.gpu_search_asym(Xdb, Xq, 3, 4, 100, scale)
    gu.assert_same(got, gu.oracle_search_asym(Xdb, Xq, 3, 4, 100, scale), "C4 4x3")
    gu.check_order_properties(got[0], got[1], w.n)


def test_asymmetric_unsupported_pairs_are_refused():
    import torch
    t = torch.zeros(1 << 16, dtype=torch.int32, device="cuda")
    for qb, db in ((3, 4), (4, 2), (4, 1), (1, 2)):
        with pytest.raises(xbq.XbqError) as e:
            xbq.xbq_search_asym(t, 64, db, t, 4, qb, 32, 1)
        assert e.value.code == xbq.EUNSUPPORTED


REFINE = [
    # n, d, m, q_bits, db_bits, k, extra
    (6000, 128, 20, 4, 4, 10, 0),
    (6000, 128, 20, 4, 3, 10, 20),
    (30000, 128, 40, 4, 3, 100, 40),
    (30000, 96, 40, 4, 4, 100, 200),
    (20000, 200, 30, 4, 3, 10, 64),
    (4000, 960, 12, 4, 3, 10, 300),
    (3000, 64, 10, 3, 3, 1024, 10),
    (2000, 32, 16, 2, 2, 5, 3),
    (900, 128, 7, 4, 3, 10, 100000),       # every row is a candidate
]


@pytest.mark.parametrize("n,d,m,qb,db,k,extra", REFINE)
def test_search_refine_matches_algorithm_1(n, d, m, qb, db, k, extra):
    _say(f"refine n={n} d={d} m={m} {qb}x{db} k={k} extra={extra}")
    rng = np.random.default_rng(n + d + extra)
    Xdb = rng.standard_normal((n, d)).astype(np.float32)
    Xdb /= np.linalg.norm(Xdb, axis=1, keepdims=True)
    Xq = rng.standard_normal((m, d)).astype(np.float32)
    Xq /= np.linalg.norm(Xq, axis=1, keepdims=True)
    scale = wl.choose_scale(Xdb)
    got = gu.gpu_search_refine(Xdb, Xq, db, qb, k, extra, scale)
    D = gu.oracle_distances(Xdb, Xq, db, qb, scale)
    gu.assert_refined_matches(got, Xdb, Xq, D, k, extra, xbq.REFINE_MAX_CANDIDATES)


def test_refine_on_clustered_rows_and_sorted_rows():
    w = wl.scaled_down(wl.WORKLOADS["C4"], n=120_000, m=48)
    Xdb, Xq, scale = wl.database(w), wl.queries(w), wl.workload_scale(w)
    for extra in (0, 30, 120):
        _say(f"refine C4 stand-in extra={extra}")
        got = gu.gpu_search_refine(Xdb, Xq, 3, 4, 10, extra, scale)
        D = gu.oracle_distances(Xdb, Xq, 3, 4, scale)
        gu.assert_refined_matches(got, Xdb, Xq, D, 10, extra, xbq.REFINE_MAX_CANDIDATES)
    # adversarial order: rows ever closer to the query overflow the survivor lists
    order = np.argsort(Xdb @ Xq[0])
    Xs = np.ascontiguousarray(Xdb[order][:40_000])
    got = gu.gpu_search_refine(Xs, Xq[:4], 3, 4, 10, 50, scale)
    D = gu.oracle_distances(Xs, Xq[:4], 3, 4, scale)
    gu.assert_refined_matches(got, Xs, Xq[:4], D, 10, 50, xbq.REFINE_MAX_CANDIDATES)


def _one_bit_rows_at_distances(D, d, rng):
    """Rows of +-1/sqrt(d) whose one-bit code differs from the all-positive query in exactly
    D[r] coordinates (Eq. 10, the POPCNT form, with one plane on each side is the Hamming distance)."""
    n = len(D)
    X = np.full((n, d), 1.0, dtype=np.float32)
    for r in range(n):
        X[r, rng.choice(d, size=int(D[r]), replace=False)] = -1.0
    return X / np.float32(np.sqrt(d))


def test_cut_candidate_list_keeps_its_ties_through_the_exact_rescan():
    # One-bit codes, rows ever closer to query 0, massive ties.  With the default schedule the
    # group of rows 13 824 .. 20 735 overflows the survivor list of query 0 and is rescanned
    # exactly, starting from a list that was cut at 2048 rows of distance 50.  The rows at 48
    # and 49 then arrive in an order in which the rescan compacts its buffer while it holds rows
    # at the threshold distance: the 55 lowest-numbered rows at 49 belong to the first 2048
    # candidates, and xbq_k_select has to see that the bounded list is not the whole list.
    rng = np.random.default_rng(41)
    d, k, extra = 64, 100, 1
    D0 = np.concatenate([np.full(13_824, 50), np.full(200, 48), np.full(3896, 49), np.full(1793, 48),
                         np.full(20_736 - 13_824 - 5889, 60)])
    Xdb = _one_bit_rows_at_distances(D0, d, rng)
    Xq = np.concatenate([np.full((1, d), 1.0, dtype=np.float32),
                         rng.choice([-1.0, 1.0], size=(5, d)).astype(np.float32)]) / np.float32(np.sqrt(d))
    D = gu.oracle_distances(Xdb, Xq, 1, 1, 1.0)
    assert np.array_equal(D[0], D0)
    _say("one-bit sorted rows: xbq_search_refine")
    got = gu.gpu_search_refine(Xdb, Xq, 1, 1, k, extra, 1.0)
    assert got[2][0] == xbq.REFINE_MAX_CANDIDATES
    gu.assert_refined_matches(got, Xdb, Xq, D, k, extra, xbq.REFINE_MAX_CANDIDATES, tol=4e-6)
    try:
        xbq.xbq_set_option("kselect_lists_min", 0)           # first stage = the bounded candidate search
        _say("one-bit sorted rows: xbq_k_select")
        got = gu.gpu_k_select(Xdb, Xq, 1, 1, k, extra, len(Xdb), 1.0)
    finally:
        xbq.xbq_set_option("kselect_lists_min", 128)
    assert got[2][0] == 1993 + 3896
    gu.assert_refined_matches(got, Xdb, Xq, D, k, extra, len(Xdb), tol=4e-6, by_levels=True)


def test_candidate_search_on_sorted_tie_heavy_rows():
    rng = np.random.default_rng(43)
    d = 48
    for trial, (k, extra) in enumerate(((10, 0), (100, 2), (1000, 1))):
        D0 = np.sort(rng.integers(0, d + 1, size=30_000))[::-1]
        if trial == 1:
            D0 = np.concatenate([np.sort(c)[::-1] for c in np.array_split(rng.permutation(D0), 5)])
        Xdb = _one_bit_rows_at_distances(D0, d, rng)
        Xq = np.concatenate([np.full((1, d), 1.0, dtype=np.float32),
                             rng.choice([-1.0, 1.0], size=(3, d)).astype(np.float32)]) / np.float32(np.sqrt(d))
        D = gu.oracle_distances(Xdb, Xq, 1, 1, 1.0)
        _say(f"sorted tie-heavy rows k={k} extra={extra}")
        got = gu.gpu_search_refine(Xdb, Xq, 1, 1, k, extra, 1.0)
        gu.assert_refined_matches(got, Xdb, Xq, D, k, extra, xbq.REFINE_MAX_CANDIDATES, tol=4e-6)
        try:
            xbq.xbq_set_option("kselect_lists_min", 0)
            got = gu.gpu_k_select(Xdb, Xq, 1, 1, k, extra, 20_000, 1.0)
        finally:
            xbq.xbq_set_option("kselect_lists_min", 128)
        gu.assert_refined_matches(got, Xdb, Xq, D, k, extra, 20_000, tol=4e-6, by_levels=True)


KSELECT = [
    # n, d, m, q_bits, db_bits, k, extra, max_candidates
    (6000, 128, 20, 4, 4, 10, 0, 6000),            # nothing cut: Algorithm 1 as printed
    (6000, 128, 20, 4, 3, 10, 60, 6000),
    (30000, 96, 40, 4, 4, 100, 200, 30000),        # lists of several thousand rows, several refine pieces
    (20000, 200, 30, 4, 3, 10, 64, 20000),
    (4000, 960, 12, 4, 3, 10, 300, 4000),          # long codes: the chunked scan collects
    (3000, 64, 10, 3, 3, 1024, 10, 3000),
    (3000, 128, 1100, 4, 4, 10, 30, 3000),         # many queries: one refine workgroup per query
    (9000, 128, 3, 4, 4, 5, 4095, 9000),           # largest extra distance: every row is a candidate
    (900, 33, 1, 2, 2, 900, 0, 900),               # k = n
    (20000, 128, 24, 4, 4, 10, 120, 700),          # lists cut back to whole distance levels
    (20000, 128, 24, 4, 3, 100, 120, 130),
    (20000, 96, 24, 3, 3, 10, 50, 10),             # max_candidates = k
    (5000, 16, 9, 1, 1, 20, 3, 40),                # one-bit codes: few levels, massive ties
    (2000, 2048, 18, 4, 4, 5, 100, 2000),          # widest rows the library takes
    (3000, 64, 40, 3, 3, 1024, 10, 3000),          # largest k, first stage = bounded candidate search
    (50, 32, 20, 2, 2, 7, 2, 50),                  # fewer rows than a bundle
    (5000, 128, 200, 4, 3, 10, 40, 64),            # whole bounded lists that exceed the caller's bound
    (6000, 100, 300, 4, 4, 10, 4095, 6000),        # every row a candidate for 300 queries
    (20001, 128, 5, 4, 4, 10, 120, 700),           # few queries: collection from the stored distances, lists cut
    (9001, 96, 8, 4, 3, 100, 60, 9001),            # eight queries, row count not a multiple of four
    (70000, 64, 2, 3, 3, 10, 300, 70000),          # several workgroups per query, most rows candidates
]


@pytest.mark.parametrize("n,d,m,qb,db,k,extra,limit", KSELECT)
def test_k_select_matches_algorithm_1_with_whole_levels(n, d, m, qb, db, k, extra, limit):
    _say(f"k_select n={n} d={d} m={m} {qb}x{db} k={k} extra={extra} max_candidates={limit}")
    rng = np.random.default_rng(n + d + extra + limit)
    Xdb = rng.standard_normal((n, d)).astype(np.float32)
    Xdb /= np.linalg.norm(Xdb, axis=1, keepdims=True)
    Xq = rng.standard_normal((m, d)).astype(np.float32)
    Xq /= np.linalg.norm(Xq, axis=1, keepdims=True)
    scale = wl.choose_scale(Xdb)
    got = gu.gpu_k_select(Xdb, Xq, db, qb, k, extra, limit, scale)
    sub = np.arange(m) if m <= 48 else np.concatenate([np.arange(24), m - 1 - np.arange(24)])
    D = gu.oracle_distances(Xdb, Xq[sub], db, qb, scale)
    gu.assert_refined_matches(tuple(x[sub] for x in got), Xdb, Xq[sub], D, k, extra, limit, by_levels=True)


def test_k_select_result_does_not_depend_on_the_first_stage():
    rng = np.random.default_rng(5)
    Xdb = rng.standard_normal((30000, 128)).astype(np.float32)
    Xdb /= np.linalg.norm(Xdb, axis=1, keepdims=True)
    Xq = rng.standard_normal((150, 128)).astype(np.float32)
    Xq /= np.linalg.norm(Xq, axis=1, keepdims=True)
    scale = wl.choose_scale(Xdb)
    D = gu.oracle_distances(Xdb, Xq[:20], 4, 4, scale)
    try:
        for lists_min in (0, 1 << 20):
            for extra, limit in ((40, 30000), (200, 3000)):
                _say(f"k_select first stage: lists_min={lists_min} extra={extra} max_candidates={limit}")
                xbq.xbq_set_option("kselect_lists_min", lists_min)
                got = gu.gpu_k_select(Xdb, Xq, 4, 4, 10, extra, limit, scale)
                gu.assert_refined_matches(tuple(x[:20] for x in got), Xdb, Xq[:20], D, 10, extra, limit, by_levels=True)
    finally:
        xbq.xbq_set_option("kselect_lists_min", 128)


def test_k_select_ties_at_the_kth_distance_exceed_the_bound():
    # 40 distinct rows repeated 100 times: every distance level holds a multiple of 100 rows
    rng = np.random.default_rng(77)
    base = rng.standard_normal((40, 64)).astype(np.float32)
    base /= np.linalg.norm(base, axis=1, keepdims=True)
    Xdb = np.ascontiguousarray(np.tile(base, (100, 1)))
    Xq = base[:6] + 0.05 * rng.standard_normal((6, 64)).astype(np.float32)
    Xq /= np.linalg.norm(Xq, axis=1, keepdims=True)
    for k, extra, limit in ((10, 5, 50), (10, 5, 100), (150, 0, 160), (150, 40, 250), (3, 4095, 3)):
        _say(f"k_select ties k={k} extra={extra} max_candidates={limit}")
        got = gu.gpu_k_select(Xdb, Xq, 4, 4, k, extra, limit, 2.0)
        D = gu.oracle_distances(Xdb, Xq, 4, 4, 2.0)
        gu.assert_refined_matches(got, Xdb, Xq, D, k, extra, limit, by_levels=True)


def test_k_select_in_batches_and_on_clustered_rows():
    # a candidate bound of 40 000 rows makes batches of 6 710 queries: 7 000 queries take two
    w = wl.scaled_down(wl.WORKLOADS["C4"], n=40_000, m=7_000)
    Xdb, Xq, scale = wl.database(w), wl.queries(w), wl.workload_scale(w)
    _say("k_select two batches, C4 stand-in")
    got = gu.gpu_k_select(Xdb, Xq, 3, 4, 10, 80, 40_000, scale)
    sub = np.concatenate([np.arange(12), 6709 + np.arange(3), 6999 - np.arange(10)])
    D = gu.oracle_distances(Xdb, Xq[sub], 3, 4, scale)
    gu.assert_refined_matches(tuple(x[sub] for x in got), Xdb, Xq[sub], D, 10, 80, 40_000, by_levels=True)
    assert got[2].max() > xbq.REFINE_MAX_CANDIDATES          # lists longer than the other entry point can hold


DOT = [
    # n, d, m, q_bits, db_bits, k   (the cross-check scan serves d <= 256)
    (5000, 128, 300, 4, 4, 10),
    (20000, 128, 300, 4, 3, 100),
    (9000, 200, 280, 3, 3, 50),
    (9000, 96, 300, 4, 4, 100),
    (7000, 250, 290, 3, 2, 10),
    (6000, 33, 300, 2, 2, 5),
    (6000, 256, 270, 1, 1, 20),
    (4097, 8, 260, 2, 1, 64),
]


@pytest.mark.parametrize("kernel", [1, 2], ids=["dot8", "mfma"])
@pytest.mark.parametrize("n,d,m,qb,db,k", DOT)
def test_dot_product_cross_check_scan_gives_the_same_result(n, d, m, qb, db, k, kernel):
    _say(f"cross-check kernel={kernel} n={n} d={d} m={m} {qb}x{db} k={k}")
    Xdb = _rand(n, d, seed=n + d + 7)
    Xq = _rand(m, d, seed=n + d + 8)
    want = gu.oracle_search_asym(Xdb, Xq, db, qb, k, 2.1)
    xbq.xbq_set_option("kernel", kernel)
    xbq.xbq_set_option("selector", 1)
    try:
        gu.assert_same(gu.gpu_search_asym(Xdb, Xq, db, qb, k, 2.1), want, "dot cross-check")
    finally:
        xbq.xbq_set_option("kernel", 0)
        xbq.xbq_set_option("selector", 0)
    gu.assert_same(gu.gpu_search_asym(Xdb, Xq, db, qb, k, 2.1), want, "xor path")


def test_all_scores_tied(selector):
    # non-negative data at scale 1: every coordinate falls in the same cell, all scores equal
    w = wl.scaled_down(wl.WORKLOADS["C3"], n=30_000, m=16)
    Xdb, Xq = wl.database(w), wl.queries(w)
    idx, score = gu.gpu_search(Xdb, Xq, 3, 10, 1.0)
    gu.assert_same((idx, score), gu.oracle_search(Xdb, Xq, 3, 10, 1.0), "all tied")
    assert (idx == np.arange(10)[None, :]).all()


def test_duplicated_rows_and_few_distinct_scores(selector):
    base = _rand(500, 24, seed=5)
    Xdb = np.tile(base, (40, 1))                        # every row occurs 40 times
    Xq = _rand(12, 24, seed=6)
    for bits, k in ((1, 100), (2, 257), (4, 64)):
        gu.assert_same(gu.gpu_search(Xdb, Xq, bits, k, 1.5), gu.oracle_search(Xdb, Xq, bits, k, 1.5), "dups")


def test_rows_sorted_by_similarity_forces_exact_rescan(selector):
    # later rows are ever closer to the queries: every group floods the candidate lists,
    # which must overflow and take the exact rescan path
    rng = np.random.default_rng(17)
    d, n, m = 64, 40_000, 6
    target = rng.standard_normal(d).astype(np.float32)
    target /= np.linalg.norm(target)
    noise = rng.standard_normal((n, d)).astype(np.float32)
    amount = np.linspace(3.0, 0.0, n, dtype=np.float32)[:, None]
    Xdb = target[None, :] + amount * noise / np.sqrt(d)
    Xdb = (Xdb / np.linalg.norm(Xdb, axis=1, keepdims=True)).astype(np.float32)
    Xq = target[None, :] + 0.05 * rng.standard_normal((m, d)).astype(np.float32)
    Xq /= np.linalg.norm(Xq, axis=1, keepdims=True)
    Xq = Xq.astype(np.float32)
    for bits, k in ((4, 10), (3, 100), (4, 1024)):
        _say(f"sorted rows bits={bits} k={k}")
        gu.assert_same(gu.gpu_search(Xdb, Xq, bits, k, 3.0), gu.oracle_search(Xdb, Xq, bits, k, 3.0), "sorted")


def test_massive_ties_take_the_streaming_path_of_the_histogram_selector():
    # one bit, low dimension: a handful of distinct distances over 300k rows, so the boundary
    # bin holds far more rows than the sort buffer and than the candidate list (the selection
    # streams over all stored distances)
    Xdb = _rand(300_000, 8, seed=41)
    Xq = _rand(5, 8, seed=42)
    xbq.xbq_set_option("selector", 2)
    try:
        for bits, k in ((1, 100), (2, 1000)):
            gu.assert_same(gu.gpu_search(Xdb, Xq, bits, k, 1.5), gu.oracle_search(Xdb, Xq, bits, k, 1.5), "ties")
        # a tight cluster around the query: some ten thousand rows up to the boundary bin, more than
        # the sort buffer and fewer than the candidate list holds (the selection streams over the list)
        rng = np.random.default_rng(43)
        n, d = 200_000, 96
        centre = rng.standard_normal(d)
        X = rng.standard_normal((n, d))
        X[:30_000] = centre + 0.02 * rng.standard_normal((30_000, d))
        X = X[rng.permutation(n)]
        Xdb = (X / np.linalg.norm(X, axis=1, keepdims=True)).astype(np.float32)
        Q = centre + 0.02 * rng.standard_normal((6, d))
        Xq = (Q / np.linalg.norm(Q, axis=1, keepdims=True)).astype(np.float32)
        for bits, k in ((4, 100), (3, 1000), (4, 1)):
            _say(f"tight cluster, stored distances: bits={bits} k={k}")
            gu.assert_same(gu.gpu_search(Xdb, Xq, bits, k, 2.0), gu.oracle_search(Xdb, Xq, bits, k, 2.0), "tight cluster")
    finally:
        xbq.xbq_set_option("selector", 0)


def test_local_selection_on_massive_ties_and_odd_piece_sizes():
    # one or two bits, low dimension: every piece's boundary bin holds far more rows than its list,
    # so every workgroup re-selects its piece exactly and the merge streams over tied keys
    Xdb = _rand(300_000, 8, seed=41)
    Xq = _rand(5, 8, seed=42)
    want = {(bits, k): gu.oracle_search(Xdb, Xq, bits, k, 1.5) for bits, k in ((1, 100), (2, 256), (4, 7))}
    try:
        xbq.xbq_set_option("selector", 3)
        for groups in (256, 1, 37, 1024):
            xbq.xbq_set_option("local_groups", groups)
            for (bits, k), w in want.items():
                _say(f"local selection, ties: groups={groups} bits={bits} k={k}")
                gu.assert_same(gu.gpu_search(Xdb, Xq, bits, k, 1.5), w, f"ties groups={groups} bits={bits} k={k}")
    finally:
        xbq.xbq_set_option("local_groups", 256)
        xbq.xbq_set_option("selector", 0)


def test_local_selection_piece_sizes_and_query_passes():
    # random rows: piece sizes from one step of 1024 rows to the whole database, 1 .. 9 queries
    # (more than one pass of four), every supported list size (k <= 128: 1024 keys, k <= 256: 2048)
    rng = np.random.default_rng(47)
    for n, d, bits in ((70_001, 128, 4), (5_000, 200, 3), (200_000, 96, 4), (33_000, 960, 3)):
        Xdb = _rand(n, d, seed=n)
        for m, k in ((1, 100), (9, 10), (3, 256), (4, 129), (2, 1)):
            Xq = _rand(m, d, seed=n + m)
            want = gu.oracle_search(Xdb, Xq, bits, k, 2.0)
            for groups in (256, 3, 64, 1000):
                _say(f"local selection n={n} d={d} bits={bits} m={m} k={k} groups={groups}")
                try:
                    xbq.xbq_set_option("selector", 3)
                    xbq.xbq_set_option("local_groups", groups)
                    got = gu.gpu_search(Xdb, Xq, bits, k, 2.0)
                finally:
                    xbq.xbq_set_option("local_groups", 256)
                    xbq.xbq_set_option("selector", 0)
                gu.assert_same(got, want, f"local n={n} m={m} k={k} groups={groups}")


def test_local_selection_very_long_pieces_compact_their_lists():
    # one or two pieces of 200 000 to 400 000 rows: thousands of chunks per workgroup, so the lists
    # are compacted on the way (ordinary data, no overflow: the exact re-selection must not be what
    # makes this pass), with one query and with three
    n, d, bits = 400_000, 96, 4
    Xdb = _rand(n, d, seed=81)
    for m, k in ((1, 100), (3, 40), (4, 256)):
        Xq = _rand(m, d, seed=82 + m)
        want = gu.oracle_search(Xdb, Xq, bits, k, 2.0)
        for groups in (1, 2):
            _say(f"local selection, long pieces: m={m} k={k} groups={groups}")
            try:
                xbq.xbq_set_option("selector", 3)
                xbq.xbq_set_option("local_groups", groups)
                got = gu.gpu_search(Xdb, Xq, bits, k, 2.0)
            finally:
                xbq.xbq_set_option("local_groups", 256)
                xbq.xbq_set_option("selector", 0)
            gu.assert_same(got, want, f"long pieces m={m} k={k} groups={groups}")


def test_local_selection_on_rows_ordered_by_cluster():
    """Rows of a cluster next to each other, clusters in random order: inside a piece, whenever a
    cluster closer to the query begins, a burst of rows passes the threshold of the moment.  The
    lists then ask for compactions on the way (no key may be lost), tight clusters put thousands
    of distances into one histogram bin (the exact cut), and the result sits in one or two pieces
    (the merge has to read whole lists)."""
    rng = np.random.default_rng(91)
    n, d, bits = 300_000, 96, 4
    for ncl, spread in ((30, 0.25), (300, 0.05), (6, 0.02)):
        base = rng.standard_normal((ncl, d))
        lab = np.sort(rng.integers(ncl, size=n))
        X = base[lab] + spread * rng.standard_normal((n, d))
        Xdb = (X / np.linalg.norm(X, axis=1, keepdims=True)).astype(np.float32)
        Q = base[rng.integers(ncl, size=4)] + spread * rng.standard_normal((4, d))
        Xq = (Q / np.linalg.norm(Q, axis=1, keepdims=True)).astype(np.float32)
        for m, k in ((1, 100), (4, 100), (2, 256), (3, 10)):
            want = gu.oracle_search(Xdb, Xq[:m], bits, k, 2.0)
            for groups in (256, 8, 2):
                _say(f"rows ordered by cluster: clusters={ncl} spread={spread} m={m} k={k} groups={groups}")
                try:
                    xbq.xbq_set_option("selector", 3)
                    xbq.xbq_set_option("local_groups", groups)
                    got = gu.gpu_search(Xdb, Xq[:m], bits, k, 2.0)
                finally:
                    xbq.xbq_set_option("local_groups", 256)
                    xbq.xbq_set_option("selector", 0)
                gu.assert_same(got, want, f"clusters={ncl} m={m} k={k} groups={groups}")


def test_search_ex_takes_its_options_per_call():
    import torch
    Xdb = _rand(60_000, 128, seed=51)
    Xq = _rand(6, 128, seed=52)
    want = gu.oracle_search(Xdb, Xq, 4, 20, 2.0)
    db = xbq.xbq_encode(gu.to_dev(Xdb), 4, 2.0, xbq.BUNDLE64)
    q = xbq.xbq_encode(gu.to_dev(Xq), 4, 2.0, xbq.ROWS)
    for fields in ({"selector": 1}, {"selector": 2}, {"selector": 3}, {"selector": 3, "local_groups": 5},
                   {"selector": 1, "growth": 2.0, "first": 256, "qsplit": 3}, {"kernel": 1, "selector": 1}, {}):
        _say(f"xbq_search_ex options {fields}")
        idx, score = xbq.xbq_search_ex(db, 60_000, 4, q, 6, 4, 128, 20, xbq.xbq_options_default(**fields))
        torch.cuda.synchronize()
        gu.assert_same((idx.cpu().numpy(), score.cpu().numpy()), want, f"options {fields}")
    idx, score = xbq.xbq_search_ex(db, 60_000, 4, q, 6, 4, 128, 20, None)          # process-wide defaults
    torch.cuda.synchronize()
    gu.assert_same((idx.cpu().numpy(), score.cpu().numpy()), want, "default options")


def test_automatic_selector_switches_with_query_count():
    Xdb = _rand(40_000, 128, seed=43)
    want_few = gu.oracle_search(Xdb, _rand(9, 128, seed=44), 4, 10, 2.0)
    gu.assert_same(gu.gpu_search(Xdb, _rand(9, 128, seed=44), 4, 10, 2.0), want_few, "auto, 9 queries")
    Xq = _rand(700, 128, seed=45)
    gu.assert_same(gu.gpu_search(Xdb, Xq, 4, 10, 2.0), gu.oracle_search(Xdb, Xq, 4, 10, 2.0), "auto, 700 queries")
    # with a large k the histogram selection serves more queries (40 here), and the workspace says so
    Xq = _rand(40, 128, seed=46)
    gu.assert_same(gu.gpu_search(Xdb, Xq, 4, 1000, 2.0), gu.oracle_search(Xdb, Xq, 4, 1000, 2.0), "auto, k = 1000")
    assert xbq.xbq_search_workspace_bytes(40_000, 40, 128, 4, 1000) >= 8 * 40_000 * 4      # stored distances


def test_many_queries_cross_the_internal_batch():
    n, d, m = 3000, 32, 20_000                          # more queries than one internal batch
    Xdb = _rand(n, d, seed=1)
    Xq = _rand(m, d, seed=2)
    gu.assert_same(gu.gpu_search(Xdb, Xq, 4, 5, 2.0), gu.oracle_search(Xdb, Xq, 4, 5, 2.0), "batches")


def test_binding_checks_buffer_sizes_before_the_call():
    import torch
    n, d, bits, k, m = 1000, 128, 4, 10, 3
    Xh = _rand(n, d, seed=1)
    X = gu.to_dev(Xh)
    rows = xbq.xbq_encode(X, bits, 1.0, xbq.ROWS)                 # the default layout: not what the scan reads
    db = xbq.xbq_encode(X, bits, 1.0, xbq.BUNDLE64)
    q = xbq.xbq_encode(X[:m], bits, 1.0, xbq.ROWS)
    assert rows.numel() < db.numel()
    with pytest.raises(ValueError, match="BUNDLE64"):
        xbq.xbq_search(rows, n, q, m, d, bits, k)                 # too small for n rows in bundles
    with pytest.raises(ValueError, match="q_codes"):
        xbq.xbq_search(db, n, q[:-1], m, d, bits, k)
    with pytest.raises(ValueError, match="db_codes"):
        xbq.xbq_search(db, n + 64, q, m, d, bits, k)              # more rows claimed than encoded
    with pytest.raises(ValueError, match="idx"):
        xbq.xbq_search(db, n, q, m, d, bits, k, idx=torch.empty((m, k + 1), dtype=torch.int32, device="cuda"))
    with pytest.raises(ValueError, match="score"):
        xbq.xbq_search(db, n, q, m, d, bits, k, score=torch.empty((m, k), dtype=torch.float32, device="cuda"))
    with pytest.raises(xbq.XbqError):
        xbq.xbq_search(db, n, q, m, d, bits, k, workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    with pytest.raises(ValueError, match="candidates"):
        xbq.xbq_k_select(X, db, bits, X[:m], q, bits, k, 5, 100, cand=torch.empty((m + 1,), dtype=torch.int32, device="cuda"))
    idx, score = xbq.xbq_search(db, n, q, m, d, bits, k)          # and the well-formed call goes through
    torch.cuda.synchronize()
    gu.assert_same((idx.cpu().numpy(), score.cpu().numpy()), gu.oracle_search(Xh, Xh[:m], bits, k, 1.0), "well-formed call")


def test_empty_inputs_are_noops():
    import torch
    db = torch.zeros(64 * 16, dtype=torch.int32, device="cuda")
    q = torch.zeros(16, dtype=torch.int32, device="cuda")
    idx, score = xbq.xbq_search(db, 0, q, 1, 128, 4, 1)
    idx, score = xbq.xbq_search(db, 64, q, 0, 128, 4, 1)
    assert idx.shape == (0, 1)
    out = xbq.xbq_encode(torch.zeros((0, 128), device="cuda"), 4)
    assert out.numel() == 0
    torch.cuda.synchronize()


def test_options_do_not_change_results():
    Xdb = _rand(30_000, 128, seed=3)
    Xq = _rand(64, 128, seed=4)
    want = gu.oracle_search(Xdb, Xq, 4, 100, 2.0)
    xbq.xbq_set_option("selector", 1)
    try:
        for growth, first, qsplit in ((1.5, 1024, 0), (4.0, 512, 16), (8.0, 4096, 1000), (2.0, 64, 7)):
            for row_order in (0, 1):
                xbq.xbq_set_option("growth", growth)
                xbq.xbq_set_option("first", first)
                xbq.xbq_set_option("qsplit", qsplit)
                xbq.xbq_set_option("row_order", row_order)
                gu.assert_same(gu.gpu_search(Xdb, Xq, 4, 100, 2.0), want,
                               f"growth={growth} first={first} row_order={row_order}")
    finally:
        xbq.xbq_set_option("growth", 4.0)
        xbq.xbq_set_option("first", 1024)
        xbq.xbq_set_option("qsplit", 0)
        xbq.xbq_set_option("row_order", 0)
        xbq.xbq_set_option("selector", 0)


def test_row_groups_in_either_order_on_ties_and_ordered_rows():
    """The threshold schedule with its row groups spread over the database (default) and as
    consecutive rows: same results on tie-heavy codes (a later group may hold a lower row with the
    same distance), on rows sorted towards the query, on rows ordered by cluster, through the plain
    search, the bounded candidate search and the whole-list K-select."""
    rng = np.random.default_rng(101)
    n, d = 50_000, 64
    base = rng.standard_normal((40, d))
    lab = np.sort(rng.integers(40, size=n))
    X = base[lab] + 0.1 * rng.standard_normal((n, d))
    Xcl = (X / np.linalg.norm(X, axis=1, keepdims=True)).astype(np.float32)
    Xq = _rand(40, d, seed=102)
    Xq[:8] = Xcl[rng.integers(n, size=8)]
    order = np.argsort(-(Xcl @ Xq[0]))                   # rows sorted towards query 0, best last
    Xsorted = np.ascontiguousarray(Xcl[order[::-1]])
    try:
        xbq.xbq_set_option("selector", 1)
        for row_order in (0, 1):
            xbq.xbq_set_option("row_order", row_order)
            for name, Xdb in (("clusters", Xcl), ("sorted", Xsorted)):
                for bits, k in ((1, 100), (2, 10), (4, 100), (3, 1000)):
                    _say(f"row_order={row_order} rows={name} bits={bits} k={k}")
                    gu.assert_same(gu.gpu_search(Xdb, Xq, bits, k, 2.0), gu.oracle_search(Xdb, Xq, bits, k, 2.0),
                                   f"row_order={row_order} {name} bits={bits} k={k}")
                sub = np.arange(16)
                for bits, k, extra in ((4, 10, 30), (1, 20, 0), (3, 50, 200)):
                    _say(f"row_order={row_order} rows={name} refine bits={bits} k={k} extra={extra}")
                    D = gu.oracle_distances(Xdb, Xq[sub], bits, bits, 2.0)
                    got = gu.gpu_search_refine(Xdb, Xq, bits, bits, k, extra, 2.0)
                    gu.assert_refined_matches(tuple(x[sub] for x in got), Xdb, Xq[sub], D, k, extra,
                                              xbq.REFINE_MAX_CANDIDATES)
                    xbq.xbq_set_option("kselect_lists_min", 0)
                    got = gu.gpu_k_select(Xdb, Xq, bits, bits, k, extra, n, 2.0)
                    xbq.xbq_set_option("kselect_lists_min", 128)
                    gu.assert_refined_matches(tuple(x[sub] for x in got), Xdb, Xq[sub], D, k, extra, n, by_levels=True)
    finally:
        xbq.xbq_set_option("kselect_lists_min", 128)
        xbq.xbq_set_option("row_order", 0)
        xbq.xbq_set_option("selector", 0)


def test_trace_reports_scan_time():
    Xdb = _rand(50_000, 128, seed=8)
    Xq = _rand(300, 128, seed=9)
    xbq.xbq_trace_enable(True)
    try:
        gu.gpu_search(Xdb, Xq, 4, 10, 2.0)
        ms, launches, pairs = xbq.xbq_trace_read()
    finally:
        xbq.xbq_trace_enable(False)
    assert launches >= 2 and ms > 0
    assert pairs == 50_000 * 300


def test_search_can_be_captured_in_a_hip_graph_and_replayed():
    """The library allocates nothing, clears with kernels and never synchronises, so a search
    can be captured once and replayed on new queries written into the same buffers."""
    import torch
    n, d, bits, k = 60_000, 128, 4, 10
    Xdb = _rand(n, d, seed=51)
    db = xbq.xbq_encode(gu.to_dev(Xdb), bits, 2.0, xbq.BUNDLE64)
    planes = oc.encode(Xdb, bits, 2.0)
    for m in (1, 3, 300):                                # local selection (one query; three: 108 KB of LDS), threshold selector
        xq = torch.zeros((m, d), dtype=torch.float32, device="cuda")
        q = torch.zeros(xbq.xbq_code_bytes(m, d, bits, xbq.ROWS) // 4, dtype=torch.int32, device="cuda")
        ws = torch.empty(xbq.xbq_search_workspace_bytes(n, m, d, bits, k), dtype=torch.uint8, device="cuda")
        idx = torch.empty((m, k), dtype=torch.int32, device="cuda")
        score = torch.empty((m, k), dtype=torch.int32, device="cuda")

        def run():
            xbq.xbq_encode(xq, bits, 2.0, xbq.ROWS, out=q)
            xbq.xbq_search(db, n, q, m, d, bits, k, workspace=ws, idx=idx, score=score)

        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            run()                                         # warm-up outside the capture
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            run()
        for rep in range(4):
            Xq = _rand(m, d, seed=60 + rep)
            xq.copy_(torch.from_numpy(Xq))                # eager work between the replays
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            want = oc.search(planes, oc.encode(Xq, bits, 2.0), d, k)
            gu.assert_same((idx.cpu().numpy(), score.cpu().numpy()), want, f"graph replay {rep}, m={m}")


def test_k_select_can_be_captured_in_a_hip_graph_and_replayed():
    """Same for Algorithm 1 with the whole candidate list: its flags, counters and level counts
    are cleared by kernels, and the collecting scans that have nothing to do return by themselves."""
    import torch
    n, d, bits, k, extra, limit = 40_000, 96, 4, 10, 80, 1500
    rng = np.random.default_rng(7)
    Xdb = rng.standard_normal((n, d)).astype(np.float32)
    Xdb /= np.linalg.norm(Xdb, axis=1, keepdims=True)
    scale = wl.choose_scale(Xdb)
    xd = gu.to_dev(Xdb)
    db = xbq.xbq_encode(xd, bits, scale, xbq.BUNDLE64)
    for m in (4, 12, 200):                  # stored distances; plain search + scans; bounded lists + scans
        xq = torch.zeros((m, d), dtype=torch.float32, device="cuda")
        q = torch.zeros(xbq.xbq_code_bytes(m, d, bits, xbq.ROWS) // 4, dtype=torch.int32, device="cuda")
        ws = torch.empty(xbq.lib().xbq_k_select_workspace_bytes(n, m, d, bits, k, extra, limit), dtype=torch.uint8,
                         device="cuda")
        idx = torch.empty((m, k), dtype=torch.int32, device="cuda")
        sim = torch.empty((m, k), dtype=torch.float32, device="cuda")
        cand = torch.empty((m,), dtype=torch.int32, device="cuda")

        def run():
            xbq.xbq_encode(xq, bits, scale, xbq.ROWS, out=q)
            xbq.xbq_k_select(xd, db, bits, xq, q, bits, k, extra, limit, workspace=ws, idx=idx, sim=sim, cand=cand)

        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            run()                                         # warm-up outside the capture
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            run()
        for rep in range(3):
            Xq = rng.standard_normal((m, d)).astype(np.float32)
            Xq /= np.linalg.norm(Xq, axis=1, keepdims=True)
            xq.copy_(torch.from_numpy(Xq))                # eager work between the replays
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            sub = np.arange(min(m, 16))
            D = gu.oracle_distances(Xdb, Xq[sub], bits, bits, scale)
            got = (idx.cpu().numpy()[sub], sim.cpu().numpy()[sub], cand.cpu().numpy()[sub])
            gu.assert_refined_matches(got, Xdb, Xq[sub], D, k, extra, limit, by_levels=True)


def test_random_shapes_against_the_oracle():
    """Seeded sweep over valid shapes: dimensions around word and chunk boundaries, row counts
    around bundle and group boundaries, every supported pair of code widths, both selectors."""
    rng = np.random.default_rng(2024)
    dims = [1, 7, 31, 32, 33, 63, 64, 65, 95, 96, 127, 128, 129, 200, 255, 256, 257, 288, 511, 700, 1023, 1500]
    rows = [1, 2, 63, 64, 65, 127, 128, 1000, 1023, 1024, 1025, 1535, 1536, 1537, 4095, 4096, 4097, 5121, 9999]
    pairs = [(1, 1), (2, 2), (3, 3), (4, 4), (2, 1), (3, 2), (4, 3)]
    try:
        for trial in range(36):
            d = int(rng.choice(dims))
            n = int(rng.choice(rows))
            qb, db = pairs[int(rng.integers(len(pairs)))]
            m = int(rng.choice([1, 3, 8, 9, 17, 40, 130]))
            k = int(min(n, rng.choice([1, 2, 10, 64, 100, 513, 1024])))
            sel = int(rng.choice([1, 2]))
            scale = float(rng.choice([1.0, 1.7, 3.3]))
            _say(f"trial {trial}: n={n} d={d} m={m} {qb}x{db} k={k} selector={sel} scale={scale}")
            Xdb = _rand(n, d, seed=1000 + trial)
            Xq = _rand(m, d, seed=2000 + trial)
            xbq.xbq_set_option("selector", sel)
            gu.assert_same(gu.gpu_search_asym(Xdb, Xq, db, qb, k, scale), gu.oracle_search_asym(Xdb, Xq, db, qb, k, scale),
                           f"trial {trial}")
    finally:
        xbq.xbq_set_option("selector", 0)


def test_random_shapes_through_every_search_entry_point():
    """Seeded sweep like the one above, over the three kinds of search call and four kinds of
    rows (uniform, Gaussian, all-positive, tight clusters with many near-ties), rows normalised."""
    rng = np.random.default_rng(31337)
    dims = [1, 7, 31, 32, 33, 64, 65, 96, 127, 128, 129, 200, 256, 257, 288, 700, 960, 1500, 2048]
    rows = [1, 2, 63, 64, 65, 128, 1000, 1024, 1025, 1536, 4096, 4097, 5121, 9999, 20011]
    pairs = [(1, 1), (2, 2), (3, 3), (4, 4), (2, 1), (3, 2), (4, 3)]

    def draw(n, d, kind):
        if kind == 0:
            X = rng.uniform(-0.5, 0.5, (n, d))
        elif kind == 1:
            X = rng.standard_normal((n, d))
        elif kind == 2:
            X = np.abs(rng.standard_normal((n, d)))
        else:
            base = rng.standard_normal((max(1, n // 50), d))
            X = base[rng.integers(len(base), size=n)] + 0.05 * rng.standard_normal((n, d))
        return (X / np.maximum(np.linalg.norm(X, axis=1, keepdims=True), 1e-9)).astype(np.float32)

    try:
        for trial in range(60):
            d = int(rng.choice(dims))
            n = int(rng.choice(rows))
            qb, db = pairs[int(rng.integers(len(pairs)))]
            m = int(rng.choice([1, 3, 8, 9, 17, 40, 130, 300]))
            k = int(min(n, rng.choice([1, 2, 10, 64, 100, 513, 1024])))
            kind = int(rng.integers(4))
            scale = float(rng.choice([1.0, 1.7, 3.3]))
            call = int(rng.integers(3))
            Xdb, Xq = draw(n, d, kind), draw(m, d, kind)
            sub = np.arange(min(m, 16))
            if call == 0:
                sel = int(rng.choice([0, 1, 2]))
                _say(f"trial {trial}: search n={n} d={d} m={m} {qb}x{db} k={k} rows={kind} selector={sel}")
                xbq.xbq_set_option("selector", sel)
                gu.assert_same(gu.gpu_search_asym(Xdb, Xq, db, qb, k, scale),
                               gu.oracle_search_asym(Xdb, Xq, db, qb, k, scale), f"trial {trial}")
                xbq.xbq_set_option("selector", 0)
            elif call == 1:
                extra = int(rng.choice([0, 3, 40, 300, 100000]))
                _say(f"trial {trial}: refine n={n} d={d} m={m} {qb}x{db} k={k} rows={kind} extra={extra}")
                got = gu.gpu_search_refine(Xdb, Xq, db, qb, k, extra, scale)
                D = gu.oracle_distances(Xdb, Xq[sub], db, qb, scale)
                gu.assert_refined_matches(tuple(x[sub] for x in got), Xdb, Xq[sub], D, k, extra,
                                          xbq.REFINE_MAX_CANDIDATES)
            else:
                extra = int(rng.choice([0, 3, 40, 300, 4095]))
                limit = int(rng.choice([k, k + 7, max(k, n // 10), max(k, n // 2), n, 4 * n + 5]))
                lists_min = int(rng.choice([0, 128, 1 << 20]))
                _say(f"trial {trial}: k_select n={n} d={d} m={m} {qb}x{db} k={k} rows={kind} extra={extra} "
                     f"max_candidates={limit} lists_min={lists_min}")
                xbq.xbq_set_option("kselect_lists_min", lists_min)
                got = gu.gpu_k_select(Xdb, Xq, db, qb, k, extra, limit, scale)
                xbq.xbq_set_option("kselect_lists_min", 128)
                D = gu.oracle_distances(Xdb, Xq[sub], db, qb, scale)
                gu.assert_refined_matches(tuple(x[sub] for x in got), Xdb, Xq[sub], D, k, extra, min(limit, n),
                                          by_levels=True)
    finally:
        xbq.xbq_set_option("selector", 0)
        xbq.xbq_set_option("kselect_lists_min", 128)


def test_random_shapes_local_selection():
    """Seeded sweep over the local selection (selector 3, options per call): one to nine queries
    (up to three passes), every supported pair of code widths, piece counts from one to a
    thousand, k up to its limit of 256, and four kinds of rows including tight clusters, whose
    near-ties fill boundary bins and whose order puts most of a result into few pieces."""
    import torch
    rng = np.random.default_rng(777)
    dims = [1, 7, 31, 32, 33, 64, 65, 96, 127, 128, 129, 200, 256, 257, 288, 700, 960, 2048]
    rows = [1, 2, 63, 64, 65, 128, 1000, 1024, 1025, 1536, 4096, 4097, 5121, 9999, 20011, 70001, 150000]
    pairs = [(1, 1), (2, 2), (3, 3), (4, 4), (2, 1), (3, 2), (4, 3)]

    def draw(n, d, kind):
        if kind == 0:
            X = rng.uniform(-0.5, 0.5, (n, d))
        elif kind == 1:
            X = rng.standard_normal((n, d))
        elif kind == 2:
            X = np.abs(rng.standard_normal((n, d)))
        else:                                            # clusters, rows of a cluster next to each other
            base = rng.standard_normal((max(1, n // 50), d))
            X = base[np.sort(rng.integers(len(base), size=n))] + 0.05 * rng.standard_normal((n, d))
        return (X / np.maximum(np.linalg.norm(X, axis=1, keepdims=True), 1e-9)).astype(np.float32)

    for trial in range(48):
        d = int(rng.choice(dims))
        n = int(rng.choice(rows))
        if n * d > 40_000_000:
            n = 40_000_000 // d
        qb, db_bits = pairs[int(rng.integers(len(pairs)))]
        m = int(rng.choice([1, 1, 2, 3, 4, 5, 9]))
        k = int(min(n, rng.choice([1, 2, 10, 64, 100, 200, 256])))
        groups = int(rng.choice([1, 2, 7, 64, 256, 1000]))
        kind = int(rng.integers(4))
        scale = float(rng.choice([1.0, 1.7, 3.3]))
        _say(f"trial {trial}: local n={n} d={d} m={m} {qb}x{db_bits} k={k} groups={groups} rows={kind} scale={scale}")
        Xdb, Xq = draw(n, d, kind), draw(m, d, kind)
        db = xbq.xbq_encode(gu.to_dev(Xdb), db_bits, scale, xbq.BUNDLE64)
        q = xbq.xbq_encode(gu.to_dev(Xq), qb, scale, xbq.ROWS)
        idx, score = xbq.xbq_search_ex(db, n, db_bits, q, m, qb, d, k,
                                       xbq.xbq_options_default(selector=3, local_groups=groups))
        torch.cuda.synchronize()
        gu.assert_same((idx.cpu().numpy(), score.cpu().numpy()), gu.oracle_search_asym(Xdb, Xq, db_bits, qb, k, scale),
                       f"trial {trial}")
