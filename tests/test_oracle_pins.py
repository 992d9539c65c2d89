"""Pins of the definition-level oracle against what the paper and arithmetic fix.

None of these tests re-types an oracle formula: each compares an oracle function
with a printed value, a closed form from another derivation, a textbook special
case, an invariant, or brute force over a different decomposition.
"""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import definition as od


def _rows(path):
    out = []
    with open(path) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                out.append(line.split())
    return out


# ---------------------------------------------------------------- Section 3.1
def test_sigma_is_group_isomorphism():
    # Proposition 1: product in {+1,-1} corresponds to XOR in {0,1}; identities map.
    assert od.sigma(1) == 0 and od.sigma(-1) == 1
    for a1, a2 in itertools.product((1, -1), repeat=2):
        assert od.sigma(a1 * a2) == od.sigma(a1) ^ od.sigma(a2)
        assert a1 * a2 == 1 - 2 * (od.sigma(a1) ^ od.sigma(a2))       # Eq. 2
        assert od.sigma_inv(od.sigma(a1)) == a1


# ---------------------------------------------------------------- Section 3.2
def test_b1_values_from_appendix(golden_dir):
    for x, want in _rows(os.path.join(golden_dir, "b1_values.txt")):
        got = od.decode_value(od.quantize_code(float(x), 1), 1)
        assert got == float(want), (x, got)


def test_hand_worked_examples(golden_dir):
    for B, t, code, value in _rows(os.path.join(golden_dir, "hand_examples.txt")):
        B, t, code, value = int(B), float(t), int(code), float(value)
        assert od.quantize_code(t, B) == code, (B, t)
        assert od.decode_value(code, B) == value, (B, t)
        arr = od.encode(np.array([[t]], dtype=np.float32), B)
        assert int(arr[0, 0]) == od.quantize_code(float(np.float32(t)), B)


def _sweep_points(B):
    pts = list(np.linspace(-0.999999, 0.999999, 4001))
    for k in range(-(1 << B), (1 << B) + 1):          # every cell boundary +- 1 ulp (fp32)
        c = np.float32(k / float(1 << B))
        pts += [float(c), float(np.nextafter(c, np.float32(2))), float(np.nextafter(c, np.float32(-2)))]
    rng = np.random.default_rng(7)
    pts += list(rng.uniform(-1, 1, 2000))
    return [p for p in pts if -1.0 < p < 1.0]


@pytest.mark.parametrize("B", range(1, 9))
def test_error_bound_prop2(B):
    # Proposition 2: |f_B(x) - x| <= 2^-B on (-1, 1).
    for x in _sweep_points(B):
        xb = od.decode_value(od.quantize_code(x, B), B)
        assert abs(xb - x) <= 2.0 ** (-B), (B, x, xb)


@pytest.mark.parametrize("B", range(2, 9))
def test_recursion_from_appendix(B):
    # Appendix A: f_k(x) - f_{k-1}(x) = +2^-k when x >= f_{k-1}(x), else -2^-k.
    for x in _sweep_points(B)[::7]:
        prev = od.decode_value(od.quantize_code(x, B - 1), B - 1)
        cur = od.decode_value(od.quantize_code(x, B), B)
        want = 2.0 ** (-B) if x >= prev else -(2.0 ** (-B))
        assert cur - prev == want, (B, x)


@pytest.mark.parametrize("B", range(1, 9))
def test_values_are_odd_multiples_and_monotone(B):
    xs = sorted(_sweep_points(B))
    prev = -math.inf
    for x in xs:
        code = od.quantize_code(x, B)
        m = od.decode_numerator(code, B)
        assert abs(m) % 2 == 1                                # odd numerator
        assert abs(m) <= (1 << B) - 1
        v = od.decode_value(code, B)
        assert v == m / float(1 << B)
        assert v >= prev
        prev = v


@pytest.mark.parametrize("B", range(1, 9))
def test_equals_uniform_midrise_quantizer(B):
    # Textbook special case: f_B is the uniform mid-rise quantizer of step 2^(1-B)
    # with saturation; cell index j counted from the bottom, stored code = 2^B-1-j.
    half = 1 << (B - 1)
    pts = _sweep_points(B) + [1.0, -1.0, 1.5, -3.0, 1e30, -1e30, 0.0, -0.0]
    for x in pts:
        j = min(max(math.floor(x * half) + half, 0), (1 << B) - 1)
        assert od.quantize_code(x, B) == (1 << B) - 1 - j, (B, x)


def test_saturation_and_signed_zero():
    assert od.quantize_code(1.0, 4) == 0 and od.quantize_code(123.0, 4) == 0
    assert od.quantize_code(-1.0, 4) == 15 and od.quantize_code(-123.0, 4) == 15
    assert od.quantize_code(float("inf"), 3) == 0 and od.quantize_code(float("-inf"), 3) == 7
    assert od.quantize_code(-0.0, 4) == od.quantize_code(0.0, 4) == 7       # sign(0) = +1


def test_vectorised_encode_matches_scalar_and_uses_fp32_scaling():
    rng = np.random.default_rng(3)
    X = rng.uniform(-0.4, 0.4, size=(5, 37)).astype(np.float32)
    scale = 2.95
    for B in (1, 3, 4, 8):
        got = od.encode(X, B, scale)
        for r in range(X.shape[0]):
            for k in range(X.shape[1]):
                t = float(np.float32(X[r, k]) * np.float32(scale))        # binary32 product
                assert int(got[r, k]) == od.quantize_code(t, B)
    # a point where rounding the product to fp32 decides the cell: the fp32 product of
    # these two is exactly 0.25 while the real product is just below it
    x = np.float32(0.083333336)
    s = np.float32(3.0)
    assert float(x * s) == 0.25 and float(x) * 3.0 != 0.25
    assert int(od.encode(np.array([[x]]), 3, float(s))[0, 0]) == od.quantize_code(0.25, 3)


# ------------------------------------------------- Section 3.2, operator and Eq. 5
@pytest.mark.parametrize("Bx,By", [(3, 3), (4, 4), (4, 3), (1, 1), (2, 5), (8, 8)])
def test_scalar_product_identity_exhaustive(Bx, By):
    # Eq. 5: x_B * y_B = ((2^Bx-1)(2^By-1) - 2 xbar(x)ybar) / 2^(Bx+By); left side from
    # the digit sums, right side from the XOR operator, over every pair of codes.
    for xbar in range(1 << Bx):
        for ybar in range(1 << By):
            lhs = od.decode_value(xbar, Bx) * od.decode_value(ybar, By)     # exact (dyadic)
            rhs = od.product_numerator(xbar, ybar, Bx, By) / float(1 << (Bx + By))
            assert lhs == rhs


def test_self_otimes_table_b3():
    # worked from the definition for B = 3: xbar (x) xbar for xbar = 0..7
    assert [od.otimes_scalar(c, c, 3, 3) for c in range(8)] == [0, 12, 20, 24, 24, 20, 12, 0]
    # and the pair of the hand example: codes 2 and 6 give 32, numerator 49 - 64 = -15
    assert od.otimes_scalar(2, 6, 3, 3) == 32
    assert od.product_numerator(2, 6, 3, 3) == -15 == 3 * -5


def test_query4_doc3_affine_relation():
    # Section 3.6: with 4-bit queries and 3-bit documents,
    # Distance = constant - 64 * ScaledSimilarity, constant = d * 15 * 7 / 2.
    rng = np.random.default_rng(11)
    d = 40
    for _ in range(50):
        cq = rng.integers(0, 16, d)
        cd = rng.integers(0, 8, d)
        dist = od.otimes_vector(cq, cd, 4, 3)
        ss = sum(od.decode_value(int(a), 4) * od.decode_value(int(b), 3) for a, b in zip(cq, cd))
        assert dist == 52.5 * d - 64.0 * ss


# ------------------------------------------------------- Section 3.3, planes (Eq. 9), POPCNT form (Eq. 10)
@pytest.mark.parametrize("d", [1, 5, 31, 32, 33, 64, 65, 96, 100, 200])
@pytest.mark.parametrize("Bx,By", [(3, 3), (4, 4), (4, 3), (1, 1), (2, 7)])
def test_popcount_form_equals_per_coordinate_operator_and_integer_dot(d, Bx, By):
    rng = np.random.default_rng(d * 100 + Bx * 10 + By)
    cx = rng.integers(0, 1 << Bx, d)
    cy = rng.integers(0, 1 << By, d)
    per_coord = od.otimes_vector(cx, cy, Bx, By)
    planes = od.popcount_distance_ints(od.plane_ints(cx, Bx), od.plane_ints(cy, By))
    assert planes == per_coord                                              # Eq. 10 = Eq. 8
    # Eq. 7: the score is the integer dot product of the decoded numerators
    mx = [sum((1 << i) if not (int(c) >> i) & 1 else -(1 << i) for i in range(Bx)) for c in cx]
    my = [sum((1 << i) if not (int(c) >> i) & 1 else -(1 << i) for i in range(By)) for c in cy]
    dot = sum(a * b for a, b in zip(mx, my))
    assert od.score_from_distance(planes, d, Bx, By) == dot


@pytest.mark.parametrize("d", [1, 31, 32, 33, 64, 96, 130, 200])
def test_packed_words_match_plane_integers(d):
    rng = np.random.default_rng(d)
    B = 4
    codes = rng.integers(0, 16, size=(3, d)).astype(np.uint8)
    words = od.pack_planes(codes, B)
    W = (d + 31) // 32
    assert words.shape == (3, B, W) and words.dtype == np.uint32
    for r in range(3):
        ints = od.plane_ints(codes[r], B)
        for b in range(B):
            rebuilt = sum(int(words[r, b, w]) << (32 * w) for w in range(W))
            assert rebuilt == ints[b]
            assert rebuilt >> d == 0                                        # pad bits are zero


def test_storage_example_32d_b3(golden_dir):
    kv = {k: int(v) for k, v in _rows(os.path.join(golden_dir, "worked_example_32d.txt"))}
    d, B = kv["dimension"], kv["bits"]
    codes = np.random.default_rng(0).integers(0, 1 << B, size=(2, d)).astype(np.uint8)
    words = od.pack_planes(codes, B)
    assert d * B == kv["code_bits_per_vector"]
    assert words.shape[1] * words.shape[2] == kv["plane_integers_per_vector"]
    assert words.dtype.itemsize == kv["bytes_per_plane_integer"]
    assert len(list(itertools.product(range(B), range(B)))) * words.shape[2] == kv["xor_popcnt_pairs"]
    assert (d * B) ** 2 == kv["bitwise_xors_without_planes"]
    assert d == kv["multiplies_without_encoding"]


def test_distance_matrix_matches_scalar_path_with_padding():
    rng = np.random.default_rng(5)
    for d, Bq, Bd in [(70, 4, 4), (33, 4, 3), (200, 3, 3), (96, 1, 1)]:
        cq = rng.integers(0, 1 << Bq, size=(4, d)).astype(np.uint8)
        cd = rng.integers(0, 1 << Bd, size=(9, d)).astype(np.uint8)
        D = od.distance_matrix(od.pack_planes(cq, Bq), od.pack_planes(cd, Bd))
        for a in range(4):
            for r in range(9):
                assert D[a, r] == od.otimes_vector(cq[a], cd[r], Bq, Bd)


def test_one_bit_reduces_to_sign_hamming():
    # B = 1: S = d - 2 * Hamming(sign bits)  (textbook sign-bit cosine estimate)
    rng = np.random.default_rng(9)
    X = rng.standard_normal((6, 77)).astype(np.float32)
    Y = rng.standard_normal((5, 77)).astype(np.float32)
    S = od.score_matrix(od.pack_planes(od.encode(Y, 1), 1), od.pack_planes(od.encode(X, 1), 1), 77, 1, 1)
    ham = ((Y[:, None, :] < 0) != (X[None, :, :] < 0)).sum(axis=2)
    assert np.array_equal(S, 77 - 2 * ham)


def test_score_invariants():
    rng = np.random.default_rng(13)
    d, B = 50, 4
    C = rng.integers(0, 16, size=(12, d)).astype(np.uint8)
    P = od.pack_planes(C, B)
    S = od.score_matrix(P, P, d, B, B)
    M = od.decode(C, B)
    assert np.array_equal(S, S.T)                                            # symmetry
    assert np.array_equal(np.diag(S), (M * M).sum(axis=1))                   # S(x,x) = |m|^2 > 0
    assert (np.diag(S) > 0).all()
    assert (S.astype(np.int64) ** 2 <= np.outer(np.diag(S), np.diag(S))).all()   # Cauchy-Schwarz
    assert (S % 2 == d % 2).all()                                            # sum of d odd products
    # bit-complement decodes to the negated vector
    Pc = od.pack_planes((15 - C).astype(np.uint8), B)
    assert np.array_equal(od.score_matrix(Pc, P, d, B, B), -S)
    # saturated codes reach the global maximum d (2^B-1)^2 and distance 0 to themselves
    sat = (rng.integers(0, 2, size=(3, d)) * 15).astype(np.uint8)
    Ps = od.pack_planes(sat, B)
    assert (np.diag(od.score_matrix(Ps, Ps, d, B, B)) == d * 225).all()
    assert (np.diag(od.distance_matrix(Ps, Ps)) == 0).all()


def test_score_equals_fp_gemm_of_decoded_vectors():
    # every partial sum is an integer far below 2^53: the float64 GEMM is exact
    rng = np.random.default_rng(17)
    d = 200
    Cq = rng.integers(0, 16, size=(7, d)).astype(np.uint8)
    Cd = rng.integers(0, 8, size=(40, d)).astype(np.uint8)
    S = od.score_matrix(od.pack_planes(Cq, 4), od.pack_planes(Cd, 3), d, 4, 3)
    G = od.decode(Cq, 4).astype(np.float64) @ od.decode(Cd, 3).astype(np.float64).T
    assert np.array_equal(S, G.astype(np.int64))


# ---------------------------------------------------------------------- top-K
def _brute_topk(row, K):
    return sorted(range(len(row)), key=lambda i: (-int(row[i]), i))[:K]


def test_topk_against_python_sort_and_edge_cases():
    rng = np.random.default_rng(21)
    S = rng.integers(-20, 20, size=(6, 300))                                 # many ties
    for K in (1, 7, 300):
        idx, val = od.topk(S, K)
        for q in range(6):
            want = _brute_topk(S[q], K)
            assert idx[q].tolist() == want
            assert val[q].tolist() == [int(S[q, i]) for i in want]
    flat = np.full((2, 50), 5)
    idx, _ = od.topk(flat, 10)
    assert idx.tolist() == [list(range(10))] * 2                             # all tied: lowest indices
    dup = np.tile(rng.integers(0, 5, size=(1, 20)), (1, 3))                  # duplicated rows
    idx, _ = od.topk(dup, 60)
    assert idx[0].tolist() == _brute_topk(dup[0], 60)
    with pytest.raises(ValueError):
        od.topk(flat, 51)
    with pytest.raises(ValueError):
        od.topk(flat, 0)


def test_self_is_best_among_equal_norm_rows():
    rng = np.random.default_rng(23)
    d, B = 64, 3
    base = rng.integers(0, 8, size=d).astype(np.uint8)
    rows = np.stack([rng.permutation(base) for _ in range(30)] + [base])     # equal quantized norm
    P = od.pack_planes(rows, B)
    S = od.score_matrix(P[-1:], P, d, B, B)
    best = S.max()
    assert S[0, -1] == best
    for r in range(30):
        assert S[0, r] < best or np.array_equal(rows[r], base)


def test_precision_at_k():
    real = np.array([[0, 1, 2, 3]])
    assert od.precision_at_k(np.array([[3, 2, 9, 8]]), real) == 0.5
    rng = np.random.default_rng(2)
    X = rng.standard_normal((200, 16)).astype(np.float32)
    X /= np.linalg.norm(X, axis=1, keepdims=True)
    idx, sim = od.exact_cosine_topk(X, X[:5], 3)
    assert idx[:, 0].tolist() == [0, 1, 2, 3, 4]                             # self is the nearest
    assert np.allclose(sim[:, 0], 1.0, atol=1e-6)


def _read_bit_order_golden(golden_dir):
    d = B = None
    codes, words, ints = {}, {}, {}
    for line in open(os.path.join(golden_dir, "plane_bit_order.txt")):
        f = line.split()
        if not f or f[0].startswith("#"):
            continue
        if f[0] == "dimension":
            d = int(f[1])
        elif f[0] == "bits":
            B = int(f[1])
        elif f[0] == "code":
            codes[int(f[1])] = int(f[2])
        elif f[0] == "word":
            words[(int(f[1]), int(f[2]))] = int(f[3], 16)
        elif f[0] == "plane_integer":
            ints[int(f[1])] = int(f[2], 16)
    row = np.zeros(d, dtype=np.uint8)
    for k, c in codes.items():
        row[k] = c
    W = (d + 31) // 32
    want = np.array([[words[(b, w)] for w in range(W)] for b in range(B)], dtype=np.uint32)
    return d, B, row, want, [ints[b] for b in range(B)]


def test_plane_bit_order_against_hand_typed_words(golden_dir):
    """Coordinate 0 sits at the least significant end of a plane (Section 3.3, the equation that
    defines xhat_b); the words are typed by hand in the golden file, so a reversed or permuted
    bit order in any of the three packers fails here."""
    from oracle import scale as oc
    d, B, row, want, ints = _read_bit_order_golden(golden_dir)
    assert od.plane_ints(row, B) == ints
    assert np.array_equal(od.pack_planes(row[None, :], B)[0], want)
    assert np.array_equal(oc.planes_as_u32(oc.pack(row[None, :], B), d)[0], want)
    # through the quantizer as well: cell centres give back the codes
    x = ((7 - 2 * row.astype(np.int64)) / 8.0).astype(np.float32)
    assert np.array_equal(od.encode(x[None, :], B), row[None, :])
    assert np.array_equal(oc.planes_as_u32(oc.encode(x[None, :], B, 1.0), d)[0], want)
    # a second row in the same call must not disturb the first (row stride of the packers)
    two = np.stack([row, row[::-1]])
    assert np.array_equal(od.pack_planes(two, B)[0], want)
    assert np.array_equal(oc.planes_as_u32(oc.pack(two, B), d)[0], want)
    assert od.plane_ints(row[::-1], B) != ints                                # the case is not symmetric


# ------------------------------------------------------------- Algorithm 1 (K-Select)
def _kselect_case(seed, n=400, d=24, m=5, Bq=4, Bd=3):
    rng = np.random.default_rng(seed)
    Xd = rng.standard_normal((n, d)).astype(np.float32)
    Xd /= np.linalg.norm(Xd, axis=1, keepdims=True)
    Xq = rng.standard_normal((m, d)).astype(np.float32)
    Xq /= np.linalg.norm(Xq, axis=1, keepdims=True)
    D = od.distance_matrix(od.pack_planes(od.encode(Xq, Bq, 2.0), Bq), od.pack_planes(od.encode(Xd, Bd, 2.0), Bd))
    return Xd, Xq, D


def test_histogram_boundary_is_kth_smallest_distance():
    _, _, D = _kselect_case(31)
    for q in range(D.shape[0]):
        for K in (1, 2, 17, 399, 400):
            assert od.kth_distance_by_histogram(D[q], K) == sorted(D[q].tolist())[K - 1]


def test_candidates_are_exactly_rows_within_the_bound():
    _, _, D = _kselect_case(32)
    for extra in (0, 3, 40):
        for K in (1, 10):
            L = od.k_select_candidates(D[0], K, extra)
            bound = sorted(D[0].tolist())[K - 1] + extra
            assert sorted(L.tolist()) == [i for i in range(D.shape[1]) if D[0, i] <= bound]
            keys = [(int(D[0, i]), int(i)) for i in L]
            assert keys == sorted(keys) and len(L) >= K


def test_candidates_with_a_limit_hand_case():
    # 10 rows, K = 3.  By hand: sorted (D, row) = (1,r4) (2,r0) (2,r7) (3,r2) (3,r5) (3,r9) (5,r1) (6,r3) (6,r8) (9,r6);
    # the 3rd smallest distance is 2; with extra 1 the boundary is 3 and six rows lie within it
    D = np.array([2, 5, 3, 6, 1, 3, 9, 2, 6, 3])
    f = od.k_select_candidates
    assert f(D, 3, 1).tolist() == [4, 0, 7, 2, 5, 9]
    assert f(D, 3, 1, limit=6).tolist() == [4, 0, 7, 2, 5, 9]
    assert f(D, 3, 1, limit=5).tolist() == [4, 0, 7, 2, 5]        # cut inside the level D = 3: lower rows stay
    assert f(D, 3, 1, limit=4).tolist() == [4, 0, 7, 2]
    assert f(D, 3, 1, limit=3).tolist() == [4, 0, 7]
    assert f(D, 3, 4, limit=8).tolist() == [4, 0, 7, 2, 5, 9, 1, 3]   # boundary 6: nine rows, the first eight kept
    assert f(D, 1, 0, limit=1).tolist() == [4]


def test_k_select_with_unbounded_extra_is_exact_search():
    # once every row is a candidate the refine stage is plain exact search
    Xd, Xq, D = _kselect_case(33)
    idx, sim, count = od.k_select(D, Xd, Xq, 10, extra=int(D.max()))
    ridx, rsim = od.exact_cosine_topk(Xd, Xq, 10)
    assert (count == Xd.shape[0]).all()
    assert np.array_equal(idx, ridx) and np.allclose(sim, rsim, atol=0)


def test_k_select_refines_within_candidates_and_precision_grows_with_extra():
    Xd, Xq, D = _kselect_case(34, n=3000, m=8)
    real, _ = od.exact_cosine_topk(Xd, Xq, 10)
    prev = -1.0
    for extra in (0, 2, 5, 10, 20, 50, 100, 100000):
        idx, sim, count = od.k_select(D, Xd, Xq, 10, extra)
        for q in range(Xq.shape[0]):
            L = set(od.k_select_candidates(D[q], 10, extra).tolist())
            assert set(idx[q].tolist()) <= L                                   # only candidates are returned
            assert (np.diff(sim[q]) <= 0).all()                                # sorted by similarity
            want = sorted(L, key=lambda r: (-float(Xd[r].astype(np.float64) @ Xq[q].astype(np.float64)), r))[:10]
            assert idx[q].tolist() == want                                     # brute-force re-ranking of L
        p = od.precision_at_k(idx, real)
        assert p >= prev - 1e-12                                               # nested candidate sets
        prev = p
    assert prev == 1.0


def test_candidates_by_levels_hand_case():
    # distances of 10 rows, K = 3: sorted (D,row) = (1,r4) (2,r0) (2,r7) (3,r2) (3,r5) (3,r9) (5,r1) (6,r3) (6,r8) (9,r6)
    D = np.array([2, 5, 3, 6, 1, 3, 9, 2, 6, 3])
    f = od.k_select_candidates_by_levels
    assert od.kth_distance_by_histogram(D, 3) == 2
    assert f(D, 3, 0, 100).tolist() == [4, 0, 7]                       # D <= 2
    assert f(D, 3, 1, 100).tolist() == [4, 0, 7, 2, 5, 9]              # D <= 3
    assert f(D, 3, 3, 100).tolist() == [4, 0, 7, 2, 5, 9, 1]           # D <= 5
    assert f(D, 3, 100, 100).tolist() == [4, 0, 7, 2, 5, 9, 1, 3, 8, 6]
    # bound on the length: levels stay whole, the boundary moves down
    assert f(D, 3, 4, 8).tolist() == [4, 0, 7, 2, 5, 9, 1]             # D <= 6 would be 9 rows: back to D <= 5
    assert f(D, 3, 4, 6).tolist() == [4, 0, 7, 2, 5, 9]                # D <= 3
    assert f(D, 3, 4, 5).tolist() == [4, 0, 7]                         # D <= 3 is 6 rows: D <= 2
    assert f(D, 3, 4, 3).tolist() == [4, 0, 7]
    # K = 4: the K-th smallest distance is 3 and six rows lie within it; a limit of 5 cannot hold them
    assert od.kth_distance_by_histogram(D, 4) == 3
    assert f(D, 4, 2, 5).tolist() == [4, 0, 7, 2]                      # the K best by (distance, row)
    assert f(D, 4, 2, 6).tolist() == [4, 0, 7, 2, 5, 9]


def test_candidates_by_levels_properties():
    _, _, D = _kselect_case(35, n=2500, m=6)
    n = D.shape[1]
    for q in range(D.shape[0]):
        for K, extra in ((1, 0), (10, 7), (10, 60), (100, 25)):
            whole = od.k_select_candidates(D[q], K, extra)
            # a generous limit leaves Algorithm 1's list untouched
            assert od.k_select_candidates_by_levels(D[q], K, extra, n).tolist() == whole.tolist()
            assert od.k_select_candidates_by_levels(D[q], K, extra, len(whole)).tolist() == whole.tolist()
            for limit in (K, K + 1, len(whole) - 1, max(K, len(whole) // 2), max(K, len(whole) // 7)):
                if limit < K:
                    continue
                L = od.k_select_candidates_by_levels(D[q], K, extra, limit)
                assert K <= len(L) <= max(limit, K)
                keys = [(int(D[q, r]), int(r)) for r in L]
                assert keys == sorted(keys)
                assert L.tolist() == whole[:len(L)].tolist()                  # a prefix of the printed list
                d_k = sorted(D[q].tolist())[K - 1]
                top = int(D[q, L[-1]])
                inside = int((D[q] <= top).sum())
                if inside == len(L):                                          # whole levels ...
                    sd = np.sort(D[q])
                    above = sd[sd > top]
                    if len(above) and above[0] <= d_k + extra:                # ... and the next occupied one would not fit
                        assert int(np.searchsorted(sd, above[0], side="right")) > limit
                else:                                                         # ties at the K-th distance exceed the limit
                    assert top == d_k and len(L) == K and int((D[q] <= d_k).sum()) > limit


def test_k_select_by_levels_equals_k_select_when_nothing_is_cut():
    Xd, Xq, D = _kselect_case(36, n=1500, m=5)
    for extra in (0, 12, 90):
        a = od.k_select(D, Xd, Xq, 10, extra)
        b = od.k_select_by_levels(D, Xd, Xq, 10, extra, limit=1500)
        for x, y in zip(a, b):
            assert np.array_equal(x, y)
    # and it re-ranks exactly its own candidate list
    idx, sim, count = od.k_select_by_levels(D, Xd, Xq, 10, 90, limit=200)
    for q in range(Xq.shape[0]):
        L = od.k_select_candidates_by_levels(D[q], 10, 90, 200).tolist()
        assert count[q] == len(L) <= 200
        want = sorted(L, key=lambda r: (-float(Xd[r].astype(np.float64) @ Xq[q].astype(np.float64)), r))[:10]
        assert idx[q].tolist() == want


def test_distance_from_score_roundtrip():
    D = np.array([[0, 5, 77], [1, 2, 3]])
    assert np.array_equal(od.distance_from_score(od.score_from_distance(D, 50, 4, 3), 50, 4, 3), D)
