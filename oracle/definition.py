"""Definition-level oracle: the paper's formulas, written out one by one.

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).  Slow on purpose: scalar
functions use Python ints and floats, array functions use plain NumPy with no
blocking or reordering, so every function can be checked against the cited
passage by eye.

Notation follows the paper: ``B`` bits per coordinate, ``a_i`` in {+1,-1} the
signed digits of a quantized value, ``abar_i`` = sigma(a_i) in {0,1} the stored
bits, ``xbar`` the B-bit integer code of one coordinate, ``xhat_b`` the b-th
bit-plane of a vector.  ``d`` is the vector dimension (the paper's N) and ``n``
the number of database vectors.

Readings taken where the text is silent or garbled (each also listed in the
design document):
  * Quantizer rule (Section 3.2, the formula after the definition of f_B) is
    read as successive approximation, most significant digit first:
    a_{B-1-i} = sign(x - f_i(x)), f_0 = 0.  The appendix proof of Proposition 2
    confirms it (f_k - f_{k-1} = +2^-k exactly when x >= f_{k-1}).
  * sign(0) = +1, as printed in Section 3.2.
  * No clamp: values at or beyond +-1 simply run into the outermost cell.
  * The scale factor of Section 3.5 is one IEEE binary32 multiply before
    quantizing.
  * Plane word layout: coordinate k is bit (k mod 32) of 32-bit word k // 32;
    pad bits are zero (Eq. 9, the bit-plane reconstruction of Section 3.3, puts coordinate 0 at the least
    significant end).
  * The exported score is S = d (2^Bx - 1)(2^By - 1) - 2 (Xbar (x) Ybar), the
    numerator of Eq. 7 (X.Y in terms of Xbar (x) Ybar, Section 3.3): larger means more similar.
  * Ties in the top-K go to the lower index; output sorted by (S desc, idx asc).
  * Algorithm 1 keeps every row within its boundary and is silent about memory.
    Two bounded forms are stated here because the implementation under test
    documents them: the first ``limit`` candidates in (distance, row) order
    (:func:`k_select_candidates`), and a boundary lowered by whole distance
    units until the candidates fit (:func:`k_select_candidates_by_levels`).
    Without a limit both are the algorithm as printed.

Every function here is pinned by ``tests/test_oracle_pins.py`` against something
the paper or the mathematics fixes.  The accuracy *figures* computed with
:func:`precision_at_k` on the synthetic workloads are parity unpinned: the paper
prints such figures for its own datasets only; the function itself is pinned by a
hand-counted case.
"""
from __future__ import annotations

import numpy as np

# --------------------------------------------------------------------------
# Section 3.1: the isomorphism between ({+1,-1}, *) and ({0,1}, xor)
# --------------------------------------------------------------------------


def sigma(a: int) -> int:
    """Proposition 1, Eq. 1: sigma(a) = (1 - a) / 2 maps +1 -> 0 and -1 -> 1."""
    if a not in (1, -1):
        raise ValueError("sigma is defined on {+1,-1}")
    return (1 - a) // 2


def sigma_inv(abar: int) -> int:
    """Inverse of sigma (Section 3.1, used in Eq. 2: a1 a2 = 1 - 2 (abar1 xor abar2)): a = 1 - 2 abar."""
    if abar not in (0, 1):
        raise ValueError("sigma_inv is defined on {0,1}")
    return 1 - 2 * abar


# --------------------------------------------------------------------------
# Section 3.2: the quantizer f_B
# --------------------------------------------------------------------------


def sign(v: float) -> int:
    """sign as printed in Section 3.2: +1 for v >= 0 (so also for -0.0), else -1."""
    return 1 if v >= 0 else -1


def quantize_digits(t: float, B: int) -> list[int]:
    """Signed digits [a_{B-1}, ..., a_0] of f_B(t), Section 3.2.

    Successive approximation: with f_0 = 0, digit a_{B-1-i} = sign(t - f_i(t))
    and f_{i+1}(t) = f_i(t) + a_{B-1-i} / 2^(i+1).  Every partial sum is a
    multiple of 2^-B below 1 in magnitude, hence exact in binary floating point,
    and the comparison ``t >= f_i`` is done directly (no subtraction).
    """
    if B < 1:
        raise ValueError("B >= 1")
    digits = []
    partial = 0.0  # f_i(t)
    for i in range(B):
        a = 1 if t >= partial else -1
        digits.append(a)
        partial += a * 2.0 ** (-(i + 1))
    return digits  # most significant first


def quantize_code(t: float, B: int) -> int:
    """B-bit integer code xbar = (abar_{B-1} ... abar_0)_2 of t (Section 3.2)."""
    code = 0
    for a in quantize_digits(t, B):
        code = (code << 1) | sigma(a)
    return code


def decode_numerator(code: int, B: int) -> int:
    """Integer m with f_B = m / 2^B:  m = sum_i a_i 2^i = (2^B - 1) - 2 xbar."""
    m = 0
    for i in range(B):
        abar = (code >> i) & 1
        m += sigma_inv(abar) * (1 << i)
    return m


def decode_value(code: int, B: int) -> float:
    """f_B as a real number: sum_i a_i / 2^(B-i) (definition of f_B)."""
    return decode_numerator(code, B) / float(1 << B)


# --------------------------------------------------------------------------
# Section 3.2: the scalar (x) operator and the product identity (Eq. 5)
# --------------------------------------------------------------------------


def otimes_scalar(xbar: int, ybar: int, Bx: int, By: int) -> int:
    """xbar (x) ybar = sum_i sum_j (abar_i xor cbar_j) << (i + j)."""
    total = 0
    for i in range(Bx):
        for j in range(By):
            total += (((xbar >> i) & 1) ^ ((ybar >> j) & 1)) << (i + j)
    return total


def product_numerator(xbar: int, ybar: int, Bx: int, By: int) -> int:
    """Numerator of Eq. 5 (x_B y_B in terms of xbar (x) ybar, Section 3.2): 2^(Bx+By) * x_B * y_B."""
    return ((1 << Bx) - 1) * ((1 << By) - 1) - 2 * otimes_scalar(xbar, ybar, Bx, By)


# --------------------------------------------------------------------------
# Array level: encode, planes, scores, top-K
# --------------------------------------------------------------------------


def scale_fp32(X: np.ndarray, scale: float) -> np.ndarray:
    """Section 3.5 scaling: one binary32 multiply per coordinate."""
    X = np.asarray(X, dtype=np.float32)
    return X * np.float32(scale)


def encode(X: np.ndarray, B: int, scale: float = 1.0) -> np.ndarray:
    """Per-coordinate codes xbar (uint8, shape of X) of scale*X, Section 3.2.

    Vectorised form of :func:`quantize_code`: the same B greedy comparisons, in
    the same order, on every coordinate at once.
    """
    if not 1 <= B <= 8:
        raise ValueError("1 <= B <= 8")
    t = scale_fp32(X, scale).astype(np.float64)  # exact widening
    partial = np.zeros_like(t)
    code = np.zeros(t.shape, dtype=np.uint8)
    for i in range(B):
        up = t >= partial
        code = (code << 1) | (~up).astype(np.uint8)
        partial = partial + np.where(up, 1.0, -1.0) * 2.0 ** (-(i + 1))
    return code


def decode(codes: np.ndarray, B: int) -> np.ndarray:
    """Integer numerators m = (2^B - 1) - 2 xbar of the decoded values (int64)."""
    return ((1 << B) - 1) - 2 * codes.astype(np.int64)


def plane_ints(codes_row, B: int) -> list[int]:
    """Eq. 9 (Section 3.3, bit-plane reconstruction): xhat_b = (abar_{b,d-1} ... abar_{b,0})_2 as Python ints."""
    planes = []
    for b in range(B):
        v = 0
        for k, c in enumerate(codes_row):
            v |= ((int(c) >> b) & 1) << k
        planes.append(v)
    return planes


def pack_planes(codes: np.ndarray, B: int) -> np.ndarray:
    """Bit-planes as uint32 words, shape [n, B, W], W = ceil(d / 32).

    Word w of plane b holds coordinates 32w .. 32w+31, coordinate 32w at bit 0;
    bits past d are zero.
    """
    codes = np.asarray(codes, dtype=np.uint8)
    n, d = codes.shape
    W = (d + 31) // 32
    out = np.zeros((n, B, W), dtype=np.uint32)
    for b in range(B):
        bits = ((codes >> b) & 1).astype(np.uint32)
        for k in range(d):
            out[:, b, k // 32] |= bits[:, k] << np.uint32(k % 32)
    return out


def otimes_vector(codes_x, codes_y, Bx: int, By: int) -> int:
    """Xbar (x) Ybar = sum_k xbar_k (x) ybar_k (Section 3.3, Eq. 6)."""
    return sum(otimes_scalar(int(cx), int(cy), Bx, By) for cx, cy in zip(codes_x, codes_y))


def popcount_distance_ints(planes_x: list[int], planes_y: list[int]) -> int:
    """Eq. 10 (Section 3.3, the POPCNT form): sum_i sum_j POPCNT(xhat_i xor yhat_j) << (i + j)."""
    total = 0
    for i, xi in enumerate(planes_x):
        for j, yj in enumerate(planes_y):
            total += bin(xi ^ yj).count("1") << (i + j)
    return total


def distance_matrix(planes_q: np.ndarray, planes_db: np.ndarray) -> np.ndarray:
    """Eq. 10 (Section 3.3, the POPCNT form) for every (query, database) pair: D[q, r], int64.

    ``planes_q`` is [m, Bq, W], ``planes_db`` is [n, Bd, W] (uint32 words).
    """
    m, Bq, W = planes_q.shape
    n, Bd, W2 = planes_db.shape
    if W != W2:
        raise ValueError("word counts differ")
    D = np.zeros((m, n), dtype=np.int64)
    for i in range(Bq):
        for j in range(Bd):
            x = planes_q[:, i, :][:, None, :] ^ planes_db[:, j, :][None, :, :]
            D += np.bitwise_count(x).sum(axis=2, dtype=np.int64) << (i + j)
    return D


def score_from_distance(D, d: int, Bq: int, Bd: int):
    """Numerator of Eq. 7 (Section 3.3): S = d (2^Bq - 1)(2^Bd - 1) - 2 D."""
    return d * ((1 << Bq) - 1) * ((1 << Bd) - 1) - 2 * D


def score_matrix(planes_q, planes_db, d: int, Bq: int, Bd: int) -> np.ndarray:
    return score_from_distance(distance_matrix(planes_q, planes_db), d, Bq, Bd)


def topk(S: np.ndarray, K: int):
    """Top-K per row of S: full sort on (S descending, index ascending)."""
    S = np.asarray(S)
    m, n = S.shape
    if not 1 <= K <= n:
        raise ValueError("1 <= K <= n")
    idx = np.empty((m, K), dtype=np.int64)
    val = np.empty((m, K), dtype=S.dtype)
    ar = np.arange(n)
    for q in range(m):
        order = np.lexsort((ar, -S[q].astype(np.int64)))[:K]
        idx[q] = order
        val[q] = S[q, order]
    return idx, val


def search(X_db, X_q, B: int, K: int, scale: float = 1.0):
    """Whole path at definition level: encode, planes, Eq. 10 distances, Eq. 7 scores, top-K."""
    d = X_db.shape[1]
    p_db = pack_planes(encode(X_db, B, scale), B)
    p_q = pack_planes(encode(X_q, B, scale), B)
    S = score_matrix(p_q, p_db, d, B, B)
    return topk(S, K)


# --------------------------------------------------------------------------
# Section 4, Algorithm 1 (K-Select): histogram of the integer distances, boundary at
# the K-th smallest distance plus an extra distance (Section 3.6), candidates, exact
# refine, sort.
# --------------------------------------------------------------------------


def kth_distance_by_histogram(dist_row: np.ndarray, K: int) -> int:
    """Algorithm 1, histogram steps: h_v = number of rows at distance v; the boundary is
    the smallest j with sum_{i <= j} h_i >= K."""
    h = np.bincount(np.asarray(dist_row, dtype=np.int64))
    cum = np.cumsum(h)
    return int(np.argmax(cum >= K))


def k_select_candidates(dist_row: np.ndarray, K: int, extra: int, limit: int | None = None) -> np.ndarray:
    """Algorithm 1, candidate list L: every row with d <= maxDistance, where
    maxDistance = (K-th smallest distance) + extraDistance.  Returned in (distance, row)
    order; if ``limit`` is given only the first ``limit`` of that order are kept (a bound
    on the list the implementation under test documents)."""
    dist_row = np.asarray(dist_row, dtype=np.int64)
    max_distance = kth_distance_by_histogram(dist_row, K) + extra
    rows = np.nonzero(dist_row <= max_distance)[0]
    order = np.lexsort((rows, dist_row[rows]))
    rows = rows[order]
    return rows if limit is None else rows[:limit]


def k_select(dist: np.ndarray, X_db: np.ndarray, X_q: np.ndarray, K: int, extra: int, limit: int | None = None):
    """Algorithm 1 from the distances on: candidates, refine by the exact inner product of
    the original vectors (accumulated in float64), sort by similarity (descending, ties to
    the lower row), first K.  Returns (idx [m, K], similarity float64 [m, K], |L| [m])."""
    m = dist.shape[0]
    idx = np.empty((m, K), dtype=np.int64)
    sim = np.empty((m, K), dtype=np.float64)
    count = np.empty(m, dtype=np.int64)
    Xd = np.asarray(X_db, dtype=np.float64)
    Xq = np.asarray(X_q, dtype=np.float64)
    for q in range(m):
        L = k_select_candidates(dist[q], K, extra, limit)
        count[q] = len(L)
        s = Xd[L] @ Xq[q]
        order = np.lexsort((L, -s))[:K]
        idx[q] = L[order]
        sim[q] = s[order]
    return idx, sim, count


def k_select_candidates_by_levels(dist_row: np.ndarray, K: int, extra: int, limit: int) -> np.ndarray:
    """Algorithm 1's candidate list L under a bound on its length that keeps distance levels
    whole: maxDistance starts at (K-th smallest distance) + extraDistance as printed and, while
    more than ``limit`` rows lie within it, is lowered one unit at a time, never below the K-th
    smallest distance itself.  If the rows within the K-th smallest distance alone exceed the
    limit (ties), L is the K best rows by (distance, row).  With limit >= number of rows within
    the printed boundary this is Algorithm 1 unchanged.  Returned in (distance, row) order."""
    dist_row = np.asarray(dist_row, dtype=np.int64)
    d_k = kth_distance_by_histogram(dist_row, K)
    max_distance = d_k + extra
    while max_distance >= d_k:
        rows = np.nonzero(dist_row <= max_distance)[0]
        if len(rows) <= limit:
            return rows[np.lexsort((rows, dist_row[rows]))]
        max_distance -= 1
    rows = np.arange(len(dist_row))
    return rows[np.lexsort((rows, dist_row))][:K]


def k_select_by_levels(dist: np.ndarray, X_db: np.ndarray, X_q: np.ndarray, K: int, extra: int, limit: int):
    """Algorithm 1 with :func:`k_select_candidates_by_levels` as its candidate list: refine by
    the exact inner product (float64), sort (similarity descending, ties to the lower row),
    first K.  Returns (idx [m, K], similarity float64 [m, K], |L| [m])."""
    m = dist.shape[0]
    idx = np.empty((m, K), dtype=np.int64)
    sim = np.empty((m, K), dtype=np.float64)
    count = np.empty(m, dtype=np.int64)
    Xq = np.asarray(X_q, dtype=np.float64)
    for q in range(m):
        L = k_select_candidates_by_levels(dist[q], K, extra, limit)
        count[q] = len(L)
        s = np.asarray(X_db[L], dtype=np.float64) @ Xq[q]
        order = np.lexsort((L, -s))[:K]
        idx[q] = L[order]
        sim[q] = s[order]
    return idx, sim, count


def distance_from_score(S, d: int, Bq: int, Bd: int):
    """Inverse of :func:`score_from_distance`."""
    return (d * ((1 << Bq) - 1) * ((1 << Bd) - 1) - np.asarray(S, dtype=np.int64)) // 2


# --------------------------------------------------------------------------
# Section 5: Precision@K (same number as recall@K for equal-size sets)
# --------------------------------------------------------------------------


def exact_cosine_topk(X_db, X_q, K: int):
    """Real top-K by inner product of the (already normalised) fp32 vectors,
    accumulated in float64, ordered (similarity desc, index asc)."""
    sim = np.asarray(X_q, dtype=np.float64) @ np.asarray(X_db, dtype=np.float64).T
    return topk_float(sim, K)


def topk_float(sim: np.ndarray, K: int):
    m, n = sim.shape
    idx = np.empty((m, K), dtype=np.int64)
    ar = np.arange(n)
    for q in range(m):
        idx[q] = np.lexsort((ar, -sim[q]))[:K]
    return idx, np.take_along_axis(sim, idx, axis=1)


def precision_at_k(found_idx: np.ndarray, real_idx: np.ndarray) -> float:
    """|calculated top K  intersect  real top K| / K, averaged over queries."""
    m, K = real_idx.shape
    hits = 0
    for q in range(m):
        hits += len(set(found_idx[q].tolist()) & set(real_idx[q].tolist()))
    return hits / float(m * K)
