"""The candidate-mode selection (Algorithm 1's list, bounded to the best 2048 keys) on the CPU.

`tests/cpu_model/candidate_lists_model.cpp` replays what select_dense, select_merge and the
exact rescan of an overflowed query do to one query's list, using the product's own rule for
the cut and the threshold (`csrc/xbq_cut.h`).  The oracle's `k_select_candidates` says what the
list must be.  The tie-heavy, sorted-row cases here are the ones in which a list that was cut
once must keep the keys it holds at the threshold distance.
"""
import ctypes
import os
import subprocess

import numpy as np
import pytest

from oracle import definition as od

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "tests", "cpu_model", "candidate_lists_model.cpp")
LIB = os.path.join(ROOT, "tests", "cpu_model", "libcandidate_lists_model.so")


@pytest.fixture(scope="module")
def model():
    subprocess.run(["g++", "-O1", "-std=c++17", "-shared", "-fPIC", "-I",
                    os.path.join(ROOT, "paper_2008_02002_amd", "csrc"), "-o", LIB, SRC], check=True)
    L = ctypes.CDLL(LIB)
    L.model_candidate_lists.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64] + [ctypes.c_int] * 9 + \
                                       [ctypes.c_void_p] * 2
    L.model_candidate_lists.restype = ctypes.c_int

    def run(D, k, extra, keep_max=2048, first=1024, group=4096, cap=2048, capacity=4096, block=256, force_rescan=0,
            rows=None):
        """rows: the row numbers in the order they are taken (a permutation); D is in that order."""
        D = np.ascontiguousarray(D, dtype=np.uint32)
        rows = None if rows is None else np.ascontiguousarray(rows, dtype=np.uint32)
        out = np.zeros(keep_max, dtype=np.uint64)
        thr = ctypes.c_uint32()
        n = L.model_candidate_lists(D.ctypes.data, None if rows is None else rows.ctypes.data, len(D), k, extra,
                                    keep_max, first, group, cap, capacity, block,
                                    force_rescan, out.ctypes.data, ctypes.byref(thr))
        assert n >= 0, f"model refused the case ({n})"
        return out[:n], thr.value
    return run


def _check(run, D, k, extra, **kw):
    keep_max = kw.get("keep_max", 2048)
    keys, thr = run(D, k, extra, **kw)
    want = od.k_select_candidates(D, k, extra, limit=keep_max)
    got_rows = (keys & np.uint64(0xffffffff)).astype(np.int64)
    assert np.array_equal(got_rows, want), (len(got_rows), len(want))
    assert np.array_equal((keys >> np.uint64(32)).astype(np.int64), np.asarray(D, dtype=np.int64)[want])
    whole = od.k_select_candidates(D, k, extra)
    # what xbq_k_select relies on: a list shorter than the bound is the whole list
    if len(keys) < keep_max:
        assert len(whole) == len(keys)
    return keys, thr


def test_cut_list_keeps_its_keys_at_the_threshold_distance(model):
    # group 0 and the first later group: 4096 rows at D = 50 (the list is cut at 2048 of them,
    # threshold 50); then rows at 48 and 49 stream in: the held D = 49 rows with low numbers are
    # within the boundary and must stay when the buffer is compacted
    D = np.concatenate([np.full(4096, 50), np.full(200, 48), np.full(3896, 49), np.full(1793, 48)])
    keys, thr = _check(model, D, 100, 1, first=4096, group=10_000, force_rescan=1)
    assert len(keys) == 2048 and thr == 49
    dist = (keys >> np.uint64(32)).astype(np.int64)
    assert (dist == 48).sum() == 1993 and (dist == 49).sum() == 55
    for first, group in ((1024, 4096), (2048, 512), (4096, 3000)):
        for force in (0, 1):
            assert len(_check(model, D, 100, 1, first=first, group=group, force_rescan=force)[0]) == 2048


def test_one_bit_like_levels_sorted_towards_the_query(model):
    # few distinct distances, rows ever closer: every group floods the list
    rng = np.random.default_rng(3)
    for k, extra in ((10, 0), (10, 1), (10, 3), (100, 2), (1024, 1)):
        D = np.sort(rng.integers(0, 17, size=30_000))[::-1]
        for force in (0, 1):
            _check(model, D, k, extra, force_rescan=force)


def test_random_tie_heavy_sequences(model):
    rng = np.random.default_rng(11)
    for trial in range(60):
        n = int(rng.integers(1100, 20_000))
        levels = int(rng.integers(2, 40))
        D = rng.integers(0, levels, size=n) + 5
        if trial % 3 == 0:
            D = np.sort(D)[::-1]
        elif trial % 3 == 1:                       # descending in blocks: partly sorted
            D = np.concatenate([np.sort(c)[::-1] for c in np.array_split(D, 7)])
        k = int(rng.choice([1, 5, 10, 100, 1000]))
        extra = int(rng.integers(0, 6))
        keep_max = int(rng.choice([2048, 1024 + 512, max(k, 64)]))
        cap = int(rng.choice([2048, 300]))
        _check(model, D, k, extra, keep_max=keep_max, cap=cap, capacity=4096, group=int(rng.choice([512, 4096, 9000])),
               force_rescan=int(trial % 2))


def test_small_buffers_compact_often(model):
    # tiny list bound, buffer and block: the compaction runs every few rows, in every state
    rng = np.random.default_rng(23)
    for trial in range(300):
        n = int(rng.integers(200, 3000))
        D = rng.integers(0, int(rng.integers(2, 12)), size=n) + 1
        if trial % 2 == 0:
            D = np.concatenate([np.sort(c)[::-1] for c in np.array_split(D, int(rng.integers(1, 5)))])
        k = int(rng.choice([1, 3, 8, 20]))
        keep_max = int(rng.choice([k, 24, 40, 64]))
        keep_max = max(keep_max, k)
        block = int(rng.choice([4, 16]))
        _check(model, D, k, int(rng.integers(0, 4)), keep_max=keep_max, first=64, group=int(rng.choice([100, 700, 5000])),
               cap=int(rng.choice([8, 64])), capacity=keep_max + 2 * block + int(rng.integers(0, 20)), block=block,
               force_rescan=int(rng.integers(0, 2)))


def test_nothing_cut_is_algorithm_1_unchanged(model):
    rng = np.random.default_rng(5)
    D = rng.integers(100, 4000, size=50_000)
    keys, thr = _check(model, D, 10, 30)
    d_k = od.kth_distance_by_histogram(D, 10)
    assert thr == d_k + 30 + 1                     # every row within the printed boundary is of interest


def test_rows_taken_in_any_order(model):
    """The threshold schedule takes its row groups spread over the database, so a later group may
    hold a lower row with the same distance: the cut must let it in (threshold one higher once the
    list is full).  Same tie-heavy sequences as above, the rows taken in a random order and in
    the schedule's own order (bundles of 64 rows, step s -> bundle s * c mod F)."""
    rng = np.random.default_rng(29)
    old_rule_wrong = 0
    for trial in range(80):
        n = int(rng.integers(1100, 20_000))
        levels = int(rng.integers(2, 40))
        D_by_row = rng.integers(0, levels, size=n) + 5
        if trial % 3 == 0:
            D_by_row = np.sort(D_by_row)[::-1]
        if trial % 2 == 0:
            order = rng.permutation(n)
        else:
            full = n // 64
            c = next(c for c in range(max(2, int(full * 0.618)), full + 2) if np.gcd(c, full) == 1) if full > 2 else 1
            steps = np.arange(full)
            bundles = np.concatenate([(steps * c) % full if full > 2 else steps, np.arange(full, (n + 63) // 64)])
            order = (bundles[:, None] * 64 + np.arange(64)[None, :]).reshape(-1)
            order = order[order < n]
        assert np.array_equal(np.sort(order), np.arange(n))
        k = int(rng.choice([1, 5, 10, 100, 1000]))
        extra = int(rng.integers(0, 6))
        keep_max = int(rng.choice([2048, 1024 + 512, max(k, 64)]))
        kw = dict(keep_max=keep_max, cap=int(rng.choice([2048, 300])), capacity=4096,
                  group=int(rng.choice([512, 4096, 9000])), force_rescan=int(trial % 2))
        keys, _ = model(D_by_row[order], k, extra, rows=order, **kw)
        want = od.k_select_candidates(D_by_row, k, extra, limit=keep_max)
        assert np.array_equal((keys & np.uint64(0xffffffff)).astype(np.int64), want), trial
        # the rule for ascending rows, applied to the same order, must get some of these wrong:
        # otherwise this test would not see the difference
        D = np.ascontiguousarray(D_by_row[order], dtype=np.uint32)
        fake = np.ascontiguousarray(order, dtype=np.uint32)
        old_keys, _ = model(D, k, extra, **kw)                       # rows = places: ascending rule
        old_rows = fake[(old_keys & np.uint64(0xffffffff)).astype(np.int64)]
        old_rule_wrong += int(not np.array_equal(np.sort(old_rows), np.sort(want)))
    assert old_rule_wrong > 0
