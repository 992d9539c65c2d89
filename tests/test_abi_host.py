"""Host-only checks of the C-ABI library: it loads, exports what the header declares,
and rejects bad arguments before touching the GPU."""
import ctypes
import os
import re

import pytest

from paper_2008_02002_amd import xbq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(xbq.LIB_PATH):
        from paper_2008_02002_amd.build import build_library
        build_library(verbose=False)
    return xbq.lib()


def test_exports_every_declared_symbol(L):
    header = open(os.path.join(ROOT, "include", "xbq.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(xbq_[a-z0-9_]+)\s*\(", header))
    assert declared == set(xbq.EXPORTS)
    for name in declared:
        assert hasattr(L, name), name


def test_version_and_strerror(L):
    assert L.xbq_version() >= 100
    assert L.xbq_strerror(0) == b"ok"
    for code in (-1, -2, -3, -4, -99):
        assert len(L.xbq_strerror(code)) > 0


def test_code_bytes(L):
    assert L.xbq_code_bytes(1000, 128, 4, xbq.ROWS) == 1000 * 4 * 4 * 4
    assert L.xbq_code_bytes(1000, 128, 4, xbq.BUNDLE64) == 1024 * 4 * 4 * 4      # 16 bundles
    assert L.xbq_code_bytes(64, 200, 3, xbq.BUNDLE64) == 64 * 3 * 7 * 4
    assert L.xbq_code_bytes(0, 128, 4, xbq.ROWS) == 0
    assert L.xbq_code_bytes(10, 128, 5, xbq.ROWS) == 0                           # bits out of range
    assert L.xbq_code_bytes(10, 0, 4, xbq.ROWS) == 0
    assert L.xbq_code_bytes(10, 4096, 4, xbq.ROWS) == 0
    assert L.xbq_code_bytes(10, 128, 4, 7) == 0
    assert L.xbq_code_bytes(-1, 128, 4, xbq.ROWS) == 0


def test_encode_argument_errors(L):
    fake = ctypes.c_void_p(0x1000)      # never dereferenced: validation fails first
    null = ctypes.c_void_p(0)
    enc = L.xbq_encode
    assert enc(null, 10, 128, 4, 1.0, xbq.ROWS, fake, null) == xbq.EINVAL
    assert enc(fake, 10, 128, 4, 1.0, xbq.ROWS, null, null) == xbq.EINVAL
    assert enc(fake, -1, 128, 4, 1.0, xbq.ROWS, fake, null) == xbq.EINVAL
    assert enc(fake, 10, 0, 4, 1.0, xbq.ROWS, fake, null) == xbq.EINVAL
    assert enc(fake, 10, 128, 0, 1.0, xbq.ROWS, fake, null) == xbq.EINVAL
    assert enc(fake, 10, 128, 5, 1.0, xbq.ROWS, fake, null) == xbq.EUNSUPPORTED
    assert enc(fake, 10, 4096, 4, 1.0, xbq.ROWS, fake, null) == xbq.EUNSUPPORTED
    assert enc(fake, 10, 128, 4, 1.0, 9, fake, null) == xbq.EUNSUPPORTED
    assert enc(fake, 10, 128, 4, 0.0, xbq.ROWS, fake, null) == xbq.EINVAL
    assert enc(fake, 10, 128, 4, -1.0, xbq.ROWS, fake, null) == xbq.EINVAL
    assert enc(fake, 10, 128, 4, float("inf"), xbq.ROWS, fake, null) == xbq.EINVAL
    assert enc(fake, 10, 128, 4, float("nan"), xbq.ROWS, fake, null) == xbq.EINVAL
    assert enc(ctypes.c_void_p(0x1002), 10, 128, 4, 1.0, xbq.ROWS, fake, null) == xbq.EINVAL   # misaligned
    assert enc(null, 0, 128, 4, 1.0, xbq.ROWS, null, null) == xbq.OK                           # n = 0: no-op


def test_search_argument_errors(L):
    fake = ctypes.c_void_p(0x1000)
    null = ctypes.c_void_p(0)
    big = 1 << 40

    def s(db=fake, n=1000, q=fake, m=10, d=128, bits=4, k=10, idx=fake, score=fake, ws=fake, wsb=big):
        return L.xbq_search(db, n, q, m, d, bits, k, idx, score, ws, wsb, null)

    assert s(db=null) == xbq.EINVAL
    assert s(q=null) == xbq.EINVAL
    assert s(idx=null) == xbq.EINVAL
    assert s(score=null) == xbq.EINVAL
    assert s(ws=null) == xbq.EINVAL
    assert s(k=0) == xbq.EINVAL
    assert s(k=1001) == xbq.EINVAL                  # k > n
    assert s(n=5000, k=1025) == xbq.EINVAL          # k > XBQ_MAX_K
    assert s(n=-1) == xbq.EINVAL
    assert s(m=-1) == xbq.EINVAL
    assert s(n=1 << 31) == xbq.EINVAL
    assert s(bits=5) == xbq.EUNSUPPORTED
    assert s(d=2049) == xbq.EUNSUPPORTED
    assert s(d=0) == xbq.EINVAL
    assert s(ws=ctypes.c_void_p(0x1010)) == xbq.EINVAL          # workspace not 256-byte aligned
    need = L.xbq_search_workspace_bytes(1000, 10, 128, 4, 10)
    assert need > 0
    assert s(wsb=need - 1) == xbq.EWORKSPACE
    assert s(n=0) == xbq.OK and s(m=0) == xbq.OK                # empty inputs are no-ops


def test_search_asym_argument_errors(L):
    fake = ctypes.c_void_p(0x1000)
    null = ctypes.c_void_p(0)

    def s(db_bits=3, q_bits=4, n=1000, m=10, d=128, k=10, db=fake, ws=fake, wsb=1 << 40):
        return L.xbq_search_asym(db, n, db_bits, fake, m, q_bits, d, k, fake, fake, ws, wsb, null)

    assert s(db_bits=4, q_bits=3) == xbq.EUNSUPPORTED       # queries may not be narrower
    assert s(db_bits=2, q_bits=4) == xbq.EUNSUPPORTED
    assert s(db_bits=4, q_bits=5) == xbq.EUNSUPPORTED
    assert s(db_bits=0) == xbq.EINVAL
    assert s(db=null) == xbq.EINVAL
    assert s(k=0) == xbq.EINVAL
    need = L.xbq_search_workspace_bytes(1000, 10, 128, 4, 10)
    assert s(wsb=need - 1) == xbq.EWORKSPACE
    assert s(n=0) == xbq.OK


def test_search_refine_argument_errors(L):
    fake = ctypes.c_void_p(0x1000)
    null = ctypes.c_void_p(0)

    def s(xdb=fake, xq=fake, n=1000, m=10, d=128, k=10, extra=5, db_bits=3, q_bits=4, sim=fake, wsb=1 << 40):
        return L.xbq_search_refine(xdb, fake, n, db_bits, xq, fake, m, q_bits, d, k, extra, fake, sim, null,
                                   fake, wsb, null)

    assert s(xdb=null) == xbq.EINVAL
    assert s(xq=null) == xbq.EINVAL
    assert s(sim=null) == xbq.EINVAL
    assert s(extra=-1) == xbq.EINVAL
    assert s(k=0) == xbq.EINVAL
    assert s(db_bits=4, q_bits=3) == xbq.EUNSUPPORTED
    need = L.xbq_search_refine_workspace_bytes(1000, 10, 128, 4, 10)
    assert need > L.xbq_search_workspace_bytes(1000, 10, 128, 4, 10)
    assert s(wsb=need - 1) == xbq.EWORKSPACE
    assert s(m=0) == xbq.OK
    assert L.xbq_search_refine_workspace_bytes(1000, 10, 128, 4, 0) == 0


def test_k_select_argument_errors(L):
    fake = ctypes.c_void_p(0x1000)
    null = ctypes.c_void_p(0)

    def s(xdb=fake, xq=fake, n=1000, m=10, d=128, k=10, extra=5, cap=500, db_bits=3, q_bits=4, sim=fake, wsb=1 << 40):
        return L.xbq_k_select(xdb, fake, n, db_bits, xq, fake, m, q_bits, d, k, extra, cap, fake, sim, null,
                              fake, wsb, null)

    assert s(xdb=null) == xbq.EINVAL
    assert s(sim=null) == xbq.EINVAL
    assert s(extra=-1) == xbq.EINVAL
    assert s(extra=4096) == xbq.EINVAL
    assert s(cap=9) == xbq.EINVAL                       # fewer candidates than k
    assert s(cap=(1 << 22) + 1) == xbq.EINVAL
    assert s(k=0) == xbq.EINVAL
    assert s(k=1001) == xbq.EINVAL
    assert s(db_bits=4, q_bits=3) == xbq.EUNSUPPORTED
    f0 = L.xbq_k_select_workspace_bytes
    f = lambda n, m, d, b, k, cap, extra=5: f0(n, m, d, b, k, extra, cap)
    need = f(1000, 10, 128, 4, 10, 500)
    assert need > L.xbq_search_workspace_bytes(1000, 10, 128, 4, 10) + 10 * 500 * 8
    assert s(wsb=need - 1) == xbq.EWORKSPACE
    assert s(m=0) == xbq.OK and s(n=0, k=1, cap=1) == xbq.OK
    assert f(1000, 10, 128, 4, 10, 9) == 0 and f(1000, 10, 128, 4, 0, 500) == 0
    assert f(1000, 10, 128, 4, 10, 500, extra=-1) == 0 and f(1000, 10, 128, 4, 10, 500, extra=4096) == 0
    assert f(1000, 10, 128, 4, 10, 500, extra=4095) > need                  # level counters
    # the candidate lists of a batch stay near 2 GiB however many queries there are; a bound above n counts as n
    big = f(2_000_000, 10_000, 200, 4, 10, 1 << 17)
    assert (1 << 31) <= big < (1 << 32)
    assert f(2_000_000, 1_000_000, 200, 4, 10, 1 << 17) == big
    assert f(1000, 10, 128, 4, 10, 1 << 20) == f(1000, 10, 128, 4, 10, 1000)
    # a short last batch that takes the few-query path (stored distances) is covered
    assert f(10_000_000, 8192 + 3, 96, 4, 10, 1 << 15) >= L.xbq_search_workspace_bytes(10_000_000, 3, 96, 4, 10)


def test_workspace_bytes(L):
    f = L.xbq_search_workspace_bytes
    assert f(1000, 10, 128, 4, 0) == 0
    assert f(1000, 10, 128, 4, 1001) == 0
    assert f(1000, 10, 128, 9, 10) == 0
    a = f(1_000_000, 10_000, 128, 4, 100)
    b = f(10_000_000, 10_000, 128, 4, 100)
    assert a == b and 0 < a < (1 << 30)             # independent of n once n is large
    assert f(1_000_000, 1_000_000, 128, 4, 100) < (1 << 30)      # bounded in m (internal batches)
    assert f(1_000_000, 1000, 960, 4, 10) > f(1_000_000, 1000, 128, 4, 10)   # repacked queries
    assert f(8_000_000, 4, 128, 4, 10) < 32 << 20                              # few queries: per-piece lists only
    assert f(1_000_000, 4, 128, 4, 1000) >= 4 * 1_000_000 * 4                   # k > 256: stored distances


def test_options(L):
    assert L.xbq_set_option(b"growth", 4.0) == xbq.OK
    assert L.xbq_set_option(b"growth", 1.0) == xbq.EINVAL
    assert L.xbq_set_option(b"nonsense", 1.0) == xbq.EINVAL
    assert L.xbq_set_option(None, 1.0) == xbq.EINVAL
    assert L.xbq_set_option(b"first", 1024) == xbq.OK
    assert L.xbq_set_option(b"qsplit", 0) == xbq.OK
    assert L.xbq_set_option(b"selector", 4) == xbq.EINVAL
    for sel in (1, 2, 3, 0):
        assert L.xbq_set_option(b"selector", sel) == xbq.OK
    assert L.xbq_set_option(b"hist_max_queries", 16) == xbq.OK
    assert L.xbq_set_option(b"kernel", 3) == xbq.EINVAL
    assert L.xbq_set_option(b"refine_growth", 1.0) == xbq.EINVAL
    assert L.xbq_set_option(b"refine_growth", 1.5) == xbq.OK
    assert L.xbq_set_option(b"kselect_lists_min", -1) == xbq.EINVAL
    assert L.xbq_set_option(b"kselect_lists_min", 128) == xbq.OK
    base = L.xbq_search_workspace_bytes(100_000, 1000, 128, 4, 10)
    assert L.xbq_set_option(b"kernel", 1) == xbq.OK
    assert L.xbq_search_workspace_bytes(100_000, 1000, 128, 4, 10) >= base + 100_000 * 64   # nibble copy of the rows
    assert L.xbq_set_option(b"kernel", 0) == xbq.OK


def test_options_per_call_do_not_touch_the_process_defaults(L):
    n, m, d, bits, k = 8_000_000, 4, 128, 4, 10
    stored = xbq.xbq_options_default(selector=2)          # histogram selection over stored distances
    local = xbq.xbq_options_default(selector=3)           # selection while the rows stream
    before = L.xbq_search_workspace_bytes(n, m, d, bits, k)
    a = xbq.xbq_search_workspace_bytes_ex(n, m, d, bits, k, stored)
    b = xbq.xbq_search_workspace_bytes_ex(n, m, d, bits, k, local)
    assert a >= m * n * 4 and b < a // 4                  # two option sets, two workspace sizes
    assert L.xbq_search_workspace_bytes(n, m, d, bits, k) == before           # the defaults did not move
    assert xbq.xbq_search_workspace_bytes_ex(n, m, d, bits, k, None) == before
    # and the other way round: changing the process defaults does not reach a call with its own options
    assert L.xbq_set_option(b"selector", 2) == xbq.OK
    try:
        assert L.xbq_search_workspace_bytes(n, m, d, bits, k) == a
        assert xbq.xbq_search_workspace_bytes_ex(n, m, d, bits, k, local) == b
    finally:
        assert L.xbq_set_option(b"selector", 0) == xbq.OK


def test_options_struct_is_validated(L):
    o = xbq.xbq_options_default()
    assert o.struct_bytes == ctypes.sizeof(xbq.XbqOptions) and o.growth == 4.0 and o.first == 1024
    assert o.selector == 0 and o.kernel == 0 and o.local_groups == 256 and o.refine_growth == 1.5
    assert o.row_order == 0
    fake, null = ctypes.c_void_p(0x1000), ctypes.c_void_p(0)

    def search(opt):
        return L.xbq_search_ex(fake, 1000, 4, fake, 10, 4, 128, 10, fake, fake, fake, 1 << 40,
                               ctypes.byref(opt) if opt is not None else None, null)

    for field, bad in (("growth", 1.0), ("selector", 7), ("kernel", -1), ("first", 5), ("qsplit", -2),
                       ("local_groups", 0), ("row_order", 2), ("hist_max_queries", -1), ("refine_growth", 100.0), ("struct_bytes", 8)):
        opt = xbq.xbq_options_default(**{field: bad})
        assert xbq.xbq_search_workspace_bytes_ex(1000, 10, 128, 4, 10, opt) == 0, field
        assert search(opt) == xbq.EINVAL, field
    # argument checks come before any GPU work for the _ex call as well
    assert L.xbq_search_ex(null, 1000, 4, fake, 10, 4, 128, 10, fake, fake, fake, 1 << 40, None, null) == xbq.EINVAL
    assert L.xbq_search_ex(fake, 1000, 4, fake, 10, 4, 128, 10, fake, fake, fake, 16, None, null) == xbq.EWORKSPACE
    assert L.xbq_search_ex(fake, 1000, 2, fake, 10, 4, 128, 10, fake, fake, fake, 1 << 40, None, null) == xbq.EUNSUPPORTED


def test_set_option_from_two_threads_keeps_a_consistent_default(L):
    import threading
    errors = []

    def worker(value):
        for _ in range(2000):
            if L.xbq_set_option(b"first", value) != xbq.OK:
                errors.append(value)
            w = L.xbq_search_workspace_bytes(100_000, 1000, 128, 4, 10)
            if w not in sizes:
                errors.append(w)

    sizes = set()
    for v in (512, 2048):
        assert L.xbq_set_option(b"first", v) == xbq.OK
        sizes.add(L.xbq_search_workspace_bytes(100_000, 1000, 128, 4, 10))
    assert len(sizes) == 2
    ts = [threading.Thread(target=worker, args=(v,)) for v in (512, 2048)]
    [t.start() for t in ts]
    [t.join() for t in ts]
    assert L.xbq_set_option(b"first", 1024) == xbq.OK
    assert not errors


def test_binding_rejects_tensors_the_library_could_not_check(L):
    """The C ABI sees raw pointers only; the binding refuses what would make a kernel read or
    write outside a buffer before anything reaches the GPU (host memory, wrong type)."""
    import torch
    cpu_codes = torch.zeros(1 << 16, dtype=torch.int32)
    with pytest.raises(ValueError, match="db_codes"):
        xbq.xbq_search(cpu_codes, 1000, cpu_codes, 4, 128, 4, 10)
    with pytest.raises(ValueError, match="db_codes"):
        xbq.xbq_search_asym(cpu_codes.float(), 1000, 3, cpu_codes, 4, 4, 128, 10)
    with pytest.raises(ValueError, match="db_codes"):
        xbq.xbq_search_ex(cpu_codes, 1000, 4, cpu_codes, 4, 4, 128, 10)
    with pytest.raises(ValueError, match="contiguous fp32 CUDA"):
        xbq.xbq_search_refine(torch.zeros(10, 8), cpu_codes, 4, torch.zeros(2, 8), cpu_codes, 4, 2, 0)
    with pytest.raises(ValueError, match="contiguous fp32 CUDA"):
        xbq.xbq_encode(torch.zeros(10, 8), 4)


def test_missing_library_is_loud(monkeypatch):
    monkeypatch.setattr(xbq, "_lib", None)
    monkeypatch.setattr(xbq, "LIB_PATH", "/nonexistent/libxbq.so")
    with pytest.raises(RuntimeError, match="no fallback"):
        xbq.lib()
