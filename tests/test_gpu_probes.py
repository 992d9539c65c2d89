"""The rate probes of the library write a checkable result: compare it with the closed
definition their header comment gives (plain NumPy here, nothing of the method)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from paper_2008_02002_amd import xbq


def _popcount(a):
    a = a.astype(np.uint64)
    c = np.zeros(a.shape, dtype=np.uint64)
    for s in range(32):
        c += (a >> np.uint64(s)) & np.uint64(1)
    return c


@pytest.mark.parametrize("iters,seed", [(1, 0), (5, 0xfffffffe), (64, 12345)])
def test_probe_valu_result(iters, seed):
    import torch
    print("probe valu", iters, seed, flush=True)
    out, ops = xbq.xbq_probe_valu(iters, seed)
    torch.cuda.synchronize()
    got = out.cpu().numpy().view(np.uint32)
    nthreads = xbq.xbq_probe_out_bytes() // 4
    assert got.shape == (nthreads,)
    assert ops == 2.0 * 16 * 4 * iters * nthreads
    t = np.concatenate([np.arange(0, 2048), np.arange(nthreads - 2048, nthreads)]).astype(np.uint64)
    want = np.zeros(t.shape, dtype=np.uint64)
    for j in range(16):
        x = ((t + 1) * 0x9E3779B1 + j * 0x85EBCA77) & 0xffffffff
        for i in range(4 * iters):
            want += _popcount(x ^ np.uint64((seed + i) & 0xffffffff))
    assert np.array_equal(got[t.astype(np.int64)].astype(np.uint64), want & 0xffffffff)


@pytest.mark.parametrize("nbytes", [16, 4096, 1 << 20, (1 << 26) + 16 * 12345])
def test_probe_read_sums_every_word_once(nbytes):
    import torch
    print("probe read", nbytes, flush=True)
    g = torch.Generator(device="cpu").manual_seed(nbytes)
    words = torch.randint(-2**31, 2**31 - 1, (nbytes // 4,), dtype=torch.int32, generator=g)
    dev = words.cuda()
    out = xbq.xbq_probe_read(dev)
    torch.cuda.synchronize()
    got = int(out.cpu().numpy().view(np.uint32).astype(np.uint64).sum()) & 0xffffffff
    want = int(words.numpy().view(np.uint32).astype(np.uint64).sum()) & 0xffffffff
    assert got == want


@pytest.mark.parametrize("n,d,bits", [(64, 128, 4), (1000, 200, 3), (130, 96, 4), (1, 4, 1), (4097, 960, 3)])
def test_probe_encode_traffic_reads_every_word_once_and_writes_every_code_word(n, d, bits):
    import torch
    print("probe encode traffic", n, d, bits, flush=True)
    g = torch.Generator(device="cpu").manual_seed(n + d)
    words = torch.randint(-2**31, 2**31 - 1, (n, d), dtype=torch.int32, generator=g)
    X = words.view(torch.float32).cuda()                 # any bit patterns: the probe only adds words
    W = (d + 31) // 32
    codes = torch.full((xbq.xbq_code_bytes(n, d, bits, xbq.BUNDLE64) // 4,), -1, dtype=torch.int32, device="cuda")
    xbq.xbq_probe_encode_traffic(X, bits, codes)
    torch.cuda.synchronize()
    got = codes.cpu().numpy().view(np.uint32).reshape(-1, bits * W * 64)
    w32 = words.numpy().view(np.uint32).astype(np.uint64)
    for b in range(got.shape[0]):
        rows = w32[b * 64:(b + 1) * 64].reshape(-1, 4).sum(axis=1)      # one sum per 16-byte group of the bundle
        want = np.zeros(256, dtype=np.uint64)
        np.add.at(want, np.arange(rows.shape[0]) % 256, rows)
        t = np.arange(bits * W * 64) % 256
        assert np.array_equal(got[b].astype(np.uint64), want[t] & 0xffffffff), f"bundle {b}"


def test_probe_argument_errors():
    import ctypes
    import torch
    L = xbq.lib()
    small = torch.empty(16, dtype=torch.int32, device="cuda")
    big = torch.empty(xbq.xbq_probe_out_bytes() // 4, dtype=torch.int32, device="cuda")
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    assert L.xbq_probe_valu(p(small), 64, 0, 1, None, None) == xbq.EWORKSPACE
    assert L.xbq_probe_valu(p(big), big.numel() * 4, 0, 0, None, None) == xbq.EINVAL
    assert L.xbq_probe_valu(None, big.numel() * 4, 0, 1, None, None) == xbq.EINVAL
    assert L.xbq_probe_read(p(big), 24, p(big), big.numel() * 4, None) == xbq.EINVAL          # not a multiple of 16
    assert L.xbq_probe_read(ctypes.c_void_p(big.data_ptr() + 4), 16, p(big), big.numel() * 4, None) == xbq.EINVAL
    assert L.xbq_probe_read(p(big), 16, p(small), 64, None) == xbq.EWORKSPACE
    assert L.xbq_probe_encode_traffic(p(big), 64, 130, 4, p(big), None) == xbq.EUNSUPPORTED     # d not a multiple of 4
    assert L.xbq_probe_encode_traffic(ctypes.c_void_p(big.data_ptr() + 4), 64, 128, 4, p(big), None) == xbq.EINVAL
    assert L.xbq_probe_encode_traffic(None, 64, 128, 4, p(big), None) == xbq.EINVAL
    assert L.xbq_probe_encode_traffic(None, 0, 128, 4, None, None) == xbq.OK


def test_binding_loaded_before_any_other_gpu_use_shares_one_runtime():
    """A fresh process that touches the binding before anything else has initialised the GPU
    must still launch on the runtime that owns the tensors."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = (
        "import sys; sys.path.insert(0, %r)\n"
        "from paper_2008_02002_amd import xbq\n"
        "xbq.xbq_set_option('growth', 4.0)\n"          # loads the library first
        "import numpy as np, torch\n"
        "X = torch.from_numpy(np.linspace(-0.9, 0.9, 64 * 32, dtype=np.float32).reshape(64, 32)).cuda()\n"
        "c = xbq.xbq_encode(X, 4, 1.0, xbq.ROWS); torch.cuda.synchronize()\n"
        "idx, score = xbq.xbq_search(xbq.xbq_encode(X, 4, 1.0, xbq.BUNDLE64), 64, c, 64, 32, 4, 1)\n"
        "torch.cuda.synchronize(); print('loaded-first ok', int(c.numel()), int(idx.numel()))\n" % root)
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stderr[-2000:]
    assert "loaded-first ok 256 64" in r.stdout
