"""ctypes binding of libxbq.so: same names as the C ABI in ``include/xbq.h``.

Argument marshalling only.  Tensors are torch CUDA tensors used as device memory; the
current torch stream is handed to the library.  Every step of the path runs in the HIP
kernels behind the C ABI; there is no CPU fallback, and a missing library is an error.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libxbq.so")

OK, EINVAL, EUNSUPPORTED, EWORKSPACE, EHIP, ESTATIC = 0, -1, -2, -3, -4, -5
STATIC_SCRATCH_BYTES = 32 << 20
ROWS, BUNDLE64 = 0, 1
MAX_BITS, MAX_DIM, MAX_K = 4, 2048, 1024
REFINE_MAX_CANDIDATES = 2048

EXPORTS = (
    "xbq_version", "xbq_strerror", "xbq_last_hip_error", "xbq_code_bytes", "xbq_encode",
    "xbq_search_workspace_bytes", "xbq_search", "xbq_search_asym", "xbq_search_static", "xbq_search_ex", "xbq_search_workspace_bytes_ex", "xbq_options_default", "xbq_search_refine_workspace_bytes", "xbq_search_refine", "xbq_k_select_workspace_bytes", "xbq_k_select", "xbq_trace_enable", "xbq_trace_read",
    "xbq_probe_out_bytes", "xbq_probe_valu", "xbq_probe_read", "xbq_probe_encode_traffic", "xbq_set_option",
)

_lib = None


class XbqOptions(ctypes.Structure):
    """struct xbq_options of the C ABI."""
    _fields_ = [("struct_bytes", ctypes.c_uint32), ("selector", ctypes.c_int32), ("kernel", ctypes.c_int32),
                ("first", ctypes.c_int32), ("qsplit", ctypes.c_int32), ("hist_max_queries", ctypes.c_int32),
                ("kselect_lists_min", ctypes.c_int32), ("local_groups", ctypes.c_int32),
                ("row_order", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("growth", ctypes.c_double), ("refine_growth", ctypes.c_double)]


class XbqError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = lib().xbq_strerror(code).decode()
        if code == EHIP:
            msg += f" (hipError {lib().xbq_last_hip_error()})"
        super().__init__(f"{where}: {msg} [{code}]")


def lib() -> ctypes.CDLL:
    """Load libxbq.so (built by ``python -m paper_2008_02002_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2008_02002_amd.build`; "
                "there is no fallback path")
        # PyTorch ships its own copy of the HIP runtime.  The tensors this binding takes live in
        # that runtime, so it has to be the one libxbq.so binds to: load it first.  (Loaded the
        # other way round, the process ends up with two runtimes and launches fail.)
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = ctypes.CDLL(LIB_PATH)
        i64, i32, vp, f32, sz = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_float, ctypes.c_size_t
        L.xbq_version.restype = i32
        L.xbq_strerror.argtypes = [i32]
        L.xbq_strerror.restype = ctypes.c_char_p
        L.xbq_last_hip_error.restype = i32
        L.xbq_code_bytes.argtypes = [i64, i32, i32, i32]
        L.xbq_code_bytes.restype = sz
        L.xbq_encode.argtypes = [vp, i64, i32, i32, f32, i32, vp, vp]
        L.xbq_encode.restype = i32
        L.xbq_search_workspace_bytes.argtypes = [i64, i64, i32, i32, i32]
        L.xbq_search_workspace_bytes.restype = sz
        L.xbq_search.argtypes = [vp, i64, vp, i64, i32, i32, i32, vp, vp, vp, sz, vp]
        L.xbq_search.restype = i32
        L.xbq_search_asym.argtypes = [vp, i64, i32, vp, i64, i32, i32, i32, vp, vp, vp, sz, vp]
        L.xbq_search_asym.restype = i32
        L.xbq_options_default.argtypes = [ctypes.POINTER(XbqOptions)]
        L.xbq_options_default.restype = None
        L.xbq_search_workspace_bytes_ex.argtypes = [i64, i64, i32, i32, i32, ctypes.POINTER(XbqOptions)]
        L.xbq_search_workspace_bytes_ex.restype = sz
        L.xbq_search_ex.argtypes = [vp, i64, i32, vp, i64, i32, i32, i32, vp, vp, vp, sz, ctypes.POINTER(XbqOptions), vp]
        L.xbq_search_ex.restype = i32
        L.xbq_search_static.argtypes = [vp, i64, vp, i64, i32, i32, i32, vp, vp, vp]
        L.xbq_search_static.restype = i32
        L.xbq_search_refine_workspace_bytes.argtypes = [i64, i64, i32, i32, i32]
        L.xbq_search_refine_workspace_bytes.restype = sz
        L.xbq_search_refine.argtypes = [vp, vp, i64, i32, vp, vp, i64, i32, i32, i32, i32, vp, vp, vp, vp, sz, vp]
        L.xbq_search_refine.restype = i32
        L.xbq_k_select_workspace_bytes.argtypes = [i64, i64, i32, i32, i32, i32, i64]
        L.xbq_k_select_workspace_bytes.restype = sz
        L.xbq_k_select.argtypes = [vp, vp, i64, i32, vp, vp, i64, i32, i32, i32, i32, i64, vp, vp, vp, vp, sz, vp]
        L.xbq_k_select.restype = i32
        L.xbq_trace_enable.argtypes = [i32]
        L.xbq_trace_enable.restype = i32
        L.xbq_trace_read.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64),
                                     ctypes.POINTER(ctypes.c_double)]
        L.xbq_trace_read.restype = i32
        L.xbq_probe_out_bytes.restype = sz
        L.xbq_probe_valu.argtypes = [vp, sz, ctypes.c_uint32, i32, ctypes.POINTER(ctypes.c_double), vp]
        L.xbq_probe_valu.restype = i32
        L.xbq_probe_read.argtypes = [vp, sz, vp, sz, vp]
        L.xbq_probe_read.restype = i32
        L.xbq_probe_encode_traffic.argtypes = [vp, i64, i32, i32, vp, vp]
        L.xbq_probe_encode_traffic.restype = i32
        L.xbq_set_option.argtypes = [ctypes.c_char_p, ctypes.c_double]
        L.xbq_set_option.restype = i32
        _lib = L
    return _lib


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(code: int, where: str):
    if code != OK:
        raise XbqError(code, where)


def _require_codes(t, n: int, d: int, bits: int, layout: int, name: str):
    """Host-side check of a codes tensor: the C ABI takes raw pointers and cannot see that a
    buffer is too small or in the wrong place, and a scan that reads past it faults the GPU."""
    import torch
    need = xbq_code_bytes(n, d, bits, layout)
    if need == 0 and n != 0:
        raise XbqError(EUNSUPPORTED, "xbq_code_bytes")
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.int32 and t.is_contiguous()):
        raise ValueError(f"{name} must be a contiguous int32 CUDA tensor (uint32 plane words)")
    if t.numel() * 4 < need:
        kind = "BUNDLE64" if layout == BUNDLE64 else "ROWS"
        raise ValueError(f"{name} holds {t.numel() * 4} bytes, but {n} rows of d={d}, bits={bits} in the {kind} layout "
                         f"take {need}: wrong layout or row count?")


def _require_out(t, shape, dtype, name: str):
    import torch
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous() and
            tuple(t.shape) == tuple(shape)):
        raise ValueError(f"{name} must be a contiguous CUDA tensor of shape {tuple(shape)} and dtype {dtype}")


def _require_workspace(t, need: int):
    import torch
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous()):
        raise ValueError("workspace must be a contiguous CUDA tensor")
    if t.numel() * t.element_size() < need:
        raise XbqError(EWORKSPACE, "workspace")
    if t.data_ptr() % 256:
        raise ValueError("workspace must be 256-byte aligned")


def xbq_version() -> int:
    return lib().xbq_version()


def xbq_code_bytes(n: int, d: int, bits: int, layout: int) -> int:
    return lib().xbq_code_bytes(n, d, bits, layout)


def xbq_search_workspace_bytes(n: int, m: int, d: int, bits: int, k: int) -> int:
    return lib().xbq_search_workspace_bytes(n, m, d, bits, k)


def xbq_set_option(name: str, value: float):
    _check(lib().xbq_set_option(name.encode(), float(value)), "xbq_set_option")


def xbq_encode(X, bits: int, scale: float = 1.0, layout: int = ROWS, out=None):
    """X: fp32 CUDA tensor [n, d] (contiguous).  Returns an int32 CUDA tensor holding the
    uint32 plane words (flat, xbq_code_bytes / 4 elements)."""
    import torch
    if not (X.is_cuda and X.dtype == torch.float32 and X.is_contiguous() and X.dim() == 2):
        raise ValueError("X must be a contiguous fp32 CUDA tensor [n, d]")
    n, d = X.shape
    nbytes = xbq_code_bytes(n, d, bits, layout)
    if nbytes == 0 and n != 0:
        raise XbqError(EUNSUPPORTED, "xbq_code_bytes")
    if out is None:
        out = torch.empty(nbytes // 4, dtype=torch.int32, device=X.device)
    elif not (out.is_cuda and out.is_contiguous() and out.numel() * out.element_size() >= nbytes):
        raise ValueError("out too small")
    rc = lib().xbq_encode(ctypes.c_void_p(X.data_ptr()), n, d, bits, scale, layout,
                          ctypes.c_void_p(out.data_ptr()), _stream())
    _check(rc, "xbq_encode")
    return out


def xbq_search(db_codes, n: int, q_codes, m: int, d: int, bits: int, k: int, workspace=None,
               idx=None, score=None):
    """Returns (idx int32 [m, k], score int32 [m, k]) CUDA tensors."""
    import torch
    dev = db_codes.device
    need = xbq_search_workspace_bytes(n, m, d, bits, k)
    if need == 0:
        raise XbqError(EINVAL, "xbq_search_workspace_bytes")
    _require_codes(db_codes, n, d, bits, BUNDLE64, "db_codes")
    _require_codes(q_codes, m, d, bits, ROWS, "q_codes")
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    if idx is None:
        idx = torch.empty((m, k), dtype=torch.int32, device=dev)
    if score is None:
        score = torch.empty((m, k), dtype=torch.int32, device=dev)
    _require_workspace(workspace, need)
    _require_out(idx, (m, k), torch.int32, "idx")
    _require_out(score, (m, k), torch.int32, "score")
    rc = lib().xbq_search(ctypes.c_void_p(db_codes.data_ptr()), n, ctypes.c_void_p(q_codes.data_ptr()), m,
                          d, bits, k, ctypes.c_void_p(idx.data_ptr()), ctypes.c_void_p(score.data_ptr()),
                          ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size(),
                          _stream())
    _check(rc, "xbq_search")
    return idx, score


def xbq_options_default(**fields) -> XbqOptions:
    """The built-in defaults, with the given fields replaced."""
    o = XbqOptions()
    lib().xbq_options_default(ctypes.byref(o))
    for name, value in fields.items():
        if name not in dict(XbqOptions._fields_):
            raise ValueError(f"no such option: {name}")
        setattr(o, name, value)
    return o


def xbq_search_workspace_bytes_ex(n: int, m: int, d: int, q_bits: int, k: int, options=None) -> int:
    return lib().xbq_search_workspace_bytes_ex(n, m, d, q_bits, k, ctypes.byref(options) if options is not None else None)


def xbq_search_ex(db_codes, n: int, db_bits: int, q_codes, m: int, q_bits: int, d: int, k: int, options=None,
                  workspace=None, idx=None, score=None):
    """xbq_search_asym with the schedule options passed per call (an XbqOptions or None)."""
    import torch
    dev = db_codes.device
    need = xbq_search_workspace_bytes_ex(n, m, d, q_bits, k, options)
    if need == 0:
        raise XbqError(EINVAL, "xbq_search_workspace_bytes_ex")
    _require_codes(db_codes, n, d, db_bits, BUNDLE64, "db_codes")
    _require_codes(q_codes, m, d, q_bits, ROWS, "q_codes")
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    if idx is None:
        idx = torch.empty((m, k), dtype=torch.int32, device=dev)
    if score is None:
        score = torch.empty((m, k), dtype=torch.int32, device=dev)
    _require_workspace(workspace, need)
    _require_out(idx, (m, k), torch.int32, "idx")
    _require_out(score, (m, k), torch.int32, "score")
    rc = lib().xbq_search_ex(ctypes.c_void_p(db_codes.data_ptr()), n, db_bits, ctypes.c_void_p(q_codes.data_ptr()), m,
                             q_bits, d, k, ctypes.c_void_p(idx.data_ptr()), ctypes.c_void_p(score.data_ptr()),
                             ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size(),
                             ctypes.byref(options) if options is not None else None, _stream())
    _check(rc, "xbq_search_ex")
    return idx, score


def xbq_search_static(db_codes, n: int, q_codes, m: int, d: int, bits: int, k: int, idx, score):
    """xbq_search without a workspace and without any allocation: idx and score ([m, k] int32
    CUDA tensors) come from the caller, the scratch memory is the library's built-in buffer."""
    import torch
    _require_codes(db_codes, n, d, bits, BUNDLE64, "db_codes")
    _require_codes(q_codes, m, d, bits, ROWS, "q_codes")
    _require_out(idx, (m, k), torch.int32, "idx")
    _require_out(score, (m, k), torch.int32, "score")
    rc = lib().xbq_search_static(ctypes.c_void_p(db_codes.data_ptr()), n, ctypes.c_void_p(q_codes.data_ptr()), m,
                                 d, bits, k, ctypes.c_void_p(idx.data_ptr()), ctypes.c_void_p(score.data_ptr()),
                                 _stream())
    _check(rc, "xbq_search_static")
    return idx, score


def xbq_search_asym(db_codes, n: int, db_bits: int, q_codes, m: int, q_bits: int, d: int, k: int,
                    workspace=None, idx=None, score=None):
    """Search with q_bits-plane query codes against db_bits-plane database codes."""
    import torch
    dev = db_codes.device
    need = xbq_search_workspace_bytes(n, m, d, q_bits, k)
    if need == 0:
        raise XbqError(EINVAL, "xbq_search_workspace_bytes")
    _require_codes(db_codes, n, d, db_bits, BUNDLE64, "db_codes")
    _require_codes(q_codes, m, d, q_bits, ROWS, "q_codes")
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    if idx is None:
        idx = torch.empty((m, k), dtype=torch.int32, device=dev)
    if score is None:
        score = torch.empty((m, k), dtype=torch.int32, device=dev)
    _require_workspace(workspace, need)
    _require_out(idx, (m, k), torch.int32, "idx")
    _require_out(score, (m, k), torch.int32, "score")
    rc = lib().xbq_search_asym(ctypes.c_void_p(db_codes.data_ptr()), n, db_bits, ctypes.c_void_p(q_codes.data_ptr()),
                               m, q_bits, d, k, ctypes.c_void_p(idx.data_ptr()), ctypes.c_void_p(score.data_ptr()),
                               ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size(),
                               _stream())
    _check(rc, "xbq_search_asym")
    return idx, score


def xbq_search_refine(X_db, db_codes, db_bits: int, X_q, q_codes, q_bits: int, k: int, extra_distance: int,
                      workspace=None, idx=None, sim=None, cand=None):
    """Candidate search + fp32 refine.  Returns (idx int32 [m, k], similarity fp32 [m, k],
    candidates int32 [m]) CUDA tensors."""
    import torch
    n, d = X_db.shape
    m = X_q.shape[0]
    for t in (X_db, X_q):
        if not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()):
            raise ValueError("X_db and X_q must be contiguous fp32 CUDA tensors")
    need = lib().xbq_search_refine_workspace_bytes(n, m, d, q_bits, k)
    if need == 0:
        raise XbqError(EINVAL, "xbq_search_refine_workspace_bytes")
    if X_q.dim() != 2 or X_db.dim() != 2 or X_q.shape[1] != d:
        raise ValueError("X_db and X_q must be [n, d] and [m, d] with the same d")
    _require_codes(db_codes, n, d, db_bits, BUNDLE64, "db_codes")
    _require_codes(q_codes, m, d, q_bits, ROWS, "q_codes")
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=X_db.device)
    if idx is None:
        idx = torch.empty((m, k), dtype=torch.int32, device=X_db.device)
    if sim is None:
        sim = torch.empty((m, k), dtype=torch.float32, device=X_db.device)
    if cand is None:
        cand = torch.empty((m,), dtype=torch.int32, device=X_db.device)
    _require_workspace(workspace, need)
    _require_out(idx, (m, k), torch.int32, "idx")
    _require_out(sim, (m, k), torch.float32, "similarity")
    _require_out(cand, (m,), torch.int32, "candidates")
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    rc = lib().xbq_search_refine(p(X_db), p(db_codes), n, db_bits, p(X_q), p(q_codes), m, q_bits, d, k,
                                 int(extra_distance), p(idx), p(sim), p(cand), p(workspace),
                                 workspace.numel() * workspace.element_size(), _stream())
    _check(rc, "xbq_search_refine")
    return idx, sim, cand


def xbq_k_select(X_db, db_codes, db_bits: int, X_q, q_codes, q_bits: int, k: int, extra_distance: int,
                 max_candidates: int, workspace=None, idx=None, sim=None, cand=None):
    """Algorithm 1 with the whole candidate list.  Returns (idx int32 [m, k], similarity fp32
    [m, k], candidates int32 [m]) CUDA tensors."""
    import torch
    n, d = X_db.shape
    m = X_q.shape[0]
    for t in (X_db, X_q):
        if not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()):
            raise ValueError("X_db and X_q must be contiguous fp32 CUDA tensors")
    need = lib().xbq_k_select_workspace_bytes(n, m, d, q_bits, k, int(extra_distance), int(max_candidates))
    if need == 0:
        raise XbqError(EINVAL, "xbq_k_select_workspace_bytes")
    if X_q.dim() != 2 or X_db.dim() != 2 or X_q.shape[1] != d:
        raise ValueError("X_db and X_q must be [n, d] and [m, d] with the same d")
    _require_codes(db_codes, n, d, db_bits, BUNDLE64, "db_codes")
    _require_codes(q_codes, m, d, q_bits, ROWS, "q_codes")
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=X_db.device)
    if idx is None:
        idx = torch.empty((m, k), dtype=torch.int32, device=X_db.device)
    if sim is None:
        sim = torch.empty((m, k), dtype=torch.float32, device=X_db.device)
    if cand is None:
        cand = torch.empty((m,), dtype=torch.int32, device=X_db.device)
    _require_workspace(workspace, need)
    _require_out(idx, (m, k), torch.int32, "idx")
    _require_out(sim, (m, k), torch.float32, "similarity")
    _require_out(cand, (m,), torch.int32, "candidates")
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    rc = lib().xbq_k_select(p(X_db), p(db_codes), n, db_bits, p(X_q), p(q_codes), m, q_bits, d, k,
                            int(extra_distance), int(max_candidates), p(idx), p(sim), p(cand), p(workspace),
                            workspace.numel() * workspace.element_size(), _stream())
    _check(rc, "xbq_k_select")
    return idx, sim, cand


def xbq_trace_enable(on: bool):
    _check(lib().xbq_trace_enable(1 if on else 0), "xbq_trace_enable")


def xbq_trace_read():
    """(scan kernel milliseconds, launches, pairs scored) since the last read."""
    ms, n, pairs = ctypes.c_double(), ctypes.c_int64(), ctypes.c_double()
    _check(lib().xbq_trace_read(ctypes.byref(ms), ctypes.byref(n), ctypes.byref(pairs)), "xbq_trace_read")
    return ms.value, n.value, pairs.value


def xbq_probe_out_bytes() -> int:
    return lib().xbq_probe_out_bytes()


def xbq_probe_valu(iters: int, seed: int = 1, out=None):
    """Launch the XOR + population-count rate probe.  Returns (out uint32-as-int32 CUDA tensor,
    lane operations of the launch)."""
    import torch
    if out is None:
        out = torch.empty(xbq_probe_out_bytes() // 4, dtype=torch.int32, device="cuda")
    ops = ctypes.c_double()
    _check(lib().xbq_probe_valu(ctypes.c_void_p(out.data_ptr()), out.numel() * out.element_size(), seed & 0xffffffff,
                                int(iters), ctypes.byref(ops), _stream()), "xbq_probe_valu")
    return out, ops.value


def xbq_probe_read(buf, out=None):
    """Launch the streaming-read probe over a contiguous CUDA tensor.  Returns the per-workgroup
    word sums (uint32 as int32, the first 2048 entries of out)."""
    import torch
    if not (buf.is_cuda and buf.is_contiguous()):
        raise ValueError("buf must be a contiguous CUDA tensor")
    if out is None:
        out = torch.empty(xbq_probe_out_bytes() // 4, dtype=torch.int32, device=buf.device)
    _check(lib().xbq_probe_read(ctypes.c_void_p(buf.data_ptr()), buf.numel() * buf.element_size(),
                                ctypes.c_void_p(out.data_ptr()), out.numel() * out.element_size(), _stream()),
           "xbq_probe_read")
    return out[:2048]


def xbq_probe_encode_traffic(X, bits: int, codes):
    """Launch the probe that moves the encoder's bytes without its arithmetic: reads X (fp32 CUDA
    tensor [n, d]) and overwrites `codes` (a BUNDLE64 codes tensor for n rows)."""
    import torch
    if not (X.is_cuda and X.dtype == torch.float32 and X.is_contiguous() and X.dim() == 2):
        raise ValueError("X must be a contiguous fp32 CUDA tensor [n, d]")
    n, d = X.shape
    if not (codes.is_cuda and codes.is_contiguous() and
            codes.numel() * codes.element_size() >= xbq_code_bytes(n, d, bits, BUNDLE64)):
        raise ValueError("codes too small")
    _check(lib().xbq_probe_encode_traffic(ctypes.c_void_p(X.data_ptr()), n, d, bits, ctypes.c_void_p(codes.data_ptr()),
                                          _stream()), "xbq_probe_encode_traffic")
    return codes
