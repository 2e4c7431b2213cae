"""ctypes binding of libsvb.so.  Same names as the C entry points (include/svb.h).

Device buffers are torch tensors (PyTorch supplies device memory and streams
only); host buffers are numpy arrays.  There is no fallback: if the library
is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

SVB_F64, SVB_F32, SVB_F16, SVB_BF16 = 0, 1, 2, 3
SVB_OK = 0

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsvb.so")
_lib = None

_i64 = ctypes.c_int64
_vp = ctypes.c_void_p
_szp = ctypes.POINTER(ctypes.c_size_t)
_dp = ctypes.POINTER(ctypes.c_double)


class SvbError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = int(status)
        super().__init__(f"{where}: {svb_status_string(status)} (status {status})")


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libsvb.so (built in-tree by paper_2508_06339_amd.build); raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} not found: build it with `python -m paper_2508_06339_amd.build` "
            "(there is no CPU fallback)")
    lib = ctypes.CDLL(_LIB_PATH)
    lib.svb_workspace_bytes.argtypes = [ctypes.c_int, _i64, _i64, ctypes.c_int, _szp, _szp]
    lib.svb_workspace_bytes.restype = ctypes.c_int
    lib.svb_svdvals.argtypes = [ctypes.c_int, _i64, _i64, _vp, _i64, _vp, ctypes.c_int, _vp,
                                ctypes.c_size_t, _vp]
    lib.svb_svdvals.restype = ctypes.c_int
    lib.svb_ge2gb.argtypes = [ctypes.c_int, _i64, _i64, _vp, _i64, ctypes.c_int, _vp, _i64, _vp,
                              ctypes.c_size_t, _vp]
    lib.svb_ge2gb.restype = ctypes.c_int
    lib.svb_gb2bd.argtypes = [ctypes.c_int, _i64, ctypes.c_int, _vp, _i64, _vp, _vp, _vp,
                              ctypes.c_size_t, _vp]
    lib.svb_gb2bd.restype = ctypes.c_int
    lib.svb_gb2bd_noalloc.argtypes = [ctypes.c_int, _i64, ctypes.c_int, _vp, _i64, _vp, _vp, _vp]
    lib.svb_gb2bd_noalloc.restype = ctypes.c_int
    lib.svb_choose_nb.argtypes = [ctypes.c_int, _i64, _i64]
    lib.svb_choose_nb.restype = ctypes.c_int
    lib.svb_gb2bd_workspace_bytes.argtypes = [_i64, ctypes.c_int, _szp]
    lib.svb_gb2bd_workspace_bytes.restype = ctypes.c_int
    lib.svb_bdsvals_dev_workspace_bytes.argtypes = [_i64, _szp]
    lib.svb_bdsvals_dev_workspace_bytes.restype = ctypes.c_int
    lib.svb_bdsvals_dev.argtypes = [ctypes.c_int, _i64, _vp, _vp, _vp, ctypes.c_double, _vp, ctypes.c_size_t, _vp]
    lib.svb_bdsvals_dev.restype = ctypes.c_int
    lib.svb_bdsvals.argtypes = [_i64, _dp, _dp, _dp]
    lib.svb_bdsvals.restype = ctypes.c_int
    lib.svb_last_timings.argtypes = [_dp, _dp, _dp, _dp]
    lib.svb_last_timings.restype = ctypes.c_int
    lib.svb_profile_enable.argtypes = [ctypes.c_int]
    lib.svb_profile_enable.restype = ctypes.c_int
    lib.svb_profile_collect.argtypes = []
    lib.svb_profile_collect.restype = ctypes.c_int
    lib.svb_profile_get.argtypes = [ctypes.c_int, _dp, ctypes.POINTER(_i64), _dp, _dp]
    lib.svb_profile_get.restype = ctypes.c_int
    lib.svb_status_string.argtypes = [ctypes.c_int]
    lib.svb_status_string.restype = ctypes.c_char_p
    _lib = lib
    return lib


def svb_status_string(status: int) -> str:
    return load_library().svb_status_string(int(status)).decode()


def dtype_code(torch_dtype) -> int:
    import torch
    return {torch.float64: SVB_F64, torch.float32: SVB_F32, torch.float16: SVB_F16,
            torch.bfloat16: SVB_BF16}[torch_dtype]


def _ptr(t):
    return _vp(0) if t is None else _vp(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        return _vp(torch.cuda.current_stream().cuda_stream)
    return _vp(int(stream))


def svb_workspace_bytes(dt: int, m: int, n: int, nb: int):
    """Returns (status, dev_bytes, host_bytes)."""
    dev = ctypes.c_size_t(0)
    host = ctypes.c_size_t(0)
    rc = load_library().svb_workspace_bytes(dt, m, n, nb, ctypes.byref(dev), ctypes.byref(host))
    return rc, dev.value, host.value


def svb_svdvals(dt, m, n, A_dev, lda, S_out_host: np.ndarray, nb, work_dev, work_bytes, stream=None) -> int:
    return load_library().svb_svdvals(dt, m, n, _ptr(A_dev), lda, _vp(S_out_host.ctypes.data), nb,
                                      _ptr(work_dev), work_bytes, _stream(stream))


def svb_ge2gb(dt, m, n, A_dev, lda, nb, band_dev, ldab, work_dev, work_bytes, stream=None) -> int:
    return load_library().svb_ge2gb(dt, m, n, _ptr(A_dev), lda, nb, _ptr(band_dev), ldab,
                                    _ptr(work_dev), work_bytes, _stream(stream))


def svb_gb2bd(band_dt, n, nb, band_dev, ldab, d_dev, e_dev, work_dev, work_bytes, stream=None) -> int:
    return load_library().svb_gb2bd(band_dt, n, nb, _ptr(band_dev), ldab, _ptr(d_dev), _ptr(e_dev),
                                    _ptr(work_dev), work_bytes, _stream(stream))


def svb_gb2bd_noalloc(band_dt, n, nb, band_dev, ldab, d_dev, e_dev, stream=None) -> int:
    return load_library().svb_gb2bd_noalloc(band_dt, n, nb, _ptr(band_dev), ldab, _ptr(d_dev), _ptr(e_dev),
                                            _stream(stream))


def svb_choose_nb(dt: int, m: int, n: int) -> int:
    return load_library().svb_choose_nb(dt, m, n)


def svb_gb2bd_workspace_bytes(n: int, nb: int):
    """Returns (status, dev_bytes)."""
    dev = ctypes.c_size_t(0)
    rc = load_library().svb_gb2bd_workspace_bytes(n, nb, ctypes.byref(dev))
    return rc, dev.value


def svb_bdsvals_dev_workspace_bytes(n: int):
    """Returns (status, dev_bytes)."""
    dev = ctypes.c_size_t(0)
    rc = load_library().svb_bdsvals_dev_workspace_bytes(n, ctypes.byref(dev))
    return rc, dev.value


def svb_bdsvals_dev(band_dt, n, d_dev, e_dev, sigma_dev, rel_tol, work_dev, work_bytes, stream=None) -> int:
    return load_library().svb_bdsvals_dev(band_dt, n, _ptr(d_dev), _ptr(e_dev), _ptr(sigma_dev), float(rel_tol),
                                          _ptr(work_dev), work_bytes, _stream(stream))


def svb_bdsvals(n: int, d: np.ndarray, e: np.ndarray, sigma: np.ndarray) -> int:
    def p(a):
        return a.ctypes.data_as(_dp) if a is not None and a.size else ctypes.cast(None, _dp)
    return load_library().svb_bdsvals(n, p(d), p(e), p(sigma))


def svb_last_timings():
    """(t_panel, t_update, t_stage2, t_stage3) in seconds; t_panel is -1 without per-kernel events."""
    t = [ctypes.c_double(0.0) for _ in range(4)]
    load_library().svb_last_timings(*[ctypes.byref(x) for x in t])
    return tuple(x.value for x in t)


SVB_PROF_PANEL, SVB_PROF_UPDATE, SVB_PROF_UPDATE_UPPER, SVB_PROF_BAND_REDUCE, SVB_PROF_NARROW, SVB_PROF_STAGE3 = range(6)
SVB_PROF_NAMES = ("panel", "update", "update_upper", "band_reduce", "narrow_chase", "stage3")


def svb_profile_enable(on: bool) -> int:
    return load_library().svb_profile_enable(1 if on else 0)


def svb_profile_collect() -> int:
    return load_library().svb_profile_collect()


def svb_profile_get(kind: int) -> dict:
    sec, fl, by = ctypes.c_double(0), ctypes.c_double(0), ctypes.c_double(0)
    cnt = _i64(0)
    rc = load_library().svb_profile_get(kind, ctypes.byref(sec), ctypes.byref(cnt), ctypes.byref(fl), ctypes.byref(by))
    if rc != SVB_OK:
        raise SvbError(rc, "svb_profile_get")
    return dict(seconds=sec.value, launches=cnt.value, flops=fl.value, bytes=by.value)


def svdvals(A, nb: int = 0, overwrite: bool = False, work=None):
    """Singular values (descending, numpy) of a 2-D torch tensor on the GPU.

    The tensor's memory is read as a column-major matrix: a row-major (C-contiguous)
    r x c tensor is handed over as the c x r matrix with lda = c, its transpose, which
    has the same singular values; a column-major one (the transpose of a contiguous
    tensor) as it is.  nb = 0 lets the library choose the tile size.  Marshals arguments
    for svb_svdvals; allocates the workspace with torch unless one is passed in.
    """
    import torch
    if A.dim() != 2 or not A.is_cuda:
        raise ValueError("expected a 2-D CUDA tensor")
    if A.is_contiguous():
        m, n = A.shape[1], A.shape[0]
    elif A.t().is_contiguous():
        m, n = A.shape[0], A.shape[1]
    else:
        raise ValueError("expected a dense row- or column-major tensor")
    dt = dtype_code(A.dtype)
    buf = A if overwrite else A.clone(memory_format=torch.preserve_format)
    rc, dev_bytes, _ = svb_workspace_bytes(dt, m, n, nb)
    if rc != SVB_OK:
        raise SvbError(rc, "svb_workspace_bytes")
    if work is None:
        work = torch.empty(dev_bytes, dtype=torch.uint8, device=A.device)
    out = np.empty(min(m, n), dtype=np.float64 if dt == SVB_F64 else np.float32)
    rc = svb_svdvals(dt, m, n, buf, m, out, nb, work, work.numel())
    if rc != SVB_OK:
        raise SvbError(rc, "svb_svdvals")
    return out
