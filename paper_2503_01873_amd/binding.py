"""ctypes binding with the same names as include/pasa.h.  Argument marshalling only.

Tensors are anything with `.data_ptr()` (torch tensors on the GPU); raw integer addresses are accepted
too.  Nothing here computes: if libpasa.so is missing or cannot be loaded the import of `lib()` fails
loudly -- there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os

MIXED, STRICT16, NAIVE16, S16, DIRECT = 0, 1, 2, 3, 4
SHIFT_MEAN, SHIFT_MATRIX, SHIFT_MATRIX_MFMA = 0, 1, 2
IO_F16, IO_BF16 = 0, 1

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.environ.get("PASA_LIB") or os.path.join(_PKG, "libpasa.so")
_lib = None


class PasaError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: status {status} ({pasa_status_string(status)})")
        self.status = status


class pasa_opts(ctypes.Structure):
    _fields_ = [
        ("beta", ctypes.c_float),
        ("variant", ctypes.c_int),
        ("shift_tile", ctypes.c_int),
        ("overflow_s", ctypes.c_void_p),
        ("nonfinite_o", ctypes.c_void_p),
        ("shift_mode", ctypes.c_int),
        ("io_dtype", ctypes.c_int),
    ]


def lib_path() -> str:
    return _LIB_PATH


def lib() -> ctypes.CDLL:
    """Load libpasa.so (built in-tree by paper_2503_01873_amd.build).  Raises if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2503_01873_amd.build` "
            "(there is no CPU fallback)")
    L = ctypes.CDLL(_LIB_PATH)
    vp, ci, cf, cd, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_double, ctypes.c_size_t
    L.pasa_attn_fwd.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, cf, vp]
    L.pasa_attn_fwd.restype = ci
    L.pasa_attn_fwd_workspace.argtypes = [ci, ci, ci, ci, ci]
    L.pasa_attn_fwd_workspace.restype = sz
    L.pasa_attn_fwd_workspace_min.argtypes = [ci, ci, ci, ci]
    L.pasa_attn_fwd_workspace_min.restype = sz
    L.pasa_attn_fwd_ex.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, cf, ctypes.POINTER(pasa_opts), vp, sz, vp]
    L.pasa_attn_fwd_ex.restype = ci
    L.pasa_attn_fwd_static.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, cf, ctypes.POINTER(pasa_opts), vp]
    L.pasa_attn_fwd_static.restype = ci
    L.pasa_prepare_kv.argtypes = [vp, vp, ci, ci, ci, ci, cf, ctypes.POINTER(pasa_opts), vp, sz, vp]
    L.pasa_prepare_kv.restype = ci
    L.pasa_attn_fwd_prepared.argtypes = [vp, vp, ci, ci, ci, ci, ci, ci, cf, ctypes.POINTER(pasa_opts), vp, sz, vp]
    L.pasa_attn_fwd_prepared.restype = ci
    L.pasa_attn_fwd_adaptive.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, cf, ctypes.POINTER(pasa_opts), vp, sz, vp]
    L.pasa_attn_fwd_adaptive.restype = ci
    L.pasa_attn_fwd_chunk.argtypes = [vp, vp, ci, ci, ci, ci, ci, ci, ci, ci, cf, ctypes.POINTER(pasa_opts), vp, sz, vp]
    L.pasa_attn_fwd_chunk.restype = ci
    L.pasa_shift_keys.argtypes = [vp, vp, ci, ci, ci, ci, cd, cd, vp]
    L.pasa_shift_keys.restype = ci
    L.pasa_shift_keys_matrix.argtypes = [vp, vp, ci, ci, ci, ci, cd, cd, vp]
    L.pasa_shift_keys_matrix.restype = ci
    L.pasa_shift_keys_matrix_mfma.argtypes = [vp, vp, ci, ci, ci, ci, cd, cd, vp]
    L.pasa_shift_keys_matrix_mfma.restype = ci
    L.pasa_shift_keys_direct.argtypes = [vp, vp, vp, ci, ci, ci, ci, cd, cd, vp]
    L.pasa_shift_keys_direct.restype = ci
    L.pasa_optimal_beta.argtypes = [cd, ci, ci]
    L.pasa_optimal_beta.restype = cd
    L.pasa_invariance_rounded.argtypes = [cd, ci, ci]
    L.pasa_invariance_rounded.restype = cd
    L.pasa_status_string.argtypes = [ci]
    L.pasa_status_string.restype = ctypes.c_char_p
    L.pasa_version.argtypes = []
    L.pasa_version.restype = ci
    _lib = L
    return L


def _ptr(x):
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _stream(stream):
    if stream is None:
        return None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None     # torch.cuda.Stream


def _check(status: int, what: str, check: bool):
    if check and status != 0:
        raise PasaError(status, what)
    return status


def pasa_status_string(status: int) -> str:
    return lib().pasa_status_string(int(status)).decode()


def pasa_version() -> int:
    return lib().pasa_version()


def pasa_optimal_beta(beta0: float, n: int, tp: int = 0) -> float:
    return lib().pasa_optimal_beta(float(beta0), int(n), int(tp))


def pasa_invariance_rounded(beta: float, n: int, tp: int = 0) -> float:
    return lib().pasa_invariance_rounded(float(beta), int(n), int(tp))


def pasa_attn_fwd_workspace(B, Hq, Hkv, N, d) -> int:
    return lib().pasa_attn_fwd_workspace(B, Hq, Hkv, N, d)


def pasa_attn_fwd_workspace_min(B, Hkv, N, d) -> int:
    return lib().pasa_attn_fwd_workspace_min(B, Hkv, N, d)


def pasa_attn_fwd(q, k, v, o, B, Hq, Hkv, N, d, causal, scale, stream=None, check=True) -> int:
    st = lib().pasa_attn_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o), B, Hq, Hkv, N, d, int(causal), float(scale),
                             _stream(stream))
    return _check(st, "pasa_attn_fwd", check)


def pasa_attn_fwd_ex(q, k, v, o, B, Hq, Hkv, N, d, causal, scale, workspace, workspace_bytes, stream=None,
                     beta=-1.0, variant=MIXED, shift_tile=128, overflow_s=None, nonfinite_o=None,
                     shift_mode=SHIFT_MEAN, io_dtype=IO_F16, opts_null=False, check=True) -> int:
    opts = pasa_opts(float(beta), int(variant), int(shift_tile), _ptr(overflow_s), _ptr(nonfinite_o), int(shift_mode),
                     int(io_dtype))
    st = lib().pasa_attn_fwd_ex(_ptr(q), _ptr(k), _ptr(v), _ptr(o), B, Hq, Hkv, N, d, int(causal), float(scale),
                                None if opts_null else ctypes.byref(opts), _ptr(workspace), int(workspace_bytes),
                                _stream(stream))
    return _check(st, "pasa_attn_fwd_ex", check)


STATIC_WORKSPACE_BYTES = 33 << 20      # PASA_STATIC_WORKSPACE_BYTES of include/pasa.h


def pasa_attn_fwd_static(q, k, v, o, B, Hq, Hkv, N, d, causal, scale, stream=None,
                         beta=-1.0, variant=MIXED, shift_tile=128, overflow_s=None, nonfinite_o=None,
                         shift_mode=SHIFT_MEAN, io_dtype=IO_F16, opts_null=False, check=True) -> int:
    opts = pasa_opts(float(beta), int(variant), int(shift_tile), _ptr(overflow_s), _ptr(nonfinite_o), int(shift_mode),
                     int(io_dtype))
    st = lib().pasa_attn_fwd_static(_ptr(q), _ptr(k), _ptr(v), _ptr(o), B, Hq, Hkv, N, d, int(causal), float(scale),
                                    None if opts_null else ctypes.byref(opts), _stream(stream))
    return _check(st, "pasa_attn_fwd_static", check)


def pasa_prepare_kv(k, v, B, Hkv, N, d, scale, workspace, workspace_bytes, stream=None, beta=-1.0, variant=MIXED,
                    shift_tile=128, shift_mode=SHIFT_MEAN, io_dtype=IO_F16, check=True) -> int:
    opts = pasa_opts(float(beta), int(variant), int(shift_tile), None, None, int(shift_mode), int(io_dtype))
    st = lib().pasa_prepare_kv(_ptr(k), _ptr(v), B, Hkv, N, d, float(scale), ctypes.byref(opts), _ptr(workspace),
                               int(workspace_bytes), _stream(stream))
    return _check(st, "pasa_prepare_kv", check)


def pasa_attn_fwd_prepared(q, o, B, Hq, Hkv, N, d, causal, scale, workspace, workspace_bytes, stream=None,
                           beta=-1.0, variant=MIXED, shift_tile=128, overflow_s=None, nonfinite_o=None,
                           shift_mode=SHIFT_MEAN, io_dtype=IO_F16, check=True) -> int:
    opts = pasa_opts(float(beta), int(variant), int(shift_tile), _ptr(overflow_s), _ptr(nonfinite_o), int(shift_mode),
                     int(io_dtype))
    st = lib().pasa_attn_fwd_prepared(_ptr(q), _ptr(o), B, Hq, Hkv, N, d, int(causal), float(scale),
                                      ctypes.byref(opts), _ptr(workspace), int(workspace_bytes), _stream(stream))
    return _check(st, "pasa_attn_fwd_prepared", check)


def pasa_shift_keys(k, kprime, B, Hkv, N, d, beta, kscale, stream=None, check=True) -> int:
    st = lib().pasa_shift_keys(_ptr(k), _ptr(kprime), B, Hkv, N, d, float(beta), float(kscale), _stream(stream))
    return _check(st, "pasa_shift_keys", check)


def pasa_shift_keys_matrix(k, kprime, B, Hkv, N, d, beta, kscale, stream=None, check=True) -> int:
    st = lib().pasa_shift_keys_matrix(_ptr(k), _ptr(kprime), B, Hkv, N, d, float(beta), float(kscale),
                                      _stream(stream))
    return _check(st, "pasa_shift_keys_matrix", check)


def pasa_shift_keys_matrix_mfma(k, kprime, B, Hkv, N, d, beta, kscale, stream=None, check=True) -> int:
    st = lib().pasa_shift_keys_matrix_mfma(_ptr(k), _ptr(kprime), B, Hkv, N, d, float(beta), float(kscale),
                                           _stream(stream))
    return _check(st, "pasa_shift_keys_matrix_mfma", check)


def pasa_attn_fwd_chunk(q, o, B, Hq, Hkv, Nq, row0, N, d, causal, scale, workspace, workspace_bytes, stream=None,
                        beta=-1.0, variant=MIXED, shift_tile=128, overflow_s=None, nonfinite_o=None,
                        shift_mode=SHIFT_MEAN, io_dtype=IO_F16, check=True) -> int:
    opts = pasa_opts(float(beta), int(variant), int(shift_tile), _ptr(overflow_s), _ptr(nonfinite_o), int(shift_mode),
                     int(io_dtype))
    st = lib().pasa_attn_fwd_chunk(_ptr(q), _ptr(o), B, Hq, Hkv, Nq, row0, N, d, int(causal), float(scale),
                                   ctypes.byref(opts), _ptr(workspace), int(workspace_bytes), _stream(stream))
    return _check(st, "pasa_attn_fwd_chunk", check)


def pasa_shift_keys_direct(k, kprime, k0, B, Hkv, N, d, beta, kscale, stream=None, check=True) -> int:
    st = lib().pasa_shift_keys_direct(_ptr(k), _ptr(kprime), _ptr(k0), B, Hkv, N, d, float(beta), float(kscale),
                                      _stream(stream))
    return _check(st, "pasa_shift_keys_direct", check)


def pasa_attn_fwd_adaptive(q, k, v, o, B, Hq, Hkv, N, d, causal, scale, workspace, workspace_bytes, stream=None,
                           beta=-1.0, variant=MIXED, shift_tile=128, overflow_s=None, nonfinite_o=None,
                           shift_mode=SHIFT_MEAN, io_dtype=IO_F16, opts_null=False, check=True) -> int:
    opts = pasa_opts(float(beta), int(variant), int(shift_tile), _ptr(overflow_s), _ptr(nonfinite_o), int(shift_mode),
                     int(io_dtype))
    st = lib().pasa_attn_fwd_adaptive(_ptr(q), _ptr(k), _ptr(v), _ptr(o), B, Hq, Hkv, N, d, int(causal), float(scale),
                                      None if opts_null else ctypes.byref(opts), _ptr(workspace), int(workspace_bytes),
                                      _stream(stream))
    return _check(st, "pasa_attn_fwd_adaptive", check)
