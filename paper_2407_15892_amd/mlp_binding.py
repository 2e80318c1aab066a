"""Thin ctypes binding of libmst_mlp.so: argument marshalling only.

Every step of the MLP path runs in the HIP kernels behind the C ABI declared in
include/mst_mlp.h.  PyTorch appears here only as the owner of device memory and
of the stream.  There is no CPU fallback: without the built library the calls
fail loudly.
"""
from __future__ import annotations

import ctypes
import os

from .binding import MST_OK, MstError, _ptr, _stream_handle
from .binding import load_library as _load_lmhead_library

HERE = os.path.dirname(os.path.abspath(__file__))
MLP_LIB_PATH = os.path.join(HERE, "libmst_mlp.so")

MLP_PROFILE_KINDS = 6

_lib = None


def load_mlp_library() -> ctypes.CDLL:
    """Load the in-tree MLP library (built by paper_2407_15892_amd.build.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(MLP_LIB_PATH):
        raise RuntimeError(
            f"{MLP_LIB_PATH} is missing: build it first (python -m paper_2407_15892_amd.build); "
            "there is no fallback path")
    _load_lmhead_library()      # loads PyTorch's HIP runtime globally first; also provides mst_strerror
    lib = ctypes.CDLL(MLP_LIB_PATH)
    c = ctypes
    lib.mst_mlp_version.restype = c.c_char_p
    lib.mst_mlp_version.argtypes = []
    lib.mst_mlp_workspace_bytes.restype = c.c_int
    lib.mst_mlp_workspace_bytes.argtypes = [c.c_int64, c.c_int64, c.c_int64, c.c_int32,
                                            c.POINTER(c.c_size_t), c.POINTER(c.c_size_t)]
    lib.mst_mlp_suggest_m.restype = c.c_int32
    lib.mst_mlp_suggest_m.argtypes = [c.c_int64, c.c_int64, c.c_int64]
    lib.mst_mlp_fwd.restype = c.c_int
    lib.mst_mlp_fwd.argtypes = [c.c_void_p] * 4 + [c.c_int64, c.c_int64, c.c_int64, c.c_int32,
                                                   c.c_void_p, c.c_size_t, c.c_void_p, c.c_void_p]
    lib.mst_mlp_bwd.restype = c.c_int
    lib.mst_mlp_bwd.argtypes = [c.c_void_p] * 5 + [c.c_int64, c.c_int64, c.c_int64, c.c_int32,
                                                   c.c_void_p, c.c_size_t] + [c.c_void_p] * 5
    lib.mst_mlp_profile_enable.restype = c.c_int
    lib.mst_mlp_profile_enable.argtypes = [c.c_int]
    lib.mst_mlp_profile_collect.restype = c.c_int
    lib.mst_mlp_profile_collect.argtypes = [c.POINTER(c.c_double), c.POINTER(c.c_int64), c.POINTER(c.c_int64)]
    lib.mst_mlp_profile_kind_name.restype = c.c_char_p
    lib.mst_mlp_profile_kind_name.argtypes = [c.c_int]
    _lib = lib
    return lib


def _check(status: int) -> None:
    if status != MST_OK:
        raise MstError(status, _load_lmhead_library().mst_strerror(status).decode())


def mst_mlp_version() -> str:
    return load_mlp_library().mst_mlp_version().decode()


def mst_mlp_workspace_bytes(S: int, d: int, I: int, M: int):
    """(fwd_bytes, bwd_bytes) as the C call reports them."""
    f, b = ctypes.c_size_t(0), ctypes.c_size_t(0)
    _check(load_mlp_library().mst_mlp_workspace_bytes(S, d, I, M, ctypes.byref(f), ctypes.byref(b)))
    return int(f.value), int(b.value)


def mst_mlp_workspace_bytes_status(S: int, d: int, I: int, M: int) -> int:
    f, b = ctypes.c_size_t(0), ctypes.c_size_t(0)
    return int(load_mlp_library().mst_mlp_workspace_bytes(S, d, I, M, ctypes.byref(f), ctypes.byref(b)))


def mst_mlp_suggest_m(S: int, d: int, I: int) -> int:
    """Chunk count of the paper's constant chunk size C = d."""
    return int(load_mlp_library().mst_mlp_suggest_m(S, d, I))


def mst_mlp_fwd(X, Wg, Wu, Wd, M: int, workspace, O, stream=None) -> None:
    """Enqueue the forward pass.  X bf16 [S,d], Wg/Wu bf16 [I,d], Wd bf16 [d,I]; O bf16 [S,d] is overwritten."""
    S, d = X.shape
    I = Wg.shape[0]
    _check(load_mlp_library().mst_mlp_fwd(
        _ptr(X), _ptr(Wg), _ptr(Wu), _ptr(Wd), S, d, I, M,
        _ptr(workspace), workspace.numel() * workspace.element_size(), _ptr(O), _stream_handle(stream)))


def mst_mlp_bwd(X, Wg, Wu, Wd, dO, M: int, workspace, dX, dWg, dWu, dWd, stream=None) -> None:
    """Enqueue the backward pass.  dX bf16 [S,d]; dWg, dWu fp32 [I,d]; dWd fp32 [d,I]; all fully overwritten."""
    S, d = X.shape
    I = Wg.shape[0]
    _check(load_mlp_library().mst_mlp_bwd(
        _ptr(X), _ptr(Wg), _ptr(Wu), _ptr(Wd), _ptr(dO), S, d, I, M,
        _ptr(workspace), workspace.numel() * workspace.element_size(),
        _ptr(dX), _ptr(dWg), _ptr(dWu), _ptr(dWd), _stream_handle(stream)))


def mst_mlp_profile_enable(every) -> None:
    """0 / False: off; n >= 1 (True = 1): bracket every n-th launch of each kernel kind with events."""
    _check(load_mlp_library().mst_mlp_profile_enable(int(every)))


def mst_mlp_profile_collect():
    """{kind name: (ms of the timed launches, timed launches, all launches)} since the last collect."""
    ms = (ctypes.c_double * MLP_PROFILE_KINDS)()
    n = (ctypes.c_int64 * MLP_PROFILE_KINDS)()
    issued = (ctypes.c_int64 * MLP_PROFILE_KINDS)()
    _check(load_mlp_library().mst_mlp_profile_collect(ms, n, issued))
    lib = load_mlp_library()
    return {lib.mst_mlp_profile_kind_name(i).decode(): (float(ms[i]), int(n[i]), int(issued[i])) for i in range(MLP_PROFILE_KINDS)}
