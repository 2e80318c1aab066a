"""Thin ctypes binding of libmst_lmhead.so: argument marshalling only.

Every step of the path runs in the HIP kernels behind the C ABI declared in
include/mst_lmhead.h.  PyTorch appears here only as the owner of device memory
and of the stream.  There is no CPU fallback: if the library is missing the
import of this module's functions fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libmst_lmhead.so")

MST_OK = 0
PROFILE_KINDS = 9     # MST_PROFILE_KINDS of include/mst_lmhead.h (checked against the library by the tests)

_lib = None


class MstError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"mst status {status}: {text}")
        self.status = status


def load_library() -> ctypes.CDLL:
    """Load the in-tree shared library (built by paper_2407_15892_amd.build.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it first (python -m paper_2407_15892_amd.build); "
            "there is no fallback path")
    # One HIP runtime per process: PyTorch ships its own libamdhip64 and owns the device
    # memory we are handed, so make sure that copy is loaded (and globally visible) before
    # our library's dependency on the same soname is resolved.
    import torch
    torch_hip = os.path.join(os.path.dirname(torch.__file__), "lib", "libamdhip64.so")
    if os.path.exists(torch_hip):
        ctypes.CDLL(torch_hip, mode=ctypes.RTLD_GLOBAL)
    lib = ctypes.CDLL(LIB_PATH)
    c = ctypes
    lib.mst_strerror.restype = c.c_char_p
    lib.mst_strerror.argtypes = [c.c_int]
    lib.mst_version.restype = c.c_char_p
    lib.mst_version.argtypes = []
    lib.mst_workspace_bytes.restype = c.c_int
    lib.mst_workspace_bytes.argtypes = [c.c_int64, c.c_int64, c.c_int64, c.c_int32,
                                        c.POINTER(c.c_size_t), c.POINTER(c.c_size_t)]
    lib.mst_suggest_m.restype = c.c_int32
    lib.mst_suggest_m.argtypes = [c.c_int64, c.c_int64, c.c_int64]
    lib.mst_mfma_probe.restype = c.c_int
    lib.mst_mfma_probe.argtypes = [c.c_int32, c.c_int32, c.c_float, c.c_void_p, c.c_void_p]
    lib.mst_shift_labels.restype = c.c_int
    lib.mst_shift_labels.argtypes = [c.c_void_p, c.c_int64, c.c_int64, c.c_int32, c.c_void_p, c.c_void_p]
    lib.mst_lmhead_ce_fwd.restype = c.c_int
    lib.mst_lmhead_ce_fwd.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_int64, c.c_int64, c.c_int64,
                                      c.c_int32, c.c_int32, c.c_void_p, c.c_size_t,
                                      c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p]
    lib.mst_lmhead_ce_fwd_static.restype = c.c_int
    lib.mst_lmhead_ce_fwd_static.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_int64, c.c_int64, c.c_int64,
                                             c.c_int32, c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p]
    lib.mst_lmhead_ce_bwd.restype = c.c_int
    lib.mst_lmhead_ce_bwd.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_int64, c.c_int64, c.c_int64,
                                      c.c_int32, c.c_int32, c.c_float, c.c_void_p, c.c_void_p,
                                      c.c_void_p, c.c_size_t, c.c_void_p, c.c_void_p, c.c_void_p]
    lib.mst_set_bwd_schedule.restype = c.c_int
    lib.mst_set_bwd_schedule.argtypes = [c.c_int32]
    lib.mst_bwd_schedule_info.restype = c.c_int
    lib.mst_bwd_schedule_info.argtypes = [c.c_int64, c.c_int64, c.c_int64, c.c_int32, c.POINTER(c.c_int64)]
    lib.mst_bwd_schedule_info_for.restype = c.c_int
    lib.mst_bwd_schedule_info_for.argtypes = [c.c_int64, c.c_int64, c.c_int64, c.c_int32, c.c_int32,
                                              c.POINTER(c.c_int64)]
    lib.mst_profile_enable.restype = c.c_int
    lib.mst_profile_enable.argtypes = [c.c_int]
    lib.mst_profile_collect.restype = c.c_int
    lib.mst_profile_collect.argtypes = [c.POINTER(c.c_double), c.POINTER(c.c_int64), c.POINTER(c.c_int64)]
    lib.mst_profile_kind_name.restype = c.c_char_p
    lib.mst_profile_kind_name.argtypes = [c.c_int]
    _lib = lib
    return lib


def _check(status: int) -> None:
    if status != MST_OK:
        raise MstError(status, load_library().mst_strerror(status).decode())


def mst_strerror(status: int) -> str:
    return load_library().mst_strerror(status).decode()


def mst_version() -> str:
    return load_library().mst_version().decode()


def mst_workspace_bytes(S: int, d: int, V: int, M: int):
    """(fwd_bytes, bwd_bytes) as the C call reports them."""
    f, b = ctypes.c_size_t(0), ctypes.c_size_t(0)
    _check(load_library().mst_workspace_bytes(S, d, V, M, ctypes.byref(f), ctypes.byref(b)))
    return int(f.value), int(b.value)


def mst_suggest_m(S: int, d: int, V: int) -> int:
    """Chunk count advised by the paper's M = V / d rule, kept to chunks of at least 256 rows."""
    return int(load_library().mst_suggest_m(S, d, V))


def mst_mfma_probe(blocks: int, iters: int, scale: float, sink, stream=None) -> float:
    """Enqueue the register-resident MFMA loop; returns the flop it executes (time it with events)."""
    _check(load_library().mst_mfma_probe(blocks, iters, float(scale), _ptr(sink), _stream_handle(stream)))
    return float(blocks) * 8 * iters * 16 * 32768.0


def mst_shift_labels(labels_in, B: int, L: int, ignore_index: int, labels_out, stream=None) -> None:
    """Enqueue the next-token alignment: labels_out[b, t] = labels_in[b, t + 1], ignore_index at t = L - 1.
    Both int32 device tensors of B * L elements."""
    _check(load_library().mst_shift_labels(_ptr(labels_in), B, L, ignore_index, _ptr(labels_out),
                                           _stream_handle(stream)))


def mst_workspace_bytes_status(S: int, d: int, V: int, M: int) -> int:
    f, b = ctypes.c_size_t(0), ctypes.c_size_t(0)
    return int(load_library().mst_workspace_bytes(S, d, V, M, ctypes.byref(f), ctypes.byref(b)))


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream_handle(stream) -> Optional[int]:
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def mst_lmhead_ce_fwd(H, W, labels, ignore_index: int, M: int, workspace, loss, lse=None, n_valid=None,
                      stream=None) -> None:
    """Enqueue the forward pass.  H bf16 [S,d], W bf16 [V,d], labels int32 [S]; loss fp32 [1],
    lse fp32 [S] or None, n_valid int64 [1] or None; workspace: a uint8 device tensor."""
    S, d = H.shape
    V = W.shape[0]
    _check(load_library().mst_lmhead_ce_fwd(
        _ptr(H), _ptr(W), _ptr(labels), S, d, V, ignore_index, M,
        _ptr(workspace), workspace.numel() * workspace.element_size(),
        _ptr(loss), _ptr(lse), _ptr(n_valid), _stream_handle(stream)))


STATIC_SCRATCH_BYTES = 32 * 1024 * 1024     # MST_STATIC_SCRATCH_BYTES of include/mst_lmhead.h


def mst_lmhead_ce_fwd_static(H, W, labels, ignore_index: int, M: int, loss, lse=None, n_valid=None,
                             stream=None) -> None:
    """Enqueue the forward pass on the library's static device scratch (no workspace argument, no allocation)."""
    S, d = H.shape
    V = W.shape[0]
    _check(load_library().mst_lmhead_ce_fwd_static(
        _ptr(H), _ptr(W), _ptr(labels), S, d, V, ignore_index, M,
        _ptr(loss), _ptr(lse), _ptr(n_valid), _stream_handle(stream)))


def mst_lmhead_ce_bwd(H, W, labels, ignore_index: int, M: int, grad_loss: float, lse, n_valid, workspace, dH, dW,
                      stream=None) -> None:
    """Enqueue the backward pass.  lse fp32 [S] and n_valid int64 [1] come from the forward call (either may
    be None).  dH bf16 [S,d] and dW fp32 [V,d] are fully overwritten."""
    S, d = H.shape
    V = W.shape[0]
    _check(load_library().mst_lmhead_ce_bwd(
        _ptr(H), _ptr(W), _ptr(labels), S, d, V, ignore_index, M, float(grad_loss), _ptr(lse), _ptr(n_valid),
        _ptr(workspace), workspace.numel() * workspace.element_size(),
        _ptr(dH), _ptr(dW), _stream_handle(stream)))


BWD_SCHEDULE_AUTO, BWD_SCHEDULE_PAIRS, BWD_SCHEDULE_BLOCKS, BWD_SCHEDULE_BLOCKS_FUSED = 0, 1, 2, 3


def mst_set_bwd_schedule(schedule: int) -> None:
    _check(load_library().mst_set_bwd_schedule(int(schedule)))


def mst_bwd_schedule_info(S: int, d: int, V: int, M: int, schedule: Optional[int] = None) -> dict:
    """What the backward call would run: under the calling thread's override, or (schedule given) under that
    override without touching any state."""
    info = (ctypes.c_int64 * 8)()
    if schedule is None:
        _check(load_library().mst_bwd_schedule_info(S, d, V, M, info))
    else:
        _check(load_library().mst_bwd_schedule_info_for(S, d, V, M, int(schedule), info))
    keys = ("schedule", "rows_per_block", "row_blocks", "vocab_per_window", "windows", "dh_split",
            "est_pairs_us", "est_blocks_us")
    return dict(zip(keys, (int(x) for x in info)))


def mst_profile_enable(every) -> None:
    """0 / False: off; n >= 1 (True = 1): bracket every n-th launch of each kernel kind with events."""
    _check(load_library().mst_profile_enable(int(every)))


def mst_profile_collect():
    """{kernel kind name: (milliseconds of the timed launches, timed launches, all launches)} since the last collect."""
    ms = (ctypes.c_double * PROFILE_KINDS)()
    n = (ctypes.c_int64 * PROFILE_KINDS)()
    issued = (ctypes.c_int64 * PROFILE_KINDS)()
    _check(load_library().mst_profile_collect(ms, n, issued))
    lib = load_library()
    return {lib.mst_profile_kind_name(i).decode(): (float(ms[i]), int(n[i]), int(issued[i])) for i in range(PROFILE_KINDS)}
