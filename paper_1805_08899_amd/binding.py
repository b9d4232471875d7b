"""ctypes binding of libechoattn: same names as include/echoattn.h, include/echodropout.h and
include/echolstm.h, argument marshalling only.  Device buffers are passed as torch tensors (their
data_ptr() is taken) or as integer addresses; nothing is computed here.

The shared library must have been built (python -m paper_1805_08899_amd.build);
loading fails loudly otherwise -- there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, c_char_p, c_float, c_int, c_int32, c_size_t, c_void_p

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libechoattn.so")

ECHO_OK, ECHO_ERR_NULL, ECHO_ERR_SHAPE, ECHO_ERR_DTYPE, ECHO_ERR_WORKSPACE, ECHO_ERR_ALIGN, ECHO_ERR_HIP = range(7)
ECHO_F32, ECHO_BF16 = 0, 1
ECHO_ATTN_MAX_TK, ECHO_ATTN_STEP_MAX_TK, ECHO_ATTN_MAX_B = 2048, 8192, 65535
DTYPES = {"f32": ECHO_F32, "bf16": ECHO_BF16}


class echo_attn_desc_t(ctypes.Structure):
    _fields_ = [("B", c_int32), ("Tq", c_int32), ("Tk", c_int32), ("H", c_int32), ("Dv", c_int32),
                ("in_dtype", c_int32)]


class EchoError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        detail = echo_last_error_detail() if status == ECHO_ERR_HIP else ""
        super().__init__(f"{where}: {echo_status_string(status)} (status {status}) {detail}")


EXPORTS = {
    # name: (restype, argtypes)
    "echo_attn_fwd_workspace_bytes": (c_size_t, [POINTER(echo_attn_desc_t)]),
    "echo_attn_bwd_workspace_bytes": (c_size_t, [POINTER(echo_attn_desc_t)]),
    "echo_attn_stash_bytes": (c_size_t, [POINTER(echo_attn_desc_t)]),
    "echo_attn_fwd_stash_workspace_bytes": (c_size_t, [POINTER(echo_attn_desc_t)]),
    "echo_attn_fwd": (c_int, [POINTER(echo_attn_desc_t)] + [c_void_p] * 8 + [c_size_t, c_void_p]),
    "echo_attn_bwd": (c_int, [POINTER(echo_attn_desc_t)] + [c_void_p] * 12 + [c_size_t, c_void_p]),
    "echo_attn_bwd_static": (c_int, [POINTER(echo_attn_desc_t)] + [c_void_p] * 12),
    "echo_attn_bwd_accumulate": (c_int, [POINTER(echo_attn_desc_t)] + [c_void_p] * 12 + [c_size_t, c_void_p]),
    "echo_attn_step_fwd": (c_int, [POINTER(echo_attn_desc_t)] + [c_void_p] * 8),
    "echo_attn_step_bwd": (c_int, [POINTER(echo_attn_desc_t)] + [c_void_p] * 12),
    "echo_attn_step_finish": (c_int, [POINTER(echo_attn_desc_t)] + [c_void_p] * 3),
    "echo_attn_steps_ds_bytes": (c_size_t, [POINTER(echo_attn_desc_t)]),
    "echo_attn_step_bwd_query": (c_int, [POINTER(echo_attn_desc_t), c_int32, c_int32] + [c_void_p] * 10),
    "echo_attn_steps_bwd_keys": (c_int, [POINTER(echo_attn_desc_t)] + [c_void_p] * 11 + [c_size_t, c_void_p]),
    "echo_attn_fwd_stash": (c_int, [POINTER(echo_attn_desc_t)] + [c_void_p] * 9 + [c_size_t, c_void_p]),
    "echo_attn_bwd_stash": (c_int, [POINTER(echo_attn_desc_t)] + [c_void_p] * 11 + [c_size_t, c_void_p]),
    "echo_attn_profile_enable": (None, [c_int]),
    "echo_attn_profile_read": (c_int, [POINTER(c_char_p), POINTER(c_int), POINTER(c_float), c_int]),
    "echo_attn_calibrate": (c_int, [c_int, c_int, c_int, c_void_p, c_void_p, c_size_t, POINTER(ctypes.c_double),
                                    c_void_p]),
    "echo_dropout_mask_words": (c_size_t, [c_size_t]),
    "echo_dropout_fwd": (c_int, [c_void_p, c_size_t, c_float, ctypes.c_uint64, ctypes.c_uint64, c_void_p, c_void_p,
                                 c_void_p]),
    "echo_dropout_bwd": (c_int, [c_void_p, c_void_p, c_size_t, c_float, c_void_p, c_void_p]),
    "echo_lstm_cell_fwd": (c_int, [ctypes.c_int64, ctypes.c_int64] + [c_void_p] * 7),
    "echo_lstm_cell_bwd": (c_int, [ctypes.c_int64, ctypes.c_int64] + [c_void_p] * 7),
    "echo_lstm_cell_fwd_stash": (c_int, [ctypes.c_int64, ctypes.c_int64] + [c_void_p] * 8),
    "echo_lstm_cell_bwd_stash": (c_int, [ctypes.c_int64, ctypes.c_int64] + [c_void_p] * 8),
    "echo_lstm_cell_kept_bytes": (c_size_t, [ctypes.c_int64, ctypes.c_int64, c_int]),
    "echo_status_string": (c_char_p, [c_int]),
    "echo_last_error_detail": (c_char_p, []),
    "echo_version": (c_char_p, []),
}

_lib = None


def lib() -> ctypes.CDLL:
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_1805_08899_amd.build` "
                "(there is no fallback implementation)")
        try:
            # The process must end up with ONE HIP runtime.  PyTorch ships its own copy; if this library is
            # loaded first it pulls in the system's copy and PyTorch then finds no device.  Loading PyTorch first
            # makes both use PyTorch's.
            import torch  # noqa: F401
        except ImportError:
            pass
        L = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in EXPORTS.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


def _ptr(x):
    """Device address of a torch tensor (must be contiguous), an int, or None."""
    if x is None:
        return None
    if isinstance(x, int):
        return c_void_p(x)
    if not x.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return c_void_p(x.data_ptr())


def _stream(stream):
    if stream is None:
        return None
    return c_void_p(stream if isinstance(stream, int) else stream.cuda_stream)


def make_desc(B, Tq, Tk, H, Dv, in_dtype="f32") -> echo_attn_desc_t:
    code = DTYPES[in_dtype] if isinstance(in_dtype, str) else int(in_dtype)
    return echo_attn_desc_t(B, Tq, Tk, H, Dv, code)


def echo_attn_fwd_workspace_bytes(desc) -> int:
    return lib().echo_attn_fwd_workspace_bytes(ctypes.byref(desc))


def echo_attn_bwd_workspace_bytes(desc) -> int:
    return lib().echo_attn_bwd_workspace_bytes(ctypes.byref(desc))


def echo_attn_fwd_stash_workspace_bytes(desc) -> int:
    return lib().echo_attn_fwd_stash_workspace_bytes(ctypes.byref(desc))


def echo_attn_stash_bytes(desc) -> int:
    return lib().echo_attn_stash_bytes(ctypes.byref(desc))


def _ws_bytes(workspace, workspace_bytes):
    if workspace_bytes is not None:
        return workspace_bytes
    if workspace is None or isinstance(workspace, int):
        return 0
    return workspace.numel() * workspace.element_size()


def echo_attn_fwd(desc, Qp, Kp, V, v, key_len, context, P, workspace, workspace_bytes=None, stream=None) -> int:
    return lib().echo_attn_fwd(ctypes.byref(desc), _ptr(Qp), _ptr(Kp), _ptr(V), _ptr(v), _ptr(key_len),
                               _ptr(context), _ptr(P), _ptr(workspace), _ws_bytes(workspace, workspace_bytes),
                               _stream(stream))


def echo_attn_bwd(desc, dContext, P, Qp, Kp, V, v, key_len, dQp, dKp, dV, dv, workspace, workspace_bytes=None,
                  stream=None) -> int:
    return lib().echo_attn_bwd(ctypes.byref(desc), _ptr(dContext), _ptr(P), _ptr(Qp), _ptr(Kp), _ptr(V), _ptr(v),
                               _ptr(key_len), _ptr(dQp), _ptr(dKp), _ptr(dV), _ptr(dv), _ptr(workspace),
                               _ws_bytes(workspace, workspace_bytes), _stream(stream))


ECHO_ATTN_STATIC_SCRATCH_BYTES = 16 << 20


def echo_attn_bwd_static(desc, dContext, P, Qp, Kp, V, v, key_len, dQp, dKp, dV, dv, stream=None) -> int:
    return lib().echo_attn_bwd_static(ctypes.byref(desc), _ptr(dContext), _ptr(P), _ptr(Qp), _ptr(Kp), _ptr(V),
                                      _ptr(v), _ptr(key_len), _ptr(dQp), _ptr(dKp), _ptr(dV), _ptr(dv),
                                      _stream(stream))


def echo_attn_bwd_accumulate(desc, dContext, P, Qp, Kp, V, v, key_len, dQp, dKp, dV, dv, workspace,
                             workspace_bytes=None, stream=None) -> int:
    return lib().echo_attn_bwd_accumulate(ctypes.byref(desc), _ptr(dContext), _ptr(P), _ptr(Qp), _ptr(Kp), _ptr(V),
                                          _ptr(v), _ptr(key_len), _ptr(dQp), _ptr(dKp), _ptr(dV), _ptr(dv),
                                          _ptr(workspace), _ws_bytes(workspace, workspace_bytes), _stream(stream))


def echo_attn_step_fwd(desc, Qp, Kp, V, v, key_len, context, P, stream=None) -> int:
    return lib().echo_attn_step_fwd(ctypes.byref(desc), _ptr(Qp), _ptr(Kp), _ptr(V), _ptr(v), _ptr(key_len),
                                    _ptr(context), _ptr(P), _stream(stream))


def echo_attn_step_bwd(desc, dContext, P, Qp, Kp, V, v, key_len, dQp, dKp, dV, dv_part, stream=None) -> int:
    return lib().echo_attn_step_bwd(ctypes.byref(desc), _ptr(dContext), _ptr(P), _ptr(Qp), _ptr(Kp), _ptr(V), _ptr(v),
                                    _ptr(key_len), _ptr(dQp), _ptr(dKp), _ptr(dV), _ptr(dv_part), _stream(stream))


def echo_attn_step_finish(desc, dv_part, dv, stream=None) -> int:
    return lib().echo_attn_step_finish(ctypes.byref(desc), _ptr(dv_part), _ptr(dv), _stream(stream))


def echo_attn_steps_ds_bytes(desc) -> int:
    return lib().echo_attn_steps_ds_bytes(ctypes.byref(desc))


def echo_attn_step_bwd_query(desc, step, steps, dContext, P, Qp, Kp, V, v, key_len, dQp, ds_rows, stream=None) -> int:
    return lib().echo_attn_step_bwd_query(ctypes.byref(desc), step, steps, _ptr(dContext), _ptr(P), _ptr(Qp), _ptr(Kp),
                                          _ptr(V), _ptr(v), _ptr(key_len), _ptr(dQp), _ptr(ds_rows), _stream(stream))


def echo_attn_steps_bwd_keys(desc, dContext, P, Qp, Kp, v, key_len, ds_rows, dKp, dV, dv, workspace,
                             workspace_bytes=None, stream=None) -> int:
    return lib().echo_attn_steps_bwd_keys(ctypes.byref(desc), _ptr(dContext), _ptr(P), _ptr(Qp), _ptr(Kp), _ptr(v),
                                          _ptr(key_len), _ptr(ds_rows), _ptr(dKp), _ptr(dV), _ptr(dv), _ptr(workspace),
                                          _ws_bytes(workspace, workspace_bytes), _stream(stream))


def echo_attn_fwd_stash(desc, Qp, Kp, V, v, key_len, context, P, tanh_map, workspace, workspace_bytes=None,
                        stream=None) -> int:
    return lib().echo_attn_fwd_stash(ctypes.byref(desc), _ptr(Qp), _ptr(Kp), _ptr(V), _ptr(v), _ptr(key_len),
                                     _ptr(context), _ptr(P), _ptr(tanh_map), _ptr(workspace),
                                     _ws_bytes(workspace, workspace_bytes), _stream(stream))


def echo_attn_bwd_stash(desc, dContext, P, tanh_map, V, v, key_len, dQp, dKp, dV, dv, workspace,
                        workspace_bytes=None, stream=None) -> int:
    return lib().echo_attn_bwd_stash(ctypes.byref(desc), _ptr(dContext), _ptr(P), _ptr(tanh_map), _ptr(V), _ptr(v),
                                     _ptr(key_len), _ptr(dQp), _ptr(dKp), _ptr(dV), _ptr(dv), _ptr(workspace),
                                     _ws_bytes(workspace, workspace_bytes), _stream(stream))


def echo_attn_profile_enable(on: bool) -> None:
    lib().echo_attn_profile_enable(1 if on else 0)


def echo_attn_profile_read(cap: int = 32):
    """{kernel name: (launches, total_ms)} since the last read."""
    names = (c_char_p * cap)()
    launches = (c_int * cap)()
    ms = (c_float * cap)()
    n = min(lib().echo_attn_profile_read(names, launches, ms, cap), cap)
    return {names[i].decode(): (launches[i], ms[i]) for i in range(n)}


ECHO_CAL_FMA, ECHO_CAL_RCP, ECHO_CAL_EXP2, ECHO_CAL_FWD_MIX, ECHO_CAL_BWD_MIX, ECHO_CAL_COPY = range(6)


def echo_attn_calibrate(kind, blocks, iters, src, dst, nbytes, stream=None):
    """Returns (status, work) -- see the header for the meaning of `work`."""
    work = ctypes.c_double(0.0)
    st = lib().echo_attn_calibrate(kind, blocks, iters, _ptr(src), _ptr(dst), nbytes, ctypes.byref(work),
                                   _stream(stream))
    return st, work.value


def echo_dropout_mask_words(n: int) -> int:
    return lib().echo_dropout_mask_words(n)


def echo_dropout_fwd(x, n, p, seed, offset, y, mask_bits, stream=None) -> int:
    return lib().echo_dropout_fwd(_ptr(x), n, p, seed, offset, _ptr(y), _ptr(mask_bits), _stream(stream))


def echo_dropout_bwd(dy, mask_bits, n, p, dx, stream=None) -> int:
    return lib().echo_dropout_bwd(_ptr(dy), _ptr(mask_bits), n, p, _ptr(dx), _stream(stream))


def echo_lstm_cell_fwd(B, H, Gx, Gh, c_prev, h, c, a, stream=None) -> int:
    return lib().echo_lstm_cell_fwd(B, H, _ptr(Gx), _ptr(Gh), _ptr(c_prev), _ptr(h), _ptr(c), _ptr(a),
                                    _stream(stream))


def echo_lstm_cell_bwd(B, H, dh, dc, a, c_prev, da, dc_prev, stream=None) -> int:
    return lib().echo_lstm_cell_bwd(B, H, _ptr(dh), _ptr(dc), _ptr(a), _ptr(c_prev), _ptr(da), _ptr(dc_prev),
                                    _stream(stream))


def echo_lstm_cell_fwd_stash(B, H, Gx, Gh, c_prev, h, c, acts, tanh_c, stream=None) -> int:
    return lib().echo_lstm_cell_fwd_stash(B, H, _ptr(Gx), _ptr(Gh), _ptr(c_prev), _ptr(h), _ptr(c), _ptr(acts),
                                          _ptr(tanh_c), _stream(stream))


def echo_lstm_cell_bwd_stash(B, H, dh, dc, acts, tanh_c, c_prev, da, dc_prev, stream=None) -> int:
    return lib().echo_lstm_cell_bwd_stash(B, H, _ptr(dh), _ptr(dc), _ptr(acts), _ptr(tanh_c), _ptr(c_prev),
                                          _ptr(da), _ptr(dc_prev), _stream(stream))


def echo_lstm_cell_kept_bytes(B: int, H: int, stash: bool) -> int:
    return lib().echo_lstm_cell_kept_bytes(B, H, 1 if stash else 0)


def echo_status_string(status: int) -> str:
    return lib().echo_status_string(int(status)).decode()


def echo_last_error_detail() -> str:
    return lib().echo_last_error_detail().decode()


def echo_version() -> str:
    return lib().echo_version().decode()


def check(status: int, where: str = "libechoattn") -> None:
    if status != ECHO_OK:
        raise EchoError(status, where)
