"""ctypes binding of libmosaic_bsa.so: argument marshalling only.

Every function here has the name and the argument order of the C entry point
it forwards to (include/mosaic_bsa.h).  Tensors are torch tensors that own
device memory; torch supplies the current HIP stream.  Nothing is computed in
Python and there is no fallback: if the library has not been built, loading
fails with an error.
"""
from __future__ import annotations

import ctypes
import dataclasses
import os

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(PKG_DIR, "libmosaic_bsa.so")
_lib = None

F32, BF16 = 0, 1
OP_SELECT, OP_FWD, OP_BWD = 0, 1, 2


class BsaError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"mosaic_bsa error {code}: {text}")
        self.code = code


class _CParams(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("heads", ctypes.c_int32),
                ("grid_h", ctypes.c_int32), ("grid_w", ctypes.c_int32),
                ("block_h", ctypes.c_int32), ("block_w", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("n_select", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("softmax_scale", ctypes.c_float),
                ("kv_heads", ctypes.c_int32)]


@dataclasses.dataclass
class Params:
    """Mirror of the C struct mosaic_bsa_params."""
    batch: int
    heads: int
    grid_h: int
    grid_w: int
    block_h: int
    block_w: int
    head_dim: int
    n_select: int
    dtype: int = BF16
    softmax_scale: float = 0.0
    kv_heads: int = 0

    def c_struct(self) -> _CParams:
        return _CParams(self.batch, self.heads, self.grid_h, self.grid_w,
                        self.block_h, self.block_w, self.head_dim,
                        self.n_select, self.dtype, self.softmax_scale, self.kv_heads)

    @property
    def n_tokens(self) -> int:
        return self.grid_h * self.grid_w

    @property
    def block_tokens(self) -> int:
        return self.block_h * self.block_w

    @property
    def n_blocks(self) -> int:
        return self.n_tokens // self.block_tokens


def library_path() -> str:
    return _LIB_PATH


def load_library() -> ctypes.CDLL:
    """Load the built library; raises if it is missing (no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(
                f"{_LIB_PATH} is not built; run `python -m paper_2604_16429_amd.build`")
        lib = ctypes.CDLL(_LIB_PATH)
        vp, sz, i32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
        pp = ctypes.POINTER(_CParams)
        lib.mosaic_bsa_workspace_bytes.restype = sz
        lib.mosaic_bsa_workspace_bytes.argtypes = [pp, i32]
        lib.mosaic_bsa_select.restype = i32
        lib.mosaic_bsa_select.argtypes = [pp, vp, vp, vp, vp, sz, vp]
        lib.mosaic_bsa_select_static.restype = i32
        lib.mosaic_bsa_select_static.argtypes = [pp, vp, vp, vp, vp]
        lib.mosaic_bsa_fwd.restype = i32
        lib.mosaic_bsa_fwd.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.mosaic_bsa_bwd.restype = i32
        lib.mosaic_bsa_bwd.argtypes = [pp] + [vp] * 10 + [vp, sz, vp]
        lib.mosaic_bsa_three_branch_workspace_bytes.restype = sz
        lib.mosaic_bsa_three_branch_workspace_bytes.argtypes = [pp, ctypes.c_int32, ctypes.c_int32]
        lib.mosaic_bsa_fwd_three_branch.restype = i32
        lib.mosaic_bsa_fwd_three_branch.argtypes = (
            [pp, ctypes.c_int32, ctypes.c_int32] + [vp] * 7 + [sz, vp])
        lib.mosaic_bsa_three_branch_bwd_workspace_bytes.restype = sz
        lib.mosaic_bsa_three_branch_bwd_workspace_bytes.argtypes = [
            pp, ctypes.c_int32, ctypes.c_int32]
        lib.mosaic_bsa_bwd_three_branch.restype = i32
        lib.mosaic_bsa_bwd_three_branch.argtypes = (
            [pp, ctypes.c_int32, ctypes.c_int32] + [vp] * 12 + [sz, vp])
        lib.mosaic_bsa_check_selection.restype = i32
        lib.mosaic_bsa_check_selection.argtypes = [pp, vp, ctypes.c_int32, vp, vp]
        lib.mosaic_bsa_probe_mfma.restype = i32
        lib.mosaic_bsa_probe_mfma.argtypes = [vp, ctypes.c_int32, ctypes.c_int32, vp]
        lib.mosaic_bsa_strerror.restype = ctypes.c_char_p
        lib.mosaic_bsa_strerror.argtypes = [i32]
        _lib = lib
    return _lib


def _ptr(t):
    """Device (or raw integer) pointer of a tensor-like argument."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_contiguous():
        raise ValueError("tensors must be contiguous")
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _nbytes(t) -> int:
    return 0 if t is None or isinstance(t, int) else t.numel() * t.element_size()


def _check(code: int) -> None:
    if code != 0:
        raise BsaError(code, mosaic_bsa_strerror(code))


def mosaic_bsa_strerror(code: int) -> str:
    return load_library().mosaic_bsa_strerror(int(code)).decode()


def mosaic_bsa_workspace_bytes(params: Params, op: int) -> int:
    cp = params.c_struct()
    return int(load_library().mosaic_bsa_workspace_bytes(ctypes.byref(cp), int(op)))


def mosaic_bsa_select(params: Params, q, k, sel_idx, workspace, stream=None,
                      workspace_bytes=None) -> None:
    cp = params.c_struct()
    wb = _nbytes(workspace) if workspace_bytes is None else workspace_bytes
    _check(load_library().mosaic_bsa_select(
        ctypes.byref(cp), _ptr(q), _ptr(k), _ptr(sel_idx), _ptr(workspace), wb,
        _stream(stream)))


def mosaic_bsa_select_static(params: Params, q, k, sel_idx, stream=None) -> None:
    cp = params.c_struct()
    _check(load_library().mosaic_bsa_select_static(
        ctypes.byref(cp), _ptr(q), _ptr(k), _ptr(sel_idx), _stream(stream)))


def mosaic_bsa_fwd(params: Params, q, k, v, sel_idx, out, lse=None,
                   workspace=None, stream=None, workspace_bytes=None) -> None:
    cp = params.c_struct()
    wb = _nbytes(workspace) if workspace_bytes is None else workspace_bytes
    _check(load_library().mosaic_bsa_fwd(
        ctypes.byref(cp), _ptr(q), _ptr(k), _ptr(v), _ptr(sel_idx), _ptr(out),
        _ptr(lse), _ptr(workspace), wb, _stream(stream)))


def mosaic_bsa_bwd(params: Params, q, k, v, out, lse, dout, sel_idx, dq, dk, dv,
                   workspace=None, stream=None, workspace_bytes=None) -> None:
    cp = params.c_struct()
    wb = _nbytes(workspace) if workspace_bytes is None else workspace_bytes
    _check(load_library().mosaic_bsa_bwd(
        ctypes.byref(cp), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse),
        _ptr(dout), _ptr(sel_idx), _ptr(dq), _ptr(dk), _ptr(dv),
        _ptr(workspace), wb, _stream(stream)))


def mosaic_bsa_three_branch_workspace_bytes(params: Params, local_h: int, local_w: int) -> int:
    cp = params.c_struct()
    return int(load_library().mosaic_bsa_three_branch_workspace_bytes(
        ctypes.byref(cp), int(local_h), int(local_w)))


def mosaic_bsa_fwd_three_branch(params: Params, local_h: int, local_w: int, q, k, v, gates,
                                out, sel_idx, workspace, stream=None,
                                workspace_bytes=None) -> None:
    cp = params.c_struct()
    wb = _nbytes(workspace) if workspace_bytes is None else workspace_bytes
    _check(load_library().mosaic_bsa_fwd_three_branch(
        ctypes.byref(cp), int(local_h), int(local_w), _ptr(q), _ptr(k), _ptr(v), _ptr(gates),
        _ptr(out), _ptr(sel_idx), _ptr(workspace), wb, _stream(stream)))


def mosaic_bsa_probe_mfma(sink, workgroups: int, iters: int, stream=None) -> None:
    _check(load_library().mosaic_bsa_probe_mfma(_ptr(sink), int(workgroups), int(iters),
                                                _stream(stream)))


def mosaic_bsa_three_branch_bwd_workspace_bytes(params: Params, local_h: int,
                                                local_w: int) -> int:
    cp = params.c_struct()
    return int(load_library().mosaic_bsa_three_branch_bwd_workspace_bytes(
        ctypes.byref(cp), int(local_h), int(local_w)))


def mosaic_bsa_bwd_three_branch(params: Params, local_h: int, local_w: int, q, k, v, gates,
                                dout, sel_idx, fwd_workspace, dq, dk, dv, dgates, workspace,
                                stream=None, workspace_bytes=None) -> None:
    cp = params.c_struct()
    wb = _nbytes(workspace) if workspace_bytes is None else workspace_bytes
    _check(load_library().mosaic_bsa_bwd_three_branch(
        ctypes.byref(cp), int(local_h), int(local_w), _ptr(q), _ptr(k), _ptr(v), _ptr(gates),
        _ptr(dout), _ptr(sel_idx), _ptr(fwd_workspace), _ptr(dq), _ptr(dk), _ptr(dv),
        _ptr(dgates), _ptr(workspace), wb, _stream(stream)))


def mosaic_bsa_check_selection(params: Params, sel_idx, own_block_allowed: bool, n_bad,
                               stream=None) -> None:
    cp = params.c_struct()
    _check(load_library().mosaic_bsa_check_selection(
        ctypes.byref(cp), _ptr(sel_idx), 1 if own_block_allowed else 0, _ptr(n_bad),
        _stream(stream)))
