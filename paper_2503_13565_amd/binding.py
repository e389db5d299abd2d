"""Thin ctypes binding of ``include/mxfp4.h``: argument marshalling only.

Every step of the path runs in the HIP kernels of ``libmxfp4_hip.so``; torch supplies device
memory and the current stream.  There is no fallback: if the library has not been built
(``python -m paper_2503_13565_amd.build``) the first call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmxfp4_hip.so")

PATH_AUTO, PATH_VALU_BITS, PATH_VALU_CVT, PATH_VALU_LUT, PATH_MFMA, PATH_VALU_REG, PATH_MFMA_GENERAL = 0, 1, 2, 3, 4, 5, 6

EXPORTS = [
    "mxfp4_direct_cast", "mxfp4_direct_cast_bits", "mxfp4_dequant", "mxfp4_dequant_hwcvt", "mxfp4_woq_gemm", "mxfp4_woq_gemm_path",
    "mxfp4_woq_gemm_workspace_bytes", "mxfp4_woq_gemm_ws", "mxfp4_woq_gemm_argmax_workspace_bytes", "mxfp4_woq_gemm_argmax", "mxfp4_woq_gemm_argmax_path",
    "mxfp4_bf16_gemm", "mxfp4_bf16_gemm_argmax_workspace_bytes", "mxfp4_bf16_gemm_argmax",
    "mxfp4_woq_gemm_verify", "mxfp4_bf16_gemm_verify",
    "mxfp4_woq_gemm_fused", "mxfp4_woq_gemm_grouped_workspace_bytes", "mxfp4_woq_gemm_grouped",
    "mxfp4_woq_gemm_argmax_noalloc_max_bytes", "mxfp4_woq_gemm_argmax_noalloc",
    "mxfp4_woq_gemm_chain_workspace_bytes", "mxfp4_woq_gemm_chain_init", "mxfp4_woq_gemm_chain",
    "mxfp4_e4m3_direct_cast", "mxfp4_e4m3_direct_cast_bits", "mxfp4_e4m3_dequant", "mxfp4_e4m3_woq_gemm",
    "mxfp4_e4m3_woq_gemm_argmax",
    "mxfp4_e2m3_direct_cast", "mxfp4_e2m3_direct_cast_bits", "mxfp4_e2m3_dequant", "mxfp4_e2m3_woq_gemm",
    "mxfp4_e2m3_woq_gemm_argmax",
    "mxfp4_fmt_block_bytes", "mxfp4_fmt_direct_cast", "mxfp4_fmt_direct_cast_bits", "mxfp4_fmt_dequant",
    "mxfp4_fmt_woq_gemm", "mxfp4_fmt_woq_gemm_argmax",
    "mxfp4_woq_gemm_t_workspace_bytes", "mxfp4_woq_gemm_t",
    "mxfp4_tile_repack_q_bytes", "mxfp4_tile_repack_s_bytes", "mxfp4_tile_repack", "mxfp4_woq_gemm_tiled",
    "mxfp4_woq_gemm_tiled_ws",
    "mxfp4_woq_gemm_tiled_argmax", "mxfp4_woq_gemm_tiled_verify", "mxfp4_woq_gemm_tiled_fused",
    "mxfp4_diag_stream_read", "mxfp4_diag_stream_copy", "mxfp4_last_error", "mxfp4_version",
]

_lib = None


class GemmDesc(ctypes.Structure):
    """``mxfp4_gemm_desc`` of the header, field for field."""
    _fields_ = [("x_bf16", ctypes.c_void_p), ("M", ctypes.c_int64), ("ldx", ctypes.c_int64),
                ("q_packed", ctypes.c_void_p), ("scales_e8m0", ctypes.c_void_p), ("N", ctypes.c_int64),
                ("K", ctypes.c_int64), ("bias_bf16", ctypes.c_void_p), ("residual_bf16", ctypes.c_void_p),
                ("ldr", ctypes.c_int64), ("y_bf16", ctypes.c_void_p), ("ldy", ctypes.c_int64),
                ("argmax_out", ctypes.c_void_p), ("max_out", ctypes.c_void_p),
                ("act", ctypes.c_int32), ("flags", ctypes.c_int32)]


class ChainOpts(ctypes.Structure):
    """``mxfp4_chain_opts`` of the header."""
    _fields_ = [("wait_us", ctypes.c_int64), ("phantom_workgroups", ctypes.c_int32), ("mode", ctypes.c_int32)]


CHAIN_STATUS_OFFSET = 4224
CHAIN_AUTO, CHAIN_PERSISTENT, CHAIN_SEPARATE = 0, 1, 2


class Mxfp4Error(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__("mxfp4 error %d: %s" % (code, text))
        self.code = code


def load() -> ctypes.CDLL:
    """Load the HIP library (torch first, so that both share one HIP runtime)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            "%s is missing: build it with `python -m paper_2503_13565_amd.build`; "
            "there is no fallback path" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t
    lib.mxfp4_direct_cast.argtypes = [vp, i64, i64, i64, vp, vp, vp]
    lib.mxfp4_direct_cast_bits.argtypes = [vp, i64, i64, i64, vp, vp, vp]
    lib.mxfp4_direct_cast_bits.restype = i32
    lib.mxfp4_dequant.argtypes = [vp, vp, i64, i64, vp, i64, vp]
    lib.mxfp4_dequant_hwcvt.argtypes = [vp, vp, i64, i64, vp, i64, vp]
    lib.mxfp4_woq_gemm.argtypes = [vp, i64, i64, vp, vp, i64, i64, vp, i64, vp]
    lib.mxfp4_woq_gemm_path.argtypes = [vp, i64, i64, vp, vp, i64, i64, vp, i64, i32, vp]
    lib.mxfp4_woq_gemm_workspace_bytes.argtypes = [i64, i64, i64]
    lib.mxfp4_woq_gemm_workspace_bytes.restype = sz
    lib.mxfp4_woq_gemm_ws.argtypes = [vp, i64, i64, vp, vp, i64, i64, vp, i64, vp, sz, i32, vp]
    lib.mxfp4_woq_gemm_ws.restype = i32
    lib.mxfp4_woq_gemm_argmax_workspace_bytes.argtypes = [i64, i64, i64]
    lib.mxfp4_woq_gemm_argmax_workspace_bytes.restype = sz
    lib.mxfp4_woq_gemm_argmax.argtypes = [vp, i64, i64, vp, vp, i64, i64, vp, vp, vp, sz, vp]
    lib.mxfp4_woq_gemm_argmax_path.argtypes = [vp, i64, i64, vp, vp, i64, i64, vp, vp, vp, sz, i32, vp]
    lib.mxfp4_bf16_gemm.argtypes = [vp, i64, i64, vp, i64, i64, i64, vp, i64, vp]
    lib.mxfp4_bf16_gemm.restype = i32
    lib.mxfp4_bf16_gemm_argmax_workspace_bytes.argtypes = [i64, i64, i64]
    lib.mxfp4_bf16_gemm_argmax_workspace_bytes.restype = sz
    lib.mxfp4_bf16_gemm_argmax.argtypes = [vp, i64, i64, vp, i64, i64, i64, vp, vp, vp, sz, vp]
    lib.mxfp4_bf16_gemm_argmax.restype = i32
    lib.mxfp4_woq_gemm_verify.argtypes = [vp, i64, i64, vp, vp, i64, i64, vp, vp, vp, vp, vp, sz, vp]
    lib.mxfp4_woq_gemm_verify.restype = i32
    lib.mxfp4_bf16_gemm_verify.argtypes = [vp, i64, i64, vp, i64, i64, i64, vp, vp, vp, vp, vp, sz, vp]
    lib.mxfp4_bf16_gemm_verify.restype = i32
    for name in ("mxfp4_e4m3_direct_cast", "mxfp4_e4m3_direct_cast_bits"):
        getattr(lib, name).argtypes = [vp, i64, i64, i64, vp, vp, vp]
        getattr(lib, name).restype = i32
    lib.mxfp4_e4m3_dequant.argtypes = [vp, vp, i64, i64, vp, i64, vp]
    lib.mxfp4_e4m3_dequant.restype = i32
    lib.mxfp4_e4m3_woq_gemm.argtypes = [vp, i64, i64, vp, vp, i64, i64, vp, i64, vp]
    lib.mxfp4_e4m3_woq_gemm.restype = i32
    lib.mxfp4_e4m3_woq_gemm_argmax.argtypes = [vp, i64, i64, vp, vp, i64, i64, vp, vp, vp, sz, vp]
    lib.mxfp4_e4m3_woq_gemm_argmax.restype = i32
    for name in ("mxfp4_e2m3_direct_cast", "mxfp4_e2m3_direct_cast_bits"):
        getattr(lib, name).argtypes = [vp, i64, i64, i64, vp, vp, vp]
        getattr(lib, name).restype = i32
    lib.mxfp4_e2m3_dequant.argtypes = [vp, vp, i64, i64, vp, i64, vp]
    lib.mxfp4_e2m3_dequant.restype = i32
    lib.mxfp4_e2m3_woq_gemm.argtypes = [vp, i64, i64, vp, vp, i64, i64, vp, i64, vp]
    lib.mxfp4_e2m3_woq_gemm.restype = i32
    lib.mxfp4_e2m3_woq_gemm_argmax.argtypes = [vp, i64, i64, vp, vp, i64, i64, vp, vp, vp, sz, vp]
    lib.mxfp4_e2m3_woq_gemm_argmax.restype = i32
    lib.mxfp4_woq_gemm_t_workspace_bytes.argtypes = [i64, i64, i64]
    lib.mxfp4_woq_gemm_t_workspace_bytes.restype = sz
    lib.mxfp4_woq_gemm_t.argtypes = [vp, i64, i64, vp, vp, i64, i64, vp, i64, vp, sz, vp]
    lib.mxfp4_woq_gemm_t.restype = i32
    lib.mxfp4_fmt_block_bytes.argtypes = [i32]
    lib.mxfp4_fmt_block_bytes.restype = i32
    for name in ("mxfp4_fmt_direct_cast", "mxfp4_fmt_direct_cast_bits"):
        getattr(lib, name).argtypes = [i32, vp, i64, i64, i64, vp, vp, vp]
        getattr(lib, name).restype = i32
    lib.mxfp4_fmt_dequant.argtypes = [i32, vp, vp, i64, i64, vp, i64, vp]
    lib.mxfp4_fmt_dequant.restype = i32
    lib.mxfp4_fmt_woq_gemm.argtypes = [i32, vp, i64, i64, vp, vp, i64, i64, vp, i64, vp]
    lib.mxfp4_fmt_woq_gemm.restype = i32
    lib.mxfp4_fmt_woq_gemm_argmax.argtypes = [i32, vp, i64, i64, vp, vp, i64, i64, vp, vp, vp, sz, vp]
    lib.mxfp4_fmt_woq_gemm_argmax.restype = i32
    lib.mxfp4_woq_gemm_fused.argtypes = [vp, i64, i64, vp, vp, i64, i64, vp, i32, vp, i64, vp, i64, vp, sz, i32, vp]
    lib.mxfp4_woq_gemm_fused.restype = i32
    lib.mxfp4_tile_repack_q_bytes.argtypes = [i64, i64]
    lib.mxfp4_tile_repack_q_bytes.restype = sz
    lib.mxfp4_tile_repack_s_bytes.argtypes = [i64, i64]
    lib.mxfp4_tile_repack_s_bytes.restype = sz
    lib.mxfp4_tile_repack.argtypes = [vp, vp, i64, i64, vp, vp, vp]
    lib.mxfp4_tile_repack.restype = i32
    lib.mxfp4_woq_gemm_tiled.argtypes = [vp, i64, i64, vp, vp, i64, i64, vp, i64, vp]
    lib.mxfp4_woq_gemm_tiled.restype = i32
    lib.mxfp4_woq_gemm_tiled_ws.argtypes = [vp, i64, i64, vp, vp, i64, i64, vp, i64, vp, sz, vp]
    lib.mxfp4_woq_gemm_tiled_ws.restype = i32
    lib.mxfp4_woq_gemm_tiled_argmax.argtypes = [vp, i64, i64, vp, vp, i64, i64, vp, vp, vp, sz, vp]
    lib.mxfp4_woq_gemm_tiled_argmax.restype = i32
    lib.mxfp4_woq_gemm_tiled_verify.argtypes = [vp, i64, i64, vp, vp, i64, i64, vp, vp, vp, vp, vp, sz, vp]
    lib.mxfp4_woq_gemm_tiled_verify.restype = i32
    lib.mxfp4_woq_gemm_tiled_fused.argtypes = [vp, i64, i64, vp, vp, i64, i64, vp, i32, vp, i64, vp, i64, vp]
    lib.mxfp4_woq_gemm_tiled_fused.restype = i32
    lib.mxfp4_woq_gemm_grouped_workspace_bytes.argtypes = [ctypes.POINTER(GemmDesc), i64]
    lib.mxfp4_woq_gemm_grouped_workspace_bytes.restype = sz
    lib.mxfp4_woq_gemm_grouped.argtypes = [ctypes.POINTER(GemmDesc), i64, vp, sz, vp]
    lib.mxfp4_woq_gemm_grouped.restype = i32
    lib.mxfp4_woq_gemm_argmax_noalloc_max_bytes.argtypes = []
    lib.mxfp4_woq_gemm_argmax_noalloc_max_bytes.restype = sz
    lib.mxfp4_woq_gemm_argmax_noalloc.argtypes = [vp, i64, i64, vp, vp, i64, i64, vp, vp, vp]
    lib.mxfp4_woq_gemm_argmax_noalloc.restype = i32
    lib.mxfp4_woq_gemm_chain_workspace_bytes.argtypes = []
    lib.mxfp4_woq_gemm_chain_workspace_bytes.restype = sz
    lib.mxfp4_woq_gemm_chain_init.argtypes = [vp, sz, vp]
    lib.mxfp4_woq_gemm_chain_init.restype = i32
    lib.mxfp4_woq_gemm_chain.argtypes = [ctypes.POINTER(GemmDesc), i64, vp, sz, ctypes.POINTER(ChainOpts), vp]
    lib.mxfp4_woq_gemm_chain.restype = i32
    lib.mxfp4_diag_stream_read.argtypes = [vp, sz, vp, vp]
    lib.mxfp4_diag_stream_copy.argtypes = [vp, vp, sz, vp]
    for name in ("mxfp4_direct_cast", "mxfp4_direct_cast_bits", "mxfp4_dequant", "mxfp4_dequant_hwcvt", "mxfp4_woq_gemm",
                 "mxfp4_woq_gemm_path", "mxfp4_woq_gemm_argmax", "mxfp4_woq_gemm_argmax_path",
                 "mxfp4_diag_stream_read", "mxfp4_diag_stream_copy"):
        getattr(lib, name).restype = i32
    lib.mxfp4_last_error.restype = ctypes.c_char_p
    lib.mxfp4_version.restype = ctypes.c_char_p
    _lib = lib
    return lib


def _check(rc: int) -> None:
    if rc != 0:
        raise Mxfp4Error(rc, load().mxfp4_last_error().decode())


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t: Optional[torch.Tensor]) -> ctypes.c_void_p:
    return ctypes.c_void_p(0 if t is None else t.data_ptr())


def _dev(t: torch.Tensor) -> None:
    if not t.is_cuda:
        raise ValueError("tensor must live in GPU memory")


def version() -> str:
    return load().mxfp4_version().decode()


def mxfp4_direct_cast(w: torch.Tensor, q: Optional[torch.Tensor] = None,
                      s: Optional[torch.Tensor] = None, integer_rule: bool = False
                      ) -> Tuple[torch.Tensor, torch.Tensor]:
    """BF16 ``[N,K]`` (last dim contiguous) -> (q uint8 ``[N,K/2]``, s uint8 ``[N,K/32]``).
    ``integer_rule`` calls ``mxfp4_direct_cast_bits``."""
    _dev(w)
    if w.dtype != torch.bfloat16 or w.dim() != 2 or w.stride(1) != 1:
        raise ValueError("w must be a 2-D BF16 tensor with a contiguous last dimension")
    n, k = w.shape
    if q is None:
        q = torch.empty((n, k // 2), dtype=torch.uint8, device=w.device)
    if s is None:
        s = torch.empty((n, k // 32), dtype=torch.uint8, device=w.device)
    ldw = w.stride(0) if n > 1 else max(k, 1)
    with torch.cuda.device(w.device):
        fn = load().mxfp4_direct_cast_bits if integer_rule else load().mxfp4_direct_cast
        _check(fn(_ptr(w), n, k, ldw, _ptr(q), _ptr(s), _stream()))
    return q, s


def mxfp4_dequant(q: torch.Tensor, s: torch.Tensor, hw_convert: bool = False) -> torch.Tensor:
    _dev(q)
    n, k = q.shape[0], q.shape[1] * 2
    w = torch.empty((n, k), dtype=torch.bfloat16, device=q.device)
    fn = load().mxfp4_dequant_hwcvt if hw_convert else load().mxfp4_dequant
    with torch.cuda.device(q.device):
        _check(fn(_ptr(q), _ptr(s), n, k, _ptr(w), k, _stream()))
    return w


def _gemm_shapes(x, q, s):
    _dev(x)
    if x.dtype != torch.bfloat16 or x.dim() != 2 or x.stride(1) != 1:
        raise ValueError("x must be a 2-D BF16 tensor with a contiguous last dimension")
    if q.dtype != torch.uint8 or s.dtype != torch.uint8 or not q.is_contiguous() or not s.is_contiguous():
        raise ValueError("q and s must be contiguous uint8 tensors")
    m, k = x.shape
    n = q.shape[0]
    if q.shape[1] * 2 != k or tuple(s.shape) != (n, k // 32):
        raise ValueError("shape mismatch: x %r q %r s %r" % (tuple(x.shape), tuple(q.shape), tuple(s.shape)))
    ldx = x.stride(0) if m > 1 else k
    return m, n, k, ldx


def mxfp4_woq_gemm(x: torch.Tensor, q: torch.Tensor, s: torch.Tensor, y: Optional[torch.Tensor] = None,
                   path: int = PATH_AUTO, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """y ``[M,N]`` BF16 = x ``[M,K]`` BF16 times dequant(q, s)^T.  With ``workspace`` (uint8, at least
    ``mxfp4_woq_gemm_workspace_bytes``) the call goes through ``mxfp4_woq_gemm_ws``."""
    m, n, k, ldx = _gemm_shapes(x, q, s)
    if y is None:
        y = torch.empty((m, n), dtype=torch.bfloat16, device=x.device)
    ldy = y.stride(0) if m > 1 else n
    with torch.cuda.device(x.device):
        if workspace is None:
            _check(load().mxfp4_woq_gemm_path(_ptr(x), m, ldx, _ptr(q), _ptr(s), n, k, _ptr(y), ldy, path,
                                             _stream()))
        else:
            _check(load().mxfp4_woq_gemm_ws(_ptr(x), m, ldx, _ptr(q), _ptr(s), n, k, _ptr(y), ldy,
                                           _ptr(workspace), workspace.numel() * workspace.element_size(),
                                           path, _stream()))
    return y


def mxfp4_woq_gemm_workspace_bytes(m: int, n: int, k: int) -> int:
    return int(load().mxfp4_woq_gemm_workspace_bytes(m, n, k))


def mxfp4_woq_gemm_argmax_workspace_bytes(m: int, n: int, k: int) -> int:
    return int(load().mxfp4_woq_gemm_argmax_workspace_bytes(m, n, k))


def mxfp4_woq_gemm_argmax(x: torch.Tensor, q: torch.Tensor, s: torch.Tensor,
                          workspace: Optional[torch.Tensor] = None, path: int = PATH_AUTO,
                          out: Optional[Tuple[torch.Tensor, torch.Tensor]] = None
                          ) -> Tuple[torch.Tensor, torch.Tensor]:
    """Row-wise (argmax int32 ``[M]``, max float32 ``[M]``) of x times dequant(q, s)^T."""
    m, n, k, ldx = _gemm_shapes(x, q, s)
    need = mxfp4_woq_gemm_argmax_workspace_bytes(m, n, k)
    if workspace is None:
        workspace = torch.empty((need,), dtype=torch.uint8, device=x.device)
    if out is None:
        idx = torch.empty((m,), dtype=torch.int32, device=x.device)
        val = torch.empty((m,), dtype=torch.float32, device=x.device)
    else:
        idx, val = out
    with torch.cuda.device(x.device):
        _check(load().mxfp4_woq_gemm_argmax_path(_ptr(x), m, ldx, _ptr(q), _ptr(s), n, k, _ptr(idx), _ptr(val),
                                                _ptr(workspace), workspace.numel() * workspace.element_size(),
                                                path, _stream()))
    return idx, val


def mxfp4_woq_gemm_argmax_noalloc(x: torch.Tensor, q: torch.Tensor, s: torch.Tensor,
                                  out: Tuple[torch.Tensor, torch.Tensor]) -> Tuple[torch.Tensor, torch.Tensor]:
    """The fused pick on the library's own scratch: nothing is allocated here either, so the caller
    brings ``out = (idx int32 [M], val float32 [M])``."""
    m, n, k, ldx = _gemm_shapes(x, q, s)
    idx, val = out
    if (idx.dtype != torch.int32 or val.dtype != torch.float32 or idx.shape != (m,) or val.shape != (m,)
            or not idx.is_contiguous() or not val.is_contiguous()):
        raise ValueError("out must be (int32 [M], float32 [M]), contiguous")
    with torch.cuda.device(x.device):
        _check(load().mxfp4_woq_gemm_argmax_noalloc(_ptr(x), m, ldx, _ptr(q), _ptr(s), n, k, _ptr(idx), _ptr(val),
                                                    _stream()))
    return idx, val


def _bf16_shapes(x, w):
    _dev(x)
    for t, what in ((x, "x"), (w, "w")):
        if t.dtype != torch.bfloat16 or t.dim() != 2 or t.stride(1) != 1:
            raise ValueError("%s must be a 2-D BF16 tensor with a contiguous last dimension" % what)
    m, k = x.shape
    n = w.shape[0]
    if w.shape[1] != k:
        raise ValueError("shape mismatch: x %r w %r" % (tuple(x.shape), tuple(w.shape)))
    return m, n, k, (x.stride(0) if m > 1 else k), (w.stride(0) if n > 1 else k)


def mxfp4_bf16_gemm(x: torch.Tensor, w: torch.Tensor, y: Optional[torch.Tensor] = None) -> torch.Tensor:
    """y ``[M,N]`` BF16 = x ``[M,K]`` BF16 times w ``[N,K]``^T with unquantised BF16 weights."""
    m, n, k, ldx, ldw = _bf16_shapes(x, w)
    if y is None:
        y = torch.empty((m, n), dtype=torch.bfloat16, device=x.device)
    with torch.cuda.device(x.device):
        _check(load().mxfp4_bf16_gemm(_ptr(x), m, ldx, _ptr(w), n, k, ldw, _ptr(y),
                                     y.stride(0) if m > 1 else n, _stream()))
    return y


def mxfp4_bf16_gemm_argmax_workspace_bytes(m: int, n: int, k: int) -> int:
    return int(load().mxfp4_bf16_gemm_argmax_workspace_bytes(m, n, k))


def mxfp4_bf16_gemm_argmax(x: torch.Tensor, w: torch.Tensor, workspace: Optional[torch.Tensor] = None,
                           out: Optional[Tuple[torch.Tensor, torch.Tensor]] = None
                           ) -> Tuple[torch.Tensor, torch.Tensor]:
    """Row-wise (argmax int32 ``[M]``, max float32 ``[M]``) of x times w^T."""
    m, n, k, ldx, ldw = _bf16_shapes(x, w)
    if workspace is None:
        workspace = torch.empty((mxfp4_bf16_gemm_argmax_workspace_bytes(m, n, k),), dtype=torch.uint8,
                                device=x.device)
    if out is None:
        idx = torch.empty((m,), dtype=torch.int32, device=x.device)
        val = torch.empty((m,), dtype=torch.float32, device=x.device)
    else:
        idx, val = out
    with torch.cuda.device(x.device):
        _check(load().mxfp4_bf16_gemm_argmax(_ptr(x), m, ldx, _ptr(w), n, k, ldw, _ptr(idx), _ptr(val),
                                            _ptr(workspace), workspace.numel() * workspace.element_size(),
                                            _stream()))
    return idx, val


def _verify_buffers(x, m, draft, need, workspace):
    if draft is not None and (draft.dtype != torch.int32 or draft.numel() != m - 1 or not draft.is_contiguous()):
        raise ValueError("draft must hold M - 1 contiguous int32 tokens")
    if workspace is None:
        workspace = torch.empty((need,), dtype=torch.uint8, device=x.device)
    accept = torch.empty((2,), dtype=torch.int32, device=x.device)
    idx = torch.empty((m,), dtype=torch.int32, device=x.device)
    val = torch.empty((m,), dtype=torch.float32, device=x.device)
    return workspace, accept, idx, val


def mxfp4_woq_gemm_verify(x: torch.Tensor, q: torch.Tensor, s: torch.Tensor, draft: Optional[torch.Tensor],
                          workspace: Optional[torch.Tensor] = None):
    """(accept int32 ``[2]`` = (G, next token), argmax int32 ``[M]``, max float32 ``[M]``)."""
    m, n, k, ldx = _gemm_shapes(x, q, s)
    workspace, accept, idx, val = _verify_buffers(x, m, draft, mxfp4_woq_gemm_argmax_workspace_bytes(m, n, k),
                                                  workspace)
    with torch.cuda.device(x.device):
        _check(load().mxfp4_woq_gemm_verify(_ptr(x), m, ldx, _ptr(q), _ptr(s), n, k, _ptr(draft), _ptr(accept),
                                           _ptr(idx), _ptr(val), _ptr(workspace),
                                           workspace.numel() * workspace.element_size(), _stream()))
    return accept, idx, val


def mxfp4_e4m3_direct_cast(w: torch.Tensor, integer_rule: bool = False) -> Tuple[torch.Tensor, torch.Tensor]:
    """BF16 ``[N, K]`` -> (``q8 [N, K]`` E4M3 bytes, ``s [N, K/32]`` E8M0 scale bytes)."""
    _dev(w)
    if w.dtype != torch.bfloat16 or w.dim() != 2 or w.stride(1) != 1:
        raise ValueError("w must be a 2-D BF16 tensor with a contiguous last dimension")
    n, k = w.shape
    q8 = torch.empty((n, k), dtype=torch.uint8, device=w.device)
    s = torch.empty((n, k // 32), dtype=torch.uint8, device=w.device)
    fn = load().mxfp4_e4m3_direct_cast_bits if integer_rule else load().mxfp4_e4m3_direct_cast
    with torch.cuda.device(w.device):
        _check(fn(_ptr(w), n, k, w.stride(0) if n > 1 else k, _ptr(q8), _ptr(s), _stream()))
    return q8, s


def mxfp4_e4m3_dequant(q8: torch.Tensor, s: torch.Tensor) -> torch.Tensor:
    _dev(q8)
    n, k = q8.shape
    w = torch.empty((n, k), dtype=torch.bfloat16, device=q8.device)
    with torch.cuda.device(q8.device):
        _check(load().mxfp4_e4m3_dequant(_ptr(q8), _ptr(s), n, k, _ptr(w), k, _stream()))
    return w


def _e4m3_shapes(x, q8, s):
    _dev(x)
    if x.dtype != torch.bfloat16 or x.dim() != 2 or x.stride(1) != 1:
        raise ValueError("x must be a 2-D BF16 tensor with a contiguous last dimension")
    if q8.dtype != torch.uint8 or s.dtype != torch.uint8 or not q8.is_contiguous() or not s.is_contiguous():
        raise ValueError("q8 and s must be contiguous uint8 tensors")
    m, k = x.shape
    n = q8.shape[0]
    if q8.shape[1] != k or tuple(s.shape) != (n, k // 32):
        raise ValueError("shape mismatch: x %r q8 %r s %r" % (tuple(x.shape), tuple(q8.shape), tuple(s.shape)))
    return m, n, k, (x.stride(0) if m > 1 else k)


def mxfp4_e4m3_woq_gemm(x: torch.Tensor, q8: torch.Tensor, s: torch.Tensor,
                        y: Optional[torch.Tensor] = None) -> torch.Tensor:
    m, n, k, ldx = _e4m3_shapes(x, q8, s)
    if y is None:
        y = torch.empty((m, n), dtype=torch.bfloat16, device=x.device)
    with torch.cuda.device(x.device):
        _check(load().mxfp4_e4m3_woq_gemm(_ptr(x), m, ldx, _ptr(q8), _ptr(s), n, k, _ptr(y),
                                         y.stride(0) if m > 1 else n, _stream()))
    return y


def mxfp4_e4m3_woq_gemm_argmax(x: torch.Tensor, q8: torch.Tensor, s: torch.Tensor,
                               workspace: Optional[torch.Tensor] = None,
                               out: Optional[Tuple[torch.Tensor, torch.Tensor]] = None
                               ) -> Tuple[torch.Tensor, torch.Tensor]:
    m, n, k, ldx = _e4m3_shapes(x, q8, s)
    if workspace is None:
        workspace = torch.empty((mxfp4_woq_gemm_argmax_workspace_bytes(m, n, k),), dtype=torch.uint8,
                                device=x.device)
    if out is None:
        idx = torch.empty((m,), dtype=torch.int32, device=x.device)
        val = torch.empty((m,), dtype=torch.float32, device=x.device)
    else:
        idx, val = out
    with torch.cuda.device(x.device):
        _check(load().mxfp4_e4m3_woq_gemm_argmax(_ptr(x), m, ldx, _ptr(q8), _ptr(s), n, k, _ptr(idx), _ptr(val),
                                                _ptr(workspace), workspace.numel() * workspace.element_size(),
                                                _stream()))
    return idx, val


def mxfp4_e2m3_direct_cast(w: torch.Tensor, integer_rule: bool = False) -> Tuple[torch.Tensor, torch.Tensor]:
    """BF16 ``[N, K]`` -> (``q6 [N, K/32*24]`` packed E2M3 codes, ``s [N, K/32]`` E8M0 scale bytes)."""
    _dev(w)
    if w.dtype != torch.bfloat16 or w.dim() != 2 or w.stride(1) != 1:
        raise ValueError("w must be a 2-D BF16 tensor with a contiguous last dimension")
    n, k = w.shape
    q6 = torch.empty((n, k // 32 * 24), dtype=torch.uint8, device=w.device)
    s = torch.empty((n, k // 32), dtype=torch.uint8, device=w.device)
    fn = load().mxfp4_e2m3_direct_cast_bits if integer_rule else load().mxfp4_e2m3_direct_cast
    with torch.cuda.device(w.device):
        _check(fn(_ptr(w), n, k, w.stride(0) if n > 1 else k, _ptr(q6), _ptr(s), _stream()))
    return q6, s


def mxfp4_e2m3_dequant(q6: torch.Tensor, s: torch.Tensor) -> torch.Tensor:
    _dev(q6)
    n, k = s.shape[0], s.shape[1] * 32
    w = torch.empty((n, k), dtype=torch.bfloat16, device=q6.device)
    with torch.cuda.device(q6.device):
        _check(load().mxfp4_e2m3_dequant(_ptr(q6), _ptr(s), n, k, _ptr(w), k, _stream()))
    return w


def _e2m3_shapes(x, q6, s):
    _dev(x)
    if x.dtype != torch.bfloat16 or x.dim() != 2 or x.stride(1) != 1:
        raise ValueError("x must be a 2-D BF16 tensor with a contiguous last dimension")
    if q6.dtype != torch.uint8 or s.dtype != torch.uint8 or not q6.is_contiguous() or not s.is_contiguous():
        raise ValueError("q6 and s must be contiguous uint8 tensors")
    m, k = x.shape
    n = q6.shape[0]
    if q6.shape[1] != k // 32 * 24 or tuple(s.shape) != (n, k // 32):
        raise ValueError("shape mismatch: x %r q6 %r s %r" % (tuple(x.shape), tuple(q6.shape), tuple(s.shape)))
    return m, n, k, (x.stride(0) if m > 1 else k)


def mxfp4_e2m3_woq_gemm(x: torch.Tensor, q6: torch.Tensor, s: torch.Tensor,
                        y: Optional[torch.Tensor] = None) -> torch.Tensor:
    m, n, k, ldx = _e2m3_shapes(x, q6, s)
    if y is None:
        y = torch.empty((m, n), dtype=torch.bfloat16, device=x.device)
    with torch.cuda.device(x.device):
        _check(load().mxfp4_e2m3_woq_gemm(_ptr(x), m, ldx, _ptr(q6), _ptr(s), n, k, _ptr(y),
                                         y.stride(0) if m > 1 else n, _stream()))
    return y


def mxfp4_e2m3_woq_gemm_argmax(x: torch.Tensor, q6: torch.Tensor, s: torch.Tensor,
                               workspace: Optional[torch.Tensor] = None,
                               out: Optional[Tuple[torch.Tensor, torch.Tensor]] = None
                               ) -> Tuple[torch.Tensor, torch.Tensor]:
    m, n, k, ldx = _e2m3_shapes(x, q6, s)
    if workspace is None:
        workspace = torch.empty((mxfp4_woq_gemm_argmax_workspace_bytes(m, n, k),), dtype=torch.uint8,
                                device=x.device)
    if out is None:
        idx = torch.empty((m,), dtype=torch.int32, device=x.device)
        val = torch.empty((m,), dtype=torch.float32, device=x.device)
    else:
        idx, val = out
    with torch.cuda.device(x.device):
        _check(load().mxfp4_e2m3_woq_gemm_argmax(_ptr(x), m, ldx, _ptr(q6), _ptr(s), n, k, _ptr(idx), _ptr(val),
                                                _ptr(workspace), workspace.numel() * workspace.element_size(),
                                                _stream()))
    return idx, val


def mxfp4_woq_gemm_t_workspace_bytes(m: int, n: int, k: int) -> int:
    return int(load().mxfp4_woq_gemm_t_workspace_bytes(m, n, k))


def mxfp4_woq_gemm_t(x: torch.Tensor, q: torch.Tensor, s: torch.Tensor, y: Optional[torch.Tensor] = None,
                     workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """``y[M, K] = x[M, N] @ dequant(q, s)[N, K]``: the product along the rows of the stored tensor."""
    _dev(x)
    if x.dtype != torch.bfloat16 or x.dim() != 2 or x.stride(1) != 1:
        raise ValueError("x must be a 2-D BF16 tensor with a contiguous last dimension")
    if q.dtype != torch.uint8 or s.dtype != torch.uint8 or not q.is_contiguous() or not s.is_contiguous():
        raise ValueError("q and s must be contiguous uint8 tensors")
    m, n = x.shape
    k = q.shape[1] * 2
    if q.shape[0] != n or tuple(s.shape) != (n, k // 32):
        raise ValueError("shape mismatch: x %r q %r s %r" % (tuple(x.shape), tuple(q.shape), tuple(s.shape)))
    if y is None:
        y = torch.empty((m, k), dtype=torch.bfloat16, device=x.device)
    if workspace is None:
        workspace = torch.empty((max(mxfp4_woq_gemm_t_workspace_bytes(m, n, k), 4),), dtype=torch.uint8,
                                device=x.device)
    with torch.cuda.device(x.device):
        _check(load().mxfp4_woq_gemm_t(_ptr(x), m, x.stride(0) if m > 1 else n, _ptr(q), _ptr(s), n, k, _ptr(y),
                                      y.stride(0) if m > 1 else k, _ptr(workspace),
                                      workspace.numel() * workspace.element_size(), _stream()))
    return y


FMT_E5M2, FMT_E3M2, FMT_T2 = 1, 2, 3


def mxfp4_fmt_block_bytes(fmt: int) -> int:
    """Bytes of one 32-element block of the format (32, 24, 8); 0 for an unknown id."""
    return int(load().mxfp4_fmt_block_bytes(fmt))


def mxfp4_fmt_direct_cast(fmt: int, w: torch.Tensor, integer_rule: bool = False) -> Tuple[torch.Tensor, torch.Tensor]:
    """BF16 ``[N, K]`` -> (``q [N, K/32 * block_bytes]`` packed codes, ``s [N, K/32]`` E8M0 scale bytes)."""
    _dev(w)
    if w.dtype != torch.bfloat16 or w.dim() != 2 or w.stride(1) != 1:
        raise ValueError("w must be a 2-D BF16 tensor with a contiguous last dimension")
    n, k = w.shape
    q = torch.empty((n, k // 32 * max(mxfp4_fmt_block_bytes(fmt), 1)), dtype=torch.uint8, device=w.device)
    s = torch.empty((n, k // 32), dtype=torch.uint8, device=w.device)
    fn = load().mxfp4_fmt_direct_cast_bits if integer_rule else load().mxfp4_fmt_direct_cast
    with torch.cuda.device(w.device):
        _check(fn(fmt, _ptr(w), n, k, w.stride(0) if n > 1 else k, _ptr(q), _ptr(s), _stream()))
    return q, s


def mxfp4_fmt_dequant(fmt: int, q: torch.Tensor, s: torch.Tensor) -> torch.Tensor:
    _dev(q)
    n, k = s.shape[0], s.shape[1] * 32
    w = torch.empty((n, k), dtype=torch.bfloat16, device=q.device)
    with torch.cuda.device(q.device):
        _check(load().mxfp4_fmt_dequant(fmt, _ptr(q), _ptr(s), n, k, _ptr(w), k, _stream()))
    return w


def _fmt_shapes(fmt, x, q, s):
    _dev(x)
    if x.dtype != torch.bfloat16 or x.dim() != 2 or x.stride(1) != 1:
        raise ValueError("x must be a 2-D BF16 tensor with a contiguous last dimension")
    if q.dtype != torch.uint8 or s.dtype != torch.uint8 or not q.is_contiguous() or not s.is_contiguous():
        raise ValueError("q and s must be contiguous uint8 tensors")
    m, k = x.shape
    n = q.shape[0]
    bb = mxfp4_fmt_block_bytes(fmt)
    if bb and (q.shape[1] != k // 32 * bb or tuple(s.shape) != (n, k // 32)):
        raise ValueError("shape mismatch: x %r q %r s %r" % (tuple(x.shape), tuple(q.shape), tuple(s.shape)))
    return m, n, k, (x.stride(0) if m > 1 else k)


def mxfp4_fmt_woq_gemm(fmt: int, x: torch.Tensor, q: torch.Tensor, s: torch.Tensor,
                       y: Optional[torch.Tensor] = None) -> torch.Tensor:
    m, n, k, ldx = _fmt_shapes(fmt, x, q, s)
    if y is None:
        y = torch.empty((m, n), dtype=torch.bfloat16, device=x.device)
    with torch.cuda.device(x.device):
        _check(load().mxfp4_fmt_woq_gemm(fmt, _ptr(x), m, ldx, _ptr(q), _ptr(s), n, k, _ptr(y),
                                        y.stride(0) if m > 1 else n, _stream()))
    return y


def mxfp4_fmt_woq_gemm_argmax(fmt: int, x: torch.Tensor, q: torch.Tensor, s: torch.Tensor,
                              workspace: Optional[torch.Tensor] = None,
                              out: Optional[Tuple[torch.Tensor, torch.Tensor]] = None
                              ) -> Tuple[torch.Tensor, torch.Tensor]:
    m, n, k, ldx = _fmt_shapes(fmt, x, q, s)
    if workspace is None:
        workspace = torch.empty((mxfp4_woq_gemm_argmax_workspace_bytes(m, n, k),), dtype=torch.uint8,
                                device=x.device)
    if out is None:
        idx = torch.empty((m,), dtype=torch.int32, device=x.device)
        val = torch.empty((m,), dtype=torch.float32, device=x.device)
    else:
        idx, val = out
    with torch.cuda.device(x.device):
        _check(load().mxfp4_fmt_woq_gemm_argmax(fmt, _ptr(x), m, ldx, _ptr(q), _ptr(s), n, k, _ptr(idx), _ptr(val),
                                               _ptr(workspace), workspace.numel() * workspace.element_size(),
                                               _stream()))
    return idx, val


ACT_NONE, ACT_SWIGLU = 0, 1


def mxfp4_woq_gemm_fused(x: torch.Tensor, q: torch.Tensor, s: torch.Tensor, bias: Optional[torch.Tensor] = None,
                         act: int = ACT_NONE, residual: Optional[torch.Tensor] = None,
                         y: Optional[torch.Tensor] = None, path: int = PATH_AUTO,
                         workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """The product with bias, gate and residual add fused; ``residual`` may be ``y`` itself."""
    m, n, k, ldx = _gemm_shapes(x, q, s)
    c = n // 2 if act == ACT_SWIGLU else n
    if bias is not None and (bias.dtype != torch.bfloat16 or bias.dim() != 1 or bias.shape[0] != n
                             or not bias.is_contiguous() or bias.device != x.device):
        raise ValueError("bias must be a contiguous BF16 tensor [N] on the device of x")
    if residual is not None and (residual.dtype != torch.bfloat16 or residual.dim() != 2
                                 or residual.shape != (m, c) or residual.stride(1) != 1
                                 or residual.device != x.device):
        raise ValueError("residual must be a BF16 tensor [M, %d] with a contiguous last dimension" % c)
    if y is None:
        y = torch.empty((m, c), dtype=torch.bfloat16, device=x.device)
    ldy = y.stride(0) if m > 1 else c
    ldr = (residual.stride(0) if m > 1 else c) if residual is not None else 0
    with torch.cuda.device(x.device):
        _check(load().mxfp4_woq_gemm_fused(
            _ptr(x), m, ldx, _ptr(q), _ptr(s), n, k, _ptr(bias), act, _ptr(residual), ldr, _ptr(y), ldy,
            _ptr(workspace), workspace.numel() * workspace.element_size() if workspace is not None else 0, path,
            _stream()))
    return y


DESC_TILED = 1
DESC_INDEPENDENT = 2


class GemmGroup:
    """A fixed sequence of products (``mxfp4_woq_gemm_grouped``): the descriptor array is built once,
    ``run()`` is one library call.  ``items``: dicts with ``x``, ``q``, ``s`` and optionally ``bias``,
    ``act``, ``residual``, ``y`` (allocated when missing), as for ``mxfp4_woq_gemm_fused``; or with
    ``argmax=True`` (optionally ``out=(idx int32 [M], val float32 [M])``) for the fused pick, whose
    entry in ``ys`` is the ``(idx, val)`` pair.  The tensors are kept alive by the group; ``ys`` lists
    the outputs in order.  An item with ``w`` (a ``TiledWeights``) in place of ``q`` and ``s`` runs on
    the tile-major copy.  ``independent=True`` on an item sets ``MXFP4_DESC_INDEPENDENT``: neighbouring
    items that carry it and do not read each other's outputs may share one launch.
    ``chained=True``: ``run()`` is ``mxfp4_woq_gemm_chain`` (a dependent sequence of one-token
    products on canonical tensors, ``mode`` = ``CHAIN_AUTO``, ``CHAIN_PERSISTENT`` or
    ``CHAIN_SEPARATE``); the group then owns a chain workspace, prepared once, and
    ``chain_status()`` reads its status word (synchronises)."""

    def __init__(self, items, chained: bool = False, wait_us: int = 0, phantom_workgroups: int = 0,
                 mode: int = 0):
        self._keep, self.ys = [], []
        self._descs = (GemmDesc * max(1, len(items)))()
        self.count = len(items)
        for d, it in zip(self._descs, items):
            x = it["x"]
            bias, residual, act = it.get("bias"), it.get("residual"), int(it.get("act", ACT_NONE))
            if "w" in it:                                  # TiledWeights in place of (q, s)
                q, s = it["w"].q, it["w"].s
                m, n, k, ldx = _tiled_shapes(x, it["w"])
                d.flags = DESC_TILED
            else:
                q, s = it["q"], it["s"]
                m, n, k, ldx = _gemm_shapes(x, q, s)
                d.flags = 0
            if it.get("independent"):
                d.flags |= DESC_INDEPENDENT
            d.x_bf16, d.M, d.ldx = x.data_ptr(), m, ldx
            d.q_packed, d.scales_e8m0, d.N, d.K = q.data_ptr(), s.data_ptr(), n, k
            d.act = act
            if it.get("argmax"):
                idx, val = it.get("out") or (torch.empty((m,), dtype=torch.int32, device=x.device),
                                             torch.empty((m,), dtype=torch.float32, device=x.device))
                if (idx.dtype != torch.int32 or val.dtype != torch.float32 or idx.shape != (m,) or val.shape != (m,)
                        or not idx.is_contiguous() or not val.is_contiguous()):
                    raise ValueError("out must be (int32 [M], float32 [M]), contiguous")
                d.argmax_out, d.max_out = idx.data_ptr(), val.data_ptr()
                self._keep.append((x, q, s, idx, val))
                self.ys.append((idx, val))
                continue
            c = n // 2 if act == ACT_SWIGLU else n
            y = it.get("y")
            if y is None:
                y = torch.empty((m, c), dtype=torch.bfloat16, device=x.device)
            if y.dtype != torch.bfloat16 or y.dim() != 2 or y.shape != (m, c) or y.stride(1) != 1:
                raise ValueError("y must be a BF16 tensor [M, %d] with a contiguous last dimension" % c)
            if bias is not None and (bias.dtype != torch.bfloat16 or bias.shape != (n,) or not bias.is_contiguous()):
                raise ValueError("bias must be a contiguous BF16 tensor [N]")
            if residual is not None and (residual.dtype != torch.bfloat16 or residual.shape != (m, c)
                                         or residual.stride(1) != 1):
                raise ValueError("residual must be a BF16 tensor [M, %d] with a contiguous last dimension" % c)
            d.bias_bf16 = bias.data_ptr() if bias is not None else None
            d.residual_bf16 = residual.data_ptr() if residual is not None else None
            d.ldr = (residual.stride(0) if m > 1 else c) if residual is not None else 0
            d.y_bf16, d.ldy = y.data_ptr(), (y.stride(0) if m > 1 else c)
            self._keep.append((x, q, s, bias, residual, y))
            self.ys.append(y)
        self.device = items[0]["x"].device if items else None
        self.chained = chained
        if chained:
            self._opts = ChainOpts(int(wait_us), int(phantom_workgroups), int(mode))
            self.workspace = None
            self.chain_ws = None
            if self.count:
                nbytes = int(load().mxfp4_woq_gemm_chain_workspace_bytes())
                self.chain_ws = torch.empty((nbytes,), dtype=torch.uint8, device=self.device)
                self.chain_reset()
            return
        need = int(load().mxfp4_woq_gemm_grouped_workspace_bytes(self._descs, self.count))
        self.workspace = torch.empty((need,), dtype=torch.uint8, device=self.device) if need else None

    def chain_reset(self) -> None:
        """Prepare the chain workspace again (after a wait that was given up)."""
        with torch.cuda.device(self.device):
            _check(load().mxfp4_woq_gemm_chain_init(_ptr(self.chain_ws), self.chain_ws.numel(), _stream()))

    def chain_status(self) -> int:
        """The chain workspace's status word (0: every wait so far was met); synchronises."""
        return int(self.chain_ws[CHAIN_STATUS_OFFSET:CHAIN_STATUS_OFFSET + 4].view(torch.int32).item())

    def run(self) -> None:
        if self.count == 0:
            return
        if self.chained:
            with torch.cuda.device(self.device):
                _check(load().mxfp4_woq_gemm_chain(self._descs, self.count, _ptr(self.chain_ws),
                                                   self.chain_ws.numel(), ctypes.byref(self._opts), _stream()))
            return
        with torch.cuda.device(self.device):
            _check(load().mxfp4_woq_gemm_grouped(
                self._descs, self.count, _ptr(self.workspace),
                self.workspace.numel() if self.workspace is not None else 0, _stream()))


class TiledWeights:
    """The tile-major copy of an MXFP4 weight pair (``mxfp4_tile_repack``) with its logical shape."""

    def __init__(self, q_tiled: torch.Tensor, s_tiled: torch.Tensor, n: int, k: int):
        self.q, self.s, self.n, self.k = q_tiled, s_tiled, n, k


def mxfp4_tile_repack(q: torch.Tensor, s: torch.Tensor) -> TiledWeights:
    _dev(q)
    if q.dtype != torch.uint8 or s.dtype != torch.uint8 or not q.is_contiguous() or not s.is_contiguous():
        raise ValueError("q and s must be contiguous uint8 tensors")
    n, k = q.shape[0], q.shape[1] * 2
    qt = torch.empty((int(load().mxfp4_tile_repack_q_bytes(n, k)),), dtype=torch.uint8, device=q.device)
    st = torch.empty((int(load().mxfp4_tile_repack_s_bytes(n, k)),), dtype=torch.uint8, device=q.device)
    with torch.cuda.device(q.device):
        _check(load().mxfp4_tile_repack(_ptr(q), _ptr(s), n, k, _ptr(qt), _ptr(st), _stream()))
    return TiledWeights(qt, st, n, k)


def _tiled_shapes(x: torch.Tensor, w: TiledWeights):
    _dev(x)
    if x.dtype != torch.bfloat16 or x.dim() != 2 or x.stride(1) != 1 or x.shape[1] != w.k:
        raise ValueError("x must be a 2-D BF16 tensor [M, %d] with a contiguous last dimension" % w.k)
    m = x.shape[0]
    return m, w.n, w.k, (x.stride(0) if m > 1 else w.k)


def mxfp4_woq_gemm_tiled(x: torch.Tensor, w: TiledWeights, y: Optional[torch.Tensor] = None,
                         workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """The product on the tile-major copy; with ``workspace`` (uint8, ``mxfp4_woq_gemm_workspace_bytes``)
    through ``mxfp4_woq_gemm_tiled_ws``, which also takes the shapes that need K split."""
    m, n, k, ldx = _tiled_shapes(x, w)
    if y is None:
        y = torch.empty((m, n), dtype=torch.bfloat16, device=x.device)
    ldy = y.stride(0) if m > 1 else n
    with torch.cuda.device(x.device):
        if workspace is None:
            _check(load().mxfp4_woq_gemm_tiled(_ptr(x), m, ldx, _ptr(w.q), _ptr(w.s), n, k, _ptr(y), ldy, _stream()))
        else:
            _check(load().mxfp4_woq_gemm_tiled_ws(_ptr(x), m, ldx, _ptr(w.q), _ptr(w.s), n, k, _ptr(y), ldy,
                                                 _ptr(workspace), workspace.numel() * workspace.element_size(),
                                                 _stream()))
    return y


def mxfp4_woq_gemm_tiled_fused(x: torch.Tensor, w: TiledWeights, bias: Optional[torch.Tensor] = None,
                               act: int = ACT_NONE, residual: Optional[torch.Tensor] = None,
                               y: Optional[torch.Tensor] = None) -> torch.Tensor:
    m, n, k, ldx = _tiled_shapes(x, w)
    c = n // 2 if act == ACT_SWIGLU else n
    if bias is not None and (bias.dtype != torch.bfloat16 or bias.dim() != 1 or bias.shape[0] != n
                             or not bias.is_contiguous() or bias.device != x.device):
        raise ValueError("bias must be a contiguous BF16 tensor [N] on the device of x")
    if residual is not None and (residual.dtype != torch.bfloat16 or residual.dim() != 2
                                 or residual.shape != (m, c) or residual.stride(1) != 1
                                 or residual.device != x.device):
        raise ValueError("residual must be a BF16 tensor [M, %d] with a contiguous last dimension" % c)
    if y is None:
        y = torch.empty((m, c), dtype=torch.bfloat16, device=x.device)
    ldy = y.stride(0) if m > 1 else c
    ldr = (residual.stride(0) if m > 1 else c) if residual is not None else 0
    with torch.cuda.device(x.device):
        _check(load().mxfp4_woq_gemm_tiled_fused(_ptr(x), m, ldx, _ptr(w.q), _ptr(w.s), n, k, _ptr(bias), act,
                                                _ptr(residual), ldr, _ptr(y), ldy, _stream()))
    return y


def mxfp4_woq_gemm_tiled_argmax(x: torch.Tensor, w: TiledWeights, workspace: Optional[torch.Tensor] = None,
                                out: Optional[Tuple[torch.Tensor, torch.Tensor]] = None
                                ) -> Tuple[torch.Tensor, torch.Tensor]:
    m, n, k, ldx = _tiled_shapes(x, w)
    if workspace is None:
        workspace = torch.empty((mxfp4_woq_gemm_argmax_workspace_bytes(m, n, k),), dtype=torch.uint8,
                                device=x.device)
    if out is None:
        idx = torch.empty((m,), dtype=torch.int32, device=x.device)
        val = torch.empty((m,), dtype=torch.float32, device=x.device)
    else:
        idx, val = out
    with torch.cuda.device(x.device):
        _check(load().mxfp4_woq_gemm_tiled_argmax(_ptr(x), m, ldx, _ptr(w.q), _ptr(w.s), n, k, _ptr(idx),
                                                 _ptr(val), _ptr(workspace),
                                                 workspace.numel() * workspace.element_size(), _stream()))
    return idx, val


def mxfp4_woq_gemm_tiled_verify(x: torch.Tensor, w: TiledWeights, draft: Optional[torch.Tensor],
                                workspace: Optional[torch.Tensor] = None):
    m, n, k, ldx = _tiled_shapes(x, w)
    workspace, accept, idx, val = _verify_buffers(x, m, draft, mxfp4_woq_gemm_argmax_workspace_bytes(m, n, k),
                                                  workspace)
    with torch.cuda.device(x.device):
        _check(load().mxfp4_woq_gemm_tiled_verify(_ptr(x), m, ldx, _ptr(w.q), _ptr(w.s), n, k, _ptr(draft),
                                                 _ptr(accept), _ptr(idx), _ptr(val), _ptr(workspace),
                                                 workspace.numel() * workspace.element_size(), _stream()))
    return accept, idx, val


def mxfp4_bf16_gemm_verify(x: torch.Tensor, w: torch.Tensor, draft: Optional[torch.Tensor],
                           workspace: Optional[torch.Tensor] = None):
    """The same with unquantised BF16 weights."""
    m, n, k, ldx, ldw = _bf16_shapes(x, w)
    workspace, accept, idx, val = _verify_buffers(x, m, draft, mxfp4_bf16_gemm_argmax_workspace_bytes(m, n, k),
                                                  workspace)
    with torch.cuda.device(x.device):
        _check(load().mxfp4_bf16_gemm_verify(_ptr(x), m, ldx, _ptr(w), n, k, ldw, _ptr(draft), _ptr(accept),
                                            _ptr(idx), _ptr(val), _ptr(workspace),
                                            workspace.numel() * workspace.element_size(), _stream()))
    return accept, idx, val


def mxfp4_diag_stream_read(src: torch.Tensor, sink: torch.Tensor) -> None:
    with torch.cuda.device(src.device):
        _check(load().mxfp4_diag_stream_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink), _stream()))


def mxfp4_diag_stream_copy(src: torch.Tensor, dst: torch.Tensor) -> None:
    with torch.cuda.device(src.device):
        _check(load().mxfp4_diag_stream_copy(_ptr(src), _ptr(dst), src.numel() * src.element_size(), _stream()))
