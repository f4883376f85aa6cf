"""Thin ctypes binding of liblory.so (C ABI: include/lory.h).

Argument marshalling only: every function takes torch tensors that already
live on the GPU, checks dtype / shape / contiguity on the host, and passes raw
device pointers plus the current torch stream to the entry point of the same
name.  No step of the layer is computed in Python or torch.

The library is built in-tree by `python -m paper_2405_03133_amd.build`; if it
is missing, loading fails with an error (there is no fallback path).
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblory.so")

LORY_OK = 0
LORY_ERR_NULL, LORY_ERR_SHAPE, LORY_ERR_DTYPE, LORY_ERR_ALIGN, LORY_ERR_WORKSPACE, LORY_ERR_DEVICE = range(1, 7)
LORY_F32, LORY_BF16 = 0, 1
LORY_PASS_FWD, LORY_PASS_BWD, LORY_PASS_DENSE = 0, 1, 2

EXPORTS = ("lory_status_string", "lory_version", "lory_set_slab_budget", "lory_set_fused_merge", "lory_profile_enable",
           "lory_profile_read", "lory_merged_save_bytes", "lory_workspace_bytes", "lory_route",
           "lory_route_bwd", "lory_merged_ffn_fwd", "lory_merged_ffn_bwd", "lory_prompt_merge",
           "lory_dense_ffn_fwd", "lory_dense_ffn_fwd_static")


class LoryShape(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("L", ctypes.c_int32), ("T", ctypes.c_int32),
                ("d", ctypes.c_int32), ("d_ff", ctypes.c_int32), ("E", ctypes.c_int32),
                ("dtype", ctypes.c_int32)]


class LoryKernelStat(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char * 32), ("launches", ctypes.c_int32), ("ms", ctypes.c_double),
                ("flops", ctypes.c_double), ("bytes", ctypes.c_double)]


class LoryError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


_lib: Optional[ctypes.CDLL] = None


def lib() -> ctypes.CDLL:
    """Load liblory.so once; raise if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} not found: build it with `python -m paper_2405_03133_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, sz, ci = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
        sp = ctypes.POINTER(LoryShape)
        L.lory_status_string.argtypes = [ci]
        L.lory_status_string.restype = ctypes.c_char_p
        L.lory_version.argtypes = []
        L.lory_version.restype = ctypes.c_char_p
        L.lory_set_slab_budget.argtypes = [sz]
        L.lory_set_slab_budget.restype = ci
        L.lory_set_fused_merge.argtypes = [ci]
        L.lory_set_fused_merge.restype = ci
        L.lory_profile_enable.argtypes = [ci]
        L.lory_profile_enable.restype = ci
        L.lory_profile_read.argtypes = [ctypes.POINTER(LoryKernelStat), ci, ctypes.POINTER(ci)]
        L.lory_profile_read.restype = ci
        L.lory_workspace_bytes.argtypes = [sp, ci, ctypes.POINTER(sz)]
        L.lory_workspace_bytes.restype = ci
        L.lory_route.argtypes = [sp, vp, vp, vp, vp, vp]
        L.lory_route.restype = ci
        L.lory_route_bwd.argtypes = [sp, vp, vp, vp, vp, vp, vp, ci, vp]
        L.lory_route_bwd.restype = ci
        L.lory_prompt_merge.argtypes = [sp] + [vp] * 9
        L.lory_prompt_merge.restype = ci
        L.lory_dense_ffn_fwd.argtypes = [sp, vp, vp, vp, vp, sz, vp]
        L.lory_dense_ffn_fwd.restype = ci
        L.lory_dense_ffn_fwd_static.argtypes = [sp, vp, vp, vp, vp]
        L.lory_dense_ffn_fwd_static.restype = ci
        L.lory_merged_save_bytes.argtypes = [sp, ctypes.POINTER(sz)]
        L.lory_merged_save_bytes.restype = ci
        L.lory_merged_ffn_fwd.argtypes = [sp] + [vp] * 10 + [sz, vp]
        L.lory_merged_ffn_fwd.restype = ci
        L.lory_merged_ffn_bwd.argtypes = [sp] + [vp] * 13 + [ci, ci, vp, vp, sz, vp]
        L.lory_merged_ffn_bwd.restype = ci
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().lory_status_string(int(status)).decode()


def version() -> str:
    return lib().lory_version().decode()


def _dtype_code(t: torch.dtype) -> int:
    if t == torch.float32:
        return LORY_F32
    if t == torch.bfloat16:
        return LORY_BF16
    raise TypeError(f"unsupported dtype {t}")


def make_shape(B: int, L: int, T: int, d: int, d_ff: int, E: int, dtype) -> LoryShape:
    code = dtype if isinstance(dtype, int) else _dtype_code(dtype)
    return LoryShape(B, L, T, d, d_ff, E, code)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("tensor must live on the GPU")
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _check(status: int, where: str) -> None:
    if status != LORY_OK:
        raise LoryError(status, where)


def lory_set_slab_budget(nbytes: int) -> None:
    _check(lib().lory_set_slab_budget(int(nbytes)), "lory_set_slab_budget")


def lory_set_fused_merge(mode: int) -> None:
    """0 = slab pipeline only, 1 = merge inside the GEMM for short segments (default), 2 = wherever it fits,
    3 = as 2 and with the backward's per-segment weight gradients kept on chip."""
    _check(lib().lory_set_fused_merge(int(mode)), "lory_set_fused_merge")


def lory_profile_enable(on: bool) -> None:
    _check(lib().lory_profile_enable(int(bool(on))), "lory_profile_enable")


def lory_profile_read() -> list:
    """Per kernel class: dict(name, launches, ms, flops, bytes) since the last read."""
    buf = (LoryKernelStat * 16)()
    n = ctypes.c_int(0)
    _check(lib().lory_profile_read(buf, 16, ctypes.byref(n)), "lory_profile_read")
    return [dict(name=buf[i].name.decode(), launches=buf[i].launches, ms=buf[i].ms, flops=buf[i].flops,
                 bytes=buf[i].bytes) for i in range(n.value)]


def lory_workspace_bytes(shape: LoryShape, which_pass: int) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().lory_workspace_bytes(ctypes.byref(shape), which_pass, ctypes.byref(out)),
           "lory_workspace_bytes")
    return out.value


def lory_merged_save_bytes(shape: LoryShape) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().lory_merged_save_bytes(ctypes.byref(shape), ctypes.byref(out)), "lory_merged_save_bytes")
    return out.value


def alloc_merged_save(shape: LoryShape, device="cuda") -> Optional[torch.Tensor]:
    """Buffer for the merged parameters saved by the forward, or None if the shape has no support."""
    n = lory_merged_save_bytes(shape)
    return torch.empty(n, dtype=torch.uint8, device=device) if n else None


def alloc_workspace(shape: LoryShape, which_pass: int, device="cuda") -> torch.Tensor:
    n = lory_workspace_bytes(shape, which_pass)
    return torch.empty(max(n, 256), dtype=torch.uint8, device=device)


def _shape_from(X: torch.Tensor, T: int, d_ff: int, E: int) -> LoryShape:
    B, L, d = X.shape
    return make_shape(B, L, T, d, d_ff, E, X.dtype)


def lory_route(X: torch.Tensor, R: torch.Tensor, T: int, w: Optional[torch.Tensor] = None,
               hbar: Optional[torch.Tensor] = None, d_ff: int = 64) -> torch.Tensor:
    """X [B,L,d], R [d,E] -> w [B*(L/T), E] fp32 (shifted, first-segment rule applied)."""
    B, L, d = X.shape
    E = R.shape[1]
    if R.shape[0] != d or R.dtype != X.dtype:
        raise ValueError("R must be [d, E] with the dtype of X")
    shape = _shape_from(X, T, d_ff, E)
    if w is None:
        w = torch.empty((B * (L // max(T, 1)), E), dtype=torch.float32, device=X.device)
    if w.dtype != torch.float32 or (hbar is not None and hbar.dtype != torch.float32):
        raise TypeError("w and hbar are fp32")
    _check(lib().lory_route(ctypes.byref(shape), _ptr(X), _ptr(R), _ptr(w), _ptr(hbar), _stream()),
           "lory_route")
    return w


def lory_route_bwd(R: torch.Tensor, w: torch.Tensor, hbar: torch.Tensor, dw: torch.Tensor,
                   dX: torch.Tensor, T: int, dR: Optional[torch.Tensor] = None, accumulate_dR: bool = False,
                   d_ff: int = 64) -> torch.Tensor:
    """Adds the router path to dX [B,L,d] in place and returns dR [d,E] fp32."""
    B, L, d = dX.shape
    E = R.shape[1]
    if R.shape[0] != d or R.dtype != dX.dtype:
        raise ValueError("R must be [d, E] with the dtype of dX")
    S = B * (L // max(T, 1))
    for name, t, shp in (("w", w, (S, E)), ("hbar", hbar, (S, d)), ("dw", dw, (S, E))):
        if t.dtype != torch.float32 or tuple(t.shape) != shp:
            raise ValueError(f"{name} must be fp32 {list(shp)}")
    shape = _shape_from(dX, T, d_ff, E)
    if dR is None:
        if accumulate_dR:
            raise ValueError("accumulate_dR needs a dR tensor")
        dR = torch.empty((d, E), dtype=torch.float32, device=dX.device)
    if dR.dtype != torch.float32 or tuple(dR.shape) != (d, E):
        raise ValueError("dR must be fp32 [d, E]")
    _check(lib().lory_route_bwd(ctypes.byref(shape), _ptr(R), _ptr(w), _ptr(hbar), _ptr(dw), _ptr(dX),
                                _ptr(dR), int(bool(accumulate_dR)), _stream()), "lory_route_bwd")
    return dR


def lory_prompt_merge(X_prompt: torch.Tensor, R: torch.Tensor, Wg: torch.Tensor, Wu: torch.Tensor,
                      Wd: torch.Tensor, w: Optional[torch.Tensor] = None,
                      Wbar: Optional[torch.Tensor] = None, prompt_len: Optional[torch.Tensor] = None):
    """Prompt-only routing: (w [B,E] fp32, Wbar [3, B, d*d_ff] of X's dtype) from the whole prompt;
    prompt_len [B] int32 gives the true lengths of prompts padded to X_prompt's L rows."""
    B, L, d = X_prompt.shape
    E, _, d_ff = Wg.shape
    if tuple(Wu.shape) != (E, d, d_ff) or tuple(Wd.shape) != (E, d_ff, d) or tuple(R.shape) != (d, E):
        raise ValueError("R / expert stack shapes do not match")
    for t in (R, Wg, Wu, Wd):
        if t.dtype != X_prompt.dtype:
            raise TypeError("R and the expert stacks must have the dtype of X_prompt")
    shape = make_shape(B, L, L, d, d_ff, E, X_prompt.dtype)
    if w is None:
        w = torch.empty((B, E), dtype=torch.float32, device=X_prompt.device)
    if Wbar is None:
        Wbar = torch.empty((3, B, d * d_ff), dtype=X_prompt.dtype, device=X_prompt.device)
    if w.dtype != torch.float32 or tuple(w.shape) != (B, E):
        raise ValueError("w must be fp32 [B, E]")
    if Wbar.dtype != X_prompt.dtype or Wbar.numel() != 3 * B * d * d_ff:
        raise ValueError("Wbar must hold 3*B*d*d_ff elements of X's dtype")
    if prompt_len is not None and (prompt_len.dtype != torch.int32 or tuple(prompt_len.shape) != (B,)):
        raise ValueError("prompt_len must be int32 [B]")
    _check(lib().lory_prompt_merge(ctypes.byref(shape), _ptr(X_prompt), _ptr(prompt_len), _ptr(R), _ptr(Wg), _ptr(Wu), _ptr(Wd),
                                   _ptr(w), _ptr(Wbar), _stream()), "lory_prompt_merge")
    return w, Wbar


def lory_dense_ffn_fwd(X: torch.Tensor, Wbar: torch.Tensor, d_ff: int, Y: Optional[torch.Tensor] = None,
                       workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Y [B,L,d] = dense SwiGLU FFN of every sequence with its merged parameters Wbar."""
    B, L, d = X.shape
    if Wbar.dtype != X.dtype or Wbar.numel() != 3 * B * d * d_ff:
        raise ValueError("Wbar must hold 3*B*d*d_ff elements of X's dtype")
    shape = make_shape(B, L, L, d, d_ff, 1, X.dtype)
    if Y is None:
        Y = torch.empty_like(X)
    if workspace is None:
        workspace = alloc_workspace(shape, LORY_PASS_DENSE, X.device)
    _check(lib().lory_dense_ffn_fwd(ctypes.byref(shape), _ptr(X), _ptr(Wbar), _ptr(Y), _ptr(workspace),
                                    workspace.numel(), _stream()), "lory_dense_ffn_fwd")
    return Y


def lory_dense_ffn_fwd_static(X: torch.Tensor, Wbar: torch.Tensor, d_ff: int, Y: torch.Tensor) -> torch.Tensor:
    """lory_dense_ffn_fwd without a workspace argument (library-held scratch); Y is the caller's."""
    B, L, d = X.shape
    if Wbar.dtype != X.dtype or Wbar.numel() != 3 * B * d * d_ff:
        raise ValueError("Wbar must hold 3*B*d*d_ff elements of X's dtype")
    shape = make_shape(B, L, L, d, d_ff, 1, X.dtype)
    _check(lib().lory_dense_ffn_fwd_static(ctypes.byref(shape), _ptr(X), _ptr(Wbar), _ptr(Y), _stream()),
           "lory_dense_ffn_fwd_static")
    return Y


def lory_merged_ffn_fwd(X: torch.Tensor, w: torch.Tensor, Wg: torch.Tensor, Wu: torch.Tensor,
                        Wd: torch.Tensor, T: int, Y: Optional[torch.Tensor] = None,
                        G_save: Optional[torch.Tensor] = None, U_save: Optional[torch.Tensor] = None,
                        workspace: Optional[torch.Tensor] = None,
                        Wbar_save: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Y = merged SwiGLU FFN of every segment; optionally saves G and U."""
    E, d, d_ff = Wg.shape
    shape = _shape_from(X, T, d_ff, E)
    for t in (Wg, Wu, Wd):
        if t.dtype != X.dtype:
            raise TypeError("expert stacks must have the dtype of X")
    if tuple(Wu.shape) != (E, d, d_ff) or tuple(Wd.shape) != (E, d_ff, d) or X.shape[2] != d:
        raise ValueError("expert stack shapes do not match")
    if w.dtype != torch.float32 or tuple(w.shape) != (X.shape[0] * (X.shape[1] // T), E):
        raise ValueError("w must be fp32 [S, E]")
    if Y is None:
        Y = torch.empty_like(X)
    if workspace is None:
        workspace = alloc_workspace(shape, LORY_PASS_FWD, X.device)
    _check(lib().lory_merged_ffn_fwd(ctypes.byref(shape), _ptr(X), _ptr(w), _ptr(Wg), _ptr(Wu), _ptr(Wd),
                                     _ptr(Y), _ptr(G_save), _ptr(U_save), _ptr(Wbar_save), _ptr(workspace),
                                     workspace.numel(), _stream()), "lory_merged_ffn_fwd")
    return Y


def lory_merged_ffn_bwd(X: torch.Tensor, w: torch.Tensor, Wg: torch.Tensor, Wu: torch.Tensor,
                        Wd: torch.Tensor, dY: torch.Tensor, T: int,
                        G_save: Optional[torch.Tensor] = None, U_save: Optional[torch.Tensor] = None,
                        dX: Optional[torch.Tensor] = None, dWg: Optional[torch.Tensor] = None,
                        dWu: Optional[torch.Tensor] = None, dWd: Optional[torch.Tensor] = None,
                        dw: Optional[torch.Tensor] = None, grad_dtype: Optional[torch.dtype] = None,
                        accumulate: bool = False, workspace: Optional[torch.Tensor] = None,
                        Wbar_save: Optional[torch.Tensor] = None
                        ) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor, torch.Tensor, torch.Tensor]:
    """Returns (dX, dWg, dWu, dWd, dw)."""
    E, d, d_ff = Wg.shape
    shape = _shape_from(X, T, d_ff, E)
    if grad_dtype is None:
        grad_dtype = dWg.dtype if dWg is not None else torch.float32
    if dX is None:
        dX = torch.empty_like(X)
    if dWg is None:
        dWg = torch.empty(Wg.shape, dtype=grad_dtype, device=X.device)
    if dWu is None:
        dWu = torch.empty(Wu.shape, dtype=grad_dtype, device=X.device)
    if dWd is None:
        dWd = torch.empty(Wd.shape, dtype=grad_dtype, device=X.device)
    for t in (dWg, dWu, dWd):
        if t.dtype != grad_dtype:
            raise TypeError("gradient stacks must all have grad_dtype")
    if dw is None:
        dw = torch.empty_like(w)
    if dY.shape != X.shape or dY.dtype != X.dtype:
        raise ValueError("dY must match X")
    if workspace is None:
        workspace = alloc_workspace(shape, LORY_PASS_BWD, X.device)
    _check(lib().lory_merged_ffn_bwd(ctypes.byref(shape), _ptr(X), _ptr(w), _ptr(Wg), _ptr(Wu), _ptr(Wd),
                                     _ptr(dY), _ptr(G_save), _ptr(U_save), _ptr(Wbar_save), _ptr(dX), _ptr(dWg), _ptr(dWu),
                                     _ptr(dWd), _dtype_code(grad_dtype), int(bool(accumulate)), _ptr(dw),
                                     _ptr(workspace), workspace.numel(), _stream()),
           "lory_merged_ffn_bwd")
    return dX, dWg, dWu, dWd, dw
