"""Thin Python binding of include/moe_offload.h (argument marshalling only)."""
from __future__ import annotations

import ctypes as C

import torch

from .binding import MoeError, Shape, _check, _ptr, _stream, lib, moe_max_rows, moe_packed_weight_bytes

_ready = False


def _lib():
    global _ready
    L = lib()
    if not _ready:
        sp, vp, i32 = C.POINTER(Shape), C.c_void_p, C.c_int32
        L.moe_offload_staging_bytes.restype = C.c_size_t
        L.moe_offload_staging_bytes.argtypes = [sp, i32]
        L.moe_offload_workspace_bytes.restype = C.c_size_t
        L.moe_offload_workspace_bytes.argtypes = [sp]
        L.moe_expert_ffn_offloaded.restype = C.c_int
        L.moe_expert_ffn_offloaded.argtypes = [sp] + [vp] * 8 + [i32, vp, vp]
        _ready = True
    return L


def moe_offload_staging_bytes(s: Shape, resident: int) -> int:
    return int(_lib().moe_offload_staging_bytes(C.byref(s), resident))


def moe_offload_workspace_bytes(s: Shape) -> int:
    return int(_lib().moe_offload_workspace_bytes(C.byref(s)))


def _host_ptr(t: torch.Tensor, nbytes: int, name: str) -> C.c_void_p:
    if t.is_cuda or not t.is_contiguous() or t.numel() * t.element_size() < nbytes:
        raise MoeError(f"{name}: need a contiguous host tensor of {nbytes} bytes")
    return C.c_void_p(t.data_ptr())


def moe_expert_ffn_offloaded(s: Shape, xe, offsets, W1p_host, W2p_host, b1, b2, ye, staging,
                             resident: int, workspace, stream=None) -> None:
    rows = moe_max_rows(s)
    wb = moe_packed_weight_bytes(s)
    if xe.numel() < rows * s.d_model or ye.numel() < rows * s.d_model or ye.dtype != s.ye_dtype:
        raise MoeError("xe / ye: need max_rows x d_model elements (ye fp16)")
    if staging.numel() * staging.element_size() < moe_offload_staging_bytes(s, resident):
        raise MoeError("staging is smaller than moe_offload_staging_bytes")
    if workspace.numel() * workspace.element_size() < moe_offload_workspace_bytes(s):
        raise MoeError("workspace is smaller than moe_offload_workspace_bytes")
    _check(_lib().moe_expert_ffn_offloaded(C.byref(s), _ptr(xe), _ptr(offsets),
                                           _host_ptr(W1p_host, wb, "W1p_host"),
                                           _host_ptr(W2p_host, wb, "W2p_host"), _ptr(b1), _ptr(b2),
                                           _ptr(ye), _ptr(staging), resident, _ptr(workspace),
                                           _stream(stream)))
